// Interface of the MFMA attention launchers (rl_attn.hip).
#pragma once
#include "rl_common.h"

struct DecodeAttnArgs {
    const f16_t* q = nullptr;        // [B, Hq, hd]
    const f16_t* pool = nullptr;     // paged K/V
    const int* block_table = nullptr;
    const int* tok_pos = nullptr;    // [B] position of the new token; context = pos + 1
    f16_t* out = nullptr;            // [B, Hq * hd]
    float* part_o = nullptr;         // [B*Hq, nsplit, hd] when nsplit > 1
    float* part_ml = nullptr;        // [B*Hq, nsplit, 2]
    int mpps = 0, layer = 0, Hq = 0, Hkv = 0;
    float scale = 0.f;               // 1 / sqrt(hd)
    KvGeom geo{};
};
void k_attn_decode(const DecodeAttnArgs& a, int B, int nsplit, hipStream_t s);
