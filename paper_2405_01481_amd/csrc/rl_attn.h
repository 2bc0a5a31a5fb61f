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
    // split = 1: q and out rows are fp16 pairs, [Hq * hd hi | Hq * hd lo]; the cache's lo planes of K and V are
    // in layer `layer_lo` of the pool
    int split = 0, layer_lo = 0;
    // qkv_part != nullptr (plain layers only, Hq / Hkv <= 8): q is not read; the kernel itself sums the QKV
    // projection's split-K partial rows [qkv_nsplit][B, (Hq + 2 Hkv) hd] (split stride in floats), rotates q and k
    // with rope[pos][hd/2] = (cos, sin), and appends k and v of the new token to the cache through pool_w
    const float* qkv_part = nullptr;
    int qkv_nsplit = 0;
    int64_t qkv_split_stride = 0;
    const float2* rope = nullptr;
    f16_t* pool_w = nullptr;
};
// Whether k_attn_decode can take the QKV partial sums itself (qkv_part) for these head counts; it launches nothing
// if asked to for others, or for a pair layer.
bool k_attn_decode_consumes_qkv(int Hq, int Hkv, int hd);
void k_attn_decode(const DecodeAttnArgs& a, int B, int nsplit, hipStream_t s);

// Causal attention over a packed token list.  Sequences start at rows that are multiples of 32
// and every row up to the next multiple of 32 past a sequence's end holds finite values.
struct PrefillAttnArgs {
    const f16_t* q = nullptr;    // [rows, Hq, hd]
    const f16_t* k = nullptr;    // [rows, Hkv, hd]
    const f16_t* vT = nullptr;   // [Hkv, hd, vt_cap]  (dim-major)
    f16_t* out = nullptr;        // [rows, Hq * hd]
    const int4* blocks = nullptr;  // per workgroup: (first row of the sequence, its length, query block, 0)
    int Hq = 0, Hkv = 0, hd = 0, vt_cap = 0;
    float scale = 0.f;
    // split = 1: fp16 pairs.  q, k and out rows are twice as wide, [hi heads | lo heads]; the lo plane of vT
    // follows the hi plane ([2][Hkv, hd, vt_cap])
    int split = 0;
};
void k_attn_prefill(const PrefillAttnArgs& a, int nblocks, hipStream_t s);
