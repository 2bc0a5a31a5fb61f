// Interface of the MFMA GEMM launcher (rl_gemm.hip).
#pragma once
#include "rl_common.h"

enum { MG_STORE_F32 = 0, MG_STORE_F16 = 1, MG_RESID = 2, MG_SWIGLU = 3, MG_QKV = 4, MG_LSE = 5, MG_KLFULL = 6, MG_SAMPLE = 7 };

struct GemmArgs {
    const f16_t* A = nullptr;   // [M, K] row-major, leading dimension lda
    int lda = 0;
    const bf16_t* W = nullptr;  // [Wrows, K] row-major
    int w_f16 = 0;              // W points at an fp16 copy made by k_bf16_to_f16 (no conversion in the kernel): decode GEMMs,
                                // and large-M GEMMs for which k_gemm_mfma_reads_f16_copy() says yes
    int M = 0, N = 0, K = 0;    // N = output columns (MG_SWIGLU: d_ffn)
    // Activations carried as fp16 pairs (value = hi + lo, about 22 significant bits): A is [M, 2 Kw] with the hi
    // halves of a row in columns [0, Kw) and the lo halves in [Kw, 2 Kw), K = 2 Kw, and the k index into W wraps
    // at Kw, i.e. C = A_hi W^T + A_lo W^T in one pass.  Kw = 0: plain operand, W has K columns.
    int Kw = 0;
    // Epilogues that emit fp16 activations (MG_SWIGLU, MG_QKV, MG_STORE_F16) write such pairs: hi where the
    // plain value would go, lo one plane further (next to it in the row for row-major outputs, whose leading
    // dimensions are then twice as wide; the cache's lo planes live in layer `layer_lo`).
    int split_out = 0;
    int layer_lo = 0;
    int Wrows = 0;              // filled by the launcher
    int n_blocks_n = 0;         // filled by the launcher
    int k_per_split = 0;        // filled by the launcher
    int up_offset = 0;          // MG_SWIGLU: row of W where the up projection starts
    float* outF = nullptr;      // MG_STORE_F32 (+ split * split_stride) / MG_RESID
    f16_t* outH = nullptr;      // MG_STORE_F16 / MG_SWIGLU
    int ldc = 0;
    int64_t split_stride = 0;
    // MG_QKV
    const int* tok_pos = nullptr;
    const int* tok_slot = nullptr;
    const float2* rope = nullptr;
    f16_t* q_out = nullptr;
    f16_t* k_out = nullptr;
    f16_t* v_out = nullptr;
    f16_t* pool = nullptr;
    const int* block_table = nullptr;
    int mpps = 0, layer = 0, Hq = 0, Hkv = 0, hd = 0;
    // MG_LSE (LM head for scoring): per row and per column group (k_gemm_mfma_lse_parts groups of equal
    // width) the pair (max, sum exp(z - max)) goes to lse_part[row][group]; the logit of the row's target token (tgt[row] >= 0) to z_tgt[row].
    // The logits themselves are never stored.
    const int* tgt = nullptr;
    float2* lse_part = nullptr;
    float* z_tgt = nullptr;
    // MG_KLFULL (both LM heads for the exact KL): the reference's logits A2 * W2^T are formed for the same
    // tile as the policy's A * W^T; per row and 64-column group five floats go to kl_part[row][N/64][5]
    // (see kl_epilogue).  No logits are stored.
    // MG_SAMPLE (LM head of a decode step): per row and 32-column block, samp_part[row][N/32] =
    // (max, sum exp((z - max) * inv_temp), sum exp(z - max), block-local column of the max [lowest on ties], as int bits).
    // The logits themselves are never stored; the sampler picks a block from these and recomputes its 32 logits.
    float4* samp_part = nullptr;
    float inv_temp = 1.0f;
    const f16_t* A2 = nullptr;
    int lda2 = 0;
    const bf16_t* W2 = nullptr;
    float* kl_part = nullptr;
    int vt_cap = 0;             // > 0: v_out is dim-major [Hkv][hd][vt_cap tokens]; 0: token-major [M][Hkv][hd]
    KvGeom geo{};
    // 256 x 256 workgroup tiles (splits == 1 only): 0 never, 1 when the grid fills the chip at one workgroup
    // per CU, 2 whenever the shape allows (N multiple of 256, K of 128)
    int big_mode = 1;
};

bool k_gemm_mfma_supported(int epi, int N, int K, int hd);
bool k_gemm_mfma_reads_f16_copy(int epi, GemmArgs a, int splits);
void k_gemm_big_reads_copy(int on);
// splits > 1 only with MG_STORE_F32: partial sums of split s go to outF + s * split_stride.
void k_gemm_mfma(int epi, GemmArgs a, int splits, hipStream_t s);
int k_gemm_mfma_splits_used(int K, int splits);
// Number of column groups per row that an MG_LSE launch of this shape writes (at most N / 64).
int k_gemm_mfma_lse_parts(int M, int N, int K, int big_mode);
// Decode GEMM (M <= 128, lda * 2 * 128 below 4 GiB) on 128-column tiles with LDS operand rings: epi MG_STORE_F32 (split-K partials to
// outF + split * split_stride; plain store when one split) or MG_SWIGLU (never split).
bool k_gemm_decode_supported(int epi, int N, int K);   // K and tile columns multiples of 128
int k_gemm_decode_splits_used(int K, int splits);
void k_gemm_decode(int epi, GemmArgs a, int splits, hipStream_t s);
// Measurement switch: k_gemm_decode takes the 128 x 128 tile kernel above this many rows (default 64; < 0: never).
void k_gemm_decode_tile_above(int rows);

// dst[i] = fp16(src[i]) for n bf16 values (n multiple of 8, both 16-byte aligned), bit for bit what the GEMM
// kernels compute when they convert on the fly.
void k_bf16_to_f16(const void* src, void* dst, int64_t n, hipStream_t s);
