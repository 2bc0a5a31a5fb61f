// Shared device helpers and the internal launcher interface of librollout.
// gfx950 only (64-wide wavefronts).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16_t;
typedef _Float16 f16_t;

#define RL_WAVE 64

// ---------------------------------------------------------------- conversions
__device__ __forceinline__ float to_f(float v) { return v; }
__device__ __forceinline__ float to_f(bf16_t v) { return (float)v; }
__device__ __forceinline__ float to_f(f16_t v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f(float v);
template <> __device__ __forceinline__ float from_f<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f<bf16_t>(float v) { return (bf16_t)v; }  // RNE (v_cvt_pk_bf16_f32)
template <> __device__ __forceinline__ f16_t from_f<f16_t>(float v) { return (f16_t)v; }     // RNE (v_cvt_f16_f32)

// ---------------------------------------------------------------- wave / block reductions
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, RL_WAVE);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, RL_WAVE));
    return v;
}
// Block-wide sum / max for blockDim.x a multiple of 64 (<= 1024); red needs 16 floats; all threads get the result.
__device__ __forceinline__ float block_sum(float v, float* red) {
    v = wave_sum(v);
    const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    float t = 0.f;
    for (int i = 0; i < nw; ++i) t += red[i];
    return t;
}
__device__ __forceinline__ float block_max(float v, float* red) {
    v = wave_max(v);
    const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    float t = red[0];
    for (int i = 1; i < nw; ++i) t = fmaxf(t, red[i]);
    return t;
}

// ---------------------------------------------------------------- paged KV addressing
// Per layer the pool holds a K region and a V region of n_pages pages each.
//   K page: [Hkv][page_tokens][hd]      (a (page, kv head) tile is contiguous, token-major)
//   V page: [Hkv][hd][page_tokens]      (dim-major: the tokens of one dim are contiguous)
struct KvGeom {
    int Hkv, hd, PT;
    int64_t n_pages;
    __host__ __device__ int64_t page_elems() const { return (int64_t)Hkv * PT * hd; }
    __host__ __device__ int64_t layer_elems() const { return 2 * n_pages * page_elems(); }
    __host__ __device__ int64_t k_off(int64_t layer, int64_t page, int g, int tok, int d) const {
        return layer * layer_elems() + page * page_elems() + ((int64_t)g * PT + tok) * hd + d;
    }
    __host__ __device__ int64_t v_off(int64_t layer, int64_t page, int g, int tok, int d) const {
        return layer * layer_elems() + (n_pages + page) * page_elems() + ((int64_t)g * hd + d) * PT + tok;
    }
};

// ---------------------------------------------------------------- launcher interface (host side)
// dtype: 0 = fp32 weights and fp32 activations; 1 = bf16 weights with fp16 activations and
// fp16 KV cache (fp32 residual stream and accumulation in both).  bf16 -> fp16 is exact for
// every weight of normal fp16 magnitude, so the weights lose nothing; activations keep an
// 11-bit significand instead of bf16's 8.  All pointers device.  Nothing here synchronises.
enum { EPI_STORE_F32 = 0, EPI_STORE_T = 1, EPI_RESID = 2, EPI_SWIGLU = 3 };

struct SampleArgs {
    uint64_t seed;
    int64_t seq_base;
    float temperature;
    int eos_id;
    // per-slot indirections of the queue mode (all dev, all optional):
    const int* out_row = nullptr;     // row of out_ids / out_logp that slot b writes (default b)
    const int* seq_id = nullptr;      // sequence id of slot b for the uniform draw, added to seq_base (default b)
    const int* gen_limit = nullptr;   // slot b finishes after this many generated tokens (default: never)
    int* out_len = nullptr;           // out_len[out_row[b]] = tokens generated, written when slot b finishes
};

// basic kernels (rl_basic.hip)
void k_fill_i32(int* p, int v, int64_t n, hipStream_t s);
void k_fill_f32(float* p, float v, int64_t n, hipStream_t s);
void k_rope_table(float2* tab, int max_seq, int hd, float base, hipStream_t s);
void k_set_pages(int* block_table, int mpps, const int* triples_host, int n_triples, hipStream_t s);
void k_step_begin(const int* tok_in, const int* last_tok, const int* seq_len, const int* finished, int* cur_tok,
                  int* tok_pos, int* tok_slot, int B, hipStream_t s);
void k_pack_tokens(const int* ids, int ld_ids, const int* seq_first, const int* row_slot, const int* row_start,
                   const int* row_len, const int* full_len, int align, int* tok_ids, int* tok_pos, int* tok_slot,
                   int* tok_tgt, int nrows, hipStream_t s);
void k_prefill_state(const int* ids, int ld_ids, const int* row_len, int* last_tok, int* seq_len, int* gen_count,
                     int* finished, int* step_count, int B, hipStream_t s);
// State of n freshly prefilled slots: slot row_slot[i] starts sequence seq_first[i] (row of ids, also its output
// row and sequence id) of prompt length row_len[i], limited to limit[i] generated tokens.
void k_prefill_state_slots(const int* ids, int ld_ids, int n, const int* seq_first, const int* row_slot,
                           const int* row_len, const int* limit, int* last_tok, int* seq_len, int* gen_count,
                           int* finished, int* step_count, int* out_row, int* seq_id, int* gen_limit, hipStream_t s);
void k_embed(int dtype, const int* ids, int n, const void* E, int d, int V, float* x, int* errflag, hipStream_t s);
// split = 1 (bf16 configurations only): the output row is a row of fp16 pairs, [d hi | d lo], value = hi + lo
void k_rmsnorm(int dtype, const float* x, const void* g, void* out, int n, int d, float eps, hipStream_t s, int split = 0);
void k_gemm_simple(int dtype, int epi, const void* A, int lda, const void* W, const void* W2, int M, int N, int K,
                   float* outF, void* outT, int ldc, hipStream_t s);
void k_rope_append(int dtype, const float* qkv, int nsplit, int64_t split_stride, int n, const int* tok_pos,
                   const int* tok_slot, const float2* rope, void* q_out, void* k_out, void* v_out, void* pool,
                   int layer, KvGeom geo, const int* block_table, int mpps, int Hq, hipStream_t s);
void k_rope_append_split(int dtype, const float* part, int nsplit, int64_t split_stride, int n, const int* tok_pos,
                         const int* tok_slot, const float2* rope, void* q_out, void* pool, int layer, KvGeom geo,
                         const int* block_table, int mpps, int Hq, hipStream_t s, int split = 0, int layer_lo = 0);
void k_resid_norm(int dtype, float* x, const float* part, int nsplit, int64_t split_stride, const void* g, void* out,
                  int n, int d, float eps, hipStream_t s, int split = 0);
void k_attn_simple(int dtype, const void* q, const void* kc, const void* vc, const void* pool, int layer, KvGeom geo,
                   const int* block_table, int mpps, const int* tok_pos, const int* tok_slot, void* out, int n,
                   int Hq, int max_ctx, hipStream_t s);
void k_sample(const float* logits, int ldz, int V, int B, SampleArgs a, int* last_tok, int* seq_len, int* gen_count,
              int* finished, int* step_count, int* tok_out, float* logp_out, int* out_ids, float* out_logp,
              int out_stride, hipStream_t s);
// The draw from the MG_SAMPLE statistics of the LM-head GEMM ([B][V / 32] float4); h: the fp16 rows that went into that
// GEMM, W: the bf16 LM head, V a multiple of 32, d of 8.
void k_sample_blocks(const float4* stats, int V, const void* h, int ldh, const void* W, int d, int B, SampleArgs a,
                     int* last_tok, int* seq_len, int* gen_count, int* finished, int* step_count, int* tok_out,
                     float* logp_out, int* out_ids, float* out_logp, int out_stride, hipStream_t s);
void k_mfma_rate(void* scratch, int n_wg, int iters, int random, hipStream_t s);
void k_lse_gather(const float* logits, int ldz, int V, int nrows, const int* tok_tgt, const int* tok_slot,
                  const int* tok_pos, float* logp_out, int ld_out, hipStream_t s);
void k_kl(const float* lp, const float* lr, const int* seq_len, const int* prompt_len, int B, int Lmax, float coef,
          float* kl, float* pen, hipStream_t s);
void k_out_len(const int* gen_count, int* out_len, int B, hipStream_t s);
void k_kl_full_reduce(const float* part, int nparts, int nrows, const int* tok_tgt, const int* tok_slot,
                      const int* tok_pos, const int* prompt_len, float* out, int ld_out, hipStream_t s);
void k_kl_full_rows(const float* zp, const float* zr, int ldz, int V, int nrows, const int* tok_tgt,
                    const int* tok_slot, const int* tok_pos, const int* prompt_len, float* out, int ld_out,
                    hipStream_t s);
void k_value_head(int dtype, const float* x, const void* g, const void* head, int n, int d, float eps,
                  const int* tok_slot, const int* tok_pos, float* out, int ld_out, hipStream_t s);
// n host ints into device memory through kernel arguments (any n; nothing is copied by the runtime)
void k_put_i32(int* dst, const int* src_host, int n, hipStream_t s);
void k_ppo_reward(const float* kl, const float* seq_reward, const int* seq_len, const int* prompt_len, int B, int Lmax,
                  float coef, float* out, hipStream_t s);
void k_lse_reduce(const float2* part, int nparts, const float* z_tgt, int nrows, const int* tok_tgt,
                  const int* tok_slot, const int* tok_pos, float* logp_out, int ld_out, hipStream_t s);
