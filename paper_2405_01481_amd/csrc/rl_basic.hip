// Plain reference kernels for every step of the rollout path (any dtype) plus the
// small bookkeeping kernels (packing, paging, sampling, log-sum-exp, KL).
// The formulas are the standard Llama-style decoder ones; the paper (Sections 3.1-3.2)
// only names the stages.
#include "rl_common.h"

// ---------------------------------------------------------------- fills / tables
__global__ void fill_i32_kernel(int* p, int v, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}
__global__ void fill_f32_kernel(float* p, float v, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}
void k_fill_i32(int* p, int v, int64_t n, hipStream_t s) {
    if (n <= 0) return;
    fill_i32_kernel<<<dim3((unsigned)((n + 255) / 256)), 256, 0, s>>>(p, v, n);
}
void k_fill_f32(float* p, float v, int64_t n, hipStream_t s) {
    if (n <= 0) return;
    fill_f32_kernel<<<dim3((unsigned)((n + 255) / 256)), 256, 0, s>>>(p, v, n);
}

// cos/sin of pos * base^(-2j/hd), evaluated in fp64 and rounded once to fp32.
__global__ void rope_table_kernel(float2* tab, int max_seq, int half, double log_base, int hd) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= max_seq * half) return;
    int pos = i / half, j = i % half;
    double theta = exp(-2.0 * (double)j / (double)hd * log_base);
    double ang = (double)pos * theta;
    tab[i] = make_float2((float)cos(ang), (float)sin(ang));
}
void k_rope_table(float2* tab, int max_seq, int hd, float base, hipStream_t s) {
    int n = max_seq * (hd / 2);
    rope_table_kernel<<<(n + 255) / 256, 256, 0, s>>>(tab, max_seq, hd / 2, log((double)base), hd);
}

// block_table[slot][idx] = page for up to 64 (slot, idx, page) triples passed by value.
struct PageTriples { int v[192]; };
__global__ void set_pages_kernel(int* bt, int mpps, PageTriples t, int n) {
    int i = threadIdx.x;
    if (i < n) bt[(int64_t)t.v[3 * i] * mpps + t.v[3 * i + 1]] = t.v[3 * i + 2];
}
void k_set_pages(int* block_table, int mpps, const int* triples_host, int n_triples, hipStream_t s) {
    for (int o = 0; o < n_triples; o += 64) {
        PageTriples t;
        int n = n_triples - o < 64 ? n_triples - o : 64;
        for (int i = 0; i < 3 * n; ++i) t.v[i] = triples_host[3 * o + i];
        set_pages_kernel<<<1, 64, 0, s>>>(block_table, mpps, t, n);
    }
}

// ---------------------------------------------------------------- token bookkeeping
// A finished sequence is parked: position -1, which every consumer reads as "no cache slot, no
// attention, zeros" (the padding-row rule of the packed token lists), so it stops growing its cache.
__global__ void step_begin_kernel(const int* tok_in, const int* last_tok, const int* seq_len, const int* finished,
                                  int* cur_tok, int* tok_pos, int* tok_slot, int B) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    cur_tok[b] = tok_in ? tok_in[b] : last_tok[b];
    tok_pos[b] = finished[b] ? -1 : seq_len[b];
    tok_slot[b] = b;
}
void k_step_begin(const int* tok_in, const int* last_tok, const int* seq_len, const int* finished, int* cur_tok,
                  int* tok_pos, int* tok_slot, int B, hipStream_t s) {
    step_begin_kernel<<<(B + 255) / 256, 256, 0, s>>>(tok_in, last_tok, seq_len, finished, cur_tok, tok_pos, tok_slot, B);
}

// Pack rows of a padded [*, ld_ids] id matrix into a flat token list.
// Row r of the chunk is batch row seq_first[r]; its row_len[r] tokens go to
// [row_start[r], row_start[r] + row_len[r]).  tok_tgt (optional) = next token id of the
// same row, or -1 when there is none inside full_len[r].
// With align > 1 every row is padded to a multiple of align tokens; padding entries carry
// token id 0, position -1 and no target.
__global__ void pack_tokens_kernel(const int* ids, int ld_ids, const int* seq_first, const int* row_slot,
                                   const int* row_start, const int* row_len, const int* full_len, int align,
                                   int* tok_ids, int* tok_pos, int* tok_slot, int* tok_tgt) {
    int r = blockIdx.x;
    int b = seq_first[r], st = row_start[r], len = row_len[r];
    const int slot = row_slot[r];
    const int alen = (len + align - 1) / align * align;
    const int* src = ids + (int64_t)b * ld_ids;
    for (int t = threadIdx.x; t < alen; t += blockDim.x) {
        const bool real = t < len;
        tok_ids[st + t] = real ? src[t] : 0;
        tok_pos[st + t] = real ? t : -1;
        tok_slot[st + t] = slot;
        if (tok_tgt) tok_tgt[st + t] = (real && t + 1 < full_len[r]) ? src[t + 1] : -1;
    }
}
void k_pack_tokens(const int* ids, int ld_ids, const int* seq_first, const int* row_slot, const int* row_start,
                   const int* row_len, const int* full_len, int align, int* tok_ids, int* tok_pos, int* tok_slot,
                   int* tok_tgt, int nrows, hipStream_t s) {
    if (nrows <= 0) return;
    pack_tokens_kernel<<<nrows, 256, 0, s>>>(ids, ld_ids, seq_first, row_slot, row_start, row_len, full_len, align,
                                             tok_ids, tok_pos, tok_slot, tok_tgt);
}

// After prefill of the first P-1 prompt tokens: remember the last prompt token, lengths, counters.
__global__ void prefill_state_kernel(const int* ids, int ld_ids, const int* prompt_len, int* last_tok, int* seq_len,
                                     int* gen_count, int* finished, int* step_count, int B) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int P = prompt_len[b];
    last_tok[b] = ids[(int64_t)b * ld_ids + P - 1];
    seq_len[b] = P - 1;
    gen_count[b] = 0;
    finished[b] = 0;
    step_count[b] = 0;
}
void k_prefill_state(const int* ids, int ld_ids, const int* row_len, int* last_tok, int* seq_len, int* gen_count,
                     int* finished, int* step_count, int B, hipStream_t s) {
    prefill_state_kernel<<<(B + 255) / 256, 256, 0, s>>>(ids, ld_ids, row_len, last_tok, seq_len, gen_count,
                                                         finished, step_count, B);
}

__global__ void prefill_state_slots_kernel(const int* ids, int ld_ids, int n, const int* seq_first, const int* row_slot,
                                           const int* row_len, const int* limit, int* last_tok, int* seq_len,
                                           int* gen_count, int* finished, int* step_count, int* out_row, int* seq_id,
                                           int* gen_limit) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int row = seq_first[i], b = row_slot[i], P = row_len[i];
    last_tok[b] = ids[(int64_t)row * ld_ids + P - 1];
    seq_len[b] = P - 1;
    gen_count[b] = 0;
    finished[b] = 0;
    step_count[b] = 0;
    out_row[b] = row;
    seq_id[b] = row;
    gen_limit[b] = limit[i];
}
void k_prefill_state_slots(const int* ids, int ld_ids, int n, const int* seq_first, const int* row_slot,
                           const int* row_len, const int* limit, int* last_tok, int* seq_len, int* gen_count,
                           int* finished, int* step_count, int* out_row, int* seq_id, int* gen_limit, hipStream_t s) {
    if (n <= 0) return;
    prefill_state_slots_kernel<<<(n + 255) / 256, 256, 0, s>>>(ids, ld_ids, n, seq_first, row_slot, row_len, limit,
                                                               last_tok, seq_len, gen_count, finished, step_count,
                                                               out_row, seq_id, gen_limit);
}

__global__ void out_len_kernel(const int* gen_count, int* out_len, int B) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) out_len[b] = gen_count[b];
}
void k_out_len(const int* gen_count, int* out_len, int B, hipStream_t s) {
    out_len_kernel<<<(B + 255) / 256, 256, 0, s>>>(gen_count, out_len, B);
}

// ---------------------------------------------------------------- embedding gather
template <typename T>
__global__ void embed_kernel(const int* ids, const T* E, int d, int V, float* x, int* errflag) {
    int n = blockIdx.x;
    int id = ids[n];
    if (id < 0 || id >= V) {
        if (threadIdx.x == 0) atomicOr(errflag, 1);
        id = id < 0 ? 0 : V - 1;
    }
    const T* row = E + (int64_t)id * d;
    float* xo = x + (int64_t)n * d;
    for (int j = threadIdx.x; j < d; j += blockDim.x) xo[j] = to_f(row[j]);
}
void k_embed(int dtype, const int* ids, int n, const void* E, int d, int V, float* x, int* errflag, hipStream_t s) {
    if (n <= 0) return;
    if (dtype == 0) embed_kernel<float><<<n, 256, 0, s>>>(ids, (const float*)E, d, V, x, errflag);
    else embed_kernel<bf16_t><<<n, 256, 0, s>>>(ids, (const bf16_t*)E, d, V, x, errflag);
}

// Store v as T at o[0]; with split also what the rounding left over, as T, at o[lo_off]: the pair hi + lo
// carries about 22 significant bits when T is fp16.
template <typename T>
__device__ __forceinline__ void put_pair(T* o, int64_t lo_off, float v, int split) {
    const T hi = from_f<T>(v);
    o[0] = hi;
    if (split) o[lo_off] = from_f<T>(v - to_f(hi));
}
// Four consecutive values (o 4-element aligned) scaled by four consecutive gains: one store per plane, one gain load.
template <typename T, typename TW>
__device__ __forceinline__ void put_pair4(T* o, int64_t lo_off, float4 v, float rs, const TW* g, int split) {
    float gf[4];
    if constexpr (sizeof(TW) == 2) {
        const uint2 gv = *reinterpret_cast<const uint2*>(g);          // four bf16
        gf[0] = __uint_as_float(gv.x << 16); gf[1] = __uint_as_float(gv.x & 0xffff0000u);
        gf[2] = __uint_as_float(gv.y << 16); gf[3] = __uint_as_float(gv.y & 0xffff0000u);
    } else {
        const float4 gv = *reinterpret_cast<const float4*>(g);
        gf[0] = gv.x; gf[1] = gv.y; gf[2] = gv.z; gf[3] = gv.w;
    }
    const float w[4] = {v.x * rs * gf[0], v.y * rs * gf[1], v.z * rs * gf[2], v.w * rs * gf[3]};
    if constexpr (sizeof(T) == 2) {
        typedef T T4 __attribute__((ext_vector_type(4)));
        T4 hi, lo;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            hi[e] = from_f<T>(w[e]);
            lo[e] = from_f<T>(w[e] - to_f(hi[e]));
        }
        *reinterpret_cast<T4*>(o) = hi;
        if (split) *reinterpret_cast<T4*>(o + lo_off) = lo;
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) put_pair(o + e, lo_off, w[e], split);
    }
}

// ---------------------------------------------------------------- RMSNorm: out = x * rsqrt(mean(x^2) + eps) * g
// split: the output row is twice as wide, [d values rounded to T | d remainders] (fp16 pairs).
template <typename T, typename TW>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float* x, const TW* g, T* out, int d, float eps, int split) {
    __shared__ float red[16];
    int n = blockIdx.x;
    const float* xr = x + (int64_t)n * d;
    T* o = out + (int64_t)n * d * (split ? 2 : 1);
    if (d % 4 == 0 && d <= 8192) {
        // the row is read once, 16 bytes per lane, and kept in registers between the two passes
        float4 keep[8];
        float ss = 0.f;
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int j = (it * 256 + threadIdx.x) * 4;
            if (j < d) {
                keep[it] = *reinterpret_cast<const float4*>(xr + j);
                ss += keep[it].x * keep[it].x + keep[it].y * keep[it].y + keep[it].z * keep[it].z + keep[it].w * keep[it].w;
            }
        }
        ss = block_sum(ss, red);
        const float rs = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int j = (it * 256 + threadIdx.x) * 4;
            if (j < d) put_pair4(o + j, d, keep[it], rs, g + j, split);
        }
        return;
    }
    float ss = 0.f;
    for (int j = threadIdx.x; j < d; j += 256) { float v = xr[j]; ss += v * v; }
    ss = block_sum(ss, red);
    float rs = 1.0f / sqrtf(ss / (float)d + eps);
    for (int j = threadIdx.x; j < d; j += 256) put_pair(o + j, d, xr[j] * rs * to_f(g[j]), split);
}
void k_rmsnorm(int dtype, const float* x, const void* g, void* out, int n, int d, float eps, hipStream_t s, int split) {
    if (n <= 0) return;
    if (dtype == 0) rmsnorm_kernel<float, float><<<n, 256, 0, s>>>(x, (const float*)g, (float*)out, d, eps, 0);
    else rmsnorm_kernel<f16_t, bf16_t><<<n, 256, 0, s>>>(x, (const bf16_t*)g, (f16_t*)out, d, eps, split);
}

// ---------------------------------------------------------------- plain tiled GEMM  C = A[M,K] * W[N,K]^T
// 64x64 output tile, 16-wide k slab, 256 threads each 4x4, fp32 FMA accumulation.
template <typename T, typename TW, int EPI>
__global__ __launch_bounds__(256) void gemm_simple_kernel(const T* __restrict__ A, int lda, const TW* __restrict__ W,
                                                          const TW* __restrict__ W2, int M, int N, int K,
                                                          float* outF, T* outT, int ldc) {
    __shared__ float As[16][65];
    __shared__ float Ws[16][65];
    __shared__ float W2s[EPI == EPI_SWIGLU ? 16 : 1][65];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    float acc[4][4] = {}, acc2[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int idx = tid + i * 256, r = idx >> 4, kk = idx & 15;
            int k = k0 + kk;
            As[kk][r] = (m0 + r < M && k < K) ? to_f(A[(int64_t)(m0 + r) * lda + k]) : 0.f;
            Ws[kk][r] = (n0 + r < N && k < K) ? to_f(W[(int64_t)(n0 + r) * K + k]) : 0.f;
            if (EPI == EPI_SWIGLU) W2s[kk][r] = (n0 + r < N && k < K) ? to_f(W2[(int64_t)(n0 + r) * K + k]) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], b[4], b2[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Ws[kk][tx * 4 + i]; }
            if (EPI == EPI_SWIGLU) {
#pragma unroll
                for (int i = 0; i < 4; ++i) b2[i] = W2s[kk][tx * 4 + i];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc[i][j] += a[i] * b[j];
                    if (EPI == EPI_SWIGLU) acc2[i][j] += a[i] * b2[j];
                }
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int m = m0 + ty * 4 + i;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int n = n0 + tx * 4 + j;
            if (n >= N) continue;
            int64_t o = (int64_t)m * ldc + n;
            float v = acc[i][j];
            if (EPI == EPI_STORE_F32) outF[o] = v;
            else if (EPI == EPI_STORE_T) outT[o] = from_f<T>(v);
            else if (EPI == EPI_RESID) outF[o] += v;
            else { float u = acc2[i][j]; outT[o] = from_f<T>(v / (1.0f + __expf(-v)) * u); }
        }
    }
}
template <typename T, typename TW>
static void gemm_simple_t(int epi, const T* A, int lda, const TW* W, const TW* W2, int M, int N, int K, float* outF,
                          T* outT, int ldc, hipStream_t s) {
    dim3 grid((N + 63) / 64, (M + 63) / 64);
    switch (epi) {
        case EPI_STORE_F32: gemm_simple_kernel<T, TW, EPI_STORE_F32><<<grid, 256, 0, s>>>(A, lda, W, W2, M, N, K, outF, outT, ldc); break;
        case EPI_STORE_T: gemm_simple_kernel<T, TW, EPI_STORE_T><<<grid, 256, 0, s>>>(A, lda, W, W2, M, N, K, outF, outT, ldc); break;
        case EPI_RESID: gemm_simple_kernel<T, TW, EPI_RESID><<<grid, 256, 0, s>>>(A, lda, W, W2, M, N, K, outF, outT, ldc); break;
        default: gemm_simple_kernel<T, TW, EPI_SWIGLU><<<grid, 256, 0, s>>>(A, lda, W, W2, M, N, K, outF, outT, ldc); break;
    }
}
void k_gemm_simple(int dtype, int epi, const void* A, int lda, const void* W, const void* W2, int M, int N, int K,
                   float* outF, void* outT, int ldc, hipStream_t s) {
    if (M <= 0 || N <= 0) return;
    if (dtype == 0) gemm_simple_t<float, float>(epi, (const float*)A, lda, (const float*)W, (const float*)W2, M, N, K, outF, (float*)outT, ldc, s);
    else gemm_simple_t<f16_t, bf16_t>(epi, (const f16_t*)A, lda, (const bf16_t*)W, (const bf16_t*)W2, M, N, K, outF, (f16_t*)outT, ldc, s);
}

// ---------------------------------------------------------------- RoPE + split + KV append
// qkv fp32 [n, (Hq+2Hkv) hd] -> rotated q (T) [n, Hq hd]; rotated k and plain v to the
// contiguous buffers (optional) and to the page slot of (slot, pos) (optional).
// With nsplit > 1 the row is the sum, in split order, of nsplit partial rows split_stride apart.
template <typename T>
__global__ __launch_bounds__(256) void rope_append_kernel(const float* qkv, int nsplit, int64_t split_stride,
                                                          const int* tok_pos, const int* tok_slot,
                                                          const float2* rope, T* q_out, T* k_out, T* v_out, T* pool,
                                                          int layer, KvGeom geo, const int* bt, int mpps, int Hq) {
    extern __shared__ float rowbuf[];
    const int n = blockIdx.x, hd = geo.hd, half = hd / 2, Hkv = geo.Hkv;
    const int pos = tok_pos[n];
    const int width = (Hq + 2 * Hkv) * hd;
    const float* row = qkv + (int64_t)n * width;
    if (nsplit > 1) {
        for (int i = threadIdx.x; i < width; i += 256) {
            float v = row[i];
            for (int sp = 1; sp < nsplit; ++sp) v += row[sp * split_stride + i];
            rowbuf[i] = v;
        }
        __syncthreads();
        row = rowbuf;
    }
    if (pos < 0) {   // parked / padding row: zero query, no key or value
        for (int i = threadIdx.x; i < Hq * hd; i += 256) q_out[(int64_t)n * Hq * hd + i] = from_f<T>(0.f);
        if (k_out) for (int i = threadIdx.x; i < Hkv * hd; i += 256) k_out[(int64_t)n * Hkv * hd + i] = from_f<T>(0.f);
        if (v_out) for (int i = threadIdx.x; i < Hkv * hd; i += 256) v_out[(int64_t)n * Hkv * hd + i] = from_f<T>(0.f);
        return;
    }
    const float2* rt = rope + (int64_t)pos * half;
    int64_t page = 0;
    int slot_tok = 0;
    if (pool) {
        page = bt[(int64_t)tok_slot[n] * mpps + pos / geo.PT];
        slot_tok = pos % geo.PT;
    }
    // q heads
    for (int i = threadIdx.x; i < Hq * half; i += 256) {
        int h = i / half, j = i % half;
        float a = row[h * hd + j], b = row[h * hd + j + half];
        float2 cs = rt[j];
        T* o = q_out + (int64_t)n * Hq * hd + h * hd;
        o[j] = from_f<T>(a * cs.x - b * cs.y);
        o[j + half] = from_f<T>(b * cs.x + a * cs.y);
    }
    // k heads
    const float* krow = row + Hq * hd;
    for (int i = threadIdx.x; i < Hkv * half; i += 256) {
        int g = i / half, j = i % half;
        float a = krow[g * hd + j], b = krow[g * hd + j + half];
        float2 cs = rt[j];
        T r0 = from_f<T>(a * cs.x - b * cs.y), r1 = from_f<T>(b * cs.x + a * cs.y);
        if (k_out) {
            T* o = k_out + (int64_t)n * Hkv * hd + g * hd;
            o[j] = r0; o[j + half] = r1;
        }
        if (pool) {
            pool[geo.k_off(layer, page, g, slot_tok, j)] = r0;
            pool[geo.k_off(layer, page, g, slot_tok, j + half)] = r1;
        }
    }
    // v heads
    const float* vrow = row + (Hq + Hkv) * hd;
    for (int i = threadIdx.x; i < Hkv * hd; i += 256) {
        int g = i / hd, dd = i % hd;
        T v = from_f<T>(vrow[i]);
        if (v_out) v_out[(int64_t)n * Hkv * hd + i] = v;
        if (pool) pool[geo.v_off(layer, page, g, slot_tok, dd)] = v;
    }
}
void k_rope_append(int dtype, const float* qkv, int nsplit, int64_t split_stride, int n, const int* tok_pos,
                   const int* tok_slot, const float2* rope, void* q_out, void* k_out, void* v_out, void* pool,
                   int layer, KvGeom geo, const int* block_table, int mpps, int Hq, hipStream_t s) {
    if (n <= 0) return;
    size_t lds = nsplit > 1 ? (size_t)(Hq + 2 * geo.Hkv) * geo.hd * sizeof(float) : 0;
    if (dtype == 0)
        rope_append_kernel<float><<<n, 256, lds, s>>>(qkv, nsplit, split_stride, tok_pos, tok_slot, rope,
                                                      (float*)q_out, (float*)k_out, (float*)v_out, (float*)pool,
                                                      layer, geo, block_table, mpps, Hq);
    else
        rope_append_kernel<f16_t><<<n, 256, lds, s>>>(qkv, nsplit, split_stride, tok_pos, tok_slot, rope,
                                                      (f16_t*)q_out, (f16_t*)k_out, (f16_t*)v_out, (f16_t*)pool,
                                                      layer, geo, block_table, mpps, Hq);
}

#define RL_MAX_SPLITS 16
// Decode variant: the qkv row arrives as nsplit split-K partial rows.  One block of 1024 threads
// per token; a thread owns (column j, column j + hd/2) pairs and requests every partial of a pair
// before summing them in split order.  Writes rotated q, and k / v into the page slot.
template <typename T>
__global__ __launch_bounds__(1024) void rope_append_split_kernel(const float* part, int nsplit, int64_t split_stride,
                                                                 const int* tok_pos, const int* tok_slot,
                                                                 const float2* rope, T* q_out, T* pool, int layer,
                                                                 KvGeom geo, const int* bt, int mpps, int Hq,
                                                                 int split, int layer_lo) {
    const int n = blockIdx.x, hd = geo.hd, half = hd / 2, Hkv = geo.Hkv;
    const int pos = tok_pos[n];
    const int width = (Hq + 2 * Hkv) * hd;
    const float* row = part + (int64_t)n * width;
    // split: q rows are fp16 pairs [Hq hd hi | Hq hd lo]; the lo planes of k and v go to layer_lo of the pool
    const int qw = (split ? 2 : 1) * Hq * hd;
    const int64_t lo_off = split ? (int64_t)(layer_lo - layer) * geo.layer_elems() : 0;
    if (pos < 0) {   // parked row: zero query, nothing appended to the cache
        for (int i = threadIdx.x; i < qw; i += 1024) q_out[(int64_t)n * qw + i] = from_f<T>(0.f);
        return;
    }
    const float2* rt = rope + (int64_t)pos * half;
    const int64_t page = bt[(int64_t)tok_slot[n] * mpps + pos / geo.PT];
    const int st = pos % geo.PT;
    // a thread owns four consecutive pairs (j .. j+3, and their partners j + hd/2 ..): 16-byte loads of every
    // split's partials, all requested before the first add
    const int nquads = (Hq + 2 * Hkv) * half / 4;
    for (int i = threadIdx.x; i < nquads; i += 1024) {
        const int head = i / (half / 4), j = (i % (half / 4)) * 4;
        const int c0 = head * hd + j;
        float a[4] = {0.f, 0.f, 0.f, 0.f}, b[4] = {0.f, 0.f, 0.f, 0.f};
        // eight splits at a time (their loads all in flight together), summed in split order
        for (int s0 = 0; s0 < nsplit; s0 += 8) {
            float4 p0[8], p1[8];
#pragma unroll
            for (int sp = 0; sp < 8; ++sp)
                if (s0 + sp < nsplit) {
                    p0[sp] = *reinterpret_cast<const float4*>(row + (s0 + sp) * split_stride + c0);
                    p1[sp] = *reinterpret_cast<const float4*>(row + (s0 + sp) * split_stride + c0 + half);
                }
#pragma unroll
            for (int sp = 0; sp < 8; ++sp)
                if (s0 + sp < nsplit) {
                    a[0] += p0[sp].x; a[1] += p0[sp].y; a[2] += p0[sp].z; a[3] += p0[sp].w;
                    b[0] += p1[sp].x; b[1] += p1[sp].y; b[2] += p1[sp].z; b[3] += p1[sp].w;
                }
        }
        if (head < Hq + Hkv) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float2 cs = rt[j + t];
                const float r0 = a[t] * cs.x - b[t] * cs.y, r1 = b[t] * cs.x + a[t] * cs.y;
                a[t] = r0; b[t] = r1;
            }
        }
        if (head < Hq) {
            T* o = q_out + (int64_t)n * qw + head * hd + j;
#pragma unroll
            for (int t = 0; t < 4; ++t) { put_pair(o + t, Hq * hd, a[t], split); put_pair(o + half + t, Hq * hd, b[t], split); }
        } else if (head < Hq + Hkv) {
            const int g = head - Hq;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                put_pair(pool + geo.k_off(layer, page, g, st, j + t), lo_off, a[t], split);
                put_pair(pool + geo.k_off(layer, page, g, st, j + t + half), lo_off, b[t], split);
            }
        } else {
            const int g = head - Hq - Hkv;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                put_pair(pool + geo.v_off(layer, page, g, st, j + t), lo_off, a[t], split);
                put_pair(pool + geo.v_off(layer, page, g, st, j + t + half), lo_off, b[t], split);
            }
        }
    }
}
void k_rope_append_split(int dtype, const float* part, int nsplit, int64_t split_stride, int n, const int* tok_pos,
                         const int* tok_slot, const float2* rope, void* q_out, void* pool, int layer, KvGeom geo,
                         const int* block_table, int mpps, int Hq, hipStream_t s, int split, int layer_lo) {
    if (n <= 0) return;
    if (dtype == 0)
        rope_append_split_kernel<float><<<n, 1024, 0, s>>>(part, nsplit, split_stride, tok_pos, tok_slot, rope,
                                                           (float*)q_out, (float*)pool, layer, geo, block_table, mpps, Hq, 0, layer);
    else
        rope_append_split_kernel<f16_t><<<n, 1024, 0, s>>>(part, nsplit, split_stride, tok_pos, tok_slot, rope,
                                                           (f16_t*)q_out, (f16_t*)pool, layer, geo, block_table, mpps, Hq,
                                                           split, layer_lo);
}

// ---------------------------------------------------------------- split-K reduce + residual add + RMSNorm
// x[n,:] += sum_s part[s][n,:] (split order);  out[n,:] = RMSNorm(x[n,:]; g).  One block of 1024
// threads per row; every thread owns float4 columns and requests all split partials of a column
// before adding them (in split order), so the row costs about one memory round trip.
template <typename T, typename TW>
__global__ __launch_bounds__(1024) void resid_norm_kernel(float* x, const float* part, int nsplit, int64_t split_stride,
                                                          const TW* g, T* out, int d, float eps, int split) {
    __shared__ float red[16];
    const int n = blockIdx.x;
    float* xr = x + (int64_t)n * d;
    const float* pr = part + (int64_t)n * d;
    float4 keep[2];
    float ss = 0.f;
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int j = (it * 1024 + threadIdx.x) * 4;
        if (j < d) {
            float4 v = *reinterpret_cast<const float4*>(xr + j);
            float4 p[RL_MAX_SPLITS];
#pragma unroll
            for (int sp = 0; sp < RL_MAX_SPLITS; ++sp)
                if (sp < nsplit) p[sp] = *reinterpret_cast<const float4*>(pr + sp * split_stride + j);
#pragma unroll
            for (int sp = 0; sp < RL_MAX_SPLITS; ++sp)
                if (sp < nsplit) { v.x += p[sp].x; v.y += p[sp].y; v.z += p[sp].z; v.w += p[sp].w; }
            *reinterpret_cast<float4*>(xr + j) = v;
            keep[it] = v;
            ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
        }
    }
    ss = block_sum(ss, red);
    const float rs = 1.0f / sqrtf(ss / (float)d + eps);
    T* o = out + (int64_t)n * d * (split ? 2 : 1);   // split: [d values rounded to T | d remainders]
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int j = (it * 1024 + threadIdx.x) * 4;
        if (j < d) put_pair4(o + j, d, keep[it], rs, g + j, split);
    }
}
// d must be a multiple of 4 and at most 8192; nsplit at most RL_MAX_SPLITS.
void k_resid_norm(int dtype, float* x, const float* part, int nsplit, int64_t split_stride, const void* g, void* out,
                  int n, int d, float eps, hipStream_t s, int split) {
    if (n <= 0) return;
    if (dtype == 0)
        resid_norm_kernel<float, float><<<n, 1024, 0, s>>>(x, part, nsplit, split_stride, (const float*)g, (float*)out, d, eps, 0);
    else
        resid_norm_kernel<f16_t, bf16_t><<<n, 1024, 0, s>>>(x, part, nsplit, split_stride, (const bf16_t*)g, (f16_t*)out, d, eps, split);
}

// ---------------------------------------------------------------- plain attention
// One block per (query token, query head).  Keys 0..pos of the query's own sequence,
// read either from contiguous [tokens, Hkv, hd] buffers (the sequence's tokens are
// consecutive, so key m sits at row n - pos + m) or from the paged pool.
template <typename T>
__global__ __launch_bounds__(256) void attn_simple_kernel(const T* q, const T* kc, const T* vc, const T* pool,
                                                          int layer, KvGeom geo, const int* bt, int mpps,
                                                          const int* tok_pos, const int* tok_slot, T* out, int Hq) {
    extern __shared__ float sm[];
    const int hd = geo.hd, Hkv = geo.Hkv;
    const int n = blockIdx.x, h = blockIdx.y, g = h / (Hq / Hkv);
    const int pos = tok_pos[n], ctx = pos + 1;
    if (ctx <= 0) {            // parked row (position -1): no keys, zeros
        if (threadIdx.x < hd) out[((int64_t)n * Hq + h) * hd + threadIdx.x] = from_f<T>(0.f);
        return;
    }
    float* qs = sm;            // [hd]
    float* red = sm + hd;      // [16]
    float* part = red + 16;    // [256]
    float* sc = part + 256;    // [ctx]
    const int* btr = pool ? bt + (int64_t)tok_slot[n] * mpps : nullptr;
    for (int j = threadIdx.x; j < hd; j += 256) qs[j] = to_f(q[((int64_t)n * Hq + h) * hd + j]);
    __syncthreads();
    const float scale = 1.0f / sqrtf((float)hd);
    float lmax = -INFINITY;
    for (int m = threadIdx.x; m < ctx; m += 256) {
        float dot = 0.f;
        if (pool) {
            int64_t base = geo.k_off(layer, btr[m / geo.PT], g, m % geo.PT, 0);
            for (int j = 0; j < hd; ++j) dot += qs[j] * to_f(pool[base + j]);
        } else {
            const T* kr = kc + ((int64_t)(n - pos + m) * Hkv + g) * hd;
            for (int j = 0; j < hd; ++j) dot += qs[j] * to_f(kr[j]);
        }
        dot *= scale;
        sc[m] = dot;
        lmax = fmaxf(lmax, dot);
    }
    float mx = block_max(lmax, red);
    float ls = 0.f;
    for (int m = threadIdx.x; m < ctx; m += 256) { float e = __expf(sc[m] - mx); sc[m] = e; ls += e; }
    float tot = block_sum(ls, red);   // has barriers: sc[] visible afterwards
    const int dd = threadIdx.x % hd, grp = threadIdx.x / hd, ngrp = 256 / hd;
    float acc = 0.f;
    for (int m = grp; m < ctx; m += ngrp) {
        float v;
        if (pool) v = to_f(pool[geo.v_off(layer, btr[m / geo.PT], g, m % geo.PT, dd)]);
        else v = to_f(vc[((int64_t)(n - pos + m) * Hkv + g) * hd + dd]);
        acc += sc[m] * v;
    }
    part[threadIdx.x] = acc;
    __syncthreads();
    if (threadIdx.x < hd) {
        float o = 0.f;
        for (int i = 0; i < ngrp; ++i) o += part[i * hd + threadIdx.x];
        out[((int64_t)n * Hq + h) * hd + threadIdx.x] = from_f<T>(o / tot);
    }
}
void k_attn_simple(int dtype, const void* q, const void* kc, const void* vc, const void* pool, int layer, KvGeom geo,
                   const int* block_table, int mpps, const int* tok_pos, const int* tok_slot, void* out, int n,
                   int Hq, int max_ctx, hipStream_t s) {
    if (n <= 0) return;
    size_t lds = (size_t)(geo.hd + 16 + 256 + max_ctx) * sizeof(float);
    dim3 grid(n, Hq);
    if (dtype == 0)
        attn_simple_kernel<float><<<grid, 256, lds, s>>>((const float*)q, (const float*)kc, (const float*)vc,
                                                         (const float*)pool, layer, geo, block_table, mpps, tok_pos,
                                                         tok_slot, (float*)out, Hq);
    else
        attn_simple_kernel<f16_t><<<grid, 256, lds, s>>>((const f16_t*)q, (const f16_t*)kc, (const f16_t*)vc,
                                                         (const f16_t*)pool, layer, geo, block_table, mpps, tok_pos,
                                                         tok_slot, (f16_t*)out, Hq);
}

// ---------------------------------------------------------------- sampling
// Counter-based uniform: two rounds of the splitmix64 output function over
// (seed, sequence id, step); top 24 bits -> [0,1).  Integer-only, so the CPU
// checker reproduces it bit for bit.
__device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
__device__ __forceinline__ float hash_uniform(uint64_t seed, uint64_t seq, uint64_t step) {
    const uint64_t G = 0x9E3779B97F4A7C15ull;
    uint64_t h = mix64(seed + G * (seq + 1));
    h = mix64(h + G * (step + 1));
    return (float)(h >> 40) * (1.0f / 16777216.0f);
}

// Row statistics shared by sampling and scoring: max, arg-max (lowest index on ties).
struct ArgMax { float v; int i; };
__device__ __forceinline__ ArgMax argmax_combine(ArgMax a, ArgMax b) {
    if (b.v > a.v || (b.v == a.v && b.i < a.i)) return b;
    return a;
}
__device__ ArgMax block_argmax(const float* z, int V, ArgMax* red) {
    ArgMax a{-INFINITY, 0x7fffffff};
    if ((V & 3) == 0 && (reinterpret_cast<uintptr_t>(z) & 15) == 0) {
        // 16-byte loads; a thread meets its candidates in increasing index order, so "first strictly greater"
        // keeps the lowest index among equals
        const float4* z4 = reinterpret_cast<const float4*>(z);
        for (int i = threadIdx.x; i < V / 4; i += blockDim.x) {
            const float4 q = z4[i];
            if (q.x > a.v) { a.v = q.x; a.i = 4 * i; }
            if (q.y > a.v) { a.v = q.y; a.i = 4 * i + 1; }
            if (q.z > a.v) { a.v = q.z; a.i = 4 * i + 2; }
            if (q.w > a.v) { a.v = q.w; a.i = 4 * i + 3; }
        }
    } else {
        for (int i = threadIdx.x; i < V; i += blockDim.x) {
            float v = z[i];
            if (v > a.v) { a.v = v; a.i = i; }
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        ArgMax b{__shfl_xor(a.v, o, RL_WAVE), __shfl_xor(a.i, o, RL_WAVE)};
        a = argmax_combine(a, b);
    }
    const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    if ((threadIdx.x & 63) == 0) red[w] = a;
    __syncthreads();
    ArgMax r = red[0];
    for (int i = 1; i < nw; ++i) r = argmax_combine(r, red[i]);
    __syncthreads();
    return r;
}

// One block of 1024 threads per sequence.  Wave w owns the contiguous vocabulary
// segment [w*seg, (w+1)*seg); sums are formed lane-column-wise then reduced, in a
// fixed order, so results are reproducible run to run.
// out_ids / out_logp (optional) are [B, out_stride]; the column is the sequence's decode-step
// counter, kept on the device so that a captured step can be replayed unchanged.
__global__ __launch_bounds__(1024) void sample_kernel(const float* logits, int ldz, int V, SampleArgs a, int* last_tok,
                                                      int* seq_len, int* gen_count, int* finished, int* step_count,
                                                      int* tok_out, float* logp_out, int* out_ids, float* out_logp,
                                                      int out_stride) {
    __shared__ ArgMax ared[16];
    __shared__ float ws1[16], wsT[16];
    __shared__ int s_tok;
    const int b = blockIdx.x;
    const int64_t orow = a.out_row ? a.out_row[b] : b;
    if (finished[b] != 0) {
        // a finished sequence keeps emitting eos_id with log-prob 0 and no longer advances
        if (threadIdx.x == 0) {
            last_tok[b] = a.eos_id >= 0 ? a.eos_id : 0;   // a parked row still feeds a valid id through the GEMMs
            if (tok_out) tok_out[b] = a.eos_id;
            if (logp_out) logp_out[b] = 0.f;
            const int st = step_count[b];
            step_count[b] = st + 1;
            if (st < out_stride) {
                if (out_ids) out_ids[orow * out_stride + st] = a.eos_id;
                if (out_logp) out_logp[orow * out_stride + st] = 0.f;
            }
        }
        return;
    }
    const float* z = logits + (int64_t)b * ldz;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    ArgMax am = block_argmax(z, V, ared);
    const float mx = am.v;
    const bool greedy = !(a.temperature > 0.f);
    const float invT = greedy ? 1.0f : 1.0f / a.temperature;
    int seg = (V + 15) / 16;
    seg = (seg + 255) / 256 * 256;
    const int s0 = w * seg, s1 = min(V, s0 + seg);
    float c1 = 0.f, cT = 0.f;
    if ((V & 3) == 0 && (reinterpret_cast<uintptr_t>(z) & 15) == 0) {
        const float4* z4 = reinterpret_cast<const float4*>(z);
        for (int i = s0 / 4 + lane; i < s1 / 4; i += 64) {
            const float4 q = z4[i];
            const float d0 = q.x - mx, d1 = q.y - mx, d2 = q.z - mx, d3 = q.w - mx;
            c1 += (__expf(d0) + __expf(d1)) + (__expf(d2) + __expf(d3));
            cT += (__expf(d0 * invT) + __expf(d1 * invT)) + (__expf(d2 * invT) + __expf(d3 * invT));
        }
    } else {
        for (int i = s0 + lane; i < s1; i += 64) {
            float dz = z[i] - mx;
            c1 += __expf(dz);
            cT += __expf(dz * invT);
        }
    }
    c1 = wave_sum(c1);
    cT = wave_sum(cT);
    if (lane == 0) { ws1[w] = c1; wsT[w] = cT; }
    if (threadIdx.x == 0) s_tok = greedy ? am.i : V - 1;
    __syncthreads();
    float tot1 = 0.f, totT = 0.f;
    for (int i = 0; i < 16; ++i) { tot1 += ws1[i]; totT += wsT[i]; }
    const int n_gen = gen_count[b];
    if (!greedy) {
        float u = hash_uniform(a.seed, (uint64_t)(a.seq_base + (a.seq_id ? a.seq_id[b] : b)), (uint64_t)n_gen);
        float target = u * totT;
        float cum = 0.f;
        int wsel = -1;
        float before = 0.f;
        for (int i = 0; i < 16; ++i) {
            float nc = cum + wsT[i];
            if (wsel < 0 && nc > target) { wsel = i; before = cum; }
            cum = nc;
        }
        if (w == wsel) {
            float run = before;
            int found = -1;
            for (int r0 = s0; r0 < s1 && found < 0; r0 += 64) {
                int i = r0 + lane;
                float e = (i < s1) ? __expf((z[i] - mx) * invT) : 0.f;
                float rowsum = wave_sum(e);
                if (run + rowsum > target) {
                    float pe = e;   // inclusive prefix over lanes
#pragma unroll
                    for (int o = 1; o < 64; o <<= 1) {
                        float t = __shfl_up(pe, o, RL_WAVE);
                        if (lane >= o) pe += t;
                    }
                    unsigned long long m = __ballot((run + pe > target) && (i < s1));
                    if (m) found = r0 + __ffsll((long long)m) - 1;
                    else run += rowsum;
                } else {
                    run += rowsum;
                }
            }
            if (found < 0) found = s1 - 1;   // crossing falls on the segment end within rounding
            if (lane == 0) s_tok = found;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        const int tok = s_tok;
        const float lp = z[tok] - mx - logf(tot1);
        gen_count[b] = n_gen + 1;
        if ((a.eos_id >= 0 && tok == a.eos_id) || (a.gen_limit && n_gen + 1 >= a.gen_limit[b])) {
            finished[b] = 1;
            if (a.out_len) a.out_len[orow] = n_gen + 1;
        }
        last_tok[b] = tok;
        seq_len[b] = seq_len[b] + 1;
        if (tok_out) tok_out[b] = tok;
        if (logp_out) logp_out[b] = lp;
        const int st = step_count[b];
        step_count[b] = st + 1;
        if (st < out_stride) {
            if (out_ids) out_ids[orow * out_stride + st] = tok;
            if (out_logp) out_logp[orow * out_stride + st] = lp;
        }
    }
}
void k_sample(const float* logits, int ldz, int V, int B, SampleArgs a, int* last_tok, int* seq_len, int* gen_count,
              int* finished, int* step_count, int* tok_out, float* logp_out, int* out_ids, float* out_logp,
              int out_stride, hipStream_t s) {
    if (B <= 0) return;
    sample_kernel<<<B, 1024, 0, s>>>(logits, ldz, V, a, last_tok, seq_len, gen_count, finished, step_count, tok_out,
                                     logp_out, out_ids, out_logp, out_stride);
}

// The same draw from per-block statistics instead of logits (the LM-head GEMM's MG_SAMPLE epilogue: per row and
// 32-column block the maximum, its column, and the sums of exp((z - max) / T) and exp(z - max)): the logits of a decode
// step never reach memory.  One block of 1024 threads per sequence; thread t owns the contiguous run of blocks
// [t * per, (t + 1) * per), sums are formed in block order and scanned in thread order, so results are
// reproducible run to run.  Greedy: the first block holding the global maximum, and its column.  Otherwise the
// block in which the cumulative sum passes u * total is found from the statistics, and only that block's 32
// logits are recomputed (h . W rows, fp32 accumulation) to place the token inside it; if rounding differences between
// those 32 values and the block's own sum keep the cumulative sum from passing the target inside the block, the
// block's last column is taken (the crossing then lies on the block's end within rounding).
__global__ __launch_bounds__(1024) void sample_blocks_kernel(const float4* stats, int nblk, const f16_t* h, int ldh,
                                                             const bf16_t* W, int d, SampleArgs a, int* last_tok,
                                                             int* seq_len, int* gen_count, int* finished,
                                                             int* step_count, int* tok_out, float* logp_out,
                                                             int* out_ids, float* out_logp, int out_stride) {
    __shared__ ArgMax ared[16];
    __shared__ float red1[16], redT[16], zs[32];
    __shared__ int s_first, s_blk, s_tok;
    __shared__ float s_before, s_ztok;
    const int b = blockIdx.x;
    const int64_t orow = a.out_row ? a.out_row[b] : b;
    if (finished[b] != 0) {
        // a finished sequence keeps emitting eos_id with log-prob 0 and no longer advances
        if (threadIdx.x == 0) {
            last_tok[b] = a.eos_id >= 0 ? a.eos_id : 0;   // a parked row still feeds a valid id through the GEMMs
            if (tok_out) tok_out[b] = a.eos_id;
            if (logp_out) logp_out[b] = 0.f;
            const int st = step_count[b];
            step_count[b] = st + 1;
            if (st < out_stride) {
                if (out_ids) out_ids[orow * out_stride + st] = a.eos_id;
                if (out_logp) out_logp[orow * out_stride + st] = 0.f;
            }
        }
        return;
    }
    const float4* st4 = stats + (int64_t)b * nblk;
    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    const int per = (nblk + 1023) / 1024;
    const int b0 = min(nblk, t * per), b1 = min(nblk, b0 + per);
    const bool greedy = !(a.temperature > 0.f);
    const float invT = greedy ? 1.0f : 1.0f / a.temperature;
    // global maximum and the first block that holds it
    ArgMax am{-INFINITY, 0x7fffffff};
    for (int i = b0; i < b1; ++i) {
        const float v = st4[i].x;
        if (v > am.v) { am.v = v; am.i = i; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        ArgMax o2{__shfl_xor(am.v, o, RL_WAVE), __shfl_xor(am.i, o, RL_WAVE)};
        am = argmax_combine(am, o2);
    }
    if (lane == 0) ared[w] = am;
    if (t == 0) { s_first = 0x7fffffff; s_blk = nblk - 1; s_before = 0.f; }
    __syncthreads();
    am = ared[0];
    for (int i = 1; i < 16; ++i) am = argmax_combine(am, ared[i]);
    const float mx = am.v;
    // this thread's share of both sums, then an inclusive scan of the temperature sum over the threads
    float l1 = 0.f, lT = 0.f;
    for (int i = b0; i < b1; ++i) {
        const float4 q = st4[i];
        l1 += q.z * __expf(q.x - mx);
        lT += q.y * __expf((q.x - mx) * invT);
    }
    float pT = lT;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const float u_ = __shfl_up(pT, o, RL_WAVE);
        if (lane >= o) pT += u_;
    }
    const float w1 = wave_sum(l1);
    if (lane == 63) redT[w] = pT;
    if (lane == 0) red1[w] = w1;
    __syncthreads();
    float tot1 = 0.f, totT = 0.f, baseT = 0.f;
    for (int i = 0; i < 16; ++i) {
        if (i == w) baseT = totT;
        tot1 += red1[i];
        totT += redT[i];
    }
    const float up1 = __shfl_up(pT, 1, RL_WAVE);
    const float incl = baseT + pT, excl = baseT + (lane > 0 ? up1 : 0.f);   // excl of thread t == incl of thread t - 1, bit for bit
    const int n_gen = gen_count[b];
    float target = 0.f;
    if (!greedy) {
        const float u = hash_uniform(a.seed, (uint64_t)(a.seq_base + (a.seq_id ? a.seq_id[b] : b)), (uint64_t)n_gen);
        target = u * totT;
        if (b0 < b1 && incl > target) atomicMin(&s_first, t);
        __syncthreads();
        if (t == s_first) {
            // the scan says this thread's run of blocks holds the crossing; summed block by block it may fall just
            // short of it within rounding: then the run's last block takes it
            float cum = excl;
            int sel = b1 - 1;
            for (int i = b0; i < b1; ++i) {
                const float4 q = st4[i];
                const float nc = cum + q.y * __expf((q.x - mx) * invT);
                if (nc > target || i == b1 - 1) { sel = i; break; }
                cum = nc;
            }
            s_blk = sel;
            s_before = cum;
        }
        __syncthreads();
        // the 32 logits of the chosen block: column t / 32, 32 threads per column over 16-byte pieces of k
        const int blk = s_blk;
        const int col = t >> 5, part = t & 31;
        const bf16_t* wrow = W + ((int64_t)blk * 32 + col) * d;
        const f16_t* hrow = h + (int64_t)b * ldh;
        float acc = 0.f;
        for (int k = part * 8; k < d; k += 256) {
            typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
            typedef unsigned short us8_t __attribute__((ext_vector_type(8)));
            const half8_t hv = *reinterpret_cast<const half8_t*>(hrow + k);
            const us8_t wv = *reinterpret_cast<const us8_t*>(wrow + k);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc += (float)hv[e] * __uint_as_float((unsigned)wv[e] << 16);
        }
#pragma unroll
        for (int o = 1; o < 32; o <<= 1) acc += __shfl_xor(acc, o, RL_WAVE);
        if (part == 0) zs[col] = acc;
        __syncthreads();
        if (t < 64) {
            const float e = t < 32 ? __expf((zs[t & 31] - mx) * invT) : 0.f;
            float pe = e;
#pragma unroll
            for (int o = 1; o < 32; o <<= 1) {
                const float u_ = __shfl_up(pe, o, RL_WAVE);
                if (lane >= o) pe += u_;
            }
            const unsigned long long hit = __ballot(t < 32 && s_before + pe > target);
            if (t == 0) {
                const int c = hit ? __ffsll((long long)hit) - 1 : 31;
                s_tok = blk * 32 + c;
                s_ztok = zs[c];
            }
        }
    } else if (t == 0) {
        s_tok = am.i * 32 + __float_as_int(st4[am.i].w);
        s_ztok = mx;
    }
    __syncthreads();
    if (t == 0) {
        const int tok = s_tok;
        const float lp = s_ztok - mx - logf(tot1);
        gen_count[b] = n_gen + 1;
        if ((a.eos_id >= 0 && tok == a.eos_id) || (a.gen_limit && n_gen + 1 >= a.gen_limit[b])) {
            finished[b] = 1;
            if (a.out_len) a.out_len[orow] = n_gen + 1;
        }
        last_tok[b] = tok;
        seq_len[b] = seq_len[b] + 1;
        if (tok_out) tok_out[b] = tok;
        if (logp_out) logp_out[b] = lp;
        const int st = step_count[b];
        step_count[b] = st + 1;
        if (st < out_stride) {
            if (out_ids) out_ids[orow * out_stride + st] = tok;
            if (out_logp) out_logp[orow * out_stride + st] = lp;
        }
    }
}
void k_sample_blocks(const float4* stats, int V, const void* h, int ldh, const void* W, int d, int B, SampleArgs a,
                     int* last_tok, int* seq_len, int* gen_count, int* finished, int* step_count, int* tok_out,
                     float* logp_out, int* out_ids, float* out_logp, int out_stride, hipStream_t s) {
    if (B <= 0) return;
    sample_blocks_kernel<<<B, 1024, 0, s>>>(stats, V / 32, (const f16_t*)h, ldh, (const bf16_t*)W, d, a, last_tok, seq_len,
                                            gen_count, finished, step_count, tok_out, logp_out, out_ids, out_logp,
                                            out_stride);
}

// ---------------------------------------------------------------- log-sum-exp + gather over materialised logits
// logp_out[slot, pos + 1] = z[target] - log sum_v exp(z_v) for rows with a target.
__global__ __launch_bounds__(1024) void lse_gather_kernel(const float* logits, int ldz, int V, const int* tok_tgt,
                                                          const int* tok_slot, const int* tok_pos, float* logp_out,
                                                          int ld_out) {
    __shared__ float red[16];
    const int r = blockIdx.x;
    const int tgt = tok_tgt[r];
    if (tgt < 0) return;
    const float* z = logits + (int64_t)r * ldz;
    float m = -INFINITY;
    for (int i = threadIdx.x; i < V; i += 1024) m = fmaxf(m, z[i]);
    m = block_max(m, red);
    float su = 0.f;
    for (int i = threadIdx.x; i < V; i += 1024) su += __expf(z[i] - m);
    su = block_sum(su, red);
    if (threadIdx.x == 0) {
        int t = min(max(tgt, 0), V - 1);
        logp_out[(int64_t)tok_slot[r] * ld_out + tok_pos[r] + 1] = z[t] - m - logf(su);
    }
}
void k_lse_gather(const float* logits, int ldz, int V, int nrows, const int* tok_tgt, const int* tok_slot,
                  const int* tok_pos, float* logp_out, int ld_out, hipStream_t s) {
    if (nrows <= 0) return;
    lse_gather_kernel<<<nrows, 1024, 0, s>>>(logits, ldz, V, tok_tgt, tok_slot, tok_pos, logp_out, ld_out);
}

// ---------------------------------------------------------------- KL term on response positions
__global__ void kl_kernel(const float* lp, const float* lr, const int* seq_len, const int* prompt_len, int Lmax,
                          float coef, float* kl, float* pen) {
    int b = blockIdx.y;
    int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= Lmax) return;
    int64_t o = (int64_t)b * Lmax + t;
    int lo = max(prompt_len[b], 1);
    float v = (t >= lo && t < seq_len[b]) ? lp[o] - lr[o] : 0.f;
    if (kl) kl[o] = v;
    if (pen) pen[o] = coef * v;
}
void k_kl(const float* lp, const float* lr, const int* seq_len, const int* prompt_len, int B, int Lmax, float coef,
          float* kl, float* pen, hipStream_t s) {
    if (B <= 0 || Lmax <= 0) return;
    dim3 grid((Lmax + 255) / 256, B);
    kl_kernel<<<grid, 256, 0, s>>>(lp, lr, seq_len, prompt_len, Lmax, coef, kl, pen);
}

// ---------------------------------------------------------------- value head of a critic / reward model
// v[slot, pos] = head . RMSNorm(x_row; g) for every packed row with pos >= 0: the final norm and the
// [d] -> 1 head in one pass over the fp32 residual stream (nothing is rounded to fp16 on the way).
template <typename TW>
__global__ __launch_bounds__(256) void value_head_kernel(const float* x, const TW* g, const TW* head, int d, float eps,
                                                         const int* tok_slot, const int* tok_pos, float* out,
                                                         int ld_out) {
    __shared__ float red[16];
    const int n = blockIdx.x;
    const int pos = tok_pos[n];
    if (pos < 0) return;
    const float* xr = x + (int64_t)n * d;
    float ss = 0.f, dot = 0.f;
    for (int j = threadIdx.x; j < d; j += 256) {
        const float v = xr[j];
        ss += v * v;
        dot += v * to_f(g[j]) * to_f(head[j]);
    }
    ss = block_sum(ss, red);
    dot = block_sum(dot, red);
    if (threadIdx.x == 0) out[(int64_t)tok_slot[n] * ld_out + pos] = dot / sqrtf(ss / (float)d + eps);
}
void k_value_head(int dtype, const float* x, const void* g, const void* head, int n, int d, float eps,
                  const int* tok_slot, const int* tok_pos, float* out, int ld_out, hipStream_t s) {
    if (n <= 0) return;
    if (dtype == 0)
        value_head_kernel<float><<<n, 256, 0, s>>>(x, (const float*)g, (const float*)head, d, eps, tok_slot, tok_pos, out, ld_out);
    else
        value_head_kernel<bf16_t><<<n, 256, 0, s>>>(x, (const bf16_t*)g, (const bf16_t*)head, d, eps, tok_slot, tok_pos, out, ld_out);
}

// ---------------------------------------------------------------- PPO reward per token
// r[b,t] = -coef * kl[b,t] on response positions [prompt_len, L), plus seq_reward[b] at t = L-1; 0 elsewhere.
__global__ void ppo_reward_kernel(const float* kl, const float* seq_reward, const int* seq_len, const int* prompt_len,
                                  int Lmax, float coef, float* out) {
    int b = blockIdx.y;
    int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= Lmax) return;
    const int64_t o = (int64_t)b * Lmax + t;
    const int L = seq_len[b], P = prompt_len[b];
    float r = 0.f;
    if (t >= P && t < L) {
        r = -coef * kl[o];
        if (t == L - 1) r += seq_reward[b];
    }
    out[o] = r;
}
// dst[first + i] = v[i] for i < n <= 192: small host arrays reach the device as kernel arguments (no copy engine,
// no pinned staging), 192 values per launch.
struct IntChunk { int v[192]; };
__global__ void put_i32_kernel(int* dst, IntChunk c, int n) {
    if ((int)threadIdx.x < n) dst[threadIdx.x] = c.v[threadIdx.x];
}
void k_put_i32(int* dst, const int* src_host, int n, hipStream_t s) {
    for (int o = 0; o < n; o += 192) {
        IntChunk c;
        const int m = n - o < 192 ? n - o : 192;
        for (int i = 0; i < m; ++i) c.v[i] = src_host[o + i];
        put_i32_kernel<<<1, 192, 0, s>>>(dst + o, c, m);
    }
}

void k_ppo_reward(const float* kl, const float* seq_reward, const int* seq_len, const int* prompt_len, int B, int Lmax,
                  float coef, float* out, hipStream_t s) {
    if (B <= 0 || Lmax <= 0) return;
    dim3 grid((Lmax + 255) / 256, B);
    ppo_reward_kernel<<<grid, 256, 0, s>>>(kl, seq_reward, seq_len, prompt_len, Lmax, coef, out);
}

// ---------------------------------------------------------------- exact KL from per-group partials
// One wave per row: combine the nparts quintuples (m_p, S_p, T, m_r, S_r) written by the dual LM-head GEMM
// into KL(pi_policy || pi_ref) = T/S_p - lse_p + lse_r and write it at [slot, pos + 1] on response
// positions (pos + 1 >= max(prompt_len, 1)); rows without a next token inside their sequence are skipped.
__global__ __launch_bounds__(64) void kl_full_reduce_kernel(const float* part, int nparts, const int* tok_tgt,
                                                            const int* tok_slot, const int* tok_pos,
                                                            const int* prompt_len, float* out, int ld_out) {
    const int r = blockIdx.x;
    if (tok_tgt[r] < 0) return;
    const int slot = tok_slot[r], t = tok_pos[r] + 1;
    if (t < max(prompt_len[slot], 1)) return;
    const float* p = part + (int64_t)r * nparts * 5;
    float mp = -INFINITY, sp = 0.f, tt = 0.f, mr = -INFINITY, sr = 0.f;
    for (int i = threadIdx.x; i < nparts; i += 64) {
        const float m1 = p[i * 5], s1 = p[i * 5 + 1], t1 = p[i * 5 + 2], m2 = p[i * 5 + 3], s2 = p[i * 5 + 4];
        const float mn = fmaxf(mp, m1), a0 = __expf(mp - mn), a1 = __expf(m1 - mn);
        sp = sp * a0 + s1 * a1;
        tt = tt * a0 + t1 * a1;
        mp = mn;
        const float mq = fmaxf(mr, m2);
        sr = sr * __expf(mr - mq) + s2 * __expf(m2 - mq);
        mr = mq;
    }
    const float Mp = wave_max(mp), Mr = wave_max(mr);
    const float wp = __expf(mp - Mp);
    sp = wave_sum(sp * wp);
    tt = wave_sum(tt * wp);
    sr = wave_sum(sr * __expf(mr - Mr));
    if (threadIdx.x == 0) out[(int64_t)slot * ld_out + t] = tt / sp - (Mp + logf(sp)) + (Mr + logf(sr));
}
void k_kl_full_reduce(const float* part, int nparts, int nrows, const int* tok_tgt, const int* tok_slot,
                      const int* tok_pos, const int* prompt_len, float* out, int ld_out, hipStream_t s) {
    if (nrows <= 0) return;
    kl_full_reduce_kernel<<<nrows, 64, 0, s>>>(part, nparts, tok_tgt, tok_slot, tok_pos, prompt_len, out, ld_out);
}

// The same from two materialised logit rows (plain path): one block per row.
__global__ __launch_bounds__(1024) void kl_full_rows_kernel(const float* zp, const float* zr, int ldz, int V,
                                                            const int* tok_tgt, const int* tok_slot,
                                                            const int* tok_pos, const int* prompt_len, float* out,
                                                            int ld_out) {
    __shared__ float red[16];
    const int r = blockIdx.x;
    if (tok_tgt[r] < 0) return;
    const int slot = tok_slot[r], t = tok_pos[r] + 1;
    if (t < max(prompt_len[slot], 1)) return;
    const float* a = zp + (int64_t)r * ldz;
    const float* b = zr + (int64_t)r * ldz;
    float mp = -INFINITY, mr = -INFINITY;
    for (int i = threadIdx.x; i < V; i += 1024) { mp = fmaxf(mp, a[i]); mr = fmaxf(mr, b[i]); }
    mp = block_max(mp, red);
    mr = block_max(mr, red);
    float sp = 0.f, tt = 0.f, sr = 0.f;
    for (int i = threadIdx.x; i < V; i += 1024) {
        const float e = __expf(a[i] - mp);
        sp += e;
        tt += e * (a[i] - b[i]);
        sr += __expf(b[i] - mr);
    }
    sp = block_sum(sp, red);
    tt = block_sum(tt, red);
    sr = block_sum(sr, red);
    if (threadIdx.x == 0) out[(int64_t)slot * ld_out + t] = tt / sp - (mp + logf(sp)) + (mr + logf(sr));
}
void k_kl_full_rows(const float* zp, const float* zr, int ldz, int V, int nrows, const int* tok_tgt,
                    const int* tok_slot, const int* tok_pos, const int* prompt_len, float* out, int ld_out,
                    hipStream_t s) {
    if (nrows <= 0) return;
    kl_full_rows_kernel<<<nrows, 1024, 0, s>>>(zp, zr, ldz, V, tok_tgt, tok_slot, tok_pos, prompt_len, out, ld_out);
}

// ---------------------------------------------------------------- log-prob from per-group (max, sum-exp) partials
// One wave per row: combine the nparts pairs written by the LM-head GEMM epilogue into
// log sum_v exp(z_v) and write logp = z_target - lse at [slot, pos + 1].
__global__ __launch_bounds__(64) void lse_reduce_kernel(const float2* part, int nparts, const float* z_tgt,
                                                        const int* tok_tgt, const int* tok_slot, const int* tok_pos,
                                                        float* logp_out, int ld_out) {
    const int r = blockIdx.x;
    if (tok_tgt[r] < 0) return;
    const float2* p = part + (int64_t)r * nparts;
    float m = -INFINITY, s = 0.f;
    for (int i = threadIdx.x; i < nparts; i += 64) {
        float2 v = p[i];
        float mn = fmaxf(m, v.x);
        s = s * __expf(m - mn) + v.y * __expf(v.x - mn);
        m = mn;
    }
    float mt = wave_max(m);
    s = wave_sum(s * __expf(m - mt));
    if (threadIdx.x == 0) logp_out[(int64_t)tok_slot[r] * ld_out + tok_pos[r] + 1] = z_tgt[r] - mt - logf(s);
}
void k_lse_reduce(const float2* part, int nparts, const float* z_tgt, int nrows, const int* tok_tgt,
                  const int* tok_slot, const int* tok_pos, float* logp_out, int ld_out, hipStream_t s) {
    if (nrows <= 0) return;
    lse_reduce_kernel<<<nrows, 64, 0, s>>>(part, nparts, z_tgt, tok_tgt, tok_slot, tok_pos, logp_out, ld_out);
}

// ---------------------------------------------------------------- instrument: sustained rate of the matrix cores
// Nothing but v_mfma_f32_16x16x32_f16 -- the shape the large-M GEMMs run -- on operands held in registers (64
// independent accumulator tiles per wave, four waves per CU, no memory traffic inside the loop): what the matrix cores
// sustain under the chip's power management on operands of the given kind.  Random operands (uniform in [-1, 1)) draw
// far more power than zeros, and the clock follows.  The accumulators are written out once at the end so that the loop
// cannot be removed.
__global__ __launch_bounds__(256, 1) void mfma_rate_kernel(const f16_t* in, float* out, int iters) {
    typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
    typedef float floatx4_t __attribute__((ext_vector_type(4)));
    const int l = threadIdx.x;
    half8_t a[8], b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = *reinterpret_cast<const half8_t*>(in + (size_t)(l + 256 * i) * 8);
        b[i] = *reinterpret_cast<const half8_t*>(in + (size_t)(l + 256 * (8 + i)) * 8);
    }
    floatx4_t acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = floatx4_t{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[i], b[j], acc[i][j], 0, 0, 0);
        asm volatile("" : "+v"(a[0]), "+v"(b[0]));
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) s += acc[i][j][1] + acc[i][j][2];
    out[blockIdx.x * 256 + l] = s;
}
__global__ void mfma_rate_fill_kernel(f16_t* p, int n, int random) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    unsigned h = (unsigned)i * 2654435761u + 12345u;
    h ^= h >> 13; h *= 0x5bd1e995u; h ^= h >> 15;
    p[i] = random ? (f16_t)(((h & 0xffff) / 65536.0f) * 2.f - 1.f) : (f16_t)0.f;
}
// scratch: at least 64 KB + n_wg * 1 KB of device memory.  One launch of n_wg workgroups x iters x 64 MFMAs per wave.
void k_mfma_rate(void* scratch, int n_wg, int iters, int random, hipStream_t s) {
    f16_t* in = reinterpret_cast<f16_t*>(scratch);
    float* out = reinterpret_cast<float*>(reinterpret_cast<char*>(scratch) + 65536);
    mfma_rate_fill_kernel<<<(16 * 256 * 8 + 255) / 256, 256, 0, s>>>(in, 16 * 256 * 8, random);
    mfma_rate_kernel<<<n_wg, 256, 0, s>>>(in, out, iters);
}
