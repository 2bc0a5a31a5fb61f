// MFMA attention kernels for gfx950 (fp16 K/V, fp32 softmax and accumulation).
//
// Both kernels compute the transposed problem so that nothing has to be shuffled
// between the two contractions:
//     S^T = K * Q^T        (rows = keys,  cols = queries / query heads)
//     O^T = V^T * P^T      (rows = dims,  cols = queries / query heads)
// In the MFMA C layout a lane owns one column, i.e. one query (head): its softmax
// statistics are lane-local, and the four S^T values a lane holds per 16-key block
// are exactly the four k-values the B operand of the 16x16x16 MFMA wants from that
// lane for P^T.  K is read token-major, V dim-major (the paged pool stores V pages
// as [kv head][dim][token] for this reason), both straight from global memory in
// operand layout -- a (page, kv head) tile is one contiguous 4 KB block.
#include "rl_common.h"
#include "rl_attn.h"

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

#define LOG2E 1.4426950408889634f

// 2^x as the hardware instruction alone.  The library's exp2f wraps it in a rescaling for results in the denormal
// range (six instructions per value); softmax weights that small are zero for every purpose here.  2^-inf = 0.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// ------------------------------------------------------------------ decode: one new query per sequence
// Workgroup = (sequence b, kv head g, split).  Its 4 waves take page pairs round-robin
// from the split's page range; query heads g*G .. g*G+G-1 are the MFMA columns 0..G-1
// (columns >= G are zero padding).  Per-wave results are merged through LDS; with more
// than one split the workgroup writes an unnormalised partial (o, m, l) per head.
// SP: queries, keys and values are fp16 pairs (value = hi + lo; the lo planes of the cache live in layer
// a.layer_lo, the lo halves of a query row after its hi halves).  Scores take the three leading terms
// k_hi q_hi + k_lo q_hi + k_hi q_lo, the probabilities are split the same way for the second contraction, and
// the output leaves as a pair: the layer then carries about 22 significant bits instead of 11.
// FU: the kernel is also the consumer of the QKV projection's split-K partial sums.  While its first page is on the
// way, the workgroup sums the partials of its own G query heads and of its kv head's new key and value (in split
// order), rotates q and k, keeps them in LDS as fp16, and -- split 0 only, after its loop -- appends k and v to the
// cache page.
// Queries are then read from LDS, and the wave that holds the page of the new token takes that token's key row and
// value column from LDS instead of from the page, so nothing depends on when the appended values become visible.
template <int HD, int PT, bool SP, bool FU>
__global__ __launch_bounds__(256, SP ? 2 : 4) void attn_decode_kernel(DecodeAttnArgs a) {
    static_assert(!(SP && FU), "the pair layers keep the separate consumer kernel");
    static_assert(PT == 16, "page tile is one 16-row MFMA block");
    constexpr int KS = HD / 32;    // k-steps of the 16x16x32 S^T MFMAs
    constexpr int DB = HD / 16;    // 16-dim blocks of O^T
    __shared__ float sm_m[4][16], sm_l[4][16];
    __shared__ float sm_o[4][8][HD + 4];
    __shared__ __attribute__((aligned(16))) f16_t sm_q[FU ? 8 : 1][HD], sm_k[HD], sm_v[HD];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 15, g4 = lane >> 4;
    const int b = blockIdx.x, g = blockIdx.y, split = blockIdx.z;
    const int G = a.Hq / a.Hkv;
    // FU: the partial sums of this thread's (at most two) column pairs are requested before anything else -- they
    // depend on nothing but the row -- so they travel together with the position, the page index and the first page.
    // Pair i = (head hh = i / (hd/2), j = i % (hd/2)) covers columns j and j + hd/2 of head hh; hh < G a query head,
    // hh == G the key, hh == G + 1 the value.
    constexpr int NE = 6;                           // splits requested up front (the rest, if any, later)
    constexpr int HALF = HD / 2;
    float pe0[FU ? 2 : 1][NE], pe1[FU ? 2 : 1][NE];
    const float* prow[2] = {nullptr, nullptr};
    if (FU) {
        const int width = (a.Hq + 2 * a.Hkv) * HD;
#pragma unroll
        for (int sl = 0; sl < 2; ++sl) {
            // no branches here (a thread without a second pair re-reads the last pair, a split past the last one
            // re-reads the last split): conditional loads would be waited for one by one
            const int i = min((int)threadIdx.x + sl * 256, (G + 2) * HALF - 1);
            const int hh = i / HALF, j = i % HALF;
            prow[sl] = a.qkv_part + (int64_t)b * width + (hh < G ? g * G + hh : hh == G ? a.Hq + g : a.Hq + a.Hkv + g) * HD + j;
#pragma unroll
            for (int sp = 0; sp < NE; ++sp) {
                const int64_t o = min(sp, a.qkv_nsplit - 1) * a.qkv_split_stride;
                pe0[sl][sp] = prow[sl][o];
                pe1[sl][sp] = prow[sl][o + HALF];
            }
        }
    }
    const int ctx = a.tok_pos[b] + 1;
    float2 cs_new[FU ? 2 : 1];                      // (cos, sin) of the new token's position for this thread's pairs
    if (FU) {
#pragma unroll
        for (int sl = 0; sl < 2; ++sl)
            cs_new[sl] = a.rope[(int64_t)max(ctx - 1, 0) * HALF + min((int)threadIdx.x + sl * 256, (G + 2) * HALF - 1) % HALF];
    }
    const int npages = (ctx + PT - 1) / PT;
    const int chunk = (npages + (int)gridDim.z - 1) / (int)gridDim.z;
    const int pbeg = split * chunk, pend = min(npages, pbeg + chunk);
    const int* bt = a.block_table + (int64_t)b * a.mpps;
    const f16_t* kbase = a.pool + a.geo.k_off(a.layer, 0, g, 0, 0) + col * HD + g4 * 8;
    const f16_t* vbase = a.pool + a.geo.v_off(a.layer, 0, g, 0, 0) + col * PT + g4 * 4;
    const int64_t page_stride = a.geo.page_elems();
    const int64_t lo_off = SP ? (int64_t)(a.layer_lo - a.layer) * a.geo.layer_elems() : 0;   // hi plane -> lo plane
    const int qrow = (SP ? 2 : 1) * a.Hq * HD;       // elements per query / output row

    // Q^T operand: lane (head col, k-group g4) holds q[head][s*32 + g4*8 .. +8)
    half8 qf[KS], ql[SP ? KS : 1];
    if (!FU) {
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const f16_t* qp = a.q + (int64_t)b * qrow + (g * G + col) * HD + s * 32 + g4 * 8;
            if (col < G) qf[s] = *reinterpret_cast<const half8*>(qp);
            else qf[s] = half8{0, 0, 0, 0, 0, 0, 0, 0};
            if (SP) {
                if (col < G) ql[s] = *reinterpret_cast<const half8*>(qp + a.Hq * HD);
                else ql[s] = half8{0, 0, 0, 0, 0, 0, 0, 0};
            }
        }
    }
    const float scale = a.scale * LOG2E;       // softmax in base 2
    float m_run = -INFINITY, l_run = 0.f;
    floatx4 acc[DB];
#pragma unroll
    for (int d = 0; d < DB; ++d) acc[d] = floatx4{0.f, 0.f, 0.f, 0.f};

    // One page per iteration; the next page's K and V tiles are requested before the current
    // page is consumed, so a wave always has a page in flight.
    half8 kf[KS], kn[KS], kfl[SP ? KS : 1], knl[SP ? KS : 1];
    half4 vf[DB], vn[DB], vfl[SP ? DB : 1], vnl[SP ? DB : 1];
    int p = pbeg + wave;
#define AD_FETCH(pg)                                                                                             \
    {                                                                                                            \
        _Pragma("unroll") for (int s = 0; s < KS; ++s) {                                                         \
            kn[s] = *reinterpret_cast<const half8*>(kbase + (pg) * page_stride + s * 32);                        \
            if (SP) knl[s] = *reinterpret_cast<const half8*>(kbase + lo_off + (pg) * page_stride + s * 32);      \
        }                                                                                                        \
        _Pragma("unroll") for (int d = 0; d < DB; ++d) {                                                         \
            vn[d] = *reinterpret_cast<const half4*>(vbase + (pg) * page_stride + d * 16 * PT);                   \
            if (SP) vnl[d] = *reinterpret_cast<const half4*>(vbase + lo_off + (pg) * page_stride + d * 16 * PT); \
        }                                                                                                        \
    }
    if (p < pend) {
        const int64_t pg = bt[p];
        AD_FETCH(pg)
    }
    const int p_new = (ctx - 1) / PT, st_new = (ctx - 1) % PT;   // page and slot of the new token
    if (FU) {
        if (ctx > 0) {   // uniform over the workgroup; a parked row has no keys and no query
#pragma unroll
            for (int sl = 0; sl < 2; ++sl) {
                const int i = threadIdx.x + sl * 256;
                if (i < (G + 2) * HALF) {
                    const int hh = i / HALF, j = i % HALF;
                    const float2 cs = cs_new[sl];
                    float x0 = 0.f, x1 = 0.f;       // summed in split order
#pragma unroll
                    for (int sp = 0; sp < NE; ++sp) {
                        x0 = sp < a.qkv_nsplit ? x0 + pe0[sl][sp] : x0;
                        x1 = sp < a.qkv_nsplit ? x1 + pe1[sl][sp] : x1;
                    }
                    for (int sp = NE; sp < a.qkv_nsplit; ++sp) {
                        x0 += prow[sl][sp * a.qkv_split_stride];
                        x1 += prow[sl][sp * a.qkv_split_stride + HALF];
                    }
                    if (hh <= G) {
                        const float r0 = x0 * cs.x - x1 * cs.y, r1 = x1 * cs.x + x0 * cs.y;
                        x0 = r0; x1 = r1;
                    }
                    const f16_t h0 = (f16_t)x0, h1 = (f16_t)x1;
                    if (hh < G) {
                        sm_q[hh][j] = h0; sm_q[hh][j + HALF] = h1;
                    } else if (hh == G) {
                        sm_k[j] = h0; sm_k[j + HALF] = h1;
                    } else {
                        sm_v[j] = h0; sm_v[j + HALF] = h1;
                    }
                }
            }
            __syncthreads();
        }
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            if (col < G && ctx > 0) qf[s] = *reinterpret_cast<const half8*>(&sm_q[col][s * 32 + g4 * 8]);
            else qf[s] = half8{0, 0, 0, 0, 0, 0, 0, 0};
        }
    }
    for (; p < pend; p += 4) {
#pragma unroll
        for (int s = 0; s < KS; ++s) { kf[s] = kn[s]; if (SP) kfl[s] = knl[s]; }
#pragma unroll
        for (int d = 0; d < DB; ++d) { vf[d] = vn[d]; if (SP) vfl[d] = vnl[d]; }
        if (FU && p == p_new) {   // the new token's key row and value column come from LDS
            if (col == st_new) {
#pragma unroll
                for (int s = 0; s < KS; ++s) kf[s] = *reinterpret_cast<const half8*>(&sm_k[s * 32 + g4 * 8]);
            }
            if (g4 == (st_new >> 2)) {
#pragma unroll
                for (int d = 0; d < DB; ++d) {
                    const f16_t v = sm_v[d * 16 + col];
#pragma unroll
                    for (int i = 0; i < 4; ++i) vf[d][i] = i == (st_new & 3) ? v : vf[d][i];
                }
            }
        }
        {
            const int pn = min(p + 4, pend - 1);          // the last iteration re-reads a valid page, unused
            const int64_t pg = bt[pn];
            AD_FETCH(pg)
        }
        floatx4 s0 = {0.f, 0.f, 0.f, 0.f};
        if (SP) {   // the two small terms first, the leading one last
#pragma unroll
            for (int s = 0; s < KS; ++s) s0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(kfl[s], qf[s], s0, 0, 0, 0);
#pragma unroll
            for (int s = 0; s < KS; ++s) s0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf[s], ql[s], s0, 0, 0, 0);
        }
#pragma unroll
        for (int s = 0; s < KS; ++s) s0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf[s], qf[s], s0, 0, 0, 0);
        // lane holds keys p*16 + g4*4 + i of head `col`
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int t0 = p * PT + g4 * 4 + i;
            s0[i] = (t0 < ctx) ? s0[i] * scale : -INFINITY;
            mx = fmaxf(mx, s0[i]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16, RL_WAVE));
        mx = fmaxf(mx, __shfl_xor(mx, 32, RL_WAVE));
        const float m_new = fmaxf(m_run, mx);       // finite: the first key of page p is always valid
        const float alpha = fast_exp2(m_run - m_new);
        half4 pf0, pl0;
        float ps = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float e0 = fast_exp2(s0[i] - m_new);
            ps += e0;
            pf0[i] = (f16_t)e0;
            if (SP) pl0[i] = (f16_t)(e0 - (float)pf0[i]);
        }
        l_run = l_run * alpha + ps;
        m_run = m_new;
#pragma unroll
        for (int d = 0; d < DB; ++d) {
            acc[d] *= alpha;
            if (SP) {
                acc[d] = __builtin_amdgcn_mfma_f32_16x16x16f16(vfl[d], pf0, acc[d], 0, 0, 0);
                acc[d] = __builtin_amdgcn_mfma_f32_16x16x16f16(vf[d], pl0, acc[d], 0, 0, 0);
            }
            acc[d] = __builtin_amdgcn_mfma_f32_16x16x16f16(vf[d], pf0, acc[d], 0, 0, 0);
        }
    }
#undef AD_FETCH
    // FU: the new token's key and value go to the cache only now -- stores count towards the same in-order
    // completion counter as loads, so stores issued before the loop would hold back every page load behind them
    if (FU && split == 0 && ctx > 0) {
        const int64_t page = bt[p_new];
        for (int i = threadIdx.x; i < HD; i += 256) {
            a.pool_w[a.geo.k_off(a.layer, page, g, st_new, i)] = sm_k[i];
            a.pool_w[a.geo.v_off(a.layer, page, g, st_new, i)] = sm_v[i];
        }
    }
    // wave totals: l over the four key groups
    l_run += __shfl_xor(l_run, 16, RL_WAVE);
    l_run += __shfl_xor(l_run, 32, RL_WAVE);
    if (col < G) {
        if (g4 == 0) { sm_m[wave][col] = m_run; sm_l[wave][col] = l_run; }
#pragma unroll
        for (int d = 0; d < DB; ++d)
#pragma unroll
            for (int i = 0; i < 4; ++i) sm_o[wave][col][d * 16 + g4 * 4 + i] = acc[d][i];
    }
    __syncthreads();
    const int nsplit = gridDim.z;
    for (int idx = threadIdx.x; idx < G * HD; idx += 256) {
        const int hh = idx / HD, d = idx % HD;
        float mt = fmaxf(fmaxf(sm_m[0][hh], sm_m[1][hh]), fmaxf(sm_m[2][hh], sm_m[3][hh]));
        float o = 0.f, l = 0.f;
        if (mt > -INFINITY) {
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                float wt = fast_exp2(sm_m[w][hh] - mt);
                o += wt * sm_o[w][hh][d];
                l += wt * sm_l[w][hh];
            }
        }
        const int64_t head = (int64_t)b * a.Hq + g * G + hh;
        if (nsplit == 1) {
            const float r = l > 0.f ? o / l : 0.f;                          // parked row (position -1): no keys, zeros
            f16_t* op = a.out + (int64_t)b * qrow + (g * G + hh) * HD + d;
            const f16_t hi = (f16_t)r;
            op[0] = hi;
            if (SP) op[a.Hq * HD] = (f16_t)(r - (float)hi);
        } else {
            a.part_o[(head * nsplit + split) * HD + d] = o;
            if (d == 0) {
                a.part_ml[(head * nsplit + split) * 2 + 0] = mt;
                a.part_ml[(head * nsplit + split) * 2 + 1] = l;
            }
        }
    }
}

// Merge of split partials: out = sum_s w_s o_s / sum_s w_s l_s, w_s = 2^(m_s - max m).
// split: the output row holds fp16 pairs, [Hq heads of hi | Hq heads of lo].
template <int HD>
__global__ __launch_bounds__(HD) void attn_merge_kernel(const float* part_o, const float* part_ml, f16_t* out,
                                                        int nsplit, int Hq, int split) {
    const int64_t head = blockIdx.x;
    const int d = threadIdx.x;
    float mt = -INFINITY;
    for (int s = 0; s < nsplit; ++s) mt = fmaxf(mt, part_ml[(head * nsplit + s) * 2]);
    float o = 0.f, l = 0.f;
    for (int s = 0; s < nsplit; ++s) {
        float m = part_ml[(head * nsplit + s) * 2];
        if (m == -INFINITY) continue;
        float wt = fast_exp2(m - mt);
        o += wt * part_o[(head * nsplit + s) * HD + d];
        l += wt * part_ml[(head * nsplit + s) * 2 + 1];
    }
    const float r = l > 0.f ? o / l : 0.f;
    const f16_t hi = (f16_t)r;
    f16_t* op = out + (head / Hq) * (int64_t)((split ? 2 : 1) * Hq * HD) + (head % Hq) * HD + d;
    op[0] = hi;
    if (split) op[Hq * HD] = (f16_t)(r - (float)hi);
}

// The consumer form of the kernel gives each of its 256 threads at most two (column, column + hd/2) pairs of the
// group's G query heads, key and value, and keeps the queries of at most 8 heads in LDS.
bool k_attn_decode_consumes_qkv(int Hq, int Hkv, int hd) {
    const int G = Hq / Hkv;
    return (hd == 64 || hd == 128) && G <= 8 && (G + 2) * (hd / 2) <= 512;
}

void k_attn_decode(const DecodeAttnArgs& a, int B, int nsplit, hipStream_t s) {
    if (B <= 0) return;
    if (a.qkv_part && (a.split || !k_attn_decode_consumes_qkv(a.Hq, a.Hkv, a.geo.hd))) return;   // callers check first
    dim3 grid(B, a.Hkv, nsplit);
    if (a.split) {
        if (a.geo.hd == 128) attn_decode_kernel<128, 16, true, false><<<grid, 256, 0, s>>>(a);
        else attn_decode_kernel<64, 16, true, false><<<grid, 256, 0, s>>>(a);
    } else if (a.qkv_part) {
        if (a.geo.hd == 128) attn_decode_kernel<128, 16, false, true><<<grid, 256, 0, s>>>(a);
        else attn_decode_kernel<64, 16, false, true><<<grid, 256, 0, s>>>(a);
    } else {
        if (a.geo.hd == 128) attn_decode_kernel<128, 16, false, false><<<grid, 256, 0, s>>>(a);
        else attn_decode_kernel<64, 16, false, false><<<grid, 256, 0, s>>>(a);
    }
    if (nsplit > 1) {
        if (a.geo.hd == 128) attn_merge_kernel<128><<<B * a.Hq, 128, 0, s>>>(a.part_o, a.part_ml, a.out, nsplit, a.Hq, a.split);
        else attn_merge_kernel<64><<<B * a.Hq, 64, 0, s>>>(a.part_o, a.part_ml, a.out, nsplit, a.Hq, a.split);
    }
}

// ------------------------------------------------------------------ prefill / scoring: causal attention over packed sequences
// Workgroup = (32-query block of one sequence, kv head g); wave w handles query head g*G + w, so the
// waves of a workgroup need the SAME keys and values.  Per 32-key block the K tile (32 keys x hd) and the
// V^T tile (hd dims x 32 keys, from the dim-major value buffer) are staged ONCE per workgroup into LDS by
// global -> LDS loads -- row-contiguous 16-byte pieces, whole rows per request; fetching the operands in
// MFMA layout straight from memory instead makes every lane of a load touch a different row, and the
// address path of the CU, not the MFMAs or the caches, then sets the pace -- and every wave reads its
// operand fragments from there.  Two stages: the tile of block kb+1 is requested right after the barrier
// that opens block kb.  16-byte chunks are XOR-swizzled on the source side of the loads (K: chunk ^ row%16
// for 256-byte rows, chunk ^ (row/2)%8 for 128-byte rows; V^T: chunk ^ (row/4)%4) so that the fragment
// reads spread over the banks.  The loads are issued from inline assembly and waited for by hand (the
// compiler would otherwise make each of them complete at the next barrier).
//   S^T (32 keys x 32 queries) by 32x32x16 MFMAs with K rows as A and Q^T as B; base-2 online softmax per
//   query (a lane owns one query column); O^T += V^T P^T where the lane's own S^T registers, rounded to
//   fp16, are the B operand.
typedef float floatx16 __attribute__((ext_vector_type(16)));

// SP: q, k, v are fp16 pairs (value = hi + lo; rows of q, k and the output are [hi heads | lo heads], the lo plane
// of V^T follows the hi plane).  A stage then holds four tiles (K hi, V^T hi, K lo, V^T lo), the scores take the
// three leading terms k_hi q_hi + k_lo q_hi + k_hi q_lo, and the probabilities are split the same way for the
// second contraction: three MFMAs where the plain kernel has one.
template <int HD, bool SP>
__global__ __launch_bounds__(512) void attn_prefill_kernel(PrefillAttnArgs a) {
    constexpr int KSTEPS = HD / 16, DB = HD / 32;
    constexpr int KT = 32 * HD * 2;              // bytes of a K tile; a V^T tile is as large
    constexpr int NT = SP ? 4 : 2;               // tiles of a stage: K, V^T (hi), then K, V^T (lo)
    constexpr int STG = NT * KT;
    constexpr int NIT = KT / 1024;               // 1 KB load instructions per tile
    constexpr int NI = NT * NIT;
    constexpr int KCH = HD / 8;                  // 16-byte chunks per K row
    constexpr int KRPI = 64 / KCH;               // K rows per load instruction
    extern __shared__ __attribute__((aligned(1024))) char smem[];   // [2 stages][STG]
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int col = lane & 31, g2 = lane >> 5;
    const int4 blk = a.blocks[blockIdx.x];          // (row start, length, query block, -)
    const int start = blk.x, len = blk.y, qb = blk.z;
    const int g = blockIdx.y, G = a.Hq / a.Hkv, h = g * G + wave;
    const int qi = qb * 32 + col;                   // this lane's query (position in the sequence)
    const int qrow = start + min(qi, len - 1);
    const int kvw = (SP ? 2 : 1) * a.Hkv * HD;      // elements per K row
    const int qw = (SP ? 2 : 1) * a.Hq * HD;        // elements per query / output row

    // staging: instruction i of the stage (i = wave, wave + G, ...) moves 1 KB
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) char*)smem;
    const f16_t* kg = a.k + (int64_t)start * kvw + g * HD;               // K rows of this sequence, head g
    const f16_t* vg = a.vT + (int64_t)g * HD * a.vt_cap + start;          // V^T rows (dims) of head g
#define AP_STAGE(stage, kb)                                                                                      \
    for (int i_ = wave; i_ < NI; i_ += G) {                                                                      \
        const unsigned sa_ = lds_base + (stage) * STG + i_ * 1024;                                               \
        const int t_ = i_ / NIT, ii_ = i_ % NIT;                                                                 \
        unsigned off_;                                                                                           \
        const f16_t* base_;                                                                                      \
        if ((t_ & 1) == 0) {                     /* K: KRPI rows of KCH chunks */                                \
            const int r_ = ii_ * KRPI + lane / KCH, pc_ = lane % KCH;                                            \
            const int lc_ = pc_ ^ (HD == 128 ? (r_ & 15) : ((r_ >> 1) & 7));                                     \
            /* tile row r_ holds key rho(r_): the middle two 4-row groups of every 16 are swapped, so that a */  \
            /* lane's S^T registers 8kk .. 8kk+7 are eight CONSECUTIVE keys (one 16-byte V^T chunk)         */  \
            const int key_ = (r_ & ~12) | ((r_ & 4) << 1) | ((r_ & 8) >> 1);                                     \
            off_ = (unsigned)(((kb) * 32 + key_) * kvw + lc_ * 8) * 2u;                                          \
            base_ = kg + (t_ >> 1) * a.Hkv * HD;                                                                 \
        } else {                                 /* V^T: 16 dims of 4 chunks (32 keys) */                        \
            const int r_ = ii_ * 16 + (lane >> 2), pc_ = lane & 3;                                               \
            const int lc_ = pc_ ^ ((r_ >> 2) & 3);                                                               \
            off_ = (unsigned)(r_ * a.vt_cap + (kb) * 32 + lc_ * 8) * 2u;                                         \
            base_ = vg + (int64_t)(t_ >> 1) * a.Hkv * HD * a.vt_cap;                                             \
        }                                                                                                        \
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"                             \
                     :: "s"(sa_), "v"(off_), "s"(base_) : "memory");                                             \
    }

    half8 qf[KSTEPS], ql[SP ? KSTEPS : 1];
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) {
        const f16_t* qp = a.q + (int64_t)qrow * qw + h * HD + s * 16 + g2 * 8;
        qf[s] = *reinterpret_cast<const half8*>(qp);
        if (SP) ql[s] = *reinterpret_cast<const half8*>(qp + a.Hq * HD);
    }
    floatx16 o[DB];
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[d][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const float scale = a.scale * LOG2E;
    // this lane's fragment addresses inside a stage
    const int ksw = HD == 128 ? (col & 15) : ((col >> 1) & 7);
    const int k_row = col * (HD * 2);                       // K row `col`
    const int vsw = (col >> 2) & 3;                         // same for rows d*32 + col

    AP_STAGE(0, 0)
    for (int kb = 0; kb <= qb; ++kb) {
        const int st = kb & 1;
        // the tile of block kb has landed (this wave's part: its only loads in flight); after the barrier
        // every wave's part has, and every wave is done with the other stage
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        AP_STAGE(1 - st, min(kb + 1, qb))                   // the last trip re-requests its own block, unused
        const char* kt = smem + st * STG;
        const char* vt = kt + KT;
        // S^T = K Q^T
        floatx16 stt;
#pragma unroll
        for (int r = 0; r < 16; ++r) stt[r] = 0.f;
        if (SP) {   // the two small terms first, the leading one last
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) {
                const int fo = k_row + (((s * 2 + g2) ^ ksw) * 16);
                const half8 kl = *reinterpret_cast<const half8*>(kt + 2 * KT + fo);
                const half8 kf = *reinterpret_cast<const half8*>(kt + fo);
                stt = __builtin_amdgcn_mfma_f32_32x32x16_f16(kl, qf[s], stt, 0, 0, 0);
                stt = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf, ql[s], stt, 0, 0, 0);
            }
        }
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) {
            const half8 kf = *reinterpret_cast<const half8*>(kt + k_row + (((s * 2 + g2) ^ ksw) * 16));
            stt = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf, qf[s], stt, 0, 0, 0);
        }
        // register r of this lane is tile row 8*(r/4) + 4*g2 + r%4, which holds key kb*32 + 16*(r/8) + 8*g2 + r%8.
        // Only the diagonal block needs the causal mask; the running maximum is kept in raw (unscaled) units,
        // so that exp2(scale * (s - m)) is one fused multiply-add and one exp2 per element.
        if (kb == qb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = kb * 32 + 16 * (r >> 3) + 8 * g2 + (r & 7);
                if (key > qi) stt[r] = -INFINITY;
            }
        }
        float mx = stt[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, stt[r]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, RL_WAVE));
        const float m_new = fmaxf(m_run, mx);        // finite: key kb*32 <= qi for every kb <= qb
        const float alpha = fast_exp2((m_run - m_new) * scale);
        const float nms = -m_new * scale;
        half8 pf[2], pl[SP ? 2 : 1];
        float ps = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float e = fast_exp2(fmaf(stt[r], scale, nms));
            ps += e;
            const f16_t eh = (f16_t)e;
            pf[r >> 3][r & 7] = eh;
            if (SP) pl[r >> 3][r & 7] = (f16_t)(e - (float)eh);
        }
        l_run = l_run * alpha + ps;
        m_run = m_new;
        // the accumulators are rescaled only when some query's maximum moved (rare after the first blocks)
        const bool rescale = __any(alpha != 1.0f);
        // O^T += V^T P^T: the lane needs keys kk*16 + 8*g2 .. +8 of dim d*32 + col: one 16-byte chunk
#pragma unroll
        for (int d = 0; d < DB; ++d) {
            if (rescale) {
#pragma unroll
                for (int r = 0; r < 16; ++r) o[d][r] *= alpha;
            }
            const char* vr = vt + (d * 32 + col) * 64;
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                const int fo = ((kk * 2 + g2) ^ vsw) * 16;
                const half8 vf = *reinterpret_cast<const half8*>(vr + fo);
                if (SP) {
                    const half8 vl = *reinterpret_cast<const half8*>(vr + 2 * KT + fo);
                    o[d] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vl, pf[kk], o[d], 0, 0, 0);
                    o[d] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pl[SP ? kk : 0], o[d], 0, 0, 0);
                }
                o[d] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pf[kk], o[d], 0, 0, 0);
            }
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // nothing may land in LDS after the workgroup has ended
#undef AP_STAGE
    l_run += __shfl_xor(l_run, 32, RL_WAVE);
    if (qi < len) {
        const float inv = 1.0f / l_run;
        f16_t* op = a.out + (int64_t)(start + qi) * qw + h * HD;
#pragma unroll
        for (int d = 0; d < DB; ++d)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                half4 w4, l4;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float r = o[d][4 * j + i] * inv;
                    w4[i] = (f16_t)r;
                    if (SP) l4[i] = (f16_t)(r - (float)w4[i]);
                }
                *reinterpret_cast<half4*>(op + d * 32 + 8 * j + 4 * g2) = w4;
                if (SP) *reinterpret_cast<half4*>(op + a.Hq * HD + d * 32 + 8 * j + 4 * g2) = l4;
            }
    }
}

template <int HD, bool SP>
static void launch_prefill(const PrefillAttnArgs& a, int nblocks, hipStream_t s) {
    constexpr int lds = 2 * (SP ? 4 : 2) * 32 * HD * 2;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void*)attn_prefill_kernel<HD, SP>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        attr_set = true;
    }
    dim3 grid(nblocks, a.Hkv);
    attn_prefill_kernel<HD, SP><<<grid, 64 * (a.Hq / a.Hkv), lds, s>>>(a);
}

void k_attn_prefill(const PrefillAttnArgs& a, int nblocks, hipStream_t s) {
    if (nblocks <= 0) return;
    if (a.hd == 128) {
        if (a.split) launch_prefill<128, true>(a, nblocks, s);
        else launch_prefill<128, false>(a, nblocks, s);
    } else {
        if (a.split) launch_prefill<64, true>(a, nblocks, s);
        else launch_prefill<64, false>(a, nblocks, s);
    }
}
