// MFMA GEMMs for gfx950:  C[M,N] = A[M,K] (fp16, row-major) * W[N,K]^T (bf16, row-major).
//
// Weights stay bf16 in HBM and are converted to fp16 while they are staged into LDS (exact
// for every weight of normal fp16 magnitude); the contraction runs on
// v_mfma_f32_32x32x16_f16 with fp32 accumulation.  One kernel template serves
//   * the large-M GEMMs of prefill / scoring (grid over M and N tiles), and
//   * the weight-streaming GEMMs of a decode step (M <= 128 rows, split over K so that all
//     256 CUs stream a slice of W; partial sums go to a [split][M][N] fp32 buffer and are
//     reduced, in a fixed order, by the consumer kernel).
// Epilogues: fp32 store / split-K partial, fp16 store, residual add, SwiGLU, and
// RoPE + q/k/v split for the QKV projection.
#include "rl_common.h"
#include "rl_gemm.h"

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef __fp16 fp16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

#define BK 64
#define LDS_STRIDE 72   // halfs per LDS row: 64 + 8 pad -> 144 B, conflict-free ds_read_b128

__device__ __forceinline__ uint4 bf16x8_to_f16x8(uint4 w) {
    union { uint4 u; fp16x2 p[4]; } o;
    unsigned ws[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float lo = __uint_as_float(ws[i] << 16), hi = __uint_as_float(ws[i] & 0xffff0000u);
        o.p[i] = __builtin_amdgcn_cvt_pkrtz(lo, hi);   // exact: bf16 has 8 significant bits
    }
    return o.u;
}

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ half8 bf16x8_to_half8(u32x4_t w) {
    fp16x2 p0 = __builtin_amdgcn_cvt_pkrtz(__uint_as_float(w[0] << 16), __uint_as_float(w[0] & 0xffff0000u));
    fp16x2 p1 = __builtin_amdgcn_cvt_pkrtz(__uint_as_float(w[1] << 16), __uint_as_float(w[1] & 0xffff0000u));
    fp16x2 p2 = __builtin_amdgcn_cvt_pkrtz(__uint_as_float(w[2] << 16), __uint_as_float(w[2] & 0xffff0000u));
    fp16x2 p3 = __builtin_amdgcn_cvt_pkrtz(__uint_as_float(w[3] << 16), __uint_as_float(w[3] & 0xffff0000u));
    return half8{(f16_t)p0[0], (f16_t)p0[1], (f16_t)p1[0], (f16_t)p1[1], (f16_t)p2[0], (f16_t)p2[1], (f16_t)p3[0], (f16_t)p3[1]};
}

// Which row of W feeds LDS row r of the B tile of column-block nb.
//  EPI_SWIGLU: the tile holds BN/2 gate rows and the matching BN/2 up rows, interleaved in
//              blocks of 32 so that a wave's adjacent 32-column MFMA tiles are (gate, up).
//  MG_QKV with head_dim 128: the halves of each head (128 tile columns) are interleaved in blocks of
//              32 so that a wave holds columns j and j + 64 in the same lane.
template <int EPI, int BN>
__device__ __forceinline__ int w_row_of(int r, int nb, const GemmArgs& a) {
    if (EPI == MG_SWIGLU) {
        int blk = r >> 5, within = r & 31;
        int col = nb * (BN / 2) + (blk >> 1) * 32 + within;
        return (blk & 1) ? a.up_offset + col : col;
    } else if (EPI == MG_QKV) {
        if (a.hd == 128) {
            int blk = (r & 127) >> 5, within = r & 31;   // per head, LDS blocks: [0:32) [64:96) [32:64) [96:128)
            int src = ((blk & 1) ? 64 : 0) + (blk >> 1) * 32 + within;
            return nb * BN + (r & ~127) + src;
        }
        return nb * BN + r;
    } else {
        return nb * BN + r;
    }
}

// Tile order.  The tile sequence walks bands of 8 row blocks column by column, so that consecutive
// tiles share few A row blocks and few W column blocks.  Workgroup ids are dealt round-robin to the 8
// XCDs, each with its own L2: XCD x takes the contiguous run [x*C, (x+1)*C) of the sequence, so the
// tiles resident on one XCD at any time form a compact block and re-use their operands from that L2.
// The grid holds 8*C ids; returns false for the (at most 7) ids past the end.
__device__ __forceinline__ bool tile_of(int id, int MB, int NB, int& mb, int& nb) {
    const int T = MB * NB, C = (T + 7) >> 3;
    const int pos = (id & 7) * C + (id >> 3);
    if (pos >= T) return false;
    const int per_group = 8 * NB;
    const int group = pos / per_group, first = group * 8, gsz = min(MB - first, 8), r = pos % per_group;
    mb = first + r % gsz;
    nb = r / gsz;
    return true;
}

// Epilogue shared by the tile kernels, for one 32-row band of a wave's accumulators: acc[j][r] of the
// wave in tile-column position wn is C(row, col) with
//   row = m_base + 8*(r/4) + 4*(lane/32) + r%4,   col(tile-local) = wn*TN*32 + j*32 + lane%32
template <int EPI, int BN, int TN, int WGN>
__device__ __forceinline__ void mg_epilogue(floatx16 (&acc)[TN], const GemmArgs& a, int m_base, int nb, int wn,
                                            int ks, int lane) {
    const int lg = lane >> 5, lrow = lane & 31;
    if (EPI == MG_RESID) {
        // read-modify-write of the fp32 residual stream: all of the band's loads are issued before the
        // first add (rows past M read row M-1 instead of branching, so nothing separates the loads)
        float old[TN][16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = min(m_base + 8 * (r >> 2) + 4 * lg + (r & 3), a.M - 1);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                old[j][r] = a.outF[(int64_t)m * a.ldc + min(nb * BN + wn * TN * 32 + j * 32 + lrow, a.N - 1)];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = m_base + 8 * (r >> 2) + 4 * lg + (r & 3);
            if (m >= a.M) continue;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                int n = nb * BN + wn * TN * 32 + j * 32 + lrow;
                if (n < a.N) a.outF[(int64_t)m * a.ldc + n] = old[j][r] + acc[j][r];
            }
        }
        return;
    }
    {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = m_base + 8 * (r >> 2) + 4 * lg + (r & 3);
            if (m >= a.M) continue;
            if (EPI == MG_STORE_F32) {
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    int n = nb * BN + wn * TN * 32 + j * 32 + lrow;
                    if (n < a.N) a.outF[(int64_t)ks * a.split_stride + (int64_t)m * a.ldc + n] = acc[j][r];
                }
            } else if (EPI == MG_STORE_F16) {
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    int n = nb * BN + wn * TN * 32 + j * 32 + lrow;
                    if (n < a.N) a.outH[(int64_t)m * a.ldc + n] = (f16_t)acc[j][r];
                }
            } else if (EPI == MG_SWIGLU) {
#pragma unroll
                for (int j = 0; j < TN; j += 2) {
                    int n = nb * (BN / 2) + (wn * TN + j) / 2 * 32 + lrow;
                    float g = acc[j][r], u = acc[j + 1][r];
                    if (n < a.N) a.outH[(int64_t)m * a.ldc + n] = (f16_t)(g / (1.0f + __expf(-g)) * u);
                }
            } else if (EPI == MG_LSE) {
                // this wave's TN*32 columns of row m: running (max, sum of exponentials) over the
                // lanes that share the row (the 32 lanes of a half-wave), and the target's logit
                float mx = acc[0][r];
#pragma unroll
                for (int j = 1; j < TN; ++j) mx = fmaxf(mx, acc[j][r]);
#pragma unroll
                for (int o = 1; o < 32; o <<= 1) mx = fmaxf(mx, __shfl_xor(mx, o, RL_WAVE));
                float se = 0.f;
#pragma unroll
                for (int j = 0; j < TN; ++j) se += __expf(acc[j][r] - mx);
#pragma unroll
                for (int o = 1; o < 32; o <<= 1) se += __shfl_xor(se, o, RL_WAVE);
                const int nparts = (a.N / BN) * WGN;
                if (lrow == 0) a.lse_part[(int64_t)m * nparts + nb * WGN + wn] = make_float2(mx, se);
                const int t = a.tgt[m];
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    if (t == nb * BN + wn * TN * 32 + j * 32 + lrow) a.z_tgt[m] = acc[j][r];
            } else if (EPI == MG_QKV) {
                // columns of this tile belong to one head (hd 128) or two (hd 64); pairs (j, j + hd/2)
                // sit in adjacent 32-column MFMA tiles of this lane.
                // pos < 0 marks a padding row of the packed token list: it gets zeros (so that
                // nothing non-finite is ever read back as a key or value) and no cache slot
                const int pos_raw = a.tok_pos[m];
                const bool pad = pos_raw < 0;
                const int pos = pad ? 0 : pos_raw;
                const int hd = a.hd, half = hd >> 1;
#pragma unroll
                for (int j = 0; j < TN; j += 2) {
                    // tile-local LDS column of acc[j]: c0; its partner acc[j+1] is c0 + 32 in LDS order
                    int c0 = wn * TN * 32 + j * 32 + lrow;
                    int col0;                             // global qkv column of v0; v1 is col0 + hd/2
                    if (hd == 128) {
                        int blk = (c0 & 127) >> 5;        // even LDS block of this head
                        col0 = nb * BN + (c0 & ~127) + (blk >> 1) * 32 + (c0 & 31);
                    } else {
                        col0 = nb * BN + c0;
                    }
                    float v0 = pad ? 0.f : acc[j][r], v1 = pad ? 0.f : acc[j + 1][r];
                    const int head = col0 / hd, jj = col0 % hd;      // jj < half
                    const int Hq = a.Hq, Hkv = a.Hkv;
                    if (head < Hq + Hkv) {
                        float2 cs = a.rope[(int64_t)pos * half + jj];
                        float r0 = v0 * cs.x - v1 * cs.y, r1 = v1 * cs.x + v0 * cs.y;
                        v0 = r0; v1 = r1;
                    }
                    if (head < Hq) {
                        f16_t* o = a.q_out + (int64_t)m * Hq * hd + head * hd + jj;
                        o[0] = (f16_t)v0; o[half] = (f16_t)v1;
                    } else if (head < Hq + Hkv) {
                        int g = head - Hq;
                        if (a.k_out) {
                            f16_t* o = a.k_out + ((int64_t)m * Hkv + g) * hd + jj;
                            o[0] = (f16_t)v0; o[half] = (f16_t)v1;
                        }
                        if (a.pool && !pad) {
                            int64_t page = a.block_table[(int64_t)a.tok_slot[m] * a.mpps + pos / a.geo.PT];
                            int st = pos % a.geo.PT;
                            a.pool[a.geo.k_off(a.layer, page, g, st, jj)] = (f16_t)v0;
                            a.pool[a.geo.k_off(a.layer, page, g, st, jj + half)] = (f16_t)v1;
                        }
                    } else {
                        int g = head - Hq - Hkv;
                        if (a.v_out) {
                            if (a.vt_cap > 0) {   // dim-major: vT[kv head][dim][token]
                                a.v_out[((int64_t)g * hd + jj) * a.vt_cap + m] = (f16_t)v0;
                                a.v_out[((int64_t)g * hd + jj + half) * a.vt_cap + m] = (f16_t)v1;
                            } else {
                                f16_t* o = a.v_out + ((int64_t)m * Hkv + g) * hd + jj;
                                o[0] = (f16_t)v0; o[half] = (f16_t)v1;
                            }
                        }
                        if (a.pool && !pad) {
                            int64_t page = a.block_table[(int64_t)a.tok_slot[m] * a.mpps + pos / a.geo.PT];
                            int st = pos % a.geo.PT;
                            a.pool[a.geo.v_off(a.layer, page, g, st, jj)] = (f16_t)v0;
                            a.pool[a.geo.v_off(a.layer, page, g, st, jj + half)] = (f16_t)v1;
                        }
                    }
                }
            }
        }
    }
}

template <int BM, int BN, int WGM, int WGN, int EPI, int BKT>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(GemmArgs a) {
    constexpr int TM = BM / WGM / 32, TN = BN / WGN / 32;
    constexpr int LSTR = BKT + 8;   // halfs per LDS row (+16 B pad: conflict-free ds_read_b128)
    constexpr int CPR = BKT / 8;    // 16-byte chunks per tile row
    constexpr int A_CH = BM * CPR / 256, W_CH = BN * CPR / 256;   // chunks per thread per k-tile
    extern __shared__ __attribute__((aligned(16))) char smem[];
    f16_t* As = reinterpret_cast<f16_t*>(smem);                   // [2][BM][LSTR]
    f16_t* Ws = As + 2 * BM * LSTR;                         // [2][BN][LSTR]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int NB = a.n_blocks_n, MB = (a.M + BM - 1) / BM, ks = blockIdx.z;
    int nb, mb;
    if (!tile_of(blockIdx.x, MB, NB, mb, nb)) return;
    const int m0 = mb * BM;
    const int kbeg = ks * a.k_per_split, kend = min(a.K, kbeg + a.k_per_split);
    const int nk = (kend - kbeg + BKT - 1) / BKT;

    // per-thread global source rows for the staged loads
    const f16_t* a_src[A_CH];
    const bf16_t* w_src[W_CH];
    int a_dst[A_CH], w_dst[W_CH];
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
        int c = tid + i * 256, r = c / CPR, kc = c % CPR;
        int m = m0 + r;
        a_src[i] = a.A + (int64_t)min(m, a.M - 1) * a.lda + kc * 8;   // rows >= M: any finite-or-not data, never stored
        a_dst[i] = r * LSTR + kc * 8;
    }
#pragma unroll
    for (int i = 0; i < W_CH; ++i) {
        int c = tid + i * 256, r = c / CPR, kc = c % CPR;
        int wr = w_row_of<EPI, BN>(r, nb, a);
        w_src[i] = a.W + (int64_t)min(wr, a.Wrows - 1) * a.K + kc * 8;
        w_dst[i] = r * LSTR + kc * 8;
    }

    // Two register sets alternate between k-tiles: a tile is requested at the start of step kt-2's
    // successor... concretely, tile kt+2 is requested at the start of step kt and parked in LDS at
    // the end of step kt+1, so every global load has two full steps to arrive.  The steady-state
    // loop issues the same requests on every path (vector loads return in order; a wait count is
    // exact only then); prologue and the last two steps are peeled.
    u32x4_t ra0[A_CH], rw0[W_CH], ra1[A_CH], rw1[W_CH];
#define MG_LOAD(sl, kt)                                                                          \
    {                                                                                            \
        _Pragma("unroll") for (int i_ = 0; i_ < A_CH; ++i_)                                      \
            ra##sl[i_] = *reinterpret_cast<const u32x4_t*>(a_src[i_] + kbeg + (kt) * BKT);        \
        _Pragma("unroll") for (int i_ = 0; i_ < W_CH; ++i_)                                      \
            rw##sl[i_] = *reinterpret_cast<const u32x4_t*>(w_src[i_] + kbeg + (kt) * BKT);        \
    }
#define MG_PARK(sl, buf)                                                                         \
    {                                                                                            \
        _Pragma("unroll") for (int i_ = 0; i_ < A_CH; ++i_)                                      \
            *reinterpret_cast<u32x4_t*>(As + (buf) * BM * LSTR + a_dst[i_]) = ra##sl[i_];  \
        _Pragma("unroll") for (int i_ = 0; i_ < W_CH; ++i_)                                      \
            *reinterpret_cast<half8*>(Ws + (buf) * BN * LSTR + w_dst[i_]) = bf16x8_to_half8(rw##sl[i_]); \
    }
    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    const int lrow = lane & 31, lk = (lane >> 5) * 8;
#define MG_FRAGS(dst_a, dst_b, kk)                                                               \
    _Pragma("unroll") for (int i = 0; i < TM; ++i)                                               \
        dst_a[i] = *reinterpret_cast<const half8*>(Ab + i * 32 * LSTR + (kk));             \
    _Pragma("unroll") for (int j = 0; j < TN; ++j)                                               \
        dst_b[j] = *reinterpret_cast<const half8*>(Wb + j * 32 * LSTR + (kk));
#define MG_MFMAS(src_a, src_b)                                                                   \
    _Pragma("unroll") for (int i = 0; i < TM; ++i) _Pragma("unroll") for (int j = 0; j < TN; ++j) \
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(src_a[i], src_b[j], acc[i][j], 0, 0, 0);
    // fragments of k-slice kk+16 are fetched from LDS while the MFMAs of slice kk run
#define MG_COMPUTE(buf)                                                                          \
    {                                                                                            \
        const f16_t* Ab = As + (buf) * BM * LSTR + (wm * TM * 32 + lrow) * LSTR + lk;            \
        const f16_t* Wb = Ws + (buf) * BN * LSTR + (wn * TN * 32 + lrow) * LSTR + lk;            \
        half8 afA[TM], bfA[TN], afB[TM], bfB[TN];                                                \
        MG_FRAGS(afA, bfA, 0)                                                                    \
        _Pragma("unroll") for (int kk = 0; kk < BKT; kk += 32) {                                 \
            MG_FRAGS(afB, bfB, kk + 16)                                                          \
            MG_MFMAS(afA, bfA)                                                                   \
            if (kk + 32 < BKT) { MG_FRAGS(afA, bfA, kk + 32) }                                   \
            MG_MFMAS(afB, bfB)                                                                   \
        }                                                                                        \
    }
    // step with tile parity p: request tile kt+2 into set p (its previous tile is already parked),
    // consume LDS buffer p, park set 1-p (tile kt+1) into buffer 1-p
#define MG_STEP_FULL(p, q, kt) { MG_LOAD(p, (kt) + 2) __builtin_amdgcn_sched_barrier(0); MG_COMPUTE(p) MG_PARK(q, q) __syncthreads(); }
#define MG_STEP_PARK(p, q)     { MG_COMPUTE(p) MG_PARK(q, q) __syncthreads(); }
#define MG_STEP_LAST(p)        { MG_COMPUTE(p) }
    if (nk >= 3) {
        MG_LOAD(0, 0)
        MG_LOAD(1, 1)
        MG_PARK(0, 0)
        __syncthreads();
        int kt = 0;
        for (; kt + 3 < nk; kt += 2) {
            MG_STEP_FULL(0, 1, kt)
            MG_STEP_FULL(1, 0, kt + 1)
        }
        if (nk - kt == 3) {
            MG_STEP_FULL(0, 1, kt)
            MG_STEP_PARK(1, 0)
            MG_STEP_LAST(0)
        } else {
            MG_STEP_PARK(0, 1)
            MG_STEP_LAST(1)
        }
    } else {
        for (int kt = 0; kt < nk; ++kt) {
            MG_LOAD(0, kt)
            MG_PARK(0, 0)
            __syncthreads();
            MG_COMPUTE(0)
            __syncthreads();
        }
    }
#undef MG_LOAD
#undef MG_PARK
#undef MG_COMPUTE
#undef MG_FRAGS
#undef MG_MFMAS
#undef MG_STEP_FULL
#undef MG_STEP_PARK
#undef MG_STEP_LAST

#pragma unroll
    for (int i = 0; i < TM; ++i) mg_epilogue<EPI, BN, TN, WGN>(acc[i], a, m0 + wm * TM * 32 + i * 32, nb, wn, ks, lane);
}

// ------------------------------------------------------------------ large-M GEMM, 256 x 256 tiles
// One workgroup of four waves per CU; each wave owns a 128 x 128 block of C (16 accumulator tiles, 256
// registers), so one k-slice of 16 costs 8 LDS fragment reads for 16 MFMAs -- half the LDS traffic per
// flop of the 128 x 128 kernel, which is bound by it.
//  * Operands are staged by global -> LDS loads (no registers in between) into four stages of 32 k each;
//    rows are 64 B and the 16-byte chunks of a row are XOR-swizzled with (row >> 2) & 3 -- on the
//    source side of the load -- so that the fragment reads are bank-conflict free without padding.
//    W stays bf16 in LDS and is converted to fp16 in registers after the fragment read.
//  * The staging loads are issued from inline assembly: the compiler's wait-count pass would otherwise
//    force every one of them to complete at each barrier.  vmcnt is therefore managed by hand -- a
//    tile's loads are issued three k-tiles ahead, and every step waits until at most the two youngest
//    tiles (16 loads per wave) are in flight.  The loop issues the same number of loads on every trip
//    (the last trips re-request the final tile), so the counts hold to the end; vmcnt(0) before the
//    epilogue makes sure no load can land in LDS after the workgroup has ended.
//  * The instruction order inside a k-slice is fixed with scheduling fences: one MFMA, then one unit of
//    the next slice's preparation (a fragment read, half a fragment's conversion, a staging load).
//  * One barrier per k-tile: after it, every wave has read its last fragments of the tile's stage, which
//    can then be refilled, and the next tile is complete in LDS.
// Requires K % 128 == 0 and operand byte offsets below 4 GiB (checked by the launcher).
template <int EPI>
__global__ __launch_bounds__(256, 1) void gemm_big_kernel(GemmArgs a) {
    constexpr int BM = 256, BN = 256;
    extern __shared__ __attribute__((aligned(1024))) char smem[];   // [4 stages][A 16 KB | W 16 KB]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int NB = a.n_blocks_n, MB = (a.M + BM - 1) / BM;
    int nb, mb;
    if (!tile_of(blockIdx.x, MB, NB, mb, nb)) return;
    const int m0 = mb * BM;
    const int nk = a.K / 32;
    // Staging: instruction t of wave w fills LDS bytes [(t*4 + w) KB, +1 KB) of the A (or W) part of a
    // stage = tile rows (t*4+w)*16 .. +16; lane -> row + lane/4, physical chunk lane%4, which holds the
    // row's logical chunk (lane%4) ^ ((row>>2)&3).
    unsigned a_off[4], w_off[4];
    {
        const int lc = (lane & 3) ^ ((lane >> 4) & 3);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int r = (t * 4 + wave) * 16 + (lane >> 2);
            a_off[t] = ((unsigned)min(m0 + r, a.M - 1) * (unsigned)a.lda + lc * 8) * 2u;   // rows >= M: clamped, never stored
            w_off[t] = ((unsigned)min(w_row_of<EPI, BN>(r, nb, a), a.Wrows - 1) * (unsigned)a.K + lc * 8) * 2u;
        }
    }
    const char* Ag = reinterpret_cast<const char*>(a.A);
    const char* Wg = reinterpret_cast<const char*>(a.W);
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) char*)smem;
#define BG_LOAD(stage, kt, q)                                                                                   \
    {                                                                                                           \
        const unsigned sa_ = lds_base + (stage) * 32768 + wave * 1024 + ((q) & 3) * 4096 + ((q) >> 2) * 16384;  \
        const char* g_ = ((q) < 4 ? Ag : Wg) + (size_t)(kt) * 64;                                               \
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"                            \
                     :: "s"(sa_), "v"((q) < 4 ? a_off[(q) & 3] : w_off[(q) & 3]), "s"(g_) : "memory");          \
    }
    // fragment addresses: row lane%32 of a 32-row block, logical chunk ks*2 + lane/32, swizzled
    int fa[2][2], fw[2][2];   // [stage pair][k-slice]
#pragma unroll
    for (int hp = 0; hp < 2; ++hp)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const int ko = ((ks * 2 + (lane >> 5)) ^ ((lane >> 2) & 3)) * 16;
            fa[hp][ks] = hp * 65536 + (wm * 128 + (lane & 31)) * 64 + ko;
            fw[hp][ks] = hp * 65536 + 16384 + (wn * 128 + (lane & 31)) * 64 + ko;
        }
    floatx16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    half8 af[2][4];
    u32x4_t bf[2][4], bw[4];
#define BG_CVT2(w) __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(__uint_as_float((w) << 16), __uint_as_float((w) & 0xffff0000u)))
#define BG_LDA(stage, ks, i) *reinterpret_cast<const half8*>(smem + fa[(stage) >> 1][ks] + ((stage) & 1) * 32768 + (i) * 2048)
#define BG_LDW(stage, ks, j) *reinterpret_cast<const u32x4_t*>(smem + fw[(stage) >> 1][ks] + ((stage) & 1) * 32768 + (j) * 2048)
    // One k-slice: 16 MFMAs on fragment set CUR; between them, in this order, the 4 W and 4 A fragment
    // reads of slice (NSTAGE, NKS) into the other set, then the conversion of those W fragments; four
    // staging loads (requests HALF*4 .. +4 of tile DKT into stage DSTAGE) share slots with the fragment
    // reads, which keeps every slot within the eight issue cycles one MFMA covers.
#define BG_SLICE(CUR, NSTAGE, NKS, HALF, DSTAGE, DKT)                                                           \
    _Pragma("unroll") for (int q = 0; q < 16; ++q) {                                                            \
        const int j_ = q >> 2, i_ = q & 3;                                                                      \
        acc[i_][j_] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[CUR][i_], __builtin_bit_cast(half8, bf[CUR][j_]), acc[i_][j_], 0, 0, 0); \
        if (q < 4) bw[q & 3] = BG_LDW(NSTAGE, NKS, q & 3);                                                      \
        else if (q < 8) af[1 - (CUR)][q & 3] = BG_LDA(NSTAGE, NKS, q & 3);                                      \
        else {                                                                                                  \
            const int jj_ = (q - 8) >> 1, h_ = ((q - 8) & 1) * 2;                                               \
            bf[1 - (CUR)][jj_][h_] = BG_CVT2(bw[jj_][h_]);                                                      \
            bf[1 - (CUR)][jj_][h_ + 1] = BG_CVT2(bw[jj_][h_ + 1]);                                              \
        }                                                                                                       \
        if (q < 8 && (q & 1)) BG_LOAD(DSTAGE, DKT, (HALF) * 4 + (q >> 1))                                           \
        __builtin_amdgcn_sched_barrier(0);                                                                      \
    }
    // k-tile kt sits in stage S = kt % 4.  Its first slice also issues the second half of the requests
    // for tile kt+3; after the barrier its stage is free and takes the first half of tile kt+4.
#define BG_STEP(S, KT)                                                                                          \
    {                                                                                                           \
        { const int dkt_ = min((KT) + 3, nk - 1);                                                               \
          BG_SLICE(0, S, 1, 1, ((S) + 3) & 3, dkt_) }                                                           \
        __builtin_amdgcn_s_waitcnt(0x4070);   /* vmcnt(16) lgkmcnt(0): own part of tile kt+1 landed */         \
        __syncthreads();                                                                                        \
        __builtin_amdgcn_sched_barrier(0);                                                                      \
        { const int dkt_ = min((KT) + 4, nk - 1);                                                               \
          BG_SLICE(1, ((S) + 1) & 3, 0, 0, S, dkt_) }                                                           \
    }
    // prologue: tiles 0..2 and the first half of tile 3
#pragma unroll
    for (int st = 0; st < 4; ++st) {
        const int kt_ = min(st, nk - 1);
#pragma unroll
        for (int q = 0; q < (st < 3 ? 8 : 4); ++q) BG_LOAD(st, kt_, q)
    }
    __builtin_amdgcn_s_waitcnt(0x4F74);   // vmcnt(20): tile 0 landed
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) af[0][i] = BG_LDA(0, 0, i);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        bw[j] = BG_LDW(0, 0, j);
#pragma unroll
        for (int c = 0; c < 4; ++c) bf[0][j][c] = BG_CVT2(bw[j][c]);
    }
    for (int kt = 0; kt < nk; kt += 4) {   // nk % 4 == 0
        BG_STEP(0, kt)
        BG_STEP(1, kt + 1)
        BG_STEP(2, kt + 2)
        BG_STEP(3, kt + 3)
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): nothing may land in LDS after the workgroup ends
#undef BG_LOAD
#undef BG_CVT2
#undef BG_LDA
#undef BG_LDW
#undef BG_SLICE
#undef BG_STEP
    // written out: with the largest epilogue the unroller gives up on a loop over the four bands
    mg_epilogue<EPI, BN, 4, 2>(acc[0], a, m0 + wm * 128, nb, wn, 0, lane);
    mg_epilogue<EPI, BN, 4, 2>(acc[1], a, m0 + wm * 128 + 32, nb, wn, 0, lane);
    mg_epilogue<EPI, BN, 4, 2>(acc[2], a, m0 + wm * 128 + 64, nb, wn, 0, lane);
    mg_epilogue<EPI, BN, 4, 2>(acc[3], a, m0 + wm * 128 + 96, nb, wn, 0, lane);
}

// ------------------------------------------------------------------ weight-streaming GEMM (decode, M <= 128)
// One workgroup = 128 rows x 128 columns of C over one K slice, computed by two teams of
// four waves: team t takes the k-tiles t, t+2, t+4, ... of the slice (a split over K inside
// the workgroup, reduced through LDS at the end), so every SIMD hosts two waves that hide
// each other's LDS / MFMA-issue latencies.  Inside a team the four waves split the columns
// (32 each, two 16-wide MFMA tiles) and each wave reads ITS OWN rows of W straight from
// global memory in B-operand layout (every row contributes 64 contiguous bytes per load
// instruction), one k-tile ahead of the one being consumed; W never touches LDS.  The
// activations (shared by a team's waves, and L2-resident) are staged through LDS.
// v_mfma_f32_16x16x32_f16, fp32 accumulation.
//   SG_PARTIAL: outF[ks][m][n] = partial sum of K slice ks
//   SG_SWIGLU : a wave's two column tiles are (gate, up) rows of W for the same 16 outputs;
//               the workgroup covers 64 outputs; outH[m][n] = silu(gate) * up
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
enum { SG_PARTIAL = 0, SG_SWIGLU = 1 };
#define SG_BK 64                       // k extent of one team step
#define SG_STRIDE (SG_BK + 16)          // halfs per LDS row: 160 B rows measured conflict-free for the 16x16x32 operand order (144 B is not)
#define SG_TILE_HALFS (128 * SG_STRIDE)
#define SG_ACH (SG_BK / 16)             // 16-byte A chunks per thread per step
#define SG_WLD (SG_BK / 16)             // W loads per wave-lane per step (k32 steps x 2 column tiles)

template <int EPI>
__global__ __launch_bounds__(512) void gemm_stream_kernel(GemmArgs a) {
    // [team][buffer][128 rows x LDS_STRIDE]; reused as a 128 x 128 fp32 tile for the team reduction
    __shared__ __attribute__((aligned(16))) f16_t As[2 * 2 * SG_TILE_HALFS];
    const int tid = threadIdx.x & 255, lane = tid & 63, wave = tid >> 6, team = threadIdx.x >> 8;
    const int c16 = lane & 15, g4 = lane >> 4;
    const int nb = blockIdx.x, ks = blockIdx.y;
    const int kbeg = ks * a.k_per_split, kend = min(a.K, kbeg + a.k_per_split);
    // team steps of the slice: (kend - kbeg) / SG_BK, an even number (the launcher guarantees it);
    // this team's steps start at kbeg + team * SG_BK and are 2 * SG_BK apart
    const int nk = (kend - kbeg) / (2 * SG_BK);
    const int k0 = kbeg + team * SG_BK;
    constexpr int KS = 2 * SG_BK;
    f16_t* As0 = As + team * 2 * SG_TILE_HALFS;
    f16_t* As1 = As0 + SG_TILE_HALFS;

    // this lane's two W rows
    const bf16_t* wp[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        int row;
        if (EPI == SG_SWIGLU) row = (j ? a.up_offset : 0) + nb * 64 + wave * 16 + c16;
        else row = nb * 128 + wave * 32 + j * 16 + c16;
        wp[j] = a.W + (int64_t)row * a.K + k0 + g4 * 8;
    }
    // A staging: 4 chunks of 16 B per thread per k-tile.  Rows >= M are read from row M-1: a row
    // of C depends on the same row of A only, and rows >= M are never stored.
    const f16_t* a_src[SG_ACH];
    int a_dst[SG_ACH];
#pragma unroll
    for (int i = 0; i < SG_ACH; ++i) {
        int c = tid + i * 256, r = c / (SG_BK / 8), kc = c % (SG_BK / 8);
        a_src[i] = a.A + (int64_t)min(r, a.M - 1) * a.lda + k0 + kc * 8;
        a_dst[i] = r * SG_STRIDE + kc * 8;
    }
    u32x4 ra[SG_ACH];               // the A tile in flight (requested after the previous one was parked in LDS)
    u32x4 wq0[SG_WLD], wq1[SG_WLD]; // W tiles in flight, index = k32 step * 2 + column tile
    floatx4 acc[8][2];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

#define SG_WLOAD(ptr, kt) (*reinterpret_cast<const u32x4*>(ptr))
#define SG_LOAD_A(kt)                                                                            \
    _Pragma("unroll") for (int i_ = 0; i_ < SG_ACH; ++i_)                                        \
        ra[i_] = *reinterpret_cast<const u32x4*>(a_src[i_] + (kt) * KS);
#define SG_LOAD_W(sl, kt)                                                                        \
    _Pragma("unroll") for (int s_ = 0; s_ < SG_BK / 32; ++s_) _Pragma("unroll") for (int j_ = 0; j_ < 2; ++j_) \
        wq##sl[s_ * 2 + j_] = SG_WLOAD(wp[j_] + (kt) * KS + s_ * 32, kt);
#define SG_CONVERT(sl)                                                                           \
    _Pragma("unroll") for (int q_ = 0; q_ < SG_WLD; ++q_) cf[q_] = bf16x8_to_half8(wq##sl[q_]);
#define SG_STORE_A(sl)                                                                           \
    _Pragma("unroll") for (int i_ = 0; i_ < SG_ACH; ++i_) *reinterpret_cast<u32x4*>(&As##sl[a_dst[i_]]) = ra[i_];
#define SG_COMPUTE(sl)                                                                           \
    _Pragma("unroll") for (int s_ = 0; s_ < SG_BK / 32; ++s_) {                                  \
        _Pragma("unroll") for (int i_ = 0; i_ < 8; ++i_) {                                       \
            half8 af_ = *reinterpret_cast<const half8*>(                                         \
                &As##sl[(i_ * 16 + c16) * SG_STRIDE + s_ * 32 + g4 * 8]);                        \
            acc[i_][0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(af_, cf[s_ * 2 + 0], acc[i_][0], 0, 0, 0); \
            acc[i_][1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(af_, cf[s_ * 2 + 1], acc[i_][1], 0, 0, 0); \
        }                                                                                        \
    }
    // Step kt (slot = kt & 1): convert W tile kt to fp16, which frees its raw registers for the
    // request of W tile kt+2 -- two full steps before it is needed; consume; park A tile kt+1 in
    // the other LDS buffer and request A tile kt+2.
#define SG_STEP_FULL(sl, other, kt)  { SG_CONVERT(sl) SG_LOAD_W(sl, (kt) + 2) __builtin_amdgcn_sched_barrier(0); SG_COMPUTE(sl) SG_STORE_A(other) SG_LOAD_A((kt) + 2) __syncthreads(); }
#define SG_STEP_NOLOAD(sl, other)    { SG_CONVERT(sl) SG_COMPUTE(sl) SG_STORE_A(other) __syncthreads(); }
#define SG_STEP_LAST(sl)             { SG_CONVERT(sl) SG_COMPUTE(sl) }

    // The steady-state path has no conditional loads anywhere between its first request and its
    // last wait: with vector loads returning in order, a wait count is exact only when every path
    // to it has issued the same requests.  Short K slices take a separate, simpler path.
    half8 cf[SG_WLD];
    if (nk >= 4) {
        SG_LOAD_A(0)
        SG_LOAD_W(0, 0)
        SG_STORE_A(0)
        SG_LOAD_A(1)
        SG_LOAD_W(1, 1)
        __syncthreads();
        int kt = 0;
        for (; kt + 3 < nk; kt += 2) {
            SG_STEP_FULL(0, 1, kt)
            SG_STEP_FULL(1, 0, kt + 1)
        }
        if (nk - kt == 3) {
            SG_STEP_FULL(0, 1, kt)
            SG_STEP_NOLOAD(1, 0)
            SG_STEP_LAST(0)
        } else {
            SG_STEP_NOLOAD(0, 1)
            SG_STEP_LAST(1)
        }
    } else {
        for (int kt = 0; kt < nk; ++kt) {
            SG_LOAD_A(kt)
            SG_LOAD_W(0, kt)
            SG_STORE_A(0)
            __syncthreads();
            SG_CONVERT(0)
            SG_COMPUTE(0)
            __syncthreads();
        }
    }
#undef SG_COMPUTE
#undef SG_STEP_FULL
#undef SG_STEP_NOLOAD
#undef SG_STEP_LAST
#undef SG_LOAD_A
#undef SG_LOAD_W
#undef SG_CONVERT
#undef SG_STORE_A

    // team reduction: team 1 parks its accumulators in LDS as a 128 x 128 fp32 tile (row m,
    // tile-local column), team 0 adds them to its own, in this fixed order
    __syncthreads();
    float* red = reinterpret_cast<float*>(As);
    if (team == 1) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    red[(i * 16 + g4 * 4 + r) * 128 + wave * 32 + j * 16 + c16] = acc[i][j][r];
    }
    __syncthreads();
    if (team == 1) return;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                acc[i][j][r] += red[(i * 16 + g4 * 4 + r) * 128 + wave * 32 + j * 16 + c16];

    // epilogue: acc[i][j][r] = C(row i*16 + g4*4 + r, column tile j, col c16)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int m = i * 16 + g4 * 4 + r;
            if (m >= a.M) continue;
            if (EPI == SG_PARTIAL) {
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    int n = nb * 128 + wave * 32 + j * 16 + c16;
                    a.outF[(int64_t)ks * a.split_stride + (int64_t)m * a.ldc + n] = acc[i][j][r];
                }
            } else {
                int n = nb * 64 + wave * 16 + c16;
                float g = acc[i][0][r], u = acc[i][1][r];
                a.outH[(int64_t)m * a.ldc + n] = (f16_t)(g / (1.0f + __expf(-g)) * u);
            }
        }
    }
}

// K slices hold an even number of team steps (two teams per workgroup).
static void stream_split(GemmArgs& a, int& splits) {
    if (splits < 1) splits = 1;
    int kt2 = a.K / (2 * SG_BK);                  // pairs of team steps
    int per = (kt2 + splits - 1) / splits;
    a.k_per_split = per * 2 * SG_BK;
    splits = (kt2 + per - 1) / per;
}

bool k_gemm_stream_supported(int N, int K) { return K % (2 * SG_BK) == 0 && N % 128 == 0; }

int k_gemm_stream_splits_used(int K, int splits) {
    GemmArgs a;
    a.K = K;
    stream_split(a, splits);
    return splits;
}

void k_gemm_stream(int epi, GemmArgs a, int splits, hipStream_t s) {
    if (a.M <= 0 || a.N <= 0) return;
    stream_split(a, splits);
    if (epi == MG_SWIGLU) {
        dim3 grid(a.N / 64, 1);
        gemm_stream_kernel<SG_SWIGLU><<<grid, 512, 0, s>>>(a);
    } else {
        dim3 grid(a.N / 128, splits);
        gemm_stream_kernel<SG_PARTIAL><<<grid, 512, 0, s>>>(a);
    }
}

template <int BM, int BN, int WGM, int WGN, int EPI, int BKT = 64>
static void launch(const GemmArgs& a, int n_blocks_n, int splits, hipStream_t s) {
    constexpr size_t lds = (size_t)2 * (BM + BN) * (BKT + 8) * sizeof(f16_t);
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void*)gemm_mfma_kernel<BM, BN, WGM, WGN, EPI, BKT>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        attr_set = true;
    }
    GemmArgs b = a;
    b.n_blocks_n = n_blocks_n;
    dim3 grid(8 * ((n_blocks_n * ((a.M + BM - 1) / BM) + 7) / 8), 1, splits);
    gemm_mfma_kernel<BM, BN, WGM, WGN, EPI, BKT><<<grid, 256, lds, s>>>(b);
}

template <int EPI>
static void launch_big(const GemmArgs& a, int n_blocks_n, hipStream_t s) {
    constexpr int lds = 4 * 32768;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void*)gemm_big_kernel<EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        attr_set = true;
    }
    GemmArgs b = a;
    b.n_blocks_n = n_blocks_n;
    dim3 grid(8 * ((n_blocks_n * ((a.M + 255) / 256) + 7) / 8));
    gemm_big_kernel<EPI><<<grid, 256, lds, s>>>(b);
}

bool k_gemm_mfma_supported(int epi, int N, int K, int hd) {
    if (K % BK != 0) return false;
    if (epi == MG_SWIGLU) return N % 64 == 0;
    if (epi == MG_QKV) return N % 128 == 0 && (hd == 64 || hd == 128);
    return N % 128 == 0;
}

// Whether the 256 x 256 kernel takes this GEMM (a.Wrows filled in).
static bool use_big(int epi, const GemmArgs& a, int splits) {
    if (!a.big_mode || splits != 1) return false;
    const int out_cols = epi == MG_SWIGLU ? 2 * a.N : a.N;   // tile columns
    if (out_cols % 256 != 0 || a.K % 128 != 0) return false;
    if ((uint64_t)a.M * a.lda * 2 >= (1ull << 32) || (uint64_t)a.Wrows * a.K * 2 >= (1ull << 32)) return false;
    const int64_t tiles = (int64_t)((a.M + 255) / 256) * (out_cols / 256);
    return a.big_mode >= 2 || tiles >= 512;   // one workgroup per CU: at least two rounds of 256
}

int k_gemm_mfma_lse_parts(int M, int N, int K, int big_mode) {
    GemmArgs a;
    a.M = M; a.N = N; a.K = K; a.lda = K; a.Wrows = N; a.big_mode = big_mode;
    return use_big(MG_LSE, a, 1) ? N / 128 : N / 64;
}

void k_gemm_mfma(int epi, GemmArgs a, int splits, hipStream_t s) {
    if (a.M <= 0 || a.N <= 0) return;
    if (splits < 1) splits = 1;
    int kt = a.K / BK;
    int per = (kt + splits - 1) / splits;
    a.k_per_split = per * BK;
    splits = (kt + per - 1) / per;
    a.Wrows = epi == MG_SWIGLU ? a.up_offset + a.N : a.N;
    const bool big = use_big(epi, a, splits);
    switch (epi) {
        case MG_STORE_F32:
            if (big) launch_big<MG_STORE_F32>(a, a.N / 256, s);
            else launch<128, 128, 2, 2, MG_STORE_F32>(a, a.N / 128, splits, s);
            break;
        case MG_STORE_F16:
            if (big) launch_big<MG_STORE_F16>(a, a.N / 256, s);
            else launch<128, 128, 2, 2, MG_STORE_F16>(a, a.N / 128, 1, s);
            break;
        case MG_RESID:
            if (big) launch_big<MG_RESID>(a, a.N / 256, s);
            else launch<128, 128, 2, 2, MG_RESID>(a, a.N / 128, 1, s);
            break;
        case MG_SWIGLU:
            if (big) launch_big<MG_SWIGLU>(a, a.N / 128, s);
            else launch<128, 128, 2, 2, MG_SWIGLU>(a, a.N / 64, 1, s);
            break;
        case MG_LSE:
            if (big) launch_big<MG_LSE>(a, a.N / 256, s);
            else launch<128, 128, 2, 2, MG_LSE>(a, a.N / 128, 1, s);
            break;
        case MG_QKV:
            if (big) launch_big<MG_QKV>(a, a.N / 256, s);
            else launch<128, 128, 2, 2, MG_QKV>(a, a.N / 128, 1, s);
            break;
        default: break;
    }
}

int k_gemm_mfma_splits_used(int K, int splits) {
    int kt = K / BK;
    if (splits < 1) splits = 1;
    int per = (kt + splits - 1) / splits;
    return (kt + per - 1) / per;
}
