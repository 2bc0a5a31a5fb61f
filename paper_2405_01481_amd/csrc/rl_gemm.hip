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

// Which row of W feeds LDS row r of the B tile of column-block nb.
//  EPI_SWIGLU: the tile holds BN/2 gate rows and the matching BN/2 up rows, interleaved in
//              blocks of 32 so that a wave's adjacent 32-column MFMA tiles are (gate, up).
//  MG_QKV with head_dim 128: the head's halves are interleaved in blocks of 32 so that a
//              wave holds columns j and j + 64 in the same lane.
template <int EPI, int BN>
__device__ __forceinline__ int w_row_of(int r, int nb, const GemmArgs& a) {
    if (EPI == MG_SWIGLU) {
        int blk = r >> 5, within = r & 31;
        int col = nb * (BN / 2) + (blk >> 1) * 32 + within;
        return (blk & 1) ? a.up_offset + col : col;
    } else if (EPI == MG_QKV && BN == 128) {
        if (a.hd == 128) {
            int blk = r >> 5, within = r & 31;      // LDS blocks: [0:32) [64:96) [32:64) [96:128)
            int src = ((blk & 1) ? 64 : 0) + (blk >> 1) * 32 + within;
            return nb * BN + src;
        }
        return nb * BN + r;
    } else {
        return nb * BN + r;
    }
}

template <int BM, int BN, int WGM, int WGN, int EPI>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(GemmArgs a) {
    constexpr int TM = BM / WGM / 32, TN = BN / WGN / 32;
    constexpr int A_CH = BM * 8 / 256, W_CH = BN * 8 / 256;   // 16-byte chunks per thread per k-tile
    extern __shared__ __attribute__((aligned(16))) char smem[];
    f16_t* As = reinterpret_cast<f16_t*>(smem);                   // [2][BM][LDS_STRIDE]
    f16_t* Ws = As + 2 * BM * LDS_STRIDE;                         // [2][BN][LDS_STRIDE]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int nb = blockIdx.x, mb = blockIdx.y, ks = blockIdx.z;
    const int m0 = mb * BM;
    const int kbeg = ks * a.k_per_split, kend = min(a.K, kbeg + a.k_per_split);
    const int nk = (kend - kbeg + BK - 1) / BK;

    // per-thread global source rows for the staged loads
    const f16_t* a_src[A_CH];
    const bf16_t* w_src[W_CH];
    int a_dst[A_CH], w_dst[W_CH];
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
        int c = tid + i * 256, r = c >> 3, kc = c & 7;
        int m = m0 + r;
        a_src[i] = (m < a.M) ? a.A + (int64_t)m * a.lda + kc * 8 : nullptr;
        a_dst[i] = r * LDS_STRIDE + kc * 8;
    }
#pragma unroll
    for (int i = 0; i < W_CH; ++i) {
        int c = tid + i * 256, r = c >> 3, kc = c & 7;
        int wr = w_row_of<EPI, BN>(r, nb, a);
        w_src[i] = (wr < a.Wrows) ? a.W + (int64_t)wr * a.K + kc * 8 : nullptr;
        w_dst[i] = r * LDS_STRIDE + kc * 8;
    }

    uint4 ra[A_CH], rw[W_CH];
    auto load_g = [&](int k0) {
#pragma unroll
        for (int i = 0; i < A_CH; ++i)
            ra[i] = a_src[i] ? *reinterpret_cast<const uint4*>(a_src[i] + k0) : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < W_CH; ++i)
            rw[i] = w_src[i] ? *reinterpret_cast<const uint4*>(w_src[i] + k0) : make_uint4(0, 0, 0, 0);
    };
    auto store_l = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_CH; ++i)
            *reinterpret_cast<uint4*>(As + buf * BM * LDS_STRIDE + a_dst[i]) = ra[i];
#pragma unroll
        for (int i = 0; i < W_CH; ++i)
            *reinterpret_cast<uint4*>(Ws + buf * BN * LDS_STRIDE + w_dst[i]) = bf16x8_to_f16x8(rw[i]);
    };

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    if (nk > 0) {
        load_g(kbeg);
        store_l(0);
    }
    __syncthreads();
    const int lrow = lane & 31, lk = (lane >> 5) * 8;
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) load_g(kbeg + (kt + 1) * BK);
        const f16_t* Ab = As + cur * BM * LDS_STRIDE + (wm * TM * 32 + lrow) * LDS_STRIDE + lk;
        const f16_t* Wb = Ws + cur * BN * LDS_STRIDE + (wn * TN * 32 + lrow) * LDS_STRIDE + lk;
#pragma unroll
        for (int kk = 0; kk < BK; kk += 16) {
            half8 af[TM], bf[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) af[i] = *reinterpret_cast<const half8*>(Ab + i * 32 * LDS_STRIDE + kk);
#pragma unroll
            for (int j = 0; j < TN; ++j) bf[j] = *reinterpret_cast<const half8*>(Wb + j * 32 * LDS_STRIDE + kk);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) store_l(cur ^ 1);
        __syncthreads();
    }

    // ---- epilogue.  acc[i][j][r] is C(row, col) with
    //   row = m0 + wm*TM*32 + i*32 + 8*(r/4) + 4*(lane/32) + r%4,   col(tile-local) = wn*TN*32 + j*32 + lane%32
    const int lg = lane >> 5;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = m0 + wm * TM * 32 + i * 32 + 8 * (r >> 2) + 4 * lg + (r & 3);
            if (m >= a.M) continue;
            if (EPI == MG_STORE_F32) {
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    int n = nb * BN + wn * TN * 32 + j * 32 + lrow;
                    if (n < a.N) a.outF[(int64_t)ks * a.split_stride + (int64_t)m * a.ldc + n] = acc[i][j][r];
                }
            } else if (EPI == MG_STORE_F16) {
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    int n = nb * BN + wn * TN * 32 + j * 32 + lrow;
                    if (n < a.N) a.outH[(int64_t)m * a.ldc + n] = (f16_t)acc[i][j][r];
                }
            } else if (EPI == MG_RESID) {
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    int n = nb * BN + wn * TN * 32 + j * 32 + lrow;
                    if (n < a.N) a.outF[(int64_t)m * a.ldc + n] += acc[i][j][r];
                }
            } else if (EPI == MG_SWIGLU) {
#pragma unroll
                for (int j = 0; j < TN; j += 2) {
                    int n = nb * (BN / 2) + (wn * TN + j) / 2 * 32 + lrow;
                    float g = acc[i][j][r], u = acc[i][j + 1][r];
                    if (n < a.N) a.outH[(int64_t)m * a.ldc + n] = (f16_t)(g / (1.0f + __expf(-g)) * u);
                }
            } else if (EPI == MG_QKV) {
                // columns of this tile belong to one head (hd 128) or two (hd 64); pairs (j, j + hd/2)
                // sit in adjacent 32-column MFMA tiles of this lane.
                const int pos = a.tok_pos[m];
                const int hd = a.hd, half = hd >> 1;
#pragma unroll
                for (int j = 0; j < TN; j += 2) {
                    // tile-local LDS column of acc[i][j]: c0; its partner acc[i][j+1] is c0 + 32 in LDS order
                    int c0 = wn * TN * 32 + j * 32 + lrow;
                    int col0;                             // global qkv column of v0; v1 is col0 + hd/2
                    if (hd == 128) {
                        int blk = c0 >> 5;                // even LDS block
                        col0 = nb * BN + (blk >> 1) * 32 + (c0 & 31);
                    } else {
                        col0 = nb * BN + c0;
                    }
                    float v0 = acc[i][j][r], v1 = acc[i][j + 1][r];
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
                        if (a.pool) {
                            int64_t page = a.block_table[(int64_t)a.tok_slot[m] * a.mpps + pos / a.geo.PT];
                            int st = pos % a.geo.PT;
                            a.pool[a.geo.k_off(a.layer, page, g, st, jj)] = (f16_t)v0;
                            a.pool[a.geo.k_off(a.layer, page, g, st, jj + half)] = (f16_t)v1;
                        }
                    } else {
                        int g = head - Hq - Hkv;
                        if (a.v_out) {
                            f16_t* o = a.v_out + ((int64_t)m * Hkv + g) * hd + jj;
                            o[0] = (f16_t)v0; o[half] = (f16_t)v1;
                        }
                        if (a.pool) {
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

template <int BM, int BN, int WGM, int WGN, int EPI>
static void launch(const GemmArgs& a, int n_blocks_n, int splits, hipStream_t s) {
    constexpr size_t lds = (size_t)2 * (BM + BN) * LDS_STRIDE * sizeof(f16_t);
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void*)gemm_mfma_kernel<BM, BN, WGM, WGN, EPI>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        attr_set = true;
    }
    dim3 grid(n_blocks_n, (a.M + BM - 1) / BM, splits);
    gemm_mfma_kernel<BM, BN, WGM, WGN, EPI><<<grid, 256, lds, s>>>(a);
}

bool k_gemm_mfma_supported(int epi, int N, int K, int hd) {
    if (K % BK != 0) return false;
    if (epi == MG_SWIGLU) return N % 64 == 0;
    if (epi == MG_QKV) return N % 128 == 0 && (hd == 64 || hd == 128);
    return N % 128 == 0;
}

void k_gemm_mfma(int epi, GemmArgs a, int splits, hipStream_t s) {
    if (a.M <= 0 || a.N <= 0) return;
    if (splits < 1) splits = 1;
    int kt = a.K / BK;
    int per = (kt + splits - 1) / splits;
    a.k_per_split = per * BK;
    splits = (kt + per - 1) / per;
    switch (epi) {
        case MG_STORE_F32: a.Wrows = a.N; launch<128, 128, 2, 2, MG_STORE_F32>(a, a.N / 128, splits, s); break;
        case MG_STORE_F16: a.Wrows = a.N; launch<128, 128, 2, 2, MG_STORE_F16>(a, a.N / 128, 1, s); break;
        case MG_RESID: a.Wrows = a.N; launch<128, 128, 2, 2, MG_RESID>(a, a.N / 128, 1, s); break;
        case MG_SWIGLU: a.Wrows = a.up_offset + a.N; launch<128, 128, 2, 2, MG_SWIGLU>(a, a.N / 64, 1, s); break;
        case MG_QKV: a.Wrows = a.N; launch<128, 128, 2, 2, MG_QKV>(a, a.N / 128, 1, s); break;
        default: break;
    }
}

int k_gemm_mfma_splits_used(int K, int splits) {
    int kt = K / BK;
    if (splits < 1) splits = 1;
    int per = (kt + splits - 1) / splits;
    return (kt + per - 1) / per;
}
