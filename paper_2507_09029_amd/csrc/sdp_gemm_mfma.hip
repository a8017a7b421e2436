// bf16 MFMA contraction for gfx950 (CDNA4) with the masked-MLP gathers and SwiGLU epilogues fused.
//
//   C[M][N] = sum_k A(m,k) B(k,n),  bf16 operands, fp32 accumulation in v_mfma_f32_32x32x16_bf16.
//
// Workgroup: 256 threads = 4 waves (2 x 2), output tile 128 x 128, depth step 64.  Each wave owns a
// 64 x 64 sub-tile = 2 x 2 MFMA tiles of 32 x 32 (64 accumulator registers per lane).
// Global -> registers -> LDS, two LDS stages, one barrier per depth step; the loads of step t+1 are
// issued before the MFMAs of step t.
//
// Operand tiles in LDS are stored in 16-byte chunks (8 bf16) exactly as they arrive from HBM:
//   "row tile"  [128 rows][64 k]   : A always; B when it is stored [N][K].  A lane's MFMA operand is
//                one chunk -> one ds_read_b128.  Chunk (r, c) sits at r*8 + (c ^ ((r >> 1) & 7)).
//   "k tile"    [64 k][128 cols]   : B when it is stored [K][N] (the gathered-row weights of the
//                down / dX contractions, X and dY of the weight-gradient contractions).  The MFMA
//                operand needs 8 consecutive k of one column, i.e. a transpose: two
//                ds_read_b64_tr_b16 per fragment.  Chunk (k, c) sits at k*16 + (c ^ ((k & 3) << 2)).
// Both XOR patterns make the per-cycle lane groups of the reads hit distinct banks.
//
// Row gathers (active-neuron indices) are applied when forming global addresses: a gathered row
// is still one contiguous run of K (or N) elements, so every global access stays a 16-byte load.
#include "sdp_internal.h"
#include "sdp_swiglu.h"

namespace sdp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;

constexpr int BM = 128, BN = 128, BK = 64, NTHREADS = 256;
constexpr int A_TILE_BYTES = BM * BK * 2;          // 16 KB
constexpr int B_TILE_BYTES = BN * BK * 2;          // 16 KB
constexpr int STAGE_BYTES = A_TILE_BYTES + B_TILE_BYTES;
constexpr int LDS_BYTES = 2 * STAGE_BYTES;         // 64 KB: two workgroups per CU

struct Dev {
    int M, N, K;
    const uint16_t *A, *A2, *B, *B2;
    int64_t lda, ldb;
    const int32_t *ag, *bg, *cs;
    uint16_t *C, *C2, *C3;
    int64_t ldc;
    const uint16_t *Gin, *Uin;
    int64_t ldg;
    uint16_t *T1, *T2, *T3;
    int64_t ldt;
    int tiles_m, tiles_n;
};

__device__ inline u32x4 ldg16(const uint16_t* p) { return *(const u32x4*)p; }

__device__ inline int row_chunk(int r, int c) { return r * 8 + (c ^ ((r >> 1) & 7)); }
__device__ inline int k_chunk(int k, int c) { return k * 16 + (c ^ ((k & 3) << 2)); }

__device__ inline uint32_t pack_bf16(float lo, float hi) {
    return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

// B_KN: 0 = B stored [N][K] (row tile), 1 = B stored [K][N] (k tile).
template <int B_KN, int EPI>
__global__ __launch_bounds__(NTHREADS, 2) void gemm_mfma_kernel(Dev g) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr bool kFwd = EPI == EPI_SWIGLU_FWD;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    const int tile_n = blockIdx.x % g.tiles_n, tile_m = blockIdx.x / g.tiles_n;
    const int m0 = tile_m * BM;
    // SWIGLU_FWD: the 128 tile columns are 64 neurons x {gate, up}
    const int n0 = kFwd ? tile_n * (BN / 2) : tile_n * BN;

    // ---- per-thread global load coordinates (fixed over the depth loop where possible) ----
    // row tile: 1024 chunks, thread -> rows tid/8 + 32 i, chunk tid%8
    const int lr = tid >> 3, lc = tid & 7;
    const uint16_t* a_row[4];
    const uint16_t* a2_row[4];
    const uint16_t* b_row[4];  // B_KN == 0 only
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int m = m0 + lr + 32 * i;
        m = m < g.M ? m : g.M - 1;
        const int64_t row = g.ag ? g.ag[m] : m;
        a_row[i] = g.A + row * g.lda + lc * 8;
        a2_row[i] = EPI == EPI_DUAL_ACC ? g.A2 + row * g.lda + lc * 8 : nullptr;
        if (!B_KN) {
            const int r = lr + 32 * i; // tile row 0..127
            int n;
            const uint16_t* base = g.B;
            if (kFwd) {
                n = n0 + (r & 63);
                if (r >= 64) base = g.B2;
            } else {
                n = n0 + r;
            }
            n = n < g.N ? n : g.N - 1;
            const int64_t brow = g.bg ? g.bg[n] : n;
            b_row[i] = base + brow * g.ldb + lc * 8;
        }
    }
    // k tile: 1024 chunks, thread -> k rows tid/16 + 16 i, chunk tid%16
    const int kr = tid >> 4, kc = tid & 15;
    const bool kcol_ok = B_KN ? (n0 + kc * 8 < g.N) : true;

    const int nk1 = (g.K + BK - 1) / BK;
    const int nk = EPI == EPI_DUAL_ACC ? 2 * nk1 : nk1;

    u32x4 ra[4], rb[4];
    const u32x4 zero4 = {0u, 0u, 0u, 0u};

    auto load_tile = [&](int kt) {
        const bool second = EPI == EPI_DUAL_ACC && kt >= nk1;
        const int k0 = (second ? kt - nk1 : kt) * BK;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const bool ok = k0 + lc * 8 < g.K;
            const uint16_t* p = (second ? a2_row[i] : a_row[i]) + k0;
            ra[i] = ok ? ldg16(p) : zero4;
        }
        if (!B_KN) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const bool ok = k0 + lc * 8 < g.K;
                rb[i] = ok ? ldg16(b_row[i] + k0) : zero4;
            }
        } else {
            const uint16_t* base = second ? g.B2 : g.B;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int k = k0 + kr + 16 * i;
                const bool ok = kcol_ok && k < g.K;
                const int kk = k < g.K ? k : g.K - 1;
                const int64_t row = g.bg ? g.bg[kk] : kk;
                rb[i] = ok ? ldg16(base + row * g.ldb + n0 + kc * 8) : zero4;
            }
        }
    };
    auto store_tile = [&](int stage) {
        unsigned char* sa = smem + stage * STAGE_BYTES;
        unsigned char* sb = sa + A_TILE_BYTES;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            *(u32x4*)(sa + row_chunk(lr + 32 * i, lc) * 16) = ra[i];
            if (!B_KN)
                *(u32x4*)(sb + row_chunk(lr + 32 * i, lc) * 16) = rb[i];
            else
                *(u32x4*)(sb + k_chunk(kr + 16 * i, kc) * 16) = rb[i];
        }
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // tile rows / columns of this wave's fragments
    const int l32 = lane & 31, lhi = lane >> 5;
    int bfrag[2];
    bfrag[0] = kFwd ? 32 * wn : 64 * wn;
    bfrag[1] = kFwd ? 64 + 32 * wn : 64 * wn + 32;

    load_tile(0);
    store_tile(0);
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const int stage = kt & 1;
        if (kt + 1 < nk) load_tile(kt + 1);
        const unsigned char* sa = smem + stage * STAGE_BYTES;
        const unsigned char* sb = sa + A_TILE_BYTES;
#pragma unroll
        for (int s = 0; s < BK / 16; ++s) {
            bf16x8 fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int r = 64 * wm + 32 * i + l32;
                fa[i] = __builtin_bit_cast(bf16x8, *(const u32x4*)(sa + row_chunk(r, 2 * s + lhi) * 16));
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                if (!B_KN) {
                    const int r = bfrag[j] + l32;
                    fb[j] = __builtin_bit_cast(bf16x8, *(const u32x4*)(sb + row_chunk(r, 2 * s + lhi) * 16));
                } else {
                    // transposing read: inside each 16-lane block, lane i addresses 4 columns of row
                    // k + i/4; the block's lane n receives rows k..k+3 of column n.
                    const int blk = lane >> 4, li = lane & 15;
                    const int col = bfrag[j] + 16 * (blk & 1) + 4 * (li & 3);
                    const int kbase = 16 * s + 8 * (blk >> 1) + (li >> 2);
                    s16x4 h[2];
#pragma unroll
                    for (int hh = 0; hh < 2; ++hh) {
                        const int k = kbase + 4 * hh;
                        const unsigned char* p = sb + k_chunk(k, col >> 3) * 16 + (col & 4) * 2;
                        h[hh] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)p);
                    }
                    typedef short s16x8 __attribute__((ext_vector_type(8)));
                    s16x8 both = {h[0][0], h[0][1], h[0][2], h[0][3], h[1][0], h[1][1], h[1][2], h[1][3]};
                    fb[j] = __builtin_bit_cast(bf16x8, both);
                }
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) store_tile(stage ^ 1);
        __syncthreads();
    }

    // ---- epilogue.  acc[i][j][4q + r] is C(m, n) with
    //      m = m0 + 64 wm + 32 i + 8 q + 4 (lane / 32) + r,  n = (fragment j column base) + lane % 32
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int mb = m0 + 64 * wm + 32 * i + 8 * q + 4 * lhi;
            if (EPI == EPI_STORE || EPI == EPI_DUAL_ACC) {
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int n = n0 + bfrag[j] + l32;
                    if (n >= g.N) continue;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int m = mb + r;
                        if (m >= g.M) continue;
                        const int64_t row = g.cs ? g.cs[m] : m;
                        g.C[row * g.ldc + n] = f32_to_bf16(acc[i][j][4 * q + r]);
                    }
                }
            } else if (EPI == EPI_SWIGLU_FWD) {
                const int n = n0 + 32 * wn + l32;
                if (n >= g.N) continue;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int m = mb + r;
                    if (m >= g.M) continue;
                    const float gv = acc[i][0][4 * q + r], uv = acc[i][1][4 * q + r];
                    const int64_t o = (int64_t)m * g.ldc + n;
                    g.C[o] = f32_to_bf16(gv);
                    g.C2[o] = f32_to_bf16(uv);
                    g.C3[o] = f32_to_bf16(swiglu_fwd<false>(gv, uv));
                }
            } else { // EPI_SWIGLU_BWD
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int n = n0 + bfrag[j] + l32;
                    if (n >= g.N) continue;
                    float dg[4], du[4], act[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int m = mb + r < g.M ? mb + r : g.M - 1;
                        const float gv = bf16_to_f32(g.Gin[(int64_t)m * g.ldg + n]);
                        const float uv = bf16_to_f32(g.Uin[(int64_t)m * g.ldg + n]);
                        swiglu_bwd<false>(acc[i][j][4 * q + r], gv, uv, dg[r], du[r], act[r]);
                        if (mb + r < g.M) {
                            const int64_t o = (int64_t)(mb + r) * g.ldc + n;
                            g.C[o] = f32_to_bf16(dg[r]);
                            g.C2[o] = f32_to_bf16(du[r]);
                        }
                    }
                    // neuron-major copies: 4 consecutive tokens of one neuron per lane
                    const int64_t t = (int64_t)n * g.ldt + mb;
                    if (mb + 3 < g.M && (g.ldt & 3) == 0) {
                        *(u32x2*)(g.T1 + t) = u32x2{pack_bf16(dg[0], dg[1]), pack_bf16(dg[2], dg[3])};
                        *(u32x2*)(g.T2 + t) = u32x2{pack_bf16(du[0], du[1]), pack_bf16(du[2], du[3])};
                        *(u32x2*)(g.T3 + t) = u32x2{pack_bf16(act[0], act[1]), pack_bf16(act[2], act[3])};
                    } else {
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            if (mb + r >= g.M) continue;
                            g.T1[t + r] = f32_to_bf16(dg[r]);
                            g.T2[t + r] = f32_to_bf16(du[r]);
                            g.T3[t + r] = f32_to_bf16(act[r]);
                        }
                    }
                }
            }
        }
    }
}

template <int B_KN, int EPI>
int launch(const GemmDesc& d, hipStream_t s) {
    Dev g;
    g.M = d.M, g.N = d.N, g.K = d.K;
    g.A = (const uint16_t*)d.A, g.A2 = (const uint16_t*)d.A2, g.B = (const uint16_t*)d.B, g.B2 = (const uint16_t*)d.B2;
    g.lda = d.lda, g.ldb = d.ldb, g.ag = d.a_gather, g.bg = d.b_gather, g.cs = d.c_scatter;
    g.C = (uint16_t*)d.C, g.C2 = (uint16_t*)d.C2, g.C3 = (uint16_t*)d.C3, g.ldc = d.ldc;
    g.Gin = (const uint16_t*)d.Gin, g.Uin = (const uint16_t*)d.Uin, g.ldg = d.ldg;
    g.T1 = (uint16_t*)d.T1, g.T2 = (uint16_t*)d.T2, g.T3 = (uint16_t*)d.T3, g.ldt = d.ldt;
    g.tiles_m = (d.M + BM - 1) / BM;
    const int ncols = EPI == EPI_SWIGLU_FWD ? BN / 2 : BN;
    g.tiles_n = (d.N + ncols - 1) / ncols;
    const int64_t blocks = (int64_t)g.tiles_m * g.tiles_n;
    if (blocks > 0x7FFFFFFF) return SDP_ERR_SHAPE;
    auto kern = gemm_mfma_kernel<B_KN, EPI>;
    static bool attr_set = false; // one flag per template instantiation
    if (!attr_set) {
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) != hipSuccess)
            return SDP_ERR_HIP;
        attr_set = true;
    }
    ProfileScope ps(d.name, s);
    kern<<<dim3((unsigned)blocks), NTHREADS, LDS_BYTES, s>>>(g);
    return launch_status();
}

} // namespace

bool gemm_mfma_supported(const GemmDesc& d) {
    if (d.M < 1 || d.N < 1 || d.K < 1) return false;
    // 16-byte global chunks: every row start and every chunk must be 8-element aligned
    if (d.K % 8 || d.lda % 8 || d.ldb % 8) return false;
    if (d.b_kn && d.N % 8) return false;
    for (const void* p : {d.A, d.B}) if (!p || !aligned16(p)) return false;
    if (d.epilogue == EPI_DUAL_ACC || d.epilogue == EPI_SWIGLU_FWD)
        if (!d.B2 || !aligned16(d.B2)) return false;
    if (d.epilogue == EPI_DUAL_ACC && (!d.A2 || !aligned16(d.A2))) return false;
    if (d.epilogue == EPI_SWIGLU_FWD && d.b_kn) return false;
    if (d.epilogue == EPI_SWIGLU_BWD && d.b_kn) return false;
    return true;
}

int gemm_mfma_bf16(const GemmDesc& d, hipStream_t s) {
    if (!gemm_mfma_supported(d)) return SDP_ERR_UNSUPPORTED;
    if (d.b_kn) {
        if (d.epilogue == EPI_STORE) return launch<1, EPI_STORE>(d, s);
        if (d.epilogue == EPI_DUAL_ACC) return launch<1, EPI_DUAL_ACC>(d, s);
    } else {
        if (d.epilogue == EPI_STORE) return launch<0, EPI_STORE>(d, s);
        if (d.epilogue == EPI_SWIGLU_FWD) return launch<0, EPI_SWIGLU_FWD>(d, s);
        if (d.epilogue == EPI_SWIGLU_BWD) return launch<0, EPI_SWIGLU_BWD>(d, s);
    }
    return SDP_ERR_UNSUPPORTED;
}

} // namespace sdp
