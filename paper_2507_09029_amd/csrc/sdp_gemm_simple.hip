// Plain LDS-tiled FMA contraction with the SwiGLU epilogues: the fp32 path of the masked MLP and
// the fallback for bf16 shapes the MFMA kernel does not take (ragged sizes).  Any M, N, K >= 1.
//
// 64 x 64 output tile per 256-thread workgroup, K step 16, 4 x 4 outputs per thread, operands
// widened to fp32 in LDS, fp32 accumulation.
#include "sdp_internal.h"
#include "sdp_swiglu.h"

namespace sdp {
namespace {

constexpr int BM = 64, BN = 64, BK = 16, NT = 256;

template <typename T>
__device__ inline float ld(const T* p);
template <>
__device__ inline float ld<float>(const float* p) {
    return *p;
}
template <>
__device__ inline float ld<uint16_t>(const uint16_t* p) {
    return bf16_to_f32(*p);
}
template <typename T>
__device__ inline void st(T* p, float v);
template <>
__device__ inline void st<float>(float* p, float v) {
    *p = v;
}
template <>
__device__ inline void st<uint16_t>(uint16_t* p, float v) {
    *p = f32_to_bf16(v);
}

struct Dev {
    int M, N, K;
    const void *A, *A2, *B, *B2;
    int64_t lda, ldb;
    const int32_t *bg, *cs;
    int a_km;
    const int32_t* ag;
    void *C, *C2, *C3;
    int64_t ldc;
    const void *Gin, *Uin;
    int64_t ldg;
    void *Cc, *Cc2, *Cc3;
    int64_t ldcc;
    const int32_t* cidx;
    int pc;
    const void* R; // STORE / DUAL_ACC: optional residual [M][ldr]
    int64_t ldr;
};

// rank of column n in the ascending index list, or -1 if it is not listed
__device__ inline int compact_rank(const int32_t* idx, int p, int n) {
    int lo = 0, hi = p;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (idx[mid] < n) lo = mid + 1; else hi = mid;
    }
    return (lo < p && idx[lo] == n) ? lo : -1;
}

template <typename T, int EPI>
__global__ __launch_bounds__(NT) void gemm_simple_kernel(Dev g) {
    constexpr bool kTwoB = EPI == EPI_SWIGLU_FWD;
    __shared__ float As[BK][BM + 4];
    __shared__ float Bs[BK][BN + 4];
    __shared__ float B2s[kTwoB ? BK : 1][BN + 4];
    const int tid = threadIdx.x;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int tm = (tid / 16) * 4, tn = (tid % 16) * 4;
    float acc[4][4] = {}, acc2[4][4] = {};

    const int passes = EPI == EPI_DUAL_ACC ? 2 : 1;
    for (int pass = 0; pass < passes; ++pass) {
        const T* A = (const T*)(pass ? g.A2 : g.A);
        const T* B = (const T*)(pass ? g.B2 : g.B);
        const T* B2 = (const T*)g.B2;
        for (int k0 = 0; k0 < g.K; k0 += BK) {
            if (!g.a_km) {
                // A tile: element e -> (m = e / BK, k = e % BK); rows contiguous along k
                for (int e = tid; e < BM * BK; e += NT) {
                    const int m = e / BK, k = e % BK;
                    float v = 0.f;
                    if (m0 + m < g.M && k0 + k < g.K) {
                        const int64_t row = g.ag ? g.ag[m0 + m] : (m0 + m);
                        v = ld<T>(A + row * g.lda + k0 + k);
                    }
                    As[k][m] = v;
                }
            } else {
                // A stored [K][M]: element e -> (k = e / BM, m = e % BM)
                for (int e = tid; e < BM * BK; e += NT) {
                    const int k = e / BM, m = e % BM;
                    float v = 0.f;
                    if (m0 + m < g.M && k0 + k < g.K) v = ld<T>(A + (int64_t)(k0 + k) * g.lda + m0 + m);
                    As[k][m] = v;
                }
            }
            for (int e = tid; e < BN * BK; e += NT) {
                const int n = e / BK, k = e % BK;
                float v = 0.f, v2 = 0.f;
                if (n0 + n < g.N && k0 + k < g.K) {
                    const int64_t row = g.bg ? g.bg[n0 + n] : (n0 + n);
                    v = ld<T>(B + row * g.ldb + k0 + k);
                    if (kTwoB) v2 = ld<T>(B2 + row * g.ldb + k0 + k);
                }
                Bs[k][n] = v;
                if (kTwoB) B2s[k][n] = v2;
            }
            __syncthreads();
#pragma unroll
            for (int k = 0; k < BK; ++k) {
                float a[4], b[4], b2[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    a[i] = As[k][tm + i];
                    b[i] = Bs[k][tn + i];
                    if (kTwoB) b2[i] = B2s[k][tn + i];
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        acc[i][j] = __builtin_fmaf(a[i], b[j], acc[i][j]);
                        if (kTwoB) acc2[i][j] = __builtin_fmaf(a[i], b2[j], acc2[i][j]);
                    }
            }
            __syncthreads();
        }
    }

#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + tm + i;
        if (m >= g.M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tn + j;
            if (n >= g.N) continue;
            if (EPI == EPI_STORE || EPI == EPI_DUAL_ACC) {
                const int64_t row = g.cs ? g.cs[m] : m;
                if (row < 0) continue; // dropped row
                const float r = g.R ? ld<T>((const T*)g.R + (int64_t)m * g.ldr + n) : 0.f;
                st<T>((T*)g.C + row * g.ldc + n, acc[i][j] + r);
            } else if (EPI == EPI_SWIGLU_FWD) {
                const float gv = acc[i][j], uv = acc2[i][j];
                st<T>((T*)g.C + (int64_t)m * g.ldc + n, gv);
                st<T>((T*)g.C2 + (int64_t)m * g.ldc + n, uv);
                st<T>((T*)g.C3 + (int64_t)m * g.ldc + n, swiglu_fwd<sizeof(T) == 4>(gv, uv));
            } else {
                const float gv = ld<T>((const T*)g.Gin + (int64_t)m * g.ldg + n);
                const float uv = ld<T>((const T*)g.Uin + (int64_t)m * g.ldg + n);
                float dg, du, act;
                swiglu_bwd<sizeof(T) == 4>(acc[i][j], gv, uv, dg, du, act);
                st<T>((T*)g.C + (int64_t)m * g.ldc + n, dg);
                st<T>((T*)g.C2 + (int64_t)m * g.ldc + n, du);
                st<T>((T*)g.C3 + (int64_t)m * g.ldc + n, act);
                if (g.cidx) {
                    const int c = compact_rank(g.cidx, g.pc, n);
                    if (c >= 0) {
                        st<T>((T*)g.Cc + (int64_t)m * g.ldcc + c, dg);
                        st<T>((T*)g.Cc2 + (int64_t)m * g.ldcc + c, du);
                        st<T>((T*)g.Cc3 + (int64_t)m * g.ldcc + c, act);
                    }
                }
            }
        }
    }
}

template <typename T, int EPI>
int launch(const GemmDesc& d, hipStream_t s) {
    Dev g{d.M, d.N, d.K, d.A, d.A2, d.B, d.B2, d.lda, d.ldb, d.b_gather, d.c_scatter, d.a_km, d.a_gather,
          d.C, d.C2, d.C3, d.ldc, d.Gin, d.Uin, d.ldg, d.Cc, d.Cc2, d.Cc3, d.ldcc, d.cidx, d.pc, d.R, d.ldr};
    dim3 grid((d.N + BN - 1) / BN, (d.M + BM - 1) / BM);
    ProfileScope ps(d.name, s);
    gemm_simple_kernel<T, EPI><<<grid, NT, 0, s>>>(g);
    return launch_status();
}

template <typename T>
int dispatch(const GemmDesc& d, hipStream_t s) {
    switch (d.epilogue) {
    case EPI_STORE: return launch<T, EPI_STORE>(d, s);
    case EPI_DUAL_ACC: return launch<T, EPI_DUAL_ACC>(d, s);
    case EPI_SWIGLU_FWD: return launch<T, EPI_SWIGLU_FWD>(d, s);
    case EPI_SWIGLU_BWD: return launch<T, EPI_SWIGLU_BWD>(d, s);
    }
    return SDP_ERR_INVALID_ARG;
}

} // namespace

int gemm_simple(int dtype, const GemmDesc& d, hipStream_t s) {
    if (d.M < 1 || d.N < 1 || d.K < 1) return SDP_ERR_SHAPE;
    if (d.a_gather && d.a_km) return SDP_ERR_UNSUPPORTED;
    if ((d.N + BN - 1) / BN > 0x7FFFFFFF || (d.M + BM - 1) / BM > 65535) return SDP_ERR_SHAPE;
    return dtype == SDP_F32 ? dispatch<float>(d, s) : dispatch<uint16_t>(d, s);
}

} // namespace sdp
