// Coverage-normalised gradient average (the paper's Sec. 3.1, eq. "average", with the load taken
// per coordinate): one streaming pass over the K workers' gradient buffers.
//
// HBM-bound.  Per neuron row of D parameters the kernel reads only the rows of workers whose mask
// covers it (16-byte loads, non-temporal), sums them in fp32 in worker order, divides by the
// coverage count and writes fp32 (non-temporal stores).  No atomics: the result is a pure function
// of the inputs.
//
// The same pass can apply the optimizer instead of storing the average (sdp_coverage_avg_adamw):
// the averaged gradient of a covered row goes straight into a decoupled-weight-decay Adam update of
// that row's fp32 parameters and moments, which are read and written once; rows nobody covers are
// left untouched.  A third form (sdp_coverage_grad_sqnorm) stores nothing and returns the squared norm of
// the average, which global gradient clipping needs before that fused update.
#include "sdp_internal.h"

#include <cmath>

namespace {

struct GradPtrs {
    const void* p[SDP_MAX_WORKERS];
};

// optimizer state and hyper-parameters of the fused update (OPT = 1)
struct AdamArgs {
    float* theta;
    float* m;
    float* v;
    uint16_t* theta_bf16; // optional bf16 copy of the updated parameters
    float decay;          // 1 - lr * weight_decay
    float beta1, beta2;
    float step_size;      // lr / (1 - beta1^t)
    float inv_sqrt_bc2;   // 1 / sqrt(1 - beta2^t)
    float eps;
    float grad_scale;
    const float* grad_scale_dev; // optional second factor, read from device memory by every workgroup
    double* partial;      // OPT = 2: one partial sum of squares per workgroup
};

constexpr int OPT_STORE = 0, OPT_ADAMW = 1, OPT_SQNORM = 2;

// Sum of one double per thread over a workgroup of 256 threads, in a fixed order: butterfly inside each wave,
// then the four waves' sums one after the other.  The result is valid in thread 0.
__device__ inline double block_sum(double x) {
    __shared__ double wave_sums[4];
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d, 64);
    if ((threadIdx.x & 63) == 0) wave_sums[threadIdx.x >> 6] = x;
    __syncthreads();
    return ((wave_sums[0] + wave_sums[1]) + wave_sums[2]) + wave_sums[3];
}

// clipping coefficient from n squared norms: min(1, max_norm / (sqrt(sum) + 1e-6)); one thread, n is small
__global__ void clip_scale_kernel(const double* __restrict__ sqnorm, int n, double max_norm, float* __restrict__ scale) {
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    double total = 0.0;
    for (int i = 0; i < n; ++i) total += sqnorm[i];
    const double coef = max_norm / (sqrt(total) + 1e-6);
    *scale = (float)(coef < 1.0 ? coef : 1.0);
}

// partial sums of the workgroups -> one number, again in a fixed order
__global__ __launch_bounds__(256) void sqnorm_finish_kernel(const double* __restrict__ partial, int n, double* __restrict__ out) {
    // four independent running sums per thread keep four loads in flight; the order of the additions is fixed
    double x0 = 0.0, x1 = 0.0, x2 = 0.0, x3 = 0.0;
    int i = threadIdx.x;
    for (; i + 768 < n; i += 1024) x0 += partial[i], x1 += partial[i + 256], x2 += partial[i + 512], x3 += partial[i + 768];
    for (; i < n; i += 256) x0 += partial[i];
    double x = block_sum((x0 + x1) + (x2 + x3));
    if (threadIdx.x == 0) *out = x;
}

__device__ inline uint32_t pack2_bf16(float lo, float hi) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const bf16x2 p = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, p);
}

// one parameter: (theta, m, v) <- AdamW(theta, m, v, g); gs = the gradient's scale
__device__ inline void adamw_one(const AdamArgs& a, float gs, float g, float& th, float& m, float& v) {
    g *= gs;
    th *= a.decay;
    m = a.beta1 * m + (1.0f - a.beta1) * g;
    v = a.beta2 * v + (1.0f - a.beta2) * g * g;
    const float denom = __builtin_sqrtf(v) * a.inv_sqrt_bc2 + a.eps;
    th -= a.step_size * (m / denom);
}

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ inline void add_bf16x8(const u32x4 w, float (&acc)[8]) {
    // a bf16 is the high half of an fp32: even elements sit in the low 16 bits of each word
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        acc[2 * i] += __uint_as_float(w[i] << 16);
        acc[2 * i + 1] += __uint_as_float(w[i] & 0xFFFF0000u);
    }
}

// One wave handles one 512-parameter segment of one row at a time (64 lanes x 8 parameters), so
// the row index, and with it every mask byte, is uniform across the wave.  Workers are taken in
// batches of kBatch: all loads of a batch are issued before the first is consumed, which keeps up
// to kBatch 16-byte (bf16) or 32-byte (fp32) requests per lane in flight.
// Requires D % 8 == 0.  BF16: 1 = bf16 input, 0 = fp32 input.
constexpr int kBatch = 8;

template <int BF16, int OPT>
__global__ __launch_bounds__(256) void avg_rows_kernel(GradPtrs g, const uint8_t* __restrict__ mask, int K, int64_t R,
                                                       int D, float* __restrict__ out, uint8_t* __restrict__ cov,
                                                       AdamArgs ad) {
    const int segs = (D + 511) / 512; // wave-segments per row
    const int64_t nitems = R * segs;
    const int lane = threadIdx.x & 63;
    const int64_t wave0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    double sq = 0.0; // OPT_SQNORM: this lane's share of the sum of squares
    float gs = ad.grad_scale;
    if (OPT == OPT_ADAMW && ad.grad_scale_dev) gs *= *ad.grad_scale_dev;
    // mask bytes of the first kBatch workers for this wave's next item, requested one item ahead: the gradient
    // loads of an item then start at once instead of waiting for a dependent load of their own.  Worth 6 - 8 % for
    // the norm pass, which only reads; the forms that store are bound by their stores and keep the plain loads.
    constexpr bool kAhead = OPT == OPT_SQNORM;
    auto request_masks = [&](int64_t item, int (&mk)[kBatch]) {
        const int64_t rr = item / segs;
#pragma unroll
        for (int i = 0; i < kBatch; ++i) mk[i] = kAhead && item < nitems && i < K ? (int)mask[(int64_t)i * R + rr] : 0;
    };
    int mask_now[kBatch];
    request_masks(wave0, mask_now);
    for (int64_t item = wave0; item < nitems; item += nwaves) {
        int mask_next[kBatch];
        request_masks(item + nwaves, mask_next);
        const int64_t r = item / segs;
        const int seg = (int)(item - r * segs);
        const int e0 = seg * 512 + lane * 8;
        const bool live = e0 < D;
        const int64_t off = r * D + e0;
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        int c = 0;
        // optimizer state of the segment: requested first, so that it travels while the gradients are summed
        // (rows nobody covers are read too, which is harmless and rare, and never written back)
        f32x4 th[2], mm[2], vv[2];
        if (OPT == OPT_ADAMW && live) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                th[h] = *((const f32x4*)(ad.theta + off) + h);
                mm[h] = *((const f32x4*)(ad.m + off) + h);
                vv[h] = *((const f32x4*)(ad.v + off) + h);
            }
        }
        for (int k0 = 0; k0 < K; k0 += kBatch) {
            bool covered[kBatch];
            u32x4 lo[kBatch];
            f32x4 hi[kBatch];
#pragma unroll
            for (int i = 0; i < kBatch; ++i) {
                covered[i] = false;
                if (kAhead && k0 == 0)
                    covered[i] = __builtin_amdgcn_readfirstlane(mask_now[i]) != 0;
                else if (k0 + i < K)
                    covered[i] = __builtin_amdgcn_readfirstlane((int)mask[(int64_t)(k0 + i) * R + r]) != 0;
                if (covered[i] && live) {
                    if (BF16) {
                        lo[i] = __builtin_nontemporal_load((const u32x4*)((const uint16_t*)g.p[k0 + i] + off));
                    } else {
                        const u32x4* src = (const u32x4*)((const float*)g.p[k0 + i] + off);
                        lo[i] = __builtin_nontemporal_load(src);
                        hi[i] = __builtin_nontemporal_load((const f32x4*)(src + 1));
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < kBatch; ++i) {
                if (!covered[i]) continue;
                ++c;
                if (!live) continue;
                if (BF16) {
                    add_bf16x8(lo[i], acc);
                } else {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        acc[q] += __uint_as_float(lo[i][q]);
                        acc[4 + q] += hi[i][q];
                    }
                }
            }
        }
        if (live && OPT == OPT_SQNORM && c > 0) {
            // squares of the very fp32 values the storing form would write, added up in double
            const float denom = (float)c;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const double a = (double)(acc[i] / denom);
                sq += a * a;
            }
        }
        if (live && OPT == OPT_STORE) {
            // c == 0: nobody covers the row, the average is defined as 0 (acc is still 0)
            const float denom = c > 0 ? (float)c : 1.0f;
            f32x4 a, b;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                a[i] = acc[i] / denom;
                b[i] = acc[4 + i] / denom;
            }
            f32x4* dst = (f32x4*)(out + off);
            __builtin_nontemporal_store(a, dst);
            __builtin_nontemporal_store(b, dst + 1);
        }
        if (live && OPT == OPT_ADAMW && c > 0) {
            // rows nobody covers keep their parameters and moments
            const float denom = (float)c;
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float t = th[h][i], m1 = mm[h][i], v1 = vv[h][i];
                    adamw_one(ad, gs, acc[4 * h + i] / denom, t, m1, v1);
                    th[h][i] = t, mm[h][i] = m1, vv[h][i] = v1;
                }
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                *((f32x4*)(ad.theta + off) + h) = th[h];
                *((f32x4*)(ad.m + off) + h) = mm[h];
                *((f32x4*)(ad.v + off) + h) = vv[h];
            }
            if (ad.theta_bf16) {
                const u32x4 packed = {pack2_bf16(th[0][0], th[0][1]), pack2_bf16(th[0][2], th[0][3]),
                                      pack2_bf16(th[1][0], th[1][1]), pack2_bf16(th[1][2], th[1][3])};
                __builtin_nontemporal_store(packed, (u32x4*)(ad.theta_bf16 + off));
            }
        }
        if (cov && seg == 0 && lane == 0) cov[r] = (uint8_t)c;
#pragma unroll
        for (int i = 0; i < kBatch; ++i) mask_now[i] = mask_next[i];
    }
    if (OPT == OPT_SQNORM) {
        sq = block_sum(sq);
        if (threadIdx.x == 0) ad.partial[blockIdx.x] = sq;
    }
}

// Any D: one thread per parameter.
template <int BF16, int OPT>
__global__ __launch_bounds__(256) void avg_elems_kernel(GradPtrs g, const uint8_t* __restrict__ mask, int K, int64_t R,
                                                        int D, float* __restrict__ out, uint8_t* __restrict__ cov,
                                                        AdamArgs ad) {
    const int64_t n = R * D;
    double sq = 0.0;
    float gs = ad.grad_scale;
    if (OPT == OPT_ADAMW && ad.grad_scale_dev) gs *= *ad.grad_scale_dev;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = i / D;
        float acc = 0.f;
        int c = 0;
        for (int k = 0; k < K; ++k) {
            if (mask[(int64_t)k * R + r] == 0) continue;
            ++c;
            if (BF16)
                acc += __uint_as_float((uint32_t)((const uint16_t*)g.p[k])[i] << 16);
            else
                acc += ((const float*)g.p[k])[i];
        }
        if (OPT == OPT_STORE) {
            out[i] = acc / (c > 0 ? (float)c : 1.0f);
        } else if (OPT == OPT_SQNORM) {
            if (c > 0) {
                const double a = (double)(acc / (float)c);
                sq += a * a;
            }
        } else if (c > 0) {
            float t = ad.theta[i], m1 = ad.m[i], v1 = ad.v[i];
            adamw_one(ad, gs, acc / (float)c, t, m1, v1);
            ad.theta[i] = t, ad.m[i] = m1, ad.v[i] = v1;
            if (ad.theta_bf16) ad.theta_bf16[i] = (uint16_t)(pack2_bf16(t, 0.f) & 0xFFFFu);
        }
        if (cov && i == r * D) cov[r] = (uint8_t)c;
    }
    if (OPT == OPT_SQNORM) {
        sq = block_sum(sq);
        if (threadIdx.x == 0) ad.partial[blockIdx.x] = sq;
    }
}

// workgroups of the norm pass: enough to keep every CU's queue full, few enough for a small table of partial sums
constexpr int64_t kNormBlocks = 1 << 13;
int64_t norm_blocks(int64_t R, int D) {
    const int64_t want = D % 8 == 0 ? (R * ((D + 511) / 512) + 3) / 4 : (R * D + 255) / 256;
    return want < 1 ? 1 : (want < kNormBlocks ? want : kNormBlocks);
}

// argument checks and launch shared by the two entry points; ad == nullptr: store the average into out
int launch_average(int K, int64_t R, int D, int gdtype, const void* const* g, const uint8_t* mask, float* out,
                   uint8_t* cov, const AdamArgs* ad, const char* name, hipStream_t s, bool norm = false) {
    GradPtrs ptrs;
    for (int k = 0; k < K; ++k) {
        if (!g[k] || !sdp::aligned16(g[k])) return SDP_ERR_INVALID_ARG;
        ptrs.p[k] = g[k];
    }
    for (int k = K; k < SDP_MAX_WORKERS; ++k) ptrs.p[k] = nullptr;
    const AdamArgs a = ad ? *ad : AdamArgs{};
    sdp::ProfileScope ps(name, s);
    if (D % 8 == 0) {
        const int segs = (D + 511) / 512;
        const int64_t items = R * segs;
        const int64_t blocks64 = (items + 3) / 4; // 4 waves per workgroup
        const unsigned blocks = norm ? (unsigned)norm_blocks(R, D) : (unsigned)(blocks64 < (1 << 20) ? blocks64 : (1 << 20));
        if (norm) {
            if (gdtype == SDP_BF16) avg_rows_kernel<1, OPT_SQNORM><<<blocks, 256, 0, s>>>(ptrs, mask, K, R, D, out, cov, a);
            else avg_rows_kernel<0, OPT_SQNORM><<<blocks, 256, 0, s>>>(ptrs, mask, K, R, D, out, cov, a);
        } else if (gdtype == SDP_BF16) {
            if (ad) avg_rows_kernel<1, 1><<<blocks, 256, 0, s>>>(ptrs, mask, K, R, D, out, cov, a);
            else avg_rows_kernel<1, 0><<<blocks, 256, 0, s>>>(ptrs, mask, K, R, D, out, cov, a);
        } else {
            if (ad) avg_rows_kernel<0, 1><<<blocks, 256, 0, s>>>(ptrs, mask, K, R, D, out, cov, a);
            else avg_rows_kernel<0, 0><<<blocks, 256, 0, s>>>(ptrs, mask, K, R, D, out, cov, a);
        }
    } else {
        const int64_t n = R * D;
        const int64_t blocks64 = (n + 255) / 256;
        const unsigned blocks = norm ? (unsigned)norm_blocks(R, D) : (unsigned)(blocks64 < (1 << 20) ? blocks64 : (1 << 20));
        if (norm) {
            if (gdtype == SDP_BF16) avg_elems_kernel<1, OPT_SQNORM><<<blocks, 256, 0, s>>>(ptrs, mask, K, R, D, out, cov, a);
            else avg_elems_kernel<0, OPT_SQNORM><<<blocks, 256, 0, s>>>(ptrs, mask, K, R, D, out, cov, a);
        } else if (gdtype == SDP_BF16) {
            if (ad) avg_elems_kernel<1, 1><<<blocks, 256, 0, s>>>(ptrs, mask, K, R, D, out, cov, a);
            else avg_elems_kernel<1, 0><<<blocks, 256, 0, s>>>(ptrs, mask, K, R, D, out, cov, a);
        } else {
            if (ad) avg_elems_kernel<0, 1><<<blocks, 256, 0, s>>>(ptrs, mask, K, R, D, out, cov, a);
            else avg_elems_kernel<0, 0><<<blocks, 256, 0, s>>>(ptrs, mask, K, R, D, out, cov, a);
        }
    }
    return sdp::launch_status();
}

} // namespace

extern "C" int sdp_coverage_grad_avg(int K, int64_t R, int D, int gdtype, const void* const* g, const uint8_t* mask,
                                     float* out, uint8_t* cov, void* stream) {
    if (K < 1 || K > SDP_MAX_WORKERS || R < 0 || D < 1) return SDP_ERR_INVALID_ARG;
    if (gdtype != SDP_F32 && gdtype != SDP_BF16) return SDP_ERR_INVALID_ARG;
    if (!g) return SDP_ERR_INVALID_ARG;
    if (R == 0) return SDP_OK; // nothing to average: empty buffers may legitimately be null
    if (!mask || !out) return SDP_ERR_INVALID_ARG;
    if (R > ((int64_t)1 << 40) / D) return SDP_ERR_SHAPE;
    if (!sdp::aligned16(out)) return SDP_ERR_INVALID_ARG;
    return launch_average(K, R, D, gdtype, g, mask, out, cov, nullptr, "coverage_grad_avg", (hipStream_t)stream);
}

extern "C" int sdp_coverage_avg_adamw(int K, int64_t R, int D, int gdtype, const void* const* g, const uint8_t* mask,
                                      float* theta, float* m, float* v, void* theta_bf16, uint8_t* cov,
                                      const sdp_adamw_params* hp, void* stream) {
    if (K < 1 || K > SDP_MAX_WORKERS || R < 0 || D < 1) return SDP_ERR_INVALID_ARG;
    if (gdtype != SDP_F32 && gdtype != SDP_BF16) return SDP_ERR_INVALID_ARG;
    if (!g || !hp) return SDP_ERR_INVALID_ARG;
    if (!(hp->lr >= 0.f) || !(hp->beta1 >= 0.f && hp->beta1 < 1.f) || !(hp->beta2 >= 0.f && hp->beta2 < 1.f) ||
        !(hp->eps > 0.f) || !(hp->weight_decay >= 0.f) || hp->step < 1 || !std::isfinite(hp->grad_scale))
        return SDP_ERR_INVALID_ARG;
    if (R == 0) return SDP_OK;
    if (!mask || !theta || !m || !v) return SDP_ERR_INVALID_ARG;
    if (R > ((int64_t)1 << 40) / D) return SDP_ERR_SHAPE;
    for (const void* q : {(const void*)theta, (const void*)m, (const void*)v, (const void*)theta_bf16})
        if (q && !sdp::aligned16(q)) return SDP_ERR_INVALID_ARG;
    if ((uintptr_t)hp->grad_scale_dev & 3) return SDP_ERR_INVALID_ARG;
    AdamArgs a;
    a.theta = theta, a.m = m, a.v = v, a.theta_bf16 = (uint16_t*)theta_bf16;
    a.decay = 1.0f - hp->lr * hp->weight_decay;
    a.beta1 = hp->beta1, a.beta2 = hp->beta2, a.eps = hp->eps, a.grad_scale = hp->grad_scale;
    a.grad_scale_dev = hp->grad_scale_dev, a.partial = nullptr;
    // bias corrections in double on the host (beta^t loses digits in fp32 for large t)
    a.step_size = (float)((double)hp->lr / (1.0 - std::pow((double)hp->beta1, (double)hp->step)));
    a.inv_sqrt_bc2 = (float)(1.0 / std::sqrt(1.0 - std::pow((double)hp->beta2, (double)hp->step)));
    return launch_average(K, R, D, gdtype, g, mask, nullptr, cov, &a, "coverage_avg_adamw", (hipStream_t)stream);
}

extern "C" size_t sdp_coverage_grad_sqnorm_workspace_bytes(int64_t R, int D) {
    if (R < 0 || D < 1) return 0;
    return sdp::round_up((size_t)norm_blocks(R, D) * sizeof(double), 256);
}

extern "C" int sdp_coverage_grad_sqnorm(int K, int64_t R, int D, int gdtype, const void* const* g, const uint8_t* mask,
                                        double* sqnorm, void* ws, size_t ws_bytes, void* stream) {
    if (K < 1 || K > SDP_MAX_WORKERS || R < 0 || D < 1) return SDP_ERR_INVALID_ARG;
    if (gdtype != SDP_F32 && gdtype != SDP_BF16) return SDP_ERR_INVALID_ARG;
    if (!g || !sqnorm || ((uintptr_t)sqnorm & 7)) return SDP_ERR_INVALID_ARG;
    if (R > 0 && !mask) return SDP_ERR_INVALID_ARG;
    if (R > 0 && R > ((int64_t)1 << 40) / D) return SDP_ERR_SHAPE;
    if (!ws || !sdp::aligned16(ws) || ws_bytes < sdp_coverage_grad_sqnorm_workspace_bytes(R, D)) return SDP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    AdamArgs a{};
    a.partial = (double*)ws;
    if (R == 0) { // nothing to add (empty buffers may legitimately be null): the norm is 0
        sqnorm_finish_kernel<<<1, 256, 0, s>>>((const double*)ws, 0, sqnorm);
        return sdp::launch_status();
    }
    sdp::ProfileScope ps("coverage_grad_sqnorm", s); // both kernels
    int rc = launch_average(K, R, D, gdtype, g, mask, nullptr, nullptr, &a, nullptr, s, true);
    if (rc != SDP_OK) return rc;
    sqnorm_finish_kernel<<<1, 256, 0, s>>>((const double*)ws, (int)norm_blocks(R, D), sqnorm);
    return sdp::launch_status();
}

extern "C" int sdp_clip_scale(int n, const double* sqnorm, float max_norm, float* scale, void* stream) {
    if (n < 1 || n > (1 << 20) || !sqnorm || !scale || !(max_norm > 0.f) || !std::isfinite(max_norm)) return SDP_ERR_INVALID_ARG;
    if (((uintptr_t)sqnorm & 7) || ((uintptr_t)scale & 3)) return SDP_ERR_INVALID_ARG;
    clip_scale_kernel<<<1, 64, 0, (hipStream_t)stream>>>(sqnorm, n, (double)max_norm, scale);
    return sdp::launch_status();
}
