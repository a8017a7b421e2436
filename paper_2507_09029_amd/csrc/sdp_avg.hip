// Coverage-normalised gradient average (the paper's Sec. 3.1, eq. "average", with the load taken
// per coordinate): one streaming pass over the K workers' gradient buffers.
//
// HBM-bound.  Per neuron row of D parameters the kernel reads only the rows of workers whose mask
// covers it (16-byte loads, non-temporal), sums them in fp32 in worker order, divides by the
// coverage count and writes fp32 (non-temporal stores).  No atomics: the result is a pure function
// of the inputs.
#include "sdp_internal.h"

namespace {

struct GradPtrs {
    const void* p[SDP_MAX_WORKERS];
};

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

template <int BF16>
__global__ __launch_bounds__(256) void avg_rows_kernel(GradPtrs g, const uint8_t* __restrict__ mask, int K, int64_t R,
                                                       int D, float* __restrict__ out, uint8_t* __restrict__ cov) {
    const int segs = (D + 511) / 512; // wave-segments per row
    const int64_t nitems = R * segs;
    const int lane = threadIdx.x & 63;
    const int64_t wave0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t item = wave0; item < nitems; item += nwaves) {
        const int64_t r = item / segs;
        const int seg = (int)(item - r * segs);
        const int e0 = seg * 512 + lane * 8;
        const bool live = e0 < D;
        const int64_t off = r * D + e0;
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        int c = 0;
        for (int k0 = 0; k0 < K; k0 += kBatch) {
            bool covered[kBatch];
            u32x4 lo[kBatch];
            f32x4 hi[kBatch];
#pragma unroll
            for (int i = 0; i < kBatch; ++i) {
                covered[i] = false;
                if (k0 + i < K) covered[i] = __builtin_amdgcn_readfirstlane((int)mask[(int64_t)(k0 + i) * R + r]) != 0;
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
        if (live) {
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
        if (cov && seg == 0 && lane == 0) cov[r] = (uint8_t)c;
    }
}

// Any D: one thread per parameter.
template <int BF16>
__global__ __launch_bounds__(256) void avg_elems_kernel(GradPtrs g, const uint8_t* __restrict__ mask, int K, int64_t R,
                                                        int D, float* __restrict__ out, uint8_t* __restrict__ cov) {
    const int64_t n = R * D;
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
        out[i] = acc / (c > 0 ? (float)c : 1.0f);
        if (cov && i == r * D) cov[r] = (uint8_t)c;
    }
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
    GradPtrs ptrs;
    for (int k = 0; k < K; ++k) {
        if (!g[k] || !sdp::aligned16(g[k])) return SDP_ERR_INVALID_ARG;
        ptrs.p[k] = g[k];
    }
    for (int k = K; k < SDP_MAX_WORKERS; ++k) ptrs.p[k] = nullptr;
    if (!sdp::aligned16(out)) return SDP_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    sdp::ProfileScope ps("coverage_grad_avg", s);
    if (D % 8 == 0) {
        const int segs = (D + 511) / 512;
        const int64_t items = R * segs;
        const int64_t blocks64 = (items + 3) / 4; // 4 waves per workgroup
        const unsigned blocks = (unsigned)(blocks64 < (1 << 20) ? blocks64 : (1 << 20));
        if (gdtype == SDP_BF16)
            avg_rows_kernel<1><<<blocks, 256, 0, s>>>(ptrs, mask, K, R, D, out, cov);
        else
            avg_rows_kernel<0><<<blocks, 256, 0, s>>>(ptrs, mask, K, R, D, out, cov);
    } else {
        const int64_t n = R * D;
        const int64_t blocks64 = (n + 255) / 256;
        const unsigned blocks = (unsigned)(blocks64 < (1 << 20) ? blocks64 : (1 << 20));
        if (gdtype == SDP_BF16)
            avg_elems_kernel<1><<<blocks, 256, 0, s>>>(ptrs, mask, K, R, D, out, cov);
        else
            avg_elems_kernel<0><<<blocks, 256, 0, s>>>(ptrs, mask, K, R, D, out, cov);
    }
    return sdp::launch_status();
}
