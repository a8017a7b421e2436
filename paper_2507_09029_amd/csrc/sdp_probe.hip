// Measurement aids.  (1) The rate at which the matrix cores of this GPU sustain a bf16 MFMA instruction on given
// operand values, with no memory traffic inside the loop.  The chip's clock under MFMA load depends on how
// many bits toggle, so the sustained rate for random operands is well below the rate for constant ones, and it
// differs between the instruction shapes: v_mfma_f32_16x16x32_bf16 (the one the contractions use) sustains more
// than v_mfma_f32_32x32x16_bf16 for the same flops.  bench.py reports these next to the published peak.
// (2) The rate at which plain streaming kernels move data through HBM: read-only, and a copy (half reads, half
// writes), with the 16-byte non-temporal accesses the average kernels use.
#include "sdp_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 512;       // 8 waves: two per SIMD
constexpr int kFragsPerLane = 6;    // 4 "A" and 2 "B" fragment registers
constexpr double kFlopPerIter = 32 * 2.0 * 32 * 32 * 16; // per wave: 32 MFMAs of 32x32x16, or 64 of 16x16x32

// SHAPE 16: 16x16x32 (64 instructions per iteration on 32 accumulator tiles); 32: 32x32x16 (32 on 8 tiles)
template <int SHAPE>
__global__ __launch_bounds__(kThreads, 1) void mfma_rate_kernel(const bf16x8* __restrict__ operands, int iters,
                                                                float* __restrict__ sink) {
    bf16x8 fa[4], fb[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) fa[i] = operands[(size_t)i * kThreads + threadIdx.x];
#pragma unroll
    for (int j = 0; j < 2; ++j) fb[j] = operands[(size_t)(4 + j) * kThreads + threadIdx.x];
    float sum = 0.f;
    if constexpr (SHAPE == 32) {
        f32x16 acc[4][2];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) sum += acc[i][j][e];
    } else {
        f32x4 acc[4][2][4]; // the same 128 accumulator registers as 16 x 16 tiles
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[i][j][q] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            acc[i][j][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fa[(i + q) & 3], acc[i][j][q], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) sum += acc[i][j][q][0] + acc[i][j][q][1] + acc[i][j][q][2] + acc[i][j][q][3];
    }
    sink[(size_t)blockIdx.x * kThreads + threadIdx.x] = sum;
}

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int kStreamUnroll = 4;

// every workgroup walks chunks of 256 x kStreamUnroll vectors of 16 bytes, grid-stride; COPY: also writes them to dst
template <bool COPY>
__global__ __launch_bounds__(256) void hbm_stream_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n,
                                                         unsigned* __restrict__ flag) {
    u32x4 seen = {0, 0, 0, 0};
    const size_t chunk = (size_t)256 * kStreamUnroll;
    for (size_t base = (size_t)blockIdx.x * chunk; base + chunk <= n; base += (size_t)gridDim.x * chunk) {
        u32x4 v[kStreamUnroll];
#pragma unroll
        for (int u = 0; u < kStreamUnroll; ++u) v[u] = __builtin_nontemporal_load(src + base + (size_t)u * 256 + threadIdx.x);
#pragma unroll
        for (int u = 0; u < kStreamUnroll; ++u) {
            if (COPY) __builtin_nontemporal_store(v[u], dst + base + (size_t)u * 256 + threadIdx.x);
            else seen ^= v[u];
        }
    }
    // keeps the loads of the read-only form alive; the comparison is false for almost any data
    if (!COPY && (seen[0] ^ seen[1] ^ seen[2] ^ seen[3]) == 0x9E3779B9u) *flag = 1;
}

} // namespace

extern "C" int sdp_probe_hbm_gbs(int copy, const void* src, void* dst, size_t bytes, int launches, double* gbs,
                                 void* stream) {
    if (!src || !dst || !gbs || launches < 1 || !sdp::aligned16(src) || !sdp::aligned16(dst)) return SDP_ERR_INVALID_ARG;
    const size_t chunk_bytes = (size_t)256 * kStreamUnroll * 16;
    const size_t n = bytes / chunk_bytes * (chunk_bytes / 16); // whole chunks only
    if (n == 0) return SDP_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return SDP_ERR_HIP;
    if (hipEventCreate(&e1) != hipSuccess) {
        hipEventDestroy(e0);
        return SDP_ERR_HIP;
    }
    const size_t chunks = n / ((size_t)256 * kStreamUnroll);
    const unsigned grid = (unsigned)(chunks < 32768 ? chunks : 32768);
    auto go = [&]() {
        if (copy) hbm_stream_kernel<true><<<grid, 256, 0, s>>>((const u32x4*)src, (u32x4*)dst, n, nullptr);
        else hbm_stream_kernel<false><<<grid, 256, 0, s>>>((const u32x4*)src, nullptr, n, (unsigned*)dst);
    };
    int rc = SDP_OK;
    float ms = 0.f;
    go(); // untimed: clock ramp, code upload
    if (hipEventRecord(e0, s) != hipSuccess) rc = SDP_ERR_HIP;
    for (int i = 0; i < launches; ++i) go();
    if (hipEventRecord(e1, s) != hipSuccess) rc = SDP_ERR_HIP;
    if (hipEventSynchronize(e1) != hipSuccess || hipGetLastError() != hipSuccess) rc = SDP_ERR_HIP;
    if (rc == SDP_OK && hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = SDP_ERR_HIP;
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    if (rc != SDP_OK) return rc;
    const double moved = (double)n * 16 * (copy ? 2 : 1) * launches;
    *gbs = moved / (ms * 1e-3) / 1e9;
    return SDP_OK;
}

extern "C" size_t sdp_probe_mfma_operand_bytes(void) { return (size_t)kFragsPerLane * kThreads * 16; }
extern "C" size_t sdp_probe_mfma_sink_bytes(int blocks) { return blocks > 0 ? (size_t)blocks * kThreads * 4 : 0; }

extern "C" int sdp_probe_mfma_shape_tflops(int shape, const void* operands, int blocks, int iters, void* sink,
                                           double* tflops, void* stream) {
    if (shape != 16 && shape != 32) return SDP_ERR_INVALID_ARG;
    if (!operands || !sink || !tflops || blocks < 1 || iters < 1 || !sdp::aligned16(operands)) return SDP_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return SDP_ERR_HIP;
    if (hipEventCreate(&e1) != hipSuccess) {
        hipEventDestroy(e0);
        return SDP_ERR_HIP;
    }
    auto go = [&]() {
        if (shape == 16)
            mfma_rate_kernel<16><<<blocks, kThreads, 0, s>>>((const bf16x8*)operands, iters, (float*)sink);
        else
            mfma_rate_kernel<32><<<blocks, kThreads, 0, s>>>((const bf16x8*)operands, iters, (float*)sink);
    };
    int rc = SDP_OK;
    float ms = 0.f;
    // one untimed launch (clock ramp, code upload), then the timed one
    go();
    if (hipEventRecord(e0, s) != hipSuccess) rc = SDP_ERR_HIP;
    go();
    if (hipEventRecord(e1, s) != hipSuccess) rc = SDP_ERR_HIP;
    if (hipEventSynchronize(e1) != hipSuccess || hipGetLastError() != hipSuccess) rc = SDP_ERR_HIP;
    if (rc == SDP_OK && hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = SDP_ERR_HIP;
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    if (rc != SDP_OK) return rc;
    *tflops = (double)blocks * (kThreads / 64) * (double)iters * kFlopPerIter / (ms * 1e-3) / 1e12;
    return SDP_OK;
}

extern "C" int sdp_probe_mfma_tflops(const void* operands, int blocks, int iters, void* sink, double* tflops,
                                     void* stream) {
    return sdp_probe_mfma_shape_tflops(16, operands, blocks, iters, sink, tflops, stream);
}
