// Measurement aid: the rate at which the matrix cores of this GPU sustain v_mfma_f32_32x32x16_bf16
// on given operand values, with no memory traffic inside the loop.  The chip's clock under MFMA load
// depends on how many bits toggle, so the sustained rate for random operands is well below the
// rate for constant ones; bench.py reports both next to the published peak.
#include "sdp_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 512;       // 8 waves: two per SIMD
constexpr int kFragsPerLane = 6;    // 4 "A" and 2 "B" fragments, as in the 256 x 256 contraction tile
constexpr int kMfmaPerIter = 32;

__global__ __launch_bounds__(kThreads, 1) void mfma_rate_kernel(const bf16x8* __restrict__ operands, int iters,
                                                                float* __restrict__ sink) {
    bf16x8 fa[4], fb[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) fa[i] = operands[(size_t)i * kThreads + threadIdx.x];
#pragma unroll
    for (int j = 0; j < 2; ++j) fb[j] = operands[(size_t)(4 + j) * kThreads + threadIdx.x];
    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < kMfmaPerIter / 8; ++s)
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) sum += acc[i][j][e];
    sink[(size_t)blockIdx.x * kThreads + threadIdx.x] = sum;
}

} // namespace

extern "C" size_t sdp_probe_mfma_operand_bytes(void) { return (size_t)kFragsPerLane * kThreads * 16; }
extern "C" size_t sdp_probe_mfma_sink_bytes(int blocks) { return blocks > 0 ? (size_t)blocks * kThreads * 4 : 0; }

extern "C" int sdp_probe_mfma_tflops(const void* operands, int blocks, int iters, void* sink, double* tflops,
                                     void* stream) {
    if (!operands || !sink || !tflops || blocks < 1 || iters < 1 || !sdp::aligned16(operands)) return SDP_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return SDP_ERR_HIP;
    if (hipEventCreate(&e1) != hipSuccess) {
        hipEventDestroy(e0);
        return SDP_ERR_HIP;
    }
    int rc = SDP_OK;
    float ms = 0.f;
    // one untimed launch (clock ramp, code upload), then the timed one
    mfma_rate_kernel<<<blocks, kThreads, 0, s>>>((const bf16x8*)operands, iters, (float*)sink);
    if (hipEventRecord(e0, s) != hipSuccess) rc = SDP_ERR_HIP;
    mfma_rate_kernel<<<blocks, kThreads, 0, s>>>((const bf16x8*)operands, iters, (float*)sink);
    if (hipEventRecord(e1, s) != hipSuccess) rc = SDP_ERR_HIP;
    if (hipEventSynchronize(e1) != hipSuccess || hipGetLastError() != hipSuccess) rc = SDP_ERR_HIP;
    if (rc == SDP_OK && hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = SDP_ERR_HIP;
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    if (rc != SDP_OK) return rc;
    const double flop = (double)blocks * (kThreads / 64) * (double)iters * kMfmaPerIter * 2.0 * 32 * 32 * 16;
    *tflops = flop / (ms * 1e-3) / 1e12;
    return SDP_OK;
}
