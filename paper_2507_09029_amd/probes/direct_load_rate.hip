// Probe: rate at which a CU streams operand tiles from L2 into LDS with direct loads
// (global_load_lds_dwordx4), in the access pattern of the contractions: one wave instruction fetches
// 8 rows x 128 bytes.  Workgroup (xcd, idx) reads rows of an "A" block private to (xcd, idx % 8) and
// of a "B" block chosen by idx / 8, as 32 tiles of one XCD would.  Varied: row stride, number of
// waves that issue the loads, and how many steps of loads a wave keeps in flight.
// Every case is checked on the host against the size of the source buffer before it is launched.
//   hipcc --offload-arch=gfx950 -O3 direct_load_rate.hip -o direct_load_rate && ./direct_load_rate
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>

#define CK(x)                                                                     \
    do {                                                                          \
        hipError_t e_ = (x);                                                      \
        if (e_ != hipSuccess) {                                                   \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            return 1;                                                             \
        }                                                                         \
    } while (0)

typedef __attribute__((address_space(3))) void* lds_ptr;
typedef __attribute__((address_space(1))) const void* glb_ptr;

// rows = rows per workgroup and step (half "A", half "B"), each step moves 128 bytes along every row.
// LDS use: 2 x rows x 128 bytes.
template <int DEPTH>
__global__ __launch_bounds__(512) void stream_kernel(const unsigned char* src, int64_t row_stride, int rows, int ksteps,
                                                     uint32_t* out, unsigned long long* cycles) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nwaves = blockDim.x >> 6;
    const int half = rows / 2, slabs = rows / 8, per_wave = slabs / nwaves;
    const int xcd = blockIdx.x % 8, idx = blockIdx.x / 8;
    const int64_t a_row0 = (int64_t)(xcd * 8 + idx % 8) * half;
    const int64_t b_row0 = (int64_t)(64 + idx / 8) * half;
    const unsigned long long c0 = __builtin_readcyclecounter();
    for (int ks = 0; ks < ksteps; ++ks) {
        for (int i = 0; i < per_wave; ++i) {
            const int slab = wave + nwaves * i;
            const int r = slab * 8 + (lane >> 3);
            const int64_t row = r < half ? a_row0 + r : b_row0 + (r - half);
            const unsigned char* p = src + row * row_stride + (int64_t)ks * 128 + (lane & 7) * 16;
            unsigned char* dst = smem + ((ks & 1) * slabs + slab) * 1024;
            __builtin_amdgcn_global_load_lds((glb_ptr)p, (lds_ptr)dst, 16, 0, 0);
        }
        // s_waitcnt vmcnt(n): how many of this wave's loads may stay in flight
        if (DEPTH == 0) __builtin_amdgcn_s_waitcnt(0x0F70);
        if (DEPTH == 1) __builtin_amdgcn_s_waitcnt(0x0F70 | 8);
        if (DEPTH == 2) __builtin_amdgcn_s_waitcnt(0x0F70 | 15);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
    const unsigned long long c1 = __builtin_readcyclecounter();
    __syncthreads();
    out[blockIdx.x * blockDim.x + threadIdx.x] = *(const uint32_t*)(smem + threadIdx.x * 4);
    if (threadIdx.x == 0) cycles[blockIdx.x] = c1 - c0;
}

struct Case {
    const char* name;
    int64_t stride;
    int rows, ksteps, blocks, threads;
};

int main() {
    const size_t bytes = (size_t)1 << 30;
    unsigned char* src;
    uint32_t* out;
    unsigned long long* cycles;
    CK(hipMalloc(&src, bytes));
    CK(hipMalloc(&out, 256 * 512 * 4));
    CK(hipMalloc(&cycles, 256 * 8));
    CK(hipMemset(src, 1, bytes));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    const Case cases[] = {
        {"256+256 rows, stride 3072 B, 24 steps, 8 waves", 3072, 512, 24, 256, 512},
        {"256+256 rows, stride 3072 B, 24 steps, 4 waves", 3072, 512, 24, 256, 256},
        {"256+256 rows, stride 3072 B, 24 steps, 2 waves", 3072, 512, 24, 256, 128},
        {"256+256 rows, stride 16512 B, 128 steps, 8 waves", 16512, 512, 128, 256, 512},
        {"256+256 rows, stride 16512 B, 128 steps, 4 waves", 16512, 512, 128, 256, 256},
        {"256+192 rows, stride 16512 B, 128 steps, 8 waves, 192 workgroups", 16512, 448, 128, 192, 512},
    };
    for (const Case& c : cases) {
        // highest row touched: block 64 + 31 of `half` rows; last byte read: row * stride + ksteps * 128
        const int64_t max_row = (int64_t)(64 + 32) * (c.rows / 2);
        if (max_row * c.stride + (int64_t)c.ksteps * 128 > (int64_t)bytes || c.blocks > 256 || c.rows % 16 ||
            (c.rows / 8) % (c.threads / 64) || 2 * c.rows * 128 > 160 * 1024) {
            printf("skipped (does not fit): %s\n", c.name);
            continue;
        }
        for (int depth = 0; depth < 3; ++depth) {
            float ms = 0;
            const size_t lds = (size_t)2 * c.rows * 128;
            for (int rep = 0; rep < 3; ++rep) {
                CK(hipEventRecord(e0));
                if (depth == 0) stream_kernel<0><<<c.blocks, c.threads, lds>>>(src, c.stride, c.rows, c.ksteps, out, cycles);
                if (depth == 1) stream_kernel<1><<<c.blocks, c.threads, lds>>>(src, c.stride, c.rows, c.ksteps, out, cycles);
                if (depth == 2) stream_kernel<2><<<c.blocks, c.threads, lds>>>(src, c.stride, c.rows, c.ksteps, out, cycles);
                CK(hipEventRecord(e1));
                CK(hipEventSynchronize(e1));
                CK(hipGetLastError());
                CK(hipEventElapsedTime(&ms, e0, e1));
            }
            unsigned long long h[256];
            CK(hipMemcpy(h, cycles, c.blocks * 8, hipMemcpyDeviceToHost));
            double cyc = 0;
            for (int i = 0; i < c.blocks; ++i) cyc += (double)h[i] / c.blocks;
            const double per_wg = (double)c.rows * 128 * c.ksteps;
            printf("%-70s in flight %s: %5.1f B/clk/CU  %6.2f TB/s in total\n", c.name,
                   depth == 0 ? "1 step " : (depth == 1 ? "2 steps" : "3 steps"), per_wg / cyc, per_wg * c.blocks / (ms * 1e-3) / 1e12);
        }
    }
    return 0;
}
