// Probe: rate at which the waves of a CU get data out of LDS, per read width and per number of waves.
// Every read is conflict-free (lane-contiguous).  All accesses stay inside the 64 KB the kernel allocates.
//   hipcc --offload-arch=gfx950 -O3 lds_read_rate.hip -o lds_read_rate && ./lds_read_rate
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

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kLdsBytes = 65536;

// NREAD independent reads of W bytes per lane and iteration, results kept in separate registers
template <int W, int NREAD>
__global__ __launch_bounds__(512) void read_kernel(uint32_t* out, unsigned long long* cycles, int iters) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    for (int i = threadIdx.x; i < kLdsBytes / 4; i += blockDim.x) ((uint32_t*)smem)[i] = i;
    __syncthreads();
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    uint32_t acc = 0;
    const unsigned long long c0 = __builtin_readcyclecounter();
    for (int it = 0; it < iters; ++it) {
        u32x4 v[NREAD];
#pragma unroll
        for (int r = 0; r < NREAD; ++r) {
            // 16 regions of 4 KB; inside a region 4 slots of 64 lanes x W bytes: offset < 65536 for W <= 16
            const int off = ((wave * NREAD + r + it) & 15) * 4096 + ((r + it) & 3) * (W * 64) + lane * W;
            if (W == 16) v[r] = *(const u32x4*)(smem + off);
            if (W == 8) {
                const u32x2 t = *(const u32x2*)(smem + off);
                v[r] = u32x4{t[0], t[1], 0, 0};
            }
            if (W == 4) v[r] = u32x4{*(const uint32_t*)(smem + off), 0, 0, 0};
        }
#pragma unroll
        for (int r = 0; r < NREAD; ++r) acc ^= v[r][0] ^ v[r][1] ^ v[r][2] ^ v[r][3];
    }
    const unsigned long long c1 = __builtin_readcyclecounter();
    out[blockIdx.x * blockDim.x + threadIdx.x] = acc;
    if (threadIdx.x == 0) cycles[blockIdx.x] = c1 - c0;
}

template <int W, int NREAD>
int run(int threads, uint32_t* out, unsigned long long* cycles) {
    const int iters = 4000, blocks = 256;
    for (int rep = 0; rep < 2; ++rep) {
        read_kernel<W, NREAD><<<blocks, threads, kLdsBytes>>>(out, cycles, iters);
        CK(hipDeviceSynchronize());
    }
    unsigned long long h[blocks];
    CK(hipMemcpy(h, cycles, sizeof(h), hipMemcpyDeviceToHost));
    double c = 0;
    for (int i = 0; i < blocks; ++i) c += (double)h[i] / blocks;
    printf("read width %2d B, %d waves per CU: %6.1f B/clk/CU, %5.1f cycles per wave instruction\n", W, threads / 64,
           (double)(threads / 64) * iters * NREAD * 64 * W / c, c / ((double)iters * NREAD));
    return 0;
}

int main() {
    uint32_t* out;
    unsigned long long* cycles;
    CK(hipMalloc(&out, 256 * 512 * 4));
    CK(hipMalloc(&cycles, 256 * 8));
    for (int threads : {512, 256, 64}) {
        if (run<16, 12>(threads, out, cycles)) return 1;
        if (run<8, 12>(threads, out, cycles)) return 1;
        if (run<4, 12>(threads, out, cycles)) return 1;
    }
    return 0;
}
