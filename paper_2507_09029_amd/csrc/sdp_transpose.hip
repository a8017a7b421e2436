// (Gathered) matrix transpose: out[c][r] = in[rows[r]][c].  HBM-bound helper of the masked MLP:
// it materialises a worker's compact weights in depth-contiguous orientation (W2T[S]^T, W1[S]^T,
// W3[S]^T, each [d][p]) and the token-contiguous copies X^T, dY^T [d][T] that the weight-gradient
// contractions read, so that every MFMA operand tile can be read from LDS with plain 16-byte reads.
//
// 64 x 64 element tiles through LDS (padded rows), 256 threads.  Reads are 64 consecutive
// elements of one (gathered) input row per 64 lanes, writes 64 consecutive elements of one output
// row.  Bytes moved: R*C element reads + R*C element writes, nothing else.
#include "sdp_internal.h"

namespace sdp {
namespace {

template <typename T>
__global__ __launch_bounds__(256) void transpose_rows_kernel(const T* __restrict__ in, int64_t ld_in,
                                                             const int32_t* __restrict__ rows, int R, int C,
                                                             T* __restrict__ out, int64_t ld_out) {
    __shared__ T tile[64][64 + 2];
    const int r0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6; // 4 rows of 64 per pass
#pragma unroll 4
    for (int i = ty; i < 64; i += 4) {
        const int r = r0 + i, c = c0 + tx;
        if (r < R && c < C) {
            const int64_t src = rows ? rows[r] : r;
            tile[i][tx] = in[src * ld_in + c];
        }
    }
    __syncthreads();
#pragma unroll 4
    for (int i = ty; i < 64; i += 4) {
        const int c = c0 + i, r = r0 + tx;
        if (r < R && c < C) out[(int64_t)c * ld_out + r] = tile[tx][i];
    }
}

} // namespace

int transpose_rows(int elem_bytes, const void* in, int64_t ld_in, const int32_t* rows, int R, int C, void* out,
                   int64_t ld_out, const char* name, hipStream_t s) {
    if (R < 1 || C < 1) return SDP_ERR_SHAPE;
    dim3 grid((R + 63) / 64, (C + 63) / 64);
    if (grid.y > 65535) return SDP_ERR_SHAPE;
    ProfileScope ps(name, s);
    if (elem_bytes == 2)
        transpose_rows_kernel<uint16_t><<<grid, 256, 0, s>>>((const uint16_t*)in, ld_in, rows, R, C, (uint16_t*)out, ld_out);
    else
        transpose_rows_kernel<uint32_t><<<grid, 256, 0, s>>>((const uint32_t*)in, ld_in, rows, R, C, (uint32_t*)out, ld_out);
    return launch_status();
}

} // namespace sdp
