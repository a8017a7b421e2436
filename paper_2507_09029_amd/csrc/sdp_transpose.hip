// (Gathered) matrix transpose: out[c][r] = in[rows[r]][c].  HBM-bound helper of the masked MLP:
// it materialises a worker's compact weights in depth-contiguous orientation (W2T[S]^T, W1[S]^T,
// W3[S]^T, each [d][p]) and the token-contiguous copies X^T, dY^T [d][T] that the weight-gradient
// contractions read, so that every MFMA operand tile can be read from LDS with plain 16-byte reads.
//
// 64 x 64 element tiles through LDS (padded rows), 256 threads.  Reads are 64 consecutive
// elements of one (gathered) input row per 64 lanes, writes 64 consecutive elements of one output
// row.  Bytes moved: R*C element reads + R*C element writes, nothing else.
#include "sdp_internal.h"

#include <algorithm>

namespace sdp {
namespace {

// 16-bit elements, 16-byte accesses on both sides.  Tile: 64 input rows x 64 columns.
// Requires C % 8 == 0, R % 8 == 0, ld_in % 8 == 0, ld_out % 8 == 0 and 16-byte aligned bases.
// Up to kMaxJobs independent transposes run as one launch (grid.z = job); workgroups beyond a job's
// own extent leave at once.
struct Jobs {
    TransposeJob j[kMaxTransposeJobs];
};

__global__ __launch_bounds__(256) void transpose_rows_vec_kernel(Jobs jobs) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    // select by comparisons: indexing a by-value kernel argument with a runtime index would go through scratch
    const int z = blockIdx.z;
    const TransposeJob& jb = z == 0 ? jobs.j[0] : (z == 1 ? jobs.j[1] : (z == 2 ? jobs.j[2] : jobs.j[3]));
    const int R = jb.R, C = jb.C;
    if ((int)blockIdx.x * 64 >= R || (int)blockIdx.y * 64 >= C) return;
    const uint16_t* __restrict__ in = (const uint16_t*)jb.in;
    uint16_t* __restrict__ out = (uint16_t*)jb.out;
    const int32_t* __restrict__ rows = jb.rows;
    const int64_t ld_in = jb.ld_in, ld_out = jb.ld_out;
    // tile[r][c], rows padded to 66 elements (33 words): a column walk hits 64 distinct banks
    __shared__ uint32_t tile[64 * 33];
    const int r0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
    const int t = threadIdx.x;
    // load: 64 rows x 8 chunks of 8 elements; thread -> rows t/8 and t/8 + 32, chunk t%8
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int r = (t >> 3) + 32 * h, cc = t & 7;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (r0 + r < R && c0 + cc * 8 < C) {
            const int64_t src = rows ? rows[r0 + r] : (r0 + r);
            v = *(const u32x4*)(in + src * ld_in + c0 + cc * 8);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) tile[r * 33 + cc * 4 + e] = v[e];
    }
    __syncthreads();
    // store: 64 output rows (columns c) x 8 chunks of 8 input rows; thread -> columns t/8 and t/8 + 32
    const uint16_t* th = (const uint16_t*)tile;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int c = (t >> 3) + 32 * h, rc = t & 7;
        if (c0 + c < C && r0 + rc * 8 < R) {
            uint32_t w[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t lo = th[(rc * 8 + 2 * e) * 66 + c], hi = th[(rc * 8 + 2 * e + 1) * 66 + c];
                w[e] = lo | (hi << 16);
            }
            *(u32x4*)(out + (int64_t)(c0 + c) * ld_out + r0 + rc * 8) = u32x4{w[0], w[1], w[2], w[3]};
        }
    }
}

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

static bool vec_ok(const TransposeJob& t) {
    return t.C % 8 == 0 && t.R % 8 == 0 && t.ld_in % 8 == 0 && t.ld_out % 8 == 0 && aligned16(t.in) && aligned16(t.out);
}

int transpose_rows(int elem_bytes, const void* in, int64_t ld_in, const int32_t* rows, int R, int C, void* out,
                   int64_t ld_out, const char* name, hipStream_t s) {
    if (R < 1 || C < 1) return SDP_ERR_SHAPE;
    dim3 grid((R + 63) / 64, (C + 63) / 64);
    if (grid.y > 65535) return SDP_ERR_SHAPE;
    ProfileScope ps(name, s);
    const TransposeJob t{in, out, ld_in, ld_out, rows, R, C};
    if (elem_bytes == 2 && vec_ok(t)) {
        Jobs jobs{};
        jobs.j[0] = t;
        transpose_rows_vec_kernel<<<grid, 256, 0, s>>>(jobs);
    } else if (elem_bytes == 2)
        transpose_rows_kernel<uint16_t><<<grid, 256, 0, s>>>((const uint16_t*)in, ld_in, rows, R, C, (uint16_t*)out, ld_out);
    else
        transpose_rows_kernel<uint32_t><<<grid, 256, 0, s>>>((const uint32_t*)in, ld_in, rows, R, C, (uint32_t*)out, ld_out);
    return launch_status();
}

int transpose_batch(int elem_bytes, const TransposeJob* t, int n, const char* name, hipStream_t s) {
    if (n < 1 || n > kMaxTransposeJobs) return SDP_ERR_INVALID_ARG;
    bool one_launch = elem_bytes == 2;
    unsigned gx = 0, gy = 0;
    for (int i = 0; i < n; ++i) {
        if (t[i].R < 1 || t[i].C < 1) return SDP_ERR_SHAPE;
        one_launch = one_launch && vec_ok(t[i]);
        gx = std::max(gx, (unsigned)((t[i].R + 63) / 64));
        gy = std::max(gy, (unsigned)((t[i].C + 63) / 64));
    }
    if (gy > 65535) return SDP_ERR_SHAPE;
    if (!one_launch) {
        for (int i = 0; i < n; ++i) {
            const int rc = transpose_rows(elem_bytes, t[i].in, t[i].ld_in, t[i].rows, t[i].R, t[i].C, t[i].out, t[i].ld_out, name, s);
            if (rc != SDP_OK) return rc;
        }
        return SDP_OK;
    }
    Jobs jobs{};
    for (int i = 0; i < n; ++i) jobs.j[i] = t[i];
    ProfileScope ps(name, s);
    transpose_rows_vec_kernel<<<dim3(gx, gy, (unsigned)n), 256, 0, s>>>(jobs);
    return launch_status();
}

} // namespace sdp
