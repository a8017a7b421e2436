// Plain causal attention core (forward, dQ, dK/dV) for the head-masked attention block: fp32 or bf16 storage,
// fp32 arithmetic throughout, any head width up to 128, no matrix instructions and no rounding of intermediate
// results.  It serves the fp32 path (parity to 1e-5) and the bf16 shapes the MFMA core does not take (head
// widths other than 64).  Same interface and the same saved statistics as the MFMA core: base-2 log-sum-exp of
// the scaled logits, delta = sum_h dO[t][h] O[t][h].
//
// One wave per (token, head, sequence).  The 64 lanes share out the other axis (keys for a query, queries for a
// key); every lane keeps a partial of the hd-wide result row, and the wave sums the partials with shuffles.
// Logits are recomputed in each sweep instead of being stored: nothing of size S x S exists.
#include "sdp_internal.h"
#include "sdp_swiglu.h"

#include <cmath>

namespace sdp {
namespace {

constexpr int MAXHD = 128; // widest head; kernels are instantiated for 64 and 128 accumulator registers per row

template <typename T>
__device__ inline float ldv(const T* p);
template <>
__device__ inline float ldv<float>(const float* p) { return *p; }
template <>
__device__ inline float ldv<uint16_t>(const uint16_t* p) { return bf16_to_f32(*p); }
template <typename T>
__device__ inline void stv(T* p, float v);
template <>
__device__ inline void stv<float>(float* p, float v) { *p = v; }
template <>
__device__ inline void stv<uint16_t>(uint16_t* p, float v) { *p = f32_to_bf16(v); }

__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

template <typename T>
struct PlainArgs {
    const T* qkv; // [T][ldq]: Q | K | V, head i at columns i * hd of each part
    int64_t ldq;
    const T* o;   // [T][ldo]
    T* o_out;
    const T* dO;
    int64_t ldo;
    float* lse;   // [Bt][n][S]
    float* delta; // [Bt][n][S]
    T* dqkv;
    int S, n, hd;
    float scale2; // log2(e) / sqrt(hd)
    float scale;  // 1 / sqrt(hd)
};

template <typename T>
__device__ inline float dot_rows(const T* a, const T* b, int hd) {
    float z = 0.f;
    for (int h = 0; h < hd; ++h) z = __builtin_fmaf(ldv(a + h), ldv(b + h), z);
    return z;
}

// forward: O[q] = sum_{k <= q} softmax(z[q][.])[k] V[k]; grid (S, n, Bt), 64 threads
template <typename T, int W>
__global__ __launch_bounds__(64) void attn_plain_fwd_kernel(PlainArgs<T> a) {
    const int q = blockIdx.x, head = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
    const int hd = a.hd;
    const T* Q = a.qkv + ((int64_t)b * a.S + q) * a.ldq + head * hd;
    const T* K0 = a.qkv + (int64_t)b * a.S * a.ldq + a.n * hd + head * hd;
    const T* V0 = K0 + a.n * hd;
    float mx = -INFINITY;
    for (int k = lane; k <= q; k += 64) mx = fmaxf(mx, dot_rows(Q, K0 + (int64_t)k * a.ldq, hd) * a.scale2);
    mx = wave_max(mx);
    float acc[W];
#pragma unroll
    for (int h = 0; h < W; ++h) acc[h] = 0.f;
    float den = 0.f;
    for (int k = lane; k <= q; k += 64) {
        const float p = exp2f(dot_rows(Q, K0 + (int64_t)k * a.ldq, hd) * a.scale2 - mx);
        den += p;
        const T* V = V0 + (int64_t)k * a.ldq;
#pragma unroll
        for (int h = 0; h < W; ++h)
            if (h < hd) acc[h] = __builtin_fmaf(p, ldv(V + h), acc[h]);
    }
    den = wave_sum(den);
    T* O = a.o_out + ((int64_t)b * a.S + q) * a.ldo + head * hd;
#pragma unroll
    for (int h = 0; h < W; ++h)
        if (h < hd) {
            const float v = wave_sum(acc[h]);
            if (lane == 0) stv(O + h, v / den);
        }
    if (lane == 0) a.lse[((int64_t)b * a.n + head) * a.S + q] = mx + log2f(den);
}

// backward, dQ and delta: dQ[q] = scale sum_{k <= q} dZ[q][k] K[k], dZ = P (dP - delta), dP[q][k] = dO[q] . V[k]
template <typename T, int W>
__global__ __launch_bounds__(64) void attn_plain_dq_kernel(PlainArgs<T> a) {
    const int q = blockIdx.x, head = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
    const int hd = a.hd;
    const int64_t tok = (int64_t)b * a.S + q;
    const T* Q = a.qkv + tok * a.ldq + head * hd;
    const T* K0 = a.qkv + (int64_t)b * a.S * a.ldq + a.n * hd + head * hd;
    const T* V0 = K0 + a.n * hd;
    const T* dO = a.dO + tok * a.ldo + head * hd;
    const T* O = a.o + tok * a.ldo + head * hd;
    const int64_t st = ((int64_t)b * a.n + head) * a.S + q;
    float d = 0.f;
    for (int h = lane; h < hd; h += 64) d = __builtin_fmaf(ldv(dO + h), ldv(O + h), d);
    d = wave_sum(d);
    if (lane == 0) a.delta[st] = d;
    const float L2 = a.lse[st];
    float acc[W];
#pragma unroll
    for (int h = 0; h < W; ++h) acc[h] = 0.f;
    for (int k = lane; k <= q; k += 64) {
        const T* K = K0 + (int64_t)k * a.ldq;
        const float p = exp2f(dot_rows(Q, K, hd) * a.scale2 - L2);
        const float dz = p * (dot_rows(dO, V0 + (int64_t)k * a.ldq, hd) - d);
#pragma unroll
        for (int h = 0; h < W; ++h)
            if (h < hd) acc[h] = __builtin_fmaf(dz, ldv(K + h), acc[h]);
    }
    T* dQ = a.dqkv + tok * a.ldq + head * hd;
#pragma unroll
    for (int h = 0; h < W; ++h)
        if (h < hd) {
            const float v = wave_sum(acc[h]);
            if (lane == 0) stv(dQ + h, v * a.scale);
        }
}

// backward, dK and dV of key k: sums over the queries q >= k (lanes share them out); reads delta
template <typename T, int W>
__global__ __launch_bounds__(64) void attn_plain_dkv_kernel(PlainArgs<T> a) {
    const int k = blockIdx.x, head = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
    const int hd = a.hd;
    const T* Q0 = a.qkv + (int64_t)b * a.S * a.ldq + head * hd;
    const T* K = Q0 + (int64_t)k * a.ldq + a.n * hd;
    const T* V = K + a.n * hd;
    const T* dO0 = a.dO + (int64_t)b * a.S * a.ldo + head * hd;
    const int64_t st = ((int64_t)b * a.n + head) * a.S;
    float ak[W], av[W];
#pragma unroll
    for (int h = 0; h < W; ++h) ak[h] = 0.f, av[h] = 0.f;
    for (int q = k + lane; q < a.S; q += 64) {
        const T* Q = Q0 + (int64_t)q * a.ldq;
        const T* dO = dO0 + (int64_t)q * a.ldo;
        const float p = exp2f(dot_rows(Q, K, hd) * a.scale2 - a.lse[st + q]);
        const float dz = p * (dot_rows(dO, V, hd) - a.delta[st + q]);
#pragma unroll
        for (int h = 0; h < W; ++h)
            if (h < hd) {
                av[h] = __builtin_fmaf(p, ldv(dO + h), av[h]);
                ak[h] = __builtin_fmaf(dz, ldv(Q + h), ak[h]);
            }
    }
    T* dK = a.dqkv + ((int64_t)b * a.S + k) * a.ldq + a.n * hd + head * hd;
    T* dV = dK + a.n * hd;
#pragma unroll
    for (int h = 0; h < W; ++h)
        if (h < hd) {
            const float vk = wave_sum(ak[h]), vv = wave_sum(av[h]);
            if (lane == 0) stv(dK + h, vk * a.scale), stv(dV + h, vv);
        }
}

template <typename T>
PlainArgs<T> make_args(const AttnCoreDesc& c) {
    PlainArgs<T> a{};
    a.qkv = (const T*)c.qkv, a.ldq = c.ldq;
    a.o = (const T*)c.o, a.o_out = (T*)c.o_out, a.dO = (const T*)c.dO, a.ldo = c.ldo;
    a.lse = c.lse, a.delta = c.delta, a.dqkv = (T*)c.dqkv;
    a.S = c.S, a.n = c.n, a.hd = c.hd;
    a.scale = 1.f / sqrtf((float)c.hd), a.scale2 = a.scale * 1.44269504088896340736f;
    return a;
}

template <typename T>
int fwd_t(const AttnCoreDesc& c, hipStream_t s) {
    ProfileScope ps("attn_core_fwd", s);
    if (c.hd <= 64) attn_plain_fwd_kernel<T, 64><<<dim3(c.S, c.n, c.Bt), 64, 0, s>>>(make_args<T>(c));
    else attn_plain_fwd_kernel<T, MAXHD><<<dim3(c.S, c.n, c.Bt), 64, 0, s>>>(make_args<T>(c));
    return launch_status();
}
template <typename T>
int bwd_t(const AttnCoreDesc& c, hipStream_t s) {
    {
        ProfileScope ps("attn_core_bwd_dq", s);
        if (c.hd <= 64) attn_plain_dq_kernel<T, 64><<<dim3(c.S, c.n, c.Bt), 64, 0, s>>>(make_args<T>(c));
        else attn_plain_dq_kernel<T, MAXHD><<<dim3(c.S, c.n, c.Bt), 64, 0, s>>>(make_args<T>(c));
        const int rc = launch_status();
        if (rc != SDP_OK) return rc;
    }
    ProfileScope ps("attn_core_bwd_dkv", s); // reads the delta written by the dQ kernel
    if (c.hd <= 64) attn_plain_dkv_kernel<T, 64><<<dim3(c.S, c.n, c.Bt), 64, 0, s>>>(make_args<T>(c));
    else attn_plain_dkv_kernel<T, MAXHD><<<dim3(c.S, c.n, c.Bt), 64, 0, s>>>(make_args<T>(c));
    return launch_status();
}

} // namespace

bool attn_plain_supported(const AttnCoreDesc& c) { return c.hd >= 1 && c.hd <= MAXHD && c.n <= 65535 && c.Bt <= 65535; }

int attn_plain_fwd(int dtype, const AttnCoreDesc& c, hipStream_t s) {
    if (!attn_plain_supported(c)) return SDP_ERR_UNSUPPORTED;
    return dtype == SDP_F32 ? fwd_t<float>(c, s) : fwd_t<uint16_t>(c, s);
}
int attn_plain_bwd(int dtype, const AttnCoreDesc& c, hipStream_t s) {
    if (!attn_plain_supported(c)) return SDP_ERR_UNSUPPORTED;
    return dtype == SDP_F32 ? bwd_t<float>(c, s) : bwd_t<uint16_t>(c, s);
}

} // namespace sdp
