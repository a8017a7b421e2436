// One worker's attention block under head-level masks (the paper's Sec. 4.1: the neuron-level variant of
// Sec. 3.2 masks attention heads on W_Q, W_K, W_V and W_O), forward masking (Sec. 3.1): the block is
// evaluated at the gated parameters, i.e. as the smaller dense block made of the worker's ph heads.  Under
// backward masking the block runs on all H heads without gather lists, and only the weight-gradient
// contraction is restricted to the held heads' rows (row gather on its left operand).
//
// With E = ph * hd, rows_qkv = the 3 E rows of [Wq; Wk; Wv] that belong to the held heads and rows_o the E
// rows of WoT (columns of W_O):
//   forward   qkv   : [Q | K | V] = X . Wqkv[rows_qkv]^T      (T x 3E, depth d; rows gathered in the load)
//             core  : O_h = softmax_causal(Q_h K_h^T / sqrt(hd)) V_h, per sequence and held head
//             out   : Y = O . WoT[rows_o]                     (T x d, depth E)
//   backward  dO = dY . WoT[rows_o]^T (T x E);  core backward -> dQ, dK, dV (T x 3E);
//             dWqkv[rows_qkv] = dQKV^T . X, dWoT[rows_o] = O^T . dY (depth T);  dX = dQKV . Wqkv[rows_qkv]
// The contractions are the ones of the MLP path (same kernels, other shapes).  The core is written here:
// causal attention on 32x32x16 bf16 MFMA tiles for hd = 64, with the running-maximum formulation of
// the softmax (logits in base 2), so that no T x T matrix is stored.
//
// Accumulator convention.  v_mfma_f32_32x32x16 computes D[m][n] += sum_k A[m][k] B[k][n]; lane L supplies
// A[L % 32][8 (L / 32) + e] and B[8 (L / 32) + e][L % 32], e = 0..7, and holds D[8 q + 4 (L / 32) + r][L % 32]
// in element 4 q + r.  Every product below puts the index that owns per-row softmax statistics on n, so that
// a lane keeps one query (or one key) and its statistics are plain per-lane scalars.  The probabilities then
// feed the next product straight from the accumulator registers: elements 8 s .. 8 s + 7 of a 32-wide tile
// are, for this lane, the depth indices {16 s + 4 (L / 32) + r} and {16 s + 8 + 4 (L / 32) + r}, and the other
// operand is read from LDS in that same order with two transposing reads (ds_read_tr16_b64), which turn a
// row-major [depth][column] tile into the per-lane layout of an A operand.
#include "sdp_internal.h"

#include <cmath>

namespace sdp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;

// Tuning knobs (compile time): waves per SIMD the forward and dQ kernels are register-allocated for, query blocks
// per wave and waves per workgroup of the forward kernel.  Measured at 4 x 2048 tokens, 12 heads: 3 waves per
// SIMD beat 2 (forward 86 -> 77 us) and 4 spill; 2 query blocks per wave spill and were slower.
#ifndef SDP_ATTN_WPE_FWD
#define SDP_ATTN_WPE_FWD 3
#endif
#ifndef SDP_ATTN_WPE_DQ
#define SDP_ATTN_WPE_DQ 3
#endif
#ifndef SDP_ATTN_FWD_QF
#define SDP_ATTN_FWD_QF 1
#endif
#ifndef SDP_ATTN_FWD_NW
#define SDP_ATTN_FWD_NW 4
#endif

constexpr int HD = 64;              // head width of the MFMA core
constexpr int RSB = 144;            // bytes per LDS tile row: 64 bf16 + 16 bytes (bank spread), 16-byte aligned
constexpr int TILE_BYTES = 64 * RSB; // one 64 x 64 tile
constexpr float kSlack = 8.f;      // forward: how far a query's maximum may run ahead of its reference exponent
constexpr int BQ = 128;             // rows (queries, or keys in the dK/dV kernel) per workgroup: 4 waves x 32

struct CoreArgs {
    const uint16_t* qkv; // [T][ldq]: Q | K | V of the held heads, head i at columns i * 64 of each part
    int64_t ldq;
    const uint16_t* o;   // [T][ldo] attention output (forward: written; backward: read)
    uint16_t* o_out;
    const uint16_t* dO;  // [T][ldo]
    int64_t ldo;
    float* lse;          // [Bt][ph][S]: base-2 log-sum-exp of the scaled logits
    float* delta;        // [Bt][ph][S]: sum_h dO[t][h] O[t][h]
    uint16_t* dqkv;      // [T][ldq]
    int S, ph;
    float scale, scale2; // 1 / sqrt(hd), and that times log2(e)
};

__device__ inline uint32_t pack_bf16(float lo, float hi) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const bf16x2 v = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, v);
}

// acc + the two bf16 halves of w (v_dot2c_f32_bf16 against a pair of ones)
__device__ inline float pair_sum(uint32_t w, float acc) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w), ones, acc, false);
}

// elements 8 s .. 8 s + 7 of an accumulator tile as a bf16 operand
__device__ inline bf16x8 pack_operand(const f32x16& a, int s) {
    const u32x4 v = {pack_bf16(a[8 * s], a[8 * s + 1]), pack_bf16(a[8 * s + 2], a[8 * s + 3]),
                     pack_bf16(a[8 * s + 4], a[8 * s + 5]), pack_bf16(a[8 * s + 6], a[8 * s + 7])};
    return __builtin_bit_cast(bf16x8, v);
}

// operand whose depth runs along a tile row: row `row` of the tile, depth 16 s + 8 lhi .. + 7
__device__ inline bf16x8 frag_rows(const unsigned char* tile, int row, int s, int lhi) {
    return __builtin_bit_cast(bf16x8, *(const u32x4*)(tile + row * RSB + 32 * s + 16 * lhi));
}

// A operand whose depth runs down the tile rows: for lane L, column col0 + L % 32 and the rows
// krow + 4 (L / 32) + e (e = 0..3), then krow + 8 + 4 (L / 32) + e.  Within each block of 16 lanes a
// transposing read hands lane n the e-th 16-bit element (e = 0..3) of what lane 4 e + n / 4 addressed,
// at position n % 4 of its 8 bytes: the 16 lanes address 4 rows x 4 groups of 4 columns.
__device__ inline bf16x8 frag_cols(const unsigned char* tile, int krow, int col0, int lane) {
    const int gi = lane >> 4, li = lane & 15;
    const unsigned char* p = tile + (krow + 4 * (gi >> 1) + (li >> 2)) * RSB + (col0 + 16 * (gi & 1) + 4 * (li & 3)) * 2;
    const s16x4 h0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)p);
    const s16x4 h1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p + 8 * RSB));
    const u32x2 a = __builtin_bit_cast(u32x2, h0), b = __builtin_bit_cast(u32x2, h1);
    return __builtin_bit_cast(bf16x8, u32x4{a[0], a[1], b[0], b[1]});
}

// The 16-byte pieces of a 64-row x 64-column tile that thread `tid` of a workgroup of NW waves moves from
// global memory to LDS through registers.  Rows are clamped to the last valid one (such rows only meet masked
// logits).  `g` is uniform over the workgroup; the per-thread part of the address is a 32-bit byte offset
// (the host checks that a sequence's rows span less than 4 GiB), which keeps the address arithmetic to a
// minimum, one multiply and add per piece.
template <int NW>
struct TileMover {
    static constexpr int PER = 512 / (64 * NW); // pieces per thread and tile
    u32x4 v[PER];
    __device__ void fetch(const uint16_t* g, uint32_t ld, int row0, int last_row, int tid) {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int c = tid + 64 * NW * i;
            int row = row0 + (c >> 3);
            row = row < last_row ? row : last_row;
            const uint32_t off = ((uint32_t)row * ld + (uint32_t)(c & 7) * 8u) * 2u;
            v[i] = *(const u32x4*)((const unsigned char*)g + off);
        }
    }
    __device__ void stash(unsigned char* tile, int tid) const {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int c = tid + 64 * NW * i;
            *(u32x4*)(tile + (c >> 3) * RSB + (c & 7) * 16) = v[i];
        }
    }
};
typedef TileMover<4> TilePieces;

// a row of 64 bf16 as the depth-along-row operand of lane (row, lhi): sub-step s holds depth 16 s + 8 lhi .. + 7
__device__ inline void load_row_operand(const uint16_t* g, int64_t ld, int row, int lhi, bf16x8 (&f)[4]) {
#pragma unroll
    for (int s = 0; s < 4; ++s) f[s] = __builtin_bit_cast(bf16x8, *(const u32x4*)(g + (int64_t)row * ld + 16 * s + 8 * lhi));
}

// accumulator tiles D[h][row] (two 32-row blocks of h) -> out[row][32 j + 8 q + 4 lhi + r], scaled, 8-byte stores
__device__ inline void store_rows(uint16_t* out_row, const f32x16 (&acc)[2], float f, int lhi) {
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q)
            *(u32x2*)(out_row + 32 * j + 8 * q + 4 * lhi) =
                u32x2{pack_bf16(acc[j][4 * q] * f, acc[j][4 * q + 1] * f), pack_bf16(acc[j][4 * q + 2] * f, acc[j][4 * q + 3] * f)};
}

__device__ inline float other_half(float x) { return __shfl_xor(x, 32, 64); }

// 2^x for x <= 0 (or -inf): the hardware instruction alone; results below the normal range may flush to zero
__device__ inline float exp2_neg(float x) { return __builtin_amdgcn_exp2f(x); }

// ---------------------------------------------------------------------------------------------------
// Forward.  Workgroup = NW waves; wave w keeps QF blocks of 32 queries (q0 + 32 QF w ..) as register
// operands and walks the key/value tiles of 64 keys up to the diagonal.  K and V tiles are double-buffered
// in LDS (one barrier per tile): while tile t is used, tile t + 1 moves from registers into the other
// buffer and tile t + 2 is fetched from memory.  Every K and V fragment read from LDS serves all QF query
// blocks of the wave.
// ---------------------------------------------------------------------------------------------------
template <int QF, int NW>
__device__ inline void attn_fwd_block(const CoreArgs& a, const int q0, const int head, const int b,
                                      unsigned char (&sK)[2][TILE_BYTES], unsigned char (&sV)[2][TILE_BYTES]) {
    constexpr int ROWS = 32 * QF * NW; // queries per block
    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, lhi = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int S = a.S;
    const uint16_t* gQ = a.qkv + (int64_t)b * S * a.ldq + head * HD;
    const uint16_t* gK = gQ + a.ph * HD;
    const uint16_t* gV = gK + a.ph * HD;
    const int qrow0 = q0 + 32 * QF * wave; // first query of the wave
    bf16x8 qf[QF][4];
#pragma unroll
    for (int f = 0; f < QF; ++f) {
        const int qrow = qrow0 + 32 * f + l32;
        load_row_operand(gQ, a.ldq, qrow < S ? qrow : S - 1, lhi, qf[f]);
    }

    const int kv_end = q0 + ROWS < S ? q0 + ROWS : S;
    const int ntiles = (kv_end + 63) / 64;
    f32x16 acc_o[QF][2];
    float m[QF], lsum[QF];
#pragma unroll
    for (int f = 0; f < QF; ++f) {
        m[f] = -INFINITY, lsum[f] = 0.f;
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc_o[f][j][e] = 0.f;
    }

    TileMover<NW> pk, pv;
    const uint32_t ld = (uint32_t)a.ldq;
    pk.fetch(gK, ld, 0, S - 1, tid);
    pv.fetch(gV, ld, 0, S - 1, tid);
    pk.stash(sK[0], tid);
    pv.stash(sV[0], tid);
    // fetches and stashes run unconditionally (rows are clamped, and a tile beyond the last one is never
    // read): no branch, hence no register copies, around the loop-carried pieces
    pk.fetch(gK, ld, 64, S - 1, tid);
    pv.fetch(gV, ld, 64, S - 1, tid);
    __syncthreads();
    for (int t = 0; t < ntiles; ++t) {
        const unsigned char* tK = sK[t & 1];
        const unsigned char* tV = sV[t & 1];
        // the other buffer was last read before the barrier that ended step t - 1
        pk.stash(sK[(t + 1) & 1], tid);
        pv.stash(sV[(t + 1) & 1], tid);
        pk.fetch(gK, ld, 64 * (t + 2), S - 1, tid);
        pv.fetch(gV, ld, 64 * (t + 2), S - 1, tid);
        const int kv0 = 64 * t;
        if (kv0 <= qrow0 + 32 * QF - 1) { // wave-uniform: otherwise every key lies after the wave's queries
            // logits, transposed: sc[f][tb] = D[key 32 tb + ..][query of block f]
            f32x16 sc[QF][2];
#pragma unroll
            for (int f = 0; f < QF; ++f)
#pragma unroll
                for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                    for (int e = 0; e < 16; ++e) sc[f][tb][e] = 0.f;
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const bf16x8 kfr = frag_rows(tK, 32 * tb + l32, s, lhi);
#pragma unroll
                    for (int f = 0; f < QF; ++f)
                        sc[f][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr, qf[f][s], sc[f][tb], 0, 0, 0);
                }
            if (kv0 + 63 > qrow0 || kv0 + 64 > S) { // wave-uniform: some logits of this tile are masked
#pragma unroll
                for (int f = 0; f < QF; ++f) {
                    const int qrow = qrow0 + 32 * f + l32;
#pragma unroll
                    for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                        for (int e = 0; e < 16; ++e) {
                            const int key = kv0 + 32 * tb + 8 * (e >> 2) + 4 * lhi + (e & 3);
                            if (key > qrow || key >= S) sc[f][tb][e] = -INFINITY;
                        }
                }
            }
            bf16x8 pf[QF][2][2]; // probabilities as operands: [query block][key block][depth half]
#pragma unroll
            for (int f = 0; f < QF; ++f) {
                float mx = -INFINITY;
#pragma unroll
                for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                    for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sc[f][tb][e]);
                mx = fmaxf(mx, other_half(mx));
                // m is the reference the exponents are taken against, in units of the scaled base-2 logits (the
                // scale rides in the multiply-add).  It follows the running maximum lazily: only when a query's
                // maximum has grown by more than kSlack is the reference moved and the accumulators rescaled, so
                // probabilities stay below 2^kSlack and the 32 multiplies of the rescale run on few tiles (the
                // first one always: it holds key 0, which no query masks, so m is finite from then on).
                const float m_cand = mx * a.scale2;
                if (__builtin_amdgcn_ballot_w64(m_cand > m[f] + kSlack) != 0) { // wave-uniform
                    const float m_new = m_cand > m[f] + kSlack ? m_cand : m[f];
                    const float alpha = exp2_neg(m[f] - m_new);
                    m[f] = m_new;
                    lsum[f] *= alpha;
#pragma unroll
                    for (int j = 0; j < 2; ++j)
#pragma unroll
                        for (int e = 0; e < 16; ++e) acc_o[f][j][e] *= alpha;
                }
                // the sum runs over the rounded probabilities, the ones the second product sees, two per instruction
                float ps = 0.f;
#pragma unroll
                for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        u32x4 w;
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float p0 = exp2_neg(__builtin_fmaf(sc[f][tb][8 * h + 2 * i], a.scale2, -m[f]));
                            const float p1 = exp2_neg(__builtin_fmaf(sc[f][tb][8 * h + 2 * i + 1], a.scale2, -m[f]));
                            w[i] = pack_bf16(p0, p1);
                            ps = pair_sum(w[i], ps);
                        }
                        pf[f][tb][h] = __builtin_bit_cast(bf16x8, w);
                    }
                lsum[f] += ps;
            }
            // O^T[h][query] += sum_key V[key][h] P[query][key]
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int s = 0; s < 2; ++s)
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        const bf16x8 vfr = frag_cols(tV, 32 * tb + 16 * s, 32 * j, lane);
#pragma unroll
                        for (int f = 0; f < QF; ++f)
                            acc_o[f][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfr, pf[f][tb][s], acc_o[f][j], 0, 0, 0);
                    }
        }
        __syncthreads(); // tile t is released, tile t + 1 is in place
    }
#pragma unroll
    for (int f = 0; f < QF; ++f) {
        const int qrow = qrow0 + 32 * f + l32;
        const float l = lsum[f] + other_half(lsum[f]);
        if (qrow < S) {
            store_rows(a.o_out + ((int64_t)b * S + qrow) * a.ldo + head * HD, acc_o[f], 1.f / l, lhi);
            if (lhi == 0) a.lse[((int64_t)b * a.ph + head) * S + qrow] = m[f] + log2f(l);
        }
    }
}

// Causal rows differ in length: block i of a sequence meets i + 1 blocks of keys, and at the sizes this
// block runs at every workgroup of a launch is resident at once (about three per CU), so nothing evens the
// work out afterwards.  One block per workgroup, and the blocks are dealt to the workgroup ids so that ids
// congruent modulo the number of CUs -- which the dispatcher places on the same CU, one pass after the other
// -- get a long, a short and a middling block: ranks in the order "longest first" run forwards in even passes
// and backwards in odd ones.  Launches with more passes than fit at once start the long blocks first.
__device__ inline void causal_item(int L, int nitems, int nbh, int nblocks, int ph, int& blk, int& head, int& b) {
    constexpr int W = 256;
    const int pass = L / W, base = pass * W;
    const int width = nitems - base < W ? nitems - base : W;
    const int w = L - base;
    const int r = (pass & 1) ? base + (width - 1 - w) : base + w;
    blk = nblocks - 1 - r / nbh;
    const int bh = r % nbh;
    head = bh % ph, b = bh / ph;
}

template <int QF, int NW>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(SDP_ATTN_WPE_FWD, SDP_ATTN_WPE_FWD)))
void attn_fwd_kernel(CoreArgs a, int nblocks, int nbh) {
    __shared__ __attribute__((aligned(16))) unsigned char sK[2][TILE_BYTES];
    __shared__ __attribute__((aligned(16))) unsigned char sV[2][TILE_BYTES];
    int blk, head, b;
    causal_item(blockIdx.x, gridDim.x, nbh, nblocks, a.ph, blk, head, b);
    attn_fwd_block<QF, NW>(a, blk * 32 * QF * NW, head, b, sK, sV);
}

// ---------------------------------------------------------------------------------------------------
// Backward, dQ (and delta).  Same walk as the forward: wave w keeps its 32 queries' Q and dO rows as
// register operands; P is recomputed from the stored log-sum-exp.
//   dP[q][k] = dO[q] . V[k];  dZ = P (dP - delta[q]);  dQ[q] = scale sum_k dZ[q][k] K[k]
// ---------------------------------------------------------------------------------------------------
__device__ inline void attn_bwd_dq_block(const CoreArgs& a, const int q0, const int head, const int b,
                                         unsigned char (&sK)[TILE_BYTES], unsigned char (&sV)[TILE_BYTES]) {
    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, lhi = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int S = a.S;
    const uint16_t* gQ = a.qkv + (int64_t)b * S * a.ldq + head * HD;
    const uint16_t* gK = gQ + a.ph * HD;
    const uint16_t* gV = gK + a.ph * HD;
    const int qrow0 = q0 + 32 * wave, qrow = qrow0 + l32;
    const int qc = qrow < S ? qrow : S - 1;
    bf16x8 qf[4], dof[4];
    load_row_operand(gQ, a.ldq, qc, lhi, qf);
    const int64_t orow = ((int64_t)b * S + qc) * a.ldo + head * HD;
    load_row_operand(a.dO + orow, 0, 0, lhi, dof);
    float delta = 0.f;
    {
        bf16x8 of[4];
        load_row_operand(a.o + orow, 0, 0, lhi, of);
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int e = 0; e < 8; ++e) delta += (float)dof[s][e] * (float)of[s][e];
        delta += other_half(delta);
    }
    const int64_t stat = ((int64_t)b * a.ph + head) * S;
    if (qrow < S && lhi == 0) a.delta[stat + qrow] = delta;
    const float L2 = a.lse[stat + qc];

    const int kv_end = q0 + BQ < S ? q0 + BQ : S;
    const int ntiles = (kv_end + 63) / 64;
    f32x16 acc[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;

    TilePieces pk, pv;
    const uint32_t ld = (uint32_t)a.ldq;
    pk.fetch(gK, ld, 0, S - 1, tid);
    pv.fetch(gV, ld, 0, S - 1, tid);
    for (int t = 0; t < ntiles; ++t) {
        __syncthreads();
        pk.stash(sK, tid);
        pv.stash(sV, tid);
        __syncthreads();
        pk.fetch(gK, ld, 64 * (t + 1), S - 1, tid); // unconditional: rows are clamped
        pv.fetch(gV, ld, 64 * (t + 1), S - 1, tid);
        const int kv0 = 64 * t;
        if (kv0 > qrow0 + 31) continue;
        const bool edge = kv0 + 63 > qrow0 || kv0 + 64 > S;
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
            f32x16 sc, dp;
#pragma unroll
            for (int e = 0; e < 16; ++e) sc[e] = 0.f, dp[e] = 0.f;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(sK, 32 * tb + l32, s, lhi), qf[s], sc, 0, 0, 0);
                dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(sV, 32 * tb + l32, s, lhi), dof[s], dp, 0, 0, 0);
            }
            if (edge) {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int key = kv0 + 32 * tb + 8 * (e >> 2) + 4 * lhi + (e & 3);
                    if (key > qrow || key >= S) sc[e] = -INFINITY;
                }
            }
#pragma unroll
            for (int e = 0; e < 16; ++e) sc[e] = exp2_neg(__builtin_fmaf(sc[e], a.scale2, -L2)) * (dp[e] - delta);
            // dQ^T[h][query] += sum_key K[key][h] dZ[query][key]
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const bf16x8 zf = pack_operand(sc, s);
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols(sK, 32 * tb + 16 * s, 32 * j, lane), zf, acc[j], 0, 0, 0);
            }
        }
    }
    if (qrow < S) store_rows(a.dqkv + ((int64_t)b * S + qrow) * a.ldq + head * HD, acc, a.scale, lhi);
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(SDP_ATTN_WPE_DQ, SDP_ATTN_WPE_DQ))) void attn_bwd_dq_kernel(CoreArgs a, int nblocks, int nbh) {
    __shared__ __attribute__((aligned(16))) unsigned char sK[TILE_BYTES];
    __shared__ __attribute__((aligned(16))) unsigned char sV[TILE_BYTES];
    int blk, head, b;
    causal_item(blockIdx.x, gridDim.x, nbh, nblocks, a.ph, blk, head, b);
    attn_bwd_dq_block(a, blk * BQ, head, b, sK, sV);
}

// ---------------------------------------------------------------------------------------------------
// Backward, dK and dV.  Workgroup = 128 keys of one (sequence, head); wave w keeps keys k0 + 32 w .. + 31
// (K and V rows) as register operands and walks the query tiles from the diagonal to the end of the
// sequence; Q, dO and the per-query statistics of a tile of 64 queries are staged in LDS.
//   dV[k] = sum_q P[q][k] dO[q];   dK[k] = scale sum_q dZ[q][k] Q[q]
// ---------------------------------------------------------------------------------------------------
__device__ inline void attn_bwd_dkv_block(const CoreArgs& a, const int k0, const int head, const int b,
                                          unsigned char (&sQ)[TILE_BYTES], unsigned char (&sO)[TILE_BYTES], float (&sL)[64],
                                          float (&sD)[64]) {
    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, lhi = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int S = a.S;
    const uint16_t* gQ = a.qkv + (int64_t)b * S * a.ldq + head * HD;
    const uint16_t* gK = gQ + a.ph * HD;
    const uint16_t* gV = gK + a.ph * HD;
    const uint16_t* gO = a.dO + (int64_t)b * S * a.ldo + head * HD;
    const int64_t stat = ((int64_t)b * a.ph + head) * S;
    const int krow0 = k0 + 32 * wave, krow = krow0 + l32;
    const int kc = krow < S ? krow : S - 1;
    bf16x8 kf[4], vf[4];
    load_row_operand(gK, a.ldq, kc, lhi, kf);
    load_row_operand(gV, a.ldq, kc, lhi, vf);

    f32x16 acc_k[2], acc_v[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc_k[j][e] = 0.f, acc_v[j][e] = 0.f;

    const int t0 = k0 / 64, t1 = (S + 63) / 64; // query tiles [t0, t1); t0 < t1 because k0 < S
    TilePieces pq, po;
    const uint32_t ldq32 = (uint32_t)a.ldq, ldo32 = (uint32_t)a.ldo;
    // per-query statistics of a tile: threads 0..63 carry the log-sum-exp, 64..127 delta
    const float* gstat = (tid < 64 ? a.lse : a.delta) + stat;
    const int sq = tid & 63;
    float pstat;
    pq.fetch(gQ, ldq32, 64 * t0, S - 1, tid);
    po.fetch(gO, ldo32, 64 * t0, S - 1, tid);
    pstat = gstat[64 * t0 + sq < S ? 64 * t0 + sq : S - 1];
    for (int t = t0; t < t1; ++t) {
        __syncthreads();
        pq.stash(sQ, tid);
        po.stash(sO, tid);
        if (tid < 64) sL[tid] = pstat;
        else if (tid < 128) sD[tid - 64] = pstat;
        __syncthreads();
        // the next tile, unconditionally: rows are clamped
        pq.fetch(gQ, ldq32, 64 * (t + 1), S - 1, tid);
        po.fetch(gO, ldo32, 64 * (t + 1), S - 1, tid);
        pstat = gstat[64 * (t + 1) + sq < S ? 64 * (t + 1) + sq : S - 1];
        const int qt0 = 64 * t;
        if (qt0 + 63 < krow0) continue; // wave-uniform: every query of the tile lies before the wave's keys
        const bool edge = qt0 < krow0 + 31 || qt0 + 64 > S;
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
            // sc = D[query 32 tb + ..][key], dp likewise
            f32x16 sc, dp;
#pragma unroll
            for (int e = 0; e < 16; ++e) sc[e] = 0.f, dp[e] = 0.f;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(sQ, 32 * tb + l32, s, lhi), kf[s], sc, 0, 0, 0);
                dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(sO, 32 * tb + l32, s, lhi), vf[s], dp, 0, 0, 0);
            }
            if (edge) { // a branch of its own: only the tiles on the diagonal and the ragged last one pay for it
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int query = qt0 + 32 * tb + 8 * (e >> 2) + 4 * lhi + (e & 3);
                    if (krow > query || query >= S) sc[e] = -INFINITY;
                }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x4 l4 = *(const f32x4*)(sL + 32 * tb + 8 * q + 4 * lhi);
                const f32x4 d4 = *(const f32x4*)(sD + 32 * tb + 8 * q + 4 * lhi);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float z = sc[4 * q + r];
                    const float p = exp2_neg(__builtin_fmaf(z, a.scale2, -l4[r]));
                    sc[4 * q + r] = p;
                    dp[4 * q + r] = p * (dp[4 * q + r] - d4[r]);
                }
            }
            // dV^T[h][key] += sum_query dO[query][h] P[query][key];  dK^T[h][key] += sum_query Q[query][h] dZ[query][key]
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const bf16x8 pf = pack_operand(sc, s), zf = pack_operand(dp, s);
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    acc_v[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols(sO, 32 * tb + 16 * s, 32 * j, lane), pf, acc_v[j], 0, 0, 0);
                    acc_k[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols(sQ, 32 * tb + 16 * s, 32 * j, lane), zf, acc_k[j], 0, 0, 0);
                }
            }
        }
    }
    if (krow < S) {
        uint16_t* row = a.dqkv + ((int64_t)b * S + krow) * a.ldq + head * HD;
        store_rows(row + a.ph * HD, acc_k, a.scale, lhi);
        store_rows(row + 2 * a.ph * HD, acc_v, 1.f, lhi);
    }
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_bwd_dkv_kernel(CoreArgs a, int nblocks, int nbh) {
    __shared__ __attribute__((aligned(16))) unsigned char sQ[TILE_BYTES];
    __shared__ __attribute__((aligned(16))) unsigned char sO[TILE_BYTES];
    __shared__ __attribute__((aligned(16))) float sL[64];
    __shared__ __attribute__((aligned(16))) float sD[64];
    int blk, head, b;
    causal_item(blockIdx.x, gridDim.x, nbh, nblocks, a.ph, blk, head, b);
    // key block i meets the query blocks i .. n - 1: the first key blocks are the long ones
    attn_bwd_dkv_block(a, (nblocks - 1 - blk) * BQ, head, b, sQ, sO, sL, sD);
}

// rows of [Wq; Wk; Wv] ([3 H hd][d]) and of WoT ([H hd][d]) that belong to the held heads
__global__ void head_rows_kernel(const int32_t* __restrict__ head_idx, int ph, int H, int hd, int32_t* __restrict__ rows_qkv,
                                 int32_t* __restrict__ rows_o) {
    const int E = ph * hd;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= 3 * E) return;
    const int part = i / E, rem = i - part * E;
    const int row = head_idx[rem / hd] * hd + rem % hd;
    rows_qkv[i] = part * H * hd + row;
    if (part == 0) rows_o[rem] = row;
}

int64_t ld_tokens(int64_t T) { return T + 64; } // see the MLP path: rows must not sit a power of two apart

// Head width the core runs on.  The MFMA core takes bf16 heads of width 64; narrower bf16 heads (the paper's
// 500M / 1B models have width 50) are padded to 64 with zero features: a zero feature of Q and K adds nothing to a
// logit, a zero feature of V gives a zero feature of O, and every gradient of a zero feature is zero.  The padding
// is made once, on the weights (pad_heads_kernel): the saved Q | K | V and O then carry 64 columns per head, of
// which the last 64 - hd are zero.  Everything else (fp32, wider heads) goes through the plain core unpadded.
int core_width(int dtype, int hd) { return dtype == SDP_BF16 && hd <= HD ? HD : hd; }
bool mfma_core(int dtype, int hd) { return core_width(dtype, hd) == HD && dtype == SDP_BF16; }
size_t esize(int dtype) { return dtype == SDP_F32 ? 4 : 2; }

// out[(i hw + r)][:] = r < hd ? in[(heads ? heads[i] : i) hd + r][:] : 0 for i < n, r < hw, per stacked matrix
// (blockIdx.y: matrix z of `in` [z][H hd][d] -> matrix z of `out` [z][n hw][d]); d % 8 == 0, 16 bytes per thread
__global__ __launch_bounds__(256) void pad_heads_kernel(const uint16_t* __restrict__ in, const int32_t* __restrict__ heads,
                                                        int n, int H, int hd, int hw, int d, uint16_t* __restrict__ out) {
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    const int chunks = d / 8;
    const int64_t total = (int64_t)n * hw * chunks;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int row = (int)(i / chunks), c = (int)(i % chunks);
    const int head = row / hw, r = row % hw;
    u32x4_t v = {0u, 0u, 0u, 0u};
    if (r < hd) {
        const int64_t src = (int64_t)blockIdx.y * H * hd + (int64_t)(heads ? heads[head] : head) * hd + r;
        v = *(const u32x4_t*)(in + src * d + c * 8);
    }
    *(u32x4_t*)(out + ((int64_t)blockIdx.y * n * hw + row) * d + c * 8) = v;
}

// Row lists of the weight-gradient launch when heads are padded: for padded row m = i hw + r of the held heads
//   gather[m]  = heads[i] hw + r            (row of the all-heads operand, backward masking)
//   scatter[m] = r < hd ? (full ? heads[i] : i) hd + r : -1     (output row; padding rows are dropped)
__global__ void pad_rows_kernel(const int32_t* __restrict__ heads, int ph, int hd, int hw, int full,
                                int32_t* __restrict__ gather, int32_t* __restrict__ scatter) {
    const int m = blockIdx.x * blockDim.x + threadIdx.x;
    if (m >= ph * hw) return;
    const int i = m / hw, r = m % hw;
    const int h = heads ? heads[i] : i;
    gather[m] = h * hw + r;
    scatter[m] = r < hd ? (full ? h : i) * hd + r : -1;
}

int check(int mode, int dtype, int Bt, int S, int d, int H, int hd, int ph) {
    if (mode != SDP_MASK_FORWARD && mode != SDP_MASK_BACKWARD) return SDP_ERR_INVALID_ARG;
    if (dtype != SDP_BF16 && dtype != SDP_F32) return SDP_ERR_INVALID_ARG;
    if (Bt < 1 || S < 1 || d < 1 || H < 1 || hd < 1) return SDP_ERR_INVALID_ARG;
    if (hd > 128) return SDP_ERR_UNSUPPORTED;
    if (ph < 1 || ph > H) return SDP_ERR_SHAPE;
    if (dtype == SDP_BF16 && (d % 8 || (hd > HD && hd % 8))) return SDP_ERR_SHAPE; // 16-byte rows; heads up to 64 are padded
    if (Bt > 65535 || H > 65535) return SDP_ERR_SHAPE;
    const int hw = core_width(dtype, hd);
    if ((int64_t)Bt * S >= ((int64_t)1 << 31) || (int64_t)Bt * S * 3 * H * hw >= ((int64_t)1 << 40)) return SDP_ERR_SHAPE;
    // MFMA core: 32-bit byte offsets inside a sequence
    if (mfma_core(dtype, hd) && (int64_t)S * 3 * H * hw * 2 >= ((int64_t)1 << 32)) return SDP_ERR_SHAPE;
    return SDP_OK;
}

// heads the forward pass and the core run on: the held ones (forward masking) or all of them (backward masking)
int heads_run(int mode, int H, int ph) { return mode == SDP_MASK_FORWARD ? ph : H; }

struct FwdWs {
    int32_t *rows_qkv, *rows_o;
    void *WoC, *Wp, *WoP; // Wp, WoP: padded copies of the run heads' rows of Wqkv / WoT (padded head widths only)
    size_t bytes;
};
FwdWs fwd_ws(char* w, size_t e, int d, int E, bool padded) {
    FwdWs r;
    size_t off = 0;
    auto take = [&](size_t n) { char* p = w ? w + off : nullptr; off += round_up(n, 256); return p; };
    r.rows_qkv = (int32_t*)take((size_t)3 * E * 4);
    r.rows_o = (int32_t*)take((size_t)E * 4);
    r.WoC = take((size_t)d * E * e);
    r.Wp = padded ? take((size_t)3 * E * d * e) : nullptr;
    r.WoP = padded ? take((size_t)E * d * e) : nullptr;
    r.bytes = off;
    return r;
}

struct BwdWs {
    int32_t *rows_qkv, *rows_o;
    void *dO, *dQKV, *dQKVt, *Ot, *Xt, *dYt, *Wc, *split, *Wp, *WoP;
    float* delta;
    size_t bytes;
};
// E = width the core runs on, Eh = width of the held heads (equal under forward masking), both in padded columns
BwdWs bwd_ws(char* w, size_t e, int64_t T, int d, int E, int Eh, int64_t stats, bool padded) {
    BwdWs r;
    size_t off = 0;
    auto take = [&](size_t n) { char* p = w ? w + off : nullptr; off += round_up(n, 256); return p; };
    r.rows_qkv = (int32_t*)take((size_t)3 * Eh * 4);
    r.rows_o = (int32_t*)take((size_t)Eh * 4);
    r.dO = take((size_t)T * E * e);
    r.dQKV = take((size_t)T * 3 * E * e);
    r.delta = (float*)take((size_t)stats * 4);
    r.dQKVt = take((size_t)3 * E * ld_tokens(T) * e);
    r.Ot = take((size_t)E * ld_tokens(T) * e);
    r.Xt = take((size_t)d * ld_tokens(T) * e);
    r.dYt = take((size_t)d * ld_tokens(T) * e);
    r.Wc = take((size_t)d * 3 * E * e);
    const size_t sp = e == 2 ? gemm_split_ws_bytes(Eh, d, (int)T, 4) : 0; // partial sums of the batched weight-gradient launch
    r.split = sp ? take(sp) : nullptr;
    r.Wp = padded ? take((size_t)3 * E * d * e) : nullptr;
    r.WoP = padded ? take((size_t)E * d * e) : nullptr;
    r.bytes = off;
    return r;
}

// padded copies of the run heads' weight rows (heads == nullptr: all n = H heads in order)
int pad_heads(const void* in, int nmat, const int32_t* heads, int n, int H, int hd, int hw, int d, void* out,
              const char* name, hipStream_t s) {
    ProfileScope ps(name, s);
    const int64_t total = (int64_t)n * hw * (d / 8);
    pad_heads_kernel<<<dim3((unsigned)((total + 255) / 256), nmat), 256, 0, s>>>((const uint16_t*)in, heads, n, H, hd, hw, d,
                                                                                  (uint16_t*)out);
    return launch_status();
}

int run(int dtype, const GemmDesc& g, hipStream_t s) {
    if (dtype == SDP_BF16 && gemm_mfma_supported(g)) return gemm_mfma_bf16(g, s);
    return gemm_simple(dtype, g, s);
}

int head_rows(const int32_t* head_idx, int ph, int H, int hd, int32_t* rows_qkv, int32_t* rows_o, hipStream_t s) {
    ProfileScope ps("attn_rows", s);
    const int n = 3 * ph * hd;
    head_rows_kernel<<<(n + 255) / 256, 256, 0, s>>>(head_idx, ph, H, hd, rows_qkv, rows_o);
    return launch_status();
}

} // namespace
} // namespace sdp

using namespace sdp;

extern "C" int sdp_masked_attn_saved_head_width(int dtype, int hd) {
    if ((dtype != SDP_BF16 && dtype != SDP_F32) || hd < 1 || hd > 128) return 0;
    return core_width(dtype, hd);
}

extern "C" size_t sdp_masked_attn_fwd_workspace_bytes(int mode, int dtype, int Bt, int S, int d, int H, int hd, int ph) {
    if (check(mode, dtype, Bt, S, d, H, hd, ph) != SDP_OK) return 0;
    const int hw = core_width(dtype, hd);
    return fwd_ws(nullptr, esize(dtype), d, heads_run(mode, H, ph) * hw, hw != hd).bytes;
}

extern "C" size_t sdp_masked_attn_bwd_workspace_bytes(int mode, int dtype, int Bt, int S, int d, int H, int hd, int ph) {
    if (check(mode, dtype, Bt, S, d, H, hd, ph) != SDP_OK) return 0;
    const int hr = heads_run(mode, H, ph), hw = core_width(dtype, hd);
    return bwd_ws(nullptr, esize(dtype), (int64_t)Bt * S, d, hr * hw, ph * hw, (int64_t)Bt * hr * S, hw != hd).bytes;
}

extern "C" int sdp_masked_attn_fwd(int mode, int dtype, int Bt, int S, int d, int H, int hd, int ph, const void* X,
                                   const void* Wqkv, const void* WoT, const int32_t* head_idx_k, void* Y, void* QKV_save,
                                   void* O_save, float* LSE_save, void* ws, size_t ws_bytes, void* stream) {
    if (mode == SDP_MASK_BACKWARD) ph = H; // the forward pass is the dense block; the list is not looked at
    int rc = check(mode, dtype, Bt, S, d, H, hd, ph);
    if (rc != SDP_OK) return rc;
    if (!X || !Wqkv || !WoT || !Y || !QKV_save || !O_save || !LSE_save) return SDP_ERR_INVALID_ARG;
    if (mode == SDP_MASK_FORWARD && !head_idx_k) return SDP_ERR_INVALID_ARG;
    for (const void* q : {X, Wqkv, WoT, (const void*)Y, (const void*)QKV_save, (const void*)O_save, (const void*)LSE_save})
        if (!aligned16(q)) return SDP_ERR_INVALID_ARG;
    if (!ws || !aligned16(ws) || ws_bytes < sdp_masked_attn_fwd_workspace_bytes(mode, dtype, Bt, S, d, H, hd, ph))
        return SDP_ERR_WORKSPACE;
    return attn_fwd_impl(mode, dtype, Bt, S, d, H, hd, ph, X, Wqkv, WoT, head_idx_k, Y, QKV_save, O_save, LSE_save, nullptr,
                         ws, (hipStream_t)stream);
}

int sdp::attn_fwd_impl(int mode, int dtype, int Bt, int S, int d, int H, int hd, int ph, const void* X, const void* Wqkv,
                       const void* WoT, const int32_t* head_idx_k, void* Y, void* QKV_save, void* O_save, float* LSE_save,
                       const void* residual, void* ws, hipStream_t s) {
    if (mode == SDP_MASK_BACKWARD) ph = H;
    int rc;
    const bool gathered = mode == SDP_MASK_FORWARD;
    const int hw = core_width(dtype, hd); // columns per head in the saved tensors
    const bool padded = hw != hd;
    const int T = Bt * S, E = ph * hw;
    const FwdWs w = fwd_ws((char*)ws, esize(dtype), d, E, padded);

    if (gathered && !padded) {
        rc = head_rows(head_idx_k, ph, H, hd, w.rows_qkv, w.rows_o, s);
        if (rc != SDP_OK) return rc;
    }
    if (padded) { // the run heads' rows of W_Q, W_K, W_V and W_O, each head padded to hw rows
        rc = pad_heads(Wqkv, 3, gathered ? head_idx_k : nullptr, ph, H, hd, hw, d, w.Wp, "attn_pad_w", s);
        if (rc != SDP_OK) return rc;
        rc = pad_heads(WoT, 1, gathered ? head_idx_k : nullptr, ph, H, hd, hw, d, w.WoP, "attn_pad_w", s);
        if (rc != SDP_OK) return rc;
    }

    GemmDesc pj;
    pj.name = "attn_qkv";
    pj.M = T, pj.N = 3 * E, pj.K = d;
    pj.A = X, pj.lda = d;
    pj.B = padded ? w.Wp : Wqkv, pj.ldb = d;
    if (gathered && !padded) pj.b_gather = w.rows_qkv, pj.b_rows = (int64_t)3 * H * hd;
    pj.epilogue = EPI_STORE;
    pj.C = QKV_save, pj.ldc = 3 * E;
    rc = run(dtype, pj, s);
    if (rc != SDP_OK) return rc;

    if (mfma_core(dtype, hd)) {
        CoreArgs a{};
        a.qkv = (const uint16_t*)QKV_save, a.ldq = 3 * E;
        a.o_out = (uint16_t*)O_save, a.ldo = E;
        a.lse = LSE_save;
        a.S = S, a.ph = ph;
        a.scale = 1.f / sqrtf((float)hd), a.scale2 = a.scale * 1.44269504088896340736f;
        ProfileScope ps("attn_core_fwd", s);
        constexpr int QF = SDP_ATTN_FWD_QF, NW = SDP_ATTN_FWD_NW, ROWS = 32 * QF * NW;
        const int nblocks = (S + ROWS - 1) / ROWS;
        if ((int64_t)nblocks * ph * Bt > INT32_MAX) return SDP_ERR_UNSUPPORTED;
        attn_fwd_kernel<QF, NW><<<dim3(nblocks * ph * Bt), 64 * NW, 0, s>>>(a, nblocks, ph * Bt);
        rc = launch_status();
    } else {
        AttnCoreDesc c;
        c.qkv = QKV_save, c.ldq = 3 * E, c.o_out = O_save, c.ldo = E, c.lse = LSE_save;
        c.Bt = Bt, c.S = S, c.n = ph, c.hd = hd;
        rc = attn_plain_fwd(dtype, c, s);
    }
    if (rc != SDP_OK) return rc;

    rc = transpose_rows((int)esize(dtype), padded ? w.WoP : WoT, d, gathered && !padded ? w.rows_o : nullptr, E, d, w.WoC, E,
                        "attn_wt_fwd", s);
    if (rc != SDP_OK) return rc;
    GemmDesc op;
    op.name = "attn_out";
    op.M = T, op.N = d, op.K = E;
    op.A = O_save, op.lda = E;
    op.B = w.WoC, op.ldb = E;
    op.epilogue = EPI_STORE;
    op.C = Y, op.ldc = d;
    op.R = residual, op.ldr = d;
    return run(dtype, op, s);
}

extern "C" int sdp_masked_attn_bwd(int mode, int dtype, int Bt, int S, int d, int H, int hd, int ph, const void* X,
                                   const void* dY, const void* Wqkv, const void* WoT, const int32_t* head_idx_k,
                                   const void* QKV_save, const void* O_save, const float* LSE_save, void* dX, void* dWqkv,
                                   void* dWoT, int dw_layout, void* ws, size_t ws_bytes, void* stream) {
    int rc = check(mode, dtype, Bt, S, d, H, hd, ph);
    if (rc != SDP_OK) return rc;
    if (dw_layout != SDP_DW_COMPACT && dw_layout != SDP_DW_SCATTER) return SDP_ERR_INVALID_ARG;
    if (!X || !dY || !Wqkv || !WoT || !head_idx_k || !QKV_save || !O_save || !LSE_save || !dX || !dWqkv || !dWoT)
        return SDP_ERR_INVALID_ARG;
    for (const void* q : {X, dY, Wqkv, WoT, QKV_save, O_save, (const void*)LSE_save, (const void*)dX, (const void*)dWqkv,
                          (const void*)dWoT})
        if (!aligned16(q)) return SDP_ERR_INVALID_ARG;
    if (!ws || !aligned16(ws) || ws_bytes < sdp_masked_attn_bwd_workspace_bytes(mode, dtype, Bt, S, d, H, hd, ph))
        return SDP_ERR_WORKSPACE;
    return attn_bwd_impl(mode, dtype, Bt, S, d, H, hd, ph, X, dY, Wqkv, WoT, head_idx_k, QKV_save, O_save, LSE_save, dX,
                         dWqkv, dWoT, dw_layout, nullptr, true, ws, (hipStream_t)stream);
}

int sdp::attn_bwd_impl(int mode, int dtype, int Bt, int S, int d, int H, int hd, int ph, const void* X, const void* dY,
                       const void* Wqkv, const void* WoT, const int32_t* head_idx_k, const void* QKV_save,
                       const void* O_save, const float* LSE_save, void* dX, void* dWqkv, void* dWoT, int dw_layout,
                       const void* dx_residual, bool want_dw, void* ws, hipStream_t s) {
    int rc;
    const bool gathered = mode == SDP_MASK_FORWARD;
    const int hr = heads_run(mode, H, ph);
    const int hw = core_width(dtype, hd);
    const bool padded = hw != hd;
    const int T = Bt * S, E = hr * hw, Eh = ph * hw; // width the core runs on, width of the held heads (padded columns)
    const BwdWs w = bwd_ws((char*)ws, esize(dtype), T, d, E, Eh, (int64_t)Bt * hr * S, padded);
    // no list under backward masking: every head is held (ph = H), no row gather and no scatter are needed
    const bool all_heads = !gathered && head_idx_k == nullptr;

    if (padded) {
        rc = pad_heads(Wqkv, 3, gathered ? head_idx_k : nullptr, hr, H, hd, hw, d, w.Wp, "attn_pad_w", s);
        if (rc != SDP_OK) return rc;
        rc = pad_heads(WoT, 1, gathered ? head_idx_k : nullptr, hr, H, hd, hw, d, w.WoP, "attn_pad_w", s);
        if (rc != SDP_OK) return rc;
        if (want_dw) { // rows of the held heads in the padded operands, and where each of them goes (padding rows: nowhere)
            ProfileScope ps("attn_rows", s);
            pad_rows_kernel<<<(Eh + 255) / 256, 256, 0, s>>>(head_idx_k, ph, hd, hw, dw_layout == SDP_DW_SCATTER, w.rows_o,
                                                             w.rows_qkv);
            rc = launch_status();
            if (rc != SDP_OK) return rc;
        }
    } else if (!all_heads) {
        rc = head_rows(head_idx_k, ph, H, hd, w.rows_qkv, w.rows_o, s);
        if (rc != SDP_OK) return rc;
    }

    GemmDesc go;
    go.name = "attn_dout";
    go.M = T, go.N = E, go.K = d;
    go.A = dY, go.lda = d;
    go.B = padded ? w.WoP : WoT, go.ldb = d;
    if (gathered && !padded) go.b_gather = w.rows_o, go.b_rows = (int64_t)H * hd;
    go.epilogue = EPI_STORE;
    go.C = w.dO, go.ldc = E;
    rc = run(dtype, go, s);
    if (rc != SDP_OK) return rc;

    if (mfma_core(dtype, hd)) {
        CoreArgs a{};
        a.qkv = (const uint16_t*)QKV_save, a.ldq = 3 * E;
        a.o = (const uint16_t*)O_save, a.dO = (const uint16_t*)w.dO, a.ldo = E;
        a.lse = const_cast<float*>(LSE_save), a.delta = w.delta;
        a.dqkv = (uint16_t*)w.dQKV;
        a.S = S, a.ph = hr;
        a.scale = 1.f / sqrtf((float)hd), a.scale2 = a.scale * 1.44269504088896340736f;
        const int nblocks = (S + BQ - 1) / BQ;
        if ((int64_t)nblocks * hr * Bt > INT32_MAX) return SDP_ERR_UNSUPPORTED;
        const dim3 grid(nblocks * hr * Bt);
        {
            ProfileScope ps("attn_core_bwd_dq", s);
            attn_bwd_dq_kernel<<<grid, 256, 0, s>>>(a, nblocks, hr * Bt);
            rc = launch_status();
            if (rc != SDP_OK) return rc;
        }
        {
            ProfileScope ps("attn_core_bwd_dkv", s); // reads the delta written by the dQ kernel
            attn_bwd_dkv_kernel<<<grid, 256, 0, s>>>(a, nblocks, hr * Bt);
            rc = launch_status();
            if (rc != SDP_OK) return rc;
        }
    } else {
        AttnCoreDesc c;
        c.qkv = QKV_save, c.ldq = 3 * E, c.o = O_save, c.dO = w.dO, c.ldo = E;
        c.lse = const_cast<float*>(LSE_save), c.delta = w.delta, c.dqkv = w.dQKV;
        c.Bt = Bt, c.S = S, c.n = hr, c.hd = hd;
        rc = attn_plain_bwd(dtype, c, s);
        if (rc != SDP_OK) return rc;
    }

    rc = transpose_rows((int)esize(dtype), padded ? w.Wp : Wqkv, d, gathered && !padded ? w.rows_qkv : nullptr, 3 * E, d, w.Wc,
                        3 * E, "attn_wt_bwd", s);
    if (rc != SDP_OK) return rc;
    GemmDesc dx;
    dx.name = "attn_dx";
    dx.M = T, dx.N = d, dx.K = 3 * E;
    dx.A = w.dQKV, dx.lda = 3 * E;
    dx.B = w.Wc, dx.ldb = 3 * E;
    dx.epilogue = EPI_STORE;
    dx.C = dX, dx.ldc = d;
    dx.R = dx_residual, dx.ldr = d;
    if (!want_dw) return run(dtype, dx, s);

    const int64_t ldt = ld_tokens(T);
    const TransposeJob tj[4] = {{w.dQKV, w.dQKVt, 3 * E, ldt, nullptr, T, 3 * E},
                                {O_save, w.Ot, E, ldt, nullptr, T, E},
                                {X, w.Xt, d, ldt, nullptr, T, d},
                                {dY, w.dYt, d, ldt, nullptr, T, d}};
    rc = transpose_batch((int)esize(dtype), tj, 4, "attn_tr_bwd", s);
    if (rc != SDP_OK) return rc;

    // the four weight gradients share one shape (Eh x d, depth T): dWq, dWk, dWv from the three row blocks of
    // dQKV^T against X^T, dWoT from O^T against dY^T; one batched launch fills the CUs four times better than
    // the four launches would.  Under backward masking the row blocks hold all heads and the contraction reads
    // the held heads' rows only (row gather on the left operand): the gradient is computed on the mask.
    GemmDesc dw;
    dw.name = "attn_dw";
    dw.M = Eh, dw.N = d, dw.K = T;
    dw.lda = ldt, dw.ldb = ldt;
    if (!gathered && !all_heads) dw.a_gather = w.rows_o, dw.a_rows = E;
    dw.epilogue = EPI_STORE;
    dw.ldc = d;
    dw.c_scatter = dw_layout == SDP_DW_SCATTER && !all_heads ? w.rows_o : nullptr; // rows of the held heads inside each matrix
    if (padded) { // padded rows: w.rows_o = the held heads' rows of the operands, w.rows_qkv = output rows (-1: dropped)
        if (gathered) dw.a_gather = nullptr;
        else dw.a_gather = w.rows_o, dw.a_rows = E;
        dw.c_scatter = w.rows_qkv;
    }
    const int64_t part = (int64_t)(dw_layout == SDP_DW_SCATTER ? H * hd : ph * hd) * d;
    dw.nbatch = 4;
    const size_t e = esize(dtype);
    for (int i = 0; i < 3; ++i) {
        dw.Ab[i] = (const char*)w.dQKVt + (size_t)i * E * ldt * e;
        dw.Bb[i] = w.Xt;
        dw.Cb[i] = (char*)dWqkv + (size_t)i * part * e;
    }
    dw.Ab[3] = w.Ot, dw.Bb[3] = w.dYt, dw.Cb[3] = dWoT;
    dw.split_ws = w.split;
    if (dtype == SDP_BF16 && gemm_mfma_supported(dw)) {
        rc = gemm_mfma_bf16(dw, s);
        if (rc != SDP_OK) return rc;
    } else {
        dw.nbatch = 0;
        for (int i = 0; i < 4; ++i) {
            dw.A = dw.Ab[i], dw.B = dw.Bb[i], dw.C = dw.Cb[i];
            rc = gemm_simple(dtype, dw, s);
            if (rc != SDP_OK) return rc;
        }
    }

    return run(dtype, dx, s);
}
