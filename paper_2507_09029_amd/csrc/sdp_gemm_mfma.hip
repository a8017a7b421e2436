// bf16 MFMA contraction for gfx950 (CDNA4) with the masked-MLP row gather and SwiGLU epilogues fused.
//
//   C[M][N] = sum_k A(m,k) B(k,n),  bf16 operands, fp32 accumulation in v_mfma_f32_16x16x32_bf16.
//   A is stored [M][K], B is stored [N][K] (rows optionally gathered through an index table): both
//   operands are read along the depth, 16 bytes (8 bf16) at a time.
//
// Tile: BM x BN outputs per workgroup, depth step 64, WAVES_M x WAVES_N waves of 64 lanes, each wave
// owning (BM/WAVES_M) x (BN/WAVES_N) outputs as 32 x 32 blocks of four 16 x 16 MFMA tiles.  The flagship shape is
// 256 x 256 with 8 waves: 128 accumulator registers per lane, two waves per SIMD, one workgroup per CU.
//
// HBM/L2 -> LDS: direct loads (global_load_lds_dwordx4).  One wave instruction moves 64 chunks of
// 16 bytes into 1 KB of consecutive LDS ("slab"); which global chunk a lane fetches is free, so the
// LDS layout below is produced by choosing the global address per lane.  No registers and no
// ds_write instructions are spent on staging.  LDS holds two stages of A and three of B.
//
// LDS layout of an operand stage, [R rows][64 k] in 16-byte chunks: chunk (r, c) sits at
// r*8 + (c ^ ((r >> 1) & 7)).  A lane's MFMA operand (8 consecutive k of one row) is one chunk, one
// ds_read_b128, and the lanes served together fall on distinct banks.
//
// Main loop: the waves form two groups that alternate between a phase of LDS reads + load issue and a
// phase of MFMAs only, one phase apart, so that on every SIMD one wave computes while the other one
// fetches (see the comment at the loop).
//
// The MFMA is issued with the B fragment as its first operand: a lane then holds, for one output
// row m, 4 consecutive columns n.  Epilogues go through LDS: each wave packs 32 x WN outputs as bf16
// into a private LDS strip with 8-byte writes and reads the strip back as 16-byte chunks of whole
// rows, so that every global store (and the loads of the saved pre-activations) is a coalesced
// 16-byte access.  SwiGLU and its backward are applied on the fp32 accumulators before packing; the
// backward epilogue can also write its three outputs transposed (transposing LDS reads of the strip).
//
// Workgroup -> tile mapping is XCD-aware: consecutive workgroup ids go round-robin to the 8 XCDs
// (each with its own L2), so ids are first regrouped per XCD and each XCD then walks a compact
// block of tiles (group_m tile-rows at a time, group_m chosen on the host per shape; in a batched
// launch the problems that share an operand are stacked into one matrix first) whose operand
// tiles are shared through that L2.
//
// Batching: the three weight-gradient contractions of one worker (same M x N x K, different operands)
// run as one launch of 3 x tiles workgroups, so that their few, deep tiles fill the CUs together.
#include "sdp_internal.h"
#include "sdp_swiglu.h"

#include <hip/hip_ext.h>

#include <algorithm>
#include <array>
#include <cstdlib>
#include <map>
#include <mutex>
#include <string>
#include <type_traits>
#include <vector>

namespace sdp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef __attribute__((address_space(1))) const void* glb_void_ptr;

constexpr int BK = 64;
constexpr int NUM_XCD = 8;

struct Dev {
    int M, N, K;
    const uint16_t *A, *A2, *B, *B2;
    int64_t lda, ldb;
    const int32_t *ag, *bg, *cs;
    uint16_t *C, *C2, *C3;
    int64_t ldc;
    const uint16_t* R; // STORE / DUAL_ACC, single problem: optional residual [M][ldr]
    int64_t ldr;
    const uint16_t *Gin, *Uin;
    int64_t ldg;
    uint16_t *Ct, *Ct2, *Ct3; // SWIGLU_BWD: neuron-major (transposed) copies [column or rank][ldct], optional
    int64_t ldct;
    const int32_t* crank; // encoded rank of every column, or null: every column is listed
    int tiles_m, tiles_n, ntot; // ntot = tiles of all problems of the launch
    int group_m, nbatch;
    int np0; // batched launches: > 0 = the first np0 problems share one B operand and the others another (see tile_of_shared)
    // batched launch (weight gradients): problem z uses Ab[z], Bb[z], Cb[z]
    const uint16_t *Ab[kMaxBatch], *Bb[kMaxBatch];
    uint16_t* Cb[kMaxBatch];
    // OP_DW_SPLIT: the depth is cut into ksplit ranges of ksteps steps; each (range, problem) is a "problem" of
    // the launch and leaves its fp32 partial sums in partial[range][problem][M][N]
    int ksplit, ksteps;
    float* partial;
    // OP_DW_TAIL: ids below n_head are whole tiles (a multiple of the CU count: the full rounds); the `tail` tiles of
    // the last round follow as tail x ksplit items, range after range, each leaving an fp32 tile in
    // partial[range][tail tile][BM][BN].  ntot counts tiles, not ids.
    int n_head, tail;
};

// two fp32 -> packed bf16, round to nearest even (the hardware's v_cvt_pk_bf16_f32)
__device__ inline uint32_t pack_bf16(float lo, float hi) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const bf16x2 v = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, v);
}
__device__ inline u32x2 pack4(float a, float b, float c, float d) { return u32x2{pack_bf16(a, b), pack_bf16(c, d)}; }
__device__ inline float lo_bf16(uint32_t w) { return __uint_as_float(w << 16); }
__device__ inline float hi_bf16(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// source of the chunks that lie beyond the depth of the matrices in a partial last step
__device__ __attribute__((aligned(256))) const uint32_t kZeroChunk[64] = {0};

// Tile order of a batched launch whose problems share B operands (the weight gradients: dG^T and dU^T against
// X^T, Act^T against dY^T).  Problems that share B are stacked into one matrix of (problems x tiles_m)
// tile-rows, and each such stack is walked like a single problem: group_m tile-rows at a time, down the rows
// first, then along the tile-columns.  The tiles that run together on one XCD then touch fewer distinct operand
// rows than with the problems interleaved tile by tile.  Per depth range (ksplit > 1: OP_DW_SPLIT) there are two
// stacks, problems [0, np0) and the rest; the ranges follow one another.  `batch` returns range * nbatch + problem.
__host__ __device__ inline void tile_of_shared(int lin, int tiles_m, int tiles_n, int np0, int nbatch, int ksplit,
                                               int group_m, int& batch, int& tile_m, int& tile_n) {
    const int n0 = np0 * tiles_m * tiles_n, n1 = (nbatch - np0) * tiles_m * tiles_n;
    const int range = lin / (n0 + n1);
    lin -= range * (n0 + n1);
    int first_problem = 0, stack = np0;
    if (lin >= n0) lin -= n0, first_problem = np0, stack = nbatch - np0;
    const int rows = stack * tiles_m;
    const int per_group = group_m * tiles_n;
    const int grp = lin / per_group;
    const int first = grp * group_m;
    const int gm = rows - first < group_m ? rows - first : group_m;
    const int in = lin - grp * per_group;
    const int v = first + in % gm;
    tile_n = in / gm;
    batch = range * nbatch + first_problem + v / tiles_m;
    tile_m = v % tiles_m;
    (void)ksplit;
}

// Linear-order position (see the kernel's workgroup -> tile mapping) of id `id` of the full rounds, and of the q-th
// tile of the last round: XCD x owns positions [start_x, start_x + count_x), the first n_head / 8 of them run in
// the full rounds, the rest are its tail tiles; tail tiles are numbered round-robin over the XCDs.
__host__ __device__ inline int head_position(int id, int ntiles) {
    const int x = id % NUM_XCD, j = id / NUM_XCD, base = ntiles / NUM_XCD, rem = ntiles % NUM_XCD;
    return x * base + (x < rem ? x : rem) + j;
}
__host__ __device__ inline int tail_position(int q, int ntiles, int n_head) {
    const int base = ntiles / NUM_XCD, rem = ntiles % NUM_XCD, jh = n_head / NUM_XCD, tb = base - jh;
    const int x = q < NUM_XCD * tb ? q % NUM_XCD : q - NUM_XCD * tb;
    const int i = q < NUM_XCD * tb ? q / NUM_XCD : tb;
    return x * base + (x < rem ? x : rem) + jh + i;
}

// s_waitcnt vmcnt(n) alone (expcnt / lgkmcnt left at their maxima), gfx9 encoding
// s_waitcnt lgkmcnt(0) alone: this wave's LDS reads have returned
#define SDP_WAIT_LGKMCNT0() __builtin_amdgcn_s_waitcnt(15 | (7 << 4) | (0 << 8) | (3 << 14))
#define SDP_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (7 << 4) | (15 << 8) | (((n) >> 4) << 14))

template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI>
struct Geometry {
    static constexpr int NW = WAVES_M * WAVES_N;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    static constexpr int FM = WM / 32, FN = WN / 32;
    static constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
    static constexpr int RING = 2 * A_BYTES + 3 * B_BYTES; // two A stages, three B stages
    // epilogue strip: 32 rows x SW columns of bf16, rows padded by 8 bytes
    static constexpr int SW = EPI == EPI_SWIGLU_FWD ? WN / 2 : WN;
    static constexpr int RS = SW * 2 + 8;
    static constexpr int STRIP = 32 * RS;
    static constexpr int NSTRIP = EPI == EPI_SWIGLU_BWD ? 3 : 1; // strips per wave
    static constexpr int RANKTAB = EPI == EPI_SWIGLU_BWD ? SW * 4 : 0; // per wave: output row of each strip column
    static constexpr int WAVE_LDS = NSTRIP * STRIP + RANKTAB;
    static constexpr int LDS = RING > NW * WAVE_LDS ? RING : NW * WAVE_LDS;
    static_assert(LDS <= 160 * 1024, "LDS of one CU");
};

template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI, int OP>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64, 1) void sdp_gemm_kernel(Dev g) {
    using Geo = Geometry<BM, BN, WAVES_M, WAVES_N, EPI>;
    constexpr int NW = Geo::NW, WM = Geo::WM, WN = Geo::WN, FM = Geo::FM, FN = Geo::FN;
    constexpr int A_BYTES = Geo::A_BYTES, B_BYTES = Geo::B_BYTES;
    constexpr bool kFwd = EPI == EPI_SWIGLU_FWD;
    constexpr int SA = (BM / 8) / NW;  // A slabs (1 KB) per wave per step
    constexpr int SB = (BN / 8) / NW;  // B slabs per wave per step
    static_assert((BM / 8) % NW == 0 && (BN / 8) % NW == 0, "slabs must divide among the waves");
    static_assert(!kFwd || FN % 2 == 0, "gate/up fragments come in pairs");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6); // wave-uniform: keeps what derives from it scalar
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int l16 = lane & 15, lq = lane >> 4; // the MFMA's lane coordinates: index along the 16 rows, depth / output quarter

    // ---- workgroup -> (problem of the batch, tile), XCD-aware ----
    // Ids congruent mod 8 share an XCD: XCD x is given the contiguous range [start_x, start_x + count_x)
    // of a linear order in which the problems of a batch vary fastest, then group_m tile-rows, then the
    // tile-columns: the tiles that run together on one XCD then form a compact block of (problems x
    // tile-rows x tile-columns) whose operand rows are fetched into that XCD's L2 once.
    constexpr bool kTail = OP == OP_DW_TAIL;
    int bid = blockIdx.x;
    bool cut = false;  // OP_DW_TAIL: this workgroup computes one depth range of a tile of the last round
    int tail_part = 0, tail_q = 0;
    if (kTail && bid >= g.n_head) {
        cut = true;
        tail_part = (bid - g.n_head) / g.tail, tail_q = (bid - g.n_head) % g.tail;
        bid = tail_position(tail_q, g.ntot, g.n_head);
    } else {
        bid = head_position(bid, g.ntot);
    }
    constexpr bool kBatched = OP == OP_DW || OP == OP_DW_SPLIT || kTail;
    constexpr bool kSplit = OP == OP_DW_SPLIT;
    const int nb = kBatched ? g.nbatch * (kSplit ? g.ksplit : 1) : 1;
    int tile_m, tile_n, batch;
    if (kBatched && g.np0 > 0) {
        tile_of_shared(bid, g.tiles_m, g.tiles_n, g.np0, g.nbatch, g.ksplit, g.group_m, batch, tile_m, tile_n);
    } else {
        const int per_group = g.group_m * g.tiles_n * nb;
        const int grp = bid / per_group;
        const int first_m = grp * g.group_m;
        const int gm = g.tiles_m - first_m < g.group_m ? g.tiles_m - first_m : g.group_m;
        int in = bid - grp * per_group;
        batch = in % nb;
        in /= nb;
        tile_m = first_m + in % gm;
        tile_n = in / gm;
    }
    const uint16_t* gA = g.A;
    const uint16_t* gB = g.B;
    uint16_t* gC = g.C;
    int kpart = 0; // depth range of this workgroup (OP_DW_SPLIT, and the cut tiles of OP_DW_TAIL)
    if (kSplit) kpart = batch / g.nbatch, batch -= kpart * g.nbatch;
    if (kTail) kpart = tail_part;
    if (kBatched) {
        // selected by comparisons: a runtime index into a by-value kernel argument would go through scratch
        static_assert(kMaxBatch == 4, "one comparison per problem");
        gA = batch == 0 ? g.Ab[0] : (batch == 1 ? g.Ab[1] : (batch == 2 ? g.Ab[2] : g.Ab[3]));
        gB = batch == 0 ? g.Bb[0] : (batch == 1 ? g.Bb[1] : (batch == 2 ? g.Bb[2] : g.Bb[3]));
        gC = batch == 0 ? g.Cb[0] : (batch == 1 ? g.Cb[1] : (batch == 2 ? g.Cb[2] : g.Cb[3]));
    }
    const int m0 = tile_m * BM;
    const int n0 = kFwd ? tile_n * (BN / 2) : tile_n * BN; // SWIGLU_FWD: BN columns = BN/2 neurons x {gate, up}
    // SWIGLU_BWD with neuron-major copies: the encoded rank of each of this wave's output columns (at most two
    // per lane), fetched now so that the epilogue does not wait for it; a column outside the matrix counts as
    // not listed
    int crank_pre[2] = {-1, -1};
    if (EPI == EPI_SWIGLU_BWD && g.Ct) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int c = n0 + Geo::WN * wn + 64 * h + lane;
            if (64 * h < Geo::WN && c < g.N) crank_pre[h] = g.crank ? g.crank[c] : c;
        }
    }

    // ---- depth steps; a partial last step (K % 64 in {16, 32, 48}) reads its missing chunks from a
    // zero buffer, so that every step issues the same loads and runs all four MFMA sub-steps ----
    const int nk_all = (g.K + BK - 1) / BK;
    const bool ranged = kSplit || (kTail && cut);
    const int kt0 = ranged ? kpart * g.ksteps : 0; // first depth step of this workgroup
    const int nk1 = ranged ? (nk_all - kt0 < g.ksteps ? nk_all - kt0 : g.ksteps) : nk_all;
    const int nk = EPI == EPI_DUAL_ACC ? 2 * nk1 : nk1;

    // ---- per-lane global source of every slab this wave fills: byte offsets from a uniform base.
    // Row indices beyond the matrix are clamped to the last valid one: such lanes fetch valid
    // memory whose products only reach outputs that are never stored.
    // Slab s holds tile rows 8s .. 8s+7; lane -> row 8s + lane/8, stored chunk position lane%8.
    uint32_t a_off[SA], b_off[SB];
    int a_k[SA], b_k[SB]; // depth offset of this lane's chunk inside a step
#pragma unroll
    for (int i = 0; i < SA; ++i) {
        const int r = 8 * (wave + NW * i) + (lane >> 3);
        const int c = (lane & 7) ^ ((r >> 1) & 7);
        int m = m0 + r;
        m = m < g.M ? m : g.M - 1;
        const int64_t arow = g.ag ? g.ag[m] : m;
        a_off[i] = (uint32_t)((arow * g.lda + c * 8) * 2);
        a_k[i] = c * 8;
    }
#pragma unroll
    for (int i = 0; i < SB; ++i) {
        const int r = 8 * (wave + NW * i) + (lane >> 3);
        const int c = (lane & 7) ^ ((r >> 1) & 7);
        int n = kFwd ? n0 + (r % (BN / 2)) : n0 + r;
        n = n < g.N ? n : g.N - 1;
        const int64_t row = g.bg ? g.bg[n] : n;
        b_off[i] = (uint32_t)((row * g.ldb + c * 8) * 2);
        b_k[i] = c * 8;
    }

    // LDS: two A stages, then a ring of three B stages
    unsigned char* const lds_a = smem;
    unsigned char* const lds_b = smem + 2 * A_BYTES;

    // loads [first, last) of the SA (resp. SB) slabs of depth step kt; TAIL: K % 64 != 0
    auto issue_a = [&](int kt, auto tail_c, int first, int last) {
        constexpr bool TAIL = decltype(tail_c)::value;
        const bool second = EPI == EPI_DUAL_ACC && kt >= nk1;
        const int k0 = (kt0 + (second ? kt - nk1 : kt)) * BK;
        const int krem = g.K - k0;
        unsigned char* sa = lds_a + (kt & 1) * A_BYTES;
        const unsigned char* abase = (const unsigned char*)(second ? g.A2 : gA) + (int64_t)k0 * 2;
#pragma unroll
        for (int i = 0; i < SA; ++i) {
            if (i < first || i >= last) continue;
            const unsigned char* src = abase + a_off[i];
            if (TAIL && a_k[i] >= krem) src = (const unsigned char*)kZeroChunk;
            __builtin_amdgcn_global_load_lds((glb_void_ptr)src, (lds_void_ptr)(sa + (wave + NW * i) * 1024), 16, 0, 0);
        }
    };
    auto issue_b = [&](int kt, int slot, auto tail_c, int first, int last) {
        constexpr bool TAIL = decltype(tail_c)::value;
        const bool second = EPI == EPI_DUAL_ACC && kt >= nk1;
        const int k0 = (kt0 + (second ? kt - nk1 : kt)) * BK;
        const int krem = g.K - k0;
        unsigned char* sb = lds_b + slot * B_BYTES;
        const unsigned char* bbase0 = (const unsigned char*)(second ? g.B2 : gB) + (int64_t)k0 * 2;
        const unsigned char* bbase1 = (const unsigned char*)g.B2 + (int64_t)k0 * 2;
#pragma unroll
        for (int i = 0; i < SB; ++i) {
            if (i < first || i >= last) continue;
            // SWIGLU_FWD: tile rows BN/2.. hold the up-projection rows (second matrix)
            const bool up = kFwd && 8 * (wave + NW * i) >= BN / 2;
            const unsigned char* src = (up ? bbase1 : bbase0) + b_off[i];
            if (TAIL && b_k[i] >= krem) src = (const unsigned char*)kZeroChunk;
            __builtin_amdgcn_global_load_lds((glb_void_ptr)src, (lds_void_ptr)(sb + (wave + NW * i) * 1024), 16, 0, 0);
        }
    };

    // Accumulators: the wave's WM x WN outputs as 16 x 16 tiles of v_mfma_f32_16x16x32_bf16, grouped by 32 x 32
    // blocks (i, j): acc[i][j][q] is the tile with rows 32 i + 16 (q >> 1) .. and columns 32 j + 16 (q & 1) ..
    // (the 16 x 16 x 32 form sustains a higher clock than 32 x 32 x 16 on random operands: the same flops draw
    // less power)
    f32x4 acc[FM][FN][4];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[i][j][q] = f32x4{0.f, 0.f, 0.f, 0.f};

    // B tile row where fragment j of this wave starts (wave-uniform)
    int bfrag[FN];
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        if (kFwd)
            bfrag[j] = (j & 1) * (BN / 2) + (WN / 2) * wn + 32 * (j >> 1);
        else
            bfrag[j] = WN * wn + 32 * j;
    }

    // ---- LDS read addresses.  Everything that depends on the lane is folded into a few byte
    // offsets; fragment index, depth sub-step and stage only add compile-time constants.
    // row tile: chunk (r, c) at r*8 + (c ^ ((r >> 1) & 7)); for r = base + lane%16 with base a
    // multiple of 16 the XOR term is (lane%16 >> 1) & 7 for every fragment.  A fragment is 16 rows x 32 depth:
    // lane (l16, lq) takes row l16, depth chunk 4 s + lq of the 32-deep sub-step s; the 16 lanes of one lq hit
    // every 16-byte slot of a 256-byte bank row once.
    int row_off[BK / 32];
#pragma unroll
    for (int s = 0; s < BK / 32; ++s) row_off[s] = (((4 * s + lq) ^ ((l16 >> 1) & 7)) * 16) + l16 * 128;
    const int a_base = WM * wm * 128;

    // fragments of sub-step s: fa[2 i + h] = rows 32 i + 16 h .. of the wave's A rows, fb[2 j + w] likewise for B
    auto read_frags = [&](const unsigned char* sa, const unsigned char* sb, int s, bf16x8 (&fa)[2 * FM], bf16x8 (&fb)[2 * FN]) {
#pragma unroll
        for (int i = 0; i < 2 * FM; ++i)
            fa[i] = __builtin_bit_cast(bf16x8, *(const u32x4*)(sa + a_base + i * 16 * 128 + row_off[s]));
#pragma unroll
        for (int j = 0; j < 2 * FN; ++j)
            fb[j] = __builtin_bit_cast(bf16x8, *(const u32x4*)(sb + (bfrag[j >> 1] + 16 * (j & 1)) * 128 + row_off[s]));
    };
    // B fragment first: the accumulator tile is then indexed [n][m] in the MFMA's own layout, i.e. lane (l16, lq)
    // holds, for output row m = l16 of the tile, its columns n = 4 lq + r in element r.
    auto mfma_step = [&](const bf16x8 (&fa)[2 * FM], const bf16x8 (&fb)[2 * FN]) {
#pragma unroll
        for (int i = 0; i < 2 * FM; ++i)
#pragma unroll
            for (int j = 0; j < 2 * FN; ++j) {
                f32x4& c = acc[i >> 1][j >> 1][2 * (i & 1) + (j & 1)];
                c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fa[i], c, 0, 0, 0);
            }
    };

    // ---- main loop: two wave groups in alternating phases.
    // Group 0 = the first half of the waves, group 1 = the second half; the hardware places wave w of
    // a workgroup on SIMD w % 4, so every SIMD holds one wave of each group.  A depth step is cut into
    // two 32-deep halves.  Each wave alternates a READ phase (the 2 (FM + FN) fragment
    // reads of one half from LDS, plus its share of the direct loads of later steps) with a COMPUTE
    // phase (the 4 FM FN MFMAs of that half, at raised priority), and the two groups are one phase
    // apart: while one wave of a SIMD computes, the other one reads.  One wave alone keeps the matrix
    // core busy, so the MFMA stream never waits for LDS or for the load unit.  Every phase ends with a
    // workgroup barrier (plain s_barrier: the waits it needs are stated explicitly, and loads of later
    // steps stay in flight across it).
    //   phase 4 k     : group 0 reads (k, half 0), issues the loads of A for step k + 1
    //   phase 4 k + 1 : group 0 computes (k, 0);  group 1 reads (k, 0), issues A(k + 1)
    //   phase 4 k + 2 : group 0 reads (k, 1), issues the loads of B for step k + 2;  group 1 computes (k, 0)
    //   phase 4 k + 3 : group 0 computes (k, 1);  group 1 reads (k, 1), issues B(k + 2)
    // A has two LDS stages and B three.  Stage contents of step k are read in phases 4 k .. 4 k + 3;
    // loads into the stages of step k - 1 are issued from phase 4 k on, after the barrier that ends
    // phase 4 k - 1, before which every wave has waited for its own LDS reads.  Before that same
    // barrier every wave waits until its loads for step k have landed (loads complete in issue
    // order; only the newest SB, B of step k + 1, may still be in flight).
    const int grp = wave / (NW / 2);
    bf16x8 fa[2 * FM], fb[2 * FN];
    auto read_half = [&](const unsigned char* sa, const unsigned char* sb, int h) { read_frags(sa, sb, h, fa, fb); };
    auto compute_half = [&]() {
        __builtin_amdgcn_s_setprio(1);
        mfma_step(fa, fb);
        __builtin_amdgcn_s_setprio(0);
    };
    auto phase_end = [&]() {
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    };
    auto step = [&](int kt, int slot, auto ia_c, auto ib_c, auto tail_c) {
        constexpr bool IA = decltype(ia_c)::value; // step kt + 1 exists
        constexpr bool IB = decltype(ib_c)::value; // step kt + 2 exists
        const unsigned char* sa = lds_a + (kt & 1) * A_BYTES;
        const unsigned char* sb = lds_b + slot * B_BYTES;
        const int slot2 = slot == 0 ? 2 : slot - 1; // (kt + 2) % 3
        // READ (kt, 0)
        read_half(sa, sb, 0);
        if (IA) issue_a(kt + 1, tail_c, 0, SA);
        SDP_WAIT_LGKMCNT0();
        phase_end();
        // COMPUTE (kt, 0)
        compute_half();
        phase_end();
        // READ (kt, 1)
        read_half(sa, sb, 1);
        if (IB) issue_b(kt + 2, slot2, tail_c, 0, SB);
        SDP_WAIT_LGKMCNT0();
        if (grp == 1) {
            if (IB) SDP_WAIT_VMCNT(SB); else SDP_WAIT_VMCNT(0);
        }
        phase_end();
        // COMPUTE (kt, 1)
        compute_half();
        if (grp == 0) {
            if (IB) SDP_WAIT_VMCNT(SB); else SDP_WAIT_VMCNT(0);
        }
        phase_end();
    };
    auto run = [&](auto tail_c) {
        issue_a(0, tail_c, 0, SA);
        issue_b(0, 0, tail_c, 0, SB);
        if (nk > 1) {
            issue_b(1, 1, tail_c, 0, SB);
            SDP_WAIT_VMCNT(SB);
        } else {
            SDP_WAIT_VMCNT(0);
        }
        phase_end();
        if (grp == 1) phase_end(); // group 1 runs one phase behind
        int slot = 0;
        int kt = 0;
        for (; kt + 2 < nk; ++kt) {
            step(kt, slot, std::true_type{}, std::true_type{}, tail_c);
            slot = slot == 2 ? 0 : slot + 1;
        }
        if (kt + 1 < nk) {
            step(kt, slot, std::true_type{}, std::false_type{}, tail_c);
            slot = slot == 2 ? 0 : slot + 1;
            ++kt;
        }
        step(kt, slot, std::false_type{}, std::false_type{}, tail_c);
        if (grp == 0) phase_end();
    };
    if (g.K % BK == 0) run(std::false_type{}); else run(std::true_type{});

    // ================================ epilogue ================================
    // acc[i][j][q][r] = C(m, n),  m = m0 + WM wm + 32 i + 16 (q >> 1) + l16,
    //                             n = n0 + (column base of block j) + 16 (q & 1) + 4 lq + r.
    if constexpr (kSplit) {
        // fp32 partial sums of this depth range, 16 bytes (4 columns) per store; N % 8 == 0
        float* P = g.partial + ((int64_t)kpart * g.nbatch + batch) * g.M * g.N;
#pragma unroll
        for (int i = 0; i < FM; ++i) {
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int m = m0 + WM * wm + 32 * i + 16 * (q >> 1) + l16;
                    const int n = n0 + WN * wn + 32 * j + 16 * (q & 1) + 4 * lq;
                    if (m < g.M && n < g.N) *(f32x4*)(P + (int64_t)m * g.N + n) = acc[i][j][q];
                }
        }
        return;
    }
    if constexpr (kTail) {
        if (cut) {
            // fp32 partial tile of this depth range, tile-local [BM][BN]; rows and columns outside the matrix hold
            // what the clamped operand rows gave and are never read back
            float* P = g.partial + ((int64_t)tail_part * g.tail + tail_q) * (BM * BN);
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        *(f32x4*)(P + (WM * wm + 32 * i + 16 * (q >> 1) + l16) * BN + WN * wn + 32 * j + 16 * (q & 1) + 4 * lq) =
                            acc[i][j][q];
            return;
        }
    }
    __syncthreads(); // all waves are done with the operand tiles: LDS becomes per-wave strips
    constexpr int SW = Geo::SW, RS = Geo::RS;
    constexpr int CPR = SW / 8;               // 16-byte chunks per strip row
    constexpr int NCH = 32 * CPR;             // chunks per strip
    unsigned char* strip0 = smem + wave * Geo::WAVE_LDS;
    const int wcol0 = kFwd ? n0 + (WN / 2) * wn : n0 + WN * wn; // first output column of this wave's strips

    // one packed 8-byte group of a strip (this lane's 4 columns of tile q of a 32 x 32 block): row 16 (q >> 1) + l16,
    // columns cbase + 16 (q & 1) + 4 lq ..
    auto strip_put = [&](unsigned char* strip, int cbase, int q, u32x2 v) {
        *(u32x2*)(strip + (16 * (q >> 1) + l16) * RS + (cbase + 16 * (q & 1) + 4 * lq) * 2) = v;
    };
    auto strip_get = [&](const unsigned char* strip, int cbase, int q) {
        return *(const u32x2*)(strip + (16 * (q >> 1) + l16) * RS + (cbase + 16 * (q & 1) + 4 * lq) * 2);
    };
    // Global accesses of the epilogue go through buffer resources whose base is this wave's corner of the tile and
    // whose extent ends with the matrix's last row: for an offset at or beyond the extent the hardware returns zero
    // to a load and drops a store.  A lane whose columns lie outside the matrix (or whose row is dropped) is given
    // such an offset.  The accesses are then unconditional instructions, so the count of those in flight is known
    // and the wait for the next fragment row's loads leaves this row's stores in flight (behind a branch per store
    // the wait would be for everything).  Offsets inside a wave's part stay below 2^30 (see gemm_mfma_supported).
    constexpr uint32_t kOutside = 0x80000000u;
    const int wrow0 = m0 + WM * wm; // first output row of this wave
    const int wrows = g.M - wrow0 < 0 ? 0 : (g.M - wrow0 > WM ? WM : g.M - wrow0); // its rows inside the matrix
    // the base is the same in all lanes; saying so keeps the resource in scalar registers
    auto uniform_rsrc = [](const uint16_t* base, uint32_t bytes) {
        const uint64_t a = (uint64_t)base;
        const uint64_t u = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(a >> 32)) << 32) |
                           (uint32_t)__builtin_amdgcn_readfirstlane((int)a);
        return __builtin_amdgcn_make_buffer_rsrc((void*)u, 0, (int)__builtin_amdgcn_readfirstlane((int)bytes), 0x00020000);
    };
    auto wave_rsrc = [&](const uint16_t* base, int64_t ld) {
        return uniform_rsrc(base + (int64_t)wrow0 * ld + wcol0, (uint32_t)(wrows * ld * 2));
    };
    // byte offset of chunk c of fragment row 0 (rows of leading dimension ld); fragment row i lies 64 i ld bytes on
    auto chunk_offset = [&](int c, int64_t ld) {
        const int row = c / CPR, cc = c % CPR;
        return (NCH % 64 == 0 || c < NCH) && wcol0 + cc * 8 < g.N ? (uint32_t)((row * ld + cc * 8) * 2) : kOutside;
    };
    // cache policy of an epilogue access: kStream marks data this kernel touches once (non-temporal), so that it
    // does not push the operand panels, which every tile of a row or column re-reads, out of the L2
    constexpr int kKeep = 0, kStream = 2;
    // strip -> global: rows of `out` (leading dimension ld)
    auto strip_store = [&](const unsigned char* strip, uint16_t* out, int64_t ld, int i, auto policy) {
        const __amdgpu_buffer_rsrc_t rs = wave_rsrc(out, ld);
#pragma unroll
        for (int it = 0; it < (NCH + 63) / 64; ++it) {
            const int c = NCH % 64 == 0 || it * 64 + lane < NCH ? it * 64 + lane : 0;
            const int row = c / CPR, cc = c % CPR;
            const u32x2 lo = *(const u32x2*)(strip + row * RS + cc * 16);
            const u32x2 hi = *(const u32x2*)(strip + row * RS + cc * 16 + 8);
            __builtin_amdgcn_raw_buffer_store_b128(u32x4{lo[0], lo[1], hi[0], hi[1]}, rs,
                                                   chunk_offset(it * 64 + lane, ld) + (uint32_t)(64 * i * ld), 0, decltype(policy)::value);
        }
    };
    // the same with a row scatter (a negative entry drops the row): destination rows may lie anywhere, plain stores
    auto strip_store_scatter = [&](const unsigned char* strip, uint16_t* out, int64_t ld, const int32_t* scatter, int i) {
#pragma unroll
        for (int it = 0; it < (NCH + 63) / 64; ++it) {
            const int c = it * 64 + lane;
            if (NCH % 64 != 0 && c >= NCH) break;
            const int row = c / CPR, cc = c % CPR;
            const u32x2 lo = *(const u32x2*)(strip + row * RS + cc * 16);
            const u32x2 hi = *(const u32x2*)(strip + row * RS + cc * 16 + 8);
            const int m = wrow0 + 32 * i + row, n = wcol0 + cc * 8;
            if (m < g.M && n < g.N) {
                const int64_t orow = scatter[m];
                if (orow >= 0) *(u32x4*)(out + orow * ld + n) = u32x4{lo[0], lo[1], hi[0], hi[1]};
            }
        }
    };
    // global -> registers -> strip: the same chunk mapping, zero outside the matrix.  The two halves are
    // separate so that the loads of fragment row i + 1 fly while row i is computed and stored.
    constexpr int NLD = (NCH + 63) / 64;
    auto strip_fetch = [&](u32x4 (&v)[NLD], const uint16_t* in, int64_t ld, int i, auto policy) {
        const __amdgpu_buffer_rsrc_t rs = wave_rsrc(in, ld);
#pragma unroll
        for (int it = 0; it < NLD; ++it)
            v[it] = __builtin_amdgcn_raw_buffer_load_b128(rs, chunk_offset(it * 64 + lane, ld) + (uint32_t)(64 * i * ld), 0,
                                                           decltype(policy)::value);
    };
    auto strip_commit = [&](unsigned char* strip, const u32x4 (&v)[NLD]) {
#pragma unroll
        for (int it = 0; it < NLD; ++it) {
            const int c = it * 64 + lane;
            if (NCH % 64 != 0 && c >= NCH) break;
            const int row = c / CPR, cc = c % CPR;
            *(u32x2*)(strip + row * RS + cc * 16) = u32x2{v[it][0], v[it][1]};
            *(u32x2*)(strip + row * RS + cc * 16 + 8) = u32x2{v[it][2], v[it][3]};
        }
    };

    // neuron-major copies: output row of each of this wave's SW strip columns, relative to trow0.  Without an
    // index list it is the column itself; with one (backward masking) it is the column's rank among the listed
    // columns, or -1 for columns that are not listed.  The encoded ranks were fetched before the main loop.
    int32_t* ranktab = (int32_t*)(strip0 + Geo::NSTRIP * Geo::STRIP);
    int trow0 = 0; // output row of the first (listed) column of this wave
    if (EPI == EPI_SWIGLU_BWD && g.Ct) {
        const int first = __builtin_amdgcn_readfirstlane(crank_pre[0]);
        trow0 = first >= 0 ? first : -1 - first;
#pragma unroll
        for (int h = 0; h < (SW + 63) / 64; ++h)
            if (SW % 64 == 0 || 64 * h + lane < SW) ranktab[64 * h + lane] = crank_pre[h] >= 0 ? crank_pre[h] - trow0 : -1;
    }
    // strip -> neuron-major global: out[trow0 + ranktab[column]][token].  A transposing LDS read hands the lanes
    // of a 16-lane block, for 4 adjacent strip columns, 4 consecutive rows each; two of them give every lane
    // 8 consecutive tokens of one column, i.e. one 16-byte store, and 4 lanes cover the 32 tokens (64 bytes).
    auto strip_store_t = [&](const unsigned char* strip, uint16_t* out, int i) {
        const int gi = lane >> 4, li = lane & 15, q = li >> 2, cn = li & 3;
        const int src_row = 8 * (li & 3) + (li >> 2); // as source lane: rows 8 q' + e for the lanes that receive from it
        const bool m_in = 32 * i + 8 * q < wrows;
        const __amdgpu_buffer_rsrc_t rs = uniform_rsrc(out + (int64_t)trow0 * g.ldct + wrow0, kOutside);
#pragma unroll
        for (int it = 0; it < SW / 16; ++it) {
            const int c4 = 16 * it + 4 * gi;
            const unsigned char* p = strip + src_row * RS + c4 * 2;
            const s16x4 h0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)p);
            const s16x4 h1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p + 4 * RS));
            const int row = ranktab[c4 + cn];
            const uint32_t off = row >= 0 && m_in ? (uint32_t)((row * g.ldct + 32 * i + 8 * q) * 2) : kOutside;
            const u32x2 a = __builtin_bit_cast(u32x2, h0), b = __builtin_bit_cast(u32x2, h1);
            __builtin_amdgcn_raw_buffer_store_b128(u32x4{a[0], a[1], b[0], b[1]}, rs, off, 0, kKeep); // read next, by the weight-gradient launch
        }
    };

    // residual of a single-problem store (the skip connection of a block): fetched one fragment row ahead like G, U
    constexpr bool kResidual = (EPI == EPI_STORE || EPI == EPI_DUAL_ACC) && !kBatched;
    u32x4 rpre[kResidual ? NLD : 1];
    const bool has_r = kResidual && g.R != nullptr;
    if constexpr (kResidual) {
        if (has_r) strip_fetch(rpre, g.R, g.ldr, 0, std::integral_constant<int, kKeep>{});
    }
    // The fragment rows, one after the other.  kT: SWIGLU_BWD with the neuron-major copies; the loop exists once
    // per case, so that between a row's loads and the next row's use of them the stores issued are the same on
    // every path and can be left in flight.
    auto rows = [&](auto with_t) __attribute__((always_inline)) {
        constexpr bool kT = decltype(with_t)::value;
        u32x4 gpre[NLD], upre[NLD]; // SWIGLU_BWD: G and U of the next fragment row, in flight
        if (EPI == EPI_SWIGLU_BWD) {
            strip_fetch(gpre, g.Gin, g.ldg, 0, std::integral_constant<int, kStream>{});
            strip_fetch(upre, g.Uin, g.ldg, 0, std::integral_constant<int, kStream>{});
        }
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            // keep the scheduler from pulling later fragment rows' work (and its registers) up here
            __builtin_amdgcn_sched_barrier(0);
            if (EPI == EPI_STORE || EPI == EPI_DUAL_ACC) {
                if constexpr (kResidual) {
                    if (has_r) {
                        // row chunks -> strip -> each lane's own accumulator positions; added in fp32
                        strip_commit(strip0, rpre);
                        if (i + 1 < FM) strip_fetch(rpre, g.R, g.ldr, i + 1, std::integral_constant<int, kKeep>{});
                        u32x2 rq[FN][4];
#pragma unroll
                        for (int j = 0; j < FN; ++j)
#pragma unroll
                            for (int q = 0; q < 4; ++q) rq[j][q] = strip_get(strip0, 32 * j, q);
#pragma unroll
                        for (int j = 0; j < FN; ++j)
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                acc[i][j][q][0] += lo_bf16(rq[j][q][0]);
                                acc[i][j][q][1] += hi_bf16(rq[j][q][0]);
                                acc[i][j][q][2] += lo_bf16(rq[j][q][1]);
                                acc[i][j][q][3] += hi_bf16(rq[j][q][1]);
                            }
                    }
                }
#pragma unroll
                for (int j = 0; j < FN; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        strip_put(strip0, 32 * j, q,
                                  pack4(acc[i][j][q][0], acc[i][j][q][1], acc[i][j][q][2], acc[i][j][q][3]));
                if (g.cs) strip_store_scatter(strip0, gC, g.ldc, g.cs, i); else strip_store(strip0, gC, g.ldc, i, std::integral_constant<int, kKeep>{});
            } else if (EPI == EPI_SWIGLU_FWD) {
                // fragments 2 jj (gate) and 2 jj + 1 (up) cover the same 32 neurons
#pragma unroll
                for (int which = 0; which < 3; ++which) {
#pragma unroll
                    for (int jj = 0; jj < FN / 2; ++jj)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            float v[4];
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                const float gv = acc[i][2 * jj][q][r], uv = acc[i][2 * jj + 1][q][r];
                                v[r] = which == 0 ? gv : (which == 1 ? uv : swiglu_fwd<false>(gv, uv));
                            }
                            strip_put(strip0, 32 * jj, q, pack4(v[0], v[1], v[2], v[3]));
                        }
                    strip_store(strip0, which == 0 ? g.C : (which == 1 ? g.C2 : g.C3), g.ldc, i, std::integral_constant<int, kKeep>{});
                }
            } else { // EPI_SWIGLU_BWD: three strips per wave (dG, dU, Act)
                unsigned char* strip1 = strip0 + Geo::STRIP;
                unsigned char* strip2 = strip1 + Geo::STRIP;
                strip_commit(strip0, gpre);
                strip_commit(strip1, upre);
                if (i + 1 < FM) {
                    strip_fetch(gpre, g.Gin, g.ldg, i + 1, std::integral_constant<int, kStream>{});
                    strip_fetch(upre, g.Uin, g.ldg, i + 1, std::integral_constant<int, kStream>{});
                }
                u32x2 gq[FN][4], uq[FN][4];
#pragma unroll
                for (int j = 0; j < FN; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        gq[j][q] = strip_get(strip0, 32 * j, q);
                        uq[j][q] = strip_get(strip1, 32 * j, q);
                    }
#pragma unroll
                for (int j = 0; j < FN; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        float dg[4], du[4], act[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const uint32_t gw = gq[j][q][r >> 1], uw = uq[j][q][r >> 1];
                            const float gv = (r & 1) ? hi_bf16(gw) : lo_bf16(gw);
                            const float uv = (r & 1) ? hi_bf16(uw) : lo_bf16(uw);
                            swiglu_bwd<false>(acc[i][j][q][r], gv, uv, dg[r], du[r], act[r]);
                        }
                        strip_put(strip0, 32 * j, q, pack4(dg[0], dg[1], dg[2], dg[3]));
                        strip_put(strip1, 32 * j, q, pack4(du[0], du[1], du[2], du[3]));
                        strip_put(strip2, 32 * j, q, pack4(act[0], act[1], act[2], act[3]));
                    }
                strip_store(strip0, g.C, g.ldc, i, std::integral_constant<int, kStream>{});
                strip_store(strip1, g.C2, g.ldc, i, std::integral_constant<int, kStream>{});
                if (g.C3) strip_store(strip2, g.C3, g.ldc, i, std::integral_constant<int, kStream>{});
                if constexpr (kT) {
                    strip_store_t(strip0, g.Ct, i);
                    strip_store_t(strip1, g.Ct2, i);
                    strip_store_t(strip2, g.Ct3, i);
                }
            }
        }
    };
    if constexpr (EPI == EPI_SWIGLU_BWD) {
        if (g.Ct) rows(std::true_type{}); else rows(std::false_type{});
    } else {
        rows(std::false_type{});
    }
}

constexpr int kNumCU = 256;

// Overrides of the tile shape and order for tuning runs.  The library's behaviour is a pure function of its
// arguments: the environment is consulted only in a build with -DSDP_TUNING_SWITCHES (never the shipped one),
// once per process, and values outside the accepted sets are ignored.
struct Tuning {
    int force_tile = 0; // 0 = choose; 128 / 192 / 256
    int group_m = 0;    // 0 = choose
    bool plain_order = false;
    int tail_parts = -1; // SDP_TAIL_PARTS: -1 = choose; 0 = no tail cut; n = cut into n ranges where a cut applies
};
const Tuning& tuning() {
    static const Tuning t = [] {
        Tuning v;
#ifdef SDP_TUNING_SWITCHES
        if (const char* e = getenv("SDP_FORCE_TILE")) {
            const int f = atoi(e);
            if (f == 128 || f == 192 || f == 256) v.force_tile = f;
        }
        if (const char* e = getenv("SDP_GROUP_M")) v.group_m = atoi(e) > 0 ? atoi(e) : 0;
        v.plain_order = getenv("SDP_PLAIN_ORDER") != nullptr;
        if (const char* e = getenv("SDP_TAIL_PARTS")) v.tail_parts = atoi(e) >= 0 && atoi(e) <= 8 ? atoi(e) : -1;
#endif
        return v;
    }();
    return t;
}

// Tile-rows per group of the workgroup -> tile order: the tiles resident on one XCD at a time (its
// share of the launch, at most one per CU) form a block of nbatch x group_m x columns; pick the
// group_m for which that block touches the fewest distinct operand rows (A rows weigh na operands,
// B rows nb), i.e. the least traffic into that XCD's L2.
int choose_group_m(int tiles_m, int tiles_n, int nbatch, int na, int nb, int bm, int bn) {
    const int64_t ntot = (int64_t)tiles_m * tiles_n * nbatch;
    const int per_xcd = kNumCU / NUM_XCD;
    int64_t c = (ntot + NUM_XCD - 1) / NUM_XCD;
    if (c > per_xcd) c = per_xcd;
    int best = 1;
    int64_t best_cost = -1;
    for (int gm = 1; gm <= tiles_m && gm <= per_xcd; ++gm) {
        const int64_t cols = (c + (int64_t)nbatch * gm - 1) / ((int64_t)nbatch * gm); // tile-columns the block needs
        const int64_t groups = (cols + tiles_n - 1) / tiles_n;
        const int64_t ncols = cols < tiles_n ? cols : tiles_n;
        const int64_t cost = (int64_t)na * gm * groups * bm + (int64_t)nb * ncols * bn;
        if (best_cost < 0 || cost < best_cost) best_cost = cost, best = gm;
    }
    return best;
}

// group_m of the stacked order (tile_of_shared): the one whose first round of resident tiles (each XCD's range,
// at most one tile per CU) touches the fewest operand bytes, counted by walking that very order.
int choose_group_shared(int tiles_m, int tiles_n, int np0, int nbatch, int ksplit, int bm, int bn) {
    // the walk costs a fraction of a millisecond of host time: remembered per shape
    static std::mutex mu;
    static std::map<std::array<int, 7>, int> known;
    const std::array<int, 7> key = {tiles_m, tiles_n, np0, nbatch, ksplit, bm, bn};
    {
        std::lock_guard<std::mutex> lk(mu);
        auto it = known.find(key);
        if (it != known.end()) return it->second;
    }
    const int ntot = tiles_m * tiles_n * nbatch * ksplit;
    const int per_xcd = kNumCU / NUM_XCD;
    const int max_rows = (np0 > nbatch - np0 ? np0 : nbatch - np0) * tiles_m;
    int best = 1;
    int64_t best_cost = -1;
    std::vector<char> seen_a((size_t)ksplit * nbatch * tiles_m), seen_b((size_t)ksplit * 2 * tiles_n);
    for (int gm = 1; gm <= max_rows && gm <= 2 * per_xcd; ++gm) {
        int64_t cost = 0;
        for (int x = 0; x < NUM_XCD; ++x) {
            const int base = ntot / NUM_XCD, rem = ntot % NUM_XCD;
            const int start = x * base + (x < rem ? x : rem);
            int count = base + (x < rem ? 1 : 0);
            count = count < per_xcd ? count : per_xcd;
            std::fill(seen_a.begin(), seen_a.end(), 0);
            std::fill(seen_b.begin(), seen_b.end(), 0);
            for (int lin = start; lin < start + count; ++lin) {
                int b, tm, tn;
                tile_of_shared(lin, tiles_m, tiles_n, np0, nbatch, ksplit, gm, b, tm, tn);
                const int range = b / nbatch, z = b % nbatch; // a depth range reads its own part of every row
                char& a = seen_a[(size_t)b * tiles_m + tm];
                char& bb = seen_b[((size_t)range * 2 + (z < np0 ? 0 : 1)) * tiles_n + tn];
                if (!a) a = 1, cost += bm;
                if (!bb) bb = 1, cost += bn;
            }
        }
        if (best_cost < 0 || cost < best_cost) best_cost = cost, best = gm;
    }
    std::lock_guard<std::mutex> lk(mu);
    known[key] = best;
    return best;
}

// last launch configuration per call-site name, kept only while per-kernel timing is on (sdp_profile_launch_shape)
std::mutex g_shape_mu;
std::map<std::string, std::array<int, 4>> g_last_shape;

// OP_DW_TAIL, second kernel: the depth ranges' fp32 tiles of every tile of the last round, added in range order,
// rounded and stored (optional row scatter).  One thread per 8 columns of a tile row; the tile's place in its
// problem comes from the same mapping as in the contraction kernel.
struct TailReduceArgs {
    const float* partial;
    int parts, tail, ntiles, n_head;
    int tiles_m, tiles_n, np0, nbatch, group_m;
    int M, N;
    uint16_t* Cb[kMaxBatch];
    int64_t ldc;
    const int32_t* cs;
};
template <int BM, int BN>
__global__ __launch_bounds__(256) void tail_reduce_kernel(TailReduceArgs r) {
    constexpr int PER_TILE = BM * BN / 8 / 256; // workgroups per tile
    const int q = blockIdx.x / PER_TILE;
    const int e = (blockIdx.x % PER_TILE) * 256 + threadIdx.x;
    const int row = e / (BN / 8), col = (e % (BN / 8)) * 8;
    const int bid = tail_position(q, r.ntiles, r.n_head);
    int batch, tile_m, tile_n;
    if (r.np0 > 0) {
        tile_of_shared(bid, r.tiles_m, r.tiles_n, r.np0, r.nbatch, 1, r.group_m, batch, tile_m, tile_n);
    } else {
        const int per_group = r.group_m * r.tiles_n * r.nbatch;
        const int grp = bid / per_group;
        const int first_m = grp * r.group_m;
        const int gm = r.tiles_m - first_m < r.group_m ? r.tiles_m - first_m : r.group_m;
        int in = bid - grp * per_group;
        batch = in % r.nbatch;
        in /= r.nbatch;
        tile_m = first_m + in % gm;
        tile_n = in / gm;
    }
    const int m = tile_m * BM + row, n = tile_n * BN + col;
    if (m >= r.M || n >= r.N) return;
    f32x4 a = {0.f, 0.f, 0.f, 0.f}, b = a;
    for (int k = 0; k < r.parts; ++k) { // ranges in depth order
        const float* p = r.partial + ((int64_t)k * r.tail + q) * (BM * BN) + row * BN + col;
        a += *(const f32x4*)p;
        b += *(const f32x4*)(p + 4);
    }
    uint16_t* out = batch == 0 ? r.Cb[0] : (batch == 1 ? r.Cb[1] : (batch == 2 ? r.Cb[2] : r.Cb[3]));
    const int64_t orow = r.cs ? r.cs[m] : m;
    if (orow < 0) return; // dropped row
    *(u32x4*)(out + orow * r.ldc + n) = u32x4{pack_bf16(a[0], a[1]), pack_bf16(a[2], a[3]), pack_bf16(b[0], b[1]), pack_bf16(b[2], b[3])};
}

template <int BM, int BN>
int tail_reduce(const Dev& g, const GemmDesc& d, hipStream_t s) {
    TailReduceArgs r{g.partial, g.ksplit, g.tail, g.ntot, g.n_head, g.tiles_m, g.tiles_n, g.np0, g.nbatch, g.group_m,
                     g.M, g.N, {}, g.ldc, g.cs};
    for (int z = 0; z < kMaxBatch; ++z) r.Cb[z] = g.Cb[z];
    ProfileScope ps(d.tail_name, s);
    tail_reduce_kernel<BM, BN><<<(unsigned)(g.tail * (BM * BN / 8 / 256)), 256, 0, s>>>(r);
    return launch_status();
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI, int OP>
int launch_cfg(const GemmDesc& d, hipStream_t s) {
    using Geo = Geometry<BM, BN, WAVES_M, WAVES_N, EPI>;
    constexpr int NTHREADS = WAVES_M * WAVES_N * 64;
    constexpr int LDS = Geo::LDS;
    Dev g;
    g.M = d.M, g.N = d.N, g.K = d.K;
    g.A = (const uint16_t*)d.A, g.A2 = (const uint16_t*)d.A2, g.B = (const uint16_t*)d.B, g.B2 = (const uint16_t*)d.B2;
    g.lda = d.lda, g.ldb = d.ldb, g.ag = d.a_gather, g.bg = d.b_gather, g.cs = d.c_scatter;
    g.C = (uint16_t*)d.C, g.C2 = (uint16_t*)d.C2, g.C3 = (uint16_t*)d.C3, g.ldc = d.ldc;
    g.R = (const uint16_t*)d.R, g.ldr = d.ldr;
    g.Gin = (const uint16_t*)d.Gin, g.Uin = (const uint16_t*)d.Uin, g.ldg = d.ldg;
    g.Ct = (uint16_t*)d.Ct, g.Ct2 = (uint16_t*)d.Ct2, g.Ct3 = (uint16_t*)d.Ct3, g.ldct = d.ldct;
    g.crank = d.crank;
    g.tiles_m = (d.M + BM - 1) / BM;
    const int ncols = EPI == EPI_SWIGLU_FWD ? BN / 2 : BN;
    g.tiles_n = (d.N + ncols - 1) / ncols;
    const int64_t ntiles = (int64_t)g.tiles_m * g.tiles_n;
    constexpr bool kBatched = OP == OP_DW || OP == OP_DW_SPLIT || OP == OP_DW_TAIL;
    const int ksplit = OP == OP_DW_SPLIT ? d.ksplit : 1;
    const int nbatch = (kBatched ? d.nbatch : 1) * ksplit; // problems of the launch
    if (ntiles * nbatch > 0x7FFFFFFF) return SDP_ERR_SHAPE;
    g.ntot = (int)(ntiles * nbatch);
    g.nbatch = kBatched ? d.nbatch : 1;
    g.ksplit = OP == OP_DW_TAIL ? d.ksplit : ksplit;
    g.ksteps = ((d.K + BK - 1) / BK + g.ksplit - 1) / g.ksplit;
    g.partial = (float*)(OP == OP_DW_TAIL ? d.tail_ws : d.split_ws);
    g.n_head = g.ntot, g.tail = 0;
    int64_t grid = (int64_t)g.ntot;
    if (OP == OP_DW_TAIL) {
        g.n_head = g.ntot / kNumCU * kNumCU, g.tail = g.ntot - g.n_head;
        grid = (int64_t)g.n_head + (int64_t)g.tail * d.ksplit;
        if (g.tail < 1 || d.ksplit < 2 || !d.tail_ws || grid > 0x7FFFFFFF) return SDP_ERR_INVALID_ARG;
    }
    int na = 1, nbo = 1; // distinct A / B operands among the problems of a batch
    for (int z = 0; z < kMaxBatch; ++z) {
        g.Ab[z] = (const uint16_t*)d.Ab[z], g.Bb[z] = (const uint16_t*)d.Bb[z], g.Cb[z] = (uint16_t*)d.Cb[z];
    }
    if (kBatched) {
        na = nbo = 0;
        for (int z = 0; z < d.nbatch; ++z) {
            bool newa = true, newb = true;
            for (int y = 0; y < z; ++y) newa &= d.Ab[y] != d.Ab[z], newb &= d.Bb[y] != d.Bb[z];
            na += newa, nbo += newb;
        }
    }
    g.group_m = choose_group_m(g.tiles_m, g.tiles_n, nbatch, na * ksplit, nbo * ksplit, BM, BN);
    g.np0 = 0;
    if (kBatched && d.nbatch > 1 && nbo <= 2 && !tuning().plain_order) {
        // problems that share B must be neighbours: [0, np0) on Bb[0], the rest on one other operand (or none)
        int np0 = 1;
        while (np0 < d.nbatch && d.Bb[np0] == d.Bb[0]) ++np0;
        bool ok = true;
        for (int z = np0; z < d.nbatch; ++z) ok = ok && d.Bb[z] == d.Bb[np0] && d.Bb[z] != d.Bb[0];
        if (ok) {
            g.np0 = np0;
            g.group_m = choose_group_shared(g.tiles_m, g.tiles_n, np0, d.nbatch, ksplit, BM, BN);
        }
    }
    if (tuning().group_m > 0) g.group_m = tuning().group_m;
    if (profiling_on() && d.name) {
        std::lock_guard<std::mutex> lk(g_shape_mu);
        g_last_shape[d.name] = {BM, BN, g.group_m, g.np0 > 0 ? 1 : 0};
    }
    auto kern = sdp_gemm_kernel<BM, BN, WAVES_M, WAVES_N, EPI, OP>;
    // once per instantiation (initialisation of a function-local static is thread-safe)
    static const hipError_t attr =
        hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    if (attr != hipSuccess) return SDP_ERR_HIP;
    // When this kernel is being timed, the launch itself carries the two events (their timestamps are the
    // kernel's own begin and end): events recorded around the launch would put a bubble of several
    // microseconds on either side of it.
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    if (profile_launch_events(d.name, &ev0, &ev1))
        hipExtLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NTHREADS), (uint32_t)LDS, s, ev0, ev1, 0u, g);
    else
        kern<<<dim3((unsigned)grid), NTHREADS, LDS, s>>>(g);
    const int rc = launch_status();
    if (OP == OP_DW_TAIL && rc == SDP_OK) return tail_reduce<BM, BN>(g, d, s);
    return rc;
}

// estimated time of a tile shape, in units of 256 x 256 tile-depths: rounds over the CUs times tile
// area, times a penalty for the smaller shapes' lower MFMA duty (more LDS traffic per flop).
double shape_cost(int M, int ncols_total, int nbatch, int bm, int bn, double penalty) {
    const int64_t tiles = (int64_t)((M + bm - 1) / bm) * ((ncols_total + bn - 1) / bn) * nbatch;
    const int64_t rounds = (tiles + kNumCU - 1) / kNumCU;
    return (double)rounds * bm * bn * penalty;
}

// tile shape of a launch: 256 (x 256), 192 (256 x 192) or 128 (x 128)
template <int EPI>
int choose_shape(const GemmDesc& d, int nbatch) {
    // columns of tile space (gate and up interleaved double the tile columns)
    const int ncols = EPI == EPI_SWIGLU_FWD ? 2 * d.N : d.N;
    const double c256 = shape_cost(d.M, ncols, nbatch, 256, 256, 1.0);
    // the SwiGLU-forward epilogue pairs gate and up columns inside a tile and has no 192-wide variant
    const double c192 = EPI == EPI_SWIGLU_FWD ? 1e300 : shape_cost(d.M, ncols, nbatch, 256, 192, 1.08);
    const double c128 = shape_cost(d.M, ncols, nbatch, 128, 128, 1.6);
    const int force = tuning().force_tile ? tuning().force_tile : d.force_tile;
    if (force == 256 || (!force && c256 <= c192 && c256 <= c128)) return 256;
    if (EPI != EPI_SWIGLU_FWD && (force == 192 || (!force && c192 <= c128))) return 192;
    return 128;
}

template <int EPI, int OP>
int launch(const GemmDesc& d, hipStream_t s) {
    const int nbatch = OP == OP_DW || OP == OP_DW_TAIL ? d.nbatch : (OP == OP_DW_SPLIT ? d.nbatch * d.ksplit : 1);
    const int shape = choose_shape<EPI>(d, nbatch);
    if (shape == 256) return launch_cfg<256, 256, 2, 4, EPI, OP>(d, s);
    if constexpr (EPI != EPI_SWIGLU_FWD) {
        if (shape == 192) return launch_cfg<256, 192, 4, 2, EPI, OP>(d, s);
    }
    return launch_cfg<128, 128, 2, 2, EPI, OP>(d, s);
}

// Tail cut of a batched launch (OP_DW_TAIL).  With T tiles on 256 CUs the launch runs floor(T / 256) full rounds
// and a last round of T mod 256 tiles; when that round leaves many CUs idle, each of its tiles is cut into
// `parts` depth ranges that spread over all CUs (every range at least 32 steps deep), at the price of one fp32
// tile per range written and read back.  Returns the number of ranges (0: no cut) for the shape choose_shape
// picks; *tail_tiles and *tile_elems describe the scratch.
int plan_tail(const GemmDesc& d, int* tail_tiles, int* tile_elems) {
    if (d.nbatch < 1 || d.N % 8 || d.M < 1 || d.K < 1) return 0;
    const int shape = choose_shape<EPI_STORE>(d, d.nbatch);
    const int bm = shape == 128 ? 128 : 256, bn = shape == 256 ? 256 : (shape == 192 ? 192 : 128);
    const int64_t tiles = (int64_t)((d.M + bm - 1) / bm) * ((d.N + bn - 1) / bn) * d.nbatch;
    if (tiles > 0x7FFFFFFF) return 0;
    const int head = (int)(tiles / kNumCU) * kNumCU, tail = (int)tiles - head;
    if (head == 0 || tail == 0) return 0; // less than a round: the uniform depth cut (gemm_choose_ksplit) covers that case
    const int nk = (d.K + BK - 1) / BK;
    int best = 0;
    double best_cost = 0.85; // a cut has to shorten the last round by at least 15 % (of a whole tile's time)
    for (int parts = 2; parts <= 6 && nk / parts >= 32; ++parts) {
        const int rounds = (tail * parts + kNumCU - 1) / kNumCU;
        const double cost = (double)rounds / parts + 0.04 * parts; // the second term: traffic of the partial tiles
        if (cost < best_cost) best_cost = cost, best = parts;
    }
    if (tuning().tail_parts >= 0) best = tuning().tail_parts >= 2 && nk / tuning().tail_parts >= 32 ? tuning().tail_parts : 0;
    if (best == 0) return 0;
    const int steps = (nk + best - 1) / best;
    best = (nk + steps - 1) / steps; // no empty range
    if (tail_tiles) *tail_tiles = tail;
    if (tile_elems) *tile_elems = bm * bn;
    return best;
}

// sum of the depth ranges' fp32 partial results -> bf16 rows of the problems' outputs (optional row scatter);
// one thread per 8 columns
struct ReduceArgs {
    const float* partial;
    int ksplit, nbatch, M, N;
    uint16_t* Cb[kMaxBatch];
    int64_t ldc;
    const int32_t* cs;
};
__global__ __launch_bounds__(256) void splitk_reduce_kernel(ReduceArgs r) {
    const int64_t per = (int64_t)r.M * (r.N / 8);
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= per * r.nbatch) return;
    const int z = (int)(i / per);
    const int64_t rem = i - z * per;
    const int m = (int)(rem / (r.N / 8)), n = (int)(rem % (r.N / 8)) * 8;
    f32x4 a = {0.f, 0.f, 0.f, 0.f}, b = a;
    for (int k = 0; k < r.ksplit; ++k) { // ranges in depth order
        const float* p = r.partial + (((int64_t)k * r.nbatch + z) * r.M + m) * r.N + n;
        a += *(const f32x4*)p;
        b += *(const f32x4*)(p + 4);
    }
    uint16_t* out = z == 0 ? r.Cb[0] : (z == 1 ? r.Cb[1] : (z == 2 ? r.Cb[2] : r.Cb[3]));
    const int64_t row = r.cs ? r.cs[m] : m;
    if (row < 0) return; // dropped row
    *(u32x4*)(out + row * r.ldc + n) = u32x4{pack_bf16(a[0], a[1]), pack_bf16(a[2], a[3]), pack_bf16(b[0], b[1]), pack_bf16(b[2], b[3])};
}

} // namespace

// A batched launch with few tiles and a deep K leaves most CUs idle for the whole depth of a tile.  Cutting
// the depth into r ranges multiplies the workgroups by r at the price of writing and re-reading r fp32
// copies of the outputs: taken when the 256 x 192 tiling has at most half as many tiles as there are CUs,
// r = as many as fit in one round (at most 4), every range at least 16 steps deep.
int gemm_choose_ksplit(int M, int N, int K, int nbatch) {
    if (nbatch < 1 || N % 8) return 1;
    const int64_t tiles = (int64_t)((M + 255) / 256) * ((N + 191) / 192) * nbatch;
    const int nk = (K + BK - 1) / BK;
    if (tiles * 2 > kNumCU) return 1;
    int r = (int)(kNumCU / tiles);
    r = r > 4 ? 4 : r;
    while (r > 1 && nk / r < 16) --r;
    if (r < 2) return 1;
    const int steps = (nk + r - 1) / r;
    return (nk + steps - 1) / steps; // no empty range
}

size_t gemm_split_ws_bytes(int M, int N, int K, int nbatch) {
    const int r = gemm_choose_ksplit(M, N, K, nbatch);
    return r > 1 ? (size_t)r * nbatch * M * N * sizeof(float) : 0;
}

size_t gemm_tail_ws_bytes(int M, int N, int K, int nbatch) {
    GemmDesc d;
    d.M = M, d.N = N, d.K = K, d.nbatch = nbatch;
    int tail = 0, elems = 0;
    const int parts = plan_tail(d, &tail, &elems);
    return parts > 1 ? (size_t)parts * tail * elems * sizeof(float) : 0;
}

bool gemm_mfma_supported(const GemmDesc& d) {
    if (d.M < 1 || d.N < 1 || d.K < 1) return false;
    if (d.force_tile != 0 && d.force_tile != 128 && d.force_tile != 192 && d.force_tile != 256) return false;
    // 16-byte global chunks, 16-deep MFMA steps, 32-bit byte offsets inside each operand
    if (d.K % 16 || d.lda % 8 || d.ldb % 8 || d.N % 8 || d.ldc % 8) return false;
    if (d.a_km) return false; // depth-major A goes through the transposing pre-pass or the plain kernel
    // the epilogue addresses a wave's part of the tile (at most 128 rows) with 32-bit byte offsets below 2^31
    constexpr int64_t kMaxLd = (int64_t)1 << 22;
    if (d.ldc >= kMaxLd || (d.R && d.ldr >= kMaxLd)) return false;
    if (d.epilogue == EPI_SWIGLU_BWD && (d.ldg >= kMaxLd || (d.Ct && d.ldct >= kMaxLd))) return false;
    if ((d.a_rows > 0 ? d.a_rows : (int64_t)d.M) * d.lda * 2 >= ((int64_t)1 << 32)) return false;
    if (d.a_gather && (d.a_rows <= 0 || d.epilogue == EPI_DUAL_ACC)) return false;
    if ((d.b_rows > 0 ? d.b_rows : (int64_t)d.N) * d.ldb * 2 >= ((int64_t)1 << 32)) return false;
    if (d.b_gather && d.b_rows <= 0) return false;
    if (d.R) {
        if (d.nbatch > 0 || (d.epilogue != EPI_STORE && d.epilogue != EPI_DUAL_ACC)) return false;
        if (!aligned16(d.R) || d.ldr % 8 || d.c_scatter) return false;
    }
    if (d.nbatch > 0) {
        if (d.nbatch > kMaxBatch || d.epilogue != EPI_STORE) return false;
        for (int z = 0; z < d.nbatch; ++z)
            if (!d.Ab[z] || !d.Bb[z] || !d.Cb[z] || !aligned16(d.Ab[z]) || !aligned16(d.Bb[z]) || !aligned16(d.Cb[z]))
                return false;
    } else {
        for (const void* p : {d.A, d.B, (const void*)d.C})
            if (!p || !aligned16(p)) return false;
    }
    if (d.epilogue == EPI_DUAL_ACC || d.epilogue == EPI_SWIGLU_FWD)
        if (!d.B2 || !aligned16(d.B2)) return false;
    if (d.epilogue == EPI_DUAL_ACC && (!d.A2 || !aligned16(d.A2))) return false;
    if (d.epilogue == EPI_SWIGLU_FWD) {
        if (!d.C2 || !d.C3 || !aligned16(d.C2) || !aligned16(d.C3)) return false;
    }
    if (d.epilogue == EPI_SWIGLU_BWD) {
        if (!d.C2 || !aligned16(d.C2) || (d.C3 && !aligned16(d.C3))) return false; // Act row-major is optional
        if (!d.Gin || !d.Uin || !aligned16(d.Gin) || !aligned16(d.Uin) || d.ldg % 8) return false;
        if (d.Cc || d.Cc2 || d.Cc3) return false; // row-major compact copies: plain kernel only
        if (d.Ct) {
            if (!d.Ct2 || !d.Ct3 || !aligned16(d.Ct) || !aligned16(d.Ct2) || !aligned16(d.Ct3)) return false;
            if (d.ldct % 8 || d.M % 8 || d.ldct < d.M) return false;
            if (d.cidx && !d.crank) return false;
        }
    }
    return true;
}

int gemm_mfma_bf16(const GemmDesc& d, hipStream_t s) {
    if (!gemm_mfma_supported(d)) return SDP_ERR_UNSUPPORTED;
    // OP only gives every call site its own kernel symbol, so that profiles name the step
    if (d.epilogue == EPI_STORE && d.nbatch > 0) {
        const int r = d.split_ws ? gemm_choose_ksplit(d.M, d.N, d.K, d.nbatch) : 1;
        if (r < 2 && d.tail_ws) {
            const int parts = plan_tail(d, nullptr, nullptr);
            if (parts > 1) {
                GemmDesc dt = d;
                dt.ksplit = parts;
                return launch<EPI_STORE, OP_DW_TAIL>(dt, s); // followed by its reduction
            }
        }
        if (r < 2) return launch<EPI_STORE, OP_DW>(d, s);
        GemmDesc ds = d;
        ds.ksplit = r;
        int rc = launch<EPI_STORE, OP_DW_SPLIT>(ds, s);
        if (rc != SDP_OK) return rc;
        ReduceArgs ra{(const float*)d.split_ws, r, d.nbatch, d.M, d.N, {}, d.ldc, d.c_scatter};
        for (int z = 0; z < kMaxBatch; ++z) ra.Cb[z] = (uint16_t*)d.Cb[z];
        const int64_t threads = (int64_t)d.nbatch * d.M * (d.N / 8);
        ProfileScope ps("splitk_reduce", s);
        splitk_reduce_kernel<<<(unsigned)((threads + 255) / 256), 256, 0, s>>>(ra);
        return launch_status();
    }
    if (d.epilogue == EPI_STORE && d.nbatch == 0) return launch<EPI_STORE, OP_DOWN>(d, s);
    if (d.epilogue == EPI_DUAL_ACC) return launch<EPI_DUAL_ACC, OP_DX>(d, s);
    if (d.epilogue == EPI_SWIGLU_FWD) return launch<EPI_SWIGLU_FWD, OP_GATE_UP>(d, s);
    if (d.epilogue == EPI_SWIGLU_BWD) return launch<EPI_SWIGLU_BWD, OP_DACT>(d, s);
    return SDP_ERR_UNSUPPORTED;
}

} // namespace sdp

extern "C" int sdp_profile_launch_shape(const char* name, int* tile_m, int* tile_n, int* group_m, int* stacked) {
    if (!name || !tile_m || !tile_n || !group_m || !stacked) return SDP_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(sdp::g_shape_mu);
    auto it = sdp::g_last_shape.find(name);
    if (it == sdp::g_last_shape.end()) return SDP_ERR_INVALID_ARG;
    *tile_m = it->second[0], *tile_n = it->second[1], *group_m = it->second[2], *stacked = it->second[3];
    return SDP_OK;
}
