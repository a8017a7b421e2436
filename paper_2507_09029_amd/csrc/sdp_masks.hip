// Mask sampling (host) and mask -> index compaction + coverage counts (gfx950 kernels).
//
// Mask matrix m in {0,1}^{K x F}: Sec. 3.1 of the paper; exact row budget p and column loads c_j:
// App. A.  The index form (ascending gather indices, ranks, per-neuron coverage) is what lets a
// forward-masked worker run as the physically smaller dense network of Sec. 3.2.
#include <mutex>
#include <vector>

#include "sdp_internal.h"

namespace {

// ---- counter-based generator: draw c of stream s is finalise(finalise(seed + g (s+1)) + g (c+1)),
// finalise = SplitMix64's output function.
constexpr uint64_t kGamma = 0x9E3779B97F4A7C15ull;

inline uint64_t finalise(uint64_t z) {
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

class Stream {
  public:
    Stream(uint64_t seed, uint64_t id) : key_(finalise(seed + kGamma * (id + 1))), n_(0) {}
    uint64_t next() {
        ++n_;
        return finalise(key_ + kGamma * n_);
    }
    // unbiased integer in [0, bound): raw draws under 2^64 mod bound are thrown away
    uint64_t below(uint64_t bound) {
        const uint64_t tail = (~bound + 1) % bound;
        uint64_t x;
        do {
            x = next();
        } while (x < tail);
        return x % bound;
    }

  private:
    uint64_t key_, n_;
};

int sample_masks(int K, int F, int p, uint64_t seed, bool cover, uint8_t* m) {
    std::fill(m, m + (size_t)K * F, (uint8_t)0);
    std::vector<int32_t> order(F);
    for (int k = 0; k < K; ++k) {
        Stream rng(seed, (uint64_t)k);
        for (int j = 0; j < F; ++j) order[j] = j;
        uint8_t* row = m + (size_t)k * F;
        for (int i = 0; i < p; ++i) {
            const int pick = i + (int)rng.below((uint64_t)(F - i));
            std::swap(order[i], order[pick]);
            row[order[i]] = 1;
        }
    }
    if (!cover) return SDP_OK;

    std::vector<int32_t> c(F, 0);
    for (int k = 0; k < K; ++k)
        for (int j = 0; j < F; ++j) c[j] += m[(size_t)k * F + j];
    Stream rng(seed, (uint64_t)K);
    std::vector<int32_t> cand;
    cand.reserve(F);
    for (int j = 0; j < F; ++j) {
        if (c[j] > 0) continue;
        const int k0 = (int)rng.below((uint64_t)K);
        for (int step = 0; step < K; ++step) {
            uint8_t* row = m + (size_t)((k0 + step) % K) * F;
            cand.clear();
            for (int q = 0; q < F; ++q)
                if (row[q] && c[q] > 1) cand.push_back(q);
            if (cand.empty()) continue;
            const int give = cand[rng.below((uint64_t)cand.size())];
            row[give] = 0;
            --c[give];
            row[j] = 1;
            c[j] = 1;
            break;
        }
    }
    return SDP_OK;
}

// Balanced construction (App. A, Algorithm "Structured Mask Construction"): exact row budget p, column loads
// pushed towards t = ceil(K p / F).
// Phase 1: worker i (stream 2^20 + i) weighs column j by max(t - c_j, 1e-6) with c the loads of the workers
// before it (kept as integers: 10^6 (t - c_j), or 1), and takes p distinct columns by successive weighted
// draws: u uniform below the weight still on offer, then the first column whose running weight exceeds u.
// A Fenwick tree over the weights finds that column in log F steps and takes its weight off the offer.
// Phase 2: for each column j in ascending order, while c_j < t, the first worker in ascending order that
// lacks j and holds some column loaded above t swaps its most loaded such column (lowest index on ties)
// for j; a column for which no worker qualifies stays as it is.  Row sums are p throughout.
class WeightTree {
  public:
    explicit WeightTree(int n) : n_(n), top_(1), node_(n + 1, 0) {
        while (top_ * 2 <= n) top_ *= 2;
    }
    void assign(const std::vector<uint64_t>& w) {
        std::fill(node_.begin(), node_.end(), (uint64_t)0);
        for (int j = 0; j < n_; ++j) node_[j + 1] = w[j];
        for (int i = 1; i <= n_; ++i) {
            const int up = i + (i & -i);
            if (up <= n_) node_[up] += node_[i];
        }
        total_ = 0;
        for (int j = 0; j < n_; ++j) total_ += w[j];
    }
    uint64_t total() const { return total_; }
    void remove(int j, uint64_t w) {
        for (int i = j + 1; i <= n_; i += i & -i) node_[i] -= w;
        total_ -= w;
    }
    // smallest j whose inclusive prefix weight exceeds u (u < total)
    int find(uint64_t u) const {
        int pos = 0;
        for (int step = top_; step > 0; step >>= 1) {
            const int nxt = pos + step;
            if (nxt <= n_ && node_[nxt] <= u) {
                pos = nxt;
                u -= node_[nxt];
            }
        }
        return pos;
    }

  private:
    int n_, top_;
    uint64_t total_ = 0;
    std::vector<uint64_t> node_;
};

int sample_masks_balanced(int K, int F, int p, uint64_t seed, uint8_t* m) {
    std::fill(m, m + (size_t)K * F, (uint8_t)0);
    if (p == 0) return SDP_OK;
    const int64_t target = ((int64_t)K * p + F - 1) / F;
    std::vector<int64_t> c(F, 0);
    std::vector<uint64_t> w(F);
    WeightTree tree(F);
    for (int i = 0; i < K; ++i) {
        Stream rng(seed, ((uint64_t)1 << 20) + (uint64_t)i);
        uint8_t* row = m + (size_t)i * F;
        for (int j = 0; j < F; ++j) w[j] = c[j] < target ? (uint64_t)(target - c[j]) * 1000000ull : 1ull;
        tree.assign(w);
        for (int d = 0; d < p; ++d) {
            const int j = tree.find(rng.below(tree.total()));
            row[j] = 1;
            tree.remove(j, w[j]);
        }
        for (int j = 0; j < F; ++j) c[j] += row[j];
    }
    // phase 2: per worker, its columns above the target, found on demand
    for (int j = 0; j < F; ++j) {
        while (c[j] < target) {
            bool swapped = false;
            for (int i = 0; i < K && !swapped; ++i) {
                uint8_t* row = m + (size_t)i * F;
                if (row[j]) continue;
                int give = -1;
                for (int k = 0; k < F; ++k)
                    if (row[k] && c[k] > target && (give < 0 || c[k] > c[give])) give = k;
                if (give < 0) continue;
                row[give] = 0, --c[give];
                row[j] = 1, ++c[j];
                swapped = true;
            }
            if (!swapped) break;
        }
    }
    return SDP_OK;
}

// ---- device side ---------------------------------------------------------------------------
constexpr int kScanThreads = 256;
constexpr int kPerThread = 8;
constexpr int kChunk = kScanThreads * kPerThread; // mask bytes per workgroup

__device__ inline int block_exclusive_scan(int v, int* total, int* lds /*[kScanThreads/64 + 1]*/) {
    // inclusive scan inside the wave by shuffles, then across the (at most 4) waves through LDS
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        int t = __shfl_up(inc, off, 64);
        if (lane >= off) inc += t;
    }
    if (lane == 63) lds[wave] = inc;
    __syncthreads();
    int base = 0, sum = 0;
#pragma unroll
    for (int w = 0; w < kScanThreads / 64; ++w) {
        int t = lds[w];
        if (w < wave) base += t;
        sum += t;
    }
    __syncthreads();
    *total = sum;
    return base + inc - v;
}

// grid (chunks, K): number of non-zero mask bytes in each chunk of each worker's row
__global__ __launch_bounds__(kScanThreads) void chunk_count_kernel(const uint8_t* __restrict__ mask, int64_t F,
                                                                   int nchunks, int32_t* __restrict__ chunk_cnt) {
    __shared__ int lds[kScanThreads / 64 + 1];
    const int k = blockIdx.y, c = blockIdx.x;
    const int64_t j0 = (int64_t)c * kChunk + (int64_t)threadIdx.x * kPerThread;
    const uint8_t* row = mask + (int64_t)k * F;
    int n = 0;
#pragma unroll
    for (int i = 0; i < kPerThread; ++i)
        if (j0 + i < F) n += row[j0 + i] != 0;
    int total;
    block_exclusive_scan(n, &total, lds);
    if (threadIdx.x == 0) chunk_cnt[(int64_t)k * nchunks + c] = total;
}

// grid (chunks, K): ranks inside the chunk + sum of the preceding chunks' counts -> idx, pos, count
__global__ __launch_bounds__(kScanThreads) void compact_kernel(const uint8_t* __restrict__ mask, int64_t F,
                                                               int nchunks, const int32_t* __restrict__ chunk_cnt,
                                                               int32_t* __restrict__ idx, int64_t idx_ld,
                                                               int32_t* __restrict__ pos, int32_t* __restrict__ count) {
    __shared__ int lds[kScanThreads / 64 + 1];
    const int k = blockIdx.y, c = blockIdx.x;
    const int32_t* cnt = chunk_cnt + (int64_t)k * nchunks;
    // every workgroup needs (a) the count of all chunks before its own, (b) the row total
    int before = 0, all = 0;
    for (int i = threadIdx.x; i < nchunks; i += kScanThreads) {
        int t = cnt[i];
        all += t;
        if (i < c) before += t;
    }
    int row_total, base;
    block_exclusive_scan(all, &row_total, lds);
    block_exclusive_scan(before, &base, lds);

    const int64_t j0 = (int64_t)c * kChunk + (int64_t)threadIdx.x * kPerThread;
    const uint8_t* row = mask + (int64_t)k * F;
    uint8_t bits[kPerThread];
    int n = 0;
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
        bits[i] = (j0 + i < F) ? (row[j0 + i] != 0) : 0;
        n += bits[i];
    }
    int dummy;
    int rank = base + block_exclusive_scan(n, &dummy, lds);
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
        if (j0 + i >= F) break;
        if (bits[i]) {
            pos[(int64_t)k * F + j0 + i] = rank;
            if (rank < idx_ld) idx[(int64_t)k * idx_ld + rank] = (int32_t)(j0 + i);
            ++rank;
        } else {
            pos[(int64_t)k * F + j0 + i] = -1;
        }
    }
    // the tail of the idx row (entries row_total .. idx_ld) is -1; chunk c fills its own slice of it
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
        const int64_t t = j0 + i;
        if (t < idx_ld && t >= row_total) idx[(int64_t)k * idx_ld + t] = -1;
    }
    if (c == 0 && threadIdx.x == 0 && count) count[k] = row_total;
}

// coverage c_j = sum_k [m_kj != 0]
__global__ __launch_bounds__(256) void coverage_kernel(const uint8_t* __restrict__ mask, int K, int64_t F,
                                                       uint8_t* __restrict__ cov) {
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= F) return;
    int c = 0;
    for (int k = 0; k < K; ++k) c += mask[(int64_t)k * F + j] != 0;
    cov[j] = (uint8_t)c;
}

// load histogram hist[c] = #{ j : c_j = c }, c = 0 .. SDP_MAX_WORKERS; one more bin, hist[SDP_MAX_WORKERS + 1],
// counts the bytes above SDP_MAX_WORKERS (no set of workers produces them: the call then fails)
constexpr int kLoads = SDP_MAX_WORKERS + 2;

__global__ void clear_histogram_kernel(unsigned long long* __restrict__ hist) {
    if (threadIdx.x < kLoads) hist[threadIdx.x] = 0ull;
}

__global__ __launch_bounds__(256) void load_histogram_kernel(const uint8_t* __restrict__ cov, int64_t F,
                                                             unsigned long long* __restrict__ hist) {
    __shared__ unsigned int local[kLoads];
    for (int i = threadIdx.x; i < kLoads; i += blockDim.x) local[i] = 0u;
    __syncthreads();
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < F; j += stride) {
        const int c = cov[j];
        atomicAdd(&local[c < kLoads - 1 ? c : kLoads - 1], 1u);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kLoads; i += blockDim.x)
        if (local[i]) atomicAdd(&hist[i], (unsigned long long)local[i]);
}

// Short rows (at most kFusedChunks chunks): everything in one launch.  Workgroup k < K walks worker k's row
// chunk by chunk, carrying the running count (no second kernel, no table of chunk counts); the workgroups
// after those compute the coverage counts of 256 neurons each.
constexpr int kFusedChunks = 16;
__global__ __launch_bounds__(kScanThreads) void index_short_rows_kernel(const uint8_t* __restrict__ mask, int K, int64_t F,
                                                                        int nchunks, int32_t* __restrict__ idx, int64_t idx_ld,
                                                                        int32_t* __restrict__ pos, int32_t* __restrict__ count,
                                                                        uint8_t* __restrict__ cov) {
    __shared__ int lds[kScanThreads / 64 + 1];
    if ((int)blockIdx.x >= K) {
        const int64_t j = (int64_t)(blockIdx.x - K) * kScanThreads + threadIdx.x;
        if (j >= F) return;
        int c = 0;
        for (int k = 0; k < K; ++k) c += mask[(int64_t)k * F + j] != 0;
        cov[j] = (uint8_t)c;
        return;
    }
    const int k = blockIdx.x;
    const uint8_t* row = mask + (int64_t)k * F;
    int base = 0;
    for (int c = 0; c < nchunks; ++c) {
        const int64_t j0 = (int64_t)c * kChunk + (int64_t)threadIdx.x * kPerThread;
        uint8_t bits[kPerThread];
        int n = 0;
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) {
            bits[i] = (j0 + i < F) ? (row[j0 + i] != 0) : 0;
            n += bits[i];
        }
        int total;
        int rank = base + block_exclusive_scan(n, &total, lds);
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) {
            if (j0 + i >= F) break;
            if (bits[i]) {
                pos[(int64_t)k * F + j0 + i] = rank;
                if (rank < idx_ld) idx[(int64_t)k * idx_ld + rank] = (int32_t)(j0 + i);
                ++rank;
            } else {
                pos[(int64_t)k * F + j0 + i] = -1;
            }
        }
        base += total;
    }
    // the tail of the idx row (entries count .. idx_ld) is -1
    for (int64_t t = (int64_t)base + threadIdx.x; t < idx_ld; t += kScanThreads) idx[(int64_t)k * idx_ld + t] = -1;
    if (threadIdx.x == 0 && count) count[k] = base;
}

int check_index_args(int K, int64_t F, const void* mask, const void* idx, int64_t idx_ld, const void* pos,
                     const void* cov, const void* ws, size_t ws_bytes) {
    if (!mask || !idx || !pos || !cov) return SDP_ERR_INVALID_ARG;
    if (K < 1 || K > SDP_MAX_WORKERS || F < 1) return SDP_ERR_INVALID_ARG;
    if (F >= ((int64_t)1 << 31) || idx_ld < 1 || idx_ld > F) return SDP_ERR_SHAPE;
    if (!ws || ws_bytes < sdp_index_masks_workspace_bytes(K, F)) return SDP_ERR_WORKSPACE;
    return SDP_OK;
}

} // namespace

extern "C" size_t sdp_index_masks_workspace_bytes(int K, int64_t F) {
    if (K < 1 || F < 1) return 0;
    const int64_t nchunks = (F + kChunk - 1) / kChunk;
    return sdp::round_up((size_t)K * (size_t)nchunks * sizeof(int32_t), 256);
}

extern "C" int sdp_index_masks(int K, int64_t F, const uint8_t* mask, int32_t* idx, int64_t idx_ld, int32_t* pos,
                               int32_t* count, uint8_t* cov, void* ws, size_t ws_bytes, void* stream) {
    int rc = check_index_args(K, F, mask, idx, idx_ld, pos, cov, ws, ws_bytes);
    if (rc != SDP_OK) return rc;
    hipStream_t s = (hipStream_t)stream;
    const int nchunks = (int)((F + kChunk - 1) / kChunk);
    if (nchunks <= kFusedChunks) {
        sdp::ProfileScope ps("mask_index", s);
        const unsigned blocks = (unsigned)(K + (F + kScanThreads - 1) / kScanThreads);
        index_short_rows_kernel<<<blocks, kScanThreads, 0, s>>>(mask, K, F, nchunks, idx, idx_ld, pos, count, cov);
        return sdp::launch_status();
    }
    int32_t* chunk_cnt = (int32_t*)ws;
    {
        sdp::ProfileScope ps("mask_chunk_count", s);
        chunk_count_kernel<<<dim3(nchunks, K), kScanThreads, 0, s>>>(mask, F, nchunks, chunk_cnt);
    }
    {
        sdp::ProfileScope ps("mask_compact", s);
        compact_kernel<<<dim3(nchunks, K), kScanThreads, 0, s>>>(mask, F, nchunks, chunk_cnt, idx, idx_ld, pos, count);
    }
    {
        sdp::ProfileScope ps("mask_coverage", s);
        coverage_kernel<<<dim3((unsigned)((F + 255) / 256)), 256, 0, s>>>(mask, K, F, cov);
    }
    return sdp::launch_status();
}

namespace {

// ---- the compaction for callers that cannot allocate ------------------------------------------------
// The table of chunk counts, which sdp_index_masks takes from the caller's workspace, lives in a fixed array of
// this library instead.  In host code the array's name is only a stand-in: the address a kernel can use is asked
// for once per device (each GPU holds its own copy at its own address) and kept.
__device__ __align__(256) int32_t g_chunk_counts[SDP_INDEX_STATIC_MAX_COUNTS];

constexpr int kMaxDevices = 64;
std::mutex g_counts_mu;
int32_t* g_counts_ptr[kMaxDevices] = {};

// device address of g_chunk_counts on the current device (looked up on first use); null on failure
int32_t* chunk_counts_on_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lk(g_counts_mu);
    if (!g_counts_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_chunk_counts)) != hipSuccess || !p) return nullptr;
        g_counts_ptr[dev] = (int32_t*)p;
    }
    return g_counts_ptr[dev];
}

} // namespace

extern "C" int sdp_index_masks_static(int K, int64_t F, const uint8_t* mask, int32_t* idx, int64_t idx_ld, int32_t* pos,
                                      int32_t* count, uint8_t* cov, void* stream) {
    if (!mask || !idx || !pos || !cov) return SDP_ERR_INVALID_ARG;
    if (K < 1 || K > SDP_MAX_WORKERS || F < 1) return SDP_ERR_INVALID_ARG;
    if (F >= ((int64_t)1 << 31) || idx_ld < 1 || idx_ld > F) return SDP_ERR_SHAPE;
    const int64_t nchunks = (F + kChunk - 1) / kChunk;
    if (nchunks > kFusedChunks && (int64_t)K * nchunks > SDP_INDEX_STATIC_MAX_COUNTS) return SDP_ERR_SHAPE;
    hipStream_t s = (hipStream_t)stream;
    if (nchunks <= kFusedChunks) { // short rows need no table at all
        sdp::ProfileScope ps("mask_index", s);
        const unsigned blocks = (unsigned)(K + (F + kScanThreads - 1) / kScanThreads);
        index_short_rows_kernel<<<blocks, kScanThreads, 0, s>>>(mask, K, F, (int)nchunks, idx, idx_ld, pos, count, cov);
        return sdp::launch_status();
    }
    int32_t* chunk_cnt = chunk_counts_on_current_device();
    if (!chunk_cnt) return SDP_ERR_HIP;
    // every entry the second kernel reads is written by the first one of the same call: nothing to clear
    {
        sdp::ProfileScope ps("mask_chunk_count", s);
        chunk_count_kernel<<<dim3((unsigned)nchunks, K), kScanThreads, 0, s>>>(mask, F, (int)nchunks, chunk_cnt);
    }
    {
        sdp::ProfileScope ps("mask_compact", s);
        compact_kernel<<<dim3((unsigned)nchunks, K), kScanThreads, 0, s>>>(mask, F, (int)nchunks, chunk_cnt, idx, idx_ld, pos, count);
    }
    {
        sdp::ProfileScope ps("mask_coverage", s);
        coverage_kernel<<<dim3((unsigned)((F + 255) / 256)), 256, 0, s>>>(mask, K, F, cov);
    }
    return sdp::launch_status();
}

extern "C" int sdp_mask_rho2(int K, int64_t F, const uint8_t* cov, uint64_t* hist, double* rho2_host, void* stream) {
    if (!cov || !hist || !rho2_host) return SDP_ERR_INVALID_ARG;
    if (K < 1 || K > SDP_MAX_WORKERS || F < 1) return SDP_ERR_INVALID_ARG;
    if (F >= ((int64_t)1 << 31)) return SDP_ERR_SHAPE;
    hipStream_t s = (hipStream_t)stream;
    unsigned long long* h = reinterpret_cast<unsigned long long*>(hist);
    {
        sdp::ProfileScope ps("mask_load_histogram", s);
        clear_histogram_kernel<<<1, 128, 0, s>>>(h);
        const int64_t blocks = (F + 256 * 16 - 1) / (256 * 16); // each block's 66 global atomics pay for 4096 columns
        load_histogram_kernel<<<dim3((unsigned)(blocks < 2048 ? blocks : 2048)), 256, 0, s>>>(cov, F, h);
    }
    int rc = sdp::launch_status();
    if (rc != SDP_OK) return rc;
    uint64_t host[kLoads];
    if (hipMemcpyAsync(host, hist, sizeof(host), hipMemcpyDeviceToHost, s) != hipSuccess) return SDP_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return SDP_ERR_HIP;
    for (int c = K + 1; c < kLoads; ++c)
        if (host[c]) return SDP_ERR_INVALID_ARG; // cov does not belong to K workers
    // a column of load c > 0 holds c entries (1/K - 1/c) and K - c entries 1/K: together 1/c - 1/K;
    // an uncovered column holds K entries 1/K
    double acc = (double)host[0] / K;
    for (int c = 1; c <= K; ++c) acc += (double)host[c] * (1.0 / c - 1.0 / K);
    *rho2_host = acc;
    return SDP_OK;
}

extern "C" int sdp_sample_masks_host(int K, int F, int p, uint64_t seed, int require_cover, uint8_t* mask_host) {
    if (!mask_host || K < 1 || K > SDP_MAX_WORKERS || F < 1 || p < 0) return SDP_ERR_INVALID_ARG;
    if (p > F) return SDP_ERR_SHAPE;
    if (require_cover < 0 || require_cover > SDP_MASKS_BALANCED) return SDP_ERR_INVALID_ARG;
    if (require_cover == SDP_MASKS_BALANCED) return sample_masks_balanced(K, F, p, seed, mask_host);
    if (require_cover && (int64_t)K * p < F) return SDP_ERR_UNCOVERED;
    return sample_masks(K, F, p, seed, require_cover != 0, mask_host);
}

extern "C" int sdp_make_masks(int K, int F, int p, uint64_t seed, int require_cover, uint8_t* mask, int32_t* idx,
                              int32_t* pos, uint8_t* cov, void* ws, size_t ws_bytes, void* stream) {
    if (!mask || !idx || !pos || !cov) return SDP_ERR_INVALID_ARG;
    if (K < 1 || K > SDP_MAX_WORKERS || F < 1 || p < 0) return SDP_ERR_INVALID_ARG;
    if (p > F) return SDP_ERR_SHAPE;
    if (require_cover < 0 || require_cover > SDP_MASKS_BALANCED) return SDP_ERR_INVALID_ARG;
    if (require_cover == SDP_MASKS_UNIFORM_COVER && (int64_t)K * p < F) return SDP_ERR_UNCOVERED;
    if (!ws || ws_bytes < sdp_index_masks_workspace_bytes(K, F)) return SDP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    std::vector<uint8_t> host((size_t)K * F);
    int rc = require_cover == SDP_MASKS_BALANCED ? sample_masks_balanced(K, F, p, seed, host.data())
                                                 : sample_masks(K, F, p, seed, require_cover != 0, host.data());
    if (rc != SDP_OK) return rc;
    if (hipMemcpyAsync(mask, host.data(), host.size(), hipMemcpyHostToDevice, s) != hipSuccess) return SDP_ERR_HIP;
    if (p > 0) {
        rc = sdp_index_masks(K, F, mask, idx, p, pos, nullptr, cov, ws, ws_bytes, stream);
    } else {
        // empty budget: no idx entries exist; pos is all -1 and cov all 0
        if (hipMemsetAsync(pos, 0xFF, (size_t)K * F * sizeof(int32_t), s) != hipSuccess) return SDP_ERR_HIP;
        if (hipMemsetAsync(cov, 0, (size_t)F, s) != hipSuccess) return SDP_ERR_HIP;
    }
    if (hipStreamSynchronize(s) != hipSuccess) return SDP_ERR_HIP;
    return rc;
}
