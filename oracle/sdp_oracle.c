/*
 * sdp_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 CPU statement of what the Subnetwork-Data-Parallel (SDP)
 * masked SwiGLU MLP path computes, written out from the paper's definitions.
 * It shares no code with the GPU library and is never called by it.  Only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may use it.
 *
 * Notation follows the paper: n = K workers, m = F components (hidden neurons),
 * p = per-worker budget, mask[k][j] = m_{k,j} (Sec. 3.1), c_j = column load
 * (App. A).  The MLP is the bias-free SwiGLU block
 *     G = X W1^T,  U = X W3^T,  A = silu(G) * U,  Y = A W2^T
 * with every weight stored neuron-major: W1[F][d], W3[F][d], W2T[F][d]
 * (W2T[j][:] is column j of W2), so that hidden neuron j owns row j of each.
 *
 * No blocking, no fusion, no reordering: every loop below is the definition.
 * OpenMP is applied to outermost independent loops only.
 *
 * Parity pins (see tests/test_oracle_*.py): the finaliser against the published
 * SplitMix64 sequence; the sampler by its invariants and a uniformity test;
 * index/coverage against brute force; the dense MLP forward against a library
 * einsum; its gradients against central finite differences; forward masking
 * against the compact-slice route and the zero-gradient property; backward
 * masking and the gated average against their C = 1 (DDP) reductions; the
 * attention block against a library attention routine with autograd, central
 * finite differences, causality, and the block built from the held heads alone.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* Counter-based random numbers.  The 64-bit finaliser is the output function */
/* of SplitMix64 (Steele, Lea, Flood 2014).  A stream is (seed, stream id);   */
/* its c-th draw is a pure function of (seed, stream, c).                     */
/* ------------------------------------------------------------------------- */
#define ORC_GOLDEN 0x9E3779B97F4A7C15ULL

uint64_t orc_mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

uint64_t orc_rand64(uint64_t seed, uint64_t stream, uint64_t ctr) {
    uint64_t key = orc_mix64(seed + ORC_GOLDEN * (stream + 1));
    return orc_mix64(key + ORC_GOLDEN * (ctr + 1));
}

typedef struct {
    uint64_t seed, stream, ctr;
} orc_rng;

static uint64_t rng_next(orc_rng* r) { return orc_rand64(r->seed, r->stream, r->ctr++); }

/* Uniform integer in [0, n): draws below 2^64 mod n are rejected, so every   */
/* residue has exactly floor(2^64 / n) accepted preimages.                    */
static uint64_t rng_below(orc_rng* r, uint64_t n) {
    uint64_t reject_below = (0 - n) % n;
    for (;;) {
        uint64_t x = rng_next(r);
        if (x >= reject_below) return x % n;
    }
}

/* Exposed so that a test can check the bounded draw on its own. */
uint64_t orc_rand_below(uint64_t seed, uint64_t stream, uint64_t* ctr, uint64_t n) {
    orc_rng r = {seed, stream, *ctr};
    uint64_t v = rng_below(&r, n);
    *ctr = r.ctr;
    return v;
}

/* ------------------------------------------------------------------------- */
/* Mask matrix m in {0,1}^{K x F} (Sec. 3.1), exact row budget sum_j m_kj = p  */
/* (App. A).  Uniform sampler: worker k draws p distinct neurons by a partial */
/* Fisher-Yates shuffle on stream k.  With require_cover, every neuron left   */
/* with column load 0 is then handed to a worker that gives up a neuron of    */
/* load >= 2 (stream K drives the repair), which keeps every row sum at p.    */
/* Returns 0, or -1 on bad arguments, -4 if coverage is impossible (K p < F). */
/* ------------------------------------------------------------------------- */
int orc_make_masks(int K, int F, int p, uint64_t seed, int require_cover, uint8_t* mask) {
    if (K < 1 || F < 1 || p < 0 || p > F || !mask) return -1;
    if (require_cover && (int64_t)K * p < F) return -4;
    memset(mask, 0, (size_t)K * F);
    int32_t* perm = (int32_t*)malloc(sizeof(int32_t) * (size_t)F);
    for (int k = 0; k < K; ++k) {
        orc_rng r = {seed, (uint64_t)k, 0};
        for (int j = 0; j < F; ++j) perm[j] = j;
        for (int i = 0; i < p; ++i) {
            int j = i + (int)rng_below(&r, (uint64_t)(F - i));
            int32_t tmp = perm[i];
            perm[i] = perm[j];
            perm[j] = tmp;
            mask[(size_t)k * F + perm[i]] = 1;
        }
    }
    free(perm);
    if (!require_cover) return 0;

    int32_t* load = (int32_t*)calloc((size_t)F, sizeof(int32_t));
    int32_t* donors = (int32_t*)malloc(sizeof(int32_t) * (size_t)F);
    for (int k = 0; k < K; ++k)
        for (int j = 0; j < F; ++j) load[j] += mask[(size_t)k * F + j];
    orc_rng r = {seed, (uint64_t)K, 0};
    for (int j = 0; j < F; ++j) {
        if (load[j] != 0) continue;
        int first = (int)rng_below(&r, (uint64_t)K);
        for (int s = 0; s < K; ++s) {
            int k = (first + s) % K;
            int nd = 0;
            for (int q = 0; q < F; ++q)
                if (mask[(size_t)k * F + q] && load[q] >= 2) donors[nd++] = q;
            if (nd == 0) continue;
            int q = donors[rng_below(&r, (uint64_t)nd)];
            mask[(size_t)k * F + q] = 0;
            load[q] -= 1;
            mask[(size_t)k * F + j] = 1;
            load[j] = 1;
            break;
        }
    }
    free(load);
    free(donors);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Balanced mask construction (App. A, Algorithm "Structured Mask             */
/* Construction"): exact row budget p, column loads pushed towards the target */
/* t = ceil(K p / F).                                                         */
/* Phase 1, worker i = 0..K-1 (stream 2^20 + i): weights from the loads of    */
/* the workers before it, w_j = max(t - c_j, eps) with eps = 1e-6, held as    */
/* integers 10^6 (t - c_j) or 1; p distinct columns by successive draws with  */
/* renormalisation: u uniform below the total weight of the columns not yet   */
/* taken, the column whose running sum first exceeds u is taken.              */
/* Phase 2, column j ascending, while c_j < t: the first worker (ascending)   */
/* that does not hold j but holds a column of load > t takes j and gives up   */
/* its most loaded such column (lowest index on ties); when no worker         */
/* qualifies the column is left as it is.  As printed, the phase asks for     */
/* rows below budget, of which there are none after phase 1, and then removes */
/* a surplus column from rows above budget: the reading here keeps every row  */
/* sum at p at all times.                                                     */
/* Returns 0, or -1 on bad arguments.                                         */
/* ------------------------------------------------------------------------- */
int orc_make_masks_balanced(int K, int F, int p, uint64_t seed, uint8_t* mask) {
    if (K < 1 || F < 1 || p < 0 || p > F || !mask) return -1;
    memset(mask, 0, (size_t)K * F);
    if (p == 0) return 0;
    const int64_t t = ((int64_t)K * p + F - 1) / F;
    int64_t* load = (int64_t*)calloc((size_t)F, sizeof(int64_t));
    uint64_t* w = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)F);
    for (int i = 0; i < K; ++i) {
        orc_rng r = {seed, (uint64_t)(1 << 20) + (uint64_t)i, 0};
        uint8_t* row = mask + (size_t)i * F;
        for (int j = 0; j < F; ++j) w[j] = load[j] < t ? (uint64_t)(t - load[j]) * 1000000ULL : 1ULL;
        for (int d = 0; d < p; ++d) {
            uint64_t total = 0;
            for (int j = 0; j < F; ++j)
                if (!row[j]) total += w[j];
            uint64_t u = rng_below(&r, total);
            uint64_t run = 0;
            for (int j = 0; j < F; ++j) {
                if (row[j]) continue;
                run += w[j];
                if (run > u) {
                    row[j] = 1;
                    break;
                }
            }
        }
        for (int j = 0; j < F; ++j) load[j] += row[j];
    }
    for (int j = 0; j < F; ++j) {
        while (load[j] < t) {
            int moved = 0;
            for (int i = 0; i < K && !moved; ++i) {
                uint8_t* row = mask + (size_t)i * F;
                if (row[j]) continue;
                int donor = -1;
                for (int k = 0; k < F; ++k)
                    if (row[k] && load[k] > t && (donor < 0 || load[k] > load[donor])) donor = k;
                if (donor < 0) continue;
                row[j] = 1, load[j] += 1;
                row[donor] = 0, load[donor] -= 1;
                moved = 1;
            }
            if (!moved) break;
        }
    }
    free(load);
    free(w);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Index form of a mask: idx[k][i] = i-th active neuron of worker k in         */
/* ascending order (entries past count[k] are -1; row stride idx_ld),          */
/* pos[k][j] = rank of j inside worker k's active set or -1,                   */
/* count[k] = row sum, cov[j] = c_j = sum_k m_kj (App. A).                     */
/* ------------------------------------------------------------------------- */
void orc_index_masks(int K, int64_t F, const uint8_t* mask, int32_t* idx, int64_t idx_ld,
                     int32_t* pos, int32_t* count, uint8_t* cov) {
    for (int k = 0; k < K; ++k) {
        int32_t seen = 0;
        for (int64_t i = 0; i < idx_ld; ++i) idx[k * idx_ld + i] = -1;
        for (int64_t j = 0; j < F; ++j) {
            if (mask[k * F + j]) {
                if (seen < idx_ld) idx[k * idx_ld + seen] = (int32_t)j;
                pos[k * F + j] = seen;
                seen += 1;
            } else {
                pos[k * F + j] = -1;
            }
        }
        count[k] = seen;
    }
    for (int64_t j = 0; j < F; ++j) {
        int c = 0;
        for (int k = 0; k < K; ++k) c += mask[k * F + j] ? 1 : 0;
        cov[j] = (uint8_t)c;
    }
}

/* ------------------------------------------------------------------------- */
/* Dense SwiGLU MLP, forward.  All arrays row-major fp64.                      */
/*   X[T][d], W1/W3/W2T[F][d] -> G,U,A[T][F], Y[T][d]                          */
/* ------------------------------------------------------------------------- */
static double sigmoid(double z) { return 1.0 / (1.0 + exp(-z)); }

void orc_mlp_fwd(int64_t T, int64_t d, int64_t F, const double* X, const double* W1,
                 const double* W3, const double* W2T, double* G, double* U, double* A, double* Y) {
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        for (int64_t j = 0; j < F; ++j) {
            double g = 0.0, u = 0.0;
            for (int64_t e = 0; e < d; ++e) {
                g += X[t * d + e] * W1[j * d + e];
                u += X[t * d + e] * W3[j * d + e];
            }
            G[t * F + j] = g;
            U[t * F + j] = u;
            A[t * F + j] = g * sigmoid(g) * u;
        }
        /* Y[t][e] = sum_j A[t][j] W2T[j][e], the sum over j taken in neuron order. */
        for (int64_t e = 0; e < d; ++e) Y[t * d + e] = 0.0;
        for (int64_t j = 0; j < F; ++j)
            for (int64_t e = 0; e < d; ++e) Y[t * d + e] += A[t * F + j] * W2T[j * d + e];
    }
}

/* ------------------------------------------------------------------------- */
/* Dense SwiGLU MLP, backward of L = <dY, Y>.  Needs G, U, A from the forward. */
/*   dA = dY W2;  dU = dA silu(G);  dG = dA U silu'(G),                        */
/*   silu'(z) = s(z) (1 + z (1 - s(z)));                                       */
/*   dW2T[j] = sum_t A[t][j] dY[t];  dW1[j] = sum_t dG[t][j] X[t];             */
/*   dW3[j] = sum_t dU[t][j] X[t];   dX = dG W1 + dU W3.                       */
/* dGbuf/dUbuf are [T][F] outputs (returned so that tests can look at them).   */
/* Every sum over t runs in token order for its (j, e).                        */
/* ------------------------------------------------------------------------- */
void orc_mlp_bwd(int64_t T, int64_t d, int64_t F, const double* X, const double* dY,
                 const double* W1, const double* W3, const double* W2T, const double* G,
                 const double* U, const double* A, double* dGbuf, double* dUbuf, double* dX,
                 double* dW1, double* dW3, double* dW2T) {
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        for (int64_t j = 0; j < F; ++j) {
            double da = 0.0;
            for (int64_t e = 0; e < d; ++e) da += dY[t * d + e] * W2T[j * d + e];
            double g = G[t * F + j], u = U[t * F + j];
            double s = sigmoid(g);
            dUbuf[t * F + j] = da * (g * s);
            dGbuf[t * F + j] = da * u * (s * (1.0 + g * (1.0 - s)));
        }
        /* dX[t][e] = sum_j (dG[t][j] W1[j][e] + dU[t][j] W3[j][e]), j in neuron order. */
        for (int64_t e = 0; e < d; ++e) dX[t * d + e] = 0.0;
        for (int64_t j = 0; j < F; ++j)
            for (int64_t e = 0; e < d; ++e)
                dX[t * d + e] += dGbuf[t * F + j] * W1[j * d + e] + dUbuf[t * F + j] * W3[j * d + e];
    }
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < F; ++j) {
        for (int64_t e = 0; e < d; ++e) dW1[j * d + e] = dW3[j * d + e] = dW2T[j * d + e] = 0.0;
        for (int64_t t = 0; t < T; ++t) {
            double dg = dGbuf[t * F + j], du = dUbuf[t * F + j], a = A[t * F + j];
            for (int64_t e = 0; e < d; ++e) {
                dW1[j * d + e] += dg * X[t * d + e];
                dW3[j * d + e] += du * X[t * d + e];
                dW2T[j * d + e] += a * dY[t * d + e];
            }
        }
    }
}

/* ------------------------------------------------------------------------- */
/* Gated parameters (eq. "gate"): theta_k = m_k (.) theta.  For the neuron     */
/* mask of Sec. 3.2 this zeroes row j of W1, W3 and column j of W2 (row j of   */
/* W2T) for every neuron j with m_kj = 0.                                      */
/* ------------------------------------------------------------------------- */
void orc_gate_rows(int64_t F, int64_t d, const uint8_t* mask_k, const double* W, double* Wg) {
    for (int64_t j = 0; j < F; ++j)
        for (int64_t e = 0; e < d; ++e) Wg[j * d + e] = mask_k[j] ? W[j * d + e] : 0.0;
}

/* ------------------------------------------------------------------------- */
/* One worker's step under either masking regime (Sec. 3.1).                   */
/*   mode 0, forward masking:  m_fwd = m_bwd = m.  Loss and gradient are       */
/*     evaluated at the gated parameters; the gradient is then zero off-mask.  */
/*   mode 1, backward masking: m_fwd = all ones, m_bwd = m.  Loss and dX come  */
/*     from the full parameters; the weight gradient is kept on the mask only. */
/* Outputs are full size: G,U[T][F], Y,dX[T][d], dW*[F][d].                    */
/* Returns the number of off-mask weight-gradient entries that are not exactly */
/* zero BEFORE any masking of the gradient (must be 0 in mode 0).              */
/* ------------------------------------------------------------------------- */
int64_t orc_worker_step(int mode, int64_t T, int64_t d, int64_t F, const uint8_t* mask_k,
                        const double* X, const double* dY, const double* W1, const double* W3,
                        const double* W2T, double* G, double* U, double* Y, double* dX,
                        double* dW1, double* dW3, double* dW2T) {
    size_t wn = (size_t)F * d, an = (size_t)T * F;
    double* A = (double*)malloc(sizeof(double) * an);
    double* dGb = (double*)malloc(sizeof(double) * an);
    double* dUb = (double*)malloc(sizeof(double) * an);
    int64_t nonzero_off_mask = 0;
    if (mode == 0) {
        double* W1g = (double*)malloc(sizeof(double) * wn);
        double* W3g = (double*)malloc(sizeof(double) * wn);
        double* W2g = (double*)malloc(sizeof(double) * wn);
        orc_gate_rows(F, d, mask_k, W1, W1g);
        orc_gate_rows(F, d, mask_k, W3, W3g);
        orc_gate_rows(F, d, mask_k, W2T, W2g);
        orc_mlp_fwd(T, d, F, X, W1g, W3g, W2g, G, U, A, Y);
        orc_mlp_bwd(T, d, F, X, dY, W1g, W3g, W2g, G, U, A, dGb, dUb, dX, dW1, dW3, dW2T);
        for (int64_t j = 0; j < F; ++j)
            if (!mask_k[j])
                for (int64_t e = 0; e < d; ++e)
                    nonzero_off_mask += (dW1[j * d + e] != 0.0) + (dW3[j * d + e] != 0.0) +
                                        (dW2T[j * d + e] != 0.0);
        free(W1g);
        free(W3g);
        free(W2g);
    } else {
        orc_mlp_fwd(T, d, F, X, W1, W3, W2T, G, U, A, Y);
        orc_mlp_bwd(T, d, F, X, dY, W1, W3, W2T, G, U, A, dGb, dUb, dX, dW1, dW3, dW2T);
        for (int64_t j = 0; j < F; ++j)
            if (!mask_k[j])
                for (int64_t e = 0; e < d; ++e)
                    dW1[j * d + e] = dW3[j * d + e] = dW2T[j * d + e] = 0.0;
    }
    free(A);
    free(dGb);
    free(dUb);
    return nonzero_off_mask;
}

/* ------------------------------------------------------------------------- */
/* Gated average (eq. "average") with the per-coordinate load:                 */
/*   out_j = (1 / c_j) sum_{k : m_kj = 1} (g_k)_j,   c_j = sum_k m_kj,         */
/* the mask being constant along a neuron row of D parameters.  Off-mask       */
/* entries are not read (the mask selects, it does not multiply); c_j = 0      */
/* gives out_j = 0.  Summation runs in worker order k = 0..K-1.                */
/* gtype: 0 = fp32, 1 = bf16 bit patterns (uint16), 2 = fp64.                  */
/* ------------------------------------------------------------------------- */
static double widen(const void* base, int gtype, int64_t i) {
    if (gtype == 0) return (double)((const float*)base)[i];
    if (gtype == 2) return ((const double*)base)[i];
    uint32_t bits = ((uint32_t)((const uint16_t*)base)[i]) << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

void orc_gated_average(int K, int64_t R, int64_t D, int gtype, const void* const* g,
                       const uint8_t* mask, double* out, uint8_t* cov) {
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < R; ++r) {
        int c = 0;
        for (int k = 0; k < K; ++k) c += mask[(int64_t)k * R + r] ? 1 : 0;
        cov[r] = (uint8_t)c;
        for (int64_t e = 0; e < D; ++e) {
            double s = 0.0;
            for (int k = 0; k < K; ++k)
                if (mask[(int64_t)k * R + r]) s += widen(g[k], gtype, r * D + e);
            out[r * D + e] = c ? s / (double)c : 0.0;
        }
    }
}

/* Squared l2 norm of the gated average: what the global gradient clipping of */
/* the LLM runs (App. "Hyperparameters for LLM Architecture": clipping at 1.0) */
/* measures before the update.  Rows nobody covers have a zero average.        */
/* Plain sequential sum in fp64, rows in order.                                */
double orc_gated_average_sqnorm(int K, int64_t R, int64_t D, int gtype, const void* const* g,
                                const uint8_t* mask) {
    double total = 0.0;
    for (int64_t r = 0; r < R; ++r) {
        int c = 0;
        for (int k = 0; k < K; ++k) c += mask[(int64_t)k * R + r] ? 1 : 0;
        if (!c) continue;
        for (int64_t e = 0; e < D; ++e) {
            double s = 0.0;
            for (int k = 0; k < K; ++k)
                if (mask[(int64_t)k * R + r]) s += widen(g[k], gtype, r * D + e);
            const double a = s / (double)c;
            total += a * a;
        }
    }
    return total;
}

/* Coefficient of global-norm clipping at max_norm (the paper states the       */
/* threshold only; this is the usual form): min(1, max_norm / (norm + 1e-6)),  */
/* norm^2 = the sum of the parameter groups' squared norms.                     */
double orc_clip_scale(int n, const double* sqnorm, double max_norm) {
    double total = 0.0;
    for (int i = 0; i < n; ++i) total += sqnorm[i];
    const double coef = max_norm / (sqrt(total) + 1e-6);
    return coef < 1.0 ? coef : 1.0;
}

/* ------------------------------------------------------------------------- */
/* The gated average followed by the optimizer the paper trains with (AdamW,   */
/* App. "Hyperparameters for LLM Architecture"), on covered rows only         */
/* (Sec. 3.2: parameters, gradients and optimizer state live only on covered  */
/* coordinates).  For every row r with c_r >= 1 and each of its parameters:   */
/*   ghat  = grad_scale * (1/c_r) * sum_{k covers r} g_k                      */
/*   theta = theta - lr * wd * theta                  (decoupled weight decay) */
/*   m     = beta1 m + (1 - beta1) ghat,   v = beta2 v + (1 - beta2) ghat^2    */
/*   theta = theta - lr * (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps)*/
/* Rows with c_r = 0 keep theta, m, v.  Everything in fp64; theta, m, v are    */
/* updated in place.                                                          */
/* ------------------------------------------------------------------------- */
void orc_avg_adamw(int K, int64_t R, int64_t D, int gtype, const void* const* g, const uint8_t* mask,
                   double* theta, double* m, double* v, uint8_t* cov, double lr, double beta1, double beta2,
                   double eps, double wd, double grad_scale, int step) {
    const double bc1 = 1.0 - pow(beta1, (double)step), bc2 = 1.0 - pow(beta2, (double)step);
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < R; ++r) {
        int c = 0;
        for (int k = 0; k < K; ++k) c += mask[(int64_t)k * R + r] ? 1 : 0;
        cov[r] = (uint8_t)c;
        if (c == 0) continue;
        for (int64_t e = 0; e < D; ++e) {
            const int64_t i = r * D + e;
            double s = 0.0;
            for (int k = 0; k < K; ++k)
                if (mask[(int64_t)k * R + r]) s += widen(g[k], gtype, i);
            const double ghat = grad_scale * (s / (double)c);
            theta[i] -= lr * wd * theta[i];
            m[i] = beta1 * m[i] + (1.0 - beta1) * ghat;
            v[i] = beta2 * v[i] + (1.0 - beta2) * ghat * ghat;
            theta[i] -= lr * (m[i] / bc1) / (sqrt(v[i] / bc2) + eps);
        }
    }
}

/* Squared Frobenius distance to uniform masking (Thm. 3.1) with per-column    */
/* loads:  rho^2 = sum_{k,j} (1/K - m_kj / c_j)^2, columns with c_j = 0 give   */
/* K (1/K)^2.                                                                  */
double orc_rho2(int K, int64_t F, const uint8_t* mask) {
    double acc = 0.0;
    for (int64_t j = 0; j < F; ++j) {
        int c = 0;
        for (int k = 0; k < K; ++k) c += mask[(int64_t)k * F + j] ? 1 : 0;
        for (int k = 0; k < K; ++k) {
            double v = 1.0 / K - ((c && mask[(int64_t)k * F + j]) ? 1.0 / c : 0.0);
            acc += v * v;
        }
    }
    return acc;
}

/* ========================================================================= */
/* Head-level masking of the attention block (Sec. 4.1: the neuron-level      */
/* variant masks attention heads on W_Q, W_K, W_V and W_O).                    */
/*                                                                             */
/* Bias-free causal multi-head self-attention over Bt sequences of S tokens    */
/* (token t = b S + s), H heads of width hd, every weight neuron-major:        */
/*   Wq, Wk, Wv [H hd][d]  (row h hd + r = feature r of head h),               */
/*   WoT        [H hd][d]  (row j = column j of W_O),                          */
/*   Q = X Wq^T, K = X Wk^T, V = X Wv^T                      [T][H hd]         */
/*   P_h[s][s'] = softmax over s' <= s of Q_h[s].K_h[s'] / sqrt(hd)            */
/*   O_h = P_h V_h,   Y = sum_h O_h WoT_h.                                     */
/* Head h owns rows h hd .. h hd + hd - 1 of each of the four matrices; the    */
/* gate of Sec. 3.1 zeroes them for a head the worker does not hold.           */
/* ========================================================================= */

/* Dense forward.  Q, K, V, O are [T][H hd] outputs, Y is [T][d].              */
void orc_attn_fwd(int64_t Bt, int64_t S, int64_t d, int64_t H, int64_t hd, const double* X,
                  const double* Wq, const double* Wk, const double* Wv, const double* WoT,
                  double* Q, double* Kp, double* V, double* O, double* Y) {
    const int64_t T = Bt * S, E = H * hd;
    const double scale = 1.0 / sqrt((double)hd);
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t)
        for (int64_t j = 0; j < E; ++j) {
            double q = 0.0, k = 0.0, v = 0.0;
            for (int64_t e = 0; e < d; ++e) {
                q += X[t * d + e] * Wq[j * d + e];
                k += X[t * d + e] * Wk[j * d + e];
                v += X[t * d + e] * Wv[j * d + e];
            }
            Q[t * E + j] = q, Kp[t * E + j] = k, V[t * E + j] = v;
        }
#pragma omp parallel for schedule(dynamic) collapse(2)
    for (int64_t b = 0; b < Bt; ++b)
        for (int64_t h = 0; h < H; ++h) {
            double* P = (double*)malloc(sizeof(double) * (size_t)S);
            for (int64_t s = 0; s < S; ++s) {
                const int64_t t = b * S + s;
                double mx = -INFINITY;
                for (int64_t s2 = 0; s2 <= s; ++s2) {
                    double z = 0.0;
                    for (int64_t r = 0; r < hd; ++r) z += Q[t * E + h * hd + r] * Kp[(b * S + s2) * E + h * hd + r];
                    P[s2] = z * scale;
                    if (P[s2] > mx) mx = P[s2];
                }
                double den = 0.0;
                for (int64_t s2 = 0; s2 <= s; ++s2) {
                    P[s2] = exp(P[s2] - mx);
                    den += P[s2];
                }
                for (int64_t r = 0; r < hd; ++r) {
                    double o = 0.0;
                    for (int64_t s2 = 0; s2 <= s; ++s2) o += (P[s2] / den) * V[(b * S + s2) * E + h * hd + r];
                    O[t * E + h * hd + r] = o;
                }
            }
            free(P);
        }
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        for (int64_t e = 0; e < d; ++e) Y[t * d + e] = 0.0;
        for (int64_t j = 0; j < E; ++j)
            for (int64_t e = 0; e < d; ++e) Y[t * d + e] += O[t * E + j] * WoT[j * d + e];
    }
}

/* Dense backward of L = <dY, Y>.  Q, K, V, O come from the forward.           */
/*   dO = dY W_O^T-rows: dO[t][j] = dY[t].WoT[j];   dWoT[j] = sum_t O[t][j] dY[t] */
/*   per (b, h), with P recomputed row by row:                                 */
/*     dV[s'] += P[s][s'] dO[s];   dP[s][s'] = dO[s].V[s']                     */
/*     dZ[s][s'] = P[s][s'] (dP[s][s'] - sum_u P[s][u] dP[s][u])               */
/*     dQ[s] += dZ[s][s'] K[s'] / sqrt(hd);   dK[s'] += dZ[s][s'] Q[s] / sqrt(hd) */
/*   dWq[j] = sum_t dQ[t][j] X[t] (same for k, v);  dX = dQ Wq + dK Wk + dV Wv. */
/* dQ, dK, dV are [T][H hd] outputs (returned so that tests can look at them).  */
void orc_attn_bwd(int64_t Bt, int64_t S, int64_t d, int64_t H, int64_t hd, const double* X,
                  const double* dY, const double* Wq, const double* Wk, const double* Wv,
                  const double* WoT, const double* Q, const double* Kp, const double* V,
                  const double* O, double* dQ, double* dK, double* dV, double* dX, double* dWq,
                  double* dWk, double* dWv, double* dWoT) {
    const int64_t T = Bt * S, E = H * hd;
    const double scale = 1.0 / sqrt((double)hd);
    double* dO = (double*)malloc(sizeof(double) * (size_t)(T * E));
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t)
        for (int64_t j = 0; j < E; ++j) {
            double a = 0.0;
            for (int64_t e = 0; e < d; ++e) a += dY[t * d + e] * WoT[j * d + e];
            dO[t * E + j] = a;
            dQ[t * E + j] = dK[t * E + j] = dV[t * E + j] = 0.0;
        }
#pragma omp parallel for schedule(dynamic) collapse(2)
    for (int64_t b = 0; b < Bt; ++b)
        for (int64_t h = 0; h < H; ++h) {
            double* P = (double*)malloc(sizeof(double) * (size_t)S);
            double* dP = (double*)malloc(sizeof(double) * (size_t)S);
            for (int64_t s = 0; s < S; ++s) {
                const int64_t t = b * S + s;
                double mx = -INFINITY;
                for (int64_t s2 = 0; s2 <= s; ++s2) {
                    double z = 0.0;
                    for (int64_t r = 0; r < hd; ++r) z += Q[t * E + h * hd + r] * Kp[(b * S + s2) * E + h * hd + r];
                    P[s2] = z * scale;
                    if (P[s2] > mx) mx = P[s2];
                }
                double den = 0.0;
                for (int64_t s2 = 0; s2 <= s; ++s2) {
                    P[s2] = exp(P[s2] - mx);
                    den += P[s2];
                }
                double dot = 0.0;
                for (int64_t s2 = 0; s2 <= s; ++s2) {
                    P[s2] /= den;
                    double a = 0.0;
                    for (int64_t r = 0; r < hd; ++r) a += dO[t * E + h * hd + r] * V[(b * S + s2) * E + h * hd + r];
                    dP[s2] = a;
                    dot += P[s2] * a;
                }
                for (int64_t s2 = 0; s2 <= s; ++s2) {
                    const int64_t t2 = b * S + s2;
                    const double dz = P[s2] * (dP[s2] - dot);
                    for (int64_t r = 0; r < hd; ++r) {
                        dV[t2 * E + h * hd + r] += P[s2] * dO[t * E + h * hd + r];
                        dQ[t * E + h * hd + r] += dz * Kp[t2 * E + h * hd + r] * scale;
                        dK[t2 * E + h * hd + r] += dz * Q[t * E + h * hd + r] * scale;
                    }
                }
            }
            free(P);
            free(dP);
        }
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        for (int64_t e = 0; e < d; ++e) dX[t * d + e] = 0.0;
        for (int64_t j = 0; j < E; ++j)
            for (int64_t e = 0; e < d; ++e)
                dX[t * d + e] += dQ[t * E + j] * Wq[j * d + e] + dK[t * E + j] * Wk[j * d + e] +
                                 dV[t * E + j] * Wv[j * d + e];
    }
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < E; ++j) {
        for (int64_t e = 0; e < d; ++e) dWq[j * d + e] = dWk[j * d + e] = dWv[j * d + e] = dWoT[j * d + e] = 0.0;
        for (int64_t t = 0; t < T; ++t)
            for (int64_t e = 0; e < d; ++e) {
                dWq[j * d + e] += dQ[t * E + j] * X[t * d + e];
                dWk[j * d + e] += dK[t * E + j] * X[t * d + e];
                dWv[j * d + e] += dV[t * E + j] * X[t * d + e];
                dWoT[j * d + e] += O[t * E + j] * dY[t * d + e];
            }
    }
    free(dO);
}

/* One worker's attention step under either masking regime of Sec. 3.1 applied  */
/* to heads (head_mask[H]; a head owns its rows of Wq, Wk, Wv, WoT).            */
/*   mode 0, forward masking:  m_fwd = m_bwd = m.  Loss and gradient are        */
/*     evaluated at the gated parameters; the gradient of every head the        */
/*     worker does not hold is then exactly zero.                               */
/*   mode 1, backward masking: m_fwd = all ones, m_bwd = m.  Loss and dX come   */
/*     from the full block; the weight gradient is kept for held heads only.    */
/* Outputs are full size.  Returns the number of weight-gradient entries of     */
/* unheld heads that are not exactly zero BEFORE any masking of the gradient    */
/* (must be 0 in mode 0).                                                       */
int64_t orc_attn_worker_step(int mode, int64_t Bt, int64_t S, int64_t d, int64_t H, int64_t hd,
                             const uint8_t* head_mask, const double* X, const double* dY,
                             const double* Wq, const double* Wk, const double* Wv, const double* WoT,
                             double* Q, double* Kp, double* V, double* O, double* Y, double* dQ,
                             double* dK, double* dV, double* dX, double* dWq, double* dWk,
                             double* dWv, double* dWoT) {
    const int64_t E = H * hd;
    const size_t wn = (size_t)E * d;
    uint8_t* row_mask = (uint8_t*)malloc((size_t)E);
    for (int64_t j = 0; j < E; ++j) row_mask[j] = head_mask[j / hd];
    int64_t nz = 0;
    if (mode == 0) {
        double* g[4];
        const double* w[4] = {Wq, Wk, Wv, WoT};
        for (int i = 0; i < 4; ++i) {
            g[i] = (double*)malloc(sizeof(double) * wn);
            orc_gate_rows(E, d, row_mask, w[i], g[i]);
        }
        orc_attn_fwd(Bt, S, d, H, hd, X, g[0], g[1], g[2], g[3], Q, Kp, V, O, Y);
        orc_attn_bwd(Bt, S, d, H, hd, X, dY, g[0], g[1], g[2], g[3], Q, Kp, V, O, dQ, dK, dV, dX, dWq, dWk, dWv, dWoT);
        for (int64_t j = 0; j < E; ++j)
            if (!row_mask[j])
                for (int64_t e = 0; e < d; ++e)
                    nz += (dWq[j * d + e] != 0.0) + (dWk[j * d + e] != 0.0) + (dWv[j * d + e] != 0.0) +
                          (dWoT[j * d + e] != 0.0);
        for (int i = 0; i < 4; ++i) free(g[i]);
    } else {
        orc_attn_fwd(Bt, S, d, H, hd, X, Wq, Wk, Wv, WoT, Q, Kp, V, O, Y);
        orc_attn_bwd(Bt, S, d, H, hd, X, dY, Wq, Wk, Wv, WoT, Q, Kp, V, O, dQ, dK, dV, dX, dWq, dWk, dWv, dWoT);
        for (int64_t j = 0; j < E; ++j)
            if (!row_mask[j])
                for (int64_t e = 0; e < d; ++e)
                    dWq[j * d + e] = dWk[j * d + e] = dWv[j * d + e] = dWoT[j * d + e] = 0.0;
    }
    free(row_mask);
    return nz;
}
