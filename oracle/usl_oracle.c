/*
 * CPU oracle for the uniformly-sparse output layer (fan-in exactly k per label).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, loop-by-loop
 * statement of what the layer computes, written from the paper, with every floating
 * sum carried in double and rounded to float once.  It shares no code with the HIP
 * library; only tests, the smoke check and the benchmark's cpu_baseline leg call it.
 *
 * Layout used everywhere here (the transpose of the paper's [s, m] arrays):
 *   idx[m][k] int32   feature feeding slot t of label j      (paper: indices[t, j])
 *   W  [m][k]         value of that connection               (paper: weights[t, j])
 *   x  [b][d]         activations of the penultimate layer   (paper: features)
 *   out, g [b][m]     scores and upstream gradient           (paper: output, backward)
 * storage: 0 = x and W are float32, 1 = x and W are bfloat16 (upper 16 bits of a float32).
 *
 * OpenMP is used only as an outer "parallel for" over independent outputs.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double widen(const void* p, int64_t i, int storage) {
    if (storage == 0) return (double)((const float*)p)[i];
    uint32_t bits = (uint32_t)((const uint16_t*)p)[i] << 16;
    float f;
    memcpy(&f, &bits, 4);
    return (double)f;
}

/* float32 -> bfloat16, round to nearest, ties to even; NaN stays NaN. */
static uint16_t to_bf16(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}

/* The layer is a dense m x d matrix A that is zero except at k places per row: A[j][col(j,t)] = val(j,t),
 * t < k (Section 3.2, the uniform format).  The three products below are the dense-layer definitions
 * restricted to those places; the accessors name the operands. */
static int32_t col(const int32_t* idx, int32_t k, int64_t j, int32_t t) { return idx[j * k + t]; }
static double val(const void* W, int32_t k, int64_t j, int32_t t, int storage) { return widen(W, j * k + t, storage); }
static double act(const void* x, int32_t d, int32_t i, int32_t c, int storage) { return widen(x, (int64_t)i * d + c, storage); }

/* Scores (Section 3.2, what Algorithm 1 computes): out = x A^T, i.e.
 * out[i][j] = sum over the k connections of label j of val(j,t) * x[i][col(j,t)]. */
void orc_forward(const void* x, const int32_t* idx, const void* W, float* out,
                 int64_t m, int32_t d, int32_t k, int32_t b, int storage) {
#pragma omp parallel for schedule(static)
    for (int32_t i = 0; i < b; ++i)
        for (int64_t j = 0; j < m; ++j) {
            double score = 0.0;
            for (int32_t t = 0; t < k; ++t) score += act(x, d, i, col(idx, k, j, t), storage) * val(W, k, j, t, storage);
            out[(int64_t)i * m + j] = (float)score;
        }
}

/* Gradient of the connection values (Section 3.3, what Algorithm 3 computes; its test for a zero
 * gradient only leaves out terms that are exactly zero): the dense gradient g^T x read at the k places
 * of every row, grad_W[j][t] = sum over the batch of g[i][j] * x[i][col(j,t)]. */
void orc_backward_weight(const float* g, const void* x, const int32_t* idx, float* grad_W,
                         int64_t m, int32_t d, int32_t k, int32_t b, int storage) {
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < m; ++j)
        for (int32_t t = 0; t < k; ++t) {
            const int32_t c = col(idx, k, j, t);
            double sum = 0.0;
            for (int32_t i = 0; i < b; ++i) sum += act(x, d, i, c, storage) * (double)g[(int64_t)i * m + j];
            grad_W[j * k + t] = (float)sum;
        }
}

/* Gradient of the input features (Section 3.3, what Algorithm 2 computes with atomic additions; here
 * the additions go one after the other into a zeroed row of doubles): grad_x = g A, i.e.
 * grad_x[i][c] = sum over all connections (j,t) with col(j,t) == c of val(j,t) * g[i][j]. */
void orc_backward_input(const float* g, const int32_t* idx, const void* W, float* grad_x,
                        int64_t m, int32_t d, int32_t k, int32_t b, int storage) {
#pragma omp parallel for schedule(static)
    for (int32_t i = 0; i < b; ++i) {
        double* sums = (double*)calloc((size_t)d, sizeof(double));
        for (int64_t j = 0; j < m; ++j) {
            const double gij = (double)g[(int64_t)i * m + j];
            for (int32_t t = 0; t < k; ++t) sums[col(idx, k, j, t)] += val(W, k, j, t, storage) * gij;
        }
        for (int32_t c = 0; c < d; ++c) grad_x[(int64_t)i * d + c] = (float)sums[c];
        free(sums);
    }
}

/* One-vs-all binary cross-entropy on the scores, summed over all labels (Section 2,
 * the decomposition of the loss into a sum over labels; BCE is the comparison loss of
 * Section 4.4).  Targets come as a CSR list: labels tgt_lab[tgt_off[i] .. tgt_off[i+1])
 * are the positives of instance i (a set: repeats count once).
 *   l(z,y) = max(z,0) - z*y + log(1 + exp(-|z|)),  dl/dz = sigmoid(z) - y
 *   loss = scale * sum_{i,j} l(out[i][j], y[i][j]),  g[i][j] = scale * dl/dz
 * g may be the same array as out.  loss_out receives the double sum. */
void orc_bce_loss_grad(const float* out, const int64_t* tgt_off, const int32_t* tgt_lab,
                       float scale, float* g, double* loss_out, int64_t m, int32_t b) {
    double total = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : total)
    for (int32_t i = 0; i < b; ++i) {
        uint8_t* y = (uint8_t*)calloc((size_t)m, 1);
        for (int64_t p = tgt_off[i]; p < tgt_off[i + 1]; ++p) y[tgt_lab[p]] = 1;
        double acc = 0.0;
        for (int64_t j = 0; j < m; ++j) {
            double z = (double)out[(int64_t)i * m + j];
            double yy = (double)y[j];
            double e = exp(-fabs(z));
            acc += fmax(z, 0.0) - z * yy + log1p(e);
            double sig = (z >= 0.0) ? 1.0 / (1.0 + e) : e / (1.0 + e);
            g[(int64_t)i * m + j] = (float)((double)scale * (sig - yy));
        }
        free(y);
        total += acc;
    }
    *loss_out = (double)scale * total;
}

/* One-vs-all squared hinge loss, the loss the paper mainly uses (Section 3.3):
 *   l(y, z) = max(0, 1 - y*z)^2 with y = +1 for listed labels and -1 otherwise,
 *   dl/dz = -2*y*max(0, 1 - y*z), exactly zero whenever y*z >= 1.
 * loss = scale * sum_{i,j} l,  g = scale * dl/dz.  g may be the same array as out. */
void orc_sqh_loss_grad(const float* out, const int64_t* tgt_off, const int32_t* tgt_lab,
                       float scale, float* g, double* loss_out, int64_t m, int32_t b) {
    double total = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : total)
    for (int32_t i = 0; i < b; ++i) {
        uint8_t* y = (uint8_t*)calloc((size_t)m, 1);
        for (int64_t p = tgt_off[i]; p < tgt_off[i + 1]; ++p) y[tgt_lab[p]] = 1;
        double acc = 0.0;
        for (int64_t j = 0; j < m; ++j) {
            double z = (double)out[(int64_t)i * m + j];
            double yy = y[j] ? 1.0 : -1.0;
            double margin = fmax(0.0, 1.0 - yy * z);
            acc += margin * margin;
            g[(int64_t)i * m + j] = (float)((double)scale * (-2.0 * yy * margin));
        }
        free(y);
        total += acc;
    }
    *loss_out = (double)scale * total;
}

/* Prediction (Section 2): the kk highest-scoring labels of every instance, best first.
 * Label p ranks before label q if out[p] > out[q], or if the scores compare equal and p < q
 * (so -0 and +0 tie).  Written as the definition: kk times, walk the whole row and take the best
 * label not taken yet.  Scores must not be NaN.  top_lab, top_val: [b][kk]. */
void orc_topk(const float* out, int64_t m, int32_t b, int32_t kk, int32_t* top_lab, float* top_val) {
#pragma omp parallel for schedule(static)
    for (int32_t i = 0; i < b; ++i) {
        const float* z = out + (int64_t)i * m;
        uint8_t* taken = (uint8_t*)calloc((size_t)m, 1);
        for (int32_t r = 0; r < kk; ++r) {
            int64_t best = -1;
            for (int64_t j = 0; j < m; ++j) {
                if (taken[j]) continue;
                if (best < 0 || z[j] > z[best]) best = j; /* strict: the first of equals stays */
            }
            taken[best] = 1;
            top_lab[(int64_t)i * kk + r] = (int32_t)best;
            top_val[(int64_t)i * kk + r] = z[best];
        }
        free(taken);
    }
}

/* Precision at k (Section 2, the equation that defines P@k): with y the 0/1 target vector and
 * yhat the 0/1 vector of the k predicted labels, P@k = (1/k) * sum_j y[j]*yhat[j], averaged over
 * instances.  hits[r] counts the instances whose rank-r prediction (0-based) is one of their
 * targets, so that P@k = (hits[0] + ... + hits[k-1]) / (k * b) for every k <= kk at once. */
void orc_precision_hits(const int32_t* top_lab, const int64_t* tgt_off, const int32_t* tgt_lab,
                        int32_t b, int32_t kk, int64_t* hits) {
    for (int32_t r = 0; r < kk; ++r) hits[r] = 0;
    for (int32_t i = 0; i < b; ++i)
        for (int32_t r = 0; r < kk; ++r) {
            int hit = 0;
            for (int64_t p = tgt_off[i]; p < tgt_off[i + 1]; ++p)
                if (tgt_lab[p] == top_lab[(int64_t)i * kk + r]) hit = 1;
            hits[r] += hit;
        }
}

/* Adam (Kingma & Ba, Algorithm 1; the optimizer named in Section 4.1) on the m*k values.
 * t is the 1-based step count.  With storage==1, W is bfloat16: the updated value is
 * rounded float -> bfloat16 (nearest even) and, if W_f32_out is not NULL, the unrounded
 * float is written there as well. */
void orc_adam_step(void* W, const float* grad_W, float* m1, float* m2, int64_t n, int64_t t,
                   float lr, float beta1, float beta2, float eps, int storage, float* W_f32_out) {
    double b1 = (double)beta1, b2 = (double)beta2;
    double c1 = 1.0 - pow(b1, (double)t);
    double c2 = 1.0 - pow(b2, (double)t);
#pragma omp parallel for schedule(static)
    for (int64_t f = 0; f < n; ++f) {
        double gw = (double)grad_W[f];
        double a = b1 * (double)m1[f] + (1.0 - b1) * gw;
        double v = b2 * (double)m2[f] + (1.0 - b2) * gw * gw;
        double w = widen(W, f, storage) - (double)lr * (a / c1) / (sqrt(v / c2) + (double)eps);
        m1[f] = (float)a;
        m2[f] = (float)v;
        if (storage == 0) {
            ((float*)W)[f] = (float)w;
        } else {
            ((uint16_t*)W)[f] = to_bf16((float)w);
            if (W_f32_out) W_f32_out[f] = (float)w;
        }
    }
}

/* ---- counter-based random numbers: Philox-4x32, 10 rounds (Salmon et al., SC'11) ---- */
static void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

void orc_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) {
    philox4x32_10(ctr, key, out);
}

/* Candidate column for (row j, slot t, attempt a) of redistribution number `epoch`:
 * first Philox word with counter (j, t, a, epoch_lo) and key (seed_lo, seed_hi ^ epoch_hi),
 * mapped to [0, d) by multiply-shift. */
int32_t orc_draw_column(uint64_t seed, uint64_t epoch, uint32_t j, uint32_t t, uint32_t a, int32_t d) {
    uint32_t ctr[4] = {j, t, a, (uint32_t)epoch};
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32) ^ (uint32_t)(epoch >> 32)};
    uint32_t r[4];
    philox4x32_10(ctr, key, r);
    return (int32_t)(((uint64_t)r[0] * (uint64_t)(uint32_t)d) >> 32);
}

/* Refill the slots of row j flagged in `empty` (length k), in increasing slot order.
 * A candidate is rejected while it equals the column of any slot that is not empty;
 * a filled slot stops being empty at once. */
static void regrow_row(int32_t* row_idx, uint8_t* empty, int64_t j, int32_t d, int32_t k,
                       uint64_t seed, uint64_t epoch) {
    for (int32_t t = 0; t < k; ++t) {
        if (!empty[t]) continue;
        uint32_t a = 0;
        for (;;) {
            int32_t c = orc_draw_column(seed, epoch, (uint32_t)j, (uint32_t)t, a++, d);
            int clash = 0;
            for (int32_t u = 0; u < k; ++u)
                if (!empty[u] && row_idx[u] == c) { clash = 1; break; }
            if (!clash) { row_idx[t] = c; empty[t] = 0; break; }
        }
    }
}

/* Initial connectivity (Section 4.1: connections drawn uniformly at random with the same
 * number per label): every slot of every row starts empty and is filled as in a
 * redistribution with the reserved epoch 2^64-1. */
void orc_init_indices(int32_t* idx, int64_t m, int32_t d, int32_t k, uint64_t seed) {
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < m; ++j) {
        uint8_t* empty = (uint8_t*)malloc((size_t)k);
        memset(empty, 1, (size_t)k);
        regrow_row(idx + j * k, empty, j, d, k, seed, ~(uint64_t)0);
        free(empty);
    }
}

static int cmp_u64(const void* a, const void* b) {
    uint64_t x = *(const uint64_t*)a, y = *(const uint64_t*)b;
    return (x > y) - (x < y);
}

/* Connection redistribution (Section 2, the prune / redistribute cycle of SET; Section 3.2
 * on why a column's slots never move): remove the n = floor(fraction * m*k) connections of
 * smallest magnitude in the whole layer, order (|W| bit pattern, flat slot number), then give
 * every removed slot a new column drawn uniformly from the structural zeros of its own row.
 * A new connection starts at +0 with zeroed Adam moments.  pruned_flags (may be NULL)
 * receives 1 for every rewired flat slot.  Returns n, or -1 if m*k does not fit 32 bits. */
int64_t orc_redistribute(int32_t* idx, void* W, float* m1, float* m2, int64_t m, int32_t d,
                         int32_t k, double fraction, uint64_t seed, uint64_t epoch, int storage,
                         uint8_t* pruned_flags) {
    int64_t N = m * (int64_t)k;
    if (N > (int64_t)0xFFFFFFFFll) return -1;
    int64_t n = (int64_t)floor(fraction * (double)N);
    if (pruned_flags) memset(pruned_flags, 0, (size_t)N);
    if (n <= 0) return 0;
    if (n > N) n = N;
    uint64_t* keys = (uint64_t*)malloc((size_t)N * sizeof(uint64_t));
    for (int64_t f = 0; f < N; ++f) {
        uint64_t mag;
        if (storage == 0) {
            uint32_t u;
            memcpy(&u, (const float*)W + f, 4);
            mag = u & 0x7FFFFFFFu;
        } else {
            mag = ((const uint16_t*)W)[f] & 0x7FFFu;
        }
        keys[f] = (mag << 32) | (uint64_t)f;
    }
    qsort(keys, (size_t)N, sizeof(uint64_t), cmp_u64);
    uint8_t* empty = (uint8_t*)calloc((size_t)N, 1);
    for (int64_t r = 0; r < n; ++r) empty[keys[r] & 0xFFFFFFFFull] = 1;
    free(keys);
    if (pruned_flags) memcpy(pruned_flags, empty, (size_t)N);
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < m; ++j) {
        int any = 0;
        for (int32_t t = 0; t < k; ++t) {
            if (!empty[j * k + t]) continue;
            any = 1;
            if (storage == 0) ((float*)W)[j * k + t] = 0.0f;
            else ((uint16_t*)W)[j * k + t] = 0;
            m1[j * k + t] = 0.0f;
            m2[j * k + t] = 0.0f;
        }
        if (any) regrow_row(idx + j * k, empty + j * k, j, d, k, seed, epoch);
    }
    free(empty);
    return n;
}

/* The per-row variant of the redistribution (Section 2 leaves open whether the prune fraction is
 * taken over the layer or over each unit; Section 3.2 only requires a constant count per label):
 * every row loses its per_row connections of smallest magnitude, order (|W| bit pattern, slot t),
 * and refills those slots exactly as orc_redistribute does.  pruned_flags as there. */
void orc_redistribute_rows(int32_t* idx, void* W, float* m1, float* m2, int64_t m, int32_t d, int32_t k,
                           int32_t per_row, uint64_t seed, uint64_t epoch, int storage,
                           uint8_t* pruned_flags) {
    if (per_row > k) per_row = k;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < m; ++j) {
        uint64_t* keys = (uint64_t*)malloc((size_t)k * sizeof(uint64_t));
        uint8_t* empty = (uint8_t*)calloc((size_t)k, 1);
        for (int32_t t = 0; t < k; ++t) {
            uint64_t mag;
            if (storage == 0) {
                uint32_t u;
                memcpy(&u, (const float*)W + j * k + t, 4);
                mag = u & 0x7FFFFFFFu;
            } else {
                mag = ((const uint16_t*)W)[j * k + t] & 0x7FFFu;
            }
            keys[t] = (mag << 32) | (uint64_t)t;
        }
        qsort(keys, (size_t)k, sizeof(uint64_t), cmp_u64);
        for (int32_t r = 0; r < per_row; ++r) empty[keys[r] & 0xFFFFFFFFull] = 1;
        for (int32_t t = 0; t < k; ++t) {
            if (pruned_flags) pruned_flags[j * k + t] = empty[t];
            if (!empty[t]) continue;
            if (storage == 0) ((float*)W)[j * k + t] = 0.0f;
            else ((uint16_t*)W)[j * k + t] = 0;
            m1[j * k + t] = 0.0f;
            m2[j * k + t] = 0.0f;
        }
        if (per_row > 0) regrow_row(idx + j * k, empty, j, d, k, seed, epoch);
        free(keys);
        free(empty);
    }
}

/* Count rows that break the uniform-sparsity invariant: an index outside [0, d) or a
 * column that appears twice in one row. */
int64_t orc_count_bad_rows(const int32_t* idx, int64_t m, int32_t d, int32_t k) {
    int64_t bad = 0;
#pragma omp parallel for schedule(static) reduction(+ : bad)
    for (int64_t j = 0; j < m; ++j) {
        int b = 0;
        for (int32_t t = 0; t < k && !b; ++t) {
            int32_t c = idx[j * k + t];
            if (c < 0 || c >= d) { b = 1; break; }
            for (int32_t u = 0; u < t; ++u)
                if (idx[j * k + u] == c) { b = 1; break; }
        }
        bad += b;
    }
    return bad;
}

int orc_num_threads(void) {
    int n = 1;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    n = omp_get_max_threads();
#endif
    return n;
}
