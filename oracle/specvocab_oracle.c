/*
 * CPU oracle for the SpecVocab draft-step output distribution.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the parity reference for the HIP
 * library: plain, slow, single-threaded loops that follow the paper's
 * definitions term by term.  It shares no code with the HIP path and the
 * product never calls it.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may load it.
 *
 * What each function follows (arxiv 2602.13836):
 *   svo_dense_logits   Section 3.1:  z_t = U h_t
 *   svo_select         Section 3.3, Step 1: h' = W_down h, s = W_vocab h'
 *                      Section 3.3, Step 2: k_t = top-k(s_t, k)
 *   svo_subset_logits  Section 3.3, Step 3: U' = U[k_t, :], z' = U' h_t
 *   svo_softmax_topk   Section 3.3: q_K = softmax(z'); draft tokens = the
 *                      top-kd entries of q_K (Appendix, inference
 *                      hyperparameters: Top-k = 10)
 *   svo_log_softmax    Section 3.4 (training): q_aux = softmax(s_t) over the
 *                      entire vocabulary, as natural-log probabilities
 *
 * Precision.  The paper does not fix storage or accumulation precision.
 * Inputs are float32 or bfloat16 (bit patterns, widened exactly to float32).
 * Each dot product is accumulated term by term in index order i = 0..d-1,
 * either in float32 (acc = SVO_ACC_F32; one rounded multiply then one rounded
 * add per term, build with -ffp-contract=off) or in float64
 * (acc = SVO_ACC_F64).  Results are returned as double (a float32 result is
 * widened exactly), so callers compare against either without another rounding.
 *
 * Readings of points the paper leaves open:
 *   - no bias, no temperature, no normalisation in either projection;
 *   - h' may be rounded to bfloat16 between the two projections
 *     (hprime_round = 1: what two chained bf16 linear layers do) or kept
 *     (hprime_round = 0);
 *   - top-k ties: the larger score wins, equal scores -> the smaller token id;
 *   - k_t is returned in ascending token-id order;
 *   - the subset softmax is renormalised over the subset only.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { SVO_F32 = 0, SVO_BF16 = 1 };
enum { SVO_IDX_PER_ROW = 0, SVO_IDX_PER_STEP = 1 };
enum { SVO_ACC_F32 = 0, SVO_ACC_F64 = 1 };

enum { SVO_OK = 0, SVO_ERR_ARG = 1, SVO_ERR_INDEX = 2, SVO_ERR_NOMEM = 3 };

/* multiply-accumulate terms executed by the dot-product loops since the last reset */
static uint64_t g_mac_count = 0;

void svo_reset_mac_count(void) { g_mac_count = 0; }
uint64_t svo_mac_count(void) { return g_mac_count; }

static float elem_f32(const void* base, int dtype, int64_t i) {
    if (dtype == SVO_F32) return ((const float*)base)[i];
    uint32_t bits = (uint32_t)((const uint16_t*)base)[i] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return f;
}

/* round-to-nearest-even float32 -> bfloat16 -> float32 (finite values) */
static float round_through_bf16(float x) {
    uint32_t u;
    memcpy(&u, &x, sizeof u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    u &= 0xFFFF0000u;
    memcpy(&x, &u, sizeof x);
    return x;
}

/* <a[0..n), b[0..n)> for two stored vectors */
static double dot_stored(const void* a, int64_t a0, const void* b, int64_t b0, int dtype,
                         int64_t n, int acc) {
    if (acc == SVO_ACC_F32) {
        float s = 0.0f;
        for (int64_t i = 0; i < n; ++i) {
            float prod = elem_f32(a, dtype, a0 + i) * elem_f32(b, dtype, b0 + i);
            s = s + prod;
        }
        g_mac_count += (uint64_t)n;
        return (double)s;
    }
    double s = 0.0;
    for (int64_t i = 0; i < n; ++i)
        s += (double)elem_f32(a, dtype, a0 + i) * (double)elem_f32(b, dtype, b0 + i);
    g_mac_count += (uint64_t)n;
    return s;
}

/* Section 3.1: z[r, v] = sum_i U[v, i] h[r, i]            out: [rows x V] */
int svo_dense_logits(const void* h, int64_t rows, int64_t d, int64_t ldh,
                     const void* U, int64_t V, int64_t ldu, int dtype, int acc, double* out) {
    if (!h || !U || !out || rows < 1 || d < 1 || V < 1 || ldh < d || ldu < d) return SVO_ERR_ARG;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t v = 0; v < V; ++v)
            out[r * V + v] = dot_stored(U, v * ldu, h, r * ldh, dtype, d, acc);
    return SVO_OK;
}

/* Section 3.3 Step 3: z'[r, j] = sum_i U[idx(r, j), i] h[r, i]    out: [rows x k]
 * idx is [rows x k] (per row) or [k] (one set for the whole step).
 * Variable subset sizes inside fixed-size lists (Section 3.3 Step 2 lets k vary): an entry -1 is a
 * padding slot, it names no token and its logit is -inf. */
int svo_subset_logits(const void* h, int64_t rows, int64_t d, int64_t ldh,
                      const void* U, int64_t V, int64_t ldu, int dtype,
                      const int32_t* idx, int64_t k, int idx_mode, int acc, double* out) {
    if (!h || !U || !idx || !out || rows < 1 || d < 1 || V < 1 || k < 1 || ldh < d || ldu < d)
        return SVO_ERR_ARG;
    for (int64_t r = 0; r < rows; ++r) {
        const int32_t* row_idx = (idx_mode == SVO_IDX_PER_STEP) ? idx : idx + r * k;
        for (int64_t j = 0; j < k; ++j) {
            int64_t tok = row_idx[j];
            if (tok == -1) {                      /* padding slot: no token, logit -inf */
                out[r * k + j] = -INFINITY;
                continue;
            }
            if (tok < 0 || tok >= V) return SVO_ERR_INDEX;
            out[r * k + j] = dot_stored(U, tok * ldu, h, r * ldh, dtype, d, acc);
        }
    }
    return SVO_OK;
}

typedef struct {
    double score;
    int32_t tok;
} scored_t;

/* descending score, then ascending token id */
static int by_score_then_id(const void* pa, const void* pb) {
    const scored_t* a = (const scored_t*)pa;
    const scored_t* b = (const scored_t*)pb;
    if (a->score > b->score) return -1;
    if (a->score < b->score) return 1;
    if (a->tok < b->tok) return -1;
    if (a->tok > b->tok) return 1;
    return 0;
}

static int by_int32(const void* pa, const void* pb) {
    int32_t a = *(const int32_t*)pa, b = *(const int32_t*)pb;
    return (a > b) - (a < b);
}

/* Section 3.3 Steps 1 and 2.
 *   h'[r, j] = sum_i W_down[j, i] h[r, i]            (W_down is [d' x d])
 *   s[r, v]  = sum_j W_vocab[v, j] h'[r, j]          (W_vocab is [V x d'])
 *   idx_out[r, :] = ids of the k largest s[r, :], ascending id order
 * With a finite tau the selected tokens scoring below tau are replaced by padding slots (-1, score
 * -inf) in place, so the list keeps its length and its id order.
 * Optional outputs (may be NULL): scores_out [rows x k] = s at idx_out;
 * s_full_out [rows x V]; hprime_out [rows x d'] (the values fed to the second projection). */
int svo_select(const void* h, int64_t rows, int64_t d, int64_t ldh,
               const void* W_down, int64_t d_prime, const void* W_vocab, int64_t V,
               int dtype, int hprime_round, int acc, int64_t k, double tau,
               int32_t* idx_out, double* scores_out, double* s_full_out, double* hprime_out) {
    if (!h || !W_down || !W_vocab || !idx_out || rows < 1 || d < 1 || d_prime < 1 || V < 1 ||
        k < 1 || k > V || ldh < d)
        return SVO_ERR_ARG;
    double* hp = (double*)malloc(sizeof(double) * (size_t)d_prime);
    double* s = (double*)malloc(sizeof(double) * (size_t)V);
    scored_t* order = (scored_t*)malloc(sizeof(scored_t) * (size_t)V);
    if (!hp || !s || !order) {
        free(hp); free(s); free(order);
        return SVO_ERR_NOMEM;
    }
    for (int64_t r = 0; r < rows; ++r) {
        /* Step 1a: down-projection */
        for (int64_t j = 0; j < d_prime; ++j) {
            double v = dot_stored(W_down, j * d, h, r * ldh, dtype, d, acc);
            if (hprime_round) v = (double)round_through_bf16((float)v);
            hp[j] = v;
            if (hprime_out) hprime_out[r * d_prime + j] = v;
        }
        /* Step 1b: approximate logits over the whole vocabulary */
        for (int64_t v = 0; v < V; ++v) {
            if (acc == SVO_ACC_F32) {
                float a = 0.0f;
                for (int64_t j = 0; j < d_prime; ++j) {
                    float prod = elem_f32(W_vocab, dtype, v * d_prime + j) * (float)hp[j];
                    a = a + prod;
                }
                s[v] = (double)a;
            } else {
                double a = 0.0;
                for (int64_t j = 0; j < d_prime; ++j)
                    a += (double)elem_f32(W_vocab, dtype, v * d_prime + j) * hp[j];
                s[v] = a;
            }
            g_mac_count += (uint64_t)d_prime;
            if (s_full_out) s_full_out[r * V + v] = s[v];
        }
        /* Step 2: full sort, keep the first k, report them in ascending id order */
        for (int64_t v = 0; v < V; ++v) {
            order[v].score = s[v];
            order[v].tok = (int32_t)v;
        }
        qsort(order, (size_t)V, sizeof(scored_t), by_score_then_id);
        int32_t* dst = idx_out + r * k;
        for (int64_t j = 0; j < k; ++j) dst[j] = order[j].tok;
        qsort(dst, (size_t)k, sizeof(int32_t), by_int32);
        /* variable subset size: of the k best, only those scoring at least tau stay; the others
         * become padding slots (tau = -inf keeps all k) */
        for (int64_t j = 0; j < k; ++j) {
            const double sc = s[dst[j]];
            const int keep = sc >= tau;
            if (scores_out) scores_out[r * k + j] = keep ? sc : -INFINITY;
            if (!keep) dst[j] = -1;
        }
    }
    free(hp); free(s); free(order);
    return SVO_OK;
}

/* Subset softmax and draft tokens.
 *   q[r, j] = exp(z'[r, j] - m_r) / sum_l exp(z'[r, l] - m_r),  m_r = max_j z'[r, j]
 *   (tok_out[r, t], prob_out[r, t]) for t = 0..kd-1: the kd entries with the largest
 *   logit, best first, ties -> smaller token id; tok_out holds vocabulary ids idx(r, j).
 * logits: [rows x k] float32 (the precision the logits are handed over in).
 * Optional: probs_full_out [rows x k]. */
int svo_softmax_topk(const float* logits, const int32_t* idx, int idx_mode,
                     int64_t rows, int64_t k, int64_t kd,
                     int32_t* tok_out, double* prob_out, double* probs_full_out) {
    if (!logits || !idx || !tok_out || !prob_out || rows < 1 || k < 1 || kd < 1 || kd > k)
        return SVO_ERR_ARG;
    scored_t* order = (scored_t*)malloc(sizeof(scored_t) * (size_t)k);
    if (!order) return SVO_ERR_NOMEM;
    for (int64_t r = 0; r < rows; ++r) {
        const float* z = logits + r * k;
        const int32_t* row_idx = (idx_mode == SVO_IDX_PER_STEP) ? idx : idx + r * k;
        double m = (double)z[0];
        for (int64_t j = 1; j < k; ++j)
            if ((double)z[j] > m) m = (double)z[j];
        /* padding slots carry -inf: probability 0; a row of nothing but padding has all probabilities 0 */
        const int empty = isinf(m) && m < 0;
        double denom = 0.0;
        for (int64_t j = 0; j < k; ++j) denom += empty ? 0.0 : exp((double)z[j] - m);
        for (int64_t j = 0; j < k; ++j) {
            order[j].score = (double)z[j];
            order[j].tok = row_idx[j];
            if (probs_full_out) probs_full_out[r * k + j] = empty ? 0.0 : exp((double)z[j] - m) / denom;
        }
        qsort(order, (size_t)k, sizeof(scored_t), by_score_then_id);
        for (int64_t t = 0; t < kd; ++t) {
            tok_out[r * kd + t] = order[t].tok;
            prob_out[r * kd + t] = empty ? 0.0 : exp(order[t].score - m) / denom;
        }
    }
    free(order);
    return SVO_OK;
}

/* Section 3.4: the vocabulary speculator's own distribution q_aux = softmax(s) over the whole
 * vocabulary, returned as log-probabilities:
 *   out[r, v] = s[r, v] - m_r - log( sum_u exp(s[r, u] - m_r) ),  m_r = max_u s[r, u]
 * s, out: [rows x V] double (s as produced by svo_select's s_full_out). */
int svo_log_softmax(const double* s, int64_t rows, int64_t V, double* out) {
    if (!s || !out || rows < 1 || V < 1) return SVO_ERR_ARG;
    for (int64_t r = 0; r < rows; ++r) {
        const double* x = s + r * V;
        double m = x[0];
        for (int64_t v = 1; v < V; ++v)
            if (x[v] > m) m = x[v];
        double denom = 0.0;
        for (int64_t v = 0; v < V; ++v) denom += exp(x[v] - m);
        const double lse = m + log(denom);
        for (int64_t v = 0; v < V; ++v) out[r * V + v] = x[v] - lse;
    }
    return SVO_OK;
}
