/*
 * CPU oracle for RainFusion's sparse 3D attention and its ARM head classifier.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU
 * library is checked against; nothing in the product path may call it, and it
 * shares no code with the HIP implementation.  All arithmetic is fp64 on the
 * fp32 input values it is handed (the callers hand it bf16-rounded values, so
 * both sides see identical inputs).
 *
 * What it follows (RainFusion, arxiv 2505.21036):
 *   - token layout, Sec. 3.1: the sequence is T frame sub-sequences of H*W
 *     tokens each; optional text tokens are appended after the video tokens
 *     (or, with text_first set, placed in front of them: the paper does not say
 *     where a model's prompt tokens sit, and models differ);
 *   - masked softmax attention, Eq. 1-2;
 *   - the three pattern masks of Sec. 3.2 (Spatial Eq. 3, Temporal, Textural
 *     Eq. 4-5) written as one token-level predicate rfo_keep();
 *   - the masked attention recall of Eq. 6 and the decision rule of Alg. 1.
 *
 * Readings taken where the paper is silent or garbled (each also listed in the
 * design notes of the repository):
 *   - Spatial: query frame f attends every token of frames f' with
 *     |f - f'| <= floor(bw_spatial * T)  (a band over frames: the frames next to f);
 *   - Temporal: with p the index of a token inside its frame, query p attends
 *     p' with |p - p'| <= floor(bw_temporal * H*W) in every frame (local inside
 *     a frame sub-sequence, periodic over the sequence);
 *   - Textural: keys at (row y, col x) of any frame are kept iff
 *     (y - x) mod tau == 0  (Eq. 4 read as "i and j share their residue");
 *     queries are never dropped (Eq. 5, all-zero mask on the kept keys);
 *   - text tokens attend and are attended densely under every pattern and are
 *     never part of an ARM sample;
 *   - Eq. 6 is read per query row: recall = mean over sampled rows of the
 *     softmax mass that falls on kept sampled keys;
 *   - global sampling interval omega defaults to T (|sample| ~= H*W, the
 *     overhead falling with the square of the frame count that Sec. 1 states);
 *   - ">=" at the threshold, Temporal tested first (Alg. 1).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { RFO_SPATIAL = 0, RFO_TEMPORAL = 1, RFO_TEXTURAL = 2, RFO_DENSE = 3 };
enum { RFO_SAMPLE_FIRST_FRAME = 0, RFO_SAMPLE_EQUAL_INTERVAL = 1 };

typedef struct {
    int32_t T, H, W, text_len;
} rfo_layout;

typedef struct {
    double bw_spatial, bw_temporal; /* band half-widths as fractions of T and of H*W */
    int32_t tex_stride;             /* tau of Eq. 4 */
    int32_t sample_interval;        /* omega of Sec. 3.3; <= 0 means T */
    int32_t two_head;               /* ablation of Sec. 4.2 / Tab. 2: only Spatial and Temporal heads are sparse,
                                       every other head is computed densely */
    int32_t text_first;             /* the text tokens are tokens 0 .. text_len-1 and the video follows */
} rfo_params;

static int64_t n_video(const rfo_layout *L) { return (int64_t)L->T * L->H * L->W; }
int64_t rfo_num_tokens(const rfo_layout *L) { return n_video(L) + L->text_len; }

/* Band half-width in whole units: floor(bw * n), never negative. */
int64_t rfo_radius(double bw, int64_t n)
{
    double r = floor(bw * (double)n);
    if (r < 0) r = 0;
    if (r > (double)n) r = (double)n;
    return (int64_t)r;
}

/* Index of token n among the video tokens (frame-major order of Sec. 3.1), or -1 for a text token. */
static int64_t video_index(int64_t n, const rfo_layout *L, const rfo_params *P)
{
    if (P->text_first) return n < L->text_len ? -1 : n - L->text_len;
    return n < n_video(L) ? n : -1;
}

/* Sec. 3.2 as one predicate: does query token i see key token j under pattern cls? */
int rfo_keep(int cls, int64_t i, int64_t j, const rfo_layout *L, const rfo_params *P)
{
    const int64_t HW = (int64_t)L->H * L->W;
    if (cls == RFO_DENSE) return 1;
    i = video_index(i, L, P);
    j = video_index(j, L, P);
    if (i < 0 || j < 0) return 1; /* text rows and text columns stay dense */
    const int64_t fi = i / HW, pi = i % HW, fj = j / HW, pj = j % HW;
    if (cls == RFO_SPATIAL) {
        int64_t r = rfo_radius(P->bw_spatial, L->T);
        return llabs(fi - fj) <= r;
    }
    if (cls == RFO_TEMPORAL) {
        int64_t r = rfo_radius(P->bw_temporal, HW);
        return llabs(pi - pj) <= r;
    }
    if (cls == RFO_TEXTURAL) {
        int64_t y = pj / L->W, x = pj % L->W, tau = P->tex_stride;
        int64_t m = (y - x) % tau;
        return m == 0;
    }
    return 0;
}

static double dot_scaled(const float *q, const float *k, int D)
{
    double acc = 0.0;
#pragma omp simd reduction(+ : acc)
    for (int d = 0; d < D; ++d) acc += (double)q[d] * (double)k[d];
    return acc / sqrt((double)D);
}

/*
 * Eq. 1-2, one head, the dense "mask as minus infinity" form, for the query
 * rows listed in rows[] (every row is independent, so a subset is exact).
 *   Q,K,V : [N, D] fp32, row-major.   O : [nrows, D] fp64.
 *   Prob  : optional [nrows, N] fp64, the softmax row S(Q,K,M) itself.
 */
void rfo_attention_rows(const float *Q, const float *K, const float *V, int D, int cls,
                        const rfo_layout *L, const rfo_params *P, const int64_t *rows,
                        int64_t nrows, double *O, double *Prob)
{
    const int64_t N = rfo_num_tokens(L);
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)N);
#pragma omp for schedule(dynamic, 4)
        for (int64_t a = 0; a < nrows; ++a) {
            const int64_t i = rows[a];
            double m = -INFINITY;
            for (int64_t j = 0; j < N; ++j) {
                /* QK^T/sqrt(d) + M with M in {0, -inf} */
                s[j] = rfo_keep(cls, i, j, L, P) ? dot_scaled(Q + i * D, K + j * D, D) : -INFINITY;
                if (s[j] > m) m = s[j];
            }
            double denom = 0.0;
            for (int64_t j = 0; j < N; ++j) {
                s[j] = exp(s[j] - m); /* exp(-inf) = 0 for masked entries */
                denom += s[j];
            }
            for (int d = 0; d < D; ++d) O[a * D + d] = 0.0;
            for (int64_t j = 0; j < N; ++j) {
                const double p = s[j] / denom;
                if (Prob) Prob[a * N + j] = p;
                if (p != 0.0)
                    for (int d = 0; d < D; ++d) O[a * D + d] += p * (double)V[j * D + d];
            }
        }
        free(s);
    }
}

/*
 * The same attention computed the way a block-skipping kernel would organise
 * it, with its own enumeration of blocks: a (query block, key block) pair is
 * visited only if some token pair inside it is kept.  Used to show that
 * skipping blocks changes nothing.  O : [N, D] fp64.  Returns, through
 * visited/total, how many block pairs were visited out of how many exist.
 */
void rfo_attention_blockskip(const float *Q, const float *K, const float *V, int D, int cls,
                             const rfo_layout *L, const rfo_params *P, int block, double *O,
                             int64_t *visited, int64_t *total)
{
    const int64_t N = rfo_num_tokens(L);
    const int64_t nb = (N + block - 1) / block;
    char *live = (char *)calloc((size_t)(nb * nb), 1);
    int64_t nvis = 0;
    for (int64_t qb = 0; qb < nb; ++qb)
        for (int64_t kb = 0; kb < nb; ++kb) {
            int any = 0;
            for (int64_t i = qb * block; i < N && i < (qb + 1) * block && !any; ++i)
                for (int64_t j = kb * block; j < N && j < (kb + 1) * block; ++j)
                    if (rfo_keep(cls, i, j, L, P)) { any = 1; break; }
            live[qb * nb + kb] = (char)any;
            nvis += any;
        }
    if (visited) *visited = nvis;
    if (total) *total = nb * nb;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t i = 0; i < N; ++i) {
        const int64_t qb = i / block;
        /* pass 1: row maximum over visited blocks */
        double m = -INFINITY;
        for (int64_t kb = 0; kb < nb; ++kb) {
            if (!live[qb * nb + kb]) continue;
            for (int64_t j = kb * block; j < N && j < (kb + 1) * block; ++j)
                if (rfo_keep(cls, i, j, L, P)) {
                    double s = dot_scaled(Q + i * D, K + j * D, D);
                    if (s > m) m = s;
                }
        }
        /* pass 2: numerator and denominator over visited blocks */
        double denom = 0.0;
        for (int d = 0; d < D; ++d) O[i * D + d] = 0.0;
        for (int64_t kb = 0; kb < nb; ++kb) {
            if (!live[qb * nb + kb]) continue;
            for (int64_t j = kb * block; j < N && j < (kb + 1) * block; ++j)
                if (rfo_keep(cls, i, j, L, P)) {
                    double e = exp(dot_scaled(Q + i * D, K + j * D, D) - m);
                    denom += e;
                    for (int d = 0; d < D; ++d) O[i * D + d] += e * (double)V[j * D + d];
                }
        }
        for (int d = 0; d < D; ++d) O[i * D + d] /= denom;
    }
    free(live);
}

/* Sec. 3.3 sampling: the token index of sample a.  Local = first frame,
 * global = every omega-th video token.  Returns the number of samples. */
int64_t rfo_sample_count(const rfo_layout *L, const rfo_params *P, int global)
{
    const int64_t HW = (int64_t)L->H * L->W, Nv = n_video(L);
    if (!global) return HW;
    const int64_t w = P->sample_interval > 0 ? P->sample_interval : L->T;
    return (Nv + w - 1) / w;
}
int64_t rfo_sample_token(const rfo_layout *L, const rfo_params *P, int global, int64_t a)
{
    const int64_t first_video = P->text_first ? L->text_len : 0; /* samples are video tokens */
    if (!global) return first_video + a;
    const int64_t w = P->sample_interval > 0 ? P->sample_interval : L->T;
    return first_video + a * w;
}

/*
 * Eq. 6 on one head: Q', K' are the sampled rows of Q, K; M' is the pattern
 * mask cls restricted to sampled rows and columns.  For every sampled query
 * the softmax over ALL sampled keys (M_init) is formed and the share of it
 * that lands on kept keys is that row's recall; the head's recall is the mean
 * over sampled rows.  row_recall (optional) receives the per-row values.
 */
double rfo_arm_recall(const float *Q, const float *K, int D, const rfo_layout *L,
                      const rfo_params *P, int global, int cls, double *row_recall)
{
    const int64_t n = rfo_sample_count(L, P, global);
    double *rr = (double *)malloc(sizeof(double) * (size_t)n);
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)n);
#pragma omp for schedule(static)
        for (int64_t a = 0; a < n; ++a) {
            const int64_t i = rfo_sample_token(L, P, global, a);
            double m = -INFINITY;
            for (int64_t b = 0; b < n; ++b) {
                const int64_t j = rfo_sample_token(L, P, global, b);
                s[b] = dot_scaled(Q + i * D, K + j * D, D);
                if (s[b] > m) m = s[b];
            }
            double all = 0.0, kept = 0.0;
            for (int64_t b = 0; b < n; ++b) {
                const int64_t j = rfo_sample_token(L, P, global, b);
                const double e = exp(s[b] - m);
                all += e;
                if (rfo_keep(cls, i, j, L, P)) kept += e;
            }
            rr[a] = kept / all;
        }
        free(s);
    }
    double total = 0.0; /* summed in row order so the result does not depend on threading */
    for (int64_t a = 0; a < n; ++a) {
        total += rr[a];
        if (row_recall) row_recall[a] = rr[a];
    }
    free(rr);
    return total / (double)n;
}

/*
 * Alg. 1 on one head.  recalls[0] = R-hat (Temporal mask; first-frame samples
 * in FIRST_FRAME mode, equal-interval samples in EQUAL_INTERVAL mode),
 * recalls[1] = R-tilde (Spatial mask, always equal-interval samples).
 */
int rfo_arm_classify(const float *Q, const float *K, int D, const rfo_layout *L,
                     const rfo_params *P, int sample_mode, double alpha, double *recalls)
{
    const double r_hat =
        rfo_arm_recall(Q, K, D, L, P, sample_mode == RFO_SAMPLE_EQUAL_INTERVAL, RFO_TEMPORAL, NULL);
    const double r_tilde = rfo_arm_recall(Q, K, D, L, P, 1, RFO_SPATIAL, NULL);
    if (recalls) { recalls[0] = r_hat; recalls[1] = r_tilde; }
    if (r_hat >= alpha) return RFO_TEMPORAL; /* Temporal has priority */
    if (r_tilde >= alpha) return RFO_SPATIAL;
    return P->two_head ? RFO_DENSE : RFO_TEXTURAL;
}

/*
 * RainFusion+ (Sec. 4.3: every head gets the narrowest of the candidate bandwidths 0.5, 0.25,
 * 0.125 whose recall still reaches 90 %), one head.  The recalls of
 * Alg. 1 are evaluated once per candidate bandwidth bws[k] (the Temporal recall with
 * bw_temporal = bws[k], the Spatial recall with bw_spatial = bws[k]).  Reading taken: Alg. 1's
 * order is kept -- if any candidate gives R-hat >= alpha the head is Temporal with the smallest
 * such bandwidth; else if any gives R-tilde >= alpha it is Spatial with the smallest such
 * bandwidth; else Textural (*bw_index = -1).
 * recalls (optional): [2][n_bw], row 0 = R-hat per candidate, row 1 = R-tilde per candidate.
 */
int rfo_arm_classify_plus(const float *Q, const float *K, int D, const rfo_layout *L, const rfo_params *P,
                          int sample_mode, double alpha, const double *bws, int n_bw, int *bw_index,
                          double *recalls)
{
    int best_t = -1, best_s = -1;
    for (int k = 0; k < n_bw; ++k) {
        rfo_params pk = *P;
        pk.bw_temporal = bws[k];
        pk.bw_spatial = bws[k];
        const double r_hat =
            rfo_arm_recall(Q, K, D, L, &pk, sample_mode == RFO_SAMPLE_EQUAL_INTERVAL, RFO_TEMPORAL, NULL);
        const double r_tilde = rfo_arm_recall(Q, K, D, L, &pk, 1, RFO_SPATIAL, NULL);
        if (recalls) { recalls[k] = r_hat; recalls[n_bw + k] = r_tilde; }
        if (r_hat >= alpha && (best_t < 0 || bws[k] < bws[best_t])) best_t = k;
        if (r_tilde >= alpha && (best_s < 0 || bws[k] < bws[best_s])) best_s = k;
    }
    if (best_t >= 0) { *bw_index = best_t; return RFO_TEMPORAL; }
    if (best_s >= 0) { *bw_index = best_s; return RFO_SPATIAL; }
    *bw_index = -1;
    return P->two_head ? RFO_DENSE : RFO_TEXTURAL;
}

/* The decision rule alone, for truth-table tests. */
int rfo_decide(double r_hat, double r_tilde, double alpha)
{
    if (r_hat >= alpha) return RFO_TEMPORAL;
    if (r_tilde >= alpha) return RFO_SPATIAL;
    return RFO_TEXTURAL;
}

/* Fraction of (query, key) token pairs kept under cls, by plain counting. */
double rfo_kept_fraction(int cls, const rfo_layout *L, const rfo_params *P)
{
    const int64_t N = rfo_num_tokens(L);
    int64_t kept = 0;
#pragma omp parallel for reduction(+ : kept) schedule(static)
    for (int64_t i = 0; i < N; ++i)
        for (int64_t j = 0; j < N; ++j) kept += rfo_keep(cls, i, j, L, P);
    return (double)kept / ((double)N * (double)N);
}

/* The whole N x N mask of pattern cls as bytes (1 = kept), by calling the predicate pair by pair. */
void rfo_keep_matrix(int cls, const rfo_layout *L, const rfo_params *P, uint8_t *out)
{
    const int64_t N = rfo_num_tokens(L);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; ++i)
        for (int64_t j = 0; j < N; ++j) out[i * N + j] = (uint8_t)rfo_keep(cls, i, j, L, P);
}
