/*
 * FastOCR decode hot path -- CPU oracle.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, fp64 transcription of the paper's definitions.  Only the test
 * suite, the smoke check and the benchmark's CPU-baseline leg may call it; the
 * product path (the HIP library) shares no code with this file and never
 * routes through it.
 *
 * What is written out here:
 *   - head-averaged attention distribution of a focal layer: softmax over the
 *     WHOLE cache per query head, mean over query heads, read off at the image
 *     positions (Sec. 3.1.1, Eq. 1 and the text under Eq. 2; softmax attention
 *     of App. B);
 *   - the image-attention ratio of Eq. 1 (sum of that distribution over image
 *     positions; its denominator is 1 because the softmax runs over I u T);
 *   - TopK_{ceil(tau N)} over image tokens (Sec. 3.1.2);
 *   - attention restricted to the kept set K = T u F (Eq. 2, non-focal branch)
 *     and attention over the full cache (Eq. 2, focal branch).
 *
 * No online softmax, no splitting, no thresholds: every logit is materialised,
 * the softmax is the two-pass textbook one, top-k is a full sort.
 * Where the paper is silent the readings are: scale = argument (1/sqrt(head
 * dim) by default in the callers); GQA query head h reads KV head h / (Hq/Hkv);
 * mean (not sum) over query heads; ties broken towards the lower index.
 *
 * Pins (tests/test_oracle_*.py): pure-Python brute force on tiny inputs,
 * closed forms (identical keys, planted key), softmax shift invariance,
 * GQA == replicated MHA, tau=1 == dense, tau=0 == text only, a library
 * softmax-attention in fp64 on explicitly gathered rows, the LSE merge
 * identity, exact rational arithmetic for ceil(tau N).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F32 = 0, ORC_BF16 = 1 };

/* One layer's cache as the oracle sees it (host memory). Strides in elements. */
typedef struct {
    const void *k;
    const void *v;
    int32_t dtype;
    int32_t n_kv_heads;
    int32_t head_dim;
    int64_t stride_token;
    int64_t stride_head;
    int64_t stride_seq;      /* contiguous mode: offset between sequences      */
    int32_t page_tokens;     /* 0: contiguous; else tokens per page            */
    int64_t stride_page;
    const int32_t *block_table; /* [B, max_pages_per_seq]                      */
    int32_t max_pages_per_seq;
} orc_kv;

static double widen(const void *base, int dtype, int64_t idx)
{
    if (dtype == ORC_F32) {
        return (double)((const float *)base)[idx];
    } else {
        uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
}

/* element offset of (sequence b, token j, kv head g, component 0) */
static int64_t row_offset(const orc_kv *kv, int b, int64_t j, int g)
{
    if (kv->page_tokens > 0) {
        int64_t page = kv->block_table[(int64_t)b * kv->max_pages_per_seq + j / kv->page_tokens];
        return page * kv->stride_page + (j % kv->page_tokens) * kv->stride_token
             + (int64_t)g * kv->stride_head;
    }
    return (int64_t)b * kv->stride_seq + j * kv->stride_token + (int64_t)g * kv->stride_head;
}

/* ceil(tau * N): the size of the focal token set (Sec. 3.1.2).  tau*N is
 * formed in double; a product that lands a hair above an integer only through
 * the rounding of tau (0.05 * 20 -> 1.0000000000000002) must not bump the
 * count, hence the 1e-9 guard.  Clamped to [0, N]. */
int64_t orc_keep_count(int64_t n_visual, double tau)
{
    if (n_visual <= 0 || !(tau > 0.0)) return 0;
    double x = ceil(tau * (double)n_visual - 1e-9);
    if (x < 0.0) x = 0.0;
    if (x > (double)n_visual) x = (double)n_visual;
    return (int64_t)x;
}

/* logits of query head h of sequence b against tokens [0, S): scale * <q, k_j> */
static void all_logits(const orc_kv *kv, const void *q, int n_q_heads, int b, int h,
                       int64_t S, double scale, double *logit)
{
    const int d = kv->head_dim;
    const int G = n_q_heads / kv->n_kv_heads;
    const int g = h / G;
    const int64_t qoff = ((int64_t)b * n_q_heads + h) * d;
    for (int64_t j = 0; j < S; ++j) {
        const int64_t ko = row_offset(kv, b, j, g);
        double acc = 0.0;
        for (int c = 0; c < d; ++c)
            acc += widen(q, kv->dtype, qoff + c) * widen(kv->k, kv->dtype, ko + c);
        logit[j] = scale * acc;
    }
}

/*
 * Head-averaged attention distribution at a focal layer, read at image tokens.
 *   scores[b*max_vis + i] = (1/Hq) sum_h softmax_j(logit_h)[vis_start_b + i]
 *   lse[b*Hq + h]         = log sum_j exp(logit_h[j])           (optional)
 *   img_mass[b]           = sum_i scores[b, i]  (= r of Eq. 1)  (optional)
 * Rows of `scores` beyond vis_len[b] are left untouched.
 */
int orc_focal_score(const orc_kv *kv, int batch, const int32_t *seq_len,
                    const int32_t *vis_start, const int32_t *vis_len,
                    const void *q, int n_q_heads, double scale,
                    double *scores, int64_t max_vis, double *lse, double *img_mass,
                    int n_threads)
{
    if (n_q_heads % kv->n_kv_heads) return -1;
    if (n_threads < 1) n_threads = 1;
    for (int b = 0; b < batch; ++b) {
        const int64_t S = seq_len[b], N = vis_len[b], v0 = vis_start[b];
        if (v0 < 0 || N < 0 || v0 + N > S) return -1;
        for (int64_t i = 0; i < N; ++i) scores[(int64_t)b * max_vis + i] = 0.0;
        /* per-head probabilities, then the mean over heads */
        double *prob = (double *)malloc(sizeof(double) * (size_t)n_q_heads * (size_t)(S > 0 ? S : 1));
        if (!prob) return -2;
#pragma omp parallel for num_threads(n_threads) schedule(static)
        for (int h = 0; h < n_q_heads; ++h) {
            double *p = prob + (int64_t)h * S;
            all_logits(kv, q, n_q_heads, b, h, S, scale, p);
            double mx = -INFINITY;
            for (int64_t j = 0; j < S; ++j) if (p[j] > mx) mx = p[j];
            double z = 0.0;
            for (int64_t j = 0; j < S; ++j) z += exp(p[j] - mx);
            if (lse) lse[(int64_t)b * n_q_heads + h] = (S > 0) ? mx + log(z) : -INFINITY;
            for (int64_t j = 0; j < S; ++j) p[j] = exp(p[j] - mx) / z;
        }
        double mass = 0.0;
        for (int64_t i = 0; i < N; ++i) {
            double s = 0.0;
            for (int h = 0; h < n_q_heads; ++h) s += prob[(int64_t)h * S + v0 + i];
            s /= (double)n_q_heads;
            scores[(int64_t)b * max_vis + i] = s;
            mass += s;
        }
        if (img_mass) img_mass[b] = mass;
        free(prob);
    }
    return 0;
}

typedef struct { double s; int32_t i; } orc_pair;

static int by_score_desc_then_index(const void *a, const void *b)
{
    const orc_pair *x = (const orc_pair *)a, *y = (const orc_pair *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->i > y->i) - (x->i < y->i);
}

static int by_int(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/*
 * TopK over one sequence's image scores: full sort by (score descending, index
 * ascending), first k kept, returned ascending by index.  Returns k.
 */
int64_t orc_topk(const double *scores, int64_t n, int64_t k, int32_t *out_idx)
{
    if (k > n) k = n;
    if (k <= 0) return 0;
    orc_pair *p = (orc_pair *)malloc(sizeof(orc_pair) * (size_t)n);
    if (!p) return -2;
    for (int64_t i = 0; i < n; ++i) { p[i].s = scores[i]; p[i].i = (int32_t)i; }
    qsort(p, (size_t)n, sizeof(orc_pair), by_score_desc_then_index);
    for (int64_t r = 0; r < k; ++r) out_idx[r] = p[r].i;
    qsort(out_idx, (size_t)k, sizeof(int32_t), by_int);
    free(p);
    return k;
}

/*
 * Decode attention of every query head over an explicit token set J.
 *   sel_idx == NULL : J = [0, S)                       (Eq. 2, focal branch)
 *   else            : J = {j outside the image span} u {vis_start + sel_idx[b, r]}
 *                                                       (Eq. 2, non-focal branch)
 *   out[(b*Hq + h)*d + c] = sum_{j in J} softmax_{J}(logit_h)[j] * V[kv(h), j, c]
 *   lse[b*Hq + h]         = log sum_{j in J} exp(logit_h[j])   (optional)
 * An empty J gives a zero row and lse = -inf.
 */
int orc_decode_attn(const orc_kv *kv, int batch, const int32_t *seq_len,
                    const int32_t *vis_start, const int32_t *vis_len,
                    const void *q, int n_q_heads, double scale,
                    const int32_t *sel_idx, const int32_t *sel_cnt, int64_t kmax,
                    double *out, double *lse, int n_threads)
{
    if (n_q_heads % kv->n_kv_heads) return -1;
    if (n_threads < 1) n_threads = 1;
    const int d = kv->head_dim;
    const int G = n_q_heads / kv->n_kv_heads;
    int status = 0;
    for (int b = 0; b < batch; ++b) {
        const int64_t S = seq_len[b], N = vis_len[b], v0 = vis_start[b];
        if (v0 < 0 || N < 0 || v0 + N > S) return -1;
        /* membership mask of J */
        unsigned char *in_set = (unsigned char *)malloc((size_t)(S > 0 ? S : 1));
        if (!in_set) return -2;
        if (!sel_idx) {
            memset(in_set, 1, (size_t)S);
        } else {
            for (int64_t j = 0; j < S; ++j) in_set[j] = (j < v0 || j >= v0 + N) ? 1 : 0;
            for (int64_t r = 0; r < sel_cnt[b]; ++r) {
                int64_t i = sel_idx[(int64_t)b * kmax + r];
                if (i < 0 || i >= N) { status = -1; break; }
                in_set[v0 + i] = 1;
            }
        }
        if (status) { free(in_set); return status; }
#pragma omp parallel for num_threads(n_threads) schedule(static)
        for (int h = 0; h < n_q_heads; ++h) {
            const int g = h / G;
            double *logit = (double *)malloc(sizeof(double) * (size_t)(S > 0 ? S : 1));
            double *o = out + ((int64_t)b * n_q_heads + h) * d;
            all_logits(kv, q, n_q_heads, b, h, S, scale, logit);
            double mx = -INFINITY;
            for (int64_t j = 0; j < S; ++j) if (in_set[j] && logit[j] > mx) mx = logit[j];
            double z = 0.0;
            for (int64_t j = 0; j < S; ++j) if (in_set[j]) z += exp(logit[j] - mx);
            for (int c = 0; c < d; ++c) o[c] = 0.0;
            for (int64_t j = 0; j < S; ++j) {
                if (!in_set[j]) continue;
                const double w = exp(logit[j] - mx) / z;
                const int64_t vo = row_offset(kv, b, j, g);
                for (int c = 0; c < d; ++c) o[c] += w * widen(kv->v, kv->dtype, vo + c);
            }
            if (lse) lse[(int64_t)b * n_q_heads + h] = (z > 0.0) ? mx + log(z) : -INFINITY;
            free(logit);
        }
        free(in_set);
    }
    return 0;
}

int orc_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
