/*
 * hg_oracle.c -- TEST INFRASTRUCTURE ONLY.  Plain fp64 CPU oracle for partitioned decode
 * attention.  It is linked by the tests, by the smoke check and by the benchmark's CPU-baseline
 * leg; the product library never calls it and shares no code, header or table with it.
 *
 * What it computes follows the paper's statement of decode attention and of its token-axis split:
 *   - logits  s_j = scale * (q . k_j), softmax over every cached token, weighted sum of the
 *     value rows (Section 2.1, where d is the per-head dimension; Section 4.2 first
 *     paragraph).  The new token's K and V are already in the cache (Section 2.1), so no
 *     mask is applied.
 *   - the logit stage is independent per token, so the cache may be cut into positional ranges
 *     that are processed separately (Section 4.2; Section 4.2.3, Token Mapper).
 *   - the split result must equal monolithic execution (Section 4.2.3, Token Concatenator;
 *     Section 4.6 step 5).
 *
 * Four routines:
 *   hgo_attn_full     the definition, two passes (max, then sums), over [0, N_b).
 *   hgo_attn_partial  per range: m = max_j s_j, l = sum_j exp(s_j - m), O = sum_j exp(s_j - m) v_j.
 *   hgo_attn_merge    M = max_p m_p; w_p = exp(m_p - M) (0 when l_p == 0); L = sum w_p l_p;
 *                     out = sum w_p O_p / L; lse = M + log L.
 *   hgo_attn_concat   the paper-literal route: raw logits per range, concatenated in ascending
 *                     token order, ONE global softmax, then P.V (Section 4.6 step 5).
 *
 *   hgo_attn_logits   the raw scaled logits of each range, the quantity an executor ships in the
 *                     paper's own wire format (Section 4.2.2, Logits Calculator).
 *   hgo_attn_select   Post-QK^T selection (Section 4.3.1; Section 4.5): per (group, query head),
 *                     keep the top_k highest logits of the group's ranges and fold them and their
 *                     V rows into one (m, l, O).  The logits are an INPUT in fp32 (the decision
 *                     which tokens are kept is taken on those fp32 values, as on the GPU); ties
 *                     go to the lower column.
 *   hgo_attn_gather   statistics over a LISTED token set per (group, query head): what an
 *                     executor computes once a selector has named the tokens (Pre-QK^T selection,
 *                     Section 4.3.2; Section 4.6 step 1).
 *
 * All arithmetic is fp64, plain sequential sums in token order, libm exp/log.  Inputs are the
 * caller's fp16 / bf16 / fp32 bit patterns widened exactly; nothing is re-rounded.  The only parallelism
 * is an OpenMP loop over independent (sequence, query head) pairs; there is no blocking, fusion
 * or reordering.
 *
 * Grouped-query attention: query head h reads KV head h / (Hq / Hkv) (contiguous groups).
 * Empty range or empty cache: (m, l, O) = (-inf, 0, 0); a merge whose L is 0 gives out = 0,
 * lse = -inf.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t seq, begin, end;
} hgo_range;

/* Problem description shared by the routines that read the KV cache.
 * dtype: 0 = IEEE binary16 bit patterns (uint16_t), 1 = binary32 (float), 2 = bfloat16 bit patterns
 * (uint16_t: the upper half of a binary32).
 * q is [B][Hq][d] contiguous.  Element (b, g, t, c) of K or V sits at
 * base + b*stride_b + g*stride_h + t*stride_t + c   (strides counted in elements). */
typedef struct {
    const void *q, *k, *v;
    int64_t stride_b, stride_h, stride_t;
    const int32_t *seq_lens; /* [B] */
    int32_t B, Hq, Hkv, d;
    int32_t dtype;
    double scale;
} hgo_problem;

/* ---- exact widening of the storage formats ------------------------------------------------ */

static double half_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int ex = (h >> 10) & 0x1f;
    int man = h & 0x3ff;
    double val;
    if (ex == 0) {
        val = ldexp((double)man, -24); /* zero or subnormal: man * 2^-24 */
    } else if (ex == 31) {
        val = man ? NAN : INFINITY;
    } else {
        val = ldexp((double)(man + 1024), ex - 25); /* (1 + man/1024) * 2^(ex-15) */
    }
    return sign ? -val : val;
}

/* bfloat16 = sign, 8 exponent bits, 7 fraction bits: the value of the binary32 whose upper 16
 * bits are these and whose lower 16 bits are zero. */
static double bf16_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int ex = (h >> 7) & 0xff;
    int man = h & 0x7f;
    double val;
    if (ex == 0) {
        val = ldexp((double)man, -133); /* zero or subnormal: man * 2^-7 * 2^-126 */
    } else if (ex == 255) {
        val = man ? NAN : INFINITY;
    } else {
        val = ldexp((double)(man + 128), ex - 134); /* (1 + man/128) * 2^(ex-127) */
    }
    return sign ? -val : val;
}

static double load_elem(const void *base, int64_t idx, int dtype)
{
    if (dtype == 0) return half_bits_to_double(((const uint16_t *)base)[idx]);
    if (dtype == 2) return bf16_bits_to_double(((const uint16_t *)base)[idx]);
    return (double)((const float *)base)[idx];
}

static int64_t kv_row(const hgo_problem *p, int b, int h, int64_t t)
{
    int G = p->Hq / p->Hkv;
    int g = h / G;
    return (int64_t)b * p->stride_b + (int64_t)g * p->stride_h + t * p->stride_t;
}

/* s_t = scale * sum_c q[b,h,c] * K[b,g,t,c] */
static double logit(const hgo_problem *p, int b, int h, int64_t t)
{
    int64_t qoff = ((int64_t)b * p->Hq + h) * p->d;
    int64_t koff = kv_row(p, b, h, t);
    double acc = 0.0;
    for (int c = 0; c < p->d; ++c)
        acc += load_elem(p->q, qoff + c, p->dtype) * load_elem(p->k, koff + c, p->dtype);
    return p->scale * acc;
}

static int check_problem(const hgo_problem *p)
{
    if (!p || !p->q || !p->k || !p->v || !p->seq_lens) return -1;
    if (p->B < 0 || p->Hq <= 0 || p->Hkv <= 0 || p->d <= 0) return -2;
    if (p->Hq % p->Hkv) return -2;
    if (p->dtype != 0 && p->dtype != 1 && p->dtype != 2) return -3;
    return 0;
}

/* (m, l, O) of tokens [begin, end) for one (b, h).  o has d entries.  Returns 0, or -7 when the
 * logit vector cannot be allocated. */
static int range_stats(const hgo_problem *p, int b, int h, int64_t begin, int64_t end, double *m_out,
                       double *l_out, double *o)
{
    int d = p->d;
    for (int c = 0; c < d; ++c) o[c] = 0.0;
    *m_out = -INFINITY;
    *l_out = 0.0;
    if (end <= begin) return 0;
    int64_t n = end - begin;
    double *s = (double *)malloc(sizeof(double) * (size_t)n);
    if (!s) return -7;
    for (int64_t j = 0; j < n; ++j) s[j] = logit(p, b, h, begin + j);
    double m = s[0];
    for (int64_t j = 1; j < n; ++j)
        if (s[j] > m) m = s[j];
    double l = 0.0;
    for (int64_t j = 0; j < n; ++j) {
        double w = exp(s[j] - m);
        int64_t voff = kv_row(p, b, h, begin + j);
        l += w;
        for (int c = 0; c < d; ++c) o[c] += w * load_elem(p->v, voff + c, p->dtype);
    }
    free(s);
    *m_out = m;
    *l_out = l;
    return 0;
}

static void set_threads(int nthreads)
{
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif
}

int hgo_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- 1. the definition --------------------------------------------------------------------- */

int hgo_attn_full(const hgo_problem *p, double *out, double *lse, int nthreads)
{
    int rc = check_problem(p);
    if (rc) return rc;
    if (!out) return -1;
    set_threads(nthreads);
    int64_t pairs = (int64_t)p->B * p->Hq;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t bh = 0; bh < pairs; ++bh) {
        int b = (int)(bh / p->Hq), h = (int)(bh % p->Hq);
        double m, l;
        double *o = out + bh * p->d;
        if (range_stats(p, b, h, 0, p->seq_lens[b], &m, &l, o)) {
#pragma omp atomic write
            failed = 1;
        }
        if (l > 0.0) {
            for (int c = 0; c < p->d; ++c) o[c] /= l;
            if (lse) lse[bh] = m + log(l);
        } else {
            if (lse) lse[bh] = -INFINITY;
        }
    }
    return failed ? -7 : 0;
}

/* ---- 2. per-range partial statistics ------------------------------------------------------- */

int hgo_attn_partial(const hgo_problem *p, const hgo_range *ranges, int32_t n_ranges, double *m, double *l,
                     double *o, int nthreads)
{
    int rc = check_problem(p);
    if (rc) return rc;
    if (n_ranges < 0) return -2;
    if (n_ranges && (!ranges || !m || !l || !o)) return -1;
    for (int r = 0; r < n_ranges; ++r) {
        if (ranges[r].seq < 0 || ranges[r].seq >= p->B) return -4;
        if (ranges[r].begin < 0 || ranges[r].begin > ranges[r].end) return -4;
        if (ranges[r].end > p->seq_lens[ranges[r].seq]) return -4;
    }
    set_threads(nthreads);
    int64_t items = (int64_t)n_ranges * p->Hq;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t rh = 0; rh < items; ++rh) {
        int r = (int)(rh / p->Hq), h = (int)(rh % p->Hq);
        if (range_stats(p, ranges[r].seq, h, ranges[r].begin, ranges[r].end, &m[rh], &l[rh], o + rh * p->d)) {
#pragma omp atomic write
            failed = 1;
        }
    }
    return failed ? -7 : 0;
}

/* ---- 2b. raw logits per range (the paper's wire format) ------------------------------------ */

/* logits is [Hq][ltok] with ltok = sum of range lengths; the logits of range r occupy columns
 * pre[r] .. pre[r] + len_r - 1, pre[r] = total length of the ranges before r (table order). */
int hgo_attn_logits(const hgo_problem *p, const hgo_range *ranges, int32_t n_ranges, double *logits, int nthreads)
{
    int rc = check_problem(p);
    if (rc) return rc;
    if (n_ranges < 0) return -2;
    if (n_ranges && (!ranges || !logits)) return -1;
    int64_t ltok = 0;
    for (int r = 0; r < n_ranges; ++r) {
        if (ranges[r].seq < 0 || ranges[r].seq >= p->B) return -4;
        if (ranges[r].begin < 0 || ranges[r].begin > ranges[r].end) return -4;
        if (ranges[r].end > p->seq_lens[ranges[r].seq]) return -4;
        ltok += ranges[r].end - ranges[r].begin;
    }
    set_threads(nthreads);
#pragma omp parallel for schedule(dynamic, 1)
    for (int h = 0; h < p->Hq; ++h) {
        int64_t col = 0;
        for (int r = 0; r < n_ranges; ++r)
            for (int64_t t = ranges[r].begin; t < ranges[r].end; ++t) logits[(int64_t)h * ltok + col++] = logit(p, ranges[r].seq, h, t);
    }
    return 0;
}

/* ---- 2c. Post-QK^T selection: top-k logits of a group, then (m, l, O) over the kept tokens ---- */

typedef struct {
    float val;
    int32_t col;
} hgo_cand;

static int cmp_cand(const void *a, const void *b)
{
    const hgo_cand *x = (const hgo_cand *)a, *y = (const hgo_cand *)b;
    if (x->val != y->val) return x->val > y->val ? -1 : 1; /* higher logit first */
    return (x->col > y->col) - (x->col < y->col);          /* ties: lower column first */
}

static int cmp_int32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* logits: fp32 [Hq][ltok] laid out as hgo_attn_logits writes them for `ranges`.  group_ptr: CSR
 * over the ranges (group_ptr[0] == 0, group_ptr[n_groups] == n_ranges, one sequence per group).
 * sel: int32 [n_groups][Hq][top_k] kept TOKEN positions in ascending column order, -1 padded.
 * m, l: [n_groups][Hq]; o: [n_groups][Hq][d]. */
int hgo_attn_select(const hgo_problem *p, const hgo_range *ranges, int32_t n_ranges, const float *logits,
                    const int32_t *group_ptr, int32_t n_groups, int32_t top_k, int32_t *sel, double *m, double *l,
                    double *o)
{
    int rc = check_problem(p);
    if (rc) return rc;
    if (n_ranges < 0 || n_groups < 0 || top_k < 1) return -2;
    if (n_groups && (!group_ptr || !sel || !m || !l || !o)) return -1;
    if (n_groups && (group_ptr[0] != 0 || group_ptr[n_groups] != n_ranges)) return -4;
    int64_t ltok = 0;
    int64_t *pre = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n_ranges + 1));
    if (!pre) return -7;
    for (int r = 0; r < n_ranges; ++r) {
        pre[r] = ltok;
        ltok += ranges[r].end - ranges[r].begin;
    }
    pre[n_ranges] = ltok;
    for (int g = 0; g < n_groups; ++g) {
        int r0 = group_ptr[g], r1 = group_ptr[g + 1];
        int64_t c0 = pre[r0], c1 = pre[r1], n = c1 - c0;
        for (int h = 0; h < p->Hq; ++h) {
            int64_t gh = (int64_t)g * p->Hq + h;
            int32_t *out_sel = sel + gh * top_k;
            double *dst = o + gh * p->d;
            for (int i = 0; i < top_k; ++i) out_sel[i] = -1;
            for (int c = 0; c < p->d; ++c) dst[c] = 0.0;
            m[gh] = -INFINITY;
            l[gh] = 0.0;
            if (n == 0) continue;
            hgo_cand *cand = (hgo_cand *)malloc(sizeof(hgo_cand) * (size_t)n);
            if (!cand) {
                free(pre);
                return -7;
            }
            for (int64_t j = 0; j < n; ++j) {
                cand[j].val = logits[(int64_t)h * ltok + c0 + j];
                cand[j].col = (int32_t)(c0 + j);
            }
            qsort(cand, (size_t)n, sizeof(hgo_cand), cmp_cand);
            int keep = n < top_k ? (int)n : top_k;
            int32_t *cols = (int32_t *)malloc(sizeof(int32_t) * (size_t)keep);
            for (int i = 0; i < keep; ++i) cols[i] = cand[i].col;
            qsort(cols, (size_t)keep, sizeof(int32_t), cmp_int32); /* back to token order */
            double mx = (double)cand[0].val;
            double lt = 0.0;
            for (int i = 0; i < keep; ++i) {
                int r = r0;
                while (!(cols[i] >= pre[r] && cols[i] < pre[r + 1])) ++r; /* the range holding this column */
                int64_t tok = ranges[r].begin + (cols[i] - pre[r]);
                out_sel[i] = (int32_t)tok;
                double w = exp((double)logits[(int64_t)h * ltok + cols[i]] - mx);
                lt += w;
                int64_t voff = kv_row(p, ranges[r].seq, h, tok);
                for (int c = 0; c < p->d; ++c) dst[c] += w * load_elem(p->v, voff + c, p->dtype);
            }
            m[gh] = mx;
            l[gh] = lt;
            free(cols);
            free(cand);
        }
    }
    free(pre);
    return 0;
}

/* ---- 2d. statistics over a LISTED token set ------------------------------------------------- */

/* The executor's side of a selection decided elsewhere: under Pre-QK^T selection the token
 * selector names the tokens before any logit exists and the executor computes logits and value
 * sums for exactly those (Section 4.3.2; Section 4.6 step 1); the same holds for a Post-QK^T
 * list taken with a proxy query (Section 4.2.1) and evaluated with the true one.
 *
 * group_seq: [n_groups] sequence of each group.  index: int32 [n_groups][Hq][max_k] token
 * positions of that sequence in any order; negative entries are padding; a token listed twice
 * counts twice.  Per (group, head): m = max over the listed tokens of s_t, l = sum exp(s_t - m),
 * O = sum exp(s_t - m) v_t, all with this problem's q; (-inf, 0, 0) for a list without tokens.
 * Returns -4 when an entry is not below the sequence's length. */
int hgo_attn_gather(const hgo_problem *p, const int32_t *group_seq, int32_t n_groups, const int32_t *index,
                    int32_t max_k, double *m, double *l, double *o)
{
    int rc = check_problem(p);
    if (rc) return rc;
    if (n_groups < 0 || max_k < 1) return -2;
    if (n_groups && (!group_seq || !index || !m || !l || !o)) return -1;
    for (int g = 0; g < n_groups; ++g) {
        if (group_seq[g] < 0 || group_seq[g] >= p->B) return -4;
        for (int64_t i = 0; i < (int64_t)p->Hq * max_k; ++i)
            if (index[(int64_t)g * p->Hq * max_k + i] >= p->seq_lens[group_seq[g]]) return -4;
    }
    double *s = (double *)malloc(sizeof(double) * (size_t)max_k);
    if (!s) return -7;
    for (int g = 0; g < n_groups; ++g) {
        int b = group_seq[g];
        for (int h = 0; h < p->Hq; ++h) {
            int64_t gh = (int64_t)g * p->Hq + h;
            const int32_t *idx = index + gh * max_k;
            double *dst = o + gh * p->d;
            for (int c = 0; c < p->d; ++c) dst[c] = 0.0;
            double mx = -INFINITY, lt = 0.0;
            for (int i = 0; i < max_k; ++i)
                if (idx[i] >= 0) {
                    s[i] = logit(p, b, h, idx[i]);
                    if (s[i] > mx) mx = s[i];
                }
            for (int i = 0; i < max_k; ++i)
                if (idx[i] >= 0) {
                    double w = exp(s[i] - mx);
                    int64_t voff = kv_row(p, b, h, idx[i]);
                    lt += w;
                    for (int c = 0; c < p->d; ++c) dst[c] += w * load_elem(p->v, voff + c, p->dtype);
                }
            m[gh] = mx;
            l[gh] = lt;
        }
    }
    free(s);
    return 0;
}

/* ---- 3. exact merge of (m, l, O) triples --------------------------------------------------- */

/* Triples are stored [n_triples][Hq] (m, l) and [n_triples][Hq][d] (o).  Group i merges the
 * triples group_ptr[i] .. group_ptr[i+1]-1, separately for every query head. */
int hgo_attn_merge(const double *m, const double *l, const double *o, const int32_t *group_ptr, int32_t n_groups,
                   int32_t Hq, int32_t d, double *out, double *lse)
{
    if (n_groups < 0 || Hq <= 0 || d <= 0) return -2;
    if (n_groups && (!group_ptr || !out)) return -1;
    for (int i = 0; i < n_groups; ++i)
        if (group_ptr[i] > group_ptr[i + 1] || group_ptr[i] < 0) return -4;
    if (n_groups && group_ptr[n_groups] > group_ptr[0] && (!m || !l || !o)) return -1;
    for (int i = 0; i < n_groups; ++i) {
        for (int h = 0; h < Hq; ++h) {
            double M = -INFINITY;
            for (int t = group_ptr[i]; t < group_ptr[i + 1]; ++t) {
                int64_t th = (int64_t)t * Hq + h;
                if (l[th] != 0.0 && m[th] > M) M = m[th];
            }
            double L = 0.0;
            double *dst = out + ((int64_t)i * Hq + h) * d;
            for (int c = 0; c < d; ++c) dst[c] = 0.0;
            for (int t = group_ptr[i]; t < group_ptr[i + 1]; ++t) {
                int64_t th = (int64_t)t * Hq + h;
                if (l[th] == 0.0) continue; /* identity element */
                double w = exp(m[th] - M);
                L += w * l[th];
                for (int c = 0; c < d; ++c) dst[c] += w * o[th * d + c];
            }
            if (L > 0.0) {
                for (int c = 0; c < d; ++c) dst[c] /= L;
                if (lse) lse[(int64_t)i * Hq + h] = M + log(L);
            } else {
                if (lse) lse[(int64_t)i * Hq + h] = -INFINITY;
            }
        }
    }
    return 0;
}

/* ---- 4. paper-literal: concatenate raw logits in token order, one softmax, then P.V -------- */

static int cmp_range_begin(const void *a, const void *b)
{
    const hgo_range *x = (const hgo_range *)a, *y = (const hgo_range *)b;
    if (x->begin != y->begin) return x->begin < y->begin ? -1 : 1;
    return (x->end > y->end) - (x->end < y->end);
}

/* out: [B][Hq][d].  The ranges of each sequence are taken in ascending order of begin; the
 * logits of all of them form one vector, softmax is taken over that vector. */
int hgo_attn_concat(const hgo_problem *p, const hgo_range *ranges, int32_t n_ranges, double *out, int nthreads)
{
    int rc = check_problem(p);
    if (rc) return rc;
    if (n_ranges < 0) return -2;
    if ((n_ranges && !ranges) || !out) return -1;
    for (int r = 0; r < n_ranges; ++r) {
        if (ranges[r].seq < 0 || ranges[r].seq >= p->B) return -4;
        if (ranges[r].begin < 0 || ranges[r].begin > ranges[r].end) return -4;
        if (ranges[r].end > p->seq_lens[ranges[r].seq]) return -4;
    }
    set_threads(nthreads);
    int failed = 0;
    for (int b = 0; b < p->B; ++b) {
        /* the Token Mapper's view of sequence b: its ranges in positional order */
        int cnt = 0;
        int64_t total = 0;
        for (int r = 0; r < n_ranges; ++r)
            if (ranges[r].seq == b) {
                ++cnt;
                total += ranges[r].end - ranges[r].begin;
            }
        hgo_range *mine = (hgo_range *)malloc(sizeof(hgo_range) * (size_t)(cnt ? cnt : 1));
        int64_t *tok = (int64_t *)malloc(sizeof(int64_t) * (size_t)(total ? total : 1));
        if (!mine || !tok) {
            free(mine);
            free(tok);
            return -7;
        }
        cnt = 0;
        for (int r = 0; r < n_ranges; ++r)
            if (ranges[r].seq == b) mine[cnt++] = ranges[r];
        qsort(mine, (size_t)cnt, sizeof(hgo_range), cmp_range_begin);
        int64_t n = 0;
        for (int i = 0; i < cnt; ++i)
            for (int64_t t = mine[i].begin; t < mine[i].end; ++t) tok[n++] = t;

#pragma omp parallel for schedule(dynamic, 1)
        for (int h = 0; h < p->Hq; ++h) {
            double *dst = out + ((int64_t)b * p->Hq + h) * p->d;
            for (int c = 0; c < p->d; ++c) dst[c] = 0.0;
            if (n == 0) continue;
            double *s = (double *)malloc(sizeof(double) * (size_t)n);
            if (!s) {
#pragma omp atomic write
                failed = 1;
                continue;
            }
            for (int64_t j = 0; j < n; ++j) s[j] = logit(p, b, h, tok[j]); /* concatenated logits */
            double mx = s[0];
            for (int64_t j = 1; j < n; ++j)
                if (s[j] > mx) mx = s[j];
            double denom = 0.0;
            for (int64_t j = 0; j < n; ++j) {
                s[j] = exp(s[j] - mx);
                denom += s[j];
            }
            for (int64_t j = 0; j < n; ++j) {
                double pj = s[j] / denom; /* attention score of token tok[j] */
                int64_t voff = kv_row(p, b, h, tok[j]);
                for (int c = 0; c < p->d; ++c) dst[c] += pj * load_elem(p->v, voff + c, p->dtype);
            }
            free(s);
        }
        free(mine);
        free(tok);
    }
    return failed ? -7 : 0;
}
