/*
 * Fier decode step -- CPU ORACLE.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, one-unit-at-a-time implementation of what the Fier decode
 * path computes, written from the paper (arxiv 2508.08256): Algorithm 1
 * (quantize K to 1 bit, approximate scores, top-k, exact attention on the
 * selected rows), the quantizer of Eq. 5 read as 1-bit round-to-nearest
 * (Sec. 3.3), and the decode-stage definition softmax(q K^T) V of Sec. 3.1.
 *
 * It shares no code with the HIP library and must never be called from the
 * product path: only tests/, __graft_entry__.smoke() and the cpu_baseline leg
 * of bench.py may load it.  Nothing here is tuned; no blocking, no fusion.
 *
 * Conventions used by every function:
 *   - a "unit" is one (batch element, kv head): K, V are [L][D] row-major,
 *     stored as raw 16-bit words of dtype 0 = IEEE binary16, 1 = bfloat16;
 *   - floating point is fp64, EXCEPT the quantizer's decision arithmetic
 *     (scale s and the bit), which is IEEE binary32 so that packed bits and
 *     metadata can be compared bit for bit with any other implementation;
 *   - groups are g consecutive tokens of ONE channel (Alg. 1 step 1:
 *     "groups of size g along each channel"); one (s, z) pair per group and
 *     channel, stored in the K dtype (Sec. 3.4 counts two 16-bit numbers per
 *     group, Eq. 8).
 *
 * Parity pins (tests/test_oracle_*.py): closed forms and invariants of the
 * 1-bit quantizer, the storage ratio of Eq. 8 / Tab. 1 / Tab. 4, numpy.dot
 * for the score, brute-force top-k, scipy softmax for full-budget attention,
 * planted-token recall (Observation 2).  The paper prints no numeric example
 * of scores or outputs, so end-to-end values are pinned only through those.
 * The page-level functions at the end (the comparison baseline of Sec. 3.2)
 * are pinned by single-token pages (library max / dot), the upper-bound
 * property, numpy means and brute force (tests/test_oracle_pages.py).
 *
 * Build: gcc -O2 -std=c99 -ffp-contract=off -fopenmp -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------------ */
/* 16-bit float formats, by their definitions.                              */

/* binary16 -> binary32: 1 sign, 5 exponent (bias 15), 10 fraction bits. */
static float f16_to_f32(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);                 /* subnormal: f * 2^-24   */
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp((double)(f | 0x400), e - 25);    /* (1024+f) * 2^(e-15-10) */
    return (float)(sign ? -v : v);                 /* exact in binary32      */
}

/* bfloat16 -> binary32: the upper half of a binary32 word. */
static float bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* binary32 -> binary16, round to nearest even, by exhaustive definition:
 * pick the representable neighbour pair around |x| on the binary16 grid. */
static uint16_t f32_to_f16_rne(float x)
{
    uint16_t sign = signbit(x) ? 0x8000u : 0;
    double a = fabs((double)x);
    if (isnan(x)) return (uint16_t)(sign | 0x7e00u);
    if (a >= 65520.0) return (uint16_t)(sign | 0x7c00u);   /* rounds to inf */
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);                 /* a = m * 2^e, m in [0.5, 1)       */
    int ulp_exp = e - 11;               /* 11 significant bits               */
    if (ulp_exp < -24) ulp_exp = -24;   /* subnormal grid                    */
    double q = ldexp(a, -ulp_exp);      /* a in units of one ulp (exact)     */
    double fl = floor(q);
    double r = q - fl;
    if (r > 0.5 || (r == 0.5 && fmod(fl, 2.0) == 1.0)) fl += 1.0;
    double v = ldexp(fl, ulp_exp);      /* rounded magnitude (may carry up)  */
    /* encode v */
    if (v >= 65520.0) return (uint16_t)(sign | 0x7c00u);
    if (v < ldexp(1.0, -14)) return (uint16_t)(sign | (uint16_t)ldexp(v, 24));
    int ev;
    double mv = frexp(v, &ev);          /* v = mv * 2^ev                     */
    int biased = ev - 1 + 15;
    int frac = (int)ldexp(mv, 11) - 1024;
    return (uint16_t)(sign | (biased << 10) | frac);
}

/* binary32 -> bfloat16, round to nearest even on the 8-bit-significand grid. */
static uint16_t f32_to_bf16_rne(float x)
{
    uint32_t u;
    memcpy(&u, &x, sizeof u);
    if (isnan(x)) return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lower = u & 0xffffu;
    uint32_t upper = u >> 16;
    if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u))) upper += 1;
    return (uint16_t)upper;
}

static float load16(uint16_t w, int dtype)
{
    return dtype == 0 ? f16_to_f32(w) : bf16_to_f32(w);
}

static uint16_t store16(float x, int dtype)
{
    return dtype == 0 ? f32_to_f16_rne(x) : f32_to_bf16_rne(x);
}

/* exported so the tests can pin the conversions against numpy / torch */
float fier_oracle_to_f32(uint16_t w, int dtype) { return load16(w, dtype); }
uint16_t fier_oracle_from_f32(float x, int dtype) { return store16(x, dtype); }

/* ------------------------------------------------------------------------ */
/* Step 1 of Alg. 1: 1-bit group quantizer (Eq. 5 read as RTN, Sec. 3.3).    */
/*
 * For one group (ntok <= g present tokens of one channel):
 *   z   = the smallest element          (an input value, kept exactly;
 *                                        -0 is stored as +0)
 *   s   = round_to_dtype( f32(max) - f32(z) )     (binary32 subtract)
 *   bit = 1  iff  2*(f32(k) - f32(z)) >= f32(s)   (binary32 ops)
 * The two reconstruction levels are z (bit 0) and z + s (bit 1); an element
 * goes to the nearer one, the exact midpoint goes up.  A constant group has
 * s = 0 and every bit 1 (0 >= 0).  If the rounded difference would overflow
 * the dtype it is held at the largest finite value.
 */
static void quantize_group(const uint16_t *K, int D, int c, int t0, int ntok,
                           int dtype, uint8_t *bits, uint16_t *s_out,
                           uint16_t *z_out)
{
    float mn = load16(K[(size_t)t0 * D + c], dtype);
    float mx = mn;
    for (int t = 1; t < ntok; ++t) {
        float x = load16(K[(size_t)(t0 + t) * D + c], dtype);
        if (x < mn) mn = x;
        if (x > mx) mx = x;
    }
    if (mn == 0.0f) mn = 0.0f;               /* -0 -> +0 */
    float diff = mx - mn;                    /* binary32 */
    float cap = dtype == 0 ? 65504.0f : 3.3895313892515355e38f;
    if (diff > cap) diff = cap;
    if (diff == 0.0f) diff = 0.0f;           /* -0 -> +0 */
    uint16_t sw = store16(diff, dtype);
    uint16_t zw = store16(mn, dtype);        /* exact: mn is a dtype value */
    float sf = load16(sw, dtype);
    float zf = load16(zw, dtype);
    for (int t = 0; t < ntok; ++t) {
        float x = load16(K[(size_t)(t0 + t) * D + c], dtype);
        float d = x - zf;                    /* binary32 */
        float twice = d + d;                 /* exact doubling */
        bits[(size_t)(t0 + t) * D + c] = (uint8_t)(twice >= sf ? 1 : 0);
    }
    *s_out = sw;
    *z_out = zw;
}

/*
 * Quantize tokens [0, L) of n_units units.
 *   K     [n_units][Lcap][D] raw 16-bit words
 *   bits  [n_units][Lcap][D] one byte (0/1) per element; rows >= L untouched
 *   s, z  [n_units][Lcap/g][D] raw 16-bit words; groups past ceil(L/g) untouched
 *   L     [n_units] tokens present per unit (the tail group may be partial:
 *         its (s, z) are over the tokens present)
 */
void fier_oracle_quantize(const uint16_t *K, int n_units, int Lcap, int D,
                          int g, int dtype, const int32_t *L, uint8_t *bits,
                          uint16_t *s, uint16_t *z, int n_threads)
{
    int ngcap = Lcap / g;
#ifdef _OPENMP
#pragma omp parallel for num_threads(n_threads > 0 ? n_threads : 1) schedule(dynamic, 1)
#endif
    for (int u = 0; u < n_units; ++u) {
        const uint16_t *Ku = K + (size_t)u * Lcap * D;
        uint8_t *bu = bits + (size_t)u * Lcap * D;
        uint16_t *su = s + (size_t)u * ngcap * D;
        uint16_t *zu = z + (size_t)u * ngcap * D;
        int Lu = L[u];
        for (int t0 = 0; t0 < Lu; t0 += g) {
            int ntok = Lu - t0 < g ? Lu - t0 : g;
            int G = t0 / g;
            for (int c = 0; c < D; ++c)
                quantize_group(Ku, D, c, t0, ntok, dtype, bu,
                               &su[(size_t)G * D + c], &zu[(size_t)G * D + c]);
        }
    }
    (void)n_threads;
}

/*
 * Decode-stage append (Sec. 3.1: K <- Concat(K0, k), V <- Concat(V0, v)) for
 * a cache that keeps 1-bit codes: write the new rows at position L[u], then
 * re-derive the (s, z) and the bits of the group that row falls in from the
 * full-precision keys present (tokens g*floor(L/g) .. L).  L is not changed.
 */
void fier_oracle_append(uint16_t *K, uint16_t *V, int n_units, int Lcap, int D,
                        int g, int dtype, const int32_t *L,
                        const uint16_t *k_new, const uint16_t *v_new,
                        uint8_t *bits, uint16_t *s, uint16_t *z)
{
    int ngcap = Lcap / g;
    for (int u = 0; u < n_units; ++u) {
        int Lu = L[u];
        if (Lu < 0 || Lu >= Lcap) continue;
        uint16_t *Ku = K + (size_t)u * Lcap * D;
        uint16_t *Vu = V + (size_t)u * Lcap * D;
        memcpy(Ku + (size_t)Lu * D, k_new + (size_t)u * D, sizeof(uint16_t) * D);
        memcpy(Vu + (size_t)Lu * D, v_new + (size_t)u * D, sizeof(uint16_t) * D);
        int G = Lu / g;
        int t0 = G * g;
        int ntok = Lu + 1 - t0;
        for (int c = 0; c < D; ++c)
            quantize_group(Ku, D, c, t0, ntok, dtype,
                           bits + (size_t)u * Lcap * D,
                           &s[((size_t)u * ngcap + G) * D + c],
                           &z[((size_t)u * ngcap + G) * D + c]);
    }
}

/* Dequantize (Eq. 5, second half): K~ = code * s + z, in fp64. */
void fier_oracle_dequantize(const uint8_t *bits, const uint16_t *s,
                            const uint16_t *z, int n_units, int Lcap, int D,
                            int g, int dtype, const int32_t *L, double *Kt)
{
    int ngcap = Lcap / g;
    for (int u = 0; u < n_units; ++u)
        for (int t = 0; t < L[u]; ++t)
            for (int c = 0; c < D; ++c) {
                size_t m = ((size_t)u * ngcap + t / g) * D + c;
                size_t e = ((size_t)u * Lcap + t) * D + c;
                Kt[e] = (double)bits[e] * (double)load16(s[m], dtype) +
                        (double)load16(z[m], dtype);
            }
}

/* ------------------------------------------------------------------------ */
/* Step 2 of Alg. 1: approximate scores  s~ = q . K~^T  (unscaled).          */
/*
 * One score per cached token and kv head.  With n_rep query heads sharing a
 * kv head (grouped-query attention, which the paper leaves open), the score
 * of a token is the SUM over those query heads of their separate dot
 * products, so that one selection serves the whole group.
 *   q       [n_units][n_rep][D] raw 16-bit words
 *   scores  [n_units][Lcap] fp64; entries >= L untouched
 */
void fier_oracle_score(const uint8_t *bits, const uint16_t *s,
                       const uint16_t *z, const uint16_t *q, int n_units,
                       int n_rep, int Lcap, int D, int g, int dtype,
                       const int32_t *L, double *scores, int n_threads)
{
    int ngcap = Lcap / g;
#ifdef _OPENMP
#pragma omp parallel for num_threads(n_threads > 0 ? n_threads : 1) schedule(dynamic, 1)
#endif
    for (int u = 0; u < n_units; ++u) {
        for (int t = 0; t < L[u]; ++t) {
            double total = 0.0;
            for (int r = 0; r < n_rep; ++r) {
                const uint16_t *qr = q + ((size_t)u * n_rep + r) * D;
                double dot = 0.0;
                for (int c = 0; c < D; ++c) {
                    size_t m = ((size_t)u * ngcap + t / g) * D + c;
                    size_t e = ((size_t)u * Lcap + t) * D + c;
                    double kt = (double)bits[e] * (double)load16(s[m], dtype) +
                                (double)load16(z[m], dtype);
                    dot += (double)load16(qr[c], dtype) * kt;
                }
                total += dot;
            }
            scores[(size_t)u * Lcap + t] = total;
        }
    }
    (void)n_threads;
}

/* ------------------------------------------------------------------------ */
/* Step 3 of Alg. 1: S_q = Top-k(s~).                                        */

typedef struct {
    double score;
    int32_t index;
} scored_t;

static int by_score_desc_then_index(const void *a, const void *b)
{
    const scored_t *x = (const scored_t *)a, *y = (const scored_t *)b;
    if (x->score > y->score) return -1;
    if (x->score < y->score) return 1;
    return (x->index > y->index) - (x->index < y->index);
}

static int by_int(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/*
 * Per unit: the min(budget, L) tokens of largest score; equal scores go to
 * the lower token index; the set is returned in ascending index order.
 *   scores [n_units][Lcap] fp64, budget [n_units]
 *   idx    [n_units][max_budget] (entries past count untouched), count [n_units]
 */
void fier_oracle_topk(const double *scores, int n_units, int Lcap,
                      const int32_t *L, const int32_t *budget, int max_budget,
                      int32_t *idx, int32_t *count)
{
    for (int u = 0; u < n_units; ++u) {
        int Lu = L[u];
        int B = budget[u];
        if (B > Lu) B = Lu;
        if (B > max_budget) B = max_budget;
        if (B < 0) B = 0;
        scored_t *tmp = (scored_t *)malloc(sizeof(scored_t) * (size_t)(Lu > 0 ? Lu : 1));
        for (int t = 0; t < Lu; ++t) {
            tmp[t].score = scores[(size_t)u * Lcap + t];
            tmp[t].index = t;
        }
        qsort(tmp, (size_t)Lu, sizeof(scored_t), by_score_desc_then_index);
        int32_t *out = idx + (size_t)u * max_budget;
        for (int i = 0; i < B; ++i) out[i] = tmp[i].index;
        qsort(out, (size_t)B, sizeof(int32_t), by_int);
        count[u] = B;
        free(tmp);
    }
}

/* ------------------------------------------------------------------------ */
/* Step 4 of Alg. 1: exact attention over the selected rows.                 */
/*
 * For every query head r of the unit:
 *   logit_i = sm_scale * (q_r . K[i])   for i in S        (fp64)
 *   p       = softmax(logit)            over S
 *   o_r     = sum_i p_i V[i]
 * idx == NULL means S = [0, L): the dense decode attention of Sec. 3.1.
 * count == 0 gives zeros.
 *   out [n_units][n_rep][D] fp64
 */
void fier_oracle_attention(const uint16_t *K, const uint16_t *V,
                           const uint16_t *q, int n_units, int n_rep, int Lcap,
                           int D, int dtype, double sm_scale, const int32_t *L,
                           const int32_t *idx, const int32_t *count,
                           int max_budget, double *out, int n_threads)
{
#ifdef _OPENMP
#pragma omp parallel for num_threads(n_threads > 0 ? n_threads : 1) schedule(dynamic, 1)
#endif
    for (int u = 0; u < n_units; ++u) {
        int n = idx ? count[u] : L[u];
        double *logit = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
        for (int r = 0; r < n_rep; ++r) {
            const uint16_t *qr = q + ((size_t)u * n_rep + r) * D;
            double *o = out + ((size_t)u * n_rep + r) * D;
            for (int c = 0; c < D; ++c) o[c] = 0.0;
            if (n <= 0) continue;
            double mx = -INFINITY;
            for (int i = 0; i < n; ++i) {
                int t = idx ? idx[(size_t)u * max_budget + i] : i;
                const uint16_t *krow = K + ((size_t)u * Lcap + t) * D;
                double dot = 0.0;
                for (int c = 0; c < D; ++c)
                    dot += (double)load16(qr[c], dtype) * (double)load16(krow[c], dtype);
                logit[i] = sm_scale * dot;
                if (logit[i] > mx) mx = logit[i];
            }
            double denom = 0.0;
            for (int i = 0; i < n; ++i) {
                logit[i] = exp(logit[i] - mx);
                denom += logit[i];
            }
            for (int i = 0; i < n; ++i) {
                int t = idx ? idx[(size_t)u * max_budget + i] : i;
                const uint16_t *vrow = V + ((size_t)u * Lcap + t) * D;
                double p = logit[i] / denom;
                for (int c = 0; c < D; ++c) o[c] += p * (double)load16(vrow[c], dtype);
            }
        }
        free(logit);
    }
    (void)n_threads;
}

/* ------------------------------------------------------------------------
 * Page-level importance (the page-retrieval baseline the paper compares with,
 * Sec. 3.2 Eq. 1-3, and its "averaged quantized score" ablation, Sec. 4.4).
 *
 * A page = `page` consecutive tokens of one unit.  Its metadata are the
 * channel-wise maximum and minimum key vectors over the tokens present
 * (input values, hence exact 16-bit words).
 * ---------------------------------------------------------------------- */
void fier_oracle_page_minmax(const uint16_t *K, int n_units, int Lcap, int D,
                             int page, int dtype, const int32_t *L,
                             uint16_t *kmin, uint16_t *kmax)
{
    int n_pages = Lcap / page;
    for (int u = 0; u < n_units; ++u)
        for (int p = 0; p < n_pages; ++p)
            for (int c = 0; c < D; ++c) {
                size_t o = ((size_t)u * n_pages + p) * D + c;
                int t0 = p * page;
                kmin[o] = 0;
                kmax[o] = 0;
                if (t0 >= L[u])
                    continue;
                int t1 = t0 + page < L[u] ? t0 + page : L[u];
                uint16_t wmin = K[((size_t)u * Lcap + t0) * D + c], wmax = wmin;
                for (int t = t0 + 1; t < t1; ++t) {
                    uint16_t w = K[((size_t)u * Lcap + t) * D + c];
                    if (load16(w, dtype) < load16(wmin, dtype)) wmin = w;
                    if (load16(w, dtype) > load16(wmax, dtype)) wmax = w;
                }
                kmin[o] = wmin;
                kmax[o] = wmax;
            }
}

/* Eq. 1-3: alpha_max = q (.) k_max, alpha_min = q (.) k_min, elementwise;
 * mode 0: s_P = max over the channels of max(alpha_max_i, alpha_min_i), the
 *         formula as the paper prints it (Eq. 3);
 * mode 1: s_P = sum over the channels of max(alpha_max_i, alpha_min_i), the
 *         channel-wise upper bound of q . k for every key of the page.
 * With several query heads per kv head the per-head page scores are added
 * (same convention as the token scores).  Pages without tokens get -inf.   */
void fier_oracle_page_score(const uint16_t *kmin, const uint16_t *kmax,
                            const uint16_t *q, int n_units, int n_rep,
                            int Lcap, int D, int page, int dtype,
                            const int32_t *L, int mode, double *out)
{
    int n_pages = Lcap / page;
    for (int u = 0; u < n_units; ++u)
        for (int p = 0; p < n_pages; ++p) {
            double total = 0.0;
            if (p * page >= L[u]) {
                out[(size_t)u * n_pages + p] = -INFINITY;
                continue;
            }
            for (int h = 0; h < n_rep; ++h) {
                double acc = mode == 0 ? -INFINITY : 0.0;
                for (int c = 0; c < D; ++c) {
                    size_t o = ((size_t)u * n_pages + p) * D + c;
                    double qc = load16(q[((size_t)u * n_rep + h) * D + c], dtype);
                    double a_max = qc * (double)load16(kmax[o], dtype);
                    double a_min = qc * (double)load16(kmin[o], dtype);
                    double m = a_max > a_min ? a_max : a_min;
                    if (mode == 0)
                        acc = m > acc ? m : acc;
                    else
                        acc += m;
                }
                total += acc;
            }
            out[(size_t)u * n_pages + p] = total;
        }
}

/* Sec. 4.4 ablation: the page metric is the average of the (1-bit) token
 * scores over the tokens present in the page.  Empty pages get -inf.      */
void fier_oracle_page_mean(const double *scores, int n_units, int Lcap,
                           int page, const int32_t *L, double *out)
{
    int n_pages = Lcap / page;
    for (int u = 0; u < n_units; ++u)
        for (int p = 0; p < n_pages; ++p) {
            int t0 = p * page;
            if (t0 >= L[u]) {
                out[(size_t)u * n_pages + p] = -INFINITY;
                continue;
            }
            int t1 = t0 + page < L[u] ? t0 + page : L[u];
            double acc = 0.0;
            for (int t = t0; t < t1; ++t)
                acc += scores[(size_t)u * Lcap + t];
            out[(size_t)u * n_pages + p] = acc / (double)(t1 - t0);
        }
}

/* All tokens of the selected pages (page_idx ascending, page_cnt of them), in
 * ascending order, clipped to the unit's length.                           */
void fier_oracle_expand_pages(const int32_t *page_idx, const int32_t *page_cnt,
                              int n_units, int max_pages, int page,
                              const int32_t *L, int max_budget, int32_t *idx,
                              int32_t *cnt)
{
    for (int u = 0; u < n_units; ++u) {
        int n = 0;
        for (int k = 0; k < page_cnt[u]; ++k) {
            int p = page_idx[(size_t)u * max_pages + k];
            for (int j = 0; j < page; ++j) {
                int t = p * page + j;
                if (t < L[u] && n < max_budget)
                    idx[(size_t)u * max_budget + n++] = t;
            }
        }
        cnt[u] = n;
    }
}

int fier_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
