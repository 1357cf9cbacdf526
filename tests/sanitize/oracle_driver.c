/* Driver for the sanitizer run of the CPU oracle (tests/test_oracle_sanitizers.py): every oracle function on the
 * edge shapes -- empty, one token, one short of / exactly / one past a quantization group, a partial tail group,
 * budgets above the length, empty pages -- with every buffer allocated at exactly the size the call is entitled to,
 * so that AddressSanitizer sees any access past an end and UBSan any undefined arithmetic.  Prints "ok". */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void fier_oracle_quantize(const uint16_t *K, int n_units, int Lcap, int D, int g, int dtype, const int32_t *L,
                          uint8_t *bits, uint16_t *s, uint16_t *z, int n_threads);
void fier_oracle_append(uint16_t *K, uint16_t *V, int n_units, int Lcap, int D, int g, int dtype, const int32_t *L,
                        const uint16_t *k_new, const uint16_t *v_new, uint8_t *bits, uint16_t *s, uint16_t *z);
void fier_oracle_dequantize(const uint8_t *bits, const uint16_t *s, const uint16_t *z, int n_units, int Lcap, int D,
                            int g, int dtype, const int32_t *L, double *Kt);
void fier_oracle_score(const uint8_t *bits, const uint16_t *s, const uint16_t *z, const uint16_t *q, int n_units,
                       int n_rep, int Lcap, int D, int g, int dtype, const int32_t *L, double *scores, int n_threads);
void fier_oracle_topk(const double *scores, int n_units, int Lcap, const int32_t *L, const int32_t *budget,
                      int max_budget, int32_t *idx, int32_t *count);
void fier_oracle_attention(const uint16_t *K, const uint16_t *V, const uint16_t *q, int n_units, int n_rep, int Lcap,
                           int D, int dtype, double sm_scale, const int32_t *L, const int32_t *idx,
                           const int32_t *count, int max_budget, double *out, int n_threads);
void fier_oracle_page_minmax(const uint16_t *K, int n_units, int Lcap, int D, int page, int dtype, const int32_t *L,
                             uint16_t *kmin, uint16_t *kmax);
void fier_oracle_page_score(const uint16_t *kmin, const uint16_t *kmax, const uint16_t *q, int n_units, int n_rep,
                            int Lcap, int D, int page, int dtype, const int32_t *L, int mode, double *out);
void fier_oracle_page_mean(const double *scores, int n_units, int Lcap, int page, const int32_t *L, double *out);
void fier_oracle_expand_pages(const int32_t *page_idx, const int32_t *page_cnt, int n_units, int max_pages, int page,
                              const int32_t *L, int max_budget, int32_t *idx, int32_t *cnt);

static uint32_t rng_state = 12345u;
static uint32_t rnd(void) { return rng_state = rng_state * 1664525u + 1013904223u; }
/* a finite 16-bit float pattern of either format: sign, a mid-range exponent, random mantissa */
static uint16_t rnd16(int dtype) {
    uint32_t r = rnd();
    uint16_t sign = (uint16_t)((r >> 31) << 15);
    if (dtype == 0) return (uint16_t)(sign | ((10u + (r >> 8) % 10u) << 10) | (r & 0x3ffu));
    return (uint16_t)(sign | ((120u + (r >> 8) % 12u) << 7) | (r & 0x7fu));
}

static void *xmalloc(size_t n) {
    void *p = malloc(n ? n : 1);
    if (!p) abort();
    return p;
}

static void run_case(int U, int n_rep, int Lcap, int g, int dtype, const int32_t *L, const int32_t *budget,
                     int max_budget, int append) {
    const int D = 128, page = 16;
    size_t rows = (size_t)U * Lcap * D;
    uint16_t *K = xmalloc(rows * 2), *V = xmalloc(rows * 2);
    uint16_t *q = xmalloc((size_t)U * n_rep * D * 2), *kn = xmalloc((size_t)U * D * 2), *vn = xmalloc((size_t)U * D * 2);
    for (size_t i = 0; i < rows; ++i) { K[i] = rnd16(dtype); V[i] = rnd16(dtype); }
    for (size_t i = 0; i < (size_t)U * n_rep * D; ++i) q[i] = rnd16(dtype);
    for (size_t i = 0; i < (size_t)U * D; ++i) { kn[i] = rnd16(dtype); vn[i] = rnd16(dtype); }
    uint8_t *bits = xmalloc(rows);
    size_t nmeta = (size_t)U * (Lcap / g) * D;
    uint16_t *s = xmalloc(nmeta * 2), *z = xmalloc(nmeta * 2);
    memset(bits, 0, rows); memset(s, 0, nmeta * 2); memset(z, 0, nmeta * 2);
    int32_t *Lw = xmalloc((size_t)U * 4);
    memcpy(Lw, L, (size_t)U * 4);
    fier_oracle_quantize(K, U, Lcap, D, g, dtype, Lw, bits, s, z, 2);
    if (append) {
        fier_oracle_append(K, V, U, Lcap, D, g, dtype, Lw, kn, vn, bits, s, z);
        for (int u = 0; u < U; ++u) if (Lw[u] < Lcap) Lw[u] += 1;
    }
    double *Kt = xmalloc(rows * 8);
    fier_oracle_dequantize(bits, s, z, U, Lcap, D, g, dtype, Lw, Kt);
    double *scores = xmalloc((size_t)U * Lcap * 8);
    fier_oracle_score(bits, s, z, q, U, n_rep, Lcap, D, g, dtype, Lw, scores, 2);
    int32_t *idx = xmalloc((size_t)U * max_budget * 4), *cnt = xmalloc((size_t)U * 4);
    fier_oracle_topk(scores, U, Lcap, Lw, budget, max_budget, idx, cnt);
    double *out = xmalloc((size_t)U * n_rep * D * 8);
    fier_oracle_attention(K, V, q, U, n_rep, Lcap, D, dtype, 0.088388347648318447, Lw, idx, cnt, max_budget, out, 2);
    /* page-level functions */
    size_t npm = (size_t)U * (Lcap / page) * D;
    uint16_t *kmin = xmalloc(npm * 2), *kmax = xmalloc(npm * 2);
    fier_oracle_page_minmax(K, U, Lcap, D, page, dtype, Lw, kmin, kmax);
    double *ps = xmalloc((size_t)U * (Lcap / page) * 8);
    for (int mode = 0; mode < 2; ++mode) fier_oracle_page_score(kmin, kmax, q, U, n_rep, Lcap, D, page, dtype, Lw, mode, ps);
    fier_oracle_page_mean(scores, U, Lcap, page, Lw, ps);
    int max_pages = Lcap / page;
    int32_t *pidx = xmalloc((size_t)U * max_pages * 4), *pcnt = xmalloc((size_t)U * 4);
    for (int u = 0; u < U; ++u) {           /* every second page that holds a token */
        int np = (Lw[u] + page - 1) / page, k = 0;
        for (int p = 0; p < np; p += 2) pidx[(size_t)u * max_pages + k++] = p;
        pcnt[u] = k;
    }
    int32_t *eidx = xmalloc((size_t)U * max_budget * 4), *ecnt = xmalloc((size_t)U * 4);
    fier_oracle_expand_pages(pidx, pcnt, U, max_pages, page, Lw, max_budget, eidx, ecnt);
    double acc = 0;
    for (size_t i = 0; i < (size_t)U * n_rep * D; ++i) acc += out[i];
    if (acc != acc) { fprintf(stderr, "NaN in attention output\n"); exit(3); }
    free(K); free(V); free(q); free(kn); free(vn); free(bits); free(s); free(z); free(Lw); free(Kt); free(scores);
    free(idx); free(cnt); free(out); free(kmin); free(kmax); free(ps); free(pidx); free(pcnt); free(eidx); free(ecnt);
}

int main(void) {
    /* lengths: empty, 1, 31, 32, 33, partial tail groups, full capacity; budgets: 1, equal to and above the length */
    const int32_t L1[8] = {0, 1, 31, 32, 33, 63, 100, 128};
    const int32_t B1[8] = {4, 4, 1, 32, 40, 64, 7, 200};
    for (int dtype = 0; dtype < 2; ++dtype)
        for (int append = 0; append < 2; ++append) {
            run_case(8, 1, 128, 32, dtype, L1, B1, 200, append);
            run_case(8, 4, 128, 32, dtype, L1, B1, 64, append);      /* budgets above the row pitch are clamped */
        }
    const int32_t L2[3] = {0, 129, 256};
    const int32_t B2[3] = {1, 129, 300};
    run_case(3, 2, 256, 128, 0, L2, B2, 300, 1);                     /* g = 128: partial group of one token */
    run_case(3, 2, 256, 256, 1, L2, B2, 16, 0);
    const int32_t L3[1] = {0};
    const int32_t B3[1] = {0};
    run_case(1, 8, 64, 64, 1, L3, B3, 1, 1);                         /* first row of an empty cache, budget 0 */
    puts("ok");
    return 0;
}
