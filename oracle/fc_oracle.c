/*
 * fc_oracle.c -- slow, plain CPU statement of what the FlexiCache decode hot path computes.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may include, link or call this file; it is
 * used by tests/, by the smoke check and by the benchmark's CPU-baseline leg.  It shares no code,
 * header, table or helper with the HIP library: it works on unpaged, token-major arrays
 * k[head][token][dim], v[head][token][dim] of bf16 bit patterns (uint16_t) and on plain page-index
 * lists, and does every floating-point step in fp64 after widening the bf16 inputs exactly.
 *
 * What each routine follows (paper = FlexiCache, arXiv 2511.00868):
 *   fco_build_minmax      Sec. 3.2: per page, the per-dimension minimum and maximum key.
 *   fco_page_scores       Sec. 3.2, page-score equation: s_p = sum_i max(q_i kmin_{p,i}, q_i kmax_{p,i}).
 *                         The paper scores per KV head and is silent on how the G query heads of a
 *                         group combine; reading taken here: maximum over the group (mode 0), which
 *                         keeps the stated meaning "largest possible q.k in the page" for every query
 *                         of the group.  Mode 1 (sum over the group) exists to audit that reading.
 *   fco_select_topk       Sec. 3.1 / 3.3: the K best pages by score; the partially filled last page is
 *                         always a member (Sec. 3.3, placement example) and counts toward K.  Ties go
 *                         to the lower page index.  Emitted in ascending page order.
 *   fco_recycle           Sec. 3.3 "Minimizing Transfer Size" + Sec. 3.4 "Physical Block Reuse During
 *                         Reranking" + "Uniformity Through Null Block": promoted = new \ old, evicted =
 *                         old \ new; evicted pages hand their physical blocks to promoted pages, their
 *                         own table entries fall back to the null block 0, and a (host block -> GPU
 *                         block) copy list is produced.
 *   fco_attention         Sec. 3.1: softmax attention of one query over the tokens of a given page set
 *                         (all pages = ordinary dense attention).
 *   fco_rco, fco_stability, fco_bottom_counts, fco_classify
 *                         Sec. 2.2 / 2.3: random-corrected overlap, temporal stability score, and the
 *                         stable / unstable classification of heads (documented at their definitions).
 *
 * Pins (tests/test_oracle_pins.py): dense numpy softmax attention when the page set is everything;
 * weights sum to one; any partition of the page set merges to the same (out, lse); s_p bounds q.k of
 * every key of the page and equals it for single-key / identical-key pages; closed forms for q >= 0
 * and q <= 0; positive homogeneity; numpy lexsort for the selection; set-algebra invariants and the
 * paper's four-page placement example for the recycling; the paper's 192 MB / 70 % byte arithmetic;
 * RCO anchors 0 (chance) and 1 (identical sets), numpy set arithmetic and argsort for the profiling.
 * Unpinned: whether this score keeps model accuracy (needs the paper's models and datasets).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double bf16_to_f64(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

int fco_num_pages(int ctx, int page_size) { return (ctx + page_size - 1) / page_size; }

/* MinMax vectors of every page of one head.  k: [tokens][D]; out mm: [num_pages][2][D] with row 0 the
 * minimum and row 1 the maximum, as bf16 bit patterns of the winning key element.  Only tokens < ctx
 * take part. */
void fco_build_minmax(const uint16_t *k, int ctx, int D, int P, uint16_t *mm)
{
    int n = fco_num_pages(ctx, P);
    for (int p = 0; p < n; ++p) {
        int t0 = p * P, t1 = t0 + P < ctx ? t0 + P : ctx;
        for (int i = 0; i < D; ++i) {
            uint16_t lo = k[(size_t)t0 * D + i], hi = lo;
            for (int t = t0 + 1; t < t1; ++t) {
                uint16_t x = k[(size_t)t * D + i];
                if (bf16_to_f64(x) < bf16_to_f64(lo)) lo = x;
                if (bf16_to_f64(x) > bf16_to_f64(hi)) hi = x;
            }
            mm[((size_t)p * 2 + 0) * D + i] = lo;
            mm[((size_t)p * 2 + 1) * D + i] = hi;
        }
    }
}

/* Page scores of one KV head against the G queries of its group.  q: [G][D]; mm: [n][2][D];
 * score: [n].  mode 0: max over the group, mode 1: sum over the group. */
void fco_page_scores(const uint16_t *q, int G, const uint16_t *mm, int n, int D, int mode, double *score)
{
    for (int p = 0; p < n; ++p) {
        double best = 0.0;
        for (int g = 0; g < G; ++g) {
            double s = 0.0;
            for (int i = 0; i < D; ++i) {
                double qi = bf16_to_f64(q[(size_t)g * D + i]);
                double a = qi * bf16_to_f64(mm[((size_t)p * 2 + 0) * D + i]);
                double b = qi * bf16_to_f64(mm[((size_t)p * 2 + 1) * D + i]);
                s += a > b ? a : b;
            }
            if (mode == 1) best = g == 0 ? s : best + s;
            else           best = (g == 0 || s > best) ? s : best;
        }
        score[p] = best;
    }
}

typedef struct { double s; int p; } fco_cand;

static int cand_cmp(const void *a, const void *b)
{
    const fco_cand *x = (const fco_cand *)a, *y = (const fco_cand *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return x->p < y->p ? -1 : (x->p > y->p ? 1 : 0);
}

static int int_cmp(const void *a, const void *b)
{
    int x = *(const int32_t *)a, y = *(const int32_t *)b;
    return x < y ? -1 : (x > y ? 1 : 0);
}

/* Select min(K, n) pages out of n.  If ctx is not a multiple of P the last page is a member
 * regardless of its score.  out: [K], ascending, padded with -1.  Returns the member count. */
int fco_select_topk(const double *score, int n, int ctx, int P, int K, int32_t *out)
{
    int want = K < n ? K : n;
    int forced = (ctx % P != 0) ? n - 1 : -1;
    int cnt = 0;
    for (int i = 0; i < K; ++i) out[i] = -1;
    if (want <= 0) return 0;
    if (forced >= 0) out[cnt++] = forced;
    fco_cand *c = (fco_cand *)malloc(sizeof(fco_cand) * (size_t)(n > 0 ? n : 1));
    int m = 0;
    for (int p = 0; p < n; ++p)
        if (p != forced) { c[m].s = score[p]; c[m].p = p; ++m; }
    qsort(c, (size_t)m, sizeof(fco_cand), cand_cmp);
    for (int i = 0; i < m && cnt < want; ++i) out[cnt++] = c[i].p;
    free(c);
    qsort(out, (size_t)cnt, sizeof(int32_t), int_cmp);
    return cnt;
}

/* Promotion bookkeeping of one stable (sequence, head).
 *   old_set[n_old], new_set[n_new]   ascending logical page ids (S_{t-1}, S_t)
 *   table[n_pages]                   logical -> physical GPU block, 0 = null block; updated in place
 *   host_table[n_pages]              logical -> host block (never modified)
 *   free_blocks[*n_free]             blocks this head owns that hold no page; updated in place
 *   copies[2 * n_new]                out: (host block, GPU block) per promoted page, ascending page id
 * Rule that makes the result unique: the pool of available blocks is the current free list in order,
 * followed by the blocks of the evicted pages in ascending page order; promoted pages, in ascending
 * page order, take pool[0], pool[1], ...; what is left is the new free list.
 * Returns the number of promoted pages, or -1 if the head owns too few blocks. */
int fco_recycle(const int32_t *old_set, int n_old, const int32_t *new_set, int n_new,
                int32_t *table, const int32_t *host_table, int32_t *free_blocks, int *n_free,
                int free_cap, int32_t *copies)
{
    int32_t *pool = (int32_t *)malloc(sizeof(int32_t) * (size_t)(*n_free + n_old + 1));
    int np = 0, n_prom = 0;
    for (int i = 0; i < *n_free; ++i) pool[np++] = free_blocks[i];
    for (int i = 0; i < n_old; ++i) {
        int found = 0;
        for (int j = 0; j < n_new; ++j) if (new_set[j] == old_set[i]) { found = 1; break; }
        if (!found) { pool[np++] = table[old_set[i]]; table[old_set[i]] = 0; }
    }
    int used = 0;
    for (int j = 0; j < n_new; ++j) {
        int found = 0;
        for (int i = 0; i < n_old; ++i) if (old_set[i] == new_set[j]) { found = 1; break; }
        if (found) continue;
        if (used >= np) { free(pool); return -1; }
        int32_t blk = pool[used++];
        table[new_set[j]] = blk;
        copies[2 * n_prom + 0] = host_table[new_set[j]];
        copies[2 * n_prom + 1] = blk;
        ++n_prom;
    }
    int left = np - used;
    if (left > free_cap) { free(pool); return -1; }
    for (int i = 0; i < left; ++i) free_blocks[i] = pool[used + i];
    *n_free = left;
    free(pool);
    return n_prom;
}

/* Attention of one query over the tokens of the listed pages (tokens >= ctx do not exist).
 * q: [D]; k, v: [tokens][D]; pages[n_pages] logical ids in any order; out: [D]; lse: log-sum-exp of
 * the scaled logits; wsum (optional): the sum of the softmax weights, which must be 1. */
void fco_attention(const uint16_t *q, const uint16_t *k, const uint16_t *v, int ctx, int D, int P,
                   const int32_t *pages, int n_pages, double scale, double *out, double *lse,
                   double *wsum)
{
    size_t cap = (size_t)n_pages * (size_t)P + 1;
    double *z = (double *)malloc(sizeof(double) * cap);
    int *tok = (int *)malloc(sizeof(int) * cap);
    int m = 0;
    double zmax = -INFINITY;
    for (int a = 0; a < n_pages; ++a) {
        for (int j = 0; j < P; ++j) {
            int t = pages[a] * P + j;
            if (pages[a] < 0 || t >= ctx) continue;
            double dot = 0.0;
            for (int i = 0; i < D; ++i) dot += bf16_to_f64(q[i]) * bf16_to_f64(k[(size_t)t * D + i]);
            z[m] = scale * dot;
            tok[m] = t;
            if (z[m] > zmax) zmax = z[m];
            ++m;
        }
    }
    for (int i = 0; i < D; ++i) out[i] = 0.0;
    double denom = 0.0;
    for (int a = 0; a < m; ++a) denom += exp(z[a] - zmax);
    double ws = 0.0;
    for (int a = 0; a < m; ++a) {
        double w = exp(z[a] - zmax) / denom;
        ws += w;
        for (int i = 0; i < D; ++i) out[i] += w * bf16_to_f64(v[(size_t)tok[a] * D + i]);
    }
    if (lse) *lse = m > 0 ? zmax + log(denom) : -INFINITY;
    if (wsum) *wsum = ws;
    free(z);
    free(tok);
}

/* ---- whole-sequence drivers: the same routines applied to every head of one sequence. ------------
 * These only loop; the heads are independent, so the loop may run on several threads. */

/* q: [Hq][D]; mm: [Hkv][n][2][D]; score: [Hkv][n]; heads with stable[h] == 0 are skipped. */
void fco_seq_scores(const uint16_t *q, int Hq, int Hkv, const uint16_t *mm, int n, int D,
                    const uint8_t *stable, int mode, double *score)
{
    int G = Hq / Hkv;
#pragma omp parallel for schedule(dynamic)
    for (int h = 0; h < Hkv; ++h) {
        if (!stable[h]) continue;
        fco_page_scores(q + (size_t)h * G * D, G, mm + (size_t)h * n * 2 * D, n, D, mode,
                        score + (size_t)h * n);
    }
}

/* k: [Hkv][tpad][D]; mm: [Hkv][n][2][D] */
void fco_seq_build_minmax(const uint16_t *k, int Hkv, int tpad, int ctx, int D, int P, uint16_t *mm)
{
    int n = fco_num_pages(ctx, P);
#pragma omp parallel for schedule(dynamic)
    for (int h = 0; h < Hkv; ++h)
        fco_build_minmax(k + (size_t)h * tpad * D, ctx, D, P, mm + (size_t)h * n * 2 * D);
}

/* page_lists: [Hkv][list_stride], page_counts: [Hkv]; out: [Hq][D]; lse: [Hq] */
void fco_seq_attention(const uint16_t *q, const uint16_t *k, const uint16_t *v, int Hq, int Hkv,
                       int tpad, int ctx, int D, int P, const int32_t *page_lists, int list_stride,
                       const int32_t *page_counts, double scale, double *out, double *lse)
{
    int G = Hq / Hkv;
#pragma omp parallel for schedule(dynamic)
    for (int hq = 0; hq < Hq; ++hq) {
        int h = hq / G;
        fco_attention(q + (size_t)hq * D, k + (size_t)h * tpad * D, v + (size_t)h * tpad * D, ctx, D,
                      P, page_lists + (size_t)h * list_stride, page_counts[h], scale,
                      out + (size_t)hq * D, lse + hq, NULL);
    }
}

/* Number of threads the whole-sequence drivers may use from now on (timing only; results do not depend on
 * it: every head is computed by one thread).  n <= 0 leaves the setting alone. */
void fco_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int fco_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}

/* ---- offline head-stability profiling (Sec. 2.2, 2.3) ----------------------------------------------
 * traces: [steps][heads][K] page ids of the top-K selection of every (layer, head) at every decode step
 * of one sample, each list ascending; num_pages[steps]: candidate pages N_t at each step.
 *
 * fco_rco            random-corrected overlap of two selections (Sec. 2.2, first equation):
 *                    max(0, (|S_s n S_t| / K - K / N_t) / (1 - K / N_t)); defined 0 when K == N_t.
 * fco_stability      temporal stability score (Sec. 2.2, second equation): mean of RCO(s, t) over
 *                    t = s+1 .. s+W-1, for every window start s with s+W-1 < steps.  ts: [steps-W+1][heads].
 * fco_bottom_counts  Sec. 2.3: for every window, the heads whose score lies in the lowest quarter
 *                    (floor(heads / 4) heads; ties to the lower head index) get one count each.
 * fco_classify       Sec. 2.3: the floor(heads * num / den) heads counted most often are unstable
 *                    (ties to the lower head index); flags[h] = 1 for unstable.
 */
double fco_rco(const int32_t *a, const int32_t *b, int K, int n_t)
{
    int inter = 0;
    for (int i = 0; i < K; ++i)
        for (int j = 0; j < K; ++j)
            if (a[i] >= 0 && a[i] == b[j]) { ++inter; break; }
    if (n_t <= K) return 0.0;
    double chance = (double)K / (double)n_t;
    double r = ((double)inter / (double)K - chance) / (1.0 - chance);
    return r > 0.0 ? r : 0.0;
}

void fco_stability(const int32_t *traces, const int32_t *num_pages, int steps, int heads, int K, int W,
                   double *ts)
{
    for (int s = 0; s + W - 1 < steps; ++s)
        for (int h = 0; h < heads; ++h) {
            double acc = 0.0;
            for (int t = s + 1; t <= s + W - 1; ++t)
                acc += fco_rco(traces + ((size_t)s * heads + h) * K, traces + ((size_t)t * heads + h) * K, K,
                               num_pages[t]);
            ts[(size_t)s * heads + h] = acc / (double)(W - 1);
        }
}

void fco_bottom_counts(const double *ts, int windows, int heads, int32_t *counts)
{
    int q = heads / 4;
    for (int w = 0; w < windows; ++w)
        for (int h = 0; h < heads; ++h) {
            int rank = 0;   /* heads that come before h in (score asc, index asc) order */
            for (int g = 0; g < heads; ++g) {
                double x = ts[(size_t)w * heads + g], y = ts[(size_t)w * heads + h];
                if (x < y || (x == y && g < h)) ++rank;
            }
            if (rank < q) counts[h] += 1;
        }
}

void fco_classify(const int32_t *counts, int heads, int num, int den, uint8_t *flags)
{
    int want = (int)(((long long)heads * num) / den);
    for (int h = 0; h < heads; ++h) {
        int rank = 0;       /* heads counted more often, or as often with a lower index */
        for (int g = 0; g < heads; ++g)
            if (counts[g] > counts[h] || (counts[g] == counts[h] && g < h)) ++rank;
        flags[h] = rank < want ? 1 : 0;
    }
}
