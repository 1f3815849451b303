// fc_rerank_topk: page scores from the MinMax cache and per-head top-K (Sec. 3.2 of the paper).
//
// Score.  max(q_i*kmin_i, q_i*kmax_i) equals q_i*kmax_i when q_i >= 0 and q_i*kmin_i otherwise, so
// with q+ = max(q, 0) and q- = min(q, 0) the page score of one query is the plain dot product
//     s_p = [q- | q+] . [kmin_p | kmax_p]           (256 terms, one of every pair is an exact zero)
// and the scores of 16 pages against the G queries of a group are one 16 x 256 x 16 contraction:
// 8 x v_mfma_f32_16x16x32_bf16 with A = 16 MinMax rows straight from memory (512 B each, lane reads
// 16 B of row n at byte 64s + 16j) and B = the sign-split queries.  Products of bf16 values are exact
// in fp32 and the accumulation is fp32.  The score of the KV head is the maximum over its G queries.
//
// Select.  One workgroup per (sequence, stable head): 4-pass 8-bit radix select on the order-
// preserving integer image of the fp32 score finds the K-th largest key; an index-ordered
// compaction (two workgroup-wide prefix sums when the keys sit in registers) then emits every page
// above it plus the lowest-indexed pages equal to it, which is "ties go to the lower page index"
// and yields the list already ascending.  A partially filled last
// page gets the largest possible key, so it is always a member and counts toward K (Sec. 3.3).
//
// Up to 8192 pages per sequence the K-th key is found faster than by radix passes: the scores of the candidates are
// spread linearly over a few hundred to two thousand bins between their minimum and maximum (a monotone map, so
// bins order the keys), one histogram and one scan find the bin that holds the K-th largest, and the handful of
// candidates in that bin are ranked against each other directly; a crowded bin (outliers, long runs of ties) is
// refined the same way, and a bin of equal scores ends the search (ties to the lower index).  The same kernel can
// go on to recycle the head's blocks (fc_rerank_promote; the fused kernel of Sec. 3.4).
#include "fc_internal.h"
#include "fc_recycle.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(8 * sizeof(short)))) short short8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float float4_t;

// 16-page tiles per wavefront, all in flight at once.  Measured on the 128k-context benchmark (100.7 MB of MinMax rows):
// 1 tile 18.1 us, 2 tiles 18.5, 4 tiles 20.2 (198 VGPRs, two workgroups per CU); 4 tiles of which 2 in flight 18.9.
// More, smaller workgroups fill and drain the chip faster, and that is what a kernel this short is made of.
constexpr int FC_SCORE_TILES_PER_WAVE = 1;
constexpr int FC_SCORE_PAGES_PER_BLOCK = 4 * FC_SCORE_TILES_PER_WAVE * 16;

struct fc_rerank_params {
    const uint16_t *q;
    const char *minmax;
    const int32_t *context_lens;
    const int32_t *k_per_seq;
    const uint8_t *rerank_mask;
    int batch, Hq, Hkv, G, Nmax, Kmax, n_stable;
    uint8_t heads[64];
    float *scores;
    int32_t *topk_pages;
    int32_t *topk_count;
};

struct fc_mm_regs { bf16x8_t a[8]; };

// Plain loads: the non-temporal hint that helps the attention kernel costs 1.5-3 us here (measured with 1, 2 and 4 tiles).
__device__ __forceinline__ void fc_load_mm_tile(fc_mm_regs &r, const char *rows, int page, int last_page, int j)
{
    const int pg = page > last_page ? last_page : page;
    const char *src = rows + (size_t)pg * FC_MM_ROW_BYTES + j * 16;
#pragma unroll
    for (int s = 0; s < 8; ++s) r.a[s] = *reinterpret_cast<const bf16x8_t *>(src + s * 64);
}

__global__ __launch_bounds__(256) void fc_score_kernel(fc_rerank_params p)
{
    const int b = blockIdx.z;
    if (p.rerank_mask && !p.rerank_mask[b]) return;
    const int h = p.heads[blockIdx.y];
    const int ctx = p.context_lens[b];
    int n_pages = (ctx + FC_P - 1) / FC_P;
    n_pages = n_pages > p.Nmax ? p.Nmax : n_pages;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int page0 = blockIdx.x * FC_SCORE_PAGES_PER_BLOCK + wave * (FC_SCORE_TILES_PER_WAVE * 16);
    if (page0 >= n_pages) return;
    const int lane = threadIdx.x & 63, n = lane & 15, j = lane >> 4;
    const size_t item = (size_t)b * p.Hkv + h;
    const char *rows = p.minmax + item * (size_t)p.Nmax * FC_MM_ROW_BYTES;
    float *score = p.scores + item * (size_t)p.Nmax;
    const int last_page = n_pages - 1;

    // every load of this wavefront's pages is issued before anything waits on one: the kernel is one memory round
    // trip deep after the context length
    fc_mm_regs buf[FC_SCORE_TILES_PER_WAVE];
#pragma unroll
    for (int t = 0; t < FC_SCORE_TILES_PER_WAVE; ++t)
        if (page0 + 16 * t < n_pages) fc_load_mm_tile(buf[t], rows, page0 + 16 * t + n, last_page, j);

    // B operand: k index 0..127 pairs kmin with q-, 128..255 pairs kmax with q+.
    bf16x8_t qb[8];
    {
        const uint16_t *qrow = p.q + ((size_t)b * p.Hq + (size_t)h * p.G + (n < p.G ? n : 0)) * FC_D;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            short8_t x = *reinterpret_cast<const short8_t *>(qrow + 32 * s + 8 * j);
            short8_t neg, pos;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const bool live = n < p.G;
                neg[e] = (live && x[e] < 0) ? x[e] : (short)0;     // sign bit set <=> negative as int16
                pos[e] = (live && x[e] >= 0) ? x[e] : (short)0;
            }
            qb[s] = __builtin_bit_cast(bf16x8_t, neg);
            qb[s + 4] = __builtin_bit_cast(bf16x8_t, pos);
        }
    }
#pragma unroll
    for (int t = 0; t < FC_SCORE_TILES_PER_WAVE; ++t) {
        const int pg = page0 + 16 * t;
        if (pg >= n_pages) break;
        float4_t s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int k = 0; k < 8; ++k) s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(buf[t].a[k], qb[k], s, 0, 0, 0);
        // lane (n, j) holds pages pg + 4j + v of query n: maximum over the G queries of the group
        for (int d = 1; d < p.G; d <<= 1) {
#pragma unroll
            for (int v = 0; v < 4; ++v) s[v] = fmaxf(s[v], __shfl_xor(s[v], d));
        }
        if (n == 0) {
            const int first = pg + 4 * j;
            if (first + 3 < n_pages) {
                *reinterpret_cast<float4_t *>(score + first) = s;
            } else {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (first + v < n_pages) score[first + v] = s[v];
            }
        }
    }
}

// ---- select ----------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t fc_order_key(float s)
{
    const uint32_t u = __float_as_uint(s);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// One count per participating lane into a 256-bin LDS histogram.  Scores of one head share their sign and
// most exponent bits, so in the high-digit passes nearly every lane of a wavefront hits the same bin and
// plain LDS atomics serialise; up to three rounds of "lanes with the first lane's digit add their count
// with one atomic" take care of the popular bins, the rest add one by one.  Must be called by whole wavefronts.
__device__ __forceinline__ void fc_hist_add(int *hist, bool on, uint32_t digit)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int round = 0; round < 3; ++round) {
        const unsigned long long todo = __ballot(on);
        if (todo == 0) return;
        const int leader = __ffsll((long long)todo) - 1;
        const uint32_t d = __shfl(digit, leader);
        const unsigned long long same = __ballot(on && digit == d);
        if (lane == leader) atomicAdd(&hist[d], __popcll(same));
        if (digit == d) on = false;
    }
    if (on) atomicAdd(&hist[digit], 1);
}

constexpr int FC_SELECT_THREADS = 1024;
constexpr int FC_SELECT_CACHED = 8;      // keys a thread keeps in registers: up to 8192 pages without re-reading

// CACHED: every thread holds the keys of `per` = ceil(n / 1024) <= 8 consecutive pages in registers, so the
// four radix passes and the compaction read the scores from memory once instead of five times, and the
// index-ordered compaction is a walk over a thread's own keys between two workgroup-wide prefix sums (ties,
// then members).
template <bool CACHED>
__device__ __forceinline__ void fc_select_body(const fc_rerank_params &p, const float *score, int32_t *out, int n,
                                               int want, int forced, int *hist, int (*wave_cnt)[FC_SELECT_THREADS / 64],
                                               uint32_t *sh_prefix, int *sh_remaining)
{
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    auto key_at = [&](int pg) -> uint32_t { return pg == forced ? 0xFFFFFFFFu : fc_order_key(score[pg]); };
    uint32_t kreg[FC_SELECT_CACHED];
    const int per = (n + FC_SELECT_THREADS - 1) / FC_SELECT_THREADS;     // 1..8 when CACHED: pages per thread
    const int pg0 = tid * per;
    if (CACHED) {
#pragma unroll
        for (int i = 0; i < FC_SELECT_CACHED; ++i) {
            const int pg = pg0 + i;
            kreg[i] = (i < per && pg < n) ? key_at(pg) : 0u;
        }
    }

    uint32_t T = 0;       // threshold key: pages with key > T are members
    int need_eq = n;      // how many pages with key == T are members (lowest indices first)
    if (want < n) {
        if (tid == 0) { *sh_prefix = 0; *sh_remaining = want; }
        uint32_t mask = 0;
        for (int shift = 24; shift >= 0; shift -= 8) {
            if (tid < 256) hist[tid] = 0;
            __syncthreads();
            const uint32_t prefix = *sh_prefix;
            if (CACHED) {
#pragma unroll
                for (int i = 0; i < FC_SELECT_CACHED; ++i) {
                    const uint32_t k = kreg[i];
                    if (i < per) fc_hist_add(hist, pg0 + i < n && (k & mask) == prefix, (k >> shift) & 255);
                }
            } else {
                for (int base = 0; base < n; base += FC_SELECT_THREADS) {     // uniform trip count: fc_hist_add votes across the wavefront
                    const int pg = base + tid;
                    const uint32_t k = pg < n ? key_at(pg) : 0u;
                    fc_hist_add(hist, pg < n && (k & mask) == prefix, (k >> shift) & 255);
                }
            }
            __syncthreads();
            // suffix sums over the 256 digit counts by 256 threads: the digit whose suffix sum first
            // reaches `rem` holds the K-th largest key
            const int rem = *sh_remaining;
            int c = 0, x = 0;
            if (tid < 256) {
                c = hist[255 - tid];
                x = c;
#pragma unroll
                for (int d = 1; d < 64; d <<= 1) {
                    const int y = __shfl_up(x, d);
                    if (lane >= d) x += y;
                }
                if (lane == 63) wave_cnt[0][wv] = x;
            }
            __syncthreads();
            if (tid < 256) {
                int incl = x;
                for (int k = 0; k < wv; ++k) incl += wave_cnt[0][k];
                const int excl = incl - c;
                if (incl >= rem && excl < rem) {
                    *sh_prefix = prefix | ((uint32_t)(255 - tid) << shift);
                    *sh_remaining = rem - excl;
                }
            }
            mask |= 0xFFu << shift;
            __syncthreads();
        }
        T = *sh_prefix;
        need_eq = *sh_remaining;
    }

    // index-ordered compaction, 1024 pages per round
    int eq_base = 0, sel_base = 0;
    auto round = [&](int pg, uint32_t k) {
        const bool live = pg < n;
        const bool gt = live && k > T, eq = live && k == T;
        const unsigned long long beq = __ballot(eq);
        if (lane == 0) wave_cnt[0][wv] = __popcll(beq);
        __syncthreads();
        int eq_before = eq_base, eq_total = 0;
        for (int w = 0; w < FC_SELECT_THREADS / 64; ++w) {
            const int c = wave_cnt[0][w];
            if (w < wv) eq_before += c;
            eq_total += c;
        }
        eq_before += __popcll(beq & ((1ull << lane) - 1ull));
        const bool sel = gt || (eq && eq_before < need_eq);
        const unsigned long long bsel = __ballot(sel);
        if (lane == 0) wave_cnt[1][wv] = __popcll(bsel);
        __syncthreads();
        int sel_before = sel_base, sel_total = 0;
        for (int w = 0; w < FC_SELECT_THREADS / 64; ++w) {
            const int c = wave_cnt[1][w];
            if (w < wv) sel_before += c;
            sel_total += c;
        }
        sel_before += __popcll(bsel & ((1ull << lane) - 1ull));
        if (sel && sel_before < p.Kmax) out[sel_before] = pg;
        eq_base += eq_total;
        sel_base += sel_total;
        __syncthreads();
    };
    if (CACHED) {
        // exclusive prefix sum of one count per thread over the workgroup (threads are in page order)
        auto scan = [&](int mine, int slot) -> int {
            int x = mine;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int y = __shfl_up(x, d);
                if (lane >= d) x += y;
            }
            if (lane == 63) wave_cnt[slot][wv] = x;
            __syncthreads();
            int before = x - mine;
            for (int w = 0; w < wv; ++w) before += wave_cnt[slot][w];
            return before;
        };
        int n_eq = 0;
#pragma unroll
        for (int i = 0; i < FC_SELECT_CACHED; ++i) n_eq += (i < per && pg0 + i < n && kreg[i] == T) ? 1 : 0;
        int eq_rank = scan(n_eq, 0);              // ties before this thread's pages
        bool sel[FC_SELECT_CACHED];
        int n_sel = 0;
#pragma unroll
        for (int i = 0; i < FC_SELECT_CACHED; ++i) {
            const bool live = i < per && pg0 + i < n;
            const bool eq = live && kreg[i] == T;
            sel[i] = (live && kreg[i] > T) || (eq && eq_rank < need_eq);
            eq_rank += eq ? 1 : 0;
            n_sel += sel[i] ? 1 : 0;
        }
        int pos = scan(n_sel, 1);                 // members before this thread's pages
#pragma unroll
        for (int i = 0; i < FC_SELECT_CACHED; ++i)
            if (sel[i]) {
                if (pos < p.Kmax) out[pos] = pg0 + i;
                ++pos;
            }
    } else {
        for (int base = 0; base < n; base += FC_SELECT_THREADS) {
            const int pg = base + tid;
            round(pg, pg < n ? key_at(pg) : 0u);
        }
    }
    for (int i = want + tid; i < p.Kmax; i += FC_SELECT_THREADS) out[i] = -1;
}

__global__ __launch_bounds__(FC_SELECT_THREADS) void fc_select_kernel(fc_rerank_params p)
{
    __shared__ int hist[256];
    __shared__ int wave_cnt[2][FC_SELECT_THREADS / 64];
    __shared__ uint32_t sh_prefix;
    __shared__ int sh_remaining;

    const int b = blockIdx.y;
    if (p.rerank_mask && !p.rerank_mask[b]) return;
    const int h = p.heads[blockIdx.x];
    const int ctx = p.context_lens[b];
    int n = (ctx + FC_P - 1) / FC_P;
    n = n > p.Nmax ? p.Nmax : (n < 0 ? 0 : n);
    int K = p.k_per_seq[b];
    K = K < 0 ? 0 : (K > p.Kmax ? p.Kmax : K);
    const int want = K < n ? K : n;
    const int forced = (ctx % FC_P != 0) ? n - 1 : -1;
    const size_t item = (size_t)b * p.Hkv + h;
    const float *score = p.scores + item * (size_t)p.Nmax;
    int32_t *out = p.topk_pages + item * (size_t)p.Kmax;
    if (n <= FC_SELECT_CACHED * FC_SELECT_THREADS)
        fc_select_body<true>(p, score, out, n, want, forced, hist, wave_cnt, &sh_prefix, &sh_remaining);
    else
        fc_select_body<false>(p, score, out, n, want, forced, hist, wave_cnt, &sh_prefix, &sh_remaining);
    if (threadIdx.x == 0) p.topk_count[item] = want;
}

// ---- select, up to 8192 pages: bucket search, then (optionally) block recycling in the same launch --------------
//
// Threads own consecutive pages (`per` <= 8 each), so thread order is page order and one workgroup-wide prefix sum of
// per-thread counts turns membership flags into ascending list positions.  The same holds for the two sets block
// recycling needs (Sec. 3.4): with the resident list as a bitmap in LDS, "evicted" = resident and not selected and
// "promoted" = selected and not resident are per-page flags of the owning thread, and their ranks in ascending page
// order come out of the same prefix sum as the list positions: no searches, no second pass over lists.  Everything a
// thread may need from memory for its pages (score, block-table entry, host-table entry) has an address that is
// known at launch, so all of it is requested at once and the kernel is one memory round trip deep up to the atomic
// that reserves the head's range of the copy list.
constexpr int FC_FAST_CACHED = 8;        // pages per thread
constexpr int FC_FAST_MAX_PAGES_256 = 256 * FC_FAST_CACHED;     // 2048 pages: 256 threads
constexpr int FC_FAST_MAX_PAGES = 1024 * FC_FAST_CACHED;        // 8192 pages: 1024 threads
constexpr int FC_FAST_CAP = 512;         // candidates ranked directly
constexpr int FC_FAST_MAX_ITERS = 64;    // refinements of a crowded bin; finite scores need at most ~26 (the range shrinks ~2047x each)

// Wavefront-wide primitives on the vector ALU's lane-shuffling operand modes (DPP): shifts inside rows of 16 lanes,
// then "lane 15 of a row to the next row" and "lane 31 to rows 2 and 3".  A few cycles per step instead of a trip
// through the LDS crossbar.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int fc_dpp(int old, int src) { return __builtin_amdgcn_update_dpp(old, src, CTRL, ROW_MASK, 0xf, false); }

__device__ __forceinline__ int fc_wave_scan_add(int x)      // inclusive prefix sum over the 64 lanes
{
    x += fc_dpp<0x111, 0xf>(0, x);      // row_shr:1 (a lane without a source keeps `old` = 0)
    x += fc_dpp<0x112, 0xf>(0, x);
    x += fc_dpp<0x114, 0xf>(0, x);
    x += fc_dpp<0x118, 0xf>(0, x);
    x += fc_dpp<0x142, 0xa>(0, x);      // row_bcast:15 into rows 1 and 3
    x += fc_dpp<0x143, 0xc>(0, x);      // row_bcast:31 into rows 2 and 3
    return x;
}

template <bool IS_MAX>
__device__ __forceinline__ float fc_wave_minmax(float x)    // minimum or maximum over the 64 lanes, in every lane
{
    auto op = [](float a, float b) { return IS_MAX ? fmaxf(a, b) : fminf(a, b); };
    // idempotent operation: a lane without a source combines with itself (`old` = its own value)
    x = op(x, __int_as_float(fc_dpp<0x111, 0xf>(__float_as_int(x), __float_as_int(x))));
    x = op(x, __int_as_float(fc_dpp<0x112, 0xf>(__float_as_int(x), __float_as_int(x))));
    x = op(x, __int_as_float(fc_dpp<0x114, 0xf>(__float_as_int(x), __float_as_int(x))));
    x = op(x, __int_as_float(fc_dpp<0x118, 0xf>(__float_as_int(x), __float_as_int(x))));
    x = op(x, __int_as_float(fc_dpp<0x142, 0xa>(__float_as_int(x), __float_as_int(x))));
    x = op(x, __int_as_float(fc_dpp<0x143, 0xc>(__float_as_int(x), __float_as_int(x))));
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}

template <int THREADS>
struct fc_fast_lds {
    int hist[2 * THREADS];
    uint32_t cand_key[FC_FAST_CAP];
    int cand_idx[FC_FAST_CAP];
    float red_lo[THREADS / 64], red_hi[THREADS / 64];
    int wave_a[THREADS / 64], wave_b[THREADS / 64];
    uint32_t resident_bits[FC_FAST_MAX_PAGES / 32];
    int bb, rem, cb, cand_n, need_eq, all_eq, list_base;
    uint32_t T;
};

// Exclusive prefix sums over the workgroup of two per-thread counts packed as a = lo | hi << 16 (each sum < 65536) and
// b; `tot_a` / `tot_b` get the workgroup sums.  One barrier; the caller separates two calls by another barrier.
template <int THREADS>
__device__ __forceinline__ void fc_block_scan2(int a, int b, fc_fast_lds<THREADS> &L, int &ex_a, int &ex_b, int &tot_a, int &tot_b)
{
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int ia = fc_wave_scan_add(a), ib = fc_wave_scan_add(b);
    if (lane == 63) { L.wave_a[wv] = ia; L.wave_b[wv] = ib; }
    __syncthreads();
    ex_a = ia - a;
    ex_b = ib - b;
    tot_a = 0;
    tot_b = 0;
#pragma unroll
    for (int k = 0; k < THREADS / 64; ++k) {
        const int ca = L.wave_a[k], cb = L.wave_b[k];
        if (k < wv) { ex_a += ca; ex_b += cb; }
        tot_a += ca;
        tot_b += cb;
    }
}

// Threshold key T and the number of pages equal to T that are members (lowest indices first), for the `rem` best of
// the candidate pages (bit i of cmask = this thread's i-th page is a candidate), 1 <= rem < number of candidates.
// *all_eq: every page whose key equals T is a member (the usual case: no tie is split at the boundary).
template <int THREADS>
__device__ __forceinline__ void fc_bucket_threshold(const float (&sreg)[FC_FAST_CACHED], const uint32_t (&kreg)[FC_FAST_CACHED],
                                                    int pg0, unsigned cmask, int rem, fc_fast_lds<THREADS> &L, uint32_t &T,
                                                    int &need_eq, bool &all_eq)
{
    constexpr int BINS = 2 * THREADS, WAVES = THREADS / 64;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    all_eq = false;
    for (int iter = 0; iter < FC_FAST_MAX_ITERS; ++iter) {
        float lo = INFINITY, hi = -INFINITY;
#pragma unroll
        for (int i = 0; i < FC_FAST_CACHED; ++i)
            if ((cmask >> i) & 1u) { lo = fminf(lo, sreg[i]); hi = fmaxf(hi, sreg[i]); }
        lo = fc_wave_minmax<false>(lo);
        hi = fc_wave_minmax<true>(hi);
        if (lane == 0) { L.red_lo[wv] = lo; L.red_hi[wv] = hi; }
        L.hist[tid] = 0;
        L.hist[tid + THREADS] = 0;
        if (tid == 0) L.cand_n = 0;
        __syncthreads();
        lo = L.red_lo[0];
        hi = L.red_hi[0];
#pragma unroll
        for (int k = 1; k < WAVES; ++k) { lo = fminf(lo, L.red_lo[k]); hi = fmaxf(hi, L.red_hi[k]); }
        if (!(hi > lo)) {          // the candidates left all have one score: ties, lowest indices first
            T = fc_order_key(hi);
            need_eq = rem;
            return;
        }
        // linear bins between lo and hi, on halves so that hi - lo cannot overflow; monotone in the score
        const float lo_h = lo * 0.5f, scale = (float)(BINS - 1) / (hi * 0.5f - lo_h);
        int bk[FC_FAST_CACHED];
#pragma unroll
        for (int i = 0; i < FC_FAST_CACHED; ++i) {
            int bkt = (int)((sreg[i] * 0.5f - lo_h) * scale);
            bkt = bkt < 0 ? 0 : (bkt > BINS - 1 ? BINS - 1 : bkt);
            bk[i] = bkt;
            if ((cmask >> i) & 1u) atomicAdd(&L.hist[bkt], 1);
        }
        __syncthreads();
        // cumulative counts from the top bin down; thread t owns bins BINS-1-2t and BINS-2-2t
        const int c0 = L.hist[BINS - 1 - 2 * tid], c1 = L.hist[BINS - 2 - 2 * tid];
        const int x = fc_wave_scan_add(c0 + c1);
        if (lane == 63) L.wave_a[wv] = x;
        __syncthreads();
        int incl = x;
#pragma unroll
        for (int k = 0; k < WAVES; ++k)
            if (k < wv) incl += L.wave_a[k];
        const int excl = incl - (c0 + c1);
        if (excl < rem && incl >= rem) {          // exactly one thread: its bins hold the rem-th best candidate
            if (excl + c0 >= rem) { L.bb = BINS - 1 - 2 * tid; L.rem = rem - excl; L.cb = c0; }
            else { L.bb = BINS - 2 - 2 * tid; L.rem = rem - excl - c0; L.cb = c1; }
        }
        __syncthreads();
        const int bb = L.bb, cb = L.cb;
        rem = L.rem;
#pragma unroll
        for (int i = 0; i < FC_FAST_CACHED; ++i)
            if (bk[i] != bb) cmask &= ~(1u << i);
        if (cb <= FC_FAST_CAP) {
#pragma unroll
            for (int i = 0; i < FC_FAST_CACHED; ++i)
                if ((cmask >> i) & 1u) {
                    const int pos = atomicAdd(&L.cand_n, 1);
                    if (pos < FC_FAST_CAP) { L.cand_key[pos] = kreg[i]; L.cand_idx[pos] = pg0 + i; }
                }
            __syncthreads();
            if (cb <= 64) {
                // the usual case: one candidate per lane of the first wavefront, the others read lane by lane
                if (wv == 0) {
                    const uint32_t mk = lane < cb ? L.cand_key[lane] : 0u;
                    const int mi = lane < cb ? L.cand_idx[lane] : 0;
                    int rank = 0, eq_before = 0, eq_all = 0;
                    for (int c = 0; c < cb; ++c) {
                        const uint32_t k = (uint32_t)__builtin_amdgcn_readlane((int)mk, c);
                        const int ix = __builtin_amdgcn_readlane(mi, c);
                        const bool eq = k == mk, eq_lower = eq && ix < mi;
                        rank += (k > mk || eq_lower) ? 1 : 0;
                        eq_before += eq_lower ? 1 : 0;
                        eq_all += eq ? 1 : 0;
                    }
                    if (lane < cb && rank == rem - 1) { L.T = mk; L.need_eq = eq_before + 1; L.all_eq = eq_before + 1 == eq_all; }
                }
            } else {
                for (int t = tid; t < cb; t += THREADS) {      // up to 512 candidates on 256 or 1024 threads
                    const uint32_t mk = L.cand_key[t];
                    const int mi = L.cand_idx[t];
                    int rank = 0, eq_before = 0, eq_all = 0;
                    for (int c = 0; c < cb; ++c) {
                        const uint32_t k = L.cand_key[c];
                        const bool eq = k == mk, eq_lower = eq && L.cand_idx[c] < mi;
                        rank += (k > mk || eq_lower) ? 1 : 0;
                        eq_before += eq_lower ? 1 : 0;
                        eq_all += eq ? 1 : 0;
                    }
                    if (rank == rem - 1) { L.T = mk; L.need_eq = eq_before + 1; L.all_eq = eq_before + 1 == eq_all; }
                }
            }
            __syncthreads();
            T = L.T;
            need_eq = L.need_eq;
            all_eq = L.all_eq != 0;
            return;
        }
    }
    // not reached with finite scores
    T = 0xFFFFFFFFu;
    need_eq = 0;
}

template <int THREADS, bool RECYCLE>
__global__ __launch_bounds__(THREADS) void fc_select_fast_kernel(fc_rerank_params p, fc_promote_params r)
{
    __shared__ fc_fast_lds<THREADS> L;
    extern __shared__ int32_t avail[];          // RECYCLE: the head's available blocks (Kmax ints)
    const int tid = threadIdx.x;
    const int b = blockIdx.y;
    const int h = p.heads[blockIdx.x];
    const size_t item = (size_t)b * p.Hkv + h;

    // ---- every load whose address is known at launch, before anything waits ----------------------------------------
    const int per = (p.Nmax + THREADS - 1) / THREADS;      // <= FC_FAST_CACHED consecutive pages per thread
    const int pg0 = tid * per;
    const float *score = p.scores + item * (size_t)p.Nmax;
    int32_t *tbl = RECYCLE ? r.block_table + item * (size_t)p.Nmax : nullptr;
    const int32_t *htbl = RECYCLE ? r.host_block_table + item * (size_t)p.Nmax : nullptr;
    float sreg[FC_FAST_CACHED];
    int32_t treg[FC_FAST_CACHED], hreg[FC_FAST_CACHED];
    // eight consecutive 4-byte values of this thread: two 16-byte loads where the row allows it
    auto load8 = [&](const int32_t *row, int32_t (&dst)[FC_FAST_CACHED]) {
        if (per == FC_FAST_CACHED && pg0 + FC_FAST_CACHED <= p.Nmax && (reinterpret_cast<uintptr_t>(row + pg0) & 15) == 0) {
            const int4 lo4 = reinterpret_cast<const int4 *>(row + pg0)[0], hi4 = reinterpret_cast<const int4 *>(row + pg0)[1];
            dst[0] = lo4.x; dst[1] = lo4.y; dst[2] = lo4.z; dst[3] = lo4.w;
            dst[4] = hi4.x; dst[5] = hi4.y; dst[6] = hi4.z; dst[7] = hi4.w;
        } else {
#pragma unroll
            for (int i = 0; i < FC_FAST_CACHED; ++i) dst[i] = (i < per && pg0 + i < p.Nmax) ? row[pg0 + i] : 0;
        }
    };
    {
        int32_t sbits[FC_FAST_CACHED];
        load8(reinterpret_cast<const int32_t *>(score), sbits);
#pragma unroll
        for (int i = 0; i < FC_FAST_CACHED; ++i) sreg[i] = __int_as_float(sbits[i]);
    }
    if (RECYCLE) {
        load8(tbl, treg);
        load8(htbl, hreg);
    }
    const bool skip = p.rerank_mask && !p.rerank_mask[b];
    int n_old = 0, n_free = 0;
    if (RECYCLE) {
        // the resident list becomes a bitmap over the pages; the free list is the head of the available blocks
        for (int i = tid; i < FC_FAST_MAX_PAGES / 32; i += THREADS) L.resident_bits[i] = 0;
        if (!skip) {
            n_old = min(max(r.resident_count[item], 0), p.Kmax);
            n_free = min(max(r.free_count[item], 0), p.Kmax);
        }
        const int32_t *fb = r.free_blocks + item * (size_t)p.Kmax;
        for (int i = tid; i < p.Kmax; i += THREADS) avail[i] = fb[i];
        __syncthreads();
        const int32_t *old_g = r.resident_pages + item * (size_t)p.Kmax;
        for (int i = tid; i < n_old; i += THREADS) {
            const int page = old_g[i];
            if (page >= 0 && page < p.Nmax) atomicOr(&L.resident_bits[page >> 5], 1u << (page & 31));
        }
    }
    int want = 0;
    unsigned sel = 0;          // bit i: this thread's i-th page is a member of the new set
    if (!skip) {
        const int ctx = p.context_lens[b];
        int n = (ctx + FC_P - 1) / FC_P;
        n = n > p.Nmax ? p.Nmax : (n < 0 ? 0 : n);
        int K = p.k_per_seq[b];
        K = K < 0 ? 0 : (K > p.Kmax ? p.Kmax : K);
        want = K < n ? K : n;
        const int forced = (ctx % FC_P != 0) ? n - 1 : -1;

        uint32_t kreg[FC_FAST_CACHED];
        unsigned cmask = 0, live = 0;
#pragma unroll
        for (int i = 0; i < FC_FAST_CACHED; ++i) {
            const int pg = pg0 + i;
            const bool lv = i < per && pg < n;
            kreg[i] = !lv ? 0u : (pg == forced ? 0xFFFFFFFFu : fc_order_key(sreg[i]));
            if (lv) live |= 1u << i;
            if (lv && pg != forced) cmask |= 1u << i;
        }
        uint32_t T = 0;       // threshold key: pages with key > T are members
        int need_eq = n;      // how many pages with key == T are members (lowest indices first)
        bool all_eq = true;   // ... or simply all of them
        if (want < n) {
            const int rem = want - (forced >= 0 ? 1 : 0);     // the partially filled last page takes one place
            if (rem >= 1) {
                fc_bucket_threshold<THREADS>(sreg, kreg, pg0, cmask, rem, L, T, need_eq, all_eq);
            } else {          // room for the forced page only (or for nothing)
                T = 0xFFFFFFFFu;
                need_eq = want;
                all_eq = false;
            }
        }
        int eq_rank = 0;
        if (!all_eq) {        // a run of equal keys is split at the boundary: the lowest page indices are the members
            int n_eq = 0;
#pragma unroll
            for (int i = 0; i < FC_FAST_CACHED; ++i) n_eq += (((live >> i) & 1u) && kreg[i] == T) ? 1 : 0;
            int dummy0, dummy1, dummy2;
            fc_block_scan2<THREADS>(n_eq, 0, L, eq_rank, dummy0, dummy1, dummy2);
            __syncthreads();
        }
#pragma unroll
        for (int i = 0; i < FC_FAST_CACHED; ++i) {
            const bool lv = (live >> i) & 1u;
            const bool eq = lv && kreg[i] == T;
            if ((lv && kreg[i] > T) || (eq && (all_eq || eq_rank < need_eq))) sel |= 1u << i;
            eq_rank += eq ? 1 : 0;
        }
    }

    // ---- positions in the new list; with recycling, the ranks of the evicted and the promoted pages ------------------
    unsigned old = 0;
    if (RECYCLE && !skip) {
        __syncthreads();      // the bitmap is complete
#pragma unroll
        for (int i = 0; i < FC_FAST_CACHED; ++i) {
            const int pg = pg0 + i;
            if (i < per && pg < p.Nmax && ((L.resident_bits[pg >> 5] >> (pg & 31)) & 1u)) old |= 1u << i;
        }
    }
    const unsigned ev = old & ~sel, pr = sel & ~old;
    int pos, r_pr, packed_tot, n_prom;
    {
        int ex_a;
        fc_block_scan2<THREADS>(__popc(sel) | (__popc(ev) << 16), __popc(pr), L, ex_a, r_pr, packed_tot, n_prom);
        pos = ex_a & 0xFFFF;
        const int r_ev0 = ex_a >> 16;
        int32_t *out = p.topk_pages + item * (size_t)p.Kmax;
        if (!skip) {
            int32_t *res = RECYCLE ? r.resident_pages + item * (size_t)p.Kmax : nullptr;
            int q = pos;
#pragma unroll
            for (int i = 0; i < FC_FAST_CACHED; ++i)
                if ((sel >> i) & 1u) {
                    if (q < want) {
                        out[q] = pg0 + i;
                        if (RECYCLE) {
                            res[q] = pg0 + i;
                            if (r.promoted_flags) r.promoted_flags[item * (size_t)p.Kmax + q] = (pr >> i) & 1u;
                        }
                    }
                    ++q;
                }
            for (int i = want + tid; i < p.Kmax; i += THREADS) {
                out[i] = -1;
                if (RECYCLE) res[i] = -1;
            }
            if (tid == 0) p.topk_count[item] = want;
        }
        if (RECYCLE) {
            int err = 0;
            const int n_ev = packed_tot >> 16;
            if (tid == 0) L.list_base = n_prom > 0 ? atomicAdd(&r.counters[2], n_prom) : 0;
            // evicted pages, in ascending page order, hand their blocks to the tail of the available list
            int q = n_free + r_ev0;
#pragma unroll
            for (int i = 0; i < FC_FAST_CACHED; ++i)
                if ((ev >> i) & 1u) {
                    if (q < p.Kmax) avail[q] = treg[i]; else err |= FC_DEV_ERR_FREE_OVERFLOW;
                    tbl[pg0 + i] = 0;
                    ++q;
                }
            const int pool = min(n_free + n_ev, p.Kmax);
            __syncthreads();
            const int list_base = L.list_base;
            // promoted pages, in ascending page order, take blocks from its front
            q = r_pr;
#pragma unroll
            for (int i = 0; i < FC_FAST_CACHED; ++i)
                if ((pr >> i) & 1u) {
                    long long blk = 0, hb = hreg[i];
                    if (q < pool) {
                        blk = avail[q];
                        if (blk < 1 || blk >= r.num_pool_blocks || hb < 0 || hb >= r.num_host_blocks) {
                            err |= FC_DEV_ERR_CLAMPED;     // never copy to or from outside the pools
                            blk = 0;
                            hb = 0;
                        }
                        tbl[pg0 + i] = (int32_t)blk;
                    } else {
                        err |= FC_DEV_ERR_NO_BLOCK;        // keep the list well formed: a no-op pair
                        hb = 0;
                    }
                    if (list_base + q < r.list_capacity) {
                        r.copy_list[2 * (size_t)(list_base + q) + 0] = (int32_t)hb;
                        r.copy_list[2 * (size_t)(list_base + q) + 1] = (int32_t)blk;
                    }
                    ++q;
                }
            // what is left of the available list is the new free list
            const int used = min(n_prom, pool), left = pool - used;
            int32_t *fb = r.free_blocks + item * (size_t)p.Kmax;
            if (!skip) {
                for (int i = tid; i < left; i += THREADS) fb[i] = avail[used + i];
                if (tid == 0) {
                    r.free_count[item] = left;
                    r.resident_count[item] = want;
                }
            }
            if (r.promoted_flags && skip)      // sequences that did not rerank promoted nothing
                for (int i = tid; i < p.Kmax; i += THREADS) r.promoted_flags[item * (size_t)p.Kmax + i] = 0;
            if (r.promoted_flags && !skip)
                for (int i = want + tid; i < p.Kmax; i += THREADS) r.promoted_flags[item * (size_t)p.Kmax + i] = 0;
            if (tid == 0 && r.promoted_count) r.promoted_count[item] = n_prom;
            if (err) atomicOr(&r.counters[1], err);
            if (tid == 0 && r.publish) {          // FC_PROMOTE_MEMCPY: the workgroup that finishes last publishes the pair count
                __threadfence();
                const int done = atomicAdd(&r.counters[4], 1);
                if (done == (int)(gridDim.x * gridDim.y) - 1) {
                    const int total = atomicAdd(&r.counters[2], 0);
                    if (r.host_total) *r.host_total = total;
                    if (r.host_total2) *r.host_total2 = total;
                    r.counters[2] = 0;
                    r.counters[4] = 0;
                }
            }
        }
    }
}

// Validates, then launches the score kernel and the selection.  With `fuse` (the filled parameters of the block
// recycling that is to follow) and shapes that allow it, selection and recycling run in one kernel and *fused is
// set; otherwise only the selection is launched and the caller launches the recycling kernel itself.
int fc_rerank_launch(fc_ctx *ctx, const fc_rerank_args *a, const fc_promote_params *fuse, hipStream_t s, bool *fused)
{
    if (fused) *fused = false;
    FC_REQUIRE(ctx, a, "fc_rerank_topk: args is NULL");
    FC_REQUIRE(ctx, a->q && a->minmax && a->context_lens && a->stable_flag && a->k_per_seq && a->topk_pages && a->topk_count,
               "fc_rerank_topk: NULL pointer among q, minmax, context_lens, stable_flag, k_per_seq, topk_pages, topk_count");
    FC_REQUIRE(ctx, a->batch >= 1 && a->batch <= ctx->cfg.max_batch, "fc_rerank_topk: batch=%d outside 1..%d", a->batch, ctx->cfg.max_batch);

    fc_rerank_params p;
    p.q = (const uint16_t *)a->q;
    p.minmax = (const char *)a->minmax;
    p.context_lens = a->context_lens;
    p.k_per_seq = a->k_per_seq;
    p.rerank_mask = a->rerank_mask;
    p.batch = a->batch;
    p.Hq = ctx->cfg.num_q_heads;
    p.Hkv = ctx->cfg.num_kv_heads;
    p.G = ctx->G;
    p.Nmax = ctx->cfg.max_pages_per_seq;
    p.Kmax = ctx->cfg.max_topk;
    p.n_stable = 0;
    memset(p.heads, 0, sizeof p.heads);
    for (int h = 0; h < p.Hkv; ++h)
        if (a->stable_flag[h]) p.heads[p.n_stable++] = (uint8_t)h;
    p.scores = a->scores_out ? a->scores_out : fc_ws_ptr<float>(ctx, ctx->lay.scores);
    p.topk_pages = a->topk_pages;
    p.topk_count = a->topk_count;
    if (p.n_stable == 0) return FC_OK;

    dim3 g1((p.Nmax + FC_SCORE_PAGES_PER_BLOCK - 1) / FC_SCORE_PAGES_PER_BLOCK, p.n_stable, p.batch);
    hipLaunchKernelGGL(fc_score_kernel, g1, dim3(256), 0, s, p);
    dim3 g2(p.n_stable, p.batch);
    if (p.Nmax <= FC_FAST_MAX_PAGES) {
        const size_t list_bytes = (size_t)p.Kmax * sizeof(int32_t);      // the head's available blocks
        const bool fuse_now = fuse && list_bytes <= FC_RECYCLE_MAX_LDS;
        fc_promote_params r;
        if (fuse_now) r = *fuse; else memset(&r, 0, sizeof r);
        if (p.Nmax <= FC_FAST_MAX_PAGES_256) {
            if (fuse_now) hipLaunchKernelGGL((fc_select_fast_kernel<256, true>), g2, dim3(256), list_bytes, s, p, r);
            else hipLaunchKernelGGL((fc_select_fast_kernel<256, false>), g2, dim3(256), 0, s, p, r);
        } else {
            if (fuse_now) hipLaunchKernelGGL((fc_select_fast_kernel<1024, true>), g2, dim3(1024), list_bytes, s, p, r);
            else hipLaunchKernelGGL((fc_select_fast_kernel<1024, false>), g2, dim3(1024), 0, s, p, r);
        }
        if (fused) *fused = fuse_now;
    } else {
        hipLaunchKernelGGL(fc_select_kernel, g2, dim3(FC_SELECT_THREADS), 0, s, p);
    }
    FC_HIP(ctx, hipGetLastError());
    return FC_OK;
}

extern "C" int fc_rerank_topk(fc_ctx *ctx, const fc_rerank_args *a, void *stream)
{
    if (!ctx) return FC_ERR_INVALID_ARG;
    return fc_rerank_launch(ctx, a, nullptr, (hipStream_t)stream, nullptr);
}
