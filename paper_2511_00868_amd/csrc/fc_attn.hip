// fc_sparse_decode_attn: head-heterogeneous paged decode attention (Sec. 3.1 of the paper; the
// split-KV + merge structure of decode attention named in Sec. 4.1).
//
// Two kernels per call.  In the first, every workgroup first derives the same schedule: the page count of every
// (sequence, KV head) item -- all pages for an unstable head, the top-K count for a stable one --
// and their prefix sums (kept in LDS).  The concatenated page lists are cut into equal shares, one
// per wavefront, independent of item boundaries, so a 2048-page unstable head and a 204-page stable
// head cost the same per page and no wavefront is left with a long tail.  Per page: QK^T and PV on
// the matrix cores, online softmax in registers.  A wavefront that saw a whole item writes the
// result directly; otherwise it leaves a partial (m, l, acc), and a second, small kernel combines
// the partials of every split item (log-sum-exp merge).  (Combining inside the first kernel by the
// last wavefront to arrive was tried and was twice as slow: every wavefront then pays a device-scope
// release fence, and the lone merging wavefront serialises the tail.)
//
// Matrix-core mapping (wave64, 16x16 tiles; lane = 16*j + n):
//   S^T[key][query] = K_page[16 x 128] . Q^T[128 x 16]   4 x v_mfma_f32_16x16x32_bf16
//       A = K straight from the page: the K half is stored as four 1 KiB chunks of 32 dims, one 64-byte row
//       per key inside a chunk, so MFMA s reads chunk s as one contiguous 1 KiB (lane: key row n, dims 32s+8j..+8),
//       B = Q^T, the G real query heads in columns 0..G-1, zero columns after them.
//       The result leaves lane (n, j) holding keys 4j..4j+3 of query n ...
//   O^T[dim][query] += V^T[16 dims x 16 keys] . P^T[16 keys x 16 queries]   8 x v_mfma_f32_16x16x16_bf16
//       ... which is exactly the B-operand layout of the 16x16x16 shape, so the probabilities never
//       move between lanes.  A = the dim-major V half of the page (lane reads 8 B: dim 16c+n,
//       keys 4j..4j+3).  P is split into a high and a low bf16 part (two MFMAs) so that PV keeps
//       ~16 mantissa bits; a single bf16 P would by itself cost 2^-9 relative error.
#include <math.h>
#include <stdarg.h>

#include <mutex>

#include "fc_internal.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short short4_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float float4_t;

constexpr int FC_ATTN_NBUF = 3;   // pages in flight per wavefront
constexpr int FC_MIN_PAGES_PER_WAVE = 2;

struct fc_attn_params {
    const uint16_t *q;
    const char *pool;
    long long num_blocks;
    const int32_t *block_table;
    const int32_t *context_lens;
    const int32_t *topk_pages;
    const int32_t *topk_count;
    unsigned long long stable_mask;
    unsigned long long active_mask;   // heads this call covers
    int batch, Hq, Hkv, G, Nmax, Kmax;
    int n_waves;
    float scale_log2;
    int32_t *seg_start;   // [2][max_items + 2]: per schedule the prefix sums, then pages per wavefront
    int sched;            // schedule / partial-slot set this attention launch writes (0 or 1)
    int sched_unstable, sched_stable;   // which set the merge reads for each class of head
    int stable_both_sets;  // merge: a stable item has partials in set 0 (resident pages) and set 1 (promoted pages)
    int page_filter;       // 0: every page; 1: skip list entries flagged as just promoted; 2: only those
    const uint8_t *promoted_flags;   // [batch][Hkv][Kmax], parallel to topk_pages (page_filter != 0)
    int sched_stride, slot_stride;
    float *part_ml;
    float *part_acc;
    float *out;
    float *lse;
    int32_t *err;          // device error word (may be NULL): set when an id had to be clamped or an attended page is not resident
    int attn_blocks;       // workgroups 0 .. attn_blocks-1 attend; any beyond them copy promoted pages (copy_blocks of them)
    int copy_blocks;
    fc_copy_job copies;
};

__device__ __forceinline__ int fc_pages_of(int ctx, int Nmax)
{
    int n = (ctx + FC_P - 1) / FC_P;
    return n < 0 ? 0 : (n > Nmax ? Nmax : n);
}

// ---- partial ---------------------------------------------------------------------------------------
// K/V pages are read once per call and never again before they have long left every cache: the
// non-temporal hint keeps them from displacing the queries, tables and partials (measured: 104 -> 92 us
// per call on the 32k-context benchmark).
#define FC_PAGE_LOAD(p) __builtin_nontemporal_load(p)

struct fc_page_regs {
    bf16x8_t k[4];
    short4_t v[8];
};

__device__ __forceinline__ void fc_load_page(fc_page_regs &r, const char *pool, int blk, int lane_k_off, int lane_v_off)
{
    const char *base = pool + (size_t)blk * FC_PAGE_BYTES;
#pragma unroll
    for (int s = 0; s < 4; ++s)
        r.k[s] = FC_PAGE_LOAD(reinterpret_cast<const bf16x8_t *>(base + lane_k_off + s * 1024));
#pragma unroll
    for (int c = 0; c < 8; ++c)
        r.v[c] = FC_PAGE_LOAD(reinterpret_cast<const short4_t *>(base + FC_HALF_BYTES + lane_v_off + c * 512));
}

struct fc_softmax_state {
    float m;          // running maximum of the scaled logits, log2 units, common to the 4 lanes of a query
    float l;          // this lane's share of the running denominator
    float4_t acc[8];  // O^T[dim 16c + 4j + v][query n]
};

__device__ __forceinline__ void fc_consume_page(fc_softmax_state &st, fc_page_regs &r, const bf16x8_t (&qb)[4],
                                                int ntok, int j, float scale_log2)
{
    float4_t s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 4; ++i) s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(r.k[i], qb[i], s, 0, 0, 0);

    float z[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) z[v] = (4 * j + v < ntok) ? s[v] * scale_log2 : -INFINITY;
    if (ntok < FC_P) {   // partial page: pad tokens may hold anything, and 0 * NaN would poison PV
#pragma unroll
        for (int c = 0; c < 8; ++c)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (4 * j + e >= ntok) r.v[c][e] = 0;
    }
    float mloc = fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3]));
    mloc = fmaxf(mloc, __shfl_xor(mloc, 16));
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
    const float m_new = fmaxf(st.m, mloc);
    const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);
    float pr[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) pr[v] = __builtin_amdgcn_exp2f(z[v] - m_new);
    st.l = st.l * alpha + ((pr[0] + pr[1]) + (pr[2] + pr[3]));
    st.m = m_new;
    if (__any(alpha != 1.0f)) {
#pragma unroll
        for (int c = 0; c < 8; ++c) st.acc[c] *= alpha;
    }
    // P = hi + lo, both bf16: hi is P truncated to 8 mantissa bits, lo the remainder (exact in fp32)
    // rounded to nearest, so P is carried with a relative error of at most 2^-17
    short4_t ph, pl;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const uint32_t u = __float_as_uint(pr[v]);
        const float hi = __uint_as_float(u & 0xFFFF0000u);
        const uint32_t r = __float_as_uint(pr[v] - hi);
        ph[v] = (short)(u >> 16);
        pl[v] = (short)((r + 0x7FFFu + ((r >> 16) & 1u)) >> 16);
    }
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        st.acc[c] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(r.v[c], ph, st.acc[c], 0, 0, 0);
        st.acc[c] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(r.v[c], pl, st.acc[c], 0, 0, 0);
    }
}

// Writes the final result of one (sequence, KV head) item for query column n of this lane.
__device__ __forceinline__ void fc_store_final(const fc_attn_params &p, size_t row, int n, int j, float m, float l,
                                               const float4_t (&acc)[8])
{
    if (n < p.G) {
        const float inv = 1.0f / l;
        float *dst = p.out + (row + n) * FC_D + 4 * j;
#pragma unroll
        for (int c = 0; c < 8; ++c) *reinterpret_cast<float4_t *>(dst + 16 * c) = acc[c] * inv;
        if (p.lse && j == 0) p.lse[row + n] = (m + __builtin_amdgcn_logf(l)) * 0.6931471805599453f;
    }
}

// SUBSET only names the launch (FC_HEADS_ALL ... FC_PAGES_PROMOTED) so that profilers list the kinds
// of launch, which move very different numbers of bytes, under separate kernel names.
template <int SUBSET>
__global__ __launch_bounds__(256, 2) void fc_decode_attn_kernel(fc_attn_params p)
{
    // Page copies riding in this launch (FC_PROMOTE_RIDE): the workgroups behind the attention ones pull the
    // promoted pages out of host memory while this launch attends over what is already in HBM -- the overlap
    // of Sec. 3.3 without a second stream and without any event.  One wavefront per copying workgroup.
    if ((int)blockIdx.x >= p.attn_blocks) {
        if (threadIdx.x < FC_COPY_THREADS) fc_copy_pages(p.copies, blockIdx.x - p.attn_blocks, p.copy_blocks, threadIdx.x);
        return;
    }
    __shared__ int seg[FC_MAX_ITEMS + 1];     // seg[i] = first page of item i in the concatenated order
    __shared__ int wave_tot[4];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int items = p.batch * p.Hkv;

    // ---- schedule: every workgroup derives the same page counts and prefix sums -------------------
    {
        int carry = 0;
        if (tid == 0) seg[0] = 0;
        for (int base = 0; base < items; base += 256) {
            const int i = base + tid;
            int cnt = 0;
            if (i < items) {
                const int b = i / p.Hkv, h = i - b * p.Hkv;
                const int n = fc_pages_of(p.context_lens[b], p.Nmax);
                if (!((p.active_mask >> h) & 1ull)) {
                    cnt = 0;
                } else if ((p.stable_mask >> h) & 1ull) {
                    const int k = p.topk_count[i];
                    cnt = k < 0 ? 0 : (k > n ? n : k);
                    if (cnt > p.Kmax) cnt = p.Kmax;
                } else {
                    cnt = n;
                }
            }
            int x = cnt;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int y = __shfl_up(x, d);
                if (lane >= d) x += y;
            }
            if (lane == 63) wave_tot[wv] = x;
            __syncthreads();
            int off = carry;
            for (int k = 0; k < 4; ++k) {
                const int c = wave_tot[k];
                if (k < wv) off += c;
                carry += c;
            }
            if (i < items) seg[i + 1] = off + x;
            __syncthreads();
        }
    }
    const int total = seg[items];
    int L = (total + p.n_waves - 1) / p.n_waves;
    if (L < FC_MIN_PAGES_PER_WAVE) L = FC_MIN_PAGES_PER_WAVE;
    if (blockIdx.x == 0) {                    // the merge kernel reads the schedule from memory
        int32_t *dst = p.seg_start + (size_t)p.sched * p.sched_stride;
        for (int i = tid; i <= items; i += 256) dst[i] = seg[i];
        if (tid == 0) dst[items + 1] = L;
    }
    const int w = blockIdx.x * 4 + wv;
    int g0 = w * L;
    const int g1 = min(g0 + L, total);
    if (g0 >= g1) return;
    int item;
    {   // the item with seg[item] <= g0 < seg[item + 1]
        int lo = 0, hi = items;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (seg[mid] <= g0) lo = mid; else hi = mid;
        }
        item = lo;
    }
    const int n = lane & 15, j = lane >> 4;
    const int lane_k_off = n * 64 + j * 16;     // chunk s of the K half: token row n, dims 32s + 8j .. + 8
    const int lane_v_off = n * 32 + j * 8;

    while (g0 < g1 && item < items) {
        const int s0 = seg[item], s1 = seg[item + 1];
        if (s1 <= g0) { ++item; continue; }             // empty item
        const int lo = g0 - s0, hi = min(g1, s1) - s0;
        const int b = item / p.Hkv, h = item - b * p.Hkv;
        const bool stable = (p.stable_mask >> h) & 1ull;
        const int ctx = p.context_lens[b];
        const int n_pages = fc_pages_of(ctx, p.Nmax);
        const int last_page = n_pages - 1;
        const int last_ntok = min(FC_P, ctx - last_page * FC_P);

        bf16x8_t qb[4];
        {
            const uint16_t *qrow = p.q + ((size_t)b * p.Hq + (size_t)h * p.G + (n < p.G ? n : 0)) * FC_D;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                bf16x8_t x = *reinterpret_cast<const bf16x8_t *>(qrow + 32 * s + 8 * j);
                if (n >= p.G) x = bf16x8_t{0, 0, 0, 0, 0, 0, 0, 0};
                qb[s] = x;
            }
        }
        fc_softmax_state st;
        st.m = -INFINITY;
        st.l = 0.f;
#pragma unroll
        for (int c = 0; c < 8; ++c) st.acc[c] = float4_t{0.f, 0.f, 0.f, 0.f};

        const int32_t *tbl = p.block_table + (size_t)item * p.Nmax;
        const int32_t *lst = p.topk_pages + (size_t)item * p.Kmax;
        for (int base = lo; base < hi; base += 64) {
            const int cnt = min(64, hi - base);
            int blk_v = 0, ntok_v = FC_P;
            int bad = 0;
            if (lane < cnt) {
                const int listed = stable ? lst[base + lane] : base + lane;
                const int logical = listed < 0 ? 0 : (listed > last_page ? last_page : listed);
                const long long entry = tbl[logical];
                const long long blk = entry < 0 ? 0 : (entry >= p.num_blocks ? p.num_blocks - 1 : entry);
                blk_v = (int)blk;
                ntok_v = logical == last_page ? last_ntok : FC_P;
                if (p.page_filter != 0) {     // 0 valid tokens = this call leaves the page to its partner call
                    const bool fresh = stable && p.promoted_flags[(size_t)item * p.Kmax + base + lane] != 0;
                    if ((p.page_filter == 1) == fresh) ntok_v = 0;
                }
                // ids stay in bounds whatever the tables hold, but a clamped id or an attended page without a block
                // (entry 0, the null block) means the caller's state is broken: say so instead of answering plausibly
                if (ntok_v > 0) {
                    if (listed != logical || entry != blk) bad = FC_DEV_ERR_CLAMPED;
                    else if (blk == 0) bad = FC_DEV_ERR_NOT_RESIDENT;
                }
            }
            if (p.err && __any(bad != 0) && bad != 0) atomicOr(p.err, bad);
            fc_page_regs buf[FC_ATTN_NBUF];
#pragma unroll
            for (int i = 0; i < FC_ATTN_NBUF; ++i)
                if (i < cnt && __builtin_amdgcn_readlane(ntok_v, i) > 0)
                    fc_load_page(buf[i], p.pool, __builtin_amdgcn_readlane(blk_v, i), lane_k_off, lane_v_off);
            for (int t0 = 0; t0 < cnt; t0 += FC_ATTN_NBUF) {
#pragma unroll
                for (int i = 0; i < FC_ATTN_NBUF; ++i) {
                    const int t = t0 + i;
                    if (t < cnt) {
                        const int ntok = __builtin_amdgcn_readlane(ntok_v, t);
                        if (ntok > 0) fc_consume_page(st, buf[i], qb, ntok, j, p.scale_log2);
                        if (t + FC_ATTN_NBUF < cnt && __builtin_amdgcn_readlane(ntok_v, t + FC_ATTN_NBUF) > 0)
                            fc_load_page(buf[i], p.pool, __builtin_amdgcn_readlane(blk_v, t + FC_ATTN_NBUF),
                                         lane_k_off, lane_v_off);
                    }
                }
            }
        }
        float l = st.l;
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);

        const size_t row = (size_t)b * p.Hq + (size_t)h * p.G;
        const int w_first = s0 / L, w_last = (s1 - 1) / L;
        if (w_first == w_last && !(stable && p.page_filter != 0)) {
            fc_store_final(p, row, n, j, st.m, l, st.acc);           // this wavefront saw the whole item
        } else {
            const int slot = p.sched * p.slot_stride + w + item;
            if (n < p.G) {
                if (j == 0) {
                    p.part_ml[((size_t)slot * 16 + n) * 2 + 0] = st.m;
                    p.part_ml[((size_t)slot * 16 + n) * 2 + 1] = l;
                }
                float *dst = p.part_acc + ((size_t)slot * p.G + n) * FC_D + 4 * j;
#pragma unroll
                for (int c = 0; c < 8; ++c) *reinterpret_cast<float4_t *>(dst + 16 * c) = st.acc[c];
            }
        }
        g0 = s0 + hi;
        ++item;
    }
}

// ---- merge -----------------------------------------------------------------------------------------
// One workgroup per (split item, query head).  Threads first run over the partials (maximum, then
// weights into LDS, 256 at a time), then over the output: thread = (sub, d4) accumulates every 8th
// partial for 4 output dims; the 8 sub-sums are combined through LDS.
constexpr int FC_MERGE_DIRECT = 128;      // partials of one item that the merge handles with every load issued up front

__global__ __launch_bounds__(256) void fc_attn_merge_kernel(fc_attn_params p)
{
    __shared__ float wts[256];
    __shared__ float red[8];
    __shared__ float4_t accs[8][32];
    const int item = blockIdx.x, g = blockIdx.y;
    const int items = p.batch * p.Hkv;
    const int b = item / p.Hkv, h = item - b * p.Hkv;
    if (!((p.active_mask >> h) & 1ull)) return;   // not covered by this call: rows stay as they are
    const bool stable = (p.stable_mask >> h) & 1ull;
    const size_t row = (size_t)b * p.Hq + (size_t)h * p.G + g;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    // up to two runs of partials: [slot_a, slot_a + n_a) and [slot_b, slot_b + n_b)
    size_t slot_a = 0, slot_b = 0;
    int n_a = 0, n_b = 0;
    bool any_pages = false, direct = false;
    {
        const int sched = stable ? (p.stable_both_sets ? 0 : p.sched_stable) : p.sched_unstable;
        const int32_t *seg = p.seg_start + (size_t)sched * p.sched_stride;
        const int s0 = seg[item], s1 = seg[item + 1], L = seg[items + 1];
        if (s1 > s0) {
            any_pages = true;
            const int w_first = s0 / L, w_last = (s1 - 1) / L;
            direct = w_first == w_last && !(stable && p.stable_both_sets);
            n_a = w_last - w_first + 1;
            slot_a = (size_t)sched * p.slot_stride + item + w_first;
        }
    }
    if (stable && p.stable_both_sets) {
        const int32_t *seg = p.seg_start + (size_t)p.sched_stride;
        const int s0 = seg[item], s1 = seg[item + 1], L = seg[items + 1];
        if (s1 > s0) {
            const int w_first = s0 / L, w_last = (s1 - 1) / L;
            n_b = w_last - w_first + 1;
            slot_b = (size_t)p.slot_stride + item + w_first;
        }
    }
    if (!any_pages) {   // an item without pages: defined output
        if (tid < FC_D) p.out[row * FC_D + tid] = 0.f;
        if (p.lse && tid == 0) p.lse[row] = -INFINITY;
        return;
    }
    if (direct) return;                       // written directly by the attention kernel
    const int n_parts = n_a + n_b;
    auto slot_of = [&](int i) -> size_t { return i < n_a ? slot_a + i : slot_b + (i - n_a); };

    const int sub = tid >> 5, d4 = tid & 31;
    if (n_parts <= 32) {
        // The usual case (an item split over a few dozen wavefronts): every load is issued before any
        // result is needed, so the kernel is two dependent memory round trips (schedule, partials) deep.
        float4_t a4[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int k = sub + 8 * i;
            a4[i] = k < n_parts ? *reinterpret_cast<const float4_t *>(p.part_acc + (slot_of(k) * p.G + g) * FC_D + 4 * d4)
                                : float4_t{0.f, 0.f, 0.f, 0.f};
        }
        float m = -INFINITY, l = 0.f;
        if (tid < n_parts) {
            const float *ml = p.part_ml + (slot_of(tid) * 16 + g) * 2;
            m = ml[0];
            l = ml[1];
        }
        float mstar = m;       // partials sit in the first wavefront's lanes 0..31
#pragma unroll
        for (int d = 16; d >= 1; d >>= 1) mstar = fmaxf(mstar, __shfl_xor(mstar, d));
        const float wt = m == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m - mstar);
        float lsum = wt * l;
#pragma unroll
        for (int d = 16; d >= 1; d >>= 1) lsum += __shfl_xor(lsum, d);
        if (tid < 32) wts[tid] = wt;
        if (tid == 0) {
            red[0] = mstar;
            red[1] = lsum;
        }
        __syncthreads();
        float4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < 4; ++i) acc += wts[sub + 8 * i] * a4[i];
        accs[sub][d4] = acc;
        __syncthreads();
        mstar = red[0];
        lsum = red[1];
        if (tid < 32) {
            float4_t r = accs[0][tid];
#pragma unroll
            for (int k = 1; k < 8; ++k) r += accs[k][tid];
            *reinterpret_cast<float4_t *>(p.out + row * FC_D + 4 * tid) = r * (1.0f / lsum);
        }
        if (p.lse && tid == 0) p.lse[row] = (mstar + __builtin_amdgcn_logf(lsum)) * 0.6931471805599453f;
        return;
    }
    if (n_parts <= FC_MERGE_DIRECT) {
        // The same for an item split over up to 128 wavefronts (117 for an 8192-page head over 70-page shares): one
        // partial per thread of the first two wavefronts, sixteen accumulator rows per thread in flight.
        float4_t a4[FC_MERGE_DIRECT / 8];
        const int rounds = (n_parts + 7) >> 3;          // the same for the whole workgroup
#pragma unroll
        for (int i = 0; i < FC_MERGE_DIRECT / 8; ++i) {
            const int k = sub + 8 * i;
            a4[i] = float4_t{0.f, 0.f, 0.f, 0.f};
            if (i < rounds && k < n_parts)
                a4[i] = *reinterpret_cast<const float4_t *>(p.part_acc + (slot_of(k) * p.G + g) * FC_D + 4 * d4);
        }
        float m = -INFINITY, l = 0.f;
        if (tid < n_parts) {
            const float *ml = p.part_ml + (slot_of(tid) * 16 + g) * 2;
            m = ml[0];
            l = ml[1];
        }
        float mstar = m;       // one partial per thread of the first two wavefronts
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) mstar = fmaxf(mstar, __shfl_xor(mstar, d));
        if (lane == 0) red[wv] = mstar;
        __syncthreads();
        mstar = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        const float wt = m == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m - mstar);
        float lsum = wt * l;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) lsum += __shfl_xor(lsum, d);
        if (tid < FC_MERGE_DIRECT) wts[tid] = wt;
        if (lane == 0) red[4 + wv] = lsum;
        __syncthreads();
        lsum = (red[4] + red[5]) + (red[6] + red[7]);
        float4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < FC_MERGE_DIRECT / 8; ++i)
            if (i < rounds) acc += wts[sub + 8 * i] * a4[i];
        accs[sub][d4] = acc;
        __syncthreads();
        if (tid < 32) {
            float4_t r = accs[0][tid];
#pragma unroll
            for (int k = 1; k < 8; ++k) r += accs[k][tid];
            *reinterpret_cast<float4_t *>(p.out + row * FC_D + 4 * tid) = r * (1.0f / lsum);
        }
        if (p.lse && tid == 0) p.lse[row] = (mstar + __builtin_amdgcn_logf(lsum)) * 0.6931471805599453f;
        return;
    }

    float mstar = -INFINITY;
    for (int i = tid; i < n_parts; i += 256) mstar = fmaxf(mstar, p.part_ml[(slot_of(i) * 16 + g) * 2]);
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) mstar = fmaxf(mstar, __shfl_xor(mstar, d));
    if (lane == 0) red[wv] = mstar;
    __syncthreads();
    mstar = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();

    float lsum = 0.f;
    float4_t acc = {0.f, 0.f, 0.f, 0.f};
    for (int base = 0; base < n_parts; base += 256) {
        const int cnt = min(256, n_parts - base);
        if (tid < cnt) {
            const float *ml = p.part_ml + (slot_of(base + tid) * 16 + g) * 2;
            const float wt = ml[0] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ml[0] - mstar);   // a share with no page
            wts[tid] = wt;
            lsum += wt * ml[1];
        }
        __syncthreads();
#pragma unroll 8
        for (int k = sub; k < cnt; k += 8)
            acc += wts[k] * *reinterpret_cast<const float4_t *>(p.part_acc + (slot_of(base + k) * p.G + g) * FC_D + 4 * d4);
        __syncthreads();
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) lsum += __shfl_xor(lsum, d);
    if (lane == 0) red[4 + wv] = lsum;
    accs[sub][d4] = acc;
    __syncthreads();
    lsum = (red[4] + red[5]) + (red[6] + red[7]);
    if (tid < 32) {
        float4_t r = accs[0][tid];
#pragma unroll
        for (int k = 1; k < 8; ++k) r += accs[k][tid];
        *reinterpret_cast<float4_t *>(p.out + row * FC_D + 4 * tid) = r * (1.0f / lsum);
    }
    if (p.lse && tid == 0) p.lse[row] = (mstar + __builtin_amdgcn_logf(lsum)) * 0.6931471805599453f;
}

extern "C" int fc_sparse_decode_attn(fc_ctx *ctx, const fc_attn_args *a, void *stream)
{
    if (!ctx) return FC_ERR_INVALID_ARG;
    FC_REQUIRE(ctx, a, "fc_sparse_decode_attn: args is NULL");
    FC_REQUIRE(ctx, a->q && a->kv_pool && a->block_table && a->context_lens && a->stable_flag && a->out,
               "fc_sparse_decode_attn: NULL pointer among q, kv_pool, block_table, context_lens, stable_flag, out");
    FC_REQUIRE(ctx, a->batch >= 1 && a->batch <= ctx->cfg.max_batch, "fc_sparse_decode_attn: batch=%d outside 1..%d", a->batch, ctx->cfg.max_batch);
    FC_REQUIRE(ctx, a->num_pool_blocks >= 2, "fc_sparse_decode_attn: num_pool_blocks must be >= 2");
    FC_REQUIRE(ctx, a->head_subset >= FC_HEADS_ALL && a->head_subset <= FC_PAGES_PROMOTED, "fc_sparse_decode_attn: unknown head_subset %d", a->head_subset);
    FC_REQUIRE(ctx, a->head_subset < FC_PAGES_RESIDENT || a->promoted_flags, "fc_sparse_decode_attn: FC_PAGES_RESIDENT / FC_PAGES_PROMOTED need promoted_flags");
    const uint64_t mask = fc_stable_mask(ctx->cfg, a->stable_flag);
    FC_REQUIRE(ctx, mask == 0 || (a->topk_pages && a->topk_count), "fc_sparse_decode_attn: stable heads need topk_pages and topk_count");
    FC_REQUIRE(ctx, !ctx->copies_deferred || stream == ctx->copies_stream,
               "fc_sparse_decode_attn: after FC_PROMOTE_RIDE the next attention call belongs on fc_promote_pages' main_stream");
    hipStream_t s = (hipStream_t)stream;

    fc_attn_params p;
    p.q = (const uint16_t *)a->q;
    p.pool = (const char *)a->kv_pool;
    p.num_blocks = a->num_pool_blocks;
    p.block_table = a->block_table;
    p.context_lens = a->context_lens;
    p.topk_pages = a->topk_pages ? a->topk_pages : a->block_table;   // never read when mask == 0
    p.topk_count = a->topk_count ? a->topk_count : a->context_lens;
    p.stable_mask = mask;
    const uint64_t all = ctx->cfg.num_kv_heads == 64 ? ~0ull : ((1ull << ctx->cfg.num_kv_heads) - 1);
    const int sub = a->head_subset;
    p.active_mask = sub == FC_HEADS_UNSTABLE ? (all & ~mask) : (sub == FC_HEADS_STABLE || sub == FC_PAGES_PROMOTED) ? mask : all;
    // A first call of a pair (FC_HEADS_UNSTABLE or FC_PAGES_RESIDENT) leaves its partials in set 0 and
    // defers the merge; the second (FC_HEADS_STABLE or FC_PAGES_PROMOTED) writes set 1 and merges both.
    p.sched = (sub == FC_HEADS_STABLE || sub == FC_PAGES_PROMOTED) ? 1 : 0;
    p.sched_unstable = 0;
    p.sched_stable = p.sched;
    p.stable_both_sets = sub == FC_PAGES_PROMOTED ? 1 : 0;
    p.page_filter = sub == FC_PAGES_RESIDENT ? 1 : sub == FC_PAGES_PROMOTED ? 2 : 0;
    p.promoted_flags = a->promoted_flags;
    p.sched_stride = ctx->max_items + 2;
    p.slot_stride = ctx->slots;
    p.batch = a->batch;
    p.Hq = ctx->cfg.num_q_heads;
    p.Hkv = ctx->cfg.num_kv_heads;
    p.G = ctx->G;
    p.Nmax = ctx->cfg.max_pages_per_seq;
    p.Kmax = ctx->cfg.max_topk;
    p.n_waves = ctx->attn_waves;
    p.scale_log2 = ctx->scale_log2;
    p.seg_start = fc_ws_ptr<int32_t>(ctx, ctx->lay.seg_start);
    p.part_ml = fc_ws_ptr<float>(ctx, ctx->lay.part_ml);
    p.part_acc = fc_ws_ptr<float>(ctx, ctx->lay.part_acc);
    p.out = a->out;
    p.lse = a->lse;
    p.err = fc_ws_ptr<int32_t>(ctx, ctx->lay.counters) + 1;

    const bool first_of_pair = sub == FC_HEADS_UNSTABLE || sub == FC_PAGES_RESIDENT;
    const bool merge_now = !first_of_pair;
    uint64_t merge_mask = p.active_mask;
    if (sub == FC_PAGES_PROMOTED) {
        FC_REQUIRE(ctx, ctx->pending_pair == FC_PAGES_RESIDENT, "fc_sparse_decode_attn: FC_PAGES_PROMOTED must follow FC_PAGES_RESIDENT");
        merge_mask = all;
    }
    if (sub == FC_HEADS_STABLE && ctx->pending_pair == FC_HEADS_UNSTABLE) merge_mask = all;
    // the two calls of a pair may sit on different streams: the merge then waits for the first call's stream
    const bool wait_first = merge_now && merge_mask == all && ctx->pending_pair != 0 && ctx->first_stream != stream;
    ctx->pending_pair = first_of_pair ? sub : 0;
    // block tables and promoted flags come from the last recycling kernel: a call on another stream than
    // that kernel's is ordered after it here (on its own stream the order is already given)
    if (ctx->diff_valid && stream != ctx->diff_stream) FC_HIP(ctx, hipStreamWaitEvent(s, ctx->ev_diff_done, 0));
    const bool needs_copies = sub != FC_HEADS_UNSTABLE && sub != FC_PAGES_RESIDENT && (p.active_mask & mask);
    // copies left by FC_PROMOTE_RIDE: a first call of a pair carries them in its own launch; before any other
    // call they are launched on their own
    p.attn_blocks = p.n_waves / 4;
    p.copy_blocks = 0;
    p.copies = fc_copy_job{};
    if (ctx->copies_deferred) {
        if (first_of_pair && p.active_mask != 0) {
            p.copy_blocks = ctx->ride_blocks;
            p.copies = ctx->deferred;
        } else {
            const int st = fc_launch_deferred_copies(ctx, stream);
            if (st != FC_OK) return st;
        }
    }
    if (needs_copies) {   // promoted pages may still be in flight
        const int st = fc_wait_for_copies(ctx, stream);
        if (st != FC_OK) return st;
    }
    if (p.active_mask != 0) {
        // kernel timing covers whole passes only: the split launches move other byte counts
        bool prof = ctx->profiling && a->head_subset == FC_HEADS_ALL && ctx->prof_used < FC_MAX_PROFILE_EVENTS;
        if (prof) prof = (ctx->prof_seen++ % ctx->prof_stride) == 0;
        if (prof) FC_HIP(ctx, hipEventRecord(ctx->prof_ev[2 * ctx->prof_used], s));
        const dim3 grid(p.attn_blocks + p.copy_blocks), block(256);
        if (sub == FC_HEADS_ALL) hipLaunchKernelGGL(fc_decode_attn_kernel<FC_HEADS_ALL>, grid, block, 0, s, p);
        else if (sub == FC_HEADS_UNSTABLE) hipLaunchKernelGGL(fc_decode_attn_kernel<FC_HEADS_UNSTABLE>, grid, block, 0, s, p);
        else if (sub == FC_HEADS_STABLE) hipLaunchKernelGGL(fc_decode_attn_kernel<FC_HEADS_STABLE>, grid, block, 0, s, p);
        else if (sub == FC_PAGES_RESIDENT) hipLaunchKernelGGL(fc_decode_attn_kernel<FC_PAGES_RESIDENT>, grid, block, 0, s, p);
        else hipLaunchKernelGGL(fc_decode_attn_kernel<FC_PAGES_PROMOTED>, grid, block, 0, s, p);
        if (prof) {
            FC_HIP(ctx, hipEventRecord(ctx->prof_ev[2 * ctx->prof_used + 1], s));
            ++ctx->prof_used;
        }
        FC_HIP(ctx, hipGetLastError());
    }
    if (p.copy_blocks) {          // the copies are in flight now, on this stream
        ctx->copies_deferred = false;
        ctx->copies_pending = true;
        ctx->copies_stream = stream;
        ctx->copies_recorded = false;
    }
    if (first_of_pair) ctx->first_stream = stream;
    if (wait_first) {   // the event goes behind the first call only now that a second stream turns out to need it
        FC_HIP(ctx, hipEventRecord(ctx->ev_first_done, (hipStream_t)ctx->first_stream));
        FC_HIP(ctx, hipStreamWaitEvent(s, ctx->ev_first_done, 0));
    }
    if (merge_now && merge_mask != 0) {
        p.active_mask = merge_mask;
        hipLaunchKernelGGL(fc_attn_merge_kernel, dim3(p.batch * p.Hkv, p.G), dim3(256), 0, s, p);
    }
    FC_HIP(ctx, hipGetLastError());
    return FC_OK;
}

// ---- whole-pass attention for callers that cannot allocate --------------------------------------------
// Same two kernels as fc_sparse_decode_attn (FC_HEADS_ALL), but the schedule and the split partials live
// in a fixed array that is part of the library's device image instead of in a caller-supplied workspace,
// and there is no context: nothing is allocated, created or freed, at set-up or per call.  Every call on
// a GPU uses that GPU's one copy of the array, so calls that overlap on one GPU race.  Nothing in the
// array has to start at zero: each call writes its schedule and every partial it later reads.
constexpr size_t FC_STATIC_SCRATCH_BYTES = (size_t)8 << 20;
static __device__ __align__(256) unsigned char fc_static_scratch[FC_STATIC_SCRATCH_BYTES];

constexpr int FC_STATIC_MAX_DEVICES = 64;
struct fc_static_device {
    bool ready;
    char *scratch;      // this device's address of fc_static_scratch
    int num_cus;
};
static fc_static_device fc_static_devices[FC_STATIC_MAX_DEVICES];
static std::mutex fc_static_mutex;
static thread_local char fc_static_err[256];

static int fc_static_fail(int status, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(fc_static_err, sizeof fc_static_err, fmt, ap);
    va_end(ap);
    return status;
}

extern "C" const char *fc_static_last_error(void) { return fc_static_err; }

extern "C" size_t fc_static_scratch_bytes(void) { return FC_STATIC_SCRATCH_BYTES; }

// Bytes of the array a call of this shape uses (one schedule, one set of partials).
static size_t fc_static_layout(int items, int waves, int G, size_t *ml_off, size_t *acc_off)
{
    const size_t slots = (size_t)waves + items;
    size_t off = fc_align_up((size_t)(items + 2) * sizeof(int32_t), 256);
    *ml_off = off;
    off = fc_align_up(off + slots * 16 * 2 * sizeof(float), 256);
    *acc_off = off;
    off = fc_align_up(off + slots * (size_t)G * FC_D * sizeof(float), 256);
    return off;
}

extern "C" int fc_sparse_decode_attn_static(const fc_config *cfg, const fc_attn_args *a, void *stream)
{
    fc_static_err[0] = 0;
    const char *why = nullptr;
    const int st = fc_check_config(cfg, &why);
    if (st != FC_OK) return fc_static_fail(st, "fc_sparse_decode_attn_static: %s", why);
    if (!a) return fc_static_fail(FC_ERR_INVALID_ARG, "fc_sparse_decode_attn_static: args is NULL");
    if (!(a->q && a->kv_pool && a->block_table && a->context_lens && a->stable_flag && a->out))
        return fc_static_fail(FC_ERR_INVALID_ARG, "fc_sparse_decode_attn_static: NULL pointer among q, kv_pool, block_table, context_lens, stable_flag, out");
    if (a->batch < 1 || a->batch > cfg->max_batch)
        return fc_static_fail(FC_ERR_INVALID_ARG, "fc_sparse_decode_attn_static: batch=%d outside 1..%d", a->batch, cfg->max_batch);
    if (a->num_pool_blocks < 2) return fc_static_fail(FC_ERR_INVALID_ARG, "fc_sparse_decode_attn_static: num_pool_blocks must be >= 2");
    if (a->head_subset != FC_HEADS_ALL)
        return fc_static_fail(FC_ERR_UNSUPPORTED, "fc_sparse_decode_attn_static: only FC_HEADS_ALL (one whole pass) is offered here");
    const uint64_t mask = fc_stable_mask(*cfg, a->stable_flag);
    if (mask != 0 && !(a->topk_pages && a->topk_count))
        return fc_static_fail(FC_ERR_INVALID_ARG, "fc_sparse_decode_attn_static: stable heads need topk_pages and topk_count");

    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fc_static_fail(FC_ERR_HIP, "fc_sparse_decode_attn_static: hipGetDevice failed: %s", hipGetErrorString(e));
    if (dev != cfg->device || dev >= FC_STATIC_MAX_DEVICES)
        return fc_static_fail(FC_ERR_INVALID_ARG, "fc_sparse_decode_attn_static: device %d of the configuration must be the current device (%d) and below %d",
                              cfg->device, dev, FC_STATIC_MAX_DEVICES);
    fc_static_device d;
    {
        std::lock_guard<std::mutex> lock(fc_static_mutex);
        d = fc_static_devices[dev];
    }
    if (!d.ready) {
        // first call on this device: where this device keeps its copy of the array, and how many compute units it has
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(fc_static_scratch));
        if (e != hipSuccess || !ptr)
            return fc_static_fail(FC_ERR_HIP, "fc_sparse_decode_attn_static: hipGetSymbolAddress failed: %s", hipGetErrorString(e));
        int cus = 0;
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess || cus <= 0)
            return fc_static_fail(FC_ERR_HIP, "fc_sparse_decode_attn_static: compute-unit count unavailable: %s", hipGetErrorString(e));
        d.scratch = (char *)ptr;
        d.num_cus = cus;
        d.ready = true;
        std::lock_guard<std::mutex> lock(fc_static_mutex);
        fc_static_devices[dev] = d;
    }

    const int G = cfg->num_q_heads / cfg->num_kv_heads;
    const int waves = fc_resolve_waves(cfg, d.num_cus);
    const int items = a->batch * cfg->num_kv_heads;
    size_t ml_off, acc_off;
    const size_t need = fc_static_layout(items, waves, G, &ml_off, &acc_off);
    if (need > FC_STATIC_SCRATCH_BYTES)
        return fc_static_fail(FC_ERR_WORKSPACE, "fc_sparse_decode_attn_static: batch %d x %d KV heads x group %d over %d wavefronts needs %zu bytes of "
                              "partials, the built-in array holds %zu: use fc_sparse_decode_attn with a workspace", a->batch, cfg->num_kv_heads, G,
                              waves, need, FC_STATIC_SCRATCH_BYTES);

    const float scale = cfg->softmax_scale > 0.0f ? cfg->softmax_scale : 1.0f / sqrtf((float)FC_D);
    fc_attn_params p;
    p.q = (const uint16_t *)a->q;
    p.pool = (const char *)a->kv_pool;
    p.num_blocks = a->num_pool_blocks;
    p.block_table = a->block_table;
    p.context_lens = a->context_lens;
    p.topk_pages = a->topk_pages ? a->topk_pages : a->block_table;   // never read when mask == 0
    p.topk_count = a->topk_count ? a->topk_count : a->context_lens;
    p.stable_mask = mask;
    p.active_mask = cfg->num_kv_heads == 64 ? ~0ull : ((1ull << cfg->num_kv_heads) - 1);
    p.batch = a->batch;
    p.Hq = cfg->num_q_heads;
    p.Hkv = cfg->num_kv_heads;
    p.G = G;
    p.Nmax = cfg->max_pages_per_seq;
    p.Kmax = cfg->max_topk;
    p.n_waves = waves;
    p.scale_log2 = scale * 1.4426950408889634f;
    p.seg_start = reinterpret_cast<int32_t *>(d.scratch);
    p.sched = 0;
    p.sched_unstable = 0;
    p.sched_stable = 0;
    p.stable_both_sets = 0;
    p.page_filter = 0;
    p.promoted_flags = nullptr;
    p.sched_stride = items + 2;
    p.slot_stride = waves + items;
    p.part_ml = reinterpret_cast<float *>(d.scratch + ml_off);
    p.part_acc = reinterpret_cast<float *>(d.scratch + acc_off);
    p.out = a->out;
    p.lse = a->lse;
    p.err = nullptr;       // no context, no error word: ids are clamped silently here
    p.attn_blocks = waves / 4;
    p.copy_blocks = 0;
    p.copies = fc_copy_job{};
    hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(fc_decode_attn_kernel<FC_HEADS_ALL>, dim3(p.attn_blocks), dim3(256), 0, s, p);
    hipLaunchKernelGGL(fc_attn_merge_kernel, dim3(items, G), dim3(256), 0, s, p);
    e = hipGetLastError();
    if (e != hipSuccess) return fc_static_fail(FC_ERR_HIP, "fc_sparse_decode_attn_static: launch failed: %s", hipGetErrorString(e));
    return FC_OK;
}
