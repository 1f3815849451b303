// Block recycling of one (sequence, stable head) (Sec. 3.3 "Minimizing Transfer Size", Sec. 3.4 "Physical Block
// Reuse During Reranking" and "Uniformity Through Null Block"), as a workgroup-wide device function shared by the
// stand-alone recycling kernel of fc_promote_pages and by the kernel of fc_rerank_promote that selects and
// recycles in one launch (the fused kernel of Sec. 3.4).
//
//   evicted = resident \ new, promoted = new \ resident (binary searches in the ascending lists);
//   available blocks = the head's free list, then the blocks of the evicted pages in ascending page order;
//   promoted pages, in ascending page order, take them from the front; evicted table entries become the null
//   block 0; one (host block, HBM block) pair per promoted page goes to the global copy list; what is left of
//   the available blocks is the new free list; the new list becomes the resident list.
//
// All three lists (old, new, available blocks) live in LDS, so the only dependent global round trips are
// (1) the table entries of the evicted pages, the host-table entries of the promoted pages and the atomic
// that reserves the copy-list range, all issued together, and (2) the stores.
#pragma once

#include "fc_internal.h"

constexpr size_t FC_RECYCLE_MAX_LDS = 48 * 1024;   // dynamic LDS the list-in-LDS kernels may ask for (3 * Kmax ints)

struct fc_promote_params {
    const int32_t *new_pages;
    const int32_t *new_count;
    int32_t *resident_pages;
    int32_t *resident_count;
    int32_t *block_table;
    const int32_t *host_block_table;
    int32_t *free_blocks;
    int32_t *free_count;
    const uint8_t *rerank_mask;
    int32_t *promoted_count;
    uint8_t *promoted_flags;
    int batch, Hkv, Nmax, Kmax, n_stable;
    uint8_t heads[64];
    long long num_pool_blocks, num_host_blocks;
    int32_t *copy_list;     // device or pinned: pairs (host block, pool block)
    int32_t *counters;      // device: [1] = error bits, [2] = pairs appended since the last copier ran, [4] = workgroups done
    int lds_lists;          // the page lists fit in dynamic LDS
    int publish;            // 1: this kernel's last workgroup publishes the pair count and clears it (FC_PROMOTE_MEMCPY: the host reads
                            // it); 0: the copier that follows does both, so this kernel ends without a device-wide ticket
    int32_t *host_total;    // pinned, may be NULL
    int32_t *host_total2;   // pinned scratch copy (memcpy mode reads it)
    int list_capacity;
};

// fc_rerank.hip: score + select, optionally with the recycling described by `fuse` in the same kernel
int fc_rerank_launch(fc_ctx *ctx, const fc_rerank_args *a, const fc_promote_params *fuse, hipStream_t s, bool *fused);

__device__ __forceinline__ bool fc_sorted_contains(const int32_t *a, int n, int x)
{
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        const int v = a[mid];
        if (v == x) return true;
        if (v < x) lo = mid + 1; else hi = mid;
    }
    return false;
}

// Exclusive prefix count of `flag` over a workgroup of THREADS threads; `total` gets the workgroup sum.
// `wave_cnt` holds THREADS / 64 ints of LDS.  Two barriers.
template <int THREADS>
__device__ __forceinline__ int fc_block_rank(bool flag, int *wave_cnt, int &total)
{
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const unsigned long long bal = __ballot(flag);
    if (lane == 0) wave_cnt[wv] = __popcll(bal);
    __syncthreads();
    int before = 0;
    total = 0;
#pragma unroll
    for (int k = 0; k < THREADS / 64; ++k) {
        const int c = wave_cnt[k];
        if (k < wv) before += c;
        total += c;
    }
    __syncthreads();
    return before + __popcll(bal & ((1ull << lane) - 1ull));
}

// LDS the body needs: 3 * Kmax ints (`lists`: old, new, available blocks) and THREADS / 64 + 1 ints (`wave_cnt`).
// On entry lists[0 .. n_old) holds the resident list and lists[Kmax .. Kmax + n_new) the new list (both already
// visible to the whole workgroup); n_old, n_new, n_free are clamped to 0..Kmax; `skip` = the sequence does not
// rerank in this call (its state stays as it is; its promoted flags and count are cleared).
template <int THREADS>
__device__ __forceinline__ void fc_recycle_body(const fc_promote_params &p, size_t item, bool skip, int n_old, int n_new,
                                                int n_free, int32_t *lists, int *wave_cnt)
{
    const int tid = threadIdx.x;
    int32_t *old_l = lists, *new_l = lists + p.Kmax, *avail = lists + 2 * p.Kmax;
    int32_t *tbl = p.block_table + item * (size_t)p.Nmax;
    const int32_t *htbl = p.host_block_table + item * (size_t)p.Nmax;
    int32_t *fb = p.free_blocks + item * (size_t)p.Kmax;
    int32_t *old_g = p.resident_pages + item * (size_t)p.Kmax;
    int err = 0;

    for (int i = tid; i < n_free; i += THREADS) avail[i] = fb[i];

    int pool = n_free, n_prom = 0, taken = 0;
    if (n_old <= THREADS && n_new <= THREADS) {
        // The usual case, one list entry per thread: the table entries of the evicted pages, the host-table entries of
        // the promoted pages and the atomic that reserves the copy-list range are all issued before any of them is
        // waited for, so the whole step is one memory round trip deep.
        int page_o = -1, page_n = -1;
        bool ev = false, pr = false;
        if (tid < n_old) {
            page_o = old_l[tid];
            ev = page_o >= 0 && page_o < p.Nmax && !fc_sorted_contains(new_l, n_new, page_o);
        }
        if (tid < n_new) {
            page_n = new_l[tid];
            pr = page_n >= 0 && page_n < p.Nmax && !fc_sorted_contains(old_l, n_old, page_n);
        }
        const int32_t blk_o = ev ? tbl[page_o] : 0;
        long long hb = pr ? htbl[page_n] : 0;
        int n_ev;
        const int r_ev = fc_block_rank<THREADS>(ev, wave_cnt, n_ev);
        const int r_pr = fc_block_rank<THREADS>(pr, wave_cnt, n_prom);
        if (tid == 0) wave_cnt[THREADS / 64] = n_prom > 0 ? atomicAdd(&p.counters[2], n_prom) : 0;
        if (ev) {
            if (pool + r_ev < p.Kmax) avail[pool + r_ev] = blk_o; else err |= FC_DEV_ERR_FREE_OVERFLOW;
            tbl[page_o] = 0;
        }
        pool = min(pool + n_ev, p.Kmax);
        __syncthreads();
        const int list_base = wave_cnt[THREADS / 64];
        if (p.promoted_flags && tid < n_new) p.promoted_flags[item * (size_t)p.Kmax + tid] = pr ? 1 : 0;
        if (pr) {
            long long blk = 0;
            if (r_pr < pool) {
                blk = avail[r_pr];
                if (blk < 1 || blk >= p.num_pool_blocks || hb < 0 || hb >= p.num_host_blocks) {
                    err |= FC_DEV_ERR_CLAMPED;     // never copy to or from outside the pools
                    blk = 0;
                    hb = 0;
                }
                tbl[page_n] = (int32_t)blk;
            } else {
                err |= FC_DEV_ERR_NO_BLOCK;        // keep the list well formed: a no-op pair
                hb = 0;
            }
            if (list_base + r_pr < p.list_capacity) {
                p.copy_list[2 * (size_t)(list_base + r_pr) + 0] = (int32_t)hb;
                p.copy_list[2 * (size_t)(list_base + r_pr) + 1] = (int32_t)blk;
            }
        }
        taken = n_prom;
    } else {
        // 1. evicted pages hand their blocks to the tail of the available list; their table entries become the null block
        for (int base = 0; base < n_old; base += THREADS) {
            const int i = base + tid;
            int page = -1;
            bool ev = false;
            if (i < n_old) {
                page = old_l[i];
                ev = page >= 0 && page < p.Nmax && !fc_sorted_contains(new_l, n_new, page);
            }
            const int32_t blk = ev ? tbl[page] : 0;
            int tot;
            const int r = fc_block_rank<THREADS>(ev, wave_cnt, tot);
            if (ev) {
                if (pool + r < p.Kmax) avail[pool + r] = blk; else err |= FC_DEV_ERR_FREE_OVERFLOW;
                tbl[page] = 0;
            }
            pool += tot;
        }
        if (pool > p.Kmax) pool = p.Kmax;

        // 2. promoted pages: their count reserves a range of the global copy list
        for (int base = 0; base < n_new; base += THREADS) {
            const int i = base + tid;
            bool pr = false;
            if (i < n_new) {
                const int page = new_l[i];
                pr = page >= 0 && page < p.Nmax && !fc_sorted_contains(old_l, n_old, page);
            }
            n_prom += __syncthreads_count(pr);
        }
        if (tid == 0) wave_cnt[THREADS / 64] = n_prom > 0 ? atomicAdd(&p.counters[2], n_prom) : 0;
        __syncthreads();      // also makes every avail[] entry of step 1 visible
        const int list_base = wave_cnt[THREADS / 64];

        // 3. promoted pages, in ascending page order, take blocks from the front of the available list
        for (int base = 0; base < n_new; base += THREADS) {
            const int i = base + tid;
            int page = -1;
            bool pr = false;
            if (i < n_new) {
                page = new_l[i];
                pr = page >= 0 && page < p.Nmax && !fc_sorted_contains(old_l, n_old, page);
            }
            long long hb = pr ? htbl[page] : 0;
            int tot;
            const int r = taken + fc_block_rank<THREADS>(pr, wave_cnt, tot);
            if (p.promoted_flags && i < n_new) p.promoted_flags[item * (size_t)p.Kmax + i] = pr ? 1 : 0;
            if (pr) {
                long long blk = 0;
                if (r < pool) {
                    blk = avail[r];
                    if (blk < 1 || blk >= p.num_pool_blocks || hb < 0 || hb >= p.num_host_blocks) {
                        err |= FC_DEV_ERR_CLAMPED;     // never copy to or from outside the pools
                        blk = 0;
                        hb = 0;
                    }
                    tbl[page] = (int32_t)blk;
                } else {
                    err |= FC_DEV_ERR_NO_BLOCK;        // keep the list well formed: a no-op pair
                    hb = 0;
                }
                if (list_base + r < p.list_capacity) {
                    p.copy_list[2 * (size_t)(list_base + r) + 0] = (int32_t)hb;
                    p.copy_list[2 * (size_t)(list_base + r) + 1] = (int32_t)blk;
                }
            }
            taken += tot;
        }
    }
    // 4. what is left of the available list is the new free list
    const int used = min(taken, pool);
    const int left = pool - used;
    for (int i = tid; i < left; i += THREADS) fb[i] = avail[used + i];
    if (p.promoted_flags)      // entries past the list, and whole lists of sequences that did not rerank, are not promoted
        for (int i = (skip ? 0 : n_new) + tid; i < p.Kmax; i += THREADS) p.promoted_flags[item * (size_t)p.Kmax + i] = 0;
    // 5. the new list becomes the resident list
    if (!skip) {
        for (int i = tid; i < p.Kmax; i += THREADS) old_g[i] = i < n_new ? new_l[i] : -1;
        if (tid == 0) {
            p.free_count[item] = left;
            p.resident_count[item] = n_new;
        }
    }
    if (tid == 0 && p.promoted_count) p.promoted_count[item] = n_prom;
    if (err) atomicOr(&p.counters[1], err);
    // 6. (FC_PROMOTE_MEMCPY only; otherwise the gather kernel does this) the workgroup that finishes last
    //    publishes the pair count and clears the other counter
    if (tid == 0 && p.publish) {
        __threadfence();
        const int done = atomicAdd(&p.counters[4], 1);
        if (done == (int)(gridDim.x * gridDim.y) - 1) {
            const int total = atomicAdd(&p.counters[2], 0);
            if (p.host_total) *p.host_total = total;
            if (p.host_total2) *p.host_total2 = total;
            p.counters[2] = 0;
            p.counters[4] = 0;
        }
    }
}
