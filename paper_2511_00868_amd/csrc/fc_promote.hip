// fc_promote_pages: set difference, physical block recycling, null block, host->HBM page copies
// (Sec. 3.3 "Minimizing Transfer Size" / "Overlapping Transfer with Compute" / "Reducing
// Fragmentation Overhead", Sec. 3.4 "Physical Block Reuse During Reranking" and "Uniformity Through
// Null Block").
//
// recycle kernel, one workgroup per (sequence, stable head), on the main stream:
//   evicted = resident \ new and promoted = new \ resident by binary search in the ascending lists;
//   the blocks of evicted pages are appended, in ascending page order, to the head's free list;
//   promoted pages, in ascending page order, take blocks from the front of that list; table entries
//   of evicted pages become the null block 0; one (host block, HBM block) pair per promoted page is
//   appended to a global copy list; the rest of the list becomes the new free list.
// page copies: a capped number of single-wavefront workgroups walk the copy list and pull each 8 KiB page
//   straight out of pinned host memory -- no host-side gather, no per-page API call, no host wait.  Three
//   ways to run them: FC_PROMOTE_RIDE leaves them to the next attention launch, which carries them in extra
//   workgroups beside its own (one stream, no event; the fastest); FC_PROMOTE_GATHER launches them here as
//   a kernel of their own, on side_stream or in line on main_stream; FC_PROMOTE_MEMCPY hands the list to the
//   host, which issues one hipMemcpyAsync per page.  The shape of the copiers is chosen for the attention
//   that runs beside them: host reads take microseconds, attention runs at about half speed while they are
//   in flight, and PCIe needs ~128 KiB in flight to stay saturated (~57 GB/s): 32-48 workgroups of one
//   wavefront with four 16 B loads per lane (measured per step on the 32k-context benchmark: as a kernel of
//   their own 16 -> 149 us, 32 -> 131, 64 -> 143; riding 32 -> 128.4, 40 -> 127.3).
#include "fc_recycle.h"

constexpr int FC_RECYCLE_THREADS = 256;

// Exclusive prefix count over the 256 threads of the fallback kernel below.
__device__ __forceinline__ int fc_block_rank256(bool flag, int *wave_cnt, int &total)
{
    return fc_block_rank<FC_RECYCLE_THREADS>(flag, wave_cnt, total);
}

// The usual kernel: one workgroup per (sequence, stable head), all three lists in LDS (3 * Kmax ints).
__global__ __launch_bounds__(FC_RECYCLE_THREADS) void fc_recycle_kernel(fc_promote_params p)
{
    __shared__ int wave_cnt[FC_RECYCLE_THREADS / 64 + 1];
    extern __shared__ int32_t lists[];
    const int b = blockIdx.y;
    const int h = p.heads[blockIdx.x];
    const size_t item = (size_t)b * p.Hkv + h;
    const int tid = threadIdx.x;
    const bool skip = p.rerank_mask && !p.rerank_mask[b];
    int n_old = 0, n_new = 0, n_free = 0;
    if (!skip) { n_old = p.resident_count[item]; n_new = p.new_count[item]; n_free = p.free_count[item]; }
    n_old = min(max(n_old, 0), p.Kmax);
    n_new = min(max(n_new, 0), p.Kmax);
    n_free = min(max(n_free, 0), p.Kmax);
    const int32_t *old_g = p.resident_pages + item * (size_t)p.Kmax;
    const int32_t *new_g = p.new_pages + item * (size_t)p.Kmax;
    for (int i = tid; i < n_old; i += FC_RECYCLE_THREADS) lists[i] = old_g[i];
    for (int i = tid; i < n_new; i += FC_RECYCLE_THREADS) lists[p.Kmax + i] = new_g[i];
    __syncthreads();
    fc_recycle_body<FC_RECYCLE_THREADS>(p, item, skip, n_old, n_new, n_free, lists, wave_cnt);
}

// Fallback for page budgets whose lists do not fit in LDS: the same steps on the lists in global memory.
__global__ __launch_bounds__(FC_RECYCLE_THREADS) void fc_recycle_global_kernel(fc_promote_params p)
{
    __shared__ int wave_cnt[FC_RECYCLE_THREADS / 64];
    __shared__ int sh_list_base;
    const int b = blockIdx.y;
    const int h = p.heads[blockIdx.x];
    const size_t item = (size_t)b * p.Hkv + h;
    const int tid = threadIdx.x;
    const bool skip = p.rerank_mask && !p.rerank_mask[b];
    int n_old = 0, n_new = 0, n_free = 0;
    if (!skip) { n_old = p.resident_count[item]; n_new = p.new_count[item]; n_free = p.free_count[item]; }
    n_old = min(max(n_old, 0), p.Kmax);
    n_new = min(max(n_new, 0), p.Kmax);
    n_free = min(max(n_free, 0), p.Kmax);
    int32_t *old_g = p.resident_pages + item * (size_t)p.Kmax;
    const int32_t *new_g = p.new_pages + item * (size_t)p.Kmax;
    const int32_t *old_l = old_g;
    const int32_t *new_l = new_g;
    int32_t *tbl = p.block_table + item * (size_t)p.Nmax;
    const int32_t *htbl = p.host_block_table + item * (size_t)p.Nmax;
    int32_t *fb = p.free_blocks + item * (size_t)p.Kmax;
    int err = 0;

    // 1. evicted pages release their blocks to the tail of the free list
    int pool = n_free;
    for (int base = 0; base < n_old; base += FC_RECYCLE_THREADS) {
        const int i = base + tid;
        int page = -1;
        bool ev = false;
        if (i < n_old) {
            page = old_l[i];
            ev = page >= 0 && page < p.Nmax && !fc_sorted_contains(new_l, n_new, page);
        }
        int tot;
        const int r = fc_block_rank256(ev, wave_cnt, tot);
        if (ev) {
            if (pool + r < p.Kmax) fb[pool + r] = tbl[page]; else err |= FC_DEV_ERR_FREE_OVERFLOW;
            tbl[page] = 0;
        }
        pool += tot;
    }
    if (pool > p.Kmax) pool = p.Kmax;
    __threadfence_block();
    __syncthreads();

    // 2. count promoted pages, reserve a range of the global copy list
    int n_prom = 0;
    for (int base = 0; base < n_new; base += FC_RECYCLE_THREADS) {
        const int i = base + tid;
        bool pr = false;
        if (i < n_new) {
            const int page = new_l[i];
            pr = page >= 0 && page < p.Nmax && !fc_sorted_contains(old_l, n_old, page);
        }
        int tot;
        fc_block_rank256(pr, wave_cnt, tot);
        n_prom += tot;
    }
    if (tid == 0) sh_list_base = n_prom > 0 ? atomicAdd(&p.counters[2], n_prom) : 0;
    __syncthreads();
    const int list_base = sh_list_base;

    // 3. promoted pages take blocks from the front of the free list
    int taken = 0;
    for (int base = 0; base < n_new; base += FC_RECYCLE_THREADS) {
        const int i = base + tid;
        int page = -1;
        bool pr = false;
        if (i < n_new) {
            page = new_l[i];
            pr = page >= 0 && page < p.Nmax && !fc_sorted_contains(old_l, n_old, page);
        }
        int tot;
        const int r = taken + fc_block_rank256(pr, wave_cnt, tot);
        if (p.promoted_flags && i < n_new) p.promoted_flags[item * (size_t)p.Kmax + i] = pr ? 1 : 0;
        if (pr) {
            if (r < pool) {
                long long blk = fb[r];
                long long hb = htbl[page];
                if (blk < 1 || blk >= p.num_pool_blocks || hb < 0 || hb >= p.num_host_blocks) {
                    err |= FC_DEV_ERR_CLAMPED;     // never copy to or from outside the pools
                    blk = 0;
                    hb = 0;
                }
                tbl[page] = (int32_t)blk;
                if (list_base + r < p.list_capacity) {
                    p.copy_list[2 * (size_t)(list_base + r) + 0] = (int32_t)hb;
                    p.copy_list[2 * (size_t)(list_base + r) + 1] = (int32_t)blk;
                }
            } else {
                err |= FC_DEV_ERR_NO_BLOCK;
                if (list_base + r < p.list_capacity) {   // keep the list well formed: a no-op pair
                    p.copy_list[2 * (size_t)(list_base + r) + 0] = 0;
                    p.copy_list[2 * (size_t)(list_base + r) + 1] = 0;
                }
            }
        }
        taken += tot;
    }
    __syncthreads();

    // 4. what is left of the free list moves to its front
    const int used = min(taken, pool);
    const int left = pool - used;
    for (int base = 0; base < left; base += FC_RECYCLE_THREADS) {   // ascending chunks: reads stay ahead of writes
        const int i = base + tid;
        int v = 0;
        if (i < left) v = fb[used + i];
        __syncthreads();
        if (i < left) fb[i] = v;
        __syncthreads();
    }
    if (p.promoted_flags)      // entries past the list, and whole lists of sequences that did not rerank, are not promoted
        for (int i = (skip ? 0 : n_new) + tid; i < p.Kmax; i += FC_RECYCLE_THREADS) p.promoted_flags[item * (size_t)p.Kmax + i] = 0;
    // 5. the new list becomes the resident list
    if (!skip) {
        for (int i = tid; i < p.Kmax; i += FC_RECYCLE_THREADS) old_g[i] = i < n_new ? new_l[i] : -1;
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

__global__ __launch_bounds__(FC_COPY_THREADS) void fc_gather_pages_kernel(fc_copy_job job)
{
    fc_copy_pages(job, blockIdx.x, gridDim.x, threadIdx.x);
}

// FC_PROMOTE_RIDE copies that no attention launch has carried yet: launched on their own, on `stream`.
int fc_launch_deferred_copies(fc_ctx *ctx, void *stream)
{
    if (!ctx->copies_deferred) return FC_OK;
    hipLaunchKernelGGL(fc_gather_pages_kernel, dim3(ctx->gather_blocks), dim3(FC_COPY_THREADS), 0, (hipStream_t)stream, ctx->deferred);
    FC_HIP(ctx, hipGetLastError());
    ctx->copies_deferred = false;
    ctx->copies_pending = true;
    ctx->copies_stream = stream;
    ctx->copies_recorded = false;
    return FC_OK;
}

// Orders `stream` after the page copies of the last fc_promote_pages, if they may still be running.
int fc_wait_for_copies(fc_ctx *ctx, void *stream)
{
    if (!ctx->copies_pending) return FC_OK;
    if (ctx->copies_stream != stream) {
        if (!ctx->copies_recorded) {
            FC_HIP(ctx, hipEventRecord(ctx->ev_copies_done, (hipStream_t)ctx->copies_stream));
            ctx->copies_recorded = true;
        }
        FC_HIP(ctx, hipStreamWaitEvent((hipStream_t)stream, ctx->ev_copies_done, 0));
    }
    ctx->copies_pending = false;
    return FC_OK;
}

// fc_promote_pages, optionally preceded by the scoring and selection of `rerank` (fc_rerank_promote): the selection
// then recycles each head's blocks in its own kernel when the shapes allow it.
static int fc_promote_impl(fc_ctx *ctx, const fc_promote_args *a, void *main_stream, void *side_stream, const fc_rerank_args *rerank)
{
    FC_REQUIRE(ctx, a, "fc_promote_pages: args is NULL");
    FC_REQUIRE(ctx, a->new_pages && a->new_count && a->resident_pages && a->resident_count && a->block_table &&
                        a->host_block_table && a->free_blocks && a->free_count && a->stable_flag && a->kv_pool && a->host_pool,
               "fc_promote_pages: NULL pointer among the required arguments");
    FC_REQUIRE(ctx, a->batch >= 1 && a->batch <= ctx->cfg.max_batch, "fc_promote_pages: batch=%d outside 1..%d", a->batch, ctx->cfg.max_batch);
    FC_REQUIRE(ctx, a->num_pool_blocks >= 2 && a->num_host_blocks >= 1, "fc_promote_pages: pool sizes must be positive");
    FC_REQUIRE(ctx, a->mode == FC_PROMOTE_GATHER || a->mode == FC_PROMOTE_MEMCPY || a->mode == FC_PROMOTE_RIDE, "fc_promote_pages: unknown mode %d", a->mode);

    fc_promote_params p;
    p.new_pages = a->new_pages;
    p.new_count = a->new_count;
    p.resident_pages = a->resident_pages;
    p.resident_count = a->resident_count;
    p.block_table = a->block_table;
    p.host_block_table = a->host_block_table;
    p.free_blocks = a->free_blocks;
    p.free_count = a->free_count;
    p.rerank_mask = a->rerank_mask;
    p.promoted_count = a->promoted_count;
    p.promoted_flags = a->promoted_flags;
    p.batch = a->batch;
    p.Hkv = ctx->cfg.num_kv_heads;
    p.Nmax = ctx->cfg.max_pages_per_seq;
    p.Kmax = ctx->cfg.max_topk;
    p.n_stable = 0;
    memset(p.heads, 0, sizeof p.heads);
    for (int h = 0; h < p.Hkv; ++h)
        if (a->stable_flag[h]) p.heads[p.n_stable++] = (uint8_t)h;
    p.num_pool_blocks = a->num_pool_blocks;
    p.num_host_blocks = a->num_host_blocks;
    p.counters = fc_ws_ptr<int32_t>(ctx, ctx->lay.counters);
    p.publish = a->mode == FC_PROMOTE_MEMCPY;
    p.host_total = a->total_promoted;
    p.list_capacity = ctx->max_items * ctx->cfg.max_topk;
    int32_t *scratch_total = reinterpret_cast<int32_t *>(ctx->scratch);
    p.host_total2 = scratch_total;
    int32_t *scratch_list = reinterpret_cast<int32_t *>(ctx->scratch + 256);
    p.copy_list = a->mode != FC_PROMOTE_MEMCPY ? fc_ws_ptr<int32_t>(ctx, ctx->lay.copy_list) : scratch_list;

    hipStream_t ms = (hipStream_t)main_stream, ss = (hipStream_t)side_stream;
    if (p.n_stable == 0) {
        if (a->total_promoted) *a->total_promoted = 0;
        return FC_OK;
    }
    if (rerank) {
        FC_REQUIRE(ctx, rerank->topk_pages == a->new_pages && rerank->topk_count == a->new_count && rerank->batch == a->batch &&
                            rerank->rerank_mask == a->rerank_mask && rerank->stable_flag &&
                            fc_stable_mask(ctx->cfg, rerank->stable_flag) == fc_stable_mask(ctx->cfg, a->stable_flag),
                   "fc_rerank_promote: the selection's outputs must be the promotion's new_pages / new_count, with the same batch, "
                   "rerank_mask and stable_flag");
    }
    if (ctx->copies_deferred) {     // copies of an earlier FC_PROMOTE_RIDE call that nothing has carried: they go first
        const int st = fc_launch_deferred_copies(ctx, main_stream);
        if (st != FC_OK) return st;
    }
    if (ctx->copies_pending) {
        // copies of an earlier call may still be running on the side stream: this call's bookkeeping
        // must not hand their destination blocks out again before they have landed
        const int st = fc_wait_for_copies(ctx, main_stream);
        if (st != FC_OK) return st;
    }
    const size_t list_bytes = 3 * (size_t)p.Kmax * sizeof(int32_t);
    p.lds_lists = list_bytes <= FC_RECYCLE_MAX_LDS;
    bool fused = false;
    if (rerank) {
        const int st = fc_rerank_launch(ctx, rerank, &p, ms, &fused);
        if (st != FC_OK) return st;
    }
    if (fused)
        ;   // the selection kernel has recycled the blocks
    else if (p.lds_lists)
        hipLaunchKernelGGL(fc_recycle_kernel, dim3(p.n_stable, p.batch), dim3(FC_RECYCLE_THREADS), list_bytes, ms, p);
    else
        hipLaunchKernelGGL(fc_recycle_global_kernel, dim3(p.n_stable, p.batch), dim3(FC_RECYCLE_THREADS), 0, ms, p);
    FC_HIP(ctx, hipGetLastError());
    if (a->mode == FC_PROMOTE_RIDE) {
        // single-stream mode: whatever follows on main_stream is ordered behind the recycle kernel by the stream
        // itself, and an event recorded here would only hold the stream up (a few microseconds)
        ctx->diff_valid = false;
    } else {
        FC_HIP(ctx, hipEventRecord(ctx->ev_diff_done, ms));
        ctx->diff_stream = main_stream;
        ctx->diff_valid = true;
    }

    fc_copy_job job;
    job.copy_list = p.copy_list;
    job.pair_count = p.counters + 2;
    job.ticket = p.counters + 6;
    job.host_total = a->total_promoted;
    job.list_capacity = p.list_capacity;
    job.host_pool = (const uint4 *)a->host_pool;
    job.kv_pool = (uint4 *)a->kv_pool;
    if (a->mode == FC_PROMOTE_RIDE) {
        // nothing is launched here: the next attention launch on main_stream carries the copies
        ctx->deferred = job;
        ctx->copies_deferred = true;
        ctx->copies_stream = main_stream;
        return FC_OK;
    }
    if (a->mode == FC_PROMOTE_GATHER) {
        if (ss != ms) FC_HIP(ctx, hipStreamWaitEvent(ss, ctx->ev_diff_done, 0));
        hipLaunchKernelGGL(fc_gather_pages_kernel, dim3(ctx->gather_blocks), dim3(FC_COPY_THREADS), 0, ss, job);
        FC_HIP(ctx, hipGetLastError());
    } else {
        FC_HIP(ctx, hipEventSynchronize(ctx->ev_diff_done));   // the one host wait: for the copy list
        int total = *scratch_total;
        if (total > p.list_capacity) total = p.list_capacity;
        const char *hp = (const char *)a->host_pool;
        char *kp = (char *)a->kv_pool;
        for (int i = 0; i < total; ++i) {
            const long long src = scratch_list[2 * i], dst = scratch_list[2 * i + 1];
            if (dst <= 0) continue;
            FC_HIP(ctx, hipMemcpyAsync(kp + dst * FC_PAGE_BYTES, hp + src * FC_PAGE_BYTES, FC_PAGE_BYTES, hipMemcpyHostToDevice, ss));
        }
    }
    // in-line copies are followed by the caller's next work on the same stream anyway; an event behind them
    // would only hold that work up (a few microseconds per record), so it is recorded when another stream asks
    ctx->copies_recorded = ss != ms;
    if (ctx->copies_recorded) FC_HIP(ctx, hipEventRecord(ctx->ev_copies_done, ss));
    ctx->copies_pending = true;
    ctx->copies_stream = side_stream;
    return FC_OK;
}

extern "C" int fc_promote_pages(fc_ctx *ctx, const fc_promote_args *a, void *main_stream, void *side_stream)
{
    if (!ctx) return FC_ERR_INVALID_ARG;
    return fc_promote_impl(ctx, a, main_stream, side_stream, nullptr);
}

extern "C" int fc_rerank_promote(fc_ctx *ctx, const fc_rerank_args *rerank, const fc_promote_args *promote, void *main_stream,
                                 void *side_stream)
{
    if (!ctx) return FC_ERR_INVALID_ARG;
    FC_REQUIRE(ctx, rerank, "fc_rerank_promote: rerank args is NULL");
    return fc_promote_impl(ctx, promote, main_stream, side_stream, rerank);
}
