// fc_append_kv: the per-step KV append of decoding (Sec. 2 of the paper: one new K/V pair per step),
// with the MinMax row of the touched page kept current (Sec. 3.2) and the one-time offload of a stable
// head's page at the moment it fills (Sec. 3.3 "Minimizing Transfer Size": each page of a stable head is
// offloaded exactly once; the partially filled last page stays resident because it is being appended to).
// fc_offload_pages: the bulk HBM -> pinned host copy used after prefill (Sec. 3.3), the mirror image of
// the promotion gather: a capped number of workgroups write pinned host memory directly.
#include "fc_internal.h"

struct fc_append_params {
    const uint16_t *k_new;       // [batch][Hkv][D]
    const uint16_t *v_new;
    const uint8_t *append_mask;  // [batch] or NULL
    int32_t *context_lens;       // in/out
    int32_t *block_table;
    const int32_t *host_block_table;
    int32_t *free_blocks;
    int32_t *free_count;
    int32_t *resident_pages;
    int32_t *resident_count;
    uint16_t *minmax;
    uint16_t *pool;
    uint16_t *host_pool;
    long long num_pool_blocks, num_host_blocks;
    unsigned long long stable_mask;
    int batch, Hkv, Nmax, Kmax;
    int32_t *counters;           // [1] = error bits, [5] = workgroups done
    int32_t *seq_flags;          // [batch]: set when a head of the sequence could not take its token; cleared by the last workgroup
};

__global__ __launch_bounds__(128) void fc_append_kernel(fc_append_params p)
{
    __shared__ long long sh_blk;
    const int h = blockIdx.x, b = blockIdx.y, d = threadIdx.x;
    const size_t item = (size_t)b * p.Hkv + h;
    const bool active = !p.append_mask || p.append_mask[b];
    int err = 0;
    bool failed = false;      // this head could not take the token (no room in the tables, no block)
    if (active) {
        const int pos = p.context_lens[b];
        const int page = pos >> 4, slot = pos & 15;
        const bool stable = (p.stable_mask >> h) & 1ull;
        if (pos < 0 || page >= p.Nmax) {
            err = FC_DEV_ERR_CLAMPED;              // no room in the tables: nothing is written
            failed = true;
        } else {
            int32_t *tbl = p.block_table + item * (size_t)p.Nmax;
            if (d == 0) {
                long long blk = 0;
                if (slot == 0) {                   // a new page starts: it takes the last block of the free list
                    const int nf = p.free_count[item];
                    if (nf >= 1 && nf <= p.Kmax) {
                        blk = p.free_blocks[item * (size_t)p.Kmax + nf - 1];
                        p.free_count[item] = nf - 1;
                        tbl[page] = (int32_t)blk;
                        if (stable) {              // and joins the head's resident list (it is the highest page id)
                            const int cnt = p.resident_count[item];
                            if (cnt >= 0 && cnt < p.Kmax) {
                                p.resident_pages[item * (size_t)p.Kmax + cnt] = page;
                                p.resident_count[item] = cnt + 1;
                            } else {
                                err |= FC_DEV_ERR_FREE_OVERFLOW;
                            }
                        }
                    } else {
                        err |= FC_DEV_ERR_NO_BLOCK;
                    }
                } else {
                    blk = tbl[page];
                }
                if (blk < 1 || blk >= p.num_pool_blocks) { blk = 0; err |= FC_DEV_ERR_CLAMPED; }
                sh_blk = blk;
            }
            __syncthreads();
            const long long blk = sh_blk;
            failed = blk <= 0;
            if (blk > 0) {
                uint16_t *pg = p.pool + (size_t)blk * FC_PAGE_ELEMS;
                const uint16_t kx = p.k_new[item * FC_D + d], vx = p.v_new[item * FC_D + d];
                pg[fc_k_elem(slot, d)] = kx;                   // K half, 32-dim chunks of token rows
                pg[FC_P * FC_D + d * FC_P + slot] = vx;        // V half, dim-major
                uint16_t *row = p.minmax + (item * (size_t)p.Nmax + page) * (2 * FC_D);
                if (slot == 0) {
                    row[d] = kx;
                    row[FC_D + d] = kx;
                } else {
                    const float f = __uint_as_float((uint32_t)kx << 16);
                    if (f < __uint_as_float((uint32_t)row[d] << 16)) row[d] = kx;
                    if (f > __uint_as_float((uint32_t)row[FC_D + d] << 16)) row[FC_D + d] = kx;
                }
                if (stable && slot == FC_P - 1) {              // the page is full: its one offload to the host copy
                    const long long hb = p.host_block_table[item * (size_t)p.Nmax + page];
                    if (hb >= 1 && hb < p.num_host_blocks) {
                        __threadfence_block();
                        __syncthreads();
                        const uint4 *src = reinterpret_cast<const uint4 *>(pg);
                        uint4 *dst = reinterpret_cast<uint4 *>(p.host_pool + (size_t)hb * FC_PAGE_ELEMS);
                        for (int i = d; i < FC_PAGE_BYTES / 16; i += 128) dst[i] = src[i];
                    } else {
                        err |= FC_DEV_ERR_CLAMPED;
                    }
                }
            }
        }
    }
    if (err && d == 0) atomicOr(&p.counters[1], err);
    if (failed && d == 0) atomicOr(&p.seq_flags[b], 1);
    // every workgroup has read the old lengths by now; the last one to finish advances them
    __syncthreads();
    if (d == 0) {
        __threadfence();
        sh_blk = atomicAdd(&p.counters[5], 1) == (int)(gridDim.x * gridDim.y) - 1;
    }
    __syncthreads();
    if (sh_blk) {
        for (int i = d; i < p.batch; i += 128) {
            const int pos = p.context_lens[i];
            // a sequence one of whose heads could not take the token keeps its length: no head is left with a
            // token position that has no block behind it
            const int failed = atomicExch(&p.seq_flags[i], 0);
            if ((!p.append_mask || p.append_mask[i]) && !failed && pos >= 0 && (pos >> 4) < p.Nmax) p.context_lens[i] = pos + 1;
        }
        if (d == 0) p.counters[5] = 0;
    }
}

__global__ __launch_bounds__(256) void fc_offload_pages_kernel(const int32_t *__restrict__ pairs, int n_pairs,
                                                               const uint4 *__restrict__ kv_pool, long long num_pool_blocks,
                                                               uint4 *__restrict__ host_pool, long long num_host_blocks)
{
    constexpr int V = FC_PAGE_BYTES / 16;
    for (int i = blockIdx.x; i < n_pairs; i += gridDim.x) {
        const long long src = pairs[2 * (size_t)i], dst = pairs[2 * (size_t)i + 1];
        if (src < 1 || src >= num_pool_blocks || dst < 1 || dst >= num_host_blocks) continue;
        const uint4 *s = kv_pool + src * V;
        uint4 *d = host_pool + dst * V;
        const uint4 x0 = s[threadIdx.x], x1 = s[threadIdx.x + 256];
        d[threadIdx.x] = x0;
        d[threadIdx.x + 256] = x1;
    }
}

extern "C" int fc_append_kv(fc_ctx *ctx, const fc_append_args *a, void *stream)
{
    if (!ctx) return FC_ERR_INVALID_ARG;
    FC_REQUIRE(ctx, a, "fc_append_kv: args is NULL");
    FC_REQUIRE(ctx, a->k_new && a->v_new && a->context_lens && a->block_table && a->free_blocks && a->free_count &&
                        a->minmax && a->kv_pool && a->stable_flag,
               "fc_append_kv: NULL pointer among the required arguments");
    FC_REQUIRE(ctx, a->batch >= 1 && a->batch <= ctx->cfg.max_batch, "fc_append_kv: batch=%d outside 1..%d", a->batch, ctx->cfg.max_batch);
    FC_REQUIRE(ctx, a->num_pool_blocks >= 2, "fc_append_kv: num_pool_blocks must be >= 2");
    const uint64_t mask = fc_stable_mask(ctx->cfg, a->stable_flag);
    FC_REQUIRE(ctx, mask == 0 || (a->resident_pages && a->resident_count && a->host_block_table && a->host_pool && a->num_host_blocks >= 2),
               "fc_append_kv: stable heads need resident_pages, resident_count, host_block_table and host_pool");
    fc_append_params p;
    p.k_new = (const uint16_t *)a->k_new;
    p.v_new = (const uint16_t *)a->v_new;
    p.append_mask = a->append_mask;
    p.context_lens = a->context_lens;
    p.block_table = a->block_table;
    p.host_block_table = a->host_block_table;
    p.free_blocks = a->free_blocks;
    p.free_count = a->free_count;
    p.resident_pages = a->resident_pages;
    p.resident_count = a->resident_count;
    p.minmax = (uint16_t *)a->minmax;
    p.pool = (uint16_t *)a->kv_pool;
    p.host_pool = (uint16_t *)a->host_pool;
    p.num_pool_blocks = a->num_pool_blocks;
    p.num_host_blocks = a->num_host_blocks;
    p.stable_mask = mask;
    p.batch = a->batch;
    p.Hkv = ctx->cfg.num_kv_heads;
    p.Nmax = ctx->cfg.max_pages_per_seq;
    p.Kmax = ctx->cfg.max_topk;
    p.counters = fc_ws_ptr<int32_t>(ctx, ctx->lay.counters);
    p.seq_flags = fc_ws_ptr<int32_t>(ctx, ctx->lay.seq_flags);
    // page copies of an earlier fc_promote_pages may still be on their way into the pool (the partially filled last
    // page of a stable head among them): they land before this call writes the pool
    FC_REQUIRE(ctx, !ctx->copies_deferred || stream == ctx->copies_stream,
               "fc_append_kv: after FC_PROMOTE_RIDE the next call that touches the pool belongs on fc_promote_pages' main_stream");
    {
        int st = fc_launch_deferred_copies(ctx, stream);
        if (st == FC_OK) st = fc_wait_for_copies(ctx, stream);
        if (st != FC_OK) return st;
    }
    hipLaunchKernelGGL(fc_append_kernel, dim3(p.Hkv, p.batch), dim3(128), 0, (hipStream_t)stream, p);
    FC_HIP(ctx, hipGetLastError());
    return FC_OK;
}

extern "C" int fc_offload_pages(fc_ctx *ctx, const void *kv_pool, int64_t num_pool_blocks, void *host_pool,
                                int64_t num_host_blocks, const int32_t *pairs, int32_t n_pairs, void *stream)
{
    if (!ctx) return FC_ERR_INVALID_ARG;
    FC_REQUIRE(ctx, kv_pool && host_pool && (pairs || n_pairs == 0), "fc_offload_pages: NULL pointer");
    FC_REQUIRE(ctx, n_pairs >= 0 && num_pool_blocks >= 2 && num_host_blocks >= 2, "fc_offload_pages: sizes out of range");
    if (n_pairs == 0) return FC_OK;
    FC_REQUIRE(ctx, !ctx->copies_deferred || stream == ctx->copies_stream,
               "fc_offload_pages: after FC_PROMOTE_RIDE the next call that touches the pool belongs on fc_promote_pages' main_stream");
    {   // pages being promoted into the pool land before the pool is read
        int st = fc_launch_deferred_copies(ctx, stream);
        if (st == FC_OK) st = fc_wait_for_copies(ctx, stream);
        if (st != FC_OK) return st;
    }
    const int grid = n_pairs < ctx->gather_blocks ? n_pairs : ctx->gather_blocks;
    hipLaunchKernelGGL(fc_offload_pages_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, pairs, n_pairs,
                       (const uint4 *)kv_pool, (long long)num_pool_blocks, (uint4 *)host_pool, (long long)num_host_blocks);
    FC_HIP(ctx, hipGetLastError());
    return FC_OK;
}
