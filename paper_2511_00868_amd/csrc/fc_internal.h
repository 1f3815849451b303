// Internal declarations shared by the translation units of libflexicache (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "flexicache.h"

constexpr int FC_D = 128;          // head_dim
constexpr int FC_P = 16;           // tokens per page
constexpr int FC_PAGE_ELEMS = 2 * FC_P * FC_D;        // bf16 elements per block (K half + V half)
constexpr int FC_PAGE_BYTES = FC_PAGE_ELEMS * 2;      // 8192
constexpr int FC_HALF_BYTES = FC_PAGE_BYTES / 2;      // 4096

// Element index of K[token t][dim d] inside the K half of a block: four 1 KiB chunks of 32 dims each,
// inside a chunk one 64-byte row per token.  One matrix-core operand load of the attention kernel
// (16 tokens x 32 dims) is then one contiguous 1 KiB read, and every 128-byte line is requested once.
__host__ __device__ __forceinline__ int fc_k_elem(int t, int d) { return (d >> 5) * (FC_P * 32) + t * 32 + (d & 31); }
constexpr int FC_MM_ROW_BYTES = 2 * FC_D * 2;         // MinMax bytes per page (512)
constexpr int FC_MAX_PROFILE_EVENTS = 1024;
constexpr int FC_MAX_ITEMS = 4096;                   // max_batch * num_kv_heads (schedule lives in LDS)

// Device-side error bits (workspace word `err`).
constexpr int FC_DEV_ERR_NO_BLOCK = 1;     // a head owned too few blocks for its promoted pages
constexpr int FC_DEV_ERR_CLAMPED = 2;      // an id outside its valid range was clamped
constexpr int FC_DEV_ERR_FREE_OVERFLOW = 4;
constexpr int FC_DEV_ERR_NOT_RESIDENT = 8; // attention was asked to read a page whose table entry is the null block

// Partition of the caller's device workspace.
struct fc_ws_layout {
    size_t scores;        // float [max_batch][Hkv][Nmax]
    size_t seg_start;     // int32 [2][max_items + 2]: schedules handed from the attention to the merge kernel
    size_t part_ml;       // float [2][slots][16][2]  (running max in log2 units, running sum)
    size_t part_acc;      // float [2][slots][G][128]
    size_t copy_list;     // int32 [max_items * Kmax][2]
    size_t counters;      // int32 [8]: 1 = err, 2 = copy-pair count, 4 = recycle workgroups done, 5 = append workgroups done, 6 = copier workgroups done
    size_t seq_flags;     // int32 [max_batch]: fc_append_kv: a head of this sequence could not take its token (cleared by the same call)
    size_t total;
};

// Page copies that fc_promote_pages left for the next attention launch (FC_PROMOTE_RIDE).
struct fc_copy_job {
    const int32_t *copy_list;    // pairs (host block, pool block)
    int32_t *pair_count;         // device counter the recycle kernel appended to; cleared by the copier's last workgroup
    int32_t *ticket;             // device counter of copier workgroups that are done
    int32_t *host_total;         // pinned, may be NULL: receives the pair count
    int list_capacity;
    const uint4 *host_pool;
    uint4 *kv_pool;
};

// One workgroup's share of the page copies: workgroup `wg` of `n_wg`, one wavefront; each 8 KiB page (512 x 16 B)
// is pulled straight out of pinned host memory in two rounds of four 16 B loads in flight per lane.
constexpr int FC_COPY_THREADS = 64;
constexpr int FC_COPY_UNROLL = 4;
__device__ __forceinline__ void fc_copy_pages(const fc_copy_job &c, int wg, int n_wg, int tid)
{
    constexpr int V = FC_PAGE_BYTES / 16;   // 512 x 16 B per page
    static_assert(V % (FC_COPY_UNROLL * FC_COPY_THREADS) == 0, "a page must be a whole number of copy rounds");
    int total = c.pair_count[0];
    if (wg == 0 && tid == 0 && c.host_total) *c.host_total = total;
    total = total > c.list_capacity ? c.list_capacity : total;
    for (int i = wg; i < total; i += n_wg) {
        const long long src = c.copy_list[2 * (size_t)i], dst = c.copy_list[2 * (size_t)i + 1];
        if (dst <= 0) continue;
        const uint4 *s = c.host_pool + src * V;
        uint4 *d = c.kv_pool + dst * V;
        for (int k = tid; k < V; k += FC_COPY_UNROLL * FC_COPY_THREADS) {
            uint4 x[FC_COPY_UNROLL];
#pragma unroll
            for (int u = 0; u < FC_COPY_UNROLL; ++u) x[u] = s[k + u * FC_COPY_THREADS];
#pragma unroll
            for (int u = 0; u < FC_COPY_UNROLL; ++u) d[k + u * FC_COPY_THREADS] = x[u];
        }
    }
    // The count has to be zero again before the next recycling kernel adds to it, and it may not change while
    // another copying workgroup has still to read it: the workgroup that finishes last clears it (every workgroup
    // has read it by then).  Nothing here depends on host-side state, so a captured launch can be replayed.
    if (tid == 0) {
        if (atomicAdd(c.ticket, 1) == n_wg - 1) {
            *c.pair_count = 0;
            *c.ticket = 0;
        }
    }
}

struct fc_ctx {
    fc_config cfg;
    int G;
    int max_items;
    int attn_waves;
    int slots;
    int num_cus;
    float scale_log2;     // softmax scale times log2(e)
    char *ws;
    size_t ws_bytes;
    char *scratch;        // pinned host scratch
    size_t scratch_bytes;
    fc_ws_layout lay;
    hipEvent_t ev_diff_done;
    hipEvent_t ev_copies_done;
    hipEvent_t ev_first_done;   // the first attention call of a pair has been enqueued up to here
    void *diff_stream;          // stream of the last block-recycling kernel (ev_diff_done), if diff_valid
    bool diff_valid;
    void *first_stream;         // stream of the pending first call of a pair
    void *copies_stream;        // stream the pending page copies were enqueued on
    bool copies_deferred;       // FC_PROMOTE_RIDE: the copies of the last fc_promote_pages have not been launched yet
    fc_copy_job deferred;
    bool copies_recorded;       // ev_copies_done has been recorded behind them (not done for in-line copies until another stream asks)
    bool copies_pending;
    int pending_pair;        // FC_HEADS_UNSTABLE or FC_PAGES_RESIDENT has left partials for its partner call to merge, else 0
    int gather_blocks;    // workgroups of the host->HBM gather kernel (few and small: see fc_promote.hip)
    int ride_blocks;      // copying workgroups added to an attention launch (FC_PROMOTE_RIDE)
    // kernel timing
    bool profiling;
    int prof_used;
    int prof_stride, prof_seen;
    double prof_empty_ms;
    hipEvent_t *prof_ev;  // 2 * FC_MAX_PROFILE_EVENTS events, created by the first fc_profile_begin (benchmarks only)
    char err[512];
};

int fc_fail(fc_ctx *ctx, int status, const char *fmt, ...);
int fc_check_config(const fc_config *c, const char **why);   // FC_OK, or a status with a static text in *why
int fc_resolve_waves(const fc_config *cfg, int num_cus);     // wavefronts of the attention kernel (a multiple of 4)
int fc_launch_deferred_copies(fc_ctx *ctx, void *stream);
int fc_wait_for_copies(fc_ctx *ctx, void *stream);
int fc_hip_fail(fc_ctx *ctx, hipError_t e, const char *what);
uint64_t fc_stable_mask(const fc_config &cfg, const uint8_t *stable_flag);

#define FC_HIP(ctx, call)                                          \
    do {                                                           \
        hipError_t e_ = (call);                                    \
        if (e_ != hipSuccess) return fc_hip_fail((ctx), e_, #call); \
    } while (0)

#define FC_REQUIRE(ctx, cond, ...)                                          \
    do {                                                                    \
        if (!(cond)) return fc_fail((ctx), FC_ERR_INVALID_ARG, __VA_ARGS__); \
    } while (0)

template <typename T>
static inline T *fc_ws_ptr(const fc_ctx *ctx, size_t off)
{
    return reinterpret_cast<T *>(ctx->ws + off);
}

static inline size_t fc_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
