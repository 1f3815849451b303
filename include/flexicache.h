/*
 * flexicache.h -- C ABI of the MI355X (gfx950) decode hot path of FlexiCache (arXiv 2511.00868).
 *
 * One attention layer, one GPU.  Every KV head of every sequence has its own page set:
 *   - unstable heads attend over all of their pages, which all live in HBM;
 *   - stable heads attend over their top-K pages only, and only those live in HBM; the full copy
 *     of a stable head lives in pinned host memory (Sec. 3.1, 3.3 of the paper).
 * Every `rerank interval` steps the caller calls fc_rerank_topk (page scores from the MinMax cache,
 * Sec. 3.2, then per-head top-K) and fc_promote_pages (set difference, physical block recycling,
 * null block, host->HBM copies of the newly selected pages; Sec. 3.3, 3.4); every step it calls
 * fc_sparse_decode_attn (split-KV decode attention restricted to each head's page set).
 *
 * Conventions
 *   - "dev" pointers are device memory of `fc_config.device`; "host" pointers are ordinary host
 *     memory read during the call; "pinned" pointers are page-locked host memory that the GPU can
 *     address (hipHostMalloc / torch pin_memory).  The library never allocates or frees device or
 *     pinned memory: all of it, including the workspace, is owned by the caller and must stay
 *     valid until the work enqueued on it has finished.  The library owns only HIP events
 *     (three for ordering streams, plus those of fc_profile_begin).
 *   - Streams are hipStream_t passed as void*; NULL is the default stream.  All calls enqueue work
 *     and return; only FC_PROMOTE_MEMCPY makes the host wait (for the small copy list).
 *   - Every function returns FC_OK (0) or a negative fc_status; fc_last_error gives the text.
 *     Argument errors are detected on the host before anything is launched.
 *   - One host thread per fc_ctx at a time.
 *   - bf16 = IEEE bfloat16 bit patterns (uint16_t).  head_dim D = 128, page_size P = 16 tokens,
 *     group G = num_q_heads / num_kv_heads in {1, 2, 4, 8, 16}.
 *
 * Memory layouts fixed by this ABI (Nmax = max_pages_per_seq, Kmax = max_topk)
 *   q            bf16 [batch][num_q_heads][D]; query head hq belongs to KV head hq / G
 *   kv_pool      bf16 [num_blocks][2][2048]: one physical block = one page of one KV head = 8 KiB,
 *                first the K half in four 1 KiB chunks of 32 dims: K[chunk 0..3][token 0..15][dim 32*chunk + 0..31],
 *                then the V half, dim-major:               V[dim 0..127][token 0..15]
 *                (fc_write_kv_pages produces this layout; nothing else needs to know it).
 *                Block 0 is the null block (Sec. 3.4 "Uniformity Through Null Block"): it is never
 *                assigned to a page and its contents are never used.
 *   host_pool    same block layout, in pinned host memory.
 *   block_table  int32 [batch][num_kv_heads][Nmax]: logical page -> physical block, 0 = not in HBM
 *   host_block_table  int32, same shape: logical page -> block of host_pool
 *   minmax       bf16 [batch][num_kv_heads][Nmax][2][D]: row 0 per-dim minimum key of the page,
 *                row 1 per-dim maximum (the MinMax cache of Sec. 3.2), over valid tokens only
 *   topk_pages   int32 [batch][num_kv_heads][Kmax]: ascending logical page ids, -1 padded
 *   topk_count   int32 [batch][num_kv_heads]
 *   context_lens int32 [batch]: tokens in the sequence; pages = ceil(len / 16) <= Nmax.  0 (or less) is an idle
 *                slot: no pages, an empty top-K list, nothing promoted, output rows 0 and lse = -inf
 *   stable_flag  uint8 [num_kv_heads] on the HOST: 1 = stable head (profiled offline, Sec. 2.3).  For
 *                fc_rerank_topk it names the heads to rescore; for fc_sparse_decode_attn the heads that
 *                attend over their list instead of over all pages (the paper's own variant, in which the
 *                unstable heads also attend over a top-K list that is rescored every step, sets it for
 *                every head there and calls fc_rerank_topk for the unstable heads at every step)
 */
#ifndef FLEXICACHE_H
#define FLEXICACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fc_ctx fc_ctx;

typedef enum {
    FC_OK = 0,
    FC_ERR_INVALID_ARG = -1,  /* null pointer, size out of range, inconsistent shapes */
    FC_ERR_UNSUPPORTED = -2,  /* head_dim != 128, page_size != 16, unsupported group size */
    FC_ERR_WORKSPACE = -3,    /* workspace or pinned scratch too small or misaligned */
    FC_ERR_HIP = -4,          /* a HIP call failed; text in fc_last_error */
    FC_ERR_STATE = -5         /* the device-side bookkeeping reported an inconsistency */
} fc_status;

typedef struct {
    int32_t num_q_heads;
    int32_t num_kv_heads;      /* <= 64 */
    int32_t head_dim;          /* 128 */
    int32_t page_size;         /* 16 */
    int32_t max_batch;
    int32_t max_pages_per_seq; /* Nmax */
    int32_t max_topk;          /* Kmax */
    float softmax_scale;       /* 0 -> 1/sqrt(head_dim) */
    int32_t device;            /* HIP device ordinal */
    int32_t attn_waves;        /* 0 -> chosen from the device (wavefronts the attention kernel runs) */
    int32_t copy_workgroups;   /* 0 -> library default; single-wavefront workgroups that pull promoted pages out of
                                  pinned host memory (32 as a kernel of their own, 40 riding in an attention launch) */
} fc_config;

/* Bytes of device workspace / pinned host scratch a context of this shape needs (0 on bad config). */
size_t fc_workspace_bytes(const fc_config *cfg);
size_t fc_host_scratch_bytes(const fc_config *cfg);

/* Creates a context on cfg->device over caller-owned memory: `dev_workspace` (256-byte aligned,
 * >= fc_workspace_bytes) and `pinned_scratch` (>= fc_host_scratch_bytes, GPU addressable).
 * No device or pinned memory is allocated here or anywhere else in the library. */
int fc_create(fc_ctx **out, const fc_config *cfg, void *dev_workspace, size_t workspace_bytes,
              void *pinned_scratch, size_t scratch_bytes);
int fc_destroy(fc_ctx *ctx);
const char *fc_status_string(int status);
const char *fc_last_error(const fc_ctx *ctx);

/* ---- support: page writer and MinMax builder -------------------------------------------------- */

/* Scatters token-major keys/values of one sequence into pool blocks in the kv_pool layout (the
 * paged-cache write every paged-attention system has; Sec. 2 of the paper).
 *   k_src, v_src  dev bf16 [num_kv_heads][tokens][D], tokens = n_pages * 16 (pad rows are copied
 *                 as they are; consumers mask them by context length)
 *   block_ids     dev int32 [num_kv_heads][ids_stride]: destination block of (head, page), pages
 *                 0..n_pages-1; an id of 0 skips that page
 *   pool          dev or pinned, `num_blocks` blocks. */
int fc_write_kv_pages(fc_ctx *ctx, const void *k_src, const void *v_src, int32_t n_pages,
                      const int32_t *block_ids, int32_t ids_stride, void *pool, int64_t num_blocks,
                      void *stream);

/* Builds MinMax rows (Sec. 3.2) of one sequence from pages resident in `pool`.
 *   block_ids   dev int32 [num_kv_heads][ids_stride], as above (0 = skip)
 *   page_list   dev int32 [n_list] logical pages to (re)build, or NULL for 0..n_pages-1 with
 *               n_list = n_pages
 *   context_len tokens in the sequence (host value): only valid tokens take part
 *   minmax_seq  dev bf16 [num_kv_heads][Nmax][2][D] of this sequence. */
int fc_build_minmax(fc_ctx *ctx, const void *pool, int64_t num_blocks, const int32_t *block_ids,
                    int32_t ids_stride, const int32_t *page_list, int32_t n_list, int32_t context_len,
                    void *minmax_seq, void *stream);

/* ---- hot path ---------------------------------------------------------------------------------- */

/* Page scoring + per-head top-K (Sec. 3.2; selection of Sec. 3.1).  For every sequence b with
 * rerank_mask[b] != 0 and every stable head h:
 *   score[p] = max over the G queries of the group of sum_i max(q_i * kmin[p][i], q_i * kmax[p][i])
 *   (fp32 accumulation of exact bf16 products; the paper gives the per-query sum, the maximum over
 *   the group is this library's reading), for p < ceil(context_len / 16);
 *   selected = min(k_per_seq[b], pages) pages: the last page if it is partially filled (Sec. 3.3),
 *   then the highest scores, ties to the lower page index; written ascending, -1 padded.
 * Sequences with rerank_mask[b] == 0 and unstable heads keep their previous lists untouched. */
typedef struct {
    const void *q;               /* dev bf16 [batch][num_q_heads][D] */
    const void *minmax;          /* dev bf16 [batch][num_kv_heads][Nmax][2][D] */
    const int32_t *context_lens; /* dev [batch] */
    const uint8_t *stable_flag;  /* host [num_kv_heads] */
    const int32_t *k_per_seq;    /* dev [batch], 1 <= K_b <= Kmax */
    const uint8_t *rerank_mask;  /* dev [batch] or NULL (= all sequences rerank) */
    int32_t batch;               /* <= max_batch */
    int32_t *topk_pages;         /* dev out [batch][num_kv_heads][Kmax] */
    int32_t *topk_count;         /* dev out [batch][num_kv_heads] */
    float *scores_out;           /* dev out [batch][num_kv_heads][Nmax] or NULL (workspace is used) */
} fc_rerank_args;
int fc_rerank_topk(fc_ctx *ctx, const fc_rerank_args *args, void *stream);

/* Promotion (Sec. 3.3 "Minimizing Transfer Size", Sec. 3.4 "Physical Block Reuse During Reranking"
 * and "Uniformity Through Null Block").  For every reranking sequence and stable head:
 *   evicted = resident \ new, promoted = new \ resident.  The head's available blocks are its free
 *   list followed by the blocks of the evicted pages in ascending page order; promoted pages, in
 *   ascending page order, take them from the front; the rest is the new free list.  Evicted entries
 *   of block_table become 0, promoted entries get their block, resident_* becomes new_*.
 *   Each promoted page is then copied host_pool[host_block_table[..]] -> kv_pool[block] on
 *   `side_stream`, ordered after the bookkeeping kernel on `main_stream`; the next
 *   fc_sparse_decode_attn on this context that reads stable heads' pages waits (on the GPU) for those
 *   copies, whatever stream it runs on.  side_stream may be the same stream as main_stream: the
 *   copies then follow the bookkeeping kernel in line, with no event between them, which is the
 *   shortest path to the promoted pages; work that should hide the copies then goes to another
 *   stream (see head_subset of fc_sparse_decode_attn).
 * mode FC_PROMOTE_GATHER: one kernel on side_stream reads pinned host memory directly; the host
 *   never waits.  mode FC_PROMOTE_MEMCPY: the host waits for the copy list, then issues one
 *   hipMemcpyAsync per page on side_stream.  mode FC_PROMOTE_RIDE: single-stream operation; this call
 *   launches the bookkeeping kernel only, and the copies ride in the next fc_sparse_decode_attn launch on
 *   main_stream (side_stream is ignored): a FC_PAGES_RESIDENT or FC_HEADS_UNSTABLE call carries them in
 *   extra workgroups of its own launch, so that they run side by side with that attention and the second
 *   call of the pair follows in stream order, with no event anywhere; before any other kind of call they
 *   are launched on their own.  That next attention call must be given main_stream. */
enum { FC_PROMOTE_GATHER = 0, FC_PROMOTE_MEMCPY = 1, FC_PROMOTE_RIDE = 2 };
typedef struct {
    const int32_t *new_pages;        /* dev [batch][num_kv_heads][Kmax] (S_t) */
    const int32_t *new_count;        /* dev [batch][num_kv_heads] */
    int32_t *resident_pages;         /* dev in/out: S_{t-1} on entry, S_t afterwards */
    int32_t *resident_count;         /* dev in/out */
    int32_t *block_table;            /* dev in/out [batch][num_kv_heads][Nmax] */
    const int32_t *host_block_table; /* dev [batch][num_kv_heads][Nmax] */
    int32_t *free_blocks;            /* dev in/out [batch][num_kv_heads][Kmax] */
    int32_t *free_count;             /* dev in/out [batch][num_kv_heads] */
    const uint8_t *stable_flag;      /* host [num_kv_heads] */
    const uint8_t *rerank_mask;      /* dev [batch] or NULL */
    void *kv_pool;                   /* dev */
    int64_t num_pool_blocks;
    const void *host_pool;           /* pinned */
    int64_t num_host_blocks;
    int32_t batch;
    int32_t mode;                    /* FC_PROMOTE_GATHER | FC_PROMOTE_MEMCPY | FC_PROMOTE_RIDE */
    int32_t *promoted_count;         /* dev out [batch][num_kv_heads] or NULL (0 for heads not touched) */
    uint8_t *promoted_flags;         /* dev out [batch][num_kv_heads][Kmax] or NULL: 1 where resident_pages[..][i]
                                        was promoted by this call (all 0 for sequences that did not rerank) */
    int32_t *total_promoted;         /* pinned out (one int32) or NULL: pages copied by this call; valid once
                                        the copies have finished (side_stream for GATHER; the attention launch
                                        that carried them for RIDE; at return for MEMCPY) */
} fc_promote_args;
int fc_promote_pages(fc_ctx *ctx, const fc_promote_args *args, void *main_stream, void *side_stream);

/* fc_rerank_topk followed by fc_promote_pages as one call, with the same results bit for bit.  Up to 8192 pages per
 * sequence and a page budget (max_topk) of up to 12288 the selection of a head and the recycling of its blocks then run in one
 * kernel (the fused recycling kernel of Sec. 3.4 "Physical Block Reuse During Reranking"), which takes two launches
 * and one trip of the new lists through memory off the path to the page copies; other shapes run the same kernels
 * as the two separate calls.  rerank->topk_pages / topk_count must be promote->new_pages / new_count, and batch,
 * rerank_mask and stable_flag must agree; everything else as documented for the two calls. */
int fc_rerank_promote(fc_ctx *ctx, const fc_rerank_args *rerank, const fc_promote_args *promote, void *main_stream,
                      void *side_stream);

/* Head-heterogeneous paged decode attention (Sec. 3.1; split-KV decode attention as in Sec. 4.1).
 * For every sequence b and KV head h the page set is topk_pages[b][h][0..topk_count) if the head is
 * stable, all pages 0..ceil(context_len/16)-1 otherwise; each of the G query heads of the group gets
 *   out = softmax(scale * q . K_set^T) V_set   over tokens < context_len, fp32,
 *   lse = natural-log-sum-exp of the scaled logits (optional).
 * Every page of the set must be resident (block_table entry != 0).
 * head_subset splits one attention pass in two so that a caller that has just promoted pages can
 * overlap the copies with compute (Sec. 3.3 "Overlapping Transfer with Compute").  Two ways to split:
 *   by page   FC_PAGES_RESIDENT attends over every head, leaving out the list entries that
 *             promoted_flags marks as promoted by the last fc_promote_pages; it does not wait for the
 *             copies.  FC_PAGES_PROMOTED then waits (on the GPU) for the copies, attends over exactly
 *             those entries and writes all output rows.  Works for any mix of heads, all-stable included.
 *   by head   FC_HEADS_UNSTABLE attends over the unstable heads only (no wait); FC_HEADS_STABLE waits for
 *             the copies, attends over the stable heads and writes the output rows of both classes (of
 *             the stable heads only, if no FC_HEADS_UNSTABLE call preceded it on this context).
 * The output rows are complete only after the second call of a pair.  FC_HEADS_ALL: everything in one pass.
 * The two calls of a pair may be given different streams: the library orders the first call after the
 * last fc_promote_pages bookkeeping kernel (whose tables and flags it reads) and the merge of the
 * second call after the first call.  Any other ordering between different streams is the caller's:
 * in particular a call on another stream than the previous attention call's must not start before
 * that call has finished (both use the context's workspace). */
enum { FC_HEADS_ALL = 0, FC_HEADS_UNSTABLE = 1, FC_HEADS_STABLE = 2, FC_PAGES_RESIDENT = 3, FC_PAGES_PROMOTED = 4 };
typedef struct {
    const void *q;               /* dev bf16 [batch][num_q_heads][D] */
    const void *kv_pool;         /* dev */
    int64_t num_pool_blocks;
    const int32_t *block_table;  /* dev [batch][num_kv_heads][Nmax] */
    const int32_t *context_lens; /* dev [batch] */
    const uint8_t *stable_flag;  /* host [num_kv_heads] */
    const int32_t *topk_pages;   /* dev [batch][num_kv_heads][Kmax] */
    const int32_t *topk_count;   /* dev [batch][num_kv_heads] */
    int32_t batch;
    float *out;                  /* dev out fp32 [batch][num_q_heads][D] */
    float *lse;                  /* dev out fp32 [batch][num_q_heads] or NULL */
    int32_t head_subset;         /* FC_HEADS_ALL | FC_HEADS_UNSTABLE | FC_HEADS_STABLE | FC_PAGES_RESIDENT | FC_PAGES_PROMOTED */
    const uint8_t *promoted_flags; /* dev [batch][num_kv_heads][Kmax], as written by fc_promote_pages; needed by
                                      FC_PAGES_RESIDENT / FC_PAGES_PROMOTED, else may be NULL */
} fc_attn_args;
int fc_sparse_decode_attn(fc_ctx *ctx, const fc_attn_args *args, void *stream);

/* For callers that cannot allocate device memory at all -- code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc: the whole-pass attention of fc_sparse_decode_attn (head_subset must be
 * FC_HEADS_ALL) with no context and no workspace.  The schedule and the split partials live in a fixed
 * array of fc_static_scratch_bytes() (8 MiB) that is part of the library's device image; each GPU holds its
 * own copy until the process ends.  The call allocates, creates and frees nothing.
 *   cfg     shapes as for fc_create (max_batch, max_pages_per_seq and max_topk give the strides of the
 *           tables; attn_waves as there); cfg->device must be the calling thread's current device
 *   args    as for fc_sparse_decode_attn; promoted_flags is ignored
 * A shape whose partials do not fit the array ((attn wavefronts + batch * num_kv_heads) * group * 512 B
 * and a little more: 1024 wavefronts with batch 64 x 8 KV heads x group 4 need 3.3 MB) is refused with
 * FC_ERR_WORKSPACE.  All calls on one GPU share that GPU's array: calls that overlap in time on one GPU
 * (different streams, different threads) race; calls on one stream are safe.  Nothing in the array has to
 * be cleared between calls.  fc_static_last_error gives the text of the calling thread's last failure. */
int fc_sparse_decode_attn_static(const fc_config *cfg, const fc_attn_args *args, void *stream);
size_t fc_static_scratch_bytes(void);
const char *fc_static_last_error(void);

/* ---- decode-time growth of the cache ------------------------------------------------------------- */

/* Appends one new token per sequence (Sec. 2: decoding appends one K/V pair per step) and keeps the
 * derived state current.  For every sequence b with append_mask[b] != 0 and every KV head h, with
 * pos = context_lens[b], page = pos / 16, slot = pos % 16:
 *   - slot == 0: a new page starts.  It takes the LAST block of the head's free list (free_count
 *     decreases by one) and block_table[b][h][page] is set; for a stable head the page also joins
 *     resident_pages (it is being appended to, so it is always a member, Sec. 3.3);
 *   - the token's key goes to token row `slot` of each chunk of the K half and its value to column `slot` of the V half;
 *   - MinMax row of the page (Sec. 3.2): set to the key when slot == 0, else elementwise min / max;
 *   - slot == 15 and the head is stable: the page is now full and is copied, once, to
 *     host_pool[host_block_table[b][h][page]] (Sec. 3.3 "Minimizing Transfer Size"); it stays resident
 *     until a later rerank evicts it.
 * Afterwards context_lens[b] += 1.  Needs: page < Nmax, a free block when a page starts, room in the
 * resident list (Kmax > budget + pages started between two reranks).  Violations set the device error
 * word (fc_check_device_state).  A head that cannot take its token (no room in the tables, no free
 * block) writes nothing, and the length of its sequence is then NOT advanced, so that no head is left
 * with a token position that has no block behind it; the other heads of that sequence have written the
 * token all the same, so after FC_ERR_STATE the caller has to drop or rebuild that sequence.
 * Page copies that an earlier fc_promote_pages left in flight (or, with FC_PROMOTE_RIDE, not yet
 * launched) are ordered before this call's writes to the pool, as for an attention call; the same holds
 * for fc_offload_pages. */
typedef struct {
    const void *k_new;               /* dev bf16 [batch][num_kv_heads][D] */
    const void *v_new;               /* dev bf16 [batch][num_kv_heads][D] */
    const uint8_t *append_mask;      /* dev [batch] or NULL (= every sequence) */
    int32_t *context_lens;           /* dev in/out [batch] */
    int32_t *block_table;            /* dev in/out */
    const int32_t *host_block_table; /* dev (stable heads) */
    int32_t *free_blocks;            /* dev in/out [batch][num_kv_heads][Kmax] */
    int32_t *free_count;             /* dev in/out [batch][num_kv_heads] */
    int32_t *resident_pages;         /* dev in/out (stable heads) */
    int32_t *resident_count;         /* dev in/out (stable heads) */
    void *minmax;                    /* dev in/out bf16 [batch][num_kv_heads][Nmax][2][D] */
    void *kv_pool;                   /* dev */
    int64_t num_pool_blocks;
    void *host_pool;                 /* pinned (stable heads) */
    int64_t num_host_blocks;
    const uint8_t *stable_flag;      /* host [num_kv_heads] */
    int32_t batch;
} fc_append_args;
int fc_append_kv(fc_ctx *ctx, const fc_append_args *args, void *stream);

/* Bulk HBM -> pinned host copy of whole pages (the offload after prefill, Sec. 3.3 "Overlapping
 * Transfer with Compute"): pairs[i] = (pool block, host block), dev int32 [n_pairs][2].  A capped
 * number of workgroups writes pinned host memory directly; pairs outside either pool are skipped. */
int fc_offload_pages(fc_ctx *ctx, const void *kv_pool, int64_t num_pool_blocks, void *host_pool,
                     int64_t num_host_blocks, const int32_t *pairs, int32_t n_pairs, void *stream);

/* ---- offline head-stability profiling (Sec. 2.2, 2.3) ------------------------------------------- */

/* One sample's top-K traces -> temporal stability scores and bottom-quartile counts.
 *   traces      dev int32 [steps][heads][topk]: the page list every (layer, head) selected at every
 *               decode step, ascending, -1 padded (what fc_rerank_topk writes); `heads` counts all
 *               (layer, head) pairs that are profiled together
 *   num_pages   dev int32 [steps]: candidate pages N_t at each step
 *   ts_out      dev fp64 [steps - window + 1][heads]:
 *               TS(s) = mean over t = s+1 .. s+window-1 of RCO(s, t),
 *               RCO(s, t) = max(0, (|S_s n S_t| / topk - topk / N_t) / (1 - topk / N_t)), 0 if N_t <= topk
 *   bottom_counts  dev int32 [heads], in/out: for every window the floor(heads / 4) heads with the lowest
 *               TS (ties to the lower head index) are incremented; call once per sample to accumulate. */
typedef struct {
    const int32_t *traces;
    const int32_t *num_pages;
    int32_t steps, heads, topk, window;
    double *ts_out;
    int32_t *bottom_counts;
} fc_stability_args;
int fc_stability_profile(fc_ctx *ctx, const fc_stability_args *args, void *stream);

/* Sec. 2.3: the floor(heads * num / den) heads counted most often in the bottom quartile (ties to the
 * lower head index) are unstable: unstable_out[h] = 1 (dev uint8 [heads]); the paper uses 1/4. */
int fc_classify_heads(fc_ctx *ctx, const int32_t *bottom_counts, int32_t heads, int32_t num, int32_t den,
                      uint8_t *unstable_out, void *stream);

/* Reads (and clears) the device-side error word set by the bookkeeping kernels (a head owning too
 * few blocks, an id out of range that was clamped) and by the attention kernel (a list or table entry
 * outside its range, which it clamps so that every access stays in bounds, or an attended page whose
 * table entry is the null block).  Synchronises `stream`.  Returns FC_OK or
 * FC_ERR_STATE. */
int fc_check_device_state(fc_ctx *ctx, void *stream);

/* Duration of the dominant kernel (the decode attention kernel, FC_HEADS_ALL launches only) measured
 * with HIP events on the stream it is launched on; used by benchmarks.
 * fc_profile_begin first measures, on `stream`, what an event pair around an empty kernel reads (the
 * bracket's own dispatch latency; it synchronises the stream for that), then arms the bracketing of
 * every `every_nth` (>= 1) such launch.  fc_profile_end synchronises and reports the average raw
 * bracket time of the attention launches, the average empty-kernel bracket time, and the count. */
int fc_profile_begin(fc_ctx *ctx, int32_t every_nth, void *stream);
int fc_profile_end(fc_ctx *ctx, double *avg_bracket_ms, double *empty_bracket_ms, int32_t *launches);

/* Same-box ceiling for the number above: a plain streaming read (16 B per lane, grid-stride, no reuse,
 * non-temporal) of `bytes` bytes at `dev_buf` (device memory, 16-byte aligned, bytes a multiple of 16 and
 * >= 4096; only read), timed the same way (HIP-event bracket per launch minus the empty-kernel bracket,
 * averaged over `launches` (1..1000) launches) for grids of 1, 2, 4, 8 and 16 workgroups per compute
 * unit; reports the best shape's GB/s and, optionally, its microseconds per launch (for a read so short
 * that it does not stand out from the bracket's own latency, the uncorrected bracket time is used).  Uses the score
 * scratch of the workspace as its sink; synchronises `stream`; must not be called between
 * fc_profile_begin and fc_profile_end (FC_ERR_STATE). */
int fc_measure_stream_read(fc_ctx *ctx, const void *dev_buf, uint64_t bytes, int32_t launches, void *stream,
                           double *gbps, double *us_per_launch);

#ifdef __cplusplus
}
#endif
#endif /* FLEXICACHE_H */
