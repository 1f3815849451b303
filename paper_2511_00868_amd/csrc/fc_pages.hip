// Support kernels: paged-cache writer (token-major K/V -> pool blocks) and MinMax builder (Sec. 3.2).
#include "fc_internal.h"

// One workgroup per (4 consecutive pages, head).  The K half is written in 16-byte pieces to their places in
// the chunked layout (fc_k_elem); the V half is transposed to dim-major through LDS.
constexpr int FC_WRITE_PAGES_PER_BLOCK = 4;

__global__ __launch_bounds__(256) void fc_write_pages_kernel(
    const uint16_t *__restrict__ k_src, const uint16_t *__restrict__ v_src, int n_pages,
    const int32_t *__restrict__ block_ids, int ids_stride, uint16_t *__restrict__ pool, long long num_blocks)
{
    __shared__ uint16_t tile[FC_P][FC_D + 8];
    const int h = blockIdx.y, t = threadIdx.x;
    for (int pp = 0; pp < FC_WRITE_PAGES_PER_BLOCK; ++pp) {
        const int page = blockIdx.x * FC_WRITE_PAGES_PER_BLOCK + pp;
        if (page >= n_pages) break;
        const long long blk = block_ids[(size_t)h * ids_stride + page];
        if (blk <= 0 || blk >= num_blocks) continue;          // uniform over the workgroup
        const size_t src_off = ((size_t)h * n_pages + page) * (FC_P * FC_D);
        uint16_t *dst = pool + (size_t)blk * FC_PAGE_ELEMS;

        // K: 256 threads x 16 B (8 dims of one token, which stay together inside a 32-dim chunk)
        *reinterpret_cast<uint4 *>(dst + fc_k_elem(t >> 4, (t & 15) * 8)) = reinterpret_cast<const uint4 *>(k_src + src_off)[t];

        // V: [16][128] -> [128][16]
        {
            const int tok = t >> 4, c = t & 15;
            uint4 x = reinterpret_cast<const uint4 *>(v_src + src_off)[t];
            *reinterpret_cast<uint4 *>(&tile[tok][c * 8]) = x;
        }
        __syncthreads();
        {
            const int d = t >> 1, half = t & 1;
            uint16_t r[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) r[e] = tile[half * 8 + e][d];
            uint4 x;
            x.x = r[0] | ((uint32_t)r[1] << 16);
            x.y = r[2] | ((uint32_t)r[3] << 16);
            x.z = r[4] | ((uint32_t)r[5] << 16);
            x.w = r[6] | ((uint32_t)r[7] << 16);
            reinterpret_cast<uint4 *>(dst + FC_P * FC_D)[t] = x;   // offset d*16 + half*8 elements = t*8
        }
        __syncthreads();      // the tile is reused by the next page
    }
}

// 16 (listed page, head) pairs per workgroup; 16 threads per page, each owning 8 dims of one 32-dim chunk of
// the K half: 16-byte loads, one per valid token, and two 16-byte stores.  Ties keep the first token's bits
// (strict comparisons in token order), so the rows are reproducible bit for bit.
__global__ __launch_bounds__(256) void fc_minmax_kernel(
    const uint16_t *__restrict__ pool, long long num_blocks, const int32_t *__restrict__ block_ids,
    int ids_stride, const int32_t *__restrict__ page_list, int n_list, int context_len, int n_pages, int max_pages,
    uint16_t *__restrict__ minmax_seq)
{
    const int h = blockIdx.y;
    const int slot = blockIdx.x * 16 + (threadIdx.x >> 4);
    if (slot >= n_list) return;
    const int page = page_list ? page_list[slot] : slot;
    if (page < 0 || page >= n_pages) return;
    const long long blk = block_ids[(size_t)h * ids_stride + page];
    if (blk <= 0 || blk >= num_blocks) return;
    const int ntok = min(FC_P, context_len - page * FC_P);
    const int d0 = ((threadIdx.x >> 2) & 3) * 32 + (threadIdx.x & 3) * 8;       // first of this thread's 8 dims
    const uint16_t *kp = pool + (size_t)blk * FC_PAGE_ELEMS;
    uint16_t lo[8], hi[8];
    float flo[8], fhi[8];
    for (int t = 0; t < ntok; ++t) {
        const uint4 x = *reinterpret_cast<const uint4 *>(kp + fc_k_elem(t, d0));
        const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint16_t b = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
            const float f = __uint_as_float((uint32_t)b << 16);
            if (t == 0 || f < flo[e]) { flo[e] = f; lo[e] = b; }
            if (t == 0 || f > fhi[e]) { fhi[e] = f; hi[e] = b; }
        }
    }
    if (ntok <= 0) return;
    uint16_t *row = minmax_seq + ((size_t)h * max_pages + page) * (2 * FC_D);
    uint4 a, b;
    a.x = lo[0] | ((uint32_t)lo[1] << 16); a.y = lo[2] | ((uint32_t)lo[3] << 16);
    a.z = lo[4] | ((uint32_t)lo[5] << 16); a.w = lo[6] | ((uint32_t)lo[7] << 16);
    b.x = hi[0] | ((uint32_t)hi[1] << 16); b.y = hi[2] | ((uint32_t)hi[3] << 16);
    b.z = hi[4] | ((uint32_t)hi[5] << 16); b.w = hi[6] | ((uint32_t)hi[7] << 16);
    *reinterpret_cast<uint4 *>(row + d0) = a;
    *reinterpret_cast<uint4 *>(row + FC_D + d0) = b;
}

extern "C" int fc_write_kv_pages(fc_ctx *ctx, const void *k_src, const void *v_src, int32_t n_pages,
                                 const int32_t *block_ids, int32_t ids_stride, void *pool,
                                 int64_t num_blocks, void *stream)
{
    if (!ctx) return FC_ERR_INVALID_ARG;
    FC_REQUIRE(ctx, k_src && v_src && block_ids && pool, "fc_write_kv_pages: NULL pointer");
    FC_REQUIRE(ctx, n_pages >= 1 && n_pages <= ctx->cfg.max_pages_per_seq, "fc_write_kv_pages: n_pages=%d outside 1..%d", n_pages, ctx->cfg.max_pages_per_seq);
    FC_REQUIRE(ctx, ids_stride >= n_pages, "fc_write_kv_pages: ids_stride < n_pages");
    FC_REQUIRE(ctx, num_blocks >= 2, "fc_write_kv_pages: pool needs at least the null block and one more");
    dim3 grid((n_pages + FC_WRITE_PAGES_PER_BLOCK - 1) / FC_WRITE_PAGES_PER_BLOCK, ctx->cfg.num_kv_heads);
    hipLaunchKernelGGL(fc_write_pages_kernel, grid, dim3(256), 0, (hipStream_t)stream,
                       (const uint16_t *)k_src, (const uint16_t *)v_src, n_pages, block_ids, ids_stride,
                       (uint16_t *)pool, (long long)num_blocks);
    FC_HIP(ctx, hipGetLastError());
    return FC_OK;
}

extern "C" int fc_build_minmax(fc_ctx *ctx, const void *pool, int64_t num_blocks, const int32_t *block_ids,
                               int32_t ids_stride, const int32_t *page_list, int32_t n_list,
                               int32_t context_len, void *minmax_seq, void *stream)
{
    if (!ctx) return FC_ERR_INVALID_ARG;
    FC_REQUIRE(ctx, pool && block_ids && minmax_seq, "fc_build_minmax: NULL pointer");
    FC_REQUIRE(ctx, context_len >= 1, "fc_build_minmax: context_len must be >= 1");
    const int n_pages = (context_len + FC_P - 1) / FC_P;
    FC_REQUIRE(ctx, n_pages <= ctx->cfg.max_pages_per_seq, "fc_build_minmax: context of %d pages exceeds max_pages_per_seq", n_pages);
    FC_REQUIRE(ctx, ids_stride >= n_pages, "fc_build_minmax: ids_stride < pages");
    FC_REQUIRE(ctx, n_list >= 0 && (page_list || n_list == n_pages), "fc_build_minmax: n_list must equal the page count when page_list is NULL");
    FC_REQUIRE(ctx, num_blocks >= 2, "fc_build_minmax: pool too small");
    if (n_list == 0) return FC_OK;
    dim3 grid((n_list + 15) / 16, ctx->cfg.num_kv_heads);
    hipLaunchKernelGGL(fc_minmax_kernel, grid, dim3(256), 0, (hipStream_t)stream, (const uint16_t *)pool,
                       (long long)num_blocks, block_ids, ids_stride, page_list, n_list, context_len, n_pages,
                       ctx->cfg.max_pages_per_seq, (uint16_t *)minmax_seq);
    FC_HIP(ctx, hipGetLastError());
    return FC_OK;
}
