// Offline head-stability profiling (Sec. 2.2, 2.3 of the paper) on top-K traces as fc_rerank_topk
// emits them (ascending page ids, -1 padded): random-corrected overlap, temporal stability score,
// bottom-quartile counting and the stable / unstable classification.  All floating point is fp64 with
// explicitly rounded operations in a fixed order, so that the ranking decisions taken from the scores
// are the same as those of a plain CPU statement of the formulas.
#include "fc_internal.h"

struct fc_stability_params {
    const int32_t *traces;     // [steps][heads][K]
    const int32_t *num_pages;  // [steps]
    int steps, heads, K, W, windows;
    double *ts;                // [windows][heads]
    int32_t *counts;           // [heads], accumulated
};

// One wavefront per (head, window start s): S_s in LDS, lanes binary-search the entries of S_t in it.
__global__ __launch_bounds__(64) void fc_stability_kernel(fc_stability_params p)
{
    extern __shared__ int32_t ref[];
    const int h = blockIdx.x, s = blockIdx.y, lane = threadIdx.x;
    const int32_t *a = p.traces + ((size_t)s * p.heads + h) * p.K;
    int n_valid = 0;
    for (int i = lane; i < p.K; i += 64) {
        const int32_t x = a[i];
        ref[i] = x;
        n_valid += x >= 0;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) n_valid += __shfl_xor(n_valid, d);
    __syncthreads();
    double acc = 0.0;
    for (int t = s + 1; t <= s + p.W - 1; ++t) {
        const int32_t *b = p.traces + ((size_t)t * p.heads + h) * p.K;
        int inter = 0;
        for (int i = lane; i < p.K; i += 64) {
            const int32_t x = b[i];
            if (x < 0) continue;
            int lo = 0, hi = n_valid;
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                const int32_t v = ref[mid];
                if (v == x) { ++inter; break; }
                if (v < x) lo = mid + 1; else hi = mid;
            }
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) inter += __shfl_xor(inter, d);
        const int n_t = p.num_pages[t];
        double r = 0.0;
        if (n_t > p.K) {
            const double chance = __ddiv_rn((double)p.K, (double)n_t);
            r = __ddiv_rn(__dsub_rn(__ddiv_rn((double)inter, (double)p.K), chance), __dsub_rn(1.0, chance));
            r = r > 0.0 ? r : 0.0;
        }
        acc = __dadd_rn(acc, r);
    }
    if (lane == 0) p.ts[(size_t)s * p.heads + h] = __ddiv_rn(acc, (double)(p.W - 1));
}

// One workgroup per window: the floor(heads / 4) lowest scores (ties to the lower head index) get a count.
__global__ __launch_bounds__(256) void fc_bottom_quartile_kernel(fc_stability_params p)
{
    extern __shared__ double row[];
    const int w = blockIdx.x;
    for (int h = threadIdx.x; h < p.heads; h += 256) row[h] = p.ts[(size_t)w * p.heads + h];
    __syncthreads();
    const int q = p.heads / 4;
    for (int h = threadIdx.x; h < p.heads; h += 256) {
        const double y = row[h];
        int rank = 0;
        for (int g = 0; g < p.heads; ++g) {
            const double x = row[g];
            rank += (x < y || (x == y && g < h)) ? 1 : 0;
        }
        if (rank < q) atomicAdd(&p.counts[h], 1);
    }
}

__global__ __launch_bounds__(256) void fc_classify_kernel(const int32_t *counts, int heads, int want, uint8_t *flags)
{
    extern __shared__ int32_t cnt[];
    for (int h = threadIdx.x; h < heads; h += 256) cnt[h] = counts[h];
    __syncthreads();
    for (int h = threadIdx.x; h < heads; h += 256) {
        const int y = cnt[h];
        int rank = 0;
        for (int g = 0; g < heads; ++g) rank += (cnt[g] > y || (cnt[g] == y && g < h)) ? 1 : 0;
        flags[h] = rank < want ? 1 : 0;
    }
}

extern "C" int fc_stability_profile(fc_ctx *ctx, const fc_stability_args *a, void *stream)
{
    if (!ctx) return FC_ERR_INVALID_ARG;
    FC_REQUIRE(ctx, a && a->traces && a->num_pages && a->ts_out && a->bottom_counts, "fc_stability_profile: NULL pointer");
    FC_REQUIRE(ctx, a->heads >= 4 && a->heads <= 4096, "fc_stability_profile: heads=%d outside 4..4096", a->heads);
    FC_REQUIRE(ctx, a->topk >= 1 && a->topk <= 8192, "fc_stability_profile: topk=%d outside 1..8192", a->topk);
    FC_REQUIRE(ctx, a->window >= 2, "fc_stability_profile: window must be >= 2");
    FC_REQUIRE(ctx, a->steps >= 1 && a->steps <= 65535 + a->window, "fc_stability_profile: steps out of range");
    fc_stability_params p;
    p.traces = a->traces;
    p.num_pages = a->num_pages;
    p.steps = a->steps;
    p.heads = a->heads;
    p.K = a->topk;
    p.W = a->window;
    p.windows = a->steps - a->window + 1;
    p.ts = a->ts_out;
    p.counts = a->bottom_counts;
    if (p.windows <= 0) return FC_OK;
    hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(fc_stability_kernel, dim3(p.heads, p.windows), dim3(64), (size_t)p.K * sizeof(int32_t), s, p);
    hipLaunchKernelGGL(fc_bottom_quartile_kernel, dim3(p.windows), dim3(256), (size_t)p.heads * sizeof(double), s, p);
    FC_HIP(ctx, hipGetLastError());
    return FC_OK;
}

extern "C" int fc_classify_heads(fc_ctx *ctx, const int32_t *bottom_counts, int32_t heads, int32_t num, int32_t den,
                                 uint8_t *unstable_out, void *stream)
{
    if (!ctx) return FC_ERR_INVALID_ARG;
    FC_REQUIRE(ctx, bottom_counts && unstable_out, "fc_classify_heads: NULL pointer");
    FC_REQUIRE(ctx, heads >= 1 && heads <= 4096, "fc_classify_heads: heads=%d outside 1..4096", heads);
    FC_REQUIRE(ctx, den >= 1 && num >= 0 && num <= den, "fc_classify_heads: fraction %d/%d is not in [0, 1]", num, den);
    const int want = (int)(((long long)heads * num) / den);
    hipLaunchKernelGGL(fc_classify_kernel, dim3(1), dim3(256), (size_t)heads * sizeof(int32_t), (hipStream_t)stream,
                       bottom_counts, heads, want, unstable_out);
    FC_HIP(ctx, hipGetLastError());
    return FC_OK;
}
