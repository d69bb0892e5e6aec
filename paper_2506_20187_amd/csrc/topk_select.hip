// chunk_topk_select: keep the front of the list of chunks ordered by
// (score descending, index ascending) while it fits a chunk-count and a token
// budget (paper Sec. 4.2: priority queue by upper bound, read from the front;
// Sec. 6.1: only the most important share of the cache is loaded).  The
// selection itself is in select_core.h; this kernel writes the kept chunk ids
// out in ascending order.
#include "select_core.h"

namespace leoam {

template <int kIpt>
__global__ __launch_bounds__(kSelThreads) void topk_select_kernel(
    const float* __restrict__ score, const int32_t* __restrict__ chunk_off, const int32_t* __restrict__ n_chunks,
    int max_chunks, int token_budget, int32_t* __restrict__ sel_idx, int32_t* __restrict__ sel_count,
    int32_t* __restrict__ sel_tokens, int c_max, int k_max, int n_kv_heads, int n_ctx) {
    __shared__ SelectLds L;

    const int bh = blockIdx.x, b = bh / n_kv_heads;
    const int tid = threadIdx.x;
    const int C = min(max(n_chunks[b], 0), c_max);
    const int32_t* off = chunk_off + (size_t)b * (c_max + 1);
    const float* srow = score + (size_t)bh * c_max;

    SelectResult<kIpt> R;
    select_keep<kIpt>(L, srow, off, C, c_max, k_max, n_ctx, max_chunks, token_budget, R);
    const int c0 = tid * kIpt;
    int32_t* out = sel_idx + (size_t)bh * k_max;
    uint32_t pos = (uint32_t)(R.kept_before >> 32);
#pragma unroll
    for (int i = 0; i < kIpt; ++i) {
        if (R.keep[i]) {
            if (pos < (uint32_t)k_max) out[pos] = c0 + i;
            ++pos;
        }
    }
    const uint32_t n_kept = (uint32_t)(R.kept_total >> 32);
    for (int i = (int)n_kept + tid; i < k_max; i += kSelThreads) out[i] = -1;
    if (tid == 0) {
        sel_count[bh] = (int32_t)n_kept;
        if (sel_tokens) sel_tokens[bh] = (int32_t)(uint32_t)R.kept_total;
    }
}

hipError_t topk_select_dispatch(const leoam_shape* s, const float* score, const int32_t* chunk_off,
                                const int32_t* n_chunks, int max_chunks, int token_budget, int32_t* sel_idx,
                                int32_t* sel_count, int32_t* sel_tokens, hipStream_t stream) {
    dim3 grid(s->batch * s->n_kv_heads), block(kSelThreads);
#define LEOAM_SEL(IPT)                                                                                         \
    hipLaunchKernelGGL(topk_select_kernel<IPT>, grid, block, 0, stream, score, chunk_off, n_chunks, max_chunks, \
                       token_budget, sel_idx, sel_count, sel_tokens, s->c_max, s->k_max, s->n_kv_heads, s->n_ctx)
    if (s->c_max <= kSelThreads) LEOAM_SEL(1);
    else if (s->c_max <= 2 * kSelThreads) LEOAM_SEL(2);
    else if (s->c_max <= 4 * kSelThreads) LEOAM_SEL(4);
    else if (s->c_max <= 6 * kSelThreads) LEOAM_SEL(6);
    else if (s->c_max <= 8 * kSelThreads) LEOAM_SEL(8);
    else if (s->c_max <= 10 * kSelThreads) LEOAM_SEL(10);
    else if (s->c_max <= 12 * kSelThreads) LEOAM_SEL(12);
    else LEOAM_SEL(16);
#undef LEOAM_SEL
    return hipGetLastError();
}

}  // namespace leoam
