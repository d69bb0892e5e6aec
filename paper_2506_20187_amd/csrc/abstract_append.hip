// kv_chunk_abstract_append: keeps the per-chunk max / min key vectors (paper
// Sec. 4.3, "KV abstract extraction") up to date while decoding adds one token
// per sequence and step (Sec. 2.1: output tokens are generated one by one and
// join the context).  The maximum / minimum over a chunk and one more key is the
// maximum / minimum of the chunk's abstract and that key, so a step costs
// O(head_dim) per kv head instead of a rebuild: the last chunk grows until it
// holds `chunk_size` tokens (the layer's initial chunk size, Sec. 6.1), then a
// new one-token chunk is opened.
//
// Latency-bound: one workgroup per sequence, a lane group per kv head row.
#include "leoam_dev.h"

namespace leoam {

constexpr int kAppendThreads = 256;

template <typename T>
__global__ __launch_bounds__(kAppendThreads) void abstract_append_kernel(
    const char* __restrict__ K, int32_t* __restrict__ chunk_off, int32_t* __restrict__ n_chunks,
    char* __restrict__ abstract, int32_t* __restrict__ status, int chunk_size, int n_ctx, int c_max, int n_kv_heads) {
    constexpr int LPR = Row<T>::kLanesPerRow;
    constexpr int EPL = T::kEpl;
    constexpr int ROWB = Row<T>::kRowBytes;
    constexpr int GROUPS = kAppendThreads / LPR;

    const int b = blockIdx.x;
    const int grp = threadIdx.x / LPR, col_bytes = (threadIdx.x % LPR) * 16;
    int32_t* off = chunk_off + (size_t)b * (c_max + 1);
    const int C = min(max(n_chunks[b], 0), c_max);
    const int t = min(max(off[C], 0), n_ctx);                 // index of the new token = current length
    const int tail_first = C > 0 ? min(max(off[C - 1], 0), t) : t;
    const bool grow = C > 0 && (t - tail_first) < chunk_size;  // the last chunk still has room
    int st = 0;
    if (t >= n_ctx) st = 1;                                    // the cache is full
    else if (!grow && C >= c_max) st = 2;                      // no room for another chunk

    if (st == 0) {
        const int c = grow ? C - 1 : C;
        for (int h = grp; h < n_kv_heads; h += GROUPS) {
            const size_t bh = (size_t)b * n_kv_heads + h;
            const uint4 knew = load16(K, (bh * (size_t)n_ctx + t) * ROWB + col_bytes);
            char* row = abstract + (bh * (size_t)c_max + c) * 2 * ROWB;
            uint4 vmax = knew, vmin = knew;
            if (grow) {
                float x[EPL], mx[EPL], mn[EPL];
                unpack<T>(knew, x);
                unpack<T>(load16(row, col_bytes), mx);
                unpack<T>(load16(row, ROWB + col_bytes), mn);
#pragma unroll
                for (int e = 0; e < EPL; ++e) {
                    mx[e] = fmaxf(mx[e], x[e]);
                    mn[e] = fminf(mn[e], x[e]);
                }
                vmax = pack<T>(mx);
                vmin = pack<T>(mn);
            }
            store16(row, col_bytes, vmax);
            store16(row, ROWB + col_bytes, vmin);
        }
    }
    __syncthreads();      // every lane has read the old boundaries
    if (threadIdx.x == 0) {
        if (st == 0) {
            if (grow) {
                off[C] = t + 1;
            } else {
                off[C + 1] = t + 1;
                n_chunks[b] = C + 1;
            }
        }
        if (status) status[b] = st;
    }
}

hipError_t abstract_append_dispatch(const leoam_shape* s, const void* K, int32_t* chunk_off, int32_t* n_chunks,
                                    int chunk_size, void* abstract, int32_t* status, hipStream_t stream) {
    dim3 grid(s->batch), block(kAppendThreads);
#define LEOAM_APPEND(TT)                                                                                          \
    hipLaunchKernelGGL(abstract_append_kernel<TT>, grid, block, 0, stream, (const char*)K, chunk_off, n_chunks,   \
                       (char*)abstract, status, chunk_size, s->n_ctx, s->c_max, s->n_kv_heads)
    switch (s->kv_dtype) {
    case LEOAM_F32: LEOAM_APPEND(F32); break;
    case LEOAM_F16: LEOAM_APPEND(F16); break;
    default: LEOAM_APPEND(BF16); break;
    }
#undef LEOAM_APPEND
    return hipGetLastError();
}

}  // namespace leoam
