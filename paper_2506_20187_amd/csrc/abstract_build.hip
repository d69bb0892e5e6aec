// kv_chunk_abstract_build: per-chunk element-wise max / min key vectors
// (paper Sec. 4.3, "KV abstract extraction").
//
// HBM-bound: every key is read once (2*D*e bytes of abstract written per chunk).
// One wavefront owns one chunk at a time.  A lane moves 16 bytes of a key row,
// so a wave-wide load covers 1 KiB = 4 rows (16-bit keys) or 2 rows (fp32) of
// contiguous memory; eight such loads are in flight per lane, none of them under
// a condition; the row groups are folded together once per chunk (16-bit keys: by
// lane swaps on the vector ALU, every lane then stores 4 bytes of the abstract).
#include "leoam_dev.h"

namespace leoam {

constexpr int kAbsWaves = 4;     // waves (= chunks in flight) per workgroup
constexpr int kAbsUnroll = 8;    // independent 1 KiB loads per wave iteration

template <typename T>
__global__ __launch_bounds__(kAbsWaves* LEOAM_WAVE) void abstract_build_kernel(
    const char* __restrict__ K, const int32_t* __restrict__ chunk_off, const int32_t* __restrict__ n_chunks,
    char* __restrict__ abstract, int n_ctx, int c_max, int n_kv_heads) {
    constexpr int LPR = Row<T>::kLanesPerRow;
    constexpr int RPL = Row<T>::kRowsPerLoad;
    constexpr int EPL = T::kEpl;
    constexpr int ROWB = Row<T>::kRowBytes;

    const int b = blockIdx.z, h = blockIdx.y;
    const int wave = threadIdx.x / LEOAM_WAVE, lane = lane_id();
    const int C = min(n_chunks[b], c_max);
    const int32_t* off = chunk_off + (size_t)b * (c_max + 1);
    const size_t bh = (size_t)b * n_kv_heads + h;
    const char* Kbh = K + bh * (size_t)n_ctx * ROWB;
    char* Abh = abstract + bh * (size_t)c_max * 2 * ROWB;
    const int rgrp = lane / LPR;                    // which row of a wave-wide load
    const int col_bytes = (lane % LPR) * 16;

    // the boundaries of the wave's next chunk are fetched while this one streams
    const int c_first = blockIdx.x * kAbsWaves + wave, c_step = gridDim.x * kAbsWaves;
    int o0 = off[min(c_first, c_max)], o1 = off[min(c_first + 1, c_max)];
    for (int c = c_first; c < C; c += c_step) {
        const int t0 = min(max(o0, 0), n_ctx);
        const int t1 = min(max(o1, t0), n_ctx);
        o0 = off[min(c + c_step, c_max)];
        o1 = off[min(c + c_step + 1, c_max)];
        float mx[EPL], mn[EPL];
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            mx[e] = -INFINITY;
            mn[e] = INFINITY;
        }
        // kAbsUnroll loads in flight per lane, all unconditional: a row past the chunk's end re-reads
        // its last row (harmless for max / min), so a chunk costs ceil(rows / (kAbsUnroll * RPL))
        // memory round trips and no load waits on a loop test
        if (t1 > t0) {
            for (int t = t0 + rgrp; t < t1; t += kAbsUnroll * RPL) {
                uint4 v[kAbsUnroll];
#pragma unroll
                for (int u = 0; u < kAbsUnroll; ++u)
                    v[u] = load16(Kbh, (size_t)min(t + u * RPL, t1 - 1) * ROWB + col_bytes);
#pragma unroll
                for (int u = 0; u < kAbsUnroll; u += 2) {
                    float x[EPL], y[EPL];
                    unpack<T>(v[u], x);
                    unpack<T>(v[u + 1], y);
#pragma unroll
                    for (int e = 0; e < EPL; ++e) {
                        mx[e] = fmaxf(fmaxf(mx[e], x[e]), y[e]);
                        mn[e] = fminf(fminf(mn[e], x[e]), y[e]);
                    }
                }
            }
        }
        if constexpr (LPR == 16) {
            // fold the four row groups on the vector ALU; row group r ends up with the
            // totals of elements 2r and 2r+1 of its columns and stores those 4 bytes
            float hi[EPL] = {}, lo[EPL] = {};
            hi[0] = rows_extreme_quad<true>(mx[0], mx[4], mx[2], mx[6]);
            hi[1] = rows_extreme_quad<true>(mx[1], mx[5], mx[3], mx[7]);
            lo[0] = rows_extreme_quad<false>(mn[0], mn[4], mn[2], mn[6]);
            lo[1] = rows_extreme_quad<false>(mn[1], mn[5], mn[3], mn[7]);
            char* row = Abh + (size_t)c * 2 * ROWB + col_bytes + 4 * rgrp;
            *reinterpret_cast<uint32_t*>(row) = pack<T>(hi).x;
            *reinterpret_cast<uint32_t*>(row + ROWB) = pack<T>(lo).x;
        } else {
            // fold the row groups (lanes that hold the same columns)
#pragma unroll
            for (int m = LPR; m < LEOAM_WAVE; m <<= 1) {
#pragma unroll
                for (int e = 0; e < EPL; ++e) {
                    mx[e] = fmaxf(mx[e], shfl_xor_f(mx[e], m));
                    mn[e] = fminf(mn[e], shfl_xor_f(mn[e], m));
                }
            }
            // row group 0 writes kmax, row group 1 writes kmin
            if (rgrp == 0) store16(Abh, ((size_t)c * 2 + 0) * ROWB + col_bytes, pack<T>(mx));
            if (rgrp == 1) store16(Abh, ((size_t)c * 2 + 1) * ROWB + col_bytes, pack<T>(mn));
        }
    }
}

template <typename T>
static hipError_t launch_abstract(const leoam_shape* s, const void* K, const int32_t* chunk_off,
                                  const int32_t* n_chunks, void* abstract, hipStream_t stream) {
    int gx = (s->c_max + kAbsWaves - 1) / kAbsWaves;
    if (gx > 8192) gx = 8192;
    dim3 grid(gx, s->n_kv_heads, s->batch);
    hipLaunchKernelGGL(abstract_build_kernel<T>, grid, dim3(kAbsWaves * LEOAM_WAVE), 0, stream, (const char*)K, chunk_off,
                       n_chunks, (char*)abstract, s->n_ctx, s->c_max, s->n_kv_heads);
    return hipGetLastError();
}

hipError_t abstract_build_dispatch(const leoam_shape* s, const void* K, const int32_t* chunk_off,
                                   const int32_t* n_chunks, void* abstract, hipStream_t stream) {
    switch (s->kv_dtype) {
    case LEOAM_F32: return launch_abstract<F32>(s, K, chunk_off, n_chunks, abstract, stream);
    case LEOAM_F16: return launch_abstract<F16>(s, K, chunk_off, n_chunks, abstract, stream);
    default: return launch_abstract<BF16>(s, K, chunk_off, n_chunks, abstract, stream);
    }
}

}  // namespace leoam
