// chunk_score: upper (and optional lower) bound of q.k over each chunk from its
// abstract (paper Sec. 4.1: chunk importance = upper bound of the token
// importance in the chunk; Sec. 4.3: bounds from abstracted keys + query).
//
//   U_j[c] = sum_d max(q_j[d]*kmax[d], q_j[d]*kmin[d])
//          = sum_d max(q_j[d],0)*kmax[d] + min(q_j[d],0)*kmin[d]     (kmax >= kmin)
//   L_j[c] = sum_d min(q_j[d],0)*kmax[d] + max(q_j[d],0)*kmin[d]
//
// The abstract of one (b,h) is a contiguous run of rows kmax(0),kmin(0),kmax(1),...
// A wave-wide 16-byte-per-lane load covers 1 KiB of it: 2 chunks (16-bit) or one
// (fp32).  Lanes on a kmax row multiply by max(q,0), lanes on a kmin row by
// min(q,0), so one fused multiply-add per (element, query head) is all the
// arithmetic.  Products of two stored values are exact in double; they are
// accumulated in double and rounded once to float, which makes the score (and
// the selection taken from it) independent of this kernel's summation layout up
// to double rounding.
#include "leoam_dev.h"

namespace leoam {

constexpr int kScoreWaves = 4;
constexpr int kScoreUnroll = 4;   // wave-wide loads in flight per iteration

// sum over the lanes [base, base + kSpan) the lane belongs to; kSpan is a power of two
template <int kSpan> __device__ __forceinline__ double span_sum(double v) {
#pragma unroll
    for (int m = 1; m < kSpan; m <<= 1) v += shfl_xor_d(v, m);
    return v;
}

template <typename T, int G, bool kLower>
__global__ __launch_bounds__(kScoreWaves* LEOAM_WAVE) void chunk_score_kernel(
    const char* __restrict__ q, const char* __restrict__ abstract, const int32_t* __restrict__ n_chunks,
    float* __restrict__ score_ub, float* __restrict__ score_lb, int c_max, int n_kv_heads) {
    constexpr int LPR = Row<T>::kLanesPerRow;
    constexpr int RPL = Row<T>::kRowsPerLoad;
    constexpr int CPL = RPL / 2;                 // chunks per wave-wide load
    constexpr int EPL = T::kEpl;
    constexpr int ROWB = Row<T>::kRowBytes;

    const int b = blockIdx.z, h = blockIdx.y;
    const int wave = threadIdx.x / LEOAM_WAVE, lane = lane_id();
    const int C = min(n_chunks[b], c_max);
    const size_t bh = (size_t)b * n_kv_heads + h;
    const char* Abh = abstract + bh * (size_t)c_max * 2 * ROWB;
    const int row = lane / LPR;                  // row inside a load: even = kmax, odd = kmin
    const bool on_min = row & 1;
    const int slot = row >> 1;                   // chunk inside a load
    const int col = (lane % LPR) * EPL;

    // this lane's share of the clamped queries, in double
    double qu[G][EPL], ql[kLower ? G : 1][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const size_t qrow = ((size_t)b * n_kv_heads * G + (size_t)h * G + g) * ROWB;
        float x[EPL];
        unpack<T>(load16(q, qrow + (size_t)col * T::kBytes), x);
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            const float pos = fmaxf(x[e], 0.f), neg = fminf(x[e], 0.f);
            qu[g][e] = (double)(on_min ? neg : pos);
            if (kLower) ql[g][e] = (double)(on_min ? pos : neg);
        }
    }

    const int n_loads = (C + CPL - 1) / CPL;
    const int stride = gridDim.x * kScoreWaves * kScoreUnroll;
    for (int l0 = (blockIdx.x * kScoreWaves + wave) * kScoreUnroll; l0 < n_loads; l0 += stride) {
        uint4 v[kScoreUnroll];
#pragma unroll
        for (int u = 0; u < kScoreUnroll; ++u) {
            const int c = (l0 + u) * CPL + slot;
            v[u] = make_uint4(0, 0, 0, 0);
            if (c < C) v[u] = load16(Abh, (size_t)(l0 + u) * (LEOAM_WAVE * 16) + (size_t)lane * 16);
        }
#pragma unroll
        for (int u = 0; u < kScoreUnroll; ++u) {
            const int c = (l0 + u) * CPL + slot;
            float x[EPL];
            unpack<T>(v[u], x);
            double xd[EPL];
#pragma unroll
            for (int e = 0; e < EPL; ++e) xd[e] = (double)x[e];
            double ub = -INFINITY, lb = INFINITY;
#pragma unroll
            for (int g = 0; g < G; ++g) {
                double a = 0.0;
#pragma unroll
                for (int e = 0; e < EPL; ++e) a = fma(qu[g][e], xd[e], a);
                a = span_sum<2 * LPR>(a);
                ub = fmax(ub, a);
                if (kLower) {
                    double z = 0.0;
#pragma unroll
                    for (int e = 0; e < EPL; ++e) z = fma(ql[g][e], xd[e], z);
                    z = span_sum<2 * LPR>(z);
                    lb = fmin(lb, z);
                }
            }
            if ((lane % (2 * LPR)) == 0 && c < C) {
                score_ub[bh * c_max + c] = (float)ub + 0.0f;
                if (kLower) score_lb[bh * c_max + c] = (float)lb + 0.0f;
            }
        }
    }
    // tail of the row: chunks that do not exist
    for (int c = C + blockIdx.x * blockDim.x + threadIdx.x; c < c_max; c += gridDim.x * blockDim.x) {
        score_ub[bh * c_max + c] = -INFINITY;
        if (kLower) score_lb[bh * c_max + c] = INFINITY;
    }
}

template <typename T, int G>
static hipError_t launch_score(const leoam_shape* s, const void* q, const void* abstract, const int32_t* n_chunks,
                               float* ub, float* lb, hipStream_t stream) {
    constexpr int CPL = Row<T>::kRowsPerLoad / 2;
    const int loads = (s->c_max + CPL - 1) / CPL;
    int gx = (loads + kScoreWaves * kScoreUnroll - 1) / (kScoreWaves * kScoreUnroll);
    if (gx < 1) gx = 1;
    dim3 grid(gx, s->n_kv_heads, s->batch), block(kScoreWaves * LEOAM_WAVE);
    if (lb)
        hipLaunchKernelGGL((chunk_score_kernel<T, G, true>), grid, block, 0, stream, (const char*)q,
                           (const char*)abstract, n_chunks, ub, lb, s->c_max, s->n_kv_heads);
    else
        hipLaunchKernelGGL((chunk_score_kernel<T, G, false>), grid, block, 0, stream, (const char*)q,
                           (const char*)abstract, n_chunks, ub, lb, s->c_max, s->n_kv_heads);
    return hipGetLastError();
}

template <typename T>
static hipError_t score_by_group(const leoam_shape* s, const void* q, const void* abstract, const int32_t* n_chunks,
                                 float* ub, float* lb, hipStream_t stream) {
    switch (s->n_q_heads / s->n_kv_heads) {
    case 1: return launch_score<T, 1>(s, q, abstract, n_chunks, ub, lb, stream);
    case 2: return launch_score<T, 2>(s, q, abstract, n_chunks, ub, lb, stream);
    case 4: return launch_score<T, 4>(s, q, abstract, n_chunks, ub, lb, stream);
    default: return launch_score<T, 8>(s, q, abstract, n_chunks, ub, lb, stream);
    }
}

hipError_t chunk_score_dispatch(const leoam_shape* s, const void* q, const void* abstract, const int32_t* n_chunks,
                                float* ub, float* lb, hipStream_t stream) {
    switch (s->kv_dtype) {
    case LEOAM_F32: return score_by_group<F32>(s, q, abstract, n_chunks, ub, lb, stream);
    case LEOAM_F16: return score_by_group<F16>(s, q, abstract, n_chunks, ub, lb, stream);
    default: return score_by_group<BF16>(s, q, abstract, n_chunks, ub, lb, stream);
    }
}

}  // namespace leoam
