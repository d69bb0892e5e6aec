// Pieces shared by the attention kernels (dense and compressed store): launch
// constants, the online-softmax helpers and the per-split partial layout.
#pragma once
#include <type_traits>

#include "leoam_dev.h"

namespace leoam {

constexpr int kAttWaves = 4;
constexpr int kAttThreads = kAttWaves * LEOAM_WAVE;
constexpr int kAttRows = 8;            // rows per lane group per tile
constexpr int kAttMaxSplits = 256;
constexpr int kAttMaxSel = 8192;       // kept chunks per (b,h) the kernel can index
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ float exp2_or_zero(float x, float m) {
    // 2^(x - m), with 2^(-inf - anything) = 0 also when m is -inf
    return (x == -INFINITY) ? 0.f : exp2f(x - m);
}

// floats per partial: D accumulators + m + l
constexpr int kPartStride = LEOAM_D + 2;


// Where the combined result of a (b, q head) goes when the splits are merged inside the launch
// (arrivals == nullptr: a second kernel merges the partials instead).
struct MergeInLaunch {
    int32_t* arrivals;      // one counter per (b, kv head), zero between launches
    float* out;             // [B, Hq, D]
    float* lse;             // [B, Hq] or nullptr
};
constexpr int kInLaunchMaxSplits = 16;      // more splits than this: a second kernel merges (measured faster from 32 on)

// Cross-wave combine of the workgroup's online-softmax states into the partial
// of this split.  xw[w][g] = (acc[D], m, l) of wave w, head g, log2 domain.
//
// With `mg.arrivals` the splits of a (b, kv head) are also merged in this launch,
// without device-scope fences (on this part a fence is an L2 write-back and
// invalidate): the partial is published with agent-scope relaxed atomic stores
// (write-through), the wave waits for them, one lane takes a ticket from the
// (b, kv head)'s agent-scope counter, and the workgroup that draws the last
// ticket reads every partial back with agent-scope atomic loads (all of them in
// one round trip), folds them in split order (so the result does not depend on
// which workgroup that is), writes out / lse and resets the counter.  No
// workgroup waits for another.  At most kInLaunchMaxSplits splits.
template <int G>
__device__ __forceinline__ void finish_split(float (*xw)[G][kPartStride], float* partial, int b, int h, int split,
                                             int n_splits, int n_kv_heads, const MergeInLaunch mg = {nullptr, nullptr, nullptr}) {
    __shared__ int32_t sh_last;
    const int tid = threadIdx.x;
    const size_t bh = (size_t)b * n_kv_heads + h;
    __syncthreads();
    float* part = partial + bh * G * (size_t)n_splits * kPartStride;
    const bool in_launch = mg.arrivals != nullptr;
    for (int i = tid; i < G * kPartStride; i += kAttThreads) {
        const int g = i / kPartStride, d = i % kPartStride;
        float m = -INFINITY;
#pragma unroll
        for (int w = 0; w < kAttWaves; ++w) m = fmaxf(m, xw[w][g][LEOAM_D]);
        float v = 0.f;
        if (d == LEOAM_D) {
            v = m;
        } else {
#pragma unroll
            for (int w = 0; w < kAttWaves; ++w) {
                const float a = exp2_or_zero(xw[w][g][LEOAM_D], m);
                v += a * (d < LEOAM_D ? xw[w][g][d] : xw[w][g][LEOAM_D + 1]);
            }
        }
        float* dst = &part[((size_t)g * n_splits + split) * kPartStride + d];
        if (in_launch) __hip_atomic_store(dst, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else *dst = v;
    }
    if (!in_launch) return;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // this wave's stores have been acknowledged
    __syncthreads();
    if (tid == 0) {
        const int ticket = __hip_atomic_fetch_add(&mg.arrivals[bh], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int is_last = ticket == n_splits - 1;
        if (is_last) __hip_atomic_store(&mg.arrivals[bh], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sh_last = is_last;
    }
    __syncthreads();
    if (!sh_last) return;
    // The (m, l) pairs of every (head, split) go through LDS, one load per lane; the accumulator
    // columns of up to two (head, channel) pairs per lane are fetched in the same round trip.
    __shared__ float sh_m[G][kInLaunchMaxSplits], sh_l[G][kInLaunchMaxSplits];
    auto merge = [&](auto width) {
        constexpr int kW = decltype(width)::value;            // >= n_splits
        constexpr int kCols = 2;
        float os[kCols][kW];
        auto load_cols = [&](int c0) {          // (a column past the end re-reads the last one)
#pragma unroll
            for (int c = 0; c < kCols; ++c) {
                const int col = min(c0 + c * kAttThreads, G * LEOAM_D - 1), g = col / LEOAM_D, d = col % LEOAM_D;
                const float* base = part + (size_t)g * n_splits * kPartStride;
#pragma unroll
                for (int j = 0; j < kW; ++j)
                    os[c][j] = __hip_atomic_load(&base[(size_t)min(j, n_splits - 1) * kPartStride + d], __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_AGENT);
            }
        };
        auto fold_cols = [&](int c0) {
#pragma unroll
            for (int c = 0; c < kCols; ++c) {
                const int col = c0 + c * kAttThreads;
                if (col >= G * LEOAM_D) continue;
                const int g = col / LEOAM_D, d = col % LEOAM_D;
                float m = -INFINITY;
                for (int j = 0; j < n_splits; ++j) m = fmaxf(m, sh_m[g][j]);
                float l = 0.f, o = 0.f;
#pragma unroll
                for (int j = 0; j < kW; ++j) {
                    if (j < n_splits) {
                        const float a = exp2_or_zero(sh_m[g][j], m);
                        o += a * os[c][j];
                        l += a * sh_l[g][j];
                    }
                }
                const size_t bj = bh * G + g;
                mg.out[bj * LEOAM_D + d] = (l > 0.f) ? o / l : 0.f;
                if (mg.lse && d == 0) mg.lse[bj] = (l > 0.f) ? (m + log2f(l)) * kLn2 : -INFINITY;
            }
        };
        load_cols(tid);
        for (int i = tid; i < G * n_splits; i += kAttThreads) {
            const int g = i / n_splits, sp = i % n_splits;
            const float* p = part + ((size_t)g * n_splits + sp) * kPartStride;
            sh_m[g][sp] = __hip_atomic_load(&p[LEOAM_D], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            sh_l[g][sp] = __hip_atomic_load(&p[LEOAM_D + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();       // every lane of the merging workgroup is here
        fold_cols(tid);
        for (int c0 = tid + kCols * kAttThreads; c0 < G * LEOAM_D; c0 += kCols * kAttThreads) {
            load_cols(c0);
            fold_cols(c0);
        }
    };
    if (n_splits <= 8) merge(std::integral_constant<int, 8>{});
    else merge(std::integral_constant<int, kInLaunchMaxSplits>{});
}


// ---- matrix-core pieces of the 16-bit kernels ----------------------------------
// v_mfma_f32_16x16x32 (bf16 / f16): D[i][j] += sum_k A[i][k] B[k][j], A lane =
// (i = lane%16, k = 8*(lane/16)..+8), B lane = (j = lane%16, same k), D lane =
// (j = lane%16, i = 4*(lane/16)..+4).
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

template <typename T> __device__ __forceinline__ f32x4_t mfma_16x16x32(const uint4& a, const uint4& b, f32x4_t c);
template <> __device__ __forceinline__ f32x4_t mfma_16x16x32<BF16>(const uint4& a, const uint4& b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}
template <> __device__ __forceinline__ f32x4_t mfma_16x16x32<F16>(const uint4& a, const uint4& b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
}

// value held by lane kSrc of this lane's 16-lane row
template <int kSrc> __device__ __forceinline__ float row_bcast(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x150 + kSrc, 0xf, 0xf, true));
}

template <int kBegin, int kEnd, typename F> __device__ __forceinline__ void static_for(F&& f) {
    if constexpr (kBegin < kEnd) {
        f(std::integral_constant<int, kBegin>{});
        static_for<kBegin + 1, kEnd>(f);
    }
}

// host-side launch of the kernel that combines the partials (sparse_attention.hip)
hipError_t launch_attention_merge(const leoam_shape* s, const float* partial, int n_splits, float* out, float* lse,
                                  hipStream_t stream);

}  // namespace leoam
