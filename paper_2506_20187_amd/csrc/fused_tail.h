// The end of a one-launch select + attention workgroup: the sixteen waves' online-softmax
// states (xw[w][g] = (acc[D], m, l), log2 domain) are folded into the split's partial;
// when a (sequence, kv head) has several splits the partial is published and the workgroup
// that arrives last combines them (see select_attention.hip for the protocol).  Every lane
// of the 1024-lane workgroup calls this.
#pragma once
#include "attention_common.h"
#include "select_core.h"

namespace leoam {

constexpr int kFusedWaves = kSelWaves;                 // 16
constexpr int kFusedMergeBatch = 16;

template <int G>
__device__ __forceinline__ void fused_tail(float (*xw)[G][kPartStride], int32_t& sh_last, float* partial,
                                           int32_t* arrivals, float* __restrict__ out, float* __restrict__ lse,
                                           size_t bh, int split, int n_splits) {
    const int tid = threadIdx.x;
    // ---- fold the waves: lane (g, d) gets the split's (m, l, o[d]) ----------------
    const int g = tid >> 7, d = tid & (LEOAM_D - 1);
    const bool owner = tid < G * LEOAM_D;
    float m = -INFINITY, l = 0.f, o = 0.f;
    if (owner) {
#pragma unroll
        for (int w = 0; w < kFusedWaves; ++w) m = fmaxf(m, xw[w][g][LEOAM_D]);
#pragma unroll
        for (int w = 0; w < kFusedWaves; ++w) {
            const float a = exp2_or_zero(xw[w][g][LEOAM_D], m);
            l += a * xw[w][g][LEOAM_D + 1];
            o += a * xw[w][g][d];
        }
    }
    const size_t bj = bh * G + g;
    if (n_splits > 1) {
        // publish the partial, take a ticket; the last workgroup to arrive merges
        float* mine = partial + (bj * (size_t)n_splits + split) * kPartStride;
        if (owner) {
            __hip_atomic_store(&mine[d], o, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (d == 0) {
                __hip_atomic_store(&mine[LEOAM_D], m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(&mine[LEOAM_D + 1], l, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // this wave's stores have been acknowledged
        __syncthreads();
        if (tid == 0) {
            const int ticket = __hip_atomic_fetch_add(&arrivals[bh], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const int is_last = ticket == n_splits - 1;
            if (is_last) __hip_atomic_store(&arrivals[bh], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            sh_last = is_last;
        }
        __syncthreads();
        if (!sh_last || !owner) return;
        const float* base = partial + bj * (size_t)n_splits * kPartStride;
        m = -INFINITY;
        l = 0.f;
        o = 0.f;
        // partials are fetched a batch at a time (one memory round trip each); two splits need a
        // small batch, the many splits of a small batch of sequences a large one
        auto merge_batch = [&](int s0, auto width) {
            constexpr int kW = decltype(width)::value;
            float ms[kW], ls[kW], os[kW];
#pragma unroll
            for (int i = 0; i < kW; ++i) {
                const float* p = base + (size_t)min(s0 + i, n_splits - 1) * kPartStride;
                ms[i] = __hip_atomic_load(&p[LEOAM_D], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ls[i] = __hip_atomic_load(&p[LEOAM_D + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                os[i] = __hip_atomic_load(&p[d], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (s0 + i >= n_splits) {
                    ms[i] = -INFINITY;
                    ls[i] = 0.f;
                    os[i] = 0.f;
                }
            }
            float mb = m;
#pragma unroll
            for (int i = 0; i < kW; ++i) mb = fmaxf(mb, ms[i]);
            const float c = exp2_or_zero(m, mb);
            o *= c;
            l *= c;
            m = mb;
#pragma unroll
            for (int i = 0; i < kW; ++i) {
                const float a = exp2_or_zero(ms[i], m);
                o += a * os[i];
                l += a * ls[i];
            }
        };
        if (n_splits <= 4) {
            merge_batch(0, std::integral_constant<int, 4>{});
        } else {
            for (int s0 = 0; s0 < n_splits; s0 += kFusedMergeBatch) merge_batch(s0, std::integral_constant<int, kFusedMergeBatch>{});
        }
    }
    if (!owner) return;
    out[bj * LEOAM_D + d] = (l > 0.f) ? o / l : 0.f;
    if (lse && d == 0) lse[bj] = (l > 0.f) ? (m + log2f(l)) * kLn2 : -INFINITY;
}

}  // namespace leoam
