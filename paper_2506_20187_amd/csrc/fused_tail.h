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

// `exchange` (two splits only, else nullptr): one 64-bit word per (b, q head, channel), zero between calls.
// The two workgroups of a (sequence, kv head) then combine without a ticket and without waiting for
// store acknowledgements: every lane swaps its normalised result (o / l, m + log2 l) into the word
// with ONE atomic exchange; the lane that finds the other split's pair there combines the two, in
// split order, writes the output and puts the word back to zero.  The value travels inside the atomic
// itself, so nothing depends on the order of separate memory operations.
template <int G>
__device__ __forceinline__ void fused_tail(float (*xw)[G][kPartStride], int32_t& sh_last, float* partial,
                                           int32_t* arrivals, float* __restrict__ out, float* __restrict__ lse,
                                           size_t bh, int split, int n_splits,
                                           unsigned long long* exchange = nullptr) {
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
    if (n_splits == 2 && exchange != nullptr) {
        if (!owner) return;
        // w = log2 of this split's softmax denominator, on = its normalised output; the high word of a
        // published pair is never zero (+0 travels as -0), which is what marks the word as taken
        const float w = (l > 0.f) ? m + log2f(l) : -INFINITY;
        const float on = (l > 0.f) ? o / l : 0.f;
        uint32_t wb = float_to_bits(w);
        if (wb == 0u) wb = 0x80000000u;
        const unsigned long long mine = ((unsigned long long)wb << 32) | float_to_bits(on);
        unsigned long long* slot = exchange + bj * LEOAM_D + d;
        const unsigned long long other = __hip_atomic_exchange(slot, mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((uint32_t)(other >> 32) == 0u) return;          // first to arrive: the other split's lane combines
        __hip_atomic_store(slot, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const float w_o = bits_to_float((uint32_t)(other >> 32)), on_o = bits_to_float((uint32_t)other);
        // operands in split order, so that the result does not depend on which split arrived last
        const float w0 = split == 0 ? w : w_o, w1 = split == 0 ? w_o : w;
        const float o0 = split == 0 ? on : on_o, o1 = split == 0 ? on_o : on;
        const float wm = fmaxf(w0, w1);
        const float e0 = exp2_or_zero(w0, wm), e1 = exp2_or_zero(w1, wm);
        const float den = e0 + e1;
        out[bj * LEOAM_D + d] = (den > 0.f) ? (o0 * e0 + o1 * e1) / den : 0.f;
        if (lse && d == 0) lse[bj] = (den > 0.f) ? (wm + log2f(den)) * kLn2 : -INFINITY;
        return;
    }
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
