// The work of one chunk_score workgroup (paper Sec. 4.1 / 4.3: upper and lower bound of q.k over
// each chunk from its abstract), shared by the chunk_score kernel and the one-launch decode step.
// See chunk_score.hip for the arithmetic and the matrix-core layout.
#pragma once
#include <type_traits>

#include "leoam_dev.h"

namespace leoam {

constexpr int kScoreWaves = 4;
constexpr int kRowsPerSet = 16;    // abstract rows per MFMA = 8 chunks
constexpr int kChunksPerSet = 8;
constexpr size_t kScoreLdsPerWg = 40 * 1024;    // static + dynamic LDS of a workgroup that takes groups of four sets
constexpr size_t kScorePairLdsPerWg = 24 * 1024;    // ... of one that takes pairs of sets (six workgroups per compute unit)

__device__ __forceinline__ double dpp_ror8_d(double v) {
    // value of the lane 8 places away inside the 16-lane row (rotation by 8 is its own inverse)
    const uint64_t u = __builtin_bit_cast(uint64_t, v);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)u, 0x128, 0xf, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)(u >> 32), 0x128, 0xf, 0xf, false);
    return __builtin_bit_cast(double, ((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}

// LDS of one score workgroup: the A operands (clamped queries in double) of every MFMA step.
template <typename T, int G, bool kLower> struct ScoreLds {
    static constexpr int kSteps = (Row<T>::kRowBytes / 64) * T::kEpl;      // 32
    static constexpr int kHeadSets = (G + 3) / 4;
    double qa[kHeadSets][kSteps][LEOAM_WAVE];
    double qb[kLower ? kHeadSets : 1][kLower ? kSteps : 1][LEOAM_WAVE];
};

// The work of workgroup `bx` of the `gx` that share (b, h): kScoreWaves waves, every lane of the
// workgroup calls this (it contains a barrier unless the workgroup has nothing to contract).
// kHeadSets = ceil(G / 4); heads beyond G contribute nothing.
// kSingle: a wave takes single row sets instead of groups of four (launches too small to
// fill the chip: what is waited for then is a wave's own chain of round trips).
// kUnit (with kSingle): row sets a wave takes at a time, all fetched before anything else is done.
// Two at a time is the shape of large launches: a wave then has 8 KiB (16-bit rows) in flight from
// its first instruction on and a workgroup reads 32 KiB; on MI355X this streamed 6-7 % faster than
// groups of four sets fetched two at a time.
template <typename T, int G, bool kLower, bool kSingle, int kUnit = 1>
__device__ __forceinline__ void score_unit(ScoreLds<T, G, kLower>& lds, const char* __restrict__ q,
                                           const char* __restrict__ abstract, const int32_t* __restrict__ n_chunks,
                                           float* __restrict__ score_ub, float* __restrict__ score_lb, int c_max,
                                           int n_kv_heads, int b, int h, int bx, int gx) {
    constexpr int EPL = T::kEpl;                       // elements per 16-byte load
    constexpr int ROWB = Row<T>::kRowBytes;
    constexpr int NLOAD = ROWB / 64;                   // 16-byte loads per lane per row: 4 (16-bit) or 8 (fp32)
    constexpr int NSTEP = NLOAD * EPL;                 // MFMA steps per row set = 32
    constexpr int HS = (G + 3) / 4;                    // passes over the heads
    constexpr int kThreads = kScoreWaves * LEOAM_WAVE;
    auto& qa_lds = lds.qa;
    auto& qb_lds = lds.qb;

    const int wave = threadIdx.x / LEOAM_WAVE, lane = lane_id();
    const int C = min(max(n_chunks[b], 0), c_max);
    const size_t bh = (size_t)b * n_kv_heads + h;
    const char* Abh = abstract + bh * (size_t)c_max * 2 * ROWB;

    // B-operand role of this lane: abstract row r of the set, channel quarter kq
    const int r = lane & 15, kq = lane >> 4;
    const int chunk_in_set = r & 7, is_min_row = r >> 3;
    // A-operand role: head a_head of the pass, block a_blk, channel quarter kq
    const int a_head = lane & 3, a_blk = (lane >> 2) & 3;
    const bool a_min = a_blk >= 2;                                          // blocks 2,3 hold kmin rows

    const int n_sets = (C + kChunksPerSet - 1) / kChunksPerSet;
    const int stride = gx * kScoreWaves;
    // Groups of four sets (16 KiB of 16-bit rows) are cut at addresses that are multiples of their
    // size, not at the start of the (b,h)'s abstract: `lead` sets of the first group lie before it
    // and are skipped.  With c_max not a multiple of 32 the abstracts of different (b,h) start at
    // different offsets inside 16 KiB, and groups cut from each one's start measured 18-30 % slower
    // on MI355X than mutually aligned ones.
    constexpr uintptr_t kSetBytes = (uintptr_t)kRowsPerSet * ROWB;
    const int lead = kSingle ? (kUnit == 2 ? (int)(((uintptr_t)Abh / kSetBytes) & 1) : 0) : (int)(((uintptr_t)Abh / kSetBytes) & 3);

    // Loads are unconditional (a guarded load would make the compiler wait for
    // every outstanding load and defeat the prefetch): a row past the end of the
    // buffer is read from the last chunk instead, and its result is dropped.
    auto fetch = [&](int set, uint4* v) {
        const int c = min(max(set * kChunksPerSet + chunk_in_set, 0), c_max - 1);
        const size_t base = ((size_t)2 * c + is_min_row) * ROWB + 16 * kq;
#pragma unroll
        for (int i = 0; i < NLOAD; ++i) v[i] = load16(Abh, base + 64 * i);
    };

    // software pipeline: the next row set is in flight while this one is contracted;
    // the first fetch goes out before the queries are converted
    uint4 buf[2 * NLOAD];
    uint4* const cur = buf;
    uint4* const nxt = buf + NLOAD;
    const int g0 = bx * kScoreWaves + wave;      // this wave's first group of four sets (or first set)
    // A workgroup past the end of a sequence with fewer chunks than the capacity has nothing to
    // contract: it writes its share of the row's tail and leaves before the queries are staged.
    static_assert(kUnit == 1 || kUnit == 2, "one or two row sets at a time");
    const int n_units = (n_sets + lead + kUnit - 1) / kUnit;
    const int units_here = kSingle ? n_units : (n_sets + lead + 3) >> 2;
    if (bx * kScoreWaves >= units_here) {
        for (int c = C + bx * kThreads + (int)threadIdx.x; c < c_max; c += gx * kThreads) {
            score_ub[bh * c_max + c] = -INFINITY;
            if (kLower) score_lb[bh * c_max + c] = INFINITY;
        }
        return;
    }
    fetch(kSingle ? kUnit * g0 - lead : 4 * g0 - lead, cur);
    if constexpr (kSingle && kUnit == 2) fetch(2 * g0 + 1 - lead, nxt);

    // A operands: clamped query values for every step, in double.  They are the same
    // for the four waves and would take 64 registers per lane, so they live in LDS
    // (each wave converts a quarter) and are read back step by step: the registers
    // this frees double the number of waves a compute unit keeps in flight.
#pragma unroll
    for (int s = 0; s < HS; ++s) {
        const int head = min(4 * s + a_head, G - 1);
        const size_t qrow = ((size_t)b * n_kv_heads * G + (size_t)h * G + head) * ROWB;
        for (int i = wave; i < NLOAD; i += kScoreWaves) {
            float x[EPL];
            unpack<T>(load16(q, qrow + 64 * i + 16 * kq), x);
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                const float xe = (4 * s + a_head < G) ? x[e] : 0.f;
                const float pos = fmaxf(xe, 0.f), neg = fminf(xe, 0.f);
                qa_lds[s][i * EPL + e][lane] = (double)(a_min ? neg : pos);
                if (kLower) qb_lds[s][i * EPL + e][lane] = (double)(a_min ? pos : neg);
            }
        }
    }
    __syncthreads();
    int q_lane = lane;

    // Scores of four consecutive row sets (32 chunks) are collected in one register
    // per lane and written as a single 128-byte line: a store after every set would
    // sit in the same in-order memory counter as the prefetched loads.
    float pend_ub = 0.f, pend_lb = 0.f;
    // the sums of one row set -> its chunks' scores, stored or collected
    auto finish = [&](int it, int set, const double (*ua)[2], const double (*la)[2]) {
        // result lane = 16*head + row; rows r and r+8 are the kmax and kmin halves of chunk r&7
        double ub = -INFINITY, lb = INFINITY;
#pragma unroll
        for (int s = 0; s < HS; ++s) {
            const bool real = (4 * s + kq) < G;                   // result row group kq = head of the pass
            const double u1 = ua[s][0] + ua[s][1];
            const double us = u1 + dpp_ror8_d(u1);
            ub = fmax(ub, real ? us : -INFINITY);
            if (kLower) {
                const double l1 = la[s][0] + la[s][1];
                const double ls = l1 + dpp_ror8_d(l1);
                lb = fmin(lb, real ? ls : INFINITY);
            }
        }
        ub = rows_extreme4_d<true>(ub);
        if (kLower) lb = rows_extreme4_d<false>(lb);
        // every lane holds the score of chunk (lane & 7) of this set
        if constexpr (kSingle) {
            const int c = set * kChunksPerSet + lane;
            if (lane < kChunksPerSet && c >= 0 && c < C) {
                score_ub[bh * c_max + c] = (float)ub + 0.0f;
                if (kLower) score_lb[bh * c_max + c] = (float)lb + 0.0f;
            }
            return;
        }
        const int slot = it & 3;
        if (((lane >> 3) & 3) == slot) {
            pend_ub = (float)ub + 0.0f;
            if (kLower) pend_lb = (float)lb + 0.0f;
        }
        if (slot == 3) {
            const int c = (set - 3) * kChunksPerSet + lane;          // lanes 0..31 <-> the 32 chunks of the group
            if (lane < 4 * kChunksPerSet && c >= 0 && c < C) {
                score_ub[bh * c_max + c] = pend_ub;
                if (kLower) score_lb[bh * c_max + c] = pend_lb;
            }
        }
    };
    // kSets row sets (v[0..NLOAD) the first, v[NLOAD..) the second) are contracted together: an A
    // operand read from LDS serves all of them, and their accumulator chains interleave.  Every
    // set's sums are formed in the same order whatever kSets is.
    auto consume = [&](int it, int set, const uint4* v, auto n_sets_tag) {
        constexpr int kSets = decltype(n_sets_tag)::value;
        asm volatile("" : "+v"(q_lane));      // keeps the LDS reads of the A operands inside this call
        // two interleaved accumulator chains per set and head pass (even / odd steps)
        double ua[kSets][HS][2], la[kSets][kLower ? HS : 1][2];
#pragma unroll
        for (int k = 0; k < kSets; ++k)
#pragma unroll
            for (int s = 0; s < HS; ++s) {
                ua[k][s][0] = ua[k][s][1] = 0.0;
                if (kLower) la[k][s][0] = la[k][s][1] = 0.0;
            }
#pragma unroll
        for (int i = 0; i < NLOAD; ++i) {
            float x[kSets][EPL];
#pragma unroll
            for (int k = 0; k < kSets; ++k) unpack<T>(v[k * NLOAD + i], x[k]);
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
#pragma unroll
                for (int s = 0; s < HS; ++s) {
                    const double qa = qa_lds[s][i * EPL + e][q_lane];
                    double qb = 0.0;
                    if (kLower) qb = qb_lds[s][i * EPL + e][q_lane];
#pragma unroll
                    for (int k = 0; k < kSets; ++k) {
                        const double xd = (double)x[k][e];
                        ua[k][s][e & 1] = __builtin_amdgcn_mfma_f64_4x4x4f64(qa, xd, ua[k][s][e & 1], 0, 0, 0);
                        if (kLower) la[k][s][e & 1] = __builtin_amdgcn_mfma_f64_4x4x4f64(qb, xd, la[k][s][e & 1], 0, 0, 0);
                    }
                }
            }
        }
#pragma unroll
        for (int k = 0; k < kSets; ++k) finish(it + k, set + k, ua[k], la[k]);
    };
    constexpr std::integral_constant<int, 1> kOneSet{};
    constexpr std::integral_constant<int, kUnit> kUnitSets{};

    // A wave takes groups of four consecutive sets, groups round-robin over the
    // waves of the (b,h).  No loads under a condition inside the loop; sets past
    // the end are computed from clamped rows and store nothing.
    if constexpr (kSingle) {
        for (int u = g0; u < n_units; u += stride) {
            if (u != g0) {          // wave-uniform; normally a wave has one unit
                fetch(kUnit * u - lead, cur);
                if constexpr (kUnit == 2) fetch(2 * u + 1 - lead, nxt);
            }
            consume(0, kUnit * u - lead, buf, kUnitSets);
        }
    }
    const int n_groups = kSingle ? 0 : (n_sets + lead + 3) >> 2;
    const int my_groups = g0 < n_groups ? (n_groups - g0 + stride - 1) / stride : 0;
    const int n_it = 4 * my_groups;
    auto set_of = [&](int it) { return 4 * (g0 + (it >> 2) * stride) + (it & 3) - lead; };
    // (n_it is a multiple of four; the last two sets are contracted after the loop, so no set
    // past the wave's last one is fetched)
    int it = 0;
    for (; it + 2 < n_it; it += 2) {
        fetch(set_of(it + 1), nxt);
        __builtin_amdgcn_sched_barrier(0);       // keep the loads ahead of the contraction
        consume(it, set_of(it), cur, kOneSet);
        fetch(set_of(it + 2), cur);
        __builtin_amdgcn_sched_barrier(0);
        consume(it + 1, set_of(it + 1), nxt, kOneSet);
    }
    if (n_it > 0) {
        fetch(set_of(it + 1), nxt);
        __builtin_amdgcn_sched_barrier(0);
        consume(it, set_of(it), cur, kOneSet);
        consume(it + 1, set_of(it + 1), nxt, kOneSet);
    }
    // tail of the row: chunks that do not exist
    for (int c = C + bx * kThreads + (int)threadIdx.x; c < c_max; c += gx * kThreads) {
        score_ub[bh * c_max + c] = -INFINITY;
        if (kLower) score_lb[bh * c_max + c] = INFINITY;
    }
}

// How a launch is cut into workgroups: `gx` workgroups per (b, h); `single`: one row set per wave.
struct ScoreGeometry {
    int gx;
    bool single;
    int unit;      // row sets per wave at a time (single only)
};
// `with_pairs`: large launches may take pairs of row sets (see launch_score for when that pays).
inline ScoreGeometry score_geometry(const leoam_shape* s, bool with_pairs) {
    // Enough workgroups that every wave takes a single group of row sets (a wave that walks on to
    // a second group, a whole grid further, measured 3-10 % slower).  The count per (b,h) is kept
    // odd: with 8, 16 or 32 workgroups per (b,h) the kernel measured 13 % slower on MI355X (the
    // workgroups that run together then walk the abstract at a power-of-two stride).
    const int sets = (s->c_max + kChunksPerSet - 1) / kChunksPerSet;
    const int units = s->batch * s->n_kv_heads;
    const int groups = (sets + 3 + 3) / 4;                  // a wave works on groups of four sets (up to three lead sets)
    // small launches (groups of four would leave the chip under four waves per SIMD): one set per wave
    const bool single = (long long)groups * units <= 4096;
    const int gx_max = ((single ? sets : groups) + kScoreWaves - 1) / kScoreWaves;
    int gx = single ? (4480 + units - 1) / units : gx_max;      // (small launches: about eighteen workgroups per CU)
    if (gx > gx_max) gx = gx_max;
    gx |= 1;
    if (!single && with_pairs) {
        // large launches: a wave takes one pair of row sets (up to one lead set)
        const int pairs = (sets + 1 + 1) / 2;
        return {((pairs + kScoreWaves - 1) / kScoreWaves) | 1, true, 2};
    }
    return {gx, single, 1};
}


}  // namespace leoam
