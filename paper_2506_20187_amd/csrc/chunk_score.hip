// chunk_score: upper (and optional lower) bound of q.k over each chunk from its
// abstract (paper Sec. 4.1: chunk importance = upper bound of the token
// importance in the chunk; Sec. 4.3: bounds from abstracted keys + query).
//
//   U_j[c] = sum_d max(q_j[d]*kmax[d], q_j[d]*kmin[d])
//          = sum_d max(q_j[d],0)*kmax[d] + min(q_j[d],0)*kmin[d]     (kmax >= kmin)
//   L_j[c] = sum_d min(q_j[d],0)*kmax[d] + max(q_j[d],0)*kmin[d]
//
// Products of two stored values are exact in double; they are accumulated in
// double and rounded once to float, so the score (and the selection taken from
// it) does not depend on this kernel's summation layout beyond double rounding.
//
// The double-precision contraction runs on the matrix cores:
// v_mfma_f64_4x4x4 multiplies four independent 4x4 blocks per instruction,
//   D_blk[i][j] += sum_k A_blk[i][k] * B_blk[k][j],
// operands one double per lane with lane = 16*k + 4*blk + i (A), 16*k + 4*blk + j
// (B), result lane = 16*i + 4*blk + j.  Here i = query head of the group (4 per
// pass), j = an abstract row, k = 4 of the 128 channels.  Sixteen abstract rows
// (8 chunks: their 8 kmax rows in blocks 0-1, their 8 kmin rows in blocks 2-3)
// are contracted per instruction; blocks 0-1 carry max(q,0) as A, blocks 2-3
// carry min(q,0), which is exactly the split of the bound above.  No cross-lane
// reduction over channels is needed; one add joins the kmax and kmin halves and
// two exchanges take the maximum over the heads.
//
// HBM-bound: a row set is 4 KiB of contiguous abstract; a lane fetches 16 bytes
// per load, four lanes cover 64 contiguous bytes of a row, four loads the row.
#include "score_core.h"

namespace leoam {

template <typename T, int G, bool kLower, bool kSingle, int kUnit = 1>
__global__ __launch_bounds__(kScoreWaves* LEOAM_WAVE) void chunk_score_kernel(
    const char* __restrict__ q, const char* __restrict__ abstract, const int32_t* __restrict__ n_chunks,
    float* __restrict__ score_ub, float* __restrict__ score_lb, int c_max, int n_kv_heads) {
    __shared__ ScoreLds<T, G, kLower> lds;
    score_unit<T, G, kLower, kSingle, kUnit>(lds, q, abstract, n_chunks, score_ub, score_lb, c_max, n_kv_heads, blockIdx.z,
                                      blockIdx.y, blockIdx.x, gridDim.x);
}

template <typename T, int G>
static hipError_t launch_score(const leoam_shape* s, const void* q, const void* abstract, const int32_t* n_chunks,
                               float* ub, float* lb, hipStream_t stream) {
    // Pairs of row sets, all fetched up front, streamed 1-6 % faster than pipelined groups of four on
    // MI355X when a set is cheap to contract (upper bound only, one pass of up to four heads); with the
    // lower bound or eight heads per group the contraction is twice as long and the pipelined groups,
    // which hide it behind the next fetch, were 8-14 % faster; with one head per group, 2 % faster.
    const bool with_pairs = lb == nullptr && G > 1 && G <= 4;
    const ScoreGeometry geo = score_geometry(s, with_pairs);
    const int gx = geo.gx;
    const bool single = geo.single;
    dim3 grid(gx, s->n_kv_heads, s->batch), block(kScoreWaves * LEOAM_WAVE);
    // Large launches ask for unused dynamic LDS, which caps the workgroups of a compute unit below the
    // seven that registers allow: with more, the requests of more waves interleave in the memory system.
    // Groups of four: 40 KiB per workgroup (four per unit; seven measured 4 % slower on MI355X, three 15 %);
    // pairs: 24 KiB (six per unit; seven measured 3 % slower, five 9 %).
    const size_t a_bytes = (size_t)((G + 3) / 4) * 32 * LEOAM_WAVE * sizeof(double) * (lb ? 2 : 1);
    const size_t lds_pad = (!single && a_bytes < kScoreLdsPerWg) ? kScoreLdsPerWg - a_bytes : 0;
#define LEOAM_SCORE(LOWER, SINGLE)                                                                              \
    hipLaunchKernelGGL((chunk_score_kernel<T, G, LOWER, SINGLE>), grid, block, lds_pad, stream, (const char*)q,  \
                       (const char*)abstract, n_chunks, ub, lb, s->c_max, s->n_kv_heads)
    if (geo.unit == 2) {
        const size_t pad = a_bytes < kScorePairLdsPerWg ? kScorePairLdsPerWg - a_bytes : 0;
        hipLaunchKernelGGL((chunk_score_kernel<T, G, false, true, 2>), grid, block, pad, stream, (const char*)q,
                           (const char*)abstract, n_chunks, ub, lb, s->c_max, s->n_kv_heads);
    } else if (lb) {
        if (single) LEOAM_SCORE(true, true); else LEOAM_SCORE(true, false);
    } else {
        if (single) LEOAM_SCORE(false, true); else LEOAM_SCORE(false, false);
    }
#undef LEOAM_SCORE
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
    switch (s->abstract_dtype) {      // dtype of the abstract and of q
    case LEOAM_F32: return score_by_group<F32>(s, q, abstract, n_chunks, ub, lb, stream);
    case LEOAM_F16: return score_by_group<F16>(s, q, abstract, n_chunks, ub, lb, stream);
    default: return score_by_group<BF16>(s, q, abstract, n_chunks, ub, lb, stream);
    }
}

}  // namespace leoam
