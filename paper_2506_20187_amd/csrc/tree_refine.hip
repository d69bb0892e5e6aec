// chunk_tree_refine: tree-structured chunk management (paper Sec. 4.2, Fig. 9).
//
// Per (sequence, kv head) the context starts as equal chunks whose bounds come
// from the prefill-time abstract (Sec. 4.3); chunks are ordered by their upper
// bound U, the front of that order is read until it covers k tokens, front
// chunks whose lower bound L beats the upper bound of all but at most k tokens
// are confirmed, the other front chunks are split in two and their halves
// evaluated from the keys themselves; runs of chunks that cannot hold one of the
// k most important tokens are merged.  Importance of a token = max over the
// group's query heads of q_j.k_t; U = max_j U_j, L = max_j L_j (every token of
// the chunk reaches it), so U = L = the importance for a single token.
//
// All order statistics are over tokens (a chunk counts `size` times):
//   v      = k-th largest U      chunks with U >= v are the front of the queue
//   mu     = (k+1)-th largest U  (-inf when k == n_ctx)
//   lambda = k-th largest L
//   confirmed: L > mu;  unimportant: U < lambda;  split: U >= v, not confirmed, size > 1.
// They are found without sorting: a radix descent over the order-preserving
// integer image of the floats (8-bit digits, token-weighted histogram in LDS;
// the bits every key shares are skipped, which also spreads the first digit
// over the bins).  v is needed in every round, lambda only for the final
// merge; mu is v if the chunks with U >= v hold more than k tokens, else the
// largest U below v.
//
// One 1024-lane workgroup per (sequence, kv head) runs every round; the node
// list (start, size, U, L) lives in the workspace, double-buffered, in position
// order (a split node is replaced by its two halves at scanned positions); a
// thread keeps its 8 consecutive nodes in registers through a round.  A lane
// group as wide as a key row evaluates a node - element-wise max / min over its
// key rows (the two abstract rows for an initial chunk), then the bounds in
// double, rounded once to float - so a wave has 4 (fp32: 2) nodes in flight.
// For four query heads the lanes of a quad trade partial sums so that the
// cross-lane reduction handles the eight sums of a node together.
// The halves of two-token nodes are single tokens (U = L = max_j q_j.k); with up
// to four heads per group a wave evaluates sixteen of them at a time on the matrix
// cores (v_mfma_f64_4x4x4 as in chunk_score.hip: the sixteen B rows are the
// tokens' key rows, every A block carries the queries), the rows of several
// such groups in flight; the initial chunks are evaluated eight at a time the
// same way, with both bounds (B rows 0-7 their kmax rows, rows 8-15 their kmin
// rows).  To bring the single tokens together the split nodes of a round are
// listed in two classes (two-token nodes from the front of the task list, the
// others from its back).  The evaluation phase dominates: its first rounds are
// chains of dependent round trips (large nodes, few of them), the later ones are
// bound by the double-precision arithmetic.
#include <cfloat>
#include <type_traits>

#include "score_core.h"

namespace leoam {

constexpr int kTreeThreads = 1024;
constexpr int kTreeCache = 8;          // nodes per thread held in registers through a round
constexpr int kTreeTile = kTreeCache * kTreeThreads;
constexpr int kTreeWaves = kTreeThreads / LEOAM_WAVE;
constexpr int kTreeMaxG = 8;

struct alignas(16) TreeNode {
    int32_t start, size;
    float U, L;
};

__device__ __forceinline__ uint32_t tree_key(float s) {
    uint32_t u = float_to_bits(s + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float tree_unkey(uint32_t k) {
    return bits_to_float((k & 0x80000000u) ? (k ^ 0x80000000u) : ~k);
}

struct TreeLds {
    alignas(16) double qpos[kTreeMaxG][LEOAM_D], qneg[kTreeMaxG][LEOAM_D];      // max(q, 0), min(q, 0); order: q_slot()
    alignas(16) double qall[kTreeMaxG][LEOAM_D];                                 // q itself (single-token nodes)
    uint32_t hist[256];
    uint32_t wave_tot[kTreeWaves];
    uint32_t key_lo, key_hi, digit, rank;
    uint32_t ge_weight, below_key, below_any;
    uint32_t carry;
};

// A operands of the evaluations on the matrix cores (groups of up to four heads): clamped queries in
// double for each of the 32 steps; lane = 16 * channel quarter + 4 * block + head.  qa (upper bound):
// blocks 0-1 carry max(q,0), blocks 2-3 min(q,0); qb (lower bound): the reverse.  qa + qb is the query
// itself in every block (one of the two is zero), which is what single tokens are multiplied with.
struct TreeMfmaLds {
    double qa[32][LEOAM_WAVE], qb[32][LEOAM_WAVE];
};

// A task of the evaluation phase: a node that is split, and where its halves go.
struct alignas(16) TreeTask {
    int32_t start, size, pos, pad;
};

// exclusive scan of v over the workgroup in lane order; *total = sum
__device__ __forceinline__ uint32_t tree_block_scan(uint32_t v, uint32_t* wave_tot, uint32_t* total) {
    const int lane = lane_id(), wave = threadIdx.x / LEOAM_WAVE;
    const uint32_t incl = wave_incl_scan_u32(v);
    __syncthreads();
    if (lane == LEOAM_WAVE - 1) wave_tot[wave] = incl;
    __syncthreads();
    const uint32_t s = wave_tot[lane & (kTreeWaves - 1)];
    const uint32_t sc = row16_incl_scan_u32(s);
    *total = (uint32_t)__builtin_amdgcn_readlane((int)sc, kTreeWaves - 1);
    const uint32_t upto = (uint32_t)__builtin_amdgcn_readlane((int)sc, wave);
    const uint32_t own = (uint32_t)__builtin_amdgcn_readlane((int)s, wave);
    return upto - own + incl - v;
}

// a double from another lane of the 16-lane row (every lane of a row is a valid source here)
template <int kCtrl> __device__ __forceinline__ double dpp_d(double v) {
    const uint64_t u = __builtin_bit_cast(uint64_t, v);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)u, kCtrl, 0xf, 0xf, true);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)(u >> 32), kCtrl, 0xf, 0xf, true);
    return __builtin_bit_cast(double, ((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}
template <int kCtrl> __device__ __forceinline__ float tree_dpp_f(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), kCtrl, 0xf, 0xf, true));
}
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E, kDppRor4 = 0x124, kDppRor8 = 0x128;

// sum of a double over the lanes of a group of kLanes (16 or 32) lanes; every lane gets it
template <int kLanes> __device__ __forceinline__ double group_sum_d(double v) {
    v += dpp_d<kDppXor1>(v);
    v += dpp_d<kDppXor2>(v);
    v += dpp_d<kDppRor4>(v);
    v += dpp_d<kDppRor8>(v);
    if (kLanes == 32) v += shfl_xor_d(v, 16);
    return v;
}

// Where channel e of a lane sits in TreeLds::qpos / qneg: a lane reads its channels two at a
// time (16 bytes) and the lanes of a row then read consecutive 16-byte pieces.
template <typename T> __device__ __forceinline__ int q_slot(int lane_in_row, int e) {
    return (e / 2) * (Row<T>::kLanesPerRow * 2) + lane_in_row * 2 + (e % 2);
}

// A lane group (the lanes that cover one key row: 16 for 16-bit keys, 32 for fp32)
// computes the bounds of one node: max / min over `n_rows` rows starting at `rows`,
// then U = max_j sum_d max(q k_max, q k_min) and L = max_j sum_d min(..), each sum
// in double, rounded once to float.  A wave evaluates 4 (2) nodes at a time.
template <typename T>
__device__ __forceinline__ void tree_eval(const char* rows, int n_rows, const double (*qpos)[LEOAM_D],
                                          const double (*qneg)[LEOAM_D], const double (*qall)[LEOAM_D], int G, float* U,
                                          float* L) {
    constexpr int LPR = Row<T>::kLanesPerRow;
    constexpr int EPL = T::kEpl;
    constexpr int ROWB = Row<T>::kRowBytes;
    const int lane_in_row = lane_id() % LPR, col = lane_in_row * EPL;
    float mx[EPL], mn[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        mx[e] = -INFINITY;
        mn[e] = INFINITY;
    }
    // kBatch rows in flight; a row index past the end re-reads the last row (harmless for max / min,
    // and the loads stay unconditional)
    auto rows_from = [&](int r0, auto batch) {
        constexpr int kBatch = decltype(batch)::value;
        uint4 v[kBatch];
#pragma unroll
        for (int j = 0; j < kBatch; ++j)
            v[j] = load16(rows, (size_t)min(r0 + j, n_rows - 1) * ROWB + (size_t)col * T::kBytes);
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            float x[EPL];
            unpack<T>(v[j], x);
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                mx[e] = fmaxf(mx[e], x[e]);
                mn[e] = fminf(mn[e], x[e]);
            }
        }
    };
    // the batch size follows the largest node of the wave, so the lane groups never take
    // different paths (a group with fewer rows re-reads its last row)
    int w_rows = n_rows;
#pragma unroll
    for (int g = 0; g < LEOAM_WAVE; g += LPR) w_rows = max(w_rows, __builtin_amdgcn_readlane(n_rows, g));
    if (w_rows == 1) {
        // Single tokens only: kmax = kmin = the key row, so U = L = max_j q_j.k.  The sums below are the
        // values the general path gives (there one of max(q,0), min(q,0) is zero in every product and
        // adds nothing), at a quarter of the multiply-adds and half of the cross-lane reduction.
        rows_from(0, std::integral_constant<int, 1>{});
        auto head_dot = [&](int j) {
            double s0 = 0.0, s1 = 0.0;
#pragma unroll
            for (int e = 0; e < EPL; e += 2) {
                const double2 qq = *reinterpret_cast<const double2*>(&qall[j][q_slot<T>(lane_in_row, e)]);
                s0 = fma(qq.x, (double)mx[e], s0);
                s1 = fma(qq.y, (double)mx[e + 1], s1);
            }
            return s0 + s1;
        };
        float ub = -INFINITY;
        if (G == 4) {
            double x[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) x[j] = head_dot(j);
            const bool b0 = lane_in_row & 1, b1 = lane_in_row & 2;
            double y[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const double keep = b0 ? x[2 + i] : x[i], send = b0 ? x[i] : x[2 + i];
                y[i] = keep + dpp_d<kDppXor1>(send);
            }
            double z = (b1 ? y[1] : y[0]) + dpp_d<kDppXor2>(b1 ? y[0] : y[1]);
            z += dpp_d<kDppRor4>(z);
            z += dpp_d<kDppRor8>(z);
            if (LPR == 32) z += shfl_xor_d(z, 16);
            // this lane: head 2 * b0 + b1; the maximum over the quad is the maximum over the heads
            ub = (float)z + 0.0f;
            ub = fmaxf(ub, tree_dpp_f<kDppXor1>(ub));
            ub = fmaxf(ub, tree_dpp_f<kDppXor2>(ub));
        } else {
            for (int j = 0; j < G; ++j) ub = fmaxf(ub, (float)group_sum_d<LPR>(head_dot(j)) + 0.0f);
        }
        *U = ub;
        *L = ub;
        return;
    }
    if (w_rows <= 2) {          // also an initial chunk: its kmax row and its kmin row
        rows_from(0, std::integral_constant<int, 2>{});
    } else if (w_rows <= 4) {
        rows_from(0, std::integral_constant<int, 4>{});
    } else {
        for (int r0 = 0; r0 < w_rows; r0 += 8) rows_from(r0, std::integral_constant<int, 8>{});
    }
    double hi[EPL], lo[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        hi[e] = (double)mx[e];
        lo[e] = (double)mn[e];
    }
    // max(q k_max, q k_min) = max(q,0) k_max + min(q,0) k_min (k_max >= k_min): one of the two
    // products is zero and every product is exact in double.  Two independent chains per bound.
    auto head_sums = [&](int j, double* u, double* l) {
        double u0 = 0.0, u1 = 0.0, l0 = 0.0, l1 = 0.0;
#pragma unroll
        for (int e = 0; e < EPL; e += 2) {
            const double2 qp = *reinterpret_cast<const double2*>(&qpos[j][q_slot<T>(lane_in_row, e)]);
            const double2 qn = *reinterpret_cast<const double2*>(&qneg[j][q_slot<T>(lane_in_row, e)]);
            u0 = fma(qp.x, hi[e], u0);
            u0 = fma(qn.x, lo[e], u0);
            l0 = fma(qp.x, lo[e], l0);
            l0 = fma(qn.x, hi[e], l0);
            u1 = fma(qp.y, hi[e + 1], u1);
            u1 = fma(qn.y, lo[e + 1], u1);
            l1 = fma(qp.y, lo[e + 1], l1);
            l1 = fma(qn.y, hi[e + 1], l1);
        }
        *u = u0 + u1;
        *l = l0 + l1;
    };
    float ub = -INFINITY, lb = -INFINITY;
    if (G == 4) {
        // Four heads at once: the lanes of a quad first trade partial sums so that each ends up
        // with one head's pair (8 -> 4 -> 2 values per lane), the quads of the row are then added.
        double x[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) head_sums(j, &x[2 * j], &x[2 * j + 1]);
        const bool b0 = lane_in_row & 1, b1 = lane_in_row & 2;
        double y[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const double keep = b0 ? x[4 + i] : x[i], send = b0 ? x[i] : x[4 + i];
            y[i] = keep + dpp_d<kDppXor1>(send);
        }
        double z[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const double keep = b1 ? y[2 + i] : y[i], send = b1 ? y[i] : y[2 + i];
            z[i] = keep + dpp_d<kDppXor2>(send);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            z[i] += dpp_d<kDppRor4>(z[i]);
            z[i] += dpp_d<kDppRor8>(z[i]);
            if (LPR == 32) z[i] += shfl_xor_d(z[i], 16);
        }
        // this lane: head 2 * b0 + b1; the maximum over the quad is the maximum over the heads
        ub = (float)z[0] + 0.0f;
        lb = (float)z[1] + 0.0f;
        ub = fmaxf(ub, tree_dpp_f<kDppXor1>(ub));
        lb = fmaxf(lb, tree_dpp_f<kDppXor1>(lb));
        ub = fmaxf(ub, tree_dpp_f<kDppXor2>(ub));
        lb = fmaxf(lb, tree_dpp_f<kDppXor2>(lb));
    } else {
        for (int j = 0; j < G; ++j) {
            double u, l;
            head_sums(j, &u, &l);
            u = group_sum_d<LPR>(u);
            l = group_sum_d<LPR>(l);
            ub = fmaxf(ub, (float)u + 0.0f);
            lb = fmaxf(lb, (float)l + 0.0f);
        }
    }
    *U = ub;
    *L = lb;
}

// Sixteen single tokens per wave on the matrix cores.  Lane (r = lane & 15, kq = lane >> 4) holds the
// four 16-byte pieces 64 i + 16 kq of token r's key row (`v`, fetched by tree_fetch_row); step (i, e)
// multiplies the four heads' values of its four channels with the sixteen rows' (block = four rows),
// so that after the 32 steps result lane 16 * head + r holds q_head . k_r; two lane swaps take the
// maximum over the heads.  Every lane returns the importance of token lane & 15.
template <typename T>
__device__ __forceinline__ void tree_fetch_row(const char* row, uint4* v) {
    constexpr int NLOAD = Row<T>::kRowBytes / 64;
    const int kq = lane_id() >> 4;
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) v[i] = load16(row, 64 * i + 16 * kq);
}
template <typename T>
__device__ __forceinline__ float tree_tokens16(const uint4* v, const TreeMfmaLds& A, int G) {
    constexpr int EPL = T::kEpl;
    constexpr int NLOAD = Row<T>::kRowBytes / 64;
    int q_lane = lane_id();
    asm volatile("" : "+v"(q_lane));      // keeps the LDS reads of the A operands inside this call
    double acc[2] = {0.0, 0.0};
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
        float x[EPL];
        unpack<T>(v[i], x);
#pragma unroll
        for (int e = 0; e < EPL; ++e)
            acc[e & 1] = __builtin_amdgcn_mfma_f64_4x4x4f64(A.qa[i * EPL + e][q_lane] + A.qb[i * EPL + e][q_lane], (double)x[e],
                                                            acc[e & 1], 0, 0, 0);
    }
    const bool real = (q_lane >> 4) < G;      // result row group = head
    return (float)rows_extreme4_d<true>(real ? acc[0] + acc[1] : -INFINITY) + 0.0f;
}

// Eight nodes of up to kRows key rows per wave on the matrix cores, both bounds.  Lane (r = lane & 15,
// kq = lane >> 4) works for node r & 7: tree_fetch_node reads its pieces of the node's rows (a row
// index past the node's end re-reads its last row), tree_nodes8 folds them into their element-wise
// maximum (r < 8) or minimum (r >= 8) - its B operand - and contracts: B rows 0-7 are the nodes' kmax
// rows, rows 8-15 their kmin rows, the sums of the two halves are joined by one add and the maximum over
// the heads by two lane swaps.  Every lane returns U and L of node lane & 7.
template <typename T, int kRows>
__device__ __forceinline__ void tree_fetch_node(const char* my_rows, int my_n, uint4 (*v)[Row<T>::kRowBytes / 64]) {
    constexpr int ROWB = Row<T>::kRowBytes;
    constexpr int NLOAD = ROWB / 64;
    const int kq = lane_id() >> 4;
#pragma unroll
    for (int t = 0; t < kRows; ++t)
#pragma unroll
        for (int i = 0; i < NLOAD; ++i) v[t][i] = load16(my_rows, (size_t)min(t, my_n - 1) * ROWB + 64 * i + 16 * kq);
}
template <typename T, int kRows>
__device__ __forceinline__ void tree_nodes8(const uint4 (*v)[Row<T>::kRowBytes / 64], const TreeMfmaLds& A, int G, float* U,
                                            float* L) {
    constexpr int EPL = T::kEpl;
    constexpr int NLOAD = Row<T>::kRowBytes / 64;
    int q_lane = lane_id();
    asm volatile("" : "+v"(q_lane));
    // minimum lanes fold -x with max: -max(-x) = min(x), exactly
    const float sign = (q_lane & 8) ? -1.f : 1.f;
    double ua[2] = {0.0, 0.0}, la[2] = {0.0, 0.0};
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
        float x[EPL];
        unpack<T>(v[0][i], x);
        if constexpr (kRows > 1) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) x[e] *= sign;
#pragma unroll
            for (int t = 1; t < kRows; ++t) {
                float y[EPL];
                unpack<T>(v[t][i], y);
#pragma unroll
                for (int e = 0; e < EPL; ++e) x[e] = fmaxf(x[e], y[e] * sign);
            }
#pragma unroll
            for (int e = 0; e < EPL; ++e) x[e] *= sign;
        }
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            const double xd = (double)x[e];
            ua[e & 1] = __builtin_amdgcn_mfma_f64_4x4x4f64(A.qa[i * EPL + e][q_lane], xd, ua[e & 1], 0, 0, 0);
            la[e & 1] = __builtin_amdgcn_mfma_f64_4x4x4f64(A.qb[i * EPL + e][q_lane], xd, la[e & 1], 0, 0, 0);
        }
    }
    // result lane = 16 * head + B row; rows r and r + 8 are the two halves of node r & 7
    const bool real = (q_lane >> 4) < G;
    const double u1 = ua[0] + ua[1], l1 = la[0] + la[1];
    const double ub = u1 + dpp_ror8_d(u1), lb = l1 + dpp_ror8_d(l1);
    *U = (float)rows_extreme4_d<true>(real ? ub : -INFINITY) + 0.0f;
    *L = (float)rows_extreme4_d<true>(real ? lb : -INFINITY) + 0.0f;
}

template <typename T>
__global__ __launch_bounds__(kTreeThreads) void tree_refine_kernel(
    const char* __restrict__ q, const char* __restrict__ K, const char* __restrict__ abstract, int chunk_size,
    int k_tokens, int max_rounds, int node_cap, int32_t* __restrict__ ref_off, float* __restrict__ ref_score,
    int32_t* __restrict__ ref_count, int32_t* __restrict__ ref_evals, int32_t* __restrict__ ref_status,
    TreeNode* nodes_a, TreeNode* nodes_b, TreeTask* task_buf, int n_ctx, int c_max, int n_kv_heads, int G) {
    constexpr int ROWB = Row<T>::kRowBytes;
    constexpr int EPL = T::kEpl;
    __shared__ TreeLds S;
    __shared__ TreeMfmaLds A;
    constexpr int NLOAD = ROWB / 64;
    constexpr int kTokenPasses = 8 / NLOAD;        // groups of sixteen tokens a wave keeps in flight (8 loads per lane)
    constexpr int kNodePasses = 16 / NLOAD;        // groups of eight one-row nodes in flight (16 loads per lane)
    const bool mfma = G <= 4;

    const int h = blockIdx.x, b = blockIdx.y;
    const size_t bh = (size_t)b * n_kv_heads + h;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid / LEOAM_WAVE;
    const int m0 = (n_ctx + chunk_size - 1) / chunk_size;
    TreeNode* cur = nodes_a + bh * (size_t)node_cap;
    TreeNode* nxt = nodes_b + bh * (size_t)node_cap;
    TreeTask* task = task_buf + bh * (size_t)((node_cap + 1) / 2);
    constexpr int LPR = Row<T>::kLanesPerRow;
    constexpr int kGroups = kTreeThreads / LPR;              // node evaluations in flight per workgroup
    const int gid = tid / LPR;
    const bool g_lead = (tid % LPR) == 0;
    const char* Kbh = K + bh * (size_t)n_ctx * ROWB;
    const char* Abh = abstract + bh * (size_t)c_max * 2 * ROWB;

    // ---- queries of the group ------------------------------------------------------
    for (int i = tid; i < G * LPR; i += kTreeThreads) {
        const int j = i / LPR, lr = i % LPR;
        float x[EPL];
        unpack<T>(load16(q, ((size_t)b * n_kv_heads * G + (size_t)h * G + j) * ROWB + (size_t)lr * EPL * T::kBytes), x);
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            S.qpos[j][q_slot<T>(lr, e)] = (double)fmaxf(x[e], 0.f);
            S.qneg[j][q_slot<T>(lr, e)] = (double)fminf(x[e], 0.f);
            S.qall[j][q_slot<T>(lr, e)] = (double)x[e];
        }
    }
    for (int i = tid; i < 256; i += kTreeThreads) S.hist[i] = 0;
    if (mfma && wave < NLOAD) {
        // wave i converts the 16-byte pieces i of the queries: lane (head, block, channel quarter)
        const int a_head = lane & 3, kq = lane >> 4, i = wave;
        const bool a_min = ((lane >> 2) & 3) >= 2;
        float x[EPL];
        unpack<T>(load16(q, ((size_t)b * n_kv_heads * G + (size_t)h * G + min(a_head, G - 1)) * ROWB + 64 * i + 16 * kq), x);
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            const float xe = (a_head < G) ? x[e] : 0.f;
            const float pos = fmaxf(xe, 0.f), neg = fminf(xe, 0.f);
            A.qa[i * EPL + e][lane] = (double)(a_min ? neg : pos);
            A.qb[i * EPL + e][lane] = (double)(a_min ? pos : neg);
        }
    }
    __syncthreads();

    // ---- initial chunks: bounds from the abstract rows (kmax row, kmin row) ----------
    if (mfma) {
        // eight chunks per wave and pass, kNodePasses passes in flight: lane (r, kq) reads its pieces of
        // row 2 c + (r >> 3) of chunk c = c0 + 8 p + (r & 7) - the chunk's kmax row or its kmin row
        for (int c0 = wave * 8 * kNodePasses; c0 < m0; c0 += kTreeWaves * 8 * kNodePasses) {
            uint4 v[kNodePasses][1][NLOAD];
#pragma unroll
            for (int p = 0; p < kNodePasses; ++p) {
                const int c = min(c0 + 8 * p + (lane & 7), m0 - 1);
                tree_fetch_node<T, 1>(Abh + ((size_t)2 * c + ((lane >> 3) & 1)) * ROWB, 1, v[p]);
            }
#pragma unroll
            for (int p = 0; p < kNodePasses; ++p) {
                const int c = c0 + 8 * p + lane;
                TreeNode nd;
                tree_nodes8<T, 1>(v[p], A, G, &nd.U, &nd.L);
                if (lane < 8 && c < m0) {
                    nd.start = c * chunk_size;
                    nd.size = min(chunk_size, n_ctx - c * chunk_size);
                    cur[c] = nd;
                }
            }
        }
    } else
    for (int c0 = wave * (LEOAM_WAVE / LPR); c0 < m0; c0 += kGroups) {      // uniform over the wave
        const int c = min(c0 + gid % (LEOAM_WAVE / LPR), m0 - 1);
        float U, L;
        tree_eval<T>(Abh + (size_t)c * 2 * ROWB, 2, S.qpos, S.qneg, S.qall, G, &U, &L);
        if (g_lead) {        // (a clamped group repeats the last chunk's store)
            TreeNode nd;
            nd.start = c * chunk_size;
            nd.size = min(chunk_size, n_ctx - c * chunk_size);
            nd.U = U;
            nd.L = L;
            cur[c] = nd;
        }
    }
    __syncthreads();

    int n = m0, evals = m0, status = 0;
    float v = 0.f, mu = 0.f;
    // The list is walked in tiles of kTreeTile nodes, kTreeCache consecutive nodes per thread.
    // The first tile's nodes are read once per round and kept in registers; a longer list
    // re-reads the other tiles from memory in every pass.
    TreeNode cn[kTreeCache];
    auto for_nodes = [&](auto&& body) {
#pragma unroll
        for (int j = 0; j < kTreeCache; ++j) {
            const int i = tid * kTreeCache + j;
            if (i < n) body(i, cn[j]);
        }
        for (int base = kTreeTile; base < n; base += kTreeTile)
#pragma unroll
            for (int j = 0; j < kTreeCache; ++j) {
                const int i = base + tid * kTreeCache + j;
                if (i < n) body(i, cur[i]);
            }
    };
    // Token-weighted k-th largest key of the list (every thread gets it).  The histogram is
    // all zero on entry and on return.
    auto kth_largest = [&](auto&& key_of) -> uint32_t {
        uint32_t lo = 0xffffffffu, hi = 0;
        for_nodes([&](int, const TreeNode& nd) {
            const uint32_t k = key_of(nd);
            lo = min(lo, k);
            hi = max(hi, k);
        });
        lo = wave_min_u32(lo);
        hi = wave_max_u32(hi);
        if (tid == 0) {
            S.key_lo = 0xffffffffu;
            S.key_hi = 0;
            S.rank = (uint32_t)k_tokens;
        }
        __syncthreads();
        if (lane == 0) {
            atomicMin(&S.key_lo, lo);
            atomicMax(&S.key_hi, hi);
        }
        __syncthreads();
        lo = S.key_lo;
        hi = S.key_hi;
        int bits = (lo ^ hi) ? 32 - __clz((int)(lo ^ hi)) : 0;      // bits below the prefix all keys share
        uint32_t prefix = (uint32_t)(((uint64_t)hi >> bits) << bits);
        while (bits > 0) {
            const int w = min(bits, 8), shift = bits - w;
            // (neighbouring nodes often fall into one bin - a desert's chunks have nearly the same bound -
            // and 64 lanes adding to one LDS word take 64 turns: a thread folds its consecutive nodes of
            // one bin into a single add)
            uint32_t run_bin = 0, run_weight = 0;
            for_nodes([&](int, const TreeNode& nd) {
                const uint32_t k = key_of(nd);
                if ((uint32_t)((uint64_t)(k ^ prefix) >> bits) == 0) {
                    const uint32_t bin = (k >> shift) & ((1u << w) - 1u);
                    if (run_weight != 0 && bin != run_bin) {
                        atomicAdd(&S.hist[run_bin], run_weight);
                        run_weight = 0;
                    }
                    run_bin = bin;
                    run_weight += (uint32_t)nd.size;
                }
            });
            if (run_weight != 0) atomicAdd(&S.hist[run_bin], run_weight);
            __syncthreads();
            if (wave == 0) {
                // lane l owns bins 4l..4l+3 (and clears them); walk from the top bin down
                uint32_t hb[4], lane_sum = 0;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    hb[t] = S.hist[4 * lane + t];
                    S.hist[4 * lane + t] = 0;
                    lane_sum += hb[t];
                }
                const uint32_t incl = wave_incl_scan_u32(lane_sum);
                const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, LEOAM_WAVE - 1);
                uint32_t above = total - incl;                // weight of the bins above this lane's bins
                const uint32_t rank = S.rank;
                int found = -1;
                uint32_t above_found = 0;
#pragma unroll
                for (int t = 3; t >= 0; --t) {
                    if (found < 0 && above < rank && rank <= above + hb[t]) {
                        found = 4 * lane + t;
                        above_found = above;
                    }
                    above += hb[t];
                }
                if (found >= 0) {       // exactly one lane: the totals reach the rank
                    S.digit = (uint32_t)found;
                    S.rank = rank - above_found;
                }
            }
            __syncthreads();
            prefix |= S.digit << shift;
            bits = shift;
        }
        return prefix;
    };

    for (int round = 0;; ++round) {
#pragma unroll
        for (int j = 0; j < kTreeCache; ++j) cn[j] = cur[min(tid * kTreeCache + j, n - 1)];
        // ---- v = k-th largest U (token-weighted) -----------------------------------------
        const uint32_t key_v = kth_largest([](const TreeNode& nd) { return tree_key(nd.U); });
        v = tree_unkey(key_v);
        // ---- mu = (k+1)-th largest U: each wave folds its lanes, then one atomic per wave -----
        if (tid == 0) {
            S.ge_weight = 0;
            S.below_key = 0;
            S.below_any = 0;
        }
        __syncthreads();
        {
            uint32_t ge = 0, below = 0, any = 0;
            for_nodes([&](int, const TreeNode& nd) {
                const uint32_t ku = tree_key(nd.U);
                if (ku >= key_v) {
                    ge += (uint32_t)nd.size;
                } else {
                    below = max(below, ku);
                    any = 1;
                }
            });
            const uint32_t ge_w =
                (uint32_t)__builtin_amdgcn_readlane((int)wave_incl_scan_u32(ge), LEOAM_WAVE - 1);
            const uint32_t below_w = wave_max_u32(below);
            const bool any_w = __ballot(any != 0) != 0;
            if (lane == 0) {
                if (ge_w) atomicAdd(&S.ge_weight, ge_w);
                if (any_w) {
                    atomicMax(&S.below_key, below_w);
                    S.below_any = 1;
                }
            }
        }
        __syncthreads();
        mu = ((uint32_t)k_tokens + 1u <= S.ge_weight) ? v : (S.below_any ? tree_unkey(S.below_key) : -INFINITY);
        if (round >= max_rounds) break;

        // ---- which nodes are split, and where everything goes --------------------------
        auto is_split = [&](const TreeNode& nd) { return nd.U >= v && !(nd.L > mu) && nd.size > 1; };
        // (a thread's nodes are consecutive: positions = scan of the threads' widths + a running sum)
        // Unsplit nodes move to their new place; split nodes are listed as tasks, in two classes: nodes of
        // two tokens (both halves are single tokens, which the evaluation handles with one dot product
        // per head) fill the task list from the front, all others from the back, so that a wave's lane
        // groups work on nodes of one kind.  Everything is written while the tiles are scanned (a position
        // is final once the tiles before it are counted); should the round turn out not to fit node_cap,
        // the writes - kept inside the buffers - are simply abandoned.
        const int task_cap = (node_cap + 1) / 2;
        uint32_t carry = 0, carry_two = 0;
        auto scan_tile = [&](int base, auto&& node_of) {
            uint32_t local[kTreeCache], local_two[kTreeCache], width = 0, n_two = 0;
#pragma unroll
            for (int j = 0; j < kTreeCache; ++j) {
                const int i = base + tid * kTreeCache + j;
                local[j] = width;
                local_two[j] = n_two;
                if (i < n) {
                    const TreeNode nd = node_of(i, j);
                    const bool sp = is_split(nd);
                    width += sp ? 2u : 1u;
                    n_two += (sp && nd.size == 2) ? 1u : 0u;
                }
            }
            uint32_t total, total_two;
            const uint32_t before = carry + tree_block_scan(width, S.wave_tot, &total);
            const uint32_t before_two = carry_two + tree_block_scan(n_two, S.wave_tot, &total_two);
#pragma unroll
            for (int j = 0; j < kTreeCache; ++j) {
                const int i = base + tid * kTreeCache + j;
                if (i < n) {
                    const TreeNode nd = node_of(i, j);
                    const int p = (int)(before + local[j]);
                    if (is_split(nd)) {
                        // (position - index = number of splits before the node)
                        const int twos = (int)(before_two + local_two[j]), others = (p - i) - twos;
                        const int slot = nd.size == 2 ? twos : task_cap - 1 - others;
                        TreeTask tk;
                        tk.start = nd.start;
                        tk.size = nd.size;
                        tk.pos = p;
                        tk.pad = 0;
                        if (slot >= 0 && slot < task_cap) task[slot] = tk;
                    } else if (p < node_cap) {
                        nxt[p] = nd;
                    }
                }
            }
            carry += total;
            carry_two += total_two;
        };
        scan_tile(0, [&](int, int j) -> const TreeNode& { return cn[j]; });
        for (int base = kTreeTile; base < n; base += kTreeTile) scan_tile(base, [&](int i, int) { return cur[i]; });
        const int n_new = (int)carry, n_split = n_new - n, n_two = (int)carry_two;
        if (n_split == 0) break;
        if (n_new > node_cap) {
            status = 1;
            break;
        }
        __syncthreads();
        // ---- a lane group takes one half of a listed node and evaluates it from its keys; the
        // next task's entry is fetched before the evaluation ----------------------------------
        // (the loops are uniform over the wave: a lane group past the end evaluates row 0 and stores nothing)
        auto eval_class = [&](int count, auto&& task_at) {
            constexpr int kGroupsPerWave = LEOAM_WAVE / LPR;
            if (count == 0) return;
            TreeTask tk = task_at(min(gid >> 1, count - 1));
            for (int t0 = wave * kGroupsPerWave; t0 < 2 * count; t0 += kGroups) {
                const int t = t0 + gid % kGroupsPerWave;
                const bool live = t < 2 * count;
                const TreeTask nx = task_at(min((t + kGroups) >> 1, count - 1));
                const int second = t & 1, left = (tk.size + 1) / 2;
                TreeNode c;
                c.start = live ? (second ? tk.start + left : tk.start) : 0;
                c.size = live ? (second ? tk.size - left : left) : 1;
                tree_eval<T>(Kbh + (size_t)c.start * ROWB, c.size, S.qpos, S.qneg, S.qall, G, &c.U, &c.L);
                if (g_lead && live) nxt[tk.pos + second] = c;
                tk = nx;
            }
        };
        if (mfma) {
            // the halves of the two-token nodes: token t of the class belongs to task t >> 1
            const int total = 2 * n_two;
            for (int t0 = wave * 16 * kTokenPasses; t0 < total; t0 += kTreeWaves * 16 * kTokenPasses) {
                uint4 v[kTokenPasses][NLOAD];
                int row[kTokenPasses], put[kTokenPasses];
#pragma unroll
                for (int p = 0; p < kTokenPasses; ++p) {
                    const int t = t0 + 16 * p + (lane & 15);
                    const TreeTask tk = task[min(t >> 1, n_two - 1)];
                    row[p] = t < total ? tk.start + (t & 1) : 0;
                    put[p] = t < total ? tk.pos + (t & 1) : -1;
                }
#pragma unroll
                for (int p = 0; p < kTokenPasses; ++p) tree_fetch_row<T>(Kbh + (size_t)row[p] * ROWB, v[p]);
#pragma unroll
                for (int p = 0; p < kTokenPasses; ++p) {
                    TreeNode c;
                    c.U = tree_tokens16<T>(v[p], A, G);
                    c.L = c.U;
                    c.start = row[p];
                    c.size = 1;
                    if (lane < 16 && put[p] >= 0) nxt[put[p]] = c;
                }
            }
        } else {
            eval_class(n_two, [&](int k) { return task[k]; });
        }
        eval_class(n_split - n_two, [&](int k) { return task[task_cap - 1 - k]; });
        __syncthreads();
        TreeNode* tmp = cur;
        cur = nxt;
        nxt = tmp;
        n = n_new;
        evals += 2 * n_split;
    }
    // lambda = k-th largest L of the final list (cn still holds this thread's nodes of it)
    const float lambda = tree_unkey(kth_largest([](const TreeNode& nd) { return tree_key(nd.L); }));

    // ---- final partition: runs of confirmed chunks and runs of unimportant chunks merge ---
    int32_t* off = ref_off + bh * (size_t)(node_cap + 1);
    uint32_t* keys = reinterpret_cast<uint32_t*>(ref_score + bh * (size_t)node_cap);
    auto kind_of = [&](const TreeNode& nd) { return (nd.L > mu) ? 1 : (nd.U < lambda ? 2 : 0); };
    __syncthreads();
    if (tid == 0) S.carry = 0;
    __syncthreads();
    // a thread takes kTreeCache consecutive nodes: one scan of the threads' head counts per tile
    for (int base = 0; base < n; base += kTreeTile) {
        const int i0 = base + tid * kTreeCache;
        TreeNode nd[kTreeCache];
#pragma unroll
        for (int j = 0; j < kTreeCache; ++j) nd[j] = cur[min(i0 + j, n - 1)];
        int kind_prev = (i0 > 0 && i0 < n) ? kind_of(cur[i0 - 1]) : 0;
        uint32_t heads_upto[kTreeCache], width = 0;
        bool head[kTreeCache];
#pragma unroll
        for (int j = 0; j < kTreeCache; ++j) {
            const int i = i0 + j, kind = kind_of(nd[j]);
            head[j] = i < n && !(i > 0 && kind != 0 && kind == kind_prev);
            width += head[j] ? 1u : 0u;
            heads_upto[j] = width;
            kind_prev = kind;
        }
        uint32_t total;
        const uint32_t before = S.carry + tree_block_scan(width, S.wave_tot, &total);
#pragma unroll
        for (int j = 0; j < kTreeCache; ++j) {
            const int i = i0 + j;
            if (i < n && head[j]) {
                const int p = (int)(before + heads_upto[j]) - 1;       // the chunk this node opens
                off[p] = nd[j].start;
                keys[p] = tree_key(kind_of(nd[j]) == 1 ? FLT_MAX : nd[j].U);
            }
        }
        __syncthreads();      // the heads' keys are in place (a run may have begun in an earlier tile)
        // an unimportant run carries the largest U of its nodes: a thread folds its consecutive nodes of
        // one run first (most of a thread's nodes share a run: one atomic instead of eight on one address)
        {
            int run_p = -1;
            uint32_t run_key = 0;
#pragma unroll
            for (int j = 0; j < kTreeCache; ++j) {
                const int i = i0 + j;
                if (i < n && !head[j] && kind_of(nd[j]) == 2) {
                    const int p = (int)(before + heads_upto[j]) - 1;
                    const uint32_t k = tree_key(nd[j].U);
                    if (p != run_p) {
                        if (run_p >= 0) atomicMax(&keys[run_p], run_key);
                        run_p = p;
                        run_key = k;
                    } else {
                        run_key = max(run_key, k);
                    }
                }
            }
            if (run_p >= 0) atomicMax(&keys[run_p], run_key);
        }
        if (tid == 0) S.carry += total;
        __syncthreads();
    }
    const int n_out = (int)S.carry;
    __syncthreads();
    for (int i = tid; i < n_out; i += kTreeThreads) ref_score[bh * (size_t)node_cap + i] = tree_unkey(keys[i]);
    if (tid == 0) {
        off[n_out] = n_ctx;
        ref_count[bh] = n_out;
        ref_evals[bh] = evals;
        ref_status[bh] = status;
    }
}

size_t tree_workspace_bytes(const leoam_shape* s, int node_cap) {
    // two node lists and the task list (a split adds a node, so at most node_cap / 2 per round)
    return (size_t)s->batch * s->n_kv_heads *
           ((size_t)node_cap * 2 * sizeof(TreeNode) + (size_t)((node_cap + 1) / 2) * sizeof(TreeTask));
}

hipError_t tree_refine_dispatch(const leoam_shape* s, const void* q, const void* K, const void* abstract,
                                int chunk_size, int k_tokens, int max_rounds, int node_cap, int32_t* ref_off,
                                float* ref_score, int32_t* ref_count, int32_t* ref_evals, int32_t* ref_status,
                                void* workspace, hipStream_t stream) {
    const size_t units = (size_t)s->batch * s->n_kv_heads;
    TreeNode* a = (TreeNode*)workspace;
    TreeNode* b = a + units * (size_t)node_cap;
    TreeTask* task = (TreeTask*)(b + units * (size_t)node_cap);
    dim3 grid(s->n_kv_heads, s->batch), block(kTreeThreads);
    const int G = s->n_q_heads / s->n_kv_heads;
#define LEOAM_TREE(TT)                                                                                           \
    hipLaunchKernelGGL(tree_refine_kernel<TT>, grid, block, 0, stream, (const char*)q, (const char*)K,            \
                       (const char*)abstract, chunk_size, k_tokens, max_rounds, node_cap, ref_off, ref_score,    \
                       ref_count, ref_evals, ref_status, a, b, task, s->n_ctx, s->c_max, s->n_kv_heads, G)
    switch (s->kv_dtype) {
    case LEOAM_F32: LEOAM_TREE(F32); break;
    case LEOAM_F16: LEOAM_TREE(F16); break;
    default: LEOAM_TREE(BF16); break;
    }
#undef LEOAM_TREE
    return hipGetLastError();
}

}  // namespace leoam
