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
// They are found without sorting: a radix descent (four 8-bit passes over the
// order-preserving integer image of the floats, token-weighted histograms in
// LDS) for v and lambda together; mu is v if the chunks with U >= v hold more
// than k tokens, else the largest U below v.
//
// One 1024-lane workgroup per (sequence, kv head) runs every round; the node
// list (start, size, U, L) lives in the workspace, double-buffered, in position
// order (a split node is replaced by its two halves at scanned positions).  A
// lane group as wide as a key row evaluates a node - element-wise max / min over
// its key rows (the two abstract rows for an initial chunk), then the bounds in
// double, rounded once to float - so a wave has 4 (fp32: 2) nodes in flight.
// Latency-bound, exact integer bookkeeping.
#include <cfloat>
#include <type_traits>

#include "leoam_dev.h"

namespace leoam {

constexpr int kTreeThreads = 1024;
constexpr int kTreeCache = 8;          // nodes per thread held in registers through a round
constexpr int kTreeWaves = kTreeThreads / LEOAM_WAVE;
constexpr int kTreeMaxG = 8;

struct TreeNode {
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
    double qpos[kTreeMaxG][LEOAM_D], qneg[kTreeMaxG][LEOAM_D];      // max(q, 0) and min(q, 0)
    uint32_t hist[2][256];
    uint32_t wave_tot[kTreeWaves];
    uint32_t prefix[2], rank[2];
    uint32_t ge_weight, below_key, below_any;
    uint32_t carry;
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

// sum of a double over the lanes of a group of kLanes (16 or 32) lanes; every lane gets it
template <int kLanes> __device__ __forceinline__ double group_sum_d(double v) {
    auto step = [&](auto ctrl) {
        constexpr int kCtrl = decltype(ctrl)::value;
        const uint64_t u = __builtin_bit_cast(uint64_t, v);
        const int lo = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)u, kCtrl, 0xf, 0xf, false);
        const int hi = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)(u >> 32), kCtrl, 0xf, 0xf, false);
        v += __builtin_bit_cast(double, ((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
    };
    step(std::integral_constant<int, 0xB1>{});       // xor 1
    step(std::integral_constant<int, 0x4E>{});       // xor 2
    step(std::integral_constant<int, 0x141>{});      // mirror inside 8 lanes
    step(std::integral_constant<int, 0x140>{});      // mirror inside 16 lanes
    if (kLanes == 32) v += shfl_xor_d(v, 16);
    return v;
}

// A lane group (the lanes that cover one key row: 16 for 16-bit keys, 32 for fp32)
// computes the bounds of one node: max / min over `n_rows` rows starting at `rows`,
// then U = max_j sum_d max(q k_max, q k_min) and L = max_j sum_d min(..), each sum
// in double, rounded once to float.  A wave evaluates 4 (2) nodes at a time.
template <typename T>
__device__ __forceinline__ void tree_eval(const char* rows, int n_rows, const double (*qpos)[LEOAM_D],
                                          const double (*qneg)[LEOAM_D], int G, float* U, float* L) {
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
    // eight rows in flight; a row index past the end re-reads the last row (harmless for max / min,
    // and the loads stay unconditional)
    constexpr int kBatch = 8;
    if (n_rows <= 2) {          // an initial chunk: its kmax row and its kmin row
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            float x[EPL];
            unpack<T>(load16(rows, (size_t)min(j, n_rows - 1) * ROWB + (size_t)col * T::kBytes), x);
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                mx[e] = fmaxf(mx[e], x[e]);
                mn[e] = fminf(mn[e], x[e]);
            }
        }
    } else
    for (int r0 = 0; r0 < n_rows; r0 += kBatch) {
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
    }
    float ub = -INFINITY, lb = -INFINITY;
    for (int j = 0; j < G; ++j) {
        // max(q k_max, q k_min) = max(q,0) k_max + min(q,0) k_min (k_max >= k_min): one of the two
        // products is zero and every product is exact in double.  Four independent chains.
        double u0 = 0.0, u1 = 0.0, l0 = 0.0, l1 = 0.0;
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            const double qp = qpos[j][e * LPR + lane_in_row], qn = qneg[j][e * LPR + lane_in_row];
            const double hi = (double)mx[e], lo = (double)mn[e];
            u0 = fma(qp, hi, u0);
            u1 = fma(qn, lo, u1);
            l0 = fma(qp, lo, l0);
            l1 = fma(qn, hi, l1);
        }
        double u = u0 + u1, l = l0 + l1;
        u = group_sum_d<LPR>(u);
        l = group_sum_d<LPR>(l);
        ub = fmaxf(ub, (float)u + 0.0f);
        lb = fmaxf(lb, (float)l + 0.0f);
    }
    *U = ub;
    *L = lb;
}

template <typename T>
__global__ __launch_bounds__(kTreeThreads) void tree_refine_kernel(
    const char* __restrict__ q, const char* __restrict__ K, const char* __restrict__ abstract, int chunk_size,
    int k_tokens, int max_rounds, int node_cap, int32_t* __restrict__ ref_off, float* __restrict__ ref_score,
    int32_t* __restrict__ ref_count, int32_t* __restrict__ ref_evals, int32_t* __restrict__ ref_status,
    TreeNode* nodes_a, TreeNode* nodes_b, int32_t* pos_buf, int32_t* task_buf, int n_ctx, int c_max, int n_kv_heads, int G) {
    constexpr int ROWB = Row<T>::kRowBytes;
    constexpr int EPL = T::kEpl;
    __shared__ TreeLds S;

    const int h = blockIdx.x, b = blockIdx.y;
    const size_t bh = (size_t)b * n_kv_heads + h;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid / LEOAM_WAVE;
    const int m0 = (n_ctx + chunk_size - 1) / chunk_size;
    TreeNode* cur = nodes_a + bh * (size_t)node_cap;
    TreeNode* nxt = nodes_b + bh * (size_t)node_cap;
    int32_t* pos = pos_buf + bh * (size_t)node_cap;
    int32_t* task = task_buf + bh * (size_t)node_cap;
    constexpr int LPR = Row<T>::kLanesPerRow;
    constexpr int kGroups = kTreeThreads / LPR;              // node evaluations in flight per workgroup
    const int gid = tid / LPR;
    const bool g_lead = (tid % LPR) == 0;
    const char* Kbh = K + bh * (size_t)n_ctx * ROWB;
    const char* Abh = abstract + bh * (size_t)c_max * 2 * ROWB;

    // ---- queries of the group in double ------------------------------------------
    for (int i = tid; i < G * (LEOAM_D / EPL); i += kTreeThreads) {
        const int j = i / (LEOAM_D / EPL), c = (i % (LEOAM_D / EPL)) * EPL;
        float x[EPL];
        unpack<T>(load16(q, ((size_t)b * n_kv_heads * G + (size_t)h * G + j) * ROWB + (size_t)c * T::kBytes), x);
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            // channel c + e sits at [e][c / EPL]: the lanes of a row then read consecutive doubles
            S.qpos[j][e * (LEOAM_D / EPL) + c / EPL] = (double)fmaxf(x[e], 0.f);
            S.qneg[j][e * (LEOAM_D / EPL) + c / EPL] = (double)fminf(x[e], 0.f);
        }
    }
    __syncthreads();

    // ---- initial chunks: bounds from the abstract rows (kmax row, kmin row) ----------
    for (int c = gid; c < m0; c += kGroups) {
        float U, L;
        tree_eval<T>(Abh + (size_t)c * 2 * ROWB, 2, S.qpos, S.qneg, G, &U, &L);
        if (g_lead) {
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
    float v = 0.f, mu = 0.f, lambda = 0.f;
    for (int round = 0;; ++round) {
        // ---- this thread's nodes (tid, tid + 1024, ...) are read once per round; lists longer
        // than kTreeCache * 1024 nodes re-read the rest from memory in every pass ------------
        TreeNode cn[kTreeCache];
#pragma unroll
        for (int j = 0; j < kTreeCache; ++j) cn[j] = cur[min(tid + j * kTreeThreads, n - 1)];
        auto for_nodes = [&](auto&& body) {
#pragma unroll
            for (int j = 0; j < kTreeCache; ++j) {
                const int i = tid + j * kTreeThreads;
                if (i < n) body(i, cn[j]);
            }
            for (int i = tid + kTreeCache * kTreeThreads; i < n; i += kTreeThreads) body(i, cur[i]);
        };
        // ---- v = k-th largest U and lambda = k-th largest L (token-weighted) ---------
        if (tid < 2) {
            S.prefix[tid] = 0;
            S.rank[tid] = (uint32_t)k_tokens;
        }
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            for (int i = tid; i < 512; i += kTreeThreads) S.hist[i >> 8][i & 255] = 0;
            __syncthreads();
            const uint32_t pu = S.prefix[0], pl = S.prefix[1];
            for_nodes([&](int, const TreeNode& nd) {
                const uint32_t ku = tree_key(nd.U), kl = tree_key(nd.L);
                if (pass == 0 || (ku >> (shift + 8)) == (pu >> (shift + 8)))
                    atomicAdd(&S.hist[0][(ku >> shift) & 255], (uint32_t)nd.size);
                if (pass == 0 || (kl >> (shift + 8)) == (pl >> (shift + 8)))
                    atomicAdd(&S.hist[1][(kl >> shift) & 255], (uint32_t)nd.size);
            });
            __syncthreads();
            if (wave < 2) {
                // lane l owns bins 4l..4l+3; walk from the top bin down
                const uint32_t* hs = S.hist[wave];
                uint32_t hb[4], lane_sum = 0;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    hb[t] = hs[4 * lane + t];
                    lane_sum += hb[t];
                }
                const uint32_t incl = wave_incl_scan_u32(lane_sum);
                const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, LEOAM_WAVE - 1);
                uint32_t above = total - incl;                // weight of the bins above this lane's bins
                const uint32_t rank = S.rank[wave];
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
                    S.prefix[wave] |= (uint32_t)found << shift;
                    S.rank[wave] = rank - above_found;
                }
            }
            __syncthreads();
        }
        const uint32_t key_v = S.prefix[0];
        v = tree_unkey(key_v);
        lambda = tree_unkey(S.prefix[1]);
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
        if (tid == 0) S.carry = 0;
        __syncthreads();
        auto is_split = [&](const TreeNode& nd) { return nd.U >= v && !(nd.L > mu) && nd.size > 1; };
        auto scan_tile = [&](int i, const TreeNode& nd) {
            const uint32_t width = i < n ? (is_split(nd) ? 2u : 1u) : 0u;
            uint32_t total;
            const uint32_t before = tree_block_scan(width, S.wave_tot, &total);
            const uint32_t carry = S.carry;
            if (i < n) pos[i] = (int32_t)(carry + before);
            __syncthreads();
            if (tid == 0) S.carry = carry + total;
            __syncthreads();
        };
#pragma unroll
        for (int j = 0; j < kTreeCache; ++j)
            if (j * kTreeThreads < n) scan_tile(tid + j * kTreeThreads, cn[j]);
        for (int base = kTreeCache * kTreeThreads; base < n; base += kTreeThreads)
            scan_tile(base + tid, cur[min(base + tid, n - 1)]);
        const int n_new = (int)S.carry, n_split = n_new - n;
        if (n_split == 0) break;
        if (n_new > node_cap) {
            status = 1;
            break;
        }
        // ---- unsplit nodes move to their new place; split nodes are listed -----------------
        // (pos[i] - i = number of splits before node i = its slot in the list)
        for_nodes([&](int i, const TreeNode& nd) {
            const int p = pos[i];
            if (is_split(nd)) task[p - i] = i;
            else nxt[p] = nd;
        });
        __syncthreads();
        // ---- a lane group takes one half of a listed node and evaluates it from its keys -----
        for (int t = gid; t < 2 * n_split; t += kGroups) {
            const int parent = task[t >> 1], second = t & 1;
            const TreeNode nd = cur[parent];
            const int left = (nd.size + 1) / 2;
            TreeNode c;
            c.start = second ? nd.start + left : nd.start;
            c.size = second ? nd.size - left : left;
            tree_eval<T>(Kbh + (size_t)c.start * ROWB, c.size, S.qpos, S.qneg, G, &c.U, &c.L);
            if (g_lead) nxt[pos[parent] + second] = c;
        }
        __syncthreads();
        TreeNode* tmp = cur;
        cur = nxt;
        nxt = tmp;
        n = n_new;
        evals += 2 * n_split;
    }

    // ---- final partition: runs of confirmed chunks and runs of unimportant chunks merge ---
    int32_t* off = ref_off + bh * (size_t)(node_cap + 1);
    uint32_t* keys = reinterpret_cast<uint32_t*>(ref_score + bh * (size_t)node_cap);
    auto kind_of = [&](const TreeNode& nd) { return (nd.L > mu) ? 1 : (nd.U < lambda ? 2 : 0); };
    __syncthreads();
    if (tid == 0) S.carry = 0;
    __syncthreads();
    for (int base = 0; base < n; base += kTreeThreads) {
        const int i = base + tid;
        uint32_t head = 0;
        TreeNode nd;
        int kind = 0;
        if (i < n) {
            nd = cur[i];
            kind = kind_of(nd);
            head = 1;
            if (i > 0 && kind != 0) {
                const TreeNode pv = cur[i - 1];
                if (kind_of(pv) == kind) head = 0;
            }
        }
        uint32_t total;
        const uint32_t before = tree_block_scan(head, S.wave_tot, &total);
        const uint32_t carry = S.carry;
        if (i < n) {
            const int p = (int)(carry + before) - (head ? 0 : 1);       // the chunk this node belongs to
            pos[i] = p;
            if (head) {
                off[p] = nd.start;
                keys[p] = tree_key(kind == 1 ? FLT_MAX : nd.U);
            }
        }
        __syncthreads();
        if (tid == 0) S.carry = carry + total;
        __syncthreads();
    }
    const int n_out = (int)S.carry;
    // (a run may cross a tile boundary: the first node of the next tile then is no head and joins it)
    for (int i = tid; i < n; i += kTreeThreads) {
        const TreeNode nd = cur[i];
        if (kind_of(nd) == 2) atomicMax(&keys[pos[i]], tree_key(nd.U));
    }
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
    return (size_t)s->batch * s->n_kv_heads * (size_t)node_cap * (2 * sizeof(TreeNode) + 2 * sizeof(int32_t));
}

hipError_t tree_refine_dispatch(const leoam_shape* s, const void* q, const void* K, const void* abstract,
                                int chunk_size, int k_tokens, int max_rounds, int node_cap, int32_t* ref_off,
                                float* ref_score, int32_t* ref_count, int32_t* ref_evals, int32_t* ref_status,
                                void* workspace, hipStream_t stream) {
    const size_t units = (size_t)s->batch * s->n_kv_heads;
    TreeNode* a = (TreeNode*)workspace;
    TreeNode* b = a + units * (size_t)node_cap;
    int32_t* pos = (int32_t*)(b + units * (size_t)node_cap);
    int32_t* task = pos + units * (size_t)node_cap;
    dim3 grid(s->n_kv_heads, s->batch), block(kTreeThreads);
    const int G = s->n_q_heads / s->n_kv_heads;
#define LEOAM_TREE(TT)                                                                                           \
    hipLaunchKernelGGL(tree_refine_kernel<TT>, grid, block, 0, stream, (const char*)q, (const char*)K,            \
                       (const char*)abstract, chunk_size, k_tokens, max_rounds, node_cap, ref_off, ref_score,    \
                       ref_count, ref_evals, ref_status, a, b, pos, task, s->n_ctx, s->c_max, s->n_kv_heads, G)
    switch (s->kv_dtype) {
    case LEOAM_F32: LEOAM_TREE(F32); break;
    case LEOAM_F16: LEOAM_TREE(F16); break;
    default: LEOAM_TREE(BF16); break;
    }
#undef LEOAM_TREE
    return hipGetLastError();
}

}  // namespace leoam
