// chunk_select_attention_decode: the selection (paper Sec. 4.2 / 6.1) and the
// attention over the kept chunks (Sec. 2.1 Eq. 1, Sec. 4.1 workflow) of a decode
// step in ONE launch, for 16-bit keys / values.
//
// The two steps are short, dependent and latency-bound at decode batch sizes: as
// separate launches they pay a launch gap, a round trip of the kept list through
// memory, and a third small launch that combines the attention splits.  Here a
// 1024-lane workgroup runs the selection of its (sequence, kv head) (the same
// code as chunk_topk_select), leaves the kept chunks' token ranges in LDS, and
// its sixteen waves then stream their shares of the kept tokens.  When a
// (sequence, kv head) is spread over several workgroups ("splits") every one of
// them repeats the selection - it reads only the score row, which the second
// reader finds in L2 - and takes its own range of the kept tokens.
//
// Splits are combined in the same launch by the workgroup that finishes last:
// each split publishes its partial (m, l, acc[D]) with agent-scope relaxed atomic
// stores (write-through, no cache write-back), waits for them, and takes a ticket
// from an agent-scope counter; the workgroup that draws the last ticket reads all
// partials with agent-scope atomic loads and folds them in split order, so the
// result does not depend on which workgroup that is.  No workgroup ever waits
// for another.  The counters live in the workspace, are zero between calls and
// are reset by the workgroup that merges.
//
// Streaming: q K^T on v_mfma_f32_16x16x32 with token = row, query head = column
// (as in sparse_attention.hip); P V in fp32 on the vector ALU.  With sixteen
// waves per workgroup a wave has 128 registers: two K/V tiles in flight and the
// accumulators; the queries (the matrix core's B operand) stay in LDS.  Nothing
// else in the tile loop goes through LDS: the running maximum over the four lane
// groups is taken with lane swaps on the vector ALU (two ds_bpermute round trips
// per tile in its place cost the launch 10 % on MI355X, the next tile's loads
// queue behind the same waits).
#include <cstdlib>

#include "fused_tail.h"

namespace leoam {

constexpr int kFusedBlock = 128;                       // tokens a wave maps to rows at a time
constexpr int kFusedGranule = kFusedWaves * 16;        // a split is a multiple of this many tokens
constexpr int kFusedMaxSel = 2048;                     // kept chunks per (b,h) whose ranges fit the LDS tables
constexpr int kFusedMaxSplits = 64;
constexpr int kFusedTargetWgs = 256;                   // one workgroup per compute unit
constexpr size_t kArrivalAlign = 256;

// one 16-token tile of a wave: K operand (4 x 16 B per lane) and V rows (4 x 16 B per lane)
struct FusedKvTile {
    uint4 k[4];
    uint4 v[4];
};

// kGiven: the kept lists (sel_idx, sel_count) are inputs - a selection made earlier, for instance by
// one chunk_topk_select call over all layers of a step - and the workgroup only builds its tables
// from them (two list positions per lane; kIpt is not used).
template <typename T, int G, int kIpt, bool kGiven = false>
__global__ __launch_bounds__(kSelThreads) void select_attention_kernel(
    const float* __restrict__ score, const int32_t* __restrict__ chunk_off, const int32_t* __restrict__ n_chunks,
    int max_chunks, int token_budget, int32_t* __restrict__ sel_idx, int32_t* __restrict__ sel_count,
    int32_t* __restrict__ sel_tokens, const char* __restrict__ q, const char* __restrict__ K,
    const char* __restrict__ V, float scale_log2, float* __restrict__ out, float* __restrict__ lse, float* partial,
    int32_t* arrivals, int n_splits, int c_max, int k_max, int n_kv_heads, int n_ctx, unsigned long long* exchange) {
    constexpr int ROWB = LEOAM_D * 2;
    constexpr int EPL = 8;
    static_assert(G <= 4, "the fused kernel keeps 8 accumulators per head per lane");

    // the three phases use LDS one after the other
    union Phase {
        SelectLds sel;
        int32_t rows[kFusedWaves][kFusedBlock];
        float xw[kFusedWaves][G][kPartStride];
    };
    __shared__ Phase ph;
    __shared__ int32_t start[kFusedMaxSel], prefix[kFusedMaxSel + 1];
    __shared__ uint4 qs[4][LEOAM_WAVE];      // matrix-core B operand (the group's queries), same for every wave
    __shared__ int32_t sh_last;

    const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid / LEOAM_WAVE;
    const int grp = lane >> 4, c16 = lane & 15;
    const size_t bh = (size_t)b * n_kv_heads + h;
    const int C = min(max(n_chunks[b], 0), c_max);
    const int32_t* off = chunk_off + (size_t)b * (c_max + 1);

    // ---- B operand: the group's queries (column = head), zero beyond G.  Fetched by
    // one wave while the selection runs, handed to the others through LDS.
    uint4 qb[4];
    if (wave == 0) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const size_t qrow = ((size_t)b * n_kv_heads * G + (size_t)h * G + min(c16, G - 1)) * ROWB;
            qb[s] = load16(q, qrow + 64 * s + 16 * grp);
        }
    }

    int cnt, total;
    if constexpr (kGiven) {
        // ---- the kept list is given: first token and size of every listed chunk, then a scan --------
        static_assert(kFusedMaxSel == 2 * kSelThreads, "two list positions per lane");
        const int32_t* ids = sel_idx + bh * (size_t)k_max;
        const int listed = min(max(sel_count[bh], 0), k_max);
        int st[2];
        uint32_t sz[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            // (unconditional, clamped loads; an id outside [0, n_chunks) contributes no tokens)
            const int p = 2 * tid + j;
            const int id = ids[min(p, k_max - 1)];
            const bool ok = p < listed && id >= 0 && id < C;
            const int c = ok ? id : 0;
            const int a = min(max(off[c], 0), n_ctx), e = min(max(off[c + 1], a), n_ctx);
            st[j] = a;
            sz[j] = ok ? (uint32_t)(e - a) : 0u;
        }
        uint64_t tot;
        uint32_t before = (uint32_t)block_excl_scan<false>(pack_tot(0, sz[0] + sz[1]), ph.sel.wave_sums2, &tot);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int p = 2 * tid + j;
            if (p < listed) {
                start[p] = st[j];
                prefix[p] = (int32_t)before;
            }
            before += sz[j];
        }
        cnt = listed;
        total = (int)(uint32_t)tot;
        if (tid == 0) prefix[cnt] = total;
        if (wave == 0) {
#pragma unroll
            for (int s = 0; s < 4; ++s) qs[s][lane] = (c16 < G) ? qb[s] : make_uint4(0, 0, 0, 0);
        }
    } else {
        // ---- selection --------------------------------------------------------------
        SelectResult<kIpt> R;
        select_keep<kIpt>(ph.sel, score + bh * (size_t)c_max, off, C, c_max, k_max, n_ctx, max_chunks, token_budget, R);
        cnt = (int)min((uint32_t)(R.kept_total >> 32), (uint32_t)k_max);
        total = (int)(uint32_t)R.kept_total;
        {
            // kept chunks in ascending order: first token and number of kept tokens before it
            int32_t* ids = sel_idx + bh * (size_t)k_max;
            const int c0 = tid * kIpt;
            uint32_t pos = (uint32_t)(R.kept_before >> 32), before = (uint32_t)R.kept_before;
            int tok = R.first_tok;
#pragma unroll
            for (int i = 0; i < kIpt; ++i) {
                if (R.keep[i]) {
                    if (pos < (uint32_t)k_max) {
                        start[pos] = tok;
                        prefix[pos] = (int32_t)before;
                        if (split == 0) ids[pos] = c0 + i;
                    }
                    ++pos;
                    before += R.size[i];
                }
                tok += (int)R.size[i];
            }
            if (tid == 0) prefix[cnt] = total;
            if (wave == 0) {
#pragma unroll
                for (int s = 0; s < 4; ++s) qs[s][lane] = (c16 < G) ? qb[s] : make_uint4(0, 0, 0, 0);
            }
            if (split == 0) {
                for (int i = cnt + tid; i < k_max; i += kSelThreads) ids[i] = -1;
                if (tid == 0) {
                    sel_count[bh] = cnt;
                    if (sel_tokens) sel_tokens[bh] = total;
                }
            }
        }
    }
    __syncthreads();      // tables complete; the selection's LDS is free

    // ---- this workgroup's range of the kept tokens, then this wave's share --------
    int per_split = (total + n_splits - 1) / n_splits;
    per_split = ((per_split + kFusedGranule - 1) / kFusedGranule) * kFusedGranule;
    const int r0 = min(total, split * per_split), r1 = min(total, r0 + per_split);
    const int per_wave = per_split / kFusedWaves;
    const int w0 = min(r1, r0 + wave * per_wave), w1 = min(r1, w0 + per_wave);

    // uniform bases; a lane adds a 32-bit offset (n_ctx * 256 bytes stays far below 4 GiB)
    const char* Kbh = K + bh * (size_t)n_ctx * ROWB;
    const char* Vbh = V + bh * (size_t)n_ctx * ROWB;
    const uint32_t k_lane = 16u * grp, v_lane = 16u * c16;
    int32_t* my_rows = ph.rows[wave];

    // lanes (grp, head) carry the softmax state of `head`; every lane carries the
    // accumulators of all heads for the V rows of its group and its 8 columns
    float m_run = -INFINITY, l_run = 0.f;
    float acc[G][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;

    // Loads are unconditional (a load under a condition is waited for on its own):
    // a position past the end reads row 0, its logit is masked to -inf, its weight is 0.
    auto fetch = [&](int t, FusedKvTile& kv) {
        const int krow = max(my_rows[16 * t + c16], 0);
#pragma unroll
        for (int s = 0; s < 4; ++s) kv.k[s] = load16(Kbh, (size_t)((uint32_t)krow * ROWB + k_lane + 64u * s));
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int vrow = max(my_rows[16 * t + 4 * grp + i], 0);
            kv.v[i] = load16(Vbh, (size_t)((uint32_t)vrow * ROWB + v_lane));
        }
    };
    int q_lane = lane;
    auto logits = [&](const uint4* k) {
        // the B operand is re-read from LDS for every tile: 16 registers a wave cannot spare
        asm volatile("" : "+v"(q_lane));
        f32x4_t sacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < 4; ++s) sacc = mfma_16x16x32<T>(k[s], qs[s][q_lane], sacc);
        return sacc;
    };
    auto accumulate = [&](f32x4_t sacc, const uint4* v, int n_valid) {
        // sacc[r] = logit of token 4grp + r of the tile, head c16
        float z[4];
        float mloc = -INFINITY;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            z[r] = (4 * grp + r < n_valid) ? sacc[r] * scale_log2 : -INFINITY;
            mloc = fmaxf(mloc, z[r]);
        }
        mloc = rows_max4(mloc);
        const float m_new = fmaxf(m_run, mloc);
        const float corr = exp2_or_zero(m_run, m_new);
        const bool changed = (c16 < G) && (m_new > m_run);
        m_run = m_new;
        float psum = 0.f;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            z[r] = exp2_or_zero(z[r], m_new);     // now the weight
            psum += z[r];
        }
        l_run = l_run * corr + psum;
        if (__ballot(changed) != 0ull) {
            // head g's correction factor sits in lane g of every row
            static_for<0, G>([&](auto gc) {
                constexpr int g = decltype(gc)::value;
                const float cg = row_bcast<g>(corr);
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[g][e] *= cg;
            });
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float x[EPL];
            unpack<T>(v[i], x);
            static_for<0, G>([&](auto gc) {
                constexpr int g = decltype(gc)::value;
                const float p = row_bcast<g>(z[i]);
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(p, x[e], acc[g][e]);
            });
        }
    };

    for (int blk = w0; blk < w1; blk += kFusedBlock) {
        const int nb = min(kFusedBlock, w1 - blk);
        // token position in the kept list -> row in the cache, for the whole block
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");      // earlier reads of my_rows are done
        {
            // a lane maps consecutive positions: one search, then a walk
            constexpr int PER = kFusedBlock / LEOAM_WAVE;
            const int i0 = lane * PER;
            int lo = 0;
            if (i0 < nb) {
                const int x = blk + i0;
                int hi = cnt;                  // largest k with prefix[k] <= x
                while (hi - lo > 1) {
                    const int mid = (lo + hi) >> 1;
                    if (prefix[mid] <= x) lo = mid; else hi = mid;
                }
            }
#pragma unroll
            for (int j = 0; j < PER; ++j) {
                int p = -1;
                if (i0 + j < nb) {
                    const int x = blk + i0 + j;
                    while (prefix[lo + 1] <= x) ++lo;      // ends: prefix[cnt] = total > x
                    p = start[lo] + (x - prefix[lo]);
                }
                my_rows[i0 + j] = p;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");      // table visible to the whole wave
        __builtin_amdgcn_wave_barrier();

        const int n_tiles = (nb + 15) >> 4, last = n_tiles - 1;
        FusedKvTile cur, nxt;
        fetch(0, cur);
        if (n_tiles == 1) {
            // a single tile (small batches spread a (b,h) over many workgroups): nothing to prefetch,
            // and the pipeline's re-reads of the last tile would triple the load instructions
            accumulate(logits(cur.k), cur.v, nb);
            continue;
        }
        for (int t = 0; t < n_tiles; t += 2) {
            // (no loads under a condition: a tile index past the end re-reads the last tile)
            fetch(min(t + 1, last), nxt);
            __builtin_amdgcn_sched_barrier(0);       // keep the loads ahead of the tile's arithmetic
            accumulate(logits(cur.k), cur.v, nb - 16 * t);
            fetch(min(t + 2, last), cur);
            __builtin_amdgcn_sched_barrier(0);
            if (t + 1 < n_tiles) accumulate(logits(nxt.k), nxt.v, nb - 16 * (t + 1));
        }
    }

    // ---- fold the four lane groups (same m everywhere in the wave) ---------------
    // four accumulators at a time: afterwards lane group r holds the total of
    // accumulator kRowOwns[r] of the quad, so all 64 lanes write to LDS
    l_run = rows_sum4(l_run, l_run, l_run, l_run);
    const int e_own = ((grp & 1) << 1) | (grp >> 1);        // rows 0,1,2,3 own accumulators 0,2,1,3
    float folded[G][2];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        folded[g][0] = rows_sum4(acc[g][0], acc[g][1], acc[g][2], acc[g][3]);
        folded[g][1] = rows_sum4(acc[g][4], acc[g][5], acc[g][6], acc[g][7]);
    }
    __syncthreads();      // every wave is done with its row table: LDS becomes the exchange buffer
#pragma unroll
    for (int g = 0; g < G; ++g) {
        ph.xw[wave][g][c16 * EPL + e_own] = folded[g][0];
        ph.xw[wave][g][c16 * EPL + 4 + e_own] = folded[g][1];
    }
    if (grp == 0 && c16 < G) {
        ph.xw[wave][c16][LEOAM_D] = m_run;
        ph.xw[wave][c16][LEOAM_D + 1] = l_run;
    }
    __syncthreads();

    fused_tail<G>(ph.xw, sh_last, partial, arrivals, out, lse, bh, split, n_splits, exchange);
}

// zero fill (arrival counters of a fresh workspace)
__global__ void workspace_zero_kernel(uint4* __restrict__ p, size_t n16) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
        p[i] = make_uint4(0, 0, 0, 0);
}

hipError_t workspace_zero_dispatch(void* workspace, size_t bytes, hipStream_t stream) {
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(workspace_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (uint4*)workspace, n16);
    return hipGetLastError();
}

hipError_t topk_select_dispatch(const leoam_shape*, const float*, const int32_t*, const int32_t*, int, int, int32_t*,
                                int32_t*, int32_t*, hipStream_t);
hipError_t attention_dispatch(const leoam_shape*, const void*, const void*, const void*, const void*, const int32_t*,
                              const int32_t*, const int32_t*, const int32_t*, float, float*, float*, void*, size_t,
                              int32_t*, hipStream_t);
size_t attention_workspace_bytes(const leoam_shape*, int);
size_t attention_min_workspace_bytes(const leoam_shape*);

bool select_attention_q_is_fused(const leoam_shape*);
int fused_q_recommended_splits(const leoam_shape*, int);
hipError_t select_attention_q_dispatch(const leoam_shape*, const float*, const void*, const void*, const void*, const void*,
                                       const int32_t*, const int32_t*, int, int, float, int32_t*, int32_t*, int32_t*,
                                       float*, float*, float*, int32_t*, int, hipStream_t);

// LEOAM_STREAM_ORDERED_MERGE=1 in the environment (read once per process) makes the one-call entry points run
// the selection kernel, the attention kernel and the merge kernel back to back instead of the one-launch
// kernels, whose in-launch merge relies on the memory system's behaviour rather than on the memory model.
static bool stream_ordered_merge_wanted() {
    static const bool wanted = [] {
        const char* v = getenv("LEOAM_STREAM_ORDERED_MERGE");
        return v && v[0] && v[0] != '0';
    }();
    return wanted;
}

static inline size_t arrival_bytes(const leoam_shape* s) {
    const size_t n = (size_t)s->batch * s->n_kv_heads * sizeof(int32_t);
    return (n + kArrivalAlign - 1) / kArrivalAlign * kArrivalAlign;
}

static inline size_t fused_part_bytes_per_split(const leoam_shape* s) {
    return (size_t)s->batch * s->n_q_heads * kPartStride * sizeof(float);
}

bool select_attention_is_fused(const leoam_shape* s) {
    const int g = s->n_q_heads / s->n_kv_heads;
    // (the kernel adds 32-bit row offsets to a per-(b,h) base: n_ctx * 256 bytes must stay below 4 GiB)
    return (s->kv_dtype == LEOAM_F16 || s->kv_dtype == LEOAM_BF16) && g <= 4 && s->k_max <= kFusedMaxSel &&
           s->c_max <= 8 * kSelThreads && s->n_ctx < (1 << 24);
}

static int fused_recommended_splits(const leoam_shape* s, int max_tokens) {
    if (max_tokens <= 0 || max_tokens > s->n_ctx) max_tokens = s->n_ctx;
    const int by_tokens = (max_tokens + kFusedGranule - 1) / kFusedGranule;
    const int units = s->batch * s->n_kv_heads;
    int want = (kFusedTargetWgs + units - 1) / units;
    if (want > by_tokens) want = by_tokens;
    if (want > kFusedMaxSplits) want = kFusedMaxSplits;
    if (want < 1) want = 1;
    return want;
}

// Exchange words of the two-split merge (fused_tail.h): one 64-bit word per (b, q head, channel), zero
// between calls like the arrival counters.  Reserved for the batch sizes that give two splits per
// (b, h), i.e. between half a workgroup and one workgroup per compute unit.
static inline size_t exchange_bytes(const leoam_shape* s) {
    const long long units = (long long)s->batch * s->n_kv_heads;
    if (!select_attention_is_fused(s) || (kFusedTargetWgs + units - 1) / units != 2) return 0;
    return (size_t)s->batch * s->n_q_heads * LEOAM_D * sizeof(unsigned long long);
}

// the leading bytes of the workspace that are zero between calls
static inline size_t control_bytes(const leoam_shape* s, bool with_exchange) {
    return arrival_bytes(s) + (with_exchange ? exchange_bytes(s) : 0);
}

// control words, then whichever is larger: the fused kernel's partials or the
// workspace of the two-launch path that shapes outside the fused kernel take
size_t select_attention_workspace_bytes(const leoam_shape* s, int max_tokens, bool with_exchange) {
    size_t body = attention_workspace_bytes(s, max_tokens);
    if (select_attention_is_fused(s)) {
        const size_t f = fused_part_bytes_per_split(s) * (size_t)fused_recommended_splits(s, max_tokens);
        if (f > body) body = f;
    }
    if (select_attention_q_is_fused(s)) {
        const size_t f = fused_part_bytes_per_split(s) * (size_t)fused_q_recommended_splits(s, max_tokens);
        if (f > body) body = f;
    }
    return control_bytes(s, with_exchange) + body;
}

size_t select_attention_counter_bytes(const leoam_shape* s, bool with_exchange) { return control_bytes(s, with_exchange); }

size_t select_attention_min_workspace_bytes(const leoam_shape* s, bool with_exchange) {
    const bool one_launch = (select_attention_is_fused(s) || select_attention_q_is_fused(s)) && !stream_ordered_merge_wanted();
    return control_bytes(s, with_exchange) + (one_launch ? 0 : attention_min_workspace_bytes(s));
}

template <typename T, int G>
static hipError_t launch_fused(const leoam_shape* s, const float* score, const void* q, const void* K, const void* V,
                               const int32_t* chunk_off, const int32_t* n_chunks, int max_chunks, int token_budget,
                               float scale, int32_t* sel_idx, int32_t* sel_count, int32_t* sel_tokens, float* out,
                               float* lse, float* partial, int32_t* arrivals, int n_splits, unsigned long long* exchange,
                               hipStream_t stream) {
    dim3 grid(n_splits, s->n_kv_heads, s->batch), block(kSelThreads);
#define LEOAM_FUSED(IPT)                                                                                              \
    hipLaunchKernelGGL((select_attention_kernel<T, G, IPT>), grid, block, 0, stream, score, chunk_off, n_chunks,       \
                       max_chunks, token_budget, sel_idx, sel_count, sel_tokens, (const char*)q, (const char*)K,       \
                       (const char*)V, scale * kLog2e, out, lse, partial, arrivals, n_splits, s->c_max, s->k_max,      \
                       s->n_kv_heads, s->n_ctx, exchange)
    if (!score)      // the kept lists are given
        hipLaunchKernelGGL((select_attention_kernel<T, G, 1, true>), grid, block, 0, stream, score, chunk_off, n_chunks,
                           max_chunks, token_budget, sel_idx, sel_count, sel_tokens, (const char*)q, (const char*)K,
                           (const char*)V, scale * kLog2e, out, lse, partial, arrivals, n_splits, s->c_max, s->k_max,
                           s->n_kv_heads, s->n_ctx, exchange);
    else if (s->c_max <= kSelThreads) LEOAM_FUSED(1);
    else if (s->c_max <= 2 * kSelThreads) LEOAM_FUSED(2);
    else if (s->c_max <= 4 * kSelThreads) LEOAM_FUSED(4);
    else if (s->c_max <= 6 * kSelThreads) LEOAM_FUSED(6);
    else LEOAM_FUSED(8);
#undef LEOAM_FUSED
    return hipGetLastError();
}

template <typename T>
static hipError_t fused_by_group(const leoam_shape* s, const float* score, const void* q, const void* K, const void* V,
                                 const int32_t* chunk_off, const int32_t* n_chunks, int max_chunks, int token_budget,
                                 float scale, int32_t* sel_idx, int32_t* sel_count, int32_t* sel_tokens, float* out,
                                 float* lse, float* partial, int32_t* arrivals, int n_splits,
                                 unsigned long long* exchange, hipStream_t stream) {
#define LEOAM_FG(GG)                                                                                                   \
    launch_fused<T, GG>(s, score, q, K, V, chunk_off, n_chunks, max_chunks, token_budget, scale, sel_idx, sel_count,   \
                        sel_tokens, out, lse, partial, arrivals, n_splits, exchange, stream)
    switch (s->n_q_heads / s->n_kv_heads) {
    case 1: return LEOAM_FG(1);
    case 2: return LEOAM_FG(2);
    default: return LEOAM_FG(4);
    }
#undef LEOAM_FG
}

hipError_t select_attention_dispatch(const leoam_shape* s, const float* score, const void* q, const void* K,
                                     const void* V, const void* qmeta, const int32_t* chunk_off,
                                     const int32_t* n_chunks, int max_chunks, int token_budget, float scale,
                                     int32_t* sel_idx, int32_t* sel_count, int32_t* sel_tokens, float* out, float* lse,
                                     void* workspace, size_t workspace_bytes, hipStream_t stream, bool with_exchange) {
    const size_t head = control_bytes(s, with_exchange);
    char* body = (char*)workspace + head;
    const size_t body_bytes = workspace_bytes - head;
    unsigned long long* exchange = (with_exchange && exchange_bytes(s) > 0)
                                       ? (unsigned long long*)((char*)workspace + arrival_bytes(s))
                                       : nullptr;
    if (stream_ordered_merge_wanted()) {
        // the kernels of the separate calls, splits combined by a kernel of their own: every hand-over
        // between workgroups is then ordered by the stream
        if (body_bytes < attention_min_workspace_bytes(s)) return hipErrorInvalidValue;
        hipError_t e = score ? topk_select_dispatch(s, score, chunk_off, n_chunks, max_chunks, token_budget, sel_idx,
                                                    sel_count, sel_tokens, stream)
                             : hipSuccess;
        if (e != hipSuccess) return e;
        return attention_dispatch(s, q, K, V, qmeta, chunk_off, n_chunks, sel_idx, sel_count, scale, out, lse, body,
                                  body_bytes, nullptr, stream);
    }
    if (select_attention_q_is_fused(s)) {
        // the compressed store's one-launch kernel (select_attention_q.hip)
        size_t n = body_bytes / fused_part_bytes_per_split(s);
        const size_t cap = (size_t)fused_q_recommended_splits(s, token_budget > 0 ? token_budget : s->n_ctx);
        if (n > cap) n = cap;
        if (n < 1) n = 1;
        return select_attention_q_dispatch(s, score, q, K, V, qmeta, chunk_off, n_chunks, max_chunks, token_budget, scale,
                                           sel_idx, sel_count, sel_tokens, out, lse, (float*)body, (int32_t*)workspace,
                                           (int)n, stream);
    }
    if (!select_attention_is_fused(s)) {
        hipError_t e = score ? topk_select_dispatch(s, score, chunk_off, n_chunks, max_chunks, token_budget, sel_idx,
                                                    sel_count, sel_tokens, stream)
                             : hipSuccess;
        if (e != hipSuccess) return e;
        // the attention kernel merges its splits in the same launch, with the arrival counters of this workspace
        return attention_dispatch(s, q, K, V, qmeta, chunk_off, n_chunks, sel_idx, sel_count, scale, out, lse, body,
                                  body_bytes, (int32_t*)workspace, stream);
    }
    size_t n = body_bytes / fused_part_bytes_per_split(s);
    const size_t cap = (size_t)fused_recommended_splits(s, token_budget > 0 ? token_budget : s->n_ctx);
    if (n > cap) n = cap;
    if (n < 1) n = 1;      // a single split needs no partials
    const int n_splits = (int)n;
    if (s->kv_dtype == LEOAM_F16)
        return fused_by_group<F16>(s, score, q, K, V, chunk_off, n_chunks, max_chunks, token_budget, scale, sel_idx,
                                   sel_count, sel_tokens, out, lse, (float*)body, (int32_t*)workspace, n_splits, exchange,
                                   stream);
    return fused_by_group<BF16>(s, score, q, K, V, chunk_off, n_chunks, max_chunks, token_budget, scale, sel_idx,
                                sel_count, sel_tokens, out, lse, (float*)body, (int32_t*)workspace, n_splits, exchange, stream);
}

}  // namespace leoam
