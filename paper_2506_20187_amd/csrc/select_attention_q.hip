// chunk_select_attention_decode over the compressed KV store (8-bit / 4-bit
// chunks; paper Sec. 4.4 dynamic KV compression, Sec. 6.1 INT4): the selection
// (Sec. 4.2 / 6.1) and the attention over the kept chunks (Sec. 2.1 Eq. 1) of a
// decode step in ONE launch.
//
// Same plan as the 16-bit one-launch kernel (select_attention.hip): a 1024-lane
// workgroup runs the selection of its (sequence, kv head), leaves what it needs
// about the kept chunks in LDS - here their records (byte offset, format, scale
// and zero point of K and of V) next to the token prefix - its sixteen waves
// stream their shares of the kept tokens, and the workgroup that finishes last
// combines the splits (fused_tail.h).  The streaming part is the matrix-core
// kernel of quant_store.hip: q . code on v_mfma_f32_16x16x32_f16 with the codes
// expanded to f16 by byte permutation, scale_k / zero_k applied to the result,
// P V in fp32 on the vector ALU.  The compressed store is used where the cache
// is large and the batch small: the launch is latency-bound, and what it saves
// against the three-launch path is two launch gaps, the kept list's round trip
// through memory and the merge kernel.
#include "fused_tail.h"
#include "quant_common.h"

namespace leoam {

constexpr int kFusedQBlock = 128;                      // positions a wave maps to chunk slots at a time
constexpr int kFusedQGranule = kFusedWaves * 16;       // a split is a multiple of this many tokens
constexpr int kFusedQMaxSel = 1024;                    // kept chunks per (b,h) whose records fit the LDS tables
constexpr int kFusedQMaxSplits = 64;
constexpr int kFusedQTargetWgs = 256;                  // one workgroup per compute unit

// kGiven: the kept lists (sel_idx, sel_count) are inputs and the workgroup only builds its tables from
// them (one list position per lane; kIpt is not used).
template <int G, int kIpt, bool kGiven = false>
__global__ __launch_bounds__(kSelThreads) void select_attention_q_kernel(
    const float* __restrict__ score, const int32_t* __restrict__ chunk_off, const int32_t* __restrict__ n_chunks,
    int max_chunks, int token_budget, int32_t* __restrict__ sel_idx, int32_t* __restrict__ sel_count,
    int32_t* __restrict__ sel_tokens, const char* __restrict__ q, const unsigned char* __restrict__ kblob,
    const unsigned char* __restrict__ vblob, const QChunk* __restrict__ qmeta, float scale_log2,
    float* __restrict__ out, float* __restrict__ lse, float* partial, int32_t* arrivals, int n_splits, int c_max,
    int k_max, int n_kv_heads, int n_ctx) {
    constexpr int EPL = 8;
    static_assert(G <= 4, "one MFMA column per head, four accumulator sets per lane");

    // the three phases use LDS one after the other
    union Phase {
        SelectLds sel;
        struct {
            int32_t slot[kFusedWaves][kFusedQBlock], tin[kFusedWaves][kFusedQBlock];
        } pos;
        float xw[kFusedWaves][G][kPartStride];
    };
    __shared__ Phase ph;
    __shared__ long long ch_off[kFusedQMaxSel];
    __shared__ float4 ch_par[kFusedQMaxSel];           // scale_k, zero_k, scale_v, zero_v
    __shared__ int32_t ch_bits[kFusedQMaxSel];
    __shared__ int32_t prefix[kFusedQMaxSel + 1];
    __shared__ uint4 qs[4][LEOAM_WAVE];                // matrix-core B operand (the group's queries), same for every wave
    __shared__ float qsums[16];                        // sum_d q of head j (0 beyond G)
    __shared__ int32_t sh_last;

    const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid / LEOAM_WAVE;
    const int grp = lane >> 4, c16 = lane & 15;
    const size_t bh = (size_t)b * n_kv_heads + h;
    const int C = min(max(n_chunks[b], 0), c_max);
    const int32_t* off = chunk_off + (size_t)b * (c_max + 1);

    // ---- the group's queries: fetched by one wave while the selection runs ----------
    uint4 qraw[4];
    if (wave == 0) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const size_t qrow = ((size_t)b * n_kv_heads * G + (size_t)h * G + min(c16, G - 1)) * (LEOAM_D * 2);
            qraw[s] = load16(q, qrow + 64 * s + 16 * grp);
        }
    }

    auto stage_queries = [&] {
        float sum = 0.f;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            qs[s][lane] = (c16 < G) ? query_operand(qraw[s]) : make_uint4(0, 0, 0, 0);
            float x[EPL];
            unpack<F16>(qraw[s], x);
#pragma unroll
            for (int e = 0; e < EPL; ++e) sum += x[e];
        }
        sum += shfl_xor_f(sum, 16);
        sum += shfl_xor_f(sum, 32);
        if (grp == 0) qsums[c16] = (c16 < G) ? sum : 0.f;
    };
    int cnt;
    if constexpr (kGiven) {
        // ---- the kept list is given: record and size of every listed chunk, then a scan ------------
        static_assert(kFusedQMaxSel == kSelThreads, "one list position per lane");
        const int listed = min(max(sel_count[bh], 0), k_max);
        const int id = sel_idx[bh * (size_t)k_max + min(tid, k_max - 1)];
        const bool ok = tid < listed && id >= 0 && id < C;
        const int c = ok ? id : 0;
        const int a = min(max(off[c], 0), n_ctx), e = min(max(off[c + 1], a), n_ctx);
        const QChunk m = qmeta[bh * c_max + c];
        uint64_t tot;
        const uint32_t before = (uint32_t)block_excl_scan<false>(pack_tot(0, ok ? (uint32_t)(e - a) : 0u), ph.sel.wave_sums2, &tot);
        if (tid < listed) {
            ch_off[tid] = m.byte_off;
            ch_bits[tid] = m.bits;
            ch_par[tid] = make_float4(m.scale_k, m.zero_k, m.scale_v, m.zero_v);
            prefix[tid] = (int32_t)before;
        }
        cnt = listed;
        if (tid == 0) prefix[cnt] = (int32_t)(uint32_t)tot;
        if (wave == 0) stage_queries();
    } else {
        // ---- selection --------------------------------------------------------------
        SelectResult<kIpt> R;
        select_keep<kIpt>(ph.sel, score + bh * (size_t)c_max, off, C, c_max, k_max, n_ctx, max_chunks, token_budget, R);
        cnt = (int)min((uint32_t)(R.kept_total >> 32), (uint32_t)k_max);
        const int total = (int)(uint32_t)R.kept_total;
        {
            // kept chunks in ascending order: their records and the number of kept tokens before them
            int32_t* ids = sel_idx + bh * (size_t)k_max;
            const int c0 = tid * kIpt;
            uint32_t pos = (uint32_t)(R.kept_before >> 32), before = (uint32_t)R.kept_before;
#pragma unroll
            for (int i = 0; i < kIpt; ++i) {
                if (R.keep[i]) {
                    if (pos < (uint32_t)k_max) {
                        const QChunk m = qmeta[bh * c_max + c0 + i];
                        ch_off[pos] = m.byte_off;
                        ch_bits[pos] = m.bits;
                        ch_par[pos] = make_float4(m.scale_k, m.zero_k, m.scale_v, m.zero_v);
                        prefix[pos] = (int32_t)before;
                        if (split == 0) ids[pos] = c0 + i;
                    }
                    ++pos;
                    before += R.size[i];
                }
            }
            if (tid == 0) prefix[cnt] = total;
            if (wave == 0) stage_queries();
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
    // (k_max may cut the kept list short of the selection's token total: stream what the list holds)
    const int listed = prefix[cnt];

    // ---- this workgroup's range of the kept tokens, then this wave's share --------
    int per_split = (listed + n_splits - 1) / n_splits;
    per_split = ((per_split + kFusedQGranule - 1) / kFusedQGranule) * kFusedQGranule;
    const int r0 = min(listed, split * per_split), r1 = min(listed, r0 + per_split);
    const int per_wave = per_split / kFusedWaves;
    const int w0 = min(r1, r0 + wave * per_wave), w1 = min(r1, w0 + per_wave);
    int32_t* my_slot = ph.pos.slot[wave];
    int32_t* my_tin = ph.pos.tin[wave];
    const float qsum = qsums[c16];

    // lanes (grp, head) carry the softmax state of `head`; every lane carries the accumulators of
    // all heads for the V rows of its group and its 8 channels (in the order 0,2,4,6,1,3,5,7)
    float m_run = -INFINITY, l_run = 0.f;
    float acc[G][EPL], accz[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        accz[g] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
    }

    auto fetch = [&](int t, QmTile& kv) {
        // unconditional loads: a position past the end reads the block's last token and gets weight 0
        {
            const int p = 16 * t + c16;
            const int raw = my_slot[p], slot = raw ^ (raw >> 31);       // a complemented slot: past the end
            const bool four = ch_bits[slot] == 4;
            const size_t row = (size_t)ch_off[slot] + (size_t)my_tin[p] * (four ? LEOAM_D / 2 : LEOAM_D) + (four ? 4 : 8) * grp;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const size_t a0 = row + (four ? 16 : 32) * s;
                kv.k0[s] = *reinterpret_cast<const uint32_t*>(kblob + a0);
                kv.k1[s] = *reinterpret_cast<const uint32_t*>(kblob + a0 + (four ? 0 : 4));      // 4-bit: the same dword again
            }
            kv.kfour = four;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int p = 16 * t + 4 * grp + i;
            kv.vslot[i] = my_slot[p];
            const int slot = kv.vslot[i] ^ (kv.vslot[i] >> 31);
            const bool four = ch_bits[slot] == 4;
            const size_t a0 = (size_t)ch_off[slot] + (size_t)my_tin[p] * (four ? LEOAM_D / 2 : LEOAM_D) + (four ? 4 : 8) * c16;
            kv.v0[i] = *reinterpret_cast<const uint32_t*>(vblob + a0);
            kv.v1[i] = *reinterpret_cast<const uint32_t*>(vblob + a0 + (four ? 0 : 4));
            kv.vfour[i] = four;
        }
    };
    int q_lane = lane;
    auto consume = [&](const QmTile& kv) {
        // the B operand is re-read from LDS for every tile: 16 registers a wave cannot spare
        asm volatile("" : "+v"(q_lane));
        const f32x4_t sacc = code_logits(kv, [&](int s) { return qs[s][q_lane]; });
        // ---- logits of tokens 4grp + r, head c16 ----
        float z[4], sv[4], zv[4];
        float mloc = -INFINITY;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float4 par = ch_par[kv.vslot[r] ^ (kv.vslot[r] >> 31)];
            sv[r] = par.z;
            zv[r] = par.w;
            z[r] = (kv.vslot[r] >= 0) ? fmaf(par.x, sacc[r], par.y * qsum) * scale_log2 : -INFINITY;
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
            static_for<0, G>([&](auto gc) {
                constexpr int g = decltype(gc)::value;
                const float cg = row_bcast<g>(corr);
                accz[g] *= cg;
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[g][e] *= cg;
            });
        }
        // ---- P V: the V codes of tokens 4grp + i, this lane's 8 channels ----
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float x[EPL];
            value_codes(kv.v0[i], kv.v1[i], kv.vfour[i], x);
            static_for<0, G>([&](auto gc) {
                constexpr int g = decltype(gc)::value;
                const float p = row_bcast<g>(z[i]);
                accz[g] = fmaf(p, zv[i], accz[g]);
                const float ps = p * sv[i];
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(ps, x[e], acc[g][e]);
            });
        }
    };

    for (int blk = w0; blk < w1; blk += kFusedQBlock) {
        const int nb = min(kFusedQBlock, w1 - blk);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");      // earlier reads of the tables are done
        {
            // a lane maps consecutive positions: one search, then a walk
            constexpr int PER = kFusedQBlock / LEOAM_WAVE;
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
            int last_slot = 0, last_tin = 0;
#pragma unroll
            for (int j = 0; j < PER; ++j) {
                if (i0 + j < nb) {
                    const int x = blk + i0 + j;
                    while (prefix[lo + 1] <= x) ++lo;      // ends: prefix[cnt] = listed > x
                    last_slot = lo;
                    last_tin = x - prefix[lo];
                    my_slot[i0 + j] = last_slot;
                    my_tin[i0 + j] = last_tin;
                }
            }
            // positions past the end point at the block's last token, slot stored complemented (< 0):
            // their loads stay inside the store and their weight is 0
            const int owner = (nb - 1) / PER;
            last_slot = __shfl(last_slot, owner, LEOAM_WAVE);
            last_tin = __shfl(last_tin, owner, LEOAM_WAVE);
#pragma unroll
            for (int j = 0; j < PER; ++j) {
                if (i0 + j >= nb) {
                    my_slot[i0 + j] = ~last_slot;
                    my_tin[i0 + j] = last_tin;
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");      // tables visible to the whole wave
        __builtin_amdgcn_wave_barrier();

        const int n_tiles = (nb + 15) >> 4, last = n_tiles - 1;
        QmTile cur, nxt;
        fetch(0, cur);
        if (n_tiles == 1) {
            consume(cur);
            continue;
        }
        for (int t = 0; t < n_tiles; t += 2) {
            fetch(min(t + 1, last), nxt);
            __builtin_amdgcn_sched_barrier(0);       // keep the loads ahead of the tile's arithmetic
            consume(cur);
            fetch(min(t + 2, last), cur);
            __builtin_amdgcn_sched_barrier(0);
            if (t + 1 < n_tiles) consume(nxt);
        }
    }

    // ---- fold the four lane groups (same m everywhere in the wave); zero_v's share is the same for
    // every channel.  Four accumulators at a time: afterwards lane group r holds the total of
    // accumulator e_own of the quad, so all 64 lanes write to LDS ------------------------------------
    l_run = rows_sum4(l_run, l_run, l_run, l_run);
    const int e_own = ((grp & 1) << 1) | (grp >> 1);        // rows 0,1,2,3 own accumulators 0,2,1,3
    float folded[G][2];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        folded[g][0] = rows_sum4(acc[g][0] + accz[g], acc[g][1] + accz[g], acc[g][2] + accz[g], acc[g][3] + accz[g]);
        folded[g][1] = rows_sum4(acc[g][4] + accz[g], acc[g][5] + accz[g], acc[g][6] + accz[g], acc[g][7] + accz[g]);
    }
    __syncthreads();      // every wave is done with its position tables: LDS becomes the exchange buffer
#pragma unroll
    for (int g = 0; g < G; ++g) {
        // accumulator e holds channel code_channel(e) = 2e (e < 4) or 2(e - 4) + 1
        ph.xw[wave][g][c16 * EPL + 2 * e_own] = folded[g][0];
        ph.xw[wave][g][c16 * EPL + 2 * e_own + 1] = folded[g][1];
    }
    if (grp == 0 && c16 < G) {
        ph.xw[wave][c16][LEOAM_D] = m_run;
        ph.xw[wave][c16][LEOAM_D + 1] = l_run;
    }
    __syncthreads();
    fused_tail<G>(ph.xw, sh_last, partial, arrivals, out, lse, bh, split, n_splits);
}

bool select_attention_q_is_fused(const leoam_shape* s) {
    const int g = s->n_q_heads / s->n_kv_heads;
    return s->kv_dtype == LEOAM_Q8Q4 && g <= 4 && s->k_max <= kFusedQMaxSel && s->c_max <= 16 * kSelThreads;
}

int fused_q_recommended_splits(const leoam_shape* s, int max_tokens) {
    if (max_tokens <= 0 || max_tokens > s->n_ctx) max_tokens = s->n_ctx;
    const int by_tokens = (max_tokens + kFusedQGranule - 1) / kFusedQGranule;
    const int units = s->batch * s->n_kv_heads;
    int want = (kFusedQTargetWgs + units - 1) / units;
    if (want > by_tokens) want = by_tokens;
    if (want > kFusedQMaxSplits) want = kFusedQMaxSplits;
    if (want < 1) want = 1;
    return want;
}

template <int G>
static hipError_t launch_fused_q(const leoam_shape* s, const float* score, const void* q, const void* K, const void* V,
                                 const void* qmeta, const int32_t* chunk_off, const int32_t* n_chunks, int max_chunks,
                                 int token_budget, float scale, int32_t* sel_idx, int32_t* sel_count,
                                 int32_t* sel_tokens, float* out, float* lse, float* partial, int32_t* arrivals,
                                 int n_splits, hipStream_t stream) {
    dim3 grid(n_splits, s->n_kv_heads, s->batch), block(kSelThreads);
#define LEOAM_FUSEDQ(IPT)                                                                                             \
    hipLaunchKernelGGL((select_attention_q_kernel<G, IPT>), grid, block, 0, stream, score, chunk_off, n_chunks,        \
                       max_chunks, token_budget, sel_idx, sel_count, sel_tokens, (const char*)q,                       \
                       (const unsigned char*)K, (const unsigned char*)V, (const QChunk*)qmeta, scale * kLog2e, out,    \
                       lse, partial, arrivals, n_splits, s->c_max, s->k_max, s->n_kv_heads, s->n_ctx)
    if (!score)      // the kept lists are given
        hipLaunchKernelGGL((select_attention_q_kernel<G, 1, true>), grid, block, 0, stream, score, chunk_off, n_chunks,
                           max_chunks, token_budget, sel_idx, sel_count, sel_tokens, (const char*)q,
                           (const unsigned char*)K, (const unsigned char*)V, (const QChunk*)qmeta, scale * kLog2e, out,
                           lse, partial, arrivals, n_splits, s->c_max, s->k_max, s->n_kv_heads, s->n_ctx);
    else if (s->c_max <= kSelThreads) LEOAM_FUSEDQ(1);
    else if (s->c_max <= 2 * kSelThreads) LEOAM_FUSEDQ(2);
    else if (s->c_max <= 4 * kSelThreads) LEOAM_FUSEDQ(4);
    else if (s->c_max <= 6 * kSelThreads) LEOAM_FUSEDQ(6);
    else if (s->c_max <= 8 * kSelThreads) LEOAM_FUSEDQ(8);
    else if (s->c_max <= 10 * kSelThreads) LEOAM_FUSEDQ(10);
    else if (s->c_max <= 12 * kSelThreads) LEOAM_FUSEDQ(12);
    else LEOAM_FUSEDQ(16);
#undef LEOAM_FUSEDQ
    return hipGetLastError();
}

hipError_t select_attention_q_dispatch(const leoam_shape* s, const float* score, const void* q, const void* K,
                                       const void* V, const void* qmeta, const int32_t* chunk_off,
                                       const int32_t* n_chunks, int max_chunks, int token_budget, float scale,
                                       int32_t* sel_idx, int32_t* sel_count, int32_t* sel_tokens, float* out,
                                       float* lse, float* partial, int32_t* arrivals, int n_splits,
                                       hipStream_t stream) {
#define LEOAM_FQ(GG)                                                                                                   \
    launch_fused_q<GG>(s, score, q, K, V, qmeta, chunk_off, n_chunks, max_chunks, token_budget, scale, sel_idx,        \
                       sel_count, sel_tokens, out, lse, partial, arrivals, n_splits, stream)
    switch (s->n_q_heads / s->n_kv_heads) {
    case 1: return LEOAM_FQ(1);
    case 2: return LEOAM_FQ(2);
    default: return LEOAM_FQ(4);
    }
#undef LEOAM_FQ
}

}  // namespace leoam
