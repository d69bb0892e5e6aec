// sparse_chunk_attention_decode: softmax(q K^T / sqrt(d)) V (paper Sec. 2.1,
// Eq. 1) over the tokens of the kept chunks only (Sec. 4.1 workflow: the
// evaluation result selects the KV used by the decoding computation).
//
// HBM-bound: each kept token costs one K row and one V row (2*D*e bytes) and
// 4*G*D flops.  Split-K over the *kept-token* axis: the kept chunks of a
// (sequence, kv head) are laid end to end, the resulting token list is cut into
// equal ranges, one workgroup per range; every workgroup streams its rows with
// 16-byte-per-lane loads (a wave-wide load = 1 KiB of contiguous row data),
// keeps an online-softmax state (m, l, acc[D]) per query head of the group, and
// writes one partial per range.  A second kernel combines the partials in range
// order, so results do not depend on scheduling.
#include <type_traits>

#include "attention_common.h"

namespace leoam {

// out[b,j,:] = sum_s 2^(m_s - m) o_s / sum_s 2^(m_s - m) l_s.  One workgroup per
// (b, query head): kMergeParts thread rows take the splits round-robin, each
// issues all of its loads before using any (one memory round trip for up to
// kMergeParts*kMergeBatch splits), and the rows are then folded in a fixed order.
constexpr int kMergeParts = 4;
constexpr int kMergeBatch = 16;
__global__ __launch_bounds__(LEOAM_D* kMergeParts) void attention_merge_kernel(const float* __restrict__ partial,
                                                                               int n_splits, float* __restrict__ out,
                                                                               float* __restrict__ lse) {
    __shared__ float sm[kMergeParts], sl[kMergeParts][LEOAM_D], so[kMergeParts][LEOAM_D];
    const size_t bj = blockIdx.x;
    const int d = threadIdx.x % LEOAM_D, part = threadIdx.x / LEOAM_D;
    const float* base = partial + bj * (size_t)n_splits * kPartStride;
    float m = -INFINITY, o = 0.f, l = 0.f;
    for (int s0 = part; s0 < n_splits; s0 += kMergeParts * kMergeBatch) {
        float ms[kMergeBatch], ls[kMergeBatch], os[kMergeBatch];
#pragma unroll
        for (int i = 0; i < kMergeBatch; ++i) {
            const int s = s0 + i * kMergeParts;
            const bool ok = s < n_splits;
            const float* p = base + (size_t)(ok ? s : 0) * kPartStride;      // unconditional loads, masked below
            ms[i] = p[LEOAM_D];
            ls[i] = p[LEOAM_D + 1];
            os[i] = p[d];
            if (!ok) {
                ms[i] = -INFINITY;
                ls[i] = 0.f;
                os[i] = 0.f;
            }
        }
        float mb = m;
#pragma unroll
        for (int i = 0; i < kMergeBatch; ++i) mb = fmaxf(mb, ms[i]);
        const float c = exp2_or_zero(m, mb);
        o *= c;
        l *= c;
        m = mb;
#pragma unroll
        for (int i = 0; i < kMergeBatch; ++i) {
            const float a = exp2_or_zero(ms[i], m);
            o += a * os[i];
            l += a * ls[i];
        }
    }
    if (d == 0) sm[part] = m;
    sl[part][d] = l;
    so[part][d] = o;
    __syncthreads();
    if (part != 0) return;
    float mm = -INFINITY;
#pragma unroll
    for (int p = 0; p < kMergeParts; ++p) mm = fmaxf(mm, sm[p]);
    float oo = 0.f, ll = 0.f;
#pragma unroll
    for (int p = 0; p < kMergeParts; ++p) {
        const float a = exp2_or_zero(sm[p], mm);
        oo += a * so[p][d];
        ll += a * sl[p][d];
    }
    out[bj * LEOAM_D + d] = (ll > 0.f) ? oo / ll : 0.f;
    if (lse && d == 0) lse[bj] = (ll > 0.f) ? (mm + log2f(ll)) * kLn2 : -INFINITY;
}

template <typename T, int G>
__global__ __launch_bounds__(kAttThreads) void sparse_attention_kernel(
    const char* __restrict__ q, const char* __restrict__ K, const char* __restrict__ V,
    const int32_t* __restrict__ chunk_off, const int32_t* __restrict__ n_chunks, const int32_t* __restrict__ sel_idx,
    const int32_t* __restrict__ sel_count, float scale_log2, float* partial, int n_splits, int c_max,
    int k_max, int n_kv_heads, int n_ctx, MergeInLaunch mg) {
    constexpr int LPR = Row<T>::kLanesPerRow;
    constexpr int RPL = Row<T>::kRowsPerLoad;          // lane groups per wave
    constexpr int EPL = T::kEpl;
    constexpr int ROWB = Row<T>::kRowBytes;
    constexpr int NG = kAttWaves * RPL;                // lane groups per workgroup
    constexpr int TILE = NG * kAttRows;                // tokens per tile

    extern __shared__ int32_t dyn[];                   // start[k_max] | prefix[k_max + 1]
    __shared__ int32_t phys[TILE];
    __shared__ float xw[kAttWaves][G][kPartStride];
    __shared__ int32_t sh_total;

    const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid / LEOAM_WAVE;
    const int grp = lane / LPR;                        // lane group inside the wave
    const int col = (lane % LPR) * EPL;                // first column this lane owns
    const size_t bh = (size_t)b * n_kv_heads + h;
    const int C = min(max(n_chunks[b], 0), c_max);
    const int cnt = min(max(sel_count[bh], 0), k_max);
    const int32_t* off = chunk_off + (size_t)b * (c_max + 1);
    const int32_t* sel = sel_idx + bh * (size_t)k_max;
    int32_t* start = dyn;
    int32_t* prefix = dyn + k_max;

    // ---- kept chunks -> token prefix ----------------------------------------
    for (int i = tid; i < cnt; i += kAttThreads) {
        const int id = sel[i];
        int t0 = 0, sz = 0;
        if (id >= 0 && id < C) {
            t0 = min(max(off[id], 0), n_ctx);
            sz = min(max(off[id + 1], t0), n_ctx) - t0;
        }
        start[i] = t0;
        prefix[i + 1] = sz;
    }
    if (tid == 0) prefix[0] = 0;
    __syncthreads();
    if (wave == 0) {
        // inclusive scan of prefix[1..cnt] by one wave: each lane a contiguous run
        const int per = (cnt + LEOAM_WAVE - 1) / LEOAM_WAVE;
        const int i0 = 1 + lane * per, i1 = min(cnt + 1, i0 + per);
        int s = 0;
        for (int i = i0; i < i1; ++i) s += prefix[i];
        int incl = s;
#pragma unroll
        for (int d = 1; d < LEOAM_WAVE; d <<= 1) {
            const int o = __shfl_up(incl, d, LEOAM_WAVE);
            if (lane >= d) incl += o;
        }
        int run = incl - s;
        for (int i = i0; i < i1; ++i) {
            run += prefix[i];
            prefix[i] = run;
        }
        if (lane == LEOAM_WAVE - 1) sh_total = incl;
    }
    __syncthreads();
    const int total = sh_total;

    // ---- this workgroup's token range ----------------------------------------
    int per_split = (total + n_splits - 1) / n_splits;
    per_split = ((per_split + TILE - 1) / TILE) * TILE;
    const int r0 = min(total, split * per_split), r1 = min(total, r0 + per_split);

    // ---- queries: this lane's columns, pre-multiplied by scale*log2(e) --------
    float qs[G][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const size_t qrow = ((size_t)b * n_kv_heads * G + (size_t)h * G + g) * ROWB;
        float x[EPL];
        unpack<T>(load16(q, qrow + (size_t)col * T::kBytes), x);
#pragma unroll
        for (int e = 0; e < EPL; ++e) qs[g][e] = x[e] * scale_log2;
    }

    const char* Kbh = K + bh * (size_t)n_ctx * ROWB;
    const char* Vbh = V + bh * (size_t)n_ctx * ROWB;
    const size_t col_bytes = (size_t)col * T::kBytes;

    float m_run[G], l_run[G], acc[G][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m_run[g] = -INFINITY;
        l_run[g] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
    }

    for (int tb = r0; tb < r1; tb += TILE) {
        // token position in the kept list -> row in the cache
        __syncthreads();
        for (int i = tid; i < TILE; i += kAttThreads) {
            const int x = tb + i;
            int p = -1;
            if (x < r1) {
                int lo = 0, hi = cnt;          // largest k with prefix[k] <= x
                while (hi - lo > 1) {
                    const int mid = (lo + hi) >> 1;
                    if (prefix[mid] <= x) lo = mid; else hi = mid;
                }
                p = start[lo] + (x - prefix[lo]);
            }
            phys[i] = p;
        }
        __syncthreads();

        int row[kAttRows];
        uint4 kv[kAttRows], vv[kAttRows];
#pragma unroll
        for (int j = 0; j < kAttRows; ++j) {
            row[j] = phys[j * NG + wave * RPL + grp];
            kv[j] = make_uint4(0, 0, 0, 0);
            vv[j] = make_uint4(0, 0, 0, 0);
            if (row[j] >= 0) {
                kv[j] = load16(Kbh, (size_t)row[j] * ROWB + col_bytes);
                vv[j] = load16(Vbh, (size_t)row[j] * ROWB + col_bytes);
            }
        }
        // logits (log2 domain) of the tile's rows for every head of the group
        float z[kAttRows][G];
        float mt[G];
#pragma unroll
        for (int g = 0; g < G; ++g) mt[g] = m_run[g];
#pragma unroll
        for (int j = 0; j < kAttRows; ++j) {
            float x[EPL];
            unpack<T>(kv[j], x);
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float d = 0.f;
#pragma unroll
                for (int e = 0; e < EPL; ++e) d = fmaf(qs[g][e], x[e], d);
                d = row16_sum(d);
                if (LPR == 32) d += shfl_xor_f(d, 16);
                z[j][g] = (row[j] >= 0) ? d : -INFINITY;
                mt[g] = fmaxf(mt[g], z[j][g]);
            }
        }
        // rescale the running state once per tile
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float corr = exp2_or_zero(m_run[g], mt[g]);
            m_run[g] = mt[g];
            l_run[g] *= corr;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[g][e] *= corr;
        }
#pragma unroll
        for (int j = 0; j < kAttRows; ++j) {
            float x[EPL];
            unpack<T>(vv[j], x);
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float p = exp2_or_zero(z[j][g], m_run[g]);
                l_run[g] += p;
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(p, x[e], acc[g][e]);
            }
        }
    }

    // ---- fold the lane groups of the wave (fixed order) -------------------------
#pragma unroll
    for (int msk = LPR; msk < LEOAM_WAVE; msk <<= 1) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float m_o = shfl_xor_f(m_run[g], msk);
            const float l_o = shfl_xor_f(l_run[g], msk);
            const float m_n = fmaxf(m_run[g], m_o);
            // lower lane's state first so both partners compute the same expression
            const bool low = (lane & msk) == 0;
            const float a_self = exp2_or_zero(m_run[g], m_n), a_oth = exp2_or_zero(m_o, m_n);
            l_run[g] = low ? (l_run[g] * a_self + l_o * a_oth) : (l_o * a_oth + l_run[g] * a_self);
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                const float o = shfl_xor_f(acc[g][e], msk);
                acc[g][e] = low ? (acc[g][e] * a_self + o * a_oth) : (o * a_oth + acc[g][e] * a_self);
            }
            m_run[g] = m_n;
        }
    }
    // ---- fold the waves through LDS ------------------------------------------
    if (grp == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) xw[wave][g][col + e] = acc[g][e];
            if (lane == 0) {
                xw[wave][g][LEOAM_D] = m_run[g];
                xw[wave][g][LEOAM_D + 1] = l_run[g];
            }
        }
    }
    finish_split<G>(xw, partial, b, h, split, n_splits, n_kv_heads, mg);
}


// ---------------------------------------------------------------------------
// 16-bit keys/values: q K^T on the matrix cores.
//
// v_mfma_f32_16x16x32 (bf16 / f16): D[i][j] += sum_k A[i][k] B[k][j], A lane =
// (i = lane%16, k = 8*(lane/16)..+8), B lane = (j = lane%16, same k), D lane =
// (j = lane%16, i = 4*(lane/16)..+4).  Here i = a token of a 16-token tile, j =
// a query head of the group (columns >= G are zero), k = 32 of the 128 channels:
// four instructions give the 16 x G logits of a tile straight from the 16-byte
// K loads (lane = token, four lanes cover 64 contiguous bytes of its row), with
// no unpacking and no cross-lane reduction.  The logits of token 4*grp+r, head h
// land in lane 16*grp+h, register r.  P V stays on the vector ALU in fp32 (P is
// never rounded to 16 bits): lane group grp streams the V rows of tokens
// 4*grp+0..3, so the weight it needs is a broadcast inside its own 16-lane row
// (DPP row_newbcast), not a shuffle.
// ---------------------------------------------------------------------------
constexpr int kMfmaWaveBlock = 256;                   // tokens a wave maps to rows at a time
constexpr int kMfmaGranule = kAttWaves * 16;           // a split is a multiple of this many tokens

// one 16-token tile of a wave: K operand (4 x 16 B per lane) and V rows (4 x 16 B per lane)
struct KvTile {
    uint4 k[4];
    uint4 v[4];
};

template <typename T, int G>
__global__ __launch_bounds__(kAttThreads) __attribute__((amdgpu_waves_per_eu(G <= 4 ? 3 : 2)))     // three workgroups per CU
void sparse_attention_mfma_kernel(
    const char* __restrict__ q, const char* __restrict__ K, const char* __restrict__ V,
    const int32_t* __restrict__ chunk_off, const int32_t* __restrict__ n_chunks, const int32_t* __restrict__ sel_idx,
    const int32_t* __restrict__ sel_count, float scale_log2, float* partial, int n_splits, int c_max,
    int k_max, int n_kv_heads, int n_ctx, MergeInLaunch mg) {
    constexpr int ROWB = LEOAM_D * 2;
    constexpr int EPL = 8;

    extern __shared__ int32_t dyn[];                   // start[k_max] | prefix[k_max + 1]
    __shared__ int32_t rows[kAttWaves][kMfmaWaveBlock];
    __shared__ float xw[kAttWaves][G][kPartStride];
    __shared__ int32_t sh_total;

    const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid / LEOAM_WAVE;
    const int grp = lane >> 4, c16 = lane & 15;
    const size_t bh = (size_t)b * n_kv_heads + h;
    const int C = min(max(n_chunks[b], 0), c_max);
    const int cnt = min(max(sel_count[bh], 0), k_max);
    const int32_t* off = chunk_off + (size_t)b * (c_max + 1);
    const int32_t* sel = sel_idx + bh * (size_t)k_max;
    int32_t* start = dyn;
    int32_t* prefix = dyn + k_max;

    // ---- B operand: the group's queries (column = head), zero beyond G ----------
    uint4 qb[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        qb[s] = make_uint4(0, 0, 0, 0);
        if (c16 < G) {
            const size_t qrow = ((size_t)b * n_kv_heads * G + (size_t)h * G + c16) * ROWB;
            qb[s] = load16(q, qrow + 64 * s + 16 * grp);
        }
    }

    // ---- kept chunks -> token prefix (same as the vector kernel) ---------------
    // (the loop bound does not depend on loaded data, so these loads go out
    // together with the loads of the counts and of the queries)
    for (int i = tid; i < k_max; i += kAttThreads) {
        const int id = sel[i];
        if (i >= cnt) continue;
        int t0 = 0, sz = 0;
        if (id >= 0 && id < C) {
            t0 = min(max(off[id], 0), n_ctx);
            sz = min(max(off[id + 1], t0), n_ctx) - t0;
        }
        start[i] = t0;
        prefix[i + 1] = sz;
    }
    if (tid == 0) prefix[0] = 0;
    __syncthreads();
    if (wave == 0) {
        const int per = (cnt + LEOAM_WAVE - 1) / LEOAM_WAVE;
        const int i0 = 1 + lane * per, i1 = min(cnt + 1, i0 + per);
        int s = 0;
        for (int i = i0; i < i1; ++i) s += prefix[i];
        int incl = s;
#pragma unroll
        for (int d = 1; d < LEOAM_WAVE; d <<= 1) {
            const int o = __shfl_up(incl, d, LEOAM_WAVE);
            if (lane >= d) incl += o;
        }
        int run = incl - s;
        for (int i = i0; i < i1; ++i) {
            run += prefix[i];
            prefix[i] = run;
        }
        if (lane == LEOAM_WAVE - 1) sh_total = incl;
    }
    __syncthreads();
    const int total = sh_total;
    // the split's range, then this wave's contiguous share of it; from here on the
    // four waves are independent streams until the final merge
    int per_split = (total + n_splits - 1) / n_splits;
    per_split = ((per_split + kMfmaGranule - 1) / kMfmaGranule) * kMfmaGranule;
    const int r0 = min(total, split * per_split), r1 = min(total, r0 + per_split);
    const int per_wave = per_split / kAttWaves;
    const int w0 = min(r1, r0 + wave * per_wave), w1 = min(r1, w0 + per_wave);

    const char* Kbh = K + bh * (size_t)n_ctx * ROWB + 16 * grp;        // + row*ROWB + 64*s
    const char* Vbh = V + bh * (size_t)n_ctx * ROWB + 16 * c16;        // + row*ROWB
    int32_t* my_rows = rows[wave];

    // lanes (grp, head) carry the softmax state of `head`; every lane carries the
    // accumulators of all heads for the V rows of its group and its 8 columns
    float m_run = -INFINITY, l_run = 0.f;
    float acc[G][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;

    auto fetch = [&](int t, KvTile& kv) {
        // tile t of the current block: K row of token 16t + c16, V rows of tokens 16t + 4grp + i.
        // Loads are unconditional (a guarded load would make the compiler wait for every
        // outstanding load and defeat the prefetch): a position past the end reads row 0,
        // its logit is masked to -inf and its weight is exactly 0.
        const int krow = max(my_rows[16 * t + c16], 0);
#pragma unroll
        for (int s = 0; s < 4; ++s) kv.k[s] = load16(Kbh, (size_t)krow * ROWB + 64 * s);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int vrow = max(my_rows[16 * t + 4 * grp + i], 0);
            kv.v[i] = load16(Vbh, (size_t)vrow * ROWB);
        }
    };

    auto consume = [&](const KvTile& kv, int n_valid) {
        // logits z[r] = token 4grp + r of the tile, head c16
        f32x4_t sacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < 4; ++s) sacc = mfma_16x16x32<T>(kv.k[s], qb[s], sacc);
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
            unpack<T>(kv.v[i], x);
            static_for<0, G>([&](auto gc) {
                constexpr int g = decltype(gc)::value;
                const float p = row_bcast<g>(z[i]);
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(p, x[e], acc[g][e]);
            });
        }
    };

    for (int blk = w0; blk < w1; blk += kMfmaWaveBlock) {
        const int nb = min(kMfmaWaveBlock, w1 - blk);
        // token position in the kept list -> row in the cache, for the whole block
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");      // earlier reads of my_rows are done
        {
            // a lane maps kMfmaWaveBlock/64 consecutive positions: one search, then a walk
            constexpr int PER = kMfmaWaveBlock / LEOAM_WAVE;
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

        const int n_tiles = (nb + 15) >> 4;
        KvTile cur, nxt;
        fetch(0, cur);
        if (n_tiles == 1) {      // nothing to prefetch: skip the pipeline's re-reads of the last tile
            consume(cur, nb);
            continue;
        }
        for (int t = 0; t < n_tiles; t += 2) {
            // (no loads under a condition: a tile index past the end re-reads the last tile)
            fetch(min(t + 1, n_tiles - 1), nxt);
            __builtin_amdgcn_sched_barrier(0);       // keep the loads ahead of the tile's arithmetic
            consume(cur, nb - 16 * t);
            fetch(min(t + 2, n_tiles - 1), cur);
            __builtin_amdgcn_sched_barrier(0);
            if (t + 1 < n_tiles) consume(nxt, nb - 16 * (t + 1));
        }
    }

    // ---- fold the four lane groups (same m everywhere in the wave) ---------------
    // (four accumulators at a time by lane swaps: afterwards lane group r holds the total of
    // accumulator e_own of the quad, so all 64 lanes write to LDS)
    l_run = rows_sum4(l_run, l_run, l_run, l_run);
    const int e_own = ((grp & 1) << 1) | (grp >> 1);        // rows 0,1,2,3 own accumulators 0,2,1,3
    static_assert(EPL == 8, "two quads of accumulators per head");
#pragma unroll
    for (int g = 0; g < G; ++g) {
        xw[wave][g][c16 * EPL + e_own] = rows_sum4(acc[g][0], acc[g][1], acc[g][2], acc[g][3]);
        xw[wave][g][c16 * EPL + 4 + e_own] = rows_sum4(acc[g][4], acc[g][5], acc[g][6], acc[g][7]);
    }
    if (grp == 0 && c16 < G) {
        xw[wave][c16][LEOAM_D] = m_run;
        xw[wave][c16][LEOAM_D + 1] = l_run;
    }
    finish_split<G>(xw, partial, b, h, split, n_splits, n_kv_heads, mg);
}

hipError_t launch_attention_merge(const leoam_shape* s, const float* partial, int n_splits, float* out, float* lse,
                                  hipStream_t stream) {
    hipLaunchKernelGGL(attention_merge_kernel, dim3(s->batch * s->n_q_heads), dim3(LEOAM_D * kMergeParts), 0, stream,
                       partial, n_splits, out, lse);
    return hipGetLastError();
}

static inline size_t part_bytes_per_split(const leoam_shape* s) {
    return (size_t)s->batch * s->n_q_heads * kPartStride * sizeof(float);
}

int attention_recommended_splits(const leoam_shape* s, int max_tokens) {
    if (max_tokens <= 0 || max_tokens > s->n_ctx) max_tokens = s->n_ctx;
    // smallest range a workgroup takes: one tile per lane group (fp32) / one 16-token tile per wave
    const int granule = (s->kv_dtype == LEOAM_F32) ? kAttWaves * 2 * kAttRows
                        : (s->kv_dtype == LEOAM_Q8Q4) ? kAttWaves * 4 * 4 : kMfmaGranule;
    const int by_tokens = (max_tokens + granule - 1) / granule;
    const int units = s->batch * s->n_kv_heads;
    // about three resident workgroups per compute unit; the compressed store is latency-bound at the
    // sizes it is used at (a split pays two dependent table look-ups before its first row arrives), and
    // one workgroup per compute unit with twice the tokens measured faster than two
    const int g = s->n_q_heads / s->n_kv_heads;
    const int target = (s->kv_dtype == LEOAM_Q8Q4) ? (g <= 4 ? 256 : 512) : 768;
    int want = (target + units - 1) / units;
    if (want > by_tokens) want = by_tokens;
    if (want > kAttMaxSplits) want = kAttMaxSplits;
    if (want < 1) want = 1;
    return want;
}

size_t attention_workspace_bytes(const leoam_shape* s, int max_tokens) {
    return part_bytes_per_split(s) * (size_t)attention_recommended_splits(s, max_tokens);
}

size_t attention_min_workspace_bytes(const leoam_shape* s) { return part_bytes_per_split(s); }

template <typename T, int G>
static hipError_t launch_attention(const leoam_shape* s, const void* q, const void* K, const void* V,
                                   const int32_t* chunk_off, const int32_t* n_chunks, const int32_t* sel_idx,
                                   const int32_t* sel_count, float scale, float* out, float* lse, void* workspace,
                                   int n_splits, int32_t* arrivals, hipStream_t stream) {
    dim3 grid(n_splits, s->n_kv_heads, s->batch);
    // merging in the launch pays while one workgroup can fetch all partials in a round trip or two
    if (n_splits > kInLaunchMaxSplits) arrivals = nullptr;
    const MergeInLaunch mg = {arrivals, out, lse};
    const size_t dyn = (size_t)(2 * s->k_max + 1) * sizeof(int32_t);
    float* ws = (float*)workspace;
    if constexpr (T::kBytes == 2)
        hipLaunchKernelGGL((sparse_attention_mfma_kernel<T, G>), grid, dim3(kAttThreads), dyn, stream, (const char*)q,
                           (const char*)K, (const char*)V, chunk_off, n_chunks, sel_idx, sel_count, scale * kLog2e, ws,
                           n_splits, s->c_max, s->k_max, s->n_kv_heads, s->n_ctx, mg);
    else
        hipLaunchKernelGGL((sparse_attention_kernel<T, G>), grid, dim3(kAttThreads), dyn, stream, (const char*)q,
                           (const char*)K, (const char*)V, chunk_off, n_chunks, sel_idx, sel_count, scale * kLog2e, ws,
                           n_splits, s->c_max, s->k_max, s->n_kv_heads, s->n_ctx, mg);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || arrivals) return e;
    return launch_attention_merge(s, ws, n_splits, out, lse, stream);
}

template <typename T>
static hipError_t attention_by_group(const leoam_shape* s, const void* q, const void* K, const void* V,
                                     const int32_t* chunk_off, const int32_t* n_chunks, const int32_t* sel_idx,
                                     const int32_t* sel_count, float scale, float* out, float* lse, void* ws,
                                     int n_splits, int32_t* arrivals, hipStream_t stream) {
#define LEOAM_ATT(GG) \
    launch_attention<T, GG>(s, q, K, V, chunk_off, n_chunks, sel_idx, sel_count, scale, out, lse, ws, n_splits, arrivals, stream)
    switch (s->n_q_heads / s->n_kv_heads) {
    case 1: return LEOAM_ATT(1);
    case 2: return LEOAM_ATT(2);
    case 4: return LEOAM_ATT(4);
    default: return LEOAM_ATT(8);
    }
#undef LEOAM_ATT
}

int attention_max_sel() { return kAttMaxSel; }

hipError_t attention_q_dispatch(const leoam_shape* s, const void* q, const void* K, const void* V, const void* qmeta,
                                const int32_t* chunk_off, const int32_t* n_chunks, const int32_t* sel_idx,
                                const int32_t* sel_count, float scale, float* out, float* lse, float* ws, int n_splits,
                                int32_t* arrivals, hipStream_t stream);      // quant_store.hip

hipError_t attention_dispatch(const leoam_shape* s, const void* q, const void* K, const void* V, const void* qmeta,
                              const int32_t* chunk_off, const int32_t* n_chunks, const int32_t* sel_idx,
                              const int32_t* sel_count, float scale, float* out, float* lse, void* workspace,
                              size_t workspace_bytes, int32_t* arrivals, hipStream_t stream) {
    size_t n = workspace_bytes / part_bytes_per_split(s);
    const size_t cap = (size_t)attention_recommended_splits(s, s->n_ctx);
    if (n > cap) n = cap;
    const int n_splits = (int)n;
    void* ws = workspace;
    switch (s->kv_dtype) {
    case LEOAM_Q8Q4:
        return attention_q_dispatch(s, q, K, V, qmeta, chunk_off, n_chunks, sel_idx, sel_count, scale, out, lse, (float*)ws,
                                    n_splits, arrivals, stream);
    case LEOAM_F32:
        return attention_by_group<F32>(s, q, K, V, chunk_off, n_chunks, sel_idx, sel_count, scale, out, lse, ws, n_splits, arrivals, stream);
    case LEOAM_F16:
        return attention_by_group<F16>(s, q, K, V, chunk_off, n_chunks, sel_idx, sel_count, scale, out, lse, ws, n_splits, arrivals, stream);
    default:
        return attention_by_group<BF16>(s, q, K, V, chunk_off, n_chunks, sel_idx, sel_count, scale, out, lse, ws, n_splits, arrivals, stream);
    }
}

}  // namespace leoam
