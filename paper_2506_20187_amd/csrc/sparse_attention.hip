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

template <typename T, int G>
__global__ __launch_bounds__(kAttThreads) void sparse_attention_kernel(
    const char* __restrict__ q, const char* __restrict__ K, const char* __restrict__ V,
    const int32_t* __restrict__ chunk_off, const int32_t* __restrict__ n_chunks, const int32_t* __restrict__ sel_idx,
    const int32_t* __restrict__ sel_count, float scale_log2, float* __restrict__ partial, int n_splits, int c_max,
    int k_max, int n_kv_heads, int n_ctx) {
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
    __syncthreads();
    float* part = partial + (((size_t)b * n_kv_heads * G + (size_t)h * G) * n_splits + 0) * kPartStride;
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
        part[((size_t)g * n_splits + split) * kPartStride + d] = v;
    }
}

// out[b,j,:] = sum_s 2^(m_s - m) o_s / sum_s 2^(m_s - m) l_s, splits in index order
__global__ __launch_bounds__(LEOAM_D) void attention_merge_kernel(const float* __restrict__ partial, int n_splits,
                                                                 float* __restrict__ out, float* __restrict__ lse) {
    const size_t bj = blockIdx.x;
    const int d = threadIdx.x;
    const float* part = partial + bj * (size_t)n_splits * kPartStride;
    float m = -INFINITY;
    for (int s = 0; s < n_splits; ++s) m = fmaxf(m, part[(size_t)s * kPartStride + LEOAM_D]);
    float o = 0.f, l = 0.f;
    for (int s = 0; s < n_splits; ++s) {
        const float a = exp2_or_zero(part[(size_t)s * kPartStride + LEOAM_D], m);
        o += a * part[(size_t)s * kPartStride + d];
        l += a * part[(size_t)s * kPartStride + LEOAM_D + 1];
    }
    out[bj * LEOAM_D + d] = (l > 0.f) ? o / l : 0.f;
    if (lse && d == 0) lse[bj] = (l > 0.f) ? (m + log2f(l)) * kLn2 : -INFINITY;
}

static inline size_t part_bytes_per_split(const leoam_shape* s) {
    return (size_t)s->batch * s->n_q_heads * kPartStride * sizeof(float);
}

int attention_recommended_splits(const leoam_shape* s, int max_tokens) {
    if (max_tokens <= 0 || max_tokens > s->n_ctx) max_tokens = s->n_ctx;
    const int rpl = (s->kv_dtype == LEOAM_F32) ? 2 : 4;
    const int tile = kAttWaves * rpl * kAttRows;
    const int by_tokens = (max_tokens + tile - 1) / tile;
    const int units = s->batch * s->n_kv_heads;
    int want = (2048 + units - 1) / units;       // ~8 workgroups per compute unit in total
    if (want > by_tokens) want = by_tokens;
    if (want > kAttMaxSplits) want = kAttMaxSplits;
    if (want < 1) want = 1;
    return want;
}

size_t attention_workspace_bytes(const leoam_shape* s, int max_tokens) {
    return part_bytes_per_split(s) * (size_t)attention_recommended_splits(s, max_tokens);
}

template <typename T, int G>
static hipError_t launch_attention(const leoam_shape* s, const void* q, const void* K, const void* V,
                                   const int32_t* chunk_off, const int32_t* n_chunks, const int32_t* sel_idx,
                                   const int32_t* sel_count, float scale, float* out, float* lse, float* ws,
                                   int n_splits, hipStream_t stream) {
    dim3 grid(n_splits, s->n_kv_heads, s->batch);
    const size_t dyn = (size_t)(2 * s->k_max + 1) * sizeof(int32_t);
    hipLaunchKernelGGL((sparse_attention_kernel<T, G>), grid, dim3(kAttThreads), dyn, stream, (const char*)q,
                       (const char*)K, (const char*)V, chunk_off, n_chunks, sel_idx, sel_count, scale * kLog2e, ws,
                       n_splits, s->c_max, s->k_max, s->n_kv_heads, s->n_ctx);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(attention_merge_kernel, dim3(s->batch * s->n_q_heads), dim3(LEOAM_D), 0, stream, ws, n_splits, out,
                       lse);
    return hipGetLastError();
}

template <typename T>
static hipError_t attention_by_group(const leoam_shape* s, const void* q, const void* K, const void* V,
                                     const int32_t* chunk_off, const int32_t* n_chunks, const int32_t* sel_idx,
                                     const int32_t* sel_count, float scale, float* out, float* lse, float* ws,
                                     int n_splits, hipStream_t stream) {
#define LEOAM_ATT(GG) \
    launch_attention<T, GG>(s, q, K, V, chunk_off, n_chunks, sel_idx, sel_count, scale, out, lse, ws, n_splits, stream)
    switch (s->n_q_heads / s->n_kv_heads) {
    case 1: return LEOAM_ATT(1);
    case 2: return LEOAM_ATT(2);
    case 4: return LEOAM_ATT(4);
    default: return LEOAM_ATT(8);
    }
#undef LEOAM_ATT
}

int attention_max_sel() { return kAttMaxSel; }

hipError_t attention_dispatch(const leoam_shape* s, const void* q, const void* K, const void* V,
                              const int32_t* chunk_off, const int32_t* n_chunks, const int32_t* sel_idx,
                              const int32_t* sel_count, float scale, float* out, float* lse, void* workspace,
                              size_t workspace_bytes, hipStream_t stream) {
    size_t n = workspace_bytes / part_bytes_per_split(s);
    const size_t cap = (size_t)attention_recommended_splits(s, s->n_ctx);
    if (n > cap) n = cap;
    const int n_splits = (int)n;
    float* ws = (float*)workspace;
    switch (s->kv_dtype) {
    case LEOAM_F32:
        return attention_by_group<F32>(s, q, K, V, chunk_off, n_chunks, sel_idx, sel_count, scale, out, lse, ws, n_splits, stream);
    case LEOAM_F16:
        return attention_by_group<F16>(s, q, K, V, chunk_off, n_chunks, sel_idx, sel_count, scale, out, lse, ws, n_splits, stream);
    default:
        return attention_by_group<BF16>(s, q, K, V, chunk_off, n_chunks, sel_idx, sel_count, scale, out, lse, ws, n_splits, stream);
    }
}

}  // namespace leoam
