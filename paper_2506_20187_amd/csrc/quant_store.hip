// Compressed KV store: abstract build and sparse decode attention over chunks
// stored as 8-bit or 4-bit codes (paper Sec. 4.4 "Dynamic KV compression": the
// price of compressed transfer is decompression on the GPU; Sec. 6.1: INT4).
//
// A stored value is scale*code + zero with one (scale, zero) per (b,h,chunk,
// tensor).  Because they are per-chunk scalars nothing is dequantised element by
// element in the attention kernel:
//   q . k_t         = scale_k * (q . code_t) + zero_k * sum_d q_d
//   sum_t p_t v_t   = sum_t (p_t * scale_v) code_t  +  (sum_t p_t * zero_v) * 1
// so the codes go straight from integer to float (exact) into the same fp32
// online-softmax pipeline as the dense kernels.
//
// Row layout: 8-bit chunks have 128-byte rows, 4-bit chunks 64-byte rows with
// channel 2i in the low nibble of byte i.  In both kernels 16 lanes share a row
// and a lane owns 8 consecutive channels (8 or 4 bytes).
#include "quant_common.h"

namespace leoam {

// the 8 codes of this lane's channels [8*c16, 8*c16+8) of the row at `row`
__device__ __forceinline__ void load_codes(const unsigned char* row, int bits, int c16, float* x) {
    if (bits == 8) {
        const uint2 w = *reinterpret_cast<const uint2*>(row + 8 * c16);
        x[0] = (float)(w.x & 0xffu); x[1] = (float)((w.x >> 8) & 0xffu);
        x[2] = (float)((w.x >> 16) & 0xffu); x[3] = (float)(w.x >> 24);
        x[4] = (float)(w.y & 0xffu); x[5] = (float)((w.y >> 8) & 0xffu);
        x[6] = (float)((w.y >> 16) & 0xffu); x[7] = (float)(w.y >> 24);
    } else {
        const uint32_t w = *reinterpret_cast<const uint32_t*>(row + 4 * c16);
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = (float)((w >> (4 * e)) & 0xfu);
    }
}
__device__ __forceinline__ void load_codes_int(const unsigned char* row, int bits, int c16, int* x) {
    if (bits == 8) {
        const uint2 w = *reinterpret_cast<const uint2*>(row + 8 * c16);
        x[0] = w.x & 0xffu; x[1] = (w.x >> 8) & 0xffu; x[2] = (w.x >> 16) & 0xffu; x[3] = w.x >> 24;
        x[4] = w.y & 0xffu; x[5] = (w.y >> 8) & 0xffu; x[6] = (w.y >> 16) & 0xffu; x[7] = w.y >> 24;
    } else {
        const uint32_t w = *reinterpret_cast<const uint32_t*>(row + 4 * c16);
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = (w >> (4 * e)) & 0xfu;
    }
}

// ---- outward rounding double -> binary16 ------------------------------------
__device__ __forceinline__ float float_next_up(float f) {
    uint32_t u = float_to_bits(f);
    if ((u & 0x7fffffffu) == 0) return bits_to_float(1u);           // +-0 -> smallest positive
    return bits_to_float((u & 0x80000000u) ? u - 1 : u + 1);
}
__device__ __forceinline__ uint16_t half_next_up(uint16_t h) {
    if ((h & 0x7fffu) == 0) return 1;
    return (h & 0x8000u) ? (uint16_t)(h - 1) : (uint16_t)(h + 1);
}
// smallest binary16 >= x (x finite), as bits
__device__ __forceinline__ uint16_t half_ceil_bits(double x) {
    float f = (float)x;                                              // nearest float
    if ((double)f < x) f = float_next_up(f);                         // smallest float >= x
    _Float16 h = (_Float16)f;                                        // nearest half
    uint16_t hb = __builtin_bit_cast(uint16_t, h);
    if ((float)h < f) hb = half_next_up(hb);                         // smallest half >= f
    return hb;
}
__device__ __forceinline__ uint16_t half_floor_bits(double x) { return (uint16_t)(half_ceil_bits(-x) ^ 0x8000u); }

// ---------------------------------------------------------------------------
// abstract of the stored values (paper Sec. 4.3), rounded outward to binary16.
// scale >= 0, so max over tokens of scale*code+zero = scale*max(code)+zero: the
// reduction runs on integer codes (exact), one evaluation per channel at the end.
// ---------------------------------------------------------------------------
constexpr int kQAbsWaves = 4;

__global__ __launch_bounds__(kQAbsWaves* LEOAM_WAVE) void abstract_build_q_kernel(
    const unsigned char* __restrict__ kblob, const QChunk* __restrict__ qmeta, const int32_t* __restrict__ chunk_off,
    const int32_t* __restrict__ n_chunks, uint16_t* __restrict__ abstract, int n_ctx, int c_max, int n_kv_heads) {
    const int b = blockIdx.z, h = blockIdx.y;
    const int wave = threadIdx.x / LEOAM_WAVE, lane = lane_id();
    const int grp = lane >> 4, c16 = lane & 15;
    const int C = min(max(n_chunks[b], 0), c_max);
    const int32_t* off = chunk_off + (size_t)b * (c_max + 1);
    const size_t bh = (size_t)b * n_kv_heads + h;
    uint16_t* Abh = abstract + bh * (size_t)c_max * 2 * LEOAM_D;

    for (int c = blockIdx.x * kQAbsWaves + wave; c < C; c += gridDim.x * kQAbsWaves) {
        const QChunk m = qmeta[bh * c_max + c];
        const int t0 = min(max(off[c], 0), n_ctx);
        const int t1 = min(max(off[c + 1], t0), n_ctx);
        const int rowb = (m.bits == 8) ? LEOAM_D : LEOAM_D / 2;
        const unsigned char* base = kblob + m.byte_off;
        int mx[8], mn[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            mx[e] = -1;
            mn[e] = 256;
        }
        // lane group grp walks rows grp, grp+4, ...; two rows in flight per lane
        int t = grp;
        const int n = t1 - t0;
        for (; t + 4 < n; t += 8) {
            int x0[8], x1[8];
            load_codes_int(base + (size_t)t * rowb, m.bits, c16, x0);
            load_codes_int(base + (size_t)(t + 4) * rowb, m.bits, c16, x1);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                mx[e] = max(mx[e], max(x0[e], x1[e]));
                mn[e] = min(mn[e], min(x0[e], x1[e]));
            }
        }
        for (; t < n; t += 4) {
            int x0[8];
            load_codes_int(base + (size_t)t * rowb, m.bits, c16, x0);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                mx[e] = max(mx[e], x0[e]);
                mn[e] = min(mn[e], x0[e]);
            }
        }
        // fold the four lane groups: pack (max, 255 - min) into one register per channel pair
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            int v = (mx[e] & 0x1ff) | ((mn[e] & 0x1ff) << 16);
#pragma unroll
            for (int msk = 16; msk < LEOAM_WAVE; msk <<= 1) {
                const int o = __shfl_xor(v, msk, LEOAM_WAVE);
                const int omx = (o << 23) >> 23, omn = o >> 16;             // 9-bit fields, max may be -1
                const int vmx = (v << 23) >> 23, vmn = v >> 16;
                v = (max(vmx, omx) & 0x1ff) | (min(vmn, omn) << 16);
            }
            mx[e] = (v << 23) >> 23;
            mn[e] = v >> 16;
        }
        if (grp < 2) {
            // group 0 writes kmax, group 1 writes kmin: 8 halves = 16 bytes per lane
            uint32_t w[4];
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                uint16_t h0, h1;
                if (n <= 0) {
                    h0 = h1 = (grp == 0) ? 0xfc00u : 0x7c00u;               // empty chunk: (-inf, +inf)
                } else if (grp == 0) {
                    h0 = half_ceil_bits((double)m.scale_k * mx[e] + (double)m.zero_k);
                    h1 = half_ceil_bits((double)m.scale_k * mx[e + 1] + (double)m.zero_k);
                } else {
                    h0 = half_floor_bits((double)m.scale_k * mn[e] + (double)m.zero_k);
                    h1 = half_floor_bits((double)m.scale_k * mn[e + 1] + (double)m.zero_k);
                }
                w[e / 2] = (uint32_t)h0 | ((uint32_t)h1 << 16);
            }
            store16(Abh, (((size_t)c * 2 + grp) * LEOAM_D + 8 * c16) * 2, make_uint4(w[0], w[1], w[2], w[3]));
        }
    }
}

// ---------------------------------------------------------------------------
// sparse decode attention over the compressed store (Eq. 1 over the kept chunks)
// ---------------------------------------------------------------------------
constexpr int kQGroups = kAttWaves * 4;            // 16-lane groups per workgroup
constexpr int kQRows = 4;                          // rows per lane group per tile
constexpr int kQTile = kQGroups * kQRows;          // tokens per tile (64)
constexpr int kQMaxSel = 1024;                     // kept chunks per (b,h) held in LDS

template <int G>
__global__ __launch_bounds__(kAttThreads) void sparse_attention_q_kernel(
    const char* __restrict__ q, const unsigned char* __restrict__ kblob, const unsigned char* __restrict__ vblob,
    const QChunk* __restrict__ qmeta, const int32_t* __restrict__ chunk_off, const int32_t* __restrict__ n_chunks,
    const int32_t* __restrict__ sel_idx, const int32_t* __restrict__ sel_count, float scale_log2,
    float* partial, int n_splits, int c_max, int k_max, int n_kv_heads, int n_ctx, MergeInLaunch mg) {
    constexpr int EPL = 8;
    __shared__ long long ch_off[kQMaxSel];
    __shared__ float4 ch_par[kQMaxSel];            // scale_k, zero_k, scale_v, zero_v
    __shared__ int32_t ch_bits[kQMaxSel];
    __shared__ int32_t prefix[kQMaxSel + 1];
    __shared__ float xw[kAttWaves][G][kPartStride];
    __shared__ int32_t sh_total;

    const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid / LEOAM_WAVE;
    const int grp = lane >> 4, c16 = lane & 15;
    const size_t bh = (size_t)b * n_kv_heads + h;
    const int C = min(max(n_chunks[b], 0), c_max);
    const int cnt = min(min(max(sel_count[bh], 0), k_max), kQMaxSel);
    const int32_t* off = chunk_off + (size_t)b * (c_max + 1);
    const int32_t* sel = sel_idx + bh * (size_t)k_max;

    for (int i = tid; i < cnt; i += kAttThreads) {
        const int id = sel[i];
        int sz = 0;
        QChunk m = {0, 8, 0.f, 0.f, 0.f, 0.f, 0};
        if (id >= 0 && id < C) {
            const int t0 = min(max(off[id], 0), n_ctx);
            sz = min(max(off[id + 1], t0), n_ctx) - t0;
            m = qmeta[bh * c_max + id];
        }
        ch_off[i] = m.byte_off;
        ch_bits[i] = m.bits;
        ch_par[i] = make_float4(m.scale_k, m.zero_k, m.scale_v, m.zero_v);
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
    int per_split = (total + n_splits - 1) / n_splits;
    per_split = ((per_split + kQTile - 1) / kQTile) * kQTile;
    const int r0 = min(total, split * per_split), r1 = min(total, r0 + per_split);

    // queries (fp16): this lane's 8 channels, pre-multiplied by scale*log2(e); and sum_d of them per head
    float qs[G][EPL], qsum[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const size_t qrow = ((size_t)b * n_kv_heads * G + (size_t)h * G + g) * (LEOAM_D * 2);
        float x[EPL];
        unpack<F16>(load16(q, qrow + 16 * c16), x);
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            qs[g][e] = x[e] * scale_log2;
            s += qs[g][e];
        }
        qsum[g] = row16_sum(s);
    }

    float m_run[G], l_run[G], accz[G], acc[G][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m_run[g] = -INFINITY;
        l_run[g] = 0.f;
        accz[g] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
    }

    // From here on the four waves are independent streams: a wave takes a contiguous quarter of
    // the split's range and walks it in tiles of 16 tokens, lane group grp holding tokens
    // 4*grp .. 4*grp+3 of the tile.  The raw codes of the next tile are in flight while this one
    // is expanded and used.  All loads are unconditional (a token past the end re-reads the last
    // one and gets weight 0); the chunk slot of a token is found by walking the prefix table
    // forward from the previous token's slot.
    const int per_wave = per_split / kAttWaves;
    const int w0 = min(r1, r0 + wave * per_wave), w1 = min(r1, w0 + per_wave);
    struct RawRows {
        uint32_t k0[kQRows], k1[kQRows], v0[kQRows], v1[kQRows];      // two dwords per row and tensor
        int slot[kQRows];                                             // kept-list slot of the row's chunk, -1 = no token
    };
    int lo = 0;
    if (w0 < w1) {
        const int x = min(w0 + kQRows * grp, w1 - 1);
        int hi = cnt;                  // largest k with prefix[k] <= x
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (prefix[mid] <= x) lo = mid; else hi = mid;
        }
    }
    auto fetch = [&](int tb, RawRows& R) {
#pragma unroll
        for (int j = 0; j < kQRows; ++j) {
            const int x = tb + kQRows * grp + j, xx = min(x, w1 - 1);
            while (prefix[lo + 1] <= xx) ++lo;      // ends: prefix[cnt] = total > xx
            const int bits = ch_bits[lo];
            const size_t row = (size_t)ch_off[lo] + (size_t)(xx - prefix[lo]) * (bits == 8 ? LEOAM_D : LEOAM_D / 2);
            // 8-bit rows: this lane's 8 bytes as two dwords; 4-bit rows: its 4 bytes (read twice)
            const size_t a0 = row + (bits == 8 ? 8 : 4) * c16, a1 = a0 + (bits == 8 ? 4 : 0);
            R.k0[j] = *reinterpret_cast<const uint32_t*>(kblob + a0);
            R.k1[j] = *reinterpret_cast<const uint32_t*>(kblob + a1);
            R.v0[j] = *reinterpret_cast<const uint32_t*>(vblob + a0);
            R.v1[j] = *reinterpret_cast<const uint32_t*>(vblob + a1);
            R.slot[j] = (x < w1) ? lo : -1;
        }
    };
    auto expand = [&](uint32_t w0_, uint32_t w1_, int bits, float* x) {
        if (bits == 8) {
            x[0] = (float)(w0_ & 0xffu); x[1] = (float)((w0_ >> 8) & 0xffu);
            x[2] = (float)((w0_ >> 16) & 0xffu); x[3] = (float)(w0_ >> 24);
            x[4] = (float)(w1_ & 0xffu); x[5] = (float)((w1_ >> 8) & 0xffu);
            x[6] = (float)((w1_ >> 16) & 0xffu); x[7] = (float)(w1_ >> 24);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = (float)((w0_ >> (4 * e)) & 0xfu);
        }
    };
    auto consume = [&](const RawRows& R) {
        float z[kQRows][G], sv[kQRows], zv[kQRows];
        int bits_of[kQRows];
        float mt[G];
#pragma unroll
        for (int g = 0; g < G; ++g) mt[g] = m_run[g];
#pragma unroll
        for (int j = 0; j < kQRows; ++j) {
            const int kk = max(R.slot[j], 0);
            const float4 par = ch_par[kk];
            bits_of[j] = ch_bits[kk];
            sv[j] = par.z;
            zv[j] = par.w;
            float kx[EPL];
            expand(R.k0[j], R.k1[j], bits_of[j], kx);
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float d = 0.f;
#pragma unroll
                for (int e = 0; e < EPL; ++e) d = fmaf(qs[g][e], kx[e], d);
                d = row16_sum(d);
                z[j][g] = (R.slot[j] >= 0) ? fmaf(par.x, d, par.y * qsum[g]) : -INFINITY;
                mt[g] = fmaxf(mt[g], z[j][g]);
            }
        }
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float corr = exp2_or_zero(m_run[g], mt[g]);
            m_run[g] = mt[g];
            l_run[g] *= corr;
            accz[g] *= corr;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[g][e] *= corr;
        }
#pragma unroll
        for (int j = 0; j < kQRows; ++j) {
            float vx[EPL];
            expand(R.v0[j], R.v1[j], bits_of[j], vx);
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float p = exp2_or_zero(z[j][g], m_run[g]);
                l_run[g] += p;
                accz[g] = fmaf(p, zv[j], accz[g]);
                const float ps = p * sv[j];
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(ps, vx[e], acc[g][e]);
            }
        }
    };
    if (w0 < w1) {
        constexpr int kWaveTile = 4 * kQRows;        // tokens of a wave's tile
        RawRows cur, nxt;
        fetch(w0, cur);
        for (int tb = w0; tb < w1; tb += 2 * kWaveTile) {
            fetch(tb + kWaveTile, nxt);
            __builtin_amdgcn_sched_barrier(0);       // keep the loads ahead of the tile's arithmetic
            consume(cur);
            fetch(tb + 2 * kWaveTile, cur);
            __builtin_amdgcn_sched_barrier(0);
            if (tb + kWaveTile < w1) consume(nxt);
        }
    }
    // the zero-point share is the same for every channel: fold it in, then merge as usual
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] += accz[g];

#pragma unroll
    for (int msk = 16; msk < LEOAM_WAVE; msk <<= 1) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float m_o = shfl_xor_f(m_run[g], msk);
            const float l_o = shfl_xor_f(l_run[g], msk);
            const float m_n = fmaxf(m_run[g], m_o);
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
    if (grp == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) xw[wave][g][c16 * EPL + e] = acc[g][e];
            if (lane == 0) {
                xw[wave][g][LEOAM_D] = m_run[g];
                xw[wave][g][LEOAM_D + 1] = l_run[g];
            }
        }
    }
    finish_split<G>(xw, partial, b, h, split, n_splits, n_kv_heads, mg);
}

// ---------------------------------------------------------------------------
// The same attention with q K^T on the matrix cores (group sizes 1, 2, 4).
//
// v_mfma_f32_16x16x32_f16: A lane = (token = lane%16, 8 of the 32 channels of the
// step: 8*(lane/16)..+8), B lane = (head = lane%16, same channels), D lane =
// (head = lane%16, tokens 4*(lane/16)..+4).  The codes of a lane's 8 channels are
// one or two dwords; they become the f16 operand without a conversion
// instruction per element: the bytes (nibbles spread to bytes for a 4-bit row)
// are paired into the 16-bit halves of a dword by v_perm_b32, or-ed with 0x6400
// (the f16 1024, whose low mantissa bits then hold the code) and a packed
// subtraction of 1024 leaves the exact codes.  Both formats produce the channel
// order (0,2,4,6,1,3,5,7) inside a lane's 8 channels - the per-lane selector of
// the byte permutation differs, nothing else - and the query operand is stored in
// that order, so a tile may mix 8-bit and 4-bit tokens.  The logit of a token is
// scale_k * (q . code) + zero_k * sum(q), applied to the MFMA result.  P V stays
// on the vector ALU in fp32 as in the dense kernel: v_cvt_f32_ubyte turns codes
// into floats, the weight is pre-multiplied by scale_v, and zero_v's share is
// accumulated once per token.
// ---------------------------------------------------------------------------
constexpr int kQmBlock = 256;                      // positions a wave maps to chunk slots at a time
constexpr int kQmGranule = kAttWaves * 16;         // a split is a multiple of this many tokens

template <int G>
__global__ __launch_bounds__(kAttThreads) void sparse_attention_qm_kernel(
    const char* __restrict__ q, const unsigned char* __restrict__ kblob, const unsigned char* __restrict__ vblob,
    const QChunk* __restrict__ qmeta, const int32_t* __restrict__ chunk_off, const int32_t* __restrict__ n_chunks,
    const int32_t* __restrict__ sel_idx, const int32_t* __restrict__ sel_count, float scale_log2,
    float* partial, int n_splits, int c_max, int k_max, int n_kv_heads, int n_ctx, MergeInLaunch mg) {
    static_assert(G <= 4, "one MFMA column per head, four accumulator sets per lane");
    constexpr int EPL = 8;
    __shared__ long long ch_off[kQMaxSel];
    __shared__ float4 ch_par[kQMaxSel];            // scale_k, zero_k, scale_v, zero_v
    __shared__ int32_t ch_bits[kQMaxSel];
    __shared__ int32_t prefix[kQMaxSel + 1];
    __shared__ int32_t pos_slot[kAttWaves][kQmBlock], pos_tin[kAttWaves][kQmBlock];
    __shared__ float xw[kAttWaves][G][kPartStride];
    __shared__ int32_t sh_total;

    const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid / LEOAM_WAVE;
    const int grp = lane >> 4, c16 = lane & 15;
    const size_t bh = (size_t)b * n_kv_heads + h;
    const int C = min(max(n_chunks[b], 0), c_max);
    const int cnt = min(min(max(sel_count[bh], 0), k_max), kQMaxSel);
    const int32_t* off = chunk_off + (size_t)b * (c_max + 1);
    const int32_t* sel = sel_idx + bh * (size_t)k_max;

    // ---- B operand: the group's queries in the channel order of the code operand; sum_d q per head ----
    uint4 qb[4];
    float qsum = 0.f;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        qb[s] = make_uint4(0, 0, 0, 0);
        if (c16 < G) {
            const size_t qrow = ((size_t)b * n_kv_heads * G + (size_t)h * G + c16) * (LEOAM_D * 2);
            const uint4 raw = load16(q, qrow + 64 * s + 16 * grp);          // channels 32s + 8grp + 0..7
            qb[s] = query_operand(raw);
            float x[EPL];
            unpack<F16>(raw, x);
#pragma unroll
            for (int e = 0; e < EPL; ++e) qsum += x[e];
        }
    }
    qsum += shfl_xor_f(qsum, 16);
    qsum += shfl_xor_f(qsum, 32);

    // ---- kept chunks: records and token prefix ------------------------------------------
    for (int i = tid; i < cnt; i += kAttThreads) {
        const int id = sel[i];
        int sz = 0;
        QChunk m = {0, 8, 0.f, 0.f, 0.f, 0.f, 0};
        if (id >= 0 && id < C) {
            const int t0 = min(max(off[id], 0), n_ctx);
            sz = min(max(off[id + 1], t0), n_ctx) - t0;
            m = qmeta[bh * c_max + id];
        }
        ch_off[i] = m.byte_off;
        ch_bits[i] = m.bits;
        ch_par[i] = make_float4(m.scale_k, m.zero_k, m.scale_v, m.zero_v);
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
    int per_split = (total + n_splits - 1) / n_splits;
    per_split = ((per_split + kQmGranule - 1) / kQmGranule) * kQmGranule;
    const int r0 = min(total, split * per_split), r1 = min(total, r0 + per_split);
    const int per_wave = per_split / kAttWaves;
    const int w0 = min(r1, r0 + wave * per_wave), w1 = min(r1, w0 + per_wave);
    int32_t* my_slot = pos_slot[wave];
    int32_t* my_tin = pos_tin[wave];

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

    auto consume = [&](const QmTile& kv) {
        const f32x4_t sacc = code_logits(kv, [&](int s) { return qb[s]; });
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

    for (int blk = w0; blk < w1; blk += kQmBlock) {
        const int nb = min(kQmBlock, w1 - blk);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");      // earlier reads of the tables are done
        {
            // a lane maps kQmBlock/64 consecutive positions: one search, then a walk
            constexpr int PER = kQmBlock / LEOAM_WAVE;
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
                    while (prefix[lo + 1] <= x) ++lo;      // ends: prefix[cnt] = total > x
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

        const int n_tiles = (nb + 15) >> 4;
        QmTile cur, nxt;
        fetch(0, cur);
        if (n_tiles == 1) {
            consume(cur);
            continue;
        }
        for (int t = 0; t < n_tiles; t += 2) {
            fetch(min(t + 1, n_tiles - 1), nxt);
            __builtin_amdgcn_sched_barrier(0);       // keep the loads ahead of the tile's arithmetic
            consume(cur);
            fetch(min(t + 2, n_tiles - 1), cur);
            __builtin_amdgcn_sched_barrier(0);
            if (t + 1 < n_tiles) consume(nxt);
        }
    }

    // ---- fold the four lane groups (same m everywhere in the wave); zero_v's share is the same for
    // every channel ---------------------------------------------------------------------------------
    // (four accumulators at a time by lane swaps: afterwards lane group r holds the total of
    // accumulator e_own of the quad, so all 64 lanes write to LDS)
    l_run = rows_sum4(l_run, l_run, l_run, l_run);
    const int e_own = ((grp & 1) << 1) | (grp >> 1);        // rows 0,1,2,3 own accumulators 0,2,1,3
    static_assert(EPL == 8, "two quads of accumulators per head");
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const float f0 = rows_sum4(acc[g][0] + accz[g], acc[g][1] + accz[g], acc[g][2] + accz[g], acc[g][3] + accz[g]);
        const float f1 = rows_sum4(acc[g][4] + accz[g], acc[g][5] + accz[g], acc[g][6] + accz[g], acc[g][7] + accz[g]);
        // accumulator e holds channel code_channel(e) = 2e (e < 4) or 2(e - 4) + 1
        xw[wave][g][c16 * EPL + 2 * e_own] = f0;
        xw[wave][g][c16 * EPL + 2 * e_own + 1] = f1;
    }
    if (grp == 0 && c16 < G) {
        xw[wave][c16][LEOAM_D] = m_run;
        xw[wave][c16][LEOAM_D + 1] = l_run;
    }
    finish_split<G>(xw, partial, b, h, split, n_splits, n_kv_heads, mg);
}

int attention_q_max_sel() { return kQMaxSel; }

hipError_t abstract_build_q_dispatch(const leoam_shape* s, const void* kblob, const void* qmeta,
                                     const int32_t* chunk_off, const int32_t* n_chunks, void* abstract,
                                     hipStream_t stream) {
    int gx = (s->c_max + kQAbsWaves - 1) / kQAbsWaves;
    if (gx > 8192) gx = 8192;
    dim3 grid(gx, s->n_kv_heads, s->batch);
    hipLaunchKernelGGL(abstract_build_q_kernel, grid, dim3(kQAbsWaves * LEOAM_WAVE), 0, stream,
                       (const unsigned char*)kblob, (const QChunk*)qmeta, chunk_off, n_chunks, (uint16_t*)abstract,
                       s->n_ctx, s->c_max, s->n_kv_heads);
    return hipGetLastError();
}

hipError_t attention_q_dispatch(const leoam_shape* s, const void* q, const void* K, const void* V, const void* qmeta,
                                const int32_t* chunk_off, const int32_t* n_chunks, const int32_t* sel_idx,
                                const int32_t* sel_count, float scale, float* out, float* lse, float* ws, int n_splits,
                                int32_t* arrivals, hipStream_t stream) {
    dim3 grid(n_splits, s->n_kv_heads, s->batch);
    if (n_splits > kInLaunchMaxSplits) arrivals = nullptr;      // many splits: the merge kernel is faster
    const MergeInLaunch mg = {arrivals, out, lse};
#define LEOAM_ATTQ(GG)                                                                                                  \
    hipLaunchKernelGGL((sparse_attention_q_kernel<GG>), grid, dim3(kAttThreads), 0, stream, (const char*)q,            \
                       (const unsigned char*)K, (const unsigned char*)V, (const QChunk*)qmeta, chunk_off, n_chunks,     \
                       sel_idx, sel_count, scale * kLog2e, ws, n_splits, s->c_max, s->k_max, s->n_kv_heads, s->n_ctx, mg)
#define LEOAM_ATTQM(GG)                                                                                                 \
    hipLaunchKernelGGL((sparse_attention_qm_kernel<GG>), grid, dim3(kAttThreads), 0, stream, (const char*)q,           \
                       (const unsigned char*)K, (const unsigned char*)V, (const QChunk*)qmeta, chunk_off, n_chunks,     \
                       sel_idx, sel_count, scale * kLog2e, ws, n_splits, s->c_max, s->k_max, s->n_kv_heads, s->n_ctx, mg)
    switch (s->n_q_heads / s->n_kv_heads) {
    case 1: LEOAM_ATTQM(1); break;
    case 2: LEOAM_ATTQM(2); break;
    case 4: LEOAM_ATTQM(4); break;
    default: LEOAM_ATTQ(8); break;
    }
#undef LEOAM_ATTQ
#undef LEOAM_ATTQM
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || arrivals) return e;
    return launch_attention_merge(s, ws, n_splits, out, lse, stream);
}

}  // namespace leoam
