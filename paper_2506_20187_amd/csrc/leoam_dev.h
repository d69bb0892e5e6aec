// Device-side helpers shared by the gfx950 kernels: 16-byte row loads, storage
// type unpacking, wave-level reductions.  64-wide wavefronts throughout.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/leoam.h"

#define LEOAM_D 128
#define LEOAM_WAVE 64

namespace leoam {

// ---- storage types ---------------------------------------------------------
// A lane always moves 16 bytes of a row: EPL elements.
struct F32 { static constexpr int kBytes = 4; static constexpr int kEpl = 4; static constexpr int kTag = LEOAM_F32; };
struct F16 { static constexpr int kBytes = 2; static constexpr int kEpl = 8; static constexpr int kTag = LEOAM_F16; };
struct BF16 { static constexpr int kBytes = 2; static constexpr int kEpl = 8; static constexpr int kTag = LEOAM_BF16; };

template <typename T> struct Row {
    static constexpr int kLanesPerRow = LEOAM_D / T::kEpl;            // 32 (fp32) or 16
    static constexpr int kRowsPerLoad = LEOAM_WAVE / kLanesPerRow;    // 2 or 4
    static constexpr int kRowBytes = LEOAM_D * T::kBytes;
};

__device__ __forceinline__ float bits_to_float(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t float_to_bits(float f) { return __builtin_bit_cast(uint32_t, f); }

// unpack the 16 bytes a lane holds into floats (exact widening)
template <typename T> __device__ __forceinline__ void unpack(const uint4& v, float* x);

template <> __device__ __forceinline__ void unpack<F32>(const uint4& v, float* x) {
    x[0] = bits_to_float(v.x); x[1] = bits_to_float(v.y); x[2] = bits_to_float(v.z); x[3] = bits_to_float(v.w);
}
template <> __device__ __forceinline__ void unpack<BF16>(const uint4& v, float* x) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        x[2 * i] = bits_to_float(w[i] << 16);
        x[2 * i + 1] = bits_to_float(w[i] & 0xffff0000u);
    }
}
template <> __device__ __forceinline__ void unpack<F16>(const uint4& v, float* x) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        x[2 * i] = (float)__builtin_bit_cast(_Float16, (uint16_t)(w[i] & 0xffffu));
        x[2 * i + 1] = (float)__builtin_bit_cast(_Float16, (uint16_t)(w[i] >> 16));
    }
}

// pack floats that are exactly representable in T back into 16 bytes
template <typename T> __device__ __forceinline__ uint4 pack(const float* x);
template <> __device__ __forceinline__ uint4 pack<F32>(const float* x) {
    return make_uint4(float_to_bits(x[0]), float_to_bits(x[1]), float_to_bits(x[2]), float_to_bits(x[3]));
}
template <> __device__ __forceinline__ uint4 pack<BF16>(const float* x) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = (float_to_bits(x[2 * i]) >> 16) | (float_to_bits(x[2 * i + 1]) & 0xffff0000u);
    return make_uint4(w[0], w[1], w[2], w[3]);
}
template <> __device__ __forceinline__ uint4 pack<F16>(const float* x) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        uint32_t lo = __builtin_bit_cast(uint16_t, (_Float16)x[2 * i]);
        uint32_t hi = __builtin_bit_cast(uint16_t, (_Float16)x[2 * i + 1]);
        w[i] = lo | (hi << 16);
    }
    return make_uint4(w[0], w[1], w[2], w[3]);
}

__device__ __forceinline__ uint4 load16(const void* base, size_t byte_off) {
    return *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(base) + byte_off);
}
__device__ __forceinline__ void store16(void* base, size_t byte_off, const uint4& v) {
    *reinterpret_cast<uint4*>(reinterpret_cast<char*>(base) + byte_off) = v;
}

// ---- wave-level helpers ------------------------------------------------------
__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (LEOAM_WAVE - 1)); }

__device__ __forceinline__ float shfl_xor_f(float v, int mask) { return __shfl_xor(v, mask, LEOAM_WAVE); }
__device__ __forceinline__ double shfl_xor_d(double v, int mask) { return __shfl_xor(v, mask, LEOAM_WAVE); }

// DPP lane exchanges inside a 16-lane row.  Applied to values that are already
// uniform inside the smaller groups these turn into xor-butterfly steps:
//   0xB1 quad_perm [1,0,3,2]  (xor 1)        0x4E quad_perm [2,3,0,1]  (xor 2)
//   0x141 row_half_mirror (lane i <-> 7-i)   0x140 row_mirror (lane i <-> 15-i)
template <int kCtrl> __device__ __forceinline__ float dpp_f(float v) {
    int x = __builtin_bit_cast(int, v);
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(x, x, kCtrl, 0xf, 0xf, false));
}

// sum over the 16 lanes of a DPP row; every lane of the row gets the total
__device__ __forceinline__ float row16_sum(float v) {
    v += dpp_f<0xB1>(v);
    v += dpp_f<0x4E>(v);
    v += dpp_f<0x141>(v);
    v += dpp_f<0x140>(v);
    return v;
}

// ---- wave-wide scans and reductions on the DPP data path --------------------------
// row_shr:n (0x110+n) shifts inside a 16-lane row, row_bcast:15 (0x142) / row_bcast:31
// (0x143) carry a row's last lane into the following rows; lanes without a source
// take `kIdentity`.  Six steps give an inclusive scan over the 64 lanes without
// touching LDS.
template <int kCtrl, int kRowMask, uint32_t kIdentity> __device__ __forceinline__ uint32_t dpp_or_identity(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp((int)kIdentity, (int)v, kCtrl, kRowMask, 0xf, false);
}

__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t v) {
    v += dpp_or_identity<0x111, 0xf, 0u>(v);
    v += dpp_or_identity<0x112, 0xf, 0u>(v);
    v += dpp_or_identity<0x114, 0xf, 0u>(v);
    v += dpp_or_identity<0x118, 0xf, 0u>(v);
    v += dpp_or_identity<0x142, 0xa, 0u>(v);
    v += dpp_or_identity<0x143, 0xc, 0u>(v);
    return v;
}

// inclusive scan inside every 16-lane row
__device__ __forceinline__ uint32_t row16_incl_scan_u32(uint32_t v) {
    v += dpp_or_identity<0x111, 0xf, 0u>(v);
    v += dpp_or_identity<0x112, 0xf, 0u>(v);
    v += dpp_or_identity<0x114, 0xf, 0u>(v);
    v += dpp_or_identity<0x118, 0xf, 0u>(v);
    return v;
}

// minimum / maximum over the wave; every lane gets the result
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
    v = min(v, dpp_or_identity<0x111, 0xf, 0xffffffffu>(v));
    v = min(v, dpp_or_identity<0x112, 0xf, 0xffffffffu>(v));
    v = min(v, dpp_or_identity<0x114, 0xf, 0xffffffffu>(v));
    v = min(v, dpp_or_identity<0x118, 0xf, 0xffffffffu>(v));
    v = min(v, dpp_or_identity<0x142, 0xa, 0xffffffffu>(v));
    v = min(v, dpp_or_identity<0x143, 0xc, 0xffffffffu>(v));
    return (uint32_t)__builtin_amdgcn_readlane((int)v, LEOAM_WAVE - 1);
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
    v = max(v, dpp_or_identity<0x111, 0xf, 0u>(v));
    v = max(v, dpp_or_identity<0x112, 0xf, 0u>(v));
    v = max(v, dpp_or_identity<0x114, 0xf, 0u>(v));
    v = max(v, dpp_or_identity<0x118, 0xf, 0u>(v));
    v = max(v, dpp_or_identity<0x142, 0xa, 0u>(v));
    v = max(v, dpp_or_identity<0x143, 0xc, 0u>(v));
    return (uint32_t)__builtin_amdgcn_readlane((int)v, LEOAM_WAVE - 1);
}
// minimum / maximum over the first 16 lanes; every lane gets the result
__device__ __forceinline__ uint32_t row0_min_u32(uint32_t v) {
    v = min(v, dpp_or_identity<0x111, 0xf, 0xffffffffu>(v));
    v = min(v, dpp_or_identity<0x112, 0xf, 0xffffffffu>(v));
    v = min(v, dpp_or_identity<0x114, 0xf, 0xffffffffu>(v));
    v = min(v, dpp_or_identity<0x118, 0xf, 0xffffffffu>(v));
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 15);
}
__device__ __forceinline__ uint32_t row0_max_u32(uint32_t v) {
    v = max(v, dpp_or_identity<0x111, 0xf, 0u>(v));
    v = max(v, dpp_or_identity<0x112, 0xf, 0u>(v));
    v = max(v, dpp_or_identity<0x114, 0xf, 0u>(v));
    v = max(v, dpp_or_identity<0x118, 0xf, 0u>(v));
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 15);
}

// ---- sums, maxima and minima across the four 16-lane rows ------------------------
// v_permlane32_swap a, b exchanges a[32..63] with b[0..31]; v_permlane16_swap
// exchanges rows 1 and 3 of a with rows 0 and 2 of b.  (Written as assembly: the
// compiler builtins of this toolchain lose the second result.  The s_nop pairs
// cover the wait states these instructions need after / before other vector ops.)
__device__ __forceinline__ void permlane32_swap(float& a, float& b) {
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ void permlane16_swap(float& a, float& b) {
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
// For each lane position j = lane % 16, the sums of a, b, c, d over lanes j, j+16,
// j+32, j+48: row 0 returns a's sum, row 1 c's, row 2 b's, row 3 d's.
__device__ __forceinline__ float rows_sum4(float a, float b, float c, float d) {
    permlane32_swap(a, b);
    float u = a + b;      // rows 0,1: a summed over lanes 32 apart; rows 2,3: b
    permlane32_swap(c, d);
    float w = c + d;
    permlane16_swap(u, w);
    return u + w;
}
// The maximum (minimum) of v over lanes j, j+16, j+32, j+48, in all four (two swaps on
// the vector ALU instead of two round trips through the LDS crossbar).
template <bool kMax> __device__ __forceinline__ float rows_extreme4(float v) {
    float a = v, b = v;
    permlane32_swap(a, b);      // a: lower half everywhere, b: upper half everywhere
    float u = kMax ? fmaxf(a, b) : fminf(a, b), w = u;
    permlane16_swap(u, w);      // u: rows 0,0,2,2; w: rows 1,1,3,3 (rows 0 = 2 and 1 = 3 by now)
    return kMax ? fmaxf(u, w) : fminf(u, w);
}
__device__ __forceinline__ float rows_max4(float v) { return rows_extreme4<true>(v); }
// Maximum (minimum) over the 64 lanes, in every lane: butterfly inside the rows on the
// DPP path, then across the rows.
template <bool kMax> __device__ __forceinline__ float wave_extreme_f(float v) {
    v = kMax ? fmaxf(v, dpp_f<0xB1>(v)) : fminf(v, dpp_f<0xB1>(v));
    v = kMax ? fmaxf(v, dpp_f<0x4E>(v)) : fminf(v, dpp_f<0x4E>(v));
    v = kMax ? fmaxf(v, dpp_f<0x141>(v)) : fminf(v, dpp_f<0x141>(v));
    v = kMax ? fmaxf(v, dpp_f<0x140>(v)) : fminf(v, dpp_f<0x140>(v));
    return rows_extreme4<kMax>(v);
}
// Four values at once: row 0 returns the maximum (minimum) of a over lanes j, j+16, j+32,
// j+48, row 1 that of c, row 2 that of b, row 3 that of d (three swaps for four folds).
template <bool kMax> __device__ __forceinline__ float rows_extreme_quad(float a, float b, float c, float d) {
    permlane32_swap(a, b);
    float u = kMax ? fmaxf(a, b) : fminf(a, b);
    permlane32_swap(c, d);
    float w = kMax ? fmaxf(c, d) : fminf(c, d);
    permlane16_swap(u, w);
    return kMax ? fmaxf(u, w) : fminf(u, w);
}
// The same for doubles: both halves of a double travel through the same swaps.
__device__ __forceinline__ void permlane32_swap_d(double& a, double& b) {
    uint64_t ua = __builtin_bit_cast(uint64_t, a), ub = __builtin_bit_cast(uint64_t, b);
    uint32_t al = (uint32_t)ua, ah = (uint32_t)(ua >> 32), bl = (uint32_t)ub, bh = (uint32_t)(ub >> 32);
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\tv_permlane32_swap_b32 %2, %3\n\ts_nop 1"
                 : "+v"(al), "+v"(bl), "+v"(ah), "+v"(bh));
    a = __builtin_bit_cast(double, ((uint64_t)ah << 32) | al);
    b = __builtin_bit_cast(double, ((uint64_t)bh << 32) | bl);
}
__device__ __forceinline__ void permlane16_swap_d(double& a, double& b) {
    uint64_t ua = __builtin_bit_cast(uint64_t, a), ub = __builtin_bit_cast(uint64_t, b);
    uint32_t al = (uint32_t)ua, ah = (uint32_t)(ua >> 32), bl = (uint32_t)ub, bh = (uint32_t)(ub >> 32);
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\tv_permlane16_swap_b32 %2, %3\n\ts_nop 1"
                 : "+v"(al), "+v"(bl), "+v"(ah), "+v"(bh));
    a = __builtin_bit_cast(double, ((uint64_t)ah << 32) | al);
    b = __builtin_bit_cast(double, ((uint64_t)bh << 32) | bl);
}
template <bool kMax> __device__ __forceinline__ double rows_extreme4_d(double v) {
    double a = v, b = v;
    permlane32_swap_d(a, b);
    double u = kMax ? fmax(a, b) : fmin(a, b), w = u;
    permlane16_swap_d(u, w);
    return kMax ? fmax(u, w) : fmin(u, w);
}
// Sum of a 64-bit value over aligned groups of 2^log2_group lanes (wave-uniform
// log2_group, 0..6); every lane of a group gets the total.  Butterfly steps inside a
// row on the DPP path, the steps across rows by lane swaps: nothing goes through LDS.
template <int kCtrl> __device__ __forceinline__ uint64_t dpp_u64(uint64_t v) {
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)v, kCtrl, 0xf, 0xf, true);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)(v >> 32), kCtrl, 0xf, 0xf, true);
    return ((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo;
}
__device__ __forceinline__ uint64_t group_sum_u64(uint64_t v, int log2_group) {
    if (log2_group > 0) v += dpp_u64<0xB1>(v);
    if (log2_group > 1) v += dpp_u64<0x4E>(v);
    if (log2_group > 2) v += dpp_u64<0x141>(v);
    if (log2_group > 3) v += dpp_u64<0x140>(v);
    if (log2_group > 4) {
        // rows 0+1 and 2+3: after the swap a holds rows (0,0,2,2) of v, b rows (1,1,3,3)
        uint32_t al = (uint32_t)v, ah = (uint32_t)(v >> 32), bl = al, bh = ah;
        asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\tv_permlane16_swap_b32 %2, %3\n\ts_nop 1"
                     : "+v"(al), "+v"(bl), "+v"(ah), "+v"(bh));
        v = (((uint64_t)ah << 32) | al) + (((uint64_t)bh << 32) | bl);
    }
    if (log2_group > 5) {
        uint32_t al = (uint32_t)v, ah = (uint32_t)(v >> 32), bl = al, bh = ah;
        asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\tv_permlane32_swap_b32 %2, %3\n\ts_nop 1"
                     : "+v"(al), "+v"(bl), "+v"(ah), "+v"(bh));
        v = (((uint64_t)ah << 32) | al) + (((uint64_t)bh << 32) | bl);
    }
    return v;
}

}  // namespace leoam
