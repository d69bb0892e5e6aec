// Pieces shared by the kernels that read the compressed KV store (8-bit / 4-bit chunks;
// paper Sec. 4.4, Sec. 6.1): the chunk record, and the exact code -> f16 expansion that
// feeds the matrix cores (see quant_store.hip).
#pragma once
#include "attention_common.h"

namespace leoam {

struct QChunk {             // device image of leoam_qchunk
    long long byte_off;
    int bits;
    float scale_k, zero_k, scale_v, zero_v;
    int reserved;
};
static_assert(sizeof(QChunk) == sizeof(leoam_qchunk), "record layout");

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

// two codes (0..255) in the 16-bit halves of p -> the same two values as f16
__device__ __forceinline__ uint32_t codes_to_f16x2(uint32_t p) {
    const half2_t h = __builtin_bit_cast(half2_t, p | 0x64006400u) - half2_t{(_Float16)1024.f, (_Float16)1024.f};
    return __builtin_bit_cast(uint32_t, h);
}

// one 16-token tile of a wave as loaded: the K dwords of token 16t + c16 (four steps), the V
// dwords of tokens 16t + 4grp + i, their kept-list slots (complemented: no token) and formats
struct QmTile {
    uint32_t k0[4], k1[4], v0[4], v1[4];
    int vslot[4];
    bool kfour, vfour[4];
};

// The group's queries (fp16) as the matrix core's B operand for step s, in the channel order
// (0,2,4,6,1,3,5,7) the code operand has; raw = channels 32s + 8grp + 0..7 of one head.
__device__ __forceinline__ uint4 query_operand(const uint4& raw) {
    uint4 qb;
    qb.x = __builtin_amdgcn_perm(raw.y, raw.x, 0x05040100u);       // (0, 2)
    qb.y = __builtin_amdgcn_perm(raw.w, raw.z, 0x05040100u);       // (4, 6)
    qb.z = __builtin_amdgcn_perm(raw.y, raw.x, 0x07060302u);       // (1, 3)
    qb.w = __builtin_amdgcn_perm(raw.w, raw.z, 0x07060302u);       // (5, 7)
    return qb;
}

// q . code for the 16 tokens of a tile (token c16's codes in k0 / k1) against the B operands
// read by `qop(s)`: the f16 A operand is built from the dwords as described in quant_store.hip.
template <typename QOp>
__device__ __forceinline__ f32x4_t code_logits(const QmTile& kv, QOp&& qop) {
    const uint32_t kmask = kv.kfour ? 0x0f0f0f0fu : 0xffffffffu, kshift = kv.kfour ? 4u : 0u;
    const uint32_t s0 = kv.kfour ? 0x0c010c00u : 0x0c020c00u, s1 = kv.kfour ? 0x0c030c02u : 0x0c060c04u;
    const uint32_t s2 = kv.kfour ? 0x0c050c04u : 0x0c030c01u, s3 = kv.kfour ? 0x0c070c06u : 0x0c070c05u;
    f32x4_t sacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const uint32_t lo4 = kv.k0[s] & kmask, hi4 = (kv.k1[s] >> kshift) & kmask;
        uint4 a;
        a.x = codes_to_f16x2(__builtin_amdgcn_perm(hi4, lo4, s0));
        a.y = codes_to_f16x2(__builtin_amdgcn_perm(hi4, lo4, s1));
        a.z = codes_to_f16x2(__builtin_amdgcn_perm(hi4, lo4, s2));
        a.w = codes_to_f16x2(__builtin_amdgcn_perm(hi4, lo4, s3));
        sacc = mfma_16x16x32<F16>(a, qop(s), sacc);
    }
    return sacc;
}

// the 8 V codes of a lane (dwords v0 / v1 of a row) as floats, channel order (0,2,4,6,1,3,5,7)
__device__ __forceinline__ void value_codes(uint32_t v0, uint32_t v1, bool four, float* x) {
    const uint32_t vmask = four ? 0x0f0f0f0fu : 0xffffffffu, vshift = four ? 4u : 0u;
    const uint32_t lo4 = v0 & vmask, hi4 = (v1 >> vshift) & vmask;
    // 8-bit rows: (0,1,2,3),(4,5,6,7) -> (0,2,4,6),(1,3,5,7), the order a 4-bit row already has
    const uint32_t te = __builtin_amdgcn_perm(hi4, lo4, four ? 0x03020100u : 0x06040200u);
    const uint32_t to = __builtin_amdgcn_perm(hi4, lo4, four ? 0x07060504u : 0x07050301u);
#pragma unroll
    for (int e = 0; e < 4; ++e) {      // (v_cvt_f32_ubyte0..3)
        x[e] = (float)((te >> (8 * e)) & 0xffu);
        x[4 + e] = (float)((to >> (8 * e)) & 0xffu);
    }
}

// channel of accumulator e inside a lane's 8 channels
__device__ __forceinline__ constexpr int code_channel(int e) { return e < 4 ? 2 * e : 2 * (e - 4) + 1; }

}  // namespace leoam
