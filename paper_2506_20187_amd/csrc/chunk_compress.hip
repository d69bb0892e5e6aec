// kv_chunk_compress: builds the compressed KV store from the 16-bit cache
// (paper Sec. 4.4 "Dynamic KV compression": the share of the data that is sent
// compressed trades transfer time against decompression on the GPU; Sec. 6.1:
// KV is held in FP16 and compressed to INT4).
//
// Per (b, h, chunk, tensor):  zero = min over the chunk's elements,
// scale = (max - min) / levels, code = round-half-even((x - zero) / scale) kept
// inside 0..levels, levels = 255 (8-bit chunk) or 15 (4-bit chunk, two codes per
// byte, even channel in the low nibble).  Every operation that decides a code is
// one correctly rounded float operation, in that order, so that the codes are
// reproducible bit for bit.  scale == 0 (all elements equal) stores code 0.
//
// Two launches.  The layout kernel (one workgroup per sequence and kv head) turns chunk
// sizes and 4-bit tags into byte offsets: the chunks of a (b,h) follow each
// other, then the next (b,h); rows are 128 or 64 bytes, so every chunk starts on
// a multiple of 16 bytes without padding.  The compression kernel gives one
// workgroup (two waves) to a (b, h, chunk, tensor): 16 lanes share a token row (16 bytes per
// lane, 8 channels), the workgroup reduces min / max, then encodes and stores
// 8 (4) bytes per lane, rows contiguous.  The first 32 tokens of a chunk stay in
// registers between the two steps (loads are unconditional: a step past the
// chunk's end re-reads its last row; loading under a condition measured 20 % slower); the rest is read a second time (from L2).
// 128 lanes per workgroup measured best: twice as many workgroups are in
// different phases (load, reduce, encode, store) on a compute unit.
// Streaming work: bound by HBM.
#include "leoam_dev.h"

namespace leoam {

struct QRecord {            // device image of leoam_qchunk
    long long byte_off;
    int bits;
    float scale_k, zero_k, scale_v, zero_v;
    int reserved;
};
static_assert(sizeof(QRecord) == sizeof(leoam_qchunk), "record layout");

constexpr int kLayThreads = 1024;
constexpr int kLayWaves = kLayThreads / LEOAM_WAVE;

// sum of v over the workgroup (every thread gets it); `slots` holds kLayWaves values
__device__ __forceinline__ unsigned long long layout_block_sum(unsigned long long v, unsigned long long* slots) {
    v = group_sum_u64(v, 6);
    __syncthreads();
    if (lane_id() == 0) slots[threadIdx.x / LEOAM_WAVE] = v;
    __syncthreads();
    unsigned long long t = 0;
#pragma unroll
    for (int w = 0; w < kLayWaves; ++w) t += slots[w];
    return t;
}

// bytes of chunk c of a sequence in one blob, for one kv head.  A chunk whose boundaries do
// not lie in the context in ascending order stores nothing (the compression kernel skips it
// by the same test).
__device__ __forceinline__ int chunk_bytes(int t0, int t1, int four, int n_ctx) {
    const int rows = t1 - t0;
    if (t0 < 0 || rows <= 0 || rows > n_ctx - t0) return 0;
    return rows * (four ? LEOAM_D / 2 : LEOAM_D);
}
// Sum of chunk_bytes over chunks first, first + step, ... below n.  The loads are
// unconditional (indices past the end are clamped, their results dropped) and kLayUnroll
// chunks are fetched per round trip.
constexpr int kLayUnroll = 8;
__device__ __forceinline__ unsigned long long chunk_bytes_sum(const int32_t* off, const uint8_t* four, int first, int step,
                                                              int n, int c_max, int n_ctx) {
    unsigned long long part = 0;
    for (int c = first; c < n; c += step * kLayUnroll) {
        int t0[kLayUnroll], t1[kLayUnroll], f[kLayUnroll];
#pragma unroll
        for (int u = 0; u < kLayUnroll; ++u) {
            const int cc = min(c + u * step, c_max - 1);
            t0[u] = off[cc];
            t1[u] = off[cc + 1];
            f[u] = four[cc];
        }
#pragma unroll
        for (int u = 0; u < kLayUnroll; ++u)
            if (c + u * step < n) part += (unsigned long long)chunk_bytes(t0[u], t1[u], f[u], n_ctx);
    }
    return part;
}

__global__ __launch_bounds__(kLayThreads) void compress_layout_kernel(
    const int32_t* __restrict__ chunk_off, const int32_t* __restrict__ n_chunks, const uint8_t* __restrict__ four_bit,
    QRecord* __restrict__ qmeta, long long* __restrict__ total_bytes, int c_max, int n_kv_heads, int batch, int n_ctx) {
    __shared__ unsigned long long slots[kLayWaves];
    __shared__ unsigned long long wave_incl[kLayWaves];
    // one workgroup per (kv head, sequence): each repeats the sequence's sums and writes its head's records
    const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = lane_id(), wave = tid / LEOAM_WAVE;

    // bytes of all the sequences before this one: a wave per sequence, kLayWaves of them at a time
    unsigned long long before = 0;
    for (int b0 = 0; b0 < b; b0 += kLayWaves) {
        const int bb = b0 + wave;
        unsigned long long part = 0;
        if (bb < b) {
            const int32_t* off = chunk_off + (size_t)bb * (c_max + 1);
            const uint8_t* four = four_bit + (size_t)bb * c_max;
            const int n = min(max(n_chunks[bb], 0), c_max);
            part = chunk_bytes_sum(off, four, lane, LEOAM_WAVE, n, c_max, n_ctx);
        }
        part = group_sum_u64(part, 6);
        __syncthreads();      // the previous round's totals have been read
        if (lane == 0) slots[wave] = part;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < kLayWaves; ++w) before += slots[w];
    }
    before *= (unsigned long long)n_kv_heads;

    const int32_t* off = chunk_off + (size_t)b * (c_max + 1);
    const uint8_t* four = four_bit + (size_t)b * c_max;
    const int n = min(max(n_chunks[b], 0), c_max);
    // bytes of one head of this sequence
    const unsigned long long per_head = layout_block_sum(chunk_bytes_sum(off, four, tid, kLayThreads, n, c_max, n_ctx), slots);

    // exclusive scan over the chunks, a tile of 1024 at a time
    unsigned long long carry = 0;
    for (int base = 0; base < c_max; base += kLayThreads) {
        const int c = base + tid;
        // (chunks that tile a context sum to less than 2^31 bytes per head, so a wave's scan stays in 32 bits)
        const int cc = min(c, c_max - 1);
        const int t0 = off[cc], t1 = off[cc + 1], f4 = four[cc];
        const unsigned long long mine = c < n ? (unsigned long long)chunk_bytes(t0, t1, f4, n_ctx) : 0ull;
        const unsigned long long incl = wave_incl_scan_u32((uint32_t)mine);
        __syncthreads();
        if (lane == LEOAM_WAVE - 1) wave_incl[wave] = incl;
        __syncthreads();
        unsigned long long wave_before = 0, tile = 0;
#pragma unroll
        for (int w = 0; w < kLayWaves; ++w) {
            if (w < wave) wave_before += wave_incl[w];
            tile += wave_incl[w];
        }
        const unsigned long long within = carry + wave_before + incl - mine;
        carry += tile;
        if (c < c_max) {
            QRecord r;
            if (c < n) {
                r.byte_off = (long long)(before + (unsigned long long)h * per_head + within);
                r.bits = f4 ? 4 : 8;
            } else {
                r.byte_off = 0;
                r.bits = 0;
            }
            r.scale_k = r.zero_k = r.scale_v = r.zero_v = 0.f;
            r.reserved = 0;
            qmeta[((size_t)b * n_kv_heads + h) * c_max + c] = r;
        }
    }
    if (b == batch - 1 && h == 0 && tid == 0 && total_bytes) *total_bytes = (long long)(before + per_head * n_kv_heads);
}

// ---- compression ---------------------------------------------------------------
constexpr int kCmpThreads = 128;
constexpr int kCmpWaves = kCmpThreads / LEOAM_WAVE;
constexpr int kCmpGroups = kCmpThreads / 16;       // token rows per step
constexpr int kCmpHeld = 4;                        // rows per lane group kept in registers
constexpr int kCmpHeldRows = kCmpGroups * kCmpHeld;

// The 8 codes of a lane's channels, as integer-valued floats: round-half-even of the
// correctly rounded quotient (x - zero) / scale.  The quotient is first approximated by a
// multiplication with inv = 1 / scale (0 for scale == 0, which gives code 0): both that
// product and the rounded quotient lie within 255.5 * 2^-23 < 2^-15 of the true quotient,
// so whenever the product is at least 2^-13 away from every half-integer the two round to
// the same integer.  A wave in which some lane is closer (ties among them) redoes its row
// with the division; the branch is taken by the whole wave so that it stays a branch.
// No clamp is needed: 0 <= x - zero <= max - min, so the quotient stays below levels + 1/2.
__device__ __forceinline__ void encode8(const float* x, float zero, float scale, float inv, float* r) {
    float diff[8], dev = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        diff[e] = __fsub_rn(x[e], zero);
        const float q = __fmul_rn(diff[e], inv);
        r[e] = rintf(q);
        dev = fmaxf(dev, fabsf(q - r[e]));
    }
    if (__builtin_amdgcn_ballot_w64(!(dev < 0.5f - 0x1p-13f)) != 0) {        // also taken for inf / nan products
#pragma unroll
        for (int e = 0; e < 8; ++e) r[e] = scale > 0.f ? rintf(__fdiv_rn(diff[e], scale)) : 0.f;
    }
}

template <typename T>
__device__ __forceinline__ void encode_row(const uint4& raw, float zero, float scale, float inv, bool four,
                                           unsigned char* dst_row, int c16) {
    float x[8], r[8];
    unpack<T>(raw, x);
    encode8(x, zero, scale, inv, r);
    if (four) {
        // four nibbles make an integer below 65536: exact in float
        const float h0 = fmaf(r[3], 4096.f, fmaf(r[2], 256.f, fmaf(r[1], 16.f, r[0])));
        const float h1 = fmaf(r[7], 4096.f, fmaf(r[6], 256.f, fmaf(r[5], 16.f, r[4])));
        *reinterpret_cast<uint32_t*>(dst_row + 4 * c16) = (uint32_t)h0 | ((uint32_t)h1 << 16);
    } else {
        uint2 w = make_uint2(0u, 0u);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            w.x = __builtin_amdgcn_cvt_pk_u8_f32(r[e], e, w.x);
            w.y = __builtin_amdgcn_cvt_pk_u8_f32(r[4 + e], e, w.y);
        }
        *reinterpret_cast<uint2*>(dst_row + 8 * c16) = w;
    }
}

template <typename T>
__global__ __launch_bounds__(kCmpThreads) void compress_kernel(
    const char* __restrict__ K, const char* __restrict__ V, const int32_t* __restrict__ chunk_off,
    const int32_t* __restrict__ n_chunks, QRecord* __restrict__ qmeta, unsigned char* __restrict__ kblob,
    unsigned char* __restrict__ vblob, long long blob_bytes, int c_max, int n_kv_heads, int n_ctx,
    const uint8_t* __restrict__ tag_old, const uint8_t* __restrict__ tag_new, const long long* __restrict__ info,
    long long* __restrict__ used_bytes) {
    static_assert(T::kEpl == 8, "16-bit sources only");
    constexpr int ROWB = Row<T>::kRowBytes;
    __shared__ float red[2][kCmpWaves];

    const int c = blockIdx.x, h = blockIdx.y >> 1, is_v = blockIdx.y & 1, b = blockIdx.z;
    if (tag_old) {
        // re-tagging a live store: only chunks whose tag changed are encoded again, and none if the
        // layout step found no room; the first workgroup also advances the used size by the fresh room taken
        if (info[0] != 0) return;
        if (c == 0 && blockIdx.y == 0 && b == 0 && threadIdx.x == 0) *used_bytes += info[2];
        if ((tag_old[(size_t)b * c_max + c] != 0) == (tag_new[(size_t)b * c_max + c] != 0)) return;
    }
    if (c >= min(max(n_chunks[b], 0), c_max)) return;
    const size_t bh = (size_t)b * n_kv_heads + h;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid / LEOAM_WAVE;
    const int grp = tid / 16, c16 = tid % 16;
    const int32_t* off = chunk_off + (size_t)b * (c_max + 1);
    const int t0 = off[c], rows = off[c + 1] - t0;
    if (t0 < 0 || rows <= 0 || t0 + rows > n_ctx) return;        // boundaries that do not tile the context
    QRecord* rec = qmeta + bh * c_max + c;
    const long long byte_off = rec->byte_off;
    const bool four = rec->bits == 4;
    // (boundaries that overlap can add up to more than the blobs hold: such a chunk is not written)
    if (byte_off < 0 || byte_off + (long long)rows * (four ? LEOAM_D / 2 : LEOAM_D) > blob_bytes) return;
    const char* src = (is_v ? V : K) + (bh * (size_t)n_ctx + t0) * ROWB + (size_t)c16 * 16;

    // ---- min / max of the chunk (a row past the end re-reads the last row) ------------
    uint4 held[kCmpHeld];
    float lo = INFINITY, hi = -INFINITY;
    auto fold2 = [&](const uint4& a, const uint4& a2) {       // two rows at a time: three-operand min / max
        float x[8], y[8];
        unpack<T>(a, x);
        unpack<T>(a2, y);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            lo = fminf(fminf(lo, x[e]), y[e]);
            hi = fmaxf(fmaxf(hi, x[e]), y[e]);
        }
    };
    static_assert(kCmpHeld % 2 == 0, "rows are folded in pairs");
#pragma unroll
    for (int j = 0; j < kCmpHeld; ++j) held[j] = load16(src, (size_t)min(grp + j * kCmpGroups, rows - 1) * ROWB);
#pragma unroll
    for (int j = 0; j < kCmpHeld; j += 2) fold2(held[j], held[j + 1]);
    for (int r0 = kCmpHeldRows; r0 < rows; r0 += kCmpHeldRows) {
        uint4 a[kCmpHeld];
#pragma unroll
        for (int j = 0; j < kCmpHeld; ++j) a[j] = load16(src, (size_t)min(r0 + grp + j * kCmpGroups, rows - 1) * ROWB);
#pragma unroll
        for (int j = 0; j < kCmpHeld; j += 2) fold2(a[j], a[j + 1]);
    }
    lo = wave_extreme_f<false>(lo);
    hi = wave_extreme_f<true>(hi);
    if (lane == 0) {
        red[0][wave] = lo;
        red[1][wave] = hi;
    }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kCmpWaves; ++w) {
        lo = fminf(lo, red[0][w]);
        hi = fmaxf(hi, red[1][w]);
    }
    const float levels = four ? 15.f : 255.f;
    const float scale = __fdiv_rn(__fsub_rn(hi, lo), levels);
    const float inv = scale > 0.f ? __fdiv_rn(1.0f, scale) : 0.f;
    if (tid == 0) {
        if (is_v) {
            rec->scale_v = scale;
            rec->zero_v = lo;
        } else {
            rec->scale_k = scale;
            rec->zero_k = lo;
        }
    }

    // ---- codes ---------------------------------------------------------------------------
    const int row_bytes = four ? LEOAM_D / 2 : LEOAM_D;
    unsigned char* dst = (is_v ? vblob : kblob) + byte_off;
#pragma unroll
    for (int j = 0; j < kCmpHeld; ++j) {
        const int r = grp + j * kCmpGroups;
        if (r < rows) encode_row<T>(held[j], lo, scale, inv, four, dst + (size_t)r * row_bytes, c16);
    }
    for (int r0 = kCmpHeldRows; r0 < rows; r0 += kCmpHeldRows) {
        uint4 a[kCmpHeld];
#pragma unroll
        for (int j = 0; j < kCmpHeld; ++j) a[j] = load16(src, (size_t)min(r0 + grp + j * kCmpGroups, rows - 1) * ROWB);
#pragma unroll
        for (int j = 0; j < kCmpHeld; ++j) {
            const int r = r0 + grp + j * kCmpGroups;
            if (r < rows) encode_row<T>(a[j], lo, scale, inv, four, dst + (size_t)r * row_bytes, c16);
        }
    }
}

// ---- re-tagging a live store ----------------------------------------------------------------
// Sec. 4.4: the compressed share follows the measured times and the scores, so the tags of a store
// change while it is in use.  Only chunks whose tag changed are encoded again: a chunk that becomes
// 4-bit stays where it lies (it takes half of its old room), a chunk that becomes 8-bit moves to fresh
// room behind the used part of the blobs, the moved chunks placed in (b, h, chunk) order.  This kernel
// (one workgroup per kv head and sequence) assigns that room and rewrites the records' format fields;
// the compression kernel then runs over the changed chunks only.  info[0] = 1 and nothing is changed
// if the fresh room does not fit the blobs; info[1] = chunks to encode again, info[2] = bytes of fresh
// room per blob.
__device__ __forceinline__ unsigned long long grown_bytes_sum(const int32_t* off, const uint8_t* was, const uint8_t* is,
                                                              int first, int step, int n, int c_max, int n_ctx,
                                                              unsigned long long* changed) {
    unsigned long long part = 0, cnt = 0;
    for (int c = first; c < n; c += step * kLayUnroll) {
        int t0[kLayUnroll], t1[kLayUnroll], fo[kLayUnroll], fn[kLayUnroll];
#pragma unroll
        for (int u = 0; u < kLayUnroll; ++u) {
            const int cc = min(c + u * step, c_max - 1);
            t0[u] = off[cc];
            t1[u] = off[cc + 1];
            fo[u] = was[cc];
            fn[u] = is[cc];
        }
#pragma unroll
        for (int u = 0; u < kLayUnroll; ++u) {
            if (c + u * step >= n || (fo[u] != 0) == (fn[u] != 0)) continue;
            const unsigned long long bytes = (unsigned long long)chunk_bytes(t0[u], t1[u], 0, n_ctx);
            if (bytes == 0) continue;              // boundaries that do not tile the context: such a chunk stores nothing
            ++cnt;
            if (fo[u] != 0) part += bytes;         // 4-bit -> 8-bit: fresh room of the 8-bit size
        }
    }
    *changed += cnt;
    return part;
}

__global__ __launch_bounds__(kLayThreads) void recompress_layout_kernel(
    const int32_t* __restrict__ chunk_off, const int32_t* __restrict__ n_chunks, const uint8_t* __restrict__ tag_old,
    const uint8_t* __restrict__ tag_new, QRecord* __restrict__ qmeta, const long long* __restrict__ used_bytes,
    long long blob_bytes, long long* __restrict__ info, int c_max, int n_kv_heads, int batch, int n_ctx) {
    __shared__ unsigned long long slots[kLayWaves], slots_cnt[kLayWaves];
    __shared__ unsigned long long wave_incl[kLayWaves];
    const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = lane_id(), wave = tid / LEOAM_WAVE;

    // fresh room of every sequence (a wave per sequence): those before this one, and all of them
    unsigned long long before = 0, all = 0, all_changed = 0;
    for (int b0 = 0; b0 < batch; b0 += kLayWaves) {
        const int bb = b0 + wave;
        unsigned long long part = 0, cnt = 0;
        if (bb < batch) {
            const int n = min(max(n_chunks[bb], 0), c_max);
            part = grown_bytes_sum(chunk_off + (size_t)bb * (c_max + 1), tag_old + (size_t)bb * c_max,
                                   tag_new + (size_t)bb * c_max, lane, LEOAM_WAVE, n, c_max, n_ctx, &cnt);
        }
        part = group_sum_u64(part, 6);
        cnt = group_sum_u64(cnt, 6);
        __syncthreads();      // the previous round's totals have been read
        if (lane == 0) {
            slots[wave] = part;
            slots_cnt[wave] = cnt;
        }
        __syncthreads();
#pragma unroll
        for (int w = 0; w < kLayWaves; ++w) {
            if (b0 + w < b) before += slots[w];
            all += slots[w];
            all_changed += slots_cnt[w];
        }
    }
    const unsigned long long heads = (unsigned long long)n_kv_heads;
    const long long used = *used_bytes;
    const bool fits = used >= 0 && (unsigned long long)used + all * heads <= (unsigned long long)blob_bytes;
    if (b == 0 && h == 0 && tid == 0) {
        info[0] = fits ? 0 : 1;
        info[1] = fits ? (long long)(all_changed * heads) : 0;
        info[2] = fits ? (long long)(all * heads) : 0;
    }
    if (!fits) return;

    const int32_t* off = chunk_off + (size_t)b * (c_max + 1);
    const uint8_t* was = tag_old + (size_t)b * c_max;
    const uint8_t* is = tag_new + (size_t)b * c_max;
    const int n = min(max(n_chunks[b], 0), c_max);
    unsigned long long dummy = 0;
    const unsigned long long per_head =
        layout_block_sum(grown_bytes_sum(off, was, is, tid, kLayThreads, n, c_max, n_ctx, &dummy), slots);

    // exclusive scan of the fresh room over the chunks, a tile of 1024 at a time
    unsigned long long carry = 0;
    for (int base = 0; base < n; base += kLayThreads) {
        const int c = base + tid;
        const int cc = min(c, c_max - 1);
        const int t0 = off[cc], t1 = off[cc + 1], fo = was[cc], fn = is[cc];
        const bool changes = c < n && (fo != 0) != (fn != 0) && chunk_bytes(t0, t1, 0, n_ctx) != 0;
        const unsigned long long mine = (changes && fo != 0) ? (unsigned long long)chunk_bytes(t0, t1, 0, n_ctx) : 0ull;
        const unsigned long long incl = wave_incl_scan_u32((uint32_t)mine);
        __syncthreads();
        if (lane == LEOAM_WAVE - 1) wave_incl[wave] = incl;
        __syncthreads();
        unsigned long long wave_before = 0, tile = 0;
#pragma unroll
        for (int w = 0; w < kLayWaves; ++w) {
            if (w < wave) wave_before += wave_incl[w];
            tile += wave_incl[w];
        }
        const unsigned long long within = carry + wave_before + incl - mine;
        carry += tile;
        if (changes) {
            QRecord* r = qmeta + ((size_t)b * n_kv_heads + h) * c_max + c;
            if (fo != 0) {
                r->byte_off = used + (long long)(before * heads + (unsigned long long)h * per_head + within);
                r->bits = 8;
            } else {
                r->bits = 4;
            }
        }
    }
}

// ---- which chunks form the compressed share --------------------------------------------
// Sec. 4.4 fixes how large the compressed share is, not which data it holds.  Here a chunk is
// stored 4-bit unless some kv head of its sequence keeps it in the given selection (Sec. 4.2
// order): one workgroup per sequence marks the kept chunks in an LDS byte map and writes the
// row out.
constexpr int kTagThreads = 1024;
constexpr int kTagMax = 16384;      // c_max limit of the library

__global__ __launch_bounds__(kTagThreads) void compression_tags_kernel(
    const int32_t* __restrict__ n_chunks, const int32_t* __restrict__ sel_idx, const int32_t* __restrict__ sel_count,
    uint8_t* __restrict__ four_bit, int c_max, int k_max, int n_kv_heads) {
    __shared__ uint8_t tag[kTagMax];
    const int b = blockIdx.x, tid = threadIdx.x;
    const int n = min(max(n_chunks[b], 0), c_max);
    for (int c = tid; c < c_max; c += kTagThreads) tag[c] = c < n ? 1 : 0;
    __syncthreads();
    for (int h = 0; h < n_kv_heads; ++h) {
        const size_t bh = (size_t)b * n_kv_heads + h;
        const int cnt = min(max(sel_count[bh], 0), k_max);
        for (int i = tid; i < cnt; i += kTagThreads) {
            const int id = sel_idx[bh * k_max + i];
            if (id >= 0 && id < n) tag[id] = 0;         // several lanes may clear the same byte
        }
    }
    __syncthreads();
    for (int c = tid; c < c_max; c += kTagThreads) four_bit[(size_t)b * c_max + c] = tag[c];
}

hipError_t compression_tags_dispatch(const leoam_shape* s, const int32_t* n_chunks, const int32_t* sel_idx,
                                     const int32_t* sel_count, uint8_t* four_bit, hipStream_t stream) {
    hipLaunchKernelGGL(compression_tags_kernel, dim3(s->batch), dim3(kTagThreads), 0, stream, n_chunks, sel_idx,
                       sel_count, four_bit, s->c_max, s->k_max, s->n_kv_heads);
    return hipGetLastError();
}

size_t compressed_bytes_bound(const leoam_shape* s) {
    return (size_t)s->batch * s->n_kv_heads * (size_t)s->n_ctx * LEOAM_D;        // every chunk 8-bit
}

hipError_t compress_dispatch(const leoam_shape* s, const void* K, const void* V, const int32_t* chunk_off,
                             const int32_t* n_chunks, const uint8_t* four_bit, void* kblob, void* vblob, void* qmeta,
                             size_t blob_bytes, long long* total_bytes, hipStream_t stream) {
    hipLaunchKernelGGL(compress_layout_kernel, dim3(s->n_kv_heads, s->batch), dim3(kLayThreads), 0, stream, chunk_off, n_chunks,
                       four_bit, (QRecord*)qmeta, total_bytes, s->c_max, s->n_kv_heads, s->batch, s->n_ctx);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    dim3 grid(s->c_max, s->n_kv_heads * 2, s->batch), block(kCmpThreads);      // y: (kv head, K or V)
    if (s->kv_dtype == LEOAM_F16)
        hipLaunchKernelGGL(compress_kernel<F16>, grid, block, 0, stream, (const char*)K, (const char*)V, chunk_off,
                           n_chunks, (QRecord*)qmeta, (unsigned char*)kblob, (unsigned char*)vblob,
                           (long long)blob_bytes, s->c_max, s->n_kv_heads, s->n_ctx, nullptr, nullptr, nullptr, nullptr);
    else
        hipLaunchKernelGGL(compress_kernel<BF16>, grid, block, 0, stream, (const char*)K, (const char*)V, chunk_off,
                           n_chunks, (QRecord*)qmeta, (unsigned char*)kblob, (unsigned char*)vblob,
                           (long long)blob_bytes, s->c_max, s->n_kv_heads, s->n_ctx, nullptr, nullptr, nullptr, nullptr);
    return hipGetLastError();
}

hipError_t recompress_dispatch(const leoam_shape* s, const void* K, const void* V, const int32_t* chunk_off,
                               const int32_t* n_chunks, const uint8_t* tag_old, const uint8_t* tag_new, void* kblob,
                               void* vblob, void* qmeta, size_t blob_bytes, long long* used_bytes, long long* info,
                               hipStream_t stream) {
    hipLaunchKernelGGL(recompress_layout_kernel, dim3(s->n_kv_heads, s->batch), dim3(kLayThreads), 0, stream, chunk_off,
                       n_chunks, tag_old, tag_new, (QRecord*)qmeta, used_bytes, (long long)blob_bytes, info, s->c_max,
                       s->n_kv_heads, s->batch, s->n_ctx);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    dim3 grid(s->c_max, s->n_kv_heads * 2, s->batch), block(kCmpThreads);
    if (s->kv_dtype == LEOAM_F16)
        hipLaunchKernelGGL(compress_kernel<F16>, grid, block, 0, stream, (const char*)K, (const char*)V, chunk_off,
                           n_chunks, (QRecord*)qmeta, (unsigned char*)kblob, (unsigned char*)vblob,
                           (long long)blob_bytes, s->c_max, s->n_kv_heads, s->n_ctx, tag_old, tag_new, info, used_bytes);
    else
        hipLaunchKernelGGL(compress_kernel<BF16>, grid, block, 0, stream, (const char*)K, (const char*)V, chunk_off,
                           n_chunks, (QRecord*)qmeta, (unsigned char*)kblob, (unsigned char*)vblob,
                           (long long)blob_bytes, s->c_max, s->n_kv_heads, s->n_ctx, tag_old, tag_new, info, used_bytes);
    return hipGetLastError();
}

}  // namespace leoam
