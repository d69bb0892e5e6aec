// Selection core shared by chunk_topk_select and the fused select + attention
// kernel: which of a (sequence, kv head)'s chunks are kept (paper Sec. 4.2:
// priority queue by upper bound, read from the front; Sec. 6.1: only the most
// important share of the cache is loaded).
//
// The ordered list is never materialised.  Because the kept set is a prefix of
// the order (score descending, index ascending), it is described by one
// threshold key T: every chunk with key > T is kept, chunks with key == T are
// kept in index order while they fit, everything below is dropped.  T is found
// by a radix descent over the 32-bit order-preserving image of the float score:
// a pass histograms (count, tokens) of the chunks still in range into 256 equal
// sub-ranges of the live key range (LDS, one packed 64-bit atomic per chunk),
// one wave walks the histogram from the top and picks the sub-range in which the
// running totals stop fitting.  As soon as that sub-range holds at most 256
// chunks (normally after the first pass) they are ranked pairwise, the n*n
// comparisons spread over the workgroup; a single key shared by more chunks than
// that falls back to a scan in index order.  All integer work, exact, no
// ordering ambiguity.
//
// One workgroup per (sequence, kv head), 1024 lanes in the library's kernels (the
// code is written for any multiple of 256 up to that); every lane keeps kIpt
// consecutive chunks in registers, so "ascending chunk index" is "lane order".
#pragma once
#include "leoam_dev.h"

namespace leoam {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / LEOAM_WAVE;
static_assert(kSelWaves == 16, "the second scan level keeps one wave total per lane of a 16-lane row");
constexpr int kBins = 256;
// Chunks of the cut sub-range that are ranked pairwise.  A pass of the descent costs about a
// microsecond whatever it narrows; the pairwise step costs n / (lanes per chunk) dependent LDS
// reads per lane, so it only pays for a few hundred chunks.  Scores that straddle zero put
// hundreds of chunks into one sub-range of the first pass (sub-ranges are equal in the bit
// pattern, i.e. two binades wide there): with a limit of 1024 the selection of 3.5K such chunks
// took 100 us on MI355X, with 256 it takes 10 (one more pass), and rows whose first pass
// already isolates a few dozen chunks are not affected.
constexpr int kMaxCand = 256;

// float -> uint32 whose unsigned order is the float order (-0 == +0)
__device__ __forceinline__ uint32_t order_key(float s) {
    uint32_t u = float_to_bits(s + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ bool fits(uint32_t cnt, uint32_t tok, uint32_t max_cnt, uint32_t max_tok) {
    return cnt <= max_cnt && tok <= max_tok;
}

__device__ __forceinline__ uint64_t pack_tot(uint32_t cnt, uint32_t tok) { return ((uint64_t)cnt << 32) | tok; }

// inclusive scan over the wave of a packed (count << 32 | tokens) total; the two
// halves are scanned separately (token sums stay below 2^32, so nothing carries)
__device__ __forceinline__ uint64_t wave_incl_scan(uint64_t v) {
    const uint32_t lo = wave_incl_scan_u32((uint32_t)v), hi = wave_incl_scan_u32((uint32_t)(v >> 32));
    return ((uint64_t)hi << 32) | lo;
}

// sum of the kWaves (a power of two, at most 16) per-wave totals in wave_sums (every lane gets it)
template <int kWaves = kSelWaves>
__device__ __forceinline__ uint64_t wave_sums_total(const uint64_t* wave_sums) {
    const uint64_t s = wave_sums[lane_id() & (kWaves - 1)];
    const uint32_t lo = row16_incl_scan_u32((uint32_t)s), hi = row16_incl_scan_u32((uint32_t)(s >> 32));
    return ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)hi, kWaves - 1) << 32) |
           (uint32_t)__builtin_amdgcn_readlane((int)lo, kWaves - 1);
}

// exclusive scan over the whole workgroup (kWaves waves) in lane order; *total gets the sum.
// kGuard: a barrier first, for callers that cannot rule out a lane still reading wave_sums.
template <bool kGuard = true, int kWaves = kSelWaves>
__device__ __forceinline__ uint64_t block_excl_scan(uint64_t v, uint64_t* wave_sums, uint64_t* total) {
    static_assert(kWaves <= 16 && (kWaves & (kWaves - 1)) == 0, "the second scan level is one 16-lane row");
    const int lane = lane_id(), wave = threadIdx.x / LEOAM_WAVE;
    const uint64_t incl = wave_incl_scan(v);
    if (kGuard) __syncthreads();           // wave_sums may still be read from a previous call
    if (lane == LEOAM_WAVE - 1) wave_sums[wave] = incl;
    __syncthreads();
    // second level: lane w of a row holds wave w's sum, a row scan gives the prefixes
    const uint64_t s = wave_sums[lane & (kWaves - 1)];
    const uint32_t lo = row16_incl_scan_u32((uint32_t)s), hi = row16_incl_scan_u32((uint32_t)(s >> 32));
    const uint32_t all_lo = (uint32_t)__builtin_amdgcn_readlane((int)lo, kWaves - 1);
    const uint32_t all_hi = (uint32_t)__builtin_amdgcn_readlane((int)hi, kWaves - 1);
    const uint32_t upto_lo = (uint32_t)__builtin_amdgcn_readlane((int)lo, wave);
    const uint32_t upto_hi = (uint32_t)__builtin_amdgcn_readlane((int)hi, wave);
    const uint32_t own_lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)s, wave);
    const uint32_t own_hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(s >> 32), wave);
    *total = ((uint64_t)all_hi << 32) | all_lo;
    const uint64_t base = (((uint64_t)upto_hi << 32) | upto_lo) - (((uint64_t)own_hi << 32) | own_lo);
    return base + incl - v;
}

// A wave transposes its items through LDS a block of whole 64-item slices at a time; a block
// must also hold whole lanes (kIpt items each): four slices when kIpt divides 256, else five
// (kIpt = 10) or three (kIpt = 6, 12).
constexpr int stage_slices(int ipt) { return (256 % ipt == 0) ? 4 : (ipt % 5 == 0 ? 5 : 3); }
constexpr int kStageItems = 5 * LEOAM_WAVE;       // the largest block
constexpr int kStageStride = kStageItems + 4;

// LDS of one selection
struct SelectLds {
    uint64_t hist[kBins];
    uint64_t wave_sums[kSelWaves];
    uint64_t wave_sums2[kSelWaves];     // the final scan's own slots: written while wave_sums may still be read
    uint32_t red_min[kSelWaves], red_max[kSelWaves];
    uint32_t sh_lo, sh_hi, sh_done, sh_nbin, sh_ncand;
    union {
        struct {
            uint64_t cand_ki[kMaxCand], cand_tot[kMaxCand];
            uint32_t cand_keep[kMaxCand];
        };
        uint32_t stage[kSelWaves][kStageStride];      // load stage only: per-wave transposition buffer
    };
    uint64_t sh_above;
};

// What a lane learns about its kIpt consecutive chunks tid*kIpt + i.
template <int kIpt> struct SelectResult {
    bool keep[kIpt];          // chunk is in the kept front
    uint32_t size[kIpt];      // tokens of the chunk (0 for a chunk >= n_chunks)
    int first_tok;            // first token of chunk tid*kIpt
    uint64_t kept_before;     // (count << 32 | tokens) of kept chunks with a lower index
    uint64_t kept_total;      // the same over the whole (sequence, kv head)
};

template <int kIpt, int kThreads = kSelThreads>
__device__ __forceinline__ void select_keep(SelectLds& L, const float* __restrict__ srow,
                                            const int32_t* __restrict__ off, int C, int c_max, int k_max, int n_ctx,
                                            int max_chunks, int token_budget, SelectResult<kIpt>& R) {
    constexpr int kWaves = kThreads / LEOAM_WAVE;
    static_assert(kThreads >= kBins && kWaves <= kSelWaves, "the histogram is cleared by one lane per bin");
    // (no more candidates than lanes: a smaller workgroup takes another pass instead)
    constexpr int kCandLimit = kThreads < kMaxCand ? kThreads : kMaxCand;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid / LEOAM_WAVE;
    uint32_t max_cnt = (uint32_t)k_max;
    if (max_chunks > 0 && (uint32_t)max_chunks < max_cnt) max_cnt = (uint32_t)max_chunks;
    const uint32_t max_tok = token_budget > 0 ? (uint32_t)token_budget : 0xffffffffu;

    // (cleared here, published by the first barrier below)
    if (tid < kBins) L.hist[tid] = 0;
    if (tid == 0) L.sh_ncand = 0;

    // ---- load this lane's chunks -------------------------------------------
    uint32_t key[kIpt];
    bool valid[kIpt];
    const int c0 = tid * kIpt;
    uint32_t kmin = 0xffffffffu, kmaxv = 0;
    uint64_t mine = 0;
    // (loads are unconditional and clamped to the buffers, not to n_chunks: a load under a
    // condition would be waited for on its own, one memory round trip per chunk)
    int offv[kIpt + 1];
    float sc[kIpt];
    if constexpr (kIpt < 4) {
#pragma unroll
        for (int i = 0; i <= kIpt; ++i) offv[i] = off[min(c0 + i, c_max)];
#pragma unroll
        for (int i = 0; i < kIpt; ++i) sc[i] = srow[min(c0 + i, c_max - 1)];
    } else {
        // A lane's kIpt consecutive items are 4*kIpt bytes apart from its neighbour's: read
        // directly, every load instruction would touch 64 * kIpt * 4 / 128 cache lines.  The
        // wave reads its 64 * kIpt items with consecutive lanes on consecutive items instead
        // and transposes them through LDS, a block of slices at a time.
        const int wbase = wave * LEOAM_WAVE * kIpt;
        float rs[kIpt];
        int ro[kIpt];
        // (the boundary after the wave's last item goes out with the others: left to the compiler the
        // load sinks into the one-lane branch that uses it, behind the wait for the others - one more
        // round trip; the empty asm is an opaque use that keeps it here)
        int ro_end = off[min(wbase + LEOAM_WAVE * kIpt, c_max)];
#pragma unroll
        for (int j = 0; j < kIpt; ++j) {
            rs[j] = srow[min(wbase + LEOAM_WAVE * j + lane, c_max - 1)];
            ro[j] = off[min(wbase + LEOAM_WAVE * j + lane, c_max)];
        }
        asm volatile("" : "+v"(ro_end));
        constexpr int kSl = stage_slices(kIpt);                // slices per block
        constexpr int kBlkItems = kSl * LEOAM_WAVE, kBlocks = kIpt / kSl;
        static_assert(kBlkItems % kIpt == 0 && kIpt % kSl == 0 && kBlkItems <= kStageItems, "unsupported items per lane");
        constexpr int kPerBlock = kBlkItems / kIpt;            // lanes whose items a block holds
        uint32_t* st = L.stage[wave];
        const int my_block = lane / kPerBlock, base = (lane % kPerBlock) * kIpt;
        auto wave_sync = [] {
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
            __builtin_amdgcn_wave_barrier();
        };
#pragma unroll
        for (int blk = 0; blk < kBlocks; ++blk) {
#pragma unroll
            for (int jj = 0; jj < kSl; ++jj) st[LEOAM_WAVE * jj + lane] = float_to_bits(rs[kSl * blk + jj]);
            wave_sync();
            if (my_block == blk) {
#pragma unroll
                for (int i = 0; i < kIpt; ++i) sc[i] = bits_to_float(st[base + i]);
            }
            wave_sync();
        }
#pragma unroll
        for (int blk = 0; blk < kBlocks; ++blk) {
#pragma unroll
            for (int jj = 0; jj < kSl; ++jj) st[LEOAM_WAVE * jj + lane] = (uint32_t)ro[kSl * blk + jj];
            // the boundary after the block's last item: the first item of the next block, or of the next wave
            int after = ro_end;
            if constexpr (kBlocks > 1) {
                if (blk + 1 < kBlocks) after = ro[kSl * (blk + 1 < kBlocks ? blk + 1 : blk)];
            }
            if (lane == 0) st[kBlkItems] = (uint32_t)after;
            wave_sync();
            if (my_block == blk) {
#pragma unroll
                for (int i = 0; i <= kIpt; ++i) offv[i] = (int)st[base + i];
            }
            wave_sync();
        }
    }
    int prev = min(max(offv[0], 0), n_ctx);
    R.first_tok = prev;
#pragma unroll
    for (int i = 0; i < kIpt; ++i) {
        const int c = c0 + i;
        valid[i] = c < C;
        key[i] = 0;
        R.size[i] = 0;
        if (valid[i]) {
            const int nxt = min(max(offv[i + 1], prev), n_ctx);
            R.size[i] = (uint32_t)(nxt - prev);
            prev = nxt;
            key[i] = order_key(sc[i]);
            kmin = min(kmin, key[i]);
            kmaxv = max(kmaxv, key[i]);
            mine += pack_tot(1, R.size[i]);
        }
    }

    // ---- range of keys and grand total: one barrier publishes the per-wave values ----
    kmin = wave_min_u32(kmin);
    kmaxv = wave_max_u32(kmaxv);
    {
        const uint64_t incl = wave_incl_scan(mine);
        if (lane == LEOAM_WAVE - 1) L.wave_sums[wave] = incl;
    }
    if (lane == 0) {
        L.red_min[wave] = kmin;
        L.red_max[wave] = kmaxv;
    }
    __syncthreads();
    const uint64_t grand = wave_sums_total<kWaves>(L.wave_sums);
    uint32_t lo = row0_min_u32(L.red_min[lane & (kWaves - 1)]);
    uint32_t hi = row0_max_u32(L.red_max[lane & (kWaves - 1)]);

    uint64_t above = 0;
    bool use_cand = false;
    bool take_all = (C == 0) || fits((uint32_t)(grand >> 32), (uint32_t)grand, max_cnt, max_tok);

    if (!take_all) {
        // ---- radix descent: invariant lo <= T <= hi, above = totals of key > hi
        for (int pass = 0; pass < 5; ++pass) {
            const uint32_t span = hi - lo;
            const int sh = span < kBins ? 0 : (32 - __clz(span)) - 8;   // (span >> sh) < 256
            // (the histogram is all zero here: cleared at the start, and by the walk below after every pass)
#pragma unroll
            for (int i = 0; i < kIpt; ++i) {
                if (valid[i] && key[i] >= lo && key[i] <= hi)
                    atomicAdd((unsigned long long*)&L.hist[(key[i] - lo) >> sh],
                              (unsigned long long)pack_tot(1, R.size[i]));
            }
            __syncthreads();
            if (wave == 0) {
                // lane l owns bins 4l..4l+3; suffix totals from the top bin down
                uint64_t hb[4];
                uint64_t lane_sum = 0;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    hb[k] = L.hist[4 * lane + k];
                    L.hist[4 * lane + k] = 0;
                    lane_sum += hb[k];
                }
                // suffix over lanes: sum of lanes > this lane
                uint64_t incl = wave_incl_scan(lane_sum);
                const uint64_t wave_total =
                    ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(incl >> 32), LEOAM_WAVE - 1) << 32) |
                    (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)incl, LEOAM_WAVE - 1);
                uint64_t run = above + (wave_total - incl);        // totals of bins above this lane's bins
                int first_bad = -1;                                // highest bin whose inclusion breaks the fit
                uint64_t above_bad = 0, in_bad = 0;
#pragma unroll
                for (int k = 3; k >= 0; --k) {
                    const uint64_t with = run + hb[k];
                    if (first_bad < 0 && !fits((uint32_t)(with >> 32), (uint32_t)with, max_cnt, max_tok)) {
                        first_bad = 4 * lane + k;
                        above_bad = run;
                        in_bad = hb[k];
                    }
                    run = with;
                }
                const uint64_t bad_mask = __ballot(first_bad >= 0);
                // the top-most lane that saw a misfit decides (one always exists: the grand total does not fit)
                const int decider = 63 - __clzll((unsigned long long)bad_mask);
                if (lane == decider) {
                    const uint32_t nlo = lo + ((uint32_t)first_bad << sh);
                    const uint32_t width_m1 = sh ? ((1u << sh) - 1u) : 0u;
                    uint32_t nhi = (nlo > 0xffffffffu - width_m1) ? 0xffffffffu : nlo + width_m1;
                    if (nhi > hi) nhi = hi;
                    L.sh_lo = nlo;
                    L.sh_hi = nhi;
                    L.sh_above = above_bad;
                    L.sh_done = (sh == 0) ? 1u : 0u;
                    L.sh_nbin = (uint32_t)(in_bad >> 32);                // chunks inside the chosen sub-range
                }
            }
            __syncthreads();
            lo = L.sh_lo;
            hi = L.sh_hi;
            above = L.sh_above;
            const bool done = L.sh_done != 0;
            const uint32_t nbin = L.sh_nbin;
            // (no barrier: wave 0 writes these again only after the next pass's barrier, which every
            // lane reaches after these reads)
            if (nbin <= (uint32_t)kCandLimit) {
                use_cand = true;
                break;
            }
            if (done) break;      // one key left, held by more chunks than the pairwise step takes
        }
    }

    // Chunks above the final range are kept, chunks below it are dropped; inside it
    // the order (score descending, index ascending) decides.
    
#pragma unroll
    for (int i = 0; i < kIpt; ++i) R.keep[i] = valid[i] && (take_all || key[i] > hi);

    if (!take_all && use_cand) {
        // ---- few chunks left: the running totals of each come from comparing it with
        // all the others; the n*n comparisons are spread over the whole workgroup
        uint32_t mypos[kIpt];                             // (sh_ncand was cleared at the start)
#pragma unroll
        for (int i = 0; i < kIpt; ++i) {
            mypos[i] = 0xffffffffu;
            if (valid[i] && key[i] >= lo && key[i] <= hi) {
                const uint32_t pos = atomicAdd(&L.sh_ncand, 1u);
                if (pos < (uint32_t)kCandLimit) {
                    mypos[i] = pos;
                    // "j comes no later than i" <=> (key_j, -idx_j) >= (key_i, -idx_i)
                    L.cand_ki[pos] = ((uint64_t)key[i] << 32) | (uint32_t)(0x7fffffff - (c0 + i));
                    L.cand_tot[pos] = pack_tot(1, R.size[i]);
                }
            }
        }
        __syncthreads();
        const int n = (int)min(L.sh_ncand, (uint32_t)kCandLimit);
        int tshift = 0;                                   // 2^tshift lanes share one chunk
        while (tshift < 6 && (n << (tshift + 1)) <= kThreads) ++tshift;
        const int sub = tid & ((1 << tshift) - 1);
        // (one round unless the workgroup has fewer lanes than there are candidates)
        for (int cand = tid >> tshift; cand - (tid >> tshift) < n; cand += kThreads >> tshift) {
            uint64_t run = 0;
            if (cand < n) {
                const uint64_t mine_ki = L.cand_ki[cand];
                for (int j = sub; j < n; j += (1 << tshift))
                    if (L.cand_ki[j] >= mine_ki) run += L.cand_tot[j];
            }
            run = group_sum_u64(run, tshift);
            if (cand < n && sub == 0) {
                run += above;
                L.cand_keep[cand] = fits((uint32_t)(run >> 32), (uint32_t)run, max_cnt, max_tok) ? 1u : 0u;
            }
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < kIpt; ++i)
            if (mypos[i] != 0xffffffffu) R.keep[i] = L.cand_keep[mypos[i]] != 0u;
    } else if (!take_all) {
        // ---- many ties on one key: running totals in index order by a workgroup scan
        const uint32_t thr = lo;
        uint64_t tie_mine = 0;
#pragma unroll
        for (int i = 0; i < kIpt; ++i)
            if (valid[i] && key[i] == thr) tie_mine += pack_tot(1, R.size[i]);
        uint64_t tie_total;
        uint64_t run = above + block_excl_scan<true, kWaves>(tie_mine, L.wave_sums, &tie_total);
#pragma unroll
        for (int i = 0; i < kIpt; ++i) {
            if (valid[i] && key[i] == thr) {
                run += pack_tot(1, R.size[i]);
                R.keep[i] = fits((uint32_t)(run >> 32), (uint32_t)run, max_cnt, max_tok);
            }
        }
    }

    // ---- position of this lane's kept chunks in the ascending list ---------------
    uint64_t kept_mine = 0;
#pragma unroll
    for (int i = 0; i < kIpt; ++i)
        if (R.keep[i]) kept_mine += pack_tot(1, R.size[i]);
    R.kept_before = block_excl_scan<false, kWaves>(kept_mine, L.wave_sums2, &R.kept_total);      // (nothing has read these slots yet)
}

}  // namespace leoam
