/*
 * Float64 CPU oracle for the chunked sparse-attention decode step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * tests, the smoke check and the benchmark's cpu_baseline leg compare the HIP
 * library against.  Nothing in the product path may call it, and it shares no
 * code, header, table or helper with the HIP sources.
 *
 * Each function follows one passage of the paper (arXiv 2506.20187):
 *   orc_abstract_build   Sec. 4.3 "KV abstract extraction": the element-wise
 *                        maximum and minimum key vectors of a chunk.
 *   orc_abstract_append  the same abstract, kept up to date for one appended key.
 *   orc_chunk_score      Sec. 4.1 (chunk importance = upper bound of token
 *                        importance inside the chunk) and Sec. 4.3 (upper and
 *                        lower bounds from the abstract and the query).
 *   orc_topk_select      Sec. 4.2 (priority queue ordered by upper bound,
 *                        read from the front) and Sec. 6.1 (load only the
 *                        most important share of the cache).
 *   orc_sparse_attention Sec. 2.1 Eq. (1), restricted to the selected tokens.
 *   orc_chunk_compress   Sec. 4.4 / 6.1: the compressed (8-bit / 4-bit) store.
 *   orc_chunk_recompress the same store brought to a new set of 4-bit tags, chunk by chunk.
 *   orc_compression_share Sec. 4.4: the share of the data that is sent compressed.
 *
 * All floating-point work is done in double.  Stored fp32/fp16/bf16 inputs
 * are widened exactly.  Pinned by tests/test_oracle_*.py; no function here is
 * "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F32 = 0, ORC_F16 = 1, ORC_BF16 = 2, ORC_F64 = 3 };

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* IEEE binary16 -> double, exact, including subnormals. */
static double half_to_double(uint16_t h) {
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0) {
        v = ldexp((double)m, -24);
    } else if (e == 31) {
        v = m ? NAN : INFINITY;
    } else {
        v = ldexp((double)(m | 0x400), e - 25);
    }
    return sign ? -v : v;
}

/* bfloat16 is the upper half of a binary32. */
static double bf16_to_double(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static inline double widen(const void *p, int dtype, size_t i) {
    switch (dtype) {
    case ORC_F32: return (double)((const float *)p)[i];
    case ORC_F16: return half_to_double(((const uint16_t *)p)[i]);
    case ORC_BF16: return bf16_to_double(((const uint16_t *)p)[i]);
    default: return ((const double *)p)[i];
    }
}

/* widen n elements starting at element index `start` */
void orc_widen(const void *src, int dtype, size_t start, size_t n, double *dst) {
    for (size_t i = 0; i < n; ++i) dst[i] = widen(src, dtype, start + i);
}

/*
 * Sec. 4.3: abstract of chunk c of (b,h) = (kmax, kmin) with
 *   kmax[d] = max over t in [off[c], off[c+1]) of K[b,h,t,d], kmin likewise.
 * K: [B,Hkv,N,D] of `dtype`.  chunk_off: [B, c_max+1].  n_chunks: [B].
 * abs_out: double [B,Hkv,c_max,2,D]; [..,0,:] = kmax, [..,1,:] = kmin.
 * Rows of chunks >= n_chunks[b] are left untouched.
 */
int orc_abstract_build(int dtype, int B, int Hkv, int N, int D, const void *K, const int32_t *chunk_off,
                       const int32_t *n_chunks, int c_max, double *abs_out) {
    int bh;
#pragma omp parallel for schedule(dynamic, 1)
    for (bh = 0; bh < B * Hkv; ++bh) {
        int b = bh / Hkv;
        const int32_t *off = chunk_off + (size_t)b * (c_max + 1);
        for (int c = 0; c < n_chunks[b]; ++c) {
            double *kmax = abs_out + (((size_t)bh * c_max + c) * 2 + 0) * D;
            double *kmin = abs_out + (((size_t)bh * c_max + c) * 2 + 1) * D;
            for (int d = 0; d < D; ++d) {
                kmax[d] = -INFINITY;
                kmin[d] = INFINITY;
            }
            for (int t = off[c]; t < off[c + 1]; ++t) {
                size_t row = ((size_t)bh * N + t) * D;
                for (int d = 0; d < D; ++d) {
                    double x = widen(K, dtype, row + d);
                    if (x > kmax[d]) kmax[d] = x;
                    if (x < kmin[d]) kmin[d] = x;
                }
            }
        }
    }
    return 0;
}

/*
 * Sec. 4.3 abstract while decoding appends one key per sequence (Sec. 2.1: tokens
 * are generated one by one).  The new token of sequence b sits at index
 * t = chunk_off[b][n_chunks[b]] of K.  While the last chunk has fewer than
 * chunk_size tokens it takes the token (its kmax / kmin rows are compared with the
 * new key, element by element); otherwise a new chunk holding just that token is
 * opened.  status[b]: 0 done, 1 cache full, 2 no room for another chunk (then
 * nothing of that sequence changes).  abstract: double [B,Hkv,c_max,2,D].
 */
int orc_abstract_append(int dtype, int B, int Hkv, int N, int D, const void *K, int32_t *chunk_off, int32_t *n_chunks,
                        int c_max, int chunk_size, double *abstract, int32_t *status) {
    for (int b = 0; b < B; ++b) {
        int32_t *off = chunk_off + (size_t)b * (c_max + 1);
        int C = n_chunks[b];
        int t = off[C];
        int room = C > 0 && (t - off[C - 1]) < chunk_size;
        status[b] = 0;
        if (t >= N) {
            status[b] = 1;
            continue;
        }
        if (!room && C >= c_max) {
            status[b] = 2;
            continue;
        }
        int c = room ? C - 1 : C;
        for (int h = 0; h < Hkv; ++h) {
            size_t bh = (size_t)b * Hkv + h;
            double *kmax = abstract + ((bh * c_max + c) * 2 + 0) * D;
            double *kmin = abstract + ((bh * c_max + c) * 2 + 1) * D;
            for (int d = 0; d < D; ++d) {
                double x = widen(K, dtype, (bh * N + t) * D + d);
                if (!room) {
                    kmax[d] = x;
                    kmin[d] = x;
                } else {
                    if (x > kmax[d]) kmax[d] = x;
                    if (x < kmin[d]) kmin[d] = x;
                }
            }
        }
        if (room) {
            off[C] = t + 1;
        } else {
            off[C + 1] = t + 1;
            n_chunks[b] = C + 1;
        }
    }
    return 0;
}

/*
 * Sec. 4.1 / 4.3: bounds on q.k over the tokens of a chunk from its abstract:
 *   U_j[c] = sum_d max(q_j[d]*kmax[d], q_j[d]*kmin[d])   (upper)
 *   L_j[c] = sum_d min(q_j[d]*kmax[d], q_j[d]*kmin[d])   (lower)
 * For grouped-query attention the kv head's chunk score is the largest U over
 * the query heads of its group and the smallest L.
 * The stored score is the double sum rounded once to float, with -0 turned
 * into +0.  ub64/lb64 (nullable) receive the unrounded double values.
 * q: double [B,Hq,D]; abstract: double [B,Hkv,c_max,2,D].
 * Scores of chunks >= n_chunks[b] are set to -inf (ub) / +inf (lb).
 */
int orc_chunk_score(int B, int Hq, int Hkv, int D, const double *q, const double *abstract,
                    const int32_t *n_chunks, int c_max, float *ub, float *lb, double *ub64, double *lb64) {
    int G = Hq / Hkv;
    int bh;
#pragma omp parallel for schedule(dynamic, 1)
    for (bh = 0; bh < B * Hkv; ++bh) {
        int b = bh / Hkv, h = bh % Hkv;
        for (int c = 0; c < c_max; ++c) {
            size_t o = (size_t)bh * c_max + c;
            if (c >= n_chunks[b]) {
                if (ub) ub[o] = -INFINITY;
                if (lb) lb[o] = INFINITY;
                if (ub64) ub64[o] = -INFINITY;
                if (lb64) lb64[o] = INFINITY;
                continue;
            }
            const double *kmax = abstract + (o * 2 + 0) * D;
            const double *kmin = abstract + (o * 2 + 1) * D;
            double best_u = -INFINITY, best_l = INFINITY;
            for (int g = 0; g < G; ++g) {
                const double *qj = q + ((size_t)b * Hq + (size_t)h * G + g) * D;
                double u = 0.0, l = 0.0;
                for (int d = 0; d < D; ++d) {
                    double a = qj[d] * kmax[d], z = qj[d] * kmin[d];
                    u += (a > z) ? a : z;
                    l += (a < z) ? a : z;
                }
                if (u > best_u) best_u = u;
                if (l < best_l) best_l = l;
            }
            if (ub) ub[o] = (float)best_u + 0.0f;
            if (lb) lb[o] = (float)best_l + 0.0f;
            if (ub64) ub64[o] = best_u;
            if (lb64) lb64[o] = best_l;
        }
    }
    return 0;
}

typedef struct {
    float s;
    int32_t id;
} orc_item;

static int item_cmp(const void *a, const void *b) {
    const orc_item *x = (const orc_item *)a, *y = (const orc_item *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->id > y->id) - (x->id < y->id);
}

static int int_cmp(const void *a, const void *b) {
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/*
 * Sec. 4.2 / 6.1: order the chunks of (b,h) by score, highest first, equal
 * scores by lowest chunk index; read the list from the front and keep chunks
 * while the count stays <= max_chunks and the token total <= token_budget;
 * stop at the first chunk that does not fit.  A limit <= 0 is "no limit".
 * sel_idx: [B,Hkv,k_max], the kept chunk ids in ascending order, rest -1.
 * margin (nullable, [B,Hkv]): score of the last kept chunk minus score of the
 * first one left out (inf when nothing is left out or nothing is kept).
 * Returns -1 if some row would keep more than k_max chunks.
 */
int orc_topk_select(int B, int Hkv, const float *score, const int32_t *chunk_off, const int32_t *n_chunks,
                    int c_max, int max_chunks, int token_budget, int k_max, int32_t *sel_idx,
                    int32_t *sel_count, int32_t *sel_tokens, double *margin) {
    int rc = 0;
    int bh;
#pragma omp parallel for schedule(dynamic, 1)
    for (bh = 0; bh < B * Hkv; ++bh) {
        int b = bh / Hkv;
        int C = n_chunks[b];
        const int32_t *off = chunk_off + (size_t)b * (c_max + 1);
        orc_item *it = (orc_item *)malloc(sizeof(orc_item) * (size_t)(C > 0 ? C : 1));
        for (int c = 0; c < C; ++c) {
            it[c].s = score[(size_t)bh * c_max + c];
            it[c].id = c;
        }
        qsort(it, (size_t)C, sizeof(orc_item), item_cmp);
        int kept = 0;
        long tokens = 0;
        for (int i = 0; i < C; ++i) {
            int sz = off[it[i].id + 1] - off[it[i].id];
            if (max_chunks > 0 && kept + 1 > max_chunks) break;
            if (token_budget > 0 && tokens + sz > token_budget) break;
            kept += 1;
            tokens += sz;
        }
        int32_t *row = sel_idx + (size_t)bh * k_max;
        for (int i = 0; i < k_max; ++i) row[i] = -1;
        if (kept > k_max) {
#pragma omp critical
            rc = -1;
            kept = 0;
            tokens = 0;
        }
        for (int i = 0; i < kept; ++i) row[i] = it[i].id;
        qsort(row, (size_t)kept, sizeof(int32_t), int_cmp);
        sel_count[bh] = kept;
        sel_tokens[bh] = (int32_t)tokens;
        if (margin) margin[bh] = (kept > 0 && kept < C) ? (double)it[kept - 1].s - (double)it[kept].s : INFINITY;
        free(it);
    }
    return rc;
}

/*
 * Sec. 2.1 Eq. (1) over the tokens T of the kept chunks, for query head j of
 * kv head h = j / G:
 *   z_t = scale * (q_j . K[h,t]),  p = softmax_T(z),  out_j = sum_T p_t V[h,t],
 *   lse_j = log sum_T exp(z_t).
 * Nothing kept: out_j = 0, lse_j = -inf.
 * q: double [B,Hq,D]; K,V: [B,Hkv,N,D] of `dtype`; out: double [B,Hq,D];
 * lse: double [B,Hq] (nullable).
 */
int orc_sparse_attention(int dtype, int B, int Hq, int Hkv, int N, int D, const double *q, const void *K,
                         const void *V, const int32_t *chunk_off, int c_max, const int32_t *sel_idx,
                         const int32_t *sel_count, int k_max, double scale, double *out, double *lse) {
    int G = Hq / Hkv;
    int bj;
#pragma omp parallel for schedule(dynamic, 1)
    for (bj = 0; bj < B * Hq; ++bj) {
        int b = bj / Hq, j = bj % Hq, h = j / G;
        size_t bh = (size_t)b * Hkv + h;
        const int32_t *off = chunk_off + (size_t)b * (c_max + 1);
        const int32_t *row = sel_idx + bh * k_max;
        const double *qj = q + (size_t)bj * D;
        double *o = out + (size_t)bj * D;
        int cnt = sel_count[bh];
        long T = 0;
        for (int i = 0; i < cnt; ++i) T += off[row[i] + 1] - off[row[i]];
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        if (T == 0) {
            if (lse) lse[bj] = -INFINITY;
            continue;
        }
        double *z = (double *)malloc(sizeof(double) * (size_t)T);
        long n = 0;
        double m = -INFINITY;
        for (int i = 0; i < cnt; ++i) {
            for (int t = off[row[i]]; t < off[row[i] + 1]; ++t) {
                size_t base = (bh * N + t) * D;
                double dot = 0.0;
                for (int d = 0; d < D; ++d) dot += qj[d] * widen(K, dtype, base + d);
                z[n] = scale * dot;
                if (z[n] > m) m = z[n];
                ++n;
            }
        }
        double denom = 0.0;
        for (long i = 0; i < T; ++i) {
            z[i] = exp(z[i] - m);
            denom += z[i];
        }
        n = 0;
        for (int i = 0; i < cnt; ++i) {
            for (int t = off[row[i]]; t < off[row[i] + 1]; ++t) {
                size_t base = (bh * N + t) * D;
                double p = z[n++] / denom;
                for (int d = 0; d < D; ++d) o[d] += p * widen(V, dtype, base + d);
            }
        }
        if (lse) lse[bj] = m + log(denom);
        free(z);
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * Compressed KV store (Sec. 4.4 dynamic KV compression; Sec. 6.1 INT4).
 * A chunk of (b,h) is stored as 8-bit codes (one byte per element) or 4-bit
 * codes (two per byte, even channel in the low nibble); a stored value is
 * scale*code + zero with one (scale, zero) per (b,h,chunk,tensor).  The oracle
 * works on the stored codes: value(t,d) = (double)scale * code + (double)zero.
 * ------------------------------------------------------------------------ */
typedef struct {
    int64_t byte_off;
    int32_t bits;
    float scale_k, zero_k, scale_v, zero_v;
    int32_t reserved;
} orc_qchunk;

static inline int q_code(const uint8_t *blob, const orc_qchunk *m, int t_in_chunk, int d, int D) {
    if (m->bits == 8) return blob[m->byte_off + (int64_t)t_in_chunk * D + d];
    uint8_t byte = blob[m->byte_off + (int64_t)t_in_chunk * (D / 2) + d / 2];
    return (d & 1) ? (byte >> 4) : (byte & 15);
}

/* smallest binary16 value >= x (as a double); +inf if x is above the largest finite half */
static double half_ceil(double x) {
    /* walk the non-negative halves by bit pattern: they are ordered like their bits */
    if (x != x) return x;
    if (x > 65504.0) return INFINITY;
    if (x <= -65504.0) return -65504.0;       /* the most negative finite half is >= x */
    if (x >= 0.0) {
        uint16_t lo = 0, hi = 0x7bff;             /* smallest pattern with value >= x */
        while (lo < hi) {
            uint16_t mid = (uint16_t)((lo + hi) / 2);
            if (half_to_double(mid) >= x) hi = mid; else lo = (uint16_t)(mid + 1);
        }
        return half_to_double(lo);
    }
    /* x < 0: the largest magnitude m with -m >= x, i.e. largest pattern with value <= -x */
    double ax = -x;
    uint16_t lo = 0, hi = 0x7bff;
    while (lo < hi) {
        uint16_t mid = (uint16_t)((lo + hi + 1) / 2);
        if (half_to_double(mid) <= ax) lo = mid; else hi = (uint16_t)(mid - 1);
    }
    return -half_to_double(lo);
}

double orc_half_ceil(double x) { return half_ceil(x); }
double orc_half_floor(double x) { return -half_ceil(-x); }

/* dequantise the whole (b,h,chunk) store to double: out [B,Hkv,N,D] */
int orc_dequant(int B, int Hkv, int N, int D, const uint8_t *blob, const orc_qchunk *qmeta, int use_v,
                const int32_t *chunk_off, const int32_t *n_chunks, int c_max, double *out) {
    int bh;
#pragma omp parallel for schedule(dynamic, 1)
    for (bh = 0; bh < B * Hkv; ++bh) {
        int b = bh / Hkv;
        const int32_t *off = chunk_off + (size_t)b * (c_max + 1);
        for (int c = 0; c < n_chunks[b]; ++c) {
            const orc_qchunk *m = qmeta + (size_t)bh * c_max + c;
            double s = use_v ? (double)m->scale_v : (double)m->scale_k;
            double z = use_v ? (double)m->zero_v : (double)m->zero_k;
            for (int t = off[c]; t < off[c + 1]; ++t)
                for (int d = 0; d < D; ++d)
                    out[((size_t)bh * N + t) * D + d] = s * q_code(blob, m, t - off[c], d, D) + z;
        }
    }
    return 0;
}

/* One chunk of one (b,h) into the compressed store at byte `pos` of both blobs (Sec. 4.4 / 6.1):
 * per tensor, zero = min, scale = (max - min) / levels, code = round-half-even((x - zero) / scale)
 * kept inside 0..levels, levels = 15 (`four`) or 255; every operation that decides a code is one
 * float (binary32) operation.  Writes the record and rows * row bytes per blob, then zeros up to the
 * next multiple of 16.  Returns the bytes taken per blob. */
static int64_t orc_encode_chunk(int dtype, int N, int D, const void *K, const void *V, size_t bh, int t0, int t1,
                                int four, uint8_t *kblob, uint8_t *vblob, int64_t pos, orc_qchunk *m) {
    float levels = four ? 15.0f : 255.0f;
    int64_t row = four ? D / 2 : D, rows = t1 - t0;
    m->byte_off = pos;
    m->bits = four ? 4 : 8;
    for (int use_v = 0; use_v < 2; ++use_v) {
        const void *X = use_v ? V : K;
        uint8_t *blob = use_v ? vblob : kblob;
        float lo = INFINITY, hi = -INFINITY;
        for (int t = t0; t < t1; ++t)
            for (int d = 0; d < D; ++d) {
                float x = (float)widen(X, dtype, (bh * N + t) * D + d);
                if (x < lo) lo = x;
                if (x > hi) hi = x;
            }
        float range = hi - lo;
        float scale = range / levels;
        if (use_v) { m->scale_v = scale; m->zero_v = lo; } else { m->scale_k = scale; m->zero_k = lo; }
        for (int t = t0; t < t1; ++t)
            for (int d = 0; d < D; ++d) {
                float x = (float)widen(X, dtype, (bh * N + t) * D + d);
                int code = 0;
                if (scale > 0.0f) {
                    float diff = x - lo;
                    float r = rintf(diff / scale);
                    if (r < 0.0f) r = 0.0f;
                    if (r > levels) r = levels;
                    code = (int)r;
                }
                uint8_t *dst = blob + pos + (int64_t)(t - t0) * row;
                if (!four) dst[d] = (uint8_t)code;
                else if (d & 1) dst[d / 2] = (uint8_t)(dst[d / 2] | (code << 4));
                else dst[d / 2] = (uint8_t)code;
            }
    }
    int64_t bytes = (rows * row + 15) / 16 * 16;
    for (int64_t i = rows * row; i < bytes; ++i) kblob[pos + i] = vblob[pos + i] = 0;
    return bytes;
}

/* Sec. 4.4 "Dynamic KV compression" / Sec. 6.1 (KV compressed to INT4): builds the
 * compressed store from the 16-bit (or fp32) cache, every chunk by orc_encode_chunk.
 * Layout: the chunks of a (b,h) follow each other, each padded to a multiple of
 * 16 bytes; the (b,h) pairs follow each other; K and V blobs use the same
 * offsets.  Records of chunks >= n_chunks[b] are zero.  Returns 1 if the blobs
 * are too small (nothing is written then).  *total_bytes = bytes of one blob. */
int orc_chunk_compress(int dtype, int B, int Hkv, int N, int D, const void *K, const void *V,
                       const int32_t *chunk_off, const int32_t *n_chunks, int c_max, const uint8_t *four_bit,
                       uint8_t *kblob, uint8_t *vblob, int64_t blob_bytes, orc_qchunk *qmeta, int64_t *total_bytes) {
    int64_t total = 0;
    for (int b = 0; b < B; ++b) {
        const int32_t *off = chunk_off + (size_t)b * (c_max + 1);
        int64_t per_head = 0;
        for (int c = 0; c < n_chunks[b]; ++c) {
            int64_t row = four_bit[(size_t)b * c_max + c] ? D / 2 : D;
            per_head += ((int64_t)(off[c + 1] - off[c]) * row + 15) / 16 * 16;
        }
        total += per_head * Hkv;
    }
    *total_bytes = total;
    if (total > blob_bytes) return 1;
    memset(qmeta, 0, (size_t)B * Hkv * c_max * sizeof(orc_qchunk));
    int64_t pos = 0;
    for (int b = 0; b < B; ++b) {
        const int32_t *off = chunk_off + (size_t)b * (c_max + 1);
        for (int h = 0; h < Hkv; ++h) {
            size_t bh = (size_t)b * Hkv + h;
            for (int c = 0; c < n_chunks[b]; ++c)
                pos += orc_encode_chunk(dtype, N, D, K, V, bh, off[c], off[c + 1], four_bit[(size_t)b * c_max + c] != 0,
                                        kblob, vblob, pos, qmeta + bh * c_max + c);
        }
    }
    return 0;
}

/* Sec. 4.4: the compressed share changes from step to step (theta follows the measured times, and which
 * chunks are unimportant follows the scores), so a store built under the tags `four_old` is brought to
 * the tags `four_new` by re-encoding ONLY the chunks whose tag changed, from the uncompressed cache:
 *   8-bit -> 4-bit  the chunk is encoded again where it lies (it takes half of its old room),
 *   4-bit -> 8-bit  the chunk moves to fresh room at the end of the used part of the blobs; these
 *                   chunks are placed in (b, h, chunk) order starting at *used_bytes.
 * Every other byte of the blobs and every other record stays as it is.  *used_bytes grows by the room
 * the moved chunks take.  If that would exceed blob_bytes nothing is changed and 1 is returned (the
 * caller then rebuilds the store with orc_chunk_compress, which also closes the holes).
 * n_changed (nullable): chunks re-encoded, counted per (b, h, chunk). */
int orc_chunk_recompress(int dtype, int B, int Hkv, int N, int D, const void *K, const void *V,
                         const int32_t *chunk_off, const int32_t *n_chunks, int c_max, const uint8_t *four_old,
                         const uint8_t *four_new, uint8_t *kblob, uint8_t *vblob, int64_t blob_bytes,
                         orc_qchunk *qmeta, int64_t *used_bytes, int64_t *n_changed) {
    int64_t grow = 0, changed = 0;
    for (int b = 0; b < B; ++b) {
        const int32_t *off = chunk_off + (size_t)b * (c_max + 1);
        for (int c = 0; c < n_chunks[b]; ++c) {
            int was = four_old[(size_t)b * c_max + c] != 0, is = four_new[(size_t)b * c_max + c] != 0;
            if (was && !is) grow += (((int64_t)(off[c + 1] - off[c]) * D + 15) / 16 * 16) * Hkv;
        }
    }
    if (n_changed) *n_changed = 0;
    if (*used_bytes + grow > blob_bytes) return 1;
    int64_t pos = *used_bytes;
    for (int b = 0; b < B; ++b) {
        const int32_t *off = chunk_off + (size_t)b * (c_max + 1);
        for (int h = 0; h < Hkv; ++h) {
            size_t bh = (size_t)b * Hkv + h;
            for (int c = 0; c < n_chunks[b]; ++c) {
                int was = four_old[(size_t)b * c_max + c] != 0, is = four_new[(size_t)b * c_max + c] != 0;
                orc_qchunk *m = qmeta + bh * c_max + c;
                if (was == is) continue;
                ++changed;
                if (is) {
                    orc_encode_chunk(dtype, N, D, K, V, bh, off[c], off[c + 1], 1, kblob, vblob, m->byte_off, m);
                } else {
                    pos += orc_encode_chunk(dtype, N, D, K, V, bh, off[c], off[c + 1], 0, kblob, vblob, pos, m);
                }
            }
        }
    }
    *used_bytes = pos;
    if (n_changed) *n_changed = changed;
    return 0;
}

/* Sec. 4.4: share theta of a layer's transmitted KV bytes that is sent compressed.
 * Sending D bytes at bandwidth B with a share theta compressed to the ratio delta takes
 * T0 + D (1 - theta + theta delta) / B (T0 = the other evaluation and transmission
 * time); it hides behind the computation Tc plus the decompression of the compressed
 * share, D theta / R for a decompression rate R (B and R come from a hardware
 * measurement made beforehand).  The transmission side falls with theta and the computation side rises, so
 * the two meet at most once: theta is that point, kept inside [0, 1] (0: already
 * hidden without compression; 1: not hidden even when everything is compressed). */
double orc_compression_share(double D, double delta, double B, double T0, double Tc, double R) {
    double excess = T0 + D / B - Tc;                         /* transmission beyond computation at theta = 0 */
    double gain = D * (1.0 - delta) / B + D / R;             /* how much one unit of theta closes of it */
    if (excess <= 0.0) return 0.0;
    if (excess >= gain) return 1.0;
    return excess / gain;
}

/* Sec. 4.3 abstract over the stored values, rounded outward to binary16:
 * kmax = half_ceil(max_t value), kmin = half_floor(min_t value). */
int orc_abstract_build_q(int B, int Hkv, int D, const uint8_t *kblob, const orc_qchunk *qmeta,
                         const int32_t *chunk_off, const int32_t *n_chunks, int c_max, double *abs_out) {
    int bh;
#pragma omp parallel for schedule(dynamic, 1)
    for (bh = 0; bh < B * Hkv; ++bh) {
        int b = bh / Hkv;
        const int32_t *off = chunk_off + (size_t)b * (c_max + 1);
        for (int c = 0; c < n_chunks[b]; ++c) {
            const orc_qchunk *m = qmeta + (size_t)bh * c_max + c;
            double *kmax = abs_out + (((size_t)bh * c_max + c) * 2 + 0) * D;
            double *kmin = abs_out + (((size_t)bh * c_max + c) * 2 + 1) * D;
            for (int d = 0; d < D; ++d) {
                double hi = -INFINITY, lo = INFINITY;
                for (int t = off[c]; t < off[c + 1]; ++t) {
                    double x = (double)m->scale_k * q_code(kblob, m, t - off[c], d, D) + (double)m->zero_k;
                    if (x > hi) hi = x;
                    if (x < lo) lo = x;
                }
                kmax[d] = half_ceil(hi);
                kmin[d] = -half_ceil(-lo);
            }
        }
    }
    return 0;
}

/* Eq. (1) over the kept chunks of the compressed store (same as orc_sparse_attention,
 * K[t] and V[t] being the stored values). */
int orc_sparse_attention_q(int B, int Hq, int Hkv, int D, const double *q, const uint8_t *kblob,
                           const uint8_t *vblob, const orc_qchunk *qmeta, const int32_t *chunk_off, int c_max,
                           const int32_t *sel_idx, const int32_t *sel_count, int k_max, double scale, double *out,
                           double *lse) {
    int G = Hq / Hkv;
    int bj;
#pragma omp parallel for schedule(dynamic, 1)
    for (bj = 0; bj < B * Hq; ++bj) {
        int b = bj / Hq, j = bj % Hq, h = j / G;
        size_t bh = (size_t)b * Hkv + h;
        const int32_t *off = chunk_off + (size_t)b * (c_max + 1);
        const int32_t *row = sel_idx + bh * k_max;
        const double *qj = q + (size_t)bj * D;
        double *o = out + (size_t)bj * D;
        int cnt = sel_count[bh];
        long T = 0;
        for (int i = 0; i < cnt; ++i) T += off[row[i] + 1] - off[row[i]];
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        if (T == 0) {
            if (lse) lse[bj] = -INFINITY;
            continue;
        }
        double *z = (double *)malloc(sizeof(double) * (size_t)T);
        long n = 0;
        double mx = -INFINITY;
        for (int i = 0; i < cnt; ++i) {
            const orc_qchunk *m = qmeta + bh * c_max + row[i];
            for (int t = off[row[i]]; t < off[row[i] + 1]; ++t) {
                double dot = 0.0;
                for (int d = 0; d < D; ++d)
                    dot += qj[d] * ((double)m->scale_k * q_code(kblob, m, t - off[row[i]], d, D) + (double)m->zero_k);
                z[n] = scale * dot;
                if (z[n] > mx) mx = z[n];
                ++n;
            }
        }
        double denom = 0.0;
        for (long i = 0; i < T; ++i) {
            z[i] = exp(z[i] - mx);
            denom += z[i];
        }
        n = 0;
        for (int i = 0; i < cnt; ++i) {
            const orc_qchunk *m = qmeta + bh * c_max + row[i];
            for (int t = off[row[i]]; t < off[row[i] + 1]; ++t) {
                double p = z[n++] / denom;
                for (int d = 0; d < D; ++d)
                    o[d] += p * ((double)m->scale_v * q_code(vblob, m, t - off[row[i]], d, D) + (double)m->zero_v);
            }
        }
        if (lse) lse[bj] = mx + log(denom);
        free(z);
    }
    return 0;
}

/* ===========================================================================
 * Tree-structured chunk refinement (Sec. 4.2, "Tree-structured KV chunk
 * management"; Fig. 9).  Per (sequence, kv head):
 *
 *   - the context starts as equal chunks of chunk_size tokens, each evaluated
 *     once: upper bound U and lower bound L of the token importance in it
 *     (importance of token t = max over the group's heads of q_j.k_t; U as in
 *     orc_chunk_score; L = the LARGEST of the heads' lower bounds, which every
 *     token's importance still reaches; both from the chunk's element-wise
 *     max / min keys, so that U = L = the importance for a single token);
 *   - chunks are kept in a queue ordered by U; the front of the queue is read
 *     until it covers k tokens.  A chunk whose lower bound beats the upper
 *     bound of all but at most k tokens holds important tokens only and is
 *     confirmed; the other front chunks are mixed: they are split in two and
 *     their halves evaluated (two evaluations per split);
 *   - this repeats until the front consists of confirmed chunks and single
 *     tokens, or max_rounds is reached;
 *   - runs of unimportant chunks (upper bound below the k-th largest lower
 *     bound: they cannot hold one of the k most important tokens) are merged,
 *     and so are runs of confirmed chunks.
 *
 * Order statistics are over tokens: a chunk counts size times.
 *   v      = k-th largest U      (chunks with U >= v are the front of the queue)
 *   mu     = (k+1)-th largest U  (-inf when k == N)
 *   lambda = k-th largest L
 *   confirmed: L > mu;  unimportant: U < lambda;  split: U >= v, not confirmed, size > 1.
 * A split puts ceil(size/2) tokens in the left half.  If a round's splits
 * would exceed node_cap nodes the refinement stops there (status 1).
 *
 * Output per (b,h): boundaries of the final partition, a score per chunk
 * (FLT_MAX for confirmed chunks, otherwise its U; merged unimportant runs carry
 * the largest U of the run), the number of chunks, and the number of
 * evaluations (initial chunks + 2 per split).  Selecting from these scores
 * with a token budget of k (orc_topk_select) gives the important tokens.
 * =========================================================================== */
typedef struct {
    int start, size;
    float U, L;
} tnode;

static void node_bounds(int dtype, const void *K, const double *q, int G, int D, size_t base_row, tnode *nd,
                        double *kmax, double *kmin) {
    for (int d = 0; d < D; ++d) {
        kmax[d] = -INFINITY;
        kmin[d] = INFINITY;
    }
    for (int t = nd->start; t < nd->start + nd->size; ++t)
        for (int d = 0; d < D; ++d) {
            double x = widen(K, dtype, (base_row + t) * D + d);
            if (x > kmax[d]) kmax[d] = x;
            if (x < kmin[d]) kmin[d] = x;
        }
    float U = -INFINITY, L = -INFINITY;
    for (int j = 0; j < G; ++j) {
        double u = 0.0, l = 0.0;
        for (int d = 0; d < D; ++d) {
            double a = q[(size_t)j * D + d] * kmax[d], b = q[(size_t)j * D + d] * kmin[d];
            u += a > b ? a : b;
            l += a > b ? b : a;
        }
        float uf = (float)u + 0.0f, lf = (float)l + 0.0f;
        if (uf > U) U = uf;
        if (lf > L) L = lf;
    }
    nd->U = U;
    nd->L = L;
}

typedef struct {
    float key;
    int weight;
} wkey;

static int wkey_desc(const void *a, const void *b) {
    float x = ((const wkey *)a)->key, y = ((const wkey *)b)->key;
    return (x < y) - (x > y);
}

/* the rank-th largest key when every key counts `weight` times (rank >= 1); -inf if there are fewer */
static float weighted_kth_largest(wkey *w, int n, long rank) {
    qsort(w, n, sizeof(wkey), wkey_desc);
    long acc = 0;
    for (int i = 0; i < n; ++i) {
        acc += w[i].weight;
        if (acc >= rank) return w[i].key;
    }
    return -INFINITY;
}

int orc_tree_refine(int dtype, int B, int Hq, int Hkv, int N, int D, const void *K, const double *q, int chunk_size,
                    int k_tokens, int max_rounds, int node_cap, int32_t *ref_off, float *ref_score,
                    int32_t *ref_count, int32_t *ref_evals, int32_t *ref_status) {
    int G = Hq / Hkv;
    int m0 = (N + chunk_size - 1) / chunk_size;
    if (m0 > node_cap || k_tokens < 1 || k_tokens > N) return -1;
    int bh;
#pragma omp parallel for schedule(dynamic, 1)
    for (bh = 0; bh < B * Hkv; ++bh) {
        int b = bh / Hkv, h = bh % Hkv;
        const double *qg = q + ((size_t)b * Hq + (size_t)h * G) * D;
        size_t base_row = (size_t)bh * N;
        tnode *cur = (tnode *)malloc(sizeof(tnode) * (size_t)node_cap), *nxt = (tnode *)malloc(sizeof(tnode) * (size_t)node_cap);
        wkey *w = (wkey *)malloc(sizeof(wkey) * (size_t)node_cap);
        double *kmax = (double *)malloc(sizeof(double) * D), *kmin = (double *)malloc(sizeof(double) * D);
        int n = m0, evals = m0, status = 0;
        for (int c = 0; c < m0; ++c) {
            cur[c].start = c * chunk_size;
            cur[c].size = (c + 1) * chunk_size <= N ? chunk_size : N - c * chunk_size;
            node_bounds(dtype, K, qg, G, D, base_row, &cur[c], kmax, kmin);
        }
        float lambda = 0.f, mu = 0.f;
        for (int round = 0;; ++round) {
            for (int i = 0; i < n; ++i) { w[i].key = cur[i].U; w[i].weight = cur[i].size; }
            float v = weighted_kth_largest(w, n, k_tokens);
            for (int i = 0; i < n; ++i) { w[i].key = cur[i].U; w[i].weight = cur[i].size; }
            mu = weighted_kth_largest(w, n, (long)k_tokens + 1);
            for (int i = 0; i < n; ++i) { w[i].key = cur[i].L; w[i].weight = cur[i].size; }
            lambda = weighted_kth_largest(w, n, k_tokens);
            if (round >= max_rounds) break;
            int n_split = 0;
            for (int i = 0; i < n; ++i)
                if (cur[i].U >= v && !(cur[i].L > mu) && cur[i].size > 1) ++n_split;
            if (n_split == 0) break;
            if (n + n_split > node_cap) {
                status = 1;
                break;
            }
            int m = 0;
            for (int i = 0; i < n; ++i) {
                if (cur[i].U >= v && !(cur[i].L > mu) && cur[i].size > 1) {
                    int left = (cur[i].size + 1) / 2;
                    nxt[m].start = cur[i].start;
                    nxt[m].size = left;
                    node_bounds(dtype, K, qg, G, D, base_row, &nxt[m], kmax, kmin);
                    ++m;
                    nxt[m].start = cur[i].start + left;
                    nxt[m].size = cur[i].size - left;
                    node_bounds(dtype, K, qg, G, D, base_row, &nxt[m], kmax, kmin);
                    ++m;
                    evals += 2;
                } else {
                    nxt[m++] = cur[i];
                }
            }
            tnode *tmp = cur;
            cur = nxt;
            nxt = tmp;
            n = m;
        }
        /* final partition: merge runs of confirmed chunks and runs of unimportant chunks */
        int32_t *off = ref_off + (size_t)bh * (node_cap + 1);
        float *sc = ref_score + (size_t)bh * node_cap;
        int m = 0, prev_kind = -1;      /* 0 mixed, 1 confirmed, 2 unimportant */
        for (int i = 0; i < n; ++i) {
            int kind = (cur[i].L > mu) ? 1 : (cur[i].U < lambda ? 2 : 0);
            if (m > 0 && kind != 0 && kind == prev_kind) {
                if (kind == 2 && cur[i].U > sc[m - 1]) sc[m - 1] = cur[i].U;
            } else {
                off[m] = cur[i].start;
                sc[m] = kind == 1 ? 3.402823466e+38f : cur[i].U;
                ++m;
            }
            prev_kind = kind;
        }
        off[m] = N;
        ref_count[bh] = m;
        ref_evals[bh] = evals;
        ref_status[bh] = status;
        free(cur);
        free(nxt);
        free(w);
        free(kmax);
        free(kmin);
    }
    return 0;
}
