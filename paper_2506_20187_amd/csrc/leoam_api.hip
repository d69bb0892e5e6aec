// C ABI of the library (include/leoam.h): argument checks, then kernel launches
// on the caller's stream.  Nothing here allocates or synchronises, except the
// debug helper leoam_validate_boundaries.
#include <mutex>
#include <vector>

#include "leoam_dev.h"

namespace leoam {
hipError_t abstract_build_dispatch(const leoam_shape*, const void*, const int32_t*, const int32_t*, void*, hipStream_t);
hipError_t chunk_score_dispatch(const leoam_shape*, const void*, const void*, const int32_t*, float*, float*, hipStream_t);
hipError_t topk_select_dispatch(const leoam_shape*, const float*, const int32_t*, const int32_t*, int, int, int32_t*,
                                int32_t*, int32_t*, hipStream_t);
hipError_t attention_dispatch(const leoam_shape*, const void*, const void*, const void*, const void*, const int32_t*,
                              const int32_t*, const int32_t*, const int32_t*, float, float*, float*, void*, size_t,
                              int32_t*, hipStream_t);
hipError_t abstract_build_q_dispatch(const leoam_shape*, const void*, const void*, const int32_t*, const int32_t*, void*,
                                     hipStream_t);
int attention_q_max_sel();
size_t attention_workspace_bytes(const leoam_shape*, int);
size_t attention_min_workspace_bytes(const leoam_shape*);
int attention_max_sel();
hipError_t select_attention_dispatch(const leoam_shape*, const float*, const void*, const void*, const void*, const void*,
                                     const int32_t*, const int32_t*, int, int, float, int32_t*, int32_t*, int32_t*,
                                     float*, float*, void*, size_t, hipStream_t, bool with_exchange = true);
size_t select_attention_workspace_bytes(const leoam_shape*, int, bool with_exchange = true);
size_t select_attention_min_workspace_bytes(const leoam_shape*, bool with_exchange = true);
size_t select_attention_counter_bytes(const leoam_shape*, bool with_exchange = true);
hipError_t workspace_zero_dispatch(void*, size_t, hipStream_t);
size_t tree_workspace_bytes(const leoam_shape*, int);
hipError_t tree_refine_dispatch(const leoam_shape*, const void*, const void*, const void*, int, int, int, int, int32_t*,
                                float*, int32_t*, int32_t*, int32_t*, void*, hipStream_t);
size_t compressed_bytes_bound(const leoam_shape*);
hipError_t compression_tags_dispatch(const leoam_shape*, const int32_t*, const int32_t*, const int32_t*, uint8_t*, hipStream_t);
hipError_t compress_dispatch(const leoam_shape*, const void*, const void*, const int32_t*, const int32_t*, const uint8_t*,
                             void*, void*, void*, size_t, long long*, hipStream_t);
hipError_t recompress_dispatch(const leoam_shape*, const void*, const void*, const int32_t*, const int32_t*, const uint8_t*,
                               const uint8_t*, void*, void*, void*, size_t, long long*, long long*, hipStream_t);
hipError_t abstract_append_dispatch(const leoam_shape*, const void*, int32_t*, int32_t*, int, void*, int32_t*, hipStream_t);

// scores of the first `sink` and the last `tail` chunks of every (b, h) row become FLT_MAX
__global__ void score_pin_kernel(const int32_t* __restrict__ n_chunks, int sink, int tail, float* __restrict__ score,
                                 int c_max, int n_kv_heads) {
    const int bh = blockIdx.x, b = bh / n_kv_heads;
    const int n = min(max(n_chunks[b], 0), c_max);
    float* row = score + (size_t)bh * c_max;
    const int head_end = min(sink, n), tail_begin = max(n - min(tail, n), head_end);
    for (int c = threadIdx.x; c < head_end; c += blockDim.x) row[c] = 3.402823466e+38f;
    for (int c = tail_begin + threadIdx.x; c < n; c += blockDim.x) row[c] = 3.402823466e+38f;
}

__global__ void copy_probe_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n16) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = src[i];
}

// Reads `n16` 16-byte words and keeps nothing: the read-only stream that HBM-bound kernels are compared with.
// Every workgroup reads one contiguous 16 KiB piece, four loads per lane in flight (many short workgroups
// walking the buffer in launch order measured fastest on MI355X: 6.3-6.8 TB/s against 5.6 for a
// grid-stride loop over resident workgroups).  The words are folded by xor and stored only if the fold
// equals a value that data does not produce in practice, which is what keeps the loads alive.
constexpr size_t kReadProbePiece = 1024;      // 16-byte words per workgroup
__global__ __launch_bounds__(256) void read_probe_kernel(const uint4* __restrict__ src, size_t n16,
                                                         uint32_t* __restrict__ sink) {
    const size_t base = (size_t)blockIdx.x * kReadProbePiece + threadIdx.x;
    uint4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const size_t i = base + 256 * u;
        v[u] = src[i < n16 ? i : n16 - 1];      // (unconditional loads; a word past the end re-reads the last one)
    }
    uint4 a = make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        a.x ^= v[u].x;
        a.y ^= v[u].y;
        a.z ^= v[u].z;
        a.w ^= v[u].w;
    }
    if ((a.x ^ a.y) == 0x9e3779b9u && (a.z ^ a.w) == 0x7f4a7c15u) sink[0] = a.x;
}

static int check_shape(const leoam_shape* s) {
    if (!s) return LEOAM_E_INVALID_ARG;
    if (s->batch < 1 || s->n_q_heads < 1 || s->n_kv_heads < 1 || s->n_ctx < 1 || s->c_max < 1 || s->k_max < 1)
        return LEOAM_E_INVALID_ARG;
    if (s->n_q_heads % s->n_kv_heads) return LEOAM_E_INVALID_ARG;
    if (s->k_max > s->c_max) return LEOAM_E_INVALID_ARG;
    if (s->head_dim != LEOAM_D) return LEOAM_E_UNSUPPORTED;
    const int g = s->n_q_heads / s->n_kv_heads;
    if (g != 1 && g != 2 && g != 4 && g != 8) return LEOAM_E_UNSUPPORTED;
    if (s->kv_dtype == LEOAM_Q8Q4) {
        if (s->abstract_dtype != LEOAM_F16) return LEOAM_E_UNSUPPORTED;
    } else {
        if (s->kv_dtype != LEOAM_F32 && s->kv_dtype != LEOAM_F16 && s->kv_dtype != LEOAM_BF16) return LEOAM_E_UNSUPPORTED;
        if (s->abstract_dtype != s->kv_dtype) return LEOAM_E_UNSUPPORTED;
    }
    if (s->c_max > 16384) return LEOAM_E_UNSUPPORTED;
    if ((long long)s->batch * s->n_kv_heads > 65535 * 8) return LEOAM_E_UNSUPPORTED;
    if (s->n_kv_heads > 65535 || s->batch > 65535) return LEOAM_E_UNSUPPORTED;
    return LEOAM_OK;
}

static inline int from_hip(hipError_t e) { return e == hipSuccess ? LEOAM_OK : LEOAM_E_HIP; }

// K, V, q, the abstract and the blobs are read with 16-byte loads
template <typename... P> static inline bool misaligned16(P... p) { return ((... | (uintptr_t)p) & 15u) != 0; }

// ---- workspace of chunk_select_attention_decode_static ------------------------------------------
// Device memory that belongs to the library image: every GPU the library runs on holds its own copy
// until the process ends.  `static_scratch` names the array in DEVICE code only; on the host the
// name is a stand-in without a device address, so host code asks the runtime for the address once per
// device (with that device current) and uses that pointer from then on.
static __device__ __align__(256) unsigned char static_scratch[LEOAM_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

static void* static_scratch_ptr() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(static_scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}
}  // namespace leoam

using namespace leoam;

extern "C" {

int kv_chunk_abstract_build(const leoam_shape* shape, const void* K, const void* qmeta, const int32_t* chunk_off,
                            const int32_t* n_chunks, void* abstract, void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!K || !chunk_off || !n_chunks || !abstract) return LEOAM_E_INVALID_ARG;
    if (misaligned16(K, abstract, qmeta)) return LEOAM_E_INVALID_ARG;
    if (shape->kv_dtype == LEOAM_Q8Q4) {
        if (!qmeta) return LEOAM_E_INVALID_ARG;
        return from_hip(abstract_build_q_dispatch(shape, K, qmeta, chunk_off, n_chunks, abstract, (hipStream_t)stream));
    }
    return from_hip(abstract_build_dispatch(shape, K, chunk_off, n_chunks, abstract, (hipStream_t)stream));
}

int kv_chunk_abstract_append(const leoam_shape* shape, const void* K, int32_t* chunk_off, int32_t* n_chunks,
                             int32_t chunk_size, void* abstract, int32_t* status, void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!K || !chunk_off || !n_chunks || !abstract || chunk_size < 1) return LEOAM_E_INVALID_ARG;
    if (misaligned16(K, abstract)) return LEOAM_E_INVALID_ARG;
    if (shape->kv_dtype == LEOAM_Q8Q4) return LEOAM_E_UNSUPPORTED;
    return from_hip(abstract_append_dispatch(shape, K, chunk_off, n_chunks, chunk_size, abstract, status,
                                             (hipStream_t)stream));
}

static int check_tree(const leoam_shape* shape, int32_t chunk_size, int32_t k_tokens, int32_t max_rounds,
                      int32_t node_cap) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (shape->kv_dtype == LEOAM_Q8Q4) return LEOAM_E_UNSUPPORTED;
    if (chunk_size < 1 || node_cap < 1 || max_rounds < 0) return LEOAM_E_INVALID_ARG;
    if (k_tokens < 1 || k_tokens > shape->n_ctx) return LEOAM_E_INVALID_ARG;
    const long long m0 = ((long long)shape->n_ctx + chunk_size - 1) / chunk_size;
    if (m0 > node_cap || m0 > shape->c_max) return LEOAM_E_INVALID_ARG;
    return LEOAM_OK;
}

size_t leoam_tree_workspace_bytes(const leoam_shape* shape, int32_t node_cap) {
    if (check_shape(shape) || node_cap < 1) return 0;
    return tree_workspace_bytes(shape, node_cap);
}

int chunk_tree_refine(const leoam_shape* shape, const void* q, const void* K, const void* abstract, int32_t chunk_size,
                      int32_t k_tokens, int32_t max_rounds, int32_t node_cap, int32_t* ref_off, float* ref_score,
                      int32_t* ref_count, int32_t* ref_evals, int32_t* ref_status, void* workspace,
                      size_t workspace_bytes, void* stream) {
    int rc = check_tree(shape, chunk_size, k_tokens, max_rounds, node_cap);
    if (rc) return rc;
    if (!q || !K || !abstract || !ref_off || !ref_score || !ref_count || !ref_evals || !ref_status)
        return LEOAM_E_INVALID_ARG;
    if (misaligned16(q, K, abstract)) return LEOAM_E_INVALID_ARG;
    if (!workspace || workspace_bytes < tree_workspace_bytes(shape, node_cap) || ((uintptr_t)workspace & 15u))
        return LEOAM_E_WORKSPACE;
    return from_hip(tree_refine_dispatch(shape, q, K, abstract, chunk_size, k_tokens, max_rounds, node_cap, ref_off,
                                         ref_score, ref_count, ref_evals, ref_status, workspace, (hipStream_t)stream));
}

double leoam_tree_evaluations(int64_t n_tokens, int64_t n_chunks, double rho) {
    if (n_chunks < 1 || n_tokens < n_chunks || n_tokens % n_chunks || !(rho >= 0.0) || !(rho <= 1.0)) return -1.0;
    int64_t size = n_tokens / n_chunks;
    if (size & (size - 1)) return -1.0;
    int levels = 0;
    while (((int64_t)1 << levels) < size) ++levels;
    double sum = 0.0, term = 1.0;
    for (int i = 0; i < levels; ++i) {
        sum += term;
        term *= 2.0 * rho;
    }
    return (double)n_chunks * sum;
}

int chunk_score(const leoam_shape* shape, const void* q, const void* abstract, const int32_t* n_chunks,
                float* score_ub, float* score_lb, void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!q || !abstract || !n_chunks || !score_ub) return LEOAM_E_INVALID_ARG;
    if (misaligned16(q, abstract)) return LEOAM_E_INVALID_ARG;
    return from_hip(chunk_score_dispatch(shape, q, abstract, n_chunks, score_ub, score_lb, (hipStream_t)stream));
}

int chunk_score_pin(const leoam_shape* shape, const int32_t* n_chunks, int32_t sink_chunks, int32_t tail_chunks,
                    float* score_ub, void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!n_chunks || !score_ub || sink_chunks < 0 || tail_chunks < 0) return LEOAM_E_INVALID_ARG;
    if (sink_chunks == 0 && tail_chunks == 0) return LEOAM_OK;
    hipLaunchKernelGGL(score_pin_kernel, dim3(shape->batch * shape->n_kv_heads), dim3(256), 0, (hipStream_t)stream,
                       n_chunks, sink_chunks, tail_chunks, score_ub, shape->c_max, shape->n_kv_heads);
    return from_hip(hipGetLastError());
}

int chunk_topk_select(const leoam_shape* shape, const float* score_ub, const int32_t* chunk_off,
                      const int32_t* n_chunks, int32_t max_chunks, int32_t token_budget, int32_t* sel_idx,
                      int32_t* sel_count, int32_t* sel_tokens, void* workspace, size_t workspace_bytes,
                      void* stream) {
    (void)workspace;
    (void)workspace_bytes;
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!score_ub || !chunk_off || !n_chunks || !sel_idx || !sel_count) return LEOAM_E_INVALID_ARG;
    return from_hip(topk_select_dispatch(shape, score_ub, chunk_off, n_chunks, max_chunks, token_budget, sel_idx,
                                         sel_count, sel_tokens, (hipStream_t)stream));
}

int sparse_chunk_attention_decode(const leoam_shape* shape, const void* q, const void* K, const void* V,
                                  const void* qmeta, const int32_t* chunk_off, const int32_t* n_chunks, const int32_t* sel_idx,
                                  const int32_t* sel_count, float softmax_scale, float* out, float* lse,
                                  void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!q || !K || !V || !chunk_off || !n_chunks || !sel_idx || !sel_count || !out) return LEOAM_E_INVALID_ARG;
    if (misaligned16(q, K, V, qmeta)) return LEOAM_E_INVALID_ARG;
    if (shape->k_max > attention_max_sel()) return LEOAM_E_UNSUPPORTED;
    if (shape->kv_dtype == LEOAM_Q8Q4) {
        if (!qmeta) return LEOAM_E_INVALID_ARG;
        if (shape->k_max > attention_q_max_sel()) return LEOAM_E_UNSUPPORTED;
    }
    if (!workspace || workspace_bytes < attention_min_workspace_bytes(shape)) return LEOAM_E_WORKSPACE;
    if (((uintptr_t)workspace & 15u) != 0) return LEOAM_E_WORKSPACE;
    return from_hip(attention_dispatch(shape, q, K, V, qmeta, chunk_off, n_chunks, sel_idx, sel_count, softmax_scale, out, lse,
                                       workspace, workspace_bytes, nullptr, (hipStream_t)stream));
}

int chunk_select_attention_decode(const leoam_shape* shape, const float* score_ub, const void* q, const void* K,
                                  const void* V, const void* qmeta, const int32_t* chunk_off, const int32_t* n_chunks,
                                  int32_t max_chunks, int32_t token_budget, float softmax_scale, int32_t* sel_idx,
                                  int32_t* sel_count, int32_t* sel_tokens, float* out, float* lse, void* workspace,
                                  size_t workspace_bytes, void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    // (score_ub == NULL: the kept lists are inputs and the call only attends)
    if (!q || !K || !V || !chunk_off || !n_chunks || !sel_idx || !sel_count || !out) return LEOAM_E_INVALID_ARG;
    if (misaligned16(q, K, V, qmeta)) return LEOAM_E_INVALID_ARG;
    if (shape->k_max > attention_max_sel()) return LEOAM_E_UNSUPPORTED;
    if (shape->kv_dtype == LEOAM_Q8Q4) {
        if (!qmeta) return LEOAM_E_INVALID_ARG;
        if (shape->k_max > attention_q_max_sel()) return LEOAM_E_UNSUPPORTED;
    }
    if (!workspace || workspace_bytes < select_attention_min_workspace_bytes(shape)) return LEOAM_E_WORKSPACE;
    if (((uintptr_t)workspace & 15u) != 0) return LEOAM_E_WORKSPACE;
    return from_hip(select_attention_dispatch(shape, score_ub, q, K, V, qmeta, chunk_off, n_chunks, max_chunks,
                                              token_budget, softmax_scale, sel_idx, sel_count, sel_tokens, out, lse,
                                              workspace, workspace_bytes, (hipStream_t)stream));
}

int chunk_select_attention_decode_static(const leoam_shape* shape, const float* score_ub, const void* q, const void* K,
                                         const void* V, const void* qmeta, const int32_t* chunk_off,
                                         const int32_t* n_chunks, int32_t max_chunks, int32_t token_budget,
                                         float softmax_scale, int32_t* sel_idx, int32_t* sel_count, int32_t* sel_tokens,
                                         float* out, float* lse, void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    // (score_ub == NULL: the kept lists are inputs and the call only attends)
    if (!q || !K || !V || !chunk_off || !n_chunks || !sel_idx || !sel_count || !out) return LEOAM_E_INVALID_ARG;
    if (misaligned16(q, K, V, qmeta)) return LEOAM_E_INVALID_ARG;
    if (shape->k_max > attention_max_sel()) return LEOAM_E_UNSUPPORTED;
    if (shape->kv_dtype == LEOAM_Q8Q4) {
        if (!qmeta) return LEOAM_E_INVALID_ARG;
        if (shape->k_max > attention_q_max_sel()) return LEOAM_E_UNSUPPORTED;
    }
    // the smallest workspace the call can run with must fit the static buffer
    if (select_attention_min_workspace_bytes(shape, false) > (size_t)LEOAM_STATIC_SCRATCH_BYTES) return LEOAM_E_WORKSPACE;
    void* ws = static_scratch_ptr();
    if (!ws) return LEOAM_E_HIP;
    size_t bytes = select_attention_workspace_bytes(shape, token_budget, false);
    if (bytes > (size_t)LEOAM_STATIC_SCRATCH_BYTES) bytes = (size_t)LEOAM_STATIC_SCRATCH_BYTES;      // fewer splits
    // The buffer keeps what the last call on this GPU left, and that call may have had another shape
    // (its partials where this one's arrival counters lie): the counters are cleared here, by a fill
    // kernel (a memset node is not safe to record into a HIP graph on this platform).
    hipError_t e = workspace_zero_dispatch(ws, select_attention_counter_bytes(shape, false), (hipStream_t)stream);
    if (e != hipSuccess) return LEOAM_E_HIP;
    return from_hip(select_attention_dispatch(shape, score_ub, q, K, V, qmeta, chunk_off, n_chunks, max_chunks,
                                              token_budget, softmax_scale, sel_idx, sel_count, sel_tokens, out, lse, ws,
                                              bytes, (hipStream_t)stream, false));
}

size_t leoam_fused_workspace_bytes(const leoam_shape* shape, int32_t max_tokens) {
    if (check_shape(shape)) return 0;
    return select_attention_workspace_bytes(shape, max_tokens);
}

size_t leoam_fused_control_bytes(const leoam_shape* shape) {
    if (check_shape(shape)) return 0;
    return select_attention_counter_bytes(shape);
}

int leoam_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
    if (!workspace || (workspace_bytes & 15u) || ((uintptr_t)workspace & 15u)) return LEOAM_E_INVALID_ARG;
    return from_hip(workspace_zero_dispatch(workspace, workspace_bytes, (hipStream_t)stream));
}

size_t leoam_workspace_bytes(const leoam_shape* shape, int32_t max_tokens) {
    if (check_shape(shape)) return 0;
    return attention_workspace_bytes(shape, max_tokens);
}

int leoam_validate_boundaries(const leoam_shape* shape, const int32_t* chunk_off, const int32_t* n_chunks,
                              void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!chunk_off || !n_chunks) return LEOAM_E_INVALID_ARG;
    const size_t row = (size_t)shape->c_max + 1;
    std::vector<int32_t> off(row * shape->batch), nc(shape->batch);
    hipStream_t st = (hipStream_t)stream;
    if (hipMemcpyAsync(off.data(), chunk_off, off.size() * sizeof(int32_t), hipMemcpyDeviceToHost, st) != hipSuccess)
        return LEOAM_E_HIP;
    if (hipMemcpyAsync(nc.data(), n_chunks, nc.size() * sizeof(int32_t), hipMemcpyDeviceToHost, st) != hipSuccess)
        return LEOAM_E_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return LEOAM_E_HIP;
    for (int b = 0; b < shape->batch; ++b) {
        const int32_t* o = off.data() + row * b;
        const int n = nc[b];
        if (n < 1 || n > shape->c_max) return LEOAM_E_BAD_BOUNDARIES;
        if (o[0] != 0 || o[n] != shape->n_ctx) return LEOAM_E_BAD_BOUNDARIES;
        for (int c = 0; c < n; ++c)
            if (o[c + 1] <= o[c]) return LEOAM_E_BAD_BOUNDARIES;
    }
    return LEOAM_OK;
}

size_t leoam_compressed_bytes_bound(const leoam_shape* shape) {
    if (check_shape(shape)) return 0;
    return compressed_bytes_bound(shape);
}

int kv_chunk_compress(const leoam_shape* shape, const void* K, const void* V, const int32_t* chunk_off,
                      const int32_t* n_chunks, const uint8_t* four_bit, void* kblob, void* vblob, size_t blob_bytes,
                      void* qmeta, int64_t* total_bytes, void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!K || !V || !chunk_off || !n_chunks || !four_bit || !kblob || !vblob || !qmeta) return LEOAM_E_INVALID_ARG;
    if (shape->kv_dtype != LEOAM_F16 && shape->kv_dtype != LEOAM_BF16) return LEOAM_E_UNSUPPORTED;
    if (misaligned16(K, V, kblob, vblob, qmeta)) return LEOAM_E_INVALID_ARG;
    if (blob_bytes < compressed_bytes_bound(shape)) return LEOAM_E_WORKSPACE;
    return from_hip(compress_dispatch(shape, K, V, chunk_off, n_chunks, four_bit, kblob, vblob, qmeta, blob_bytes,
                                      (long long*)total_bytes, (hipStream_t)stream));
}

int kv_chunk_recompress(const leoam_shape* shape, const void* K, const void* V, const int32_t* chunk_off,
                        const int32_t* n_chunks, const uint8_t* four_bit_old, const uint8_t* four_bit_new, void* kblob,
                        void* vblob, size_t blob_bytes, void* qmeta, int64_t* used_bytes, int64_t* info, void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!K || !V || !chunk_off || !n_chunks || !four_bit_old || !four_bit_new || !kblob || !vblob || !qmeta ||
        !used_bytes || !info)
        return LEOAM_E_INVALID_ARG;
    if (shape->kv_dtype != LEOAM_F16 && shape->kv_dtype != LEOAM_BF16) return LEOAM_E_UNSUPPORTED;
    if (misaligned16(K, V, kblob, vblob, qmeta) || ((uintptr_t)used_bytes & 7u) || ((uintptr_t)info & 7u))
        return LEOAM_E_INVALID_ARG;
    return from_hip(recompress_dispatch(shape, K, V, chunk_off, n_chunks, four_bit_old, four_bit_new, kblob, vblob, qmeta,
                                        blob_bytes, (long long*)used_bytes, (long long*)info, (hipStream_t)stream));
}

int chunk_compression_tags(const leoam_shape* shape, const int32_t* n_chunks, const int32_t* sel_idx,
                           const int32_t* sel_count, uint8_t* four_bit, void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!n_chunks || !sel_idx || !sel_count || !four_bit) return LEOAM_E_INVALID_ARG;
    return from_hip(compression_tags_dispatch(shape, n_chunks, sel_idx, sel_count, four_bit, (hipStream_t)stream));
}

double leoam_compression_share(double n_bytes, double ratio, double bandwidth, double t_other, double t_compute,
                               double decompress_rate) {
    if (!(n_bytes > 0.0) || !(bandwidth > 0.0) || !(decompress_rate > 0.0) || !(ratio > 0.0) || ratio > 1.0 ||
        !(t_other >= 0.0) || !(t_compute >= 0.0))
        return -1.0;
    // transfer time beyond the computation with nothing compressed, and what a full share takes off it
    const double uncovered = t_other + n_bytes / bandwidth - t_compute;
    const double per_share = n_bytes * (1.0 - ratio) / bandwidth + n_bytes / decompress_rate;
    if (uncovered <= 0.0) return 0.0;
    return uncovered >= per_share ? 1.0 : uncovered / per_share;
}

int leoam_copy_probe(void* dst, const void* src, size_t bytes, void* stream) {
    if (!dst || !src || (bytes & 15u) || ((uintptr_t)dst & 15u) || ((uintptr_t)src & 15u)) return LEOAM_E_INVALID_ARG;
    if (bytes == 0) return LEOAM_OK;
    const size_t n16 = bytes / 16;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    hipLaunchKernelGGL(copy_probe_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, (uint4*)dst,
                       (const uint4*)src, n16);
    return from_hip(hipGetLastError());
}

int leoam_read_probe(const void* src, size_t bytes, void* sink, void* stream) {
    if (!src || !sink || (bytes & 15u) || ((uintptr_t)src & 15u) || ((uintptr_t)sink & 3u)) return LEOAM_E_INVALID_ARG;
    if (bytes == 0) return LEOAM_OK;
    const size_t n16 = bytes / 16;
    const size_t blocks = (n16 + kReadProbePiece - 1) / kReadProbePiece;
    if (blocks > 0x7fffffffu) return LEOAM_E_UNSUPPORTED;
    hipLaunchKernelGGL(read_probe_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, (const uint4*)src,
                       n16, (uint32_t*)sink);
    return from_hip(hipGetLastError());
}

const char* leoam_status_string(int status) {
    switch (status) {
    case LEOAM_OK: return "ok";
    case LEOAM_E_INVALID_ARG: return "invalid argument";
    case LEOAM_E_BAD_BOUNDARIES: return "chunk boundaries do not tile the context";
    case LEOAM_E_UNSUPPORTED: return "unsupported shape or dtype";
    case LEOAM_E_WORKSPACE: return "workspace missing, misaligned or too small";
    case LEOAM_E_HIP: return "HIP error";
    default: return "unknown status";
    }
}

int leoam_version(void) { return 100; }

}  // extern "C"
