// C ABI of libqvg: argument validation and the order in which kernels are enqueued.
// Compiled as HIP host code; holds no kernel and no arithmetic of the method.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "qvg.h"
#include "qvg_internal.hpp"

using namespace qvg;

namespace {

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round256(size_t v) { return (v + 255u) & ~(size_t)255u; }

int check_params(const qvg_params *p) {
    if (!p) return QVG_ERR_NULL;
    if (p->n_heads < 1 || p->n_heads > 65535) return QVG_ERR_BAD_PARAM;
    if (p->n_clusters < 1 || p->n_clusters > kMaxClusters) return QVG_ERR_BAD_PARAM;
    if (p->n_stages < 1 || p->n_stages > kMaxStages) return QVG_ERR_BAD_PARAM;
    if (p->kmeans_iters < 0) return QVG_ERR_BAD_PARAM;
    if (p->head_dim < 1 || p->n_smooth_stages < 1) return QVG_ERR_BAD_PARAM;
    if (p->group_size < 1 || p->head_dim % p->group_size != 0) return QVG_ERR_BAD_PARAM;
    if (p->bits != 2 && p->bits != 4) return QVG_ERR_BAD_PARAM;
    if (p->scale_format != QVG_SCALE_F16 && p->scale_format != QVG_SCALE_E4M3) return QVG_ERR_BAD_PARAM;
    // valid in the paper, not built here
    if (p->head_dim != kHeadDim) return QVG_ERR_UNSUPPORTED;
    if (p->n_smooth_stages > kMaxSmooth) return QVG_ERR_UNSUPPORTED;
    const int B = p->group_size;
    if (B != 16 && B != 32 && B != 64 && B != 128) return QVG_ERR_UNSUPPORTED;
    return QVG_OK;
}

// more than 256 centroids: an id is a 16-bit word (2-byte aligned arrays)
inline int id_wide(const qvg_params *p) { return p->n_clusters > 256 ? 1 : 0; }
inline bool ids_aligned(const qvg_params *p, const void *ids) {
    return !id_wide(p) || (reinterpret_cast<uintptr_t>(ids) & 1u) == 0;
}
inline int format_of(const qvg_params *p) {
    return (p->bits == 4 ? kFmtInt4 : 0) | (p->scale_format == QVG_SCALE_E4M3 ? kFmtE4M3 : 0);
}
// scale arrays: binary16 arrays follow the 16-byte rule, E4M3 bytes may start anywhere
inline bool scales_aligned(const qvg_params *p, const void *sc) {
    return p->scale_format == QVG_SCALE_E4M3 || aligned16(sc);
}

struct EncodeWs { size_t assign; size_t cent[2]; size_t perm; size_t offs; size_t resid[2]; size_t total; };

// with_assign: scratch of the assignment kernel; with_tables: two centroid tables for the Lloyd
// loop; with_update: permutation and offsets of the update step
EncodeWs encode_ws(const qvg_params *p, int64_t N, bool with_assign, bool with_tables, bool with_update = true) {
    EncodeWs w{};
    size_t o = 0;
    if (with_assign) { w.assign = o; o += assign_workspace_bytes(p->n_heads, p->n_clusters); }
    const size_t table = round256((size_t)p->n_heads * p->n_clusters * kHeadDim * sizeof(bf16_t));
    if (with_tables) { w.cent[0] = o; o += table; w.cent[1] = o; o += table; }
    if (with_update) {
        w.perm = o; o += round256((size_t)p->n_heads * (size_t)(N > 0 ? N : 1) * sizeof(int32_t));
        w.offs = o; o += round256((size_t)p->n_heads * (p->n_clusters + 1) * sizeof(int32_t));
    }
    // bf16 residual tensors that carry the data from one smoothing stage to the next
    if (with_assign && p->n_smooth_stages > 1) {
        const size_t r = round256((size_t)p->n_heads * (size_t)(N > 0 ? N : 1) * kHeadDim * sizeof(bf16_t));
        w.resid[0] = o; o += r;
        if (p->n_smooth_stages > 2) { w.resid[1] = o; o += r; }
    }
    w.total = o;
    return w;
}

int check_view(const void *base, int64_t stride_head, int64_t stride_token, int64_t N) {
    if (!aligned16(base)) return QVG_ERR_ALIGN;
    if (stride_token < kHeadDim || (stride_token & 7) || (stride_head & 7)) return QVG_ERR_ALIGN;
    if (stride_head < 0 || (N > 0 && stride_head < stride_token)) return QVG_ERR_BAD_PARAM;
    return QVG_OK;
}

}  // namespace

extern "C" {

int qvg_version(void) { return 100; }

const char *qvg_status_string(int status) {
    switch (status) {
        case QVG_OK: return "ok";
        case QVG_ERR_NULL: return "a required pointer is NULL";
        case QVG_ERR_BAD_PARAM: return "a size or parameter is out of range";
        case QVG_ERR_UNSUPPORTED: return "parameter combination not built (head_dim 128, up to 4 smoothing stages, group 16/32/64/128)";
        case QVG_ERR_WORKSPACE: return "workspace missing or too small";
        case QVG_ERR_ALIGN: return "pointer not 16-byte aligned or stride not a multiple of 8 elements";
        case QVG_ERR_LAUNCH: return "HIP runtime error while enqueuing";
        case QVG_ERR_SCRATCH_LIMIT: return "the call needs more scratch memory than the library's static buffer holds";
        default: return "unknown status";
    }
}

int qvg_workspace_bytes(const qvg_params *p, int which_entry, int64_t n_tokens, int64_t n_q,
                        size_t *out) {
    if (!out) return QVG_ERR_NULL;
    int st = check_params(p);
    if (st != QVG_OK) return st;
    if (n_tokens < 0 || n_q < 0) return QVG_ERR_BAD_PARAM;
    switch (which_entry) {
        case QVG_ENTRY_ENCODE:
            *out = n_tokens == 0 ? 0 : encode_ws(p, n_tokens, true, p->kmeans_iters > 0 || p->n_smooth_stages > 1,
                                                 p->kmeans_iters > 0).total;   // same call as qvg_encode_chunk
            return QVG_OK;
        case QVG_ENTRY_KMEANS_UPDATE:
            *out = encode_ws(p, n_tokens, false, false).total;
            return QVG_OK;
        case QVG_ENTRY_KMEANS_ASSIGN:
            *out = n_tokens == 0 ? 0 : encode_ws(p, n_tokens, true, false, false).total;
            return QVG_OK;
        case QVG_ENTRY_DECODE:
            *out = 0;
            return QVG_OK;
        case QVG_ENTRY_ATTN:
            // optional: the queries' running state + the decoded tiles of n_tokens tokens (whole
            // chunks, each counted as a multiple of 64 tokens)
            *out = attn_slab_state_bytes(p->n_heads, n_q) + attn_slab_chunk_bytes(p->n_heads, n_tokens);
            return QVG_OK;
        default:
            return QVG_ERR_BAD_PARAM;
    }
}

int64_t qvg_compressed_bytes(const qvg_params *p, int64_t n_tokens) {
    int st = check_params(p);
    if (st != QVG_OK) return st;
    if (n_tokens < 0) return QVG_ERR_BAD_PARAM;
    const int64_t d = p->head_dim, T = p->n_stages;
    const int64_t S = p->n_smooth_stages;
    const int64_t scale_bytes = p->scale_format == QVG_SCALE_E4M3 ? 1 : 2;
    const int64_t per_token = T * (d * p->bits / 8 + scale_bytes * (d / p->group_size)) + S * (id_wide(p) ? 2 : 1);
    return (int64_t)p->n_heads * (n_tokens * per_token + S * (int64_t)p->n_clusters * d * 2);
}

int qvg_kmeans_assign(const qvg_params *p, int64_t n_tokens, const void *x, int64_t stride_head,
                      int64_t stride_token, const void *centroids, uint8_t *ids_out, void *workspace,
                      size_t workspace_bytes, void *stream) {
    int st = check_params(p);
    if (st != QVG_OK) return st;
    if (n_tokens < 0 || n_tokens > kMaxTokensPerChunk) return QVG_ERR_BAD_PARAM;
    if (n_tokens == 0) return QVG_OK;
    if (!x || !centroids || !ids_out) return QVG_ERR_NULL;
    if ((st = check_view(x, stride_head, stride_token, n_tokens)) != QVG_OK) return st;
    if (!aligned16(centroids) || !ids_aligned(p, ids_out)) return QVG_ERR_ALIGN;
    const EncodeWs w = encode_ws(p, n_tokens, true, false, false);
    if (!workspace || workspace_bytes < w.total) return QVG_ERR_WORKSPACE;
    if (!aligned16(workspace)) return QVG_ERR_ALIGN;
    AssignArgs a{};
    assign_workspace_split(static_cast<unsigned char *>(workspace) + w.assign, p->n_heads, p->n_clusters, &a.nh3, &a.cmax);
    a.x = static_cast<const bf16_t *>(x); a.stride_head = stride_head; a.stride_token = stride_token;
    a.n_tokens = n_tokens; a.cent = static_cast<const bf16_t *>(centroids);
    a.H = p->n_heads; a.K = p->n_clusters; a.B = p->group_size; a.T = p->n_stages;
    a.ids = ids_out; a.codes = nullptr; a.scales = nullptr; a.out_stride = n_tokens; a.fused = 0;
    a.ids_step = 1; a.ids_off = 0; a.id_wide = id_wide(p);
    return launch_assign(a, static_cast<hipStream_t>(stream)) == hipSuccess ? QVG_OK : QVG_ERR_LAUNCH;
}

int qvg_kmeans_update(const qvg_params *p, int64_t n_tokens, const void *x, int64_t stride_head,
                      int64_t stride_token, const uint8_t *ids, const void *cent_prev,
                      void *cent_out, int32_t *counts_out, void *workspace, size_t workspace_bytes,
                      void *stream) {
    int st = check_params(p);
    if (st != QVG_OK) return st;
    if (n_tokens < 0 || n_tokens > kMaxTokensPerChunk) return QVG_ERR_BAD_PARAM;
    if (!cent_prev || !cent_out) return QVG_ERR_NULL;
    if (n_tokens > 0 && (!x || !ids)) return QVG_ERR_NULL;
    if (n_tokens > 0 && (st = check_view(x, stride_head, stride_token, n_tokens)) != QVG_OK) return st;
    if (!aligned16(cent_prev) || !aligned16(cent_out) || !ids_aligned(p, ids)) return QVG_ERR_ALIGN;
    const EncodeWs w = encode_ws(p, n_tokens, false, false);
    if (!workspace || workspace_bytes < w.total) return QVG_ERR_WORKSPACE;
    if (!aligned16(workspace)) return QVG_ERR_ALIGN;
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    UpdateArgs u{};
    u.x = static_cast<const bf16_t *>(x); u.stride_head = stride_head; u.stride_token = stride_token;
    u.n_tokens = n_tokens; u.ids = ids; u.ids_stride = n_tokens; u.ids_step = 1; u.ids_off = 0;
    u.id_wide = id_wide(p);
    u.cent_prev = static_cast<const bf16_t *>(cent_prev);
    u.cent_out = static_cast<bf16_t *>(cent_out); u.counts_out = counts_out;
    u.perm = reinterpret_cast<int32_t *>(ws + w.perm); u.offsets = reinterpret_cast<int32_t *>(ws + w.offs);
    u.H = p->n_heads; u.K = p->n_clusters;
    return launch_update(u, static_cast<hipStream_t>(stream)) == hipSuccess ? QVG_OK : QVG_ERR_LAUNCH;
}

int qvg_encode_chunk(const qvg_params *p, int64_t n_tokens, const void *x, int64_t stride_head,
                     int64_t stride_token, const void *init_centroids, void *centroids_out,
                     int64_t cent_out_stride_head, uint8_t *ids_out, uint8_t *codes_out,
                     void *scales_out, int64_t out_stride_head_tokens, void *workspace,
                     size_t workspace_bytes, void *stream) {
    int st = check_params(p);
    if (st != QVG_OK) return st;
    if (n_tokens < 0 || n_tokens > kMaxTokensPerChunk) return QVG_ERR_BAD_PARAM;
    if (!init_centroids || !centroids_out) return QVG_ERR_NULL;
    if (!aligned16(init_centroids) || !aligned16(centroids_out)) return QVG_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t row = (size_t)p->n_clusters * kHeadDim * sizeof(bf16_t);    // one unit's table
    if (cent_out_stride_head == 0) cent_out_stride_head = (int64_t)p->n_smooth_stages * p->n_clusters * kHeadDim;
    if (out_stride_head_tokens == 0) out_stride_head_tokens = n_tokens;
    if (cent_out_stride_head < (int64_t)p->n_smooth_stages * p->n_clusters * kHeadDim || (cent_out_stride_head & 7))
        return QVG_ERR_ALIGN;
    if (out_stride_head_tokens < n_tokens) return QVG_ERR_BAD_PARAM;
    // n_tokens == 0: the start tables go out unchanged, H rows of S*K*d bf16 with the caller's pitch
    auto copy_out = [&](const void *src) -> int {
        const size_t all = row * (size_t)p->n_smooth_stages;
        if (src == centroids_out && cent_out_stride_head == (int64_t)p->n_smooth_stages * p->n_clusters * kHeadDim) return QVG_OK;
        return hipMemcpy2DAsync(centroids_out, (size_t)cent_out_stride_head * sizeof(bf16_t), src, all, all,
                                (size_t)p->n_heads, hipMemcpyDeviceToDevice, s) == hipSuccess
                   ? QVG_OK : QVG_ERR_LAUNCH;
    };
    if (n_tokens == 0) return copy_out(init_centroids);
    if (!x || !ids_out || !codes_out || !scales_out) return QVG_ERR_NULL;
    if ((st = check_view(x, stride_head, stride_token, n_tokens)) != QVG_OK) return st;
    if (!aligned16(codes_out) || !scales_aligned(p, scales_out) || !ids_aligned(p, ids_out)) return QVG_ERR_ALIGN;
    const int I = p->kmeans_iters;
    const int fmt = format_of(p);
    const int S = p->n_smooth_stages;
    const EncodeWs w = encode_ws(p, n_tokens, true, I > 0 || S > 1, I > 0);
    if (!workspace || workspace_bytes < w.total) return QVG_ERR_WORKSPACE;
    if (!aligned16(workspace)) return QVG_ERR_ALIGN;
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    uint2 *nh3; float *cmax;
    assign_workspace_split(ws + w.assign, p->n_heads, p->n_clusters, &nh3, &cmax);
    // input of the current smoothing stage: the caller's view first, then dense residual tensors
    const bf16_t *xin = static_cast<const bf16_t *>(x);
    int64_t sh = stride_head, stt = stride_token;
    for (int stage = 0; stage < S; ++stage) {
        const bf16_t *cur = static_cast<const bf16_t *>(init_centroids) + (size_t)stage * p->n_clusters * kHeadDim;
        const int64_t init_stride = (int64_t)S * p->n_clusters * kHeadDim;     // init [H][S][K][d]
        AssignArgs a{};
        a.x = xin; a.stride_head = sh; a.stride_token = stt;
        a.n_tokens = n_tokens; a.H = p->n_heads; a.K = p->n_clusters; a.B = p->group_size;
        a.T = p->n_stages; a.ids = ids_out; a.out_stride = out_stride_head_tokens; a.fused = 0;
        a.ids_step = S; a.ids_off = stage; a.nh3 = nh3; a.cmax = cmax; a.id_wide = id_wide(p);
        bf16_t *buf[2] = {reinterpret_cast<bf16_t *>(ws + w.cent[0]), reinterpret_cast<bf16_t *>(ws + w.cent[1])};
        if (S > 1) {
            // the kernels want a dense [H][K][d] table; the caller's start tables are [H][S][K][d]
            if (hipMemcpy2DAsync(buf[1], row, cur, (size_t)init_stride * sizeof(bf16_t), row,
                                 (size_t)p->n_heads, hipMemcpyDeviceToDevice, s) != hipSuccess)
                return QVG_ERR_LAUNCH;
            cur = buf[1];
        }
        if (I > 0) {
            UpdateArgs u{};
            u.x = a.x; u.stride_head = sh; u.stride_token = stt; u.n_tokens = n_tokens;
            u.ids = ids_out; u.ids_stride = out_stride_head_tokens; u.ids_step = S; u.ids_off = stage;
            u.counts_out = nullptr; u.id_wide = id_wide(p);
            u.perm = reinterpret_cast<int32_t *>(ws + w.perm); u.offsets = reinterpret_cast<int32_t *>(ws + w.offs);
            u.H = p->n_heads; u.K = p->n_clusters;
            for (int it = 0; it < I; ++it) {
                a.cent = cur;
                if (launch_assign(a, s) != hipSuccess) return QVG_ERR_LAUNCH;
                u.cent_prev = cur; u.cent_out = buf[it & 1];
                if (launch_update(u, s) != hipSuccess) return QVG_ERR_LAUNCH;
                cur = buf[it & 1];
            }
        }
        // this stage's table goes out as H rows of K*d bf16 with the caller's pitch: the stage's
        // last assignment writes them while it stages the table (no copy of its own)
        bf16_t *cdst = static_cast<bf16_t *>(centroids_out) + (size_t)stage * p->n_clusters * kHeadDim;
        if (!(cur == cdst && cent_out_stride_head == (int64_t)p->n_clusters * kHeadDim)) {
            a.cent_copy = cdst; a.cent_copy_stride = cent_out_stride_head;
        }
        if (stage + 1 < S) {
            // final assignment of this stage, then the bf16 residual becomes the next input
            a.cent = cur;
            if (launch_assign(a, s) != hipSuccess) return QVG_ERR_LAUNCH;
            ResidualArgs r{};
            r.x = xin; r.stride_head = sh; r.stride_token = stt; r.n_tokens = n_tokens;
            r.cent = cur; r.ids = ids_out; r.ids_stride = out_stride_head_tokens; r.ids_step = S; r.ids_off = stage;
            r.out = reinterpret_cast<bf16_t *>(ws + w.resid[stage & 1]); r.H = p->n_heads; r.K = p->n_clusters;
            r.id_wide = id_wide(p);
            if (launch_residual(r, s) != hipSuccess) return QVG_ERR_LAUNCH;
            xin = r.out; sh = n_tokens * kHeadDim; stt = kHeadDim;
        } else if (fmt == 0) {
            a.cent = cur; a.codes = codes_out; a.scales = static_cast<f16_t *>(scales_out); a.fused = 1;
            if (launch_assign(a, s) != hipSuccess) return QVG_ERR_LAUNCH;
        } else {
            // the other stored formats: assignment, then the quantization kernel
            a.cent = cur;
            if (launch_assign(a, s) != hipSuccess) return QVG_ERR_LAUNCH;
            QuantArgs q{};
            q.x = xin; q.stride_head = sh; q.stride_token = stt; q.n_tokens = n_tokens; q.cent = cur;
            q.ids = ids_out; q.ids_step = S; q.ids_off = stage; q.codes = codes_out; q.scales = scales_out;
            q.out_stride = out_stride_head_tokens; q.H = p->n_heads; q.K = p->n_clusters; q.B = p->group_size;
            q.T = p->n_stages; q.fmt = fmt; q.id_wide = id_wide(p);
            if (launch_quantize(q, s) != hipSuccess) return QVG_ERR_LAUNCH;
        }
    }
    return QVG_OK;
}

}  // extern "C"

// ---- scratch memory owned by the library, for qvg_encode_chunk_static -------------------------
// One array per GPU the library's code object is loaded on (each device has its own copy at its
// own address), alive until the process ends.  The name below is only a handle on the host: the
// device address comes from hipGetSymbolAddress, once per device, and only that address is ever
// passed to a kernel or a copy.
static __device__ __align__(256) unsigned char scratch[QVG_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
// device address of `scratch` on the current device (looked up on the first call on that device)
int static_scratch_address(void **out) {
    static std::mutex mu;
    static void *address[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return QVG_ERR_LAUNCH;
    if (dev < 0 || dev >= kMaxDevices) return QVG_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(mu);
    if (!address[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return QVG_ERR_LAUNCH;
        address[dev] = ptr;
    }
    *out = address[dev];
    return QVG_OK;
}
}  // namespace

extern "C" {

int qvg_encode_chunk_static(const qvg_params *p, int64_t n_tokens, const void *x, int64_t stride_head,
                            int64_t stride_token, const void *init_centroids, void *centroids_out,
                            int64_t cent_out_stride_head, uint8_t *ids_out, uint8_t *codes_out,
                            void *scales_out, int64_t out_stride_head_tokens, void *stream) {
    int st = check_params(p);
    if (st != QVG_OK) return st;
    if (n_tokens < 0 || n_tokens > kMaxTokensPerChunk) return QVG_ERR_BAD_PARAM;
    // the same workspace layout as qvg_encode_chunk, placed in the static array
    const size_t need = n_tokens == 0 ? 0 : encode_ws(p, n_tokens, true, p->kmeans_iters > 0 || p->n_smooth_stages > 1,
                                                      p->kmeans_iters > 0).total;
    if (need > (size_t)QVG_STATIC_SCRATCH_BYTES) return QVG_ERR_SCRATCH_LIMIT;
    void *ws = nullptr;
    if (need > 0 && (st = static_scratch_address(&ws)) != QVG_OK) return st;
    // nothing in the workspace has to start at zero: every kernel writes what it later reads
    return qvg_encode_chunk(p, n_tokens, x, stride_head, stride_token, init_centroids, centroids_out,
                            cent_out_stride_head, ids_out, codes_out, scales_out, out_stride_head_tokens,
                            need > 0 ? ws : nullptr, need, stream);
}

int qvg_decode(const qvg_params *p, int64_t n_tokens, int64_t chunk_len, const void *centroids,
               const uint8_t *ids, const uint8_t *codes, const void *scales, void *x_out,
               int64_t stride_head, int64_t stride_token, void *stream) {
    return qvg_decode_ex(p, n_tokens, chunk_len, 0, 0, centroids, ids, codes, scales, x_out, stride_head,
                         stride_token, stream);
}

int qvg_decode_ex(const qvg_params *p, int64_t n_tokens, int64_t chunk_len, int64_t kv_capacity_tokens,
                  int64_t first_token, const void *centroids, const uint8_t *ids, const uint8_t *codes,
                  const void *scales, void *x_out, int64_t stride_head, int64_t stride_token,
                  void *stream) {
    int st = check_params(p);
    if (st != QVG_OK) return st;
    if (n_tokens < 0 || n_tokens > 0x7fffffff || chunk_len < 1) return QVG_ERR_BAD_PARAM;
    if (first_token < 0 || first_token % chunk_len != 0) return QVG_ERR_BAD_PARAM;
    if (kv_capacity_tokens == 0) kv_capacity_tokens = first_token + n_tokens;
    if (kv_capacity_tokens < first_token + n_tokens) return QVG_ERR_BAD_PARAM;
    const int64_t cap_chunks = (kv_capacity_tokens + chunk_len - 1) / chunk_len;
    if (cap_chunks > 0x7fffffff) return QVG_ERR_BAD_PARAM;
    if (n_tokens == 0) return QVG_OK;
    if (!centroids || !ids || !codes || !scales || !x_out) return QVG_ERR_NULL;
    if ((st = check_view(x_out, stride_head, stride_token, n_tokens)) != QVG_OK) return st;
    if (!aligned16(centroids) || !aligned16(codes) || !scales_aligned(p, scales) || !ids_aligned(p, ids)) return QVG_ERR_ALIGN;
    const int64_t n_chunks = (n_tokens + chunk_len - 1) / chunk_len;
    if (n_chunks > 0x7fffffff) return QVG_ERR_BAD_PARAM;
    DecodeArgs a{};
    // the range starts on a chunk boundary: move the unit-0 pointers to it, keep the unit strides
    const int64_t S_ = p->n_smooth_stages, T_ = p->n_stages, G_ = p->head_dim / p->group_size;
    a.cent = static_cast<const bf16_t *>(centroids) + (first_token / chunk_len) * S_ * p->n_clusters * kHeadDim;
    a.ids = ids + first_token * S_ * (id_wide(p) ? 2 : 1);
    a.id_wide = id_wide(p);
    a.codes = codes + first_token * T_ * (kHeadDim * p->bits / 8);
    a.scales = reinterpret_cast<const f16_t *>(static_cast<const uint8_t *>(scales) +
                                               first_token * T_ * G_ * (p->scale_format == QVG_SCALE_E4M3 ? 1 : 2));
    a.out = static_cast<bf16_t *>(x_out);
    a.kv_stride = kv_capacity_tokens; a.chunk_stride = (int)cap_chunks;
    a.n_tokens = n_tokens; a.chunk_len = chunk_len; a.n_chunks = (int)n_chunks;
    a.H = p->n_heads; a.K = p->n_clusters; a.B = p->group_size; a.T = p->n_stages;
    a.stride_head = stride_head; a.stride_token = stride_token; a.S = p->n_smooth_stages; a.fmt = format_of(p);
    return launch_decode(a, static_cast<hipStream_t>(stream)) == hipSuccess ? QVG_OK : QVG_ERR_LAUNCH;
}

int qvg_attn_decode(const qvg_params *p, int64_t n_q, const void *q, int64_t n_kv_tokens,
                    int64_t chunk_len, const void *k_centroids, const uint8_t *k_ids,
                    const uint8_t *k_codes, const void *k_scales, const void *v_centroids,
                    const uint8_t *v_ids, const uint8_t *v_codes, const void *v_scales,
                    float softmax_scale, void *out, float *lse_out, void *workspace,
                    size_t workspace_bytes, void *stream) {
    return qvg_attn_decode_ex(p, n_q, q, n_kv_tokens, chunk_len, 0, k_centroids, k_ids, k_codes, k_scales,
                              v_centroids, v_ids, v_codes, v_scales, nullptr, softmax_scale, out, lse_out,
                              workspace, workspace_bytes, stream);
}

int qvg_attn_merge(int64_t n_rows, int32_t head_dim, const void *out_a, const float *lse_a,
                   const void *out_b, const float *lse_b, void *out, float *lse_out, void *stream) {
    if (n_rows < 0) return QVG_ERR_BAD_PARAM;
    if (head_dim != kHeadDim) return QVG_ERR_UNSUPPORTED;
    if (n_rows == 0) return QVG_OK;
    if (!out_a || !lse_a || !out_b || !lse_b || !out) return QVG_ERR_NULL;
    if (!aligned16(out_a) || !aligned16(out_b) || !aligned16(out)) return QVG_ERR_ALIGN;
    MergeArgs m{};
    m.oa = static_cast<const bf16_t *>(out_a); m.lsea = lse_a; m.ob = static_cast<const bf16_t *>(out_b);
    m.lseb = lse_b; m.out = static_cast<bf16_t *>(out); m.lse = lse_out; m.rows = n_rows;
    return launch_attn_merge(m, static_cast<hipStream_t>(stream)) == hipSuccess ? QVG_OK : QVG_ERR_LAUNCH;
}

int qvg_attn_decode_ex(const qvg_params *p, int64_t n_q, const void *q, int64_t n_kv_tokens,
                       int64_t chunk_len, int64_t kv_capacity_tokens, const void *k_centroids,
                       const uint8_t *k_ids, const uint8_t *k_codes, const void *k_scales,
                       const void *v_centroids, const uint8_t *v_ids, const uint8_t *v_codes,
                       const void *v_scales, const void *k_rope, float softmax_scale, void *out,
                       float *lse_out, void *workspace, size_t workspace_bytes, void *stream) {
    return qvg_attn_decode_causal(p, n_q, q, n_kv_tokens, chunk_len, kv_capacity_tokens, k_centroids, k_ids, k_codes,
                                  k_scales, v_centroids, v_ids, v_codes, v_scales, k_rope, nullptr, softmax_scale, out,
                                  lse_out, workspace, workspace_bytes, stream);
}

}  // extern "C"

namespace {
// the one implementation behind every attention entry point; exactly one of out / out_f32 is set
int attn_call(const qvg_params *p, int64_t n_q, const void *q, int64_t n_kv_tokens,
              int64_t chunk_len, int64_t kv_capacity_tokens, const void *k_centroids,
              const uint8_t *k_ids, const uint8_t *k_codes, const void *k_scales,
              const void *v_centroids, const uint8_t *v_ids, const uint8_t *v_codes,
              const void *v_scales, const void *k_rope, const int32_t *q_kv_len,
              float softmax_scale, void *out, float *out_f32, float *lse_out, void *workspace,
              size_t workspace_bytes, void *stream) {
    int st = check_params(p);
    if (st != QVG_OK) return st;
    if (n_q < 0 || n_kv_tokens < 1 || n_kv_tokens > 0x7fffffff || chunk_len < 1) return QVG_ERR_BAD_PARAM;
    if (!(softmax_scale > 0.0f) || softmax_scale - softmax_scale != 0.0f) return QVG_ERR_BAD_PARAM;   // positive, finite
    if (n_q == 0) return QVG_OK;
    if (!q || (!out && !out_f32) || !k_centroids || !k_ids || !k_codes || !k_scales || !v_centroids || !v_ids ||
        !v_codes || !v_scales)
        return QVG_ERR_NULL;
    if (!aligned16(q) || !aligned16(out) || !aligned16(out_f32) || !aligned16(k_centroids) || !aligned16(v_centroids) ||
        !aligned16(k_codes) || !aligned16(v_codes) || !scales_aligned(p, k_scales) || !scales_aligned(p, v_scales))
        return QVG_ERR_ALIGN;
    const int64_t n_chunks = (n_kv_tokens + chunk_len - 1) / chunk_len;
    if (n_chunks > 0x7fffffff) return QVG_ERR_BAD_PARAM;
    if ((n_q + 127) / 128 > 0x7fffffff) return QVG_ERR_BAD_PARAM;
    if (kv_capacity_tokens == 0) kv_capacity_tokens = n_kv_tokens;
    if (kv_capacity_tokens < n_kv_tokens) return QVG_ERR_BAD_PARAM;
    const int64_t cap_chunks = (kv_capacity_tokens + chunk_len - 1) / chunk_len;
    if (cap_chunks > 0x7fffffff) return QVG_ERR_BAD_PARAM;
    if (k_rope && !aligned16(k_rope)) return QVG_ERR_ALIGN;
    AttnArgs a{};
    a.q = static_cast<const bf16_t *>(q); a.out = static_cast<bf16_t *>(out); a.out_f32 = out_f32; a.lse = lse_out;
    a.n_q = n_q; a.n_kv = n_kv_tokens; a.chunk_len = chunk_len; a.n_chunks = (int)n_chunks;
    a.H = p->n_heads; a.K = p->n_clusters; a.B = p->group_size; a.T = p->n_stages;
    a.scale = softmax_scale;
    a.k_cent = static_cast<const bf16_t *>(k_centroids); a.k_ids = k_ids; a.k_codes = k_codes;
    a.k_scales = static_cast<const f16_t *>(k_scales);
    a.v_cent = static_cast<const bf16_t *>(v_centroids); a.v_ids = v_ids; a.v_codes = v_codes;
    a.v_scales = static_cast<const f16_t *>(v_scales);
    a.S = p->n_smooth_stages; a.fmt = format_of(p);
    a.kv_stride = kv_capacity_tokens; a.chunk_stride = (int)cap_chunks;
    a.rope = static_cast<const f16_t *>(k_rope);
    a.id_wide = id_wide(p);
    if (!ids_aligned(p, k_ids) || !ids_aligned(p, v_ids)) return QVG_ERR_ALIGN;
    if (q_kv_len && (reinterpret_cast<uintptr_t>(q_kv_len) & 3u)) return QVG_ERR_ALIGN;
    a.q_len = q_kv_len;
    // a workspace that holds at least one chunk's decoded tiles switches to the shared-tile path
    if (workspace && attn_slab_applicable(a, workspace, workspace_bytes)) {
        if (!aligned16(workspace)) return QVG_ERR_ALIGN;
        return launch_attn_slab(a, workspace, workspace_bytes, static_cast<hipStream_t>(stream)) == hipSuccess
                   ? QVG_OK : QVG_ERR_LAUNCH;
    }
    return launch_attn(a, static_cast<hipStream_t>(stream)) == hipSuccess ? QVG_OK : QVG_ERR_LAUNCH;
}
}  // namespace

extern "C" {

int qvg_attn_decode_causal(const qvg_params *p, int64_t n_q, const void *q, int64_t n_kv_tokens,
                           int64_t chunk_len, int64_t kv_capacity_tokens, const void *k_centroids,
                           const uint8_t *k_ids, const uint8_t *k_codes, const void *k_scales,
                           const void *v_centroids, const uint8_t *v_ids, const uint8_t *v_codes,
                           const void *v_scales, const void *k_rope, const int32_t *q_kv_len,
                           float softmax_scale, void *out, float *lse_out, void *workspace,
                           size_t workspace_bytes, void *stream) {
    return attn_call(p, n_q, q, n_kv_tokens, chunk_len, kv_capacity_tokens, k_centroids, k_ids, k_codes, k_scales,
                     v_centroids, v_ids, v_codes, v_scales, k_rope, q_kv_len, softmax_scale, out, nullptr, lse_out,
                     workspace, workspace_bytes, stream);
}

int qvg_attn_decode_f32(const qvg_params *p, int64_t n_q, const void *q, int64_t n_kv_tokens,
                        int64_t chunk_len, int64_t kv_capacity_tokens, const void *k_centroids,
                        const uint8_t *k_ids, const uint8_t *k_codes, const void *k_scales,
                        const void *v_centroids, const uint8_t *v_ids, const uint8_t *v_codes,
                        const void *v_scales, const void *k_rope, const int32_t *q_kv_len,
                        float softmax_scale, float *out_f32, float *lse_out, void *stream) {
    return attn_call(p, n_q, q, n_kv_tokens, chunk_len, kv_capacity_tokens, k_centroids, k_ids, k_codes, k_scales,
                     v_centroids, v_ids, v_codes, v_scales, k_rope, q_kv_len, softmax_scale, nullptr, out_f32, lse_out,
                     nullptr, 0, stream);
}

}  // extern "C"
