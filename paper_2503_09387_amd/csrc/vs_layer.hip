// C ABI of the dense layers and of the whole decoder layer around the attention (Section 4.1:
// the backbone; Sections 3.2, 3.3: a frame's tokens and its carrier pass through the layers once).
// Checks and dispatch only; the kernels are in vs_linear.hip and the attention files.
#include <math.h>

#include <algorithm>

#include "vs_internal.h"

using namespace vs;

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round256(size_t x) { return (x + 255) & ~size_t(255); }
constexpr int32_t kMaxRows = 192;

vs_status check_linear(const void* x, const void* w, int32_t n_rows, int32_t k, int32_t n, int32_t mode,
                       const void* residual, const void* out, const void* workspace, size_t workspace_bytes) {
    if (!x || !w || !out) return VS_ERR_NULL;
    if (mode != VS_LINEAR_STORE && mode != VS_LINEAR_RESIDUAL && mode != VS_LINEAR_GATED) return VS_ERR_SHAPE;
    if (mode == VS_LINEAR_RESIDUAL && !residual) return VS_ERR_NULL;
    if (n_rows < 1 || n_rows > kMaxRows || k < 64 || k % 64 != 0 || k > (1 << 20) || n < 2 || n % 2 != 0 || n > (1 << 24))
        return VS_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(w) || !aligned16(out) || !aligned16(residual) || !aligned16(workspace)) return VS_ERR_ALIGN;
    const size_t need = linear_workspace_bytes(n_rows, k, n);
    if (need > 0 && (!workspace || workspace_bytes < need)) return VS_ERR_WORKSPACE;
    return VS_OK;
}

struct LayerLayout {
    size_t attn, x, q, k, v, a, h1, act, lin, total;  // byte offsets of the parts of the layer's workspace
};

LayerLayout layer_layout(const vs_shape* s, const vs_layer_weights* wt, int32_t T) {
    LayerLayout l;
    const size_t e = 2, nq = (size_t)s->n_q_heads * s->head_dim, nk = (size_t)s->n_kv_heads * s->head_dim;
    size_t off = 0;
    l.attn = off; off += round256(vs_workspace_bytes(s, T, 0, 0));
    l.x = off;    off += round256((size_t)T * wt->d_model * e);
    l.q = off;    off += round256((size_t)T * nq * e);
    l.k = off;    off += round256((size_t)T * nk * e);
    l.v = off;    off += round256((size_t)T * nk * e);
    l.a = off;    off += round256((size_t)T * nq * e);
    l.h1 = off;   off += round256((size_t)T * wt->d_model * e);
    l.act = off;  off += round256((size_t)T * wt->d_ff * e);
    l.lin = off;
    size_t lin = linear_workspace_bytes(T, wt->d_model, (int32_t)(nq + 2 * nk));
    lin = std::max(lin, linear_workspace_bytes(T, (int32_t)nq, wt->d_model));
    lin = std::max(lin, linear_workspace_bytes(T, wt->d_model, 2 * wt->d_ff));
    lin = std::max(lin, linear_workspace_bytes(T, wt->d_ff, wt->d_model));
    off += round256(lin);
    l.total = off;
    return l;
}

vs_status check_layer(const vs_shape* s, const vs_layer_weights* wt, int32_t T) {
    if (!s || !wt) return VS_ERR_NULL;
    if (s->dtype != VS_BF16) return VS_ERR_UNSUPPORTED;
    if (vs_workspace_bytes(s, 1, 0, 0) == 0) return VS_ERR_UNSUPPORTED;  // (the attention's own shape rules)
    if (T < 1 || T > kMaxRows) return VS_ERR_SHAPE;
    if (wt->d_model < 64 || wt->d_model % 64 != 0 || wt->d_ff < 64 || wt->d_ff % 64 != 0 || wt->d_model > (1 << 20) ||
        wt->d_ff > (1 << 22) || ((int64_t)s->n_q_heads * s->head_dim) % 64 != 0)
        return VS_ERR_SHAPE;
    if (!isfinite(wt->eps) || wt->eps < 0.f) return VS_ERR_SHAPE;
    if (!wt->norm1 || !wt->w_qkv || !wt->w_o || !wt->norm2 || !wt->w_gate_up || !wt->w_down) return VS_ERR_NULL;
    if (!aligned16(wt->norm1) || !aligned16(wt->w_qkv) || !aligned16(wt->w_o) || !aligned16(wt->norm2) ||
        !aligned16(wt->w_gate_up) || !aligned16(wt->w_down))
        return VS_ERR_ALIGN;
    return VS_OK;
}

}  // namespace

extern "C" {

vs_status vs_rmsnorm(const void* x, const void* gamma, int32_t n_rows, int32_t d, float eps, void* out,
                     void* hip_stream) {
    (void)hipGetLastError();
    if (!x || !gamma || !out) return VS_ERR_NULL;
    if (n_rows < 1 || n_rows > (1 << 20) || d < 8 || d % 8 != 0 || d > (1 << 24) || !isfinite(eps) || eps < 0.f) return VS_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(gamma) || !aligned16(out)) return VS_ERR_ALIGN;
    return launch_rmsnorm(x, gamma, n_rows, d, eps, out, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? VS_OK
                                                                                                           : VS_ERR_HIP;
}

size_t vs_linear_workspace_bytes(int32_t n_rows, int32_t k, int32_t n) {
    if (n_rows < 1 || n_rows > kMaxRows || k < 64 || k % 64 != 0 || k > (1 << 20) || n < 2 || n % 2 != 0 || n > (1 << 24)) return 0;
    return linear_workspace_bytes(n_rows, k, n);
}

vs_status vs_linear(const void* x, const void* w, int32_t n_rows, int32_t k, int32_t n, int32_t mode,
                    const void* residual, void* out, void* workspace, size_t workspace_bytes, void* hip_stream) {
    (void)hipGetLastError();
    const vs_status st = check_linear(x, w, n_rows, k, n, mode, residual, out, workspace, workspace_bytes);
    if (st != VS_OK) return st;
    return launch_linear(x, k, w, n_rows, k, n, mode, residual, out, workspace, static_cast<hipStream_t>(hip_stream)) ==
                   hipSuccess ? VS_OK : VS_ERR_HIP;
}

size_t vs_layer_workspace_bytes(const vs_shape* shape, const vs_layer_weights* weights, int32_t n_tokens) {
    if (!shape || !weights || shape->dtype != VS_BF16 || vs_workspace_bytes(shape, 1, 0, 0) == 0) return 0;
    if (n_tokens < 1 || n_tokens > kMaxRows || weights->d_model < 64 || weights->d_model % 64 != 0 || weights->d_ff < 64 ||
        weights->d_ff % 64 != 0 || weights->d_model > (1 << 20) || weights->d_ff > (1 << 22))
        return 0;
    return layer_layout(shape, weights, n_tokens).total;
}

vs_status vs_frame_decoder_layer(const vs_shape* shape, const vs_layer_weights* wt, vs_cache* cache, const void* h_in,
                                 int32_t n_tokens, void* h_out, void* workspace, size_t workspace_bytes,
                                 void* hip_stream) {
    (void)hipGetLastError();
    vs_status st = check_layer(shape, wt, n_tokens);
    if (st != VS_OK) return st;
    if (!cache || !h_in || !h_out) return VS_ERR_NULL;
    if (!aligned16(h_in) || !aligned16(h_out)) return VS_ERR_ALIGN;
    if (cache->capacity < 0 || cache->len < 0) return VS_ERR_SHAPE;
    if (cache->len >= cache->capacity) return VS_ERR_CAPACITY;  // (before anything is launched)
    const LayerLayout l = layer_layout(shape, wt, n_tokens);
    if (!workspace || workspace_bytes < l.total) return VS_ERR_WORKSPACE;
    if (!aligned16(workspace)) return VS_ERR_ALIGN;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    char* ws = static_cast<char*>(workspace);
    const int32_t T = n_tokens, d = wt->d_model;
    // the arrival counters of the attention's control block also serve the split-K launches (every
    // kernel leaves them at zero)
    void* const counters = ws + l.attn + prefill_counter_offset(*shape);
    const int32_t n_counters = kMaxRowTiles * shape->n_kv_heads;
    const int32_t nq = shape->n_q_heads * shape->head_dim, nk = shape->n_kv_heads * shape->head_dim;
    // x1 = rmsnorm(h_in); [q k v] = x1 w_qkv^T
    if (launch_rmsnorm(h_in, wt->norm1, T, d, wt->eps, ws + l.x, stream) != hipSuccess) return VS_ERR_HIP;
    if (launch_linear(ws + l.x, d, wt->w_qkv, T, d, nq + 2 * nk, VS_LINEAR_STORE, nullptr, ws + l.q, ws + l.lin, stream,
                      ws + l.k, ws + l.v, nq, nq + nk, counters, n_counters) != hipSuccess)
        return VS_ERR_HIP;
    // the attention of the frame over what has been kept; the carrier's K/V row stays
    st = vs_frame_prefill_compact(shape, cache, ws + l.q, ws + l.k, ws + l.v, T, ws + l.a, nullptr, ws + l.attn,
                                  l.x - l.attn, hip_stream);
    if (st != VS_OK) return st;
    // h1 = h_in + a w_o^T; x2 = rmsnorm(h1); act = silu(x2 w_gate^T) * (x2 w_up^T); h_out = h1 + act w_down^T
    if (launch_linear(ws + l.a, nq, wt->w_o, T, nq, d, VS_LINEAR_RESIDUAL, h_in, ws + l.h1, ws + l.lin, stream, nullptr,
                      nullptr, 0, 0, counters, n_counters) != hipSuccess)
        return VS_ERR_HIP;
    if (launch_rmsnorm(ws + l.h1, wt->norm2, T, d, wt->eps, ws + l.x, stream) != hipSuccess) return VS_ERR_HIP;
    if (launch_linear(ws + l.x, d, wt->w_gate_up, T, d, 2 * wt->d_ff, VS_LINEAR_GATED, nullptr, ws + l.act, ws + l.lin,
                      stream) != hipSuccess)
        return VS_ERR_HIP;
    if (launch_linear(ws + l.act, wt->d_ff, wt->w_down, T, wt->d_ff, d, VS_LINEAR_RESIDUAL, ws + l.h1, h_out, ws + l.lin,
                      stream, nullptr, nullptr, 0, 0, counters, n_counters) != hipSuccess)
        return VS_ERR_HIP;
    return VS_OK;
}

}  // extern "C"
