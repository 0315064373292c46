// C ABI of the library: argument checks, host-side length bookkeeping, dispatch.
// Everything that can be refused is refused here, before any launch, so that the
// kernels may assume consistent shapes.  See include/videoscan.h for the contract.
#include <math.h>

#include <algorithm>
#include <vector>

#include <cstdio>
#include <cstdlib>
#include "vs_internal.h"

using namespace vs;

namespace vs {
int g_tune_prefill_splits = 0;
int g_tune_prefill_kv_groups = 0;
int g_tune_decode_chunk_rows = 0;
int g_tune_prefill_merge = 0;
}  // namespace vs

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

vs_status check_shape(const vs_shape* s) {
    if (!s) return VS_ERR_NULL;
    if (s->n_q_heads < 1 || s->n_kv_heads < 1 || s->head_dim < 1) return VS_ERR_SHAPE;
    if (s->n_q_heads % s->n_kv_heads != 0) return VS_ERR_SHAPE;
    if (!isfinite(s->softmax_scale) || !(s->softmax_scale > 0.f)) return VS_ERR_SHAPE;
    if (s->dtype != VS_F32 && s->dtype != VS_BF16) return VS_ERR_UNSUPPORTED;
    if (s->n_q_heads / s->n_kv_heads > kMaxGroup) return VS_ERR_UNSUPPORTED;
    if (s->n_q_heads > 4096) return VS_ERR_UNSUPPORTED;
    if (s->dtype == VS_F32 && s->head_dim != 64 && s->head_dim != 128) return VS_ERR_UNSUPPORTED;
    if (s->dtype == VS_BF16 && s->head_dim != 128) return VS_ERR_UNSUPPORTED;
    return VS_OK;
}

inline size_t elem_bytes(const vs_shape* s) { return s->dtype == VS_F32 ? 4 : 2; }
inline int64_t row_bytes(const vs_shape* s) {
    return (int64_t)s->n_kv_heads * s->head_dim * (int64_t)elem_bytes(s);
}

vs_status check_cache(const vs_cache* c, bool need_room) {
    if (!c) return VS_ERR_NULL;
    if (c->capacity < 0 || c->len < 0) return VS_ERR_SHAPE;
    if (c->len > c->capacity) return VS_ERR_CAPACITY;
    if ((c->len > 0 || need_room) && (!c->k || !c->v)) return VS_ERR_NULL;
    if (!aligned16(c->k) || !aligned16(c->v)) return VS_ERR_ALIGN;
    if (need_room && c->len == c->capacity) return VS_ERR_CAPACITY;
    return VS_OK;
}

// A launch is checked with hipGetLastError(), which also reports an error that some earlier
// call of this thread left behind (another library's probing, say).  Every entry point that
// launches starts by dropping such a leftover, so that what it reports is its own.
inline void forget_stale_hip_error() { (void)hipGetLastError(); }

// Has a workgroup of an earlier bf16 prefill launch on the current device found itself on an
// XCD other than the one its unit's merge relies on?  (Reported once; see videoscan.h.)
inline bool placement_fault_reported() {
    int dev = 0;
    return hipGetDevice(&dev) == hipSuccess && prefill_placement_fault(dev);
}

constexpr int32_t kMaxTokens = 4096;
constexpr int32_t kMaxStreams = 1024;

size_t round256(size_t x) { return (x + 255) & ~size_t(255); }

// append: the run's last row goes to the cache (a frame and its carrier); append_all: every row
// of the run does (a question, whose tokens all stay for the answer)
vs_status prefill_common(const vs_shape* shape, vs_cache* cache, bool append, const void* q,
                         const void* k_f, const void* v_f, int32_t n_tokens, void* out,
                         int32_t* row_written, void* workspace, size_t workspace_bytes,
                         void* hip_stream, bool append_all = false) {
    forget_stale_hip_error();
    vs_status st = check_shape(shape);
    if (st != VS_OK) return st;
    st = check_cache(cache, append);
    if (st != VS_OK) return st;
    if (!q || !k_f || !v_f || !out) return VS_ERR_NULL;
    if (n_tokens < 1 || n_tokens > kMaxTokens) return VS_ERR_SHAPE;
    const int32_t n_kept = append ? (append_all ? n_tokens : 1) : 0;
    if (cache->len > cache->capacity - n_kept) return VS_ERR_CAPACITY;
    if (!aligned16(q) || !aligned16(k_f) || !aligned16(v_f) || !aligned16(out)) return VS_ERR_ALIGN;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int64_t rb = row_bytes(shape);
    char* kdst = append ? static_cast<char*>(cache->k) + (int64_t)cache->len * rb : nullptr;
    char* vdst = append ? static_cast<char*>(cache->v) + (int64_t)cache->len * rb : nullptr;
    hipError_t e;
    if (shape->dtype == VS_BF16) {
        const size_t ctrl = control_block_bytes(*shape);
        const size_t need = ctrl + prefill_mfma_workspace_bytes(*shape, n_tokens);
        if (!workspace || workspace_bytes < need) return VS_ERR_WORKSPACE;
        if (!aligned16(workspace)) return VS_ERR_ALIGN;
        if (placement_fault_reported()) return VS_ERR_PLACEMENT;
        char* wsb = static_cast<char*>(workspace);
        e = launch_prefill_mfma(*shape, cache->k, cache->v, cache->len, q, k_f, v_f, n_tokens, out,
                                kdst, vdst, wsb + prefill_counter_offset(*shape), wsb + ctrl, stream, 1, append_all);
    } else {
        e = launch_prefill_simple(*shape, cache->k, cache->v, cache->len, q, k_f, v_f, n_tokens, out,
                                  stream);
        if (e == hipSuccess && append) {
            // (the kept rows are contiguous in the run and in the cache: one block of n_kept rows,
            // handed to the row copy as a single long row at the destination itself)
            LenTable t{};
            e = launch_append_rows(1, kdst, vdst, 0, &t, nullptr, k_f, v_f, 0,
                                   (int64_t)(n_tokens - n_kept) * rb, (int32_t)(n_kept * rb), stream);
        }
    }
    if (e != hipSuccess) return VS_ERR_HIP;
    if (append) {
        if (row_written) *row_written = cache->len;
        cache->len += n_kept;
    }
    return VS_OK;
}

}  // namespace

// vs_decode_attn, and the entry point that brings its own scratch memory.
vs_status vs::decode_entry(const vs_shape* shape, int32_t n_streams, void* k_slab, void* v_slab,
                           int32_t capacity, int32_t* lens, const void* q, const void* k_new,
                           const void* v_new, void* out, void* workspace, size_t workspace_bytes,
                           void* hip_stream) {
    forget_stale_hip_error();
    vs_status st = check_shape(shape);
    if (st != VS_OK) return st;
    if (!k_slab || !v_slab || !lens || !q || !out) return VS_ERR_NULL;
    if ((k_new == nullptr) != (v_new == nullptr)) return VS_ERR_NULL;
    if (n_streams < 1 || n_streams > kMaxStreams || capacity < 1) return VS_ERR_SHAPE;
    if (!aligned16(k_slab) || !aligned16(v_slab) || !aligned16(q) || !aligned16(out) ||
        !aligned16(k_new) || !aligned16(v_new))
        return VS_ERR_ALIGN;
    const int add = k_new ? 1 : 0;
    int32_t max_rows = 0;
    for (int32_t s = 0; s < n_streams; ++s) {
        if (lens[s] < 0) return VS_ERR_SHAPE;
        if (lens[s] > capacity || lens[s] + add > capacity) return VS_ERR_CAPACITY;
        if (lens[s] + add < 1) return VS_ERR_SHAPE;
        if (lens[s] + add > max_rows) max_rows = lens[s] + add;
    }
    const bool mfma = shape->dtype == VS_BF16;
    const size_t ctrl = control_block_bytes(*shape);
    if (mfma) {
        const int chunk = n_streams < kMaxStreamsPerLaunch ? n_streams : kMaxStreamsPerLaunch;
        if (!workspace || workspace_bytes < ctrl + decode_mfma_workspace_bytes(*shape, chunk, max_rows))
            return VS_ERR_WORKSPACE;
        if (!aligned16(workspace)) return VS_ERR_ALIGN;
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int64_t rb = row_bytes(shape);
    const int64_t qo_stride = (int64_t)shape->n_q_heads * shape->head_dim * (int64_t)elem_bytes(shape);
    for (int32_t s0 = 0; s0 < n_streams; s0 += kMaxStreamsPerLaunch) {
        const int32_t ns = (n_streams - s0) < kMaxStreamsPerLaunch ? (n_streams - s0) : kMaxStreamsPerLaunch;
        char* ks = static_cast<char*>(k_slab) + (int64_t)s0 * capacity * rb;
        char* vs_ = static_cast<char*>(v_slab) + (int64_t)s0 * capacity * rb;
        const char* kn = add ? static_cast<const char*>(k_new) + (int64_t)s0 * rb : nullptr;
        const char* vn = add ? static_cast<const char*>(v_new) + (int64_t)s0 * rb : nullptr;
        const char* qs = static_cast<const char*>(q) + (int64_t)s0 * qo_stride;
        char* os = static_cast<char*>(out) + (int64_t)s0 * qo_stride;
        LenTable t{};
        hipError_t e = hipSuccess;
        if (mfma) {
            // the kernel reads the new row from k_new/v_new and stores it into the slab itself
            for (int32_t i = 0; i < ns; ++i) t.v[i] = lens[s0 + i] + add;
            e = launch_decode_mfma(*shape, ns, ks, vs_, capacity, t, qs, kn, vn, os, workspace,
                                   static_cast<char*>(workspace) + ctrl, stream);
        } else {
            if (add) {
                for (int32_t i = 0; i < ns; ++i) t.v[i] = lens[s0 + i];
                e = launch_append_rows(ns, ks, vs_, (int64_t)capacity * rb, &t, nullptr, kn, vn, rb, 0,
                                       (int32_t)rb, stream);
                if (e != hipSuccess) return VS_ERR_HIP;  // (a row copy that did not start leaves nothing behind)
            }
            for (int32_t i = 0; i < ns; ++i) t.v[i] = lens[s0 + i] + add;
            e = launch_decode_simple(*shape, ns, ks, vs_, capacity, t, qs, os, stream);
        }
        if (e != hipSuccess) return VS_ERR_HIP;
        // the lengths follow the launches group by group: after a failure in a later group, lens
        // still says exactly which rows have been written
        if (add)
            for (int32_t i = 0; i < ns; ++i) lens[s0 + i] += 1;
    }
    return VS_OK;
}

extern "C" {

const char* vs_status_string(vs_status s) {
    switch (s) {
        case VS_OK: return "ok";
        case VS_ERR_NULL: return "required pointer is NULL";
        case VS_ERR_SHAPE: return "sizes out of range or inconsistent";
        case VS_ERR_UNSUPPORTED: return "head_dim / dtype / head ratio not supported";
        case VS_ERR_CAPACITY: return "cache full or len > capacity";
        case VS_ERR_WORKSPACE: return "workspace missing or too small";
        case VS_ERR_ALIGN: return "device pointer not 16-byte aligned";
        case VS_ERR_HIP: return "HIP launch failure";
        case VS_ERR_PLACEMENT: return "an earlier prefill launch was not placed on the XCDs as probed";
    }
    return "unknown status";
}

size_t vs_workspace_bytes(const vs_shape* shape, int32_t max_q_tokens, int32_t max_cache_rows,
                          int32_t n_streams) {
    if (check_shape(shape) != VS_OK) return 0;
    if (max_q_tokens < 0 || max_cache_rows < 0 || n_streams < 0) return 0;
    if (max_q_tokens > kMaxTokens || n_streams > (1 << 20)) return 0;
    size_t need = 256;
    if (shape->dtype == VS_BF16) {
        if (max_q_tokens > 0) need = std::max(need, prefill_mfma_workspace_bytes(*shape, max_q_tokens));
        if (n_streams > 0) {
            const int chunk = n_streams < kMaxStreamsPerLaunch ? n_streams : kMaxStreamsPerLaunch;
            need = std::max(need, decode_mfma_workspace_bytes(*shape, chunk, max_cache_rows));
        }
    }
    // batched compaction of more than 64 caches stages the lengths in the scratch area
    need = std::max(need, sizeof(int32_t) * (size_t)n_streams);
    return control_block_bytes(*shape) + round256(need);
}

vs_status vs_workspace_init(const vs_shape* shape, void* workspace, size_t workspace_bytes,
                            void* hip_stream) {
    forget_stale_hip_error();
    vs_status st = check_shape(shape);
    if (st != VS_OK) return st;
    if (!workspace) return VS_ERR_NULL;
    if (!aligned16(workspace)) return VS_ERR_ALIGN;
    if (workspace_bytes < control_block_bytes(*shape)) return VS_ERR_WORKSPACE;
    // the first call on a device also finds out how that device deals workgroups to its XCDs
    // (one tiny launch into the control block and a wait for it)
    hipError_t e = probe_xcd_mapping(workspace, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) {
        if (getenv("VS_DEBUG")) fprintf(stderr, "vs_workspace_init: probe: %s\n", hipGetErrorString(e));
        return VS_ERR_HIP;
    }
    e = launch_zero_fill(workspace, control_block_bytes(*shape), static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess && getenv("VS_DEBUG")) fprintf(stderr, "vs_workspace_init: fill: %s\n", hipGetErrorString(e));
    return e == hipSuccess ? VS_OK : VS_ERR_HIP;
}

vs_status vs_frame_prefill_attn(const vs_shape* shape, const vs_cache* cache, const void* q,
                                const void* k_f, const void* v_f, int32_t n_tokens, void* out,
                                void* workspace, size_t workspace_bytes, void* hip_stream) {
    return prefill_common(shape, const_cast<vs_cache*>(cache), false, q, k_f, v_f, n_tokens, out,
                          nullptr, workspace, workspace_bytes, hip_stream);
}

vs_status vs_frame_prefill_compact(const vs_shape* shape, vs_cache* cache, const void* q,
                                   const void* k_f, const void* v_f, int32_t n_tokens, void* out,
                                   int32_t* row_written, void* workspace, size_t workspace_bytes,
                                   void* hip_stream) {
    return prefill_common(shape, cache, true, q, k_f, v_f, n_tokens, out, row_written, workspace,
                          workspace_bytes, hip_stream);
}

vs_status vs_question_prefill_append(const vs_shape* shape, vs_cache* cache, const void* q,
                                     const void* k_t, const void* v_t, int32_t n_tokens, void* out,
                                     void* workspace, size_t workspace_bytes, void* hip_stream) {
    return prefill_common(shape, cache, true, q, k_t, v_t, n_tokens, out, nullptr, workspace,
                          workspace_bytes, hip_stream, true);
}

vs_status vs_carrier_compact_append(const vs_shape* shape, vs_cache* cache, const void* k_f,
                                    const void* v_f, int32_t n_tokens, int32_t carrier_index,
                                    int32_t* row_written, void* hip_stream) {
    forget_stale_hip_error();
    vs_status st = check_shape(shape);
    if (st != VS_OK) return st;
    if (!k_f || !v_f) return VS_ERR_NULL;
    if (n_tokens < 1 || carrier_index < 0 || carrier_index >= n_tokens) return VS_ERR_SHAPE;
    st = check_cache(cache, true);
    if (st != VS_OK) return st;
    if (!aligned16(k_f) || !aligned16(v_f)) return VS_ERR_ALIGN;
    const int64_t rb = row_bytes(shape);
    LenTable t{};
    t.v[0] = cache->len;
    hipError_t e = launch_append_rows(1, cache->k, cache->v, 0, &t, nullptr, k_f, v_f, 0,
                                      (int64_t)carrier_index * rb, (int32_t)rb,
                                      static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return VS_ERR_HIP;
    if (row_written) *row_written = cache->len;
    cache->len += 1;
    return VS_OK;
}

vs_status vs_carrier_compact_append_batched(const vs_shape* shape, int32_t n_caches, void* k_slab,
                                            void* v_slab, int32_t capacity, int32_t* lens,
                                            const void* k_f, const void* v_f, int32_t n_tokens,
                                            int32_t carrier_index, int32_t* rows_written,
                                            void* workspace, size_t workspace_bytes,
                                            void* hip_stream) {
    forget_stale_hip_error();
    vs_status st = check_shape(shape);
    if (st != VS_OK) return st;
    if (!k_slab || !v_slab || !lens || !k_f || !v_f) return VS_ERR_NULL;
    if (n_caches < 1 || n_caches > (1 << 20) || capacity < 1) return VS_ERR_SHAPE;
    if (n_tokens < 1 || carrier_index < 0 || carrier_index >= n_tokens) return VS_ERR_SHAPE;
    if (!aligned16(k_slab) || !aligned16(v_slab) || !aligned16(k_f) || !aligned16(v_f)) return VS_ERR_ALIGN;
    for (int32_t i = 0; i < n_caches; ++i) {
        if (lens[i] < 0) return VS_ERR_SHAPE;
        if (lens[i] >= capacity) return VS_ERR_CAPACITY;
    }
    const int64_t rb = row_bytes(shape);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipError_t e;
    if (n_caches <= kMaxStreamsPerLaunch) {
        LenTable t{};
        for (int32_t i = 0; i < n_caches; ++i) t.v[i] = lens[i];
        e = launch_append_rows(n_caches, k_slab, v_slab, (int64_t)capacity * rb, &t, nullptr, k_f, v_f,
                               (int64_t)n_tokens * rb, (int64_t)carrier_index * rb, (int32_t)rb, stream);
    } else {
        // The device needs the lengths as they are now, and lens is incremented below.  The
        // kernel takes them from rows_written when the caller gives one (filled here with the old
        // lengths and not touched again), else from lens.  Pinned host memory is read by the
        // kernel in place, 32 bytes per batch of rows, next to the rows' own loads; if that
        // memory is lens itself, the stream is waited for before lens changes.  Pageable memory
        // is staged in the workspace: the runtime has taken its copy when hipMemcpyAsync returns.
        const int32_t* from = rows_written ? rows_written : lens;
        const int32_t* on_device = nullptr;
        hipPointerAttribute_t attr;
        if (hipPointerGetAttributes(&attr, from) == hipSuccess) {
            if (attr.type == hipMemoryTypeHost && attr.devicePointer)
                on_device = static_cast<const int32_t*>(attr.devicePointer);
        } else {
            (void)hipGetLastError();  // ordinary pageable memory is unknown to the runtime
        }
        bool wait = on_device && from == lens;
        void* staged = nullptr;
        if (!on_device) {
            const size_t ctrl = control_block_bytes(*shape);
            if (!workspace || workspace_bytes < ctrl + sizeof(int32_t) * (size_t)n_caches) return VS_ERR_WORKSPACE;
            if (!aligned16(workspace)) return VS_ERR_ALIGN;
            staged = static_cast<char*>(workspace) + ctrl;
            if (!rows_written && hipPointerGetAttributes(&attr, lens) == hipSuccess) wait = attr.type != hipMemoryTypeUnregistered;
            else (void)hipGetLastError();
        }
        if (rows_written)
            for (int32_t i = 0; i < n_caches; ++i) rows_written[i] = lens[i];
        e = hipSuccess;
        if (staged) {
            e = hipMemcpyAsync(staged, from, sizeof(int32_t) * (size_t)n_caches, hipMemcpyHostToDevice, stream);
            on_device = static_cast<const int32_t*>(staged);
        }
        if (e == hipSuccess)
            e = launch_append_rows(n_caches, k_slab, v_slab, (int64_t)capacity * rb, nullptr, on_device, k_f, v_f,
                                   (int64_t)n_tokens * rb, (int64_t)carrier_index * rb, (int32_t)rb, stream);
        if (e == hipSuccess && wait) e = hipStreamSynchronize(stream);
    }
    if (e != hipSuccess) return VS_ERR_HIP;
    if (rows_written && n_caches <= kMaxStreamsPerLaunch)
        for (int32_t i = 0; i < n_caches; ++i) rows_written[i] = lens[i];
    for (int32_t i = 0; i < n_caches; ++i) lens[i] += 1;
    return VS_OK;
}

vs_status vs_decode_attn(const vs_shape* shape, int32_t n_streams, void* k_slab, void* v_slab,
                         int32_t capacity, int32_t* lens, const void* q, const void* k_new,
                         const void* v_new, void* out, void* workspace, size_t workspace_bytes,
                         void* hip_stream) {
    return vs::decode_entry(shape, n_streams, k_slab, v_slab, capacity, lens, q, k_new, v_new, out, workspace,
                            workspace_bytes, hip_stream);
}

size_t vs_frames_workspace_bytes(const vs_shape* shape, int32_t n_frames, int32_t n_tokens,
                                 int32_t max_cache_rows) {
    if (check_shape(shape) != VS_OK || shape->dtype != VS_BF16) return 0;
    if (n_frames < 1 || n_frames > 64 || n_tokens < 1 || (int64_t)n_frames * n_tokens > kMaxTokens ||
        max_cache_rows < 0)
        return 0;
    // the plan's number of splits grows with the rows: size for the longest cache
    int ns = prefill_frames_splits(*shape, n_frames, n_tokens, max_cache_rows);
    // (short caches run one key group per workgroup and may take a split or two more)
    for (int tiles = 1; tiles <= 7; ++tiles) {
        const int len = tiles * 64 - n_tokens - (n_frames - 1);
        if (len >= 0 && len <= max_cache_rows) ns = std::max(ns, prefill_frames_splits(*shape, n_frames, n_tokens, len));
    }
    size_t need = prefill_frames_workspace_bytes(*shape, n_frames, n_tokens, ns);
    if (n_frames == 1) need = std::max(need, prefill_mfma_workspace_bytes(*shape, n_tokens));
    return control_block_bytes(*shape) + round256(need);
}

vs_status vs_frames_prefill_attn(const vs_shape* shape, vs_cache* cache, const void* q, const void* k_f,
                                 const void* v_f, int32_t n_frames, int32_t n_tokens, void* out,
                                 void* workspace, size_t workspace_bytes, void* hip_stream) {
    forget_stale_hip_error();
    vs_status st = check_shape(shape);
    if (st != VS_OK) return st;
    if (shape->dtype != VS_BF16) return VS_ERR_UNSUPPORTED;
    st = check_cache(cache, true);
    if (st != VS_OK) return st;
    if (!q || !k_f || !v_f || !out) return VS_ERR_NULL;
    if (n_frames < 1 || n_frames > 64 || n_tokens < 1 || (int64_t)n_frames * n_tokens > kMaxTokens) return VS_ERR_SHAPE;
    if ((int64_t)cache->len + n_frames > cache->capacity) return VS_ERR_CAPACITY;
    if (!aligned16(q) || !aligned16(k_f) || !aligned16(v_f) || !aligned16(out)) return VS_ERR_ALIGN;
    const size_t ctrl = control_block_bytes(*shape);
    const int ns = prefill_frames_splits(*shape, n_frames, n_tokens, cache->len);
    const size_t need = ctrl + prefill_frames_workspace_bytes(*shape, n_frames, n_tokens, ns);
    if (!workspace || workspace_bytes < need) return VS_ERR_WORKSPACE;
    if (!aligned16(workspace)) return VS_ERR_ALIGN;
    if (placement_fault_reported()) return VS_ERR_PLACEMENT;
    const int64_t rb = row_bytes(shape);
    char* wsb = static_cast<char*>(workspace);
    char* kdst = static_cast<char*>(cache->k) + (int64_t)cache->len * rb;
    char* vdst = static_cast<char*>(cache->v) + (int64_t)cache->len * rb;
    if (launch_prefill_mfma(*shape, cache->k, cache->v, cache->len, q, k_f, v_f, n_tokens, out, kdst, vdst,
                            wsb + prefill_counter_offset(*shape), wsb + ctrl, static_cast<hipStream_t>(hip_stream),
                            n_frames) != hipSuccess)
        return VS_ERR_HIP;
    cache->len += n_frames;
    return VS_OK;
}

size_t vs_memory_bank_workspace_bytes(int32_t capacity) {
    if (capacity < 1 || capacity > 1024) return 0;
    return round256(sizeof(double) * (size_t)capacity);
}

vs_status vs_memory_bank_push(vs_bank* bank, const void* e_new, int32_t policy, int32_t* victim,
                              void* workspace, size_t workspace_bytes, void* hip_stream) {
    forget_stale_hip_error();
    if (!bank || !e_new || !victim || !bank->e) return VS_ERR_NULL;
    if (bank->dtype != VS_F32 && bank->dtype != VS_BF16) return VS_ERR_UNSUPPORTED;
    const int64_t rb = (int64_t)bank->d * (bank->dtype == VS_F32 ? 4 : 2);
    if (bank->capacity < 1 || bank->capacity > 1024 || bank->len < 0 || bank->len > bank->capacity ||
        bank->d < 1 || rb % 16 != 0 || (policy != 0 && policy != 1))
        return VS_ERR_SHAPE;
    if (!aligned16(bank->e) || !aligned16(e_new) || (reinterpret_cast<uintptr_t>(victim) & 3u)) return VS_ERR_ALIGN;
    if (!workspace || workspace_bytes < vs_memory_bank_workspace_bytes(bank->capacity)) return VS_ERR_WORKSPACE;
    if (!aligned16(workspace)) return VS_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    void* base = bank->e;
    const void* row = e_new;
    if (bank->len < bank->capacity) {
        if (launch_bank_shift(1, &base, &row, rb, 0, bank->capacity, bank->len, nullptr, victim, st) != hipSuccess)
            return VS_ERR_HIP;
        bank->len += 1;
        return VS_OK;
    }
    double* cosines = static_cast<double*>(workspace);
    if (launch_bank_cosines(bank->e, e_new, bank->capacity, bank->d, bank->dtype, policy, cosines, st) != hipSuccess)
        return VS_ERR_HIP;
    return launch_bank_shift(1, &base, &row, rb, 0, bank->capacity, -1, cosines, victim, st) == hipSuccess
               ? VS_OK : VS_ERR_HIP;
}

vs_status vs_carrier_evict_append(const vs_shape* shape, int32_t n_layers, vs_cache* caches, int32_t first_row,
                                  int32_t bank_capacity, const void* k_rows, const void* v_rows,
                                  int64_t layer_stride_bytes, const int32_t* victim, void* hip_stream) {
    forget_stale_hip_error();
    vs_status st = check_shape(shape);
    if (st != VS_OK) return st;
    if (!caches || !k_rows || !v_rows || !victim) return VS_ERR_NULL;
    const int64_t rb = row_bytes(shape);
    if (n_layers < 1 || n_layers > 1024 || first_row < 0 || bank_capacity < 1 || bank_capacity > 1024 ||
        layer_stride_bytes < 0 || layer_stride_bytes % 16 != 0 || (n_layers > 1 && layer_stride_bytes < rb))
        return VS_ERR_SHAPE;
    if (!aligned16(k_rows) || !aligned16(v_rows) || (reinterpret_cast<uintptr_t>(victim) & 3u)) return VS_ERR_ALIGN;
    const int32_t len = caches[0].len;
    for (int32_t l = 0; l < n_layers; ++l) {
        st = check_cache(&caches[l], false);
        if (st != VS_OK) return st;
        if (!caches[l].k || !caches[l].v) return VS_ERR_NULL;
        if (caches[l].len != len || len < first_row || len > first_row + bank_capacity) return VS_ERR_SHAPE;
        if ((int64_t)first_row + bank_capacity > caches[l].capacity) return VS_ERR_CAPACITY;
    }
    const bool room = len < first_row + bank_capacity;
    std::vector<void*> bases(2 * (size_t)n_layers);
    std::vector<const void*> rows(2 * (size_t)n_layers);
    for (int32_t l = 0; l < n_layers; ++l) {
        bases[2 * l] = caches[l].k;
        bases[2 * l + 1] = caches[l].v;
        rows[2 * l] = static_cast<const char*>(k_rows) + (int64_t)l * layer_stride_bytes;
        rows[2 * l + 1] = static_cast<const char*>(v_rows) + (int64_t)l * layer_stride_bytes;
    }
    if (launch_bank_shift(2 * n_layers, bases.data(), rows.data(), rb, first_row, bank_capacity,
                          room ? len - first_row : -1, nullptr, room ? nullptr : const_cast<int32_t*>(victim),
                          static_cast<hipStream_t>(hip_stream)) != hipSuccess)
        return VS_ERR_HIP;
    if (room)
        for (int32_t l = 0; l < n_layers; ++l) caches[l].len += 1;
    return VS_OK;
}

vs_status vs_set_tuning(int32_t knob, int32_t value) {
    if (value < 0) return VS_ERR_SHAPE;
    switch (knob) {
        case VS_TUNE_PREFILL_SPLITS:
            if (value > kMaxPrefillSplits) return VS_ERR_SHAPE;
            g_tune_prefill_splits = value;
            return VS_OK;
        case VS_TUNE_PREFILL_KV_GROUPS:
            if (value > 2) return VS_ERR_SHAPE;
            g_tune_prefill_kv_groups = value;
            return VS_OK;
        case VS_TUNE_DECODE_CHUNK_ROWS:
            if (value % 32 != 0) return VS_ERR_SHAPE;
            g_tune_decode_chunk_rows = value;
            return VS_OK;
        case VS_TUNE_PREFILL_MERGE:
            if (value > 4) return VS_ERR_SHAPE;
            g_tune_prefill_merge = value <= 2 ? value : 0;
            prefill_guard_test_mode(value >= 3 ? value : 0);
            return VS_OK;
        default: break;
    }
    return VS_ERR_SHAPE;
}

vs_status vs_carrier_mean_pool(const void* e, int32_t n, int32_t d, int32_t dtype, void* c_out,
                               void* hip_stream) {
    forget_stale_hip_error();
    if (!e || !c_out) return VS_ERR_NULL;
    if (dtype != VS_F32 && dtype != VS_BF16) return VS_ERR_UNSUPPORTED;
    if (n < 1 || d < 1) return VS_ERR_SHAPE;
    if (d % (dtype == VS_F32 ? 4 : 8) != 0) return VS_ERR_SHAPE;
    if (!aligned16(e) || !aligned16(c_out)) return VS_ERR_ALIGN;
    return launch_mean_pool(e, n, d, dtype, c_out, static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? VS_OK : VS_ERR_HIP;
}

vs_status vs_frame_qkv_project(const vs_shape* shape, const void* e, int32_t n_visual, int32_t d_model,
                               const void* w_qkv, void* q_out, void* k_out, void* v_out, void* c_out,
                               void* hip_stream) {
    forget_stale_hip_error();
    vs_status st = check_shape(shape);
    if (st != VS_OK) return st;
    if (shape->dtype != VS_BF16) return VS_ERR_UNSUPPORTED;
    if (!e || !w_qkv || !q_out || !k_out || !v_out) return VS_ERR_NULL;
    if (n_visual < 1 || n_visual > 191 || d_model < 64 || d_model % 64 != 0 || d_model > (1 << 20)) return VS_ERR_SHAPE;
    if (!aligned16(e) || !aligned16(w_qkv) || !aligned16(q_out) || !aligned16(k_out) || !aligned16(v_out) ||
        !aligned16(c_out))
        return VS_ERR_ALIGN;
    return launch_frame_qkv(*shape, e, n_visual, d_model, w_qkv, q_out, k_out, v_out, c_out,
                            static_cast<hipStream_t>(hip_stream)) == hipSuccess ? VS_OK : VS_ERR_HIP;
}

}  // extern "C"
