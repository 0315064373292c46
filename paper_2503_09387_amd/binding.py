"""ctypes binding of libvideoscan.so.  Function names mirror the C ABI without the vs_
prefix.  Tensors are torch CUDA(ROCm) tensors; the current torch stream is used unless
one is given.  There is no fallback: if the library is missing, importing `lib()` raises."""
import ctypes
import os

VS_F32, VS_BF16 = 0, 1
_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

EXPORTS = [
    "vs_status_string", "vs_workspace_bytes", "vs_workspace_init", "vs_frame_prefill_attn", "vs_frame_prefill_compact",
    "vs_carrier_compact_append", "vs_carrier_compact_append_batched", "vs_decode_attn",
    "vs_carrier_mean_pool", "vs_set_tuning", "vs_memory_bank_push", "vs_carrier_evict_append",
    "vs_frames_prefill_attn", "vs_decode_attn_static", "vs_question_prefill_append", "vs_frame_qkv_project",
    "vs_rmsnorm", "vs_linear", "vs_frame_decoder_layer", "vs_linear_workspace_bytes", "vs_layer_workspace_bytes", "vs_memory_bank_workspace_bytes", "vs_frames_workspace_bytes",
    "vs_decode_static_scratch_bytes",
]


class VSError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"{what}: {status_string(code)} (vs_status {code})")
        self.code = code


class Shape(ctypes.Structure):
    _fields_ = [("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("softmax_scale", ctypes.c_float)]

    @classmethod
    def make(cls, n_q_heads, n_kv_heads, head_dim, dtype, softmax_scale=None):
        code = {"f32": VS_F32, "bf16": VS_BF16}.get(dtype, dtype)
        if softmax_scale is None:
            softmax_scale = float(head_dim) ** -0.5
        return cls(n_q_heads, n_kv_heads, head_dim, code, softmax_scale)


class _CCache(ctypes.Structure):
    _fields_ = [("k", ctypes.c_void_p), ("v", ctypes.c_void_p),
                ("capacity", ctypes.c_int32), ("len", ctypes.c_int32)]


class Cache:
    """Retained K/V rows of one layer of one stream: device tensors [capacity][Hkv][D] and a
    host-side length."""

    def __init__(self, k, v, length=0):
        assert k.shape == v.shape and k.is_contiguous() and v.is_contiguous()
        self.k, self.v = k, v
        self.c = _CCache(k.data_ptr(), v.data_ptr(), k.shape[0], int(length))

    @property
    def len(self):
        return self.c.len

    @len.setter
    def len(self, n):
        self.c.len = int(n)

    @property
    def capacity(self):
        return self.c.capacity


def lib_path():
    return os.path.join(_HERE, "libvideoscan.so")


def lib():
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
        # torch ships a HIP runtime of its own under the same soname as the one the library was
        # linked against; whichever is loaded first serves both.  torch's has to be the one: with
        # the system's loaded first, torch ends up on a mix of its own and the system's ROCm
        # libraries and finds no device.  So torch, when installed, is imported before the library.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = ctypes.CDLL(path)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        sp, cp, ip = ctypes.POINTER(Shape), ctypes.POINTER(_CCache), ctypes.POINTER(ctypes.c_int32)
        L.vs_status_string.restype = ctypes.c_char_p
        L.vs_status_string.argtypes = [ctypes.c_int]
        L.vs_workspace_bytes.restype = sz
        L.vs_workspace_bytes.argtypes = [sp, i32, i32, i32]
        L.vs_workspace_init.argtypes = [sp, vp, sz, vp]
        L.vs_frame_prefill_attn.argtypes = [sp, cp, vp, vp, vp, i32, vp, vp, sz, vp]
        L.vs_frame_prefill_compact.argtypes = [sp, cp, vp, vp, vp, i32, vp, ip, vp, sz, vp]
        L.vs_question_prefill_append.argtypes = [sp, cp, vp, vp, vp, i32, vp, vp, sz, vp]
        L.vs_carrier_compact_append.argtypes = [sp, cp, vp, vp, i32, i32, ip, vp]
        L.vs_carrier_compact_append_batched.argtypes = [sp, i32, vp, vp, i32, ip, vp, vp, i32, i32, ip,
                                                        vp, sz, vp]
        L.vs_decode_attn.argtypes = [sp, i32, vp, vp, i32, ip, vp, vp, vp, vp, vp, sz, vp]
        L.vs_carrier_mean_pool.argtypes = [vp, i32, i32, i32, vp, vp]
        L.vs_decode_attn_static.argtypes = [sp, i32, vp, vp, i32, ip, vp, vp, vp, vp, vp]
        L.vs_decode_static_scratch_bytes.argtypes = []
        L.vs_rmsnorm.argtypes = [vp, vp, i32, i32, ctypes.c_float, vp, vp]
        L.vs_linear.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, vp, sz, vp]
        L.vs_linear_workspace_bytes.argtypes = [i32, i32, i32]
        L.vs_linear_workspace_bytes.restype = sz
        L.vs_layer_workspace_bytes.argtypes = [sp, vp, i32]
        L.vs_layer_workspace_bytes.restype = sz
        L.vs_frame_decoder_layer.argtypes = [sp, vp, cp, vp, i32, vp, vp, sz, vp]
        L.vs_decode_static_scratch_bytes.restype = sz
        L.vs_set_tuning.argtypes = [i32, i32]
        L.vs_memory_bank_push.argtypes = [vp, vp, i32, vp, vp, sz, vp]
        L.vs_carrier_evict_append.argtypes = [sp, i32, vp, i32, i32, vp, vp, ctypes.c_int64, vp, vp]
        L.vs_memory_bank_workspace_bytes.argtypes = [i32]
        L.vs_memory_bank_workspace_bytes.restype = sz
        L.vs_frames_prefill_attn.argtypes = [sp, vp, vp, vp, vp, i32, i32, vp, vp, sz, vp]
        L.vs_frames_workspace_bytes.argtypes = [sp, i32, i32, i32]
        L.vs_frames_workspace_bytes.restype = sz
        L.vs_frame_qkv_project.argtypes = [sp, vp, i32, i32, vp, vp, vp, vp, vp, vp]
        for name in EXPORTS[2:-5]:
            getattr(L, name).restype = ctypes.c_int
        _LIB = L
    return _LIB


def status_string(code):
    return lib().vs_status_string(int(code)).decode()


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    """hipStream_t for the call: an int handle, a torch stream, or None = torch's current stream."""
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    elif not isinstance(stream, int):
        stream = stream.cuda_stream
    return ctypes.c_void_p(stream)


def current_stream_handle():
    """The raw handle of torch's current stream; pass it as `stream=` to skip the lookup per call."""
    import torch
    return int(torch.cuda.current_stream().cuda_stream)


def _ws(workspace):
    if workspace is None:
        return None, 0
    return _ptr(workspace), workspace.numel() * workspace.element_size()


def _check(rc, what):
    if rc != 0:
        raise VSError(rc, what)


def workspace_bytes(shape, max_q_tokens, max_cache_rows, n_streams):
    return int(lib().vs_workspace_bytes(ctypes.byref(shape), max_q_tokens, max_cache_rows, n_streams))


def workspace_init(shape, workspace, stream=None):
    wp, wb = _ws(workspace)
    _check(lib().vs_workspace_init(ctypes.byref(shape), wp, wb, _stream(stream)), "vs_workspace_init")


def make_workspace(shape, max_q_tokens, max_cache_rows, n_streams, device="cuda:0"):
    """Allocate (torch uint8 tensor) and initialise a workspace for the given limits."""
    import torch
    n = workspace_bytes(shape, max_q_tokens, max_cache_rows, n_streams)
    if n == 0:
        raise VSError(3, "vs_workspace_bytes")
    ws = torch.empty(n, dtype=torch.uint8, device=device)
    workspace_init(shape, ws)
    return ws


def frame_prefill_attn(shape, cache, q, k_f, v_f, out, workspace, stream=None):
    wp, wb = _ws(workspace)
    _check(lib().vs_frame_prefill_attn(ctypes.byref(shape), ctypes.byref(cache.c), _ptr(q), _ptr(k_f),
                                       _ptr(v_f), q.shape[0], _ptr(out), wp, wb, _stream(stream)),
           "vs_frame_prefill_attn")


def frame_prefill_compact(shape, cache, q, k_f, v_f, out, workspace, stream=None):
    wp, wb = _ws(workspace)
    row = ctypes.c_int32(-1)
    _check(lib().vs_frame_prefill_compact(ctypes.byref(shape), ctypes.byref(cache.c), _ptr(q), _ptr(k_f),
                                          _ptr(v_f), q.shape[0], _ptr(out), ctypes.byref(row), wp, wb,
                                          _stream(stream)), "vs_frame_prefill_compact")
    return row.value


def question_prefill_append(shape, cache, q, k_t, v_t, out, workspace, stream=None):
    """The question's tokens over the retained rows; all their K/V rows are appended."""
    wp, wb = _ws(workspace)
    _check(lib().vs_question_prefill_append(ctypes.byref(shape), ctypes.byref(cache.c), _ptr(q), _ptr(k_t), _ptr(v_t),
                                            q.shape[0], _ptr(out), wp, wb, _stream(stream)),
           "vs_question_prefill_append")


def frame_qkv_project(shape, e, w_qkv, q_out, k_out, v_out, c_out=None, stream=None):
    """e [N][d] -> q_out [N+1][Hq][D], k_out / v_out [N+1][Hkv][D] (carrier = mean of e, last row)."""
    _check(lib().vs_frame_qkv_project(ctypes.byref(shape), _ptr(e), e.shape[0], e.shape[1], _ptr(w_qkv), _ptr(q_out),
                                      _ptr(k_out), _ptr(v_out), _ptr(c_out), _stream(stream)),
           "vs_frame_qkv_project")


def carrier_compact_append(shape, cache, k_f, v_f, carrier_index=None, stream=None):
    n = k_f.shape[0]
    row = ctypes.c_int32(-1)
    _check(lib().vs_carrier_compact_append(ctypes.byref(shape), ctypes.byref(cache.c), _ptr(k_f), _ptr(v_f),
                                           n, n - 1 if carrier_index is None else carrier_index,
                                           ctypes.byref(row), _stream(stream)), "vs_carrier_compact_append")
    return row.value


def carrier_compact_append_batched(shape, k_slab, v_slab, lens, k_f, v_f, carrier_index=None,
                                   workspace=None, stream=None, rows_out=None):
    """lens: int32 [n_caches] in host memory, updated in place: a ctypes array, or a CPU int32
    torch tensor (pinned memory makes the copy of more than 64 lengths to the device
    asynchronous).  Returns the rows written as a list, or fills rows_out (ctypes int32 array or
    CPU int32 tensor; pinned, it is what the device copy is taken from, so leave it alone until
    the stream has passed the call) and returns it, which costs no Python work per cache."""
    n_caches, capacity = k_slab.shape[0], k_slab.shape[1]
    n = k_f.shape[1]
    rows = rows_out if rows_out is not None else (ctypes.c_int32 * n_caches)()

    def host_i32(t):
        assert t.device.type == "cpu" and t.numel() == n_caches and t.element_size() == 4 and t.is_contiguous()
        return ctypes.cast(t.data_ptr(), ctypes.POINTER(ctypes.c_int32))
    if hasattr(lens, "data_ptr"):
        lens = host_i32(lens)
    rows_arg = host_i32(rows) if hasattr(rows, "data_ptr") else rows
    wp, wb = _ws(workspace)
    _check(lib().vs_carrier_compact_append_batched(
        ctypes.byref(shape), n_caches, _ptr(k_slab), _ptr(v_slab), capacity, lens, _ptr(k_f), _ptr(v_f),
        n, n - 1 if carrier_index is None else carrier_index, rows_arg, wp, wb, _stream(stream)),
        "vs_carrier_compact_append_batched")
    return rows if rows_out is not None else list(rows)


def decode_attn(shape, k_slab, v_slab, lens, q, k_new, v_new, out, workspace, stream=None):
    """lens: ctypes int32 array [n_streams] (host), += 1 per stream when k_new is given."""
    n_streams, capacity = k_slab.shape[0], k_slab.shape[1]
    wp, wb = _ws(workspace)
    _check(lib().vs_decode_attn(ctypes.byref(shape), n_streams, _ptr(k_slab), _ptr(v_slab), capacity, lens,
                                _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out), wp, wb, _stream(stream)),
           "vs_decode_attn")


def decode_attn_static(shape, k_slab, v_slab, lens, q, k_new, v_new, out, stream=None):
    """decode_attn over the library's own scratch array (no workspace, nothing allocated)."""
    n_streams, capacity = k_slab.shape[0], k_slab.shape[1]
    _check(lib().vs_decode_attn_static(ctypes.byref(shape), n_streams, _ptr(k_slab), _ptr(v_slab), capacity, lens,
                                       _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out), _stream(stream)),
           "vs_decode_attn_static")


def decode_static_scratch_bytes():
    return int(lib().vs_decode_static_scratch_bytes())


LINEAR_STORE, LINEAR_RESIDUAL, LINEAR_GATED = 0, 1, 2


def rmsnorm(x, gamma, out, eps=1e-6, stream=None):
    """out [rows][d] = x * gamma / sqrt(mean(x^2) + eps)."""
    _check(lib().vs_rmsnorm(_ptr(x), _ptr(gamma), x.shape[0], x.shape[1], float(eps), _ptr(out), _stream(stream)),
           "vs_rmsnorm")


def linear_workspace_bytes(n_rows, k, n):
    return int(lib().vs_linear_workspace_bytes(n_rows, k, n))


def linear(x, w, out, mode=LINEAR_STORE, residual=None, workspace=None, stream=None):
    """out = x w^T (x [rows][k], w [n][k]); see vs_linear for the modes."""
    wp, wb = _ws(workspace)
    _check(lib().vs_linear(_ptr(x), _ptr(w), x.shape[0], x.shape[1], w.shape[0], int(mode), _ptr(residual), _ptr(out), wp, wb,
                           _stream(stream)), "vs_linear")


class _CLayerWeights(ctypes.Structure):
    _fields_ = [("norm1", ctypes.c_void_p), ("w_qkv", ctypes.c_void_p), ("w_o", ctypes.c_void_p),
                ("norm2", ctypes.c_void_p), ("w_gate_up", ctypes.c_void_p), ("w_down", ctypes.c_void_p),
                ("d_model", ctypes.c_int32), ("d_ff", ctypes.c_int32), ("eps", ctypes.c_float)]


class LayerWeights:
    """Device tensors of one decoder layer: norm1, norm2 [d]; w_qkv [(Hq+2Hkv)D][d]; w_o [d][Hq D];
    w_gate_up [2 d_ff][d] (rows alternate gate and value projections); w_down [d][d_ff]."""

    def __init__(self, norm1, w_qkv, w_o, norm2, w_gate_up, w_down, eps=1e-6):
        self.tensors = (norm1, w_qkv, w_o, norm2, w_gate_up, w_down)
        self.c = _CLayerWeights(norm1.data_ptr(), w_qkv.data_ptr(), w_o.data_ptr(), norm2.data_ptr(),
                                w_gate_up.data_ptr(), w_down.data_ptr(), norm1.shape[0], w_down.shape[1], float(eps))


def layer_workspace_bytes(shape, weights, n_tokens):
    return int(lib().vs_layer_workspace_bytes(ctypes.byref(shape), ctypes.byref(weights.c), n_tokens))


def frame_decoder_layer(shape, weights, cache, h_in, h_out, workspace, stream=None):
    """One decoder layer for one frame run h_in [T][d] -> h_out [T][d]; the carrier's K/V row is appended."""
    wp, wb = _ws(workspace)
    _check(lib().vs_frame_decoder_layer(ctypes.byref(shape), ctypes.byref(weights.c), ctypes.byref(cache.c), _ptr(h_in),
                                        h_in.shape[0], _ptr(h_out), wp, wb, _stream(stream)), "vs_frame_decoder_layer")


def frames_workspace_bytes(shape, n_frames, n_tokens, max_cache_rows):
    return int(lib().vs_frames_workspace_bytes(ctypes.byref(shape), n_frames, n_tokens, max_cache_rows))


def frames_prefill_attn(shape, cache, q, k_f, v_f, out, workspace, stream=None):
    """A run of frames under the semantic-aware mask: q, out [F][T][Hq][D], k_f, v_f [F][T][Hkv][D]."""
    wp, wb = _ws(workspace)
    _check(lib().vs_frames_prefill_attn(ctypes.byref(shape), ctypes.byref(cache.c), _ptr(q), _ptr(k_f), _ptr(v_f),
                                        q.shape[0], q.shape[1], _ptr(out), wp, wb, _stream(stream)),
           "vs_frames_prefill_attn")


class _CBank(ctypes.Structure):
    _fields_ = [("e", ctypes.c_void_p), ("capacity", ctypes.c_int32), ("len", ctypes.c_int32),
                ("d", ctypes.c_int32), ("dtype", ctypes.c_int32)]


class Bank:
    """Memory bank of the carriers' embeddings: a device tensor [capacity][d] and a host-side count."""

    def __init__(self, e, dtype, length=0):
        assert e.dim() == 2 and e.is_contiguous()
        self.e = e
        code = {"f32": VS_F32, "bf16": VS_BF16}.get(dtype, dtype)
        self.c = _CBank(e.data_ptr(), e.shape[0], int(length), e.shape[1], code)

    @property
    def len(self):
        return self.c.len


def memory_bank_workspace_bytes(capacity):
    return int(lib().vs_memory_bank_workspace_bytes(capacity))


def memory_bank_push(bank, e_new, victim, workspace, policy=0, stream=None):
    """victim: device int32 tensor with one element (written by the call)."""
    wp, wb = _ws(workspace)
    _check(lib().vs_memory_bank_push(ctypes.byref(bank.c), _ptr(e_new), policy, _ptr(victim), wp, wb,
                                     _stream(stream)), "vs_memory_bank_push")


def carrier_evict_append(shape, caches, first_row, bank_capacity, k_rows, v_rows, victim, stream=None):
    """caches: list of Cache (one per layer); k_rows / v_rows: device tensors [n_layers][Hkv][D]."""
    n = len(caches)
    arr = (_CCache * n)(*[c.c for c in caches])
    stride = k_rows.stride(0) * k_rows.element_size() if n > 1 else 0
    try:
        _check(lib().vs_carrier_evict_append(ctypes.byref(shape), n, arr, first_row, bank_capacity, _ptr(k_rows),
                                             _ptr(v_rows), stride, _ptr(victim), _stream(stream)),
               "vs_carrier_evict_append")
    finally:
        for c, a in zip(caches, arr):
            c.c.len = a.len


def carrier_mean_pool(e, c_out, dtype, stream=None):
    code = {"f32": VS_F32, "bf16": VS_BF16}.get(dtype, dtype)
    _check(lib().vs_carrier_mean_pool(_ptr(e), e.shape[0], e.shape[1], code, _ptr(c_out), _stream(stream)),
           "vs_carrier_mean_pool")


TUNE_PREFILL_SPLITS, TUNE_PREFILL_KV_GROUPS, TUNE_DECODE_CHUNK_ROWS, TUNE_PREFILL_MERGE = 0, 1, 2, 4


def set_tuning(knob, value):
    _check(lib().vs_set_tuning(int(knob), int(value)), "vs_set_tuning")
