"""ctypes binding of oracle/vs_oracle.c (TEST INFRASTRUCTURE, fp64, CPU only).

Every function takes/returns numpy float64 arrays, row-major:
Q [Tq][Hq][D], K/V [rows][Hkv][D].  The arithmetic is all in the C file; this
module only marshals arguments.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None


class OracleError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"oracle {what} failed with code {code}")
        self.code = code


ERR_ARG, ERR_CAPACITY, ERR_NOMEM = 1, 2, 3


def _need(ok, what):
    if not ok:
        raise OracleError(ERR_ARG, what)


def _lib():
    global _LIB
    if _LIB is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build()
        lib = ctypes.CDLL(path)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int64)
        i64, i32, f64 = ctypes.c_int64, ctypes.c_int32, ctypes.c_double
        lib.vs_oracle_num_threads.restype = ctypes.c_int
        lib.vs_oracle_attention.argtypes = [dp, i64, i32, i32, i32, dp, dp, i64, ip, f64, dp, dp]
        lib.vs_oracle_frame_prefill.argtypes = [dp, dp, dp, i64, dp, dp, i64, i32, i32, i32, f64, dp, dp]
        lib.vs_oracle_compact_append.argtypes = [dp, dp, i64, ip, dp, dp, i64, i64, i32, i32, ip]
        lib.vs_oracle_decode.argtypes = [dp, dp, dp, i64, ip, dp, dp, i32, i32, i32, f64, dp]
        lib.vs_oracle_mean_pool.argtypes = [dp, i64, i64, dp]
        lib.vs_oracle_frames_prefill.argtypes = [dp, dp, dp, i64, dp, dp, i64, i64, i32, i32, i32, f64, dp]
        lib.vs_oracle_query_prefill.argtypes = [dp, dp, dp, i64, ip, dp, dp, i64, i32, i32, i32, f64, dp]
        lib.vs_oracle_frame_qkv.argtypes = [dp, i64, i64, dp, i64, dp]
        lib.vs_oracle_bank_victim.argtypes = [dp, i64, i64, dp, i32, dp, ip]
        lib.vs_oracle_rmsnorm.argtypes = [dp, i64, i64, dp, f64, dp]
        lib.vs_oracle_linear.argtypes = [dp, i64, i64, dp, i64, dp]
        lib.vs_oracle_gated_unit.argtypes = [dp, dp, i64, i64, dp]
        lib.vs_oracle_decoder_layer.argtypes = [dp, i64, i64, i32, i32, i32, i64, dp, dp, dp, dp, dp, dp, dp, dp, dp, f64,
                                                dp, dp, i64, f64, dp, dp, dp]
        lib.vs_oracle_bank_apply.argtypes = [dp, i64, i64, i64, i64, i64, i64, dp, ip]
        _LIB = lib
    return _LIB


def _c(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def num_threads():
    return int(_lib().vs_oracle_num_threads())


def attention(Q, Kall, Vall, vis, scale, return_probs=False):
    """Eq. 1 with query row i seeing key rows 0..vis[i]-1.  Q [Tq][Hq][D], K/V [R][Hkv][D]."""
    Q, Kall, Vall = _c(Q), _c(Kall), _c(Vall)
    Tq, Hq, D = Q.shape
    R, Hkv, D2 = Kall.shape
    assert D2 == D and Vall.shape == Kall.shape
    vis = np.ascontiguousarray(vis, dtype=np.int64)
    assert vis.shape == (Tq,)
    O = np.empty((Tq, Hq, D), dtype=np.float64)
    P = np.empty((Hq, Tq, R), dtype=np.float64) if return_probs else None
    rc = _lib().vs_oracle_attention(_p(Q), Tq, Hq, Hkv, D, _p(Kall), _p(Vall), R,
                                    vis.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                                    float(scale), _p(O), _p(P))
    if rc:
        raise OracleError(rc, "attention")
    return (O, P) if return_probs else O


def frame_prefill(Q, Kc, Vc, Kf, Vf, scale, return_probs=False):
    """Prefill of one frame run [T] (carrier last) over L retained rows + causal run."""
    Q, Kf, Vf = _c(Q), _c(Kf), _c(Vf)
    T, Hq, D = Q.shape
    T2, Hkv, D2 = Kf.shape
    assert T2 == T and D2 == D and Vf.shape == Kf.shape
    if Kc is None or len(Kc) == 0:
        L, Kc, Vc = 0, None, None
    else:
        Kc, Vc = _c(Kc), _c(Vc)
        L = Kc.shape[0]
        assert Kc.shape[1:] == (Hkv, D) and Vc.shape == Kc.shape
    O = np.empty((T, Hq, D), dtype=np.float64)
    P = np.empty((Hq, T, L + T), dtype=np.float64) if return_probs else None
    rc = _lib().vs_oracle_frame_prefill(_p(Q), _p(Kc), _p(Vc), L, _p(Kf), _p(Vf), T,
                                        Hq, Hkv, D, float(scale), _p(O), _p(P))
    if rc:
        raise OracleError(rc, "frame_prefill")
    return (O, P) if return_probs else O


def compact_append(Kc, Vc, length, Kf, Vf, carrier=None):
    """In place: cache row `length` <- frame row `carrier` (default last).  Returns (row, new_len)."""
    assert Kc.dtype == np.float64 and Vc.dtype == np.float64
    assert Kc.flags.c_contiguous and Vc.flags.c_contiguous
    Kf, Vf = _c(Kf), _c(Vf)
    cap, Hkv, D = Kc.shape
    T = Kf.shape[0]
    assert Kf.shape[1:] == (Hkv, D) and Vf.shape == Kf.shape and Vc.shape == Kc.shape
    if carrier is None:
        carrier = T - 1
    ln = ctypes.c_int64(int(length))
    row = ctypes.c_int64(-1)
    rc = _lib().vs_oracle_compact_append(_p(Kc), _p(Vc), cap, ctypes.byref(ln), _p(Kf), _p(Vf),
                                         T, int(carrier), Hkv, D, ctypes.byref(row))
    if rc:
        raise OracleError(rc, "compact_append")
    return int(row.value), int(ln.value)


def decode(q, Kc, Vc, length, k_new, v_new, scale):
    """One stream, one step: append (k_new, v_new) at row `length` (if given), attend over all rows.
    Kc/Vc [capacity][Hkv][D] are modified in place.  Returns (o [Hq][D], new_len)."""
    assert Kc.dtype == np.float64 and Vc.dtype == np.float64
    assert Kc.flags.c_contiguous and Vc.flags.c_contiguous
    q = _c(q)
    Hq, D = q.shape
    cap, Hkv, D2 = Kc.shape
    assert D2 == D
    if k_new is not None:
        k_new, v_new = _c(k_new), _c(v_new)
        assert k_new.shape == (Hkv, D) and v_new.shape == (Hkv, D)
    ln = ctypes.c_int64(int(length))
    o = np.empty((Hq, D), dtype=np.float64)
    rc = _lib().vs_oracle_decode(_p(q), _p(Kc), _p(Vc), cap, ctypes.byref(ln), _p(k_new), _p(v_new),
                                 Hq, Hkv, D, float(scale), _p(o))
    if rc:
        raise OracleError(rc, "decode")
    return o, int(ln.value)


def mean_pool(E):
    """Carrier embedding: arithmetic mean of the N rows of E [N][d]."""
    E = _c(E)
    N, d = E.shape
    c = np.empty((d,), dtype=np.float64)
    rc = _lib().vs_oracle_mean_pool(_p(E), N, d, _p(c))
    if rc:
        raise OracleError(rc, "mean_pool")
    return c


def bank_victim(E, e_new, policy=0):
    """Section 3.3, memory mechanism: which carrier a full bank drops.  E [M][d] bank embeddings
    (oldest first), e_new [d].  Returns (victim index, cosines [M])."""
    E, e_new = _c(E), _c(e_new)
    M, d = E.shape
    cos = np.empty(M, dtype=np.float64)
    victim = ctypes.c_int64(-1)
    rc = _lib().vs_oracle_bank_victim(_p(E), M, d, _p(e_new), policy, _p(cos), ctypes.byref(victim))
    if rc:
        raise OracleError(rc, "bank_victim")
    return int(victim.value), cos


def bank_apply(rows, first, M, n, victim, row_new):
    """A carrier arrives: rows [capacity][...] (modified in place) holds n <= M carrier rows behind
    `first` other rows.  Appends, or drops row first+victim, closes the gap and puts the new row
    last.  Returns the carrier count after the call."""
    assert rows.dtype == np.float64 and rows.flags.c_contiguous
    width = int(np.prod(rows.shape[1:]))
    row_new = _c(row_new).reshape(-1)
    assert row_new.size == width
    n_out = ctypes.c_int64(-1)
    rc = _lib().vs_oracle_bank_apply(_p(rows), rows.shape[0], width, first, M, n, victim, _p(row_new), ctypes.byref(n_out))
    if rc:
        raise OracleError(rc, "bank_apply")
    return int(n_out.value)


def frames_prefill(Q, Kc, Vc, Kf, Vf, scale):
    """Several frames in one run with the semantic-aware mask (Section 3.4): a token sees the
    retained rows, the carriers (last tokens) of earlier frames of the run, and its own frame up
    to itself.  Q [F][T][Hq][D], Kf/Vf [F][T][Hkv][D], Kc/Vc [L][Hkv][D] or None."""
    Q, Kf, Vf = _c(Q), _c(Kf), _c(Vf)
    F, T, Hq, D = Q.shape
    Hkv = Kf.shape[2]
    assert Kf.shape == (F, T, Hkv, D) and Vf.shape == Kf.shape
    if Kc is None or len(Kc) == 0:
        L, Kc, Vc = 0, None, None
    else:
        Kc, Vc = _c(Kc), _c(Vc)
        L = Kc.shape[0]
    O = np.empty((F, T, Hq, D), dtype=np.float64)
    rc = _lib().vs_oracle_frames_prefill(_p(Q), _p(Kc), _p(Vc), L, _p(Kf), _p(Vf), F, T, Hq, Hkv, D, float(scale), _p(O))
    if rc:
        raise OracleError(rc, "frames_prefill")
    return O


def query_prefill(Q, Kc, Vc, length, Kt, Vt, scale):
    """The question's Tq tokens over the retained rows (Section 3.3, decoding phase): token j is
    appended at row length + j and attends over every row up to and including its own.
    Kc/Vc [capacity][Hkv][D] are modified in place.  Returns (O [Tq][Hq][D], new_len)."""
    assert Kc.dtype == np.float64 and Vc.dtype == np.float64
    assert Kc.flags.c_contiguous and Vc.flags.c_contiguous
    Q, Kt, Vt = _c(Q), _c(Kt), _c(Vt)
    Tq, Hq, D = Q.shape
    cap, Hkv, D2 = Kc.shape
    assert D2 == D and Kt.shape == (Tq, Hkv, D) and Vt.shape == Kt.shape and Vc.shape == Kc.shape
    ln = ctypes.c_int64(int(length))
    O = np.empty((Tq, Hq, D), dtype=np.float64)
    rc = _lib().vs_oracle_query_prefill(_p(Q), _p(Kc), _p(Vc), cap, ctypes.byref(ln), _p(Kt), _p(Vt), Tq,
                                        Hq, Hkv, D, float(scale), _p(O))
    if rc:
        raise OracleError(rc, "query_prefill")
    return O, int(ln.value)


def frame_qkv(E, W, n_q_heads, n_kv_heads, head_dim):
    """The frame's N token embeddings E [N][d] plus the carrier (their mean, appended last)
    projected with W [(Hq + 2 Hkv) D][d] (rows: the features of W_Q, then W_K, then W_V; Section
    3.1).  Returns Q [N+1][Hq][D], K, V [N+1][Hkv][D]."""
    E, W = _c(E), _c(W)
    N, d = E.shape
    n_out = (n_q_heads + 2 * n_kv_heads) * head_dim
    assert W.shape == (n_out, d)
    Y = np.empty((N + 1, n_out), dtype=np.float64)
    rc = _lib().vs_oracle_frame_qkv(_p(E), N, d, _p(W), n_out, _p(Y))
    if rc:
        raise OracleError(rc, "frame_qkv")
    nq, nk = n_q_heads * head_dim, n_kv_heads * head_dim
    return (Y[:, :nq].reshape(N + 1, n_q_heads, head_dim).copy(),
            Y[:, nq:nq + nk].reshape(N + 1, n_kv_heads, head_dim).copy(),
            Y[:, nq + nk:].reshape(N + 1, n_kv_heads, head_dim).copy())


def rmsnorm(X, g, eps):
    """Y[t][j] = X[t][j] g[j] / sqrt(mean_k X[t][k]^2 + eps)  (reading of the backbone's norm)."""
    X, g = _c(X), _c(g)
    T, d = X.shape
    _need(g.shape == (d,), "rmsnorm")
    Y = np.empty_like(X)
    rc = _lib().vs_oracle_rmsnorm(_p(X), T, d, _p(g), float(eps), _p(Y))
    if rc:
        raise OracleError(rc, "rmsnorm")
    return Y


def linear(X, W):
    """Y = X W^T: X [T][K], W [N][K] (one row of weights per output feature; Section 3.1)."""
    X, W = _c(X), _c(W)
    T, K = X.shape
    N = W.shape[0]
    _need(W.shape == (N, K), "linear")
    Y = np.empty((T, N), dtype=np.float64)
    rc = _lib().vs_oracle_linear(_p(X), T, K, _p(W), N, _p(Y))
    if rc:
        raise OracleError(rc, "linear")
    return Y


def gated_unit(G, U):
    """silu(G) * U, silu(a) = a / (1 + exp(-a))."""
    G, U = _c(G), _c(U)
    _need(G.shape == U.shape and G.ndim == 2, "gated_unit")
    Y = np.empty_like(G)
    rc = _lib().vs_oracle_gated_unit(_p(G), _p(U), G.shape[0], G.shape[1], _p(Y))
    if rc:
        raise OracleError(rc, "gated_unit")
    return Y


def decoder_layer(H, g1, Wq, Wk, Wv, Wo, g2, Wg, Wu, Wd, eps, Kc, Vc, n_q_heads, n_kv_heads, head_dim, scale):
    """One pre-norm decoder layer for one frame run H [T][d] over the retained rows Kc, Vc [L][Hkv][D]
    (None for an empty cache).  Returns (H_out [T][d], K_f, V_f [T][Hkv][D])."""
    H = _c(H)
    T, d = H.shape
    nq, nk = n_q_heads * head_dim, n_kv_heads * head_dim
    g1, Wq, Wk, Wv, Wo, g2, Wg, Wu, Wd = (_c(a) for a in (g1, Wq, Wk, Wv, Wo, g2, Wg, Wu, Wd))
    F = Wg.shape[0]
    _need(Wq.shape == (nq, d) and Wk.shape == (nk, d) and Wv.shape == (nk, d) and Wo.shape == (d, nq), "decoder_layer")
    _need(Wg.shape == (F, d) and Wu.shape == (F, d) and Wd.shape == (d, F) and g1.shape == (d,) and g2.shape == (d,), "decoder_layer")
    L = 0 if Kc is None else Kc.shape[0]
    if L:
        Kc, Vc = _c(Kc), _c(Vc)
    Kf = np.empty((T, n_kv_heads, head_dim), dtype=np.float64)
    Vf = np.empty_like(Kf)
    Hout = np.empty_like(H)
    rc = _lib().vs_oracle_decoder_layer(_p(H), T, d, n_q_heads, n_kv_heads, head_dim, F, _p(g1), _p(Wq), _p(Wk), _p(Wv),
                                        _p(Wo), _p(g2), _p(Wg), _p(Wu), _p(Wd), float(eps),
                                        _p(Kc) if L else None, _p(Vc) if L else None, L, float(scale), _p(Kf), _p(Vf),
                                        _p(Hout))
    if rc:
        raise OracleError(rc, "decoder_layer")
    return Hout, Kf, Vf
