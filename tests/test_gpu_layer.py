"""GPU parity of the dense layers and of the decoder layer around the attention, through the C ABI.

Each dense stage is one fp32 computation rounded once to bf16, so it is held to one rounding
(2^-8 relative) plus an fp32 accumulation term, against the oracle's stage function
evaluated on the very bytes the GPU stage read.  The fused layer must equal, bit for bit, the chain
of the separate entry points (same kernels in the same order), whose stages are checked one by one;
end to end it is also compared with the oracle's fp64 layer under a gate derived below."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_09387_amd as vs
from gpu_util import DEV, check_close, scale32, vs_shape
from synth import AttnShape, cache_rows, draw, hidden_rows, layer_weights, to_f64

pytestmark = pytest.mark.gpu

QW = AttnShape(28, 4, 128, "bf16")
BF = torch.bfloat16

# one rounding to bf16 (8 significand bits, to nearest) moves a value by at most 2^-8 of itself; what
# the fp32 arithmetic before it may add (it can also tip the rounding) is each stage's slack
ONE_ROUNDING = 2.0 ** -8
# fp32 sums of K products, accumulated in blocks: error well below sqrt(K) 2^-24 sum|x||w| for the K
# here (<= 18944: 2^-16.9); the gate is 2^-16 of sum|x||w|
ACC = 2.0 ** -16


def _dev(t):
    return t.to(DEV)


def _f64(t):
    return t.detach().to(torch.float64).cpu().numpy()


def _check_stage(got, ref, slack, what):
    """|got - ref| <= 2^-8 |ref| + slack, element by element."""
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, f"{what}: shape {got.shape} vs {ref.shape}"
    assert np.all(np.isfinite(got)), f"{what}: non-finite"
    err = np.abs(got - ref)
    use = float((err / (ONE_ROUNDING * np.abs(ref) + slack + 1e-300)).max())
    assert use <= 1.0, f"{what}: {use:.2f}x the gate (max-abs {err.max():.3e})"
    print(f"[parity] {what}: max-abs {err.max():.2e} gate-use {use:.2f}")


def _linear_ws(T, K, N):
    n = vs.linear_workspace_bytes(T, K, N)
    return torch.empty(max(n, 16), dtype=torch.uint8, device=DEV) if n else None


def _ref_linear(x, w, mode, res, cols=None):
    """Oracle value and accumulation slack of one vs_linear call on host tensors x, w (res) for the
    output columns `cols` (all if None)."""
    X, W = to_f64(x), to_f64(w)
    N = W.shape[0]
    if mode == vs.LINEAR_GATED:
        cols = np.arange(N // 2) if cols is None else np.asarray(cols)
        G, U = oracle.linear(X, W[2 * cols]), oracle.linear(X, W[2 * cols + 1])
        ag, au = np.abs(X) @ np.abs(W[2 * cols]).T, np.abs(X) @ np.abs(W[2 * cols + 1]).T
        ref = oracle.gated_unit(G, U)
        silu = oracle.gated_unit(G, np.ones_like(G))
        # d silu / dg is within [-0.1, 1.1]
        return ref, ACC * (1.1 * ag * np.abs(U) + np.abs(silu) * au)
    cols = np.arange(N) if cols is None else np.asarray(cols)
    ref = oracle.linear(X, W[cols])
    slack = ACC * (np.abs(X) @ np.abs(W[cols]).T)
    if mode == vs.LINEAR_RESIDUAL:
        R = to_f64(res)[:, cols]
        ref = ref + R
        slack = slack + ACC * np.abs(R)
    return ref, slack


# ---------------------------------------------------------------------------- RMS norm
@pytest.mark.parametrize("T,d,eps", [(1, 8, 1e-6), (5, 1000, 1e-5), (170, 3584, 1e-6), (192, 3584, 0.0), (33, 18944, 1e-6),
                                     (3, 64, 0.5)])
def test_rmsnorm_against_the_oracle(T, d, eps):
    x = draw(900 + T, (T, d), 1.7, "bf16")
    g = (1.0 + 0.2 * draw(901 + T, (d,), 1.0, "f32")).to(BF)
    out = torch.full((T, d), float("nan"), dtype=BF, device=DEV)
    vs.rmsnorm(_dev(x), _dev(g), out, eps=eps)
    torch.cuda.synchronize()
    eps32 = float(np.float32(eps))
    _check_stage(_f64(out), oracle.rmsnorm(to_f64(x), to_f64(g), eps32), 1e-7, f"rmsnorm {T}x{d} eps {eps}")


def test_rmsnorm_in_place_and_zero_rows():
    """A row of zeros stays zero when eps > 0; writing over the input is allowed."""
    x = draw(77, (4, 256), 1.0, "bf16")
    x[2] = 0
    g = torch.ones(256, dtype=BF)
    xd = _dev(x)
    vs.rmsnorm(xd, _dev(g), xd, eps=1e-6)
    torch.cuda.synchronize()
    assert torch.all(xd[2] == 0)
    _check_stage(_f64(xd), oracle.rmsnorm(to_f64(x), to_f64(g), float(np.float32(1e-6))), 1e-7, "rmsnorm in place")


# ---------------------------------------------------------------------------- dense layers
LINEAR_CASES = [
    # T, K, N: single tile, ragged features, ragged rows, every block width, with and without split-K
    (1, 64, 2), (7, 128, 70), (16, 64, 16), (192, 64, 160), (170, 192, 330), (3, 3584, 512), (170, 512, 4608),
    (191, 1024, 130), (64, 2048, 1536), (170, 3584, 640), (33, 4096, 96),
]


@pytest.mark.parametrize("mode", [vs.LINEAR_STORE, vs.LINEAR_RESIDUAL, vs.LINEAR_GATED])
@pytest.mark.parametrize("T,K,N", LINEAR_CASES)
def test_linear_against_the_oracle(T, K, N, mode):
    x = draw(1000 + T + K, (T, K), 1.0, "bf16")
    w = draw(2000 + N + K, (N, K), K ** -0.5, "bf16")
    n_out = N // 2 if mode == vs.LINEAR_GATED else N
    res = draw(3000 + N, (T, N), 1.0, "bf16") if mode == vs.LINEAR_RESIDUAL else None
    # guard rows around the output catch stores past the ragged edges
    canvas = torch.full((T + 16, n_out), float("nan"), dtype=BF, device=DEV)
    out = canvas[8:T + 8]  # (8 rows in: the start stays 16-byte aligned for any width)
    ws = _linear_ws(T, K, N)
    vs.linear(_dev(x), _dev(w), out, mode=mode, residual=None if res is None else _dev(res), workspace=ws)
    torch.cuda.synchronize()
    assert torch.isnan(canvas[:8]).all() and torch.isnan(canvas[T + 8:]).all(), "wrote outside its rows"
    ref, slack = _ref_linear(x, w, mode, res)
    _check_stage(_f64(out), ref, slack, f"linear mode {mode} T={T} K={K} N={N} split-K ws {0 if ws is None else ws.numel()}")


def test_linear_is_deterministic_and_leaves_inputs_alone():
    T, K, N = 170, 3584, 3584
    x, w = _dev(draw(11, (T, K), 1.0, "bf16")), _dev(draw(12, (N, K), K ** -0.5, "bf16"))
    res = _dev(draw(13, (T, N), 1.0, "bf16"))
    x0, w0, r0 = x.clone(), w.clone(), res.clone()
    ws = _linear_ws(T, K, N)
    assert ws is not None, "this shape is expected to split K"
    a, b = torch.empty((T, N), dtype=BF, device=DEV), torch.empty((T, N), dtype=BF, device=DEV)
    vs.linear(x, w, a, mode=vs.LINEAR_RESIDUAL, residual=res, workspace=ws)
    ws.fill_(0xFF)  # what the last call left in the workspace does not matter
    vs.linear(x, w, b, mode=vs.LINEAR_RESIDUAL, residual=res, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(a, b) and torch.equal(x, x0) and torch.equal(w, w0) and torch.equal(res, r0)


def test_linear_residual_in_place():
    """out may be the residual itself (each element is read once, by the thread that writes it)."""
    T, K, N = 170, 1024, 768
    x, w = draw(21, (T, K), 1.0, "bf16"), draw(22, (N, K), K ** -0.5, "bf16")
    res = draw(23, (T, N), 1.0, "bf16")
    buf = _dev(res)
    vs.linear(_dev(x), _dev(w), buf, mode=vs.LINEAR_RESIDUAL, residual=buf, workspace=_linear_ws(T, K, N))
    torch.cuda.synchronize()
    ref, slack = _ref_linear(x, w, vs.LINEAR_RESIDUAL, res)
    _check_stage(_f64(buf), ref, slack, "residual in place")


@pytest.mark.parametrize("which", ["qkv", "o", "gate_up", "down"])
def test_linear_7b_shapes_on_sampled_features(which):
    """The four dense layers at the 7B backbone's sizes (d 3584, d_ff 18944), 170 rows: all rows of
    256 output features drawn at random plus the first and last 16, against the oracle."""
    d, F, nq, nk, T = 3584, 18944, 28 * 128, 4 * 128, 170
    K, N, mode = {"qkv": (d, nq + 2 * nk, vs.LINEAR_STORE), "o": (nq, d, vs.LINEAR_RESIDUAL),
                  "gate_up": (d, 2 * F, vs.LINEAR_GATED), "down": (F, d, vs.LINEAR_RESIDUAL)}[which]
    x = draw(31, (T, K), 1.0, "bf16")
    w = draw(32, (N, K), K ** -0.5, "bf16")
    res = draw(33, (T, N), 1.0, "bf16") if mode == vs.LINEAR_RESIDUAL else None
    n_out = N // 2 if mode == vs.LINEAR_GATED else N
    out = torch.full((T, n_out), float("nan"), dtype=BF, device=DEV)
    vs.linear(_dev(x), _dev(w), out, mode=mode, residual=None if res is None else _dev(res), workspace=_linear_ws(T, K, N))
    torch.cuda.synchronize()
    assert not torch.isnan(out).any()
    rng = np.random.default_rng(5)
    cols = np.unique(np.concatenate([np.arange(16), np.arange(n_out - 16, n_out), rng.integers(0, n_out, 256)]))
    ref, slack = _ref_linear(x, w, mode, res, cols)
    _check_stage(_f64(out)[:, cols], ref, slack, f"{which} at the 7B shape, {len(cols)} features")


# ---------------------------------------------------------------------------- the decoder layer
def _pack(w):
    """Device tensors in the layouts vs_layer_weights asks for."""
    w_qkv = torch.cat([w["w_q"], w["w_k"], w["w_v"]], dim=0).contiguous()
    F, d = w["w_gate"].shape
    w_gate_up = torch.stack([w["w_gate"], w["w_up"]], dim=1).reshape(2 * F, d).contiguous()
    return dict(norm1=_dev(w["norm1"]), w_qkv=_dev(w_qkv), w_o=_dev(w["w_o"]), norm2=_dev(w["norm2"]),
                w_gate_up=_dev(w_gate_up), w_down=_dev(w["w_down"]))


def _cache(s, hk, hv, L, cap):
    k = torch.zeros((cap, s.n_kv_heads, s.head_dim), dtype=BF, device=DEV)
    v = torch.zeros_like(k)
    if L:
        k[:L].copy_(hk[:L])
        v[:L].copy_(hv[:L])
    return vs.Cache(k, v, L)


def _chain(s, pk, eps, cache, h, T, d, F):
    """The layer as separate entry points; returns every stage's device tensor."""
    nq, nk = s.n_q_heads * s.head_dim, s.n_kv_heads * s.head_dim
    sh = vs_shape(s)
    x1 = torch.empty((T, d), dtype=BF, device=DEV)
    vs.rmsnorm(h, pk["norm1"], x1, eps=eps)
    qkv = torch.empty((T, nq + 2 * nk), dtype=BF, device=DEV)
    vs.linear(x1, pk["w_qkv"], qkv, workspace=_linear_ws(T, d, nq + 2 * nk))
    q = qkv[:, :nq].contiguous().view(T, s.n_q_heads, s.head_dim)
    k = qkv[:, nq:nq + nk].contiguous().view(T, s.n_kv_heads, s.head_dim)
    v = qkv[:, nq + nk:].contiguous().view(T, s.n_kv_heads, s.head_dim)
    a = torch.empty((T, s.n_q_heads, s.head_dim), dtype=BF, device=DEV)
    L = cache.len
    ws = vs.make_workspace(sh, T, L + 1, 0, DEV)
    vs.frame_prefill_compact(sh, cache, q, k, v, a, ws)
    h1 = torch.empty((T, d), dtype=BF, device=DEV)
    vs.linear(a.view(T, nq), pk["w_o"], h1, mode=vs.LINEAR_RESIDUAL, residual=h, workspace=_linear_ws(T, nq, d))
    x2 = torch.empty((T, d), dtype=BF, device=DEV)
    vs.rmsnorm(h1, pk["norm2"], x2, eps=eps)
    act = torch.empty((T, F), dtype=BF, device=DEV)
    vs.linear(x2, pk["w_gate_up"], act, mode=vs.LINEAR_GATED, workspace=_linear_ws(T, d, 2 * F))
    out = torch.empty((T, d), dtype=BF, device=DEV)
    vs.linear(act, pk["w_down"], out, mode=vs.LINEAR_RESIDUAL, residual=h1, workspace=_linear_ws(T, F, d))
    torch.cuda.synchronize()
    return dict(x1=x1, qkv=qkv, q=q, k=k, v=v, a=a, h1=h1, x2=x2, act=act, out=out)


LAYER_CASES = [
    # T, d, F, L, shape
    (170, 512, 1536, 300, AttnShape(8, 2, 128, "bf16")),
    (21, 256, 704, 0, AttnShape(4, 4, 128, "bf16")),
    (1, 128, 64, 5, AttnShape(2, 1, 128, "bf16")),
    (192, 1024, 2816, 1200, AttnShape(28, 4, 128, "bf16")),
]


@pytest.mark.parametrize("T,d,F,L,s", LAYER_CASES)
def test_decoder_layer_against_the_oracle(T, d, F, L, s):
    """Fused layer == chain of the separate entry points (bits); every stage of the chain against the
    oracle's stage on the bytes that stage read; the whole against the oracle's fp64 layer.

    End-to-end gate.  Between the input and the output eight values are rounded to bf16 (x1, q/k/v,
    P and the attention output, h1, x2, the gated product, the output): each rounding is noise of
    ~1.6e-3 rms of the value it touches (at most 2^-8, averaged over a binade), the dense layers pass
    relative noise on unchanged, and the two residual sums add the unrounded input back, so the
    output carries at most sqrt(8) x 1.6e-3 = 4.5e-3 rms of relative noise, whose 5 sigma tail over
    ~1e5 elements is 2.3e-2 rms.  Gates: element 2^-7 |ref| + 3.5e-2 rms(ref) (1.5x the tail), mean
    1e-2 rms(ref) (2.7x the mean of such noise)."""
    eps = 1e-6
    w = layer_weights(41, s, d, F)
    pk = _pack(w)
    h = hidden_rows(42, T, d)
    hk, hv = cache_rows(43, s, max(L, 1), 0.5)
    hd = _dev(h)
    weights = vs.LayerWeights(pk["norm1"], pk["w_qkv"], pk["w_o"], pk["norm2"], pk["w_gate_up"], pk["w_down"], eps=eps)
    sh = vs_shape(s)
    # fused
    cache = _cache(s, hk, hv, L, L + 2)
    n = vs.layer_workspace_bytes(sh, weights, T)
    assert n > 0
    ws = torch.empty(n, dtype=torch.uint8, device=DEV)
    vs.workspace_init(sh, ws)
    out = torch.full((T, d), float("nan"), dtype=BF, device=DEV)
    vs.frame_decoder_layer(sh, weights, cache, hd, out, ws)
    torch.cuda.synchronize()
    assert cache.len == L + 1
    # chain
    cache2 = _cache(s, hk, hv, L, L + 2)
    st = _chain(s, pk, eps, cache2, hd, T, d, F)
    assert torch.equal(out, st["out"]), "fused layer differs from the chain of its stages"
    assert torch.equal(cache.k, cache2.k) and torch.equal(cache.v, cache2.v) and cache2.len == L + 1
    assert torch.equal(cache.k[L], st["k"][T - 1]) and torch.equal(cache.v[L], st["v"][T - 1]), "carrier row"
    # stages, each on the bytes it read
    eps32 = float(np.float32(eps))
    host = {k_: v_.cpu() for k_, v_ in st.items()}
    _check_stage(_f64(st["x1"]), oracle.rmsnorm(to_f64(h), to_f64(w["norm1"]), eps32), 1e-7, "stage norm1")
    ref, slack = _ref_linear(host["x1"], torch.cat([w["w_q"], w["w_k"], w["w_v"]]), vs.LINEAR_STORE, None)
    _check_stage(_f64(st["qkv"]), ref, slack, "stage qkv")
    ref = oracle.frame_prefill(to_f64(host["q"]), to_f64(hk[:L]) if L else None, to_f64(hv[:L]) if L else None,
                               to_f64(host["k"]), to_f64(host["v"]), scale32(s))
    check_close(st["a"], ref, "bf16", "stage attention", absolute=False)
    ref, slack = _ref_linear(host["a"].view(T, -1), w["w_o"], vs.LINEAR_RESIDUAL, h)
    _check_stage(_f64(st["h1"]), ref, slack, "stage output projection + residual")
    _check_stage(_f64(st["x2"]), oracle.rmsnorm(to_f64(host["h1"]), to_f64(w["norm2"]), eps32), 1e-7, "stage norm2")
    gu = torch.stack([w["w_gate"], w["w_up"]], dim=1).reshape(2 * F, d)
    ref, slack = _ref_linear(host["x2"], gu, vs.LINEAR_GATED, None)
    _check_stage(_f64(st["act"]), ref, slack, "stage gated feed-forward")
    ref, slack = _ref_linear(host["act"], w["w_down"], vs.LINEAR_RESIDUAL, host["h1"])
    _check_stage(_f64(st["out"]), ref, slack, "stage down projection + residual")
    # end to end
    Href, Kf, Vf = oracle.decoder_layer(to_f64(h), to_f64(w["norm1"]), to_f64(w["w_q"]), to_f64(w["w_k"]), to_f64(w["w_v"]),
                                        to_f64(w["w_o"]), to_f64(w["norm2"]), to_f64(w["w_gate"]), to_f64(w["w_up"]),
                                        to_f64(w["w_down"]), eps32, to_f64(hk[:L]) if L else None,
                                        to_f64(hv[:L]) if L else None, s.n_q_heads, s.n_kv_heads, s.head_dim, scale32(s))
    got = _f64(out)
    err = np.abs(got - Href)
    rms = float(np.sqrt(np.mean(Href ** 2)))
    use = float((err / (2.0 ** -7 * np.abs(Href) + 3.5e-2 * rms)).max())
    print(f"[parity] layer T={T} d={d} F={F} L={L}: max-abs {err.max():.2e} mean/rms {err.mean() / rms:.1e} gate-use {use:.2f}")
    assert use <= 1.0 and err.mean() <= 1e-2 * rms
    # the appended row: its own rounding plus the rounding of x1 carried through the projection
    # (~1.6e-3 rms of the row's size; slack 1e-2 rms, six such sigmas)
    _check_stage(_f64(cache.k[L]), Kf[T - 1], 1e-2 * float(np.sqrt(np.mean(Kf ** 2))), "carrier K row, end to end")
    _check_stage(_f64(cache.v[L]), Vf[T - 1], 1e-2 * float(np.sqrt(np.mean(Vf ** 2))), "carrier V row, end to end")


def test_decoder_layer_7b_shape_two_frames():
    """Two frames through one layer at the 7B backbone's sizes: the fused call equals the chain of
    entry points bit for bit, frame after frame (the second sees the first one's carrier), and the
    stages of the chain are held to the oracle on sampled features."""
    s, d, F, T, L, eps = QW, 3584, 18944, 170, 700, 1e-6
    w = layer_weights(51, s, d, F)
    pk = _pack(w)
    hk, hv = cache_rows(53, s, L, 0.5)
    weights = vs.LayerWeights(pk["norm1"], pk["w_qkv"], pk["w_o"], pk["norm2"], pk["w_gate_up"], pk["w_down"], eps=eps)
    sh = vs_shape(s)
    cache, cache2 = _cache(s, hk, hv, L, L + 2), _cache(s, hk, hv, L, L + 2)
    ws = torch.empty(vs.layer_workspace_bytes(sh, weights, T), dtype=torch.uint8, device=DEV)
    vs.workspace_init(sh, ws)
    rng = np.random.default_rng(9)
    eps32 = float(np.float32(eps))
    for f in range(2):
        h = hidden_rows(52, T, d, frame=f)
        hd = _dev(h)
        out = torch.full((T, d), float("nan"), dtype=BF, device=DEV)
        vs.frame_decoder_layer(sh, weights, cache, hd, out, ws)
        st = _chain(s, pk, eps, cache2, hd, T, d, F)
        assert torch.equal(out, st["out"]), f"frame {f}: fused layer differs from the chain"
        assert cache.len == L + f + 1 and torch.equal(cache.k, cache2.k) and torch.equal(cache.v, cache2.v)
        host = {k_: v_.cpu() for k_, v_ in st.items()}
        _check_stage(_f64(st["x1"]), oracle.rmsnorm(to_f64(h), to_f64(w["norm1"]), eps32), 1e-7, f"frame {f} norm1")
        cols = np.unique(rng.integers(0, 4608, 200))
        ref, slack = _ref_linear(host["x1"], torch.cat([w["w_q"], w["w_k"], w["w_v"]]), vs.LINEAR_STORE, None, cols)
        _check_stage(_f64(st["qkv"])[:, cols], ref, slack, f"frame {f} qkv")
        Lnow = L + f
        kc, vc = to_f64(cache2.k[:Lnow].cpu()), to_f64(cache2.v[:Lnow].cpu())
        ref = oracle.frame_prefill(to_f64(host["q"]), kc, vc, to_f64(host["k"]), to_f64(host["v"]), scale32(s))
        check_close(st["a"], ref, "bf16", f"frame {f} attention", absolute=False)
        cols = np.unique(rng.integers(0, d, 200))
        ref, slack = _ref_linear(host["a"].view(T, -1), w["w_o"], vs.LINEAR_RESIDUAL, h, cols)
        _check_stage(_f64(st["h1"])[:, cols], ref, slack, f"frame {f} output projection")
        _check_stage(_f64(st["x2"]), oracle.rmsnorm(to_f64(host["h1"]), to_f64(w["norm2"]), eps32), 1e-7, f"frame {f} norm2")
        cols = np.unique(rng.integers(0, F, 200))
        gu = torch.stack([w["w_gate"], w["w_up"]], dim=1).reshape(2 * F, d)
        ref, slack = _ref_linear(host["x2"], gu, vs.LINEAR_GATED, None, cols)
        _check_stage(_f64(st["act"])[:, cols], ref, slack, f"frame {f} gated feed-forward")
        cols = np.unique(rng.integers(0, d, 200))
        ref, slack = _ref_linear(host["act"], w["w_down"], vs.LINEAR_RESIDUAL, host["h1"], cols)
        _check_stage(_f64(st["out"])[:, cols], ref, slack, f"frame {f} down projection")


def test_decoder_layer_reports_a_full_cache_before_any_launch():
    s, d, F, T = AttnShape(4, 4, 128, "bf16"), 256, 704, 8
    pk = _pack(layer_weights(61, s, d, F))
    weights = vs.LayerWeights(pk["norm1"], pk["w_qkv"], pk["w_o"], pk["norm2"], pk["w_gate_up"], pk["w_down"])
    sh = vs_shape(s)
    hk, hv = cache_rows(62, s, 4, 0.5)
    cache = _cache(s, hk, hv, 4, 4)
    ws = torch.empty(vs.layer_workspace_bytes(sh, weights, T), dtype=torch.uint8, device=DEV)
    vs.workspace_init(sh, ws)
    out = torch.full((T, d), 7.0, dtype=BF, device=DEV)
    with pytest.raises(vs.VSError) as e:
        vs.frame_decoder_layer(sh, weights, cache, _dev(hidden_rows(63, T, d)), out, ws)
    torch.cuda.synchronize()
    assert "capacity" in str(e.value).lower() and cache.len == 4 and torch.all(out == 7.0)


def test_decoder_layer_adds_the_split_k_shares_inside_the_launch_or_not_same_bits():
    """Inside the layer the split-K shares of a product are added by the workgroups of a block
    together, in the multiplying launch (they wait for the last of them a bounded number of looks);
    with tuning value 2 a second kernel adds them, with value 4 the waiting workgroups give up at
    once: the first two give the same bits, the third reports (VS_ERR_PLACEMENT on the next call)
    and the calls after it, which use the second kernel, give the same bits again."""
    s, d, F, T, L = QW, 3584, 2048, 170, 300
    pk = _pack(layer_weights(71, s, d, F))
    weights = vs.LayerWeights(pk["norm1"], pk["w_qkv"], pk["w_o"], pk["norm2"], pk["w_gate_up"], pk["w_down"])
    sh = vs_shape(s)
    hk, hv = cache_rows(72, s, L, 0.5)
    hd = _dev(hidden_rows(73, T, d))
    ws = torch.empty(vs.layer_workspace_bytes(sh, weights, T), dtype=torch.uint8, device=DEV)
    vs.workspace_init(sh, ws)

    def run():
        cache = _cache(s, hk, hv, L, L + 1)
        out = torch.full((T, d), float("nan"), dtype=BF, device=DEV)
        vs.frame_decoder_layer(sh, weights, cache, hd, out, ws)
        torch.cuda.synchronize()
        return out

    inside = run()
    assert bool(torch.isfinite(inside.float()).all())
    try:
        vs.set_tuning(vs.TUNE_PREFILL_MERGE, 2)
        assert torch.equal(run(), inside), "second-kernel addition differs"
        vs.set_tuning(vs.TUNE_PREFILL_MERGE, 0)
        assert torch.equal(run(), inside)
        vs.set_tuning(vs.TUNE_PREFILL_MERGE, 4)
        run()                                   # ends; its output is incomplete
        vs.set_tuning(vs.TUNE_PREFILL_MERGE, 0)
        with pytest.raises(vs.VSError) as err:
            run()
        assert err.value.code == 8
        for _ in range(2):                      # second kernels from now on
            assert torch.equal(run(), inside)
    finally:
        vs.set_tuning(vs.TUNE_PREFILL_MERGE, 0)
        vs.workspace_init(sh, ws)               # probes the device again: merging inside is back
    assert torch.equal(run(), inside)
