"""Seeded draws.  Every tensor is drawn on the host in fp32 from N(0,1), multiplied by
`sigma`, and rounded once (RNE) to the config's storage type; those bytes are what both
the GPU and the oracle see.  Each tensor has a seed of its own, a function of
(config seed, tensor kind, frame/step, layer), so any (frame, layer) can be drawn
without replaying the stream."""
import numpy as np
import torch

_KIND = {"cache_k": 1, "cache_v": 2, "q": 3, "k_f": 4, "v_f": 5, "e": 6,
         "dq": 7, "dk": 8, "dv": 9, "lens": 10, "h": 11, "w_q": 12, "w_k": 13, "w_v": 14, "w_o": 15,
         "w_gate": 16, "w_up": 17, "w_down": 18, "norm1": 19, "norm2": 20}

_TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


def _seed(base, kind, a=0, b=0):
    """One seed per (config seed, tensor kind, frame/step, layer).  The fields are packed and then
    mixed (the 64-bit finaliser of splitmix64), because torch's host generator keys its stream on
    the low 32 bits of the seed alone: unmixed, tensors that differ only in the high fields would
    share their draws."""
    x = ((int(base) & 0xFFFF) << 45) | (_KIND[kind] << 40) | ((int(a) & 0xFFFFF) << 16) | (int(b) & 0xFFFF)
    m = (1 << 64) - 1
    x = (x + 0x9E3779B97F4A7C15) & m
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & m
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & m
    return (x ^ (x >> 31)) & 0x7FFFFFFFFFFFFFFF


def draw(seed, shape, sigma, dtype):
    """N(0,1)*sigma on the host, fp32 draw, rounded once to `dtype` ("f32"/"bf16")."""
    g = torch.Generator(device="cpu").manual_seed(int(seed))
    x = torch.randn(tuple(shape), generator=g, dtype=torch.float32)
    if sigma != 1.0:
        x = x * float(sigma)
    return x.to(_TORCH_DTYPE[dtype]).contiguous()


def to_f64(t):
    """Exact upcast of a host tensor (fp32 or bf16) to a numpy float64 array."""
    return t.detach().cpu().to(torch.float64).numpy()


def cache_rows(base_seed, shape, rows, sigma, layer=0, stream=0):
    """Retained K/V rows [rows][Hkv][D] of one layer (prefix + carriers; all synthetic)."""
    dims = (rows, shape.n_kv_heads, shape.head_dim)
    k = draw(_seed(base_seed, "cache_k", stream, layer), dims, sigma, shape.dtype)
    v = draw(_seed(base_seed, "cache_v", stream, layer), dims, sigma, shape.dtype)
    return k, v


def frame_inputs(base_seed, shape, n_tokens, sigma, frame=0, layer=0, q_gain=1.0):
    """Q [T][Hq][D], K_f/V_f [T][Hkv][D] of one frame run (visual tokens then the carrier).
    q_gain > 1 gives the 'peaked' variant whose softmax is far from uniform."""
    q = draw(_seed(base_seed, "q", frame, layer), (n_tokens, shape.n_q_heads, shape.head_dim),
             sigma * q_gain, shape.dtype)
    k = draw(_seed(base_seed, "k_f", frame, layer), (n_tokens, shape.n_kv_heads, shape.head_dim),
             sigma, shape.dtype)
    v = draw(_seed(base_seed, "v_f", frame, layer), (n_tokens, shape.n_kv_heads, shape.head_dim),
             sigma, shape.dtype)
    return q, k, v


def decode_lengths(base_seed, streams, lo, hi, extra):
    """Ragged retained lengths: uniform integer in [lo, hi] per stream, plus `extra` text rows."""
    # (numpy's generator uses all 64 bits of its seed: the plain packing of (seed, kind) is kept here, and with it
    # the lengths that earlier measurements of this configuration were taken on)
    rng = np.random.default_rng(((int(base_seed) & 0xFFFF) << 44) | (_KIND["lens"] << 40))
    return (rng.integers(lo, hi + 1, size=streams).astype(np.int64) + int(extra)).tolist()


def decode_step_inputs(base_seed, shape, streams, sigma, step=0, layer=0, q_gain=1.0):
    """q [S][Hq][D], k_new/v_new [S][Hkv][D] of one decode step of one layer."""
    q = draw(_seed(base_seed, "dq", step, layer), (streams, shape.n_q_heads, shape.head_dim),
             sigma * q_gain, shape.dtype)
    k = draw(_seed(base_seed, "dk", step, layer), (streams, shape.n_kv_heads, shape.head_dim),
             sigma, shape.dtype)
    v = draw(_seed(base_seed, "dv", step, layer), (streams, shape.n_kv_heads, shape.head_dim),
             sigma, shape.dtype)
    return q, k, v


def cfg1_inputs(cfg):
    """The tiny fp32 case: one generator, drawn in the fixed order
    K_c, V_c, E, Q, K_f, V_f (all N(0,1))."""
    s = cfg["shape"]
    g = torch.Generator(device="cpu").manual_seed(int(cfg["seed"]))
    L, N, T = cfg["prefix"], cfg["n_visual"], cfg["n_visual"] + 1

    def rn(*dims):
        return torch.randn(dims, generator=g, dtype=torch.float32).contiguous()

    k_c = rn(L, s.n_kv_heads, s.head_dim)
    v_c = rn(L, s.n_kv_heads, s.head_dim)
    e = rn(N, cfg["hidden"])
    q = rn(T, s.n_q_heads, s.head_dim)
    k_f = rn(T, s.n_kv_heads, s.head_dim)
    v_f = rn(T, s.n_kv_heads, s.head_dim)
    return dict(k_c=k_c, v_c=v_c, e=e, q=q, k_f=k_f, v_f=v_f)


def carrier_embeddings(seed, n, d, dtype):
    """Embeddings [n][d] of the carriers of a slowly changing scene with cuts: neighbours are
    similar, as the pooled embeddings of consecutive video frames are (synthetic stand-in)."""
    g = torch.Generator(device="cpu").manual_seed(int(seed))
    e = torch.empty((n, d), dtype=torch.float32)
    cur = torch.randn(d, generator=g)
    for t in range(n):
        if t % 11 == 10:
            cur = torch.randn(d, generator=g)  # a cut
        step = 0.2 + 0.8 * float(torch.rand((), generator=g))
        cur = 0.8 * cur + 0.6 * step * torch.randn(d, generator=g)
        e[t] = cur
    return e.to(_TORCH_DTYPE[dtype]).contiguous()


def hidden_rows(base_seed, n_tokens, d_model, sigma=1.0, frame=0, layer=0, dtype="bf16"):
    """Hidden states [T][d] of one frame run entering a decoder layer (synthetic)."""
    return draw(_seed(base_seed, "h", frame, layer), (n_tokens, d_model), sigma, dtype)


def layer_weights(base_seed, shape, d_model, d_ff, layer=0, dtype="bf16"):
    """Random-init weights of one decoder layer, one row per output feature: w_q [Hq D][d], w_k, w_v
    [Hkv D][d], w_o [d][Hq D], w_gate, w_up [F][d], w_down [d][F], each N(0, 1/fan_in) so that
    activations keep the size of their inputs; the two norm gains are 1 + N(0, 0.1^2)."""
    nq, nk = shape.n_q_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim
    dims = {"w_q": (nq, d_model), "w_k": (nk, d_model), "w_v": (nk, d_model), "w_o": (d_model, nq),
            "w_gate": (d_ff, d_model), "w_up": (d_ff, d_model), "w_down": (d_model, d_ff)}
    w = {name: draw(_seed(base_seed, name, 0, layer), dim, dim[1] ** -0.5, dtype) for name, dim in dims.items()}
    for name in ("norm1", "norm2"):
        g = torch.Generator(device="cpu").manual_seed(_seed(base_seed, name, 0, layer))
        w[name] = (1.0 + 0.1 * torch.randn(d_model, generator=g, dtype=torch.float32)).to(_TORCH_DTYPE[dtype]).contiguous()
    return w
