"""Seeded draws.  Every tensor is drawn on the host in fp32 from N(0,1), multiplied by
`sigma`, and rounded once (RNE) to the config's storage type; those bytes are what both
the GPU and the oracle see.  Each tensor has a seed of its own, a function of
(config seed, tensor kind, frame/step, layer), so any (frame, layer) can be drawn
without replaying the stream."""
import numpy as np
import torch

_KIND = {"cache_k": 1, "cache_v": 2, "q": 3, "k_f": 4, "v_f": 5, "e": 6,
         "dq": 7, "dk": 8, "dv": 9, "lens": 10}

_TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


def _seed(base, kind, a=0, b=0):
    return ((int(base) & 0xFFFF) << 44) | (_KIND[kind] << 40) | ((int(a) & 0xFFFFF) << 16) | (int(b) & 0xFFFF)


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
    rng = np.random.default_rng(_seed(base_seed, "lens"))
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
