"""Pins for an implementation of the VideoScan attention path.

Each pin takes an `impl` exposing the oracle's five functions and raises
AssertionError if the implementation violates something the paper or the
mathematics fixes (Eq. 1, Section 3.1; carrier last, Section 3.2; mean pool,
prefill/discard/decode, Section 3.3).  None of the expected values here comes
from the implementation under test.  The same pins run against the real oracle
(must pass) and against deliberately broken variants of an independent numpy
evaluation (each must fail at least one pin) so that the pins are known to bite.
"""
import json
import math
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


# ----------------------------------------------------------------------------
# independent brute force: pure Python, lists, math.fsum/math.exp, no max shift
# ----------------------------------------------------------------------------
def brute_attention(Q, K, V, vis, scale):
    Tq, Hq, D = len(Q), len(Q[0]), len(Q[0][0])
    Hkv = len(K[0])
    G = Hq // Hkv
    out = [[[0.0] * D for _ in range(Hq)] for _ in range(Tq)]
    probs = [[[0.0] * len(K) for _ in range(Tq)] for _ in range(Hq)]
    for i in range(Tq):
        for h in range(Hq):
            g = h // G
            e = []
            for j in range(vis[i]):
                dot = math.fsum(Q[i][h][d] * K[j][g][d] for d in range(D))
                e.append(math.exp(scale * dot))
            tot = math.fsum(e)
            for j in range(vis[i]):
                probs[h][i][j] = e[j] / tot
            for d in range(D):
                out[i][h][d] = math.fsum(probs[h][i][j] * V[j][g][d] for j in range(vis[i]))
    return out, probs


def _rng(seed):
    return np.random.default_rng(seed)


def _close(a, b, tol, what):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    assert a.shape == b.shape, f"{what}: shape {a.shape} vs {b.shape}"
    err = float(np.max(np.abs(a - b))) if a.size else 0.0
    assert err <= tol, f"{what}: max-abs error {err:.3e} > {tol:.1e}"


# ----------------------------------------------------------------------------
# attention core
# ----------------------------------------------------------------------------
def pin_golden_rational(impl):
    with open(os.path.join(GOLDEN, "eq1_rational_softmax.json")) as f:
        g = json.load(f)
    keys = np.array([[[math.log(a), math.log(b)]] for a, b in zip(g["a"], g["b"])])  # [3][1][2]
    vals = np.array(g["v"], dtype=np.float64)[:, None, :]
    L = g["n_cache_rows"]
    Q = np.array(g["q"], dtype=np.float64)
    O, P = impl.frame_prefill(Q, keys[:L], vals[:L], keys[L:], vals[L:], g["scale"], return_probs=True)
    _close(O, g["expected_out"], 1e-13, "golden rational softmax, outputs")
    _close(P[0], g["expected_probs_head0"], 1e-14, "golden probabilities head 0")
    _close(P[1], g["expected_probs_head1"], 1e-14, "golden probabilities head 1")


def pin_uniform_scores_mean_of_visible(impl):
    """Q = 0 makes every score equal, so row i is the plain mean of its L+i+1 visible V rows:
    an exact count of the mask."""
    r = _rng(10)
    L, T, Hq, Hkv, D = 5, 7, 4, 2, 8
    Kc, Vc = r.normal(size=(L, Hkv, D)), r.normal(size=(L, Hkv, D))
    Kf, Vf = r.normal(size=(T, Hkv, D)), r.normal(size=(T, Hkv, D))
    O = impl.frame_prefill(np.zeros((T, Hq, D)), Kc, Vc, Kf, Vf, 0.37)
    Vall = np.concatenate([Vc, Vf])
    for i in range(T):
        for h in range(Hq):
            _close(O[i, h], Vall[: L + i + 1, h // (Hq // Hkv)].mean(axis=0), 1e-14,
                   f"uniform scores row {i} head {h}")


def pin_single_key(impl):
    """Empty cache: frame row 0 sees one key, so its output is that V row exactly; likewise a
    decode step into an empty cache returns v_new."""
    r = _rng(11)
    T, Hq, Hkv, D = 3, 6, 3, 4
    Q = r.normal(size=(T, Hq, D))
    Kf, Vf = r.normal(size=(T, Hkv, D)), r.normal(size=(T, Hkv, D))
    O = impl.frame_prefill(Q, None, None, Kf, Vf, 0.5)
    for h in range(Hq):
        assert np.array_equal(O[0, h], Vf[0, h // 2]), "single visible key must return its V row exactly"
    Kc, Vc = np.zeros((4, Hkv, D)), np.zeros((4, Hkv, D))
    o, ln = impl.decode(Q[0], Kc, Vc, 0, Kf[1], Vf[1], 0.5)
    assert ln == 1
    for h in range(Hq):
        assert np.array_equal(o[h], Vf[1, h // 2])


def pin_one_hot_limit(impl):
    """One key aligned with q and scaled up: softmax collapses onto it."""
    r = _rng(12)
    R, Hq, Hkv, D = 9, 2, 1, 16
    Q = r.normal(size=(1, Hq, D))
    Q[0, 1] = Q[0, 0]  # both heads share the kv head and the query direction
    K, V = r.normal(size=(R, Hkv, D)), r.normal(size=(R, Hkv, D))
    K[4, 0] = 400.0 * Q[0, 0] / np.linalg.norm(Q[0, 0])
    O = impl.attention(Q, K, V, np.array([R]), 1.0)
    _close(O[0, 0], V[4, 0], 1e-12, "one-hot limit")


def pin_row_stochastic_and_masked_zero(impl):
    r = _rng(13)
    L, T, Hq, Hkv, D = 4, 6, 4, 2, 8
    args = [r.normal(size=s) for s in [(T, Hq, D), (L, Hkv, D), (L, Hkv, D), (T, Hkv, D), (T, Hkv, D)]]
    _, P = impl.frame_prefill(*args, 0.35, return_probs=True)
    assert P.shape == (Hq, T, L + T)
    assert np.all(P >= 0.0)
    _close(P.sum(axis=-1), np.ones((Hq, T)), 1e-14, "row sums")
    for i in range(T):
        assert np.all(P[:, i, L + i + 1:] == 0.0), "masked keys must carry exactly zero weight"
        assert np.all(P[:, i, : L + i + 1] > 0.0)


def pin_brute_force_tiny(impl):
    """Against the pure-Python evaluation, over several tiny shapes incl. GQA and D odd."""
    for seed, (L, T, Hq, Hkv, D) in enumerate([(2, 3, 2, 1, 4), (0, 2, 2, 2, 3), (1, 1, 4, 2, 2),
                                               (2, 3, 6, 2, 1)]):
        r = _rng(100 + seed)
        Q = r.normal(size=(T, Hq, D))
        Kc, Vc = r.normal(size=(L, Hkv, D)), r.normal(size=(L, Hkv, D))
        Kf, Vf = r.normal(size=(T, Hkv, D)), r.normal(size=(T, Hkv, D))
        scale = 0.7
        O, P = impl.frame_prefill(Q, Kc, Vc, Kf, Vf, scale, return_probs=True)
        Kall, Vall = np.concatenate([Kc, Kf]), np.concatenate([Vc, Vf])
        bo, bp = brute_attention(Q.tolist(), Kall.tolist(), Vall.tolist(),
                                 [L + i + 1 for i in range(T)], scale)
        _close(O, bo, 1e-13, f"brute force outputs, case {seed}")
        _close(P, bp, 1e-14, f"brute force probabilities, case {seed}")


def pin_library_second_opinion(impl):
    """With the causal frame mask written as a boolean matrix, a library softmax-attention in fp64
    must agree (second opinion only, on a mid-size case spanning GQA groups)."""
    import torch
    r = _rng(14)
    L, T, Hq, Hkv, D = 37, 23, 8, 2, 32
    Q = r.normal(size=(T, Hq, D))
    Kc, Vc = r.normal(size=(L, Hkv, D)), r.normal(size=(L, Hkv, D))
    Kf, Vf = r.normal(size=(T, Hkv, D)), r.normal(size=(T, Hkv, D))
    scale = D ** -0.5
    O = impl.frame_prefill(Q, Kc, Vc, Kf, Vf, scale)
    G = Hq // Hkv
    Kall = torch.from_numpy(np.concatenate([Kc, Kf])).repeat_interleave(G, dim=1)
    Vall = torch.from_numpy(np.concatenate([Vc, Vf])).repeat_interleave(G, dim=1)
    mask = torch.zeros(T, L + T, dtype=torch.bool)
    for i in range(T):
        mask[i, : L + i + 1] = True
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q).permute(1, 0, 2), Kall.permute(1, 0, 2), Vall.permute(1, 0, 2),
        attn_mask=mask, scale=scale).permute(1, 0, 2).numpy()
    _close(O, ref, 1e-13, "library second opinion")


# ----------------------------------------------------------------------------
# mask, GQA, invariances
# ----------------------------------------------------------------------------
def pin_causality(impl):
    r = _rng(15)
    L, T, Hq, Hkv, D = 3, 6, 2, 1, 8
    Q = r.normal(size=(T, Hq, D))
    Kc, Vc = r.normal(size=(L, Hkv, D)), r.normal(size=(L, Hkv, D))
    Kf, Vf = r.normal(size=(T, Hkv, D)), r.normal(size=(T, Hkv, D))
    base = impl.frame_prefill(Q, Kc, Vc, Kf, Vf, 0.4)
    cut = 3
    Kf2, Vf2 = Kf.copy(), Vf.copy()
    Kf2[cut + 1:] += 5.0
    Vf2[cut + 1:] -= 7.0
    pert = impl.frame_prefill(Q, Kc, Vc, Kf2, Vf2, 0.4)
    assert np.array_equal(base[: cut + 1], pert[: cut + 1]), "future frame rows leaked into earlier rows"
    assert np.all(np.abs(base[cut + 1:] - pert[cut + 1:]).max(axis=(1, 2)) > 1e-3)
    # every row sees every cache row
    Vc2 = Vc.copy()
    Vc2[1] += 3.0
    pert = impl.frame_prefill(Q, Kc, Vc2, Kf, Vf, 0.4)
    assert np.all(np.abs(base - pert).max(axis=(1, 2)) > 1e-6), "a cache row is invisible to some frame row"
    # the row itself is visible (diagonal)
    Vf3 = Vf.copy()
    Vf3[2] += 3.0
    pert = impl.frame_prefill(Q, Kc, Vc, Kf, Vf3, 0.4)
    assert np.abs(base[2] - pert[2]).max() > 1e-6, "a frame row must see itself"
    assert np.array_equal(base[:2], pert[:2])


def pin_carrier_row_is_unmasked_attention(impl):
    """The carrier is last in the run, so its output is plain attention over all L+T rows."""
    r = _rng(16)
    L, T, Hq, Hkv, D = 4, 5, 4, 2, 8
    Q = r.normal(size=(T, Hq, D))
    Kc, Vc = r.normal(size=(L, Hkv, D)), r.normal(size=(L, Hkv, D))
    Kf, Vf = r.normal(size=(T, Hkv, D)), r.normal(size=(T, Hkv, D))
    O = impl.frame_prefill(Q, Kc, Vc, Kf, Vf, 0.3)
    Kall, Vall = np.concatenate([Kc, Kf]), np.concatenate([Vc, Vf])
    for h in range(Hq):
        g = h // 2
        z = 0.3 * Kall[:, g] @ Q[T - 1, h]
        w = np.exp(z - z.max())
        _close(O[T - 1, h], (w / w.sum()) @ Vall[:, g], 1e-14, "carrier row")


def pin_gqa_equals_replicated_mha(impl):
    r = _rng(17)
    R, Tq, Hq, Hkv, D = 11, 4, 6, 2, 8
    Q, K, V = r.normal(size=(Tq, Hq, D)), r.normal(size=(R, Hkv, D)), r.normal(size=(R, Hkv, D))
    vis = np.array([3, 11, 7, 1])
    a = impl.attention(Q, K, V, vis, 0.4)
    b = impl.attention(Q, np.repeat(K, 3, axis=1), np.repeat(V, 3, axis=1), vis, 0.4)
    _close(a, b, 1e-15, "GQA vs replicated MHA")
    # and the grouping is by consecutive query heads: heads 0..2 read kv head 0
    V2 = V.copy()
    V2[:, 1] += 1.0
    c = impl.attention(Q, K, V2, vis, 0.4)
    assert np.array_equal(a[:, :3], c[:, :3]) and np.all(np.abs(a[:, 3:] - c[:, 3:]) > 0.5)


def pin_invariances(impl):
    r = _rng(18)
    L, T, Hq, Hkv, D = 6, 4, 2, 1, 8
    Q = r.normal(size=(T, Hq, D))
    Kc, Vc = r.normal(size=(L, Hkv, D)), r.normal(size=(L, Hkv, D))
    Kf, Vf = r.normal(size=(T, Hkv, D)), r.normal(size=(T, Hkv, D))
    base = impl.frame_prefill(Q, Kc, Vc, Kf, Vf, 0.4)
    # key shift: adds a per-row constant to every score
    u = r.normal(size=(D,))
    _close(impl.frame_prefill(Q, Kc + u, Vc, Kf + u, Vf, 0.4), base, 1e-13, "key shift")
    # permutation of cache rows (K and V together)
    perm = r.permutation(L)
    _close(impl.frame_prefill(Q, Kc[perm], Vc[perm], Kf, Vf, 0.4), base, 1e-14, "cache permutation")
    # linear in V
    Vc2, Vf2 = r.normal(size=Vc.shape), r.normal(size=Vf.shape)
    both = impl.frame_prefill(Q, Kc, Vc + Vc2, Kf, Vf + Vf2, 0.4)
    _close(both, base + impl.frame_prefill(Q, Kc, Vc2, Kf, Vf2, 0.4), 1e-14, "linearity in V")
    # convex hull of visible V rows
    Vall = np.concatenate([Vc, Vf])
    for i in range(T):
        lo, hi = Vall[: L + i + 1, 0].min(axis=0), Vall[: L + i + 1, 0].max(axis=0)
        assert np.all(base[i] >= lo - 1e-14) and np.all(base[i] <= hi + 1e-14)
    # the scale matters and is applied to the scores (doubling scale == doubling Q)
    _close(impl.frame_prefill(Q, Kc, Vc, Kf, Vf, 0.8), impl.frame_prefill(2 * Q, Kc, Vc, Kf, Vf, 0.4),
           1e-13, "scale acts on scores")
    assert np.abs(impl.frame_prefill(Q, Kc, Vc, Kf, Vf, 0.8) - base).max() > 1e-3


def pin_transposition_sensitive(impl):
    """Non-square, non-symmetric case with a closed form: scores depend on <q,k> only.
    K rows are multiples of one direction u, so z_j = scale*c_j*<q,u>; V is distinct from K."""
    r = _rng(19)
    R, D = 5, 3
    u = np.array([1.0, -2.0, 0.5])
    c = np.array([0.3, -1.0, 2.0, 0.0, 1.5])
    K = (c[:, None] * u[None, :])[:, None, :]
    V = r.normal(size=(R, 1, D))
    q = np.array([[[0.2, 0.1, -0.4]]])
    z = 0.9 * c * float(q[0, 0] @ u)
    w = np.exp(z) / np.exp(z).sum()
    _close(impl.attention(q, K, V, np.array([R]), 0.9)[0, 0], w @ V[:, 0], 1e-14, "closed-form scores")


# ----------------------------------------------------------------------------
# compaction, streaming, decode, pool
# ----------------------------------------------------------------------------
def pin_compaction(impl):
    r = _rng(20)
    P0, F, T, Hkv, D = 3, 5, 4, 2, 4
    cap = P0 + F
    Kc, Vc = np.full((cap, Hkv, D), np.nan), np.full((cap, Hkv, D), np.nan)
    Kc[:P0], Vc[:P0] = r.normal(size=(P0, Hkv, D)), r.normal(size=(P0, Hkv, D))
    ln = P0
    frames = []
    for f in range(F):
        Kf, Vf = r.normal(size=(T, Hkv, D)), r.normal(size=(T, Hkv, D))
        before_k, before_v = Kc[:ln].copy(), Vc[:ln].copy()
        row, new_len = impl.compact_append(Kc, Vc, ln, Kf, Vf)
        assert row == P0 + f and new_len == ln + 1, "appended row index / length sequence"
        assert np.array_equal(Kc[:ln], before_k) and np.array_equal(Vc[:ln], before_v), "older rows touched"
        assert np.array_equal(Kc[row], Kf[T - 1]) and np.array_equal(Vc[row], Vf[T - 1]), "carrier row bytes"
        assert np.all(np.isnan(Kc[new_len:])) and np.all(np.isnan(Vc[new_len:])), "wrote past the new row"
        frames.append((Kf, Vf))
        ln = new_len
    assert ln == P0 + F  # retained length = prefix + frames seen
    # none of the visual rows is retained
    for Kf, Vf in frames:
        for t in range(T - 1):
            assert not any(np.array_equal(Kc[j], Kf[t]) for j in range(ln))
    # full cache -> capacity error, nothing changes
    snap = Kc.copy()
    try:
        impl.compact_append(Kc, Vc, ln, *frames[0])
        raise AssertionError("append into a full cache must fail")
    except AssertionError:
        raise
    except Exception:
        pass
    assert np.array_equal(Kc, snap)
    # explicit carrier index other than last
    Kc2, Vc2 = np.zeros((2, Hkv, D)), np.zeros((2, Hkv, D))
    row, _ = impl.compact_append(Kc2, Vc2, 0, *frames[1], carrier=1)
    assert row == 0 and np.array_equal(Kc2[0], frames[1][0][1]) and np.array_equal(Vc2[0], frames[1][1][1])


def pin_streaming_equals_one_shot(impl):
    """F frames with compaction, then one more frame == that frame against a cache built directly
    as [prefix | carrier rows]."""
    r = _rng(21)
    P0, F, T, Hq, Hkv, D = 2, 4, 3, 2, 1, 4
    cap = P0 + F
    Kc, Vc = np.zeros((cap, Hkv, D)), np.zeros((cap, Hkv, D))
    pk, pv = r.normal(size=(P0, Hkv, D)), r.normal(size=(P0, Hkv, D))
    Kc[:P0], Vc[:P0] = pk, pv
    ln = P0
    carriers_k, carriers_v = [], []
    for f in range(F):
        Kf, Vf = r.normal(size=(T, Hkv, D)), r.normal(size=(T, Hkv, D))
        impl.frame_prefill(r.normal(size=(T, Hq, D)), Kc[:ln], Vc[:ln], Kf, Vf, 0.5)
        _, ln = impl.compact_append(Kc, Vc, ln, Kf, Vf)
        carriers_k.append(Kf[T - 1])
        carriers_v.append(Vf[T - 1])
    Q, Kf, Vf = r.normal(size=(T, Hq, D)), r.normal(size=(T, Hkv, D)), r.normal(size=(T, Hkv, D))
    streamed = impl.frame_prefill(Q, Kc[:ln], Vc[:ln], Kf, Vf, 0.5)
    direct = impl.frame_prefill(Q, np.concatenate([pk, np.stack(carriers_k)]),
                                np.concatenate([pv, np.stack(carriers_v)]), Kf, Vf, 0.5)
    assert np.array_equal(streamed, direct)


def pin_decode(impl):
    r = _rng(22)
    L, Hq, Hkv, D = 7, 4, 2, 8
    cap = L + 2
    Kc, Vc = np.zeros((cap, Hkv, D)), np.zeros((cap, Hkv, D))
    Kc[:L], Vc[:L] = r.normal(size=(L, Hkv, D)), r.normal(size=(L, Hkv, D))
    q, kn, vn = r.normal(size=(Hq, D)), r.normal(size=(Hkv, D)), r.normal(size=(Hkv, D))
    K0, V0 = Kc.copy(), Vc.copy()
    o, ln = impl.decode(q, Kc, Vc, L, kn, vn, 0.4)
    assert ln == L + 1
    assert np.array_equal(Kc[L], kn) and np.array_equal(Vc[L], vn), "new row goes to index old-length"
    assert np.array_equal(Kc[:L], K0[:L]) and np.array_equal(Kc[L + 1:], K0[L + 1:])
    # decode == prefill with a one-token run against the old cache
    pre = impl.frame_prefill(q[None], K0[:L], V0[:L], kn[None], vn[None], 0.4)
    _close(o, pre[0], 1e-15, "decode vs one-token prefill")
    # the new row is attended to
    o2, _ = impl.decode(q, K0.copy(), V0.copy(), L, kn, vn + 10.0, 0.4)
    assert np.all(np.abs(o2 - o) > 1e-6)
    # without a new row: plain attention over the L valid rows, rows beyond `len` ignored
    Kc3, Vc3 = K0.copy(), V0.copy()
    Kc3[L:], Vc3[L:] = 99.0, 99.0
    o3, ln3 = impl.decode(q, Kc3, Vc3, L, None, None, 0.4)
    assert ln3 == L
    ref = impl.attention(q[None], K0[:L], V0[:L], np.array([L]), 0.4)[0]
    _close(o3, ref, 1e-15, "decode without append")


def pin_mean_pool(impl):
    with open(os.path.join(GOLDEN, "mean_pool_integers.json")) as f:
        g = json.load(f)
    assert np.array_equal(impl.mean_pool(np.array(g["e"], dtype=np.float64)), np.array(g["expected"]))
    r = _rng(23)
    row = r.normal(size=(17,))
    _close(impl.mean_pool(np.tile(row, (9, 1))), row, 1e-15, "constant rows")
    assert np.array_equal(impl.mean_pool(row[None]), row), "N = 1 is the identity"
    E, W = r.normal(size=(49, 32)), r.normal(size=(32, 8))
    _close(impl.mean_pool(E) @ W, impl.mean_pool(E @ W), 1e-13, "pool commutes with a linear map")
    _close(impl.mean_pool(E), E.mean(axis=0, dtype=np.float64), 1e-15, "numpy mean")
    # pooled over rows, not columns; and divided by N (not N-1, not d)
    E2 = np.arange(12, dtype=np.float64).reshape(3, 4)
    assert np.array_equal(impl.mean_pool(E2), np.array([4.0, 5.0, 6.0, 7.0]))


def pin_memory_bank(impl):
    """Section 3.3, memory mechanism: at capacity the OLDER carrier of the most similar ADJACENT
    pair goes (the incoming carrier is the last element of the sequence); order is kept, the
    incoming carrier becomes the last."""
    # closed form: unit vectors at known angles.  s_i = (cos t_i, sin t_i): cos(s_i, s_j) = cos(t_i - t_j)
    t = np.array([0.0, 1.0, 1.9, 2.0, 3.5, 5.0])           # bank of 5 + incoming at 5.0
    S = np.stack([np.cos(t), np.sin(t)], axis=1)
    v, c = impl.bank_victim(S[:5], S[5])
    _close(c, np.cos(np.diff(t)), 1e-14, "cosines of adjacent pairs, the last pair with the incoming one")
    assert v == 2, "pair (1.9, 2.0) is the most similar one; its OLDER member is index 2"
    # the other reading: similarity to the incoming carrier only
    v1, c1 = impl.bank_victim(S[:5], S[5], 1)
    _close(c1, np.cos(t[:5] - t[5]), 1e-14, "cosines with the incoming carrier")
    assert v1 == int(np.argmax(np.cos(t[:5] - t[5])))
    # cosine, not dot product: scaling any vector changes nothing; a long vector does not win
    r = _rng(31)
    E, e = r.normal(size=(9, 12)), r.normal(size=12)
    v0, c0 = impl.bank_victim(E, e)
    scale = r.uniform(0.1, 50.0, size=(9, 1))
    v2, c2 = impl.bank_victim(E * scale, e * 7.0)
    assert v2 == v0
    _close(c2, c0, 1e-13, "scale invariance")
    # brute force with math.fsum
    seq = np.concatenate([E, e[None]])
    want = []
    for i in range(9):
        a, b = seq[i], seq[i + 1]
        want.append(math.fsum(a * b) / math.sqrt(math.fsum(a * a) * math.fsum(b * b)))
    _close(c0, np.array(want), 1e-14, "brute force cosines")
    assert v0 == int(np.argmax(want))
    # the incoming carrier takes part: a bank of mutually orthogonal vectors and an incoming copy of the last
    E = np.eye(6)[:5] * 3.0
    v, c = impl.bank_victim(E, E[4] * 0.5)
    assert v == 4 and c[4] == 1.0 and np.all(c[:4] == 0.0)
    # ties: the smallest index (the oldest pair)
    E = np.array([[1.0, 0], [1, 0], [0, 1], [0, 1], [1, 1]])
    v, c = impl.bank_victim(E, np.array([-1.0, 0.0]))
    assert c[0] == c[2] == 1.0 and v == 0
    # a zero vector has cosine 0 with everything (and is never not-a-number)
    E = np.array([[0.0, 0], [1, 0], [-1, 0.1]])
    v, c = impl.bank_victim(E, np.array([1.0, 0.0]))
    assert c[0] == 0.0 and np.all(np.isfinite(c)) and v == 0   # the other cosines are negative
    # applying it: append while there is room, then drop / close the gap / new row last
    rows = np.zeros((7, 2, 2))
    rows[0] = -1.0                                            # one row in front that is no carrier
    n = 0
    for k in range(4):
        n = impl.bank_apply(rows, 1, 4, n, -1, np.full((2, 2), 10.0 + k))
    assert n == 4 and np.array_equal(rows[1:5, 0, 0], [10, 11, 12, 13]) and np.all(rows[5:] == 0)
    n = impl.bank_apply(rows, 1, 4, n, 1, np.full((2, 2), 14.0))
    assert n == 4 and np.array_equal(rows[1:5, 0, 0], [10, 12, 13, 14]), "victim 1 dropped, order kept, new last"
    assert np.all(rows[0] == -1.0) and np.all(rows[5:] == 0), "rows outside the bank untouched"
    n = impl.bank_apply(rows, 1, 4, n, 3, np.full((2, 2), 15.0))
    assert np.array_equal(rows[1:5, 0, 0], [10, 12, 13, 15]), "dropping the newest of the bank"
    n = impl.bank_apply(rows, 1, 4, n, 0, np.full((2, 2), 16.0))
    assert np.array_equal(rows[1:5, 0, 0], [12, 13, 15, 16]) and np.all(rows[1:5, 1, 1] == rows[1:5, 0, 0])
    # a stream: the bank never exceeds M and always ends with the newest carrier
    M, d = 5, 8
    bank = np.zeros((M, d))
    ids = np.zeros((M, 1))
    n = 0
    for f in range(20):
        e = r.normal(size=d)
        v = impl.bank_victim(bank, e)[0] if n == M else -1
        n2 = impl.bank_apply(ids, 0, M, n, v, np.array([float(f)]))
        n = impl.bank_apply(bank, 0, M, n, v, e)
        assert n == n2 == min(f + 1, M) and ids[n - 1, 0] == f and np.array_equal(bank[n - 1], e)
        assert np.all(np.diff(ids[:n, 0]) > 0), "arrival order is kept"


def pin_frames_with_semantic_mask(impl):
    """Section 3.4: several frames in one run; a token reaches earlier frames only through their
    carriers (last tokens)."""
    r = _rng(41)
    F, T, Hq, Hkv, D, L = 4, 5, 4, 2, 6, 3
    Q = r.normal(size=(F, T, Hq, D))
    Kf, Vf = r.normal(size=(F, T, Hkv, D)), r.normal(size=(F, T, Hkv, D))
    Kc, Vc = r.normal(size=(L, Hkv, D)), r.normal(size=(L, Hkv, D))
    O = impl.frames_prefill(Q, Kc, Vc, Kf, Vf, 0.5)
    # one frame: the ordinary frame prefill
    _close(impl.frames_prefill(Q[:1], Kc, Vc, Kf[:1], Vf[:1], 0.5)[0], impl.frame_prefill(Q[0], Kc, Vc, Kf[0], Vf[0], 0.5),
           1e-14, "a run of one frame")
    # the run equals streaming: frame by frame, each followed by the carrier compaction
    cap = L + F
    K2, V2 = np.zeros((cap, Hkv, D)), np.zeros((cap, Hkv, D))
    K2[:L], V2[:L] = Kc, Vc
    n = L
    for a in range(F):
        _close(O[a], impl.frame_prefill(Q[a], K2[:n], V2[:n], Kf[a], Vf[a], 0.5), 1e-13, f"frame {a} of the run vs streaming")
        _, n = impl.compact_append(K2, V2, n, Kf[a], Vf[a])
    # brute force of the mask on the flattened run: key (b, j) visible to query (a, i) iff
    # (b == a and j <= i) or (b < a and j == T-1)
    Kall = np.concatenate([Kc, Kf.reshape(F * T, Hkv, D)])
    Vall = np.concatenate([Vc, Vf.reshape(F * T, Hkv, D)])
    for a, i, h in ((0, 0, 0), (1, 2, 3), (3, 4, 1), (2, 0, 2)):
        vis = list(range(L)) + [L + b * T + j for b in range(F) for j in range(T)
                                if (b == a and j <= i) or (b < a and j == T - 1)]
        g = h // (Hq // Hkv)
        z = [0.5 * math.fsum(Q[a, i, h] * Kall[k, g]) for k in vis]
        m = max(z)
        w = [math.exp(x - m) for x in z]
        want = [math.fsum(w[n_] * Vall[k, g, d] for n_, k in enumerate(vis)) / math.fsum(w) for d in range(D)]
        _close(O[a, i, h], np.array(want), 1e-13, f"brute force ({a},{i},{h})")
    # no leak: changing the visual tokens (not the carrier) of frame 1 changes no later frame at all,
    # changing its carrier changes every later frame, and nothing ever changes an earlier frame
    Kp, Vp = Kf.copy(), Vf.copy()
    Kp[1, :T - 1] += 1.0
    Vp[1, :T - 1] -= 2.0
    O2 = impl.frames_prefill(Q, Kc, Vc, Kp, Vp, 0.5)
    assert np.array_equal(O2[0], O[0]) and np.array_equal(O2[2:], O[2:]) and not np.array_equal(O2[1], O[1])
    Kp, Vp = Kf.copy(), Vf.copy()
    Vp[1, T - 1] += 1.0
    O3 = impl.frames_prefill(Q, Kc, Vc, Kp, Vp, 0.5)
    assert np.array_equal(O3[0], O[0]) and np.array_equal(O3[1, :T - 1], O[1, :T - 1])
    assert all(np.abs(O3[a] - O[a]).min() > 0 for a in (2, 3)) and np.abs(O3[1, T - 1] - O[1, T - 1]).min() > 0


def pin_question_after_the_video(impl):
    """Section 3.3, decoding phase: the question's tokens are appended in order, each attends over
    everything up to itself, and all of them stay in the cache for the answer."""
    r = _rng(53)
    L, Tq, Hq, Hkv, D = 6, 5, 4, 2, 6
    cap = L + Tq + 2
    Kc, Vc = r.normal(size=(cap, Hkv, D)), r.normal(size=(cap, Hkv, D))   # rows >= L: junk that must not count
    Q, Kt, Vt = r.normal(size=(Tq, Hq, D)), r.normal(size=(Tq, Hkv, D)), r.normal(size=(Tq, Hkv, D))
    K0, V0 = Kc.copy(), Vc.copy()
    O, n = impl.query_prefill(Q, Kc, Vc, L, Kt, Vt, 0.6)
    assert n == L + Tq
    assert np.array_equal(Kc[L:n], Kt) and np.array_equal(Vc[L:n], Vt), "all question rows stay, in order"
    assert np.array_equal(Kc[:L], K0[:L]) and np.array_equal(Vc[:L], V0[:L])
    assert np.array_equal(Kc[n:], K0[n:]) and np.array_equal(Vc[n:], V0[n:])
    # the same numbers as a causal run over the old rows (the frame prefill, which keeps nothing) ...
    _close(O, impl.frame_prefill(Q, K0[:L], V0[:L], Kt, Vt, 0.6), 1e-14, "question vs causal run")
    # ... and as Tq decoding steps one after the other
    K2, V2, m = K0.copy(), V0.copy(), L
    for j in range(Tq):
        o, m = impl.decode(Q[j], K2, V2, m, Kt[j], Vt[j], 0.6)
        _close(O[j], o, 1e-14, f"question token {j} vs a decoding step")
    assert m == n and np.array_equal(K2, Kc) and np.array_equal(V2, Vc)
    # brute force for a few (token, head) pairs
    for j, h in ((0, 0), (2, 3), (4, 1)):
        g = h // (Hq // Hkv)
        rows_k = [K0[i, g] for i in range(L)] + [Kt[i, g] for i in range(j + 1)]
        rows_v = [V0[i, g] for i in range(L)] + [Vt[i, g] for i in range(j + 1)]
        z = [0.6 * math.fsum(Q[j, h] * k) for k in rows_k]
        mx = max(z)
        w = [math.exp(x - mx) for x in z]
        want = [math.fsum(w[i] * rows_v[i][d] for i in range(len(w))) / math.fsum(w) for d in range(D)]
        _close(O[j, h], np.array(want), 1e-13, f"brute force ({j},{h})")
    # the answer's first decoding step sees every question row
    qd = r.normal(size=(Hq, D))
    o1, _ = impl.decode(qd, Kc.copy(), Vc.copy(), n, None, None, 0.6)
    for j in range(Tq):
        Vp = Vc.copy()
        Vp[L + j] += 3.0
        o2, _ = impl.decode(qd, Kc.copy(), Vp, n, None, None, 0.6)
        assert np.abs(o2 - o1).min() > 0, f"question row {j} is not seen by the answer"
    # a full cache is refused and nothing is touched
    Kf_, Vf_ = K0[:L + Tq - 1].copy(), V0[:L + Tq - 1].copy()
    try:
        impl.query_prefill(Q, Kf_, Vf_, L, Kt, Vt, 0.6)
    except Exception:
        assert np.array_equal(Kf_, K0[:L + Tq - 1]) and np.array_equal(Vf_, V0[:L + Tq - 1])
    else:
        raise AssertionError("a question that does not fit must be refused")


def pin_frame_rows_and_their_projections(impl):
    """Section 3.1 (Q = X W_Q, K = X W_K, V = X W_V) on the frame's rows, the carrier = mean of the
    token embeddings appended last (Sections 3.2, 3.3)."""
    r = _rng(67)
    N, d, Hq, Hkv, D = 5, 7, 4, 2, 3
    n_out = (Hq + 2 * Hkv) * D
    E, W = r.normal(size=(N, d)), r.normal(size=(n_out, d))
    Q, K, V = impl.frame_qkv(E, W, Hq, Hkv, D)
    assert Q.shape == (N + 1, Hq, D) and K.shape == (N + 1, Hkv, D) and V.shape == K.shape
    Y = np.concatenate([Q.reshape(N + 1, -1), K.reshape(N + 1, -1), V.reshape(N + 1, -1)], axis=1)
    # brute force, every entry: feature n of row t is the dot product of X[t] with W's row n
    X = [list(E[t]) for t in range(N)] + [[math.fsum(E[:, k]) / N for k in range(d)]]
    for t in range(N + 1):
        for n in range(n_out):
            assert abs(Y[t, n] - math.fsum(X[t][k] * W[n, k] for k in range(d))) < 1e-13, (t, n)
    # a projection is linear: the carrier's Q/K/V are the means of the tokens' Q/K/V
    _close(Y[N], Y[:N].mean(axis=0), 1e-13, "carrier row vs mean of the projected tokens")
    # weights that pick single input features (not symmetric): outputs are copies of those features,
    # so rows, features and the carrier's place are all visible
    d2, Hq2, Hkv2, D2 = 8, 2, 1, 2          # n_out = 8 = d2
    perm = [3, 0, 7, 1, 6, 2, 5, 4]
    P = np.zeros((8, d2))
    for n, k in enumerate(perm):
        P[n, k] = 1.0
    E2 = r.normal(size=(4, d2))
    Q2, K2, V2 = impl.frame_qkv(E2, P, Hq2, Hkv2, D2)
    X2 = np.concatenate([E2, E2.mean(axis=0, keepdims=True)])
    _close(Q2.reshape(5, 4), X2[:, perm[:4]], 1e-15, "Q picks features 3, 0, 7, 1")
    _close(K2.reshape(5, 2), X2[:, perm[4:6]], 1e-15, "K picks features 6, 2")
    _close(V2.reshape(5, 2), X2[:, perm[6:]], 1e-15, "V picks features 5, 4")
    # a single token: the carrier equals it
    Q1, K1, V1 = impl.frame_qkv(E[:1], W, Hq, Hkv, D)
    assert np.array_equal(Q1[0], Q1[1]) and np.array_equal(V1[0], V1[1])
    # what comes out is what the frame prefill takes: attention of the carrier over the frame,
    # worked out from E and W alone
    O = impl.frame_prefill(Q, None, None, K, V, 0.7)
    h, g = 3, 1
    qc = [math.fsum(X[N][k] * W[h * D + j, k] for k in range(d)) for j in range(D)]
    keys = [[math.fsum(X[t][k] * W[Hq * D + g * D + j, k] for k in range(d)) for j in range(D)] for t in range(N + 1)]
    vals = [[math.fsum(X[t][k] * W[(Hq + Hkv) * D + g * D + j, k] for k in range(d)) for j in range(D)] for t in range(N + 1)]
    z = [0.7 * math.fsum(a * b for a, b in zip(qc, kk)) for kk in keys]
    w = [math.exp(x - max(z)) for x in z]
    want = [math.fsum(w[t] * vals[t][j] for t in range(N + 1)) / math.fsum(w) for j in range(D)]
    _close(O[N, h], np.array(want), 1e-12, "carrier's attention from E and W")


def pin_decoder_layer(impl):
    """The layer around the attention (Section 4.1 names the backbone; Section 3.1 the projections).
    Pins of the readings taken: RMS norm, bias-free projections as X W^T, SiLU-gated feed-forward,
    residual sums around both blocks."""
    r = _rng(71)
    # --- RMS norm: closed forms
    x = np.array([[3.0, -4.0, 0.0, 0.0]])                     # mean of squares 25/4: rms 5/2
    _close(impl.rmsnorm(x, np.ones(4), 0.0), x / 2.5, 1e-15, "rms of (3, -4, 0, 0) is 5/2")
    _close(impl.rmsnorm(x, np.array([2.0, 1.0, 7.0, 7.0]), 0.0), np.array([[2.4, -1.6, 0.0, 0.0]]), 1e-15, "gain per feature")
    _close(impl.rmsnorm(np.array([[1.0, 1.0, 1.0, 1.0]]), np.ones(4), 3.0), np.full((1, 4), 0.5), 1e-15, "eps under the root: 1/sqrt(1+3)")
    X = r.normal(size=(5, 12))
    g = r.normal(size=12)
    Y = impl.rmsnorm(X, g, 0.0)
    _close(impl.rmsnorm(7.5 * X, g, 0.0), Y, 1e-13, "scale invariance without eps")
    _close(np.sqrt(np.mean((Y / g) ** 2, axis=1)), np.ones(5), 1e-13, "unit rms before the gain")
    for t in range(5):                                           # rows are independent, brute force
        rms = math.sqrt(math.fsum(v * v for v in X[t]) / 12 + 1e-3)
        _close(impl.rmsnorm(X, g, 1e-3)[t], np.array([X[t, j] * g[j] / rms for j in range(12)]), 1e-14, f"row {t}")
    # --- linear: brute force, identity, and weights that pick single features (transposition shows)
    W = r.normal(size=(7, 12))
    L = impl.linear(X, W)
    assert L.shape == (5, 7)
    for t in range(5):
        for n in range(7):
            assert abs(L[t, n] - math.fsum(X[t, k] * W[n, k] for k in range(12))) < 1e-13
    pick = np.zeros((3, 12))
    pick[0, 11], pick[1, 0], pick[2, 5] = 1.0, 1.0, 1.0
    _close(impl.linear(X, pick), X[:, [11, 0, 5]], 1e-15, "rows of W pick features 11, 0, 5")
    # --- gated unit: silu(a) - silu(-a) = a; silu(ln 3) = (3/4) ln 3; silu(0) = 0; the second factor multiplies
    a = r.normal(size=(2, 6))
    _close(impl.gated_unit(a, np.ones_like(a)) - impl.gated_unit(-a, np.ones_like(a)), a, 1e-14, "silu is x sigmoid(x)")
    _close(impl.gated_unit(np.array([[math.log(3.0), 0.0]]), np.array([[2.0, 5.0]])), np.array([[1.5 * math.log(3.0), 0.0]]), 1e-15,
           "silu(ln 3) = 3/4 ln 3")
    # --- the layer.  Tiny shape, everything worked out with fsum from the definitions above.
    T, d, Hq, Hkv, D, F, Lc = 3, 4, 2, 1, 2, 3, 2
    H = r.normal(size=(T, d))
    g1, g2 = r.normal(size=d), r.normal(size=d)
    Wq, Wk, Wv = r.normal(size=(Hq * D, d)), r.normal(size=(Hkv * D, d)), r.normal(size=(Hkv * D, d))
    Wo, Wg, Wu, Wd = r.normal(size=(d, Hq * D)), r.normal(size=(F, d)), r.normal(size=(F, d)), r.normal(size=(d, F))
    Kc, Vc = r.normal(size=(Lc, Hkv, D)), r.normal(size=(Lc, Hkv, D))
    eps, scale = 1e-2, 0.6
    Hout, Kf, Vf = impl.decoder_layer(H, g1, Wq, Wk, Wv, Wo, g2, Wg, Wu, Wd, eps, Kc, Vc, Hq, Hkv, D, scale)

    def norm(M, gain):
        return [[M[t][j] * gain[j] / math.sqrt(math.fsum(v * v for v in M[t]) / len(M[t]) + eps) for j in range(len(M[t]))]
                for t in range(len(M))]

    def mat(M, Wm):
        return [[math.fsum(M[t][k] * Wm[n][k] for k in range(len(M[t]))) for n in range(len(Wm))] for t in range(len(M))]
    x1 = norm(H.tolist(), g1)
    q, k, v = mat(x1, Wq), mat(x1, Wk), mat(x1, Wv)
    _close(Kf.reshape(T, -1), np.array(k), 1e-13, "the run's K rows")
    _close(Vf.reshape(T, -1), np.array(v), 1e-13, "the run's V rows")
    Q3 = [[[q[t][h * D + j] for j in range(D)] for h in range(Hq)] for t in range(T)]
    Kall = Kc.tolist() + [[[k[t][j] for j in range(D)]] for t in range(T)]
    Vall = Vc.tolist() + [[[v[t][j] for j in range(D)]] for t in range(T)]
    att, _ = brute_attention(Q3, Kall, Vall, [Lc + t + 1 for t in range(T)], scale)
    aflat = [[att[t][h][j] for h in range(Hq) for j in range(D)] for t in range(T)]
    o = mat(aflat, Wo)
    h1 = [[H[t][j] + o[t][j] for j in range(d)] for t in range(T)]
    x2 = norm(h1, g2)
    gg, uu = mat(x2, Wg), mat(x2, Wu)
    act = [[gg[t][f] / (1.0 + math.exp(-gg[t][f])) * uu[t][f] for f in range(F)] for t in range(T)]
    dn = mat(act, Wd)
    want = [[h1[t][j] + dn[t][j] for j in range(d)] for t in range(T)]
    _close(Hout, np.array(want), 1e-12, "layer output from the definitions")
    # with the two output projections at zero both blocks add nothing: the residual path alone
    Hz, _, _ = impl.decoder_layer(H, g1, Wq, Wk, Wv, 0 * Wo, g2, Wg, Wu, 0 * Wd, eps, Kc, Vc, Hq, Hkv, D, scale)
    _close(Hz, H, 0.0, "zero output projections leave the hidden state alone")
    # causality survives the layer: a later token changes no earlier row; the retained rows reach all rows
    H2 = H.copy()
    H2[T - 1] += 1.0
    Hc, _, _ = impl.decoder_layer(H2, g1, Wq, Wk, Wv, Wo, g2, Wg, Wu, Wd, eps, Kc, Vc, Hq, Hkv, D, scale)
    assert np.array_equal(Hc[:T - 1], Hout[:T - 1]) and not np.allclose(Hc[T - 1], Hout[T - 1])
    Hk, _, _ = impl.decoder_layer(H, g1, Wq, Wk, Wv, Wo, g2, Wg, Wu, Wd, eps, Kc + 0.5, Vc, Hq, Hkv, D, scale)
    assert all(not np.allclose(Hk[t], Hout[t]) for t in range(T))
    # an empty cache is allowed
    He, _, _ = impl.decoder_layer(H[:1], g1, Wq, Wk, Wv, Wo, g2, Wg, Wu, Wd, eps, None, None, Hq, Hkv, D, scale)
    x1e = norm(H[:1].tolist(), g1)
    ve = mat(x1e, Wv)[0]                       # one token, one key: the attention returns its own V row, for both heads
    oe = mat([[ve[j] for _ in range(Hq) for j in range(D)]], Wo)[0]
    h1e = [[H[0][j] + oe[j] for j in range(d)]]
    x2e = norm(h1e, g2)
    ge, ue = mat(x2e, Wg)[0], mat(x2e, Wu)[0]
    acte = [[ge[f] / (1.0 + math.exp(-ge[f])) * ue[f] for f in range(F)]]
    _close(He, np.array([[h1e[0][j] + mat(acte, Wd)[0][j] for j in range(d)]]), 1e-12, "one token, empty cache")


ALL_PINS = [
    pin_golden_rational,
    pin_uniform_scores_mean_of_visible,
    pin_single_key,
    pin_one_hot_limit,
    pin_row_stochastic_and_masked_zero,
    pin_brute_force_tiny,
    pin_library_second_opinion,
    pin_causality,
    pin_carrier_row_is_unmasked_attention,
    pin_gqa_equals_replicated_mha,
    pin_invariances,
    pin_transposition_sensitive,
    pin_compaction,
    pin_streaming_equals_one_shot,
    pin_decode,
    pin_mean_pool,
    pin_memory_bank,
    pin_frames_with_semantic_mask,
    pin_question_after_the_video,
    pin_frame_rows_and_their_projections,
    pin_decoder_layer,
]
