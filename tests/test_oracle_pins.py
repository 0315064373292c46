"""The oracle against its pins, and the pins against planted mistakes (CPU only)."""
import numpy as np
import pytest

import oracle
from pins import ALL_PINS


@pytest.mark.parametrize("pin", ALL_PINS, ids=lambda p: p.__name__)
def test_oracle_passes_pin(pin):
    pin(oracle)


# ----------------------------------------------------------------------------
# An independent numpy evaluation with switchable, plausible mistakes.  Unbroken
# it must pass every pin; each mistake must be caught by at least one pin.
# ----------------------------------------------------------------------------
class NumpyImpl:
    def __init__(self, bug=None):
        self.bug = bug

    def attention(self, Q, Kall, Vall, vis, scale, return_probs=False):
        Q, Kall, Vall = (np.asarray(a, dtype=np.float64) for a in (Q, Kall, Vall))
        Tq, Hq, D = Q.shape
        R, Hkv, _ = Kall.shape
        G = Hq // Hkv
        O = np.zeros((Tq, Hq, D))
        P = np.zeros((Hq, Tq, R))
        for h in range(Hq):
            g = h % Hkv if self.bug == "gqa_interleaved" else h // G
            src = Vall if self.bug == "scores_from_v" else Kall
            for i in range(Tq):
                n = int(vis[i])
                z = src[:n, g] @ Q[i, h]
                if self.bug != "no_scale":
                    z = z * scale
                if self.bug == "scale_squared":
                    z = z * scale
                w = np.exp(z - z.max())
                p = w if self.bug == "no_normalise" else w / w.sum()
                if self.bug == "negated_scores":
                    w = np.exp(-(z - z.min()))
                    p = w / w.sum()
                P[h, i, :n] = p
                O[i, h] = p @ Vall[:n, g]
        return (O, P) if return_probs else O

    def frame_prefill(self, Q, Kc, Vc, Kf, Vf, scale, return_probs=False):
        Kf, Vf = np.asarray(Kf, dtype=np.float64), np.asarray(Vf, dtype=np.float64)
        T = Kf.shape[0]
        L = 0 if Kc is None else len(Kc)
        Kall = Kf if L == 0 else np.concatenate([Kc, Kf])
        Vall = Vf if L == 0 else np.concatenate([Vc, Vf])
        if self.bug == "self_invisible":
            vis = [max(L + i, 1) for i in range(T)]
        elif self.bug == "sees_next":
            vis = [min(L + i + 2, L + T) for i in range(T)]
        elif self.bug == "no_mask":
            vis = [L + T] * T
        elif self.bug == "frame_before_cache":
            Kall = Kf if L == 0 else np.concatenate([Kf, Kc])
            Vall = Vf if L == 0 else np.concatenate([Vf, Vc])
            vis = [L + i + 1 for i in range(T)]
        else:
            vis = [L + i + 1 for i in range(T)]
        return self.attention(Q, Kall, Vall, np.array(vis), scale, return_probs)

    def compact_append(self, Kc, Vc, length, Kf, Vf, carrier=None):
        T = len(Kf)
        if carrier is None:
            carrier = 0 if self.bug == "keeps_first_token" else T - 1
        cap = Kc.shape[0]
        if length >= cap and self.bug != "no_capacity_check":
            raise RuntimeError("capacity")
        at = length - 1 if self.bug == "overwrites_last" else length
        at = min(at, cap - 1)
        Kc[at] = Kf[carrier]
        Vc[at] = Kf[carrier] if self.bug == "v_gets_k" else Vf[carrier]
        return (at, length + 1)

    def decode(self, q, Kc, Vc, length, k_new, v_new, scale):
        n = length
        if k_new is not None:
            Kc[length], Vc[length] = k_new, v_new
            n = length + 1
        seen = length if (self.bug == "decode_attends_before_append" and k_new is not None) else n
        o = self.attention(np.asarray(q)[None], Kc[:seen], Vc[:seen], np.array([seen]), scale)[0]
        return o, n

    def query_prefill(self, Q, Kc, Vc, length, Kt, Vt, scale):
        Q, Kt, Vt = (np.asarray(a, dtype=np.float64) for a in (Q, Kt, Vt))
        Tq = Q.shape[0]
        if length + Tq > len(Kc) and self.bug != "question_no_capacity_check":
            raise ValueError("cache full")
        at = length + 1 if self.bug == "question_rows_off_by_one" else length
        keep = range(Tq - 1, Tq) if self.bug == "question_keeps_last_token_only" else range(Tq)
        Kall = np.concatenate([Kc[:length], Kt])
        Vall = np.concatenate([Vc[:length], Vt])
        if self.bug == "question_not_causal":
            vis = np.full(Tq, length + Tq)
        elif self.bug == "question_blind_to_itself":
            vis = length + np.arange(Tq) + (np.arange(Tq) == 0)
        else:
            vis = length + np.arange(Tq) + 1
        O = self.attention(Q, Kall, Vall, vis, scale)
        for j in keep:
            row = min(at + (j if len(keep) > 1 else 0), len(Kc) - 1)
            Kc[row], Vc[row] = Kt[j], Vt[j]
        return O, length + (len(keep) if self.bug != "question_length_plus_one" else 1)

    def frame_qkv(self, E, W, n_q_heads, n_kv_heads, head_dim):
        E, W = np.asarray(E, dtype=np.float64), np.asarray(W, dtype=np.float64)
        N = E.shape[0]
        c = E.sum(axis=0) if self.bug == "proj_carrier_is_sum" else E.mean(axis=0)
        if self.bug == "proj_carrier_is_last_token":
            c = E[-1]
        X = np.concatenate([c[None], E]) if self.bug == "proj_carrier_first" else np.concatenate([E, c[None]])
        if self.bug == "proj_weights_transposed" and W.shape[0] == W.shape[1]:
            Y = X @ W
        elif self.bug == "proj_weights_transposed":
            Y = X @ W.T.reshape(W.shape).T   # the same numbers read in the other order
        else:
            Y = X @ W.T
        nq, nk = n_q_heads * head_dim, n_kv_heads * head_dim
        parts = [Y[:, :nq], Y[:, nq:nq + nk], Y[:, nq + nk:]]
        if self.bug == "proj_k_and_v_swapped":
            parts[1], parts[2] = parts[2], parts[1]
        if self.bug == "proj_heads_interleaved":
            parts[0] = parts[0].reshape(N + 1, head_dim, n_q_heads).transpose(0, 2, 1).reshape(N + 1, nq)
        return (parts[0].reshape(N + 1, n_q_heads, head_dim).copy(), parts[1].reshape(N + 1, n_kv_heads, head_dim).copy(),
                parts[2].reshape(N + 1, n_kv_heads, head_dim).copy())

    def rmsnorm(self, X, g, eps):
        X, g = np.asarray(X, dtype=np.float64), np.asarray(g, dtype=np.float64)
        ms = (X ** 2).sum(axis=1, keepdims=True) if self.bug == "norm_sum_not_mean" else (X ** 2).mean(axis=1, keepdims=True)
        if self.bug == "norm_centres":
            X = X - X.mean(axis=1, keepdims=True)
        if self.bug == "norm_eps_outside_root":
            return X * g / (np.sqrt(ms) + eps)
        if self.bug == "norm_no_gain":
            return X / np.sqrt(ms + eps)
        return X * g / np.sqrt(ms + eps)

    def linear(self, X, W):
        X, W = np.asarray(X, dtype=np.float64), np.asarray(W, dtype=np.float64)
        if self.bug == "linear_weights_transposed":
            return X @ W.reshape(W.shape[1], W.shape[0])
        return X @ W.T

    def gated_unit(self, G, U):
        G, U = np.asarray(G, dtype=np.float64), np.asarray(U, dtype=np.float64)
        if self.bug == "gate_is_sigmoid_only":
            return U / (1.0 + np.exp(-G))
        if self.bug == "gate_acts_on_value":
            return G * (U / (1.0 + np.exp(-U)))
        if self.bug == "gate_relu":
            return np.maximum(G, 0.0) * U
        return G / (1.0 + np.exp(-G)) * U

    def decoder_layer(self, H, g1, Wq, Wk, Wv, Wo, g2, Wg, Wu, Wd, eps, Kc, Vc, n_q_heads, n_kv_heads, head_dim, scale):
        H = np.asarray(H, dtype=np.float64)
        T = H.shape[0]
        x1 = H if self.bug == "layer_no_first_norm" else self.rmsnorm(H, g1, eps)
        q = self.linear(x1, Wq).reshape(T, n_q_heads, head_dim)
        k = self.linear(x1, Wk).reshape(T, n_kv_heads, head_dim)
        v = self.linear(x1, Wv).reshape(T, n_kv_heads, head_dim)
        a = self.frame_prefill(q, Kc, Vc, k, v, scale).reshape(T, -1)
        o = self.linear(a, Wo)
        h1 = o if self.bug == "layer_no_attention_residual" else H + o
        x2 = self.rmsnorm(H if self.bug == "layer_post_norm_of_input" else h1, g1 if self.bug == "layer_same_gain_twice" else g2, eps)
        act = self.gated_unit(self.linear(x2, Wg), self.linear(x2, Wu))
        dn = self.linear(act, Wd)
        out = (H + dn) if self.bug == "layer_second_residual_from_input" else (h1 + dn)
        if self.bug == "layer_no_mlp_residual":
            out = dn
        return out, k, v

    def mean_pool(self, E):
        E = np.asarray(E, dtype=np.float64)
        if self.bug == "pool_sum":
            return E.sum(axis=0)
        if self.bug == "pool_unbiased":
            return E.sum(axis=0) / max(E.shape[0] - 1, 1)
        if self.bug == "pool_over_features":
            return np.resize(E.mean(axis=1), E.shape[1])
        return E.sum(axis=0) / E.shape[0]

    def frames_prefill(self, Q, Kc, Vc, Kf, Vf, scale):
        Q, Kf, Vf = (np.asarray(a, dtype=np.float64) for a in (Q, Kf, Vf))
        F, T, Hq, D = Q.shape
        Hkv = Kf.shape[2]
        L = 0 if Kc is None else len(Kc)
        parts_k = ([np.asarray(Kc, dtype=np.float64)] if L else []) + [Kf.reshape(F * T, Hkv, D)]
        parts_v = ([np.asarray(Vc, dtype=np.float64)] if L else []) + [Vf.reshape(F * T, Hkv, D)]
        Kall, Vall = np.concatenate(parts_k), np.concatenate(parts_v)
        car = 0 if self.bug == "run_carrier_is_first_token" else T - 1
        O = np.zeros((F, T, Hq, D))
        for a in range(F):
            for i in range(T):
                mask = np.zeros(L + F * T, dtype=bool)
                mask[:L] = True
                for b in range(F):
                    for j in range(T):
                        own = b == a and (j <= i or self.bug == "run_sees_own_future")
                        earlier = b < a and (j == car or self.bug == "run_no_semantic_mask")
                        if self.bug == "run_no_earlier_carriers":
                            earlier = False
                        if self.bug == "run_sees_later_carriers":
                            earlier = b != a and j == car
                        mask[L + b * T + j] = own or earlier
                idx = np.nonzero(mask)[0]
                for h in range(Hq):
                    g = h // (Hq // Hkv)
                    z = (Kall[idx, g] @ Q[a, i, h]) * scale
                    w = np.exp(z - z.max())
                    O[a, i, h] = (w / w.sum()) @ Vall[idx, g]
        return O

    def bank_victim(self, E, e_new, policy=0):
        E, e_new = np.asarray(E, dtype=np.float64), np.asarray(e_new, dtype=np.float64)
        M = len(E)
        if self.bug == "bank_ignores_incoming":
            nxt = np.concatenate([E[1:], E[-1:]])
        else:
            nxt = np.concatenate([E[1:], e_new[None]])
        if policy == 1:
            nxt = np.tile(e_new, (M, 1))
        dots = (E * nxt).sum(axis=1)
        na, nb = np.sqrt((E * E).sum(axis=1)), np.sqrt((nxt * nxt).sum(axis=1))
        ok = (na > 0) & (nb > 0)
        cos = np.where(ok, dots / np.where(ok, na * nb, 1.0), 0.0)
        if self.bug == "bank_dot_not_cosine":
            cos = dots
        if self.bug == "bank_least_similar":
            return int(np.argmin(cos)), cos
        if self.bug == "bank_tie_last":
            return int(M - 1 - np.argmax(cos[::-1])), cos
        v = int(np.argmax(cos))
        if self.bug == "bank_drops_newer" and policy == 0:
            v = min(v + 1, M - 1)
        return v, cos

    def bank_apply(self, rows, first, M, n, victim, row_new):
        row_new = np.asarray(row_new, dtype=np.float64).reshape(rows.shape[1:])
        if n < M:
            rows[first + n] = row_new
            return n + 1
        if self.bug == "bank_overwrites_victim":
            rows[first + victim] = row_new
            return M
        rows[first + victim:first + M - 1] = rows[first + victim + 1:first + M].copy()
        rows[first + M - (2 if self.bug == "bank_new_row_off_by_one" else 1)] = row_new
        return M


BUGS = ["gqa_interleaved", "scores_from_v", "no_scale", "scale_squared", "no_normalise",
        "negated_scores", "self_invisible", "sees_next", "no_mask", "frame_before_cache",
        "keeps_first_token", "no_capacity_check", "overwrites_last", "v_gets_k",
        "decode_attends_before_append", "pool_sum", "pool_unbiased", "pool_over_features",
        "bank_ignores_incoming", "bank_dot_not_cosine", "bank_least_similar", "bank_tie_last",
        "bank_drops_newer", "bank_overwrites_victim", "bank_new_row_off_by_one",
        "run_carrier_is_first_token", "run_sees_own_future", "run_no_semantic_mask", "run_no_earlier_carriers",
        "run_sees_later_carriers", "question_rows_off_by_one", "question_keeps_last_token_only",
        "question_not_causal", "question_blind_to_itself", "question_length_plus_one", "question_no_capacity_check",
        "proj_carrier_is_sum", "proj_carrier_is_last_token", "proj_carrier_first", "proj_weights_transposed",
        "proj_k_and_v_swapped", "proj_heads_interleaved",
        "norm_sum_not_mean", "norm_centres", "norm_eps_outside_root", "norm_no_gain", "linear_weights_transposed",
        "gate_is_sigmoid_only", "gate_acts_on_value", "gate_relu", "layer_no_first_norm", "layer_no_attention_residual",
        "layer_post_norm_of_input", "layer_same_gain_twice", "layer_second_residual_from_input", "layer_no_mlp_residual"]


def _failures(impl):
    failed = []
    for pin in ALL_PINS:
        try:
            pin(impl)
        except Exception:  # a broken implementation may also crash a pin; that counts as caught
            failed.append(pin.__name__)
    return failed


def test_unbroken_numpy_evaluation_passes_all_pins():
    assert _failures(NumpyImpl()) == []


@pytest.mark.parametrize("bug", BUGS)
def test_pins_catch_planted_mistake(bug):
    assert _failures(NumpyImpl(bug)), f"no pin notices the planted mistake '{bug}'"


def test_oracle_matches_numpy_evaluation_midsize():
    """Two independently written evaluations agree on a GQA case with a ragged visible prefix."""
    r = np.random.default_rng(5)
    Q, K, V = r.normal(size=(9, 8, 16)), r.normal(size=(40, 2, 16)), r.normal(size=(40, 2, 16))
    vis = r.integers(1, 41, size=9)
    a, pa = oracle.attention(Q, K, V, vis, 0.25, return_probs=True)
    b, pb = NumpyImpl().attention(Q, K, V, vis, 0.25, return_probs=True)
    assert np.abs(a - b).max() < 1e-14 and np.abs(pa - pb).max() < 1e-15


def test_oracle_layer_matches_numpy_evaluation_midsize():
    """The layer, two independently written evaluations, at a shape with grouped heads and a ragged cache."""
    r = np.random.default_rng(6)
    T, d, Hq, Hkv, D, F, L = 11, 24, 6, 2, 8, 40, 13
    H, g1, g2 = r.normal(size=(T, d)), r.normal(size=d), r.normal(size=d)
    Wq, Wk, Wv = (r.normal(size=(n, d)) / 5 for n in (Hq * D, Hkv * D, Hkv * D))
    Wo, Wg, Wu, Wd = r.normal(size=(d, Hq * D)) / 7, r.normal(size=(F, d)) / 5, r.normal(size=(F, d)) / 5, r.normal(size=(d, F)) / 6
    Kc, Vc = r.normal(size=(L, Hkv, D)), r.normal(size=(L, Hkv, D))
    a = oracle.decoder_layer(H, g1, Wq, Wk, Wv, Wo, g2, Wg, Wu, Wd, 1e-6, Kc, Vc, Hq, Hkv, D, 0.3)
    b = NumpyImpl().decoder_layer(H, g1, Wq, Wk, Wv, Wo, g2, Wg, Wu, Wd, 1e-6, Kc, Vc, Hq, Hkv, D, 0.3)
    for x, y in zip(a, b):
        assert x.shape == y.shape and np.abs(x - y).max() < 1e-12


def test_oracle_layer_rejects_bad_arguments():
    H, g = np.zeros((2, 4)), np.ones(4)
    W = np.zeros((4, 4))
    with pytest.raises(oracle.OracleError):  # projection width is not heads x head_dim
        oracle.decoder_layer(H, g, np.zeros((6, 4)), W[:2], W[:2], W, g, W, W, W, 1e-6, None, None, 2, 1, 2, 1.0)
    with pytest.raises(oracle.OracleError):  # gain of the wrong length
        oracle.rmsnorm(H, np.ones(3), 1e-6)
    with pytest.raises(oracle.OracleError):  # inner sizes differ
        oracle.linear(H, np.zeros((3, 5)))
    with pytest.raises(oracle.OracleError):  # the two halves of the gated unit differ in shape
        oracle.gated_unit(np.zeros((2, 3)), np.zeros((2, 4)))


def test_oracle_rejects_bad_arguments():
    Q, K = np.zeros((2, 3, 4)), np.zeros((5, 2, 4))
    with pytest.raises(oracle.OracleError):  # Hq not a multiple of Hkv
        oracle.attention(Q, K, K, np.array([1, 1]), 1.0)
    Q = np.zeros((2, 4, 4))
    with pytest.raises(oracle.OracleError):  # visible prefix beyond the rows
        oracle.attention(Q, K, K, np.array([1, 6]), 1.0)
    with pytest.raises(oracle.OracleError):  # empty visible set
        oracle.attention(Q, K, K, np.array([0, 1]), 1.0)
    Kc = np.zeros((2, 2, 4))
    with pytest.raises(oracle.OracleError) as e:
        oracle.compact_append(Kc, Kc.copy(), 2, K, K)
    assert e.value.code == 2
    with pytest.raises(oracle.OracleError):
        oracle.compact_append(Kc, Kc.copy(), 0, K, K, carrier=5)


def test_retained_length_of_the_configs():
    """Retained rows = prefix + frames seen: 17 for the tiny case, 264 for the 64-frame stream."""
    from synth import CONFIGS
    for name, want in (("cfg1", 17), ("cfg2", 264), ("cfg3", 4552)):
        c = CONFIGS[name]
        s = c["shape"]
        cap = c["prefix"] + c["frames"]
        Kc, Vc = np.zeros((cap, s.n_kv_heads, 2)), np.zeros((cap, s.n_kv_heads, 2))
        Kf = np.ones((c["n_visual"] + 1, s.n_kv_heads, 2))
        ln = c["prefix"]
        rows = []
        for _ in range(c["frames"]):
            row, ln = oracle.compact_append(Kc, Vc, ln, Kf, Kf)
            rows.append(row)
        assert ln == want and rows == list(range(c["prefix"], want))
