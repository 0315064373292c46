"""GPU parity: the HIP path behind the C ABI against the CPU fp64 oracle on the same seeded
bytes.  Integer results (row indices, lengths, copied rows) must be bit-exact; floats within
the tolerances in gpu_util."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2503_09387_amd as vs
from gpu_util import (DEV, check_close, lens_array, oracle_prefill_rows, run_prefill, scale32,
                      torch_dtype, vs_shape, workspace)
from synth import (CONFIGS, AttnShape, cache_rows, carrier_embeddings, cfg1_inputs, decode_lengths, decode_step_inputs,
                   draw, frame_inputs, to_f64)

pytestmark = pytest.mark.gpu

QW = CONFIGS["cfg2"]["shape"]


@pytest.fixture(autouse=True)
def _reset_tuning():
    yield
    for knob in (0, 1, 2, 4):
        vs.set_tuning(knob, 0)


def same_bits(dev_t, host_t):
    return torch.equal(dev_t.cpu().view(torch.uint8), host_t.contiguous().view(torch.uint8))


# ---------------------------------------------------------------------------- cfg1
def test_cfg1_tiny_fp32_pool_prefill_compact():
    c = CONFIGS["cfg1"]
    s = c["shape"]
    x = cfg1_inputs(c)
    L, T = c["prefix"], c["n_visual"] + 1
    # carrier embedding
    e = x["e"].to(DEV)
    pooled = torch.empty(c["hidden"], dtype=torch.float32, device=DEV)
    vs.carrier_mean_pool(e, pooled, "f32")
    check_close(pooled, oracle.mean_pool(to_f64(x["e"])), "f32", "mean pool")
    # prefill
    out, cache, _ = run_prefill(s, x["k_c"], x["v_c"], L, x["q"], x["k_f"], x["v_f"], capacity=L + 1)
    ref = oracle_prefill_rows(s, x["q"], x["k_c"], x["v_c"], L, x["k_f"], x["v_f"])
    check_close(out, ref, "f32", "cfg1 prefill")
    # compaction
    row = vs.carrier_compact_append(vs_shape(s), cache, x["k_f"].to(DEV), x["v_f"].to(DEV))
    torch.cuda.synchronize()
    ok_k, ok_v = to_f64(x["k_c"]).copy(), to_f64(x["v_c"]).copy()
    ok_k, ok_v = np.concatenate([ok_k, np.zeros((1,) + ok_k.shape[1:])]), np.concatenate([ok_v, np.zeros((1,) + ok_v.shape[1:])])
    orow, olen = oracle.compact_append(ok_k, ok_v, L, to_f64(x["k_f"]), to_f64(x["v_f"]))
    assert (row, cache.len) == (orow, olen) == (16, 17)
    assert np.array_equal(cache.k.double().cpu().numpy(), ok_k) and np.array_equal(cache.v.double().cpu().numpy(), ok_v)
    # fused entry point gives the same bits
    out2, cache2, row2 = run_prefill(s, x["k_c"], x["v_c"], L, x["q"], x["k_f"], x["v_f"], capacity=L + 1, fused=True)
    assert row2 == 16 and cache2.len == 17
    assert torch.equal(out2, out) and torch.equal(cache2.k, cache.k) and torch.equal(cache2.v, cache.v)


# ---------------------------------------------------------------------------- cfg2
@pytest.mark.parametrize("fused", [False, True])
def test_cfg2_stream_of_64_frames(fused):
    c = CONFIGS["cfg2"]
    s, P0, F, T = c["shape"], c["prefix"], c["frames"], c["n_visual"] + 1
    pk, pv = cache_rows(c["seed"], s, P0, c["sigma"])
    cap = P0 + F
    kc = torch.zeros((cap, s.n_kv_heads, s.head_dim), dtype=torch.bfloat16, device=DEV)
    vc = torch.zeros_like(kc)
    kc[:P0].copy_(pk)
    vc[:P0].copy_(pv)
    cache = vs.Cache(kc, vc, P0)
    ws = workspace(s, T, cap, 0)
    ok, ov = np.zeros((cap, s.n_kv_heads, s.head_dim)), np.zeros((cap, s.n_kv_heads, s.head_dim))
    ok[:P0], ov[:P0] = to_f64(pk), to_f64(pv)
    olen = P0
    sh = vs_shape(s)
    worst = (0.0, 0.0)
    for f in range(F):
        q, kf, vf = frame_inputs(c["seed"], s, T, c["sigma"], frame=f)
        qd, kfd, vfd = q.to(DEV), kf.to(DEV), vf.to(DEV)
        out = torch.empty_like(qd)
        if fused:
            row = vs.frame_prefill_compact(sh, cache, qd, kfd, vfd, out, ws)
        else:
            vs.frame_prefill_attn(sh, cache, qd, kfd, vfd, out, ws)
            row = vs.carrier_compact_append(sh, cache, kfd, vfd)
        ref = oracle.frame_prefill(to_f64(q), ok[:olen], ov[:olen], to_f64(kf), to_f64(vf), scale32(s))
        orow, olen = oracle.compact_append(ok, ov, olen, to_f64(kf), to_f64(vf))
        assert (row, cache.len) == (orow, olen), f"frame {f}"
        torch.cuda.synchronize()
        e = check_close(out, ref, "bf16", f"cfg2 frame {f}")
        worst = (max(worst[0], e[0]), max(worst[1], e[1]))
    assert cache.len == 264
    assert np.array_equal(kc.double().cpu().numpy(), ok) and np.array_equal(vc.double().cpu().numpy(), ov)
    print(f"cfg2 worst max-abs {worst[0]:.2e} mean-abs {worst[1]:.2e}")


# ---------------------------------------------------------------------------- cfg3
def test_cfg3_whole_stream_all_frames_all_layers():
    """The whole long stream: 256 frames x 28 layers through vs_frame_prefill_compact, starting from
    4296 retained rows per layer.  Row index and length of EVERY (frame, layer) call are compared
    with oracle.compact_append run beside it, and at the end every cache byte (retained rows,
    the 256 appended carrier rows, untouched tail) with the oracle's arrays.  Floats are checked
    against the oracle on frames whose cache length is 0, 1 and 63 past a multiple of the kernel's
    64-row tile (and the first, a middle and the last frame), three layers, eight tokens each.
    The frames' Q/K/V come from a pool of 8 distinct frames per layer (frame f uses f % 8), as in
    bench.py: the draw of 7168 frame-layers would take minutes, and the retained state does not
    depend on which values move."""
    c = CONFIGS["cfg3"]
    s, T, NL, P0, F = c["shape"], c["n_visual"] + 1, c["layers"], c["prefix"], c["frames"]
    sh = vs_shape(s)
    cap = P0 + F
    POOL = 8
    ws = workspace(s, T, cap, 0)
    sample_layers = (0, 13, 27)
    float_frames = {0, 55, 56, 57, 128, 255}          # 4296 + f = 63, 0, 1 (mod 64) at f = 55, 56, 57
    assert [(P0 + f) % 64 for f in (55, 56, 57)] == [63, 0, 1]
    tokens = np.array([0, 1, 37, 84, 85, 127, 168, 169])
    tok_dev = torch.from_numpy(tokens).to(DEV)
    pool_host = [[frame_inputs(c["seed"], s, T, c["sigma"], frame=f, layer=l) for l in range(NL)] for f in range(POOL)]
    pool_dev = [[tuple(x.to(DEV) for x in fl) for fl in fr] for fr in pool_host]
    pool_kv64 = [[(to_f64(fl[1]), to_f64(fl[2])) for fl in fr] for fr in pool_host]
    caches, ok, ov, olen = [], [], [], []
    for l in range(NL):
        hk, hv = cache_rows(c["seed"], s, P0, c["sigma"], layer=l)
        kc = torch.zeros((cap, s.n_kv_heads, s.head_dim), dtype=torch.bfloat16, device=DEV)
        vc = torch.zeros_like(kc)
        kc[:P0].copy_(hk)
        vc[:P0].copy_(hv)
        caches.append(vs.Cache(kc, vc, P0))
        k64, v64 = np.zeros((cap, s.n_kv_heads, s.head_dim)), np.zeros((cap, s.n_kv_heads, s.head_dim))
        k64[:P0], v64[:P0] = to_f64(hk), to_f64(hv)
        ok.append(k64)
        ov.append(v64)
        olen.append(P0)
    outs = [torch.empty((T, s.n_q_heads, s.head_dim), dtype=torch.bfloat16, device=DEV) for _ in sample_layers]
    unchecked = torch.empty_like(outs[0])
    for f in range(F):
        pending = []
        for l in range(NL):
            qd, kfd, vfd = pool_dev[f % POOL][l]
            sampled = f in float_frames and l in sample_layers
            out = outs[sample_layers.index(l)] if sampled else unchecked
            if sampled:  # the oracle's view of the cache before this frame
                q, kf, vf = pool_host[f % POOL][l]
                ref = oracle.attention(to_f64(q)[tokens], np.concatenate([ok[l][:olen[l]], to_f64(kf)]),
                                       np.concatenate([ov[l][:olen[l]], to_f64(vf)]), olen[l] + tokens + 1, scale32(s))
                pending.append((l, out, ref))
            row = vs.frame_prefill_compact(sh, caches[l], qd, kfd, vfd, out, ws)
            orow, olen[l] = oracle.compact_append(ok[l], ov[l], olen[l], *pool_kv64[f % POOL][l])
            assert (row, caches[l].len) == (orow, olen[l]) == (P0 + f, P0 + f + 1), f"frame {f} layer {l}"
        if pending:
            torch.cuda.synchronize()
            for l, out, ref in pending:
                check_close(out[tok_dev], ref, "bf16", f"cfg3 whole stream, frame {f} layer {l}")
    torch.cuda.synchronize()
    for l in range(NL):
        assert caches[l].len == olen[l] == 4552
        assert np.array_equal(caches[l].k.double().cpu().numpy(), ok[l]), f"K cache of layer {l}"
        assert np.array_equal(caches[l].v.double().cpu().numpy(), ov[l]), f"V cache of layer {l}"


# ---------------------------------------------------------------------------- cfg4
def test_cfg4_decode_16_ragged_streams():
    """Full launch shape (16 streams, lengths U[512,8192]+128, capacity 8384); 2 of the 28 layers
    (each layer is the same launch), 6 of the 64 steps with floats checked on every one."""
    c = CONFIGS["cfg4"]
    s, S = c["shape"], c["streams"]
    sh = vs_shape(s)
    lens0 = decode_lengths(c["seed"], S, c["carrier_lo"], c["carrier_hi"], c["text_hist"])
    assert min(lens0) >= 640 and max(lens0) <= 8320
    cap = c["carrier_hi"] + c["text_hist"] + c["steps"]
    ws = workspace(s, 0, cap, S)
    for layer in (0, 27):
        ks = torch.zeros((S, cap, s.n_kv_heads, s.head_dim), dtype=torch.bfloat16, device=DEV)
        vsl = torch.zeros_like(ks)
        ok = [np.zeros((cap, s.n_kv_heads, s.head_dim)) for _ in range(S)]
        ov = [np.zeros((cap, s.n_kv_heads, s.head_dim)) for _ in range(S)]
        for i in range(S):
            hk, hv = cache_rows(c["seed"], s, lens0[i], c["sigma"], layer=layer, stream=i)
            ks[i, :lens0[i]].copy_(hk)
            vsl[i, :lens0[i]].copy_(hv)
            ok[i][:lens0[i]], ov[i][:lens0[i]] = to_f64(hk), to_f64(hv)
        lens = lens_array(lens0)
        olens = list(lens0)
        for step in range(6):
            q, kn, vn = decode_step_inputs(c["seed"], s, S, c["sigma"], step=step, layer=layer)
            out = torch.full(q.shape, float("nan"), dtype=torch.bfloat16, device=DEV)
            vs.decode_attn(sh, ks, vsl, lens, q.to(DEV), kn.to(DEV), vn.to(DEV), out, ws)
            ref = np.zeros((S, s.n_q_heads, s.head_dim))
            for i in range(S):
                ref[i], olens[i] = oracle.decode(to_f64(q[i]), ok[i], ov[i], olens[i], to_f64(kn[i]),
                                                 to_f64(vn[i]), scale32(s))
            assert list(lens) == olens, f"lengths after step {step}"
            torch.cuda.synchronize()
            check_close(out, ref, "bf16", f"cfg4 layer {layer} step {step}")
        for i in range(S):
            assert np.array_equal(ks[i].double().cpu().numpy(), ok[i])
            assert np.array_equal(vsl[i].double().cpu().numpy(), ov[i])


def test_cfg4_whole_decode_64_steps_28_layers():
    """All 64 steps on all 28 layers of the 16 ragged streams.  After every call the lengths are
    compared with the oracle's; at the end every appended row (64 per stream and layer) is compared
    bit for bit with what oracle.compact_append put there, and the rows in front of them and behind
    them with what was there before.  Floats against oracle.decode for all 16 streams at
    (layer, step) = (0, 0), (13, 31) and (27, 63), the last step included.
    The oracle's row copy works on a window of each stream's cache that starts at the stream's
    initial length (an append is the same operation wherever the row sits; whole caches in fp64
    would take 30 GB).  Four distinct layer slabs are drawn and copied to the 28 layers, as in
    bench.py; the inputs of every (step, layer) are drawn on their own."""
    c = CONFIGS["cfg4"]
    s, S, NL, steps = c["shape"], c["streams"], c["layers"], c["steps"]
    sh = vs_shape(s)
    lens0 = decode_lengths(c["seed"], S, c["carrier_lo"], c["carrier_hi"], c["text_hist"])
    cap = c["carrier_hi"] + c["text_hist"] + steps
    ws = workspace(s, 0, cap, S)
    DISTINCT = 4
    base_host, base_dev = [], []
    for l in range(DISTINCT):
        k = torch.zeros((S, cap, s.n_kv_heads, s.head_dim), dtype=torch.bfloat16)
        v = torch.zeros_like(k)
        for i in range(S):
            hk, hv = cache_rows(c["seed"], s, lens0[i], c["sigma"], layer=l, stream=i)
            k[i, :lens0[i]], v[i, :lens0[i]] = hk, hv
        base_host.append((k, v))
        base_dev.append((k.to(DEV), v.to(DEV)))
    slabs = [(base_dev[l % DISTINCT][0].clone(), base_dev[l % DISTINCT][1].clone()) for l in range(NL)]
    lens = [lens_array(lens0) for _ in range(NL)]
    # oracle state: the rows appended to (layer, stream), as a window starting at the initial length
    wk = [[np.zeros((steps, s.n_kv_heads, s.head_dim)) for _ in range(S)] for _ in range(NL)]
    wv = [[np.zeros((steps, s.n_kv_heads, s.head_dim)) for _ in range(S)] for _ in range(NL)]
    wlen = [[0] * S for _ in range(NL)]
    float_at = {(0, 0), (13, 31), (27, steps - 1)}
    out = torch.empty((S, s.n_q_heads, s.head_dim), dtype=torch.bfloat16, device=DEV)
    for step in range(steps):
        for l in range(NL):
            q, kn, vn = decode_step_inputs(c["seed"], s, S, c["sigma"], step=step, layer=l)
            kn64, vn64 = to_f64(kn), to_f64(vn)
            ref = None
            if (l, step) in float_at:
                ref = np.zeros((S, s.n_q_heads, s.head_dim))
                for i in range(S):
                    n0 = lens0[i]
                    k_all = np.concatenate([to_f64(base_host[l % DISTINCT][0][i, :n0]), wk[l][i][:step], np.zeros((1, s.n_kv_heads, s.head_dim))])
                    v_all = np.concatenate([to_f64(base_host[l % DISTINCT][1][i, :n0]), wv[l][i][:step], np.zeros((1, s.n_kv_heads, s.head_dim))])
                    ref[i], n_after = oracle.decode(to_f64(q[i]), k_all, v_all, n0 + step, kn64[i], vn64[i], scale32(s))
                    assert n_after == n0 + step + 1
            vs.decode_attn(sh, slabs[l][0], slabs[l][1], lens[l], q.to(DEV), kn.to(DEV), vn.to(DEV), out, ws)
            for i in range(S):
                row, wlen[l][i] = oracle.compact_append(wk[l][i], wv[l][i], wlen[l][i], kn64[i:i + 1], vn64[i:i + 1])
                assert row == step
            assert list(lens[l]) == [lens0[i] + wlen[l][i] for i in range(S)], f"lengths after step {step}, layer {l}"
            if ref is not None:
                torch.cuda.synchronize()
                check_close(out, ref, "bf16", f"cfg4 whole decode, layer {l} step {step}")
    torch.cuda.synchronize()
    for l in range(NL):
        kd, vd = slabs[l][0].cpu(), slabs[l][1].cpu()
        for i in range(S):
            n0 = lens0[i]
            assert lens[l][i] == n0 + steps
            assert np.array_equal(to_f64(kd[i, n0:n0 + steps]), wk[l][i]), f"appended K rows, layer {l} stream {i}"
            assert np.array_equal(to_f64(vd[i, n0:n0 + steps]), wv[l][i]), f"appended V rows, layer {l} stream {i}"
            assert torch.equal(kd[i, :n0], base_host[l % DISTINCT][0][i, :n0]) and torch.equal(vd[i, :n0], base_host[l % DISTINCT][1][i, :n0])
            assert not kd[i, n0 + steps:].any() and not vd[i, n0 + steps:].any()


# ---------------------------------------------------------------------------- cfg5
def test_cfg5_dense_and_compact_cache_same_frame():
    c = CONFIGS["cfg5"]
    s, T = c["shape"], c["n_visual"] + 1
    q, kf, vf = frame_inputs(c["seed"], s, T, c["sigma"])
    tokens = np.array([0, 2, 36, 37, 90, 128, 168, 169])
    for name, rows, stream in (("dense", c["dense_rows"], 0), ("compact", c["compact_rows"], 1)):
        hk, hv = cache_rows(c["seed"], s, rows, c["sigma"], stream=stream)
        out, _, _ = run_prefill(s, hk, hv, rows, q, kf, vf)
        if name == "compact":
            ref = oracle_prefill_rows(s, q, hk, hv, rows, kf, vf)
            check_close(out, ref, "bf16", "cfg5 compact")
        else:
            ref = oracle_prefill_rows(s, q, hk, hv, rows, kf, vf, tokens)
            check_close(out[torch.from_numpy(tokens).to(DEV)], ref, "bf16", "cfg5 dense (sampled tokens)")


# ---------------------------------------------------------------------------- prefill edges
@pytest.mark.parametrize("L,T,gain", [(0, 1, 1), (0, 5, 1), (1, 1, 1), (63, 2, 1), (64, 64, 1), (65, 170, 1),
                                      (200, 170, 8), (263, 170, 1), (1000, 19, 8), (4551, 170, 8), (130, 512, 1)])
def test_prefill_bf16_shapes_and_peaked_softmax(L, T, gain):
    s = QW
    hk, hv = cache_rows(11, s, max(L, 1), 0.5)
    q, kf, vf = frame_inputs(11, s, T, 0.5, frame=L, layer=T % 7, q_gain=gain)
    out, _, _ = run_prefill(s, hk, hv, L, q, kf, vf)
    check_close(out, oracle_prefill_rows(s, q, hk, hv, L, kf, vf), "bf16", f"L={L} T={T} gain={gain}")
    if L == 0:  # a single visible key returns its V row exactly
        assert same_bits(out[0].reshape(s.n_kv_heads, s.group, -1)[:, 0], vf[0])


@pytest.mark.parametrize("hq,hkv", [(8, 8), (8, 1), (12, 4), (16, 2)])
def test_prefill_other_head_groupings(hq, hkv):
    s = AttnShape(hq, hkv, 128, "bf16")
    L, T = 150, 70
    hk, hv = cache_rows(12, s, L, 0.5)
    q, kf, vf = frame_inputs(12, s, T, 0.5, q_gain=4)
    out, _, _ = run_prefill(s, hk, hv, L, q, kf, vf)
    check_close(out, oracle_prefill_rows(s, q, hk, hv, L, kf, vf), "bf16", f"Hq={hq} Hkv={hkv}")


@pytest.mark.parametrize("kv_groups", [1, 2])
def test_prefill_result_does_not_depend_on_the_split(kv_groups):
    s = QW
    L, T = 1500, 170
    hk, hv = cache_rows(13, s, L, 0.5)
    q, kf, vf = frame_inputs(13, s, T, 0.5, q_gain=4)
    ref = oracle_prefill_rows(s, q, hk, hv, L, kf, vf)
    vs.set_tuning(vs.TUNE_PREFILL_KV_GROUPS, kv_groups)
    outs = []
    for splits in (1, 2, 5, 12, 32):
        vs.set_tuning(vs.TUNE_PREFILL_SPLITS, splits)
        out, _, _ = run_prefill(s, hk, hv, L, q, kf, vf)
        check_close(out, ref, "bf16", f"splits={splits} kv_groups={kv_groups}")
        outs.append(out.float())
    for o in outs[1:]:
        assert (o - outs[0]).abs().max().item() <= 2 ** -7 * outs[0].abs().max().item()


@pytest.mark.parametrize("L,T,splits", [(4424, 170, 0), (1500, 170, 0), (1500, 170, 3), (3000, 300, 8), (700, 40, 2),
                                          (200, 170, 0), (264, 170, 3), (100, 20, 2),
                                          # more than 8 splits (questions of a few tokens; several rounds of workgroups)
                                          (4552, 16, 0), (4552, 64, 0), (1500, 170, 12), (3000, 170, 32), (2100, 30, 9)])
def test_prefill_merge_inside_the_kernel_equals_the_second_kernel(L, T, splits):
    """Split results are merged inside the attention kernel, by the workgroups of a row tile together
    once the last of them has arrived (the library's choice) or by that last one alone, or by a
    second kernel: the same sums in the same order, so the same bits; also on repeated calls
    through one workspace (the arrival counters return to zero, launch numbers move on) and with
    the three ways taking turns."""
    s = QW
    hk, hv = cache_rows(31, s, L, 0.5)
    q, kf, vf = frame_inputs(31, s, T, 0.5, q_gain=4)
    ref = oracle_prefill_rows(s, q, hk, hv, L, kf, vf)
    ws = workspace(s, T, L, 0)
    vs.set_tuning(vs.TUNE_PREFILL_SPLITS, splits)
    vs.set_tuning(vs.TUNE_PREFILL_MERGE, 2)
    two_kernels, _, _ = run_prefill(s, hk, hv, L, q, kf, vf, ws=ws)
    check_close(two_kernels, ref, "bf16", f"second-kernel merge L={L} T={T} splits={splits}")
    for mode in (0, 0, 0, 1, 0, 1, 2, 0):
        vs.set_tuning(vs.TUNE_PREFILL_MERGE, mode)
        inside, _, _ = run_prefill(s, hk, hv, L, q, kf, vf, ws=ws)
        assert same_bits(inside, two_kernels.cpu()), f"merge mode {mode} differs from the second kernel's"
    vs.set_tuning(vs.TUNE_PREFILL_MERGE, 0)


@pytest.mark.parametrize("F,T,L,splits", [(2, 170, 4296, 0), (2, 170, 4296, 5), (3, 170, 2000, 4), (4, 60, 900, 2),
                                          (8, 21, 700, 3)])
def test_runs_of_frames_merge_inside_the_kernel_equals_the_second_kernel(F, T, L, splits):
    """The same for runs of frames: units are (KV head, frame, row tile), every frame reads its own
    number of retained rows; both ways of merging give the same bits, call after call."""
    s = QW
    sh = vs_shape(s)
    hk, hv = cache_rows(71, s, L, 0.5)
    q = draw(72, (F, T, s.n_q_heads, s.head_dim), 1.5, "bf16").to(DEV)
    kf = draw(73, (F, T, s.n_kv_heads, s.head_dim), 0.5, "bf16").to(DEV)
    vf = draw(74, (F, T, s.n_kv_heads, s.head_dim), 0.5, "bf16").to(DEV)
    kc = torch.zeros((L + F, s.n_kv_heads, s.head_dim), dtype=torch.bfloat16, device=DEV)
    vc = torch.zeros_like(kc)
    kc[:L].copy_(hk)
    vc[:L].copy_(hv)
    ws = torch.empty(vs.frames_workspace_bytes(sh, F, T, L + F), dtype=torch.uint8, device=DEV)
    vs.workspace_init(sh, ws)
    vs.set_tuning(vs.TUNE_PREFILL_SPLITS, splits)

    def run():
        cache = vs.Cache(kc, vc, L)
        out = torch.full(q.shape, float("nan"), dtype=torch.bfloat16, device=DEV)
        vs.frames_prefill_attn(sh, cache, q, kf, vf, out, ws)
        torch.cuda.synchronize()
        return out
    vs.set_tuning(vs.TUNE_PREFILL_MERGE, 2)
    two_kernels = run()
    assert bool(torch.isfinite(two_kernels.float()).all())
    for mode in (0, 0, 1, 0):
        vs.set_tuning(vs.TUNE_PREFILL_MERGE, mode)
        assert torch.equal(run().view(torch.int16), two_kernels.view(torch.int16)), f"merge mode {mode}"
    vs.set_tuning(vs.TUNE_PREFILL_MERGE, 0)


def test_prefill_placement_guard_reports_and_falls_back():
    """Every workgroup of an in-kernel-merge launch checks that it runs on the XCD that the probe
    saw for its id.  With the probed order handed over rotated by one (tuning value 3) all of them
    report themselves misplaced: the launch itself is still right (the real placement is
    unchanged), the next call launches nothing and returns VS_ERR_PLACEMENT, the calls after it merge
    with the second kernel and give the same bits, and a new vs_workspace_init probes again and
    brings the in-kernel merge back."""
    s, L, T = QW, 1500, 170
    hk, hv = cache_rows(75, s, L, 0.5)
    q, kf, vf = frame_inputs(75, s, T, 0.5, q_gain=4)
    ws = workspace(s, T, L, 0)
    good, _, _ = run_prefill(s, hk, hv, L, q, kf, vf, ws=ws)
    vs.set_tuning(vs.TUNE_PREFILL_MERGE, 3)
    flagged, _, _ = run_prefill(s, hk, hv, L, q, kf, vf, ws=ws)      # runs, reports, result still right
    vs.set_tuning(vs.TUNE_PREFILL_MERGE, 0)
    assert same_bits(flagged, good.cpu())
    with pytest.raises(vs.VSError) as err:
        run_prefill(s, hk, hv, L, q, kf, vf, ws=ws)
    assert err.value.code == 8
    for _ in range(2):                                                # second-kernel merge from now on
        after, _, _ = run_prefill(s, hk, hv, L, q, kf, vf, ws=ws)
        assert same_bits(after, good.cpu())
    ws2 = workspace(s, T, L, 0)                                       # probes the device again
    again, _, _ = run_prefill(s, hk, hv, L, q, kf, vf, ws=ws2)
    assert same_bits(again, good.cpu())
    run_prefill(s, hk, hv, L, q, kf, vf, ws=ws2)                      # and nothing is reported this time


def test_prefill_shared_merge_gives_up_waiting_and_reports():
    """In the shared merge the workgroups of a row tile wait for the last of them, looking at a word
    in memory a bounded number of times.  With tuning value 4 that number is zero: every kernel
    still ends, the workgroups that would have waited report through the host word (and leave their
    share unmerged), the next call launches nothing and returns VS_ERR_PLACEMENT, the
    calls after it merge with the second kernel and are right, and a new vs_workspace_init brings
    the in-kernel merge back."""
    s, L, T = QW, 1500, 170
    hk, hv = cache_rows(76, s, L, 0.5)
    q, kf, vf = frame_inputs(76, s, T, 0.5, q_gain=4)
    ws = workspace(s, T, L, 0)
    good, _, _ = run_prefill(s, hk, hv, L, q, kf, vf, ws=ws)
    vs.set_tuning(vs.TUNE_PREFILL_MERGE, 4)
    run_prefill(s, hk, hv, L, q, kf, vf, ws=ws)                       # ends; its output is incomplete
    vs.set_tuning(vs.TUNE_PREFILL_MERGE, 0)
    with pytest.raises(vs.VSError) as err:
        run_prefill(s, hk, hv, L, q, kf, vf, ws=ws)
    assert err.value.code == 8
    for _ in range(2):                                                # second-kernel merge from now on
        after, _, _ = run_prefill(s, hk, hv, L, q, kf, vf, ws=ws)
        assert same_bits(after, good.cpu())
    ws2 = workspace(s, T, L, 0)                                       # probes the device again
    for _ in range(2):
        again, _, _ = run_prefill(s, hk, hv, L, q, kf, vf, ws=ws2)
        assert same_bits(again, good.cpu())


@pytest.mark.parametrize("L", [130, 1500])
@pytest.mark.parametrize("mode", ["all_low", "all_high", "rising", "falling", "jump"])
def test_prefill_extreme_score_ranges(mode, L):
    """Scaled scores far from 0 (in log2 units: around -400, around +400, climbing or falling by
    400 along the keys, or jumping by 60 in the middle): the speculative softmax reference has to
    be dropped and rebuilt, at the first sub-block and later ones, with the accumulators rescaled."""
    s = QW
    T = 170
    hk, hv = cache_rows(21, s, L, 0.5)
    q, kf, vf = frame_inputs(21, s, T, 0.5)
    n = L + T
    ramp = torch.arange(n, dtype=torch.float32) / n
    a = {"all_low": torch.full((n,), -10.0), "all_high": torch.full((n,), 10.0), "rising": 10.0 * ramp,
         "falling": -10.0 * ramp, "jump": 1.5 * (ramp > 0.5).float()}[mode]
    # k_j += a_j * u, q += 10 * u with u = 0.5 * ones: score_j moves by 0.1275 * 10 * a_j * 32 log2 units
    hk = (hk.float() + 0.5 * a[:L, None, None]).to(torch.bfloat16)
    kf = (kf.float() + 0.5 * a[L:, None, None]).to(torch.bfloat16)
    q = (q.float() + 5.0).to(torch.bfloat16)
    out, _, _ = run_prefill(s, hk, hv, L, q, kf, vf)
    check_close(out, oracle_prefill_rows(s, q, hk, hv, L, kf, vf), "bf16", f"{mode} L={L}")


def test_prefill_uniform_scores_is_running_mean_at_full_size():
    """Q = 0: every row is the mean of its visible V rows (closed form, any size)."""
    s = QW
    L, T = 4296, 170
    hk, hv = cache_rows(14, s, L, 0.5)
    _, kf, vf = frame_inputs(14, s, T, 0.5)
    q = torch.zeros((T, s.n_q_heads, s.head_dim), dtype=torch.bfloat16)
    out, _, _ = run_prefill(s, hk, hv, L, q, kf, vf)
    v_all = np.concatenate([to_f64(hv), to_f64(vf)])
    csum = np.cumsum(v_all, axis=0)
    ref = np.stack([csum[L + t] / (L + t + 1) for t in range(T)])  # [T][Hkv][D]
    ref = np.repeat(ref, s.group, axis=1)
    check_close(out, ref, "bf16", "uniform scores")


def test_prefill_fp32_path_larger_shapes():
    for (hq, hkv, d, L, T) in [(4, 2, 128, 700, 9), (6, 3, 64, 0, 3), (8, 1, 64, 300, 40)]:
        s = AttnShape(hq, hkv, d, "f32")
        hk, hv = cache_rows(15, s, max(L, 1), 1.0)
        q, kf, vf = frame_inputs(15, s, T, 1.0)
        out, _, _ = run_prefill(s, hk, hv, L, q, kf, vf)
        check_close(out, oracle_prefill_rows(s, q, hk, hv, L, kf, vf), "f32", f"fp32 {hq}/{hkv}/{d} L={L}")


# ---------------------------------------------------------------------------- decode edges
def _decode_case(s, lens0, cap, seed, gain=1.0, with_new=True):
    S = len(lens0)
    dt = torch_dtype(s.dtype)
    sigma = 0.5 if s.dtype == "bf16" else 1.0
    ks = torch.zeros((S, cap, s.n_kv_heads, s.head_dim), dtype=dt, device=DEV)
    vsl = torch.zeros_like(ks)
    ok, ov = [], []
    for i in range(S):
        hk, hv = cache_rows(seed, s, max(lens0[i], 1), sigma, stream=i)
        ks[i, :lens0[i]].copy_(hk[:lens0[i]])
        vsl[i, :lens0[i]].copy_(hv[:lens0[i]])
        a, b = np.zeros((cap, s.n_kv_heads, s.head_dim)), np.zeros((cap, s.n_kv_heads, s.head_dim))
        a[:lens0[i]], b[:lens0[i]] = to_f64(hk[:lens0[i]]), to_f64(hv[:lens0[i]])
        ok.append(a)
        ov.append(b)
    q, kn, vn = decode_step_inputs(seed, s, S, sigma, q_gain=gain)
    lens = lens_array(lens0)
    out = torch.full(q.shape, float("nan"), dtype=dt, device=DEV)
    ws = workspace(s, 0, cap, S)
    vs.decode_attn(vs_shape(s), ks, vsl, lens, q.to(DEV), kn.to(DEV) if with_new else None,
                   vn.to(DEV) if with_new else None, out, ws)
    torch.cuda.synchronize()
    ref = np.zeros((S, s.n_q_heads, s.head_dim))
    for i in range(S):
        ref[i], n = oracle.decode(to_f64(q[i]), ok[i], ov[i], lens0[i], to_f64(kn[i]) if with_new else None,
                                  to_f64(vn[i]) if with_new else None, scale32(s))
        assert lens[i] == n
        assert np.array_equal(ks[i].double().cpu().numpy(), ok[i]) and np.array_equal(vsl[i].double().cpu().numpy(), ov[i])
    return out, ref, (q, kn, vn)


@pytest.mark.parametrize("lens0,gain", [([0], 1), ([1, 2, 30, 31, 32, 33, 126, 127, 128, 129, 1000, 5], 1),
                                        ([777], 8), ([8319, 640, 4000], 8)])
def test_decode_ragged_lengths(lens0, gain):
    out, ref, (q, kn, vn) = _decode_case(QW, lens0, 8384 if max(lens0) > 1000 else 1024, 21, gain)
    check_close(out, ref, "bf16", f"decode lens={lens0}")
    if lens0 == [0]:  # empty cache: the output is the new V row exactly
        assert same_bits(out[0].reshape(QW.n_kv_heads, QW.group, -1)[:, 0], vn[0])


def test_decode_without_new_row_and_many_streams():
    lens0 = [40 + 13 * i for i in range(70)]  # more than one launch worth of streams
    out, ref, _ = _decode_case(QW, lens0, 1024, 22, with_new=False)
    check_close(out, ref, "bf16", "decode, 70 streams, no append")


def test_decode_result_does_not_depend_on_the_chunking():
    ref_out = None
    for chunk in (128, 256, 1024, 8192):
        vs.set_tuning(vs.TUNE_DECODE_CHUNK_ROWS, chunk)
        out, ref, _ = _decode_case(QW, [3000, 129, 5000], 5120, 23, gain=4)
        check_close(out, ref, "bf16", f"chunk_rows={chunk}")
        if ref_out is None:
            ref_out = out.float()
        assert (out.float() - ref_out).abs().max().item() <= 2 ** -7 * ref_out.abs().max().item()


@pytest.mark.parametrize("hq,hkv", [(6, 3), (12, 6), (5, 5), (16, 2), (8, 1), (24, 8)])
@pytest.mark.parametrize("chunk", [0, 32])
def test_decode_other_kv_head_counts(hq, hkv, chunk):
    """KV head counts that are not multiples of 4 (a workgroup then takes 1 or 2 heads and its spare
    wavefronts take sub-ranges of the share), with the library's own shares and with the smallest
    ones (one tile per share: the most workgroups, the highest partial-result slots)."""
    s = AttnShape(hq, hkv, 128, "bf16")
    vs.set_tuning(vs.TUNE_DECODE_CHUNK_ROWS, chunk)
    lens0 = [3000, 1, 129, 64, 700, 33] + [40 + 37 * i for i in range(20)]
    out, ref, _ = _decode_case(s, lens0, 3072, 26, gain=4)
    check_close(out, ref, "bf16", f"decode Hq={hq} Hkv={hkv} chunk_rows={chunk}")


def test_decode_equals_one_token_prefill():
    s, L = QW, 900
    out, ref, (q, kn, vn) = _decode_case(s, [L], 1024, 24, gain=4)
    hk, hv = cache_rows(24, s, L, 0.5, stream=0)
    pre, _, _ = run_prefill(s, hk, hv, L, q[0:1], kn[0:1], vn[0:1])
    check_close(pre, ref, "bf16", "one-token prefill vs oracle decode")
    assert (pre.float() - out.float()).abs().max().item() <= 2 ** -7 * out.float().abs().max().item()


def test_decode_fp32_path():
    s = AttnShape(4, 2, 64, "f32")
    out, ref, _ = _decode_case(s, [5, 300, 1], 512, 25)
    check_close(out, ref, "f32", "fp32 decode")


def test_prefill_largest_run_and_head_ratio():
    """4096 tokens in one run (the limit), 8 query heads per KV head (the limit): 32768 query rows
    per KV head, 256 row tiles; sampled tokens against the oracle."""
    s = AttnShape(16, 2, 128, "bf16")
    L, T = 300, 4096
    hk, hv = cache_rows(71, s, L, 0.5)
    q, kf, vf = frame_inputs(71, s, T, 0.5, q_gain=2)
    tokens = np.array([0, 1, 63, 64, 127, 128, 1000, 2047, 2048, 3333, 4094, 4095])
    ref = oracle_prefill_rows(s, q, hk, hv, L, kf, vf, tokens)
    out, cache, row = run_prefill(s, hk, hv, L, q, kf, vf, capacity=L + 1, fused=True)
    check_close(out[torch.from_numpy(tokens).to(DEV)], ref, "bf16", "4096-token run, 8 heads per KV head")
    assert row == L and cache.len == L + 1 and same_bits(cache.k[L], kf[T - 1]) and same_bits(cache.v[L], vf[T - 1])
    assert bool(torch.isfinite(out.float()).all())
    c = vs.Cache(cache.k, cache.v, L)
    too_many = torch.empty((4097, s.n_q_heads, s.head_dim), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(vs.VSError):
        vs.frame_prefill_attn(vs_shape(s), c, too_many, too_many, too_many, too_many, workspace(s, 4096, L + 1, 0))


def test_decode_longest_stream_mix():
    """64 streams in one launch (the most one launch takes), lengths from 1 row to 12000 rows."""
    s = QW
    lens0 = [12000, 1, 2, 31, 32, 33] + [int(x) for x in np.random.default_rng(9).integers(1, 3000, size=58)]
    out, ref, _ = _decode_case(s, lens0, 12008, 27, gain=4)
    check_close(out, ref, "bf16", "64 streams, up to 12000 rows")


# ---------------------------------------------------------------------------- the question after the video
@pytest.mark.parametrize("L,Tq,dtype,splits", [(4424, 32, "bf16", 0), (200, 7, "bf16", 0), (0, 19, "bf16", 0),
                                                (1500, 130, "bf16", 3), (700, 1, "bf16", 0), (300, 600, "bf16", 0),
                                                (150, 9, "f32", 0)])
def test_question_prefill_keeps_all_rows_and_decoding_continues(L, Tq, dtype, splits):
    """vs_question_prefill_append against the oracle's token-by-token evaluation: outputs, the Tq
    rows appended bit for bit, the length; then one decoding step on top of them."""
    s = QW if dtype == "bf16" else AttnShape(4, 2, 64, "f32")
    dt = torch_dtype(dtype)
    cap = L + Tq + 4
    hk, hv = cache_rows(61, s, L, 0.5)
    q, kt, vt = frame_inputs(61, s, Tq, 0.5, q_gain=4)
    Kc, Vc = np.zeros((cap, s.n_kv_heads, s.head_dim)), np.zeros((cap, s.n_kv_heads, s.head_dim))
    if L:
        Kc[:L], Vc[:L] = to_f64(hk), to_f64(hv)
    ref, n = oracle.query_prefill(to_f64(q), Kc, Vc, L, to_f64(kt), to_f64(vt), scale32(s))
    assert n == L + Tq
    k = torch.full((cap, s.n_kv_heads, s.head_dim), 7.0, dtype=dt, device=DEV)  # junk beyond len must not count
    v = torch.full_like(k, -7.0)
    if L:
        k[:L].copy_(hk)
        v[:L].copy_(hv)
    cache = vs.Cache(k, v, L)
    ws = workspace(s, Tq, cap, 1)
    vs.set_tuning(vs.TUNE_PREFILL_SPLITS, splits)
    out = torch.full(q.shape, float("nan"), dtype=dt, device=DEV)
    vs.question_prefill_append(vs_shape(s), cache, q.to(DEV), kt.to(DEV), vt.to(DEV), out, ws)
    torch.cuda.synchronize()
    vs.set_tuning(vs.TUNE_PREFILL_SPLITS, 0)
    check_close(out, ref, dtype, f"question L={L} Tq={Tq}")
    assert cache.len == L + Tq
    assert same_bits(cache.k[L:L + Tq], kt) and same_bits(cache.v[L:L + Tq], vt)
    assert bool((cache.k[L + Tq:] == 7.0).all()) and bool((cache.v[L + Tq:] == -7.0).all())
    if L:
        assert same_bits(cache.k[:L], hk) and same_bits(cache.v[:L], hv)
    # the answer's first token
    qd, kn, vn = decode_step_inputs(62, s, 1, 0.5, step=0)
    o_ref, n2 = oracle.decode(to_f64(qd[0]), Kc, Vc, n, to_f64(kn[0]), to_f64(vn[0]), scale32(s))
    lens = lens_array([cache.len])
    od = torch.empty((1, s.n_q_heads, s.head_dim), dtype=dt, device=DEV)
    vs.decode_attn(vs_shape(s), k[None], v[None], lens, qd.to(DEV), kn.to(DEV), vn.to(DEV), od, ws)
    torch.cuda.synchronize()
    check_close(od[0], o_ref, dtype, f"decoding step after the question, L={L} Tq={Tq}")
    assert lens[0] == n2 == L + Tq + 1


# ---------------------------------------------------------------------------- the frame's rows and their projections
def _projection_case(s, N, d, seed):
    e = draw(seed, (N, d), 1.0, "bf16")
    n_out = (s.n_q_heads + 2 * s.n_kv_heads) * s.head_dim
    w = draw(seed + 1, (n_out, d), d ** -0.5, "bf16")
    rq, rk, rv = oracle.frame_qkv(to_f64(e), to_f64(w), s.n_q_heads, s.n_kv_heads, s.head_dim)
    sh = vs_shape(s)
    q = torch.full((N + 1, s.n_q_heads, s.head_dim), float("nan"), dtype=torch.bfloat16, device=DEV)
    k = torch.full((N + 1, s.n_kv_heads, s.head_dim), float("nan"), dtype=torch.bfloat16, device=DEV)
    v = torch.full_like(k, float("nan"))
    c = torch.full((d,), float("nan"), dtype=torch.bfloat16, device=DEV)
    outs = []
    for rep in range(2):
        vs.frame_qkv_project(sh, e.to(DEV), w.to(DEV), q, k, v, c_out=c)
        torch.cuda.synchronize()
        outs.append((q.clone(), k.clone(), v.clone()))
    assert all(same_bits(a, b.cpu()) for a, b in zip(outs[1], outs[0])), "the same call twice gives the same bits"
    return (q, k, v, c), (rq, rk, rv), (e, w)


@pytest.mark.parametrize("N,d,heads", [(169, 3584, (28, 4)), (49, 256, (8, 2)), (1, 64, (8, 8)), (191, 448, (16, 2)),
                                        (16, 128, (8, 1)), (100, 1024, (12, 4)), (160, 64, (3, 1)), (17, 192, (7, 1))])
def test_frame_projection_matches_oracle(N, d, heads):
    """vs_frame_qkv_project against the oracle: every row incl. the carrier's, Q/K/V in the layouts
    the prefill takes; the carrier embedding equals vs_carrier_mean_pool bit for bit."""
    s = AttnShape(heads[0], heads[1], 128, "bf16")
    (q, k, v, c), (rq, rk, rv), (e, w) = _projection_case(s, N, d, 500 + N)
    check_close(q, rq, "bf16", f"Q N={N} d={d}")
    check_close(k, rk, "bf16", f"K N={N} d={d}")
    check_close(v, rv, "bf16", f"V N={N} d={d}")
    pooled = torch.empty(d, dtype=torch.bfloat16, device=DEV)
    vs.carrier_mean_pool(e.to(DEV), pooled, "bf16")
    torch.cuda.synchronize()
    assert same_bits(c, pooled.cpu())
    # without the embedding asked for, the same Q/K/V
    q2, k2, v2 = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    vs.frame_qkv_project(vs_shape(s), e.to(DEV), w.to(DEV), q2, k2, v2)
    torch.cuda.synchronize()
    assert same_bits(q2, q.cpu()) and same_bits(k2, k.cpu()) and same_bits(v2, v.cpu())


def test_frame_projection_feeds_the_prefill():
    """E and W in, attention out: projection, then prefill with compaction, against the oracle's
    projection followed by its prefill (inputs of the second stage rounded to bf16 on both sides)."""
    s, N, d, L = QW, 169, 3584, 300
    (q, k, v, c), (rq, rk, rv), _ = _projection_case(s, N, d, 91)
    hk, hv = cache_rows(92, s, L, 0.5)
    out, cache, row = run_prefill(s, hk, hv, L, q.cpu(), k.cpu(), v.cpu(), capacity=L + 1, fused=True)
    ref = oracle_prefill_rows(s, q.cpu(), hk, hv, L, k.cpu(), v.cpu())
    check_close(out, ref, "bf16", "prefill on projected rows")
    assert row == L and same_bits(cache.k[L], k[N].cpu()) and same_bits(cache.v[L], v[N].cpu())


# ---------------------------------------------------------------------------- pool, batched append
@pytest.mark.parametrize("n,d,dtype", [(169, 3584, "bf16"), (49, 256, "f32"), (1, 8, "bf16"), (7, 1000, "f32")])
def test_mean_pool(n, d, dtype):
    e = draw(31, (n, d), 1.0, dtype)
    out = torch.empty(d, dtype=torch_dtype(dtype), device=DEV)
    vs.carrier_mean_pool(e.to(DEV), out, dtype)
    torch.cuda.synchronize()
    ref = oracle.mean_pool(to_f64(e))
    got = out.double().cpu().numpy()
    if dtype == "f32":
        assert np.abs(got - ref).max() <= 1e-6
    else:  # one bf16 rounding of an fp32 mean
        assert np.all(np.abs(got - ref) <= np.abs(ref) * 2.0 ** -8 + 1e-30)


@pytest.mark.parametrize("n_caches,pinned", [(28, False), (4096, False), (4095, True), (4096, True), (4097, True), (50, True)])
def test_batched_compaction(n_caches, pinned):
    s, T, cap = QW, 6, 5
    rng = np.random.default_rng(5)
    lens0 = rng.integers(0, cap, size=n_caches).tolist()
    if pinned:  # lengths in a pinned host tensor, row indices into a caller's array
        lens_t = torch.tensor(lens0, dtype=torch.int32).pin_memory()
        ks = torch.zeros((n_caches, cap, s.n_kv_heads, s.head_dim), dtype=torch.bfloat16, device=DEV)
        vsl = torch.zeros_like(ks)
        kf = draw(41, (n_caches, T, s.n_kv_heads, s.head_dim), 0.5, "bf16")
        vf = draw(42, (n_caches, T, s.n_kv_heads, s.head_dim), 0.5, "bf16")
        # rows into a pinned tensor (the device copy is taken from it), into a plain array, or
        # nowhere (then the call waits for the stream, lens being pinned)
        rows_c = [torch.zeros(n_caches, dtype=torch.int32).pin_memory(), (ctypes.c_int32 * n_caches)(), None][n_caches % 3]
        got = vs.carrier_compact_append_batched(vs_shape(s), ks, vsl, lens_t, kf.to(DEV), vf.to(DEV),
                                                workspace=workspace(s, 0, 0, n_caches), rows_out=rows_c)
        torch.cuda.synchronize()
        assert (got is rows_c if rows_c is not None else got == lens0) and lens_t.tolist() == [n + 1 for n in lens0]
        assert rows_c is None or [int(x) for x in rows_c] == lens0
        idx = torch.tensor(lens0)
        ar = torch.arange(n_caches)
        assert same_bits(ks[ar, idx], kf[:, T - 1]) and same_bits(vsl[ar, idx], vf[:, T - 1])
        assert int((ks != 0).any(dim=-1).any(dim=-1).sum()) == n_caches  # one row per cache, no other
        return
    ks = torch.zeros((n_caches, cap, s.n_kv_heads, s.head_dim), dtype=torch.bfloat16, device=DEV)
    vsl = torch.zeros_like(ks)
    kf = draw(41, (n_caches, T, s.n_kv_heads, s.head_dim), 0.5, "bf16")
    vf = draw(42, (n_caches, T, s.n_kv_heads, s.head_dim), 0.5, "bf16")
    lens = lens_array(lens0)
    ws = workspace(s, 0, 0, n_caches)
    rows = vs.carrier_compact_append_batched(vs_shape(s), ks, vsl, lens, kf.to(DEV), vf.to(DEV), workspace=ws)
    torch.cuda.synchronize()
    assert rows == lens0 and list(lens) == [n + 1 for n in lens0]
    want_k, want_v = torch.zeros(ks.shape, dtype=torch.bfloat16), torch.zeros(ks.shape, dtype=torch.bfloat16)
    for i in range(n_caches):
        want_k[i, lens0[i]] = kf[i, T - 1]
        want_v[i, lens0[i]] = vf[i, T - 1]
    assert same_bits(ks, want_k) and same_bits(vsl, want_v)


# ---------------------------------------------------------------------------- memory bank
@pytest.mark.parametrize("dtype,M,d,policy", [("bf16", 128, 3584, 0), ("f32", 16, 256, 0), ("bf16", 64, 3584, 1),
                                              ("bf16", 5, 8, 0), ("f32", 130, 64, 0)])
def test_memory_bank_stream(dtype, M, d, policy):
    """Carriers arrive one by one: the bank fills, then drops the older carrier of the most similar
    adjacent pair.  Victim indices against the fp64 oracle (the device sums in fp64 too, in another
    order: equal whenever the two best cosines differ by more than 1e-6, far above what the order of
    summation can move), embeddings and the K/V rows of three layers bit for bit."""
    s = AttnShape(4, 2, 64, "f32") if dtype == "f32" else QW
    n_layers, first, extra = 3, 5, 40
    n = M + extra
    emb = carrier_embeddings(7, n, d, dtype)
    kv = draw(99, (n, n_layers, 2, s.n_kv_heads, s.head_dim), 1.0, dtype)   # [carrier][layer][k|v]
    dt = torch_dtype(dtype)
    bank = vs.Bank(torch.zeros((M, d), dtype=dt, device=DEV), dtype)
    caches = [vs.Cache(torch.full((first + M + 2, s.n_kv_heads, s.head_dim), 7.0, dtype=dt, device=DEV),
                       torch.full((first + M + 2, s.n_kv_heads, s.head_dim), -7.0, dtype=dt, device=DEV), first)
              for _ in range(n_layers)]
    victim = torch.full((1,), -5, dtype=torch.int32, device=DEV)
    ws = torch.empty(vs.memory_bank_workspace_bytes(M), dtype=torch.uint8, device=DEV)
    # the oracle's state
    o_emb = np.zeros((M, d))
    o_k = [np.full((first + M + 2, s.n_kv_heads, s.head_dim), 7.0) for _ in range(n_layers)]
    o_v = [np.full((first + M + 2, s.n_kv_heads, s.head_dim), -7.0) for _ in range(n_layers)]
    o_n = 0
    near_ties = 0
    for t in range(n):
        e_dev = emb[t].to(DEV)
        rows = kv[t].to(DEV)
        vs.memory_bank_push(bank, e_dev, victim, ws, policy=policy)
        vs.carrier_evict_append(vs_shape(s), caches, first, M, rows[:, 0], rows[:, 1], victim)
        got = int(victim.cpu()[0])
        e64 = to_f64(emb[t])
        if o_n < M:
            assert got == -1
            want = -1
        else:
            want, cos = oracle.bank_victim(o_emb, e64, policy)
            top = np.sort(cos)[::-1]
            assert 0 <= got < M and cos[got] >= top[0] - 1e-6, f"carrier {t}: victim {got}, cosine {cos[got]} vs best {top[0]}"
            if top[0] - top[1] > 1e-6:
                assert got == want, f"carrier {t}: victim {got}, oracle {want}"
            else:
                near_ties += 1
        n2 = oracle.bank_apply(o_emb, 0, M, o_n, got, e64)
        for l in range(n_layers):
            oracle.bank_apply(o_k[l], first, M, o_n, got, to_f64(kv[t, l, 0]))
            oracle.bank_apply(o_v[l], first, M, o_n, got, to_f64(kv[t, l, 1]))
        o_n = n2
        assert bank.len == o_n and all(c.len == first + o_n for c in caches)
        if t % 13 == 0 or t >= n - 3:
            assert np.array_equal(bank.e.double().cpu().numpy(), o_emb), f"embeddings after carrier {t}"
            for l in range(n_layers):
                assert np.array_equal(caches[l].k.double().cpu().numpy(), o_k[l]), f"K rows of layer {l} after carrier {t}"
                assert np.array_equal(caches[l].v.double().cpu().numpy(), o_v[l]), f"V rows of layer {l} after carrier {t}"
    assert near_ties <= extra // 4


def test_memory_bank_ties_and_zero_vectors():
    """Equal cosines: the smallest index goes; a zero vector has cosine 0 and never wins over a
    positive one."""
    M, d = 6, 16
    e = torch.zeros((M, d), dtype=torch.float32)
    e[0, 0] = 1.0
    e[1, 1] = 2.0
    e[2, 1] = 0.5          # pair (1, 2): cosine 1
    e[3, 2] = 1.0
    e[4, 3] = 3.0
    e[5, 3] = 1.0          # pair (4, 5): cosine 1 as well
    new = torch.zeros(d)
    bank = vs.Bank(e.to(DEV), "f32", M)
    victim = torch.zeros(1, dtype=torch.int32, device=DEV)
    ws = torch.empty(vs.memory_bank_workspace_bytes(M), dtype=torch.uint8, device=DEV)
    vs.memory_bank_push(bank, new.to(DEV), victim, ws)
    assert int(victim.cpu()[0]) == 1 == oracle.bank_victim(e.double().numpy(), new.double().numpy())[0]
    want = e.double().numpy().copy()
    oracle.bank_apply(want, 0, M, M, 1, new.double().numpy())
    assert np.array_equal(bank.e.double().cpu().numpy(), want)


def test_memory_bank_rejects_bad_arguments():
    s = QW
    e = torch.zeros((4, 8), dtype=torch.bfloat16, device=DEV)
    victim = torch.zeros(1, dtype=torch.int32, device=DEV)
    ws = torch.empty(256, dtype=torch.uint8, device=DEV)
    bank = vs.Bank(e, "bf16")
    with pytest.raises(vs.VSError) as err:
        vs.memory_bank_push(bank, e[0], victim, ws, policy=3)
    assert err.value.code == 2
    with pytest.raises(vs.VSError) as err:
        vs.memory_bank_push(bank, e[0], victim, ws[:8])
    assert err.value.code == 5 and bank.len == 0
    k = torch.zeros((6, s.n_kv_heads, s.head_dim), dtype=torch.bfloat16, device=DEV)
    cache = vs.Cache(k, k.clone(), 2)
    rows = torch.zeros((1, s.n_kv_heads, s.head_dim), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(vs.VSError) as err:       # prefix + bank does not fit the cache
        vs.carrier_evict_append(vs_shape(s), [cache], 2, 5, rows, rows, victim)
    assert err.value.code == 4 and cache.len == 2
    with pytest.raises(vs.VSError) as err:       # fewer rows than the prefix
        vs.carrier_evict_append(vs_shape(s), [cache], 3, 2, rows, rows, victim)
    assert err.value.code == 2


def test_stream_with_memory_bank_prefill_reads_the_bank():
    """Frames arrive at a bank of 4 carriers behind a 3-row prefix, two layers: every frame's
    prefill attends to [prefix | carriers held], then its carrier is pushed (evicting one once the
    bank is full).  Outputs against the oracle run over the oracle's own bank; victims, lengths and
    retained rows as the oracle has them."""
    s = QW
    M, first, n_layers, frames, T, d = 4, 3, 2, 10, 21, 64
    emb = carrier_embeddings(17, frames, d, "bf16")
    dt = torch.bfloat16
    caches, o_k, o_v = [], [], []
    for l in range(n_layers):
        hk, hv = cache_rows(40 + l, s, first, 0.5)
        k = torch.zeros((first + M, s.n_kv_heads, s.head_dim), dtype=dt, device=DEV)
        v = torch.zeros_like(k)
        k[:first].copy_(hk)
        v[:first].copy_(hv)
        caches.append(vs.Cache(k, v, first))
        ok, ov = np.zeros((first + M, s.n_kv_heads, s.head_dim)), np.zeros((first + M, s.n_kv_heads, s.head_dim))
        ok[:first], ov[:first] = to_f64(hk), to_f64(hv)
        o_k.append(ok)
        o_v.append(ov)
    bank = vs.Bank(torch.zeros((M, d), dtype=dt, device=DEV), "bf16")
    o_emb, o_n = np.zeros((M, d)), 0
    victim = torch.zeros(1, dtype=torch.int32, device=DEV)
    bws = torch.empty(vs.memory_bank_workspace_bytes(M), dtype=torch.uint8, device=DEV)
    ws = workspace(s, T, first + M, 0)
    for f in range(frames):
        rows_k = torch.empty((n_layers, s.n_kv_heads, s.head_dim), dtype=dt, device=DEV)
        rows_v = torch.empty_like(rows_k)
        o_rows = []
        for l in range(n_layers):
            q, kf, vf = frame_inputs(500 + 10 * f + l, s, T, 0.5, q_gain=2)
            out = torch.full(q.shape, float("nan"), dtype=dt, device=DEV)
            vs.frame_prefill_attn(vs_shape(s), caches[l], q.to(DEV), kf.to(DEV), vf.to(DEV), out, ws)
            L = first + o_n
            ref = oracle.frame_prefill(to_f64(q), o_k[l][:L], o_v[l][:L], to_f64(kf), to_f64(vf), scale32(s))
            check_close(out, ref, "bf16", f"frame {f} layer {l} over {o_n} carriers")
            rows_k[l].copy_(kf[T - 1])
            rows_v[l].copy_(vf[T - 1])
            o_rows.append((to_f64(kf[T - 1]), to_f64(vf[T - 1])))
        vs.memory_bank_push(bank, emb[f].to(DEV), victim, bws)
        vs.carrier_evict_append(vs_shape(s), caches, first, M, rows_k, rows_v, victim)
        got = int(victim.cpu()[0])
        e64 = to_f64(emb[f])
        if o_n == M:
            want, cos = oracle.bank_victim(o_emb, e64)
            top = np.sort(cos)[::-1]
            assert got == want or top[0] - top[1] <= 1e-6
        else:
            assert got == -1
        for l in range(n_layers):
            oracle.bank_apply(o_k[l], first, M, o_n, got, o_rows[l][0])
            oracle.bank_apply(o_v[l], first, M, o_n, got, o_rows[l][1])
        o_n = oracle.bank_apply(o_emb, 0, M, o_n, got, e64)
        assert bank.len == o_n and all(c.len == first + o_n for c in caches)
    for l in range(n_layers):
        assert np.array_equal(caches[l].k.double().cpu().numpy(), o_k[l]) and np.array_equal(caches[l].v.double().cpu().numpy(), o_v[l])


# ---------------------------------------------------------------------------- run of several frames
@pytest.mark.parametrize("F,T,L,splits", [(1, 170, 300, 0), (4, 170, 1500, 0), (8, 170, 4296, 0), (3, 21, 0, 0),
                                          (6, 40, 70, 0), (2, 170, 4296, 5), (64, 20, 500, 0)])
def test_run_of_frames_with_semantic_mask(F, T, L, splits):
    """Several frames in one call: outputs against the oracle's definition of the mask, the carriers
    appended in frame order bit for bit, and the same as feeding the frames one call at a time."""
    s = QW
    hk, hv = cache_rows(61, s, L, 0.5)
    q = draw(62, (F, T, s.n_q_heads, s.head_dim), 0.5 * 3, "bf16")
    kf = draw(63, (F, T, s.n_kv_heads, s.head_dim), 0.5, "bf16")
    vf = draw(64, (F, T, s.n_kv_heads, s.head_dim), 0.5, "bf16")
    ref = oracle.frames_prefill(to_f64(q), to_f64(hk) if L else None, to_f64(hv) if L else None, to_f64(kf), to_f64(vf),
                                scale32(s))
    dt = torch.bfloat16

    def fresh_cache():
        k = torch.zeros((L + F, s.n_kv_heads, s.head_dim), dtype=dt, device=DEV)
        v = torch.zeros_like(k)
        if L:
            k[:L].copy_(hk)
            v[:L].copy_(hv)
        return vs.Cache(k, v, L)

    vs.set_tuning(vs.TUNE_PREFILL_SPLITS, splits)
    cache = fresh_cache()
    ws = torch.empty(vs.frames_workspace_bytes(vs_shape(s), F, T, L + F), dtype=torch.uint8, device=DEV)
    vs.workspace_init(vs_shape(s), ws)
    out = torch.full(q.shape, float("nan"), dtype=dt, device=DEV)
    vs.frames_prefill_attn(vs_shape(s), cache, q.to(DEV), kf.to(DEV), vf.to(DEV), out, ws)
    torch.cuda.synchronize()
    assert cache.len == L + F
    check_close(out, ref, "bf16", f"run of {F} frames of {T} over {L} rows")
    assert same_bits(cache.k[L:], kf[:, T - 1]) and same_bits(cache.v[L:], vf[:, T - 1])
    if L:
        assert same_bits(cache.k[:L], hk) and same_bits(cache.v[:L], hv)
    # one call per frame gives the same values up to the rounding of differently split sums
    c2 = fresh_cache()
    ws1 = workspace(s, T, L + F, 0)
    for a in range(F):
        o1 = torch.full(q.shape[1:], float("nan"), dtype=dt, device=DEV)
        vs.frame_prefill_compact(vs_shape(s), c2, q[a].to(DEV), kf[a].to(DEV), vf[a].to(DEV), o1, ws1)
        torch.cuda.synchronize()
        d = (o1.float() - out[a].float()).abs().max().item()
        assert d <= 2 ** -7 * out[a].float().abs().max().item() + 1e-6, f"frame {a}: {d}"
    assert torch.equal(c2.k, cache.k) and torch.equal(c2.v, cache.v) and c2.len == cache.len


def test_prefill_random_shapes_sweep():
    """Seeded sweep over cache lengths, run lengths, head groupings, forced splits and key-group
    counts: exercises every way the key tiles can fall onto the (split, key group) lanes (fewer
    tiles than lanes, frame tiles on several lanes, a lane made of frame tiles only, ...)."""
    rng = np.random.default_rng(2024)
    groupings = [(28, 4), (8, 8), (8, 1), (12, 4), (16, 2)]
    for case in range(96):
        hq, hkv = groupings[rng.integers(len(groupings))]
        s = AttnShape(hq, hkv, 128, "bf16")
        L = int(rng.choice([0, 1, 63, 64, 65, 127, 200, 449, 512, 1000, 1733]))
        T = int(rng.choice([1, 2, 9, 19, 37, 64, 101, 170, 257]))
        splits = int(rng.choice([0, 0, 1, 2, 3, 5, 8, 13, 32]))
        kvg = int(rng.choice([0, 0, 1, 2]))
        gain = float(rng.choice([1, 1, 6]))
        vs.set_tuning(vs.TUNE_PREFILL_SPLITS, splits)
        vs.set_tuning(vs.TUNE_PREFILL_KV_GROUPS, kvg)
        hk, hv = cache_rows(700 + case, s, L, 0.5)
        q, kf, vf = frame_inputs(700 + case, s, T, 0.5, q_gain=gain)
        out, cache, row = run_prefill(s, hk, hv, L, q, kf, vf, fused=bool(case & 1))
        ref = oracle_prefill_rows(s, q, hk, hv, L, kf, vf)
        bound = oracle_prefill_rows(s, q, hk, hv.abs(), L, kf, vf.abs())
        check_close(out, ref, "bf16", f"case {case}: Hq/Hkv {hq}/{hkv} L={L} T={T} splits={splits} kv_groups={kvg} gain={gain}",
                    abs_v_out=bound)
        if case & 1:
            assert row == L and cache.len == L + 1 and same_bits(cache.k[L], kf[T - 1]) and same_bits(cache.v[L], vf[T - 1])


def test_runs_of_frames_random_shapes_sweep():
    rng = np.random.default_rng(77)
    for case in range(24):
        hq, hkv = [(28, 4), (8, 8), (8, 1)][rng.integers(3)]
        s = AttnShape(hq, hkv, 128, "bf16")
        F = int(rng.choice([1, 2, 3, 5, 9, 17]))
        T = int(rng.choice([1, 3, 19, 40, 101]))
        L = int(rng.choice([0, 5, 64, 130, 700]))
        splits = int(rng.choice([0, 0, 2, 4, 7]))
        vs.set_tuning(vs.TUNE_PREFILL_SPLITS, splits)
        hk, hv = cache_rows(900 + case, s, L, 0.5)
        q = draw(1000 + case, (F, T, hq, 128), 1.0, "bf16")
        kf = draw(1100 + case, (F, T, hkv, 128), 0.5, "bf16")
        vf = draw(1200 + case, (F, T, hkv, 128), 0.5, "bf16")
        ref = oracle.frames_prefill(to_f64(q), to_f64(hk) if L else None, to_f64(hv) if L else None, to_f64(kf),
                                    to_f64(vf), scale32(s))
        k = torch.zeros((L + F, hkv, 128), dtype=torch.bfloat16, device=DEV)
        v = torch.zeros_like(k)
        if L:
            k[:L].copy_(hk)
            v[:L].copy_(hv)
        cache = vs.Cache(k, v, L)
        ws = torch.empty(max(vs.frames_workspace_bytes(vs_shape(s), F, T, L + F), 1 << 24), dtype=torch.uint8, device=DEV)
        vs.workspace_init(vs_shape(s), ws)
        out = torch.full(q.shape, float("nan"), dtype=torch.bfloat16, device=DEV)
        vs.frames_prefill_attn(vs_shape(s), cache, q.to(DEV), kf.to(DEV), vf.to(DEV), out, ws)
        torch.cuda.synchronize()
        bound = oracle.frames_prefill(to_f64(q), to_f64(hk) if L else None, np.abs(to_f64(hv)) if L else None, to_f64(kf),
                                      np.abs(to_f64(vf)), scale32(s))
        check_close(out, ref, "bf16", f"case {case}: Hq/Hkv {hq}/{hkv} F={F} T={T} L={L} splits={splits}", abs_v_out=bound)
        assert cache.len == L + F and same_bits(cache.k[L:], kf[:, T - 1]) and same_bits(cache.v[L:], vf[:, T - 1])


def test_package_used_before_torch_is_imported():
    """A fresh process that touches the library before it imports torch (here: a tuning call)
    must still find the device afterwards: library and torch share one HIP runtime, torch's,
    whichever of the two the program names first."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = (
        "import sys; sys.path.insert(0, %r)\n"
        "import paper_2503_09387_amd as vs\n"
        "vs.set_tuning(vs.TUNE_PREFILL_SPLITS, 0)\n"
        "import torch\n"
        "sh = vs.Shape.make(28, 4, 128, 'bf16', 0.0883883)\n"
        "ws = vs.make_workspace(sh, 8, 64, 2, 'cuda:0')\n"
        "e = torch.ones((4, 64), dtype=torch.float32, device='cuda:0'); c = torch.empty(64, device='cuda:0')\n"
        "vs.carrier_mean_pool(e, c, 'f32'); torch.cuda.synchronize()\n"
        "assert bool((c == 1).all())\n"
        "print('ok')\n" % root)
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=100)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout + r.stderr
