"""The C-ABI library on a machine without a GPU: it loads, exports what the header declares,
and refuses bad arguments before launching anything."""
import ctypes
import os
import re
import sys

import pytest

import paper_2503_09387_amd as vs
from paper_2503_09387_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000001000  # 16-byte aligned, never dereferenced: every call below must fail first
ODD = FAKE + 4


def _declared():
    text = open(os.path.join(ROOT, "include", "videoscan.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vs_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported():
    names = _declared()
    assert {"vs_frame_prefill_attn", "vs_carrier_compact_append", "vs_decode_attn",
            "vs_carrier_mean_pool", "vs_workspace_bytes"} <= set(names)
    lib = vs.lib()
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in the header but not exported"
    assert sorted(binding.EXPORTS) == names


def test_status_strings():
    seen = {vs.status_string(c) for c in range(8)}
    assert len(seen) == 8 and "ok" in seen
    assert vs.status_string(99) == "unknown status"


def _shape(hq=28, hkv=4, d=128, dt=vs.VS_BF16, scale=None):
    return vs.Shape.make(hq, hkv, d, dt, scale)


def _cache(k=FAKE, v=FAKE, cap=8, ln=2):
    return binding._CCache(k, v, cap, ln)


def _prefill(shape, cache, q=FAKE, kf=FAKE, vf=FAKE, n=4, out=FAKE, ws=FAKE, wsb=1 << 30):
    return vs.lib().vs_frame_prefill_attn(ctypes.byref(shape), ctypes.byref(cache), q, kf, vf, n, out,
                                          ws, wsb, None)


def test_shape_validation():
    c = _cache()
    assert _prefill(_shape(hq=28, hkv=5), c) == 2          # Hq % Hkv
    assert _prefill(_shape(hq=36, hkv=4), c) == 3          # ratio above 8
    assert _prefill(_shape(d=96), c) == 3                  # head_dim
    assert _prefill(_shape(d=64), c) == 3                  # bf16 needs 128
    assert _prefill(_shape(dt=7), c) == 3
    assert _prefill(_shape(scale=float("nan")), c) == 2
    assert _prefill(_shape(scale=-1.0), c) == 2
    assert vs.lib().vs_frame_prefill_attn(None, ctypes.byref(c), FAKE, FAKE, FAKE, 4, FAKE, FAKE, 64, None) == 1
    assert vs.workspace_bytes(_shape(d=96), 16, 16, 1) == 0
    assert vs.workspace_bytes(_shape(), 170, 4552, 16) >= 256


def test_prefill_argument_errors():
    s = _shape()
    assert _prefill(s, _cache(), q=None) == 1
    assert _prefill(s, _cache(), out=None) == 1
    assert _prefill(s, _cache(k=None)) == 1
    assert _prefill(s, _cache(), n=0) == 2
    assert _prefill(s, _cache(), n=5000) == 2
    assert _prefill(s, _cache(ln=9)) == 4                  # len > capacity
    assert _prefill(s, _cache(ln=-1)) == 2
    assert _prefill(s, _cache(), q=ODD) == 6
    assert _prefill(s, _cache(k=ODD)) == 6
    assert _prefill(s, _cache(), ws=None) == 5
    assert _prefill(s, _cache(), wsb=16) == 5
    assert _prefill(s, _cache(), ws=ODD) == 6


def test_question_prefill_argument_errors_leave_len_untouched():
    s = _shape()

    def call(c, q=FAKE, kt=FAKE, vt=FAKE, n=4, out=FAKE, ws=FAKE, wsb=1 << 30):
        return vs.lib().vs_question_prefill_append(ctypes.byref(s), ctypes.byref(c), q, kt, vt, n, out, ws, wsb, None)

    c = _cache(cap=8, ln=5)
    assert call(c, n=4) == 4 and c.len == 5                # 5 + 4 rows do not fit 8
    assert call(_cache(cap=8, ln=8), n=1) == 4
    assert call(c, q=None) == 1 and call(c, kt=None, n=3) == 1 and call(c, out=None, n=3) == 1
    assert call(c, n=0) == 2 and call(c, n=5000) == 2
    assert call(c, vt=ODD, n=3) == 6 and call(c, ws=None, n=3) == 5 and call(c, wsb=16, n=3) == 5
    assert call(_cache(k=None, cap=8, ln=0), n=3) == 1     # room is needed, so the cache must exist
    assert c.len == 5


def test_append_argument_errors_leave_len_untouched():
    s = _shape()
    L = vs.lib()
    row = ctypes.c_int32(-7)

    def app(cache, kf=FAKE, vf=FAKE, n=4, ci=3):
        return L.vs_carrier_compact_append(ctypes.byref(s), ctypes.byref(cache), kf, vf, n, ci,
                                           ctypes.byref(row), None)

    full = _cache(cap=8, ln=8)
    assert app(full) == 4 and full.len == 8 and row.value == -7
    c = _cache()
    assert app(c, ci=4) == 2 and app(c, ci=-1) == 2 and app(c, n=0) == 2
    assert app(c, kf=None) == 1 and app(c, vf=ODD) == 6
    assert app(_cache(k=None)) == 1
    assert c.len == 2
    # fused prefill+compaction refuses a full cache before launching
    assert L.vs_frame_prefill_compact(ctypes.byref(s), ctypes.byref(full), FAKE, FAKE, FAKE, 4, FAKE,
                                      ctypes.byref(row), FAKE, 1 << 30, None) == 4
    assert full.len == 8


def test_batched_append_argument_errors():
    s = _shape()
    L = vs.lib()
    lens = (ctypes.c_int32 * 3)(1, 8, 2)

    def go(n=3, cap=8, ci=3, ks=FAKE, ws=None, wsb=0, lens_=lens):
        return L.vs_carrier_compact_append_batched(ctypes.byref(s), n, ks, FAKE, cap, lens_, FAKE, FAKE, 4,
                                                   ci, None, ws, wsb, None)

    assert go() == 4 and list(lens) == [1, 8, 2]           # one cache is full: nothing happens
    assert go(n=0) == 2 and go(ci=9) == 2 and go(ks=None) == 1 and go(ks=ODD) == 6
    many = (ctypes.c_int32 * 100)(*([0] * 100))
    assert go(n=100, lens_=many) == 5                      # needs workspace for the lengths
    assert list(many) == [0] * 100


def test_decode_argument_errors():
    s = _shape()
    L = vs.lib()
    lens = (ctypes.c_int32 * 2)(5, 8)

    def dec(n=2, cap=8, q=FAKE, kn=FAKE, vn=FAKE, ws=FAKE, wsb=1 << 30, lens_=lens):
        return L.vs_decode_attn(ctypes.byref(s), n, FAKE, FAKE, cap, lens_, q, kn, vn, FAKE, ws, wsb, None)

    assert dec() == 4 and list(lens) == [5, 8]             # stream 1 has no room for the new row
    assert dec(kn=None) == 1                               # k_new without v_new
    assert dec(n=0) == 2 and dec(n=2000) == 2 and dec(q=None) == 1 and dec(q=ODD) == 6
    ok_lens = (ctypes.c_int32 * 2)(5, 7)
    assert dec(lens_=ok_lens, ws=None) == 5 and dec(lens_=ok_lens, wsb=8) == 5
    empty = (ctypes.c_int32 * 2)(0, 3)
    assert dec(lens_=empty, kn=None, vn=None) == 2         # a stream with nothing to attend to
    assert list(ok_lens) == [5, 7] and list(empty) == [0, 3]


def test_decode_workspace_holds_every_partial_slot():
    """The decode workspace has a slot per (workgroup + stream of the segment), each with a row per
    (KV head, sub-range of the share, query head of the group): 4 wavefronts per workgroup are 1, 2
    or 4 KV heads, the rest sub-ranges.  Shapes whose KV head count is not a multiple of 4 used to
    be sized short."""
    for hq, hkv in ((28, 4), (6, 3), (12, 6), (8, 1), (16, 2), (7, 7), (40, 5), (64, 8)):
        nh = 4 if hkv % 4 == 0 else 2 if hkv % 2 == 0 else 1
        rows = (1024 + 16) * hkv * (4 // nh) * (hq // hkv)
        assert vs.workspace_bytes(_shape(hq, hkv, 128, vs.VS_BF16), 0, 1000, 16) >= rows * (128 * 2 + 16), (hq, hkv)


def test_mean_pool_and_tuning_argument_errors():
    L = vs.lib()
    assert L.vs_carrier_mean_pool(None, 4, 8, 0, FAKE, None) == 1
    assert L.vs_carrier_mean_pool(FAKE, 0, 8, 0, FAKE, None) == 2
    assert L.vs_carrier_mean_pool(FAKE, 4, 6, 0, FAKE, None) == 2   # d % 4
    assert L.vs_carrier_mean_pool(FAKE, 4, 12, 1, FAKE, None) == 2  # d % 8 for bf16
    assert L.vs_carrier_mean_pool(FAKE, 4, 8, 5, FAKE, None) == 3
    assert L.vs_carrier_mean_pool(ODD, 4, 8, 0, FAKE, None) == 6
    assert L.vs_set_tuning(0, 33) == 2 and L.vs_set_tuning(1, 3) == 2
    assert L.vs_set_tuning(2, 100) == 2 and L.vs_set_tuning(9, 1) == 2
    assert L.vs_set_tuning(3, 1) == 2 and L.vs_set_tuning(3, 0) == 2      # no such knob
    assert L.vs_set_tuning(0, 4) == 0 and L.vs_set_tuning(0, 0) == 0
    assert L.vs_set_tuning(4, 5) == 2 and L.vs_set_tuning(4, 1) == 0 and L.vs_set_tuning(4, 2) == 0 and L.vs_set_tuning(4, 0) == 0
    assert L.vs_set_tuning(99, 7) == 2 and L.vs_set_tuning(99, 0) == 2    # no such knob


def test_frame_projection_argument_errors():
    s = _shape()

    def call(e=FAKE, n=169, d=3584, w=FAKE, q=FAKE, k=FAKE, v=FAKE, c=None, shape=s):
        return vs.lib().vs_frame_qkv_project(ctypes.byref(shape), e, n, d, w, q, k, v, c, None)

    assert call(e=None) == 1 and call(w=None) == 1 and call(q=None) == 1 and call(v=None) == 1
    assert call(n=0) == 2 and call(n=192) == 2                 # the carrier makes it at most 192 rows
    assert call(d=0) == 2 and call(d=100) == 2                 # multiples of 64
    assert call(shape=_shape(hq=4, hkv=2, d=64, dt=vs.VS_F32)) == 3
    assert call(e=ODD) == 6 and call(c=ODD) == 6 and call(k=ODD) == 6


def test_dense_layer_argument_errors():
    L = vs.lib()
    assert L.vs_rmsnorm(None, FAKE, 4, 64, ctypes.c_float(1e-6), FAKE, None) == 1
    assert L.vs_rmsnorm(FAKE, FAKE, 0, 64, ctypes.c_float(1e-6), FAKE, None) == 2
    assert L.vs_rmsnorm(FAKE, FAKE, 4, 60, ctypes.c_float(1e-6), FAKE, None) == 2          # d % 8
    assert L.vs_rmsnorm(FAKE, FAKE, 4, 64, ctypes.c_float(-1.0), FAKE, None) == 2
    assert L.vs_rmsnorm(FAKE, FAKE, 4, 64, ctypes.c_float(float("nan")), FAKE, None) == 2
    assert L.vs_rmsnorm(FAKE, ODD, 4, 64, ctypes.c_float(1e-6), FAKE, None) == 6

    def lin(x=FAKE, w=FAKE, t=170, k=3584, n=3584, mode=0, res=None, out=FAKE, ws=FAKE, wsb=1 << 30):
        return L.vs_linear(x, w, t, k, n, mode, res, out, ws, wsb, None)

    assert lin(x=None) == 1 and lin(w=None) == 1 and lin(out=None) == 1
    assert lin(mode=1) == 1 and lin(mode=1, res=FAKE) != 1            # the residual is required in its mode only
    assert lin(mode=3) == 2 and lin(mode=-1) == 2
    assert lin(t=0) == 2 and lin(t=193) == 2
    assert lin(k=0) == 2 and lin(k=100) == 2 and lin(n=0) == 2 and lin(n=7) == 2
    assert lin(x=ODD) == 6 and lin(out=ODD) == 6 and lin(mode=1, res=ODD) == 6 and lin(ws=ODD) == 6
    need = L.vs_linear_workspace_bytes(170, 3584, 3584)
    assert need > 0 and lin(ws=None) == 5 and lin(wsb=need - 1) == 5    # this shape splits K
    assert L.vs_linear_workspace_bytes(170, 3584, 37888) == 0           # this one does not
    assert L.vs_linear_workspace_bytes(0, 3584, 3584) == 0 and L.vs_linear_workspace_bytes(170, 100, 3584) == 0


def test_decoder_layer_argument_errors():
    L = vs.lib()
    s = _shape()

    def weights(d=3584, f=18944, eps=1e-6, **kw):
        p = dict(norm1=FAKE, w_qkv=FAKE, w_o=FAKE, norm2=FAKE, w_gate_up=FAKE, w_down=FAKE)
        p.update(kw)
        return binding._CLayerWeights(p["norm1"], p["w_qkv"], p["w_o"], p["norm2"], p["w_gate_up"], p["w_down"], d, f, eps)

    def cache(cap=100, ln=10):
        return binding._CCache(FAKE, FAKE, cap, ln)

    def layer(w=None, c=None, h=FAKE, t=170, out=FAKE, ws=FAKE, wsb=1 << 40, shape=s):
        w = w or weights()
        c = c or cache()
        return L.vs_frame_decoder_layer(ctypes.byref(shape), ctypes.byref(w), ctypes.byref(c), h, t, out, ws, wsb, None)

    need = L.vs_layer_workspace_bytes(ctypes.byref(s), ctypes.byref(weights()), 170)
    assert need > 170 * 18944 * 2
    assert L.vs_layer_workspace_bytes(ctypes.byref(s), ctypes.byref(weights(d=100)), 170) == 0
    assert L.vs_layer_workspace_bytes(ctypes.byref(s), ctypes.byref(weights()), 193) == 0
    assert layer(h=None) == 1 and layer(out=None) == 1 and layer(w=weights(w_o=None)) == 1
    assert layer(t=0) == 2 and layer(t=193) == 2
    assert layer(w=weights(d=3600)) == 2 and layer(w=weights(f=1000)) == 2 and layer(w=weights(eps=-1.0)) == 2
    assert layer(shape=_shape(hq=4, hkv=2, d=64, dt=vs.VS_F32)) == 3
    full = cache(cap=10, ln=10)
    assert layer(c=full) == 4 and full.len == 10                        # reported before anything is launched
    assert layer(ws=None) == 5 and layer(wsb=need - 1) == 5
    assert layer(h=ODD) == 6 and layer(w=weights(w_down=ODD)) == 6 and layer(ws=ODD) == 6


def test_memory_bank_argument_errors():
    L = vs.lib()
    assert L.vs_memory_bank_workspace_bytes(0) == 0 and L.vs_memory_bank_workspace_bytes(1025) == 0
    assert L.vs_memory_bank_workspace_bytes(128) >= 8 * 128

    def bank(e=FAKE, cap=4, ln=0, d=8, dt=vs.VS_BF16):
        return binding._CBank(e, cap, ln, d, dt)

    def push(b, e_new=FAKE, policy=0, victim=FAKE, ws=FAKE, wsb=1 << 20):
        return L.vs_memory_bank_push(ctypes.byref(b), e_new, policy, victim, ws, wsb, None)

    assert push(bank(e=None)) == 1 and push(bank(), e_new=None) == 1 and push(bank(), victim=None) == 1
    assert push(bank(dt=7)) == 3
    assert push(bank(cap=0)) == 2 and push(bank(cap=2000)) == 2 and push(bank(ln=5)) == 2
    assert push(bank(d=4)) == 2                                    # 8 bytes per row: not a multiple of 16
    assert push(bank(), policy=2) == 2
    assert push(bank(e=ODD)) == 6 and push(bank(), victim=FAKE + 2) == 6
    b = bank(ln=4)
    assert push(b, ws=None) == 5 and push(b, wsb=8) == 5 and b.len == 4
    # the K/V side
    sh = _shape()

    def evict(caches, n=1, first=2, cap=4, k=FAKE, v=FAKE, stride=0, victim=FAKE):
        arr = (binding._CCache * len(caches))(*caches)
        rc = L.vs_carrier_evict_append(ctypes.byref(sh), n, arr, first, cap, k, v, stride, victim, None)
        return rc, [c.len for c in arr]

    assert evict([_cache()], k=None)[0] == 1 and evict([_cache()], victim=None)[0] == 1
    assert evict([_cache()], n=0)[0] == 2 and evict([_cache()], cap=0)[0] == 2 and evict([_cache()], stride=8)[0] == 2
    assert evict([_cache(ln=1)])[0] == 2                           # fewer rows than the prefix
    assert evict([_cache(ln=7)])[0] == 2                           # more carriers than the bank holds
    assert evict([_cache(cap=5)]) == (4, [2])                      # prefix + bank does not fit, length untouched
    assert evict([_cache(), _cache(ln=3)], n=2, stride=1024)[0] == 2   # layers out of step
    assert evict([_cache()], k=ODD)[0] == 6


def test_runs_of_frames_argument_errors():
    L = vs.lib()
    sh = _shape()
    L.vs_frames_workspace_bytes.restype = ctypes.c_size_t
    assert L.vs_frames_workspace_bytes(ctypes.byref(sh), 0, 170, 100) == 0
    assert L.vs_frames_workspace_bytes(ctypes.byref(sh), 65, 10, 100) == 0
    assert L.vs_frames_workspace_bytes(ctypes.byref(sh), 8, 1000, 100) == 0      # more than 4096 tokens in the run
    assert L.vs_frames_workspace_bytes(ctypes.byref(_shape(4, 1, 64, vs.VS_F32)), 2, 10, 100) == 0
    need = L.vs_frames_workspace_bytes(ctypes.byref(sh), 4, 170, 5000)
    assert need > 0 and L.vs_frames_workspace_bytes(ctypes.byref(sh), 8, 170, 5000) >= need

    def run(cache, q=FAKE, kf=FAKE, vf=FAKE, F=2, n=4, out=FAKE, ws=FAKE, wsb=1 << 30, shape=sh):
        return L.vs_frames_prefill_attn(ctypes.byref(shape), ctypes.byref(cache), q, kf, vf, F, n, out, ws, wsb, None)

    c = _cache(cap=8, ln=2)
    assert run(c, q=None) == 1 and run(c, out=None) == 1
    assert run(c, F=0) == 2 and run(c, F=65) == 2 and run(c, n=0) == 2 and run(c, F=8, n=1000) == 2
    assert run(c, shape=_shape(4, 1, 64, vs.VS_F32)) == 3
    assert run(_cache(cap=3, ln=2)) == 4 and run(c, F=7) == 4     # no room for the run's carriers
    assert run(c, kf=ODD) == 6
    assert run(c, ws=None) == 5 and run(c, wsb=64) == 5
    assert c.len == 2


def test_product_path_does_not_touch_the_oracle():
    """The package must not import or mention the oracle: it is test infrastructure only."""
    pkg = os.path.join(ROOT, "paper_2503_09387_amd")
    for base, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(base, f)).read()
                assert "oracle" not in text.lower(), f"{f} refers to the oracle"


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_LIB", None)
    monkeypatch.setattr(binding, "_HERE", str(tmp_path))
    with pytest.raises(RuntimeError):
        binding.lib()


def test_prefill_workgroup_placement_map(tmp_path):
    """The id -> (unit, split, XCD) mapping behind the in-kernel merge of the bf16 prefill, checked on
    the host for every (units, splits, XCD count) the planner can emit (tests/prefill_map_check.cpp
    includes the header the kernel uses)."""
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = str(tmp_path / "map_check")
    subprocess.run(["g++", "-O2", "-std=c++17", "-I", os.path.join(root, "paper_2503_09387_amd", "csrc"),
                    os.path.join(root, "tests", "prefill_map_check.cpp"), "-o", exe], check=True)
    r = subprocess.run([exe], capture_output=True, text=True)
    assert r.returncode == 0 and r.stdout.startswith("ok"), r.stdout + r.stderr


def test_bench_refuses_more_than_one_gpu():
    """bench.py --gpus N with N above 1 exits with a message that says so (nothing here uses a second GPU)."""
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in (r.stderr + r.stdout) and r.stdout.strip() == ""
