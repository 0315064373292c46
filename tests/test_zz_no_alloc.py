"""vs_decode_attn_static (decode attention over the library's own scratch array, nothing allocated)
against vs_decode_attn on the same inputs: same kernels, so the same bits, the appended rows and the
lengths included; two calls in a row, the second on a smaller input, so that what the first call
left in the array cannot leak into the second."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2503_09387_amd as vs
from gpu_util import DEV, check_close, lens_array, scale32, vs_shape, workspace
from synth import CONFIGS, cache_rows, decode_step_inputs, to_f64

pytestmark = pytest.mark.gpu

QW = CONFIGS["cfg2"]["shape"]


def _case(s, lens0, cap, seed):
    S = len(lens0)
    ks = torch.zeros((S, cap, s.n_kv_heads, s.head_dim), dtype=torch.bfloat16, device=DEV)
    vsl = torch.zeros_like(ks)
    for i in range(S):
        hk, hv = cache_rows(seed, s, max(lens0[i], 1), 0.5, stream=i)
        ks[i, :lens0[i]].copy_(hk[:lens0[i]])
        vsl[i, :lens0[i]].copy_(hv[:lens0[i]])
    q, kn, vn = decode_step_inputs(seed, s, S, 0.5, q_gain=4)
    return ks, vsl, q.to(DEV), kn.to(DEV), vn.to(DEV)


def test_decode_static_scratch_equals_decode_with_workspace():
    s = QW
    sh = vs_shape(s)
    assert vs.decode_static_scratch_bytes() == 16 << 20
    # first call: 16 ragged streams of up to 8319 rows; second call: 3 short streams
    for call, (lens0, cap) in enumerate((([8319, 640, 4000, 33, 1, 129] + [500 + 311 * i for i in range(10)], 8384),
                                         ([77, 2, 300], 512))):
        ks, vsl, q, kn, vn = _case(s, lens0, cap, 41 + call)
        ks2, vsl2 = ks.clone(), vsl.clone()
        ws = workspace(s, 0, cap, len(lens0))
        lens_a, lens_b = lens_array(lens0), lens_array(lens0)
        out_a = torch.full(q.shape, float("nan"), dtype=torch.bfloat16, device=DEV)
        out_b = torch.full(q.shape, float("nan"), dtype=torch.bfloat16, device=DEV)
        vs.decode_attn(sh, ks, vsl, lens_a, q, kn, vn, out_a, ws)
        # through the raw C ABI: no workspace argument at all
        rc = vs.lib().vs_decode_attn_static(ctypes.byref(sh), len(lens0), ks2.data_ptr(), vsl2.data_ptr(), cap, lens_b,
                                            q.data_ptr(), kn.data_ptr(), vn.data_ptr(), out_b.data_ptr(),
                                            ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert rc == 0, vs.status_string(rc)
        torch.cuda.synchronize()
        assert list(lens_a) == list(lens_b) == [n + 1 for n in lens0]
        assert torch.equal(out_a.view(torch.int16), out_b.view(torch.int16)), f"call {call}: outputs differ"
        assert torch.equal(ks, ks2) and torch.equal(vsl, vsl2), f"call {call}: appended rows differ"
        # and the existing entry point is itself held to the oracle
        i = 0
        okk = np.zeros((cap, s.n_kv_heads, s.head_dim))
        ovv = np.zeros_like(okk)
        okk[:lens0[i]], ovv[:lens0[i]] = to_f64(ks2[i, :lens0[i]].cpu()), to_f64(vsl2[i, :lens0[i]].cpu())
        ref, _ = oracle.decode(to_f64(q[i].cpu()), okk, ovv, lens0[i], to_f64(kn[i].cpu()), to_f64(vn[i].cpu()), scale32(s))
        check_close(out_b[i], ref, "bf16", f"static scratch, call {call}, stream 0")


def test_decode_static_rejects_what_does_not_fit_and_bad_arguments():
    s = QW
    sh = vs_shape(s)
    L = vs.lib()
    FAKE = 0x10000
    lens = lens_array([5])
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    assert L.vs_decode_attn_static(None, 1, FAKE, FAKE, 8, lens, FAKE, None, None, FAKE, st) == 1
    assert L.vs_decode_attn_static(ctypes.byref(sh), 0, FAKE, FAKE, 8, lens, FAKE, None, None, FAKE, st) == 2
    assert L.vs_decode_attn_static(ctypes.byref(sh), 1, None, FAKE, 8, lens, FAKE, None, None, FAKE, st) == 1
    assert L.vs_decode_attn_static(ctypes.byref(sh), 1, FAKE, FAKE, 8, lens, FAKE + 2, None, None, FAKE, st) == 6
    big = vs.Shape.make(512, 64, 128, "bf16")   # 64 KV heads x 8 query heads each: more partial results than the array holds
    assert vs.workspace_bytes(big, 0, 8, 1) > vs.decode_static_scratch_bytes()
    assert L.vs_decode_attn_static(ctypes.byref(big), 1, FAKE, FAKE, 8, lens, FAKE, None, None, FAKE, st) == 5
    assert list(lens) == [5]
