"""The decode entry point that allocates nothing (static device scratch inside the
library) against palu_attn_decode with a caller workspace: same kernels, same launch
geometry, so the outputs must be bit-identical; two calls in a row on the same GPU,
the second on a smaller input (the scratch then still holds the first call's data).
The first case is also held to the oracle's tolerance."""

import ctypes

import numpy as np
import pytest
import torch

import paper_2407_21118_amd as P
from workloads import synth

pytestmark = pytest.mark.gpu

from gpu_util import TOL_FP, make_desc, rel_err, run_oracle, say, to_dev  # noqa: E402


def _device_inputs(case):
    layer = case.layer
    d = dict(desc=make_desc(layer, case.dtype), q=to_dev(case.q, case.dtype),
             q_pos=torch.from_numpy(np.asarray(case.q_pos, np.int32)).cuda(),
             hk=to_dev(case.Hk, case.dtype), hv=to_dev(case.Hv, case.dtype),
             Bk=to_dev(case.Bk, case.dtype), Bv=to_dev(case.Bv, case.dtype),
             seq_lens=None if case.seq_lens is None else torch.from_numpy(np.asarray(case.seq_lens, np.int32)).cuda())
    d["table"] = P.palu_rope_table_init(layer.rope_theta, layer.d_head, case.seq)
    return d


def _both(case):
    d = _device_inputs(case)
    B, L = case.batch, case.seq
    ref = P.palu_attn_decode(d["desc"], B, L, L, d["q"], d["q_pos"], d["hk"], d["hv"], d["Bk"], d["Bv"], d["table"], L,
                             seq_lens=d["seq_lens"])
    out = torch.full((B, d["desc"].n_q_heads, d["desc"].d_head), float("nan"), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    P.palu_attn_decode_noalloc(d["desc"], B, L, L, d["q"], d["q_pos"], d["hk"], d["hv"], d["Bk"], d["Bv"], d["table"], L,
                               out, seq_lens=d["seq_lens"])
    torch.cuda.synchronize()
    return ref.cpu().numpy(), out.cpu().numpy()


def test_noalloc_matches_workspace_entry_point_twice():
    layer = synth.config_layer("2")
    big = synth.make_case_svd(layer, 2, 777, seed=0)
    big.seq_lens = np.array([777, 300], np.int32)
    big.q_pos = np.array([776, 299], np.int32)
    say("[noalloc] call 1: 7B shape, batch 2, L 777")
    ref, got = _both(big)
    assert np.isfinite(got).all()
    assert np.array_equal(ref, got)
    whole, rows = rel_err(got, run_oracle(big))
    say(f"          vs oracle whole={whole:.3e} rows={rows:.3e}")
    assert whole <= TOL_FP and rows <= TOL_FP

    small_layer = synth.config_layer("1")
    small = synth.make_case_orthonormal(small_layer, 1, 100, seed=1)
    say("[noalloc] call 2: 8 heads, batch 1, L 100 (smaller than the first)")
    ref, got = _both(small)
    assert np.isfinite(got).all()
    assert np.array_equal(ref, got)
    whole, rows = rel_err(got, run_oracle(small))
    assert whole <= TOL_FP and rows <= TOL_FP


def test_noalloc_rejects_sizes_beyond_the_static_scratch():
    layer = synth.config_layer("2")
    desc = make_desc(layer, "f16")
    lib = P.load_library()
    need = P.palu_attn_decode_workspace_bytes(desc, 64, 65536)
    assert need > 32 * 1024 * 1024
    one = torch.zeros(16, dtype=torch.uint8, device="cuda")      # valid pointers; nothing is launched
    vp = ctypes.c_void_p
    st = lib.palu_attn_decode_noalloc(desc.ref(), 64, 65536, 65536, vp(one.data_ptr()), vp(one.data_ptr()),
                                      vp(one.data_ptr()), None, None, vp(one.data_ptr()), None, None, None, None,
                                      vp(one.data_ptr()), vp(one.data_ptr()), vp(one.data_ptr()), 65536,
                                      vp(one.data_ptr()), None)
    assert st == -3
