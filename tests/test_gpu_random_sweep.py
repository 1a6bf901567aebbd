"""Seeded random sweep over everything palu_attn_decode_multi takes at once: group sizes and
ranks, query heads per key/value head, query tokens per sequence, RoPE base (or none), key and
value latents in fp16 / bf16 / 4 / 3 / 2 bits independently, batch, ragged lengths, explicit
cache positions, and queries scaled by 1, 4, 8 or 12 (logits up to about +-40).  Each case is compared with the oracle (fed the same dequantized latents).
A second sweep runs whole decode steps (append + attend) through both weight layouts."""

import numpy as np
import pytest
import torch

import paper_2407_21118_amd as P
from oracle import palu_oracle as O
from workloads import synth

pytestmark = pytest.mark.gpu

from gpu_util import TOL_FP, TOL_I4, rel_err, say, to_dev  # noqa: E402


def one_case(seed):
    rng = np.random.default_rng([4242, seed])
    qpk = int(rng.choice([1, 1, 2, 3, 4, 8]))
    n_q = int(rng.choice([1, 1, 2, 3, 5]))
    theta = float(rng.choice([0.0, 10000.0, 10000.0, 500000.0]))
    kb = int(rng.choice([16, 16, 4, 3, 2]))
    vb = int(rng.choice([16, 16, 4, 3, 2]))
    dtype = "bf16" if (kb == 16 and vb == 16 and rng.random() < 0.3) else "f16"
    quant = kb != 16 or vb != 16
    sizes = [int(rng.choice([1, 2, 4, 8] if qpk * n_q <= 4 else [1, 2, 4])) for _ in range(int(rng.integers(1, 5)))]
    while sum(sizes) * qpk * n_q > 256:
        sizes.pop()
    step = 128 if quant else 32

    def ranks():
        return [int(rng.integers(1, min(512, s * 128) // step + 1)) * step for s in sizes]

    kr, vr = ranks(), ranks()
    head_off = [0] + list(np.cumsum(sizes))
    layer = synth.Layer(int(head_off[-1]), 128, head_off, [0] + list(np.cumsum(kr)), [0] + list(np.cumsum(vr)),
                        rope_theta=theta, q_per_kv=qpk)
    B = int(rng.integers(1, 4))
    L = int(rng.choice([1, 7, 32, 33, 64, 100, 257, 300]))
    case = synth.make_case_orthonormal(layer, B, L, seed=1000 + seed, dtype=dtype)
    lens = np.array([L] + [int(rng.integers(1, L + 1)) for _ in range(B - 1)], np.int32)
    # logits of order +-3 (unit queries) up to +-40, the sizes trained models produce: the tolerance does not change
    q_scale = float(np.random.default_rng([4243, seed]).choice([1.0, 1.0, 4.0, 8.0, 12.0]))
    q = synth.round_to(rng.standard_normal((B, n_q, layer.n_q_heads, 128)) * q_scale, dtype)
    q_len = np.maximum(1, lens[:, None] - n_q + np.arange(n_q)[None, :] + 1).astype(np.int32)
    q_pos = (q_len - 1 + int(rng.integers(0, 3000))).astype(np.int32)
    k_pos = np.sort(rng.choice(8192, size=L, replace=False)).astype(np.int32) if rng.random() < 0.4 else None
    act = P.PALU_F16 if dtype == "f16" else P.PALU_BF16
    qd = {4: P.PALU_I4, 3: P.PALU_I3, 2: P.PALU_I2}
    desc = P.LayerDesc(layer.n_heads, 128, layer.group_head_off, layer.k_rank_off, layer.v_rank_off, act,
                       qd.get(kb, act), qd.get(vb, act), 128, theta, qpk)
    kw = {}
    Hk_ref, Hv_ref = case.Hk, case.Hv

    def quantized(H, bits, prefix):
        pk, s, z = O.quant_latent(H, bits=bits)
        kw[prefix + "_scale"] = torch.from_numpy(s.view(np.int16)).cuda().view(torch.float16)
        kw[prefix + "_zero"] = torch.from_numpy(z.view(np.int16)).cuda().view(torch.float16)
        return torch.from_numpy(pk).cuda(), O.dequant_latent(pk, s, z, bits=bits)

    hk, hv = to_dev(case.Hk, dtype), to_dev(case.Hv, dtype)
    if kb != 16:
        hk, Hk_ref = quantized(case.Hk, kb, "hk")
    if vb != 16:
        hv, Hv_ref = quantized(case.Hv, vb, "hv")
    n_pos = max(L, (int(k_pos.max()) + 1) if k_pos is not None else L)
    table = P.palu_rope_table_init(theta, 128, n_pos)
    if k_pos is not None:
        kw["k_pos"] = torch.from_numpy(k_pos).cuda()
    # the score kernel's schedules: 0 = the library's choice, 8 / 4 = wavefronts per workgroup of the general kernel
    waves = int(np.random.default_rng([4244, seed]).choice([0, 0, 8, 4]))
    P.palu_set_option("score_waves", waves)
    try:
        out = P.palu_attn_decode_multi(desc, B, n_q, L, L, to_dev(q, dtype), torch.from_numpy(q_pos).cuda(), hk, hv,
                                       to_dev(case.Bk, dtype), to_dev(case.Bv, dtype), table, n_pos,
                                       q_len=torch.from_numpy(q_len).cuda(), seq_lens=torch.from_numpy(lens).cuda(), **kw)
        torch.cuda.synchronize()
    finally:
        P.palu_set_option("score_waves", 0)
    got = out.cpu().numpy()
    ref = O.attn_decode_multi(q, q_pos, q_len, Hk_ref, Hv_ref, case.Bk, case.Bv, layer.group_head_off, layer.k_rank_off,
                              layer.v_rank_off, 128, theta, k_pos, qpk)
    whole, rows = rel_err(got.reshape(B, -1, 128), ref.reshape(B, -1, 128))
    tol = TOL_I4 if quant else TOL_FP
    what = (f"seed {seed}: q_per_kv={qpk} n_q={n_q} q_scale={q_scale:g} theta={theta:g} k_bits={kb} v_bits={vb} {dtype} groups={sizes} "
            f"k_ranks={kr} v_ranks={vr} B={B} L={L} k_pos={k_pos is not None} score_waves={waves}")
    return what, bool(np.isfinite(got).all()), max(whole, rows), tol


@pytest.mark.parametrize("first", [0, 40, 80])
def test_random_sweep(first):
    worst = 0.0
    for seed in range(first, first + 40):
        what, finite, err, tol = one_case(seed)
        worst = max(worst, err / tol)
        assert finite and err <= tol, f"{what}: error {err:.3e} above {tol}"
    say(f"[sweep] seeds {first}..{first + 39}: worst error / tolerance {worst:.2f}")


def step_case(seed):
    """One random decode step (append, then attend) through both weight layouts: palu_decode_step with
    A [d, R] and palu_decode_step_t with A^T [R, d]; the appended rows against the oracle's projection,
    the outputs against the oracle's attention over each call's own cache."""
    rng = np.random.default_rng([777, seed])
    qpk = int(rng.choice([1, 1, 2, 4]))
    theta = float(rng.choice([0.0, 10000.0, 10000.0, 500000.0]))
    dtype = "bf16" if rng.random() < 0.3 else "f16"
    sizes = [int(rng.choice([1, 2, 4, 8])) for _ in range(int(rng.integers(1, 5)))]
    kr = [int(rng.integers(1, min(512, s * 128) // 32 + 1)) * 32 for s in sizes]
    vr = [int(rng.integers(1, min(512, s * 128) // 32 + 1)) * 32 for s in sizes]
    head_off = [0] + list(np.cumsum(sizes))
    layer = synth.Layer(int(head_off[-1]), 128, head_off, [0] + list(np.cumsum(kr)), [0] + list(np.cumsum(vr)),
                        rope_theta=theta, q_per_kv=qpk)
    B = int(rng.choice([1, 1, 2, 3, 5, 8, 9]))
    L = int(rng.choice([1, 7, 33, 100, 257]))
    case = synth.make_case_orthonormal(layer, B, L, seed=2000 + seed, dtype=dtype)
    d = layer.n_q_heads * 128
    A = {side: synth.round_to(rng.standard_normal((d, R)) / np.sqrt(d), dtype) for side, R in (("k", layer.R_k), ("v", layer.R_v))}
    x = synth.round_to(rng.standard_normal((B, d)), dtype)
    lens = np.array([L] + [int(rng.integers(1, L + 1)) for _ in range(B - 1)], np.int32)
    rows = (np.arange(B) * L + lens - 1).astype(np.int32)          # the new token is each sequence's last attended row
    q_pos = (lens - 1 + int(rng.integers(0, 3000))).astype(np.int32)
    act = P.PALU_F16 if dtype == "f16" else P.PALU_BF16
    desc = P.LayerDesc(layer.n_heads, 128, layer.group_head_off, layer.k_rank_off, layer.v_rank_off, act, act, act, 128, theta, qpk)
    n_pos = int(q_pos.max()) + 1 + L
    table = P.palu_rope_table_init(theta, 128, n_pos)
    common = dict(q=to_dev(case.q, dtype), q_pos=torch.from_numpy(q_pos).cuda(), Bk=to_dev(case.Bk, dtype), Bv=to_dev(case.Bv, dtype))
    d_rows, d_lens, xd = torch.from_numpy(rows).cuda(), torch.from_numpy(lens).cuda(), to_dev(x, dtype)
    eps = 2.0 ** -11 if dtype == "f16" else 2.0 ** -8
    worst = 0.0
    for transposed in (False, True):
        hk, hv = to_dev(case.Hk, dtype), to_dev(case.Hv, dtype)
        if transposed:
            got = P.palu_decode_step_t(desc, B, L, L, xd, to_dev(np.ascontiguousarray(A["k"].T), dtype),
                                       to_dev(np.ascontiguousarray(A["v"].T), dtype), d_rows, common["q"], common["q_pos"], hk, hv,
                                       common["Bk"], common["Bv"], table, n_pos, seq_lens=d_lens)
        else:
            got = P.palu_decode_step(desc, B, L, L, xd, to_dev(A["k"], dtype), to_dev(A["v"], dtype), d_rows, common["q"],
                                     common["q_pos"], hk, hv, common["Bk"], common["Bv"], table, n_pos, seq_lens=d_lens)
        torch.cuda.synchronize()
        Hk = hk.float().cpu().numpy().astype(np.float64)
        Hv = hv.float().cpu().numpy().astype(np.float64)
        keep = np.setdiff1d(np.arange(B * L), rows)
        for H, H0, side in ((Hk, case.Hk, "k"), (Hv, case.Hv, "v")):
            ref = O.encode(x, A[side])
            flat = H.reshape(B * L, -1)
            err = np.abs(flat[rows] - ref).max(axis=1) / np.abs(ref).max(axis=1)
            assert err.max() <= eps * 1.05 + 1e-6, (seed, transposed, side, err.max())
            np.testing.assert_array_equal(flat[keep], H0.reshape(B * L, -1)[keep])
        want = O.attn_decode(case.q, q_pos, Hk, Hv, case.Bk, case.Bv, layer.group_head_off, layer.k_rank_off,
                             layer.v_rank_off, 128, theta, None, lens, qpk)
        out = got.cpu().numpy()
        assert np.isfinite(out).all()
        whole, per_row = rel_err(out, want)
        worst = max(worst, whole, per_row)
        assert max(whole, per_row) <= TOL_FP, (seed, transposed, sizes, kr, vr, qpk, theta, dtype, B, L, whole, per_row)
    return worst


def test_sweep_decode_step_both_weight_layouts():
    worst = 0.0
    for seed in range(30):
        worst = max(worst, step_case(seed))
    say(f"[sweep-step] 30 cases x 2 weight layouts, worst rel err {worst:.3e}")
