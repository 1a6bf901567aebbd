"""Parity at the benchmark's full sizes, in the launch configuration bench.py
times: the HIP path runs the whole configuration on the GPU; the CPU oracle
recomputes it from the same bits, one whole sequence (every head) at a time, for
every sequence of the batch.  Only where a full pass would take minutes (one
rank-2048 latent shared by 32 heads, a 1.2 M-token sequence) does the oracle take
some whole sequences or sampled (sequence, group, heads) slices instead."""

import numpy as np
import pytest
import torch

import paper_2407_21118_amd as P
from oracle import palu_oracle as O
from workloads import device as wd
from workloads import synth

pytestmark = pytest.mark.gpu

from gpu_util import TOL_FP, TOL_I4, make_desc, rel_err, say  # noqa: E402


def group_slice(layer, j, heads):
    """Layer holding only `heads` (indices inside group j) of group j."""
    rk = layer.k_rank_off[j + 1] - layer.k_rank_off[j]
    rv = layer.v_rank_off[j + 1] - layer.v_rank_off[j]
    return synth.Layer(len(heads), layer.d_head, [0, len(heads)], [0, rk], [0, rv], layer.rope_theta,
                       q_per_kv=layer.q_per_kv)


def b_slice(flat, layer, which, j, heads):
    """Columns of group j's reconstruction matrix that belong to `heads`."""
    off = layer.k_rank_off if which == "k" else layer.v_rank_off
    start = sum((off[i + 1] - off[i]) * layer.group_size(i) * layer.d_head for i in range(j))
    r, w = off[j + 1] - off[j], layer.group_size(j) * layer.d_head
    Bj = flat[start:start + r * w].reshape(r, w)
    cols = np.concatenate([np.arange(u * layer.d_head, (u + 1) * layer.d_head) for u in heads])
    return np.ascontiguousarray(Bj[:, cols]).reshape(-1)


def run_full(cfg, samples=None, k_i4=False, v_i4=False, tol=TOL_FP, no_rope=False, bits=4, seq=None, seqs=None,
             q_scale=1.0):
    """samples: (sequence, group, heads) slices for the oracle; None: whole sequences, all of the batch or `seqs`.
    q_scale: the queries are multiplied by it (logits of tens)."""
    layer = None
    if no_rope:
        import dataclasses
        layer = dataclasses.replace(synth.config_layer(cfg.split("-")[0]), rope_theta=0.0)
    case = wd.make_device_case(cfg, seed=0, n_sets=1, layer=layer, seq=seq)
    layer, B, L = case.layer, case.batch, case.seq
    say(f"[full] cfg {cfg} B={B} L={L} groups={layer.n_groups} R_k={layer.R_k} k_i4={k_i4} v_i4={v_i4}")
    desc = make_desc(layer, "f16", k_i4, v_i4, bits)
    table = P.palu_rope_table_init(layer.rope_theta, layer.d_head, L)
    hk, hv, kw = case.Hk[0], case.Hv[0], {}
    nbk, nbv = layer.R_k // 128, layer.R_v // 128
    quant = {}
    for side, flag, H, R, nb in (("k", k_i4, case.Hk[0], layer.R_k, nbk), ("v", v_i4, case.Hv[0], layer.R_v, nbv)):
        if not flag:
            continue
        codes = torch.empty((B, L, R * bits // 8), dtype=torch.uint8, device="cuda")
        sc = torch.empty((B, L, nb), dtype=torch.float16, device="cuda")
        zp = torch.empty_like(sc)
        P.palu_quant_latent(desc, 0 if side == "k" else 1, H, R, B * L, codes, sc, zp)
        quant[side] = (codes, sc, zp)
        if side == "k":
            hk, kw["hk_scale"], kw["hk_zero"] = codes, sc, zp
        else:
            hv, kw["hv_scale"], kw["hv_zero"] = codes, sc, zp
    if q_scale != 1.0:
        case.q = (case.q.float() * q_scale).half()
    out = P.palu_attn_decode(desc, B, L, L, case.q, case.q_pos, hk, hv, case.Bk, case.Bv, table, L, **kw)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.isfinite(got).all()
    Bk, Bv = case.Bk.float().cpu().numpy(), case.Bv.float().cpu().numpy()
    worst = 0.0
    if samples is None:
        # whole sequences: every head of the layer against the oracle
        for b in (range(B) if seqs is None else seqs):
            Hs = {}
            for side, H in (("k", case.Hk[0]), ("v", case.Hv[0])):
                Hb = H[b].float().cpu().numpy()
                if side in quant:
                    # the oracle quantizes the same rows itself; the bytes the GPU wrote must equal its bytes
                    pk, s_, z_ = O.quant_latent(Hb, bits=bits)
                    codes, sc, zp = quant[side]
                    np.testing.assert_array_equal(codes[b].cpu().numpy(), pk)
                    np.testing.assert_array_equal(sc[b].cpu().view(torch.int16).numpy(), s_.view(np.int16))
                    np.testing.assert_array_equal(zp[b].cpu().view(torch.int16).numpy(), z_.view(np.int16))
                    Hb = O.dequant_latent(pk, s_, z_, bits=bits)
                Hs[side] = Hb[None]
            ref = O.attn_decode(case.q[b].float().cpu().numpy()[None], [int(case.q_pos[b])], Hs["k"], Hs["v"], Bk, Bv,
                                layer.group_head_off, layer.k_rank_off, layer.v_rank_off, layer.d_head, layer.rope_theta,
                                None, None, layer.q_per_kv)
            whole, rows = rel_err(got[b][None], ref)
            say(f"       sequence {b}, all {layer.n_q_heads} heads: rel err {whole:.3e} (worst head {rows:.3e})")
            worst = max(worst, whole, rows)
        assert worst <= tol
        return
    for (b, j, heads) in samples:
        sub = group_slice(layer, j, heads)
        kc = slice(layer.k_rank_off[j], layer.k_rank_off[j + 1])
        vc = slice(layer.v_rank_off[j], layer.v_rank_off[j + 1])
        Hk = case.Hk[0][b, :, kc].float().cpu().numpy()[None]
        Hv = case.Hv[0][b, :, vc].float().cpu().numpy()[None]
        for side, H, cols in (("k", Hk, kc), ("v", Hv, vc)):
            if side not in quant:
                continue
            # the oracle quantizes the same rows itself; the codes the GPU wrote must equal its codes
            pk, s, z = O.quant_latent(H[0], bits=bits)
            codes, sc, zp = quant[side]
            got_codes = O.unpack_codes(codes[b].cpu().numpy(), bits)[:, cols]
            np.testing.assert_array_equal(got_codes, O.unpack_codes(pk, bits))
            np.testing.assert_array_equal(sc[b, :, cols.start // 128:cols.stop // 128].cpu().view(torch.int16).numpy(),
                                          s.view(np.int16))
            np.testing.assert_array_equal(zp[b, :, cols.start // 128:cols.stop // 128].cpu().view(torch.int16).numpy(),
                                          z.view(np.int16))
            deq = O.dequant_latent(pk, s, z, bits=bits)[None]
            if side == "k":
                Hk = deq
            else:
                Hv = deq
        # query heads of the sampled key/value heads (one each unless the layer is grouped-query)
        h_abs = [(layer.group_head_off[j] + u) * layer.q_per_kv + w for u in heads for w in range(layer.q_per_kv)]
        q = case.q[b, h_abs].float().cpu().numpy()[None]
        ref = O.attn_decode(q, [int(case.q_pos[b])], Hk, Hv, b_slice(Bk, layer, "k", j, heads),
                            b_slice(Bv, layer, "v", j, heads), sub.group_head_off, sub.k_rank_off, sub.v_rank_off,
                            layer.d_head, layer.rope_theta, None, None, layer.q_per_kv)
        whole, rows = rel_err(got[b, h_abs][None], ref)
        say(f"       sample b={b} group={j} heads={heads}: rel err {whole:.3e} (rows {rows:.3e})")
        worst = max(worst, whole, rows)
    assert worst <= tol


def test_full_config1():
    run_full("1")


def test_full_config2_4k():
    run_full("2-4k")


def test_full_config2_16k():
    run_full("2")


@pytest.mark.parametrize("q_scale", [4.0, 12.0])
def test_full_config2_16k_large_logits(q_scale):
    """The headline configuration with queries scaled so that the logits reach tens: same tolerance."""
    run_full("2", q_scale=q_scale)


def test_full_config2_64k():
    run_full("2-64k")


def test_full_config3_ragged():
    run_full("3")


def test_full_config4_int4_both():
    run_full("4", k_i4=True, v_i4=True, tol=TOL_I4)


def test_full_config4_int4_values_only():
    run_full("4", v_i4=True, tol=TOL_I4)


def test_full_config5a_per_head():
    run_full("5a")


def test_full_config5b_joint():
    """Two whole sequences (the oracle rebuilds 16384 x 4096 keys and values from rank 2048 for each), and
    sampled heads of two more."""
    run_full("5b", seqs=[0, 6])
    run_full("5b", [(3, 0, [0, 31]), (5, 0, [13])])


def test_full_config2_paper_rank_allocation():
    """Keys at rank 128, values at rank 384 per group (the paper's latency runs, Sec. 4.5)."""
    run_full("2p")


def test_full_config2_16k_no_rope():
    run_full("2", no_rope=True)


def test_full_config2_16k_no_rope_large_logits():
    run_full("2", no_rope=True, q_scale=8.0)


def test_full_config4_no_rope_int4():
    run_full("4", k_i4=True, v_i4=True, tol=TOL_I4, no_rope=True, seqs=[0, 9, 15])


def test_full_config5b_no_rope():
    run_full("5b", seqs=[2], no_rope=True)
    run_full("5b", [(0, 0, [0, 13]), (6, 0, [31])], no_rope=True)


def test_full_gqa_16k():
    """32 query heads on 8 key/value heads (Llama-3-8B / Mistral-7B shape), batch 4 at 16K."""
    run_full("gqa")


def test_full_gqa_16k_no_rope():
    run_full("gqa", no_rope=True, seqs=[1, 3])


def test_full_config4_three_bit_latents():
    run_full("4", k_i4=True, v_i4=True, tol=TOL_I4, bits=3, seqs=[3, 12])


def test_full_config4_two_bit_latents_no_rope():
    run_full("4", k_i4=True, v_i4=True, tol=TOL_I4, bits=2, no_rope=True, seqs=[9])


def test_full_config2_16k_four_query_tokens():
    """A causal block of four new tokens per sequence at the 7B shape and 16K: every query against
    its own single-query call of the library (itself checked against the oracle above), and one
    sampled (query, group) against the oracle."""
    case = wd.make_device_case("2", seed=0, n_sets=1)
    layer, B, L, n_q = case.layer, case.batch, case.seq, 4
    say(f"[full] cfg 2 with {n_q} query tokens per sequence, B={B} L={L}")
    desc = make_desc(layer, "f16")
    table = P.palu_rope_table_init(layer.rope_theta, layer.d_head, L)
    g = torch.Generator(device="cuda")
    g.manual_seed(1234)
    q = torch.randn((B, n_q, layer.n_heads, 128), generator=g, device="cuda", dtype=torch.float32).half()
    q_len = (torch.full((B, 1), L, dtype=torch.int32, device="cuda") - n_q + 1 +
             torch.arange(n_q, dtype=torch.int32, device="cuda")[None]).contiguous()
    q_pos = (q_len - 1).contiguous()
    out = P.palu_attn_decode_multi(desc, B, n_q, L, L, q, q_pos, case.Hk[0], case.Hv[0], case.Bk, case.Bv, table, L,
                                   q_len=q_len)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.isfinite(got).all()
    for j in range(n_q):
        one = P.palu_attn_decode(desc, B, L, L, q[:, j].contiguous(), q_pos[:, j].contiguous(), case.Hk[0], case.Hv[0],
                                 case.Bk, case.Bv, table, L, seq_lens=q_len[:, j].contiguous())
        torch.cuda.synchronize()
        whole, rows = rel_err(got[:, j], one.cpu().numpy().astype(np.float64))
        say(f"       query {j}: against its single-query call {whole:.3e} (rows {rows:.3e})")
        assert whole <= TOL_FP and rows <= TOL_FP
    j, grp, heads = 2, 3, [1, 2]
    sub = group_slice(layer, grp, heads)
    kc = slice(layer.k_rank_off[grp], layer.k_rank_off[grp + 1])
    vc = slice(layer.v_rank_off[grp], layer.v_rank_off[grp + 1])
    n_rows = int(q_len[0, j])
    Hk = case.Hk[0][0, :n_rows, kc].float().cpu().numpy()[None]
    Hv = case.Hv[0][0, :n_rows, vc].float().cpu().numpy()[None]
    h_abs = [layer.group_head_off[grp] + u for u in heads]
    Bk, Bv = case.Bk.float().cpu().numpy(), case.Bv.float().cpu().numpy()
    ref = O.attn_decode(q[0, j, h_abs].float().cpu().numpy()[None], [int(q_pos[0, j])], Hk, Hv,
                        b_slice(Bk, layer, "k", grp, heads), b_slice(Bv, layer, "v", grp, heads),
                        sub.group_head_off, sub.k_rank_off, sub.v_rank_off, 128, layer.rope_theta)
    whole, rows = rel_err(got[0, j, h_abs][None], ref)
    say(f"       oracle sample query {j} group {grp} heads {heads}: {whole:.3e}")
    assert whole <= TOL_FP and rows <= TOL_FP


@pytest.mark.parametrize("quantized", [False, True])
def test_cache_rows_beyond_4gib(quantized):
    """Caches whose rows lie more than 4 GiB from the base pointer: few attended tokens per
    sequence, but a row pitch (max_seq) that puts the later sequences beyond 32-bit byte
    offsets.  Rows past a sequence's length hold NaN bit patterns: they must not reach
    the result.  The oracle sees only the attended rows."""
    layer = synth.uniform_layer(8, 4, 256)
    B, L = (4, 1500) if quantized else (3, 2500)
    max_seq = (6 << 20) if quantized else (3 << 20)
    case = synth.make_case_svd(layer, B, L, seed=11, dtype="f16")
    case.seq_lens = np.array([L, L - 723, L - 400, L - 1][:B], np.int32)
    case.q_pos = (case.seq_lens - 1).astype(np.int32)
    desc = make_desc(layer, "f16", quantized, quantized)
    row_bytes = layer.R_k // 2 if quantized else layer.R_k * 2
    assert (B - 1) * max_seq * row_bytes > (1 << 32)
    say(f"[4gib] B={B} L={L} max_seq={max_seq} quantized={quantized}: {B * max_seq * row_bytes / 2**30:.1f} GiB per cache")
    kw, quant = {}, {}
    if quantized:
        caches = []
        for side, H in (("k", case.Hk), ("v", case.Hv)):
            pk, s, z = O.quant_latent(H.reshape(B * L, -1))
            quant[side] = (pk.reshape(B, L, -1), s.reshape(B, L, -1), z.reshape(B, L, -1))
            codes = torch.full((B, max_seq, pk.shape[-1]), 0xFF, dtype=torch.uint8, device="cuda")
            sc = torch.full((B, max_seq, s.shape[-1]), float("nan"), dtype=torch.float16, device="cuda")
            zp = torch.full((B, max_seq, s.shape[-1]), float("nan"), dtype=torch.float16, device="cuda")
            for b in range(B):
                n = int(case.seq_lens[b])
                codes[b, :n] = torch.from_numpy(quant[side][0][b, :n]).cuda()
                sc[b, :n] = torch.from_numpy(quant[side][1][b, :n].view(np.int16)).cuda().view(torch.float16)
                zp[b, :n] = torch.from_numpy(quant[side][2][b, :n].view(np.int16)).cuda().view(torch.float16)
            caches.append(codes)
            kw[f"h{side}_scale"], kw[f"h{side}_zero"] = sc, zp
        hk, hv = caches
    else:
        hk = torch.full((B, max_seq, layer.R_k), float("nan"), dtype=torch.float16, device="cuda")
        hv = torch.full((B, max_seq, layer.R_v), float("nan"), dtype=torch.float16, device="cuda")
        for b in range(B):
            n = int(case.seq_lens[b])
            hk[b, :n] = torch.from_numpy(case.Hk[b, :n]).to(torch.float16).cuda()
            hv[b, :n] = torch.from_numpy(case.Hv[b, :n]).to(torch.float16).cuda()
    from gpu_util import run_oracle, to_dev
    table = P.palu_rope_table_init(layer.rope_theta, layer.d_head, L)
    out = P.palu_attn_decode(desc, B, L, max_seq, to_dev(case.q, "f16"), torch.from_numpy(case.q_pos).cuda(), hk, hv,
                             to_dev(case.Bk, "f16"), to_dev(case.Bv, "f16"), table, L,
                             seq_lens=torch.from_numpy(case.seq_lens).cuda(), **kw)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.isfinite(got).all()
    ref = run_oracle(case, quant if quantized else None, quantized, quantized)
    whole, rows = rel_err(got, ref)
    say(f"       rel err {whole:.3e} (rows {rows:.3e})")
    assert max(whole, rows) <= (TOL_I4 if quantized else TOL_FP)


def test_one_sequence_longer_than_4gib():
    """One sequence of 1.2 M tokens in the 7B shape: 4.6 GiB of key latents attended in one
    call, more splits than compute units, the value kernel's split count at its limit."""
    run_full("2", [(0, 3, [2])], seq=1_200_007)
