"""GPU checks of the cache-append entry points: encode (tolerance) and the
int4 quantizer (bit-exact), plus the rope table."""

import numpy as np
import pytest
import torch

import paper_2407_21118_amd as P
from oracle import palu_oracle as O
from workloads import synth

pytestmark = pytest.mark.gpu

from gpu_util import make_desc, say, to_dev  # noqa: E402


@pytest.mark.parametrize("dtype,n_tok", [("f16", 1), ("f16", 16), ("bf16", 5), ("f16", 19)])
def test_encode_matches_oracle(dtype, n_tok):
    say(f"[encode] dtype={dtype} n_tok={n_tok}")
    layer = synth.config_layer("3")                       # ragged ranks, R = 2048
    rng = np.random.default_rng(7)
    d = layer.n_heads * layer.d_head
    A = synth.round_to(rng.standard_normal((d, layer.R_k)) / 64.0, dtype)
    x = synth.round_to(rng.standard_normal((n_tok, d)), dtype)
    desc = make_desc(layer, dtype)
    rows = 40
    cache = torch.full((rows, layer.R_k), 7.0, dtype=torch.float16 if dtype == "f16" else torch.bfloat16, device="cuda")
    dst = torch.from_numpy(((np.arange(n_tok) * 2 + 1) % rows).astype(np.int32)).cuda()
    P.palu_encode(desc, 0, to_dev(x, dtype), to_dev(A, dtype), cache, layer.R_k, dst)
    torch.cuda.synchronize()
    got = cache.float().cpu().numpy()
    ref = O.encode(x, A)
    eps = 2.0 ** -11 if dtype == "f16" else 2.0 ** -8
    for t in range(n_tok):
        r = (2 * t + 1) % rows
        # one rounding to the cache dtype plus float32 accumulation noise
        assert np.abs(got[r] - ref[t]).max() <= (eps * 1.01) * np.abs(ref[t]).max() + 1e-6
    untouched = np.setdiff1d(np.arange(rows), (np.arange(n_tok) * 2 + 1) % rows)
    assert (got[untouched] == 7.0).all()


def test_encode_sequential_rows_default():
    layer = synth.uniform_layer(8, 4, 64)
    rng = np.random.default_rng(8)
    d = layer.n_heads * layer.d_head
    A = synth.round_to(rng.standard_normal((d, layer.R_v)) / 32.0, "f16")
    x = synth.round_to(rng.standard_normal((3, d)), "f16")
    desc = make_desc(layer, "f16")
    cache = torch.zeros((3, layer.R_v + 64), dtype=torch.float16, device="cuda")     # padded row stride
    P.palu_encode(desc, 1, to_dev(x, "f16"), to_dev(A, "f16"), cache, layer.R_v + 64)
    torch.cuda.synchronize()
    got = cache.float().cpu().numpy()
    ref = O.encode(x, A)
    assert np.abs(got[:, :layer.R_v] - ref).max() <= 2.0 ** -11 * 1.01 * np.abs(ref).max() + 1e-6
    assert (got[:, layer.R_v:] == 0).all()


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_quantizer_bit_exact(dtype):
    say(f"[quant] dtype={dtype}")
    layer = synth.config_layer("4")
    rng = np.random.default_rng(9)
    n_tok = 300
    h = rng.standard_normal((n_tok, layer.R_k)) * rng.uniform(0.01, 40.0, size=(n_tok, 1))
    h[:20] += 11.0                       # all-positive blocks: negative zero-points
    h[20:24] = 2.5                       # constant blocks
    h[24, :128] = np.arange(128) % 16    # exact grid
    h[25, :128] = (np.arange(128) % 16) * 0.5 + 0.25      # ties
    h = synth.round_to(h, dtype)
    desc = make_desc(layer, dtype)
    codes = torch.empty((n_tok, layer.R_k // 2), dtype=torch.uint8, device="cuda")
    scale = torch.empty((n_tok, layer.R_k // 128), dtype=torch.float16, device="cuda")
    zero = torch.empty_like(scale)
    P.palu_quant_latent(desc, 0, to_dev(h, dtype), layer.R_k, n_tok, codes, scale, zero)
    torch.cuda.synchronize()
    pk, s, z = O.quant_latent(h)
    np.testing.assert_array_equal(codes.cpu().numpy(), pk)
    np.testing.assert_array_equal(scale.cpu().view(torch.int16).numpy(), s.view(np.int16))
    np.testing.assert_array_equal(zero.cpu().view(torch.int16).numpy(), z.view(np.int16))


def test_rope_table_values():
    """Every tested (position, pair) of the table against float64 cos/sin.  The table is tiles of 32
    positions, each a float32 part [pair][cos | sin][position in tile] (read by the score kernel; checked
    entry by entry to float32 rounding) and float16 rows [position][128] in a private slot order (the
    opt-in shared-key form; checked as sorted multisets per position)."""
    n_pos = 70000
    tiles = (n_pos + 31) // 32
    table = P.palu_rope_table_init(10000.0, 128, n_pos)
    torch.cuda.synchronize()
    assert table.numel() == tiles * (16384 + 8192) == P.palu_rope_table_bytes(128, n_pos)
    raw = table.cpu().numpy().reshape(tiles, 16384 + 8192)
    f32 = raw[:, :16384].copy().view(np.float32).reshape(tiles, 64, 2, 32).astype(np.float64)
    f16 = raw[:, 16384:].copy().view(np.float16).reshape(tiles * 32, 128).astype(np.float64)
    inv = O.rope_inv_freq(128, 10000.0)
    for p in (0, 1, 31, 32, 4095, 65535, 69999, tiles * 32 - 1):       # the last tile is filled to its end
        ang = p * inv
        assert np.abs(f32[p // 32, :, 0, p % 32] - np.cos(ang)).max() <= 2.0 ** -24
        assert np.abs(f32[p // 32, :, 1, p % 32] - np.sin(ang)).max() <= 2.0 ** -24
        want = np.sort(np.concatenate([np.cos(ang), np.sin(ang)]))
        assert np.abs(np.sort(f16[p]) - want).max() <= 2.0 ** -11
    none = P.palu_rope_table_init(0.0, 128, 4).cpu().numpy().reshape(1, 16384 + 8192)
    flat = none[:, :16384].copy().view(np.float32).reshape(64, 2, 32)
    assert (flat[:, 0, :] == 1.0).all() and (flat[:, 1, :] == 0.0).all()


def test_argument_errors_leave_output_untouched():
    layer = synth.uniform_layer(8, 4, 64)
    desc = make_desc(layer, "f16")
    q = torch.zeros((1, 8, 128), dtype=torch.float16, device="cuda")
    pos = torch.zeros(1, dtype=torch.int32, device="cuda")
    h = torch.zeros((1, 64, 128), dtype=torch.float16, device="cuda")
    Bm = torch.zeros(layer.b_elems("k"), dtype=torch.float16, device="cuda")
    table = P.palu_rope_table_init(10000.0, 128, 64)
    out = torch.full((1, 8, 128), 3.0, dtype=torch.float32, device="cuda")
    with pytest.raises(P.PaluError) as e:
        P.palu_attn_decode(desc, 1, 65, 64, q, pos, h, h, Bm, Bm, table, 64, out=out)      # seq_len > max_seq
    assert e.value.status == -1
    with pytest.raises(P.PaluError) as e:
        P.palu_attn_decode(desc, 1, 64, 64, q, pos, h, h, Bm, Bm, table, 10, out=out)      # table too short
    assert e.value.status == -1
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(P.PaluError) as e:
        P.palu_attn_decode(desc, 1, 64, 64, q, pos, h, h, Bm, Bm, table, 64, out=out, workspace=small)
    assert e.value.status == -3
    torch.cuda.synchronize()
    assert (out == 3.0).all()


def test_encode_kv_matches_oracle_and_single_side_calls():
    say("[encode_kv]")
    layer = synth.config_layer("3")
    rng = np.random.default_rng(12)
    d = layer.n_heads * layer.d_head
    Ak = synth.round_to(rng.standard_normal((d, layer.R_k)) / 64.0, "f16")
    Av = synth.round_to(rng.standard_normal((d, layer.R_v)) / 64.0, "f16")
    x = synth.round_to(rng.standard_normal((4, d)), "f16")
    desc = make_desc(layer, "f16")
    hk = torch.zeros((9, layer.R_k), dtype=torch.float16, device="cuda")
    hv = torch.zeros((9, layer.R_v), dtype=torch.float16, device="cuda")
    dst = torch.tensor([8, 0, 3, 5], dtype=torch.int32, device="cuda")
    P.palu_encode_kv(desc, to_dev(x, "f16"), to_dev(Ak, "f16"), to_dev(Av, "f16"), hk, layer.R_k, hv, layer.R_v, dst)
    hk1 = torch.zeros_like(hk)
    hv1 = torch.zeros_like(hv)
    P.palu_encode(desc, 0, to_dev(x, "f16"), to_dev(Ak, "f16"), hk1, layer.R_k, dst)
    P.palu_encode(desc, 1, to_dev(x, "f16"), to_dev(Av, "f16"), hv1, layer.R_v, dst)
    torch.cuda.synchronize()
    assert torch.equal(hk, hk1) and torch.equal(hv, hv1)
    for got, A in ((hk, Ak), (hv, Av)):
        ref = O.encode(x, A)
        g = got.float().cpu().numpy()
        for t, r in enumerate([8, 0, 3, 5]):
            assert np.abs(g[r] - ref[t]).max() <= 2.0 ** -11 * 1.01 * np.abs(ref[t]).max() + 1e-6


def test_quantizer_scatter_rows():
    layer = synth.config_layer("4")
    rng = np.random.default_rng(13)
    h = synth.round_to(rng.standard_normal((3, layer.R_v)) * 3.0, "f16")
    desc = make_desc(layer, "f16")
    rows = 7
    codes = torch.zeros((rows, layer.R_v // 2), dtype=torch.uint8, device="cuda")
    scale = torch.zeros((rows, layer.R_v // 128), dtype=torch.float16, device="cuda")
    zero = torch.zeros_like(scale)
    dst = torch.tensor([6, 2, 4], dtype=torch.int32, device="cuda")
    P.palu_quant_latent(desc, 1, to_dev(h, "f16"), layer.R_v, 3, codes, scale, zero, dst)
    torch.cuda.synchronize()
    pk, s, z = O.quant_latent(h)
    c = codes.cpu().numpy()
    for t, r in enumerate([6, 2, 4]):
        np.testing.assert_array_equal(c[r], pk[t])
        np.testing.assert_array_equal(scale[r].cpu().view(torch.int16).numpy(), s[t].view(np.int16))
        np.testing.assert_array_equal(zero[r].cpu().view(torch.int16).numpy(), z[t].view(np.int16))
    assert not c[[0, 1, 3, 5]].any()


@pytest.mark.parametrize("theta,v_i4,cfg", [(10000.0, False, "3"), (0.0, False, "3"), (10000.0, True, "4"),
                                            (500000.0, False, "gqa")])
def test_latent_output_matches_oracle(theta, v_i4, cfg):
    """palu_attn_decode_latent: the output stays in the value latent space (Sec. 3.1.1);
    compared with the oracle's latent output, and times B_v with the full decode call."""
    import dataclasses
    from gpu_util import TOL_FP, TOL_I4, make_desc, to_dev
    layer = dataclasses.replace(synth.config_layer(cfg), rope_theta=theta)
    case = synth.make_case_svd(layer, 2, 300, seed=9, rotate=v_i4)
    case.seq_lens = np.array([300, 77], np.int32)
    case.q_pos = np.array([299, 76], np.int32)
    desc = make_desc(layer, "f16", False, v_i4)
    q, Bk = to_dev(case.q, "f16"), to_dev(case.Bk, "f16")
    hk = to_dev(case.Hk, "f16")
    kw = {}
    Hv_ref = case.Hv
    if v_i4:
        pv, sv, zv = O.quant_latent(case.Hv)
        hv = torch.from_numpy(pv).cuda()
        kw["hv_scale"] = torch.from_numpy(sv.view(np.int16)).cuda().view(torch.float16)
        kw["hv_zero"] = torch.from_numpy(zv.view(np.int16)).cuda().view(torch.float16)
        Hv_ref = O.dequant_latent(pv, sv, zv)
    else:
        hv = to_dev(case.Hv, "f16")
    table = P.palu_rope_table_init(theta, 128, 300)
    q_pos = torch.from_numpy(case.q_pos).cuda()
    lens = torch.from_numpy(case.seq_lens).cuda()
    got = P.palu_attn_decode_latent(desc, 2, 300, 300, q, q_pos, hk, hv, Bk, table, 300, seq_lens=lens, **kw)
    torch.cuda.synchronize()
    ref = O.attn_decode_latent(case.q, case.q_pos, case.Hk, Hv_ref, case.Bk, layer.group_head_off, layer.k_rank_off,
                               layer.v_rank_off, 128, theta, seq_lens=case.seq_lens, q_per_kv=layer.q_per_kv)
    got = got.cpu().numpy()
    assert got.shape == ref.shape
    err = np.abs(got - ref).max() / np.abs(ref).max()
    say(f"[latent] theta={theta} v_i4={v_i4} width={ref.shape[1]} rel err {err:.3e}")
    assert err <= (TOL_I4 if v_i4 else TOL_FP)


@pytest.mark.parametrize("one_call", [False, True, "transposed"])
def test_decode_step_in_a_captured_graph(one_call):
    """Append + decode captured into a HIP graph (the calls allocate nothing and never
    synchronise): four replays with fresh inputs written into the captured buffers, each
    compared bit for bit with the same step launched eagerly in between."""
    from workloads import device as wd
    layer = synth.config_layer("2")
    batch, seq = 2, 1111
    case = wd.make_device_case("2", seed=1, dtype="f16", n_sets=1, batch=batch, seq=seq)
    desc = P.LayerDesc(layer.n_heads, layer.d_head, layer.group_head_off, layer.k_rank_off, layer.v_rank_off)
    table = P.palu_rope_table_init(layer.rope_theta, layer.d_head, seq)
    ws = torch.empty(P.palu_attn_decode_workspace_bytes(desc, batch, seq), dtype=torch.uint8, device="cuda")
    ws_e = torch.empty(P.palu_encode_workspace_bytes(desc, 2, batch), dtype=torch.uint8, device="cuda")
    out = torch.empty((batch, layer.n_heads, layer.d_head), dtype=torch.float32, device="cuda")
    dst_row = (torch.arange(batch, dtype=torch.int32, device="cuda") * seq + (seq - 1)).contiguous()
    q_buf, x_buf = case.q.clone(), case.x_new.clone()
    side = torch.cuda.Stream()

    Akt, Avt = case.Ak.t().contiguous(), case.Av.t().contiguous()

    def step():
        s = torch.cuda.current_stream()
        if one_call == "transposed":      # palu_decode_step_t: the whole append is one launch
            P.palu_decode_step_t(desc, batch, seq, seq, x_buf, Akt, Avt, dst_row, q_buf, case.q_pos, case.Hk[0],
                                 case.Hv[0], case.Bk, case.Bv, table, seq, out=out, workspace=ws, stream=s)
            return
        if one_call:          # palu_decode_step: the projection's first launch carries the query fold
            P.palu_decode_step(desc, batch, seq, seq, x_buf, case.Ak, case.Av, dst_row, q_buf, case.q_pos, case.Hk[0],
                               case.Hv[0], case.Bk, case.Bv, table, seq, out=out, workspace=ws, encode_workspace=ws_e, stream=s)
            return
        P.palu_encode_kv(desc, x_buf, case.Ak, case.Av, case.Hk[0], layer.R_k, case.Hv[0], layer.R_v, dst_row, ws_e, stream=s)
        P.palu_attn_decode(desc, batch, seq, seq, q_buf, case.q_pos, case.Hk[0], case.Hv[0], case.Bk, case.Bv, table,
                           seq, out=out, workspace=ws, stream=s)

    with torch.cuda.stream(side):
        step()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    for it in range(4):
        q_buf.copy_(torch.randn(q_buf.shape, generator=gen, device="cuda").half())
        x_buf.copy_(torch.randn(x_buf.shape, generator=gen, device="cuda").half())
        graph.replay()
        torch.cuda.synchronize()
        got = out.clone()
        with torch.cuda.stream(side):
            step()
        torch.cuda.synchronize()
        say(f"[graph] replay {it}: max abs diff to eager {float((got - out).abs().max()):.3e}")
        assert torch.equal(got, out)


@pytest.fixture
def encode_tile(request):
    """Forces the projection's tile (the library picks it from the token count: short prompts get
    64 x 128, the tall tiles are otherwise reached only by prompts of thousands of tokens; 32 names
    the 64 x 128 tile)."""
    P.palu_set_option("encode_tile_rows", request.param)
    yield request.param
    P.palu_set_option("encode_tile_rows", 0)


@pytest.mark.parametrize("dtype,n_tok,encode_tile", [("f16", 64, 0), ("f16", 300, 0), ("bf16", 129, 0), ("f16", 300, 128),
                                                     ("f16", 300, 256), ("bf16", 700, 256), ("bf16", 129, 128), ("f16", 300, 64), ("bf16", 129, 64),
                                                     ("f16", 700, 32)],
                         indirect=["encode_tile"])
def test_encode_many_tokens_gemm_path(dtype, n_tok, encode_tile):
    """Prompt-sized append: from 64 tokens on palu_encode runs as a tiled GEMM on the matrix
    cores.  A layer whose total rank (1344) is not a multiple of the 256-column tile, a
    ragged token count, scattered destination rows, every tile height; palu_encode_kv covers
    both sides."""
    say(f"[encode-gemm] dtype={dtype} n_tok={n_tok} tile rows={encode_tile or 'auto'}")
    k_ranks = [32, 64, 128, 96, 128, 384, 512]
    v_ranks = [64, 32, 128, 256, 96, 128, 512]
    layer = synth.Layer(16, 128, [0, 1, 2, 4, 6, 7, 10, 16], [0] + list(np.cumsum(k_ranks)), [0] + list(np.cumsum(v_ranks)))
    rng = np.random.default_rng(11)
    d = layer.n_heads * layer.d_head
    Ak = synth.round_to(rng.standard_normal((d, layer.R_k)) / 45.0, dtype)
    Av = synth.round_to(rng.standard_normal((d, layer.R_v)) / 45.0, dtype)
    x = synth.round_to(rng.standard_normal((n_tok, d)), dtype)
    desc = make_desc(layer, dtype)
    td = torch.float16 if dtype == "f16" else torch.bfloat16
    rows = n_tok + 50
    perm = rng.permutation(rows)[:n_tok].astype(np.int32)
    hk = torch.full((rows, layer.R_k), 7.0, dtype=td, device="cuda")
    hv = torch.full((rows, layer.R_v + 32), 7.0, dtype=td, device="cuda")
    P.palu_encode_kv(desc, to_dev(x, dtype), to_dev(Ak, dtype), to_dev(Av, dtype), hk, layer.R_k, hv, layer.R_v + 32,
                     torch.from_numpy(perm).cuda())
    torch.cuda.synchronize()
    eps = 2.0 ** -11 if dtype == "f16" else 2.0 ** -8
    for got, ref, R in ((hk.float().cpu().numpy(), O.encode(x, Ak), layer.R_k), (hv.float().cpu().numpy(), O.encode(x, Av), layer.R_v)):
        err = np.abs(got[perm, :R] - ref).max(axis=1) / np.abs(ref).max(axis=1)
        say(f"       worst row error {err.max():.3e} (bound {eps * 1.05:.3e})")
        assert err.max() <= eps * 1.05 + 1e-6
        untouched = np.setdiff1d(np.arange(rows), perm)
        assert (got[untouched] == 7.0).all() and (got[:, R:] == 7.0).all()


@pytest.mark.parametrize("dtype,n_tok,encode_tile", [("f16", 1, 0), ("f16", 64, 0), ("f16", 300, 0), ("bf16", 129, 0),
                                                     ("f16", 300, 128), ("f16", 600, 256), ("bf16", 300, 256), ("f16", 300, 64), ("bf16", 200, 32)],
                         indirect=["encode_tile"])
def test_encode_quant_fused(dtype, n_tok, encode_tile):
    """Down-projection with the quantizer fused into the GEMM's write-out.  Two checks:
    the dequantized cache is within half a quantization step (plus the rounding of the
    latent) of the oracle's float64 product; and, where palu_encode runs the same GEMM
    (n_tok >= 64), codes, scales and zero-points are bit for bit what the oracle's
    quantizer gives for the latents that call stores."""
    say(f"[encode-quant] dtype={dtype} n_tok={n_tok} tile rows={encode_tile or 'auto'}")
    layer = synth.config_layer("4")
    rng = np.random.default_rng(12)
    d = layer.n_heads * layer.d_head
    R = layer.R_v
    A = synth.round_to(rng.standard_normal((d, R)) / 45.0 * rng.uniform(0.05, 3.0, size=(1, R)), dtype)
    x = synth.round_to(rng.standard_normal((n_tok, d)) * rng.uniform(0.1, 8.0, size=(n_tok, 1)), dtype)
    desc = make_desc(layer, dtype)
    td = torch.float16 if dtype == "f16" else torch.bfloat16
    rows = n_tok + 9
    perm = rng.permutation(rows)[:n_tok].astype(np.int32)
    dst = torch.from_numpy(perm).cuda()
    codes = torch.full((rows, R // 2), 0xA5, dtype=torch.uint8, device="cuda")
    scale = torch.full((rows, R // 128), 3.0, dtype=torch.float16, device="cuda")
    zero = torch.full((rows, R // 128), 3.0, dtype=torch.float16, device="cuda")
    P.palu_encode_quant(desc, 1, to_dev(x, dtype), n_tok, to_dev(A, dtype), codes, scale, zero, dst)
    torch.cuda.synchronize()
    c = codes.cpu().numpy()
    s = scale.float().cpu().numpy().astype(np.float64)
    z = zero.float().cpu().numpy().astype(np.float64)
    untouched = np.setdiff1d(np.arange(rows), perm)
    assert (c[untouched] == 0xA5).all() and (s[untouched] == 3.0).all() and (z[untouched] == 3.0).all()
    ref = O.encode(x, A)
    unpacked = np.empty((rows, R), dtype=np.float64)
    unpacked[:, 0::2] = c & 15
    unpacked[:, 1::2] = c >> 4
    deq = (unpacked.reshape(rows, R // 128, 128) - z[:, :, None]) * s[:, :, None]
    err = np.abs(deq[perm] - ref.reshape(n_tok, R // 128, 128))
    eps = 2.0 ** -11 if dtype == "f16" else 2.0 ** -8
    bound = s[perm][:, :, None] * 0.51 + eps * 1.05 * np.abs(ref).max(axis=1)[:, None, None] + 1e-6
    say(f"       worst error / bound {float((err / bound).max()):.3f}")
    assert (err <= bound).all()
    if n_tok >= 64:
        lat = torch.zeros((rows, R), dtype=td, device="cuda")
        P.palu_encode(desc, 1, to_dev(x, dtype), to_dev(A, dtype), lat, R, dst)
        torch.cuda.synchronize()
        pk, so, zo = O.quant_latent(lat.float().cpu().numpy()[perm])
        np.testing.assert_array_equal(c[perm], pk)
        np.testing.assert_array_equal(scale.cpu().view(torch.int16).numpy()[perm], so.view(np.int16))
        np.testing.assert_array_equal(zero.cpu().view(torch.int16).numpy()[perm], zo.view(np.int16))


@pytest.mark.parametrize("bits,dtype", [(2, "f16"), (3, "f16")])
def test_low_bit_quantizer_bit_exact(bits, dtype):
    """palu_quant_latent on a side declared PALU_I3 / PALU_I2: codes in the 2- and 3-bit layouts,
    scales and zero-points, bit for bit the oracle's; scattered destination rows."""
    say(f"[quant] bits={bits} dtype={dtype}")
    layer = synth.config_layer("4")
    rng = np.random.default_rng(90 + bits)
    n_tok = 200
    h = rng.standard_normal((n_tok, layer.R_k)) * rng.uniform(0.01, 40.0, size=(n_tok, 1))
    h[:10] += 9.0
    h[10:12] = -1.5                                            # constant blocks
    h[12, :128] = np.arange(128) % (1 << bits)                 # exact grid
    h[13, :128] = (np.arange(128) % (1 << bits)) * 0.5 + 0.25  # ties
    h = synth.round_to(h, dtype)
    act = P.PALU_F16 if dtype == "f16" else P.PALU_BF16
    qd = {3: P.PALU_I3, 2: P.PALU_I2}[bits]
    # a quantized side needs an fp16 layer for decoding; the quantizer itself also takes bf16 inputs
    desc = P.LayerDesc(layer.n_heads, layer.d_head, layer.group_head_off, layer.k_rank_off, layer.v_rank_off,
                       P.PALU_F16, qd, qd) if dtype == "f16" else None
    if desc is None:
        pytest.skip("quantized sides are declared on fp16 layers")
    rows = n_tok + 7
    perm = rng.permutation(rows)[:n_tok].astype(np.int32)
    codes = torch.full((rows, layer.R_k * bits // 8), 0x5A, dtype=torch.uint8, device="cuda")
    scale = torch.zeros((rows, layer.R_k // 128), dtype=torch.float16, device="cuda")
    zero = torch.zeros_like(scale)
    P.palu_quant_latent(desc, 0, to_dev(h, dtype), layer.R_k, n_tok, codes, scale, zero, torch.from_numpy(perm).cuda())
    torch.cuda.synchronize()
    pk, s, z = O.quant_latent(h, bits=bits)
    np.testing.assert_array_equal(codes.cpu().numpy()[perm], pk)
    np.testing.assert_array_equal(scale.cpu().view(torch.int16).numpy()[perm], s.view(np.int16))
    np.testing.assert_array_equal(zero.cpu().view(torch.int16).numpy()[perm], z.view(np.int16))
    untouched = np.setdiff1d(np.arange(rows), perm)
    assert (codes.cpu().numpy()[untouched] == 0x5A).all()


@pytest.mark.parametrize("cfg,batch,theta,dtype", [("2", 1, 10000.0, "f16"), ("3", 3, 10000.0, "f16"), ("2", 8, 10000.0, "bf16"),
                                                   ("2", 2, 0.0, "f16"), ("gqa", 2, 500000.0, "f16")])
def test_decode_step_equals_encode_then_decode(cfg, batch, theta, dtype):
    """palu_decode_step (append + attend in one call, the projection's first launch sharing a grid
    with the query fold where the step has one) against palu_encode_kv followed by
    palu_attn_decode: same caches and same output, bit for bit; and against the oracle."""
    import dataclasses
    from gpu_util import TOL_FP, make_desc, to_dev
    layer = dataclasses.replace(synth.config_layer(cfg), rope_theta=theta)
    L = 200
    case = synth.make_case_svd(layer, batch, L, seed=17, dtype=dtype)
    say(f"[step] cfg={cfg} batch={batch} theta={theta} dtype={dtype}")
    desc = make_desc(layer, dtype)
    td = torch.float16 if dtype == "f16" else torch.bfloat16
    rng = np.random.default_rng(18)
    d = layer.n_q_heads * 128
    x = synth.round_to(rng.standard_normal((batch, d)), dtype)
    dst = torch.arange(batch, dtype=torch.int32, device="cuda") * L + (L - 1)
    args = dict(q=to_dev(case.q, dtype), q_pos=torch.from_numpy(case.q_pos).cuda(), Bk=to_dev(case.Bk, dtype),
                Bv=to_dev(case.Bv, dtype))
    Ak, Av, xd = to_dev(case.Ak, dtype), to_dev(case.Av, dtype), to_dev(x, dtype)
    table = P.palu_rope_table_init(theta, 128, L)
    hk1, hv1 = to_dev(case.Hk, dtype), to_dev(case.Hv, dtype)
    hk2, hv2 = hk1.clone(), hv1.clone()
    P.palu_encode_kv(desc, xd, Ak, Av, hk1, layer.R_k, hv1, layer.R_v, dst)
    ref_out = P.palu_attn_decode(desc, batch, L, L, args["q"], args["q_pos"], hk1, hv1, args["Bk"], args["Bv"], table, L)
    got = P.palu_decode_step(desc, batch, L, L, xd, Ak, Av, dst, args["q"], args["q_pos"], hk2, hv2, args["Bk"], args["Bv"],
                             table, L)
    torch.cuda.synchronize()
    assert torch.equal(hk1, hk2) and torch.equal(hv1, hv2)
    assert torch.equal(got, ref_out)
    Hk = hk2.float().cpu().numpy().astype(np.float64)
    Hv = hv2.float().cpu().numpy().astype(np.float64)
    want = O.attn_decode(case.q, case.q_pos, Hk, Hv, case.Bk, case.Bv, layer.group_head_off, layer.k_rank_off,
                         layer.v_rank_off, 128, theta, None, None, layer.q_per_kv)
    err = np.abs(got.cpu().numpy() - want).max() / np.abs(want).max()
    say(f"       rel err to the oracle on the appended cache {err:.3e}")
    assert err <= TOL_FP


@pytest.mark.parametrize("dtype,n_tok", [("f16", 1), ("f16", 2), ("bf16", 5), ("f16", 8), ("f16", 19), ("bf16", 63)])
def test_encode_from_transposed_weights(dtype, n_tok):
    """palu_encode_kv_t: the down-projection from A^T (one launch, a wavefront per pair of columns)
    against the oracle's float64 product, on a ragged layer (total ranks 1344 and 1216), with
    scattered destination rows and padded cache rows; untouched memory stays untouched."""
    say(f"[encode-t] dtype={dtype} n_tok={n_tok}")
    k_ranks = [32, 64, 128, 96, 128, 384, 512]
    v_ranks = [64, 32, 128, 256, 96, 128, 512]
    layer = synth.Layer(16, 128, [0, 1, 2, 4, 6, 7, 10, 16], [0] + list(np.cumsum(k_ranks)), [0] + list(np.cumsum(v_ranks)))
    rng = np.random.default_rng(21)
    d = layer.n_heads * layer.d_head
    Ak = synth.round_to(rng.standard_normal((d, layer.R_k)) / 45.0, dtype)
    Av = synth.round_to(rng.standard_normal((d, layer.R_v)) / 45.0, dtype)
    x = synth.round_to(rng.standard_normal((n_tok, d)), dtype)
    desc = make_desc(layer, dtype)
    td = torch.float16 if dtype == "f16" else torch.bfloat16
    rows = n_tok + 11
    perm = rng.permutation(rows)[:n_tok].astype(np.int32)
    hk = torch.full((rows, layer.R_k + 2), 7.0, dtype=td, device="cuda")
    hv = torch.full((rows, layer.R_v + 32), 7.0, dtype=td, device="cuda")
    P.palu_encode_kv_t(desc, to_dev(x, dtype), to_dev(np.ascontiguousarray(Ak.T), dtype), to_dev(np.ascontiguousarray(Av.T), dtype),
                       hk, layer.R_k + 2, hv, layer.R_v + 32, torch.from_numpy(perm).cuda())
    torch.cuda.synchronize()
    eps = 2.0 ** -11 if dtype == "f16" else 2.0 ** -8
    for got, ref, R in ((hk.float().cpu().numpy(), O.encode(x, Ak), layer.R_k), (hv.float().cpu().numpy(), O.encode(x, Av), layer.R_v)):
        err = np.abs(got[perm, :R] - ref).max(axis=1) / np.abs(ref).max(axis=1)
        say(f"       worst row error {err.max():.3e} (bound {eps * 1.05:.3e})")
        assert err.max() <= eps * 1.05 + 1e-6
        untouched = np.setdiff1d(np.arange(rows), perm)
        assert (got[untouched] == 7.0).all() and (got[:, R:] == 7.0).all()


@pytest.mark.parametrize("cfg,batch,theta,dtype", [("2", 1, 10000.0, "f16"), ("3", 3, 10000.0, "f16"), ("2", 8, 10000.0, "bf16"),
                                                   ("2", 2, 0.0, "f16"), ("gqa", 2, 500000.0, "f16"), ("5a", 11, 10000.0, "f16")])
def test_decode_step_from_transposed_weights(cfg, batch, theta, dtype):
    """palu_decode_step_t (the projection from A^T, the query fold riding in its workgroups where the
    step has one): the appended rows against the oracle's projection, the rest of the caches
    untouched, and the output against the oracle's attention over the cache as it then stands."""
    import dataclasses
    from gpu_util import TOL_FP, make_desc, to_dev
    layer = dataclasses.replace(synth.config_layer(cfg), rope_theta=theta)
    L = 200
    case = synth.make_case_svd(layer, batch, L, seed=19, dtype=dtype)
    say(f"[step-t] cfg={cfg} batch={batch} theta={theta} dtype={dtype}")
    desc = make_desc(layer, dtype)
    rng = np.random.default_rng(20)
    d = layer.n_q_heads * 128
    x = synth.round_to(rng.standard_normal((batch, d)), dtype)
    rows = (np.arange(batch) * L + (L - 1)).astype(np.int32)
    table = P.palu_rope_table_init(theta, 128, L)
    hk, hv = to_dev(case.Hk, dtype), to_dev(case.Hv, dtype)
    got = P.palu_decode_step_t(desc, batch, L, L, to_dev(x, dtype), to_dev(np.ascontiguousarray(case.Ak.T), dtype),
                               to_dev(np.ascontiguousarray(case.Av.T), dtype), torch.from_numpy(rows).cuda(),
                               to_dev(case.q, dtype), torch.from_numpy(case.q_pos).cuda(), hk, hv, to_dev(case.Bk, dtype),
                               to_dev(case.Bv, dtype), table, L)
    torch.cuda.synchronize()
    Hk = hk.float().cpu().numpy().astype(np.float64).reshape(batch * L, -1)
    Hv = hv.float().cpu().numpy().astype(np.float64).reshape(batch * L, -1)
    eps = 2.0 ** -11 if dtype == "f16" else 2.0 ** -8
    keep = np.setdiff1d(np.arange(batch * L), rows)
    for H, H0, A in ((Hk, case.Hk, case.Ak), (Hv, case.Hv, case.Av)):
        ref = O.encode(x, A)
        err = np.abs(H[rows] - ref).max(axis=1) / np.abs(ref).max(axis=1)
        assert err.max() <= eps * 1.05 + 1e-6
        np.testing.assert_array_equal(H[keep], H0.reshape(batch * L, -1)[keep])
    want = O.attn_decode(case.q, case.q_pos, Hk.reshape(batch, L, -1), Hv.reshape(batch, L, -1), case.Bk, case.Bv,
                         layer.group_head_off, layer.k_rank_off, layer.v_rank_off, 128, theta, None, None, layer.q_per_kv)
    err = np.abs(got.cpu().numpy() - want).max() / np.abs(want).max()
    say(f"       rel err to the oracle on the appended cache {err:.3e}")
    assert err <= TOL_FP
