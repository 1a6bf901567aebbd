"""GPU parity: HIP path through the C ABI vs the CPU oracle, element by element,
on seeded inputs at sizes the oracle finishes in seconds.  Shapes span several
32-token tiles, several sequence splits and a ragged tail."""

import numpy as np
import pytest
import torch

from oracle import palu_oracle as O
from workloads import synth

pytestmark = pytest.mark.gpu

from gpu_util import TOL_FP, TOL_I4, rel_err, run_hip, run_oracle, say  # noqa: E402


def check(case, tol, **kw):
    say(f"[parity] {case.name} dtype={case.dtype} B={case.batch} L={case.seq} "
        f"groups={case.layer.n_groups} Rk={case.layer.R_k} kw={ {k: v for k, v in kw.items() if k != 'quant'} }")
    got = run_hip(case, **kw)
    ref = run_oracle(case, **{k: v for k, v in kw.items() if k in ("quant", "k_i4", "v_i4", "bits")})
    assert np.isfinite(got).all()
    whole, rows = rel_err(got, ref)
    say(f"         rel err whole={whole:.3e} worst row={rows:.3e} (tol {tol})")
    assert whole <= tol and rows <= tol
    return whole


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_config1_tiny_full_size(dtype):
    """Configuration 1 at full size: 8 heads, 2 groups of 4, rank 128, L = 1024."""
    layer = synth.config_layer("1")
    case = synth.make_case_orthonormal(layer, 1, 1024, seed=0, dtype=dtype)
    case.name = "cfg1"
    check(case, TOL_FP)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_config2_shape_reduced_length(dtype):
    """7B shape (32 heads, 8 groups of 4, rank 256), two sequences of different
    length, ragged tail (777 = 24 tiles + 9)."""
    layer = synth.config_layer("2")
    case = synth.make_case_svd(layer, 2, 777, seed=0, dtype=dtype)
    case.seq_lens = np.array([777, 300], np.int32)
    case.q_pos = np.array([776, 299], np.int32)
    case.name = "cfg2-reduced"
    check(case, TOL_FP)


def test_config3_ragged_ranks_reduced_length():
    layer = synth.config_layer("3")
    assert max(np.diff(layer.k_rank_off)) > 256 and min(np.diff(layer.k_rank_off)) < 256
    case = synth.make_case_svd(layer, 2, 500, seed=0)
    case.name = "cfg3-reduced"
    check(case, TOL_FP)


@pytest.mark.parametrize("k_i4,v_i4", [(True, True), (False, True)])
def test_config4_int4_reduced_length(k_i4, v_i4):
    layer = synth.config_layer("4")
    case = synth.make_case_svd(layer, 2, 400, seed=0, rotate=True)
    case.name = "cfg4-reduced"
    quant = {"k": O.quant_latent(case.Hk), "v": O.quant_latent(case.Hv)}
    check(case, TOL_I4, k_i4=k_i4, v_i4=v_i4, quant=quant)


def test_config5a_group_size_1_reduced_length():
    layer = synth.config_layer("5a")
    case = synth.make_case_svd(layer, 2, 333, seed=0)
    case.name = "cfg5a-reduced"
    check(case, TOL_FP)


def test_custom_positions_and_single_token():
    layer = synth.uniform_layer(8, 4, 64)
    case = synth.make_case_orthonormal(layer, 2, 70, seed=3)
    case.k_pos = (np.arange(70) * 37 + 5).astype(np.int32)
    case.q_pos = np.array([4000, 17], np.int32)
    case.name = "custom-pos"
    check(case, TOL_FP)
    one = synth.make_case_orthonormal(layer, 1, 1, seed=4)
    one.name = "L=1"
    check(one, TOL_FP)


def test_no_rope():
    """rope_theta <= 0: scores are (q B_k^T) H_k^T / sqrt(d_h) (Eq. 5)."""
    layer = synth.uniform_layer(8, 2, 96, rope_theta=0.0)
    case = synth.make_case_orthonormal(layer, 1, 200, seed=5)
    case.name = "no-rope"
    check(case, TOL_FP)


@pytest.mark.parametrize("cfg,batch,seq,dtype", [("2", 2, 777, "f16"), ("2", 1, 300, "bf16"), ("3", 2, 500, "f16"),
                                                 ("5a", 2, 333, "f16"), ("5b", 1, 200, "f16")])
def test_no_rope_configs(cfg, batch, seq, dtype):
    """The paper's non-RoPE attention (Eq. 5) on the shapes of the configurations: the
    query is folded into the latent space and the keys are never rebuilt."""
    import dataclasses
    layer = dataclasses.replace(synth.config_layer(cfg), rope_theta=0.0)
    kw = {"d_model": 2048} if cfg == "5b" else {}
    case = synth.make_case_svd(layer, batch, seq, seed=2, dtype=dtype, **kw)
    if batch > 1:
        case.seq_lens = np.array([seq, max(1, seq // 3)], np.int32)
        case.q_pos = case.seq_lens - 1
    case.name = f"no-rope cfg{cfg}"
    check(case, TOL_FP)


@pytest.mark.parametrize("k_i4,v_i4", [(True, True), (True, False)])
def test_no_rope_int4(k_i4, v_i4):
    """Non-RoPE path on 4-bit key latents: codes go to the matrix cores as integers,
    scale and zero-point are applied per (token, 128-channel block)."""
    import dataclasses
    layer = dataclasses.replace(synth.config_layer("4"), rope_theta=0.0)
    case = synth.make_case_svd(layer, 2, 400, seed=3, rotate=True)
    case.name = "no-rope int4"
    quant = {"k": O.quant_latent(case.Hk), "v": O.quant_latent(case.Hv)}
    check(case, TOL_I4, k_i4=k_i4, v_i4=v_i4, quant=quant)


@pytest.mark.parametrize("scale", [4.0, 8.0, 12.0])
def test_peaked_softmax_and_large_logits(scale):
    """Queries scaled by 4, 8 and 12 give logits of order +-13, +-27, +-40, the sizes trained models
    produce: the max-subtracted softmax must not overflow, and the logit error must not grow with the
    logit (keys are rebuilt and rotated in float32 from the exact 16-bit inputs): same tolerance."""
    layer = synth.uniform_layer(8, 4, 128)
    case = synth.make_case_orthonormal(layer, 1, 600, seed=6)
    case.q = synth.round_to(case.q * scale, "f16")
    case.name = f"peaked x{scale:g}"
    check(case, TOL_FP)


@pytest.mark.parametrize("theta,dtype,scale", [(0.0, "f16", 12.0), (0.0, "bf16", 12.0), (0.0, "f16", 4.0),
                                               (10000.0, "bf16", 12.0), (500000.0, "f16", 8.0)])
def test_large_logits_other_paths(theta, dtype, scale):
    """The same for the non-RoPE form (folded query kept as an fp16 pair hi + lo), bf16 layers and
    grouped-query heads (each query head rebuilds its keys in float32 by default)."""
    import dataclasses
    layer = dataclasses.replace(synth.uniform_layer(8, 4, 128), rope_theta=theta, q_per_kv=2 if theta > 10000.0 else 1)
    case = synth.make_case_orthonormal(layer, 2, 500, seed=16, dtype=dtype)
    case.q = synth.round_to(case.q * scale, dtype)
    case.name = f"large logits theta={theta:g} x{scale:g}"
    check(case, TOL_FP)


def _bf16_to_fp16_as_documented(h):
    """include/palu.h: clamp to +-65504, else truncate toward zero onto the fp16 grid (exact from 2^-17 up)."""
    h = np.clip(np.asarray(h, np.float64), -65504.0, 65504.0)
    r = h.astype(np.float16)                                    # nearest; step back toward zero where it rounded away
    away = np.abs(r.astype(np.float64)) > np.abs(h)
    r[away] = np.nextafter(r[away], np.float16(0.0))
    return r.astype(np.float64)


@pytest.mark.parametrize("theta", [10000.0, 0.0])
def test_bf16_latents_outside_the_fp16_range(theta):
    """bf16 latents beyond +-65504 and below 2^-17.  RoPE keys: no narrowing (bf16 matrix instruction): all key
    latents times 2^17 with B_k times 2^-17 (both exact in bf16) must give the result of the unscaled layer.
    Values, and keys of the non-RoPE form: the documented conversion to fp16 (clamp, truncate toward zero),
    which the oracle is fed."""
    import dataclasses
    layer = dataclasses.replace(synth.uniform_layer(8, 4, 128), rope_theta=theta)
    case = synth.make_case_orthonormal(layer, 2, 300, seed=23, dtype="bf16")
    rng = np.random.default_rng(5)

    def sprinkle(H):
        tiny = rng.random(H.shape) < 0.2
        huge = rng.random(H.shape) < 0.01
        return synth.round_to(np.where(huge, H * 9.0e4, np.where(tiny, H * 3.0e-6, H)), "bf16")

    case.Hv = sprinkle(case.Hv)
    assert (np.abs(case.Hv) > 65504).any() and ((np.abs(case.Hv) < 2.0 ** -17) & (case.Hv != 0)).any()
    case.name = f"bf16 range theta={theta:g}"
    ref_case = dataclasses.replace(case, Hv=_bf16_to_fp16_as_documented(case.Hv))
    if theta > 0:
        case.Hk = synth.round_to(case.Hk * 2.0 ** 17, "bf16")
        case.Bk = synth.round_to(case.Bk * 2.0 ** -17, "bf16")
        assert (np.abs(case.Hk) > 65504).mean() > 0.5
        ref_case.Hk, ref_case.Bk = case.Hk, case.Bk              # the oracle sees the same scaled pair: same keys
    else:
        case.q = synth.round_to(case.q * 1.0e-4, "bf16")         # keeps the logits of the clamped entries moderate
        case.Hk = sprinkle(case.Hk)
        assert (np.abs(case.Hk) > 65504).any()
        ref_case.q, ref_case.Hk = case.q, _bf16_to_fp16_as_documented(case.Hk)
    got = run_hip(case)
    assert np.isfinite(got).all()
    whole, rows = rel_err(got, run_oracle(ref_case))
    say(f"         {case.name}: rel err {whole:.3e} rows {rows:.3e}")
    assert max(whole, rows) <= TOL_FP


@pytest.mark.parametrize("cfg,L,scale", [("1", 300, 1.0), ("2", 500, 1.0), ("2", 333, 8.0), ("5a", 200, 1.0)])
def test_score_fp8_option(cfg, L, scale):
    """Opt-in low-precision key reconstruction (Sec. 4.5.2, last paragraph): keys rebuilt from E4M3-rounded latents
    and column-scaled E4M3 weights on the 8-bit matrix instruction.  The oracle rounds the same operands the same
    way (O.attn_decode_fp8_keys); what remains is float32 accumulation, so the plain tolerance applies.  The
    distance to the unrounded attention is printed: it is the price of the format, not an error of the kernel."""
    import paper_2407_21118_amd as P
    layer = synth.config_layer(cfg)
    case = synth.make_case_svd(layer, 2, L, seed=31) if cfg != "1" else synth.make_case_orthonormal(layer, 2, L, seed=31)
    case.q = synth.round_to(case.q * scale, "f16")
    case.seq_lens = np.array([L, L - 37], np.int32)
    case.q_pos = (case.seq_lens - 1).astype(np.int32)
    case.name = f"fp8 keys cfg {cfg} x{scale:g}"
    P.palu_set_option("score_fp8", 1)
    try:
        got = run_hip(case)
    finally:
        P.palu_set_option("score_fp8", 0)
    assert np.isfinite(got).all()
    ref8 = O.attn_decode_fp8_keys(case.q, case.q_pos, case.Hk, case.Hv, case.Bk, case.Bv, layer.group_head_off, layer.k_rank_off,
                                  layer.v_rank_off, layer.d_head, layer.rope_theta, case.k_pos, case.seq_lens, layer.q_per_kv)
    whole, rows = rel_err(got, ref8)
    w2, r2 = rel_err(got, run_oracle(case))
    say(f"[parity] {case.name}: against the oracle on the same rounded operands {whole:.3e} (rows {rows:.3e}); "
        f"against unrounded attention {w2:.3e} (rows {r2:.3e})")
    assert whole <= TOL_FP and rows <= TOL_FP


def test_shared_key_fp16_option():
    """The opt-in shared-key score form (fp16-rounded keys and angles in the query contraction, each key rebuilt
    once for the queries that share it): within the tolerance at logits of order +-3; its error grows with the
    logit, which is why it is not the default."""
    import dataclasses
    import paper_2407_21118_amd as P
    layer = dataclasses.replace(synth.uniform_layer(8, 4, 128), q_per_kv=4)
    case = synth.make_case_orthonormal(layer, 2, 300, seed=21)
    case.name = "shared-key fp16"
    P.palu_set_option("shared_key_fp16", 1)
    try:
        check(case, TOL_FP)
    finally:
        P.palu_set_option("shared_key_fp16", 0)


def test_config5b_joint_group_reduced_length():
    """J-LRD: one group of all 32 heads, rank 2048 (contracted in rank slices)."""
    layer = synth.config_layer("5b")
    case = synth.make_case_svd(layer, 1, 200, seed=0, d_model=2048)
    case.name = "cfg5b-reduced"
    check(case, TOL_FP)


def test_mixed_group_sizes_and_ranks():
    """Groups of 1, 2, 3 and 6 heads with ranks 32 .. 512 in one layer."""
    k_ranks = [32, 64, 128, 96, 128, 384, 512]          # each at most the group's width (heads * 128)
    v_ranks = [64, 32, 128, 256, 96, 128, 512]
    layer = synth.Layer(16, 128, [0, 1, 2, 4, 6, 7, 10, 16], [0] + list(np.cumsum(k_ranks)),
                        [0] + list(np.cumsum(v_ranks)))
    case = synth.make_case_orthonormal(layer, 2, 150, seed=8)
    case.seq_lens = np.array([150, 33], np.int32)
    case.q_pos = np.array([149, 32], np.int32)
    case.name = "mixed"
    check(case, TOL_FP)


@pytest.mark.parametrize("mode", [1, 0, 3])
def test_rank_classes_in_one_score_launch(mode):
    """A layer whose groups have different key ranks (the ranks a per-group search assigns, Sec. 3.3; above 256 in two
    slices): by default ONE score launch covers all rank classes, each with its own chunk length (mode 1); the
    option's other values give a launch per class (0) and several rounds of mixed workgroups (3).  Long enough for
    several chunks per class, ragged lengths, bf16 in one case."""
    k_ranks = [416, 352, 224, 256, 128, 64, 96]
    v_ranks = [128, 256, 96, 128, 64, 128, 32]
    sizes = [4, 4, 4, 2, 2, 1, 1]
    layer = synth.Layer(sum(sizes), 128, [0] + list(np.cumsum(sizes)), [0] + list(np.cumsum(k_ranks)),
                        [0] + list(np.cumsum(v_ranks)))
    case = synth.make_case_orthonormal(layer, 3, 1500, seed=77 + mode, dtype="bf16" if mode == 3 else "f16")
    case.seq_lens = np.array([1500, 1, 700], np.int32)
    case.q_pos = np.array([1499, 5, 800], np.int32)
    case.q = synth.round_to(case.q * 4.0, case.dtype)
    case.name = f"rank classes in one launch, score_mixed={mode}"
    import paper_2407_21118_amd as P
    P.palu_set_option("score_mixed", mode)
    try:
        check(case, TOL_FP)
    finally:
        P.palu_set_option("score_mixed", 1)


@pytest.mark.parametrize("kind", ["rising", "large-scale", "tiny-scale"])
def test_value_kernel_lazy_maximum_4bit(kind):
    """4-bit value latents under the value kernel's lazy running maximum: logits that keep rising along the sequence
    (the maximum is raised again and again, in steps above and below its threshold), value latents whose quantization
    scales exceed 128 (the kernel then keeps the exact maximum so that probability x scale stays inside fp16), and
    tiny scales (weights near the bottom of the fp16 range)."""
    layer = synth.uniform_layer(8, 4, 256)
    case = synth.make_case_orthonormal(layer, 2, 700, seed=55)
    case.seq_lens = np.array([700, 90], np.int32)
    case.q_pos = (case.seq_lens - 1).astype(np.int32)
    if kind == "rising":
        # keys that grow along the sequence in the query's direction: scores rise by a fraction of a unit per token, with jumps
        ramp = (1.0 + np.arange(700, dtype=np.float32) / 100.0 + 3.0 * (np.arange(700) % 97 == 0))[None, :, None]
        case.Hk = synth.round_to(case.Hk * ramp, "f16")
    elif kind == "large-scale":
        case.Hv = synth.round_to(case.Hv * 3000.0, "f16")
    else:
        case.Hv = synth.round_to(case.Hv * 1e-3, "f16")
    quant = {"k": O.quant_latent(case.Hk), "v": O.quant_latent(case.Hv)}
    if kind == "large-scale":
        assert np.asarray(quant["v"][1], np.float32).max() > 128.0
    case.name = f"4-bit values, lazy maximum: {kind}"
    check(case, TOL_I4, k_i4=False, v_i4=True, quant=quant)


def _random_layer(rng, theta):
    """A random legal layer: groups of 1..8 heads, ranks in multiples of 32 up to
    min(512, width of the group), different for keys and values."""
    sizes = []
    while sum(sizes) < 4 or (len(sizes) < 6 and rng.random() < 0.6):
        sizes.append(int(rng.choice([1, 1, 2, 3, 4, 4, 8])))
    head_off = [0] + list(np.cumsum(sizes))

    def ranks():
        return [int(rng.integers(1, min(512, s * 128) // 32 + 1)) * 32 for s in sizes]

    return synth.Layer(int(head_off[-1]), 128, head_off, [0] + list(np.cumsum(ranks())), [0] + list(np.cumsum(ranks())),
                       rope_theta=theta)


@pytest.mark.parametrize("seed", list(range(12)))
def test_random_layers_and_lengths(seed):
    """Seeded random layers (group sizes, ranks, with and without RoPE), batch sizes,
    lengths and ragged sequence lengths: exercises the merging and slicing of work
    units, partial tiles and sets, and sequences much shorter than the batch's longest."""
    rng = np.random.default_rng([77, seed])
    theta = 10000.0 if seed % 3 else 0.0
    layer = _random_layer(rng, theta)
    batch = int(rng.integers(1, 4))
    seq = int(rng.choice([1, 2, 31, 32, 33, 65, 130, 257, 300]))
    dtype = "bf16" if seed % 4 == 1 else "f16"
    case = synth.make_case_orthonormal(layer, batch, seq, seed=100 + seed, dtype=dtype)
    lens = np.array([seq] + [int(rng.integers(1, seq + 1)) for _ in range(batch - 1)], np.int32)
    case.seq_lens = lens
    case.q_pos = (lens - 1 + int(rng.integers(0, 5000))).astype(np.int32)
    if seed % 2:
        case.k_pos = np.sort(rng.choice(8192, size=seq, replace=False)).astype(np.int32)
    case.name = f"random-{seed} heads={layer.n_heads} groups={layer.n_groups} theta={theta}"
    check(case, TOL_FP)


@pytest.mark.parametrize("bits", [4, 3])
def test_quantized_keys_far_off_centre(bits):
    """Key latents with a large common offset and a small spread: zero-points in the thousands, outside the range in
    which the score kernel dequantizes in packed fp16 arithmetic; it must take its float32 form and still agree."""
    layer = synth.uniform_layer(8, 4, 256)
    case = synth.make_case_orthonormal(layer, 2, 150, seed=41)
    case.Hk = synth.round_to(0.01 * case.Hk + 12.0, "f16")
    case.name = f"far-off-centre keys, {bits} bits"
    quant = {"k": O.quant_latent(case.Hk, bits=bits), "v": O.quant_latent(case.Hv, bits=bits)}
    assert np.abs(np.asarray(quant["k"][2], np.float32)).max() > 1000.0
    check(case, TOL_I4, k_i4=True, v_i4=False, quant=quant, bits=bits)


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_random_layers_int4(seed):
    """Random layers whose ranks are multiples of the 128-channel quantization block,
    key and / or value latents 4-bit, with and without RoPE."""
    rng = np.random.default_rng([78, seed])
    sizes = [int(rng.choice([1, 2, 4, 8])) for _ in range(int(rng.integers(2, 5)))]
    head_off = [0] + list(np.cumsum(sizes))
    kr = [int(rng.integers(1, min(512, s * 128) // 128 + 1)) * 128 for s in sizes]
    vr = [int(rng.integers(1, min(512, s * 128) // 128 + 1)) * 128 for s in sizes]
    layer = synth.Layer(int(head_off[-1]), 128, head_off, [0] + list(np.cumsum(kr)), [0] + list(np.cumsum(vr)),
                        rope_theta=0.0 if seed % 2 else 10000.0)
    batch, seq = 2, int(rng.choice([33, 100, 260]))
    case = synth.make_case_orthonormal(layer, batch, seq, seed=200 + seed)
    case.seq_lens = np.array([seq, int(rng.integers(1, seq + 1))], np.int32)
    case.q_pos = (case.seq_lens - 1).astype(np.int32)
    case.name = f"random-int4-{seed} groups={sizes} k_ranks={kr} v_ranks={vr}"
    quant = {"k": O.quant_latent(case.Hk), "v": O.quant_latent(case.Hv)}
    check(case, TOL_I4, k_i4=seed != 3, v_i4=seed != 2, quant=quant)


@pytest.mark.parametrize("qpk,theta,dtype", [(4, 500000.0, "f16"), (4, 0.0, "f16"), (2, 10000.0, "bf16"), (8, 10000.0, "f16"),
                                             (3, 10000.0, "f16"), (5, 500000.0, "f16"), (12, 10000.0, "f16")])
def test_grouped_query_attention(qpk, theta, dtype):
    """Grouped-query attention (the Llama-3 / Mistral models of Sec. 4.1): the latents and
    B matrices cover the key/value heads, q_per_kv query heads share each of them.  Groups
    of unequal size and rank (64 .. 256 in one layer), ragged lengths, with and without RoPE; with RoPE
    each key is rebuilt once for the query heads that share it (2 .. 12 of them: passes of 4 rows)."""
    n_kv = 8 if qpk <= 4 else 4
    sizes = [4, 2, 1, 1] if n_kv == 8 else [2, 1, 1]
    head_off = [0] + list(np.cumsum(sizes))
    kr = [256, 96, 64, 128][:len(sizes)]
    vr = [192, 128, 32, 96][:len(sizes)]
    layer = synth.Layer(n_kv, 128, head_off, [0] + list(np.cumsum(kr)), [0] + list(np.cumsum(vr)), rope_theta=theta,
                        q_per_kv=qpk)
    case = synth.make_case_orthonormal(layer, 2, 300, seed=300 + qpk, dtype=dtype)
    case.seq_lens = np.array([300, 131], np.int32)
    case.q_pos = np.array([310, 130], np.int32)
    if qpk in (3, 8):
        case.k_pos = np.sort(np.random.default_rng(qpk).choice(4096, size=300, replace=False)).astype(np.int32)
        case.q_pos = np.array([4100, 2000], np.int32)
    case.name = f"gqa q_per_kv={qpk} kv_heads={n_kv} groups={sizes} theta={theta}"
    check(case, TOL_FP)


@pytest.mark.parametrize("rank,qpk,sizes,dtype,scale", [(256, 4, [4, 4], "f16", 8.0), (256, 8, [2, 4, 2], "f16", 1.0),
                                                        (192, 8, [4], "bf16", 4.0), (224, 2, [4, 3, 2], "f16", 12.0),
                                                        (160, 4, [2, 2], "f16", 1.0), (128, 2, [4, 4, 1], "bf16", 8.0),
                                                        (256, 3, [4, 2], "f16", 8.0), (192, 5, [2, 2], "f16", 1.0),
                                                        (128, 6, [4, 1], "bf16", 1.0), (256, 12, [2, 2], "f16", 4.0),
                                                        (224, 16, [4], "f16", 1.0), (160, 7, [2], "f16", 12.0),
                                                        (384, 4, [4, 3], "f16", 8.0), (512, 2, [4], "bf16", 1.0),
                                                        (288, 3, [3, 4], "f16", 4.0)])
def test_shared_keys_exact_form(rank, qpk, sizes, dtype, scale):
    """Layers whose key ranks are all 128 .. 512 (above 256: two slices) with several query heads per key/value head: the score kernel
    rebuilds and rotates each key once in float32 for the queries that share it (in passes of up to 8 query rows, 4
    at ranks below 192; a pass of 3 or 5 .. 7 rows runs the 4- or 8-row kernel with idle rows).  Same tolerance as one
    query per head, also at the large logits of scaled queries; ragged lengths, gathered positions in one case."""
    n_kv = sum(sizes)
    head_off = [0] + list(np.cumsum(sizes))
    kr = [rank] * len(sizes)
    vr = [128 if s == 1 else 192 for s in sizes]
    layer = synth.Layer(n_kv, 128, head_off, [0] + list(np.cumsum(kr)), [0] + list(np.cumsum(vr)), rope_theta=500000.0,
                        q_per_kv=qpk)
    case = synth.make_case_orthonormal(layer, 2, 333, seed=700 + rank + qpk, dtype=dtype)
    case.q = synth.round_to(case.q * scale, dtype)
    case.seq_lens = np.array([333, 150], np.int32)
    case.q_pos = np.array([340, 149], np.int32)
    if qpk == 4:
        case.k_pos = np.sort(np.random.default_rng(rank).choice(5000, size=333, replace=False)).astype(np.int32)
        case.q_pos = np.array([5001, 3000], np.int32)
    case.name = f"shared keys rank={rank} q_per_kv={qpk} groups={sizes} {dtype} q x{scale:g}"
    check(case, TOL_FP)


@pytest.mark.parametrize("rank,qpk,sizes,offset", [(128, 4, [2, 4, 1], 0.0), (256, 8, [4, 2], 0.0), (256, 3, [4], 0.0),
                                                  (128, 6, [4, 4], 0.0), (256, 2, [2, 2], 12.0)])
def test_shared_keys_quantized(rank, qpk, sizes, offset):
    """4-bit key latents of rank 128 / 256 with several query heads per key/value head: a key tile is dequantized,
    rebuilt and rotated once per pass for the queries that share it.  One case has key latents far off centre
    (zero-points in the thousands: the float32 form of the dequantizer)."""
    n_kv = sum(sizes)
    head_off = [0] + list(np.cumsum(sizes))
    kr = [rank] * len(sizes)
    vr = [128] * len(sizes)
    layer = synth.Layer(n_kv, 128, head_off, [0] + list(np.cumsum(kr)), [0] + list(np.cumsum(vr)), rope_theta=10000.0,
                        q_per_kv=qpk)
    case = synth.make_case_orthonormal(layer, 2, 211, seed=900 + rank + qpk)
    if offset:
        case.Hk = synth.round_to(0.01 * case.Hk + offset, "f16")
    case.seq_lens = np.array([211, 70], np.int32)
    case.q_pos = (case.seq_lens - 1).astype(np.int32)
    case.name = f"shared keys, 4-bit, rank={rank} q_per_kv={qpk} groups={sizes} offset={offset:g}"
    quant = {"k": O.quant_latent(case.Hk), "v": O.quant_latent(case.Hv)}
    if offset:
        assert np.abs(np.asarray(quant["k"][2], np.float32)).max() > 1000.0
    check(case, TOL_I4, k_i4=True, v_i4=True, quant=quant)


@pytest.mark.parametrize("k_i4,v_i4,theta", [(True, True, 500000.0), (True, True, 0.0)])
def test_grouped_query_attention_int4(k_i4, v_i4, theta):
    import dataclasses
    layer = dataclasses.replace(synth.config_layer("gqa"), rope_theta=theta)
    case = synth.make_case_svd(layer, 2, 260, seed=31, rotate=True)
    case.seq_lens = np.array([260, 97], np.int32)
    case.q_pos = (case.seq_lens - 1).astype(np.int32)
    case.name = f"gqa-int4 theta={theta}"
    quant = {"k": O.quant_latent(case.Hk), "v": O.quant_latent(case.Hv)}
    check(case, TOL_I4, k_i4=k_i4, v_i4=v_i4, quant=quant)


def test_parallel_queries_share_the_cache():
    """Several queries per sequence at the same position (parallel samples or beams over a
    shared prefix) are the grouped-query case with q_per_kv = number of queries: query j of
    head i goes to row i * n_q + j.  One call must agree with the oracle and with n_q
    single-query calls on the same cache."""
    import dataclasses
    n_q = 4
    base = synth.uniform_layer(8, 4, 128, 96)
    multi = dataclasses.replace(base, q_per_kv=n_q)
    case = synth.make_case_orthonormal(multi, 2, 200, seed=41)
    case.seq_lens = np.array([200, 61], np.int32)
    case.q_pos = np.array([205, 60], np.int32)
    case.name = f"parallel queries n_q={n_q}"
    check(case, TOL_FP)
    got = run_hip(case)
    for j in range(n_q):
        single = dataclasses.replace(case, layer=base, q=np.ascontiguousarray(case.q[:, j::n_q]))
        one = run_hip(single)
        whole, rows = rel_err(got[:, j::n_q], one.astype(np.float64))
        say(f"         query {j}: against its own single-query call {whole:.3e}")
        assert whole <= TOL_FP and rows <= TOL_FP


@pytest.mark.parametrize("n_q,qpk,theta,i4", [(4, 1, 10000.0, False), (2, 4, 500000.0, False), (5, 2, 10000.0, False),
                                              (3, 1, 0.0, False), (4, 1, 10000.0, True), (16, 1, 10000.0, False), (24, 1, 10000.0, False)])
def test_several_queries_per_sequence(n_q, qpk, theta, i4):
    """palu_attn_decode_multi: a causal block of n_q new tokens per sequence (rows appended
    first; query j attends len - n_q + j + 1 rows at its own position), multi-head and
    grouped-query layers, with and without RoPE, fp16 and 4-bit latents.  The oracle runs
    every query as its own decode step."""
    import paper_2407_21118_amd as P
    from gpu_util import make_desc, to_dev
    sizes = [4, 2, 2] if qpk == 1 else [2, 1, 1]
    head_off = [0] + list(np.cumsum(sizes))
    kr = [256, 128, 128]
    vr = [128, 256, 128] if qpk == 1 else [128, 128, 128]      # a rank cannot exceed the group's width
    layer = synth.Layer(int(head_off[-1]), 128, head_off, [0] + list(np.cumsum(kr)), [0] + list(np.cumsum(vr)),
                        rope_theta=theta, q_per_kv=qpk)
    B, L = 2, 300
    case = synth.make_case_orthonormal(layer, B, L, seed=500 + n_q)
    rng = np.random.default_rng([9, n_q, qpk])
    q = synth.round_to(rng.standard_normal((B, n_q, layer.n_q_heads, 128)), "f16")
    lens = np.array([L, 157], np.int32)
    q_len = (lens[:, None] - n_q + np.arange(n_q)[None, :] + 1).astype(np.int32)
    q_pos = (q_len - 1 + 7).astype(np.int32)
    say(f"[multi] n_q={n_q} q_per_kv={qpk} theta={theta} int4={i4} groups={sizes}")
    desc = make_desc(layer, "f16", i4, i4)
    kw, Hk_ref, Hv_ref = {}, case.Hk, case.Hv
    if i4:
        (pk, sk, zk), (pv, sv, zv) = O.quant_latent(case.Hk), O.quant_latent(case.Hv)
        hk, hv = torch.from_numpy(pk).cuda(), torch.from_numpy(pv).cuda()
        for name, arr in (("hk_scale", sk), ("hk_zero", zk), ("hv_scale", sv), ("hv_zero", zv)):
            kw[name] = torch.from_numpy(arr.view(np.int16)).cuda().view(torch.float16)
        Hk_ref, Hv_ref = O.dequant_latent(pk, sk, zk), O.dequant_latent(pv, sv, zv)
    else:
        hk, hv = to_dev(case.Hk, "f16"), to_dev(case.Hv, "f16")
    n_pos = int(q_pos.max()) + 1
    table = P.palu_rope_table_init(theta, 128, max(n_pos, L))
    out = P.palu_attn_decode_multi(desc, B, n_q, L, L, to_dev(q, "f16"), torch.from_numpy(q_pos).cuda(), hk, hv,
                                   to_dev(case.Bk, "f16"), to_dev(case.Bv, "f16"), table, max(n_pos, L),
                                   q_len=torch.from_numpy(q_len).cuda(), seq_lens=torch.from_numpy(lens).cuda(), **kw)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    ref = O.attn_decode_multi(q, q_pos, q_len, Hk_ref, Hv_ref, case.Bk, case.Bv, layer.group_head_off, layer.k_rank_off,
                              layer.v_rank_off, 128, theta, None, qpk)
    assert np.isfinite(got).all()
    whole, rows = rel_err(got.reshape(B, -1, 128), ref.reshape(B, -1, 128))
    say(f"        rel err whole={whole:.3e} worst row={rows:.3e}")
    tol = TOL_I4 if i4 else TOL_FP
    assert whole <= tol and rows <= tol


@pytest.mark.parametrize("bits,theta,k_q,v_q", [(2, 10000.0, True, True), (3, 10000.0, True, True), (2, 0.0, True, True),
                                                 (3, 0.0, True, True), (3, 10000.0, False, True), (2, 10000.0, True, False)])
def test_low_bit_latents(bits, theta, k_q, v_q):
    """2- and 3-bit latents (Sec. 4.4), Hadamard-rotated factors as in Sec. 3.4: key and / or value
    side, with and without RoPE, a ragged layer (ranks 128 .. 384), ragged lengths.  The oracle is fed
    the same dequantized values; what is measured is the kernels' arithmetic, as for 4 bits."""
    import dataclasses
    layer = synth.Layer(10, 128, [0, 4, 6, 7, 10], [0, 256, 384, 512, 896], [0, 384, 512, 640, 896], rope_theta=theta)
    case = synth.make_case_svd(layer, 2, 270, seed=60 + bits, rotate=False)
    case.seq_lens = np.array([270, 99], np.int32)
    case.q_pos = (case.seq_lens - 1).astype(np.int32)
    case.name = f"{bits}-bit latents theta={theta} K={k_q} V={v_q}"
    quant = {"k": O.quant_latent(case.Hk, bits=bits), "v": O.quant_latent(case.Hv, bits=bits)}
    check(case, TOL_I4, k_i4=k_q, v_i4=v_q, quant=quant, bits=bits)


def test_low_bit_latents_grouped_query_and_config4_shape():
    """3-bit keys and 2-bit-free mix on the 7B shape at reduced length and on a grouped-query layer."""
    for cfg, bits in (("4", 3), ("gqa", 2)):
        layer = synth.config_layer(cfg)
        case = synth.make_case_svd(layer, 2, 200, seed=70 + bits, rotate=True)
        case.name = f"config {cfg} with {bits}-bit latents"
        quant = {"k": O.quant_latent(case.Hk, bits=bits), "v": O.quant_latent(case.Hv, bits=bits)}
        check(case, TOL_I4, k_i4=True, v_i4=True, quant=quant, bits=bits)


@pytest.mark.parametrize("theta", [10000.0, 0.0])
def test_build_limits_256_heads_64_groups(theta):
    """The largest layer the build accepts: 256 heads in 64 groups (PALU_MAX_HEADS, PALU_MAX_GROUPS)."""
    layer = synth.uniform_layer(256, 4, 64, 32, rope_theta=theta)
    case = synth.make_case_orthonormal(layer, 1, 77, seed=88)
    case.name = f"256 heads / 64 groups theta={theta}"
    check(case, TOL_FP)


@pytest.mark.parametrize("theta,i4", [(10000.0, False), (0.0, False), (10000.0, True), (0.0, True)])
def test_idle_sequences_and_queries_give_zeros(theta, i4):
    """A sequence with no cached row (an idle slot of the batch) and a query that attends no row get
    output rows of zeros, exactly; their neighbours in the batch are unaffected.  Single-query call,
    latent output and the several-queries call, with and without RoPE, fp16 and 4-bit latents."""
    import paper_2407_21118_amd as P
    from gpu_util import make_desc, to_dev
    layer = synth.Layer(8, 128, [0, 4, 8], [0, 256, 384], [0, 128, 384], rope_theta=theta)
    B, L, n_q = 3, 200, 3
    case = synth.make_case_orthonormal(layer, B, L, seed=77)
    lens = np.array([L, 0, 57], np.int32)
    case.seq_lens, case.q_pos = lens, np.maximum(lens - 1, 0).astype(np.int32)
    say(f"[idle] theta={theta} int4={i4} lens={lens.tolist()}")
    quant = {"k": O.quant_latent(case.Hk), "v": O.quant_latent(case.Hv)} if i4 else None
    tol = TOL_I4 if i4 else TOL_FP
    got = run_hip(case, k_i4=i4, v_i4=i4, quant=quant)
    ref = run_oracle(case, quant, i4, i4)
    assert np.isfinite(got).all() and not got[1].any() and not ref[1].any()
    live = [0, 2]
    whole, rows = rel_err(got[live], ref[live])
    say(f"       single query: rel err {whole:.3e}")
    assert max(whole, rows) <= tol

    desc = make_desc(layer, "f16", i4, i4)
    kw, Hk_ref, Hv_ref = {}, case.Hk, case.Hv
    if i4:
        (pk, sk, zk), (pv, sv, zv) = quant["k"], quant["v"]
        hk, hv = torch.from_numpy(pk).cuda(), torch.from_numpy(pv).cuda()
        for name, arr in (("hk_scale", sk), ("hk_zero", zk), ("hv_scale", sv), ("hv_zero", zv)):
            kw[name] = torch.from_numpy(arr.view(np.int16)).cuda().view(torch.float16)
        Hk_ref, Hv_ref = O.dequant_latent(pk, sk, zk), O.dequant_latent(pv, sv, zv)
    else:
        hk, hv = to_dev(case.Hk, "f16"), to_dev(case.Hv, "f16")
    table = P.palu_rope_table_init(theta, 128, L + 8)
    d_lens, Bk, Bv = torch.from_numpy(lens).cuda(), to_dev(case.Bk, "f16"), to_dev(case.Bv, "f16")

    lat = P.palu_attn_decode_latent(desc, B, L, L, to_dev(case.q, "f16"), torch.from_numpy(case.q_pos).cuda(), hk, hv, Bk,
                                    table, L + 8, seq_lens=d_lens, **kw)
    torch.cuda.synchronize()
    lat = lat.cpu().numpy()
    lat_ref = O.attn_decode_latent(case.q, case.q_pos, Hk_ref, Hv_ref, case.Bk, layer.group_head_off, layer.k_rank_off,
                                   layer.v_rank_off, 128, theta, None, lens)
    assert np.isfinite(lat).all() and not lat[1].any()
    whole = np.abs(lat[live] - lat_ref[live]).max() / np.abs(lat_ref[live]).max()
    say(f"       latent output: rel err {whole:.3e}")
    assert whole <= tol

    rng = np.random.default_rng([78, int(theta), int(i4)])
    q = synth.round_to(rng.standard_normal((B, n_q, layer.n_q_heads, 128)), "f16")
    q_len = np.array([[L, 0, 150], [0, 0, 0], [57, 20, 0]], np.int32)
    q_pos = (np.maximum(q_len - 1, 0) + 3).astype(np.int32)
    out = P.palu_attn_decode_multi(desc, B, n_q, L, L, to_dev(q, "f16"), torch.from_numpy(q_pos).cuda(), hk, hv, Bk, Bv,
                                   table, L + 8, q_len=torch.from_numpy(q_len).cuda(), seq_lens=d_lens, **kw)
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    mref = O.attn_decode_multi(q, q_pos, q_len, Hk_ref, Hv_ref, case.Bk, case.Bv, layer.group_head_off, layer.k_rank_off,
                               layer.v_rank_off, 128, theta, None, 1)
    assert np.isfinite(out).all()
    for b in range(B):
        for j in range(n_q):
            if q_len[b, j] == 0:
                assert not out[b, j].any() and not mref[b, j].any()
            else:
                whole, rows = rel_err(out[b, j][None], mref[b, j][None])
                assert max(whole, rows) <= tol, (b, j, whole, rows)
    say("       several queries: idle rows zero, the rest within tolerance")
