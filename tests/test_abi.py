"""CPU-side checks of the boundary: the library loads, exports every symbol the
header declares, and validates arguments on the host (no kernel is launched)."""

import ctypes
import os
import re

import pytest

import paper_2407_21118_amd as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "palu.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(palu_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = P.load_library()
    names = declared_symbols()
    assert {"palu_encode", "palu_attn_decode", "palu_quant_latent"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings_and_version():
    assert P.palu_version() >= 100
    assert P.palu_status_string(0) == "ok"
    for s in (-1, -2, -3, -4, -99):
        assert P.palu_status_string(s)


def desc(**kw):
    a = dict(n_heads=8, d_head=128, group_head_off=[0, 4, 8], k_rank_off=[0, 64, 128], v_rank_off=[0, 64, 128])
    a.update(kw)
    return P.LayerDesc(**a)


def test_workspace_queries_are_host_only():
    d = desc()
    assert P.palu_attn_decode_workspace_bytes(d, 2, 1000) > 0
    assert P.palu_encode_workspace_bytes(d, 0, 3) > 0
    assert P.palu_rope_table_bytes(128, 1000) == 32 * (16384 + 8192)      # whole tiles of 32 positions: float32 angles + float16 rows


@pytest.mark.parametrize("kw,status", [
    (dict(k_rank_off=[0, 60, 128]), -1),                 # rank not a multiple of 32
    (dict(group_head_off=[0, 4, 7]), -1),                # heads do not add up
    (dict(group_head_off=[0, 8, 8]), -1),                # empty group
    (dict(d_head=64), -2),                               # unsupported head width
    (dict(act_dtype=5), -1),
    (dict(k_latent_dtype=P.PALU_I4, k_rank_off=[0, 64, 128]), -1),   # int4 needs ranks in multiples of the block
    (dict(k_rank_off=[0, 4096, 8192]), -2),              # rank above the build limit
    (dict(q_per_kv=-1), -1),                             # negative query-head count
    (dict(q_per_kv=64), -2),                             # 8 * 64 query heads: above the build limit
    (dict(v_latent_dtype=7), -1),                        # unknown latent dtype
    (dict(v_latent_dtype=P.PALU_I2, v_rank_off=[0, 64, 128]), -1),   # 2-bit latents need ranks in multiples of the block
    (dict(k_latent_dtype=P.PALU_I3, act_dtype=P.PALU_BF16, k_rank_off=[0, 128, 256]), -2),   # quantized sides: fp16 layers only
])
def test_descriptor_validation(kw, status):
    with pytest.raises(P.PaluError) as e:
        P.palu_attn_decode_workspace_bytes(desc(**kw), 1, 128)
    assert e.value.status == status


def test_grouped_query_and_multi_query_workspace_grow_with_the_queries():
    lib = P.load_library()
    base = P.palu_attn_decode_workspace_bytes(desc(), 2, 4096)
    gqa = P.palu_attn_decode_workspace_bytes(desc(q_per_kv=4), 2, 4096)
    assert gqa > base
    out = ctypes.c_size_t(0)
    assert lib.palu_attn_decode_multi_workspace_bytes(desc().ref(), 2, 4, 4096, ctypes.byref(out)) == 0
    assert out.value == gqa                              # 4 queries per key/value head either way
    assert lib.palu_attn_decode_multi_workspace_bytes(desc().ref(), 2, 0, 4096, ctypes.byref(out)) == -1
    assert lib.palu_attn_decode_multi_workspace_bytes(desc().ref(), 2, 64, 4096, ctypes.byref(out)) == -2
    # the fused projection + quantizer writes 4-bit codes only
    d3 = desc(k_latent_dtype=P.PALU_I3, k_rank_off=[0, 128, 256])
    one = ctypes.c_void_p(256)                           # non-NULL, aligned; never dereferenced: the call is refused first
    assert lib.palu_encode_quant(d3.ref(), 0, one, 1, one, one, one, one, None, None) == -2


def test_null_and_range_arguments():
    lib = P.load_library()
    d = desc()
    out = ctypes.c_size_t(0)
    assert lib.palu_attn_decode_workspace_bytes(None, 1, 1, ctypes.byref(out)) == -1
    assert lib.palu_attn_decode_workspace_bytes(d.ref(), 0, 1, ctypes.byref(out)) == -1
    assert lib.palu_attn_decode_workspace_bytes(d.ref(), 1, 1, None) == -1
    assert lib.palu_rope_table_bytes(128, 0, ctypes.byref(out)) == -1
    assert lib.palu_rope_table_init(10000.0, 128, 16, None, None) == -1
    assert lib.palu_encode(d.ref(), 2, None, 1, None, None, 128, None, None, 0, None) == -1
    assert lib.palu_quant_latent(d.ref(), 0, None, 128, 1, None, None, None, None, None) == -1
    assert lib.palu_attn_decode(d.ref(), 1, 8, 8, *([None] * 13), 8, None, None, 0, None) == -1


def test_transposed_weight_entry_points_refuse_what_they_do_not_do():
    """palu_encode_kv_t / palu_decode_step_t: NULL and misaligned pointers, prompt-sized token counts and
    quantized caches are refused on the host, before anything is launched."""
    lib = P.load_library()
    d = desc()
    one, odd = ctypes.c_void_p(256), ctypes.c_void_p(264)    # non-NULL; never dereferenced: the calls are refused first
    R = 128                                                  # desc(): two groups of rank 64
    assert lib.palu_encode_kv_t(None, one, 1, one, one, one, R, one, R, None, None) == -1
    assert lib.palu_encode_kv_t(d.ref(), None, 1, one, one, one, R, one, R, None, None) == -1
    assert lib.palu_encode_kv_t(d.ref(), one, 0, one, one, one, R, one, R, None, None) == -1
    assert lib.palu_encode_kv_t(d.ref(), one, 1, odd, one, one, R, one, R, None, None) == -1      # weights: 16-byte aligned
    assert lib.palu_encode_kv_t(d.ref(), one, 1, one, one, one, R - 2, one, R, None, None) == -1  # row stride below the rank
    assert lib.palu_encode_kv_t(d.ref(), one, 64, one, one, one, R, one, R, None, None) == -2     # a prompt: the GEMM form
    dq = desc(v_latent_dtype=P.PALU_I4, v_rank_off=[0, 128, 256])
    assert lib.palu_encode_kv_t(dq.ref(), one, 1, one, one, one, R, one, R, None, None) == -2
    args = [one, one, one, one, one, one, one, one, None, None, one, one, one, 8, one, one, 1 << 20, None]
    assert lib.palu_decode_step_t(d.ref(), 64, 8, 8, *args) == -2
    assert lib.palu_decode_step_t(d.ref(), 0, 8, 8, *args) == -1
    assert lib.palu_decode_step_t(dq.ref(), 1, 8, 8, *args) == -2


def test_options_are_validated_on_the_host():
    """palu_set_option: unknown names, NULL and out-of-range values are refused (-1) and leave the setting alone;
    the documented values are accepted.  Every option is put back to its default."""
    lib = P.load_library()
    assert lib.palu_set_option(None, 0) == -1
    assert lib.palu_set_option(b"no_such_option", 1) == -1
    assert lib.palu_set_option(b"score_mixed", -1) == -1
    for name, good, bad, default in ((b"score_mixed", (0, 1, 3, 16), (17,), 1), (b"score_waves", (0, 4, 8), (3, 16), 0),
                                     (b"value_split_tokens", (0, 32, 4096), (48, 8192), 0), (b"score_fp8", (0, 1), (2,), 0),
                                     (b"shared_key_fp16", (0, 1), (2,), 0), (b"encode_tile_rows", (0, 32, 256), (48,), 0)):
        try:
            for v in good:
                assert lib.palu_set_option(name, v) == 0, (name, v)
            for v in bad:
                assert lib.palu_set_option(name, v) == -1, (name, v)
        finally:
            assert lib.palu_set_option(name, default) == 0
