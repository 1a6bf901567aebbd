"""Helpers shared by the GPU parity tests: move a workloads.synth.Case to the
device, run the HIP path through the C ABI, run the CPU oracle on the same
bits, and measure the error the way the tolerance is stated."""

from __future__ import annotations

import sys

import numpy as np
import torch

import paper_2407_21118_amd as P
from oracle import palu_oracle as O

TOL_FP = 2e-3      # max |y - y_ref| / max |y_ref|, fp16 / bf16 latents
TOL_I4 = 5e-3      # same with int4 latents (oracle fed the same dequantized values)


def say(msg: str) -> None:
    print(msg, flush=True)
    sys.stdout.flush()


def torch_dtype(name: str):
    return {"f16": torch.float16, "bf16": torch.bfloat16}[name]


def to_dev(x: np.ndarray, dtype: str):
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch_dtype(dtype)).cuda()


def make_desc(layer, dtype: str, k_i4: bool = False, v_i4: bool = False, bits: int = 4) -> "P.LayerDesc":
    """k_i4 / v_i4: the side's latents are quantized, to `bits` bits (4, 3 or 2)."""
    act = P.PALU_F16 if dtype == "f16" else P.PALU_BF16
    qd = {4: P.PALU_I4, 3: P.PALU_I3, 2: P.PALU_I2}[bits]
    return P.LayerDesc(layer.n_heads, layer.d_head, layer.group_head_off, layer.k_rank_off, layer.v_rank_off,
                       act, qd if k_i4 else act, qd if v_i4 else act, layer.quant_block,
                       layer.rope_theta, layer.q_per_kv)


def rel_err(got: np.ndarray, ref: np.ndarray):
    """(whole-tensor, worst per-(batch, head) row) max-abs error over max-abs reference."""
    diff = np.abs(got.astype(np.float64) - ref)
    whole = diff.max() / np.abs(ref).max()
    rows = (diff.max(axis=-1) / np.abs(ref).max(axis=-1)).max()
    return float(whole), float(rows)


def run_hip(case, k_i4=False, v_i4=False, quant=None, rope_len=None, bits=4):
    """HIP path on the case; `quant` = dict(k=(packed, scale, zero), v=(...)) of numpy arrays."""
    layer = case.layer
    desc = make_desc(layer, case.dtype, k_i4, v_i4, bits)
    B, L = case.batch, case.seq
    q = to_dev(case.q, case.dtype)
    q_pos = torch.from_numpy(np.asarray(case.q_pos, np.int32)).cuda()
    Bk, Bv = to_dev(case.Bk, case.dtype), to_dev(case.Bv, case.dtype)
    kw = {}
    if k_i4:
        pk, sk, zk = quant["k"]
        hk = torch.from_numpy(pk).cuda()
        kw["hk_scale"] = torch.from_numpy(sk.view(np.int16)).cuda().view(torch.float16)
        kw["hk_zero"] = torch.from_numpy(zk.view(np.int16)).cuda().view(torch.float16)
    else:
        hk = to_dev(case.Hk, case.dtype)
    if v_i4:
        pv, sv, zv = quant["v"]
        hv = torch.from_numpy(pv).cuda()
        kw["hv_scale"] = torch.from_numpy(sv.view(np.int16)).cuda().view(torch.float16)
        kw["hv_zero"] = torch.from_numpy(zv.view(np.int16)).cuda().view(torch.float16)
    else:
        hv = to_dev(case.Hv, case.dtype)
    if case.k_pos is not None:
        kw["k_pos"] = torch.from_numpy(np.asarray(case.k_pos, np.int32)).cuda()
        n_pos = int(max(np.max(case.k_pos), 0)) + 1
    else:
        n_pos = L
    if case.seq_lens is not None:
        kw["seq_lens"] = torch.from_numpy(np.asarray(case.seq_lens, np.int32)).cuda()
    n_pos = n_pos if rope_len is None else rope_len
    table = P.palu_rope_table_init(layer.rope_theta, layer.d_head, n_pos)
    out = P.palu_attn_decode(desc, B, L, L, q, q_pos, hk, hv, Bk, Bv, table, n_pos, **kw)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def run_oracle(case, quant=None, k_i4=False, v_i4=False, bits=4):
    layer = case.layer
    Hk = O.dequant_latent(*quant["k"], bits=bits) if k_i4 else case.Hk
    Hv = O.dequant_latent(*quant["v"], bits=bits) if v_i4 else case.Hv
    return O.attn_decode(case.q, case.q_pos, Hk, Hv, case.Bk, case.Bv, layer.group_head_off, layer.k_rank_off,
                         layer.v_rank_off, layer.d_head, layer.rope_theta, case.k_pos, case.seq_lens, layer.q_per_kv)
