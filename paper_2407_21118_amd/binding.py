"""ctypes binding of include/palu.h: argument marshalling only.

Functions carry the names of the C entry points.  Tensors are torch tensors
on the GPU; the binding passes their data pointers and the current HIP
stream.  There is no fallback: if the shared library is missing the import of
a symbol raises, and a non-zero status raises PaluError.
"""

from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

PALU_F16, PALU_BF16, PALU_I4, PALU_I3, PALU_I2 = 0, 1, 2, 3, 4
PALU_DECODE_STAGES = 4

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libpalu_hip.so"
_lib = None


class PaluError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        try:
            text = load_library().palu_status_string(status).decode()
        except Exception:
            text = "?"
        super().__init__(f"{where} failed with status {status} ({text})")


class _Desc(ctypes.Structure):
    _fields_ = [
        ("n_heads", ctypes.c_int32), ("d_head", ctypes.c_int32), ("n_groups", ctypes.c_int32),
        ("group_head_off", ctypes.POINTER(ctypes.c_int32)),
        ("k_rank_off", ctypes.POINTER(ctypes.c_int32)),
        ("v_rank_off", ctypes.POINTER(ctypes.c_int32)),
        ("act_dtype", ctypes.c_int32), ("k_latent_dtype", ctypes.c_int32), ("v_latent_dtype", ctypes.c_int32),
        ("quant_block", ctypes.c_int32), ("rope_theta", ctypes.c_float), ("q_per_kv", ctypes.c_int32),
    ]


def lib_path() -> str:
    """Path of the shared library: the in-tree build, or the file named by the
    PALU_LIB environment variable (to try another build of the same ABI)."""
    return os.environ.get("PALU_LIB") or os.path.join(_HERE, _LIB_NAME)


def load_library():
    """Load libpalu_hip.so (built in-tree by paper_2407_21118_amd.build).  torch
    is imported first so that the library binds to the HIP runtime torch uses."""
    global _lib
    if _lib is not None:
        return _lib
    import torch  # noqa: F401  (loads the HIP runtime the streams and tensors belong to)
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2407_21118_amd.build`")
    lib = ctypes.CDLL(path)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    dp = ctypes.POINTER(_Desc)
    szp = ctypes.POINTER(ctypes.c_size_t)
    lib.palu_status_string.restype = ctypes.c_char_p
    lib.palu_status_string.argtypes = [ctypes.c_int]
    lib.palu_version.restype = ctypes.c_int
    lib.palu_version.argtypes = []
    lib.palu_set_option.restype = ctypes.c_int
    lib.palu_set_option.argtypes = [ctypes.c_char_p, ctypes.c_int]
    lib.palu_probe_mfma.argtypes = [i32, vp, vp, ctypes.POINTER(ctypes.c_double)]
    lib.palu_probe_mfma.restype = ctypes.c_int
    lib.palu_probe_read.argtypes = [vp, sz, vp, vp]
    lib.palu_probe_read.restype = ctypes.c_int
    lib.palu_rope_table_bytes.argtypes = [i32, i32, szp]
    lib.palu_rope_table_init.argtypes = [ctypes.c_float, i32, i32, vp, vp]
    lib.palu_encode_workspace_bytes.argtypes = [dp, ctypes.c_int, i32, szp]
    lib.palu_encode.argtypes = [dp, ctypes.c_int, vp, i32, vp, vp, i64, vp, vp, sz, vp]
    lib.palu_encode_kv.argtypes = [dp, vp, i32, vp, vp, vp, i64, vp, i64, vp, vp, sz, vp]
    lib.palu_encode_kv.restype = ctypes.c_int
    lib.palu_quant_latent.argtypes = [dp, ctypes.c_int, vp, i64, i32, vp, vp, vp, vp, vp]
    lib.palu_encode_quant.argtypes = [dp, ctypes.c_int, vp, i32, vp, vp, vp, vp, vp, vp]
    lib.palu_encode_quant.restype = ctypes.c_int
    lib.palu_attn_decode_workspace_bytes.argtypes = [dp, i32, i32, szp]
    lib.palu_attn_decode.argtypes = [dp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                     vp, i32, vp, vp, sz, vp]
    lib.palu_attn_decode_noalloc.argtypes = lib.palu_attn_decode.argtypes[:-3] + [vp]
    lib.palu_attn_decode_noalloc.restype = ctypes.c_int
    lib.palu_attn_decode_staged.argtypes = lib.palu_attn_decode.argtypes + [ctypes.POINTER(vp)]
    lib.palu_attn_decode_staged.restype = ctypes.c_int
    lib.palu_attn_decode_latent.argtypes = [dp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                            vp, i32, vp, vp, sz, vp]
    lib.palu_attn_decode_latent.restype = ctypes.c_int
    lib.palu_attn_decode_multi_workspace_bytes.argtypes = [dp, i32, i32, i32, szp]
    lib.palu_attn_decode_multi_workspace_bytes.restype = ctypes.c_int
    lib.palu_attn_decode_multi.argtypes = [dp, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                           vp, i32, vp, vp, sz, vp]
    lib.palu_attn_decode_multi.restype = ctypes.c_int
    lib.palu_decode_step.argtypes = [dp, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32,
                                     vp, vp, sz, vp]
    lib.palu_decode_step.restype = ctypes.c_int
    lib.palu_encode_kv_t.argtypes = [dp, vp, i32, vp, vp, vp, i64, vp, i64, vp, vp]
    lib.palu_encode_kv_t.restype = ctypes.c_int
    lib.palu_decode_step_t.argtypes = [dp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32,
                                       vp, vp, sz, vp]
    lib.palu_decode_step_t.restype = ctypes.c_int
    for name in ("palu_rope_table_bytes", "palu_rope_table_init", "palu_encode_workspace_bytes", "palu_encode",
                 "palu_quant_latent", "palu_attn_decode_workspace_bytes", "palu_attn_decode"):
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


class LayerDesc:
    """Owns a palu_layer_desc and the host offset arrays it points to."""

    def __init__(self, n_heads: int, d_head: int, group_head_off: Sequence[int], k_rank_off: Sequence[int],
                 v_rank_off: Sequence[int], act_dtype: int = PALU_F16, k_latent_dtype: Optional[int] = None,
                 v_latent_dtype: Optional[int] = None, quant_block: int = 128, rope_theta: float = 10000.0,
                 q_per_kv: int = 1):
        n_groups = len(group_head_off) - 1
        arr = ctypes.c_int32 * (n_groups + 1)
        self._gho = arr(*[int(v) for v in group_head_off])
        self._kro = arr(*[int(v) for v in k_rank_off])
        self._vro = arr(*[int(v) for v in v_rank_off])
        self.n_heads, self.d_head, self.n_groups = int(n_heads), int(d_head), n_groups
        self.group_head_off = [int(v) for v in group_head_off]
        self.k_rank_off = [int(v) for v in k_rank_off]
        self.v_rank_off = [int(v) for v in v_rank_off]
        self.act_dtype = act_dtype
        self.k_latent_dtype = act_dtype if k_latent_dtype is None else k_latent_dtype
        self.v_latent_dtype = act_dtype if v_latent_dtype is None else v_latent_dtype
        self.quant_block = quant_block
        self.rope_theta = float(rope_theta)
        self.q_per_kv = int(q_per_kv)
        self.n_q_heads = self.n_heads * max(self.q_per_kv, 1)
        self.c = _Desc(self.n_heads, self.d_head, n_groups, self._gho, self._kro, self._vro, act_dtype,
                       self.k_latent_dtype, self.v_latent_dtype, quant_block, self.rope_theta, self.q_per_kv)

    @property
    def R_k(self) -> int:
        return self.k_rank_off[-1]

    @property
    def R_v(self) -> int:
        return self.v_rank_off[-1]

    def ref(self):
        return ctypes.byref(self.c)


def _ptr(t) -> Optional[int]:
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check(status: int, where: str) -> None:
    if status != 0:
        raise PaluError(status, where)


def _need_cuda(*tensors) -> None:
    for t in tensors:
        if t is not None and not t.is_cuda:
            raise ValueError("device tensors required")
        if t is not None and not t.is_contiguous():
            raise ValueError("contiguous tensors required")


def palu_status_string(status: int) -> str:
    return load_library().palu_status_string(int(status)).decode()


def palu_version() -> int:
    return int(load_library().palu_version())


def palu_set_option(name: str, value: int) -> None:
    _check(load_library().palu_set_option(name.encode(), int(value)), "palu_set_option")


def palu_rope_table_bytes(d_head: int, n_pos: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load_library().palu_rope_table_bytes(d_head, n_pos, ctypes.byref(out)), "palu_rope_table_bytes")
    return int(out.value)


def palu_rope_table_init(rope_theta: float, d_head: int, n_pos: int, table=None, stream=None):
    """Fills (allocating with torch when `table` is None) and returns the table tensor."""
    import torch
    if table is None:
        table = torch.empty(palu_rope_table_bytes(d_head, n_pos), dtype=torch.uint8, device="cuda")
    _need_cuda(table)
    _check(load_library().palu_rope_table_init(float(rope_theta), d_head, n_pos, _ptr(table), _stream(stream)),
           "palu_rope_table_init")
    return table


def palu_encode_workspace_bytes(desc: LayerDesc, which: int, n_tok: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load_library().palu_encode_workspace_bytes(desc.ref(), which, n_tok, ctypes.byref(out)),
           "palu_encode_workspace_bytes")
    return int(out.value)


def palu_encode(desc: LayerDesc, which: int, x, A, latent, row_stride_elems: int, dst_row=None,
                workspace=None, stream=None):
    import torch
    n_tok = int(x.shape[0])
    if workspace is None:
        workspace = torch.empty(palu_encode_workspace_bytes(desc, which, n_tok), dtype=torch.uint8, device=x.device)
    _need_cuda(x, A, latent, dst_row, workspace)
    _check(load_library().palu_encode(desc.ref(), which, _ptr(x), n_tok, _ptr(A), _ptr(latent),
                                      int(row_stride_elems), _ptr(dst_row), _ptr(workspace),
                                      workspace.numel() * workspace.element_size(), _stream(stream)), "palu_encode")
    return latent


def palu_encode_kv(desc: LayerDesc, x, Ak, Av, hk, hk_row_stride_elems: int, hv, hv_row_stride_elems: int,
                   dst_row=None, workspace=None, stream=None):
    import torch
    n_tok = int(x.shape[0])
    if workspace is None:
        workspace = torch.empty(palu_encode_workspace_bytes(desc, 2, n_tok), dtype=torch.uint8, device=x.device)
    _need_cuda(x, Ak, Av, hk, hv, dst_row, workspace)
    _check(load_library().palu_encode_kv(desc.ref(), _ptr(x), n_tok, _ptr(Ak), _ptr(Av), _ptr(hk),
                                         int(hk_row_stride_elems), _ptr(hv), int(hv_row_stride_elems),
                                         _ptr(dst_row), _ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _stream(stream)),
           "palu_encode_kv")


def palu_quant_latent(desc: LayerDesc, which: int, latent, row_stride_elems: int, n_tok: int,
                      codes, scale, zero, dst_row=None, stream=None):
    _need_cuda(latent, codes, scale, zero, dst_row)
    _check(load_library().palu_quant_latent(desc.ref(), which, _ptr(latent), int(row_stride_elems), int(n_tok),
                                            _ptr(codes), _ptr(scale), _ptr(zero), _ptr(dst_row), _stream(stream)),
           "palu_quant_latent")
    return codes, scale, zero


def palu_encode_quant(desc: LayerDesc, which: int, x, n_tok: int, A, codes, scale, zero, dst_row=None, stream=None):
    _need_cuda(x, A, codes, scale, zero, dst_row)
    _check(load_library().palu_encode_quant(desc.ref(), which, _ptr(x), int(n_tok), _ptr(A), _ptr(codes),
                                            _ptr(scale), _ptr(zero), _ptr(dst_row), _stream(stream)),
           "palu_encode_quant")
    return codes, scale, zero


def palu_attn_decode_workspace_bytes(desc: LayerDesc, batch: int, max_seq: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load_library().palu_attn_decode_workspace_bytes(desc.ref(), batch, max_seq, ctypes.byref(out)),
           "palu_attn_decode_workspace_bytes")
    return int(out.value)


def palu_attn_decode(desc: LayerDesc, batch: int, seq_len: int, max_seq: int, q, q_pos, hk, hv, Bk, Bv,
                     rope_table, rope_table_len: int, out=None, workspace=None, k_pos=None, seq_lens=None,
                     hk_scale=None, hk_zero=None, hv_scale=None, hv_zero=None, stream=None, stage_events=None):
    """stage_events: optional list of PALU_DECODE_STAGES + 1 torch.cuda.Event(enable_timing=True) that were
    already recorded once (so that their HIP handles exist); routes through palu_attn_decode_staged."""
    import torch
    if out is None:
        out = torch.empty((batch, desc.n_q_heads, desc.d_head), dtype=torch.float32, device=q.device)
    if workspace is None:
        workspace = torch.empty(palu_attn_decode_workspace_bytes(desc, batch, max_seq), dtype=torch.uint8,
                                device=q.device)
    _need_cuda(q, q_pos, hk, hv, Bk, Bv, rope_table, out, workspace, k_pos, seq_lens, hk_scale, hk_zero,
               hv_scale, hv_zero)
    args = (desc.ref(), batch, seq_len, max_seq, _ptr(q), _ptr(q_pos), _ptr(hk), _ptr(hk_scale), _ptr(hk_zero),
            _ptr(hv), _ptr(hv_scale), _ptr(hv_zero), _ptr(k_pos), _ptr(seq_lens), _ptr(Bk), _ptr(Bv),
            _ptr(rope_table), int(rope_table_len), _ptr(out), _ptr(workspace),
            workspace.numel() * workspace.element_size(), _stream(stream))
    if stage_events is None:
        _check(load_library().palu_attn_decode(*args), "palu_attn_decode")
    else:
        if len(stage_events) != PALU_DECODE_STAGES + 1:
            raise ValueError("stage_events needs PALU_DECODE_STAGES + 1 events")
        arr = (ctypes.c_void_p * len(stage_events))(*[ctypes.c_void_p(e.cuda_event) for e in stage_events])
        _check(load_library().palu_attn_decode_staged(*args, arr), "palu_attn_decode_staged")
    return out


def palu_attn_decode_noalloc(desc: LayerDesc, batch: int, seq_len: int, max_seq: int, q, q_pos, hk, hv, Bk, Bv,
                             rope_table, rope_table_len: int, out, k_pos=None, seq_lens=None,
                             hk_scale=None, hk_zero=None, hv_scale=None, hv_zero=None, stream=None):
    """palu_attn_decode on the library's static scratch; `out` is the caller's (nothing is allocated here)."""
    _need_cuda(q, q_pos, hk, hv, Bk, Bv, rope_table, out, k_pos, seq_lens, hk_scale, hk_zero, hv_scale, hv_zero)
    _check(load_library().palu_attn_decode_noalloc(
        desc.ref(), batch, seq_len, max_seq, _ptr(q), _ptr(q_pos), _ptr(hk), _ptr(hk_scale), _ptr(hk_zero),
        _ptr(hv), _ptr(hv_scale), _ptr(hv_zero), _ptr(k_pos), _ptr(seq_lens), _ptr(Bk), _ptr(Bv),
        _ptr(rope_table), int(rope_table_len), _ptr(out), _stream(stream)), "palu_attn_decode_noalloc")
    return out


def palu_attn_decode_latent(desc: LayerDesc, batch: int, seq_len: int, max_seq: int, q, q_pos, hk, hv, Bk,
                            rope_table, rope_table_len: int, out_latent=None, workspace=None, k_pos=None,
                            seq_lens=None, hk_scale=None, hk_zero=None, hv_scale=None, hv_zero=None, stream=None):
    """Decode step whose output stays in the value latent space: [batch, sum over heads of r_v(group)] float32."""
    import torch
    if out_latent is None:
        width = sum((desc.v_rank_off[j + 1] - desc.v_rank_off[j]) * (desc.group_head_off[j + 1] - desc.group_head_off[j])
                    for j in range(desc.n_groups)) * max(desc.q_per_kv, 1)
        out_latent = torch.empty((batch, width), dtype=torch.float32, device=q.device)
    if workspace is None:
        workspace = torch.empty(palu_attn_decode_workspace_bytes(desc, batch, max_seq), dtype=torch.uint8,
                                device=q.device)
    _need_cuda(q, q_pos, hk, hv, Bk, rope_table, out_latent, workspace, k_pos, seq_lens, hk_scale, hk_zero,
               hv_scale, hv_zero)
    _check(load_library().palu_attn_decode_latent(
        desc.ref(), batch, seq_len, max_seq, _ptr(q), _ptr(q_pos), _ptr(hk), _ptr(hk_scale), _ptr(hk_zero),
        _ptr(hv), _ptr(hv_scale), _ptr(hv_zero), _ptr(k_pos), _ptr(seq_lens), _ptr(Bk),
        _ptr(rope_table), int(rope_table_len), _ptr(out_latent), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream)), "palu_attn_decode_latent")
    return out_latent


def palu_probe_mfma(iters: int, sink, stream=None) -> float:
    """Launches the bare matrix-core loop; returns the FLOPs of the launch (time it with events)."""
    _need_cuda(sink)
    fl = ctypes.c_double(0.0)
    _check(load_library().palu_probe_mfma(int(iters), _ptr(sink), _stream(stream), ctypes.byref(fl)), "palu_probe_mfma")
    return float(fl.value)


def palu_probe_read(src, sink, stream=None) -> int:
    """Launches the bare streaming read over `src`; returns the bytes read."""
    _need_cuda(src, sink)
    nbytes = (src.numel() * src.element_size()) // 16 * 16
    _check(load_library().palu_probe_read(_ptr(src), nbytes, _ptr(sink), _stream(stream)), "palu_probe_read")
    return nbytes


def palu_attn_decode_multi(desc: LayerDesc, batch: int, n_q: int, seq_len: int, max_seq: int, q, q_pos, hk, hv, Bk, Bv,
                           rope_table, rope_table_len: int, q_len=None, out=None, workspace=None, k_pos=None,
                           seq_lens=None, hk_scale=None, hk_zero=None, hv_scale=None, hv_zero=None, stream=None):
    """n_q queries per sequence: q [batch, n_q, heads, d_head], q_pos and q_len [batch, n_q]."""
    import torch
    lib = load_library()
    if out is None:
        out = torch.empty((batch, n_q, desc.n_q_heads, desc.d_head), dtype=torch.float32, device=q.device)
    if workspace is None:
        nbytes = ctypes.c_size_t(0)
        _check(lib.palu_attn_decode_multi_workspace_bytes(desc.ref(), batch, n_q, max_seq, ctypes.byref(nbytes)),
               "palu_attn_decode_multi_workspace_bytes")
        workspace = torch.empty(int(nbytes.value), dtype=torch.uint8, device=q.device)
    _need_cuda(q, q_pos, q_len, hk, hv, Bk, Bv, rope_table, out, workspace, k_pos, seq_lens, hk_scale, hk_zero,
               hv_scale, hv_zero)
    _check(lib.palu_attn_decode_multi(desc.ref(), batch, n_q, seq_len, max_seq, _ptr(q), _ptr(q_pos), _ptr(q_len),
                                      _ptr(hk), _ptr(hk_scale), _ptr(hk_zero), _ptr(hv), _ptr(hv_scale), _ptr(hv_zero),
                                      _ptr(k_pos), _ptr(seq_lens), _ptr(Bk), _ptr(Bv), _ptr(rope_table),
                                      int(rope_table_len), _ptr(out), _ptr(workspace),
                                      workspace.numel() * workspace.element_size(), _stream(stream)),
           "palu_attn_decode_multi")
    return out


def palu_encode_kv_t(desc: LayerDesc, x, Akt, Avt, hk, hk_row_stride_elems: int, hv, hv_row_stride_elems: int,
                     dst_row=None, stream=None):
    """palu_encode_kv from transposed weights Akt [R_k, d], Avt [R_v, d]; fewer than 64 tokens, no workspace."""
    n_tok = int(x.shape[0])
    _need_cuda(x, Akt, Avt, hk, hv, dst_row)
    _check(load_library().palu_encode_kv_t(desc.ref(), _ptr(x), n_tok, _ptr(Akt), _ptr(Avt), _ptr(hk),
                                           int(hk_row_stride_elems), _ptr(hv),
                                           int(hv_row_stride_elems), _ptr(dst_row), _stream(stream)),
           "palu_encode_kv_t")


def palu_decode_step_t(desc: LayerDesc, batch: int, seq_len: int, max_seq: int, x, Akt, Avt, dst_row, q, q_pos, hk, hv,
                       Bk, Bv, rope_table, rope_table_len: int, out=None, workspace=None, k_pos=None, seq_lens=None,
                       stream=None):
    """palu_decode_step from transposed weights (Akt [R_k, d], Avt [R_v, d])."""
    import torch
    if out is None:
        out = torch.empty((batch, desc.n_q_heads, desc.d_head), dtype=torch.float32, device=q.device)
    if workspace is None:
        workspace = torch.empty(palu_attn_decode_workspace_bytes(desc, batch, max_seq), dtype=torch.uint8,
                                device=q.device)
    _need_cuda(x, Akt, Avt, dst_row, q, q_pos, hk, hv, Bk, Bv, rope_table, out, workspace, k_pos, seq_lens)
    _check(load_library().palu_decode_step_t(
        desc.ref(), batch, seq_len, max_seq, _ptr(x), _ptr(Akt), _ptr(Avt), _ptr(dst_row), _ptr(q), _ptr(q_pos),
        _ptr(hk), _ptr(hv), _ptr(k_pos), _ptr(seq_lens), _ptr(Bk), _ptr(Bv), _ptr(rope_table), int(rope_table_len),
        _ptr(out), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)), "palu_decode_step_t")
    return out


def palu_decode_step(desc: LayerDesc, batch: int, seq_len: int, max_seq: int, x, Ak, Av, dst_row, q, q_pos, hk, hv,
                     Bk, Bv, rope_table, rope_table_len: int, out=None, workspace=None, encode_workspace=None,
                     k_pos=None, seq_lens=None, stream=None):
    """Append the new tokens (x) to both caches and attend, in one call."""
    import torch
    if out is None:
        out = torch.empty((batch, desc.n_q_heads, desc.d_head), dtype=torch.float32, device=q.device)
    if workspace is None:
        workspace = torch.empty(palu_attn_decode_workspace_bytes(desc, batch, max_seq), dtype=torch.uint8,
                                device=q.device)
    if encode_workspace is None:
        encode_workspace = torch.empty(palu_encode_workspace_bytes(desc, 2, batch), dtype=torch.uint8, device=q.device)
    _need_cuda(x, Ak, Av, dst_row, q, q_pos, hk, hv, Bk, Bv, rope_table, out, workspace, encode_workspace, k_pos, seq_lens)
    _check(load_library().palu_decode_step(
        desc.ref(), batch, seq_len, max_seq, _ptr(x), _ptr(Ak), _ptr(Av), _ptr(dst_row), _ptr(encode_workspace),
        encode_workspace.numel() * encode_workspace.element_size(), _ptr(q), _ptr(q_pos), _ptr(hk), _ptr(hv),
        _ptr(k_pos), _ptr(seq_lens), _ptr(Bk), _ptr(Bv), _ptr(rope_table), int(rope_table_len), _ptr(out),
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)), "palu_decode_step")
    return out
