"""Full-size synthetic workloads built on the GPU with torch (input preparation
only: random draws and the library GEMM x . A that fills the cache).

The factor matrices come from workloads.synth (numpy SVDs of seeded random W);
token activations x ~ N(0,1) are drawn with a seeded torch generator on the
device and multiplied by A in float32, rounded once to the cache dtype.  None
of the decode-time arithmetic lives here.
"""

from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch

from . import synth


@dataclass
class DeviceCase:
    """Device-resident inputs of one configuration; `sets` holds several
    statistically identical latent caches so that a benchmark can cycle through
    more bytes than the last-level cache keeps."""
    cfg: str
    layer: synth.Layer
    dtype: str
    batch: int
    seq: int
    q: torch.Tensor                 # [B, n, d_h]
    q_pos: torch.Tensor             # [B] int32
    x_new: torch.Tensor             # [B, d] activation of the token being appended
    Ak: torch.Tensor                # [d, R_k]
    Av: torch.Tensor
    Bk: torch.Tensor                # flat
    Bv: torch.Tensor
    Hk: List[torch.Tensor] = field(default_factory=list)     # each [B, L, R_k]
    Hv: List[torch.Tensor] = field(default_factory=list)
    rotate: bool = False


def _tdtype(name: str):
    return {"f16": torch.float16, "bf16": torch.bfloat16}[name]


def fill_latents(A: torch.Tensor, batch: int, seq: int, seed: int, stream_id: int, dtype,
                 chunk: int = 8192) -> torch.Tensor:
    """[batch, seq, R] latents = round(x . A), x ~ N(0,1) drawn per (seed,
    stream_id) on the device, float32 GEMM."""
    g = torch.Generator(device=A.device)
    g.manual_seed(seed * 1000003 + stream_id)
    R = A.shape[1]
    out = torch.empty((batch, seq, R), dtype=dtype, device=A.device)
    A32 = A.float()
    flat = out.view(batch * seq, R)
    for r0 in range(0, batch * seq, chunk):
        r1 = min(r0 + chunk, batch * seq)
        x = torch.randn((r1 - r0, A.shape[0]), generator=g, device=A.device, dtype=torch.float32).to(dtype)
        flat[r0:r1] = (x.float() @ A32).to(dtype)
    return out


def make_device_case(cfg: str, seed: int = 0, dtype: str = "f16", n_sets: int = 1,
                     batch: Optional[int] = None, seq: Optional[int] = None,
                     layer: Optional[synth.Layer] = None, device: str = "cuda") -> DeviceCase:
    """Configuration `cfg` ("1", "2", "2-4k", "2-64k", "3", "4", "5a", "5b") at
    full size unless batch/seq override it.  Configuration 1 uses the
    orthonormal-B recipe with N(0,1) latents, the others the SVD recipe;
    configuration 4 folds the Hadamard rotation into (A, B)."""
    base = cfg.split("-")[0]
    layer = synth.config_layer(base, seed) if layer is None else layer
    fb, fs = synth.FULL_SIZES[cfg]
    batch = fb if batch is None else batch
    seq = fs if seq is None else seq
    td = _tdtype(dtype)
    d = layer.n_q_heads * layer.d_head
    rotate = base == "4"
    dev = torch.device(device)

    def dv(x):
        return torch.from_numpy(np.ascontiguousarray(x, np.float32)).to(td).to(dev)

    g = torch.Generator(device=dev)
    g.manual_seed(seed * 7919 + 17)
    q = torch.randn((batch, layer.n_q_heads, layer.d_head), generator=g, device=dev, dtype=torch.float32).to(td)
    x_new = torch.randn((batch, d), generator=g, device=dev, dtype=torch.float32).to(td)
    q_pos = torch.full((batch,), seq - 1, dtype=torch.int32, device=dev)
    if base == "1":
        Bk, Bv = dv(synth.make_orthonormal_B(layer, seed, "k")), dv(synth.make_orthonormal_B(layer, seed, "v"))
        rng = np.random.default_rng([seed, 30])
        Ak = dv(rng.standard_normal((d, layer.R_k)) / np.sqrt(d))
        Av = dv(rng.standard_normal((d, layer.R_v)) / np.sqrt(d))
        case = DeviceCase(cfg, layer, dtype, batch, seq, q, q_pos, x_new, Ak, Av, Bk, Bv)
        for s in range(n_sets):
            gs = torch.Generator(device=dev)
            gs.manual_seed(seed * 1000003 + 100 + s)
            case.Hk.append(torch.randn((batch, seq, layer.R_k), generator=gs, device=dev, dtype=torch.float32).to(td))
            case.Hv.append(torch.randn((batch, seq, layer.R_v), generator=gs, device=dev, dtype=torch.float32).to(td))
        return case
    Ak64, Bk64 = synth.make_factors(layer, seed, "k", rotate=rotate)
    Av64, Bv64 = synth.make_factors(layer, seed, "v", rotate=rotate)
    case = DeviceCase(cfg, layer, dtype, batch, seq, q, q_pos, x_new, dv(Ak64), dv(Av64), dv(Bk64), dv(Bv64),
                      rotate=rotate)
    for s in range(n_sets):
        # K and V latents of one cache come from the same token activations x
        case.Hk.append(fill_latents(case.Ak, batch, seq, seed, 2 * s, td))
        case.Hv.append(fill_latents(case.Av, batch, seq, seed, 2 * s, td))
    return case
