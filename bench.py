#!/usr/bin/env python3
"""Decode-attention benchmark over a low-rank latent KV-cache on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input,
with everything already resident in HBM: down-project the new token into the
key and value caches (palu_encode x2), quantize the new rows when the cache is
int4 (palu_quant_latent), then one attention decode step (palu_attn_decode:
fold, scores with on-the-fly key reconstruction + RoPE, softmax partials +
P.H_v per split, merge + B_v).  Consecutive steps cycle through a ring of
distinct latent caches larger than the 256 MB last-level cache so that every
step streams its latents from HBM.

Prints ONE JSON line: the step time (metric/value/unit/ms_per_step), the
workload (config), the roofline of the dominant kernel (roofline: algorithmic
FLOPs or bytes per launch over its measured duration, against the MI355X peak),
the same for the value kernel (roofline_value), per-stage times (stage_us) and
the CPU oracle timed beside it (cpu_baseline).
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_F16_PEAK_TFLOPS = 2500.0      # MI355X dense fp16 matrix peak
MFMA_F8_PEAK_TFLOPS = 5000.0       # MI355X dense fp8 matrix peak
HBM_PEAK_GBS = 8000.0              # MI355X HBM3E peak


def log(msg: str) -> None:
    print(msg, file=sys.stderr, flush=True)


def algorithmic_work(layer, batch, seq, k_i4, v_i4, bits=4):
    """FLOPs and HBM bytes the method itself needs per decode step."""
    T = batch * seq
    d_h = layer.d_head
    recon = 0
    pv = 0
    for j in range(layer.n_groups):
        s = layer.group_size(j)
        recon += 2 * T * (layer.k_rank_off[j + 1] - layer.k_rank_off[j]) * s * d_h
        pv += 2 * T * (layer.v_rank_off[j + 1] - layer.v_rank_off[j]) * s * layer.q_per_kv

    def side_bytes(R, i4):
        return T * (R * bits // 8 + (R // layer.quant_block) * 4) if i4 else T * R * 2

    return {
        "score_flops": recon,                               # H_k . B_k reconstruction (the q.K product adds < 1 %)
        "pv_flops": pv,
        "k_latent_bytes": side_bytes(layer.R_k, k_i4),
        "v_latent_bytes": side_bytes(layer.R_v, v_i4),
        "b_bytes": 2 * (layer.b_elems("k") + layer.b_elems("v")),
        "a_bytes": 2 * layer.n_q_heads * d_h * (layer.R_k + layer.R_v),
    }


def prompt_encode(args, P, torch) -> int:
    """Cache fill from a prompt: x [N, d] . (A_k | A_v) -> latents, timed with events around `steps` calls."""
    from workloads import synth
    layer = synth.config_layer(args.config.split("-")[0])
    desc = P.LayerDesc(layer.n_heads, layer.d_head, layer.group_head_off, layer.k_rank_off, layer.v_rank_off,
                       P.PALU_F16, P.PALU_F16, P.PALU_F16, layer.quant_block, layer.rope_theta, layer.q_per_kv)
    n, d = args.prompt_tokens, layer.n_q_heads * layer.d_head
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    x = torch.randn((n, d), generator=g, device="cuda").half()
    Ak = (torch.randn((d, layer.R_k), generator=g, device="cuda") / d ** 0.5).half()
    Av = (torch.randn((d, layer.R_v), generator=g, device="cuda") / d ** 0.5).half()
    hk = torch.empty((n, layer.R_k), dtype=torch.float16, device="cuda")
    hv = torch.empty((n, layer.R_v), dtype=torch.float16, device="cuda")
    ws = torch.empty(max(16, P.palu_encode_workspace_bytes(desc, 2, n)), dtype=torch.uint8, device="cuda")

    def call():
        P.palu_encode_kv(desc, x, Ak, Av, hk, layer.R_k, hv, layer.R_v, None, ws)
    for _ in range(args.warmup):
        call()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(args.steps):
        call()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    flops = 2.0 * n * d * (layer.R_k + layer.R_v)
    ref = x[:64].float() @ Ak.float()
    err = float((hk[:64].float() - ref).abs().max() / ref.abs().max())
    print(json.dumps({"metric": "prompt_encode_tokens_per_s", "value": n / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1,
                      "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
                      "dtype": "f16", "data": "synthetic",
                      "config": {"workload": f"config {args.config} layer, {n}-token prompt, K and V projections"},
                      "roofline": {"bound": "mfma", "achieved": flops / (ms * 1e-3) / 1e12, "peak": 2500.0,
                                   "unit": "TFLOP/s", "frac": flops / (ms * 1e-3) / 2.5e15, "traffic": None},
                      "max_rel_err_vs_fp32_matmul": err}))
    return 0


def multi_query_decode(args, P, torch) -> int:
    """palu_attn_decode_multi: N query tokens per sequence (a speculative-decoding check, a chunk of a prompt)
    over the cache of the chosen configuration; attention only, timed with events around `steps` calls."""
    import numpy as np
    from workloads import device as wd, synth
    cfg = args.config
    layer = synth.config_layer(cfg.split("-")[0])
    batch, seq = synth.FULL_SIZES[cfg]
    n_q = args.query_tokens
    case = wd.make_device_case(cfg, seed=0, dtype="f16", n_sets=2, layer=layer)
    desc = P.LayerDesc(layer.n_heads, layer.d_head, layer.group_head_off, layer.k_rank_off, layer.v_rank_off,
                       P.PALU_F16, P.PALU_F16, P.PALU_F16, layer.quant_block, layer.rope_theta, layer.q_per_kv)
    table = P.palu_rope_table_init(layer.rope_theta, layer.d_head, seq)
    g = torch.Generator(device="cuda")
    g.manual_seed(11)
    q = torch.randn((batch, n_q, layer.n_q_heads, layer.d_head), generator=g, device="cuda").half()
    rows = seq - n_q + 1 + torch.arange(n_q, dtype=torch.int32, device="cuda")          # a causal block over the last n_q rows
    q_len = rows[None].expand(batch, n_q).contiguous()
    q_pos = (q_len - 1).contiguous()
    out = torch.empty((batch, n_q, layer.n_q_heads, layer.d_head), dtype=torch.float32, device="cuda")
    lib = P.load_library()
    import ctypes
    nbytes = ctypes.c_size_t(0)
    if lib.palu_attn_decode_multi_workspace_bytes(desc.ref(), batch, n_q, seq, ctypes.byref(nbytes)) != 0:
        print("unsupported configuration", file=sys.stderr)
        return 2
    ws = torch.empty(int(nbytes.value), dtype=torch.uint8, device="cuda")

    def call(i):
        s = i % 2
        P.palu_attn_decode_multi(desc, batch, n_q, seq, seq, q, q_pos, case.Hk[s], case.Hv[s], case.Bk, case.Bv, table, seq,
                                 q_len=q_len, out=out, workspace=ws)
    for i in range(args.warmup):
        call(i)
    torch.cuda.synchronize()
    kGroup, n_groups = 5, max(20, -(-args.steps // 5))
    gev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_groups)]
    it = 0
    for a, b in gev:
        a.record()
        for _ in range(kGroup):
            call(it)
            it += 1
        b.record()
    torch.cuda.synchronize()
    us = np.array([a.elapsed_time(b) for a, b in gev]) * 1e3 / kGroup
    flops = 2.0 * batch * seq * 128 * sum((layer.k_rank_off[j + 1] - layer.k_rank_off[j]) *
                                          (layer.group_head_off[j + 1] - layer.group_head_off[j]) for j in range(layer.n_groups))
    med = float(np.median(us))
    print(json.dumps({"metric": "decode_attn_multi_us_per_call", "value": med, "unit": "us/call", "n_gpus": 1,
                      "steps": n_groups * kGroup, "warmup": args.warmup, "ms_per_step": med * 1e-3, "higher_is_better": False,
                      "step_us_median": med, "step_us_min": float(np.min(us)), "dtype": "f16", "data": "synthetic",
                      "config": {"workload": f"config {cfg}: {n_q} query tokens per sequence over batch {batch}, seq {seq} "
                                             f"(palu_attn_decode_multi, attention only)"},
                      "us_per_query_token": med / n_q,
                      "roofline": {"bound": "mfma", "note": "key reconstruction FLOPs of ONE pass over the cache (shared by the query tokens)",
                                   "achieved": flops / (med * 1e-6) / 1e12, "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                   "frac": flops / (med * 1e-6) / 1e12 / MFMA_F16_PEAK_TFLOPS, "traffic": None}}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="2", help="workload: 1, 2 (7B shape, seq 16K, headline), 2-4k, 2-64k, 3, 4, 4v, gqa4, 5a, 5b, "
                         "2p / 2p-64k (the paper's latency allocation: K rank 128, V rank 384 per group), "
                         "gqa / gqa-64k (32 query heads on 8 key/value heads, the Llama-3-8B / Mistral-7B shape)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--ring-gib", type=float, default=1.0, help="distinct latent bytes to cycle through")
    ap.add_argument("--opt", action="append", default=[], help="tuning knob name=value (palu_set_option)")
    ap.add_argument("--latent-bits", type=int, default=4, choices=(4, 3, 2),
                    help="config 4 / 4v: bits per quantized latent code (3 and 2: the low-bit settings of the paper's Sec. 4.4)")
    ap.add_argument("--row-major-weights", action="store_true",
                    help="give the step A_k, A_v as [d, R] (palu_decode_step) instead of transposed, [R, d] (palu_decode_step_t)")
    ap.add_argument("--transposed-weights", action="store_true",
                    help="use palu_decode_step_t for any batch below 64 (by default only for batches of one and two)")
    ap.add_argument("--separate-calls", action="store_true",
                    help="time palu_encode_kv + palu_attn_decode instead of the one-call palu_decode_step")
    ap.add_argument("--no-probes", action="store_true", help="skip the bare MFMA / read probes (measured_peaks)")
    ap.add_argument("--no-rope", action="store_true",
                    help="the paper's non-RoPE attention (rope_theta = 0): the query is folded into the latent "
                         "space and the scores come straight from the key latents")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MiB",
                    help="after the timed region also run a plain device copy of this size three times: "
                         "the known-size kernel that scales rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--query-tokens", type=int, default=0, metavar="N",
                    help="time palu_attn_decode_multi with N query tokens per sequence (attention only) instead of the decode step")
    ap.add_argument("--prompt-tokens", type=int, default=0, metavar="N",
                    help="instead of the decode step, time the projection of an N-token prompt into both latent "
                         "caches (palu_encode_kv on its tiled-GEMM path) and print its own JSON line")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2407_21118_amd as P
    from workloads import device as wd

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    P.load_library()
    torch.cuda.set_device(0)
    for kv in args.opt:
        k, v = kv.split("=")
        P.palu_set_option(k, int(v))

    if args.prompt_tokens > 0:
        return prompt_encode(args, P, torch)
    if args.query_tokens > 0:
        return multi_query_decode(args, P, torch)

    cfg = args.config
    v_only = cfg == "4v"
    gqa4 = cfg == "gqa4"                          # the grouped-query layer with quantized key and value latents
    base_cfg = "4" if v_only else ("gqa" if gqa4 else cfg)
    k_i4 = (base_cfg == "4" and not v_only) or gqa4
    v_i4 = base_cfg == "4" or gqa4

    # ---- inputs -----------------------------------------------------------
    t0 = time.time()
    from workloads import synth
    layer = synth.config_layer(base_cfg.split("-")[0])
    if args.no_rope:
        import dataclasses
        layer = dataclasses.replace(layer, rope_theta=0.0)
    batch, seq = synth.FULL_SIZES[base_cfg]
    bits = args.latent_bits
    work = algorithmic_work(layer, batch, seq, k_i4, v_i4, bits)
    set_bytes = batch * seq * (layer.R_k + layer.R_v) * 2
    free_b = torch.cuda.mem_get_info()[0]
    n_sets = max(1, min(int(np.ceil(args.ring_gib * 2 ** 30 / set_bytes)) + 1, int(0.5 * free_b / set_bytes)))
    case = wd.make_device_case(base_cfg, seed=0, dtype="f16", n_sets=n_sets, layer=layer)
    log(f"[bench] config {cfg}: batch {batch} seq {seq} groups {layer.n_groups} R_k {layer.R_k} R_v {layer.R_v}; "
        f"{n_sets} cache sets of {set_bytes / 2**20:.0f} MiB built in {time.time() - t0:.1f}s")

    act = P.PALU_F16
    qdt = {4: P.PALU_I4, 3: P.PALU_I3, 2: P.PALU_I2}[bits]
    desc = P.LayerDesc(layer.n_heads, layer.d_head, layer.group_head_off, layer.k_rank_off, layer.v_rank_off, act,
                       qdt if k_i4 else act, qdt if v_i4 else act, layer.quant_block, layer.rope_theta,
                       layer.q_per_kv)
    table = P.palu_rope_table_init(layer.rope_theta, layer.d_head, seq)
    ws = torch.empty(P.palu_attn_decode_workspace_bytes(desc, batch, seq), dtype=torch.uint8, device="cuda")
    ws_e = torch.empty(P.palu_encode_workspace_bytes(desc, 2, batch), dtype=torch.uint8, device="cuda")
    out = torch.empty((batch, layer.n_q_heads, layer.d_head), dtype=torch.float32, device="cuda")
    dst_row = (torch.arange(batch, dtype=torch.int32, device="cuda") * seq + (seq - 1)).contiguous()
    nbk, nbv = layer.R_k // layer.quant_block, layer.R_v // layer.quant_block

    # int4 caches: quantize every set once with the library's own quantizer
    qk, qv = [], []
    if k_i4 or v_i4:
        for s in range(n_sets):
            for side, flag, H, R, nb, store in ((0, k_i4, case.Hk, layer.R_k, nbk, qk), (1, v_i4, case.Hv, layer.R_v, nbv, qv)):
                if not flag:
                    continue
                codes = torch.empty((batch, seq, R * bits // 8), dtype=torch.uint8, device="cuda")
                sc = torch.empty((batch, seq, nb), dtype=torch.float16, device="cuda")
                zp = torch.empty_like(sc)
                P.palu_quant_latent(desc, side, H[s], R, batch * seq, codes, sc, zp)
                store.append((codes, sc, zp))
        torch.cuda.synchronize()
    # staging rows for the new token when the cache is int4 (encode -> fp16 row -> quantize into the cache)
    new_k = torch.empty((batch, layer.R_k), dtype=torch.float16, device="cuda")
    new_v = torch.empty((batch, layer.R_v), dtype=torch.float16, device="cuda")

    fused = not (k_i4 or v_i4 or args.separate_calls)          # one call per step (append + attend); quantized caches take the separate calls
    # with more than two tokens per step the row-major split-K form is the faster one
    transposed = fused and not args.row_major_weights and (batch <= 2 or (args.transposed_weights and batch < 64))
    if transposed:                                             # the projection weights column by column: made once, like the decomposition
        Akt, Avt = case.Ak.t().contiguous(), case.Av.t().contiguous()

    def step(i: int, events=None, decode_events=None):
        s = i % n_sets
        if transposed and events is None and decode_events is None:
            P.palu_decode_step_t(desc, batch, seq, seq, case.x_new, Akt, Avt, dst_row, case.q, case.q_pos,
                                 case.Hk[s], case.Hv[s], case.Bk, case.Bv, table, seq, out=out, workspace=ws)
            return
        if fused and events is None and decode_events is None:
            P.palu_decode_step(desc, batch, seq, seq, case.x_new, case.Ak, case.Av, dst_row, case.q, case.q_pos,
                               case.Hk[s], case.Hv[s], case.Bk, case.Bv, table, seq, out=out, workspace=ws,
                               encode_workspace=ws_e)
            return
        # down-project the new token into both caches (fp16 row first when the cache is int4)
        k_dst, k_stride, k_rows = (new_k, layer.R_k, None) if k_i4 else (case.Hk[s], layer.R_k, dst_row)
        v_dst, v_stride, v_rows = (new_v, layer.R_v, None) if v_i4 else (case.Hv[s], layer.R_v, dst_row)
        if k_rows is v_rows:
            P.palu_encode_kv(desc, case.x_new, case.Ak, case.Av, k_dst, k_stride, v_dst, v_stride, k_rows, ws_e)
        else:
            P.palu_encode(desc, 0, case.x_new, case.Ak, k_dst, k_stride, k_rows, ws_e)
            P.palu_encode(desc, 1, case.x_new, case.Av, v_dst, v_stride, v_rows, ws_e)
        hk, kq, hv, vq = case.Hk[s], {}, case.Hv[s], {}
        if k_i4:
            codes, sc, zp = qk[s]
            P.palu_quant_latent(desc, 0, new_k, layer.R_k, batch, codes, sc, zp, dst_row)
            hk, kq = codes, dict(hk_scale=sc, hk_zero=zp)
        if v_i4:
            codes, sc, zp = qv[s]
            P.palu_quant_latent(desc, 1, new_v, layer.R_v, batch, codes, sc, zp, dst_row)
            hv, vq = codes, dict(hv_scale=sc, hv_zero=zp)
        if decode_events:
            decode_events[0].record()
        P.palu_attn_decode(desc, batch, seq, seq, case.q, case.q_pos, hk, hv, case.Bk, case.Bv, table, seq,
                           out=out, workspace=ws, stage_events=events, **kq, **vq)
        if decode_events:
            decode_events[1].record()

    # ---- timed region ------------------------------------------------------
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_wall = time.perf_counter()
    ev0.record()
    for i in range(args.steps):
        step(args.warmup + i)
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t_wall) * 1e3
    gpu_ms = ev0.elapsed_time(ev1)
    ms_per_step = max(gpu_ms, 0.0) / args.steps
    log(f"[bench] {args.steps} steps: {gpu_ms:.3f} ms on the stream, {wall_ms:.3f} ms wall")

    # ---- distribution of the step time: the same steps again, bracketed in groups of kGroup (an event between
    # two steps costs marker time the steps do not have back to back; a group spreads it over kGroup steps);
    # median and minimum over at least 100 steps
    kGroup = 5
    n_groups = max(20, -(-args.steps // kGroup))
    gev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_groups)]
    it = args.warmup + args.steps
    # with few warm-up and timed steps the chip is still ramping its clocks here (the first ~100 steps run 3 - 8 % slower):
    # the distribution is taken after at least 200 steps in all
    while it < 200:
        step(it)
        it += 1
    for a, b in gev:
        a.record()
        for _ in range(kGroup):
            step(it)
            it += 1
        b.record()
    torch.cuda.synchronize()
    group_us = np.array([a.elapsed_time(b) for a, b in gev]) * 1e3 / kGroup
    step_us_median, step_us_min = float(np.median(group_us)), float(np.min(group_us))
    log(f"[bench] per step over {n_groups} groups of {kGroup}: median {step_us_median:.2f} us, min {step_us_min:.2f} us, "
        f"mean of the {args.steps} bracketed steps {ms_per_step * 1e3:.2f} us")

    # ---- per-stage durations: same steps again with event hooks between the stages
    n_prof = min(args.steps, 100)
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(P.PALU_DECODE_STAGES + 1)] for _ in range(n_prof)]
    for row in evs:
        for e in row:
            e.record()              # creates the HIP event handles
    torch.cuda.synchronize()
    for i in range(n_prof):
        step(args.warmup + i, evs[i])
    torch.cuda.synchronize()
    stage_ms = np.array([[row[k].elapsed_time(row[k + 1]) for k in range(P.PALU_DECODE_STAGES)] for row in evs])
    names = ["fold", "score", "value", "combine"]
    bracket_us = {n: float(np.mean(stage_ms[:, k]) * 1e3) for k, n in enumerate(names)}
    # An event between two kernels costs marker time that the kernels do not have without it.  Measure it
    # live: the same decode calls with one event pair around the whole call hold one marker gap, the staged
    # ones four, so (sum of stage brackets - whole-call bracket) / 3 is the gap of one interior event.
    dec = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_prof)]
    for i in range(n_prof):
        step(args.warmup + i, None, dec[i])
    torch.cuda.synchronize()
    whole_us = float(np.mean([a.elapsed_time(b) for a, b in dec]) * 1e3)
    gap_us = max(0.0, (sum(bracket_us.values()) - whole_us) / (P.PALU_DECODE_STAGES - 1))
    gap_us = min(gap_us, min(bracket_us.values()))         # no stage is shorter than nothing (a near-empty first stage)
    stage_us = {n: bracket_us[n] - gap_us for n in names}
    stage_us_med = {n: float(np.median(stage_ms[:, k]) * 1e3) - gap_us for k, n in enumerate(names)}
    log(f"[bench] stage brackets us: {bracket_us}; whole decode call {whole_us:.2f} us; marker gap {gap_us:.2f} us")
    log(f"[bench] stage us (bracket - gap): {stage_us}")

    score_tflops = work["score_flops"] / (stage_us["score"] * 1e-6) / 1e12
    k_gbs = work["k_latent_bytes"] / (stage_us["score"] * 1e-6) / 1e9
    v_gbs = work["v_latent_bytes"] / (stage_us["value"] * 1e-6) / 1e9
    total_gbs = (work["k_latent_bytes"] + work["v_latent_bytes"] + work["b_bytes"] + work["a_bytes"]) / (ms_per_step * 1e-3) / 1e9

    result = {
        "metric": "decode_attn_us_per_step",
        "value": step_us_median,
        "value_is": f"median over {n_groups} groups of {kGroup} consecutive steps, each group between two events on the launch stream "
                    f"(ms_per_step: mean over the {args.steps} steps of the bracketed region)",
        "step_us_median": step_us_median,
        "step_us_min": step_us_min,
        "step_us_mean": ms_per_step * 1e3,
        "unit": "us/step",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16" if not (k_i4 or v_i4) else (f"i{bits}+f16" if k_i4 else f"f16 keys, i{bits} values"),
        "data": "synthetic",
        "config": {"workload": f"config {cfg}{' without RoPE' if args.no_rope else ''}: Llama-2-7B-shaped layer decode, batch {batch}, seq {seq}, "
                               f"{layer.n_groups} groups, R_k {layer.R_k}, R_v {layer.R_v}",
                   "batch": batch, "seq_len": seq, "n_heads": layer.n_heads, "q_per_kv": layer.q_per_kv, "group_size": layer.group_size(0),
                   "cache_sets": n_sets,
                   "step": ("palu_decode_step_t: encode K + encode V (transposed weights) + attn_decode in one call" if transposed
                            else "palu_decode_step: encode K + encode V + attn_decode in one call" if fused
                            else "encode K + encode V + quantize + attn_decode")},
        "roofline": {
            "kernel": "score16_kernel / score_kernel (key reconstruction on MFMA + RoPE + q.K in float32)",
            "bound": "mfma", "achieved": score_tflops, "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": score_tflops / MFMA_F16_PEAK_TFLOPS, "traffic": None,
            "launch_us": stage_us["score"], "flops_per_launch": work["score_flops"],
            "latent_read_GBps": k_gbs,
        },
        "roofline_value": {
            "kernel": "pv_kernel (softmax partials + P.H_v on MFMA, one wavefront per sequence split)",
            "bound": "hbm", "achieved": v_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": v_gbs / HBM_PEAK_GBS,
            "traffic": None, "launch_us": stage_us["value"], "bytes_per_launch": work["v_latent_bytes"],
        },
        "stage_us": stage_us,
        "stage_us_median": stage_us_med,
        "stage_us_bracketed": bracket_us,
        "event_gap_us": gap_us,
        "step_GBps_algorithmic": total_gbs,
        "wall_ms_per_step": wall_ms / args.steps,
    }

    # ---- what this GPU sustains on a bare matrix-core loop and a bare streaming read (device probes of the
    # library): the rooflines above use the data-sheet peaks, these give the fractions of measured ceilings
    if not args.no_probes:
        props = torch.cuda.get_device_properties(0)
        sink = torch.zeros(4, dtype=torch.float32, device="cuda")
        pe0, pe1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        best_tf = 0.0
        for _ in range(3):                                   # ~1.3 ms each
            pe0.record()
            fl = P.palu_probe_mfma(10000, sink)
            pe1.record()
            torch.cuda.synchronize()
            best_tf = max(best_tf, fl / (pe0.elapsed_time(pe1) * 1e-3) / 1e12)
        big = torch.empty(2 * 2 ** 30, dtype=torch.uint8, device="cuda").fill_(1)
        best_big = best_small = 0.0
        for _ in range(3):
            pe0.record()
            nb = P.palu_probe_read(big, sink)
            pe1.record()
            torch.cuda.synchronize()
            best_big = max(best_big, nb / (pe0.elapsed_time(pe1) * 1e-3) / 1e9)
        small_b = int(work["v_latent_bytes"])
        for i in range(6):                                   # one launch of the value kernel's size, distinct memory each time
            view = big[(i * small_b) % (big.numel() - small_b):][:small_b]
            pe0.record()
            nb = P.palu_probe_read(view, sink)
            pe1.record()
            torch.cuda.synchronize()
            best_small = max(best_small, nb / (pe0.elapsed_time(pe1) * 1e-3) / 1e9)
        del big
        result["measured_peaks"] = {
            "device": props.name, "compute_units": props.multi_processor_count,
            "mfma_f16_TFLOPs": best_tf, "hbm_read_GBps_2GiB": best_big,
            "hbm_read_GBps_one_launch_of_value_bytes": best_small,
            "note": "best of 3 (6) launches of the library's probe kernels, timed with events on the launch stream",
        }
        result["roofline"]["frac_of_measured"] = (result["roofline"]["achieved"] /
                                                  (best_tf if result["roofline"]["bound"] == "mfma" else best_big))
        result["roofline_value"]["frac_of_measured"] = result["roofline_value"]["achieved"] / best_big
        log(f"[bench] probes: MFMA fp16 {best_tf:.0f} TFLOP/s, read {best_big:.0f} GB/s (2 GiB), "
            f"{best_small:.0f} GB/s (one {small_b / 2**20:.0f} MiB launch)")

    if args.copy_probe > 0:
        src = torch.empty(args.copy_probe * 2 ** 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        log(f"[bench] copy probe: 3 device copies of {args.copy_probe} MiB (reads and writes that many bytes each)")

    if "score_fp8=1" in args.opt and not (k_i4 or args.no_rope):
        # opt-in: keys rebuilt from E4M3-rounded latents and weights on the 8-bit matrix instructions
        result["dtype"] = "e4m3 keys (option score_fp8), f16 values"
        result["roofline"].update(kernel="score8_kernel (8-bit key reconstruction on MFMA + RoPE + q.K in float32)",
                                  peak=MFMA_F8_PEAK_TFLOPS, frac=score_tflops / MFMA_F8_PEAK_TFLOPS)
        result["roofline"].pop("frac_of_measured", None)
    if args.no_rope:        # no reconstruction: the score kernel is a latent-streaming matrix-vector product
        result["roofline"] = {
            "kernel": "qk_kernel (folded query x key latents)", "bound": "hbm", "achieved": k_gbs, "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": k_gbs / HBM_PEAK_GBS, "traffic": None, "launch_us": stage_us["score"],
            "bytes_per_launch": work["k_latent_bytes"],
        }

    # measured HBM traffic per launch of the dominant kernel, from counter runs kept under profiles/
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
            tr = json.load(f).get(cfg + (":no-rope" if args.no_rope else ""))
        if tr and args.latent_bits == 4 and not args.opt:
            result["roofline"]["traffic"] = tr["score_kernel_bytes"]
            result["roofline_value"]["traffic"] = tr["value_kernel_bytes"]
            # not measured in this run: rocprofv3 counter runs of this same command, kept under profiles/
            result["roofline"]["traffic_source"] = result["roofline_value"]["traffic_source"] = tr.get(
                "source", "profiles/hbm_traffic.json")
    except OSError:
        pass

    # ---- CPU baseline: the oracle as it stands, one decode step ------------------
    if not args.no_cpu_baseline:
        from oracle import palu_oracle as O
        try:
            from threadpoolctl import threadpool_info
            threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            threads = len(os.sched_getaffinity(0))
        nb = 1                                          # one sequence of the batch, scaled by batch
        lim = min(seq, 16384)
        Hk = case.Hk[0][:nb, :lim].float().cpu().numpy()
        Hv = case.Hv[0][:nb, :lim].float().cpu().numpy()
        qn = case.q[:nb].float().cpu().numpy()
        Bk = case.Bk.float().cpu().numpy()
        Bv = case.Bv.float().cpu().numpy()
        reps, t_c = 0, time.perf_counter()
        while reps < 20 and (reps == 0 or time.perf_counter() - t_c < 10.0):     # about 10 s of CPU work
            O.attn_decode(qn, np.full((nb,), lim - 1), Hk, Hv, Bk, Bv, layer.group_head_off, layer.k_rank_off,
                          layer.v_rank_off, layer.d_head, layer.rope_theta, None, None, layer.q_per_kv)
            reps += 1
        cpu_s = (time.perf_counter() - t_c) / reps
        scale = (batch / nb) * (seq / lim)
        result["cpu_baseline"] = {
            "value": cpu_s * scale * 1e6, "unit": "us/step", "cores": threads, "kind": "oracle",
            "sample": f"{nb} of {batch} sequences x {lim} of {seq} cached tokens, all heads, attention only "
                      f"(no encode); mean of {reps} runs {cpu_s:.2f} s, scaled x{scale:g}",
            "affinity_cores": len(os.sched_getaffinity(0)),
        }
    print(json.dumps(result, default=lambda o: o.item() if hasattr(o, "item") else str(o)), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
