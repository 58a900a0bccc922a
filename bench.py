#!/usr/bin/env python3
"""Benchmark of the capacity-aware MoE layer forward on one MI355X.

A step is one pass of the whole hot path (route+top-k, capacity drop, dispatch, grouped FFN,
combine: the C-ABI calls back to back on one stream) over one batch of synthetic, skew-routed
input that is already resident in HBM.  The headline workload is the Mixtral-shaped layer (the
largest configuration, the one the matrix cores bind).  Prints ONE JSON line:
  value            tokens/s of the layer with Token Drop at gamma = 1 (N * steps / wall time between
                   two device syncs)
  expanded_drop    the same workload and step count with Expanded Drop (its own value, rooflines,
                   cpu_baseline)
  roofline         the dominant kernel (gate/up GEMM with the SwiGLU epilogue), timed per launch with
                   HIP events the library records around that kernel inside the timed loop;
                   roofline_down: the second GEMM, timed the same way
  cpu_baseline     the CPU oracle on a bounded sample of the same workload, on the host cores
  stages / other_workloads / gamma_sweep / straggler   per-kernel times, the other configurations,
                   the capacity-factor curve and the per-device FFN times of the latency model
"""
import argparse
import hashlib
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0   # dense bf16 matrix peak
FP32_VECTOR_PEAK_TFLOPS = 157.3

# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE per launch, recorded beside the kernel source they were measured on
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_of_the_expert_gemms.md")
# the expert GEMMs, their tile schedule and the constants both share
KERNEL_SOURCES = [os.path.join(ROOT, "paper_2503_05066_amd", "csrc", f) for f in ("ffn.hip", "schedule.h", "common.h")]


def kernel_source_version():
    """First 12 hex digits of the SHA-1 over the sources that decide how the expert GEMMs run."""
    h = hashlib.sha1()
    for path in KERNEL_SOURCES:
        h.update(open(path, "rb").read())
    return h.hexdigest()[:12]

MODES = {"none": 0, "token": 1, "expanded": 2}
SCOPES = {"local": 0, "global": 1, "local_device": 2, "global_device": 3}
METRICS = {"score": 0, "order": 1, "reverse_order": 2, "random": 3}


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=200)
    p.add_argument("--warmup", type=int, default=20)
    p.add_argument("--workload", default="mixtral", help="tiny | olmoe | mixtral | finegrained | decode")
    p.add_argument("--mode", default="token", choices=list(MODES))
    p.add_argument("--scope", default="local", choices=list(SCOPES))
    p.add_argument("--gamma", type=float, default=1.0)
    p.add_argument("--metric", default="score", choices=list(METRICS), help="what ranks the tokens of a full expert")
    p.add_argument("--overselect", type=int, default=0, help="m: candidate lists are top-(k+m) instead of top-k")
    p.add_argument("--max-experts", action="store_true", help="at most k surviving experts per token (w/ max)")
    p.add_argument("--tokens", type=int, default=0, help="override the workload's token count (batch x length sweeps)")
    p.add_argument("--sweep-gamma", default="0.5,1.0,1.5,2.0,inf",
                   help="comma list of capacity factors measured after the main line ('' for none)")
    p.add_argument("--no-expanded", action="store_true", help="skip the Expanded Drop line of the same workload")
    p.add_argument("--no-straggler", action="store_true",
                   help="skip the per-device FFN timing (the one-GPU stand-in for the latency model of Eq. 4)")
    p.add_argument("--no-peaks", action="store_true", help="skip the measured-ceiling probes (MFMA loop, device copy)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--unfused", action="store_true",
                   help="the five separate calls (with moe_dispatch and moe_grouped_ffn) instead of moe_layer_forward")
    p.add_argument("--calibration-copy", action="store_true",
                   help="also run a plain 1 GiB device copy (the known-size kernel that scales FETCH_SIZE/WRITE_SIZE)")
    p.add_argument("--ffn-uniform", default="mixtral",
                   help="comma list of workloads whose expert FFN is also timed alone on experts of equal size "
                        "(N*k/E rows each, no router, no drop) with the vendor library's dense GEMM of the same "
                        "dimensions beside it ('' for none; skipped with --no-peaks)")
    p.add_argument("--others", default="mixtral:none,mixtral:token:local_device,olmoe:token,olmoe:none,"
                                       "finegrained:expanded,finegrained:token,finegrained:none,decode:token,"
                                       "decode:expanded,decode:none",
                   help="comma list of workload:mode[:scope] measured after the main line ('' for none)")
    return p.parse_args()


_uploaded = {}
_host_weights = {}


def upload(w, keep_host=False):
    """Synthetic inputs of a workload as device tensors (storage type of the workload).

    The last workload stays resident, so that several modes of one workload share one upload.  keep_host: also
    keep the fp32-valued host copies of the expert weights (the CPU baseline reads them)."""
    import numpy as np
    import torch

    key = (w.name, w.n_tokens)
    if key in _uploaded:
        return _uploaded[key]
    _uploaded.clear()
    _host_weights.clear()
    torch.cuda.empty_cache()

    from paper_2503_05066_amd import synth

    def dev(st):
        if st.bits is not None:
            return torch.from_numpy(st.bits.view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(st.f32).cuda()

    act = torch.bfloat16 if w.dtype == synth.DTYPE_BF16 else torch.float32
    e, h, d = w.n_experts, w.d_hidden, w.d_model
    t = {"x": dev(synth.tokens(w)), "w_router": torch.from_numpy(synth.router_weight(w)).cuda(),
         "bias": torch.from_numpy(synth.router_bias(w)).cuda(),
         "w_gate": torch.empty((e, h, d), dtype=act, device="cuda"),
         "w_up": torch.empty((e, h, d), dtype=act, device="cuda"),
         "w_down": torch.empty((e, d, h), dtype=act, device="cuda")}
    # every expert has a random stream of its own: draw them on a few host threads, copy from this one
    with ThreadPoolExecutor(max_workers=min(8, e)) as ex:
        for j, (g, u, dn) in enumerate(ex.map(lambda j: synth.expert_weights(w, j, keep_f32=keep_host), range(e))):
            t["w_gate"][j].copy_(dev(g))
            t["w_up"][j].copy_(dev(u))
            t["w_down"][j].copy_(dev(dn))
            if keep_host:
                _host_weights[j] = (g.f32, u.f32, dn.f32)
    _uploaded[key] = t
    return t


def algorithmic_work(w, S, rows, active, elem):
    """Bytes each kernel must move and flops it must do for `rows` surviving pairs: inputs read once, outputs written once."""
    n, d, e, k, h = w.n_tokens, w.d_model, w.n_experts, w.top_k, w.d_hidden
    m = S - k
    return {
        "router_logits": {"bytes": n * d * elem + e * d * 4 + n * e * 4, "flops": 2 * n * d * e},
        "softmax_topk": {"bytes": 2 * n * e * 4 + n * k * 8, "flops": 0},
        "drop": {"bytes": n * k * 8 + n * m * 4 + rows * 8 + n * S * 4, "flops": 0},
        "dispatch": {"bytes": 2 * rows * d * elem, "flops": 0},
        "ffn_gate_up": {"bytes": active * 2 * h * d * elem + rows * (d + h) * elem, "flops": 4 * d * h * rows},
        "ffn_down": {"bytes": active * h * d * elem + rows * (d + h) * elem, "flops": 2 * d * h * rows},
        "combine": {"bytes": rows * d * elem + n * d * elem, "flops": 0},
    }


def event_pairs(n):
    import torch

    return [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]


def load_statistics(w, buf, gamma, mode):
    """The paper's load statistics of one plan: loads before and after the drop (Sec. 3.1 and Sec. 4), the dropped
    share, and Eq. (11) evaluated on the loads before the drop with the per-expert capacity gamma * N_bar."""
    import numpy as np

    counts = buf.expert_count.cpu().numpy()
    rows = int(buf.expert_offset[-1])
    nbar = w.n_tokens * w.top_k / w.n_experts
    before = np.bincount(buf.topk_idx[:, :w.top_k].cpu().numpy().ravel(), minlength=w.n_experts)
    g = w.device_groups
    dev_before = before.reshape(g, -1).sum(1)
    dev_after = counts.reshape(g, -1).sum(1)
    loads = {"max_expert_load_over_mean_topk": float(before.max() / nbar),
             "max_expert_load_over_mean_kept": float(counts.max() / nbar),
             "max_device_load_over_mean_topk": float(dev_before.max() / dev_before.mean()),
             "max_device_load_over_mean_kept": float(dev_after.max() / max(dev_after.mean(), 1e-9))}
    per_token = (buf.pair_row >= 0).sum(1)
    dt_eq11 = float(np.maximum(before - gamma * nbar, 0.0).sum() / before.sum()) if mode != 0 else 0.0
    return {"rows": rows, "active_experts": int((counts > 0).sum()), "dropped_ratio": 1.0 - rows / (w.n_tokens * w.top_k),
            "dt_eq11": dt_eq11, "experts_per_token_mean": rows / max(w.n_tokens, 1),
            "experts_per_token_max": int(per_token.max()), "tokens_without_expert": int((per_token == 0).sum()),
            "max_load_over_mean": float(counts.max() / nbar), "max_segment_load": int(buf.seg_count.max()),
            "kept_fraction": rows / (w.n_tokens * w.top_k), "loads": {k: round(v, 3) for k, v in loads.items()}}


def measure(w, mode, scope, gamma, steps, warmup, fused=True, metric=0, overselect=0, max_experts=0, per_kernel=True,
            keep_host=False):
    import torch

    from paper_2503_05066_amd import capmoe, synth

    t = upload(w, keep_host)
    desc = capmoe.make_desc(w.n_tokens, w.d_model, w.n_experts, w.top_k, w.d_hidden, w.device_groups, mode, scope,
                            gamma, w.dtype, metric, overselect, max_experts)
    buf = capmoe.LayerBuffers(desc)
    K_GU, K_DN = capmoe.KERNELS.index("ffn_gate_up"), capmoe.KERNELS.index("ffn_down")

    def step():
        if fused:   # the whole layer through the one-call entry point
            capmoe.moe_layer_forward(desc, t["x"], t["w_router"], t["bias"], t["w_gate"], t["w_up"], t["w_down"], None, 0,
                                     buf)
        else:       # the five separate calls
            capmoe.layer_forward(buf, t["x"], t["w_router"], t["bias"], t["w_gate"], t["w_up"], t["w_down"],
                                 fused_dispatch=False)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    gu, dn = event_pairs(steps), event_pairs(steps)
    tab = capmoe.MoeProfile()
    for a, b in gu + dn:      # materialise the events before the timed region
        tab.set_events(K_GU, a, b)
    torch.cuda.synchronize()
    capmoe.moe_profile_attach(tab)
    t0 = time.perf_counter()
    for i in range(steps):
        tab.set_events(K_GU, *gu[i])
        tab.set_events(K_DN, *dn[i])
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    capmoe.moe_profile_attach(None)
    launched = {capmoe.KERNELS[k]: int(tab.launches[k]) for k in range(len(capmoe.KERNELS))}
    gu_ms = sum(a.elapsed_time(b) for a, b in gu) / steps if launched["ffn_gate_up"] else None
    dn_ms = sum(a.elapsed_time(b) for a, b in dn) / steps if launched["ffn_down"] else None

    # per-step durations (event pairs around whole steps), outside the timed region
    pairs = event_pairs(steps)
    for a, b in pairs:
        a.record()
        step()
        b.record()
    torch.cuda.synchronize()
    step_ms = sorted(a.elapsed_time(b) for a, b in pairs)

    # per-kernel durations: every kernel's event pair in one table, a few steps, outside the timed region.
    # A kernel id the call sequence never launched (the library counts launches) reports None.
    kernel_ms = {name: None for name in capmoe.KERNELS}
    if per_kernel:
        reps = max(5, min(steps, 20))
        evs = {k: event_pairs(reps) for k in range(len(capmoe.KERNELS))}
        tab = capmoe.MoeProfile()
        for k, prs in evs.items():
            for a, b in prs:
                tab.set_events(k, a, b)
        torch.cuda.synchronize()
        capmoe.moe_profile_attach(tab)
        for i in range(reps):
            for k, prs in evs.items():
                tab.set_events(k, *prs[i])
            step()
        torch.cuda.synchronize()
        capmoe.moe_profile_attach(None)
        for k, name in enumerate(capmoe.KERNELS):
            if tab.launches[k] > 0:
                kernel_ms[name] = sum(a.elapsed_time(b) for a, b in evs[k]) / reps

    stats = load_statistics(w, buf, gamma, mode)
    elem = 2 if w.dtype == synth.DTYPE_BF16 else 4
    work = algorithmic_work(w, buf.slots, stats["rows"], stats["active_experts"], elem)
    if fused:   # the permuted copy is never written: the first GEMM reads x through row_token
        work["dispatch"]["bytes"] = 0
    res = dict(stats)
    res.update({
        "step_ms_median": step_ms[len(step_ms) // 2], "step_ms_min": step_ms[0],
        "wall_s": wall, "ms_per_step": 1e3 * wall / steps, "tokens_per_s": w.n_tokens * steps / wall,
        "gate_up_ms": gu_ms, "down_ms": dn_ms, "kernel_ms": kernel_ms, "launches_in_timed_loop": launched,
        "cap": buf.cap, "max_rows": buf.max_rows, "work": work,
    })
    del buf
    return res


def device_slices(w, buf, t):
    """One simulated device's share of a plan as a layer call of its own: for every device the descriptor (its
    E/G experts, any of the N tokens may hold a row at each), the row range of the plan and the arguments of
    moe_dispatch_ffn without the workspace.  Yields (device, r0, r1, desc, args)."""
    from paper_2503_05066_amd import capmoe, synth

    g, e = w.device_groups, w.n_experts
    m = e // g
    offs = buf.expert_offset.cpu().numpy()
    sub = capmoe.make_desc(w.n_tokens, w.d_model, m, m, w.d_hidden, 1, synth.MODE_NONE, synth.SCOPE_GLOBAL, 1.0,
                           w.dtype)
    for dev in range(g):
        r0, r1 = int(offs[dev * m]), int(offs[(dev + 1) * m])
        local_offset = (buf.expert_offset[dev * m:(dev + 1) * m + 1] - r0).contiguous()   # the device's own row numbering
        args = (sub, t["x"], local_offset, buf.row_token[r0:], t["w_gate"][dev * m:(dev + 1) * m],
                t["w_up"][dev * m:(dev + 1) * m], t["w_down"][dev * m:(dev + 1) * m], buf.yp[r0:])
        yield dev, r0, r1, sub, args


def per_device_ffn(w, mode, scope, gamma, reps=5, overselect=0, max_experts=0):
    """Expert computation of every simulated device on its own: the device's E/G experts over the rows the
    plan gives them, timed as separate launches of the layer's FFN.  In the paper's latency model
    (Eq. 4) all devices wait for the slowest one, so max / mean of these times is the straggler effect
    this plan would cause, and the maximum is what the drop shortens."""
    import torch

    from paper_2503_05066_amd import capmoe

    t = upload(w)
    desc = capmoe.make_desc(w.n_tokens, w.d_model, w.n_experts, w.top_k, w.d_hidden, w.device_groups, mode, scope,
                            gamma, w.dtype, 0, overselect, max_experts)
    buf = capmoe.LayerBuffers(desc)
    capmoe.layer_forward(buf, t["x"], t["w_router"], t["bias"], t["w_gate"], t["w_up"], t["w_down"],
                         fused_dispatch=True)
    torch.cuda.synchronize()
    ws = None
    rows, ms = [], []
    for dev, r0, r1, sub, args in device_slices(w, buf, t):
        if ws is None:
            ws = torch.empty(max(capmoe.moe_query(sub)[3], 256), dtype=torch.uint8, device="cuda")
        rows.append(r1 - r0)
        if r1 == r0:
            ms.append(0.0)
            continue
        for _ in range(2):
            capmoe.moe_dispatch_ffn(*args, ws)
        evs = event_pairs(reps)
        for a, b in evs:
            a.record()
            capmoe.moe_dispatch_ffn(*args, ws)
            b.record()
        torch.cuda.synchronize()
        ms.append(sorted(a.elapsed_time(b) for a, b in evs)[reps // 2])
    del buf, ws
    mean_ms = sum(ms) / len(ms)
    return {"per_device_rows": rows, "per_device_ffn_ms": [round(v, 4) for v in ms], "max_ms": round(max(ms), 4),
            "mean_ms": round(mean_ms, 4), "max_over_mean_ms": round(max(ms) / max(mean_ms, 1e-9), 3),
            "max_over_mean_rows": round(max(rows) / max(sum(rows) / len(rows), 1e-9), 3)}


def straggler(w, mode, scope, gamma, overselect=0, max_experts=0):
    from paper_2503_05066_amd import synth

    base = per_device_ffn(w, synth.MODE_NONE, synth.SCOPE_LOCAL, 1.0)
    drop = per_device_ffn(w, mode, scope, gamma, overselect=overselect, max_experts=max_experts)
    return {"note": "expert FFN of each simulated device timed alone; Eq. 4: the slowest device sets the layer's pace",
            "no_drop": base, "with_drop": drop,
            "slowest_device_speedup": round(base["max_ms"] / max(drop["max_ms"], 1e-9), 3)}


def measured_peaks():
    """What this chip sustains: a register-only MFMA loop and a plain device copy (denominators beside the
    published peaks)."""
    import torch

    from paper_2503_05066_amd import capmoe

    sink = torch.empty(2048 * 256, dtype=torch.float32, device="cuda")
    loop = {}
    for random_operands in (False, True):
        best = 0.0
        for _ in range(3):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            flops = capmoe.moe_probe_mfma_bf16(2048, 4096, sink, random_operands)
            b.record()
            torch.cuda.synchronize()
            best = max(best, flops / (a.elapsed_time(b) * 1e-3) / 1e12)
        loop[random_operands] = best
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    copy = 0.0
    for _ in range(4):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        dst.copy_(src)
        b.record()
        torch.cuda.synchronize()
        copy = max(copy, 2 * (1 << 30) / (a.elapsed_time(b) * 1e-3) / 1e9)
    del src, dst
    torch.cuda.empty_cache()
    return {"mfma_bf16_TFLOPs": round(loop[False], 1), "mfma_bf16_random_operands_TFLOPs": round(loop[True], 1),
            "copy_GBs": round(copy, 1),
            "how": "best of 3 launches of 2048 blocks x 4 waves x 4096 x 64 register-only MFMAs (the big GEMM tile's "
                   "k-step), operands of zeros and ones / random bf16 values in (-2, 2): the clock under the loop depends "
                   "on the switching operand bits; best of 4 1 GiB device copies (read + written bytes)"}


def ffn_uniform(w, reps=9, experts=None, vendor=True):
    """The grouped FFN alone on experts of equal size (N*k/E rows each): what the two GEMM kernels sustain when no
    tile is ragged, and torch.matmul (the vendor library) on one dense GEMM of the same M, N, K for comparison.
    experts=1: all N*k rows on the first expert, i.e. the same kernels with the weight traffic of a dense GEMM
    (one weight matrix, re-read from the memory-side cache instead of streamed from HBM)."""
    import torch

    from paper_2503_05066_amd import capmoe

    e, d, h = experts or w.n_experts, w.d_model, w.d_hidden
    m = max(1, w.n_tokens * w.top_k // e)
    rows = m * e
    t = upload(w)
    desc = capmoe.make_desc(rows, d, e, 1, h, 1, MODES["none"], SCOPES["local"], 1.0, w.dtype)
    _, _, max_rows, wsb = capmoe.moe_query(desc)
    assert max_rows == rows
    gen = torch.Generator(device="cuda").manual_seed(1)
    xp = torch.randn(rows, d, device="cuda", generator=gen).to(torch.bfloat16)
    off = torch.arange(0, rows + 1, m, dtype=torch.int32, device="cuda")
    yp = torch.empty(rows, d, dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(max(wsb, 256), dtype=torch.uint8, device="cuda")

    def run():
        capmoe.moe_grouped_ffn(desc, xp, off, t["w_gate"][:e], t["w_up"][:e], t["w_down"][:e], yp, ws)

    for _ in range(2):
        run()
    torch.cuda.synchronize()
    out = {"workload": w.name, "experts": e, "rows_per_expert": m, "d": d, "h": h}
    kids = {name: capmoe.KERNELS.index(name) for name in ("ffn_gate_up", "ffn_down")}
    evs = {name: event_pairs(reps) for name in kids}
    tab = capmoe.MoeProfile()
    for name, prs in evs.items():
        for s0, s1 in prs:
            tab.set_events(kids[name], s0, s1)
    torch.cuda.synchronize()
    capmoe.moe_profile_attach(tab)
    for i in range(reps):
        for name, prs in evs.items():
            tab.set_events(kids[name], *prs[i])
        run()
    torch.cuda.synchronize()
    capmoe.moe_profile_attach(None)
    for name, flops in (("ffn_gate_up", 4 * d * h * rows), ("ffn_down", 2 * d * h * rows)):
        ms = sorted(s0.elapsed_time(s1) for s0, s1 in evs[name])[reps // 2]
        out[name] = {"ms": round(ms, 4), "TFLOP/s": round(flops / ms / 1e9, 1),
                     "frac_of_peak": round(flops / ms / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4)}
    # the same dimensions as one dense NT GEMM each, through the vendor library
    for name, (mm, nn, kk) in (("vendor_dense_gate_up", (rows, 2 * h, d)), ("vendor_dense_down", (rows, d, h))) if vendor else ():
        a_ = torch.randn(mm, kk, device="cuda", generator=gen).to(torch.bfloat16)
        b_ = torch.randn(nn, kk, device="cuda", generator=gen).to(torch.bfloat16)
        for _ in range(2):
            c_ = a_ @ b_.T
        prs = event_pairs(reps)
        for s0, s1 in prs:
            s0.record()
            c_ = a_ @ b_.T
            s1.record()
        torch.cuda.synchronize()
        ms = sorted(s0.elapsed_time(s1) for s0, s1 in prs)[reps // 2]
        out[name] = {"ms": round(ms, 4), "TFLOP/s": round(2 * mm * nn * kk / ms / 1e9, 1)}
        del a_, b_, c_
    if vendor:
        out["note"] = ("vendor_dense_*: torch.matmul on ONE dense NT GEMM with the same M, N, K (a single weight matrix, "
                       "so E times less weight traffic than the grouped GEMM: compare it with the experts=1 entry)")
    return out


def roofline_of(work, ms):
    """The binding roof of a kernel: the larger of its MFMA time and its HBM time at peak."""
    t_mfma = work["flops"] / (MFMA_BF16_PEAK_TFLOPS * 1e12)
    t_hbm = work["bytes"] / (HBM_PEAK_GBS * 1e9)
    sec = ms * 1e-3
    mfma = {"bound": "mfma", "achieved": work["flops"] / sec / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s"}
    hbm = {"bound": "hbm", "achieved": work["bytes"] / sec / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    for r in (mfma, hbm):
        r["frac"] = r["achieved"] / r["peak"]
        r["traffic"] = None
    return (mfma, hbm) if t_mfma >= t_hbm else (hbm, mfma)


def recorded_traffic(workload, mode, scope, gamma, kernel):
    """HBM bytes per launch of one of the expert GEMMs from the tracked table of rocprofv3 --pmc runs
    (FETCH_SIZE + WRITE_SIZE, each scaled by a plain device copy), or None.

    The table names the kernel source it was measured on (first 12 hex digits of the SHA-1 of ffn.hip): a row
    recorded for another version of the kernel is not reported."""
    try:
        text = open(TRAFFIC_TABLE).read()
        sha = kernel_source_version()
    except OSError:
        return None
    for line in text.splitlines():
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) >= 8 and cells[:5] == [workload, mode, scope, f"{gamma:g}", kernel] and cells[7] == sha:
            return float(cells[5]) + float(cells[6])
    return None


def cpu_baseline(w, mode, scope, gamma, budget_s=4.0):
    """The oracle, as it stands, on the host cores: routing on the full batch, FFN on a token sample."""
    import numpy as np

    from oracle import oracle
    from paper_2503_05066_amd import synth

    x = synth.tokens(w).f32
    wr, b = synth.router_weight(w), synth.router_bias(w)
    t0 = time.perf_counter()
    logits = oracle.router_logits(x, wr, b)
    ref = oracle.route_and_drop(logits, w.top_k, w.device_groups, mode, scope, gamma)
    t_route = time.perf_counter() - t0
    rng = np.random.default_rng(1)
    # grow the sample until the FFN leg takes a few seconds
    sample = 16
    weights = dict(_host_weights) if (w.name, w.n_tokens) in _uploaded else {}
    while True:
        toks = np.sort(rng.choice(w.n_tokens, size=min(sample, w.n_tokens), replace=False)).astype(np.int32)
        need = np.flatnonzero(ref.keep[toks].sum(0))
        for j in need:
            if j not in weights:
                weights[j] = tuple(s.f32 for s in synth.expert_weights(w, int(j)))
        tabs = [[weights[j][i] if j in weights else None for j in range(w.n_experts)] for i in range(3)]
        t0 = time.perf_counter()
        oracle.layer_output(x, ref.scores, ref.keep, tabs[0], tabs[1], tabs[2], token_list=toks)
        t_ffn = time.perf_counter() - t0
        if t_ffn > budget_s or len(toks) >= w.n_tokens or sample >= 4096:
            break
        sample *= 4
    n_s = len(toks)
    est = t_route * n_s / w.n_tokens + t_ffn   # seconds for n_s tokens
    # the same on one thread, on a sixteenth of the sample
    threads = oracle.num_threads()
    one = toks[:max(1, n_s // 16)]
    oracle.set_num_threads(1)
    t0 = time.perf_counter()
    oracle.layer_output(x, ref.scores, ref.keep, tabs[0], tabs[1], tabs[2], token_list=one)
    t_one = time.perf_counter() - t0
    oracle.set_num_threads(threads)
    # (routing and drop are serial except for the logits; their share is small either way)
    single = len(one) / (t_route * len(one) / w.n_tokens + t_one)
    return {"value": n_s / est, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "single_thread_tokens_per_s": round(single, 1),
            "sample": f"extrapolated from a subset: routing+drop on all {w.n_tokens} tokens ({t_route:.2f} s, prorated), "
                      f"expert FFN+combine on {n_s} sampled tokens ({t_ffn:.2f} s); single thread: FFN+combine on "
                      f"{len(one)} of them ({t_one:.2f} s)"}


def rounded(d):
    return {k: (round(v, 4) if isinstance(v, float) else v) for k, v in d.items()}


def line_of(w, a, mode_name, scope_name, r):
    """The reported objects of one measured (workload, mode): rooflines of both GEMMs, stages, statistics."""
    out = {}
    for key, kernel, ms, label in (("roofline", "ffn_gate_up", r["gate_up_ms"],
                                    "ffn_gemm_bf16_kernel<..., SWIGLU> (gate/up GEMM + SwiGLU epilogue)"),
                                   ("roofline_down", "ffn_down", r["down_ms"], "ffn_gemm_bf16_kernel<...> (down GEMM)")):
        if ms is None:
            out[key] = None
            continue
        primary, other = roofline_of(r["work"][kernel], ms)
        plain = not (a.tokens or a.overselect or a.max_experts or a.metric != "score" or a.unfused)
        tr = recorded_traffic(w.name, mode_name, scope_name, a.gamma, kernel) if plain else None
        primary["traffic"] = other["traffic"] = tr
        primary["traffic_source"] = (os.path.relpath(TRAFFIC_TABLE, ROOT) + " (rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE "
                                     "of this command, recorded for this version of the kernel source)") if tr else \
            "none recorded for this command and this version of the kernel source"
        primary["kernel"] = label
        primary["ms_per_launch"] = round(ms, 5)
        primary["other_roof"] = {k: other[k] for k in ("bound", "achieved", "peak", "unit", "frac")}
        out[key] = primary
    stages = {}
    km = r["kernel_ms"]
    drop_ids = [k for k in ("drop_prepare", "drop_select", "drop_emit", "drop_limit") if km[k] is not None]
    merged = dict(km)
    merged["drop"] = sum(km[k] for k in drop_ids) if drop_ids else None
    for name in ("router_logits", "softmax_topk", "drop", "dispatch", "ffn_schedule", "ffn_gate_up", "ffn_down", "combine"):
        ms = merged[name]
        if ms is None:
            note = {"dispatch": "fused into ffn_gate_up",
                    "ffn_schedule": "no launch of its own: built by the last launch of the drop"}.get(name, "not launched")
            stages[name] = {"ms": None, "note": note}
            continue
        stages[name] = {"ms": round(ms, 4)}
        wk = r["work"].get(name)
        if wk:
            stages[name].update({"GB/s": round(wk["bytes"] / ms / 1e6, 1),
                                 "hbm_frac": round(wk["bytes"] / ms / 1e6 / HBM_PEAK_GBS, 4)})
            if wk["flops"]:
                stages[name]["TFLOP/s"] = round(wk["flops"] / ms / 1e9, 2)
        if name == "drop":
            stages[name]["kernels"] = drop_ids
    out["stages"] = stages
    out["kernel_ms"] = {k: (round(v, 4) if v is not None else None) for k, v in km.items()}
    out["step_ms_median"] = round(r["step_ms_median"], 4)
    out["step_ms_min"] = round(r["step_ms_min"], 4)
    out["config"] = {
        "workload": f"{w.name}: N={w.n_tokens} d={w.d_model} E={w.n_experts} k={w.top_k} h={w.d_hidden} "
                    f"G={w.device_groups}, {mode_name} drop, gamma={a.gamma}, {scope_name} capacity, {a.metric} metric"
                    + (f", top-(k+{a.overselect}) candidates" if a.overselect else "")
                    + (", at most k experts per token" if a.max_experts else ""),
        "cap": r["cap"], "surviving_pairs": r["rows"], "kept_fraction": round(r["kept_fraction"], 4),
        "active_experts": r["active_experts"], "max_segment_load": r["max_segment_load"],
        "max_load_over_mean_after_drop": round(r["max_load_over_mean"], 3), "loads": r["loads"],
        "dropped_ratio": round(r["dropped_ratio"], 4), "DT_eq11": round(r["dt_eq11"], 4),
        "experts_per_token_mean": round(r["experts_per_token_mean"], 3),
        "experts_per_token_max": r["experts_per_token_max"], "tokens_without_expert": r["tokens_without_expert"],
        "calls": "route_topk, capacity_drop, dispatch, grouped_ffn, combine" if a.unfused else
                 "moe_layer_forward = route_topk, capacity_drop (its last launch also builds the tile schedule of "
                 "the expert GEMMs), dispatch_ffn (dispatch fused into the first GEMM), combine"}
    return out


def gamma_sweep(w, mode, scope, gammas, steps, warmup, fused=True, metric=0, overselect=0, max_experts=0):
    """Throughput, dropped share and Eq. (11) over capacity factors (inf = no drop)."""
    sweep = []
    for gm in gammas:
        o = measure(w, mode if gm != float("inf") else MODES["none"], scope, gm if gm != float("inf") else 1.0, steps,
                    warmup, fused=fused, metric=metric, overselect=overselect, max_experts=max_experts, per_kernel=False)
        sweep.append({"gamma": gm if gm != float("inf") else "inf", "tokens_per_s": round(o["tokens_per_s"], 1),
                      "ms_per_step": round(o["ms_per_step"], 4), "dropped_ratio": round(o["dropped_ratio"], 4),
                      "DT_eq11": round(o["dt_eq11"], 4), "surviving_pairs": o["rows"], "loads": o["loads"]})
    return sweep


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (use --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch

    from paper_2503_05066_amd import build, capmoe, synth

    if not os.path.exists(capmoe.LIB_PATH):
        build.build()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    w = synth.WORKLOADS[a.workload]
    if a.tokens:
        w = synth.scaled(w, n_tokens=a.tokens)
    mode, scope = MODES[a.mode], SCOPES[a.scope]
    common = dict(fused=not a.unfused, metric=METRICS[a.metric], overselect=a.overselect,
                  max_experts=int(a.max_experts))
    keep_host = not a.no_cpu_baseline
    r = measure(w, mode, scope, a.gamma, a.steps, a.warmup, keep_host=keep_host, **common)
    main_line = line_of(w, a, a.mode, a.scope, r)
    out = {
        "metric": "MoE-layer tokens/sec at gamma=1.0 (Token & Expanded Drop); % MFMA/HBM roofline",
        "value": r["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == synth.DTYPE_BF16 else "f32", "data": "synthetic",
    }
    out.update(main_line)
    if not a.no_peaks:
        pk = measured_peaks()
        out["measured_peaks"] = pk
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, mode, scope, a.gamma)
    # Expanded Drop on the same workload, same step count (the metric names both policies)
    if not a.no_expanded and a.mode == "token" and w.device_groups > 1:
        re_ = measure(w, MODES["expanded"], scope, a.gamma, a.steps, a.warmup, **common)
        ed = {"value": re_["tokens_per_s"], "unit": "tokens/s", "steps": a.steps, "warmup": a.warmup,
              "ms_per_step": re_["ms_per_step"]}
        ed.update(line_of(w, a, "expanded", a.scope, re_))
        if not a.no_cpu_baseline:
            ed["cpu_baseline"] = cpu_baseline(w, MODES["expanded"], scope, a.gamma)
        out["expanded_drop"] = ed
    if not a.no_peaks:
        for line in (out, out.get("expanded_drop") or {}):
            for key in ("roofline", "roofline_down"):
                rf = line.get(key)
                if rf:
                    ceiling = pk["mfma_bf16_TFLOPs"] if rf["bound"] == "mfma" else pk["copy_GBs"]
                    rf["frac_of_measured_ceiling"] = round(rf["achieved"] / ceiling, 4)
                    if rf["bound"] == "mfma":   # the same loop on operands like the layer's (random bits)
                        rf["frac_of_mfma_loop_on_random_operands"] = round(
                            rf["achieved"] / pk["mfma_bf16_random_operands_TFLOPs"], 4)
    if a.sweep_gamma:
        gammas = [float(g) for g in a.sweep_gamma.split(",")]
        out["gamma_sweep"] = {"mode": a.mode, "scope": a.scope, "steps": max(20, a.steps // 10),
                              "points": gamma_sweep(w, mode, scope, gammas, max(20, a.steps // 10),
                                                    max(5, a.warmup // 4), **common)}
    if not a.no_straggler and w.device_groups > 1:
        out["straggler"] = straggler(w, mode, scope, a.gamma, a.overselect, int(a.max_experts))
    uniform = []
    for n in ([] if a.no_peaks else [n for n in a.ffn_uniform.split(",") if n]):
        uniform.append(ffn_uniform(synth.WORKLOADS[n]))
        if synth.WORKLOADS[n].n_experts > 1:
            uniform.append(ffn_uniform(synth.WORKLOADS[n], experts=1, vendor=False))
    if uniform:
        out["ffn_uniform_experts"] = uniform
    others = []
    o_steps, o_warm = max(20, a.steps // 4), max(5, a.warmup // 4)
    for item in [s for s in a.others.split(",") if s]:
        parts = item.split(":")
        name, m = parts[0], parts[1]
        osc = parts[2] if len(parts) > 2 else a.scope
        if name == a.workload and m in (a.mode, "expanded") and osc == a.scope:
            continue
        ow = synth.WORKLOADS[name]
        o = measure(ow, MODES[m], SCOPES[osc], a.gamma, o_steps, o_warm, fused=not a.unfused, metric=METRICS[a.metric])
        entry = {"workload": name, "mode": m, "scope": osc, "gamma": a.gamma, "steps": o_steps,
                 "tokens_per_s": o["tokens_per_s"], "ms_per_step": o["ms_per_step"],
                 "step_ms_median": round(o["step_ms_median"], 4), "step_ms_min": round(o["step_ms_min"], 4),
                 "dropped_ratio": round(o["dropped_ratio"], 4),
                 "experts_per_token_mean": round(o["experts_per_token_mean"], 3), "surviving_pairs": o["rows"],
                 "cap": o["cap"], "max_segment_load": o["max_segment_load"], "loads": o["loads"],
                 "kernel_ms": {k: (round(v, 4) if v is not None else None) for k, v in o["kernel_ms"].items()}}
        for key, kernel, ms in (("ffn_gate_up", "ffn_gate_up", o["gate_up_ms"]), ("ffn_down", "ffn_down", o["down_ms"])):
            if ms is not None:
                entry[key] = rounded(roofline_of(o["work"][kernel], ms)[0])
        others.append(entry)
    if others:
        out["other_workloads"] = others
    if a.calibration_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["calibration_copy_bytes"] = 1 << 30
    print(json.dumps(out))


if __name__ == "__main__":
    main()
