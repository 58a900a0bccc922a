"""GPU checks behind the latency-model measurements of bench.py (Eq. 4 on one GPU, Eq. 11): the per-device FFN
launches compute the rows the full layer call computes, and the statistics of the capacity-factor sweep equal
what the oracle counts."""
import math
import os
import sys

import numpy as np
import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402

from paper_2503_05066_amd import capmoe, synth  # noqa: E402

from gpu_util import DeviceLayer  # noqa: E402

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("built_library")]

TD, ED, NONE = synth.MODE_TOKEN_DROP, synth.MODE_EXPANDED_DROP, synth.MODE_NONE
LOCAL, GLOBAL = synth.SCOPE_LOCAL, synth.SCOPE_GLOBAL


@pytest.fixture(scope="module")
def mixtral():
    """The Mixtral-shaped workload on the device, registered as bench.py's resident upload."""
    w = synth.WORKLOADS["mixtral"]
    layer = DeviceLayer(w, host_weights=False)
    t = {"x": layer.x, "w_router": layer.w_router, "bias": layer.bias, "w_gate": layer.w_gate, "w_up": layer.w_up,
         "w_down": layer.w_down}
    bench._uploaded.clear()
    bench._uploaded[(w.name, w.n_tokens)] = t
    yield w, layer, t
    bench._uploaded.clear()
    del layer, t
    torch.cuda.empty_cache()


@pytest.mark.parametrize("mode", [TD, ED, NONE])
def test_per_device_launches_compute_the_rows_of_the_full_call(mixtral, mode):
    """bench.py times each simulated device's experts as a layer call of its own on a slice of the plan (Eq. 4:
    the slowest device sets the pace).  Every row such a launch writes must be the row the full call writes.
    The two launches may cut the K dimension of their last work items differently (a split sum is added in
    another order), so values agree to the last bf16 digit, and nearly all of them bit for bit."""
    w, layer, t = mixtral
    desc = layer.desc(mode, LOCAL, 1.0)
    buf = capmoe.LayerBuffers(desc)
    capmoe.layer_forward(buf, t["x"], t["w_router"], t["bias"], t["w_gate"], t["w_up"], t["w_down"],
                         fused_dispatch=True)
    torch.cuda.synchronize()
    rows = int(buf.expert_offset[-1])
    full = buf.yp[:rows].clone()
    assert torch.isfinite(full.float()).all()
    covered = 0
    for dev, r0, r1, sub, args in bench.device_slices(w, buf, t):
        print("device", dev, "rows", r0, r1, flush=True)
        ws = torch.empty(max(capmoe.moe_query(sub)[3], 256), dtype=torch.uint8, device="cuda")
        buf.yp[r0:r1].fill_(float("nan"))
        capmoe.moe_dispatch_ffn(*args, ws)
        torch.cuda.synchronize()
        got, ref = buf.yp[r0:r1].float(), full[r0:r1].float()
        assert torch.equal(buf.yp[:r0], full[:r0]) and torch.equal(buf.yp[r1:rows], full[r1:rows])  # nothing else written
        assert torch.isfinite(got).all()
        # one bf16 step of the value, plus what another order of the fp32 sum can move a value that cancels
        bound = ref.abs() * 2.0 ** -7 + ref.abs().amax(dim=1, keepdim=True) * 2.0 ** -14
        assert ((got - ref).abs() <= bound).all()
        assert (got == ref).float().mean() > 0.99
        buf.yp[r0:r1].copy_(full[r0:r1])
        covered += r1 - r0
    assert covered == rows


def test_gamma_sweep_statistics_equal_the_oracles_counts(orc, mixtral):
    """dropped_ratio, surviving pairs and Eq. (11) of bench.py's capacity-factor sweep against the oracle run on
    the library's own logits (read back), for both capacity scopes."""
    w, layer, t = mixtral
    desc = layer.desc(NONE, LOCAL, 1.0)
    buf = capmoe.LayerBuffers(desc)
    capmoe.moe_route_topk(desc, t["x"], t["w_router"], t["bias"], 0, buf.logits, buf.scores, buf.topk_idx,
                          buf.topk_score, buf.workspace)
    torch.cuda.synchronize()
    logits = buf.logits.cpu().numpy()
    gammas = [0.5, 1.0, 1.5, 2.0, math.inf]
    nbar = w.n_tokens * w.top_k / w.n_experts
    for scope_name, scope in (("local", LOCAL), ("global", GLOBAL)):
        points = bench.gamma_sweep(w, TD, scope, gammas, steps=2, warmup=1)
        for gm, pt in zip(gammas, points):
            print("sweep", scope_name, gm, pt, flush=True)
            ref = orc.route_and_drop(logits, w.top_k, w.device_groups, TD if gm != math.inf else NONE, scope,
                                     gm if gm != math.inf else 1.0)
            before = np.bincount(ref.topk_idx.ravel(), minlength=w.n_experts)
            dt = float(np.maximum(before - gm * nbar, 0.0).sum() / before.sum()) if gm != math.inf else 0.0
            assert pt["surviving_pairs"] == ref.plan.rows
            assert pt["dropped_ratio"] == round(1.0 - ref.plan.rows / (w.n_tokens * w.top_k), 4)
            assert pt["DT_eq11"] == round(dt, 4)
            if scope == GLOBAL and gm != math.inf:
                # Eq. (11): with one capacity per expert over all tokens the dropped share IS the overflow share
                assert pt["dropped_ratio"] == pt["DT_eq11"]
            assert pt["tokens_per_s"] > 0
        drops = [p["dropped_ratio"] for p in points]
        assert all(a >= b for a, b in zip(drops, drops[1:])) and drops[-1] == 0.0    # a larger capacity drops less
