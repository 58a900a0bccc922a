"""moe_route_topk_static (the entry point that allocates nothing: its split-K partial sums live in a buffer
built into the library) against moe_route_topk through the C ABI: every output equal bit for bit, on calls in a
row that share the built-in buffer, the later ones with smaller inputs."""
import numpy as np
import pytest
import torch

from paper_2503_05066_amd import capmoe, synth

from gpu_util import to_device

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("built_library")]

W = synth.WORKLOADS
_looked_up = [False]     # the first call on a device looks the built-in buffer up; the runtime places it then


def both(w, bias=True):
    print("static route", w, flush=True)
    x = to_device(synth.tokens(w))
    wr = torch.from_numpy(synth.router_weight(w)).cuda()
    b = torch.from_numpy(synth.router_bias(w)).cuda() if bias else None
    desc = capmoe.make_desc(w.n_tokens, w.d_model, w.n_experts, w.top_k, w.d_hidden, 1, synth.MODE_TOKEN_DROP,
                            synth.SCOPE_LOCAL, 1.0, w.dtype)
    ref, got = capmoe.LayerBuffers(desc), capmoe.LayerBuffers(desc)
    capmoe.moe_route_topk(desc, x, wr, b, 0, ref.logits, ref.scores, ref.topk_idx, ref.topk_score, ref.workspace)
    for t in (got.logits, got.scores, got.topk_score):
        t.fill_(float("nan"))
    got.topk_idx.fill_(-7)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    capmoe.moe_route_topk_static(desc, x, wr, b, 0, got.logits, got.scores, got.topk_idx, got.topk_score)
    torch.cuda.synchronize()
    if _looked_up[0]:
        assert torch.cuda.mem_get_info()[0] == free_before      # nothing was allocated on the device
    _looked_up[0] = True
    for name in ("logits", "scores", "topk_score"):
        assert torch.equal(getattr(ref, name).view(torch.int32), getattr(got, name).view(torch.int32)), name
    assert torch.equal(ref.topk_idx, got.topk_idx)
    return desc, got


def test_static_scratch_route_matches_workspace_route():
    # split-K partial sums in the built-in buffer: 8 slices at the OLMoE shape, then smaller inputs that leave
    # most of the previous call's partial sums in place, then the decode shape (32 slices), then a larger one again
    both(W["olmoe"])
    both(synth.scaled(W["olmoe"], n_tokens=1000))
    both(synth.scaled(W["olmoe"], n_tokens=77, n_experts=48, top_k=5), bias=False)
    both(W["decode"])
    both(W["mixtral"])
    # a single K slice (no scratch needed) and the fp32 router kernel (no matrix cores, no scratch)
    both(synth.scaled(W["finegrained"], n_tokens=33000))
    both(W["tiny"])


def test_static_scratch_given_logits_and_limits():
    w = synth.scaled(W["olmoe"], n_tokens=512)
    desc, got = both(w)
    # logits handed in: the softmax / top-k half alone
    again = capmoe.LayerBuffers(desc)
    again.logits.copy_(got.logits)
    capmoe.moe_route_topk_static(desc, None, None, None, 1, again.logits, again.scores, again.topk_idx,
                                 again.topk_score)
    torch.cuda.synchronize()
    assert torch.equal(again.scores.view(torch.int32), got.scores.view(torch.int32))
    assert torch.equal(again.topk_idx, got.topk_idx)
    # more partial sums than the built-in buffer holds: refused, nothing enqueued
    big = capmoe.make_desc(4096 * 3, 4096, 256, 8, 1024, 1, synth.MODE_TOKEN_DROP, synth.SCOPE_LOCAL, 1.0,
                           synth.DTYPE_BF16)
    with pytest.raises(capmoe.CapMoeError) as ei:
        capmoe.moe_route_topk_static(big, got.logits, got.logits, None, 0, got.logits, got.scores, got.topk_idx,
                                     got.topk_score)
    assert ei.value.status == 5 and "scratch" in str(ei.value)
    with pytest.raises(capmoe.CapMoeError) as ei:     # the usual argument checks still apply
        capmoe.moe_route_topk_static(desc, None, None, None, 0, got.logits, got.scores, got.topk_idx, got.topk_score)
    assert ei.value.status == 1
