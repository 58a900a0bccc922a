"""Host-side checks of the C ABI that need no GPU: the library loads, exports what the header
declares, sizes come out as the paper's capacity formula says, and bad arguments are refused
before anything is launched."""
import ctypes
import math
import os
import re

import pytest

from paper_2503_05066_amd import capmoe, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

pytestmark = pytest.mark.usefixtures("built_library")


def declared_functions():
    text = open(os.path.join(ROOT, "include", "capmoe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = capmoe.load()
    names = declared_functions()
    assert {"moe_route_topk", "moe_capacity_drop", "moe_dispatch", "moe_grouped_ffn", "moe_dispatch_ffn", "moe_combine",
            "moe_query", "moe_profile_attach", "moe_layer_forward", "moe_probe_mfma_bf16", "moe_capacity_drop_ranked",
            "moe_status_string", "moe_route_topk_static", "moe_ffn_schedule_query"} <= set(names)
    for n in names:
        assert getattr(lib, n) is not None
    assert capmoe.status_string(0) == "ok" and "workspace" in capmoe.status_string(3)


def test_descriptor_layout_matches_header():
    # 8 int32, one double at offset 32, four int32: 56 bytes
    assert ctypes.sizeof(capmoe.MoeDesc) == 56 and capmoe.MoeDesc.gamma.offset == 32
    assert capmoe.MoeDesc.overselect.offset == 48 and capmoe.MoeDesc.max_experts.offset == 52


@pytest.mark.parametrize("name,mode,scope,gamma,cap,slots,rows", [
    ("tiny", 1, 0, 1.0, 32, 2, 256), ("olmoe", 1, 0, 1.0, 512, 8, 32768), ("olmoe", 1, 0, 1.5, 768, 8, 32768),
    ("olmoe", 1, 0, 2.0, 1024, 8, 32768), ("mixtral", 1, 0, 1.0, 512, 2, 16384), ("mixtral", 2, 0, 1.0, 512, 4, 16384),
    ("mixtral", 1, 1, 1.0, 2048, 2, 16384), ("finegrained", 2, 0, 1.0, 128, 24, 131072),
    ("finegrained", 2, 1, 1.25, 1280, 24, 163840), ("decode", 2, 0, 1.0, 3, 14, 1536),
    ("olmoe", 0, 0, 1.0, 4096, 8, 32768), ("olmoe", 1, 0, math.inf, 4096, 8, 32768), ("olmoe", 1, 0, 0.0, 0, 8, 0),
    ("mixtral", 1, 2, 1.0, 1024, 2, 16384), ("finegrained", 2, 2, 1.0, 2048, 24, 131072),
    ("finegrained", 1, 3, 1.25, 20480, 8, 131072),
])
def test_query_sizes(orc, name, mode, scope, gamma, cap, slots, rows):
    w = synth.WORKLOADS[name]
    d = capmoe.make_desc(w.n_tokens, w.d_model, w.n_experts, w.top_k, w.d_hidden, w.device_groups, mode, scope, gamma,
                         w.dtype)
    got = capmoe.moe_query(d)
    assert got[:3] == (cap, slots, rows)
    blocks = w.device_groups if scope in (0, 2) else 1
    if mode != 0 and scope < 2:
        assert cap == orc.capacity(gamma, w.n_tokens // blocks, w.top_k, w.n_experts)
    if mode != 0 and scope >= 2:
        assert cap == orc.device_budget(gamma, w.n_tokens // blocks, w.top_k, w.n_experts,
                                        w.n_experts // w.device_groups)
    assert got[3] > 0


def test_overselection_sizes(orc):
    w = synth.WORKLOADS["olmoe"]
    for mode, g, m, slots in [(1, 1, 16, 24), (2, 8, 8, 24), (0, 1, 24, 32)]:
        d = capmoe.make_desc(w.n_tokens, w.d_model, w.n_experts, w.top_k, w.d_hidden, g, mode, 0, 1.0, w.dtype,
                             overselect=m, max_experts=1)
        cap, s, rows, _ = capmoe.moe_query(d)
        assert s == slots == orc.slots_per_token(w.top_k, w.n_experts, g, mode, m)
        # the capacity keeps using the model's k
        assert cap == (w.n_tokens // g if mode == 0 else orc.capacity(1.0, w.n_tokens // g, w.top_k, w.n_experts))
    with pytest.raises(capmoe.CapMoeError) as ei:
        capmoe.moe_query(capmoe.make_desc(1024, 64, 128, 40, 128, overselect=30))   # k + m > 64
    assert ei.value.status == 2


def test_capacity_truncation_matches_oracle(orc):
    for gamma in (1.3, 0.7, 1.1, 2.5, 0.05, 0.999):
        for n, k, e, g in [(128, 2, 8, 1), (120, 3, 12, 4), (96, 5, 16, 2)]:
            d = capmoe.make_desc(n, 64, e, k, 128, g, 1, 0, gamma, 0)
            assert capmoe.moe_query(d)[0] == orc.capacity(gamma, n // g, k, e)


MODES = {"none": 0, "token": 1, "expanded": 2}


@pytest.mark.parametrize("name,mode,tiles,gate_up,down", [
    # Mixtral shape, Token Drop: 34 big + 3 short tiles.  Gate/up (K = 4096: never cut; 37 x 112 items = 16 rounds)
    # walks the joint list and shares out its last 256 items; down (K = 14336) cuts the 4 big items an XCD has
    # left after two rounds into 4 units (18 of 32 compute units: the 6 short items count half) and the 6 short
    # ones into 5
    ("mixtral", "token", (34, 3), [0, 1, 0, 1, 1, 256, 0, 0], [4, 4, 6, 5, 0, 0, 0, 0]),
    # no drop: 130 big items per XCD are four rounds and 2 left (5 units each beside 8 short items in 4 units)
    ("mixtral", "none", (65, 4), [0, 1, 0, 1, 1, 256, 0, 0], [2, 5, 8, 4, 0, 0, 0, 0]),
    # Expanded Drop: 86 big items per XCD leave 22, too many to cut; the 4 short ones run as 8 units each
    ("mixtral", "expanded", (43, 2), [0, 1, 0, 1, 1, 256, 0, 0], [0, 1, 4, 8, 0, 0, 0, 0]),
    # OLMoE shape: 2.7 rounds of items, K too short to cut, exactly two rounds of big items: nothing special
    ("olmoe", "token", (64, 22), [0, 1, 0, 1, 0, 0, 0, 0], [0, 1, 0, 1, 0, 0, 0, 0]),
    # fine-grained, Expanded Drop: gate/up has 161.25 big items per XCD, the 2 after the fifth round run as row pieces
    ("finegrained", "expanded", (215, 11), [0, 1, 0, 1, 0, 0, 2, 0], [0, 1, 0, 1, 0, 0, 0, 0]),
    # decode shape: short tiles only
    ("decode", "token", (0, 64), [0, 1, 0, 1, 0, 0, 0, 0], [0, 1, 0, 1, 0, 0, 0, 0]),
])
def test_tile_schedule_decisions_on_the_named_workloads(orc, name, mode, tiles, gate_up, down):
    """The launch form each benchmarked workload gets on 256 compute units (the library runs the same decision
    code on the device): a change that silently sends a workload down a slower form fails here."""
    w = synth.WORKLOADS[name]
    logits = orc.router_logits(synth.tokens(w).f32, synth.router_weight(w), synth.router_bias(w))
    ref = orc.route_and_drop(logits, w.top_k, w.device_groups, MODES[mode], 0, 1.0)
    d = capmoe.make_desc(w.n_tokens, w.d_model, w.n_experts, w.top_k, w.d_hidden, w.device_groups, MODES[mode], 0, 1.0,
                         w.dtype)
    got_tiles, (got_gate_up, got_down) = capmoe.moe_ffn_schedule_query(d, ref.plan.expert_count, 256)
    assert got_tiles == tiles
    assert got_gate_up == gate_up and got_down == down


def test_tile_schedule_query_edge_cases():
    d = capmoe.make_desc(1024, 256, 4, 1, 512, 1, 0, 1, 1.0, 1)
    # empty plan; one row; more rows than the plan can hold; a negative count
    assert capmoe.moe_ffn_schedule_query(d, [0, 0, 0, 0])[0] == (0, 0)
    assert capmoe.moe_ffn_schedule_query(d, [0, 1, 0, 0])[0] == (0, 1)
    assert capmoe.moe_ffn_schedule_query(d, [64, 65, 256, 257])[0] == (3, 2)   # 64 -> short, 65 -> partly filled big
    for bad in ([1024, 1, 0, 0], [-1, 0, 0, 0]):
        with pytest.raises(capmoe.CapMoeError) as ei:
            capmoe.moe_ffn_schedule_query(d, bad)
        assert ei.value.status == 1
    # fp32 layers use none of it
    f = capmoe.make_desc(128, 64, 8, 2, 128, 1, 1, 0, 1.0, 0)
    assert capmoe.moe_ffn_schedule_query(f, [32] * 8)[1] == [[0] * 8, [0] * 8]


def test_bad_arguments_are_refused_on_the_host():
    lib = capmoe.load()
    ok = capmoe.make_desc(128, 64, 8, 2, 128)
    bad = [
        capmoe.make_desc(128, 64, 8, 9, 128),                   # k > E
        capmoe.make_desc(130, 64, 8, 2, 128, device_groups=4),  # N not a multiple of G
        capmoe.make_desc(128, 64, 6, 2, 128, device_groups=4),  # E not a multiple of G
        capmoe.make_desc(128, 64, 8, 2, 128, gamma=-1.0),
        capmoe.make_desc(128, 64, 8, 2, 128, gamma=math.nan),
        capmoe.make_desc(128, 64, 8, 2, 128, mode=7),
        capmoe.make_desc(128, 64, 8, 2, 128, dtype=5),
        capmoe.make_desc(128, 0, 8, 2, 128),
        capmoe.make_desc(128, 64, 8, 2, 128, metric=4),
        capmoe.make_desc(128, 64, 8, 2, 128, overselect=-1),
        capmoe.make_desc(128, 64, 8, 2, 128, overselect=7),    # k + m > E
        capmoe.make_desc(128, 64, 8, 2, 128, max_experts=2),
    ]
    for d in bad:
        with pytest.raises(capmoe.CapMoeError) as ei:
            capmoe.moe_query(d)
        assert ei.value.status == 1
    with pytest.raises(capmoe.CapMoeError) as ei:
        capmoe.moe_query(capmoe.make_desc(128, 64, 4096, 2, 128))
    assert ei.value.status == 2
    # null pointers: every entry point answers MOE_ERR_INVALID_ARG without launching anything
    z = ctypes.c_void_p(None)
    assert lib.moe_route_topk(ctypes.byref(ok), z, z, z, 0, z, z, z, z, z, 0, z) == 1
    assert lib.moe_capacity_drop(ctypes.byref(ok), z, z, z, z, z, z, z, z, z, 0, z) == 1
    assert lib.moe_capacity_drop_ranked(ctypes.byref(ok), z, z, z, 0, z, z, z, z, z, z, z, 0, z) == 1
    assert lib.moe_dispatch(ctypes.byref(ok), z, z, z, z, z) == 1
    assert lib.moe_grouped_ffn(ctypes.byref(ok), z, z, z, z, z, z, z, 0, z) == 1
    assert lib.moe_dispatch_ffn(ctypes.byref(ok), z, z, z, z, z, z, z, z, 0, z) == 1
    assert lib.moe_combine(ctypes.byref(ok), z, z, z, z, z) == 1
    assert lib.moe_layer_forward(ctypes.byref(ok), *([z] * 7), 0, *([z] * 13), 0, z) == 1
    assert lib.moe_query(None, None, None, None, None) == 1
    assert lib.moe_ffn_schedule_query(ctypes.byref(ok), z, 256, z, z) == 1
    # x of 4 GiB or more: the gathered form of the bf16 FFN refuses (it addresses x with 32-bit byte offsets), the
    # form on permuted rows does not (it stops at the workspace check here; nothing is launched either way)
    big = capmoe.make_desc(1 << 21, 1024, 8, 2, 1024, dtype=1)
    f = ctypes.c_void_p(0x1000)
    assert lib.moe_dispatch_ffn(ctypes.byref(big), f, f, f, f, f, f, f, f, 0, z) == 2
    assert lib.moe_grouped_ffn(ctypes.byref(big), f, f, f, f, f, f, f, 0, z) == 3
    # the drop reads its lists in 16-byte pieces: a misaligned scores / topk_idx / pair_row pointer is refused
    g = ctypes.c_void_p(0x1004)
    assert lib.moe_capacity_drop(ctypes.byref(ok), g, f, f, f, f, f, f, f, f, 1 << 30, z) == 1
    assert lib.moe_capacity_drop(ctypes.byref(ok), f, g, f, f, f, f, f, f, f, 1 << 30, z) == 1
    assert lib.moe_capacity_drop(ctypes.byref(ok), f, f, f, f, f, f, f, g, f, 1 << 30, z) == 1
    # the static-scratch router: a descriptor whose partial sums exceed the built-in buffer is refused on the host
    huge = capmoe.make_desc(4096 * 3, 4096, 256, 8, 1024, dtype=1)
    assert lib.moe_route_topk_static(ctypes.byref(huge), f, f, z, 0, f, f, f, f, z) == 5
    assert "scratch" in capmoe.status_string(5)
