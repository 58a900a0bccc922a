"""Helpers of the GPU parity tests: move synthetic inputs to the device and compare results.

No arithmetic of the method lives here: the oracle (oracle/) supplies expected values, the
library (through paper_2503_05066_amd.capmoe) supplies actual values.
"""
import numpy as np
import torch

from paper_2503_05066_amd import capmoe, synth


def to_device(stored: synth.Stored):
    """A synth.Stored tensor as a device tensor of its storage type."""
    if stored.bits is not None:
        return torch.from_numpy(stored.bits.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(stored.f32).cuda()


def to_host_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


class DeviceLayer:
    """Inputs of one workload on the device, plus the fp32-valued host copies the oracle reads."""

    def __init__(self, w: synth.Workload, trial: int = 0, experts=None, host_weights=True):
        self.w = w
        x = synth.tokens(w, trial)
        self.x_host = x.f32
        self.x = to_device(x)
        self.w_router_host = synth.router_weight(w, trial)
        self.bias_host = synth.router_bias(w, trial)
        self.w_router = torch.from_numpy(self.w_router_host).cuda()
        self.bias = torch.from_numpy(self.bias_host).cuda()
        e, h, d = w.n_experts, w.d_hidden, w.d_model
        act = torch.bfloat16 if w.dtype == synth.DTYPE_BF16 else torch.float32
        self.w_gate = torch.empty((e, h, d), dtype=act, device="cuda")
        self.w_up = torch.empty((e, h, d), dtype=act, device="cuda")
        self.w_down = torch.empty((e, d, h), dtype=act, device="cuda")
        # host copies (fp32 values) only for the experts the oracle will need
        self.host_gate, self.host_up, self.host_down = [None] * e, [None] * e, [None] * e
        keep_host = set(range(e)) if experts is None else set(experts)
        for j in range(e):
            g, u, dn = synth.expert_weights(w, j, trial, keep_f32=host_weights and j in keep_host)
            self.w_gate[j].copy_(to_device(g))
            self.w_up[j].copy_(to_device(u))
            self.w_down[j].copy_(to_device(dn))
            if host_weights and j in keep_host:
                self.host_gate[j], self.host_up[j], self.host_down[j] = g.f32, u.f32, dn.f32

    def desc(self, mode, scope, gamma, groups=None):
        w = self.w
        return capmoe.make_desc(w.n_tokens, w.d_model, w.n_experts, w.top_k, w.d_hidden,
                                w.device_groups if groups is None else groups, mode, scope, gamma, w.dtype)


def assert_plan_equal(buf: capmoe.LayerBuffers, ref, what=""):
    """Bit-exact comparison of the device plan with the oracle's plan."""
    torch.cuda.synchronize()
    p = ref.plan
    rows = p.rows
    np.testing.assert_array_equal(buf.expert_count.cpu().numpy(), p.expert_count, err_msg=what + " expert_count")
    np.testing.assert_array_equal(buf.expert_offset.cpu().numpy(), p.expert_offset, err_msg=what + " expert_offset")
    np.testing.assert_array_equal(buf.seg_count.cpu().numpy(), p.seg_count, err_msg=what + " seg_count")
    np.testing.assert_array_equal(buf.row_token.cpu().numpy()[:rows], p.row_token, err_msg=what + " row_token")
    np.testing.assert_array_equal(buf.row_weight.cpu().numpy()[:rows].view(np.uint32), p.row_weight.view(np.uint32),
                                  err_msg=what + " row_weight")
    np.testing.assert_array_equal(buf.pair_row.cpu().numpy(), p.pair_row, err_msg=what + " pair_row")


def assert_output_close(y: np.ndarray, y_ref: np.ndarray, tol: float, what=""):
    """Relative error in the Frobenius norm and in the maximum norm; rows that are zero in the
    reference (no surviving expert) must be exactly zero."""
    y = np.asarray(y, np.float64)
    zero_rows = ~np.any(y_ref != 0.0, axis=1)
    assert np.all(y[zero_rows] == 0.0), what + ": a token without surviving pairs must give y = 0"
    num = np.linalg.norm(y - y_ref)
    den = np.linalg.norm(y_ref)
    assert num <= tol * den, f"{what}: Frobenius error {num / max(den, 1e-300):.3e} > {tol}"
    mx = np.abs(y - y_ref).max() if y.size else 0.0
    assert mx <= tol * np.abs(y_ref).max(), f"{what}: max error {mx:.3e} vs {tol} * {np.abs(y_ref).max():.3e}"
