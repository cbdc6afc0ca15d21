"""Shared helpers for the GPU parity tests: move a seeded workload to the device, build the
library context for it, and error metrics.  No method arithmetic lives here."""
from __future__ import annotations

import numpy as np
import torch

from paper_2511_17885_amd import binding
from paper_2511_17885_amd import workloads as W

TOL = {W.F32: 1e-5, W.BF16: 2e-2}   # max-norm relative error bound per storage dtype


def dev(a, dtype=None):
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    if dtype is not None:
        t = t.to(dtype)
    return t.contiguous()


def torch_dtype(wl):
    return torch.bfloat16 if wl.dtype == W.BF16 else torch.float32


def make_layer(wl, layer=0, k_text=None, k_visual=None, renormalize=True, ffn_shape=0):
    lw = wl.layers[layer]
    td = torch_dtype(wl)
    m = binding.FMoE(d_model=wl.d, n_experts=wl.E, d_ffn=wl.F, n_shared=wl.n_shared,
                     d_ffn_shared=wl.F_shared if wl.n_shared else 0,
                     k_text=wl.k_text if k_text is None else k_text,
                     k_visual=wl.k_visual if k_visual is None else k_visual,
                     dtype=wl.dtype, renormalize=renormalize)
    m.set_weights(dev(lw.router_w, td), dev(lw.router_bias), dev(lw.w_gate, td), dev(lw.w_up, td),
                  dev(lw.w_down, td), dev(lw.ws_gate, td), dev(lw.ws_up, td), dev(lw.ws_down, td))
    m.set_ffn_shape(ffn_shape)
    return m


def inputs(wl):
    return dev(wl.x, torch_dtype(wl)), dev(wl.is_visual), dev(wl.cu_seqlens)


def host(t):
    if t is None:
        return None
    if t.dtype == torch.bfloat16:
        t = t.float()
    return t.detach().cpu().numpy()


def max_rel_err(got, ref):
    """max |got - ref| / max |ref| over the tensor (element-wise relative error is meaningless on
    sums that cancel)."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    scale = np.abs(ref).max()
    if scale == 0:
        return float(np.abs(got).max())
    return float(np.abs(got - ref).max() / scale)


def elementwise_rel_err(got, ref):
    """max over elements of |got - ref| / max(|ref|, 1e-3 * max |ref|): the element-wise figure, with a
    floor so that elements near a cancellation do not divide by nothing."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    scale = np.abs(ref).max()
    if scale == 0:
        return float(np.abs(got).max())
    return float((np.abs(got - ref) / np.maximum(np.abs(ref), 1e-3 * scale)).max())


def assert_outputs_close(got, ref, dtype, what=""):
    """The output bar: max-norm relative error within the storage dtype's tolerance.  The message carries
    the element-wise figure as well."""
    err = max_rel_err(got, ref)
    assert err <= TOL[dtype], (f"{what}: max|d|/max|ref| = {err:.3e} > {TOL[dtype]:.0e}; element-wise "
                               f"(floor 1e-3 max|ref|) = {elementwise_rel_err(got, ref):.3e}")
    return err


# relative size of half a unit in the last place of a stored value
HALF_ULP = {W.F32: 2.0 ** -24, W.BF16: 2.0 ** -8}


def assert_residual_outputs_close(got, ref_f64, x_rows, dtype, what=""):
    """Outputs of a run with the residual added, x + MoE(x).  The input x is O(1) while the expert term
    can be two orders of magnitude smaller, so an error bound relative to max |x + MoE(x)| would hide a
    wrong expert term.  Bound used instead, per element: the tolerance times the largest |MoE term| of
    the oracle (ref - x), plus the one rounding of the stored sum (half a unit in the last place of the
    element itself), plus the roundings of the fp32 accumulator that holds x while the expert terms are
    added to it (residual, shared experts, up to 16 slots: at most 20 additions of half an fp32 unit)."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref_f64, np.float64)
    moe = ref - np.asarray(x_rows, np.float64)
    scale = np.abs(moe).max()
    bound = TOL[dtype] * scale + (HALF_ULP[dtype] + 20 * 2.0 ** -24) * np.maximum(np.abs(ref), np.abs(got))
    diff = np.abs(got - ref)
    worst = int(np.argmax(diff - bound))
    assert (diff <= bound).all(), (f"{what}: |d| = {diff.flat[worst]:.3e} > bound {bound.flat[worst]:.3e} "
                                   f"(max|MoE term| = {scale:.3e}, max|ref| = {np.abs(ref).max():.3e})")
