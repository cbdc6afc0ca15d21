"""The entry point that allocates nothing: fmoe_permute_noalloc (scratch in the library's static device
array) against fmoe_permute (caller's workspace) through the C ABI -- integer work, so bit for bit --
on two calls in a row, the second with a smaller input, so that whatever the first call left in the
shared scratch array is shown not to leak into the second."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_17885_amd import workloads as W
from harness import dev, host, make_layer

pytestmark = pytest.mark.gpu


def _routing(seed, T_v, T_t, E, k_text, k_visual):
    wl = W.small_random(seed, T_v=T_v, T_t=T_t, d=64, E=E, F=32, k_text=k_text, k_visual=k_visual,
                        retention=0.5, window=3, bias_std=2.0)
    _, idx, _ = oracle.route(wl.x, wl.is_visual, wl.weights.router_w, wl.weights.router_bias, k_text, k_visual)
    o = oracle.layer_forward(wl.x, wl.is_visual, wl.cu_seqlens, wl.weights, k_text=k_text, k_visual=k_visual,
                             is_bf16=False, retention=0.5, window=3, ffn=False)
    return wl, idx, o["kept_idx"]


def _compare(m, idx, kept, E):
    n = len(kept)
    ws_out = m.permute(dev(idx), dev(kept), n)
    na_out = m.permute_noalloc(dev(idx), dev(kept), n)
    torch.cuda.synchronize()
    o_offs, o_perm, o_inv = oracle.permute(idx, kept, E)
    M = int(o_offs[-1])
    for got in (ws_out, na_out):
        assert np.array_equal(host(got[0]), o_offs)
        assert np.array_equal(host(got[1])[:M], o_perm)
        assert np.array_equal(host(got[2])[:n], o_inv)
    return M


def test_permute_noalloc_matches_permute_on_two_calls_the_second_smaller():
    # first call: several 256-position blocks, 33 experts; second: fewer tokens on the same context
    wl1, idx1, kept1 = _routing(301, [1500, 700], [100, 30], 33, 5, 2)
    m = make_layer(wl1)
    M1 = _compare(m, idx1, kept1, 33)
    wl2, idx2, kept2 = _routing(302, [90], [11], 33, 5, 2)
    M2 = _compare(m, idx2, kept2, 33)
    assert M2 < M1 and len(kept2) < len(kept1)
    # a device-side count below the capacity, as the fused layer passes it
    n = len(kept1)
    cap = np.concatenate([kept1, np.zeros(wl1.T - n, np.int32)])
    n_dev = dev(np.array([n], np.int32))
    a = m.permute(dev(idx1), dev(cap), wl1.T, n_kept_dev=n_dev)
    b = m.permute_noalloc(dev(idx1), dev(cap), wl1.T, n_kept_dev=n_dev)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1][:M1], b[1][:M1]) and torch.equal(a[2][:n], b[2][:n])


def test_permute_noalloc_other_context_and_empty_input():
    # another context (other E, Kmax) shares the same static array
    wl, idx, kept = _routing(303, [300], [40], 128, 8, 4)
    m = make_layer(wl)
    _compare(m, idx, kept, 128)
    offs, perm, inv = m.permute_noalloc(dev(idx), None, 0)
    torch.cuda.synchronize()
    assert not host(offs).any()
