"""mixkv_compress_static (the entry point that allocates nothing: its workspace is a static array
inside the library) against mixkv_compress on a caller-provided workspace: same kernels, so every
output must agree bit for bit.  Two calls in a row share the array, the second on a smaller input."""
import ctypes as C

import pytest
import torch

from paper_2510_20707_amd import binding as B
from paper_2510_20707_amd import synth
from tests import harness as H

pytestmark = pytest.mark.gpu


def _both(wl, layers, **over):
    """Run the same layers through mixkv_compress and mixkv_compress_static; return both outputs."""
    dev = "cuda:0"
    p = H.gpu_params(wl, **over)
    Ks = [H.to_device(wl, l.K, dev) for l in layers]
    Vs = [H.to_device(wl, l.V, dev) for l in layers]
    Qs = [H.to_device(wl, l.Q, dev) for l in layers]
    ref = [B.alloc_layer_out(p, dev, scores=True) for _ in layers]
    new = [B.alloc_layer_out(p, dev, scores=True) for _ in layers]
    for o in new:                                      # poison, so that an output the call never wrote shows
        o.indices.fill_(-7)
        _bits(o.K_out).fill_(0x7fc1)
        _bits(o.V_out).fill_(0x7fc1)
        o.scores.fill_(float("nan"))
    ws = B.alloc_workspace(p, len(layers), dev)
    B.mixkv_compress(p, Ks, Vs, Qs, ref, ws)
    B.mixkv_compress_static(p, Ks, Vs, Qs, new)
    torch.cuda.synchronize()
    return p, ref, new


def _bits(t):
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32)


def _assert_same(ref, new):
    for r, n in zip(ref, new):
        for name in ("indices", "counts", "offsets", "K_out", "V_out", "scores", "redundancy"):
            assert torch.equal(_bits(getattr(r, name)), _bits(getattr(n, name))), name      # bit for bit


def test_static_workspace_matches_caller_workspace_on_two_calls_in_a_row():
    # first call: two layers of the Qwen2-VL-shaped single-layer config (bf16, N = 4096)
    wl = synth.WORKLOADS["c2"].with_(n_layers=2)
    layers = [synth.make_layer(wl, l) for l in range(2)]
    p, ref, new = _both(wl, layers)
    _assert_same(ref, new)
    st = H.check_layer(wl, layers[1], p, new[1], units=[(0, 1)])       # and against the oracle, one unit
    assert st["checked"] == 1
    # second call, smaller input (fp32, N = 512): the array still holds the first call's contents
    wl1 = synth.WORKLOADS["c1"]
    lay1 = synth.make_layer(wl1, 0)
    p1, ref1, new1 = _both(wl1, [lay1])
    _assert_same(ref1, new1)
    st = H.check_layer(wl1, lay1, p1, new1[0])
    assert st["checked"] == wl1.batch * wl1.n_kv_heads
    # and once more with head-adaptive budgets on a ragged shape
    wl2 = synth.WORKLOADS["c2"].with_(seq_len=1000, text_suffix_start=940, budget_mode="adaptive", budget_floor=8)
    lay2 = synth.make_layer(wl2, 0)
    p2, ref2, new2 = _both(wl2, [lay2])
    _assert_same(ref2, new2)


def test_static_workspace_rejects_shapes_beyond_its_size():
    wl = synth.WORKLOADS["c5"]                          # 28 layers x batch 4 x 32K tokens: 288 MiB of workspace
    p = H.gpu_params(wl)
    assert B.mixkv_workspace_size(p, wl.n_layers) > B.STATIC_SCRATCH_BYTES
    n = wl.n_layers
    ins, outs = (B.MixkvLayerIn * n)(), (B.MixkvLayerOut * n)()
    assert B.lib().mixkv_compress_static(C.byref(p), ins, outs, n, None) == B.MIXKV_ERR_WORKSPACE_TOO_SMALL
    # argument errors come first, as in mixkv_compress
    assert B.lib().mixkv_compress_static(C.byref(p), ins, outs, 0, None) == B.MIXKV_ERR_INVALID_ARG
    # a shape that fits but null layer pointers: rejected on the host, nothing launched
    wl3 = synth.WORKLOADS["c1"]
    p3 = H.gpu_params(wl3)
    ins1, outs1 = (B.MixkvLayerIn * 1)(), (B.MixkvLayerOut * 1)()
    assert B.lib().mixkv_compress_static(C.byref(p3), ins1, outs1, 1, None) == B.MIXKV_ERR_INVALID_ARG
    torch.cuda.synchronize()
