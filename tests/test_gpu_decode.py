"""GPU parity of mixkv_decode_attention: the new token's attention over the cache that
mixkv_compress just compacted (plus rows appended since), against the float64 oracle fed with the
same rows.

Tolerance, per output row (one query head): |gpu - ora| <= tol * max_d |ora_d| with tol = 1e-5 for
fp32 inputs (fp32 accumulation over at most a few thousand rows) and 2^-8 + 1e-4 for bf16 inputs
(the output is rounded to bf16, whose half ulp is up to 2^-8 of the element; 1e-4 covers the fp32
sums in front of the rounding)."""
import numpy as np
import pytest
import torch

from oracle import mixkv_oracle as O
from paper_2510_20707_amd import binding as B
from paper_2510_20707_amd import synth
from tests import harness as H

pytestmark = pytest.mark.gpu
WL = synth.WORKLOADS
TOL = {"f32": 1e-5, "bf16": 2.0 ** -8 + 1e-4}


def _quant(wl, a):
    if wl.dtype == "bf16":
        return (synth.round_to_bf16_bits(a.astype(np.float32)).astype(np.uint32) << 16).view(np.float32)
    return a.astype(np.float32)


def _decode_and_check(wl, layer_ids, tail_len, tail_cap=None, head_budgets=None, **over):
    tail_cap = tail_len if tail_cap is None else tail_cap
    print(f"[case] decode {wl.name} dtype={wl.dtype} D={wl.head_dim} Hq={wl.n_q_heads} Hkv={wl.n_kv_heads} "
          f"B={over.get('budget', wl.budget)} mode={over.get('budget_mode', wl.budget_mode)} tail={tail_len}/{tail_cap} "
          f"L={len(layer_ids)}", flush=True)
    layers = [synth.make_layer(wl, l) for l in layer_ids]
    p, caches = H.run_compress(wl, layers, head_budgets=head_budgets, **over)
    Bt, Hq, Hkv, D, G = wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.group
    rng = np.random.default_rng([81, wl.cfg_id, tail_len])
    qs, kts, vts = [], [], []
    for _ in layers:
        qs.append(_quant(wl, rng.standard_normal((Bt, Hq, D)) / np.sqrt(D) * 4.0))
        kts.append(_quant(wl, rng.standard_normal((Bt, Hkv, max(tail_cap, 1), D)) + 0.3))
        vts.append(_quant(wl, rng.standard_normal((Bt, Hkv, max(tail_cap, 1), D))))
    Qd = [H.to_device(wl, q) for q in qs]
    tails = [(H.to_device(wl, k), H.to_device(wl, v)) for k, v in zip(kts, vts)] if tail_cap > 0 else None
    outs = B.mixkv_decode_attention(p, caches, tails, Qd, tail_len)
    torch.cuda.synchronize()
    Bud = p.budget
    worst = 0.0
    for lay, c, q, kt, vt, o in zip(layers, caches, qs, kts, vts, outs):
        got = o.float().cpu().numpy().astype(np.float64)
        idx = c.indices.cpu().numpy().reshape(Bt, Hkv * Bud)
        cnt, off = c.counts.cpu().numpy(), c.offsets.cpu().numpy()
        for b in range(Bt):
            Ks, Vs = [], []
            for h in range(Hkv):
                rows = idx[b, off[b, h]:off[b, h] + cnt[b, h]]
                Ks.append(np.concatenate([_quant(wl, lay.K[b, h][rows]), kt[b, h, :tail_len]]))
                Vs.append(np.concatenate([_quant(wl, lay.V[b, h][rows]), vt[b, h, :tail_len]]))
            want = O.decode_attention(q[b], Ks, Vs, wl.softmax_scale)
            for g in range(Hq):
                err = np.abs(got[b, g] - want[g]).max() / np.abs(want[g]).max()
                worst = max(worst, err)
                assert err <= TOL[wl.dtype], f"b{b} g{g}: error {err:.2e}"
    print(f"       max error {worst:.2e} of the row's largest element", flush=True)


@pytest.mark.parametrize("tail_len", [0, 1, 5])
def test_c1_f32(tail_len):
    _decode_and_check(WL["c1"], [0], tail_len)


@pytest.mark.parametrize("tail_len,tail_cap", [(0, 0), (1, 16), (13, 16)])
def test_c2_bf16(tail_len, tail_cap):
    _decode_and_check(WL["c2"], [0], tail_len, tail_cap)


def test_packed_layouts_adaptive_and_per_head():
    wl = WL["c2"].with_(name="adaptive-dec", seq_len=1024, text_suffix_start=960, batch=2, budget=96,
                        budget_mode="adaptive", budget_floor=16, sigma=(0.1, 0.8))
    _decode_and_check(wl, [0, 1], 3, 8)
    wl = WL["c2"].with_(name="perhead-dec", seq_len=1024, text_suffix_start=960, batch=2)
    hb = np.array([[32, 64, 500, 1024], [40, 41, 42, 43]], dtype=np.int32)
    _decode_and_check(wl, [0, 1], 2, 4, head_budgets=hb, budget_mode="per_head", budget=405)


@pytest.mark.parametrize("dtype,D,Hq,Hkv,B", [("f32", 64, 32, 2, 37), ("bf16", 64, 6, 2, 21), ("f32", 128, 3, 3, 100),
                                              ("bf16", 128, 24, 2, 77)])
def test_group_sizes_and_ragged_row_counts(dtype, D, Hq, Hkv, B):
    # G = 16 and 12 take two workgroups per KV head; G = 3 pads to four query heads
    wl = WL["c2"].with_(name="ragged-dec", dtype=dtype, head_dim=D, seq_len=300, window=5, n_q_heads=Hq, n_kv_heads=Hkv,
                        budget=B, batch=2, text_prefix=16, text_suffix_start=260)
    _decode_and_check(wl, [0], 7, 9)


def test_bf16_more_query_heads_than_one_tile_of_columns():
    # G = 40: the matrix-core path serves 32 query heads per workgroup, so a KV head takes two (32 + 8)
    wl = WL["c2"].with_(name="wide-group-dec", seq_len=300, window=5, n_q_heads=80, n_kv_heads=2, budget=70, batch=1,
                        text_prefix=16, text_suffix_start=260)
    _decode_and_check(wl, [0], 3, 4)


@pytest.mark.parametrize("budget", [90, 700])
def test_bf16_offsets_that_have_to_move(budget):
    # logits with a spread of a few hundred: the weights are formed against an offset that only moves
    # when a sum leaves the range of a float, which here happens in several tiles and in every row
    # range; the softmax is close to one-hot, so the output is a value row almost bit for bit
    wl = WL["c2"].with_(name="steep-dec", softmax_scale=30.0)
    _decode_and_check(wl, [0], 9, 12, budget=budget)


def test_c3_whole_cache_and_more_layers_than_one_launch_group():
    _decode_and_check(WL["c3"], [0, 9, 27], 1, 4)
    wl = WL["c1"].with_(n_layers=35)
    _decode_and_check(wl, list(range(35)), 2, 2)


def test_long_caches_are_split_over_workgroups():
    # 1024 + 7 rows per head: three row ranges per head, merged in order; a per-head table with one very long head
    _decode_and_check(WL["c2"], [0], 7, 8, budget=1024)
    wl = WL["c2"].with_(name="perhead-long", batch=2)
    hb = np.array([[32, 40, 3000, 500]], dtype=np.int32)
    _decode_and_check(wl, [0], 2, 4, head_budgets=hb, budget_mode="per_head", budget=900)
    wl = WL["c1"].with_(n_layers=34)
    _decode_and_check(wl, list(range(34)), 3, 4, budget=500)          # f32, two launch groups of partials
    # bf16 with 64-element rows (two waves per workgroup on the matrix-core path), 12 query heads per KV head, 905 rows
    wl = WL["c2"].with_(name="d64-long", head_dim=64, n_q_heads=24, n_kv_heads=2, seq_len=2048, text_suffix_start=1900)
    _decode_and_check(wl, [0], 5, 8, budget=900)


def test_split_needs_its_workspace():
    wl = WL["c2"]
    p, caches = H.run_compress(wl, [synth.make_layer(wl, 0)], budget=1024)
    q = torch.zeros((wl.batch, wl.n_q_heads, wl.head_dim), device="cuda:0", dtype=torch.bfloat16)
    assert B.mixkv_decode_workspace_size(p, 1, 0) > 0
    with pytest.raises(B.MixkvError) as e:
        B.mixkv_decode_attention(p, caches, None, [q], 0, workspace=None)
    assert e.value.status == B.MIXKV_ERR_INVALID_ARG
    small = torch.empty(256, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(B.MixkvError) as e:
        B.mixkv_decode_attention(p, caches, None, [q], 0, workspace=small)
    assert e.value.status == B.MIXKV_ERR_WORKSPACE_TOO_SMALL


def test_bad_arguments_are_rejected_before_any_launch():
    wl = WL["c1"]
    p, caches = H.run_compress(wl, [synth.make_layer(wl, 0)])
    q = torch.zeros((wl.batch, wl.n_q_heads, wl.head_dim), device="cuda:0")
    for tail_len, tails in ((1, None), (-1, None)):
        with pytest.raises((B.MixkvError, AssertionError)) as e:
            B.mixkv_decode_attention(p, caches, tails, [q], tail_len)
        if isinstance(e.value, B.MixkvError):
            assert e.value.status == B.MIXKV_ERR_INVALID_ARG
    kt = torch.zeros((wl.batch, wl.n_kv_heads, 2, wl.head_dim), device="cuda:0")
    with pytest.raises(B.MixkvError) as e:                       # more rows than the tail holds
        B.mixkv_decode_attention(p, caches, [(kt, kt)], [q], 3)
    assert e.value.status == B.MIXKV_ERR_INVALID_ARG


def test_window_only_cache_and_single_row():
    wl = WL["c1"]
    _decode_and_check(wl, [0], 0, budget=wl.window)              # the cache holds the window rows only
    _decode_and_check(wl, [0], 1, budget=wl.window)
    tiny = WL["c1"].with_(name="tiny-dec", seq_len=2, window=1, budget=1, n_q_heads=1, n_kv_heads=1)
    _decode_and_check(tiny, [0], 0)                              # one row: the output is that value row


@pytest.mark.parametrize("name,over", [("c1", {}), ("c2", {}),
                                       ("c2", dict(seq_len=1024, text_suffix_start=960, batch=2, budget=96,
                                                   budget_mode="adaptive", budget_floor=16))])
def test_append_then_decode_token_by_token(name, over):
    """Three decoding steps on a compacted cache: every step appends the new token's rows with
    mixkv_append and attends with mixkv_decode_attention.  The tails must hold the appended rows
    bit for bit (and nothing else may change), the outputs must match the oracle on the grown cache."""
    wl = WL[name].with_(name="append", **over) if over else WL[name]
    layer_ids, steps, cap = [0, 1], 3, 5
    print(f"[case] append+decode {wl.name} dtype={wl.dtype} mode={wl.budget_mode} steps={steps} cap={cap}", flush=True)
    layers = [synth.make_layer(wl, l) for l in layer_ids]
    p, caches = H.run_compress(wl, layers)
    Bt, Hq, Hkv, D = wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim
    rng = np.random.default_rng([82, wl.cfg_id])
    fill = 3.0                                             # what the untouched tail rows must still hold at the end
    tails_host = [(np.full((Bt, Hkv, cap, D), fill, np.float32), np.full((Bt, Hkv, cap, D), -fill, np.float32)) for _ in layers]
    tails = [(H.to_device(wl, k), H.to_device(wl, v)) for k, v in tails_host]
    Bud = p.budget
    for t in range(steps):
        new_host = [(_quant(wl, rng.standard_normal((Bt, Hkv, D)) + 0.3), _quant(wl, rng.standard_normal((Bt, Hkv, D))))
                    for _ in layers]
        qs = [_quant(wl, rng.standard_normal((Bt, Hq, D)) / np.sqrt(D) * 4.0) for _ in layers]
        B.mixkv_append(p, [(H.to_device(wl, k), H.to_device(wl, v)) for k, v in new_host], tails, t)
        outs = B.mixkv_decode_attention(p, caches, tails, [H.to_device(wl, q) for q in qs], t + 1)
        torch.cuda.synchronize()
        for li, (lay, c) in enumerate(zip(layers, caches)):
            for b in range(Bt):                            # the oracle's copy of the same append
                O.append_token(tails_host[li][0][b], tails_host[li][1][b], new_host[li][0][b], new_host[li][1][b], t)
            for dev_t, host_t in zip(tails[li], tails_host[li]):
                assert np.array_equal(dev_t.float().cpu().numpy(), host_t), f"tail differs at step {t}, layer {li}"
            got = outs[li].float().cpu().numpy().astype(np.float64)
            idx = c.indices.cpu().numpy().reshape(Bt, Hkv * Bud)
            cnt, off = c.counts.cpu().numpy(), c.offsets.cpu().numpy()
            for b in range(Bt):
                Ks = [np.concatenate([_quant(wl, lay.K[b, h][idx[b, off[b, h]:off[b, h] + cnt[b, h]]]),
                                      tails_host[li][0][b, h, :t + 1]]) for h in range(Hkv)]
                Vs = [np.concatenate([_quant(wl, lay.V[b, h][idx[b, off[b, h]:off[b, h] + cnt[b, h]]]),
                                      tails_host[li][1][b, h, :t + 1]]) for h in range(Hkv)]
                want = O.decode_attention(qs[li][b], Ks, Vs, wl.softmax_scale)
                for g in range(Hq):
                    err = np.abs(got[b, g] - want[g]).max() / np.abs(want[g]).max()
                    assert err <= TOL[wl.dtype], f"step {t} layer {li} b{b} g{g}: error {err:.2e}"
