"""The synthetic caches hit the redundancy regimes the paper reports (Sec. 1, Fig. 1-2)."""
import numpy as np

from oracle import mixkv_oracle as O
from paper_2510_20707_amd import synth


def _rbar(K):
    return O.redundancy(O.normalised_keys(K))


def test_bf16_rounding_is_nearest_even_and_idempotent():
    x = np.array([1.0, 1.00390625, 1.01171875, -3.1415927, 1e-3, 65504.0], dtype=np.float32)
    b = synth.round_to_bf16_bits(x)
    y = synth.bf16_bits_to_f32(b)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7 -> even mantissa (1.0); 1 + 3*2^-8 ties up to 1 + 2^-6
    assert y[0] == 1.0 and y[1] == 1.0 and y[2] == 1.015625
    assert np.all(np.abs(y - x) <= np.abs(x) * 2.0 ** -8)
    np.testing.assert_array_equal(synth.round_to_bf16_bits(y), b)
    import torch
    t = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(b, t)


def test_same_seed_same_bits_and_values_fit_dtype():
    wl = synth.WORKLOADS["c2"].with_(seq_len=512, text_suffix_start=448)
    a, b = synth.make_layer(wl, 0), synth.make_layer(wl, 0)
    np.testing.assert_array_equal(a.K, b.K)
    np.testing.assert_array_equal(a.Q, b.Q)
    assert not np.array_equal(a.K, synth.make_layer(wl, 1).K)
    np.testing.assert_array_equal(synth.bf16_bits_to_f32(synth.round_to_bf16_bits(a.K)), a.K)
    assert a.K.shape == (1, 4, 512, 128) and a.Q.shape == (1, 28, 32, 128)


def test_redundancy_regimes():
    c1 = synth.make_layer(synth.WORKLOADS["c1"], 0)
    assert abs(_rbar(c1.K[0, 0])) < 0.01                        # i.i.d. keys: no redundancy
    c2 = synth.make_layer(synth.WORKLOADS["c2"], 0)
    vis = _rbar(c2.K[0, 0, 64:3648])
    txt = _rbar(c2.K[0, 0, 3648:])
    assert abs(vis - 0.70) < 0.05 and abs(txt - 0.30) < 0.05
    c4 = synth.WORKLOADS["c4"].with_(seq_len=4096)
    assert abs(_rbar(synth.make_layer(c4, 0).K[0, 0]) - 0.002) < 0.003
    # c3: per-head noise level spreads the redundancy across heads
    c3 = synth.WORKLOADS["c3"].with_(seq_len=2048, text_suffix_start=1984)
    rs = [_rbar(synth.make_layer(c3, l).K[0, h]) for l in range(3) for h in range(4)]
    assert 0.35 < min(rs) < max(rs) < 0.85 and max(rs) - min(rs) > 0.1


def test_window_lse_stand_in_matches_a_library_logsumexp():
    from scipy.special import logsumexp
    wl = synth.WORKLOADS["c1"]
    lay = synth.make_layer(wl, 0)
    nc = wl.seq_len - wl.window
    for causal in (True, False):
        got = synth.window_lse(wl, lay, causal)
        assert got.dtype == np.float32 and got.shape == (wl.batch, wl.n_q_heads, wl.window)
        for g in (0, 3):
            for w in (0, wl.window - 1):
                n = nc + w + 1 if causal else wl.seq_len
                s = wl.softmax_scale * (lay.Q[0, g, w].astype(np.float64) @ lay.K[0, g // wl.group, :n].astype(np.float64).T)
                assert abs(float(got[0, g, w]) - logsumexp(s)) < 1e-5
