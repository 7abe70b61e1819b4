"""Pins for the CPU oracle: brute force, closed forms, library routines, invariants.

None of these retype the oracle's own formulas: each expected value comes from
the definition written out in tests/brute.py, from a closed form derived by
hand, or from an independent library routine (torch CPU softmax / pooling).
"""
import json
import math
import os

import numpy as np
import pytest
import torch

from oracle import mixkv_oracle as O
from tests import brute

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_unit(seed, N=24, D=8, G=2, W=3, kscale=1.0, offset=0.0):
    rng = np.random.default_rng(seed)
    K = rng.standard_normal((N, D)) * kscale + offset
    V = rng.standard_normal((N, D))
    Q = rng.standard_normal((G, W, D))
    return K, V, Q


def _params(G=2, W=3, B=8, **kw):
    base = dict(n_q_heads=G, n_kv_heads=1, window=W, budget=B, pool="none", pool_kernel=1,
                softmax_scale=0.5)
    base.update(kw)
    return O.Params(**base)


# ------------------------------------------------------------------ attention (Sec. 3.2, extrinsic)

@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("seed", [0, 1])
def test_window_attention_matches_brute_force(seed, causal):
    K, V, Q = _rand_unit(seed)
    W = Q.shape[1]
    Nc = K.shape[0] - W
    want = brute.window_mean_attention(K.tolist(), Q.tolist(), 0.5, causal)
    P = O.window_attention(K, Q, 0.5, causal)
    got = P.sum(axis=(0, 1)) / (Q.shape[0] * W)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-15)
    p = _params(causal_window=causal)
    np.testing.assert_allclose(O.extrinsic_importance(K, Q, p), want[:Nc], rtol=1e-12, atol=1e-15)


def test_attention_rows_sum_to_one_and_mask_is_causal():
    K, V, Q = _rand_unit(3)
    W = Q.shape[1]
    Nc = K.shape[0] - W
    P = O.window_attention(K, Q, 1.0, True)
    np.testing.assert_allclose(P.sum(axis=2), 1.0, rtol=1e-13)
    for w in range(W):
        assert np.all(P[:, w, Nc + w + 1:] == 0.0)
        assert np.all(P[:, w, :Nc + w + 1] > 0.0)


def test_zero_queries_closed_form():
    # uniform attention: causal row w spreads 1 over Nc+w+1 keys, non-causal over N
    K, V, _ = _rand_unit(4, N=40, D=8)
    G, W = 3, 5
    Nc = 40 - W
    Q = np.zeros((G, W, 8))
    got = O.extrinsic_importance(K, Q, _params(G=G, W=W, B=10, causal_window=True))
    want = sum(1.0 / (Nc + w + 1) for w in range(W)) / W
    np.testing.assert_allclose(got, want, rtol=1e-13)
    got = O.extrinsic_importance(K, Q, _params(G=G, W=W, B=10, causal_window=False))
    np.testing.assert_allclose(got, 1.0 / 40, rtol=1e-13)


def test_single_group_matches_torch_softmax():
    K, V, Q = _rand_unit(5, N=64, D=16, G=1, W=4)
    scale = 1.0 / math.sqrt(16)
    logits = torch.from_numpy(Q[0]) @ torch.from_numpy(K).T * scale
    want = torch.softmax(logits, dim=-1).mean(dim=0).numpy()[:60]
    got = O.extrinsic_importance(K, Q, _params(G=1, W=4, B=8, causal_window=False, softmax_scale=scale))
    np.testing.assert_allclose(got, want, rtol=1e-12)


def test_gqa_group_is_mean_of_single_head_results():
    K, V, Q = _rand_unit(6, G=4)
    p1 = _params(G=1)
    singles = [O.extrinsic_importance(K, Q[g:g + 1], p1) for g in range(4)]
    got = O.extrinsic_importance(K, Q, _params(G=4))
    np.testing.assert_allclose(got, np.mean(singles, axis=0), rtol=1e-13)


# ------------------------------------------------------------------ pooling

@pytest.mark.parametrize("k", [1, 3, 7])
def test_pooling_matches_torch_and_brute(k):
    rng = np.random.default_rng(7)
    a = rng.random(50)
    t = torch.from_numpy(a)[None, None]
    want_max = torch.nn.functional.max_pool1d(t, k, stride=1, padding=k // 2)[0, 0].numpy()
    want_avg = torch.nn.functional.avg_pool1d(t, k, stride=1, padding=k // 2, count_include_pad=True)[0, 0].numpy()
    np.testing.assert_array_equal(O.pool1d(a, "max", k), want_max)
    np.testing.assert_allclose(O.pool1d(a, "avg", k), want_avg, rtol=1e-14)
    np.testing.assert_array_equal(O.pool1d(a, "max", k), brute.pool(a.tolist(), "max", k))
    np.testing.assert_allclose(O.pool1d(a, "avg", k), brute.pool(a.tolist(), "avg", k), rtol=1e-14)
    np.testing.assert_array_equal(O.pool1d(a, "none", k), a)


def test_pooling_sees_candidates_only():
    # a huge attention weight on a window key must not leak into the last candidates
    K, V, Q = _rand_unit(8, N=32, D=8, G=1, W=4)
    K[28:] = 10.0 * Q[0]            # window keys line up with the window queries
    p = _params(G=1, W=4, pool="max", pool_kernel=7, softmax_scale=1.0)
    P = O.window_attention(K, Q, 1.0, True)
    a = P[:, :, :28].mean(axis=(0, 1))
    np.testing.assert_array_equal(O.extrinsic_importance(K, Q, p), brute.pool(a.tolist(), "max", 7))


# ------------------------------------------------------------------ redundancy (Sec. 3.3, Eq. 3-4)

@pytest.mark.parametrize("seed,offset", [(0, 0.0), (1, 1.0), (2, 3.0)])
def test_redundancy_equals_offdiagonal_mean_of_cosine_matrix(seed, offset):
    K, _, _ = _rand_unit(seed, N=20, D=6, offset=offset)
    R = brute.cosine_matrix(K.tolist())
    want = brute.offdiag_mean(R)
    got = O.redundancy(O.normalised_keys(K))
    assert abs(got - want) < 1e-13


def test_redundancy_closed_forms():
    with open(os.path.join(GOLDEN, "redundancy_closed_forms.json")) as f:
        cases = json.load(f)["cases"]
    for c in cases:
        K = np.array(c["K"], dtype=np.float64)
        got = O.redundancy(O.normalised_keys(K))
        assert abs(got - eval(c["expect"], {"T": K.shape[0]})) < 1e-14, c["name"]


def test_redundancy_offset_gaussian_estimate():
    # keys mu + z, z ~ N(0, I_D): E cos ~ |mu|^2 / (|mu|^2 + D)
    rng = np.random.default_rng(9)
    D, N = 128, 4000
    mu = np.zeros(D)
    mu[0] = 7.4
    K = mu + rng.standard_normal((N, D))
    got = O.redundancy(O.normalised_keys(K))
    assert abs(got - 7.4 ** 2 / (7.4 ** 2 + D)) < 0.01


def test_key_rescaling_leaves_redundancy_and_diversity_unchanged():
    K, _, _ = _rand_unit(10, N=30, D=8, offset=0.7)
    c = np.random.default_rng(1).uniform(0.1, 9.0, size=(30, 1))
    a, b = O.normalised_keys(K), O.normalised_keys(K * c)
    assert abs(O.redundancy(a) - O.redundancy(b)) < 1e-14
    np.testing.assert_allclose(O.diversity(a), O.diversity(b), rtol=1e-12, atol=1e-15)


def test_zero_key_normalises_to_zero_vector():
    K = np.eye(4)
    K[2] = 0.0
    Kh = O.normalised_keys(K)
    assert np.all(Kh[2] == 0.0) and np.all(np.isfinite(Kh))


# ------------------------------------------------------------------ diversity (Sec. 3.2)

def test_diversity_is_affine_in_mean_cosine_to_the_other_keys():
    # c_i = mean_{j != i} cos(K_i, K_j) = (T * Khat_i.Kbar - 1)/(T - 1)  =>  s_div_i = -((T-1) c_i + 1)/T
    K, _, _ = _rand_unit(11, N=18, D=5, offset=0.5)
    T = 18
    c = np.array(brute.mean_cos_to_others(brute.cosine_matrix(K.tolist())))
    got = O.diversity(O.normalised_keys(K))
    np.testing.assert_allclose(got, -((T - 1) * c + 1.0) / T, rtol=1e-12)
    # hence the min-max normalised diversity equals the min-max normalised dissimilarity (eps -> 0)
    np.testing.assert_allclose(O.minmax(got, 0.0), O.minmax(-c, 0.0), rtol=1e-10, atol=1e-12)


def test_diversity_sign_outlier_scores_highest():
    K = np.tile(np.array([1.0, 0.1, 0.0]), (10, 1))
    K[4] = [-1.0, 0.3, 0.2]
    s = O.diversity(O.normalised_keys(K))
    assert np.argmax(s) == 4 and s[4] > 0 > s[0]


# ------------------------------------------------------------------ scaling + mixing (Sec. 3.2, 3.3, Eq. 2, Eq. 5)

def test_minmax_and_mean_matching_invariants():
    K, V, Q = _rand_unit(12, N=40, D=8)
    p = _params(B=10)
    u = O.score_unit(K, V, Q, p)
    eps = p.eps
    vn = [math.sqrt(brute.dot(v, v)) for v in V[:37].tolist()]
    s_in_norm = [(x - min(vn)) / (max(vn) - min(vn) + eps) for x in vn]
    m = sum(s_in_norm) / len(s_in_norm)
    ex_mean = float(np.mean(u["s_ex"]))
    want = [x * ex_mean / (m + eps) for x in s_in_norm]
    np.testing.assert_allclose(u["s_in_scaled"], want, rtol=1e-12, atol=1e-18)
    assert u["s_in_scaled"].min() == 0.0
    np.testing.assert_allclose(u["s_in_scaled"].mean(), ex_mean * m / (m + eps), rtol=1e-12)
    np.testing.assert_allclose(u["s_imp"], u["s_ex"] + u["s_in_scaled"], rtol=0, atol=0)
    # diversity: min exactly 0, max < 1, mean matched to mean(s_imp)
    dmin, dmax = u["s_div"].min(), u["s_div"].max()
    dn = (u["s_div"] - dmin) / (dmax - dmin + eps)
    b = dn.mean()
    np.testing.assert_allclose(u["s_div_scaled"], dn * u["s_imp"].mean() / (b + eps), rtol=1e-12, atol=1e-18)
    assert u["s_div_scaled"].min() == 0.0 and dn.max() < 1.0
    # Eq. 5
    r = float(u["r"])
    np.testing.assert_allclose(u["s_comp"], (1 - r) * u["s_imp"] + r * u["s_div_scaled"], rtol=1e-14)
    # V rescaling leaves the normalised VNorm unchanged up to eps
    u2 = O.score_unit(K, 3.0 * V, Q, p)
    np.testing.assert_allclose(u2["s_in_scaled"], u["s_in_scaled"], rtol=1e-5)


def test_mix_weights_are_one_minus_r_and_r():
    # Two units with identical importance inputs (same Q.K logits pattern is not needed here):
    # check s_comp against a hand mix for a head whose redundancy is known in closed form.
    rng = np.random.default_rng(13)
    D, N, W = 6, 26, 2
    K = np.abs(rng.standard_normal((N, D))) + 2.0       # clearly redundant head
    V = rng.standard_normal((N, D))
    Q = rng.standard_normal((1, W, D))
    p = _params(G=1, W=W, B=6)
    u = O.score_unit(K, V, Q, p)
    r = brute.offdiag_mean(brute.cosine_matrix(K.tolist()))
    assert 0.5 < r < 1.0
    np.testing.assert_allclose(u["s_comp"], (1 - r) * u["s_imp"] + r * u["s_div_scaled"], rtol=1e-11)


def test_limit_identical_keys_all_ties_select_smallest_indices():
    # r = 1 and constant diversity => s_comp == 0 everywhere => ties => lowest indices win
    rng = np.random.default_rng(14)
    N, D, W = 32, 8, 4
    K = np.tile(rng.standard_normal(D), (N, 1))
    V = rng.standard_normal((N, D))
    Q = rng.standard_normal((2, W, D))
    p = _params(G=2, W=W, B=10)
    u = O.score_unit(K, V, Q, p)
    assert abs(float(u["r"]) - 1.0) < 1e-12
    assert np.all(np.abs(u["s_comp"]) < 1e-9 * np.abs(u["s_imp"]).max() + 1e-15)
    idx = O.select_unit(np.zeros(N - W), 6, N, W)
    np.testing.assert_array_equal(idx, list(range(6)) + list(range(28, 32)))


def test_limit_zero_redundancy_reduces_to_importance_topk():
    # orthonormal keys: r = 0 exactly => s_comp = s_imp; with intrinsic off this is softmax + pool + top-k
    N = D = 16
    W = 2
    K = np.eye(N)
    rng = np.random.default_rng(15)
    V = rng.standard_normal((N, D))
    Q = rng.standard_normal((1, W, D))
    p = _params(G=1, W=W, B=6, intrinsic="none", pool="max", pool_kernel=3, causal_window=False,
                softmax_scale=1.0)
    u = O.score_unit(K, V, Q, p)
    assert abs(float(u["r"])) < 1e-15
    attn = torch.softmax(torch.from_numpy(Q[0]) @ torch.from_numpy(K).T, dim=-1).mean(0)[:N - W]
    pooled = torch.nn.functional.max_pool1d(attn[None, None], 3, stride=1, padding=1)[0, 0]
    np.testing.assert_allclose(u["s_comp"], pooled.numpy(), rtol=1e-12)
    want = torch.topk(pooled, 4).indices.sort().values.numpy()
    np.testing.assert_array_equal(O.select_unit(u["s_comp"], 4, N, W)[:4], want)


# ------------------------------------------------------------------ selection / budgets / whole layer

@pytest.mark.parametrize("seed", [0, 1, 2])
def test_top_indices_matches_full_sort_with_ties(seed):
    rng = np.random.default_rng(seed)
    s = rng.integers(0, 6, size=40).astype(np.float64)     # many exact ties
    for b in [0, 1, 7, 39, 40]:
        np.testing.assert_array_equal(O.top_indices(s, b), brute.topk_sorted(s.tolist(), b))


def _brute_adaptive(s_heads, bp, floor):
    Hkv, Nc = len(s_heads), len(s_heads[0])
    kept = [set(brute.topk_sorted(s_heads[h], floor)) for h in range(Hkv)]
    rest = [(-s_heads[h][i], h, i) for h in range(Hkv) for i in range(Nc) if i not in kept[h]]
    rest.sort()
    for _, h, i in rest[:Hkv * (bp - floor)]:
        kept[h].add(i)
    return kept


@pytest.mark.parametrize("seed", [0, 1])
def test_adaptive_budgets_match_brute_force(seed):
    rng = np.random.default_rng(seed)
    Hkv, Nc, B, W, floor = 3, 50, 14, 2, 3
    s = rng.standard_normal((Hkv, Nc)) * np.array([[1.0], [2.0], [0.5]])
    s[1, 5] = s[0, 9]                                        # a cross-head tie
    counts = O.adaptive_budgets(s, B, W, floor)
    kept = _brute_adaptive(s.tolist(), B - W, floor)
    assert counts.sum() == Hkv * (B - W) and counts.min() >= floor
    for h in range(Hkv):
        assert counts[h] == len(kept[h])
        # each head's kept set is its own top-b'_h
        assert set(O.top_indices(s[h], int(counts[h])).tolist()) == kept[h]


@pytest.mark.parametrize("mode", ["fixed", "adaptive"])
def test_compress_layer_invariants(mode):
    rng = np.random.default_rng(20)
    Bt, Hq, Hkv, N, D, W, B = 2, 4, 2, 48, 8, 4, 12
    K = rng.standard_normal((Bt, Hkv, N, D)) + 0.5
    V = rng.standard_normal((Bt, Hkv, N, D))
    Q = rng.standard_normal((Bt, Hq, W, D))
    p = O.Params(Hq, Hkv, W, B, pool="max", pool_kernel=3, budget_mode=mode, budget_floor=2)
    out = O.compress_layer(K, V, Q, p)
    assert np.all(np.isinf(out["scores"][:, :, N - W:])) and np.all(np.isfinite(out["scores"][:, :, :N - W]))
    for b in range(Bt):
        assert out["counts"][b].sum() == Hkv * B
        for h in range(Hkv):
            idx = out["indices"][b][h]
            assert len(set(idx.tolist())) == idx.shape[0] == out["counts"][b, h]
            assert np.all(np.diff(idx) > 0) and idx.min() >= 0 and idx.max() == N - 1
            np.testing.assert_array_equal(idx[-W:], np.arange(N - W, N))
            if mode == "fixed":
                assert idx.shape[0] == B
            else:
                assert idx.shape[0] >= W + 2
            np.testing.assert_array_equal(out["K_out"][b][h], K[b, h][idx])
            np.testing.assert_array_equal(out["V_out"][b][h], V[b, h][idx])
            # kept candidates beat every dropped candidate (ties to the smaller index)
            s = out["scores"][b, h, :N - W]
            kept = idx[:-W]
            dropped = np.setdiff1d(np.arange(N - W), kept)
            if kept.size and dropped.size:
                worst = min((s[i], -i) for i in kept)
                best = max((s[i], -i) for i in dropped)
                assert worst > best
            # group mapping: head h must use query heads [h*G, (h+1)*G)
            G = Hq // Hkv
            u = O.score_unit(K[b, h], V[b, h], Q[b, h * G:(h + 1) * G], p)
            np.testing.assert_array_equal(out["scores"][b, h, :N - W], u["s_comp"])
        np.testing.assert_array_equal(out["offsets"][b], np.concatenate([[0], np.cumsum(out["counts"][b])]))


def test_permutation_equivariance_without_pooling():
    K, V, Q = _rand_unit(21, N=30, D=8, G=2, W=3)
    p = _params(causal_window=False, B=9)
    u = O.score_unit(K, V, Q, p)
    perm = np.random.default_rng(2).permutation(27)
    full = np.concatenate([perm, np.arange(27, 30)])
    u2 = O.score_unit(K[full], V[full], Q, p)
    np.testing.assert_allclose(u2["s_comp"], u["s_comp"][perm], rtol=1e-10, atol=1e-16)


@pytest.mark.parametrize("seed,pool,causal,vnorm", [(0, "max", True, True), (1, "avg", False, True),
                                                    (2, "none", True, False), (3, "max", True, True)])
def test_score_unit_matches_brute_force_chain(seed, pool, causal, vnorm):
    K, V, Q = _rand_unit(seed, N=28, D=6, G=2, W=3, offset=0.8)
    p = _params(B=9, pool=pool, pool_kernel=5, causal_window=causal, softmax_scale=0.7,
                intrinsic="vnorm" if vnorm else "none")
    want, r = brute.mixkv_scores(K.tolist(), V.tolist(), Q.tolist(), 0.7, causal, pool, 5, p.eps, vnorm)
    u = O.score_unit(K, V, Q, p)
    assert abs(float(u["r"]) - r) < 1e-13
    np.testing.assert_allclose(u["s_comp"], want, rtol=1e-10, atol=1e-16)
    np.testing.assert_array_equal(O.select_unit(u["s_comp"], 6, 28, 3)[:6], brute.topk_sorted(want, 6))


# ------------------------------------------------------------------ ablation variants (Sec. 4.3, Table 4)

@pytest.mark.parametrize("intrinsic", ["vnorm", "knorm", "none"])
@pytest.mark.parametrize("mix,rg", [("sum", None), ("div_only", None), ("imp_only", None), ("given_r", 0.37),
                                    ("head_adaptive", None)])
def test_variants_match_brute_force_chain(intrinsic, mix, rg):
    K, V, Q = _rand_unit(31, N=26, D=6, G=2, W=3, offset=0.6)
    K *= np.linspace(0.5, 2.0, 26)[:, None]              # spread the key norms
    p = _params(B=9, pool="max", pool_kernel=3, softmax_scale=0.7, intrinsic=intrinsic, mix=mix)
    want, r = brute.mixkv_scores(K.tolist(), V.tolist(), Q.tolist(), 0.7, True, "max", 3, p.eps,
                                 intrinsic=intrinsic, mix=mix, r_given=rg)
    u = O.score_unit(K, V, Q, p, rg)
    assert abs(float(u["r"]) - r) < 1e-13                # the head's own redundancy is reported in every mode
    np.testing.assert_allclose(u["s_comp"], want, rtol=1e-10, atol=1e-16)


def test_given_r_limits_and_sum_decomposition():
    K, V, Q = _rand_unit(32, N=30, D=8, G=2, W=3, offset=0.5)
    base = dict(B=9, pool="avg", pool_kernel=3)
    ha = O.score_unit(K, V, Q, _params(**base))
    imp = O.score_unit(K, V, Q, _params(mix="imp_only", **base))["s_comp"]
    div = O.score_unit(K, V, Q, _params(mix="div_only", **base))["s_comp"]
    tot = O.score_unit(K, V, Q, _params(mix="sum", **base))["s_comp"]
    g = _params(mix="given_r", **base)
    np.testing.assert_array_equal(O.score_unit(K, V, Q, g, 0.0)["s_comp"], imp)
    np.testing.assert_array_equal(O.score_unit(K, V, Q, g, 1.0)["s_comp"], div)
    np.testing.assert_array_equal(O.score_unit(K, V, Q, g, float(ha["r"]))["s_comp"], ha["s_comp"])
    np.testing.assert_allclose(tot, imp + div, rtol=1e-15)
    np.testing.assert_array_equal(imp, ha["s_imp"])
    # diversity alone: mean matched to the importance, smallest exactly zero, ranking that of s_div
    np.testing.assert_allclose(div.mean(), imp.mean(), rtol=1e-4)
    assert div.min() == 0.0
    np.testing.assert_array_equal(np.argsort(-div, kind="stable"), np.argsort(-ha["s_div"], kind="stable"))
    # importance alone with the intrinsic score off is the pooled window attention
    ex = O.score_unit(K, V, Q, _params(mix="imp_only", intrinsic="none", **base))
    np.testing.assert_array_equal(ex["s_comp"], ex["s_ex"])


def test_knorm_equals_vnorm_on_values_with_mirrored_norms():
    # min-max of -||K_i|| equals min-max of C - ||K_i||: feed the VNorm path values whose norms are
    # C - ||K_i|| and both intrinsic terms must agree.
    K, V, Q = _rand_unit(33, N=28, D=8, G=2, W=3)
    K *= np.linspace(0.3, 3.0, 28)[:, None]
    kn = np.sqrt((K * K).sum(axis=1))
    C = kn.max() + 1.0
    Vm = np.zeros_like(V)
    Vm[:, 2] = C - kn
    p = _params(B=9, pool="max", pool_kernel=3)
    a = O.score_unit(K, V, Q, _params(B=9, pool="max", pool_kernel=3, intrinsic="knorm"))
    b = O.score_unit(K, Vm, Q, p)
    np.testing.assert_allclose(a["s_in_scaled"], b["s_in_scaled"], rtol=1e-12, atol=1e-18)
    np.testing.assert_allclose(a["s_comp"], b["s_comp"], rtol=1e-12, atol=1e-18)
    # the longest candidate key gets no intrinsic credit, the shortest the most
    Nc = 25
    assert a["s_in_scaled"][np.argmax(kn[:Nc])] == 0.0
    assert np.argmax(a["s_in_scaled"]) == np.argmin(kn[:Nc])
    # scaling all keys by c > 0 changes neither the cosine terms nor (up to eps) the KNorm term;
    # the attention does change, so compare the intrinsic term relative to its own mean
    a2 = O.score_unit(2.0 * K, V, Q, _params(B=9, pool="max", pool_kernel=3, intrinsic="knorm"))
    np.testing.assert_allclose(a2["s_in_scaled"] / a2["s_ex"].mean(), a["s_in_scaled"] / a["s_ex"].mean(), rtol=1e-5)
    np.testing.assert_allclose(a2["s_div"], a["s_div"], rtol=1e-12)


def test_compress_layer_passes_given_r_per_unit():
    rng = np.random.default_rng(34)
    Bt, Hq, Hkv, N, D, W, B = 2, 4, 2, 24, 8, 3, 8
    K = rng.standard_normal((Bt, Hkv, N, D)) + 0.5
    V = rng.standard_normal((Bt, Hkv, N, D))
    Q = rng.standard_normal((Bt, Hq, W, D))
    rg = rng.uniform(0, 1, (Bt, Hkv))
    p = O.Params(Hq, Hkv, W, B, pool="max", pool_kernel=3, mix="given_r")
    out = O.compress_layer(K, V, Q, p, rg)
    for b in range(Bt):
        for h in range(Hkv):
            want, r = brute.mixkv_scores(K[b, h].tolist(), V[b, h].tolist(), Q[b, 2 * h:2 * h + 2].tolist(), 1.0, True,
                                         "max", 3, p.eps, mix="given_r", r_given=float(rg[b, h]))
            np.testing.assert_allclose(out["scores"][b, h, :N - W], want, rtol=1e-10, atol=1e-16)
            assert abs(out["redundancy"][b, h] - r) < 1e-13
            np.testing.assert_array_equal(out["indices"][b][h][:B - W], brute.topk_sorted(want, B - W))


# ------------------------------------------------------------------ budgets given per layer and head

def test_per_head_budgets_are_independent_fixed_selections():
    rng = np.random.default_rng(41)
    Bt, Hq, Hkv, N, D, W = 2, 6, 3, 40, 8, 4
    K = rng.standard_normal((Bt, Hkv, N, D)) + 0.4
    V = rng.standard_normal((Bt, Hkv, N, D))
    Q = rng.standard_normal((Bt, Hq, W, D))
    hb = np.array([4, 17, 40])                            # window only / some / everything
    p = O.Params(Hq, Hkv, W, 20, pool="max", pool_kernel=3, budget_mode="per_head")
    out = O.compress_layer(K, V, Q, p, head_budgets=hb)
    np.testing.assert_array_equal(out["counts"], np.tile(hb, (Bt, 1)))
    for b in range(Bt):
        np.testing.assert_array_equal(out["offsets"][b], [0, 4, 21, 61])
        for h in range(Hkv):
            want, _ = brute.mixkv_scores(K[b, h].tolist(), V[b, h].tolist(), Q[b, 2 * h:2 * h + 2].tolist(), 1.0, True,
                                         "max", 3, p.eps)
            idx = out["indices"][b][h]
            np.testing.assert_array_equal(idx[:hb[h] - W], brute.topk_sorted(want, int(hb[h]) - W))
            np.testing.assert_array_equal(idx[hb[h] - W:], np.arange(N - W, N))
            np.testing.assert_array_equal(out["K_out"][b][h], K[b, h][idx])
            np.testing.assert_array_equal(out["V_out"][b][h], V[b, h][idx])
            # a head's result is the fixed-budget result at its own budget
            fixed = O.compress_layer(K, V, Q, O.Params(Hq, Hkv, W, int(hb[h]), pool="max", pool_kernel=3))
            np.testing.assert_array_equal(idx, fixed["indices"][b][h])


def test_per_head_budgets_nest():
    # the candidates kept at budget b are among those kept at budget b + 1
    K, V, Q = _rand_unit(42, N=30, D=8, G=2, W=3)
    p = O.Params(2, 1, 3, 10, budget_mode="per_head")
    prev = set()
    for b in range(3, 31):
        out = O.compress_layer(K[None, None], V[None, None], Q[None], p, head_budgets=np.array([b]))
        cur = set(out["indices"][0][0].tolist())
        assert len(cur) == b and prev <= cur
        prev = cur


# ------------------------------------------------------------------ redundancy analysis (similarity heat-maps)

@pytest.mark.parametrize("N,block", [(13, 4), (16, 4), (9, 16)])
def test_similarity_analysis_matches_brute_force_matrix(N, block):
    rng = np.random.default_rng(51)
    X = rng.standard_normal((N, 5)) + 0.7
    R = brute.cosine_matrix(X.tolist())
    out = O.similarity_analysis(X, block)
    assert abs(float(out["redundancy"]) - brute.offdiag_mean(R)) < 1e-13
    nb = -(-N // block)
    assert out["block_map"].shape == (nb, nb)
    for a in range(nb):
        for b in range(nb):
            cells = [R[i][j] for i in range(a * block, min(N, (a + 1) * block))
                     for j in range(b * block, min(N, (b + 1) * block))]
            assert abs(out["block_map"][a, b] - sum(cells) / len(cells)) < 1e-13
    np.testing.assert_allclose(out["block_map"], out["block_map"].T, rtol=0, atol=1e-15)


def test_similarity_analysis_closed_forms():
    # identical rows: every similarity is 1; orthonormal rows: R is the identity, so a diagonal
    # block of b rows averages 1/b; the same value as Eq. 4 through the keys' own routine
    X = np.tile(np.array([0.3, -1.0, 2.0]), (12, 1))
    out = O.similarity_analysis(X, 4)
    np.testing.assert_allclose(out["block_map"], 1.0, rtol=1e-14)
    assert abs(float(out["redundancy"]) - 1.0) < 1e-14
    out = O.similarity_analysis(np.eye(12) * 3.0, 4)
    np.testing.assert_allclose(out["block_map"], np.eye(3) / 4.0, atol=1e-15)
    assert abs(float(out["redundancy"])) < 1e-15
    K, _, _ = _rand_unit(52, N=40, D=8, offset=0.5)
    assert abs(float(O.similarity_analysis(K, 8)["redundancy"]) - O.redundancy(O.normalised_keys(K))) < 1e-13
    # block size 1 is the cosine matrix itself; one block covering everything is its overall mean
    R = np.array(brute.cosine_matrix(K.tolist()))
    np.testing.assert_allclose(O.similarity_analysis(K, 1)["block_map"], R, atol=1e-13)
    np.testing.assert_allclose(O.similarity_analysis(K, 64)["block_map"], [[R.mean()]], atol=1e-13)


# ------------------------------------------------------------------ log-sum-exp handed in by the caller

@pytest.mark.parametrize("causal", [True, False])
def test_given_lse_reproduces_the_softmax_and_is_actually_used(causal):
    from scipy.special import logsumexp
    K, V, Q = _rand_unit(61, N=26, D=8, G=2, W=3)
    N, W = 26, 3
    logits = 0.5 * np.einsum("gwd,nd->gwn", Q, K)
    lse = np.empty((2, W))
    for w in range(W):
        hi = N - W + w + 1 if causal else N
        lse[:, w] = logsumexp(logits[:, w, :hi], axis=1)       # library routine over the visible keys
    P = O.window_attention(K, Q, 0.5, causal)
    P2 = O.window_attention(K, Q, 0.5, causal, lse)
    np.testing.assert_allclose(P2, P, rtol=1e-12, atol=1e-300)
    p = _params(B=8, causal_window=causal, pool="max", pool_kernel=3)
    a, b = O.score_unit(K, V, Q, p), O.score_unit(K, V, Q, p, lse=lse)
    np.testing.assert_allclose(b["s_comp"], a["s_comp"], rtol=1e-11)
    # a normaliser larger by ln 2 halves every weight: the given value is what normalises
    np.testing.assert_allclose(O.window_attention(K, Q, 0.5, causal, lse + math.log(2.0)), 0.5 * P, rtol=1e-12)
    want = brute.window_mean_attention(K.tolist(), Q.tolist(), 0.5, causal)
    np.testing.assert_allclose(O.extrinsic_importance(K, Q, _params(causal_window=causal), lse), want[:N - W], rtol=1e-11)


def test_compress_layer_maps_given_lse_to_the_heads_of_each_group():
    from scipy.special import logsumexp
    rng = np.random.default_rng(62)
    Bt, Hq, Hkv, N, D, W, B = 2, 4, 2, 24, 8, 3, 8
    K = rng.standard_normal((Bt, Hkv, N, D)) + 0.5
    V = rng.standard_normal((Bt, Hkv, N, D))
    Q = rng.standard_normal((Bt, Hq, W, D))
    lse = np.empty((Bt, Hq, W))
    for b in range(Bt):
        for g in range(Hq):
            for w in range(W):
                lse[b, g, w] = logsumexp(Q[b, g, w] @ K[b, g // 2, :N - W + w + 1].T)
    p = O.Params(Hq, Hkv, W, B, pool="max", pool_kernel=3)
    a, c = O.compress_layer(K, V, Q, p), O.compress_layer(K, V, Q, p, window_lse=lse)
    np.testing.assert_allclose(c["scores"][:, :, :N - W], a["scores"][:, :, :N - W], rtol=1e-11)
    for b in range(Bt):
        for h in range(Hkv):
            np.testing.assert_array_equal(c["indices"][b][h], a["indices"][b][h])


# ------------------------------------------------------------------ decoding on the compacted cache

def test_decode_attention_matches_library_attention_on_ragged_heads():
    rng = np.random.default_rng(71)
    Hq, Hkv, D = 6, 3, 8
    q = rng.standard_normal((Hq, D))
    lens = [5, 1, 17]
    Ks = [rng.standard_normal((n, D)) for n in lens]
    Vs = [rng.standard_normal((n, D)) for n in lens]
    out = O.decode_attention(q, Ks, Vs, 0.35)
    for g in range(Hq):
        h = g // 2
        want = torch.nn.functional.scaled_dot_product_attention(
            torch.from_numpy(q[g])[None, None], torch.from_numpy(Ks[h])[None], torch.from_numpy(Vs[h])[None], scale=0.35)
        np.testing.assert_allclose(out[g], want[0, 0].numpy(), rtol=1e-12, atol=1e-14)
        # and the definition with plain loops
        lg = [0.35 * brute.dot(q[g].tolist(), k) for k in Ks[h].tolist()]
        w = brute.softmax_row(lg)
        ref = [sum(w[j] * Vs[h][j][d] for j in range(lens[h])) for d in range(D)]
        np.testing.assert_allclose(out[g], ref, rtol=1e-12, atol=1e-14)


def test_decode_attention_closed_forms():
    rng = np.random.default_rng(72)
    D = 6
    q = rng.standard_normal((2, D))
    V = rng.standard_normal((9, D))
    same = np.tile(rng.standard_normal(D), (9, 1))
    out = O.decode_attention(q, [same], [V], 1.0)             # equal logits: the plain mean of the values
    np.testing.assert_allclose(out, np.tile(V.mean(axis=0), (2, 1)), rtol=1e-12)
    K = rng.standard_normal((9, D))
    K[4] = 50.0 * q[0] / np.linalg.norm(q[0])                 # one key far ahead for query 0: its value wins
    out = O.decode_attention(q[:1], [K], [V], 1.0)
    np.testing.assert_allclose(out[0], V[4], atol=1e-9)
    out1 = O.decode_attention(q, [K[:1]], [V[:1]], 3.0)       # a single row: its value, whatever the logit
    np.testing.assert_allclose(out1, np.tile(V[0], (2, 1)), rtol=1e-14)


def test_append_token_fills_rows_in_order_and_touches_nothing_else():
    # appending t tokens one by one gives the tail whose first t rows are the tokens in order
    # (numpy's stack is the independent statement of that), later rows keep what they held
    rng = np.random.default_rng(44)
    Hkv, cap, D, t = 3, 6, 8, 4
    Kt, Vt = np.full((Hkv, cap, D), 7.0), np.full((Hkv, cap, D), -7.0)
    ks, vs = rng.standard_normal((t, Hkv, D)), rng.standard_normal((t, Hkv, D))
    for j in range(t):
        O.append_token(Kt, Vt, ks[j], vs[j], j)
    assert np.array_equal(Kt[:, :t], np.stack(list(ks), axis=1)) and np.array_equal(Vt[:, :t], np.stack(list(vs), axis=1))
    assert np.all(Kt[:, t:] == 7.0) and np.all(Vt[:, t:] == -7.0)
    with pytest.raises(ValueError):
        O.append_token(Kt, Vt, ks[0], vs[0], cap)
    with pytest.raises(ValueError):
        O.append_token(Kt, Vt, ks[0], vs[0], -1)
    # attention over the grown cache: a token appended with a very large logit takes all the weight
    q = np.zeros((Hkv, D)); q[:, 0] = 1.0
    big = np.zeros((Hkv, D)); big[:, 0] = 200.0
    O.append_token(Kt, Vt, big, vs[0], t)
    out = O.decode_attention(q, [Kt[h, :t + 1] for h in range(Hkv)], [Vt[h, :t + 1] for h in range(Hkv)], 1.0)
    assert np.allclose(out, vs[0], atol=1e-12)
