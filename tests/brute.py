"""Brute-force definitions used to pin the oracle (pure Python loops, tiny inputs only).

Nothing here is shared with the oracle or with the HIP path: every quantity is
written out from its textbook definition -- explicit softmax rows, the explicit
T x T cosine matrix the paper's Eq. 3-4 avoid, a full sort.
"""
import math


def softmax_row(x):
    m = max(x)
    e = [math.exp(v - m) for v in x]
    s = sum(e)
    return [v / s for v in e]


def dot(a, b):
    return sum(float(x) * float(y) for x, y in zip(a, b))


def window_mean_attention(K, Qg, scale, causal):
    """mean over (g, w) of softmax_i(scale * q.k_i), visible keys only. Returns N values."""
    N = len(K)
    G, W = len(Qg), len(Qg[0])
    Nc = N - W
    acc = [0.0] * N
    for g in range(G):
        for w in range(W):
            vis = Nc + w + 1 if causal else N
            row = softmax_row([scale * dot(Qg[g][w], K[i]) for i in range(vis)])
            for i in range(vis):
                acc[i] += row[i]
    return [a / (G * W) for a in acc]


def cosine_matrix(K):
    nrm = [math.sqrt(dot(k, k)) for k in K]
    T = len(K)
    return [[dot(K[i], K[j]) / (nrm[i] * nrm[j]) for j in range(T)] for i in range(T)]


def offdiag_mean(R):
    T = len(R)
    tot = sum(R[i][j] for i in range(T) for j in range(T) if i != j)
    return tot / (T * (T - 1))


def mean_cos_to_others(R):
    T = len(R)
    return [sum(R[i][j] for j in range(T) if j != i) / (T - 1) for i in range(T)]


def pool(a, mode, k):
    n, half = len(a), k // 2
    out = []
    for i in range(n):
        taps = [a[j] for j in range(i - half, i + half + 1) if 0 <= j < n]
        out.append(max(taps) if mode == "max" else sum(taps) / k)
    return out


def topk_sorted(s, b):
    """b largest by (-score, index) full sort; returned ascending by index."""
    order = sorted(range(len(s)), key=lambda i: (-s[i], i))
    return sorted(order[:b])


def mixkv_scores(K, V, Qg, scale, causal, pool_mode, pool_k, eps, use_vnorm=True, intrinsic=None,
                 mix="head_adaptive", r_given=None):
    """s_comp over the candidates and the redundancy, through the explicit T x T cosine matrix.

    Follows Algorithm 1 step by step with plain loops; the diversity term uses
    Khat_i . Kbar = (1/T) * sum_j R_ij (row mean of the cosine matrix, diagonal
    included) and the redundancy the off-diagonal mean of R, i.e. the quadratic
    forms that Eq. 3-4 of the paper collapse.  `intrinsic` ("vnorm" | "knorm" |
    "none", default from use_vnorm) and `mix` pick the ablation's variants
    (Table 4): KNorm scores a key by minus its norm; "sum" adds importance and
    scaled diversity without weights; "div_only" / "imp_only" keep one of them;
    "given_r" mixes with the caller's weight.
    """
    if intrinsic is None:
        intrinsic = "vnorm" if use_vnorm else "none"
    N, W = len(K), len(Qg[0])
    Nc = N - W
    a = window_mean_attention(K, Qg, scale, causal)[:Nc]
    s_ex = pool(a, pool_mode, pool_k) if pool_mode != "none" else a
    mean = lambda x: sum(x) / len(x)
    if intrinsic != "none":
        if intrinsic == "vnorm":
            vn = [math.sqrt(dot(v, v)) for v in V[:Nc]]
        else:
            vn = [-math.sqrt(dot(k, k)) for k in K[:Nc]]
        lo, hi = min(vn), max(vn)
        s_in = [(x - lo) / (hi - lo + eps) for x in vn]
        f = mean(s_ex) / (mean(s_in) + eps)
        s_imp = [e + f * x for e, x in zip(s_ex, s_in)]
    else:
        s_imp = list(s_ex)
    R = cosine_matrix(K)
    r = offdiag_mean(R)
    s_div = [-sum(R[i]) / N for i in range(Nc)]
    lo, hi = min(s_div), max(s_div)
    dn = [(x - lo) / (hi - lo + eps) for x in s_div]
    f = mean(s_imp) / (mean(dn) + eps)
    wi, wd = {"head_adaptive": (1 - r, r), "sum": (1.0, 1.0), "div_only": (0.0, 1.0), "imp_only": (1.0, 0.0),
              "given_r": (None, None)}[mix]
    if mix == "given_r":
        wi, wd = 1 - r_given, r_given
    return [wi * si + wd * f * d for si, d in zip(s_imp, dn)], r
