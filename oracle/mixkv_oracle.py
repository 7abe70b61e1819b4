"""CPU oracle for MixKV's prefill-time KV-cache compression step.

TEST INFRASTRUCTURE ONLY.  This is a plain, slow, float64 numpy statement of
what the path computes, written from the paper.  Only the tests, the smoke
check and the benchmark's CPU-baseline leg may import it; the product path
(the HIP library and its binding) never does, and shares no code with it.

One *unit* is one (layer, batch item, KV head).  Under grouped-query attention
the G = Hq/Hkv query heads g in [h*G, (h+1)*G) share KV head h.

Notation follows the paper: T (here N) cached tokens, D head dim, window = the
last W prompt positions, B the per-head budget (window included) and
B' = B - W (Algorithm 1, budget adjustment line).  "Candidates" are the
Nc = N - W non-window positions, the only ones that are ranked (Algorithm 1,
TopB "exclude window").

Readings taken where the paper is silent (each is a parameter or a stated
constant):
  * extrinsic importance is the *mean* over window queries (Sec. 3.2,
    extrinsic importance; Algorithm 1 step 1);
  * GQA: softmax per (query head, window row), then the mean over the G*W rows
    of the group;
  * the softmax runs over all N keys; window query w (position Nc+w) sees keys
    0..Nc+w when `causal_window` is set;
  * 1-D pooling (none / avg / max, odd kernel k, stride 1, same length) is
    applied to the attention part only, over candidates only; max ignores
    out-of-range taps, avg counts them as zeros and divides by k;
  * min / max / mean of Sec. 3.2 and 3.3 are taken over the candidates;
  * the mean normalised key and the redundancy use all N keys (Sec. 3.3, Eq. 3-4);
  * a key of norm below 1e-30 normalises to the zero vector;
  * the redundancy is not clamped;
  * ties in TopB go to the smaller index; kept rows are in ascending position
    order with the window rows last;
  * the ablation's scoring variants (Sec. 4.3, Table 4): the KNorm intrinsic
    score -||K_i|| (Sec. 3.2) goes through the same min-max and mean matching
    as VNorm; the un-weighted row "s_imp + s_div" adds the scaled diversity
    (the one Eq. 5 mixes), "s_div only" ranks by that scaled diversity alone,
    "importance only" by s_imp alone; the offline head weights of Table 4 are a
    caller-given r per unit that replaces Eq. 4's value in Eq. 5;
  * the budget B of Sec. 3.1 / Algorithm 1 may be given per (layer, KV head),
    as the layer-wise and head-wise allocation schemes the method is combined
    with do (Sec. 4.1 and the appendix's baseline details; Table 1): head h
    then keeps its own
    b_h - W best candidates and the window, exactly as in the fixed case;
  * the softmax normaliser of the window rows may be handed in as the
    log-sum-exp the prefill attention already produced for those rows
    (Sec. 3.2: the extrinsic score reuses the attention of the window queries):
    the weight of key i in row r is then exp(logit_ri - lse_r), masked entries 0.

Every function is pinned by tests/test_oracle_*.py against brute force, closed
forms and library routines; the whole path against the authors' own code is
"parity unpinned" (that code is not available).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List

import numpy as np

KEY_NORM_FLOOR = 1e-30


@dataclass(frozen=True)
class Params:
    n_q_heads: int
    n_kv_heads: int
    window: int
    budget: int
    pool: str = "max"              # "none" | "avg" | "max"
    pool_kernel: int = 7
    causal_window: bool = True
    softmax_scale: float = 1.0
    eps: float = 1e-6
    intrinsic: str = "vnorm"       # "none" | "vnorm" | "knorm"
    mix: str = "head_adaptive"     # "head_adaptive" | "sum" | "div_only" | "imp_only" | "given_r"
    budget_mode: str = "fixed"     # "fixed" | "adaptive" | "per_head" (budgets passed to compress_layer)
    budget_floor: int = 0

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


# --------------------------------------------------------------------------- scores

def window_attention(K: np.ndarray, Qg: np.ndarray, scale: float, causal: bool,
                     lse: np.ndarray | None = None) -> np.ndarray:
    """Softmax attention weights of the window queries over all N keys.

    K [N, D], Qg [G, W, D] -> P [G, W, N].  (Sec. 3.2, extrinsic importance:
    Attention(Q_j, K_i) for j in the window.)  With `lse` [G, W] (natural-log
    sum of exp(logit) over the keys each row attends to, as produced elsewhere)
    the rows are normalised by it instead of by their own sum.
    """
    K = np.asarray(K, dtype=np.float64)
    Qg = np.asarray(Qg, dtype=np.float64)
    G, W, _ = Qg.shape
    N = K.shape[0]
    Nc = N - W
    logits = scale * np.einsum("gwd,nd->gwn", Qg, K)
    if causal:
        pos = np.arange(N)
        for w in range(W):
            logits[:, w, pos > Nc + w] = -np.inf
    if lse is not None:
        return np.exp(logits - np.asarray(lse, dtype=np.float64)[:, :, None])
    m = logits.max(axis=2, keepdims=True)
    e = np.exp(logits - m)
    return e / e.sum(axis=2, keepdims=True)


def pool1d(a: np.ndarray, mode: str, k: int) -> np.ndarray:
    """Same-length 1-D pooling, stride 1, window centred on each position."""
    a = np.asarray(a, dtype=np.float64)
    if mode == "none" or k == 1:
        return a.copy()
    assert k % 2 == 1 and k >= 1
    n, half = a.shape[0], k // 2
    out = np.empty(n, dtype=np.float64)
    for i in range(n):
        lo, hi = max(0, i - half), min(n, i + half + 1)
        if mode == "max":
            out[i] = a[lo:hi].max()
        elif mode == "avg":
            out[i] = a[lo:hi].sum() / k
        else:
            raise ValueError(mode)
    return out


def extrinsic_importance(K, Qg, p: Params, lse: np.ndarray | None = None) -> np.ndarray:
    """s_ex over the candidates: window/group mean of attention, then pooling."""
    G, W, _ = np.asarray(Qg).shape
    Nc = np.asarray(K).shape[0] - W
    P = window_attention(K, Qg, p.softmax_scale, p.causal_window, lse)
    a = P[:, :, :Nc].sum(axis=(0, 1)) / (G * W)
    return pool1d(a, p.pool, p.pool_kernel)


def minmax(x: np.ndarray, eps: float) -> np.ndarray:
    """(x - min) / (max - min + eps)   (Sec. 3.2 for VNorm, Sec. 3.3 for diversity)."""
    lo, hi = x.min(), x.max()
    return (x - lo) / (hi - lo + eps)


def scale_to_mean(x_norm: np.ndarray, target_mean: float, eps: float) -> np.ndarray:
    """x_norm * target_mean / (mean(x_norm) + eps)   (Sec. 3.2 / 3.3 mean matching)."""
    return x_norm * (target_mean / (x_norm.mean() + eps))


def normalised_keys(K: np.ndarray) -> np.ndarray:
    K = np.asarray(K, dtype=np.float64)
    nrm = np.sqrt((K * K).sum(axis=1, keepdims=True))
    return K / np.maximum(nrm, KEY_NORM_FLOOR)


def redundancy(Khat: np.ndarray) -> float:
    """Off-diagonal mean of Khat Khat^T through the mean key (Sec. 3.3, Eq. 3-4)."""
    T = Khat.shape[0]
    kbar = Khat.sum(axis=0) / T
    return float((T * T * np.dot(kbar, kbar) - T) / (T * (T - 1)))


def diversity(Khat: np.ndarray) -> np.ndarray:
    """s_div_i = -Khat_i . mean_j Khat_j, all N positions (Sec. 3.2, diversity metrics)."""
    kbar = Khat.sum(axis=0) / Khat.shape[0]
    return -(Khat @ kbar)


def score_unit(K: np.ndarray, V: np.ndarray, Qg: np.ndarray, p: Params,
               r_given: float | None = None, lse: np.ndarray | None = None) -> Dict[str, np.ndarray]:
    """All scores of one unit.  K, V [N, D]; Qg [G, W, D].  Arrays over the Nc candidates.

    `r_given` is the caller's head weight for mix "given_r" (Table 4, offline W^head);
    `lse` [G, W] the window rows' log-sum-exp if the caller has it (see window_attention).
    """
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    N = K.shape[0]
    W = np.asarray(Qg).shape[1]
    Nc = N - W
    assert N >= 2 and Nc >= 1
    s_ex = extrinsic_importance(K, Qg, p, lse)
    if p.intrinsic in ("vnorm", "knorm"):
        if p.intrinsic == "vnorm":
            s_in = np.sqrt((V[:Nc] * V[:Nc]).sum(axis=1))     # VNorm: ||V_i||
        else:
            s_in = -np.sqrt((K[:Nc] * K[:Nc]).sum(axis=1))    # KNorm: -||K_i||
        s_in_norm = minmax(s_in, p.eps)
        s_in_scaled = scale_to_mean(s_in_norm, s_ex.mean(), p.eps)
        s_imp = s_ex + s_in_scaled                       # Eq. 2
    elif p.intrinsic == "none":
        s_in_scaled = np.zeros(Nc)
        s_imp = s_ex.copy()
    else:
        raise ValueError(p.intrinsic)
    Khat = normalised_keys(K)
    r = redundancy(Khat)                                  # Eq. 4
    s_div = diversity(Khat)[:Nc]
    s_div_norm = minmax(s_div, p.eps)
    s_div_scaled = scale_to_mean(s_div_norm, s_imp.mean(), p.eps)
    if p.mix == "head_adaptive":
        s_comp = (1.0 - r) * s_imp + r * s_div_scaled     # Eq. 5
    elif p.mix == "given_r":
        assert r_given is not None
        s_comp = (1.0 - r_given) * s_imp + r_given * s_div_scaled
    elif p.mix == "sum":
        s_comp = s_imp + s_div_scaled
    elif p.mix == "div_only":
        s_comp = s_div_scaled.copy()
    elif p.mix == "imp_only":
        s_comp = s_imp.copy()
    else:
        raise ValueError(p.mix)
    return dict(s_ex=s_ex, s_in_scaled=s_in_scaled, s_imp=s_imp, s_div=s_div,
                s_div_scaled=s_div_scaled, r=np.float64(r), s_comp=s_comp)


# --------------------------------------------------------------------------- redundancy analysis

def similarity_analysis(X: np.ndarray, block: int) -> Dict[str, np.ndarray]:
    """Pairwise cosine similarity of the rows of X [N, D] (keys or values of one head), as the
    paper's redundancy figures show it (Sec. 1, the figures on key/value similarity inside a head
    and across heads; Sec. 3.3, Eq. 3 for the matrix itself).

    Written as the definition: the full N x N matrix R of cosine similarities, then
      redundancy  the mean of its off-diagonal entries (Eq. 4 applied to X),
      block_map   [nb, nb], nb = ceil(N / block): the mean of R over rows of block a and columns
                  of block b (the last block may be short; diagonal entries are part of diagonal
                  blocks), i.e. the heat-map at a resolution of `block` tokens.
    """
    Xh = normalised_keys(X)
    N = Xh.shape[0]
    R = Xh @ Xh.T
    red = (R.sum() - np.trace(R)) / (N * (N - 1))
    nb = (N + block - 1) // block
    bm = np.empty((nb, nb))
    for a in range(nb):
        for b in range(nb):
            bm[a, b] = R[a * block:(a + 1) * block, b * block:(b + 1) * block].mean()
    return dict(redundancy=np.float64(red), block_map=bm)


# --------------------------------------------------------------------------- decoding on the compacted cache

def decode_attention(q: np.ndarray, K_rows: List[np.ndarray], V_rows: List[np.ndarray], scale: float) -> np.ndarray:
    """Attention of one new token over a compressed cache (Sec. 3.1: the compacted K, V serve the
    attention of the decoding phase).

    q [Hq, D]; K_rows / V_rows: per KV head the rows it holds, [n_h, D] (the kept rows followed by
    whatever was appended since; n_h may differ between heads).  Query head g reads KV head
    g // G.  Returns [Hq, D]: softmax_j(scale * q_g . k_j) weighted sum of the v_j.
    """
    q = np.asarray(q, dtype=np.float64)
    Hq, Hkv = q.shape[0], len(K_rows)
    G = Hq // Hkv
    out = np.empty_like(q)
    for g in range(Hq):
        K = np.asarray(K_rows[g // G], dtype=np.float64)
        V = np.asarray(V_rows[g // G], dtype=np.float64)
        logit = scale * (K @ q[g])
        e = np.exp(logit - logit.max())
        out[g] = (e / e.sum()) @ V
    return out


def append_token(K_tail: np.ndarray, V_tail: np.ndarray, k_new: np.ndarray, v_new: np.ndarray, position: int):
    """The cache grows by one token after the compression (Sec. 3.1: decoding continues on the
    compacted cache): row `position` of every head's tail receives the new key and value row.

    K_tail / V_tail [Hkv, capacity, D] are changed in place; k_new / v_new [Hkv, D].  A copy, so the
    stored values pass through unchanged whatever their dtype.
    """
    if not 0 <= position < K_tail.shape[1]:
        raise ValueError("position outside the tail")
    for h in range(K_tail.shape[0]):
        K_tail[h, position] = k_new[h]
        V_tail[h, position] = v_new[h]


# --------------------------------------------------------------------------- selection

def top_indices(s: np.ndarray, b: int) -> np.ndarray:
    """The b positions with the largest s, ties to the smaller index, ascending."""
    order = np.argsort(-np.asarray(s), kind="stable")
    return np.sort(order[:b])


def adaptive_budgets(s_heads: np.ndarray, budget: int, window: int, floor: int) -> np.ndarray:
    """Head-adaptive split of one layer's pool of Hkv*B' non-window slots.

    s_heads [Hkv, Nc].  Every head first keeps its own top-`floor` candidates;
    the remaining Hkv*(B'-floor) slots go to the best remaining candidates of
    all heads together (ties: smaller head, then smaller index).  Returns
    b'_h [Hkv].  (The paper only names the AdaKV-style allocator; this rule is
    the workload definition's.)
    """
    s_heads = np.asarray(s_heads)
    Hkv, Nc = s_heads.shape
    bp = budget - window
    assert 0 <= floor <= bp and bp <= Nc
    taken = np.zeros((Hkv, Nc), dtype=bool)
    for h in range(Hkv):
        taken[h, top_indices(s_heads[h], floor)] = True
    rest = Hkv * (bp - floor)
    flat = np.where(taken, -np.inf, s_heads).reshape(-1)
    order = np.argsort(-flat, kind="stable")[:rest]       # flat index = h*Nc + i
    counts = np.full(Hkv, floor, dtype=np.int64)
    for f in order:
        counts[f // Nc] += 1
    return counts


def select_unit(s_comp: np.ndarray, b_prime: int, N: int, W: int) -> np.ndarray:
    """Kept positions of one head: its top-b' candidates ascending, then the window."""
    Nc = N - W
    assert s_comp.shape[0] == Nc and 0 <= b_prime <= Nc
    return np.concatenate([top_indices(s_comp, b_prime), np.arange(Nc, N)]).astype(np.int64)


# --------------------------------------------------------------------------- whole layer

def compress_layer(K: np.ndarray, V: np.ndarray, Q: np.ndarray, p: Params,
                   r_given: np.ndarray | None = None, head_budgets: np.ndarray | None = None,
                   window_lse: np.ndarray | None = None) -> Dict[str, object]:
    """Algorithm 1 for every (batch item, KV head) of one layer.

    K, V [Bt, Hkv, N, D]; Q [Bt, Hq, W, D]; r_given [Bt, Hkv] for mix "given_r";
    head_budgets [Hkv] (rows kept by each head of this layer, window included)
    for budget mode "per_head"; window_lse [Bt, Hq, W] the window rows'
    log-sum-exp when the caller has it.  Returns
      scores [Bt, Hkv, N] (s_comp at candidates, +inf at window slots),
      redundancy [Bt, Hkv], counts [Bt, Hkv], offsets [Bt, Hkv+1],
      indices: list over batch of list over heads of int64 arrays,
      K_out / V_out: same nesting, rows copied verbatim from K / V.
    """
    Bt, Hkv, N, D = K.shape
    W, G = p.window, p.group
    Nc = N - W
    assert Q.shape == (Bt, p.n_q_heads, W, D) and p.n_kv_heads == Hkv
    assert W <= p.budget <= N
    scores = np.full((Bt, Hkv, N), np.inf)
    red = np.zeros((Bt, Hkv))
    counts = np.zeros((Bt, Hkv), dtype=np.int64)
    offsets = np.zeros((Bt, Hkv + 1), dtype=np.int64)
    indices: List[List[np.ndarray]] = []
    K_out: List[List[np.ndarray]] = []
    V_out: List[List[np.ndarray]] = []
    for b in range(Bt):
        for h in range(Hkv):
            u = score_unit(K[b, h], V[b, h], Q[b, h * G:(h + 1) * G], p,
                           None if r_given is None else float(r_given[b, h]),
                           None if window_lse is None else window_lse[b, h * G:(h + 1) * G])
            scores[b, h, :Nc] = u["s_comp"]
            red[b, h] = u["r"]
        if p.budget_mode == "fixed":
            bp = np.full(Hkv, p.budget - W, dtype=np.int64)
        elif p.budget_mode == "adaptive":
            bp = adaptive_budgets(scores[b, :, :Nc], p.budget, W, p.budget_floor)
        elif p.budget_mode == "per_head":
            hb = np.asarray(head_budgets, dtype=np.int64)
            assert hb.shape == (Hkv,) and np.all(hb >= W) and np.all(hb <= N)
            bp = hb - W                                   # Algorithm 1's budget line, per head
        else:
            raise ValueError(p.budget_mode)
        idx_b, k_b, v_b = [], [], []
        for h in range(Hkv):
            idx = select_unit(scores[b, h, :Nc], int(bp[h]), N, W)
            idx_b.append(idx)
            k_b.append(K[b, h][idx].copy())
            v_b.append(V[b, h][idx].copy())
            counts[b, h] = idx.shape[0]
        offsets[b, 1:] = np.cumsum(counts[b])
        indices.append(idx_b)
        K_out.append(k_b)
        V_out.append(v_b)
    return dict(scores=scores, redundancy=red, counts=counts, offsets=offsets,
                indices=indices, K_out=K_out, V_out=V_out)
