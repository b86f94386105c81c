"""Plain fp64 CPU oracle for the D2O KV-cache compression hot path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module;
only tests/, the smoke check and the benchmark's cpu_baseline leg call it.  It
shares no code with the HIP library and never receives values computed by it.

All arithmetic is numpy float64.  Inputs are the given fp32 / bf16 values
converted exactly.  Each function follows one passage of the paper (arxiv
2406.13035), cited in its docstring; where the paper is silent or garbled the
reading taken is stated there.  Parity pins live in tests/test_oracle_pins.py.
Functions without an external pin: none at present (the whole-method
composition is pinned by brute force on tiny inputs only; beyond those sizes
there is no published numeric trace of D2O's state: "parity unpinned" applies
to full-size end-to-end traces, see the tests' notes).

Summation order: rows of the attention matrix are processed in row blocks only
to bound memory (each row is independent; the per-key column sum adds the
blocks' partial column sums in ascending row order).  No other blocking,
fusion or reordering is applied.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np

E = math.e  # exp(1): self-similarity term of the merge weights (Sec. 4.2.2, Eq. 12)


# --------------------------------------------------------------------------- storage rounding

def round_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp64 values to the cache's storage type (round-to-nearest-even), returned as fp64.

    The paper does not state a cache precision; the reading taken is: the cache
    holds the input dtype and merged rows are rounded to it once, on write.
    "f64" leaves values untouched (pure mode)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    if dtype == "f64":
        return x.copy()
    if dtype == "f32":
        return x.astype(np.float32).astype(np.float64)
    if dtype == "bf16":
        # bfloat16 keeps 7 of the 52 fraction bits (same exponent range as fp32; values
        # here are far from its limits).  Round to nearest, ties to even, on the bit pattern.
        b = x.view(np.uint64)
        lsb = (b >> np.uint64(45)) & np.uint64(1)
        r = (b + np.uint64((1 << 44) - 1) + lsb) & ~np.uint64((1 << 45) - 1)
        return r.view(np.float64).copy()
    if dtype == "fp8":
        return quantise_fp8_rows(round_storage(x, "bf16"))
    raise ValueError(dtype)


def quantise_fp8_rows(x: np.ndarray) -> np.ndarray:
    """The fp8 cache encoding (the conclusion of the paper names the combination with KV-cache
    quantisation as future work and defines no format; this is the reading taken).  A cache row
    (last axis) is stored as d codes of the 8-bit floating-point format E4M3 (1 sign, 4 exponent
    bits with bias 7, 3 fraction bits, subnormals down to 2^-9, largest magnitude 448, no
    infinities) and one power of two per row:
      e   = the smallest integer with max|x| * 2^-e <= 448 (0 for an all-zero row; not below
            -120, so that it fits a signed byte: rows of magnitude 1e-34 and less lose bits),
      q_i = x_i * 2^-e rounded to the nearest E4M3 value, ties to the even fraction,
    and the row then holds the values q_i * 2^e, which is what this function returns (fp64).
    The cache's logical type stays the input type: "fp8" storage rounds a row to bf16 first and
    encodes that (round_storage), so prompt-phase rows, new tokens and merged rows all enter the
    cache the same way."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    if x.ndim == 1:
        return quantise_fp8_rows(x[None, :])[0]
    amax = np.abs(x).max(axis=-1, keepdims=True)
    frac, ex = np.frexp(amax)                      # amax = frac * 2^ex, 0.5 <= frac < 1; 448 = 0.875 * 2^9
    e = np.where(frac <= 0.875, ex - 9, ex - 8)
    e = np.where(amax > 0.0, np.maximum(e, -120), 0)
    y = np.ldexp(x, -e)                            # exact; |y| <= 448
    _, ey = np.frexp(y)                            # |y| in [2^(ey-1), 2^ey)
    E = np.maximum(ey - 1, -6)                     # binade of y, the subnormal range counts as binade -6
    q = np.ldexp(np.rint(np.ldexp(y, 3 - E)), E - 3)   # spacing 2^(E-3); rint rounds ties to even
    return np.ldexp(q, e) + 0.0                    # (+ 0.0: a negative zero becomes zero)


# --------------------------------------------------------------------------- upstream: Q, K, V from the hidden states

def rope_rotate(x, positions, base: float = 10000.0):
    """Rotary position embedding on vectors x [..., n, d] at integer positions [n] (the models the
    paper evaluates - Llama, Mistral - apply it to queries and keys before Eq. 3; the paper
    itself does not print it).  Half-split convention of those models: element i < d/2 is paired
    with element i + d/2, and the pair is rotated by the angle pos * base^(-2i/d):
      y_i = x_i cos - x_{i+d/2} sin,   y_{i+d/2} = x_{i+d/2} cos + x_i sin."""
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    half = d // 2
    inv_freq = base ** (-(2.0 * np.arange(half)) / float(d))
    ang = np.asarray(positions, dtype=np.float64)[:, None] * inv_freq[None, :]      # [n, d/2]
    c, s_ = np.cos(ang), np.sin(ang)
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s_, b * c + a * s_], axis=-1)


def qkv_project(X, W, n_q_heads: int, n_kv_heads: int, head_dim: int, pos0: int = 0, base: float = 10000.0,
                storage: str = "f64"):
    """Sec. 3 Eq. 1 for one layer: Q = X W_Q, K = X W_K, V = X W_V from the hidden states X
    [n, hidden], with the three weight matrices stacked as the rows of W [(Hq + 2 Hkv) d, hidden]
    (queries first, then keys, then values; a row of W is one output feature), rotary embedding
    (rope_rotate) on queries and keys at positions pos0 .. pos0 + n - 1, values left as they are.
    Results are rounded to `storage` once, at the end (the tensors handed to the attention of
    Eq. 3 are stored in the model's dtype).  Returns Q [Hq, n, d], K [Hkv, n, d], V [Hkv, n, d]."""
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    n = X.shape[0]
    Y = X @ W.T                                                   # [n, (Hq + 2 Hkv) d]
    nq, nk = n_q_heads * head_dim, n_kv_heads * head_dim
    pos = np.arange(pos0, pos0 + n)
    Q = Y[:, :nq].reshape(n, n_q_heads, head_dim).transpose(1, 0, 2)
    K = Y[:, nq:nq + nk].reshape(n, n_kv_heads, head_dim).transpose(1, 0, 2)
    V = Y[:, nq + nk:].reshape(n, n_kv_heads, head_dim).transpose(1, 0, 2)
    Q = rope_rotate(Q, pos, base)
    K = rope_rotate(K, pos, base)
    return round_storage(Q, storage), round_storage(K, storage), round_storage(V, storage)


# --------------------------------------------------------------------------- a1: prefill attention

def prefill_attention_head(q, k, v, causal: bool = True, row_block: int = 2048,
                           row_range: tuple[int, int] | None = None):
    """Attention of one query head over the prompt, Sec. 4.1 Eq. 4 (and Sec. 3 Eq. 3).

    A = softmax(Q K^T / sqrt(d)) row-wise (causal: keys j <= i only; the paper's
    models are decoder-only), O = A V, and the column sums s[j] = sum_i A[i, j]
    (Sec. 4.1), the initial cumulative attention score (Eq. 6, prompt case).  d is the head dimension.
    Returns (O [N, d], s [N]).

    row_range = (lo, hi) restricts the work to query rows lo <= i < hi (rows are independent
    of each other): O then holds those rows only ([hi - lo, d]) and s the column sums over
    those rows only, which is the complete sum for every column j >= lo when hi = N."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    n, d = q.shape
    lo, hi = (0, n) if row_range is None else row_range
    out = np.empty((hi - lo, d))
    colsum = np.zeros(n)
    root_d = np.sqrt(float(d))
    for i0 in range(lo, hi, row_block):
        i1 = min(hi, i0 + row_block)
        ncol = i1 if causal else n
        s = (q[i0:i1] @ k[:ncol].T) / root_d
        if causal:
            rows = np.arange(i0, i1)[:, None]
            cols = np.arange(ncol)[None, :]
            s = np.where(cols <= rows, s, -np.inf)
        s = s - s.max(axis=1, keepdims=True)
        p = np.exp(s)
        p = p / p.sum(axis=1, keepdims=True)
        out[i0 - lo:i1 - lo] = p @ v[:ncol]
        colsum[:ncol] += p.sum(axis=0)
    return out, colsum


# --------------------------------------------------------------------------- a2: density statistic

def head_variance(colsum) -> float:
    """Population variance of one head's cumulative attention sequence (Sec. 4.1 Eq. 4;
    per-head form in App. A.8).  Population (divide by N): the paper does not say which."""
    s = np.asarray(colsum, dtype=np.float64)
    mu = s.sum() / s.size
    return float(((s - mu) ** 2).sum() / s.size)


def layer_density(colsums_per_q_head) -> float:
    """F_v^l of one layer: mean over its query heads of the per-head variances
    (Eq. 4 omits heads; the figures of Sec. 1 and App. A.6 plot the per-layer mean over heads)."""
    vs = [head_variance(s) for s in colsums_per_q_head]
    return float(sum(vs) / len(vs))


# --------------------------------------------------------------------------- a3: budget allocation

ALLOCATION_POLICIES = ("softmax", "reciprocal", "exp_decay", "uniform")


def allocate_budgets(F, seq_len: int, total_budget: int, min_budget: int = 64, policy: str = "softmax"):
    """Integer per-layer cache sizes S_l from the density statistics, Sec. 4.1 Eq. 5 and
    App. A.2: alpha_l proportional to exp(-F_l), sum_l S_l = total_budget (= round(rho*S*L)).

    `policy` selects the design of alpha_l among the four that the allocation-policy analysis
    of Sec. 5 compares: "softmax" (Eq. 5, the method's own, weight exp(-F_l)), "reciprocal"
    (weight 1/F_l, needs F_l > 0), "uniform" (weight 1: alpha_l = rho for every layer) - these
    three split the same total budget and differ only in the weight that enters step 1 below -
    and "exp_decay" (alpha_l = exp(-F_l) taken as the layer's own compression ratio, not
    normalised over the layers: S_l = floor(exp(-F_l) * seq_len) clipped to [min_budget,
    seq_len]; the total budget is not used, as the definition has no sum constraint).

    The paper bounds neither S_l <= S nor S_l > 0, and gives no integer rule.  Reading:
      1. split the budget over the layers in proportion to exp(-F_l) (exponent shifted by
         the smallest F among the layers still free, which changes no ratio);
      2. shares above seq_len or below min_budget violate the bounds.  When the total excess
         above seq_len is at least the total deficit below min_budget, every layer above
         seq_len is pinned to seq_len (the budget it frees can only raise the others);
         otherwise every layer below min_budget is pinned to min_budget.  What is left is
         re-split over the free layers; repeat until no share violates.  This is the unique
         allocation S_l = clip(lambda * exp(-F_l), min_budget, seq_len) that sums to the budget;
      3. floor the free layers' shares and hand the remaining units, one each, to the largest
         fractional parts (ties: lower layer index), never above seq_len.
    Raises ValueError when n_layers*min_budget <= total_budget <= n_layers*seq_len fails."""
    F = np.asarray(F, dtype=np.float64)
    L = F.size
    if policy not in ALLOCATION_POLICIES:
        raise ValueError("unknown allocation policy")
    if policy == "exp_decay":
        if min_budget < 0 or min_budget > seq_len:
            raise ValueError("infeasible bounds")
        S = np.floor(np.exp(-F) * float(seq_len)).astype(np.int64)
        return np.clip(S, min_budget, seq_len)
    if policy == "reciprocal" and not np.all(F > 0.0):
        raise ValueError("the reciprocal policy needs positive variances")
    if not (L * min_budget <= total_budget <= L * seq_len) or min_budget < 0:
        raise ValueError("infeasible total budget")
    S = np.zeros(L, dtype=np.int64)
    free = np.ones(L, dtype=bool)
    remaining = int(total_budget)
    share = np.zeros(L)
    while free.any():
        idx = np.flatnonzero(free)
        if policy == "softmax":
            w = np.exp(-(F[idx] - F[idx].min()))
        elif policy == "reciprocal":
            w = 1.0 / F[idx]
        else:
            w = np.ones(idx.size)
        wsum = 0.0
        for x in w:                      # ascending layer order
            wsum += x
        share[idx] = float(remaining) * (w / wsum)
        over = idx[share[idx] > seq_len]
        under = idx[share[idx] < min_budget]
        excess = 0.0
        for l in over:
            excess += share[l] - seq_len
        deficit = 0.0
        for l in under:
            deficit += min_budget - share[l]
        if over.size == 0 and under.size == 0:
            break
        if over.size and excess >= deficit:
            S[over] = seq_len
            free[over] = False
            remaining -= seq_len * over.size
        else:
            S[under] = min_budget
            free[under] = False
            remaining -= min_budget * under.size
    idx = np.flatnonzero(free)
    if idx.size:
        fl = np.floor(share[idx]).astype(np.int64)
        S[idx] = fl
        left = remaining - int(fl.sum())
        frac = share[idx] - fl
        order = sorted(range(idx.size), key=lambda t: (-frac[t], idx[t]))
        t = 0
        while left > 0:
            l = idx[order[t % idx.size]]
            if S[l] < seq_len:
                S[l] += 1
                left -= 1
            t += 1
    assert int(S.sum()) == total_budget
    return S


def allocate_budgets_heads(F_heads, group: int, seq_len: int, total_budget: int, min_budget: int = 64):
    """Per-head allocation of App. A.8: alpha_l^h proportional to exp(-F^{l,h}) with the sum taken
    over ALL layers and heads, S_l^h = alpha_l^h * S_total (S_total = rho * L * H * S), the
    layer's proportion being alpha_l = sum_h alpha_l^h.  That is Eq. 5 with one entry per (layer,
    head) instead of one per layer, so it takes the same bounds and integer rule (the reading
    documented at allocate_budgets).  F_heads [L, Hq] holds the per-query-head variances; caches
    are kept per KV head, and under grouped-query attention a KV head's statistic is read as
    the mean of the variances of the `group` query heads it serves (the paper names the
    attention types but not this case).  total_budget counts rows over all layers and KV heads.
    Returns S [L, Hkv]; S.sum(axis=1) are the layer totals."""
    F = np.asarray(F_heads, dtype=np.float64)
    L, Hq = F.shape
    if Hq % group:
        raise ValueError("query heads must be a multiple of the group size")
    Hkv = Hq // group
    Fkv = np.zeros((L, Hkv))
    for l in range(L):
        for h in range(Hkv):
            acc = 0.0
            for g in range(group):               # ascending head order
                acc += F[l, h * group + g]
            Fkv[l, h] = acc / float(group)
    return allocate_budgets(Fkv.reshape(-1), seq_len, total_budget, min_budget).reshape(L, Hkv)


# --------------------------------------------------------------------------- a4: selection

def select(score, budget: int, recent: int, n_sink: int = 0):
    """Eviction choice of Sec. 4.2.1 Eq. 7-8 on a score vector ordered by token position.

    Retained = first n_sink (T) entries, the `recent` (M) last entries and the Top_N of the
    entries in between, N = budget - T - M.  Ties in Top_N: the lower index is kept
    (the paper is silent).  Returns (retained, evicted) as ascending index arrays;
    budget >= len(score) retains everything."""
    score = np.asarray(score, dtype=np.float64)
    n = score.size
    if budget >= n:
        return np.arange(n, dtype=np.int64), np.zeros(0, dtype=np.int64)
    n_hh = budget - n_sink - recent
    if n_hh < 0 or n_sink < 0 or recent < 0:
        raise ValueError("budget smaller than sinks + recent window")
    mid = np.arange(n_sink, n - recent)
    order = np.argsort(-score[mid], kind="stable")      # descending score, lower index first
    top = mid[order[:n_hh]]
    keep = np.zeros(n, dtype=bool)
    keep[:n_sink] = True
    keep[n - recent:] = True
    keep[top] = True
    return np.flatnonzero(keep).astype(np.int64), np.flatnonzero(~keep).astype(np.int64)


# --------------------------------------------------------------------------- a6: matching

def cosine_matrix(Ke, Kc):
    """u_ij = k_i . k_j / (|k_i| |k_j|), Sec. 4.2.2 Eq. 9; 0 where a norm is 0 (paper silent)."""
    Ke = np.asarray(Ke, dtype=np.float64)
    Kc = np.asarray(Kc, dtype=np.float64)
    dots = Ke @ Kc.T
    ne = np.sqrt((Ke * Ke).sum(axis=1))
    nc = np.sqrt((Kc * Kc).sum(axis=1))
    den = ne[:, None] * nc[None, :]
    with np.errstate(divide="ignore", invalid="ignore"):
        U = np.where(den > 0.0, dots / den, 0.0)
    return U


def match(Ke, Kc):
    """Many-to-one nearest-neighbour matching, Eq. 9: for every evicted key the retained key
    of largest cosine similarity; the first maximum in ascending retained order wins.
    Returns (u_star [Le], target [Le] as an index into Kc)."""
    if len(Ke) == 0:
        return np.zeros(0), np.zeros(0, dtype=np.int64)
    U = cosine_matrix(Ke, Kc)
    t = np.argmax(U, axis=1)
    return U[np.arange(U.shape[0]), t], t.astype(np.int64)


# --------------------------------------------------------------------------- a7: threshold

def prefill_threshold(u_star):
    """tau_0 = mean of the evicted tokens' best similarities, Eq. 10 (t = 0 case); a token is
    merged iff its best similarity is not lower than the threshold (text after Eq. 10).
    Returns (tau, passed); tau is NaN (unset) when nothing was evicted."""
    u_star = np.asarray(u_star, dtype=np.float64)
    if u_star.size == 0:
        return float("nan"), np.zeros(0, dtype=bool)
    tau = float(u_star.sum() / u_star.size)
    return tau, u_star >= tau


def ema_threshold(tau_prev: float, u_star: float, beta: float) -> float:
    """tau_t = beta * max(U_t) + (1 - beta) * tau_{t-1}, Eq. 10 (t > 0 case).  While no
    threshold exists yet (nothing was evicted during prompt encoding) the first eviction's
    similarity initialises it, which is the t = 0 formula over one evicted token."""
    if math.isnan(tau_prev):
        return float(u_star)
    return float(beta * u_star + (1.0 - beta) * tau_prev)


# --------------------------------------------------------------------------- a8: merge

def merge(Kc, Vc, Ke, Ve, u_star, target, passed, storage: str = "f64", weighted: bool = True):
    """Similarity-weighted merge, Sec. 4.2.2 Eq. 11-12.

    Eq. 12 as printed gives every evicted token the same weight; the reading taken is the
    softmax over the group {retained j} + {evicted i matched to j and passing the threshold}:
      Z_j = e + sum_i exp(u_ij),  w_cj = e / Z_j,  w_ei = exp(u_ij) / Z_j
    (e = exp(1) is the retained token's self-similarity term, so it keeps the largest weight).
    Keys and values share the weights.  All merges read pre-merge rows.  Sources are added
    in ascending evicted order.  Retained rows without sources are returned unchanged;
    changed rows are rounded to `storage`.  Returns (K', V', group sizes).
    weighted=False is the "average merging" that the merge-policy ablation of Sec. 5 compares
    against: the plain mean of the retained row and its sources (every weight 1, Z_j = 1 + n_j)."""
    Kc = np.array(Kc, dtype=np.float64)
    Vc = np.array(Vc, dtype=np.float64)
    Ke = np.asarray(Ke, dtype=np.float64)
    Ve = np.asarray(Ve, dtype=np.float64)
    Kout, Vout = Kc.copy(), Vc.copy()
    nsrc = np.zeros(len(Kc), dtype=np.int64)
    groups: dict[int, list[int]] = {}
    for i in range(len(Ke)):
        if passed[i]:
            groups.setdefault(int(target[i]), []).append(i)
    for j, src in groups.items():
        w_self = E if weighted else 1.0
        z = w_self
        ka = w_self * Kc[j]
        va = w_self * Vc[j]
        for i in src:
            w = math.exp(float(u_star[i])) if weighted else 1.0
            z += w
            ka = ka + w * Ke[i]
            va = va + w * Ve[i]
        Kout[j] = round_storage(ka / z, storage)
        Vout[j] = round_storage(va / z, storage)
        nsrc[j] = len(src)
    return Kout, Vout, nsrc


# --------------------------------------------------------------------------- a4-a8 composed

@dataclasses.dataclass
class HeadCache:
    """Compressed cache of one (sequence, layer, KV head): rows in ascending token position."""
    K: np.ndarray            # [count, d] fp64 holding storage-dtype values
    V: np.ndarray
    score: np.ndarray        # [count] cumulative attention score (Eq. 6), fp64
    pos: np.ndarray          # [count] original token positions
    tau: float               # EMA threshold (NaN = unset)
    storage: str = "f64"


@dataclasses.dataclass
class PrefillEvents:
    retained: np.ndarray     # positions, ascending
    evicted: np.ndarray      # positions, ascending
    target: np.ndarray       # [Le] position of the matched retained token
    u_star: np.ndarray       # [Le]
    passed: np.ndarray       # [Le] bool
    tau: float


def compress_head(K, V, score, budget: int, recent: int, n_sink: int = 0,
                  storage: str = "f64", tau_force: float = float("nan"), weighted: bool = True):
    """Token-level operation on one KV head after prompt encoding (Sec. 4.2): eviction
    (Eq. 7-8), matching on the pre-merge keys (Eq. 9), tau_0 (Eq. 10), merge (Eq. 11-12).
    The cumulative score of a slot that absorbs tokens is left unchanged (paper silent).
    tau_force: NaN = Eq. 10; +inf = never merge (pure eviction); -inf = merge everything.
    weighted: Eq. 11-12 weights, or the ablation's average merging."""
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    score = np.asarray(score, dtype=np.float64)
    ret, evi = select(score, budget, recent, n_sink)
    u_star, t = match(K[evi], K[ret])
    tau, passed = prefill_threshold(u_star)
    if not math.isnan(tau_force):
        passed = u_star >= tau_force
    Kc, Vc, _ = merge(K[ret], V[ret], K[evi], V[evi], u_star, t, passed, storage, weighted)
    if storage == "fp8":    # every row that enters the cache is encoded, the unmerged ones too
        Kc, Vc = round_storage(Kc, storage), round_storage(Vc, storage)
    cache = HeadCache(Kc, Vc, score[ret].copy(), ret.copy(), tau, storage)
    ev = PrefillEvents(ret, evi, ret[t] if len(evi) else np.zeros(0, dtype=np.int64),
                       u_star, passed, tau)
    return cache, ev


# --------------------------------------------------------------------------- a9-a12: decode step

@dataclasses.dataclass
class DecodeEvent:
    evicted_pos: int         # -1: nothing evicted this step
    target_pos: int          # -1: discarded (or nothing evicted)
    u_star: float            # NaN when nothing evicted
    tau: float


def decode_step_head(cache: HeadCache, q, k_new, v_new, new_pos: int, budget: int, recent: int,
                     n_sink: int, beta: float, tau_force: float = float("nan"), weighted: bool = True):
    """One generation step on one KV head (Sec. 3 Eq. 2-3; Sec. 4.2 Eq. 6-12).

    q [G, d] are the queries of the G query heads sharing this KV head (their softmax rows
    add into one score, the grouped-query reading).  Steps: append (k, v) with score 0;
    p_g = softmax(q_g K^T / sqrt(d)) over all slots; out_g = p_g V; score += sum_g p_g
    (Eq. 6, generation case); if the cache now exceeds `budget`, Eq. 7-8 applied to the
    count+1 entries drops exactly one token; its best cosine among the survivors (Eq. 9)
    updates the EMA threshold (Eq. 10; update first, then test against the new value) and
    the token is merged into its match (Eq. 11-12 with one source) or discarded.
    Mutates `cache`; returns (out [G, d], DecodeEvent)."""
    q = np.asarray(q, dtype=np.float64)
    d = q.shape[1]
    k_new = np.asarray(k_new, dtype=np.float64)
    v_new = np.asarray(v_new, dtype=np.float64)
    if cache.storage == "fp8":   # the new row is encoded when it enters the cache, before it is attended to
        k_new, v_new = round_storage(k_new, "fp8"), round_storage(v_new, "fp8")
    cache.K = np.vstack([cache.K, k_new[None, :]])
    cache.V = np.vstack([cache.V, v_new[None, :]])
    cache.score = np.append(cache.score, 0.0)
    cache.pos = np.append(cache.pos, new_pos)
    root_d = np.sqrt(float(d))
    out = np.empty_like(q)
    for g in range(q.shape[0]):
        s = (cache.K @ q[g]) / root_d
        s = s - s.max()
        p = np.exp(s)
        p = p / p.sum()
        out[g] = p @ cache.V
        cache.score = cache.score + p
    count = cache.pos.size
    if count <= budget:
        return out, DecodeEvent(-1, -1, float("nan"), cache.tau)
    assert np.all(np.diff(cache.pos) > 0)
    ret, evi = select(cache.score, budget, recent, n_sink)
    assert evi.size == 1
    e = int(evi[0])
    u_star, t = match(cache.K[evi], cache.K[ret])
    u = float(u_star[0])
    tj = int(ret[int(t[0])])
    if math.isnan(tau_force):
        cache.tau = ema_threshold(cache.tau, u, beta)
        do_merge = u >= cache.tau
    else:
        do_merge = u >= tau_force
    target_pos = -1
    if do_merge:
        Km, Vm, _ = merge(cache.K[[tj]], cache.V[[tj]], cache.K[[e]], cache.V[[e]],
                          np.array([u]), np.array([0]), np.array([True]), cache.storage, weighted)
        cache.K[tj] = Km[0]
        cache.V[tj] = Vm[0]
        target_pos = int(cache.pos[tj])
    evicted_pos = int(cache.pos[e])
    cache.K = cache.K[ret]
    cache.V = cache.V[ret]
    cache.score = cache.score[ret]
    cache.pos = cache.pos[ret]
    return out, DecodeEvent(evicted_pos, target_pos, u, cache.tau)


# --------------------------------------------------------------------------- multi-token append

@dataclasses.dataclass
class AppendEvents:
    evicted: np.ndarray      # positions, ascending (empty when the cache stayed within its budget)
    target: np.ndarray       # [Le] position of the matched retained token
    u_star: np.ndarray       # [Le]
    passed: np.ndarray       # [Le] bool
    tau: float


def append_chunk_head(cache: HeadCache, q, k_new, v_new, first_pos: int, budget: int, recent: int,
                      n_sink: int, beta: float, tau_force: float = float("nan"), weighted: bool = True):
    """A block of m new tokens on one KV head: the chunked / multi-turn form of a generation
    step (Sec. 3 Eq. 2-3 and Sec. 4.2 Eq. 6-12 applied to m tokens at once; the multi-turn
    experiment of the appendix feeds whole turns into a cache of fixed budget).

    q [G, m, d], k_new, v_new [m, d]; the tokens get positions first_pos .. first_pos + m - 1.
      1. Attention and scores, token by token in causal order: token i is appended (score 0),
         attends to everything cached so far including itself, p = softmax(q K^T / sqrt(d)),
         out = p V, and every visible entry's score grows by p, for each of the G query heads in
         turn (Eq. 6, generation case, with no eviction between the tokens of the block; the
         totals equal the column sums of the block's attention matrix, Eq. 6 prompt case).
      2. If the cache now holds more than `budget` entries, Eq. 7-8 applied once to all of them
         (ordered by position) keeps T sinks, the top scores of the middle and the last M, so
         count - budget tokens are evicted together.
      3. Each evicted token is matched to its nearest retained key on the pre-merge keys (Eq. 9).
      4. Threshold (Eq. 10).  The paper gives the t = 0 form for many evicted tokens (their mean
         best similarity) and the t > 0 form for one; for a step that evicts several, the reading
         taken joins the two: the step's similarity is the mean of the evicted tokens' best
         similarities, tau <- beta * mean + (1 - beta) * tau (tau <- mean while unset).  With one
         evicted token this is the generation step, with an unset tau the prompt-phase formula.
         A token is merged iff its best similarity is not lower than the updated threshold.
      5. Merge (Eq. 11-12, many sources per retained token), rounded to the cache's storage.
    Mutates `cache`; returns (out [G, m, d], AppendEvents)."""
    q = np.asarray(q, dtype=np.float64)
    k_new = np.asarray(k_new, dtype=np.float64)
    v_new = np.asarray(v_new, dtype=np.float64)
    G, m, d = q.shape
    root_d = np.sqrt(float(d))
    out = np.empty_like(q)
    if cache.storage == "fp8":   # rows are encoded when they enter the cache
        k_new, v_new = round_storage(k_new, "fp8"), round_storage(v_new, "fp8")
    for i in range(m):
        cache.K = np.vstack([cache.K.reshape(-1, d), k_new[i][None, :]])
        cache.V = np.vstack([cache.V.reshape(-1, d), v_new[i][None, :]])
        cache.score = np.append(cache.score, 0.0)
        cache.pos = np.append(cache.pos, first_pos + i).astype(np.int64)
        for g in range(G):
            s = (cache.K @ q[g, i]) / root_d
            s = s - s.max()
            p = np.exp(s)
            p = p / p.sum()
            out[g, i] = p @ cache.V
            cache.score = cache.score + p
    count = cache.pos.size
    none = np.zeros(0, dtype=np.int64)
    if count <= budget:
        return out, AppendEvents(none, none, np.zeros(0), np.zeros(0, dtype=bool), cache.tau)
    assert np.all(np.diff(cache.pos) > 0)
    ret, evi = select(cache.score, budget, recent, n_sink)
    u_star, t = match(cache.K[evi], cache.K[ret])
    if math.isnan(tau_force):
        cache.tau = ema_threshold(cache.tau, float(u_star.sum() / u_star.size), beta)
        passed = u_star >= cache.tau
    else:
        passed = u_star >= tau_force
    Kc, Vc, _ = merge(cache.K[ret], cache.V[ret], cache.K[evi], cache.V[evi], u_star, t, passed,
                      cache.storage, weighted)
    events = AppendEvents(cache.pos[evi].copy(), cache.pos[ret][t].copy(), u_star, passed, cache.tau)
    cache.K, cache.V = Kc, Vc
    cache.score = cache.score[ret]
    cache.pos = cache.pos[ret]
    return out, events


# --------------------------------------------------------------------------- whole layer / config

def prefill_kv_head(Q, K, V, causal: bool = True):
    """a1-a2 for one KV head with its G query heads: Q [G, N, d].  Returns
    (O [G, N, d], group score [N] = sum over the G heads' column sums, per-head variances [G])."""
    outs, total, var = [], None, []
    for g in range(Q.shape[0]):
        o, s = prefill_attention_head(Q[g], K, V, causal)
        outs.append(o)
        var.append(head_variance(s))
        total = s.copy() if total is None else total + s
    return np.stack(outs), total, np.array(var)
