"""Brute-force transcription of the D2O steps for tiny inputs, in pure Python (lists, math).

Written independently of oracle/d2o_ref.py (no numpy kernels, no shared helpers): it builds
the full attention matrix, picks heavy hitters by repeated removal of the weakest token, and
merges with explicit weight lists.  Used only to pin the oracle on small cases."""
import math


def dot(a, b):
    return math.fsum(x * y for x, y in zip(a, b))


def attention_matrix(Q, K, causal=True):
    n, d = len(Q), len(Q[0])
    A = [[0.0] * n for _ in range(n)]
    for i in range(n):
        last = i if causal else n - 1
        logits = [dot(Q[i], K[j]) / math.sqrt(d) for j in range(last + 1)]
        m = max(logits)
        ex = [math.exp(x - m) for x in logits]
        z = math.fsum(ex)
        for j in range(last + 1):
            A[i][j] = ex[j] / z
    return A


def column_sums(A):
    n = len(A)
    return [math.fsum(A[i][j] for i in range(n)) for j in range(n)]


def attend(A, V):
    n, d = len(A), len(V[0])
    return [[math.fsum(A[i][j] * V[j][c] for j in range(n)) for c in range(d)] for i in range(n)]


def variance(s):
    mu = math.fsum(s) / len(s)
    return math.fsum((x - mu) ** 2 for x in s) / len(s)


def choose_retained(score, budget, recent, n_sink):
    """Drop the weakest middle token (ties: the later one) until the budget is met."""
    n = len(score)
    if budget >= n:
        return list(range(n)), []
    alive = list(range(n))
    dropped = []
    while len(alive) > budget:
        middle = [p for p in alive if p >= n_sink and p < n - recent]
        worst = middle[0]
        for p in middle[1:]:
            if score[p] <= score[worst]:
                worst = p
        alive.remove(worst)
        dropped.append(worst)
    return alive, sorted(dropped)


def cosine(a, b):
    na, nb = math.sqrt(dot(a, a)), math.sqrt(dot(b, b))
    if na == 0.0 or nb == 0.0:
        return 0.0
    return dot(a, b) / (na * nb)


def nearest(K, ret, evi):
    best_u, best_j = [], []
    for i in evi:
        bu, bj = -2.0, -1
        for j in ret:
            u = cosine(K[i], K[j])
            if u > bu:
                bu, bj = u, j
        best_u.append(bu)
        best_j.append(bj)
    return best_u, best_j


def merged_rows(K, V, ret, evi, best_u, best_j, passed):
    """Softmax-weighted group means: weight e for the kept token, exp(u) for each source."""
    Kc, Vc = {}, {}
    for j in ret:
        members = [(math.e, K[j], V[j])]
        for i, u, t, ok in zip(evi, best_u, best_j, passed):
            if ok and t == j:
                members.append((math.exp(u), K[i], V[i]))
        z = math.fsum(w for w, _, _ in members)
        d = len(K[j])
        if len(members) == 1:
            Kc[j], Vc[j] = list(K[j]), list(V[j])
        else:
            Kc[j] = [math.fsum(w * kk[c] for w, kk, _ in members) / z for c in range(d)]
            Vc[j] = [math.fsum(w * vv[c] for w, _, vv in members) / z for c in range(d)]
    return Kc, Vc


def compress(K, V, score, budget, recent, n_sink):
    ret, evi = choose_retained(score, budget, recent, n_sink)
    best_u, best_j = nearest(K, ret, evi)
    tau = math.fsum(best_u) / len(best_u) if evi else float("nan")
    passed = [u >= tau for u in best_u]
    Kc, Vc = merged_rows(K, V, ret, evi, best_u, best_j, passed)
    state = {"pos": list(ret), "K": [Kc[j] for j in ret], "V": [Vc[j] for j in ret],
             "score": [score[j] for j in ret], "tau": tau}
    return state, {"ret": ret, "evi": evi, "u": best_u, "t": best_j, "passed": passed}


def decode_step(state, q_heads, k_new, v_new, new_pos, budget, recent, n_sink, beta):
    state["pos"].append(new_pos)
    state["K"].append(list(k_new))
    state["V"].append(list(v_new))
    state["score"].append(0.0)
    n, d = len(state["pos"]), len(k_new)
    outs = []
    for q in q_heads:
        logits = [dot(q, kk) / math.sqrt(d) for kk in state["K"]]
        m = max(logits)
        ex = [math.exp(x - m) for x in logits]
        z = math.fsum(ex)
        p = [x / z for x in ex]
        outs.append([math.fsum(p[j] * state["V"][j][c] for j in range(n)) for c in range(d)])
        state["score"] = [s + pj for s, pj in zip(state["score"], p)]
    if n <= budget:
        return outs, (-1, -1, float("nan"))
    order = sorted(range(n), key=lambda s: state["pos"][s])
    assert order == list(range(n))
    alive, dropped = choose_retained(state["score"], budget, recent, n_sink)
    e = dropped[0]
    bu, bj = -2.0, -1
    for j in alive:
        u = cosine(state["K"][e], state["K"][j])
        if u > bu:
            bu, bj = u, j
    tau = state["tau"]
    tau = bu if math.isnan(tau) else beta * bu + (1.0 - beta) * tau
    state["tau"] = tau
    tgt = -1
    if bu >= tau:
        z = math.e + math.exp(bu)
        state["K"][bj] = [(math.e * a + math.exp(bu) * b) / z
                          for a, b in zip(state["K"][bj], state["K"][e])]
        state["V"][bj] = [(math.e * a + math.exp(bu) * b) / z
                          for a, b in zip(state["V"][bj], state["V"][e])]
        tgt = state["pos"][bj]
    ev = (state["pos"][e], tgt, bu)
    for key in ("pos", "K", "V", "score"):
        del state[key][e]
    return outs, ev


def append_chunk(state, q_heads_per_token, k_new, v_new, first_pos, budget, recent, n_sink, beta):
    """m tokens at once: each attends causally (cache + earlier tokens of the block + itself) and
    adds its softmax row to the scores; then one eviction down to the budget, matching on the
    keys as they are, threshold from the mean best similarity (EMA with the previous one), and
    a merge of every passing token into its match.  q_heads_per_token[i] = the G queries of token i."""
    m, d = len(k_new), len(k_new[0])
    outs = []
    for i in range(m):
        state["pos"].append(first_pos + i)
        state["K"].append(list(k_new[i]))
        state["V"].append(list(v_new[i]))
        state["score"].append(0.0)
        n = len(state["pos"])
        row = []
        for q in q_heads_per_token[i]:
            logits = [dot(q, kk) / math.sqrt(d) for kk in state["K"]]
            mx = max(logits)
            ex = [math.exp(x - mx) for x in logits]
            z = math.fsum(ex)
            p = [x / z for x in ex]
            row.append([math.fsum(p[j] * state["V"][j][c] for j in range(n)) for c in range(d)])
            state["score"] = [s + pj for s, pj in zip(state["score"], p)]
        outs.append(row)
    n = len(state["pos"])
    if n <= budget:
        return outs, {"evi": [], "t": [], "u": [], "passed": []}
    alive, dropped = choose_retained(state["score"], budget, recent, n_sink)
    best_u, best_j = nearest(state["K"], alive, dropped)
    mean_u = math.fsum(best_u) / len(best_u)
    tau = state["tau"]
    tau = mean_u if math.isnan(tau) else beta * mean_u + (1.0 - beta) * tau
    state["tau"] = tau
    passed = [u >= tau for u in best_u]
    Kc, Vc = merged_rows(state["K"], state["V"], alive, dropped, best_u, best_j, passed)
    ev = {"evi": [state["pos"][e] for e in dropped], "t": [state["pos"][j] for j in best_j],
          "u": best_u, "passed": passed}
    state["K"] = [Kc[j] for j in alive]
    state["V"] = [Vc[j] for j in alive]
    state["score"] = [state["score"][j] for j in alive]
    state["pos"] = [state["pos"][j] for j in alive]
    return outs, ev
