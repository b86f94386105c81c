"""Parity of the HIP path against the fp64 oracle, through the C ABI (run with -m gpu).

Protocol.  Index outputs (retained / evicted / merge-target positions, threshold flags, layer
budgets) must be identical whenever both sides decide on the same numbers: the token-level
stages are driven from the oracle's scores rounded to fp32 (the library's score type), and
decode runs start from the oracle's cache state.  The matrix-core attention itself is compared
as floats (<= 2e-3 row-normalised); where its fp32 scores then feed the top-N selection, a
differing index is accepted only if the oracle's own score gap at the selection boundary is
below 1e-4 relative (several selections are then equally valid), and every such case is
counted and printed."""
import math

import numpy as np
import pytest
import torch

from oracle import d2o_ref as ref
from paper_2406_13035_amd import binding, synth
from tests import helpers as H

pytestmark = pytest.mark.gpu

W1 = synth.WORKLOADS[1]
W2 = synth.WORKLOADS[2]
W4 = synth.WORKLOADS[4]


def _small_bf16(gqa: bool):
    w = W4 if gqa else W2
    return w.scaled(n_q_heads=4, n_kv_heads=2 if gqa else 4, n_clusters=16)


# ------------------------------------------------------------------ a1-a2: attention, scores, density

@pytest.mark.parametrize("case", ["cfg1-f32", "bf16-mha-ragged", "bf16-gqa-ragged", "bf16-short", "bf16-gqa8", "f32-gqa4-d128"])
def test_prefill_attention_scores_density(case):
    if case == "cfg1-f32":
        w, n, B, layer = W1, W1.prompt_len, 1, 0
    elif case == "bf16-mha-ragged":
        w, n, B, layer = _small_bf16(False), 1000, 1, 20
    elif case == "bf16-gqa-ragged":
        w, n, B, layer = _small_bf16(True), 777, 2, 9
    elif case == "bf16-gqa8":       # the largest group size: eight query heads on one KV head
        w, n, B, layer = W4.scaled(n_q_heads=16, n_kv_heads=2, n_clusters=16), 600, 1, 14
    elif case == "f32-gqa4-d128":   # the fp32 kernels with grouped queries and head_dim 128
        w, n, B, layer = W1.scaled(n_q_heads=8, n_kv_heads=2, head_dim=128), 333, 2, 1
    else:
        w, n, B, layer = _small_bf16(True), 50, 1, 3
    print(f"case={case} n={n} B={B}", flush=True)
    Q, K, V = H.make_inputs(w, B, layer, n)
    ctx = H.new_ctx(w, B, 1, n, n + 8)
    O = torch.empty(Q.shape, dtype=ctx.out_dtype, device=Q.device)
    ctx.d2o_prefill_attend(0, Q, K, V, O)
    torch.cuda.synchronize()
    wantO, want_score, want_var = H.oracle_prefill_layer(Q, K, V, w.group)
    err_o = H.rownorm_err(binding.tensor_to_f64(O), wantO)
    got_score = ctx.d2o_scores_export(0, n).astype(np.float64)
    err_s = H.rownorm_err(got_score, want_score)
    F, Fh = ctx.d2o_get_density(heads=True)
    rel_f = np.max(np.abs(Fh[:, 0] - want_var) / np.maximum(np.abs(want_var), 1e-12))
    print(f"  O err {err_o:.2e}  score err {err_s:.2e}  F_head rel err {rel_f:.2e}", flush=True)
    assert err_o <= H.FLOAT_TOL and err_s <= H.FLOAT_TOL and rel_f <= H.FLOAT_TOL
    np.testing.assert_allclose(F[:, 0], want_var.mean(axis=1), rtol=H.FLOAT_TOL)
    # invariant at any size: every query row sums to 1, so a head's column sums add up to n
    np.testing.assert_allclose(got_score.sum(axis=2), w.group * n, rtol=1e-4)
    ctx.close()


def test_bf16_output_storage_adds_only_its_rounding():
    """With outputs stored in bf16 (out_f32 = 0, the form the benchmark runs) every element must
    be the fp32-accumulated value rounded once: |got - want| <= 2e-3 * |row|_inf + 2^-8 * |want|
    (bf16 unit roundoff), for the prompt-phase O and for the decode step's out, whose caches
    are driven from the oracle's scores so that both sides hold the same rows."""
    w, n, B, layer, budget, recent, steps = _small_bf16(True), 777, 1, 9, 300, 75, 6
    Q, K, V = H.make_inputs(w, B, layer, n)
    ctx = H.new_ctx(w, B, 1, n, 400, out_f32=False)
    assert ctx.out_dtype == torch.bfloat16
    O = torch.empty_like(Q)
    ctx.d2o_prefill_attend(0, Q, K, V, O)
    torch.cuda.synchronize()
    wantO, score, _ = H.oracle_prefill_layer(Q, K, V, w.group)
    got = binding.tensor_to_f64(O)
    bound = H.FLOAT_TOL * np.abs(wantO).max(axis=-1, keepdims=True) + 2.0 ** -8 * np.abs(wantO)
    assert np.all(np.abs(got - wantO) <= bound)
    score32 = score.astype(np.float32)
    ctx.d2o_scores_import(0, score32)
    ctx.d2o_compress_layer(0, K, V, budget, recent)
    _, caches = H.check_compress_against_oracle(ctx, 0, K, V, score32, budget, recent, 0, w.dtype)
    q, k, v = H.decode_inputs(w, B, [layer], steps)
    qd, kd, vd = (binding.tensor_to_f64(t) for t in (q, k, v))
    out = torch.empty_like(q[0])
    G = w.group
    worst = 0.0
    for t in range(steps):
        ctx.d2o_decode_step(0, 1, q[t], k[t], v[t], out)
        torch.cuda.synchronize()
        ev, tg, _ = ctx.d2o_last_events(0)
        od = binding.tensor_to_f64(out)
        for h in range(w.n_kv_heads):
            want, e = ref.decode_step_head(caches[(0, h)], qd[t, 0, 0, h * G:(h + 1) * G], kd[t, 0, 0, h],
                                           vd[t, 0, 0, h], n + t, budget, recent, 0, w.beta)
            assert (ev[0, h], tg[0, h]) == (e.evicted_pos, e.target_pos)
            g_ = od[0, 0, h * G:(h + 1) * G]
            bnd = H.FLOAT_TOL * np.abs(want).max(axis=-1, keepdims=True) + 2.0 ** -8 * np.abs(want)
            assert np.all(np.abs(g_ - want) <= bnd), f"step {t} head {h}"
            worst = max(worst, float((np.abs(g_ - want) / bnd).max()))
    print(f"  bf16 decode out: worst element error / bound = {worst:.3f}", flush=True)
    ctx.close()


# ------------------------------------------------------------------ a4-a8 from given scores

@pytest.mark.parametrize("case,budget,recent,sink,tau_force", [
    ("cfg1-f32", 128, 64, 0, float("nan")),
    ("cfg1-f32", 128, 32, 4, float("nan")),
    ("bf16-mha", 200, 50, 0, float("nan")),
    ("bf16-gqa", [150, 333], [37, 83], 2, float("nan")),
    ("bf16-gqa", 96, 96, 0, float("nan")),          # no heavy hitters: sinks + window only
    ("bf16-gqa", 5000, 10, 0, float("nan")),        # budget >= n: nothing evicted
    ("bf16-gqa", [5000, 150], [10, 37], 0, float("nan")),  # one sequence keeps everything, the other evicts
    ("bf16-mha", 200, 50, 0, float("inf")),         # never merge: pure eviction
    ("bf16-mha", 200, 50, 1, float("-inf")),        # merge everything
])
def test_compress_from_oracle_scores(case, budget, recent, sink, tau_force):
    if case == "cfg1-f32":
        w, n, B, layer = W1, W1.prompt_len, 1, 0
    elif case == "bf16-mha":
        w, n, B, layer = _small_bf16(False), 1000, 1, 20
    else:
        w, n, B, layer = _small_bf16(True), 777, 2, 9
    print(f"case={case} budget={budget} recent={recent} sink={sink} tau_force={tau_force}", flush=True)
    Q, K, V = H.make_inputs(w, B, layer, n)
    _, score, _ = H.oracle_prefill_layer(Q, K, V, w.group)
    score32 = score.astype(np.float32)
    cap = int(np.max(budget)) + 1
    ctx = H.new_ctx(w, B, 1, n, cap + 8, n_sink=sink, tau_force=tau_force)
    ctx.d2o_scores_import(0, score32)
    ctx.d2o_compress_layer(0, K, V, budget, recent)
    torch.cuda.synchronize()
    stats, _ = H.check_compress_against_oracle(ctx, 0, K, V, score32, budget, recent, sink, w.dtype,
                                               tau_force)
    print(f"  {stats}", flush=True)
    if math.isinf(tau_force) and tau_force > 0:
        assert stats["passed"] == 0
    ctx.close()


def test_selection_ties_keep_the_lower_position():
    w, n = _small_bf16(False), 600
    Q, K, V = H.make_inputs(w, 1, 0, n)
    g = np.random.default_rng(5)
    score32 = g.integers(0, 7, size=(1, w.n_kv_heads, n)).astype(np.float32)  # massive ties
    score32[0, 1] = 0.0                                                        # all equal
    score32[0, 2, ::2] = -0.0
    ctx = H.new_ctx(w, 1, 1, n, 200)
    ctx.d2o_scores_import(0, score32)
    ctx.d2o_compress_layer(0, K, V, 150, 30)
    torch.cuda.synchronize()
    H.check_compress_against_oracle(ctx, 0, K, V, score32, 150, 30, 0, w.dtype)
    ctx.close()


def test_matching_with_duplicate_keys_takes_first_maximum():
    w, n = _small_bf16(False), 512
    Q, K, V = H.make_inputs(w, 1, 0, n)
    K = K.clone()
    K[0, :, 100:140] = K[0, :, 300:340]          # twins: evicted rows equal to retained rows
    V = V.clone()
    V[0, :, 100:140] = V[0, :, 300:340]          # (equal values too: a mean of two different
                                                 # bf16 numbers can sit exactly on a rounding tie)
    K[0, :, 400:420] = K[0, :, 300:320]          # and duplicated retained keys
    score32 = np.zeros((1, w.n_kv_heads, n), dtype=np.float32)
    score32[:, :, 300:340] = 5.0
    score32[:, :, 400:420] = 4.0
    ctx = H.new_ctx(w, 1, 1, n, 200)
    ctx.d2o_scores_import(0, score32)
    ctx.d2o_compress_layer(0, K, V, 100, 20)
    torch.cuda.synchronize()
    stats, _ = H.check_compress_against_oracle(ctx, 0, K, V, score32, 100, 20, 0, w.dtype)
    ret, evi, tgt, us, ps = ctx.d2o_prefill_events(0, 0, 0, n)
    twin = {int(e): int(t) for e, t in zip(evi, tgt)}
    assert all(twin[100 + i] == 300 + i for i in range(40))   # never the later duplicate 400+i
    ctx.close()


def test_twin_keys_with_different_values_differ_by_rounding_ties_only():
    """Evicted tokens whose key equals a retained key (u = 1) but whose value differs.  The
    merged value is then the equal-weight mean of two bf16 numbers, which sits exactly on a
    bf16 rounding tie whenever their last mantissa bits differ.  The fp64 merge arithmetic
    reaches that midpoint only up to its own rounding (exp(1.0) from the device's and the
    host's math libraries need not be the same double), so the stored element may be either
    neighbour.  Bar: every element equals the storage-rounded oracle's, or the two are adjacent
    bf16 numbers and the unrounded oracle value lies within 1e-12 (relative) of their midpoint
    (or both are fp64 rounding noise, where the two values cancel);
    rows without such a tie are identical, and every row is within 2e-3 of the unrounded
    result of Eq. 11-12 (row-normalised) plus the storage rounding of 2^-8 per element."""
    w, n = _small_bf16(False), 512
    Q, K, V = H.make_inputs(w, 1, 0, n)
    K = K.clone()
    K[0, :, 100:140] = K[0, :, 300:340]          # twins: evicted keys equal to retained keys, own values
    score32 = np.zeros((1, w.n_kv_heads, n), dtype=np.float32)
    score32[:, :, 300:340] = 5.0
    ctx = H.new_ctx(w, 1, 1, n, 200)
    ctx.d2o_scores_import(0, score32)
    ctx.d2o_compress_layer(0, K, V, 100, 20)
    torch.cuda.synchronize()
    Kd, Vd = binding.tensor_to_f64(K), binding.tensor_to_f64(V)
    flipped = total = 0
    for h in range(w.n_kv_heads):
        sc = score32[0, h].astype(np.float64)
        cache, ev = ref.compress_head(Kd[0, h], Vd[0, h], sc, 100, 20, 0, w.dtype)
        exact, _ = ref.compress_head(Kd[0, h], Vd[0, h], sc, 100, 20, 0, "f64")
        ret, evi, tgt, us, ps = ctx.d2o_prefill_events(0, 0, h, n)
        assert np.array_equal(ret, ev.retained) and np.array_equal(tgt, ev.target)
        assert np.array_equal(ps, ev.passed)
        twin = {int(e): int(t) for e, t in zip(evi, tgt)}
        assert all(twin[100 + i] == 300 + i for i in range(40))
        gK, gV, gs, gp, gtau = ctx.d2o_cache_export(0, 0, h, 101)
        assert np.array_equal(gp, cache.pos)
        for got, want, ex in ((gK, cache.K, exact.K), (gV, cache.V, exact.V)):
            bound = H.FLOAT_TOL * np.abs(ex).max(axis=1, keepdims=True) + 2.0 ** -8 * np.abs(ex)
            assert np.all(np.abs(got - ex) <= bound)
            diff = got != want
            total += diff.size
            flipped += int(diff.sum())
            if diff.any():
                g_, w_, e_ = got[diff], want[diff], ex[diff]
                rowmax = np.broadcast_to(np.abs(ex).max(axis=1, keepdims=True), ex.shape)[diff]
                # (a) values that cancel to fp64 rounding noise (v_e = -v_c): both sides store noise
                noise = np.abs(g_ - w_) <= 1e-12 * rowmax
                # (b) adjacent bf16 numbers (one unit in the 8th significant bit) around a midpoint
                #     that the unrounded result of Eq. 11-12 hits to fp64 accuracy
                mid = 0.5 * (g_ + w_)
                adjacent = np.abs(g_ - w_) <= 2.0 ** -7 * np.maximum(np.abs(g_), np.abs(w_))
                on_tie = np.abs(e_ - mid) <= 1e-12 * np.abs(mid)
                assert np.all(noise | (adjacent & on_tie)), "difference away from a rounding tie"
    print(f"  twin merges: {flipped} of {total} stored elements sit on a rounding tie and took the "
          f"other neighbour", flush=True)
    ctx.close()


def test_merge_with_long_source_lists():
    """One retained key attracts about 700 evicted tokens, another about 200, the rest a few:
    the merge visits a slot's sources in ascending order whatever their number (the library
    ranks up to 64 of them in registers, up to 512 in LDS and scans beyond that)."""
    w, n = _small_bf16(False), 2600
    Q, K, V = H.make_inputs(w, 1, 3, n)
    g = torch.Generator().manual_seed(77)
    K = K.clone()
    r1, r2 = 40, 900
    for h in range(w.n_kv_heads):
        c1, c2 = K[0, h, r1].float().cpu(), K[0, h, r2].float().cpu()
        K[0, h, 100:800] = (c1[None] + 0.05 * torch.randn(700, w.head_dim, generator=g)).to(K.dtype).to(K.device)
        K[0, h, 1000:1200] = (c2[None] + 0.05 * torch.randn(200, w.head_dim, generator=g)).to(K.dtype).to(K.device)
    score32 = np.zeros((1, w.n_kv_heads, n), dtype=np.float32)
    keep = np.concatenate([[r1, r2], np.arange(1300, 1330)])
    score32[:, :, keep] = 3.0
    ctx = H.new_ctx(w, 1, 1, n, 64, tau_force=float("-inf"))
    ctx.d2o_scores_import(0, score32)
    ctx.d2o_compress_layer(0, K, V, 40, 8)
    torch.cuda.synchronize()
    stats, _ = H.check_compress_against_oracle(ctx, 0, K, V, score32, 40, 8, 0, w.dtype, float("-inf"))
    ret, evi, tgt, us, ps = ctx.d2o_prefill_events(0, 0, 0, n)
    sizes = np.bincount(tgt[ps.astype(bool)], minlength=n)
    print(f"  {stats}; largest source lists {np.sort(sizes)[-3:]}", flush=True)
    assert sizes[r1] > 512 and 64 < sizes[r2] <= 512
    ctx.close()


# ------------------------------------------------------------------ a9-a12: decode from oracle state

def _run_decode_parity(w, n, B, layer, budget, recent, sink, steps, tau_force=float("nan"), random_scores=False,
                       merge_average=False, split_rows=0, cache_fp8=False):
    Q, K, V = H.make_inputs(w, B, layer, n)
    if random_scores:  # long prompts: the token-level stages and decode do not care where scores come from
        score32 = np.random.default_rng(n).random((B, w.n_kv_heads, n), dtype=np.float32) * w.group
    else:
        _, score, _ = H.oracle_prefill_layer(Q, K, V, w.group)
        score32 = score.astype(np.float32)
    cap = int(np.max(budget)) + 1
    ctx = H.new_ctx(w, B, 1, max(n, cap) if cache_fp8 else n, cap + 8, n_sink=sink, tau_force=tau_force,
                    merge_average=merge_average, split_rows=split_rows, cache_fp8=cache_fp8)
    ctx.d2o_scores_import(0, score32)
    ctx.d2o_compress_layer(0, K, V, budget, recent)
    _, caches = H.check_compress_against_oracle(ctx, 0, K, V, score32, budget, recent, sink,
                                                "fp8" if cache_fp8 else w.dtype, tau_force, not merge_average)
    q, k, v = H.decode_inputs(w, B, [layer], steps)
    out = torch.empty(q[0].shape, dtype=ctx.out_dtype, device=q.device)
    qd, kd, vd = (binding.tensor_to_f64(t) for t in (q, k, v))
    G = w.group
    worst = 0.0
    merges = 0
    for t in range(steps):
        ctx.d2o_decode_step(0, 1, q[t], k[t], v[t], out)
        torch.cuda.synchronize()
        ev, tg, us = ctx.d2o_last_events(0)
        od = binding.tensor_to_f64(out)
        for b in range(B):
            bud = int(np.broadcast_to(budget, (B,))[b])
            rec = int(np.broadcast_to(recent, (B,))[b])
            for h in range(w.n_kv_heads):
                want, e = ref.decode_step_head(caches[(b, h)], qd[t, 0, b, h * G:(h + 1) * G],
                                               kd[t, 0, b, h], vd[t, 0, b, h], n + t, bud, rec, sink,
                                               w.beta, tau_force, not merge_average)
                assert (ev[b, h], tg[b, h]) == (e.evicted_pos, e.target_pos), \
                    f"step {t} b={b} h={h}: gpu ({ev[b, h]}, {tg[b, h]}) oracle {e}"
                if e.evicted_pos >= 0:
                    assert abs(us[b, h] - e.u_star) < 1e-13
                    merges += e.target_pos >= 0
                worst = max(worst, H.rownorm_err(od[0, b, h * G:(h + 1) * G], want))
    assert worst <= H.FLOAT_TOL
    for (b, h), cache in caches.items():
        bud = int(np.broadcast_to(budget, (B,))[b])
        gK, gV, gs, gp, gtau = ctx.d2o_cache_export(0, b, h, bud + 1)
        assert np.array_equal(gp, cache.pos)
        np.testing.assert_allclose(gs, cache.score, rtol=1e-12)
        assert np.array_equal(gK, cache.K) and np.array_equal(gV, cache.V)
        assert (math.isnan(gtau) and math.isnan(cache.tau)) or abs(gtau - cache.tau) < 1e-13
    print(f"  decode steps={steps} worst out err {worst:.2e} merges {merges}", flush=True)
    ctx.close()


@pytest.mark.parametrize("case", ["cfg1", "bf16-mha", "bf16-gqa-ragged-budgets", "bf16-grow",
                                  "bf16-no-window", "bf16-never-merge", "bf16-long", "bf16-gqa4",
                                  "bf16-mha-many-rounds", "bf16-mha-256-steps", "bf16-beta-0", "bf16-beta-0.95"])
def test_decode_from_oracle_state(case):
    print(f"case={case}", flush=True)
    if case == "cfg1":
        _run_decode_parity(W1, 512, 1, 0, 128, 64, 0, W1.decode_steps)
    elif case == "bf16-mha":
        _run_decode_parity(_small_bf16(False), 1000, 1, 20, 300, 75, 0, 24)
    elif case == "bf16-gqa-ragged-budgets":
        _run_decode_parity(_small_bf16(True), 777, 2, 9, [150, 333], [37, 83], 2, 20)
    elif case == "bf16-grow":      # budget above the prompt: the cache grows, then starts evicting
        _run_decode_parity(_small_bf16(True), 60, 1, 3, 66, 16, 0, 14)
    elif case == "bf16-no-window":  # M = 0: the new token itself may be evicted
        _run_decode_parity(_small_bf16(False), 300, 1, 31, 40, 0, 0, 12)
    elif case == "bf16-long":      # many steps: the eviction candidates are carried from step to step
        _run_decode_parity(_small_bf16(True), 400, 2, 17, [90, 130], [20, 30], 1, 96)
    elif case == "bf16-gqa4":      # four query heads per KV head, as configurations 4 and 5
        _run_decode_parity(W4.scaled(n_q_heads=8, n_kv_heads=2, n_clusters=16), 1500, 2, 6, [700, 410],
                           [175, 100], 0, 10, random_scores=True)
    elif case == "bf16-mha-many-rounds":   # 4000 rows: sixteen workgroups per head
        _run_decode_parity(_small_bf16(False).scaled(n_q_heads=2, n_kv_heads=2), 6000, 1, 25, 4000, 1000, 0, 5,
                           random_scores=True)
    elif case.startswith("bf16-beta-"):    # the ends of the range of the EMA constant of Eq. 10
        _run_decode_parity(_small_bf16(True).scaled(beta=float(case[len("bf16-beta-"):])), 600, 1, 8, 150, 40, 0, 30)
    elif case == "bf16-mha-256-steps":     # three chunks per head, as many steps as configuration 1 generates
        _run_decode_parity(_small_bf16(False), 3000, 1, 11, 700, 150, 0, 256, random_scores=True)
    else:
        _run_decode_parity(_small_bf16(False), 500, 1, 12, 100, 25, 0, 10, tau_force=float("inf"))


@pytest.mark.parametrize("budget", [12000, 15000])
def test_decode_one_large_head_with_eight_query_heads(budget):
    """A head of 188 / 235 sub-chunks of 64 slots with 8 query heads: the closing workgroup's
    table of per-sub-chunk softmax factors fits its LDS region in the first case and does not
    in the second (it then lives in the sub-chunk records).  split_rows is set out of reach so
    that one workgroup closes the head, whatever the library would choose for this launch."""
    w = W1.scaled(n_q_heads=8, n_kv_heads=1)
    _run_decode_parity(w, 16000, 1, 0, budget, budget // 4, 0, 4, random_scores=True, split_rows=1 << 30)


@pytest.mark.parametrize("case", ["bf16-mha-16-parts", "bf16-gqa4-ragged", "bf16-gqa8-12-parts", "f32-d64",
                                  "bf16-never-merge", "bf16-average"])
def test_decode_large_heads_closed_in_parts(case):
    """split_rows lowered so that the heads of these small caches take the path of very large
    ones: their closing work is done by one workgroup per part (1, 2 or 4 chunks here) and a
    final workgroup per head.  Events, caches and scores against the oracle as in the
    single-workgroup form."""
    print(f"case={case}", flush=True)
    if case == "bf16-mha-16-parts":
        _run_decode_parity(_small_bf16(False).scaled(n_q_heads=2, n_kv_heads=2), 6000, 1, 25, 4000, 1000, 0, 5,
                           random_scores=True, split_rows=1024)
    elif case == "bf16-gqa4-ragged":   # 3 parts and 2 parts of one chunk; the smaller sequence's last part is ragged
        _run_decode_parity(W4.scaled(n_q_heads=8, n_kv_heads=2, n_clusters=16), 1500, 2, 6, [700, 410],
                           [175, 100], 0, 10, random_scores=True, split_rows=256)
    elif case == "bf16-gqa8-12-parts":
        _run_decode_parity(W1.scaled(n_q_heads=8, n_kv_heads=1), 16000, 1, 0, 12000, 3000, 0, 4,
                           random_scores=True, split_rows=4096)
    elif case == "f32-d64":
        _run_decode_parity(W1, 2000, 1, 0, 600, 150, 2, 12, random_scores=True, split_rows=256)
    elif case == "bf16-never-merge":
        _run_decode_parity(_small_bf16(False), 1500, 1, 12, 900, 225, 0, 8, tau_force=float("inf"),
                           random_scores=True, split_rows=2048)   # one part of two chunks + a ragged one
    else:
        _run_decode_parity(_small_bf16(True), 1777, 2, 9, [650, 333], [37, 83], 2, 12, merge_average=True,
                           random_scores=True, split_rows=512)    # only the first sequence's heads are large


def test_decode_large_head_after_cache_import_scans_for_the_match():
    """The first step after a cache import has no predicted candidates, so the evicted token's
    match comes from a pass over the head's keys: here in the final workgroup of the split
    form (700 entries, split_rows 256)."""
    w = _small_bf16(False).scaled(n_q_heads=1, n_kv_heads=1)
    d, n0, budget, recent, steps = w.head_dim, 900, 700, 100, 3
    g = torch.Generator().manual_seed(5)
    K = torch.randn(budget, d, generator=g).to(torch.bfloat16)
    V = torch.randn(budget, d, generator=g).to(torch.bfloat16)
    score = 1.0 + torch.rand(budget, generator=g).double().numpy()
    # survivors of a 900-token prompt: the recent window complete (Eq. 7 keeps it), the rest a random subset
    pos = np.concatenate([np.sort(np.random.default_rng(5).choice(n0 - recent, budget - recent, replace=False)),
                          np.arange(n0 - recent, n0)]).astype(np.int32)
    ctx = H.new_ctx(w, 1, 1, n0, budget + 8, beta=0.7, split_rows=256)
    ctx.d2o_layer_reserve(0, n0, budget, recent)
    Kd, Vd = binding.tensor_to_f64(K), binding.tensor_to_f64(V)
    ctx.d2o_cache_import(0, 0, 0, Kd, Vd, score, pos, 0.5, n0)
    cache = ref.HeadCache(Kd.copy(), Vd.copy(), score.copy(), pos.astype(np.int64), 0.5, "bf16")
    q = torch.randn(steps, 1, 1, 1, d, generator=g).to(torch.bfloat16)
    k = torch.randn(steps, 1, 1, 1, d, generator=g).to(torch.bfloat16)
    v = torch.randn(steps, 1, 1, 1, d, generator=g).to(torch.bfloat16)
    qg, kg, vg = q.cuda(), k.cuda(), v.cuda()
    out = torch.empty(qg[0].shape, dtype=ctx.out_dtype, device="cuda")
    for t in range(steps):
        ctx.d2o_decode_step(0, 1, qg[t], kg[t], vg[t], out)
        torch.cuda.synchronize()
        ev, tg, us = ctx.d2o_last_events(0)
        want, e = ref.decode_step_head(cache, binding.tensor_to_f64(q[t, 0, 0]), binding.tensor_to_f64(k[t, 0, 0, 0]),
                                       binding.tensor_to_f64(v[t, 0, 0, 0]), n0 + t, budget, recent, 0, 0.7)
        assert e.evicted_pos >= 0
        assert (ev[0, 0], tg[0, 0]) == (e.evicted_pos, e.target_pos), f"step {t}"
        assert abs(us[0, 0] - e.u_star) < 1e-13
        assert H.rownorm_err(binding.tensor_to_f64(out)[0, 0], want) <= H.FLOAT_TOL
    gK, gV, gs, gp, gtau = ctx.d2o_cache_export(0, 0, 0, budget + 1)
    assert np.array_equal(gp, cache.pos) and np.array_equal(gK, cache.K) and np.array_equal(gV, cache.V)
    np.testing.assert_allclose(gs, cache.score, rtol=1e-12)
    assert abs(gtau - cache.tau) < 1e-13
    ctx.close()


@pytest.mark.parametrize("case", ["bf16-gqa", "f32", "bf16-merge-everything"])
def test_average_merging_prefill_and_decode(case):
    """merge_average = 1, the alternative of the merge-policy ablation (Sec. 5): prompt-phase
    merges (groups of many sources) and the one-token merges of the decode steps against the
    oracle's plain mean."""
    print(f"case={case}", flush=True)
    if case == "bf16-gqa":
        _run_decode_parity(_small_bf16(True), 777, 2, 9, [150, 333], [37, 83], 2, 20, merge_average=True)
    elif case == "f32":
        _run_decode_parity(W1, 512, 1, 0, 128, 64, 0, W1.decode_steps, merge_average=True)
    else:
        _run_decode_parity(_small_bf16(False), 1000, 1, 20, 200, 50, 1, 12, tau_force=float("-inf"),
                           merge_average=True)


def test_decode_evicted_token_outside_the_predicted_candidates():
    """The library predicts the next evicted token (the lowest scores after a step) to compute
    its similarities during the attention pass; when the prediction misses, a second pass must
    give the same result.  State: three tokens with the lowest scores share one key u, a
    fourth, slightly higher, has another key.  Step 1 evicts nothing special; the query of step
    2 is a multiple of u, so the three predicted tokens receive almost all the attention and
    the fourth becomes the lowest: it is evicted although it was not predicted."""
    w = _small_bf16(False).scaled(n_q_heads=1, n_kv_heads=1)
    d, n0, budget, recent = w.head_dim, 60, 40, 4
    g = torch.Generator().manual_seed(11)
    K = torch.randn(budget, d, generator=g).to(torch.bfloat16)
    V = torch.randn(budget, d, generator=g).to(torch.bfloat16)
    u = (3.0 * torch.randn(d, generator=g)).to(torch.bfloat16)
    K[1] = u
    K[2] = u
    K[3] = u
    K[4] = u
    V[2] = V[1]                                           # equal values too: the mean of two different
    V[3] = V[1]                                           # bf16 numbers can sit exactly on a rounding tie
    V[4] = V[1]
    score = 1.0 + torch.rand(budget, generator=g).double().numpy()
    score[:6] = [0.05, 0.10, 0.11, 0.12, 0.13, 0.14]     # slot 0 goes first; 1-3 are then predicted; 5 has another key
    pos = np.arange(budget, dtype=np.int32)               # prompt positions 0..39 of a 60-token prompt's survivors
    ctx = H.new_ctx(w, 1, 1, n0, budget + 8, beta=0.7)
    ctx.d2o_layer_reserve(0, n0, budget, recent)
    Kd, Vd = binding.tensor_to_f64(K), binding.tensor_to_f64(V)
    ctx.d2o_cache_import(0, 0, 0, Kd, Vd, score, pos, 0.5, n0)
    cache = ref.HeadCache(Kd.copy(), Vd.copy(), score.copy(), pos.astype(np.int64), 0.5, "bf16")
    steps = 4
    q = (0.05 * torch.randn(steps, 1, 1, 1, d, generator=g)).to(torch.bfloat16)
    q[1, 0, 0, 0] = (4.0 * u.float()).to(torch.bfloat16)
    k = torch.randn(steps, 1, 1, 1, d, generator=g).to(torch.bfloat16)
    v = torch.randn(steps, 1, 1, 1, d, generator=g).to(torch.bfloat16)
    qg, kg, vg = q.cuda(), k.cuda(), v.cuda()
    out = torch.empty(qg[0].shape, dtype=ctx.out_dtype, device="cuda")
    evicted = []
    for t in range(steps):
        ctx.d2o_decode_step(0, 1, qg[t], kg[t], vg[t], out)
        torch.cuda.synchronize()
        ev, tg, us = ctx.d2o_last_events(0)
        want, e = ref.decode_step_head(cache, binding.tensor_to_f64(q[t, 0, 0]), binding.tensor_to_f64(k[t, 0, 0, 0]),
                                       binding.tensor_to_f64(v[t, 0, 0, 0]), n0 + t, budget, recent, 0, 0.7)
        assert (ev[0, 0], tg[0, 0]) == (e.evicted_pos, e.target_pos), f"step {t}"
        assert abs(us[0, 0] - e.u_star) < 1e-13
        assert H.rownorm_err(binding.tensor_to_f64(out)[0, 0], want) <= H.FLOAT_TOL
        evicted.append(e.evicted_pos)
    assert evicted[0] == 0 and evicted[1] == 5, evicted   # the scenario really took the unpredicted token
    assert ctx.d2o_candidate_misses() >= 1                # ... and the library counted the second pass over the keys
    gK, gV, gs, gp, gtau = ctx.d2o_cache_export(0, 0, 0, budget + 1)
    assert np.array_equal(gp, cache.pos) and np.array_equal(gK, cache.K) and np.array_equal(gV, cache.V)
    np.testing.assert_allclose(gs, cache.score, rtol=1e-12)
    assert abs(gtau - cache.tau) < 1e-13
    ctx.close()


# ------------------------------------------------------------------ multi-token append

def _block_inputs(w, B, layer, m, seed):
    """Q [B, Hq, m, d], K, V [B, Hkv, m, d] of a block: the workload's decode-token law."""
    qs, ks, vs = [], [], []
    for b in range(B):
        q, k, v = synth.layer_decode_inputs(w.scaled(cfg=w.cfg), b, layer + 100 * seed, m, "cpu")
        qs.append(q.transpose(0, 1))
        ks.append(k.transpose(0, 1))
        vs.append(v.transpose(0, 1))
    return (torch.stack(qs).contiguous().cuda(), torch.stack(ks).contiguous().cuda(),
            torch.stack(vs).contiguous().cuda())


def _run_append_parity(w, n, B, layer, budget, recent, sink, blocks, tau_force=float("nan"), decode_between=2,
                       cache_fp8=False):
    """Prompt compression from given scores, then blocks of new tokens (d2o_append_chunk) with a
    few single-token steps in between; outputs, events and caches against the oracle after
    every call."""
    Q, K, V = H.make_inputs(w, B, layer, n)
    score32 = np.random.default_rng(n + layer).random((B, w.n_kv_heads, n), dtype=np.float32) * w.group
    bud = np.broadcast_to(np.asarray(budget), (B,))
    rec = np.broadcast_to(np.asarray(recent), (B,))
    ctx = H.new_ctx(w, B, 1, max(n, int(bud.max()) + max(blocks)), int(bud.max()) + max(blocks) + 8, n_sink=sink,
                    tau_force=tau_force, max_append=max(blocks), cache_fp8=cache_fp8)
    ctx.d2o_scores_import(0, score32)
    ctx.d2o_compress_layer(0, K, V, budget, recent)
    _, caches = H.check_compress_against_oracle(ctx, 0, K, V, score32, budget, recent, sink,
                                                "fp8" if cache_fp8 else w.dtype, tau_force)
    G, pos, worst, evicted_total = w.group, n, 0.0, 0
    dq, dk, dv = H.decode_inputs(w, B, [layer], decode_between * len(blocks) + 1)
    dqd, dkd, dvd = (binding.tensor_to_f64(t) for t in (dq, dk, dv))
    dout = torch.empty(dq[0].shape, dtype=ctx.out_dtype, device=dq.device)
    step = 0
    for bi, m in enumerate(blocks):
        Qb, Kb, Vb = _block_inputs(w, B, layer, m, bi + 1)
        Ob = torch.empty(Qb.shape, dtype=ctx.out_dtype, device=Qb.device)
        ctx.d2o_append_chunk(0, Qb, Kb, Vb, Ob)
        torch.cuda.synchronize()
        qd, kd, vd, od = (binding.tensor_to_f64(t) for t in (Qb, Kb, Vb, Ob))
        for b in range(B):
            for h in range(w.n_kv_heads):
                cache = caches[(b, h)]
                want, ev = ref.append_chunk_head(cache, qd[b, h * G:(h + 1) * G], kd[b, h], vd[b, h], pos,
                                                 int(bud[b]), int(rec[b]), sink, w.beta, tau_force)
                worst = max(worst, H.rownorm_err(od[b, h * G:(h + 1) * G], want))
                evi, tgt, us, ps = ctx.d2o_append_events(0, b, h, int(bud[b]) + m)
                assert np.array_equal(evi, ev.evicted), f"block {bi} b={b} h={h}: evicted differ"
                assert np.array_equal(tgt, ev.target), f"block {bi} b={b} h={h}: targets differ"
                assert np.array_equal(ps, ev.passed), f"block {bi} b={b} h={h}: flags differ"
                if len(evi):
                    assert np.max(np.abs(us - ev.u_star)) < 1e-13
                evicted_total += len(evi)
                gK, gV, gs, gp, gtau = ctx.d2o_cache_export(0, b, h, int(bud[b]) + m)
                assert np.array_equal(gp, cache.pos), f"block {bi} b={b} h={h}: cache positions differ"
                np.testing.assert_allclose(gs, cache.score, rtol=1e-12)
                assert np.array_equal(gK, cache.K) and np.array_equal(gV, cache.V)
                assert (math.isnan(gtau) and math.isnan(cache.tau)) or abs(gtau - cache.tau) < 1e-13
        pos += m
        for _ in range(decode_between):      # single-token steps continue on the block's result
            ctx.d2o_decode_step(0, 1, dq[step], dk[step], dv[step], dout)
            torch.cuda.synchronize()
            e_, t_, _ = ctx.d2o_last_events(0)
            dd = binding.tensor_to_f64(dout)
            for b in range(B):
                for h in range(w.n_kv_heads):
                    want, e = ref.decode_step_head(caches[(b, h)], dqd[step, 0, b, h * G:(h + 1) * G],
                                                   dkd[step, 0, b, h], dvd[step, 0, b, h], pos, int(bud[b]),
                                                   int(rec[b]), sink, w.beta, tau_force)
                    assert (e_[b, h], t_[b, h]) == (e.evicted_pos, e.target_pos), f"step after block {bi}"
                    worst = max(worst, H.rownorm_err(dd[0, b, h * G:(h + 1) * G], want))
            pos += 1
            step += 1
    assert worst <= H.FLOAT_TOL
    print(f"  blocks {blocks}: worst out err {worst:.2e}, evicted {evicted_total}", flush=True)
    ctx.close()


@pytest.mark.parametrize("case", ["bf16-gqa", "f32", "bf16-mha-sinks", "bf16-no-window", "bf16-grow",
                                  "bf16-never-merge", "multi-turn"])
def test_append_chunk_against_oracle(case):
    print(f"case={case}", flush=True)
    if case == "bf16-gqa":          # ragged budgets, blocks of different sizes, a block of one token
        _run_append_parity(_small_bf16(True), 777, 2, 9, [150, 333], [37, 83], 0, [40, 7, 1, 64])
    elif case == "f32":
        _run_append_parity(W1, 512, 1, 0, 128, 64, 0, [16, 50])
    elif case == "bf16-mha-sinks":
        _run_append_parity(_small_bf16(False), 1000, 1, 20, 300, 75, 4, [100, 33])
    elif case == "bf16-no-window":  # M = 0: tokens of the block itself can be evicted
        _run_append_parity(_small_bf16(False), 300, 1, 31, 40, 0, 0, [12, 30])
    elif case == "bf16-grow":       # budget above the prompt: the first block fits, the second evicts
        _run_append_parity(_small_bf16(True), 60, 1, 3, 100, 25, 0, [30, 30])
    elif case == "bf16-never-merge":
        _run_append_parity(_small_bf16(False), 500, 1, 12, 100, 25, 0, [20, 20], tau_force=float("inf"))
    else:
        # the shape of the multi-turn experiment (appendix): budget 2048 = 48 heavy hitters + 2000
        # recent tokens, whole turns of a few hundred tokens appended at once
        w = _small_bf16(False).scaled(n_q_heads=2, n_kv_heads=2)
        _run_append_parity(w, 2500, 1, 7, 2048, 2000, 0, [300, 120], decode_between=1)


# ------------------------------------------------------------------ per-head allocation, ragged per-head caches

def test_per_head_budgets_ragged_caches_prefill_decode_and_append():
    """App. A.8 end to end on two layers: per-head variances from the library's attention pass,
    per-(layer, KV head) budgets from d2o_allocate_budgets_heads (equal to the oracle's on the
    same variances), d2o_compress_layer_heads with those budgets (every KV head its own cache
    size and recent window), then generation steps over both layers in one call and a block of
    tokens on each layer: every head against the oracle run with that head's budget."""
    w = _small_bf16(True).scaled(n_layers=2)            # 4 query heads, 2 KV heads
    n, B, L, G = 900, 2, 2, 2
    total = int(0.2 * n * L * w.n_kv_heads)
    data = [H.make_inputs(w, B, l, n) for l in range(L)]
    probe = H.new_ctx(w, B, L, n, 8)                      # a first context only measures the densities
    for l in range(L):
        probe.d2o_prefill_attend(l, *data[l], None)
    _, Fh = probe.d2o_get_density(heads=True)            # [B, L, Hq]
    probe.close()
    S = np.stack([binding.d2o_allocate_budgets_heads(Fh[b], w.n_kv_heads, n, total, 32) for b in range(B)])
    for b in range(B):
        assert np.array_equal(S[b], ref.allocate_budgets_heads(Fh[b], G, n, total, 32)) and int(S[b].sum()) == total
    assert len(set(S.reshape(-1).tolist())) > 4, S      # really ragged
    print(f"  per-head budgets [b][layer][kv head]: {S.tolist()}", flush=True)
    m = 24
    ctx = H.new_ctx(w, B, L, n, int(S.sum(axis=1).max()) + L * (m + 8), max_append=m)
    caches = {}
    for l in range(L):
        Q, K, V = data[l]
        bud = S[:, l, :]                                 # [B, Hkv]
        rec = bud // 4
        score32 = np.random.default_rng(l).random((B, w.n_kv_heads, n), dtype=np.float32) * G
        ctx.d2o_scores_import(l, score32)
        ctx.d2o_compress_layer_heads(l, K, V, bud, rec)
        torch.cuda.synchronize()
        Kd, Vd = binding.tensor_to_f64(K), binding.tensor_to_f64(V)
        for b in range(B):
            for h in range(w.n_kv_heads):
                cache, ev = ref.compress_head(Kd[b, h], Vd[b, h], score32[b, h].astype(np.float64), int(bud[b, h]),
                                              int(rec[b, h]), 0, w.dtype)
                ret, evi, tgt, us, ps = ctx.d2o_prefill_events(l, b, h, n)
                assert np.array_equal(ret, ev.retained) and np.array_equal(tgt, ev.target)
                assert np.array_equal(ps, ev.passed) and len(ret) == int(bud[b, h])
                gK, gV, gs, gp, gtau = ctx.d2o_cache_export(l, b, h, int(bud[b, h]) + 1)
                assert np.array_equal(gp, cache.pos) and np.array_equal(gK, cache.K) and np.array_equal(gV, cache.V)
                caches[(l, b, h)] = cache
    steps = 5
    q, k, v = H.decode_inputs(w, B, list(range(L)), steps)
    qd, kd, vd = (binding.tensor_to_f64(t) for t in (q, k, v))
    out = torch.empty(q[0].shape, dtype=ctx.out_dtype, device=q.device)
    worst, pos = 0.0, n
    for t in range(steps):
        ctx.d2o_decode_step(0, L, q[t], k[t], v[t], out)
        torch.cuda.synchronize()
        od = binding.tensor_to_f64(out)
        for l in range(L):
            e_, t_, _ = ctx.d2o_last_events(l)
            for b in range(B):
                for h in range(w.n_kv_heads):
                    bud = int(S[b, l, h])
                    want, e = ref.decode_step_head(caches[(l, b, h)], qd[t, l, b, h * G:(h + 1) * G], kd[t, l, b, h],
                                                   vd[t, l, b, h], pos, bud, bud // 4, 0, w.beta)
                    assert (e_[b, h], t_[b, h]) == (e.evicted_pos, e.target_pos), f"step {t} l={l} b={b} h={h}"
                    worst = max(worst, H.rownorm_err(od[l, b, h * G:(h + 1) * G], want))
        pos += 1
    for l in range(L):
        Qb, Kb, Vb = _block_inputs(w, B, l, m, 3)
        Ob = torch.empty(Qb.shape, dtype=ctx.out_dtype, device=Qb.device)
        ctx.d2o_append_chunk(l, Qb, Kb, Vb, Ob)
        torch.cuda.synchronize()
        bq, bk, bv, bo = (binding.tensor_to_f64(x) for x in (Qb, Kb, Vb, Ob))
        for b in range(B):
            for h in range(w.n_kv_heads):
                bud = int(S[b, l, h])
                want, ev = ref.append_chunk_head(caches[(l, b, h)], bq[b, h * G:(h + 1) * G], bk[b, h], bv[b, h], pos,
                                                 bud, bud // 4, 0, w.beta)
                worst = max(worst, H.rownorm_err(bo[b, h * G:(h + 1) * G], want))
                evi, tgt, us, ps = ctx.d2o_append_events(l, b, h, bud + m)
                assert np.array_equal(evi, ev.evicted) and np.array_equal(tgt, ev.target) and np.array_equal(ps, ev.passed)
                gK, gV, gs, gp, gtau = ctx.d2o_cache_export(l, b, h, bud + m)
                cache = caches[(l, b, h)]
                assert np.array_equal(gp, cache.pos) and np.array_equal(gK, cache.K) and np.array_equal(gV, cache.V)
                np.testing.assert_allclose(gs, cache.score, rtol=1e-12)
    assert worst <= H.FLOAT_TOL
    print(f"  worst output err {worst:.2e}", flush=True)
    ctx.close()


# ------------------------------------------------------------------ whole path, free running

def test_cfg1_end_to_end_free_running():
    """Config 1 in full: prefill attention on the GPU feeds its own selection.  Selection
    differences against the oracle must be explained by a score gap below 1e-4 relative at
    the boundary; everything downstream is then compared on the heads that agree."""
    w, n = W1, W1.prompt_len
    Q, K, V = H.make_inputs(w, 1, 0, n)
    ctx = H.new_ctx(w, 1, 1, n, w.fixed_budget + 8)
    O = torch.empty(Q.shape, dtype=ctx.out_dtype, device=Q.device)
    ctx.d2o_prefill_compress(0, Q, K, V, w.fixed_budget, w.fixed_recent, O)
    torch.cuda.synchronize()
    wantO, score, var = H.oracle_prefill_layer(Q, K, V, w.group)
    assert H.rownorm_err(binding.tensor_to_f64(O), wantO) <= H.FLOAT_TOL
    Kd, Vd = binding.tensor_to_f64(K), binding.tensor_to_f64(V)
    q, k, v = H.decode_inputs(w, 1, [0], w.decode_steps)
    qd, kd, vd = (binding.tensor_to_f64(t) for t in (q, k, v))
    agree, explained = [], 0
    caches = {}
    for h in range(w.n_kv_heads):
        cache, ev = ref.compress_head(Kd[0, h], Vd[0, h], score[0, h], w.fixed_budget, w.fixed_recent, 0,
                                      w.dtype)
        ret, evi, tgt, us, ps = ctx.d2o_prefill_events(0, 0, h, n)
        if np.array_equal(ret, ev.retained):
            agree.append(h)
            assert np.array_equal(tgt, ev.target) and np.array_equal(ps, ev.passed)
            caches[h] = cache
        else:
            diff = np.setxor1d(ret, ev.retained)
            mid = np.arange(0, n - w.fixed_recent)
            kth = np.sort(score[0, h][mid])[::-1][w.fixed_budget - w.fixed_recent - 1]
            assert np.all(np.abs(score[0, h][diff] - kth) <= 1e-4 * abs(kth)), "unexplained selection"
            explained += 1
    print(f"  heads agreeing {len(agree)}/{w.n_kv_heads}, margin-explained {explained}", flush=True)
    out = torch.empty(q[0].shape, dtype=ctx.out_dtype, device=q.device)
    for t in range(w.decode_steps):
        ctx.d2o_decode_step(0, 1, q[t], k[t], v[t], out)
        torch.cuda.synchronize()
        ev_, tg_, us_ = ctx.d2o_last_events(0)
        od = binding.tensor_to_f64(out)
        for h in list(agree):
            want, e = ref.decode_step_head(caches[h], qd[t, 0, 0, h:h + 1], kd[t, 0, 0, h], vd[t, 0, 0, h],
                                           n + t, w.fixed_budget, w.fixed_recent, 0, w.beta)
            assert H.rownorm_err(od[0, 0, h:h + 1], want) <= H.FLOAT_TOL
            assert (ev_[0, h], tg_[0, h]) == (e.evicted_pos, e.target_pos)
    ctx.close()


def test_decode_all_layers_in_one_call_equals_one_call_per_layer():
    """The layers of a decode call are independent (Sec. 4: every stage lives inside one layer's
    KV group), so one call over three layers of very different budgets and three calls of one
    layer each must leave bit-identical outputs, events and caches.  Covers the layer table of
    the multi-layer launch (layers sorted by size, chunk -> layer search, per-layer strides)."""
    w, n, L, B, steps = _small_bf16(True), 700, 3, 2, 6
    budgets = [np.array([520, 300], np.int32), np.array([40, 64], np.int32), np.array([260, 130], np.int32)]
    ctxs = [H.new_ctx(w, B, L, n, sum(int(b.max()) for b in budgets) + 3 * 8) for _ in range(2)]
    for l in range(L):
        Q, K, V = H.make_inputs(w, B, l, n)
        for ctx in ctxs:
            ctx.d2o_prefill_compress(l, Q, K, V, budgets[l], budgets[l] // 4)
    q, k, v = H.decode_inputs(w, B, list(range(L)), steps)
    outs = [torch.zeros(q[0].shape, dtype=ctxs[0].out_dtype, device=q.device) for _ in range(2)]
    for t in range(steps):
        ctxs[0].d2o_decode_step(0, L, q[t], k[t], v[t], outs[0])
        for l in (2, 0, 1):  # any order
            ctxs[1].d2o_decode_step(l, 1, q[t][l:l + 1], k[t][l:l + 1], v[t][l:l + 1], outs[1][l:l + 1])
        torch.cuda.synchronize()
        assert torch.equal(outs[0], outs[1]), f"outputs differ at step {t}"
        for l in range(L):
            ea, eb = ctxs[0].d2o_last_events(l), ctxs[1].d2o_last_events(l)
            for x, y in zip(ea, eb):
                assert np.array_equal(x, y, equal_nan=True), f"events differ at step {t}, layer {l}"
    for l in range(L):
        for b in range(B):
            for h in range(w.n_kv_heads):
                ca = ctxs[0].d2o_cache_export(l, b, h, int(budgets[l][b]) + 1)
                cb = ctxs[1].d2o_cache_export(l, b, h, int(budgets[l][b]) + 1)
                for x, y in zip(ca, cb):
                    assert np.array_equal(np.asarray(x), np.asarray(y)), f"cache differs: layer {l}, b {b}, head {h}"
    for ctx in ctxs:
        ctx.close()


def _run_multi_layer_decode(w, n, layers, budgets, recents, steps, split_rows=0, cache_fp8=False, ranges=None):
    """Several layers in one decode call per step (or in one call per range of layers, `ranges` =
    [(first, count), ...]), every head against the oracle at every step.  Returns the number of
    evictions per layer."""
    B, L = 1, len(layers)
    ctx = H.new_ctx(w, B, L, max([n] + [b + 1 for b in budgets]) if cache_fp8 else n, sum(budgets) + 8 * L,
                    split_rows=split_rows, cache_fp8=cache_fp8)
    caches = {}
    for li, layer in enumerate(layers):
        Q, K, V = H.make_inputs(w, B, layer, n)
        score32 = np.random.default_rng(layer).random((B, w.n_kv_heads, n), dtype=np.float32) * w.group
        ctx.d2o_scores_import(li, score32)
        ctx.d2o_compress_layer(li, K, V, budgets[li], recents[li])
        _, c = H.check_compress_against_oracle(ctx, li, K, V, score32, budgets[li], recents[li], 0,
                                               "fp8" if cache_fp8 else w.dtype)
        for (b, h), cache in c.items():
            caches[(li, h)] = cache
    q, k, v = H.decode_inputs(w, B, layers, steps)
    qd, kd, vd = (binding.tensor_to_f64(t) for t in (q, k, v))
    out = torch.empty(q[0].shape, dtype=ctx.out_dtype, device=q.device)
    G, worst, evictions = w.group, 0.0, [0] * L
    for t in range(steps):
        for (l0, nl) in (ranges or [(0, L)]):
            ctx.d2o_decode_step(l0, nl, q[t][l0:l0 + nl], k[t][l0:l0 + nl], v[t][l0:l0 + nl], out[l0:l0 + nl])
        torch.cuda.synchronize()
        od = binding.tensor_to_f64(out)
        for li in range(L):
            ev, tg, us = ctx.d2o_last_events(li)
            for h in range(w.n_kv_heads):
                want, e = ref.decode_step_head(caches[(li, h)], qd[t, li, 0, h * G:(h + 1) * G], kd[t, li, 0, h],
                                               vd[t, li, 0, h], n + t, budgets[li], recents[li], 0, w.beta)
                assert (ev[0, h], tg[0, h]) == (e.evicted_pos, e.target_pos), f"step {t} layer {li} head {h}"
                evictions[li] += e.evicted_pos >= 0
                worst = max(worst, H.rownorm_err(od[li, 0, h * G:(h + 1) * G], want))
    assert worst <= H.FLOAT_TOL
    for (li, h), cache in caches.items():
        gK, gV, gs, gp, gtau = ctx.d2o_cache_export(li, 0, h, budgets[li] + 1)
        assert np.array_equal(gp, cache.pos) and np.array_equal(gK, cache.K) and np.array_equal(gV, cache.V)
        np.testing.assert_allclose(gs, cache.score, rtol=1e-12)
    print(f"  {steps} steps, worst out err {worst:.2e}, evictions per layer {evictions}", flush=True)
    ctx.close()
    return evictions


def test_decode_growing_cache_crosses_chunk_boundaries_in_a_multi_layer_call():
    """Two layers in one call: layer 0's budget is above its prompt, so its caches grow by one
    token per step through 256 and 512 entries (the sizes at which a new workgroup joins a
    head) and then start evicting; layer 1 evicts from the first
    step.  Every step's events and outputs against the oracle, final caches identical."""
    w, n, steps = _small_bf16(True), 250, 275
    budgets = [520, 100]
    ev = _run_multi_layer_decode(w, n, [4, 11], budgets, [130, 25], steps)
    assert ev[0] == (steps - (budgets[0] - n)) * w.n_kv_heads and ev[1] == steps * w.n_kv_heads


def test_decode_growing_cache_becomes_large_in_a_multi_layer_call():
    """The same two layers with split_rows = 256: layer 0's heads pass from the single-workgroup
    closing form to the split form while they grow (and gain a second and a third part);
    layer 1's heads stay small, so both forms run in every launch."""
    w, n, steps = _small_bf16(True), 250, 275
    budgets = [520, 100]
    ev = _run_multi_layer_decode(w, n, [4, 11], budgets, [130, 25], steps, split_rows=256)
    assert ev[0] == (steps - (budgets[0] - n)) * w.n_kv_heads and ev[1] == steps * w.n_kv_heads


def test_decode_layers_of_very_different_sizes_in_one_call():
    """Three layers in one call whose caches hold 10500, 200 and 3000 rows (42, 1 and 12 workgroups
    per head): each head against the oracle at every step."""
    w = _small_bf16(False).scaled(n_q_heads=2, n_kv_heads=2)
    ev = _run_multi_layer_decode(w, 12000, [2, 30, 17], [10500, 200, 3000], [2600, 50, 750], 5)
    assert ev == [10, 10, 10]


def test_decode_more_layers_than_one_launch_takes():
    """70 layers in one call (a launch's layer table holds 64: the call becomes two groups of
    launches), budgets cycling through four sizes: every head against the oracle at every step."""
    w = _small_bf16(True)
    L = 70
    budgets = [[48, 300, 64, 130][i % 4] for i in range(L)]
    ev = _run_multi_layer_decode(w, 350, list(range(L)), budgets, [b // 4 for b in budgets], 3)
    assert ev == [3 * w.n_kv_heads] * L


def test_decode_in_calls_over_layer_ranges():
    """A step issued as two calls, layers [0, 1) and [1, 4): the second range starts above layer 0
    and holds layers of different sizes; every head against the oracle at every step."""
    w = _small_bf16(True)
    ev = _run_multi_layer_decode(w, 900, [7, 1, 19, 28], [300, 520, 64, 700], [75, 130, 16, 175], 6,
                                 ranges=[(0, 1), (1, 3)])
    assert ev == [6 * w.n_kv_heads] * 4


def test_density_to_budgets_to_compress_free_running():
    """The chain a1 -> a2 -> a3 -> a4-a8 on the library's own numbers (Sec. 4.1 Eq. 4-5, App. A.2;
    Sec. 4.2): four layers of the 32-head stack's law at N = 4000 (ragged against every tile
    size), the library's densities against the oracle's, the library's budgets from its own
    densities equal to the oracle's allocation of the same densities and summing to the total,
    then compression with those budgets driven by the library's OWN scores.  The oracle runs
    on its own scores; where the retained sets differ, every differing position must have an
    oracle score within 1e-4 (relative) of the oracle's score at the selection boundary (such
    selections are equally valid under fp32 score rounding); heads that agree must agree on
    every later index output as well.  Prints explained / total."""
    w = W2.scaled(n_q_heads=4, n_kv_heads=4, n_layers=4)
    n, L, B = 4000, 4, 1
    total = int(math.floor(0.2 * n * L + 0.5))
    ctx = H.new_ctx(w, B, L, n, total + L + 8)
    inputs, want_scores, F_ref = [], [], np.zeros(L)
    for l in range(L):
        Q, K, V = H.make_inputs(w, B, l, n)
        ctx.d2o_prefill_attend(l, Q, K, V, None)
        _, score, var = H.oracle_prefill_layer(Q, K, V, w.group)
        F_ref[l] = ref.layer_density([score[0, h] for h in range(w.n_kv_heads)])   # G = 1: a KV head's scores are its query head's
        assert abs(F_ref[l] - var[0].mean()) <= 1e-12 * F_ref[l]
        inputs.append((K, V))
        want_scores.append(score)
    F = ctx.d2o_get_density()[0]
    np.testing.assert_allclose(F, F_ref, rtol=H.FLOAT_TOL)
    S = binding.d2o_allocate_budgets(F, n, total, 64)
    assert np.array_equal(S, ref.allocate_budgets(F, n, total, 64)) and int(S.sum()) == total
    S_ref = ref.allocate_budgets(F_ref, n, total, 64)
    print(f"  F gpu {F}  oracle {F_ref}\n  budgets from the library's F {S}, from the oracle's F {S_ref}", flush=True)
    assert np.max(np.abs(S.astype(np.int64) - S_ref)) <= max(2, int(2 * H.FLOAT_TOL * n))
    agree = explained = 0
    for l in range(L):
        K, V = inputs[l]
        bud, rec = int(S[l]), int(S[l]) // 4
        ctx.d2o_compress_layer(l, K, V, bud, rec)
        torch.cuda.synchronize()
        Kd, Vd = binding.tensor_to_f64(K), binding.tensor_to_f64(V)
        for h in range(w.n_kv_heads):
            sc = want_scores[l][0, h]
            cache, ev = ref.compress_head(Kd[0, h], Vd[0, h], sc, bud, rec, 0, w.dtype)
            ret, evi, tgt, us, ps = ctx.d2o_prefill_events(l, 0, h, n)
            assert len(ret) == min(bud, n) and len(ret) + len(evi) == n
            if np.array_equal(ret, ev.retained):
                agree += 1
                assert np.array_equal(tgt, ev.target) and np.array_equal(ps, ev.passed)
                assert np.max(np.abs(us - ev.u_star)) < 1e-13
                gK, gV, gs, gp, gtau = ctx.d2o_cache_export(l, 0, h, bud + 1)
                assert np.array_equal(gp, cache.pos) and np.array_equal(gK, cache.K) and np.array_equal(gV, cache.V)
            else:
                diff = np.setxor1d(ret, ev.retained)
                mid = sc[: n - rec]
                kth = np.sort(mid)[::-1][bud - rec - 1]
                assert np.all(np.abs(sc[diff] - kth) <= 1e-4 * abs(kth)), f"unexplained selection l={l} h={h}"
                explained += 1
    print(f"  free running at n={n}: heads identical to the oracle {agree}/{L * w.n_kv_heads}, "
          f"margin-explained {explained}", flush=True)
    ctx.close()


def test_prefill_and_decode_enqueue_without_host_synchronisation():
    """d2o_prefill_attend, d2o_compress_layer and d2o_decode_step only enqueue work: two layers
    and one generation step issued back to back on a side stream, with no synchronisation
    between the calls, leave exactly what the same calls leave when the host waits after each."""
    w, n, B, L = _small_bf16(True), 700, 2, 2
    budgets = [np.array([200, 120], np.int32), np.array([90, 333], np.int32)]
    data = [H.make_inputs(w, B, l, n) for l in range(L)]
    q, k, v = H.decode_inputs(w, B, list(range(L)), 1)
    results = []
    for mode in ("sync", "async"):
        ctx = H.new_ctx(w, B, L, n, sum(int(b.max()) for b in budgets) + 16)
        out = torch.zeros(q[0].shape, dtype=ctx.out_dtype, device=q.device)
        stream = torch.cuda.Stream() if mode == "async" else torch.cuda.current_stream()
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            for l in range(L):
                Q, K, V = data[l]
                ctx.d2o_prefill_attend(l, Q, K, V, None)
                if mode == "sync":
                    torch.cuda.synchronize()
                ctx.d2o_compress_layer(l, K, V, budgets[l], budgets[l] // 4)
                if mode == "sync":
                    torch.cuda.synchronize()
            ctx.d2o_decode_step(0, L, q[0], k[0], v[0], out)
        torch.cuda.synchronize()
        state = [out.clone()]
        for l in range(L):
            state += [torch.from_numpy(x.copy()) for x in ctx.d2o_last_events(l)]
            for b in range(B):
                for h in range(w.n_kv_heads):
                    state += [torch.from_numpy(np.ascontiguousarray(x)) if isinstance(x, np.ndarray) else torch.tensor(x)
                              for x in ctx.d2o_cache_export(l, b, h, int(budgets[l][b]) + 1)]
        results.append(state)
        ctx.close()
    assert len(results[0]) == len(results[1])
    for a, b_ in zip(*results):
        assert torch.equal(torch.nan_to_num(a.double().cpu(), nan=-7.0), torch.nan_to_num(b_.double().cpu(), nan=-7.0))


def test_timing_aid_samples_decode_launches():
    """d2o_timing_enable(n): every launch of the prompt-phase kernels is timed, the decode kernels
    on every n-th launch (the n-th, 2n-th, ...); reading forgets what it returned."""
    w, n = _small_bf16(False), 300
    Q, K, V = H.make_inputs(w, 1, 0, n)
    ctx = H.new_ctx(w, 1, 1, n, 64 + 8)
    ctx.d2o_timing_enable(4)
    ctx.d2o_prefill_compress(0, Q, K, V, 64, 16)
    q, k, v = H.decode_inputs(w, 1, [0], 9)
    out = torch.empty(q[0].shape, dtype=ctx.out_dtype, device=q.device)
    for t in range(9):
        ctx.d2o_decode_step(0, 1, q[t], k[t], v[t], out)
    for name, want in (("attn_fwd", 1), ("colsum", 1), ("merge", 1), ("decode_attend", 2), ("decode_prepare", 2)):
        ms, cnt = ctx.d2o_timing_read(name)
        assert cnt == want and ms > 0.0, (name, cnt, ms)
    assert ctx.d2o_timing_read("decode_attend") == (0.0, 0)
    ctx.d2o_timing_enable(0)
    ctx.d2o_decode_step(0, 1, q[0], k[0], v[0], out)
    assert ctx.d2o_timing_read("decode_attend")[1] == 0
    ctx.close()


def test_error_paths_return_codes():
    w, n = _small_bf16(False), 256
    Q, K, V = H.make_inputs(w, 1, 0, n)
    ctx = H.new_ctx(w, 1, 2, n, 300)
    with pytest.raises(binding.D2OError):      # compress before attend
        ctx.d2o_compress_layer(0, K, V, 64, 16)
    ctx.d2o_prefill_attend(0, Q, K, V, None)
    with pytest.raises(binding.D2OError):      # budget below sinks + window
        ctx.d2o_compress_layer(0, K, V, 10, 16)
    with pytest.raises(binding.D2OError):      # capacity: 400 + 1 > 300 slots
        ctx.d2o_compress_layer(0, K, V, 400, 16)
    ctx.d2o_compress_layer(0, K, V, 64, 16)
    with pytest.raises(binding.D2OError):      # second compress of the same layer
        ctx.d2o_compress_layer(0, K, V, 64, 16)
    q, k, v = H.decode_inputs(w, 1, [0, 1], 1)
    out = torch.empty(q[0].shape, dtype=ctx.out_dtype, device=q.device)
    with pytest.raises(binding.D2OError):      # layer 1 was never compressed
        ctx.d2o_decode_step(0, 2, q[0], k[0], v[0], out)
    ctx.d2o_decode_step(0, 1, q[0][:1], k[0][:1], v[0][:1], out[:1])
    torch.cuda.synchronize()
    ctx.close()


# ------------------------------------------------------------------ repeatability, non-finite inputs

def _token_major(t):
    """The same [b][head][token][d] values as a strided view of a [b][token][head][d + 8] buffer
    (the layout a model's projection leaves them in, with padded rows)."""
    B, Hh, n, d = t.shape
    buf = torch.zeros((B, n, Hh, d + 8), dtype=t.dtype, device=t.device)
    buf[..., :d] = t.permute(0, 2, 1, 3)
    return buf[..., :d].permute(0, 2, 1, 3)


def _padded_heads(t):
    """[layers][b][head][d] values as a view with padded head and sequence strides."""
    L, B, Hh, d = t.shape
    buf = torch.zeros((L, B + 1, Hh + 1, d + 16), dtype=t.dtype, device=t.device)
    buf[:, :B, :Hh, :d] = t
    return buf[:, :B, :Hh, :d]


def _whole_path_in(ctx, w, n, budget, recent, steps, m, strided=False):
    """Prompt phase on the library's own scores, generation steps, a block: every result as bytes.
    strided: every tensor handed to the library is a non-contiguous view."""
    lay4 = _token_major if strided else (lambda x: x)
    layd = _padded_heads if strided else (lambda x: x)
    Q, K, V = (lay4(x) for x in H.make_inputs(w, 2, 5, n))
    O = lay4(torch.empty(Q.shape, dtype=ctx.out_dtype, device=Q.device))
    ctx.d2o_prefill_compress(0, Q, K, V, budget, recent, O)
    raw = lambda x: x.contiguous().view(torch.uint8).cpu().numpy().tobytes()  # the values in logical order
    got = [raw(O), ctx.d2o_scores_export(0, n).tobytes()]
    got += [a.tobytes() for a in ctx.d2o_get_density(heads=True)]
    q, k, v = H.decode_inputs(w, 2, [5], steps)
    out = layd(torch.empty(q[0].shape, dtype=ctx.out_dtype, device=q.device))
    for t in range(steps):
        ctx.d2o_decode_step(0, 1, layd(q[t]), layd(k[t]), layd(v[t]), out)
        got.append(raw(out))
        got += [a.tobytes() for a in ctx.d2o_last_events(0)]
    Qb, Kb, Vb = (lay4(x) for x in _block_inputs(w, 2, 5, m, 1))
    Ob = lay4(torch.empty(Qb.shape, dtype=ctx.out_dtype, device=Qb.device))
    ctx.d2o_append_chunk(0, Qb, Kb, Vb, Ob)
    got.append(raw(Ob))
    for b in range(2):
        for h in range(w.n_kv_heads):
            gK, gV, gs, gp, gtau = ctx.d2o_cache_export(0, b, h, budget + m)
            got += [gK.tobytes(), gV.tobytes(), gs.tobytes(), gp.tobytes(), np.float64(gtau).tobytes()]
    return got


@pytest.mark.parametrize("cache_fp8", [False, True])
def test_two_runs_give_the_same_bits(cache_fp8):
    """No result depends on the order in which workgroups run (no floating-point atomics, fixed
    summation trees, ordered merge sources): the whole path - attention outputs, scores,
    densities, every generation step's outputs and events, a block append, the final caches -
    gives identical bytes when it is run again in a fresh context, and again in the first
    context after d2o_reset (which therefore leaves nothing of the first run behind)."""
    w = _small_bf16(True)
    n, budget, recent, steps, m = 1500, 300, 60, 12, 40
    mk = lambda: H.new_ctx(w, 2, 1, max(n, budget + m), budget + m + 8, max_append=m, cache_fp8=cache_fp8)
    ctx = mk()
    first = _whole_path_in(ctx, w, n, budget, recent, steps, m)
    ctx.d2o_reset()
    again = _whole_path_in(ctx, w, n, budget, recent, steps, m)
    ctx.close()
    ctx = mk()
    fresh = _whole_path_in(ctx, w, n, budget, recent, steps, m)
    ctx.close()
    assert len(first) == len(again) == len(fresh)
    for i, (a, b, c) in enumerate(zip(first, again, fresh)):
        assert a == b, f"result {i} differs after d2o_reset"
        assert a == c, f"result {i} differs between two contexts"


def test_strided_views_give_the_same_bits_as_contiguous_tensors():
    """Every tensor argument is a view with its own strides (d contiguous).  Prompt tensors as
    views of token-major buffers with padded rows, generation-step tensors with padded head and
    sequence strides, outputs written through such views: the whole path gives the bytes it
    gives on contiguous tensors."""
    w = _small_bf16(True)
    n, budget, recent, steps, m = 700, 200, 40, 6, 24
    results = []
    for strided in (False, True):
        ctx = H.new_ctx(w, 2, 1, max(n, budget + m), budget + m + 8, max_append=m, out_f32=False)
        results.append(_whole_path_in(ctx, w, n, budget, recent, steps, m, strided=strided))
        ctx.close()
    assert len(results[0]) == len(results[1])
    for i, (a, b) in enumerate(zip(*results)):
        assert a == b, f"result {i} differs between contiguous and strided tensors"


def test_non_finite_inputs_reach_the_density_and_the_budget_call_rejects_them():
    """The kernels do not scan their inputs.  A NaN in a query or a key row spreads through the
    softmax normaliser into that head's column sums, variance and the layer's density, and
    d2o_allocate_budgets answers a non-finite density with an error; the other layer's density
    stays finite."""
    w, n = _small_bf16(False), 600
    ctx = H.new_ctx(w, 1, 2, n, n + 8)
    for layer, poison in ((0, None), (1, "q")):
        Q, K, V = H.make_inputs(w, 1, layer, n)
        if poison:
            Q[0, 2, 17, 5] = float("nan")
        ctx.d2o_prefill_attend(layer, Q, K, V, None)
    torch.cuda.synchronize()
    F = ctx.d2o_get_density()
    assert np.isfinite(F[0, 0]) and not np.isfinite(F[0, 1])
    with pytest.raises(binding.D2OError):
        binding.d2o_allocate_budgets(F[0], n, 300, 16)
    ctx.close()


# ------------------------------------------------------------------ degenerate sizes

@pytest.mark.parametrize("n,budget,recent", [
    (1, 1, 0),      # a prompt of one token, a cache of one entry: every step evicts one of two and merges
    (1, 1, 1),      # ... with the window covering the whole cache: the oldest of the two leaves
    (2, 1, 0),      # the prompt phase itself evicts: one token merged into the only retained one
    (5, 2, 1),
    (33, 3, 0),     # one row past a 32-row tile
    (3, 8, 2),      # budget above the prompt: nothing to evict until the cache has grown to it
])
def test_tiny_prompts_and_budgets_through_every_call(n, budget, recent):
    """The smallest shapes the calls accept: attention and scores of the prompt, compression,
    single-token steps and blocks (one token, then more tokens than the cache holds), bf16 and
    fp32, all against the oracle."""
    for w in (_small_bf16(True), W1):
        print(f"n={n} budget={budget} recent={recent} dtype={w.dtype}", flush=True)
        Q, K, V = H.make_inputs(w, 1, 2, n)
        ctx = H.new_ctx(w, 1, 1, n, n + 8)
        O = torch.empty(Q.shape, dtype=ctx.out_dtype, device=Q.device)
        ctx.d2o_prefill_attend(0, Q, K, V, O)
        torch.cuda.synchronize()
        wantO, want_score, want_var = H.oracle_prefill_layer(Q, K, V, w.group)
        assert H.rownorm_err(binding.tensor_to_f64(O), wantO) <= H.FLOAT_TOL
        assert H.rownorm_err(ctx.d2o_scores_export(0, n).astype(np.float64), want_score) <= H.FLOAT_TOL
        _, Fh = ctx.d2o_get_density(heads=True)
        assert np.max(np.abs(Fh[:, 0] - want_var)) <= H.FLOAT_TOL * max(1.0, float(np.abs(want_var).max()))
        ctx.close()
        _run_decode_parity(w, n, 1, 2, budget, recent, 0, 6)
        _run_append_parity(w, n, 1, 2, budget, recent, 0, [1, budget + 3, 2], decode_between=1)


# ------------------------------------------------------------------ upstream: Q, K, V from the hidden states

@pytest.mark.parametrize("B,n,hidden,Hq,Hkv,pos0,base", [
    (1, 300, 256, 4, 2, 0, 10000.0),          # ragged against the 256-token tile, grouped-query
    (2, 513, 128, 2, 2, 4000, 500000.0),      # two sequences, a position offset, a large rotary base
    (1, 64, 1024, 3, 1, 131000, 10000.0),     # positions beyond 10^5
])
def test_qkv_projection_with_rotary_embedding(B, n, hidden, Hq, Hkv, pos0, base):
    """Sec. 3 Eq. 1 on the matrix cores (bf16 operands, fp32 accumulation, bf16 results) against
    the oracle's fp64 product and rotation: |got - want| <= 2e-3 * |row|_inf + 2^-8 * |want|
    (the second term is the result's own bf16 rounding)."""
    d = 128
    g = torch.Generator().manual_seed(B * 1000 + n)
    X = torch.randn(B, n, hidden, generator=g).to(torch.bfloat16)
    W = (torch.randn((Hq + 2 * Hkv) * d, hidden, generator=g) / hidden ** 0.5).to(torch.bfloat16)
    Q, K, V = binding.d2o_qkv_project(X.cuda(), W.cuda(), Hq, Hkv, d, pos0, base)
    torch.cuda.synchronize()
    Xd, Wd = binding.tensor_to_f64(X), binding.tensor_to_f64(W)
    worst = 0.0
    for b in range(B):
        wq, wk, wv = ref.qkv_project(Xd[b], Wd, Hq, Hkv, d, pos0, base)
        for got, want in ((Q[b], wq), (K[b], wk), (V[b], wv)):
            got = binding.tensor_to_f64(got)
            bound = H.FLOAT_TOL * np.abs(want).max(axis=-1, keepdims=True) + 2.0 ** -8 * np.abs(want)
            assert np.all(np.abs(got - want) <= bound)
            worst = max(worst, float((np.abs(got - want) / bound).max()))
    print(f"  worst element error / bound = {worst:.3f}", flush=True)


def test_fp32_tensors_with_head_dim_128():
    """The fp32 kernels at head_dim 128 (the benchmark's fp32 configuration has 64): attention,
    scores and densities, compression, generation steps and blocks of tokens."""
    w = W1.scaled(head_dim=128, n_q_heads=4, n_kv_heads=2)
    n, B = 300, 1
    Q, K, V = H.make_inputs(w, B, 0, n)
    ctx = H.new_ctx(w, B, 1, n, 200)
    O = torch.empty(Q.shape, dtype=ctx.out_dtype, device=Q.device)
    ctx.d2o_prefill_attend(0, Q, K, V, O)
    want_O, want_score, want_var = H.oracle_prefill_layer(Q, K, V, w.group)
    assert H.rownorm_err(binding.tensor_to_f64(O), want_O) <= H.FLOAT_TOL
    got_score = ctx.d2o_scores_export(0, n)
    assert np.abs(got_score - want_score).max() <= H.FLOAT_TOL * np.abs(want_score).max()
    ctx.close()
    _run_decode_parity(w, n, B, 0, 96, 24, 1, 10)
    _run_append_parity(w, n, B, 0, 96, 24, 0, [20, 33])
