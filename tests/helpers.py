"""Shared helpers of the parity tests: drive the HIP library and the oracle on the same inputs."""
from __future__ import annotations

import math

import numpy as np
import torch

from oracle import d2o_ref as ref
from paper_2406_13035_amd import binding, synth

FLOAT_TOL = 2e-3  # max row-normalised error on attention outputs and merged K/V (bf16 inputs,
                  # fp32 accumulation), the bar the benchmark definition states


def rownorm_err(got: np.ndarray, want: np.ndarray) -> float:
    """max over rows of |got - want|_inf / |want|_inf (a row = one token's vector)."""
    got = np.asarray(got, dtype=np.float64).reshape(-1, got.shape[-1])
    want = np.asarray(want, dtype=np.float64).reshape(-1, want.shape[-1])
    den = np.abs(want).max(axis=1)
    den = np.where(den > 0, den, 1.0)
    return float((np.abs(got - want).max(axis=1) / den).max())


def make_inputs(w: synth.Workload, b_count: int, layer: int, n: int, device="cuda"):
    """Q [B, Hq, n, d], K, V [B, Hkv, n, d] on `device` in the workload dtype."""
    qs, ks, vs = [], [], []
    for b in range(b_count):
        Q, K, V = synth.layer_inputs(w, b, layer, "cpu", n)
        qs.append(Q)
        ks.append(K)
        vs.append(V)
    Q, K, V = torch.stack(qs), torch.stack(ks), torch.stack(vs)
    return Q.to(device), K.to(device), V.to(device)


def oracle_prefill_layer(Q, K, V, G):
    """Oracle a1-a2 for every (b, kv head).  Returns O [B,Hq,n,d], score [B,Hkv,n], var [B,Hq]."""
    Qd, Kd, Vd = (binding.tensor_to_f64(t) for t in (Q, K, V))
    B, Hq, n, d = Qd.shape
    Hkv = Kd.shape[1]
    O = np.zeros_like(Qd)
    score = np.zeros((B, Hkv, n))
    var = np.zeros((B, Hq))
    for b in range(B):
        for h in range(Hkv):
            o, s, v = ref.prefill_kv_head(Qd[b, h * G:(h + 1) * G], Kd[b, h], Vd[b, h])
            O[b, h * G:(h + 1) * G] = o
            score[b, h] = s
            var[b, h * G:(h + 1) * G] = v
    return O, score, var


def new_ctx(w: synth.Workload, batch, n_layers, max_n, slots, n_sink=0, beta=None,
            tau_force=float("nan"), out_f32=True, merge_average=False, max_append=0, split_rows=0,
            cache_fp8=False):
    """Contexts of the parity tests write attention outputs in fp32 unless asked otherwise, so
    that the float bar applies to the arithmetic and not to bf16 output storage."""
    return binding.D2O(batch, n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim, max_n, slots,
                       dtype=w.dtype, n_sink=n_sink, beta=w.beta if beta is None else beta,
                       tau_force=tau_force, out_f32=out_f32, merge_average=merge_average,
                       max_append=max_append, split_rows=split_rows, cache_fp8=cache_fp8)


def check_compress_against_oracle(ctx, layer, K, V, score32, budget, recent, n_sink, storage,
                                  tau_force=float("nan"), weighted=True):
    """After ctx.d2o_compress_layer ran on given fp32 scores: compare every (b, kv head) with the
    oracle fed the same fp32 scores.  Index outputs must be identical; floats near-exact."""
    Kd, Vd = binding.tensor_to_f64(K), binding.tensor_to_f64(V)
    B, Hkv, n, d = Kd.shape
    stats = {"heads": 0, "evicted": 0, "passed": 0}
    caches = {}
    for b in range(B):
        for h in range(Hkv):
            bud = int(np.broadcast_to(budget, (B,))[b])
            rec = int(np.broadcast_to(recent, (B,))[b])
            cache, ev = ref.compress_head(Kd[b, h], Vd[b, h], score32[b, h].astype(np.float64), bud,
                                          rec, n_sink, storage, tau_force, weighted)
            ret, evi, tgt, us, ps = ctx.d2o_prefill_events(layer, b, h, n)
            assert np.array_equal(ret, ev.retained), f"retained differ b={b} h={h}"
            assert np.array_equal(evi, ev.evicted), f"evicted differ b={b} h={h}"
            assert np.array_equal(tgt, ev.target), f"merge targets differ b={b} h={h}"
            assert np.array_equal(ps, ev.passed), f"threshold flags differ b={b} h={h}"
            if len(evi):
                assert np.max(np.abs(us - ev.u_star)) < 1e-13
            gK, gV, gs, gp, gtau = ctx.d2o_cache_export(layer, b, h, min(bud, n) + 1)
            assert np.array_equal(gp, cache.pos)
            assert np.array_equal(gs, cache.score)
            if len(evi):
                assert abs(gtau - cache.tau) < 1e-13
            else:
                assert math.isnan(gtau) and math.isnan(cache.tau)
            assert rownorm_err(gK, cache.K) <= FLOAT_TOL and rownorm_err(gV, cache.V) <= FLOAT_TOL
            stats["kv_exact"] = stats.get("kv_exact", True) and np.array_equal(gK, cache.K) \
                and np.array_equal(gV, cache.V)
            stats["heads"] += 1
            stats["evicted"] += len(evi)
            stats["passed"] += int(ev.passed.sum())
            caches[(b, h)] = cache
    return stats, caches


def decode_inputs(w: synth.Workload, batch, layers, steps, device="cuda"):
    """q [steps, L, B, Hq, d], k, v [steps, L, B, Hkv, d] for the listed layers."""
    qs, ks, vs = [], [], []
    for l in layers:
        ql, kl, vl = [], [], []
        for b in range(batch):
            q, k, v = synth.layer_decode_inputs(w, b, l, steps, "cpu")
            ql.append(q)
            kl.append(k)
            vl.append(v)
        qs.append(torch.stack(ql, 1))
        ks.append(torch.stack(kl, 1))
        vs.append(torch.stack(vl, 1))
    q, k, v = torch.stack(qs, 1), torch.stack(ks, 1), torch.stack(vs, 1)
    return q.to(device).contiguous(), k.to(device).contiguous(), v.to(device).contiguous()
