"""d2o_decode_step_static, the decode step for callers that cannot allocate: its kernels keep
their temporaries in a static device array inside the library.  It must leave exactly what
d2o_decode_step leaves (outputs, events, caches, bit for bit), also when the array still holds
a larger earlier call's contents, and must refuse contexts whose step does not fit."""
import numpy as np
import pytest
import torch

from paper_2406_13035_amd import binding, synth
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _pair_run(w, n, B, L, budgets, steps, split_rows=0):
    """Two contexts with identical state; one steps through d2o_decode_step, the other through
    d2o_decode_step_static.  Returns nothing; asserts bit-identical results at every step."""
    slots = sum(int(np.max(b)) for b in budgets) + 8 * L
    ctxs = [H.new_ctx(w, B, L, n, slots, out_f32=False, split_rows=split_rows) for _ in range(2)]
    for l in range(L):
        Q, K, V = H.make_inputs(w, B, l, n)
        for ctx in ctxs:
            ctx.d2o_prefill_compress(l, Q, K, V, budgets[l], np.asarray(budgets[l]) // 4)
    q, k, v = H.decode_inputs(w, B, list(range(L)), steps)
    outs = [torch.zeros(q[0].shape, dtype=ctxs[0].out_dtype, device=q.device) for _ in range(2)]
    for t in range(steps):
        ctxs[0].d2o_decode_step(0, L, q[t], k[t], v[t], outs[0])
        ctxs[1].d2o_decode_step_static(0, L, q[t], k[t], v[t], outs[1])
        torch.cuda.synchronize()
        assert torch.equal(outs[0], outs[1]), f"outputs differ at step {t}"
        for l in range(L):
            for x, y in zip(ctxs[0].d2o_last_events(l), ctxs[1].d2o_last_events(l)):
                assert np.array_equal(x, y, equal_nan=True), f"events differ at step {t}, layer {l}"
    for l in range(L):
        for b in range(B):
            cap = int(np.broadcast_to(budgets[l], (B,))[b]) + 1
            for h in range(w.n_kv_heads):
                for x, y in zip(ctxs[0].d2o_cache_export(l, b, h, cap), ctxs[1].d2o_cache_export(l, b, h, cap)):
                    assert np.array_equal(np.asarray(x), np.asarray(y), equal_nan=True), \
                        f"cache differs: layer {l}, sequence {b}, head {h}"
    for ctx in ctxs:
        ctx.close()


def test_static_scratch_decode_equals_decode_step_then_again_on_a_smaller_input():
    w = synth.WORKLOADS[4].scaled(n_q_heads=4, n_kv_heads=2, n_clusters=16)
    print("call 1: three layers, two sequences, budgets up to 520", flush=True)
    _pair_run(w, 700, 2, 3, [np.array([520, 300], np.int32), np.array([40, 64], np.int32),
                             np.array([260, 130], np.int32)], 6)
    print("call 2: smaller input (one layer, one sequence, budget 48) on the array the first call used", flush=True)
    _pair_run(w, 200, 1, 1, [np.array([48], np.int32)], 5)
    print("call 3: the first input with the large-head closing form (its part records live in the array too)", flush=True)
    _pair_run(w, 700, 2, 3, [np.array([520, 300], np.int32), np.array([40, 64], np.int32),
                             np.array([260, 130], np.int32)], 6, split_rows=256)


def test_static_scratch_rejects_a_context_that_does_not_fit():
    # eight query heads per KV head and 140000 slots: the per-slot softmax terms alone need 72 MB
    n = 64
    ctx = binding.D2O(1, 1, 64, 8, 128, n, 140000, dtype="bf16")
    ctx.d2o_layer_reserve(0, n, 139000, 0)
    q = torch.zeros((1, 1, 64, 128), dtype=torch.bfloat16, device="cuda:0")
    kv = torch.zeros((1, 1, 8, 128), dtype=torch.bfloat16, device="cuda:0")
    out = torch.empty_like(q)
    with pytest.raises(binding.D2OError, match="static array holds 67108864"):
        ctx.d2o_decode_step_static(0, 1, q, kv, kv, out)
    ctx.d2o_decode_step(0, 1, q, kv, kv, out)      # the workspace form still runs on the same context
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    ctx.close()
