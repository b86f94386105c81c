"""Shape, law and determinism checks of the seeded workload generator (no method arithmetic)."""
import math

import torch

from paper_2406_13035_amd import synth


def test_workload_table_matches_the_benchmark_configs():
    w = synth.WORKLOADS
    assert (w[1].n_q_heads, w[1].head_dim, w[1].prompt_len, w[1].decode_steps) == (4, 64, 512, 16)
    assert w[1].fixed_budget == 128 and w[1].fixed_recent == 64 and w[1].beta == 0.5
    assert (w[2].n_layers, w[2].n_q_heads, w[2].n_kv_heads, w[2].prompt_len) == (32, 32, 32, 4096)
    assert w[2].total_budget() == 26214 and w[3].total_budget() == 104858
    assert w[4].total_budget() == 52429 and w[5].total_budget() == 209715
    assert w[4].group == 4 and w[4].batch == 16 and w[5].n_sink_keys == 16
    assert w[2].query_scale(0) == 0.5 and abs(w[2].query_scale(31) - 3.0) < 1e-12


def test_generator_is_deterministic_and_has_the_stated_structure():
    w = synth.WORKLOADS[2]
    Q, K, V = synth.kv_head_inputs(w, 0, 5, 3, n=512)
    Q2, K2, V2 = synth.kv_head_inputs(w, 0, 5, 3, n=512)
    assert torch.equal(Q, Q2) and torch.equal(K, K2) and torch.equal(V, V2)
    assert Q.dtype == torch.bfloat16 and Q.shape == (1, 512, 128) and K.shape == (512, 128)
    Kb = synth.kv_head_inputs(w, 0, 5, 4, n=512)[1]
    assert not torch.equal(K, Kb)
    norms = K.float().norm(dim=1)
    # centre norm sqrt(d) plus noise 0.3 per dim; token 0 is scaled x4
    base = math.sqrt(128 + 128 * 0.09)
    assert abs(float(norms[1:].mean()) - base) < 0.3
    assert abs(float(norms[0]) - 4 * base) < 4.0
    L = synth.layer_inputs(synth.WORKLOADS[1], 0, 0)
    assert L[0].shape == (4, 512, 64) and L[0].dtype == torch.float32
    q, k, v = synth.layer_decode_inputs(synth.WORKLOADS[4], 1, 2, 3)
    assert q.shape == (3, 32, 128) and k.shape == (3, 8, 128)
    assert len(synth.sink_positions(synth.WORKLOADS[5], 0, 0, 0, 131072)) == 16
