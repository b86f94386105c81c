"""Host-side checks that need no GPU: the built library loads, exports every symbol the
header declares, rejects bad configurations, and its host-only budget allocation (Sec. 4.1
Eq. 5) returns exactly the oracle's integers."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import d2o_ref as ref
from paper_2406_13035_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2406_13035_amd import build
        build.build()
    return binding.load_library()


def test_library_exports_every_declared_symbol(lib):
    text = open(os.path.join(ROOT, "include", "d2o.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = sorted(set(re.findall(r"\b(d2o_[a-z_0-9]+)\s*\(", text)))
    assert len(declared) >= 15
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in d2o.h but not exported"
    assert sorted(binding.EXPORTS) == declared


def test_workspace_query_and_config_validation(lib):
    cfg = binding.d2o_config(1, 32, 32, 32, 128, 4096, 30000, binding.D2O_BF16, 0, 0.7, float("nan"), 0)
    p, s = C.c_size_t(), C.c_size_t()
    assert lib.d2o_workspace_bytes(C.byref(cfg), C.byref(p), C.byref(s)) == 0
    assert p.value > 32 * 30000 * 128 * 2 * 2 and s.value > 0
    bad = binding.d2o_config(1, 32, 32, 5, 128, 4096, 30000, binding.D2O_BF16, 0, 0.7, float("nan"), 0)
    assert lib.d2o_workspace_bytes(C.byref(bad), C.byref(p), C.byref(s)) == -1      # Hq % Hkv
    bad = binding.d2o_config(1, 32, 32, 32, 96, 4096, 30000, binding.D2O_BF16, 0, 0.7, float("nan"), 0)
    assert lib.d2o_workspace_bytes(C.byref(bad), C.byref(p), C.byref(s)) == -2      # head_dim
    bad = binding.d2o_config(1, 32, 32, 32, 128, 4096, 30000, binding.D2O_BF16, 0, 1.0, float("nan"), 0)
    assert lib.d2o_workspace_bytes(C.byref(bad), C.byref(p), C.byref(s)) == -1      # beta = 1
    for hkv in (8, 4, 2, 1, 3, 6):    # G = 24 / Hkv = 3, 6, 12, 24 have no decode kernel; 8 and 4 do
        cfg = binding.d2o_config(1, 2, 24, hkv, 128, 512, 300, binding.D2O_BF16, 0, 0.7, float("nan"), 0)
        g = 24 // hkv
        want = 0 if g in (1, 2, 4, 8) else -2
        assert lib.d2o_workspace_bytes(C.byref(cfg), C.byref(p), C.byref(s)) == want, (hkv, g)
    # the fields this build added: split_rows (0 or >= 256), cache_fp8 (bf16 tensors only)
    def cfg_with(**kw):
        c = binding.d2o_config(1, 32, 32, 32, 128, 4096, 30000, binding.D2O_BF16, 0, 0.7, float("nan"), 0)
        for k, v in kw.items():
            setattr(c, k, v)
        return c
    assert lib.d2o_workspace_bytes(C.byref(cfg_with(split_rows=100)), C.byref(p), C.byref(s)) == -1
    assert lib.d2o_workspace_bytes(C.byref(cfg_with(split_rows=256)), C.byref(p), C.byref(s)) == 0
    assert lib.d2o_workspace_bytes(C.byref(cfg_with(cache_fp8=2)), C.byref(p), C.byref(s)) == -1
    assert lib.d2o_workspace_bytes(C.byref(cfg_with(cache_fp8=1, dtype=binding.D2O_F32)), C.byref(p), C.byref(s)) == -2
    assert lib.d2o_workspace_bytes(C.byref(cfg_with()), C.byref(p), C.byref(s)) == 0
    bf16_bytes = p.value
    assert lib.d2o_workspace_bytes(C.byref(cfg_with(cache_fp8=1)), C.byref(p), C.byref(s)) == 0
    # K and V rows shrink from 256 to 128 bytes (+ 1 byte per row for the power of two)
    assert bf16_bytes - p.value > 0.9 * 32 * 30000 * 128 * 2


def test_allocate_budgets_matches_oracle_bit_for_bit(lib):
    g = np.random.default_rng(2024)
    for trial in range(300):
        L = int(g.integers(1, 40))
        scale = g.choice([0.01, 0.3, 1.0, 10.0, 300.0, 5000.0])
        F = g.uniform(0, 1, size=L) * scale
        if trial % 7 == 0:
            F[:] = F[0]                        # equal densities: uniform allocation
        if trial % 11 == 0:
            F[g.integers(0, L)] = 0.0
        n = int(g.choice([512, 4096, 32768]))
        lo = int(g.choice([0, 1, 16, 64]))
        tot = int(g.integers(L * lo, L * n + 1))
        want = ref.allocate_budgets(F, n, tot, lo)
        got = binding.d2o_allocate_budgets(F, n, tot, lo)
        assert np.array_equal(got, want), (F, n, tot, lo, got, want)
    with pytest.raises(binding.D2OError):
        binding.d2o_allocate_budgets(np.zeros(4), 100, 4 * 100 + 1, 0)
    with pytest.raises(binding.D2OError):
        binding.d2o_allocate_budgets(np.array([0.0, np.nan]), 100, 50, 0)


def test_allocation_policies_match_oracle_bit_for_bit(lib):
    """The designs of alpha_l compared in Sec. 5 (allocation-policy analysis): the host function
    against the oracle on random densities, bounds and totals."""
    g = np.random.default_rng(77)
    for trial in range(200):
        L = int(g.integers(1, 40))
        F = g.uniform(0.01, 1, size=L) * g.choice([0.3, 1.0, 10.0, 300.0])
        if trial % 7 == 0:
            F[:] = F[0]
        n = int(g.choice([512, 4096, 32768]))
        lo = int(g.choice([0, 1, 16, 64]))
        tot = int(g.integers(L * lo, L * n + 1))
        for pol in ref.ALLOCATION_POLICIES:
            want = ref.allocate_budgets(F, n, tot, lo, policy=pol)
            got = binding.d2o_allocate_budgets_policy(pol, F, n, tot, lo)
            assert np.array_equal(got, want), (pol, F, n, tot, lo, got, want)
        assert np.array_equal(binding.d2o_allocate_budgets_policy("softmax", F, n, tot, lo),
                              binding.d2o_allocate_budgets(F, n, tot, lo))
    with pytest.raises(binding.D2OError):
        binding.d2o_allocate_budgets_policy("reciprocal", np.array([1.0, 0.0]), 100, 50, 0)
    assert lib.d2o_allocate_budgets_policy(7, None, 1, 1, 1, 0, None) < 0


def test_benchmark_allocations_have_the_stated_totals(lib):
    from paper_2406_13035_amd import synth
    for cfg in (2, 3, 4, 5):
        w = synth.WORKLOADS[cfg]
        F = np.linspace(0.05, 4.0, w.n_layers)
        S = binding.d2o_allocate_budgets(F, w.prompt_len, w.total_budget(), 64)
        assert S.sum() == w.total_budget() and S.min() >= 64 and S.max() <= w.prompt_len
        assert np.all(np.diff(S) <= 0)


def test_allocate_budgets_heads_matches_oracle_bit_for_bit(lib):
    g = np.random.default_rng(77)
    for trial in range(100):
        L, Hkv = int(g.integers(1, 12)), int(g.choice([1, 2, 4, 8]))
        G = int(g.choice([1, 2, 4]))
        F = g.uniform(0, 1, size=(L, Hkv * G)) * g.choice([0.1, 1.0, 30.0, 2000.0])
        n = int(g.choice([512, 4096, 32768]))
        lo = int(g.choice([0, 1, 64]))
        tot = int(g.integers(L * Hkv * lo, L * Hkv * n + 1))
        want = ref.allocate_budgets_heads(F, G, n, tot, lo)
        got = binding.d2o_allocate_budgets_heads(F, Hkv, n, tot, lo)
        assert np.array_equal(got, want), (trial, L, Hkv, G)
        assert int(got.sum()) == tot
