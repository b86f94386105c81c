"""Seeded synthetic workloads for the D2O hot path.

This module only draws random inputs (queries, keys, values) with the shapes and
structure of the five benchmark configurations.  It holds none of the method's
arithmetic: no attention, no scores, no selection, no merging.  Both the HIP
path's tests/bench and the CPU oracle's tests consume the tensors it returns.

Generator (per sequence b, layer l, KV head h, C clusters, head dim d):
  centres  c_m = sqrt(d) * g_m / |g_m|,  g_m ~ N(0, I_d)
  key j    k_j = c_{z_j} + 0.3 * N(0, I),  z_j ~ U{0..C-1};  sink keys scaled x4
  query i  q_i = a_l * (c_{z'_i} + 0.5 * N(0, I)),  z'_i ~ U (centres of its KV head)
  value j  v_j ~ N(0, I)
bf16 configurations are generated in fp32 and rounded once to bf16.
Every (config, b, layer, kv head, purpose) has its own seed, so single heads can
be regenerated without the rest.
"""
from __future__ import annotations

import dataclasses
import math

import torch

BASE_SEED = 20240613


@dataclasses.dataclass(frozen=True)
class Workload:
    cfg: int                 # 1..5, position in the benchmark's config list
    name: str
    dtype: str               # "f32" or "bf16"
    batch: int
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    prompt_len: int
    decode_steps: int
    n_clusters: int
    rho: float | None        # compression ratio of the total budget (None: fixed budget)
    fixed_budget: int | None  # per-layer budget when rho is None
    fixed_recent: int | None  # recent window when rho is None
    beta: float
    n_sink_keys: int         # number of keys scaled x4
    random_sinks: bool       # False: token 0 is the sink; True: random positions
    query_scale_lo: float
    query_scale_hi: float

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    def query_scale(self, layer: int) -> float:
        if self.n_layers == 1:
            return self.query_scale_lo
        t = layer / (self.n_layers - 1)
        return self.query_scale_lo + (self.query_scale_hi - self.query_scale_lo) * t

    def total_budget(self) -> int:
        """Total slots per KV head over all layers: round(rho * N * L)."""
        if self.rho is None:
            return self.fixed_budget * self.n_layers
        return int(math.floor(self.rho * self.prompt_len * self.n_layers + 0.5))

    def scaled(self, **kw) -> "Workload":
        """Same law, other sizes (used by tests for reduced shapes)."""
        return dataclasses.replace(self, **kw)


WORKLOADS = {
    1: Workload(1, "tiny-f32", "f32", 1, 1, 4, 4, 64, 512, 16, 32, None, 128, 64, 0.5,
                1, False, 1.0, 1.0),
    2: Workload(2, "llama2-7b-4k", "bf16", 1, 32, 32, 32, 128, 4096, 256, 64, 0.2, None, None,
                0.7, 1, False, 0.5, 3.0),
    3: Workload(3, "llama2-7b-32k", "bf16", 1, 32, 32, 32, 128, 32768, 512, 64, 0.1, None, None,
                0.7, 1, False, 0.5, 3.0),
    4: Workload(4, "llama3-8b-gqa-8k-b16", "bf16", 16, 32, 32, 8, 128, 8192, 512, 64, 0.2, None,
                None, 0.7, 1, False, 0.5, 3.0),
    5: Workload(5, "gqa-128k", "bf16", 1, 32, 32, 8, 128, 131072, 1024, 256, 0.05, None, None,
                0.7, 16, True, 0.5, 3.0),
}

_PURPOSE = {"centres": 0, "keys": 1, "values": 2, "queries": 3, "sinks": 4,
            "dec_keys": 5, "dec_values": 6, "dec_queries": 7}


def _seed(w: Workload, b: int, layer: int, kv_head: int, purpose: str, extra: int = 0) -> int:
    s = BASE_SEED + 1000 * w.cfg + b
    # mix the remaining coordinates into a 63-bit seed (plain integer hashing)
    x = (s * 0x9E3779B97F4A7C15 + layer * 0xBF58476D1CE4E5B9 + kv_head * 0x94D049BB133111EB
         + _PURPOSE[purpose] * 0xD6E8FEB86659FD93 + extra * 0xA0761D6478BD642F) & ((1 << 63) - 1)
    x ^= x >> 31
    return x & ((1 << 63) - 1)


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _centres(w: Workload, b: int, layer: int, h: int, device) -> torch.Tensor:
    g = _gen(device, _seed(w, b, layer, h, "centres"))
    c = torch.randn(w.n_clusters, w.head_dim, generator=g, device=device, dtype=torch.float32)
    return c * (math.sqrt(w.head_dim) / c.norm(dim=1, keepdim=True))


def sink_positions(w: Workload, b: int, layer: int, h: int, n: int) -> list[int]:
    if not w.random_sinks:
        return list(range(min(w.n_sink_keys, n)))
    g = _gen("cpu", _seed(w, b, layer, h, "sinks"))
    perm = torch.randperm(n, generator=g)[: w.n_sink_keys]
    return sorted(int(x) for x in perm)


def kv_head_inputs(w: Workload, b: int, layer: int, h: int, device="cpu", n: int | None = None):
    """Prompt tensors of one KV head: (Q [G, n, d], K [n, d], V [n, d]) in the workload dtype."""
    n = w.prompt_len if n is None else n
    d, C, G = w.head_dim, w.n_clusters, w.group
    cen = _centres(w, b, layer, h, device)
    gk = _gen(device, _seed(w, b, layer, h, "keys"))
    z = torch.randint(0, C, (n,), generator=gk, device=device)
    K = cen[z] + 0.3 * torch.randn(n, d, generator=gk, device=device, dtype=torch.float32)
    sp = sink_positions(w, b, layer, h, n)
    if sp:
        K[torch.tensor(sp, device=device)] *= 4.0
    gv = _gen(device, _seed(w, b, layer, h, "values"))
    V = torch.randn(n, d, generator=gv, device=device, dtype=torch.float32)
    gq = _gen(device, _seed(w, b, layer, h, "queries"))
    zq = torch.randint(0, C, (G, n), generator=gq, device=device)
    Q = cen[zq] + 0.5 * torch.randn(G, n, d, generator=gq, device=device, dtype=torch.float32)
    Q *= w.query_scale(layer)
    dt = w.torch_dtype
    return Q.to(dt), K.to(dt), V.to(dt)


def layer_inputs(w: Workload, b: int, layer: int, device="cpu", n: int | None = None):
    """Prompt tensors of one layer: Q [Hq, n, d], K [Hkv, n, d], V [Hkv, n, d]."""
    qs, ks, vs = [], [], []
    for h in range(w.n_kv_heads):
        Q, K, V = kv_head_inputs(w, b, layer, h, device, n)
        qs.append(Q)
        ks.append(K)
        vs.append(V)
    return torch.cat(qs, 0), torch.stack(ks, 0), torch.stack(vs, 0)


def kv_head_decode_inputs(w: Workload, b: int, layer: int, h: int, steps: int, device="cpu"):
    """Decode-phase tensors of one KV head: q [steps, G, d], k [steps, d], v [steps, d]."""
    d, C, G = w.head_dim, w.n_clusters, w.group
    cen = _centres(w, b, layer, h, device)
    gk = _gen(device, _seed(w, b, layer, h, "dec_keys"))
    z = torch.randint(0, C, (steps,), generator=gk, device=device)
    k = cen[z] + 0.3 * torch.randn(steps, d, generator=gk, device=device, dtype=torch.float32)
    gv = _gen(device, _seed(w, b, layer, h, "dec_values"))
    v = torch.randn(steps, d, generator=gv, device=device, dtype=torch.float32)
    gq = _gen(device, _seed(w, b, layer, h, "dec_queries"))
    zq = torch.randint(0, C, (steps, G), generator=gq, device=device)
    q = cen[zq] + 0.5 * torch.randn(steps, G, d, generator=gq, device=device, dtype=torch.float32)
    q *= w.query_scale(layer)
    dt = w.torch_dtype
    return q.to(dt), k.to(dt), v.to(dt)


def layer_decode_inputs(w: Workload, b: int, layer: int, steps: int, device="cpu"):
    """Decode tensors of one layer: q [steps, Hq, d], k [steps, Hkv, d], v [steps, Hkv, d]."""
    qs, ks, vs = [], [], []
    for h in range(w.n_kv_heads):
        q, k, v = kv_head_decode_inputs(w, b, layer, h, steps, device)
        qs.append(q)
        ks.append(k)
        vs.append(v)
    return torch.cat(qs, 1), torch.stack(ks, 1), torch.stack(vs, 1)


def default_split(budget: int) -> int:
    """Recent-window size for heavy-hitter : recent = 3 : 1 (integer division)."""
    return budget // 4
