"""Seeded synthetic inputs for the KVComm reuse step.

This module only draws random tensors of the right shapes; it contains none of the
method's arithmetic and is the one piece shared by the HIP path's tests/benchmark and the
CPU oracle's tests.  The tensors stand in for the paper's Llama-3.1-8B KV-caches
([32, 8, seq_len, 128], appendix on long-context anchor matching) and its fully connected
multi-agent workload (Sec. 4.1, Table 2): no dataset item or model weight is involved.

Recipe (all values iid normal, seeded):
  base K/V of a segment, anchors' base K, prefix and suffix K/V, suffix Q ~ N(0, 1);
  anchors' stored deviations dK, dV ~ N(0, sigma_delta);
  bf16 tensors are drawn in fp32 and rounded to bf16 once; both the GPU path and the oracle
  read the rounded values.
Base positions of every standalone cache are [0, S); a segment placed at cache offset p0
has delta_pos = p0.
"""
from dataclasses import dataclass, field, replace
from typing import List, Optional, Tuple

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    n_kv_heads: int
    n_q_heads: int
    head_dim: int
    dtype: torch.dtype
    rope_theta: float
    n_agents: int
    prefix_len: int                 # agent-specific prefix tokens at the head of the cache
    seg_len: int                    # tokens per shared segment
    n_segments: int                 # shared segments per agent
    n_anchors: int                  # anchor pool size per segment
    tq: int                         # non-shared suffix query tokens (0 = no attention step)
    sigma_delta: float
    temperature: float = 1.0
    seed: int = 0
    anchor_delta_choices: Optional[Tuple[int, ...]] = None  # per-anchor recording deltas drawn from here
    anchor_lens: Optional[Tuple[int, ...]] = None            # per-anchor valid lengths (default seg_len)

    @property
    def n_ctx(self):
        return self.prefix_len + self.n_segments * self.seg_len

    @property
    def cache_len(self):
        return self.n_ctx + self.tq

    @property
    def aligned_tokens(self):
        return self.n_agents * self.n_segments * self.seg_len

    def seg_offset(self, j):
        return self.prefix_len + j * self.seg_len

    def align_bytes(self):
        """Algorithmic HBM bytes of the align step: 2*(A+2) rows of D elements per (l, h, token)."""
        es = 2 if self.dtype == torch.bfloat16 else 4
        rows = self.n_layers * self.n_kv_heads * self.aligned_tokens
        return rows * self.head_dim * es * 2 * (self.n_anchors + 2)

    def distance_bytes(self):
        """Algorithmic HBM bytes of the distance step: (A+1) key rows per (l, h, token)."""
        es = 2 if self.dtype == torch.bfloat16 else 4
        rows = self.n_layers * self.n_kv_heads * self.aligned_tokens
        return rows * self.head_dim * es * (self.n_anchors + 1)

    def attn_flops(self):
        """4*D*Hq*L*(Tq*Nctx + Tq(Tq+1)/2) per agent: QK^T and PV, causal half counted once."""
        per_agent = 4 * self.head_dim * self.n_q_heads * self.n_layers * (
            self.tq * self.n_ctx + self.tq * (self.tq + 1) // 2)
        return per_agent * self.n_agents


# The five configurations of the build's baseline description.
TINY = Workload("tiny", 2, 4, 8, 64, torch.float32, 1e4, n_agents=1, prefix_len=64, seg_len=128, n_segments=1,
                n_anchors=4, tq=32, sigma_delta=0.1, seed=0)
LLAMA8B_5AGENTS = Workload("llama8b_5agents", 32, 8, 32, 128, torch.bfloat16, 5e5, n_agents=5, prefix_len=512,
                           seg_len=512, n_segments=4, n_anchors=8, tq=512, sigma_delta=0.05, seed=0)
POOL_SCALING = tuple(
    Workload(f"pool_scaling_a{a}", 32, 8, 32, 128, torch.bfloat16, 5e5, n_agents=1, prefix_len=1024, seg_len=1024,
             n_segments=1, n_anchors=a, tq=0, sigma_delta=0.05, seed=0, anchor_delta_choices=(256, 1024, 2048))
    for a in (4, 16, 32, 64))
LONG_CONTEXT = Workload("long_context", 32, 8, 32, 128, torch.bfloat16, 5e5, n_agents=8, prefix_len=1024,
                        seg_len=1024, n_segments=2, n_anchors=16, tq=1024, sigma_delta=0.05, seed=0)
LLAMA70B = Workload("llama70b", 80, 8, 64, 128, torch.bfloat16, 5e5, n_agents=4, prefix_len=0, seg_len=2048,
                    n_segments=4, n_anchors=16, tq=512, sigma_delta=0.05, seed=0)

WORKLOADS = {w.name: w for w in (TINY, LLAMA8B_5AGENTS, *POOL_SCALING, LONG_CONTEXT, LLAMA70B)}


def scaled(w: Workload, **kw) -> Workload:
    """A smaller (or otherwise modified) copy of a workload, e.g. fewer layers for parity tests."""
    return replace(w, **kw)


@dataclass
class Segment:
    base_k: torch.Tensor                 # [L, Hkv, S, D]
    base_v: torch.Tensor
    anchor_k: List[torch.Tensor]         # A x [L, Hkv, cap, D] (cap = common capacity >= every length)
    anchor_dk: List[torch.Tensor]
    anchor_dv: List[torch.Tensor]
    anchor_len: List[int]
    delta_pos: int
    anchor_delta_pos: Optional[List[int]]


@dataclass
class Agent:
    q: Optional[torch.Tensor]            # [L, Hq, Tq, D]
    cache_k: torch.Tensor                # [L, Hkv, cache_len, D]; prefix and suffix rows filled
    cache_v: torch.Tensor
    segments: List[Segment] = field(default_factory=list)


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _normal(shape, sigma, dtype, g, device):
    x = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    if sigma != 1.0:
        x.mul_(sigma)
    return x.to(dtype)


def make_segment(w: Workload, agent: int, j: int, device="cpu", share_anchor_k_from: Optional[Segment] = None):
    """Segment j of an agent: base K/V, its anchor pool (base K, dK, dV) and position deltas."""
    g = _gen(w.seed + 100 * agent + j + 1, device)
    L, H, S, D = w.n_layers, w.n_kv_heads, w.seg_len, w.head_dim
    lens = list(w.anchor_lens) if w.anchor_lens else [S] * w.n_anchors
    assert len(lens) == w.n_anchors
    cap = max(lens + [S])
    base_k = _normal((L, H, S, D), 1.0, w.dtype, g, device)
    base_v = _normal((L, H, S, D), 1.0, w.dtype, g, device)
    if share_anchor_k_from is not None:
        anchor_k = share_anchor_k_from.anchor_k
    else:
        anchor_k = [_normal((L, H, cap, D), 1.0, w.dtype, g, device) for _ in range(w.n_anchors)]
    anchor_dk = [_normal((L, H, cap, D), w.sigma_delta, w.dtype, g, device) for _ in range(w.n_anchors)]
    anchor_dv = [_normal((L, H, cap, D), w.sigma_delta, w.dtype, g, device) for _ in range(w.n_anchors)]
    delta_pos = w.seg_offset(j)
    anchor_delta_pos = None
    if w.anchor_delta_choices:
        gc = _gen(w.seed + 100 * agent + j + 7919, "cpu")
        ch = torch.tensor(w.anchor_delta_choices)
        anchor_delta_pos = ch[torch.randint(len(ch), (w.n_anchors,), generator=gc)].tolist()
        delta_pos = int(ch[torch.randint(len(ch), (1,), generator=gc)])
    return Segment(base_k, base_v, anchor_k, anchor_dk, anchor_dv, lens, delta_pos, anchor_delta_pos)


def make_agent(w: Workload, agent: int, device="cpu", with_segments=True):
    """One agent's inputs: suffix queries, a cache with prefix and suffix rows filled, its segments."""
    g = _gen(w.seed + 100 * agent + 50, device)
    L, H, D = w.n_layers, w.n_kv_heads, w.head_dim
    cache_k = torch.zeros((L, H, w.cache_len, D), dtype=w.dtype, device=device)
    cache_v = torch.zeros((L, H, w.cache_len, D), dtype=w.dtype, device=device)
    if w.prefix_len:
        cache_k[:, :, : w.prefix_len] = _normal((L, H, w.prefix_len, D), 1.0, w.dtype, g, device)
        cache_v[:, :, : w.prefix_len] = _normal((L, H, w.prefix_len, D), 1.0, w.dtype, g, device)
    q = None
    if w.tq:
        cache_k[:, :, w.n_ctx:] = _normal((L, H, w.tq, D), 1.0, w.dtype, g, device)
        cache_v[:, :, w.n_ctx:] = _normal((L, H, w.tq, D), 1.0, w.dtype, g, device)
        q = _normal((L, w.n_q_heads, w.tq, D), 1.0, w.dtype, g, device)
    segs = [make_segment(w, agent, j, device) for j in range(w.n_segments)] if with_segments else []
    return Agent(q, cache_k, cache_v, segs)
