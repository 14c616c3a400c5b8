"""Seeded synthetic workloads: confidence vectors and per-layer Q/K/V tensors.

These stand in for the long-context prompts (8K-32K tokens) and generation blocks the paper
evaluates on (Sec. "Experiments", Table 4): the datasets and model weights are not
available, so shapes follow a 32-head, head_dim-128 model and values follow the recipes
below.  Nothing here computes any part of the attention method; the module only produces
inputs, which the CPU oracle and the GPU library both consume as the same bytes.

Recipe (per layer l, all in fp32, rounded to bf16 once at the end):
  Q[l] : [H, n_gen, d]   ~ N(0,1)  + q_gain * u          on every row
  K[l] : [H, M+N, d]     ~ N(0,1)  + k_gain * u          on rows listed in `sink_positions`
  V[l] : [H, M+N, d]     ~ N(0,1)
  u    : one unit vector in R^d shared by all heads and layers
  conf : fp32 [n_gen];  "uniform": U[0,1);  "correlated": 0.8*prev + 0.2*noise, both U[0,1)
"""
from __future__ import annotations

import dataclasses
import math
from dataclasses import dataclass

import torch

from . import rng

_T_Q, _T_K, _T_V, _T_U, _T_CONF_PREV, _T_CONF_NOISE, _T_SINKPOS = 1, 2, 3, 4, 5, 6, 7


@dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    n_heads: int          # H
    head_dim: int         # d
    n_ctx: int            # M, prompt tokens (prunable)
    n_resp: int           # N, response rows held after the prompt in K/V (always kept)
    n_gen: int            # rows of Q = positions of the current generation block
    block: int            # B, prompt KV block size
    k_focus: int          # k, size of I_focus
    window: int           # w of the window expansion (0/1: I_active = I_focus)
    n_keep: int           # C, kept prompt blocks
    n_sink: int           # N_sink
    sink_positions: tuple  # where the generator plants the biased keys
    conf_model: str       # "uniform" | "correlated"
    seed: int
    probe_layer: int = 0  # layer whose attention identifies the sinks
    first_sparse_layer: int = 0
    k_gain: float = 4.0
    q_gain: float = 0.5

    @property
    def n_kv(self) -> int:
        return self.n_ctx + self.n_resp

    @property
    def n_blocks(self) -> int:
        return -(-self.n_ctx // self.block)

    def layer_seed(self, layer: int) -> int:
        return self.seed + 1000 * layer

    def with_(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


_BASE_SEED = 20260215


def _seeded_sinks(seed: int, n_ctx: int, n: int) -> tuple:
    return tuple(rng.choice_without_replacement(rng.stream_key(seed, _T_SINKPOS), n_ctx, n))


def _mk_single(name, idx, n_ctx, keep_ratio):
    seed = _BASE_SEED + idx
    n_blocks = n_ctx // 128
    return Workload(name=name, n_layers=1, n_heads=32, head_dim=128, n_ctx=n_ctx, n_resp=64, n_gen=64,
                    block=128, k_focus=16, window=0, n_keep=int(math.floor(keep_ratio * n_blocks)),
                    n_sink=4, sink_positions=_seeded_sinks(seed, n_ctx, 4), conf_model="correlated", seed=seed)


TINY = Workload(name="tiny", n_layers=1, n_heads=4, head_dim=64, n_ctx=1024, n_resp=32, n_gen=32, block=64,
                k_focus=8, window=0, n_keep=4, n_sink=2, sink_positions=(0, 1), conf_model="uniform",
                seed=_BASE_SEED + 0)
CTX8K = _mk_single("ctx8k", 1, 8192, 0.10)
CTX16K = _mk_single("ctx16k", 2, 16384, 0.05)
CTX32K = _mk_single("ctx32k", 3, 32768, 0.03)
STACK32K = CTX32K.with_(name="stack32k", n_layers=32, seed=_BASE_SEED + 4, probe_layer=16, first_sparse_layer=17,
                        sink_positions=(0, 1, 8191, 20000))

# The paper's own hyper-parameters (Sec. "Implementation details": rho = 4, w = 8, alpha = 0.5, N_sink = 0.01 M,
# prompt block 64) on the 32K shape, one token unmasked per step (generation length = steps): k = round(4 * 1) = 4,
# 9-wide windows, 256 of 512 blocks kept, 327 sinks.  Not a timed configuration; used to check the same kernels
# on the shapes the paper ran.
PAPER32K = Workload(name="paper32k", n_layers=1, n_heads=32, head_dim=128, n_ctx=32768, n_resp=64, n_gen=64, block=64,
                    k_focus=4, window=8, n_keep=256, n_sink=327, sink_positions=_seeded_sinks(_BASE_SEED + 5, 32768, 4),
                    conf_model="correlated", seed=_BASE_SEED + 5)

# The same with the paper's generation layout: 256 response tokens decoded in blocks of 32.  The queries are the 32
# positions of the current block; all 256 response rows are keys that are always kept.
PAPER32K_GEN256 = PAPER32K.with_(name="paper32k_gen256", n_resp=256, n_gen=32, seed=_BASE_SEED + 6,
                                 sink_positions=_seeded_sinks(_BASE_SEED + 6, 32768, 4))

# Four times the longest measured context: not a timed configuration; checks that nothing in the path is tied to 32K
# (block counts, the limits of the small-N_sink tournament, index widths).
CTX128K = _mk_single("ctx128k", 7, 131072, 0.03)

WORKLOADS = {w.name: w for w in (TINY, CTX8K, CTX16K, CTX32K, STACK32K, PAPER32K, PAPER32K_GEN256, CTX128K)}


def strong_sinks(w: Workload, logit_shift: float = 6.0) -> Workload:
    """Same workload with the planted bias scaled so a sink's logit exceeds the others by `logit_shift`.

    With the literal gains (4.0 and 0.5) the shift is only 2/sqrt(d), too small for the planted keys to collect
    much attention mass; this variant exists for tests that need the planted positions to be true sinks.
    """
    s = math.sqrt(logit_shift * math.sqrt(w.head_dim) / (w.k_gain * w.q_gain))
    return w.with_(name=w.name + "_strong", k_gain=w.k_gain * s, q_gain=w.q_gain * s)


def shared_direction(w: Workload, device="cpu") -> torch.Tensor:
    """The unit vector u (fp32 [d]) shared by all heads and layers of a workload."""
    u = rng.normal(rng.stream_key(w.seed, _T_U), 0, w.head_dim, device)
    return u / torch.linalg.vector_norm(u)


def confidence(w: Workload, device="cpu") -> torch.Tensor:
    """Previous-step confidence c^(t-1), fp32 [n_gen]; every slot of the block is still masked."""
    prev = rng.uniform(rng.stream_key(w.seed, _T_CONF_PREV), 0, w.n_gen, device)
    if w.conf_model == "uniform":
        return prev
    noise = rng.uniform(rng.stream_key(w.seed, _T_CONF_NOISE), 0, w.n_gen, device)
    return 0.8 * prev + 0.2 * noise


def masked_all(w: Workload, device="cpu") -> torch.Tensor:
    return torch.ones(w.n_gen, dtype=torch.uint8, device=device)


def _normal_hnd(key: int, h: int, n: int, d: int, device) -> torch.Tensor:
    out = torch.empty((h, n, d), dtype=torch.float32, device=device)
    per_head = n * d
    for i in range(h):  # head by head keeps the int64 temporaries small
        out[i] = rng.normal(key, i * per_head, per_head, device).view(n, d)
    return out


def layer_qkv(w: Workload, layer: int = 0, device="cpu", which="qkv"):
    """bf16 tensors of one layer in [H, rows, d] layout; `which` selects a subset, returned in q,k,v order."""
    ls = w.layer_seed(layer)
    u = shared_direction(w, device)
    out = []
    if "q" in which:
        q = _normal_hnd(rng.stream_key(ls, _T_Q), w.n_heads, w.n_gen, w.head_dim, device)
        q += w.q_gain * u
        out.append(q.to(torch.bfloat16))
    if "k" in which:
        k = _normal_hnd(rng.stream_key(ls, _T_K), w.n_heads, w.n_kv, w.head_dim, device)
        if len(w.sink_positions):
            pos = torch.tensor(w.sink_positions, dtype=torch.int64, device=device)
            k[:, pos, :] += w.k_gain * u
        out.append(k.to(torch.bfloat16))
    if "v" in which:
        v = _normal_hnd(rng.stream_key(ls, _T_V), w.n_heads, w.n_kv, w.head_dim, device)
        out.append(v.to(torch.bfloat16))
    return out[0] if len(out) == 1 else tuple(out)


def bf16_bits(t: torch.Tensor):
    """The raw 16-bit patterns of a bf16 tensor as a numpy uint16 array (host copy)."""
    import numpy as np
    return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)
