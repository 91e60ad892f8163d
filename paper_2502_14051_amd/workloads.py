"""Seeded synthetic inputs shaped like RocketKV's workloads.

This module only *draws data*: it holds none of the method's arithmetic (no
summaries, scores, top-k or attention) and is the one piece shared by the GPU
tests, the CPU oracle tests and the benchmark.  All tensors are bf16, carried
on the host as ``uint16`` bit patterns in plain token-major layouts:

    q    [B][Hq][D]          decode-step queries
    K,V  [B][Hkv][n][D]      keys / values of the cache
    qobs [B][Hq][W][D]       queries of the last W prompt positions (SnapKV)

Recipe (stands in for Llama3.1-8B / Mistral-7B / LongChat-7B activations on
the long-context suites of Section 4.1 of the paper, whose items and weights
are not available here): per (KV head, channel) a scale drawn from
LogNormal(0, sigma) is shared by K and q, so that a few channels dominate |q|
(the head-dimension sparsity Section 3.4 Step 2 relies on); the query heads of
a GQA group share a common component (weight 0.6, own part 0.8); V is standard
normal; a small number of "heavy" tokens have their key pulled towards the
direction of the group-summed query so that they dominate the attention mass
(the heavy-hitter structure of Section 3.1).
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


# --------------------------------------------------------------------------
# bf16 <-> float helpers (data format only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bf16 bit patterns (uint16)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(b).astype(np.float64)


# --------------------------------------------------------------------------
# workload descriptions
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    context: int          # tokens in the (uncompressed) cache / prompt
    page_size: int
    channel_budget: int   # k1
    token_budget: int     # T, tokens of exact attention
    n_layers: int = 1
    snap_keep: int = 0    # N of the SnapKV stage, 0 = stage not used
    window: int = 32
    pool_kernel: int = 63
    n_heavy: int = 64
    heavy_nats: float = 8.0  # planted logits sit this far above the expected background maximum
    scale_sigma: float = 0.5
    n_outlier: int = 0    # config-1 style: unit scales, a few channels x8
    seed: int = 0

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


# The five configurations of the benchmark description.  Budgets that the
# description lists as alternatives are exposed through ``with_budget``.
CONFIGS = {
    "tiny": Workload("tiny", 1, 16, 4, 128, 4096, 16, 32, 256, n_heavy=8,
                     scale_sigma=0.0, n_outlier=4, seed=0),
    "llama8b_layer_32k": Workload("llama8b_layer_32k", 1, 32, 8, 128, 32768, 16, 32, 1024, seed=1),
    "llama8b_step_b16": Workload("llama8b_step_b16", 16, 32, 8, 128, 32768, 16, 32, 1024,
                                 n_layers=32, snap_keep=4096, seed=2),
    "mistral_snap_128k": Workload("mistral_snap_128k", 1, 32, 8, 128, 131072, 16, 32, 2048,
                                  snap_keep=8192, seed=3),
    "llama70b_step_b16": Workload("llama70b_step_b16", 16, 64, 8, 128, 32768, 16, 32, 1024,
                                  n_layers=80, snap_keep=4096, seed=4),
}


def with_budget(w: Workload, token_budget: int) -> Workload:
    return replace(w, token_budget=token_budget)


def scaled(w: Workload, **kw) -> Workload:
    """A copy with some fields replaced (smaller batch / context for slices)."""
    return replace(w, **kw)


# --------------------------------------------------------------------------
# host generator (numpy PCG64)
# --------------------------------------------------------------------------
def _heavy_gain(qf: np.ndarray, scale: np.ndarray, n: int, nats: float = 8.0):
    """Direction and gain for the planted keys of one group.

    qf: [G][D] float32 queries, scale: [D] key channel scales.  The gain puts
    every head's logit on a planted key about ``nats`` above the expected
    maximum background logit (mean 0, std sigma_h, n draws).
    """
    D = qf.shape[-1]
    ssum = qf.sum(axis=0)
    nrm = float(np.linalg.norm(ssum))
    u = ssum / nrm if nrm > 0 else np.zeros_like(ssum)
    proj = qf @ u
    proj = np.maximum(proj, max(0.25 * float(proj.mean()), 1e-3))
    sigma = np.sqrt(((qf * scale[None, :]) ** 2).sum(axis=1) / D)
    target = sigma * np.sqrt(2.0 * np.log(max(n, 2))) + nats
    gamma = float((target * np.sqrt(D) / proj).max())
    return u.astype(np.float32), gamma


def generate(w: Workload, layer: int = 0, context: int | None = None, with_obs: bool = False):
    """Draw one layer's inputs on the host.

    Returns a dict with uint16 arrays ``q``, ``K``, ``V`` (and ``qobs`` when
    ``with_obs``), ``seq_lens`` (int32 [B]) and ``heavy`` (int32 [B][Hkv][n_heavy],
    positions of the planted tokens).
    """
    n = w.context if context is None else context
    B, Hq, Hkv, D, G = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.group
    rng = np.random.Generator(np.random.PCG64([w.seed, layer]))
    if w.n_outlier:
        scale = np.ones((B, Hkv, D), dtype=np.float32)
        for b in range(B):
            for g in range(Hkv):
                scale[b, g, rng.choice(D, size=w.n_outlier, replace=False)] = 8.0
    else:
        scale = rng.lognormal(0.0, w.scale_sigma, size=(1, Hkv, D)).astype(np.float32)
        scale = np.broadcast_to(scale, (B, Hkv, D)).copy()
    q_shared = rng.standard_normal((B, Hkv, 1, D), dtype=np.float32)
    q_own = rng.standard_normal((B, Hkv, G, D), dtype=np.float32)
    q = (0.6 * q_shared + 0.8 * q_own) * scale[:, :, None, :]
    q_bits = f32_to_bf16_bits(q)
    qf = bf16_bits_to_f32(q_bits)
    K = rng.standard_normal((B, Hkv, n, D), dtype=np.float32)
    K *= scale[:, :, None, :]
    V = rng.standard_normal((B, Hkv, n, D), dtype=np.float32)
    n_heavy = min(w.n_heavy, n)
    heavy = np.zeros((B, Hkv, n_heavy), dtype=np.int32)
    for b in range(B):
        for g in range(Hkv):
            pos = np.sort(rng.choice(n, size=n_heavy, replace=False)).astype(np.int32)
            heavy[b, g] = pos
            u, gamma = _heavy_gain(qf[b, g], scale[b, g], n, w.heavy_nats)
            K[b, g, pos] = 0.25 * K[b, g, pos] + gamma * u[None, :]
    out = dict(q=q_bits.reshape(B, Hq, D), K=f32_to_bf16_bits(K), V=f32_to_bf16_bits(V),
               seq_lens=np.full(B, n, dtype=np.int32), heavy=heavy)
    if with_obs:
        W = w.window
        noise = rng.standard_normal((B, Hkv, G, W, D), dtype=np.float32) * scale[:, :, None, None, :]
        qobs = 0.7 * qf[:, :, :, None, :] + 0.7 * noise
        out["qobs"] = f32_to_bf16_bits(qobs).reshape(B, Hq, W, D)
    return out


# --------------------------------------------------------------------------
# device generator (torch), for shapes too large to draw on the host
# --------------------------------------------------------------------------
def generate_device(w: Workload, layer: int, device, context: int | None = None,
                    with_obs: bool = False):
    """Same recipe drawn with torch's seeded device generator.

    Returns bf16 torch tensors ``q`` [B][Hq][D], ``K``/``V`` [B][Hkv][n][D],
    optionally ``qobs``, plus ``seq_lens`` (int32) and ``heavy``.  The device
    stream differs from the host one; consumers that need host copies must
    download these very tensors.
    """
    import torch

    n = w.context if context is None else context
    B, Hq, Hkv, D, G = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.group
    gen = torch.Generator(device=device)
    gen.manual_seed(1_000_003 * w.seed + layer)
    if w.n_outlier:
        scale = torch.ones((B, Hkv, D), device=device)
        idx = torch.rand((B, Hkv, D), generator=gen, device=device).argsort(dim=-1)[..., :w.n_outlier]
        scale.scatter_(-1, idx, 8.0)
    else:
        z = torch.randn((1, Hkv, D), generator=gen, device=device)
        scale = torch.exp(w.scale_sigma * z).expand(B, Hkv, D).contiguous()
    q_shared = torch.randn((B, Hkv, 1, D), generator=gen, device=device)
    q_own = torch.randn((B, Hkv, G, D), generator=gen, device=device)
    q = ((0.6 * q_shared + 0.8 * q_own) * scale[:, :, None, :]).bfloat16()
    qf = q.float()
    K = torch.randn((B, Hkv, n, D), generator=gen, device=device, dtype=torch.bfloat16)
    K *= scale[:, :, None, :].bfloat16()
    V = torch.randn((B, Hkv, n, D), generator=gen, device=device, dtype=torch.bfloat16)
    n_heavy = min(w.n_heavy, n)
    heavy = torch.rand((B, Hkv, n), generator=gen, device=device).argsort(dim=-1)[..., :n_heavy]
    heavy = heavy.sort(dim=-1).values
    ssum = qf.sum(dim=2)
    u = ssum / ssum.norm(dim=-1, keepdim=True).clamp_min(1e-20)
    proj = (qf * u[:, :, None, :]).sum(-1)
    floor = torch.maximum(0.25 * proj.mean(dim=-1, keepdim=True), torch.full_like(proj, 1e-3))
    proj = torch.maximum(proj, floor)
    sigma = ((qf * scale[:, :, None, :]) ** 2).sum(-1).div(D).sqrt()
    target = sigma * (2.0 * float(np.log(max(n, 2)))) ** 0.5 + w.heavy_nats
    gamma = (target * (D ** 0.5) / proj).max(dim=-1).values
    idx = heavy[..., None].expand(B, Hkv, n_heavy, D)
    planted = 0.25 * K.gather(2, idx).float() + gamma[:, :, None, None] * u[:, :, None, :]
    K.scatter_(2, idx, planted.bfloat16())
    out = dict(q=q.reshape(B, Hq, D), K=K, V=V,
               seq_lens=torch.full((B,), n, dtype=torch.int32, device=device),
               heavy=heavy.to(torch.int32))
    if with_obs:
        W = w.window
        noise = torch.randn((B, Hkv, G, W, D), generator=gen, device=device) * scale[:, :, None, None, :]
        qobs = 0.7 * qf[:, :, :, None, :] + 0.7 * noise
        out["qobs"] = qobs.bfloat16().reshape(B, Hq, W, D)
    return out


def to_bits(t) -> np.ndarray:
    """bf16 torch tensor (any device) -> uint16 numpy bit patterns."""
    import torch

    return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)


def from_bits(a: np.ndarray, device=None):
    """uint16 numpy bit patterns -> bf16 torch tensor."""
    import torch

    t = torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16)
    return t.to(device) if device is not None else t
