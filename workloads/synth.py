"""Seeded synthetic workloads for the LSH-MoE compression path.

The paper evaluates on RoBERTa-MoE, T5-MoE, GPT-MoE and Swin-MoE layers
(Table 1) whose activations show a clustered structure (Section 3.1).  Its
datasets and checkpoints are not available, so tokens are drawn from a seeded
Gaussian mixture with the layer shapes of Table 1.  Nothing here hashes,
groups, averages or restores anything: these are inputs only.

Storage convention shared by every consumer:
  * "f32"  arrays are numpy float32;
  * "bf16" arrays are numpy uint16 holding the upper 16 bits of the IEEE
    binary32 pattern (the cast from fp32 is done by torch's CPU routine).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional

import numpy as np
import torch

BASE_SEED = 20241108


@dataclass(frozen=True)
class Config:
    name: str
    index: int
    T: int            # tokens
    d: int            # model dimension
    dtype: str        # "f32" | "bf16"
    k: int            # experts per token
    E: int            # experts
    L: int            # hash functions
    r: int            # rotated dimensions per hash (2r buckets per hash)
    centers: int      # mixture components
    sigma: float      # within-cluster noise
    gate: str         # "uniform" | "zipf" | "topk_logits" | "center_mod" | "content"
    outlier_frac: float = 0.0
    expert: str = "mlp"   # "linear" (d x d) | "mlp" (d x 4d x d, GELU)

    @property
    def N(self) -> int:
        return self.T * self.k

    @property
    def itemsize(self) -> int:
        return 4 if self.dtype == "f32" else 2


CONFIGS = {
    "tiny": Config("tiny", 0, 2048, 256, "f32", 1, 4, 2, 16, 64, 0.1, "uniform", 0.0, "linear"),
    "swin": Config("swin", 1, 25088, 512, "bf16", 1, 32, 2, 32, 512, 0.2, "zipf"),
    "roberta": Config("roberta", 2, 16384, 768, "bf16", 1, 16, 2, 32, 1024, 0.15, "uniform"),
    "gpt": Config("gpt", 3, 32768, 1024, "bf16", 2, 32, 3, 32, 2048, 0.15, "topk_logits"),
    "t5": Config("t5", 4, 65536, 1024, "bf16", 2, 64, 4, 64, 4096, 0.1, "topk_logits", 0.05),
}


def config(name: str, **overrides) -> Config:
    """Look up one of the five named configs, optionally overriding fields
    (e.g. ``T=`` for a scaled-down copy or ``gate="content"`` for the
    supplementary content-correlated gate)."""
    cfg = CONFIGS[name]
    return replace(cfg, **overrides) if overrides else cfg


@dataclass
class Workload:
    cfg: Config
    seed: int
    tokens: np.ndarray       # [T, d] storage
    rot: np.ndarray          # [L, r, d] storage
    expert: np.ndarray       # [T, k] int32, distinct per row
    gate_weight: np.ndarray  # [T, k] float32 (not used by the path)
    center_id: np.ndarray    # [T] int32 (-1 for outliers); diagnostics only


def f32_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Cast an fp32 array to the storage convention above (bf16 via torch, RNE)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "bf16":
        t = torch.from_numpy(x).to(torch.bfloat16)
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    raise ValueError(dtype)


def storage_to_f32(x: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of a storage array to fp32 (via torch for bf16)."""
    if dtype == "f32":
        return np.asarray(x, dtype=np.float32)
    if dtype == "bf16":
        t = torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).view(torch.bfloat16)
        return t.to(torch.float32).numpy()
    raise ValueError(dtype)


def _gate(cfg: Config, rng: np.random.Generator, tokens_f32: np.ndarray, center_id: np.ndarray):
    T, k, E = cfg.T, cfg.k, cfg.E
    if cfg.gate == "uniform":
        assert k == 1
        e = rng.integers(0, E, size=(T, 1), dtype=np.int64)
        w = np.ones((T, 1), np.float32)
    elif cfg.gate == "zipf":
        assert k == 1
        p = (np.arange(E, dtype=np.float64) + 1.0) ** -1.1
        p /= p.sum()
        e = rng.choice(E, size=(T, 1), p=p)
        w = np.ones((T, 1), np.float32)
    elif cfg.gate in ("topk_logits", "content"):
        if cfg.gate == "topk_logits":
            logits = rng.standard_normal((T, E), dtype=np.float32)
        else:  # content-correlated: logits are a seeded linear map of the token
            wg = rng.standard_normal((cfg.d, E), dtype=np.float32) / np.sqrt(cfg.d)
            logits = tokens_f32 @ wg
        order = np.argsort(-logits, axis=1, kind="stable")[:, :k]
        top = np.take_along_axis(logits, order, axis=1).astype(np.float64)
        top -= top.max(axis=1, keepdims=True)
        w = np.exp(top)
        w = (w / w.sum(axis=1, keepdims=True)).astype(np.float32)
        e = order
    elif cfg.gate == "center_mod":
        assert k == 1
        e = np.where(center_id >= 0, center_id % E, rng.integers(0, E, size=T))[:, None]
        w = np.ones((T, 1), np.float32)
    else:
        raise ValueError(cfg.gate)
    return np.ascontiguousarray(e, dtype=np.int32), w


def generate(cfg: Config, seed: Optional[int] = None) -> Workload:
    """Draw one workload.  Default seed is ``BASE_SEED + cfg.index``."""
    seed = BASE_SEED + cfg.index if seed is None else int(seed)
    rng = np.random.Generator(np.random.PCG64(seed))
    T, d = cfg.T, cfg.d
    centers = rng.standard_normal((cfg.centers, d), dtype=np.float32)
    center_id = rng.integers(0, cfg.centers, size=T).astype(np.int32)
    x = centers[center_id]
    x += np.float32(cfg.sigma) * rng.standard_normal((T, d), dtype=np.float32)
    if cfg.outlier_frac > 0.0:
        out = rng.random(T) < cfg.outlier_frac
        n_out = int(out.sum())
        s3 = np.sqrt(3.0)
        x[out] = rng.uniform(-s3, s3, size=(n_out, d)).astype(np.float32)
        center_id = np.where(out, -1, center_id).astype(np.int32)
    tokens = f32_to_storage(x, cfg.dtype)
    x_stored = storage_to_f32(tokens, cfg.dtype)
    rot = f32_to_storage(rng.standard_normal((cfg.L, cfg.r, d), dtype=np.float32), cfg.dtype)
    expert, w = _gate(cfg, rng, x_stored, center_id)
    return Workload(cfg, seed, tokens, rot, expert, w, center_id)


def expert_standin(centroids: torch.Tensor, cfg: Config, seed: int) -> torch.Tensor:
    """Seeded stand-in for the expert network, applied to centroid rows.

    One weight set shared by all experts: a d x d linear map ("linear") or a
    d x 4d x d GELU MLP ("mlp").  ``centroids`` is a torch tensor (float32 or
    bfloat16, any device); the result has the same dtype, device and shape.
    It runs outside the compression path: its output is handed unchanged to
    whichever implementation restores the tokens.
    """
    d = cfg.d
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed) + 7919)
    dev, dt = centroids.device, centroids.dtype
    if cfg.expert == "linear":
        w = (torch.randn(d, d, generator=g) / d ** 0.5).to(device=dev, dtype=dt)
        return (centroids @ w).contiguous()
    w1 = (torch.randn(d, 4 * d, generator=g) / d ** 0.5).to(device=dev, dtype=dt)
    w2 = (torch.randn(4 * d, d, generator=g) / (4 * d) ** 0.5).to(device=dev, dtype=dt)
    out = torch.empty_like(centroids)
    step = 16384
    for lo in range(0, centroids.shape[0], step):
        h = torch.nn.functional.gelu(centroids[lo:lo + step] @ w1)
        out[lo:lo + step] = h @ w2
    return out
