"""Seeded synthetic inputs for the FCCO step: shapes, index draws and state sizes.

This module holds data recipes only (random embeddings, index draws, the table of
workload shapes).  It contains none of the method's arithmetic and is the one
module that both the GPU tests/bench and the CPU oracle's callers use, so that both
sides see bit-identical inputs.  numpy only.

Recipe (all workloads): image rows are i.i.d. N(0,1) vectors scaled to unit L2 norm;
text row i = unit-normalised (image row i + noise * N(0,1)).  For bf16 workloads the
values are rounded to bf16 (round to nearest even) AFTER normalisation and both
sides consume the rounded values.  Batch indices are distinct uniform draws from
[0, N).  The datasets of the paper (CC3M 2.7M, CC12M 9.1M, LAION 315M pairs) are
represented only by their sizes N and by ViT-class embedding widths.
"""
from __future__ import annotations

import numpy as np

V0, V1, V2, V3 = 0, 1, 2, 3

# name -> workload description.  "gamma" is either a constant or ("cosine", E, gamma_min)
# meaning one epoch per step, E decay epochs.
WORKLOADS = {
    "cfg0": dict(B=64, b=64, off=0, d=32, N=1024, dtype="f32", version=V1, tau=0.07,
                 gamma=0.8, eps=1e-14, rho=0.0, noise=0.5, steps=10),
    "cfg1": dict(B=1024, b=1024, off=0, d=512, N=2_700_000, dtype="bf16", version=V3, tau=0.07,
                 gamma=("cosine", 100, 0.2), eps=1e-14, rho=6.5, noise=0.5, steps=100),
    "cfg2": dict(B=8192, b=256, off=1280, d=512, N=9_100_000, dtype="bf16", version=V3, tau=0.07,
                 gamma=0.6, eps=1e-14, rho=8.5, noise=0.5, steps=20),
    "cfg3": dict(B=4096, b=4096, off=0, d=768, N=9_100_000, dtype="bf16", version=V2, tau=0.07,
                 gamma=0.8, eps=1e-14, rho=8.5, noise=0.5, steps=20),
    "cfg4": dict(B=32768, b=1024, off=17408, d=1024, N=315_000_000, dtype="bf16", version=V2,
                 tau=0.07, gamma=("cosine", 100, 0.2), eps=1e-6, rho=8.5, noise=0.3, steps=20),
}


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 array -> float32 array holding the nearest bf16 values (ties to even)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def make_embeddings(seed: int, B: int, d: int, noise: float, dtype: str):
    """Return (img, txt), float32 [B, d]; values are bf16-representable when dtype == 'bf16'."""
    rng = np.random.default_rng(seed)
    img = rng.standard_normal((B, d), dtype=np.float32)
    img /= np.linalg.norm(img, axis=1, keepdims=True)
    txt = img + np.float32(noise) * rng.standard_normal((B, d), dtype=np.float32)
    txt /= np.linalg.norm(txt, axis=1, keepdims=True)
    if dtype == "bf16":
        img, txt = round_to_bf16(img), round_to_bf16(txt)
    elif dtype != "f32":
        raise ValueError(dtype)
    return np.ascontiguousarray(img), np.ascontiguousarray(txt)


def draw_indices(seed: int, b: int, N: int) -> np.ndarray:
    """b distinct uniform indices from [0, N), int64, in draw order (not sorted)."""
    rng = np.random.default_rng(seed)
    return rng.choice(N, size=b, replace=False).astype(np.int64)


def step_seed(workload: str, step: int) -> int:
    """Seed convention: 1000 * (workload number) + step."""
    return 1000 * int(workload[3:]) + step
