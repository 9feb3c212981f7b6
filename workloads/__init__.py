"""Seeded synthetic inputs for the Sign-Muon hot path.

This module holds shapes and random-number recipes only; none of the
method's arithmetic lives here.  It serves both the CPU oracle's tests and
the GPU tests / benchmark, so the two sides see identical inputs.

The matrix sets stand in for the paper's workloads (CIFAR-10 ResNet-50 and
nanoGPT on OpenWebText): the shapes are the weight blocks of those models
flattened to matrices (conv kernels as out x in*k*k, the paper's
"tensor-flattened-to-matrix" blocks); the gradients are drawn from the
distributions named below, not computed from data.

Base seed 1337 is the seed the paper fixes for its nanoGPT runs.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 1337

# name -> dict(shapes=[(rows, cols), ...], M=workers, ...)
WORKLOADS = {
    # single 256x256 fp32 matrix, M=4, N(0,1) gradients, no local polar
    "single256": dict(shapes=[(256, 256)], M=4, grad="normal", grad_std=1.0,
                      ns_steps=5, local_polar_steps=0, sign_fmt="1bit", stream=1),
    # ResNet-50-shaped blocks, M=4, N(0, var 1e-2) gradients
    "resnet50": dict(shapes=[(64, 576), (128, 1152), (256, 2304), (512, 4608),
                             (2048, 512), (1000, 2048)],
                     M=4, grad="normal", grad_std=0.1,
                     ns_steps=5, local_polar_steps=0, sign_fmt="1bit", stream=2),
    # nanoGPT-124M-shaped blocks: 12 layers x {qkv, proj, mlp up, mlp down}
    "nanogpt124m": dict(shapes=[(768, 2304), (768, 768), (768, 3072), (3072, 768)] * 12,
                        M=8, grad="lowrank", grad_std=1.0, rank=8,
                        ns_steps=5, local_polar_steps=5, sign_fmt="1bit", stream=3),
    # large-model-shaped blocks, heavy-tailed gradients
    "large": dict(shapes=[(4096, 4096)] * 8 + [(4096, 11008)] * 8,
                  M=16, grad="student_t", nu=3, grad_std=1.0,
                  ns_steps=5, local_polar_steps=5, sign_fmt="1bit", stream=4),
    # int8 vote path
    "int8vote": dict(shapes=[(2048, 8192)] * 32, M=16, grad="normal", grad_std=1.0,
                     ns_steps=5, local_polar_steps=5, sign_fmt="int8", stream=5),
    # The paper's own nanoGPT (6 layers, width 384) in its weak-scaling setting: 10 Newton-Schulz
    # steps, spectral scale with 2 power iterations, update by the voted signs (no local polar step).
    "nanogpt_paper_k10": dict(shapes=[(384, 1152), (384, 384), (384, 1536), (1536, 384)] * 6,
                              M=8, grad="lowrank", grad_std=1.0, rank=8, scale="spectral",
                              ns_steps=10, local_polar_steps=0, sign_fmt="1bit", stream=6),
    # The ResNet-50-shaped set in the paper's best CIFAR-10 setting: one Newton-Schulz step, spectral scale.
    "resnet50_k1": dict(shapes=[(64, 576), (128, 1152), (256, 2304), (512, 4608),
                                (2048, 512), (1000, 2048)],
                        M=4, grad="normal", grad_std=0.1, scale="spectral",
                        ns_steps=1, local_polar_steps=0, sign_fmt="1bit", stream=7),
}


def rng_for(stream, block=0, worker=0, what=0, seed=BASE_SEED):
    """Counter-based generator keyed on (seed, stream, block, worker, what)."""
    key = (int(seed) & 0xFFFFFFFF) | ((int(stream) & 0xFFFF) << 32) | ((int(what) & 0xFFFF) << 48)
    ctr = [int(block), int(worker), 0, 0]
    return np.random.Generator(np.random.Philox(key=key, counter=ctr))


def normal(shape, std=1.0, dtype=np.float32, **key):
    return (rng_for(**key).standard_normal(shape) * std).astype(dtype)


def student_t(shape, nu=3, dtype=np.float32, **key):
    """Z / sqrt(chi2_nu / nu) with independent normals."""
    g = rng_for(**key)
    z = g.standard_normal(shape)
    chi2 = np.sum(np.square(g.standard_normal((nu,) + tuple(shape))), axis=0)
    return (z / np.sqrt(chi2 / nu)).astype(dtype)


def worker_grads(name_or_cfg, block, rows, cols, M=None, dtype=np.float32, seed=BASE_SEED):
    """Per-worker stochastic gradients [M, rows, cols] for one block of a workload."""
    cfg = WORKLOADS[name_or_cfg] if isinstance(name_or_cfg, str) else name_or_cfg
    M = cfg["M"] if M is None else M
    kind, stream = cfg["grad"], cfg["stream"]
    out = np.empty((M, rows, cols), dtype=dtype)
    if kind == "lowrank":
        k = cfg["rank"]
        A = normal((rows, k), 1.0, np.float64, stream=stream, block=block, worker=0xFFFF, what=1, seed=seed)
        B = normal((cols, k), 1.0, np.float64, stream=stream, block=block, worker=0xFFFF, what=2, seed=seed)
        shared = (A @ B.T) / np.sqrt(k)
    for p in range(M):
        key = dict(stream=stream, block=block, worker=p, what=0, seed=seed)
        if kind == "normal":
            out[p] = normal((rows, cols), cfg["grad_std"], dtype, **key)
        elif kind == "student_t":
            out[p] = student_t((rows, cols), cfg["nu"], dtype, **key)
        elif kind == "lowrank":
            out[p] = (shared + normal((rows, cols), cfg["grad_std"], np.float64, **key)).astype(dtype)
        else:
            raise ValueError(kind)
    return out


def weights(rows, cols, block=0, stream=0, dtype=np.float32, seed=BASE_SEED):
    """W ~ N(0, 0.02^2)."""
    return normal((rows, cols), 0.02, dtype, stream=stream, block=block, worker=0xFFFE, what=3, seed=seed)


def start_vectors(M, cols, block=0, stream=0, dtype=np.float32, seed=BASE_SEED):
    """PowerIter start vectors v0 [M, cols] ~ N(0, 1)."""
    return normal((M, cols), 1.0, dtype, stream=stream, block=block, worker=0xFFFD, what=4, seed=seed)


def with_condition(rows, cols, cond, seed=0, dtype=np.float64):
    """Random matrix with prescribed singular values, log-spaced in [1/cond, 1]."""
    g = rng_for(99, block=rows, worker=cols, what=int(seed))
    s = min(rows, cols)
    Qu, _ = np.linalg.qr(g.standard_normal((rows, s)))
    Qv, _ = np.linalg.qr(g.standard_normal((cols, s)))
    sv = np.logspace(0.0, -np.log10(cond), s)
    return ((Qu * sv) @ Qv.T).astype(dtype), Qu, sv, Qv


def special_values_f32():
    """Sign-decision edge values: +-0, NaN, +-inf, denormals, tiny/huge normals."""
    return np.array([0.0, -0.0, np.nan, -np.nan, np.inf, -np.inf,
                     1e-45, -1e-45, 1e-39, -1e-39, 1.1754944e-38, -1.1754944e-38,
                     1.0, -1.0, 3.3895314e38, -3.3895314e38], dtype=np.float32)


def to_bf16_bits(x_f32):
    """float32 -> bfloat16 bit patterns (uint16), round-to-nearest-even; NaN kept NaN."""
    x = np.ascontiguousarray(x_f32, dtype=np.float32)
    u = x.view(np.uint32)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    nan = np.isnan(x)
    out = rounded.astype(np.uint16)
    out[nan] = ((u[nan] >> 16) | 0x0040).astype(np.uint16)
    return out


def from_bf16_bits(b_u16):
    """bfloat16 bit patterns -> float32 (exact)."""
    return (np.ascontiguousarray(b_u16, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)
