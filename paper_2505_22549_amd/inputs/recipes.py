"""Synthetic workload recipes: tensor lists, hyper-parameters and gradient
distributions of the five benchmark configurations.  INPUT DESCRIPTIONS ONLY: no
optimizer arithmetic lives here.

The tensor lists are shaped like the language models the paper trains (GPT-style
decoder blocks; the 1.7B entry follows the paper's model table: 24 blocks, d = 2048,
expansion ratio 4, gated SiLU MLP, rotary positions so no position table, vocabulary
50257 with tied embeddings).  Gradients are synthetic stand-ins for real training
gradients, which need the paper's datasets and models.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List

import numpy as np

ADAM, ADOPT, SGDM = 0, 1, 2
GAUSS, STUDENT_T3 = 0, 1


@dataclass
class Workload:
    name: str
    variant: int
    M: int
    steps: int
    Kx: int
    Ku: int
    Kv: int
    numel: np.ndarray             # uint64 [n_tensors]
    grad_scale: np.ndarray        # float32 [n_tensors], per-tensor gradient scale s_k
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    rho: float = float("inf")
    flags: int = 0
    grad_bf16: bool = False
    dist: int = GAUSS
    grad_mean0: float = 0.0
    grad_mean_per_replica: float = 0.0
    x0_std: float = 0.02
    seed: int = 0
    notes: str = ""

    @property
    def n_tensors(self) -> int:
        return int(self.numel.size)

    @property
    def total_numel(self) -> int:
        return int(self.numel.sum())

    @property
    def bytes_per_update(self) -> int:
        """Algorithmic HBM bytes per replica-parameter per step: every array read once
        and written once except the gradient (read only)."""
        gb = 2 if self.grad_bf16 else 4
        return (8 + 8 + gb) if self.variant == SGDM else (8 + 8 + 8 + gb)


def gpt2_style(layers: int, d: int, vocab: int = 50257, ctx: int = 1024) -> List[int]:
    t = [vocab * d, ctx * d]
    for _ in range(layers):
        t += [d, d, d * 3 * d, 3 * d, d * d, d, d, d, d * 4 * d, 4 * d, 4 * d * d, d]
    t += [d, d]
    return t


def llama_style(layers: int, d: int, vocab: int = 50257, ratio: int = 4) -> List[int]:
    t = [vocab * d]
    for _ in range(layers):
        t += [d, d * d, d * d, d * d, d * d, d, d * ratio * d, d * ratio * d, ratio * d * d]
    t += [d]
    return t


def _log_uniform(rng, lo, hi, n):
    return np.exp(rng.uniform(np.log(lo), np.log(hi), size=n))


def config1() -> Workload:
    return Workload("c1_adam_flat_1M_M4", ADAM, 4, 64, 16, 32, 64,
                    np.array([1 << 20], dtype=np.uint64), np.array([1e-2], dtype=np.float32),
                    lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, grad_mean_per_replica=0.01,
                    x0_std=0.02, seed=0)


def config2() -> Workload:
    numel = np.array(gpt2_style(12, 768), dtype=np.uint64)
    rng = np.random.default_rng(1)
    return Workload("c2_adam_gpt2small_124M_M8", ADAM, 8, 256, 32, 96, 192, numel,
                    _log_uniform(rng, 1e-4, 1e-1, numel.size).astype(np.float32),
                    rho=1.0, x0_std=768 ** -0.5, seed=1)


def config3() -> Workload:
    numel = np.array(gpt2_style(24, 1024), dtype=np.uint64)
    rng = np.random.default_rng(2)
    return Workload("c3_adopt_350M_M8", ADOPT, 8, 256, 64, 192, 384, numel,
                    _log_uniform(rng, 1e-4, 1e-1, numel.size).astype(np.float32),
                    lr=2.1e-3, beta1=0.9, beta2=0.9999, eps=1e-6, rho=1.0, dist=STUDENT_T3,
                    flags=4,  # ADOPT_INIT_G0SQ: keeps the first step O(1), as base ADOPT does
                    x0_std=1024 ** -0.5, seed=2)


def config4() -> Workload:
    rng = np.random.default_rng(3)
    numel = np.floor(_log_uniform(rng, 64, 262144, 7000)).astype(np.uint64)
    return Workload("c4_sgdm_7000_small_M4", SGDM, 4, 512, 16, 64, 0, numel,
                    np.full(7000, 1e-2, dtype=np.float32), lr=1e-3, beta1=0.9, grad_bf16=True,
                    x0_std=0.02, seed=3)


def config5() -> Workload:
    numel = np.array(llama_style(24, 2048), dtype=np.uint64)
    return Workload("c5_adam_1p7B_M4", ADAM, 4, 128, 128, 384, 768, numel,
                    np.full(numel.size, 1e-2, dtype=np.float32), rho=1.0,
                    grad_mean_per_replica=0.01, x0_std=2048 ** -0.5, seed=4)


def rosenbrock_toy() -> Workload:
    """The paper's toy example (Sec. 2.1 take-away box and its figure caption): minimise
    f(x1, x2) = (1 - x1)^2 + 100 (x2 - x1^2)^2 with M = 256 workers, IID Gaussian gradient noise
    sigma = 1.5 and periods (Kx, Ku, Kv) = (192, 192, 692).  Learning rate, betas and the start
    point are not printed; lr = 0.03, betas (0.9, 0.999) and the classical start (-1.2, 1) are
    this build's choice.  The gradient itself is the "model" and is evaluated by the caller
    (rosenbrock_grad below)."""
    return Workload("toy_rosenbrock_M256", ADAM, 256, 3000, 192, 192, 692,
                    np.array([2], dtype=np.uint64), np.array([1.5], dtype=np.float32),
                    lr=0.03, beta1=0.9, beta2=0.999, eps=1e-8, x0_std=0.0, seed=7,
                    notes="x0 = (-1.2, 1.0) on every worker")


def rosenbrock_grad(x: np.ndarray) -> np.ndarray:
    """Gradient of the Rosenbrock function at x[..., 2] (closed form)."""
    x1, x2 = x[..., 0], x[..., 1]
    return np.stack([-2.0 * (1.0 - x1) - 400.0 * x1 * (x2 - x1 * x1), 200.0 * (x2 - x1 * x1)], axis=-1)


CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}


def scaled_down(w: Workload, max_total: int, keep_tensors: int | None = None) -> Workload:
    """A smaller workload of the same structure for CPU-sized parity runs: every tensor
    is shrunk by a common factor (at least 1 element, odd sizes kept ragged)."""
    import copy
    s = copy.copy(w)
    numel = w.numel if keep_tensors is None else w.numel[:keep_tensors]
    scale = w.grad_scale if keep_tensors is None else w.grad_scale[:keep_tensors]
    f = max(1.0, float(numel.sum()) / max_total)
    s.numel = np.maximum(1, (numel / f).astype(np.uint64))
    s.grad_scale = scale.copy()
    s.name = w.name + "_small"
    return s
