"""Seeded synthetic inputs for the adaptive-batch local-gradient hot path.

This module only *makes inputs*: datasets, labels, initial parameters and the
per-step sample indices.  It holds none of the method's arithmetic (no
gradients, statistics, tests, optimizers or averaging), so both the CPU oracle's
tests and the HIP path's tests can draw the very same arrays from it without
sharing any code of the method itself.

Every workload is synthetic and stands in for the shape of a public workload
(MNIST-like 784 inputs, CIFAR-100-like 3x32x32 inputs with 100 classes); no
real dataset is read.
"""
from __future__ import annotations

import dataclasses
from typing import Optional, Tuple

import numpy as np

ACT_NONE, ACT_RELU, ACT_GELU = 0, 1, 2
OPT_SGD, OPT_SHB, OPT_ADAMW, OPT_ADAGRAD = 0, 1, 2, 3
TEST_NORM, TEST_IP, TEST_AUG_IP = 0, 1, 2
PREC_F32, PREC_BF16 = 0, 1


@dataclasses.dataclass(frozen=True)
class Workload:
    """One configuration of the hot path (model, data recipe, schedule)."""

    name: str
    dims: Tuple[int, ...]          # layer widths, dims[0] = input features
    act: int
    has_bias: bool
    prec: int
    N: int                         # dataset size
    M: int                         # worker replicas
    H: int                         # local steps per communication round
    rounds: int
    b0: int
    b_cap: int
    opt: int
    lr: float
    momentum: float = 0.0
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.0
    test: int = TEST_NORM
    eta: float = 0.5               # norm test constant
    theta: float = 0.9             # inner-product test constant
    nu: float = 0.0                # orthogonality constant (augmented test)
    data: str = "mixture"          # data recipe key
    seed: int = 0

    @property
    def n_layers(self) -> int:
        return len(self.dims) - 1

    @property
    def n_params(self) -> int:
        p = 0
        for l in range(self.n_layers):
            p += self.dims[l] * self.dims[l + 1]
            if self.has_bias:
                p += self.dims[l + 1]
        return p


def config1() -> Workload:
    """Multinomial logistic regression, fp32, Gaussian-mixture data."""
    return Workload("cfg1_mlr256x10_f32", (256, 10), ACT_NONE, True, PREC_F32,
                    N=8192, M=4, H=4, rounds=20, b0=16, b_cap=512, opt=OPT_SGD,
                    lr=0.1, test=TEST_NORM, eta=0.5, data="mixture", seed=0)


def config2() -> Workload:
    """MLP 784-512-512-10, ReLU, bf16 operands, teacher-MLP labels."""
    return Workload("cfg2_mlp784_relu_bf16", (784, 512, 512, 10), ACT_RELU, True,
                    PREC_BF16, N=60000, M=8, H=16, rounds=50, b0=32, b_cap=4096,
                    opt=OPT_SGD, lr=0.05, test=TEST_NORM, eta=0.3,
                    data="teacher_mlp", seed=0)


def config3() -> Workload:
    """MLP 3072-2048x3-100, GELU, heavy ball, inner-product test."""
    return Workload("cfg3_mlp3072_gelu_bf16_shb", (3072, 2048, 2048, 2048, 100),
                    ACT_GELU, True, PREC_BF16, N=50000, M=16, H=8, rounds=30,
                    b0=64, b_cap=8192, opt=OPT_SHB, lr=0.1, momentum=0.9,
                    test=TEST_IP, theta=0.9, data="pixels_linear_teacher", seed=0)


def config4() -> Workload:
    """Same net and data as config 3, AdamW and the augmented test."""
    return Workload("cfg4_mlp3072_gelu_bf16_adamw", (3072, 2048, 2048, 2048, 100),
                    ACT_GELU, True, PREC_BF16, N=50000, M=32, H=32, rounds=20,
                    b0=128, b_cap=16384, opt=OPT_ADAMW, lr=1e-3, beta1=0.9,
                    beta2=0.999, eps=1e-8, weight_decay=0.05, test=TEST_AUG_IP,
                    theta=0.9, nu=0.5, data="pixels_linear_teacher", seed=0)


def scaled_twin(w: Workload, width_div: int = 8, cap_div: int = 16,
                N: Optional[int] = None, M: Optional[int] = None,
                rounds: Optional[int] = None) -> Workload:
    """A small twin of a workload: same depth, activation, optimizer and test,
    hidden and input widths divided by `width_div`, cap divided by `cap_div`."""
    dims = [max(8, (d // width_div) // 8 * 8) for d in w.dims[:-1]] + [w.dims[-1]]
    return dataclasses.replace(
        w, name=w.name + f"_twin{width_div}", dims=tuple(dims),
        b_cap=max(w.b0 * 2, w.b_cap // cap_div), N=N or max(2048, w.N // 8),
        M=M or w.M, rounds=rounds or w.rounds)


# --------------------------------------------------------------------------
# datasets
# --------------------------------------------------------------------------

def _gaussian_mixture(w: Workload, rng: np.random.Generator):
    d, K = w.dims[0], w.dims[-1]
    means = 3.0 * rng.normal(0.0, 1.0 / np.sqrt(d), size=(K, d))
    y = rng.integers(0, K, size=w.N)
    X = means[y] + rng.normal(0.0, 1.0, size=(w.N, d))
    return X.astype(np.float32), y.astype(np.int32)


def _teacher_mlp(w: Workload, rng: np.random.Generator, hidden: int = 256,
                 gumbel_scale: float = 0.5):
    d, K = w.dims[0], w.dims[-1]
    X = rng.normal(0.0, 1.0, size=(w.N, d)).astype(np.float32)
    T1 = rng.normal(0.0, 1.0 / np.sqrt(d), size=(d, hidden))
    T2 = rng.normal(0.0, 1.0 / np.sqrt(hidden), size=(hidden, K))
    logits = np.maximum(X.astype(np.float64) @ T1, 0.0) @ T2
    u = rng.uniform(1e-12, 1.0, size=logits.shape)
    logits = logits + gumbel_scale * (-np.log(-np.log(u)))
    return X, np.argmax(logits, axis=1).astype(np.int32)


def _pixels_linear_teacher(w: Workload, rng: np.random.Generator, channels: int = 3):
    d, K = w.dims[0], w.dims[-1]
    X = np.empty((w.N, d), dtype=np.float32)
    chunk = 4096
    for s in range(0, w.N, chunk):                     # bounded host memory
        e = min(w.N, s + chunk)
        X[s:e] = rng.random(size=(e - s, d), dtype=np.float32)
    per = d // channels if d % channels == 0 else d
    nch = d // per
    Xc = X.reshape(w.N, nch, per)
    for c in range(nch):                               # per-channel standardise
        mu = float(Xc[:, c, :].mean(dtype=np.float64))
        sd = float(Xc[:, c, :].std(dtype=np.float64))
        Xc[:, c, :] = (Xc[:, c, :] - np.float32(mu)) / np.float32(sd)
    T = rng.normal(0.0, 1.0 / np.sqrt(d), size=(d, K)).astype(np.float32)
    y = np.empty(w.N, dtype=np.int32)
    for s in range(0, w.N, chunk):
        e = min(w.N, s + chunk)
        y[s:e] = np.argmax(X[s:e] @ T, axis=1)
    return X, y


def make_dataset(w: Workload):
    """(X float32 [N, d], y int32 [N]) for the workload's recipe and seed."""
    rng = np.random.default_rng([w.seed, 0xDA7A])
    if w.data == "mixture":
        return _gaussian_mixture(w, rng)
    if w.data == "teacher_mlp":
        return _teacher_mlp(w, rng)
    if w.data == "pixels_linear_teacher":
        return _pixels_linear_teacher(w, rng)
    raise ValueError(w.data)


def make_x0(w: Workload) -> np.ndarray:
    """Initial parameters, packed layer-major: W_l row-major (out x in) then
    beta_l.  W ~ U(-1/sqrt(in), 1/sqrt(in)), biases zero."""
    rng = np.random.default_rng([w.seed, 0x1417])
    parts = []
    for l in range(w.n_layers):
        fin, fout = w.dims[l], w.dims[l + 1]
        bound = 1.0 / np.sqrt(fin)
        parts.append(rng.uniform(-bound, bound, size=fout * fin))
        if w.has_bias:
            parts.append(np.zeros(fout))
    return np.concatenate(parts).astype(np.float32)


# --------------------------------------------------------------------------
# sample indices: a counter-based generator, so element j of the batch drawn
# at (round k, local step h, worker m) does not depend on the batch size.
# --------------------------------------------------------------------------

_MASK = np.uint64(0xFFFFFFFFFFFFFFFF)


def _mix64(z: np.ndarray) -> np.ndarray:
    z = (z + np.uint64(0x9E3779B97F4A7C15)) & _MASK
    z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _MASK
    z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _MASK
    return z ^ (z >> np.uint64(31))


def batch_indices(seed: int, k: int, h: int, m: int, b: int, N: int) -> np.ndarray:
    """b indices in [0, N), uniform with replacement, for (k, h, m)."""
    with np.errstate(over="ignore"):
        key = _mix64(np.array([seed], dtype=np.uint64))
        for c in (k, h, m):
            key = _mix64(key ^ np.uint64(c))
        j = np.arange(b, dtype=np.uint64)
        u = _mix64(key ^ (j * np.uint64(0xD1342543DE82EF95) & _MASK)) >> np.uint64(32)
        return ((u * np.uint64(N)) >> np.uint64(32)).astype(np.int32)


def step_indices(w: Workload, k: int, h: int, b: int) -> np.ndarray:
    """int32 [M, b] indices of all replicas for local step (k, h)."""
    return np.stack([batch_indices(w.seed, k, h, m, b, w.N) for m in range(w.M)])


# --------------------------------------------------------------------------
# statistics-only stress inputs (stacked square layers, no model run)
# --------------------------------------------------------------------------

def stats_stress_layer(seed: int, m: int, l: int, b: int, fin: int, fout: int):
    """(a [b, fin], delta [b, fout]) ~ N(0,1) float32 for replica m, layer l."""
    rng = np.random.default_rng([seed, 0x57A7, m, l])
    a = rng.standard_normal(size=(b, fin), dtype=np.float32)
    d = rng.standard_normal(size=(b, fout), dtype=np.float32)
    return a, d
