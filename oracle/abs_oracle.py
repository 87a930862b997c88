"""CPU oracle for adaptive-batch-size local gradient methods (test infrastructure).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the smoke
check and the benchmark's `cpu_baseline` leg may import it.  It is a plain,
slow, fp64 numpy restatement of what the hot path computes, written from the
paper's definitions; it shares no code with the HIP library and never calls it.

What it follows (paper: "Communication-Efficient Adaptive Batch Size Strategies
for Distributed Local Gradient Methods"):

* local batch gradient                      -- Sec. 3.1, eq. (batch_grad)
* Local SGD with averaging every H steps    -- Sec. 3.2, eq. (local_sgd_alt)
* batch variance with the 1/(b-1) factor    -- Sec. 4.1, eq. (def_var)
* approximate (local) norm test             -- eqs. (approx_norm), (approx_norm_local)
* batch-size rule, ceiling of the ratio     -- eqs. (norm_test), (test_stat)
* common size = max over workers            -- unnumbered display after (test_stat)
* the loop itself                           -- Appendix "Main Algorithm", Alg. 1
* inner optimizers beyond SGD (momentum SGD, AdaGrad, Adam, AdamW are named, not written out)
                                            -- Sec. 4.2, last paragraph; warm-up + cosine schedule: Sec. 6.1
* cross-worker estimator / once-per-round   -- Sec. 4.3 and Alg. 2

The (augmented) inner-product test is only *named* by the paper (end of
Sec. 4.1); its definition here is the one of the cited adaptive-sampling work
(Bollapragada, Byrd, Nocedal 2018): the sample variance of the inner products
<g_i, gbar> against theta^2 ||gbar||^4, and the variance of the components of
g_i orthogonal to gbar against nu^2 ||gbar||^2.

The model family (softmax cross-entropy on an MLP) is fixed by the workloads,
not by the paper.  Two numeric modes:

* exact : everything in fp64.
* mixed : same fp64 accumulation, but values are rounded to bfloat16
          (round-to-nearest-even) at the points where the bf16 device path
          stores bf16: dataset, weight shadow, stored activations a^l, stored
          activation derivative phi'(z^l), every backprop signal delta^l, and
          the batch gradient when it is used as the operand of the
          inner-product contraction (long batches only: for short ones the
          device sums the products <g_i, g_j> over j and never stores a bf16
          batch gradient, see `Replicas.gram_max_b`).  Biases, batch
          gradients, statistics, optimizer state and master weights are never
          rounded.

Parity status: every function here is pinned by tests/test_oracle_*.py (finite
differences, explicit per-sample gradients, closed forms, invariants).  The
inner-product test's *definition* is recalled from the cited work, not printed
in the paper: its arithmetic is pinned (explicit per-sample gradients), its
choice is a documented reading.
"""
from __future__ import annotations

import math
from typing import Callable, List, Optional, Sequence, Tuple

import numpy as np
from scipy.special import erf

ACT_NONE, ACT_RELU, ACT_GELU = 0, 1, 2
OPT_SGD, OPT_SHB, OPT_ADAMW, OPT_ADAGRAD = 0, 1, 2, 3
TEST_NORM, TEST_IP, TEST_AUG_IP = 0, 1, 2


# ---------------------------------------------------------------------------
# rounding
# ---------------------------------------------------------------------------

def bf16_round(x):
    """Round fp64 values to the nearest bfloat16 (8 significant bits, ties to
    even), returned as fp64."""
    x = np.asarray(x, dtype=np.float64)
    _, e = np.frexp(x)                       # |x| = m 2^e with 0.5 <= m < 1
    e = np.maximum(e, -125)                  # below 2^-126 the spacing is fixed
    q = np.ldexp(1.0, e - 8)
    return np.round(x / q) * q               # numpy rounds halves to even


def _ident(x):
    return np.asarray(x, dtype=np.float64)


# ---------------------------------------------------------------------------
# model: MLP with softmax cross-entropy
# ---------------------------------------------------------------------------

class Net:
    """dims[0] inputs, dims[-1] classes; layer l maps dims[l-1] -> dims[l]."""

    def __init__(self, dims: Sequence[int], act: int, has_bias: bool):
        self.dims = tuple(int(d) for d in dims)
        self.act = int(act)
        self.has_bias = bool(has_bias)
        self.L = len(self.dims) - 1

    @property
    def n_params(self) -> int:
        p = 0
        for l in range(self.L):
            p += self.dims[l] * self.dims[l + 1]
            if self.has_bias:
                p += self.dims[l + 1]
        return p

    def unpack(self, x: np.ndarray):
        """Packed vector -> [(W_l [out, in], beta_l [out] or None)], layer-major,
        W row-major then bias."""
        out, o = [], 0
        for l in range(self.L):
            fin, fout = self.dims[l], self.dims[l + 1]
            W = x[o:o + fin * fout].reshape(fout, fin)
            o += fin * fout
            beta = None
            if self.has_bias:
                beta = x[o:o + fout]
                o += fout
            out.append((W, beta))
        return out

    def pack(self, parts) -> np.ndarray:
        flat = []
        for W, beta in parts:
            flat.append(np.asarray(W, dtype=np.float64).reshape(-1))
            if self.has_bias:
                flat.append(np.asarray(beta, dtype=np.float64).reshape(-1))
        return np.concatenate(flat)


def _phi(z, act):
    if act == ACT_NONE:
        return z
    if act == ACT_RELU:
        return np.maximum(z, 0.0)
    return 0.5 * z * (1.0 + erf(z / math.sqrt(2.0)))          # exact GELU


def _dphi(z, act):
    if act == ACT_NONE:
        return np.ones_like(z)
    if act == ACT_RELU:
        return (z > 0.0).astype(np.float64)                    # phi'(0) = 0
    cdf = 0.5 * (1.0 + erf(z / math.sqrt(2.0)))
    pdf = np.exp(-0.5 * z * z) / math.sqrt(2.0 * math.pi)
    return cdf + z * pdf


def backprop(net: Net, x: np.ndarray, Xb: np.ndarray, yb: np.ndarray,
             mixed: bool = False):
    """Forward and backward pass over one batch.

    Per-sample loss f_i = -log softmax(z_i^L)[y_i]; delta_i^l = d f_i / d z_i^l
    (NOT divided by b).  Returns a dict with
      a      : [a^0 .. a^{L-1}]   inputs of each layer, [b, in_l]
      delta  : [delta^1 .. delta^L]                    [b, out_l]
      loss   : per-sample losses                        [b]
      G      : [(Gbar_l [out,in], betabar_l [out] | None)]  batch gradient,
               eq. (batch_grad): the mean of the per-sample gradients.
    """
    rnd = bf16_round if mixed else _ident
    params = net.unpack(np.asarray(x, dtype=np.float64))
    b = Xb.shape[0]
    a = [rnd(Xb)]
    dact = []
    z = None
    for l, (W, beta) in enumerate(params):
        z = a[-1] @ rnd(W).T
        if beta is not None:
            z = z + beta
        if l < net.L - 1:
            a.append(rnd(_phi(z, net.act)))
            dact.append(rnd(_dphi(z, net.act)))
    zmax = z.max(axis=1, keepdims=True)
    ez = np.exp(z - zmax)
    p = ez / ez.sum(axis=1, keepdims=True)
    rows = np.arange(b)
    loss = -(z[rows, yb] - zmax[:, 0] - np.log(ez.sum(axis=1)))
    d = p.copy()
    d[rows, yb] -= 1.0
    delta = [None] * net.L
    delta[net.L - 1] = rnd(d)
    for l in range(net.L - 1, 0, -1):
        W = rnd(params[l][0])
        delta[l - 1] = rnd((delta[l] @ W) * dact[l - 1])
    return {"a": a, "delta": delta, "loss": loss, "G": layer_gradients(a, delta, net.has_bias)}


def layer_gradients(a, delta, has_bias: bool):
    """Local batch gradient, eq. (batch_grad), layer by layer from the layer inputs a[l] [b, in_l] and the
    per-sample signals delta[l] [b, out_l]: the mean over the batch of the per-sample gradients
    delta_i^l a_i^{l-1 T} (and delta_i^l for the bias)."""
    b = a[0].shape[0]
    G = []
    for al, dl in zip(a, delta):
        Gl = (dl.T @ al) / b
        bl = dl.sum(axis=0) / b if has_bias else None
        G.append((Gl, bl))
    return G


def batch_gradient(net: Net, x, Xb, yb, mixed=False) -> np.ndarray:
    """Packed local batch gradient, eq. (batch_grad)."""
    return net.pack(backprop(net, x, Xb, yb, mixed)["G"])


def mean_loss(net: Net, x, Xb, yb) -> float:
    return float(backprop(net, x, Xb, yb)["loss"].mean())


def per_sample_gradients(net: Net, x, Xb, yb, mixed=False) -> np.ndarray:
    """[b, P] matrix of the per-sample gradients, each one obtained by running
    backprop on that sample alone (Alg. 1, "compute per-sample gradients").
    Tiny inputs only."""
    rows = []
    for i in range(Xb.shape[0]):
        rows.append(batch_gradient(net, x, Xb[i:i + 1], yb[i:i + 1], mixed))
    return np.stack(rows)


# ---------------------------------------------------------------------------
# statistics
# ---------------------------------------------------------------------------

def stats_explicit(g: np.ndarray) -> dict:
    """All test statistics from a materialised [b, P] per-sample gradient
    matrix, by the definitions written out (eq. def_var for every variance)."""
    b = g.shape[0]
    gbar = g.mean(axis=0)
    S1 = float((g * g).sum())
    S2 = float(gbar @ gbar)
    var = float(((g - gbar) ** 2).sum() / (b - 1))
    q = g @ gbar
    var_q = float(((q - q.mean()) ** 2).sum() / (b - 1))
    if S2 > 0.0:
        perp = g - np.outer(q / S2, gbar)
        var_perp = float((perp ** 2).sum() / (b - 1))
    else:
        var_perp = 0.0
    return {"b": b, "S1": S1, "S2": S2, "S3": float((q * q).sum()),
            "S4": float(q.sum()), "var": var, "var_q": var_q,
            "var_perp": var_perp, "n": (g * g).sum(axis=1), "q": q, "gbar": gbar}


def stats_factored(net: Net, bp: dict, want_ip: bool = True, mixed: bool = False,
                   round_gbar: bool = True) -> dict:
    """The same statistics without per-sample gradients.

    g_i restricted to layer l is the outer product delta_i^l a_i^{l-1 T} (plus
    delta_i^l for the bias), so
      ||g_i||^2   = sum_l ||delta_i^l||^2 (||a_i^{l-1}||^2 + [bias])
      <g_i, gbar> = sum_l delta_i^l . (Gbar_l a_i^{l-1} + betabar_l)
      sum_i ||g_i - gbar||^2 = S1 - b S2.
    In mixed mode Gbar_l is rounded to bf16 where it enters the contraction
    Gbar_l a_i (betabar_l stays unrounded), unless round_gbar is False."""
    a, delta, G = bp["a"], bp["delta"], bp["G"]
    b = a[0].shape[0]
    n = np.zeros(b)
    S2 = 0.0
    for l in range(net.L):
        an = (a[l] * a[l]).sum(axis=1)
        dn = (delta[l] * delta[l]).sum(axis=1)
        n += dn * (an + (1.0 if net.has_bias else 0.0))
        S2 += float((G[l][0] ** 2).sum())
        if net.has_bias:
            S2 += float((G[l][1] ** 2).sum())
    S1 = float(n.sum())
    out = {"b": b, "S1": S1, "S2": S2, "n": n,
           "var": (S1 - b * S2) / (b - 1), "loss_sum": float(bp["loss"].sum())}
    if want_ip:
        q = np.zeros(b)
        for l in range(net.L):
            Gl = bf16_round(G[l][0]) if (mixed and round_gbar) else G[l][0]
            u = a[l] @ Gl.T
            if net.has_bias:
                u = u + G[l][1]
            q += (delta[l] * u).sum(axis=1)
        S3, S4 = float((q * q).sum()), float(q.sum())
        out.update({"q": q, "S3": S3, "S4": S4,
                    "var_q": (S3 - S4 * S4 / b) / (b - 1),
                    "var_perp": ((S1 - S3 / S2) / (b - 1)) if S2 > 0.0 else 0.0})
    return out


# ---------------------------------------------------------------------------
# tests and batch-size rule
# ---------------------------------------------------------------------------

def _ceil_ratio(num: float, den: float, b: int) -> Tuple[float, int]:
    """ratio = num/den and its ceiling; a zero batch gradient (den == 0) leaves
    the batch size unchanged."""
    if not (den > 0.0):
        return float(b), int(b)
    r = num / den
    return r, int(math.ceil(r))


def norm_test(var: float, S2: float, b: int, eta: float, n_total: int = 0) -> dict:
    """Approximate norm test, eq. (approx_norm): var/b <= eta^2 ||gbar||^2;
    statistic T = ceil(var / (eta^2 ||gbar||^2)), eq. (norm_test) / Alg. 1.
    With n_total > 0 the variance carries the finite-population factor (n - b)/(n - 1) of the
    estimate of delta_B^2 in Sec. 4.1 (sampling b of n without replacement), taken at the
    current b."""
    if n_total > 0:
        var = var * (n_total - b) / (n_total - 1)
    ratio, T = _ceil_ratio(var, eta * eta * S2, b)
    return {"lhs": var / b, "rhs": eta * eta * S2, "ratio": ratio, "T": T,
            "pass": bool(var / b <= eta * eta * S2)}


def inner_product_test(var_q: float, var_perp: float, S2: float, b: int,
                       theta: float, nu: float = 0.0) -> dict:
    """Inner-product test: var_i(<g_i,gbar>)/b <= theta^2 ||gbar||^4.
    With nu > 0 also the orthogonality condition
    var_perp/b <= nu^2 ||gbar||^2; the statistic is the larger ceiling."""
    r_ip, T_ip = _ceil_ratio(var_q, theta * theta * S2 * S2, b)
    ok = bool(var_q / b <= theta * theta * S2 * S2)
    out = {"lhs": var_q / b, "rhs": theta * theta * S2 * S2, "ratio": r_ip,
           "T": T_ip, "pass": ok, "ratio_ip": r_ip, "ratio_perp": 0.0}
    if nu > 0.0:
        r_o, T_o = _ceil_ratio(var_perp, nu * nu * S2, b)
        out["ratio_perp"] = r_o
        out["T"] = max(T_ip, T_o)
        out["ratio"] = max(r_ip, r_o)
        out["pass"] = ok and bool(var_perp / b <= nu * nu * S2)
    return out


def next_batch_size(T: Sequence[int], b_cur: Sequence[int], cap: int,
                    sync_max: bool = True) -> List[int]:
    """b_next^m = max(T^m, b^m) (Alg. 1); with sync_max every worker takes the
    maximum over workers (display after eq. test_stat); never above `cap`."""
    nxt = [max(int(t), int(b)) for t, b in zip(T, b_cur)]
    if sync_max:
        nxt = [max(nxt)] * len(nxt)
    return [min(int(cap), v) for v in nxt]


def cross_worker_test(grads: np.ndarray, b: int, eta: float) -> dict:
    """Once-per-round test of Alg. 2 from the M local batch gradients:
    var = b/(M-1) sum_m ||g^m - gbar||^2, T = ceil(var / (M eta^2 ||gbar||^2))."""
    M = grads.shape[0]
    gbar = grads.mean(axis=0)
    var = b * float(((grads - gbar) ** 2).sum()) / (M - 1)
    S2 = float(gbar @ gbar)
    ratio, T = _ceil_ratio(var, M * eta * eta * S2, b)
    return {"var": var, "S2": S2, "ratio": ratio, "T": T,
            "sum_sq": float((grads * grads).sum())}


# ---------------------------------------------------------------------------
# inner optimizers (state is per worker, never averaged)
# ---------------------------------------------------------------------------

class OptState:
    def __init__(self, P: int):
        self.v = np.zeros(P)       # heavy-ball buffer / Adam second moment
        self.m = np.zeros(P)       # Adam first moment
        self.t = 0


def opt_step(x, g, st: OptState, opt: int, lr: float, momentum=0.0, beta1=0.9,
             beta2=0.999, eps=1e-8, weight_decay=0.0):
    if opt == OPT_SGD:
        return x - lr * g
    if opt == OPT_SHB:                       # v <- mu v + g ; x <- x - lr v
        st.v = momentum * st.v + g
        return x - lr * st.v
    if opt == OPT_ADAMW:                     # decoupled weight decay
        st.t += 1
        st.m = beta1 * st.m + (1.0 - beta1) * g
        st.v = beta2 * st.v + (1.0 - beta2) * g * g
        mhat = st.m / (1.0 - beta1 ** st.t)
        vhat = st.v / (1.0 - beta2 ** st.t)
        return x * (1.0 - lr * weight_decay) - lr * mhat / (np.sqrt(vhat) + eps)
    if opt == OPT_ADAGRAD:                   # v <- v + g^2 ; x <- x - lr g / (sqrt(v) + eps)
        st.v = st.v + g * g
        den = np.sqrt(st.v) + eps            # zero only where no gradient has ever arrived: no move
        return x - lr * np.divide(g, den, out=np.zeros_like(x), where=den > 0)
    raise ValueError(opt)


def lr_schedule(step: int, total_steps: int, warmup_steps: int, peak: float, floor: float) -> float:
    """Linear warm-up to `peak` over the first warmup_steps steps, then cosine decay to `floor`
    at total_steps (the schedule of the paper's experiments, Sec. 6.1 / hyper-parameter tables)."""
    if step < warmup_steps:
        return peak * (step + 1) / warmup_steps
    if step >= total_steps:
        return floor
    t = (step - warmup_steps) / max(1, total_steps - warmup_steps)
    return floor + 0.5 * (peak - floor) * (1.0 + math.cos(math.pi * t))


def lr_linear_scaling(lr_ref: float, b: int, b_ref: int) -> float:
    """Linear scaling of the learning rate with the batch size (Sec. 6.1, constant-batch
    baselines): lr = lr_ref * b / b_ref."""
    return lr_ref * b / b_ref


def average(xs: np.ndarray) -> np.ndarray:
    """Model averaging over the worker axis, eq. (local_sgd_alt)."""
    return np.tile(xs.mean(axis=0), (xs.shape[0], 1))


# ---------------------------------------------------------------------------
# the replicas, stepped call by call (mirrors the library's boundary)
# ---------------------------------------------------------------------------

class Replicas:
    def __init__(self, net: Net, x0, X, y, M: int, opt: int = OPT_SGD,
                 momentum=0.0, beta1=0.9, beta2=0.999, eps=1e-8,
                 weight_decay=0.0, mixed=False, want_ip=False, gram_max_b=0):
        self.net, self.M, self.opt, self.mixed = net, M, opt, mixed
        # mixed mode: a step whose largest local batch is at most this size keeps Gbar unrounded in
        # <g_i, gbar> (the device then adds <g_i, g_j> over j instead of contracting a stored bf16 Gbar)
        self.gram_max_b = gram_max_b
        self.hp = dict(momentum=momentum, beta1=beta1, beta2=beta2, eps=eps,
                       weight_decay=weight_decay)
        self.X = np.asarray(X, dtype=np.float64)
        self.y = np.asarray(y)
        self.x = np.tile(np.asarray(x0, dtype=np.float64), (M, 1))
        self.st = [OptState(net.n_params) for _ in range(M)]
        self.want_ip = want_ip
        self.stats: List[dict] = []
        self.grads: Optional[np.ndarray] = None

    def local_step(self, idx: np.ndarray, lr: float, only: Optional[Sequence[int]] = None):
        """One local step of every worker; idx[m] holds worker m's sample indices (an [M, b]
        array, or M arrays of different lengths for per-worker batch sizes).  The statistics
        refer to the gradient at the pre-update iterate.  With `only`, just the listed workers
        are stepped (the workers are independent between averages); the others keep their
        iterate, their optimizer state does not advance, and their entries of `stats` / `grads`
        are None / zero."""
        self.stats = []
        grads = []
        stepped = [m for m in range(self.M) if only is None or m in only]
        round_gbar = max(len(idx[m]) for m in stepped) > self.gram_max_b
        for m in range(self.M):
            if only is not None and m not in only:
                self.stats.append(None)
                grads.append(np.zeros(self.net.n_params))
                continue
            bp = backprop(self.net, self.x[m], self.X[idx[m]], self.y[idx[m]],
                          self.mixed)
            self.stats.append(stats_factored(self.net, bp, self.want_ip, self.mixed, round_gbar))
            g = self.net.pack(bp["G"])
            grads.append(g)
            self.x[m] = opt_step(self.x[m], g, self.st[m], self.opt, lr, **self.hp)
        self.grads = np.stack(grads)
        return self.stats

    def test(self, kind: int, eta=0.5, theta=0.9, nu=0.0) -> List[dict]:
        """Per-worker test on each worker's own batch (its own b^m; eta may be one constant per
        worker, eq. (approx_norm_local))."""
        out = []
        for m, s in enumerate(self.stats):
            if s is None:                        # worker left out of the last step
                out.append(None)
                continue
            if kind == TEST_NORM:
                eta_m = eta[m] if np.ndim(eta) else eta
                out.append(norm_test(s["var"], s["S2"], s["b"], eta_m))
            else:
                out.append(inner_product_test(
                    s["var_q"], s["var_perp"], s["S2"], s["b"], theta,
                    nu if kind == TEST_AUG_IP else 0.0))
        return out

    def average(self):
        self.x = average(self.x)


def run_alg2(net: Net, x0, X, y, M: int, H: int, rounds: int, b0: int, cap: int, lr: float,
             idx_fn: Callable[[int, int, int], np.ndarray], eta=0.5, mixed=False, **opt_kw):
    """Alg. 2 for a fixed number of rounds: H local steps at one batch size b_k for every worker, then the
    model average, then ONE test per round from the M local batch gradients of the round's last local step
    (cross_worker_test), b_{k+1} = max(T, b_k) (never above `cap`), and B grows by H M b_k.
    idx_fn(k, h, b) -> int [M, b].  Returns (final parameters [M, P], schedule [(k, b_k, T)], samples)."""
    rep = Replicas(net, x0, X, y, M, mixed=mixed, **opt_kw)
    b, B, sched = int(b0), 0, []
    for k in range(rounds):
        for h in range(H):
            rep.local_step(idx_fn(k, h, b), lr)
        rep.average()
        r = cross_worker_test(rep.grads, b, eta)
        sched.append((k, b, r["T"]))
        B += H * M * b
        b = min(int(cap), max(int(r["T"]), b))
    return rep.x, sched, B


def run(net: Net, x0, X, y, M: int, H: int, rounds: int, b0: int, cap: int,
        lr: float, idx_fn: Callable[[int, int, int], np.ndarray],
        test: int = TEST_NORM, eta=0.5, theta=0.9, nu=0.0, sync_max=True,
        mixed=False, **opt_kw):
    """Alg. 1 for a fixed number of rounds.  idx_fn(k, h, b) -> int [M, b].
    Returns (final parameters [M, P], schedule [(k, h, b, [T^m])], samples)."""
    rep = Replicas(net, x0, X, y, M, mixed=mixed, want_ip=(test != TEST_NORM), **opt_kw)
    b, B, sched = int(b0), 0, []
    for k in range(rounds):
        for h in range(H):
            rep.local_step(idx_fn(k, h, b), lr)
            res = rep.test(test, eta, theta, nu)
            sched.append((k, h, b, [r["T"] for r in res]))
            B += M * b
            b = next_batch_size([r["T"] for r in res], [b] * M, cap, sync_max)[0]
        rep.average()
    return rep.x, sched, B
