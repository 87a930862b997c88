"""Pins for the CPU oracle: each check ties one of its functions to something
other than itself (finite differences, explicit per-sample gradients, closed
forms, hand-worked fixtures, invariants of the method)."""
import math
import os

import numpy as np
import pytest

from oracle import abs_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _tiny(dims, act, has_bias, b, seed=0):
    rng = np.random.default_rng(seed)
    net = O.Net(dims, act, has_bias)
    x = rng.normal(0, 0.5, size=net.n_params)
    Xb = rng.normal(0, 1, size=(b, dims[0]))
    yb = rng.integers(0, dims[-1], size=b)
    return net, x, Xb, yb


# ---- backprop ------------------------------------------------------------

@pytest.mark.parametrize("act", [O.ACT_NONE, O.ACT_RELU, O.ACT_GELU])
@pytest.mark.parametrize("has_bias", [True, False])
def test_backprop_matches_central_differences(act, has_bias):
    net, x, Xb, yb = _tiny((5, 4, 6, 3), act, has_bias, b=7, seed=1)
    g = O.batch_gradient(net, x, Xb, yb)
    h = 1e-6
    for j in range(net.n_params):
        e = np.zeros_like(x)
        e[j] = h
        fd = (O.mean_loss(net, x + e, Xb, yb) - O.mean_loss(net, x - e, Xb, yb)) / (2 * h)
        assert abs(fd - g[j]) <= 1e-6 * max(1.0, abs(fd)), (j, fd, g[j])


def test_two_class_head_is_the_logistic_gradient():
    # K = 2, no hidden layer: d f / d W[1] = (sigmoid(z1 - z0) - y) x, and
    # the two rows of the gradient are opposite.
    net, x, Xb, yb = _tiny((6, 2), O.ACT_NONE, True, b=9, seed=2)
    (W, beta), = net.unpack(x)
    z = Xb @ W.T + beta
    p1 = 1.0 / (1.0 + np.exp(-(z[:, 1] - z[:, 0])))
    gw1 = ((p1 - yb)[:, None] * Xb).mean(axis=0)
    (G, gb), = net.unpack(O.batch_gradient(net, x, Xb, yb))
    np.testing.assert_allclose(G[1], gw1, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(G[0], -gw1, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(gb[1], (p1 - yb).mean(), rtol=1e-12)


def test_output_deltas_sum_to_zero_and_loss_is_minus_log_prob():
    net, x, Xb, yb = _tiny((5, 4, 3), O.ACT_RELU, True, b=6, seed=3)
    bp = O.backprop(net, x, Xb, yb)
    np.testing.assert_allclose(bp["delta"][-1].sum(axis=1), 0.0, atol=1e-14)
    # uniform logits (all-zero parameters) -> loss = log K
    bp0 = O.backprop(net, np.zeros_like(x), Xb, yb)
    np.testing.assert_allclose(bp0["loss"], math.log(3), rtol=1e-14)


def test_batch_gradient_is_mean_of_per_sample_gradients():
    net, x, Xb, yb = _tiny((5, 4, 3), O.ACT_GELU, True, b=6, seed=4)
    g = O.per_sample_gradients(net, x, Xb, yb)
    np.testing.assert_allclose(g.mean(axis=0), O.batch_gradient(net, x, Xb, yb),
                               rtol=1e-12, atol=1e-15)


# ---- statistics ------------------------------------------------------------

@pytest.mark.parametrize("act,has_bias,dims", [
    (O.ACT_RELU, True, (5, 4, 3)), (O.ACT_GELU, True, (6, 5, 4, 3)),
    (O.ACT_GELU, False, (6, 5, 3)), (O.ACT_NONE, True, (7, 4))])
def test_factored_statistics_equal_explicit_per_sample_gradients(act, has_bias, dims):
    net, x, Xb, yb = _tiny(dims, act, has_bias, b=6, seed=5)
    ex = O.stats_explicit(O.per_sample_gradients(net, x, Xb, yb))
    fa = O.stats_factored(net, O.backprop(net, x, Xb, yb), want_ip=True)
    for key in ("S1", "S2", "S3", "S4", "var", "var_q", "var_perp"):
        assert fa[key] == pytest.approx(ex[key], rel=1e-10, abs=1e-14), key
    np.testing.assert_allclose(fa["n"], ex["n"], rtol=1e-12)
    np.testing.assert_allclose(fa["q"], ex["q"], rtol=1e-10, atol=1e-14)


def test_variance_identities_and_inequalities():
    net, x, Xb, yb = _tiny((6, 5, 3), O.ACT_RELU, True, b=8, seed=6)
    g = O.per_sample_gradients(net, x, Xb, yb)
    s = O.stats_explicit(g)
    b = 8
    lit = sum(float(((g[i] - s["gbar"]) ** 2).sum()) for i in range(b))
    assert lit == pytest.approx(s["S1"] - b * s["S2"], rel=1e-12)
    assert s["var"] == pytest.approx(lit / (b - 1), rel=1e-12)
    assert s["S1"] >= b * s["S2"]                              # Jensen
    assert s["S4"] == pytest.approx(b * s["S2"], rel=1e-12)    # sum_i <g_i,gbar> = b||gbar||^2
    assert np.all(s["q"] ** 2 <= s["n"] * s["S2"] * (1 + 1e-12))   # Cauchy-Schwarz
    assert s["S3"] / s["S2"] <= s["S1"] * (1 + 1e-12)
    perp = g - np.outer(s["q"] / s["S2"], s["gbar"])
    np.testing.assert_allclose(perp.sum(axis=0), 0.0, atol=1e-12)  # orthogonal parts have zero mean
    assert s["var_perp"] == pytest.approx((s["S1"] - s["S3"] / s["S2"]) / (b - 1), rel=1e-12)


def test_identical_samples_have_zero_variance_and_keep_the_batch_size():
    net, x, Xb, yb = _tiny((5, 4, 3), O.ACT_RELU, True, b=1, seed=7)
    Xr, yr = np.repeat(Xb, 6, axis=0), np.repeat(yb, 6)
    s = O.stats_factored(net, O.backprop(net, x, Xr, yr))
    assert abs(s["var"]) <= 1e-12 * s["S1"]
    r = O.norm_test(max(s["var"], 0.0), s["S2"], 6, 0.5)
    assert r["pass"] and r["T"] <= 1
    assert O.next_batch_size([r["T"]], [6], 512) == [6]


def test_two_sample_variance_closed_form():
    net, x, Xb, yb = _tiny((5, 4, 3), O.ACT_GELU, True, b=2, seed=8)
    g = O.per_sample_gradients(net, x, Xb, yb)
    s = O.stats_factored(net, O.backprop(net, x, Xb, yb))
    assert s["var"] == pytest.approx(0.5 * float(((g[0] - g[1]) ** 2).sum()), rel=1e-11)


def test_ratio_scales_and_is_loss_scale_invariant():
    rng = np.random.default_rng(9)
    g = rng.normal(size=(10, 12)) + 0.3
    s, s3 = O.stats_explicit(g), O.stats_explicit(3.0 * g)
    r = O.norm_test(s["var"], s["S2"], 10, 0.5)
    r3 = O.norm_test(s3["var"], s3["S2"], 10, 0.5)
    assert r["ratio"] == pytest.approx(r3["ratio"], rel=1e-12)
    r_half = O.norm_test(s["var"], s["S2"], 10, 0.25)
    assert r_half["ratio"] == pytest.approx(4.0 * r["ratio"], rel=1e-12)
    i1 = O.inner_product_test(s["var_q"], s["var_perp"], s["S2"], 10, 0.9, 0.5)
    i3 = O.inner_product_test(s3["var_q"], s3["var_perp"], s3["S2"], 10, 0.9, 0.5)
    assert i1["ratio_ip"] == pytest.approx(i3["ratio_ip"], rel=1e-12)
    assert i1["ratio_perp"] == pytest.approx(i3["ratio_perp"], rel=1e-12)


def test_inner_product_test_on_a_hand_made_batch():
    # g_1 = (2, 0), g_2 = (0, 2): gbar = (1, 1), ||gbar||^2 = 2, q = (2, 2):
    # var_q = 0; orthogonal parts (1,-1), (-1,1): var_perp = (2 + 2)/(2-1) = 4.
    s = O.stats_explicit(np.array([[2.0, 0.0], [0.0, 2.0]]))
    assert s["var_q"] == 0.0 and s["var_perp"] == pytest.approx(4.0)
    r = O.inner_product_test(s["var_q"], s["var_perp"], s["S2"], 2, 0.9, 0.5)
    assert r["ratio_ip"] == 0.0
    assert r["ratio_perp"] == pytest.approx(4.0 / (0.25 * 2.0))     # = 8
    assert r["T"] == 8 and not r["pass"]
    # g = (1,0),(3,0): gbar=(2,0), q=(2,6), mean 4, var_q = (4+4)/1 = 8,
    # theta^2 ||gbar||^4 = 0.81*16 -> ratio = 8/12.96
    s = O.stats_explicit(np.array([[1.0, 0.0], [3.0, 0.0]]))
    r = O.inner_product_test(s["var_q"], s["var_perp"], s["S2"], 2, 0.9)
    assert r["ratio"] == pytest.approx(8.0 / 12.96) and r["T"] == 1 and r["pass"]


# ---- rule ------------------------------------------------------------------

def test_batch_rule_hand_worked_cases():
    rows = [l.split() for l in open(os.path.join(GOLD, "batch_rule_cases.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) >= 8
    for var, s2, b, eta, cap, T, bn, ok in rows:
        r = O.norm_test(float(var), float(s2), int(b), float(eta))
        assert r["T"] == int(T), (var, s2, b, eta)
        assert r["pass"] == bool(int(ok))
        assert O.next_batch_size([r["T"]], [int(b)], int(cap)) == [int(bn)]
        # "violated -> ceil, else unchanged" equals max{T, b} for integer b
        assert (r["T"] <= int(b)) == r["pass"]


def test_rule_max_over_workers_and_zero_gradient():
    assert O.next_batch_size([5, 40, 17], [16, 16, 16], 512, sync_max=True) == [40, 40, 40]
    assert O.next_batch_size([5, 40, 17], [16, 16, 16], 512, sync_max=False) == [16, 40, 17]
    assert O.next_batch_size([5, 4000, 17], [16, 16, 16], 512, sync_max=True) == [512] * 3
    r = O.norm_test(3.0, 0.0, 16, 0.5)
    assert r["T"] == 16                     # zero batch gradient: size unchanged


def test_cross_worker_estimator_closed_form():
    # M = 2: sum_m ||g^m - gbar||^2 = ||g^1 - g^2||^2 / 2
    g = np.array([[1.0, 2.0, 0.0], [3.0, 0.0, 0.0]])
    r = O.cross_worker_test(g, b=10, eta=0.5)
    assert r["var"] == pytest.approx(10 * 0.5 * 8.0 / 1.0)
    assert r["S2"] == pytest.approx(5.0)
    assert r["T"] == math.ceil(40.0 / (2 * 0.25 * 5.0))


# ---- optimizers --------------------------------------------------------------

def test_adamw_hand_worked_scalar():
    want = [float(l) for l in open(os.path.join(GOLD, "adamw_scalar_steps.txt"))
            if l.strip() and not l.startswith("#")]
    st, x = O.OptState(1), np.array([2.0])
    for g, w in zip((1.0, -1.0, 2.0), want):
        x = O.opt_step(x, np.array([g]), st, O.OPT_ADAMW, 0.5, beta1=0.5, beta2=0.75,
                       eps=0.0, weight_decay=0.25)
        assert x[0] == pytest.approx(w, rel=1e-14)


def test_adamw_first_step_is_a_sign_step():
    rng = np.random.default_rng(10)
    x, g = rng.normal(size=20), rng.normal(size=20)
    x1 = O.opt_step(x, g, O.OptState(20), O.OPT_ADAMW, 1e-2, eps=1e-8, weight_decay=0.1)
    want = x * (1 - 1e-3) - 1e-2 * g / (np.abs(g) + 1e-8)
    np.testing.assert_allclose(x1, want, rtol=1e-12)


def test_heavy_ball_closed_forms():
    rng = np.random.default_rng(11)
    x, g1, g2 = rng.normal(size=8), rng.normal(size=8), rng.normal(size=8)
    a = O.opt_step(x, g1, O.OptState(8), O.OPT_SHB, 0.1, momentum=0.0)
    np.testing.assert_allclose(a, O.opt_step(x, g1, O.OptState(8), O.OPT_SGD, 0.1))
    st = O.OptState(8)
    y = O.opt_step(x, g1, st, O.OPT_SHB, 0.1, momentum=0.9)
    y = O.opt_step(y, g2, st, O.OPT_SHB, 0.1, momentum=0.9)
    np.testing.assert_allclose(y, x - 0.1 * g1 - 0.1 * (0.9 * g1 + g2), rtol=1e-13)


# ---- local-gradient structure --------------------------------------------------

def _problem(seed=12, N=64, dims=(6, 5, 3), act=O.ACT_RELU):
    rng = np.random.default_rng(seed)
    net = O.Net(dims, act, True)
    X = rng.normal(size=(N, dims[0]))
    y = rng.integers(0, dims[-1], size=N)
    x0 = rng.normal(0, 0.4, size=net.n_params)
    return net, X, y, x0


def _idx_fn(N, M, seed=0):
    def f(k, h, b):
        rng = np.random.default_rng([seed, k, h])
        return rng.integers(0, N, size=(M, b))
    return f


def test_single_worker_is_minibatch_sgd():
    net, X, y, x0 = _problem()
    f = _idx_fn(64, 1)
    xs, sched, B = O.run(net, x0, X, y, M=1, H=3, rounds=4, b0=4, cap=32, lr=0.1,
                         idx_fn=f, eta=0.5, opt=O.OPT_SGD)
    x, b = x0.copy(), 4
    for k in range(4):
        for h in range(3):
            idx = f(k, h, b)[0]
            g = O.per_sample_gradients(net, x, X[idx], y[idx])
            s = O.stats_explicit(g)
            x = x - 0.1 * s["gbar"]
            T = math.ceil(s["var"] / (0.25 * s["S2"]))
            b = min(32, max(T, b))
    np.testing.assert_allclose(xs[0], x, rtol=1e-10, atol=1e-13)
    assert sched[-1][2] <= 32 and B == sum(s[2] for s in sched)
    assert [s[2] for s in sched] == sorted(s[2] for s in sched)   # sizes never decrease


@pytest.mark.parametrize("opt,kw", [(O.OPT_SGD, {}), (O.OPT_SHB, {"momentum": 0.9})])
def test_one_local_step_is_synchronous_large_batch(opt, kw):
    # H = 1 with equal local sizes: the averaged model follows the synchronous
    # method on the concatenated batch of size M b (mean of the local means).
    net, X, y, x0 = _problem(seed=13)
    M, b = 4, 5
    f = _idx_fn(64, M, seed=3)
    xs, _, _ = O.run(net, x0, X, y, M=M, H=1, rounds=6, b0=b, cap=b, lr=0.2,
                     idx_fn=f, opt=opt, **kw)
    g = lambda k, h, bb: f(k, h, b).reshape(1, M * b)
    x1, _, _ = O.run(net, x0, X, y, M=1, H=1, rounds=6, b0=M * b, cap=M * b, lr=0.2,
                     idx_fn=g, opt=opt, **kw)
    np.testing.assert_allclose(xs[0], x1[0], rtol=1e-9, atol=1e-12)


def test_average_properties():
    rng = np.random.default_rng(14)
    xs = rng.normal(size=(8, 11))
    av = O.average(xs)
    assert all(np.array_equal(av[0], av[m]) for m in range(8))
    np.testing.assert_allclose(av[0], xs.sum(axis=0) / 8, rtol=1e-15)
    same = np.tile(xs[0], (4, 1))
    np.testing.assert_array_equal(O.average(same), same)


def test_replicas_equal_after_each_round_and_smaller_eta_grows_faster():
    net, X, y, x0 = _problem(seed=15, N=256)
    f = _idx_fn(256, 3, seed=5)
    xs, s_big, _ = O.run(net, x0, X, y, M=3, H=2, rounds=3, b0=4, cap=128, lr=0.05,
                         idx_fn=f, eta=0.9)
    assert np.array_equal(xs[0], xs[1]) and np.array_equal(xs[0], xs[2])
    _, s_small, _ = O.run(net, x0, X, y, M=3, H=2, rounds=3, b0=4, cap=128, lr=0.05,
                          idx_fn=f, eta=0.2)
    assert s_small[1][2] >= s_big[1][2]      # first decision, same gradients


# ---- rounding ------------------------------------------------------------------

def test_bf16_rounding_against_known_values_and_torch():
    f = O.bf16_round
    assert f(1.0) == 1.0
    assert f(1.0 + 2.0 ** -8) == 1.0                       # tie -> even
    assert f(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6       # tie -> even
    assert f(1.0 + 2.0 ** -8 + 2.0 ** -20) == 1.0 + 2.0 ** -7
    assert f(-0.3) == -0.30078125
    assert f(0.0) == 0.0
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(16)
    v = (rng.normal(size=4000) * np.exp(rng.uniform(-20, 20, size=4000))).astype(np.float32)
    want = torch.from_numpy(v).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(f(v.astype(np.float64)), want)


def test_adagrad_closed_forms():
    # first step: x - lr g / (|g| + eps); two steps by hand on a scalar
    rng = np.random.default_rng(18)
    x, g = rng.normal(size=12), rng.normal(size=12)
    x1 = O.opt_step(x, g, O.OptState(12), O.OPT_ADAGRAD, 0.1, eps=1e-8)
    np.testing.assert_allclose(x1, x - 0.1 * g / (np.abs(g) + 1e-8), rtol=1e-13)
    st, y = O.OptState(1), np.array([1.0])
    y = O.opt_step(y, np.array([3.0]), st, O.OPT_ADAGRAD, 0.5, eps=0.0)      # v = 9  -> 1 - 0.5*3/3 = 0.5
    assert y[0] == pytest.approx(0.5)
    y = O.opt_step(y, np.array([4.0]), st, O.OPT_ADAGRAD, 0.5, eps=0.0)      # v = 25 -> 0.5 - 0.5*4/5 = 0.1
    assert y[0] == pytest.approx(0.1)


def test_lr_schedule_endpoints_and_shape():
    peak, floor, total, warm = 0.05, 0.005, 1000, 100
    f = lambda s: O.lr_schedule(s, total, warm, peak, floor)
    assert f(0) == pytest.approx(peak / warm) and f(warm - 1) == pytest.approx(peak)
    assert f(warm) == pytest.approx(peak) and f(total) == floor and f(total + 5) == floor
    assert f(warm + (total - warm) // 2) == pytest.approx(0.5 * (peak + floor))   # cosine midpoint
    vals = [f(s) for s in range(total + 1)]
    assert all(a <= b + 1e-15 for a, b in zip(vals[:warm], vals[1:warm]))          # warm-up rises
    assert all(a >= b - 1e-15 for a, b in zip(vals[warm:], vals[warm + 1:]))       # then decays
    assert min(vals[warm:]) >= floor - 1e-15


def test_finite_population_factor_in_the_norm_test():
    # b = n: the batch is the population, no sampling error -> T = 0 and the test passes
    r = O.norm_test(7.0, 0.01, 50, 0.5, n_total=50)
    assert r["T"] == 0 and r["pass"] and r["lhs"] == 0.0
    # n -> infinity: the factor tends to 1
    big = O.norm_test(7.0, 2.0, 50, 0.5, n_total=10 ** 15)
    ref = O.norm_test(7.0, 2.0, 50, 0.5)
    assert big["ratio"] == pytest.approx(ref["ratio"], rel=1e-12) and big["T"] == ref["T"]
    # hand case: var 12, b 4, n 10 -> 12 * 6/9 = 8; eta^2 S2 = 0.25 * 2 -> ratio 16
    r = O.norm_test(12.0, 2.0, 4, 0.5, n_total=10)
    assert r["ratio"] == pytest.approx(16.0) and r["T"] == 16 and not r["pass"]
    # brute force: the factor is the exact variance ratio of a mean of b draws without replacement
    # from a population of n versus b i.i.d. draws with the (n-1)-normalised population variance.
    import itertools
    pop = np.array([0.3, -1.2, 2.0, 0.7, -0.4])
    n, b = len(pop), 3
    means = [np.mean(c) for c in itertools.combinations(pop, b)]
    exact = float(np.mean((np.array(means) - pop.mean()) ** 2))
    assert exact == pytest.approx(pop.var(ddof=1) / b * (n - b) / n, rel=1e-12)        # textbook form
    # the paper's factor uses n - 1 with the 1/(b-1)-style variance; the two agree up to (n-1)/n
    assert (n - b) / (n - 1) == pytest.approx((n - b) / n * n / (n - 1))


def test_linear_lr_scaling():
    assert O.lr_linear_scaling(0.05, 2048, 256) == pytest.approx(0.4)
    assert O.lr_linear_scaling(0.05, 256, 256) == 0.05


def test_ragged_workers_are_independent_single_worker_runs():
    # a step with per-worker batch sizes equals M separate one-worker steps on the same batches
    net, x, Xb, yb = _tiny((6, 5, 3), O.ACT_RELU, True, b=40, seed=21)
    rows = [np.arange(0, 7), np.arange(7, 40), np.arange(3, 5)]
    rep = O.Replicas(net, x, Xb, yb, 3, opt=O.OPT_SHB, momentum=0.9, want_ip=True)
    rep.local_step(rows, 0.1)
    res = rep.test(O.TEST_NORM, eta=[0.3, 0.5, 0.7])
    for m, r in enumerate(rows):
        one = O.Replicas(net, x, Xb, yb, 1, opt=O.OPT_SHB, momentum=0.9, want_ip=True)
        one.local_step([r], 0.1)
        assert rep.stats[m]["b"] == len(r)
        for k in ("S1", "S2", "S3", "S4", "var"):
            assert rep.stats[m][k] == one.stats[0][k]
        np.testing.assert_array_equal(rep.x[m], one.x[0])
        np.testing.assert_allclose(rep.grads[m], O.per_sample_gradients(net, x, Xb[r], yb[r]).mean(axis=0),
                                   rtol=1e-11, atol=1e-15)
        assert res[m] == O.norm_test(one.stats[0]["var"], one.stats[0]["S2"], len(r), [0.3, 0.5, 0.7][m])
    assert O.next_batch_size([r["T"] for r in res], [7, 33, 2], 64, sync_max=False) == \
        [min(64, max(r["T"], b)) for r, b in zip(res, [7, 33, 2])]
