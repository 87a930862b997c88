"""Pins for the oracle's `mixed` (bf16-rounding) mode and for the pieces of its driver loop that the
other pin file leaves open.  The rounding points are tied to (i) a hand-worked rational fixture in which
every single rounding call changes a stated output, and (ii) a recomputation in which the stored
tensors really are torch.bfloat16 tensors (the library's own cast, not the oracle's rounding routine)."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import abs_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _golden(name):
    out = {}
    for line in open(os.path.join(GOLD, name)):
        if line.strip() and not line.startswith("#"):
            key, *vals = line.split()
            out[key] = np.array([float(Fraction(v)) for v in vals])
    return out


def _chain_case():
    net = O.Net((2, 1, 3), O.ACT_GELU, True)
    u, c = 383 / 256, 645 / 512
    x = net.pack([(np.array([[259 / 256, 0.0]]), np.array([-1 / 64])),
                  (np.array([[u], [-u], [0.0]]), np.array([-c, c, 0.0]))])
    Xb = np.array([[257 / 256, 0.5], [257 / 256, -1.0], [257 / 256, 2.0]])
    yb = np.array([0, 0, 1])
    return net, x, Xb, yb


def _chain_outputs():
    net, x, Xb, yb = _chain_case()
    bp = O.backprop(net, x, Xb, yb, mixed=True)
    st = O.stats_factored(net, bp, True, mixed=True)
    return {"a1": bp["a"][1][0], "delta1": bp["delta"][0][:, 0], "gbar1": bp["G"][0][0][0],
            "betabar1": bp["G"][0][1], "gbar2": bp["G"][1][0][:, 0], "betabar2": bp["G"][1][1],
            "n": st["n"], "S2": np.array([st["S2"]]), "q": st["q"], "loss": bp["loss"]}


def _matches(got, want):
    ok = all(np.allclose(got[k], want[k], rtol=1e-13, atol=1e-15) for k in want)
    return ok and np.allclose(got["loss"], math.log(3.0), rtol=1e-13)


def test_mixed_chain_equals_the_hand_worked_fixture():
    want = _golden("mixed_chain.txt")
    got = _chain_outputs()
    for k in want:
        np.testing.assert_allclose(got[k], want[k], rtol=1e-13, atol=1e-15, err_msg=k)
    np.testing.assert_allclose(got["loss"], math.log(3.0), rtol=1e-13)
    # the gradient and the statistics are NOT rounded: -209/384 and S2 have no 8-bit representation
    assert got["gbar1"][0] != O.bf16_round(got["gbar1"][0])
    assert got["n"][0] != O.bf16_round(got["n"][0])
    # q was taken with the rounded gradient: its sum differs from b ||gbar||^2 by the rounding of Gbar
    assert abs(got["q"].sum() - 3 * got["S2"][0]) > 1e-4


def test_every_rounding_call_of_the_chain_changes_a_stated_output(monkeypatch):
    """Sensitivity of the fixture: skipping any single rounding call of the forward pass, the backward
    pass or the inner products (dataset, W1, GELU, GELU', W2 forward, delta^2, W2 backward, delta^1,
    Gbar1 operand, Gbar2 operand: ten calls) breaks the agreement with the hand-worked values; so does
    an extra rounding of a bias or of the batch gradient."""
    want = _golden("mixed_chain.txt")
    real = O.bf16_round
    counter = {"n": 0}

    def count(v):
        counter["n"] += 1
        return real(v)

    monkeypatch.setattr(O, "bf16_round", count)
    assert _matches(_chain_outputs(), want)
    n_calls = counter["n"]
    assert n_calls == 10
    for skip in range(n_calls):
        counter["n"] = 0

        def one_left_out(v, skip=skip):
            counter["n"] += 1
            return O._ident(v) if counter["n"] - 1 == skip else real(v)

        monkeypatch.setattr(O, "bf16_round", one_left_out)
        assert not _matches(_chain_outputs(), want), "rounding call %d does not matter" % skip
    monkeypatch.setattr(O, "bf16_round", real)
    # a rounded last-layer bias (161/128 instead of 645/512) moves the logits off zero: the loss is no longer ln 3
    net, x, Xb, yb = _chain_case()
    parts = net.unpack(x.copy())
    xb = net.pack([(parts[0][0], parts[0][1]), (parts[1][0], real(parts[1][1]))])
    assert not np.allclose(O.backprop(net, xb, Xb, yb, mixed=True)["loss"], math.log(3.0), rtol=1e-6)


def _torch_mixed(net, x, Xb, yb, leave_out=None):
    """The same pass with every stored tensor held as a real torch.bfloat16 tensor and every contraction
    taken in fp64 on the upcast values.  leave_out names one storage point that is kept in fp64."""
    torch = pytest.importorskip("torch")

    def store64(v, site):      # round an fp64 value straight to bf16 (no double rounding through fp32)
        t = torch.from_numpy(np.ascontiguousarray(v, dtype=np.float64))
        return t if site == leave_out else t.to(torch.bfloat16).to(torch.float64)

    params = net.unpack(np.asarray(x, dtype=np.float64))
    b = Xb.shape[0]
    a = [store64(Xb, "X")]
    dact, z = [], None
    for l, (Wl, beta) in enumerate(params):
        z = a[-1] @ store64(Wl, "W").T
        if beta is not None:
            z = z + torch.from_numpy(beta)
        if l < net.L - 1:
            zn = z.numpy()
            a.append(store64(O._phi(zn, net.act), "a"))
            dact.append(store64(O._dphi(zn, net.act), "dphi"))
    p = torch.softmax(z, dim=1)
    loss = -torch.log(p[torch.arange(b), torch.from_numpy(yb)])
    d = p.clone()
    d[torch.arange(b), torch.from_numpy(yb)] -= 1.0
    delta = [None] * net.L
    delta[-1] = store64(d.numpy(), "deltaL")
    for l in range(net.L - 1, 0, -1):
        delta[l - 1] = store64(((delta[l] @ store64(params[l][0], "W")) * dact[l - 1]).numpy(), "delta")
    n = torch.zeros(b, dtype=torch.float64)
    q = torch.zeros(b, dtype=torch.float64)
    S2, G = 0.0, []
    for l in range(net.L):
        Gl = delta[l].T @ a[l] / b
        bl = delta[l].sum(0) / b
        G.append((Gl.numpy(), bl.numpy()))
        n += (delta[l] ** 2).sum(1) * ((a[l] ** 2).sum(1) + (1.0 if net.has_bias else 0.0))
        S2 += float((Gl ** 2).sum()) + (float((bl ** 2).sum()) if net.has_bias else 0.0)
        uu = a[l] @ store64(Gl.numpy(), "Gop").T
        if net.has_bias:
            uu = uu + bl
        q += (delta[l] * uu).sum(1)
    return {"n": n.numpy(), "q": q.numpy(), "S2": S2, "loss": loss.numpy(), "G": G}


@pytest.mark.parametrize("act,dims,seed", [(O.ACT_GELU, (12, 9, 7, 5), 31), (O.ACT_RELU, (10, 8, 4), 32)])
def test_mixed_mode_equals_a_pass_with_real_bf16_storage(act, dims, seed):
    rng = np.random.default_rng(seed)
    net = O.Net(dims, act, True)
    x = rng.normal(0, 0.5, size=net.n_params)
    Xb = rng.normal(0, 1, size=(11, dims[0]))
    yb = rng.integers(0, dims[-1], size=11)
    bp = O.backprop(net, x, Xb, yb, mixed=True)
    st = O.stats_factored(net, bp, True, mixed=True)
    ref = _torch_mixed(net, x, Xb, yb)
    np.testing.assert_allclose(st["n"], ref["n"], rtol=1e-12)
    np.testing.assert_allclose(st["q"], ref["q"], rtol=1e-10, atol=1e-13)
    assert st["S2"] == pytest.approx(ref["S2"], rel=1e-12)
    np.testing.assert_allclose(bp["loss"], ref["loss"], rtol=1e-12)
    for (Gl, bl), (Rl, rl) in zip(bp["G"], ref["G"]):
        np.testing.assert_allclose(Gl, Rl, rtol=1e-11, atol=1e-14)
        np.testing.assert_allclose(bl, rl, rtol=1e-11, atol=1e-14)
    # and each storage point matters on this net: the recomputation with that point kept in fp64 differs
    sites = ["X", "W", "a", "deltaL", "delta", "Gop"] + (["dphi"] if act == O.ACT_GELU else [])
    for site in sites:
        alt = _torch_mixed(net, x, Xb, yb, leave_out=site)
        moved = max(np.abs(alt["n"] - ref["n"]).max() / np.abs(ref["n"]).max(),
                    np.abs(alt["q"] - ref["q"]).max() / np.abs(ref["q"]).max())
        assert moved > 1e-5, site


def test_mixed_mode_stays_within_the_bf16_bound_of_exact():
    rng = np.random.default_rng(17)
    net = O.Net((32, 24, 16, 5), O.ACT_GELU, True)
    x = rng.normal(0, 0.5, size=net.n_params)
    Xb = rng.normal(0, 1, size=(40, 32))
    yb = rng.integers(0, 5, size=40)
    ex = O.stats_factored(net, O.backprop(net, x, Xb, yb), True)
    mx = O.stats_factored(net, O.backprop(net, x, Xb, yb, mixed=True), True, mixed=True)
    for key in ("S1", "S2", "S3", "S4"):
        assert mx[key] == pytest.approx(ex[key], rel=2e-2), key
        assert mx[key] != ex[key]


# ---- remaining pieces of the driver loop -------------------------------------------------------

def test_relu_derivative_at_zero_is_zero():
    # hidden pre-activation exactly 0 (zero weights, zero bias): no signal passes, the first layer's
    # gradient vanishes and n_i keeps only the last layer's term ||delta^2||^2 (||a^1||^2 + 1) = ||delta^2||^2
    net = O.Net((3, 2, 2), O.ACT_RELU, True)
    x = net.pack([(np.zeros((2, 3)), np.zeros(2)), (np.array([[1.0, -2.0], [0.5, 3.0]]), np.zeros(2))])
    Xb = np.array([[1.0, 2.0, 3.0], [-1.0, 0.5, 2.0]])
    yb = np.array([0, 1])
    bp = O.backprop(net, x, Xb, yb)
    assert np.all(bp["delta"][0] == 0.0) and np.all(bp["G"][0][0] == 0.0)
    st = O.stats_factored(net, bp, False)
    np.testing.assert_allclose(st["n"], [0.5, 0.5], rtol=1e-14)      # p = (1/2, 1/2): ||delta^2||^2 = 1/2


def test_sample_counter_adds_the_sizes_of_all_workers():
    rng = np.random.default_rng(40)
    net = O.Net((6, 5, 3), O.ACT_RELU, True)
    X, y = rng.normal(size=(64, 6)), rng.integers(0, 3, size=64)
    x0 = rng.normal(0, 0.4, size=net.n_params)

    def idx(k, h, b):
        return np.random.default_rng([7, k, h]).integers(0, 64, size=(3, b))

    # constant size (cap = b0): Alg. 1 adds b for every worker and local step: 2 rounds x 2 steps x 3 workers x 4
    _, sched, B = O.run(net, x0, X, y, M=3, H=2, rounds=2, b0=4, cap=4, lr=0.1, idx_fn=idx)
    assert B == 48 and [s[2] for s in sched] == [4, 4, 4, 4]
    # growing sizes: the sum over steps of M times the size each step actually used
    _, sched, B = O.run(net, x0, X, y, M=3, H=2, rounds=3, b0=4, cap=64, lr=0.1, idx_fn=idx, eta=0.3)
    assert sched[-1][2] > 4 and B == 3 * sum(s[2] for s in sched)


def test_inner_product_test_fails_on_its_own_condition():
    # g = (0,0), (4,0): gbar = (2,0), ||gbar||^2 = 4, q = (0, 8), mean 4, var_q = (16 + 16)/(2 - 1) = 32;
    # var_q / b = 16 > theta^2 ||gbar||^4 = 0.81 * 16 = 12.96: the inner-product condition fails although both
    # samples are parallel to gbar (orthogonal parts 0: the orthogonality condition holds for any nu).
    s = O.stats_explicit(np.array([[0.0, 0.0], [4.0, 0.0]]))
    assert s["var_q"] == pytest.approx(32.0) and s["var_perp"] == 0.0
    for nu in (0.0, 0.5):
        r = O.inner_product_test(s["var_q"], s["var_perp"], s["S2"], 2, 0.9, nu)
        assert not r["pass"] and r["T"] == 3 and r["ratio"] == pytest.approx(32.0 / 12.96)
        assert r["lhs"] == pytest.approx(16.0) and r["rhs"] == pytest.approx(12.96)
    assert O.next_batch_size([3], [2], 64) == [3]


def test_plain_inner_product_test_ignores_nu():
    # statistics of the batch (2,0), (0,2): var_q = 0, var_perp = 4, ||gbar||^2 = 2.  The plain test sees only
    # var_q (T = 0, pass); the augmented one with nu = 0.5 gives ceil(4 / (0.25 * 2)) = 8 and fails.
    net = O.Net((2, 2), O.ACT_NONE, False)
    rep = O.Replicas(net, np.zeros(4), np.zeros((2, 2)), np.zeros(2, dtype=int), 1, want_ip=True)
    rep.stats = [{"b": 2, "S2": 2.0, "var_q": 0.0, "var_perp": 4.0, "var": 4.0}]
    plain = rep.test(O.TEST_IP, theta=0.9, nu=0.5)[0]
    aug = rep.test(O.TEST_AUG_IP, theta=0.9, nu=0.5)[0]
    assert plain["T"] == 0 and plain["pass"] and plain["ratio_perp"] == 0.0
    assert aug["T"] == 8 and not aug["pass"] and aug["ratio_perp"] == pytest.approx(8.0)


def test_alg2_loop_tests_once_per_round_on_the_last_gradients():
    rng = np.random.default_rng(41)
    net = O.Net((6, 5, 3), O.ACT_RELU, True)
    X, y = rng.normal(size=(128, 6)), rng.integers(0, 3, size=128)
    x0 = rng.normal(0, 0.4, size=net.n_params)
    M, H = 3, 2

    def idx(k, h, b):
        return np.random.default_rng([9, k, h]).integers(0, 128, size=(M, b))

    # constant size (cap = b0): the iterates are those of Alg. 1 at that size, and B = rounds * H * M * b
    xs2, sched2, B2 = O.run_alg2(net, x0, X, y, M=M, H=H, rounds=3, b0=4, cap=4, lr=0.1, idx_fn=idx)
    xs1, _, B1 = O.run(net, x0, X, y, M=M, H=H, rounds=3, b0=4, cap=4, lr=0.1, idx_fn=idx)
    np.testing.assert_array_equal(xs2, xs1)
    assert B2 == B1 == 3 * H * M * 4 and [s[1] for s in sched2] == [4, 4, 4]
    # growing: replay the loop by hand with explicit per-sample gradients; the test uses the gradients of the
    # round's last local step, taken at the iterates before that step, and the round's size for every step
    xs, sched, B = O.run_alg2(net, x0, X, y, M=M, H=H, rounds=3, b0=4, cap=64, lr=0.1, idx_fn=idx, eta=0.4)
    x = np.tile(x0, (M, 1))
    b, Bh = 4, 0
    for k in range(3):
        for h in range(H):
            ii = idx(k, h, b)
            g = np.stack([O.per_sample_gradients(net, x[m], X[ii[m]], y[ii[m]]).mean(axis=0) for m in range(M)])
            x = x - 0.1 * g
        x = np.tile(x.mean(axis=0), (M, 1))
        gbar = g.mean(axis=0)
        var = b / (M - 1) * sum(float(((g[m] - gbar) ** 2).sum()) for m in range(M))
        T = math.ceil(var / (M * 0.16 * float(gbar @ gbar)))
        assert sched[k] == (k, b, T)
        Bh += H * M * b
        b = min(64, max(T, b))
    assert B == Bh and sched[-1][1] > 4
    np.testing.assert_allclose(xs, x, rtol=1e-10, atol=1e-13)


# ---- <g_i, gbar> with and without the rounding of Gbar ----------------------------------------

def test_unrounded_gbar_operand_equals_the_sum_of_per_sample_products():
    """With round_gbar off the mixed q_i is the mean over j of <g_i, g_j> taken from per-sample gradients
    that were each formed on their own (batches of one sample through the same rounding points); with it on,
    q_i is the product with the rounded mean, which differs by at most the bf16 rounding of that mean."""
    rng = np.random.default_rng(23)
    net = O.Net((12, 9, 7, 4), O.ACT_GELU, True)
    x = O.bf16_round(rng.normal(0, 0.5, size=net.n_params))
    Xb = rng.normal(0, 1, size=(11, 12))
    yb = rng.integers(0, 4, size=11)
    g = O.per_sample_gradients(net, x, Xb, yb, mixed=True)              # [b, P], one backprop per sample
    gram = g @ g.T
    want = gram.mean(axis=1)
    bp = O.backprop(net, x, Xb, yb, mixed=True)
    plain = O.stats_factored(net, bp, True, mixed=True, round_gbar=False)
    np.testing.assert_allclose(plain["q"], want, rtol=1e-12, atol=1e-15)
    # the same sum layer by layer: (delta_i . delta_j)(a_i . a_j + 1), the form the short-batch device path adds up
    by_layer = np.zeros_like(gram)
    for a, d in zip(bp["a"], bp["delta"]):
        by_layer += (d @ d.T) * (a @ a.T + 1.0)
    np.testing.assert_allclose(by_layer, gram, rtol=1e-12, atol=1e-15)
    rounded = O.stats_factored(net, bp, True, mixed=True, round_gbar=True)
    diff = np.abs(rounded["q"] - plain["q"])
    assert diff.max() > 0.0
    # |<g_i, bf16(gbar) - gbar>| <= 2^-9 sum_k |g_ik gbar_k| over the weight entries
    gbar = g.mean(axis=0)
    assert np.all(diff <= 2.0 ** -9 * (np.abs(g) * np.abs(gbar)).sum(axis=1) + 1e-15)
    # exact mode has no rounding to switch off
    e1 = O.stats_factored(net, O.backprop(net, x, Xb, yb), True, round_gbar=False)
    e2 = O.stats_factored(net, O.backprop(net, x, Xb, yb), True, round_gbar=True)
    assert np.array_equal(e1["q"], e2["q"])


def test_replicas_choose_the_operand_rounding_by_the_largest_local_batch():
    rng = np.random.default_rng(29)
    net = O.Net((6, 5, 3), O.ACT_RELU, True)
    X, y = rng.normal(size=(64, 6)), rng.integers(0, 3, size=64)
    x0 = rng.normal(0, 0.4, size=net.n_params)

    def q_of(gram_max_b, sizes):
        rep = O.Replicas(net, x0, X, y, len(sizes), mixed=True, want_ip=True, gram_max_b=gram_max_b)
        rep.local_step([np.arange(n) for n in sizes], 0.1)
        return [s["q"] for s in rep.stats]

    def direct(n, round_gbar):
        bp = O.backprop(net, x0, X[:n], y[:n], mixed=True)
        return O.stats_factored(net, bp, True, mixed=True, round_gbar=round_gbar)["q"]

    assert np.array_equal(q_of(0, [8, 8])[0], direct(8, True))          # default: always the rounded operand
    assert np.array_equal(q_of(8, [8, 8])[1], direct(8, False))         # b <= limit: unrounded
    assert np.array_equal(q_of(7, [8, 8])[1], direct(8, True))          # b above the limit
    ragged = q_of(8, [6, 9])                                            # the largest batch decides for every worker
    assert np.array_equal(ragged[0], direct(6, True)) and np.array_equal(ragged[1], direct(9, True))
    assert not np.array_equal(direct(8, True), direct(8, False))
