"""Host-only checks of the seeded input generators that the oracle's tests and the GPU tests share:
determinism, ranges, the recipe's shapes, and the property that sample j of a batch does not depend on
the batch size (which lets an adaptive run and its oracle replay the same samples at any size)."""
import numpy as np
import pytest

from paper_2406_13936_amd import workloads as W


def test_index_j_does_not_depend_on_the_batch_size():
    a = W.batch_indices(0, 3, 1, 2, 16, 8192)
    b = W.batch_indices(0, 3, 1, 2, 512, 8192)
    assert np.array_equal(a, b[:16])
    assert a.dtype == np.int32 and a.min() >= 0 and b.max() < 8192


def test_indices_differ_between_steps_and_workers_and_repeat_exactly():
    base = W.batch_indices(7, 0, 0, 0, 256, 60000)
    assert np.array_equal(base, W.batch_indices(7, 0, 0, 0, 256, 60000))
    for other in (W.batch_indices(7, 1, 0, 0, 256, 60000), W.batch_indices(7, 0, 1, 0, 256, 60000),
                  W.batch_indices(7, 0, 0, 1, 256, 60000), W.batch_indices(8, 0, 0, 0, 256, 60000)):
        assert (other != base).mean() > 0.9


def test_indices_are_close_to_uniform():
    N = 1000
    idx = np.concatenate([W.batch_indices(1, k, 0, 0, 4096, N) for k in range(25)])
    counts = np.bincount(idx, minlength=N)
    # 102400 draws over 1000 cells: mean 102.4, std about 10.1
    assert counts.min() > 55 and counts.max() < 155
    assert abs(counts.std() - np.sqrt(102.4)) < 1.5


def test_step_indices_stack_the_workers():
    w = W.config1()
    idx = W.step_indices(w, 2, 3, 64)
    assert idx.shape == (w.M, 64)
    for m in range(w.M):
        assert np.array_equal(idx[m], W.batch_indices(w.seed, 2, 3, m, 64, w.N))


@pytest.mark.parametrize("cfg", ["config1", "config2"])
def test_datasets_follow_their_recipes(cfg):
    w = getattr(W, cfg)()
    X, y = W.make_dataset(w)
    X2, y2 = W.make_dataset(w)
    assert np.array_equal(X, X2) and np.array_equal(y, y2)            # seeded
    assert X.shape == (w.N, w.dims[0]) and X.dtype == np.float32
    assert y.shape == (w.N,) and y.dtype == np.int32
    assert y.min() >= 0 and y.max() < w.dims[-1]
    assert len(np.unique(y)) == w.dims[-1]                            # every class occurs
    if cfg == "config2":                                              # x ~ N(0, I)
        assert abs(X.mean()) < 5e-3 and abs(X.std() - 1.0) < 5e-3


def test_scaled_twin_keeps_depth_optimizer_and_test():
    w = W.config3()
    t = W.scaled_twin(w)
    assert len(t.dims) == len(w.dims) and t.dims[-1] == w.dims[-1]
    assert t.dims[1] == w.dims[1] // 8 and t.b_cap == w.b_cap // 16
    assert (t.act, t.opt, t.test, t.M, t.H) == (w.act, w.opt, w.test, w.M, w.H)
    X, y = W.make_dataset(t)
    # pixels in [0, 1] standardised per channel with the data's own statistics
    C = 3
    per = X.reshape(t.N, C, -1)
    assert np.abs(per.mean(axis=(0, 2))).max() < 1e-3 and np.abs(per.std(axis=(0, 2)) - 1.0).max() < 1e-3


def test_initial_parameters_are_bounded_and_biases_zero():
    w = W.config2()
    x0 = W.make_x0(w)
    assert x0.dtype == np.float32 and x0.size == w.n_params
    assert np.array_equal(x0, W.make_x0(w))
    o = 0
    for l in range(w.n_layers):
        fin, fout = w.dims[l], w.dims[l + 1]
        Wl = x0[o:o + fin * fout]
        o += fin * fout
        assert np.abs(Wl).max() <= 1.0 / np.sqrt(fin) and np.abs(Wl).max() > 0.99 / np.sqrt(fin)
        assert abs(Wl.mean()) < 3.0 / np.sqrt(fin) / np.sqrt(12.0 * Wl.size) * 3
        b = x0[o:o + fout]
        o += fout
        assert not b.any()


def test_stress_layers_are_standard_normal_and_per_replica():
    a, d = W.stats_stress_layer(0, 1, 2, 256, 128, 64)
    a2, d2 = W.stats_stress_layer(0, 1, 2, 256, 128, 64)
    assert np.array_equal(a, a2) and np.array_equal(d, d2)
    assert a.shape == (256, 128) and d.shape == (256, 64)
    assert abs(a.std() - 1.0) < 0.02 and abs(d.mean()) < 0.03
    b, _ = W.stats_stress_layer(0, 2, 2, 256, 128, 64)
    assert not np.array_equal(a, b)
