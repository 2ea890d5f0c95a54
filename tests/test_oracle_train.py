"""Pins of the oracle's loss, update and training iteration (Section II: cross-entropy risk and gradient
descent; Algorithm 1) and of the schedules of Section IV / Appendix "Scheduler"."""
import numpy as np
import pytest
import scipy.special as sps

from oracle import layer as olayer
from oracle import mask as omask
from oracle import partition as opart
from oracle import train as otrain
from paper_2406_17611_amd import synth

KEY = 0x240617611


def test_cross_entropy_closed_forms():
    n, c = 7, 5
    labels = np.array([0, 4, -1, 2, 2, -1, 1])
    loss, d, correct = otrain.softmax_xent(np.zeros((n, c)), labels, 0.5)
    assert np.isclose(loss, 0.5 * 5 * np.log(c))                     # uniform prediction: log C per labelled row
    assert correct == 1                                              # all-equal logits: index 0 wins, one label is 0
    assert np.all(d[[2, 5]] == 0.0)                                  # unlabelled rows carry no gradient
    assert np.allclose(d.sum(axis=1), 0.0)                           # softmax minus one-hot sums to zero
    assert np.isclose(d[0, 0], 0.5 * (1 / c - 1)) and np.isclose(d[0, 1], 0.5 / c)
    # a confident correct prediction has (almost) no loss, a confident wrong one about the logit gap
    z = np.array([[30.0, 0.0, 0.0], [0.0, 30.0, 0.0]])
    loss, _, correct = otrain.softmax_xent(z, np.array([0, 0]), 1.0)
    assert correct == 1 and abs(loss - 30.0) < 1e-9
    # shift invariance and no overflow for large logits
    z = np.random.default_rng(0).standard_normal((6, 4)) * 50
    a = otrain.softmax_xent(z, np.arange(6) % 4, 1.0)
    b = otrain.softmax_xent(z + 1000.0, np.arange(6) % 4, 1.0)
    assert np.isclose(a[0], b[0]) and np.allclose(a[1], b[1]) and np.isfinite(b[0])


def test_cross_entropy_against_library_and_finite_differences():
    rng = np.random.default_rng(1)
    z = rng.standard_normal((40, 9)) * 3
    y = rng.integers(-1, 9, size=40)
    scale = 1.0 / max(1, int((y >= 0).sum()))
    loss, d, correct = otrain.softmax_xent(z, y, scale)
    logp = sps.log_softmax(z, axis=1)
    on = y >= 0
    assert np.isclose(loss, -scale * logp[on, y[on]].sum())
    assert correct == int((z.argmax(1)[on] == y[on]).sum())
    eps = 1e-6
    for _ in range(20):
        i, j = rng.integers(0, 40), rng.integers(0, 9)
        zp, zm = z.copy(), z.copy()
        zp[i, j] += eps
        zm[i, j] -= eps
        fd = (otrain.softmax_xent(zp, y, scale)[0] - otrain.softmax_xent(zm, y, scale)[0]) / (2 * eps)
        assert abs(fd - d[i, j]) < 1e-8


def test_gradient_step():
    w = np.array([[1.0, -2.0], [0.5, 0.0]])
    g = np.array([[0.5, 1.0], [-1.0, 2.0]])
    assert np.array_equal(otrain.sgd(w, g, 0.1), np.array([[0.95, -2.1], [0.6, -0.2]]))


def _task(conv="sage"):
    t = synth.labelled_sbm(n_blocks=3, block_size=60, p_in=0.12, p_out=0.01, width=8, hidden=12, n_parts=3, conv=conv,
                           seed=5)
    g = t.graph
    parts = opart.build_partitions(g.n, g.rowptr, g.colidx, g.vals, t.part, t.n_parts)
    rng = np.random.default_rng(3)
    weights = []
    for l in range(2):
        h1 = rng.standard_normal((t.widths[l], t.widths[l + 1])) * 0.4
        h0 = rng.standard_normal((t.widths[l], t.widths[l + 1])) * 0.4 if conv == "sage" else None
        weights.append((h1, h0))
    labels = np.where(t.train, t.labels, -1)
    return t, parts, weights, labels


@pytest.mark.parametrize("conv,ratio", [("sage", (1, 1)), ("gcn", (2, 1)), ("sage", (1, 0))])
def test_training_gradient_is_the_derivative_of_the_partitioned_loss(conv, ratio):
    """End to end: the weight gradients a training iteration applies are the derivatives of the loss that the same
    compressed forward pass evaluates (kept positions frozen), by central finite differences."""
    t, parts, weights, labels = _task(conv)
    acts = [olayer.RELU, olayer.IDENTITY]
    keep = [omask.keep_count(w, *ratio) for w in t.widths[:-1]]
    x0 = [t.features[p.local_gid].astype(np.float64) for p in parts]
    lab = [labels[p.local_gid] for p in parts]
    scale = 1.0 / int(t.train.sum())
    lr = 0.3
    new_w, loss, _, _, bwd, _ = otrain.train_step(parts, x0, weights, acts, keep, KEY, 4, lab, scale, lr)

    def loss_at(ws):
        fwd = olayer.network_forward(parts, x0, ws, acts, keep, KEY, 4)
        return sum(otrain.softmax_xent(fwd["x"][-1][p.q], lab[p.q], scale)[0] for p in parts)

    assert np.isclose(loss, loss_at(weights))
    rng = np.random.default_rng(9)
    eps = 1e-6
    for l in range(2):
        for tap in range(2 if conv == "sage" else 1):
            for _ in range(4):
                i, j = rng.integers(0, t.widths[l]), rng.integers(0, t.widths[l + 1])
                wp = [[a.copy() if a is not None else None for a in pair] for pair in weights]
                wm = [[a.copy() if a is not None else None for a in pair] for pair in weights]
                wp[l][tap][i, j] += eps
                wm[l][tap][i, j] -= eps
                fd = (loss_at(wp) - loss_at(wm)) / (2 * eps)
                assert abs(fd - bwd["dh"][l][tap][i, j]) <= 1e-6 * max(1.0, abs(fd))
            assert np.allclose(new_w[l][tap], weights[l][tap] - lr * bwd["dh"][l][tap])


def test_training_reduces_the_loss_and_learns_the_blocks():
    t, parts, weights, labels = _task("sage")
    acts = [olayer.RELU, olayer.IDENTITY]
    x0 = [t.features[p.local_gid].astype(np.float64) for p in parts]
    lab = [labels[p.local_gid] for p in parts]
    scale = 1.0 / int(t.train.sum())
    losses = []
    for step in range(60):
        ratio = omask.linear_ratio(8, 1, 2, 60, step)
        keep = [omask.keep_count(w, *ratio) for w in t.widths[:-1]]
        weights, loss, correct, *_ = otrain.train_step(parts, x0, weights, acts, keep, KEY, step, lab, scale, 0.5)
        losses.append(loss)
    assert losses[-1] < 0.5 * losses[0]
    assert correct > 0.8 * int(t.train.sum())


def test_schedules():
    # Section V's setting: linear, slope 5, maximum 128, minimum 1, 300 iterations
    assert omask.linear_ratio(128, 1, 5, 300, 0) == (128, 1)
    assert omask.linear_ratio(128, 1, 5, 300, 30) == (129, 2)          # 128 - 5 * 127 * 30 / 300 = 64.5
    assert omask.linear_ratio(128, 1, 5, 300, 60) == (1, 1)            # reaches the minimum after K / slope steps
    assert omask.linear_ratio(128, 1, 5, 300, 299) == (1, 1)
    seq = [omask.linear_ratio(16, 1, 1, 100, s) for s in range(100)]
    assert all(a[0] * b[1] > b[0] * a[1] for a, b in zip(seq, seq[1:]))   # strictly decreasing (Section IV)
    assert omask.fixed_increment_ratio(32, -3, 2, 0) == (32, 1) and omask.fixed_increment_ratio(32, -3, 2, 10) == (2, 1)
    # exponential: ratio base^(K - k + 1), clamped
    assert omask.exponential_ratio(2, 128, 1, 10, 10) == (2, 1)
    assert omask.exponential_ratio(2, 128, 1, 10, 8) == (8, 1)
    assert omask.exponential_ratio(2, 128, 1, 10, 4) == (128, 1) and omask.exponential_ratio(2, 128, 1, 10, 0) == (128, 1)
    assert omask.exponential_ratio(3, 100, 5, 6, 6) == (5, 1)          # 3 < c_min
    vals = [omask.exponential_ratio(2, 128, 1, 10, s)[0] for s in range(11)]
    assert vals == sorted(vals, reverse=True)
