"""Pins of the training-loop oracle (oracle/train.py) against things other than itself: library routines
(torch's CPU cross-entropy with autograd, torch.optim), closed forms, a published test vector, finite
differences through the whole chunked model, and invariances of Algorithm 1."""
from __future__ import annotations

import math
import os

import numpy as np
import pytest
import torch

from helpers import make_train_problem, new_oracle_trainer
from oracle.train import adam_step, bf16_round, chunk_order, sgd_step, softmax_xent, splitmix64

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


# ---------------------------------------------------------------- chunk shuffling (Section 3.4, technique 1)
def test_splitmix64_published_vector():
    # first outputs of the reference generator seeded with 1234567 (state advances by the golden gamma)
    want = [int(x) for x in open(os.path.join(GOLDEN, "splitmix64_seed1234567.txt")).read().split("\n") if x and not x.startswith("#")]
    got = [splitmix64((1234567 + (i + 1) * 0x9E3779B97F4A7C15) & ((1 << 64) - 1)) for i in range(len(want))]
    assert got == want


def test_chunk_order_is_a_seeded_permutation():
    for K in (1, 2, 3, 8, 32, 255):
        seen = set()
        for epoch in range(6):
            o = chunk_order(11, epoch, K)
            assert sorted(o.tolist()) == list(range(K))
            assert np.array_equal(o, chunk_order(11, epoch, K))
            seen.add(tuple(o.tolist()))
        if K >= 8:
            assert len(seen) == 6  # a fresh order every epoch
        assert np.array_equal(chunk_order(11, 3, K, shuffle=False), np.arange(K))


def test_chunk_order_spreads_staleness_evenly():
    # the point of the technique: over many epochs every chunk sits at every position about equally often
    K, E = 8, 8000
    counts = np.zeros((K, K))
    for e in range(E):
        o = chunk_order(5, e, K)
        counts[o, np.arange(K)] += 1
    expected = E / K
    chi2 = ((counts - expected) ** 2 / expected).sum()
    assert chi2 < 120.0  # 49 degrees of freedom; 120 is far in the tail
    assert abs(counts / E - 1.0 / K).max() < 0.02


# ---------------------------------------------------------------- loss head
def test_softmax_xent_against_library_autograd():
    rng = np.random.default_rng(1)
    for rows, C in ((1, 2), (7, 5), (64, 41), (33, 100)):
        z = rng.normal(size=(rows, C)) * 3
        y = rng.integers(0, C, size=rows)
        mask = rng.random(rows) < 0.6
        if not mask.any():
            mask[0] = True
        n_train = int(mask.sum())
        loss, g = softmax_xent(z, y, mask, n_train)
        zt = torch.tensor(z, dtype=torch.float64, requires_grad=True)
        lt = torch.nn.functional.cross_entropy(zt[torch.tensor(mask)], torch.tensor(y)[torch.tensor(mask)], reduction="sum") / n_train
        lt.backward()
        assert abs(loss - lt.item()) < 1e-12 * max(1.0, abs(lt.item()))
        np.testing.assert_allclose(g, zt.grad.numpy(), rtol=0, atol=1e-14)


def test_softmax_xent_closed_forms_and_invariances():
    rows, C = 5, 7
    y = np.array([0, 3, 6, 2, 2])
    loss, g = softmax_xent(np.zeros((rows, C)), y, None, rows)
    assert abs(loss - math.log(C)) < 1e-15            # uniform prediction
    want = np.full((rows, C), 1.0 / C)
    want[np.arange(rows), y] -= 1.0
    np.testing.assert_allclose(g, want / rows, atol=1e-16)
    rng = np.random.default_rng(2)
    z = rng.normal(size=(rows, C))
    l1, g1 = softmax_xent(z, y, None, rows)
    l2, g2 = softmax_xent(z + rng.normal(size=(rows, 1)) * 50, y, None, rows)   # a shift per row changes nothing
    assert abs(l1 - l2) < 1e-12 and np.abs(g1 - g2).max() < 1e-14
    assert np.abs(g1.sum(axis=1)).max() < 1e-16        # probabilities sum to one
    l3, g3 = softmax_xent(z * 1e4, y, None, rows)      # no overflow
    assert np.isfinite(l3) and np.isfinite(g3).all()
    # a confident, correct prediction has (almost) no loss and no gradient
    zc = np.full((rows, C), -40.0)
    zc[np.arange(rows), y] = 40.0
    l4, g4 = softmax_xent(zc, y, None, rows)
    assert l4 < 1e-30 and np.abs(g4).max() < 1e-30
    # unlabelled rows are ignored whatever they hold
    mask = np.array([1, 0, 1, 0, 1], bool)
    z2 = z.copy()
    z2[~mask] = 1e3
    la, ga = softmax_xent(z, y, mask, 3)
    lb, gb = softmax_xent(z2, y, mask, 3)
    assert la == lb and np.array_equal(ga, gb) and np.all(ga[~mask] == 0)


# ---------------------------------------------------------------- optimisers
def test_adam_against_library_and_closed_forms():
    rng = np.random.default_rng(3)
    p0 = rng.normal(size=(6, 5))
    for wd in (0.0, 0.01):
        p, m, v = p0.copy(), np.zeros_like(p0), np.zeros_like(p0)
        pt = torch.tensor(p0, dtype=torch.float64, requires_grad=True)
        opt = torch.optim.Adam([pt], lr=0.01, betas=(0.9, 0.999), eps=1e-8, weight_decay=wd)
        for t in range(1, 8):
            g = rng.normal(size=p0.shape) * (0.1 if t % 2 else 3.0)
            adam_step(p, g, m, v, t, 0.01, 0.9, 0.999, 1e-8, wd)
            pt.grad = torch.tensor(g)
            opt.step()
            np.testing.assert_allclose(p, pt.detach().numpy(), rtol=0, atol=1e-13)
    # first step: m_hat = g, v_hat = g^2, so every entry moves by lr * g / (|g| + eps)
    g = rng.normal(size=p0.shape)
    p, m, v = p0.copy(), np.zeros_like(p0), np.zeros_like(p0)
    adam_step(p, g, m, v, 1, 0.5, 0.9, 0.999, 1e-8)
    np.testing.assert_allclose(p, p0 - 0.5 * g / (np.abs(g) + 1e-8), atol=1e-13)
    # a constant gradient keeps m_hat = g and v_hat = g^2 at every step: T steps move by T * lr * sign(g)
    p, m, v = p0.copy(), np.zeros_like(p0), np.zeros_like(p0)
    for t in range(1, 21):
        adam_step(p, g, m, v, t, 0.01, 0.9, 0.999, 0.0)
    np.testing.assert_allclose(p, p0 - 20 * 0.01 * np.sign(g), atol=1e-12)


def test_adam_two_steps_by_hand():
    # beta1 = beta2 = 1/2, g1 = 1, g2 = 3, eps = 0, lr = 1, p0 = 0 (worked out in the fixture's header)
    vals = [float(x) for x in open(os.path.join(GOLDEN, "adam_two_steps.txt")).read().split("\n") if x and not x.startswith("#")]
    p, m, v = np.zeros(1), np.zeros(1), np.zeros(1)
    adam_step(p, np.array([1.0]), m, v, 1, 1.0, 0.5, 0.5, 0.0)
    assert abs(p[0] - vals[0]) < 1e-15
    adam_step(p, np.array([3.0]), m, v, 2, 1.0, 0.5, 0.5, 0.0)
    assert abs(m[0] - vals[1]) < 1e-15 and abs(v[0] - vals[2]) < 1e-15
    assert abs(p[0] - vals[3]) < 1e-12


def test_sgd_against_library():
    rng = np.random.default_rng(4)
    p0 = rng.normal(size=(4, 3))
    for wd in (0.0, 0.1):
        p = p0.copy()
        pt = torch.tensor(p0, dtype=torch.float64, requires_grad=True)
        opt = torch.optim.SGD([pt], lr=0.05, weight_decay=wd)
        for _ in range(4):
            g = rng.normal(size=p0.shape)
            sgd_step(p, g, 0.05, wd)
            pt.grad = torch.tensor(g)
            opt.step()
            np.testing.assert_allclose(p, pt.detach().numpy(), rtol=0, atol=1e-14)


def test_bf16_round_against_library():
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.normal(size=4000) * 10.0 ** rng.integers(-6, 6, size=4000),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38]]).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(bf16_round(x).view(np.uint32), want.view(np.uint32))


# ---------------------------------------------------------------- the whole loop (Algorithm 1 around the stage)
def test_gradients_of_the_whole_chunked_model_by_finite_differences():
    """L = mean cross-entropy of the chunked forward pass with the history held constant; every weight,
    bias and head gradient of one epoch must be its derivative."""
    tp = make_train_problem(n=60, n_classes=3, stage_dims=((6, 5), (5, 4, 4)), K=3, deg_in=4.0, deg_out=1.0, signal=1.0)
    rng = np.random.default_rng(6)

    def fresh():
        tr = new_oracle_trainer(tp, f64=True, optimizer="sgd", lr=0.0, shuffle=True, seed=9, alpha_hist=10**9)
        for st in tr.stages:  # arbitrary non-trivial history, and biases away from zero
            for j in range(st.L):
                if not (st is tr.stages[0] and j == 0):
                    st.hist[j][...] = np.random.default_rng(100 + j).normal(size=st.hist[j].shape) * 0.5
        return tr

    def set_params(tr, params):
        for x, p in zip(tr.master, params):
            x[...] = p
        tr._publish()

    base = fresh()
    params = [x + 0.3 * rng.normal(size=x.shape) for x in base.master]
    set_params(base, params)
    base.epoch(0)
    grads = [np.array(g, dtype=np.float64) for g in base.grads()]
    assert any(np.abs(g).max() > 1e-4 for g in grads)
    h = 1e-6
    checked = 0
    for pi, p in enumerate(params):
        flat_idx = rng.choice(p.size, size=min(4, p.size), replace=False)
        for fi in flat_idx:
            vals = []
            for sgn in (+1, -1):
                tr = fresh()
                q = [x.copy() for x in params]
                q[pi].reshape(-1)[fi] += sgn * h
                set_params(tr, q)
                vals.append(tr.epoch(0))
            fd = (vals[0] - vals[1]) / (2 * h)
            an = grads[pi].reshape(-1)[fi]
            assert abs(fd - an) < 1e-6 * max(1.0, abs(an)) + 2e-8, (pi, fi, fd, an)
            checked += 1
    assert checked >= 20


def test_splitting_the_layers_into_stages_changes_nothing():
    """Stages are a placement of consecutive layers; run back to back on one device, 1 x 4 layers,
    2 x 2 layers and 1 + 3 layers are the same computation."""
    results = []
    for split in (((12, 10, 8, 8, 6),), ((12, 10, 8), (8, 8, 6)), ((12, 10), (10, 8, 8, 6))):
        tp = make_train_problem(n=300, n_classes=4, stage_dims=split, K=4, ragged=True)
        # same weights whatever the split: generated per stage, so copy them from the flat model
        flat = make_train_problem(n=300, n_classes=4, stage_dims=((12, 10, 8, 8, 6),), K=4, ragged=True)
        j = 0
        for si, dims in enumerate(split):
            for l in range(len(dims) - 1):
                tp.W[si][l] = flat.W[0][j]
                j += 1
        tr = new_oracle_trainer(tp, optimizer="adam", lr=0.01, shuffle=True, seed=4, alpha_hist=2)
        losses = [tr.epoch(e) for e in range(5)]
        results.append((losses, [x.copy() for x in tr.master if x.ndim == 2]))
    for losses, weights in results[1:]:
        assert losses == results[0][0]
        for a, b in zip(weights, results[0][1]):
            assert np.array_equal(a, b)


def test_one_chunk_is_full_graph_training():
    """K = 1 never reads history, so the loop is ordinary full-graph training: compare with autograd on
    dense matrices."""
    tp = make_train_problem(n=40, n_classes=3, stage_dims=((5, 4, 4),), K=1, deg_in=3.0, deg_out=1.0, label_rate=0.7)
    tr = new_oracle_trainer(tp, f64=True, optimizer="sgd", lr=0.1, shuffle=False)
    n = tp.n
    A = np.zeros((n, n))
    import oracle
    val = oracle.gcn_norm(tp.row_ptr, tp.col, f64=True)
    for v in range(n):
        A[v, tp.col[tp.row_ptr[v]:tp.row_ptr[v + 1]]] = val[tp.row_ptr[v]:tp.row_ptr[v + 1]]
    At = torch.tensor(A)
    Ws = [torch.tensor(np.array(w, dtype=np.float64), requires_grad=True) for w in tp.W[0]]
    bs = [torch.tensor(np.array(b, dtype=np.float64), requires_grad=True) for b in tp.b[0]]
    Wo = torch.tensor(np.array(tp.head_W, dtype=np.float64), requires_grad=True)
    bo = torch.tensor(np.array(tp.head_b, dtype=np.float64), requires_grad=True)
    mask = torch.tensor(tp.mask.astype(bool))
    y = torch.tensor(tp.labels.astype(np.int64))
    for step in range(3):
        h = torch.tensor(tp.x0.astype(np.float64))
        for W, b in zip(Ws, bs):
            h = torch.relu(At @ h @ W + b)
        loss = torch.nn.functional.cross_entropy((h @ Wo + bo)[mask], y[mask])
        for t in Ws + bs + [Wo, bo]:
            t.grad = None
        loss.backward()
        got = tr.epoch(step)
        assert abs(got - loss.item()) < 1e-12
        with torch.no_grad():
            for t in Ws + bs + [Wo, bo]:
                t -= 0.1 * t.grad
    for x, t in zip(tr.master, Ws + bs + [Wo, bo]):
        np.testing.assert_allclose(x, t.detach().numpy(), atol=1e-12)


def test_history_is_refreshed_every_alpha_epochs():
    """Section 3.4, technique 2: epochs 1..alpha read the initial history, alpha+1..2 alpha that of epoch alpha."""
    tp = make_train_problem(n=200, n_classes=3, stage_dims=((8, 6, 6),), K=4)
    tr = new_oracle_trainer(tp, optimizer="adam", lr=0.01, shuffle=True, seed=1, alpha_hist=3)
    st = tr.stages[0]
    snaps = []
    for e in range(7):
        before = st.hist[1].copy()
        tr.epoch(e)
        refreshed = (e + 1) % 3 == 0
        if refreshed:
            assert np.array_equal(st.hist[1], st.cur[1]) and not np.array_equal(st.hist[1], before)
        else:
            assert np.array_equal(st.hist[1], before)
        snaps.append(refreshed)
    assert snaps == [False, False, True, False, False, True, False]
    assert np.array_equal(st.hist[0], tp.x0)  # features never change


def test_training_reduces_the_loss_on_the_planted_task():
    tp = make_train_problem(n=1500, n_classes=5, stage_dims=((24, 16), (16, 16)), K=4)
    tr = new_oracle_trainer(tp, optimizer="adam", lr=0.01, shuffle=True, seed=3, alpha_hist=2)
    losses = [tr.epoch(e) for e in range(30)]
    assert abs(losses[0] - math.log(5)) < 0.3           # starts near the uniform prediction
    assert losses[-1] < 0.2 * losses[0]
    test = ~tp.mask.astype(bool)
    assert (tr.predict()[test] == tp.labels[test]).mean() > 0.9
