"""GPU parity of the training loop (include/gnntrain.h) against oracle/train.py: the steps one by one
(softmax cross-entropy, fixed-order sum, SGD and Adam steps), then whole epochs through the C ABI."""
from __future__ import annotations

import numpy as np
import pytest
import torch

from helpers import make_train_problem, max_rel, new_oracle_trainer
from oracle.train import adam_step, bf16_round, sgd_step, softmax_xent

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
TOL_F32 = 1e-5   # fp32 path: max |x - ref| / max |ref| per tensor
TOL_BF16 = 1e-2  # bf16 path


def _g():
    import paper_2308_10087_amd as g
    return g


def F(x):
    """The C ABI takes its hyper-parameters as floats: hand the oracle the value that actually arrives."""
    return float(np.float32(x))


@pytest.mark.parametrize("rows,C", [(1, 1), (1, 2), (7, 5), (1000, 41), (333, 64), (130, 100), (65, 257)])
@pytest.mark.parametrize("dl_dtype", ["f32", "bf16"])
@pytest.mark.parametrize("masked", [False, True])
def test_softmax_xent_kernel(rows, C, dl_dtype, masked):
    g = _g()
    rng = np.random.default_rng(rows * 1000 + C)
    ld = (C + 7) // 8 * 8
    z = (rng.normal(size=(rows, ld)) * 4).astype(np.float32)
    bias = (rng.normal(size=C)).astype(np.float32)
    y = rng.integers(0, C, size=rows).astype(np.int32)
    mask = (rng.random(rows) < 0.6).astype(np.uint8) if masked else None
    if masked and mask.sum() == 0:
        mask[0] = 1
    n_train = int(mask.sum()) if masked else rows
    loss_ref, g_ref = softmax_xent(z[:, :C].astype(np.float64) + bias, y, mask, n_train)
    zt = torch.from_numpy(z).to(DEV)
    dt = torch.bfloat16 if dl_dtype == "bf16" else torch.float32
    dl = torch.full((rows, ld), 7.0, dtype=dt, device=DEV)
    row_loss = torch.full((rows,), -1.0, device=DEV)
    g.gnntrain_softmax_xent(zt, torch.from_numpy(bias).to(DEV), torch.from_numpy(y).to(DEV),
                            None if mask is None else torch.from_numpy(mask).to(DEV), C, 1.0 / n_train, dl, row_loss)
    scratch, out = torch.zeros(1024, device=DEV), torch.zeros(1, device=DEV)
    g.gnntrain_sum(row_loss, 1.0 / n_train, scratch, out)
    torch.cuda.synchronize()
    got = dl.to(torch.float32).cpu().numpy()
    assert np.all(got[:, C:] == 0)                       # padding columns are written as zeros
    if masked:
        assert np.all(got[mask == 0] == 0)
    if C == 1:
        assert np.all(got == 0) and abs(out.item()) < 1e-7   # one class: nothing to learn
    else:
        assert max_rel(got[:, :C], g_ref) <= (TOL_BF16 if dl_dtype == "bf16" else TOL_F32)
        assert abs(out.item() - loss_ref) <= TOL_F32 * max(1.0, abs(loss_ref))


def test_softmax_xent_handles_no_rows_and_extreme_logits():
    g = _g()
    empty = torch.zeros((0, 8), device=DEV)
    g.gnntrain_softmax_xent(empty, None, torch.zeros(0, dtype=torch.int32, device=DEV), None, 5, 1.0, empty.clone(),
                            torch.zeros(0, device=DEV))
    z = np.array([[1e4, -1e4, 0, 0, 0, 0, 0, 0], [-80, -80, -80, 0, 0, 0, 0, 0]], np.float32)
    y = np.array([1, 2], np.int32)
    dl, rl = torch.zeros((2, 8), device=DEV), torch.zeros(2, device=DEV)
    g.gnntrain_softmax_xent(torch.from_numpy(z).to(DEV), None, torch.from_numpy(y).to(DEV), None, 3, 0.5, dl, rl)
    torch.cuda.synchronize()
    loss_ref, g_ref = softmax_xent(z[:, :3].astype(np.float64), y, None, 2)
    assert torch.isfinite(dl).all() and torch.isfinite(rl).all()
    assert max_rel(dl.cpu().numpy()[:, :3], g_ref) <= TOL_F32
    assert abs(rl.sum().item() / 2 - loss_ref) <= TOL_F32 * loss_ref


@pytest.mark.parametrize("n", [0, 1, 255, 4097, 1_000_003])
def test_fixed_order_sum(n):
    g = _g()
    rng = np.random.default_rng(n)
    x = rng.normal(size=n).astype(np.float32) + 0.5
    xt = torch.from_numpy(x).to(DEV)
    scratch, out = torch.zeros(1024, device=DEV), torch.full((1,), 3.0, device=DEV)
    g.gnntrain_sum(xt, 0.25, scratch, out)
    first = out.item()
    g.gnntrain_sum(xt, 0.25, scratch, out)
    torch.cuda.synchronize()
    assert out.item() == first                          # reproducible
    ref = 0.25 * x.astype(np.float64).sum()
    assert abs(first - ref) <= 1e-6 * max(1.0, np.abs(x).sum() * 0.25)


@pytest.mark.parametrize("count", [1, 1000, 70_001])
@pytest.mark.parametrize("opt", ["adam", "sgd"])
@pytest.mark.parametrize("compute", [None, "bf16", "f32"])
def test_optimizer_step_kernels(count, opt, compute):
    g = _g()
    rng = np.random.default_rng(count)
    p = rng.normal(size=count).astype(np.float32)
    gr = (rng.normal(size=count) * 10.0 ** rng.integers(-4, 2, size=count)).astype(np.float32)
    m = (rng.normal(size=count) * 0.1).astype(np.float32)
    v = (rng.random(size=count) * 0.01).astype(np.float32)
    for t, wd in ((1, 0.0), (7, 0.01), (1000, 0.0)):
        pt, gt, mt, vt = (torch.from_numpy(a.copy()).to(DEV) for a in (p, gr, m, v))
        ct = None if compute is None else torch.zeros(count, dtype=torch.bfloat16 if compute == "bf16" else torch.float32, device=DEV)
        pr, mr, vr = p.astype(np.float64), m.astype(np.float64), v.astype(np.float64)
        if opt == "adam":
            g.gnntrain_adam_step(pt, gt, mt, vt, ct, 0.01, 0.9, 0.999, 1e-8, wd, t)
            adam_step(pr, gr.astype(np.float64), mr, vr, t, F(0.01), F(0.9), F(0.999), F(1e-8), F(wd))
        else:
            g.gnntrain_sgd_step(pt, gt, ct, 0.01, wd)
            sgd_step(pr, gr.astype(np.float64), F(0.01), F(wd))
        torch.cuda.synchronize()
        assert max_rel(pt.cpu().numpy(), pr) <= 1e-6
        if opt == "adam":
            assert max_rel(mt.cpu().numpy(), mr) <= 1e-6 and max_rel(vt.cpu().numpy(), vr) <= 1e-6
        if ct is not None:  # the copy the kernels read is the rounding of the new master value
            want = pt.to(ct.dtype)
            assert torch.equal(ct, want)
            if compute == "bf16":
                assert np.array_equal(ct.to(torch.float32).cpu().numpy(), bf16_round(pt.cpu().numpy()))


def _run_pair(tp, epochs, **opt):
    from gpu_harness import GpuTrainRun
    ref = new_oracle_trainer(tp, **{k: (F(v) if isinstance(v, float) else v) for k, v in opt.items()})
    run = GpuTrainRun(tp, **opt)
    out = []
    for e in range(epochs):
        lr_ = ref.epoch(e)
        lg = run.epoch(e)
        assert np.array_equal(run.trainer.gnntrain_last_order(), ref.last_order)
        out.append((lg, lr_))
    return ref, run, out


@pytest.mark.parametrize("stage_dims", [((24, 16, 16),), ((24, 16), (16, 16, 12)), ((20, 24, 9), (9, 17), (17, 8))])
@pytest.mark.parametrize("ragged", [False, True])
def test_one_sgd_epoch_fp32(stage_dims, ragged):
    """Loss, every gradient and every updated parameter of one epoch against the oracle."""
    tp = make_train_problem(n=1500, n_classes=5, stage_dims=stage_dims, K=4, ragged=ragged)
    ref, run, out = _run_pair(tp, 1, optimizer="sgd", lr=0.05, shuffle=True, seed=7, alpha_hist=1)
    lg, lr_ = out[0]
    assert abs(lg - lr_) <= TOL_F32 * lr_
    for a, b in zip(run.grads(), ref.grads()):
        assert max_rel(a.reshape(b.shape), b) <= TOL_F32
    for a, b in zip(run.master_values(), ref.master):
        assert max_rel(a.reshape(b.shape), b) <= TOL_F32
    # history was refreshed (alpha = 1): every historical level equals the current one
    for st_cur, st_hist in zip(run.cur, run.hist):
        for j in range(len(st_hist)):
            assert torch.equal(st_hist[j], st_cur[j])


@pytest.mark.parametrize("variants,stage_dims", [(("sage",), ((24, 16, 16),)), (("resgcn",), ((16, 16, 16),)),
                                                 (("sage", "resgcn", "gcn"), ((24, 16), (16, 16, 16), (16, 8)))])
def test_one_sgd_epoch_fp32_other_layer_types(variants, stage_dims):
    """The loop is generic over the stages' layer types: GraphSage, ResGCN+ (LayerNorm parameters are
    trained too) and a mix of all three in one model."""
    tp = make_train_problem(n=1500, n_classes=5, stage_dims=stage_dims, K=4, ragged=True, variants=variants)
    ref, run, out = _run_pair(tp, 3, optimizer="sgd", lr=0.05, shuffle=True, seed=11, alpha_hist=2)
    for lg, lr_ in out:
        assert abs(lg - lr_) <= 1e-4 * lr_
    for a, b in zip(run.grads(), ref.grads()):
        assert max_rel(a.reshape(b.shape), b) <= 1e-4
    for a, b in zip(run.master_values(), ref.master):
        assert max_rel(a.reshape(b.shape), b) <= 1e-4
    assert out[-1][0] < out[0][0]


def test_sgd_epochs_with_empty_chunks_and_shuffling():
    """Chunks without vertices take part in the shuffled order like any other.  With seed 5 an empty chunk
    comes first in the forward order of epochs 0 to 3, i.e. last in their backward pass, where the stage still
    owes the history-side weight gradient of its transform-first layer (24 -> 8)."""
    tp = make_train_problem(n=1500, n_classes=5, stage_dims=((24, 8, 16),), K=5)
    tp.chunk_ptr = np.array([0, 0, 400, 400, 900, 1500], dtype=np.int64)
    from gpu_harness import GpuTrainRun
    opt = dict(optimizer="sgd", lr=0.05, shuffle=True, seed=5, alpha_hist=1)
    ref = new_oracle_trainer(tp, **{k: (F(v) if isinstance(v, float) else v) for k, v in opt.items()})
    run = GpuTrainRun(tp, **opt)
    assert run.stages[0].gnnstage_layer_order(0) == 1
    firsts = []
    for e in range(4):
        lr_, lg = ref.epoch(e), run.epoch(e)
        assert np.array_equal(run.trainer.gnntrain_last_order(), ref.last_order)
        firsts.append(int(ref.last_order[0]))
        assert abs(lg - lr_) <= 1e-4 * lr_
        for a, b in zip(run.grads(), ref.grads()):
            assert max_rel(a.reshape(b.shape), b) <= 1e-4, e
    assert set(firsts) <= {0, 2}, firsts


def test_sgd_epochs_with_dropout_in_the_resgcn_stage():
    """A fresh set of dropout decisions every epoch, the same on both sides."""
    tp = make_train_problem(n=1500, n_classes=5, stage_dims=((24, 16), (16, 16, 16), (16, 8)), K=4, ragged=True,
                            variants=("sage", "resgcn", "gcn"))
    tp.dropout_p = 0.5
    ref, run, out = _run_pair(tp, 3, optimizer="sgd", lr=0.05, shuffle=True, seed=11, alpha_hist=2)
    for lg, lr_ in out:
        assert abs(lg - lr_) <= 1e-4 * lr_
    for a, b in zip(run.grads(), ref.grads()):
        assert max_rel(a.reshape(b.shape), b) <= 1e-4
    nodrop = make_train_problem(n=1500, n_classes=5, stage_dims=((24, 16), (16, 16, 16), (16, 8)), K=4, ragged=True,
                                variants=("sage", "resgcn", "gcn"))
    ref0 = new_oracle_trainer(nodrop, optimizer="sgd", lr=F(0.05), shuffle=True, seed=11, alpha_hist=2)
    assert abs(ref0.epoch(0) - out[0][1]) > 1e-3       # dropout really changed the pass


def test_sgd_epochs_with_dropout_in_every_stage_but_the_last():
    """GCN and GraphSage stages drop on their layers' outputs, the ResGCN+ stage inside its block; the last stage feeds
    the loss head and is created without dropout."""
    tp = make_train_problem(n=1500, n_classes=5, stage_dims=((24, 16, 16), (16, 16, 16), (16, 16), (16, 8)), K=4, ragged=True,
                            variants=("sage", "resgcn", "gcn", "gcn"))
    tp.dropout_p = 0.5
    tp.dropout_everywhere = True
    assert [tp.stage_dropout(si) for si in range(4)] == [0.5, 0.5, 0.5, 0.0]
    ref, run, out = _run_pair(tp, 3, optimizer="sgd", lr=0.05, shuffle=True, seed=13, alpha_hist=2)
    for lg, lr_ in out:
        assert abs(lg - lr_) <= 1e-4 * lr_
    for a, b in zip(run.grads(), ref.grads()):
        assert max_rel(a.reshape(b.shape), b) <= 1e-4
    only_res = make_train_problem(n=1500, n_classes=5, stage_dims=((24, 16, 16), (16, 16, 16), (16, 16), (16, 8)), K=4,
                                  ragged=True, variants=("sage", "resgcn", "gcn", "gcn"))
    only_res.dropout_p = 0.5
    ref0 = new_oracle_trainer(only_res, optimizer="sgd", lr=F(0.05), shuffle=True, seed=13, alpha_hist=2)
    assert abs(ref0.epoch(0) - out[0][1]) > 1e-3       # the other stages' dropout really changed the pass


@pytest.mark.parametrize("stage_dims", [((24, 16, 16),), ((24, 16), (16, 16, 8))])
def test_one_sgd_epoch_bf16(stage_dims):
    """bf16 levels: the oracle rounds at the same points.  A pre-activation that sits within rounding noise of
    zero may still fall on different sides of the ReLU in the two runs (there is no teacher forcing inside an
    epoch), which moves sums with heavy cancellation (bias gradients) by more than 1e-2 of their own size.
    The bound therefore adds the tensor's own bf16 noise floor: the distance between the oracle with and
    without bf16 rounding."""
    import dataclasses
    tp = make_train_problem(n=1500, n_classes=5, stage_dims=stage_dims, K=4, dtype="bf16")
    opt = dict(optimizer="sgd", lr=0.05, shuffle=True, seed=7, alpha_hist=1)
    ref, run, out = _run_pair(tp, 1, **opt)
    exact = new_oracle_trainer(dataclasses.replace(tp, quant=False), **{k: (F(v) if isinstance(v, float) else v) for k, v in opt.items()})
    exact.epoch(0)
    lg, lr_ = out[0]
    assert abs(lg - lr_) <= TOL_BF16 * lr_
    worst = 0.0
    for a, b, c in zip(run.grads(), ref.grads(), exact.grads()):
        floor = float(np.abs(np.asarray(b, np.float64) - np.asarray(c, np.float64)).max())
        err = float(np.abs(a.reshape(b.shape).astype(np.float64) - b).max())
        assert err <= TOL_BF16 * float(np.abs(b).max()) + floor
        worst = max(worst, max_rel(a.reshape(b.shape), b))
    assert worst <= 5 * TOL_BF16
    for a, b, c in zip(run.master_values(), ref.master, exact.master):
        floor = float(np.abs(b - c).max())
        assert float(np.abs(a.reshape(b.shape).astype(np.float64) - b).max()) <= TOL_BF16 * float(np.abs(b).max()) + floor
    # the stages read the bf16 rounding of the fp32 master weights
    for master, compute, _ in run.params:
        if compute is not None:
            assert torch.equal(compute, master.to(torch.bfloat16))
    # ReLU decisions of the two runs differ only in a sliver of the entries
    for si, st in enumerate(ref.stages):
        for j in range(1, st.L + 1):
            gpu_on = run.cur[si][j].to(torch.float32).cpu().numpy() > 0
            assert np.mean(gpu_on != (st.cur[j] > 0)) < 2e-3


def test_adam_epochs_track_the_oracle_and_learn_fp32():
    tp = make_train_problem(n=1500, n_classes=5, stage_dims=((24, 16), (16, 16)), K=4)
    ref, run, out = _run_pair(tp, 12, optimizer="adam", lr=0.01, shuffle=True, seed=3, alpha_hist=2)
    l0 = out[0][1]
    for e, (lg, lr_) in enumerate(out):
        assert abs(lg - lr_) <= 2e-3 * l0, (e, lg, lr_)
    assert out[-1][0] < 0.7 * out[0][0]
    # history refresh period 2: after 12 epochs the buffers hold the levels of epoch 12
    assert torch.equal(run.hist[1][0], run.cur[1][0])
    ref.epoch(12)
    run.epoch(12)
    assert not torch.equal(run.hist[1][0], run.cur[1][0])   # epoch 13 does not refresh


def test_adam_epochs_learn_bf16():
    tp = make_train_problem(n=1500, n_classes=5, stage_dims=((24, 16), (16, 16)), K=4, dtype="bf16")
    ref, run, out = _run_pair(tp, 12, optimizer="adam", lr=0.01, shuffle=True, seed=3, alpha_hist=2)
    l0 = out[0][1]
    for e, (lg, lr_) in enumerate(out):
        assert abs(lg - lr_) <= 5e-2 * l0, (e, lg, lr_)
    assert out[-1][0] < 0.7 * out[0][0]


@pytest.mark.parametrize("dtype,alpha,variants", [("f32", 1, ("sage", "resgcn", "gcn")), ("f32", 2, None), ("bf16", 1, None)])
def test_epochs_with_the_history_refreshed_by_trading_buffers(dtype, alpha, variants):
    """history_swap: the loop refreshes with gnnstage_update_history_swap.  The historical levels hold the same
    values as after a copy, so losses and parameters are bit-identical to a run that copies, epoch after epoch."""
    from gpu_harness import GpuTrainRun
    dims = ((24, 16, 16), (16, 16, 16), (16, 16, 12)) if variants else ((24, 16, 16), (16, 16, 12))
    tp = make_train_problem(n=1200, n_classes=5, stage_dims=dims, K=4, dtype=dtype, ragged=True, variants=variants)
    a = GpuTrainRun(tp, optimizer="adam", lr=0.01, shuffle=True, seed=5, alpha_hist=alpha)
    b = GpuTrainRun(tp, optimizer="adam", lr=0.01, shuffle=True, seed=5, alpha_hist=alpha, history_swap=True)
    for e in range(6):
        la, lb = a.epoch(e), b.epoch(e)
        assert la == lb, (e, la, lb)
    for x, y in zip(a.master_values(), b.master_values()):
        assert np.array_equal(x, y)
    traded = False
    for sa, sb in zip(a.stages, b.stages):
        for j in range(sa.L):
            assert sb.gnnstage_level_buffers(j) == (sb.cur[j].data_ptr(), sb.hist[j].data_ptr())
            assert torch.equal(sa.hist[j], sb.hist[j]), j       # epoch 6 refreshed (alpha 1 or 2)
        traded = traded or any(sb.cur[j].data_ptr() != b.cur[b.stages.index(sb)][j].data_ptr() for j in range(1, sb.L))
    assert traded == (6 // alpha % 2 == 1)   # an odd number of trades leaves the buffers in the other places


def test_splitting_layers_into_stages_changes_nothing_on_the_gpu():
    from gpu_harness import GpuTrainRun
    losses = []
    flat = make_train_problem(n=900, n_classes=4, stage_dims=((12, 10, 8, 8, 6),), K=4, ragged=True)
    for split in (((12, 10, 8, 8, 6),), ((12, 10, 8), (8, 8, 6)), ((12, 10), (10, 8, 8, 6))):
        tp = make_train_problem(n=900, n_classes=4, stage_dims=split, K=4, ragged=True)
        j = 0
        for si, dims in enumerate(split):
            for l in range(len(dims) - 1):
                tp.W[si][l] = flat.W[0][j]
                j += 1
        run = GpuTrainRun(tp, optimizer="adam", lr=0.01, shuffle=True, seed=4, alpha_hist=2)
        losses.append([run.epoch(e) for e in range(4)])
    for other in losses[1:]:
        for a, b in zip(other, losses[0]):
            assert abs(a - b) <= TOL_F32 * abs(b)


def test_create_rejects_bad_descriptors():
    from gpu_harness import GpuTrainRun
    g = _g()
    tp = make_train_problem(n=300, n_classes=4, stage_dims=((8, 6), (6, 6)), K=3)
    with pytest.raises(g.GnnStageError) as e:
        GpuTrainRun(tp, chain=False)        # level 0 of stage 2 is not the last level of stage 1
    assert e.value.code == -1
    bad = make_train_problem(n=300, n_classes=4, stage_dims=((8, 6),), K=3)
    bad.labels = bad.labels.copy()
    bad.labels[17] = 4                      # outside [0, n_classes)
    with pytest.raises(g.GnnStageError) as e:
        GpuTrainRun(bad)
    assert e.value.code == -1
    with pytest.raises(g.GnnStageError):
        GpuTrainRun(make_train_problem(n=300, n_classes=4, stage_dims=((8, 6),), K=3), alpha_hist=0)
