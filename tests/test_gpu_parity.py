"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element,
on the same seeded inputs.  Tolerances (per tensor, max|x - ref| / max|ref|):
1e-5 for the fp32 stage, 1e-2 for the bf16 / matrix-core stage; integer bookkeeping bit-exact."""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from synth import graphs, values
from synth.configs import CONFIGS, Workload

from helpers import make_problem, max_rel, run_oracle

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-5
TOL_BF16 = 1e-2


# Share of a level's elements whose ReLU decision may differ between the two sides (each of them a near-tie, see
# _check_forward).  How many elements sit that close to zero is a property of the data, not of either side's
# arithmetic.  Measured over this file: at most 9.3e-4 (and 7 of 4,800 elements = 1.5e-3 in one 600-vertex case);
# at full size 7.8e-4 on configs[2] and 1.5e-5 on configs[4].
FLIP_SHARE = 2e-3


def _note_flip_share(level, share, count, size):
    """One line per level with differing ReLU decisions into the run's output folder (what the bound above is judged by)."""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    try:
        os.makedirs(os.path.join(root, "gpurun_out"), exist_ok=True)
        with open(os.path.join(root, "gpurun_out", "flip_shares.log"), "a") as f:
            f.write(f"{share:.3e} {count} of {size} level {level} {os.environ.get('PYTEST_CURRENT_TEST', '')}\n")
    except OSError:
        pass


def _gpu(p, **kw):
    from gpu_harness import GpuRun
    return GpuRun(p, **kw)


def _check_forward(run, ref, p, tol):
    """Levels within tolerance; ReLU on/off decisions may differ only at near-ties: the side that is
    non-zero holds a value no larger than the tolerance itself (tol * max).  How many elements sit that
    close to zero is a property of the data; the share of such elements is bounded by FLIP_SHARE (measured
    values beside its definition)."""
    worst = {}
    for j in range(1, p.L + 1):
        a, b = run.np(run.cur[j]), ref.cur[j]
        worst[f"level{j}"] = max_rel(a, b)
        flips = (a > 0) != (b > 0)
        if flips.any():
            _note_flip_share(j, float(flips.mean()), int(flips.sum()), a.size)
            assert flips.mean() <= FLIP_SHARE, (j, flips.sum())
            assert np.maximum(np.abs(a[flips]), np.abs(b[flips])).max() <= tol * np.abs(b).max(), j
    bad = {k: v for k, v in worst.items() if not (v <= tol)}
    assert not bad, f"over tolerance {tol}: {bad} (all: {worst})"


def _parity(p, tol, need_input_grad=True, **kw):
    """Forward parity, then backward parity with both sides deciding every ReLU derivative on the
    SAME level values: the oracle's levels are written into the GPU's caller-owned level buffers
    before the backward pass (a single near-tie flip of a mask bit moves one weight-gradient entry by
    several percent on graphs this small, which is not an arithmetic error of either side)."""
    ref = run_oracle(p, need_input_grad=need_input_grad)
    run = _gpu(p, need_input_grad=need_input_grad, **kw)
    run.forward()
    torch.cuda.synchronize()
    _check_forward(run, ref, p, tol)
    for j in range(1, p.L + 1):
        run.cur[j].copy_(torch.from_numpy(ref.cur[j]).to(run.cur[j].dtype))
    run.backward()
    torch.cuda.synchronize()
    return _compare(run, ref, p, tol, need_input_grad)


def _compare(run, ref, p, tol, need_input_grad=True):
    worst = {}
    for j in range(1, p.L + 1):
        worst[f"level{j}"] = max_rel(run.np(run.cur[j]), ref.cur[j])
    for j in range(p.L):
        worst[f"dW{j}"] = max_rel(run.np(run.dW[j]), ref.dW[j])
        if p.w.variant in ("gcn", "sage", "resgcn"):
            worst[f"db{j}"] = max_rel(run.np(run.dbias[j]), ref.db[j])
        if p.w.variant == "resgcn":
            worst[f"dgamma{j}"] = max_rel(run.np(run.d_ln_gamma[j]), ref.d_ln_g[j])
            worst[f"dbeta{j}"] = max_rel(run.np(run.d_ln_beta[j]), ref.d_ln_b[j])
    if need_input_grad:
        worst["grad_in"] = max_rel(run.np(run.grad_in), ref.grad_in)
    if p.w.variant == "gcnii":
        worst["grad_h0"] = max_rel(run.np(run.grad_h0), ref.dH0)
    bad = {k: v for k, v in worst.items() if not (v <= tol)}
    assert not bad, f"over tolerance {tol}: {bad} (all: {worst})"
    return worst


@pytest.mark.parametrize("name", ["c1_s", "c2_s", "c3_s", "c4_s"])
def test_bf16_backward_on_the_gpus_own_levels(name):
    """The one comparison in which nothing is forced: the GPU's backward pass runs on the levels and saved
    aggregations of its OWN forward pass, and every gradient is compared with the oracle's own pass.

    Beyond the arithmetic of the two sides (1e-2, as everywhere) the two passes now differ in ReLU decisions:
    where a pre-activation lies within rounding distance of zero (|y| <= 1e-2 max|y|, checked by the forward
    comparison) one side passes the upstream gradient of that element and the other replaces it by zero.  If a
    share s of a layer's elements is decided differently, dY of that layer differs by about sqrt(s) of its
    Frobenius norm; everything below that layer is linear in dY once the masks are fixed, so the relative errors
    of the L layers add at most.  Hence the bound on the relative Frobenius error of every gradient:
        1e-2 + L * sqrt(s),   s = largest share of differing decisions over the levels (measured in the test).
    Measured (error / bound): c1_s 0.083 / 0.116, c2_s 0.176 / 0.233, c3_s 0.0037 / 0.045, c4_s 0.013 / 0.039.
    The max-norm used elsewhere is not bounded here: one flipped element moves single gradient rows by their
    full size (c3_s: about 100 flipped elements in 2 * 10^7 put max|x - ref| / max|ref| of grad_in at 0.24)."""
    p = make_problem(CONFIGS[name], bias_std=0.05)
    ref = run_oracle(p)
    run = _gpu(p)
    run.forward()
    torch.cuda.synchronize()
    _check_forward(run, ref, p, TOL_BF16)
    share = max(float(((run.np(run.cur[j]) > 0) != (ref.cur[j] > 0)).mean()) for j in range(1, p.L + 1))
    assert share <= 2e-3, share
    run.backward()
    torch.cuda.synchronize()
    def fro(x, r):
        r = np.asarray(r, dtype=np.float64)
        return float(np.linalg.norm(np.asarray(x, dtype=np.float64) - r) / max(np.linalg.norm(r), 1e-300))

    worst = {}
    for j in range(p.L):
        worst[f"dW{j}"] = fro(run.np(run.dW[j]), ref.dW[j])
        if p.w.variant == "gcn":
            worst[f"db{j}"] = fro(run.np(run.dbias[j]), ref.db[j])
    worst["grad_in"] = fro(run.np(run.grad_in), ref.grad_in)
    if p.w.variant == "gcnii":
        worst["grad_h0"] = fro(run.np(run.grad_h0), ref.dH0)
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    try:
        with open(os.path.join(root, "gpurun_out", "unforced.log"), "a") as f:
            f.write(f"{name} flip share {share:.2e} worst {max(worst.values()):.3e} {worst}\n")
    except OSError:
        pass
    bound = TOL_BF16 + p.L * math.sqrt(share)
    bad = {k: v for k, v in worst.items() if not (v <= bound)}
    assert not bad, f"over {bound}: {bad} (all: {worst})"


def small(n=700, k=5, dims=(24, 40, 16, 32), variant="gcn", dtype="f32", seed=5, deg=6.0, level0_f32=False):
    return Workload("small", "er", n, seed, list(dims), k, variant=variant, dtype=dtype, avg_degree=deg,
                    level0_f32=level0_f32, gcnii_first_layer=5)


# ----------------------------------------------------------------------------- fp32 stage
def test_c0_fp32_full_config():
    p = make_problem(CONFIGS["c0"], bias_std=0.0)
    _parity(p, TOL_F32)


@pytest.mark.parametrize("dims", [(24, 40, 16, 32), (100, 128, 128), (602, 64), (7, 5, 3), (64, 64, 64, 64, 64)])
def test_fp32_shapes_ragged_chunks_shuffled(dims):
    w = small(dims=dims, n=911, k=6)
    p = make_problem(w, chunk_ptr=graphs.ragged_chunks(911, 6, 4))
    _parity(p, TOL_F32)


def test_fp32_directed_graph_and_empty_chunks():
    rng = np.random.default_rng(8)
    n = 400
    dst = np.concatenate([rng.integers(0, n, 3000), np.arange(n)])
    src = np.concatenate([rng.integers(0, n, 3000), np.arange(n)])
    graph = graphs.from_directed_pairs(n, dst, src)
    w = small(n=n, k=5, dims=(16, 24, 8))
    chunk_ptr = np.array([0, 0, 150, 150, 151, n], dtype=np.int64)  # two empty chunks and a single-row chunk
    p = make_problem(w, graph=graph, chunk_ptr=chunk_ptr, first_stage=False)
    _parity(p, TOL_F32)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("empty_at", ["first", "last", "middle"])
def test_empty_chunk_at_either_end_of_the_order_with_a_transform_first_layer(dtype, empty_at):
    """The backward pass walks the forward order in reverse, so an empty chunk that is FIRST in the forward
    order is the last backward call - the call after which the history-side weight gradient of a
    transform-first layer (24 -> 8 narrows the gathered rows) is taken.  That work must run although the
    call itself has no rows."""
    n = 600
    w = small(n=n, k=5, dims=(24, 8, 16), dtype=dtype)
    chunk_ptr = np.array([0, 0, 200, 200, 420, n], dtype=np.int64)   # chunks 0 and 2 are empty
    order = {"first": [0, 3, 2, 1, 4], "last": [4, 1, 3, 0, 2], "middle": [1, 0, 4, 2, 3]}[empty_at]
    p = make_problem(w, chunk_ptr=chunk_ptr, order=order, first_stage=False)
    run = _gpu(p)
    assert run.stage.gnnstage_layer_order(0) == 1
    del run
    _parity(p, TOL_F32 if dtype == "f32" else TOL_BF16)


def test_fp32_long_rows_are_split(monkeypatch):
    monkeypatch.setenv("GNNSTAGE_SPLIT_EDGES", "64")
    w = CONFIGS["c2_s"]
    wf = Workload("c2_s_f32", "rmat", 3001, w.seed, [20, 24, 12], 4, n_candidates=60_000, rmat_abc=w.rmat_abc)
    p = make_problem(wf)
    assert np.diff(p.row_ptr).max() > 64 * 3
    _parity(p, TOL_F32)


def test_fp32_one_chunk_and_no_input_grad():
    w = small(k=1)
    p = make_problem(w)
    _parity(p, TOL_F32, need_input_grad=False)


def test_computed_normalisation_matches_given_bit_for_bit():
    p = make_problem(small())
    a = _gpu(p, edge_val="given").run()
    b = _gpu(p, edge_val="computed").run()
    for j in range(1, p.L + 1):
        assert torch.equal(a.cur[j], b.cur[j])
    assert torch.equal(a.grad_in, b.grad_in)


def test_two_runs_are_bit_identical():
    p = make_problem(CONFIGS["c3_s"])
    a = _gpu(p).run()
    b = _gpu(p).run()
    for j in range(1, p.L + 1):
        assert torch.equal(a.cur[j], b.cur[j])
    for j in range(p.L):
        assert torch.equal(a.dW[j], b.dW[j])
    assert torch.equal(a.grad_in, b.grad_in) and torch.equal(a.grad_h0, b.grad_h0)


# ----------------------------------------------------------------------------- bf16 stage
@pytest.mark.parametrize("name", ["c1_s", "c2_s", "c3_s", "c4_s"])
def test_bf16_shrunk_configs(name):
    p = make_problem(CONFIGS[name], bias_std=0.05)
    _parity(p, TOL_BF16)


@pytest.mark.parametrize("dims,variant", [((40, 72, 136), "gcn"), ((130, 258, 64), "gcn"), ((96, 96, 96), "gcnii")])
def test_bf16_odd_shapes(dims, variant):
    w = small(n=1300, k=4, dims=dims, variant=variant, dtype="bf16", deg=9.0)
    p = make_problem(w, chunk_ptr=graphs.ragged_chunks(1300, 4, 2))
    _parity(p, TOL_BF16)


@pytest.mark.parametrize("classes,min_row,split", [(8, 4, 64), (32, 16, 128), (5, 2, 4096), (1, 1, 64)])
@pytest.mark.parametrize("name", ["c2_s", "c3_s"])
def test_source_class_schedules(monkeypatch, classes, min_row, split, name):
    """The aggregation schedule cuts rows by source-id class and deals the classes to the XCDs at launch
    time (classes whose chunks are all unprocessed are skipped in the backward).  Force many classes,
    tiny rows into the class path and small pieces, with ragged chunks that straddle class boundaries."""
    monkeypatch.setenv("GNNSTAGE_XCD_CLASSES", str(classes))
    monkeypatch.setenv("GNNSTAGE_CLASS_MIN_ROW", str(min_row))
    monkeypatch.setenv("GNNSTAGE_SPLIT_EDGES", str(split))
    w = CONFIGS[name]
    row_ptr, col = __import__("synth").make_graph(w)
    n = len(row_ptr) - 1
    p = make_problem(w, graph=(row_ptr, col), chunk_ptr=graphs.ragged_chunks(n, w.n_chunks, 17), bias_std=0.05)
    _parity(p, TOL_BF16)


@pytest.mark.parametrize("weights", ["given", "computed"])
@pytest.mark.parametrize("classes,rows,min_row,split,dense", [(4, 32, 8, 64, False), (16, 8, 4, 128, False),
                                                              (32, 3, 2, 4096, False), (8, 24, 8, 64, True)])
@pytest.mark.parametrize("name", ["c2_s", "c4_s", "c3_s"])
def test_hotness_class_schedules(monkeypatch, classes, rows, min_row, split, dense, name, weights):
    """For tables beyond every cache the schedule cuts long rows by classes of the most often gathered sources
    (their entries re-ordered by hotness first) and runs a class's pieces together on one XCD.  Forced on the
    shrunk graphs with tiny classes, tiny rows cut, ragged chunks, forward and backward; with the caller's
    weights (which must follow their entries through the re-ordering) and with weights the library computes;
    also on top of dense blocks (the re-ordering then acts on what the dense plan leaves)."""
    monkeypatch.setenv("GNNSTAGE_HOT_CLASSES", str(classes))
    monkeypatch.setenv("GNNSTAGE_HOT_ROWS", str(rows))
    monkeypatch.setenv("GNNSTAGE_HOT_MIN_ROW", str(min_row))
    monkeypatch.setenv("GNNSTAGE_SPLIT_EDGES", str(split))
    if dense:
        monkeypatch.setenv("GNNSTAGE_DENSE_MIN_NNZ", "6")
        monkeypatch.setenv("GNNSTAGE_DENSE_MIN_SHARE", "0")
        monkeypatch.setenv("GNNSTAGE_DENSE_MIN_ENTRIES", "0")
    w = CONFIGS[name]
    row_ptr, col = __import__("synth").make_graph(w)
    n = len(row_ptr) - 1
    p = make_problem(w, graph=(row_ptr, col), chunk_ptr=graphs.ragged_chunks(n, w.n_chunks, 17), bias_std=0.05)
    _parity(p, TOL_BF16, edge_val=weights)


def test_hotness_class_schedule_fp32_probe(monkeypatch):
    """Exact-integer check of the hotness-class path: unit weights, ones, W = I - every level-1 value is a count
    of selected neighbours, every input gradient a count of processed readers."""
    monkeypatch.setenv("GNNSTAGE_HOT_CLASSES", "8")
    monkeypatch.setenv("GNNSTAGE_HOT_ROWS", "16")
    monkeypatch.setenv("GNNSTAGE_HOT_MIN_ROW", "4")
    monkeypatch.setenv("GNNSTAGE_SPLIT_EDGES", "64")
    w = small(n=1200, k=6, dims=(8, 8), deg=10.0, seed=33)
    p = make_problem(w, chunk_ptr=graphs.ragged_chunks(1200, 6, 5), bias_std=0.0)
    p.val = np.ones_like(p.val)
    p.W = [np.eye(8, dtype=np.float32)]
    p.x0 = np.ones_like(p.x0)
    p.hist = [np.zeros_like(p.hist[0])]
    p.grad_out = np.ones_like(p.grad_out)
    ref = run_oracle(p)
    run = _gpu(p).run()
    assert np.array_equal(run.np(run.cur[1]), ref.cur[1])
    assert np.array_equal(run.np(run.grad_in), ref.grad_in)


@pytest.mark.parametrize("short", [2, 8, 40])
@pytest.mark.parametrize("name,dims", [("c2_s", None), ("c3_s", None), ("c4_s", None), ("c4_s", (40, 72, 136)), ("c4_s", (64, 256, 200))])
def test_short_rows_served_a_row_per_lane_group(monkeypatch, short, name, dims):
    """Whole rows of at most a few entries can be served by 16-lane groups (a row each, vector-ALU sums) instead
    of a wavefront per row; forced here for several thresholds, full and ragged tile widths, forward and backward."""
    monkeypatch.setenv("GNNSTAGE_SHORT_ROW", str(short))
    w = CONFIGS[name]
    if dims is not None:
        w = Workload(w.name + "_w", "rmat", w.n, w.seed, list(dims), w.n_chunks, dtype="bf16", n_candidates=w.n_candidates,
                     rmat_abc=w.rmat_abc)
    p = make_problem(w, bias_std=0.05)
    _parity(p, TOL_BF16)


@pytest.mark.parametrize("name", ["c0", "c1_s", "c3_s"])
def test_weight_gradients_per_chunk_instead_of_one_product_per_layer(monkeypatch, name):
    """By default the stage keeps the gradient rows of a pass and takes every layer's weight gradient in one
    product after the last backward call; the per-chunk form must give the same gradients."""
    monkeypatch.setenv("GNNSTAGE_WGRAD_DEFER", "0")
    p = make_problem(CONFIGS[name], bias_std=0.05)
    _parity(p, TOL_F32 if name == "c0" else TOL_BF16)


@pytest.mark.parametrize("variant,dtype", [("gcn", "f32"), ("gcn", "bf16"), ("sage", "bf16"), ("gcnii", "bf16")])
def test_flushing_the_weight_gradients_of_a_backward_pass_that_stops_early(variant, dtype):
    """gnnstage_flush_weight_gradients after every backward call: the gradients then hold exactly the
    contributions of the calls made so far (compared with the oracle after each call), nothing is added twice,
    and the last call of the pass leaves the same totals."""
    dims = (16, 16, 16) if variant == "gcnii" else (24, 40, 48)
    w = small(n=900, k=5, dims=dims, variant=variant, dtype=dtype)
    p = make_problem(w, chunk_ptr=graphs.ragged_chunks(900, 5, 9), first_stage=False)
    tol = TOL_F32 if dtype == "f32" else TOL_BF16
    ref = p.new_oracle()
    ref.forward_pass(p.order)
    run = _gpu(p)
    assert all(run.stage.gnnstage_layer_order(j) == 0 for j in range(p.L))   # no transform-first layer here
    run.forward()
    torch.cuda.synchronize()
    for j in range(1, p.L + 1):
        run.cur[j].copy_(torch.from_numpy(ref.cur[j]).to(run.cur[j].dtype))
    for k in reversed([int(x) for x in p.order]):
        ref.backward_chunk(k, p.grad_out[ref.rows(k)])
        run.stage.stage_backward_chunk(k, run.grad_out[run.stage.rows(k)])
        run.stage.gnnstage_flush_weight_gradients()
        run.stage.gnnstage_flush_weight_gradients()          # nothing is owed any more: a no-op
        torch.cuda.synchronize()
        for j in range(p.L):
            assert max_rel(run.np(run.dW[j]), ref.dW[j]) <= tol, (k, j)
            if variant != "gcnii":
                assert max_rel(run.np(run.dbias[j]), ref.db[j]) <= tol, (k, j)


@pytest.mark.parametrize("slots", [4, 8])
@pytest.mark.parametrize("name", ["c1_s", "c3_s"])
def test_deeper_gather_queues(monkeypatch, slots, name):
    """The matrix-core aggregation normally keeps two gather slots per wave; run its 4- and 8-slot forms
    (other steady-loop lengths, other tails) against the same oracle."""
    monkeypatch.setenv("GNNSTAGE_SPMM_UNROLL", str(slots))
    p = make_problem(CONFIGS[name], bias_std=0.05)
    _parity(p, TOL_BF16)


@pytest.mark.parametrize("weights", ["given", "computed"])
@pytest.mark.parametrize("min_nnz,classes", [(6, 1), (24, 8), (2, 1)])
@pytest.mark.parametrize("name", ["c1_s", "c2_s", "c3_s"])
def test_dense_blocks_forced_on_small_graphs(monkeypatch, min_nnz, classes, name, weights):
    """Blocks of the degree-ordered matrix with enough entries are multiplied as dense tiles on the matrix
    cores, the rest stays sparse; force that split on the shrunk graphs (tiny thresholds, with and without
    source classes, ragged chunks), forward and backward, against the one oracle.  With weights given by
    the caller a block is a pair of bf16 weight tiles; when the library computes the normalisation itself
    (w = s(v) s(u)) it is a bit pattern and the scales move to the source rows and the result rows."""
    monkeypatch.setenv("GNNSTAGE_DENSE_MIN_NNZ", str(min_nnz))
    monkeypatch.setenv("GNNSTAGE_DENSE_MIN_SHARE", "0")
    monkeypatch.setenv("GNNSTAGE_DENSE_MIN_ENTRIES", "0")
    monkeypatch.setenv("GNNSTAGE_XCD_CLASSES", str(classes))
    monkeypatch.setenv("GNNSTAGE_CLASS_MIN_ROW", "16")
    w = CONFIGS[name]
    row_ptr, col = __import__("synth").make_graph(w)
    n = len(row_ptr) - 1
    p = make_problem(w, graph=(row_ptr, col), chunk_ptr=graphs.ragged_chunks(n, w.n_chunks, 23), bias_std=0.05)
    probe = _gpu(p, edge_val=weights)
    assert probe.stage.gnnstage_dense_entries(False) > 0 and probe.stage.gnnstage_dense_entries(True) > 0
    _parity(p, TOL_BF16, edge_val=weights)


def test_dense_blocks_switched_off_give_the_same_levels(monkeypatch):
    """The split into dense blocks and sparse remainder only regroups the same sum."""
    p = make_problem(CONFIGS["c1_s"], bias_std=0.05)
    monkeypatch.setenv("GNNSTAGE_DENSE_MIN_NNZ", "6")
    monkeypatch.setenv("GNNSTAGE_DENSE_MIN_SHARE", "0")
    monkeypatch.setenv("GNNSTAGE_DENSE_MIN_ENTRIES", "0")
    a = _gpu(p)
    a.forward()
    monkeypatch.setenv("GNNSTAGE_DENSE", "0")
    b = _gpu(p)
    b.forward()
    torch.cuda.synchronize()
    for j in range(1, p.L + 1):
        assert max_rel(a.np(a.cur[j]), b.np(b.cur[j])) <= 1e-2


@pytest.mark.parametrize("defer", ["1", "0"])
@pytest.mark.parametrize("name,dims", [("c1_s", None), ("c3_s", None), ("c4_s", None), ("c4_s", (200, 256, 136, 256))])
def test_one_workgroup_per_split_weight_gradient_on_small_inputs(monkeypatch, name, dims, defer):
    """Long weight-gradient products of up to 256 x 256 outputs run as one workgroup per row split that reads every
    operand row once (fused bias gradient as per-thread column sums); forced here on small inputs, ragged widths
    (200, 136: partial tiles, padded operand columns) and both the deferred and the per-chunk form."""
    monkeypatch.setenv("GNNSTAGE_GEMM_WIDE_MIN_ROWS", "1")
    monkeypatch.setenv("GNNSTAGE_WGRAD_DEFER", defer)
    w = CONFIGS[name]
    if dims is not None:
        w = Workload(w.name + "_w", "rmat", w.n, w.seed, list(dims), w.n_chunks, dtype="bf16", n_candidates=w.n_candidates,
                     rmat_abc=w.rmat_abc)
    p = make_problem(w, bias_std=0.05)
    _parity(p, TOL_BF16)


@pytest.mark.parametrize("name", ["c1_s", "c2_s", "c3_s", "c4_s"])
def test_persistent_gemm_on_small_inputs(monkeypatch, name):
    """The weight-stationary persistent GEMM normally serves only long operands; force it everywhere."""
    monkeypatch.setenv("GNNSTAGE_GEMM_WS_MIN_ROWS", "1")
    p = make_problem(CONFIGS[name], bias_std=0.05)
    _parity(p, TOL_BF16)


def test_source_class_schedule_fp32_probe(monkeypatch):
    """Exact-integer check of the class path: unit weights, ones, W = I (see the indicator probes below)."""
    monkeypatch.setenv("GNNSTAGE_XCD_CLASSES", "8")
    monkeypatch.setenv("GNNSTAGE_CLASS_MIN_ROW", "4")
    monkeypatch.setenv("GNNSTAGE_SPLIT_EDGES", "64")
    w = small(n=1200, k=6, dims=(8, 8), deg=10.0, seed=33)
    p = make_problem(w, chunk_ptr=graphs.ragged_chunks(1200, 6, 5), bias_std=0.0)
    p.val = np.ones_like(p.val)
    p.W = [np.eye(8, dtype=np.float32)]
    p.x0 = np.ones_like(p.x0)
    p.hist = [np.zeros_like(p.hist[0])]
    p.grad_out = np.ones_like(p.grad_out)
    ref = run_oracle(p)
    run = _gpu(p).run()
    assert np.array_equal(run.np(run.cur[1]), ref.cur[1])
    assert np.array_equal(run.np(run.grad_in), ref.grad_in)


@pytest.mark.parametrize("order_mode", ["aggregate", "transform"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_both_layer_orders(monkeypatch, order_mode, dtype):
    """(A H) W and A (H W) are the same layer; force each order on every layer of a stage whose
    widths go up and down, against the one oracle (which aggregates first)."""
    monkeypatch.setenv("GNNSTAGE_ORDER", order_mode)
    w = small(n=1100, k=5, dims=(48, 80, 32, 64), dtype=dtype, deg=8.0, seed=12, level0_f32=(dtype == "bf16"))
    p = make_problem(w, chunk_ptr=graphs.ragged_chunks(1100, 5, 7), first_stage=False)
    _parity(p, TOL_F32 if dtype == "f32" else TOL_BF16)


@pytest.mark.parametrize("dtype,d0", [("f32", 200), ("bf16", 200), ("bf16", 201), ("bf16", 602)])
def test_first_stage_with_aliased_history(dtype, d0):
    """hist[0] is the very same buffer as cur[0]; the wide first layer runs transform-first and shares
    one transformed table between current and historical reads.  In the bf16 stage the fp32 features are
    read as float pairs when their width is even (602: with a ragged last k-tile), element-wise when odd."""
    w = small(n=900, k=4, dims=(d0, 32, 32), dtype=dtype, deg=8.0, seed=13, level0_f32=(dtype == "bf16"))
    p = make_problem(w, first_stage=True)
    _parity(p, TOL_F32 if dtype == "f32" else TOL_BF16, need_input_grad=False, alias_hist0=True)
    _parity(p, TOL_F32 if dtype == "f32" else TOL_BF16, need_input_grad=True, alias_hist0=True)


def test_full_size_c1_in_the_benchmark_configuration():
    """configs[1] at full size, exactly as bench.py runs it (first stage: history of level 0 is the feature
    buffer itself, no input gradient, library-computed weights, dense blocks + source classes active): every
    level and every weight gradient against the oracle.  About a minute of oracle time on 16 host threads."""
    p = make_problem(CONFIGS["c1"], bias_std=0.05)
    probe = _gpu(p, need_input_grad=False, alias_hist0=True, edge_val="computed")
    assert probe.stage.gnnstage_dense_entries(False) > 10_000_000 and probe.stage.gnnstage_dense_entries(True) > 10_000_000
    del probe
    torch.cuda.empty_cache()
    _parity(p, TOL_BF16, need_input_grad=False, alias_hist0=True, edge_val="computed")


@pytest.mark.parametrize("name", ["c1_sage", "c1_res"])
def test_full_size_c1_graph_under_the_other_layer_types(name):
    """The 233 k vertex graph of configs[1] as a middle stage (256 -> 256 x 4, bf16, input gradient wanted) of GraphSage
    layers (mean aggregator computed by the library: dense blocks run as bit patterns with row / column scales) and
    of ResGCN+ layers (LayerNorm tables, end-of-pass aggregations for the LayerNorm parameters), at full size."""
    p = make_problem(CONFIGS[name], bias_std=0.05)
    _parity(p, TOL_BF16, edge_val="computed")


def test_full_size_c3_gcnii_stage():
    """configs[3] at full size: 16 GCNII layers over the 169k-vertex power-law graph, bf16."""
    p = make_problem(CONFIGS["c3"], bias_std=0.0)
    _parity(p, TOL_BF16)


# ----------------------------------------------------------------------------- select mask, bit-exact
@pytest.mark.parametrize("roles", ["cur1_hist0", "cur0_hist1"])
def test_indicator_probe_counts_selected_neighbours(roles):
    """edge weight 1, current rows all ones, history all zeros, W = I, b = 0: level 1 of every row is
    the NUMBER of neighbours read from the current buffers, an exact integer in fp32."""
    w = small(n=1500, k=7, dims=(8, 8), deg=12.0, seed=31)
    p = make_problem(w, chunk_ptr=graphs.ragged_chunks(1500, 7, 6), bias_std=0.0)
    p.val = np.ones_like(p.val)
    p.W = [np.eye(8, dtype=np.float32)]
    cur_v, hist_v = (1.0, 0.0) if roles == "cur1_hist0" else (0.0, 1.0)
    p.x0 = np.full_like(p.x0, cur_v)
    p.hist = [np.full_like(p.hist[0], hist_v)]
    st = p.new_oracle()
    st.begin_pass()
    run = _gpu(p)
    deg = np.diff(p.row_ptr).astype(np.int32)
    for pos, k in enumerate(p.order):
        want = st.select_counts(int(k))                      # oracle's integer count
        got_host = run.stage.gnnstage_debug_select_counts(int(k))  # library's packed tables, before the call
        assert np.array_equal(got_host, want)
        st.forward_chunk(int(k))
        run.stage.stage_forward_chunk(int(k), pos)
        torch.cuda.synchronize()
        rows = st.rows(int(k))
        got = run.np(run.cur[1][rows])
        expect = want if roles == "cur1_hist0" else deg[rows] - want
        assert np.array_equal(got, np.repeat(expect[:, None], 8, axis=1).astype(np.float32))


@pytest.mark.parametrize("d,deg,wbits,xmax", [(128, 9.0, 12, 4), (256, 9.0, 12, 4), (256, 200.0, 12, 4),
                                              (512, 70.0, 12, 4), (256, 9.0, 16, 2), (128, 30.0, 16, 2)])
def test_bf16_aggregation_is_exact_on_exactly_summable_inputs(monkeypatch, d, deg, wbits, xmax):
    """Edge weights with 12 or 16 significant bits (more than one bf16 holds), rows of small integers, W = I,
    b = 0: every product and every partial sum is exact in fp32, so level 1 and the input gradient are the
    bf16 rounding of the exact sum - bit for bit.  Fails if the matrix-core aggregation loses the low half
    of a weight, drops or repeats an entry, or reads a row from the wrong buffer.  Rows of 200 entries
    span several metadata batches."""
    monkeypatch.setenv("GNNSTAGE_DENSE_MIN_ENTRIES", "0")  # small graph: let its dense blocks (if any) be used
    n = 1500
    w = small(n=n, k=5, dims=(d, d), dtype="bf16", deg=deg, seed=41)
    p = make_problem(w, chunk_ptr=graphs.ragged_chunks(n, 5, 11), bias_std=0.0)
    rng = np.random.default_rng(7)
    p.val = (rng.integers(1 << (wbits - 1), 1 << wbits, size=p.val.shape) / float(1 << (wbits - 1))).astype(np.float32)
    p.W = [np.eye(d, dtype=np.float32)]
    p.x0 = rng.integers(0, xmax, size=p.x0.shape).astype(np.float32)
    p.hist = [rng.integers(0, xmax, size=p.hist[0].shape).astype(np.float32)]
    p.grad_out = rng.integers(-1, 2, size=p.grad_out.shape).astype(np.float32)
    ref = run_oracle(p)
    run = _gpu(p).run()
    # the denser graphs take the dense-block path (rows of width 128 or 256 only)
    assert (run.stage.gnnstage_dense_entries(False) > 0) == (deg >= 70.0 and d in (128, 256))
    assert np.array_equal(run.np(run.cur[1]), ref.cur[1])
    assert np.array_equal(run.np(run.grad_in), ref.grad_in)
    assert len(np.unique(ref.cur[1])) > 50


def test_backward_mask_probe_counts_processed_readers():
    """dZ == 1 everywhere it is defined: with W = I the input gradient of u is the number of
    readers v (u in N(v)) whose chunk was processed at or after u's chunk, an exact integer."""
    w = small(n=1200, k=6, dims=(8, 8), deg=10.0, seed=32)
    p = make_problem(w, chunk_ptr=graphs.ragged_chunks(1200, 6, 9), bias_std=0.0)
    p.val = np.ones_like(p.val)
    p.W = [np.eye(8, dtype=np.float32)]
    p.x0 = np.ones_like(p.x0)
    p.hist = [np.ones_like(p.hist[0])]
    p.grad_out = np.ones_like(p.grad_out)
    ref = run_oracle(p)
    run = _gpu(p).run()
    assert np.array_equal(run.np(run.grad_in), ref.grad_in)
    assert ref.grad_in.max() > 3 and np.all(ref.grad_in == np.round(ref.grad_in))


# ----------------------------------------------------------------------------- history + protocol
def test_update_history_and_second_epoch():
    p = make_problem(small(k=3), first_stage=False)
    ref = run_oracle(p)
    run = _gpu(p).run()
    ref.update_history()
    run.stage.update_history()
    torch.cuda.synchronize()
    for j in range(p.L):
        assert np.array_equal(run.np(run.hist[j]), run.np(run.cur[j]))
    order2 = values.permutation(99, 1, 3)
    ref.zero_grads()
    for t in run.dW + run.dbias:
        t.zero_()
    ref.forward_pass(order2)
    ref.backward_pass(p.grad_out)
    run.forward(order2)
    run.backward(order2)
    torch.cuda.synchronize()
    _compare(run, ref, p, TOL_F32)


@pytest.mark.parametrize("variant,dtype,first_stage", [("gcn", "f32", False), ("gcn", "f32", True), ("gcnii", "bf16", False),
                                                        ("sage", "bf16", False), ("resgcn", "f32", False)])
def test_history_refreshed_by_trading_buffers(variant, dtype, first_stage):
    """gnnstage_update_history_swap: after a complete pass the buffers of levels 1 .. L-1 trade places inside the
    library instead of being copied (level 0 is copied).  The historical levels then hold exactly what the current
    ones held, and three further epochs (each refreshed the same way, new chunk order every epoch) match the oracle,
    which copies.  Guards: no second trade, and no copying refresh, before another complete pass."""
    import paper_2308_10087_amd as g
    dims = (16, 16, 16, 16) if variant in ("gcnii", "resgcn") else (24, 40, 16, 32)
    w = small(n=800, k=4, dims=dims, variant=variant, dtype=dtype)
    p = make_problem(w, first_stage=first_stage, bias_std=0.05)
    tol = TOL_F32 if dtype == "f32" else TOL_BF16
    ref = run_oracle(p)
    run = _gpu(p, alias_hist0=first_stage).run()
    st = run.stage
    order0 = [int(k) for k in p.order]
    st.stage_forward_chunk(order0[0], 0)               # a new pass, one chunk in: no trade now
    with pytest.raises(g.GnnStageError) as e:
        st.gnnstage_update_history_swap()
    assert e.value.code == -3
    for pos, k in enumerate(order0[1:], start=1):      # complete it (same order, same inputs: same levels)
        st.stage_forward_chunk(k, pos)
    run.backward()
    torch.cuda.synchronize()
    for epoch in range(1, 4):
        before = [st.cur[j].clone() for j in range(p.L)]
        ptrs = [(st.cur[j].data_ptr(), st.hist[j].data_ptr()) for j in range(p.L)]
        ref.update_history()
        st.gnnstage_update_history_swap()
        torch.cuda.synchronize()
        for j in range(p.L):
            assert torch.equal(st.hist[j], before[j]), (epoch, j)
            now = st.gnnstage_level_buffers(j)
            if j >= 1 and ptrs[j][0] != ptrs[j][1]:
                assert now == (ptrs[j][1], ptrs[j][0]), (epoch, j)      # traded places
            else:
                assert now == ptrs[j], (epoch, j)                        # level 0 keeps its buffers
        assert st.gnnstage_level_buffers(p.L) == (st.cur[p.L].data_ptr(), None)
        with pytest.raises(g.GnnStageError) as e:
            st.gnnstage_update_history_swap()
        assert e.value.code == -3
        if any(a != b for a, b in ptrs[1:]):
            with pytest.raises(g.GnnStageError) as e:
                st.update_history()
            assert e.value.code == -3
        run.cur, run.hist = st.cur, st.hist    # the harness reads results through these lists
        order = [int(k) for k in values.permutation(77, epoch, len(p.chunk_ptr) - 1)]
        ref.zero_grads()
        for t in run.dW + (run.dbias or []) + ([run.grad_h0] if run.grad_h0 is not None else []) + \
                (run.d_ln_gamma or []) + (run.d_ln_beta or []):
            t.zero_()
        ref.forward_pass(order)
        run.forward(order)
        torch.cuda.synchronize()
        _check_forward(run, ref, p, tol)
        for j in range(1, p.L + 1):
            run.cur[j].copy_(torch.from_numpy(ref.cur[j]).to(run.cur[j].dtype))
        ref.backward_pass(p.grad_out)
        run.backward(order)
        torch.cuda.synchronize()
        _compare(run, ref, p, tol)


@pytest.mark.parametrize("variant,dims", [("gcn", (24, 40, 16, 32)), ("gcnii", (32, 32, 32)), ("sage", (24, 40, 16))])
def test_a_pass_captured_in_a_hip_graph_replays_bit_for_bit(variant, dims):
    """The per-chunk calls only launch kernels on the caller's stream (no allocation, no synchronisation, no memset
    node), so a whole forward + backward pass with a fixed chunk order can be captured in a HIP graph.  Three replays,
    with the caller's own eager work (zeroing the gradient accumulators) and a synchronisation between them, each
    leave exactly what the eager pass left."""
    w = small(n=900, k=4, dims=dims, variant=variant, dtype="bf16", deg=9.0)
    p = make_problem(w, first_stage=False, bias_std=0.05)
    run = _gpu(p)
    outs = lambda: [run.cur[p.L], run.grad_in] + run.dW + (run.dbias or []) + ([run.grad_h0] if run.grad_h0 is not None else [])
    accum = lambda: run.dW + (run.dbias or []) + ([run.grad_h0] if run.grad_h0 is not None else [])
    run.run()                                   # eager, also warms every kernel
    for t in accum():
        t.zero_()
    run.run()
    want = [t.clone() for t in outs()]
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            run.forward()
            run.backward()
    torch.cuda.synchronize()
    for rep in range(3):
        for t in accum():
            t.zero_()
        run.cur[p.L].zero_()
        run.grad_in.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(outs(), want):
            assert torch.equal(a, b), rep


def test_protocol_errors():
    import paper_2308_10087_amd as g
    p = make_problem(small(k=3))
    run = _gpu(p)
    s = run.stage
    with pytest.raises(g.GnnStageError) as e:
        s.stage_forward_chunk(3, 0)
    assert e.value.code == -2
    with pytest.raises(g.GnnStageError) as e:
        s.stage_forward_chunk(0, 1)  # pass not started
    assert e.value.code == -3
    s.stage_forward_chunk(1, 0)
    with pytest.raises(g.GnnStageError) as e:
        s.stage_forward_chunk(1, 1)  # same chunk twice
    assert e.value.code == -3
    with pytest.raises(g.GnnStageError) as e:
        s.stage_backward_chunk(1, run.grad_out[s.rows(1)])  # forward pass incomplete
    assert e.value.code == -3
    s.stage_forward_chunk(2, 1)
    s.stage_forward_chunk(0, 2)
    with pytest.raises(g.GnnStageError) as e:
        s.stage_backward_chunk(1, run.grad_out[s.rows(1)])  # must start with the last forwarded chunk
    assert e.value.code == -3
    s.stage_backward_chunk(0, run.grad_out[s.rows(0)])
    s.stage_backward_chunk(2, run.grad_out[s.rows(2)])
    s.stage_backward_chunk(1, run.grad_out[s.rows(1)])
    with pytest.raises(g.GnnStageError) as e:
        s.stage_backward_chunk(1, run.grad_out[s.rows(1)])
    assert e.value.code == -3
    torch.cuda.synchronize()


# ----------------------------------------------------------------------------- GraphSage variant
@pytest.mark.parametrize("dims", [(24, 40, 16, 32), (7, 5, 3), (100, 128, 64)])
def test_sage_fp32(dims):
    w = small(dims=dims, n=911, k=6, variant="sage")
    p = make_problem(w, chunk_ptr=graphs.ragged_chunks(911, 6, 4))
    _parity(p, TOL_F32)
    _parity(make_problem(w, first_stage=False, noise_std=0.3), TOL_F32)


def test_sage_fp32_mean_aggregator_computed_by_the_library():
    """edge_val == NULL with the GraphSage variant means the mean aggregator, 1 / (row length)."""
    p = make_problem(small(variant="sage"))
    a = _gpu(p, edge_val="given").run()
    b = _gpu(p, edge_val="computed").run()
    for j in range(1, p.L + 1):
        assert torch.equal(a.cur[j], b.cur[j])
    for j in range(p.L):
        assert torch.equal(a.dW[j], b.dW[j])
    assert torch.equal(a.grad_in, b.grad_in)


@pytest.mark.parametrize("dims,level0_f32", [((64, 128, 128, 64), False), ((100, 128, 256), True), ((256, 256, 256), False)])
def test_sage_bf16(dims, level0_f32):
    w = Workload("sage_s", "rmat", 5003, 2308100890, list(dims), 6, variant="sage", dtype="bf16", level0_f32=level0_f32,
                 n_candidates=60_000)
    p = make_problem(w, first_stage=level0_f32)
    _parity(p, TOL_BF16)


@pytest.mark.parametrize("weights", ["given", "computed"])
def test_sage_bf16_dense_blocks(monkeypatch, weights):
    """Given weights go through the tile kernel; the mean aggregator computed by the library is a pattern with
    1 / |N(v)| as the row scale of a forward block and as the column scale of a block of the transposed index."""
    monkeypatch.setenv("GNNSTAGE_DENSE_MIN_ENTRIES", "0")
    monkeypatch.setenv("GNNSTAGE_DENSE_MIN_NNZ", "64")
    monkeypatch.setenv("GNNSTAGE_DENSE_MIN_SHARE", "0.05")
    w = Workload("sage_d", "rmat", 6007, 2308100891, [128, 128, 128], 4, variant="sage", dtype="bf16", n_candidates=260_000)
    p = make_problem(w, first_stage=False)
    probe = _gpu(p, edge_val=weights)
    assert probe.stage.gnnstage_dense_entries(False) > 0 and probe.stage.gnnstage_dense_entries(True) > 0
    _parity(p, TOL_BF16, edge_val=weights)


# ----------------------------------------------------------------------------- ResGCN+ variant
@pytest.mark.parametrize("d,L", [(24, 3), (7, 2), (64, 4), (200, 2)])
def test_resgcn_fp32(d, L):
    w = small(dims=(d,) * (L + 1), n=911, k=6, variant="resgcn")
    _parity(make_problem(w, chunk_ptr=graphs.ragged_chunks(911, 6, 4)), TOL_F32)
    _parity(make_problem(w, first_stage=False, noise_std=0.3), TOL_F32)
    _parity(make_problem(w, first_stage=False, noise_std=0.3), TOL_F32, need_input_grad=False)


@pytest.mark.parametrize("d,L", [(128, 3), (256, 2), (72, 4)])
def test_resgcn_bf16(d, L):
    w = Workload("res_s", "rmat", 5003, 2308100892, [d] * (L + 1), 6, variant="resgcn", dtype="bf16", n_candidates=60_000)
    _parity(make_problem(w, first_stage=False), TOL_BF16)
    _parity(make_problem(w), TOL_BF16)


def test_resgcn_bf16_dense_blocks(monkeypatch):
    monkeypatch.setenv("GNNSTAGE_DENSE_MIN_ENTRIES", "0")
    monkeypatch.setenv("GNNSTAGE_DENSE_MIN_NNZ", "64")
    monkeypatch.setenv("GNNSTAGE_DENSE_MIN_SHARE", "0.05")
    w = Workload("res_d", "rmat", 6007, 2308100893, [128, 128, 128], 4, variant="resgcn", dtype="bf16", n_candidates=260_000)
    p = make_problem(w, first_stage=False)
    probe = _gpu(p)
    assert probe.stage.gnnstage_dense_entries(False) > 0 and probe.stage.gnnstage_dense_entries(True) > 0
    _parity(p, TOL_BF16)


@pytest.mark.parametrize("rate,seed", [(0.5, 7), (0.3, 2**63 + 12345), (0.9, 1)])
def test_resgcn_dropout(rate, seed):
    """Same keep decisions on both sides (an integer comparison of counter-based draws), so the usual
    tolerances hold element by element; the rate crosses the C ABI as a float and the oracle gets that float."""
    rate = float(np.float32(rate))
    w = small(dims=(40,) * 4, n=911, k=6, variant="resgcn")
    p = make_problem(w, chunk_ptr=graphs.ragged_chunks(911, 6, 4), first_stage=False, noise_std=0.3,
                     dropout_p=rate, dropout_seed=seed)
    worst = _parity(p, TOL_F32)
    ref = run_oracle(p)
    keep = ref.dropout_keep_mask(0)
    assert abs(keep.mean() - (1 - rate)) < 0.02
    wb = Workload("res_drop", "rmat", 5003, 2308100894, [128] * 4, 6, variant="resgcn", dtype="bf16", n_candidates=60_000)
    _parity(make_problem(wb, first_stage=False, dropout_p=rate, dropout_seed=seed), TOL_BF16)


@pytest.mark.parametrize("order", ["aggregate", "transform"])
@pytest.mark.parametrize("variant", ["gcn", "sage"])
@pytest.mark.parametrize("rate,seed", [(0.5, 7), (0.3, 2**63 + 12345)])
def test_output_dropout_of_gcn_and_sage_layers(monkeypatch, rate, seed, variant, order):
    """Dropout on every layer's output, applied to the chunk's rows right behind the kernel that writes the level (the
    transform when the layer aggregates first, the aggregation when it transforms first); the backward masks carry
    1 / (1 - p)."""
    monkeypatch.setenv("GNNSTAGE_ORDER", order)
    rate = float(np.float32(rate))
    w = small(dims=(40, 24, 32, 16), n=911, k=6, variant=variant)
    p = make_problem(w, chunk_ptr=graphs.ragged_chunks(911, 6, 4), first_stage=False, noise_std=0.3,
                     dropout_p=rate, dropout_seed=seed)
    _parity(p, TOL_F32)
    ref = run_oracle(p)
    keep = ref.dropout_keep_mask(0)
    assert keep.shape == (911, 24) and abs(keep.mean() - (1 - rate)) < 0.02
    assert np.all(ref.cur[1][keep == 0] == 0)
    wb = Workload("out_drop", "rmat", 5003, 2308100895, [100, 128, 256, 128], 6, variant=variant, dtype="bf16",
                  level0_f32=True, n_candidates=60_000)
    _parity(make_problem(wb, dropout_p=rate, dropout_seed=seed), TOL_BF16)
    _parity(make_problem(wb, dropout_p=rate, dropout_seed=seed), TOL_BF16, need_input_grad=False)


@pytest.mark.parametrize("variant", ["gcn", "resgcn"])
def test_dropout_rate_switched_off_for_an_evaluation_pass_and_on_again(variant):
    import paper_2308_10087_amd as g
    dims = (24, 24, 24)
    p = make_problem(small(dims=dims, n=500, k=4, variant=variant), first_stage=False, dropout_p=0.5, dropout_seed=3)
    p0 = make_problem(small(dims=dims, n=500, k=4, variant=variant), first_stage=False)
    plain = _gpu(p0).run()
    run = _gpu(p)
    run.forward()
    dropped = run.cur[p.L].clone()
    assert not torch.equal(dropped, plain.cur[p.L])
    run.stage.gnnstage_set_dropout_rate(0.0)
    run.stage.forward_pass(p.order)
    assert torch.equal(run.cur[p.L], plain.cur[p.L])            # the evaluation pass is the stage without dropout
    run.stage.stage_forward_chunk(int(p.order[0]), 0)
    with pytest.raises(g.GnnStageError) as e:
        run.stage.gnnstage_set_dropout_rate(0.5)                # not inside a pass
    assert e.value.code == -3
    for pos, k in enumerate(p.order[1:], start=1):
        run.stage.stage_forward_chunk(int(k), pos)
    run.stage.gnnstage_set_dropout_rate(0.5)
    run.forward()
    assert torch.equal(run.cur[p.L], dropped)                   # and training goes on as before
    with pytest.raises(g.GnnStageError) as e:
        run.stage.gnnstage_set_dropout_rate(1.0)
    assert e.value.code == -1


def test_no_dropout_in_gcnii_layers():
    import paper_2308_10087_amd as g
    p = make_problem(small(dims=(16,) * 3, n=300, k=3, variant="gcnii"))
    p.dropout_p = 0.5
    with pytest.raises(g.GnnStageError) as e:
        _gpu(p)
    assert e.value.code == -1


def test_resgcn_dropout_seed_changes_the_pass_and_is_locked_inside_one():
    import paper_2308_10087_amd as g
    w = small(dims=(24,) * 3, n=500, k=4, variant="resgcn")
    p = make_problem(w, first_stage=False, dropout_p=0.5, dropout_seed=3)
    run = _gpu(p)
    run.forward()
    a = run.cur[p.L].clone()
    run.forward()
    assert torch.equal(run.cur[p.L], a)                 # same seed, same pass
    run.stage.gnnstage_set_dropout_seed(4)
    run.stage.forward_pass(p.order)
    assert not torch.equal(run.cur[p.L], a)
    run.stage.stage_forward_chunk(int(p.order[0]), 0)
    with pytest.raises(g.GnnStageError) as e:
        run.stage.gnnstage_set_dropout_seed(5)
    assert e.value.code == -3
    for pos, k in enumerate(p.order[1:], start=1):
        run.stage.stage_forward_chunk(int(k), pos)
    run.stage.stage_backward_chunk(int(p.order[-1]), run.grad_out[run.stage.rows(int(p.order[-1]))])
    with pytest.raises(g.GnnStageError) as e:
        run.stage.gnnstage_set_dropout_seed(6)      # the backward pass must see the forward pass's decisions
    assert e.value.code == -3


def test_seed_set_between_forward_and_backward_belongs_to_the_next_pass():
    """A pass keeps the seed and the rate it started with: a new seed (or rate) set after the forward pass is
    taken by the NEXT pass, and the backward pass still redraws the masks of its own forward pass."""
    w = small(dims=(24,) * 3, n=500, k=4, variant="resgcn")
    p = make_problem(w, first_stage=False, dropout_p=0.5, dropout_seed=3)
    ref = _gpu(p).run()
    run = _gpu(p)
    run.forward()
    run.stage.gnnstage_set_dropout_seed(99)
    run.stage.gnnstage_set_dropout_rate(0.25)
    run.backward()
    torch.cuda.synchronize()
    for j in range(p.L):
        assert torch.equal(run.dW[j], ref.dW[j]) and torch.equal(run.d_ln_gamma[j], ref.d_ln_gamma[j])
    assert torch.equal(run.grad_in, ref.grad_in)
    run.stage.forward_pass(p.order)                      # the next pass runs with seed 99 and rate 0.25
    torch.cuda.synchronize()
    assert not torch.equal(run.cur[p.L], ref.cur[p.L])


# ----------------------------------------------------------------------------- size limits and degenerate inputs
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_maximum_chunk_count_with_tiny_chunks(dtype):
    """256 chunks (the most the packed index word's chunk field is sized for here), most of one to four
    vertices, shuffled order."""
    n = 700
    w = small(n=n, k=256, dims=(16, 24, 16), dtype=dtype, deg=5.0)
    chunk_ptr = graphs.ragged_chunks(n, 256, 11)
    assert np.diff(chunk_ptr).min() == 1
    p = make_problem(w, chunk_ptr=chunk_ptr, first_stage=False, noise_std=0.2)
    _parity(p, TOL_BF16 if dtype == "bf16" else TOL_F32)


def test_rows_without_entries_and_a_single_vertex_graph():
    """Vertices nobody points at (empty rows: the aggregation is zero, the layer output ReLU(b)), given weights;
    and the smallest graph there is."""
    rng = np.random.default_rng(3)
    n = 300
    dst = rng.integers(0, n // 2, 2500)          # rows n/2 .. n-1 stay empty
    src = rng.integers(0, n, 2500)
    row_ptr, col = graphs.from_directed_pairs(n, dst, src)
    assert np.diff(row_ptr)[n // 2:].max() == 0
    w = small(n=n, k=4, dims=(12, 20, 8))
    p = make_problem(w, graph=(row_ptr, col), first_stage=False, noise_std=0.2)
    p.val[...] = rng.uniform(0.1, 1.0, size=p.val.shape).astype(np.float32)   # D = 0 has no normalisation: weights are given
    _parity(p, TOL_F32)
    one = small(n=1, k=1, dims=(4, 4, 4))
    g1 = (np.array([0, 1], dtype=np.int64), np.array([0], dtype=np.int32))
    _parity(make_problem(one, graph=g1), TOL_F32)


@pytest.mark.parametrize("name", ["c1_s", "c2_s"])
def test_chunks_from_the_partitioner(monkeypatch, name):
    """Locality-aware chunks: about half of a chunk's neighbours are its own vertices, so the source classes of a
    launch are far from equal id ranges, and the chunks differ in their entry counts."""
    import paper_2308_10087_amd as g
    from synth.configs import make_graph
    monkeypatch.setenv("GNNSTAGE_XCD_CLASSES", "8")
    monkeypatch.setenv("GNNSTAGE_CLASS_MIN_ROW", "16")
    w = CONFIGS[name]
    row_ptr, col = make_graph(w)
    part, perm, chunk_ptr = g.gnnstage_partition_chunks(row_ptr, col, w.n_chunks)
    graph = g.gnnstage_permute_csr(row_ptr, col, perm)
    rows = np.repeat(np.arange(len(row_ptr) - 1), np.diff(row_ptr))
    assert np.mean(part[rows] != part[col]) < 0.8 * (1 - 1 / w.n_chunks)
    p = make_problem(w, graph=graph, chunk_ptr=chunk_ptr)
    _parity(p, TOL_BF16)
