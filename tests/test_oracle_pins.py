"""Pins of the CPU oracle against things other than itself (all run without a GPU).

  P1  dense  A_hat . H . W  products from a library matmul (Section 2.1)
  P2  one chunk never reads history (Section 3.3)
  P3  history == full-graph levels  =>  chunked == full graph, any K, any order
  P4  first-stage aliasing hist[0] == cur[0]  =>  level 1 is the full-graph level 1
  P5  hand-computed 5-vertex example (tests/golden/k4_plus_isolated.txt)
  P6  finite differences and torch autograd of an independent dense chunked forward
  P7  GCNII special cases
  +   normalisation closed forms / eigenvector invariant, transposed index round trip,
      select counts by brute force, bf16 rounding against torch, update_history.
"""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from synth import graphs, values
from synth.configs import CONFIGS, Workload

from helpers import edge_weights, gcnii_beta, make_problem, max_rel, run_oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- helpers
def dense_adj(row_ptr, col, val, n):
    A = np.zeros((n, n), dtype=np.float64)
    for v in range(n):
        for e in range(row_ptr[v], row_ptr[v + 1]):
            A[v, col[e]] = val[e]
    return A


def tiny_workload(n=41, k=3, dims=(5, 7, 6, 4), variant="gcn", seed=77):
    return Workload("tiny", "er", n, seed, list(dims), k, variant=variant, avg_degree=4.0,
                    gcnii_first_layer=3)


def ln_relu_np(x, gamma, beta, eps=1e-5):
    mu = x.mean(axis=1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=1, keepdims=True)
    return np.maximum(gamma * (x - mu) / np.sqrt(var + eps) + beta, 0.0)


def dense_full_graph_levels(A, x0, W, b, variant="gcn", a=0.0, beta=None, h0=None, ln=None):
    levels = [x0.astype(np.float64)]
    for j in range(len(W)):
        if variant == "resgcn":
            r = ln_relu_np(levels[-1], ln[0][j].astype(np.float64), ln[1][j].astype(np.float64))
            levels.append(levels[-1] + (A @ r) @ W[j].astype(np.float64) + b[j].astype(np.float64))
            continue
        z = A @ levels[-1]
        if variant == "gcn":
            y = z @ W[j].astype(np.float64) + b[j].astype(np.float64)
        elif variant == "sage":
            d = levels[-1].shape[1]
            y = levels[-1] @ W[j][:d].astype(np.float64) + z @ W[j][d:].astype(np.float64) + b[j].astype(np.float64)
        else:
            p = (1 - a) * z + a * h0.astype(np.float64)
            y = (1 - beta[j]) * p + beta[j] * (p @ W[j].astype(np.float64))
        levels.append(np.maximum(y, 0.0))
    return levels


def torch_dense_chunked(p, A, order, x0_t, W_t, b_t, h0_t=None, ln_t=None, drop=None):
    """Independent dense formulation of Algorithm 1's forward for autograd: per chunk and
    layer, split the dense adjacency columns into processed / unprocessed blocks."""
    n, L, K = p.n, p.L, p.chunk_ptr.shape[0] - 1
    A_t = torch.from_numpy(A)
    chunk_of = np.zeros(n, dtype=np.int64)
    for c in range(K):
        chunk_of[p.chunk_ptr[c]:p.chunk_ptr[c + 1]] = c
    hist = [torch.from_numpy(h.astype(np.float64)) for h in p.hist]
    # cur_rows[j][c] = tensor of rows of chunk c at level j (None until produced)
    cur_rows = [[None] * K for _ in range(L + 1)]
    for c in range(K):
        cur_rows[0][c] = x0_t[p.chunk_ptr[c]:p.chunk_ptr[c + 1]]
    done = []
    for k in order:
        done.append(int(k))
        rows = slice(int(p.chunk_ptr[k]), int(p.chunk_ptr[k + 1]))
        for j in range(L):
            z = torch.zeros((rows.stop - rows.start, p.dims[j]), dtype=torch.float64)
            for c in range(K):
                cols = slice(int(p.chunk_ptr[c]), int(p.chunk_ptr[c + 1]))
                src = cur_rows[j][c] if c in done else hist[j][cols]
                if p.w.variant == "resgcn":  # a library LayerNorm, then ReLU, on whichever row is read
                    src = torch.relu(torch.nn.functional.layer_norm(src, (p.dims[j],), ln_t[0][j], ln_t[1][j], 1e-5))
                    if drop is not None:  # keep decisions are an input here; 1 / (1 - p) rescales the survivors
                        src = src * drop[j][cols] / (1.0 - p.dropout_p)
                z = z + A_t[rows, cols] @ src
            if p.w.variant == "gcn":
                y = z @ W_t[j] + b_t[j]
            elif p.w.variant == "sage":
                d = p.dims[j]
                y = cur_rows[j][k] @ W_t[j][:d] + z @ W_t[j][d:] + b_t[j]
            elif p.w.variant == "resgcn":
                cur_rows[j + 1][k] = cur_rows[j][k] + z @ W_t[j] + b_t[j]
                continue
            else:
                pm = (1 - p.a) * z + p.a * h0_t[rows]
                y = (1 - p.beta[j]) * pm + p.beta[j] * (pm @ W_t[j])
            cur_rows[j + 1][k] = torch.relu(y)
            if drop is not None:  # GCN, GraphSage: dropout on the layer's output; keep decisions are an input here
                cur_rows[j + 1][k] = cur_rows[j + 1][k] * drop[j][rows] / (1.0 - p.dropout_p)
    return torch.cat([cur_rows[L][c] for c in range(K)], dim=0)


# ----------------------------------------------------------------------------- normalisation
def test_norm_regular_ring_closed_form():
    n = 12
    iu = np.arange(n)
    ju = (iu + 1) % n
    lo, hi = np.minimum(iu, ju), np.maximum(iu, ju)
    row_ptr, col = graphs.from_undirected_pairs(n, lo, hi)
    val = oracle.gcn_norm(row_ptr, col)
    assert np.all(np.diff(row_ptr) == 3)
    assert np.array_equal(val, np.full(3 * n, np.float32(1.0 / 3.0)))


def test_norm_sqrt_degree_is_fixed_point():
    # D^-1/2 (A+I) D^-1/2 has eigenvector sqrt(D) with eigenvalue 1, and is symmetric.
    w = tiny_workload(n=60)
    row_ptr, col = graphs.erdos_renyi(w.n, 5.0, 5)
    val = oracle.gcn_norm(row_ptr, col, f64=True)
    A = dense_adj(row_ptr, col, val, w.n)
    sd = np.sqrt(np.diff(row_ptr).astype(np.float64))
    assert np.allclose(A @ sd, sd, rtol=0, atol=1e-12)
    assert np.allclose(A, A.T, rtol=0, atol=0)
    # a directed (non-symmetric) structure uses the row length of each endpoint's own row
    rp2, col2 = graphs.from_directed_pairs(3, [0, 0, 1, 2, 0, 1], [0, 1, 1, 2, 2, 2])
    v2 = oracle.gcn_norm(rp2, col2, f64=True)
    A2 = dense_adj(rp2, col2, v2, 3)
    assert A2[0, 1] == pytest.approx(1 / np.sqrt(3 * 2)) and A2[1, 2] == pytest.approx(1 / np.sqrt(2 * 1))


# ----------------------------------------------------------------------------- P1 / P2
@pytest.mark.parametrize("variant", ["gcn", "gcnii", "sage", "resgcn"])
def test_p1_p2_one_chunk_equals_dense(variant):
    dims = (5, 7, 6, 4) if variant in ("gcn", "sage") else (6, 6, 6, 6)
    w = tiny_workload(k=1, dims=dims, variant=variant)
    p = make_problem(w)
    # poison the history: with one chunk it must never be read
    for h in p.hist:
        h[...] = 1e6
    st = p.new_oracle(f64=True)
    st.forward_pass([0])
    A = dense_adj(p.row_ptr, p.col, edge_weights(variant, p.row_ptr, p.col, f64=True), p.n)
    ref = dense_full_graph_levels(A, p.x0, p.W, p.b, variant, p.a, p.beta, p.h0, ln=(p.ln_gamma, p.ln_beta))
    for j in range(1, p.L + 1):
        assert np.allclose(st.cur[j], ref[j], rtol=1e-12, atol=1e-12), j
    # the fp32-storage build agrees to fp32 rounding
    st32 = p.new_oracle()
    st32.forward_pass([0])
    for j in range(1, p.L + 1):
        assert max_rel(st32.cur[j], ref[j]) < 2e-6


# ----------------------------------------------------------------------------- P3 / P4
@pytest.mark.parametrize("k,seed", [(2, 1), (5, 2), (7, 3)])
def test_p3_history_equal_to_full_graph_removes_staleness(k, seed):
    w = tiny_workload(n=53, k=k, seed=seed)
    p = make_problem(w, chunk_ptr=graphs.ragged_chunks(53, k, seed))
    full = make_problem(w, chunk_ptr=np.array([0, 53]))
    ref = full.new_oracle()
    ref.forward_pass([0])
    st = p.new_oracle()
    for j in range(p.L):
        st.hist[j][...] = ref.cur[j]
    st.forward_pass(values.permutation(seed, 9, k))
    for j in range(1, p.L + 1):
        assert np.array_equal(st.cur[j], ref.cur[j]), j  # bit-exact: same sums in the same order


def test_p4_first_stage_level1_has_no_staleness():
    w = tiny_workload(n=47, k=4)
    p = make_problem(w, first_stage=True)
    assert np.array_equal(p.hist[0], p.x0)
    full = make_problem(w, chunk_ptr=np.array([0, 47]))
    ref = full.new_oracle()
    ref.forward_pass([0])
    st = p.new_oracle()
    st.forward_pass(p.order)
    assert np.array_equal(st.cur[1], ref.cur[1])
    # deeper levels DO differ (stale level-1 history was perturbed)
    assert not np.array_equal(st.cur[2], ref.cur[2])


# ----------------------------------------------------------------------------- P5
def _read_gold(name):
    out = {}
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *nums = line.split()
            out[key] = np.array([float(x) for x in nums])
    return out


def test_p5_hand_example():
    gold = _read_gold("k4_plus_isolated.txt")
    iu, ju = np.triu_indices(4, k=1)
    row_ptr, col = graphs.from_undirected_pairs(5, iu, ju)
    val = oracle.gcn_norm(row_ptr, col)
    assert np.array_equal(val, np.array([0.25] * 16 + [1.0], dtype=np.float32))
    st = oracle.OracleStage(row_ptr, col, val, [0, 2, 5], [1, 1, 1],
                            [gold["W1"].reshape(1, 1), gold["W2"].reshape(1, 1)], [gold["b1"], gold["b2"]])
    st.cur[0][:, 0] = gold["cur0"]
    st.hist[0][:, 0] = gold["cur0"]
    st.hist[1][:, 0] = gold["hist1"]
    st.forward_pass([0, 1])
    assert np.array_equal(st.cur[1][:, 0], gold["level1"])
    assert np.array_equal(st.cur[2][:, 0], gold["level2"])
    assert np.array_equal(st.Z[1][:, 0], gold["Z1saved"])
    for dz in st.dZ:
        dz[...] = -77.0  # stale gradient rows from an earlier epoch: never read (technique 3)
    st.backward_pass(gold["grad_out"].reshape(5, 1))
    assert st.dW[1][0, 0] == gold["dW2"][0] and st.db[1][0] == gold["db2"][0]
    assert st.dW[0][0, 0] == gold["dW1"][0] and st.db[0][0] == gold["db1"][0]
    assert np.array_equal(st.grad_in[:, 0], gold["grad_in"])
    # one chunk: the exact full-graph answer
    st1 = oracle.OracleStage(row_ptr, col, val, [0, 5], [1, 1, 1],
                             [gold["W1"].reshape(1, 1), gold["W2"].reshape(1, 1)], [gold["b1"], gold["b2"]])
    st1.cur[0][:, 0] = gold["cur0"]
    st1.forward_pass([0])
    assert np.array_equal(st1.cur[2][:, 0], gold["full_graph_level2"])
    # select counts: chunk a first sees 2 current + 2 historical neighbours
    st.begin_pass()
    assert np.array_equal(st.select_counts(0), [2, 2])
    st.forward_chunk(0)
    assert np.array_equal(st.select_counts(1), [4, 4, 1])


# ----------------------------------------------------------------------------- P6
@pytest.mark.parametrize("variant", ["gcn", "gcnii", "sage", "resgcn"])
def test_p6_backward_is_the_gradient_of_the_chunked_forward(variant):
    dims = (4, 6, 5, 3) if variant in ("gcn", "sage") else (5, 5, 5, 5)
    w = tiny_workload(n=29, k=4, dims=dims, variant=variant, seed=11)
    p = make_problem(w, chunk_ptr=graphs.ragged_chunks(29, 4, 3), first_stage=False, noise_std=0.3)
    st = p.new_oracle(f64=True)
    st.forward_pass(p.order)
    for dz in st.dZ:  # leftovers of an earlier epoch must be masked out by the zero rule
        dz[...] = 1e3
    st.backward_pass(p.grad_out)
    A = dense_adj(p.row_ptr, p.col, edge_weights(variant, p.row_ptr, p.col, f64=True), p.n)

    # (a) torch autograd on an independent dense formulation
    x0_t = torch.from_numpy(p.x0.astype(np.float64)).requires_grad_(True)
    W_t = [torch.from_numpy(x.astype(np.float64)).requires_grad_(True) for x in p.W]
    b_t = [torch.from_numpy(x.astype(np.float64)).requires_grad_(True) for x in p.b]
    h0_t = None if p.h0 is None else torch.from_numpy(p.h0.astype(np.float64)).requires_grad_(True)
    ln_t = None
    if variant == "resgcn":
        ln_t = ([torch.from_numpy(x.astype(np.float64)).requires_grad_(True) for x in p.ln_gamma],
                [torch.from_numpy(x.astype(np.float64)).requires_grad_(True) for x in p.ln_beta])
    out = torch_dense_chunked(p, A, p.order, x0_t, W_t, b_t, h0_t, ln_t)
    assert np.allclose(out.detach().numpy(), st.cur[p.L], rtol=1e-11, atol=1e-12)
    loss = (out * torch.from_numpy(p.grad_out.astype(np.float64))).sum()
    loss.backward()
    for j in range(p.L):
        assert np.allclose(st.dW[j], W_t[j].grad.numpy(), rtol=1e-9, atol=1e-11), j
        if variant != "gcnii":
            assert np.allclose(st.db[j], b_t[j].grad.numpy(), rtol=1e-9, atol=1e-11), j
    assert np.allclose(st.grad_in, x0_t.grad.numpy(), rtol=1e-9, atol=1e-11)
    if variant == "gcnii":
        assert np.allclose(st.dH0, h0_t.grad.numpy(), rtol=1e-9, atol=1e-11)
    if variant == "resgcn":  # LayerNorm's parameters, including what reaches them through the historical rows
        for j in range(p.L):
            assert np.allclose(st.d_ln_g[j], ln_t[0][j].grad.numpy(), rtol=1e-9, atol=1e-11), j
            assert np.allclose(st.d_ln_b[j], ln_t[1][j].grad.numpy(), rtol=1e-9, atol=1e-11), j

    # (b) central finite differences on the oracle itself, history held constant
    def loss_of(mutate):
        s2 = p.new_oracle(f64=True)
        mutate(s2)
        s2.forward_pass(p.order)
        return float((s2.cur[p.L] * p.grad_out.astype(np.float64)).sum())

    rng = np.random.default_rng(0)
    eps = 1e-6
    for _ in range(6):
        j = int(rng.integers(p.L))
        i, o = int(rng.integers(p.W[j].shape[0])), int(rng.integers(p.dims[j + 1]))

        def bump_w(s2, sgn, j=j, i=i, o=o):
            s2.W[j][i, o] += sgn * eps
        fd = (loss_of(lambda s2: bump_w(s2, +1)) - loss_of(lambda s2: bump_w(s2, -1))) / (2 * eps)
        assert fd == pytest.approx(st.dW[j][i, o], rel=1e-6, abs=1e-7)
        v, c = int(rng.integers(p.n)), int(rng.integers(p.dims[0]))

        def bump_x(s2, sgn, v=v, c=c):
            s2.cur[0][v, c] += sgn * eps
        fd = (loss_of(lambda s2: bump_x(s2, +1)) - loss_of(lambda s2: bump_x(s2, -1))) / (2 * eps)
        assert fd == pytest.approx(st.grad_in[v, c], rel=1e-6, abs=1e-7)


def test_backward_order_is_enforced_and_mask_matters():
    w = tiny_workload(n=29, k=3)
    p = make_problem(w)
    st = p.new_oracle()
    st.forward_pass([2, 0, 1])
    with pytest.raises(AssertionError):
        st.backward_chunk(2, p.grad_out[st.rows(2)])
    st.backward_chunk(1, p.grad_out[st.rows(1)])  # last forwarded chunk goes first


# ----------------------------------------------------------------------------- P7
def test_p7_gcnii_special_cases():
    dims = (6, 6, 6)
    w = tiny_workload(n=37, k=3, dims=dims, variant="gcnii", seed=5)
    p = make_problem(w, first_stage=False)
    # a = 0, beta = 1  ==  GCN without bias
    p.a, p.beta = 0.0, np.ones(2)
    s_ii = run_oracle(p)
    w_gcn = tiny_workload(n=37, k=3, dims=dims, variant="gcn", seed=5)
    pg = make_problem(w_gcn, bias_std=0.0, first_stage=False)
    pg.W, pg.x0, pg.hist, pg.grad_out, pg.order = p.W, p.x0, p.hist, p.grad_out, p.order
    s_g = run_oracle(pg)
    for j in range(1, 3):
        assert np.array_equal(s_ii.cur[j], s_g.cur[j])
    for j in range(2):
        assert np.array_equal(s_ii.dW[j], s_g.dW[j])
    assert np.array_equal(s_ii.grad_in, s_g.grad_in)
    assert not s_ii.dH0.any()
    # beta = 0: no weights involved, dW == 0, output = ReLU((1-a) A h + a h0)
    p.a, p.beta = 0.25, np.zeros(2)
    s0 = run_oracle(p, f64=True)
    assert not s0.dW[0].any() and not s0.dW[1].any()
    A = dense_adj(p.row_ptr, p.col, oracle.gcn_norm(p.row_ptr, p.col, f64=True), p.n)
    one = p.new_oracle(f64=True)
    for j in range(2):
        one.hist[j][...] = 0
    k1 = oracle.OracleStage(p.row_ptr, p.col, oracle.gcn_norm(p.row_ptr, p.col, f64=True), [0, p.n], dims, p.W,
                            variant="gcnii", a=0.25, beta=np.zeros(2), h0=p.h0, f64=True)
    k1.cur[0][...] = p.x0
    k1.forward_pass([0])
    lvl1 = np.maximum(0.75 * (A @ p.x0.astype(np.float64)) + 0.25 * p.h0, 0)
    assert np.allclose(k1.cur[1], lvl1, rtol=1e-12, atol=1e-13)
    assert gcnii_beta(1, 1)[0] == pytest.approx(np.log(1.5))


# ----------------------------------------------------------------------------- bookkeeping
def test_graphsage_special_cases():
    """UPDATE(h_v, z_v) = ReLU(h_v W_self + z_v W_neigh + b) (Equation 1 takes both arguments).
    W_self = 0 is the GCN update on the same edge weights; W_neigh = 0 is a plain MLP that neither the
    graph nor the history can reach."""
    w = tiny_workload(n=37, k=3, dims=(5, 6, 4), variant="sage", seed=5)
    p = make_problem(w, first_stage=False, noise_std=0.3)
    # (a) W_self = 0
    pa = make_problem(w, first_stage=False, noise_std=0.3)
    for j in range(pa.L):
        pa.W[j][:pa.dims[j]] = 0.0
    sa = run_oracle(pa)
    gcn = oracle.OracleStage(pa.row_ptr, pa.col, pa.val, pa.chunk_ptr, pa.dims, [pa.W[j][pa.dims[j]:] for j in range(pa.L)], pa.b)
    gcn.cur[0][...] = pa.x0
    for j in range(pa.L):
        gcn.hist[j][...] = pa.hist[j]
    gcn.forward_pass(pa.order)
    gcn.backward_pass(pa.grad_out)
    for j in range(1, pa.L + 1):
        assert np.array_equal(sa.cur[j], gcn.cur[j])
    for j in range(pa.L):
        assert np.array_equal(sa.dW[j][pa.dims[j]:], gcn.dW[j]) and np.array_equal(sa.db[j], gcn.db[j])
    # the history those runs started from was made by a GraphSage pass, so it differs from zero
    assert np.abs(sa.grad_in - gcn.grad_in).max() <= 1e-6 * np.abs(gcn.grad_in).max()
    assert np.abs(sa.cur[pa.L]).max() > 0
    # (b) W_neigh = 0: rows are independent of each other
    pb = make_problem(w, first_stage=False, noise_std=0.3)
    for j in range(pb.L):
        pb.W[j][pb.dims[j]:] = 0.0
    sb = run_oracle(pb)
    h = pb.x0.astype(np.float64)
    for j in range(pb.L):
        h = np.maximum(h @ pb.W[j][:pb.dims[j]].astype(np.float64) + pb.b[j], 0.0)
    assert max_rel(sb.cur[pb.L], h) < 2e-6
    hist_free = make_problem(w, first_stage=False, noise_std=0.3)
    for j in range(hist_free.L):
        hist_free.W[j][hist_free.dims[j]:] = 0.0
        hist_free.hist[j][...] = 123.0                     # no output may depend on the history
    sc = run_oracle(hist_free)
    assert np.array_equal(sc.cur[pb.L], sb.cur[pb.L]) and np.array_equal(sc.grad_in, sb.grad_in)
    for j in range(pb.L):
        assert np.array_equal(sc.dW[j][:pb.dims[j]], sb.dW[j][:pb.dims[j]])


def test_resgcn_parameter_gradients_do_not_depend_on_asking_for_the_input_gradient():
    """LayerNorm of layer 0 sits in front of the aggregation, so its parameters need the transposed
    aggregation of layer 0 even when nobody wants the gradient of the stage input."""
    w = tiny_workload(n=33, k=3, dims=(6, 6, 6), variant="resgcn", seed=9)
    p = make_problem(w, first_stage=False, noise_std=0.3)
    a = run_oracle(p, need_input_grad=True)
    b = run_oracle(p, need_input_grad=False)
    for j in range(p.L):
        assert np.array_equal(a.d_ln_g[j], b.d_ln_g[j]) and np.array_equal(a.d_ln_b[j], b.d_ln_b[j])
        assert np.array_equal(a.dW[j], b.dW[j]) and np.abs(a.d_ln_g[j]).max() > 0
    assert np.abs(a.grad_in).max() > 0 and np.abs(b.grad_in).max() == 0
    # identity-like special case: W = 0, b = 0 leaves every level equal to the input (pure residual)
    for j in range(p.L):
        p.W[j][...] = 0
        p.b[j][...] = 0
    c = run_oracle(p)
    assert np.array_equal(c.cur[p.L], p.x0)
    assert np.abs(c.grad_in - p.grad_out).max() <= 1e-6 * np.abs(p.grad_out).max()


@pytest.mark.parametrize("f64", [False, True])
def test_the_c_oracles_splitmix64_and_keep_rule_against_the_published_vector(f64):
    """The dropout decisions of the C oracle come from its own copy of SplitMix64's output function.  Pinned to
    the test vector published with the reference implementation (seed 1234567: the state advances by the golden
    gamma, the outputs are the file's values), and the keep rule is pinned to its definition written out with
    Python integers: key_j = out(seed + (j + 1) G), draw = out(key_j + (u d + c + 1) G), keep iff the draw's top
    24 bits reach ceil(p 2^24).  A mistyped mixing constant or shift, a wrong counter or threshold fails here."""
    from oracle.stage import _lib, splitmix64_c
    golden = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "splitmix64_seed1234567.txt")
    want = [int(x) for x in open(golden).read().split("\n") if x and not x.startswith("#")]
    G, M = 0x9E3779B97F4A7C15, (1 << 64) - 1
    got = [splitmix64_c((1234567 + (i + 1) * G) & M, f64=f64) for i in range(len(want))]
    assert got == want

    def out(z):  # the published output function, in Python integers
        z &= M
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M
        return z ^ (z >> 31)

    assert [out(1234567 + (i + 1) * G) for i in range(len(want))] == want   # the definition above is the published one
    lib = _lib(f64)
    rng = np.random.default_rng(3)
    for seed, p in ((7, 0.5), (2**63 + 12345, 0.3), (0, 0.9), (M, 0.125)):
        thr = math.ceil(p * (1 << 24))
        for _ in range(200):
            j, u, d = int(rng.integers(0, 40)), int(rng.integers(0, 10**7)), int(rng.integers(1, 1025))
            c = int(rng.integers(0, d))
            key = out(seed + (j + 1) * G)
            keep = (out(key + (u * d + c + 1) * G) >> 40) >= thr
            assert bool(lib.oracle_dropout_keep(seed, j, u, d, c, p)) == keep, (seed, p, j, u, d, c)


def test_resgcn_dropout():
    """Dropout between ReLU and the convolution of the ResGCN+ block: counter-based keep decisions per
    (layer, vertex, feature), survivors scaled by 1 / (1 - p)."""
    w = tiny_workload(n=31, k=4, dims=(6, 6, 6, 6), variant="resgcn", seed=21)
    chunks = graphs.ragged_chunks(31, 4, 3)
    p0 = make_problem(w, chunk_ptr=chunks, first_stage=False, noise_std=0.3)
    pz = make_problem(w, chunk_ptr=chunks, first_stage=False, noise_std=0.3, dropout_p=0.0, dropout_seed=99)
    a, b = run_oracle(p0), run_oracle(pz)
    assert np.array_equal(a.cur[p0.L], b.cur[p0.L]) and np.array_equal(a.grad_in, b.grad_in)   # rate 0 is no dropout
    # keep decisions: a fair, repeatable coin per element that depends on seed and layer
    big = oracle.OracleStage(p0.row_ptr, p0.col, p0.val, p0.chunk_ptr, [64, 64, 64], [np.zeros((64, 64))] * 2,
                             variant="resgcn", dropout_p=0.4)
    masks = {}
    for seed in (1, 2):
        big.set_dropout_seed(seed)
        for j in range(2):
            masks[seed, j] = big.dropout_keep_mask(j)
    m = masks[1, 0]
    assert set(np.unique(m)) == {0.0, 1.0} and abs(m.mean() - 0.6) < 4 * np.sqrt(0.24 / m.size)
    assert abs(np.corrcoef(m[:, :-1].ravel(), m[:, 1:].ravel())[0, 1]) < 0.08
    big.set_dropout_seed(1)
    assert np.array_equal(big.dropout_keep_mask(0), m)
    for other in ((1, 1), (2, 0)):
        assert 0.3 < np.mean(masks[other] != m) < 0.7
    # forward and every gradient against autograd on the dense chunked model, the keep decisions as an input
    p = make_problem(w, chunk_ptr=chunks, first_stage=False, noise_std=0.3, dropout_p=0.5, dropout_seed=7)
    st = p.new_oracle(f64=True)
    st.forward_pass(p.order)
    st.backward_pass(p.grad_out)
    drop = [torch.from_numpy(st.dropout_keep_mask(j)) for j in range(p.L)]
    assert 0.3 < float(drop[0].mean()) < 0.7
    A = dense_adj(p.row_ptr, p.col, edge_weights("resgcn", p.row_ptr, p.col, f64=True), p.n)
    x0_t = torch.from_numpy(p.x0.astype(np.float64)).requires_grad_(True)
    W_t = [torch.from_numpy(x.astype(np.float64)).requires_grad_(True) for x in p.W]
    b_t = [torch.from_numpy(x.astype(np.float64)).requires_grad_(True) for x in p.b]
    ln_t = ([torch.from_numpy(x.astype(np.float64)).requires_grad_(True) for x in p.ln_gamma],
            [torch.from_numpy(x.astype(np.float64)).requires_grad_(True) for x in p.ln_beta])
    out = torch_dense_chunked(p, A, p.order, x0_t, W_t, b_t, None, ln_t, drop)
    assert np.allclose(out.detach().numpy(), st.cur[p.L], rtol=1e-11, atol=1e-12)
    (out * torch.from_numpy(p.grad_out.astype(np.float64))).sum().backward()
    for j in range(p.L):
        assert np.allclose(st.dW[j], W_t[j].grad.numpy(), rtol=1e-9, atol=1e-11)
        assert np.allclose(st.d_ln_g[j], ln_t[0][j].grad.numpy(), rtol=1e-9, atol=1e-11)
        assert np.allclose(st.d_ln_b[j], ln_t[1][j].grad.numpy(), rtol=1e-9, atol=1e-11)
    assert np.allclose(st.grad_in, x0_t.grad.numpy(), rtol=1e-9, atol=1e-11)
    # the decisions belong to (vertex, feature), not to the chunking: with the full-graph levels as history
    # every chunking of the same seed gives the full-graph result
    full = make_problem(w, chunk_ptr=np.array([0, 31]), first_stage=False, dropout_p=0.5, dropout_seed=7)
    sf = full.new_oracle(f64=True)
    sf.forward_pass([0])
    for j in range(p.L):
        p.hist[j] = sf.cur[j].copy()
    sc = p.new_oracle(f64=True)
    sc.forward_pass(p.order)
    assert np.allclose(sc.cur[p.L], sf.cur[p.L], rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("variant", ["gcn", "sage"])
def test_output_dropout_of_gcn_and_sage_layers(variant):
    """Dropout on the output of a GCN / GraphSage layer: what is stored, and read later as current or historical
    embedding, is the value after dropout; the gradient of a surviving element carries 1 / (1 - p)."""
    w = tiny_workload(n=31, k=4, dims=(6, 5, 7, 4), variant=variant, seed=23)
    chunks = graphs.ragged_chunks(31, 4, 3)
    p0 = make_problem(w, chunk_ptr=chunks, first_stage=False, noise_std=0.3)
    pz = make_problem(w, chunk_ptr=chunks, first_stage=False, noise_std=0.3, dropout_p=0.0, dropout_seed=99)
    a, b = run_oracle(p0), run_oracle(pz)
    assert np.array_equal(a.cur[p0.L], b.cur[p0.L]) and np.array_equal(a.grad_in, b.grad_in)   # rate 0 is no dropout
    # forward and every gradient against autograd on the dense chunked model, the keep decisions as an input
    p = make_problem(w, chunk_ptr=chunks, first_stage=False, noise_std=0.3, dropout_p=0.5, dropout_seed=11)
    st = p.new_oracle(f64=True)
    st.forward_pass(p.order)
    st.backward_pass(p.grad_out)
    drop = [torch.from_numpy(st.dropout_keep_mask(j)) for j in range(p.L)]
    assert [tuple(m.shape) for m in drop] == [(p.n, d) for d in p.dims[1:]] and 0.3 < float(drop[0].mean()) < 0.7
    for j in range(p.L):  # dropped elements are stored as zeros, survivors are positive or were zero before
        assert np.all(st.cur[j + 1][drop[j].numpy() == 0] == 0)
    A = dense_adj(p.row_ptr, p.col, edge_weights(variant, p.row_ptr, p.col, f64=True), p.n)
    x0_t = torch.from_numpy(p.x0.astype(np.float64)).requires_grad_(True)
    W_t = [torch.from_numpy(x.astype(np.float64)).requires_grad_(True) for x in p.W]
    b_t = [torch.from_numpy(x.astype(np.float64)).requires_grad_(True) for x in p.b]
    out = torch_dense_chunked(p, A, p.order, x0_t, W_t, b_t, None, None, drop)
    assert np.allclose(out.detach().numpy(), st.cur[p.L], rtol=1e-11, atol=1e-12)
    (out * torch.from_numpy(p.grad_out.astype(np.float64))).sum().backward()
    for j in range(p.L):
        assert np.allclose(st.dW[j], W_t[j].grad.numpy(), rtol=1e-9, atol=1e-11)
        assert np.allclose(st.db[j], b_t[j].grad.numpy(), rtol=1e-9, atol=1e-11)
    assert np.allclose(st.grad_in, x0_t.grad.numpy(), rtol=1e-9, atol=1e-11)
    # unbiased: over many seeds the mean of one layer's output is the output without dropout
    one = tiny_workload(n=31, k=1, dims=(6, 5), variant=variant, seed=23)
    base = run_oracle(make_problem(one, first_stage=False, noise_std=0.3)).cur[1].astype(np.float64)
    acc = np.zeros_like(base)
    seeds = 400
    for seed in range(seeds):
        acc += run_oracle(make_problem(one, first_stage=False, noise_std=0.3, dropout_p=0.5, dropout_seed=seed)).cur[1]
    err = np.abs(acc / seeds - base)
    assert np.all(err <= 5.0 * base / np.sqrt(seeds) + 1e-6)   # survivors are 2 x base with probability 1/2: std = base


def test_transposed_index_round_trip_and_push_pull():
    rng = np.random.default_rng(3)
    n = 23
    dst, src = rng.integers(0, n, 90), rng.integers(0, n, 90)
    row_ptr, col = graphs.from_directed_pairs(n, np.concatenate([dst, np.arange(n)]), np.concatenate([src, np.arange(n)]))
    val = oracle.gcn_norm(row_ptr, col)
    st = oracle.OracleStage(row_ptr, col, val, [0, 7, 15, n], [3, 2], [np.ones((3, 2), np.float32)])
    # transposing twice gives the CSR back; t_edge points at the same (row, col) entry
    pairs = sorted((int(st.t_row[p]), u) for u in range(n) for p in range(st.t_ptr[u], st.t_ptr[u + 1]))
    csr_pairs = [(v, int(col[e])) for v in range(n) for e in range(row_ptr[v], row_ptr[v + 1])]
    assert pairs == csr_pairs
    for u in range(n):
        for p in range(st.t_ptr[u], st.t_ptr[u + 1]):
            e = st.t_edge[p]
            assert col[e] == u and row_ptr[st.t_row[p]] <= e < row_ptr[st.t_row[p] + 1]
    # backward pull over the transposed index == brute-force push over CSR rows with the zero rule
    st.cur[0][...] = rng.random((n, 3)).astype(np.float32) + 0.5
    st.hist[0][...] = st.cur[0]
    order = [1, 2, 0]
    st.forward_pass(order)
    gout = rng.standard_normal((n, 2)).astype(np.float32)
    st.backward_pass(gout)
    chunk_of = st.chunk_of
    pos = {c: i for i, c in enumerate(order)}
    want = np.zeros((n, 3))
    for v in range(n):
        for e in range(row_ptr[v], row_ptr[v + 1]):
            u = col[e]
            # v contributes to u iff v's chunk was processed at or after u's chunk in the forward pass
            if pos[chunk_of[v]] >= pos[chunk_of[u]]:
                want[u] += float(val[e]) * st.dZ[0][v].astype(np.float64)
    assert np.allclose(st.grad_in, want, rtol=1e-6, atol=1e-7)


def test_select_counts_brute_force():
    w = tiny_workload(n=61, k=5)
    p = make_problem(w, chunk_ptr=graphs.ragged_chunks(61, 5, 8))
    st = p.new_oracle()
    st.begin_pass()
    done = set()
    for k in [3, 0, 4, 1, 2]:
        got = st.select_counts(k)
        want = [sum(1 for e in range(p.row_ptr[v], p.row_ptr[v + 1])
                    if st.chunk_of[p.col[e]] in done | {k}) for v in range(*st.rows(k).indices(61)[:2])]
        assert np.array_equal(got, want)
        st.forward_chunk(k)
        done.add(k)
    assert sum(int(st.select_counts(k).sum()) for k in range(5)) == p.row_ptr[-1]  # all processed => every edge


def test_quantised_storage_is_torch_bf16_rounding():
    w = Workload("q", "er", 64, 21, [8, 8, 8], 2, dtype="bf16", avg_degree=5.0)
    p = make_problem(w)
    st = run_oracle(p)
    for arr in st.cur[1:] + st.Z + st.dZ + [st.grad_in]:
        bits = np.ascontiguousarray(arr).view(np.uint32)
        assert not (bits & 0xFFFF).any()
    # rounding rule itself: recompute one stored row in fp64 and round with torch
    v = 5
    z = np.zeros(8)
    for e in range(p.row_ptr[v], p.row_ptr[v + 1]):
        u = p.col[e]
        src = st.cur[0] if True else None
        z += float(p.val[e]) * (st.cur[0][u] if st.chunk_of[u] == st.chunk_of[v] or
                                list(p.order).index(st.chunk_of[u]) < list(p.order).index(st.chunk_of[v])
                                else p.hist[0][u]).astype(np.float64)
    want = torch.tensor(z, dtype=torch.float64).to(torch.float32).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(st.Z[0][v], want)


def test_update_history_copies_levels():
    w = tiny_workload(n=31, k=2)
    p = make_problem(w)
    st = run_oracle(p)
    st.update_history()
    for j in range(p.L):
        assert np.array_equal(st.hist[j], st.cur[j])
    # a second pass with refreshed history and the same weights reproduces the full-graph result
    # only if the first pass was exact; it is not (staleness), so levels move:
    before = st.cur[p.L].copy()
    st.forward_pass(p.order)
    assert not np.array_equal(before, st.cur[p.L])
