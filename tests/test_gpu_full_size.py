"""GPU parity at the sizes the benchmark definition names for its two largest graphs, in the launch
configuration bench.py times (first stage: level-0 history is the feature buffer itself, no input gradient,
weights computed by the library), against the CPU oracle on the same seeded inputs.

configs[2] (2.45 M vertices, 16 chunks, 8 layers): one complete forward pass and one complete backward pass.
configs[4] (10 M vertices, 32 chunks, 4 layers of width 256; a level is 5.12 GB, so row offsets pass 2^32 bytes
from vertex 8.4 M on): the oracle cannot afford a whole pass, so the chunks at both ends of a pass are compared
in full - see test_full_size_c4_chunks_at_both_ends_of_a_pass.

The level tables of these two tests are drawn on the device by torch's seeded generator (the numpy generator
of synth.values needs minutes for 10^10 values) and copied to the host for the oracle: inputs, nothing the
library computed.  Tolerance 1e-2 per tensor (max |x - ref| / max |ref|), as for every bf16 stage.
"""
import ctypes
import os
import time

import numpy as np
import pytest
import torch

import oracle
from synth import values
from synth.configs import CONFIGS, make_graph
from synth.graphs import equal_chunks

from helpers import max_rel, to_bf16_grid

pytestmark = pytest.mark.gpu

TOL_BF16 = 1e-2
DEV = "cuda:0"


def _progress(msg):
    """A line per step into the run's output folder (a test here runs for minutes, and a long silence reads as a hang)."""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    try:
        os.makedirs(os.path.join(root, "gpurun_out"), exist_ok=True)
        with open(os.path.join(root, "gpurun_out", "full_size_progress.log"), "a") as f:
            f.write(f"{time.strftime('%H:%M:%S')} {msg}\n")
    except OSError:
        pass


class _Case:
    """configs[name] as bench.py builds it, with random (not clean-pass) level tables S_j: hist[j] = S_j on both
    sides; cur[j] starts as a copy of S_j on the GPU."""

    def __init__(self, name):
        import paper_2308_10087_amd as g
        w = self.w = CONFIGS[name]
        assert w.variant == "gcn" and w.dtype == "bf16"
        _progress(f"{name}: building the graph")
        self.row_ptr, self.col = make_graph(w)
        n = self.n = len(self.row_ptr) - 1
        K, dims = w.n_chunks, list(w.dims)
        L = self.L = len(dims) - 1
        self.K, self.dims = K, dims
        self.chunk_ptr = equal_chunks(n, K)
        self.Wn = [to_bf16_grid(values.glorot_uniform(w.seed, 100 + j, dims[j], dims[j + 1])) for j in range(L)]
        self.bn = [values.normal(w.seed, 200 + j, (dims[j + 1],), 0.05) for j in range(L)]
        gen = torch.Generator(device=DEV)
        gen.manual_seed(w.seed)
        self.gen = gen
        l0 = torch.float32 if w.level0_f32 else torch.bfloat16
        # level 0: features ~ N(0, 1); levels >= 1: |N(0, 1)|, like post-ReLU embeddings
        self.S = [torch.randn((n, dims[0]), generator=gen, device=DEV).to(l0)]
        for j in range(1, L):
            self.S.append(torch.randn((n, dims[j]), generator=gen, device=DEV).abs_().to(torch.bfloat16))
        self.cur = [self.S[0]] + [self.S[j].clone() for j in range(1, L)] + \
                   [torch.zeros((n, dims[L]), dtype=torch.bfloat16, device=DEV)]
        self.hist = list(self.S)
        self.W = [torch.from_numpy(x).to(DEV, torch.bfloat16) for x in self.Wn]
        self.bias = [torch.from_numpy(x).to(DEV) for x in self.bn]
        self.dW = [torch.zeros((dims[j], dims[j + 1]), device=DEV) for j in range(L)]
        self.dbias = [torch.zeros(dims[j + 1], device=DEV) for j in range(L)]
        _progress(f"{name}: gnnstage_create")
        self.stage = g.GnnStage(self.row_ptr, self.col, self.chunk_ptr, dims, W=self.W, cur=self.cur, hist=self.hist,
                                dW=self.dW, bias=self.bias, dbias=self.dbias, edge_val=None, variant=g.GNNSTAGE_GCN,
                                dtype=g.GNNSTAGE_BF16, level0_f32=w.level0_f32, grad_in=None, device=DEV)
        _progress(f"{name}: oracle set-up")
        val = oracle.gcn_norm(self.row_ptr, self.col)
        st = self.ref = oracle.OracleStage(self.row_ptr, self.col, val, self.chunk_ptr, dims, self.Wn, self.bn,
                                           variant="gcn", quant=True, level0_f32=w.level0_f32)
        for j in range(L):
            # one host array serves as the oracle's current AND historical level j: a row is read as current only
            # once its chunk counts as processed, and what the oracle computes only ever lands in such rows
            a = self.S[j].to(torch.float32).cpu().numpy()
            st.cur[j] = a
            st.hist[j] = a
        st._refresh()

    def rows(self, k):
        return slice(int(self.chunk_ptr[k]), int(self.chunk_ptr[k + 1]))

    def check_levels(self, k, where):
        """Rows of chunk k at every level the stage wrote, element by element."""
        r = self.rows(k)
        for j in range(1, self.L + 1):
            a = self.cur[j][r].to(torch.float32).cpu().numpy()
            b = self.ref.cur[j][r]
            err = max_rel(a, b)
            assert err <= TOL_BF16, (where, k, j, err)
            flips = (a > 0) != (b > 0)   # ReLU decisions may differ at near-ties only
            self.flip_share = max(getattr(self, "flip_share", 0.0), float(flips.mean()))
            self.worst = max(getattr(self, "worst", 0.0), err)
            assert flips.mean() <= 1e-3, (where, k, j, float(flips.mean()))
            if flips.any():
                assert np.maximum(np.abs(a[flips]), np.abs(b[flips])).max() <= TOL_BF16 * np.abs(b).max(), (where, k, j)

    def force_levels(self, k):
        """Both sides decide the ReLU derivatives of the backward pass on the same (the oracle's) level values."""
        r = self.rows(k)
        for j in range(1, self.L + 1):
            self.cur[j][r].copy_(torch.from_numpy(self.ref.cur[j][r]).to(torch.bfloat16))

    def check_grads(self, where, layers=None):
        for j in (range(self.L) if layers is None else layers):
            e = max_rel(self.dW[j].cpu().numpy(), self.ref.dW[j])
            assert e <= TOL_BF16, (where, f"dW{j}", e)
            e = max_rel(self.dbias[j].cpu().numpy(), self.ref.db[j])
            assert e <= TOL_BF16, (where, f"db{j}", e)


def test_full_size_c2_one_complete_pass():
    """configs[2] at full size: forward over all 16 chunks (shuffled order), every level of every vertex; then the
    backward pass over all 16 chunks, every weight and bias gradient of the 8 layers (layer 0 runs
    transform-first, its weight gradient is complete only after the last backward call)."""
    c = _Case("c2")
    order = [int(k) for k in values.permutation(c.w.seed, 4, c.K)]
    grad_out = torch.randn((c.n, c.dims[-1]), generator=c.gen, device=DEV).to(torch.bfloat16)
    _progress("c2: oracle forward pass")
    c.ref.begin_pass()
    for k in order:
        c.ref.forward_chunk(k)
    _progress("c2: GPU forward pass")
    c.stage.forward_pass(order)
    torch.cuda.synchronize()
    for k in order:
        c.check_levels(k, "forward")
    for k in order:
        c.force_levels(k)
    _progress("c2: oracle backward pass")
    g_host = grad_out.to(torch.float32).cpu().numpy()
    c.ref.backward_pass(g_host, need_input_grad=False)
    _progress("c2: GPU backward pass")
    c.stage.backward_pass(order, grad_out)
    torch.cuda.synchronize()
    c.check_grads("backward")
    _progress(f"c2: done; worst level error {c.worst:.2e}, largest share of differing ReLU decisions {c.flip_share:.2e}")


def test_full_size_c4_chunks_at_both_ends_of_a_pass():
    """configs[4] at full size.  A pass over all 32 chunks in the order (3, 29 others, 7, 31):

    * chunk 3 comes first: every neighbour outside it is read from the HISTORICAL tables, rows up to vertex 10 M
      (byte offsets up to 5.1 GB);
    * the 29 chunks in between run on the GPU only; afterwards the test puts the table values S_j back into their
      rows of the caller-owned current levels, so that the oracle - which marks them processed without computing
      them - sees the same current rows;
    * chunk 7 is last but one: everything but chunk 31 is read from the CURRENT tables;
    * chunk 31 (vertices 9.69 M .. 10 M: every row it reads and writes of its own lies beyond 2^32 bytes) is
      last: no historical read at all.

    Every level of the rows of chunks 3, 7 and 31 is compared.  Then the backward calls of chunks 31 and 7 (the
    first two of the reverse order; chunk 7 gathers gradient rows of chunk 31, nothing flows from the other 30):
    weight and bias gradients of all four layers after the two calls."""
    c = _Case("c4")
    first, before_last, last = 3, 7, 31
    middle = [k for k in range(c.K) if k not in (first, before_last, last)]
    order = [first] + middle + [before_last, last]
    st = c.ref
    _progress("c4: first chunk of the pass")
    st.begin_pass()
    st.forward_chunk(first)
    c.stage.stage_forward_chunk(first, 0)
    torch.cuda.synchronize()
    c.check_levels(first, "first chunk")
    _progress("c4: chunks in between (GPU only)")
    for pos, k in enumerate(middle, start=1):
        c.stage.stage_forward_chunk(k, pos)
    torch.cuda.synchronize()
    for k in middle:
        r = c.rows(k)
        st.processed[k] = 1
        for j in range(1, c.L):
            c.cur[j][r].copy_(c.S[j][r])
    _progress("c4: last two chunks of the pass")
    for pos, k in ((c.K - 2, before_last), (c.K - 1, last)):
        st.forward_chunk(k)
        c.stage.stage_forward_chunk(k, pos)
        torch.cuda.synchronize()
        c.check_levels(k, "end of the pass")
    _progress("c4: backward calls of the last two chunks")
    for k in (last, before_last):
        c.force_levels(k)
    for k in (last, before_last):
        m = int(c.chunk_ptr[k + 1] - c.chunk_ptr[k])
        g_dev = torch.randn((m, c.dims[-1]), generator=c.gen, device=DEV).to(torch.bfloat16)
        g_host = np.ascontiguousarray(g_dev.to(torch.float32).cpu().numpy())
        st.lib.oracle_backward_chunk(ctypes.byref(st._cs), k, g_host.ctypes.data, 0)
        c.stage.stage_backward_chunk(k, g_dev)
        # the pass stops here: have the weight gradients of the calls made so far now (the library would take
        # them in one product per layer after the last call of the pass)
        c.stage.gnnstage_flush_weight_gradients()
        torch.cuda.synchronize()
        c.check_grads(f"backward call of chunk {k}")
    assert order[-2:] == [before_last, last]
    _progress(f"c4: done; worst level error {c.worst:.2e}, largest share of differing ReLU decisions {c.flip_share:.2e}")
