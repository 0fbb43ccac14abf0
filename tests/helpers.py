"""Shared test scaffolding: turns a workload recipe into concrete seeded arrays and an
oracle instance.  Inputs come from ``synth`` (structure + random values); edge weights and
every expected value come from ``oracle`` only."""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch

import oracle
from synth import graphs, values
from synth.configs import Workload, make_graph


def edge_weights(variant: str, row_ptr: np.ndarray, col: np.ndarray, f64: bool = False) -> np.ndarray:
    """The aggregator's per-edge weights handed to oracle and library alike: the GCN normalisation of
    Section 2.1 (from the oracle), or, for the GraphSage variant, the mean aggregator's 1 / |N(v)| on every
    entry of row v (an input: a plain reciprocal of the row length)."""
    if variant != "sage":
        return oracle.gcn_norm(row_ptr, col, f64=f64)
    deg = np.diff(row_ptr).astype(np.float64)
    w = np.repeat(1.0 / np.maximum(deg, 1.0), np.diff(row_ptr))
    return w if f64 else w.astype(np.float32)


def to_bf16_grid(x: np.ndarray) -> np.ndarray:
    """Nearest bf16-representable fp32 values (library rounding, used to make INPUTS exact in bf16)."""
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16).to(torch.float32).numpy()


@dataclass
class Problem:
    w: Workload
    row_ptr: np.ndarray
    col: np.ndarray
    val: np.ndarray
    chunk_ptr: np.ndarray
    dims: List[int]
    W: List[np.ndarray]
    b: List[np.ndarray]
    x0: np.ndarray
    hist: List[np.ndarray]
    grad_out: np.ndarray
    order: np.ndarray
    h0: Optional[np.ndarray] = None
    a: float = 0.0
    beta: Optional[np.ndarray] = None
    quant: bool = False
    level0_f32: bool = False
    ln_gamma: Optional[List[np.ndarray]] = None   # ResGCN+ only
    ln_beta: Optional[List[np.ndarray]] = None
    dropout_p: float = 0.0                        # ResGCN+: inside the block; GCN, GraphSage: on every layer's output
    dropout_seed: int = 0

    @property
    def n(self):
        return self.row_ptr.shape[0] - 1

    @property
    def L(self):
        return len(self.dims) - 1

    def new_oracle(self, f64: bool = False) -> "oracle.OracleStage":
        st = oracle.OracleStage(self.row_ptr, self.col,
                                self.val if not f64 else edge_weights(self.w.variant, self.row_ptr, self.col, f64=True),
                                self.chunk_ptr, self.dims, self.W, self.b,
                                variant=self.w.variant, a=self.a, beta=self.beta, h0=self.h0,
                                quant=self.quant and not f64, level0_f32=self.level0_f32, f64=f64,
                                ln_gamma=self.ln_gamma, ln_beta=self.ln_beta, dropout_p=self.dropout_p)
        st.set_dropout_seed(self.dropout_seed)
        st.cur[0][...] = self.x0
        for j in range(self.L):
            st.hist[j][...] = self.hist[j]
        return st


def gcnii_beta(first_layer: int, n_layers: int) -> np.ndarray:
    """beta_l = ln(0.5 / l + 1), l = global 1-based layer index (benchmark definition)."""
    return np.array([math.log(0.5 / l + 1.0) for l in range(first_layer, first_layer + n_layers)], dtype=np.float64)


def make_problem(w: Workload, *, graph=None, chunk_ptr=None, order=None, bias_std: float = 0.1,
                 first_stage: Optional[bool] = None, shuffle: bool = True, noise_std: float = 0.01,
                 history: str = "clean", dropout_p: float = 0.0, dropout_seed: int = 0) -> Problem:
    row_ptr, col = graph if graph is not None else make_graph(w)
    n = row_ptr.shape[0] - 1
    val = edge_weights(w.variant, row_ptr, col)
    if chunk_ptr is None:
        chunk_ptr = graphs.equal_chunks(n, w.n_chunks)
    K = chunk_ptr.shape[0] - 1
    dims = list(w.dims)
    L = len(dims) - 1
    quant = w.dtype == "bf16"
    if first_stage is None:
        first_stage = w.variant in ("gcn", "sage", "resgcn")
    g = to_bf16_grid if quant else (lambda x: x)
    g0 = (lambda x: x) if (w.level0_f32 or not quant) else to_bf16_grid
    W = [g(values.glorot_uniform(w.seed, 100 + j, dims[j], dims[j + 1])) for j in range(L)]
    if w.variant == "sage":  # [W_self ; W_neigh]
        W = [np.concatenate([g(values.glorot_uniform(w.seed, 150 + j, dims[j], dims[j + 1])), W[j]], axis=0) for j in range(L)]
    ln_gamma = ln_beta = None
    if w.variant == "resgcn":  # LayerNorm parameters away from their trivial initial values
        ln_gamma = [(1.0 + values.normal(w.seed, 400 + j, (dims[j],), 0.1)).astype(np.float32) for j in range(L)]
        ln_beta = [values.normal(w.seed, 450 + j, (dims[j],), 0.1) for j in range(L)]
    if w.variant in ("gcn", "sage", "resgcn"):
        b = [values.normal(w.seed, 200 + j, (dims[j + 1],), bias_std) if bias_std > 0
             else np.zeros(dims[j + 1], np.float32) for j in range(L)]
        x0 = g0(values.normal(w.seed, 1, (n, dims[0])))
        h0, a, beta = None, 0.0, None
    else:
        b = [np.zeros(dims[j + 1], np.float32) for j in range(L)]
        x0 = g0(values.half_normal(w.seed, 1, (n, dims[0])))
        h0 = g(values.normal(w.seed, 2, (n, dims[0])))
        a, beta = w.gcnii_alpha, gcnii_beta(w.gcnii_first_layer, L)
    grad_out = g(values.normal(w.seed, 3, (n, dims[-1])))
    if order is None:
        order = values.permutation(w.seed, 4, K) if shuffle else np.arange(K, dtype=np.int32)
    # historical buffers: a clean full-graph pass (one chunk => no staleness) plus N(0, noise_std^2);
    # history="random" skips the pass (full-size graphs): |N(0,1)| rows, like post-ReLU embeddings
    clean = None
    if history == "clean":
        clean = oracle.OracleStage(row_ptr, col, val, np.array([0, n], dtype=np.int64), dims, W, b,
                                   variant=w.variant, a=a, beta=beta, h0=h0, quant=quant, level0_f32=w.level0_f32,
                                   ln_gamma=ln_gamma, ln_beta=ln_beta)
        clean.cur[0][...] = x0
        clean.forward_pass([0])
    hist = []
    for j in range(L):
        if j == 0 and first_stage:
            hist.append(x0.copy())
        elif clean is None:
            hj = values.half_normal(w.seed, 300 + j, (n, dims[j]))
            hist.append(g0(hj) if j == 0 else g(hj))
        else:
            hj = clean.cur[j] + values.normal(w.seed, 300 + j, (n, dims[j]), noise_std)
            hist.append(g0(hj) if j == 0 else g(hj))
    return Problem(w, row_ptr, col, val, np.asarray(chunk_ptr, dtype=np.int64), dims, W, b, x0, hist, grad_out,
                   np.asarray(order, dtype=np.int32), h0=h0, a=a, beta=beta, quant=quant,
                   level0_f32=w.level0_f32 and quant, ln_gamma=ln_gamma, ln_beta=ln_beta,
                   dropout_p=dropout_p, dropout_seed=dropout_seed)


def run_oracle(p: Problem, need_input_grad: bool = True, f64: bool = False):
    st = p.new_oracle(f64=f64)
    st.forward_pass(p.order)
    st.backward_pass(p.grad_out, need_input_grad)
    return st


def max_rel(x: np.ndarray, ref: np.ndarray) -> float:
    """Per-tensor error measure used by every floating-point parity check:
    max |x - ref| / max |ref| (relative error is undefined at the zeros ReLU produces)."""
    ref = np.asarray(ref, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    denom = float(np.max(np.abs(ref))) if ref.size else 1.0
    if denom == 0.0:
        denom = 1.0
    return float(np.max(np.abs(x - ref))) / denom if ref.size else 0.0


# ---------------------------------------------------------------- training loop (epoch driver) problems
@dataclass
class TrainProblem:
    row_ptr: np.ndarray
    col: np.ndarray
    val: np.ndarray
    chunk_ptr: np.ndarray
    stage_dims: List[List[int]]      # one width list per stage; last width of a stage = first of the next
    W: List[List[np.ndarray]]
    b: List[List[np.ndarray]]
    x0: np.ndarray
    labels: np.ndarray
    mask: Optional[np.ndarray]
    head_W: np.ndarray
    head_b: np.ndarray
    quant: bool
    n_classes: int
    variants: Optional[List[str]] = None        # per stage: "gcn" (default), "sage", "resgcn"
    ln_gamma: Optional[List[List[np.ndarray]]] = None
    ln_beta: Optional[List[List[np.ndarray]]] = None
    dropout_p: float = 0.0                      # of the ResGCN+ stages, and ...
    dropout_everywhere: bool = False            # ... of the GCN / GraphSage stages too, except the last stage

    def stage_dropout(self, si: int) -> float:
        if self.variant(si) == "resgcn":
            return self.dropout_p
        return self.dropout_p if self.dropout_everywhere and si < len(self.stage_dims) - 1 else 0.0

    @property
    def n(self):
        return self.row_ptr.shape[0] - 1

    def variant(self, si: int) -> str:
        return "gcn" if self.variants is None else self.variants[si]


def make_train_problem(*, n=1500, n_classes=5, stage_dims=((24, 16, 16),), K=4, dtype="f32", seed=2308100900,
                       deg_in=8.0, deg_out=2.0, signal=0.6, label_rate=0.5, ragged=False, variants=None) -> TrainProblem:
    """A synthetic node-classification task on a planted-partition graph (labels = planted groups)."""
    row_ptr, col, group = graphs.planted_partition(n, n_classes, deg_in, deg_out, seed)
    val = oracle.gcn_norm(row_ptr, col)
    chunk_ptr = graphs.ragged_chunks(n, K, seed) if ragged else graphs.equal_chunks(n, K)
    quant = dtype == "bf16"
    stage_dims = [list(d) for d in stage_dims]
    x0 = values.group_features(seed, 1, group, stage_dims[0][0], signal)
    W, b, stream = [], [], 100
    ln_gamma, ln_beta = [], []
    for si, dims in enumerate(stage_dims):
        var = "gcn" if variants is None else variants[si]
        Ws = [values.glorot_uniform(seed, stream + j, dims[j], dims[j + 1]) for j in range(len(dims) - 1)]
        if var == "sage":  # [W_self ; W_neigh]
            Ws = [np.concatenate([values.glorot_uniform(seed, stream + 10 + j, dims[j], dims[j + 1]), Ws[j]], axis=0)
                  for j in range(len(dims) - 1)]
        W.append(Ws)
        b.append([np.zeros(dims[j + 1], np.float32) for j in range(len(dims) - 1)])
        ln_gamma.append([np.ones(dims[j], np.float32) for j in range(len(dims) - 1)])
        ln_beta.append([np.zeros(dims[j], np.float32) for j in range(len(dims) - 1)])
        stream += 20
    d_last = stage_dims[-1][-1]
    head_W = values.glorot_uniform(seed, 900, d_last, n_classes)
    head_b = np.zeros(n_classes, np.float32)
    mask = values.bernoulli_mask(seed, 5, n, label_rate) if label_rate < 1.0 else None
    return TrainProblem(row_ptr, col, val, np.asarray(chunk_ptr, np.int64), stage_dims, W, b, x0,
                        group.astype(np.int32), mask, head_W, head_b, quant, n_classes,
                        variants=None if variants is None else list(variants), ln_gamma=ln_gamma, ln_beta=ln_beta)


def new_oracle_trainer(tp: TrainProblem, f64: bool = False, **opt):
    """Oracle stages (history starts at zero; the first stage's level-0 history is the features) + trainer."""
    from oracle.train import OracleTrainer
    stages = []
    val = tp.val if not f64 else oracle.gcn_norm(tp.row_ptr, tp.col, f64=True)
    for si, dims in enumerate(tp.stage_dims):
        var = tp.variant(si)
        st = oracle.OracleStage(tp.row_ptr, tp.col, val, tp.chunk_ptr, dims, tp.W[si], tp.b[si], variant=var,
                                quant=tp.quant and not f64,
                                level0_f32=(si == 0 and tp.quant and not f64 and var != "resgcn"), f64=f64,
                                ln_gamma=tp.ln_gamma[si], ln_beta=tp.ln_beta[si],
                                dropout_p=tp.stage_dropout(si))
        if si == 0:
            st.cur[0][...] = tp.x0
            st.hist[0][...] = tp.x0
        stages.append(st)
    return OracleTrainer(stages, tp.head_W, tp.head_b, tp.labels, tp.mask, quant=tp.quant and not f64, **opt)
