"""CPU oracle of the training loop around the stage (TEST INFRASTRUCTURE ONLY).

Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline`` leg may import
this module.  Plain numpy in fp64, one step per line of the method:

* Algorithm 1: per epoch, every chunk goes through all layers (all stages, first to last), the
  backward pass follows, then the weights are updated (its last line is the plain gradient step;
  Section 5 trains with Adam, learning rate 0.001).
* Section 3.4, technique 1: the chunk order is shuffled at the beginning of every epoch.
* Section 3.4, technique 2: epoch t (1-based) reads the historical embeddings of epoch
  alpha * floor((t - 1) / alpha), i.e. the buffers are refreshed after the epochs alpha, 2 alpha, ...
* The paper does not print its loss; the reading taken here is the usual node-classification head:
  a linear classifier on the last level and the mean softmax cross-entropy over the labelled vertices.
* Adam follows Algorithm 1 of Kingma & Ba (2015), with the optional L2 term added to the gradient.

The stage arithmetic itself is ``oracle.stage.OracleStage``.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np

from .stage import OracleStage

_M64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15


def splitmix64(x: int) -> int:
    """Output function of the SplitMix64 generator (Steele, Lea, Flood 2014) for the state ``x``."""
    z = x & _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def chunk_order(seed: int, epoch: int, K: int, shuffle: bool = True) -> np.ndarray:
    """Section 3.4, technique 1.  Epoch ``epoch`` (0-based) owns the SplitMix64 stream that starts at state
    ``seed + (epoch + 1) * golden``; draw i is the output for state ``start + (i + 1) * golden``.  A
    Fisher-Yates pass from the top swaps position i with position ``draw mod (i + 1)``."""
    order = np.arange(K, dtype=np.int32)
    if not shuffle:
        return order
    start = (seed + (epoch + 1) * _GOLDEN) & _M64
    for n, i in enumerate(range(K - 1, 0, -1)):
        r = splitmix64(start + (n + 1) * _GOLDEN)
        j = r % (i + 1)
        order[i], order[j] = order[j], order[i]
    return order


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even), returned as fp32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    out = (r & 0xFFFFFFFF).astype(np.uint32).view(np.float32)
    return np.where(np.isfinite(x), out, x).astype(np.float32).reshape(np.shape(x))


def softmax_xent(logits: np.ndarray, labels: np.ndarray, mask: Optional[np.ndarray], n_train: int):
    """Mean softmax cross-entropy over the labelled rows.  Returns (sum of the row losses / n_train,
    gradient w.r.t. the logits); rows with mask 0 contribute nothing and get a zero gradient."""
    z = np.asarray(logits, dtype=np.float64)
    rows, C = z.shape
    m = np.ones(rows, dtype=bool) if mask is None else np.asarray(mask).astype(bool)
    zmax = z.max(axis=1, keepdims=True) if C else np.zeros((rows, 1))
    e = np.exp(z - zmax)
    s = e.sum(axis=1, keepdims=True)
    p = e / s
    logp_label = (z - zmax)[np.arange(rows), labels] - np.log(s[:, 0])
    loss = -(logp_label[m]).sum() / n_train
    g = p.copy()
    g[np.arange(rows), labels] -= 1.0
    g[~m] = 0.0
    return float(loss), g / n_train


def sgd_step(p: np.ndarray, g: np.ndarray, lr: float, weight_decay: float = 0.0) -> None:
    """Last line of Algorithm 1: W <- W - eta * grad (with the optional L2 term)."""
    p -= lr * (g + weight_decay * p)


def adam_step(p, g, m, v, t: int, lr: float, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
              weight_decay: float = 0.0) -> None:
    """Step t (1-based) of Adam, in place on p, m, v."""
    g = g + weight_decay * p
    m *= beta1
    m += (1.0 - beta1) * g
    v *= beta2
    v += (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** t)
    v_hat = v / (1.0 - beta2 ** t)
    p -= lr * m_hat / (np.sqrt(v_hat) + eps)


class OracleTrainer:
    """Stages chained on one device (level L of stage s is level 0 of stage s + 1), a linear head, an
    optimiser.  ``stages`` are OracleStage objects whose ``cur`` arrays this object links together.

    ``quant``: the product's bf16 mode keeps an fp32 master copy of every weight and hands the stages its
    bf16 rounding; it stores the gradient of the logits and the gradient of the last level in bf16.  With
    quant=True the same roundings are applied here, at the same points."""

    def __init__(self, stages: Sequence[OracleStage], head_W: np.ndarray, head_b: np.ndarray, labels: np.ndarray,
                 train_mask: Optional[np.ndarray], *, optimizer: str = "adam", lr: float = 1e-3, beta1: float = 0.9,
                 beta2: float = 0.999, eps: float = 1e-8, weight_decay: float = 0.0, shuffle: bool = True,
                 seed: int = 0, alpha_hist: int = 1, quant: bool = False):
        self.stages = list(stages)
        for a, b in zip(self.stages[:-1], self.stages[1:]):
            assert int(a.dims[-1]) == int(b.dims[0])
            b.cur[0] = a.cur[a.L]  # the same array: what stage a writes, stage b reads
            b._refresh()
        self.K = self.stages[0].K
        self.chunk_ptr = self.stages[0].chunk_ptr
        self.n = self.stages[0].n
        self.labels = np.asarray(labels, dtype=np.int64)
        self.mask = None if train_mask is None else np.asarray(train_mask).astype(bool)
        self.n_train = int(self.n if self.mask is None else self.mask.sum())
        self.optimizer, self.lr, self.beta1, self.beta2, self.eps, self.wd = optimizer, lr, beta1, beta2, eps, weight_decay
        self.shuffle, self.seed, self.alpha_hist, self.quant = shuffle, seed, int(alpha_hist), quant
        # fp64 master copies of every parameter, in a fixed order: stage weights and biases, then the head
        self.master: List[np.ndarray] = []
        self._targets = []  # (stage index or None, kind, layer)
        for si, st in enumerate(self.stages):
            for j in range(st.L):
                self.master.append(np.array(st.W[j], dtype=np.float64))
                self._targets.append((si, "W", j))
            if st.variant != 1:  # every variant but GCNII has a bias vector per layer
                for j in range(st.L):
                    self.master.append(np.array(st.b[j], dtype=np.float64))
                    self._targets.append((si, "b", j))
            if st.variant == 3:  # ResGCN+: LayerNorm scale and shift of every layer
                for j in range(st.L):
                    self.master.append(np.array(st.ln_g[j], dtype=np.float64))
                    self._targets.append((si, "ln_g", j))
                for j in range(st.L):
                    self.master.append(np.array(st.ln_b[j], dtype=np.float64))
                    self._targets.append((si, "ln_b", j))
        self.master.append(np.array(head_W, dtype=np.float64))
        self._targets.append((None, "W", 0))
        self.master.append(np.array(head_b, dtype=np.float64))
        self._targets.append((None, "b", 0))
        self.m = [np.zeros_like(x) for x in self.master]
        self.v = [np.zeros_like(x) for x in self.master]
        self.head_W = np.array(head_W, dtype=np.float64)
        self.head_b = np.array(head_b, dtype=np.float64)
        self.head_dW = np.zeros_like(self.head_W)
        self.head_db = np.zeros_like(self.head_b)
        self.step = 0
        self._publish()

    def _publish(self) -> None:
        """Hand the compute copies of the master weights to the stages and the head."""
        for x, (si, kind, j) in zip(self.master, self._targets):
            w = bf16_round(x.astype(np.float32)).astype(np.float64) if (self.quant and kind == "W") else x
            if si is None:
                if kind == "W":
                    self.head_W[...] = w
                else:
                    self.head_b[...] = x
            else:
                st = self.stages[si]
                {"W": st.W, "b": st.b, "ln_g": st.ln_g, "ln_b": st.ln_b}[kind][j][...] = w.astype(st.rt)

    def grads(self) -> List[np.ndarray]:
        out = []
        for si, kind, j in self._targets:
            if si is None:
                out.append(self.head_dW if kind == "W" else self.head_db)
            else:
                st = self.stages[si]
                out.append({"W": st.dW, "b": st.db, "ln_g": st.d_ln_g, "ln_b": st.d_ln_b}[kind][j])
        return out

    def rows(self, k: int) -> slice:
        return slice(int(self.chunk_ptr[k]), int(self.chunk_ptr[k + 1]))

    def epoch(self, t: int) -> float:
        """Epoch t (0-based).  Returns the training loss of this epoch's forward pass."""
        order = chunk_order(self.seed, t, self.K, self.shuffle)
        self.last_order = order
        last = self.stages[-1]
        top = last.cur[last.L]
        C = self.head_W.shape[1]
        for si, st in enumerate(self.stages):
            st.zero_grads()
            st.set_dropout_seed(splitmix64(self.seed + (t + 1) * _GOLDEN) + si)  # this epoch's dropout decisions
            st.begin_pass()
        self.head_dW[...] = 0
        self.head_db[...] = 0
        dlogits = np.zeros((self.n, C))
        loss = 0.0
        # forward: chunk by chunk, each chunk through every stage, then through the head
        for k in order:
            k = int(k)
            for st in self.stages:
                st.forward_chunk(k)
            r = self.rows(k)
            logits = top[r].astype(np.float64) @ self.head_W + self.head_b
            lk, g = softmax_xent(logits, self.labels[r], None if self.mask is None else self.mask[r], self.n_train)
            loss += lk
            dlogits[r] = bf16_round(g.astype(np.float32)) if self.quant else g
        # backward: reverse chunk order, last stage first
        for k in reversed(order):
            k = int(k)
            r = self.rows(k)
            self.head_dW += top[r].astype(np.float64).T @ dlogits[r]
            self.head_db += dlogits[r].sum(axis=0)
            g = dlogits[r] @ self.head_W.T
            for si in range(len(self.stages) - 1, -1, -1):
                st = self.stages[si]
                gq = bf16_round(g.astype(np.float32)) if self.quant else g
                st.backward_chunk(k, gq.astype(st.rt), need_input_grad=si > 0)
                g = st.grad_in[r]
        # weight update
        self.step += 1
        for x, g, m, v in zip(self.master, self.grads(), self.m, self.v):
            if self.optimizer == "adam":
                adam_step(x, np.asarray(g, dtype=np.float64), m, v, self.step, self.lr, self.beta1, self.beta2, self.eps, self.wd)
            else:
                sgd_step(x, np.asarray(g, dtype=np.float64), self.lr, self.wd)
        self._publish()
        # historical embeddings are those of epoch alpha * floor((t - 1) / alpha) for the 1-based epoch t
        if (t + 1) % self.alpha_hist == 0:
            for st in self.stages:
                st.update_history()
        return loss

    def predict(self) -> np.ndarray:
        """Class with the largest logit, from the levels of the last forward pass."""
        last = self.stages[-1]
        return np.argmax(last.cur[last.L].astype(np.float64) @ self.head_W + self.head_b, axis=1)
