"""GPU parity on randomly drawn combinations (seeded, so repeatable): layer type, widths, chunking, which kernels serve the
aggregation (dense-block threshold, source classes, class cut length), weights given or computed, dropout, first or
middle stage, with or without the input gradient.  The single-feature tests pin each kernel; this one looks for
trouble where features meet."""
import random

import pytest

from synth import graphs
from synth.configs import Workload

from helpers import make_problem
from test_gpu_parity import TOL_BF16, _parity

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", [7, 11, 23, 31])
def test_random_combinations_bf16(monkeypatch, seed):
    rng = random.Random(seed)
    for case in range(8):
        variant = rng.choice(["gcn", "gcn", "sage", "resgcn", "gcnii"])
        L = rng.choice([2, 3])
        if variant in ("resgcn", "gcnii"):
            dims = [rng.choice([128, 256])] * (L + 1)
        else:
            dims = [rng.choice([128, 256]) for _ in range(L + 1)]
        n = rng.choice([3001, 4099, 6007])
        K = rng.choice([3, 5, 8])
        graph_seed = rng.randrange(1 << 30)
        drop = 0.0 if variant == "gcnii" else rng.choice([0.0, 0.0, 0.5, 0.25])
        monkeypatch.setenv("GNNSTAGE_DENSE_MIN_ENTRIES", "0")
        monkeypatch.setenv("GNNSTAGE_DENSE_MIN_SHARE", "0")
        monkeypatch.setenv("GNNSTAGE_DENSE_MIN_NNZ", str(rng.choice([2, 6, 24, 64])))
        monkeypatch.setenv("GNNSTAGE_XCD_CLASSES", str(rng.choice([1, 4, 8])))
        monkeypatch.setenv("GNNSTAGE_CLASS_MIN_ROW", str(rng.choice([8, 32, 128])))
        extra = {"gcnii_first_layer": 3} if variant == "gcnii" else {}
        w = Workload(f"sweep{seed}_{case}", "rmat", n, graph_seed, dims, K, variant=variant, dtype="bf16",
                     n_candidates=rng.choice([60_000, 200_000]), **extra)
        weights = rng.choice(["given", "computed"])
        first = rng.choice([True, False]) if variant in ("gcn", "sage") else False
        p = make_problem(w, chunk_ptr=graphs.ragged_chunks(n, K, rng.randrange(100)), first_stage=first, dropout_p=drop,
                         dropout_seed=rng.randrange(1 << 40), bias_std=0.05)
        need_input_grad = rng.choice([True, False]) if variant != "gcnii" else True
        what = (f"seed {seed} case {case}: {variant} dims={dims} n={n} K={K} dropout={drop} weights={weights} first={first} "
                f"need_input_grad={need_input_grad}")
        print(what, flush=True)  # names the case before the GPU runs it
        _parity(p, TOL_BF16, need_input_grad=need_input_grad, edge_val=weights)


@pytest.mark.parametrize("seed", [5, 13, 29])
def test_random_combinations_fp32(monkeypatch, seed):
    """The fp32 stage (vector-ALU aggregation, odd widths, fp32 products) on random shapes."""
    from test_gpu_parity import TOL_F32, small
    rng = random.Random(seed)
    for case in range(8):
        variant = rng.choice(["gcn", "sage", "resgcn", "gcnii"])
        L = rng.choice([1, 2, 3, 4])
        if variant in ("resgcn", "gcnii"):
            dims = (rng.choice([3, 8, 17, 40, 64, 100]),) * (L + 1)
        else:
            dims = tuple(rng.choice([1, 3, 7, 8, 16, 24, 33, 64, 72]) for _ in range(L + 1))
        n = rng.choice([257, 700, 911])
        K = rng.choice([1, 2, 5, 9])
        drop = 0.0 if variant == "gcnii" else rng.choice([0.0, 0.5, 0.3])
        monkeypatch.setenv("GNNSTAGE_XCD_CLASSES", str(rng.choice([1, 4, 8])))
        monkeypatch.setenv("GNNSTAGE_CLASS_MIN_ROW", str(rng.choice([4, 16, 128])))
        monkeypatch.setenv("GNNSTAGE_ORDER", rng.choice(["aggregate", "transform", "auto"]))
        w = small(n=n, k=K, dims=dims, variant=variant, seed=rng.randrange(1 << 20), deg=rng.choice([3.0, 6.0, 12.0]))
        first = rng.choice([True, False]) if variant in ("gcn", "sage") else False
        p = make_problem(w, chunk_ptr=graphs.ragged_chunks(n, K, rng.randrange(100)), first_stage=first, noise_std=0.3,
                         dropout_p=drop, dropout_seed=rng.randrange(1 << 40))
        need_input_grad = rng.choice([True, False]) if variant != "gcnii" else True
        weights = rng.choice(["given", "computed"])
        print(f"seed {seed} case {case}: {variant} dims={dims} n={n} K={K} dropout={drop} weights={weights} first={first} "
              f"need_input_grad={need_input_grad}", flush=True)
        _parity(p, TOL_F32, need_input_grad=need_input_grad, edge_val=weights)
