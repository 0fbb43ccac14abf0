"""Trains a small multi-stage model with the epoch loop of include/gnntrain.h on a synthetic
node-classification task (a planted-partition graph whose labels are the planted groups) and prints the
loss and the held-out accuracy.  Everything on the device runs in the library's kernels; torch only holds
the buffers.

    python -m paper_2308_10087_amd.examples.train_planted_partition --epochs 60 --layers gcn,resgcn,sage

Stages run back to back on one GPU (the pipeline's sequential schedule); chunk order is shuffled every epoch,
the historical embeddings are refreshed every --alpha-hist epochs (Section 3.4 of the paper).
"""
from __future__ import annotations

import argparse
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--vertices", type=int, default=20000)
    ap.add_argument("--classes", type=int, default=8)
    ap.add_argument("--hidden", type=int, default=64)
    ap.add_argument("--features", type=int, default=64)
    ap.add_argument("--layers", default="gcn,resgcn", help="one stage of two layers per entry: gcn, sage or resgcn")
    ap.add_argument("--chunks", type=int, default=8)
    ap.add_argument("--epochs", type=int, default=60)
    ap.add_argument("--alpha-hist", type=int, default=2)
    ap.add_argument("--lr", type=float, default=0.005)
    ap.add_argument("--dropout", type=float, default=0.0,
                    help="inside ResGCN+ blocks and on the layer outputs of gcn / sage stages (not of the last stage, which feeds the head)")
    ap.add_argument("--bf16", action="store_true")
    ap.add_argument("--partition", action="store_true",
                    help="chunks from the locality-aware partitioner (Algorithm 1's first step) instead of index ranges")
    ap.add_argument("--seed", type=int, default=1)
    args = ap.parse_args()

    import torch
    import paper_2308_10087_amd as g
    from synth import graphs, values

    dev = "cuda:0"
    n, C, K = args.vertices, args.classes, args.chunks
    row_ptr, col, group = graphs.planted_partition(n, C, 10.0, 4.0, args.seed)
    x0 = values.group_features(args.seed, 1, group, args.features, 0.4)
    train_mask = values.bernoulli_mask(args.seed, 2, n, 0.3)
    chunk_ptr = graphs.equal_chunks(n, K)
    if args.partition:  # renumber the vertices chunk by chunk; features, labels and mask follow
        part, perm, chunk_ptr = g.gnnstage_partition_chunks(row_ptr, col, K)
        rows_all = np.repeat(np.arange(n), np.diff(row_ptr))
        print(f"neighbours in other chunks: {np.mean((rows_all * K // n) != (col.astype(np.int64) * K // n)):.3f} with index ranges, "
              f"{np.mean(part[rows_all] != part[col]):.3f} with the partitioner", flush=True)
        row_ptr, col = g.gnnstage_permute_csr(row_ptr, col, perm)
        inverse = np.argsort(perm)
        x0, group, train_mask = x0[inverse], group[inverse], train_mask[inverse]
    sdt = torch.bfloat16 if args.bf16 else torch.float32
    kinds = args.layers.split(",")
    variant = {"gcn": g.GNNSTAGE_GCN, "sage": g.GNNSTAGE_SAGE, "resgcn": g.GNNSTAGE_RESGCN}

    stages, params, prev_top, width = [], [], None, args.features
    keep = []
    for si, kind in enumerate(kinds):
        first = si == 0
        if kind == "resgcn" and width != args.hidden:
            raise SystemExit("a resgcn stage keeps its width: put a gcn or sage stage in front of it")
        dims = [width, args.hidden, args.hidden]
        wr = 2 if kind == "sage" else 1
        master = [torch.from_numpy(np.concatenate([values.glorot_uniform(args.seed, 100 + 20 * si + 10 * h + j, dims[j], dims[j + 1])
                                                   for h in range(wr)])).to(dev) for j in range(2)]
        W = [m.to(sdt) for m in master] if args.bf16 else master
        bias = [torch.zeros(dims[j + 1], device=dev) for j in range(2)]
        l0 = torch.float32 if (first and args.bf16 and kind != "resgcn") else sdt
        level0 = torch.from_numpy(x0).to(dev, l0) if first else prev_top
        cur = [level0] + [torch.zeros((n, dims[j]), dtype=sdt, device=dev) for j in (1, 2)]
        hist = [cur[0] if first else torch.zeros((n, dims[0]), dtype=sdt, device=dev), torch.zeros((n, dims[1]), dtype=sdt, device=dev)]
        dW = [torch.zeros_like(m) for m in master]
        dbias = [torch.zeros_like(b) for b in bias]
        grad_in = None if first else torch.zeros((n, dims[0]), dtype=sdt, device=dev)
        ln = [None] * 4
        if kind == "resgcn":
            ln = [[torch.ones(dims[j], device=dev) for j in range(2)], [torch.zeros(dims[j], device=dev) for j in range(2)],
                  [torch.zeros(dims[j], device=dev) for j in range(2)], [torch.zeros(dims[j], device=dev) for j in range(2)]]
        st = g.GnnStage(row_ptr, col, chunk_ptr, dims, W=W, cur=cur, hist=hist, dW=dW, bias=bias, dbias=dbias, variant=variant[kind],
                        dtype=g.GNNSTAGE_BF16 if args.bf16 else g.GNNSTAGE_F32, level0_f32=(l0 == torch.float32 and args.bf16),
                        grad_in=grad_in, device=dev, ln_gamma=ln[0], ln_beta=ln[1], d_ln_gamma=ln[2], d_ln_beta=ln[3],
                        dropout_p=args.dropout if (kind == "resgcn" or si < len(kinds) - 1) else 0.0)
        stages.append(st)
        params += [(master[j], W[j] if args.bf16 else None, dW[j]) for j in range(2)]
        params += [(bias[j], None, dbias[j]) for j in range(2)]
        if kind == "resgcn":
            params += [(ln[0][j], None, ln[2][j]) for j in range(2)] + [(ln[1][j], None, ln[3][j]) for j in range(2)]
        keep.append((cur, hist, grad_in))
        prev_top, width = cur[2], args.hidden

    head_master = torch.from_numpy(values.glorot_uniform(args.seed, 900, args.hidden, C)).to(dev)
    head_W = head_master.to(sdt) if args.bf16 else head_master
    head_b = torch.zeros(C, device=dev)
    head_dW, head_db = torch.zeros((args.hidden, C), device=dev), torch.zeros(C, device=dev)
    params += [(head_master, head_W if args.bf16 else None, head_dW), (head_b, None, head_db)]
    labels = torch.from_numpy(group.astype(np.int32)).to(dev)
    mask = torch.from_numpy(train_mask).to(dev)
    trainer = g.GnnTrainer(stages, head_W=head_W, head_b=head_b, head_dW=head_dW, head_db=head_db, labels=labels, train_mask=mask,
                           params=params, optimizer=g.GNNTRAIN_ADAM, lr=args.lr, shuffle=True, seed=args.seed,
                           alpha_hist=args.alpha_hist, device=dev)
    held_out = torch.from_numpy(train_mask == 0).to(dev)
    for epoch in range(args.epochs):
        loss = trainer.gnntrain_epoch(epoch)
        if epoch % 5 == 0 or epoch == args.epochs - 1:
            # reporting only: accuracy of the last forward pass's levels on the unlabelled vertices
            pred = (prev_top.float() @ head_master + head_b).argmax(dim=1)
            acc = (pred[held_out] == labels[held_out].long()).float().mean().item()
            print(f"epoch {epoch:4d}  loss {loss:.4f}  held-out accuracy {acc:.3f}", flush=True)


if __name__ == "__main__":
    main()
