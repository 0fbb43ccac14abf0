"""What the GPU's memory system gives random whole-row gathers, by table size and row width: the yardstick for the
aggregation kernels (python -m paper_2308_10087_amd.examples.gather_rate).  Prints one line per case."""
import argparse

import torch

import paper_2308_10087_amd as g


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--sizes-mb", default="2,32,128,512,2048,5120,10240")
    ap.add_argument("--row-bytes", default="256,512")
    ap.add_argument("--gather-gb", type=float, default=4.0, help="bytes gathered per launch")
    ap.add_argument("--mode", type=int, default=0, help="0 plain loads, 1 non-temporal loads, 2 hot rows spread over the table")
    args = ap.parse_args()
    dev = "cuda:0"
    sizes = [int(x) for x in args.sizes_mb.split(",")]
    table = torch.empty(max(sizes) << 20, dtype=torch.uint8, device=dev)
    table.random_(0, 255)  # touch every page
    torch.cuda.synchronize()
    print(f"mode {args.mode}\ntable MB | row bytes | hot rows | hot share | gathered GB/s")
    for rb in [int(x) for x in args.row_bytes.split(",")]:
        for mb in sizes:
            n_rows = (mb << 20) // rb
            n_g = int(args.gather_gb * 1e9 / rb)
            r = g.gnnstage_debug_gather_rate(table, n_rows, rb, n_g, mode=args.mode)
            print(f"{mb:8d} | {rb:9d} | {0:8d} | {0.0:9.2f} | {r / 1e9:10.0f}", flush=True)
        # the benchmark's largest graph: 10 M rows, 37 % of the gathers to the 65,536 hottest, 58 % to the 262,144 hottest
        for hot_rows, share in ((65536, 0.37), (262144, 0.58), (524288, 0.71)):
            mb = max(sizes)
            if hot_rows >= (mb << 20) // rb:  # the table given on the command line is smaller than this hot set
                continue
            r = g.gnnstage_debug_gather_rate(table, (mb << 20) // rb, rb, int(args.gather_gb * 1e9 / rb), hot_rows=hot_rows, hot_share=share, mode=args.mode)
            print(f"{mb:8d} | {rb:9d} | {hot_rows:8d} | {share:9.2f} | {r / 1e9:10.0f}", flush=True)


if __name__ == "__main__":
    main()
