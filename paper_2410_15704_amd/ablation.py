"""Section 3.2's ablation on synthetic activations: number of codebooks in {4, 6, 8} x codes per
codebook in {1024, 2048}, one 128-channel head per vector (d / dhat = 4 groups of 32), keys with
the channels of a group 4 apart (strided) and values with contiguous groups (Section 3.1).

Training follows Section 3: k-means initialisation on the first batch, then `steps` steps that
update every stage's codebook by exponential moving average (decay 0.99), each step on a fresh
batch.  Host loops only: every step of the method runs in librvq's kernels.

The paper trains on language-model activations; none are available here, so the batches are seeded
synthetic stand-ins: keys = Gaussian rows with log-normal per-channel scales and a few outlier
channels (the structure Section 3.1 gives as the reason for strided groups), values = the same
without outliers.  The printed errors therefore show how the settings rank and how far grouping
matters on such data; they are not the paper's table.

    python -m paper_2410_15704_amd.ablation --steps 150 --tokens 65536

prints one JSON line per (tensor, grouping, codebooks, codes per codebook): bits per head vector
(codes + fp16 std), compression against fp16, and the relative reconstruction error
mean((x - xhat)^2) / mean(x^2) on a held-out batch.
"""
from __future__ import annotations

import argparse
import json
import math

import torch

from . import binding as b
from . import train

HEAD = 128
DHAT = 32


def synthetic_batch(kind: str, rows: int, step: int, seed: int, device) -> torch.Tensor:
    """bf16 [rows][128]: Gaussian rows times per-channel scales exp(N(0, 0.5^2)) that are fixed for
    the run; keys ("k") carry 4 outlier channels of 10 times the scale."""
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    sigma = torch.exp(0.5 * torch.randn(HEAD, generator=g, device=device))
    if kind == "k":
        ch = torch.randperm(HEAD, generator=g, device=device)[:4]
        sigma[ch] *= 10.0
    g.manual_seed(seed * 1000003 + 17 * step + 1)
    x = torch.randn((rows, HEAD), generator=g, device=device) * sigma
    return x.to(torch.bfloat16)


def run_setting(kind: str, grouping: int, depth: int, K: int, steps: int, rows: int, seed: int,
                kmeans_iters: int, device) -> dict:
    def groups(step):
        X = synthetic_batch(kind, rows, step, seed, device)
        return train.scaled_groups(X, d=HEAD, dhat=DHAT, grouping=grouping, in_dtype=b.BF16)

    Z0 = groups(0)
    gen = torch.Generator(device="cpu")
    gen.manual_seed(seed + depth * 131 + K)
    picks = [torch.randperm(Z0.shape[0], generator=gen)[:K].sort().values for _ in range(depth)]
    C = train.kmeans_init_codebooks(Z0, depth, K, kmeans_iters, picks)
    C = train.ema_train_online(Z0, depth, K, steps, 0.99, 1e-5, picks, init=C,
                               batches=lambda t: groups(t + 1))
    # held-out batch: quantize, reconstruct, compare
    X = synthetic_batch(kind, rows, steps + 1, seed, device)
    q = b.Quantizer(d=HEAD, dhat=DHAT, depth=depth, K=K, grouping=grouping, in_dtype=b.BF16,
                    out_dtype=b.F32, std_dtype=b.F16)
    q.set_codebooks(C)
    codes, std, _ = q.encode(X)
    Xh = q.decode(codes, std)
    Xf = X.float()
    err = float(((Xf - Xh) ** 2).mean() / (Xf ** 2).mean())
    q.close()
    bits = (HEAD // DHAT) * depth * max(1, math.ceil(math.log2(K))) + 16
    return dict(tensor=kind, grouping="strided" if grouping == b.STRIDED else "contiguous",
                codebooks=depth, codes_per_codebook=K, bits_per_head_vector=bits,
                compression_vs_fp16=round(HEAD * 16 / bits, 3), relative_error=err,
                steps=steps, rows_per_batch=rows)


def main(argv=None) -> list:
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--steps", type=int, default=150)
    ap.add_argument("--tokens", type=int, default=65536, help="tokens per batch (8 heads each)")
    ap.add_argument("--heads", type=int, default=8)
    ap.add_argument("--kmeans-iters", type=int, default=10)
    ap.add_argument("--seed", type=int, default=241015704)
    ap.add_argument("--depths", type=int, nargs="+", default=[4, 6, 8])
    ap.add_argument("--codes", type=int, nargs="+", default=[1024, 2048])
    ap.add_argument("--all-groupings", action="store_true",
                    help="also keys with contiguous and values with strided groups")
    args = ap.parse_args(argv)
    if not torch.cuda.is_available():
        raise SystemExit("the ablation runs the HIP library: a GPU is required")
    device = torch.device("cuda:0")
    rows = args.tokens * args.heads
    out = []
    plan = [("k", b.STRIDED), ("v", b.CONTIGUOUS)]
    if args.all_groupings:
        plan += [("k", b.CONTIGUOUS), ("v", b.STRIDED)]
    for kind, grouping in plan:
        for depth in args.depths:
            for K in args.codes:
                r = run_setting(kind, grouping, depth, K, args.steps, rows, args.seed,
                                args.kmeans_iters, device)
                print(json.dumps(r), flush=True)
                out.append(r)
    return out


if __name__ == "__main__":
    main()
