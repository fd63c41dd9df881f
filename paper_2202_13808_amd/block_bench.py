"""Training-step time and peak memory of a DeiT-S-shaped encoder with and without DropIT.

    python -m paper_2202_13808_amd.block_bench [--batch 128] [--depth 12] [--steps 20]

Reproduces the *shape* of the paper's memory / speed comparison (Sec. 4.3, the table that lists maximum
memory and ms per iteration at batch size 128, and the cached-tensor table): synthetic tokens, random
weights, bf16, one GPU.  DropIT is applied to the fully-connected layers of the attention and MLP halves
of every block (Sec. 3.5); the embedding and the classifier are the first and last layers and stay plain.
Prints one JSON line per gamma.
"""
import argparse
import json
import time

import torch

from . import nn as dnn


class Block(torch.nn.Module):
    def __init__(self, dim: int, heads: int, hidden: int) -> None:
        super().__init__()
        self.heads = heads
        self.norm1 = torch.nn.LayerNorm(dim)
        self.qkv = torch.nn.Linear(dim, 3 * dim)
        self.proj = torch.nn.Linear(dim, dim)
        self.norm2 = torch.nn.LayerNorm(dim)
        self.fc1 = torch.nn.Linear(dim, hidden)
        self.act = torch.nn.GELU()
        self.fc2 = torch.nn.Linear(hidden, dim)

    def forward(self, x: torch.Tensor) -> torch.Tensor:
        b, t, d = x.shape
        q, k, v = self.qkv(self.norm1(x)).reshape(b, t, 3, self.heads, d // self.heads).permute(2, 0, 3, 1, 4)
        a = torch.nn.functional.scaled_dot_product_attention(q, k, v).transpose(1, 2).reshape(b, t, d)
        x = x + self.proj(a)
        return x + self.fc2(self.act(self.fc1(self.norm2(x))))


def encoder(depth: int, dim: int, heads: int, hidden: int, classes: int) -> torch.nn.Module:
    class Net(torch.nn.Module):
        def __init__(self) -> None:
            super().__init__()
            self.embed = torch.nn.Linear(dim, dim)              # stands in for the patch projection
            self.blocks = torch.nn.Sequential(*[Block(dim, heads, hidden) for _ in range(depth)])
            self.norm = torch.nn.LayerNorm(dim)
            self.head = torch.nn.Linear(dim, classes)

        def forward(self, x: torch.Tensor) -> torch.Tensor:
            return self.head(self.norm(self.blocks(self.embed(x)))[:, 0])

    return Net()


def run(gamma: float, args) -> dict:
    torch.manual_seed(0)
    model = encoder(args.depth, args.dim, args.heads, 4 * args.dim, 1000).to("cuda:0", torch.bfloat16)
    layers = dnn.apply_dropit(model, gamma, index_format=args.index) if gamma > 0 else []
    opt = torch.optim.SGD(model.parameters(), lr=1e-3)
    x = torch.randn(args.batch, args.tokens, args.dim, device="cuda:0", dtype=torch.bfloat16)
    target = torch.randint(0, 1000, (args.batch,), device="cuda:0")
    meter = None

    def step() -> None:
        opt.zero_grad(set_to_none=True)
        torch.nn.functional.cross_entropy(model(x).float(), target).backward()
        opt.step()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    torch.cuda.reset_peak_memory_stats()
    with dnn.cache_meter() as meter:
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / args.steps
    gib = 1.0 / (1 << 30)
    return {"gamma": gamma, "index": args.index, "dropit_layers": len(layers), "ms_per_iter": round(dt * 1e3, 2),
            "max_memory_GiB": round(torch.cuda.max_memory_allocated() * gib, 3),
            "dense_cache_GiB": round(meter.dense_bytes / args.steps * gib, 3),
            "value_cache_GiB": round(meter.value_bytes / args.steps * gib, 3),
            "index_cache_GiB": round(meter.index_bytes / args.steps * gib, 3)}


def main() -> None:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--batch", type=int, default=128)
    ap.add_argument("--tokens", type=int, default=197)
    ap.add_argument("--dim", type=int, default=384)
    ap.add_argument("--heads", type=int, default=6)
    ap.add_argument("--depth", type=int, default=12)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--index", choices=["flat", "rows", "mask"], default="flat",
                    help="cached index form: int32 flat indices, 16-bit in-row positions + row offsets, or one "
                         "bit per element + block offsets")
    ap.add_argument("--gammas", type=float, nargs="*", default=[0.0, 0.6, 0.7, 0.8, 0.9])
    args = ap.parse_args()
    if not torch.cuda.is_available():
        raise SystemExit("block_bench needs a GPU: DropIT layers have no CPU path")
    for gamma in args.gammas:
        print(json.dumps(run(gamma, args)), flush=True)


if __name__ == "__main__":
    main()
