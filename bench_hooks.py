"""End-to-end demonstration of the paper's system claim on PyTorch-ROCm: a GPT-style transformer on
synthetic tokens trained with (a) plain gradient accumulation + Adam, (b) AdamA through backward
hooks (torch_hooks.AdamAccumulation) and (c) the same with the folds on a side stream, same model,
same micro-batches.

    python bench_hooks.py [--layers 24] [--hidden 2048] [--heads 16] [--seq 1024] [--micro-batch 4] [--N 8] [--steps 3]

Prints one JSON line: step time and tokens/s of both, and the peak device memory each needed on top
of parameters and optimizer state (Sec. 3.1: AdamA keeps one layer's gradients alive instead of the
whole model's).  PyTorch produces the gradients (autocast bfloat16 matmuls, float32 parameters and
gradients); all optimizer arithmetic of (b) runs in libadama.  Baseline (a) uses torch.optim.Adam's
fused implementation and divides each micro-batch loss by N, as gradient accumulation does.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import torch  # noqa: E402
import torch.nn.functional as F  # noqa: E402

from paper_2305_19982_amd.torch_hooks import AdamAccumulation  # noqa: E402


class Block(torch.nn.Module):
    def __init__(self, hidden: int, heads: int):
        super().__init__()
        self.heads = heads
        self.ln_1 = torch.nn.LayerNorm(hidden)
        self.qkv = torch.nn.Linear(hidden, 3 * hidden)
        self.proj = torch.nn.Linear(hidden, hidden)
        self.ln_2 = torch.nn.LayerNorm(hidden)
        self.fc = torch.nn.Linear(hidden, 4 * hidden)
        self.out = torch.nn.Linear(4 * hidden, hidden)

    def forward(self, x):
        b, s, h = x.shape
        q, k, v = self.qkv(self.ln_1(x)).view(b, s, 3, self.heads, h // self.heads).permute(2, 0, 3, 1, 4)
        a = F.scaled_dot_product_attention(q, k, v, is_causal=True).transpose(1, 2).reshape(b, s, h)
        x = x + self.proj(a)
        return x + self.out(F.gelu(self.fc(self.ln_2(x))))


class TinyGPT(torch.nn.Module):
    def __init__(self, layers: int, hidden: int, heads: int, vocab: int, seq: int):
        super().__init__()
        self.wte = torch.nn.Embedding(vocab, hidden)
        self.wpe = torch.nn.Embedding(seq, hidden)
        self.blocks = torch.nn.ModuleList([Block(hidden, heads) for _ in range(layers)])
        self.ln_f = torch.nn.LayerNorm(hidden)
        self.head = torch.nn.Linear(hidden, vocab, bias=False)

    def forward(self, tokens):
        pos = torch.arange(tokens.shape[1], device=tokens.device)
        x = self.wte(tokens) + self.wpe(pos)
        for blk in self.blocks:
            x = blk(x)
        return self.head(self.ln_f(x))


def block_layers(model: TinyGPT) -> list:
    """One fold launch per transformer block, as the paper's per-layer granularity."""
    groups = [list(model.wte.parameters()) + list(model.wpe.parameters())]
    groups += [list(b.parameters()) for b in model.blocks]
    groups.append(list(model.ln_f.parameters()) + list(model.head.parameters()))
    return groups


def run(mode: str, args, data) -> dict:
    torch.manual_seed(0)
    model = TinyGPT(args.layers, args.hidden, args.heads, args.vocab, args.seq).cuda()
    n_params = sum(p.numel() for p in model.parameters())
    adama = mode.startswith("adama")
    if adama:
        opt = AdamAccumulation(block_layers(model), lr=1e-4, N=args.N, fused_edges=True,
                               overlap=mode == "adama_overlap")
    else:
        opt = torch.optim.Adam(model.parameters(), lr=1e-4, fused=True)

    def mini_batch(batch):
        if adama:
            opt.begin_mini_batch()
        for tokens in batch:
            with torch.autocast("cuda", dtype=torch.bfloat16):
                logits = model(tokens[:, :-1])
            loss = F.cross_entropy(logits.float().view(-1, logits.shape[-1]), tokens[:, 1:].reshape(-1))
            if adama:
                loss.backward()                    # raw gradients: the fold applies 1/N
                opt.micro_batch_done()
            else:
                (loss / args.N).backward()         # accumulate into p.grad
        opt.step()
        if not adama:
            opt.zero_grad(set_to_none=True)
        return loss

    mini_batch(data[0])                            # warm-up: allocator pools, optimizer state
    torch.cuda.synchronize()
    base = torch.cuda.memory_allocated()           # parameters + optimizer state (+ nothing else alive)
    torch.cuda.reset_peak_memory_stats()
    t0 = time.perf_counter()
    for batch in data[1:]:
        loss = mini_batch(batch)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / (len(data) - 1)
    peak = torch.cuda.max_memory_allocated()
    tokens = args.N * args.micro_batch * (args.seq - 1)
    out = {"step_ms": round(dt * 1e3, 2), "tokens_per_s": round(tokens / dt, 1), "params": n_params,
           "resident_bytes": base, "peak_bytes": peak, "peak_over_resident_bytes": peak - base,
           "final_loss": round(float(loss.detach()), 4)}
    if adama:
        out["peak_live_grad_bytes"] = opt.peak_live_grad_bytes
        opt.remove_hooks()
    del model, opt
    torch.cuda.empty_cache()
    return out


def compare(args) -> dict:
    torch.backends.cuda.matmul.allow_tf32 = False
    g = torch.Generator(device="cuda").manual_seed(1)
    data = [[torch.randint(0, args.vocab, (args.micro_batch, args.seq), device="cuda", generator=g)
             for _ in range(args.N)] for _ in range(args.steps + 1)]
    accum = run("accumulation", args, data)
    adama = run("adama", args, data)
    over = run("adama_overlap", args, data)
    return {
        "model": {"layers": args.layers, "hidden": args.hidden, "heads": args.heads, "seq": args.seq,
                  "micro_batch": args.micro_batch, "N": args.N, "params": accum["params"]},
        "gradient_accumulation_adam": accum, "adama_hooks": adama, "adama_hooks_side_stream": over,
        "throughput_ratio": round(adama["tokens_per_s"] / accum["tokens_per_s"], 4),
        "throughput_ratio_side_stream": round(over["tokens_per_s"] / accum["tokens_per_s"], 4),
        "peak_memory_saved_frac_side_stream": round(1.0 - over["peak_bytes"] / accum["peak_bytes"], 4),
        "peak_memory_saved_bytes": accum["peak_bytes"] - adama["peak_bytes"],
        "peak_memory_saved_frac": round(1.0 - adama["peak_bytes"] / accum["peak_bytes"], 4),
        "data": "synthetic tokens"}


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--layers", type=int, default=24)
    ap.add_argument("--hidden", type=int, default=2048)
    ap.add_argument("--heads", type=int, default=16)
    ap.add_argument("--vocab", type=int, default=32000)
    ap.add_argument("--seq", type=int, default=1024)
    ap.add_argument("--micro-batch", type=int, default=4)
    ap.add_argument("--N", type=int, default=8)
    ap.add_argument("--steps", type=int, default=3)
    print(json.dumps(compare(ap.parse_args())), flush=True)


if __name__ == "__main__":
    main()
