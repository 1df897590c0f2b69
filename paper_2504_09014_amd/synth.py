"""Seeded synthetic inputs shaped like the paper's workloads.

This module holds no arithmetic of the method: it only draws random inputs.  Both the
tests (which feed the CPU oracle) and the benchmark (which feeds the HIP library) take
their inputs from here, so the two sides see identical data.

Shapes stand in for: message-size sweeps of 1 KB .. 1 GB per rank (the paper's collective
benchmarks), the [tokens, 8192] activations of an 8-way tensor-parallel Llama3-70b decode
step, and the DeepSeek-V3 expert-parallel setting (hidden 7168, top-8 of 256 experts).
Rank r of a workload with seed s draws from generator seed s*1000 + r.
"""
import torch


def _gen(seed: int, rank: int, device="cpu") -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) * 1000 + int(rank))
    return g


def int_valued_f32(nranks: int, count: int, seed: int = 0, lo: int = -1000, hi: int = 1000,
                   device="cpu") -> torch.Tensor:
    """[nranks, count] float32 holding uniform integers in [lo, hi] (sums are exact)."""
    rows = [torch.randint(lo, hi + 1, (count,), generator=_gen(seed, r, device), device=device,
                          dtype=torch.int32).to(torch.float32) for r in range(nranks)]
    return torch.stack(rows) if count else torch.zeros((nranks, 0), dtype=torch.float32, device=device)


def normal(nranks: int, count: int, seed: int = 0, std: float = 1.0, dtype=torch.bfloat16,
           device="cpu") -> torch.Tensor:
    """[nranks, count] values N(0, std^2), drawn in fp32 and rounded to dtype by torch."""
    out = torch.empty((nranks, count), dtype=dtype, device=device)
    for r in range(nranks):
        g = _gen(seed, r, device)
        # draw in slabs so that a 1 GiB row never needs a 2 GiB fp32 temporary
        slab = 1 << 26
        for lo in range(0, count, slab):
            m = min(slab, count - lo)
            out[r, lo:lo + m] = (torch.randn(m, generator=g, device=device, dtype=torch.float32) * std).to(dtype)
    return out


def decode_activations(nranks: int, tokens: int, hidden: int = 8192, seed: int = 0, device="cpu"):
    """Tensor-parallel decode shape: per-rank partial sums [tokens, hidden] ~ N(0, 0.5^2) and
    one residual [tokens, hidden] ~ N(0,1) that every rank holds a copy of.  bf16."""
    x = normal(nranks, tokens * hidden, seed=seed, std=0.5, device=device)
    res = normal(1, tokens * hidden, seed=seed + 7919, std=1.0, device=device)[0]
    return x, res


def moe_routing(nranks: int, tokens: int, topk: int = 8, n_experts: int = 256, seed: int = 0,
                device="cpu") -> torch.Tensor:
    """[nranks, tokens, topk] int32: per token, topk DISTINCT experts uniform over n_experts."""
    rows = []
    for r in range(nranks):
        g = _gen(seed + 31, r, device)
        score = torch.rand((tokens, n_experts), generator=g, device=device)
        rows.append(score.topk(topk, dim=1).indices.to(torch.int32))
    return torch.stack(rows)


def moe_tokens(nranks: int, tokens: int, hidden: int = 7168, seed: int = 0, device="cpu") -> torch.Tensor:
    """[nranks, tokens, hidden] bf16 ~ N(0,1)."""
    return normal(nranks, tokens * hidden, seed=seed + 17, device=device).view(nranks, tokens, hidden)


def bf16_bits(t: torch.Tensor):
    """bf16 tensor (any device) -> numpy uint16 array of its bit patterns."""
    return t.detach().cpu().contiguous().view(torch.uint16).numpy()
