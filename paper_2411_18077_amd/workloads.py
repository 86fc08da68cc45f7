"""Seeded synthetic inputs with the shapes of the paper's workloads (no arithmetic of the method).

The paper evaluates on LongBench / InfiniteBench / GSM8K prompts run through LLaMA-2, Llama-3 and
Mistral checkpoints (Section 4).  Neither the datasets nor the weights exist here, so these seeded
tensors stand in for them: the same head counts and head dimension (LLaMA2-7B: 32 MHA heads x 128;
Llama-3-8B / Mistral-7B: 32 query / 8 KV heads x 128), prompt 4096 with a 50 % budget and
n_r = 128 as in the paper's hyper-parameters, and a few large-magnitude key CHANNELS because the
paper motivates per-channel key quantization by channel outliers (Section 3.1.1).

This module is shared by the tests, the benchmark and the smoke check.  It only draws random
numbers, scales outlier channels, picks retained-token index sets and counts bytes.
"""
from dataclasses import dataclass, field
import math

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    Hq: int
    Hkv: int
    L: int                 # context length the retained tokens are drawn from
    keep: float            # fraction of the context retained per KV head (None: ragged, see keep_range)
    G: int
    Rcap: int              # residual capacity n_r; the measured step holds r = Rcap fp16 tokens
    seed: int
    dist: str = "normal"   # "normal" or "student_t4"
    n_outlier: int = 0     # K channels per head multiplied by outlier_scale
    outlier_scale: float = 1.0
    keep_range: tuple = None   # (lo, hi) fractions for ragged per-unit lengths
    D: int = 128

    @property
    def units(self):
        return self.B * self.Hkv

    def retained_lengths(self, gen):
        """Quantized tokens per (batch, KV head): floor(keep * L) rounded DOWN to a multiple of G."""
        if self.keep_range is None:
            n = int(math.floor(self.keep * self.L)) // self.G * self.G
            return torch.full((self.units,), n, dtype=torch.int32)
        lo, hi = self.keep_range
        frac = lo + (hi - lo) * torch.rand(self.units, generator=gen)
        n = torch.floor(frac * self.L).to(torch.int64) // self.G * self.G
        return n.clamp_(min=self.G, max=self.L // self.G * self.G).to(torch.int32)

    def tcap(self, n_max):
        """Token capacity: the retained tokens plus room for one residual flush, in 128-token tiles."""
        return (int(n_max) + self.Rcap + 127) // 128 * 128


# The five configurations of the build's baseline file, in its order (index 0 = the small case).
WORKLOADS = [
    Workload("cfg1_mha8_1k", B=1, Hq=8, Hkv=8, L=1024, keep=1.0, G=32, Rcap=32, seed=1001,
             n_outlier=4, outlier_scale=10.0),
    Workload("cfg2_llama2_7b_4k", B=8, Hq=32, Hkv=32, L=4096, keep=0.5, G=32, Rcap=128, seed=1002,
             n_outlier=3, outlier_scale=8.0),
    Workload("cfg3_mha32_16k_b32", B=32, Hq=32, Hkv=32, L=16384, keep=0.3, G=32, Rcap=128, seed=1003),
    Workload("cfg4_llama3_8b_gqa_32k", B=16, Hq=32, Hkv=8, L=32768, keep=0.4, G=32, Rcap=128, seed=1004,
             n_outlier=3, outlier_scale=8.0),
    Workload("cfg5_ragged_gqa_128k", B=4, Hq=32, Hkv=8, L=131072, keep=None, keep_range=(0.05, 1.0),
             G=64, Rcap=256, seed=1005, dist="student_t4"),
]


def by_name(name):
    for w in WORKLOADS:
        if w.name == name or w.name.split("_")[0] == name:
            return w
    raise KeyError(name)


def _draw(shape, dist, gen, device, chunk_rows=None):
    """fp16 samples of N(0,1) or Student-t(df=4) (a normal over the root of a chi-square(4)/4)."""
    if dist == "normal":
        return torch.randn(shape, generator=gen, device=device, dtype=torch.float32).to(torch.float16)
    if dist == "student_t4":
        out = torch.empty(shape, device=device, dtype=torch.float16)
        flat = out.view(-1)
        step = 1 << 24
        for s in range(0, flat.numel(), step):
            n = min(step, flat.numel() - s)
            z = torch.randn(n, generator=gen, device=device, dtype=torch.float32)
            chi = torch.randn(4, n, generator=gen, device=device, dtype=torch.float32).square_().sum(0)
            flat[s:s + n] = (z / torch.sqrt(chi / 4.0)).to(torch.float16)
        return out
    raise ValueError(dist)


@dataclass
class Inputs:
    w: Workload
    K: torch.Tensor        # fp16 [units, L, D] full-context keys (before eviction)
    V: torch.Tensor        # fp16 [units, L, D]
    idx: torch.Tensor      # int32 [units, n_max] ascending retained positions (first n_tok[u] valid)
    n_tok: torch.Tensor    # int32 [units]
    q: torch.Tensor        # fp16 [B, Hq, D]
    Rk: torch.Tensor       # fp16 [units, Rcap, D] the Rcap newest (un-evicted, un-quantized) tokens
    Rv: torch.Tensor
    Tcap: int
    outlier_channels: torch.Tensor = field(default=None)


def make_inputs(w: Workload, device="cpu", seed_offset=0, unit_chunk=None):
    """All tensors one decode step needs, drawn from torch's seeded generator on `device`.

    Units are generated in order from one generator, so a (workload, device kind, seed_offset)
    triple always gives the same tensors.
    """
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed + 7919 * seed_offset)
    cgen = torch.Generator(device="cpu")
    cgen.manual_seed(w.seed + 7919 * seed_offset + 1)
    U, L, D = w.units, w.L, w.D

    n_tok = w.retained_lengths(cgen)
    n_max = int(n_tok.max())
    Tcap = w.tcap(n_max)

    K = _draw((U, L, D), w.dist, gen, dev)
    V = _draw((U, L, D), w.dist, gen, dev)
    Rk = _draw((U, w.Rcap, D), w.dist, gen, dev)
    Rv = _draw((U, w.Rcap, D), w.dist, gen, dev)
    q = _draw((w.B, w.Hq, D), w.dist, gen, dev)

    out_ch = None
    if w.n_outlier:
        # per KV head, n_outlier channels (seeded choice) of K are scaled up, context and residual alike
        out_ch = torch.stack([torch.randperm(D, generator=cgen)[: w.n_outlier] for _ in range(U)])
        mult = torch.ones(U, 1, D, dtype=torch.float16)
        mult.scatter_(2, out_ch.unsqueeze(1), w.outlier_scale)
        mult = mult.to(dev)
        K.mul_(mult)
        Rk.mul_(mult)

    # retained positions: a uniformly random subset of size n_tok[u] of 0..L-1, ascending
    keys = torch.rand(U, L, generator=gen, device=dev)
    order = keys.argsort(dim=1)[:, :n_max]
    pos = torch.arange(n_max, device=dev).unsqueeze(0)
    valid = pos < n_tok.to(dev).unsqueeze(1)
    order = torch.where(valid, order, torch.full_like(order, L))      # invalid tail sorts last
    idx = order.sort(dim=1).values
    idx = torch.where(valid, idx, torch.zeros_like(idx)).to(torch.int32).contiguous()
    if w.keep is not None and w.keep >= 1.0:
        idx = torch.arange(n_max, device=dev, dtype=torch.int32).repeat(U, 1).contiguous()

    return Inputs(w, K, V, idx, n_tok.to(dev), q, Rk, Rv, Tcap, out_ch)


def make_prefill_inputs(B, Hq, Hkv, L, seed, device="cpu", D=128, gain=1.0):
    """fp16 Q [B, Hq, L, D], K and V [B, Hkv, L, D] of a prompt: N(0,1) draws (Q and K times `gain`, which makes
    the softmax rows more peaked), as the projections of a real prompt are not available."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    Q = (torch.randn(B, Hq, L, D, generator=gen, device=dev) * gain).to(torch.float16)
    K = (torch.randn(B, Hkv, L, D, generator=gen, device=dev) * gain).to(torch.float16)
    V = torch.randn(B, Hkv, L, D, generator=gen, device=dev).to(torch.float16)
    return Q, K, V


def prefill_flops(B, Hq, L, D=128):
    """Floating-point operations of the two passes on the causal part: L(L+1)/2 (query, key) pairs per head,
    2D for a score and 2D for its share of the output in the first pass, 2D for the score again in the second."""
    pairs = L * (L + 1) // 2
    return B * Hq * pairs * (2 * D + 2 * D + 2 * D)


def make_scores(rows, L, seed, device="cpu", kind="attention"):
    """fp32 [rows, L] stand-ins for the cumulative attention score of each prompt token (the column sums
    of a causal attention map, one row per query head).  Real maps need a model; these have their shape:
    "attention": heavy-tailed positive values (a Pareto draw with tail index 1.2) times the share of query
                 rows that can see the column, (L - i) / L, with a few sink tokens at the start made large;
    "ties":      values on a grid of 8 levels, so most comparisons are between equal scores;
    "signed":    N(0,1) draws, negative values and both zeros included (not attention-like; exercises the
                 ordering of arbitrary finite floats).
    """
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    if kind == "attention":
        u = torch.rand(rows, L, generator=gen, device=dev, dtype=torch.float32).clamp_(min=1e-7)
        visible = (L - torch.arange(L, device=dev, dtype=torch.float32)) / float(L)
        a = (u.pow(-1.0 / 1.2) - 1.0 + 0.05) * visible
        a[:, : min(4, L)] *= 50.0
        return a.contiguous()
    if kind == "ties":
        return (torch.randint(0, 8, (rows, L), generator=gen, device=dev).to(torch.float32) / 8.0).contiguous()
    if kind == "signed":
        a = torch.randn(rows, L, generator=gen, device=dev, dtype=torch.float32)
        a[:, ::7] = 0.0
        a[:, 3::14] = -0.0
        return a.contiguous()
    raise ValueError(kind)


def selection_bytes(units, rep, L, n_tok):
    """Bytes the token selection must move: rep fp32 score rows of L tokens in, the kept positions
    (int32) and the three per-unit counts out/in."""
    return units * rep * L * 4 + int(sum(int(t) for t in n_tok)) * 4 + units * 12


def algorithmic_bytes(w: Workload, q_len, r_len):
    """Bytes one decode-attention step must move: per retained token 2*D/4 code bytes plus
    2*(D/G) fp16 (scale, zero) pairs for K and for V, i.e. 64 + 8*D/G bytes; per residual token
    4*D bytes (fp16 K and V rows); q in and out (2*B*Hq*D fp16); the two length arrays."""
    per_tok = 64 + 8 * w.D // w.G
    total = int(sum(int(t) for t in q_len)) * per_tok
    total += int(sum(int(r) for r in r_len)) * 4 * w.D
    total += 2 * w.B * w.Hq * w.D * 2
    total += 2 * 4 * w.units
    return total
