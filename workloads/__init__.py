"""Seeded synthetic inputs for the PaRO update-stage hot path.

This module is the only code shared by the CPU oracle's tests and the HIP
path's tests / benchmark.  It holds no arithmetic of the method: it only
names tensor-size lists and draws random buffers (torch's own generators and
dtype casts).  The paper trains LLaMA-7B / LLaMA-65B on C4 (Sec. 4.2); the
update stage is oblivious to the values it streams, so the shapes below with
seeded random gradients stand in for that workload.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import torch

BF16 = 0  # gradient dtype codes, same numbering on both sides of the boundary
F32 = 1
F16 = 2
TORCH_DTYPE = {BF16: torch.bfloat16, F32: torch.float32, F16: torch.float16}

ADAM_DEFAULT = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)


# --------------------------------------------------------------------------
# tensor-size lists
# --------------------------------------------------------------------------
def gpt2_small_sizes() -> List[int]:
    """GPT-2-small-shaped list: two embeddings, 12 blocks of four matrices and
    four 768-vectors, and a final pair of 768-vectors (100 tensors)."""
    d = 768
    sizes = [50257 * d, 1024 * d]
    for _ in range(12):
        sizes += [d, d, d * 3 * d, d * d, d, d, d * 4 * d, 4 * d * d]
    sizes += [d, d]
    return sizes


def gpt2_small_no_decay() -> List[int]:
    """1 for the 768-vectors (norm gains / biases), 0 for matrices."""
    return [1 if s == 768 else 0 for s in gpt2_small_sizes()]


def llama_total(layers: int, d: int, ffn: int, vocab: int) -> int:
    """Parameter count of a Llama-shaped decoder: per layer four d*d attention
    matrices, three d*ffn MLP matrices and two d-vectors; two vocab*d
    embeddings and a final d-vector."""
    return layers * (4 * d * d + 3 * d * ffn + 2 * d) + 2 * vocab * d + d


def llama7b_total() -> int:
    return llama_total(32, 4096, 11008, 32000)


def llama_sizes(layers: int, d: int, ffn: int, vocab: int) -> List[int]:
    """The tensor list behind llama_total, in model order: the input embedding;
    per layer a d-vector, four d*d matrices, a d-vector and three d*ffn
    matrices; the final d-vector and the output embedding."""
    sizes = [vocab * d]
    for _ in range(layers):
        sizes += [d, d * d, d * d, d * d, d * d, d, d * ffn, d * ffn, ffn * d]
    sizes += [d, vocab * d]
    return sizes


def llama7b_sizes() -> List[int]:
    return llama_sizes(32, 4096, 11008, 32000)


def llama65b_sizes() -> List[int]:
    return llama_sizes(80, 8192, 22016, 32000)


def llama65b_total() -> int:
    return llama_total(80, 8192, 22016, 32000)


def ragged_sizes(n: int = 10000, seed: int = 5, lo: int = 1, hi: int = 65536) -> List[int]:
    """n sizes log-uniform in [lo, hi]: floor(2**(log2(hi) * u)), u ~ U[0,1)."""
    gen = torch.Generator().manual_seed(seed)
    u = torch.rand(n, generator=gen, dtype=torch.float64)
    s = torch.floor(torch.pow(2.0, math.log2(hi) * u)).to(torch.int64).clamp_(lo, hi)
    return [int(x) for x in s]


def ragged_dtypes(n: int = 10000, seed: int = 55, frac_f32: float = 0.25) -> List[int]:
    gen = torch.Generator().manual_seed(seed)
    u = torch.rand(n, generator=gen, dtype=torch.float64)
    return [F32 if float(x) < frac_f32 else BF16 for x in u]


# --------------------------------------------------------------------------
# named configurations (cluster shape + strategy; sizes resolved lazily)
# --------------------------------------------------------------------------
@dataclass
class Config:
    name: str
    P: int                      # number of ranks in the cluster
    G: int                      # ranks per group
    strategy: str               # param / grad / optimizer-state letters
    sizes: List[int]
    max_norm: float = 0.0
    steps: int = 1
    layout: str = "chunk"       # "chunk" or "tensors"
    dist: str = "normal"        # "normal" | "student_t"
    dtypes: Optional[List[int]] = None
    no_decay: Optional[List[int]] = None
    adam: dict = field(default_factory=lambda: dict(ADAM_DEFAULT))


def config(name: str) -> Config:
    if name == "tiny":
        return Config("tiny", 4, 2, "IIG", [1 << 20], max_norm=0.0, steps=1)
    if name == "gpt2":
        return Config("gpt2", 8, 8, "NGG", gpt2_small_sizes(), max_norm=1.0, steps=3,
                      layout="tensors", no_decay=gpt2_small_no_decay())
    if name == "llama7b_share":
        return Config("llama7b_share", 16, 8, "IIG", [llama7b_total()], max_norm=1.0)
    if name == "llama65b_share":
        return Config("llama65b_share", 64, 8, "IGG", [llama65b_total()], max_norm=1.0)
    if name == "ragged":
        return Config("ragged", 8, 4, "IIG", ragged_sizes(), max_norm=1.0, steps=5,
                      layout="tensors", dist="student_t", dtypes=ragged_dtypes())
    raise KeyError(name)


# --------------------------------------------------------------------------
# random buffers
# --------------------------------------------------------------------------
def _seed(base: int, step: int, rank: int, salt: int = 0) -> int:
    return (base * 1_000_003 + step * 10_007 + rank * 101 + salt) & 0x7FFFFFFFFFFFFFFF


def _generator(device, seed: int) -> torch.Generator:
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    return gen


def draw(n: int, seed: int, *, dist: str = "normal", scale: float = 1e-3,
         dtype: int = BF16, device="cpu", piece: int = 1 << 27) -> torch.Tensor:
    """n seeded values, scale * N(0,1) or scale * Student-t(df=3), as bf16 or
    fp32.  Drawn in pieces so the fp32 temporaries stay small on the device."""
    tdt = TORCH_DTYPE[dtype]
    out = torch.empty(n, dtype=tdt, device=device)
    gen = _generator(device, seed)
    for lo in range(0, n, piece):
        m = min(piece, n - lo)
        z = torch.randn(m, generator=gen, device=device, dtype=torch.float32)
        if dist == "student_t":
            chi = torch.zeros(m, device=device, dtype=torch.float32)
            for _ in range(3):
                w = torch.randn(m, generator=gen, device=device, dtype=torch.float32)
                chi += w * w
            z = z / torch.sqrt(chi / 3.0)
        elif dist != "normal":
            raise ValueError(dist)
        out[lo:lo + m] = (z * scale).to(tdt)
    return out


def draw_int(n: int, seed: int, *, lo: int = -8, hi: int = 8, dtype: int = BF16,
             device="cpu") -> torch.Tensor:
    """Small-integer-valued gradients (exactly representable in bf16)."""
    gen = _generator(device, seed)
    z = torch.randint(lo, hi + 1, (n,), generator=gen, device=device, dtype=torch.int32)
    return z.to(TORCH_DTYPE[dtype])


def chunk_contribs(P: int, n: int, base_seed: int, step: int = 0, *, dist="normal",
                   dtype: int = BF16, device="cpu", integer: bool = False) -> List[torch.Tensor]:
    """One buffer of n gradient elements per simulated rank (shard coordinates)."""
    out = []
    for q in range(P):
        s = _seed(base_seed, step, q)
        out.append(draw_int(n, s, dtype=dtype, device=device) if integer
                   else draw(n, s, dist=dist, dtype=dtype, device=device))
    return out


@dataclass
class TensorSet:
    """One simulated rank's full gradients: tensors[t] is a view into flat[dtype]
    starting at element start[t]."""
    tensors: List[torch.Tensor]
    flat: dict
    start: List[int]


def tensor_contribs(P: int, sizes: List[int], dtypes: Optional[List[int]], base_seed: int,
                    step: int = 0, *, dist="normal", device="cpu", align_elems: int = 128) -> List[TensorSet]:
    """Per simulated rank, one full gradient per tensor.  Values are drawn as one
    flat stream per (rank, dtype) and tensors are views into it, each starting on
    a multiple of align_elems elements (128 = the alignment separate allocations
    would have; 1 = packed tight, arbitrary base alignment)."""
    kinds = sorted(set(dtypes)) if dtypes is not None else [BF16]
    start, fill = [], {k: 0 for k in kinds}
    for t, n in enumerate(sizes):
        k = dtypes[t] if dtypes is not None else BF16
        start.append(fill[k])
        fill[k] += -(-n // align_elems) * align_elems
    out = []
    for q in range(P):
        flat = {k: draw(max(fill[k], 1), _seed(base_seed, step, q, salt=k + 1), dist=dist, dtype=k, device=device)
                for k in kinds}
        per = []
        for t, n in enumerate(sizes):
            k = dtypes[t] if dtypes is not None else BF16
            per.append(flat[k][start[t]:start[t] + n])
        out.append(TensorSet(per, flat, start))
    return out


def tensor_contribs_over_range(P: int, sizes: List[int], begin: int, length: int, base_seed: int, step: int = 0, *,
                               dist="normal", device="cpu") -> List[TensorSet]:
    """Like tensor_contribs for all-bf16 lists too large to hold P times: per
    simulated rank only the tensors that meet flat elements [begin, begin+length)
    exist (whole, packed back to back); tensors[t] is None for the others, which a
    step over that range never reads."""
    first, last, off = None, None, 0
    offs = []
    for t, n in enumerate(sizes):
        offs.append(off)
        if n and off < begin + length and off + n > begin:
            first = t if first is None else first
            last = t
        off += n
    assert first is not None
    span = offs[last] + sizes[last] - offs[first]
    out = []
    for q in range(P):
        flat = draw(span, _seed(base_seed, step, q, salt=1), dist=dist, dtype=BF16, device=device)
        per: List[Optional[torch.Tensor]] = [None] * len(sizes)
        start = [0] * len(sizes)
        for t in range(first, last + 1):
            start[t] = offs[t] - offs[first]
            per[t] = flat[start[t]:start[t] + sizes[t]]
        out.append(TensorSet(per, {BF16: flat}, start))
    return out


def master_state(n: int, base_seed: int, *, device="cpu"):
    """fp32 master parameters N(0, 0.02) and zero first / second moments."""
    p = draw(n, _seed(base_seed, 0, 0, salt=77), scale=0.02, dtype=F32, device=device)
    m = torch.zeros(n, dtype=torch.float32, device=device)
    v = torch.zeros(n, dtype=torch.float32, device=device)
    return p, m, v
