"""Seeded synthetic inputs shaped like the paper's long-context decode workloads.

This module holds input generation only -- none of the attention arithmetic.  Both the HIP path
and the CPU oracle consume the tensors made here (the same bits), and neither is imported here.

The five standard workloads mirror a tiny MHA case, three OPT-family decoder-layer shapes
(heads x head_dim of the 6.7B / 13B / 30B models the paper's evaluation section draws on, here
with longer contexts) and a 70B-class grouped-query layer.  Real model weights and evaluation
data are replaced by N(0,1) tensors of those shapes; see ``WORKLOADS``.

Recipe (every draw seeded; seed 0 unless stated):
  * q, K, V are drawn as fp32 N(0,1), one (sequence, KV head) slab at a time, and rounded once
    to the storage dtype.
  * "outlier channels": per KV head, 4 distinct channels (seeded choice) are multiplied by 8
    after rounding (exact in fp16).
  * partition tables are positional ranges that tile [0, N_b) exactly once:
      - "at": fixed cut points;  - "half": one cut at N_b // 2;
      - "ratios": w_i ~ U[0.1, 0.8], cut points round(N_b * cumsum(w / sum w));
      - "dirichlet": r ~ Dirichlet(1,...,1), cut points round(N_b * cumsum r); empty ranges kept.
"""
from __future__ import annotations

import dataclasses
import math
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch

Range = Tuple[int, int, int]  # (seq, begin, end)


@dataclasses.dataclass(frozen=True)
class WorkloadSpec:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str  # "f16" | "f32" | "bf16"
    n_min: int  # context length is uniform in [n_min, n_max]
    n_max: int
    partition: str  # "at" | "half" | "ratios" | "dirichlet" | "none"
    n_parts: int = 1
    cuts: Tuple[int, ...] = ()
    outlier_k: bool = False
    outlier_v: bool = False
    seed: int = 0

    def scaled(self, **kw) -> "WorkloadSpec":
        return dataclasses.replace(self, **kw)


# The benchmark configurations, in order.  Index 1 is the one the headline metric is timed on.
WORKLOADS: List[WorkloadSpec] = [
    WorkloadSpec("tiny-mha-512", 1, 4, 4, 64, "f32", 512, 512, "at", 2, cuts=(300,)),
    WorkloadSpec("opt6.7b-b8-8k", 8, 32, 32, 128, "f16", 8192, 8192, "half", 2, outlier_k=True, outlier_v=True),
    WorkloadSpec("opt13b-b16-ragged16k-32k", 16, 40, 40, 128, "f16", 16384, 32768, "ratios", 3),
    WorkloadSpec("opt30b-b4-128k", 4, 56, 56, 128, "f16", 131072, 131072, "dirichlet", 8),
    WorkloadSpec("gqa70b-b1-1m", 1, 64, 8, 128, "f16", 1048576, 1048576, "dirichlet", 16, outlier_k=True),
]

# Further shapes, measured and parity-tested like the benchmark configurations but not part of
# them: they exercise kernel variants that no benchmark configuration reaches.  Indices continue
# after WORKLOADS (ALL_WORKLOADS[5] is the first).
EXTRA_WORKLOADS: List[WorkloadSpec] = [
    # fp16, head_dim 64, 4 query heads per KV head: the matrix-core kernel for 128-byte rows
    WorkloadSpec("gqa4-d64-b8-64k", 8, 32, 8, 64, "f16", 65536, 65536, "dirichlet", 4, seed=5),
    # bf16, head_dim 128, 4 query heads per KV head (the head structure of an 8B Llama-class model)
    WorkloadSpec("gqa4-d128-bf16-b8-32k", 8, 32, 8, 128, "bf16", 32768, 32768, "dirichlet", 4, seed=6),
]
ALL_WORKLOADS: List[WorkloadSpec] = WORKLOADS + EXTRA_WORKLOADS


@dataclasses.dataclass
class Workload:
    spec: WorkloadSpec
    q: torch.Tensor  # [B, Hq, d]
    k: torch.Tensor  # [B, Hkv, Nmax, d]  (or a strided view, see layout)
    v: torch.Tensor
    seq_lens: np.ndarray  # int32 [B]
    scale: float
    ranges: List[Range]  # all sequences, grouped by sequence, ascending token order
    group_ptr: np.ndarray  # int32 [B+1]: ranges[group_ptr[b]:group_ptr[b+1]] belong to sequence b

    @property
    def kv_bytes(self) -> int:
        """K and V bytes inside the valid caches, each row counted once per KV head."""
        es = self.k.element_size()
        return int(2 * self.spec.n_kv_heads * int(self.seq_lens.sum()) * self.spec.head_dim * es)


def _torch_dtype(name: str) -> torch.dtype:
    return {"f16": torch.float16, "f32": torch.float32, "bf16": torch.bfloat16}[name]


def _stream_seed(seed: int, *keys: int) -> int:
    """Independent stream ids from small integer keys (no hashing of strings, no arithmetic of
    the method): a fixed mixed-radix combination."""
    s = seed
    for key in keys:
        s = (s * 1000003 + key + 1) % (2**31 - 1)
    return s


def make_seq_lens(spec: WorkloadSpec) -> np.ndarray:
    rng = np.random.RandomState(_stream_seed(spec.seed, 11))
    if spec.n_min == spec.n_max:
        return np.full(spec.batch, spec.n_max, dtype=np.int32)
    return rng.randint(spec.n_min, spec.n_max + 1, size=spec.batch).astype(np.int32)


def make_partitions(spec: WorkloadSpec, seq_lens: np.ndarray) -> Tuple[List[Range], np.ndarray]:
    """Positional ranges per sequence that tile [0, N_b) exactly once (empty ranges allowed)."""
    rng = np.random.RandomState(_stream_seed(spec.seed, 13))
    ranges: List[Range] = []
    group_ptr = [0]
    for b in range(spec.batch):
        n = int(seq_lens[b])
        if spec.partition == "none":
            bounds = [0, n]
        elif spec.partition == "at":
            bounds = [0] + [min(int(c), n) for c in spec.cuts] + [n]
        elif spec.partition == "half":
            bounds = [0, n // 2, n]
        elif spec.partition == "ratios":
            w = rng.uniform(0.1, 0.8, size=spec.n_parts)
            cum = np.cumsum(w / w.sum())
            bounds = [0] + [int(round(n * c)) for c in cum]
        elif spec.partition == "dirichlet":
            r = rng.dirichlet(np.ones(spec.n_parts))
            cum = np.cumsum(r)
            bounds = [0] + [int(round(n * c)) for c in cum]
        else:
            raise ValueError(spec.partition)
        bounds[-1] = n
        for i in range(1, len(bounds)):  # keep the cut points monotone after rounding
            bounds[i] = min(max(bounds[i], bounds[i - 1]), n)
        for i in range(len(bounds) - 1):
            ranges.append((b, bounds[i], bounds[i + 1]))
        group_ptr.append(len(ranges))
    return ranges, np.asarray(group_ptr, dtype=np.int32)


def _outlier_channels(spec: WorkloadSpec, which: int) -> np.ndarray:
    """[B, Hkv, 4] distinct channel indices per KV head."""
    rng = np.random.RandomState(_stream_seed(spec.seed, 17, which))
    idx = np.empty((spec.batch, spec.n_kv_heads, 4), dtype=np.int64)
    for b in range(spec.batch):
        for g in range(spec.n_kv_heads):
            idx[b, g] = rng.choice(spec.head_dim, size=4, replace=False)
    return idx


def _fill_normal(dst: torch.Tensor, seed: int) -> None:
    """dst[...] <- N(0,1) drawn in fp32 on dst's device, rounded once to dst's dtype.
    Filled slab by slab over the leading axes so the fp32 temporary stays small."""
    gen = torch.Generator(device=dst.device)
    gen.manual_seed(seed)
    if dst.ndim <= 2:
        dst.copy_(torch.randn(dst.shape, generator=gen, device=dst.device, dtype=torch.float32))
        return
    flat = dst.reshape(-1, dst.shape[-2], dst.shape[-1]) if dst.is_contiguous() else None
    if flat is None:
        for i in range(dst.shape[0]):
            _fill_normal(dst[i], _stream_seed(seed, i))
        return
    for i in range(flat.shape[0]):
        flat[i].copy_(torch.randn(flat[i].shape, generator=gen, device=dst.device, dtype=torch.float32))


def make_workload(spec: WorkloadSpec, device="cpu", layout: str = "bhtd") -> Workload:
    """Build the tensors of a workload on ``device``.

    layout "bhtd": K, V are contiguous [B, Hkv, Nmax, d] (stride_t = d).
    layout "bthd": storage is [B, Nmax, Hkv, d]; the returned K, V are the [B, Hkv, Nmax, d]
                   views of it (stride_t = Hkv * d, stride_h = d).
    Rows at t >= seq_lens[b] hold finite filler that no correct reader touches.
    """
    dt = _torch_dtype(spec.dtype)
    dev = torch.device(device)
    B, Hq, Hkv, d, nmax = spec.batch, spec.n_q_heads, spec.n_kv_heads, spec.head_dim, spec.n_max
    seq_lens = make_seq_lens(spec)
    ranges, group_ptr = make_partitions(spec, seq_lens)

    q = torch.empty((B, Hq, d), dtype=dt, device=dev)
    _fill_normal(q, _stream_seed(spec.seed, 1))
    if layout == "bhtd":
        k = torch.empty((B, Hkv, nmax, d), dtype=dt, device=dev)
        v = torch.empty((B, Hkv, nmax, d), dtype=dt, device=dev)
        _fill_normal(k, _stream_seed(spec.seed, 2))
        _fill_normal(v, _stream_seed(spec.seed, 3))
    elif layout == "bthd":
        ks = torch.empty((B, nmax, Hkv, d), dtype=dt, device=dev)
        vs = torch.empty((B, nmax, Hkv, d), dtype=dt, device=dev)
        _fill_normal(ks, _stream_seed(spec.seed, 2))
        _fill_normal(vs, _stream_seed(spec.seed, 3))
        k, v = ks.permute(0, 2, 1, 3), vs.permute(0, 2, 1, 3)
    else:
        raise ValueError(layout)

    for flag, tensor, which in ((spec.outlier_k, k, 0), (spec.outlier_v, v, 1)):
        if not flag:
            continue
        idx = _outlier_channels(spec, which)
        for b in range(B):
            for g in range(Hkv):
                ch = torch.as_tensor(idx[b, g], device=dev)
                tensor[b, g, :, ch] = tensor[b, g, :, ch] * 8
    return Workload(spec, q, k, v, seq_lens, 1.0 / math.sqrt(d), ranges, group_ptr)


def bitplane_values(n_tokens: int, head_dim: int, dtype: torch.dtype, device="cpu") -> torch.Tensor:
    """[n_tokens, head_dim] with entry (j, c) = bit c of the token index j for c < 24, else 0.
    With all-zero queries every softmax weight is equal, so the unnormalised value sum of a
    range is, per channel, the COUNT of member tokens whose index has that bit set -- an integer
    that pins exactly which tokens a range covered."""
    j = torch.arange(n_tokens, device=device, dtype=torch.int64).unsqueeze(1)
    c = torch.arange(head_dim, device=device, dtype=torch.int64).unsqueeze(0)
    bits = torch.where(c < 24, (j >> torch.clamp(c, max=23)) & 1, torch.zeros_like(j))
    return bits.to(dtype)


def random_ranges(seq_lens: Sequence[int], n_ranges: int, seed: int, max_len: Optional[int] = None) -> List[Range]:
    """Arbitrary (possibly overlapping, empty, unordered) ranges for stress tests."""
    rng = np.random.RandomState(seed)
    out: List[Range] = []
    B = len(seq_lens)
    for _ in range(n_ranges):
        b = int(rng.randint(0, B))
        n = int(seq_lens[b])
        a = int(rng.randint(0, n + 1))
        e = int(rng.randint(a, n + 1))
        if max_len is not None:
            e = min(e, a + max_len)
        out.append((b, a, e))
    return out


def proxy_query(q: torch.Tensor, cosine: float, seed: int) -> torch.Tensor:
    """A stand-in for the paper's proxy query (the previous layer's input pushed through this
    layer's weights, Section 4.2): q rotated towards seeded noise so that every head's cosine
    similarity to the true query is `cosine`, same norm, rounded once to q's dtype."""
    gen = torch.Generator(device=q.device)
    gen.manual_seed(_stream_seed(seed, 23))
    q32 = q.float()
    noise = torch.randn(q32.shape, generator=gen, device=q.device, dtype=torch.float32)
    qn = q32 / q32.norm(dim=-1, keepdim=True)
    noise = noise - (noise * qn).sum(-1, keepdim=True) * qn  # orthogonal to q
    noise = noise / noise.norm(dim=-1, keepdim=True)
    mixed = cosine * qn + math.sqrt(max(0.0, 1.0 - cosine * cosine)) * noise
    return (mixed * q32.norm(dim=-1, keepdim=True)).to(q.dtype)


def make_dyadic_(w: "Workload", seed: int) -> None:
    """Overwrite q and K of a workload, in place, with seeded multiples of 1/4 in [-2, 2].  With a
    power-of-two scale every logit is then exact in fp32 (and in any summation order), so a
    selection decided on fp32 logits and one decided on exactly computed logits must agree bit
    for bit, ties included -- of which such coarse values produce many."""
    gen = torch.Generator(device=w.q.device)
    gen.manual_seed(_stream_seed(seed, 31))
    for t in (w.q, w.k):
        vals = torch.randint(-8, 9, t.shape, generator=gen, device=t.device, dtype=torch.int32)
        t.copy_((vals.float() / 4).to(t.dtype))


def listed_tokens(limits: Sequence[int], n_q_heads: int, max_k: int, seed: int) -> np.ndarray:
    """A stand-in for a Pre-QK^T token selector (Section 4.3.2; Section 4.5): per (sequence,
    query head) up to `max_k` distinct token positions below limits[b], seeded, in ascending
    order, -1 padded.  Returns int32 [B, Hq, max_k].  The paper's selectors are third-party
    predictors that need trained models; what the executor receives from any of them is such a
    list, and its cost depends only on the list's length and scatter."""
    rng = np.random.RandomState(_stream_seed(seed, 29) % (2 ** 31))
    B = len(limits)
    idx = np.full((B, n_q_heads, max_k), -1, dtype=np.int32)
    for b in range(B):
        n = int(limits[b])
        kk = min(max_k, n)
        for h in range(n_q_heads):
            if n <= 4 * max_k:
                row = rng.permutation(n)[:kk]
            else:  # long caches: draw with replacement, de-duplicate, top up
                row = np.unique(rng.randint(0, n, size=2 * kk))
                rng.shuffle(row)
                row = row[:kk]
            idx[b, h, :row.size] = np.sort(row)
    return idx


def make_paged(w: Workload, block_tokens: int, seed: int = 0):
    """The same cache as a paged pool: K, V pools [n_blocks, Hkv, block_tokens, d] whose physical
    blocks are in a seeded random order, and the block table int32 [B, max_blocks] (unused
    entries point at block 0, which holds real data of some other place, so that a reader which
    consults them computes a wrong answer rather than touching unmapped memory)."""
    B, Hkv, nmax, d = w.k.shape
    bt = int(block_tokens)
    per_seq = [(int(n) + bt - 1) // bt for n in w.seq_lens]
    max_blocks = max(max(per_seq), 1)
    n_blocks = max(sum(per_seq), 1)
    rng = np.random.RandomState(_stream_seed(seed, 29))
    perm = rng.permutation(n_blocks)
    table = np.zeros((B, max_blocks), dtype=np.int32)
    dev = w.k.device
    k_pool = torch.zeros((n_blocks, Hkv, bt, d), dtype=w.k.dtype, device=dev)
    v_pool = torch.zeros((n_blocks, Hkv, bt, d), dtype=w.v.dtype, device=dev)
    nxt = 0
    for b in range(B):
        n = int(w.seq_lens[b])
        for i in range(per_seq[b]):
            p = int(perm[nxt])
            nxt += 1
            table[b, i] = p
            rows = min(bt, n - i * bt)
            k_pool[p, :, :rows] = w.k[b, :, i * bt:i * bt + rows]
            v_pool[p, :, :rows] = w.v[b, :, i * bt:i * bt + rows]
    return k_pool, v_pool, torch.from_numpy(table).to(dev)
