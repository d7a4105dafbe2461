"""Seeded synthetic workloads shaped like a dLLM denoising step's attention inputs.

This module only draws random numbers and lays them out in the packed
variable-length format the library takes (token-major Q [total_q, Hq, D],
K/V [total_kv, Hkv, D], prefix-sum offsets).  It holds none of the method's
arithmetic (no scoring, no selection, no softmax), so both the CPU oracle's
tests and the GPU path's tests can draw their inputs from it.

Shapes follow the paper's serving regime (Table 2: decoding block of 32,
generation 256, retention 10-50 %; Section 3.2: LLaDA-8B-like 32 heads x 128,
batch 16, L up to 2048), with activations replaced by seeded Gaussians since
neither the model weights nor the request traces exist here.

Draw order for every workload: per-sequence KV lengths, per-sequence keep
ratios, Q, K, V (fp32 normal), salient-row mask, sequence-order shuffle.
Casting to bf16 (round to nearest even) happens once, here, so that every
consumer sees identical bits.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional

import numpy as np
import torch

SEED_BASE = 20251217 * 10

MODE_SPARSE = 0
MODE_DENSE = 1


@dataclasses.dataclass
class Workload:
    """One packed variable-length batch (all tensors on the CPU)."""

    name: str
    dtype: torch.dtype                 # torch.float32 or torch.bfloat16
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    q: torch.Tensor                    # [total_q, Hq, D]
    k: torch.Tensor                    # [total_kv, Hkv, D]
    v: torch.Tensor                    # [total_kv, Hkv, D]
    cu_q: np.ndarray                   # int32 [B+1]
    cu_kv: np.ndarray                  # int32 [B+1]
    cu_k: np.ndarray                   # int32 [B+1]  prefix sums of kept rows per head
    seq_mode: np.ndarray               # uint8 [B]  MODE_SPARSE / MODE_DENSE
    softmax_scale: float

    @property
    def batch(self) -> int:
        return len(self.cu_q) - 1

    @property
    def q_lens(self) -> np.ndarray:
        return np.diff(self.cu_q)

    @property
    def kv_lens(self) -> np.ndarray:
        return np.diff(self.cu_kv)

    @property
    def keep(self) -> np.ndarray:
        return np.diff(self.cu_k)

    @property
    def total_q(self) -> int:
        return int(self.cu_q[-1])

    @property
    def total_kv(self) -> int:
        return int(self.cu_kv[-1])

    @property
    def total_k(self) -> int:
        return int(self.cu_k[-1])

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == torch.float32 else 2

    def select_bytes(self) -> int:
        """Algorithmic bytes of selection: K rows of sparse sequences streamed
        once per KV head, the block's Q rows, and the indices written."""
        e, d = self.elem_bytes, self.head_dim
        sp = self.seq_mode == MODE_SPARSE
        kv = int(self.kv_lens[sp].sum())
        nq = int(self.q_lens[sp].sum())
        nk = int(self.keep[sp].sum())
        return kv * self.n_kv_heads * d * e + nq * self.n_q_heads * d * e + nk * self.n_q_heads * 4

    def attend_sparse_bytes(self) -> int:
        """Algorithmic bytes of Reuse attention: one K row and one V row per
        kept (query head, position) pair, Q in, O out, indices in."""
        e, d = self.elem_bytes, self.head_dim
        sp = self.seq_mode == MODE_SPARSE
        nq = int(self.q_lens[sp].sum())
        nk = int(self.keep[sp].sum())
        return 2 * nk * self.n_q_heads * d * e + 2 * nq * self.n_q_heads * d * e + nk * self.n_q_heads * 4

    def pack_bytes(self) -> int:
        """Algorithmic bytes of packing: every kept (query head, position) pair reads one K row and
        one V row and writes them again, plus the indices read."""
        e, d = self.elem_bytes, self.head_dim
        sp = self.seq_mode == MODE_SPARSE
        nk = int(self.keep[sp].sum())
        return 4 * nk * self.n_q_heads * d * e + nk * self.n_q_heads * 4

    def attend_packed_bytes(self) -> int:
        """Algorithmic bytes of Reuse attention over a packed cache: as attend_sparse_bytes, without indices."""
        sp = self.seq_mode == MODE_SPARSE
        return self.attend_sparse_bytes() - int(self.keep[sp].sum()) * self.n_q_heads * 4

    def attend_dense_flops(self) -> int:
        """4 * Lq * Lkv * D per (sequence, query head) for dense sequences."""
        dn = self.seq_mode == MODE_DENSE
        pairs = int((self.q_lens[dn].astype(np.int64) * self.kv_lens[dn].astype(np.int64)).sum())
        return 4 * pairs * self.head_dim * self.n_q_heads

    def attend_sparse_flops(self) -> int:
        sp = self.seq_mode == MODE_SPARSE
        pairs = int((self.q_lens[sp].astype(np.int64) * self.keep[sp].astype(np.int64)).sum())
        return 4 * pairs * self.head_dim * self.n_q_heads


def keep_count(ratio: float, kv_len: int) -> int:
    """Rows kept per head for a retention ratio: nearest integer, at least 1."""
    return max(1, min(int(kv_len), int(math.floor(float(ratio) * int(kv_len) + 0.5))))


def _prefix(x) -> np.ndarray:
    out = np.zeros(len(x) + 1, dtype=np.int64)
    np.cumsum(np.asarray(x, dtype=np.int64), out=out[1:])
    assert out[-1] < 2**31
    return out.astype(np.int32)


def _normal(shape, gen: torch.Generator, dtype: torch.dtype, chunk_rows: int = 1 << 15) -> torch.Tensor:
    """N(0,1) in fp32 drawn from `gen`, cast once to `dtype` (chunked so the
    fp32 staging copy stays small for the large workloads)."""
    out = torch.empty(shape, dtype=dtype)
    n = shape[0]
    for r0 in range(0, n, chunk_rows):
        r1 = min(n, r0 + chunk_rows)
        blk = torch.randn((r1 - r0,) + tuple(shape[1:]), generator=gen, dtype=torch.float32)
        out[r0:r1] = blk.to(dtype)
    return out


def make_workload(
    name: str,
    seed: int,
    dtype: torch.dtype,
    n_q_heads: int,
    n_kv_heads: int,
    head_dim: int,
    kv_lens,
    q_lens,
    keep,
    seq_mode=None,
    salient_frac: float = 0.0,
    salient_gain: float = 4.0,
    softmax_scale: Optional[float] = None,
    gen: Optional[torch.Generator] = None,
) -> Workload:
    """Draw Q, K, V for given per-sequence lengths (lengths already decided)."""
    if gen is None:
        gen = torch.Generator(device="cpu")
        gen.manual_seed(seed)
    kv_lens = np.asarray(kv_lens, dtype=np.int64)
    q_lens = np.asarray(q_lens, dtype=np.int64)
    keep = np.asarray(keep, dtype=np.int64)
    nb = len(kv_lens)
    assert len(q_lens) == nb and len(keep) == nb
    if seq_mode is None:
        seq_mode = np.zeros(nb, dtype=np.uint8)
    seq_mode = np.asarray(seq_mode, dtype=np.uint8)
    cu_q, cu_kv, cu_k = _prefix(q_lens), _prefix(kv_lens), _prefix(keep)
    tq, tkv = int(cu_q[-1]), int(cu_kv[-1])
    q = _normal((tq, n_q_heads, head_dim), gen, dtype)
    k = _normal((tkv, n_kv_heads, head_dim), gen, dtype)
    v = _normal((tkv, n_kv_heads, head_dim), gen, dtype)
    if salient_frac > 0.0 and tkv > 0:
        # each (token, kv-head) row independently, so heads favour different tokens
        mask = torch.rand((tkv, n_kv_heads), generator=gen) < salient_frac
        k = torch.where(mask[:, :, None], (k.float() * salient_gain).to(dtype), k)
    if softmax_scale is None:
        softmax_scale = 1.0 / math.sqrt(head_dim)
    return Workload(name, dtype, n_q_heads, n_kv_heads, head_dim, q, k, v,
                    cu_q, cu_kv, cu_k, seq_mode, float(softmax_scale))


def subset(w: Workload, seqs, name: Optional[str] = None) -> Workload:
    """The sequences `seqs` (batch positions, in the given order) of a workload as a batch of their own."""
    seqs = [int(b) for b in seqs]
    qrows = [torch.arange(int(w.cu_q[b]), int(w.cu_q[b + 1])) for b in seqs]
    kvrows = [torch.arange(int(w.cu_kv[b]), int(w.cu_kv[b + 1])) for b in seqs]
    qsel = torch.cat(qrows) if qrows else torch.zeros(0, dtype=torch.long)
    kvsel = torch.cat(kvrows) if kvrows else torch.zeros(0, dtype=torch.long)
    return Workload(name or w.name + "_subset", w.dtype, w.n_q_heads, w.n_kv_heads, w.head_dim,
                    w.q[qsel].contiguous(), w.k[kvsel].contiguous(), w.v[kvsel].contiguous(),
                    _prefix(w.q_lens[seqs]), _prefix(w.kv_lens[seqs]), _prefix(w.keep[seqs]),
                    w.seq_mode[seqs].copy(), w.softmax_scale)


def with_keep(w: Workload, keep, name: Optional[str] = None) -> Workload:
    """The same batch with other per-sequence numbers of kept rows (tensors shared, offsets rebuilt)."""
    keep = np.asarray(keep, dtype=np.int64)
    assert len(keep) == w.batch and (keep <= w.kv_lens).all() and (keep >= 0).all()
    return dataclasses.replace(w, name=name or w.name + "_rekept", cu_k=_prefix(keep), seq_mode=w.seq_mode.copy())


def at_retention(w: Workload, ratio: float, name: Optional[str] = None) -> Workload:
    """The same batch with every sparse sequence keeping `ratio` of its positions (Table 2's default is 0.5)."""
    keep = [keep_count(ratio, l) if m == MODE_SPARSE else 0 for l, m in zip(w.kv_lens, w.seq_mode)]
    return with_keep(w, keep, name or f"{w.name}_r{ratio:g}")


def config(c: int, scale_down: int = 1) -> Workload:
    """The five benchmark workloads.  `scale_down` > 1 divides sequence lengths
    (configs 3-5) to get a same-structure case the CPU oracle finishes quickly."""
    seed = SEED_BASE + c
    gen = torch.Generator(device="cpu")
    gen.manual_seed(seed)
    if c == 1:
        # tiny single layer, fp32: 4 heads x 64, KV 256, block 32, keep 64
        return make_workload("c1_tiny_fp32", seed, torch.float32, 4, 4, 64,
                             [256], [32], [64], gen=gen)
    if c == 2:
        # LLaDA-8B-shaped layer: prompt 768 + generation 256, keep 25 %
        return make_workload("c2_llada_layer", seed, torch.bfloat16, 32, 32, 128,
                             [1024], [32], [keep_count(0.25, 1024)], gen=gen)
    if c == 3:
        # batched Reuse phase: 16 sequences, KV ~ U{512..4096}, keep ratio ~ U[0.1, 0.5]
        nb = 16
        lo, hi = 512 // scale_down, 4096 // scale_down
        lens = torch.randint(lo, hi + 1, (nb,), generator=gen).numpy().astype(np.int64)
        ratios = (0.1 + 0.4 * torch.rand((nb,), generator=gen, dtype=torch.float64)).numpy()
        keep = [keep_count(r, l) for r, l in zip(ratios, lens)]
        return make_workload("c3_batched_reuse", seed, torch.bfloat16, 32, 32, 128,
                             lens, [32] * nb, keep, salient_frac=0.05, gen=gen)
    if c == 4:
        # Refresh phase: dense bidirectional attention, 8 x L=2048
        nb, L = 8, 2048 // scale_down
        return make_workload("c4_refresh_dense", seed, torch.bfloat16, 32, 32, 128,
                             [L] * nb, [L] * nb, [0] * nb,
                             seq_mode=np.ones(nb, dtype=np.uint8), gen=gen)
    if c == 5:
        # long-context mixed burst, GQA 32/8: 24 Reuse (KV 8192, keep 5 %) + 8 Refresh (L=2048)
        n_reuse, n_refresh = 24, 8
        l_reuse, l_refresh = 8192 // scale_down, 2048 // scale_down
        order = torch.randperm(n_reuse + n_refresh, generator=gen).numpy()
        mode = np.zeros(n_reuse + n_refresh, dtype=np.uint8)
        mode[order[:n_refresh]] = MODE_DENSE
        kv = np.where(mode == MODE_DENSE, l_refresh, l_reuse)
        ql = np.where(mode == MODE_DENSE, l_refresh, 32)
        keep = np.where(mode == MODE_DENSE, 0, keep_count(0.05, l_reuse))
        return make_workload("c5_mixed_burst_gqa", seed, torch.bfloat16, 32, 8, 128,
                             kv, ql, keep, seq_mode=mode, gen=gen)
    raise ValueError(f"unknown config {c}")


def to_bits(t: torch.Tensor) -> np.ndarray:
    """CPU tensor -> numpy array the oracle takes: float32 as is, bf16 as its
    raw uint16 bit patterns (numpy has no bf16)."""
    t = t.contiguous()
    if t.dtype == torch.float32:
        return t.numpy()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    raise TypeError(t.dtype)
