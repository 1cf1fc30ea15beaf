"""Seeded synthetic inputs for the ESP attention hot path.

This module only *draws and arranges* inputs: random bf16 tensors, token
positions of contiguous / striped sequence-parallel layouts (LoongServe,
arXiv 2404.09526, Sec. 2.3 / Fig. 1), request-length mixes that stand in for
the paper's ShareGPT / L-Eval / LV-Eval traces (Sec. 7.1), and the slot
assignment of a token-granular KV pool (Sec. 6).  It contains none of the
method's arithmetic (no scores, softmax, merge or scatter) and is the only
module used by both the HIP path's callers and the CPU oracle's callers.

Values: Q, K, V ~ N(0,1) drawn in fp32 from a seeded torch generator on the
target device, in the fixed order Q, K, V, (pool rows, new rows, partials),
then rounded to bf16 (round-to-nearest-even).  The materialised bf16 tensors
are what both sides read.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

HEAD_DIM = 128


# --------------------------------------------------------------------------- helpers
def randn_bf16(shape, gen: torch.Generator, device, chunk_rows: int = 1 << 16) -> torch.Tensor:
    """N(0,1) in fp32 -> bf16, drawn in row chunks so the fp32 temporary stays small."""
    shape = tuple(int(s) for s in shape)
    out = torch.empty(shape, dtype=torch.bfloat16, device=device)
    if out.numel() == 0:
        return out
    flat = out.view(shape[0], -1)
    for lo in range(0, shape[0], chunk_rows):
        hi = min(shape[0], lo + chunk_rows)
        flat[lo:hi] = torch.randn((hi - lo, flat.shape[1]), generator=gen, device=device,
                                  dtype=torch.float32).to(torch.bfloat16)
    return out


def bits(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> numpy uint16 bit patterns on the host (what the oracle reads)."""
    assert t.dtype == torch.bfloat16
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def host_i32(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy().astype(np.int32)


def lognormal_lengths(n: int, median: int, lo: int, hi: int, seed: int, sigma: float = 1.0) -> np.ndarray:
    """len = clip(floor(exp(ln(median) + sigma*z)), lo, hi), z ~ N(0,1) from numpy default_rng(seed)."""
    z = np.random.default_rng(seed).standard_normal(n)
    return np.clip(np.floor(np.exp(math.log(median) + sigma * z)), lo, hi).astype(np.int64)


# --------------------------------------------------------------------------- prefill
@dataclass
class Shard:
    k: torch.Tensor          # bf16 [Tkv, Hkv, D]
    v: torch.Tensor          # bf16 [Tkv, Hkv, D]
    kv_pos: torch.Tensor     # int32 [Tkv] global token positions
    cu_kv: torch.Tensor      # int32 [batch+1] request offsets into the shard
    max_kv: int


@dataclass
class PrefillCase:
    name: str
    Hq: int
    Hkv: int
    D: int
    scale: float
    causal: bool
    q: torch.Tensor          # bf16 [Tq, Hq, D]
    q_pos: torch.Tensor      # int32 [Tq]
    cu_q: torch.Tensor       # int32 [batch+1]
    max_q: int
    shards: List[Shard]
    visible_pairs_per_head: int   # number of (q, kv) pairs with kv_pos <= q_pos, all shards

    @property
    def batch(self) -> int:
        return self.cu_q.numel() - 1

    @property
    def Tq(self) -> int:
        return self.q.shape[0]

    def flops(self) -> float:
        """4 * D * Hq per visible pair (QK^T and PV, multiply+add each)."""
        return 4.0 * self.D * self.Hq * self.visible_pairs_per_head


def _cu(lengths: Sequence[int], device) -> torch.Tensor:
    return torch.tensor(np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32), device=device)


def striped_prefill(name: str, chunks: Sequence[int], n_shards: int, r_q: int, Hq: int, Hkv: int,
                    seed: int, device, D: int = HEAD_DIM) -> PrefillCase:
    """Striped sequence-parallel prefill share (Sec. 2.3): for each request with local
    chunk c, the global sequence has n_shards*c tokens; the token at global position p
    lives on instance p % n_shards at local index p // n_shards.  The local queries are
    stripe r_q (q_pos = n_shards*i + r_q) and shard j holds kv_pos = n_shards*m + j.
    All requests of the batch are packed back to back (cu_q / cu_kv)."""
    gen = torch.Generator(device=device).manual_seed(seed)
    Tq = int(sum(chunks))
    q = randn_bf16((Tq, Hq, D), gen, device)
    ks = [randn_bf16((Tq, Hkv, D), gen, device) for _ in range(n_shards)]
    vs = [randn_bf16((Tq, Hkv, D), gen, device) for _ in range(n_shards)]
    local = np.concatenate([np.arange(c, dtype=np.int64) for c in chunks])
    q_pos = torch.tensor((n_shards * local + r_q).astype(np.int32), device=device)
    cu = _cu(chunks, device)
    shards = []
    pairs = 0
    for j in range(n_shards):
        kv_pos = torch.tensor((n_shards * local + j).astype(np.int32), device=device)
        shards.append(Shard(ks[j], vs[j], kv_pos, cu, int(max(chunks))))
        for c in chunks:      # local mask: m <= i if j <= r_q else m < i
            pairs += c * (c + 1) // 2 if j <= r_q else c * (c - 1) // 2
    return PrefillCase(name, Hq, Hkv, D, 1.0 / math.sqrt(D), True, q, q_pos, cu, int(max(chunks)),
                       shards, pairs)


def contiguous_prefill(name: str, Tq: int, q_start: int, shard_ranges: Sequence[Sequence[int]],
                       Hq: int, Hkv: int, seed: int, device, D: int = HEAD_DIM,
                       causal: bool = True) -> PrefillCase:
    """One request; queries at positions q_start..q_start+Tq-1; shard s holds the
    contiguous positions shard_ranges[s] = (lo, hi)."""
    gen = torch.Generator(device=device).manual_seed(seed)
    q = randn_bf16((Tq, Hq, D), gen, device)
    ks = [randn_bf16((hi - lo, Hkv, D), gen, device) for lo, hi in shard_ranges]
    vs = [randn_bf16((hi - lo, Hkv, D), gen, device) for lo, hi in shard_ranges]
    q_pos = torch.arange(q_start, q_start + Tq, dtype=torch.int32, device=device)
    shards = []
    pairs = 0
    for s, (lo, hi) in enumerate(shard_ranges):
        kv_pos = torch.arange(lo, hi, dtype=torch.int32, device=device)
        shards.append(Shard(ks[s], vs[s], kv_pos, _cu([hi - lo], device), hi - lo))
        if causal:
            qp = np.arange(q_start, q_start + Tq, dtype=np.int64)
            pairs += int(np.clip(qp + 1 - lo, 0, hi - lo).sum())
        else:
            pairs += Tq * (hi - lo)
    return PrefillCase(name, Hq, Hkv, D, 1.0 / math.sqrt(D), causal, q, q_pos, _cu([Tq], device), Tq,
                       shards, pairs)


# --------------------------------------------------------------------------- decode
@dataclass
class DecodeCase:
    name: str
    Hq: int
    Hkv: int
    D: int
    scale: float
    num_slots: int
    lens: np.ndarray                 # int64 [B] resident KV rows of each request on this instance
    q: torch.Tensor                  # bf16 [B, Hq, D]
    k_pool: torch.Tensor             # bf16 [S, Hkv, D]
    v_pool: torch.Tensor             # bf16 [S, Hkv, D]
    slot_idx: torch.Tensor           # int32 [sum(lens)]
    seq_offsets: torch.Tensor        # int32 [B+1]
    new_k: torch.Tensor              # bf16 [T_new, Hkv, D] rows to append
    new_v: torch.Tensor
    new_slots: torch.Tensor          # int32 [T_new] free slots (negative = do not keep)
    peer_O: torch.Tensor             # bf16 [P_peer, B, Hq, D] synthetic partials of the other instances
    peer_LSE: torch.Tensor           # fp32 [P_peer, B, Hq]
    # host copies of the pool rows of the sampled requests, in slot_idx order: b -> (k_bits, v_bits)
    host_rows: Dict[int, tuple] = field(default_factory=dict)

    @property
    def B(self) -> int:
        return self.q.shape[0]

    @property
    def total_tokens(self) -> int:
        return int(self.lens.sum())

    def kv_bytes(self) -> float:
        """Algorithmic HBM bytes of one decode call: every resident K and V row once, the
        slot indices, q, and the (O, LSE) outputs."""
        row = 2 * self.Hkv * self.D * 2
        return (self.total_tokens * (row + 4) + self.B * self.Hq * self.D * 2
                + self.B * self.Hq * (self.D * 2 + 4))


def decode_pool(name: str, lens: Sequence[int], num_slots: int, Hq: int, Hkv: int, seed: int, device,
                n_new: int, n_peers: int = 3, sample_reqs: Optional[Sequence[int]] = None,
                D: int = HEAD_DIM, skip_new_every: int = 0) -> DecodeCase:
    """Token-granular pool (Sec. 6) with request b's rows at the random, non-contiguous,
    unique slots perm[off[b]:off[b+1]], perm = numpy default_rng(seed).permutation(S); rows to
    append go to the next unused entries of perm ("random free slots").  Only used slots
    hold N(0,1) data; the rest of the pool is zero.  Rows of the requests in sample_reqs
    (default: all) are also kept on the host for the oracle."""
    lens = np.asarray(lens, dtype=np.int64)
    B = len(lens)
    total = int(lens.sum())
    if total + n_new > num_slots:
        raise ValueError(f"{name}: {total}+{n_new} tokens do not fit {num_slots} slots")
    gen = torch.Generator(device=device).manual_seed(seed)
    q = randn_bf16((B, Hq, D), gen, device)
    perm = np.random.default_rng(seed).permutation(num_slots).astype(np.int32)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    k_pool = torch.zeros((num_slots, Hkv, D), dtype=torch.bfloat16, device=device)
    v_pool = torch.zeros((num_slots, Hkv, D), dtype=torch.bfloat16, device=device)
    sample = set(range(B)) if sample_reqs is None else set(int(b) for b in sample_reqs)
    host_rows: Dict[int, tuple] = {}
    for b in range(B):
        n = int(lens[b])
        kr = randn_bf16((n, Hkv, D), gen, device)
        vr = randn_bf16((n, Hkv, D), gen, device)
        if n:
            sl = torch.from_numpy(perm[off[b]:off[b + 1]].astype(np.int64)).to(device)
            k_pool[sl] = kr
            v_pool[sl] = vr
        if b in sample:
            host_rows[b] = (bits(kr), bits(vr))
        del kr, vr
    new_k = randn_bf16((n_new, Hkv, D), gen, device)
    new_v = randn_bf16((n_new, Hkv, D), gen, device)
    new_slots = perm[total:total + n_new].copy()
    if skip_new_every:
        new_slots[::skip_new_every] = -1
    peer_O = randn_bf16((n_peers, B, Hq, D), gen, device)
    peer_LSE = (torch.randn((n_peers, B, Hq), generator=gen, device=device, dtype=torch.float32)
                + math.log(8192.0))
    return DecodeCase(name, Hq, Hkv, D, 1.0 / math.sqrt(D), num_slots, lens, q, k_pool, v_pool,
                      torch.from_numpy(perm[:total].copy()).to(device),
                      torch.from_numpy(off.astype(np.int32)).to(device),
                      new_k, new_v, torch.from_numpy(new_slots).to(device), peer_O, peer_LSE, host_rows)


# --------------------------------------------------------------------------- which outputs the oracle is asked for
def sample_rows(rng, lo, hi, n_random, edges=(16, 32, 64, 128, 256)):
    """Row indices in [lo, hi): first/last, tile edges +-1, plus random rows."""
    rows = {lo, hi - 1}
    for e in edges:
        for base in range(lo, hi, e):
            for d in (-1, 0, 1):
                r = base + d
                if lo <= r < hi:
                    rows.add(r)
            if len(rows) > 64:
                break
    rows = sorted(rows)
    if len(rows) > 48:
        keep = rng.choice(len(rows), 48, replace=False)
        rows = sorted({rows[i] for i in keep} | {lo, hi - 1})
    extra = rng.integers(lo, hi, n_random)
    return np.unique(np.concatenate([np.asarray(rows, np.int64), extra.astype(np.int64)]))


# (number of sampled (row, head) pairs, seed) of the full-size parity tests, per configuration; the benchmark's
# CPU baseline times the oracle on the same samples
PARITY_SAMPLES = {"C2-prefill": (2300, 102), "C4-prefill": (1045, 104), "C5-prefill": (2110, 105)}


def prefill_parity_samples(pc: PrefillCase, n_total: int, seed: int):
    """About n_total (row, head) pairs of a prefill case for a sampled comparison with the oracle: per request its
    first and last row (in a striped layout the first one sees nothing in the later stripes: an empty visible set),
    rows at multiples of 16 .. 256 and their neighbours, random rows; the heads cycle through all of them.
    Returns (rows, heads, request of each row)."""
    rng = np.random.default_rng(seed)
    cu = host_i32(pc.cu_q)
    rows, reqs = [], []
    for r in range(pc.batch):
        rr = sample_rows(rng, int(cu[r]), int(cu[r + 1]), max(8, n_total // pc.batch - 48))
        rows.append(rr); reqs.append(np.full(len(rr), r))
    rows, reqs = np.concatenate(rows), np.concatenate(reqs)
    heads = (np.arange(len(rows)) * 7 + rng.integers(0, pc.Hq)) % pc.Hq
    return rows.astype(np.int64), heads.astype(np.int64), reqs


# --------------------------------------------------------------------------- the five configurations
def config1_prefill(device, r_q_unused: int = 0) -> PrefillCase:
    """Tiny ESP step: 4 heads, query chunk 256 at positions 768..1023, two contiguous shards of 512."""
    return contiguous_prefill("C1-prefill", 256, 768, [(0, 512), (512, 1024)], 4, 4, 0, device)


def config1_decode(device) -> DecodeCase:
    return decode_pool("C1-decode", [64, 128, 300, 512], 2048, 4, 4, 0, device, n_new=4)


def config2_prefill(device, N: int = 8192, r_q: int = 0, Hq: int = 32, Hkv: int = 32) -> PrefillCase:
    """LWM-7B-shaped prefill share: chunk N against 4 striped shards of N tokens each."""
    return striped_prefill("C2-prefill", [N], 4, r_q, Hq, Hkv, 1, device)


def config3_decode(device, B: int = 64, num_slots: int = 1 << 22, median: int = 8192, lo: int = 1024,
                   hi: int = 131072, Hq: int = 32, Hkv: int = 32,
                   sample_reqs: Optional[Sequence[int]] = None) -> DecodeCase:
    """Distributed-decode share: lognormal KV-slice lengths in a 4M-slot pool, 3 peer partials, 64 appends."""
    lens = lognormal_lengths(B, median, lo, hi, 2)
    return decode_pool("C3-decode", lens, num_slots, Hq, Hkv, 2, device, n_new=B, sample_reqs=sample_reqs)


def config4_prefill(device, Tq: int = 32768, Tkv: int = 262144, Hq: int = 32, Hkv: int = 32) -> PrefillCase:
    """Long-context share: the last Tq positions of a 2*Tkv-token sequence against its first half."""
    total = 2 * Tkv
    return contiguous_prefill("C4-prefill", Tq, total - Tq, [(0, Tkv)], Hq, Hkv, 3, device)


C5_CHUNKS = (2048, 4096, 8192, 8192, 16384, 32768)


def config5_prefill(device, chunks: Sequence[int] = C5_CHUNKS, Hq: int = 32, Hkv: int = 8) -> PrefillCase:
    """Mixed iteration, prefill part: var-len batch, each request striped over 4 shards, GQA 32/8."""
    return striped_prefill("C5-prefill", list(chunks), 4, 0, Hq, Hkv, 4, device)


def config5_decode(device, B: int = 256, num_slots: int = 1 << 24, median: int = 16384, lo: int = 512,
                   hi: int = 1 << 20, Hq: int = 32, Hkv: int = 8,
                   sample_reqs: Optional[Sequence[int]] = None) -> DecodeCase:
    lens = lognormal_lengths(B, median, lo, hi, 4)
    return decode_pool("C5-decode", lens, num_slots, Hq, Hkv, 4, device, n_new=B, sample_reqs=sample_reqs)
