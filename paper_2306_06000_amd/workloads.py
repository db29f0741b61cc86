"""Seeded synthetic inputs shaped like the paper's serving workloads.

This module only DRAWS inputs (lengths, predicted lengths, N(0,1) tensors rounded
once to the 16-bit storage type).  It holds none of the method's arithmetic and
imports neither the HIP binding nor the CPU oracle, so both sides can be fed from
it.  The paper's evaluation used a question-answering dataset run through real
models (section 4.1); neither is available here, so length distributions and
Gaussian activations of the same shapes (model shapes of table 1, maximum
sequence length 2048 of section 2.2, half-precision cache of section 2.1) stand in.

Every workload is a function of ``SEED_BASE + index`` only.
"""
from dataclasses import dataclass, field
from typing import List

import numpy as np

SEED_BASE = 230606000
F16, BF16 = 0, 1
E4M3 = 3  # 8-bit cache rows (the library's S3_E4M3); queries and new rows keep a 16-bit type


def f32_to_f16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> IEEE binary16 bit patterns."""
    return np.asarray(x, np.float32).astype(np.float16).view(np.uint16)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return u.astype(np.uint16)


def f32_to_e4m3_codes(x: np.ndarray) -> np.ndarray:
    """float32 -> e4m3 codes (uint8) through torch's float8_e4m3fn conversion; inputs stay far below
    the format's largest value, where every convention agrees."""
    import torch

    t = torch.from_numpy(np.ascontiguousarray(x, np.float32)).to(torch.float8_e4m3fn)
    return t.view(torch.uint8).numpy()


def to_bits(x: np.ndarray, dtype: int) -> np.ndarray:
    if dtype == E4M3:
        return f32_to_e4m3_codes(x)
    return f32_to_f16_bits(x) if dtype == F16 else f32_to_bf16_bits(x)


def normal_bits(rng: np.random.Generator, shape, dtype: int) -> np.ndarray:
    """N(0,1) drawn in float32 and rounded once to the storage type."""
    return to_bits(rng.standard_normal(shape, dtype=np.float32), dtype)


@dataclass
class Seq:
    prompt: int      # rows already cached when the sequence joins the batch
    output: int      # tokens it will generate before it finishes (true value)
    predicted: int   # predicted TOTAL length handed to the allocator
    start: int = -1  # rows cached at the first timed step (default: prompt)

    def __post_init__(self):
        if self.start < 0:
            self.start = self.prompt

    @property
    def total(self) -> int:
        return self.prompt + self.output


@dataclass
class Workload:
    name: str
    index: int
    n_layers: int
    n_heads: int
    head_dim: int
    dtype: int
    granule: int
    max_len: int
    batch: int
    steps: int
    seqs: List[Seq] = field(default_factory=list)   # the initial batch, in admission order
    pool: List[Seq] = field(default_factory=list)   # newcomers that replace finished sequences
    refill: bool = False
    arena_bytes: int = 0                            # 0: sized by the harness from the slots
    note: str = ""
    n_kv_heads: int = 0                             # 0: every head has its own K/V (multi-head attention)
    act_dtype: int = -1                             # type of q / new rows; -1: the cache type (16-bit caches)

    @property
    def seed(self) -> int:
        return SEED_BASE + self.index

    @property
    def elem_bytes(self) -> int:
        return 1 if self.dtype == E4M3 else 2

    @property
    def q_dtype(self) -> int:
        return self.dtype if self.act_dtype < 0 else self.act_dtype

    @property
    def kv_heads(self) -> int:
        return self.n_kv_heads or self.n_heads

    @property
    def row_bytes(self) -> int:
        return self.kv_heads * self.head_dim * self.elem_bytes

    @property
    def bytes_per_token(self) -> int:
        return 2 * self.n_layers * self.row_bytes


def c0() -> Workload:
    """Tiny step, GPT-J head shape.  The listed lengths are what attention sees after the
    append, so the slots hold {16,63,99,127} rows before the step; the reservation equals
    the final length, which puts two sequences exactly at capacity."""
    final = [17, 64, 100, 128]
    seqs = [Seq(prompt=L - 1, output=1, predicted=L) for L in final]
    return Workload("C0-tiny", 0, 1, 16, 256, F16, 64, 2048, 4, 1, seqs)


def _refill_pool(rng, n, draw):
    return [draw(rng) for _ in range(n)]


def c1(batch: int = 64, steps: int = 128) -> Workload:
    """GPT-J-shaped single layer, batch 64, 128 decode steps.  Prompt ~ U{32..512}, output ~
    U{1..512}; the prediction is the true total length times lognormal(0, 0.2), never below
    prompt + 1, so under-predicted sequences outgrow their slot mid-run."""
    rng = np.random.default_rng(SEED_BASE + 1)

    def draw(r):
        p = int(r.integers(32, 513))
        g = int(r.integers(1, 513))
        f = float(r.lognormal(0.0, 0.2))
        pred = min(2048, max(p + 1, int(round((p + g) * f))))
        return Seq(p, g, pred)

    seqs = [draw(rng) for _ in range(batch)]
    pool = _refill_pool(rng, 4 * batch, draw)
    return Workload("C1-gptj-b64", 1, 1, 16, 256, F16, 64, 2048, batch, steps, seqs, pool, refill=True)


def c2(batch: int = 512, steps: int = 256) -> Workload:
    """Ragged large batch with mispredictions: output ~ lognormal(5, 0.8) clipped to [1, 2048],
    prompt ~ U{16..256}, total clipped to 2048; one sequence in ten (Bernoulli) is predicted at
    half its output, the others exactly."""
    rng = np.random.default_rng(SEED_BASE + 2)

    def draw(r):
        g = int(np.clip(np.rint(r.lognormal(5.0, 0.8)), 1, 2048))
        p = int(r.integers(16, 257))
        under = bool(r.random() < 0.1)
        if p + g > 2048:
            g = 2048 - p
        pred = p + (max(1, g // 2) if under else g)
        return Seq(p, g, pred)

    seqs = [draw(rng) for _ in range(batch)]
    pool = _refill_pool(rng, 4 * batch, draw)
    return Workload("C2-ragged-b512", 2, 1, 16, 256, F16, 64, 2048, batch, steps, seqs, pool, refill=True)


def c3(target_bytes: int = 200 * 10**9, n_layers: int = 28, max_seqs: int = 4096) -> Workload:
    """Full-model KV footprint: 28 GPT-J layers in bf16; candidate sequences drawn as in C1, each
    caught at a uniform point of its generation.  The harness admits candidates in order until
    the arena of `target_bytes` is full; one decode step runs over all layers."""
    rng = np.random.default_rng(SEED_BASE + 3)
    seqs = []
    for _ in range(max_seqs):
        p = int(rng.integers(32, 513))
        g = int(rng.integers(1, 513))
        f = float(rng.lognormal(0.0, 0.2))
        u = float(rng.random())
        pred = min(2048, max(p + 1, int(round((p + g) * f))))
        pred = max(pred, p + int(u * g) + 1)  # the row written by the timed step must fit
        seqs.append(Seq(p, g, pred, start=p + int(u * g)))
    w = Workload("C3-gptj-28layers", 3, n_layers, 16, 256, BF16, 64, 2048, 0, 1, seqs)
    w.arena_bytes = target_bytes
    return w


def c4(batch: int = 128, steps: int = 64) -> Workload:
    """One GPU's share of a GPT-3-175B layer: 12 of the 96 heads, head_dim 128, bf16; long
    contexts, start ~ U{512..1984} so that every sequence ends at or below 2048."""
    rng = np.random.default_rng(SEED_BASE + 4)
    seqs = []
    for _ in range(batch):
        s = int(rng.integers(512, 1985))
        seqs.append(Seq(prompt=s, output=steps, predicted=s + steps))
    return Workload("C4-gpt3-share", 4, 1, 12, 128, BF16, 128, 2048, batch, steps, seqs)


def c5(batch: int = 256, steps: int = 128, n_heads: int = 32, n_kv_heads: int = 8, head_dim: int = 128,
       dtype: int = BF16) -> Workload:
    """Shared key/value heads (grouped-query; n_kv_heads = 1 is multi-query attention, which the
    paper's related-work section names as complementary): C1's lengths, mispredictions and refill
    on a 32-query-head / 8-KV-head, d = 128 shape, at four times C1's batch (a cache row is a
    quarter of the multi-head one).  Not one of the paper's measured models."""
    base = c1(batch, steps)
    eight = dtype == E4M3  # both footprint variants at once: 8-bit rows of the shared heads, bf16 queries
    return Workload(f"C5-shared-kv-{n_heads}q{n_kv_heads}kv" + ("-e4m3" if eight else ""), 5, 1, n_heads, head_dim, dtype,
                    base.granule, base.max_len, batch, steps, base.seqs, base.pool, base.refill, n_kv_heads=n_kv_heads,
                    act_dtype=BF16 if eight else -1)


def c6(batch: int = 128, steps: int = 128) -> Workload:
    """8-bit cache rows (quantisation, which the paper's related-work section names as complementary):
    C1's shape, lengths, mispredictions and refill with e4m3 rows and fp16 queries / new rows, at twice
    C1's batch (a cache row is half the size).  Not one of the paper's measured configurations."""
    base = c1(batch, steps)
    return Workload("C6-e4m3-rows", 6, 1, 16, 256, E4M3, base.granule, base.max_len, batch, steps, base.seqs, base.pool,
                    base.refill, act_dtype=F16)


def by_name(name: str) -> Workload:
    return {"c0": c0, "c1": c1, "c2": c2, "c3": c3, "c4": c4, "c5": c5, "c6": c6}[name.lower()]()


def step_tensors(w: Workload, step: int, layer: int, n: int):
    """q, k_new, v_new for one (step, layer): [n][H][D] 16-bit patterns, N(0,1)."""
    rng = np.random.default_rng([w.seed, 1, step, layer])
    shape = (3, n, w.n_heads, w.head_dim)
    t = normal_bits(rng, shape, w.q_dtype)  # queries and new rows: the activation type
    hk = w.kv_heads  # shared K/V heads: the first kv_heads of the same draw
    return t[0], np.ascontiguousarray(t[1][:, :hk]), np.ascontiguousarray(t[2][:, :hk])


def prefill_rows(w: Workload, seq_serial: int, layer: int, rows: int):
    """K and V rows [rows][H][D] a sequence holds when it joins (stand-in for the prompt phase)."""
    rng = np.random.default_rng([w.seed, 2, seq_serial, layer])
    t = normal_bits(rng, (2, rows, w.n_heads, w.head_dim), w.dtype)
    hk = w.kv_heads
    return np.ascontiguousarray(t[0][:, :hk]), np.ascontiguousarray(t[1][:, :hk])


class PooledSource:
    """Cheap seeded inputs for full-size runs: N(0,1) pools drawn once; every (sequence, layer) and
    (step, layer) takes a window of them at an offset that depends on its indices.  Same role as
    step_tensors / prefill_rows (which draw fresh numbers every call and are too slow for hundreds of
    steps of a 512-sequence batch)."""

    def __init__(self, w: Workload, n_max: int, ring: int = 5):
        rng = np.random.default_rng([w.seed, 3])
        self.w = w
        self.rows = normal_bits(rng, (2, w.max_len + 128, w.n_heads, w.head_dim), w.dtype)
        self.qkv = normal_bits(rng, (ring, 3, n_max, w.n_heads, w.head_dim), w.q_dtype)
        self.ring = ring

    def prefill_rows(self, serial: int, layer: int, rows: int):
        start = (serial * 37 + layer * 11) % 128
        hk = self.w.kv_heads
        return self.rows[0, start:start + rows, :hk], self.rows[1, start:start + rows, :hk]

    def step_tensors(self, step: int, layer: int, n: int):
        t = self.qkv[(step * self.w.n_layers + layer) % self.ring]
        shift = (step * 131 + layer * 17) % self.w.head_dim
        t = np.roll(t[:, :n], shift, axis=-1)
        hk = self.w.kv_heads
        return t[0], t[1][:, :hk], t[2][:, :hk]
