"""Seeded synthetic DynSplit-KV workloads (token streams, bf16 K/V, queries).

Stand-ins for the long-context benchmark token streams and real model K/V the
paper evaluates on (Sec. 5.1): lengths and budgets follow the paper's context
and budget scales (Sec. 5.2, passkey budgets 256-4096 at 100k tokens), values
are Gaussian with a few outlier channels.  Nothing here computes any step of
the method: it only draws inputs and converts fp32 draws to bf16 bit patterns.
"""
from __future__ import annotations

import dataclasses
import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

VOCAB = 32000
N_CLASS = 16


# ----------------------------------------------------------------------------
# bf16 bit helpers (input preparation only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even); returns uint16 bit patterns.

    Inputs must be finite (the generators never draw inf/NaN)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to the fp32 values they denote (exact)."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------
# configuration table
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class WorkloadConfig:
    cfg_id: int
    name: str
    B: int
    Hq: int
    Hkv: int
    seqlens: Optional[Sequence[int]]      # None -> ragged U{len_lo..len_hi}
    b: int                                # fixed mapped block ("slot") length
    T: int                                # token budget per sequence
    gap_means: Sequence[int]              # choices for the per-sequence mean delimiter gap
    C: Optional[int]                      # base chunk size; None -> per-seq = gap mean
    delta: Optional[int]                  # max deviation; None -> C // 2
    long_span_prob: float = 0.0           # probability that a gap is U{200..800}
    n_queries: int = 1
    len_lo: int = 0
    len_hi: int = 0
    D: int = 128
    a_num: int = 5                        # alpha_sel = a_num / a_den
    a_den: int = 10
    n_class: int = N_CLASS
    M: int = 8                            # sampled occurrences per delimiter class
    W: int = 8
    R: int = 128
    alpha_imp: float = 1.0

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def k(self) -> int:
        return self.T // self.b


CONFIGS = {
    1: WorkloadConfig(1, "cfg1_1head_4k", 1, 1, 1, [4096], 16, 256, [24], 24, 12),
    2: WorkloadConfig(2, "cfg2_llama3_8b_32k", 1, 32, 8, [32768], 16, 2048, [30], 30, 15),
    3: WorkloadConfig(3, "cfg3_llama3_8b_128k", 1, 32, 8, [131072], 32, 4096, [30], 32, 16,
                      long_span_prob=0.05, n_queries=32),
    4: WorkloadConfig(4, "cfg4_llama2_13b_128k", 1, 40, 40, [131072], 16, 4096, [40], 40, 20),
    5: WorkloadConfig(5, "cfg5_llama3_8b_b8_ragged", 8, 32, 8, None, 16, 2048, [16, 32, 64],
                      None, None, len_lo=16384, len_hi=65536),
}


@dataclass
class Workload:
    cfg: WorkloadConfig
    seqlens: np.ndarray          # int32 [B]
    cu_seqlens: np.ndarray       # int32 [B+1]
    C: np.ndarray                # int32 [B]
    delta: np.ndarray            # int32 [B]
    gap_mean: np.ndarray         # int32 [B]
    delim_ids: np.ndarray        # int32 [n_class], distinct
    token_ids: np.ndarray        # int32 [Ltot]
    class_weight_q: np.ndarray   # uint8 [B, n_class], tenths in 5..10 (table mode)
    K: Optional[np.ndarray] = None   # uint16 bf16 bits [Hkv, Ltot, D]
    V: Optional[np.ndarray] = None
    q: Optional[np.ndarray] = None   # uint16 bf16 bits [n_queries, B, Hq, D]
    qwin: Optional[np.ndarray] = None  # uint16 bf16 bits [B, n_class*M, W, Hq, D]
    outlier_k: np.ndarray = field(default_factory=lambda: np.zeros((0, 4), np.int64))
    outlier_v: np.ndarray = field(default_factory=lambda: np.zeros((0, 4), np.int64))

    @property
    def total_tokens(self) -> int:
        return int(self.cu_seqlens[-1])


def _rng(cfg_id: int, seq: int, part: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([1000 * cfg_id + seq, part])))


# ----------------------------------------------------------------------------
# pieces
# ----------------------------------------------------------------------------
def make_tokens(rng: np.random.Generator, L: int, delim_ids: np.ndarray, gap_mean: float,
                long_span_prob: float = 0.0, vocab: int = VOCAB) -> np.ndarray:
    """Token ids of one sequence: delimiters at cumulative geometric gaps, the rest
    uniform over the non-delimiter ids."""
    n_class = len(delim_ids)
    nondelim = np.setdiff1d(np.arange(vocab, dtype=np.int64), delim_ids.astype(np.int64))
    tok = nondelim[rng.integers(0, len(nondelim), size=L)].astype(np.int32)
    # enough gaps to run past L (every gap >= 1)
    n_gaps = int(L / max(gap_mean, 1.0) * 2) + 64
    pos_list: List[np.ndarray] = []
    last = -1
    while last < L:
        gaps = rng.geometric(1.0 / gap_mean, size=n_gaps).astype(np.int64)
        if long_span_prob > 0.0:
            is_long = rng.random(n_gaps) < long_span_prob
            long_gaps = rng.integers(200, 801, size=n_gaps)
            gaps = np.where(is_long, long_gaps, gaps)
        pos = last + np.cumsum(gaps)
        pos_list.append(pos)
        last = int(pos[-1])
    pos = np.concatenate(pos_list)
    pos = pos[pos < L]
    cls = rng.integers(0, n_class, size=len(pos))
    tok[pos] = delim_ids[cls].astype(np.int32)
    return tok


def make_kv(rng: np.random.Generator, Hkv: int, L: int, D: int, outliers: np.ndarray) -> np.ndarray:
    """bf16 bits [Hkv, L, D]: N(0,1) with the given per-head outlier channels scaled x8."""
    out = np.empty((Hkv, L, D), dtype=np.uint16)
    for h in range(Hkv):
        x = rng.standard_normal((L, D), dtype=np.float32)
        x[:, outliers[h]] *= np.float32(8.0)
        out[h] = f32_to_bf16_bits(x)
    return out


def make_queries(rng: np.random.Generator, n: int, B: int, Hq: int, D: int) -> np.ndarray:
    return f32_to_bf16_bits(rng.standard_normal((n, B, Hq, D), dtype=np.float32))


def make_drifting_queries(rng: np.random.Generator, n: int, B: int, Hq: int, D: int, rho: float) -> np.ndarray:
    """bf16 bits [n, B, Hq, D] of a decode-like query stream: a first-order autoregressive walk
    q[t+1] = rho*q[t] + sqrt(1 - rho^2)*noise, every q[t] ~ N(0,1) per channel, so that
    consecutive steps resemble each other (rho = 0 gives independent queries)."""
    out = np.empty((n, B, Hq, D), dtype=np.float32)
    cur = rng.standard_normal((B, Hq, D), dtype=np.float32)
    mix = np.float32(math.sqrt(max(0.0, 1.0 - rho * rho)))
    for t in range(n):
        out[t] = cur
        cur = np.float32(rho) * cur + mix * rng.standard_normal((B, Hq, D), dtype=np.float32)
    return f32_to_bf16_bits(out)


def make_qwin(rng: np.random.Generator, B: int, n_samp: int, W: int, Hq: int, D: int) -> np.ndarray:
    return f32_to_bf16_bits(rng.standard_normal((B, n_samp, W, Hq, D), dtype=np.float32))


# ----------------------------------------------------------------------------
# whole workload
# ----------------------------------------------------------------------------
def make_workload(cfg, *, with_kv: bool = True, with_qwin: bool = False, **overrides) -> Workload:
    """Build the seeded workload of one configuration.

    `cfg` is a key of CONFIGS or a WorkloadConfig; `overrides` replace config
    fields (e.g. seqlens=[8192] for a reduced-size parity case)."""
    if not isinstance(cfg, WorkloadConfig):
        cfg = CONFIGS[cfg]
    if overrides:
        cfg = dataclasses.replace(cfg, **overrides)
    crng = _rng(cfg.cfg_id, 0, 0)                     # config-level draws
    delim_ids = np.sort(crng.choice(VOCAB, size=cfg.n_class, replace=False)).astype(np.int32)
    crng.shuffle(delim_ids)                           # class index is not ordered by id
    outlier_k = np.stack([crng.choice(cfg.D, size=4, replace=False) for _ in range(cfg.Hkv)])
    outlier_v = np.stack([crng.choice(cfg.D, size=4, replace=False) for _ in range(cfg.Hkv)])
    if cfg.seqlens is None:
        seqlens = crng.integers(cfg.len_lo, cfg.len_hi + 1, size=cfg.B).astype(np.int32)
    else:
        seqlens = np.asarray(cfg.seqlens, dtype=np.int32)
        assert len(seqlens) == cfg.B
    gap_mean = np.asarray(crng.choice(np.asarray(cfg.gap_means), size=cfg.B), dtype=np.int32)
    C = np.full(cfg.B, cfg.C, np.int32) if cfg.C is not None else gap_mean.copy()
    delta = np.full(cfg.B, cfg.delta, np.int32) if cfg.delta is not None else (C // 2).astype(np.int32)
    class_weight_q = crng.integers(5, 11, size=(cfg.B, cfg.n_class)).astype(np.uint8)
    cu = np.zeros(cfg.B + 1, dtype=np.int32)
    cu[1:] = np.cumsum(seqlens)
    Ltot = int(cu[-1])

    token_ids = np.empty(Ltot, dtype=np.int32)
    K = V = None
    if with_kv:
        K = np.empty((cfg.Hkv, Ltot, cfg.D), dtype=np.uint16)
        V = np.empty((cfg.Hkv, Ltot, cfg.D), dtype=np.uint16)
    for s in range(cfg.B):
        L = int(seqlens[s])
        lo, hi = int(cu[s]), int(cu[s + 1])
        token_ids[lo:hi] = make_tokens(_rng(cfg.cfg_id, s, 1), L, delim_ids, float(gap_mean[s]),
                                       cfg.long_span_prob)
        if with_kv:
            K[:, lo:hi] = make_kv(_rng(cfg.cfg_id, s, 2), cfg.Hkv, L, cfg.D, outlier_k)
            V[:, lo:hi] = make_kv(_rng(cfg.cfg_id, s, 3), cfg.Hkv, L, cfg.D, outlier_v)
    q = make_queries(_rng(cfg.cfg_id, 0, 4), cfg.n_queries, cfg.B, cfg.Hq, cfg.D)
    qwin = None
    if with_qwin:
        qwin = make_qwin(_rng(cfg.cfg_id, 0, 5), cfg.B, cfg.n_class * cfg.M, cfg.W, cfg.Hq, cfg.D)
    return Workload(cfg=cfg, seqlens=seqlens, cu_seqlens=cu, C=C, delta=delta, gap_mean=gap_mean,
                    delim_ids=delim_ids, token_ids=token_ids, class_weight_q=class_weight_q,
                    K=K, V=V, q=q, qwin=qwin, outlier_k=outlier_k, outlier_v=outlier_v)


def extra_queries(cfg: WorkloadConfig, n: int) -> np.ndarray:
    """n further seeded decode queries [n, B, Hq, D] (bf16 bits) for a configuration whose own
    query list is shorter than a measurement needs; a stream of its own, so the configuration's
    queries are unchanged."""
    return make_queries(_rng(cfg.cfg_id, 0, 6), n, cfg.B, cfg.Hq, cfg.D)

