"""Helpers shared by the GPU parity tests: device upload, and the oracle run over a whole
(ragged) workload in the library's global coordinates."""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, List, Optional

import numpy as np
import torch

from oracle import dynsplit_oracle as O


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def dev_i32(a) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def dev_u8(a) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint8)).cuda()


def bf16_bits_of(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def canon_zero(bits: np.ndarray) -> np.ndarray:
    """Map bf16 -0 to +0 so that summaries compare as numbers."""
    out = bits.copy()
    out[out == 0x8000] = 0
    return out


@dataclass
class OracleSeg:
    cand_pos: np.ndarray          # global positions, all sequences
    cand_class: np.ndarray
    cand_cu: np.ndarray           # [B+1]
    block_start: np.ndarray       # global, [nblk_total+1]
    cu_blocks: np.ndarray         # [B+1]
    slot_base: np.ndarray         # global, [nblk_total+1]
    per_seq_block_start: List[np.ndarray]   # local coordinates


def oracle_segment(wl, class_weight_q: Optional[np.ndarray] = None, b: Optional[int] = None) -> OracleSeg:
    cfg = wl.cfg
    b = cfg.b if b is None else b
    wq_all = wl.class_weight_q if class_weight_q is None else class_weight_q
    cpos, ccls, ccu = [], [], [0]
    bs_glob, sb_glob, cu_blocks, per_seq = [], [], [0], []
    slot_off = 0
    for s in range(cfg.B):
        lo, hi = int(wl.cu_seqlens[s]), int(wl.cu_seqlens[s + 1])
        pos, cls = O.extract_candidates(wl.token_ids[lo:hi], wl.delim_ids)
        cpos.append(pos + lo)
        ccls.append(cls)
        ccu.append(ccu[-1] + len(pos))
        if hi > lo:
            bs = O.dd_select(hi - lo, pos, cls, wq_all[s], int(wl.C[s]), int(wl.delta[s]), cfg.a_num, cfg.a_den)
        else:
            bs = np.zeros(1, dtype=np.int64)
        sb = O.slot_map(bs, b)
        per_seq.append(bs)
        bs_glob.append(bs[:-1] + lo)
        sb_glob.append(sb[:-1] + slot_off)
        slot_off += int(sb[-1])
        cu_blocks.append(cu_blocks[-1] + len(bs) - 1)
    bs_glob.append(np.asarray([int(wl.cu_seqlens[-1])]))
    sb_glob.append(np.asarray([slot_off]))
    return OracleSeg(np.concatenate(cpos), np.concatenate(ccls), np.asarray(ccu), np.concatenate(bs_glob),
                     np.asarray(cu_blocks), np.concatenate(sb_glob), per_seq)


def oracle_summaries(Xbits: np.ndarray, block_start: np.ndarray, heads=None):
    """(min, max) bf16 bit patterns [len(heads), nblk, D] via the fp64 oracle."""
    from workloads import f32_to_bf16_bits
    heads = range(Xbits.shape[0]) if heads is None else heads
    mins, maxs = [], []
    for h in heads:
        X = O.widen_bf16(Xbits[h])[None]
        mn, mx = O.block_summaries(X, block_start)
        mins.append(f32_to_bf16_bits(mn[0].astype(np.float32)))   # exact: values are bf16 numbers
        maxs.append(f32_to_bf16_bits(mx[0].astype(np.float32)))
    return np.stack(mins), np.stack(maxs)


def oracle_means_bf16(Xbits: np.ndarray, block_start: np.ndarray, heads=None) -> np.ndarray:
    """fp64 block means of the oracle, as floats (not yet rounded to bf16), [len(heads), nblk, D]."""
    heads = range(Xbits.shape[0]) if heads is None else heads
    return np.stack([O.block_means(O.widen_bf16(Xbits[h])[None], block_start)[0] for h in heads])


def assert_bf16_of(got_bits: np.ndarray, exact: np.ndarray, max_off_frac: float = 2e-3) -> float:
    """got_bits must be the bf16 rounding (nearest even) of `exact`, except that an fp32-accumulated
    mean may land on the neighbouring bf16 value when the exact mean sits next to a rounding
    midpoint: every element within one bf16 step, and only a small fraction off at all."""
    from workloads import f32_to_bf16_bits
    want_bits = f32_to_bf16_bits(exact.astype(np.float32))
    got = O.widen_bf16(got_bits)
    want = O.widen_bf16(want_bits)
    off = canon_zero(got_bits) != canon_zero(want_bits)
    step = np.maximum(np.abs(want), np.abs(got)) * 2.0 ** -7 + 1e-38      # one bf16 step is at most this
    assert (np.abs(got - want)[off] <= step[off]).all(), "a mean is more than one bf16 step from the oracle"
    frac = float(off.mean())
    assert frac <= max_off_frac, "fraction of means off by one bf16 step: %.2e" % frac
    return frac


def selection_check(gpu_slots: np.ndarray, ora_slots: np.ndarray, tau: float, block_score: np.ndarray,
                    slot_base: np.ndarray, rel: float = 1e-4) -> int:
    """Bit-exact set equality, except that a slot may differ when its block's oracle score is
    within rel*|tau| of the threshold score tau (near-tie rule).  Returns the swapped count;
    raises AssertionError otherwise."""
    g, o = set(int(x) for x in gpu_slots), set(int(x) for x in ora_slots)
    assert len(g) == len(gpu_slots), "duplicate slots selected"
    assert len(g) == len(o), "selected %d slots, oracle %d" % (len(g), len(o))
    diff = g ^ o
    for slot in diff:
        i = int(np.searchsorted(slot_base, slot, side="right")) - 1
        gap = abs(float(block_score[i]) - tau)
        assert gap <= rel * abs(tau), "slot %d (block %d) differs: score gap %.3e vs tau %.6e" % (slot, i, gap, tau)
    return len(diff) // 2


def rel_err(got: np.ndarray, want: np.ndarray) -> float:
    return float(np.abs(got.astype(np.float64) - want).max() / max(np.abs(want).max(), 1e-30))


DEFAULT_SCALE = 1.0 / math.sqrt(128.0)


def heads_to_check(cfg) -> List[int]:
    """Query heads the full-size decode parity samples (all of them up to 8 heads)."""
    return list(range(cfg.Hq)) if cfg.Hq <= 8 else sorted({0, 1, cfg.G, cfg.Hq // 2 + 1, cfg.Hq - 1})


def kv_heads_to_check(cfg) -> List[int]:
    """KV heads whose summaries are compared with the oracle: all of them up to 8, else exactly
    the KV heads behind heads_to_check(), so that every summary the decode parity reads from the
    GPU has itself been checked bit for bit."""
    if cfg.Hkv <= 8:
        return list(range(cfg.Hkv))
    return sorted({h // cfg.G for h in heads_to_check(cfg)})


# ---------------------------------------------------------------------------------------------
# cached workloads on host and device
# ---------------------------------------------------------------------------------------------
class GpuCase:
    """One seeded workload, its device copies, and the oracle's segmentation."""

    def __init__(self, cfg_id: int, **overrides):
        from workloads import make_workload
        self.summary_mode = overrides.pop("summary_mode", 0)     # 0 = (min,max), 1 = mean pooling
        self.wl = make_workload(cfg_id, with_kv=True, with_qwin=False, **overrides)
        wl = self.wl
        self.cfg = wl.cfg
        self.seg = oracle_segment(wl)
        self.cu_seqlens = dev_i32(wl.cu_seqlens)
        self.K = dev_bf16(wl.K)
        self.V = dev_bf16(wl.V)
        self.token_ids = dev_i32(wl.token_ids)
        self.delim_ids = dev_i32(wl.delim_ids)
        self.class_weight_q = dev_u8(wl.class_weight_q)
        self.C_per_seq = dev_i32(wl.C)
        self.delta_per_seq = dev_i32(wl.delta)
        self.max_seqlen = int(wl.seqlens.max())
        self._comp = None

    def compress_kwargs(self, **kw):
        wl, cfg = self.wl, self.cfg
        d = dict(cu_seqlens=self.cu_seqlens, max_seqlen=self.max_seqlen, Hq=cfg.Hq, K=self.K, V=self.V,
                 n_class=cfg.n_class, class_weight_q=self.class_weight_q,
                 C_=int(wl.C.max()), delta=int(wl.delta.max()),
                 C_per_seq=self.C_per_seq if cfg.B > 1 else None,
                 delta_per_seq=self.delta_per_seq if cfg.B > 1 else None,
                 min_chunk=int((wl.C - wl.delta).min()),
                 alpha_num=cfg.a_num, alpha_den=cfg.a_den, b=cfg.b, summary_mode=self.summary_mode)
        d.update(kw)
        return d

    def compressed(self):
        """Full table-mode compression on the GPU (candidates from token ids), cached."""
        import paper_2602_03184_amd as dsk
        if self._comp is None:
            self._comp = dsk.compress(**self.compress_kwargs(
                stages=dsk.DSK_STAGE_CANDIDATES | dsk.DSK_STAGE_SEGMENT | dsk.DSK_STAGE_SUMMARIES,
                token_ids=self.token_ids, delim_ids=self.delim_ids))
            torch.cuda.synchronize()
        return self._comp


_CASES: Dict[tuple, GpuCase] = {}


def gpu_case(cfg_id: int, **overrides) -> GpuCase:
    key = (cfg_id, tuple(sorted((k, str(v)) for k, v in overrides.items())))
    if key not in _CASES:
        _CASES[key] = GpuCase(cfg_id, **overrides)
    return _CASES[key]


def drop_cases():
    _CASES.clear()
    torch.cuda.empty_cache()
