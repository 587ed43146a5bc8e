"""GPU parity of dsk_dense_decode_attn (full attention over the whole cache, the full-KV
baseline of Sec. 5) against the oracle's written-out definition: max relative error of the
output <= 2e-3 (fp32 accumulation of bf16 inputs), lse within 1e-3."""
import math

import numpy as np
import pytest
import torch

from oracle import dynsplit_oracle as O
from dsk_testutil import DEFAULT_SCALE, dev_bf16, dev_i32, gpu_case, rel_err

pytestmark = pytest.mark.gpu

ATTN_TOL = 2e-3
LSE_TOL = 1e-3


def _dsk():
    import paper_2602_03184_amd as dsk
    return dsk


def _check(case, q_bits, seqs, heads, scale=0.0):
    dsk = _dsk()
    wl, cfg = case.wl, case.cfg
    att = dsk.dense_decode_attn(dev_bf16(q_bits), case.K, case.V, case.cu_seqlens, case.max_seqlen, scale=scale)
    torch.cuda.synchronize()
    out, lse = att.out.cpu().numpy(), att.lse.cpu().numpy()
    sc = DEFAULT_SCALE if scale == 0.0 else scale
    worst = 0.0
    for s in seqs:
        lo, hi = int(wl.cu_seqlens[s]), int(wl.cu_seqlens[s + 1])
        if hi == lo:
            assert (out[s] == 0).all() and np.isneginf(lse[s]).all()
            continue
        for h in heads:
            hk = h // cfg.G
            o, l = O.dense_attention(O.widen_bf16(q_bits[s, h]), O.widen_bf16(wl.K[hk, lo:hi]),
                                     O.widen_bf16(wl.V[hk, lo:hi]), sc)
            e = rel_err(out[s, h], o)
            worst = max(worst, e)
            assert e <= ATTN_TOL, (s, h, e)
            assert abs(float(lse[s, h]) - l) <= LSE_TOL, (s, h)
    return worst


@pytest.mark.parametrize("cfg_id", [1, 2])
def test_dense_attention_parity_all_heads(cfg_id):
    case = gpu_case(cfg_id)
    cfg = case.cfg
    worst = _check(case, case.wl.q[0], range(cfg.B), range(cfg.Hq))
    print("cfg%d dense attention: worst rel err %.3e" % (cfg_id, worst))


@pytest.mark.parametrize("cfg_id", [3, 4, 5])
def test_dense_attention_parity_full_size_sampled_heads(cfg_id):
    case = gpu_case(cfg_id)
    cfg = case.cfg
    heads = sorted({0, cfg.G, cfg.Hq - 1})
    seqs = [0] if cfg.B == 1 else [0, cfg.B - 1]
    worst = _check(case, case.wl.q[0], seqs, heads)
    print("cfg%d dense attention (sampled heads): worst rel err %.3e" % (cfg_id, worst))


@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (8, 4), (8, 2), (8, 1), (6, 2), (5, 1)])
def test_dense_attention_group_widths_and_ragged_lengths(Hq, Hkv):
    """Group widths 1, 2, 4, 8 and two that no group tile divides; sequence lengths around the
    128-row step of a workgroup and the 32-row tile of a wavefront, one empty, one of one token."""
    seqlens = [0, 1, 31, 32, 33, 127, 128, 129, 700, 2049]
    case = gpu_case(5, B=len(seqlens), seqlens=seqlens, Hq=Hq, Hkv=Hkv, n_queries=1)
    _check(case, case.wl.q[0], range(len(seqlens)), range(Hq))
    _check(case, case.wl.q[0], [4, 8], [0, Hq - 1], scale=0.21)


def test_dense_equals_sparse_with_everything_selected():
    """Same query, budget covering every slot: the sparse path and the dense baseline must agree
    to fp32 rounding (they fold the same rows in different groupings)."""
    dsk = _dsk()
    case = gpu_case(1)
    cfg, wl = case.cfg, case.wl
    comp = case.compressed()
    q = dev_bf16(wl.q[0])
    nslots = int(comp.slot_base.cpu()[int(comp.cu_blocks.cpu()[-1])])
    sel = dsk.select_topk(comp, q, nslots * cfg.b)
    sp = dsk.sparse_decode_attn(q, case.K, case.V, sel.sel_start, sel.sel_len, sel.sel_count, cfg.b)
    de = dsk.dense_decode_attn(q, case.K, case.V, case.cu_seqlens, case.max_seqlen)
    torch.cuda.synchronize()
    assert rel_err(sp.out.cpu().numpy(), de.out.cpu().numpy().astype(np.float64)) <= 1e-5
    assert float((sp.lse - de.lse).abs().max().item()) <= 1e-5


def test_dense_is_deterministic_and_validates():
    dsk = _dsk()
    case = gpu_case(2)
    q = dev_bf16(case.wl.q[0])
    a = dsk.dense_decode_attn(q, case.K, case.V, case.cu_seqlens, case.max_seqlen)
    b = dsk.dense_decode_attn(q, case.K, case.V, case.cu_seqlens, case.max_seqlen)
    torch.cuda.synchronize()
    assert torch.equal(a.out, b.out) and torch.equal(a.lse, b.lse)
    args = dsk.make_dense_attn_args(q, case.K, case.V, case.cu_seqlens, case.max_seqlen).args
    args.max_seqlen = 0
    assert dsk.dsk_dense_decode_attn(args, check=False) == dsk.DSK_ERR_SHAPE
    args.max_seqlen = case.max_seqlen
    args.workspace_bytes = 16
    assert dsk.dsk_dense_decode_attn(args, check=False) == dsk.DSK_ERR_WORKSPACE


def test_bf16_copies_of_the_outputs_are_the_rounded_fp32_outputs():
    """out_bf16 (optional, for a consumer that takes bf16 activations) must be `out` rounded to
    nearest even, on every path that finishes an output: single-chunk heads, the merge kernel,
    empty selections, and the dense baseline."""
    dsk = _dsk()
    for cfg_id in (1, 3):                                  # 1: few slots; 3: 8 chunks per head, merged
        case = gpu_case(cfg_id)
        cfg = case.cfg
        comp = case.compressed()
        q = dev_bf16(case.wl.q[0])
        sel = dsk.select_topk(comp, q, cfg.T)
        att = dsk.sparse_decode_attn(q, case.K, case.V, sel.sel_start, sel.sel_len, sel.sel_count, cfg.b, want_bf16=True)
        den = dsk.dense_decode_attn(q, case.K, case.V, case.cu_seqlens, case.max_seqlen, want_bf16=True)
        torch.cuda.synchronize()
        for r in (att, den):
            assert torch.equal(r.out_bf16.view(torch.int16), r.out.to(torch.bfloat16).view(torch.int16))
    # one slot only (a head finished by the gather kernel itself) and an empty selection
    case = gpu_case(1)
    q = dev_bf16(case.wl.q[0])
    starts, lens = dev_i32(np.asarray([[[5, 0]]])), dev_i32(np.asarray([[[7, 0]]]))
    for count in (1, 0):
        att = dsk.sparse_decode_attn(q, case.K, case.V, starts, lens, dev_i32([[count]]), 16, want_bf16=True)
        torch.cuda.synchronize()
        assert torch.equal(att.out_bf16.view(torch.int16), att.out.to(torch.bfloat16).view(torch.int16))


def test_token_major_padded_layout_gives_identical_results():
    """K/V handed over as token-major (NHD) views with a padded token stride: selection, sparse
    attention, the dense baseline and an incremental update must give bit-identical results to
    the head-major contiguous layout (same arithmetic, different addresses)."""
    dsk = _dsk()
    case = gpu_case(2, seqlens=[5000])
    cfg, wl = case.cfg, case.wl
    L = wl.total_tokens
    buf = torch.zeros(L, cfg.Hkv, 2, 128 + 64, dtype=torch.bfloat16, device="cuda")
    buf[:, :, 0, :128] = case.K.permute(1, 0, 2)
    buf[:, :, 1, :128] = case.V.permute(1, 0, 2)
    Kv = buf[:, :, 0, :128].permute(1, 0, 2)
    Vv = buf[:, :, 1, :128].permute(1, 0, 2)
    assert Kv.stride(1) == cfg.Hkv * 2 * 192 and not Kv.is_contiguous()
    q = dev_bf16(wl.q[0])
    L0 = 4000

    def run(K, V):
        kw = case.compress_kwargs(
            stages=dsk.DSK_STAGE_CANDIDATES | dsk.DSK_STAGE_SEGMENT | dsk.DSK_STAGE_SUMMARIES, K=K, V=V,
            token_ids=case.token_ids, delim_ids=case.delim_ids, cu_seqlens=dev_i32([0, L0]), max_seqlen=L0,
            total_tokens=L0, Hkv=cfg.Hkv, max_cand_total=L,
            max_blocks_total=dsk.dsk_block_capacity(L, 1, int((wl.C - wl.delta).min())))
        comp = dsk.compress(**kw)
        app = dsk.make_appender(comp, K, V, case.token_ids, case.delim_ids, case.class_weight_q, C_=int(wl.C[0]),
                                delta=int(wl.delta[0]), alpha_num=cfg.a_num, alpha_den=cfg.a_den, b=cfg.b)
        app.step(L0, 4700)
        app.step(4700, L)
        sel = dsk.select_topk(comp, q, cfg.T)
        att = dsk.sparse_decode_attn(q, K, V, sel.sel_start, sel.sel_len, sel.sel_count, cfg.b)
        den = dsk.dense_decode_attn(q, K, V, dev_i32([0, L]), L)
        torch.cuda.synchronize()
        assert int(comp.dev_status.item()) == 0
        nblk = int(comp.cu_blocks.cpu()[1])
        return comp.ksum[:, :nblk].clone(), sel.sel_slot.clone(), att.out.clone(), att.lse.clone(), den.out.clone()

    ref = run(case.K, case.V)
    got = run(Kv, Vv)
    for a, b_ in zip(ref, got):
        assert a.shape == b_.shape and torch.equal(a, b_)
