"""GPU parity of the selection shared by the query heads of a KV group (an extension that is not
in the paper: DSK_SELECT_SHARED_BY_KV_GROUP / DSK_ATTN_SHARED_SELECTION) against the oracle.

Group scores are the maximum of the per-head scores; the slot set of every (sequence, KV head)
must equal the oracle's bit-exactly except for near ties (1e-4 relative, counted); attention of
every query head over its group's selection within 2e-3 of the fp64 oracle."""
import numpy as np
import pytest
import torch

from oracle import dynsplit_oracle as O
from dsk_testutil import DEFAULT_SCALE, bf16_bits_of, dev_bf16, gpu_case, rel_err, selection_check
from test_gpu_decode import ATTN_TOL, LSE_TOL, _oracle_scores, _seqs_to_check

pytestmark = pytest.mark.gpu


def _dsk():
    import paper_2602_03184_amd as dsk
    return dsk


def _check_shared(case, n_q, seqs, kv_heads, label):
    dsk = _dsk()
    cfg, seg, wl = case.cfg, case.seg, case.wl
    G = cfg.G
    comp = case.compressed()
    sums = bf16_bits_of(comp.ksum)
    kmin_bits, kmax_bits = sums[:, :, 0], sums[:, :, 1]
    swapped = 0
    worst = 0.0
    for qi in range(n_q):
        q_bits = wl.q[qi]
        q = dev_bf16(q_bits)
        sel = dsk.select_topk(comp, q, cfg.T, want_scores=True, shared=True)
        per_head = dsk.select_topk(comp, q, cfg.T, want_scores=True)
        att = dsk.sparse_decode_attn(q, case.K, case.V, sel.sel_start, sel.sel_len, sel.sel_count, cfg.b,
                                     flags=dsk.DSK_ATTN_SHARED_SELECTION)
        torch.cuda.synchronize()
        assert sel.sel_slot.shape == (cfg.B, cfg.Hkv, cfg.k) and sel.scores.shape[0] == cfg.Hkv
        g_slot, g_start = sel.sel_slot.cpu().numpy(), sel.sel_start.cpu().numpy()
        g_len, g_cnt = sel.sel_len.cpu().numpy(), sel.sel_count.cpu().numpy()
        g_scores = sel.scores.cpu().numpy()
        g_out, g_lse = att.out.cpu().numpy(), att.lse.cpu().numpy()
        nblk = int(seg.cu_blocks[-1])
        # the maximum of fp32 numbers is exact: the group row is the largest of the per-head rows the
        # same library computes
        ph = per_head.scores[:, :nblk].reshape(cfg.Hkv, G, nblk).max(dim=1).values
        assert torch.equal(sel.scores[:, :nblk], ph)
        for s in seqs:
            b0, b1 = int(seg.cu_blocks[s]), int(seg.cu_blocks[s + 1])
            sb = seg.slot_base[b0: b1 + 1]
            bs = seg.block_start[b0: b1 + 1]
            if b1 == b0:
                assert (g_cnt[s] == 0).all() and (g_slot[s] == -1).all()
                assert (g_out[s] == 0).all() and np.isneginf(g_lse[s]).all()
                continue
            for hk in kv_heads:
                heads = list(range(hk * G, (hk + 1) * G))
                osc = _oracle_scores(case, kmin_bits, kmax_bits, q_bits, s, heads)
                grp = O.group_block_scores(np.stack([osc[h] for h in heads]), G)[0]
                np.testing.assert_allclose(g_scores[hk, b0:b1], grp, rtol=2e-5, atol=2e-4)
                o_sel, tau = O.select_slots(grp, sb - sb[0], cfg.k)
                o_sel = o_sel + int(sb[0])
                cnt = int(g_cnt[s, hk])
                assert cnt == len(o_sel)
                gs = g_slot[s, hk, :cnt]
                assert (np.diff(gs) > 0).all()
                assert (g_slot[s, hk, cnt:] == -1).all() and (g_len[s, hk, cnt:] == 0).all()
                swapped += selection_check(gs, o_sel, tau, grp, sb)
                for j in range(cnt):
                    _, st, ln = O.slot_span(int(gs[j]) - int(sb[0]), bs, sb - sb[0], cfg.b)
                    assert (int(g_start[s, hk, j]), int(g_len[s, hk, j])) == (st, ln)
                toks = np.concatenate([np.arange(g_start[s, hk, j], g_start[s, hk, j] + g_len[s, hk, j])
                                       for j in range(cnt)])
                Kh, Vh = O.widen_bf16(wl.K[hk][toks]), O.widen_bf16(wl.V[hk][toks])
                for h in heads:                      # every query head of the group attends over the shared set
                    o, lse = O.sparse_attention(O.widen_bf16(q_bits[s, h]), Kh, Vh, np.arange(len(toks)), DEFAULT_SCALE)
                    e = rel_err(g_out[s, h], o)
                    worst = max(worst, e)
                    assert e <= ATTN_TOL, (s, h, e)
                    assert abs(float(g_lse[s, h]) - lse) <= LSE_TOL
    print("%s: swapped selections (near ties) = %d, worst attention rel err = %.3e" % (label, swapped, worst))


@pytest.mark.parametrize("cfg_id", [2, 3, 5])
def test_shared_selection_parity_full_size(cfg_id):
    case = gpu_case(cfg_id)
    cfg = case.cfg
    _check_shared(case, min(cfg.n_queries, 2), _seqs_to_check(cfg), sorted({0, cfg.Hkv // 2, cfg.Hkv - 1}),
                  "cfg%d shared" % cfg_id)


@pytest.mark.parametrize("Hq,Hkv", [(4, 2), (16, 2), (6, 2), (10, 2)])
def test_shared_selection_group_widths(Hq, Hkv):
    """Group widths 2 and 8 (the register-tiled score kernel), 3 and 5 (the any-width one)."""
    case = gpu_case(2, Hq=Hq, Hkv=Hkv, seqlens=[5000], T=512, n_queries=2)
    _check_shared(case, 2, [0], [0, 1], "G=%d shared" % (Hq // Hkv))


def test_shared_selection_with_one_head_per_group_is_the_per_head_selection():
    dsk = _dsk()
    case = gpu_case(4, seqlens=[9000], n_queries=1)        # 40 query heads on 40 KV heads
    cfg = case.cfg
    comp = case.compressed()
    q = dev_bf16(case.wl.q[0])
    a = dsk.select_topk(comp, q, cfg.T, want_scores=True, shared=True)
    b_ = dsk.select_topk(comp, q, cfg.T, want_scores=True)
    oa = dsk.sparse_decode_attn(q, case.K, case.V, a.sel_start, a.sel_len, a.sel_count, cfg.b,
                                flags=dsk.DSK_ATTN_SHARED_SELECTION)
    ob = dsk.sparse_decode_attn(q, case.K, case.V, b_.sel_start, b_.sel_len, b_.sel_count, cfg.b)
    torch.cuda.synchronize()
    for name in ("sel_slot", "sel_start", "sel_len", "sel_count"):
        assert torch.equal(getattr(a, name), getattr(b_, name)), name
    nblk = int(case.seg.cu_blocks[-1])                      # entries past the block count are not written
    assert torch.equal(a.scores[:, :nblk], b_.scores[:, :nblk])
    assert torch.equal(oa.out, ob.out) and torch.equal(oa.lse, ob.lse)


def test_shared_selection_ragged_batch_with_empty_and_short_sequences():
    case = gpu_case(5, B=5, seqlens=[2500, 0, 40, 7000, 1], T=256, n_queries=2)
    _check_shared(case, 2, list(range(5)), [0, 3, 7], "ragged shared")


@pytest.mark.parametrize("cfg_id,Hq,Hkv,B", [(5, 4, 2, 16), (5, 16, 2, 16), (3, 32, 8, 4)])
def test_shared_selection_tiled_gather(cfg_id, Hq, Hkv, B):
    """Launches of 4096 slots and more go through the kernel that folds every loaded K/V row
    into all query heads of the group: group widths 2, 8 (16 sequences, b = 16) and 4 (b = 32),
    ragged lengths with one empty sequence."""
    rng = np.random.default_rng(100 + Hq)
    seqlens = [int(x) for x in rng.integers(4200, 6000, size=B)]
    seqlens[1] = 0
    seqlens[2] = 5 * 128 * (32 if cfg_id == 3 else 16) // 8      # fewer slots than k: short selection
    case = gpu_case(cfg_id, B=B, Hq=Hq, Hkv=Hkv, seqlens=seqlens, n_queries=1,
                    T=128 * (32 if cfg_id == 3 else 16))
    assert case.cfg.B * case.cfg.Hkv * case.cfg.k >= 4096
    _check_shared(case, 1, [0, 1, 2, B - 1], sorted({0, Hkv - 1}), "tiled G=%d" % (Hq // Hkv))
