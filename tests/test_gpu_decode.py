"""GPU parity of dsk_select_topk and dsk_sparse_decode_attn against the fp64 oracle.

Selections must equal the oracle's slot sets bit-exactly, except where the oracle's score gap
to the threshold is below 1e-4 relative (then the swap is counted and reported).  Attention
outputs must be within 2e-3 max relative error (fp32 accumulation), lse within 1e-3."""
import math

import numpy as np
import pytest
import torch

from oracle import dynsplit_oracle as O
from dsk_testutil import (DEFAULT_SCALE, bf16_bits_of, dev_bf16, dev_i32, gpu_case, heads_to_check, rel_err,
                          selection_check)

pytestmark = pytest.mark.gpu

ATTN_TOL = 2e-3
LSE_TOL = 1e-3


def _dsk():
    import paper_2602_03184_amd as dsk
    return dsk


def _oracle_scores(case, comp_bits_min, comp_bits_max, q_bits, s, heads):
    """fp64 block scores of sequence s for the given query heads, from the (verified
    bit-exact) summaries."""
    cfg, seg = case.cfg, case.seg
    b0, b1 = int(seg.cu_blocks[s]), int(seg.cu_blocks[s + 1])
    G = cfg.G
    out = {}
    for h in heads:
        hk = h // G
        kmin = O.widen_bf16(comp_bits_min[hk, b0:b1])[None]
        kmax = O.widen_bf16(comp_bits_max[hk, b0:b1])[None]
        q = O.widen_bf16(q_bits[s, h])[None]
        out[h] = O.block_scores(q, kmin, kmax)[0]
    return out


def _heads_to_check(cfg):
    return heads_to_check(cfg)


def _seqs_to_check(cfg):
    return list(range(cfg.B)) if cfg.B <= 2 else [0, cfg.B // 2, cfg.B - 1]


def _check_decode(case, n_q, seqs, heads, label, all_heads_first_query=False, **select_kw):
    """Scores, slot sets, spans and attention of the GPU path against the oracle for the given
    sequences and query heads."""
    dsk = _dsk()
    cfg, seg, wl = case.cfg, case.seg, case.wl
    comp = case.compressed()
    sums = bf16_bits_of(comp.ksum)
    kmin_bits, kmax_bits = sums[:, :, 0], sums[:, :, 1]
    swapped_total = 0
    worst_attn = 0.0
    for qi in range(n_q):
        q_bits = wl.q[qi]                                   # [B, Hq, D]
        q = dev_bf16(q_bits)
        sel = dsk.select_topk(comp, q, cfg.T, want_scores=True, **select_kw)
        att = dsk.sparse_decode_attn(q, case.K, case.V, sel.sel_start, sel.sel_len, sel.sel_count, cfg.b)
        torch.cuda.synchronize()
        g_slot = sel.sel_slot.cpu().numpy()
        g_start = sel.sel_start.cpu().numpy()
        g_len = sel.sel_len.cpu().numpy()
        g_cnt = sel.sel_count.cpu().numpy()
        g_scores = sel.scores.cpu().numpy()
        g_out = att.out.cpu().numpy()
        g_lse = att.lse.cpu().numpy()
        # the first query is checked on every query head when the summaries of all KV heads are
        # themselves compared with the oracle (up to 8 KV heads), the others on the sampled heads
        heads_q = list(range(cfg.Hq)) if (all_heads_first_query and qi == 0 and cfg.Hkv <= 8) else heads
        for s in seqs:
            b0, b1 = int(seg.cu_blocks[s]), int(seg.cu_blocks[s + 1])
            sb = seg.slot_base[b0: b1 + 1]
            bs = seg.block_start[b0: b1 + 1]
            if b1 == b0:                                    # empty sequence: defined empty result
                assert (g_cnt[s] == 0).all() and (g_slot[s] == -1).all()
                assert (g_out[s] == 0).all() and np.isneginf(g_lse[s]).all()
                continue
            osc = _oracle_scores(case, kmin_bits, kmax_bits, q_bits, s, heads_q)
            for h in heads_q:
                # a6: fp32 scores against fp64
                np.testing.assert_allclose(g_scores[h, b0:b1], osc[h], rtol=2e-5, atol=2e-4)
                # a7: slot set
                o_sel, tau = O.select_slots(osc[h], sb - sb[0], cfg.k)
                o_sel = o_sel + int(sb[0])
                cnt = int(g_cnt[s, h])
                assert cnt == len(o_sel)
                gs = g_slot[s, h, :cnt]
                assert (np.diff(gs) > 0).all()
                assert (g_slot[s, h, cnt:] == -1).all() and (g_len[s, h, cnt:] == 0).all()
                swapped_total += selection_check(gs, o_sel, tau, osc[h], sb)
                # spans of the GPU's own slots must be what the slot map says
                for j in range(cnt):
                    _, st, ln = O.slot_span(int(gs[j]) - int(sb[0]), bs, sb - sb[0], cfg.b)
                    assert (int(g_start[s, h, j]), int(g_len[s, h, j])) == (st, ln)
                # a8 end to end: attention over the GPU's own selection vs the oracle on that set
                toks = np.concatenate([np.arange(g_start[s, h, j], g_start[s, h, j] + g_len[s, h, j])
                                       for j in range(cnt)])
                hk = h // cfg.G
                Kh = O.widen_bf16(wl.K[hk][toks])
                Vh = O.widen_bf16(wl.V[hk][toks])
                o, lse = O.sparse_attention(O.widen_bf16(q_bits[s, h]), Kh, Vh, np.arange(len(toks)), DEFAULT_SCALE)
                e = rel_err(g_out[s, h], o)
                worst_attn = max(worst_attn, e)
                assert e <= ATTN_TOL, (s, h, e)
                assert abs(float(g_lse[s, h]) - lse) <= LSE_TOL
    print("%s: swapped selections (near ties) = %d, worst attention rel err = %.3e" %
          (label, swapped_total, worst_attn))


@pytest.mark.parametrize("cfg_id", [1, 2, 3, 4, 5])
def test_select_and_attention_parity(cfg_id):
    case = gpu_case(cfg_id)
    cfg = case.cfg
    _check_decode(case, min(cfg.n_queries, 3), _seqs_to_check(cfg), _heads_to_check(cfg), "cfg%d" % cfg_id,
                  all_heads_first_query=True)


def test_many_short_sequences_share_score_groups():
    """40 ragged sequences of a few blocks each (two of them empty, one of a single token): the
    groups of consecutive blocks that the score kernel handles together straddle up to several
    sequences, and there are more sequence starts than one wavefront ballot covers."""
    rng = np.random.default_rng(7)
    seqlens = [int(x) for x in rng.integers(20, 400, size=40)]
    seqlens[5] = 0
    seqlens[6] = 0
    seqlens[17] = 1
    seqlens[39] = 3000
    case = gpu_case(5, B=40, seqlens=seqlens, T=128, n_queries=2)
    _check_decode(case, 2, list(range(40)), [0, 3, 4, 17, 31], "40 short sequences")


@pytest.mark.parametrize("cfg_id", [2, 3, 5])
def test_block_count_hint_does_not_change_results(cfg_id):
    """max_blocks_used (a host-side upper bound on the block count; it sizes the score launch and
    picks the workgroup size and register tile of the selection kernel: 512 x 4, 1024 x 4 and
    1024 x 8 blocks for these three configurations) must leave every output bit-identical, whether exact, loose or absent."""
    dsk = _dsk()
    case = gpu_case(cfg_id)
    cfg = case.cfg
    comp = case.compressed()
    nblk = int(comp.cu_blocks.cpu()[-1])
    q = dev_bf16(case.wl.q[0])
    ref = dsk.select_topk(comp, q, cfg.T, want_scores=True)
    torch.cuda.synchronize()
    for hint in (nblk, nblk + 10):
        got = dsk.select_topk(comp, q, cfg.T, want_scores=True, max_blocks_used=hint)
        torch.cuda.synchronize()
        for name in ("sel_slot", "sel_start", "sel_len", "sel_count"):
            assert torch.equal(getattr(ref, name), getattr(got, name)), (hint, name)
        assert torch.equal(ref.scores[:, :nblk], got.scores[:, :nblk])
    # the per-sequence bound picks the selection kernel's tile; one that is too small must still
    # give the same result (such sequences go through the memory-resident path)
    cub = comp.cu_blocks.cpu().numpy()
    per_seq = int((cub[1:] - cub[:-1]).max())
    for hint in (per_seq, 16):
        got = dsk.select_topk(comp, q, cfg.T, max_blocks_used=nblk, max_blocks_per_seq=hint)
        torch.cuda.synchronize()
        for name in ("sel_slot", "sel_start", "sel_len", "sel_count"):
            assert torch.equal(getattr(ref, name), getattr(got, name)), ("per-sequence hint", hint, name)
    _check_decode(case, 1, [0, cfg.B - 1] if cfg.B > 1 else [0], [0, cfg.Hq - 1],
                  "cfg%d with block-count hint" % cfg_id, max_blocks_used=nblk, max_blocks_per_seq=per_seq)


@pytest.mark.parametrize("cfg_id", [1, 2])
def test_attention_on_oracle_selection(cfg_id):
    """dsk_sparse_decode_attn fed the oracle's index set (not its own selection)."""
    dsk = _dsk()
    case = gpu_case(cfg_id)
    cfg, seg, wl = case.cfg, case.seg, case.wl
    q_bits = wl.q[0]
    k = cfg.k
    starts = np.zeros((cfg.B, cfg.Hq, k), np.int32)
    lens = np.zeros((cfg.B, cfg.Hq, k), np.int32)
    cnts = np.zeros((cfg.B, cfg.Hq), np.int32)
    want = {}
    for s in range(cfg.B):
        bs, sb = seg.per_seq_block_start[s], O.slot_map(seg.per_seq_block_start[s], cfg.b)
        lo = int(wl.cu_seqlens[s])
        for h in range(cfg.Hq):
            hk = h // cfg.G
            Kh = O.widen_bf16(wl.K[hk, lo: lo + int(bs[-1])])
            Vh = O.widen_bf16(wl.V[hk, lo: lo + int(bs[-1])])
            kmin, kmax = O.block_summaries(Kh[None], bs)
            sc = O.block_scores(O.widen_bf16(q_bits[s, h])[None], kmin, kmax)[0]
            sel, _ = O.select_slots(sc, sb, k)
            for j, g in enumerate(sel):
                _, st, ln = O.slot_span(int(g), bs, sb, cfg.b)
                starts[s, h, j], lens[s, h, j] = st + lo, ln
            cnts[s, h] = len(sel)
            toks = O.selected_tokens(sel, bs, sb, cfg.b)
            want[(s, h)] = O.sparse_attention(O.widen_bf16(q_bits[s, h]), Kh, Vh, toks, DEFAULT_SCALE)
        if cfg.Hq > 8:
            break
    att = dsk.sparse_decode_attn(dev_bf16(q_bits), case.K, case.V, dev_i32(starts), dev_i32(lens), dev_i32(cnts), cfg.b)
    torch.cuda.synchronize()
    out, lse = att.out.cpu().numpy(), att.lse.cpu().numpy()
    for (s, h), (o, l) in want.items():
        assert rel_err(out[s, h], o) <= ATTN_TOL
        assert abs(float(lse[s, h]) - l) <= LSE_TOL


def test_budget_all_equals_dense_attention():
    """Budget >= sequence length selects every slot; the result is dense softmax attention."""
    dsk = _dsk()
    case = gpu_case(1)
    cfg, wl = case.cfg, case.wl
    comp = case.compressed()
    q_bits = wl.q[0]
    q = dev_bf16(q_bits)
    L = wl.total_tokens
    budget = (int(case.seg.slot_base[-1]) + 5) * cfg.b
    sel = dsk.select_topk(comp, q, budget)
    att = dsk.sparse_decode_attn(q, case.K, case.V, sel.sel_start, sel.sel_len, sel.sel_count, cfg.b)
    torch.cuda.synchronize()
    assert int(sel.sel_count.cpu()[0, 0]) == int(case.seg.slot_base[-1])
    assert int(sel.sel_len.sum().item()) == L
    Kh, Vh, qv = O.widen_bf16(wl.K[0]), O.widen_bf16(wl.V[0]), O.widen_bf16(q_bits[0, 0])
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(qv)[None, None, None], torch.from_numpy(Kh)[None, None], torch.from_numpy(Vh)[None, None],
        scale=DEFAULT_SCALE)[0, 0, 0].numpy()
    assert rel_err(att.out.cpu().numpy()[0, 0], ref) <= ATTN_TOL
    lse_ref = float(torch.logsumexp(torch.from_numpy(Kh @ qv) * DEFAULT_SCALE, 0))
    assert abs(float(att.lse.cpu()[0, 0]) - lse_ref) <= LSE_TOL


def test_exact_ties_go_to_lowest_slot_index():
    """A zero query scores every block 0: the k lowest-numbered slots must be chosen."""
    dsk = _dsk()
    case = gpu_case(2)
    cfg = case.cfg
    comp = case.compressed()
    q = torch.zeros(cfg.B, cfg.Hq, 128, dtype=torch.bfloat16, device="cuda")
    sel = dsk.select_topk(comp, q, cfg.T)
    torch.cuda.synchronize()
    want = np.arange(cfg.k)
    for h in (0, 7, cfg.Hq - 1):
        np.testing.assert_array_equal(sel.sel_slot.cpu().numpy()[0, h], want)
    # duplicate block scores made on purpose: copy one head's summaries of block 10 into 20..40
    ksum = comp.ksum.clone()
    ksum[:, 20:41] = ksum[:, 10:11]
    import dataclasses
    comp2 = dataclasses.replace(comp, ksum=ksum)
    wl = case.wl
    qb = wl.q[0]
    sel2 = dsk.select_topk(comp2, dev_bf16(qb), cfg.T, want_scores=True)
    torch.cuda.synchronize()
    sums = bf16_bits_of(ksum)
    seg = case.seg
    nb = int(seg.cu_blocks[-1])
    for h in (0, 3, 13):
        hk = h // cfg.G
        sc = O.block_scores(O.widen_bf16(qb[0, h])[None], O.widen_bf16(sums[hk, :nb, 0])[None],
                            O.widen_bf16(sums[hk, :nb, 1])[None])[0]
        o_sel, tau = O.select_slots(sc, seg.slot_base, cfg.k)
        cnt = int(sel2.sel_count.cpu()[0, h])
        selection_check(sel2.sel_slot.cpu().numpy()[0, h, :cnt], o_sel, tau, sc, seg.slot_base)


def test_small_and_large_budgets_and_b1():
    """k = 1, b = 1 (token-level mapping of Sec. 4.2), budgets that end inside a block, and
    budgets large enough for the staged emission of the selection kernel."""
    dsk = _dsk()
    case = gpu_case(1)
    cfg, wl, seg = case.cfg, case.wl, case.seg
    # the last three select more than 512 slots per head: emission staged through the work list,
    # with b = 1 in more than one round of it
    for b, budget in ((1, 1), (1, 37), (4, 4), (4, 50), (16, 16), (64, 200), (1, 513), (1, 2600), (4, 4000)):
        comp = dsk.compress(**case.compress_kwargs(
            stages=dsk.DSK_STAGE_CANDIDATES | dsk.DSK_STAGE_SEGMENT | dsk.DSK_STAGE_SUMMARIES,
            token_ids=case.token_ids, delim_ids=case.delim_ids, b=b))
        q_bits = wl.q[0]
        q = dev_bf16(q_bits)
        sel = dsk.select_topk(comp, q, budget)
        att = dsk.sparse_decode_attn(q, case.K, case.V, sel.sel_start, sel.sel_len, sel.sel_count, b)
        torch.cuda.synchronize()
        bs = seg.per_seq_block_start[0]
        sb = O.slot_map(bs, b)
        np.testing.assert_array_equal(comp.slot_base.cpu().numpy()[: len(sb)], sb)
        Kh, Vh, qv = O.widen_bf16(wl.K[0]), O.widen_bf16(wl.V[0]), O.widen_bf16(q_bits[0, 0])
        kmin, kmax = O.block_summaries(Kh[None], bs)
        sc = O.block_scores(qv[None], kmin, kmax)[0]
        o_sel, tau = O.select_slots(sc, sb, budget // b)
        cnt = int(sel.sel_count.cpu()[0, 0])
        gs = sel.sel_slot.cpu().numpy()[0, 0, :cnt]
        selection_check(gs, o_sel, tau, sc, sb)
        toks = O.selected_tokens(gs, bs, sb, b)
        o, lse = O.sparse_attention(qv, Kh, Vh, toks, DEFAULT_SCALE)
        assert rel_err(att.out.cpu().numpy()[0, 0], o) <= ATTN_TOL
        assert abs(float(att.lse.cpu()[0, 0]) - lse) <= LSE_TOL


def test_empty_selection_and_custom_scale():
    dsk = _dsk()
    case = gpu_case(1)
    wl = case.wl
    q = dev_bf16(wl.q[0])
    k = 4
    starts = dev_i32(np.asarray([[[5, 100, 0, 0]]]))
    lens = dev_i32(np.asarray([[[3, 16, 0, 0]]]))
    att = dsk.sparse_decode_attn(q, case.K, case.V, starts, lens, dev_i32([[0]]), 16)
    torch.cuda.synchronize()
    assert float(att.out.abs().max().item()) == 0.0 and float(att.lse.item()) == -math.inf
    att = dsk.sparse_decode_attn(q, case.K, case.V, starts, lens, dev_i32([[2]]), 16, scale=0.25)
    torch.cuda.synchronize()
    toks = np.concatenate([np.arange(5, 8), np.arange(100, 116)])
    o, lse = O.sparse_attention(O.widen_bf16(wl.q[0][0, 0]), O.widen_bf16(wl.K[0]), O.widen_bf16(wl.V[0]), toks, 0.25)
    assert rel_err(att.out.cpu().numpy()[0, 0], o) <= ATTN_TOL
    assert abs(float(att.lse.item()) - lse) <= LSE_TOL


def test_decode_is_deterministic():
    dsk = _dsk()
    case = gpu_case(2)
    cfg = case.cfg
    comp = case.compressed()
    q = dev_bf16(case.wl.q[0])
    outs = []
    for _ in range(2):
        sel = dsk.select_topk(comp, q, cfg.T)
        att = dsk.sparse_decode_attn(q, case.K, case.V, sel.sel_start, sel.sel_len, sel.sel_count, cfg.b)
        torch.cuda.synchronize()
        outs.append((sel.sel_slot.cpu().numpy().copy(), att.out.cpu().numpy().copy()))
    np.testing.assert_array_equal(outs[0][0], outs[1][0])
    np.testing.assert_array_equal(outs[0][1], outs[1][1])


def test_sequences_with_more_blocks_than_the_register_tile():
    """> 8189 blocks in one sequence: the memory-resident variant of the slot top-k."""
    dsk = _dsk()
    case = gpu_case(1, seqlens=[40000], C=4, delta=1, gap_means=[4], b=2, T=96, Hq=2, Hkv=1)
    cfg, seg, wl = case.cfg, case.seg, case.wl
    assert int(seg.cu_blocks[-1]) > 8192
    comp = case.compressed()
    nb = int(seg.cu_blocks[-1])
    np.testing.assert_array_equal(comp.block_start.cpu().numpy()[: nb + 1], seg.block_start)
    sums = bf16_bits_of(comp.ksum)
    for qi, q_bits in enumerate([wl.q[0], np.zeros_like(wl.q[0])]):
        q = dev_bf16(q_bits)
        sel = dsk.select_topk(comp, q, cfg.T)
        att = dsk.sparse_decode_attn(q, case.K, case.V, sel.sel_start, sel.sel_len, sel.sel_count, cfg.b)
        torch.cuda.synchronize()
        for h in range(cfg.Hq):
            sc = O.block_scores(O.widen_bf16(q_bits[0, h])[None], O.widen_bf16(sums[0, :nb, 0])[None],
                                O.widen_bf16(sums[0, :nb, 1])[None])[0]
            o_sel, tau = O.select_slots(sc, seg.slot_base, cfg.k)
            cnt = int(sel.sel_count.cpu()[0, h])
            gs = sel.sel_slot.cpu().numpy()[0, h, :cnt]
            selection_check(gs, o_sel, tau, sc, seg.slot_base)
            toks = O.selected_tokens(gs, seg.block_start, seg.slot_base, cfg.b)
            o, lse = O.sparse_attention(O.widen_bf16(q_bits[0, h]), O.widen_bf16(wl.K[0]), O.widen_bf16(wl.V[0]),
                                        toks, DEFAULT_SCALE)
            assert rel_err(att.out.cpu().numpy()[0, h], o) <= ATTN_TOL


def test_partials_only_leaves_mergeable_partials():
    """With DSK_ATTN_PARTIALS_ONLY the call stops after the per-chunk partials; merging them on
    the host by the documented formula must reproduce the library's own merged output (and
    hence the oracle's), and the layout query must describe where they are."""
    dsk = _dsk()
    case = gpu_case(2)
    cfg, wl = case.cfg, case.wl
    comp = case.compressed()
    q = dev_bf16(wl.q[0])
    sel = dsk.select_topk(comp, q, cfg.T)
    full = dsk.sparse_decode_attn(q, case.K, case.V, sel.sel_start, sel.sel_len, sel.sel_count, cfg.b)
    torch.cuda.synchronize()
    part = dsk.make_attn_args(q, case.K, case.V, sel.sel_start, sel.sel_len, sel.sel_count, cfg.b,
                              flags=dsk.DSK_ATTN_PARTIALS_ONLY)
    part.out.fill_(7.0)
    dsk.dsk_sparse_decode_attn(part.args)
    torch.cuda.synchronize()
    lay = dsk.dsk_attn_partials_layout(part.args)
    assert lay.nchunks == -(-cfg.k // lay.slots_per_chunk) and lay.nchunks > 1
    assert float(part.out.min().item()) == 7.0            # untouched: every head needs a merge here
    ws = part.keep[-1]                                    # the workspace tensor made by the binding
    assert ws.data_ptr() == int(part.args.workspace)
    raw = ws.view(torch.uint8).cpu().numpy()[:int(part.args.workspace_bytes)]
    n = cfg.B * cfg.Hq * lay.nchunks
    ml = raw[lay.ml_offset: lay.ml_offset + n * 8].view(np.float32).reshape(cfg.B, cfg.Hq, lay.nchunks, 2)
    acc = raw[lay.acc_offset: lay.acc_offset + n * 128 * 4].view(np.float32).reshape(cfg.B, cfg.Hq, lay.nchunks, 128)
    cnt = sel.sel_count.cpu().numpy()
    want_out = full.out.cpu().numpy()
    want_lse = full.lse.cpu().numpy()
    for s in range(cfg.B):
        for h in range(cfg.Hq):
            used = -(-min(int(cnt[s, h]), cfg.k) // lay.slots_per_chunk)
            m = ml[s, h, :used, 0].astype(np.float64)
            l = ml[s, h, :used, 1].astype(np.float64)
            M = m.max()
            wgt = np.exp2(m - M)
            den = float((l * wgt).sum())
            out = (acc[s, h, :used].astype(np.float64) * wgt[:, None]).sum(axis=0) / den
            assert rel_err(want_out[s, h], out) <= 1e-5
            assert abs(float(want_lse[s, h]) - (math.log(2.0) * M + math.log(den))) <= 1e-4


def test_decode_step_replays_correctly_from_a_hip_graph():
    """The decode calls hold no host state and enqueue only kernels, so a step captured once in a
    HIP graph can be replayed for new queries written into the same buffer: every replay (with
    eager work and synchronisations in between) must equal the eager result bit for bit."""
    dsk = _dsk()
    case = gpu_case(2)
    cfg, wl = case.cfg, case.wl
    comp = case.compressed()
    stream = torch.cuda.Stream()
    qbuf = dev_bf16(wl.q[0]).clone()
    with torch.cuda.stream(stream):
        sel = dsk.make_select_args(comp, qbuf, cfg.T)
        att = dsk.make_attn_args(qbuf, case.K, case.V, sel.sel_start, sel.sel_len, sel.sel_count, cfg.b)
        dsk.dsk_select_topk(sel.args, stream)                 # warm-up outside the capture
        dsk.dsk_sparse_decode_attn(att.args, stream)
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            dsk.dsk_select_topk(sel.args, stream)
            dsk.dsk_sparse_decode_attn(att.args, stream)
        gen = torch.Generator(device="cpu").manual_seed(11)
        for _ in range(4):
            q_new = torch.randn(cfg.B, cfg.Hq, 128, generator=gen).to(torch.bfloat16).cuda()
            ref_sel = dsk.select_topk(comp, q_new, cfg.T, stream=stream)
            ref_att = dsk.sparse_decode_attn(q_new, case.K, case.V, ref_sel.sel_start, ref_sel.sel_len,
                                             ref_sel.sel_count, cfg.b, stream=stream)
            qbuf.copy_(q_new)
            att.out.fill_(-1.0)
            stream.synchronize()
            graph.replay()
            stream.synchronize()
            assert torch.equal(sel.sel_slot, ref_sel.sel_slot) and torch.equal(sel.sel_count, ref_sel.sel_count)
            assert torch.equal(att.out, ref_att.out) and torch.equal(att.lse, ref_att.lse)


def test_batch_without_any_token():
    """Every sequence of the batch is empty: the tables are empty, nothing is selected, attention
    (sparse and full) returns the defined empty result; K and V have no row and are never read."""
    dsk = _dsk()
    case = gpu_case(5, B=3, seqlens=[0, 0, 0], T=256, n_queries=1)
    cfg = case.cfg
    assert case.K.numel() == 0
    comp = case.compressed()
    assert int(comp.dev_status.item()) == 0 and (comp.cu_blocks.cpu().numpy() == 0).all()
    q = dev_bf16(case.wl.q[0])
    sel = dsk.select_topk(comp, q, cfg.T)
    att = dsk.sparse_decode_attn(q, case.K, case.V, sel.sel_start, sel.sel_len, sel.sel_count, cfg.b)
    # selection arrays that claim slots although no token exists must not make the kernels read
    bogus = sel.sel_count.clone().fill_(cfg.k)
    att2 = dsk.sparse_decode_attn(q, case.K, case.V, sel.sel_start, sel.sel_len, bogus, cfg.b)
    dense = dsk.dense_decode_attn(q, case.K, case.V, case.cu_seqlens, 0)
    torch.cuda.synchronize()
    assert (sel.sel_count == 0).all() and (sel.sel_slot == -1).all()
    for r in (att, att2, dense):
        assert (r.out == 0).all() and torch.isneginf(r.lse).all()


def test_two_streams_with_their_own_workspaces_do_not_interfere():
    """The library keeps no state of its own: decode steps enqueued on two streams at once, each
    with its own outputs and workspace, give exactly what each gives alone."""
    dsk = _dsk()
    case = gpu_case(2)
    cfg, wl = case.cfg, case.wl
    comp = case.compressed()
    gen = torch.Generator(device="cpu").manual_seed(3)
    qs = [torch.randn(cfg.B, cfg.Hq, 128, generator=gen).to(torch.bfloat16).cuda() for _ in range(2)]
    alone = []
    for q in qs:
        sel = dsk.select_topk(comp, q, cfg.T)
        att = dsk.sparse_decode_attn(q, case.K, case.V, sel.sel_start, sel.sel_len, sel.sel_count, cfg.b)
        torch.cuda.synchronize()
        alone.append((sel.sel_slot.clone(), att.out.clone(), att.lse.clone()))
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]          # default priority both
    sels = [dsk.make_select_args(comp, q, cfg.T) for q in qs]
    atts = [dsk.make_attn_args(q, case.K, case.V, s.sel_start, s.sel_len, s.sel_count, cfg.b) for q, s in zip(qs, sels)]
    torch.cuda.synchronize()
    for _ in range(50):
        for i in (0, 1):
            dsk.dsk_select_topk(sels[i].args, streams[i])
            dsk.dsk_sparse_decode_attn(atts[i].args, streams[i])
    for st in streams:
        st.synchronize()
    for i in (0, 1):
        assert torch.equal(sels[i].sel_slot, alone[i][0])
        assert torch.equal(atts[i].out, alone[i][1]) and torch.equal(atts[i].lse, alone[i][2])


@pytest.mark.parametrize("shared", [False, True])
def test_per_sequence_budgets(shared):
    """budget_per_seq: every sequence takes its own number of slots (a budget that follows the
    sequence length), clamped to 1..k; the arrays keep k entries per head."""
    dsk = _dsk()
    case = gpu_case(5, B=5, seqlens=[6000, 900, 0, 3000, 40], T=512, n_queries=1)
    cfg, seg, wl = case.cfg, case.seg, case.wl
    comp = case.compressed()
    budgets = np.asarray([512, 100, 64, 7, 100000], dtype=np.int32)      # 7 < b -> one slot; 100000 -> k
    want_k = [min(cfg.k, max(1, int(x) // cfg.b)) for x in budgets]
    q_bits = wl.q[0]
    q = dev_bf16(q_bits)
    sel = dsk.select_topk(comp, q, cfg.T, want_scores=True, shared=shared, budget_per_seq=dev_i32(budgets))
    att = dsk.sparse_decode_attn(q, case.K, case.V, sel.sel_start, sel.sel_len, sel.sel_count, cfg.b,
                                 flags=dsk.DSK_ATTN_SHARED_SELECTION if shared else 0)
    torch.cuda.synchronize()
    sums = bf16_bits_of(comp.ksum)
    g_slot, g_cnt, g_len = sel.sel_slot.cpu().numpy(), sel.sel_count.cpu().numpy(), sel.sel_len.cpu().numpy()
    g_start = sel.sel_start.cpu().numpy()
    out = att.out.cpu().numpy()
    G = cfg.G
    rows = [0, cfg.Hkv - 1] if shared else [0, 5, cfg.Hq - 1]
    for s in range(cfg.B):
        b0, b1 = int(seg.cu_blocks[s]), int(seg.cu_blocks[s + 1])
        if b1 == b0:
            assert (g_cnt[s] == 0).all()
            continue
        sb = seg.slot_base[b0: b1 + 1]
        for row in rows:
            heads = list(range(row * G, (row + 1) * G)) if shared else [row]
            osc = _oracle_scores(case, sums[:, :, 0], sums[:, :, 1], q_bits, s, heads)
            sc = O.group_block_scores(np.stack([osc[h] for h in heads]), G)[0] if shared else osc[row]
            o_sel, tau = O.select_slots(sc, sb - sb[0], want_k[s])
            cnt = int(g_cnt[s, row])
            assert cnt == len(o_sel) == min(want_k[s], int(sb[-1] - sb[0]))
            selection_check(g_slot[s, row, :cnt], o_sel + int(sb[0]), tau, sc, sb)
            assert (g_slot[s, row, cnt:] == -1).all() and (g_len[s, row, cnt:] == 0).all()
            toks = np.concatenate([np.arange(g_start[s, row, j], g_start[s, row, j] + g_len[s, row, j]) for j in range(cnt)])
            for h in heads:
                hk = h // G
                o, _ = O.sparse_attention(O.widen_bf16(q_bits[s, h]), O.widen_bf16(wl.K[hk][toks]),
                                          O.widen_bf16(wl.V[hk][toks]), np.arange(len(toks)), DEFAULT_SCALE)
                assert rel_err(out[s, h], o) <= ATTN_TOL
    # the same budget for every sequence through the array = the scalar budget
    same = dsk.select_topk(comp, q, cfg.T, shared=shared, budget_per_seq=dev_i32(np.full(cfg.B, cfg.T)))
    plain = dsk.select_topk(comp, q, cfg.T, shared=shared)
    torch.cuda.synchronize()
    assert torch.equal(same.sel_slot, plain.sel_slot) and torch.equal(same.sel_count, plain.sel_count)


def test_per_sequence_budget_on_the_memory_resident_selection_path():
    """A block-count hint that is too small sends a long sequence through the selection variant
    that keeps its keys in memory; the per-sequence budget must act there as well."""
    dsk = _dsk()
    case = gpu_case(5, B=2, seqlens=[80000, 900], T=1024, n_queries=1)
    cfg, seg = case.cfg, case.seg
    assert int(seg.cu_blocks[1]) > 1024                         # more blocks than the smallest register tile
    comp = case.compressed()
    q = dev_bf16(case.wl.q[0])
    budgets = dev_i32([160, 48])
    small_tile = dsk.select_topk(comp, q, cfg.T, budget_per_seq=budgets, max_blocks_per_seq=32)
    fitting = dsk.select_topk(comp, q, cfg.T, budget_per_seq=budgets)
    torch.cuda.synchronize()
    for name in ("sel_slot", "sel_start", "sel_len", "sel_count"):
        assert torch.equal(getattr(small_tile, name), getattr(fitting, name)), name
    assert (fitting.sel_count.cpu().numpy() == np.asarray([[160 // cfg.b] * cfg.Hq, [48 // cfg.b] * cfg.Hq])).all()
