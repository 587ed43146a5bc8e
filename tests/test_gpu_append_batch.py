"""GPU parity of dsk_append_tokens_batch (Sec. 4.1, incremental update during decoding, for all
sequences of a batch at once).  Every sequence owns a region of the tables; after every step each
region must hold, bit for bit, the table, slot map and summaries the oracle computes from scratch on
that sequence, and the decode step on such tables must select and attend as it does on the packed
tables of a batched compression of the same sequences."""
import numpy as np
import pytest
import torch

from oracle import dynsplit_oracle as O
from dsk_testutil import (DEFAULT_SCALE, assert_bf16_of, bf16_bits_of, canon_zero, dev_bf16, dev_i32, dev_u8, gpu_case,
                          oracle_means_bf16, oracle_summaries, rel_err, selection_check)

ATTN_TOL = 2e-3     # max relative error of the attention output against the fp64 oracle

pytestmark = pytest.mark.gpu


def _dsk():
    import paper_2602_03184_amd as dsk
    return dsk


class _Batch:
    """The sequences of a workload spread over regions with room to grow; sequence s starts with
    L0[s] of its tokens, the rest is appended step by step."""

    def __init__(self, case, L0, slack_rows=64, want_vsum=False, region_entries=None, summary_mode=0):
        dsk = _dsk()
        wl, cfg = case.wl, case.cfg
        self.dsk, self.case, self.wl, self.cfg = dsk, case, wl, cfg
        B = cfg.B
        self.full = [int(x) for x in wl.seqlens]
        self.src0 = [int(x) for x in wl.cu_seqlens[:-1]]
        self.L = [int(x) for x in L0]
        self.row0, r = [], 5                                  # an odd first row: nothing relies on alignment of regions
        for s in range(B):
            self.row0.append(r)
            r += self.full[s] + slack_rows + s
        self.total_rows = r + 3
        Hkv, D = wl.K.shape[0], wl.K.shape[2]
        self.K_bits = np.full((Hkv, self.total_rows, D), 0x7FC0, dtype=np.uint16)   # NaN rows between the regions
        self.V_bits = np.full((Hkv, self.total_rows, D), 0x7FC0, dtype=np.uint16)
        self.tok = np.full(self.total_rows, -7, dtype=np.int64)
        for s in range(B):
            a, n = self.src0[s], self.full[s]
            self.K_bits[:, self.row0[s]: self.row0[s] + n] = wl.K[:, a: a + n]
            self.V_bits[:, self.row0[s]: self.row0[s] + n] = wl.V[:, a: a + n]
            self.tok[self.row0[s]: self.row0[s] + n] = wl.token_ids[a: a + n]
        self.K, self.V = dev_bf16(self.K_bits), dev_bf16(self.V_bits)
        self.d_tok, self.d_delim = dev_i32(self.tok), dev_i32(wl.delim_ids)
        self.d_wq = dev_u8(wl.class_weight_q)
        self.C = [int(x) for x in wl.C]
        self.delta = [int(x) for x in wl.delta]
        if region_entries is None:
            region_entries = [dsk.dsk_block_capacity(self.full[s], 1, self.C[s] - self.delta[s]) + 1 + (s % 3)
                              for s in range(B)]
        self.entries = [int(x) for x in region_entries]
        self.blk0 = np.concatenate([[0], np.cumsum(self.entries)]).astype(np.int64)
        self.cand = [O.extract_candidates(wl.token_ids[self.src0[s]: self.src0[s] + self.full[s]], wl.delim_ids)
                     for s in range(B)]
        self.rb = dsk.compress_regions(
            seq_row0=self.row0, seq_len=self.L, region_entries=self.entries, Hq=cfg.Hq, K=self.K, V=self.V,
            token_ids=self.d_tok, delim_ids=self.d_delim, class_weight_q=self.d_wq, C_per_seq=self.C,
            delta_per_seq=self.delta, alpha_num=cfg.a_num, alpha_den=cfg.a_den, b=cfg.b, want_vsum=want_vsum,
            summary_mode=summary_mode)
        self.app = dsk.make_batch_appender(
            self.rb, self.K, self.V, self.d_tok, self.d_delim, self.d_wq, C_=max(self.C), delta=max(self.delta),
            C_per_seq=dev_i32(self.C), delta_per_seq=dev_i32(self.delta), alpha_num=cfg.a_num, alpha_den=cfg.a_den,
            max_new_tokens=64)
        torch.cuda.synchronize()
        assert int(self.rb.dev_status.item()) == 0
        self.ora = [self.oracle_table(s, self.L[s]) for s in range(B)]

    def oracle_table(self, s, n):
        if n == 0:
            return np.zeros(1, dtype=np.int64)
        pos, cls = self.cand[s]
        m = pos < n
        return O.dd_select(n, pos[m], cls[m], self.wl.class_weight_q[s], self.C[s], self.delta[s], self.cfg.a_num,
                           self.cfg.a_den)

    def append(self, n_new):
        want_i0 = []
        new_len = []
        for s in range(self.cfg.B):
            L_new = min(self.L[s] + int(n_new[s]), self.full[s])
            pos, cls = self.cand[s]
            m = pos < L_new
            tab, i0 = O.dd_select_append(self.ora[s], L_new, pos[m], cls[m], self.wl.class_weight_q[s], self.C[s],
                                         self.delta[s], self.cfg.a_num, self.cfg.a_den)
            self.ora[s] = tab
            want_i0.append(i0)
            new_len.append(L_new)
        self.app.len_new.copy_(dev_i32(new_len))
        self.app.step()
        torch.cuda.synchronize()
        self.L = new_len
        return want_i0

    def check_tables(self, want_i0=None):
        assert int(self.rb.dev_status.item()) == 0
        used = self.rb.blocks_used.cpu().numpy()
        bs = self.rb.block_start.cpu().numpy()
        sb = self.rb.slot_base.cpu().numpy()
        np.testing.assert_array_equal(self.rb.seq_len.cpu().numpy(), self.L)
        for s in range(self.cfg.B):
            want = self.ora[s]
            nb = len(want) - 1
            b0 = int(self.blk0[s])
            assert int(used[s]) == nb, (s, int(used[s]), nb)
            np.testing.assert_array_equal(bs[b0: b0 + nb + 1], want)
            np.testing.assert_array_equal(sb[b0: b0 + nb + 1], O.slot_map(want, self.cfg.b))
            if want_i0 is not None:
                assert int(self.app.first_recomputed[s].item()) == want_i0[s]
                assert int(self.app.first_stale_slot[s].item()) == int(O.slot_map(want, self.cfg.b)[want_i0[s]])

    def check_summaries(self, vsum=False, mean=False):
        sums = bf16_bits_of(self.rb.vsum if vsum else self.rb.ksum)
        X = self.V_bits if vsum else self.K_bits
        for s in range(self.cfg.B):
            want = self.ora[s]
            nb = len(want) - 1
            if nb == 0:
                continue
            b0 = int(self.blk0[s])
            rows = X[:, self.row0[s]: self.row0[s] + self.L[s]]
            got = sums[:, b0: b0 + nb]
            if mean:
                np.testing.assert_array_equal(got[:, :, 0], got[:, :, 1])      # the mean sits in both rows
                assert_bf16_of(got[:, :, 0], oracle_means_bf16(rows, want), max_off_frac=5e-3)
            else:
                mn, mx = oracle_summaries(rows, want)
                np.testing.assert_array_equal(canon_zero(got[:, :, 0]), canon_zero(mn))
                np.testing.assert_array_equal(canon_zero(got[:, :, 1]), canon_zero(mx))


def test_ragged_batch_grows_step_by_step():
    """Per-sequence C and delta, a sequence that starts empty, one that starts with one token, one
    that does not grow in some steps, bursts of several tokens."""
    case = gpu_case(5, B=5, seqlens=[1500, 400, 2600, 90, 900])
    bt = _Batch(case, [1100, 0, 2300, 1, 640], want_vsum=True)
    bt.check_tables()
    bt.check_summaries()
    r = np.random.default_rng(11)
    for step in range(140):
        n_new = r.choice([0, 1, 1, 1, 2, 5], size=case.cfg.B)
        if step % 37 == 36:
            n_new = r.integers(0, 64, size=case.cfg.B)
        i0 = bt.append(n_new)
        bt.check_tables(i0)
        if step % 35 == 34:
            bt.check_summaries()
            bt.check_summaries(vsum=True)
    while any(bt.L[s] < bt.full[s] for s in range(case.cfg.B)):     # run every sequence to its end
        i0 = bt.append([64] * case.cfg.B)
        bt.check_tables(i0)
    bt.check_summaries()
    bt.check_summaries(vsum=True)
    for s in range(case.cfg.B):                                     # = the table of a pass from scratch
        np.testing.assert_array_equal(bt.ora[s], bt.oracle_table(s, bt.full[s]))


def test_decode_on_region_tables_equals_decode_on_packed_tables():
    """dsk_select_topk with blocks_used / seq_row0 on the grown regions against the same call on a
    batched compression of the same sequences from scratch (itself checked against the oracle
    elsewhere): same slots, spans that differ by the region offsets only, bit-equal attention; one
    head per sequence also straight against the oracle."""
    dsk = _dsk()
    case = gpu_case(5, B=4, seqlens=[3000, 700, 5200, 64])
    cfg, wl = case.cfg, case.wl
    bt = _Batch(case, [2900, 640, 5100, 3])
    r = np.random.default_rng(3)
    while any(bt.L[s] < bt.full[s] for s in range(cfg.B)):
        bt.append(r.integers(1, 9, size=cfg.B))
    bt.check_tables()
    packed = case.compressed()
    q_bits = wl.q[0]
    q = dev_bf16(q_bits)
    sel_r = dsk.select_topk(bt.rb, q, cfg.T, want_scores=True)
    sel_p = dsk.select_topk(packed, q, cfg.T)
    att_r = dsk.sparse_decode_attn(q, bt.K, bt.V, sel_r.sel_start, sel_r.sel_len, sel_r.sel_count, cfg.b)
    att_p = dsk.sparse_decode_attn(q, case.K, case.V, sel_p.sel_start, sel_p.sel_len, sel_p.sel_count, cfg.b)
    torch.cuda.synchronize()
    assert torch.equal(sel_r.sel_count, sel_p.sel_count)
    assert torch.equal(sel_r.sel_len, sel_p.sel_len)
    cnt = sel_r.sel_count.cpu().numpy()
    st_r, st_p = sel_r.sel_start.cpu().numpy(), sel_p.sel_start.cpu().numpy()
    sl_r, sl_p = sel_r.sel_slot.cpu().numpy(), sel_p.sel_slot.cpu().numpy()
    cu_slots = packed.cu_slots.cpu().numpy()
    for s in range(cfg.B):
        for h in range(cfg.Hq):
            n = int(cnt[s, h])
            np.testing.assert_array_equal(st_r[s, h, :n] - bt.row0[s], st_p[s, h, :n] - int(wl.cu_seqlens[s]))
            np.testing.assert_array_equal(sl_r[s, h, :n], sl_p[s, h, :n] - int(cu_slots[s]))
            assert (sl_r[s, h, n:] == -1).all()
    assert torch.equal(att_r.out, att_p.out) and torch.equal(att_r.lse, att_p.lse)
    # one head per sequence against the oracle: scores of the region's blocks, slot set, attention
    sums = bf16_bits_of(bt.rb.ksum)
    g_scores = sel_r.scores.cpu().numpy()
    g_out = att_r.out.cpu().numpy()
    g_len = sel_r.sel_len.cpu().numpy()
    for s in range(cfg.B):
        h = (5 * s + 1) % cfg.Hq
        hk = h // cfg.G
        tab = bt.ora[s]
        nb = len(tab) - 1
        b0 = int(bt.blk0[s])
        kmin = O.widen_bf16(sums[hk, b0: b0 + nb, 0])
        kmax = O.widen_bf16(sums[hk, b0: b0 + nb, 1])
        osc = O.block_scores(O.widen_bf16(q_bits[s, h])[None], kmin[None], kmax[None])[0]
        np.testing.assert_allclose(g_scores[h, b0: b0 + nb], osc, rtol=2e-5, atol=2e-4)
        sb = O.slot_map(tab, cfg.b)
        o_sel, tau = O.select_slots(osc, sb, cfg.k)
        n = int(cnt[s, h])
        assert n == len(o_sel)
        selection_check(sl_r[s, h, :n], o_sel, tau, osc, sb)
        toks = np.concatenate([np.arange(st_r[s, h, j], st_r[s, h, j] + g_len[s, h, j]) for j in range(n)])
        o, _ = O.sparse_attention(O.widen_bf16(q_bits[s, h]), O.widen_bf16(bt.K_bits[hk][toks]),
                                  O.widen_bf16(bt.V_bits[hk][toks]), np.arange(len(toks)), DEFAULT_SCALE)
        assert rel_err(g_out[s, h], o) <= ATTN_TOL


def test_full_region_is_reported_and_does_not_touch_its_neighbour():
    """A region with too few entries for its sequence: DSK_ERR_CAPACITY, that sequence's table is
    truncated, the next region's entries are what they were."""
    dsk = _dsk()
    case = gpu_case(5, B=2, seqlens=[800, 600])
    bt = _Batch(case, [300, 600])
    # rebuild with a first region that holds the 300-token table but not the 800-token one
    nb_300 = len(bt.ora[0]) - 1
    nb_800 = len(bt.oracle_table(0, 800)) - 1
    assert nb_800 > nb_300 + 2
    entries = [nb_300 + 3, bt.entries[1]]
    bt = _Batch(case, [300, 600], region_entries=entries)
    before = bt.rb.block_start.cpu().numpy().copy()
    b1 = int(bt.blk0[1])
    for _ in range(8):
        new_len = [min(bt.L[0] + 64, 800), 600]
        bt.app.len_new.copy_(dev_i32(new_len))
        bt.app.step()
        bt.L = new_len
    torch.cuda.synchronize()
    assert int(bt.rb.dev_status.item()) == dsk.DSK_ERR_CAPACITY
    assert int(bt.rb.blocks_used.cpu()[0]) <= entries[0] - 1
    after = bt.rb.block_start.cpu().numpy()
    np.testing.assert_array_equal(after[b1: b1 + entries[1]], before[b1: b1 + entries[1]])


def test_mean_pooling_summaries_and_graph_replay():
    """Mean-pooling records through the batched update; the step captured in a HIP graph and
    replayed on fresh lengths gives the eager result."""
    dsk = _dsk()
    case = gpu_case(5, B=3, seqlens=[1200, 500, 900])
    bt = _Batch(case, [1000, 300, 2], summary_mode=dsk.DSK_SUMMARY_MEAN)
    for _ in range(5):
        bt.append([3, 1, 7])
    bt.check_tables()
    bt.check_summaries(mean=True)
    stream = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        bt.app.len_new.copy_(bt.rb.seq_len)                 # a no-op step while capturing
        with torch.cuda.graph(g, stream=stream):
            dsk.dsk_append_tokens_batch(bt.app.args, stream)
    stream.synchronize()
    for n_new in ([1, 1, 1], [0, 4, 2], [9, 0, 1]):
        new_len = [min(bt.L[s] + n_new[s], bt.full[s]) for s in range(3)]
        for s in range(3):
            pos, cls = bt.cand[s]
            m = pos < new_len[s]
            bt.ora[s], _ = O.dd_select_append(bt.ora[s], new_len[s], pos[m], cls[m], bt.wl.class_weight_q[s], bt.C[s],
                                              bt.delta[s], bt.cfg.a_num, bt.cfg.a_den)
        bt.app.len_new.copy_(dev_i32(new_len))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        bt.L = new_len
        bt.check_tables()
        bt.check_summaries(mean=True)
