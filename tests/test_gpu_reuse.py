"""GPU parity of dsk_reuse_update (App. B.2, KVCache Reuse with V2F) against the oracle.

The plan is integer work: r, the resident table, the load list and the buffer's description
must equal the oracle's bit for bit, step after step, starting from an empty buffer.  The copied
K/V rows must equal the source rows byte for byte (zero beyond a slot's length).  Attention over
the resident buffers must match the fp64 oracle on the selected tokens within 2e-3, like the
attention that gathers straight from the cache."""
import numpy as np
import pytest
import torch

from oracle import dynsplit_oracle as O
from workloads import make_drifting_queries
from dsk_testutil import DEFAULT_SCALE, bf16_bits_of, dev_bf16, dev_i32, gpu_case, rel_err

pytestmark = pytest.mark.gpu

ATTN_TOL = 2e-3
LSE_TOL = 1e-3


def _dsk():
    import paper_2602_03184_amd as dsk
    return dsk


class _Mirror:
    """The oracle's copy of the resident state of one batch."""

    def __init__(self, B, Hq, k, b, D):
        self.B, self.Hq, self.k, self.b = B, Hq, k, b
        self.resident = [[[-1] * k for _ in range(Hq)] for _ in range(B)]
        self.length = np.zeros((B, Hq, k), dtype=np.int64)
        self.Kbuf = np.zeros((Hq, B * k * b, D), dtype=np.uint16)
        self.Vbuf = np.zeros((Hq, B * k * b, D), dtype=np.uint16)

    def step(self, s, sel_lists, spans, Kbits, Vbits, G, stale=None):
        r, new_res, loads = O.kv_reuse_plan(self.resident[s], sel_lists, stale)
        self.resident[s] = new_res
        k, b = self.k, self.b
        lo, hi = s * k * b, (s + 1) * k * b
        O.kv_reuse_apply(self.Kbuf[:, lo:hi], loads, Kbits, spans, b, G)
        O.kv_reuse_apply(self.Vbuf[:, lo:hi], loads, Vbits, spans, b, G)
        for h in range(self.Hq):
            for p in range(k):
                slot = new_res[h][p]
                self.length[s, h, p] = spans[slot][1] if slot >= 0 else 0
        return r, loads


def _check_step(dsk, case, mir, sel, reuser, q_bits, att_res, att_dir, heads, stale=None, check_rows=True):
    cfg, wl = case.cfg, case.wl
    B, Hq, k, b = cfg.B, cfg.Hq, mir.k, mir.b
    g_slot, g_start = sel.sel_slot.cpu().numpy(), sel.sel_start.cpu().numpy()
    g_len, g_cnt = sel.sel_len.cpu().numpy(), sel.sel_count.cpu().numpy()
    res_slot, res_len = reuser.res_slot.cpu().numpy(), reuser.res_len.cpu().numpy()
    res_start, res_count = reuser.res_start.cpu().numpy(), reuser.res_count.cpu().numpy()
    l_pos, l_slot = reuser.load_pos.cpu().numpy(), reuser.load_slot.cpu().numpy()
    l_start, l_len = reuser.load_start.cpu().numpy(), reuser.load_len.cpu().numpy()
    l_cnt, r_cnt = reuser.load_count.cpu().numpy(), reuser.reuse_count.cpu().numpy()
    rs = []
    for s in range(B):
        sel_lists = [[int(x) for x in g_slot[s, h, :g_cnt[s, h]]] for h in range(Hq)]
        spans = {}
        for h in range(Hq):
            for j in range(int(g_cnt[s, h])):
                spans[int(g_slot[s, h, j])] = (int(g_start[s, h, j]), int(g_len[s, h, j]))
        r, loads = mir.step(s, sel_lists, spans, wl.K, wl.V, cfg.G, None if stale is None else int(stale[s]))
        rs.append(r)
        assert int(r_cnt[s]) == r, (s, int(r_cnt[s]), r)
        for h in range(Hq):
            n = len(loads[h])
            assert int(l_cnt[s, h]) == n
            assert [(int(l_pos[s, h, i]), int(l_slot[s, h, i])) for i in range(n)] == loads[h]
            for i in range(n):
                assert (int(l_start[s, h, i]), int(l_len[s, h, i])) == spans[loads[h][i][1]]
            assert (l_pos[s, h, n:] == -1).all() and (l_slot[s, h, n:] == -1).all() and (l_len[s, h, n:] == 0).all()
            assert res_slot[s, h].tolist() == mir.resident[s][h]
            np.testing.assert_array_equal(res_len[s, h], mir.length[s, h])
            np.testing.assert_array_equal(res_start[s, h], (s * k + np.arange(k)) * b)
            held = [p for p in range(k) if mir.resident[s][h][p] >= 0]
            assert int(res_count[s, h]) == (held[-1] + 1 if held else 0)
    if check_rows:
        np.testing.assert_array_equal(bf16_bits_of(reuser.Kres), mir.Kbuf)
        np.testing.assert_array_equal(bf16_bits_of(reuser.Vres), mir.Vbuf)
    # attention over the resident buffers: against the oracle on the selected tokens, and next to
    # the attention that gathers from the cache
    o_res, lse_res = att_res.out.cpu().numpy(), att_res.lse.cpu().numpy()
    o_dir, lse_dir = att_dir.out.cpu().numpy(), att_dir.lse.cpu().numpy()
    for s in range(B):
        for h in heads:
            cnt = int(g_cnt[s, h])
            if cnt == 0:
                assert (o_res[s, h] == 0).all() and np.isneginf(lse_res[s, h])
                continue
            toks = np.concatenate([np.arange(g_start[s, h, j], g_start[s, h, j] + g_len[s, h, j]) for j in range(cnt)])
            hk = h // cfg.G
            o, lse = O.sparse_attention(O.widen_bf16(q_bits[s, h]), O.widen_bf16(wl.K[hk][toks]),
                                        O.widen_bf16(wl.V[hk][toks]), np.arange(len(toks)), DEFAULT_SCALE)
            assert rel_err(o_res[s, h], o) <= ATTN_TOL, (s, h)
            assert abs(float(lse_res[s, h]) - lse) <= LSE_TOL
    assert rel_err(o_res, o_dir.astype(np.float64)) <= 2 * ATTN_TOL
    np.testing.assert_allclose(lse_res, lse_dir, atol=2 * LSE_TOL)
    return rs


def _run(case, n_steps, rho, heads, *, T=None, K_src=None, V_src=None, repeat_at=(), stale_at=None, seed=11):
    dsk = _dsk()
    cfg, wl = case.cfg, case.wl
    comp = case.compressed()
    T = cfg.T if T is None else T
    qs = make_drifting_queries(np.random.default_rng(seed), n_steps, cfg.B, cfg.Hq, cfg.D, rho)
    q = dev_bf16(qs[0])
    sel = dsk.make_select_args(comp, q, T)
    stale_t = dev_i32(np.full(cfg.B, 0x7FFFFFFF)) if stale_at is not None else None
    Ks = case.K if K_src is None else K_src
    Vs = case.V if V_src is None else V_src
    reuser = dsk.make_reuser(sel, Ks, Vs, cfg.Hkv, stale_from=stale_t)
    mir = _Mirror(cfg.B, cfg.Hq, sel.k, cfg.b, cfg.D)
    att_res = att_dir = prev_bits = None
    history = []
    for t in range(n_steps):
        q_bits = prev_bits if t in repeat_at else qs[t]       # a repeated step sees the previous query again
        prev_bits = q_bits
        q.copy_(dev_bf16(q_bits))
        stale = None
        if stale_at is not None:
            stale = np.full(cfg.B, 0x7FFFFFFF, dtype=np.int64)
            if t == stale_at[0]:
                stale[:] = stale_at[1]
            stale_t.copy_(dev_i32(stale))
        dsk.dsk_select_topk(sel.args)
        reuser.step()
        att_res = reuser.attn_args(q, out=att_res)
        dsk.dsk_sparse_decode_attn(att_res.args)
        att_dir = dsk.make_attn_args(q, case.K, case.V, sel.sel_start, sel.sel_len, sel.sel_count, cfg.b, out=att_dir)
        dsk.dsk_sparse_decode_attn(att_dir.args)
        torch.cuda.synchronize()
        rs = _check_step(dsk, case, mir, sel, reuser, q_bits, att_res, att_dir, heads, stale)
        if t == 0:
            assert rs == [0] * cfg.B                         # nothing held yet
        if t in repeat_at and not (stale_at is not None and t == stale_at[0]):   # the same query again: all reused
            cnt = sel.sel_count.cpu().numpy()
            assert rs == [int(cnt[s].min()) for s in range(cfg.B)]
            assert int(reuser.load_count.sum()) == int((cnt - np.asarray(rs)[:, None]).sum())
        history.append(rs)
    return history, sel.k


def test_reuse_parity_single_head():
    """Configuration 1 (one head, 4K tokens): no truncation across heads, r is the plain overlap."""
    hist, k = _run(gpu_case(1), 6, 0.95, [0], repeat_at=(3,))
    assert max(r[0] for r in hist[1:]) > 0


def test_reuse_parity_gqa_reduced():
    """32 query heads over 8 KV heads on a reduced cache; the minimum over 32 heads truncates."""
    case = gpu_case(2, seqlens=[6000], T=512, n_queries=1)
    hist, k = _run(case, 6, 0.97, [0, 5, 17, 31], T=512, repeat_at=(2, 5))
    assert k == 32 and hist[2][0] == k and hist[5][0] == k


def test_reuse_parity_ragged_batch_with_short_sequences():
    """Four sequences; one has fewer slots than k (positions stay empty and the load lists are
    shorter), one is empty."""
    case = gpu_case(5, B=4, seqlens=[3000, 300, 0, 5000], T=512, n_queries=1)
    hist, k = _run(case, 5, 0.95, [0, 9, 31], T=512, repeat_at=(4,))
    assert all(r[2] == 0 for r in hist)                       # the empty sequence never reuses anything


def test_reuse_stale_tail_is_reloaded():
    """stale_from cuts reuse at a slot index for one step: held slots from there on are loaded
    again although they are selected."""
    case = gpu_case(2, seqlens=[6000], T=512, n_queries=1)
    comp = case.compressed()
    nslots = int(comp.slot_base.cpu().numpy()[int(comp.cu_blocks.cpu().numpy()[-1])])
    hist, k = _run(case, 4, 0.97, [0, 31], T=512, repeat_at=(2, 3), stale_at=(2, nslots // 2))
    assert hist[2][0] < k and hist[3][0] == k


def test_reuse_from_pinned_host_memory():
    """The K/V source lives in pinned host memory (the offloaded tier); the kernels read it in place."""
    case = gpu_case(2, seqlens=[6000], T=512, n_queries=1)
    Kh = torch.empty(case.K.shape, dtype=torch.bfloat16, pin_memory=True)
    Vh = torch.empty(case.V.shape, dtype=torch.bfloat16, pin_memory=True)
    Kh.copy_(case.K)
    Vh.copy_(case.V)
    torch.cuda.synchronize()
    _run(case, 3, 0.97, [0, 31], T=512, K_src=Kh, V_src=Vh)


def test_reuse_plan_only_and_full_size_plan():
    """Configuration 3 at full size (k = 128, b = 32, 32 heads): the plan alone (no K/V touched),
    every head checked."""
    dsk = _dsk()
    case = gpu_case(3)
    cfg = case.cfg
    comp = case.compressed()
    qs = make_drifting_queries(np.random.default_rng(5), 4, cfg.B, cfg.Hq, cfg.D, 0.98)
    q = dev_bf16(qs[0])
    sel = dsk.make_select_args(comp, q, cfg.T)
    reuser = dsk.make_reuser(sel, None, None, cfg.Hkv, plan_only=True)
    assert reuser.Kres is None
    resident = [[-1] * sel.k for _ in range(cfg.Hq)]
    seen_r = []
    for t in range(4):
        q.copy_(dev_bf16(qs[t]))
        dsk.dsk_select_topk(sel.args)
        reuser.step()
        torch.cuda.synchronize()
        g_slot, g_cnt = sel.sel_slot.cpu().numpy()[0], sel.sel_count.cpu().numpy()[0]
        r, resident, loads = O.kv_reuse_plan(resident, [g_slot[h, :g_cnt[h]].tolist() for h in range(cfg.Hq)])
        assert int(reuser.reuse_count[0]) == r
        assert reuser.res_slot.cpu().numpy()[0].tolist() == resident
        l_pos, l_slot = reuser.load_pos.cpu().numpy()[0], reuser.load_slot.cpu().numpy()[0]
        for h in range(cfg.Hq):
            n = len(loads[h])
            assert int(reuser.load_count[0, h]) == n == sel.k - r
            assert list(zip(l_pos[h, :n].tolist(), l_slot[h, :n].tolist())) == loads[h]
        seen_r.append(r)
    assert seen_r[0] == 0
    print("config 3 reuse counts over drifting queries (rho 0.98):", seen_r, "of k =", sel.k)


def test_reuse_large_k_spans_several_wave_chunks():
    """k = 320 positions per head (five 64-lane chunks, the last one ragged) with b = 16."""
    case = gpu_case(2, seqlens=[12000], T=5120, n_queries=1)
    hist, k = _run(case, 3, 0.97, [0, 13, 31], T=5120, repeat_at=(2,))
    assert k == 320


@pytest.mark.parametrize("cfg_id", [3, 4, 5])
def test_reuse_parity_full_size(cfg_id):
    """The full-size configurations (k = 128 x 32 rows, 256 x 16 rows with 40 separate KV heads,
    and the ragged batch of 8): plan, copied rows and attention over the buffers."""
    case = gpu_case(cfg_id)
    cfg = case.cfg
    heads = sorted({0, cfg.G, cfg.Hq // 2 + 1, cfg.Hq - 1})
    hist, k = _run(case, 3, 0.98, heads, repeat_at=(2,))
    assert k == cfg.k
    print("config %d reuse counts:" % cfg_id, hist, "of k =", k)


def test_reuse_in_a_decode_loop_with_appends():
    """The cache grows while decoding: dsk_append_tokens re-maps the slots of the open chunks and
    hands the first re-mapped slot to dsk_reuse_update as stale_from (device to device, nothing is
    read back).  Every step: plan and buffers against the oracle run with the oracle's own stale
    bound, attention over the buffers against the oracle on the current cache."""
    from test_gpu_append import _Seq
    dsk = _dsk()
    case = gpu_case(2, seqlens=[6000], T=512, n_queries=1)
    wl, cfg = case.wl, case.cfg
    seq = _Seq(wl.K, wl.V, wl.token_ids, wl.delim_ids, wl.class_weight_q[0], 4000, int(wl.C[0]), int(wl.delta[0]),
               cfg.a_num, cfg.a_den, cfg.b, Hq=cfg.Hq)
    n_steps = 10
    qs = make_drifting_queries(np.random.default_rng(3), n_steps, 1, cfg.Hq, cfg.D, 0.98)
    q = dev_bf16(qs[0])
    sel = dsk.make_select_args(seq.comp, q, 512)
    reuser = dsk.make_reuser(sel, seq.K, seq.V, cfg.Hkv, stale_from=seq.app.first_stale_slot)
    mir = _Mirror(1, cfg.Hq, sel.k, cfg.b, cfg.D)
    att_res = att_dir = None
    r_seen = []
    grow = [1, 1, 3, 1, 40, 1, 1, 200, 1, 1]
    for t in range(n_steps):
        q.copy_(dev_bf16(qs[t]))
        want, i0 = seq.append(grow[t])
        seq.check_tables(want, i0)
        stale = [int(O.slot_map(want, cfg.b)[i0])]
        dsk.dsk_select_topk(sel.args)
        reuser.step()
        att_res = reuser.attn_args(q, out=att_res)
        dsk.dsk_sparse_decode_attn(att_res.args)
        att_dir = dsk.make_attn_args(q, seq.K, seq.V, sel.sel_start, sel.sel_len, sel.sel_count, cfg.b, out=att_dir)
        dsk.dsk_sparse_decode_attn(att_dir.args)
        torch.cuda.synchronize()
        rs = _check_step(dsk, case, mir, sel, reuser, qs[t], att_res, att_dir, [0, 9, 31], stale)
        r_seen.append(rs[0])
    assert r_seen[0] == 0 and max(r_seen[1:]) > 0
    print("reuse counts while the cache grows:", r_seen, "of k =", sel.k)


def test_reuse_at_the_position_limit():
    """k = DSK_REUSE_MAX_K = 2048 positions per head (the most the per-wavefront LDS rows hold), on the
    32K-token cache of configuration 2, where that budget takes nearly every slot."""
    dsk = _dsk()
    case = gpu_case(2)
    hist, k = _run(case, 3, 0.9, [0, 31], T=dsk.DSK_REUSE_MAX_K * case.cfg.b, repeat_at=(2,))
    assert k == dsk.DSK_REUSE_MAX_K
    print("k = 2048 reuse counts:", hist)


def test_reuse_on_a_selection_shared_per_kv_head():
    """The two additions compose: with one selection per KV head the resident buffers are per KV
    head too (a quarter of the rows to hold and to load at G = 4), and all query heads of the group
    attend over their KV head's buffer."""
    dsk = _dsk()
    case = gpu_case(2, seqlens=[6000], T=512, n_queries=1)
    cfg, wl = case.cfg, case.wl
    comp = case.compressed()
    n_steps = 4
    qs = make_drifting_queries(np.random.default_rng(21), n_steps, 1, cfg.Hq, cfg.D, 0.97)
    q = dev_bf16(qs[0])
    sel = dsk.make_select_args(comp, q, 512, shared=True)
    reuser = dsk.make_reuser(sel, case.K, case.V, cfg.Hkv)
    assert reuser.Kres.shape[0] == cfg.Hkv
    resident = [[-1] * sel.k for _ in range(cfg.Hkv)]
    att = None
    seen = []
    for t in range(n_steps):
        q.copy_(dev_bf16(qs[t]))
        dsk.dsk_select_topk(sel.args)
        reuser.step()
        att = reuser.attn_args(q, out=att)
        dsk.dsk_sparse_decode_attn(att.args)
        torch.cuda.synchronize()
        g_slot, g_cnt = sel.sel_slot.cpu().numpy()[0], sel.sel_count.cpu().numpy()[0]
        g_start, g_len = sel.sel_start.cpu().numpy()[0], sel.sel_len.cpu().numpy()[0]
        r, resident, loads = O.kv_reuse_plan(resident, [g_slot[h, :g_cnt[h]].tolist() for h in range(cfg.Hkv)])
        seen.append(r)
        assert int(reuser.reuse_count[0]) == r
        assert reuser.res_slot.cpu().numpy()[0].tolist() == resident
        out, lse = att.out.cpu().numpy()[0], att.lse.cpu().numpy()[0]
        for hk in (0, cfg.Hkv - 1):
            toks = np.concatenate([np.arange(g_start[hk, j], g_start[hk, j] + g_len[hk, j]) for j in range(g_cnt[hk])])
            Kh, Vh = O.widen_bf16(wl.K[hk][toks]), O.widen_bf16(wl.V[hk][toks])
            for h in range(hk * cfg.G, (hk + 1) * cfg.G):
                o, l = O.sparse_attention(O.widen_bf16(qs[t][0, h]), Kh, Vh, np.arange(len(toks)), DEFAULT_SCALE)
                assert rel_err(out[h], o) <= ATTN_TOL and abs(float(lse[h]) - l) <= LSE_TOL
    assert seen[0] == 0 and max(seen[1:]) > 0


def test_reuse_step_replays_correctly_from_a_hip_graph():
    """select + reuse update + attention over the buffers captured once; each replay continues from
    the resident state the previous one left (with eager work and synchronisations in between) and
    must equal, bit for bit, an eager twin fed the same queries."""
    dsk = _dsk()
    case = gpu_case(2, seqlens=[6000], T=512, n_queries=1)
    cfg = case.cfg
    comp = case.compressed()
    stream = torch.cuda.Stream()
    qs = make_drifting_queries(np.random.default_rng(33), 6, 1, cfg.Hq, cfg.D, 0.97)
    qbuf, qref = dev_bf16(qs[0]).clone(), dev_bf16(qs[0]).clone()
    with torch.cuda.stream(stream):
        twins = []
        for qq in (qbuf, qref):
            sel = dsk.make_select_args(comp, qq, 512)
            ru = dsk.make_reuser(sel, case.K, case.V, cfg.Hkv)
            att = ru.attn_args(qq)
            twins.append((sel, ru, att))
        (gsel, gru, gatt), (esel, eru, eatt) = twins

        def step(sel, ru, att):
            dsk.dsk_select_topk(sel.args, stream)
            dsk.dsk_reuse_update(ru.args, stream)
            dsk.dsk_sparse_decode_attn(att.args, stream)

        step(gsel, gru, gatt)                                # warm-up outside the capture, then back to empty
        stream.synchronize()
        gru.res_slot.fill_(-1)
        gru.res_len.zero_()
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            step(gsel, gru, gatt)
        for t in range(6):
            qref.copy_(dev_bf16(qs[t]))
            stream.synchronize()
            step(esel, eru, eatt)                            # the program's own eager work between replays
            stream.synchronize()
            qbuf.copy_(dev_bf16(qs[t]))
            gatt.out.fill_(-1.0)
            stream.synchronize()
            graph.replay()
            stream.synchronize()
            for name in ("res_slot", "res_len", "res_count", "load_pos", "load_slot", "load_count", "reuse_count",
                         "Kres", "Vres"):
                assert torch.equal(getattr(gru, name), getattr(eru, name)), (t, name)
            assert torch.equal(gatt.out, eatt.out) and torch.equal(gatt.lse, eatt.lse), t
        assert int(gru.reuse_count[0]) > 0
