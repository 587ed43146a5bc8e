"""GPU parity of dsk_compress (candidates, DD-Select segmentation, slot map, min/max
summaries) against the fp64 oracle.  Integer outputs and bf16 summaries must be bit-exact."""
import numpy as np
import pytest
import torch

from oracle import dynsplit_oracle as O
from workloads import CONFIGS, f32_to_bf16_bits
from dsk_testutil import (GpuCase, bf16_bits_of, canon_zero, dev_bf16, dev_i32, dev_u8, gpu_case,
                          kv_heads_to_check, oracle_segment, oracle_summaries)

pytestmark = pytest.mark.gpu


def _dsk():
    import paper_2602_03184_amd as dsk
    return dsk


def _check_tables(comp, seg, status=0):
    nb = int(seg.cu_blocks[-1])
    assert int(comp.dev_status.item()) == status
    np.testing.assert_array_equal(comp.cu_blocks.cpu().numpy(), seg.cu_blocks)
    np.testing.assert_array_equal(comp.block_start.cpu().numpy()[: nb + 1], seg.block_start)
    np.testing.assert_array_equal(comp.slot_base.cpu().numpy()[: nb + 1], seg.slot_base)
    if comp.cu_slots is not None:      # slot range of every sequence = slot_base at its first block
        np.testing.assert_array_equal(comp.cu_slots.cpu().numpy(), seg.slot_base[seg.cu_blocks])
    if (status == 0 and comp.cand_pos is not None and (comp.args.stages & _dsk().DSK_STAGE_CANDIDATES)
            and getattr(seg, "cand_cu", None) is not None):
        n = int(seg.cand_cu[-1])       # lists written by this call (by the candidate or the segmentation kernels)
        np.testing.assert_array_equal(comp.cand_cu.cpu().numpy(), seg.cand_cu)
        np.testing.assert_array_equal(comp.cand_pos.cpu().numpy()[:n], seg.cand_pos)
        np.testing.assert_array_equal(comp.cand_class.cpu().numpy()[:n], seg.cand_class)


# --------------------------------------------------------------------------- full configs
@pytest.mark.parametrize("cfg_id", [1, 2, 3, 4, 5])
def test_candidates_and_segmentation_bit_exact(cfg_id):
    dsk = _dsk()
    case = gpu_case(cfg_id)
    cfg, seg = case.cfg, case.seg
    comp = dsk.compress(**case.compress_kwargs(
        stages=dsk.DSK_STAGE_CANDIDATES | dsk.DSK_STAGE_SEGMENT, token_ids=case.token_ids,
        delim_ids=case.delim_ids, M=cfg.M, W=cfg.W, R=cfg.R))
    torch.cuda.synchronize()
    n = int(seg.cand_cu[-1])
    np.testing.assert_array_equal(comp.cand_cu.cpu().numpy(), seg.cand_cu)
    np.testing.assert_array_equal(comp.cand_pos.cpu().numpy()[:n], seg.cand_pos)
    np.testing.assert_array_equal(comp.cand_class.cpu().numpy()[:n], seg.cand_class)
    _check_tables(comp, seg)
    # sampled candidates for Alg. 1
    samp = comp.samp_pos.cpu().numpy()
    for s in range(cfg.B):
        lo, hi = int(case.wl.cu_seqlens[s]), int(case.wl.cu_seqlens[s + 1])
        a, b = int(seg.cand_cu[s]), int(seg.cand_cu[s + 1])
        want = O.sample_candidates(seg.cand_pos[a:b] - lo, seg.cand_class[a:b], cfg.n_class, cfg.M, cfg.R,
                                   cfg.W, hi - lo)
        want = np.where(want >= 0, want + lo, -1)
        np.testing.assert_array_equal(samp[s], want)


@pytest.mark.parametrize("cfg_id", [1, 2, 5])
def test_candidate_lists_alone_and_from_the_segmentation_kernels(cfg_id):
    """Stage CANDIDATES on its own runs the candidate kernels; together with stage SEGMENT (weights
    from a table) the segmentation kernels write the lists on their way.  Both must give the
    oracle's lists, and a list that is too short is reported the same way by both."""
    dsk = _dsk()
    case = gpu_case(cfg_id)
    cfg, seg = case.cfg, case.seg
    n = int(seg.cand_cu[-1])
    for stages in (dsk.DSK_STAGE_CANDIDATES, dsk.DSK_STAGE_CANDIDATES | dsk.DSK_STAGE_SEGMENT):
        comp = dsk.compress(**case.compress_kwargs(stages=stages, token_ids=case.token_ids,
                                                   delim_ids=case.delim_ids, M=cfg.M, W=cfg.W, R=cfg.R))
        torch.cuda.synchronize()
        assert int(comp.dev_status.cpu()[0]) == dsk.DSK_OK
        np.testing.assert_array_equal(comp.cand_cu.cpu().numpy(), seg.cand_cu)
        np.testing.assert_array_equal(comp.cand_pos.cpu().numpy()[:n], seg.cand_pos)
        np.testing.assert_array_equal(comp.cand_class.cpu().numpy()[:n], seg.cand_class)
        short = n // 2
        comp = dsk.compress(**case.compress_kwargs(stages=stages, token_ids=case.token_ids,
                                                   delim_ids=case.delim_ids, max_cand_total=short))
        torch.cuda.synchronize()
        assert int(comp.dev_status.cpu()[0]) == dsk.DSK_ERR_CAPACITY
        np.testing.assert_array_equal(comp.cand_cu.cpu().numpy(), seg.cand_cu)      # the true totals
        np.testing.assert_array_equal(comp.cand_pos.cpu().numpy()[:short], seg.cand_pos[:short])
        np.testing.assert_array_equal(comp.cand_class.cpu().numpy()[:short], seg.cand_class[:short])
        if stages & dsk.DSK_STAGE_SEGMENT:
            _check_tables(comp, seg, status=dsk.DSK_ERR_CAPACITY)                   # the segmentation does not read the lists


@pytest.mark.parametrize("cfg_id", [1, 3])
def test_segmentation_with_paper_window_14(cfg_id):
    """Base chunk size 14 (Sec. 5.1 setup), delta 7, from explicit candidate lists."""
    dsk = _dsk()
    case = gpu_case(cfg_id)
    wl = case.wl
    import dataclasses
    wl14 = dataclasses.replace(wl, C=np.full(wl.cfg.B, 14, np.int32), delta=np.full(wl.cfg.B, 7, np.int32))
    seg = oracle_segment(wl14)
    comp = dsk.compress(**case.compress_kwargs(
        stages=dsk.DSK_STAGE_SEGMENT, cand_pos=dev_i32(seg.cand_pos), cand_class=dev_u8(seg.cand_class),
        cand_cu=dev_i32(seg.cand_cu), C_=14, delta=7, C_per_seq=None, delta_per_seq=None, min_chunk=7))
    torch.cuda.synchronize()
    _check_tables(comp, seg)


@pytest.mark.parametrize("cfg_id", [1, 3, 5])
def test_compression_without_candidate_lists(cfg_id):
    """Table-mode weights need no candidate list: with the lists left out the class map goes
    straight to the segmentation, and the tables and summaries are those of the full call."""
    dsk = _dsk()
    case = gpu_case(cfg_id)
    full = case.compressed()
    lean = dsk.compress(**case.compress_kwargs(
        stages=dsk.DSK_STAGE_CANDIDATES | dsk.DSK_STAGE_SEGMENT | dsk.DSK_STAGE_SUMMARIES,
        token_ids=case.token_ids, delim_ids=case.delim_ids, want_candidates=False))
    torch.cuda.synchronize()
    assert lean.cand_pos is None and lean.args.max_cand_total == 0
    assert int(lean.dev_status.item()) == 0
    _check_tables(lean, case.seg)
    nb = int(case.seg.cu_blocks[-1])
    assert torch.equal(lean.ksum[:, :nb], full.ksum[:, :nb])


@pytest.mark.parametrize("cfg_id", [1, 2, 3, 4, 5])
def test_summaries_bit_exact(cfg_id):
    case = gpu_case(cfg_id)
    cfg, seg, wl = case.cfg, case.seg, case.wl
    comp = case.compressed()
    _check_tables(comp, seg)
    nb = int(seg.cu_blocks[-1])
    heads = kv_heads_to_check(cfg)           # covers every KV head the decode parity reads summaries of
    got = bf16_bits_of(comp.ksum)            # [Hkv, cap, 2, D]
    kmin, kmax = oracle_summaries(wl.K, seg.block_start, heads)
    for j, h in enumerate(heads):
        np.testing.assert_array_equal(canon_zero(got[h, :nb, 0]), canon_zero(kmin[j]))
        np.testing.assert_array_equal(canon_zero(got[h, :nb, 1]), canon_zero(kmax[j]))


def test_v_summaries_and_strided_layout():
    """V summaries on request; K/V given as token-major (NHD) views with a padded token stride."""
    dsk = _dsk()
    case = gpu_case(2)
    cfg, seg, wl = case.cfg, case.seg, case.wl
    L = wl.total_tokens
    buf = torch.zeros(L, cfg.Hkv, 2, 128 + 64, dtype=torch.bfloat16, device="cuda")
    buf[:, :, 0, :128] = case.K.permute(1, 0, 2)
    buf[:, :, 1, :128] = case.V.permute(1, 0, 2)
    Kv = buf[:, :, 0, :128].permute(1, 0, 2)
    Vv = buf[:, :, 1, :128].permute(1, 0, 2)
    comp = dsk.compress(**case.compress_kwargs(
        stages=dsk.DSK_STAGE_SUMMARIES, K=Kv, V=Vv, want_vsum=True, block_start=dev_i32(seg.block_start),
        cu_blocks=dev_i32(seg.cu_blocks), total_tokens=L, Hkv=cfg.Hkv))
    torch.cuda.synchronize()
    nb = int(seg.cu_blocks[-1])
    heads = [0, 5]
    for X, got in ((wl.K, comp.ksum), (wl.V, comp.vsum)):
        mn, mx = oracle_summaries(X, seg.block_start, heads)
        g = bf16_bits_of(got)
        for j, h in enumerate(heads):
            np.testing.assert_array_equal(canon_zero(g[h, :nb, 0]), canon_zero(mn[j]))
            np.testing.assert_array_equal(canon_zero(g[h, :nb, 1]), canon_zero(mx[j]))


# --------------------------------------------------------------------------- edge cases
def _segment_from_lists(seqlens, cands, wq, C, delta, a_num, a_den, b, *, per_seq=None):
    """Run stage SEGMENT on explicit per-sequence candidate lists; return (comp, oracle tables)."""
    dsk = _dsk()
    B = len(seqlens)
    cu = np.zeros(B + 1, np.int64)
    cu[1:] = np.cumsum(seqlens)
    pos_g, cls_g, ccu = [], [], [0]
    bs_g, sb_g, cub, slot_off = [], [], [0], 0
    for s in range(B):
        pos, cls = cands[s]
        pos, cls = np.asarray(pos, np.int64), np.asarray(cls, np.int64)
        pos_g.append(pos + cu[s])
        cls_g.append(cls)
        ccu.append(ccu[-1] + len(pos))
        Cs, ds = (C, delta) if per_seq is None else per_seq[s]
        bs = O.dd_select(int(seqlens[s]), pos, cls, wq[s], Cs, ds, a_num, a_den) if seqlens[s] > 0 else np.zeros(1, np.int64)
        sb = O.slot_map(bs, b)
        bs_g.append(bs[:-1] + cu[s])
        sb_g.append(sb[:-1] + slot_off)
        slot_off += int(sb[-1])
        cub.append(cub[-1] + len(bs) - 1)
    bs_g.append(np.asarray([cu[-1]]))
    sb_g.append(np.asarray([slot_off]))
    pos_all = np.concatenate(pos_g) if pos_g else np.zeros(0, np.int64)
    cls_all = np.concatenate(cls_g) if cls_g else np.zeros(0, np.int64)
    kw = dict(cu_seqlens=dev_i32(cu), max_seqlen=int(max(seqlens)), Hq=1, K=None, Hkv=1, total_tokens=int(cu[-1]),
              stages=dsk.DSK_STAGE_SEGMENT, n_class=len(wq[0]), class_weight_q=dev_u8(np.asarray(wq)),
              cand_pos=dev_i32(pos_all) if len(pos_all) else None,
              cand_class=dev_u8(cls_all) if len(pos_all) else None, cand_cu=dev_i32(ccu),
              max_cand_total=len(pos_all), C_=C, delta=delta, alpha_num=a_num, alpha_den=a_den, b=b)
    if per_seq is not None:
        kw["C_per_seq"] = dev_i32([p[0] for p in per_seq])
        kw["delta_per_seq"] = dev_i32([p[1] for p in per_seq])
        kw["min_chunk"] = min(p[0] - p[1] for p in per_seq)
    comp = dsk.compress(**kw)
    torch.cuda.synchronize()
    return comp, np.concatenate(bs_g), np.asarray(cub), np.concatenate(sb_g)


def _assert_seg(comp, bs, cub, sb):
    nb = int(cub[-1])
    assert int(comp.dev_status.item()) == 0
    np.testing.assert_array_equal(comp.cu_blocks.cpu().numpy(), cub)
    np.testing.assert_array_equal(comp.block_start.cpu().numpy()[: nb + 1], bs)
    np.testing.assert_array_equal(comp.slot_base.cpu().numpy()[: nb + 1], sb)
    np.testing.assert_array_equal(comp.cu_slots.cpu().numpy(), sb[cub])


@pytest.mark.parametrize("L", [1, 2, 23, 24, 25, 36, 37, 1023, 1024, 1025, 2048 + 17])
def test_short_and_tile_edge_lengths(L):
    r = np.random.default_rng(L)
    pos = np.nonzero(r.random(L) < 0.08)[0]
    cls = r.integers(0, 4, len(pos))
    wq = [r.integers(0, 11, 4)]
    comp, bs, cub, sb = _segment_from_lists([L], [(pos, cls)], wq, 24, 12, 5, 10, 16)
    _assert_seg(comp, bs, cub, sb)


@pytest.mark.parametrize("C,delta,b,dens", [(2, 1, 1, 0.5), (3, 0, 2, 0.3), (16, 15, 4, 0.2), (1500, 700, 32, 0.01),
                                            (64, 32, 1024, 0.05), (1, 0, 1, 0.5), (4096, 4095, 16, 0.002)])
def test_extreme_chunk_parameters(C, delta, b, dens):
    r = np.random.default_rng(C * 31 + delta)
    L = 7000
    pos = np.nonzero(r.random(L) < dens)[0]
    cls = r.integers(0, 3, len(pos))
    wq = [r.integers(0, 11, 3)]
    for a_num in (0, 3, 10):
        comp, bs, cub, sb = _segment_from_lists([L], [(pos, cls)], wq, C, delta, a_num, 10, b)
        _assert_seg(comp, bs, cub, sb)


def test_degenerate_candidate_sets():
    L = 5000
    allpos = np.arange(L)
    for cands in ((np.zeros(0, int), np.zeros(0, int)), (allpos, np.zeros(L, int)), (allpos, allpos % 3)):
        for a_num in (0, 5, 10):
            comp, bs, cub, sb = _segment_from_lists([L], [cands], [[7, 3, 9]], 30, 15, a_num, 10, 16)
            _assert_seg(comp, bs, cub, sb)


def test_ragged_batch_with_empty_and_tiny_sequences():
    r = np.random.default_rng(77)
    seqlens = [3000, 0, 1, 1024, 17, 0, 4097]
    per_seq = [(16, 8), (32, 16), (64, 32), (16, 8), (64, 10), (32, 1), (40, 39)]
    cands, wq = [], []
    for L in seqlens:
        pos = np.nonzero(r.random(L) < 0.06)[0]
        cands.append((pos, r.integers(0, 5, len(pos))))
        wq.append(r.integers(0, 11, 5))
    comp, bs, cub, sb = _segment_from_lists(seqlens, cands, wq, 64, 39, 5, 10, 16, per_seq=per_seq)
    _assert_seg(comp, bs, cub, sb)


def test_block_capacity_overflow_is_reported_not_fatal():
    dsk = _dsk()
    L = 4000
    cu = dev_i32([0, L])
    comp = dsk.compress(cu_seqlens=cu, max_seqlen=L, Hq=1, K=None, Hkv=1, total_tokens=L,
                        stages=dsk.DSK_STAGE_SEGMENT, n_class=1, class_weight_q=dev_u8([5]),
                        cand_cu=dev_i32([0, 0]), max_cand_total=0, C_=10, delta=0, b=4, max_blocks_total=100)
    torch.cuda.synchronize()
    assert int(comp.dev_status.item()) == dsk.DSK_ERR_CAPACITY
    assert int(comp.cu_blocks.cpu()[1]) == 400
    np.testing.assert_array_equal(comp.block_start.cpu().numpy()[:100], np.arange(100) * 10)


@pytest.mark.parametrize("C,delta,gap", [(1312, 944, 1), (4000, 3900, 1), (700, 699, 2)])
def test_wide_search_ranges_with_delimiters_everywhere(C, delta, gap):
    """Thousands of delimiters in reach, each offering its boundary to thousands of chunk starts:
    tens of millions of (delimiter, start) votes per tile, far more than fit a 32-bit
    reciprocal-multiply division of the pair number."""
    from dsk_testutil import drop_cases
    dsk = _dsk()
    case = gpu_case(2, B=3, Hq=1, Hkv=1, seqlens=[8915, 5297, 85], b=4, T=16, C=C, delta=delta, a_num=0,
                    n_queries=1, n_class=3, gap_means=[gap])
    _check_tables(case.compressed(), case.seg)
    one = gpu_case(2, B=1, Hq=1, Hkv=1, seqlens=[7000], b=16, T=64, C=C, delta=delta, a_num=7, n_queries=1,
                   n_class=3, gap_means=[gap])
    _check_tables(one.compressed(), one.seg)
    drop_cases()


def test_compress_is_deterministic():
    case = gpu_case(2)
    dsk = _dsk()
    outs = []
    for _ in range(2):
        comp = dsk.compress(**case.compress_kwargs(
            stages=dsk.DSK_STAGE_CANDIDATES | dsk.DSK_STAGE_SEGMENT | dsk.DSK_STAGE_SUMMARIES,
            token_ids=case.token_ids, delim_ids=case.delim_ids))
        torch.cuda.synchronize()
        nb = int(comp.cu_blocks.cpu()[-1])
        outs.append((comp.block_start.cpu().numpy()[: nb + 1].copy(), bf16_bits_of(comp.ksum)[:, :nb].copy()))
    np.testing.assert_array_equal(outs[0][0], outs[1][0])
    np.testing.assert_array_equal(outs[0][1], outs[1][1])


def test_compression_pass_replays_correctly_from_a_hip_graph():
    """The pass enqueues kernels only (no allocation, no memset, no synchronisation), so it can be
    captured once and replayed on new token ids and K written into the same buffers: every replay,
    with eager work and synchronisations in between, must reproduce the eager result bit for bit."""
    dsk = _dsk()
    case = gpu_case(2, seqlens=[9000])
    wl = case.wl
    stream = torch.cuda.Stream()
    tok = case.token_ids.clone()
    K = case.K.clone()
    kw = case.compress_kwargs(stages=dsk.DSK_STAGE_CANDIDATES | dsk.DSK_STAGE_SEGMENT | dsk.DSK_STAGE_SUMMARIES,
                              delim_ids=case.delim_ids)
    with torch.cuda.stream(stream):
        captured = dsk.compress(**dict(kw, token_ids=tok, K=K, stream=stream))       # also the warm-up
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            dsk.dsk_compress(captured.args, stream)
        for shift in (0, 1, 17, 300):
            tok.copy_(torch.roll(case.token_ids, shift))
            K.copy_(torch.roll(case.K, shift, dims=1))
            stream.synchronize()
            eager = dsk.compress(**dict(kw, token_ids=tok, K=K, stream=stream))       # the program's own eager work
            stream.synchronize()
            captured.ksum.fill_(0)
            captured.block_start.fill_(-7)
            stream.synchronize()
            graph.replay()
            stream.synchronize()
            nb = int(eager.cu_blocks.cpu()[1])
            assert int(captured.dev_status.item()) == 0 and int(captured.cu_blocks.cpu()[1]) == nb
            assert torch.equal(captured.block_start[: nb + 1], eager.block_start[: nb + 1])
            assert torch.equal(captured.slot_base[: nb + 1], eager.slot_base[: nb + 1])
            assert torch.equal(captured.ksum[:, :nb], eager.ksum[:, :nb])
            n = int(eager.cand_cu.cpu()[1])
            assert torch.equal(captured.cand_pos[:n], eager.cand_pos[:n])


def test_unordered_candidate_list_is_reported():
    """Caller-provided candidate positions must ascend within a sequence: a swapped pair is
    reported through dev_status (DSK_ERR_ORDER) while the tables, which depend only on which
    positions are delimiters, still come out as for the sorted list."""
    dsk = _dsk()
    L, C, delta, b = 3000, 24, 12, 16
    rng = np.random.default_rng(5)
    pos = np.sort(rng.choice(L, size=120, replace=False))
    cls = rng.integers(0, 4, size=120)
    wq = [np.asarray([10, 5, 8, 6], np.uint8)]
    good, bs, cub, sb = _segment_from_lists([L], [(pos, cls)], wq, C, delta, 5, 10, b)
    _assert_seg(good, bs, cub, sb)
    bad_pos, bad_cls = pos.copy(), cls.copy()
    bad_pos[[40, 41]] = bad_pos[[41, 40]]
    bad_cls[[40, 41]] = bad_cls[[41, 40]]
    bad, _, _, _ = _segment_from_lists([L], [(bad_pos, bad_cls)], wq, C, delta, 5, 10, b)
    assert int(bad.dev_status.item()) == dsk.DSK_ERR_ORDER
    nb = int(cub[-1])
    np.testing.assert_array_equal(bad.block_start.cpu().numpy()[: nb + 1], bs)
    # a repeated position is not ascending either
    dup_pos = pos.copy()
    dup_pos[7] = dup_pos[6]
    dup, _, _, _ = _segment_from_lists([L], [(dup_pos, cls)], wq, C, delta, 5, 10, b)
    assert int(dup.dev_status.item()) == dsk.DSK_ERR_ORDER


@pytest.mark.parametrize("n_class,C,delta", [(1, 24, 12), (3, 7, 3), (5, 30, 0), (63, 100, 99), (64, 2, 1), (17, 900, 600)])
def test_tiles_classify_their_own_tokens(n_class, C, delta):
    """Candidates from token ids with no list asked for: the segmentation tiles compare the tokens
    in their reach with the delimiter ids themselves.  Class counts that are not multiples of the
    ids' vector width, search ranges from none to wider than a tile's vote window, a ragged batch
    with an empty and a one-token sequence: tables equal the oracle's and those of the call that
    goes through the candidate lists."""
    dsk = _dsk()
    case = gpu_case(5, B=5, seqlens=[4100, 0, 1, 2047, 9000], n_class=n_class, C=C, delta=delta,
                    gap_means=[max(2, C // 2)], Hq=2, Hkv=1)
    full = case.compressed()
    lean = dsk.compress(**case.compress_kwargs(
        stages=dsk.DSK_STAGE_CANDIDATES | dsk.DSK_STAGE_SEGMENT | dsk.DSK_STAGE_SUMMARIES,
        token_ids=case.token_ids, delim_ids=case.delim_ids, want_candidates=False))
    torch.cuda.synchronize()
    _check_tables(full, case.seg)
    _check_tables(lean, case.seg)
    nb = int(case.seg.cu_blocks[-1])
    assert torch.equal(lean.ksum[:, :nb], full.ksum[:, :nb])
