"""Pins of the fp64 oracle to things other than itself: hand-worked fixtures,
closed forms, brute force on tiny inputs, invariants, and special cases that
reduce to textbook / library routines.  CPU only."""
import itertools
import json
import math
import os

import numpy as np
import pytest
import torch

from oracle import dynsplit_oracle as O
from workloads import f32_to_bf16_bits, make_tokens

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


# ---------------------------------------------------------------- widen_bf16
def test_widen_bf16_matches_torch_bfloat16():
    bits = np.arange(0, 65536, dtype=np.uint32).astype(np.uint16)
    finite = ((bits >> 7) & 0xFF) != 0xFF
    bits = bits[finite]
    ref = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(O.widen_bf16(bits), ref)


# ---------------------------------------------------------------- candidates
def test_extract_candidates_matches_isin():
    r = rng(1)
    delim = np.asarray([7, 3, 11, 5], dtype=np.int32)
    tok = r.integers(0, 16, size=500).astype(np.int32)
    pos, cls = O.extract_candidates(tok, delim)
    np.testing.assert_array_equal(pos, np.nonzero(np.isin(tok, delim))[0])
    np.testing.assert_array_equal(delim[cls], tok[pos])


def test_sample_candidates_first_M_in_range():
    # class 0 at 1, 10, 20, 30, 40; class 1 at 5, 95
    pos = np.asarray([1, 5, 10, 20, 30, 40, 95])
    cls = np.asarray([0, 1, 0, 0, 0, 0, 1])
    samp = O.sample_candidates(pos, cls, n_class=3, M=2, R=8, W=4, L=100)
    # t must satisfy 8 <= t <= 95
    np.testing.assert_array_equal(samp, [[10, 20], [95, -1], [-1, -1]])
    samp = O.sample_candidates(pos, cls, n_class=3, M=2, R=8, W=5, L=100)   # t <= 94
    np.testing.assert_array_equal(samp[1], [-1, -1])
    # both edges are inclusive: t = R has a full retained region {1..R} behind it and a
    # non-empty discarded region {0}; t = L-1-W has its last window query at position L-1
    pos = np.asarray([7, 8, 95, 96])
    cls = np.asarray([0, 0, 0, 0])
    samp = O.sample_candidates(pos, cls, n_class=1, M=4, R=8, W=4, L=100)
    np.testing.assert_array_equal(samp, [[8, 95, -1, -1]])


# ---------------------------------------------------------------- Alg. 1
def _torch_causal_attention_map(Q, K, scale):
    """Textbook dense causal softmax map with a library softmax. Q,K: [L,D]."""
    Qt, Kt = torch.from_numpy(Q), torch.from_numpy(K)
    z = (Qt @ Kt.T) * scale
    L = z.shape[0]
    mask = torch.ones(L, L, dtype=torch.bool).tril()
    z = z.masked_fill(~mask, float("-inf"))
    return torch.softmax(z, dim=-1).numpy()


@pytest.mark.parametrize("t,R", [(40, 16), (17, 16), (16, 16), (5, 16)])
def test_importance_equals_sum_over_dense_attention_map(t, R):
    r = rng(2)
    L, D, Hq, Hkv, W = 64, 8, 4, 2, 3
    alpha = 0.75
    scale = 1.0 / math.sqrt(D)
    K = r.standard_normal((Hkv, L, D))
    Qfull = r.standard_normal((Hq, L, D))
    qwin = np.stack([Qfull[:, t + 1 + w] for w in range(W)])           # [W,Hq,D]
    got = O.delimiter_importance(qwin, K, t, R, alpha, scale)
    acc = 0.0
    for h in range(Hq):
        A = _torch_causal_attention_map(Qfull[h], K[h // (Hq // Hkv)], scale)
        for qpos in range(t + 1, t + 1 + W):
            ov = sum(A[qpos, k] for k in range(max(0, t - R + 1), t + 1))
            dr = sum(A[qpos, k] for k in range(0, max(0, t - R) + 1))
            acc += ov - alpha * dr
    assert got == pytest.approx(acc / (Hq * W), abs=1e-13)


def test_importance_closed_form_uniform_attention():
    # zero queries -> A[q,k] = 1/(q+1); s_t = (1/W) sum_q (R - alpha (t-R+1)) / (q+1)
    L, D, Hq, Hkv, W, R, t = 400, 4, 2, 1, 8, 128, 200
    for alpha in (1.0, 0.25):
        K = rng(3).standard_normal((Hkv, L, D))
        qwin = np.zeros((W, Hq, D))
        got = O.delimiter_importance(qwin, K, t, R, alpha, 0.5)
        want = sum((R - alpha * (t - R + 1)) / (q + 1) for q in range(t + 1, t + W + 1)) / W
        assert got == pytest.approx(want, abs=1e-14)


def test_importance_partition_identity_and_range():
    # alpha = -1 turns the score into the total mass on keys <= t; adding the mass
    # on the window's own keys (t+1..q) must give exactly 1 per row.
    r = rng(4)
    L, D, Hq, Hkv, W, R, t = 200, 16, 2, 2, 4, 32, 100
    K = r.standard_normal((Hkv, L, D))
    qwin = r.standard_normal((W, Hq, D))
    scale = 0.25
    mass_le_t = O.delimiter_importance(qwin, K, t, R, -1.0, scale)
    rest = 0.0
    for h in range(Hq):
        for w in range(W):
            qpos = t + 1 + w
            z = K[h, : qpos + 1] @ qwin[w, h] * scale
            A = np.exp(z - z.max())
            A /= A.sum()
            rest += A[t + 1:].sum()
    assert mass_le_t + rest / (Hq * W) == pytest.approx(1.0, abs=1e-13)
    for alpha in (1.0, 0.5):
        s = O.delimiter_importance(qwin, K, t, R, alpha, scale)
        assert -alpha <= s <= 1.0


def test_importance_concentrated_attention_hits_the_right_region():
    # one key aligned with every query and scaled up grabs (almost) all attention
    D, Hq, Hkv, W, R, L, t = 8, 1, 1, 2, 10, 60, 40
    qwin = np.zeros((W, Hq, D))
    qwin[:, :, 0] = 1.0
    for hot, want in ((35, 1.0), (31, 1.0), (30, -0.5), (0, -0.5), (41, 0.0)):
        K = np.zeros((Hkv, L, D))
        K[0, hot, 0] = 200.0
        s = O.delimiter_importance(qwin, K, t, R, 0.5, 1.0)
        assert s == pytest.approx(want, abs=1e-9), (hot, s)


def test_importance_over_layers_is_the_pooled_expectation():
    """Two layers through the layer-wise function = one call on a model whose heads are the two
    layers' heads side by side (every (layer, head, query) row weighs the same)."""
    r = rng(5200)
    W, Hq, Hkv, D, L, t, R = 3, 4, 2, 8, 40, 20, 6
    q1, q2 = r.standard_normal((W, Hq, D)), r.standard_normal((W, Hq, D))
    K1, K2 = r.standard_normal((Hkv, L, D)), r.standard_normal((Hkv, L, D))
    got = O.delimiter_importance_layers([q1, q2], [K1, K2], t, R, 1.0, 0.3)
    pooled = O.delimiter_importance(np.concatenate([q1, q2], axis=1), np.concatenate([K1, K2], axis=0), t, R, 1.0, 0.3)
    assert abs(got - pooled) < 1e-14
    one = O.delimiter_importance_layers([q1], [K1], t, R, 1.0, 0.3)
    assert one == O.delimiter_importance(q1, K1, t, R, 1.0, 0.3)
    # layers with different head counts are weighted by their rows
    q3, K3 = r.standard_normal((W, 2, D)), r.standard_normal((1, L, D))
    a, b = O.delimiter_importance(q1, K1, t, R, 1.0, 0.3), O.delimiter_importance(q3, K3, t, R, 1.0, 0.3)
    assert abs(O.delimiter_importance_layers([q1, q3], [K1, K3], t, R, 1.0, 0.3) - (4 * a + 2 * b) / 6) < 1e-14


def test_class_weights_table():
    samp = np.asarray([[5, 9], [7, -1], [-1, -1], [3, 4], [8, 9], [1, 2]])
    s = np.asarray([[1.0, 1.0], [0.12, 99.0], [0.0, 0.0], [-1.0, -1.0], [0.08, 0.08], [-0.3, 0.5]])
    prior = np.asarray([3, 3, 7, 3, 3, 3])
    wq, mean, edge = O.class_weights(s, samp, 1.0, prior)
    # (1+1)/2=1 ->10 ; (0.12+1)/2=.56 -> 6 ; empty keeps 7 ; (-1+1)/2=0 -> 0 ; .54 -> 5 ; mean .1 -> .55: edge
    assert list(wq[:5]) == [10, 6, 7, 0, 5]
    assert wq[5] in (5, 6) and edge[5] < 1e-9
    assert math.isnan(mean[2]) and mean[1] == pytest.approx(0.12)
    assert edge[1] == pytest.approx(0.1, abs=1e-9)          # 10*.56+.5 = 6.1
    # alpha = 0.5: range [-0.5, 1] -> (s + .5) / 1.5
    wq2, _, _ = O.class_weights(np.asarray([[0.4]]), np.asarray([[1]]), 0.5, np.asarray([0]))
    assert wq2[0] == 6                                        # .9/1.5 = .6
    # clamping outside the attainable range
    wq3, _, _ = O.class_weights(np.asarray([[5.0], [-7.0]]), np.asarray([[1], [1]]), 1.0, np.asarray([0, 0]))
    assert list(wq3) == [10, 0]


# ---------------------------------------------------------------- DD-Select
def test_dd_select_handworked_fixture():
    with open(os.path.join(GOLDEN, "dd_select_handworked.json")) as f:
        cases = json.load(f)["cases"]
    assert len(cases) >= 5
    for c in cases:
        got = O.dd_select(c["L"], c["cand_pos"], c["cand_class"], c["wq"], c["C"], c["delta"],
                          c["a_num"], c["a_den"])
        assert list(got) == c["block_start"], c["name"]


def _declarative_ok(bounds, L, offered, C, delta, alpha):
    """Is `bounds` (0=b0<...<bn=L) a segmentation in which every chunk end is what
    the procedure of Sec. 4.1 prescribes, stated as a predicate in real arithmetic
    (alpha*w + (1-alpha)*p with p = 1-|e-s_e|/max(delta,1)), not as a loop?"""
    dd = max(delta, 1)

    def f(e, s_e):
        return alpha * offered[e] + (1 - alpha) * (1 - abs(e - s_e) / dd)
    for s_c, e in zip(bounds[:-1], bounds[1:]):
        s_e = s_c + C
        if s_e >= L:
            if e != L:
                return False
            continue
        E = [x for x in offered if s_e - delta <= x <= min(L, s_e + delta)]
        if not E:
            if e != s_e:
                return False
            continue
        if e not in E:
            return False
        # exact rational comparison: weights are tenths, p is a multiple of 1/dd
        if any(f(x, s_e) > f(e, s_e) + 1e-12 for x in E):
            return False
        if any(abs(f(x, s_e) - f(e, s_e)) <= 1e-12 and x < e for x in E):
            return False
    return True


@pytest.mark.parametrize("seed", range(12))
def test_dd_select_unique_valid_split_by_enumeration(seed):
    r = rng(100 + seed)
    L = int(r.integers(6, 14))
    C = int(r.integers(2, 7))
    delta = int(r.integers(0, C))
    a_num, a_den = int(r.integers(0, 5)), 4
    n_class = 3
    wq = r.integers(0, 11, size=n_class)
    is_c = r.random(L) < 0.45
    pos = np.nonzero(is_c)[0]
    cls = r.integers(0, n_class, size=len(pos))
    offered = {int(t) + 1: wq[c] / 10.0 for t, c in zip(pos, cls)}
    got = list(O.dd_select(L, pos, cls, wq, C, delta, a_num, a_den))
    valid = []
    for mask in itertools.product([0, 1], repeat=L - 1):
        bounds = [0] + [i + 1 for i, m in enumerate(mask) if m] + [L]
        if _declarative_ok(bounds, L, offered, C, delta, a_num / a_den):
            valid.append(bounds)
    assert valid == [got]


def test_boundary_score_is_scaled_real_formula():
    for delta in range(0, 6):
        dd = max(delta, 1)
        for a_num, a_den in ((0, 1), (1, 1), (1, 2), (3, 10), (7, 10)):
            for wq in range(0, 11):
                for off in range(-delta, delta + 1):
                    s_e = 50
                    e = s_e + off
                    real = (a_num / a_den) * (wq / 10) + (1 - a_num / a_den) * (1 - abs(off) / dd)
                    assert O.boundary_score(e, s_e, wq, delta, a_num, a_den) == pytest.approx(
                        10 * a_den * dd * real, abs=1e-9)


def test_dd_select_closed_forms():
    L, C, delta = 1000, 24, 12
    fixed = list(range(0, L, C)) + [L]
    # no candidates, or delta = 0 with any candidates -> rigid fixed-interval splitting
    assert list(O.dd_select(L, [], [], [5], C, delta, 5, 10)) == fixed
    allpos, allcls = np.arange(L), np.zeros(L, dtype=int)
    # candidate everywhere, proximity only -> the ideal end always wins
    assert list(O.dd_select(L, allpos, allcls, [7], C, delta, 0, 10)) == fixed
    # candidate everywhere, equal weights, weight only -> all tie -> smallest e = s_e - delta
    got = O.dd_select(L, allpos, allcls, [7], C, delta, 10, 10)
    step = C - delta
    n_full = 0
    s = 0
    want = [0]
    while s + C < L:
        s += step
        want.append(s)
    want.append(L)
    assert list(got) == want
    # delta = 0: only a candidate exactly at s_e could matter, result is fixed anyway
    r = rng(5)
    pos = np.nonzero(r.random(L) < 0.1)[0]
    assert list(O.dd_select(L, pos, np.zeros(len(pos), int), [9], C, 0, 5, 10)) == fixed
    # L <= C: one chunk
    assert list(O.dd_select(10, [3], [0], [9], 10, 4, 5, 10)) == [0, 10]
    assert list(O.dd_select(1, [], [], [9], 3, 1, 5, 10)) == [0, 1]


@pytest.mark.parametrize("seed", range(6))
def test_dd_select_invariants_on_synthetic_streams(seed):
    r = rng(200 + seed)
    L = int(r.integers(2000, 6000))
    C = int(r.choice([14, 24, 32, 64]))
    delta = C // 2
    delim = np.arange(16, dtype=np.int32) * 7 + 3
    tok = make_tokens(r, L, delim, float(C), 0.05 if seed % 2 else 0.0)
    pos, cls = O.extract_candidates(tok, delim)
    wq = r.integers(5, 11, size=16)
    bs = O.dd_select(L, pos, cls, wq, C, delta, 5, 10)
    assert bs[0] == 0 and bs[-1] == L
    lens = np.diff(bs)
    assert (lens[:-1] >= C - delta).all() and (lens[:-1] <= C + delta).all()
    assert 1 <= lens[-1] <= C
    offered = set(int(t) + 1 for t in pos)
    for s_c, e in zip(bs[:-2], bs[1:-1]):
        window_has = any((x in offered) for x in range(s_c + C - delta, s_c + C + delta + 1))
        assert (e in offered) if window_has else (e == s_c + C)
    assert len(lens) <= -(-L // (C - delta))


# ---------------------------------------------------------------- slot map
@pytest.mark.parametrize("b", [1, 4, 16, 32])
def test_slot_map_invariants(b):
    r = rng(7)
    cuts = np.sort(r.choice(np.arange(1, 999), size=60, replace=False))
    bs = np.concatenate([[0], cuts, [999]])
    base = O.slot_map(bs, b)
    n_slots = int(base[-1])
    if b == 1:
        assert n_slots == 999
    covered = []
    prev_end = 0
    for g in range(n_slots):
        i, start, ln = O.slot_span(g, bs, base, b)
        assert 1 <= ln <= b and start == prev_end
        last_of_block = (g == base[i + 1] - 1)
        assert ln == b or last_of_block
        assert bs[i] <= start and start + ln <= bs[i + 1]
        prev_end = start + ln
        covered.append(ln)
    assert sum(covered) == 999 and prev_end == 999


# ---------------------------------------------------------------- summaries
def test_block_summaries_match_reduceat_and_singletons():
    r = rng(8)
    H, L, D = 2, 300, 8
    X = O.widen_bf16(f32_to_bf16_bits(r.standard_normal((H, L, D)).astype(np.float32)))
    cuts = np.sort(r.choice(np.arange(1, L), size=40, replace=False))
    bs = np.concatenate([[0], cuts, [L]])
    xmin, xmax = O.block_summaries(X, bs)
    for h in range(H):
        np.testing.assert_array_equal(xmin[h], np.minimum.reduceat(X[h], bs[:-1], axis=0))
        np.testing.assert_array_equal(xmax[h], np.maximum.reduceat(X[h], bs[:-1], axis=0))
    single = np.arange(L + 1)
    xmin, xmax = O.block_summaries(X, single)
    np.testing.assert_array_equal(xmin, X)
    np.testing.assert_array_equal(xmax, X)


# ---------------------------------------------------------------- block scores
def test_block_score_is_max_over_bounding_box_corners():
    r = rng(9)
    Hq, Hkv, nblk, D = 4, 2, 5, 6
    q = r.standard_normal((Hq, D))
    q[0, 2] = 0.0
    a, b = r.standard_normal((Hkv, nblk, D)), r.standard_normal((Hkv, nblk, D))
    kmin, kmax = np.minimum(a, b), np.maximum(a, b)
    s = O.block_scores(q, kmin, kmax)
    for h in range(Hq):
        hk = h // 2
        for i in range(nblk):
            best = -np.inf
            for corner in itertools.product([0, 1], repeat=D):
                k = np.where(np.asarray(corner) == 1, kmax[hk, i], kmin[hk, i])
                best = max(best, float(q[h] @ k))
            assert s[h, i] == pytest.approx(best, abs=1e-12)


def test_block_score_upper_bounds_token_scores_and_is_tight_for_singletons():
    r = rng(10)
    Hq, Hkv, L, D = 4, 2, 200, 16
    K = r.standard_normal((Hkv, L, D))
    q = r.standard_normal((Hq, D))
    bs = np.asarray([0, 1, 2, 30, 31, 90, 200])
    kmin, kmax = O.block_summaries(K, bs)
    s = O.block_scores(q, kmin, kmax)
    for h in range(Hq):
        tokscore = K[h // 2] @ q[h]
        for i in range(len(bs) - 1):
            seg = tokscore[bs[i]: bs[i + 1]]
            assert s[h, i] >= seg.max() - 1e-12
            if bs[i + 1] - bs[i] == 1:
                assert s[h, i] == pytest.approx(seg[0], abs=1e-12)
    # identity: one dot product of length 2D against (q+, q-)
    qp, qm = np.maximum(q, 0), np.minimum(q, 0)
    for h in range(Hq):
        np.testing.assert_allclose(s[h], kmax[h // 2] @ qp[h] + kmin[h // 2] @ qm[h], atol=1e-12)


# ---------------------------------------------------------------- slot top-k
def test_select_slots_b1_is_token_level_topk_transcription():
    # Sec. 4.2 block-to-token mapping: assign s_i to every token of B_i, top-k tokens.
    r = rng(11)
    L = 300
    cuts = np.sort(r.choice(np.arange(1, L), size=30, replace=False))
    bs = np.concatenate([[0], cuts, [L]])
    score = np.round(r.standard_normal(len(bs) - 1), 1)          # rounded -> real ties
    base = O.slot_map(bs, 1)
    for T in (1, 17, 64, 299, 300, 500):
        sel, tau = O.select_slots(score, base, T)
        tok_score = np.repeat(score, np.diff(bs))
        order = np.argsort(-tok_score, kind="stable")[: min(T, L)]
        np.testing.assert_array_equal(sel, np.sort(order))
        assert tau == tok_score[order[-1]]


def test_select_slots_general_b_and_budget_all():
    bs = np.asarray([0, 5, 6, 16, 20])          # lens 5,1,10,4 ; b=4 -> slots 2,1,3,1
    base = O.slot_map(bs, 4)
    assert list(base) == [0, 2, 3, 6, 7]
    score = np.asarray([1.0, 3.0, 2.0, 2.0])
    sel, tau = O.select_slots(score, base, 3)
    assert list(sel) == [2, 3, 4] and tau == 2.0   # block1's slot, then lowest slots of the 2.0 tie
    sel, tau = O.select_slots(score, base, 5)
    assert list(sel) == [2, 3, 4, 5, 6] and tau == 2.0
    sel, _ = O.select_slots(score, base, 7)
    assert list(sel) == list(range(7))
    sel, _ = O.select_slots(score, base, 100)
    assert list(sel) == list(range(7))
    toks = O.selected_tokens([0, 1, 6], bs, base, 4)
    assert list(toks) == [0, 1, 2, 3, 4, 16, 17, 18, 19]


# ---------------------------------------------------------------- selection shared by a KV group (extension)
def test_group_scores_defining_properties():
    r = rng(8100)
    Hkv, G, nblk = 3, 4, 37
    s = r.standard_normal((Hkv * G, nblk))
    g = O.group_block_scores(s, G)
    assert g.shape == (Hkv, nblk)
    for hk in range(Hkv):
        rows = s[hk * G:(hk + 1) * G]
        # an upper bound of every head of the group, attained by one of them, and by no head outside it
        assert (g[hk][None, :] >= rows).all()
        assert ((g[hk][None, :] == rows).sum(axis=0) >= 1).all()
        np.testing.assert_array_equal(g[hk], np.sort(rows, axis=0)[-1])
    # G = 1 changes nothing; identical heads in a group give that head's scores
    np.testing.assert_array_equal(O.group_block_scores(s, 1), s)
    same = np.repeat(r.standard_normal((Hkv, nblk)), G, axis=0)
    np.testing.assert_array_equal(O.group_block_scores(same, G), same[::G])


def test_group_selection_keeps_every_heads_favourite_and_reduces_to_per_head():
    r = rng(8101)
    G, nblk, b = 4, 50, 4
    bs = np.concatenate([[0], np.cumsum(r.integers(1, 10, size=nblk))])
    sb = O.slot_map(bs, b)
    s = r.standard_normal((G, nblk))
    g = O.group_block_scores(s, G)[0]
    for k in (1, 3, 17, int(sb[-1])):
        sel, tau = O.select_slots(g, sb, k)
        # a slot is taken iff fewer than k slots rank before it by (largest head score, slot index)
        slot_blk = np.searchsorted(sb, np.arange(sb[-1]), side="right") - 1
        best = s.max(axis=0)[slot_blk]
        for slot in range(int(sb[-1])):
            before = int(((best > best[slot]) | ((best == best[slot]) & (np.arange(sb[-1]) < slot))).sum())
            assert (slot in set(sel.tolist())) == (before < k)
    # the block any head likes best is selected as soon as k covers its slots and those of the better-liked ones
    top_blocks = {int(np.argmax(s[h])) for h in range(G)}
    sel, _ = O.select_slots(g, sb, int(sb[-1]) // 2)
    picked_blocks = set((np.searchsorted(sb, sel, side="right") - 1).tolist())
    assert top_blocks <= picked_blocks
    # one query head per group: the shared selection is the per-head selection
    np.testing.assert_array_equal(O.select_slots(O.group_block_scores(s[:1], 1)[0], sb, 9)[0],
                                  O.select_slots(s[0], sb, 9)[0])


# ---------------------------------------------------------------- mean pooling (App. A.2)
def test_block_means_and_their_scores():
    r = rng(40)
    H, L, D = 3, 97, 8
    X = r.standard_normal((H, L, D))
    bs = np.asarray([0, 1, 9, 10, 40, 41, 97])
    m = O.block_means(X, bs)
    for h in range(H):
        ref = np.add.reduceat(X[h], bs[:-1], axis=0) / np.diff(bs)[:, None]
        np.testing.assert_allclose(m[h], ref, rtol=0, atol=1e-14)
    np.testing.assert_array_equal(m[:, 0], X[:, 0])                     # one-token block: the token
    np.testing.assert_allclose(O.block_means(np.ones((1, 12, 4)) * 2.5, np.asarray([0, 5, 12])), 2.5)
    # scores: a plain dot product per (query head, block), GQA head h reads KV head h // G
    q = r.standard_normal((6, D))
    s = O.block_scores_mean(q, m)
    ref = np.einsum("hgd,hid->hgi", q.reshape(3, 2, D), m).reshape(6, -1)
    np.testing.assert_allclose(s, ref, atol=1e-13)
    # the (min,max) score of a degenerate box [m, m] is the same dot product: what lets a
    # mean summary stored in both rows go through the unchanged score path
    np.testing.assert_allclose(O.block_scores(q, m, m), s, atol=1e-13)
    # linearity pins the mean itself: q . mean(K_block) = mean_t (q . K_t)
    tok = np.einsum("hd,htd->ht", q[::2], X)                             # heads 0, 2, 4 -> KV heads 0, 1, 2
    for i in range(len(bs) - 1):
        np.testing.assert_allclose(s[::2, i], tok[:, bs[i]: bs[i + 1]].mean(axis=1), atol=1e-13)


# ---------------------------------------------------------------- incremental update
def _random_stream(r, L, n_class=4):
    isd = r.random(L) < r.choice([0.02, 0.1, 0.5])
    pos = np.nonzero(isd)[0]
    return pos, r.integers(0, n_class, size=len(pos))


@pytest.mark.parametrize("seed", range(8))
def test_append_equals_segmentation_from_scratch(seed):
    """Sec. 4.1, incremental update: keeping the final chunks and re-running the procedure from
    the first open one must give exactly the chunks of a run over the grown sequence."""
    r = rng(300 + seed)
    for _ in range(40):
        L = int(r.integers(1, 300))
        C = int(r.integers(1, 40))
        delta = int(r.integers(0, C))
        a_num = int(r.integers(0, 11))
        wq = r.integers(0, 11, size=4)
        pos, cls = _random_stream(r, L)
        full = O.dd_select(L, pos, cls, wq, C, delta, a_num, 10)
        L0 = int(r.integers(1, L + 1))
        m = pos < L0
        old = O.dd_select(L0, pos[m], cls[m], wq, C, delta, a_num, 10)
        new, i0 = O.dd_select_append(old, L, pos, cls, wq, C, delta, a_num, 10)
        np.testing.assert_array_equal(new, full)
        np.testing.assert_array_equal(new[:i0], old[:i0])          # kept chunks are untouched


def test_append_one_token_at_a_time_tracks_the_full_run():
    r = rng(321)
    L, C, delta = 260, 12, 5
    pos, cls = _random_stream(r, L)
    wq = r.integers(3, 11, size=4)
    cur = O.dd_select(1, pos[pos < 1], cls[pos < 1], wq, C, delta, 4, 10)
    recomputed = []
    for n in range(2, L + 1):
        m = pos < n
        cur, i0 = O.dd_select_append(cur, n, pos[m], cls[m], wq, C, delta, 4, 10)
        np.testing.assert_array_equal(cur, O.dd_select(n, pos[m], cls[m], wq, C, delta, 4, 10))
        recomputed.append(len(cur) - 1 - i0)
    # "only the most recent segmentation ranges are recomputed": the open chunks start within
    # C + delta of the end, and every chunk has at least C - delta tokens
    assert max(recomputed) <= (C + delta) // (C - delta) + 2


def test_first_open_block_by_hand():
    # C = 8, delta = 2: the chunk that starts at s was decided on boundaries up to s + 10
    assert O.first_open_block([0, 10, 20], 20, 8, 2) == 2        # 0+10 <= 20, 10+10 <= 20: all final
    assert O.first_open_block([0, 10, 19], 19, 8, 2) == 1        # 10+10 > 19: chunk 1 may still change
    assert O.first_open_block([0, 7], 7, 8, 2) == 0              # the only chunk is the open last one
    assert O.first_open_block([0, 9, 17, 26, 31], 31, 8, 2) == 3  # 10, 19, 27 <= 31 final; 26+10 = 36 > 31 open


# ---------------------------------------------------------------- KV reuse with V2F (App. B.2)
def _random_reuse_case(r, H, k, universe):
    """A resident table (distinct held slots, some empty) and an ascending selection per head."""
    resident, sel = [], []
    for _ in range(H):
        held = r.permutation(universe)[:k].tolist()
        for p in range(k):
            if r.random() < 0.15:
                held[p] = -1
        resident.append(held)
        n = int(r.integers(0, k + 1))
        sel.append(sorted(r.permutation(universe)[:n].tolist()))
    return resident, sel


def test_kv_reuse_handworked_fixture():
    with open(os.path.join(GOLDEN, "kv_reuse_handworked.json")) as f:
        cases = json.load(f)["cases"]
    assert len(cases) >= 5
    for c in cases:
        r, new_res, loads = O.kv_reuse_plan(c["resident"], c["sel"], c.get("stale_from"))
        assert r == c["r"], c["name"]
        assert new_res == c["new_resident"], c["name"]
        assert [[list(x) for x in plan] for plan in loads] == c["loads"], c["name"]


@pytest.mark.parametrize("seed", range(40))
def test_kv_reuse_plan_set_formulation_and_invariants(seed):
    r_ = rng(7000 + seed)
    H, k = int(r_.integers(1, 6)), int(r_.integers(1, 9))
    universe = int(r_.integers(k, 3 * k + 2))
    resident, sel = _random_reuse_case(r_, H, k, universe)
    stale = None if seed % 3 else int(r_.integers(0, universe + 1))
    r, new_res, loads = O.kv_reuse_plan(resident, sel, stale)
    # Step 1 through sets: reusable = held AND selected (AND not stale); r = the smallest such set
    overlap = []
    for h in range(H):
        held = {x for x in resident[h] if x >= 0 and (stale is None or x < stale)}
        overlap.append(held & set(sel[h]))
    assert r == min(len(o) for o in overlap)
    for h in range(H):
        row, plan = new_res[h], loads[h]
        kept_pos = [p for p in range(k) if p not in {q for q, _ in plan} and row[p] >= 0]
        # exactly r entries stay where they were, each of them reusable, and they are the first
        # r reusable ones in position order
        assert len(kept_pos) == r
        reusable_pos = [p for p in range(k) if resident[h][p] in overlap[h]]
        assert kept_pos == reusable_pos[:r]
        assert all(row[p] == resident[h][p] for p in kept_pos)
        # the buffer now holds exactly the selection, once each
        assert sorted(x for x in row if x >= 0) == list(sel[h])
        # every head loads (selected - r) slots: k - r when its selection is full
        assert len(plan) == len(sel[h]) - r
        if len(sel[h]) == k:
            assert len(plan) == k - r
        # loads: ascending slots into ascending positions, never onto a kept position
        assert [x for _, x in plan] == sorted(x for _, x in plan)
        assert [q for q, _ in plan] == sorted(q for q, _ in plan)
        free = [p for p in range(k) if p not in kept_pos]
        assert [q for q, _ in plan] == free[:len(plan)]
        assert all(row[q] == x for q, x in plan)


def test_kv_reuse_special_cases():
    # the same selection twice: everything is reused, nothing moves, nothing is loaded
    sel = [[1, 4, 6], [0, 2, 9]]
    r0, res0, loads0 = O.kv_reuse_plan([[-1] * 3, [-1] * 3], sel)
    assert r0 == 0 and res0 == sel and [len(p) for p in loads0] == [3, 3]
    r1, res1, loads1 = O.kv_reuse_plan(res0, sel)
    assert r1 == 3 and res1 == res0 and loads1 == [[], []]
    # disjoint selection: nothing reusable, the whole selection is loaded from position 0
    r2, res2, loads2 = O.kv_reuse_plan(res0, [[2, 3, 5], [1, 4, 7]])
    assert r2 == 0 and res2 == [[2, 3, 5], [1, 4, 7]]
    assert loads2 == [[(0, 2), (1, 3), (2, 5)], [(0, 1), (1, 4), (2, 7)]]
    # a single head is never truncated: r = |held AND selected|
    r3, res3, loads3 = O.kv_reuse_plan([[8, 3, 5, 1]], [[1, 2, 3, 4]])
    assert r3 == 2 and res3 == [[2, 3, 4, 1]] and loads3 == [[(0, 2), (2, 4)]]
    # one head without overlap drags every head to r = 0: all heads reload their selection
    r4, res4, loads4 = O.kv_reuse_plan([[1, 2], [3, 4]], [[1, 2], [5, 6]])
    assert r4 == 0 and loads4 == [[(0, 1), (1, 2)], [(0, 5), (1, 6)]]
    # stale_from = 0 disables reuse altogether; a bound above every slot changes nothing
    assert O.kv_reuse_plan(res0, sel, stale_from=0)[0] == 0
    assert O.kv_reuse_plan(res0, sel, stale_from=10) == (r1, res1, loads1)


def test_kv_reuse_sequence_of_steps_keeps_buffer_equal_to_selection_and_data_in_place():
    """Over many steps the buffers built by applying the loads hold, slot by slot, the K rows
    of the current selection -- so attention over the buffer is attention over the selection."""
    r_ = rng(7100)
    Hkv, G, k, b, D, nslots = 2, 2, 6, 4, 8, 20
    Hq = Hkv * G
    spans, start = {}, 0
    for g in range(nslots):
        ln = int(r_.integers(1, b + 1))
        spans[g] = (start, ln)
        start += ln
    X = r_.standard_normal((Hkv, start, D))
    buf = np.full((Hq, k * b, D), np.nan)
    resident = [[-1] * k for _ in range(Hq)]
    total_loaded = 0
    for step in range(12):
        sel = [sorted(r_.permutation(nslots)[:k].tolist()) for _ in range(Hq)]
        if step % 4 == 3:
            sel = [list(row) for row in prev_sel]          # a repeated query reuses everything
        r, resident, loads = O.kv_reuse_plan(resident, sel)
        O.kv_reuse_apply(buf, loads, X, spans, b, G)
        total_loaded += sum(len(p) for p in loads)
        if step % 4 == 3:
            assert r == k and all(len(p) == 0 for p in loads)
        for h in range(Hq):
            assert sorted(resident[h]) == sel[h]
            for p, slot in enumerate(resident[h]):
                st, ln = spans[slot]
                np.testing.assert_array_equal(buf[h, p * b:p * b + ln], X[h // G, st:st + ln])
                assert not buf[h, p * b + ln:(p + 1) * b].any()
        prev_sel = sel
    assert total_loaded < 12 * Hq * k


# ---------------------------------------------------------------- attention
def test_attention_budget_all_equals_dense_sdpa():
    r = rng(12)
    L, D = 257, 32
    q, K, V = r.standard_normal(D), r.standard_normal((L, D)), r.standard_normal((L, D))
    scale = 1.0 / math.sqrt(D)
    o, lse = O.sparse_attention(q, K, V, np.arange(L), scale)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None, None, None], torch.from_numpy(K)[None, None],
        torch.from_numpy(V)[None, None], scale=scale)[0, 0, 0].numpy()
    np.testing.assert_allclose(o, ref, atol=1e-12)
    assert lse == pytest.approx(float(torch.logsumexp(torch.from_numpy(K @ q) * scale, 0)), abs=1e-12)


def test_dense_attention_is_sdpa_and_its_closed_forms():
    r = rng(21)
    L, D = 193, 16
    q, K, V = r.standard_normal(D), r.standard_normal((L, D)), r.standard_normal((L, D))
    scale = 0.37
    o, lse = O.dense_attention(q, K, V, scale)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None, None, None], torch.from_numpy(K)[None, None],
        torch.from_numpy(V)[None, None], scale=scale)[0, 0, 0].numpy()
    np.testing.assert_allclose(o, ref, atol=1e-12)
    assert lse == pytest.approx(float(torch.logsumexp(torch.from_numpy(K @ q) * scale, 0)), abs=1e-12)
    # the sparse path with every token selected is the same function
    o2, lse2 = O.sparse_attention(q, K, V, np.arange(L), scale)
    np.testing.assert_allclose(o, o2, atol=1e-13)
    assert lse == pytest.approx(lse2, abs=1e-12)
    # one token: its V row; identical keys: the mean of V, lse = z + log L
    o, lse = O.dense_attention(q, K[:1], V[:1], scale)
    np.testing.assert_allclose(o, V[0], atol=1e-15)
    assert lse == pytest.approx(float(K[0] @ q) * scale)
    Kc = np.tile(K[3], (L, 1))
    o, lse = O.dense_attention(q, Kc, V, scale)
    np.testing.assert_allclose(o, V.mean(axis=0), atol=1e-13)
    assert lse == pytest.approx(float(K[3] @ q) * scale + math.log(L))
    # one key far ahead of the rest: the output is that token's V row
    Kp = K.copy()
    Kp[77] = 200.0 * q / (q @ q) / scale + 0.0        # logit 200 above a field of O(1) logits
    o, _ = O.dense_attention(q, Kp, V, scale)
    np.testing.assert_allclose(o, V[77], atol=1e-12)


def test_attention_special_cases():
    r = rng(13)
    L, D = 50, 8
    q, K, V = r.standard_normal(D), r.standard_normal((L, D)), r.standard_normal((L, D))
    # single token -> its V row, lse = its logit
    o, lse = O.sparse_attention(q, K, V, np.asarray([7]), 0.3)
    np.testing.assert_allclose(o, V[7], atol=1e-15)
    assert lse == pytest.approx(float(K[7] @ q) * 0.3)
    # order of the index set does not matter
    idx = np.asarray([3, 9, 11, 40, 41])
    o1, l1 = O.sparse_attention(q, K, V, idx, 0.3)
    o2, l2 = O.sparse_attention(q, K, V, idx[::-1].copy(), 0.3)
    np.testing.assert_allclose(o1, o2, atol=1e-14)
    assert l1 == pytest.approx(l2)
    # identical keys -> uniform weights -> mean of V rows, lse = z + log n
    Kc = np.tile(K[0], (L, 1))
    o, lse = O.sparse_attention(q, Kc, V, idx, 0.3)
    np.testing.assert_allclose(o, V[idx].mean(axis=0), atol=1e-14)
    assert lse == pytest.approx(float(K[0] @ q) * 0.3 + math.log(len(idx)))
    # subset attention = dense attention on the gathered rows (library softmax)
    z = torch.from_numpy(K[idx] @ q * 0.3)
    ref = (torch.softmax(z, 0)[:, None] * torch.from_numpy(V[idx])).sum(0).numpy()
    np.testing.assert_allclose(o1, ref, atol=1e-14)


# ---------------------------------------------------------------- end to end
def test_pipeline_with_fixed_chunks_is_fixed_page_topk_attention():
    """No delimiters and b dividing C: the whole path must collapse to the fixed-page
    scheme of Sec. 2.1 (pages of C tokens, page score = max attainable q.k from
    per-channel min/max, top pages, attention over their tokens), written here
    independently with array ops."""
    r = rng(14)
    L, D, C, b, T = 512, 16, 32, 16, 128
    Kb = f32_to_bf16_bits(r.standard_normal((1, L, D)).astype(np.float32))
    Vb = f32_to_bf16_bits(r.standard_normal((1, L, D)).astype(np.float32))
    qb = f32_to_bf16_bits(r.standard_normal((1, D)).astype(np.float32))
    K, V, q = O.widen_bf16(Kb), O.widen_bf16(Vb), O.widen_bf16(qb)
    scale = 1 / math.sqrt(D)
    bs = O.dd_select(L, [], [], [5], C, C // 2, 5, 10)
    base = O.slot_map(bs, b)
    kmin, kmax = O.block_summaries(K, bs)
    sc = O.block_scores(q, kmin, kmax)
    sel, _ = O.select_slots(sc[0], base, T // b)
    toks = O.selected_tokens(sel, bs, base, b)
    o, _ = O.sparse_attention(q[0], K[0], V[0], toks, scale)
    # independent fixed-page reference
    pages = K[0].reshape(L // C, C, D)
    pscore = np.maximum(q[0] * pages.max(1), q[0] * pages.min(1)).sum(-1)
    n_pages = T // C
    top = np.sort(np.argsort(-pscore, kind="stable")[:n_pages])
    ptoks = (top[:, None] * C + np.arange(C)[None, :]).ravel()
    np.testing.assert_array_equal(toks, ptoks)
    z = K[0][ptoks] @ q[0] * scale
    p = np.exp(z - z.max())
    np.testing.assert_allclose(o, (p[:, None] * V[0][ptoks]).sum(0) / p.sum(), atol=1e-13)
