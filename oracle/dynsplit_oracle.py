"""fp64 CPU oracle for the DynSplit-KV hot path.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain statement of what the path computes, written from
the paper's definitions; it shares no code with the HIP library and is imported
only by tests, the smoke check and the bench's CPU-baseline leg.  Every
function works on one sequence (ragged batches are loops in the caller) and on
float64 arrays obtained by widening bf16 bit patterns exactly.

Parity status against the authors' implementation (none is public):
  * class_weights   -- "parity unpinned": the paper gives no score->weight map.
  * dd_select       -- pinned to the declarative rule by brute force and to
                       closed forms; the proximity term p_e, the empty-window
                       fallback and Delta are readings ("parity unpinned" vs
                       the authors' choice of those).
  * block_scores    -- pinned as the exact maximum of q.k over the block's
                       bounding box; whether the authors use this form of the
                       "query-compressed vector product" is unpinned.
  * dd_select_append -- pinned to dd_select run from scratch on the grown
                       sequence (every split point of random streams); the
                       paper only says that the most recent ranges are
                       recomputed, the finality rule is derived from dd_select.
  * block_means / block_scores_mean -- the mean and the dot product are
                       textbook; that the authors score a mean summary with
                       q.mean is a reading ("parity unpinned").
  * group_block_scores -- the extension "one selection per KV group" (maximum over the
                       group's query heads) is NOT in the paper; pinned to its
                       defining properties only ("parity unpinned").
  * kv_reuse_plan   -- pinned to a set formulation (Python sets, brute force),
                       to invariants and to hand-worked cases; which reusable
                       entries the truncation drops, the order of the loads and
                       "minimum over the heads of one sequence" are readings
                       ("parity unpinned" vs the authors' choice of those).
Everything else (dense_attention included) reduces to a textbook definition and
is pinned to it in tests/test_oracle_pins.py; tests/test_oracle_mutations.py
checks that planted mistakes in any of these functions are rejected by a pin.
"""
from __future__ import annotations

import math
from typing import List, Sequence, Tuple

import numpy as np


# ----------------------------------------------------------------------------
# input widening
# ----------------------------------------------------------------------------
def widen_bf16(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> the float64 values they denote (exact)."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


# ----------------------------------------------------------------------------
# Candidate delimiter positions (input D of Alg. 1; boundary tokens B of Sec. 4.1)
# ----------------------------------------------------------------------------
def extract_candidates(token_ids: np.ndarray, delim_ids: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Positions t (ascending) whose token is a boundary token, and the index of
    that token in `delim_ids` (its delimiter class)."""
    pos: List[int] = []
    cls: List[int] = []
    index_of = {int(d): c for c, d in enumerate(delim_ids)}
    for t, tok in enumerate(token_ids):
        c = index_of.get(int(tok))
        if c is not None:
            pos.append(t)
            cls.append(c)
    return np.asarray(pos, dtype=np.int64), np.asarray(cls, dtype=np.int64)


def sample_candidates(cand_pos: np.ndarray, cand_class: np.ndarray, n_class: int, M: int,
                      R: int, W: int, L: int) -> np.ndarray:
    """"A few tokens" per delimiter class (Sec. 3, stability remark): the first M
    occurrences of each class, in position order, among candidates with
    R <= t <= L-1-W (full retained region behind, full future window ahead).
    Returns samp_pos[n_class, M], -1 where a class has fewer occurrences."""
    samp = np.full((n_class, M), -1, dtype=np.int64)
    seen = [0] * n_class
    for t, c in zip(cand_pos, cand_class):
        t = int(t)
        c = int(c)
        if t < R or t > L - 1 - W:
            continue
        if seen[c] < M:
            samp[c, seen[c]] = t
            seen[c] += 1
    return samp


# ----------------------------------------------------------------------------
# Alg. 1 / Sec. 3 equation: delimiter importance via attention dependency
# ----------------------------------------------------------------------------
def delimiter_importance(qwin: np.ndarray, K: np.ndarray, t: int, R: int, alpha_imp: float,
                         scale: float) -> float:
    """Importance s_t of the candidate at position t on one layer.

    qwin[w, h, :] is the query of head h at position t+1+w (w = 0..W-1, the
    future window F_t); K[hk, k, :] are the keys of the sequence; head h reads
    KV head h // G.  For every (h, q in F_t) the causal attention row
    A_{q,k} = softmax_k(q.K_k * scale), k = 0..q, is split into the retained
    region O_t = {max(0,t-R+1)..t} and the discarded region D_t = {0..max(0,t-R)};
    s_t is the mean over heads and window queries of (sum_O A - alpha * sum_D A)."""
    W, Hq, D = qwin.shape
    Hkv = K.shape[0]
    G = Hq // Hkv
    o_lo, o_hi = max(0, t - R + 1), t            # inclusive
    d_lo, d_hi = 0, max(0, t - R)                # inclusive
    acc = 0.0
    for h in range(Hq):
        Kh = K[h // G]
        for w in range(W):
            qpos = t + 1 + w
            z = (Kh[: qpos + 1] @ qwin[w, h]) * scale
            z = z - z.max()
            e = np.exp(z)
            A = e / e.sum()
            acc += float(A[o_lo: o_hi + 1].sum()) - alpha_imp * float(A[d_lo: d_hi + 1].sum())
    return acc / (Hq * W)


def delimiter_importance_layers(qwins: Sequence[np.ndarray], Ks: Sequence[np.ndarray], t: int, R: int,
                                alpha_imp: float, scale: float) -> float:
    """Importance s_t with the expectation of Alg. 1 taken over several layers as well: layer l
    has its own queries qwins[l] and keys Ks[l]; every (layer, head, window query) row weighs the
    same, so with equally many heads per layer the result is the mean of the layers' values."""
    n_rows = 0
    acc = 0.0
    for qwin, K in zip(qwins, Ks):
        W, Hq, _ = qwin.shape
        acc += delimiter_importance(qwin, K, t, R, alpha_imp, scale) * (Hq * W)
        n_rows += Hq * W
    return acc / n_rows


def class_weights(s: np.ndarray, samp_pos: np.ndarray, alpha_imp: float,
                  prior_wq: np.ndarray) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Per-class weight in tenths from the sampled importance scores (Sec. 4.1:
    w in [0,1]; App. B.1 prints weights in steps of 0.1).

    s[c, m] is the score of sample samp_pos[c, m] (ignored where samp_pos < 0).
    Class mean -> affine map of the attainable range [-alpha, 1] onto [0, 1]
    (monotone, keeps the ordering) -> clamp -> round half up to tenths.
    A class with no sample keeps prior_wq[c].
    Returns (wq[n_class] int, mean[n_class] with NaN for empty classes,
    edge_dist[n_class] = distance of 10*w to the nearest rounding edge)."""
    n_class = s.shape[0]
    wq = np.asarray(prior_wq, dtype=np.int64).copy()
    mean = np.full(n_class, np.nan)
    edge = np.full(n_class, np.inf)
    for c in range(n_class):
        vals = [float(s[c, m]) for m in range(s.shape[1]) if samp_pos[c, m] >= 0]
        if not vals:
            continue
        mean[c] = sum(vals) / len(vals)
        w = (mean[c] + alpha_imp) / (1.0 + alpha_imp)
        w = min(1.0, max(0.0, w))
        x = 10.0 * w
        wq[c] = int(math.floor(x + 0.5))
        edge[c] = abs((x + 0.5) - round(x + 0.5))
    return wq, mean, edge


# ----------------------------------------------------------------------------
# DD-Select (Sec. 4.1, Dynamic Segmentation Procedure)
# ----------------------------------------------------------------------------
def boundary_score(e: int, s_e: int, wq_e: int, delta: int, a_num: int, a_den: int) -> int:
    """10 * a_den * max(delta,1) times  alpha*w_e + (1-alpha)*p_e  with
    alpha = a_num/a_den, w_e = wq_e/10 and p_e = 1 - |e - s_e| / max(delta,1)
    (linear proximity: 1 at the ideal end, 0 at the edge of the search range).
    All operands are small integers, so the value is exact."""
    dd = max(delta, 1)
    return a_num * wq_e * dd + (a_den - a_num) * 10 * (dd - abs(e - s_e))


def dd_select(L: int, cand_pos: Sequence[int], cand_class: Sequence[int], wq: Sequence[int],
              C: int, delta: int, a_num: int, a_den: int) -> np.ndarray:
    """Chunk boundaries block_start[0..nblk] (block_start[0]=0, block_start[nblk]=L).

    A boundary token at position t closes its chunk: it offers the boundary
    e = t+1.  From the current position s_c: the ideal end is s_e = s_c + C; if
    s_e >= L the last chunk ends at L; otherwise among the offered boundaries in
    [s_e-delta, s_e+delta] (clipped to L) the best-scored one is taken, ties to
    the smallest e; with none in range the chunk ends at s_e.  Requires
    C >= 1 and 0 <= delta < C, which makes every chunk non-empty."""
    assert C >= 1 and 0 <= delta < C and 0 <= a_num <= a_den and a_den > 0
    wq_at = {int(t) + 1: int(wq[int(c)]) for t, c in zip(cand_pos, cand_class)}
    starts = [0]
    s_c = 0
    while s_c < L:
        s_e = s_c + C
        if s_e >= L:
            e_star = L
        else:
            lo, hi = s_e - delta, min(L, s_e + delta)
            best_e, best_score = None, None
            for e in range(lo, hi + 1):
                if e in wq_at:
                    sc = boundary_score(e, s_e, wq_at[e], delta, a_num, a_den)
                    if best_score is None or sc > best_score:
                        best_e, best_score = e, sc
            e_star = s_e if best_e is None else best_e
        starts.append(e_star)
        s_c = e_star
    return np.asarray(starts, dtype=np.int64)


# ----------------------------------------------------------------------------
# V2F (Sec. 4.2): fixed-length slots, min/max summaries, scores, top-k
# ----------------------------------------------------------------------------
def slot_map(block_start: np.ndarray, b: int) -> np.ndarray:
    """slot_base[0..nblk]: block i owns the ceil(len_i / b) consecutive slots
    slot_base[i] .. slot_base[i+1]-1; slot j of block i covers tokens
    [s_i + j*b, min(s_i + (j+1)*b, e_i)).  b = 1 is the paper's token-level
    block-to-token mapping."""
    base = [0]
    for i in range(len(block_start) - 1):
        ln = int(block_start[i + 1]) - int(block_start[i])
        base.append(base[-1] + (ln + b - 1) // b)
    return np.asarray(base, dtype=np.int64)


def slot_span(g: int, block_start: np.ndarray, slot_base: np.ndarray, b: int) -> Tuple[int, int, int]:
    """(block index, first token, token count) of slot g."""
    i = int(np.searchsorted(slot_base, g, side="right")) - 1
    start = int(block_start[i]) + (g - int(slot_base[i])) * b
    ln = min(b, int(block_start[i + 1]) - start)
    return i, start, ln


def block_summaries(X: np.ndarray, block_start: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Element-wise minimum and maximum over the tokens of every block
    (Sec. 4.2, KVCache Compression).  X[h, t, d] -> (xmin, xmax)[h, i, d]."""
    H, _, D = X.shape
    nblk = len(block_start) - 1
    xmin = np.empty((H, nblk, D), dtype=np.float64)
    xmax = np.empty((H, nblk, D), dtype=np.float64)
    for h in range(H):
        for i in range(nblk):
            seg = X[h, int(block_start[i]): int(block_start[i + 1])]
            xmin[h, i] = seg.min(axis=0)
            xmax[h, i] = seg.max(axis=0)
    return xmin, xmax


def block_scores(q: np.ndarray, kmin: np.ndarray, kmax: np.ndarray) -> np.ndarray:
    """score[hq, i] = sum_d max(q_d * kmax[hk,i,d], q_d * kmin[hk,i,d]), hk = hq // G:
    the largest value q.k can take over the block's per-channel bounding box
    (Sec. 4.2, Top-k Block Selection, for a (min,max) summary; the fixed-page
    scheme of Sec. 2.1 "approximating the maximum attention score")."""
    Hq = q.shape[0]
    Hkv, nblk, _ = kmin.shape
    G = Hq // Hkv
    s = np.empty((Hq, nblk), dtype=np.float64)
    for h in range(Hq):
        hk = h // G
        s[h] = np.maximum(q[h][None, :] * kmax[hk], q[h][None, :] * kmin[hk]).sum(axis=1)
    return s


def select_slots(score: np.ndarray, slot_base: np.ndarray, k: int) -> Tuple[np.ndarray, float]:
    """Top-k over block scores mapped onto slots (Sec. 4.2, Block-to-Token
    Mapping; App. B.2 Step 1): every slot inherits the score of its block; slots
    are ranked by (score descending, slot index ascending) and the first
    min(k, N_slots) are taken.  Returns (selected slot indices ascending,
    score tau of the last-ranked selected slot; nan if nothing selected)."""
    n_slots = int(slot_base[-1])
    slot_score = np.empty(n_slots, dtype=np.float64)
    for i in range(len(slot_base) - 1):
        slot_score[int(slot_base[i]): int(slot_base[i + 1])] = score[i]
    order = sorted(range(n_slots), key=lambda g: (-slot_score[g], g))
    take = order[: min(k, n_slots)]
    tau = float(slot_score[take[-1]]) if take else float("nan")
    return np.asarray(sorted(take), dtype=np.int64), tau


def group_block_scores(score: np.ndarray, G: int) -> np.ndarray:
    """Selection shared by the query heads of a KV group -- an extension, NOT in the paper (which
    selects per head and is silent on grouped-query models): the group's score of a block is the
    largest score any of its G query heads gives it, so a block that matters to one head of the
    group is kept for all of them and the group gathers one slot set.  score[hq, i] -> [Hq//G, i]."""
    Hq, nblk = score.shape
    out = np.empty((Hq // G, nblk), dtype=np.float64)
    for hk in range(Hq // G):
        for i in range(nblk):
            best = score[hk * G, i]
            for g in range(1, G):
                if score[hk * G + g, i] > best:
                    best = score[hk * G + g, i]
            out[hk, i] = best
    return out


def selected_tokens(sel_slots: Sequence[int], block_start: np.ndarray, slot_base: np.ndarray,
                    b: int) -> np.ndarray:
    """Token positions covered by the selected slots, ascending."""
    toks: List[int] = []
    for g in sel_slots:
        _, start, ln = slot_span(int(g), block_start, slot_base, b)
        toks.extend(range(start, start + ln))
    return np.asarray(toks, dtype=np.int64)


# ----------------------------------------------------------------------------
# Attention over the selected tokens (App. B.2 Steps 2-3)
# ----------------------------------------------------------------------------
def sparse_attention(q: np.ndarray, K: np.ndarray, V: np.ndarray, tokens: np.ndarray,
                     scale: float) -> Tuple[np.ndarray, float]:
    """One head: o = softmax_{t in tokens}(q.K_t * scale) . V_t and
    lse = log sum_t exp(q.K_t * scale).  q[D], K[L,D], V[L,D]."""
    z = (K[tokens] @ q) * scale
    m = z.max()
    p = np.exp(z - m)
    den = p.sum()
    o = (p[:, None] * V[tokens]).sum(axis=0) / den
    return o, float(m + math.log(den))


# ----------------------------------------------------------------------------
# Full attention over the whole cache (the full-KV baseline of Sec. 5, GPU
# Inference analysis, Figure 8) -- the definition, written out
# ----------------------------------------------------------------------------
def dense_attention(q: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float) -> Tuple[np.ndarray, float]:
    """One head, one decode query: A_t = exp(q.K_t * scale) / sum_u exp(q.K_u * scale) over
    every token t of the sequence, o = sum_t A_t V_t, lse = log sum_t exp(q.K_t * scale).
    q[D], K[L,D], V[L,D]; L >= 1."""
    L = K.shape[0]
    z = np.empty(L, dtype=np.float64)
    for t in range(L):
        z[t] = float(np.dot(q, K[t])) * scale
    zmax = float(z.max())
    w = np.exp(z - zmax)
    den = float(w.sum())
    o = np.zeros(V.shape[1], dtype=np.float64)
    for t in range(L):
        o += (w[t] / den) * V[t]
    return o, zmax + math.log(den)


# ----------------------------------------------------------------------------
# Incremental update during decoding (Sec. 4.1): chunks already computed are
# kept; only the most recent segmentation ranges are recomputed
# ----------------------------------------------------------------------------
def first_open_block(block_start: Sequence[int], L_old: int, C: int, delta: int) -> int:
    """Index of the first chunk whose end was decided without seeing its whole search range.

    The end of the chunk that starts at s is chosen among boundaries up to s + C + delta; with
    only L_old tokens present that choice is final exactly when s + C + delta <= L_old.  Chunk
    starts ascend, so every chunk before the returned index is final, and -- the procedure
    running left to right -- stays as it is however many tokens follow."""
    nblk = len(block_start) - 1
    for i in range(nblk):
        if int(block_start[i]) + C + delta > L_old:
            return i
    return nblk


def dd_select_append(block_start_old: Sequence[int], L_new: int, cand_pos: Sequence[int],
                     cand_class: Sequence[int], wq: Sequence[int], C: int, delta: int, a_num: int,
                     a_den: int) -> Tuple[np.ndarray, int]:
    """Chunk boundaries of the sequence grown to L_new tokens, from the boundaries computed
    when it had L_old = block_start_old[-1] tokens: the final chunks are kept, the procedure of
    Sec. 4.1 is re-run from the start of the first open chunk.  cand_pos / cand_class describe
    the grown sequence.  Returns (block_start_new, index of the first recomputed chunk)."""
    L_old = int(block_start_old[-1])
    assert L_new >= L_old
    i0 = first_open_block(block_start_old, L_old, C, delta)
    s0 = int(block_start_old[i0]) if i0 < len(block_start_old) - 1 else L_old
    keep = [int(x) for x in block_start_old[:i0]]
    # the tail is an ordinary DD-Select run on the suffix that starts at s0
    tail_pos = [int(t) - s0 for t in cand_pos if int(t) >= s0]
    tail_cls = [int(c) for t, c in zip(cand_pos, cand_class) if int(t) >= s0]
    tail = dd_select(L_new - s0, tail_pos, tail_cls, wq, C, delta, a_num, a_den)
    return np.asarray(keep + [int(x) + s0 for x in tail], dtype=np.int64), i0


# ----------------------------------------------------------------------------
# Mean-pooling summaries (App. A.2, additional ablation: min/max compression
# replaced by mean pooling, everything else unchanged)
# ----------------------------------------------------------------------------
def block_means(X: np.ndarray, block_start: np.ndarray) -> np.ndarray:
    """Per-channel arithmetic mean over the tokens of every block.  X[h, t, d] -> mean[h, i, d]."""
    H, _, D = X.shape
    nblk = len(block_start) - 1
    out = np.empty((H, nblk, D), dtype=np.float64)
    for h in range(H):
        for i in range(nblk):
            s, e = int(block_start[i]), int(block_start[i + 1])
            acc = np.zeros(D, dtype=np.float64)
            for t in range(s, e):
                acc += X[h, t]
            out[h, i] = acc / (e - s)
    return out


def block_scores_mean(q: np.ndarray, kmean: np.ndarray) -> np.ndarray:
    """score[hq, i] = q[hq] . kmean[hk, i], hk = hq // G: the query-compressed-vector product
    (Sec. 4.2) when the compressed vector is the block's mean key."""
    Hq = q.shape[0]
    Hkv, nblk, _ = kmean.shape
    G = Hq // Hkv
    s = np.empty((Hq, nblk), dtype=np.float64)
    for h in range(Hq):
        for i in range(nblk):
            s[h, i] = float(np.dot(q[h], kmean[h // G, i]))
    return s


# ----------------------------------------------------------------------------
# KV reuse with V2F (App. B.2, "KVCache Reuse with V2F"): a per-head resident
# buffer of k fixed-size slots is updated from one decode step to the next
# ----------------------------------------------------------------------------
def kv_reuse_plan(resident: Sequence[Sequence[int]], sel: Sequence[Sequence[int]],
                  stale_from: int | None = None) -> Tuple[int, List[List[int]], List[List[Tuple[int, int]]]]:
    """One sequence.  resident[h][p] is the slot held at position p of head h's buffer (-1 =
    empty; held slots are distinct), sel[h] the slots selected for this step (ascending, at most
    k = len(resident[h])).  A held slot whose index is >= stale_from no longer matches the cache
    (its chunk was re-segmented) and cannot be reused.

    Step 1: head by head, the reusable entries are the held slots that are selected again; all
            heads are cut to the smallest reusable count r, keeping each head's first r reusable
            entries in position order.
    Step 2: what a head must load is every selected slot it does not keep -- the new ones and
            the reusable ones cut in Step 1 -- so that every head with a full selection loads
            k - r slots.
    Step 3: the loads go, in selection order, into the positions that are not kept, in position
            order; positions left over are empty.

    Returns (r, new resident table, per head the list of (position, slot) loads)."""
    H = len(resident)
    k = len(resident[0]) if H else 0
    reusable: List[List[int]] = []
    for h in range(H):
        chosen = set(int(x) for x in sel[h])
        pos = []
        for p in range(k):
            x = int(resident[h][p])
            if x >= 0 and x in chosen and (stale_from is None or x < stale_from):
                pos.append(p)
        reusable.append(pos)
    r = min((len(pos) for pos in reusable), default=0)
    new_resident: List[List[int]] = []
    loads: List[List[Tuple[int, int]]] = []
    for h in range(H):
        keep = reusable[h][:r]
        kept_slots = set(int(resident[h][p]) for p in keep)
        need = [int(x) for x in sel[h] if int(x) not in kept_slots]
        free = [p for p in range(k) if p not in set(keep)]
        row = [-1] * k
        for p in keep:
            row[p] = int(resident[h][p])
        plan = []
        for i, x in enumerate(need):
            row[free[i]] = x
            plan.append((free[i], x))
        new_resident.append(row)
        loads.append(plan)
    return r, new_resident, loads


def kv_reuse_apply(buf: np.ndarray, loads: Sequence[Sequence[Tuple[int, int]]], X: np.ndarray,
                   spans: dict, b: int, G: int) -> None:
    """Carries out the loads of kv_reuse_plan on head-major resident buffers: buf[h, p*b + j] =
    X[h // G, start + j] for j < len, zero for len <= j < b, where (start, len) = spans[slot].
    X is K or V as [Hkv, T, D]; buf is [Hq, k*b, D] and is modified in place."""
    for h, plan in enumerate(loads):
        for p, slot in plan:
            start, ln = spans[slot]
            buf[h, p * b:(p + 1) * b] = 0
            buf[h, p * b:p * b + ln] = X[h // G, start:start + ln]
