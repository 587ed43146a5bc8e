"""GPU parity of the delimiter-importance stage of dsk_compress (Alg. 1 on one layer, sampled
candidates, class weights in tenths) against the fp64 oracle."""
import math

import numpy as np
import pytest
import torch

from oracle import dynsplit_oracle as O
from workloads import make_workload
from dsk_testutil import dev_bf16, dev_i32, dev_u8

pytestmark = pytest.mark.gpu

SCORE_TOL = 2e-5      # fp32 MFMA accumulation + fp32 softmax vs fp64
EDGE_TOL = 1e-3       # a weight may differ by one tenth only this close to a rounding edge


def _run(cfg_id, **ov):
    import paper_2602_03184_amd as dsk
    wl = make_workload(cfg_id, with_kv=True, with_qwin=True, **ov)
    cfg = wl.cfg
    K = dev_bf16(wl.K)
    prior = np.full((cfg.B, cfg.n_class), 3, np.uint8)
    comp = dsk.compress(
        cu_seqlens=dev_i32(wl.cu_seqlens), max_seqlen=int(wl.seqlens.max()), Hq=cfg.Hq, K=K, V=None,
        stages=dsk.DSK_STAGE_CANDIDATES | dsk.DSK_STAGE_IMPORTANCE,
        token_ids=dev_i32(wl.token_ids), delim_ids=dev_i32(wl.delim_ids), n_class=cfg.n_class,
        M=cfg.M, W=cfg.W, R=cfg.R, alpha_imp=cfg.alpha_imp, qwin=dev_bf16(wl.qwin), class_weight_q=dev_u8(prior))
    torch.cuda.synchronize()
    assert int(comp.dev_status.item()) == 0
    return wl, comp, prior


def _check(wl, comp, prior, seqs=None):
    cfg = wl.cfg
    samp = comp.samp_pos.cpu().numpy()
    score = comp.samp_score.cpu().numpy()
    mean = comp.class_mean.cpu().numpy()
    wq = comp.class_weight_q.cpu().numpy()
    scale = 1.0 / math.sqrt(128.0)
    worst = 0.0
    for s in (range(cfg.B) if seqs is None else seqs):
        lo, hi = int(wl.cu_seqlens[s]), int(wl.cu_seqlens[s + 1])
        Kf = O.widen_bf16(wl.K[:, lo:hi])
        pos, cls = O.extract_candidates(wl.token_ids[lo:hi], wl.delim_ids)
        want_samp = O.sample_candidates(pos, cls, cfg.n_class, cfg.M, cfg.R, cfg.W, hi - lo)
        np.testing.assert_array_equal(samp[s], np.where(want_samp >= 0, want_samp + lo, -1))
        s_or = np.zeros((cfg.n_class, cfg.M))
        for c in range(cfg.n_class):
            for m in range(cfg.M):
                t = int(want_samp[c, m])
                if t < 0:
                    assert math.isnan(score[s, c, m])
                    continue
                qw = O.widen_bf16(wl.qwin[s, c * cfg.M + m])          # [W, Hq, D]
                s_or[c, m] = O.delimiter_importance(qw, Kf, t, cfg.R, cfg.alpha_imp, scale)
                err = abs(float(score[s, c, m]) - s_or[c, m])
                worst = max(worst, err)
                assert err <= SCORE_TOL, (s, c, m, t, float(score[s, c, m]), s_or[c, m])
        wq_or, mean_or, edge = O.class_weights(s_or, want_samp, cfg.alpha_imp, prior[s])
        for c in range(cfg.n_class):
            if math.isnan(mean_or[c]):
                assert math.isnan(mean[s, c]) and wq[s, c] == prior[s, c]
                continue
            assert abs(float(mean[s, c]) - mean_or[c]) <= SCORE_TOL
            if edge[c] > EDGE_TOL:
                assert int(wq[s, c]) == int(wq_or[c]), (s, c, mean_or[c])
            else:
                assert abs(int(wq[s, c]) - int(wq_or[c])) <= 1
    return worst


def test_importance_single_head_small():
    wl, comp, prior = _run(1)
    print("cfg1 worst |s_gpu - s_oracle| = %.2e" % _check(wl, comp, prior))


def test_importance_gqa4_llama_shape():
    wl, comp, prior = _run(2, seqlens=[12288])
    print("cfg2 worst = %.2e" % _check(wl, comp, prior))


def test_importance_gqa8_two_row_tiles_and_odd_window():
    wl, comp, prior = _run(2, seqlens=[6000], Hkv=4, W=5, R=100, M=3, alpha_imp=0.5)
    print("G=8 worst = %.2e" % _check(wl, comp, prior))


def test_importance_mha_ragged_batch():
    wl, comp, prior = _run(5, B=3, seqlens=[3000, 150, 5000], Hq=6, Hkv=6, M=4)
    print("MHA ragged worst = %.2e" % _check(wl, comp, prior))


def test_importance_feeds_segmentation_in_one_call():
    """All four stages in one dsk_compress call: weights estimated on the GPU drive DD-Select."""
    import paper_2602_03184_amd as dsk
    wl = make_workload(2, with_kv=True, with_qwin=True, seqlens=[8192])
    cfg = wl.cfg
    prior = np.full((1, cfg.n_class), 3, np.uint8)
    comp = dsk.compress(
        cu_seqlens=dev_i32(wl.cu_seqlens), max_seqlen=8192, Hq=cfg.Hq, K=dev_bf16(wl.K), V=None,
        stages=dsk.DSK_STAGE_ALL, token_ids=dev_i32(wl.token_ids), delim_ids=dev_i32(wl.delim_ids),
        n_class=cfg.n_class, M=cfg.M, W=cfg.W, R=cfg.R, alpha_imp=cfg.alpha_imp, qwin=dev_bf16(wl.qwin),
        class_weight_q=dev_u8(prior), C_=30, delta=15, alpha_num=5, alpha_den=10, b=16)
    torch.cuda.synchronize()
    assert int(comp.dev_status.item()) == 0
    wq = comp.class_weight_q.cpu().numpy()[0]
    pos, cls = O.extract_candidates(wl.token_ids, wl.delim_ids)
    bs = O.dd_select(8192, pos, cls, wq, 30, 15, 5, 10)     # oracle segmentation with the GPU's weights
    nb = len(bs) - 1
    assert int(comp.cu_blocks.cpu()[1]) == nb
    np.testing.assert_array_equal(comp.block_start.cpu().numpy()[: nb + 1], bs)


def test_importance_mean_over_layers():
    """Three layers (their own keys and window queries) through stage IMPORTANCE with the running
    sum: after the last call the class means and weights are those of the oracle's expectation
    over (layer, head, query); the per-layer scores of each call are still reported."""
    import paper_2602_03184_amd as dsk
    layers = [make_workload(2, with_kv=True, with_qwin=True, seqlens=[7000], M=4) for _ in range(1)]
    wl = layers[0]
    cfg = wl.cfg
    # further layers: same tokens (the positions are a property of the text), other keys and queries
    r = np.random.default_rng(77)
    from workloads import f32_to_bf16_bits
    Ks = [wl.K, wl.V, f32_to_bf16_bits(r.standard_normal(wl.K.shape, dtype=np.float32))]
    qwins = [wl.qwin, f32_to_bf16_bits(r.standard_normal(wl.qwin.shape, dtype=np.float32)),
             f32_to_bf16_bits(r.standard_normal(wl.qwin.shape, dtype=np.float32))]
    prior = np.full((1, cfg.n_class), 3, np.uint8)
    wq_dev = dev_u8(prior)
    acc = torch.zeros(1, cfg.n_class, cfg.M, dtype=torch.float32, device="cuda")
    comp = None
    per_layer = []
    for l in range(3):
        comp = dsk.compress(
            cu_seqlens=dev_i32(wl.cu_seqlens), max_seqlen=7000, Hq=cfg.Hq, K=dev_bf16(Ks[l]), V=None,
            stages=dsk.DSK_STAGE_CANDIDATES | dsk.DSK_STAGE_IMPORTANCE,
            token_ids=dev_i32(wl.token_ids), delim_ids=dev_i32(wl.delim_ids), n_class=cfg.n_class,
            M=cfg.M, W=cfg.W, R=cfg.R, alpha_imp=cfg.alpha_imp, qwin=dev_bf16(qwins[l]), class_weight_q=wq_dev,
            samp_score_sum=acc, imp_layers=l + 1)
        torch.cuda.synchronize()
        per_layer.append(comp.samp_score.cpu().numpy()[0].copy())
    samp = comp.samp_pos.cpu().numpy()[0]
    scale = 1.0 / math.sqrt(128.0)
    Kf = [O.widen_bf16(k) for k in Ks]
    s_or = np.zeros((cfg.n_class, cfg.M))
    for c in range(cfg.n_class):
        for m in range(cfg.M):
            t = int(samp[c, m])
            if t < 0:
                continue
            qs = [O.widen_bf16(qw[0, c * cfg.M + m]) for qw in qwins]
            s_or[c, m] = O.delimiter_importance_layers(qs, Kf, t, cfg.R, cfg.alpha_imp, scale)
            for l in range(3):           # each call still reports its own layer
                one = O.delimiter_importance(qs[l], Kf[l], t, cfg.R, cfg.alpha_imp, scale)
                assert abs(float(per_layer[l][c, m]) - one) <= SCORE_TOL
            assert abs(float(acc[0, c, m]) / 3.0 - s_or[c, m]) <= SCORE_TOL
    wq_or, mean_or, edge = O.class_weights(s_or, samp, cfg.alpha_imp, prior[0])
    mean = comp.class_mean.cpu().numpy()[0]
    wq = wq_dev.cpu().numpy()[0]
    for c in range(cfg.n_class):
        if math.isnan(mean_or[c]):
            assert math.isnan(mean[c]) and wq[c] == prior[0, c]
            continue
        assert abs(float(mean[c]) - mean_or[c]) <= SCORE_TOL
        if edge[c] > EDGE_TOL:
            assert int(wq[c]) == int(wq_or[c])
        else:
            assert abs(int(wq[c]) - int(wq_or[c])) <= 1


# ---------------------------------------------------------------------------------------------
# the many-workgroup launch shape (3 sample slots x 4 wavefronts), taken when
# ceil(n_samp / 4) * Hkv * B >= 1024, and Alg. 1 at the full 128K context
# ---------------------------------------------------------------------------------------------
def test_importance_many_workgroups_gqa_batch():
    """Llama-3-8B head shape, 4 sequences, 16 classes x 8 samples: 32 * 8 * 4 = 1024 sample groups."""
    wl, comp, prior = _run(5, B=4, seqlens=[3300, 2100, 4000, 2600])
    cfg = wl.cfg
    assert (cfg.n_class * cfg.M + 3) // 4 * cfg.Hkv * cfg.B >= 1024
    print("many-workgroup GQA batch worst = %.2e" % _check(wl, comp, prior))


def test_importance_many_workgroups_mha():
    """Llama2-13B head shape (40 KV heads, no grouping), one sequence: 32 * 40 = 1280 sample groups."""
    wl, comp, prior = _run(4, seqlens=[6000])
    cfg = wl.cfg
    assert (cfg.n_class * cfg.M + 3) // 4 * cfg.Hkv * cfg.B >= 1024
    print("many-workgroup MHA worst = %.2e" % _check(wl, comp, prior))


def test_importance_at_full_128k_context_both_launch_shapes():
    """Stage IMPORTANCE alone at 131072 tokens with sample positions given by the caller, spread
    over the whole context (the first and the last admissible position, the middle, tile edges),
    so that the key loop runs thousands of tiles and nearly all of them lie in the discarded
    region.  512 samples take the many-workgroup launch, a 6-sample call the other one; a
    handful of samples (all 32 heads, every window query) is compared with the oracle."""
    import paper_2602_03184_amd as dsk
    from workloads import f32_to_bf16_bits
    wl = make_workload(3, with_kv=True, with_qwin=False)
    cfg = wl.cfg
    L = wl.total_tokens
    assert L == 131072
    n_class, M = 16, 32
    n_samp = n_class * M
    assert (n_samp + 3) // 4 * cfg.Hkv >= 1024
    r = np.random.default_rng(2024)
    t_all = r.integers(cfg.R, L - cfg.W, size=n_samp).astype(np.int64)
    t_all[0] = cfg.R                      # first admissible position
    t_all[1] = L - 1 - cfg.W              # last admissible position: the window ends at the last token
    t_all[2] = L // 2                     # middle
    t_all[3] = 32 * 1000 - 1              # last key of a 32-key tile
    t_all[4] = 4096 + cfg.R               # retained region starts on a tile edge
    t_all[n_samp - 1] = 97 * 1024 + 13
    checked = [0, 1, 2, 3, 4, n_samp - 1]
    qwin_bits = f32_to_bf16_bits(r.standard_normal((1, n_samp, cfg.W, cfg.Hq, 128), dtype=np.float32))
    K = dev_bf16(wl.K)
    scale = 1.0 / math.sqrt(128.0)
    Kf = O.widen_bf16(wl.K)
    want = {j: O.delimiter_importance(O.widen_bf16(qwin_bits[0, j]), Kf, int(t_all[j]), cfg.R, cfg.alpha_imp, scale)
            for j in checked}
    del Kf

    def run(samp_idx, n_class_, M_):
        samp = torch.from_numpy(t_all[samp_idx].astype(np.int32).reshape(1, n_class_, M_)).cuda()
        qw = dev_bf16(np.ascontiguousarray(qwin_bits[:, samp_idx]))
        comp = dsk.compress(
            cu_seqlens=dev_i32(wl.cu_seqlens), max_seqlen=L, Hq=cfg.Hq, K=K, V=None,
            stages=dsk.DSK_STAGE_IMPORTANCE, n_class=n_class_, M=M_, W=cfg.W, R=cfg.R, alpha_imp=cfg.alpha_imp,
            samp_pos=samp, qwin=qw, class_weight_q=dev_u8(np.full((1, n_class_), 3, np.uint8)))
        torch.cuda.synchronize()
        assert int(comp.dev_status.item()) == 0
        return comp.samp_score.cpu().numpy().reshape(-1)

    big = run(np.arange(n_samp), n_class, M)              # many-workgroup launch
    assert np.isfinite(big).all() and (big >= -cfg.alpha_imp - 1e-5).all() and (big <= 1.0 + 1e-5).all()
    small = run(np.asarray(checked), 2, 3)                # few-workgroup launch on the checked samples
    worst = 0.0
    for i, j in enumerate(checked):
        for got in (float(big[j]), float(small[i])):
            worst = max(worst, abs(got - want[j]))
            assert abs(got - want[j]) <= SCORE_TOL, (j, int(t_all[j]), got, want[j])
    print("128K importance worst |s_gpu - s_oracle| = %.2e over %d samples" % (worst, len(checked)))
