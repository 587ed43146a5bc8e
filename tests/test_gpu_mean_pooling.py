"""GPU parity of the mean-pooling summary mode (App. A.2: min/max compression replaced by mean
pooling, everything else unchanged).  The mean is accumulated in fp32 on the GPU and in fp64 in
the oracle, then rounded to bf16: equal bits except, rarely, a neighbouring bf16 value where the
exact mean sits next to a rounding midpoint (counted, bounded).  Scores, selection and attention
on top of the GPU's own means meet the bars of the (min,max) path."""
import numpy as np
import pytest
import torch

from oracle import dynsplit_oracle as O
from dsk_testutil import (assert_bf16_of, bf16_bits_of, dev_bf16, gpu_case, oracle_means_bf16, selection_check)
from test_gpu_decode import _check_decode, _heads_to_check, _seqs_to_check

pytestmark = pytest.mark.gpu
MEAN = 1


def _dsk():
    import paper_2602_03184_amd as dsk
    return dsk


@pytest.mark.parametrize("cfg_id", [1, 2, 5])
def test_mean_summaries_match_the_oracle(cfg_id):
    case = gpu_case(cfg_id, summary_mode=MEAN)
    comp = case.compressed()
    seg, wl = case.seg, case.wl
    nblk = int(seg.cu_blocks[-1])
    assert int(comp.cu_blocks.cpu()[-1]) == nblk
    sums = bf16_bits_of(comp.ksum)[:, :nblk]
    np.testing.assert_array_equal(sums[:, :, 0], sums[:, :, 1])          # the mean sits in both rows
    heads = range(wl.K.shape[0]) if cfg_id != 5 else [0, 7]
    exact = oracle_means_bf16(wl.K, seg.block_start, heads)
    frac = assert_bf16_of(sums[list(heads), :, 0], exact)
    print("cfg%d: means off by one bf16 step: %.2e of elements" % (cfg_id, frac))


@pytest.mark.parametrize("cfg_id", [1, 2, 3])
def test_decode_on_mean_summaries(cfg_id):
    dsk = _dsk()
    case = gpu_case(cfg_id, summary_mode=MEAN)
    cfg, wl, seg = case.cfg, case.wl, case.seg
    _check_decode(case, 1, _seqs_to_check(cfg), _heads_to_check(cfg), "cfg%d mean pooling" % cfg_id)
    # the score is the plain dot product with the mean (written out, not via the box formula)
    comp = case.compressed()
    nblk = int(seg.cu_blocks[-1])
    mean_bits = bf16_bits_of(comp.ksum)[:, :nblk, 0]
    q_bits = wl.q[0]
    sel = dsk.select_topk(comp, dev_bf16(q_bits), cfg.T, want_scores=True)
    torch.cuda.synchronize()
    h = cfg.Hq - 1
    want = O.block_scores_mean(O.widen_bf16(q_bits[0, h])[None], O.widen_bf16(mean_bits[h // cfg.G])[None])[0]
    np.testing.assert_allclose(sel.scores.cpu().numpy()[h, :nblk], want, rtol=2e-5, atol=2e-4)


def test_append_keeps_mean_summaries_current():
    from test_gpu_append import _Seq
    case = gpu_case(2, seqlens=[5000])
    wl, cfg = case.wl, case.cfg
    seq = _Seq(wl.K, wl.V, wl.token_ids, wl.delim_ids, wl.class_weight_q[0], 2000, int(wl.C[0]), int(wl.delta[0]),
               cfg.a_num, cfg.a_den, cfg.b, Hq=cfg.Hq, summary_mode=MEAN)
    r = np.random.default_rng(9)
    while seq.L < 4900:
        want, i0 = seq.append(int(r.integers(1, 200)))
        seq.check_tables(want, i0)
    nblk = len(want) - 1
    sums = bf16_bits_of(seq.comp.ksum)[:, :nblk]
    np.testing.assert_array_equal(sums[:, :, 0], sums[:, :, 1])
    assert_bf16_of(sums[:, :, 0], oracle_means_bf16(wl.K[:, : seq.L], want))
