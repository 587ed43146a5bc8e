"""GPU parity on seeded random geometries: head counts and group widths, slot lengths from 1 to 128,
budgets, ragged batches with empty and tiny sequences, segmentation parameters from C = 1 to
C + delta in the thousands, class counts from 1 to 64 -- every case through the same checks as
the fixed configurations (tables bit-exact, selections up to counted near ties, attention within
2e-3 of the fp64 oracle, reuse plans bit-exact, appended tables equal to the from-scratch run)."""
import numpy as np
import pytest

import dsk_testutil as U
import test_gpu_append as TA
import test_gpu_compress as TC
import test_gpu_decode as TD
import test_gpu_dense as TDe
import test_gpu_group_select as TG
import test_gpu_importance as TI
import test_gpu_reuse as TR

pytestmark = pytest.mark.gpu


def _geometry(r, max_len, b_choices, C_choices, class_choices):
    Hkv = int(r.choice([1, 2, 4, 8]))
    G = int(r.choice([1, 2, 3, 4, 8]))
    b = int(r.choice(b_choices))
    B = int(r.integers(1, 6))
    seqlens = [int(x) for x in r.integers(0, max_len, size=B)]
    if r.random() < 0.3:
        seqlens[int(r.integers(0, B))] = int(r.integers(0, 40))
    C = int(r.choice(C_choices)) if C_choices else int(r.integers(2, 80))
    k = int(r.integers(1, 200))
    return dict(B=B, Hq=Hkv * G, Hkv=Hkv, seqlens=seqlens, b=b, T=k * b, C=C, delta=int(r.integers(0, C)),
                a_num=int(r.integers(0, 11)), n_queries=2, gap_means=[int(r.integers(2, 90))],
                n_class=int(r.choice(class_choices)))


@pytest.mark.parametrize("seed", range(12))
def test_decode_shared_selection_and_reuse_on_random_geometries(seed):
    r = np.random.default_rng(40000 + seed)
    kw = _geometry(r, 7000, [4, 8, 16, 32, 64], None, [16])
    case = U.gpu_case(2, **kw)
    cfg = case.cfg
    TC._check_tables(case.compressed(), case.seg)
    heads = sorted({0, cfg.Hq - 1, int(r.integers(0, cfg.Hq))})
    seqs = list(range(cfg.B))
    TD._check_decode(case, 2, seqs, heads, "random %d %s" % (seed, kw))
    if cfg.G > 1:
        TG._check_shared(case, 1, seqs, sorted({0, cfg.Hkv - 1}), "random shared %d" % seed)
    if sum(kw["seqlens"]) > 0:
        TR._run(case, 3, 0.95, heads, T=cfg.T, repeat_at=(2,), seed=seed)
    U.drop_cases()


@pytest.mark.parametrize("seed", range(8))
def test_summaries_dense_and_mean_pooling_on_random_geometries(seed):
    r = np.random.default_rng(41000 + seed)
    kw = _geometry(r, 4000, [1, 2, 4, 16, 32, 128], [1, 2, 7, 30, 200, 3000], [1, 3, 16, 64])
    kw["n_queries"] = 1
    case = U.gpu_case(2, **kw)
    cfg = case.cfg
    comp = case.compressed()
    TC._check_tables(comp, case.seg)
    nb = int(case.seg.cu_blocks[-1])
    if nb > 0:
        got = U.bf16_bits_of(comp.ksum)
        kmin, kmax = U.oracle_summaries(case.wl.K, case.seg.block_start, [cfg.Hkv - 1])
        np.testing.assert_array_equal(U.canon_zero(got[cfg.Hkv - 1, :nb, 0]), U.canon_zero(kmin[0]))
        np.testing.assert_array_equal(U.canon_zero(got[cfg.Hkv - 1, :nb, 1]), U.canon_zero(kmax[0]))
    TDe._check(case, case.wl.q[0], list(range(cfg.B)), sorted({0, cfg.Hq - 1}))
    TD._check_decode(case, 1, list(range(cfg.B)), sorted({0, cfg.Hq - 1}), "random extreme %d" % seed)
    U.drop_cases()
    mean_case = U.gpu_case(2, summary_mode=1, **kw)
    TD._check_decode(mean_case, 1, list(range(cfg.B)), sorted({0, cfg.Hq - 1}), "random mean %d" % seed)
    U.drop_cases()


@pytest.mark.parametrize("seed", range(6))
def test_append_loops_on_random_parameters(seed):
    r = np.random.default_rng(42000 + seed)
    Hkv = int(r.choice([1, 2, 4]))
    L_cap = int(r.integers(300, 3000))
    case = U.gpu_case(2, Hq=Hkv * int(r.choice([1, 4])), Hkv=Hkv, seqlens=[L_cap], n_queries=1,
                      gap_means=[int(r.integers(2, 90))], n_class=int(r.choice([1, 3, 16, 64])))
    wl = case.wl
    C = int(r.choice([1, 2, 7, 30, 200]))
    seq = TA._Seq(wl.K, wl.V, wl.token_ids, wl.delim_ids, wl.class_weight_q[0], int(r.integers(0, L_cap)), C,
                  int(r.integers(0, C)), int(r.integers(0, 11)), 10, int(r.choice([1, 4, 16, 32])),
                  want_vsum=bool(r.integers(0, 2)), Hq=case.cfg.Hq)
    want = None
    while seq.L < L_cap:
        want, i0 = seq.append(min(int(r.choice([0, 1, 1, 1, 2, 17, 300])), L_cap - seq.L))
        seq.check_tables(want, i0)
    if want is not None and seq.L > 0:
        seq.check_summaries(want)
    U.drop_cases()


@pytest.mark.parametrize("seed", range(6))
def test_importance_on_random_shapes(seed):
    r = np.random.default_rng(43000 + seed)
    Hkv = int(r.choice([1, 2, 4]))
    B = int(r.integers(1, 5))
    seqlens = [int(x) for x in r.integers(0, 3000, size=B)]
    seqlens[0] = max(seqlens[0], 50)
    ov = dict(B=B, Hq=Hkv * int(r.choice([1, 2, 3, 4, 8])), Hkv=Hkv, seqlens=seqlens, M=int(r.choice([1, 3, 8])),
              W=int(r.choice([1, 4, 8, 13])), R=int(r.choice([1, 16, 128, 500])), n_class=int(r.choice([1, 3, 16])),
              gap_means=[int(r.integers(2, 60))], alpha_imp=float(r.choice([0.0, 0.5, 1.0, 2.0])))
    wl, comp, prior = TI._run(2, **ov)
    TI._check(wl, comp, prior)
