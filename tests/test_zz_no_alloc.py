"""dsk_sparse_decode_attn_static (the attention call that takes no workspace and allocates nothing: its
split-K partials live in a static device array inside the library) against dsk_sparse_decode_attn on
the same arguments, through the C ABI.  Same kernels, same fixed merge order: outputs must agree bit
for bit, and with the oracle to the attention bar.  Two calls in a row share the array, the second on
a smaller input."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import dynsplit_oracle as O
from dsk_testutil import DEFAULT_SCALE, gpu_case, rel_err

pytestmark = pytest.mark.gpu


def _dsk():
    import paper_2602_03184_amd as dsk
    return dsk


def _attend_both_ways(case, q, budget):
    """Selection for q, then attention through both entry points; returns (selection, workspace
    result, static result) with the static call made on argument structs that carry no workspace."""
    dsk = _dsk()
    comp = case.compressed()
    sel = dsk.select_topk(comp, q, budget)
    ref = dsk.sparse_decode_attn(q, case.K, case.V, sel.sel_start, sel.sel_len, sel.sel_count, case.cfg.b)
    st = dsk.make_attn_args(q, case.K, case.V, sel.sel_start, sel.sel_len, sel.sel_count, case.cfg.b)
    st.out.fill_(float("nan"))
    st.lse.fill_(float("nan"))
    st.args.workspace = None
    st.args.workspace_bytes = 0
    assert dsk.dsk_attn_workspace_bytes(st.args) <= dsk.DSK_STATIC_SCRATCH_BYTES
    dsk.dsk_sparse_decode_attn_static(st.args)
    torch.cuda.synchronize()
    return sel, ref, st


def _oracle_attention(case, q_bits, sel, s, h):
    cfg, wl = case.cfg, case.wl
    cnt = int(sel.sel_count[s, h])
    starts = sel.sel_start[s, h, :cnt].cpu().numpy()
    lens = sel.sel_len[s, h, :cnt].cpu().numpy()
    toks = np.concatenate([np.arange(a, a + n) for a, n in zip(starts, lens)])
    hk = h // cfg.G
    return O.sparse_attention(O.widen_bf16(q_bits[s, h]), O.widen_bf16(wl.K[hk]), O.widen_bf16(wl.V[hk]), toks,
                              DEFAULT_SCALE)


def test_static_scratch_attention_two_calls_second_smaller():
    from dsk_testutil import dev_bf16
    big = gpu_case(2)                                   # 32 heads x 128 slots: 8 partials per head
    small = gpu_case(1)                                 # 1 head x 16 slots: a single chunk, no partial at all
    mid = gpu_case(2, seqlens=[6000], T=512)            # 32 heads x 32 slots: 2 partials per head
    for case in (big, mid, small, big):                 # the last call finds the smaller calls' leftovers
        q_bits = case.wl.q[0]
        q = dev_bf16(q_bits)
        sel, ref, st = _attend_both_ways(case, q, case.cfg.T)
        assert torch.equal(st.out, ref.out), "static-scratch output differs from the workspace variant"
        assert torch.equal(st.lse, ref.lse)
        cfg = case.cfg
        for h in sorted({0, cfg.Hq // 2, cfg.Hq - 1}):
            o, lse = _oracle_attention(case, q_bits, sel, 0, h)
            assert rel_err(st.out[0, h].cpu().numpy(), o) <= 2e-3
            assert abs(float(st.lse[0, h]) - lse) <= 1e-3


def test_static_scratch_rejects_what_does_not_fit():
    """More partials than the static array holds: a clear error before anything is enqueued."""
    dsk = _dsk()
    a = dsk.dsk_attn_args()
    a.struct_size = C.sizeof(a)
    a.B, a.Hq, a.Hkv, a.D = 64, 32, 8, 128
    a.k, a.b, a.total_tokens = 256, 16, 1 << 20          # 64 * 32 * 16 chunks = 32768 partials
    fake = 0x10000
    for f in ("q", "K", "V", "sel_start", "sel_len", "sel_count", "out"):
        setattr(a, f, fake)
    a.k_stride_tok = a.v_stride_tok = 128
    a.k_stride_head = a.v_stride_head = 128 << 20
    assert dsk.dsk_attn_workspace_bytes(a) > dsk.DSK_STATIC_SCRATCH_BYTES
    assert dsk.dsk_sparse_decode_attn_static(a, 0, check=False) == dsk.DSK_ERR_WORKSPACE
    a.q = None
    assert dsk.dsk_sparse_decode_attn_static(a, 0, check=False) == dsk.DSK_ERR_NULL
