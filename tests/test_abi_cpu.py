"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function
include/dsk.h declares, the ctypes structs mirror the C structs, and argument validation
rejects bad input before anything is launched."""
import ctypes as C
import os
import re
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "dsk.h")


@pytest.fixture(scope="module")
def dsk():
    import paper_2602_03184_amd as d
    return d


def _declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(dsk_[a-z_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol(dsk):
    names = _declared_functions()
    assert {"dsk_compress", "dsk_select_topk", "dsk_sparse_decode_attn"} <= set(names)
    lib = C.CDLL(dsk.binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert dsk.dsk_version() == 3
    assert dsk.dsk_strerror(0) == "ok" and "capacity" in dsk.dsk_strerror(dsk.DSK_ERR_CAPACITY)
    assert dsk.dsk_block_capacity(131072, 1, 16) == 8193
    assert dsk.dsk_block_capacity(10, 0, 16) == -1


def test_ctypes_structs_mirror_the_header(dsk, tmp_path):
    prog = tmp_path / "sizes.c"
    prog.write_text(r'''
#include <stdio.h>
#include <stddef.h>
#include "dsk.h"
int main(void) {
  printf("%zu %zu %zu ", sizeof(dsk_compress_args), sizeof(dsk_select_args), sizeof(dsk_attn_args));
  printf("%zu %zu %zu ", offsetof(dsk_compress_args, qwin), offsetof(dsk_compress_args, C_per_seq), offsetof(dsk_compress_args, workspace_bytes));
  printf("%zu %zu %zu ", offsetof(dsk_select_args, budget), offsetof(dsk_select_args, workspace_bytes), offsetof(dsk_select_args, max_blocks_per_seq));
  printf("%zu %zu ", offsetof(dsk_select_args, flags), offsetof(dsk_select_args, sel_slot));
  printf("%zu %zu %zu ", offsetof(dsk_attn_args, total_tokens), offsetof(dsk_attn_args, scale), offsetof(dsk_attn_args, workspace_bytes));
  printf("%zu %zu %zu %zu ", sizeof(dsk_dense_attn_args), offsetof(dsk_dense_attn_args, cu_seqlens), offsetof(dsk_dense_attn_args, scale), offsetof(dsk_dense_attn_args, workspace_bytes));
  printf("%zu %zu ", sizeof(dsk_attn_partials), offsetof(dsk_attn_partials, nchunks));
  printf("%zu %zu %zu %zu\n", offsetof(dsk_compress_args, summary_mode), sizeof(dsk_append_args), offsetof(dsk_append_args, summary_mode), offsetof(dsk_append_args, workspace_bytes));
  return 0;
}''')
    exe = tmp_path / "sizes"
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(prog), "-o", str(exe)])
    got = [int(x) for x in subprocess.check_output([str(exe)]).split()]
    ca, sa, aa = dsk.dsk_compress_args, dsk.dsk_select_args, dsk.dsk_attn_args
    want = [C.sizeof(ca), C.sizeof(sa), C.sizeof(aa), ca.qwin.offset, ca.C_per_seq.offset, ca.workspace_bytes.offset,
            sa.budget.offset, sa.workspace_bytes.offset, sa.max_blocks_per_seq.offset, sa.flags.offset, sa.sel_slot.offset,
            aa.total_tokens.offset, aa.scale.offset,
            aa.workspace_bytes.offset]
    da, pa = dsk.dsk_dense_attn_args, dsk.dsk_attn_partials
    want += [C.sizeof(da), da.cu_seqlens.offset, da.scale.offset, da.workspace_bytes.offset, C.sizeof(pa),
             pa.nchunks.offset]
    ap = dsk.dsk_append_args
    want += [ca.summary_mode.offset, C.sizeof(ap), ap.summary_mode.offset, ap.workspace_bytes.offset]
    assert got == want


def test_reuse_struct_mirrors_the_header_field_by_field(dsk, tmp_path):
    ra = dsk.dsk_reuse_args
    fields = [f[0] for f in ra._fields_]
    prog = tmp_path / "reuse.c"
    prog.write_text("#include <stdio.h>\n#include <stddef.h>\n#include \"dsk.h\"\nint main(void) {\n"
                    "  printf(\"%zu \", sizeof(dsk_reuse_args));\n"
                    + "".join('  printf("%%zu ", offsetof(dsk_reuse_args, %s));\n' % f for f in fields)
                    + "  printf(\"%d %d\\n\", (int)DSK_REUSE_PLAN_ONLY, (int)DSK_REUSE_MAX_K);\n  return 0;\n}\n")
    exe = tmp_path / "reuse"
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(prog), "-o", str(exe)])
    got = [int(x) for x in subprocess.check_output([str(exe)]).split()]
    want = [C.sizeof(ra)] + [getattr(ra, f).offset for f in fields] + [dsk.DSK_REUSE_PLAN_ONLY, dsk.DSK_REUSE_MAX_K]
    assert got == want


@pytest.mark.parametrize("name", ["dsk_append_batch_args", "dsk_select_args", "dsk_compress_args"])
def test_struct_mirrors_the_header_field_by_field(dsk, tmp_path, name):
    st = getattr(dsk.binding, name)
    fields = [f[0] for f in st._fields_]
    prog = tmp_path / "st.c"
    prog.write_text("#include <stdio.h>\n#include <stddef.h>\n#include \"dsk.h\"\nint main(void) {\n"
                    "  printf(\"%%zu \", sizeof(%s));\n" % name
                    + "".join('  printf("%%zu ", offsetof(%s, %s));\n' % (name, f) for f in fields)
                    + "  return 0;\n}\n")
    exe = tmp_path / "st"
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(prog), "-o", str(exe)])
    got = [int(x) for x in subprocess.check_output([str(exe)]).split()]
    assert got == [C.sizeof(st)] + [getattr(st, f).offset for f in fields]


def test_append_batch_validation(dsk):
    fake = 0x10000
    a = dsk.binding.dsk_append_batch_args()
    assert dsk.dsk_append_tokens_batch(a, 0, check=False) == dsk.DSK_ERR_VERSION
    a.struct_size = C.sizeof(a)
    assert dsk.dsk_append_batch_workspace_bytes(a) == 0            # B < 1
    a.B, a.Hkv, a.D = 3, 2, 128
    assert dsk.dsk_append_batch_workspace_bytes(a) == 256
    a.total_rows, a.max_new_tokens = 1000, 1
    a.n_class, a.C, a.delta, a.alpha_num, a.alpha_den, a.b, a.max_blocks_total = 4, 16, 8, 5, 10, 16, 64
    assert dsk.dsk_append_tokens_batch(a, 0, check=False) == dsk.DSK_ERR_NULL
    for f in ("seq_row0", "seq_len", "K", "token_ids", "delim_ids", "class_weight_q", "cu_blocks",
              "blocks_used", "block_start", "slot_base", "ksum"):
        setattr(a, f, fake)
    a.k_stride_tok, a.k_stride_head = 128, 128 * 1000
    assert dsk.dsk_append_tokens_batch(a, 0, check=False) == dsk.DSK_ERR_WORKSPACE
    a.delta = 16
    assert dsk.dsk_append_tokens_batch(a, 0, check=False) == dsk.DSK_ERR_PARAM
    a.delta, a.D = 8, 64
    assert dsk.dsk_append_tokens_batch(a, 0, check=False) == dsk.DSK_ERR_SHAPE


def test_reuse_validation(dsk):
    fake = 0x10000

    def args():
        a = dsk.dsk_reuse_args()
        a.struct_size = C.sizeof(a)
        a.B, a.Hq, a.Hkv, a.D = 2, 4, 2, 128
        a.k, a.b = 8, 16
        for f in ("sel_slot", "sel_start", "sel_len", "sel_count", "res_slot", "res_len", "res_start", "res_count",
                  "load_pos", "load_slot", "load_start", "load_len", "load_count", "reuse_count", "K", "V", "Kres",
                  "Vres"):
            setattr(a, f, fake)
        a.k_stride_tok = a.v_stride_tok = 128
        a.k_stride_head = a.v_stride_head = 128000
        a.total_tokens = 1000
        return a
    assert dsk.dsk_reuse_update(args(), 0, check=False) == dsk.DSK_ERR_WORKSPACE
    assert dsk.dsk_reuse_workspace_bytes(args()) >= 2 * 4 * 4
    for field, value, want in (("struct_size", 4, dsk.DSK_ERR_VERSION), ("Hkv", 3, dsk.DSK_ERR_SHAPE),
                               ("k", 0, dsk.DSK_ERR_SHAPE), ("k", dsk.DSK_REUSE_MAX_K + 1, dsk.DSK_ERR_SHAPE),
                               ("b", 0, dsk.DSK_ERR_SHAPE), ("flags", 2, dsk.DSK_ERR_PARAM),
                               ("sel_slot", None, dsk.DSK_ERR_NULL), ("res_slot", None, dsk.DSK_ERR_NULL),
                               ("load_len", None, dsk.DSK_ERR_NULL), ("reuse_count", None, dsk.DSK_ERR_NULL),
                               ("K", None, dsk.DSK_ERR_NULL), ("Vres", None, dsk.DSK_ERR_NULL),
                               ("K", fake + 2, dsk.DSK_ERR_ALIGN), ("k_stride_tok", 64, dsk.DSK_ERR_SHAPE),
                               ("v_stride_head", 4, dsk.DSK_ERR_ALIGN)):
        a = args()
        setattr(a, field, value)
        assert dsk.dsk_reuse_update(a, 0, check=False) == want, field
    # the plan alone needs neither the source nor the buffers
    a = args()
    a.flags = dsk.DSK_REUSE_PLAN_ONLY
    a.K = a.V = a.Kres = a.Vres = None
    assert dsk.dsk_reuse_update(a, 0, check=False) == dsk.DSK_ERR_WORKSPACE
    a = args()
    a.B, a.k, a.b = 65535, 2048, 1024       # more rows per resident head than int32 holds
    assert dsk.dsk_reuse_update(a, 0, check=False) == dsk.DSK_ERR_SHAPE


def _valid_compress(dsk):
    a = dsk.dsk_compress_args()
    a.struct_size = C.sizeof(a)
    a.stages = dsk.DSK_STAGE_SEGMENT
    a.B, a.Hq, a.Hkv, a.D = 1, 4, 2, 128
    a.total_tokens = a.max_seqlen = 1000
    fake = 0x10000   # never dereferenced: validation fails first in every case below
    a.cu_seqlens = fake
    a.n_class, a.max_cand_total = 4, 10
    a.cand_pos = a.cand_class = a.cand_cu = fake
    a.class_weight_q = fake
    a.C, a.delta, a.alpha_num, a.alpha_den, a.b = 24, 12, 5, 10, 16
    a.max_blocks_total = 100
    a.block_start = a.cu_blocks = a.slot_base = fake
    return a


def test_compress_validation_rejects_before_launch(dsk):
    a = _valid_compress(dsk)
    # valid so far except for the workspace -> WORKSPACE proves every earlier check passed
    assert dsk.dsk_compress(a, 0, check=False) == dsk.DSK_ERR_WORKSPACE
    assert dsk.dsk_compress_workspace_bytes(a) > 0
    cases = [
        ("struct_size", 8, dsk.DSK_ERR_VERSION), ("stages", 0, dsk.DSK_ERR_PARAM), ("stages", 64, dsk.DSK_ERR_PARAM),
        ("B", 0, dsk.DSK_ERR_SHAPE), ("D", 64, dsk.DSK_ERR_SHAPE), ("Hkv", 3, dsk.DSK_ERR_SHAPE),
        ("max_seqlen", 2000, dsk.DSK_ERR_SHAPE), ("cu_seqlens", None, dsk.DSK_ERR_NULL),
        ("n_class", 0, dsk.DSK_ERR_PARAM), ("n_class", 65, dsk.DSK_ERR_PARAM), ("cand_cu", None, dsk.DSK_ERR_NULL),
        ("cand_pos", None, dsk.DSK_ERR_NULL), ("class_weight_q", None, dsk.DSK_ERR_NULL),
        ("delta", 24, dsk.DSK_ERR_PARAM), ("delta", -1, dsk.DSK_ERR_PARAM), ("C", 0, dsk.DSK_ERR_PARAM),
        ("C", 8190, dsk.DSK_ERR_PARAM), ("alpha_num", 11, dsk.DSK_ERR_PARAM), ("alpha_den", 0, dsk.DSK_ERR_PARAM),
        ("b", 0, dsk.DSK_ERR_PARAM), ("b", 2048, dsk.DSK_ERR_PARAM), ("max_blocks_total", 0, dsk.DSK_ERR_PARAM),
        ("block_start", None, dsk.DSK_ERR_NULL), ("slot_base", None, dsk.DSK_ERR_NULL),
    ]
    for field, value, want in cases:
        a = _valid_compress(dsk)
        setattr(a, field, value)
        assert dsk.dsk_compress(a, 0, check=False) == want, field
    with pytest.raises(dsk.DskError):
        dsk.dsk_compress(_valid_compress(dsk), 0)
    # candidate lists left out: only together with the segmentation, without sampling
    a = _valid_compress(dsk)
    a.stages = dsk.DSK_STAGE_CANDIDATES | dsk.DSK_STAGE_SEGMENT
    a.token_ids = a.delim_ids = 0x10000
    a.cand_pos = a.cand_class = a.cand_cu = None
    a.max_cand_total = 0
    assert dsk.dsk_compress(a, 0, check=False) == dsk.DSK_ERR_WORKSPACE      # accepted up to the workspace
    a.samp_pos, a.M = 0x10000, 4
    assert dsk.dsk_compress(a, 0, check=False) == dsk.DSK_ERR_NULL          # sampling reads the lists
    a.samp_pos, a.M = None, 0
    a.stages = dsk.DSK_STAGE_CANDIDATES
    assert dsk.dsk_compress(a, 0, check=False) == dsk.DSK_ERR_NULL          # nothing would be produced
    # summaries stage: alignment and stride rules
    for field, value, want in (("K", 0x10002, dsk.DSK_ERR_ALIGN), ("k_stride_tok", 132, dsk.DSK_ERR_ALIGN),
                               ("k_stride_tok", 64, dsk.DSK_ERR_SHAPE), ("ksum", None, dsk.DSK_ERR_NULL),
                               ("k_stride_head", 0, dsk.DSK_ERR_SHAPE)):
        a2 = _valid_compress(dsk)
        a2.stages = dsk.DSK_STAGE_SUMMARIES
        a2.K, a2.ksum = 0x10000, 0x20000
        a2.k_stride_tok, a2.k_stride_head = 128, 128000
        setattr(a2, field, value)
        assert dsk.dsk_compress(a2, 0, check=False) == want, field


def test_select_and_attn_validation(dsk):
    fake = 0x10000

    def sel():
        a = dsk.dsk_select_args()
        a.struct_size = C.sizeof(a)
        a.B, a.Hq, a.Hkv, a.D = 1, 4, 2, 128
        a.max_blocks_total = 100
        for f in ("cu_blocks", "block_start", "slot_base", "ksum", "q", "sel_slot", "sel_start", "sel_len", "sel_count"):
            setattr(a, f, fake)
        a.b, a.budget = 16, 64
        return a
    assert dsk.dsk_select_topk(sel(), 0, check=False) == dsk.DSK_ERR_WORKSPACE
    assert dsk.dsk_select_workspace_bytes(sel()) >= 4 * 100 * 4
    a = sel()
    a.slot_base = fake + 8
    assert dsk.dsk_select_topk(a, 0, check=False) == dsk.DSK_ERR_ALIGN
    for field, value, want in (("struct_size", 1, dsk.DSK_ERR_VERSION), ("Hq", 5, dsk.DSK_ERR_SHAPE),
                               ("budget", 15, dsk.DSK_ERR_PARAM), ("b", 0, dsk.DSK_ERR_PARAM),
                               ("q", None, dsk.DSK_ERR_NULL), ("q", fake + 4, dsk.DSK_ERR_ALIGN),
                               ("max_blocks_total", 0, dsk.DSK_ERR_SHAPE), ("sel_count", None, dsk.DSK_ERR_NULL),
                               ("flags", 2, dsk.DSK_ERR_PARAM)):
        a = sel()
        setattr(a, field, value)
        assert dsk.dsk_select_topk(a, 0, check=False) == want, field

    def att():
        a = dsk.dsk_attn_args()
        a.struct_size = C.sizeof(a)
        a.B, a.Hq, a.Hkv, a.D = 1, 4, 2, 128
        for f in ("q", "K", "V", "sel_start", "sel_len", "sel_count", "out"):
            setattr(a, f, fake)
        a.k_stride_tok = a.v_stride_tok = 128
        a.k_stride_head = a.v_stride_head = 128 * 1000
        a.total_tokens, a.k, a.b = 1000, 8, 16
        return a
    assert dsk.dsk_sparse_decode_attn(att(), 0, check=False) == dsk.DSK_ERR_WORKSPACE
    assert dsk.dsk_attn_workspace_bytes(att()) > 0
    for field, value, want in (("k", 0, dsk.DSK_ERR_PARAM), ("scale", -1.0, dsk.DSK_ERR_PARAM),
                               ("scale", float("nan"), dsk.DSK_ERR_PARAM), ("flags", 4, dsk.DSK_ERR_PARAM),
                               ("V", None, dsk.DSK_ERR_NULL),
                               ("v_stride_tok", 100, dsk.DSK_ERR_SHAPE), ("k_stride_tok", 129, dsk.DSK_ERR_ALIGN),
                               ("out", None, dsk.DSK_ERR_NULL), ("D", 256, dsk.DSK_ERR_SHAPE)):
        a = att()
        setattr(a, field, value)
        assert dsk.dsk_sparse_decode_attn(a, 0, check=False) == want, field
    # a cache without any token has no K/V row: the pointers may be NULL then, and only then
    a = att()
    a.K = a.V = None
    assert dsk.dsk_sparse_decode_attn(a, 0, check=False) == dsk.DSK_ERR_NULL
    a.total_tokens = 0
    assert dsk.dsk_sparse_decode_attn(a, 0, check=False) == dsk.DSK_ERR_WORKSPACE


def test_binding_never_imports_the_oracle(dsk):
    assert not any(m == "oracle" or m.startswith("oracle.") for m in sys.modules
                   if "paper_2602_03184_amd" in (getattr(sys.modules[m], "__package__", "") or ""))
    src = open(os.path.join(ROOT, "paper_2602_03184_amd", "binding.py")).read()
    assert "oracle" not in src.replace("no CPU fallback", "")
