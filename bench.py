#!/usr/bin/env python3
"""Benchmark of the DynSplit-KV hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3]

A step is one decode step of the whole per-token path -- dsk_select_topk (block scores +
slot top-k) followed by dsk_sparse_decode_attn -- on the configuration the headline metric is
quoted on (Llama-3-8B layer shape, 128K context, b=32, budget 4096),
cycling over 32 distinct queries.  Inputs are resident in HBM before the timed region; the
K timed steps are captured in one HIP graph so that host launch cost is not what is timed.
The compression pass (dsk_compress) is timed separately and reported in the same line, as
are the roofline of the dominant kernel and the CPU oracle timed on this machine's host cores.
Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM traffic of the dominant kernel per launch, from `rocprofv3 --pmc FETCH_SIZE` and
# `--pmc WRITE_SIZE` runs of this file (summaries under profiles/), each scaled by what the same
# counter reads for the plain 256 MiB device copy of --calib-copy-mib (FETCH_SIZE reads half the
# copied bytes on this part -> x2; WRITE_SIZE reads them exactly -> x1).  Keyed by workload.
MEASURED_TRAFFIC_BYTES = {
    "cfg3_llama3_8b_128k": {"attn_kernel": int(16795.0 * 1024 * 2.000 + 130.0 * 1024 * 1.000)},
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=320)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--replays", type=int, default=7,
                    help="timed replays of every HIP graph; the median is reported")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-parity", action="store_true", help="skip the oracle parity summary")
    ap.add_argument("--append-steps", type=int, default=256,
                    help="steps of the decode loop that appends one token per step before selecting; 0 = skip")
    ap.add_argument("--no-shared-selection", action="store_true",
                    help="skip the leg that measures the shared-selection extension")
    ap.add_argument("--reuse-steps", type=int, default=48,
                    help="decode steps of the KV-reuse leg (K/V in pinned host memory); 0 disables it")
    ap.add_argument("--reuse-rho", type=float, default=0.98,
                    help="step-to-step correlation of the drifting query stream of the KV-reuse leg")
    ap.add_argument("--cold-instances", type=int, default=16,
                    help="copies of the cache (K, V, summaries) the cold-cache measurement rotates over; 0 = skip")
    ap.add_argument("--stream-read-mib", type=int, default=2048,
                    help="size of the buffer the streaming-read reference reads; 0 = skip")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (reference dispatch for rocprofv3 "
                         "--pmc FETCH_SIZE / WRITE_SIZE scaling)")
    return ap.parse_args()


def stream_read_probe():
    """The streaming-read yardstick of the bench (its own shared object, not part of libdsk)."""
    import ctypes
    path = os.path.join(ROOT, "paper_2602_03184_amd", "libdsk_benchaid.so")
    if not os.path.exists(path):
        raise RuntimeError("libdsk_benchaid.so is not built: run `python paper_2602_03184_amd/build.py`")
    lib = ctypes.CDLL(path)
    lib.dsk_benchaid_stream_read.restype = ctypes.c_int
    lib.dsk_benchaid_stream_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]

    def read_once(buf, stream, sink):
        rc = lib.dsk_benchaid_stream_read(buf.data_ptr(), buf.numel() * buf.element_size(), sink.data_ptr(),
                                          stream.cuda_stream or None)
        if rc != 0:
            raise RuntimeError("dsk_benchaid_stream_read failed (%d)" % rc)
    return read_once


def replay_us(graph, stream, n_nodes, replays):
    """Median over `replays` timed replays of a captured graph, in us per captured step."""
    graph.replay()
    stream.synchronize()
    t = sorted(event_ms(graph.replay, stream) for _ in range(max(1, replays)))
    return t[len(t) // 2] * 1e3 / n_nodes, [round(x * 1e3 / n_nodes, 3) for x in t]


def event_ms(fn, stream):
    import torch
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    fn()
    e1.record(stream)
    e1.synchronize()
    return e0.elapsed_time(e1)


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus %d is not supported. Run with --gpus 1." % args.gpus, file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import paper_2602_03184_amd as dsk
    from workloads import CONFIGS, make_workload

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    cfg = CONFIGS[args.config]
    t0 = time.time()
    wl = make_workload(args.config, with_kv=True, with_qwin=True)
    gen_s = time.time() - t0

    def bf16(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev).view(torch.bfloat16)

    def i32(a):
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)

    K, V = bf16(wl.K), bf16(wl.V)
    q_bits = [wl.q[i] for i in range(cfg.n_queries)]
    if len(q_bits) < 8:     # a workload that names one query: more seeded draws, so that consecutive steps differ
        from workloads import extra_queries
        q_bits += list(extra_queries(cfg, 8 - len(q_bits)))
    queries = [bf16(qb) for qb in q_bits]
    cu = i32(wl.cu_seqlens)
    ckw = dict(cu_seqlens=cu, max_seqlen=int(wl.seqlens.max()), Hq=cfg.Hq, K=K, V=V,
               stages=dsk.DSK_STAGE_CANDIDATES | dsk.DSK_STAGE_SEGMENT | dsk.DSK_STAGE_SUMMARIES,
               token_ids=i32(wl.token_ids), delim_ids=i32(wl.delim_ids), n_class=cfg.n_class,
               class_weight_q=torch.from_numpy(wl.class_weight_q).to(dev),
               C_=int(wl.C.max()), delta=int(wl.delta.max()),
               C_per_seq=i32(wl.C) if cfg.B > 1 else None, delta_per_seq=i32(wl.delta) if cfg.B > 1 else None,
               min_chunk=int((wl.C - wl.delta).min()), alpha_num=cfg.a_num, alpha_den=cfg.a_den, b=cfg.b)
    stream = torch.cuda.Stream()   # default priority
    if args.calib_copy_mib > 0:
        src = torch.empty(args.calib_copy_mib << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)               # reads and writes exactly calib_copy_mib MiB
        torch.cuda.synchronize()
        del src, dst
    with torch.cuda.stream(stream):
        comp = dsk.compress(**ckw)
        stream.synchronize()
        assert int(comp.dev_status.item()) == 0
        cub = comp.cu_blocks.cpu().numpy()
        nblk = int(cub[-1])
        nblk_seq = int((cub[1:] - cub[:-1]).max())     # read back once, like nblk: a launch-sizing hint
        nslots = int(comp.slot_base.cpu()[nblk])

        # ---- compression pass, timed by itself (same buffers re-used) -------------------------
        cargs = comp.args
        for _ in range(3):
            dsk.dsk_compress(cargs, stream)
        n_c = 10

        def compress_graph_ms(cargs_):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                for _ in range(n_c):
                    dsk.dsk_compress(cargs_, stream)
            return replay_us(g, stream, n_c, args.replays)[0] * 1e-3
        compress_ms = compress_graph_ms(cargs)
        compress_bytes = wl.total_tokens * cfg.Hkv * 128 * 2 + nblk * cfg.Hkv * 512 + wl.total_tokens * 4
        # the same pass without the candidate lists (weights from a table need none: the classes go
        # straight to the segmentation), reported beside the full figure
        lean = dsk.compress(**dict(ckw, want_candidates=False))
        for _ in range(3):
            dsk.dsk_compress(lean.args, stream)
        compress_lean_ms = compress_graph_ms(lean.args)
        stream.synchronize()
        assert torch.equal(lean.block_start[: nblk + 1], comp.block_start[: nblk + 1])

        # ---- delimiter importance (Alg. 1 on the sampled windows), timed by itself: the weights are
        #      estimated once per scenario, so it is not part of the per-prefill figure above ---------
        ikw = dict(ckw)
        ikw.update(stages=dsk.DSK_STAGE_CANDIDATES | dsk.DSK_STAGE_IMPORTANCE, V=None, M=cfg.M, W=cfg.W, R=cfg.R,
                   alpha_imp=cfg.alpha_imp, qwin=bf16(wl.qwin),
                   class_weight_q=torch.full((cfg.B, cfg.n_class), 5, dtype=torch.uint8, device=dev))
        icomp = dsk.compress(**ikw)
        stream.synchronize()
        n_samples = int((icomp.samp_pos >= 0).sum().item())
        icomp.args.stages = dsk.DSK_STAGE_IMPORTANCE
        dsk.dsk_compress(icomp.args, stream)
        importance_us = event_ms(lambda: [dsk.dsk_compress(icomp.args, stream) for _ in range(5)], stream) * 1e3 / 5

        # ---- decode step: per-query argument structs, buffers shared --------------------------
        nq = len(queries)
        # the block count was read back once after compression: it sizes the score launch
        sels = [dsk.make_select_args(comp, queries[0], cfg.T, max_blocks_used=nblk, max_blocks_per_seq=nblk_seq)]
        for i in range(1, nq):
            sels.append(dsk.make_select_args(comp, queries[i], cfg.T, out=sels[0], max_blocks_used=nblk,
                                             max_blocks_per_seq=nblk_seq))
        atts = [dsk.make_attn_args(queries[0], K, V, sels[0].sel_start, sels[0].sel_len, sels[0].sel_count, cfg.b)]
        for i in range(1, nq):
            atts.append(dsk.make_attn_args(queries[i], K, V, sels[0].sel_start, sels[0].sel_len, sels[0].sel_count,
                                           cfg.b, out=atts[0]))

        def step(i):
            dsk.dsk_select_topk(sels[i % nq].args, stream)
            dsk.dsk_sparse_decode_attn(atts[i % nq].args, stream)

        for i in range(args.warmup):
            step(i)
        stream.synchronize()

        # algorithmic bytes of one step: every summary once + K/V rows of the selected tokens
        sel_tokens = []
        for i in range(nq):
            step(i)
            stream.synchronize()
            sel_tokens.append(int(sels[0].sel_len.sum().item()))
        mean_sel_tokens = float(np.mean(sel_tokens))
        bytes_scores = nblk * cfg.Hkv * 512
        bytes_attn = mean_sel_tokens * 512          # 256 B of K + 256 B of V per selected (head, token)
        bytes_small = cfg.B * cfg.Hq * (128 * 2 + 128 * 4 + 3 * cfg.k * 4 * 2)
        step_bytes = bytes_scores + bytes_attn + bytes_small

        # ---- K steps in one graph --------------------------------------------------------------
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for i in range(args.steps):
                step(i)
        torch.cuda.synchronize()
        us_per_step, step_samples = replay_us(graph, stream, args.steps, args.replays)
        torch.cuda.synchronize()

        # eager launches, for reference (host launch cost included)
        eager_ms = event_ms(lambda: [step(i) for i in range(args.steps)], stream)
        eager_us = eager_ms * 1e3 / args.steps

        # ---- dominant kernel: the attention gather (attn_kernel) alone, HIP events on its stream.
        #      Every query keeps the selection made for it (its own span lists), so that consecutive
        #      launches gather different rows, as consecutive steps do. -----------------------------
        own = [dsk.make_select_args(comp, queries[i], cfg.T, max_blocks_used=nblk, max_blocks_per_seq=nblk_seq)
               for i in range(nq)]
        for i in range(nq):
            dsk.dsk_select_topk(own[i].args, stream)
        stream.synchronize()
        own_tokens = float(np.mean([int(o.sel_len.sum().item()) for o in own]))
        assert own_tokens == mean_sel_tokens
        gathers = [dsk.make_attn_args(queries[i], K, V, own[i].sel_start, own[i].sel_len, own[i].sel_count,
                                      cfg.b, out=atts[0], flags=dsk.DSK_ATTN_PARTIALS_ONLY) for i in range(nq)]
        g_gather = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_gather, stream=stream):
            for i in range(args.steps):
                dsk.dsk_sparse_decode_attn(gathers[i % nq].args, stream)
        gather_us = replay_us(g_gather, stream, args.steps, args.replays)[0]
        # the same launches on ONE selection (the rows of every launch then sit in the memory-side
        # cache): what the kernel does when HBM is out of the way
        same = [dsk.make_attn_args(queries[i], K, V, own[0].sel_start, own[0].sel_len, own[0].sel_count,
                                   cfg.b, out=atts[0], flags=dsk.DSK_ATTN_PARTIALS_ONLY) for i in range(nq)]
        g_same = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_same, stream=stream):
            for i in range(args.steps):
                dsk.dsk_sparse_decode_attn(same[i % nq].args, stream)
        gather_same_rows_us = replay_us(g_same, stream, args.steps, args.replays)[0]
        # the whole attention call (gather + merge of the partials) and the whole selection call
        own_att = [dsk.make_attn_args(queries[i], K, V, own[i].sel_start, own[i].sel_len, own[i].sel_count, cfg.b,
                                      out=atts[0]) for i in range(nq)]
        g_attn = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_attn, stream=stream):
            for i in range(args.steps):
                dsk.dsk_sparse_decode_attn(own_att[i % nq].args, stream)
        attn_us = replay_us(g_attn, stream, args.steps, args.replays)[0]
        g_sel = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_sel, stream=stream):
            for i in range(args.steps):
                dsk.dsk_select_topk(sels[i % nq].args, stream)
        select_us = replay_us(g_sel, stream, args.steps, args.replays)[0]
        # the gather's share of a step (the kernel right behind the selection whose lists it reads,
        # and the dependency gap in front of it): (selection + gather) - (selection), both as graphs
        # of the same length
        g_sgat = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_sgat, stream=stream):
            for i in range(args.steps):
                dsk.dsk_select_topk(sels[i % nq].args, stream)
                dsk.dsk_sparse_decode_attn(gathers[i % nq].args, stream)
        gather_in_step_us = replay_us(g_sgat, stream, args.steps, args.replays)[0] - select_us

        # ---- extension (not in the paper): one selection per KV head, shared by its query heads ----
        shared = None
        if cfg.G > 1 and not args.no_shared_selection:
            ssel = [dsk.make_select_args(comp, queries[0], cfg.T, max_blocks_used=nblk, max_blocks_per_seq=nblk_seq,
                                         shared=True)]
            for i in range(1, nq):
                ssel.append(dsk.make_select_args(comp, queries[i], cfg.T, out=ssel[0], max_blocks_used=nblk,
                                                 max_blocks_per_seq=nblk_seq, shared=True))
            sflag = dsk.DSK_ATTN_SHARED_SELECTION
            satt = [dsk.make_attn_args(queries[0], K, V, ssel[0].sel_start, ssel[0].sel_len, ssel[0].sel_count, cfg.b,
                                       flags=sflag)]
            for i in range(1, nq):
                satt.append(dsk.make_attn_args(queries[i], K, V, ssel[0].sel_start, ssel[0].sel_len, ssel[0].sel_count,
                                               cfg.b, out=satt[0], flags=sflag))
            # gather alone: every query on its own shared selection (different rows per launch)
            sown = [dsk.make_select_args(comp, queries[i], cfg.T, max_blocks_used=nblk, max_blocks_per_seq=nblk_seq,
                                         shared=True) for i in range(nq)]
            stok = []
            for i in range(nq):
                dsk.dsk_select_topk(sown[i].args, stream)
                stream.synchronize()
                stok.append(int(sown[i].sel_len.sum().item()))
            sgat = [dsk.make_attn_args(queries[i], K, V, sown[i].sel_start, sown[i].sel_len, sown[i].sel_count, cfg.b,
                                       out=satt[0], flags=sflag | dsk.DSK_ATTN_PARTIALS_ONLY) for i in range(nq)]
            g_sh = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_sh, stream=stream):
                for i in range(args.steps):
                    dsk.dsk_select_topk(ssel[i % nq].args, stream)
                    dsk.dsk_sparse_decode_attn(satt[i % nq].args, stream)
            shared_us = replay_us(g_sh, stream, args.steps, args.replays)[0]
            g_sg = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_sg, stream=stream):
                for i in range(args.steps):
                    dsk.dsk_sparse_decode_attn(sgat[i % nq].args, stream)
            shared_gather_us = replay_us(g_sg, stream, args.steps, args.replays)[0]
            sbytes = float(np.mean(stok)) * 512           # K/V rows the group gathers once
            shared = {"us_per_step": round(shared_us, 3), "gather_us": round(shared_gather_us, 3),
                      "gather_bytes_per_kv_head_model": int(sbytes),
                      "gather_GBps": round(sbytes / (shared_gather_us * 1e-6) / 1e9, 1),
                      "gather_frac": round(sbytes / (shared_gather_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                      "what": "DSK_SELECT_SHARED_BY_KV_GROUP + DSK_ATTN_SHARED_SELECTION: group score = max over "
                              "the group's query heads; not the paper's per-head selection"}
            del g_sh, g_sg

        # ---- full attention over the whole cache on the same device (the full-KV baseline) --------
        dense = dsk.make_dense_attn_args(queries[0], K, V, cu, int(wl.seqlens.max()))
        dense_args = [dense] + [dsk.make_dense_attn_args(queries[i], K, V, cu, int(wl.seqlens.max()), out=dense)
                                for i in range(1, nq)]
        n_dense = max(8, min(args.steps, 64))
        g_dense = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_dense, stream=stream):
            for i in range(n_dense):
                dsk.dsk_dense_decode_attn(dense_args[i % nq].args, stream)
        dense_us = replay_us(g_dense, stream, n_dense, args.replays)[0]
        dense_bytes = 2 * wl.total_tokens * cfg.Hkv * 128 * 2

        # ---- streaming-read reference: what a plain coalesced read reaches on this device ------
        stream_read_gbs = None
        if args.stream_read_mib > 0:
            big = torch.empty(args.stream_read_mib << 20, dtype=torch.uint8, device=dev).fill_(1)
            sink = torch.zeros(1, dtype=torch.int32, device=dev)
            stream.wait_stream(torch.cuda.current_stream())
            read_once = stream_read_probe()
            for _ in range(2):
                read_once(big, stream, sink)
            reps = 10
            ms = event_ms(lambda: [read_once(big, stream, sink) for _ in range(reps)], stream) / reps
            stream_read_gbs = big.numel() / (ms * 1e-3) / 1e9
            del big
            torch.cuda.empty_cache()

        # ---- cold caches: rotate over N copies of (K, V, summaries) so that no step finds the data
        #      of an earlier one in L2 or the memory-side cache; block tables are shared ----------
        cold = None
        if args.cold_instances > 1:
            n_inst = args.cold_instances
            Ks = [K] + [K.clone() for _ in range(n_inst - 1)]
            Vs = [V] + [V.clone() for _ in range(n_inst - 1)]
            ksums = [comp.ksum] + [comp.ksum.clone() for _ in range(n_inst - 1)]
            torch.cuda.synchronize()
            csel, catt, cgat = [], [], []
            n_cold = max(nq, n_inst)
            for i in range(n_cold):
                inst = i % n_inst
                sa = dsk.make_select_args(comp, queries[i % nq], cfg.T, out=sels[0], max_blocks_used=nblk,
                                          max_blocks_per_seq=nblk_seq)
                sa.args.ksum = ksums[inst].data_ptr()
                csel.append(sa)
                catt.append(dsk.make_attn_args(queries[i % nq], Ks[inst], Vs[inst], sels[0].sel_start, sels[0].sel_len,
                                               sels[0].sel_count, cfg.b, out=atts[0]))
                cgat.append(dsk.make_attn_args(queries[i % nq], Ks[inst], Vs[inst], sels[0].sel_start, sels[0].sel_len,
                                               sels[0].sel_count, cfg.b, out=atts[0], flags=dsk.DSK_ATTN_PARTIALS_ONLY))

            def cold_step(i):
                dsk.dsk_select_topk(csel[i % n_cold].args, stream)
                dsk.dsk_sparse_decode_attn(catt[i % n_cold].args, stream)

            g_cold = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_cold, stream=stream):
                for i in range(args.steps):
                    cold_step(i)
            cold_us = replay_us(g_cold, stream, args.steps, args.replays)[0]
            # gather alone, cold: each launch follows the selection of its own step's query, so run
            # select (untimed share subtracted) is not possible inside one graph; time gather-only
            # launches on the rotating copies with the last selection instead
            g_cg = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_cg, stream=stream):
                for i in range(args.steps):
                    dsk.dsk_sparse_decode_attn(cgat[i % n_cold].args, stream)
            cold_gather_us = replay_us(g_cg, stream, args.steps, args.replays)[0]
            last_sel_bytes = float(sels[0].sel_len.sum().item()) * 512
            cold = {"instances": n_inst, "cache_bytes_per_instance": int(2 * K.numel() * 2 + comp.ksum.numel() * 2),
                    "us_per_step": round(cold_us, 3),
                    "gather_us": round(cold_gather_us, 3),
                    "gather_GBps": round(last_sel_bytes / (cold_gather_us * 1e-6) / 1e9, 1),
                    "gather_frac": round(last_sel_bytes / (cold_gather_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)}
            del Ks, Vs, ksums, csel, catt, cgat, g_cold, g_cg
            torch.cuda.empty_cache()

        # ---- decode loop with the incremental update: the cache of the first L - n tokens is
        #      compressed, then every step appends one token (dsk_append_tokens), selects and attends.
        #      Single-sequence workloads only (the update takes one sequence per call). ---------------
        loop = None
        if cfg.B == 1 and args.append_steps > 0:
            n_app = min(args.append_steps, wl.total_tokens // 2)
            L0 = wl.total_tokens - n_app
            lkw = dict(ckw)
            lkw.update(cu_seqlens=i32([0, L0]), max_seqlen=L0, total_tokens=L0, max_cand_total=wl.total_tokens,
                       max_blocks_total=dsk.dsk_block_capacity(wl.total_tokens, 1, int((wl.C - wl.delta).min())),
                       C_per_seq=None, delta_per_seq=None)
            lcomp = dsk.compress(**lkw)
            stream.synchronize()
            wq_dev = lkw["class_weight_q"]
            appenders = []
            for i in range(n_app):
                ap = dsk.make_appender(lcomp, K, V, lkw["token_ids"], lkw["delim_ids"], wq_dev, C_=int(wl.C[0]),
                                       delta=int(wl.delta[0]), alpha_num=cfg.a_num, alpha_den=cfg.a_den, b=cfg.b)
                ap.args.len_old, ap.args.len_new = L0 + i, L0 + i + 1
                appenders.append(ap)
            hint = nblk + 8                                  # the grown table ends at the full table's size
            lsel = [dsk.make_select_args(lcomp, queries[0], cfg.T, max_blocks_used=hint)]
            for i in range(1, nq):
                lsel.append(dsk.make_select_args(lcomp, queries[i], cfg.T, out=lsel[0], max_blocks_used=hint))
            latt = [dsk.make_attn_args(queries[0], K, V, lsel[0].sel_start, lsel[0].sel_len, lsel[0].sel_count, cfg.b)]
            for i in range(1, nq):
                latt.append(dsk.make_attn_args(queries[i], K, V, lsel[0].sel_start, lsel[0].sel_len,
                                               lsel[0].sel_count, cfg.b, out=latt[0]))
            g_loop = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_loop, stream=stream):   # capture runs nothing: the table stays at L0
                for i in range(n_app):
                    dsk.dsk_append_tokens(appenders[i].args, stream)
                    dsk.dsk_select_topk(lsel[i % nq].args, stream)
                    dsk.dsk_sparse_decode_attn(latt[i % nq].args, stream)
            loop_us = event_ms(g_loop.replay, stream) * 1e3 / n_app      # one replay: L0 -> L
            stream.synchronize()
            ok = int(lcomp.dev_status.item()) == 0 and int(lcomp.cu_blocks.cpu()[1]) == nblk and \
                torch.equal(lcomp.block_start[: nblk + 1], comp.block_start[: nblk + 1]) and \
                torch.equal(lcomp.ksum[:, :nblk], comp.ksum[:, :nblk])
            loop = {"steps": n_app, "us_per_step": round(loop_us, 3),
                    "append_us": round(loop_us - us_per_step, 3),
                    "grown_table_equals_full_compress": bool(ok)}

        # ---- the same loop for a batch: every sequence owns a region of the tables with room to
        #      grow, and one dsk_append_tokens_batch call per step appends a token to each. ------------
        if cfg.B > 1 and args.append_steps > 0:
            n_app = int(min(args.append_steps, 128, int(wl.seqlens.min()) // 2))
            full = [int(x) for x in wl.seqlens]
            row0, r = [], 0
            for s_ in range(cfg.B):
                row0.append(r)
                r += (full[s_] + 15) // 16 * 16
            Kr = torch.zeros(K.shape[0], r, K.shape[2], dtype=K.dtype, device=dev)
            Vr = torch.zeros_like(Kr)
            tokr = torch.zeros(r, dtype=torch.int32, device=dev)
            for s_ in range(cfg.B):
                a0 = int(wl.cu_seqlens[s_])
                Kr[:, row0[s_]: row0[s_] + full[s_]] = K[:, a0: a0 + full[s_]]
                Vr[:, row0[s_]: row0[s_] + full[s_]] = V[:, a0: a0 + full[s_]]
                tokr[row0[s_]: row0[s_] + full[s_]] = ckw["token_ids"][a0: a0 + full[s_]]
            Cs, Ds = [int(x) for x in wl.C], [int(x) for x in wl.delta]
            entries = [dsk.dsk_block_capacity(full[s_], 1, Cs[s_] - Ds[s_]) + 1 for s_ in range(cfg.B)]
            rkw = dict(seq_row0=row0, region_entries=entries, Hq=cfg.Hq, K=Kr, V=Vr, token_ids=tokr,
                       delim_ids=ckw["delim_ids"], class_weight_q=ckw["class_weight_q"], C_per_seq=Cs,
                       delta_per_seq=Ds, alpha_num=cfg.a_num, alpha_den=cfg.a_den, b=cfg.b)
            with torch.cuda.stream(stream):
                rb = dsk.compress_regions(seq_len=[x - n_app for x in full], stream=stream, **rkw)
                rb_full = dsk.compress_regions(seq_len=full, stream=stream, **rkw)
            stream.synchronize()
            bap = dsk.make_batch_appender(rb, Kr, Vr, tokr, ckw["delim_ids"], ckw["class_weight_q"], C_=max(Cs),
                                          delta=max(Ds), C_per_seq=i32(Cs), delta_per_seq=i32(Ds),
                                          alpha_num=cfg.a_num, alpha_den=cfg.a_den, max_new_tokens=1, lockstep=True)
            used_bound = int(rb.cu_blocks[-1].item())
            # host-known bound on the blocks of one sequence: its count after the compression, read
            # back once, plus what the appended tokens can add
            seq_bound = int(rb.blocks_used.max().item()) + n_app + 8
            bkw = dict(max_blocks_used=used_bound, max_blocks_per_seq=seq_bound)
            bsel = [dsk.make_select_args(rb, queries[0], cfg.T, **bkw)]
            for i in range(1, nq):
                bsel.append(dsk.make_select_args(rb, queries[i], cfg.T, out=bsel[0], **bkw))
            batt = [dsk.make_attn_args(queries[0], Kr, Vr, bsel[0].sel_start, bsel[0].sel_len, bsel[0].sel_count, cfg.b)]
            for i in range(1, nq):
                batt.append(dsk.make_attn_args(queries[i], Kr, Vr, bsel[0].sel_start, bsel[0].sel_len,
                                               bsel[0].sel_count, cfg.b, out=batt[0]))
            g_b = torch.cuda.CUDAGraph()
            g_b0 = torch.cuda.CUDAGraph()
            with torch.cuda.stream(stream):
                with torch.cuda.graph(g_b0, stream=stream):  # the decode step alone on these tables
                    for i in range(n_app):
                        dsk.dsk_select_topk(bsel[i % nq].args, stream)
                        dsk.dsk_sparse_decode_attn(batt[i % nq].args, stream)
                base_us = event_ms(g_b0.replay, stream) * 1e3 / n_app
                with torch.cuda.graph(g_b, stream=stream):   # capture runs nothing: the tables stay where they are
                    for i in range(n_app):
                        dsk.dsk_append_tokens_batch(bap.args, stream)
                        dsk.dsk_select_topk(bsel[i % nq].args, stream)
                        dsk.dsk_sparse_decode_attn(batt[i % nq].args, stream)
                loop_us = event_ms(g_b.replay, stream) * 1e3 / n_app
            stream.synchronize()
            ok = int(rb.dev_status.item()) == 0 and torch.equal(rb.blocks_used, rb_full.blocks_used) and \
                torch.equal(rb.seq_len, rb_full.seq_len)
            used = rb_full.blocks_used.cpu().numpy()
            cub = rb_full.cu_blocks.cpu().numpy()
            for s_ in range(cfg.B):
                a0, n_ = int(cub[s_]), int(used[s_])
                ok = ok and torch.equal(rb.block_start[a0: a0 + n_ + 1], rb_full.block_start[a0: a0 + n_ + 1]) and \
                    torch.equal(rb.slot_base[a0: a0 + n_ + 1], rb_full.slot_base[a0: a0 + n_ + 1]) and \
                    torch.equal(rb.ksum[:, a0: a0 + n_], rb_full.ksum[:, a0: a0 + n_])
            loop = {"steps": n_app, "us_per_step": round(loop_us, 3),
                    "us_per_step_without_append": round(base_us, 3),
                    "append_us": round(loop_us - base_us, 3),
                    "grown_table_equals_full_compress": bool(ok),
                    "layout": "one region of the tables per sequence; dsk_append_tokens_batch appends a token to "
                              "each of the %d sequences per step" % cfg.B}
            del Kr, Vr, rb, rb_full, g_b, g_b0
            torch.cuda.empty_cache()

        # ---- KV reuse with the slot map (App. B.2): K/V live in pinned host memory, every (sequence,
        #      head) keeps its last selection in a resident buffer, and a step loads only the slots
        #      it does not hold.  Queries drift (AR(1)), so consecutive selections overlap. -------------
        reuse = None
        kv_bytes = 2 * K.numel() * 2
        if args.reuse_steps > 0 and kv_bytes <= (8 << 30):
            from workloads import make_drifting_queries
            n_r = args.reuse_steps
            dq = make_drifting_queries(np.random.default_rng(20260203), n_r + 1, cfg.B, cfg.Hq, cfg.D, args.reuse_rho)
            dqs = [bf16(dq[i]) for i in range(n_r + 1)]
            Kh = torch.empty(K.shape, dtype=torch.bfloat16, pin_memory=True)
            Vh = torch.empty(V.shape, dtype=torch.bfloat16, pin_memory=True)
            Kh.copy_(K)
            Vh.copy_(V)
            torch.cuda.synchronize()
            rsel = [dsk.make_select_args(comp, dqs[0], cfg.T, max_blocks_used=nblk, max_blocks_per_seq=nblk_seq)]
            for i in range(1, n_r + 1):
                rsel.append(dsk.make_select_args(comp, dqs[i], cfg.T, out=rsel[0], max_blocks_used=nblk,
                                                 max_blocks_per_seq=nblk_seq))
            r_per_step = torch.zeros(n_r + 1, cfg.B, dtype=torch.int32, device=dev)
            loads_per_step = torch.zeros(n_r + 1, cfg.B, cfg.Hq, dtype=torch.int32, device=dev)

            def reuse_variant(Ksrc, Vsrc, rsel=rsel):
                ru = dsk.make_reuser(rsel[0], Ksrc, Vsrc, cfg.Hkv)
                rargs = []
                loads_per_step.zero_()
                for i in range(n_r + 1):
                    a = type(ru.args).from_buffer_copy(ru.args)
                    a.reuse_count = r_per_step[i].data_ptr()
                    a.load_count = loads_per_step[i].data_ptr()      # [B, heads of the selection] of a [B, Hq] row
                    rargs.append(a)
                ratt = [ru.attn_args(dqs[0])]
                for i in range(1, n_r + 1):
                    ratt.append(ru.attn_args(dqs[i], out=ratt[0]))

                def rstep(i):
                    dsk.dsk_select_topk(rsel[i].args, stream)
                    dsk.dsk_reuse_update(rargs[i], stream)
                    dsk.dsk_sparse_decode_attn(ratt[i].args, stream)

                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream):
                    for i in range(1, n_r + 1):
                        rstep(i)
                us = []
                for _ in range(2):                       # same work both times: the buffer restarts empty
                    ru.res_slot.fill_(-1)
                    ru.res_len.zero_()
                    stream.wait_stream(torch.cuda.current_stream())
                    rstep(0)                             # untimed: fills the empty buffer
                    us.append(event_ms(g.replay, stream) * 1e3 / n_r)
                stream.synchronize()
                return us[-1], (ru, rargs, ratt, g)

            host_us, keep_h = reuse_variant(Kh, Vh)
            mean_r = float(r_per_step[1:].float().mean().item())
            mean_loads = float(loads_per_step[1:].float().sum(dim=(1, 2)).mean().item())
            hbm_us, keep_d = reuse_variant(K, V)
            shared_host = None
            if cfg.G > 1 and not args.no_shared_selection:
                rsel_sh = [dsk.make_select_args(comp, dqs[0], cfg.T, max_blocks_used=nblk, max_blocks_per_seq=nblk_seq,
                                                shared=True)]
                for i in range(1, n_r + 1):
                    rsel_sh.append(dsk.make_select_args(comp, dqs[i], cfg.T, out=rsel_sh[0], max_blocks_used=nblk,
                                                        max_blocks_per_seq=nblk_seq, shared=True))
                sh_us, keep_s = reuse_variant(Kh, Vh, rsel_sh)
                shared_host = {"us": round(sh_us, 2),
                               "mean_reused_slots_per_head": round(float(r_per_step[1:].float().mean().item()), 1),
                               "slots_loaded_per_step": round(float(loads_per_step[1:].float().sum(dim=(1, 2)).mean().item()), 1)}
                del keep_s
            # without reuse: the attention gathers every selected slot from host memory, every step
            natt = [dsk.make_attn_args(dqs[i], Kh, Vh, rsel[0].sel_start, rsel[0].sel_len, rsel[0].sel_count, cfg.b,
                                       out=atts[0]) for i in range(n_r + 1)]
            g_nr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g_nr, stream=stream):
                for i in range(1, n_r + 1):
                    dsk.dsk_select_topk(rsel[i].args, stream)
                    dsk.dsk_sparse_decode_attn(natt[i].args, stream)
            noreuse_us = replay_us(g_nr, stream, n_r, args.replays)[0]
            # full attention with K/V in host memory: every byte of the cache crosses the link
            hd = dsk.make_dense_attn_args(dqs[0], Kh, Vh, cu, int(wl.seqlens.max()))
            dsk.dsk_dense_decode_attn(hd.args, stream)
            dense_host_us = event_ms(lambda: [dsk.dsk_dense_decode_attn(hd.args, stream) for _ in range(2)], stream) * 1e3 / 2
            tok_per_slot = mean_sel_tokens / max(1, cfg.B * cfg.Hq * cfg.k)
            load_bytes = mean_loads * tok_per_slot * 512
            reuse = {"steps": n_r, "rho": args.reuse_rho, "k": cfg.k,
                     "mean_reused_slots_per_head": round(mean_r, 1),
                     "slots_loaded_per_step": round(mean_loads, 1),
                     "link_bytes_per_step": int(load_bytes),
                     "host_kv_with_reuse_us": round(host_us, 2),
                     "host_kv_with_reuse_link_GBps": round(load_bytes / (host_us * 1e-6) / 1e9, 1),
                     "host_kv_without_reuse_us": round(noreuse_us, 2),
                     "host_kv_full_attention_us": round(dense_host_us, 1),
                     "hbm_kv_with_reuse_us": round(hbm_us, 2),
                     "host_kv_with_reuse_shared_selection_extension": shared_host,
                     "speedup_reuse_vs_no_reuse": round(noreuse_us / host_us, 2),
                     "speedup_reuse_vs_full_attention_host": round(dense_host_us / host_us, 1),
                     "what": "select + dsk_reuse_update + attention over the resident buffers; K/V source in "
                             "pinned host memory read in place by the kernels"}
            del keep_h, keep_d, g_nr, natt, hd, Kh, Vh
    torch.cuda.synchronize()

    attn_gbs = bytes_attn / (gather_us * 1e-6) / 1e9
    traffic = MEASURED_TRAFFIC_BYTES.get(cfg.name, {}).get("attn_kernel")
    step_gbs = step_bytes / (us_per_step * 1e-6) / 1e9
    out = {
        "metric": "decode attn \u00b5s/step + achieved HBM GB/s at 128K ctx (Llama-3-8B shape)",
        "value": round(us_per_step, 3),
        "unit": "us/step",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(us_per_step / 1e3, 6),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16 in, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": cfg.name, "context": int(wl.total_tokens), "Hq": cfg.Hq, "Hkv": cfg.Hkv, "b": cfg.b,
                   "budget": cfg.T, "blocks": nblk, "slots": nslots, "queries": nq,
                   "selection": "per query head",
                   "timing": "HIP graph of %d steps, median of %d replays" % (args.steps, args.replays)},
        "achieved_GBps": round(step_gbs, 1),
        "step_bytes": int(step_bytes),
        "eager_us_per_step": round(eager_us, 3),
        "select_us": round(select_us, 3),
        "attn_us": round(attn_us, 3),
        "compress": {"us": round(compress_ms * 1e3, 2), "bytes": int(compress_bytes),
                     "GBps": round(compress_bytes / (compress_ms * 1e-3) / 1e9, 1),
                     "frac_of_hbm_peak": round(compress_bytes / (compress_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                     "stages": "candidates+segment+summaries(K)",
                     "us_without_candidate_lists": round(compress_lean_ms * 1e3, 2),
                     "importance_us": round(importance_us, 1), "importance_samples": n_samples},
        # the dominant kernel, priced where the metric lives: what it adds to a decode step, from HIP
        # events on the kernels' stream: median time of the graph "selection + gather" minus that of
        # the graph "selection".  The difference holds the kernel, the dependency gap in front of it
        # and what its cache traffic costs the selection that follows (the summaries it evicts), so it
        # is an upper bound of the kernel's own in-step duration (the kernel trace under profiles/ has
        # that).  Events around a single launch inside a step were tried and dropped: a pair of event
        # markers with nothing between them already measures 5 us.  The figure for the kernel launched
        # back to back on independent selections is kept beside it as `isolated_*`.
        "roofline": {"bound": "hbm", "kernel": "attn_kernel (K/V gather + online softmax of dsk_sparse_decode_attn)",
                     "achieved": round(bytes_attn / (gather_in_step_us * 1e-6) / 1e9, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s",
                     "frac": round(bytes_attn / (gather_in_step_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                     "traffic": traffic,
                     "traffic_frac": None if traffic is None else
                     round(traffic / (gather_in_step_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                     "bytes_per_launch": int(bytes_attn), "us_per_launch": round(gather_in_step_us, 3),
                     "measured": "inside a decode step: graph(select + gather) - graph(select), medians of %d replays"
                                 % args.replays,
                     "isolated_us_per_launch": round(gather_us, 3),
                     "isolated_frac": round(attn_gbs / HBM_PEAK_GBS, 4),
                     "same_rows_us_per_launch": round(gather_same_rows_us, 3),
                     "same_rows_frac": round(bytes_attn / (gather_same_rows_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                     "attn_call_us": round(attn_us, 3),
                     "attn_call_frac": round(bytes_attn / (attn_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                     "step_frac": round(step_gbs / HBM_PEAK_GBS, 4),
                     "step_target": "decode step at >= 70 %% of the HBM roofline = %.1f us; measured %.1f us: not reached"
                                    % (step_bytes / (0.7 * HBM_PEAK_GBS * 1e3), us_per_step)
                     if step_gbs / HBM_PEAK_GBS < 0.7 else "decode step at >= 70 % of the HBM roofline: reached"},
        "step_us_replays": step_samples,
        "workload_gen_s": round(gen_s, 1),
    }
    out["dense_baseline"] = {"us": round(dense_us, 2), "bytes": int(dense_bytes),
                             "GBps": round(dense_bytes / (dense_us * 1e-6) / 1e9, 1),
                             "frac_of_hbm_peak": round(dense_bytes / (dense_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                             "speedup_of_sparse_step": round(dense_us / us_per_step, 2),
                             "what": "dsk_dense_decode_attn, full attention over the whole cache, same queries"}
    if stream_read_gbs is not None:
        out["stream_read"] = {"GBps": round(stream_read_gbs, 1), "mib": args.stream_read_mib,
                              "gather_frac_of_stream_read": round(attn_gbs / stream_read_gbs, 4),
                              "compress_frac_of_stream_read":
                                  round(compress_bytes / (compress_ms * 1e-3) / 1e9 / stream_read_gbs, 4)}
    if cold is not None:
        out["cold"] = cold
    if loop is not None:
        out["decode_loop_with_append"] = loop
    if reuse is not None:
        out["kv_reuse"] = reuse
    if shared is not None:
        out["shared_selection_extension"] = shared
    if not args.no_parity:
        out["parity"] = parity_summary(dsk, wl, comp, nblk, q_bits, queries, K, V)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, comp, nblk, q_bits)
    print(json.dumps(out))


def parity_summary(dsk, wl, comp, nblk, q_bits, queries, K, V, n_queries=2, n_heads=4):
    """Outside every timed region: the GPU results of this workload against the fp64 oracle.
    Segmentation of every sequence (block boundaries and slot bases, bit for bit), then for the
    first queries and a sample of (sequence, head) pairs: the selected slot set (a slot that differs
    counts as swapped when its block's oracle score is within 1e-4 of the threshold score, and as a
    mismatch otherwise) and the attention output over the GPU's own selection."""
    import numpy as np
    import torch

    from oracle import dynsplit_oracle as O
    cfg = wl.cfg
    bs_g = comp.block_start.cpu().numpy().astype(np.int64)
    sb_g = comp.slot_base.cpu().numpy().astype(np.int64)
    cub = comp.cu_blocks.cpu().numpy().astype(np.int64)
    boundary_mismatches = 0
    blocks_checked = 0
    seqs = list(range(cfg.B)) if cfg.B <= 2 else [0, cfg.B // 2, cfg.B - 1]
    for s in range(cfg.B):
        lo, hi = int(wl.cu_seqlens[s]), int(wl.cu_seqlens[s + 1])
        pos, cls = O.extract_candidates(wl.token_ids[lo:hi], wl.delim_ids)
        bs = O.dd_select(hi - lo, pos, cls, wl.class_weight_q[s], int(wl.C[s]), int(wl.delta[s]), cfg.a_num, cfg.a_den)
        sb = O.slot_map(bs, cfg.b)
        b0, b1 = int(cub[s]), int(cub[s + 1])
        blocks_checked += len(bs) - 1
        if b1 - b0 != len(bs) - 1:
            boundary_mismatches += abs((b1 - b0) - (len(bs) - 1)) + 1
            continue
        boundary_mismatches += int((bs_g[b0: b1 + 1] - lo != bs).sum())
        boundary_mismatches += int((sb_g[b0: b1 + 1] - sb_g[b0] != sb).sum())
    sums = comp.ksum[:, :nblk].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    heads = sorted(h for h in {0, cfg.G, cfg.Hq // 2 + 1, cfg.Hq - 1} if h < cfg.Hq)[:n_heads]
    swapped = mismatched = pairs = 0
    worst_attn = worst_lse = worst_score = 0.0
    scale = 1.0 / np.sqrt(128.0)
    for qi in range(min(n_queries, len(queries))):
        sel = dsk.select_topk(comp, queries[qi], cfg.T, want_scores=True, max_blocks_used=nblk)
        att = dsk.sparse_decode_attn(queries[qi], K, V, sel.sel_start, sel.sel_len, sel.sel_count, cfg.b)
        torch.cuda.synchronize()
        g_slot, g_cnt = sel.sel_slot.cpu().numpy(), sel.sel_count.cpu().numpy()
        g_start, g_len = sel.sel_start.cpu().numpy(), sel.sel_len.cpu().numpy()
        g_scores = sel.scores.cpu().numpy()
        g_out, g_lse = att.out.cpu().numpy(), att.lse.cpu().numpy()
        for s in seqs:
            b0, b1 = int(cub[s]), int(cub[s + 1])
            if b1 == b0:
                continue
            sb = sb_g[b0: b1 + 1]
            for h in heads:
                hk = h // cfg.G
                qf = O.widen_bf16(q_bits[qi][s, h])
                sc = O.block_scores(qf[None], O.widen_bf16(sums[hk, b0:b1, 0])[None], O.widen_bf16(sums[hk, b0:b1, 1])[None])[0]
                worst_score = max(worst_score, float(np.abs(g_scores[h, b0:b1] - sc).max() / max(np.abs(sc).max(), 1e-30)))
                o_sel, tau = O.select_slots(sc, sb - sb[0], cfg.k)
                cnt = int(g_cnt[s, h])
                gs = set(int(x) - int(sb[0]) for x in g_slot[s, h, :cnt])
                for slot in gs ^ set(int(x) for x in o_sel):
                    i = int(np.searchsorted(sb - sb[0], slot, side="right")) - 1
                    if abs(sc[i] - tau) <= 1e-4 * abs(tau):
                        swapped += 1
                    else:
                        mismatched += 1
                toks = np.concatenate([np.arange(g_start[s, h, j], g_start[s, h, j] + g_len[s, h, j]) for j in range(cnt)])
                o, lse = O.sparse_attention(qf, O.widen_bf16(wl.K[hk][toks]), O.widen_bf16(wl.V[hk][toks]),
                                            np.arange(len(toks)), scale)
                worst_attn = max(worst_attn, float(np.abs(g_out[s, h] - o).max() / max(np.abs(o).max(), 1e-30)))
                worst_lse = max(worst_lse, abs(float(g_lse[s, h]) - lse))
                pairs += 1
    return {"boundary_mismatches": int(boundary_mismatches), "blocks_checked": int(blocks_checked),
            "selection_mismatches": int(mismatched), "swapped_selections_near_tie": int(swapped) // 2,
            "max_score_rel_err": float("%.3g" % worst_score),
            "max_attention_rel_err": float("%.3g" % worst_attn), "max_lse_abs_err": float("%.3g" % worst_lse),
            "checked": "%d (query, sequence, head) cases: heads %s of sequences %s, first %d queries; all %d sequences' "
                       "segmentation" % (pairs, heads, seqs, min(n_queries, len(queries)), cfg.B),
            "bar": "boundaries exact; selections exact except near ties (1e-4 rel. of the threshold score); "
                   "attention <= 2e-3 max rel. err., lse <= 1e-3"}


def cpu_baseline(wl, comp, nblk, q_bits):
    """The fp64 oracle, as it stands, timed on this machine's host cores on a bounded sample:
    decode steps (scores + slot top-k + attention over the selection) for all query heads of
    the first queries of the workload, on the GPU-produced (parity-tested) block table and
    summaries.  BLAS/OpenMP pools are limited to one thread so the thread count is known."""
    import numpy as np
    from threadpoolctl import threadpool_limits

    from oracle import dynsplit_oracle as O
    cfg = wl.cfg
    bs = comp.block_start.cpu().numpy()[: nblk + 1].astype(np.int64)
    sb = comp.slot_base.cpu().numpy()[: nblk + 1].astype(np.int64)
    sums = comp.ksum[:, :nblk].contiguous().view(__import__("torch").int16).cpu().numpy().view(np.uint16)
    scale = 1.0 / np.sqrt(128.0)
    budget_s, n_done, t_spent = 12.0, 0, 0.0
    with threadpool_limits(limits=1):
        kmin = O.widen_bf16(sums[:, :, 0])
        kmax = O.widen_bf16(sums[:, :, 1])
        while n_done < len(q_bits) and t_spent < budget_s:
            qb = q_bits[n_done]
            t0 = time.perf_counter()
            for s in range(cfg.B):
                b0, b1 = int(comp.cu_blocks.cpu()[s]), int(comp.cu_blocks.cpu()[s + 1])
                qf = O.widen_bf16(qb[s])
                sc = O.block_scores(qf, kmin[:, b0:b1], kmax[:, b0:b1])
                for h in range(cfg.Hq):
                    sel, _ = O.select_slots(sc[h], sb[b0: b1 + 1] - sb[b0], cfg.k)
                    toks = O.selected_tokens(sel, bs[b0: b1 + 1], sb[b0: b1 + 1] - sb[b0], cfg.b)
                    hk = h // cfg.G
                    O.sparse_attention(qf[h], O.widen_bf16(wl.K[hk][toks]), O.widen_bf16(wl.V[hk][toks]),
                                       np.arange(len(toks)), scale)
            t_spent += time.perf_counter() - t0
            n_done += 1
        # the compression pass the bench times on the GPU (candidates, segmentation, slot map,
        # K summaries), on the first sequence and at most two KV heads of summaries
        lo, hi = int(wl.cu_seqlens[0]), int(wl.cu_seqlens[1])
        n_heads = min(2, cfg.Hkv)
        t0 = time.perf_counter()
        pos, cls = O.extract_candidates(wl.token_ids[lo:hi], wl.delim_ids)
        bs0 = O.dd_select(hi - lo, pos, cls, wl.class_weight_q[0], int(wl.C[0]), int(wl.delta[0]), cfg.a_num, cfg.a_den)
        O.slot_map(bs0, cfg.b)
        t_seg = time.perf_counter() - t0
        t0 = time.perf_counter()
        O.block_summaries(O.widen_bf16(wl.K[:n_heads, lo:hi]), bs0)
        t_sum = (time.perf_counter() - t0) / n_heads * cfg.Hkv        # scaled to all KV heads
    return {"value": round(t_spent / n_done * 1e6, 1), "unit": "us/step", "cores": 1, "kind": "oracle",
            "sample": "%d full decode steps (scores + slot top-k + attention, all %d query heads) of %s"
                      % (n_done, cfg.Hq, cfg.name),
            "compress_us": round((t_seg + t_sum) * 1e6, 1),
            "compress_sample": "sequence 0 (%d tokens): candidates + DD-Select + slot map, and K summaries of %d "
                               "of %d KV heads scaled to all" % (hi - lo, n_heads, cfg.Hkv)}


if __name__ == "__main__":
    main()
