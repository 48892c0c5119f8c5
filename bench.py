#!/usr/bin/env python3
"""Benchmark of the ISD-step hot path on one MI355X.

One "step" = one idlm_isd_attention call (one layer's paged stride attention) plus one
idlm_isd_accept call (introspective acceptance over the step's logits) on the large-
concurrency serving workload (B=256, S=16; `serve256`), inputs resident in HBM.  Prints ONE
JSON line: whole-step throughput in stride positions (tokens verified + proposed) per second,
the roofline record of the dominant kernel (timed with HIP events that the library records
around each of its kernels, on the stream they run on), the CPU oracle timed on the same
workload on this machine's host cores, and a `configs` block with the per-kernel times of the
other workloads (small, 8b, the long-context stride sweep).

  python bench.py                                  the default line (everything)
  python bench.py --sections step,probe            only the timed step, its kernels and the streaming probes (profiling runs)
  python bench.py --workload long32k --stride 16 --sections step
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16, published
MIN_KERNEL_SAMPLES = 24         # launches timed with events per kernel
CACHE_BYTES = 256 << 20         # memory-side cache: smaller working sets are rotated over several copies
ROOT = os.path.dirname(os.path.abspath(__file__))
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_counters.txt")


class HipEvents:
    """Minimal HIP event access (create / elapsed time) through libamdhip64."""

    def __init__(self):
        self.hip = C.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.hip.hipEventDestroy.argtypes = [C.c_void_p]

    def create(self, n):
        out = []
        for _ in range(n):
            e = C.c_void_p()
            rc = self.hip.hipEventCreate(C.byref(e))
            if rc != 0:
                raise RuntimeError("hipEventCreate failed: %d" % rc)
            out.append(e.value)
        return out

    def elapsed_ms(self, a, b):
        ms = C.c_float()
        rc = self.hip.hipEventElapsedTime(C.byref(ms), C.c_void_p(a), C.c_void_p(b))
        if rc != 0:
            raise RuntimeError("hipEventElapsedTime failed: %d" % rc)
        return float(ms.value)

    def destroy(self, evs):
        for e in evs:
            self.hip.hipEventDestroy(C.c_void_p(e))


def measured_traffic(workload, kernel, lib_version):
    """HBM bytes per launch of `kernel` on `workload` from the committed counter summary
    (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a copy of known size), or None when the
    file has no line for this library version: a stale figure is never reported."""
    try:
        lines = open(TRAFFIC_FILE).read().splitlines()
    except OSError:
        return None
    for ln in lines:
        f = ln.split()
        if len(f) >= 4 and not ln.startswith("#") and f[0] == workload and f[1] == kernel:
            kv = dict(x.split("=", 1) for x in f[2:] if "=" in x)
            if int(kv.get("lib_version", -1)) == lib_version:
                return int(kv["bytes"])
    return None


def attention_algorithmic_bytes(ctx_lens, cfg):
    """One read of every context token's K and V rows, Q in, O out, and the block table."""
    esz = 2 if cfg.dtype == "bf16" else 4
    kv = int(ctx_lens.sum()) * cfg.Hkv * cfg.D * esz * 2
    qo = cfg.B * 2 * cfg.S * cfg.Hq * cfg.D * esz
    table = int(((ctx_lens + cfg.P - 1) // cfg.P).sum()) * 4
    return kv + qo + table


def attention_flops(ctx_lens, cfg):
    """2 contractions x 2 flop x D per (query row, head, visible key)."""
    c = ctx_lens.astype(np.int64)
    vis = int((cfg.S * (c - cfg.S) + cfg.S * (cfg.S + 1) // 2).sum())
    return 4 * cfg.D * cfg.Hq * vis


class Case:
    """One workload resident in HBM, in `copies` identical copies at different addresses (launches
    rotate over them so that a working set smaller than the memory-side cache is read cold)."""

    def __init__(self, cfg, dev, copies=1, kop=True, workgroups=0):
        import torch
        import paper_2604_11035_amd as idlm
        from isd_inputs import k_pages_in_operand_order, make_accept_inputs, make_attention_inputs
        self.cfg, self.idlm, self.torch = cfg, idlm, torch
        self.workgroups = workgroups
        att = make_attention_inputs(cfg, device=dev)
        acc = make_accept_inputs(cfg, device=dev)
        self.att, self.acc = att, acc
        B, S, V = cfg.B, cfg.S, cfg.V
        self.kop = bool(kop) and cfg.dtype == "bf16" and cfg.D == 128
        k_gpu = k_pages_in_operand_order(att.k_cache) if self.kop else att.k_cache
        drafts = acc.draft_tokens[:, :S - 1].contiguous() if S > 1 else None
        dcode = 1 if cfg.dtype == "bf16" else 0
        max_pages = att.block_table.shape[1]
        self.ws_att = torch.empty(max(256, idlm.idlm_isd_attention_workspace(B, S, cfg.Hq, cfg.Hkv, cfg.D, cfg.P, max_pages,
                                                                             dcode, workgroups)),
                                  dtype=torch.uint8, device=dev)
        self.ws_acc = torch.empty(max(256, idlm.idlm_isd_accept_workspace(B, S, V)), dtype=torch.uint8, device=dev)
        self.accept_len = torch.empty(B, dtype=torch.int32, device=dev)
        self.new_tokens = torch.empty(B, S, dtype=torch.int32, device=dev)
        self.draft_probs = torch.empty(B, max(S - 1, 1), dtype=torch.float32, device=dev)
        self.drafts = drafts
        self.k_gpu = k_gpu
        self.out = torch.empty_like(att.q)
        self.sets = [(att.q, k_gpu, att.v_cache, acc.logits, self.out)]
        for _ in range(copies - 1):
            self.sets.append((att.q.clone(), k_gpu.clone(), att.v_cache.clone(), acc.logits.clone(), torch.empty_like(att.q)))
        self.ctx_np = att.ctx_lens.cpu().numpy().astype(np.int64)

    def working_set_bytes(self):
        q, k, v, lg, out = self.sets[0]
        return sum(t.numel() * t.element_size() for t in (q, k, v, lg, out))

    def step(self, i, stream, ev_att=None, ev_acc=None):
        cfg, att, acc, idlm = self.cfg, self.att, self.acc, self.idlm
        q, k, v, lg, out = self.sets[i % len(self.sets)]
        idlm.idlm_isd_attention(q, k, v, att.block_table, att.ctx_lens, cfg.S, out, num_workgroups=self.workgroups,
                                workspace=self.ws_att, stream=stream, events=ev_att, k_operand_order=self.kop)
        idlm.idlm_isd_accept(lg, self.drafts, acc.rng_seed, self.accept_len, self.new_tokens, n_draft=acc.n_draft,
                             greedy=acc.greedy, rng_offset=i, draft_probs=self.draft_probs if cfg.S > 1 else None,
                             workspace=self.ws_acc, stream=stream, events=ev_acc)


def copies_for(cfg_bytes):
    """Copies needed so that consecutive launches never find their inputs in the memory-side cache."""
    if cfg_bytes >= 4 * CACHE_BYTES:
        return 1
    return int(min(16, max(2, -(-3 * CACHE_BYTES // max(cfg_bytes, 1)))))


def stats_of(samples):
    v = sorted(samples)
    return {"ms": sum(v) / len(v), "min_ms": v[0], "median_ms": v[len(v) // 2], "max_ms": v[-1], "samples": len(v)}


def attention_kernel_name(cfg):
    """The kernel idlm_isd_attention launches for this configuration (bf16: more than 64 query rows per KV head with
    128-wide heads go to the kernel that shares the K/V tiles of a workgroup through LDS)."""
    if cfg.dtype != "bf16":
        return "isd_attention_f32_kernel"
    return "isd_attention_shared_kernel" if cfg.D == 128 and cfg.S * (cfg.Hq // cfg.Hkv) > 64 else "isd_attention_bf16_kernel"


def kernel_record(case, hev, events):
    """Per-kernel figures from the hooked launches: events = [(attention events, accept events), ...]."""
    cfg = case.cfg
    t = {name: stats_of([hev.elapsed_ms(e[w][a], e[w][b]) for e in events])
         for name, (w, a, b) in {"attention": (0, 0, 1), "merge": (0, 1, 2), "row_stats": (1, 0, 1), "tail": (1, 1, 2)}.items()}
    att_bytes = attention_algorithmic_bytes(case.ctx_np, cfg)
    att_flops = attention_flops(case.ctx_np, cfg)
    acc_bytes = cfg.B * cfg.S * cfg.V * 4
    a, r = t["attention"], t["row_stats"]
    kernels = {
        attention_kernel_name(cfg): dict(
            a, algorithmic_bytes=att_bytes, GBps=att_bytes / a["ms"] / 1e6, frac_hbm=att_bytes / a["ms"] / 1e6 / HBM_PEAK_GBS,
            TFLOPs=att_flops / a["ms"] / 1e9, frac_mfma=att_flops / a["ms"] / 1e9 / MFMA_BF16_PEAK_TFLOPS),
        "isd_attention_merge_kernel": {"ms": t["merge"]["ms"]},
        "isd_row_stats_kernel": dict(r, algorithmic_bytes=acc_bytes, GBps=acc_bytes / r["ms"] / 1e6,
                                     frac_hbm=acc_bytes / r["ms"] / 1e6 / HBM_PEAK_GBS),
        "isd_accept_chain+sample+emit_kernels": {"ms": t["tail"]["ms"]},
    }
    return kernels


def hooked_launches(case, hev, stream, n, first_index):
    torch = case.torch
    events = [(hev.create(3), hev.create(3)) for _ in range(n)]
    for j, (ea, eb) in enumerate(events):
        case.step(first_index + j, stream, ea, eb)
    torch.cuda.synchronize()
    return events


def config_line(name, cfg, dev, hev, stream):
    """Compact per-kernel record of one of the other workloads: >= MIN_KERNEL_SAMPLES hooked launches,
    inputs rotated over enough copies that a small working set is read from HBM, not from the cache."""
    import torch
    probe = Case(cfg, dev, copies=1)
    nbytes = probe.working_set_bytes()
    n = copies_for(nbytes)
    case = probe
    if n > 1:
        del probe
        case = Case(cfg, dev, copies=n)
    for i in range(3):
        case.step(i, stream)
    torch.cuda.synchronize()
    ev = hooked_launches(case, hev, stream, MIN_KERNEL_SAMPLES, 3)
    k = kernel_record(case, hev, ev)
    for ea, eb in ev:
        hev.destroy(ea + eb)
    att = next(v for kk, v in k.items() if kk.startswith("isd_attention_") and "merge" not in kk)
    rs = k["isd_row_stats_kernel"]
    rec = {
        "shape": "B=%d S=%d Hq=%d Hkv=%d D=%d V=%d ctx %s [%d,%d]" % (cfg.B, cfg.S, cfg.Hq, cfg.Hkv, cfg.D, cfg.V, cfg.ctx_kind,
                                                                    cfg.ctx_lo or min(cfg.ctx_list or (0,)),
                                                                    cfg.ctx_hi or max(cfg.ctx_list or (0,))),
        "input_copies_rotated": n, "working_set_MB": round(nbytes / 1e6, 1), "samples": att["samples"],
        "attention_ms": att["ms"], "attention_median_ms": att["median_ms"], "attention_frac_hbm": att["frac_hbm"],
        "attention_frac_mfma": att["frac_mfma"], "attention_merge_ms": k["isd_attention_merge_kernel"]["ms"],
        "row_stats_ms": rs["ms"], "row_stats_median_ms": rs["median_ms"], "row_stats_frac_hbm": rs["frac_hbm"],
        "accept_tail_ms": k["isd_accept_chain+sample+emit_kernels"]["ms"],
        "rows_per_kv_head": cfg.S * cfg.G,
    }
    del case
    torch.cuda.empty_cache()
    return rec


def cpu_baseline(att, acc, cfg, n_seq, threads=0):
    """Times the oracle (as it stands) on the first n_seq sequences of the workload."""
    import torch
    import oracle
    if threads > 0:
        oracle.set_num_threads(threads)
    from isd_inputs import to_numpy

    ctx = att.ctx_lens[:n_seq].cpu().numpy()
    pages = (ctx + cfg.P - 1) // cfg.P
    # compact the sample's pages into a small pool (pure data movement)
    ids = torch.cat([att.block_table[b, :int(pages[b])] for b in range(n_seq)]).long()
    k_small = att.k_cache.index_select(0, ids)
    v_small = att.v_cache.index_select(0, ids)
    table = np.full((n_seq, int(pages.max())), -1, dtype=np.int32)
    off = 0
    for b in range(n_seq):
        table[b, :pages[b]] = np.arange(off, off + pages[b])
        off += pages[b]
    q = to_numpy(att.q[:n_seq])
    k_np, v_np = to_numpy(k_small), to_numpy(v_small)
    logits = to_numpy(acc.logits[:n_seq])
    drafts = to_numpy(acc.draft_tokens[:n_seq])[:, :cfg.S - 1]
    nd = to_numpy(acc.n_draft[:n_seq])
    gr = to_numpy(acc.greedy[:n_seq])
    oracle.lib()
    t0 = time.perf_counter()
    oracle.attention(q, k_np, v_np, table, ctx, cfg.S, Hq=cfg.Hq, Hkv=cfg.Hkv, D=cfg.D, P=cfg.P)
    t1 = time.perf_counter()
    oracle.accept(logits, drafts, acc.rng_seed, n_draft=nd, greedy=gr, rng_offset=acc.rng_offset)
    t2 = time.perf_counter()
    return {
        "value": n_seq * cfg.S / (t2 - t0),
        "unit": "tokens/s",
        "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": "first %d of %d sequences of %s (%d context tokens): attention %.2f s, acceptance %.2f s"
                  % (n_seq, cfg.B, cfg.name, int(ctx.sum()), t1 - t0, t2 - t1),
    }


def wavefront_times(case, stream, launches=8):
    """When the wavefronts of the attention main kernel start and finish (the library's debug trace on the device's
    constant 100 MHz clock), summarised over `launches` launches: the launch lasts as long as its slowest wavefront."""
    torch, idlm, cfg, att = case.torch, case.idlm, case.cfg, case.att
    rec = torch.zeros(4096, 4, dtype=torch.int64, device=att.q.device)
    idlm.idlm_isd_attention_wave_trace(rec)
    runs = []
    try:
        for j in range(launches + 2):
            q, k, v, _, out = case.sets[j % len(case.sets)]
            rec.zero_()
            idlm.idlm_isd_attention(q, k, v, att.block_table, att.ctx_lens, cfg.S, out, num_workgroups=case.workgroups,
                                    workspace=case.ws_att, stream=stream, k_operand_order=case.kop)
            torch.cuda.synchronize()
            if j >= 2:
                runs.append(rec.cpu().numpy().copy())
    finally:
        idlm.idlm_isd_attention_wave_trace(None)
    keys = ("launch_us", "start_last_us", "finish_min_us", "finish_p10_us", "finish_median_us", "finish_p90_us",
            "mean_idle_share", "finish_even_xcd_us", "finish_odd_xcd_us", "tiles_min", "tiles_mean", "tiles_max", "parts_mean",
            "us_per_tile_median", "finish_by_parts")
    acc = {k: [] for k in keys}
    for r in runs:
        act = r[:, 1] > 0
        if not act.any():
            continue
        v = np.nonzero(act)[0]
        t0 = r[act, 0].min()
        start = (r[act, 0] - t0) / 100.0
        end = (r[act, 1] - t0) / 100.0
        tiles, parts = r[act, 2].astype(np.float64), r[act, 3]
        xcd = (v // 4) % 8
        acc["launch_us"].append(end.max()); acc["start_last_us"].append(start.max())
        acc["finish_min_us"].append(end.min())
        for name, q_ in (("finish_p10_us", 10), ("finish_median_us", 50), ("finish_p90_us", 90)):
            acc[name].append(np.percentile(end, q_))
        acc["mean_idle_share"].append(1.0 - end.mean() / end.max())
        acc["finish_even_xcd_us"].append(end[xcd % 2 == 0].mean()); acc["finish_odd_xcd_us"].append(end[xcd % 2 == 1].mean())
        acc["tiles_min"].append(tiles.min()); acc["tiles_mean"].append(tiles.mean()); acc["tiles_max"].append(tiles.max())
        acc["parts_mean"].append(parts.mean())
        acc["us_per_tile_median"].append(np.median((end - start) / np.maximum(tiles, 1)))
        acc["finish_by_parts"].append({int(k_): float(end[parts == k_].mean()) for k_ in np.unique(parts)})
    out = {k: float(np.mean(acc[k])) for k in keys if k != "finish_by_parts" and acc[k]}
    by = {}
    for d in acc["finish_by_parts"]:
        for k_, x in d.items():
            by.setdefault(k_, []).append(x)
    out["mean_finish_us_by_sequence_parts"] = {str(k_): float(np.mean(x)) for k_, x in sorted(by.items())}
    out["wavefronts"] = int((runs[-1][:, 1] > 0).sum()) if runs else 0
    out["launches"] = len(runs)
    return out


def stream_probe(idlm, dev):
    """Plain streaming kernels of known size: practical bandwidth ceiling of this device, and the reference
    that hardware byte counters are scaled by in the committed profiles (4 GiB, so that the 256 MB memory-
    side cache holds a negligible part of it from one pass to the next)."""
    import torch
    probe = torch.empty(1 << 32, dtype=torch.uint8, device=dev)
    probe_dst = torch.empty_like(probe)
    sink = torch.zeros(1, dtype=torch.int32, device=dev)

    def timed(fn, n=5):
        fn()
        torch.cuda.synchronize()
        a, b_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(n):
            fn()
        b_.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b_) / n

    t_read = timed(lambda: idlm.idlm_stream_read(probe, sink))
    t_copy = timed(lambda: idlm.idlm_stream_copy(probe, probe_dst))
    return {"read_GBps": probe.numel() / t_read / 1e6, "copy_read_plus_write_GBps": 2 * probe.numel() / t_copy / 1e6,
            "bytes": probe.numel()}


def extras(case, args, hev, stream, dev, ms_per_step):
    """Everything around the step that is reported but not part of `value`."""
    import torch
    idlm, cfg, att, acc = case.idlm, case.cfg, case.att, case.acc
    B, S, V = cfg.B, cfg.S, cfg.V
    kop, k_gpu, drafts, out = case.kop, case.k_gpu, case.drafts, case.out
    accept_len, new_tokens = case.accept_len, case.new_tokens
    res = {}

    def timed(fn, n=5):
        fn()
        torch.cuda.synchronize()
        a, b_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(n):
            fn()
        b_.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b_) / n

    # the same step launched without the timing hooks, and replayed from a captured HIP graph (the
    # calls allocate nothing and never synchronise, so they can be captured as they are)
    cur = torch.cuda.current_stream()
    torch.cuda.synchronize()
    t_plain = timed(lambda: [case.step(args.warmup + i, cur) for i in range(args.steps)], n=1) / args.steps
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        case.step(0, side)
    torch.cuda.synchronize()
    t_graph = timed(lambda: [graph.replay() for _ in range(args.steps)], n=1) / args.steps
    # four steps per graph: what a replay costs per launch of a graph, as against per kernel node
    graph4 = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph4, stream=side):
        for j in range(4):
            case.step(j, side)
    torch.cuda.synchronize()
    n4 = max(1, args.steps // 4)
    t_graph4 = timed(lambda: [graph4.replay() for _ in range(n4)], n=1) / (4 * n4)
    res["launch_modes"] = {"timed_region_ms": ms_per_step, "eager_ms": t_plain, "graph_replay_ms": t_graph,
                           "graph_of_four_steps_replay_ms_per_step": t_graph4}

    # the attention call alone with the K pool in the other page layout (slot-major rows / operand order)
    if cfg.dtype == "bf16" and cfg.D == 128:
        from isd_inputs import k_pages_in_operand_order
        k_other = att.k_cache if kop else k_pages_in_operand_order(att.k_cache)
        t_a, t_b = (timed(lambda: idlm.idlm_isd_attention(att.q, kk, att.v_cache, att.block_table, att.ctx_lens, S, out,
                                                          num_workgroups=args.workgroups, workspace=case.ws_att,
                                                          k_operand_order=flag), n=10)
                    for kk, flag in ((k_gpu, kop), (k_other, not kop)))
        del k_other
        res["k_page_layouts"] = {"attention_call_ms_as_timed": t_a, "attention_call_ms_other_k_page_layout": t_b,
                                 "timed_layout": "operand order" if kop else "slot-major"}

    # the two small kernels between steps (scatter of the stride's K/V rows; trim-and-commit and next
    # stride), timed on the same workload outside the timed region above
    k_new = torch.randn(B, S, cfg.Hkv, cfg.D, device=dev).to(att.q.dtype)
    v_new = torch.randn(B, S, cfg.Hkv, cfg.D, device=dev).to(att.q.dtype)
    t_append = timed(lambda: idlm.idlm_isd_kv_append(k_new, v_new, k_gpu, att.v_cache, att.block_table,
                                                     att.ctx_lens, S, k_operand_order=kop), n=20)
    pages_used = (att.ctx_lens + cfg.P - 1) // cfg.P
    n_steady = max(0, (S - 1) // 2)

    def commit_state():
        return dict(n_draft=acc.n_draft.clone(), ctx_lens=(att.ctx_lens - 64).clamp(min=S).contiguous(),
                    stride_tokens=torch.empty(B, S, dtype=torch.int32, device=dev),
                    draft_tokens=torch.empty(B, max(S - 1, 1), dtype=torch.int32, device=dev)[:, :S - 1].contiguous(),
                    out_tokens=torch.empty(B, 64, dtype=torch.int32, device=dev),
                    out_lens=torch.zeros(B, dtype=torch.int32, device=dev), block_table=att.block_table.clone(),
                    pages_used=pages_used.to(torch.int32).contiguous(),
                    free_list=torch.arange(4 * B, dtype=torch.int32, device=dev),
                    free_top=torch.full((1,), 4 * B, dtype=torch.int32, device=dev),
                    status=torch.full((1,), -1, dtype=torch.int32, device=dev))

    states = [commit_state() for _ in range(21)]
    it = iter(states)
    t_commit = timed(lambda: idlm.idlm_isd_commit(accept_len, new_tokens, next(it), n_draft_steady=n_steady,
                                                  mask_token=cfg.V - 1, P=cfg.P), n=20)
    commit_ok = all(int(st_["status"].item()) == 0 for st_ in states)
    append_bytes = 2 * 2 * B * S * cfg.Hkv * cfg.D * att.q.element_size()
    res["between_steps"] = {
        "isd_kv_append_kernel": {"ms": t_append, "bytes_read_plus_written": append_bytes,
                                 "GBps": append_bytes / t_append / 1e6},
        "isd_commit_kernel": {"ms": t_commit, "status_ok": commit_ok},
    }
    del states

    # the general acceptance entry point (proposal distributions, temperature, relaxed threshold,
    # sampled proposals) on the same logits; the proposal logits are a second buffer of the same size
    gen = None
    if S > 1:
        ws_gen = torch.empty(max(256, idlm.idlm_isd_accept_general_workspace(B, S, V)), dtype=torch.uint8, device=dev)
        q_logits = acc.logits.flip(1).contiguous()
        q_row = torch.full((B,), S - 1 - int(acc.n_draft.max().item()), dtype=torch.int32, device=dev)
        q_lse = torch.empty(B, S, dtype=torch.float32, device=dev)
        idlm.idlm_isd_accept_general(q_logits, drafts, acc.rng_seed, accept_len, new_tokens, n_draft=0, greedy=acc.greedy,
                                     temperature=0.9, row_lse=q_lse, workspace=ws_gen)

        def general(**kw):
            return timed(lambda: idlm.idlm_isd_accept_general(acc.logits, drafts, acc.rng_seed, accept_len, new_tokens,
                                                              n_draft=acc.n_draft, greedy=acc.greedy, workspace=ws_gen,
                                                              **kw), n=5)
        gen = {"point_mass_ms": general(),
               "proposal_distributions_ms": general(q_logits=q_logits, q_row=q_row, q_lse=q_lse, temperature=0.9, tau=0.1),
               "proposal_distributions_without_kept_lse_ms": general(q_logits=q_logits, q_row=q_row, temperature=0.9,
                                                                      tau=0.1),
               "with_sampled_proposals_ms": general(q_logits=q_logits, q_row=q_row, q_lse=q_lse, temperature=0.9,
                                                    tau=0.1, sample_proposals=True)}
        del q_logits, ws_gen
        ws_f = torch.empty(max(256, idlm.idlm_isd_accept_filtered_workspace(B, S, V)), dtype=torch.uint8, device=dev)
        gen["filtered_top_k50_top_p095_ms"] = timed(lambda: idlm.idlm_isd_accept_filtered(
            acc.logits, drafts, acc.rng_seed, accept_len, new_tokens, n_draft=acc.n_draft, greedy=acc.greedy, top_k=50,
            top_p=0.95, workspace=ws_f), n=5)
        gen["filtered_with_sampled_proposals_ms"] = timed(lambda: idlm.idlm_isd_accept_filtered(
            acc.logits, drafts, acc.rng_seed, accept_len, new_tokens, n_draft=acc.n_draft, greedy=acc.greedy, top_k=50,
            top_p=0.95, sample_proposals=True, workspace=ws_f), n=5)
        # the paper's sampler with sampled drafts, two calls in a row: the first keeps its candidate record,
        # the second verifies against it (and, last, the same over bf16 logits)
        rec = [torch.zeros((B, S, 64), dtype=torch.int64, device=dev) for _ in range(2)]
        q_row1 = torch.ones(B, dtype=torch.int32, device=dev)
        idlm.idlm_isd_accept_filtered_q(acc.logits, drafts, acc.rng_seed, accept_len, new_tokens, n_draft=0, greedy=acc.greedy,
                                        top_k=50, top_p=0.95, sample_proposals=True, cand_out=rec[0])
        nd_q = acc.n_draft.clamp(max=S - 1)
        gen["filtered_sampled_drafts_verified_ms"] = timed(lambda: idlm.idlm_isd_accept_filtered_q(
            acc.logits, drafts, acc.rng_seed, accept_len, new_tokens, n_draft=nd_q, greedy=acc.greedy, top_k=50, top_p=0.95,
            sample_proposals=True, q_cand=rec[0], q_row=q_row1, cand_out=rec[1]), n=5)
        if V % 8 == 0:
            lg16f = acc.logits.to(torch.bfloat16)
            gen["filtered_sampled_drafts_verified_bf16_logits_ms"] = timed(lambda: idlm.idlm_isd_accept_filtered_q(
                lg16f, drafts, acc.rng_seed, accept_len, new_tokens, n_draft=nd_q, greedy=acc.greedy, top_k=50, top_p=0.95,
                sample_proposals=True, q_cand=rec[0], q_row=q_row1, cand_out=rec[1]), n=5)
            del lg16f
        del rec
    res["accept_general"] = gen

    # the acceptance pass over the same logits stored as bf16 (half the bytes per row); not the timed path,
    # whose logits are fp32 as the metric's workload states
    bf16_acc = None
    if V % 8 == 0:
        lg16 = acc.logits.to(torch.bfloat16)
        evs = hev.create(3)
        t_stats = []
        for i in range(6):
            idlm.idlm_isd_accept_bf16(lg16, drafts, acc.rng_seed, accept_len, new_tokens, n_draft=acc.n_draft,
                                      greedy=acc.greedy, workspace=case.ws_acc, stream=stream, events=evs)
            torch.cuda.synchronize()
            if i:
                t_stats.append((hev.elapsed_ms(evs[0], evs[1]), hev.elapsed_ms(evs[1], evs[2])))
        hev.destroy(evs)
        t_rs = sum(t[0] for t in t_stats) / len(t_stats)
        rs_bytes = B * S * V * 2
        bf16_acc = {"isd_row_stats_kernel_ms": t_rs, "rest_ms": sum(t[1] for t in t_stats) / len(t_stats),
                    "algorithmic_bytes": rs_bytes, "GBps": rs_bytes / t_rs / 1e6,
                    "frac_hbm": rs_bytes / t_rs / 1e6 / 8000.0}
        del lg16
    res["accept_bf16_logits"] = bf16_acc

    # one linear layer of the lossless variant (gated low-rank adapter) on this step's tokens: an attention
    # projection of the 8B-class model (d_in = d_out = Hq*D) with the paper's rank-128 adapter, MASK rows from
    # the step's draft counts; and the same layer on the paper's own serving shape (64 sequences, stride N = 4)
    lora = None
    if cfg.dtype == "bf16":
        from isd_inputs import make_lora_inputs

        def lora_case(nseq, rows, nd):
            d = cfg.Hq * cfg.D
            li = make_lora_inputs(nseq, rows, d, d, 128, device=dev, seed=1)
            li.n_draft.copy_(nd)
            T = nseq * rows
            h = torch.empty(T, d, dtype=torch.bfloat16, device=dev)
            ws_l = torch.empty(max(256, idlm.idlm_gated_lora_linear_workspace(T, d, d, 128)), dtype=torch.uint8,
                               device=dev)
            t_full = timed(lambda: idlm.idlm_gated_lora_linear(li.x, li.W, li.A, li.Bm, h, n_draft=li.n_draft, S=rows,
                                                               workspace=ws_l), n=20)
            t_base = timed(lambda: idlm.idlm_gated_lora_linear(li.x, li.W, None, None, h, workspace=ws_l), n=20)
            masked = int((torch.arange(rows, device=dev)[None, :] > li.n_draft[:, None]).sum().item())
            flops = 2 * T * d * d + 2 * masked * 128 * (d + d)
            return {"tokens": T, "mask_tokens": masked, "d_in": d, "d_out": d, "rank": 128, "ms": t_full,
                    "base_layer_only_ms": t_base, "flops": flops, "TFLOPs": flops / t_full / 1e9,
                    "frac_mfma": flops / t_full / 1e9 / 2500.0}
        lora = {"step_tokens": lora_case(B, S, acc.n_draft.clamp(max=S - 1)),
                "paper_serving_shape_64x7": lora_case(64, 7, torch.full((64,), 3, dtype=torch.int32, device=dev))}
    res["gated_lora_linear"] = lora
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="serve256")
    ap.add_argument("--stride", type=int, default=0, help="override the workload's S (the long32k stride sweep)")
    ap.add_argument("--head-dim", type=int, default=0, help="override the workload's head dimension (64 or 128)")
    ap.add_argument("--workgroups", type=int, default=0, help="persistent attention grid (0 = one per CU)")
    ap.add_argument("--cpu-sample", type=int, default=256, help="sequences given to the CPU oracle (0 = skip)")
    ap.add_argument("--cpu-threads", type=int, default=0, help="threads of the CPU oracle (0 = all the box gives it)")
    ap.add_argument("--k-operand-order", type=int, default=1,
                    help="1: the K pool's pages are kept in the attention kernel's operand order (IDLM_DTYPE_BF16_KOP)")
    ap.add_argument("--sections", default="all",
                    help="comma list of step,probe,cpu,extras,configs,wavefronts (all = every one; configs only with the default workload)")
    ap.add_argument("--copies", type=int, default=0, help="input copies the launches rotate over (0 = as many as the "
                                                          "memory-side cache needs)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (no collectives, no sharding); --gpus %d is not supported"
                 % args.gpus)
    sections = ({"step", "probe", "cpu", "extras", "configs", "wavefronts"} if args.sections == "all"
                else set(args.sections.split(",")))

    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    sys.path.insert(0, ROOT)
    import paper_2604_11035_amd as idlm
    from isd_inputs import get_config
    from isd_inputs.configs import LONG32K_STRIDES

    cfg = get_config(args.workload, **({"S": args.stride} if args.stride else {}),
                     **({"D": args.head_dim} if args.head_dim else {}))
    dev = "cuda:0"
    torch.cuda.set_device(0)
    hev = HipEvents()
    stream = torch.cuda.current_stream()
    probe = Case(cfg, dev, copies=1, kop=args.k_operand_order, workgroups=args.workgroups)
    ncopies = args.copies or copies_for(probe.working_set_bytes())
    case = probe if ncopies == 1 else Case(cfg, dev, copies=ncopies, kop=args.k_operand_order, workgroups=args.workgroups)
    del probe
    B, S, V = cfg.B, cfg.S, cfg.V
    nwg = args.workgroups or torch.cuda.get_device_properties(0).multi_processor_count * (
        2 if attention_kernel_name(cfg) == "isd_attention_shared_kernel" else 1)   # the library's own choice

    for i in range(args.warmup):
        case.step(i, stream)
    torch.cuda.synchronize()
    # Every second timed step carries the library's event hooks (each recorded event separates two kernels by a
    # few microseconds, so a hooked step is 3-4 % slower than a plain one); more hooked launches follow the
    # timed region until every kernel has MIN_KERNEL_SAMPLES samples.
    hooked = [i for i in range(args.steps) if i % 2 == 0]
    events = [(hev.create(3), hev.create(3)) for _ in hooked]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        if i % 2 == 0:
            case.step(args.warmup + i, stream, events[i // 2][0], events[i // 2][1])
        else:
            case.step(args.warmup + i, stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    in_region = len(events)
    if in_region < MIN_KERNEL_SAMPLES:
        events += hooked_launches(case, hev, stream, MIN_KERNEL_SAMPLES - in_region, args.warmup + args.steps)
    kernels = kernel_record(case, hev, events)
    for ea, eb in events:
        hev.destroy(ea + eb)

    # what the last step accepted on these synthetic inputs (bookkeeping on the outputs): the introspective
    # acceptance rate is the mean accept probability of the verified drafts, here p(draft)
    acc = case.acc
    acceptance = None
    if S > 1:
        nd_f = acc.n_draft.clamp(max=S - 1).float()
        verified = torch.arange(S - 1, device=dev)[None, :] < acc.n_draft[:, None]
        stochastic = (acc.greedy == 0) if acc.greedy is not None else torch.ones(B, dtype=torch.bool, device=dev)
        acceptance = {
            "mean_drafts_per_sequence": float(nd_f.mean().item()),
            "mean_accept_len": float(case.accept_len.float().mean().item()),
            "tokens_finalised_per_sequence_per_step": float((case.accept_len.float() + 1).mean().item()),
            "introspective_acceptance_rate_mean_p_draft": float(case.draft_probs[verified].mean().item()) if bool(verified.any()) else None,
            "stochastic_share": float(stochastic.float().mean().item()),
        }

    att_name = next(k for k in kernels if k.startswith("isd_attention_") and "merge" not in k)
    kernels[att_name]["workgroups"] = nwg
    for k in (att_name, "isd_row_stats_kernel"):
        kernels[k]["samples_in_timed_region"] = in_region
    t_att_call = kernels[att_name]["ms"] + kernels["isd_attention_merge_kernel"]["ms"]
    t_acc_call = kernels["isd_row_stats_kernel"]["ms"] + kernels["isd_accept_chain+sample+emit_kernels"]["ms"]
    per_call = {
        "attention_positions_per_s": B * S / (t_att_call / 1e3), "accept_positions_per_s": B * S / (t_acc_call / 1e3),
        # context only: a forward of the 8B-class model the paper converts has 36 attention layers per acceptance
        # pass; its linear layers are not part of this figure
        "model_shaped_positions_per_s_36_attention_layers_no_gemms": B * S / ((36 * t_att_call + t_acc_call) / 1e3),
    }
    if kernels[att_name]["ms"] >= kernels["isd_row_stats_kernel"]["ms"]:
        dom_name, dom_key = att_name, "attention"
    else:
        dom_name, dom_key = "isd_row_stats_kernel", "row_stats"
    dom = kernels[dom_name]
    version = idlm.idlm_version()
    roofline = {"bound": "hbm", "achieved": dom["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": dom["GBps"] / HBM_PEAK_GBS,
                "traffic": measured_traffic(cfg.name + ("" if not args.stride else "_S%d" % args.stride), dom_key, version),
                "kernel": dom_name, "ms": dom["ms"], "samples": dom["samples"], "lib_version": version}

    line = {
        "metric": "ISD tokens verified+proposed/sec at B=256 on 1 GPU; % of peak HBM GB/s",
        "value": B * S / (ms_per_step / 1e3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": "%s: B=%d S=%d Hq=%d Hkv=%d D=%d P=%d V=%d, ctx %s [%d,%d] (sum %d), one attention "
                               "layer + one acceptance pass per step"
                               % (cfg.name, B, S, cfg.Hq, cfg.Hkv, cfg.D, cfg.P, V, cfg.ctx_kind, cfg.ctx_lo,
                                  cfg.ctx_hi, int(case.ctx_np.sum())),
                   "attention_workgroups": nwg, "logits_dtype": "f32", "input_copies_rotated": ncopies,
                   "k_pages": "operand order" if case.kop else "slot-major"},
        "roofline": roofline,
        "cpu_baseline": None,
        "kernels": kernels,
        "per_call": per_call,
        "acceptance": acceptance,
        "hbm_frac_both": {"attention": kernels[att_name]["frac_hbm"], "accept": kernels["isd_row_stats_kernel"]["frac_hbm"]},
    }
    if "probe" in sections:
        line["stream_ceiling"] = stream_probe(idlm, dev)
        for name in (att_name, "isd_row_stats_kernel"):
            kernels[name]["frac_of_measured_stream_read"] = kernels[name]["GBps"] / line["stream_ceiling"]["read_GBps"]
    if "wavefronts" in sections and cfg.dtype == "bf16":
        line["attention_wavefront_times"] = wavefront_times(case, stream)
    if "extras" in sections:
        line.update(extras(case, args, hev, stream, dev, ms_per_step))
    if "cpu" in sections and args.cpu_sample > 0:
        line["cpu_baseline"] = cpu_baseline(case.att, case.acc, cfg, min(args.cpu_sample, B), args.cpu_threads)
    if "configs" in sections and args.workload == "serve256" and not args.stride and not args.head_dim:
        del case
        torch.cuda.empty_cache()
        configs = {}
        for name, strides in (("small", (0,)), ("8b", (0,)), ("long32k", LONG32K_STRIDES)):
            for s_ in strides:
                c = get_config(name, **({"S": s_} if s_ else {}))
                configs[name + ("_S%d" % s_ if s_ else "")] = config_line(name, c, dev, hev, stream)
        # the 8B-class step with 64-wide heads (half the K/V bytes per token): the same kernels, other head dimension
        configs["8b_D64"] = config_line("8b", get_config("8b", D=64), dev, hev, stream)
        line["configs"] = configs
    print(json.dumps(line))


if __name__ == "__main__":
    main()
