#!/usr/bin/env python3
"""Benchmark of the ISD-step hot path on one MI355X.

One "step" = one idlm_isd_attention call (one layer's paged stride attention) plus one
idlm_isd_accept call (introspective acceptance over the step's logits) on the large-
concurrency serving workload (B=256, S=16; `serve256`), inputs resident in HBM.  Prints ONE
JSON line: whole-step throughput in stride positions (tokens verified + proposed) per second,
the roofline record of the dominant kernel (timed with HIP events recorded by the library
around each of its kernels on every fourth timed step, on the stream they run on), and the CPU oracle timed on a bounded
sample of the same workload on this machine's host cores.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16, published

# HBM traffic per launch measured offline with rocprofv3 --pmc (FETCH_SIZE and WRITE_SIZE runs,
# scaled by what the same counters read for idlm_stream_copy of known size); bytes per launch of
# the named kernel on the named workload.  None where no measurement is committed under profiles/.
MEASURED_TRAFFIC = {
    ("serve256", "attention"): 3326077105,   # profiles/serve256_pmc_hbm_traffic.txt (1.025 x algorithmic)
    ("serve256", "accept"): 2603501474,      # row-statistics kernel, same file (1.046 x algorithmic)
}


class HipEvents:
    """Minimal HIP event access (create / elapsed time) through libamdhip64."""

    def __init__(self):
        self.hip = C.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [C.c_void_p]
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


def attention_algorithmic_bytes(ctx_lens, cfg):
    """One read of every context token's K and V rows, Q in, O out, and the block table."""
    kv = int(ctx_lens.sum()) * cfg.Hkv * cfg.D * 2 * 2
    qo = cfg.B * 2 * cfg.S * cfg.Hq * cfg.D * 2
    table = int(((ctx_lens + cfg.P - 1) // cfg.P).sum()) * 4
    return kv + qo + table


def attention_flops(ctx_lens, cfg):
    """2 contractions x 2 flop x D per (query row, head, visible key)."""
    vis = sum(int(c) - cfg.S + i + 1 for c in ctx_lens for i in range(cfg.S))
    return 4 * cfg.D * cfg.Hq * vis


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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="serve256")
    ap.add_argument("--stride", type=int, default=0, help="override the workload's S (the long32k stride sweep)")
    ap.add_argument("--workgroups", type=int, default=0, help="persistent attention grid (0 = one per CU)")
    ap.add_argument("--cpu-sample", type=int, default=256, help="sequences given to the CPU oracle (0 = skip)")
    ap.add_argument("--cpu-threads", type=int, default=0, help="threads of the CPU oracle (0 = all the box gives it)")
    ap.add_argument("--k-operand-order", type=int, default=1,
                    help="1: the K pool's pages are kept in the attention kernel's operand order (IDLM_DTYPE_BF16_KOP)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (no collectives, no sharding); --gpus %d is not supported"
                 % args.gpus)

    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    import paper_2604_11035_amd as idlm
    from isd_inputs import get_config, make_accept_inputs, make_attention_inputs

    cfg = get_config(args.workload, **({"S": args.stride} if args.stride else {}))
    dev = "cuda:0"
    torch.cuda.set_device(0)
    att = make_attention_inputs(cfg, device=dev)
    acc = make_accept_inputs(cfg, device=dev)
    B, S, V = cfg.B, cfg.S, cfg.V
    dcode = 1 if cfg.dtype == "bf16" else 0
    max_pages = att.block_table.shape[1]
    nwg = args.workgroups or torch.cuda.get_device_properties(0).multi_processor_count
    ws_att = torch.empty(max(256, idlm.idlm_isd_attention_workspace(B, S, cfg.Hq, cfg.Hkv, cfg.D, cfg.P, max_pages,
                                                                    dcode)),
                         dtype=torch.uint8, device=dev)
    ws_acc = torch.empty(max(256, idlm.idlm_isd_accept_workspace(B, S, V)), dtype=torch.uint8, device=dev)
    out = torch.empty_like(att.q)
    accept_len = torch.empty(B, dtype=torch.int32, device=dev)
    new_tokens = torch.empty(B, S, dtype=torch.int32, device=dev)
    draft_probs = torch.empty(B, max(S - 1, 1), dtype=torch.float32, device=dev)
    drafts = acc.draft_tokens[:, :S - 1].contiguous() if S > 1 else None

    hev = HipEvents()
    stream = torch.cuda.current_stream()
    kop = bool(args.k_operand_order) and cfg.dtype == "bf16"
    k_gpu = att.k_cache
    if kop:   # the same pool, pages permuted once (what idlm_isd_kv_append maintains when given the same option)
        from isd_inputs import k_pages_in_operand_order
        k_gpu = k_pages_in_operand_order(att.k_cache)

    def step(i, ev_att=None, ev_acc=None):
        idlm.idlm_isd_attention(att.q, k_gpu, att.v_cache, att.block_table, att.ctx_lens, S, out,
                                num_workgroups=args.workgroups, workspace=ws_att, stream=stream, events=ev_att,
                                k_operand_order=kop)
        idlm.idlm_isd_accept(acc.logits, drafts, acc.rng_seed, accept_len, new_tokens, n_draft=acc.n_draft,
                             greedy=acc.greedy, rng_offset=i, draft_probs=draft_probs if S > 1 else None,
                             workspace=ws_acc, stream=stream, events=ev_acc)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    # every fourth timed step carries the library's event hooks (each recorded event separates two
    # kernels by a few microseconds, so hooking every step would slow the step it measures by 3-4 %)
    hooked = [i for i in range(args.steps) if i % 4 == 0]
    events = [(hev.create(3), hev.create(3)) for _ in hooked]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        if i % 4 == 0:
            step(args.warmup + i, events[i // 4][0], events[i // 4][1])
        else:
            step(args.warmup + i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # what the last timed step accepted on these synthetic inputs (bookkeeping on the outputs): the
    # introspective acceptance rate is the mean accept probability of the verified drafts, here p(draft)
    acceptance = None
    if S > 1:
        nd_f = acc.n_draft.clamp(max=S - 1).float()
        verified = torch.arange(S - 1, device=dev)[None, :] < acc.n_draft[:, None]
        stochastic = (acc.greedy == 0) if acc.greedy is not None else torch.ones(B, dtype=torch.bool, device=dev)
        acceptance = {
            "mean_drafts_per_sequence": float(nd_f.mean().item()),
            "mean_accept_len": float(accept_len.float().mean().item()),
            "tokens_finalised_per_sequence_per_step": float((accept_len.float() + 1).mean().item()),
            "introspective_acceptance_rate_mean_p_draft": float(draft_probs[verified].mean().item()) if bool(verified.any()) else None,
            "stochastic_share": float(stochastic.float().mean().item()),
        }

    def avg(which, a, b):
        return sum(hev.elapsed_ms(e[which][a], e[which][b]) for e in events) / len(events)

    def spread(which, a, b):
        v = sorted(hev.elapsed_ms(e[which][a], e[which][b]) for e in events)
        return {"min_ms": v[0], "median_ms": v[len(v) // 2], "max_ms": v[-1], "samples": len(v)}

    t_att_main, t_att_merge = avg(0, 0, 1), avg(0, 1, 2)
    t_acc_stats, t_acc_final = avg(1, 0, 1), avg(1, 1, 2)
    spreads = {"isd_attention_bf16_kernel": spread(0, 0, 1), "isd_row_stats_kernel": spread(1, 0, 1)}
    for ea, eb in events:
        hev.destroy(ea + eb)

    ctx_np = att.ctx_lens.cpu().numpy().astype(np.int64)
    att_bytes = attention_algorithmic_bytes(ctx_np, cfg)
    acc_bytes = B * S * V * 4
    att_flops = attention_flops(ctx_np, cfg)
    kernels = {
        "isd_attention_bf16_kernel": {
            "ms": t_att_main, "algorithmic_bytes": att_bytes, "GBps": att_bytes / t_att_main / 1e6,
            "frac_hbm": att_bytes / t_att_main / 1e6 / HBM_PEAK_GBS,
            "TFLOPs": att_flops / t_att_main / 1e9, "frac_mfma": att_flops / t_att_main / 1e9 / MFMA_BF16_PEAK_TFLOPS,
            "workgroups": nwg},
        "isd_attention_merge_kernel": {"ms": t_att_merge},
        "isd_row_stats_kernel": {
            "ms": t_acc_stats, "algorithmic_bytes": acc_bytes, "GBps": acc_bytes / t_acc_stats / 1e6,
            "frac_hbm": acc_bytes / t_acc_stats / 1e6 / HBM_PEAK_GBS},
        "isd_accept_chain+sample+emit_kernels": {"ms": t_acc_final},
    }
    for name, sp in spreads.items():
        kernels[name].update(sp)
    t_att_call, t_acc_call = t_att_main + t_att_merge, t_acc_stats + t_acc_final
    per_call = {
        "attention_positions_per_s": B * S / (t_att_call / 1e3), "accept_positions_per_s": B * S / (t_acc_call / 1e3),
        # context only: a forward of the 8B-class model the paper converts has 36 attention layers per acceptance
        # pass; its linear layers are not part of this figure
        "model_shaped_positions_per_s_36_attention_layers_no_gemms": B * S / ((36 * t_att_call + t_acc_call) / 1e3),
    }
    if t_att_main >= t_acc_stats:
        dom, dom_name, dom_key = kernels["isd_attention_bf16_kernel"], "isd_attention_bf16_kernel", "attention"
    else:
        dom, dom_name, dom_key = kernels["isd_row_stats_kernel"], "isd_row_stats_kernel", "accept"
    roofline = {"bound": "hbm", "achieved": dom["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": dom["GBps"] / HBM_PEAK_GBS, "traffic": MEASURED_TRAFFIC.get((args.workload, dom_key)),
                "kernel": dom_name, "ms": dom["ms"]}

    # plain streaming kernels of known size: practical bandwidth ceiling of this device, and the
    # reference that hardware byte counters are scaled by in the committed profiles (4 GiB, so that
    # the 256 MB memory-side cache holds a negligible part of it from one pass to the next)
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
    stream_probe = {"read_GBps": probe.numel() / t_read / 1e6, "copy_read_plus_write_GBps": 2 * probe.numel() / t_copy / 1e6,
              "bytes": probe.numel()}
    for name in ("isd_attention_bf16_kernel", "isd_row_stats_kernel"):
        kernels[name]["frac_of_measured_stream_read"] = kernels[name]["GBps"] / stream_probe["read_GBps"]
    del probe, probe_dst

    # the same step launched without the timing hooks, and replayed from a captured HIP graph (the
    # calls allocate nothing and never synchronise, so they can be captured as they are)
    def plain_steps(n):
        for i in range(n):
            step(args.warmup + i)
    torch.cuda.synchronize()
    t_plain = timed(lambda: plain_steps(args.steps), n=1) / args.steps
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    stream = side
    with torch.cuda.graph(graph, stream=side):
        step(0)
    stream = torch.cuda.current_stream()
    torch.cuda.synchronize()

    def replay_steps(n):
        for _ in range(n):
            graph.replay()
    t_graph = timed(lambda: replay_steps(args.steps), n=1) / args.steps
    # the attention call alone with the K pool in the other page layout (slot-major rows / operand order)
    k_other = att.k_cache
    if not kop and cfg.dtype == "bf16":
        from isd_inputs import k_pages_in_operand_order
        k_other = k_pages_in_operand_order(att.k_cache)
    t_att_kop, t_att_other = (timed(lambda: idlm.idlm_isd_attention(
        att.q, kk, att.v_cache, att.block_table, att.ctx_lens, S, out, num_workgroups=args.workgroups, workspace=ws_att,
        k_operand_order=flag), n=10) for kk, flag in ((k_gpu, kop), (k_other, (not kop) and cfg.dtype == "bf16")))
    del k_other
    launch_modes = {"timed_region_ms": ms_per_step, "eager_ms": t_plain, "graph_replay_ms": t_graph}
    k_layouts = {"attention_call_ms_as_timed": t_att_kop, "attention_call_ms_other_k_page_layout": t_att_other,
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
    loop_kernels = {
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

    # the acceptance pass over the same logits stored as bf16 (half the bytes per row); not the timed path,
    # whose logits are fp32 as the metric's workload states
    bf16_acc = None
    if V % 8 == 0:
        lg16 = acc.logits.to(torch.bfloat16)
        evs = hev.create(3)
        t_stats = []
        for i in range(6):
            idlm.idlm_isd_accept_bf16(lg16, drafts, acc.rng_seed, accept_len, new_tokens, n_draft=acc.n_draft,
                                      greedy=acc.greedy, workspace=ws_acc, stream=stream, events=evs)
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

    cpu = None
    if args.cpu_sample > 0:
        cpu = cpu_baseline(att, acc, cfg, min(args.cpu_sample, B), args.cpu_threads)

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
                                  cfg.ctx_hi, int(ctx_np.sum())),
                   "attention_workgroups": nwg, "logits_dtype": "f32",
                   "k_pages": "operand order" if kop else "slot-major"},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "kernels": kernels,
        "per_call": per_call,
        "stream_ceiling": stream_probe,
        "between_steps": loop_kernels,
        "launch_modes": launch_modes,
        "k_page_layouts": k_layouts,
        "acceptance": acceptance,
        "accept_general": gen,
        "accept_bf16_logits": bf16_acc,
        "gated_lora_linear": lora,
        "hbm_frac_both": {"attention": kernels["isd_attention_bf16_kernel"]["frac_hbm"],
                          "accept": kernels["isd_row_stats_kernel"]["frac_hbm"]},
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
