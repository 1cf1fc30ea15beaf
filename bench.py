#!/usr/bin/env python3
"""Benchmark of the ESP attention hot path on ONE MI355X.

A step is one pass of the whole hot path over one batch of synthetic input, already resident in HBM:
    prefill partial attention of the local query chunk against each of the 4 striped KV shards
    -> merge of the 4 partials -> KV append of the new decode tokens into free pool slots
    -> decode partial attention over the token pool, combined with 3 peer partials in the same call.
Default workload: the LWM-7B (Llama-2-7B shape, 32 heads x 128, MHA) shares of the benchmark spec:
configs[1] for prefill (8192-token chunk, 4 x 8192 striped KV) and configs[2] for decode (64 requests,
lognormal KV slices in a 4M-slot pool).  `value` is the prefill TFLOP/s; the decode GB/s is reported in
the same line (`decode`), each with its roofline object.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="lwm7b", choices=["lwm7b", "long", "mixed"],
                    help="lwm7b = configs[1]+configs[2] (default, the bench line); long = configs[3]; mixed = configs[4]")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true",
                    help="skip the other full-size configurations that the default run times after its own steps "
                         "(configs[3] and configs[4]; a profiled run then holds launches of the headline shapes only)")
    ap.add_argument("--retain", action="store_true",
                    help="proactive retention (scale-down during prefill): every shard's rows are ALL kept in a token pool while the "
                         "shard is attended, by esp_kv_append from a second stream and by esp_partial_attn_prefill_retain (from "
                         "the tiles in on-chip memory); reports both overheads against prefill alone")
    ap.add_argument("--one-call", action="store_true",
                    help="also time one prefill call over all shards put together in order of position (not part of the default "
                         "run, so that the kernel statistics of a profiled default run hold launches of one shape only)")
    ap.add_argument("--multi-master", action="store_true",
                    help="distributed decoding with several masters on one GPU: this instance decodes the requests it is master "
                         "of while the queries of the other masters' requests arrive (host-to-device copies on a second stream), "
                         "then decodes those and sends their results back; reports the time against one decode call over all")
    ap.add_argument("--from-pool", action="store_true",
                    help="prefill over pool-resident shards: every shard's rows sit at random slots of a token pool and are "
                         "attended through esp_partial_attn_prefill_pool (gather into staging rows, then the dense kernel) and through "
                         "esp_partial_attn_prefill_pool_direct (the tile transfers read the pool rows); reports both overheads "
                         "against the dense call")
    ap.add_argument("--fit-model", action="store_true",
                    help="also time whole-request causal prefill batches of several length mixes, fit the iteration-time model "
                         "(alpha + beta*sum(len) + gamma*sum(len^2)) with esp_fit_prefill_model and report its error")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 1 GiB device-to-device copy kernel (known traffic, to scale rocprofv3 --pmc byte counters)")
    ap.add_argument("--traffic-json", default=os.path.join(ROOT, "profiles", "bench_lwm7b_hbm_traffic.json"),
                    help="JSON with HBM bytes per launch measured by rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on this workload "
                         "(see profiles/bench_lwm7b_hbm_traffic.md); used for roofline.traffic of the default workload")
    return ap.parse_args()


def cpu_baseline(pc, dc, wl, oracle):
    """The oracle as it stands, timed on this host's cores on a bounded sample of the same workload: for prefill
    the very (row, head) samples the full-size parity test evaluates, against every shard."""
    import numpy as np
    out = {"kind": "oracle", "cores": oracle.num_threads()}
    sample = []
    if pc is not None:
        n_total, seed = wl.PARITY_SAMPLES.get(pc.name, (1024, 0))
        rows, heads, reqs = wl.prefill_parity_samples(pc, n_total, seed)
        qb, qp = wl.bits(pc.q), wl.host_i32(pc.q_pos)
        pairs, dt = 0, 0.0
        for s in pc.shards:
            cu_kv = wl.host_i32(s.cu_kv)
            kb, vb, kp = wl.bits(s.k), wl.bits(s.v), wl.host_i32(s.kv_pos)
            # visible pairs of the sample, to convert seconds into the metric's unit
            for r in range(pc.batch):
                m = reqs == r
                if m.any():
                    seg = np.sort(kp[cu_kv[r]:cu_kv[r + 1]])
                    pairs += int(np.searchsorted(seg, qp[rows[m]], side="right").sum()) if pc.causal else int(m.sum()) * len(seg)
            t0 = time.perf_counter()
            oracle.partial_attn(qb, kb, vb, qp, kp, pc.scale, pc.causal, rows, heads, cu_kv[reqs], cu_kv[reqs + 1])
            dt += time.perf_counter() - t0
        out["value"] = 4.0 * pc.D * pairs / dt / 1e12
        out["unit"] = "TFLOP/s"
        out["seconds"] = dt
        sample.append(f"prefill: the {len(rows)} (row, head) samples of the full-size parity test against each of the "
                      f"{len(pc.shards)} shards ({pairs} visible pairs)")
        out["extrapolated_full_prefill_s"] = dt * pc.visible_pairs_per_head * pc.Hq / max(pairs, 1)
    if dc is not None:
        slots, off = wl.host_i32(dc.slot_idx), wl.host_i32(dc.seq_offsets)
        kpool = np.zeros((dc.num_slots, dc.Hkv, dc.D), np.uint16)
        vpool = np.zeros_like(kpool)
        reqs_s = sorted(dc.host_rows)
        tok = 0
        for b in reqs_s:
            kr, vr = dc.host_rows[b]
            oracle.kv_append(kr, vr, slots[off[b]:off[b + 1]], kpool, vpool)
            tok += int(off[b + 1] - off[b])
        heads = np.arange(dc.Hq, dtype=np.int64)
        reqs = np.repeat(np.asarray(reqs_s, np.int64), len(heads))
        hs = np.tile(heads, len(reqs_s))
        t0 = time.perf_counter()
        oracle.partial_attn_decode(wl.bits(dc.q), kpool, vpool, slots, off, dc.scale, reqs, hs)
        dt = time.perf_counter() - t0
        # bytes the oracle touched: K and V rows of the sampled heads only
        byts = tok * len(heads) * 2 * dc.D * 2
        out["decode_value"] = byts / dt / 1e9
        out["decode_unit"] = "GB/s"
        out["decode_seconds"] = dt
        sample.append(f"decode: requests {reqs_s} x {len(heads)} heads ({tok} resident tokens)")
    out["sample"] = "; ".join(sample)
    return out


MODEL_FIT_BATCHES = ([1024], [2048], [4096], [8192], [12288], [16384], [24576], [32768], [49152],
                     [2048, 2048, 4096], [8192, 4096, 1024], [16384, 8192], [12288, 12288], [1024] * 8, [32768, 16384, 4096])


def fit_model(esp, wl, torch, np, dev, batches=MODEL_FIT_BATCHES, Hq=32, Hkv=32, reps=5):
    """Times one prefill call per batch of whole requests (causal self-attention, one shard holding every key),
    fits the iteration-time model to the measurements and reports how well it reproduces them."""
    s1, s2, ms = [], [], []
    for bi, lens in enumerate(batches):
        pc = wl.striped_prefill("fit", lens, 1, 0, Hq, Hkv, 100 + bi, dev)
        sh = pc.shards[0]
        ws = torch.empty(esp.esp_prefill_workspace_bytes(pc.Tq, sh.k.shape[0], pc.batch, pc.Hq, pc.Hkv, pc.D), dtype=torch.uint8, device=dev)
        O = torch.empty_like(pc.q); L = torch.empty((pc.Tq, pc.Hq), dtype=torch.float32, device=dev)
        single = pc.batch == 1
        run = lambda: esp.esp_partial_attn_prefill(pc.q, sh.k, sh.v, pc.q_pos, sh.kv_pos, None if single else pc.cu_q,
                                                   None if single else sh.cu_kv, None if single else pc.max_q,
                                                   None if single else sh.max_kv, softmax_scale=pc.scale, causal=True,
                                                   O=O, LSE=L, workspace=ws)
        run(); torch.cuda.synchronize()
        best = float("inf")
        for _ in range(3):                       # least of three averages: the short calls are noisy
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                run()
            e1.record(); torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1) / reps)
        ms.append(best)
        s1.append(float(sum(lens))); s2.append(float(sum(x * x for x in lens)))
        del pc, sh, O, L
    t = np.array(ms) * 1e-3
    coef = esp.esp_fit_prefill_model(s1, s2, t, weights=1.0 / t)     # relative residuals: the times span 500x
    pred = coef[0] + coef[1] * np.array(s1) + coef[2] * np.array(s2)
    rel = np.abs(pred - t) / t
    return {"alpha_s": float(coef[0]), "beta_s_per_token": float(coef[1]), "gamma_s_per_token2": float(coef[2]),
            "max_rel_err": float(rel.max()), "mean_rel_err": float(rel.mean()),
            "samples": [{"lens": list(l), "ms": float(m), "model_ms": float(p * 1e3)} for l, m, p in zip(batches, ms, pred)]}


def note(msg):
    """Progress line on stderr (stdout carries only the JSON line)."""
    print("[bench] " + msg, file=sys.stderr, flush=True)


def make_workload(which, wl, np, dev):
    """(prefill case, decode case, description) of one of the three benchmark workloads."""
    pc = dc = None
    if which == "lwm7b":
        pc = wl.config2_prefill(dev)
        lens = wl.lognormal_lengths(64, 8192, 1024, 131072, 2)
        order = np.argsort(lens)
        dc = wl.config3_decode(dev, sample_reqs=[int(i) for i in order[::4]])
        name = "LWM-7B shape: prefill chunk 8192 x 4 striped shards of 8192 (configs[1]) + decode B=64 in a 4M-slot pool (configs[2])"
    elif which == "long":
        pc = wl.config4_prefill(dev)
        name = "long-context prefill share: chunk 32768 against 262144 local KV (configs[3])"
    else:
        pc = wl.config5_prefill(dev)
        lens = wl.lognormal_lengths(256, 16384, 512, 1 << 20, 4)
        order = np.argsort(lens)
        dc = wl.config5_decode(dev, sample_reqs=[int(order[0]), int(order[len(order) // 2])])
        name = "mixed iteration: var-len GQA prefill of 6 requests x 4 striped shards + decode B=256 in a 16M-slot pool (configs[4])"
    return pc, dc, name


class Step:
    """One pass of the hot path over a workload, with its buffers.  Partials of several shards stay on this GPU, so
    they are written as fp32 and rounded to bf16 once, by the merge; a single shard's output is bf16 right away."""

    def __init__(self, esp, torch, pc, dc, dev):
        self.esp, self.torch, self.pc, self.dc = esp, torch, pc, dc
        self.single = pc.batch == 1
        several = len(pc.shards) > 1
        self.ws_pf = torch.empty(max(esp.esp_prefill_workspace_bytes(pc.Tq, pc.shards[0].k.shape[0], pc.batch, pc.Hq, pc.Hkv, pc.D), 256),
                                 dtype=torch.uint8, device=dev)
        self.part_O = [torch.empty(pc.q.shape, dtype=torch.float32 if several else torch.bfloat16, device=dev) for _ in pc.shards]
        self.part_L = [torch.empty((pc.Tq, pc.Hq), dtype=torch.float32, device=dev) for _ in pc.shards]
        self.out_O = torch.empty_like(pc.q)
        self.out_L = torch.empty((pc.Tq, pc.Hq), dtype=torch.float32, device=dev)
        if dc is not None:
            self.max_len = int(dc.lens.max())
            self.ws_dc = torch.empty(esp.esp_decode_workspace_bytes(dc.B, dc.total_tokens, self.max_len, dc.Hq, dc.Hkv, dc.D),
                                     dtype=torch.uint8, device=dev)
            self.dO = torch.empty_like(dc.q)
            self.dL = torch.empty((dc.B, dc.Hq), dtype=torch.float32, device=dev)
            self.mO = torch.empty_like(dc.q)
            self.mL = torch.empty_like(self.dL)

    def prefill_shard(self, i, O=None, L=None, ws=None):
        pc, s, single = self.pc, self.pc.shards[i], self.single
        self.esp.esp_partial_attn_prefill(pc.q, s.k, s.v, pc.q_pos, s.kv_pos,
                                          None if single else pc.cu_q, None if single else s.cu_kv,
                                          None if single else pc.max_q, None if single else s.max_kv,
                                          softmax_scale=pc.scale, causal=pc.causal, O=self.part_O[i] if O is None else O,
                                          LSE=self.part_L[i] if L is None else L, workspace=self.ws_pf if ws is None else ws)

    def __call__(self, rec=None):
        esp, pc, dc = self.esp, self.pc, self.dc
        e = [self.torch.cuda.Event(enable_timing=True) for _ in range(6)] if rec is not None else None
        if e: e[0].record()
        for i in range(len(pc.shards)):
            self.prefill_shard(i)
        if e: e[1].record()
        if len(pc.shards) > 1:
            esp.esp_merge_partials(self.part_O, self.part_L, O=self.out_O, LSE=self.out_L)
        if e: e[2].record()
        if dc is not None:
            esp.esp_kv_append(dc.new_k, dc.new_v, dc.new_slots, dc.k_pool, dc.v_pool)
            if e: e[3].record()
            # local partial attention and the combination with the peers' results, one call (Sec. 4.2)
            esp.esp_partial_attn_decode_merge(dc.q, dc.k_pool, dc.v_pool, dc.slot_idx, dc.seq_offsets, self.max_len,
                                              list(dc.peer_O), list(dc.peer_LSE), softmax_scale=dc.scale, O=self.mO,
                                              LSE=self.mL, workspace=self.ws_dc)
            if e: e[4].record()
            if e: e[5].record()
        if rec is not None:
            rec.append(e)


def time_steps(torch, step, steps, warmup):
    """`warmup` untimed and `steps` timed passes; returns (event records, wall seconds of the timed passes)."""
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    recs = []
    t0 = time.perf_counter()
    for _ in range(steps):
        step(recs)
    torch.cuda.synchronize()
    return recs, time.perf_counter() - t0


def summarize(recs, pc, dc):
    """Per-phase averages of the event records, in the units of the metric."""
    avg = lambda i, j: sum(e[i].elapsed_time(e[j]) for e in recs) / len(recs)   # ms

    def spread(i, j):
        v = sorted(e[i].elapsed_time(e[j]) for e in recs)
        return {"min": v[0], "median": v[len(v) // 2], "max": v[-1]}

    n_calls = len(pc.shards)
    ms_prefill = avg(0, 1)
    flops = pc.flops()
    tflops = flops / (ms_prefill * 1e-3) / 1e12
    out = {"prefill": {"ms_all_shards": ms_prefill, "ms_all_shards_spread": spread(0, 1), "ms_per_shard_call": ms_prefill / n_calls,
                       "ms_merge": avg(1, 2) if n_calls > 1 else 0.0, "partials": "fp32" if n_calls > 1 else "bf16 (one shard, no merge)",
                       "tflops": tflops, "pct_of_peak": 100.0 * tflops / PEAK_BF16_TFLOPS, "flops": flops, "launches_per_step": n_calls}}
    if dc is not None:
        ms_decode = avg(3, 4)
        byts = dc.kv_bytes()
        gbs = byts / (ms_decode * 1e-3) / 1e9
        out["decode"] = {"ms": ms_decode, "ms_spread": spread(3, 4), "ms_append": avg(2, 3), "merge": "with the 3 peer partials, inside the decode call", "bytes": byts, "gbs": gbs,
                         "pct_of_peak": 100.0 * gbs / PEAK_HBM_GBS, "B": dc.B, "total_tokens": dc.total_tokens, "sigma": 1.0}
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding): the figure it reports is one GPU's "
              "throughput on its share of the sequence-parallel work; use --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2404_09526_amd import binding as esp, workloads as wl

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    note("generating the synthetic inputs of workload '%s'" % args.workload)
    pc, dc, name = make_workload(args.workload, wl, np, dev)
    step = Step(esp, torch, pc, dc, dev)
    single = step.single
    ws_pf, part_O, part_L, out_O, out_L = step.ws_pf, step.part_O, step.part_L, step.out_O, step.out_L
    if dc is not None:
        max_len, ws_dc, dO, dL, mO, mL = step.max_len, step.ws_dc, step.dO, step.dL, step.mO, step.mL
    ev = lambda: torch.cuda.Event(enable_timing=True)

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                      # 1 GiB read + 1 GiB written by one elementwise kernel
        torch.cuda.synchronize()
        del src, dst
    note("inputs ready; %d warm-up and %d timed steps" % (args.warmup, args.steps))
    recs, wall = time_steps(torch, step, args.steps, args.warmup)
    summ = summarize(recs, pc, dc)
    tflops, flops, n_calls = summ["prefill"]["tflops"], summ["prefill"]["flops"], len(pc.shards)
    ms_prefill = summ["prefill"]["ms_all_shards"]
    result = {
        "metric": "prefill partial-attn TFLOP/s + decode partial-attn HBM GB/s (% of peak)",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": name, "Hq": pc.Hq, "Hkv": pc.Hkv, "head_dim": pc.D, "prefill_Tq": pc.Tq,
                   "prefill_shards": n_calls, "prefill_flops": flops},
        "prefill": summ["prefill"],
        "roofline": {"kernel": "prefill_kernel", "bound": "mfma", "achieved": tflops, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": tflops / PEAK_BF16_TFLOPS, "traffic": None,
                     "launch_ms": ms_prefill / n_calls, "flops_per_launch": flops / n_calls},
    }
    if dc is not None:
        result["decode"] = summ["decode"]
        gbs = summ["decode"]["gbs"]
        # whole pool rows on the vector ALU for MHA-like layouts, one KV head at a time on the matrix cores otherwise
        burst = dc.Hkv in (4, 8, 16) or dc.Hkv % 32 == 0
        dkernel = "decode_partial_kernel" if burst and dc.Hq // dc.Hkv <= 2 else "decode_partial_gq_kernel"
        result["roofline_decode"] = {"kernel": dkernel, "bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS,
                                     "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS, "traffic": None, "launch_ms": summ["decode"]["ms"],
                                     "bytes_per_launch": summ["decode"]["bytes"]}
        result["config"].update({"decode_B": dc.B, "decode_total_tokens": dc.total_tokens, "pool_slots": dc.num_slots})
    if args.fit_model:
        result["model_fit"] = fit_model(esp, wl, torch, np, dev)
    if args.retain:
        # pool with room for every row of every shard, slots = seeded permutation (any token-level placement is legal)
        n_rows = sum(s.k.shape[0] for s in pc.shards)
        S = 1 << (n_rows - 1).bit_length()
        kp = torch.zeros((S, pc.Hkv, pc.D), dtype=torch.bfloat16, device=dev)
        vp = torch.zeros_like(kp)
        perm = torch.from_numpy(np.random.default_rng(99).permutation(S)[:n_rows].astype(np.int32)).to(dev)
        slots, o = [], 0
        for s in pc.shards:
            slots.append(perm[o:o + s.k.shape[0]].contiguous()); o += s.k.shape[0]
        side = torch.cuda.Stream()

        cu = lambda i: (None if single else pc.cu_q, None if single else pc.shards[i].cu_kv,
                        None if single else pc.max_q, None if single else pc.shards[i].max_kv)

        def prefill_only(mode):
            for i, s in enumerate(pc.shards):
                if mode == "side_stream":
                    side.wait_stream(torch.cuda.current_stream())
                    with torch.cuda.stream(side):
                        esp.esp_kv_append(s.k, s.v, slots[i], kp, vp)
                if mode == "fused":
                    esp.esp_partial_attn_prefill_retain(pc.q, s.k, s.v, pc.q_pos, s.kv_pos, slots[i], kp, vp, *cu(i),
                                                        softmax_scale=pc.scale, causal=pc.causal, O=part_O[i], LSE=part_L[i], workspace=ws_pf)
                else:
                    esp.esp_partial_attn_prefill(pc.q, s.k, s.v, pc.q_pos, s.kv_pos, *cu(i),
                                                 softmax_scale=pc.scale, causal=pc.causal, O=part_O[i], LSE=part_L[i], workspace=ws_pf)
            if mode == "side_stream":
                torch.cuda.current_stream().wait_stream(side)

        times, pool_ok = {}, {}
        for mode in ("alone", "side_stream", "fused", "alone", "side_stream", "fused"):
            if mode != "alone":
                kp.zero_(); vp.zero_()
            prefill_only(mode); torch.cuda.synchronize()
            e0, e1 = ev(), ev()
            e0.record()
            for _ in range(args.steps):
                prefill_only(mode)
            e1.record(); torch.cuda.synchronize()
            times.setdefault(mode, []).append(e0.elapsed_time(e1) / args.steps)
            if mode != "alone":
                pool_ok[mode] = all(torch.equal(kp[slots[i].long()], s.k) and torch.equal(vp[slots[i].long()], s.v) for i, s in enumerate(pc.shards))
        t_plain, t_side, t_fused = min(times["alone"]), min(times["side_stream"]), min(times["fused"])
        result["retain"] = {"ms_prefill_alone": t_plain, "ms_with_side_stream_scatter": t_side, "ms_fused": t_fused,
                            "overhead_pct_side_stream": 100.0 * (t_side / t_plain - 1.0), "overhead_pct_fused": 100.0 * (t_fused / t_plain - 1.0),
                            "rows_retained": n_rows, "bytes_written": 2 * n_rows * pc.Hkv * pc.D * 2,
                            "pool_matches": {k: bool(v) for k, v in pool_ok.items()}}
    if args.one_call and single and len(pc.shards) > 1:
        # the same keys in one call: the shards concatenated and put in order of position (any order of rows is a
        # valid shard; ascending positions are what lets whole tiles be skipped or left unmasked)
        p_all = torch.cat([s.kv_pos for s in pc.shards])
        order = torch.argsort(p_all)
        k_all = torch.cat([s.k for s in pc.shards])[order].contiguous(); v_all = torch.cat([s.v for s in pc.shards])[order].contiguous()
        p_all = p_all[order].contiguous()
        ws1 = torch.empty(esp.esp_prefill_workspace_bytes(pc.Tq, k_all.shape[0], 1, pc.Hq, pc.Hkv, pc.D), dtype=torch.uint8, device=dev)
        one = lambda: esp.esp_partial_attn_prefill(pc.q, k_all, v_all, pc.q_pos, p_all, softmax_scale=pc.scale, causal=pc.causal,
                                                   O=out_O, LSE=out_L, workspace=ws1)
        one(); torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record()
        for _ in range(max(3, args.steps // 2)):
            one()
        e1.record(); torch.cuda.synchronize()
        ms_one = e0.elapsed_time(e1) / max(3, args.steps // 2)
        result["prefill"]["one_call_over_all_shards"] = {"ms": ms_one, "tflops": flops / (ms_one * 1e-3) / 1e12,
                                                          "note": "the four shards as one shard of 32768 rows in order of position"}
        del k_all, v_all
    # what a bare loop sustains on this box, for "fraction of achievable" beside "fraction of the published peak"
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    gen = torch.Generator(device=dev).manual_seed(7)
    ops_n = torch.randn(1 << 16, generator=gen, device=dev).to(torch.bfloat16)
    probe = {}
    for label, ops in (("normal", ops_n), ("constant", torch.full_like(ops_n, 1.0))):
        best = None
        for _ in range(4):
            e0, e1 = ev(), ev()
            e0.record()
            fl = esp.esp_probe_mfma_bf16(ops, 20000, sink)
            e1.record(); torch.cuda.synchronize()
            t = e0.elapsed_time(e1)
            best = t if best is None else min(best, t)
        probe["mfma_bf16_tflops_%s_operands" % label] = fl / (best * 1e-3) / 1e12
    buf = torch.empty(1 << 30, dtype=torch.int32, device=dev).fill_(1)       # 4 GiB, far beyond the last-level cache
    best = None
    for _ in range(4):
        e0, e1 = ev(), ev()
        e0.record()
        nb = esp.esp_probe_stream_read(buf, sink)
        e1.record(); torch.cuda.synchronize()
        t = e0.elapsed_time(e1)
        best = t if best is None else min(best, t)
    probe["hbm_read_gbs"] = nb / (best * 1e-3) / 1e9
    del buf
    result["achievable"] = probe
    result["roofline"]["frac_of_bare_mfma_loop_normal_operands"] = tflops / probe["mfma_bf16_tflops_normal_operands"]
    if "roofline_decode" in result:
        result["roofline_decode"]["frac_of_streaming_read"] = result["decode"]["gbs"] / probe["hbm_read_gbs"]
    if args.multi_master and dc is not None and dc.B >= 2:
        # Sec. 4.2 / Fig. 8: every instance is master of some requests (it has their queries) and a helper for the
        # rest, whose queries come from their masters and whose partial results go back to them
        h = dc.B // 2
        off_h = int(dc.seq_offsets[h].item())
        own_off = dc.seq_offsets[:h + 1].contiguous()
        peer_off = (dc.seq_offsets[h:] - off_h).contiguous()
        own_slots, peer_slots = dc.slot_idx[:off_h].contiguous(), dc.slot_idx[off_h:].contiguous()
        lens = dc.lens
        ml_own, ml_peer = int(lens[:h].max()), int(lens[h:].max())
        q_host = dc.q[h:].cpu().pin_memory()                       # the other masters' queries, as they come off the wire
        q_peer = torch.empty_like(dc.q[h:])
        O_peer, L_peer = torch.empty_like(dc.q[h:]), torch.empty((dc.B - h, dc.Hq), dtype=torch.float32, device=dev)
        O_back = torch.empty(O_peer.shape, dtype=O_peer.dtype).pin_memory(); L_back = torch.empty(L_peer.shape, dtype=L_peer.dtype).pin_memory()
        ws_own = torch.empty(esp.esp_decode_workspace_bytes(h, off_h, ml_own, dc.Hq, dc.Hkv, dc.D), dtype=torch.uint8, device=dev)
        ws_peer = torch.empty(esp.esp_decode_workspace_bytes(dc.B - h, dc.total_tokens - off_h, ml_peer, dc.Hq, dc.Hkv, dc.D),
                              dtype=torch.uint8, device=dev)
        mO_own, mL_own = torch.empty_like(dc.q[:h]), torch.empty((h, dc.Hq), dtype=torch.float32, device=dev)
        wire = torch.cuda.Stream()

        def masters():
            main = torch.cuda.current_stream()
            wire.wait_stream(main)
            with torch.cuda.stream(wire):
                q_peer.copy_(q_host, non_blocking=True)           # peers' queries arrive while the own requests are decoded
            # own requests: local partial attention and the merge with what the peers sent, one call
            esp.esp_partial_attn_decode_merge(dc.q[:h], dc.k_pool, dc.v_pool, own_slots, own_off, ml_own,
                                              [p[:h] for p in dc.peer_O], [p[:h] for p in dc.peer_LSE], softmax_scale=dc.scale,
                                              O=mO_own, LSE=mL_own, workspace=ws_own)
            main.wait_stream(wire)
            esp.esp_partial_attn_decode(q_peer, dc.k_pool, dc.v_pool, peer_slots, peer_off, ml_peer, softmax_scale=dc.scale,
                                        O=O_peer, LSE=L_peer, workspace=ws_peer)
            wire.wait_stream(main)
            with torch.cuda.stream(wire):
                O_back.copy_(O_peer, non_blocking=True); L_back.copy_(L_peer, non_blocking=True)   # results go back to their masters
            main.wait_stream(wire)

        def one_call():
            esp.esp_partial_attn_decode_merge(dc.q, dc.k_pool, dc.v_pool, dc.slot_idx, dc.seq_offsets, max_len,
                                              list(dc.peer_O), list(dc.peer_LSE), softmax_scale=dc.scale, O=mO, LSE=mL,
                                              workspace=ws_dc)

        # the helped requests' partial results, for comparison: one plain call over all requests
        esp.esp_partial_attn_decode(dc.q, dc.k_pool, dc.v_pool, dc.slot_idx, dc.seq_offsets, max_len,
                                    softmax_scale=dc.scale, O=dO, LSE=dL, workspace=ws_dc)
        torch.cuda.synchronize()

        times = {}
        for fn in (one_call, masters, one_call, masters):
            fn(); torch.cuda.synchronize()
            e0, e1 = ev(), ev()
            e0.record()
            for _ in range(args.steps):
                fn()
            e1.record(); torch.cuda.synchronize()
            times.setdefault(fn.__name__, []).append(e0.elapsed_time(e1) / args.steps)
        t_one, t_mm = min(times["one_call"]), min(times["masters"])
        diff = max(float((mO_own.float() - mO[:h].float()).abs().max()), float((O_peer.float() - dO[h:].float()).abs().max()),
                   float((O_back.float() - dO[h:].float().cpu()).abs().max()))
        result["multi_master"] = {"ms_one_decode_call": t_one, "ms_two_masters": t_mm, "overhead_pct": 100.0 * (t_mm / t_one - 1.0),
                                  "own_requests": h, "peer_requests": dc.B - h, "query_bytes_in": q_host.numel() * 2,
                                  "result_bytes_out": O_back.numel() * 2 + L_back.numel() * 4, "max_abs_diff_vs_one_call": diff}
    if args.from_pool:
        # shards as a later chunk of a long prompt finds them: in the token pool, at scattered slots
        n_rows = sum(s.k.shape[0] for s in pc.shards)
        S = 1 << (n_rows - 1).bit_length()
        kp = torch.zeros((S, pc.Hkv, pc.D), dtype=torch.bfloat16, device=dev)
        vp = torch.zeros_like(kp)
        perm = torch.from_numpy(np.random.default_rng(98).permutation(S)[:n_rows].astype(np.int32)).to(dev)
        slots, o = [], 0
        for s in pc.shards:
            slots.append(perm[o:o + s.k.shape[0]].contiguous()); o += s.k.shape[0]
            esp.esp_kv_append(s.k, s.v, slots[-1], kp, vp)
        ws_pool = torch.empty(max(esp.esp_prefill_pool_workspace_bytes(pc.Tq, max(s.k.shape[0] for s in pc.shards), pc.batch, pc.Hq,
                                                                       pc.Hkv, pc.D), 256), dtype=torch.uint8, device=dev)
        pool_O = [torch.empty_like(pc.q) for _ in part_O]; pool_L = [torch.empty_like(x) for x in part_L]
        dense_O = [torch.empty_like(pc.q) for _ in part_O]

        direct_O = [torch.empty_like(pc.q) for _ in part_O]; direct_L = [torch.empty_like(x) for x in part_L]

        def prefill_all(from_pool):
            for i, s in enumerate(pc.shards):
                if from_pool == "direct":
                    esp.esp_partial_attn_prefill_pool_direct(pc.q, kp, vp, slots[i], pc.q_pos, s.kv_pos,
                                                             None if single else pc.cu_q, None if single else s.cu_kv,
                                                             None if single else pc.max_q, None if single else s.max_kv,
                                                             softmax_scale=pc.scale, causal=pc.causal, O=direct_O[i], LSE=direct_L[i],
                                                             workspace=ws_pf)
                elif from_pool:
                    esp.esp_partial_attn_prefill_pool(pc.q, kp, vp, slots[i], pc.q_pos, s.kv_pos,
                                                      None if single else pc.cu_q, None if single else s.cu_kv,
                                                      None if single else pc.max_q, None if single else s.max_kv,
                                                      softmax_scale=pc.scale, causal=pc.causal, O=pool_O[i], LSE=pool_L[i],
                                                      workspace=ws_pool)
                else:
                    esp.esp_partial_attn_prefill(pc.q, s.k, s.v, pc.q_pos, s.kv_pos,
                                                 None if single else pc.cu_q, None if single else s.cu_kv,
                                                 None if single else pc.max_q, None if single else s.max_kv,
                                                 softmax_scale=pc.scale, causal=pc.causal, O=dense_O[i], LSE=part_L[i], workspace=ws_pf)

        times = {}
        for mode in (False, True, "direct", False, True, "direct"):
            prefill_all(mode); torch.cuda.synchronize()
            e0, e1 = ev(), ev()
            e0.record()
            for _ in range(args.steps):
                prefill_all(mode)
            e1.record(); torch.cuda.synchronize()
            times.setdefault(mode, []).append(e0.elapsed_time(e1) / args.steps)
        t_dense, t_pool, t_direct = min(times[False]), min(times[True]), min(times["direct"])
        same_direct = all(torch.equal(a_, b_) for a_, b_ in zip(dense_O, direct_O)) and all(torch.equal(a_, b_) for a_, b_ in zip(part_L, direct_L))
        same = all(torch.equal(a_, b_) for a_, b_ in zip(dense_O, pool_O)) and all(torch.equal(a_, b_) for a_, b_ in zip(part_L, pool_L))
        moved = 2 * 2 * n_rows * pc.Hkv * pc.D * 2                  # K and V, read from the pool and written to the staging rows
        result["from_pool"] = {"ms_dense": t_dense, "ms_from_pool": t_pool, "overhead_pct": 100.0 * (t_pool / t_dense - 1.0),
                               "rows": n_rows, "gather_bytes": moved, "gather_gbs": moved / ((t_pool - t_dense) * 1e-3) / 1e9,
                               "same_bits_as_dense": bool(same),
                               "ms_direct": t_direct, "direct_overhead_pct": 100.0 * (t_direct / t_dense - 1.0),
                               "direct_same_bits_as_dense": bool(same_direct)}
    if args.workload == "lwm7b" and os.path.exists(args.traffic_json):
        tr = json.load(open(args.traffic_json))
        result["roofline"]["traffic"] = tr.get("prefill_kernel")
        if "roofline_decode" in result:
            result["roofline_decode"]["traffic"] = tr.get("decode_partial_kernel")
    if not args.no_cpu_baseline:
        import oracle
        note("timing the CPU oracle on the parity samples of this workload")
        result["cpu_baseline"] = cpu_baseline(pc, dc, wl, oracle)
        note("done")
    if args.workload == "lwm7b" and not args.no_extra:
        # the other full-size configurations, one after the other with the pools freed in between: the same
        # step, fewer repetitions, reported under keys of their own (they are not part of `value`)
        del step, pc, dc, ws_pf, part_O, part_L, out_O, out_L, ws_dc, dO, dL, mO, mL
        torch.cuda.empty_cache()
        for which, reps in (("long", 5), ("mixed", 5)):
            note("extra workload '%s': %d timed steps" % (which, reps))
            pc2, dc2, name2 = make_workload(which, wl, np, dev)
            step2 = Step(esp, torch, pc2, dc2, dev)
            recs2, _ = time_steps(torch, step2, reps, 1)
            s2 = summarize(recs2, pc2, dc2)
            tag = "c4" if which == "long" else "c5"
            result["prefill_" + tag] = dict(s2["prefill"], workload=name2, steps=reps, frac=s2["prefill"]["tflops"] / PEAK_BF16_TFLOPS,
                                            bound="mfma", peak=PEAK_BF16_TFLOPS, unit="TFLOP/s")
            if dc2 is not None:
                result["decode_" + tag] = dict(s2["decode"], workload=name2, steps=reps, frac=s2["decode"]["gbs"] / PEAK_HBM_GBS,
                                               bound="hbm", peak=PEAK_HBM_GBS, unit="GB/s")
            del step2, pc2, dc2, recs2
            torch.cuda.empty_cache()
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
