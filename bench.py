#!/usr/bin/env python3
"""Benchmark of the resume + checkpoint-emit prefill on one MI355X.

Headline workload (configs[4], the largest single-GPU configuration): a layer-group serving step.
256 concurrent requests with suffix lengths log-uniform in [64, 8192] run through 8 stacked
GatedDeltaNet layers of 16 heads (d_k = d_v = 128, bf16 inputs, fp32 state and outputs).  Each
request gathers its start state by slot id from a 4096-slot HBM checkpoint pool (32 GiB of fp32
states), replays its suffix and stores the exact state at every multiple of 1024 inside the suffix
and at its end to freshly assigned slots.  A step is ONE call of gdn_resume_prefill over the whole
batch (host planning, plan upload, one fused launch: 32768 chains).  Inputs are generated on the
device with a fixed seed and are resident in HBM before the timed region.

Prints ONE JSON line.  `value` = suffix tokens per second through the whole 8-layer group.
`roofline` is that of the dominant kernel (gdn_fused_kernel, one launch per step) from HIP events
the library records on the launch stream: algorithmic HBM bytes over the launch duration against
8 TB/s (the binding roof: 140 flop per byte against a ridge of 312), with the matrix-core view
beside it.  configs[1] (batch 1, latency bound) is reported as the side object `latency`.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

N_PREFIX, M_CKPT, HEADS, D = 8192, 16, 16, 128
N_DRAWS = 16
SEED = 1001
C = 64
# algorithmic flops per token.head (dense tiles, chunk 64): chunk preparation and recurrence
FLOP_PREP = C * (6 * D + 2 * D)             # K K^T, K Q^T, W (each 2 C d_k) + U~ (2 C d_v)
FLOP_RECUR = 6 * D * D + 2 * C * D          # W S^T, Q S^T, state update (2 d_k d_v each) + P U (2 C d_v)
# algorithmic HBM bytes per token.head: q, k, v in bf16, beta, gate, o in fp32 (bf16 o: 2 d_v less)
BYTES_TOKEN_HEAD = (2 * D + D) * 2 + 2 * 2 + D * 4
BYTES_TOKEN_HEAD_BF16_O = (2 * D + D) * 2 + 2 * 2 + D * 2
STATE_BYTES = D * D * 4                      # one head's state, read once per chain and written once per emission
SLAB_TOKENS = 32 * C           # configs[1]: the latency variant's slab at 16 chains (checked against the launch count)
PEAK_MFMA_TFLOPS = 2500.0                   # dense fp16/bf16 MFMA, MI355X
PEAK_HBM_GBS = 8000.0
PROFILES = os.path.join(ROOT, "profiles")


def measured_traffic(name: str, key: str):
    """A figure from a committed rocprofv3 summary under profiles/ (a line `key: number`), or None."""
    try:
        with open(os.path.join(PROFILES, name)) as f:
            m = re.search(r"^" + re.escape(key) + r":\s*([0-9.eE+-]+)", f.read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def bench_config4(args, torch, B, dev):
    """The headline: configs[4] at full size, one call per step."""
    from paper_2605_05219_amd.device_call import config4_device
    step = config4_device()
    n_chains = step.n_req * step.L * step.H
    th = step.T * step.L * step.H                       # token.heads of one step
    state_moves = (step.n_req + step.n_emit) * step.L * step.H
    alg_bytes = th * BYTES_TOKEN_HEAD + state_moves * STATE_BYTES
    alg_flops = th * (FLOP_PREP + FLOP_RECUR)

    for _ in range(args.warmup):
        step.run()
    torch.cuda.synchronize()

    def timed(events):
        if events:
            B.gdn_profile_enable(True)
        torch.cuda.synchronize()
        ta = time.perf_counter()
        for _ in range(args.steps):
            step.run()
        torch.cuda.synchronize()
        tb = time.perf_counter()
        if not events:
            return tb - ta, 0.0, 0
        _, k_ms, n_prof, _, k_n = B.gdn_profile_collect()
        B.gdn_profile_enable(False)
        assert n_prof == args.steps and k_n == args.steps, (n_prof, k_n)
        return tb - ta, k_ms, k_n

    if args.no_kernel_events:
        wall, k_ms, k_n = timed(False)
    elif args.events_in_timed_region:
        wall, k_ms, k_n = timed(True)
    else:
        wall = timed(False)[0]
        _, k_ms, k_n = timed(True)

    ms = 1e3 * wall / args.steps
    out = {
        "metric": "recomputed suffix tokens/sec/GPU (resume+ckpt emit)",
        "value": step.T / (ms * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "config": {
            "workload": "configs[4]: layer-group serving step, 256 requests x 8 GatedDeltaNet layers x 16 heads, "
                        "d_k=d_v=128, suffix ~ logU[64,8192], 4096-slot fp32 checkpoint pool in HBM addressed by int32 slot "
                        "ids, states stored every 1024 positions and at each request's end; bf16 inputs, fp32 state and outputs",
            "seed": 1004, "requests": step.n_req, "layers": step.L, "heads": step.H,
            "suffix_tokens_per_layer": step.T, "chains": n_chains, "emitted_states": step.n_emit,
            "token_layers_per_s": step.T * step.L / (ms * 1e-3),
            "token_heads_per_s": th / (ms * 1e-3),
            "workspace_bytes": int(step.workspace.numel()),
            "chunk": C,
        },
    }
    if not args.no_kernel_events:
        launch_ms = k_ms / k_n
        gbs = alg_bytes / (launch_ms * 1e-3) / 1e9
        tfl = alg_flops / (launch_ms * 1e-3) / 1e12
        traffic = measured_traffic("fused_kernel_config4_hbm_traffic.txt", "traffic_bytes_per_launch")
        out["roofline"] = {
            "bound": "hbm", "kernel": "gdn_fused_kernel (one launch per step)",
            "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
            # HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, scaled by a copy of known size),
            # read from the committed summary of the same command; None when that file is absent
            "traffic": traffic,
            "avg_launch_ms": launch_ms, "launches": k_n,
            "algorithmic_bytes_per_launch": alg_bytes,
            "bytes_per_token_head": BYTES_TOKEN_HEAD, "token_heads_per_launch": th,
            "state_bytes_per_launch": state_moves * STATE_BYTES,
            "flop_per_byte": alg_flops / alg_bytes, "ridge_flop_per_byte": PEAK_MFMA_TFLOPS * 1e3 / PEAK_HBM_GBS,
            "mfma_view": {"achieved": tfl, "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": tfl / PEAK_MFMA_TFLOPS,
                          "flop_per_token_head": FLOP_PREP + FLOP_RECUR,
                          "at_hbm_peak_frac": PEAK_HBM_GBS * 1e9 * (alg_flops / alg_bytes) / 1e12 / PEAK_MFMA_TFLOPS},
            "host_ms_per_step_outside_the_kernel": ms - launch_ms,
        }
    if args.main_only:
        return out, None

    # ---- the same step with bf16 outputs (a throughput variant with its own tolerance, 2e-3 + 2^-8: o in fp32 is 40 % of
    #      the algorithmic bytes)
    try:
        o16 = torch.empty(step.o.shape, dtype=torch.bfloat16, device=dev)
        s16 = dataclasses.replace(step, o=o16, shape=B.make_shape(step.L, step.H, step.H, step.d, step.d, "bf16", "bf16", step.T))
        for _ in range(2):
            s16.run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(5):
            s16.run()
        torch.cuda.synchronize()
        ms16 = 1e3 * (time.perf_counter() - t0) / 5
        b16 = th * BYTES_TOKEN_HEAD_BF16_O + state_moves * STATE_BYTES
        out["bf16_outputs"] = {"ms_per_step": ms16, "tokens_per_s": step.T / (ms16 * 1e-3), "algorithmic_bytes": b16,
                               "achieved_gbs": b16 / (ms16 * 1e-3) / 1e9, "frac_of_hbm_peak": b16 / (ms16 * 1e-3) / 1e9 / PEAK_HBM_GBS,
                               "mfma_frac": alg_flops / (ms16 * 1e-3) / 1e12 / PEAK_MFMA_TFLOPS,
                               "note": "whole call on the host clock; same step with o stored as bf16"}
        del o16, s16
    except Exception as exc:
        out["bf16_outputs"] = {"error": str(exc)}

    # ---- the oracle on the host cores: a bounded, seeded subsample of the same step (every layer and head of 16
    #      48 seeded requests, then layer 0 of the other requests, until about 25 s are spent)
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import gdn_oracle as orc
        rng = np.random.default_rng(4004)
        picks = sorted(int(x) for x in rng.choice(step.n_req, size=48, replace=False))
        jobs = [(r, list(range(step.L))) for r in picks] + [(r, [0]) for r in range(step.n_req) if r not in picks]
        subs = []
        for r, layers in jobs:                       # host copies made outside the timed loop
            sub = step.host_request(r, layers)
            start = step.pool[int(step.src_slot[r])][layers].cpu().numpy()[None]
            subs.append((sub, start))
        orc.resume_prefill(*subs[0][0].streams.slice(0, 64).fields(), [0, 64], [0], [-1], [0, 0], [])      # load + warm
        tc0 = time.perf_counter()
        th_cpu = n_done = 0
        for sub, start in subs:
            orc.resume_prefill(*sub.streams.fields(), sub.cu_seqlens, sub.start_pos, [0], sub.emit_cu, sub.emit_pos,
                               state_src=start)
            th_cpu += sub.total_tokens * sub.L * sub.H_v
            n_done += 1
            if time.perf_counter() - tc0 > 25.0:
                break
        tc1 = time.perf_counter()
        per_token = step.L * step.H                   # token.heads one suffix token costs in this workload
        cpu = {
            "value": th_cpu / per_token / (tc1 - tc0), "unit": "tokens/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"{n_done} of {len(subs)} oracle calls on the same step's inputs: all 8 layers x 16 heads of 48 seeded requests, "
                      f"then layer 0 of the other requests; {th_cpu} token.heads in {tc1 - tc0:.1f} s; fp64 token loop, one (layer, head) "
                      f"chain per thread; tokens/s = token.heads/s / {per_token} (a token passes 8 layers x 16 heads)",
            "token_heads_per_s": th_cpu / (tc1 - tc0), "seconds": tc1 - tc0,
        }
    del step
    torch.cuda.empty_cache()

    out["grouped_value_heads"] = bench_grouped_heads(torch, B)
    return out, cpu


def bench_grouped_heads(torch, B, reps: int = 5):
    """configs[4]'s recipe with grouped value heads: 8 query/key heads under the 16 value heads.  Two value heads of a
    query/key head then share a workgroup of eight waves that reads and stages their q and k rows once (the library's choice
    for a call of this size; gdn_tune_fused_pair switches it off for the comparison)."""
    from paper_2605_05219_amd.device_call import config4_device
    try:
        gv = config4_device(seed=1044, H_qk=8, n_slots=2048)
        th_g = gv.T * gv.L * gv.H
        moves_g = (gv.n_req + gv.n_emit) * gv.L * gv.H
        res = {}
        for name, pair, per_th in (("one_head_per_workgroup", 0, BYTES_TOKEN_HEAD), ("two_heads_per_workgroup", 1, BYTES_TOKEN_HEAD - 2 * 128)):
            prev = B.gdn_tune_fused_pair(pair)
            try:
                for _ in range(2):
                    gv.run()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(reps):
                    gv.run()
                torch.cuda.synchronize()
            finally:
                B.gdn_tune_fused_pair(prev)
            msg = 1e3 * (time.perf_counter() - t0) / reps
            bts = th_g * per_th + moves_g * STATE_BYTES
            res[name] = {"ms_per_step": msg, "tokens_per_s": gv.T / (msg * 1e-3), "algorithmic_bytes": bts,
                         "bytes_per_token_head": per_th, "achieved_gbs": bts / (msg * 1e-3) / 1e9,
                         "frac_of_hbm_peak": bts / (msg * 1e-3) / 1e9 / PEAK_HBM_GBS, "launches": reps + 2}
        res["note"] = ("configs[4]'s recipe with H_qk = 8, H_v = 16 (seed 1044, 2048-slot pool); whole call on the host clock; "
                       "with two heads per workgroup a q and a k row (256 bytes each) are read once per pair of value heads")
        del gv
        torch.cuda.empty_cache()
        return res
    except Exception as exc:
        return {"error": str(exc)}


def bench_other_configs(torch, B, wl, reps: int = 20):
    """configs[2] and configs[3] as specified, one call each on the library's own choice of path (both take the fused
    kernel), start states seeded random states; whole call on the host clock.  configs[3]: 32 value heads on 16 query/key
    heads, bound by its longest chain."""
    from paper_2605_05219_amd.device_call import GpuCall
    out = {}
    for name, mk in (("configs[2]", wl.config2), ("configs[3]", wl.config3)):
        try:
            sc = mk(B.gdn_deepest_ckpt)
            call = sc.resume
            rng = np.random.default_rng(2003)
            pool = (rng.standard_normal((sc.n_slots,) + sc.build.slot_shape) * 0.3).astype(np.float32)
            g = GpuCall(call, pool)
            lens = np.diff(call.cu_seqlens)
            for _ in range(3):
                g.run()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                g.run()
            torch.cuda.synchronize()
            ms = 1e3 * (time.perf_counter() - t0) / reps
            th = call.total_tokens * call.L * call.H_v
            per_th = (2 * D * call.H_qk // call.H_v + D) * 2 + 2 * 2 + D * 4
            out[name] = {"ms_per_call": ms, "tokens_per_s": call.total_tokens / (ms * 1e-3), "requests": call.n_req,
                         "chains": call.n_req * call.L * call.H_v, "suffix_tokens": int(call.total_tokens),
                         "longest_chain_chunks": int((lens.max() + C - 1) // C), "launches": reps + 3,
                         "algorithmic_gbs": th * per_th / (ms * 1e-3) / 1e9,
                         "us_per_chunk_of_the_longest_chain": 1e3 * ms / float((lens.max() + C - 1) // C)}
            del g
        except Exception as exc:
            out[name] = {"error": repr(exc)}
    torch.cuda.empty_cache()
    return out


def bench_ckpt_copy(torch, B, dev):
    """Standalone checkpoint pool copies (HBM bound): 256 states of 1 MiB gathered, then scattered."""
    out = {}
    # ---- standalone checkpoint pool copies (HBM bound): 256 states of 1 MiB each way
    try:
        n_copy, elems = 256, HEADS * D * D
        big = torch.randn((n_copy * 2, elems), dtype=torch.float32, device=dev)
        stage = torch.empty((n_copy, elems), dtype=torch.float32, device=dev)
        ids = np.random.default_rng(SEED).permutation(n_copy * 2)[:n_copy].astype(np.int32)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        for _ in range(3):
            B.ckpt_gather(big, ids, stage)
            B.ckpt_scatter(big, ids, stage)
        reps = 20
        ev[0].record()
        for _ in range(reps):
            B.ckpt_gather(big, ids, stage)
        ev[1].record()
        for _ in range(reps):
            B.ckpt_scatter(big, ids, stage)
        ev[2].record()
        torch.cuda.synchronize()
        nbytes = 2.0 * n_copy * elems * 4
        out["ckpt_copy"] = {
            "states": n_copy, "state_bytes": elems * 4,
            "gather_gbs": nbytes * reps / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9,
            "scatter_gbs": nbytes * reps / (ev[1].elapsed_time(ev[2]) * 1e-3) / 1e9,
            "peak_gbs": PEAK_HBM_GBS,
        }
        del big, stage
    except Exception as exc:  # the copies are a side measurement; never lose the main line
        out["ckpt_copy"] = {"error": str(exc)}

    return out["ckpt_copy"]


def bench_config1(args, torch, B, wl, dev):
    """configs[1], batch 1: latency bound by construction (16 chains of up to 128 dependent chunk steps)."""
    from paper_2605_05219_amd.device_call import GpuCall
    steps, warmup = args.latency_steps, 16
    # ---- the cache entry and the requests (host side, seeded)
    sc = wl.config1(B.gdn_deepest_ckpt, seed=SEED, n_draws=N_DRAWS, N=N_PREFIX, M=M_CKPT, H=HEADS, d=D)
    n_slots = M_CKPT + M_CKPT + 1
    pool = torch.zeros((n_slots, 1, HEADS, D, D), dtype=torch.float32, device=dev)
    build = GpuCall(sc.build, pool)
    build.run()                       # fills slots 0..M-1 with the prefix checkpoints (untimed set-up)
    torch.cuda.synchronize()

    # one call object per draw (its own packed suffix tokens, resident in HBM)
    r = sc.resume
    calls = []
    for i in range(N_DRAWS):
        lo, hi = int(r.cu_seqlens[i]), int(r.cu_seqlens[i + 1])
        e0, e1 = int(r.emit_cu[i]), int(r.emit_cu[i + 1])
        one = wl.pack_call(1, HEADS, HEADS, D, D, "bf16", [r.streams.slice(lo, hi)], [r.start_pos[i]],
                           [r.src_slot[i]], [list(r.emit_pos[e0:e1])],
                           [list(range(M_CKPT, M_CKPT + e1 - e0))], n_slots)
        calls.append(GpuCall(one, pool))
    suffix = [c.call.total_tokens for c in calls]

    def step(i):
        calls[i % N_DRAWS].run()

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()

    def timed(events):
        if events:
            B.gdn_profile_enable(True)
        torch.cuda.synchronize()
        ta = time.perf_counter()
        for i in range(steps):
            step(i)
        torch.cuda.synchronize()
        tb = time.perf_counter()
        if not events:
            return tb - ta, 0.0, 0.0, 0, 0
        p_ms, r_ms, n_prof, p_n, r_n = B.gdn_profile_collect()
        B.gdn_profile_enable(False)
        assert n_prof == steps
        return tb - ta, p_ms, r_ms, p_n, r_n

    # The timed region; the per-kernel durations come from HIP events the library records on the
    # launch stream between its kernels, by default in an immediate repeat of the same steps so
    # that the events' own cost stays out of `value`.
    events_wall = None
    wall_s = timed(False)[0]
    events_wall, prep_ms, recur_ms, prep_n, recur_n = timed(True)

    tokens = sum(suffix[i % N_DRAWS] for i in range(steps))
    wall = wall_s
    token_heads = tokens * HEADS
    out = {
        "workload": "configs[1]: 1 layer, batch 1, 16 heads, d_k=d_v=128, N=8192, M=16 checkpoints at 512 i, depth ~ U[0,N), "
                    "bf16 inputs, fp32 state and outputs; a step is one request",
        "tokens_per_s": tokens / wall, "ms_per_step": 1e3 * wall / steps, "steps": steps,
        "draws": N_DRAWS, "seed": SEED, "depths": [int(x) for x in r.meta["depths"]], "suffix_tokens": suffix,
        "mean_suffix_tokens": float(np.mean(suffix)),
        "emits_per_step": float(np.mean([int(r.emit_cu[i + 1] - r.emit_cu[i]) for i in range(N_DRAWS)])),
    }
    if True:
        # A step prepares its first slab (32 chunk rounds) in a launch of its own; every recurrence launch
        # but the last also prepares the next slab (gdn_quad_overlap_kernel).  The recurrence launches are
        # therefore priced at the recurrence's flops of every token plus the preparation's flops of the
        # tokens beyond the first slab; the preparation launches at the first slab's preparation flops.
        step_suffix = [suffix[i % N_DRAWS] for i in range(steps)]
        slabs_ok = recur_n == sum(-(-t // SLAB_TOKENS) for t in step_suffix) and prep_n == steps
        later = sum(max(0, t - SLAB_TOKENS) for t in step_suffix) * HEADS if slabs_ok else 0
        first = token_heads - later
        rec_dom = recur_ms >= prep_ms
        dom = "recurrence launches (gdn_quad_overlap_kernel, gdn_recur_quad_kernel)" if rec_dom else "gdn_prep_kernel"
        dom_ms, dom_n = (recur_ms, recur_n) if rec_dom else (prep_ms, prep_n)
        dom_flops_total = token_heads * FLOP_RECUR + later * FLOP_PREP if rec_dom else first * FLOP_PREP
        dom_flop = dom_flops_total / token_heads
        # measured HBM bytes per token.head of these launches (rocprofv3 --pmc, committed summary), or None
        dom_traffic = measured_traffic("prefill_kernels_config1_hbm_traffic.txt",
                                       "recurrence_launch_bytes_per_token_head" if rec_dom else "first_preparation_launch_bytes_per_token_head")
        units_per_launch = token_heads / dom_n
        achieved = dom_flops_total / (dom_ms * 1e-3) / 1e12
        out["roofline"] = {
            "bound": "mfma", "kernel": dom,
            "achieved": achieved, "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s",
            "frac": achieved / PEAK_MFMA_TFLOPS,
            # HBM bytes per launch: rocprofv3 FETCH_SIZE + WRITE_SIZE per token.head of this build
            # (profiles/, scaled by the copy-kernel calibration) x the token.heads of one launch
            "traffic": None if dom_traffic is None else dom_traffic * units_per_launch,
            "avg_launch_ms": dom_ms / dom_n,
            "launches": dom_n,
            "token_heads_per_launch": units_per_launch,
            "flop_per_token_head": dom_flop,
        }
        # The same launches against the memory roof: by arithmetic intensity (flop per algorithmic byte, below the
        # ridge of 2500 TFLOP/s over 8 TB/s = 312) the memory roof is the one a saturated run of this path would hit
        # first; this batch-1 workload saturates neither (it is bound by the per-chunk dependent chain).
        if rec_dom:
            in_bytes = (2 * D + D) * 2 + 2 * 2          # q, k, v, beta, gate per token.head (read by the preparation)
            dom_bytes = token_heads * (D * 4) + later * in_bytes
            gbs = dom_bytes / (dom_ms * 1e-3) / 1e9
            out["roofline"]["memory_view"] = {
                "algorithmic_bytes_per_launch": dom_bytes / dom_n, "achieved_gbs": gbs, "peak_gbs": PEAK_HBM_GBS,
                "frac": gbs / PEAK_HBM_GBS, "flop_per_byte": dom_flops_total / dom_bytes,
                "ridge_flop_per_byte": PEAK_MFMA_TFLOPS * 1e3 / PEAK_HBM_GBS,
            }
        out["kernels"] = {
            "gdn_prep_kernel": {"avg_ms": prep_ms / steps, "launches": prep_n,
                                "avg_launch_ms": prep_ms / max(prep_n, 1),
                                "tflops": first * FLOP_PREP / (prep_ms * 1e-3) / 1e12},
            "gdn_recur_kernel": {"avg_ms": recur_ms / steps, "launches": recur_n,
                                 "avg_launch_ms": recur_ms / max(recur_n, 1),
                                 "tflops": (token_heads * FLOP_RECUR + later * FLOP_PREP) / (recur_ms * 1e-3) / 1e12},
            "token_heads_prepared_in_recurrence_launches": later,
            "both_kernels_hbm_gbs_algorithmic": token_heads * BYTES_TOKEN_HEAD / ((prep_ms + recur_ms) * 1e-3) / 1e9,
            "events": "immediate repeat of the timed steps",
            "ms_per_step_with_events": 1e3 * events_wall / steps,
            "other_ms_per_step_with_events": 1e3 * events_wall / steps - (prep_ms + recur_ms) / steps,
        }

    # ---- latency against suffix length (Sec. 6, overhead decomposition: the resume cost is a small constant
    #      for loading the checkpoint plus a term linear in the replayed suffix): every draw timed on its own
    try:
        per_draw = []
        for i in range(N_DRAWS):
            for _ in range(2):
                step(i)
            torch.cuda.synchronize()
            ta = time.perf_counter()
            for _ in range(8):
                step(i)
            torch.cuda.synchronize()
            per_draw.append((suffix[i], 1e3 * (time.perf_counter() - ta) / 8))
        xs = np.array([p_[0] / C for p_ in per_draw], dtype=np.float64)
        ys = np.array([p_[1] for p_ in per_draw], dtype=np.float64)
        slope, offset = np.polyfit(xs, ys, 1)
        out["latency_vs_suffix"] = {
            "suffix_tokens_ms": sorted(set((int(a), round(float(b), 5)) for a, b in per_draw)),
            "fit_ms": {"per_chunk_step": float(slope), "offset": float(offset)},
            "note": "whole call (planning, upload, every launch), 8 back-to-back calls per draw; chunk step = 64 tokens",
        }
    except Exception as exc:
        out["latency_vs_suffix"] = {"error": str(exc)}

    return out, calls, pool, suffix


def side_measurements(args, torch, B, wl, dev, calls, pool, suffix, wall_cfg1_ms):
    """Side objects: pool copies, host tier, decode step, layer front/back end, attention side, optional sweeps."""
    from paper_2605_05219_amd.device_call import GpuCall
    out = {}
    r_steps = args.latency_steps

    def step(i):
        calls[i % N_DRAWS].run()

    out["ckpt_copy"] = bench_ckpt_copy(torch, B, dev)
    out["other_configs"] = bench_other_configs(torch, B, wl)

    # ---- host tier (Sec. 6: loading the stored checkpoint from host memory is overhead (i) of a hit): the same
    #      draws with the checkpoint pool in pinned host memory, and the raw host -> HBM state copy rate
    try:
        host_pool = pool.cpu().pin_memory()
        ws_host = torch.empty(max(B.gdn_workspace_bytes_host(c.shape, 1, c.call.total_tokens, int(c.call.emit_pos.size))
                                  for c in calls), dtype=torch.uint8, device=dev)

        def host_step(i):
            c = calls[i % N_DRAWS]
            cc = c.call
            B.gdn_resume_prefill_host(c.shape, c.q, c.k, c.v, c.beta, c.gate, cc.cu_seqlens, cc.start_pos, host_pool,
                                      cc.src_slot, cc.emit_cu, cc.emit_pos, pool, cc.emit_slot, c.o, ws_host)
        for i in range(N_DRAWS):
            host_step(i)
        torch.cuda.synchronize()
        ta = time.perf_counter()
        for i in range(r_steps):
            host_step(i)
        torch.cuda.synchronize()
        host_ms = 1e3 * (time.perf_counter() - ta) / r_steps
        n_f = 64
        stage_f = torch.empty((n_f,) + tuple(pool.shape[1:]), dtype=torch.float32, device=dev)
        big_host = torch.randn((n_f,) + tuple(pool.shape[1:]), dtype=torch.float32).pin_memory()
        ids_f = np.arange(n_f, dtype=np.int32)
        B.ckpt_fetch_host(big_host, ids_f, stage_f, ids_f)
        torch.cuda.synchronize()
        ta = time.perf_counter()
        for _ in range(4):
            B.ckpt_fetch_host(big_host, ids_f, stage_f, ids_f)
        torch.cuda.synchronize()
        f_s = (time.perf_counter() - ta) / 4
        out["host_tier"] = {
            "ms_per_step_pool_in_pinned_host_memory": host_ms,
            "ms_per_step_pool_in_hbm": wall_cfg1_ms,
            "state_bytes": int(pool[0].numel() * 4),
            "fetch_gbs": n_f * pool[0].numel() * 4 / f_s / 1e9,
            "draws_that_load_a_state": int(sum(int(c.call.src_slot[0]) >= 0 for c in calls)),
            "note": "start state fetched from pinned host memory by workgroups appended to the first preparation launch",
        }
        del stage_f, big_host, ws_host
    except Exception as exc:
        out["host_tier"] = {"error": str(exc)}

    # ---- decode step (one token per request, states updated in place): 1024 requests x 16 heads, HBM bound
    try:
        n_dec = 1024                # 1 GiB of states: four times the memory-side cache
        dpool = torch.randn((n_dec, 1, HEADS, D, D), dtype=torch.float32, device=dev) * 0.1
        dshape = B.make_shape(1, HEADS, HEADS, D, D, "bf16", "f32", n_dec)
        dq = torch.nn.functional.normalize(torch.randn((1, n_dec, HEADS, D), device=dev), dim=-1).bfloat16()
        dk = torch.nn.functional.normalize(torch.randn((1, n_dec, HEADS, D), device=dev), dim=-1).bfloat16()
        dv = torch.randn((1, n_dec, HEADS, D), device=dev).bfloat16()
        db = torch.sigmoid(torch.randn((1, n_dec, HEADS), device=dev)).bfloat16()
        dg = torch.exp(-torch.nn.functional.softplus(torch.randn((1, n_dec, HEADS), device=dev))).bfloat16()
        do = torch.empty((1, n_dec, HEADS, D), dtype=torch.float32, device=dev)
        dslots = np.arange(n_dec, dtype=np.int32)
        for _ in range(3):
            B.gdn_decode_step(dshape, dq, dk, dv, db, dg, dpool, dslots, do)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        reps = 20
        ev[0].record()
        for _ in range(reps):
            B.gdn_decode_step(dshape, dq, dk, dv, db, dg, dpool, dslots, do)
        ev[1].record()
        torch.cuda.synchronize()
        dbytes = 2.0 * n_dec * HEADS * D * D * 4
        dms = ev[0].elapsed_time(ev[1]) / reps
        out["decode_step"] = {"requests": n_dec, "state_bytes_read_and_written": dbytes, "ms": dms,
                              "gbs": dbytes / (dms * 1e-3) / 1e9, "peak_gbs": PEAK_HBM_GBS,
                              "tokens_per_s": n_dec / (dms * 1e-3)}
        del dpool
    except Exception as exc:
        out["decode_step"] = {"error": str(exc)}

    # ---- optional: one call of k requests (k configs[1]-style draws packed together), to show how the variant
    #      choice (latency variant, two or four slices per workgroup, fused kernel) behaves between the
    #      batch-1 bench line and the throughput regime
    if args.batch_sweep:
        sweep = []
        for kreq in (1, 2, 4, 8, 16, 32, 64):
            try:
                scs = wl.config1(B.gdn_deepest_ckpt, seed=SEED, n_draws=kreq, N=N_PREFIX, M=M_CKPT, H=HEADS, d=D)
                gk = GpuCall(scs.resume, torch.randn((scs.n_slots, 1, HEADS, D, D), device=dev) * 0.1)
                for _ in range(2):
                    gk.run()
                torch.cuda.synchronize()
                tk0 = time.perf_counter()
                for _ in range(5):
                    gk.run()
                torch.cuda.synchronize()
                msk = 1e3 * (time.perf_counter() - tk0) / 5
                sweep.append({"requests": kreq, "chains": kreq * HEADS, "suffix_tokens": scs.resume.total_tokens,
                              "longest": int(np.diff(scs.resume.cu_seqlens).max()), "ms_per_call": msk,
                              "tokens_per_s": scs.resume.total_tokens / (msk * 1e-3)})
                del gk
            except Exception as exc:
                sweep.append({"requests": kreq, "error": str(exc)})
        out["batch_sweep"] = sweep

    # ---- layer front end (short convolution + SiLU + q/k norm + gates, resumed from stored convolution states) and
    #      back end (gated output norm): memory bound; 32 requests x 2048 tokens of this layer shape, bf16
    try:
        from paper_2605_05219_amd import layer as LY
        n_rq, ln = 32, 2048
        Tl, Cl = n_rq * ln, 3 * HEADS * D
        lsh = LY.make_layer_shape(HEADS, HEADS, D, D, 4, "bf16", "bf16", "f32")
        bf = lambda *sh: torch.randn(sh, device=dev).bfloat16()
        xq, ap, bp, zz = bf(Tl, Cl), bf(Tl, HEADS), bf(Tl, HEADS), bf(Tl, HEADS, D)
        cw, cb = torch.randn((Cl, 4), device=dev) * 0.5, torch.randn(Cl, device=dev) * 0.1
        Al, dtb, nw = torch.zeros(HEADS, device=dev), torch.zeros(HEADS, device=dev), torch.ones(D, device=dev)
        cpool = bf(2 * n_rq, 3, Cl)
        lq, lk, lv = (torch.empty((Tl, HEADS, D), dtype=torch.bfloat16, device=dev) for _ in range(3))
        lb, lg = (torch.empty((Tl, HEADS), dtype=torch.bfloat16, device=dev) for _ in range(2))
        lo_ = torch.randn((Tl, HEADS, D), device=dev)
        ly = torch.empty((Tl, HEADS, D), dtype=torch.bfloat16, device=dev)
        lcu = np.arange(n_rq + 1, dtype=np.int32) * ln
        lst = np.full(n_rq, 4096, np.int32)
        lws = torch.empty(LY.gdn_layer_workspace_bytes(n_rq, n_rq), dtype=torch.uint8, device=dev)

        def front():
            LY.gdn_layer_inputs(lsh, xq, cw, cb, ap, bp, Al, dtb, lcu, lst, cpool, np.arange(n_rq, dtype=np.int32),
                                np.arange(n_rq + 1, dtype=np.int32), lst + ln, cpool, n_rq + np.arange(n_rq, dtype=np.int32),
                                lq, lk, lv, lb, lg, lws)

        def back():
            LY.gdn_layer_output(lsh, lo_, zz, nw, ly, Tl)

        res = {}
        for name, fn, nbytes in (("inputs", front, Tl * (2 * Cl * 2 + 4 * HEADS * 2)), ("output", back, Tl * HEADS * D * (4 + 2 + 2))):
            for _ in range(3):
                fn()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            reps = 20
            ev[0].record()
            for _ in range(reps):
                fn()
            ev[1].record()
            torch.cuda.synchronize()
            ms = ev[0].elapsed_time(ev[1]) / reps
            res[name] = {"ms": ms, "bytes_read_and_written": nbytes, "gbs": nbytes / (ms * 1e-3) / 1e9}
        out["layer_io"] = {"tokens": Tl, "requests": n_rq, "channels": Cl, "peak_gbs": PEAK_HBM_GBS, **res,
                           "note": "gdn_layer_inputs / gdn_layer_output, bf16 activations, fp32 o; algorithmic bytes"}
        del xq, zz, lq, lk, lv, lo_, ly, cpool
    except Exception as exc:
        out["layer_io"] = {"error": str(exc)}

    # ---- the layers' projections (gdn_linear, bf16 on the matrix cores): in-projection of a GatedDeltaNet layer
    #      (d_model 2048 -> conv input 6144 | z 2048 | a 16 | b 16) and its out-projection, at a miss's token count and at
    #      a serving step's
    try:
        from paper_2605_05219_amd import linear as LN
        rows = []
        for Tp, Np, Kp in ((N_PREFIX, 3 * HEADS * D, 2048), (N_PREFIX, 2048, 2048), (131072, 3 * HEADS * D, 2048), (131072, 2048, 2048)):
            xp = torch.randn((Tp, Kp), device=dev).bfloat16()
            wp = (torch.randn((Np, Kp), device=dev) / Kp ** 0.5).bfloat16()
            yp_ = torch.empty((Tp, Np), dtype=torch.bfloat16, device=dev)
            for _ in range(3):
                LN.gdn_linear(xp, wp, None, yp_)
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            reps = 20
            ev[0].record()
            for _ in range(reps):
                LN.gdn_linear(xp, wp, None, yp_)
            ev[1].record()
            torch.cuda.synchronize()
            ms = ev[0].elapsed_time(ev[1]) / reps
            tf = 2.0 * Tp * Np * Kp / (ms * 1e-3) / 1e12
            rows.append({"tokens": Tp, "out": Np, "in": Kp, "ms": ms, "TFLOPs": tf, "frac": tf / PEAK_MFMA_TFLOPS})
            del xp, wp, yp_
        out["projections"] = {"peak_TFLOPs": PEAK_MFMA_TFLOPS, "shapes": rows,
                              "note": "gdn_linear, bf16 in and out, fp32 accumulation; 2 T N K flops against the dense bf16 peak"}
    except Exception as exc:
        out["projections"] = {"error": str(exc)}

    # ---- the attention layer of the layer group on the same draws: suffix attention over the restored prefix
    #      (16 query heads, 2 key/value heads, d = 128, bf16), the KV cache resident in HBM; matrix-core bound
    try:
        from paper_2605_05219_amd import attention as AT
        HKV = 2
        ash = AT.make_attn_shape(HEADS, HKV, D, "bf16")
        kc = torch.randn((1, N_PREFIX, HKV, D), device=dev).bfloat16()
        vc = torch.randn((1, N_PREFIX, HKV, D), device=dev).half()
        starts = [int(c.call.start_pos[0]) for c in calls]
        aq = [torch.randn((n, HEADS, D), device=dev).bfloat16() for n in suffix]
        akn = [torch.randn((n, HKV, D), device=dev).bfloat16() for n in suffix]
        avn = [torch.randn((n, HKV, D), device=dev).bfloat16() for n in suffix]
        ao_ = torch.empty((N_PREFIX, HEADS, D), dtype=torch.bfloat16, device=dev)
        aws = torch.empty(AT.attn_workspace_bytes(ash, 1, N_PREFIX), dtype=torch.uint8, device=dev)

        def attn_step(i):
            j = i % N_DRAWS
            AT.attn_suffix_prefill(ash, aq[j], akn[j], avn[j], None, [0, suffix[j]], [starts[j]], kc, vc, [0], ao_, aws)

        for i in range(N_DRAWS):
            attn_step(i)
        torch.cuda.synchronize()
        ta0 = time.perf_counter()
        for i in range(r_steps):
            attn_step(i)
        torch.cuda.synchronize()
        a_ms = 1e3 * (time.perf_counter() - ta0) / r_steps
        a_tok = sum(suffix[i % N_DRAWS] for i in range(r_steps))
        # (query, key) pairs inside the causal limit; 4 d flops each (two contractions)
        pairs = sum(suffix[i % N_DRAWS] * starts[i % N_DRAWS] + suffix[i % N_DRAWS] * (suffix[i % N_DRAWS] + 1) // 2
                    for i in range(r_steps))
        a_tf = 4.0 * D * pairs * HEADS / (a_ms * 1e-3 * r_steps) / 1e12
        out["attention"] = {"ms_per_step": a_ms, "tokens_per_s": a_tok / (a_ms * 1e-3 * r_steps), "TFLOPs": a_tf,
                            "peak_TFLOPs": PEAK_MFMA_TFLOPS, "frac": a_tf / PEAK_MFMA_TFLOPS,
                            "heads": [HEADS, HKV], "d": D,
                            "note": "attn_suffix_prefill on the same draws (append + attention [+ merge of split key walks]); "
                                    "wall time per call; causal flops 4 d per visible (query, key) pair against the dense "
                                    "bf16 peak"}
        del kc, vc, aq, akn, avn, ao_, aws
    except Exception as exc:
        out["attention"] = {"error": str(exc)}

    # ---- a whole cache hit on a layer group as in the paper's runtime experiment (Sec. 6, prototype wall-clock time: one full attention layer
    #      and three GatedDeltaNet layers, with their projections): checkpoint states and the attention KV prefix are
    #      restored from pinned host memory, then the suffix runs through the layers' front ends, the resumed
    #      recurrence (3 layers in one call, downstream checkpoints stored), the back ends and the attention layer.
    if args.layer_group:
        try:
            from paper_2605_05219_amd import attention as AT, layer as LY, linear as LN
            Lg, HKV, N, DM = 3, 2, N_PREFIX, 2048
            Cc = 3 * HEADS * D
            step_ck = N // M_CKPT
            lsh = LY.make_layer_shape(HEADS, HEADS, D, D, 4, "bf16", "bf16", "f32", L=Lg, T_alloc=N)   # the three layers in one call
            ash = AT.make_attn_shape(HEADS, HKV, D, "bf16")
            gsh = B.make_shape(Lg, HEADS, HEADS, D, D, "bf16", "f32", N)
            bf = lambda *sh_: torch.randn(sh_, device=dev).bfloat16()
            xs, aps, bps, zs = bf(Lg, N, Cc), bf(Lg, N, HEADS), bf(Lg, N, HEADS), bf(Lg, N, HEADS, D)
            cw, cb = torch.randn((Lg, Cc, 4), device=dev) * 0.5, torch.randn((Lg, Cc), device=dev) * 0.1
            Al, dtb, nw = torch.zeros((Lg, HEADS), device=dev), torch.zeros((Lg, HEADS), device=dev), torch.ones((Lg, D), device=dev)
            qp, kp, vp = (torch.empty((Lg, N, HEADS, D), dtype=torch.bfloat16, device=dev) for _ in range(3))
            bp_, gp_ = (torch.empty((Lg, N, HEADS), dtype=torch.bfloat16, device=dev) for _ in range(2))
            op = torch.empty((Lg, N, HEADS, D), dtype=torch.float32, device=dev)
            yp = torch.empty((Lg, N, HEADS, D), dtype=torch.bfloat16, device=dev)
            spool = torch.zeros((M_CKPT + 2, Lg, HEADS, D, D), dtype=torch.float32, device=dev)   # slot 0: the loaded state
            hstate = (torch.randn((M_CKPT + 1, Lg, HEADS, D, D)) * 0.05).pin_memory()
            cpool = bf(M_CKPT + 2, Lg, 3, Cc)
            hk = torch.randn((1, N, HKV, D)).bfloat16().pin_memory()
            hv = torch.randn((1, N, HKV, D)).half().pin_memory()
            kc2 = torch.empty((1, N, HKV, D), dtype=torch.bfloat16, device=dev)
            vc2 = torch.empty((1, N, HKV, D), dtype=torch.float16, device=dev)
            aq2, akn2, avn2 = bf(N, HEADS, D), bf(N, HKV, D), bf(N, HKV, D)
            ao2 = torch.empty((N, HEADS, D), dtype=torch.bfloat16, device=dev)
            gws = torch.empty(B.gdn_workspace_bytes(gsh, 1, N, M_CKPT), dtype=torch.uint8, device=dev)
            lws = torch.empty(LY.gdn_layer_workspace_bytes(1, M_CKPT), dtype=torch.uint8, device=dev)
            aws2 = torch.empty(AT.attn_workspace_bytes(ash, 1, N), dtype=torch.uint8, device=dev)
            # the projections: the hidden stream of d_model 2048 into [conv input | z | a | b] per GatedDeltaNet layer and
            # [q | k | v] for the attention layer, and each layer's output back to d_model (seeded synthetic weights)
            HV = HEADS * D
            hid = bf(N, DM)
            hid_out = torch.empty((Lg + 1, N, DM), dtype=torch.bfloat16, device=dev)
            w_in = (torch.randn((Lg, Cc + HV + 2 * HEADS, DM), device=dev) / DM ** 0.5).bfloat16()
            w_out = (torch.randn((Lg + 1, DM, HV), device=dev) / HV ** 0.5).bfloat16()
            w_att = (torch.randn((HV + 2 * HKV * D, DM), device=dev) / DM ** 0.5).bfloat16()
            cur = torch.cuda.current_stream().cuda_stream
            BF = B.GDN_BF16

            def lin(x, ldx, w, n_out, k_in, y, ldy, n_tok):
                rc = LN.gdn_linear_raw(x, ldx, w, k_in, 0, y, ldy, BF, n_tok, n_out, k_in, cur)
                if rc < 0:
                    raise B.GdnError(rc, "gdn_linear")

            def lin_split(x, w, plan, n_tok):
                rc = LN.gdn_linear_split_raw(x, DM, w, DM, 0, plan, BF, n_tok, DM, cur)
                if rc < 0:
                    raise B.GdnError(rc, "gdn_linear_split")

            def proj_in(c, n):
                # one launch per layer: [conv input | z | a | b] to the four tensors the layer's front and back ends read;
                # one more for the attention layer's [q | k | v]
                x = hid.data_ptr() + 2 * c * DM
                for l in range(Lg):
                    plan = LN.SplitPlan([Cc, HV, HEADS, HEADS],
                                        [xs.data_ptr() + 2 * (l * N + c) * Cc, zs.data_ptr() + 2 * (l * N + c) * HV,
                                         aps.data_ptr() + 2 * (l * N + c) * HEADS, bps.data_ptr() + 2 * (l * N + c) * HEADS],
                                        [Cc, HV, HEADS, HEADS])
                    lin_split(x, w_in.data_ptr() + 2 * l * w_in.stride(0), plan, n)
                plan = LN.SplitPlan([HV, HKV * D, HKV * D],
                                    [aq2.data_ptr() + 2 * c * HV, akn2.data_ptr() + 2 * c * HKV * D, avn2.data_ptr() + 2 * c * HKV * D],
                                    [HV, HKV * D, HKV * D])
                lin_split(x, w_att.data_ptr(), plan, n)

            def proj_out_gdn(c, n):
                for l in range(Lg):
                    lin(yp.data_ptr() + 2 * l * N * HV, HV, w_out.data_ptr() + 2 * l * DM * HV, DM, HV,
                        hid_out.data_ptr() + 2 * (l * N + c) * DM, DM, n)

            def proj_out_attn(c, n):
                lin(ao2.data_ptr(), HV, w_out.data_ptr() + 2 * Lg * DM * HV, DM, HV, hid_out.data_ptr() + 2 * (Lg * N + c) * DM, DM, n)

            def hit(n, from_host, proj=True):
                c = N - n                                   # the checkpoint the request resumes from
                emits = list(range(c + step_ck, N + 1, step_ck))
                eslots = list(range(1, 1 + len(emits)))
                if c > 0 and from_host:
                    B.ckpt_fetch_host(hstate, [c // step_ck], spool, [0])
                    AT.attn_kv_restore(ash, [c], hk, hv, [0], kc2, vc2, [0])
                if proj:
                    proj_in(c, n)
                LY.gdn_layer_inputs(lsh, xs[0, c:], cw, cb, aps[0, c:], bps[0, c:], Al, dtb, [0, n], [c], cpool,
                                    [0 if c > 0 else -1], [0, len(emits)], emits, cpool, eslots, qp, kp, vp, bp_, gp_, lws)
                B.gdn_resume_prefill(gsh, qp, kp, vp, bp_, gp_, [0, n], [c], spool, [0 if c > 0 else -1], [0, len(emits)], emits,
                                     spool, eslots, op, gws)
                LY.gdn_layer_output(lsh, op, zs[0, c:], nw, yp, n)
                if proj:
                    proj_out_gdn(c, n)
                AT.attn_suffix_prefill(ash, aq2[c:], akn2[c:], avn2[c:], None, [0, n], [c], kc2, vc2, [0], ao2, aws2)
                if proj:
                    proj_out_attn(c, n)

            pts = []
            keys = (("ms_host_tier", True, True), ("ms_hbm_tier", False, True), ("ms_hbm_tier_without_projections", False, False))
            for n in (512, 1024, 2048, 4096, 6144, 8192):
                row = {"suffix_tokens": n}
                for key, from_host, proj in keys:
                    for _ in range(3):
                        hit(n, from_host, proj)
                    torch.cuda.synchronize()
                    reps, batches = 8, []
                    for _ in range(5):                      # the median of five batches: one slow copy does not decide a point
                        tg0 = time.perf_counter()
                        for _ in range(reps):
                            hit(n, from_host, proj)
                        torch.cuda.synchronize()
                        batches.append(1e3 * (time.perf_counter() - tg0) / reps)
                    row[key] = float(np.median(batches))
                c = N - n
                row["restored_bytes"] = (Lg * HEADS * D * D * 4 + 2 * c * HKV * D * 2) if c > 0 else 0
                pts.append(row)
            xs_ = np.array([p["suffix_tokens"] for p in pts], float)
            fit = {}
            for key, _, _ in keys:
                slope, icpt = np.polyfit(xs_[:-1], np.array([p[key] for p in pts[:-1]]), 1)    # the hits; the last point is the miss
                fit[key] = {"per_1k_tokens": 1e3 * slope, "offset": icpt}
            proj_flops_per_token = 2.0 * DM * (Lg * (Cc + HV + 2 * HEADS) + HV + 2 * HKV * D + (Lg + 1) * HV)
            out["layer_group"] = {"layers": "3 GatedDeltaNet + 1 attention (16 query / 2 kv heads), d = 128, d_model 2048, projections included",
                                  "points": pts, "fit_ms": fit, "projection_flops_per_token": proj_flops_per_token,
                                  "note": "wall time of a whole hit per suffix length (8192 = a miss: nothing restored): in-projections of "
                                          "the four layers (gdn_linear_split, one launch per layer, bf16), front ends of the three GatedDeltaNet layers, recurrence, "
                                          "back ends, their out-projections, attention and its out-projection; every layer reads the same "
                                          "hidden rows (the cost of a stacked group, not its data flow); host tier: checkpoint states "
                                          "(3 MiB) and the KV prefix come from pinned host memory inside the timed region; hbm tier: both "
                                          "are already in device memory; the last column leaves the projections out"}
            del xs, zs, qp, kp, vp, op, spool, hstate, cpool, kc2, vc2
        except Exception as exc:
            out["layer_group"] = {"error": repr(exc)}

    # ---- side measurement: what this chip delivers (fp16 matrix-instruction loop, plain 1 GiB copy), as context
    #      for the data-sheet peaks the roofline is priced against
    try:
        scratch = torch.empty(2 << 30, dtype=torch.uint8, device=dev)
        tf, gbs = B.gdn_probe_ceilings(scratch)
        out["ceilings"] = {"mfma_f16_TFLOPs": tf, "copy_GBs": gbs, "copy_bytes_each_way": scratch.numel() // 2,
                           "note": "measured by gdn_probe_ceilings on this device; data-sheet: 2500 TFLOP/s, 8000 GB/s"}
        del scratch
    except Exception as exc:
        out["ceilings"] = {"error": str(exc)}

    return out


def phase_table(torch, B) -> int:
    """The fused kernel's clocks per phase of one 64-token chunk, from the profiling build of the library (cycle stamps at
    the phase boundaries of the 40th item of every eighth workgroup, one set per wave), on the configs[4] step."""
    import ctypes
    from paper_2605_05219_amd import build as BLD
    from paper_2605_05219_amd.device_call import config4_device
    if not os.path.exists(BLD.LIB_PHASES):
        print("bench.py --phase-table needs the profiling build: python -m paper_2605_05219_amd.build --phase-stamps", file=sys.stderr)
        return 2
    B.LIB_PATH = BLD.LIB_PHASES          # before the first call: the binding loads the library lazily
    step = config4_device()
    for _ in range(3):
        step.run()
    torch.cuda.synchronize()
    raw = np.zeros(64 * 4 * 16, dtype=np.uint64)
    rc = int(B.lib().gdn_phase_stamps(raw.ctypes.data_as(ctypes.c_void_p)))
    if rc != 0:
        print(f"gdn_phase_stamps: {rc}", file=sys.stderr)
        return 1
    t = raw.reshape(64 * 4, 16).astype(np.int64)
    t = t[(t[:, 0] > 0) & (t[:, 9] > t[:, 0])]
    names = ["gates; stage K, Q, V, the next chunk's K loads in between", "the next chunk's gate loads", "barrier after staging",
             "the next chunk's Q loads, diagonal gram block and its inverse", "the next chunk's V loads, L and P blocks",
             "barrier after preparation", "substitution and outputs", "state update", "emission"]
    d = np.diff(t[:, :10], axis=1)
    print(json.dumps({"phase_table": {"workload": "configs[4] step, fused kernel, 40th item (a full 64-token chunk of a long chain) of every eighth workgroup",
                                      "waves_sampled": int(d.shape[0]), "unit": "shader clocks per wave",
                                      "mean": {n: float(x) for n, x in zip(names, d.mean(0))},
                                      "min": {n: float(x) for n, x in zip(names, d.min(0))},
                                      "max": {n: float(x) for n, x in zip(names, d.max(0))},
                                      "total_mean": float(d.sum(1).mean())}}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--latency-steps", type=int, default=64, help="steps of the configs[1] side measurement")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--main-only", action="store_true",
                    help="only the timed steps and their event pass (no side objects, no CPU baseline): what the "
                         "profiler runs use")
    ap.add_argument("--latency-only", action="store_true",
                    help="only the configs[1] side measurement (what the profiler runs of the latency kernels use)")
    ap.add_argument("--copy-only", action="store_true",
                    help="only the checkpoint pool copies (256 MiB read and written per launch: the known-size copy the "
                         "profiler's byte counters are calibrated on)")
    ap.add_argument("--other-configs-only", action="store_true",
                    help="only configs[2] and configs[3], one call each (side object `other_configs`; what their profiler run uses)")
    ap.add_argument("--grouped-heads-only", action="store_true",
                    help="only the grouped-value-heads side measurement (configs[4]'s recipe with 8 query/key heads; what "
                         "the profiler runs of the two-heads-per-workgroup kernel use)")
    ap.add_argument("--phase-table", action="store_true",
                    help="run the configs[4] step on the profiling build of the library (python -m paper_2605_05219_amd.build "
                         "--phase-stamps) and print the fused kernel's clocks per phase of a chunk")
    ap.add_argument("--sides-only", action="store_true",
                    help="only the side objects (configs[1] latency, copies, host tier, decode, layer ends, projections, "
                         "attention, ceilings): what the profiler runs of the side kernels use")
    ap.add_argument("--batch-sweep", action="store_true",
                    help="also time ONE call of k = 1..64 configs[1]-style requests (side object `batch_sweep`; about "
                         "a minute of host-side input generation)")
    ap.add_argument("--layer-group", action="store_true",
                    help="also time a whole cache hit on a layer group (3 GatedDeltaNet layers + 1 attention layer, "
                         "checkpoint and KV cache restored from pinned host memory) against the suffix length")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="skip the per-kernel HIP event pass (no roofline object)")
    ap.add_argument("--events-in-timed-region", action="store_true",
                    help="record the per-kernel events inside the timed steps themselves instead of in a "
                         "repeat of them (the events cost some microseconds per launch)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    from paper_2605_05219_amd import binding as B, workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.phase_table:
        return phase_table(torch, B)
    if args.copy_only:
        print(json.dumps({"ckpt_copy": bench_ckpt_copy(torch, B, dev)}))
        return 0
    if args.other_configs_only:
        print(json.dumps({"other_configs": bench_other_configs(torch, B, wl)}))
        return 0
    if args.grouped_heads_only:
        print(json.dumps({"grouped_value_heads": bench_grouped_heads(torch, B, reps=3)}))
        return 0
    if args.latency_only:
        lat, _, _, _ = bench_config1(args, torch, B, wl, dev)
        print(json.dumps({"latency": lat}))
        return 0

    if args.sides_only:
        lat, calls, pool, suffix = bench_config1(args, torch, B, wl, dev)
        out = {"latency": lat}
        out.update(side_measurements(args, torch, B, wl, dev, calls, pool, suffix, lat["ms_per_step"]))
        print(json.dumps(out))
        return 0

    out, cpu = bench_config4(args, torch, B, dev)
    if args.main_only:
        print(json.dumps(out))
        return 0
    try:
        lat, calls, pool, suffix = bench_config1(args, torch, B, wl, dev)
        out["latency"] = lat
        out.update(side_measurements(args, torch, B, wl, dev, calls, pool, suffix, lat["ms_per_step"]))
    except Exception as exc:       # side measurements never lose the main line
        out["latency"] = {"error": repr(exc)}
    if cpu is not None:
        out["cpu_baseline"] = cpu
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
