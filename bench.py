#!/usr/bin/env python3
"""Benchmark of the resume + checkpoint-emit prefill on one MI355X.

Workload (configs[1]): one GatedDeltaNet layer, batch 1, 16 heads, d_k = d_v = 128, bf16 inputs,
fp32 state and outputs, cached prefix N = 8192 with M = 16 uniformly spaced checkpoints.  A
step is one request: its overlap depth t is a seeded draw from U[0, N); it loads the state of
the deepest checkpoint at or below t straight from the HBM pool, replays tokens l+1..N and
stores every downstream checkpoint state to fresh pool slots.  Steps cycle through a fixed
list of seeded draws.  Inputs are resident in HBM before the timed region; the timed region
covers the whole call per step (host planning, plan upload, both kernels).

Prints ONE JSON line.  Roofline accounting: algorithmic flops (dense tiles of the chunked form) of the launches
that run the recurrence, over their HIP-event time, against the fp16 MFMA peak.
"""
from __future__ import annotations

import argparse
import json
import os
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
# algorithmic HBM bytes per token.head: q, k, v in bf16, beta, gate, o in fp32
BYTES_TOKEN_HEAD = (2 * D + D) * 2 + 2 * 2 + D * 4
# measured HBM bytes per token.head of a call (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, see profiles/), by launch
# kind: the first slab's preparation launch; the recurrence launches, which also prepare every later slab
TRAFFIC_PREP = 319 + 444       # read + written
TRAFFIC_RECUR = 1671 + 1347
SLAB_TOKENS = 32 * C           # the latency variant's slab at 16 chains (checked against the launch count below)
PEAK_MFMA_TFLOPS = 2500.0                   # dense fp16/bf16 MFMA, MI355X
PEAK_HBM_GBS = 8000.0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--main-only", action="store_true",
                    help="only the timed steps and their event pass (no latency sweep, pool copies, host tier, decode, "
                         "CPU baseline): what the profiler runs use")
    ap.add_argument("--batch-sweep", action="store_true",
                    help="also time ONE call of k = 1..64 requests of this workload's kind (side object "
                         "`batch_sweep`; about a minute of host-side input generation)")
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
    from tests.harness import GpuCall

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

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

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    def timed(events):
        if events:
            B.gdn_profile_enable(True)
        torch.cuda.synchronize()
        ta = time.perf_counter()
        for i in range(args.steps):
            step(i)
        torch.cuda.synchronize()
        tb = time.perf_counter()
        if not events:
            return tb - ta, 0.0, 0.0, 0, 0
        p_ms, r_ms, n_prof, p_n, r_n = B.gdn_profile_collect()
        B.gdn_profile_enable(False)
        assert n_prof == args.steps
        return tb - ta, p_ms, r_ms, p_n, r_n

    # The timed region; the per-kernel durations come from HIP events the library records on the
    # launch stream between its kernels, by default in an immediate repeat of the same steps so
    # that the events' own cost stays out of `value`.
    events_wall = None
    if args.no_kernel_events:
        wall_s, prep_ms, recur_ms, prep_n, recur_n = timed(False)
    elif args.events_in_timed_region:
        wall_s, prep_ms, recur_ms, prep_n, recur_n = timed(True)
        events_wall = wall_s
    else:
        wall_s = timed(False)[0]
        events_wall, prep_ms, recur_ms, prep_n, recur_n = timed(True)

    tokens = sum(suffix[i % N_DRAWS] for i in range(args.steps))
    wall = wall_s
    value = tokens / wall
    token_heads = tokens * HEADS

    out = {
        "metric": "recomputed suffix tokens/sec/GPU (resume+ckpt emit)",
        "value": value,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": 1e3 * wall / args.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "config": {
            "workload": "configs[1]: 1 layer, batch 1, 16 heads, d_k=d_v=128, N=8192, M=16 checkpoints at 512 i, "
                        "depth ~ U[0,N), bf16 inputs, fp32 state and outputs",
            "draws": N_DRAWS, "seed": SEED,
            "depths": [int(x) for x in r.meta["depths"]],
            "suffix_tokens": suffix,
            "mean_suffix_tokens": float(np.mean(suffix)),
            "emits_per_step": float(np.mean([int(r.emit_cu[i + 1] - r.emit_cu[i]) for i in range(N_DRAWS)])),
            "chunk": C,
        },
    }

    if not args.no_kernel_events:
        # A step prepares its first slab (32 chunk rounds) in a launch of its own; every recurrence launch
        # but the last also prepares the next slab (gdn_quad_overlap_kernel).  The recurrence launches are
        # therefore priced at the recurrence's flops of every token plus the preparation's flops of the
        # tokens beyond the first slab; the preparation launches at the first slab's preparation flops.
        step_suffix = [suffix[i % N_DRAWS] for i in range(args.steps)]
        slabs_ok = recur_n == sum(-(-t // SLAB_TOKENS) for t in step_suffix) and prep_n == args.steps
        later = sum(max(0, t - SLAB_TOKENS) for t in step_suffix) * HEADS if slabs_ok else 0
        first = token_heads - later
        rec_dom = recur_ms >= prep_ms
        dom = "recurrence launches (gdn_quad_overlap_kernel, gdn_recur_quad_kernel)" if rec_dom else "gdn_prep_kernel"
        dom_ms, dom_n = (recur_ms, recur_n) if rec_dom else (prep_ms, prep_n)
        dom_flops_total = token_heads * FLOP_RECUR + later * FLOP_PREP if rec_dom else first * FLOP_PREP
        dom_flop = dom_flops_total / token_heads
        dom_traffic = TRAFFIC_RECUR if rec_dom else TRAFFIC_PREP
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
            "gdn_prep_kernel": {"avg_ms": prep_ms / args.steps, "launches": prep_n,
                                "avg_launch_ms": prep_ms / max(prep_n, 1),
                                "tflops": first * FLOP_PREP / (prep_ms * 1e-3) / 1e12},
            "gdn_recur_kernel": {"avg_ms": recur_ms / args.steps, "launches": recur_n,
                                 "avg_launch_ms": recur_ms / max(recur_n, 1),
                                 "tflops": (token_heads * FLOP_RECUR + later * FLOP_PREP) / (recur_ms * 1e-3) / 1e12},
            "token_heads_prepared_in_recurrence_launches": later,
            "both_kernels_hbm_gbs_algorithmic": token_heads * BYTES_TOKEN_HEAD / ((prep_ms + recur_ms) * 1e-3) / 1e9,
            "events": "same steps, inside the timed region" if args.events_in_timed_region
                      else "immediate repeat of the timed steps",
            "ms_per_step_with_events": 1e3 * events_wall / args.steps,
            "other_ms_per_step_with_events": 1e3 * events_wall / args.steps - (prep_ms + recur_ms) / args.steps,
        }

    if args.main_only:
        print(json.dumps(out))
        return 0

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
        for i in range(args.steps):
            host_step(i)
        torch.cuda.synchronize()
        host_ms = 1e3 * (time.perf_counter() - ta) / args.steps
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
            "ms_per_step_pool_in_hbm": 1e3 * wall / args.steps,
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

    # ---- throughput regime (not the bench line): a configs[4]-shaped serving step -- 256 requests of log-uniform
    #      suffix length through 8 independent layers x 16 heads, start states gathered by slot id from a 4096-slot
    #      (32 GiB) pool, states stored every 1024 positions and at the end; inputs generated on the device
    try:
        from paper_2605_05219_amd import workloads as wl4
        n_rq4, L4, n_slots4 = 256, 8, 4096
        free_b, _ = torch.cuda.mem_get_info()
        rng4 = np.random.default_rng(1004)
        lens4 = wl4.lengths_log_uniform(rng4, n_rq4, 64, 8192)
        starts4 = (rng4.integers(1, 64, size=n_rq4) * 128).astype(np.int32)
        ids4 = rng4.permutation(n_slots4)
        T4 = int(lens4.sum())
        need4 = n_slots4 * L4 * HEADS * D * D * 4 + L4 * T4 * HEADS * (3 * D * 2 + D * 4 + 4) + (8 << 30)
        if free_b < need4:
            raise RuntimeError(f"needs {need4 >> 30} GiB of device memory, {free_b >> 30} free")
        rule4 = wl4.emit_every(1024)
        cu4 = np.concatenate([[0], np.cumsum(lens4)]).astype(np.int32)
        epos4, ecu4, eslot4, nxt4 = [], [0], [], n_rq4
        for r in range(n_rq4):
            e = rule4(int(starts4[r]), int(starts4[r] + lens4[r]))
            epos4 += e
            ecu4.append(len(epos4))
            eslot4 += [int(x) for x in ids4[nxt4:nxt4 + len(e)]]
            nxt4 += len(e)
        g4 = torch.Generator(device=dev)
        g4.manual_seed(1004)
        rn4 = lambda *sh: torch.randn(sh, device=dev, generator=g4, dtype=torch.float32)
        q4 = torch.empty((L4, T4, HEADS, D), dtype=torch.bfloat16, device=dev)
        k4, v4 = torch.empty_like(q4), torch.empty_like(q4)
        for l in range(L4):
            q4[l] = torch.nn.functional.normalize(rn4(T4, HEADS, D), dim=-1).bfloat16()
            k4[l] = torch.nn.functional.normalize(rn4(T4, HEADS, D), dim=-1).bfloat16()
            v4[l] = rn4(T4, HEADS, D).bfloat16()
        b4 = torch.sigmoid(rn4(L4, T4, HEADS)).bfloat16()
        a4 = torch.exp(-torch.nn.functional.softplus(rn4(L4, T4, HEADS))).bfloat16()
        pool4 = torch.empty((n_slots4, L4, HEADS, D, D), dtype=torch.float32, device=dev)
        for s0 in range(0, n_slots4, 256):
            pool4[s0:s0 + 256] = rn4(256, L4, HEADS, D, D) * 0.1
        o4 = torch.empty((L4, T4, HEADS, D), dtype=torch.float32, device=dev)
        shape4 = B.make_shape(L4, HEADS, HEADS, D, D, "bf16", "f32", T4)
        ws4 = torch.empty(B.gdn_workspace_bytes(shape4, n_rq4, T4, len(epos4)), dtype=torch.uint8, device=dev)

        def run4():
            B.gdn_resume_prefill(shape4, q4, k4, v4, b4, a4, cu4, starts4, pool4, ids4[:n_rq4].astype(np.int32), ecu4, epos4, pool4,
                                 eslot4, o4, ws4)

        run4()
        torch.cuda.synchronize()
        reps4 = 3
        t40 = time.perf_counter()
        for _ in range(reps4):
            run4()
        torch.cuda.synchronize()
        ms4 = 1e3 * (time.perf_counter() - t40) / reps4
        th4 = T4 * L4 * HEADS
        bytes4 = th4 * BYTES_TOKEN_HEAD + (n_rq4 + len(epos4)) * L4 * HEADS * D * D * 4
        out["throughput"] = {
            "workload": "configs[4]: 256 requests x 8 layers x 16 heads, d=128, bf16, suffix ~ logU[64,8192], pool of 4096 slots",
            "tokens_per_layer": T4, "chains": n_rq4 * L4 * HEADS, "emits": len(epos4), "ms_per_call": ms4,
            "tokens_per_s": T4 / (ms4 * 1e-3), "token_layers_per_s": T4 * L4 / (ms4 * 1e-3),
            "hbm": {"algorithmic_bytes": bytes4, "achieved_gbs": bytes4 / (ms4 * 1e-3) / 1e9, "peak_gbs": PEAK_HBM_GBS,
                    "frac": bytes4 / (ms4 * 1e-3) / 1e9 / PEAK_HBM_GBS},
            "mfma": {"achieved_tflops": th4 * (FLOP_PREP + FLOP_RECUR) / (ms4 * 1e-3) / 1e12, "peak_tflops": PEAK_MFMA_TFLOPS,
                     "frac": th4 * (FLOP_PREP + FLOP_RECUR) / (ms4 * 1e-3) / 1e12 / PEAK_MFMA_TFLOPS},
            "note": "whole call on the host clock (planning, plan upload, kernels); the library picks the fused kernel here",
        }
        del q4, k4, v4, b4, a4, pool4, o4, ws4
        torch.cuda.empty_cache()
    except Exception as exc:
        out["throughput"] = {"error": str(exc)}

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
        for i in range(args.steps):
            attn_step(i)
        torch.cuda.synchronize()
        a_ms = 1e3 * (time.perf_counter() - ta0) / args.steps
        a_tok = sum(suffix[i % N_DRAWS] for i in range(args.steps))
        # (query, key) pairs inside the causal limit; 4 d flops each (two contractions)
        pairs = sum(suffix[i % N_DRAWS] * starts[i % N_DRAWS] + suffix[i % N_DRAWS] * (suffix[i % N_DRAWS] + 1) // 2
                    for i in range(args.steps))
        a_tf = 4.0 * D * pairs * HEADS / (a_ms * 1e-3 * args.steps) / 1e12
        out["attention"] = {"ms_per_step": a_ms, "tokens_per_s": a_tok / (a_ms * 1e-3 * args.steps), "TFLOPs": a_tf,
                            "peak_TFLOPs": PEAK_MFMA_TFLOPS, "frac": a_tf / PEAK_MFMA_TFLOPS,
                            "heads": [HEADS, HKV], "d": D,
                            "note": "attn_suffix_prefill on the same draws (append + attention [+ merge of split key walks]); "
                                    "wall time per call; causal flops 4 d per visible (query, key) pair against the dense "
                                    "bf16 peak"}
        del kc, vc, aq, akn, avn, ao_, aws
    except Exception as exc:
        out["attention"] = {"error": str(exc)}

    # ---- a whole cache hit on a layer group as in the paper's runtime experiment (Sec. 5: one full attention layer
    #      and three GatedDeltaNet layers; projections excluded): checkpoint states and the attention KV prefix are
    #      restored from pinned host memory, then the suffix runs through the layers' front ends, the resumed
    #      recurrence (3 layers in one call, downstream checkpoints stored), the back ends and the attention layer.
    if args.layer_group:
        try:
            from paper_2605_05219_amd import attention as AT, layer as LY
            Lg, HKV, N = 3, 2, N_PREFIX
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

            def hit(n, from_host):
                c = N - n                                   # the checkpoint the request resumes from
                emits = list(range(c + step_ck, N + 1, step_ck))
                eslots = list(range(1, 1 + len(emits)))
                if c > 0 and from_host:
                    B.ckpt_fetch_host(hstate, [c // step_ck], spool, [0])
                    AT.attn_kv_restore(ash, [c], hk, hv, [0], kc2, vc2, [0])
                LY.gdn_layer_inputs(lsh, xs[0, c:], cw, cb, aps[0, c:], bps[0, c:], Al, dtb, [0, n], [c], cpool,
                                    [0 if c > 0 else -1], [0, len(emits)], emits, cpool, eslots, qp, kp, vp, bp_, gp_, lws)
                B.gdn_resume_prefill(gsh, qp, kp, vp, bp_, gp_, [0, n], [c], spool, [0 if c > 0 else -1], [0, len(emits)], emits,
                                     spool, eslots, op, gws)
                LY.gdn_layer_output(lsh, op, zs[0, c:], nw, yp, n)
                AT.attn_suffix_prefill(ash, aq2[c:], akn2[c:], avn2[c:], None, [0, n], [c], kc2, vc2, [0], ao2, aws2)

            pts = []
            for n in (512, 1024, 2048, 4096, 6144, 8192):
                row = {"suffix_tokens": n}
                for key, from_host in (("ms_host_tier", True), ("ms_hbm_tier", False)):
                    for _ in range(3):
                        hit(n, from_host)
                    torch.cuda.synchronize()
                    reps, batches = 8, []
                    for _ in range(5):                      # the median of five batches: one slow copy does not decide a point
                        tg0 = time.perf_counter()
                        for _ in range(reps):
                            hit(n, from_host)
                        torch.cuda.synchronize()
                        batches.append(1e3 * (time.perf_counter() - tg0) / reps)
                    row[key] = float(np.median(batches))
                c = N - n
                row["restored_bytes"] = (Lg * HEADS * D * D * 4 + 2 * c * HKV * D * 2) if c > 0 else 0
                pts.append(row)
            xs_ = np.array([p["suffix_tokens"] for p in pts], float)
            fit = {}
            for key in ("ms_host_tier", "ms_hbm_tier"):
                slope, icpt = np.polyfit(xs_[:-1], np.array([p[key] for p in pts[:-1]]), 1)    # the hits; the last point is the miss
                fit[key] = {"per_1k_tokens": 1e3 * slope, "offset": icpt}
            out["layer_group"] = {"layers": "3 GatedDeltaNet + 1 attention (16 query / 2 kv heads), d = 128, projections excluded",
                                  "points": pts, "fit_ms": fit,
                                  "note": "wall time of a whole hit per suffix length (8192 = a miss: nothing restored; four entry-point calls "
                                          "per hit: front ends of the three layers, recurrence, back ends, attention); host tier: "
                                          "checkpoint states (3 MiB) and the KV prefix come from pinned host memory inside the timed "
                                          "region; hbm tier: both are already in device memory"}
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

    # ---- the oracle on the host cores, same workload (all draws once)
    if not args.no_cpu_baseline:
        from oracle import gdn_oracle as orc
        pool_host = pool.cpu().numpy()
        s0 = calls[0].call
        orc.resume_prefill(*s0.streams.slice(0, 64).fields(), [0, 64], [0], [-1], [0, 0], [])  # load + warm
        tc0 = time.perf_counter()
        cpu_tokens = cpu_calls = 0
        while time.perf_counter() - tc0 < 10.0:      # about 10 s of CPU work, whole draws only
            cc = calls[cpu_calls % N_DRAWS].call
            orc.resume_prefill(*cc.streams.fields(), cc.cu_seqlens, cc.start_pos, cc.src_slot, cc.emit_cu,
                               cc.emit_pos, state_src=pool_host)
            cpu_tokens += cc.total_tokens
            cpu_calls += 1
        tc1 = time.perf_counter()
        out["cpu_baseline"] = {
            "value": cpu_tokens / (tc1 - tc0), "unit": "tokens/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"the same {N_DRAWS} draws cycled for about 10 s: {cpu_calls} requests, {cpu_tokens} suffix tokens "
                      f"x {HEADS} heads; fp64 token loop, one (layer, head) chain per thread",
            "seconds": tc1 - tc0,
        }

    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
