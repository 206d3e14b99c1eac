#!/usr/bin/env python3
"""Benchmark of the KVReviver decode hot path on one MI355X.

A "step" is one decode step of the whole path for every layer of the workload:
per layer  append -> select -> encode (one kvr_step_update launch) ->
kvr_attend_decode  on all (sequence, kv head) units, layers one after another
on one stream.  Inputs are synthetic (kvr_synth) and resident in HBM before the
timed region.

Prints ONE JSON line: decode steps/s, achieved algorithmic HBM bandwidth, the
roofline object of the dominant kernels (the token-touching attention kernels
of a layer, timed live with HIP events on the launch stream) and the CPU oracle
timed on a bounded sample.

    python bench.py [--workload c4] [--steps K] [--warmup W] [--gpus 1]
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X published HBM3E bandwidth

# Off-line counter readings (rocprofv3 --pmc, one run per counter group; the files give the commands), per
# workload: they cannot be collected inside this program.  `traffic`: bytes per kvr_attend_decode call at the
# memory side of the L2, checked against a copy kernel of known size and against kernels of this library whose
# traffic is known exactly (None: not measured for this workload).  `alu`: the staged kernel that rebuilds
# the Vague tokens, which is bound by vector-ALU issue and LDS, not by HBM.
OFFLINE_COUNTERS = {
    "c4": {
        # bytes per kvr_attend_decode call at the memory side of the L2: read requests priced by their size
        # (32 / 64 / 128 B request counters) + WRITE_SIZE, summed over the call's three kernels
        "traffic": 781.5e6,
        "traffic_note": "off-line counter reading (profiles/attend_call_c4_hbm_traffic.txt): 680.6 MB read "
                        "(TCC_EA0_RDREQ by request size; FETCH_SIZE prices this chip's 128-byte requests at 64 "
                        "bytes and reads half of that) + 100.9 MB written (WRITE_SIZE), retained + staged + merge "
                        "kernel of one call; the 198 MB above the algorithmic bytes are the logits handed from the "
                        "attention kernels to the score pass, the slice partials and whole lines pulled by "
                        "4-byte score accesses",
        "alu": {"file": "profiles/attend_kernels_c4_sq_counters.txt", "kernel": "attend_vague_staged64_kernel<4>",
                "valu_insts_per_launch": 60048000.0, "waves_per_launch": 10240,
                "valu_busy": 0.71, "lds_busy": 0.41, "lds_bank_conflict_share": 0.46},
    },
}
# plain vector ALU peak: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-operations per second (the 157.3 TFLOP/s
# fp32 vector figure / 2 flops per FMA / 2 for packed math, which this build switches off)
ALU_PEAK_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12
# LDS peak: 256 CUs x 128 bytes per clock x 2.4 GHz
LDS_PEAK_TBS = 256 * 128 * 2.4e9 / 1e12


def algorithmic_bytes_per_unit(wl, n_ctx):
    """Bytes one unit must move per decode step, by definition: retained K and V,
    the K and V sketch, the Vague index list, the cumulative scores (read and
    write) and q / out.  Nothing an implementation adds (partials, spills,
    re-reads) is counted."""
    e = 4 if wl.dtype == "f32" else 2
    D, G = wl.head_dim, wl.group
    R, S = wl.n_retained, wl.sketch_slots
    a = n_ctx - R
    return 2 * R * D * e + 2 * S * D * e + 4 * a + 8 * n_ctx + 2 * G * D * e


def _oracle_unit_step(args):
    """One unit of the workload at full shape: prompt state (not timed), then one
    decode step of the oracle (timed).  Runs in a worker process."""
    name, layer, b, h = args
    os.environ["OMP_NUM_THREADS"] = "1"
    import numpy as np
    import torch
    torch.set_num_threads(1)
    import kvr_synth as S
    from oracle import kvr_oracle as O
    try:
        from threadpoolctl import threadpool_limits
        threadpool_limits(1)
    except Exception:
        pass
    wl = S.WORKLOADS[name]
    scale = 1.0 / math.sqrt(wl.head_dim)
    G = wl.group
    params = O.hash_params_from_seed(S.BASE_SEED + layer, wl.r)
    q0, q1 = S.queries(wl, layer, 0), S.queries(wl, layer, 1)
    kn, vn = S.new_tokens(wl, layer, 0)
    f64 = lambda t: t.to("cpu").double().numpy()
    K, V = S.kv_unit(wl, layer, b, h)
    st = O.dense_prefill_state(f64(K), f64(V), f64(q0[b, h * G:(h + 1) * G]), scale, wl.r, wl.w, params,
                               wl.dtype, n_recent=wl.n_recent, k_candidate=wl.n_candidate,
                               n_cap=wl.context + 2, acc_dtype=np.float32)
    st.compress()
    st = O.compact(st, wl.n_retained + 1)
    t0 = time.perf_counter()
    st.decode_step(f64(kn[b, h]), f64(vn[b, h]), f64(q1[b, h * G:(h + 1) * G]), scale)
    t1 = time.perf_counter()
    return t0, t1


def cpu_baseline(wl, n_units):
    """Time the oracle's decode step on the host for a few units of the same workload
    (full shape; building a unit's prompt state is not timed), once with one process
    per core running side by side and once on a single core, and scale to the whole
    job.  The oracle is used as it stands: numpy, one unit at a time, one thread each."""
    import multiprocessing as mp

    cores = max(1, min(16, os.cpu_count() or 1))       # a one-GPU machine's share of the host
    total_units = wl.layers * wl.units_per_layer
    todo = [(wl.name, 0, u // wl.n_kv_heads, u % wl.n_kv_heads) for u in range(min(n_units, wl.units_per_layer))]
    # one core: the first unit alone
    t0, t1 = _oracle_unit_step(todo[0])
    per_unit_1 = t1 - t0
    # all cores: `cores` workers, one unit each at a time; the figure is unit-steps per second of
    # wall time while all workers are inside their timed step (mean step time under full load)
    ctx = mp.get_context("spawn")
    batch = todo[:cores] if len(todo) >= cores else (todo * cores)[:cores]
    with ctx.Pool(processes=cores) as pool:
        spans = pool.map(_oracle_unit_step, batch, chunksize=1)
    per_unit_all = sum(b - a for a, b in spans) / len(spans)
    return {
        "value": cores / (per_unit_all * total_units),
        "unit": "decode steps/s",
        "cores": cores,
        "kind": "oracle",
        "value_1core": 1.0 / (per_unit_1 * total_units),
        "host_cpus_visible": os.cpu_count(),
        "sample": f"{len(batch)} unit(s) of layer 0 (sequence, head {batch[0][2:]}..{batch[-1][2:]}) x 1 decode step "
                  f"at full shape, one single-threaded process per core, {cores} side by side: "
                  f"{per_unit_all:.3f} s per unit-step under load ({per_unit_1:.3f} s alone on one core), scaled by "
                  f"{total_units} units per step",
    }


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--workload", default="c4", choices=["c2", "c3", "c4", "c5"])
    ap.add_argument("--layers", type=int, default=None, help="debug: run fewer layers (result is then not the named workload)")
    ap.add_argument("--replace-rate", type=float, default=None,
                    help="also run the swap loop of Algorithm 3 in every step with this ReplaceRate (the paper "
                         "fixes 1.1); off by default: the headline configuration evicts and encodes only")
    ap.add_argument("--layer-budget-ramp", type=float, default=0.0,
                    help="non-uniform per-layer budgets: layer l gets budget * (1 - s + 2 s l / (L - 1)), the same "
                         "total; 0 (default) = the uniform budget of the headline configuration")
    ap.add_argument("--max-swaps", type=int, default=4, help="bound of the swap loop per unit and step")
    ap.add_argument("--multi-q", type=int, default=0,
                    help="also time kvr_attend_multi with this many query tokens per sequence on every layer "
                         "(queries at the newest positions of the state after the timed steps; reported beside "
                         "the headline figure, not part of it)")
    ap.add_argument("--event-every", type=int, default=5,
                    help="record the HIP event pair around the attention kernels on every n-th launch of the timed "
                         "region (the two event records cost about 10 us per launch they bracket; 5 does not "
                         "divide the layer count, so every layer is sampled)")
    ap.add_argument("--slack", type=int, default=0,
                    help="Slack of Algorithm 3: the Recent part may outgrow its budget by this many tokens, then "
                         "slack + 1 tokens leave each unit at once (0, the headline configuration: one token in, "
                         "one out per step)")
    ap.add_argument("--no-side-stream", action="store_true",
                    help="do not lend kvr_attend_decode a second stream: its two main kernels run back to back")
    ap.add_argument("--skip-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-units", type=int, default=8)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three elementwise kernels that read and write 768 MiB each (reference for "
                         "scaling the profiler's byte counters)")
    ap.add_argument("--reconstruct", action="store_true",
                    help="also time the stand-alone kvr_reconstruct (Algorithm 2 for every Vague token of a layer, "
                         "rebuilt K and V written to memory) on every layer; reported beside the headline figure")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the short runs of the other named workloads (c3, c5, c2) that a default run "
                         "reports beside the headline figure")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    return args


def run_workload(args):
    """Builds the compressed state of every layer of args.workload, times the decode steps and returns the
    result object (without the CPU baseline).  Everything it allocates on the GPU is released on return."""
    import torch
    import kvr_synth as S
    from paper_2512_17917_amd import binding as kvr
    from paper_2512_17917_amd.state import LayerState

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    kvr.lib()                                  # fails loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    wl = S.WORKLOADS[args.workload]
    L = wl.layers if args.layers is None else args.layers
    K_steps = args.steps if args.steps is not None else min(wl.steps, 128)
    W = args.warmup
    T = K_steps + W
    B, Hkv, Hq, D = wl.batch, wl.n_kv_heads, wl.n_q_heads, wl.head_dim
    log = lambda *a: print(*a, file=sys.stderr, flush=True)
    log(f"[bench] workload {wl.name}: {L} layers x {B} seq x {Hkv} kv heads, N={wl.context}, r={wl.r}, w={wl.w}, "
        f"R={wl.n_retained}, a0={wl.n_vague0}; {W} warmup + {K_steps} timed steps")

    # ---- build the compressed state of every layer (not timed as steps) ---------
    descs, layers = [], []
    n_ctx = torch.zeros(B, dtype=torch.int32, device=dev)
    ws_att = ws_enc = None
    side = None if args.no_side_stream else kvr.SideStream(dev)
    knew, vnew, qs = [], [], []
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_compress_ms = 0.0
    t_setup = time.perf_counter()
    s_ramp = args.layer_budget_ramp
    if s_ramp != 0.0:
        ratios = [1.0 - s_ramp + 2.0 * s_ramp * l / max(wl.layers - 1, 1) for l in range(wl.layers)]
        wl_layers = S.layer_budgets(wl, ratios)
    else:
        wl_layers = [wl] * wl.layers
    for l in range(L):
        wll = wl_layers[l]
        params = kvr.kvr_hash_params_from_seed(S.BASE_SEED + l, wl.r)
        d = kvr.make_desc(B, Hq, Hkv, wl.r, wll.w, wl.torch_dtype, hash_params=params)
        Kf, Vf = S.kv_layer(wll, l, device=dev)
        qall = S.queries_many(wll, l, 0, T + 1, device=dev)          # q[0] initialises the scores
        ls, _ = LayerState.from_prefill(d, Kf, Vf, qall[0].contiguous(), n_recent=wll.n_recent,
                                        k_candidate=wll.n_candidate, max_new_tokens=T, ws_attend=ws_att,
                                        ws_encode=ws_enc, n_ctx=n_ctx, timers=(ev0, ev1), slack=args.slack,
                                        side=side)
        torch.cuda.synchronize()
        t_compress_ms += ev0.elapsed_time(ev1)
        ne = ls.n_evict.min().item()
        if ne != wll.n_vague0 or ls.n_evict.max().item() != wll.n_vague0:
            raise RuntimeError(f"layer {l}: prompt compression evicted {ne}, expected {wll.n_vague0}")
        if s_ramp == 0.0:            # layers of one size share the workspaces
            ws_att, ws_enc = ls.ws_attend, ls.ws_encode
        del Kf, Vf
        kn, vn = S.kv_layer(wll, l, wl.context, wl.context + T, device=dev)      # [B, Hkv, T, D]
        knew.append(kn.permute(2, 0, 1, 3).contiguous())
        vnew.append(vn.permute(2, 0, 1, 3).contiguous())
        qs.append(qall[1:].contiguous())
        descs.append(d)
        layers.append(ls)
        if l == 0 or (l + 1) % 12 == 0:
            log(f"[bench] layer {l + 1}/{L} compressed ({time.perf_counter() - t_setup:.1f} s)")
    torch.cuda.empty_cache()

    swap_kw = {} if args.replace_rate is None else {"replace_rate": args.replace_rate, "max_swaps": args.max_swaps}

    def run_step(t):
        n_ctx.add_(1)
        for l in range(L):
            layers[l].decode_step(knew[l][t], vnew[l][t], qs[l][t], bump_n_ctx=False, **swap_kw)

    for t in range(W):
        run_step(t)
    torch.cuda.synchronize()

    # ---- timed region ----------------------------------------------------------
    ev_every = max(1, args.event_every)
    pairs = [(kvr.event_create(True), kvr.event_create(True)) for _ in range((K_steps * L + ev_every - 1) // ev_every)]

    def attend_opts(a=None, b=None):
        if side is not None:
            return side.opts(a, b)
        return kvr.kvr_attend_opts(None, None, None, a, b) if a is not None else None

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    i = 0
    for t in range(W, T):
        n_ctx.add_(1)
        for l in range(L):
            opts = attend_opts(*pairs[i // ev_every]) if i % ev_every == 0 else attend_opts()
            i += 1
            layers[l].decode_step(knew[l][t], vnew[l][t], qs[l][t], bump_n_ctx=False, opts=opts, **swap_kw)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    elapsed = t1 - t0
    kern_ms = [kvr.event_elapsed_ms(a, b) for a, b in pairs]
    for a, b in pairs:
        kvr.hip().hipEventDestroy(a)
        kvr.hip().hipEventDestroy(b)

    # sanity of the state after the run: every unit could evict what it had to, and what went into
    # the sketch is what Algorithm 3 sends there (one token per unit per step; with Slack s, s + 1
    # tokens every s + 1 steps)
    for ls in layers:
        ls.check_evictions()
    nv = layers[0].n_vague
    want_nv = wl_layers[0].n_vague0 + (T // (args.slack + 1)) * (args.slack + 1)
    if nv.min().item() != want_nv or nv.max().item() != want_nv:
        raise RuntimeError(f"bookkeeping drifted: n_vague is {nv.min().item()}..{nv.max().item()}, expected {want_nv}")
    if not torch.isfinite(layers[-1].out).all():
        raise RuntimeError("non-finite attention output")

    e_bytes = 4 if wl.dtype == "f32" else 2
    prompt_bytes_layer = wl.units_per_layer * (2 * wl.n_vague0 * D * e_bytes + 2 * wl.sketch_slots * D * e_bytes
                                               + 4 * wl.context)
    steps_per_s = K_steps / elapsed
    n_mid = wl.context + W + (K_steps + 1) // 2
    bytes_layer = [algorithmic_bytes_per_unit(wl_layers[l], n_mid) * wl.units_per_layer for l in range(L)]
    bytes_launch = sum(bytes_layer) / L            # per launch (mean over the layers when budgets differ)
    bytes_step = sum(bytes_layer)
    avg_kern_s = (sum(kern_ms) / len(kern_ms)) * 1e-3
    achieved = bytes_launch / avg_kern_s / 1e9
    off = OFFLINE_COUNTERS.get(wl.name, {}) if (L == wl.layers and s_ramp == 0.0) else {}
    alu_obj = None
    if "alu" in off:
        c = off["alu"]
        # lane-operations the staged kernel issues per launch (64 lanes per vector instruction) over the live
        # duration of the call it dominates
        lane_ops = c["valu_insts_per_launch"] * 64
        n_vague_mid = wl.n_vague0 + W + (K_steps + 1) // 2
        alu_obj = {
            "bound": "alu", "kernel": c["kernel"], "source": c["file"],
            "achieved": lane_ops / avg_kern_s / 1e12, "peak": ALU_PEAK_TLANEOPS, "unit": "T lane-ops/s",
            "frac": lane_ops / avg_kern_s / 1e12 / ALU_PEAK_TLANEOPS,
            "peak_derivation": "256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz, no packed math",
            "valu_busy_alone": c["valu_busy"], "lds_busy_alone": c["lds_busy"],
            "lds_bank_conflict_share": c["lds_bank_conflict_share"],
            "valu_insts_per_wave": c["valu_insts_per_launch"] / c["waves_per_launch"],
            "valu_insts_per_rebuilt_token": c["valu_insts_per_launch"] * 64 / (wl.units_per_layer * n_vague_mid),
            # what the rebuilt part must gather out of the on-chip sketch copy: r rows of K and of V per token
            "lds_gather_bytes_per_launch": wl.units_per_layer * n_vague_mid * 2 * wl.r * D * e_bytes,
            "lds_gather_tbs": wl.units_per_layer * n_vague_mid * 2 * wl.r * D * e_bytes / avg_kern_s / 1e12,
            "lds_peak_tbs": LDS_PEAK_TBS,
            "lds_frac": wl.units_per_layer * n_vague_mid * 2 * wl.r * D * e_bytes / avg_kern_s / 1e12 / LDS_PEAK_TBS,
            "lds_peak_derivation": "256 CUs x 128 B per clock x 2.4 GHz",
            "note": "instruction counts and busy fractions are off-line counter readings of the kernel running "
                    "alone (the file gives the command); the duration is this run's",
        }
    result = {
        "metric": "decode steps/sec (encode+reconstruct+attend, all layers) + achieved HBM GB/s",
        "value": steps_per_s,
        "unit": "decode steps/s",
        "n_gpus": 1,
        "steps": K_steps,
        "warmup": W,
        "ms_per_step": 1e3 * elapsed / K_steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if wl.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: {L} layers, batch {B}, {Hq} q / {Hkv} kv heads, head_dim {D}, "
                               f"context {wl.context}, budget {wl.budget}, sketch r={wl.r} w={wl.w}, "
                               f"retained {wl.n_retained}, vague {wl.n_vague0}+t",
                   "global_batch": B, "seq_len": wl.context, "parallelism": "1 GPU"},
        "achieved_hbm_gbs": bytes_step * steps_per_s / 1e9,
        "hbm_frac_whole_step": bytes_step * steps_per_s / 1e9 / HBM_PEAK_GBS,
        "algorithmic_bytes_per_step": bytes_step,
        "tokens_per_s": steps_per_s * B,
        "prompt_compress_ms_total": t_compress_ms,
        # prompt compression (kvr_select over the whole prompt + bulk kvr_encode), once per layer, outside the
        # timed steps; algorithmic bytes = evicted K and V rows read once + sketch written + scores read
        "prompt_compress": {
            "ms_per_layer": t_compress_ms / L,
            "algorithmic_bytes_per_layer": prompt_bytes_layer,
            "achieved_gbs": prompt_bytes_layer / (t_compress_ms / L * 1e-3) / 1e9,
            "hbm_frac": prompt_bytes_layer / (t_compress_ms / L * 1e-3) / 1e9 / HBM_PEAK_GBS,
        },
        "roofline": {
            "kernel": "one kvr_attend_decode call = attention over retained + reconstructed tokens of one layer, all "
                      "units: attend_retained_shared_kernel (streams the retained rows; on the lent side stream) next "
                      "to attend_vague_staged64_kernel (rebuilds the Vague tokens from the sketch in LDS), then "
                      "attend_combine_kernel (merge + score accumulation); HIP events on the caller's stream before "
                      "the first and after the last of them" if wl.name in ("c4",) and side is not None else
                      "one kvr_attend_decode call (retained-slot kernel, Vague-list kernel, merge kernel of one "
                      "layer, all units); HIP events on the caller's stream before the first and after the last",
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": off.get("traffic") if L == wl.layers else None,
            "traffic_note": off.get("traffic_note", "not measured for this workload"),
            "algorithmic_bytes_per_launch": bytes_launch,
            "algorithmic_bytes_note": "retained K,V + sketch K,V + Vague index list + scores read and written + q, out: "
                                      "all of it moved by the three kernels inside the timed region",
            "avg_launch_ms": avg_kern_s * 1e3,
            "launches_timed": len(kern_ms),
            "launch_sampling": f"HIP events on every {ev_every}. call of the timed region",
            "note": "the call is not HBM-bound: its longest kernel is bound by vector-ALU issue and LDS (roofline_alu)",
        },
        "roofline_alu": alu_obj,
    }
    if args.multi_q > 0:
        nq = args.multi_q
        qm = S.queries_many(wl, 0, 1, 1 + nq, device=dev).permute(1, 0, 2, 3).contiguous()    # [B, nq, Hq, D]
        ws_bytes = max(kvr.kvr_attend_multi_workspace_size(descs[l], nq, layers[l].ret_cap, layers[l].vague_cap)
                       for l in range(L))
        ws_m = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        for l in range(min(L, 4)):
            layers[l].attend_multi(qm, nq, accumulate_scores=True, ws=ws_m)
        torch.cuda.synchronize()
        reps = 3
        tm0 = time.perf_counter()
        for _ in range(reps):
            for l in range(L):
                layers[l].attend_multi(qm, nq, accumulate_scores=True, ws=ws_m)
        torch.cuda.synchronize()
        ms_layer = (time.perf_counter() - tm0) * 1e3 / (reps * L)
        result["attend_multi"] = {"n_q": nq, "ms_per_layer": ms_layer,
                                  "query_tokens_per_s": nq * B / (ms_layer * 1e-3 * L),
                                  "decode_ms_per_layer_for_comparison": result["ms_per_step"] / L}
        log(f"[bench] attend_multi n_q={nq}: {ms_layer * 1e3:.1f} us per layer")
        del ws_m
    if args.reconstruct:
        ls0 = layers[0]
        cap_r = ls0.vague_cap
        k_out = torch.empty(B, Hkv, cap_r, D, dtype=wl.torch_dtype, device=dev)
        v_out = torch.empty_like(k_out)
        for l in range(min(L, 4)):
            kvr.kvr_reconstruct(descs[l], layers[l].sketch_k, layers[l].sketch_v, layers[l].vague_pos,
                                layers[l].n_vague, layers[l].vague_cap, k_out, v_out)
        torch.cuda.synchronize()
        reps = 3
        tr0 = time.perf_counter()
        for _ in range(reps):
            for l in range(L):
                kvr.kvr_reconstruct(descs[l], layers[l].sketch_k, layers[l].sketch_v, layers[l].vague_pos,
                                    layers[l].n_vague, layers[l].vague_cap, k_out, v_out)
        torch.cuda.synchronize()
        ms_layer = (time.perf_counter() - tr0) * 1e3 / (reps * L)
        n_v = int(ls0.n_vague.max().item())
        # rebuilt K and V written once, the sketch and the index list read once
        rbytes = wl.units_per_layer * (2 * n_v * D * e_bytes + 2 * wl.sketch_slots * D * e_bytes + 4 * n_v)
        result["reconstruct"] = {"ms_per_layer": ms_layer, "tokens_per_layer": wl.units_per_layer * n_v,
                                 "algorithmic_bytes_per_layer": rbytes,
                                 "achieved_gbs": rbytes / (ms_layer * 1e-3) / 1e9,
                                 "hbm_frac": rbytes / (ms_layer * 1e-3) / 1e9 / HBM_PEAK_GBS}
        log(f"[bench] kvr_reconstruct: {ms_layer * 1e3:.1f} us per layer, {result['reconstruct']['achieved_gbs']:.0f} GB/s "
            f"({100 * result['reconstruct']['hbm_frac']:.1f}% of HBM peak)")
        del k_out, v_out
    if args.replace_rate is not None:
        n_sw = torch.zeros(B, Hkv, dtype=torch.int32, device=dev)
        layers[0].swap_back(args.replace_rate, args.max_swaps, n_sw)       # one more loop, to report its count
        result["config"]["workload"] += f" + swap loop (ReplaceRate {args.replace_rate}, <= {args.max_swaps} per unit and step)"
        result["swap_back"] = {"replace_rate": args.replace_rate, "max_swaps": args.max_swaps,
                               "swaps_per_unit_after_last_step": float(n_sw.float().mean().item())}
    if s_ramp != 0.0:
        result["config"]["workload"] += (f" + per-layer budgets {wl_layers[0].budget:.4f} .. {wl_layers[L - 1].budget:.4f} "
                                         f"(w {wl_layers[0].w} .. {wl_layers[L - 1].w})")
    if args.layers is not None and args.layers != wl.layers:
        result["config"]["workload"] += f" [DEBUG: only {L} of {wl.layers} layers]"
    log(f"[bench] {steps_per_s:.2f} steps/s, {result['ms_per_step']:.3f} ms/step, "
        f"{result['achieved_hbm_gbs']:.0f} GB/s algorithmic ({100 * result['hbm_frac_whole_step']:.1f}% of HBM peak); "
        f"main kernel {avg_kern_s * 1e6:.1f} us/launch -> {achieved:.0f} GB/s")

    if args.calibrate_copy:
        # an elementwise kernel of known traffic: reads 768 MiB, writes 768 MiB (a size nothing else in this
        # program has, so that its dispatches can be told apart by grid size: 50 331 648 work-items)
        src = torch.empty(3 << 26, dtype=torch.float32, device=dev)      # no fill kernel of the same size
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    return result


# the other named workloads, measured briefly in a default run so that their figures come from the same
# program on the same machine as the headline: (name, timed steps, warm-up steps)
OTHER_WORKLOADS = (("c3", 32, 4), ("c5", 12, 2), ("c2", 128, 4))


def main():
    args = parse_args()
    import torch
    import kvr_synth as S
    log = lambda *a: print(*a, file=sys.stderr, flush=True)
    result = run_workload(args)
    torch.cuda.empty_cache()
    headline = (args.workload == "c4" and args.layers is None and args.replace_rate is None
                and args.layer_budget_ramp == 0.0 and args.slack == 0 and args.multi_q == 0
                and not args.calibrate_copy and not args.reconstruct)
    if headline and not args.no_other_workloads:
        others = {}
        for name, k, w_ in OTHER_WORKLOADS:
            a2 = argparse.Namespace(**vars(args))
            a2.workload, a2.steps, a2.warmup = name, k, w_
            r = run_workload(a2)
            torch.cuda.empty_cache()
            others[name] = {"value": r["value"], "unit": r["unit"], "ms_per_step": r["ms_per_step"],
                            "steps": k, "warmup": w_, "workload": r["config"]["workload"],
                            "hbm_frac_whole_step": r["hbm_frac_whole_step"],
                            "attend_call_us": r["roofline"]["avg_launch_ms"] * 1e3,
                            "attend_call_hbm_frac": r["roofline"]["frac"],
                            "prompt_compress_ms_per_layer": r["prompt_compress"]["ms_per_layer"]}
        result["other_workloads"] = others
    if args.skip_cpu_baseline:
        result["cpu_baseline"] = None
    else:
        torch.set_num_threads(1)
        result["cpu_baseline"] = cpu_baseline(S.WORKLOADS[args.workload], args.cpu_units)
        log(f"[bench] oracle: {result['cpu_baseline']['value']:.3e} steps/s ({result['cpu_baseline']['sample']})")
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
