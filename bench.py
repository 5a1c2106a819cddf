#!/usr/bin/env python3
"""Benchmark of the ThinK hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input: prune the key caches
of all layers of the workload in one thk_prune call (score -> Top_T -> compaction), then the
workload's decode-attention steps over the pruned cache (one thk_decode_attn call per layer
and step, with thk_tail_append before it where the workload grows a tail).  Inputs are resident
in HBM before the timed region.  Prints ONE JSON line.

The headline (`value`, `ms_per_step`, `roofline`, `cpu_baseline`, `value_cache`) is the
LLaMA-2-7B-shaped workload (configs[1]), the one the metric is quoted on; with no --config the
other four workloads are run as well and every workload gets an entry in `per_config`.

Bytes.  `value` and every fraction are computed from the bytes the path has to move:
  prune  per layer  U * S * e * (D + T) + |Q_obs|   when thk_prune keeps the rows on chip (K read
                    once, T kept channels written once); the metric's own definition counts
                    D + 2T per row (kept channels read a second time) and is reported beside it as
                    `*_metric_def`, as a rate only -- the one-pass kernel moves fewer bytes than
                    that, so a fraction of the HBM peak computed from it could exceed 1;
  decode per step   U * e * [S * (T + D) + s_tail * 2 D].
"""
import argparse
import gc
import glob
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak
HEADLINE = 2            # the workload the metric is quoted on


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=0,
                    help="workload id 1..5 (synth.CONFIGS) to run alone; 0 = headline workload + all five in per_config")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--no-value-cache", action="store_true",
                    help="skip the value-cache extension leg (value score, value prune, decode over both caches)")
    ap.add_argument("--no-graph", action="store_true",
                    help="skip the replay of the step from a HIP graph (graph_ms_per_step)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain 1 GiB device copies (reference dispatches of known size "
                         "for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def cpu_baseline(cfg_id, cfg, T, device, budget_s=20.0):
    """Time the oracle, as it stands, on the same workload, layer after layer, until the
    workload is done or about budget_s seconds of oracle time have been spent."""
    from oracle import oracle as O
    from paper_2407_21018_amd import synth
    dt = cfg["dtype"]
    eb = 2 if dt == "bf16" else 4
    U = cfg["B"] * cfg["N_kv"]
    O.lib()
    t_prune = t_dec = 0.0
    nbytes = 0
    layers = 0
    for l in range(cfg["L"]):
        q_obs, k, v = synth.gen_prefill(cfg_id, l, device, **cfg)
        q, _, _ = synth.gen_decode(cfg_id, l, 0, device, **cfg)
        qn, kn, vn, q1 = synth.as_numpy(q_obs), synth.as_numpy(k), synth.as_numpy(v), synth.as_numpy(q)
        del q_obs, k, v
        t0 = time.perf_counter()
        sc = O.score(qn, kn, dt)
        idx = O.select_topk(sc, T)
        kp = O.compact_keys(kn, idx, dt)
        t1 = time.perf_counter()
        O.decode_attn(q1[0], kp[0], idx[0], vn[0], dt)
        t2 = time.perf_counter()
        t_prune += t1 - t0
        t_dec += t2 - t1
        # the same byte accounting as the GPU figure: K once, kept channels written once, decode stream
        nbytes += U * cfg["S"] * eb * (cfg["D"] + T) + qn.nbytes + U * cfg["S"] * eb * (T + cfg["D"])
        layers += 1
        if t_prune + t_dec > budget_s:
            break
    return {"value": nbytes / (t_prune + t_dec) / 1e9, "unit": "GB/s", "cores": O.max_threads(), "kind": "oracle",
            "sample": f"{layers} of {cfg['L']} layers of configs[{cfg_id - 1}], all {U} units each: prune + 1 decode "
                      f"step per layer ({t_prune + t_dec:.1f} s of oracle time)",
            "prune_ms_per_layer": t_prune / layers * 1e3, "decode_us_per_step": t_dec / layers * 1e6}


def value_cache_leg(thk, torch, cfg, T, tdt, dt, eb, q_obs, k, v, kp, idx, dec, kt, vt, out, reps):
    """The value-cache extension (not part of `value`): prune V with the same ratio as K
    (value score on the matrix cores -> Top_T -> compaction) over all layers in one call, then
    one decode step per layer over both pruned caches.  Reports the score kernel against the
    HBM roofline (it streams K and V once) with its matrix-core rate beside it."""
    L, B, N_q, N_kv, D, S, S_obs = (cfg[n] for n in ("L", "B", "N_q", "N_kv", "D", "S", "S_obs"))
    U, G, dev = B * N_kv, N_q // N_kv, q_obs.device
    cap = cfg["tail_cap"]
    T_v = T
    ld_v = (T_v + 3) // 4 * 4
    shape_v = thk.make_shape(L, B, N_q, N_kv, D, S, S_obs, T_v, ld_v, tdt, 0)
    shape_1 = thk.make_shape(1, B, N_q, N_kv, D, S, S_obs, T, 0, tdt, 0)
    score_v = torch.empty(L * U, D, dtype=torch.float32, device=dev)
    idx_v = torch.empty(L * U, T_v, dtype=torch.int16, device=dev)
    vp = torch.empty(L, U, S, ld_v, dtype=dt, device=dev)
    ws = torch.empty(max(thk.thk_workspace_bytes(shape_v, thk.THK_OP_PRUNE_VALUE),
                         thk.thk_workspace_bytes(shape_1, thk.THK_OP_DECODE), 16), dtype=torch.uint8, device=dev)

    def ev():
        e = torch.cuda.Event(enable_timing=True)
        e.record()
        return e

    def prune_v(pair=None):
        if pair is not None:
            thk.thk_profile_next(*pair)
        thk.thk_prune_value(shape_v, q_obs, k, v, 1, score_v, idx_v, vp, ws)

    def decode_all():
        for l in range(L):
            q = dec[l][0][0]
            thk.thk_decode_attn_kv(shape_1, q, kp[l], idx[l * U:(l + 1) * U], vp[l], idx_v[l * U:(l + 1) * U],
                                   T_v, ld_v, kt[l] if cap else None, vt[l] if cap else None,
                                   1 if cap else 0, cap, out[l], ws)

    prune_v(); decode_all()
    pairs = [(ev(), ev()) for _ in range(reps)]
    marks = [ev() for _ in range(3)]
    torch.cuda.synchronize()
    marks[0].record()
    for i in range(reps):
        prune_v(pairs[i])
    marks[1].record()
    for i in range(reps):
        decode_all()
    marks[2].record()
    torch.cuda.synchronize()
    score_us = sum(a.elapsed_time(b) for a, b in pairs) / reps * 1e3
    prune_ms_layer = marks[0].elapsed_time(marks[1]) / reps / L
    dec_us = marks[1].elapsed_time(marks[2]) / reps / L * 1e3
    score_bytes = L * (2 * U * S * D * eb + B * N_q * S_obs * D * eb)
    score_flops = 4.0 * L * U * G * S_obs * S * D
    prune_v_bytes = score_bytes + L * U * S * eb * (D + T_v)
    dec_bytes = U * eb * (S * (T + T_v) + (2 * D if cap else 0))
    return {"T_v": T_v, "causal": 1,
            "score_kernel": "k_value_attn", "score_us": score_us, "score_bytes": score_bytes,
            "score_GBps": score_bytes / score_us / 1e3, "score_frac_of_hbm_peak": score_bytes / score_us / 1e3 / HBM_PEAK_GBS,
            "score_TFLOPs": score_flops / score_us / 1e6,
            "prune_value_ms_per_layer": prune_ms_layer, "prune_value_GBps": prune_v_bytes / L / prune_ms_layer / 1e6,
            "prune_value_frac_of_hbm_peak": prune_v_bytes / L / prune_ms_layer / 1e6 / HBM_PEAK_GBS,
            "decode_kv_us_per_step": dec_us, "decode_kv_GBps": dec_bytes / dec_us / 1e3,
            "decode_kv_frac_of_hbm_peak": dec_bytes / dec_us / 1e3 / HBM_PEAK_GBS,
            "decode_kv_bytes_vs_k_only": (T + T_v) / (T + D)}


def measured_traffic(cfg_id, kernel):
    """HBM-side bytes per launch of `kernel` at workload cfg_id from the committed rocprofv3
    counter summaries (profiles/*.txt, lines 'traffic_bytes_per_launch cfg<N> <kernel> <bytes>').
    Returns (bytes, file name) or (None, None): the counters are not collected in this run."""
    for f in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt"))):
        for line in open(f):
            w = line.split()
            if len(w) == 4 and w[0] == "traffic_bytes_per_launch" and w[1] == f"cfg{cfg_id}" and w[2] == kernel:
                return float(w[3]), "profiles/" + os.path.basename(f)
    return None, None


def device_facts(torch):
    """What the runtime reports about the card the numbers were taken on."""
    p = torch.cuda.get_device_properties(0)
    return {"arch": p.gcnArchName, "compute_units": p.multi_processor_count, "wavefront": p.warp_size,
            "lds_bytes_per_block_max": p.shared_memory_per_block, "l2_bytes_per_xcd": p.L2_cache_size,
            "memory_bytes": p.total_memory}


def run_config(cfg_id, args, torch, thk, synth, full):
    """Time workload cfg_id.  full: also the value-cache leg and the oracle leg (headline only)."""
    dev = "cuda:0"
    cfg = synth.CONFIGS[cfg_id]
    L, B, N_q, N_kv, D, S, S_obs = (cfg[k] for k in ("L", "B", "N_q", "N_kv", "D", "S", "S_obs"))
    T = thk.thk_keep_count(D, cfg["lam"])
    dt = synth.torch_dtype(cfg["dtype"])
    tdt = thk.THK_BF16 if cfg["dtype"] == "bf16" else thk.THK_F32
    eb = 2 if cfg["dtype"] == "bf16" else 4
    U = B * N_kv                      # units per layer
    steps_per_layer = cfg["steps"]
    cap = cfg["tail_cap"]
    steps = args.steps

    # ---- inputs, resident in HBM ------------------------------------------
    q_obs = torch.empty(L, B, N_q, S_obs, D, dtype=dt, device=dev)
    k = torch.empty(L, B, N_kv, S, D, dtype=dt, device=dev)
    v = torch.empty(L, B, N_kv, S, D, dtype=dt, device=dev)
    for l in range(L):
        q_obs[l], k[l], v[l] = (t[0] for t in synth.gen_prefill(cfg_id, l, dev, **cfg))
    dec = [[synth.gen_decode(cfg_id, l, s, dev, **cfg) for s in range(steps_per_layer)] for l in range(L)]
    score = torch.empty(L * U, D, dtype=torch.float32, device=dev)
    idx = torch.empty(L * U, T, dtype=torch.int16, device=dev)
    kp = torch.empty(L, U, S, T, dtype=dt, device=dev)
    out = torch.empty(L, B * N_q, D, dtype=dt, device=dev)
    kt = torch.zeros(L, U, max(cap, 1), D, dtype=dt, device=dev)
    vt = torch.zeros_like(kt)
    shape_all = thk.make_shape(L, B, N_q, N_kv, D, S, S_obs, T, 0, tdt, 0)
    shape_1 = thk.make_shape(1, B, N_q, N_kv, D, S, S_obs, T, 0, tdt, 0)
    ws = torch.empty(max(thk.thk_workspace_bytes(shape_all, thk.THK_OP_PRUNE),
                         thk.thk_workspace_bytes(shape_1, thk.THK_OP_DECODE), 16), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()

    def ev():
        e = torch.cuda.Event(enable_timing=True)
        e.record()          # torch creates the HIP event on first record; done outside the timed region
        return e

    n_dec = steps_per_layer * L
    # event pairs the library attaches to the main kernel of a call (thk_profile_next: the
    # interval is the kernel's own begin-to-end time): the prune call of every step, and every
    # eighth decode call (offset rotating with the step)
    n_prof = max(1, n_dec // 8)
    pairs = [[(ev(), ev()) for _ in range(1 + n_prof)] for _ in range(steps)]
    torch.cuda.synchronize()

    def step(evs=None, ph=None, rot=0):
        """Whole hot path once.  evs: this step's event pairs (prune first, then one per decode call);
        ph: three events recorded before the prune, after it, and after the last decode call."""
        if evs is not None:
            thk.thk_profile_next(*evs[0])
        if ph is not None:
            ph[0].record()
        thk.thk_prune(shape_all, q_obs, k, score, idx, kp, ws)
        if ph is not None:
            ph[1].record()
        i, call = 1, 0
        used = []
        for s in range(steps_per_layer):
            for l in range(L):
                q, k_new, v_new = dec[l][s]
                if cap:
                    thk.thk_tail_append(shape_1, k_new, v_new, kt[l], vt[l], s, cap)
                if evs is not None and call % 8 == rot % min(8, n_dec) and i < len(evs):
                    thk.thk_profile_next(*evs[i])
                    used.append(evs[i])
                    i += 1
                call += 1
                thk.thk_decode_attn(shape_1, q, kp[l], idx[l * U:(l + 1) * U], v[l],
                                    kt[l] if cap else None, vt[l] if cap else None,
                                    s + 1 if cap else 0, cap, out[l], ws)
        if ph is not None:
            ph[2].record()
        return used

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)          # reads 1 GiB, writes 1 GiB per dispatch
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
    phases = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    e0.record()
    used_pairs = []
    # A workload with only a few calls per step would carry an event pair on every call, and a
    # launch with events attached costs the host ~12 us more than a plain one, which a step of
    # a few short calls does not hide; there the kernels are timed on every fourth step only and
    # the phases are read off the other steps.
    sparse = n_dec < 8 and steps >= 2
    kernel_steps = [i for i in range(steps) if not sparse or i % 4 == 0]
    phase_steps = [i for i in range(steps) if not sparse or i % 4 != 0]
    for i in range(steps):
        used_pairs += step(pairs[i] if i in kernel_steps else None, phases[i], i)
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = e0.elapsed_time(e1) / steps

    graph_ms = None
    if not args.no_graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr):
            step()
        gr.replay()
        torch.cuda.synchronize()
        g0 = torch.cuda.Event(enable_timing=True); g1 = torch.cuda.Event(enable_timing=True)
        g0.record()
        for _ in range(steps):
            gr.replay()
        g1.record()
        torch.cuda.synchronize()
        graph_ms = g0.elapsed_time(g1) / steps
        del gr

    # main-kernel durations measured inside the timed region
    prune_kernel_us = [pairs[i][0][0].elapsed_time(pairs[i][0][1]) * 1e3 for i in kernel_steps]
    dec_kernel_us = [a.elapsed_time(b) * 1e3 for (a, b) in used_pairs]
    prune_k_us = sum(prune_kernel_us) / len(prune_kernel_us)
    dec_k_us = sum(dec_kernel_us) / len(dec_kernel_us)
    # whole calls (all kernels of a call and the gaps between them)
    prune_ms_layer = sum(phases[i][0].elapsed_time(phases[i][1]) for i in phase_steps) / len(phase_steps) / L
    dec_us_step = sum(phases[i][1].elapsed_time(phases[i][2]) for i in phase_steps) / len(phase_steps) / n_dec * 1e3

    # ---- bytes the path has to move (per layer), K and V counted once per KV head -----
    form = thk.thk_prune_is_fused(shape_all)     # 2: rows held on chip, K read once
    qobs_bytes = B * N_q * S_obs * D * eb
    prune_bytes_def = U * S * eb * (D + 2 * T) + qobs_bytes          # the metric's definition
    prune_bytes = U * S * eb * (D + T) + qobs_bytes if form == 2 else prune_bytes_def
    mean_tail = (steps_per_layer + 1) / 2 if cap else 0
    decode_bytes = U * eb * (S * (T + D) + mean_tail * 2 * D)
    step_bytes = L * (prune_bytes + steps_per_layer * decode_bytes)
    value = step_bytes / (ms_per_step * 1e-3) / 1e9

    prune_launches = thk.thk_prune_launches(shape_all)
    prune_kernel = {2: "k_prune_solo" if prune_launches == 1 else "k_prune_onepass", 1: "k_prune_fused",
                    0: "k_compact_flat"}[form]
    # what the timed kernel itself has to move per launch (the staged form's compaction kernel
    # is only the last of three: rows in, kept channels out)
    prune_kernel_bytes = L * prune_bytes if form else L * U * S * eb * (D + T)
    decode_kernel = "k_decode_mq" if thk.thk_decode_on_matrix_cores(shape_1) else "k_decode"
    kernels = {
        prune_kernel: {"launches_per_step": 1, "avg_us": prune_k_us, "bytes_per_launch": prune_kernel_bytes,
                       "GBps": prune_kernel_bytes / prune_k_us / 1e3},
        decode_kernel: {"launches_per_step": n_dec, "avg_us": dec_k_us, "max_us": max(dec_kernel_us),
                        "timed_launches": len(dec_kernel_us), "bytes_per_launch": decode_bytes,
                        "GBps": decode_bytes / dec_k_us / 1e3},
    }

    def roof_of(name):
        traffic, src = measured_traffic(cfg_id, name)
        return {"bound": "hbm", "kernel": name, "achieved": kernels[name]["GBps"], "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": kernels[name]["GBps"] / HBM_PEAK_GBS,
                "traffic": traffic, "traffic_source": src,
                "launch_us": kernels[name]["avg_us"], "bytes_per_launch": kernels[name]["bytes_per_launch"]}
    # the dominant kernel = most time inside a step
    dom = max(kernels, key=lambda n: kernels[n]["avg_us"] * kernels[n]["launches_per_step"])
    roof = roof_of(dom)
    roof_other = roof_of(next(n for n in kernels if n != dom))

    res = {
        "workload": f"configs[{cfg_id - 1}]: L={L} B={B} N_q={N_q} N_kv={N_kv} D={D} S={S} "
                    f"S_obs={S_obs} lambda={cfg['lam']} T={T} {cfg['dtype']}; prune all layers, "
                    f"then {steps_per_layer} decode step(s) per layer",
        "dtype": cfg["dtype"], "steps": steps, "ms_per_step": ms_per_step, "graph_ms_per_step": graph_ms,
        "step_bytes": step_bytes, "GBps": value, "frac_of_hbm_peak": value / HBM_PEAK_GBS,
        "prune_form": {2: "rows held on chip, K read once", 1: "K read twice", 0: "staged: three kernels per group"}[form],
        "prune_launches": prune_launches,
        "prune_ms_per_layer": prune_ms_layer, "prune_bytes_per_layer": prune_bytes,
        "prune_GBps": prune_bytes / prune_ms_layer / 1e6,
        "prune_frac": prune_bytes / prune_ms_layer / 1e6 / HBM_PEAK_GBS,
        "prune_bytes_per_layer_metric_def": prune_bytes_def,
        "prune_GBps_metric_def": prune_bytes_def / prune_ms_layer / 1e6,
        "decode_us_per_step": dec_us_step, "decode_bytes_per_step": decode_bytes,
        "decode_GBps": decode_bytes / dec_us_step / 1e3,
        "decode_frac": decode_bytes / dec_us_step / 1e3 / HBM_PEAK_GBS,
        "host_wall_s": wall,
        "kernels": kernels, "roofline": roof, "roofline_other": roof_other,
    }
    if full and not args.no_value_cache:
        res["value_cache"] = value_cache_leg(thk, torch, cfg, T, tdt, dt, eb, q_obs, k, v, kp, idx, dec, kt, vt, out,
                                             steps)
    del q_obs, k, v, dec, score, idx, kp, out, kt, vt, ws, pairs, phases, used_pairs
    gc.collect()
    torch.cuda.empty_cache()
    if full and not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(cfg_id, cfg, T, dev)
    return res


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (units are independent; no collective "
              "exists in the path) -- run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2407_21018_amd as thk
    from paper_2407_21018_amd import synth

    torch.cuda.set_device(0)
    head_id = args.config if args.config else HEADLINE
    head = run_config(head_id, args, torch, thk, synth, full=True)
    per_config = []
    for cid in ([args.config] if args.config else sorted(synth.CONFIGS)):
        r = head if cid == head_id else run_config(cid, args, torch, thk, synth, full=False)
        per_config.append({k: v for k, v in r.items() if k not in ("value_cache", "cpu_baseline", "host_wall_s")}
                          | {"config": cid})

    res = {
        "metric": "pruned-K decode attention us/step + achieved HBM GB/s; prune ms per layer",
        "value": head["GBps"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head["dtype"], "data": "synthetic",
        "config": {"workload": head["workload"], "step_bytes": head["step_bytes"]},
        "frac_of_hbm_peak": head["frac_of_hbm_peak"],
        "prune_ms_per_layer": head["prune_ms_per_layer"], "prune_GBps": head["prune_GBps"],
        "prune_frac": head["prune_frac"], "prune_GBps_metric_def": head["prune_GBps_metric_def"],
        "decode_us_per_step": head["decode_us_per_step"], "decode_GBps": head["decode_GBps"],
        "decode_frac": head["decode_frac"],
        "host_wall_s": head["host_wall_s"], "graph_ms_per_step": head["graph_ms_per_step"],
        "kernels": head["kernels"],
        "roofline": head["roofline"],
        "roofline_other": head["roofline_other"],
        "per_config": per_config,
        "device": device_facts(torch),
    }
    for key in ("value_cache", "cpu_baseline"):
        if key in head:
            res[key] = head[key]
    print(json.dumps(res))


if __name__ == "__main__":
    main()
