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

Ceilings.  `plain_streams` (every workload) times the library's plain read and copy kernels
(thk_bench_stream) on cold buffers of the workload's own sizes -- a read of the bytes of one decode
launch, a copy with the traffic of one prune launch -- and gives the library's kernels' rates as
fractions of those: what the chip grants a launch of that size, beside the 8 TB/s peak.
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
    ap.add_argument("--no-plain-streams", action="store_true",
                    help="skip the plain read / copy kernels of the workload's own sizes (plain_streams: the ceilings)")
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
            "decode_kv_us_per_step": dec_us, "decode_kv_bytes": dec_bytes, "decode_kv_GBps": dec_bytes / dec_us / 1e3,
            "decode_kv_frac_of_hbm_peak": dec_bytes / dec_us / 1e3 / HBM_PEAK_GBS,
            "decode_kv_bytes_vs_k_only": (T + T_v) / (T + D)}


def plain_streams(thk, torch, k_launch_bytes, T, D, decode_bytes, reps=6):
    """What the chip gives kernels that only move the bytes of one prune launch and of one decode
    launch (thk_bench_stream: plain read; copy with the rows held in registers and w / 32 = T / D
    of them written, no exchange between blocks), on cold buffers, by events attached to the
    launches like the library's own kernels: the ceilings at the workload's own size."""
    dev = "cuda:0"
    blk = 128 << 10
    nb_copy = max(1, k_launch_bytes // blk)
    w = max(1, min(32, round(32 * T / D)))
    nb_read = max(1, -(-int(decode_bytes) // blk))
    # windows of a buffer of at least 1.5 GiB, so that a window is cold when its turn comes again
    nwin_r = max(1, min(16, -(-(3 << 29) // (nb_read * blk))))
    nwin_c = max(1, min(16, -(-(3 << 29) // (nb_copy * blk))))
    src = torch.empty(max(nb_read * nwin_r, nb_copy * nwin_c) * blk, dtype=torch.uint8, device=dev).random_(0, 255)
    dst = torch.empty(nb_copy * w * 4096 * nwin_c, dtype=torch.uint8, device=dev)

    def run(mode, nb, nwin, wbytes):
        us = []
        for i in range(reps + 2):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(); b.record()
            k = i % nwin
            thk.thk_profile_next(a, b)
            thk.thk_bench_stream(mode, src[k * nb * blk:(k + 1) * nb * blk],
                                 dst[k * wbytes:(k + 1) * wbytes] if mode == thk.THK_STREAM_COPY else None, nb, w)
            torch.cuda.synchronize()
            if i >= 2:
                us.append(a.elapsed_time(b) * 1e3)
        return us
    r_us = run(thk.THK_STREAM_READ, nb_read, nwin_r, 0)
    c_us = run(thk.THK_STREAM_COPY, nb_copy, nwin_c, nb_copy * w * 4096)
    r_bytes, c_bytes = nb_read * blk, nb_copy * (blk + w * 4096)
    del src, dst
    torch.cuda.empty_cache()
    mean = lambda x: sum(x) / len(x)
    return {"kernel": "thk_bench_stream (plain kernels: no exchange, no arithmetic)", "launches_timed": reps,
            "read": {"bytes": r_bytes, "us": mean(r_us), "best_us": min(r_us), "GBps": r_bytes / mean(r_us) / 1e3},
            "copy": {"bytes": c_bytes, "written_fraction": w / 32, "us": mean(c_us), "best_us": min(c_us),
                     "GBps": c_bytes / mean(c_us) / 1e3}}


def plain_read_us(thk, torch, nbytes, reps=6):
    """Mean and best duration (us) of a plain read (thk_bench_stream) of nbytes, on cold windows
    of a buffer of at least 1.5 GiB, by events attached to the launches."""
    blk = 128 << 10
    nb = max(1, -(-int(nbytes) // blk))
    nwin = max(1, min(16, -(-(3 << 29) // (nb * blk))))
    src = torch.empty(nb * nwin * blk, dtype=torch.uint8, device="cuda:0").random_(0, 255)
    us = []
    for i in range(reps + 2):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(); b.record()
        k = i % nwin
        thk.thk_profile_next(a, b)
        thk.thk_bench_stream(thk.THK_STREAM_READ, src[k * nb * blk:(k + 1) * nb * blk], None, nb, 1)
        torch.cuda.synchronize()
        if i >= 2:
            us.append(a.elapsed_time(b) * 1e3)
    del src
    torch.cuda.empty_cache()
    return sum(us) / len(us), min(us)


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
    """Time workload cfg_id.  full: also the value-cache leg and the oracle leg (headline only).

    Four timed regions, all with inputs resident and warmed up:
      A  `steps` whole steps back to back, two events around all of them -> ms_per_step, value;
      B  the step's prune call alone, back to back                        -> prune_ms_per_layer;
      C  the step's decode calls alone (all layers and steps), back to back -> decode_us_per_step;
      D  a few steps whose main kernels carry event pairs (thk_profile_next) -> kernel durations.
    Small workloads rotate over several input sets so that no region re-reads a cache-resident
    tensor: a set is used again only after more than 1.5 GiB of other sets' tensors (the
    memory-side cache holds 256 MB)."""
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
    n_dec = steps_per_layer * L

    # ---- inputs, resident in HBM ------------------------------------------
    set_bytes = L * U * S * eb * (2 * D + T)
    nrot = max(1, min(16, -(-(3 << 29) // set_bytes)))
    q_obs = torch.empty(L, B, N_q, S_obs, D, dtype=dt, device=dev)
    k0 = torch.empty(L, B, N_kv, S, D, dtype=dt, device=dev)
    v0 = torch.empty(L, B, N_kv, S, D, dtype=dt, device=dev)
    for l in range(L):
        q_obs[l], k0[l], v0[l] = (t[0] for t in synth.gen_prefill(cfg_id, l, dev, **cfg))
    # further sets hold the same values (the timing does not depend on them, parity is checked elsewhere)
    ks = [k0] + [k0.clone() for _ in range(nrot - 1)]
    vs = [v0] + [v0.clone() for _ in range(nrot - 1)]
    kps = [torch.empty(L, U, S, T, dtype=dt, device=dev) for _ in range(nrot)]
    dec = [[synth.gen_decode(cfg_id, l, s, dev, **cfg) for s in range(steps_per_layer)] for l in range(L)]
    score = torch.empty(L * U, D, dtype=torch.float32, device=dev)
    idx = torch.empty(L * U, T, dtype=torch.int16, device=dev)
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
        e.record()          # torch creates the HIP event on first record; done outside the timed regions
        return e

    # per-(set, layer) views made once: slicing a tensor costs the host several microseconds, which
    # the smallest workload's calls (about 10 us each) would not hide
    kp_l = [[kps[r][l] for l in range(L)] for r in range(nrot)]
    v_l = [[vs[r][l] for l in range(L)] for r in range(nrot)]
    idx_l = [idx[l * U:(l + 1) * U] for l in range(L)]
    kt_l = [kt[l] if cap else None for l in range(L)]
    vt_l = [vt[l] if cap else None for l in range(L)]
    out_l = [out[l] for l in range(L)]

    def prune(r, pair=None):
        if pair is not None:
            thk.thk_profile_next(*pair)
        thk.thk_prune(shape_all, q_obs, ks[r], score, idx, kps[r], ws)

    def decode(r, pairs=None, rot=0):
        """The decode calls of one step; pairs: event pairs for every eighth call (offset rot)."""
        i, call, used = 0, 0, []
        for s in range(steps_per_layer):
            for l in range(L):
                q, k_new, v_new = dec[l][s]
                if cap:
                    thk.thk_tail_append(shape_1, k_new, v_new, kt_l[l], vt_l[l], s, cap)
                if pairs is not None and call % 8 == rot % min(8, n_dec) and i < len(pairs):
                    thk.thk_profile_next(*pairs[i])
                    used.append(pairs[i])
                    i += 1
                call += 1
                thk.thk_decode_attn(shape_1, q, kp_l[r][l], idx_l[l], v_l[r][l], kt_l[l], vt_l[l],
                                    s + 1 if cap else 0, cap, out_l[l], ws)
        return used

    def step(r):
        prune(r)
        decode(r)

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)          # reads 1 GiB, writes 1 GiB per dispatch
        torch.cuda.synchronize()
        del src, dst

    def timed(fn, reps):
        """fn(i) for i < reps back to back between two events: milliseconds per repetition."""
        a, b = ev(), ev()
        torch.cuda.synchronize()
        a.record()
        for i in range(reps):
            fn(i)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    for r in range(max(args.warmup, nrot)):
        step(r % nrot)          # every set gets its pruned cache
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ms_per_step = timed(lambda i: step(i % nrot), steps)                       # region A
    wall = time.perf_counter() - t0
    # the phase loops of a short step run longer than `steps` repetitions (about 30 ms each)
    reps_ph = min(300, max(steps, int(30.0 / ms_per_step)))
    prune_ms_layer = timed(lambda i: prune(i % nrot), reps_ph) / L             # region B
    dec_us_step = timed(lambda i: decode(i % nrot), reps_ph) / n_dec * 1e3     # region C
    # region D: kernel durations from events attached to the launches themselves.  Such a launch
    # costs the host ~12 us more than a plain one, so only every eighth decode call carries a pair.
    n_prof = max(1, n_dec // 8)
    ksteps = min(steps, 5)
    pairs = [[(ev(), ev()) for _ in range(1 + n_prof)] for _ in range(ksteps)]
    torch.cuda.synchronize()
    used_pairs = []
    for i in range(ksteps):
        prune(i % nrot, pairs[i][0])
        used_pairs += decode(i % nrot, pairs[i][1:], i)
    torch.cuda.synchronize()
    prune_k_us = sum(p[0][0].elapsed_time(p[0][1]) for p in pairs) / ksteps * 1e3
    dec_kernel_us = [a.elapsed_time(b) * 1e3 for (a, b) in used_pairs]
    dec_k_us = sum(dec_kernel_us) / len(dec_kernel_us)

    graph_ms = None
    if not args.no_graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step(0)
        torch.cuda.current_stream().wait_stream(side)
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr):
            for r in range(nrot):
                step(r)
        gr.replay()
        graph_ms = timed(lambda i: gr.replay(), max(1, steps // nrot)) / nrot
        del gr

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
        "input_sets_rotated": nrot, "phase_loop_reps": reps_ph,
        "cache_state": "cold: more than 1.5 GiB of other tensors pass between two uses of a tensor",
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
        "phases_vs_step": (prune_ms_layer * L + dec_us_step * n_dec / 1e3) / ms_per_step,
        "host_wall_s": wall,
        "kernels": kernels, "roofline": roof, "roofline_other": roof_other,
    }
    if full and not args.no_value_cache:
        res["value_cache"] = value_cache_leg(thk, torch, cfg, T, tdt, dt, eb, q_obs, k0, v0, kps[0], idx, dec, kt, vt,
                                             out, steps)
    del q_obs, k0, v0, ks, vs, kps, dec, score, idx, out, kt, vt, ws, pairs, used_pairs, kp_l, v_l, idx_l, kt_l, vt_l, out_l
    gc.collect()
    torch.cuda.empty_cache()
    if not args.no_plain_streams:
        ps = plain_streams(thk, torch, L * U * S * D * eb, T, D, decode_bytes)
        ps["decode_kernel_vs_read"] = kernels[decode_kernel]["GBps"] / ps["read"]["GBps"]
        if form == 2:
            ps["prune_kernel_vs_copy"] = kernels[prune_kernel]["GBps"] / ps["copy"]["GBps"]
        res["plain_streams"] = ps
        if "value_cache" in res:
            # the decode step over both pruned caches moves fewer bytes per launch: its own ceiling
            vc = res["value_cache"]
            r_us, r_best = plain_read_us(thk, torch, vc["decode_kv_bytes"])
            vc["decode_kv_plain_read_us"] = r_us
            vc["decode_kv_call_vs_read"] = r_us / vc["decode_kv_us_per_step"]
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
    for key in ("plain_streams", "value_cache", "cpu_baseline"):
        if key in head:
            res[key] = head[key]
    print(json.dumps(res))


if __name__ == "__main__":
    main()
