#!/usr/bin/env python3
"""Benchmark of the G-KV decode/evict hot path on one MI355X.

A "step" is one decode step of the whole path for the whole batch: gkv_attend_decode over every
layer, plus, every s steps, one compression (gkv_score_window, gkv_global_update,
gkv_select_topk, gkv_compact).  The timed region is whole steady-state compression cycles
(cache length cycling b+1 .. b+s), at least TEN of them whatever --steps says, on synthetic
inputs that are already resident in HBM; it is bracketed by device synchronisation on both
sides (wall clock, the figure `value` is computed from) and by HIP events on the launch streams.

Prints ONE JSON line: metric/value (tokens/s = batch * steps / seconds); `roofline`, the attend
kernel against the HBM peak from per-launch HIP events on the launch stream; the same for a
second workload whose K+V cache is more than twice the 256 MB memory-side cache
(`roofline_out_of_cache`); the rate a no-arithmetic reader with the kernel's access pattern gets on
the same caches (`read_ceiling`); and the CPU oracle's rate on a bounded sample (`cpu_baseline`).
"""
import argparse
import ctypes
import json
import os
import statistics
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X published HBM3E bandwidth
MIN_TIMED_CYCLES = 10
CPU_WORKERS_MAX = 16             # the CPU share of a one-GPU machine, whatever its nproc says
OUT_OF_CACHE_WORKLOAD = "cfg4_b512"   # 587 MB of K+V: more than twice the memory-side cache


# ------------------------------------------------------------------------------------------------
# CPU baseline: the fp64 oracle, as it stands, on a bounded sample of the same workload
# ------------------------------------------------------------------------------------------------
def cpu_worker(workload: str, layer: int, seq: int, seconds: float, combine: str, alpha: float):
    """Child process: run the oracle for one (layer, sequence) pair to steady state, then time
    whole compression cycles (s steps + one event) for about `seconds`."""
    from threadpoolctl import threadpool_limits
    import numpy as np  # noqa: F401
    from gkv_traces import CONFIGS, Trace
    from oracle import gkv_oracle as O
    wl = CONFIGS[workload].with_(combine=combine, alpha=alpha)
    with threadpool_limits(limits=1):
        tr = Trace(wl)
        orc = O.OracleA(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.budget, wl.window, wl.interval,
                        capacity=wl.capacity, alpha=wl.alpha, form=wl.combine)
        s = wl.interval
        pre = ((wl.budget + s - 1) // s + 1) * s
        q, k, v = tr.unit_steps(layer, seq, 0, pre)
        for t in range(pre):
            orc.step(t, q[t], k[t], v[t])
        t_next, done, elapsed = pre, 0, 0.0
        while elapsed < seconds:
            q, k, v = tr.unit_steps(layer, seq, t_next, s)
            t0 = time.perf_counter()
            for i in range(s):
                orc.step(t_next + i, q[i], k[i], v[i])
            elapsed += time.perf_counter() - t0
            t_next += s
            done += s
    print(json.dumps({"pair_steps": done, "seconds": elapsed, "events": len(orc.events)}))


def cpu_baseline(workload: str, seconds: float, combine: str, alpha: float):
    from gkv_traces import CONFIGS
    wl = CONFIGS[workload]
    nproc = os.cpu_count() or 1
    n_workers = max(1, min(CPU_WORKERS_MAX, nproc, wl.n_layers * wl.batch))
    procs = []
    for i in range(n_workers):
        layer, seq = (i * 7) % wl.n_layers, i % wl.batch
        procs.append(subprocess.Popen(
            [sys.executable, os.path.abspath(__file__), "--cpu-worker", workload, str(layer), str(seq), str(seconds),
             combine, str(alpha)],
            stdout=subprocess.PIPE, text=True, cwd=ROOT))
    rate, total_steps = 0.0, 0
    for p in procs:
        out, _ = p.communicate()
        try:
            rec = json.loads(out.strip().splitlines()[-1])
        except (IndexError, ValueError):                      # a worker died: count the ones that finished
            n_workers -= 1
            continue
        rate += rec["pair_steps"] / rec["seconds"]            # (layer, sequence)-steps per second
        total_steps += rec["pair_steps"]
    if n_workers == 0:
        return None
    # a decoded token needs one step of every layer of its sequence
    tokens_per_s = rate / wl.n_layers
    return {"value": tokens_per_s, "unit": "tokens/s", "cores": n_workers, "nproc": nproc, "kind": "oracle",
            "sample": (f"{n_workers} (layer, sequence) pairs of {wl.n_layers * wl.batch}, steady-state "
                       f"cycles of {wl.interval} steps + 1 compression, {total_steps} pair-steps in "
                       f"~{seconds:.0f} s per worker, one single-threaded process per pair (the box reports "
                       f"nproc = {nproc}; at most {CPU_WORKERS_MAX} are used, the CPU share of one GPU); "
                       f"scaled by 1/n_layers")}


# ------------------------------------------------------------------------------------------------
def algorithmic_bytes(wl):
    """Bytes the method must move (per unit): attend at length l: e*d*(2l + 2g + 2);
    compression at l = b+s: score e*d*(l + g*w) + 4(l-w); update 4(n_hist + l - w);
    top-k 4(l-w) + 4(b-w); compaction 2*(2*e*d + 8)*m with m <= b rows that move (upper bound m = b)."""
    e = 4 if wl.dtype == "f32" else 2
    d, g, b, w, s = wl.head_dim, wl.group, wl.budget, wl.window, wl.interval
    units = wl.n_units
    l_mean = b + (s + 1) / 2.0
    l = b + s
    return {
        "attend": units * e * d * (2 * l_mean + 2 * g + 2),
        "score": units * (e * d * (l + g * w) + 4 * (l - w)),
        "global": units * 4 * ((b - w) + (l - w)),
        "topk": units * (4 * (l - w) + 4 * (b - w)),
        "compact": units * 2 * (2 * e * d + 8) * b,
        "redundancy": units * (e * d * l + 12 * l),
    }


def read_traffic(workload: str, tag: str):
    """HBM bytes per attend launch from the committed rocprofv3 --pmc summary of this workload, if any
    (counters cannot be read from inside the run; the file names the command that produced it)."""
    name = f"attend_{workload}_{tag}_pmc.txt"
    try:
        with open(os.path.join(ROOT, "profiles", name)) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    return float(line.split(":")[1]), "profiles/" + name
    except OSError:
        pass
    return None, None


def run_workload(wl, args, n_streams, timed_cycles, warm_cycles, kernel_cycles, full_launch, params, workers):
    """Set up `wl` on the GPU in steady state, time `timed_cycles` compression cycles, then measure
    per-launch kernel durations and the read ceiling on the same caches.  Returns a dict."""
    import torch
    from gkv_traces import Trace
    from paper_2512_00504_amd.binding import probe_attend_read
    from paper_2512_00504_amd.state import DecodeState
    dev = torch.device("cuda:0")
    s, b, w = wl.interval, wl.budget, wl.window
    assert b % s == 0 and s % w == 0
    mfma = wl.dtype == "bf16" and wl.head_dim == 128
    # The layers are split into NS groups, each with its own context, buffers and HIP stream.
    # Every decode step launches every group; units are independent, so the groups' kernels may
    # overlap and one group's kernel boundary (launch, first-load latency, final stores) is
    # covered by the other group's streaming.  NS = 1 is the plain one-launch-per-step form.
    NS = max(1, min(n_streams, wl.n_layers))
    bounds = [wl.n_layers * g // NS for g in range(NS + 1)]
    Lgs = [bounds[g + 1] - bounds[g] for g in range(NS)]
    tr = Trace(wl)
    dt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    esz = 2 if wl.dtype == "bf16" else 4
    streams = [torch.cuda.Stream(device=dev) for _ in range(NS)]
    groups = [DecodeState.from_workload(wl.with_(n_layers=Lgs[g]), device=dev, params=params) for g in range(NS)]
    lib = groups[0].ctx.lib
    P = lambda t: ctypes.c_void_p(t.data_ptr())
    ptrs = [dict(h=st.ctx.h, K=P(st.K), V=P(st.V), pos=P(st.pos), qwin=P(st.qwin), state=P(st.d_state),
                 out=P(st.out), ws=P(st.workspace), Fh=P(st.F_hist), S=P(st.S), F=P(st.F), keep=P(st.keep_idx),
                 R=P(st.R), Fsel=P(st.F_sel))
            for st in groups]
    host = {"len": 0}
    rings = [None] * NS

    def split_layers(x):
        """[n, L, ...] numpy -> per-group contiguous device tensors [n, layers of the group, ...]."""
        return [torch.from_numpy(x[:, bounds[g]:bounds[g + 1]]).to(dt).to(dev).contiguous() for g in range(NS)]

    def upload(t0, n):
        q, k, v = tr.batch_steps(t0, n, workers=workers)
        return list(zip(split_layers(q), split_layers(k), split_layers(v)))

    def run(chunk, t0, n, stream_of, cycle_events=None, pre_evict_events=None):
        """n decode steps starting at absolute step t0 on pre-uploaded inputs; raw C calls."""
        len_host = host["len"]
        addr = [(qd.data_ptr(), qd.stride(0) * esz, kd.data_ptr(), kd.stride(0) * esz, vd.data_ptr(), vd.stride(0) * esz)
                for (qd, kd, vd) in chunk]
        for i in range(n):
            t = t0 + i
            for g in range(NS):
                p = ptrs[g]
                qb, qs, kb_, ks, vb, vs = addr[g]
                # Default: q is copied into the context's own ring by the decode kernel.
                # --ring-in-place: the pre-uploaded q tensors of w consecutive steps are laid out
                # exactly like a ring [w, L, B, h_q, d] (chunks start at multiples of s, and w divides
                # s), so step t's q already is slot t % w of that ring and nothing is copied.
                ring = qb + (i - i % w) * qs if args.ring_in_place else p["qwin"]
                rings[g] = ring
                rc = lib.gkv_attend_decode(p["h"], qb + i * qs, kb_ + i * ks, vb + i * vs, p["K"], p["V"], p["pos"], t,
                                           ring, p["state"], len_host, p["out"], p["ws"], stream_of[g])
                if rc:
                    raise RuntimeError(f"gkv_attend_decode failed: {rc}")
            len_host += 1
            if (t + 1) % s == 0 and len_host > b:
                if pre_evict_events is not None:          # end of this cycle's decode launches, per stream
                    evs = []
                    for g in range(NS):
                        ev = torch.cuda.Event(enable_timing=True)
                        ev.record(streams[g])
                        evs.append(ev)
                    pre_evict_events.append(evs)
                for g in range(NS):
                    p = ptrs[g]
                    if args.redundancy is None:
                        rc = lib.gkv_evict(p["h"], rings[g], p["K"], p["V"], p["Fh"], p["pos"], p["state"], t, len_host,
                                           p["S"], p["F"], p["keep"], p["ws"], stream_of[g])
                    else:
                        lam, tau = args.redundancy
                        sg = stream_of[g]
                        rc = (lib.gkv_score_window(p["h"], rings[g], p["K"], p["state"], t, len_host, p["S"], p["ws"], sg)
                              or lib.gkv_global_update(p["h"], p["S"], p["Fh"], p["state"], t, len_host, p["F"], sg)
                              or lib.gkv_redundancy_combine(p["h"], p["K"], p["state"], t, len_host, p["F"], lam, tau,
                                                            1e-8, wl.window, p["R"], p["Fsel"], p["ws"], sg)
                              or lib.gkv_select_topk(p["h"], p["Fsel"], p["state"], t, len_host, p["keep"], p["ws"], sg)
                              or lib.gkv_compact(p["h"], p["keep"], p["F"], p["K"], p["V"], p["Fh"], p["pos"], p["state"],
                                                 t, p["ws"], sg))
                    if rc:
                        raise RuntimeError(f"compression failed: {rc}")
                len_host = b
        host["len"] = len_host
        if cycle_events is not None:
            evs = []
            for g in range(NS):
                ev = torch.cuda.Event(enable_timing=True)
                ev.record(streams[g])
                evs.append(ev)
            cycle_events.append(evs)

    own_streams = [ctypes.c_void_p(st_.cuda_stream) for st_ in streams]
    one_stream = [own_streams[0]] * NS

    # The first b tokens are placed in the cache directly: no compression happens before the
    # cache exceeds the budget, so this is the state b decode steps leave behind, and every
    # attend launch of this process then runs at a steady-state length b+1 .. b+s.
    if args.fast_prefix:
        _, k0, v0 = tr.batch_steps(0, s, workers=workers, need_q=False)
        reps = (b + s - 1) // s
        k0s = [x.repeat(reps, 1, 1, 1, 1)[:b] for x in split_layers(k0)]
        v0s = [x.repeat(reps, 1, 1, 1, 1)[:b] for x in split_layers(v0)]
    else:
        _, k0, v0 = tr.batch_steps(0, b, workers=workers, need_q=False)
        k0s, v0s = split_layers(k0), split_layers(v0)
    for g, st in enumerate(groups):
        st.load_prefix(k0s[g], v0s[g])
    del k0, v0, k0s, v0s
    host["len"] = b
    torch.cuda.synchronize()
    t_abs = b
    for _ in range(max(1, warm_cycles)):                  # untimed warm-up cycles (first compression)
        chunk = upload(t_abs, s)
        torch.cuda.synchronize()
        run(chunk, t_abs, s, own_streams)
        t_abs += s
    torch.cuda.synchronize()
    for st in groups:
        lens = st.lengths(t_abs)
        assert int(lens.max()) == b and int(lens.min()) == b

    # ---- the timed region: whole compression cycles, inputs resident in HBM ---------------------
    K = timed_cycles * s
    chunks = [upload(t_abs + c * s, s) for c in range(timed_cycles)]
    torch.cuda.synchronize()
    if not args.graph:
        cyc, pre = [], []
        run([], 0, 0, own_streams, cyc)                   # records the start events, enqueues nothing else
        t_wall = time.perf_counter()
        for ci, chunk in enumerate(chunks):
            run(chunk, t_abs + ci * s, s, own_streams, cyc, pre)
        torch.cuda.synchronize()
        wall_s = time.perf_counter() - t_wall
        start = cyc[0]
        gpu_s = 1e-3 * max(start[h].elapsed_time(cyc[-1][g]) for g in range(NS) for h in range(NS))
        cyc_ms = [max(cyc[c][g].elapsed_time(cyc[c + 1][g]) for g in range(NS)) for c in range(timed_cycles)]
        # the decode launches alone, as the timed region runs them: per stream, from the end of one
        # compression to the start of the next (s launches); the streams' rates add up
        attend_ms = [[cyc[c][g].elapsed_time(pre[c][g]) for c in range(timed_cycles)] for g in range(NS)]
        t_abs += K
    else:
        attend_ms = None
        # The same launches recorded once into a HIP graph (one branch per layer group) and replayed
        # with a single call: the step number comes from a device-side step base that the graph
        # itself advances, so the recording is valid for every replay.  Replays reuse the inputs
        # of the recorded cycles.
        bases = [torch.tensor([t_abs], dtype=torch.int32, device=dev) for _ in range(NS)]
        for g, st in enumerate(groups):
            st.ctx.set_step_base(bases[g])
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=streams[0]):
            for g in range(1, NS):
                streams[g].wait_stream(streams[0])
            for ci, chunk in enumerate(chunks):
                run(chunk, ci * s, s, own_streams)        # steps relative to the step base
            for g in range(NS):
                if lib.gkv_advance_step_base(ptrs[g]["h"], K, own_streams[g]):
                    raise RuntimeError("gkv_advance_step_base failed")
            for g in range(1, NS):
                streams[0].wait_stream(streams[g])
        torch.cuda.synchronize()
        with torch.cuda.stream(streams[0]):
            graph.replay()                                # untimed: first replay uploads the graph
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            t_wall = time.perf_counter()
            e0.record()
            graph.replay()
            e1.record()
            torch.cuda.synchronize()
            wall_s = time.perf_counter() - t_wall
        gpu_s = 1e-3 * e0.elapsed_time(e1)
        cyc_ms = [1e3 * gpu_s / timed_cycles]
        t_abs += 2 * K
        assert all(int(x.item()) == t_abs for x in bases)
        for st in groups:
            st.ctx.set_step_base(None)

    # ---- per-kernel durations: a few of the same cycles again with every launch bracketed by its
    # own HIP events, all groups on ONE stream so that a launch's duration is the kernel's own
    for st in groups:
        st.ctx.profile_reset()
        st.ctx.profile_enable(True)
    for ci, chunk in enumerate(chunks[:kernel_cycles]):
        run(chunk, t_abs + ci * s, s, one_stream)
    torch.cuda.synchronize()
    t_abs += kernel_cycles * s
    per_kernel = {}
    for name in ("attend", "score", "global", "topk", "compact") + (("redundancy",) if args.redundancy else ()):
        ms = n = 0
        for st in groups:
            st.ctx.profile_enable(False)
            m_, n_ = st.ctx.profile_read(name)
            ms += m_; n += n_
        per_kernel[name] = {"launches": n, "avg_us": (1e3 * ms / n) if n else None}

    alg = algorithmic_bytes(wl)                       # whole batch, all layers
    for name in per_kernel:
        us = per_kernel[name]["avg_us"]
        per_kernel[name]["algorithmic_MB"] = alg[name] / NS / 1e6
        per_kernel[name]["GBps"] = (alg[name] / NS / (us * 1e-6) / 1e9) if us else None
        per_kernel[name]["hbm_frac"] = (per_kernel[name]["GBps"] / HBM_PEAK_GBS) if us else None

    # ---- the read ceiling on these very caches: the decode kernel's access pattern, no arithmetic
    def ceiling(K_t, V_t):
        if not mfma:
            return None
        rows = (b + s // 2) // 16 * 16
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        for _ in range(5):
            probe_attend_read(K_t, V_t, rows, sink)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 40
        e0.record()
        for _ in range(reps):
            probe_attend_read(K_t, V_t, rows, sink)
        e1.record()
        torch.cuda.synchronize()
        units = K_t.numel() // (K_t.shape[-2] * K_t.shape[-1])
        nbytes = units * rows * 512
        us = 1e3 * e0.elapsed_time(e1) / reps
        return {"units": units, "rows": rows, "bytes_per_launch": nbytes, "avg_launch_us": us,
                "GBps": nbytes / (us * 1e-6) / 1e9, "hbm_frac": nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS}

    ceil_group = ceiling(groups[0].K, groups[0].V)

    # the reader's rate against the size of what it re-reads (fresh buffers of the same layout): if the
    # 256 MB memory-side cache served repeated reads faster than HBM, the small sets would stand out
    sweep = None
    if mfma and not args.leg and wl.n_units >= 448:
        sweep = []
        for units in (448, 896, 1792, 3584):
            Kb = torch.ones(units, wl.capacity, wl.head_dim, dtype=dt, device=dev)
            Vb = torch.ones(units, wl.capacity, wl.head_dim, dtype=dt, device=dev)
            c = ceiling(Kb, Vb)
            sweep.append({"working_set_MB": 2 * Kb.numel() * esz / 1e6, "GBps": c["GBps"]})
            del Kb, Vb

    # the same reader on every group's cache at once, each on its group's stream, as the timed
    # region runs the decode kernel: the ceiling for the overlapped launches
    ceil_overlap = None
    if mfma and NS > 1:
        rows = (b + s // 2) // 16 * 16
        sinks = [torch.zeros(4, dtype=torch.int32, device=dev) for _ in range(NS)]
        reps = 40
        torch.cuda.synchronize()
        e0 = [torch.cuda.Event(enable_timing=True) for _ in range(NS)]
        e1 = [torch.cuda.Event(enable_timing=True) for _ in range(NS)]
        for g in range(NS):
            e0[g].record(streams[g])
        for _ in range(reps):
            for g in range(NS):
                with torch.cuda.stream(streams[g]):
                    probe_attend_read(groups[g].K, groups[g].V, rows, sinks[g])
        for g in range(NS):
            e1[g].record(streams[g])
        torch.cuda.synchronize()
        ms = max(e0[h].elapsed_time(e1[g]) for g in range(NS) for h in range(NS))
        nbytes = sum(st.K.numel() // (st.K.shape[-2] * st.K.shape[-1]) for st in groups) * rows * 512
        ceil_overlap = {"bytes_per_round": nbytes, "avg_round_us": 1e3 * ms / reps,
                        "GBps": nbytes * reps / (ms * 1e-3) / 1e9, "hbm_frac": nbytes * reps / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}

    # ---- the same kernel launched once for all layers (one context, one stream): its duration at
    # the full shape.  The cache contents are the groups' current ones, the inputs the timed chunks.
    full = ceil_full = None
    if NS > 1 and full_launch:
        fs = DecodeState.from_workload(wl, device=dev, params=params)
        for name in ("K", "V", "pos", "F_hist"):
            getattr(fs, name).copy_(torch.cat([getattr(g_, name) for g_ in groups], dim=0))
        fs.qwin.copy_(torch.cat([g_.qwin for g_ in groups], dim=1))
        fs.d_state.copy_(torch.cat([g_.d_state for g_ in groups], dim=0))
        fs.len_host = host["len"]
        fs.ctx.profile_enable(True)
        t_f = t_abs
        for ci, chunk in enumerate(chunks[:kernel_cycles]):
            qf, kf, vf = [torch.cat([chunk[g][i] for g in range(NS)], dim=1).contiguous() for i in range(3)]
            for i in range(s):
                fs.attend_decode(qf[i], kf[i], vf[i], t_f)
                if fs.is_trigger(t_f):
                    fs.evict(t_f)
                t_f += 1
        torch.cuda.synchronize()
        ms, n = fs.ctx.profile_read("attend")
        fs.ctx.profile_enable(False)
        us = 1e3 * ms / n
        full = {"launches": n, "avg_launch_us": us, "algorithmic_bytes_per_launch": alg["attend"],
                "achieved": alg["attend"] / (us * 1e-6) / 1e9,
                "frac": alg["attend"] / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, "unit": "GB/s"}
        ceil_full = ceiling(fs.K, fs.V)
        del fs

    sustained = None
    if attend_ms is not None:
        # algorithmic bytes of a stream's s launches of a cycle over the time that stream spent on them
        rate = sum(alg["attend"] / NS * s / (statistics.median(ms) * 1e-3) / 1e9 for ms in attend_ms)
        sustained = {"GBps": rate, "frac": rate / HBM_PEAK_GBS,
                     "note": "decode launches only, timed in the timed region itself with HIP events per stream and cycle; "
                             "with more than one stream the launches overlap, so this is a sustained rate, not a launch duration"}
    att_us = per_kernel["attend"]["avg_us"]           # one launch = one group = n_layers / NS layers
    achieved = alg["attend"] / NS / (att_us * 1e-6) / 1e9
    evict_bytes = alg["score"] + alg["global"] + alg["topk"] + alg["compact"] + (alg["redundancy"] if args.redundancy else 0)
    bytes_per_step = alg["attend"] + evict_bytes / s
    kv_bytes = sum(st.K.numel() * esz * 2 for st in groups)
    tag = f"s{NS}"
    traffic, traffic_src = read_traffic(wl.name, tag)
    return {
        "workload": wl.name, "steps": K, "cycles": timed_cycles, "streams": NS, "layers_per_launch": max(Lgs),
        "tokens_per_s": wl.batch * K / wall_s, "ms_per_step": 1e3 * wall_s / K,
        "wall_seconds": wall_s, "gpu_seconds": gpu_s,
        "tokens_per_s_gpu_clock": wl.batch * K / gpu_s,
        "cycle_ms": {"min": min(cyc_ms), "median": statistics.median(cyc_ms), "max": max(cyc_ms)},
        "kv_cache_bytes": kv_bytes,
        "roofline": {"bound": "hbm", "kernel": "attend_mfma_kernel" if mfma else "attend_generic_kernel",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_src,
                     "algorithmic_bytes_per_launch": alg["attend"] / NS, "avg_launch_us": att_us,
                     "launches_per_step": NS, "launches_timed": per_kernel["attend"]["launches"],
                     "sustained_in_timed_region": sustained,
                     "note": "launch durations from HIP events on the launch stream, the groups' launches "
                             "serialised on one stream so that a duration is the kernel's own; the timed region "
                             "runs the groups on separate streams"},
        "roofline_all_layers_one_launch": full,
        "read_ceiling": {"per_group_launch": ceil_group, "all_layers": ceil_full, "groups_overlapped": ceil_overlap,
                         "working_set_sweep": sweep,
                         "note": "the decode kernel's load pattern with no arithmetic, merge or stores, on the same caches "
                                 "(the sweep: on fresh buffers of growing size, each re-read 45 times)"},
        "whole_step": {"algorithmic_bytes_per_step": bytes_per_step,
                       "GBps": bytes_per_step * K / wall_s / 1e9,
                       "hbm_frac": bytes_per_step * K / wall_s / 1e9 / HBM_PEAK_GBS,
                       "fits_memory_side_cache_twice": kv_bytes < 2 * (256 << 20),
                       "note": ("K+V cache of %.0f MB against a 256 MB memory-side cache: part of a step's reads may be "
                                "served from that cache, so this is a rate in algorithmic bytes, not proven HBM traffic; "
                                "see roofline_out_of_cache for a cache more than twice that size, and "
                                "read_ceiling.working_set_sweep for what the cache does to this access pattern"
                                % (kv_bytes / 1e6)) if kv_bytes < 2 * (256 << 20) else
                               ("K+V cache of %.0f MB, more than twice the 256 MB memory-side cache" % (kv_bytes / 1e6))},
        "per_kernel": per_kernel,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1280)
    ap.add_argument("--warmup", type=int, default=256)
    ap.add_argument("--workload", default="cfg3_28layer_b512")
    ap.add_argument("--combine", choices=["max", "avg", "sum"], default=None,
                    help="global-score form (default: the workload's, max)")
    ap.add_argument("--alpha", type=float, default=None, help="memory-decay rate (default: the workload's, 0.8)")
    ap.add_argument("--redundancy", nargs=2, type=float, metavar=("LAMBDA", "TAU"), default=None,
                    help="select on lambda*F - (1-lambda)*R' (redundancy score with threshold TAU, the window "
                         "rows exempt): the paper's full G-KV; the CPU baseline leg is then skipped")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--streams", type=int, default=2,
                    help="split the layers into this many groups, each launched on its own HIP stream")
    ap.add_argument("--ring-in-place", action="store_true",
                    help="treat the pre-uploaded q tensors as the window ring itself (q of step t already is slot "
                         "t %% w), so the decode kernel copies nothing; by default q is copied into the context's ring")
    ap.add_argument("--splits", type=int, default=0)
    ap.add_argument("--tile", type=int, default=0, help="attend_tile knob (16 or 32); 0 = library default")
    ap.add_argument("--param", action="append", default=[], metavar="NAME=VALUE",
                    help="set a library tuning knob (gkv_set_param), e.g. compact_ppt=8; may be repeated")
    ap.add_argument("--fast-prefix", action="store_true",
                    help="fill the cache prefix by repeating the first s generated steps (for the largest workloads)")
    ap.add_argument("--min-cycles", type=int, default=MIN_TIMED_CYCLES,
                    help="time at least this many compression cycles whatever --steps says")
    ap.add_argument("--no-full-launch", action="store_true",
                    help="skip the extra pass that times the attend kernel launched once for all layers")
    ap.add_argument("--no-out-of-cache-leg", action="store_true",
                    help="skip the second workload (K+V cache over twice the memory-side cache) of the default run")
    ap.add_argument("--graph", action="store_true",
                    help="record the timed cycles into one HIP graph (one branch per layer group, device-side step "
                         "base) and time a single replay instead of launching call by call")
    ap.add_argument("--leg", action="store_true",
                    help="(internal) run as the second workload of a default run: print the workload's own record")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain 1 GiB device copy (for scaling rocprofv3 --pmc counters)")
    ap.add_argument("--cpu-worker", nargs=6, metavar=("WORKLOAD", "LAYER", "SEQ", "SECONDS", "COMBINE", "ALPHA"))
    args = ap.parse_args()

    if args.cpu_worker:
        wlname, layer, seq, secs, comb, alpha = args.cpu_worker
        cpu_worker(wlname, int(layer), int(seq), float(secs), comb, float(alpha))
        return
    if args.gpus != 1:
        print("bench.py: this build measures one GPU; --gpus must be 1 (no multi-GPU path exists)", file=sys.stderr)
        sys.exit(2)

    from gkv_traces import CONFIGS
    wl = CONFIGS[args.workload]
    if args.combine is not None:
        wl = wl.with_(combine=args.combine)
    if args.alpha is not None:
        wl = wl.with_(alpha=args.alpha)

    # CPU leg first, before this process touches the GPU (children are plain CPU processes)
    cpu = None
    if not args.no_cpu_baseline and not args.copy_calibration and not args.leg and args.redundancy is None:
        cpu = cpu_baseline(args.workload, args.cpu_seconds, wl.combine, wl.alpha)

    # Second workload of the default run: the same shape at batch 16, whose 587 MB of K+V cannot sit
    # in the 256 MB memory-side cache.  Same measurement, fewer cycles, in a process of its own that
    # has finished before this one touches the GPU (a fresh address space and allocator state).
    ooc = None
    if (wl.name == "cfg3_28layer_b512" and not args.no_out_of_cache_leg and not args.leg
            and not args.copy_calibration and args.redundancy is None):
        cmd = [sys.executable, os.path.abspath(__file__), "--leg", "--workload", OUT_OF_CACHE_WORKLOAD,
               "--min-cycles", "4", "--steps", "1", "--warmup", "1", "--streams", str(args.streams),
               "--combine", wl.combine, "--alpha", str(wl.alpha)]
        for item in args.param:
            cmd += ["--param", item]
        if args.ring_in_place:
            cmd.append("--ring-in-place")
        if args.no_full_launch:
            cmd.append("--no-full-launch")
        child = subprocess.run(cmd, stdout=subprocess.PIPE, text=True, cwd=ROOT)
        try:                                              # the main line is printed whatever happens to this leg
            if child.returncode != 0:
                raise RuntimeError(f"exit status {child.returncode}")
            ooc = json.loads(child.stdout.strip().splitlines()[-1])
        except Exception as e:                            # noqa: BLE001
            ooc = {"workload": OUT_OF_CACHE_WORKLOAD, "error": f"leg failed: {e}"}

    import torch
    dev = torch.device("cuda:0")

    if args.copy_calibration:
        n = 1 << 30
        src = torch.empty(n, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": n, "copy_bytes_written": n, "launches": 5}))
        return

    s, b = wl.interval, wl.budget
    timed_cycles = max(args.min_cycles, (args.steps + s - 1) // s, 1)     # whole compression cycles
    warm_cycles = max(1, (args.warmup + s - 1) // s)
    params = {}
    if args.splits:
        params["attend_splits"] = args.splits
    if args.tile:
        params["attend_tile"] = args.tile
    for item in args.param:
        name, val = item.split("=")
        params[name] = int(val)
    workers = max(1, min(CPU_WORKERS_MAX, os.cpu_count() or 1))

    res = run_workload(wl, args, args.streams, timed_cycles, warm_cycles, kernel_cycles=min(2, timed_cycles),
                       full_launch=not args.no_full_launch, params=params, workers=workers)

    if args.leg:
        print(json.dumps({k: res[k] for k in ("workload", "kv_cache_bytes", "steps", "streams", "tokens_per_s",
                                              "ms_per_step", "roofline", "roofline_all_layers_one_launch",
                                              "read_ceiling", "whole_step", "per_kernel")}))
        return

    out = {
        "metric": "decode tokens/sec through attend+score+evict at budget 512; % HBM roofline"
                  if b == 512 else f"decode tokens/sec through attend+score+evict at budget {b}",
        "value": res["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": res["steps"], "warmup": warm_cycles * s,
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "n_layers": wl.n_layers, "batch": wl.batch,
                   "n_q_heads": wl.n_q_heads, "n_kv_heads": wl.n_kv_heads, "head_dim": wl.head_dim,
                   "budget": b, "window": wl.window, "interval": s, "alpha": wl.alpha,
                   "combine": wl.combine, "trace": wl.recipe, "preroll_steps": b,
                   "params": params, "fast_prefix": args.fast_prefix,
                   "streams": res["streams"], "layers_per_launch": res["layers_per_launch"],
                   "redundancy": args.redundancy, "ring": "in place" if args.ring_in_place else "copy",
                   "launch": "one HIP graph replay" if args.graph else "call by call",
                   "steps_requested": args.steps, "timed_cycles": res["cycles"],
                   "note": f"the timed region is whole compression cycles, at least {args.min_cycles}"},
        "roofline": res["roofline"],
        "roofline_all_layers_one_launch": res["roofline_all_layers_one_launch"],
        "roofline_out_of_cache": ooc,
        "read_ceiling": res["read_ceiling"],
        "cpu_baseline": cpu,
        "whole_step": dict(res["whole_step"], wall_seconds=res["wall_seconds"], gpu_seconds=res["gpu_seconds"],
                           tokens_per_s_gpu_clock=res["tokens_per_s_gpu_clock"], cycle_ms=res["cycle_ms"]),
        "per_kernel": res["per_kernel"],
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
