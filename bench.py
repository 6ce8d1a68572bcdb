#!/usr/bin/env python3
"""Benchmark of the G-KV decode/evict hot path on one MI355X.

A "step" is one decode step of the whole path for the whole batch: one
gkv_attend_decode launch covering every layer, plus, every s steps, one
compression (gkv_score_window, gkv_global_update, gkv_select_topk,
gkv_compact).  The timed region is K consecutive steady-state steps (cache
length cycling b+1 .. b+s) on synthetic inputs that are already resident in
HBM; it is bracketed by device synchronisation on both sides.

Prints ONE JSON line: metric/value (tokens/s = batch * K / seconds), the
roofline object of the dominant kernel (attend) from per-launch HIP events
recorded on the launch stream, and the CPU oracle's rate on a bounded sample.
"""
import argparse
import ctypes
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X published HBM3E bandwidth


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
    n_workers = max(1, min(16, os.cpu_count() or 1, wl.n_layers * wl.batch))
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
        rec = json.loads(out.strip().splitlines()[-1])
        rate += rec["pair_steps"] / rec["seconds"]            # (layer, sequence)-steps per second
        total_steps += rec["pair_steps"]
    # a decoded token needs one step of every layer of its sequence
    tokens_per_s = rate / wl.n_layers
    return {"value": tokens_per_s, "unit": "tokens/s", "cores": n_workers, "kind": "oracle",
            "sample": (f"{n_workers} (layer, sequence) pairs of {wl.n_layers * wl.batch}, steady-state "
                       f"cycles of {wl.interval} steps + 1 compression, {total_steps} pair-steps in "
                       f"~{seconds:.0f} s per worker, one thread each; scaled by 1/n_layers")}


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
    }


def read_traffic(workload: str):
    """HBM bytes per attend launch from the committed rocprofv3 --pmc summary, if present."""
    path = os.path.join(ROOT, "profiles", f"attend_{workload}_pmc.txt")
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    return float(line.split(":")[1])
    except OSError:
        pass
    return None


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
    ap.add_argument("--no-full-launch", action="store_true",
                    help="skip the extra pass that times the attend kernel launched once for all layers")
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

    from gkv_traces import CONFIGS, Trace
    wl = CONFIGS[args.workload]
    if args.combine is not None:
        wl = wl.with_(combine=args.combine)
    if args.alpha is not None:
        wl = wl.with_(alpha=args.alpha)

    # CPU leg first, before this process touches the GPU (children are plain CPU processes)
    cpu = None
    if not args.no_cpu_baseline and not args.copy_calibration and args.redundancy is None:
        cpu = cpu_baseline(args.workload, args.cpu_seconds, wl.combine, wl.alpha)

    import torch
    from paper_2512_00504_amd.state import DecodeState
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
    K = max(s, (args.steps + s - 1) // s * s)            # whole compression cycles
    W = max(s, (args.warmup + s - 1) // s * s)
    preroll = b                                          # tokens placed in the cache before step b
    params = {}
    if args.splits:
        params["attend_splits"] = args.splits
    if args.tile:
        params["attend_tile"] = args.tile
    for item in args.param:
        name, val = item.split("=")
        params[name] = int(val)
    # The layers are split into NS groups, each with its own context, buffers and HIP stream.
    # Every decode step launches every group; units are independent, so the groups' kernels may
    # overlap and one group's kernel boundary (launch, first-load latency, final stores) is
    # covered by the other group's streaming.  NS = 1 is the plain one-launch-per-step form.
    NS = max(1, min(args.streams, wl.n_layers))
    bounds = [wl.n_layers * g // NS for g in range(NS + 1)]          # as even as possible
    Lgs = [bounds[g + 1] - bounds[g] for g in range(NS)]
    Lg = max(Lgs)
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
    assert s % wl.window == 0

    def split_layers(x):
        """[n, L, ...] numpy -> per-group contiguous device tensors [n, layers of the group, ...]."""
        return [torch.from_numpy(x[:, bounds[g]:bounds[g + 1]]).to(dt).to(dev).contiguous() for g in range(NS)]

    def upload(t0, n):
        q, k, v = tr.batch_steps(t0, n, workers=8)
        return list(zip(split_layers(q), split_layers(k), split_layers(v)))

    def run(chunk, t0, n, stream_of):
        """n decode steps starting at absolute step t0 on pre-uploaded inputs; raw C calls."""
        len_host = host["len"]
        addr = [(qd.data_ptr(), qd.stride(0) * esz, kd.data_ptr(), kd.stride(0) * esz, vd.data_ptr(), vd.stride(0) * esz)
                for (qd, kd, vd) in chunk]
        w = wl.window
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

    own_streams = [ctypes.c_void_p(st_.cuda_stream) for st_ in streams]
    one_stream = [own_streams[0]] * NS

    # The first b tokens are placed in the cache directly: no compression happens before the
    # cache exceeds the budget, so this is the state b decode steps leave behind, and every
    # attend launch of this process then runs at a steady-state length b+1 .. b+s.
    if args.fast_prefix:
        _, k0, v0 = tr.batch_steps(0, s, workers=8)
        reps = (b + s - 1) // s
        k0s = [x.repeat(reps, 1, 1, 1, 1)[:b] for x in split_layers(k0)]
        v0s = [x.repeat(reps, 1, 1, 1, 1)[:b] for x in split_layers(v0)]
    else:
        _, k0, v0 = tr.batch_steps(0, b, workers=8)
        k0s, v0s = split_layers(k0), split_layers(v0)
    for g, st in enumerate(groups):
        st.load_prefix(k0s[g], v0s[g])
    del k0, v0, k0s, v0s
    host["len"] = b
    torch.cuda.synchronize()
    t_abs = b
    assert b % s == 0 and W >= s, "warm-up must cover one whole compression cycle"
    for c0 in range(0, W, s):                             # untimed warm-up cycles (first compression)
        chunk = upload(t_abs, s)
        torch.cuda.synchronize()
        run(chunk, t_abs, s, own_streams)
        t_abs += s
    torch.cuda.synchronize()
    for st in groups:
        lens = st.lengths(t_abs)
        assert int(lens.max()) == b and int(lens.min()) == b

    chunks = [upload(t_abs + c0, s) for c0 in range(0, K, s)]     # all timed inputs resident in HBM
    torch.cuda.synchronize()
    t_wall = time.perf_counter()
    for ci, chunk in enumerate(chunks):
        run(chunk, t_abs + ci * s, s, own_streams)
    torch.cuda.synchronize()
    elapsed = wall_s = time.perf_counter() - t_wall
    gpu_s = None
    t_abs += K

    # per-kernel durations: the same steps again with every launch bracketed by its own HIP events,
    # all groups on ONE stream so that a launch's duration is the kernel's own (no overlap)
    for st in groups:
        st.ctx.profile_reset()
        st.ctx.profile_enable(True)
    for ci, chunk in enumerate(chunks):
        run(chunk, t_abs + ci * s, s, one_stream)
    torch.cuda.synchronize()
    per_kernel = {}
    for name in ("attend", "score", "global", "topk", "compact") + (("redundancy",) if args.redundancy else ()):
        ms = n = 0
        for st in groups:
            st.ctx.profile_enable(False)
            m_, n_ = st.ctx.profile_read(name)
            ms += m_; n += n_
        per_kernel[name] = {"launches": n, "avg_us": (1e3 * ms / n) if n else None}
    st = groups[0]

    # The same kernel launched once for all layers (one context, one stream): its duration at the
    # full 28-layer shape, for comparison with the per-group launches above.  The cache contents
    # are the groups' current ones, the inputs the timed chunks.
    full = None
    if NS > 1 and not args.no_full_launch:
        fs = DecodeState.from_workload(wl, device=dev, params=params)
        for name in ("K", "V", "pos", "F_hist"):
            getattr(fs, name).copy_(torch.cat([getattr(g_, name) for g_ in groups], dim=0))
        fs.qwin.copy_(torch.cat([g_.qwin for g_ in groups], dim=1))
        fs.d_state.copy_(torch.cat([g_.d_state for g_ in groups], dim=0))
        fs.len_host = host["len"]
        fs.ctx.profile_enable(True)
        t_f = t_abs + K
        for ci, chunk in enumerate(chunks[:4]):
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
        full = {"launches": n, "avg_launch_us": us, "algorithmic_bytes_per_launch": algorithmic_bytes(wl)["attend"],
                "achieved": algorithmic_bytes(wl)["attend"] / (us * 1e-6) / 1e9,
                "frac": algorithmic_bytes(wl)["attend"] / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, "unit": "GB/s"}
        del fs

    # read bandwidth a trivial streaming kernel sustains on this GPU, for context: over a buffer
    # far larger than any cache, and over one the size of this workload's K+V cache
    from paper_2512_00504_amd.binding import probe_stream_read
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    ceilings = {}
    for label, nbytes in (("4GiB", 4 << 30), ("kv_cache_size", int(st.K.numel() * st.K.element_size() * 2 * NS))):
        buf = torch.empty(nbytes // 16 * 16, dtype=torch.uint8, device=dev).fill_(3)
        for _ in range(3):
            probe_stream_read(buf, sink)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 10
        e0.record()
        for _ in range(reps):
            probe_stream_read(buf, sink)
        e1.record()
        torch.cuda.synchronize()
        ceilings[label] = {"bytes": buf.numel(), "GBps": buf.numel() * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9}
        del buf

    alg = algorithmic_bytes(wl)                       # whole batch, all layers
    att_us = per_kernel["attend"]["avg_us"]           # one launch = one group = n_layers / NS layers
    achieved = alg["attend"] / NS / (att_us * 1e-6) / 1e9
    alg["redundancy"] = wl.n_units * ((2 if wl.dtype == "bf16" else 4) * wl.head_dim * (b + s) + 12 * (b + s))
    for name in per_kernel:
        us = per_kernel[name]["avg_us"]
        per_kernel[name]["algorithmic_MB"] = alg[name] / NS / 1e6
        per_kernel[name]["GBps"] = (alg[name] / NS / (us * 1e-6) / 1e9) if us else None
        per_kernel[name]["hbm_frac"] = (per_kernel[name]["GBps"] / HBM_PEAK_GBS) if us else None
    bytes_per_step = alg["attend"] + (alg["score"] + alg["global"] + alg["topk"] + alg["compact"]) / s
    tokens_per_s = wl.batch * K / elapsed
    out = {
        "metric": "decode tokens/sec through attend+score+evict at budget 512; % HBM roofline"
                  if b == 512 else f"decode tokens/sec through attend+score+evict at budget {b}",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": 1e3 * elapsed / K, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "n_layers": wl.n_layers, "batch": wl.batch,
                   "n_q_heads": wl.n_q_heads, "n_kv_heads": wl.n_kv_heads, "head_dim": wl.head_dim,
                   "budget": b, "window": wl.window, "interval": s, "alpha": wl.alpha,
                   "combine": wl.combine, "trace": wl.recipe, "preroll_steps": preroll,
                   "attend_splits": args.splits, "attend_tile": args.tile, "params": params, "fast_prefix": args.fast_prefix,
                   "streams": NS, "layers_per_launch": Lg,
                   "redundancy": args.redundancy, "ring": "in place" if args.ring_in_place else "copy"},
        "roofline": {"bound": "hbm", "kernel": "attend_mfma_kernel" if wl.dtype == "bf16" and wl.head_dim == 128 else "attend_generic_kernel",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": read_traffic(wl.name),
                     "algorithmic_bytes_per_launch": alg["attend"] / NS, "avg_launch_us": att_us,
                     "launches_per_step": NS,
                     "note": "launch durations from HIP events with the launches serialised on one stream; "
                             "the timed region overlaps the groups' launches on separate streams"},
        "roofline_all_layers_one_launch": full,
        "cpu_baseline": cpu,
        "whole_step": {"algorithmic_bytes_per_step": bytes_per_step,
                       "GBps": bytes_per_step * K / elapsed / 1e9,
                       "hbm_frac": bytes_per_step * K / elapsed / 1e9 / HBM_PEAK_GBS,
                       "gpu_seconds": gpu_s, "wall_seconds": wall_s},
        "per_kernel": per_kernel,
        "stream_read_ceiling": ceilings,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
