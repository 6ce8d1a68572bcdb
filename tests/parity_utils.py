"""Helpers for the GPU-vs-oracle parity tests: drive both sides with the same
seeded trace, compare every step's output and every compression event's
intermediates, and apply the tolerated-swap rule to kept sets."""
from __future__ import annotations

import numpy as np
import torch

from gkv_traces import Trace
from oracle import gkv_oracle as O
from paper_2512_00504_amd.state import DecodeState, k_cache_to_rows, k_rows_to_cache

TORCH_DT = {"f32": torch.float32, "bf16": torch.bfloat16}
# output tolerance: 1e-5 relative (to the row's largest magnitude) for fp32, 2e-2 absolute for bf16
OUT_TOL = {"f32": ("rel", 1e-5), "bf16": ("abs", 2e-2)}
SWAP_REL = 1e-6          # kept sets may differ only between scores closer than this (relative)
SWAP_TINY = 1e-30        # ... or both below anything fp32 softmax can resolve
SCORE_REL = 1e-5         # fp32 score arithmetic on exact inputs vs fp64 (measured worst: 1.9e-6)


def make_oracle(wl, **kw):
    args = dict(capacity=wl.capacity, alpha=wl.alpha, form=wl.combine)
    args.update(kw)
    return O.OracleA(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.budget, wl.window, wl.interval, **args)


def check_output(out_gpu, out_ref, dtype, what=""):
    """out_gpu, out_ref: [h_q, d] float64 arrays."""
    kind, tol = OUT_TOL[dtype]
    err = np.abs(out_gpu - out_ref)
    if kind == "rel":
        bound = tol * np.abs(out_ref).max(axis=-1, keepdims=True) + 1e-30
    else:
        bound = tol
    assert (err <= bound).all(), f"{what}: max err {err.max():.3e} (tol {kind} {tol})"
    return float(err.max())


def check_scores(s_gpu, s_ref, what=""):
    """Elementwise fp32-vs-fp64 score comparison; values too small for fp32 are exempt."""
    s_gpu = np.asarray(s_gpu, np.float64)
    err = np.abs(s_gpu - s_ref)
    bound = SCORE_REL * np.abs(s_ref) + 1e-30
    bad = err > bound
    assert not bad.any(), (f"{what}: {bad.sum()} score mismatches, worst rel "
                           f"{(err / (np.abs(s_ref) + 1e-300)).max():.3e}")


def check_keep(keep_gpu, keep_ref, F_ref, what="", abs_tol=None):
    """Kept index sets must be identical, except swaps between candidates whose oracle scores
    differ by less than SWAP_REL relative (or are both below SWAP_TINY).  Returns #swapped."""
    keep_gpu = np.asarray(keep_gpu, np.int64)
    assert keep_gpu.shape == keep_ref.shape, what
    assert (np.diff(keep_gpu) > 0).all(), f"{what}: kept indices not strictly ascending"
    assert keep_gpu.min() >= 0 and keep_gpu.max() < F_ref.shape[0], f"{what}: index out of range"
    if np.array_equal(keep_gpu, keep_ref):
        return 0
    only_gpu = np.setdiff1d(keep_gpu, keep_ref)
    only_ref = np.setdiff1d(keep_ref, keep_gpu)
    vals = np.concatenate([F_ref[only_gpu], F_ref[only_ref]])
    hi, lo = vals.max(), vals.min()
    if abs_tol is not None:
        ok = (hi - lo) <= abs_tol
    else:
        ok = (hi - lo) <= SWAP_REL * hi or hi < SWAP_TINY
    assert ok, (f"{what}: kept sets differ beyond tolerance: gpu-only {only_gpu.tolist()} "
                f"ref-only {only_ref.tolist()} scores {vals.tolist()}")
    return len(only_gpu)


def upload_oracle_state(st: DecodeState, orc, l, b, next_step):
    """Overwrite the GPU state of (layer l, sequence b) with the oracle's (teacher forcing);
    `next_step` is the index of the decode step that comes next."""
    dt = st.K.dtype
    dev = st.device
    n_tiled = int(st.d_state[l, b, 3])
    st.K[l, b] = k_rows_to_cache(torch.from_numpy(orc.K).to(dt), n_tiled).to(dev)
    st.V[l, b] = torch.from_numpy(orc.V).to(dt).to(dev)
    st.pos[l, b] = torch.from_numpy(orc.pos).to(torch.int32).to(dev)
    st.F_hist[l, b] = torch.from_numpy(orc.F_hist).to(torch.float32).to(dev)
    st.d_state[l, b] = torch.tensor([orc.len, next_step, orc.n_hist, n_tiled], dtype=torch.int32)


RED_MARGIN = 4e-7        # the oracle thresholds an fp32 cosine like the kernel's; closer than this may still differ
RED_SWAP_ABS = 2e-6      # combined scores are O(1) and can be negative: absolute swap tolerance


def run_parity(wl, n_steps, pairs=None, params=None, chunk=128, check_state_every_event=True,
               cfg_over=None, fused_evict=False, redundancy=None):
    """Run GPU (all units) and oracle (the (layer, seq) `pairs`, default all) side by side.
    Returns a dict of statistics.  Asserts parity at every step and event."""
    tr = Trace(wl)
    st = DecodeState.from_workload(wl, params=params, **(cfg_over or {}))
    if pairs is None:
        pairs = [(l, b) for l in range(wl.n_layers) for b in range(wl.batch)]
    if redundancy is not None:
        redundancy = dict(redundancy, fp32_decisions=True)
    orcs = {p: make_oracle(wl, redundancy=redundancy) for p in pairs}
    dt = TORCH_DT[wl.dtype]
    dev = st.device
    stats = dict(events=0, swaps=0, max_out_err=0.0, steps=n_steps, ambiguous=0)
    hkv = wl.n_kv_heads
    for t0 in range(0, n_steps, chunk):
        n = min(chunk, n_steps - t0)
        q, k, v = tr.batch_steps(t0, n, workers=8)
        qd = torch.from_numpy(q).to(dt).to(dev)
        kd = torch.from_numpy(k).to(dt).to(dev)
        vd = torch.from_numpy(v).to(dt).to(dev)
        outs = []
        for i in range(n):
            t = t0 + i
            out = st.attend_decode(qd[i], kd[i], vd[i], t)
            outs.append(out.clone())
            ev_gpu = None
            if st.is_trigger(t):
                if redundancy is not None:
                    st.score_window(t); st.global_update(t)
                    st.redundancy_combine(t, redundancy["lam"], redundancy["tau"], redundancy["n_recent"],
                                          redundancy.get("eps", 1e-8))
                    st.select_topk(t, on_combined=True); st.compact(t)
                elif fused_evict:
                    st.evict(t)
                else:
                    st.score_window(t); st.global_update(t); st.select_topk(t)
                    st.evicted_positions(t); st.compact(t)
                ev_gpu = dict(S=st.S.cpu().numpy(), F=st.F.cpu().numpy(), keep=st.keep_idx.cpu().numpy(),
                              R=st.R.cpu().numpy(), Fsel=st.F_sel.cpu().numpy(),
                              evicted=st.evicted.cpu().numpy())
            for (l, b), orc in orcs.items():
                n_ev = len(orc.events)
                ref = orc.step(t, q[i, l, b], k[i, l, b], v[i, l, b])
                outs_ref = ref
                og = outs[-1][l, b].double().cpu().numpy() if (ev_gpu is not None or i == n - 1 or t % 7 == 0) else None
                if og is not None:
                    e = check_output(og, outs_ref, wl.dtype, f"out t={t} pair=({l},{b})")
                    stats["max_out_err"] = max(stats["max_out_err"], e)
                if len(orc.events) > n_ev:
                    assert ev_gpu is not None, f"oracle compressed at t={t} but the GPU host trigger did not"
                    ev = orc.events[-1]
                    c = ev["len"] - wl.window
                    swapped = 0
                    for j in range(hkv):
                        what = f"t={t} pair=({l},{b}) head={j}"
                        check_scores(ev_gpu["S"][l, b, j, :c], ev["S"][j], "S " + what)
                        check_scores(ev_gpu["F"][l, b, j, :c], ev["F"][j], "F " + what)
                        if redundancy is None:
                            swapped += check_keep(ev_gpu["keep"][l, b, j], ev["keep"][j], ev["F"][j], "keep " + what)
                        elif ev["tau_margin"][j] < RED_MARGIN:
                            stats["ambiguous"] += 1              # threshold decision not robust: skip, resync
                            swapped += 1
                        else:
                            Rn = ev["R"][j] / ev["R"][j].max()
                            np.testing.assert_allclose(ev_gpu["R"][l, b, j, :ev["len"]], Rn, rtol=2e-5, atol=1e-30,
                                                       err_msg="R " + what)
                            np.testing.assert_allclose(ev_gpu["Fsel"][l, b, j, :c], ev["Fsel"][j], rtol=0, atol=1e-5,
                                                       err_msg="Fsel " + what)
                            swapped += check_keep(ev_gpu["keep"][l, b, j], ev["keep"][j], ev["Fsel"][j],
                                                  "keep " + what, abs_tol=RED_SWAP_ABS)
                    if not swapped and redundancy is None and not fused_evict:
                        for j in range(hkv):                 # eviction log: bit-exact when the kept sets agree
                            log = ev_gpu["evicted"][l, b, j]
                            n_ev_rows = len(ev["evicted_pos"][j])
                            assert log[:n_ev_rows].tolist() == ev["evicted_pos"][j], f"eviction log t={t} ({l},{b},{j})"
                            assert (log[n_ev_rows:] == -1).all()
                    stats["swaps"] += swapped
                    if swapped:
                        upload_oracle_state(st, orc, l, b, t + 1)
                    elif check_state_every_event:
                        check_state(st, orc, l, b, t + 1, f"state t={t} pair=({l},{b})")
                elif ev_gpu is not None:
                    raise AssertionError(f"GPU host trigger fired at t={t} but the oracle did not compress")
            if ev_gpu is not None:
                stats["events"] += 1
    for (l, b), orc in orcs.items():
        check_state(st, orc, l, b, n_steps, f"final state pair=({l},{b})")
    stats["state"] = st
    stats["oracles"] = orcs
    return stats


def check_state(st: DecodeState, orc, l, b, next_step, what=""):
    """Cache contents: length, positions, K, V bit-exact; F_hist to fp32 accuracy."""
    n = orc.len
    rec = st.d_state[l, b].cpu().tolist()
    got = rec[0] + (next_step - rec[1])
    assert got == n, f"{what}: len {got} != {n}"
    assert rec[2] == orc.n_hist, what
    np.testing.assert_array_equal(st.pos[l, b, :, :n].cpu().numpy(), orc.pos[:, :n], err_msg=what)
    Kg = k_cache_to_rows(st.K[l, b], rec[3])[:, :n].double().cpu().numpy()
    Vg = st.V[l, b, :, :n].double().cpu().numpy()
    np.testing.assert_array_equal(Kg, orc.K[:, :n], err_msg=what + " K")
    np.testing.assert_array_equal(Vg, orc.V[:, :n], err_msg=what + " V")
    nh = orc.n_hist
    check_scores(st.F_hist[l, b, :, :nh].cpu().numpy(), orc.F_hist[:, :nh], what + " F_hist")
