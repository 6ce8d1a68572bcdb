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

# Redundancy score.  The threshold turns each cosine into a yes/no.  The GPU forms a cosine as
# (fp32 dot product of exact products) x (two fp64 reciprocal norms), so it can differ from the fp64
# cosine by the dot product's rounding only, a few 1e-7 relative.  An entry whose fp64 cosine lies
# within RED_MARGIN of tau may therefore legitimately fall on either side.  Nothing is skipped for
# it: each such entry moves its column sum by about tau, i.e. R' by a factor e^tau, so the checker
# reads off R' which of them the GPU counted, builds the column sums with exactly those entries
# from the oracle's own cosines, and then compares R', the combined score and the kept set in full.
RED_MARGIN = 1e-6
RED_REL = 1e-5           # R' = exp(col - max col): same bar as the other fp32 scores
RED_SWAP_ABS = 2e-6      # combined scores are O(1) and can be negative: absolute swap tolerance


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


def check_scores(s_gpu, s_ref, what="", rel=SCORE_REL):
    """Elementwise fp32-vs-fp64 score comparison; values too small for fp32 are exempt."""
    s_gpu = np.asarray(s_gpu, np.float64)
    err = np.abs(s_gpu - s_ref)
    bound = rel * np.abs(s_ref) + 1e-30
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


def check_redundancy_head(ev, j, R_gpu, Fsel_gpu, keep_gpu, red, w, k, what=""):
    """One KV head of a compression with the redundancy term, against the fp64 oracle event `ev`.
    R_gpu [>=l] is the GPU's R / max R, Fsel_gpu [>=c] its combined score, keep_gpu [k] its kept set.
    Returns (entries within RED_MARGIN of tau, how many of those the GPU decided the other way,
    swapped rows, whether the GPU's legitimate kept set differs from the oracle's own)."""
    l = ev["len"]
    c = l - w
    tau, lam, n_recent = red["tau"], red["lam"], red["n_recent"]
    C, col = ev["C"][j], ev["col"][j]
    amb = np.abs(C - tau) < RED_MARGIN
    np.fill_diagonal(amb, False)
    if n_recent > 0:
        amb[:, l - n_recent:] = False
    rows, cols = np.nonzero(amb)
    col_gpu = col.copy()
    flipped = 0
    if len(rows):
        logR = np.log(np.maximum(np.asarray(R_gpu[:l], np.float64), 1e-300))
        clean = np.ones(l, bool); clean[cols] = False
        assert clean.any(), what
        # max col as the GPU saw it, from the untouched column with the largest sum
        ref_col = int(np.flatnonzero(clean)[np.argmax(col[clean])])
        assert R_gpu[ref_col] > 0, what
        colmax_gpu = col[ref_col] - logR[ref_col]
        for jj in np.unique(cols):
            ks = rows[cols == jj]
            assert len(ks) <= 8, f"{what}: {len(ks)} entries of column {jj} on the threshold"
            vals = C[ks, jj]
            base = col[jj] - vals[vals >= tau].sum()           # column sum without any of them
            if R_gpu[jj] <= 0:                                 # below fp32 range either way
                continue
            cands = base + np.concatenate([[0.0], np.cumsum(vals)])     # entries all equal tau to 1e-6
            # matched as R' values: the GPU's R' is an fp32 number and may be subnormal, where its
            # logarithm no longer resolves 1e-3 (readings that give the same fp32 value cannot be
            # told apart, and need not be: R' is what the path uses)
            R_cands = np.exp(cands - colmax_gpu)
            miss = np.abs(R_cands - float(R_gpu[jj]))
            m = int(np.argmin(miss))
            assert miss[m] <= 1e-3 * R_cands[m] + 3e-45, \
                f"{what}: column {jj}: R' = {R_gpu[jj]} matches no reading {R_cands} (sums {cands})"
            col_gpu[jj] = cands[m]
            flipped += abs(m - int((vals >= tau).sum()))
    R_alt = O.softmax(col_gpu)
    Rn = R_alt / R_alt.max()
    check_scores(R_gpu[:l], Rn, "R' " + what, rel=RED_REL)
    Fsel = O.combine_redundancy(ev["F"][j][None], R_alt[None], lam, n_cand=c)
    np.testing.assert_allclose(Fsel_gpu[:c], Fsel[0], rtol=0, atol=1e-5, err_msg="Fsel " + what)
    keep_alt = O.select_topk(Fsel, k)[0]
    swapped = check_keep(keep_gpu, keep_alt, Fsel[0], "keep " + what, abs_tol=RED_SWAP_ABS)
    return len(rows), flipped, swapped, not np.array_equal(keep_alt, ev["keep"][j])


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


def run_parity(wl, n_steps, pairs=None, params=None, chunk=128, check_state_every_event=True,
               cfg_over=None, fused_evict=False, redundancy=None, prompts=None, workers=8, say=None):
    """Run GPU (all units) and oracle (the (layer, seq) `pairs`, default all) side by side for
    n_steps decode steps.  `prompts`: per-sequence prompt lengths P_i; the prompt of sequence i is
    the trace positions [t0 - P_i, t0) with t0 = max P_i, placed in the cache without decoding, and
    decoding starts at step t0 for every sequence.  Returns a dict of statistics.  Asserts parity at
    every step (outputs) and every event (scores, kept sets, eviction log, cache contents).
    `say`: optional print function, called once per chunk of steps (long runs show progress)."""
    tr = Trace(wl)
    st = DecodeState.from_workload(wl, params=params, **(cfg_over or {}))
    if pairs is None:
        pairs = [(l, b) for l in range(wl.n_layers) for b in range(wl.batch)]
    if redundancy is not None:     # both sides take the very same parameter values: the fp32 ones
        redundancy = dict(redundancy, lam=float(np.float32(redundancy["lam"])), tau=float(np.float32(redundancy["tau"])),
                          eps=float(np.float32(redundancy.get("eps", 1e-8))))
    cap = (cfg_over or {}).get("capacity", wl.capacity)
    orcs = {p: make_oracle(wl, redundancy=redundancy, capacity=cap) for p in pairs}
    dt = TORCH_DT[wl.dtype]
    dev = st.device
    li = torch.tensor([p[0] for p in pairs], device=dev)
    bi = torch.tensor([p[1] for p in pairs], device=dev)
    stats = dict(events=0, pair_events=0, swaps=0, resyncs=0, max_out_err=0.0, steps=n_steps,
                 ambiguous=0, flipped=0)
    hkv, w, kk = wl.n_kv_heads, wl.window, wl.budget - wl.window

    t0 = 0
    if prompts is not None:
        assert len(prompts) == wl.batch
        t0 = max(prompts)
        for c0 in range(0, t0, chunk):
            n = min(chunk, t0 - c0)
            _, k, v = tr.batch_steps(c0, n, workers=workers, need_q=False)
            st.load_prompt_rows(c0, torch.from_numpy(k).to(dev), torch.from_numpy(v).to(dev), t0, prompts)
            if say:
                say(f"    prompt rows {c0}..{c0 + n - 1} placed")
            for (l, b), orc in orcs.items():
                lo = max(c0, t0 - prompts[b])
                if lo < c0 + n:
                    orc.prefill(lo, k[lo - c0:, l, b], v[lo - c0:, l, b])
        st.begin_decode(t0, prompts)

    for c0 in range(t0, t0 + n_steps, chunk):
        n = min(chunk, t0 + n_steps - c0)
        q, k, v = tr.batch_steps(c0, n, workers=workers)
        qd = torch.from_numpy(q).to(dt).to(dev)
        kd = torch.from_numpy(k).to(dt).to(dev)
        vd = torch.from_numpy(v).to(dt).to(dev)
        for i in range(n):
            t = c0 + i
            out = st.attend_decode(qd[i], kd[i], vd[i], t)
            og_all = out[li, bi].double().cpu().numpy()               # the sampled pairs, every step
            ev_gpu = None
            if st.is_trigger(t):
                if redundancy is not None:
                    st.score_window(t); st.global_update(t)
                    st.redundancy_combine(t, redundancy["lam"], redundancy["tau"], redundancy["n_recent"],
                                          redundancy["eps"])
                    st.select_topk(t, on_combined=True); st.compact(t)
                elif fused_evict:
                    st.evict(t)
                else:
                    st.score_window(t); st.global_update(t); st.select_topk(t)
                    st.evicted_positions(t); st.compact(t)
                pick = lambda x: x[li, bi].cpu().numpy()
                ev_gpu = dict(S=pick(st.S), F=pick(st.F), keep=pick(st.keep_idx), R=pick(st.R),
                              Fsel=pick(st.F_sel), evicted=pick(st.evicted), lens=pick(st.lengths(t + 1)))
                stats["events"] += 1
            for pi, ((l, b), orc) in enumerate(orcs.items()):
                n_ev = len(orc.events)
                ref = orc.step(t, q[i, l, b], k[i, l, b], v[i, l, b])
                e = check_output(og_all[pi], ref, wl.dtype, f"out t={t} pair=({l},{b})")
                stats["max_out_err"] = max(stats["max_out_err"], e)
                if len(orc.events) == n_ev:
                    if ev_gpu is not None:      # a ragged batch: this sequence must have been left alone
                        assert ev_gpu["lens"][pi] == orc.len, f"t={t} pair=({l},{b}): GPU compressed, oracle did not"
                    continue
                assert ev_gpu is not None, f"oracle compressed at t={t} but the GPU host trigger did not"
                stats["pair_events"] += 1
                ev = orc.events[-1]
                c = ev["len"] - w
                swapped, resync = 0, False
                for j in range(hkv):
                    what = f"t={t} pair=({l},{b}) head={j}"
                    check_scores(ev_gpu["S"][pi, j, :c], ev["S"][j], "S " + what)
                    check_scores(ev_gpu["F"][pi, j, :c], ev["F"][j], "F " + what)
                    if redundancy is None:
                        swapped += check_keep(ev_gpu["keep"][pi, j], ev["keep"][j], ev["F"][j], "keep " + what)
                    else:
                        n_amb, n_flip, n_swap, differs = check_redundancy_head(
                            ev, j, ev_gpu["R"][pi, j], ev_gpu["Fsel"][pi, j], ev_gpu["keep"][pi, j],
                            redundancy, w, kk, what)
                        stats["ambiguous"] += n_amb; stats["flipped"] += n_flip
                        swapped += n_swap
                        resync |= differs
                ev.pop("C", None)                          # [h_kv, l, l] per event: do not keep them all
                if not swapped and redundancy is None and not fused_evict:
                    for j in range(hkv):                   # eviction log: bit-exact when the kept sets agree
                        log = ev_gpu["evicted"][pi, j]
                        n_ev_rows = len(ev["evicted_pos"][j])
                        assert log[:n_ev_rows].tolist() == ev["evicted_pos"][j], f"eviction log t={t} ({l},{b},{j})"
                        assert (log[n_ev_rows:] == -1).all()
                stats["swaps"] += swapped
                if swapped or resync:
                    stats["resyncs"] += 1
                    upload_oracle_state(st, orc, l, b, t + 1)
                elif check_state_every_event:
                    check_state(st, orc, l, b, t + 1, f"state t={t} pair=({l},{b})")
            if say and i == n - 1:
                say(f"    steps {c0}..{t} checked, {stats['pair_events']} pair-events so far")
    for (l, b), orc in orcs.items():
        check_state(st, orc, l, b, t0 + n_steps, f"final state pair=({l},{b})")
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
