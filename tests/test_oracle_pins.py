"""Pins for the fp64 oracle: closed forms, hand-derived fixtures, library
routines on special cases, brute force on tiny inputs, and the invariants the
method fixes.  CPU only."""
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy.special import softmax as sp_softmax

from gkv_traces import CONFIGS, Trace
from oracle import gkv_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, val = line.split(":")
            out[key.strip()] = float(Fraction(val.strip()))
    return out


# ---------------------------------------------------------------- attend ----
def test_attend_uniform_keys_gives_mean_of_values():
    rng = np.random.default_rng(1)
    h_q, h_kv, d, l = 4, 2, 8, 11
    K = np.tile(rng.standard_normal((h_kv, 1, d)), (1, l + 3, 1))
    V = rng.standard_normal((h_kv, l + 3, d))
    q = rng.standard_normal((h_q, d))
    o = O.attend(q, K, V, l)
    for i in range(h_q):
        np.testing.assert_allclose(o[i], V[i // 2, :l].mean(axis=0), rtol=1e-13, atol=1e-14)


def test_attend_identity_values_returns_library_softmax():
    # V = I makes the output the probability vector itself; compare with scipy's softmax.
    rng = np.random.default_rng(2)
    h_q, h_kv, d, l = 6, 3, 16, 16
    K = rng.standard_normal((h_kv, l, d)) * 3
    V = np.tile(np.eye(l, d)[None], (h_kv, 1, 1))
    q = rng.standard_normal((h_q, d))
    o = O.attend(q, K, V, l)
    for i in range(h_q):
        ref = sp_softmax(K[i // 2] @ q[i] / np.sqrt(d))
        np.testing.assert_allclose(o[i], ref, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(o.sum(axis=1), 1.0, rtol=1e-13)


def test_attend_head_to_group_map_is_contiguous():
    # head i must read KV head i // g: make KV head 1's values all 7, head 0's all 3.
    h_q, h_kv, d, l = 4, 2, 4, 5
    K = np.zeros((h_kv, l, d)); V = np.zeros((h_kv, l, d))
    V[0] = 3.0; V[1] = 7.0
    o = O.attend(np.ones((h_q, d)), K, V, l)
    np.testing.assert_allclose(o[:2], 3.0); np.testing.assert_allclose(o[2:], 7.0)


def test_attend_ignores_rows_beyond_length_and_uses_scale():
    rng = np.random.default_rng(3)
    K = rng.standard_normal((1, 9, 4)); V = rng.standard_normal((1, 9, 4)); q = rng.standard_normal((1, 4))
    a = O.attend(q, K, V, 6)
    K2, V2 = K.copy(), V.copy(); K2[:, 6:] = 99; V2[:, 6:] = -99
    np.testing.assert_array_equal(a, O.attend(q, K2, V2, 6))
    ref = sp_softmax(K[0, :6] @ q[0] * 0.25) @ V[0, :6]
    np.testing.assert_allclose(O.attend(q, K, V, 6, scale=0.25)[0], ref, rtol=1e-12)


# ----------------------------------------------------------- local score ----
def test_local_and_global_score_hand_fixture():
    gold = _read_golden("local_score_hand.txt")
    K = np.log(np.array([1.0, 2.0, 3.0, 4.0])).reshape(1, 4, 1)
    Qwin = np.array([[[1.0], [1.0]], [[-1.0], [-1.0]]])          # [h_q=2, w=2, d=1]
    A = O.window_probs(Qwin, K, 4)
    S = O.local_score(A, 1)
    for n in range(4):
        assert S[0, n] == pytest.approx(gold[f"S {n}"], rel=1e-14)
    F_hist = np.array([[0.5, 0.9]])
    for form in ("max", "avg", "sum"):
        F = O.global_score(S, F_hist, 2, 0.8, form, n_cand=2)
        for n in range(2):
            assert F[0, n] == pytest.approx(gold[f"F_{form} {n}"], rel=1e-14)
    Sn = O.global_score(S, None, 0, 0.8, "max", n_cand=2)
    assert Sn[0, 0] == pytest.approx(gold["Sn 0"]) and Sn[0, 1] == pytest.approx(gold["Sn 1"], rel=1e-14)
    S_nomask = O.local_score(O.window_probs(Qwin, K, 4, causal_window=False), 1)
    assert S_nomask[0, 0] == pytest.approx(gold["S_nomask 0"], rel=1e-14)


def test_local_score_closed_form_equal_keys():
    # All keys equal (or Q = 0): every visible entry gets 1/(number visible), so a candidate's
    # score is (1/w) * sum_k 1/(l-w+k+1) under the causal reading and 1/l without the mask.
    h_q, h_kv, d, w, l = 6, 2, 8, 5, 23
    K = np.ones((h_kv, l, d)); Qwin = np.random.default_rng(4).standard_normal((h_q, w, d))
    S = O.local_score(O.window_probs(Qwin, K, l), h_kv)
    c = l - w
    expect = sum(1.0 / (c + k + 1) for k in range(w)) / w
    np.testing.assert_allclose(S[:, :c], expect, rtol=1e-13)
    S2 = O.local_score(O.window_probs(Qwin, K, l, causal_window=False), h_kv)
    np.testing.assert_allclose(S2, 1.0 / l, rtol=1e-13)
    # window entry c+m is visible to rows k >= m only
    for m in range(w):
        np.testing.assert_allclose(S[:, c + m], sum(1.0 / (c + k + 1) for k in range(m, w)) / w, rtol=1e-13)


def test_local_score_single_head_single_row_is_decode_probability():
    # g = 1, w = 1: S is the attention distribution of the last query, i.e. what attend()
    # uses; read it out of attend() with identity values.
    rng = np.random.default_rng(5)
    h, d, l = 3, 16, 12
    K = rng.standard_normal((h, l, d)) * 2; q = rng.standard_normal((h, d))
    S = O.local_score(O.window_probs(q[:, None, :], K, l), h)
    V = np.tile(np.eye(l, d)[None], (h, 1, 1))
    np.testing.assert_allclose(S, O.attend(q, K, V, l)[:, :l], rtol=1e-12, atol=1e-16)


def test_local_score_bounds_and_brute_force():
    rng = np.random.default_rng(6)
    h_q, h_kv, d, w, l = 6, 2, 4, 3, 9
    g = h_q // h_kv
    K = rng.standard_normal((h_kv, l, d)); Qwin = rng.standard_normal((h_q, w, d))
    A = O.window_probs(Qwin, K, l)
    np.testing.assert_allclose(A.sum(axis=2), 1.0, rtol=1e-13)
    S = O.local_score(A, h_kv)
    assert (S >= 0).all()
    tot = S.sum(axis=1) * w          # sum over rows of sum_n max_i A  in [1, g] per row
    assert ((tot >= w - 1e-12) & (tot <= g * w + 1e-12)).all()
    # scalar loops, written independently with math.exp
    import math
    for j in range(h_kv):
        for n in range(l):
            acc = 0.0
            for k in range(w):
                vis = l - w + k + 1
                best = 0.0
                for i in range(j * g, (j + 1) * g):
                    z = [sum(Qwin[i, k, c] * K[j, m, c] for c in range(d)) / math.sqrt(d) for m in range(vis)]
                    den = sum(math.exp(x) for x in z)
                    if n < vis:
                        best = max(best, math.exp(z[n]) / den)
                acc += best
            assert S[j, n] == pytest.approx(acc / w, rel=1e-12)


def test_group_max_is_taken_before_the_window_mean():
    # two heads, two rows: head 0 attends entry 0 in row 0 only, head 1 in row 1 only.
    # max-then-mean gives (p + p)/2 = p; mean-then-max would give about p/2.
    K = np.array([[[10.0], [0.0], [0.0], [0.0]]])
    Qwin = np.array([[[1.0], [-1.0]], [[-1.0], [1.0]]])
    S = O.local_score(O.window_probs(Qwin, K, 4), 1)
    p0 = np.exp(10) / (np.exp(10) + 2); p1 = np.exp(10) / (np.exp(10) + 3)
    assert S[0, 0] == pytest.approx((p0 + p1) / 2, rel=1e-13)


# ---------------------------------------------------------- global score ----
def test_global_score_properties():
    rng = np.random.default_rng(7)
    S = rng.random((3, 20)) ** 4
    H = rng.random((3, 12))
    Sn = S[:, :16] / S[:, :16].max(axis=1, keepdims=True)
    F = O.global_score(S, H, 12, 0.8, "max", n_cand=16)
    assert F.shape == (3, 16)
    assert (F <= 1 + 1e-15).all() and (F >= Sn - 1e-15).all() and (F[:, :12] >= 0.8 * H - 1e-15).all()
    np.testing.assert_array_equal(F[:, 12:], Sn[:, 12:])           # no history -> normalised local score
    assert (np.isclose(Sn.max(axis=1), 1.0)).all()
    for form in O.COMBINE_FORMS:                                   # alpha = 0 collapses every form
        np.testing.assert_allclose(O.global_score(S, H, 12, 0.0, form, n_cand=16), Sn, rtol=1e-15)
        np.testing.assert_array_equal(O.global_score(S, H, 0, 0.8, form, n_cand=16), Sn)
    # zero history equals no history for max and sum, but not for avg
    Z = np.zeros_like(H)
    np.testing.assert_array_equal(O.global_score(S, Z, 12, 0.8, "max", n_cand=16), Sn)
    np.testing.assert_array_equal(O.global_score(S, Z, 12, 0.8, "sum", n_cand=16), Sn)
    Favg = O.global_score(S, Z, 12, 0.8, "avg", n_cand=16)
    np.testing.assert_allclose(Favg[:, :12], 0.2 * Sn[:, :12], rtol=1e-14)
    np.testing.assert_array_equal(Favg[:, 12:], Sn[:, 12:])
    # normalisation domain: a huge window column must not set the scale
    S2 = S.copy(); S2[:, 18] = 50.0
    np.testing.assert_array_equal(O.global_score(S2, H, 12, 0.8, "max", n_cand=16), F)
    assert not np.array_equal(O.global_score(S2, H, 12, 0.8, "max", n_cand=16, norm_over="all"), F)


def test_global_score_decay_of_a_token_never_attended_again():
    # max form: a token whose local score stays at 0 decays 0.8, 0.64, 0.512, ...
    f = np.array([[1.0, 1.0]])
    seen = []
    for _ in range(4):
        S = np.array([[0.0, 1.0, 0.3]])
        f = O.global_score(S, f, 2, 0.8, "max", n_cand=2)
        seen.append(f[0, 0])
    np.testing.assert_allclose(seen, [0.8, 0.64, 0.512, 0.4096], rtol=1e-15)
    # the three cases of the paper's discussion (low/low, low/high, high/low)
    S = np.array([[0.01, 0.9, 0.02, 1.0]])
    H = np.array([[0.02, 0.05, 0.9]])
    F = O.global_score(S, H, 3, 0.8, "max", n_cand=4)[0]
    assert F[0] < 0.05 and F[1] == pytest.approx(0.9) and F[2] == pytest.approx(0.72)


# ----------------------------------------------------------------- top-k ----
def _beats(F, m, n):
    return F[m] > F[n] or (F[m] == F[n] and m < n)


def test_select_topk_against_counting_brute_force():
    rng = np.random.default_rng(8)
    for trial in range(20):
        c = int(rng.integers(5, 40)); k = int(rng.integers(1, c))
        F = np.round(rng.random((2, c)), 1 if trial % 2 else 6)     # odd trials: many ties
        keep = O.select_topk(F, k)
        for j in range(2):
            expect = [n for n in range(c) if sum(_beats(F[j], m, n) for m in range(c)) < k]
            assert keep[j].tolist() == expect


def test_select_topk_ties_scale_and_permutation():
    assert O.select_topk(np.full((1, 9), 0.25), 4)[0].tolist() == [0, 1, 2, 3]
    rng = np.random.default_rng(9)
    F = rng.random((1, 30))
    keep = O.select_topk(F, 11)[0]
    assert (np.diff(keep) > 0).all() and len(keep) == 11
    np.testing.assert_array_equal(O.select_topk(F * 7.5, 11)[0], keep)      # positive scaling
    perm = rng.permutation(30)
    kept_perm = O.select_topk(F[:, perm], 11)[0]
    assert sorted(perm[kept_perm].tolist()) == keep.tolist()


def test_select_topk_and_pool_scores_random_properties():
    # seeded sweep over shapes and tie densities: the kept set is exactly the k best under
    # (score descending, index ascending), i.e. every kept entry beats every dropped one
    rng = np.random.default_rng(80)
    for trial in range(60):
        c = int(rng.integers(2, 70)); k = int(rng.integers(1, c)); h = int(rng.integers(1, 4))
        F = np.round(rng.standard_normal((h, c)), int(rng.integers(0, 4)))
        keep = O.select_topk(F, k)
        assert keep.shape == (h, k) and (np.diff(keep, axis=1) > 0).all()
        for j in range(h):
            kept = set(keep[j].tolist())
            worst_kept = max(kept, key=lambda n: (-F[j, n], n))            # last in the ranking among the kept
            for n in range(c):
                if n not in kept:
                    assert _beats(F[j], worst_kept, n)
        half = int(rng.integers(0, 5))
        P = O.pool_scores(F, 2 * half + 1)
        for j in range(h):
            for n in range(c):
                assert P[j, n] == F[j, max(0, n - half):n + half + 1].max()


# ---------------------------------------------------- the whole state machine
def _run(cfg, n_steps, cls=O.OracleA, **kw):
    tr = Trace(cfg)
    q, k, v = tr.unit_steps(0, 0, 0, n_steps)
    kwargs = dict(alpha=cfg.alpha, form=cfg.combine)
    kwargs.update(kw)
    orc = cls(cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.budget, cfg.window, cfg.interval, **kwargs)
    outs = [orc.step(t, q[t], k[t], v[t]) for t in range(n_steps)]
    return orc, np.stack(outs), (q, k, v)


SMALL = CONFIGS["cfg1_tiny"].with_(n_q_heads=4, n_kv_heads=2, head_dim=8, budget=12, window=3,
                                   interval=4, n_steps=60)


def test_budget_is_exact_and_positions_stay_sorted():
    cfg = CONFIGS["cfg1_tiny"]
    tr = Trace(cfg)
    q, k, v = tr.unit_steps(0, 0, 0, cfg.n_steps)
    orc = O.OracleA(cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.budget, cfg.window, cfg.interval)
    n_events = 0
    for t in range(cfg.n_steps):
        orc.step(t, q[t], k[t], v[t])
        assert orc.len <= cfg.budget + cfg.interval
        if len(orc.events) > n_events:
            n_events = len(orc.events)
            assert orc.len == cfg.budget and orc.n_hist == cfg.budget - cfg.window
            for j in range(cfg.n_kv_heads):
                p = orc.pos[j, :orc.len]
                assert (np.diff(p) > 0).all()
                assert p[-cfg.window:].tolist() == list(range(t - cfg.window + 1, t + 1))
                assert (orc.pos[j, orc.len:] == -1).all()
            assert orc.events[-1]["keep"].shape == (cfg.n_kv_heads, cfg.budget - cfg.window)
    assert n_events == 12            # t+1 = 80, 96, ..., 256


def test_no_eviction_while_cache_fits_and_output_is_dense_attention():
    cfg = CONFIGS["cfg1_tiny"]
    orc, outs, (q, k, v) = _run(cfg, cfg.budget)        # 64 steps, 4 triggers with len <= b
    assert orc.events == [] and orc.len == cfg.budget
    g = cfg.group
    for t in (0, 17, 63):
        for i in range(cfg.n_q_heads):
            p = sp_softmax(k[:t + 1, i // g].astype(np.float64) @ q[t, i].astype(np.float64) / np.sqrt(cfg.head_dim))
            np.testing.assert_allclose(outs[t, i], p @ v[:t + 1, i // g].astype(np.float64), rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("form", O.COMBINE_FORMS)
def test_compacting_oracle_equals_mask_oracle(form):
    a, outs_a, _ = _run(SMALL, SMALL.n_steps, O.OracleA, form=form)
    b, outs_b, _ = _run(SMALL, SMALL.n_steps, O.OracleB, form=form)
    assert len(a.events) == len(b.kept_log) > 5
    np.testing.assert_allclose(outs_a, outs_b, rtol=1e-10, atol=1e-12)
    for j in range(SMALL.n_kv_heads):
        alive = sorted(b.alive[j])
        assert a.pos[j, :a.len].tolist() == alive
        np.testing.assert_allclose(a.F_hist[j, :a.n_hist], [b.hist[j][n] for n in alive[:a.n_hist]], rtol=1e-12)


def test_eviction_log_matches_the_mask_oracle():
    # what oracle A logs as evicted is exactly what leaves oracle B's alive set at each event
    a, _, _ = _run(SMALL, SMALL.n_steps, O.OracleA)
    tr = Trace(SMALL)
    q, k, v = tr.unit_steps(0, 0, 0, SMALL.n_steps)
    b = O.OracleB(SMALL.n_q_heads, SMALL.n_kv_heads, SMALL.head_dim, SMALL.budget, SMALL.window, SMALL.interval)
    n_ev = 0
    for t in range(SMALL.n_steps):
        before = [set(x) | {t} for x in b.alive]
        b.step(t, q[t], k[t], v[t])
        if len(b.kept_log) > n_ev:
            for j in range(SMALL.n_kv_heads):
                assert sorted(before[j] - b.alive[j]) == a.events[n_ev]["evicted_pos"][j]
                assert len(a.events[n_ev]["evicted_pos"][j]) == a.events[n_ev]["len"] - SMALL.budget
            n_ev += 1
    assert n_ev == len(a.events) > 5


def test_compacted_attention_equals_masked_dense_attention_over_history():
    cfg = SMALL
    orc, outs, (q, k, v) = _run(cfg, 41)
    t = 40
    for j in range(cfg.n_kv_heads):
        alive = orc.pos[j, :orc.len]
        for i in range(j * cfg.group, (j + 1) * cfg.group):
            z = k[:t + 1, j].astype(np.float64) @ q[t, i].astype(np.float64) / np.sqrt(cfg.head_dim)
            mask = np.full(t + 1, -np.inf); mask[alive] = 0.0
            p = sp_softmax(z + mask)
            np.testing.assert_allclose(outs[t, i], p @ v[:t + 1, j].astype(np.float64), rtol=1e-11, atol=1e-13)


def test_history_disabled_reduces_to_local_score_eviction():
    # alpha = 0 in any form must evict exactly like a local-score-only policy (n_hist pinned to 0).
    cfg = SMALL

    class LocalOnly(O.OracleA):
        def compress(self):
            self.n_hist = 0
            super().compress()

    ref, outs_ref, _ = _run(cfg, cfg.n_steps, LocalOnly)
    for form in O.COMBINE_FORMS:
        a, outs, _ = _run(cfg, cfg.n_steps, O.OracleA, alpha=0.0, form=form)
        np.testing.assert_array_equal(a.pos, ref.pos)
        np.testing.assert_allclose(outs, outs_ref, rtol=1e-13)
    g, _, _ = _run(cfg, cfg.n_steps, O.OracleA, alpha=0.8, form="max")
    assert not np.array_equal(g.pos, ref.pos)             # the history term does change the kept set


def test_first_compression_selects_on_raw_local_score():
    cfg = SMALL
    orc, _, _ = _run(cfg, 16)                   # first event at t+1 = 16 (len 16 > 12)
    ev = orc.events[0]
    assert ev["n_hist"] == 0
    np.testing.assert_array_equal(O.select_topk(ev["S"], cfg.budget - cfg.window), ev["keep"])


def test_recurring_keys_survive_with_history_but_not_without():
    # the synthetic "recurring" recipe exists to make the two policies differ: boosted keys are
    # only attended during bursts; count how many boosted positions each policy still holds.
    cfg = CONFIGS["cfg2_single_layer"].with_(n_q_heads=7, n_kv_heads=1, n_steps=2560)
    tr = Trace(cfg)
    q, k, v = tr.unit_steps(0, 0, 0, cfg.n_steps)
    u, _ = tr.static(0)
    boosted = set(np.nonzero((k[:, 0].astype(np.float64) @ u[0].astype(np.float64)) > 0.6 * tr.boost)[0].tolist())
    held = {}
    for alpha in (0.0, 0.8):
        orc = O.OracleA(cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.budget, cfg.window, cfg.interval, alpha=alpha)
        for t in range(cfg.n_steps):
            orc.step(t, q[t], k[t], v[t])
        old = {p for p in boosted if p < cfg.n_steps - cfg.budget - cfg.interval}
        held[alpha] = len(old & set(orc.pos[0, :orc.len].tolist()))
    assert len(boosted) >= 10
    assert held[0.8] >= held[0.0] + 3


def test_trace_generator_is_chunking_invariant_and_dtype_exact():
    cfg = CONFIGS["cfg2_single_layer"]
    tr = Trace(cfg)
    q, k, v = tr.unit_steps(0, 0, 50, 100)
    q2, k2, v2 = tr.unit_steps(0, 0, 90, 20)
    np.testing.assert_array_equal(q[40:60], q2); np.testing.assert_array_equal(k[40:60], k2)
    from gkv_traces import bf16_round
    np.testing.assert_array_equal(bf16_round(k), k)
    qb, kb, vb = tr.batch_steps(50, 8)
    np.testing.assert_array_equal(qb[:, 0, 0], q[:8])
    qn, kn, vn = tr.batch_steps(50, 8, need_q=False)             # prompts draw keys and values only
    assert qn is None
    np.testing.assert_array_equal(kn, kb); np.testing.assert_array_equal(vn, vb)


# ------------------------------------------------------------------------ prompts ----
def _steps_with_prompt(cfg, cls, P, t0, n_decode, **kw):
    """Tokens t0-P .. t0-1 as a prompt, then n_decode decode steps from t0 (trace steps are positions)."""
    tr = Trace(cfg)
    q, k, v = tr.unit_steps(0, 0, 0, t0 + n_decode)
    orc = cls(cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.budget, cfg.window, cfg.interval, **kw)
    orc.prefill(t0 - P, k[t0 - P:t0], v[t0 - P:t0])
    outs = [orc.step(t, q[t], k[t], v[t]) for t in range(t0, t0 + n_decode)]
    return orc, np.stack(outs)


def test_prompt_within_budget_equals_decoding_it():
    # A prompt of P <= b tokens leaves the state P decode steps leave (no compression can happen
    # while the cache fits), so everything after it must agree with the run that decoded it.
    cfg = SMALL
    P = 7
    ref, outs_ref, _ = _run(cfg, cfg.n_steps)
    orc, outs = _steps_with_prompt(cfg, O.OracleA, P, P, cfg.n_steps - P, alpha=cfg.alpha)
    np.testing.assert_array_equal(outs, outs_ref[P:])
    np.testing.assert_array_equal(orc.pos, ref.pos)
    np.testing.assert_array_equal(orc.F_hist, ref.F_hist)
    assert len(orc.events) == len(ref.events) > 5


@pytest.mark.parametrize("P,t0", [(5, 9), (12, 12), (0, 6)])
def test_prompt_compacting_oracle_equals_mask_oracle(P, t0):
    # shorter prompt than the common start (left-padded batch frame): positions t0-P .. t0-1
    cfg = SMALL
    a, outs_a = _steps_with_prompt(cfg, O.OracleA, P, t0, 50)
    b, outs_b = _steps_with_prompt(cfg, O.OracleB, P, t0, 50)
    assert len(a.events) == len(b.kept_log) > 5
    np.testing.assert_allclose(outs_a, outs_b, rtol=1e-10, atol=1e-12)
    for j in range(cfg.n_kv_heads):
        assert a.pos[j, :a.len].tolist() == sorted(b.alive[j])


def test_prompt_longer_than_budget_waits_for_a_full_window():
    # b = 12, w = 3, s = 4.  Prompt of 20 rows, decoding from t0 = 22: the trigger after step 23 has
    # seen only 2 generated tokens, fewer than the window, so nothing happens; the one after step 27
    # compresses 26 rows down to the budget, window = the last 3 generated tokens.
    cfg = SMALL
    for cls in (O.OracleA, O.OracleB):
        kw = dict(capacity=32) if cls is O.OracleA else {}
        orc, _ = _steps_with_prompt(cfg, cls, 20, 22, 2, **kw)
        n_ev = len(orc.events) if cls is O.OracleA else len(orc.kept_log)
        assert n_ev == 0
        orc, _ = _steps_with_prompt(cfg, cls, 20, 22, 6, **kw)
        if cls is O.OracleA:
            assert len(orc.events) == 1 and orc.events[0]["len"] == 26 and orc.len == cfg.budget
            assert orc.pos[0, cfg.budget - 3:cfg.budget].tolist() == [25, 26, 27]
            keep_a = [orc.pos[j, :orc.len].tolist() for j in range(cfg.n_kv_heads)]
        else:
            assert len(orc.kept_log) == 1
            assert [sorted(x) for x in orc.alive] == keep_a


# ------------------------------------------------------------- redundancy score ----
def test_redundancy_closed_forms():
    l, d = 12, 16
    eye = np.eye(l, d)[None] * 3.0                       # orthogonal keys: no similarity at all
    R = O.redundancy_score(eye, l, tau=0.5)
    np.testing.assert_allclose(R, 1.0 / l, rtol=1e-13)
    # all keys identical, last m columns masked: column sums are l-1 (diagonal excluded) or 0
    m = 3
    same = np.tile(np.arange(1.0, d + 1)[None, None], (1, l, 1))
    R = O.redundancy_score(same, l, tau=0.5, n_recent=m, eps=0.0)
    den = (l - m) * np.exp(l - 1.0) + m
    np.testing.assert_allclose(R[0, :l - m], np.exp(l - 1.0) / den, rtol=1e-12)
    np.testing.assert_allclose(R[0, l - m:], 1.0 / den, rtol=1e-12)
    # one duplicated key among orthogonal ones: both copies get column sum 1
    K = np.eye(l, d)[None].copy(); K[0, 5] = 7.0 * K[0, 2]
    R = O.redundancy_score(K, l, tau=0.5, eps=0.0)
    den = 2 * np.e + (l - 2)
    np.testing.assert_allclose(R[0, [2, 5]], np.e / den, rtol=1e-13)
    np.testing.assert_allclose(np.delete(R[0], [2, 5]), 1.0 / den, rtol=1e-13)


def test_redundancy_threshold_scale_invariance_and_hand_values():
    # keys (1,0), (3,4)/5-direction, (0,1): cos(0,1) = 0.6, cos(1,2) = 0.8, cos(0,2) = 0
    K = np.array([[[2.0, 0.0], [3.0, 4.0], [0.0, 5.0]]])
    R = O.redundancy_score(K, 3, tau=0.5, eps=0.0)
    col = np.array([0.6, 1.4, 0.8])
    np.testing.assert_allclose(R[0], np.exp(col) / np.exp(col).sum(), rtol=1e-13)
    R = O.redundancy_score(K, 3, tau=0.7, eps=0.0)          # 0.6 now falls below the threshold
    col = np.array([0.0, 0.8, 0.8])
    np.testing.assert_allclose(R[0], np.exp(col) / np.exp(col).sum(), rtol=1e-13)
    R = O.redundancy_score(K, 3, tau=0.6, eps=0.0)          # an entry equal to the threshold is kept
    np.testing.assert_allclose(R[0], np.exp([0.6, 1.4, 0.8]) / np.exp([0.6, 1.4, 0.8]).sum(), rtol=1e-13)
    rng = np.random.default_rng(11)
    K = rng.standard_normal((2, 9, 6))
    scaled = K * rng.uniform(0.5, 4.0, size=(2, 9, 1))
    np.testing.assert_allclose(O.redundancy_score(scaled, 9, 0.2, eps=0.0), O.redundancy_score(K, 9, 0.2, eps=0.0), rtol=1e-12)
    R = O.redundancy_score(K, 9, 0.2, n_recent=2)
    np.testing.assert_allclose(R.sum(axis=1), 1.0, rtol=1e-13)
    # brute force with scalar loops
    import math
    for j in range(2):
        nrm = [math.sqrt(sum(x * x for x in K[j, n])) + 1e-8 for n in range(9)]
        col = []
        for c in range(9):
            tot = 0.0
            for k in range(9):
                cs = sum(K[j, k, i] * K[j, c, i] for i in range(6)) / (nrm[k] * nrm[c])
                if k != c and cs >= 0.2 and c < 9 - 2:
                    tot += cs
            col.append(tot)
        z = [math.exp(x) for x in col]
        for c in range(9):
            assert R[j, c] == pytest.approx(z[c] / sum(z), rel=1e-12)


def test_redundancy_parts_and_margin():
    # the intermediates a checker may look at: C is the cosine matrix (symmetric, unit diagonal with
    # eps = 0, equal to the hand values of the three-key example), col its thresholded column sums,
    # the margin the distance of the nearest counted entry from tau
    K = np.array([[[2.0, 0.0], [3.0, 4.0], [0.0, 5.0]]])
    R, margin, parts = O.redundancy_score(K, 3, tau=0.5, eps=0.0, return_margin=True, return_parts=True)
    np.testing.assert_allclose(parts["C"][0], [[1.0, 0.6, 0.0], [0.6, 1.0, 0.8], [0.0, 0.8, 1.0]], atol=1e-15)
    np.testing.assert_allclose(parts["col"][0], [0.6, 1.4, 0.8], rtol=1e-15)
    assert margin[0] == pytest.approx(0.1, rel=1e-12)                # |0.6 - 0.5|
    np.testing.assert_allclose(R[0], sp_softmax(parts["col"][0]), rtol=1e-14)
    # with the newest row exempt its column counts for nothing, and only entries of the other
    # columns set the margin: |0.6 - 0.55| in column 0/1, not |0.8 - 0.55| ... of column 2
    R, margin, parts = O.redundancy_score(K, 3, tau=0.55, n_recent=1, eps=0.0, return_margin=True, return_parts=True)
    np.testing.assert_allclose(parts["col"][0], [0.6, 1.4, 0.0], rtol=1e-15)
    assert margin[0] == pytest.approx(0.05, rel=1e-12)
    rng = np.random.default_rng(13)
    K = rng.standard_normal((2, 40, 16))
    R, parts = O.redundancy_score(K, 40, 0.3, n_recent=4, return_parts=True)
    C = parts["C"]
    np.testing.assert_allclose(C, np.swapaxes(C, 1, 2), rtol=0, atol=1e-15)
    np.testing.assert_allclose(np.einsum("hii->hi", C), 1.0, rtol=1e-7)   # eps = 1e-8 in the norm


def test_combine_redundancy_properties():
    rng = np.random.default_rng(12)
    F = rng.random((2, 10)); R = rng.random((2, 14)); R /= R.sum(axis=1, keepdims=True)
    np.testing.assert_array_equal(O.combine_redundancy(F, R, 1.0, n_cand=10), F)
    Fp = O.combine_redundancy(F, R, 0.7, n_cand=10)
    np.testing.assert_allclose(Fp, 0.7 * F - 0.3 * R[:, :10] / R.max(axis=1, keepdims=True), rtol=1e-14)
    # uniform redundancy shifts every candidate equally: the selection does not change
    U = np.full((2, 14), 1.0 / 14)
    np.testing.assert_array_equal(O.select_topk(O.combine_redundancy(F, U, 0.7, 10), 4), O.select_topk(F, 4))
    # a redundant copy loses against an equally scored unique token
    F2 = np.array([[0.5, 0.5, 0.5, 0.1]]); R2 = np.array([[0.4, 0.1, 0.4, 0.1]])
    assert O.select_topk(O.combine_redundancy(F2, R2, 0.7), 1)[0].tolist() == [1]


def test_oracle_with_redundancy_keeps_budget_and_records_global_score():
    cfg = SMALL
    red = dict(lam=0.7, tau=0.3, n_recent=cfg.window)
    orc, _, _ = _run(cfg, cfg.n_steps, O.OracleA, redundancy=red)
    assert len(orc.events) > 5 and orc.len <= cfg.budget + cfg.interval
    ev = orc.events[-1]
    assert ev["keep"].shape == (cfg.n_kv_heads, cfg.budget - cfg.window)
    # lam = 1 is plain global-score eviction
    a, _, _ = _run(cfg, cfg.n_steps, O.OracleA, redundancy=dict(lam=1.0, tau=0.3, n_recent=0))
    b, _, _ = _run(cfg, cfg.n_steps, O.OracleA)
    np.testing.assert_array_equal(a.pos, b.pos)
    # the history that is carried is the global score F, not the combined one
    last = orc.events[-1]
    for j in range(cfg.n_kv_heads):
        np.testing.assert_array_equal(orc.F_hist[j, :orc.n_hist], last["F"][j, last["keep"][j]])


def test_pool_scores():
    rng = np.random.default_rng(14)
    F = rng.random((2, 17))
    np.testing.assert_array_equal(O.pool_scores(F, 1), F)
    spike = np.zeros((1, 11)); spike[0, 4] = 1.0
    assert O.pool_scores(spike, 5)[0].tolist() == [0, 0, 1, 1, 1, 1, 1, 0, 0, 0, 0]
    assert O.pool_scores(spike, 3)[0].tolist() == [0, 0, 0, 1, 1, 1, 0, 0, 0, 0, 0]
    P7 = O.pool_scores(F, 7)
    assert (P7 >= F).all()
    for j in range(2):
        for n in range(17):
            assert P7[j, n] == max(F[j, m] for m in range(17) if abs(m - n) <= 3)
    np.testing.assert_array_equal(O.pool_scores(F, 99), np.broadcast_to(F.max(axis=1, keepdims=True), F.shape))
