"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle on the same
seeded inputs.  Integer results (kept indices, positions, cache rows) bit-exact up to the
tolerated-swap rule; outputs within 1e-5 relative (fp32) / 2e-2 absolute (bf16)."""
import numpy as np
import pytest
import torch

from gkv_traces import CONFIGS
from oracle import gkv_oracle as O
from paper_2512_00504_amd import make_config
from paper_2512_00504_amd.state import DecodeState, k_cache_to_rows, k_rows_to_cache

from parity_utils import check_keep, check_scores, run_parity

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------ whole-path parity ------
def test_cfg1_tiny_full_trace_fp32():
    wl = CONFIGS["cfg1_tiny"]
    _say("cfg1 tiny fp32, 256 steps")
    st = run_parity(wl, wl.n_steps)
    assert st["events"] == 12 and st["swaps"] == 0
    _say(f"  max out err {st['max_out_err']:.2e}")


def test_cfg1_fused_evict_entry_point():
    wl = CONFIGS["cfg1_tiny"]
    st = run_parity(wl, 128, fused_evict=True)
    assert st["events"] == 4


@pytest.mark.parametrize("form", ["avg", "sum"])
def test_cfg1_other_combine_forms(form):
    wl = CONFIGS["cfg1_tiny"].with_(combine=form, alpha=0.9)
    st = run_parity(wl, 160)
    assert st["events"] == 6


def test_cfg1_shape_in_bf16_generic_kernels():
    # bf16 with d = 64 is not covered by the matrix-core kernels: exercises the generic bf16 path
    wl = CONFIGS["cfg1_tiny"].with_(dtype="bf16", seed=11)
    st = run_parity(wl, 160)
    assert st["events"] == 6


def test_cfg2_single_layer_full_trace():
    wl = CONFIGS["cfg2_single_layer"]
    _say("cfg2 single layer bf16, 4096 steps (split-K attend, MFMA score)")
    st = run_parity(wl, wl.n_steps, check_state_every_event=False)
    assert st["events"] == 28
    _say(f"  max out err {st['max_out_err']:.2e} swaps {st['swaps']}")


def test_cfg2_generic_kernels_match_too():
    wl = CONFIGS["cfg2_single_layer"]
    st = run_parity(wl, 896, params={"force_generic": 1}, check_state_every_event=False)
    assert st["events"] == 3


@pytest.mark.parametrize("splits", [1, 3, 5])
def test_cfg2_split_counts(splits):
    wl = CONFIGS["cfg2_single_layer"]
    st = run_parity(wl, 768, params={"attend_splits": splits}, check_state_every_event=False)
    assert st["events"] == 2


def test_cfg3_shape_small_batch_many_layers():
    # 28-layer head shape, 3 layers x 2 sequences so that every unit is checked
    wl = CONFIGS["cfg3_28layer_b512"].with_(n_layers=3, batch=2)
    st = run_parity(wl, 1024, check_state_every_event=False)
    assert st["events"] == 4


@pytest.mark.parametrize("form", ["max", "avg", "sum"])
def test_cfg3_shape_evict_entry_point(form):
    # gkv_evict (the four compression calls in one entry point) on the matrix-core kernels
    wl = CONFIGS["cfg3_28layer_b512"].with_(n_layers=2, batch=2, combine=form)
    st = run_parity(wl, 1024, fused_evict=True, check_state_every_event=False)
    assert st["events"] == 4


def test_cfg3_shape_evict_with_the_global_score_in_the_score_kernels_tail():
    # optional one-launch local + global score (S stays in LDS for the update): same results
    wl = CONFIGS["cfg3_28layer_b512"].with_(n_layers=2, batch=2)
    st = run_parity(wl, 1024, fused_evict=True, params={"evict_fuse_global": 1}, check_state_every_event=False)
    assert st["events"] == 4
    wl5 = CONFIGS["cfg5_large_batch"].with_(n_layers=1, batch=2)
    st = run_parity(wl5, 1216, fused_evict=True, params={"evict_fuse_global": 1, "score_reuse_stats": 0},
                    check_state_every_event=False)
    assert st["events"] == 3


def test_compaction_without_a_workspace_rewrites_the_state_in_a_second_launch():
    # same compaction twice from the same state: with the workspace (the last workgroup of each
    # (layer, sequence) rewrites the record) and without (a launch of its own does): same bits
    wl = CONFIGS["cfg3_28layer_b512"].with_(n_layers=2, batch=3)
    from gkv_traces import Trace
    tr = Trace(wl)
    n = wl.budget + wl.interval
    q, k, v = [torch.from_numpy(x).to(torch.bfloat16).cuda() for x in tr.batch_steps(0, n)]
    results = []
    for use_ws in (True, False):
        st = DecodeState.from_workload(wl)
        for t in range(n):
            st.attend_decode(q[t], k[t], v[t], t)
        st.score_window(n - 1); st.global_update(n - 1); st.select_topk(n - 1)
        st.ctx.compact(st.keep_idx, st.F, st.K, st.V, st.F_hist, st.pos, st.d_state, n - 1,
                       st.workspace if use_ws else None)
        torch.cuda.synchronize()
        assert (st.d_state[..., 0] == wl.budget).all() and (st.d_state[..., 1] == n).all()
        results.append([x.clone() for x in (st.K, st.V, st.pos, st.F_hist, st.d_state)])
    for a_, b_ in zip(*results):
        assert torch.equal(a_.view(torch.uint8), b_.view(torch.uint8))
    # and the ticket counters are back at zero: a second compression on the same workspace works
    st = DecodeState.from_workload(wl)
    q2, k2, v2 = [torch.from_numpy(x).to(torch.bfloat16).cuda() for x in tr.batch_steps(n, wl.interval)]
    for t in range(n):
        st.attend_decode(q[t], k[t], v[t], t)
    st.evict(n - 1)
    for i in range(wl.interval):
        st.attend_decode(q2[i], k2[i], v2[i], n + i)
    st.evict(n + wl.interval - 1)
    torch.cuda.synchronize()
    assert (st.d_state[..., 0] == wl.budget).all() and (st.d_state[..., 1] == n + wl.interval).all()
    units = wl.n_layers * wl.batch * wl.n_kv_heads
    off = ((units * 4 + 255) & ~255) // 4                  # the per-(layer, sequence) counters follow the per-unit ones
    tickets = st.workspace[: 4 * (off + wl.n_layers * wl.batch)].view(torch.int32)
    assert int(tickets.abs().sum()) == 0


def test_evict_with_the_global_score_in_a_launch_of_its_own():
    # gkv_evict forms the global score at the head of the selection kernel by default; with that
    # switched off it takes the gkv_global_update launch: same results (both against the oracle)
    wl = CONFIGS["cfg3_28layer_b512"].with_(n_layers=2, batch=2, combine="avg")
    st = run_parity(wl, 1024, fused_evict=True, params={"evict_fuse_select": 0}, check_state_every_event=False)
    assert st["events"] == 4
    st = run_parity(CONFIGS["cfg1_tiny"], 128, fused_evict=True, params={"evict_fuse_select": 0})
    assert st["events"] == 4


def test_cfg3_shape_32_key_slices():
    # the other slice size of the matrix-core attend kernel
    wl = CONFIGS["cfg3_28layer_b512"].with_(n_layers=2, batch=2)
    st = run_parity(wl, 768, params={"attend_tile": 32}, check_state_every_event=False)
    assert st["events"] == 2


def test_cfg3_shape_window_score_computes_its_own_row_statistics():
    # by default the window score takes the rows' softmax statistics from the decode kernel's
    # record; with that switched off it computes them in a first pass over the keys
    wl = CONFIGS["cfg3_28layer_b512"].with_(n_layers=2, batch=2)
    st = run_parity(wl, 768, params={"score_reuse_stats": 0}, check_state_every_event=False)
    assert st["events"] == 2


def test_window_score_with_and_without_recorded_statistics_agree():
    # same state, both routes: each within 1e-5 of the oracle (checked in the whole-path tests),
    # and within 3e-6 of each other
    from gkv_traces import Trace
    for name, over in (("cfg3_28layer_b512", dict(n_layers=2, batch=2)), ("cfg5_large_batch", dict(n_layers=1, batch=2))):
        wl = CONFIGS[name].with_(**over)
        tr = Trace(wl)
        n = wl.budget + wl.interval
        st = DecodeState.from_workload(wl)
        q, k, v = [torch.from_numpy(x).to(torch.bfloat16).cuda() for x in tr.batch_steps(0, n)]
        for t in range(n):
            st.attend_decode(q[t], k[t], v[t], t)
        assert st.is_trigger(n - 1)
        st.score_window(n - 1)
        S1 = st.S.clone()
        st.ctx.set_param("score_reuse_stats", 0)
        st.S.zero_()
        st.score_window(n - 1)
        c = n - wl.window
        a, b = S1[..., :c].double().cpu().numpy(), st.S[..., :c].double().cpu().numpy()
        assert (a > 0).any()
        np.testing.assert_allclose(a, b, rtol=3e-6, atol=1e-30)


@pytest.mark.parametrize("waves", [8, 16])
def test_cfg3_shape_more_wavefronts_per_unit(waves):
    # the matrix-core attend kernel with 8 or 16 wavefronts per workgroup instead of 4
    wl = CONFIGS["cfg3_28layer_b512"].with_(n_layers=2, batch=2)
    st = run_parity(wl, 768, params={"attend_waves": waves}, check_state_every_event=False)
    assert st["events"] == 2


def test_cfg3_full_size_sampled_units():
    # the launch configuration the benchmark times: all 896 units on the GPU, the oracle on a
    # sample of (layer, sequence) pairs that covers first/last layer and sequence
    wl = CONFIGS["cfg3_28layer_b512"]
    pairs = [(0, 0), (0, 7), (13, 3), (27, 0), (27, 7)]
    _say("cfg3 full size, 768 steps, 5 sampled pairs (20 units)")
    st = run_parity(wl, 768, pairs=pairs, check_state_every_event=False)
    assert st["events"] == 2
    _say(f"  max out err {st['max_out_err']:.2e} swaps {st['swaps']}")


def test_cfg3_layer_group_launch_as_the_benchmark_times_it():
    # the benchmark's default splits the 28 layers into two contexts of 14: that launch size
    # (448 units), layers 14..27 of the trace, oracle on sampled pairs
    wl = CONFIGS["cfg3_28layer_b512"].with_(n_layers=14)
    pairs = [(0, 0), (0, 7), (6, 2), (13, 0), (13, 7)]
    st = run_parity(wl, 2 * wl.interval, pairs=pairs, prompts=[wl.budget] * wl.batch, workers=16)
    assert st["events"] == 2 and st["pair_events"] == 10


def test_cfg3_full_size_longer_run():
    # 44 compressions at the benchmark's launch configuration, free-running between them
    wl = CONFIGS["cfg3_28layer_b512"]
    pairs = [(5, 1), (20, 6), (27, 4)]
    _say("cfg3 full size, 6144 steps, 3 sampled pairs (12 units)")
    st = run_parity(wl, 6144, pairs=pairs, check_state_every_event=False)
    assert st["events"] == 44
    _say(f"  max out err {st['max_out_err']:.2e} swaps {st['swaps']}")


# The launch configurations the benchmark times, whole: every unit runs on the GPU, the oracle
# follows a seeded sample of (layer, sequence) pairs that covers the first and last layer and
# sequence.  The first b tokens are placed in the cache as a prompt (no compression can happen
# before the cache exceeds the budget), then two whole compression cycles are decoded and every
# step's output of the sampled pairs is compared.
CFG4_PAIRS = [(0, 0), (0, 15), (27, 0), (27, 15), (13, 7), (5, 3), (20, 11), (9, 14)]
CFG5_PAIRS = [(0, 0), (0, 63), (35, 0), (35, 63), (17, 31), (8, 50), (26, 5), (30, 40)]


@pytest.mark.parametrize("name", ["cfg4_b512", "cfg4_b1024", "cfg4_b2048", "cfg4_b512_local"])
def test_cfg4_full_launch_sampled_pairs(name):
    wl = CONFIGS[name]
    _say(f"{name}: 28 layers x 16 sequences = {wl.n_units} units, prompt {wl.budget}, 2 cycles, 8 sampled pairs")
    st = run_parity(wl, 2 * wl.interval, pairs=CFG4_PAIRS, prompts=[wl.budget] * wl.batch,
                    check_state_every_event=True, workers=16, say=_say)
    assert st["events"] == 2 and st["pair_events"] == 16
    _say(f"  max out err {st['max_out_err']:.2e} swaps {st['swaps']}")


def test_cfg5_full_launch_sampled_pairs():
    wl = CONFIGS["cfg5_large_batch"]
    _say(f"cfg5: 36 layers x 64 sequences = {wl.n_units} units, prompt {wl.budget}, 2 cycles, 8 sampled pairs")
    st = run_parity(wl, 2 * wl.interval, pairs=CFG5_PAIRS, prompts=[wl.budget] * wl.batch, chunk=64,
                    check_state_every_event=True, workers=16, say=_say)
    assert st["events"] == 2 and st["pair_events"] == 16
    _say(f"  max out err {st['max_out_err']:.2e} swaps {st['swaps']}")


# ------------------------------------------------------------------ prompts, ragged batches
def test_ragged_prompts_small_shape():
    # b = 96, w = 16, s = 32: prompts of 0, 37 and 150 rows (one longer than the budget), decoding
    # starts at step 150 for all; every compression sees a different length per sequence, and the
    # long prompt has to wait for a full window before its first compression
    wl = CONFIGS["cfg2_single_layer"].with_(n_layers=2, batch=3, n_q_heads=8, n_kv_heads=2, budget=96, window=16,
                                            interval=32, seed=31)
    st = run_parity(wl, 200, prompts=[0, 37, 150], chunk=64, cfg_over=dict(capacity=192))
    lens = sorted({ev["len"] for orc in st["oracles"].values() for ev in orc.events})
    _say(f"  lengths seen by compressions: {lens}")
    assert len(lens) >= 4 and st["pair_events"] >= 20


def test_ragged_prompts_cfg3_shape():
    # P = 0, 37, 300 at the 28q/4kv x 128 head shape (matrix-core kernels): at the trigger after
    # step 895 the three sequences compress from 596, 633 and 640 rows
    wl = CONFIGS["cfg3_28layer_b512"].with_(n_layers=2, batch=3)
    st = run_parity(wl, 640, prompts=[0, 37, 300], check_state_every_event=True)
    lens = sorted({ev["len"] for orc in st["oracles"].values() for ev in orc.events})
    _say(f"  lengths seen by compressions: {lens}")
    assert {596, 633, 640} <= set(lens)


@pytest.mark.parametrize("budget,steps", [(1024, 1408), (2048, 2432)])
def test_cfg4_budgets(budget, steps):
    wl = CONFIGS["cfg4_b512"].with_(n_layers=1, batch=2, budget=budget)
    st = run_parity(wl, steps, check_state_every_event=False)
    assert st["events"] == 3


def test_cfg4_local_only_leg():
    wl = CONFIGS["cfg4_b512_local"].with_(n_layers=2, batch=1)
    st = run_parity(wl, 1024, check_state_every_event=False)
    assert st["events"] == 4
    # alpha = 0: the recorded history never matters, so the max form with zeroed n_hist agrees
    for orc in st["oracles"].values():
        for ev in orc.events:
            np.testing.assert_array_equal(O.select_topk(ev["S"], wl.budget - wl.window), ev["keep"])


def test_cfg5_shape_heavy_tailed_keys():
    wl = CONFIGS["cfg5_large_batch"].with_(n_layers=1, batch=2)
    _say("cfg5 shape (g=5, w=32, s=64, b=1024, Student-t keys), 1216 steps")
    st = run_parity(wl, 1216, check_state_every_event=False)
    assert st["events"] == 3
    _say(f"  max out err {st['max_out_err']:.2e} swaps {st['swaps']}")


@pytest.mark.parametrize("seed", [101, 102, 103])
def test_cfg3_shape_other_seeds(seed):
    # other draws of the same recipe: other tie patterns, other burst alignments
    wl = CONFIGS["cfg3_28layer_b512"].with_(n_layers=1, batch=2, seed=seed)
    st = run_parity(wl, 1280, check_state_every_event=False)
    assert st["events"] == 6


def test_cfg5_shape_many_events_heavy_tails():
    # ten compressions of one sequence with Student-t keys: probabilities far below fp32's range
    # compete in the top-k (the tolerated-swap rule's second clause), free-running between events
    wl = CONFIGS["cfg5_large_batch"].with_(n_layers=1, batch=1, seed=77)
    st = run_parity(wl, 1024 + 10 * 64, check_state_every_event=False, chunk=64)
    assert st["events"] == 10
    _say(f"  max out err {st['max_out_err']:.2e} swaps {st['swaps']}")


@pytest.mark.parametrize("shape", [
    dict(n_q_heads=4, n_kv_heads=4, budget=96, window=16, interval=32),          # MHA, g = 1
    dict(n_q_heads=16, n_kv_heads=2, budget=100, window=16, interval=40),        # g = 8, b and s not multiples of 16, w does not divide s
    dict(n_q_heads=32, n_kv_heads=2, budget=80, window=16, interval=16),         # g = 16 (generic score kernel), w = s
    dict(n_q_heads=12, n_kv_heads=4, budget=72, window=32, interval=56),         # g = 3 (generic score), w = 32
    dict(n_q_heads=10, n_kv_heads=2, budget=64, window=32, interval=32, head_dim=64),   # d = 64: generic everywhere
])
def test_odd_shapes_bf16(shape):
    kw = dict(n_layers=2, batch=3, head_dim=128, dtype="bf16", n_steps=400, seed=21)
    kw.update(shape)
    wl = CONFIGS["cfg2_single_layer"].with_(**kw)
    st = run_parity(wl, wl.n_steps, chunk=64)
    assert st["events"] >= 3


@pytest.mark.parametrize("params", [None, {"force_generic": 1}])
def test_largest_capacity_prompt_fills_the_cache(params):
    # b = 3840, s = 96: capacity 3936 rows, the largest the kernels' 64 KiB of LDS admit at d = 128.
    # Sequence 0 starts with a prompt of b rows, so its first compression sees every row of the
    # cache in use (l = capacity); sequence 1 starts with 1000 rows and is left alone.
    wl = CONFIGS["cfg2_single_layer"].with_(n_layers=1, batch=2, budget=3840, interval=96, seed=41)
    assert wl.capacity == 3936
    st = run_parity(wl, 96, prompts=[3840, 1000], params=params, chunk=96, say=_say)
    assert st["pair_events"] == 1
    ev = st["oracles"][(0, 0)].events[0]
    assert ev["len"] == 3936 and st["oracles"][(0, 1)].len == 1096


@pytest.mark.parametrize("shape", [
    dict(dtype="f32", head_dim=64, n_q_heads=4, n_kv_heads=2, budget=9, window=8, interval=8),       # keeps ONE candidate
    dict(dtype="bf16", head_dim=128, n_q_heads=8, n_kv_heads=2, budget=17, window=16, interval=16),   # same, matrix cores
    dict(dtype="bf16", head_dim=128, n_q_heads=4, n_kv_heads=1, budget=64, window=16, interval=32),   # MQA: one KV head
    dict(dtype="bf16", head_dim=128, n_q_heads=14, n_kv_heads=2, budget=64, window=16, interval=32,
         alpha=1.0, combine="avg"),                                                                    # no decay: history rows keep F
])
def test_degenerate_shapes_and_parameters(shape):
    kw = dict(n_layers=2, batch=2, n_steps=200, seed=51)
    kw.update(shape)
    wl = CONFIGS["cfg2_single_layer"].with_(**kw)
    st = run_parity(wl, wl.n_steps, chunk=64)
    assert st["events"] >= 4
    if shape.get("alpha") == 1.0:          # avg form with alpha = 1: F_t = F_{t-1} for every row with history
        for orc in st["oracles"].values():
            ev0, ev1 = orc.events[-2], orc.events[-1]
            for j in range(wl.n_kv_heads):
                kept = ev0["F"][j][ev0["keep"][j]]
                np.testing.assert_array_equal(ev1["F"][j][:ev1["n_hist"]], kept)


@pytest.mark.parametrize("params", [None, {"attend_splits": 3}, {"force_generic": 1}])
def test_results_are_deterministic(params):
    # same inputs, same bits: outputs, kept indices, scores and cache contents of two runs
    from gkv_traces import Trace
    wl = CONFIGS["cfg3_28layer_b512"].with_(n_layers=2, batch=2, budget=96, interval=32, n_steps=160)
    tr = Trace(wl)
    q, k, v = [torch.from_numpy(x).to(torch.bfloat16).cuda() for x in tr.batch_steps(0, wl.n_steps)]
    runs = []
    for _ in range(2):
        st = DecodeState.from_workload(wl, params=params)
        outs = []
        for t in range(wl.n_steps):
            outs.append(st.attend_decode(q[t], k[t], v[t], t).clone())
            if st.is_trigger(t):
                st.evict(t)
        runs.append((torch.stack(outs), st.keep_idx.clone(), st.F.clone(), st.K.clone(), st.V.clone(), st.F_hist.clone()))
    for x, y in zip(*runs):
        assert torch.equal(x.view(torch.uint8), y.view(torch.uint8))


def test_cfg5_shape_medium_batch_sampled():
    # 4 layers x 8 sequences of the 40q/8kv shape (256 units), oracle on 3 sampled pairs
    wl = CONFIGS["cfg5_large_batch"].with_(n_layers=4, batch=8)
    st = run_parity(wl, 1280, pairs=[(0, 0), (2, 5), (3, 7)], check_state_every_event=False, chunk=64)
    assert st["events"] == 4


# ------------------------------------------------------------------ redundancy score (full G-KV)
def test_redundancy_cfg1_generic_fp32():
    wl = CONFIGS["cfg1_tiny"]
    st = run_parity(wl, 160, redundancy=dict(lam=0.7, tau=0.1, n_recent=wl.window))
    assert st["events"] == 6
    _say(f"  entries on the threshold {st['ambiguous']} (decided the other way: {st['flipped']}) swaps {st['swaps']}")
    assert st["ambiguous"] <= 2


def test_redundancy_cfg3_shape_matrix_cores():
    wl = CONFIGS["cfg3_28layer_b512"].with_(n_layers=2, batch=2)
    st = run_parity(wl, 1024, redundancy=dict(lam=0.7, tau=0.5, n_recent=wl.window), check_state_every_event=False)
    assert st["events"] == 4 and st["pair_events"] == 16
    _say(f"  entries on the threshold {st['ambiguous']} (decided the other way: {st['flipped']}) swaps {st['swaps']}")
    # 64 head-events of ~4e5 cosines each, a 2e-6 wide band around tau: a handful, never a head's worth
    assert st["ambiguous"] <= 400 and st["flipped"] <= st["ambiguous"]


def test_redundancy_cfg5_shape_and_lambda_one():
    wl = CONFIGS["cfg5_large_batch"].with_(n_layers=1, batch=1)
    st = run_parity(wl, 1152, redundancy=dict(lam=0.9, tau=0.4, n_recent=0), check_state_every_event=False)
    assert st["events"] == 2
    _say(f"  entries on the threshold {st['ambiguous']} (decided the other way: {st['flipped']}) swaps {st['swaps']}")
    assert st["ambiguous"] <= 200
    # lambda = 1 must reproduce plain global-score eviction bit for bit
    wl2 = CONFIGS["cfg2_single_layer"]
    a = run_parity(wl2, 768, redundancy=dict(lam=1.0, tau=0.5, n_recent=0), check_state_every_event=False)
    b = run_parity(wl2, 768, check_state_every_event=False)
    n = wl2.budget
    assert torch.equal(a["state"].pos[..., :n], b["state"].pos[..., :n])
    assert torch.equal(a["state"].V[..., :n, :], b["state"].V[..., :n, :])


def test_redundancy_ragged_lengths_cfg3_shape():
    # lengths 596, 633 and 640 at the first trigger: row and column tiles with ragged tails, column
    # shares of unequal size per wavefront, clamped duplicates past the last tile
    wl = CONFIGS["cfg3_28layer_b512"].with_(n_layers=1, batch=3)
    st = run_parity(wl, 640, prompts=[0, 37, 300], redundancy=dict(lam=0.7, tau=0.5, n_recent=wl.window),
                    check_state_every_event=False)
    lens = sorted({ev["len"] for orc in st["oracles"].values() for ev in orc.events})
    _say(f"  lengths {lens}; entries on the threshold {st['ambiguous']} (decided the other way: {st['flipped']}) "
         f"swaps {st['swaps']}")
    assert {596, 633, 640} <= set(lens)
    assert st["ambiguous"] <= 400 and st["flipped"] <= st["ambiguous"]


def test_redundancy_b2048_shape():
    # l = 2176: 136 tiles, seven passes per wavefront, and a workgroup needs more LDS than the default allowance
    wl = CONFIGS["cfg4_b2048"].with_(n_layers=1, batch=1)
    st = run_parity(wl, 2176, redundancy=dict(lam=0.7, tau=0.5, n_recent=wl.window), check_state_every_event=False,
                    chunk=256)
    assert st["events"] == 1
    _say(f"  entries on the threshold {st['ambiguous']} (decided the other way: {st['flipped']}) swaps {st['swaps']}")
    assert st["ambiguous"] <= 400 and st["flipped"] <= st["ambiguous"]


def test_redundancy_largest_capacity():
    # l = capacity = 3936: 246 tiles, 13 passes, 96 KiB of LDS per workgroup; sequence 1 (1096 rows) is left alone
    wl = CONFIGS["cfg2_single_layer"].with_(n_layers=1, batch=2, budget=3840, interval=96, seed=41)
    st = run_parity(wl, 96, prompts=[3840, 1000], redundancy=dict(lam=0.7, tau=0.5, n_recent=wl.window),
                    chunk=96, check_state_every_event=False, say=_say)
    assert st["pair_events"] == 1 and st["oracles"][(0, 0)].events[0]["len"] == 3936
    _say(f"  entries on the threshold {st['ambiguous']} (decided the other way: {st['flipped']}) swaps {st['swaps']}")
    assert st["ambiguous"] <= 400 and st["flipped"] <= st["ambiguous"]


def test_redundancy_closed_form_duplicate_keys():
    # orthogonal keys with one duplicated pair: R' = 1 for the pair, exp(-1) for everyone else
    st = _state("bf16", head_dim=128, n_q_heads=2, n_kv_heads=2, budget=32, window=4, interval=8, capacity=64)
    l = 40
    K = torch.zeros(1, 2, 2, 64, 128)
    for n in range(l):
        K[..., n, n] = 2.0
    K[..., 9, :] = 0; K[..., 9, 3] = 5.0                    # row 9 duplicates the direction of row 3
    st.K.copy_(K.to(torch.bfloat16)); st.F.fill_(0.5)
    _set_lengths(st, (l, l), step_next=l, decoded=4)
    st.redundancy_combine(l - 1, lam=0.7, tau=0.5, n_recent=0, eps=0.0)
    R = st.R[0, 0, 0, :l].double().cpu().numpy()
    expect = np.full(l, np.exp(-1.0)); expect[[3, 9]] = 1.0
    np.testing.assert_allclose(R, expect, rtol=1e-6)
    Fs = st.F_sel[0, 1, 1, :l - 4].double().cpu().numpy()
    np.testing.assert_allclose(Fs, 0.7 * 0.5 - 0.3 * expect[:l - 4], rtol=1e-6)


def test_pool_scores_against_oracle():
    st = _state()
    l, w = 45, 4
    c = l - w
    F = torch.rand(1, 2, 2, 64)
    st.F.copy_(F)
    _set_lengths(st, (l, 20), step_next=l, decoded=w)           # sequence 1 is below the budget: untouched
    st.F_sel.fill_(-7.0)
    for kernel in (1, 5, 8, 200):
        st.ctx.pool_scores(st.F, st.d_state, l - 1, kernel, st.F_sel)
        got = st.F_sel.cpu().numpy()
        ref = O.pool_scores(F[0, 0, :, :c].double().numpy(), kernel)
        np.testing.assert_array_equal(got[0, 0, :, :c].astype(np.float64), ref)
        assert (got[0, 1] == -7.0).all()


# ------------------------------------------------------------------ single calls, edge cases
def _state(dtype="f32", **kw):
    base = dict(n_layers=1, batch=2, n_q_heads=4, n_kv_heads=2, head_dim=64, budget=32, window=4,
                interval=8, capacity=64, dtype=dtype)
    base.update(kw)
    return DecodeState(make_config(**base))


def _set_lengths(st, lens, step_next, n_hist=(0, 0), n_tiled=(0, 0), decoded=0):
    """d_state for a 1-layer, 2-sequence state: lengths `lens` before decode step `step_next`, of
    which the last `decoded` rows were decoded since the cache was loaded (compression wants a
    full window of them, so tests of the compression calls pass decoded = w)."""
    rec = [[lens[i] - decoded, step_next - decoded, n_hist[i], n_tiled[i]] for i in range(2)]
    st.d_state.copy_(torch.tensor([rec], dtype=torch.int32))
    st.len_host = max(lens)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_attend_ragged_lengths_formats_and_empty_append(dtype):
    kw = {} if dtype == "f32" else dict(head_dim=128, n_q_heads=14, n_kv_heads=2)
    st = _state(dtype, **kw)
    d, hq = st.cfg.head_dim, st.cfg.n_q_heads
    g = torch.Generator().manual_seed(1)
    K = torch.randn(1, 2, 2, 64, d, generator=g).to(st.K.dtype)
    V = torch.randn(1, 2, 2, 64, d, generator=g).to(st.K.dtype)
    q = torch.randn(1, 2, hq, d, generator=g).to(st.K.dtype)
    # sequence 0: 5 rows, all row-major; sequence 1: 37 rows, the first 32 in tiled format
    st.K[0, 0] = K[0, 0].cuda(); st.K[0, 1] = k_rows_to_cache(K[0, 1], 32).cuda(); st.V.copy_(V)
    _set_lengths(st, (5, 37), step_next=3, n_tiled=(0, 32))
    state0 = st.d_state.clone()
    out = st.attend_decode(q.cuda(), None, None, 3).double().cpu().numpy()
    assert torch.equal(st.d_state, state0)                        # the decode kernel never writes lengths
    tol = 1e-5 if dtype == "f32" else None
    for b, n in enumerate((5, 37)):
        ref = O.attend(q[0, b].double().numpy(), K[0, b].double().numpy(), V[0, b].double().numpy(), n)
        if tol:
            np.testing.assert_allclose(out[0, b], ref, rtol=0, atol=tol * np.abs(ref).max())
        else:
            np.testing.assert_allclose(out[0, b], ref, rtol=0, atol=2e-2)
    # window ring slot 3 now holds q (ring layout [w, L, B, h_q, d])
    assert torch.equal(st.qwin[3].cpu(), q)


def test_attend_length_follows_the_step_number():
    # LEN = 5 before step 10: at step 12 the cache holds 7 rows and row 7 is appended
    st = _state()
    g = torch.Generator().manual_seed(2)
    K = torch.randn(1, 2, 2, 64, 64, generator=g); V = torch.randn(1, 2, 2, 64, 64, generator=g)
    q = torch.randn(1, 2, 4, 64, generator=g); kn = torch.randn(1, 2, 2, 64, generator=g); vn = torch.randn(1, 2, 2, 64, generator=g)
    st.K.copy_(K); st.V.copy_(V)
    _set_lengths(st, (5, 5), step_next=10)
    st.len_host = 7
    out = st.attend_decode(q.cuda(), kn.cuda(), vn.cuda(), 12).double().cpu().numpy()
    K2, V2 = K.clone(), V.clone()
    K2[0, :, :, 7] = kn[0]; V2[0, :, :, 7] = vn[0]
    for b in range(2):
        ref = O.attend(q[0, b].numpy(), K2[0, b].numpy(), V2[0, b].numpy(), 8)
        np.testing.assert_allclose(out[0, b], ref, rtol=0, atol=1e-5 * np.abs(ref).max())
    assert torch.equal(st.K[0, :, :, 7].cpu(), kn[0]) and torch.equal(st.V[0, :, :, 7].cpu(), vn[0])
    assert (st.pos[0, :, :, 7] == 12).all()
    assert torch.equal(st.qwin[12 % 4].cpu(), q)


def test_attend_zero_copy_ring_slot():
    # q handed over inside its ring slot: same output, the rest of the ring untouched
    st = _state("bf16", head_dim=128, n_q_heads=14, n_kv_heads=2)
    g = torch.Generator().manual_seed(3)
    K = torch.randn(st.K.shape, generator=g).to(torch.bfloat16); V = torch.randn(st.V.shape, generator=g).to(torch.bfloat16)
    q = torch.randn(1, 2, 14, 128, generator=g).to(torch.bfloat16)
    kn = torch.randn(1, 2, 2, 128, generator=g).to(torch.bfloat16); vn = torch.randn(1, 2, 2, 128, generator=g).to(torch.bfloat16)
    outs = []
    for in_place in (False, True):
        st.K.copy_(K); st.V.copy_(V); st.qwin.fill_(9.0)
        _set_lengths(st, (30, 17), step_next=6)
        qd = q.cuda()
        if in_place:
            st.qwin[6 % 4].copy_(q)
            qd = st.qwin[6 % 4]
        outs.append(st.attend_decode(qd, kn.cuda(), vn.cuda(), 6).clone())
        assert torch.equal(st.qwin[6 % 4].cpu(), q)
        assert (st.qwin[[0, 1, 3]] == 9.0).all()
    assert torch.equal(outs[0], outs[1])


def test_attend_rejects_bad_arguments():
    from paper_2512_00504_amd import GkvError
    st = _state()
    q = torch.zeros(1, 2, 4, 64, device="cuda")
    kv = torch.zeros(1, 2, 2, 64, device="cuda")
    st.len_host = 64                                              # would overflow the capacity
    with pytest.raises(GkvError) as e:
        st.attend_decode(q, kv, kv, 0)
    assert e.value.status == 6
    st.len_host = 0
    with pytest.raises(GkvError) as e:
        st.ctx.attend_decode(q, kv, None, st.K, st.V, st.pos, 0, st.qwin, st.d_state, 0, st.out, st.workspace)
    assert e.value.status == 1
    with pytest.raises(GkvError) as e:
        st.ctx.attend_decode(q, kv, kv, st.K, st.V, st.pos, 0, st.qwin, st.d_state, 0, st.out, None)
    assert e.value.status == 3


def test_score_window_closed_form_equal_keys():
    # all keys equal: S[n] = (1/w) sum_k 1/(c+k+1) for every candidate
    for dtype, kw in (("f32", {}), ("bf16", dict(head_dim=128, n_q_heads=8, n_kv_heads=2, window=16,
                                                  interval=16, budget=48, capacity=96))):
        st = _state(dtype, **kw)
        w, cap = st.cfg.window, st.cfg.capacity
        l = st.cfg.budget + st.cfg.interval - 3
        st.K.fill_(0.5)
        st.qwin.copy_(torch.randn(st.qwin.shape).to(st.qwin.dtype))
        _set_lengths(st, (l, l), step_next=l, n_tiled=(0, 32), decoded=w)     # constant keys: format does not matter
        st.score_window(step=l - 1)
        c = l - w
        expect = sum(1.0 / (c + k + 1) for k in range(w)) / w
        S = st.S[..., :c].double().cpu().numpy()
        np.testing.assert_allclose(S, expect, rtol=2e-6)


def test_eviction_is_a_noop_at_or_below_budget():
    st = _state()
    _set_lengths(st, (32, 40), step_next=40, decoded=4)
    st.K.copy_(torch.randn(st.K.shape)); st.V.copy_(torch.randn(st.V.shape))
    st.qwin.copy_(torch.randn(st.qwin.shape))
    K0, V0 = st.K.clone(), st.V.clone()
    st.evict(step=39)
    assert st.d_state.cpu().tolist() == [[[28, 36, 0, 0], [32, 40, 28, 32]]]
    assert torch.equal(st.K[0, 0], K0[0, 0]) and torch.equal(st.V[0, 0], V0[0, 0])     # sequence 0 untouched
    assert not torch.equal(st.V[0, 1], V0[0, 1])


def test_eviction_waits_for_a_full_window_of_generated_tokens():
    # both sequences are above the budget (b = 32, w = 4) at the trigger, but sequence 0 has decoded
    # only 3 tokens since its cache was loaded: its ring does not hold a window yet, nothing happens
    st = _state()
    st.d_state.copy_(torch.tensor([[[37, 37, 0, 0], [36, 36, 0, 0]]], dtype=torch.int32))
    st.len_host = 40
    st.K.copy_(torch.randn(st.K.shape)); st.V.copy_(torch.randn(st.V.shape))
    st.qwin.copy_(torch.randn(st.qwin.shape))
    st.pos.copy_(torch.arange(64, dtype=torch.int32).expand(1, 2, 2, 64))
    K0, V0 = st.K.clone(), st.V.clone()
    st.evicted.fill_(5)
    st.score_window(39); st.global_update(39); st.select_topk(39); st.evicted_positions(39); st.compact(39)
    assert st.d_state.cpu().tolist() == [[[37, 37, 0, 0], [32, 40, 28, 32]]]
    assert torch.equal(st.K[0, 0], K0[0, 0]) and torch.equal(st.V[0, 0], V0[0, 0])
    assert (st.evicted[0, 0] == -1).all() and (st.evicted[0, 1, :, :8] >= 0).all()
    assert not torch.equal(st.V[0, 1], V0[0, 1])


def test_global_update_three_forms_against_oracle():
    rng = np.random.default_rng(5)
    for form in ("max", "avg", "sum"):
        st = _state(combine=form, alpha=0.8)
        l, w = 40, 4
        c = l - w
        S = rng.random((1, 2, 2, 64)).astype(np.float32) ** 3
        H = rng.random((1, 2, 2, 64)).astype(np.float32)
        st.S.copy_(torch.from_numpy(S)); st.F_hist.copy_(torch.from_numpy(H))
        _set_lengths(st, (l, l), step_next=l, n_hist=(0, 28), decoded=w)
        st.global_update(l - 1)
        F = st.F.cpu().numpy()
        for b, nh in enumerate((0, 28)):
            ref = O.global_score(S[0, b].astype(np.float64), H[0, b].astype(np.float64), nh, 0.8, form, n_cand=c)
            np.testing.assert_allclose(F[0, b, :, :c], ref, rtol=3e-7, atol=1e-30)


def test_select_topk_ties_nan_and_brute_force():
    st = _state()
    l, w, k = 40, 4, 28
    c = l - w
    _set_lengths(st, (l, l), step_next=l, decoded=w)
    rng = np.random.default_rng(6)
    F = np.zeros((1, 2, 2, 64), np.float32)
    F[0, 0, 0, :c] = 0.25                                   # all tied: first k indices
    F[0, 0, 1, :c] = np.round(rng.random(c), 1)            # many ties
    F[0, 1, 0, :c] = rng.random(c)
    F[0, 1, 1, :c] = rng.random(c); F[0, 1, 1, 3] = np.nan; F[0, 1, 1, 7] = np.inf; F[0, 1, 1, 9] = -0.0
    st.F.copy_(torch.from_numpy(F))
    st.select_topk(l - 1)
    keep = st.keep_idx.cpu().numpy()
    assert keep[0, 0, 0].tolist() == list(range(k))
    for (b, j) in ((0, 1), (1, 0)):
        ref = O.select_topk(F[0, b, j, :c][None].astype(np.float64), k)[0]
        np.testing.assert_array_equal(keep[0, b, j], ref)
    odd = keep[0, 1, 1]
    assert len(set(odd.tolist())) == k and odd.min() >= 0 and odd.max() < c and (np.diff(odd) > 0).all()
    assert 7 in odd.tolist()


@pytest.mark.parametrize("seed", range(6))
def test_select_topk_random_shapes_signs_and_ties(seed):
    # seeded sweep: budgets/windows/lengths that are not round numbers, negative and tied scores,
    # several decimal granularities; the GPU must equal the oracle's (score desc, index asc) rule
    rng = np.random.default_rng(100 + seed)
    b = int(rng.integers(40, 300)); w = int(rng.integers(1, 33)); s_ = int(rng.integers(max(w, 8), 200))
    cap = (b + s_ + 31) // 32 * 32
    st = _state(budget=b, window=w, interval=s_, capacity=cap, n_q_heads=2, n_kv_heads=2)
    lens = (int(rng.integers(b + 1, b + s_ + 1)), b + s_)
    _set_lengths(st, lens, step_next=1000, decoded=w)
    F = np.zeros((1, 2, 2, cap), np.float32)
    for bb in range(2):
        for j in range(2):
            x = rng.standard_normal(cap).astype(np.float32)
            mode = (seed + bb + 2 * j) % 4
            if mode == 1: x = np.round(x, 1)                      # heavy ties, both signs
            elif mode == 2: x = np.abs(np.round(x, 0))            # a handful of distinct values
            elif mode == 3: x[rng.integers(0, cap, 20)] = 0.0; x[rng.integers(0, cap, 5)] = -0.0
            F[0, bb, j] = x
    st.F.copy_(torch.from_numpy(F))
    st.select_topk(999)
    keep = st.keep_idx.cpu().numpy()
    for bb in range(2):
        c = lens[bb] - w
        for j in range(2):
            ref = O.select_topk(F[0, bb, j, :c][None].astype(np.float64), b - w)[0]
            np.testing.assert_array_equal(keep[0, bb, j], ref)


@pytest.mark.parametrize("pattern", ["front", "back", "alternate", "random"])
@pytest.mark.parametrize("dtype,nt_old", [("f32", 0), ("bf16", 0), ("bf16", 160), ("f32", 96)])
def test_compact_adversarial_keep_patterns(pattern, dtype, nt_old):
    kw = {} if dtype == "f32" else dict(head_dim=128)
    st = _state(dtype, budget=160, window=8, interval=32, capacity=192, **kw)
    b, w, l = 160, 8, 192
    c, k = l - w, b - w
    rng = np.random.default_rng(7)
    if pattern == "front":
        keep = np.arange(c - k, c)
    elif pattern == "back":
        keep = np.arange(k)
    elif pattern == "alternate":
        keep = np.sort(np.concatenate([np.arange(0, 64, 2), np.arange(64, 64 + k - 32)]))
    else:
        keep = np.sort(rng.permutation(c)[:k])
    keep_all = np.broadcast_to(keep, (1, 2, 2, k)).astype(np.int32).copy()
    keep_all[0, 1, 1] = np.sort(rng.permutation(c)[:k])
    K = torch.randn(st.K.shape).to(st.K.dtype); V = torch.randn(st.V.shape).to(st.V.dtype)
    pos = torch.arange(192, dtype=torch.int32).expand(1, 2, 2, 192).contiguous() + 1000
    F = torch.rand(1, 2, 2, 192)
    # the first nt_old rows start in tiled format, the rest row-major (as appended)
    st.K.copy_(k_rows_to_cache(K, nt_old)); st.V.copy_(V); st.pos.copy_(pos); st.F.copy_(F)
    st.keep_idx.copy_(torch.from_numpy(keep_all))
    _set_lengths(st, (l, l), step_next=500, n_tiled=(nt_old, nt_old), decoded=w)
    st.compact(step=499)
    assert st.d_state.cpu().tolist() == [[[b, 500, k, 160], [b, 500, k, 160]]]
    Kr = k_cache_to_rows(st.K, 160).cpu()
    for bb in range(2):
        for j in range(2):
            src = np.concatenate([keep_all[0, bb, j], np.arange(c, l)])
            assert torch.equal(Kr[0, bb, j, :b], K[0, bb, j, src])
            assert torch.equal(st.V[0, bb, j, :b].cpu(), V[0, bb, j, src])
            assert torch.equal(st.pos[0, bb, j, :b].cpu(), pos[0, bb, j, src])
            assert torch.equal(st.F_hist[0, bb, j, :k].cpu(), F[0, bb, j, keep_all[0, bb, j]])
