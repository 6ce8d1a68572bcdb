"""One compression cycle (s decode steps + the compression) recorded into a HIP graph through the
C ABI and replayed: the step number comes from a device-side step base, so the recorded launches
are valid for every cycle.  Each replay is checked against the eager run of the same steps, with
eager work and synchronisations between the replays."""
import pytest
import torch

from gkv_traces import CONFIGS, Trace
from paper_2512_00504_amd.state import DecodeState

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,over", [
    ("cfg3_28layer_b512", dict(n_layers=2, batch=2)),                    # matrix-core kernels
    ("cfg1_tiny", dict(budget=64, interval=16, window=8)),               # plain kernels, fp32
])
def test_recorded_cycle_replays_match_eager_steps(name, over):
    wl = CONFIGS[name].with_(**over)
    s, b, w = wl.interval, wl.budget, wl.window
    assert b % s == 0 and s % w == 0
    n_cycles = 3
    t0 = b + s                                   # first steady-state step: after the first compression
    T = t0 + n_cycles * s
    tr = Trace(wl)
    dt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    q, k, v = [torch.from_numpy(x).to(dt).cuda() for x in tr.batch_steps(0, T)]

    # eager reference: absolute steps, ordinary calls
    ref = DecodeState.from_workload(wl)
    outs_ref = []
    for t in range(T):
        outs_ref.append(ref.attend_decode(q[t], k[t], v[t], t).clone())
        if ref.is_trigger(t):
            ref.evict(t)
    torch.cuda.synchronize()

    # the graph path: eager up to the steady state, then one recorded cycle replayed n_cycles times
    st = DecodeState.from_workload(wl)
    for t in range(t0):
        st.attend_decode(q[t], k[t], v[t], t)
        if st.is_trigger(t):
            st.evict(t)
    base = torch.tensor([t0], dtype=torch.int32, device="cuda")
    st.ctx.set_step_base(base)
    q_in, k_in, v_in = q[t0:t0 + s].clone(), k[t0:t0 + s].clone(), v[t0:t0 + s].clone()   # static inputs of the graph
    out_buf = torch.zeros((s,) + tuple(st.out.shape), dtype=dt, device="cuda")            # one output slot per step

    def cycle():
        for i in range(s):                        # relative steps 0 .. s-1; len_max_host = b + i
            st.ctx.attend_decode(q_in[i], k_in[i], v_in[i], st.K, st.V, st.pos, i, st.qwin, st.d_state,
                                 b + i, out_buf[i], st.workspace)
        st.ctx.evict(st.qwin, st.K, st.V, st.F_hist, st.pos, st.d_state, s - 1, b + s, st.S, st.F, st.keep_idx,
                     st.workspace)
        st.ctx.advance_step_base(s)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        cycle()
    torch.cuda.synchronize()
    assert int(base.item()) == t0                 # recording executes nothing

    for c in range(n_cycles):
        lo = t0 + c * s
        q_in.copy_(q[lo:lo + s]); k_in.copy_(k[lo:lo + s]); v_in.copy_(v[lo:lo + s])      # eager work between replays
        out_buf.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert int(base.item()) == lo + s
        for i in range(s):
            assert torch.equal(out_buf[i].view(torch.uint8), outs_ref[lo + i].view(torch.uint8)), f"cycle {c} step {i}"
    for name_ in ("K", "V", "pos", "F_hist", "d_state", "keep_idx"):
        assert torch.equal(getattr(st, name_).view(torch.uint8), getattr(ref, name_).view(torch.uint8)), name_
