"""The compression entry point that allocates nothing (gkv_evict_static) against gkv_evict:
same kernels on the library's fixed scratch array instead of caller buffers, so the resulting
cache must be identical bit for bit.  Two calls in a row on the same GPU, the second with a
smaller configuration, so that whatever the first call left in the array is still there."""
import pytest
import torch

from gkv_traces import CONFIGS, Trace
from paper_2512_00504_amd import GkvError
from paper_2512_00504_amd.state import DecodeState

pytestmark = pytest.mark.gpu


def _decode_to_trigger(wl, seed_note=""):
    """A state decoded up to (and including) the step whose trigger compresses, not yet compressed."""
    tr = Trace(wl)
    st = DecodeState.from_workload(wl)
    n = wl.budget + wl.interval
    n = (n + wl.interval - 1) // wl.interval * wl.interval
    q, k, v = [torch.from_numpy(x).to(st.K.dtype).to(st.device) for x in tr.batch_steps(0, n)]
    t_trig = None
    for t in range(n):
        st.attend_decode(q[t], k[t], v[t], t)
        if st.is_trigger(t):
            t_trig = t
            break
    assert t_trig is not None
    return st, t_trig


def _compare(wl):
    st, t = _decode_to_trigger(wl)
    ref = {name: getattr(st, name).clone() for name in ("K", "V", "pos", "F_hist", "d_state")}
    len_host = st.len_host
    st.evict(t)                                           # existing entry point, caller-provided S, F, keep_idx
    torch.cuda.synchronize()
    want = {name: getattr(st, name).clone() for name in ref}
    assert not torch.equal(want["d_state"], ref["d_state"])          # it did compress
    for name, val in ref.items():                         # rewind, then the entry point under test
        getattr(st, name).copy_(val)
    st.S.fill_(-1.0); st.F.fill_(-1.0); st.keep_idx.fill_(-1)       # it must not touch the caller's buffers
    st.ctx.evict_static(st.qwin, st.K, st.V, st.F_hist, st.pos, st.d_state, t, len_host, st.workspace)
    torch.cuda.synchronize()
    for name in ref:
        got = getattr(st, name)
        assert torch.equal(got.view(torch.uint8), want[name].view(torch.uint8)), name
    assert (st.S == -1.0).all() and (st.F == -1.0).all() and (st.keep_idx == -1).all()


def test_evict_static_matches_evict_twice_second_call_smaller():
    print("gkv_evict_static vs gkv_evict: cfg3 head shape, 3 layers x 2 sequences", flush=True)
    _compare(CONFIGS["cfg3_28layer_b512"].with_(n_layers=3, batch=2))
    print("gkv_evict_static vs gkv_evict: tiny fp32 shape, second call on the same array", flush=True)
    _compare(CONFIGS["cfg1_tiny"])


def test_evict_static_rejects_configurations_beyond_the_array():
    wl = CONFIGS["cfg5_large_batch"].with_(n_layers=8)          # 4096 units x 1088 rows: 38 MB of scores
    st = DecodeState.from_workload(wl.with_(n_layers=1, batch=1))
    from paper_2512_00504_amd import Context, make_config
    big = Context(make_config(wl.n_layers, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.budget,
                              wl.window, wl.interval, wl.capacity, wl.dtype))
    with pytest.raises(GkvError) as e:                          # refused on the host: pointers never used
        big.evict_static(st.qwin, st.K, st.V, st.F_hist, st.pos, st.d_state, 0, 0, st.workspace)
    assert e.value.status == 7
