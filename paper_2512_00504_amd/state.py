"""Device buffers for one decode job, allocated through torch, plus the K-layout
permutations.  No arithmetic of the method lives here: each method below is one
call into the C ABI."""
from __future__ import annotations

import torch

from .binding import ST_LEN, ST_LEN_STEP, ST_N_HIST, ST_N_TILED, Context, GkvConfig, make_config

_TORCH_DTYPE = {0: torch.float32, 1: torch.bfloat16}


def k_rows_to_cache(K_rows: torch.Tensor, n_tiled: int) -> torch.Tensor:
    """[..., cap, d] row-major -> the library's K layout with the first n_tiled rows tiled."""
    n_tiled = n_tiled // 16 * 16
    out = K_rows.clone()
    if n_tiled:
        *lead, cap, d = K_rows.shape
        epc = 16 // K_rows.element_size()
        t = K_rows[..., :n_tiled, :].reshape(*lead, n_tiled // 16, 16, d // epc, epc)
        n = len(lead)
        t = t.permute(*range(n), n, n + 2, n + 1, n + 3).contiguous()
        out[..., :n_tiled, :] = t.reshape(*lead, n_tiled, d)
    return out


def k_cache_to_rows(K_cache: torch.Tensor, n_tiled: int) -> torch.Tensor:
    """Inverse of k_rows_to_cache."""
    n_tiled = n_tiled // 16 * 16
    out = K_cache.clone()
    if n_tiled:
        *lead, cap, d = K_cache.shape
        epc = 16 // K_cache.element_size()
        t = K_cache[..., :n_tiled, :].reshape(*lead, n_tiled // 16, d // epc, 16, epc)
        n = len(lead)
        t = t.permute(*range(n), n, n + 2, n + 1, n + 3).contiguous()
        out[..., :n_tiled, :] = t.reshape(*lead, n_tiled, d)
    return out


class DecodeState:
    """All device state of the path for L layers x B sequences."""

    def __init__(self, cfg: GkvConfig, device="cuda:0", params=None):
        self.cfg = cfg
        self.ctx = Context(cfg)
        for name, val in (params or {}).items():
            self.ctx.set_param(name, val)
        L, B, Hq, Hkv, d = cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
        cap, w, b = cfg.capacity, cfg.window, cfg.budget
        dt = _TORCH_DTYPE[cfg.dtype]
        dev = torch.device(device)
        self.device = dev
        z = lambda *s, dtype: torch.zeros(*s, dtype=dtype, device=dev)
        self.K = z(L, B, Hkv, cap, d, dtype=dt)          # rows below N_TILED tiled, the rest row-major
        self.V = z(L, B, Hkv, cap, d, dtype=dt)
        self.pos = torch.full((L, B, Hkv, cap), -1, dtype=torch.int32, device=dev)
        self.qwin = z(w, L, B, Hq, d, dtype=dt)          # ring of the last w q tensors
        self.d_state = z(L, B, 4, dtype=torch.int32)     # {len, len_step, n_hist, n_tiled}
        self.F_hist = z(L, B, Hkv, cap, dtype=torch.float32)
        self.S = z(L, B, Hkv, cap, dtype=torch.float32)
        self.F = z(L, B, Hkv, cap, dtype=torch.float32)
        self.R = z(L, B, Hkv, cap, dtype=torch.float32)      # normalised redundancy score
        self.F_sel = z(L, B, Hkv, cap, dtype=torch.float32)  # lambda*F - (1-lambda)*R'
        self.keep_idx = z(L, B, Hkv, b - w, dtype=torch.int32)
        self.evicted = torch.full((L, B, Hkv, cap - b), -1, dtype=torch.int32, device=dev)
        self.out = z(L, B, Hq, d, dtype=dt)
        self.workspace = torch.zeros(self.ctx.workspace_bytes(), dtype=torch.uint8, device=dev)
        self.ctx.workspace_init(self.workspace)
        # host mirror of the device records, for launch sizing and the trigger only: per sequence,
        # the cache length and the steps decoded since the cache was loaded or last compacted
        self._len = [0] * B
        self._since = [0] * B

    @classmethod
    def from_workload(cls, wl, device="cuda:0", params=None, **over):
        kw = dict(n_layers=wl.n_layers, batch=wl.batch, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads,
                  head_dim=wl.head_dim, budget=wl.budget, window=wl.window, interval=wl.interval,
                  capacity=wl.capacity, dtype=wl.dtype, combine=wl.combine, alpha=wl.alpha)
        kw.update(over)
        return cls(make_config(**kw), device=device, params=params)

    @property
    def len_host(self) -> int:
        """Upper bound of every sequence's length, as the calls' len_max_host wants it."""
        return max(self._len)

    @len_host.setter
    def len_host(self, value: int):
        """Declare every sequence `value` rows long with a full observation window."""
        self._len = [int(value)] * self.cfg.batch
        self._since = [self.cfg.window] * self.cfg.batch

    # lengths as the kernels see them ---------------------------------------------------------
    def lengths(self, next_step: int) -> torch.Tensor:
        """[L,B] cache lengths before decode step `next_step` (LEN + next_step - LEN_STEP)."""
        return self.d_state[..., ST_LEN] + (next_step - self.d_state[..., ST_LEN_STEP])

    def set_state(self, length, len_step, n_hist, n_tiled):
        """Fill every (layer, sequence) record with the same values."""
        self.d_state[..., ST_LEN] = length
        self.d_state[..., ST_LEN_STEP] = len_step
        self.d_state[..., ST_N_HIST] = n_hist
        self.d_state[..., ST_N_TILED] = n_tiled
        self._len = [int(length)] * self.cfg.batch
        self._since = [0] * self.cfg.batch

    def load_prefix(self, k, v, t0=0):
        """Place tokens t0..t0+n-1 (k, v: [n, L, B, h_kv, d]) as cache rows 0..n-1 with positions
        t0..t0+n-1, K row-major (N_TILED = 0).  For n <= budget this is exactly the state n
        appending decode steps leave behind (nothing is evicted before the cache exceeds the
        budget); pure data placement."""
        n = k.shape[0]
        assert n <= self.cfg.budget
        self.K.zero_(); self.V.zero_()
        self.K[..., :n, :] = k.to(self.V.dtype).permute(1, 2, 3, 0, 4)
        self.V[..., :n, :] = v.to(self.V.dtype).permute(1, 2, 3, 0, 4)
        self.pos.fill_(-1)
        self.pos[..., :n] = torch.arange(t0, t0 + n, dtype=torch.int32, device=self.device)
        self.set_state(n, t0 + n, 0, 0)

    def load_prompt_rows(self, t_first, k, v, t0, prompt_lens):
        """Place prompt tokens.  k, v [n, L, B, h_kv, d] hold positions t_first .. t_first+n-1 of
        every sequence's token stream; sequence i's prompt is the positions [t0 - P_i, t0) (a
        left-padded batch: decoding starts at step t0 for everyone) and goes to cache rows
        [0, P_i), K row-major.  May be called chunk by chunk; finish with begin_decode().
        Pure data placement."""
        n = k.shape[0]
        for i, P in enumerate(prompt_lens):
            lo = max(t_first, t0 - P)
            hi = min(t_first + n, t0)
            if hi <= lo:
                continue
            r0 = lo - (t0 - P)
            src = slice(lo - t_first, hi - t_first)
            self.K[:, i, :, r0:r0 + hi - lo] = k[src, :, i].to(self.K.dtype).permute(1, 2, 0, 3)
            self.V[:, i, :, r0:r0 + hi - lo] = v[src, :, i].to(self.V.dtype).permute(1, 2, 0, 3)
            self.pos[:, i, :, r0:r0 + hi - lo] = torch.arange(lo, hi, dtype=torch.int32, device=self.device)

    def begin_decode(self, t0, prompt_lens):
        """Records {P_i, t0, 0, 0}: sequence i holds P_i prompt rows before decode step t0."""
        rec = torch.tensor([[P, t0, 0, 0] for P in prompt_lens], dtype=torch.int32)
        self.d_state.copy_(rec.to(self.device).expand(self.cfg.n_layers, -1, -1))
        self._len = [int(P) for P in prompt_lens]
        self._since = [0] * self.cfg.batch

    def _after_compression(self):
        """Host mirror of what the compression kernels decide per sequence."""
        b, w = self.cfg.budget, self.cfg.window
        for i in range(self.cfg.batch):
            if self._len[i] > b and self._since[i] >= w:
                self._len[i], self._since[i] = b, 0

    # one call each -------------------------------------------------------------------------
    def attend_decode(self, q, k_new, v_new, step):
        self.ctx.attend_decode(q, k_new, v_new, self.K, self.V, self.pos, step, self.qwin, self.d_state,
                               self.len_host, self.out, self.workspace)
        if k_new is not None:
            self._len = [x + 1 for x in self._len]
        self._since = [x + 1 for x in self._since]
        return self.out

    def score_window(self, step):
        self.ctx.score_window(self.qwin, self.K, self.d_state, step, self.len_host, self.S, self.workspace)

    def global_update(self, step):
        self.ctx.global_update(self.S, self.F_hist, self.d_state, step, self.len_host, self.F)

    def redundancy_combine(self, step, lam, tau, n_recent, eps=1e-8):
        self.ctx.redundancy_combine(self.K, self.d_state, step, self.len_host, self.F, lam, tau, eps, n_recent,
                                    self.R, self.F_sel, self.workspace)

    def select_topk(self, step, on_combined=False):
        self.ctx.select_topk(self.F_sel if on_combined else self.F, self.d_state, step, self.len_host,
                             self.keep_idx, self.workspace)

    def evicted_positions(self, step):
        """Eviction log of this compression; call between select_topk and compact."""
        self.ctx.evicted_positions(self.keep_idx, self.pos, self.d_state, step, self.evicted)

    def compact(self, step):
        self.ctx.compact(self.keep_idx, self.F, self.K, self.V, self.F_hist, self.pos, self.d_state, step,
                         self.workspace)
        self._after_compression()

    def evict(self, step):
        self.ctx.evict(self.qwin, self.K, self.V, self.F_hist, self.pos, self.d_state, step,
                       self.len_host, self.S, self.F, self.keep_idx, self.workspace)
        self._after_compression()

    def is_trigger(self, step) -> bool:
        """Host-side trigger: compression after every s generated tokens, if some sequence is above
        the budget with a full observation window (the kernels skip the others)."""
        b, w = self.cfg.budget, self.cfg.window
        return (step + 1) % self.cfg.interval == 0 and any(
            n > b and k >= w for n, k in zip(self._len, self._since))
