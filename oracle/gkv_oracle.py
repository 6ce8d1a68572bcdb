"""fp64 CPU oracle of the G-KV decode/evict path.  TEST INFRASTRUCTURE ONLY.

A plain, slow restatement of what the paper defines, written from the paper
and sharing no code with the HIP path.  Only the tests, the smoke check and
the benchmark's cpu_baseline leg may import this module; the product path
never does.

Notation (Preliminary section): h_q query heads, h_kv KV heads, g = h_q/h_kv,
d head dim, l cache length, b budget, w observation-window size, s compression
interval, alpha memory-decay rate, S local score, F global score.  Query head
i reads KV head j = i // g.

Readings taken where the paper is silent (each is a switch or a comment here):
  * window rows are causal: window query k (k-th oldest of the last w) is
    normalised over cache entries [0, l-w+k], i.e. exactly the keys it saw
    when it was decoded; `causal_window=False` gives the unmasked variant;
  * the w window entries are always kept and never compete; the l-w others
    are the candidates, of which b-w are kept;
  * max_j in the normalisation runs over the candidates (`norm_over="all"`
    takes it over all l columns instead);
  * compression runs after step t when (t+1) % s == 0 and l > b, and only once w queries
    have been decoded since the cache was loaded (the observation window consists of
    generated tokens; a prompt brings keys and values but no window queries);
  * a prompt is P rows appended before decoding starts; in a batch every sequence shares the
    step counter, so a sequence with a shorter prompt simply starts with a shorter cache
    (its prompt occupies the positions just before the first decode step);
  * at the first compression there is no history (n_hist = 0) and the
    recorded history is the normalised score of the kept entries;
  * kept entries are stored in ascending original position, then the window;
  * ties in the top-k: higher score first, then lower index;
  * redundancy score (the paper gives no threshold, recency rule or diagonal
    rule): see redundancy_score(); with it, selection uses lam*F - (1-lam)*R'
    while the recorded history stays the global score F.  Parity unpinned
    against the authors' settings; pinned here by closed forms and brute force.

Pins: tests/test_oracle_pins.py (closed forms, hand-derived fixtures under
tests/golden/, brute force, invariants).  Every function below has a pin.
"""
from __future__ import annotations

import numpy as np

COMBINE_FORMS = ("max", "avg", "sum")


# --------------------------------------------------------------------------
# building blocks
# --------------------------------------------------------------------------
def softmax(z: np.ndarray) -> np.ndarray:
    """Softmax of a 1-D fp64 vector (row max subtracted first)."""
    z = np.asarray(z, dtype=np.float64)
    e = np.exp(z - z.max())
    return e / e.sum()


def attend(q, K, V, length, scale=None):
    """Decode attention of the newest query over the first `length` cache rows.

    q [h_q, d]; K, V [h_kv, >=length, d].  Returns o [h_q, d] (fp64).
    Ordinary softmax attention; entries that were evicted are simply absent
    (Section "Enhancing KV Cache Compression through Training", sparse-mask
    figure).
    """
    q = np.asarray(q, np.float64); K = np.asarray(K, np.float64); V = np.asarray(V, np.float64)
    h_q, d = q.shape
    h_kv = K.shape[0]
    g = h_q // h_kv
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    o = np.zeros((h_q, d))
    for i in range(h_q):
        j = i // g
        p = softmax((K[j, :length] @ q[i]) * scale)
        o[i] = p @ V[j, :length]
    return o


def window_probs(Qwin, K, length, scale=None, causal_window=True):
    """Attention probabilities of the observation window (Preliminary, Eq. 1).

    Qwin [h_q, w, d], row k = k-th oldest of the last w queries; K [h_kv, >=l, d].
    Returns A [h_q, w, l]; with `causal_window`, row k covers cache entries
    [0, l-w+k] and is zero beyond.
    """
    Qwin = np.asarray(Qwin, np.float64); K = np.asarray(K, np.float64)
    h_q, w, d = Qwin.shape
    h_kv = K.shape[0]
    g = h_q // h_kv
    l = int(length)
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    A = np.zeros((h_q, w, l))
    for i in range(h_q):
        j = i // g
        for k in range(w):
            n_vis = l - w + k + 1 if causal_window else l
            A[i, k, :n_vis] = softmax((K[j, :n_vis] @ Qwin[i, k]) * scale)
    return A


def local_score(A, h_kv):
    """Local score S [h_kv, l]: max over the query heads of each KV group,
    then the mean over the w window rows (Preliminary, Eq. 2)."""
    h_q, w, l = A.shape
    g = h_q // h_kv
    A_grp = A.reshape(h_kv, g, w, l).max(axis=1)        # A' [h_kv, w, l]
    return A_grp.sum(axis=1) / w


def global_score(S, F_hist, n_hist, alpha, form="max", n_cand=None, norm_over="candidates"):
    """Global score F_t over the candidates (Section 4, the three forms).

    S [h_kv, l] local score; the first n_cand columns are candidates
    (default: all).  F_hist [h_kv, >=n_hist] history of the first n_hist
    candidates.  S is normalised by its per-head maximum; entries with
    history combine it with alpha * F_hist, the others take it unchanged.
    Returns F [h_kv, n_cand].
    """
    S = np.asarray(S, np.float64)
    n_cand = S.shape[1] if n_cand is None else n_cand
    if norm_over == "candidates":
        m = S[:, :n_cand].max(axis=1, keepdims=True)
    elif norm_over == "all":
        m = S.max(axis=1, keepdims=True)
    else:
        raise ValueError(norm_over)
    Sn = S[:, :n_cand] / m
    F = Sn.copy()
    if n_hist > 0:
        H = np.asarray(F_hist, np.float64)[:, :n_hist]
        if form == "max":
            F[:, :n_hist] = np.maximum(alpha * H, Sn[:, :n_hist])
        elif form == "avg":
            F[:, :n_hist] = alpha * H + (1.0 - alpha) * Sn[:, :n_hist]
        elif form == "sum":
            F[:, :n_hist] = alpha * H + Sn[:, :n_hist]
        else:
            raise ValueError(form)
    return F


def select_topk(F, k):
    """Ascending indices of the k largest entries of each row of F [h_kv, c];
    among equal scores the lower index wins (Preliminary: top-(b-w) per head)."""
    F = np.asarray(F, np.float64)
    h_kv, c = F.shape
    keep = np.zeros((h_kv, k), dtype=np.int64)
    idx = np.arange(c)
    for j in range(h_kv):
        order = np.lexsort((idx, -F[j]))        # primary: score descending; secondary: index ascending
        keep[j] = np.sort(order[:k])
    return keep


def pool_scores(F, kernel):
    """Sequence-wise max-pooling of a score over the candidates, the SnapKV-style plug-in the
    appendix applies to the global score: out[n] = max F[m] for |m - n| <= kernel // 2, clipped at
    the ends.  The paper does not give the kernel size (parameter; odd sizes are symmetric)."""
    F = np.asarray(F, np.float64)
    h, c = F.shape
    half = kernel // 2
    out = np.empty_like(F)
    for n in range(c):
        out[:, n] = F[:, max(0, n - half):min(c, n + half + 1)].max(axis=1)
    return out


def redundancy_score(K, length, tau=0.5, n_recent=0, eps=1e-8, return_margin=False, return_parts=False):
    """Redundancy score R [h_kv, l] of the cached keys (appendix "Integrating the Global Score
    with Other Methods"): keys normalised to K/(||K||_2 + eps), cosine-similarity matrix C,
    entries below the threshold tau set to zero as well as those of the most recent tokens,
    column sums, softmax over the l columns.

    Readings (the paper gives neither the threshold nor the recent-token rule): an entry is
    kept when C >= tau; the diagonal (a key with itself) is zeroed; "most recent tokens" zeroes
    the columns of the last n_recent rows, so those tokens collect no redundancy.

    return_margin adds, per head, the smallest |C - tau| over the entries that count (how far
    the yes/no decisions were from the threshold).  return_parts adds the intermediates
    dict(C=[h_kv,l,l] cosines, col=[h_kv,l] column sums) so that a checker can see which
    entries sit on the threshold.
    """
    K = np.asarray(K, np.float64)
    l = int(length)
    h = K.shape[0]
    R = np.zeros((h, l))
    margin = np.full(h, np.inf)
    C_all = np.zeros((h, l, l))
    col_all = np.zeros((h, l))
    for j in range(h):
        Kj = K[j, :l]
        Kn = Kj / (np.linalg.norm(Kj, axis=1, keepdims=True) + eps)
        C = Kn @ Kn.T
        Cm = np.where(C >= tau, C, 0.0)
        np.fill_diagonal(Cm, 0.0)
        if n_recent > 0:
            Cm[:, l - n_recent:] = 0.0
        col = Cm.sum(axis=0)
        R[j] = softmax(col)
        off = np.abs(C - tau) + np.eye(l) * 10.0
        margin[j] = off[:, :l - n_recent].min() if l > n_recent else np.inf
        C_all[j], col_all[j] = C, col
    out = (R,)
    if return_margin:
        out += (margin,)
    if return_parts:
        out += (dict(C=C_all, col=col_all),)
    return out if len(out) > 1 else R


def combine_redundancy(F, R, lam, n_cand=None):
    """F' = lam * F - (1 - lam) * R / max_j R over the candidates (same appendix).
    F [h_kv, >=n_cand], R [h_kv, l]; the maximum runs over all l columns."""
    F = np.asarray(F, np.float64); R = np.asarray(R, np.float64)
    n_cand = F.shape[1] if n_cand is None else n_cand
    Rn = R / R.max(axis=1, keepdims=True)
    return lam * F[:, :n_cand] - (1.0 - lam) * Rn[:, :n_cand]


# --------------------------------------------------------------------------
# oracle A: compacting cache, the state machine the HIP path mirrors
# --------------------------------------------------------------------------
class OracleA:
    """One (layer, sequence) pair: all h_kv heads, compacted cache."""

    def __init__(self, h_q, h_kv, d, budget, window, interval, capacity=None,
                 alpha=0.8, form="max", scale=None, causal_window=True,
                 norm_over="candidates", redundancy=None):
        """redundancy: None, or dict(lam=, tau=, n_recent=, eps=) to select on
        lam*F - (1-lam)*R' (the combination the paper calls G-KV); the recorded history stays F."""
        assert h_q % h_kv == 0 and window <= interval and window < budget
        self.h_q, self.h_kv, self.d = h_q, h_kv, d
        self.b, self.w, self.s = budget, window, interval
        self.cap = budget + interval if capacity is None else capacity
        assert self.cap >= budget + interval
        self.alpha, self.form = alpha, form
        self.scale = 1.0 / np.sqrt(d) if scale is None else scale
        self.causal_window, self.norm_over = causal_window, norm_over
        self.redundancy = redundancy
        self.K = np.zeros((h_kv, self.cap, d))
        self.V = np.zeros((h_kv, self.cap, d))
        self.F_hist = np.zeros((h_kv, self.cap))
        self.pos = np.full((h_kv, self.cap), -1, dtype=np.int64)
        self.len = 0
        self.n_hist = 0
        self.q_recent = []           # the last w queries, oldest first
        self.events = []             # one dict of intermediates per compression

    # -- every decode step ---------------------------------------------------
    def append(self, t, q, k, v):
        n = self.len
        self.K[:, n] = k; self.V[:, n] = v; self.pos[:, n] = t
        self.len = n + 1
        self.q_recent.append(np.asarray(q, np.float64))
        self.q_recent = self.q_recent[-self.w:]

    def prefill(self, t_first, k, v):
        """Prompt of P tokens (k, v [P, h_kv, d]) at positions t_first .. t_first+P-1: rows are
        appended, nothing attends and no window query is recorded."""
        k = np.asarray(k, np.float64); v = np.asarray(v, np.float64)
        for i in range(k.shape[0]):
            n = self.len
            self.K[:, n] = k[i]; self.V[:, n] = v[i]; self.pos[:, n] = t_first + i
            self.len = n + 1

    def is_trigger(self, t):
        """After step t: every s steps, once the cache exceeds the budget and the window is full."""
        return (t + 1) % self.s == 0 and self.len > self.b and len(self.q_recent) >= self.w

    def step(self, t, q, k, v):
        """Append (k, v), attend with q, then compress if this step is a trigger."""
        self.append(t, q, k, v)
        o = attend(q, self.K, self.V, self.len, self.scale)
        if self.is_trigger(t):
            self.compress()
        return o

    # -- every s steps -------------------------------------------------------
    def qwin(self):
        return np.stack(self.q_recent, axis=1)          # [h_q, w, d]

    def score(self):
        """(S over all l columns, F over the l-w candidates)."""
        l, c = self.len, self.len - self.w
        A = window_probs(self.qwin(), self.K, l, self.scale, self.causal_window)
        S = local_score(A, self.h_kv)
        F = global_score(S, self.F_hist, self.n_hist, self.alpha, self.form,
                         n_cand=c, norm_over=self.norm_over)
        return S, F

    def compress(self):
        l, b, w = self.len, self.b, self.w
        c = l - w
        S, F = self.score()
        ev = dict(len=l, n_hist=self.n_hist, S=S[:, :c].copy(), F=F.copy())
        if self.redundancy is None:
            keep = select_topk(F, b - w)
        else:
            rp = self.redundancy
            R, margin, parts = redundancy_score(self.K, l, rp["tau"], rp["n_recent"], rp.get("eps", 1e-8),
                                                return_margin=True, return_parts=True)
            Fsel = combine_redundancy(F, R, rp["lam"], n_cand=c)
            keep = select_topk(Fsel, b - w)
            ev.update(R=R, Fsel=Fsel, tau_margin=margin, C=parts["C"], col=parts["col"])
        ev["keep"] = keep.copy()
        # eviction log: original positions of the candidates that are dropped (Section 5)
        ev["evicted_pos"] = [sorted(set(self.pos[j, :c].tolist()) - set(self.pos[j, keep[j]].tolist()))
                             for j in range(self.h_kv)]
        self.events.append(ev)
        K, V, pos = self.K.copy(), self.V.copy(), self.pos.copy()
        for j in range(self.h_kv):
            kj = keep[j]
            self.K[j, :b - w] = K[j, kj]; self.V[j, :b - w] = V[j, kj]
            self.pos[j, :b - w] = pos[j, kj]
            self.F_hist[j, :b - w] = F[j, kj]
            self.K[j, b - w:b] = K[j, c:l]; self.V[j, b - w:b] = V[j, c:l]
            self.pos[j, b - w:b] = pos[j, c:l]
        self.K[:, b:] = 0.0; self.V[:, b:] = 0.0; self.pos[:, b:] = -1
        self.F_hist[:, b - w:] = 0.0
        self.len = b
        self.n_hist = b - w


# --------------------------------------------------------------------------
# oracle B: never moves data; an alive-set over the full history
# --------------------------------------------------------------------------
class OracleB:
    """Same method, stated as a sparse attention mask over the full history:
    an evicted position is invisible to every later token (sparse-mask figure).
    Bookkeeping is by original position, in dicts and sets; nothing is gathered."""

    def __init__(self, h_q, h_kv, d, budget, window, interval, alpha=0.8, form="max",
                 scale=None):
        self.h_q, self.h_kv, self.d = h_q, h_kv, d
        self.g = h_q // h_kv
        self.b, self.w, self.s = budget, window, interval
        self.alpha, self.form = alpha, form
        self.scale = 1.0 / np.sqrt(d) if scale is None else scale
        self.q_all, self.k_all, self.v_all = {}, {}, {}  # position -> vectors (prompt positions have no q)
        self.alive = [set() for _ in range(h_kv)]
        self.hist = [dict() for _ in range(h_kv)]       # position -> recorded global score
        self.kept_log = []                              # per event: per head sorted kept positions

    def _probs(self, q_vec, j, positions):
        z = np.array([np.dot(self.k_all[p][j], q_vec) for p in positions]) * self.scale
        return softmax(z)

    def prefill(self, t_first, k, v):
        for i in range(len(k)):
            p = t_first + i
            self.k_all[p] = np.asarray(k[i], np.float64); self.v_all[p] = np.asarray(v[i], np.float64)
            for j in range(self.h_kv):
                self.alive[j].add(p)

    def step(self, t, q, k, v):
        q = np.asarray(q, np.float64); k = np.asarray(k, np.float64); v = np.asarray(v, np.float64)
        self.q_all[t] = q; self.k_all[t] = k; self.v_all[t] = v
        o = np.zeros((self.h_q, self.d))
        for j in range(self.h_kv):
            self.alive[j].add(t)
            positions = sorted(self.alive[j])
            for i in range(j * self.g, (j + 1) * self.g):
                p = self._probs(q[i], j, positions)
                for pn, n in zip(p, positions):
                    o[i] += pn * self.v_all[n][j]
        win = range(t - self.w + 1, t + 1)
        if (t + 1) % self.s == 0 and len(self.alive[0]) > self.b and all(p in self.q_all for p in win):
            self._compress(t)
        return o

    def _compress(self, t):
        w, b, g = self.w, self.b, self.g
        kept_all = []
        for j in range(self.h_kv):
            win = list(range(t - w + 1, t + 1))
            cand = sorted(self.alive[j] - set(win))
            score = {n: 0.0 for n in cand}
            for tq in win:
                visible = [n for n in sorted(self.alive[j]) if n <= tq]
                best = {n: 0.0 for n in cand}
                for i in range(j * g, (j + 1) * g):
                    p = self._probs(self.q_all[tq][i], j, visible)
                    for pn, n in zip(p, visible):
                        if n in best and pn > best[n]:
                            best[n] = pn
                for n in cand:
                    score[n] += best[n] / w
            top = max(score.values())
            glob = {}
            for n in cand:
                sn = score[n] / top
                if n in self.hist[j]:
                    h = self.alpha * self.hist[j][n]
                    glob[n] = (max(h, sn) if self.form == "max" else
                               h + (1.0 - self.alpha) * sn if self.form == "avg" else h + sn)
                else:
                    glob[n] = sn
            ranked = sorted(cand, key=lambda n: (-glob[n], n))
            kept = sorted(ranked[:b - w])
            self.hist[j] = {n: glob[n] for n in kept}
            self.alive[j] = set(kept) | set(win)
            kept_all.append(kept)
        self.kept_log.append(kept_all)
