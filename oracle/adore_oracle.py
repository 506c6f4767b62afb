"""CPU oracle for ADORE's per-step decode path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 implementation of what one decode step computes, written
from the paper's definitions (arXiv 2407.02328): sparse single-query attention
over the retained rows (Sec. 2.1, Eq. 1 and the unnumbered "target" equation),
the controller score (Sec. 2.2, Eq. 2 and App. "Implementation Details"), the
release of the lowest-scored rows (Sec. 2.2), the choice of the top-R released
tokens (Sec. 2.3) and the re-projection of their K/V states (Sec. 2.3).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this module.  It shares no code with the HIP path and must never be used as a
fallback for it.

Every function below is pinned by a CPU test against something other than
itself (a library routine, a closed form, brute force or an invariant); none
is "parity unpinned".  What cannot be pinned at all are the paper's numeric
results on real text (datasets, fine-tuned backbone and trained controller
are not available).

Readings of points the paper leaves open (each used exactly as stated here):
  * K physical slots = m persistent rows + R rebuilt rows + the current token
    (Sec. 2.3: K/V of (m+R+1) x d).
  * Heads are independent and the softmax scale uses the head dimension.
  * The GRU is the textbook cell with the reset gate applied to the recurrent
    pre-activation (the variant common libraries implement), z_{-1} = 0.
  * Position feature of token i is the scalar i * pos_scale fed to a 1 -> d'
    fully connected layer (App. "Implementation Details", position layer).
  * sigma_i is computed once, when token i arrives, and never changes
    (Eq. 2 carries no dependence on the current step).  The other reading of
    Sec. 2.2 and the caption of Fig. 2 (the controller rates every cached
    token "for the current token") is the `rescore` mode: at step n every
    token i <= n is scored again from its stored GRU state z_i with the
    RELATIVE position (n - i) * pos_scale in place of i * pos_scale, and
    both selections of that step use the new values.
  * The current token is not released in its own step (Sec. 2.2: an "older"
    state is removed).
  * Tokens released in this step may be rebuilt in this step (Sec. 2.3).
  * Ties on sigma are broken in favour of the lower position.
  * Rebuild forward (Sec. 2.3 read in full: the rebuilt tokens are queries too and their
    outputs feed the next layer): the paper prints no mask for the R+1 query rows; here a
    row at position p attends to the cache rows at positions <= p (a decoder's causal
    rule), so that a rebuilt state equals the state the token had when it was first
    computed whenever all earlier tokens are present.  A layer is attention only:
    x' = x + W_o . concat_h(attention output); norms and the feed-forward block belong to
    the backbone, which is not available.  q, k, v, the attention output and x' are each
    rounded once to the storage type.  K/V of the rebuilt tokens are written at the start
    of the step that uses them (layer by layer), not at the end of the step that chose
    them; the choice itself is unchanged.
  * Rotary position embedding (the paper names it only in its related work on length
    extrapolation, but the backbones it evaluates rotate q and k by the token's position
    before the product, so a key that is rebuilt from a hidden state has to be rotated to the
    position the token had, or it cannot stand next to the cached keys): optional, off when
    `rope_base` is 0.  The pairing is the half-split one (element j < d/2 of a head and
    element j + d/2 span a plane that is turned by pos * rope_base**(-2j/d)).  As in those
    backbones the projection leaves the matrix product in the storage type and the
    rotation works on that: a rotated row is rounded twice, once as a projection and once
    after the rotation.  Keys and queries the caller supplies are taken as they are.  In the rebuild forward the
    queries of the R+1 rows are rotated as well.
  * Top-K attention over a whole sequence (Sec. 2.1: computing the full weights and keeping
    the highest is the ideal sparsity; Sec. 2.2, first strategy, and App. "Implementation
    Details": the backbone is fine-tuned with attention whose weights outside the top K are
    masked out): causal, per head; the K largest products q_i . k_j over j <= i are kept (all
    of them while i + 1 <= K), equal products go to the lower position, the softmax runs over
    the kept ones only (masking before the softmax, as an attention mask does).
  * H2O(Rebuilt) (Sec. 3.1, baselines): see AdoreH2OOracle for the reading of the two sentences the paper
    spends on it (per-head cumulative attention as the score, per-sequence rebuild on the sum over heads).
  * Rows never move: a released row frees its slot; incoming rows take the
    lowest free slots (rebuilt rank rho -> rho-th lowest free slot; the next
    token -> lowest free slot at its insert).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------
# storage rounding
# --------------------------------------------------------------------------
def round_to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """One round-to-nearest-even from fp64 to the storage type, returned as fp64."""
    a = np.asarray(a, dtype=F64)
    if dtype == "f32":
        return a.astype(np.float32).astype(F64)
    if dtype == "bf16":
        # bf16: 8 significand bits, exponent range of fp32.
        mant, exp = np.frexp(a)                    # a = mant * 2**exp, 0.5 <= |mant| < 1
        exp = np.maximum(exp, -125)                # below that: fixed (subnormal) spacing
        mant = a / np.ldexp(1.0, exp)
        return np.ldexp(np.rint(mant * 256.0), exp - 8)   # rint rounds half to even
    raise ValueError(dtype)


# --------------------------------------------------------------------------
# Sec. 2.1: attention
# --------------------------------------------------------------------------
def softmax_row(logits: np.ndarray) -> np.ndarray:
    """softmax over a 1-D vector, max-subtracted."""
    e = np.exp(logits - np.max(logits))
    return e / np.sum(e)


def attention_row(q: np.ndarray, Kmat: np.ndarray, Vmat: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. 1 for one head and one query: softmax(q K^T / sqrt(d)) V.

    q: [d]; Kmat, Vmat: [rows, d].  Returns (output [d], probabilities [rows]).
    """
    d = q.shape[0]
    p = softmax_row((Kmat @ q) / np.sqrt(F64(d)))
    return p @ Vmat, p


def slice_rows_by_matmul(Kmat: np.ndarray, j: int) -> np.ndarray:
    """Sec. 2.4: remove row j as S_j K with S_j = identity without its j-th row."""
    mrows = Kmat.shape[0]
    S_j = np.delete(np.eye(mrows), j, axis=0)
    return S_j @ Kmat


# --------------------------------------------------------------------------
# Sec. 2.2: controller
# --------------------------------------------------------------------------
def sigmoid(a):
    return 1.0 / (1.0 + np.exp(-a))


def gru_cell(x: np.ndarray, h: np.ndarray, W_ih: np.ndarray, W_hh: np.ndarray,
             b_ih: np.ndarray, b_hh: np.ndarray) -> np.ndarray:
    """z_i = GRU(x_i, z_{i-1}) (Eq. 2, first line).  Gate order in the stacked weights: r, z, n."""
    dp = h.shape[0]
    gi = W_ih @ x + b_ih
    gh = W_hh @ h + b_hh
    r = sigmoid(gi[0:dp] + gh[0:dp])
    u = sigmoid(gi[dp:2 * dp] + gh[dp:2 * dp])
    cand = np.tanh(gi[2 * dp:] + r * gh[2 * dp:])
    return (1.0 - u) * cand + u * h


def keep_probability(z: np.ndarray, delta: float, wts: Dict[str, np.ndarray]) -> float:
    """sigma_i = Sigmoid(MLP(p_i + z_i)) (Eq. 2, second line).

    p_i = pos_w * delta + pos_b (position layer, 1 -> d'), interaction layer
    with tanh, output layer followed by a sigmoid.
    """
    p = wts["pos_w"] * delta + wts["pos_b"]
    u = np.tanh(wts["mlp_w1"] @ (p + z) + wts["mlp_b1"])
    return float(sigmoid(wts["out_w"] @ u + wts["out_b"][0]))


# --------------------------------------------------------------------------
# Sec. 2.2 / 2.3: the order on tokens and the two selections
# --------------------------------------------------------------------------
def ranked(positions: Sequence[int], score: np.ndarray) -> List[int]:
    """Positions sorted best first: higher sigma first, equal sigma -> lower position first."""
    return sorted((int(p) for p in positions), key=lambda p: (-float(score[p]), p))


def release_lowest(slot_pos: np.ndarray, score: np.ndarray, current: int, m: int) -> List[int]:
    """Slots to free so that at most m rows stay: the lowest-ranked occupied rows, never `current`.

    slot_pos: [K] position per slot, -1 = free.  Returns slot indices, ascending.
    """
    occupied = [k for k in range(slot_pos.shape[0]) if slot_pos[k] >= 0]
    x = max(0, len(occupied) - m)
    if x == 0:
        return []
    slot_of = {int(slot_pos[k]): k for k in occupied}
    order = ranked([p for p in slot_of if p != current], score)    # best first
    return sorted(slot_of[p] for p in order[len(order) - x:])


def rebuild_choice(resident: Sequence[int], n: int, score: np.ndarray, R: int) -> List[int]:
    """Top-R of the released tokens (positions 0..n that hold no cache row), best first."""
    res = set(int(p) for p in resident)
    pool = [p for p in range(n + 1) if p not in res]
    return ranked(pool, score)[:min(R, len(pool))]


# --------------------------------------------------------------------------
# rotary position embedding (optional; see the readings in the header)
# --------------------------------------------------------------------------
def rotary(rows: np.ndarray, positions: Sequence[int], base: float) -> np.ndarray:
    """rows [r, ..., d] (any number of head axes in between), positions [r]: every vector of
    row i turned by its position.  With t_j = positions[i] * base**(-2j/d) for j < d/2:
        out[j]       = x[j] cos t_j - x[j + d/2] sin t_j
        out[j + d/2] = x[j] sin t_j + x[j + d/2] cos t_j"""
    x = np.asarray(rows, dtype=F64)
    d = x.shape[-1]
    half = d // 2
    out = np.empty_like(x)
    for i, pos in enumerate(positions):
        for j in range(half):
            t = F64(pos) * F64(base) ** (F64(-2.0) * j / d)
            lo, hi = x[i, ..., j], x[i, ..., j + half]
            out[i, ..., j] = lo * np.cos(t) - hi * np.sin(t)
            out[i, ..., j + half] = lo * np.sin(t) + hi * np.cos(t)
    return out


# --------------------------------------------------------------------------
# the whole path
# --------------------------------------------------------------------------
@dataclass
class OracleConfig:
    L: int
    B: int
    H: int
    d: int
    D: int
    K: int
    R: int
    N_max: int
    dprime: int
    dtype: str            # "f32" | "bf16"
    pos_scale: float
    rescore: bool = False # score every token again at every step, with its distance to the current token
    rope_base: float = 0.0  # > 0: keys (and, in the rebuild forward, queries) made from hidden states are rotated

    @property
    def m(self) -> int:
        return self.K - self.R - 1


class AdoreOracle:
    """State of one decode job and its init / step functions.

    Inputs are float arrays whose values are already exact in the storage
    type; everything is upcast to fp64 where it is used.
    """

    def __init__(self, cfg: OracleConfig, weights: Dict[str, np.ndarray]):
        if not (0 <= cfg.R <= cfg.K - 2):
            raise ValueError("need 0 <= R <= K-2")
        self.cfg = cfg
        self.wts = weights
        # fp64 copies of the controller parameters; W_kv is upcast per layer on first use
        self.w64 = {k: np.asarray(v, dtype=F64) for k, v in weights.items() if k != "w_kv"}
        self._wkv64: Dict[int, np.ndarray] = {}
        c = cfg
        self.Kc = np.zeros((c.L, c.B, c.H, c.K, c.d), dtype=F64)
        self.Vc = np.zeros((c.L, c.B, c.H, c.K, c.d), dtype=F64)
        self.slot_pos = np.full((c.B, c.H, c.K), -1, dtype=np.int32)
        self.score = np.zeros((c.B, c.N_max), dtype=np.float32)
        self.z = np.zeros((c.B, c.dprime), dtype=F64)
        self.z_all = np.zeros((c.B, c.N_max, c.dprime), dtype=F64) if c.rescore else None   # z_i of every token
        self.own_scores = None           # rescore mode: the scores of the last step before any override
        self.n = 0                       # position of the next token to arrive
        self.last_probs = None           # attention probabilities of the last step (diagnostics)

    # -- controller ---------------------------------------------------------
    def _controller(self, b: int, x: np.ndarray, i: int) -> float:
        w = self.w64
        self.z[b] = gru_cell(x.astype(F64), self.z[b], w["gru_w_ih"], w["gru_w_hh"],
                             w["gru_b_ih"], w["gru_b_hh"])
        if self.cfg.rescore:
            self.z_all[b, i] = self.z[b]
            delta = F64(0.0)             # the arriving token is at distance 0 from itself
        else:
            delta = F64(np.float32(i) * np.float32(self.cfg.pos_scale))
        return keep_probability(self.z[b], delta, w)

    def _rescore(self, b: int, n: int) -> np.ndarray:
        """Rescore mode: sigma_i for every token i <= n as seen from the current token n (Eq. 2 with the
        position feature of the distance n - i and the stored state z_i)."""
        out = np.zeros(n + 1, dtype=F64)
        for i in range(n + 1):
            delta = F64(np.float32(n - i) * np.float32(self.cfg.pos_scale))
            out[i] = keep_probability(self.z_all[b, i], delta, self.w64)
        return out

    # -- rebuild ------------------------------------------------------------
    def _project(self, layer: int, x_rows: np.ndarray, positions: Sequence[int]) -> np.ndarray:
        """K/V states of tokens from their hidden states: one rounding of x W_kv^T; when the rotary
        embedding is on, the rounded key half is then turned to the tokens' positions and rounded again."""
        c = self.cfg
        if layer not in self._wkv64:                     # [2*H*d, D], rows 0..H*d-1 = W_k
            self._wkv64[layer] = np.asarray(self.wts["w_kv"][layer], dtype=F64)
        kv = round_to_storage(x_rows.astype(F64) @ self._wkv64[layer].T, c.dtype)
        if c.rope_base > 0:
            Hd = c.H * c.d
            kv[:, :Hd] = round_to_storage(
                rotary(kv[:, :Hd].reshape(-1, c.H, c.d), positions, c.rope_base).reshape(-1, Hd), c.dtype)
        return kv

    def _place_rebuilt(self, b: int, rebuilt: List[int], hidden_store: np.ndarray) -> None:
        c = self.cfg
        if not rebuilt:
            return
        for l in range(c.L):
            kv = self._project(l, hidden_store[l, b, rebuilt, :], rebuilt)  # [r, 2*H*d]
            for h in range(c.H):
                free = [k for k in range(c.K) if self.slot_pos[b, h, k] < 0]    # ascending
                for rho, pos in enumerate(rebuilt):
                    s = free[rho]
                    self.Kc[l, b, h, s] = kv[rho, h * c.d:(h + 1) * c.d]
                    self.Vc[l, b, h, s] = kv[rho, c.H * c.d + h * c.d: c.H * c.d + (h + 1) * c.d]
        for h in range(c.H):
            free = [k for k in range(c.K) if self.slot_pos[b, h, k] < 0]
            for rho, pos in enumerate(rebuilt):
                self.slot_pos[b, h, free[rho]] = pos

    # -- init ---------------------------------------------------------------
    def init_cache(self, prompt_k: np.ndarray, prompt_v: np.ndarray, hidden_store: np.ndarray,
                   ctrl_input: np.ndarray, S: int, score_override: Optional[np.ndarray] = None):
        """One-shot application of the step rules to a prompt of S tokens.

        prompt_k/v: [L,B,H,S,d]; hidden_store: [L,B,N_max,D] (rows < S valid);
        ctrl_input: [B,S,D]; score_override: [B,S] or None.
        Residents = {S-1} plus the best min(S,m)-1 of the older tokens, in
        ascending position from slot 0; then the best min(R, |rest|) of the
        rest, by rank, re-projected from their hidden states.
        """
        c = self.cfg
        self.slot_pos[:] = -1
        self.z[:] = 0.0
        rebuilt_all = []
        for b in range(c.B):
            for i in range(S):
                s = self._controller(b, ctrl_input[b, i], i)
                self.score[b, i] = np.float32(s) if score_override is None else score_override[b, i]
            if c.rescore:                # all prompt tokens as seen from the last one
                own = self._rescore(b, S - 1)
                if self.own_scores is None or self.own_scores.shape[1] != S:
                    self.own_scores = np.zeros((c.B, S), dtype=F64)
                self.own_scores[b] = own
                self.score[b, :S] = own.astype(np.float32) if score_override is None else score_override[b, :S]
            keep = min(S, c.m)
            older = ranked(range(S - 1), self.score[b])[:keep - 1]
            residents = sorted(older + [S - 1])
            for h in range(c.H):
                for s_idx, pos in enumerate(residents):
                    self.Kc[:, b, h, s_idx] = prompt_k[:, b, h, pos]
                    self.Vc[:, b, h, s_idx] = prompt_v[:, b, h, pos]
                    self.slot_pos[b, h, s_idx] = pos
            rebuilt = rebuild_choice(residents, S - 1, self.score[b], c.R)
            self._place_rebuilt(b, rebuilt, hidden_store)
            rebuilt_all.append(rebuilt)
        self.n = S
        return rebuilt_all

    # -- one decode step ----------------------------------------------------
    def decode_step(self, q: np.ndarray, k_new: np.ndarray, v_new: np.ndarray,
                    hidden_store: np.ndarray, x_n: np.ndarray,
                    score_override: Optional[np.ndarray] = None):
        """q, k_new, v_new: [L,B,H,d]; hidden_store: [L,B,N_max,D]; x_n: [B,D].

        Returns (out [L,B,H,d] fp64, slot_map [B,H,K] i32, released_pos [B,H,R+1] i32,
        rebuilt_pos [B,R] i32, own_score [B] fp64) where own_score is the controller's
        value before any override.  In rescore mode score_override, if given, is [B, n+1]
        (every token's score of this step) and `own_scores` [B, n+1] keeps the oracle's own.
        """
        c = self.cfg
        n = self.n
        if n >= c.N_max:
            raise RuntimeError("step past N_max")
        out = np.zeros((c.L, c.B, c.H, c.d), dtype=F64)
        released_pos = np.full((c.B, c.H, c.R + 1), -1, dtype=np.int32)
        rebuilt_pos = np.full((c.B, c.R), -1, dtype=np.int32)
        own_score = np.zeros(c.B, dtype=F64)
        probs = {}

        for b in range(c.B):
            # 1. insert the current token's k, v into the lowest free slot of every head
            for h in range(c.H):
                free = [k for k in range(c.K) if self.slot_pos[b, h, k] < 0]
                s = free[0]
                self.Kc[:, b, h, s] = k_new[:, b, h]
                self.Vc[:, b, h, s] = v_new[:, b, h]
                self.slot_pos[b, h, s] = n
            # 2. attention over the occupied slots
            for l in range(c.L):
                for h in range(c.H):
                    valid = np.nonzero(self.slot_pos[b, h] >= 0)[0]
                    out[l, b, h], p = attention_row(q[l, b, h].astype(F64),
                                                    self.Kc[l, b, h, valid], self.Vc[l, b, h, valid])
                    probs[(l, b, h)] = (valid, p)
            # 3. controller: score of the arriving token; older scores unchanged
            own_score[b] = self._controller(b, x_n[b], n)
            if c.rescore:
                if b == 0:
                    self.own_scores = np.zeros((c.B, n + 1), dtype=F64)
                self.own_scores[b] = self._rescore(b, n)
                self.score[b, :n + 1] = (self.own_scores[b].astype(np.float32) if score_override is None
                                         else np.asarray(score_override[b], dtype=np.float32))
            else:
                self.score[b, n] = (np.float32(own_score[b]) if score_override is None
                                    else np.float32(score_override[b]))
            # 4. release
            for h in range(c.H):
                freed = release_lowest(self.slot_pos[b, h], self.score[b], n, c.m)
                for j, s in enumerate(freed):
                    released_pos[b, h, j] = self.slot_pos[b, h, s]
                for s in freed:
                    self.slot_pos[b, h, s] = -1
            # 5. rebuild choice (uniform policy: residency is the same for every head; head 0 is read)
            resident = [int(p) for p in self.slot_pos[b, 0] if p >= 0]
            rebuilt = rebuild_choice(resident, n, self.score[b], c.R)
            rebuilt_pos[b, :len(rebuilt)] = rebuilt
            # 6. rebuild: re-project and scatter into the lowest free slots
            self._place_rebuilt(b, rebuilt, hidden_store)

        self.n = n + 1
        self.last_probs = probs
        return out, self.slot_pos.copy(), released_pos, rebuilt_pos, own_score


class AdoreForwardOracle(AdoreOracle):
    """Sec. 2.3 in full: at step n the embeddings of the R tokens chosen in the previous step and of the
    current token, X_{R+1}, go through every layer as R+1 query rows; each layer projects them to q, k, v,
    puts k, v into the rows' slots, attends, and hands x + W_o o to the next layer.  The last layer's row
    of the current token is the step's output.  Release and the choice of the next R tokens follow as in
    the base class.  `weights` additionally holds w_q [L,H*d,D] and w_o [L,D,H*d]."""

    def __init__(self, cfg: OracleConfig, weights: Dict[str, np.ndarray]):
        super().__init__(cfg, weights)
        self._wq64: Dict[int, np.ndarray] = {}
        self._wo64: Dict[int, np.ndarray] = {}
        self.pending: List[List[int]] = [[] for _ in range(cfg.B)]   # chosen last step, rebuilt in the next
        self.last_rows = None            # [L+1][B] list of (positions, X) of the last step (diagnostics)
        self.own = None                  # the last step's own per-layer values when it ran with `adopt`

    def _place_rebuilt(self, b, rebuilt, hidden_store):
        """Slots are assigned now (rank rho -> rho-th lowest free slot); their K/V follow at the next step."""
        c = self.cfg
        for h in range(c.H):
            free = [k for k in range(c.K) if self.slot_pos[b, h, k] < 0]
            for rho, pos in enumerate(rebuilt):
                self.slot_pos[b, h, free[rho]] = pos
        self.pending[b] = list(rebuilt)

    def init_cache(self, prompt_k, prompt_v, hidden_store, ctrl_input, S, score_override=None):
        return super().init_cache(prompt_k, prompt_v, None, ctrl_input, S, score_override)

    def _w(self, cache, name, layer):
        if layer not in cache:
            cache[layer] = np.asarray(self.wts[name][layer], dtype=F64)
        return cache[layer]

    def forward_step(self, embed: np.ndarray, score_override: Optional[np.ndarray] = None,
                     adopt: Optional[Dict[str, np.ndarray]] = None):
        """embed: [B, N_max, D] token embeddings (rows <= n valid).  Returns (x_out [B,D] fp64: last layer's
        row of the current token, rows_out [B,R+1,D]: last layer's rows in rank order with the current token
        last (unused rows zero), slot_map, released_pos, rebuilt_pos, own_score).

        adopt (lockstep runs against another implementation of this step): what that implementation stored
        for the rows of this step, "x" [L,B,R+1,D] (the rows leaving every layer) and "k", "v" [L,B,H,R+1,d]
        (the rows' K/V states), rank j at index j and the current token at index R.  Every layer then computes
        its own K/V and rows from the inputs it is given, keeps them in self.own (same keys and shapes, for the
        caller to compare), and hands the adopted ones on: to its attention (K/V) and to the next layer (rows).
        The arithmetic of a layer is the same with and without it."""
        c = self.cfg
        n = self.n
        if n >= c.N_max:
            raise RuntimeError("step past N_max")
        Hd = c.H * c.d
        if adopt is not None:
            self.own = dict(x=np.zeros((c.L, c.B, c.R + 1, c.D), dtype=F64),
                            k=np.zeros((c.L, c.B, c.H, c.R + 1, c.d), dtype=F64),
                            v=np.zeros((c.L, c.B, c.H, c.R + 1, c.d), dtype=F64))
        released_pos = np.full((c.B, c.H, c.R + 1), -1, dtype=np.int32)
        rebuilt_pos = np.full((c.B, c.R), -1, dtype=np.int32)
        own_score = np.zeros(c.B, dtype=F64)
        rows_out = np.zeros((c.B, c.R + 1, c.D), dtype=F64)
        for b in range(c.B):
            positions = list(self.pending[b]) + [n]                      # rank order, current token last
            X = embed[b, positions, :].astype(F64)                       # X_{R+1}
            # the current token takes the lowest free slot of every head (its k, v differ per layer)
            cur_slot = []
            for h in range(c.H):
                free = [k for k in range(c.K) if self.slot_pos[b, h, k] < 0]
                self.slot_pos[b, h, free[0]] = n
                cur_slot.append(free[0])
            for l in range(c.L):
                Wq = self._w(self._wq64, "w_q", l)
                Wo = self._w(self._wo64, "w_o", l)
                Q = round_to_storage(X @ Wq.T, c.dtype)                  # [r+1, H*d]
                if c.rope_base > 0:
                    Q = round_to_storage(rotary(Q.reshape(-1, c.H, c.d), positions, c.rope_base).reshape(-1, Hd),
                                         c.dtype)
                KV = self._project(l, X, positions)                      # [r+1, 2*H*d], rounded
                if adopt is not None:
                    at = list(range(len(positions) - 1)) + [c.R]         # where the rows sit in the adopted arrays
                    self.own["k"][l, b][:, at] = KV[:, :Hd].reshape(-1, c.H, c.d).transpose(1, 0, 2)
                    self.own["v"][l, b][:, at] = KV[:, Hd:].reshape(-1, c.H, c.d).transpose(1, 0, 2)
                    KV = np.concatenate([adopt["k"][l, b][:, at].transpose(1, 0, 2).reshape(-1, Hd),
                                         adopt["v"][l, b][:, at].transpose(1, 0, 2).reshape(-1, Hd)], axis=1).astype(F64)
                O = np.zeros((len(positions), Hd), dtype=F64)
                for h in range(c.H):
                    slot_of = {int(p): k for k, p in enumerate(self.slot_pos[b, h]) if p >= 0}
                    for j, pos in enumerate(positions):
                        s = slot_of[pos]
                        self.Kc[l, b, h, s] = KV[j, h * c.d:(h + 1) * c.d]
                        self.Vc[l, b, h, s] = KV[j, Hd + h * c.d: Hd + (h + 1) * c.d]
                    for j, pos in enumerate(positions):
                        valid = np.nonzero((self.slot_pos[b, h] >= 0) & (self.slot_pos[b, h] <= pos))[0]
                        O[j, h * c.d:(h + 1) * c.d], _ = attention_row(Q[j, h * c.d:(h + 1) * c.d],
                                                                       self.Kc[l, b, h, valid],
                                                                       self.Vc[l, b, h, valid])
                O = round_to_storage(O, c.dtype)
                X = round_to_storage(X + O @ Wo.T, c.dtype)
                if adopt is not None:
                    self.own["x"][l, b, at] = X
                    if l < c.L - 1:
                        X = np.asarray(adopt["x"][l, b, at], dtype=F64)
            rows_out[b, :len(positions) - 1] = X[:-1]
            rows_out[b, c.R] = X[-1]
            # controller, release, choice of the next rebuild set: as in the base class
            own_score[b] = self._controller(b, embed[b, n], n)
            if c.rescore:
                if b == 0:
                    self.own_scores = np.zeros((c.B, n + 1), dtype=F64)
                self.own_scores[b] = self._rescore(b, n)
                self.score[b, :n + 1] = (self.own_scores[b].astype(np.float32) if score_override is None
                                         else np.asarray(score_override[b], dtype=np.float32))
            else:
                self.score[b, n] = (np.float32(own_score[b]) if score_override is None
                                    else np.float32(score_override[b]))
            for h in range(c.H):
                freed = release_lowest(self.slot_pos[b, h], self.score[b], n, c.m)
                for j, s in enumerate(freed):
                    released_pos[b, h, j] = self.slot_pos[b, h, s]
                for s in freed:
                    self.slot_pos[b, h, s] = -1
            resident = [int(p) for p in self.slot_pos[b, 0] if p >= 0]
            rebuilt = rebuild_choice(resident, n, self.score[b], c.R)
            rebuilt_pos[b, :len(rebuilt)] = rebuilt
            self._place_rebuilt(b, rebuilt, None)
        self.n = n + 1
        return rows_out[:, c.R].copy(), rows_out, self.slot_pos.copy(), released_pos, rebuilt_pos, own_score


class AdoreH2OOracle(AdoreOracle):
    """H2O(Rebuilt) (Sec. 3.1, baselines 6 and 7): the score of a token is the attention it has received so far,
    counted per head, and the tokens a head has evicted are candidates for this paper's rebuild.

    The paper gives the two baselines one sentence each (H2O evicts the tokens that contribute least to the
    cumulative attention; the rebuilt variant rebuilds K/V states of evicted tokens on top of it), so the rest is
    a reading, stated here and used exactly so:
      * score[b, h, i] = sum over the steps at which head h held a row of token i (its own step included) of the
        probability the step's query gave that row (Eq. 1's softmax); kept in fp32, added to in the order of the
        steps.  A token a head has evicted keeps the score it had; when it is rebuilt it collects again.
        Prompt tokens start from score_init (the attention they collected during the prompt, which is computed
        by whoever ran the prompt) or from zero.
      * Release: per head, as in the base class, on that head's scores: the current token is exempt, ties go to
        the lower position.  Heads evict different tokens, so every head has its own slot map.
      * Rebuild: one row of the re-projection makes the K/V of a token for all heads, so the choice is per
        sequence.  Candidates: the tokens at least one head is missing.  Order: the sum of a token's scores over
        the heads (fp32, heads added in order from head 0), equal sums to the lower position; the best
        min(R, candidates) are rebuilt.  A head that still holds a chosen token keeps its row; the others put the
        token into their free slots, lowest slot first in the order of the ranks.
      * One layer per job (the cumulative attention of H2O belongs to a layer)."""

    def __init__(self, cfg: OracleConfig, weights: Dict[str, np.ndarray]):
        if cfg.L != 1:
            raise ValueError("H2O scores are kept per layer: one layer per job")
        super().__init__(cfg, weights)
        self.hscore = np.zeros((cfg.B, cfg.H, cfg.N_max), dtype=np.float32)
        self.own_scores = None           # [B,H,n+1] fp64: the scores of the last step before any override

    def _aggregate(self, b: int, n: int) -> np.ndarray:
        agg = np.zeros(n + 1, dtype=np.float32)
        for h in range(self.cfg.H):
            agg = (agg + self.hscore[b, h, :n + 1]).astype(np.float32)
        return agg

    def _choose_and_place(self, b: int, n: int, hidden_store: np.ndarray) -> List[int]:
        c = self.cfg
        held = [set(int(p) for p in self.slot_pos[b, h] if p >= 0) for h in range(c.H)]
        pool = [i for i in range(n + 1) if any(i not in held[h] for h in range(c.H))]
        rebuilt = ranked(pool, self._aggregate(b, n))[:min(c.R, len(pool))]
        if rebuilt:
            kv = self._project(0, hidden_store[0, b, rebuilt, :], rebuilt)     # [r, 2*H*d]
            for h in range(c.H):
                free = [k for k in range(c.K) if self.slot_pos[b, h, k] < 0]   # ascending
                taken = 0
                for rho, pos in enumerate(rebuilt):
                    if pos in held[h]:
                        continue
                    s = free[taken]
                    taken += 1
                    self.Kc[0, b, h, s] = kv[rho, h * c.d:(h + 1) * c.d]
                    self.Vc[0, b, h, s] = kv[rho, c.H * c.d + h * c.d: c.H * c.d + (h + 1) * c.d]
                    self.slot_pos[b, h, s] = pos
        return rebuilt

    def init_cache(self, prompt_k, prompt_v, hidden_store, S: int, score_init: Optional[np.ndarray] = None):
        """prompt_k/v: [1,B,H,S,d]; hidden_store: [1,B,N_max,D]; score_init: [B,H,S] or None (zeros).
        Per head: token S-1 and the best min(S,m)-1 older tokens by that head's scores, in ascending position
        from slot 0; then the rebuild choice above.  Returns the rebuilt positions per sequence."""
        c = self.cfg
        self.slot_pos[:] = -1
        self.hscore[:] = 0.0
        if score_init is not None:
            self.hscore[:, :, :S] = np.asarray(score_init, dtype=np.float32)
        rebuilt_all = []
        keep = min(S, c.m)
        for b in range(c.B):
            for h in range(c.H):
                older = ranked(range(S - 1), self.hscore[b, h])[:keep - 1]
                for s_idx, pos in enumerate(sorted(older + [S - 1])):
                    self.Kc[:, b, h, s_idx] = prompt_k[:, b, h, pos]
                    self.Vc[:, b, h, s_idx] = prompt_v[:, b, h, pos]
                    self.slot_pos[b, h, s_idx] = pos
            rebuilt_all.append(self._choose_and_place(b, S - 1, hidden_store))
        self.n = S
        return rebuilt_all

    def decode_step(self, q, k_new, v_new, hidden_store, score_override: Optional[np.ndarray] = None):
        """q, k_new, v_new: [1,B,H,d]; hidden_store: [1,B,N_max,D]; score_override: [B,H,n+1] or None: the scores
        after this step's attention as another implementation holds them (adopted once the caller has checked
        them against own_scores).  Returns (out [1,B,H,d], slot_map [B,H,K], released_pos [B,H,R+1] in ascending
        slot order, rebuilt_pos [B,R])."""
        c = self.cfg
        n = self.n
        if n >= c.N_max:
            raise RuntimeError("step past N_max")
        out = np.zeros((1, c.B, c.H, c.d), dtype=F64)
        released_pos = np.full((c.B, c.H, c.R + 1), -1, dtype=np.int32)
        rebuilt_pos = np.full((c.B, c.R), -1, dtype=np.int32)
        self.own_scores = self.hscore[:, :, :n + 1].astype(F64)
        for b in range(c.B):
            for h in range(c.H):
                free = [k for k in range(c.K) if self.slot_pos[b, h, k] < 0]
                s = free[0]
                self.Kc[0, b, h, s] = k_new[0, b, h]
                self.Vc[0, b, h, s] = v_new[0, b, h]
                self.slot_pos[b, h, s] = n
                valid = np.nonzero(self.slot_pos[b, h] >= 0)[0]
                out[0, b, h], p = attention_row(q[0, b, h].astype(F64), self.Kc[0, b, h, valid], self.Vc[0, b, h, valid])
                for k, pk in zip(valid, p):                      # every row collects what the query gave it
                    self.own_scores[b, h, self.slot_pos[b, h, k]] += pk
            self.hscore[b, :, :n + 1] = (self.own_scores[b].astype(np.float32) if score_override is None
                                         else np.asarray(score_override[b], dtype=np.float32))
            for h in range(c.H):
                freed = release_lowest(self.slot_pos[b, h], self.hscore[b, h], n, c.m)
                for j, s in enumerate(freed):
                    released_pos[b, h, j] = self.slot_pos[b, h, s]
                for s in freed:
                    self.slot_pos[b, h, s] = -1
            rebuilt = self._choose_and_place(b, n, hidden_store)
            rebuilt_pos[b, :len(rebuilt)] = rebuilt
        self.n = n + 1
        return out, self.slot_pos.copy(), released_pos, rebuilt_pos


def full_attention(q: np.ndarray, Kall: np.ndarray, Vall: np.ndarray) -> np.ndarray:
    """Eq. 1 over all past rows, per head.  q: [H,d]; Kall, Vall: [H,n,d]."""
    return np.stack([attention_row(q[h].astype(F64), Kall[h].astype(F64), Vall[h].astype(F64))[0]
                     for h in range(q.shape[0])])


# --------------------------------------------------------------------------
# top-K attention over a whole sequence (Sec. 2.1 / 2.2; see the readings in the header)
# --------------------------------------------------------------------------
def topk_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, top_k: int) -> Tuple[np.ndarray, np.ndarray]:
    """q, k, v: [rows, S, d] (rows = sequences x heads).  Returns (out [rows, S, d] fp64,
    kept [rows, S, S] bool: kept[r, i, j] = query i of row r keeps key j)."""
    q, k, v = (np.asarray(a, dtype=F64) for a in (q, k, v))
    rows, S, d = q.shape
    out = np.zeros((rows, S, d), dtype=F64)
    kept = np.zeros((rows, S, S), dtype=bool)
    for r in range(rows):
        for i in range(S):
            w = k[r, :i + 1] @ q[r, i]                          # the weights of query i, before scaling
            if i + 1 > top_k:
                order = np.argsort(-w, kind="stable")           # descending; equal weights: lower position first
                sel = np.sort(order[:top_k])
            else:
                sel = np.arange(i + 1)
            kept[r, i, sel] = True
            out[r, i] = softmax_row(w[sel] / np.sqrt(F64(d))) @ v[r, sel]
    return out, kept
