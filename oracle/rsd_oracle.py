"""CPU checker for Reward-Guided Speculative Decoding (RSD), in fp64 NumPy.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain statement of what
the accelerated path has to compute.  It shares no code with that path and
must never be imported by it; only the tests, the smoke check and the
benchmark's CPU-baseline leg call it.

What is written out here, and where the paper defines it:

* ``generate_sequence`` - the RSD loop (Section 2.1, Algorithm 1): per
  reasoning step the draft model proposes a step, the process reward model
  scores it, the acceptance criterion keeps it or the target model regenerates
  the step from the same context; stop when the committed step holds EOS.
* ``accept`` / ``omega`` - the acceptance criterion (Section 2.2, Algorithm 2)
  and the weighting functions of Table 1; the binary step 1(r >= delta) is the
  paper's default (Section 3, "Default Setting"; Proposition 3).
* ``mixture_distribution`` - the law of one RSD step (Proposition 1):
  P_RSD = omega_r P_m + nu P_M with nu = 1 - E_{P_m}[omega_r].
* ``gen_step_sd`` - regeneration of a rejected step by token-level speculative
  decoding with the draft and the target (Section 5, "Combine RSD with SD";
  the method itself is the cited speculative-decoding algorithm: the draft
  proposes gamma tokens, the target scores them in one pass, each is kept with
  probability min(1, p/q), the first refusal is replaced by a draw from the
  normalised positive part of p - q, and a fully kept run earns one more
  target token).  The paper runs SD greedily with gamma = 7 (Section 3).
* ``generate_sequence_bon`` - process Best-of-N, one of the paper's comparison
  procedures (Section 3, "Baselines": sample N candidate steps and select the
  one with the highest reward; run with a base model and a reward model only,
  Table 3).  Every candidate continues the same committed context.
* ``reward`` - the reward model's head (Appendix, "Model Merge"): a projection
  of the final hidden state to one scalar, mapped to [0, 1] (Section 3,
  "Models") by a logistic function.
* the transformer itself (RMSNorm, rotary embedding with rotate-half pairing,
  grouped-query causal attention, SwiGLU MLP, untied head) is not defined by
  the paper, which treats the three models as black boxes; it follows the
  workload definition and is pinned by the tests against library routines and
  invariants.  Parity of the full-width models is otherwise unpinned: no
  trained weights or printed logits exist to compare with.

All arithmetic is fp64.  Weights arrive as arrays holding the storage-type
values exactly (fp32, or bf16 widened) and are widened to fp64 without any
further rounding.  Sequences never interact, so everything is per sequence.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence

import numpy as np

F64 = np.float64

OMEGA_BINARY, OMEGA_CONSTANT, OMEGA_CLIP, OMEGA_RATIO, OMEGA_LOGISTIC = 0, 1, 2, 3, 4
RUNNING, FIN_EOS, FIN_MAX_CTX, FIN_MAX_STEPS = 0, 1, 2, 3


# --------------------------------------------------------------------------
# model pieces
# --------------------------------------------------------------------------
class OracleModel:
    """Weights of one model, widened to fp64 on first use and kept."""

    def __init__(self, shape, weights: Dict[str, np.ndarray]):
        self.s = shape
        self._w = weights
        self._c: Dict[str, np.ndarray] = {}

    def mat(self, name: str) -> np.ndarray:
        a = self._c.get(name)
        if a is None:
            a = np.ascontiguousarray(self._w[name], dtype=F64)
            self._c[name] = a
        return a


def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """g * x / sqrt(mean(x^2) + eps) over the last axis."""
    x = np.asarray(x, dtype=F64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return g * (x / np.sqrt(ms + eps))


def rope(x: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotary embedding, rotate-half pairing: element i is paired with
    i + hd/2 and the pair is rotated by pos * theta^(-2i/hd).
    ``x`` is [T, heads, hd], ``pos`` is [T] (absolute positions, first is 0)."""
    x = np.asarray(x, dtype=F64)
    hd = x.shape[-1]
    half = hd // 2
    inv = theta ** (-2.0 * np.arange(half, dtype=F64) / hd)
    ang = np.asarray(pos, dtype=F64)[:, None] * inv[None, :]          # [T, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def softmax(z: np.ndarray) -> np.ndarray:
    z = np.asarray(z, dtype=F64)
    e = np.exp(z - np.max(z, axis=-1, keepdims=True))
    return e / np.sum(e, axis=-1, keepdims=True)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def attention_probs(q: np.ndarray, k: np.ndarray, q_pos: np.ndarray) -> np.ndarray:
    """Causal attention weights of one head.  ``q`` [T, hd] sits at absolute
    positions ``q_pos``; ``k`` [S, hd] holds keys of positions 0..S-1.  A query
    sees keys at positions <= its own.  Returns [T, S], rows summing to 1."""
    hd = q.shape[-1]
    s = (q @ k.T) / np.sqrt(F64(hd))
    mask = np.arange(k.shape[0])[None, :] > np.asarray(q_pos)[:, None]
    s = np.where(mask, -np.inf, s)
    return softmax(s)


def gqa_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, q_pos: np.ndarray) -> np.ndarray:
    """Grouped-query attention.  q [T, H, hd]; k, v [S, Hkv, hd].  Query head j
    reads KV head j // (H / Hkv).  Returns [T, H, hd]."""
    T, H, hd = q.shape
    Hkv = k.shape[1]
    group = H // Hkv
    out = np.empty((T, H, hd), dtype=F64)
    for j in range(H):
        g = j // group
        p = attention_probs(q[:, j, :], k[:, g, :], q_pos)
        out[:, j, :] = p @ v[:, g, :]
    return out


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Nearest bf16 value (8-bit significand, ties to even) of each fp64 entry,
    returned as fp64.  One rounding, straight from the fp64 bits; inputs are
    finite and within the normal range of bf16."""
    b = np.ascontiguousarray(x, dtype=F64).view(np.uint64)
    lsb = (b >> np.uint64(45)) & np.uint64(1)
    r = (b + np.uint64((1 << 44) - 1) + lsb) & ~np.uint64((1 << 45) - 1)
    return r.view(F64)


class KVCache:
    """Dense per-layer key/value store of one (model, sequence).  ``length`` is
    the number of leading positions held; truncation just lowers it.

    ``kv_dtype`` states how entries are stored: "exact" keeps the fp64 values;
    "bf16" rounds every (rotated) key and every value to bf16 as it is written,
    which is the storage format the workload definition fixes for the bf16
    models' caches (a quantisation step of the method as specified, not a
    shortcut of this checker: all arithmetic on the stored values stays fp64)."""

    def __init__(self, shape, capacity: int, kv_dtype: str = "exact"):
        assert kv_dtype in ("exact", "bf16")
        L, Hkv, hd = shape.n_layers, shape.n_kv_heads, shape.head_dim
        self.k = np.zeros((L, capacity, Hkv, hd), dtype=F64)
        self.v = np.zeros((L, capacity, Hkv, hd), dtype=F64)
        self.length = 0
        self.kv_dtype = kv_dtype

    def truncate(self, n: int) -> None:
        assert 0 <= n <= self.length
        self.length = n


def forward_chunk(m: OracleModel, kv: KVCache, tokens: Sequence[int]) -> np.ndarray:
    """Feed ``tokens`` as positions kv.length .. kv.length+T-1, append their
    keys/values to ``kv`` and return the final-norm hidden states [T, d]."""
    s = m.s
    T = len(tokens)
    p0 = kv.length
    pos = np.arange(p0, p0 + T)
    H, Hkv, hd = s.n_heads, s.n_kv_heads, s.head_dim
    h = m.mat("embed")[np.asarray(tokens, dtype=np.int64)]            # [T, d]
    for l in range(s.n_layers):
        p = f"l{l}."
        a = rmsnorm(h, m.mat(p + "attn_norm"), s.rms_eps)
        q = (a @ m.mat(p + "wq").T).reshape(T, H, hd)
        k = (a @ m.mat(p + "wk").T).reshape(T, Hkv, hd)
        v = (a @ m.mat(p + "wv").T).reshape(T, Hkv, hd)
        q = rope(q, pos, s.rope_theta)
        k = rope(k, pos, s.rope_theta)
        if kv.kv_dtype == "bf16":
            k, v = round_to_bf16(k), round_to_bf16(v)
        kv.k[l, p0:p0 + T] = k
        kv.v[l, p0:p0 + T] = v
        o = gqa_attention(q, kv.k[l, :p0 + T], kv.v[l, :p0 + T], pos)
        h = h + o.reshape(T, H * hd) @ m.mat(p + "wo").T
        b = rmsnorm(h, m.mat(p + "ffn_norm"), s.rms_eps)
        gate = b @ m.mat(p + "w_gate").T
        up = b @ m.mat(p + "w_up").T
        h = h + (silu(gate) * up) @ m.mat(p + "w_down").T
    kv.length = p0 + T
    return rmsnorm(h, m.mat("final_norm"), s.rms_eps)


def forward_full(m: OracleModel, tokens: Sequence[int], kv_dtype: str = "exact") -> np.ndarray:
    """Plain causal forward over the whole sequence with no cache kept:
    final-norm hidden states [len(tokens), d]."""
    return forward_chunk(m, KVCache(m.s, len(tokens), kv_dtype), tokens)


def lm_logits(m: OracleModel, y: np.ndarray) -> np.ndarray:
    """Vocabulary logits of final-norm hidden state(s) ``y``."""
    return np.asarray(y, dtype=F64) @ m.mat("lm_head").T


def reward(m: OracleModel, y: np.ndarray) -> float:
    """Reward head: logistic(w_r . y + b_r) on one final-norm hidden state."""
    z = float(np.dot(m.mat("w_r"), np.asarray(y, dtype=F64)) + m.mat("b_r")[0])
    return 1.0 / (1.0 + np.exp(-z))


# --------------------------------------------------------------------------
# decoding
# --------------------------------------------------------------------------
def sample(logits: np.ndarray, u: float, temperature: float, top_p: float) -> int:
    """Pick the next token.

    temperature == 0: the largest logit, lowest id on ties.  Otherwise, with
    p = softmax(logits / temperature): the nucleus S holds every token whose
    probability is at least tau*, the largest threshold for which the mass of
    {p_t >= tau} still reaches top_p (so ties at the boundary are all kept; if
    rounding keeps even the full mass below top_p, S is everything).  The draw
    walks S in ascending token id and returns the first token whose running
    mass exceeds u * mass(S), or the last member of S if none does."""
    logits = np.asarray(logits, dtype=F64)
    if temperature == 0.0:
        return int(np.argmax(logits))
    p = softmax(logits / F64(temperature))
    order = np.argsort(-p, kind="stable")
    cum = np.cumsum(p[order])
    reach = np.nonzero(cum >= top_p)[0]
    tau = p[order[reach[0]]] if reach.size else np.min(p)
    members = np.nonzero(p >= tau)[0]                 # ascending ids
    run = np.cumsum(p[members])
    z = run[-1]
    hit = np.nonzero(run > F64(u) * z)[0]
    return int(members[hit[0]] if hit.size else members[-1])


def token_distribution(logits: np.ndarray, temperature: float, top_p: float) -> np.ndarray:
    """The distribution ``sample`` draws from, as a vector over the vocabulary:
    one-hot at the arg max for temperature 0, else softmax(logits/temperature)
    restricted to the nucleus and renormalised."""
    logits = np.asarray(logits, dtype=F64)
    out = np.zeros(logits.shape[0], dtype=F64)
    if temperature == 0.0:
        out[int(np.argmax(logits))] = 1.0
        return out
    p = softmax(logits / F64(temperature))
    order = np.argsort(-p, kind="stable")
    cum = np.cumsum(p[order])
    reach = np.nonzero(cum >= top_p)[0]
    tau = p[order[reach[0]]] if reach.size else np.min(p)
    keep = p >= tau
    out[keep] = p[keep] / np.sum(p[keep])
    return out


def draw(dist: np.ndarray, u: float) -> int:
    """Inverse-CDF draw in ascending token id: the first token whose running
    mass exceeds u * total, or the last token of positive mass if none does."""
    members = np.nonzero(dist > 0.0)[0]
    run = np.cumsum(dist[members])
    hit = np.nonzero(run > F64(u) * run[-1])[0]
    return int(members[hit[0]] if hit.size else members[-1])


def sd_verify(q_rows: Sequence[np.ndarray], p_rows: Sequence[np.ndarray], proposals: Sequence[int],
              u_acc: Sequence[float], u_new: Sequence[float]):
    """One verification of speculative decoding.  ``proposals[i]`` was drawn from
    ``q_rows[i]``; ``p_rows`` holds the target's distributions at the same
    positions plus one more.  Proposal i is kept iff u_acc[i] < p_i(x)/q_i(x);
    the first refused one is replaced by a draw (uniform u_new[i]) from the
    normalised positive part of p_i - q_i; if all are kept, one more token is
    drawn from the last row of ``p_rows`` (uniform u_new[len(proposals)]).
    Returns (tokens emitted, number of proposals kept)."""
    g = len(proposals)
    assert len(q_rows) == g and len(p_rows) == g + 1
    out = []
    for i, x in enumerate(proposals):
        p, q = p_rows[i], q_rows[i]
        if F64(u_acc[i]) * q[x] < p[x]:
            out.append(int(x))
            continue
        res = np.maximum(p - q, 0.0)
        out.append(draw(res, u_new[i]))
        return out, i
    out.append(draw(p_rows[g], u_new[g]))
    return out, g


def omega(r: float, kind: int, delta: float, a: float = 0.0) -> float:
    """Weighting functions of Table 1.  ``delta`` is the threshold of the
    binary step and the centre of the logistic; ``a`` is the constant p, or
    the logistic slope alpha."""
    if kind == OMEGA_BINARY:
        return 1.0 if r >= delta else 0.0
    if kind == OMEGA_CONSTANT:
        return float(a)
    if kind == OMEGA_CLIP:
        return min(1.0, max(0.0, r))
    if kind == OMEGA_RATIO:
        return max(0.0, r / (1.0 + r))
    if kind == OMEGA_LOGISTIC:
        return 1.0 / (1.0 + np.exp(-a * (r - delta)))
    raise ValueError(kind)


def accept(r: float, kind: int, delta: float, a: float, u: float) -> bool:
    """Acceptance criterion (Algorithm 2): a weight of exactly 0 or 1 decides by
    itself; any other weight is compared with a uniform draw, accept iff
    omega(r) >= u."""
    w = omega(r, kind, delta, a)
    if w == 0.0 or w == 1.0:
        return w == 1.0
    return w >= u


def mixture_distribution(p_m: np.ndarray, p_M: np.ndarray, w: np.ndarray):
    """Law of one RSD step over a finite set of candidate steps
    (Proposition 1): returns (P_RSD, nu) with nu = 1 - sum(w * p_m)."""
    p_m, p_M, w = (np.asarray(x, dtype=F64) for x in (p_m, p_M, w))
    nu = 1.0 - float(np.sum(w * p_m))
    return w * p_m + nu * p_M, nu


@dataclass
class Params:
    delta: float
    sep_id: int
    step_cap: int
    max_steps: int
    max_ctx: int
    eos_id: int = -1
    temperature: float = 0.0
    top_p: float = 1.0
    sep_logit_bias: float = 0.0
    omega_kind: int = OMEGA_BINARY
    omega_a: float = 0.0
    page_tokens: int = 16
    kv_dtype: str = "exact"      # "bf16": keys and values are stored rounded to bf16 (see KVCache)
    merge: str = "none"          # "draft" / "target": the reward head sits on that model's trunk (Appendix "Model Merge")
    sd_k: int = 0                # > 0: rejected steps are regenerated by speculative decoding with this many proposals per round


class _Runner:
    """One model bound to one sequence: either keeps a KV cache and feeds only
    the tokens it has not seen (kv_len tracks how many it holds), or - with
    ``use_cache=False`` - recomputes the whole prefix every time."""

    def __init__(self, model: OracleModel, max_ctx: int, use_cache: bool, kv_dtype: str = "exact"):
        self.m = model
        self.use_cache = use_cache
        self.kv_dtype = kv_dtype
        self.kv = KVCache(model.s, max_ctx, kv_dtype) if use_cache else None
        self.kv_len = 0

    def last_hidden(self, tokens: Sequence[int]) -> np.ndarray:
        """Final-norm hidden state at the last of ``tokens``; afterwards the
        model holds keys/values for all of them."""
        n = len(tokens)
        if self.use_cache:
            assert self.kv.length == self.kv_len < n
            y = forward_chunk(self.m, self.kv, tokens[self.kv_len:n])[-1]
        else:
            y = forward_full(self.m, tokens, self.kv_dtype)[-1]
        self.kv_len = n
        return y

    def last_hiddens(self, tokens: Sequence[int], count: int) -> np.ndarray:
        """Final-norm hidden states at the last ``count`` of ``tokens`` (all of
        which the model must not have been fed yet)."""
        n = len(tokens)
        if self.use_cache:
            assert self.kv.length == self.kv_len <= n - count
            y = forward_chunk(self.m, self.kv, tokens[self.kv_len:n])[-count:]
        else:
            y = forward_full(self.m, tokens, self.kv_dtype)[-count:]
        self.kv_len = n
        return y

    def truncate(self, n: int) -> None:
        if n < self.kv_len:
            self.kv_len = n
            if self.use_cache:
                self.kv.truncate(n)


def gen_step(run: _Runner, tokens: List[int], u_row: np.ndarray, P: Params, margins: Optional[list] = None):
    """Generate one reasoning step with ``run``'s model, appending to
    ``tokens`` in place: sample until the separator or EOS has been appended,
    or the step holds step_cap tokens, or the context is full.  The uniform
    for the token placed at absolute position i is u_row[i].  Returns the
    step's tokens.  ``margins``, when given, collects the top-2 logit gap at
    every sampled position (used by parity tests to excuse near-ties)."""
    start = len(tokens)
    while True:
        y = run.last_hidden(tokens)
        lg = lm_logits(run.m, y).copy()
        lg[P.sep_id] += P.sep_logit_bias
        t = sample(lg, float(u_row[len(tokens)]), P.temperature, P.top_p)
        if margins is not None:                     # diagnostic only: gap between the two largest logits
            top2 = np.partition(lg, -2)[-2:]
            margins.append(float(top2[1] - top2[0]))
        tokens.append(t)
        n = len(tokens) - start
        if t == P.sep_id or t == P.eos_id or n >= P.step_cap or len(tokens) >= P.max_ctx:
            return tokens[start:]


def gen_step_sd(rd: _Runner, rt: _Runner, tokens: List[int], u_prop: np.ndarray, u_acc: np.ndarray,
                u_target: np.ndarray, P: Params, margins: Optional[list] = None,
                rounds: Optional[list] = None, prop_margins: Optional[list] = None,
                proposed: Optional[list] = None, draws: Optional[list] = None):
    """Generate one reasoning step of the target model by speculative decoding
    with the draft model (Section 5, "Combine RSD with SD"), appending to
    ``tokens`` in place; the step ends exactly as in ``gen_step``.

    Every round: with ``used`` tokens of the step so far, the draft proposes up
    to g = min(sd_k, step_cap - used - 1, max_ctx - len - 1) tokens one by one
    from its own distribution (uniform u_prop[position]), stopping early after a
    separator or EOS; the target reads the unseen tokens and the proposals in
    one pass and ``sd_verify`` decides (u_acc[position], and u_target[position]
    for a token the target draws itself).  Emitted tokens are appended until one
    of them ends the step.  Afterwards each model keeps keys/values only for the
    committed tokens it was fed, never for the newest one.

    ``rounds`` collects (proposed, kept) per round; ``margins`` the top-2 gap of
    the target's logits at every committed position and ``prop_margins`` that of
    the draft's at every proposal (diagnostics for parity tests); ``proposed``
    (place in the step, token) of every proposal; ``draws`` one entry per random
    decision with the logits it was taken on (what a parity test needs to judge
    whether a differing decision of another implementation lies within the reach
    of its logits' error): proposals ("prop"), acceptance tests up to a round's
    first refusal ("acc"), replacement draws ("res") and the target's own draw
    after a fully kept round ("tgt")."""
    def logits_of(run, y):
        lg = lm_logits(run.m, y).copy()
        lg[P.sep_id] += P.sep_logit_bias
        return lg

    def gap(lg):
        top2 = np.partition(lg, -2)[-2:]
        return float(top2[1] - top2[0])

    def uni(arr, i):                 # greedy decoding draws nothing: the arrays may be absent
        return 0.0 if arr is None else float(arr[i])

    start = len(tokens)
    while True:
        n = len(tokens)
        g = max(0, min(P.sd_k, P.step_cap - (n - start) - 1, P.max_ctx - n - 1))
        rd.truncate(n - 1)
        rt.truncate(n - 1)
        spec, q_rows, q_lgs = list(tokens), [], []
        for _ in range(g):
            lg = logits_of(rd, rd.last_hidden(spec))
            q = token_distribution(lg, P.temperature, P.top_p)
            x = draw(q, uni(u_prop, len(spec)))
            if prop_margins is not None:
                prop_margins.append(gap(lg))
            if proposed is not None:
                proposed.append((len(spec) - start, x))
            if draws is not None:
                draws.append(dict(kind="prop", place=len(spec) - start, lg=lg, u=uni(u_prop, len(spec)), tok=x))
            q_rows.append(q)
            q_lgs.append(lg)
            spec.append(x)
            if x == P.sep_id or x == P.eos_id:
                break
        props = spec[n:]
        ys = rt.last_hiddens(spec, len(props) + 1)
        lgs = [logits_of(rt, y) for y in ys]
        p_rows = [token_distribution(lg, P.temperature, P.top_p) for lg in lgs]
        emitted, kept = sd_verify(q_rows, p_rows, props, [uni(u_acc, n + i) for i in range(len(props))],
                                  [uni(u_target, n + i) for i in range(len(props) + 1)])
        if rounds is not None:
            rounds.append((len(props), kept))
        if draws is not None:
            for i in range(min(kept + 1, len(props))):
                draws.append(dict(kind="acc", place=n - start + i, lg_p=lgs[i], lg_q=q_lgs[i], u=uni(u_acc, n + i),
                                  tok=props[i], kept=i < kept))
            if kept < len(props):
                draws.append(dict(kind="res", place=n - start + kept, lg_p=lgs[kept], lg_q=q_lgs[kept],
                                  u=uni(u_target, n + kept), tok=emitted[kept]))
            else:
                draws.append(dict(kind="tgt", place=n - start + kept, lg=lgs[kept], u=uni(u_target, n + kept), tok=emitted[kept]))
        done = False
        for i, t in enumerate(emitted):
            tokens.append(t)
            if margins is not None:
                margins.append(gap(lgs[i]))
            if t == P.sep_id or t == P.eos_id or len(tokens) - start >= P.step_cap or len(tokens) >= P.max_ctx:
                done = True
                break
        rd.truncate(len(tokens) - 1)
        rt.truncate(len(tokens) - 1)
        if done:
            return tokens[start:]


def generate_sequence(draft: OracleModel, target: OracleModel, prm: OracleModel,
                      prompt: Sequence[int], u_draft: np.ndarray, u_target: np.ndarray,
                      u_gate: np.ndarray, P: Params, use_cache: bool = True,
                      max_steps: Optional[int] = None, u_prop: Optional[np.ndarray] = None,
                      u_acc: Optional[np.ndarray] = None, keep_draws: bool = False) -> dict:
    """RSD for one sequence (Algorithm 1 with the criterion of Algorithm 2).

    Returns the committed tokens, the per-step records and, after every step,
    how many leading tokens each model holds keys/values for (the target is
    only ever fed when a rejection needs it).

    P.merge = "draft" or "target" (Appendix "Model Merge": the reward model shares
    every layer below the heads with a policy model and keeps only its own
    projection): ``prm`` then contributes nothing but w_r and b_r, the reward is
    read off the final-norm hidden state of that policy model at the step's last
    token, and no third model or cache exists (its kv_len stays 0).  The policy
    model is fed up to the last token for this; afterwards it drops that one
    position again, so that its next use starts by feeding the last token, as
    it would without the merge."""
    delta = float(np.float32(P.delta))       # the threshold is an fp32 argument
    tokens = [int(t) for t in prompt]
    rd = _Runner(draft, P.max_ctx, use_cache, P.kv_dtype)
    rt = _Runner(target, P.max_ctx, use_cache, P.kv_dtype)
    rp = _Runner(prm, P.max_ctx, use_cache, P.kv_dtype)
    records = []
    reason = RUNNING
    n_steps = P.max_steps if max_steps is None else max_steps
    if len(tokens) >= P.max_ctx:
        reason = FIN_MAX_CTX
    for i in range(n_steps):
        if reason != RUNNING:
            break
        ctx_pre = len(tokens)
        dm, fm, pm, sd_rounds, proposed = [], [], [], [], []
        draws = [] if keep_draws else None
        draft_step = gen_step(rd, tokens, u_draft, P, dm)
        if P.merge == "none":
            r = reward(prm, rp.last_hidden(tokens))
        else:
            scorer = rd if P.merge == "draft" else rt
            r = reward(prm, scorer.last_hidden(tokens))
            scorer.truncate(len(tokens) - 1)
        ok = accept(r, P.omega_kind, delta, P.omega_a, float(u_gate[i]))
        if ok:
            final, fm = draft_step, dm
        else:
            del tokens[ctx_pre:]
            rd.truncate(ctx_pre)
            rp.truncate(ctx_pre)
            if P.merge == "target":
                rt.truncate(ctx_pre - 1)
            if P.sd_k > 0:
                final = gen_step_sd(rd, rt, tokens, u_prop, u_acc, u_target, P, fm, sd_rounds, pm, proposed, draws)
            else:
                final = gen_step(rt, tokens, u_target, P, fm)
        if P.eos_id >= 0 and P.eos_id in final:
            reason = FIN_EOS
        elif len(tokens) >= P.max_ctx:
            reason = FIN_MAX_CTX
        elif i + 1 >= P.max_steps:
            reason = FIN_MAX_STEPS
        kv = [rd.kv_len, rt.kv_len, rp.kv_len]
        records.append(dict(step=i, ctx_pre=ctx_pre, draft_tokens=list(draft_step), reward=r,
                            accepted=bool(ok), final_tokens=list(final), ctx_len=len(tokens),
                            kv_len=kv, n_pages=[-(-n // P.page_tokens) for n in kv],
                            draft_margins=dm, final_margins=fm, sd_rounds=sd_rounds, proposal_margins=pm, proposed=proposed,
                            draws=draws, finished=reason))
    return dict(tokens=tokens, prompt_len=len(prompt), records=records, finished=reason,
                kv_len=[rd.kv_len, rt.kv_len, rp.kv_len])


def generate_sequence_bon(draft: OracleModel, prm: OracleModel, prompt: Sequence[int], u_cand: np.ndarray,
                          P: Params, n_cand: int, max_steps: Optional[int] = None) -> dict:
    """Process Best-of-N for one sequence (Section 3, "Baselines"): at every
    reasoning step the base model samples ``n_cand`` candidate steps from the
    same committed context, the reward model scores each at its last token, and
    the candidate with the highest reward is committed (the lowest candidate
    index among equal rewards); generation stops as in the RSD loop (EOS in the
    committed step, context limit, step limit).

    ``u_cand[n][i]`` is the uniform of the token candidate ``n`` places at
    absolute position ``i``.  No cache is shared between candidates here: each
    one is evaluated on the whole prefix (committed tokens + its own step), with
    keys and values stored as ``P.kv_dtype`` says."""
    tokens = [int(t) for t in prompt]
    records = []
    reason = RUNNING
    n_steps = P.max_steps if max_steps is None else max_steps
    if len(tokens) >= P.max_ctx:
        reason = FIN_MAX_CTX
    for i in range(n_steps):
        if reason != RUNNING:
            break
        ctx_pre = len(tokens)
        cands, rewards, margins = [], [], []
        for n in range(n_cand):
            rd = _Runner(draft, P.max_ctx, False, P.kv_dtype)
            trial = list(tokens)
            mg: list = []
            step = gen_step(rd, trial, u_cand[n], P, mg)
            y = forward_full(prm, trial, P.kv_dtype)[-1]
            cands.append(step)
            rewards.append(reward(prm, y))
            margins.append(mg)
        # the decision is taken on the rewards as fp32 numbers (the precision they are reported in)
        r32 = np.asarray(rewards, dtype=np.float32)
        best = int(np.argmax(r32))                 # first index of the maximum
        tokens.extend(cands[best])
        if P.eos_id >= 0 and P.eos_id in cands[best]:
            reason = FIN_EOS
        elif len(tokens) >= P.max_ctx:
            reason = FIN_MAX_CTX
        elif i + 1 >= P.max_steps:
            reason = FIN_MAX_STEPS
        # caches after the step: the base model has been fed all but the newest token, the reward model all
        kv = [len(tokens) - 1, 0, len(tokens)]
        records.append(dict(step=i, ctx_pre=ctx_pre, candidates=cands, rewards=rewards, chosen=best,
                            final_tokens=list(cands[best]), ctx_len=len(tokens), kv_len=kv,
                            n_pages=[-(-v // P.page_tokens) for v in kv], margins=margins, finished=reason))
    return dict(tokens=tokens, prompt_len=len(prompt), records=records, finished=reason)


def decode_plain(model: OracleModel, prompt: Sequence[int], u_row: np.ndarray, P: Params,
                 n_tokens: int) -> List[int]:
    """Ordinary autoregressive decoding with one model and no cache: every
    token comes from a fresh forward over the whole prefix.  Steps play no
    role here; used to pin the fixed points of the gate."""
    tokens = [int(t) for t in prompt]
    for _ in range(n_tokens):
        lg = lm_logits(model, forward_full(model, tokens)[-1]).copy()
        lg[P.sep_id] += P.sep_logit_bias
        tokens.append(sample(lg, float(u_row[len(tokens)]), P.temperature, P.top_p))
    return tokens[len(prompt):]
