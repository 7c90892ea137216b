"""CPU oracle for Superposed Decoding (SPD).  TEST INFRASTRUCTURE ONLY.

A plain, slow, obviously-correct implementation of what one SPD generation computes,
written from the paper (arXiv 2405.18400) so that the HIP path can be compared with it.
Only the tests, the smoke check and the benchmark's CPU-baseline leg may import this file;
the product path never does.  It shares no code with the HIP path.

Arithmetic is numpy in a caller-chosen float type (float32 by default -- the precision the
comparison tolerances are stated for -- or float64 for self-checks).  Scores are kept as
natural-log probabilities: the paper's products of probabilities (Section 3, Eq. 2) become
sums.  There is no blocking, fusion or reordering: each function is the paper's formula
or Algorithm 1's step written out.

Readings taken where the paper is silent (each is an explicit option or documented here):
  * generation length G means G tokens per draft (1 from the prefix pass + G-1 steps);
  * temperature divides the logits of the full-vocabulary softmax, before KeepTopK, and
    the kept probabilities are not renormalised;
  * p_{n-gram}(x | ctx) = count(ctx, x) / sum_x' count(ctx, x') within the order-n table;
    an unseen context, an empty table or a history shorter than n-1 contributes 0;
  * "overlap" (Section 3.2) is judged per draft (option overlap="per_draft") or per
    (draft, token) pair (overlap="per_token");
  * alpha = 0 bypasses the n-gram stage altogether (the paper's smoothing-disabled mode);
  * ties: vocabulary top-k prefers the lower token id; the prune prefers the lower parent
    index, then the lower rank of the token among the kept k;
  * rotary embedding rotates adjacent pairs (x_{2i}, x_{2i+1}) by pos * theta^(-2i/d_head).

Parity pins: see tests/test_oracle_*.py.  "parity unpinned" items (nothing in the paper
fixes them): the value of delta, where the temperature applies, the rotary pairing
convention, the overlap granularity, the distribution a reset samples its draft from
(choose_draft: the superposition weights), and how the nucleus sampler breaks ties and maps
the caller's uniform draw to a token (nucleus_sample: inverse CDF in (probability
descending, id ascending) order).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

LAMBDAS_PAPER = (0.01, 0.04, 0.15, 0.18, 0.12)   # Appendix B, n = 2..6


# =============================================================================== LM forward
def _as_float(a: np.ndarray, dtype) -> np.ndarray:
    """Weights arrive as float32 or as bf16 bit patterns (uint16); widen the latter exactly."""
    if a.dtype == np.uint16:
        a = (a.astype(np.uint32) << 16).view(np.float32)
    return a.astype(dtype, copy=False)


def rmsnorm(x, gain, eps):
    """x * rsqrt(mean(x^2) + eps) * gain over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + x.dtype.type(eps)) * gain


def rope(x, positions, theta):
    """Rotary position embedding on x [T, n_heads, d_head]; pair (2i, 2i+1) turns by
    positions[t] * theta^(-2i/d_head)."""
    T, H, dh = x.shape
    i = np.arange(dh // 2, dtype=np.float64)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * theta ** (-2.0 * i / dh)[None, :]
    c = np.cos(ang).astype(x.dtype)[:, None, :]
    s = np.sin(ang).astype(x.dtype)[:, None, :]
    out = np.empty_like(x)
    xe, xo = x[..., 0::2], x[..., 1::2]
    out[..., 0::2] = xe * c - xo * s
    out[..., 1::2] = xe * s + xo * c
    return out


def silu(x):
    return x / (1 + np.exp(-x))


class OracleLM:
    """Decoder-only transformer f_theta (RMSNorm, rotary, SwiGLU, causal attention) run
    incrementally over one key/value cache that every draft shares (Section 3, "Next
    Timesteps": the model is conditioned on M and the superposed inputs so far)."""

    def __init__(self, weights: dict, n_layers: int, n_heads: int, n_kv_heads: int,
                 rms_eps: float = 1e-5, rope_theta: float = 10000.0, dtype=np.float32):
        self.w, self.L, self.H, self.Hkv = weights, n_layers, n_heads, n_kv_heads
        self.eps, self.theta, self.dtype = rms_eps, rope_theta, np.dtype(dtype)
        self.vocab, self.d = weights["embed"].shape
        self.dh = self.d // n_heads
        self.reset()

    def reset(self):
        self.pos = 0
        self.K = [np.zeros((0, self.Hkv, self.dh), self.dtype) for _ in range(self.L)]
        self.V = [np.zeros((0, self.Hkv, self.dh), self.dtype) for _ in range(self.L)]

    def W(self, name):
        return _as_float(self.w[name], self.dtype)

    def embedding_rows(self, tokens):
        return _as_float(self.w["embed"][np.asarray(tokens, dtype=np.int64)], self.dtype)

    def forward(self, X, all_positions: bool = False):
        """Feed T input vectors X [T, d] at positions pos..pos+T-1; append their keys and
        values to the cache; return the logits [V] at the last position (or [T, V])."""
        h = np.array(X, dtype=self.dtype, ndmin=2)
        T = h.shape[0]
        positions = np.arange(self.pos, self.pos + T)
        group = self.H // self.Hkv
        scale = self.dtype.type(1.0 / np.sqrt(self.dh))
        for l in range(self.L):
            p = f"layers.{l}."
            a = rmsnorm(h, self.W(p + "attn_norm"), self.eps)
            q = (a @ self.W(p + "wq").T).reshape(T, self.H, self.dh)
            k = (a @ self.W(p + "wk").T).reshape(T, self.Hkv, self.dh)
            v = (a @ self.W(p + "wv").T).reshape(T, self.Hkv, self.dh)
            q, k = rope(q, positions, self.theta), rope(k, positions, self.theta)
            self.K[l] = np.concatenate([self.K[l], k])
            self.V[l] = np.concatenate([self.V[l], v])
            att = np.empty((T, self.H, self.dh), self.dtype)
            for t in range(T):
                n_ctx = self.pos + t + 1                      # causal: positions 0..pos+t
                for hd in range(self.H):
                    kk, vv = self.K[l][:n_ctx, hd // group], self.V[l][:n_ctx, hd // group]
                    s = (kk @ q[t, hd]) * scale
                    e = np.exp(s - s.max())
                    att[t, hd] = (e / e.sum()) @ vv
            h = h + att.reshape(T, self.H * self.dh) @ self.W(p + "wo").T
            b = rmsnorm(h, self.W(p + "ffn_norm"), self.eps)
            u = silu(b @ self.W(p + "w_gate").T) * (b @ self.W(p + "w_up").T)
            h = h + u @ self.W(p + "w_down").T
        self.pos += T
        hn = rmsnorm(h if all_positions else h[-1:], self.W("final_norm"), self.eps)
        logits = hn @ self.W("lm_head").T
        return logits if all_positions else logits[0]


# =============================================================================== n-grams
class NgramTables:
    """Frequency tables for n = 2..6: every stored n-gram with its count (Section 4).
    Lookups are exhaustive scans of the raw arrays -- the definition, not an index."""

    def __init__(self, tables: dict):
        self.t = {}
        for n in range(2, 7):
            keys, counts = tables.get(n, (np.zeros((0, n), np.int32), np.zeros((0,), np.uint32)))
            keys = np.asarray(keys, dtype=np.int64).reshape(-1, n)
            self.t[n] = (keys, np.asarray(counts, dtype=np.uint64))

    def count(self, gram) -> int:
        keys, counts = self.t[len(gram)]
        if len(keys) == 0:
            return 0
        hit = np.all(keys == np.asarray(gram, dtype=np.int64), axis=1)
        return int(counts[hit].sum())

    def context_total(self, n: int, ctx) -> int:
        keys, counts = self.t[n]
        if len(keys) == 0:
            return 0
        hit = np.all(keys[:, : n - 1] == np.asarray(ctx, dtype=np.int64), axis=1)
        return int(counts[hit].sum())

    def prob(self, n: int, history, tok: int, dtype=np.float32):
        """p_{n-gram}(tok | last n-1 tokens of history); 0 if that cannot be formed."""
        dt = np.dtype(dtype).type
        if len(history) < n - 1:
            return dt(0)
        ctx = list(history[len(history) - (n - 1):])
        total = self.context_total(n, ctx)
        if total == 0:
            return dt(0)
        return dt(self.count(ctx + [int(tok)])) / dt(total)


def p_ngram(tables: NgramTables, lambdas, history, tok: int, dtype=np.float32):
    """Section 3.2, Eq. 3: sum over n = 2..6 of lambda_n * p_{n-gram}(tok | history)."""
    dt = np.dtype(dtype).type
    acc = dt(0)
    for n in range(2, 7):
        acc = acc + dt(lambdas[n - 2]) * tables.prob(n, history, tok, dtype)
    return acc


# =============================================================================== SPD pieces
@dataclass
class DecodeCfg:
    k: int = 3
    alpha: float = 0.54          # interpolation weight (Appendix B)
    tau: float = 1.0             # temperature
    delta: float = 0.1           # no-overlap penalty; the paper gives no value
    lambdas: tuple = LAMBDAS_PAPER
    overlap: str = "per_draft"   # or "per_token"


def log_softmax_tau(logits, tau, dtype=np.float32):
    """log p_theta over the full vocabulary with temperature."""
    z = np.asarray(logits, dtype=dtype) / np.dtype(dtype).type(tau)
    m = z.max()
    return z - (m + np.log(np.sum(np.exp(z - m), dtype=dtype)))


def top_k_ids(values, k: int):
    """Indices of the k largest entries, largest first; equal values -> lower index first."""
    values = np.asarray(values)
    order = np.lexsort((np.arange(len(values)), -values))
    return order[:k].astype(np.int64)


def superposition_weights(logscores):
    """Section 3.1, Eq. 2: gamma_i = p_i / sum_j p_j, from log p_i."""
    s = np.asarray(logscores)
    e = np.exp(s - s.max())
    return e / e.sum(dtype=s.dtype)


def superposed_embedding(rows, gamma):
    """Section 3.1, Eq. 1: x~ = sum_i gamma_i * z_i, rows = the drafts' last-token
    embeddings z_i [k, d]."""
    acc = np.zeros(rows.shape[1], rows.dtype)
    for i in range(rows.shape[0]):
        acc = acc + gamma[i] * rows[i]
    return acc


@dataclass
class Candidate:
    parent: int      # index i of the draft it extends
    rank: int        # rank j of its token among the kept top-k
    token: int
    logscore: float  # log p_i + log p_f
    overlap: bool    # True: Eq. 4 (interpolated); False: Eq. 5 (delta form) or alpha = 0


@dataclass
class StepRecord:
    logits: np.ndarray | None
    top_ids: np.ndarray            # kept k token ids, most probable first
    top_logp: np.ndarray           # their log p_theta (full-vocabulary softmax)
    candidates: list               # every candidate draft option of this step
    kept: list                     # the k surviving Candidates, best first
    gamma_in: np.ndarray | None    # superposition weights that formed this step's input
    gap_vocab: float               # min gap between adjacent logits among ranks 1..k+1
    gap_prune: float               # min gap between adjacent candidate scores, ranks 1..k+1
    pngram: np.ndarray | None = None   # [k, k] mixture values p_ngram(i, j)
    state_in: "SpdState | None" = None  # the drafts and scores this step started from


@dataclass
class SpdState:
    prefix: list
    drafts: list = field(default_factory=list)        # generated tokens of each draft
    logscores: np.ndarray | None = None

    def history(self, i):
        return list(self.prefix) + list(self.drafts[i])


def _adjacent_gap(sorted_desc, upto):
    v = np.asarray(sorted_desc, dtype=np.float64)[: upto + 1]
    return float(np.min(v[:-1] - v[1:])) if len(v) > 1 else float("inf")


def first_step(logits, prefix, cfg: DecodeCfg, dtype=np.float32, keep_logits=True):
    """Section 3, "First Timestep": draft i takes the i-th most probable token of
    p_theta(. | M); its score is that token's probability.  No n-gram term."""
    logp = log_softmax_tau(logits, cfg.tau, dtype)
    ids = top_k_ids(logits, cfg.k)
    state = SpdState(list(map(int, prefix)), [[int(t)] for t in ids], logp[ids].astype(dtype))
    srt = np.sort(np.asarray(logits, dtype=np.float64))[::-1]
    cands = [Candidate(-1, j, int(ids[j]), float(logp[ids[j]]), False) for j in range(len(ids))]
    rec = StepRecord(np.array(logits) if keep_logits else None, ids, logp[ids], cands, list(cands),
                     None, _adjacent_gap(srt, cfg.k), float("inf"))
    return state, rec


def expand_and_prune(state: SpdState, logits, tables: NgramTables | None, cfg: DecodeCfg,
                     dtype=np.float32, keep_logits=True, gamma_in=None):
    """One "next timestep" after the forward pass (Algorithm 1, else-branch): KeepTopK,
    per-draft n-gram distribution, interpolation (Eq. 4 / Eq. 5), k^2 options, TopK."""
    dt = np.dtype(dtype).type
    k = len(state.drafts)
    logp = log_softmax_tau(logits, cfg.tau, dtype)
    ids = top_k_ids(logits, cfg.k)
    a = dt(cfg.alpha)
    cands, png = [], None
    if cfg.alpha == 0:
        for i in range(k):
            for j, tok in enumerate(ids):
                cands.append(Candidate(i, j, int(tok), dt(state.logscores[i]) + logp[tok], False))
    else:
        png = np.zeros((k, len(ids)), dtype)
        log_delta = np.log(dt(cfg.delta))
        for i in range(k):
            hist = state.history(i)
            for j, tok in enumerate(ids):
                png[i, j] = p_ngram(tables, cfg.lambdas, hist, int(tok), dtype)
            any_overlap = bool(np.any(png[i] > 0))
            for j, tok in enumerate(ids):
                lm_term = (dt(1) - a) * logp[tok]
                if png[i, j] > 0:
                    lpf, ov = lm_term + a * np.log(png[i, j]), True          # Eq. 4
                elif cfg.overlap == "per_draft" and any_overlap:
                    continue                              # token not in both distributions
                else:
                    lpf, ov = log_delta + lm_term, False                     # Eq. 5
                cands.append(Candidate(i, j, int(tok), dt(state.logscores[i]) + lpf, ov))
    order = sorted(range(len(cands)), key=lambda c: (-float(cands[c].logscore), cands[c].parent, cands[c].rank))
    kept = [cands[c] for c in order[:k]]
    new = SpdState(state.prefix, [state.drafts[c.parent] + [c.token] for c in kept],
                   np.array([c.logscore for c in kept], dtype=dtype))
    srt = np.sort(np.asarray(logits, dtype=np.float64))[::-1]
    rec = StepRecord(np.array(logits) if keep_logits else None, ids, logp[ids], cands, kept, gamma_in,
                     _adjacent_gap(srt, cfg.k),
                     _adjacent_gap([cands[c].logscore for c in order], k), png, state)
    return new, rec


def generate(lm, tables, prefix, cfg: DecodeCfg, n_tokens: int, dtype=np.float32, keep_logits=True):
    """Algorithm 1: k drafts of n_tokens tokens each from one pass per timestep.
    `lm` needs reset(), embedding_rows(tokens) and forward(X) -> logits of the last position.
    Returns (final SpdState with drafts best-first, list of per-timestep StepRecords)."""
    lm.reset()
    logits = lm.forward(lm.embedding_rows(prefix))
    state, rec = first_step(logits, prefix, cfg, dtype, keep_logits)
    records = [rec]
    for _ in range(1, n_tokens):
        gamma = superposition_weights(state.logscores)
        x = superposed_embedding(lm.embedding_rows([d[-1] for d in state.drafts]), gamma.astype(dtype))
        logits = lm.forward(x[None, :])
        state, rec = expand_and_prune(state, logits, tables, cfg, dtype, keep_logits, gamma)
        records.append(rec)
    return state, records


# ===================================================================== nucleus sampling
# The comparison decoder of Section 4.3 (one of k independent passes): Section 2 describes it
# as truncating the next-token distribution to the smallest set of tokens whose cumulative
# probability reaches p, then sampling from the renormalised set.  Readings: the cumulative
# probability has to reach (>=) p; the vocabulary is ordered by probability descending with
# the lower token id first among equals, the nucleus is the shortest prefix of that order,
# and the draw u in [0, 1) picks the first token whose cumulative probability within that
# order exceeds u times the nucleus mass (inverse CDF).  The temperature divides the logits
# of the full-vocabulary softmax, as for SPD.  The uniform number u is an input.
@dataclass
class NucleusRecord:
    token: int
    logp: float            # log p_theta(token) under the full-vocabulary softmax
    nucleus_size: int
    nucleus_mass: float
    margin_sample: float   # distance of u * mass to the nearer cumulative boundary of the chosen token
    margin_nucleus: float  # distance of p to the nearer cumulative boundary at the nucleus edge
    p_edge: float          # probability of the token just past the nucleus (0 if none)
    logits: np.ndarray | None = None


def nucleus_sample(logits, top_p: float, tau: float, u: float, keep_logits: bool = False) -> NucleusRecord:
    lp = log_softmax_tau(np.asarray(logits), tau, np.float64)
    p = np.exp(lp)
    order = np.lexsort((np.arange(p.size), -p))          # probability descending, then id ascending
    cs = np.cumsum(p[order])
    n = int(np.searchsorted(cs, top_p, side="left"))     # first index with cs >= top_p
    n = min(n, p.size - 1)
    mass = float(cs[n])
    target = u * mass
    j = int(np.searchsorted(cs[: n + 1], target, side="right"))   # first index with cs > target
    j = min(j, n)
    lo = float(cs[j - 1]) if j > 0 else 0.0
    below = float(cs[n - 1]) if n > 0 else 0.0
    return NucleusRecord(token=int(order[j]), logp=float(lp[order[j]]), nucleus_size=n + 1, nucleus_mass=mass,
                         margin_sample=min(target - lo, float(cs[j]) - target),
                         margin_nucleus=min(top_p - below, mass - top_p),
                         p_edge=float(p[order[n + 1]]) if n + 1 < p.size else 0.0,
                         logits=np.asarray(logits).copy() if keep_logits else None)


def nucleus_generate(lm, prefix, top_p: float, tau: float, us, keep_logits: bool = False):
    """One pass of nucleus sampling: len(us) tokens after `prefix`, us[t] the draw of token t.
    Returns (tokens, sum of their log-probabilities, records)."""
    lm.reset()
    logits = lm.forward(lm.embedding_rows(np.asarray(prefix, dtype=np.int64)))
    toks, recs, total = [], [], 0.0
    for t, u in enumerate(us):
        if t > 0:
            logits = lm.forward(lm.embedding_rows(np.asarray([toks[-1]], dtype=np.int64)))
        rec = nucleus_sample(logits, top_p, tau, float(u), keep_logits)
        toks.append(rec.token)
        total += rec.logp
        recs.append(rec)
    return toks, total, recs


# ================================================================ resets and the splice
# Section 5.3 ("Superposed Decoding Resets"): every s timesteps one of the k drafts is
# sampled and draft generation restarts from the text extended by it.  Section 4.5: a
# nucleus-sampled generation can serve as the prefix, whatever timestep it ends at.  Both are
# "commit one draft, restart from the longer prefix".  Reading: the draft is sampled with its
# superposition weight gamma_i = p_i / sum_j p_j (Eq. 2) -- the paper only says "sample" --
# by inverse CDF over the drafts in rank order with a draw u in [0, 1) supplied by the caller.
def choose_draft(logscores, u: float) -> int:
    gamma = superposition_weights(logscores).astype(np.float64)
    cum = np.cumsum(gamma)
    i = int(np.searchsorted(cum, u * cum[-1], side="right"))
    return min(i, len(gamma) - 1)


def commit_draft(state: SpdState, u: float):
    """-> (index of the sampled draft, the new prefix = old prefix + that draft)."""
    i = choose_draft(state.logscores, u)
    return i, list(state.prefix) + list(state.drafts[i])


def generate_with_resets(lm, tables, prefix, cfg: DecodeCfg, n_tokens: int, s: int, us, dtype=np.float32):
    """n_tokens tokens per draft in segments of s timesteps; after each full segment one draft
    is committed (draw us[j] for the j-th reset) and generation restarts.  Returns (committed
    text beyond the original prefix, final SpdState of the last segment, chosen indices)."""
    text, chosen, left, j = list(map(int, prefix)), [], n_tokens, 0
    state = None
    while left > 0:
        seg = min(s, left)
        state, _ = generate(lm, tables, text, cfg, seg, dtype, keep_logits=False)
        left -= seg
        if left > 0:
            i, text = commit_draft(state, float(us[j]))
            chosen.append(i)
            j += 1
    return text[len(prefix):], state, chosen
