"""Pins for the oracle's decoding logic: what the paper and the mathematics fix."""
import itertools
import math

import numpy as np
import pytest

import synth
from helpers import oracle_lm, toy_shape
from oracle import spd_oracle as O
from test_oracle_ngram import corpus_tables


class ScriptedLM:
    """Stands in for f_theta: returns prescribed logits per call, records its inputs."""

    def __init__(self, logits_per_call, vocab, d=4):
        self.script, self.E = logits_per_call, np.eye(vocab, d, dtype=np.float64) + 0.1
        self.inputs = []

    def reset(self):
        self.calls = 0
        self.inputs = []

    def embedding_rows(self, tokens):
        return self.E[np.asarray(tokens)]

    def forward(self, X):
        self.inputs.append(np.array(X))
        self.calls += 1
        return np.asarray(self.script[self.calls - 1], dtype=np.float64)


def toy_tables(vocab, seed=0, length=400):
    rng = np.random.default_rng(seed)
    corpus = list(rng.integers(0, vocab, size=length))
    return corpus, corpus_tables(corpus)


# ------------------------------------------------------------------ 1. k = 1 is greedy decoding
@pytest.mark.parametrize("alpha,delta", [(0.0, 0.1), (0.54, 0.1), (0.54, 1e-3)])
def test_k1_is_greedy(alpha, delta):
    shape = toy_shape(vocab=32, d=32, heads=4, kv=4, ffn=64, layers=2)
    lm, w = oracle_lm(shape, seed=11)
    corpus, tabs = toy_tables(32, 1)
    prefix = corpus[:6]
    state, recs = O.generate(lm, O.NgramTables(tabs), prefix, O.DecodeCfg(1, alpha, 1.0, delta), 8)
    # independent greedy loop: feed back the argmax token's own embedding
    g, _ = oracle_lm(shape, weights=w)
    logits = g.forward(g.embedding_rows(prefix))
    greedy = []
    for _ in range(8):
        tok = int(np.argmax(logits))
        greedy.append(tok)
        logits = g.forward(g.embedding_rows([tok]))
    assert state.drafts[0] == greedy
    assert all(np.array_equal(r.gamma_in, [1.0]) for r in recs[1:])


# ------------------------------------------------------------------ 2. superposition weights
def test_gamma_is_normalised_probability():
    s = np.log(np.array([0.2, 0.05, 0.0125], np.float64))
    g = O.superposition_weights(s)
    np.testing.assert_allclose(g, np.array([0.2, 0.05, 0.0125]) / 0.2625, rtol=1e-14)
    g32 = O.superposition_weights(np.array([-300.0, -301.0, -305.0], np.float32))  # products would underflow
    assert abs(float(g32.sum()) - 1.0) < 1e-6 and np.all(g32 >= 0) and g32[0] > g32[1] > g32[2]
    rows = np.array([[1.0, 0.0], [0.0, 2.0], [4.0, 4.0]])
    np.testing.assert_allclose(O.superposed_embedding(rows, np.array([0.5, 0.25, 0.25])), [1.5, 1.5])


def test_gamma_sums_to_one_every_step_and_input_is_the_weighted_embedding_sum():
    vocab = 12
    rng = np.random.default_rng(3)
    script = rng.standard_normal((6, vocab)) * 2
    lm = ScriptedLM(script, vocab, d=vocab)
    state, recs = O.generate(lm, None, [1, 2, 3], O.DecodeCfg(3, 0.0), 6, dtype=np.float64)
    prev_tokens, prev_scores = [c.token for c in recs[0].kept], [c.logscore for c in recs[0].kept]
    for t, rec in enumerate(recs[1:], start=1):
        assert abs(rec.gamma_in.sum() - 1) < 1e-12 and np.all(rec.gamma_in >= 0)
        p = np.exp(np.array(prev_scores))
        np.testing.assert_allclose(rec.gamma_in, p / p.sum(), rtol=1e-12)
        np.testing.assert_allclose(lm.inputs[t][0], (p / p.sum()) @ lm.E[prev_tokens], rtol=1e-12)
        prev_tokens, prev_scores = [c.token for c in rec.kept], [c.logscore for c in rec.kept]


# ------------------------------------------------------------------ 3. expansion + prune = brute force
def test_alpha0_prune_equals_brute_force_over_all_k_times_V_pairs():
    """Without n-grams, restricting to the LM's top-k tokens loses nothing: the k best of
    all (draft, token) pairs are found."""
    vocab, k = 16, 3
    shape = toy_shape(vocab=vocab, d=16, heads=2, kv=2, ffn=32, layers=1)
    lm, _ = oracle_lm(shape, seed=2, dtype=np.float64)
    state, recs = O.generate(lm, None, [3, 1, 4], O.DecodeCfg(k, 0.0), 7, dtype=np.float64)
    scores = [c.logscore for c in recs[0].kept]
    drafts = [[c.token] for c in recs[0].kept]
    for rec in recs[1:]:
        logp = rec.logits - np.log(np.sum(np.exp(rec.logits)))
        allpairs = sorted(((scores[i] + logp[x], i, x) for i in range(k) for x in range(vocab)), reverse=True)[:k]
        got = [(c.logscore, c.parent, c.token) for c in rec.kept]
        for (ws, wi, wx), (gs, gi, gx) in zip(allpairs, got):
            assert (wi, wx) == (gi, gx) and abs(ws - gs) < 1e-12
        drafts = [drafts[i] + [x] for _, i, x in allpairs]
        scores = [s for s, _, _ in allpairs]
    assert drafts == state.drafts


@pytest.mark.parametrize("overlap", ["per_draft", "per_token"])
def test_interpolated_prune_equals_brute_force_over_k_times_k_pairs(overlap):
    vocab, k, alpha, delta = 8, 3, 0.54, 0.1
    corpus, tabs = toy_tables(6, 5, 300)          # tokens 6 and 7 never occur: unseen contexts
    lam = O.LAMBDAS_PAPER
    rng = np.random.default_rng(8)
    script = rng.standard_normal((6, vocab))
    script[0, 6] = 5.0                            # a first-timestep draft ends in an unseen token
    lm = ScriptedLM(script, vocab)
    prefix = corpus[10:13]
    cfg = O.DecodeCfg(k, alpha, 1.0, delta, lam, overlap)
    state, recs = O.generate(lm, O.NgramTables(tabs), prefix, cfg, 6, dtype=np.float64)

    def png(hist, x):   # the test's own n-gram model: straight recount over the corpus
        tot = 0.0
        for n in range(2, 7):
            if len(hist) < n - 1:
                continue
            ctx = hist[len(hist) - (n - 1):]
            den = sum(1 for i in range(len(corpus) - n + 1) if corpus[i:i + n - 1] == ctx)
            num = sum(1 for i in range(len(corpus) - n + 1) if corpus[i:i + n] == ctx + [x])
            tot += lam[n - 2] * (num / den if den else 0.0)
        return tot

    drafts = [[c.token] for c in recs[0].kept]
    scores = [c.logscore for c in recs[0].kept]
    saw_overlap = saw_fallback = saw_dropped = False
    for step, rec in enumerate(recs[1:], start=1):
        p = np.exp(script[step]) / np.exp(script[step]).sum()
        top = sorted(range(vocab), key=lambda x: (-p[x], x))[:k]
        options = []
        for i in range(k):
            hist = list(prefix) + drafts[i]
            ng = [png(hist, x) for x in top]
            for j, x in enumerate(top):
                if ng[j] > 0:
                    pf = p[x] ** (1 - alpha) * ng[j] ** alpha
                    saw_overlap = True
                elif overlap == "per_draft" and any(v > 0 for v in ng):
                    saw_dropped = True
                    continue
                else:
                    pf = delta * p[x] ** (1 - alpha)
                    saw_fallback = True
                options.append((math.exp(scores[i]) * pf, i, x))
        assert len(options) >= k
        best = sorted(options, key=lambda o: -o[0])[:k]
        assert [(i, x) for _, i, x in best] == [(c.parent, c.token) for c in rec.kept]
        np.testing.assert_allclose([math.log(s) for s, _, _ in best], [c.logscore for c in rec.kept], rtol=1e-10)
        assert len(rec.candidates) == len(options)
        drafts = [drafts[i] + [x] for _, i, x in best]
        scores = [math.log(s) for s, _, _ in best]
    assert saw_overlap and saw_fallback and (saw_dropped or overlap == "per_token")
    assert drafts == state.drafts


# ------------------------------------------------------------------ 4. alpha = 0: product of LM probabilities
def test_alpha0_score_is_product_of_the_models_own_probabilities():
    shape = toy_shape(vocab=40, d=32, heads=4, kv=2, ffn=64, layers=2)
    lm, _ = oracle_lm(shape, seed=9)
    state, recs = O.generate(lm, None, [5, 6, 7, 8], O.DecodeCfg(3, 0.0, tau=0.7), 9)
    for i, draft in enumerate(state.drafts):
        prod = 1.0
        for t, tok in enumerate(draft):
            z = recs[t].logits.astype(np.float64) / 0.7
            prod *= math.exp(z[tok]) / np.exp(z).sum()
        assert abs(math.log(prod) - float(state.logscores[i])) < 2e-5
    # log-domain fp32 sums agree with a float64 rerun
    lm64, _ = oracle_lm(shape, seed=9, dtype=np.float64)
    s64, _ = O.generate(lm64, None, [5, 6, 7, 8], O.DecodeCfg(3, 0.0, tau=0.7), 9, dtype=np.float64)
    assert s64.drafts == state.drafts
    np.testing.assert_allclose(state.logscores, s64.logscores, rtol=1e-5)


# ------------------------------------------------------------------ hand-worked step
def test_hand_worked_step():
    """vocab 4, k = 2.  p_theta fixed by the script; bigram table by hand."""
    p1 = np.array([0.5, 0.3, 0.15, 0.05])           # first timestep: drafts (0), (1); scores .5, .3
    p2 = np.array([0.1, 0.2, 0.3, 0.4])             # second: kept tokens 3 (p .4) and 2 (p .3)
    tabs = O.NgramTables({2: (np.array([[0, 3], [0, 1], [1, 0]]), np.array([1, 3, 5]))})
    # draft (..,0): p_2gram(3|0) = 1/4, p_2gram(2|0) = 0  -> overlap {3}: only token 3 survives
    # draft (..,1): context 1 has continuations {0} only -> no overlap -> delta form for both
    lam, alpha, delta = (0.5, 0, 0, 0, 0), 0.5, 0.1
    lm = ScriptedLM([np.log(p1), np.log(p2)], 4)
    state, recs = O.generate(lm, tabs, [2], O.DecodeCfg(2, alpha, 1.0, delta, lam), 2, dtype=np.float64)
    a = 0.5 * math.sqrt(0.4) * math.sqrt(0.5 * 0.25)          # draft 0 + token 3, Eq. 4
    b = 0.3 * delta * math.sqrt(0.4)                          # draft 1 + token 3, Eq. 5
    c = 0.3 * delta * math.sqrt(0.3)                          # draft 1 + token 2, Eq. 5
    assert [(x.parent, x.token) for x in recs[1].candidates] == [(0, 3), (1, 3), (1, 2)]
    np.testing.assert_allclose([math.exp(x.logscore) for x in recs[1].candidates], [a, b, c], rtol=1e-12)
    assert a > b > c
    assert state.drafts == [[0, 3], [1, 3]]
    np.testing.assert_allclose(np.exp(state.logscores), [a, b], rtol=1e-12)
    np.testing.assert_allclose(recs[1].gamma_in, [0.625, 0.375], rtol=1e-12)
    np.testing.assert_allclose(lm.inputs[1][0], 0.625 * lm.E[0] + 0.375 * lm.E[1], rtol=1e-12)
    # per-token reading keeps (0, 2) with the delta form as a fourth option
    s2, r2 = O.generate(lm, tabs, [2], O.DecodeCfg(2, alpha, 1.0, delta, lam, "per_token"), 2, dtype=np.float64)
    assert [(x.parent, x.token) for x in r2[1].candidates] == [(0, 3), (0, 2), (1, 3), (1, 2)]
    np.testing.assert_allclose(math.exp(r2[1].candidates[1].logscore), 0.5 * delta * math.sqrt(0.3), rtol=1e-12)


# ------------------------------------------------------------------ 5-7. invariants
@pytest.mark.parametrize("alpha", [0.0, 0.54])
def test_drafts_distinct_ordered_and_cache_grows_by_one(alpha):
    shape = toy_shape(vocab=32, d=32, heads=4, kv=4, ffn=64, layers=2)
    lm, _ = oracle_lm(shape, seed=4)
    corpus, tabs = toy_tables(32, 2)
    k, G, m = 4, 8, 5
    lens = []
    orig = lm.forward
    lm.forward = lambda X: (lens.append(lm.pos), orig(X))[1]
    state, recs = O.generate(lm, O.NgramTables(tabs), corpus[:m], O.DecodeCfg(k, alpha), G)
    assert lens == [0] + list(range(m, m + G - 1)) and lm.pos == m + G - 1
    assert all(len(d) == G for d in state.drafts) and len(recs) == G
    assert len({tuple(d) for d in state.drafts}) == k
    for rec in recs:
        sc = [c.logscore for c in rec.kept]
        assert all(sc[i] >= sc[i + 1] for i in range(len(sc) - 1))
        assert len(rec.candidates) >= k
    # first timestep: draft i holds the i-th most probable token
    z = recs[0].logits
    assert [d[0] for d in state.drafts] != [] and list(recs[0].top_ids) == sorted(range(32), key=lambda x: (-z[x], x))[:k]


def test_ties_lower_token_id_then_lower_parent_then_lower_rank():
    assert list(O.top_k_ids(np.array([1.0, 3.0, 3.0, 0.0, 3.0]), 3)) == [1, 2, 4]
    # two drafts with equal scores and a flat LM: prune keeps (0, j0), (0, j1)
    lm = ScriptedLM([np.zeros(4), np.zeros(4)], 4)
    state, recs = O.generate(lm, None, [0], O.DecodeCfg(2, 0.0), 2, dtype=np.float64)
    assert [(c.parent, c.token) for c in recs[1].kept] == [(0, 0), (0, 1)]


def test_temperature_rescales_probabilities_but_not_the_kept_ids():
    z = np.random.default_rng(1).standard_normal(50)
    for tau in (0.06, 0.5, 1.0, 3.0):
        st, rec = O.first_step(z, [0], O.DecodeCfg(4, 0.0, tau), np.float64)
        assert list(rec.top_ids) == list(np.argsort(-z)[:4])
        np.testing.assert_allclose(np.exp(rec.top_logp), (np.exp(z / tau) / np.exp(z / tau).sum())[rec.top_ids], rtol=1e-10)


def test_lower_delta_never_promotes_an_uninterpolated_option():
    vocab, k = 8, 3
    corpus, tabs = toy_tables(6, 5, 300)
    rng = np.random.default_rng(8)
    script = rng.standard_normal((2, vocab))
    script[0, 6] = 5.0
    kept = {}
    for delta in (1.0, 0.1, 1e-3):
        lm = ScriptedLM(script, vocab)
        _, recs = O.generate(lm, O.NgramTables(tabs), corpus[10:13], O.DecodeCfg(k, 0.54, 1.0, delta), 2, dtype=np.float64)
        kept[delta] = sum(1 for c in recs[1].kept if not c.overlap)
    assert kept[1.0] >= kept[0.1] >= kept[1e-3]
