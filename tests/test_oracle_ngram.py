"""Pins for the oracle's n-gram stage: recount on a toy corpus, closed forms, printed values."""
import itertools
import os
from collections import Counter

import numpy as np
import pytest

import synth
from helpers import read_golden
from oracle import spd_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden", "hyperparameters.txt")


def corpus_tables(corpus, orders=range(2, 7)):
    """Frequency tables built the way Section 4 describes: one entry per distinct n-gram, holding how often it occurs."""
    tabs = {}
    for n in orders:
        c = Counter(tuple(corpus[i:i + n]) for i in range(len(corpus) - n + 1))
        tabs[n] = (np.array(list(c.keys()), np.int32).reshape(-1, n), np.array(list(c.values()), np.uint32))
    return tabs


@pytest.fixture(scope="module")
def toy():
    rng = np.random.default_rng(0)
    corpus = list(rng.integers(0, 6, size=200))
    return corpus, O.NgramTables(corpus_tables(corpus))


def test_printed_hyperparameters():
    g = read_golden(GOLD)
    assert list(O.LAMBDAS_PAPER) == g["lambda_2_to_6"] == list(synth.PAPER_LAMBDAS)
    assert abs(sum(O.LAMBDAS_PAPER) - 0.50) < 1e-12          # printed weights sum to 0.5, used as is
    assert O.DecodeCfg().alpha == g["alpha"][0]
    mb = g["table_mb_2_to_6"]
    share = np.array([mb[i] / (i + 2) for i in range(5)])
    np.testing.assert_allclose(synth.ORDER_SHARE, share / share.sum(), rtol=1e-12)


def test_probability_is_recount_ratio_on_toy_corpus(toy):
    corpus, tabs = toy
    for n in range(2, 7):
        for start in range(0, 150, 7):
            ctx = corpus[start:start + n - 1]
            for tok in range(6):
                num = sum(1 for i in range(len(corpus) - n + 1) if corpus[i:i + n] == ctx + [tok])
                den = sum(1 for i in range(len(corpus) - n + 1) if corpus[i:i + n - 1] == ctx)
                got = tabs.prob(n, [9, 9, 9] + ctx, tok, np.float64)   # only the last n-1 tokens matter
                assert got == num / den


def test_conditional_distribution_sums_to_one_for_seen_contexts(toy):
    corpus, tabs = toy
    for n in range(2, 7):
        ctx = corpus[20:20 + n - 1]
        assert abs(sum(tabs.prob(n, ctx, t, np.float64) for t in range(6)) - 1.0) < 1e-12


def test_unseen_context_short_history_and_empty_table_contribute_zero(toy):
    corpus, tabs = toy
    assert tabs.prob(3, [7, 7], 1) == 0                       # context never seen
    assert tabs.prob(4, [1, 2], 1) == 0                       # history shorter than n-1
    empty = O.NgramTables({})
    assert O.p_ngram(empty, O.LAMBDAS_PAPER, [1, 2, 3, 4, 5], 1) == 0
    # m = 1: only the bigram order can fire
    lam = (1.0, 1.0, 1.0, 1.0, 1.0)
    assert O.p_ngram(tabs, lam, [corpus[0]], corpus[1], np.float64) == tabs.prob(2, [corpus[0]], corpus[1], np.float64)


def test_mixture_is_lambda_weighted_sum_as_printed(toy):
    corpus, tabs = toy
    hist = corpus[50:55]
    tok = corpus[55]
    parts = [tabs.prob(n, hist, tok, np.float64) for n in range(2, 7)]
    assert all(p > 0 for p in parts)
    want = 0.01 * parts[0] + 0.04 * parts[1] + 0.15 * parts[2] + 0.18 * parts[3] + 0.12 * parts[4]
    assert abs(O.p_ngram(tabs, O.LAMBDAS_PAPER, hist, tok, np.float64) - want) < 1e-15
    assert O.p_ngram(tabs, O.LAMBDAS_PAPER, hist, tok, np.float64) <= 0.5
    # hand-sized case: bigram table {(1,2):3, (1,3):1}: p(2|1) = 3/4
    t = O.NgramTables({2: (np.array([[1, 2], [1, 3]]), np.array([3, 1]))})
    assert t.prob(2, [5, 1], 2, np.float64) == 0.75 and t.context_total(2, [1]) == 4 and t.count([1, 3]) == 1
    assert O.p_ngram(t, O.LAMBDAS_PAPER, [5, 1], 2, np.float64) == 0.01 * 0.75


def test_synthetic_tables_have_distinct_keys_and_positive_counts():
    for tabs in (synth.make_ngram_tables_uniform(64, {2: 500, 3: 700}, seed=1),
                 synth.make_ngram_tables_zipf(100, 5000, seed=2)):
        for n, (keys, counts) in tabs.items():
            assert keys.shape == (len(counts), n) and keys.dtype == np.int32 and counts.dtype == np.uint32
            assert len(np.unique(keys, axis=0)) == len(keys)
            assert np.all(counts > 0)
    u = synth.make_ngram_tables_uniform(64, {2: 500, 3: 700}, seed=1)
    assert len(u[2][0]) == 500 and len(u[3][0]) == 700 and len(u[4][0]) == 0


def test_planting_makes_visited_ngrams_hit():
    base = synth.make_ngram_tables_uniform(1000, {2: 50, 3: 50}, seed=0)
    visits = [((1, 2, 3, 4, 5, 6), 7), ((9, 8), 3)] * 5
    tabs = O.NgramTables(synth.plant_ngrams(base, visits, 1000, seed=0, frac=1.0))
    assert O.p_ngram(tabs, O.LAMBDAS_PAPER, [1, 2, 3, 4, 5, 6], 7) > 0
    for n, (keys, counts) in synth.plant_ngrams(base, visits, 1000, seed=0, frac=1.0).items():
        assert len(np.unique(keys, axis=0)) == len(keys)


def test_reduced_orders_are_the_full_mixture_without_the_missing_terms(toy):
    """The storage-saving variant (appendix "Perplexity Evaluation with Fewer N-Grams") loads
    n = 2..4 only and keeps the same interpolation weights: an order without a table adds
    nothing.  Recounted from the corpus, and equal to the full tables with those weights at 0."""
    corpus, full = toy
    small = O.NgramTables(corpus_tables(corpus, orders=(2, 3, 4)))
    lam = synth.PAPER_LAMBDAS
    rng = np.random.default_rng(3)
    n_pos = 0
    for _ in range(60):
        at = int(rng.integers(6, len(corpus) - 1))
        hist, tok = corpus[:at], int(corpus[at]) if rng.random() < 0.7 else int(rng.integers(0, 6))
        want = 0.0
        for n in (2, 3, 4):
            ctx = tuple(hist[-(n - 1):])
            total = sum(1 for i in range(len(corpus) - n + 1) if tuple(corpus[i:i + n - 1]) == ctx)
            hits = sum(1 for i in range(len(corpus) - n + 1) if tuple(corpus[i:i + n]) == ctx + (tok,))
            want += lam[n - 2] * (hits / total if total else 0.0)
        got = float(O.p_ngram(small, lam, hist, tok, np.float64))
        assert abs(got - want) < 1e-12
        assert got == float(O.p_ngram(full, lam[:3] + (0.0, 0.0), hist, tok, np.float64))
        assert got <= float(O.p_ngram(full, lam, hist, tok, np.float64)) + 1e-15
        n_pos += got > 0
    assert n_pos > 20
