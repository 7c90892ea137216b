"""Pins for the oracle's nucleus sampler (the comparison decoder of Section 4.3): a hand-worked
example, the limits that reduce to textbook routines, and invariants."""
import os

import numpy as np
import pytest

from oracle import spd_oracle as O

HERE = os.path.dirname(os.path.abspath(__file__))


def _example():
    probs, top_p, size, mass, draws = None, None, None, None, []
    for line in open(os.path.join(HERE, "golden", "nucleus_worked_example.txt")):
        f = line.split()
        if not f or f[0].startswith("#"):
            continue
        if f[0] == "probs": probs = np.array([float(x) for x in f[1:]])
        elif f[0] == "top_p": top_p = float(f[1])
        elif f[0] == "nucleus_size": size = int(f[1])
        elif f[0] == "nucleus_mass": mass = float(f[1])
        elif f[0] == "draw": draws.append((float(f[1]), int(f[2])))
    return probs, top_p, size, mass, draws


def test_hand_worked_example():
    probs, top_p, size, mass, draws = _example()
    logits = np.log(probs / probs.sum())
    for u, tok in draws:
        r = O.nucleus_sample(logits, top_p, 1.0, u)
        assert r.nucleus_size == size
        assert abs(r.nucleus_mass - mass / probs.sum()) < 1e-9
        assert r.token == tok, (u, r.token, tok)


def test_top_p_one_is_plain_inverse_cdf_sampling():
    rng = np.random.default_rng(0)
    logits = rng.normal(size=200)
    p = np.exp(logits - logits.max()); p /= p.sum()
    order = np.argsort(-p, kind="stable")
    cdf = np.cumsum(p[order])
    for u in rng.random(300):
        r = O.nucleus_sample(logits, 1.0, 1.0, u)
        # (the last cumulative value may round to just under 1; then the nucleus is everything)
        want = order[min(np.searchsorted(cdf, u * r.nucleus_mass, side="right"), p.size - 1)]
        assert r.token == want


def test_tiny_top_p_is_greedy_whatever_the_draw():
    rng = np.random.default_rng(1)
    for _ in range(50):
        logits = rng.normal(size=64)
        for u in (0.0, 0.3, 0.999999):
            r = O.nucleus_sample(logits, 1e-9, 1.0, u)
            assert r.token == int(np.argmax(logits)) and r.nucleus_size == 1


def test_nucleus_is_the_smallest_set_that_reaches_p():
    rng = np.random.default_rng(2)
    for _ in range(100):
        logits = rng.normal(size=50) * 2
        p = np.exp(logits - logits.max()); p /= p.sum()
        top_p = float(rng.uniform(0.05, 0.99))
        r = O.nucleus_sample(logits, top_p, 1.0, 0.5)
        srt = np.sort(p)[::-1]
        assert srt[: r.nucleus_size].sum() >= top_p - 1e-12
        assert srt[: r.nucleus_size - 1].sum() < top_p + 1e-12
        assert abs(r.nucleus_mass - srt[: r.nucleus_size].sum()) < 1e-12


def test_draws_on_a_grid_reproduce_the_renormalised_probabilities():
    rng = np.random.default_rng(3)
    logits = rng.normal(size=30) * 1.5
    p = np.exp(logits - logits.max()); p /= p.sum()
    N = 20000
    counts = np.zeros(30)
    size = None
    for i in range(N):
        r = O.nucleus_sample(logits, 0.8, 1.0, (i + 0.5) / N)
        counts[r.token] += 1
        size = r.nucleus_size
    keep = np.argsort(-p, kind="stable")[:size]
    want = np.zeros(30); want[keep] = p[keep] / p[keep].sum()
    assert np.all(counts[np.setdiff1d(np.arange(30), keep)] == 0)       # never outside the nucleus
    assert np.max(np.abs(counts / N - want)) <= 1.0 / N + 1e-12          # closed form up to one grid cell


def test_token_is_monotone_in_the_draw_and_ties_prefer_the_lower_id():
    logits = np.log(np.array([0.2, 0.3, 0.3, 0.2]))
    ranks = {1: 0, 2: 1, 0: 2, 3: 3}                                     # probability order with id tie-break
    last = -1
    for u in np.linspace(0, 0.999, 200):
        r = O.nucleus_sample(logits, 1.0, 1.0, float(u))
        assert ranks[r.token] >= last
        last = ranks[r.token]
    assert O.nucleus_sample(logits, 1.0, 1.0, 0.0).token == 1
    assert O.nucleus_sample(logits, 0.55, 1.0, 0.99).token == 2           # nucleus {1, 2}: 0.6 >= 0.55


def test_temperature_divides_the_logits():
    rng = np.random.default_rng(4)
    logits = rng.normal(size=40)
    for u in (0.1, 0.6, 0.95):
        a = O.nucleus_sample(logits, 0.9, 0.5, u)
        b = O.nucleus_sample(logits / 0.5, 0.9, 1.0, u)
        assert a.token == b.token and abs(a.logp - b.logp) < 1e-12


def test_generate_feeds_the_sampled_token_back():
    """One pass = prefix pass, then one forward per sampled token: the log-probabilities it reports
    equal those of a full-sequence evaluation of the same tokens."""
    import synth
    shape = synth.ModelShape("nuc", 2, 64, 4, 2, 128, 98, "fp32")
    w = synth.make_weights(shape, seed=3)
    lm = O.OracleLM(w, shape.n_layers, shape.n_heads, shape.n_kv_heads, shape.rms_eps, shape.rope_theta, np.float64)
    prefix = [5, 17, 3, 88]
    us = [0.3, 0.9, 0.01, 0.5]
    toks, total, recs = O.nucleus_generate(lm, prefix, 0.9, 1.0, us)
    lm.reset()
    seq = prefix + toks
    all_logits = lm.forward(lm.embedding_rows(np.array(seq[:-1])), all_positions=True)
    lps = [O.log_softmax_tau(all_logits[len(prefix) - 1 + t], 1.0, np.float64)[toks[t]] for t in range(len(toks))]
    assert abs(sum(lps) - total) < 1e-9
    assert all(abs(r.logp - lp) < 1e-9 for r, lp in zip(recs, lps))
