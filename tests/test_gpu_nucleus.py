"""Nucleus (top-p) sampling pass on the GPU against the oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import synth
from gpu_common import RTOL, assert_close_scaled, make_oracle
from oracle import spd_oracle as O

pytestmark = pytest.mark.gpu


def P():
    import paper_2405_18400_amd as pkg
    return pkg


def acceptable(logits, top_p, tau, u, token, tol):
    """Is `token` what nucleus sampling returns for SOME cumulative probabilities within `tol`
    of the exact ones?  (Both sides sum probabilities in floating point; a draw that lands
    within rounding of a boundary may legitimately select either neighbour.)"""
    lp = O.log_softmax_tau(np.asarray(logits, np.float64), tau, np.float64)
    p = np.exp(lp)
    order = np.lexsort((np.arange(p.size), -p))
    cs = np.cumsum(p[order])
    n = int(min(np.searchsorted(cs, top_p, side="left"), p.size - 1))
    masses = {float(cs[n])}
    if n > 0 and cs[n - 1] >= top_p - tol: masses.add(float(cs[n - 1]))
    if n + 1 < p.size and cs[n] < top_p + tol: masses.add(float(cs[n + 1]))
    j = int(np.nonzero(order == token)[0][0])
    lo = cs[j - 1] if j > 0 else 0.0
    return any(lo - tol <= u * m <= cs[j] + tol for m in masses)


def check_draw(sess, rec, top_p, tau, u, got_token, got_logp, tol):
    decisive = rec.margin_sample > tol + (u * rec.p_edge if rec.margin_nucleus <= tol else 0.0)
    if decisive:
        assert got_token == rec.token, (got_token, rec.token, rec.margin_sample)
        assert abs(got_logp - rec.logp) <= tol * max(1.0, abs(rec.logp)) + 1e-4
    else:
        assert acceptable(rec.logits, top_p, tau, u, got_token, tol)
    return decisive


# Cumulative probabilities are fp32 sums of up to a few thousand terms on the GPU and fp64 sums
# in the oracle, from logits that agree to about 1e-6 of their scale: a draw closer than this
# to a boundary is not held to the oracle's choice, only to a valid one.
TOL = 1e-5


@pytest.fixture(scope="module")
def tiny():
    shape = synth.TINY
    return shape, synth.make_weights(shape, seed=0), synth.make_prefix_uniform(shape.vocab, 16, seed=0)


@pytest.mark.parametrize("top_p,tau", [(0.9, 1.0), (0.5, 0.7), (1.0, 1.3)])
def test_pass_teacher_forced(tiny, top_p, tau):
    """BASELINE config 3's comparison decoder on the tiny model: 12 tokens, seeded draws; after
    every token the oracle's token is written back so each step is compared on its own."""
    shape, w, prefix = tiny
    pkg = P()
    us = np.random.default_rng(11).random(12).astype(np.float32)
    lm = make_oracle(shape, w)
    toks, total, recs = O.nucleus_generate(lm, prefix, top_p, tau, [float(u) for u in us], keep_logits=True)
    sess = pkg.Session(shape, w, max_ctx=64, k_max=8)
    try:
        sc = pkg.SpdSampleCfg(top_p, tau)
        sess.spd_prefill(prefix)
        n_decisive, run_total, tail = 0, 0.0, [-1] * 5
        tail = ([-1] * 5 + list(prefix))[-5:]
        for t, rec in enumerate(recs):
            tok, lp = sess.spd_nucleus_step(sc, float(us[t]))
            assert_close_scaled(sess.spd_read_logits(), rec.logits, RTOL[shape.dtype], "logits")
            n_decisive += check_draw(sess, rec, top_p, tau, float(us[t]), tok, lp, TOL)
            size, mass, _ = sess.spd_get_nucleus_info()
            assert abs(mass - rec.nucleus_mass) < 1e-4
            if rec.margin_nucleus > 1e-4:
                assert size == rec.nucleus_size
            run_total += rec.logp
            tail = tail[1:] + [rec.token]
            sess.spd_set_state(np.array([tail], np.int32), np.array([run_total], np.float32))   # teacher forcing
        assert n_decisive >= len(recs) - 4
        assert sess.spd_position() == len(prefix) + len(recs) - 1
    finally:
        sess.close()


def test_free_running_pass_and_graph_replay_agree(tiny):
    shape, w, prefix = tiny
    pkg = P()
    us = np.random.default_rng(12).random(10).astype(np.float32)
    out = []
    for graph in (True, False):
        sess = pkg.Session(shape, w, max_ctx=64, k_max=8)
        try:
            sess.spd_set_graph(graph)
            sc = pkg.SpdSampleCfg(0.9, 1.0)
            sess.spd_prefill(prefix)
            out.append([sess.spd_nucleus_step(sc, float(u)) for u in us])
            assert abs(sess.spd_get_nucleus_info()[2] - sum(lp for _, lp in out[-1])) < 1e-3
        finally:
            sess.close()
    assert out[0] == out[1]


def _sample_only(sess, sc, logits, u, first=True):
    sess.spd_nucleus_sample(sc, u, torch.tensor(logits, dtype=torch.float32, device="cuda"), first)
    tails, _, _ = sess.spd_get_state()
    return int(tails[0, -1])


def test_sampler_on_scripted_logits_ties_and_limits(tiny):
    shape, w, prefix = tiny
    pkg = P()
    sess = pkg.Session(shape, w, max_ctx=64, k_max=8)
    try:
        sess.spd_prefill(prefix)
        V = shape.vocab
        base = np.full(V, -30.0, np.float32)
        # four tokens carry all the mass: ids 7 and 900 tie at 0.3, id 3 has 0.2, id 2000 has 0.2
        lg = base.copy()
        lg[[7, 900, 3, 2000]] = np.log([0.3, 0.3, 0.2, 0.2]).astype(np.float32)
        sc = pkg.SpdSampleCfg(1.0, 1.0)
        want = lambda u, p=1.0: O.nucleus_sample(lg, p, 1.0, u).token
        for u in (0.0, 0.1, 0.29, 0.31, 0.59, 0.61, 0.79, 0.81, 0.99):
            assert _sample_only(sess, sc, lg, u) == want(u), u
        assert _sample_only(sess, sc, lg, 0.0) == 7 and _sample_only(sess, sc, lg, 0.45) == 900    # lower id first
        assert _sample_only(sess, sc, lg, 0.7) == 3 and _sample_only(sess, sc, lg, 0.9) == 2000
        # nucleus that ends inside the tie: p = 0.25 keeps only id 7; p = 0.55 keeps 7 and 900
        assert all(_sample_only(sess, pkg.SpdSampleCfg(0.25, 1.0), lg, u) == 7 for u in (0.0, 0.5, 0.99))
        got = {_sample_only(sess, pkg.SpdSampleCfg(0.55, 1.0), lg, u) for u in np.linspace(0, 0.99, 23)}
        assert got == {7, 900}
        assert sess.spd_get_nucleus_info()[0] == 2
        # tiny top_p: greedy whatever the draw
        rng = np.random.default_rng(5)
        rl = (rng.normal(size=V) * 3).astype(np.float32)
        assert all(_sample_only(sess, pkg.SpdSampleCfg(1e-6, 1.0), rl, u) == int(np.argmax(rl)) for u in (0.0, 0.5, 0.999))
        # random logits, many draws, both temperatures: equal to the oracle wherever it is decisive
        for tau in (1.0, 0.4):
            n_dec = 0
            for u in rng.random(60):
                rec = O.nucleus_sample(rl, 0.9, tau, float(np.float32(u)), keep_logits=True)
                tok = _sample_only(sess, pkg.SpdSampleCfg(0.9, tau), rl, float(np.float32(u)))
                n_dec += check_draw(sess, rec, 0.9, tau, float(np.float32(u)), tok, rec.logp, 1e-5)
            assert n_dec >= 45
    finally:
        sess.close()


def test_draws_on_a_grid_follow_the_renormalised_distribution(tiny):
    shape, w, prefix = tiny
    pkg = P()
    sess = pkg.Session(shape, w, max_ctx=64, k_max=8)
    try:
        sess.spd_prefill(prefix)
        rng = np.random.default_rng(6)
        lg = (rng.normal(size=shape.vocab) * 3).astype(np.float32)
        p = np.exp(lg.astype(np.float64) - lg.max()); p /= p.sum()
        order = np.argsort(-p, kind="stable")
        n = int(np.searchsorted(np.cumsum(p[order]), 0.8))
        keep = order[: n + 1]
        N = 400
        counts = np.zeros(shape.vocab)
        sc = pkg.SpdSampleCfg(0.8, 1.0)
        for i in range(N):
            counts[_sample_only(sess, sc, lg, (i + 0.5) / N)] += 1
        want = np.zeros(shape.vocab); want[keep] = p[keep] / p[keep].sum()
        assert counts[np.setdiff1d(np.arange(shape.vocab), keep)].sum() == 0
        assert np.max(np.abs(counts / N - want)) <= 1.5 / N
    finally:
        sess.close()


def test_large_vocabulary_uses_the_uncached_path():
    """More than 32768 entries: the sampler recomputes probabilities instead of holding them."""
    pkg = P()
    shape = synth.ModelShape("bigvocab", 1, 64, 2, 2, 128, 40000, "fp32")
    w = synth.make_weights(shape, seed=2)
    sess = pkg.Session(shape, w, max_ctx=32, k_max=8)
    try:
        sess.spd_prefill([1, 2, 3])
        rng = np.random.default_rng(7)
        lg = (rng.normal(size=shape.vocab) * 4).astype(np.float32)
        n_dec = 0
        for u in rng.random(20):
            rec = O.nucleus_sample(lg, 0.9, 1.0, float(np.float32(u)), keep_logits=True)
            tok = _sample_only(sess, pkg.SpdSampleCfg(0.9, 1.0), lg, float(np.float32(u)))
            n_dec += check_draw(sess, rec, 0.9, 1.0, float(np.float32(u)), tok, rec.logp, 1e-5)
        assert n_dec >= 12
    finally:
        sess.close()


def test_error_paths(tiny):
    shape, w, prefix = tiny
    pkg = P()
    sess = pkg.Session(shape, w, max_ctx=64, k_max=8)
    try:
        sc = pkg.SpdSampleCfg(0.9, 1.0)
        with pytest.raises(pkg.SpdError): sess.spd_nucleus_step(sc, 0.5)              # before prefill
        sess.spd_prefill(prefix)
        for bad in (pkg.SpdSampleCfg(0.0, 1.0), pkg.SpdSampleCfg(1.5, 1.0), pkg.SpdSampleCfg(0.9, 0.0)):
            with pytest.raises(pkg.SpdError): sess.spd_nucleus_step(bad, 0.5)
        for u in (-0.1, 1.0):
            with pytest.raises(pkg.SpdError): sess.spd_nucleus_step(sc, u)
        sess.spd_step(pkg.SpdDecodeCfg(3, 0.0, 1.0, 0.1))
        with pytest.raises(pkg.SpdError): sess.spd_nucleus_step(sc, 0.5)              # SPD generation in progress
        sess.spd_prefill(prefix)
        assert sess.spd_nucleus_step(sc, 0.5)[0] >= 0
    finally:
        sess.close()
