"""N-gram tables as a parameter of a live context: the storage-saving variant with orders
n = 2..4 only (appendix "Perplexity Evaluation with Fewer N-Grams": same interpolation weights,
alpha = 0.55, tau = 0.1), k up to 10 (the largest k the paper evaluates), and tables replaced
between two timesteps of a generation.  HIP path against the oracle, through the C ABI."""
import numpy as np
import pytest

import synth
from gpu_common import RTOL, compare_step, make_oracle, tails_of, teacher_forced
from oracle import spd_oracle as O

pytestmark = pytest.mark.gpu


def P():
    import paper_2405_18400_amd as pkg
    return pkg


def visits_of(shape, w, prefix, k, n_tokens):
    lm = make_oracle(shape, w)
    _, recs = O.generate(lm, None, prefix, O.DecodeCfg(k, 0.0), n_tokens)
    return [(tuple(rec.state_in.history(i)), int(tok)) for rec in recs[1:] for i in range(k) for tok in rec.top_ids]


@pytest.fixture(scope="module")
def tiny():
    shape = synth.TINY
    w = synth.make_weights(shape, seed=0)
    prefix = synth.make_prefix_uniform(shape.vocab, 16, seed=0)
    return shape, w, prefix


@pytest.mark.parametrize("k", [3, 10])
def test_orders_2_to_4_only(tiny, k):
    shape, w, prefix = tiny
    pkg = P()
    base = synth.make_ngram_tables_zipf(shape.vocab, 40_000, seed=4)
    planted = synth.plant_ngrams(base, visits_of(shape, w, prefix, k, 6), shape.vocab, seed=k)
    small = {n: planted[n] for n in (2, 3, 4)}
    lam = synth.PAPER_LAMBDAS
    sess = pkg.Session(shape, w, max_ctx=64, k_max=16)
    try:
        sess.spd_load_ngrams(small, lam)
        dc = pkg.SpdDecodeCfg(k, 0.55, 0.1, 0.1)
        cfg = O.DecodeCfg(k, 0.55, 0.1, 0.1, tuple(lam))
        _, recs, stats = teacher_forced(sess, make_oracle(shape, w), small, lam, prefix, cfg, 6, RTOL[shape.dtype], dc)
        assert any(c.overlap for r in recs[1:] for c in r.candidates), "planting produced no n-gram hit"
        # the two missing orders change the result: the same run with all five orders differs
        otabs = O.NgramTables(planted)
        _, recs_full = O.generate(make_oracle(shape, w), otabs, prefix, cfg, 6)
        assert any(not np.array_equal(a.pngram, b.pngram) for a, b in zip(recs[1:], recs_full[1:]))
    finally:
        sess.close()


def test_tables_replaced_between_timesteps(tiny):
    """Three timesteps with five orders, then the tables are replaced by a different set with
    orders 2..4 on the live context, three more timesteps.  The oracle is driven step by step
    with the same switch."""
    shape, w, prefix = tiny
    pkg = P()
    k, lam = 3, synth.PAPER_LAMBDAS
    visits = visits_of(shape, w, prefix, k, 6)
    tabs_a = synth.plant_ngrams(synth.make_ngram_tables_zipf(shape.vocab, 40_000, seed=5), visits, shape.vocab, seed=1)
    tabs_b = synth.plant_ngrams(synth.make_ngram_tables_zipf(shape.vocab, 30_000, seed=6), visits, shape.vocab, seed=2, frac=0.8)
    tabs_b = {n: tabs_b[n] for n in (2, 3, 4)}
    cfg = O.DecodeCfg(k, 0.54, 1.0, 0.1, tuple(lam))
    dc = pkg.SpdDecodeCfg(k, 0.54, 1.0, 0.1)
    lm = make_oracle(shape, w)
    lm.reset()
    sess = pkg.Session(shape, w, max_ctx=64, k_max=8)
    try:
        sess.spd_load_ngrams(tabs_a, lam)
        sess.spd_prefill(prefix)
        state, rec = O.first_step(lm.forward(lm.embedding_rows(prefix)), prefix, cfg)
        sess.spd_step_outputs = sess.spd_step(dc)
        compare_step(sess, rec, dc, RTOL[shape.dtype], first=True, cfg=cfg, otabs=O.NgramTables(tabs_a), prefix=prefix)
        seen = []
        for t in range(1, 6):
            if t == 3:
                sess.spd_load_ngrams(tabs_b, lam)
            otabs = O.NgramTables(tabs_a if t < 3 else tabs_b)
            gamma = O.superposition_weights(state.logscores)
            x = O.superposed_embedding(lm.embedding_rows([d[-1] for d in state.drafts]), gamma.astype(np.float32))
            sess.spd_set_state(tails_of(state), state.logscores)
            state, rec = O.expand_and_prune(state, lm.forward(x[None, :]), otabs, cfg, gamma_in=gamma)
            sess.spd_step_outputs = sess.spd_step(dc)
            compare_step(sess, rec, dc, RTOL[shape.dtype], first=False, cfg=cfg, otabs=otabs, prefix=prefix)
            seen.append(rec.pngram.copy())
        assert all(np.any(p > 0) for p in seen), "a timestep without any n-gram hit does not test the tables"
    finally:
        sess.close()
