"""Committing a draft and restarting (resets, Section 5.3; nucleus pass spliced in front of
Superposed Decoding, Section 4.5) on the GPU against the oracle, through the C ABI."""
import numpy as np
import pytest

import synth
from gpu_common import RTOL, assert_close_scaled, make_oracle, teacher_forced
from oracle import spd_oracle as O

pytestmark = pytest.mark.gpu


def P():
    import paper_2405_18400_amd as pkg
    return pkg


def free_steps(sess, dc, n):
    """n free-running steps; the drafts rebuilt here from each step's (token, parent) pairs."""
    drafts = None
    for t in range(n):
        tokens, parents, _ = sess.spd_step(dc)
        if t == 0:
            drafts = [[int(tok)] for tok in tokens]
        else:
            drafts = [drafts[int(par)] + [int(tok)] for tok, par in zip(tokens, parents)]
    return drafts


def draws_inside_every_interval(logscores):
    """One draw per draft, in the middle of that draft's interval of the cumulative weights."""
    cum = np.concatenate([[0.0], np.cumsum(O.superposition_weights(logscores).astype(np.float64))])
    return [float((cum[i] + cum[i + 1]) / 2 / cum[-1]) for i in range(len(cum) - 1)]


def after_commit_checks(sess, shape, w, tabs, lam, text, k, alpha, n_more):
    """The context must stand exactly as after a prefix pass over `text`: its logits are the
    oracle's, and so is every step of a generation that starts there."""
    lm = make_oracle(shape, w)
    assert sess.spd_position() == len(text)
    want = lm.forward(lm.embedding_rows(text))                 # the whole text in one causal pass
    assert_close_scaled(sess.spd_read_logits(), want, RTOL[shape.dtype], "logits after the commit")
    dc = P().SpdDecodeCfg(k, alpha, 1.0, 0.1)
    cfg = O.DecodeCfg(k, alpha, 1.0, 0.1, tuple(lam))
    teacher_forced(sess, make_oracle(shape, w), tabs, lam, text, cfg, n_more, RTOL[shape.dtype], dc, prefilled=True)
    assert sess.spd_position() == len(text) + n_more - 1


@pytest.fixture(scope="module")
def tiny():
    shape = synth.TINY
    w = synth.make_weights(shape, seed=0)
    tabs = synth.make_ngram_tables_uniform(shape.vocab, {2: 50_000, 3: 50_000}, seed=0)
    prefix = synth.make_prefix_uniform(shape.vocab, 16, seed=0)
    return shape, w, tabs, prefix


@pytest.mark.parametrize("which", [0, 1, 2])
@pytest.mark.parametrize("path", ["fused", "per_operator"])
def test_commit_each_draft_then_restart(tiny, which, path):
    shape, w, tabs, prefix = tiny
    lam = (0.01, 0.04, 0.0, 0.0, 0.0)
    pkg = P()
    sess = pkg.Session(shape, w, max_ctx=64, k_max=8)
    try:
        if path == "per_operator":
            sess.spd_set_fused(False)
        sess.spd_load_ngrams(tabs, lam)
        dc = pkg.SpdDecodeCfg(3, 0.5, 1.0, 0.1)
        sess.spd_prefill(prefix)
        drafts = free_steps(sess, dc, 4)
        _, logscores, gamma = sess.spd_get_state()
        u = draws_inside_every_interval(logscores)[which]
        chosen, toks = sess.spd_commit(u)
        assert chosen == which == O.choose_draft(np.asarray(logscores, np.float64), u)
        assert toks.tolist() == drafts[which]
        after_commit_checks(sess, shape, w, tabs, lam, list(prefix) + drafts[which], 3, 0.5, 4)
    finally:
        sess.close()


def test_resets_every_s_steps_follow_the_oracle(tiny):
    """Generation with a reset every s = 3 timesteps, free-running on both sides.  The oracle
    is re-run on the text the GPU committed, so a step whose deciding gap is inside the float
    tolerance cannot send the comparison astray."""
    shape, w, tabs, prefix = tiny
    lam = (0.01, 0.04, 0.0, 0.0, 0.0)
    pkg = P()
    lm = make_oracle(shape, w)
    otabs = O.NgramTables(tabs)
    cfg = O.DecodeCfg(3, 0.5, 1.0, 0.1, lam)
    us = np.random.default_rng(21).random(4)
    sess = pkg.Session(shape, w, max_ctx=64, k_max=8)
    try:
        sess.spd_load_ngrams(tabs, lam)
        dc = pkg.SpdDecodeCfg(3, 0.5, 1.0, 0.1)
        sess.spd_prefill(prefix)
        text = list(map(int, prefix))
        n_equal = 0
        for j in range(4):
            drafts = free_steps(sess, dc, 3)
            state, recs = O.generate(lm, otabs, text, cfg, 3)
            tol = 2 * RTOL[shape.dtype] * max(float(np.max(np.abs(r.logits))) for r in recs)
            decisive = all(r.gap_vocab > 4 * tol and (t == 0 or r.gap_prune > 4 * tol) for t, r in enumerate(recs))
            _, logscores, _ = sess.spd_get_state()
            if decisive:
                assert drafts == [list(d) for d in state.drafts]
                np.testing.assert_allclose(logscores, state.logscores, atol=1e-3)
                n_equal += 1
            cum = np.cumsum(O.superposition_weights(state.logscores).astype(np.float64))
            u = float(us[j])
            near_edge = np.min(np.abs(cum[:-1] / cum[-1] - u)) < 1e-4
            chosen, toks = sess.spd_commit(u)
            if decisive and not near_edge:
                want_i, want_text = O.commit_draft(state, u)
                assert chosen == want_i and text + toks.tolist() == want_text
            assert toks.tolist() == drafts[chosen]
            text = text + toks.tolist()
            assert sess.spd_position() == len(text)
        assert n_equal >= 3
        after_commit_checks(sess, shape, w, tabs, lam, text, 3, 0.5, 3)
    finally:
        sess.close()


@pytest.mark.parametrize("n_first", [1, 6])
def test_nucleus_pass_spliced_in_front_of_superposed_decoding(tiny, n_first):
    """A nucleus-sampled opening becomes the prefix of a Superposed Decoding run (Section 4.5).
    With one draft the cache already holds the text: only its newest token is passed again."""
    shape, w, tabs, prefix = tiny
    lam = (0.01, 0.04, 0.0, 0.0, 0.0)
    pkg = P()
    us = np.random.default_rng(31).random(n_first).astype(np.float32)
    sess = pkg.Session(shape, w, max_ctx=64, k_max=8)
    try:
        sess.spd_load_ngrams(tabs, lam)
        sess.spd_prefill(prefix)
        sc = pkg.SpdSampleCfg(0.9, 1.0)
        opening = [sess.spd_nucleus_step(sc, float(u))[0] for u in us]
        chosen, toks = sess.spd_commit(0.7)
        assert chosen == 0 and toks.tolist() == opening
        after_commit_checks(sess, shape, w, tabs, lam, list(prefix) + opening, 3, 0.5, 5)
    finally:
        sess.close()


def test_greedy_draft_commit_keeps_the_cache(tiny):
    """k = 1 Superposed Decoding is greedy decoding; committing its single draft must leave the
    cache of the earlier positions as it is (weight 1 on one token is that token's embedding)."""
    shape, w, tabs, prefix = tiny
    pkg = P()
    sess = pkg.Session(shape, w, max_ctx=64, k_max=8)
    try:
        dc = pkg.SpdDecodeCfg(1, 0.0, 1.0, 0.1)
        sess.spd_prefill(prefix)
        drafts = free_steps(sess, dc, 5)
        chosen, toks = sess.spd_commit(0.0)
        assert chosen == 0 and toks.tolist() == drafts[0]
        after_commit_checks(sess, shape, w, None, synth.PAPER_LAMBDAS, list(prefix) + drafts[0], 2, 0.0, 3)
    finally:
        sess.close()


@pytest.mark.parametrize("kv_dtype", ["fp32", "fp16"])
@pytest.mark.parametrize("dense", [True, False])
def test_commit_through_the_dense_prefix_pass(dense, kv_dtype):
    """A 12-token segment on a bf16 model: the committed tokens are passed again as one chunk on
    the matrix cores, starting at a cache position that is no multiple of any tile (an odd one:
    with an fp16 cache, rows that start in the middle of a 16-byte piece)."""
    shape = synth.ModelShape("small-bf16", 2, 512, 8, 2, 1408, 2048, "bf16")
    w = synth.make_weights(shape, seed=5)
    prefix = synth.make_prefix_zipf(shape.vocab, 37, seed=5)
    pkg = P()
    sess = pkg.Session(shape, w, max_ctx=128, k_max=8, kv_dtype=kv_dtype)
    try:
        sess.spd_set_dense_prefill(dense)
        assert sess.spd_get_dense_prefill() == dense
        dc = pkg.SpdDecodeCfg(3, 0.0, 1.0, 0.1)
        sess.spd_prefill(prefix)
        drafts = free_steps(sess, dc, 12)
        _, logscores, _ = sess.spd_get_state()
        u = draws_inside_every_interval(logscores)[1]
        chosen, toks = sess.spd_commit(u)
        assert chosen == 1 and toks.tolist() == drafts[1]
        after_commit_checks(sess, shape, w, None, synth.PAPER_LAMBDAS, list(prefix) + drafts[1], 3, 0.0, 3)
    finally:
        sess.close()


def test_commit_error_paths(tiny):
    shape, w, tabs, prefix = tiny
    pkg = P()
    sess = pkg.Session(shape, w, max_ctx=24, k_max=8)
    try:
        with pytest.raises(pkg.SpdError, match="no drafts"):
            sess.spd_commit(0.5)
        sess.spd_prefill(prefix)
        with pytest.raises(pkg.SpdError, match="no drafts"):
            sess.spd_commit(0.5)
        dc = pkg.SpdDecodeCfg(2, 0.0, 1.0, 0.1)
        free_steps(sess, dc, 2)
        for bad in (-0.1, 1.0, float("nan")):
            with pytest.raises(pkg.SpdError, match=r"\[0, 1\)"):
                sess.spd_commit(bad)
        chosen, toks = sess.spd_commit(0.999999)
        assert chosen == 1 and len(toks) == 2
        with pytest.raises(pkg.SpdError, match="no drafts"):       # already committed
            sess.spd_commit(0.5)
        free_steps(sess, dc, 6)                                     # 16 + 2 + 6 = 24 = max_ctx
        with pytest.raises(pkg.SpdError, match="max_ctx"):
            sess.spd_commit(0.5)
    finally:
        sess.close()
