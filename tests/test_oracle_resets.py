"""Pins for the oracle's reset / splice operations (Sections 5.3 and 4.5)."""
import numpy as np

import synth
from oracle import spd_oracle as O


def test_draft_is_sampled_with_its_superposition_weight():
    ls = np.log(np.array([0.5, 0.3, 0.2], np.float32) * 1e-3)      # gamma = 0.5, 0.3, 0.2 (Eq. 2)
    N = 1000
    counts = np.bincount([O.choose_draft(ls, (i + 0.5) / N) for i in range(N)], minlength=3)
    assert list(counts) == [500, 300, 200]
    assert O.choose_draft(ls, 0.0) == 0 and O.choose_draft(ls, 0.999999) == 2
    assert O.choose_draft(np.array([-3.0], np.float32), 0.7) == 0   # one draft: nothing to choose


def _lm(seed=4):
    shape = synth.ModelShape("rs", 2, 64, 4, 2, 128, 98, "fp32")
    w = synth.make_weights(shape, seed=seed)
    return O.OracleLM(w, shape.n_layers, shape.n_heads, shape.n_kv_heads, shape.rms_eps, shape.rope_theta, np.float64)


def test_commit_extends_the_prefix_by_the_sampled_draft():
    lm = _lm()
    prefix = [3, 14, 15, 92, 65]
    state, _ = O.generate(lm, None, prefix, O.DecodeCfg(3, 0.0), 4, np.float64)
    for u, in [(0.0,), (0.5,), (0.99,)]:
        i, new_prefix = O.commit_draft(state, u)
        assert new_prefix == prefix + state.drafts[i] and len(new_prefix) == len(prefix) + 4


def test_restart_equals_a_fresh_generation_from_the_longer_prefix():
    lm = _lm()
    prefix = [3, 14, 15, 92, 65]
    cfg = O.DecodeCfg(3, 0.0)
    text, state, chosen = O.generate_with_resets(lm, None, prefix, cfg, 10, 4, [0.3, 0.8], np.float64)
    assert len(chosen) == 2 and len(text) == 8 and all(len(d) == 2 for d in state.drafts)
    # the last segment is exactly what SPD generates from the committed text
    ref, _ = O.generate(lm, None, prefix + text, cfg, 2, np.float64)
    assert ref.drafts == state.drafts and np.allclose(ref.logscores, state.logscores)
    # and the committed text is made of drafts of the earlier segments
    s1, _ = O.generate(lm, None, prefix, cfg, 4, np.float64)
    assert text[:4] == s1.drafts[chosen[0]]


def test_no_reset_when_the_segment_covers_the_generation():
    lm = _lm()
    prefix = [9, 8, 7]
    cfg = O.DecodeCfg(2, 0.0)
    text, state, chosen = O.generate_with_resets(lm, None, prefix, cfg, 5, 5, [], np.float64)
    ref, _ = O.generate(lm, None, prefix, cfg, 5, np.float64)
    assert text == [] and chosen == [] and ref.drafts == state.drafts


def test_k1_commit_is_the_splice_of_a_single_pass():
    """A pass with one draft (greedy here, nucleus on the GPU side) committed = that text as prefix."""
    lm = _lm()
    prefix = [1, 2, 3, 4]
    s1, _ = O.generate(lm, None, prefix, O.DecodeCfg(1, 0.0), 3, np.float64)
    i, new_prefix = O.commit_draft(s1, 0.42)
    assert i == 0 and new_prefix == prefix + s1.drafts[0]
