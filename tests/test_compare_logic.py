"""The comparison logic of the GPU parity tests, exercised on the CPU: it accepts what is
correct (the oracle's own result, a swap inside the tolerance) and rejects planted mistakes."""
import numpy as np
import pytest

import synth
from gpu_common import (check_valid_prune, check_valid_topk, compare_decision_on_own_logits, option_tables,
                        plant_both_forms)
from helpers import oracle_lm, toy_shape
from oracle import spd_oracle as O


def test_valid_topk_accepts_swaps_inside_the_slack_only():
    z = np.array([5.0, 4.0, 3.0005, 3.0, 1.0, 0.0])
    check_valid_topk([0, 1, 2], z, 3, 1e-2)
    check_valid_topk([1, 0, 3], z, 3, 1e-2)            # 3 ties with 2 inside the slack; order is free here
    with pytest.raises(AssertionError):
        check_valid_topk([0, 1, 3], z, 3, 1e-4)        # outside a tighter slack
    with pytest.raises(AssertionError):
        check_valid_topk([0, 2, 3], z, 3, 1e-2)        # the clear winner 1 is missing
    with pytest.raises(AssertionError):
        check_valid_topk([0, 1, 4], z, 3, 1e-2)        # far below the k-th
    with pytest.raises(AssertionError):
        check_valid_topk([0, 1, 1], z, 3, 1e-2)        # not distinct


def _step_with_tables(k=3, alpha=0.54):
    shape = toy_shape(vocab=40, d=16, layers=1)
    lm, _ = oracle_lm(shape, seed=3)
    prefix = [3, 7, 1, 9, 2, 5]
    cfg0 = O.DecodeCfg(k, 0.0)
    _, recs0 = O.generate(lm, None, prefix, cfg0, 3)
    base = synth.make_ngram_tables_uniform(shape.vocab, {2: 30, 3: 30}, seed=1)
    tabs = plant_both_forms(base, recs0, k, shape.vocab, seed=2)
    cfg = O.DecodeCfg(k, alpha, 1.0, 0.1, synth.PAPER_LAMBDAS)
    otabs = O.NgramTables(tabs)
    _, recs = O.generate(lm, otabs, prefix, cfg, 3)
    return prefix, cfg, otabs, recs


def _as_gpu(rec, k):
    """The oracle's record in the shape the GPU reports a step in."""
    valid, score = option_tables(rec, k)
    cs = np.where(valid == 1, score, 0.0).astype(np.float32)
    cp = rec.pngram if rec.pngram is not None else np.zeros((k, k), np.float32)
    return [np.array(rec.top_ids, np.int32), np.array(rec.top_logp, np.float32), cs, valid, cp,
            np.array([c.token for c in rec.kept], np.int32), np.array([c.parent for c in rec.kept], np.int32),
            np.array([c.logscore for c in rec.kept], np.float32)]


class _Dc:
    def __init__(self, k):
        self.k = k


def test_planting_gives_both_forms_at_the_first_full_timestep():
    prefix, cfg, otabs, recs = _step_with_tables()
    step1 = recs[1]
    assert all(not c.overlap for c in step1.candidates if c.parent == 0) and sum(c.parent == 0 for c in step1.candidates) == 3
    assert any(c.overlap for c in step1.candidates if c.parent == 1)


def test_decision_comparison_accepts_the_oracle_and_rejects_planted_mistakes():
    k = 3
    prefix, cfg, otabs, recs = _step_with_tables(k)
    rec = recs[1]
    good = _as_gpu(rec, k)
    out = compare_decision_on_own_logits(good, rec.logits, rec, _Dc(k), cfg, otabs, prefix, first=False)
    assert out["own_overlap"] >= 1 and out["own_penalty"] >= 1

    def broken(i, change):
        g = [np.array(a, copy=True) for a in good]
        change(g[i])
        with pytest.raises(AssertionError):
            compare_decision_on_own_logits(g, rec.logits, rec, _Dc(k), cfg, otabs, prefix, first=False)

    broken(0, lambda a: a.__setitem__(slice(None), a[::-1].copy()))          # ids in the wrong order
    broken(1, lambda a: a.__setitem__(0, a[0] + 1e-3))                       # a log-probability off
    broken(3, lambda a: a.__setitem__((0, 0), 1 - a[0, 0]))                  # option mask flipped
    hit = tuple(np.argwhere(good[4] > 0)[0])
    broken(4, lambda a: a.__setitem__(hit, a[hit] * (1 + 1e-4)))             # a mixture value off
    broken(2, lambda a: a.__setitem__(tuple(np.argwhere(good[3] == 1)[0]), 0.5))   # an option score off
    broken(5, lambda a: a.__setitem__(0, (a[0] + 1) % 40))                   # a kept token that is no option
    broken(6, lambda a: a.__setitem__(slice(None), a[::-1].copy()) if len(set(a.tolist())) > 1 else a.__setitem__(0, 2 - a[0]))
    broken(7, lambda a: a.__setitem__(0, a[0] - 1e-2))                       # a kept score off
    # the first timestep
    first = _as_gpu(recs[0], k)
    first[6] = np.full(k, -1, np.int32)
    compare_decision_on_own_logits(first, recs[0].logits, recs[0], _Dc(k), cfg, otabs, prefix, first=True)
    first[5][0] += 1
    with pytest.raises(AssertionError):
        compare_decision_on_own_logits(first, recs[0].logits, recs[0], _Dc(k), cfg, otabs, prefix, first=True)


def test_valid_prune_rules():
    k = 3
    prefix, cfg, otabs, recs = _step_with_tables(k)
    rec = recs[1]
    pairs = [(c.parent, c.token) for c in rec.kept]
    scores = [c.logscore for c in rec.kept]
    check_valid_prune(pairs, scores, rec, k, 1e-4)
    ranked = sorted(rec.candidates, key=lambda c: -c.logscore)
    assert len(ranked) > k
    worst = ranked[-1]
    with pytest.raises(AssertionError):   # the worst option in place of a kept one
        check_valid_prune(pairs[:-1] + [(worst.parent, worst.token)], scores[:-1] + [worst.logscore], rec, k, 1e-4)
    with pytest.raises(AssertionError):   # a pair that is no option at all
        check_valid_prune(pairs[:-1] + [(0, -5)], scores, rec, k, 1e-4)
    with pytest.raises(AssertionError):   # right pairs, wrong score
        check_valid_prune(pairs, [scores[0] + 1.0] + scores[1:], rec, k, 1e-4)
    # a swap is accepted exactly when the two scores lie inside the slack
    gap = ranked[k - 1].logscore - ranked[k].logscore
    swapped = pairs[:-1] + [(ranked[k].parent, ranked[k].token)]
    swapped_scores = scores[:-1] + [ranked[k].logscore]
    check_valid_prune(swapped, swapped_scores, rec, k, gap * 1.01 + 1e-7)
    if gap > 1e-6:
        with pytest.raises(AssertionError):
            check_valid_prune(swapped, swapped_scores, rec, k, gap * 0.5)
