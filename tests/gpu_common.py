"""Shared pieces of the GPU parity tests: tolerances and the step-by-step comparison."""
import numpy as np

import synth
from oracle import spd_oracle as O

# Tolerances (north-star): logits and probabilities agree to within a relative 1e-4 on the fp32
# path and 2e-2 on the bf16 path.  "Relative" is taken against the largest magnitude of the
# vector compared (an element-wise ratio is meaningless for logits that cross zero).
RTOL = {"fp32": 1e-4, "bf16": 2e-2}

# The decision stage (log-softmax, KeepTopK, n-gram mixture, Eq. 4 / Eq. 5, prune) works on fp32
# logits whatever the weight type.  Given the SAME logits the two sides differ only by the
# order of a few fp32 sums: log-probabilities and scores agree to this relative bound, and two
# option scores closer than it count as tied.
SAME_INPUT_RTOL = 2e-5


def make_oracle(shape, weights, dtype=np.float32):
    return O.OracleLM(weights, shape.n_layers, shape.n_heads, shape.n_kv_heads, shape.rms_eps, shape.rope_theta, dtype)


def tails_of(state):
    out = np.full((len(state.drafts), 5), -1, np.int32)
    for i in range(len(state.drafts)):
        h = state.history(i)[-5:]
        out[i, 5 - len(h):] = h
    return out


def assert_close_scaled(got, want, rtol, what):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    scale = max(np.max(np.abs(want)), 1e-30)
    err = np.max(np.abs(got - want)) / scale
    assert err <= rtol, f"{what}: scaled error {err:.3e} > {rtol}"
    return err


def option_tables(rec, k):
    """[k, k] option mask and scores of an oracle record."""
    valid = np.zeros((k, k), np.int32)
    score = np.full((k, k), -np.inf)
    for c in rec.candidates:
        valid[c.parent, c.rank] = 1
        score[c.parent, c.rank] = c.logscore
    return valid, score


def check_valid_topk(ids, oracle_logits, k, slack):
    """Several KeepTopK results are correct when logits lie closer than the tolerance: the ids
    must be distinct, each within `slack` of the oracle's k-th logit, and every id that beats
    the oracle's (k+1)-th logit by more than `slack` must be among them."""
    z = np.asarray(oracle_logits, np.float64)
    srt = np.sort(z)[::-1]
    ids = [int(t) for t in ids]
    assert len(set(ids)) == k, f"KeepTopK ids not distinct: {ids}"
    for t in ids:
        assert z[t] >= srt[k - 1] - slack, f"kept id {t} (logit {z[t]:.5f}) lies below the k-th logit {srt[k - 1]:.5f} by more than {slack:.3e}"
    if len(srt) > k:
        for t in np.nonzero(z > srt[k] + slack)[0]:
            assert int(t) in ids, f"id {int(t)} clearly among the k largest (logit {z[t]:.5f} vs (k+1)-th {srt[k]:.5f}) is missing from {ids}"


def check_valid_prune(got_pairs, got_scores, rec, k, slack):
    """The same for the prune: kept (parent, token) pairs are distinct options, each within
    `slack` of the oracle's k-th best score, every clear winner is kept, and each kept pair's
    score agrees with the oracle's score of that option."""
    by_pair = {(c.parent, c.token): float(c.logscore) for c in rec.candidates}
    srt = sorted(by_pair.values(), reverse=True)
    assert len(set(got_pairs)) == k and set(got_pairs) <= set(by_pair), f"kept options {got_pairs} are not {k} distinct options"
    for pair, sc in zip(got_pairs, got_scores):
        assert by_pair[pair] >= srt[k - 1] - slack, f"kept option {pair} (score {by_pair[pair]:.5f}) lies below the k-th score {srt[k - 1]:.5f}"
        assert abs(float(sc) - by_pair[pair]) <= slack, f"score of {pair}: {sc} vs oracle {by_pair[pair]}"
    if len(srt) > k:
        for pair, sc in by_pair.items():
            if sc > srt[k] + slack:
                assert pair in got_pairs, f"option {pair} clearly among the k best is missing from {got_pairs}"


def compare_decision_on_own_logits(gpu, gpu_logits, rec, dc, cfg, otabs, prefix, first):
    """The decision stage given identical input: run the oracle's KeepTopK / expansion / n-gram
    mixture / interpolation / prune on the logits the GPU itself produced (and the drafts and
    scores both sides started the step from) and require the GPU's decisions to be the
    oracle's: ids, option mask and kept (parent, token) pairs exactly, p_ngram to 1e-6,
    log-probabilities and scores to fp32 rounding.  Only an exact-to-rounding tie between two
    option scores relaxes the kept pairs to the validity check."""
    k = dc.k
    ids, lp, cs, cv, cp, tokens, parents, scores = gpu
    if first:
        _, own = O.first_step(gpu_logits, prefix, cfg)
    else:
        _, own = O.expand_and_prune(rec.state_in, gpu_logits, otabs, cfg)
    out = {"own_overlap": 0, "own_penalty": 0, "own_dropped": 0}
    assert list(ids) == list(own.top_ids), f"KeepTopK on the GPU's own logits: {list(ids)} != {list(own.top_ids)}"
    lp_scale = max(1.0, float(np.max(np.abs(own.top_logp))))
    np.testing.assert_allclose(lp, own.top_logp, atol=SAME_INPUT_RTOL * lp_scale, rtol=0)
    if first:
        assert list(tokens) == list(own.top_ids) and list(parents) == [-1] * k
        np.testing.assert_allclose(scores, own.top_logp, atol=SAME_INPUT_RTOL * lp_scale, rtol=0)
        return out
    want_valid, want_score = option_tables(own, k)
    assert np.array_equal(cv, want_valid), f"option mask on the GPU's own logits differs:\n{cv}\n{want_valid}"
    if own.pngram is not None:
        np.testing.assert_allclose(cp, own.pngram, rtol=1e-6, atol=0)
    sc_scale = max(1.0, float(np.max(np.abs(want_score[want_valid == 1]))))
    np.testing.assert_allclose(cs[want_valid == 1], want_score[want_valid == 1], atol=SAME_INPUT_RTOL * sc_scale, rtol=0)
    got = list(zip(parents.tolist(), tokens.tolist()))
    if own.gap_prune > 4 * SAME_INPUT_RTOL * sc_scale:
        assert got == [(c.parent, c.token) for c in own.kept], f"kept options {got} != oracle on the same logits {[(c.parent, c.token) for c in own.kept]}"
        np.testing.assert_allclose(scores, [c.logscore for c in own.kept], atol=SAME_INPUT_RTOL * sc_scale, rtol=0)
    else:
        check_valid_prune(got, scores, own, k, 4 * SAME_INPUT_RTOL * sc_scale)
        out["own_prune_tied"] = True
    out["own_overlap"] = sum(1 for c in own.candidates if c.overlap)
    out["own_penalty"] = sum(1 for c in own.candidates if not c.overlap)
    out["own_dropped"] = k * k - len(own.candidates)
    return out


def compare_step(sess, rec, dc, rtol, first, cfg=None, otabs=None, prefix=None, check_logits=True):
    """Compare what the GPU decided in its latest step with the oracle, in two ways.
    (A) Against the oracle's own record of the step (its logits): logits within the tolerance;
    integer results exactly wherever the oracle's deciding gap exceeds the tolerance, otherwise
    the GPU result must be one of the correct ones (check_valid_topk / check_valid_prune).
    (B) Against the oracle's decision stage run on the GPU's own logits: exact, on every step
    (compare_decision_on_own_logits).  stats["fully_compared"] says (B) ran."""
    k = dc.k
    stats = {}
    logits = sess.spd_read_logits()
    if check_logits:
        stats["logit_err"] = assert_close_scaled(logits, rec.logits, rtol, "logits")
    tol_abs = rtol * float(np.max(np.abs(rec.logits)))
    ids, lp, cs, cv, cp = sess.spd_get_step_info(k)
    tokens, parents, scores = sess.spd_step_outputs

    if cfg is not None:
        stats.update(compare_decision_on_own_logits((ids, lp, cs, cv, cp, tokens, parents, scores), logits, rec, dc,
                                                    cfg, otabs, prefix, first))
        stats["fully_compared"] = True

    vocab_decisive = rec.gap_vocab > 2 * tol_abs
    stats["vocab_decisive"] = vocab_decisive
    lp_tol = 2 * tol_abs / dc.tau + 1e-5
    if vocab_decisive:
        assert list(ids) == list(rec.top_ids), f"KeepTopK ids {ids} != oracle {rec.top_ids} (gap {rec.gap_vocab:.3e})"
    else:
        check_valid_topk(ids, rec.logits, k, 2 * tol_abs)
        if list(ids) != list(rec.top_ids):
            # a different, equally correct set of kept tokens: options, hits and scores of this
            # step legitimately differ from the oracle's record; (B) above has checked them
            stats["ids_permuted"] = True
            return stats
    # log-probabilities: error of a logit difference, scaled by 1/tau
    np.testing.assert_allclose(lp, rec.top_logp, atol=lp_tol, rtol=0)
    if first:
        assert list(tokens) == list(rec.top_ids) and list(parents) == [-1] * k
        np.testing.assert_allclose(scores, rec.top_logp, atol=lp_tol, rtol=0)
        return stats
    # option table: which (draft, token) pairs are options is integer-exact (n-gram hits)
    want_valid, want_score = option_tables(rec, k)
    assert np.array_equal(cv, want_valid), f"option mask differs:\n{cv}\n{want_valid}"
    if rec.pngram is not None:
        np.testing.assert_allclose(cp, rec.pngram, rtol=1e-6, atol=0)
    score_tol = lp_tol + 1e-4 * max(1.0, float(np.max(np.abs(want_score[want_valid == 1]))))
    np.testing.assert_allclose(cs[want_valid == 1], want_score[want_valid == 1], atol=score_tol, rtol=0)
    prune_decisive = rec.gap_prune > 2 * score_tol
    stats["prune_decisive"] = prune_decisive
    got = list(zip(parents.tolist(), tokens.tolist()))
    want = [(c.parent, c.token) for c in rec.kept]
    if prune_decisive:
        assert got == want, f"kept options {got} != oracle {want} (gap {rec.gap_prune:.3e})"
        np.testing.assert_allclose(scores, [c.logscore for c in rec.kept], atol=score_tol, rtol=0)
    else:
        check_valid_prune(got, scores, rec, k, 2 * score_tol)
    return stats


def teacher_forced(sess, lm, tables_np, lambdas, prefix, cfg, n_tokens, rtol, dc, prefilled=False):
    """Run the oracle free; before every GPU step load the oracle's drafts and scores into the
    GPU (its KV cache stays its own), so each step is compared on its own.  With `prefilled`
    the session already stands at the end of `prefix` (after a commit) and is not prefilled."""
    otabs = O.NgramTables(tables_np) if tables_np is not None else None
    state, recs = O.generate(lm, otabs, prefix, cfg, n_tokens)
    if not prefilled:
        sess.spd_prefill(prefix)
    all_stats = []
    for t, rec in enumerate(recs):
        if t > 0:
            sess.spd_set_state(tails_of(rec.state_in), rec.state_in.logscores)
        sess.spd_step_outputs = sess.spd_step(dc)
        all_stats.append(compare_step(sess, rec, dc, rtol, first=(t == 0), cfg=cfg, otabs=otabs, prefix=prefix))
    assert all(s.get("fully_compared") for s in all_stats) and len(all_stats) == n_tokens
    return state, recs, all_stats


def assert_hit_paths_compared(stats, need_penalty=True):
    """With planted tables: the steps compared exactly (on the GPU's own logits) contained at
    least one option in both distributions (Eq. 4) and one in the penalty form (Eq. 5) -- or,
    where the tables are so dense that every draft finds some overlap, one dropped option."""
    assert sum(s.get("own_overlap", 0) for s in stats) >= 1, "no interpolated (Eq. 4) option was compared"
    if need_penalty:
        assert sum(s.get("own_penalty", 0) for s in stats) >= 1, "no penalty-form (Eq. 5) option was compared"
    else:
        assert sum(s.get("own_dropped", 0) for s in stats) >= 1, "no option outside the overlap set was compared"


def plant_both_forms(base, recs0, k, vocab, seed):
    """Planted tables from the records of an alpha = 0 oracle run such that the first full
    timestep certainly shows both forms: nothing is planted for draft 0 at that step (no
    overlap: Eq. 5 for all its options), the best token is planted for draft 1 at every order
    (Eq. 4), and the rest is planted at random (half of the visited pairs) as elsewhere."""
    step1 = recs0[1]
    skip = tuple(step1.state_in.history(0))
    visits = [(tuple(r.state_in.history(i)), int(t)) for r in recs0[1:] for i in range(k) for t in r.top_ids]
    visits = [v for v in visits if v[0] != skip]
    tabs = synth.plant_ngrams(base, visits, vocab, seed=seed, frac=0.5)
    forced = [(tuple(step1.state_in.history(1)), int(step1.top_ids[0]))]
    return synth.plant_ngrams(tabs, forced, vocab, seed=seed + 1, frac=1.0)
