"""Shared pieces of the GPU parity tests: tolerances and the step-by-step comparison."""
import numpy as np

import synth
from oracle import spd_oracle as O

# Tolerances (north-star): logits and probabilities agree to within a relative 1e-4 on the fp32
# path and 2e-2 on the bf16 path.  "Relative" is taken against the largest magnitude of the
# vector compared (an element-wise ratio is meaningless for logits that cross zero).
RTOL = {"fp32": 1e-4, "bf16": 2e-2}


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


def compare_step(sess, rec, dc, rtol, first, check_logits=True):
    """Compare what the GPU decided in its latest step with the oracle's record of the same
    step.  Integer results must match exactly wherever the oracle's deciding gap exceeds the
    float tolerance; elsewhere the GPU result must be a permutation inside the gap."""
    k = dc.k
    stats = {}
    if check_logits:
        logits = sess.spd_read_logits()
        stats["logit_err"] = assert_close_scaled(logits, rec.logits, rtol, "logits")
    tol_abs = rtol * float(np.max(np.abs(rec.logits)))
    ids, lp, cs, cv, cp = sess.spd_get_step_info(k)
    vocab_decisive = rec.gap_vocab > 2 * tol_abs
    stats["vocab_decisive"] = vocab_decisive
    if vocab_decisive:
        assert list(ids) == list(rec.top_ids), f"KeepTopK ids {ids} != oracle {rec.top_ids} (gap {rec.gap_vocab:.3e})"
        # log-probabilities: error of a logit difference, scaled by 1/tau
        np.testing.assert_allclose(lp, rec.top_logp, atol=2 * tol_abs / dc.tau + 1e-5, rtol=0)
    else:
        assert len(set(ids.tolist())) == k
        return stats
    tokens, parents, scores = sess.spd_step_outputs
    if first:
        assert list(tokens) == list(rec.top_ids) and list(parents) == [-1] * k
        np.testing.assert_allclose(scores, rec.top_logp, atol=2 * tol_abs / dc.tau + 1e-5, rtol=0)
        return stats
    # option table: which (draft, token) pairs are options is integer-exact (n-gram hits)
    want_valid = np.zeros((k, k), np.int32)
    want_score = np.full((k, k), -np.inf)
    for c in rec.candidates:
        want_valid[c.parent, c.rank] = 1
        want_score[c.parent, c.rank] = c.logscore
    assert np.array_equal(cv, want_valid), f"option mask differs:\n{cv}\n{want_valid}"
    if rec.pngram is not None:
        np.testing.assert_allclose(cp, rec.pngram, rtol=1e-6, atol=0)
    score_tol = 2 * tol_abs / dc.tau + 1e-4 * max(1.0, float(np.max(np.abs(want_score[want_valid == 1]))))
    np.testing.assert_allclose(cs[want_valid == 1], want_score[want_valid == 1], atol=score_tol, rtol=0)
    prune_decisive = rec.gap_prune > 2 * score_tol
    stats["prune_decisive"] = prune_decisive
    got = list(zip(parents.tolist(), tokens.tolist()))
    want = [(c.parent, c.token) for c in rec.kept]
    if prune_decisive:
        assert got == want, f"kept options {got} != oracle {want} (gap {rec.gap_prune:.3e})"
        np.testing.assert_allclose(scores, [c.logscore for c in rec.kept], atol=score_tol, rtol=0)
    else:
        valid_pairs = {(c.parent, c.token) for c in rec.candidates}
        assert len(set(got)) == k and set(got) <= valid_pairs
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
        all_stats.append(compare_step(sess, rec, dc, rtol, first=(t == 0)))
    return state, recs, all_stats
