"""End-to-end parity of the HIP path with the CPU oracle (through the C ABI)."""
import numpy as np
import pytest
import torch

import synth
from gpu_common import RTOL, assert_hit_paths_compared, plant_both_forms, compare_step, make_oracle, tails_of, teacher_forced
from oracle import spd_oracle as O

pytestmark = pytest.mark.gpu


def P():
    import paper_2405_18400_amd as pkg
    return pkg


def session(shape, weights, max_ctx=64, k_max=8, kv_dtype="fp32"):
    return P().Session(shape, weights, max_ctx=max_ctx, k_max=k_max, kv_dtype=kv_dtype)


def planted_tables(shape, weights, base, prefix, k, n_tokens, seed=0, tau=1.0):
    """Insert n-grams along the paths an alpha = 0 oracle run visits, so lookups hit."""
    lm = make_oracle(shape, weights)
    _, recs = O.generate(lm, None, prefix, O.DecodeCfg(k, 0.0, tau), n_tokens)
    visits = []
    for rec in recs[1:]:
        for i in range(k):
            for tok in rec.top_ids:
                visits.append((tuple(rec.state_in.history(i)), int(tok)))
    return synth.plant_ngrams(base, visits, shape.vocab, seed=seed, frac=0.5)


@pytest.fixture(scope="module")
def tiny():
    shape = synth.TINY
    w = synth.make_weights(shape, seed=0)
    tabs = synth.make_ngram_tables_uniform(shape.vocab, {2: 50_000, 3: 50_000}, seed=0)
    prefix = synth.make_prefix_uniform(shape.vocab, 16, seed=0)
    return shape, w, tabs, prefix


@pytest.fixture(params=["fused", "per_operator"])
def forward_path(request):
    """Both ways the library can run the transformer forward: one persistent kernel, or one
    kernel per matrix-vector product."""
    return request.param


def select_path(sess, path):
    if path == "fused":
        assert sess.spd_get_fused(), "no fused forward kernel was selected for this shape"
    else:
        sess.spd_set_fused(False)
        assert not sess.spd_get_fused()


def run_teacher_forced(shape, w, tabs, lambdas, prefix, k, alpha, n_tokens, tau=1.0, delta=0.1, max_ctx=64,
                       path="fused", kv_dtype="fp32"):
    pkg = P()
    sess = session(shape, w, max_ctx=max_ctx, kv_dtype=kv_dtype)
    try:
        select_path(sess, path)
        if tabs is not None:
            sess.spd_load_ngrams(tabs, lambdas)
        dc = pkg.SpdDecodeCfg(k, alpha, tau, delta)
        cfg = O.DecodeCfg(k, alpha, tau, delta, tuple(lambdas))
        lm = make_oracle(shape, w)
        state, recs, stats = teacher_forced(sess, lm, tabs, lambdas, prefix, cfg, n_tokens, RTOL[shape.dtype], dc)
        assert sess.spd_position() == len(prefix) + n_tokens - 1
        return state, recs, stats
    finally:
        sess.close()


def test_tiny_config_as_specified(tiny, forward_path):
    """BASELINE config 1: 2-layer fp32 model, bigram+trigram tables, k = 3, 10 tokens, alpha 0.5."""
    shape, w, tabs, prefix = tiny
    lam = (0.01, 0.04, 0.0, 0.0, 0.0)
    _, recs, stats = run_teacher_forced(shape, w, tabs, lam, prefix, 3, 0.5, 10, path=forward_path)
    assert sum(s.get("vocab_decisive", False) for s in stats) >= 8


def test_tiny_config_with_planted_hits(tiny, forward_path):
    shape, w, tabs, prefix = tiny
    lam = (0.01, 0.04, 0.0, 0.0, 0.0)
    planted = planted_tables(shape, w, tabs, prefix, 3, 10)
    _, recs, stats = run_teacher_forced(shape, w, planted, lam, prefix, 3, 0.5, 10, path=forward_path)
    assert any(c.overlap for r in recs[1:] for c in r.candidates), "planting produced no n-gram hit"
    assert any(not c.overlap for r in recs[1:] for c in r.candidates)


@pytest.mark.parametrize("k", [1, 2, 5, 8])
@pytest.mark.parametrize("alpha", [0.0, 0.54])
@pytest.mark.parametrize("tau", [0.7, 0.06])
def test_tiny_k_sweep_all_orders(tiny, k, alpha, tau):
    """k from 1 to 8, with and without the n-gram stage, at a mild temperature and at the one the
    paper tuned for its generation experiments (Appendix B, "Hyperparameter Choices": 0.06)."""
    shape, w, _, prefix = tiny
    base = synth.make_ngram_tables_zipf(shape.vocab, 40_000, seed=3)
    planted = planted_tables(shape, w, base, prefix, k, 6, seed=k, tau=tau)
    _, _, stats = run_teacher_forced(shape, w, planted, synth.PAPER_LAMBDAS, prefix, k, alpha, 6, tau=tau)
    if alpha > 0 and k > 1:
        assert_hit_paths_compared(stats)


def test_bf16_small_model_gqa(forward_path):
    shape = synth.ModelShape("small-bf16", 3, 512, 8, 2, 1408, 2048, "bf16")
    w = synth.make_weights(shape, seed=5)
    prefix = synth.make_prefix_zipf(shape.vocab, 37, seed=5)
    base = synth.make_ngram_tables_zipf(shape.vocab, 30_000, seed=5)
    planted = planted_tables(shape, w, base, prefix, 3, 8)
    _, _, stats = run_teacher_forced(shape, w, planted, synth.PAPER_LAMBDAS, prefix, 3, 0.54, 8, path=forward_path)
    assert sum(bool(s.get("fully_compared")) for s in stats) == 8
    assert_hit_paths_compared(stats, need_penalty=False)   # vocabulary of 2048: every draft finds some overlap


def test_long_prefix_crosses_attention_chunks(forward_path):
    shape = synth.ModelShape("small-fp32", 2, 256, 4, 2, 512, 1024, "fp32")
    w = synth.make_weights(shape, seed=6)
    prefix = synth.make_prefix_uniform(shape.vocab, 300, seed=6)
    run_teacher_forced(shape, w, None, synth.PAPER_LAMBDAS, prefix, 3, 0.0, 4, max_ctx=600, path=forward_path)


def test_many_attention_items(forward_path):
    """More (query head, chunk) items than a quarter of the fused kernel's blocks: the blocks
    that hold an item also take rows of the O projection and ask for them behind the item's
    own loads; the last chunk is ragged, so some waves of a block have no position in it."""
    shape = synth.ModelShape("heads32-fp32", 2, 512, 32, 8, 512, 1024, "fp32")
    w = synth.make_weights(shape, seed=9)
    prefix = synth.make_prefix_uniform(shape.vocab, 261, seed=9)
    run_teacher_forced(shape, w, None, synth.PAPER_LAMBDAS, prefix, 3, 0.0, 4, max_ctx=400, path=forward_path)


def test_vocabulary_of_140k_tokens(forward_path):
    """A vocabulary larger than 128 slices of 1024 entries: the per-slice top-k kernel then has
    more entries per slice than its threads keep in registers and walks the rest from memory;
    k = 5 of 140000."""
    shape = synth.ModelShape("vocab140k-fp32", 1, 128, 2, 2, 256, 140000, "fp32")
    w = synth.make_weights(shape, seed=14)
    prefix = synth.make_prefix_uniform(shape.vocab, 7, seed=14)
    run_teacher_forced(shape, w, None, synth.PAPER_LAMBDAS, prefix, 5, 0.0, 4, path=forward_path)


def test_many_small_kv_heads(forward_path):
    """128 key/value heads of d_head 16: four lanes per cached position, and more heads than a
    wave has lanes."""
    shape = synth.ModelShape("heads128-fp32", 2, 2048, 128, 128, 1024, 1024, "fp32")
    w = synth.make_weights(shape, seed=12)
    prefix = synth.make_prefix_uniform(shape.vocab, 19, seed=12)
    run_teacher_forced(shape, w, None, synth.PAPER_LAMBDAS, prefix, 3, 0.0, 4, path=forward_path)


def test_wide_ffn_three_pass_rows(forward_path):
    """d_ffn wider than one block pass (bf16: 4096 columns), ragged against the pass width,
    like the 7B shape's 11008: exercises the multi-pass rows of the fused kernel."""
    shape = synth.ModelShape("wide-ffn-bf16", 2, 512, 4, 4, 4096 * 2 + 1416, 1024, "bf16")
    w = synth.make_weights(shape, seed=7)
    prefix = synth.make_prefix_uniform(shape.vocab, 21, seed=7)
    run_teacher_forced(shape, w, None, synth.PAPER_LAMBDAS, prefix, 2, 0.0, 5, path=forward_path)


def test_two_pass_ffn_rows(forward_path):
    """d_ffn between one and two block passes."""
    shape = synth.ModelShape("ffn2-bf16", 2, 512, 4, 4, 4096 + 2056, 1024, "bf16")
    w = synth.make_weights(shape, seed=8)
    prefix = synth.make_prefix_uniform(shape.vocab, 9, seed=8)
    run_teacher_forced(shape, w, None, synth.PAPER_LAMBDAS, prefix, 2, 0.0, 4, path=forward_path)


def _layer_truncated(shape, n_layers, prefix_len, k, n_tokens, seed, forward_path, alpha=0.54, kv_dtype="fp32"):
    """A published shape with its real widths and head layout but few layers (the oracle runs on
    the host): weights drawn on the GPU, n-gram tables planted along the oracle's path."""
    pkg = P()
    shape = shape.truncated(n_layers)
    wdev = synth.make_weights_device(shape, seed=seed)
    host = {k_: synth.host_view(v) for k_, v in wdev.items() if not k_.endswith("wqkv")}
    prefix = synth.make_prefix_zipf(shape.vocab, prefix_len, seed=seed)
    base = synth.make_ngram_tables_zipf(shape.vocab, 100_000, seed=seed)
    lm = make_oracle(shape, host)
    _, recs0 = O.generate(lm, None, prefix, O.DecodeCfg(k, 0.0), n_tokens)
    tabs = plant_both_forms(base, recs0, k, shape.vocab, seed + 1)
    sess = pkg.Session(shape, wdev, max_ctx=prefix_len + n_tokens + 8, k_max=8, kv_dtype=kv_dtype)
    try:
        select_path(sess, forward_path)
        sess.spd_load_ngrams(tabs, synth.PAPER_LAMBDAS)
        dc = pkg.SpdDecodeCfg(k, alpha, 1.0, 0.1)
        cfg = O.DecodeCfg(k, alpha, 1.0, 0.1, synth.PAPER_LAMBDAS)
        _, recs, stats = teacher_forced(sess, lm, tabs, synth.PAPER_LAMBDAS, prefix, cfg, n_tokens, RTOL["bf16"], dc)
        print(shape.name, "scaled logit errors:", [f"{s['logit_err']:.2e}" for s in stats if "logit_err" in s])
        name = shape.name + (" (fp16 cache)" if kv_dtype == "fp16" else "")
        report_decisions(name, stats, n_tokens)
        return stats
    finally:
        sess.close()


REPORT = []   # one line per large-shape test, printed once past pytest's capture when the module ends


@pytest.fixture(scope="module", autouse=True)
def _print_report(request):
    yield
    if REPORT:
        capman = request.config.pluginmanager.getplugin("capturemanager")
        with capman.global_and_fixture_disabled():
            print()
            for line in REPORT:
                print("  " + line)


def report_decisions(name, stats, n_steps):
    """Every step's decision stage was compared exactly (on the GPU's own logits), and with the
    planted tables both the interpolated and the penalty form of an option occurred."""
    full = sum(bool(s.get("fully_compared")) for s in stats)
    line = (f"{name}: {full}/{n_steps} steps compared exactly on the GPU's own logits; options in both distributions: "
            f"{sum(s.get('own_overlap', 0) for s in stats)}, penalty form: {sum(s.get('own_penalty', 0) for s in stats)}, "
            f"dropped: {sum(s.get('own_dropped', 0) for s in stats)}; steps decisive against the oracle's logits: "
            f"{sum(bool(s.get('vocab_decisive')) for s in stats)}; worst scaled logit error "
            f"{max(s['logit_err'] for s in stats):.1e}")
    print(line)
    REPORT.append(line)
    assert full == n_steps
    assert_hit_paths_compared(stats)


@pytest.mark.timeout(600)
def test_7b_shape_two_layers_context_of_two_load_batches(forward_path):
    """Llama-2-7B widths (32 heads of 128), two layers, 200 cached positions: past the 160 rows
    a block's lanes hold per batch of loads, so the fused kernel's single attention item per
    head walks two batches (the per-operator path cuts the context into two chunks instead)."""
    _layer_truncated(synth.LLAMA7B, 2, 200, 3, 3, 8, forward_path)


@pytest.mark.timeout(600)
def test_7b_shape_two_layers_config3_context(forward_path):
    """BASELINE config 3's context and largest k at the 7B widths, two layers: a 1030-token
    prefix (dense prefix pass over a chunk boundary of its token arena), attention cut into
    chunks that are merged across blocks, k = 8."""
    _layer_truncated(synth.LLAMA7B, 2, 1030, 8, 3, 7, forward_path)


@pytest.mark.timeout(600)
def test_13b_shape_two_layers(forward_path):
    """BASELINE config 4's widths (d_model 5120, 40 heads, FFN 13824: rows of 1.25 and 3.375
    block passes), k = 5, two of its 40 layers."""
    _layer_truncated(synth.LLAMA13B, 2, 140, 5, 4, 13, forward_path)


@pytest.mark.timeout(600)
def test_70b_shape_one_layer(forward_path):
    """BASELINE config 5's widths (d_model 8192, 64 query heads on 8 key/value heads, FFN
    28672), k = 3, one of its 80 layers; the prefix crosses an attention chunk."""
    _layer_truncated(synth.LLAMA70B, 1, 131, 3, 3, 70, forward_path)


@pytest.mark.parametrize("m", [8, 31, 33, 64, 96, 160, 257, 300, 531, 1043])
def test_dense_prefix_pass_matches_the_oracle_and_the_token_by_token_pass(m):
    """The prefix pass on the matrix cores (1024 tokens per weight pass) against the oracle's
    full-sequence forward and against the token-by-token pass: logits after the prefix, and
    three timesteps on top of the cache it filled.  Sizes straddle the 32- and 64-token tiles
    the 128-token activation tiles, the switch between the two GEMM kernels (96 tokens) and
    the 1024-token chunk (1043 = one full chunk + a short one at a non-zero position); grouped
    key/value heads."""
    pkg = P()
    shape = synth.ModelShape("small-bf16-dense", 3, 512, 8, 2, 1408, 2048, "bf16")
    w = synth.make_weights(shape, seed=21)
    prefix = synth.make_prefix_zipf(shape.vocab, m, seed=m)
    lm = make_oracle(shape, w)
    cfg = O.DecodeCfg(3, 0.0)
    dc = pkg.SpdDecodeCfg(3, 0.0, 1.0, 0.1)
    logits = {}
    for dense in (True, False):
        sess = session(shape, w, max_ctx=m + 16)
        try:
            assert sess.spd_get_dense_prefill()
            sess.spd_set_dense_prefill(dense)
            state, recs, stats = teacher_forced(sess, lm, None, synth.PAPER_LAMBDAS, prefix, cfg, 4, RTOL["bf16"], dc)
            assert max(s["logit_err"] for s in stats if "logit_err" in s) < 1e-4      # far inside the bf16 tolerance
            sess.spd_prefill(prefix)
            logits[dense] = sess.spd_read_logits()
        finally:
            sess.close()
    assert np.max(np.abs(logits[True] - logits[False])) <= 1e-4 * np.max(np.abs(logits[False]))


# ---- the fp16 key/value cache a bf16 model may ask for (spd_model_cfg.kv_dtype): every kernel that
# writes or reads the cache, against the same oracle (which keeps its keys and values unrounded), to
# the bf16 tolerance; the rounding of the cache is the only difference to the fp32-cache cases above,
# whose tighter bounds pin the logic.
FP16_CACHE_LOGIT_ERR = 8e-3   # of the largest |logit|: 11 significant bits in every cached key and value


def test_fp16_cache_small_model_gqa(forward_path):
    shape = synth.ModelShape("small-bf16", 3, 512, 8, 2, 1408, 2048, "bf16")
    w = synth.make_weights(shape, seed=5)
    prefix = synth.make_prefix_zipf(shape.vocab, 37, seed=5)
    base = synth.make_ngram_tables_zipf(shape.vocab, 30_000, seed=5)
    planted = planted_tables(shape, w, base, prefix, 3, 8)
    _, _, stats = run_teacher_forced(shape, w, planted, synth.PAPER_LAMBDAS, prefix, 3, 0.54, 8, path=forward_path, kv_dtype="fp16")
    assert max(s["logit_err"] for s in stats if "logit_err" in s) < FP16_CACHE_LOGIT_ERR


@pytest.mark.timeout(600)
@pytest.mark.parametrize("prefix_len,k", [(40, 3), (200, 3), (300, 5), (1030, 8)])
def test_fp16_cache_7b_shape_two_layers(forward_path, prefix_len, k):
    """Llama-2-7B widths, two layers, fp16 cache: a short context, one attention item per head in
    two batches of loads (200), chunks merged across blocks (300, and BASELINE config 3's 1030
    with k = 8, whose prefix also crosses a chunk of the dense prefix pass)."""
    stats = _layer_truncated(synth.LLAMA7B, 2, prefix_len, k, 3, 8, forward_path, kv_dtype="fp16")
    assert max(s["logit_err"] for s in stats if "logit_err" in s) < FP16_CACHE_LOGIT_ERR


@pytest.mark.timeout(600)
def test_fp16_cache_13b_shape_two_layers():
    stats = _layer_truncated(synth.LLAMA13B, 2, 140, 5, 4, 13, "fused", kv_dtype="fp16")
    assert max(s["logit_err"] for s in stats if "logit_err" in s) < FP16_CACHE_LOGIT_ERR


@pytest.mark.timeout(600)
def test_fp16_cache_70b_shape_one_layer():
    """Grouped key/value heads (8 query heads per cached head) over an attention chunk boundary."""
    stats = _layer_truncated(synth.LLAMA70B, 1, 131, 3, 3, 70, "fused", kv_dtype="fp16")
    assert max(s["logit_err"] for s in stats if "logit_err" in s) < FP16_CACHE_LOGIT_ERR


@pytest.mark.parametrize("m", [8, 33, 96, 300, 1043])
def test_fp16_cache_dense_prefix_pass(m):
    """The prefix pass on the matrix cores and the token-by-token pass fill the fp16 cache with the
    same roundings of (nearly) the same values: their logits agree far more closely than either
    agrees with the oracle."""
    shape = synth.ModelShape("small-bf16-dense", 3, 512, 8, 2, 1408, 2048, "bf16")
    w = synth.make_weights(shape, seed=21)
    prefix = synth.make_prefix_zipf(shape.vocab, m, seed=m)
    lm = make_oracle(shape, w)
    cfg = O.DecodeCfg(3, 0.0)
    dc = P().SpdDecodeCfg(3, 0.0, 1.0, 0.1)
    logits = {}
    for dense in (True, False):
        sess = session(shape, w, max_ctx=m + 16, kv_dtype="fp16")
        try:
            sess.spd_set_dense_prefill(dense)
            state, recs, stats = teacher_forced(sess, lm, None, synth.PAPER_LAMBDAS, prefix, cfg, 4, RTOL["bf16"], dc)
            assert max(s["logit_err"] for s in stats if "logit_err" in s) < FP16_CACHE_LOGIT_ERR
            sess.spd_prefill(prefix)
            logits[dense] = sess.spd_read_logits()
        finally:
            sess.close()
    assert np.max(np.abs(logits[True] - logits[False])) <= 1e-3 * np.max(np.abs(logits[False]))


def test_fp16_cache_head_width_32_plain_prefix_attention():
    """d_head 32: the prefix pass uses its plain (not matrix-core) attention kernel."""
    shape = synth.ModelShape("small-bf16-dh32", 2, 256, 8, 4, 512, 1024, "bf16")
    w = synth.make_weights(shape, seed=23)
    prefix = synth.make_prefix_zipf(shape.vocab, 150, seed=23)
    _, _, stats = run_teacher_forced(shape, w, None, synth.PAPER_LAMBDAS, prefix, 3, 0.0, 4, max_ctx=200, kv_dtype="fp16")
    assert max(s["logit_err"] for s in stats if "logit_err" in s) < FP16_CACHE_LOGIT_ERR


def test_fp16_cache_graph_replay_is_bit_exact_across_the_switch_of_reading_widths():
    """A free-running generation whose context passes 160 positions (where the persistent kernel
    goes from 8-byte to 16-byte pieces of the fp16 cache): graph replay, plain launches and a
    second replayed generation give the same bits; the per-operator forward agrees to rounding."""
    pkg = P()
    shape = synth.ModelShape("small-bf16", 3, 512, 8, 2, 1408, 2048, "bf16")
    w = synth.make_weights(shape, seed=5)
    prefix = synth.make_prefix_zipf(shape.vocab, 150, seed=9)
    dc = pkg.SpdDecodeCfg(3, 0.0, 1.0, 0.1)
    sess = session(shape, w, max_ctx=200, kv_dtype="fp16")
    try:
        drafts, scores = sess.spd_generate(prefix, dc, 24)
        logits = sess.spd_read_logits()
        sess.spd_set_graph(False)
        drafts2, scores2 = sess.spd_generate(prefix, dc, 24)
        assert np.array_equal(drafts, drafts2) and np.array_equal(scores, scores2)
        assert np.array_equal(logits, sess.spd_read_logits())
        sess.spd_set_graph(True)
        drafts3, scores3 = sess.spd_generate(prefix, dc, 24)
        assert np.array_equal(drafts, drafts3) and np.array_equal(scores, scores3)
        # the same prefix and the same first timesteps through one kernel per operator
        sess.spd_prefill(prefix)
        sess.spd_step(dc)
        sess.spd_step(dc)
        fused = sess.spd_read_logits()
        sess.spd_set_fused(False)
        sess.spd_prefill(prefix)
        sess.spd_step(dc)
        sess.spd_step(dc)
        per_op = sess.spd_read_logits()
        np.testing.assert_allclose(fused, per_op, rtol=0, atol=2e-5 * np.abs(per_op).max())
    finally:
        sess.close()


def test_dense_prefix_pass_is_refused_where_it_does_not_exist(tiny):
    shape, w, tabs, prefix = tiny           # fp32 weights
    sess = session(shape, w)
    try:
        assert not sess.spd_get_dense_prefill()
        with pytest.raises(P().SpdError):
            sess.spd_set_dense_prefill(True)
        sess.spd_set_dense_prefill(False)
    finally:
        sess.close()


def test_fused_and_per_operator_forward_agree(tiny):
    """Same inputs through both forward paths: logits agree to fp32 rounding, drafts are equal."""
    shape, w, tabs, prefix = tiny
    pkg = P()
    out = {}
    for path in ("fused", "per_operator"):
        sess = session(shape, w)
        try:
            select_path(sess, path)
            sess.spd_prefill(prefix)
            logits = sess.spd_read_logits()
            drafts, scores = sess.spd_generate(prefix, pkg.SpdDecodeCfg(3, 0.0, 1.0, 0.1), 6)
            out[path] = (logits, drafts, scores)
        finally:
            sess.close()
    np.testing.assert_allclose(out["fused"][0], out["per_operator"][0], rtol=0, atol=2e-5 * np.abs(out["fused"][0]).max())


def test_generate_free_running_matches_until_first_undecided_step(tiny):
    shape, w, tabs, prefix = tiny
    pkg = P()
    lam = (0.01, 0.04, 0.0, 0.0, 0.0)
    planted = planted_tables(shape, w, tabs, prefix, 3, 10)
    sess = session(shape, w)
    try:
        sess.spd_load_ngrams(planted, lam)
        dc = pkg.SpdDecodeCfg(3, 0.5, 1.0, 0.1)
        drafts, scores = sess.spd_generate(prefix, dc, 10)
        lm = make_oracle(shape, w)
        state, recs = O.generate(lm, O.NgramTables(planted), prefix, O.DecodeCfg(3, 0.5, 1.0, 0.1, lam), 10)
        tol = RTOL["fp32"] * max(float(np.max(np.abs(r.logits))) for r in recs)
        decided = 0
        for r in recs:
            if r.gap_vocab <= 4 * tol or r.gap_prune <= 4 * tol:
                break
            decided += 1
        assert decided >= 5, "synthetic case too close to ties to say anything"
        if decided == len(recs):
            assert drafts.tolist() == state.drafts
            np.testing.assert_allclose(scores, state.logscores, atol=1e-3)
        else:
            # up to the first undecided step both sides hold the same set of drafts; whatever the
            # GPU kept later descends from that set
            upto = {tuple(d) for d in recs[decided].state_in.drafts}
            assert {tuple(d[:decided]) for d in drafts.tolist()} <= upto
        # graph replay and plain launches agree bit for bit
        sess.spd_set_graph(False)
        drafts2, scores2 = sess.spd_generate(prefix, dc, 10)
        assert np.array_equal(drafts, drafts2) and np.array_equal(scores, scores2)
        # and so does a second replayed generation (determinism, counters reset, state reset)
        sess.spd_set_graph(True)
        drafts3, scores3 = sess.spd_generate(prefix, dc, 10)
        assert np.array_equal(drafts, drafts3) and np.array_equal(scores, scores3)
    finally:
        sess.close()


def test_k1_is_greedy_on_the_gpu(tiny):
    shape, w, _, prefix = tiny
    pkg = P()
    sess = session(shape, w)
    try:
        drafts, _ = sess.spd_generate(prefix, pkg.SpdDecodeCfg(1, 0.0, 1.0, 0.1), 8)
        lm = make_oracle(shape, w)
        logits = lm.forward(lm.embedding_rows(prefix))
        for t in range(8):
            srt = np.sort(logits)[::-1]
            if srt[0] - srt[1] < 1e-3:
                break
            assert drafts[0, t] == int(np.argmax(logits))
            logits = lm.forward(lm.embedding_rows([int(np.argmax(logits))]))
    finally:
        sess.close()


def test_expand_prune_on_scripted_logits_with_ties(tiny):
    """Decision logic alone: crafted logits (exact ties included) fed straight to the
    post-forward kernels; everything here is integer- or fp32-exact, so results are compared
    without a gap allowance."""
    shape, w, tabs, prefix = tiny
    pkg = P()
    lam = synth.PAPER_LAMBDAS
    rng = np.random.default_rng(0)
    sess = session(shape, w)
    try:
        k = 4
        corpus = rng.integers(0, 12, size=600)
        from collections import Counter
        ctabs = {}
        for n in range(2, 7):
            c = Counter(tuple(corpus[i:i + n]) for i in range(len(corpus) - n + 1))
            ctabs[n] = (np.array(list(c.keys()), np.int32).reshape(-1, n), np.array(list(c.values()), np.uint32))
        sess.spd_load_ngrams(ctabs, lam)
        otabs = O.NgramTables(ctabs)
        pre = corpus[:7].astype(np.int32)
        sess.spd_prefill(pre)
        for alpha in (0.54, 0.0):
            dc = pkg.SpdDecodeCfg(k, alpha, 1.0, 0.1)
            cfg = O.DecodeCfg(k, alpha, 1.0, 0.1, lam)
            state = None
            for step in range(6):
                z = np.full(shape.vocab, -8.0, np.float32)
                z[:14] = rng.integers(0, 4, size=14).astype(np.float32)      # many exact ties among 14 tokens
                if state is None:
                    state, rec = O.first_step(z, pre, cfg)
                else:
                    state, rec = O.expand_and_prune(state, z, otabs, cfg)
                sess.spd_expand_prune(dc, torch.from_numpy(z).cuda(), first=(step == 0))
                tails, sc, gamma = sess.spd_get_state()
                ids, lp, cs, cv, cp = sess.spd_get_step_info(k)
                assert list(ids) == list(rec.top_ids)
                np.testing.assert_allclose(lp, rec.top_logp, rtol=2e-6)
                assert np.array_equal(tails, tails_of(state))
                np.testing.assert_allclose(sc, state.logscores, rtol=1e-5, atol=1e-5)
                np.testing.assert_allclose(gamma, O.superposition_weights(state.logscores), rtol=1e-5)
                assert abs(float(gamma.sum()) - 1.0) < 1e-6
                if step > 0 and alpha > 0:
                    np.testing.assert_allclose(cp, rec.pngram, rtol=1e-6)
                    assert rec.pngram.max() > 0
                # keep both sides on identical scores so ties stay ties
                sess.spd_set_state(tails_of(state), state.logscores)
    finally:
        sess.close()


def test_many_small_hash_tables_against_the_oracle(tiny):
    """The n-gram probabilities of the k x k options on 150 different tiny tables (about a
    hundred keys in about two hundred slots each): clusters of displaced keys occur all over
    such a table, at its end too, where the probe sequence wraps round to slot 0; the oracle
    looks the same n-grams up in plain dictionaries.  Exact comparison (counts are integers,
    the mixture of Eq. 3 is a handful of fp32 operations in a fixed order)."""
    shape, w, _, _ = tiny
    pkg = P()
    lam = synth.PAPER_LAMBDAS
    from collections import Counter
    sess = session(shape, w)
    try:
        k = 3
        dc = pkg.SpdDecodeCfg(k, 0.54, 1.0, 0.1)
        cfg = O.DecodeCfg(k, 0.54, 1.0, 0.1, lam)
        hits = 0
        for seed in range(150):
            rng = np.random.default_rng(1000 + seed)
            corpus = rng.integers(0, 6, size=16)
            ctabs = {}
            for n in range(2, 7):
                c = Counter(tuple(corpus[i:i + n]) for i in range(len(corpus) - n + 1))
                ctabs[n] = (np.array(list(c.keys()), np.int32).reshape(-1, n), np.array(list(c.values()), np.uint32))
            sess.spd_load_ngrams(ctabs, lam)
            otabs = O.NgramTables(ctabs)
            pre = corpus[:6].astype(np.int32)
            sess.spd_prefill(pre)
            state = None
            for step in range(3):
                z = np.full(shape.vocab, -8.0, np.float32)
                z[:6] = rng.permutation(6).astype(np.float32)   # distinct: no ties, top-k inside the corpus alphabet
                if state is None:
                    state, rec = O.first_step(z, pre, cfg)
                else:
                    state, rec = O.expand_and_prune(state, z, otabs, cfg)
                sess.spd_expand_prune(dc, torch.from_numpy(z).cuda(), first=(step == 0))
                ids, lp, cs, cv, cp = sess.spd_get_step_info(k)
                assert list(ids) == list(rec.top_ids), f"table {seed} step {step}"
                if step > 0:
                    np.testing.assert_allclose(cp, rec.pngram, rtol=1e-6, err_msg=f"table {seed} step {step}")
                    hits += int(np.count_nonzero(rec.pngram))
                sess.spd_set_state(tails_of(state), state.logscores)
        assert hits > 300   # the tables were hit, not merely missed consistently
    finally:
        sess.close()


def test_error_paths(tiny):
    shape, w, tabs, prefix = tiny
    pkg = P()
    sess = session(shape, w, max_ctx=20, k_max=4)
    try:
        dc = pkg.SpdDecodeCfg(3, 0.0, 1.0, 0.1)
        with pytest.raises(pkg.SpdError) as e:
            sess.spd_step(dc)
        assert e.value.code == -2
        with pytest.raises(pkg.SpdError) as e:
            sess.spd_prefill(np.arange(20))
        assert e.value.code == -3
        with pytest.raises(pkg.SpdError) as e:
            sess.spd_prefill([0, shape.vocab])
        assert e.value.code == -1
        sess.spd_prefill(prefix)                      # 16 positions of 20
        with pytest.raises(pkg.SpdError) as e:
            sess.spd_step(pkg.SpdDecodeCfg(5, 0.0, 1.0, 0.1))      # k > k_max
        assert e.value.code == -1
        with pytest.raises(pkg.SpdError) as e:
            sess.spd_step(pkg.SpdDecodeCfg(3, 0.5, 1.0, 0.1))      # alpha > 0 without tables
        assert e.value.code == -1
        for _ in range(5):                            # first step + 4 forwards fill the cache
            sess.spd_step(dc)
        with pytest.raises(pkg.SpdError) as e:
            sess.spd_step(dc)
        assert e.value.code == -3
        bad = {2: (np.array([[1, 2], [1, 2]], np.int32), np.array([1, 1], np.uint32))}
        with pytest.raises(pkg.SpdError) as e:
            sess.spd_load_ngrams(bad, synth.PAPER_LAMBDAS)
        assert e.value.code == -5 and "duplicate" in str(e.value)
        for keys, counts in (([[1, shape.vocab]], [1]), ([[1, 2]], [0])):
            with pytest.raises(pkg.SpdError) as e:
                sess.spd_load_ngrams({2: (np.array(keys, np.int32), np.array(counts, np.uint32))}, synth.PAPER_LAMBDAS)
            assert e.value.code == -5
    finally:
        sess.close()


@pytest.mark.timeout(900)
@pytest.mark.parametrize("kv_dtype", ["fp16", "fp32"])
def test_full_size_7b_shape_teacher_forced(kv_dtype):
    """BASELINE config 2 at its real size and in the launch configuration the benchmark times
    (fused forward, graph replay, fp16 cache; and with the fp32 cache): Llama-2-7B shape, bf16,
    64-token Zipf prefix, k = 3, alpha = 0.54, synthetic n = 2..6 tables.  The oracle runs the
    full model on the host (a few seconds per step), so three timesteps are compared,
    teacher-forced."""
    pkg = P()
    shape = synth.LLAMA7B
    wdev = synth.make_weights_device(shape, seed=0)
    host = {k: synth.host_view(v) for k, v in wdev.items() if not k.endswith("wqkv")}
    prefix = synth.make_prefix_zipf(shape.vocab, 64, seed=0)
    base = synth.make_ngram_tables_zipf(shape.vocab, 200_000, seed=0)
    lm = make_oracle(shape, host)
    _, recs0 = O.generate(lm, None, prefix, O.DecodeCfg(3, 0.0), 3)
    tabs = plant_both_forms(base, recs0, 3, shape.vocab, 1)
    sess = pkg.Session(shape, wdev, max_ctx=128, k_max=8, kv_dtype=kv_dtype)
    try:
        assert sess.spd_get_fused()
        sess.spd_load_ngrams(tabs, synth.PAPER_LAMBDAS)
        dc = pkg.SpdDecodeCfg(3, 0.54, 1.0, 0.1)
        cfg = O.DecodeCfg(3, 0.54, 1.0, 0.1, synth.PAPER_LAMBDAS)
        _, recs, stats = teacher_forced(sess, lm, tabs, synth.PAPER_LAMBDAS, prefix, cfg, 3, RTOL["bf16"], dc)
        assert all("logit_err" in s for s in stats)
        print("7B scaled logit errors:", [f"{s['logit_err']:.2e}" for s in stats])
        report_decisions(f"7B full size ({kv_dtype} cache)", stats, 3)
    finally:
        sess.close()


def test_device_error_word_reaches_the_caller(tiny):
    """The getters (and every call that fetches results) report SPD_EHIP once the device-side
    error word is set; here it is written by a fill kernel after the work has finished -- no
    wait fails, no kernel runs while it is set -- and the next prefix pass clears it."""
    shape, w, _, prefix = tiny
    pkg = P()
    sess = session(shape, w)
    try:
        dc = pkg.SpdDecodeCfg(3, 0.0, 1.0, 0.1)
        sess.spd_prefill(prefix)
        sess.spd_step(dc)
        sess.spd_step(dc)
        sess.spd_get_state()
        sess.spd_test_poke_err(1)
        for call in (sess.spd_get_state, lambda: sess.spd_get_step_info(3)):
            with pytest.raises(pkg.SpdError) as e:
                call()
            assert e.value.code == -6 and "barrier" in str(e.value)
        sess.spd_prefill(prefix)
        tok, par, sc = sess.spd_step(dc)
        assert len(tok) == 3
        sess.spd_get_state()
    finally:
        sess.close()
