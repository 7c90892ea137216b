"""Pins for the oracle's transformer forward: library routines, closed forms, invariants."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth
from helpers import oracle_lm, toy_shape
from oracle import spd_oracle as O


def torch_full_forward(w, shape, X):
    """Non-cached, whole-sequence causal forward from torch library ops in float64:
    F.rms_norm, F.scaled_dot_product_attention(is_causal), F.silu, complex-multiply rotary."""
    t = lambda n: torch.from_numpy(np.asarray(w[n], dtype=np.float64))
    h = torch.from_numpy(np.asarray(X, dtype=np.float64))
    T, d = h.shape
    H, Hkv, dh = shape.n_heads, shape.n_kv_heads, shape.d_head
    freqs = shape.rope_theta ** (-torch.arange(0, dh, 2, dtype=torch.float64) / dh)
    rot = torch.polar(torch.ones(T, dh // 2, dtype=torch.float64),
                      torch.arange(T, dtype=torch.float64)[:, None] * freqs[None])

    def rotary(x):  # [T, heads, dh]
        xc = torch.view_as_complex(x.reshape(T, -1, dh // 2, 2).contiguous())
        return torch.view_as_real(xc * rot[:, None, :]).reshape(T, -1, dh)

    for l in range(shape.n_layers):
        p = f"layers.{l}."
        a = F.rms_norm(h, (d,), t(p + "attn_norm"), shape.rms_eps)
        q = rotary((a @ t(p + "wq").T).reshape(T, H, dh)).transpose(0, 1)
        k = rotary((a @ t(p + "wk").T).reshape(T, Hkv, dh)).transpose(0, 1)
        v = (a @ t(p + "wv").T).reshape(T, Hkv, dh).transpose(0, 1)
        k, v = k.repeat_interleave(H // Hkv, 0), v.repeat_interleave(H // Hkv, 0)
        att = F.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True)[0]
        h = h + att.transpose(0, 1).reshape(T, H * dh) @ t(p + "wo").T
        b = F.rms_norm(h, (d,), t(p + "ffn_norm"), shape.rms_eps)
        h = h + (F.silu(b @ t(p + "w_gate").T) * (b @ t(p + "w_up").T)) @ t(p + "w_down").T
    return (F.rms_norm(h, (d,), t("final_norm"), shape.rms_eps) @ t("lm_head").T).numpy()


@pytest.mark.parametrize("kv", [4, 2, 1])
def test_forward_matches_torch_library_full_sequence(kv):
    shape = toy_shape(vocab=50, d=32, heads=4, kv=kv, ffn=48, layers=3)
    lm, w = oracle_lm(shape, seed=3, dtype=np.float64)
    toks = synth.make_prefix_uniform(shape.vocab, 9, seed=1)
    X = lm.embedding_rows(toks)
    want = torch_full_forward(w, shape, X)
    got = lm.forward(X, all_positions=True)
    np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-12)
    # float32 arithmetic agrees with the float64 library result to float32 accuracy
    lm32, _ = oracle_lm(shape, dtype=np.float32, weights=w)
    got32 = lm32.forward(lm32.embedding_rows(toks), all_positions=True)
    np.testing.assert_allclose(got32, want, rtol=2e-4, atol=2e-5)


def test_incremental_cache_equals_whole_sequence():
    shape = toy_shape(vocab=40, d=32, heads=4, kv=2, ffn=64, layers=2)
    lm, w = oracle_lm(shape, seed=5, dtype=np.float64)
    X = lm.embedding_rows(synth.make_prefix_uniform(shape.vocab, 7, seed=2))
    whole = lm.forward(X, all_positions=True)
    lm.reset()
    step = np.stack([lm.forward(X[t:t + 1]) for t in range(len(X))])
    np.testing.assert_allclose(step, whole, rtol=1e-11, atol=1e-13)
    assert lm.pos == 7 and all(len(K) == 7 for K in lm.K) and all(len(V) == 7 for V in lm.V)
    # split 4 + 3 as prefill + continuation
    lm.reset()
    lm.forward(X[:4])
    np.testing.assert_allclose(lm.forward(X[4:]), whole[-1], rtol=1e-11, atol=1e-13)


def test_zero_layers_is_head_of_normalised_embedding():
    shape = toy_shape(vocab=30, d=16, layers=0)
    lm, w = oracle_lm(shape, seed=1, dtype=np.float64)
    x = lm.embedding_rows([7])[0]
    want = w["lm_head"].astype(np.float64) @ (x / np.sqrt(np.mean(x * x) + shape.rms_eps) * w["final_norm"])
    np.testing.assert_allclose(lm.forward(x[None]), want, rtol=1e-12)


def test_single_position_attention_returns_value_vector():
    """With one cached position softmax is 1, so the attention output is v itself:
    after one layer with a zero FFN, h = x + Wo Wv norm(x)."""
    shape = toy_shape(vocab=20, d=16, heads=2, kv=2, ffn=8, layers=1)
    w = synth.make_weights(shape, 2, threads=1, norm_jitter=0.1)
    w["layers.0.w_down"] = np.zeros_like(w["layers.0.w_down"])
    lm, _ = oracle_lm(shape, dtype=np.float64, weights=w)
    x = lm.embedding_rows([3])[0]
    a = x / np.sqrt(np.mean(x * x) + shape.rms_eps) * w["layers.0.attn_norm"]
    h = x + w["layers.0.wo"].astype(np.float64) @ (w["layers.0.wv"].astype(np.float64) @ a)
    want = w["lm_head"].astype(np.float64) @ (h / np.sqrt(np.mean(h * h) + shape.rms_eps) * w["final_norm"])
    np.testing.assert_allclose(lm.forward(x[None]), want, rtol=1e-11)


def test_rope_properties():
    rng = np.random.default_rng(0)
    q = rng.standard_normal((1, 3, 8))
    k = rng.standard_normal((1, 3, 8))
    np.testing.assert_array_equal(O.rope(q, [0], 10000.0), q)                       # position 0: identity
    np.testing.assert_allclose(np.linalg.norm(O.rope(q, [11], 10000.0), axis=-1),
                               np.linalg.norm(q, axis=-1), rtol=1e-12)              # a rotation
    dots = [np.sum(O.rope(q, [m], 10000.0) * O.rope(k, [m - 3], 10000.0), -1) for m in (3, 9, 40)]
    np.testing.assert_allclose(dots[0], dots[1], rtol=1e-9)                         # depends on m - n only
    np.testing.assert_allclose(dots[0], dots[2], rtol=1e-9)
    # pair (0, 1) turns by pos * theta^0 = pos radians; last pair by pos * theta^(-(dh-2)/dh)
    x = np.zeros((1, 1, 8)); x[0, 0, 0] = 1.0; x[0, 0, 6] = 1.0
    y = O.rope(x, [2], 10000.0)[0, 0]
    np.testing.assert_allclose(y[:2], [np.cos(2.0), np.sin(2.0)], rtol=1e-12)
    ang = 2.0 * 10000.0 ** (-6 / 8)
    np.testing.assert_allclose(y[6:], [np.cos(ang), np.sin(ang)], rtol=1e-12)


def test_gqa_equals_mha_with_replicated_kv_heads():
    gqa = toy_shape(vocab=24, d=32, heads=4, kv=2, ffn=32, layers=2)
    w = synth.make_weights(gqa, 7, threads=1)
    mha = toy_shape(vocab=24, d=32, heads=4, kv=4, ffn=32, layers=2)
    w2 = dict(w)
    for l in range(2):
        for nm in ("wk", "wv"):
            m = w[f"layers.{l}.{nm}"].reshape(2, 8, 32)
            w2[f"layers.{l}.{nm}"] = np.repeat(m, 2, axis=0).reshape(32, 32)
    a, _ = oracle_lm(gqa, dtype=np.float64, weights=w)
    b, _ = oracle_lm(mha, dtype=np.float64, weights=w2)
    X = a.embedding_rows([1, 5, 9, 2])
    np.testing.assert_allclose(a.forward(X), b.forward(X), rtol=1e-12)


def test_bf16_bit_patterns_are_widened_exactly():
    shape = toy_shape(vocab=20, d=16, layers=1, dtype="bf16")
    bits = synth.make_weights(shape, 4, threads=1)
    assert bits["embed"].dtype == np.uint16
    wide = {k: synth.bf16_widen(v) for k, v in bits.items()}
    a, _ = oracle_lm(shape, weights=bits)
    b, _ = oracle_lm(shape, weights=wide)
    np.testing.assert_array_equal(a.forward(a.embedding_rows([3, 4])), b.forward(b.embedding_rows([3, 4])))
    # round-to-nearest-even on a hand-checked pattern: 1 + 2^-8 is a tie -> even mantissa (1.0)
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -2.5, 0.0], np.float32)
    np.testing.assert_array_equal(synth.bf16_widen(synth.bf16_bits(x)), np.array([1.0, 1.0 + 2.0 ** -6, -2.5, 0.0], np.float32))
