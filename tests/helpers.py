"""Small shared helpers for the tests (no method arithmetic)."""
import numpy as np

import synth
from oracle import spd_oracle as O


def toy_shape(vocab=16, d=16, heads=2, kv=2, ffn=32, layers=1, dtype="fp32", std=0.5):
    return synth.ModelShape("toy", layers, d, heads, kv, ffn, vocab, dtype, init_std=std)


def oracle_lm(shape, seed=0, dtype=np.float32, norm_jitter=0.1, weights=None):
    w = weights if weights is not None else synth.make_weights(shape, seed, threads=1, norm_jitter=norm_jitter)
    return O.OracleLM(w, shape.n_layers, shape.n_heads, shape.n_kv_heads, shape.rms_eps,
                      shape.rope_theta, dtype), w


def read_golden(path):
    out = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, *vals = line.split()
            out[name] = [float(v) for v in vals]
    return out
