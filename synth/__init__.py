"""Seeded synthetic inputs for Superposed Decoding: model weights, n-gram tables, prefixes.

This module only *draws inputs*.  It holds none of the decoding method's arithmetic and
is the one piece shared by the CPU oracle's tests and the HIP path's tests/benchmarks, so
that both sides consume bit-identical weights, tables and token ids.

Shapes and distributions stand in for the paper's workloads (Section 4: Llama-2-7B
weights, RedPajama n-gram frequency tables for n = 2..6, 15-token OpenWebText prefixes),
none of which are available offline; contents are random.
"""
from __future__ import annotations

import zlib
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field

import numpy as np

__all__ = [
    "ModelShape", "TINY", "LLAMA7B", "LLAMA13B", "LLAMA70B", "bf16_bits", "bf16_widen",
    "make_weights", "make_weights_device", "host_view", "weight_names", "zipf_token_sampler", "make_ngram_tables_uniform",
    "make_ngram_tables_zipf", "plant_ngrams", "make_prefix_uniform", "make_prefix_zipf",
    "PAPER_LAMBDAS", "ORDER_SHARE",
]

# Interpolation weights for n = 2..6 (Appendix B, "N-Gram Interpolation").
PAPER_LAMBDAS = (0.01, 0.04, 0.15, 0.18, 0.12)
# Entry share per order n = 2..6: the paper's on-disk sizes (Section 4: 57 MB, 433 MB,
# 2.15 GB, 4.7 GB, 6.8 GB) divided by n, normalised.
_DISK_MB = (57.0, 433.0, 2150.0, 4700.0, 6800.0)
ORDER_SHARE = tuple((_DISK_MB[i] / (i + 2)) / sum(_DISK_MB[j] / (j + 2) for j in range(5))
                    for i in range(5))


@dataclass(frozen=True)
class ModelShape:
    """Decoder-only transformer shape (RMSNorm, rotary, SwiGLU, untied embed / LM head)."""
    name: str
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    d_ffn: int
    vocab: int
    dtype: str = "bf16"          # "bf16" or "fp32": the storage type of the weights
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0
    init_std: float = 0.02

    @property
    def d_head(self) -> int:
        return self.d_model // self.n_heads

    def streamed_params(self) -> int:
        """Weights every decode step must read once: all layers plus the LM head."""
        dh = self.d_head
        per_layer = ((self.n_heads + 2 * self.n_kv_heads) * dh * self.d_model
                     + self.d_model * self.n_heads * dh + 3 * self.d_ffn * self.d_model)
        return self.n_layers * per_layer + self.vocab * self.d_model

    def truncated(self, n_layers: int) -> "ModelShape":
        return ModelShape(f"{self.name}-L{n_layers}", n_layers, self.d_model, self.n_heads,
                          self.n_kv_heads, self.d_ffn, self.vocab, self.dtype, self.rms_eps,
                          self.rope_theta, self.init_std)


TINY = ModelShape("tiny", 2, 256, 4, 4, 1024, 4096, "fp32")
LLAMA7B = ModelShape("llama2-7b-shape", 32, 4096, 32, 32, 11008, 32000, "bf16")
LLAMA13B = ModelShape("llama2-13b-shape", 40, 5120, 40, 40, 13824, 32000, "bf16")
LLAMA70B = ModelShape("llama2-70b-shape", 80, 8192, 64, 8, 28672, 32000, "bf16")


# ----------------------------------------------------------------------------- bf16 bits
def bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def bf16_widen(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns -> the fp32 values they denote (exact)."""
    return (bits.astype(np.uint32) << 16).view(np.float32)


# ----------------------------------------------------------------------------- weights
def weight_names(shape: ModelShape) -> list[tuple[str, tuple[int, ...], str]]:
    """(name, shape, kind) for every tensor; kind is 'normal' (N(0, std)) or 'ones'."""
    d, dh = shape.d_model, shape.d_head
    out = [("embed", (shape.vocab, d), "normal")]
    for l in range(shape.n_layers):
        p = f"layers.{l}."
        out += [
            (p + "attn_norm", (d,), "ones"),
            (p + "wq", (shape.n_heads * dh, d), "normal"),
            (p + "wk", (shape.n_kv_heads * dh, d), "normal"),
            (p + "wv", (shape.n_kv_heads * dh, d), "normal"),
            (p + "wo", (d, shape.n_heads * dh), "normal"),
            (p + "ffn_norm", (d,), "ones"),
            (p + "w_gate", (shape.d_ffn, d), "normal"),
            (p + "w_up", (shape.d_ffn, d), "normal"),
            (p + "w_down", (d, shape.d_ffn), "normal"),
        ]
    out += [("final_norm", (d,), "ones"), ("lm_head", (shape.vocab, d), "normal")]
    return out


def _tensor_rng(seed: int, name: str) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, zlib.crc32(name.encode())])))


def _draw(seed: int, name: str, shp: tuple[int, ...], kind: str, std: float, dtype: str,
          norm_jitter: float) -> np.ndarray:
    rng = _tensor_rng(seed, name)
    if kind == "ones":
        x = np.ones(shp, dtype=np.float32)
        if norm_jitter:
            x += norm_jitter * rng.standard_normal(shp, dtype=np.float32)
    else:
        x = rng.standard_normal(shp, dtype=np.float32)
        x *= np.float32(std)
    if dtype == "bf16":
        return bf16_bits(x).reshape(shp)
    return x


def make_weights(shape: ModelShape, seed: int = 0, threads: int = 8,
                 norm_jitter: float = 0.0) -> dict[str, np.ndarray]:
    """All tensors of the model, each from its own generator keyed by (seed, name).

    bf16 models come back as uint16 bit patterns (the exact bytes the GPU gets); fp32 models
    as float32.  Matrices are row-major [out_features, in_features].  Norm gains are 1
    (plus N(0, norm_jitter) when asked, so tests can tell a gain apart from no gain).
    """
    specs = weight_names(shape)

    def job(spec):
        name, shp, kind = spec
        return name, _draw(seed, name, shp, kind, shape.init_std, shape.dtype, norm_jitter)

    if threads <= 1:
        return dict(job(s) for s in specs)
    with ThreadPoolExecutor(max_workers=threads) as ex:
        return dict(ex.map(job, specs))


def make_weights_device(shape: ModelShape, seed: int = 0, device: str = "cuda") -> dict:
    """Same tensor set drawn on the GPU with torch's seeded generator (one seed per tensor),
    for shapes too large to draw on the host in reasonable time.  Returns torch tensors in
    the storage dtype, with q/k/v of a layer stored as one fused `wqkv` matrix and
    `wq`/`wk`/`wv` as row-slice views of it.  `host_view` turns any of them into the numpy
    array format `make_weights` returns (bf16 as uint16 bit patterns)."""
    import torch
    tdt = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
    out = {}
    dh = shape.d_head
    nq, nkv = shape.n_heads * dh, shape.n_kv_heads * dh

    def draw(name, shp, kind):
        if kind == "ones":
            return torch.ones(shp, dtype=tdt, device=device)
        g = torch.Generator(device=device)
        g.manual_seed((seed << 32) ^ zlib.crc32(name.encode()))
        x = torch.empty(shp, dtype=torch.float32, device=device)
        x.normal_(0.0, shape.init_std, generator=g)
        return x.to(tdt)

    for name, shp, kind in weight_names(shape):
        base = name.rsplit(".", 1)[-1]
        if base in ("wk", "wv"):
            continue
        if base == "wq":
            p = name[:-2]
            fused = draw(p + "wqkv", (nq + 2 * nkv, shape.d_model), kind)
            out[p + "wqkv"] = fused
            out[p + "wq"], out[p + "wk"], out[p + "wv"] = fused[:nq], fused[nq:nq + nkv], fused[nq + nkv:]
        else:
            out[name] = draw(name, shp, kind)
    return out


def host_view(t) -> np.ndarray:
    """torch tensor (any device) -> numpy array in make_weights' format."""
    import torch
    t = t.detach().contiguous().cpu()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


# ----------------------------------------------------------------------------- token draws
@dataclass
class zipf_token_sampler:
    """Bounded Zipf(a) over ranks 1..vocab; rank -> token id through a seeded permutation."""
    vocab: int
    a: float = 1.1
    seed: int = 0
    _cdf: np.ndarray = field(init=False, repr=False)
    _perm: np.ndarray = field(init=False, repr=False)

    def __post_init__(self):
        w = np.arange(1, self.vocab + 1, dtype=np.float64) ** (-self.a)
        self._cdf = np.cumsum(w / w.sum())
        self._cdf[-1] = 1.0
        self._perm = _tensor_rng(self.seed, "zipf-rank-to-id").permutation(self.vocab).astype(np.int32)

    def draw(self, rng: np.random.Generator, size) -> np.ndarray:
        r = np.searchsorted(self._cdf, rng.random(size), side="right")
        return self._perm[np.minimum(r, self.vocab - 1)]


def _zipf_counts(rng: np.random.Generator, n: int, a: float = 1.1, cap: int = 2 ** 31) -> np.ndarray:
    return np.minimum(rng.zipf(a, n), cap).astype(np.uint32)


def _merge_duplicates(keys: np.ndarray, counts: np.ndarray, cap: int = 2 ** 32 - 1):
    """Sort rows, merge equal keys by summing their counts (clipped to uint32)."""
    if len(keys) == 0:
        return keys, counts
    order = np.lexsort(keys.T[::-1])
    keys, counts = keys[order], counts[order].astype(np.uint64)
    new = np.ones(len(keys), dtype=bool)
    new[1:] = np.any(keys[1:] != keys[:-1], axis=1)
    starts = np.flatnonzero(new)
    summed = np.add.reduceat(counts, starts)
    return np.ascontiguousarray(keys[starts]), np.minimum(summed, cap).astype(np.uint32)


def make_ngram_tables_uniform(vocab: int, entries: dict[int, int], seed: int = 0):
    """Tables with keys uniform over [0, vocab)^n, distinct, and Zipf(1.1) counts.

    `entries` maps order n -> number of distinct n-grams.  Returns {n: (keys int32 [N, n],
    counts uint32 [N])} for n = 2..6 (absent orders come back empty).
    """
    out = {}
    for n in range(2, 7):
        want = entries.get(n, 0)
        rng = _tensor_rng(seed, f"ngram-uniform-{n}")
        keys = np.zeros((0, n), dtype=np.int32)
        while len(keys) < want:
            extra = rng.integers(0, vocab, size=(want - len(keys) + 16, n), dtype=np.int32)
            keys = np.unique(np.concatenate([keys, extra]), axis=0)
        if want:
            keys = keys[rng.permutation(len(keys))[:want]]
        out[n] = (np.ascontiguousarray(keys), _zipf_counts(rng, len(keys)))
    return out


def make_ngram_tables_zipf(vocab: int, total_entries: int, seed: int = 0, orders=(2, 3, 4, 5, 6)):
    """Tables whose tokens are i.i.d. bounded-Zipf(1.1) ids; duplicates merged by summing.

    The draw count per order follows ORDER_SHARE (renormalised over `orders`).
    """
    sampler = zipf_token_sampler(vocab, 1.1, seed)
    share = np.array([ORDER_SHARE[n - 2] for n in orders])
    share = share / share.sum()
    out = {n: (np.zeros((0, n), np.int32), np.zeros((0,), np.uint32)) for n in range(2, 7)}
    for n, s in zip(orders, share):
        rng = _tensor_rng(seed, f"ngram-zipf-{n}")
        draws = int(round(total_entries * s))
        keys = sampler.draw(rng, (draws, n)).astype(np.int32)
        out[n] = _merge_duplicates(keys, _zipf_counts(rng, draws))
    return out


def plant_ngrams(tables, visits, vocab: int, seed: int = 0, frac: float = 0.5, decoys: int = 2):
    """Add n-grams that complete given (history, token) pairs so lookups actually hit.

    `visits` is an iterable of (history tuple of token ids, next token id).  A seeded
    fraction `frac` of them is inserted at every order that fits the history, together with
    `decoys` other continuations of the same context (so context totals exceed the hit
    count).  Duplicates, including with the existing table, are merged by summing.
    """
    rng = _tensor_rng(seed, "ngram-plant")
    add = {n: ([], []) for n in range(2, 7)}
    for hist, tok in visits:
        if rng.random() >= frac:
            continue
        for n in range(2, 7):
            if len(hist) < n - 1 or rng.random() < 0.25:
                continue
            ctx = list(hist[len(hist) - (n - 1):])
            add[n][0].append(ctx + [int(tok)])
            add[n][1].append(int(_zipf_counts(rng, 1)[0]))
            for _ in range(decoys):
                add[n][0].append(ctx + [int(rng.integers(0, vocab))])
                add[n][1].append(int(_zipf_counts(rng, 1)[0]))
    out = {}
    for n in range(2, 7):
        keys, counts = tables.get(n, (np.zeros((0, n), np.int32), np.zeros((0,), np.uint32)))
        if add[n][0]:
            keys = np.concatenate([keys, np.array(add[n][0], dtype=np.int32).reshape(-1, n)])
            counts = np.concatenate([counts, np.array(add[n][1], dtype=np.uint32)])
        out[n] = _merge_duplicates(keys, counts)
    return out


def make_prefix_uniform(vocab: int, m: int, seed: int = 0) -> np.ndarray:
    return _tensor_rng(seed, "prefix-uniform").integers(0, vocab, size=m, dtype=np.int32)


def make_prefix_zipf(vocab: int, m: int, seed: int = 0) -> np.ndarray:
    return zipf_token_sampler(vocab, 1.1, seed).draw(_tensor_rng(seed, "prefix-zipf"), m).astype(np.int32)
