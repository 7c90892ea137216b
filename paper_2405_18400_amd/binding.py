"""ctypes binding for libspd (include/spd.h): argument marshalling only.

PyTorch appears here solely as the owner of device memory and of the HIP stream; every
step of the decoding path runs inside the library's kernels.  There is no fallback: if the
library has not been built this module raises on first use.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
SPD_K_MAX, SPD_TAIL, SPD_N_ORDERS = 16, 5, 5
SPD_DTYPE = {"fp32": 0, "bf16": 1, "fp16": 2}   # fp16: key/value cache only
_lib = None


class SpdError(RuntimeError):
    def __init__(self, code, where, detail=""):
        self.code = code
        super().__init__(f"{where}: {spd_strerror(code)} ({code}) {detail}".strip())


class SpdModelCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "n_kv_heads", "d_ffn", "vocab",
                                          "max_ctx", "k_max", "dtype")] + [("rms_eps", C.c_float), ("rope_theta", C.c_float),
                                                                      ("kv_dtype", C.c_int32)]


class SpdLayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")]


class SpdWeightPtrs(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("layers", C.POINTER(SpdLayerWeights)), ("final_norm", C.c_void_p),
                ("lm_head", C.c_void_p)]


class SpdNgramHostTables(C.Structure):
    _fields_ = [("keys", C.c_void_p * SPD_N_ORDERS), ("counts", C.c_void_p * SPD_N_ORDERS),
                ("n_entries", C.c_int64 * SPD_N_ORDERS), ("lambda_", C.c_float * SPD_N_ORDERS)]


class SpdDecodeCfg(C.Structure):
    _fields_ = [("k", C.c_int32), ("alpha", C.c_float), ("tau", C.c_float), ("delta", C.c_float)]


class SpdSampleCfg(C.Structure):
    _fields_ = [("top_p", C.c_float), ("tau", C.c_float)]


def library_path() -> str:
    return os.environ.get("SPD_LIBRARY", os.path.join(HERE, "libspd.so"))


def lib():
    """The loaded C-ABI library.  Fails loudly when it has not been built."""
    global _lib
    if _lib is None:
        path = library_path()
        if not os.path.exists(path):
            raise ImportError(f"{path} is missing: build it first (python -m paper_2405_18400_amd.build)")
        L = C.CDLL(path)
        vp, i32, f32, sz = C.c_void_p, C.c_int32, C.c_float, C.c_size_t
        sig = {
            "spd_workspace_bytes": [C.POINTER(SpdModelCfg), C.POINTER(sz)],
            "spd_create": [C.POINTER(SpdModelCfg), C.POINTER(SpdWeightPtrs), vp, sz, vp, C.POINTER(vp)],
            "spd_ngram_table_bytes": [C.POINTER(SpdNgramHostTables), C.POINTER(sz)],
            "spd_load_ngrams": [vp, C.POINTER(SpdNgramHostTables), vp, sz],
            "spd_prefill": [vp, vp, i32],
            "spd_step": [vp, C.POINTER(SpdDecodeCfg), vp, vp, vp],
            "spd_nucleus_step": [vp, C.POINTER(SpdSampleCfg), C.c_float, vp, vp],
            "spd_get_nucleus_info": [vp, vp, vp, vp],
            "spd_commit": [vp, C.c_float, vp, vp, i32, vp],
            "spd_set_dense_prefill": [vp, i32],
            "spd_get_dense_prefill": [vp, C.POINTER(i32)],
            "spd_nucleus_sample": [vp, C.POINTER(SpdSampleCfg), C.c_float, vp, i32],
            "spd_generate": [vp, vp, i32, C.POINTER(SpdDecodeCfg), i32, vp, vp],
            "spd_get_state": [vp, C.POINTER(i32), vp, vp, vp],
            "spd_set_state": [vp, i32, vp, vp],
            "spd_read_logits": [vp, vp],
            "spd_get_step_info": [vp, vp, vp, vp, vp, vp],
            "spd_expand_prune": [vp, C.POINTER(SpdDecodeCfg), vp, i32],
            "spd_position": [vp, C.POINTER(i32)],
            "spd_set_graph": [vp, i32],
            "spd_set_kernel_timing": [vp, i32],
            "spd_get_phase_clock": [vp, i32, C.POINTER(C.c_int64), C.POINTER(i32), C.POINTER(i32)],
            "spd_set_fused": [vp, i32],
            "spd_get_fused": [vp, C.POINTER(i32)],
            "spd_get_kernel_timing": [vp, i32, C.POINTER(C.c_char_p), C.POINTER(f32), C.POINTER(C.c_int64), C.POINTER(i32)],
            "spd_test_state_layout": [C.POINTER(sz), C.POINTER(sz)],
            "spd_test_state_status": [vp, sz],
            "spd_test_poke_err": [vp, i32],
            "spd_op_gemv": [i32, vp, vp, f32, vp, vp, vp, i32, i32, vp],
            "spd_op_swiglu": [i32, vp, vp, vp, f32, vp, vp, i32, i32, vp],
            "spd_op_attention": [i32, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp],
            "spd_op_attention_static": [i32, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp],
        }
        for name, args in sig.items():
            fn = getattr(L, name)
            fn.argtypes, fn.restype = args, C.c_int
        L.spd_destroy.argtypes, L.spd_destroy.restype = [vp], None
        L.spd_last_error.argtypes, L.spd_last_error.restype = [vp], C.c_char_p
        L.spd_strerror.argtypes, L.spd_strerror.restype = [C.c_int], C.c_char_p
        L.spd_op_attention_scratch_bytes.argtypes, L.spd_op_attention_scratch_bytes.restype = [i32, i32, i32], sz
        _lib = L
    return _lib


def spd_strerror(code: int) -> str:
    return lib().spd_strerror(int(code)).decode()


def _np_ptr(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def model_cfg(shape, max_ctx: int, k_max: int, kv_dtype: str = "fp32") -> SpdModelCfg:
    return SpdModelCfg(shape.n_layers, shape.d_model, shape.n_heads, shape.n_kv_heads, shape.d_ffn, shape.vocab,
                       max_ctx, k_max, SPD_DTYPE[shape.dtype], shape.rms_eps, shape.rope_theta, SPD_DTYPE[kv_dtype])


def spd_workspace_bytes(cfg: SpdModelCfg) -> int:
    out = C.c_size_t(0)
    rc = lib().spd_workspace_bytes(C.byref(cfg), C.byref(out))
    if rc:
        raise SpdError(rc, "spd_workspace_bytes")
    return out.value


def ngram_struct(tables: dict, lambdas) -> tuple[SpdNgramHostTables, list]:
    """{n: (keys int32 [N, n], counts uint32 [N])} -> the C struct (+ the arrays kept alive)."""
    t, keep = SpdNgramHostTables(), []
    for o in range(SPD_N_ORDERS):
        keys, counts = tables.get(o + 2, (None, None))
        n = 0 if keys is None else len(keys)
        if n:
            keys = np.ascontiguousarray(keys, dtype=np.int32)
            counts = np.ascontiguousarray(counts, dtype=np.uint32)
            keep += [keys, counts]
            t.keys[o], t.counts[o] = keys.ctypes.data, counts.ctypes.data
        t.n_entries[o] = n
        t.lambda_[o] = float(lambdas[o])
    return t, keep


def spd_ngram_table_bytes(tables: dict, lambdas=(0, 0, 0, 0, 0)) -> int:
    t, _keep = ngram_struct(tables, lambdas)
    out = C.c_size_t(0)
    rc = lib().spd_ngram_table_bytes(C.byref(t), C.byref(out))
    if rc:
        raise SpdError(rc, "spd_ngram_table_bytes")
    return out.value


def _torch():
    import torch
    return torch


def to_device(arr, dtype: str, device="cuda"):
    """Host array -> device tensor holding the same bits (uint16 patterns become bfloat16).
    Tensors already on the device pass through."""
    torch = _torch()
    if isinstance(arr, torch.Tensor):
        assert arr.dtype == (torch.bfloat16 if dtype == "bf16" else torch.float32)
        return arr.to(device).contiguous()
    if dtype == "bf16":
        assert arr.dtype == np.uint16
        return torch.from_numpy(arr.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32)).to(device)


class Session:
    """Owns the device tensors (weights, workspace, n-gram buffer), the stream and the spd_ctx.
    Methods carry the C function names and only marshal arguments."""

    def __init__(self, shape, weights: dict, max_ctx: int, k_max: int = 8, device="cuda", stream=None, kv_dtype: str = "fp32"):
        torch = _torch()
        if not torch.cuda.is_available():
            raise RuntimeError("libspd needs a GPU: no HIP device is visible")
        self.shape, self.device, self.L = shape, device, lib()
        self.stream = stream if stream is not None else torch.cuda.Stream(device=device)
        self.cfg = model_cfg(shape, max_ctx, k_max, kv_dtype)
        dev = lambda a: to_device(a, shape.dtype, device)
        self.t = {"embed": dev(weights["embed"]), "final_norm": dev(weights["final_norm"]), "lm_head": dev(weights["lm_head"])}
        self.layers = (SpdLayerWeights * max(shape.n_layers, 1))()
        for l in range(shape.n_layers):
            p = f"layers.{l}."
            qkv = weights.get(p + "wqkv")
            if qkv is None:
                qkv = np.concatenate([weights[p + "wq"], weights[p + "wk"], weights[p + "wv"]], axis=0)
            names = {"attn_norm": weights[p + "attn_norm"], "wqkv": qkv, "wo": weights[p + "wo"],
                     "ffn_norm": weights[p + "ffn_norm"], "w_gate": weights[p + "w_gate"],
                     "w_up": weights[p + "w_up"], "w_down": weights[p + "w_down"]}
            for nm, arr in names.items():
                self.t[p + nm] = dev(arr)
                setattr(self.layers[l], nm, self.t[p + nm].data_ptr())
        self.wp = SpdWeightPtrs(self.t["embed"].data_ptr(), self.layers, self.t["final_norm"].data_ptr(),
                                self.t["lm_head"].data_ptr())
        self.workspace = torch.empty(spd_workspace_bytes(self.cfg) + 256, dtype=torch.uint8, device=device)
        ws_ptr = (self.workspace.data_ptr() + 255) // 256 * 256
        torch.cuda.synchronize()
        self.ctx = C.c_void_p()
        rc = self.L.spd_create(C.byref(self.cfg), C.byref(self.wp), ws_ptr, self.workspace.numel() - 256,
                               self.stream.cuda_stream, C.byref(self.ctx))
        if rc:
            self.ctx = None
            raise SpdError(rc, "spd_create")
        self.ngram_buf = None

    # -- error plumbing
    def _chk(self, rc, where):
        if rc:
            raise SpdError(rc, where, self.L.spd_last_error(self.ctx).decode())

    def close(self):
        if getattr(self, "ctx", None):
            self.L.spd_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the boundary, one method per C entry point
    def spd_load_ngrams(self, tables: dict, lambdas):
        torch = _torch()
        t, _keep = ngram_struct(tables, lambdas)
        need = C.c_size_t(0)
        self._chk(self.L.spd_ngram_table_bytes(C.byref(t), C.byref(need)), "spd_ngram_table_bytes")
        buf = torch.empty(need.value + 256, dtype=torch.uint8, device=self.device)
        ptr = (buf.data_ptr() + 255) // 256 * 256
        torch.cuda.synchronize()
        self._chk(self.L.spd_load_ngrams(self.ctx, C.byref(t), ptr, need.value), "spd_load_ngrams")
        self.ngram_buf = buf      # the previous buffer (if any) is released only now

    def spd_prefill(self, prefix):
        p = np.ascontiguousarray(prefix, dtype=np.int32)
        self._chk(self.L.spd_prefill(self.ctx, _np_ptr(p), len(p)), "spd_prefill")

    def spd_step(self, dc: SpdDecodeCfg, fetch: bool = True):
        if not fetch:
            self._chk(self.L.spd_step(self.ctx, C.byref(dc), None, None, None), "spd_step")
            return None
        tok, par, sc = np.zeros(dc.k, np.int32), np.zeros(dc.k, np.int32), np.zeros(dc.k, np.float32)
        self._chk(self.L.spd_step(self.ctx, C.byref(dc), _np_ptr(tok), _np_ptr(par), _np_ptr(sc)), "spd_step")
        return tok, par, sc

    def spd_commit(self, u: float):
        """-> (index of the sampled draft, its tokens since the last prefill / commit)."""
        cap = self.cfg.max_ctx
        chosen, n = C.c_int32(0), C.c_int32(0)
        toks = np.zeros(cap, np.int32)
        self._chk(self.L.spd_commit(self.ctx, float(u), C.byref(chosen), _np_ptr(toks), cap, C.byref(n)), "spd_commit")
        return chosen.value, toks[:n.value].copy()

    def spd_set_dense_prefill(self, enable: bool):
        self._chk(self.L.spd_set_dense_prefill(self.ctx, int(enable)), "spd_set_dense_prefill")

    def spd_get_dense_prefill(self) -> bool:
        out = C.c_int32(0)
        self._chk(self.L.spd_get_dense_prefill(self.ctx, C.byref(out)), "spd_get_dense_prefill")
        return bool(out.value)

    def spd_nucleus_step(self, sc: SpdSampleCfg, u: float, fetch: bool = True):
        if not fetch:
            self._chk(self.L.spd_nucleus_step(self.ctx, C.byref(sc), float(u), None, None), "spd_nucleus_step")
            return None
        tok, lp = C.c_int32(0), C.c_float(0)
        self._chk(self.L.spd_nucleus_step(self.ctx, C.byref(sc), float(u), C.byref(tok), C.byref(lp)), "spd_nucleus_step")
        return tok.value, lp.value

    def spd_nucleus_sample(self, sc: SpdSampleCfg, u: float, dev_logits, first: bool):
        assert dev_logits.is_cuda and dev_logits.dtype == _torch().float32 and dev_logits.numel() == self.shape.vocab
        self._chk(self.L.spd_nucleus_sample(self.ctx, C.byref(sc), float(u), dev_logits.data_ptr(), int(first)),
                  "spd_nucleus_sample")

    def spd_get_nucleus_info(self):
        size, mass, total = C.c_int32(0), C.c_float(0), C.c_float(0)
        self._chk(self.L.spd_get_nucleus_info(self.ctx, C.byref(size), C.byref(mass), C.byref(total)), "spd_get_nucleus_info")
        return size.value, mass.value, total.value

    def spd_generate(self, prefix, dc: SpdDecodeCfg, n_tokens: int):
        p = np.ascontiguousarray(prefix, dtype=np.int32)
        drafts, sc = np.zeros((dc.k, n_tokens), np.int32), np.zeros(dc.k, np.float32)
        self._chk(self.L.spd_generate(self.ctx, _np_ptr(p), len(p), C.byref(dc), n_tokens, _np_ptr(drafts), _np_ptr(sc)),
                  "spd_generate")
        return drafts, sc

    def spd_get_state(self):
        k = C.c_int32(0)
        tails, sc, g = np.zeros((SPD_K_MAX, SPD_TAIL), np.int32), np.zeros(SPD_K_MAX, np.float32), np.zeros(SPD_K_MAX, np.float32)
        self._chk(self.L.spd_get_state(self.ctx, C.byref(k), _np_ptr(tails), _np_ptr(sc), _np_ptr(g)), "spd_get_state")
        return tails[:k.value].copy(), sc[:k.value].copy(), g[:k.value].copy()

    def spd_set_state(self, tails, logscores):
        t = np.ascontiguousarray(tails, dtype=np.int32)
        s = np.ascontiguousarray(logscores, dtype=np.float32)
        self._chk(self.L.spd_set_state(self.ctx, len(s), _np_ptr(t), _np_ptr(s)), "spd_set_state")

    def spd_read_logits(self):
        out = np.zeros(self.shape.vocab, np.float32)
        self._chk(self.L.spd_read_logits(self.ctx, _np_ptr(out)), "spd_read_logits")
        return out

    def spd_get_step_info(self, k: int):
        ids, lp = np.zeros(k, np.int32), np.zeros(k, np.float32)
        cs, cv, cp = np.zeros((k, k), np.float32), np.zeros((k, k), np.int32), np.zeros((k, k), np.float32)
        self._chk(self.L.spd_get_step_info(self.ctx, _np_ptr(ids), _np_ptr(lp), _np_ptr(cs), _np_ptr(cv), _np_ptr(cp)),
                  "spd_get_step_info")
        return ids, lp, cs, cv, cp

    def spd_expand_prune(self, dc: SpdDecodeCfg, dev_logits, first: bool):
        assert dev_logits.is_cuda and dev_logits.dtype == _torch().float32 and dev_logits.numel() == self.shape.vocab
        self._chk(self.L.spd_expand_prune(self.ctx, C.byref(dc), dev_logits.data_ptr(), int(first)), "spd_expand_prune")

    def spd_test_poke_err(self, value: int):
        self._chk(self.L.spd_test_poke_err(self.ctx, int(value)), "spd_test_poke_err")

    def spd_position(self) -> int:
        out = C.c_int32(0)
        self._chk(self.L.spd_position(self.ctx, C.byref(out)), "spd_position")
        return out.value

    def spd_set_graph(self, enable: bool):
        self._chk(self.L.spd_set_graph(self.ctx, int(enable)), "spd_set_graph")

    def spd_set_fused(self, enable: bool):
        self._chk(self.L.spd_set_fused(self.ctx, int(enable)), "spd_set_fused")

    def spd_get_fused(self) -> bool:
        out = C.c_int32(0)
        self._chk(self.L.spd_get_fused(self.ctx, C.byref(out)), "spd_get_fused")
        return bool(out.value)

    def spd_set_kernel_timing(self, enable: bool):
        self._chk(self.L.spd_set_kernel_timing(self.ctx, int(enable)), "spd_set_kernel_timing")

    def spd_get_kernel_timing(self) -> dict:
        cap = 32
        names, ms, cnt, n = (C.c_char_p * cap)(), (C.c_float * cap)(), (C.c_int64 * cap)(), C.c_int32(0)
        self._chk(self.L.spd_get_kernel_timing(self.ctx, cap, names, ms, cnt, C.byref(n)), "spd_get_kernel_timing")
        return {names[i].decode(): (ms[i], cnt[i]) for i in range(n.value)}

    def spd_get_phase_clock(self):
        """Clock stamps [blocks, 2 (5 n_layers + 2)] of the most recent fused forward."""
        cap = 2 * (5 * self.shape.n_layers + 2) * 2048
        out, n, nb = np.zeros(cap, dtype=np.int64), C.c_int32(0), C.c_int32(0)
        self._chk(self.L.spd_get_phase_clock(self.ctx, cap, out.ctypes.data_as(C.POINTER(C.c_int64)), C.byref(n),
                                             C.byref(nb)), "spd_get_phase_clock")
        return out[:n.value * nb.value].reshape(nb.value, n.value).copy()

    def synchronize(self):
        self.stream.synchronize()


# ---- stand-alone operators (device tensors in, device tensors out; caller's current stream)
def _stream_ptr():
    return _torch().cuda.current_stream().cuda_stream


def spd_op_gemv(dtype: str, W, x, y, gain=None, eps=0.0, residual=None):
    rows, cols = W.shape
    rc = lib().spd_op_gemv(SPD_DTYPE[dtype], W.data_ptr(), gain.data_ptr() if gain is not None else None, eps,
                           x.data_ptr(), residual.data_ptr() if residual is not None else None, y.data_ptr(),
                           rows, cols, _stream_ptr())
    if rc:
        raise SpdError(rc, "spd_op_gemv")


def spd_op_swiglu(dtype: str, Wg, Wu, x, u, gain=None, eps=0.0):
    rows, cols = Wg.shape
    rc = lib().spd_op_swiglu(SPD_DTYPE[dtype], Wg.data_ptr(), Wu.data_ptr(), gain.data_ptr() if gain is not None else None,
                             eps, x.data_ptr(), u.data_ptr(), rows, cols, _stream_ptr())
    if rc:
        raise SpdError(rc, "spd_op_swiglu")


def spd_op_attention(dtype: str, q, K, V, out, n_ctx: int):
    torch = _torch()
    n_heads, d_head = q.shape
    n_kv, cap_ctx, _ = K.shape
    scratch = torch.empty(lib().spd_op_attention_scratch_bytes(n_heads, d_head, cap_ctx) + 256, dtype=torch.uint8, device=q.device)
    ptr = (scratch.data_ptr() + 255) // 256 * 256
    rc = lib().spd_op_attention(SPD_DTYPE[dtype], q.data_ptr(), K.data_ptr(), V.data_ptr(), out.data_ptr(), ptr,
                                n_heads, n_kv, d_head, n_ctx, cap_ctx, _stream_ptr())
    if rc:
        raise SpdError(rc, "spd_op_attention")
    torch.cuda.current_stream().synchronize()   # scratch must outlive the kernel


def spd_op_attention_static(dtype: str, q, K, V, out, n_ctx: int):
    """The same on the library's static scratch: no allocation here or in the library."""
    n_heads, d_head = q.shape
    n_kv, cap_ctx, _ = K.shape
    rc = lib().spd_op_attention_static(SPD_DTYPE[dtype], q.data_ptr(), K.data_ptr(), V.data_ptr(), out.data_ptr(),
                                       n_heads, n_kv, d_head, n_ctx, cap_ctx, _stream_ptr())
    if rc:
        raise SpdError(rc, "spd_op_attention_static")


def spd_test_state_layout():
    words, err_word = C.c_size_t(0), C.c_size_t(0)
    rc = lib().spd_test_state_layout(C.byref(words), C.byref(err_word))
    if rc:
        raise SpdError(rc, "spd_test_state_layout")
    return words.value, err_word.value


def spd_test_state_status(state_words) -> int:
    a = np.ascontiguousarray(state_words, dtype=np.int32)
    return lib().spd_test_state_status(_np_ptr(a), a.size)
