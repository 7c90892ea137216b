"""Host-only checks of the C-ABI boundary: the library loads, exports what the header
declares, and rejects bad arguments without touching a GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def pkg():
    import paper_2405_18400_amd as P
    if not os.path.exists(P.library_path()):
        from paper_2405_18400_amd.build import build_library
        build_library()
    return P


def declared_functions():
    text = open(os.path.join(ROOT, "include", "spd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spd_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(pkg):
    L = pkg.lib()
    names = declared_functions()
    assert len(names) >= 20 and "spd_create" in names and "spd_step" in names and "spd_generate" in names
    for n in names:
        assert hasattr(L, n), f"{n} declared in spd.h but not exported by libspd.so"


def test_workspace_bytes_and_config_validation(pkg):
    cfg = pkg.binding.model_cfg(synth.LLAMA7B, 128, 8)
    need = pkg.spd_workspace_bytes(cfg)
    kv = 2 * 32 * 32 * 128 * 128 * 4                      # K and V, 32 layers, 32 heads, 128 positions, d_head 128, fp32
    # arena of the dense prefix pass, 1024 token rows: residual stream twice and queries in fp32,
    # the (hi, lo) bf16 pairs of the normalised input and of the SwiGLU output, the rotary table
    arena = 1024 * (3 * 4096 * 4 + 2 * 4096 * 2 + 2 * 11008 * 2 + 64 * 8)
    # partial tiles of the split-k products: two per 32-row tile of the widest product (QKV, 12288 rows), gate + up
    arena += (12288 // 32) * 2 * 2 * 16 * 64 * 4
    # the rest: two arenas of per-layer activation vectors (3.6 MB each), logits, history, counters
    assert kv + arena <= need < kv + arena + 12 * 2 ** 20
    for field, bad in [("dtype", 7), ("n_heads", 3), ("n_kv_heads", 5), ("k_max", 17), ("k_max", 0), ("max_ctx", 1),
                       ("vocab", 31999), ("d_ffn", 11004), ("d_model", 0)]:
        c = pkg.binding.model_cfg(synth.LLAMA7B, 128, 8)
        setattr(c, field, bad)
        with pytest.raises(pkg.SpdError) as e:
            pkg.spd_workspace_bytes(c)
        assert e.value.code == -1
    for shape in (synth.TINY, synth.LLAMA13B, synth.LLAMA70B):
        assert pkg.spd_workspace_bytes(pkg.binding.model_cfg(shape, 1100, 8)) > 0
    # an fp16 cache: half the cache bytes, bf16 models only, nothing but fp32 / fp16 is a cache type
    assert pkg.spd_workspace_bytes(pkg.binding.model_cfg(synth.LLAMA7B, 128, 8, "fp16")) == need - kv // 2
    for shape, kv_dtype in [(synth.TINY, "fp16"), (synth.LLAMA7B, "bf16")]:
        with pytest.raises(pkg.SpdError) as e:
            pkg.spd_workspace_bytes(pkg.binding.model_cfg(shape, 128, 8, kv_dtype))
        assert e.value.code == -1


def test_create_rejects_null_arguments_before_any_gpu_work(pkg):
    L = pkg.lib()
    cfg = pkg.binding.model_cfg(synth.TINY, 64, 8)
    out = C.c_void_p()
    assert L.spd_create(C.byref(cfg), None, None, 0, None, C.byref(out)) == -1 and not out.value
    assert L.spd_create(None, None, None, 0, None, C.byref(out)) == -1
    assert L.spd_create(C.byref(cfg), None, None, 0, None, None) == -1
    for fn in ("spd_prefill",):
        assert getattr(L, fn)(None, None, 0) == -1
    assert L.spd_step(None, None, None, None, None) == -1
    assert L.spd_position(None, None) == -1
    assert pkg.spd_strerror(0) == "ok" and "max_ctx" in pkg.spd_strerror(-3)


def test_ngram_table_bytes(pkg):
    t = synth.make_ngram_tables_uniform(100, {2: 300, 3: 200}, seed=0)
    need = pkg.spd_ngram_table_bytes(t)
    assert need >= 2 * 500 * 32 and need % 256 == 0     # an entry plus a context total each, 32-byte slots
    assert pkg.spd_ngram_table_bytes({}) > 0


def test_missing_library_fails_loudly(pkg, monkeypatch):
    import paper_2405_18400_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "library_path", lambda: "/nonexistent/libspd.so")
    with pytest.raises(ImportError):
        b.lib()


def test_bench_refuses_more_than_one_gpu():
    """The benchmark measures one GPU's throughput; asked for more it must say so and exit."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr and res.stdout.strip() == ""


def test_entry_points_exist():
    import importlib
    ge = importlib.import_module("__graft_entry__")
    assert callable(ge.build) and callable(ge.smoke)


def test_device_error_word_maps_to_ehip(pkg):
    """A bounded wait of the persistent kernel that gives up leaves an error word in the
    device-side draft state; the one function every entry point passes its host copy of that
    state through turns it into SPD_EHIP.  Host only: the state is filled by hand here."""
    words, err_word = pkg.spd_test_state_layout()
    assert words > 100 and 0 <= err_word < 8
    state = np.zeros(words, np.int32)
    assert pkg.spd_test_state_status(state) == 0
    state[:] = np.arange(words) % 7                   # whatever the other fields hold ...
    state[err_word] = 0
    assert pkg.spd_test_state_status(state) == 0      # ... only the error word decides
    for bad in (1, -1, 12345):
        state[err_word] = bad
        assert pkg.spd_test_state_status(state) == -6
        assert "HIP" in pkg.spd_strerror(-6)
    assert pkg.spd_test_state_status(state[: words - 1]) == -1    # too short a copy is refused
    assert pkg.lib().spd_test_state_status(None, words) == -1


def test_static_scratch_variant_refuses_oversized_shapes_before_any_gpu_work(pkg):
    """spd_op_attention_static: argument errors and a scratch need beyond the static array are
    refused on the host (no GPU is touched: this runs without one)."""
    L = pkg.lib()
    dummy = C.c_void_p(256)
    need = L.spd_op_attention_scratch_bytes(64, 128, 8192)
    assert need <= 4 << 20
    assert L.spd_op_attention_scratch_bytes(64, 128, 32768) > 4 << 20
    assert L.spd_op_attention_static(1, dummy, dummy, dummy, dummy, 64, 8, 128, 100, 32768, None) == -4
    assert L.spd_op_attention_static(1, None, dummy, dummy, dummy, 8, 8, 128, 10, 64, None) == -1
    assert L.spd_op_attention_static(1, dummy, dummy, dummy, dummy, 8, 3, 128, 10, 64, None) == -1
    assert L.spd_op_attention_static(1, dummy, dummy, dummy, dummy, 8, 8, 128, 65, 64, None) == -1
    assert L.spd_op_attention_static(5, dummy, dummy, dummy, dummy, 8, 8, 128, 10, 64, None) == -1
