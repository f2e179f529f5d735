"""The C-ABI library loads and exports every symbol include/sd.h declares, and its
argument checks fail cleanly without touching a GPU (CPU only)."""
import ctypes as C
import os
import re

import pytest

from paper_2505_08600_amd import api

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    txt = open(os.path.join(ROOT, "include", "sd.h")).read()
    txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
    return sorted(set(re.findall(r"\b(sd_[a-z_0-9]+)\s*\(", txt)))


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert "sd_load_model" in names and "sd_draft" in names and "sd_verify" in names and "sd_route" in names
    L = C.CDLL(api.LIB_PATH)
    for n in names:
        assert hasattr(L, n), n
    assert sorted(api.EXPORTS) == names


def test_argument_errors_do_not_need_a_gpu():
    L = api.lib()
    assert L.sd_set_option(b"no_such_option", 1) == api.SD_EINVAL
    assert b"unknown option" in L.sd_last_error()
    assert L.sd_set_option(None, 1) == api.SD_EINVAL
    assert L.sd_load_model(None, None, None) == api.SD_EINVAL
    cfg = api._Config(2, 64, 4, 16, 96, 50, 0, 10000.0, 1e-5, 16, 64)
    w = api._Weights()
    h = C.c_void_p()
    assert L.sd_load_model(C.byref(cfg), C.byref(w), C.byref(h)) == api.SD_EINVAL  # vocab % 4, null weights
    cfg.n_heads = 3
    assert L.sd_load_model(C.byref(cfg), C.byref(w), C.byref(h)) == api.SD_EINVAL
    assert b"n_heads" in L.sd_last_error()
    big = api._Config(2, 64, 4, 16, 96, 262148, 0, 10000.0, 1e-5, 16, 64)   # the samplers' segment table ends at 262144
    assert L.sd_load_model(C.byref(big), C.byref(w), C.byref(h)) == api.SD_EINVAL
    assert b"vocab above 262144" in L.sd_last_error()
    assert L.sd_set_option(b"stream_read_nt", 4) == api.SD_EINVAL
    assert L.sd_set_option(b"norm_fold", 3) == api.SD_EINVAL and L.sd_set_option(b"norm_fold", 0) == api.SD_OK
    assert L.sd_set_option(b"rope_group", 2) == api.SD_EINVAL and L.sd_set_option(b"rope_group", 1) == api.SD_OK
    assert L.sd_set_option(b"prefill_attn", 2) == api.SD_EINVAL and L.sd_set_option(b"prefill_attn", 1) == api.SD_OK
    assert L.sd_set_option(b"gemm_tile_cols", 64) == api.SD_EINVAL and L.sd_set_option(b"gemm_tile_cols", 128) == api.SD_OK
    assert L.sd_set_option(b"gemm_tile_cols", 0) == api.SD_OK
    assert L.sd_set_option(b"no_such_option", 1) == api.SD_EINVAL
    assert L.sd_ctx_create(0, None, None) == api.SD_EINVAL
    assert L.sd_draft(None, None, None, 1, 4, 1.0, None, None, None, None) == api.SD_EINVAL
    assert L.sd_verify(None, None, None, 1, 4, 1.0, None, None, None, None, None, 1, None) == api.SD_EINVAL
    assert L.sd_commit(None, None, 1, 4, None, None, None, None) == api.SD_EINVAL
    assert L.sd_route(None, None, 4, 256, None, 1, None, None) == api.SD_EINVAL
    assert L.sd_prefill(None, None, None, 1, 1, None) == api.SD_EINVAL
    assert L.sd_model_set_lora(None, None) == api.SD_EINVAL
    assert L.sd_ctx_set_adapters(None, None, None) == api.SD_EINVAL
    assert L.sd_free_model(None) == api.SD_OK and L.sd_ctx_free(None) == api.SD_OK
    assert L.sd_classifier_create(None, None, None) == api.SD_EINVAL
    assert L.sd_route_classifier(None, None, None, 1, 1, None, None, None) == api.SD_EINVAL
    L.sd_classifier_destroy(None)
    shape = api._ClsShape(100, 32, 96, 8, 4, 4, 3)              # d_inner not a multiple of 64
    cw, ch = api._ClsWeights(), C.c_void_p(1)
    assert L.sd_classifier_create(C.byref(shape), C.byref(cw), C.byref(ch)) == api.SD_EINVAL and not ch.value
    assert b"d_inner" in L.sd_last_error()
    shape.d_inner = 128
    assert L.sd_classifier_create(C.byref(shape), C.byref(cw), C.byref(ch)) == api.SD_EINVAL  # null weights
    assert b"null weight" in L.sd_last_error()


def test_product_package_does_not_import_the_oracle():
    """The HIP path must not route through the CPU oracle."""
    import glob
    pk = os.path.join(ROOT, "paper_2505_08600_amd")
    for f in glob.glob(os.path.join(pk, "**", "*"), recursive=True):
        if f.endswith((".py", ".hip", ".h", ".cpp")):
            src = open(f).read()
            assert "oracle" not in src.lower() or f.endswith("datagen.py"), f


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: asking bench.py for more exits with a message instead of running."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2 and "one GPU only" in r.stderr and r.stdout.strip() == ""
