"""CPU-side checks of the C ABI: the library loads, exports every entry point declared in
include/esp.h, and rejects bad arguments on the host before any GPU work (no compute call
here needs a GPU)."""
import ctypes as C
import os
import re

import pytest

from util import ROOT

from paper_2603_17942_amd import binding as B
from paper_2603_17942_amd import synth


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2603_17942_amd import build
        build.build(verbose=False)
    return B.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "esp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(esp_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_entry_point_is_exported(lib):
    names = declared_functions()
    assert {"esp_tree_forward", "esp_mask_topk", "esp_build_prune_tree", "esp_verify_accept"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.EXPORTS) == names          # the binding wraps exactly what the header declares


def test_status_strings(lib):
    assert lib.esp_status_str(0) == b"ok"
    assert lib.esp_status_str(3) == b"capacity exceeded"


def test_workspace_bytes_and_model_validation(lib):
    d = B.model_desc(synth.SHAPES["llama3_8b"])
    n = lib.esp_workspace_bytes(C.byref(d), 1, 320, 4096)
    assert n > 100 << 20
    assert lib.esp_workspace_bytes(C.byref(d), 0, 320, 4096) == 0
    assert lib.esp_workspace_bytes(C.byref(d), 1, B.MAX_ROWS_PER_SEQ + 1, 4096) == 0
    bad = B.model_desc(synth.SHAPES["llama3_8b"].replace(head_dim=96))
    assert lib.esp_workspace_bytes(C.byref(bad), 1, 64, 4096) == 0
    odd = B.model_desc(synth.SHAPES["llama3_8b"].replace(d_ff=14336 + 32))    # bf16 needs K % 64 == 0
    assert lib.esp_workspace_bytes(C.byref(odd), 1, 64, 4096) == 0
    tiny = B.model_desc(synth.SHAPES["tiny"])                                   # fp32: 688 is fine
    assert lib.esp_workspace_bytes(C.byref(tiny), 1, 64, 512) > 0


def test_create_rejects_bad_arguments_without_touching_the_gpu(lib):
    d = B.model_desc(synth.SHAPES["tiny"])
    ctx = C.c_void_p()
    w = B.Weights()
    assert lib.esp_create(C.byref(d), None, 1, 64, 512, 4096, 1 << 20, None, C.byref(ctx)) == 1      # EINVAL
    assert lib.esp_create(C.byref(d), C.byref(w), 1, 64, 512, None, 1 << 20, None, C.byref(ctx)) == 1
    assert lib.esp_create(C.byref(d), C.byref(w), 1, 64, 512, 4096, 1 << 20, None, None) == 1
    assert lib.esp_create(C.byref(d), C.byref(w), 1, 64, 512, 4096, 1 << 20, None, C.byref(ctx)) == 1  # null weights
    assert lib.esp_create(C.byref(d), C.byref(w), 1, 5000, 512, 4096, 1 << 20, None, C.byref(ctx)) == 3  # ECAPACITY
    bad = B.model_desc(synth.SHAPES["tiny"].replace(n_q_heads=3))
    assert lib.esp_create(C.byref(bad), C.byref(w), 1, 64, 512, 4096, 1 << 20, None, C.byref(ctx)) == 2   # ESHAPE
    bad = B.model_desc(synth.SHAPES["tiny"])
    bad.dtype = 7
    assert lib.esp_create(C.byref(bad), C.byref(w), 1, 64, 512, 4096, 1 << 20, None, C.byref(ctx)) == 4   # EDTYPE
    assert ctx.value is None
    assert lib.esp_destroy(None) == 1


def test_null_context_and_stage_calls_validate(lib):
    blk, kv = B.Block(), B.Kv()
    assert lib.esp_tree_forward(None, C.byref(blk), None, C.byref(kv), None, None, None) == 1
    assert lib.esp_verify_accept(None, C.byref(blk), None, C.byref(kv), None, None, None, None) == 1
    assert lib.esp_mask_topk(None, C.byref(blk), None, None, None, 4, None, None, None, None) == 1
    assert lib.esp_build_prune_tree(None, None, None, None, 4, None, None, None, C.byref(blk)) == 1
    assert lib.esp_block_from_tree(None, C.byref(blk)) == 1
    assert lib.esp_profile_enable(None, 1) == 1
    assert lib.esp_mask_mean(None, 4096, 4, 2, 4096) == 1
    assert lib.esp_mask_last_k(None, 4096, 4, 2, 4096) == 1
    assert lib.esp_mask_gaussian(None, None, 0.0, 2, 4096) == 1
    # stage entry points: shapes and sizes are checked before anything is launched
    p = 4096
    assert lib.esp_gemm(None, B.ESP_BF16, p, p, 0, p, 4, 48, 64, p, 1 << 20) == 2      # N % 32
    assert lib.esp_gemm(None, B.ESP_BF16, p, p, 0, p, 4, 64, 96, p, 1 << 20) == 2      # K % 64
    assert lib.esp_gemm(None, B.ESP_F32, p, p, 1, p, 4, 64, 64, p, 1 << 20) == 4       # packed needs bf16
    assert lib.esp_gemm(None, 5, p, p, 0, p, 4, 64, 64, p, 1 << 20) == 4
    assert lib.esp_gemm(None, B.ESP_BF16, None, p, 0, p, 4, 64, 64, p, 1 << 20) == 1
    assert lib.esp_gemm(None, B.ESP_BF16, p, p, 0, p, 68, 4096, 4096, p, 16) == 3      # split-K scratch too small
    assert lib.esp_pack_weight(None, p, 2 * p, 48, 64) == 2
    assert lib.esp_pack_weight(None, p, p, 64, 64) == 1                                # must not alias
    assert lib.esp_softmax_topk(None, p, 4, 1000, 0, p, p, p, 1 << 20) == 1
    assert lib.esp_softmax_topk(None, p, 4, 1000, B.MAX_TOPK + 1, p, p, p, 1 << 20) == 1
    assert lib.esp_softmax_topk(None, p, 4, 8, 9, p, p, p, 1 << 20) == 1               # Kp > vocab
    assert lib.esp_softmax_topk(None, p, 4, 128256, 8, p, p, p, 16) == 3
    assert lib.esp_softmax_topk_scratch_bytes(4, 128256, 10) > 0
    assert lib.esp_gemm_scratch_bytes(68, 4096, 4096) >= 8 * 68 * 4096 * 4


def test_engine_refuses_to_run_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    shape = synth.SHAPES["tiny"]
    with pytest.raises(RuntimeError):
        B.Engine(shape, {"layers": []}, 1, 64, 512)


def test_static_topk_rejects_on_the_host(lib):
    """esp_softmax_topk_static validates before any HIP call: null pointers, bad Kp, and sizes
    beyond its fixed device array (128 rows at the largest vocabulary and Kp)."""
    one = C.c_void_p(256)      # never dereferenced: every case below is rejected first
    f = lib.esp_softmax_topk_static
    assert f(None, None, 4, 4096, 4, one, one) == 1
    assert f(None, one, 4, 4096, 4, None, one) == 1
    assert f(None, one, 0, 4096, 4, one, one) == 1
    assert f(None, one, 4, 4096, 0, one, one) == 1
    assert f(None, one, 4, 4096, B.MAX_TOPK + 1, one, one) == 1
    assert f(None, one, 4, 3, 4, one, one) == 1                       # Kp > vocab
    assert f(None, one, 132, 128256, 32, one, one) == 3               # ESP_ECAPACITY
    assert f(None, one, 100000, 128256, 1, one, one) == 3
