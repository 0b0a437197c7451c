"""CPU-side checks of the C-ABI library: it loads, exports every symbol that
include/aed.h declares, and rejects bad configurations on the host (no GPU
work is launched here)."""
import ctypes as C
import os
import re

import pytest

from paper_2503_05931_amd import binding, workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2503_05931_amd import build
        build.build()
    return binding.load()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "aed.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(aed_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert len(names) >= 13
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/aed.h but not exported"
    assert sorted(binding.EXPORTS) == names


def good_config():
    return binding.make_config(W.config("canary24_b64"), max_batch=64, max_total_enc_frames=64 * 500, max_dec_len=132)


def test_workspace_bytes_counts_the_caches(lib):
    c = good_config()
    n = binding.aed_workspace_bytes(c)
    L, d, e = 24, 1024, 2
    cross = 2 * L * 64 * 500 * d * e
    self_kv = 2 * L * 64 * 9 * 16 * d * e            # ceil(132/16) = 9 pages per sequence
    weights = (L * 16 * d * d + 4096 * d) * e         # the library's re-ordered copy of every matrix
    enc_copy = 64 * 500 * d * e                       # the batch's encoder frames in fragment order
    assert cross + self_kv + weights + enc_copy < n < cross + self_kv + weights + enc_copy + (64 << 20)
    # 8-bit caches: one byte per cached key / value element, everything else unchanged
    c.kv_fp8 = 1
    n8 = binding.aed_workspace_bytes(c)
    assert abs((n - n8) - (cross + self_kv) // 2) < (1 << 20)


@pytest.mark.parametrize("field,value,status", [
    ("struct_size", 4, binding.AED_EINVAL),
    ("n_layers", 0, binding.AED_EINVAL),
    ("n_heads", 7, binding.AED_EINVAL),
    ("dtype", 3, binding.AED_EINVAL),
    ("max_batch", 0, binding.AED_EINVAL),
    ("eos_id", 4096, binding.AED_EINVAL),
    ("kv_pages", -1, binding.AED_EINVAL),
    ("kv_fp8", 2, binding.AED_EINVAL),
    ("prefill_rows", -1, binding.AED_EINVAL),
    ("norm_type", 2, binding.AED_EINVAL),
    ("page_size", 32, binding.AED_EUNSUPPORTED),
    ("d_ffn", 1000, binding.AED_EUNSUPPORTED),
    ("vocab", 1000, binding.AED_EUNSUPPORTED),
])
def test_bad_configs_are_rejected(lib, field, value, status):
    c = good_config()
    setattr(c, field, value)
    with pytest.raises(binding.AedError) as ei:
        binding.aed_workspace_bytes(c)
    assert ei.value.status == status
    assert len(str(ei.value)) > 10


def test_fp8_caches_need_bfloat16(lib):
    c = good_config()
    c.dtype, c.kv_fp8 = 0, 1
    with pytest.raises(binding.AedError) as ei:
        binding.aed_workspace_bytes(c)
    assert ei.value.status == binding.AED_EUNSUPPORTED


def test_bench_refuses_more_than_one_gpu():
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_unsupported_head_dim(lib):
    c = good_config()
    c.n_heads, c.head_dim = 32, 32
    with pytest.raises(binding.AedError) as ei:
        binding.aed_workspace_bytes(c)
    assert ei.value.status == binding.AED_EUNSUPPORTED


def test_create_rejects_bad_arguments_before_touching_the_device(lib):
    c = good_config()
    handle = C.c_void_p(None)
    w = binding.AedWeights()
    st = lib.aed_decoder_create(C.byref(c), C.byref(w), C.c_void_p(256), 1 << 40, None, C.byref(handle))
    assert st == binding.AED_EINVAL and not handle.value      # NULL weight pointers
    assert b"NULL" in lib.aed_last_error(None)
    st = lib.aed_decoder_create(C.byref(c), None, C.c_void_p(256), 1 << 40, None, C.byref(handle))
    assert st == binding.AED_EINVAL
    st = lib.aed_decoder_create(C.byref(c), C.byref(w), None, 0, None, None)
    assert st == binding.AED_EINVAL


def test_null_handles(lib):
    assert lib.aed_decoder_destroy(None) == binding.AED_OK
    assert lib.aed_decode_step(None, None, None, None) == binding.AED_EINVAL
    assert lib.aed_greedy_decode(None, None, 1, 1, None, None, None) == binding.AED_EINVAL
    assert lib.aed_cross_kv_precompute(None, None, None, 1) == binding.AED_EINVAL


def test_param_count_matches_paper(lib):
    # removing 20 of 24 decoder layers removes 1016M - 680M = 336M parameters
    # (Sec. "Transferring model capacity from decoder to encoder")
    c = good_config()
    c.n_layers = 20
    assert abs(binding.aed_layer_matrix_params(c) - 336e6) / 336e6 < 0.005


def test_workloads_follow_the_recipe():
    wl = W.make("canary24_b64")
    assert wl.enc_lens.min() >= 12 and wl.enc_lens.max() <= 500 and len(wl.enc_lens) == 64
    assert wl.enc.shape == (int(wl.enc_lens.sum()), 1024)
    assert (W.bf16_round(wl.enc) == wl.enc).all() and (W.bf16_round(wl.weights["w_out"]) == wl.weights["w_out"]).all()
    assert wl.prompt.shape == (64, 4) and wl.prompt.min() >= 3 and wl.prompt.max() < 4096
    # bf16 rounding is round-to-nearest-even
    import numpy as np
    x = np.array([1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -7], np.float32)
    assert (W.bf16_round(x) == np.array([1.0, 1.0 + 2 ** -6, 1.0 + 2 ** -7], np.float32)).all()
    r = W.make("ragged24_b128", with_enc=False)
    a = W.random_batches(r.extra["pool_enc"], r.extra["pool_dec"], r.extra["perm"], 128)
    b = W.bucketed_2d_batches(r.extra["pool_enc"], r.extra["pool_dec"], 128)
    assert len(a) == 16 and len(b) == 16
    pe, pd = r.extra["pool_enc"], r.extra["pool_dec"]
    pad_a = W.padding_fraction([pe[i] for i in a]), W.padding_fraction([pd[i] for i in a])
    pad_b = W.padding_fraction([pe[i] for i in b]), W.padding_fraction([pd[i] for i in b])
    # bucketing removes most encoder-axis padding and less of the output-axis padding
    # (the direction the paper reports: 57%/59% -> 4.5%/19%)
    assert pad_a[0] > 0.4 and pad_a[1] > 0.4 and pad_b[0] < 0.15 and pad_b[0] < pad_b[1] < pad_a[1]
