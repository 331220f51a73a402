"""The C-ABI library without a GPU: it loads, exports every function that
include/gram.h declares, and its host-side argument logic behaves (no kernel is
launched here)."""
import ctypes as C
import os
import re

import pytest

from paper_2204_04179_amd import gram

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "gram.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gram_[a-z0-9_]+)\s*\(", text)))


def test_header_functions_are_exported_and_bound():
    names = declared_functions()
    assert {"gram_unique", "gram_encode_gather", "gram_grad_accumulate", "gram_encoder_wgrad",
            "gram_flush", "gram_create", "gram_destroy"} <= set(names)
    lib = gram.load()
    for name in names:
        assert hasattr(lib, name), f"{name} declared in gram.h but not exported by libgram.so"
    assert set(gram.EXPORTS) == set(names)


def test_library_is_built_in_tree():
    assert os.path.dirname(gram.LIB_PATH) == os.path.join(ROOT, "paper_2204_04179_amd")
    assert os.path.exists(gram.LIB_PATH)


def test_workspace_query_validates_the_config():
    ok = gram.make_config(13000, 768, 256, 6400, 1, 0, 0, gram.BF16)
    n = gram.workspace_bytes(ok)
    assert n > 6400 * 256 * 4          # at least the persistent buffer
    bigger = gram.make_config(13000, 768, 256, 6400, 4, 0, 0, gram.BF16)
    assert gram.workspace_bytes(bigger) > n
    bad = [
        gram.make_config(0, 768, 256, 6400),                 # empty vocabulary
        gram.make_config(13000, 770, 256, 6400),             # bf16 d_in not a multiple of 8
        gram.make_config(13000, 768, 254, 6400),             # d not a multiple of 4
        gram.make_config(13000, 768, 256, 0),                # no positions
        gram.make_config(13000, 768, 256, 6400, 0),          # K < 1
        gram.make_config(13000, 768, 256, 6400, 1, 13000),   # pad_id outside the vocabulary
        gram.make_config(13000, 768, 256, 6400, 1, 0, -5),   # negative capacity
        gram.make_config(13000, 768, 256, 6400, 1, 0, 0, 7), # unknown dtype
    ]
    for cfg in bad:
        assert gram.workspace_bytes(cfg) == 0
    # float32 features need no multiple-of-8 width
    assert gram.workspace_bytes(gram.make_config(100, 30, 32, 64, 1, 0, 0, gram.F32)) > 0


def test_workspace_query_for_the_dense_buffer_and_the_two_layer_encoder():
    base = gram.make_config(20000, 768, 256, 51200, 8, 0, 0, gram.BF16)
    dense = gram.make_config(20000, 768, 256, 51200, 8, 0, 0, gram.BF16, 1)
    assert 0 < gram.workspace_bytes(dense) < gram.workspace_bytes(base)      # no slot map, no transposed copies
    assert gram.workspace_bytes(gram.make_config(20000, 768, 256, 51200, 8, 0, 20000, gram.BF16, 1)) > 0
    mlp = gram.make_config(20000, 768, 256, 51200, 8, 0, 0, gram.BF16, 0, 512)
    assert gram.workspace_bytes(mlp) > gram.workspace_bytes(base)
    bad = [
        gram.make_config(20000, 768, 256, 51200, 8, 0, 500, gram.BF16, 1),       # dense: one row per ID, no other size
        gram.make_config(20000, 768, 256, 51200, 8, 0, 0, gram.BF16, 2),         # unknown layout
        gram.make_config(20000, 768, 256, 51200, 8, 0, 0, gram.BF16, 0, -8),     # negative hidden width
        gram.make_config(20000, 768, 256, 51200, 8, 0, 0, gram.BF16, 0, 100),    # hidden width not a multiple of 8
        gram.make_config(20000, 768, 252, 51200, 8, 0, 0, gram.BF16, 0, 512),    # two-layer: d not a multiple of 8
        gram.make_config(20000, 768, 256, 51200, 8, 0, 0, gram.F32, 0, 512),     # two-layer: bf16 only
    ]
    for cfg in bad:
        assert gram.workspace_bytes(cfg) == 0
    # matrices beyond the 4 GiB of a buffer descriptor are served by wide-address kernel variants
    assert gram.workspace_bytes(gram.make_config(1 << 22, 768, 256, 51200, 8, 0, 0, gram.BF16, 1)) > (1 << 32)
    assert gram.workspace_bytes(gram.make_config(1 << 21, 64, 1024, 51200, 8, 0, 0, gram.BF16, 1)) > (1 << 33)
    lib = gram.load()
    assert lib.gram_mlp_batch_bytes(None, 100) == 0
    assert lib.gram_flush64(None, None, None, None, None, None, None) == gram.ERR_ARG
    assert lib.gram_window_import(None, None, None, None, 0, None) == gram.ERR_ARG
    assert lib.gram_pseudo_loss_grad(None, None, None, None, None, 0, None, None, 0, None, None) == gram.ERR_ARG
    assert lib.gram_mlp_backward(None, None, None, None, None, None, None, 0, None, None, None, 0, None, None) == gram.ERR_ARG


def test_kernel_names_and_null_context_errors():
    lib = gram.load()
    n = lib.gram_kernel_count()
    names = [lib.gram_kernel_name(k).decode() for k in range(n)]
    assert n == len(set(names)) and "seg_reduce" in names and "unique_small" in names
    assert lib.gram_kernel_name(n) == b""
    # calls on a NULL context are argument errors, not crashes
    assert lib.gram_check(None, None) == gram.ERR_ARG
    assert lib.gram_grad_accumulate(None, None, 0, 0, None) == gram.ERR_ARG
    assert lib.gram_destroy(None) == gram.OK
    out = C.c_void_p(123)
    assert lib.gram_create(C.byref(out), None) == gram.ERR_ARG and not out.value
    assert b"cfg is NULL" in lib.gram_last_error(None)
