"""The C-ABI boundary without a GPU: the library loads, exports what include/dapq.h declares,
and rejects bad arguments on the host before anything is enqueued."""
import ctypes as C
import os
import re

import pytest

import paper_2603_11564_amd as D
from paper_2603_11564_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ERR_INVALID, ERR_UNSUPPORTED, ERR_WORKSPACE = -1, -2, -3


@pytest.fixture(scope="module")
def lib():
    return D.load_library()


def good_shape(**kw):
    args = dict(n_layers=2, batch=1, n_q_heads=32, n_kv_heads=8, n_pseudo=64, total_tokens=4096,
                k_strides=(4096 * 8 * 128, 0, 128, 8 * 128), v_strides=(4096 * 8 * 128, 0, 128, 8 * 128),
                q_strides=(32 * 64 * 128, 32 * 64 * 128, 64 * 128, 128))
    args.update(kw)
    return D.make_shape(**args)


def test_header_and_library_agree(lib):
    header = open(os.path.join(ROOT, "include", "dapq.h")).read()
    declared = set(re.findall(r"\b(dapq_[a-z0-9_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    # the struct mirror has the layout the header describes (6 int32, int64, pointer, 12 int64, float)
    assert C.sizeof(binding.Shape) == 6 * 4 + 8 + 8 + 12 * 8 + 8


def test_workspace_bytes_is_a_function_of_the_shape(lib):
    a = D.workspace_bytes(good_shape())
    assert a > 0 and a % 256 == 0 and a == D.workspace_bytes(good_shape())
    assert D.workspace_bytes(good_shape(n_layers=4)) > a
    assert D.workspace_bytes(good_shape(head_dim=64)) == 0
    assert b"head_dim" in lib.dapq_last_error()
    assert D.workspace_bytes(good_shape(n_q_heads=30)) == 0


FAKE = 0x1000  # never dereferenced: every call below must fail validation first


def call(lib, fn, *args):
    return getattr(lib, fn)(*args)


def test_invalid_arguments_are_rejected_on_the_host(lib):
    s = good_shape()
    ws = D.workspace_bytes(s)
    sp = C.byref(s)
    assert lib.dapq_score(sp, None, FAKE, FAKE, FAKE, ws, None) == ERR_INVALID
    assert b"q is NULL" in lib.dapq_last_error()
    assert lib.dapq_score(sp, FAKE, FAKE, FAKE, FAKE, ws - 1, None) == ERR_WORKSPACE
    assert lib.dapq_score(sp, FAKE + 2, FAKE, FAKE, FAKE, ws, None) == ERR_UNSUPPORTED      # misaligned q
    assert lib.dapq_score(None, FAKE, FAKE, FAKE, FAKE, ws, None) == ERR_INVALID
    bad = good_shape(n_q_heads=30)
    assert lib.dapq_score(C.byref(bad), FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == ERR_INVALID
    bad = good_shape(head_dim=64)
    assert lib.dapq_score(C.byref(bad), FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == ERR_UNSUPPORTED
    bad = good_shape(k_strides=(4096 * 8 * 128, 0, 132, 8 * 128))
    assert lib.dapq_score(C.byref(bad), FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == ERR_UNSUPPORTED
    bad = good_shape(scale=0.0)
    assert lib.dapq_score_stats(C.byref(bad), FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == ERR_INVALID
    bad = good_shape(n_pseudo=0)
    assert lib.dapq_score_accumulate(C.byref(bad), FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == ERR_INVALID
    bad = good_shape(batch=3, total_tokens=4096)                     # dense batch must divide evenly
    assert lib.dapq_pool(C.byref(bad), FAKE, FAKE + 64, 7, None) == ERR_INVALID

    assert lib.dapq_pool(sp, FAKE, FAKE + 64, 4, None) == ERR_INVALID          # even width
    assert lib.dapq_pool(sp, FAKE, FAKE + 64, 65, None) == ERR_INVALID
    assert lib.dapq_pool(sp, FAKE, FAKE, 7, None) == ERR_INVALID               # aliasing
    assert lib.dapq_pool(sp, None, FAKE, 7, None) == ERR_INVALID
    assert lib.dapq_topk(sp, FAKE, 0, None, FAKE, FAKE, None, 0, None) == ERR_INVALID
    assert lib.dapq_topk(sp, FAKE, 8, None, None, FAKE, None, 0, None) == ERR_INVALID
    assert lib.dapq_gather(sp, FAKE, FAKE, FAKE, FAKE, 0, FAKE, FAKE, None) == ERR_INVALID
    assert lib.dapq_gather(sp, FAKE, FAKE + 2, FAKE, FAKE, 8, FAKE, FAKE, None) == ERR_UNSUPPORTED
    assert lib.dapq_gather(sp, FAKE, None, FAKE, FAKE, 8, FAKE, FAKE, None) == ERR_INVALID

    assert lib.dapq_rope_apply(None, FAKE, FAKE, 4, 2, 128, 256, 128, 5e5, 0, None) == ERR_INVALID
    assert lib.dapq_rope_apply(FAKE, FAKE, FAKE, 4, 2, 127, 256, 128, 5e5, 0, None) == ERR_INVALID
    assert lib.dapq_rope_apply(FAKE, FAKE, FAKE, 4, 2, 128, 256, 128, 5e5, 2, None) == ERR_INVALID
    assert lib.dapq_rope_apply(FAKE, FAKE, FAKE, 4, 2, 128, 256, 128, -1.0, 0, None) == ERR_INVALID
    assert lib.dapq_rope_apply(FAKE, FAKE, FAKE, 4, 2, 128, 256, 64, 5e5, 0, None) == ERR_INVALID
    assert lib.dapq_rope_apply(FAKE, FAKE, FAKE, 0, 2, 128, 256, 128, 5e5, 0, None) == 0       # nothing to do


def test_binding_raises_with_the_library_message():
    with pytest.raises(D.DapqError) as e:
        D.dapq_pool(good_shape(), None, None, 7, stream=0)
    assert e.value.code == ERR_INVALID and "NULL" in str(e.value)


def test_product_path_does_not_touch_the_oracle():
    for root, _, files in os.walk(os.path.join(ROOT, "paper_2603_11564_amd")):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(root, f)).read()
                assert "oracle" not in text, f
    assert "oracle" not in open(os.path.join(ROOT, "include", "dapq.h")).read()
    assert "paper_2603_11564_amd" not in open(os.path.join(ROOT, "oracle", "dapq_oracle.py")).read()
