"""Host-side checks of the C ABI that need no GPU: every declared symbol is exported, argument
validation happens before any launch, workspace queries are pure functions of host values."""
import ctypes
import os
import re

import pytest

from paper_2604_09562_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2604_09562_amd import build
        build.build()
    return binding.lib()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "specverify.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ss_[a-z_0-9]+)\s*\(", text)))


def test_header_and_exports_agree(L):
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS), (names, binding.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_no_torch_or_cxx_types_in_the_header():
    text = open(os.path.join(ROOT, "include", "specverify.h")).read()
    assert "torch" not in text.lower() and "std::" not in text and "template" not in text


def test_version_and_error_string(L):
    assert L.ss_version() >= 100
    assert isinstance(L.ss_last_error(), bytes)


def _desc(**kw):
    kv = binding.ss_paged_kv(10, 16, 8, 128, binding.SS_BF16, 0, 0, 0, 0)
    bt = binding.ss_batch(4, 8, 0, 0, 0, 0, 0)
    for k, v in kw.items():
        setattr(kv if hasattr(kv, k) else bt, k, v)
    return kv, bt


def test_attention_validation_runs_before_any_launch(L):
    cases = [(dict(block_size=32), b"block_size"), (dict(head_dim=96), b"head_dim"),
             (dict(num_kv_heads=5), b"multiple"), (dict(dtype=7), b"dtype"),
             (dict(max_q_len=22), b"max_q_len"), (dict(batch=-1), b"negative")]
    for kw, msg in cases:
        kv, bt = _desc(**kw)
        rc = L.ss_spec_verify_attn(ctypes.byref(kv), ctypes.byref(bt), None, 1, 32, 20, ctypes.c_float(0.1),
                                   None, None, None, 0, None)
        assert rc == 1, kw
        assert msg in L.ss_last_error(), (kw, L.ss_last_error())
    kv, bt = _desc()
    rc = L.ss_spec_verify_attn(ctypes.byref(kv), ctypes.byref(bt), None, 1, 32, 20, ctypes.c_float(0.1), None,
                               None, None, 0, None)
    assert rc == 1 and b"NULL" in L.ss_last_error()   # null device pointers are refused, nothing is launched
    rc = L.ss_spec_verify_attn(ctypes.byref(kv), ctypes.byref(bt), None, 1, 32, 2, ctypes.c_float(0.1), None,
                               None, None, 0, None)
    assert rc == 1 and b"total_rows" in L.ss_last_error()
    assert L.ss_spec_verify_attn(None, None, None, 1, 32, 2, ctypes.c_float(0.1), None, None, None, 0, None) == 1


def test_attention_workspace_query_is_monotone(L):
    kv, bt = _desc()
    a = L.ss_spec_verify_attn_workspace(ctypes.byref(kv), ctypes.byref(bt), 32, 20)
    bt.batch = 64
    b = L.ss_spec_verify_attn_workspace(ctypes.byref(kv), ctypes.byref(bt), 32, 320)
    assert 0 < a < b
    kv.head_dim = 100
    assert L.ss_spec_verify_attn_workspace(ctypes.byref(kv), ctypes.byref(bt), 32, 320) == 0


def test_accept_validation(L):
    def call(batch=4, vocab=1000, stride=1000, dtype=0, rows=12, greedy=0, T=1.0, mq=0):
        return L.ss_spec_accept(batch, vocab, stride, dtype, rows, mq, None, None, None, None, None, None, None,
                                ctypes.c_float(T), greedy, None, None, None, None, 0, None)
    assert call(vocab=0) == 1
    assert call(rows=3) == 1 and b"total_rows" in L.ss_last_error()
    assert call(stride=999) == 1 and b"row_stride" in L.ss_last_error()
    assert call(dtype=2) == 1 and b"logit_dtype" in L.ss_last_error()
    assert call(mq=-1) == 1 and b"max_q_len" in L.ss_last_error()
    assert call(mq=4) == 1 and b"NULL" in L.ss_last_error()
    assert call() == 1 and b"NULL" in L.ss_last_error()
    assert call(batch=0, rows=0) == 0          # empty batch: no-op
    assert L.ss_spec_accept_workspace(4, 12, 1000) > 0
    assert L.ss_spec_accept_workspace(4, 100, 1000) == 0


def test_options(L):
    assert L.ss_set_option(b"attn_path", 1) == 0
    assert L.ss_set_option(b"attn_path", 0) == 0
    assert L.ss_set_option(b"attn_path", 9) == 1
    assert L.ss_set_option(b"attn_waves", 6) == 1      # not a multiple of the workgroup's wave count
    assert L.ss_set_option(b"attn_unit_weight", 65) == 1   # outside 0..64
    assert L.ss_set_option(b"attn_unit_weight", -1) == 1
    assert L.ss_set_option(b"attn_unit_weight", 0) == 0
    assert L.ss_set_option(b"attn_unit_weight", 3) == 0    # back to the default
    assert L.ss_set_option(b"no_such_option", 1) == 1
    assert L.ss_set_option(None, 1) == 1
