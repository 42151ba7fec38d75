"""The C-ABI library loads without a GPU and exports every symbol include/ss.h declares;
host-only entry points and argument validation work without touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest
import torch

from conftest import ROOT
from paper_2402_11131_amd import api


def _declared():
    text = open(os.path.join(ROOT, "include", "ss.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ss_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = api.load_library()
    names = _declared()
    assert len(names) >= 12
    for n in names:
        assert getattr(lib, n) is not None
    assert set(names) == set(api.EXPORTS)
    assert lib.ss_version() >= 100


def test_one_hip_runtime_in_process():
    api.load_library()
    maps = open("/proc/self/maps").read()
    libs = set(re.findall(r"(/\S*libamdhip64\.so\S*)", maps))
    assert len(libs) == 1, libs


def test_check_tree_host():
    api.ss_check_tree_host(torch.tensor([[-1, 0, 0, 1]], dtype=torch.int32), max_depth=2)
    with pytest.raises(api.SSError) as e:
        api.ss_check_tree_host(torch.tensor([[-1, 0, 2, 1]], dtype=torch.int32))
    assert e.value.code == 3 and "parent[2]" in str(e.value)
    with pytest.raises(api.SSError):
        api.ss_check_tree_host(torch.tensor([[0, 0]], dtype=torch.int32))
    with pytest.raises(api.SSError):
        api.ss_check_tree_host(torch.tensor([[-1, 0, 1, 2]], dtype=torch.int32), max_depth=2)


def test_full_tree_template_host_matches_closed_form(golden):
    for gamma, k, nodes, _rows in golden("tree_size_closed_form.txt")[""]:
        if nodes > api.SS_MAX_T:
            with pytest.raises(api.SSError):
                api.ss_full_tree_template_host([k] * gamma)
            continue
        par, rank, dep = api.ss_full_tree_template_host([k] * gamma)
        assert len(par) == nodes
        assert [int((dep == j).sum()) for j in range(gamma + 1)] == [k ** j for j in range(gamma + 1)]


def test_argument_validation_needs_no_device():
    lib = api.load_library()
    one = ctypes.c_void_p(8)  # never dereferenced: validation fails first
    assert lib.ss_build_mask(None, 1, 4, 2, 0, None, None, None, None) == 1
    assert lib.ss_build_mask(one, 1, 65, 2, 0, None, None, None, None) == 2
    assert lib.ss_build_mask(one, 1, 4, 9, 0, None, None, None, None) == 2
    assert b"gamma" in lib.ss_last_error()
    assert lib.ss_msa_workspace_bytes(1, 8, 3, 4, 4, 96, 128, 0) == 0      # head dim 96
    assert lib.ss_msa_workspace_bytes(4, 16, 4, 32, 32, 128, 4096, 1) > 0
    assert lib.ss_lm_head_workspace_bytes(320, 4096, 32000, 4, 1) >= 320 * 250 * 4 * 8
    assert lib.ss_lm_head_workspace_bytes(320, 4096, 32000, 9, 1) == 0
    assert lib.ss_lm_head_argmax_topk(one, one, 4, 100, 50, 2, 1, one, one, one, 1 << 20, None) == 2  # d % 64
    assert lib.ss_tree_verify(one, one, one, 4, 1, 1, 70, 3, one, one, one, one, one, None) == 2
    assert lib.ss_tree_draft(one, 8, 2, one, one, None, None, None, 1, 4, 2, 7, one, one, None) == 1
    br = (ctypes.c_int32 * 2)(2, 2)
    assert lib.ss_tree_draft(one, 8, 2, one, one, None, None, br, 1, 4, 2, 6, one, one, None) == 1  # T2 != 7
    assert b"7" in lib.ss_last_error()
    args = [one] * 6 + [8, 16, one, one, 1, 8, 3, 4, 4, 64, 24, ctypes.c_float(0.125), 0, 0, one, one, 1 << 20, None]
    assert lib.ss_msa_attention(*args) == 2                                  # page size 24
    assert b"page_size" in lib.ss_last_error()


def test_argument_validation_of_the_rows_around_the_hot_path():
    lib = api.load_library()
    one = ctypes.c_void_p(8)  # never dereferenced: validation fails first
    f = ctypes.c_float
    assert lib.ss_linear_rows(one, one, 4, 100, 50, 1, one, None) == 2            # bf16 needs d % 64 == 0
    assert lib.ss_linear_rows(one, one, 4, 128, 50, 7, one, None) == 2            # dtype
    assert lib.ss_linear_rows(None, one, 4, 128, 50, 1, one, None) == 1           # NULL tensor
    assert lib.ss_linear_rows(None, None, 0, 128, 50, 1, None, None) == 0         # N == 0: no-op
    assert lib.ss_stream_insert(one, None, one, 1, 65, 2, 64, 1, one, None) == 2  # T above the limit
    assert lib.ss_stream_insert(one, None, one, 1, 4, 9, 64, 1, one, None) == 2   # gamma above the limit
    assert lib.ss_stream_insert(one, None, None, 1, 4, 2, 64, 1, one, None) == 1  # P missing with gamma > 0
    assert lib.ss_stream_insert(None, None, None, 0, 4, 2, 64, 1, None, None) == 0
    assert lib.ss_value_rotate(one, 1, 4, 2, 2, 63, f(0.1), 1, None) == 1         # odd head dim
    assert lib.ss_value_rotate(one, 1, 65, 2, 2, 64, f(0.1), 1, None) == 2
    assert lib.ss_value_rotate(None, 1, 4, 2, 2, 64, f(0.1), 1, None) == 1
    assert lib.ss_value_rotate(ctypes.c_void_p(6), 1, 4, 2, 2, 64, f(0.1), 1, None) == 1  # not aligned to a pair
    assert lib.ss_value_rotate(None, 1, 4, 0, 2, 64, f(0.1), 1, None) == 0          # no streams: no-op
    assert lib.ss_probe_hbm_read(one, 1 << 20, 1, one, None) == 1                  # less than one round of all waves
    assert lib.ss_probe_hbm_read(ctypes.c_void_p(8), 1 << 30, 0, one, None) == 1    # not 16-byte aligned
    assert lib.ss_probe_mfma_bf16(0, None, one, None) == 1
    assert lib.ss_lm_head_logsumexp(one, one, 4, 100, 50, 1, one, one, 1 << 20, None) == 2
    assert lib.ss_lm_head_logsumexp(one, one, 4, 128, 50, 1, one, one, 8, None) == 4  # workspace too small
    assert b"workspace" in lib.ss_last_error()
    assert lib.ss_transition_probs(one, one, one, one, one, 1, 65, 64, 50, 1, one, None) == 2
    assert lib.ss_transition_probs(one, one, one, one, None, 1, 4, 64, 50, 1, one, None) == 1
    assert lib.ss_tree_prune(one, one, one, f(0.5), 1, 0, one, one, one, one, one, None) == 2
    assert lib.ss_tree_prune(one, one, one, f(0.5), 1, 4, one, one, one, one, one, None) == 1  # outputs alias inputs
    assert lib.ss_kv_commit(one, one, one, one, one, 8, 16, one, one, one, 1, 8, 3, 4, 64, 24, 3, 1, one, None) == 2
    assert b"page_size" in lib.ss_last_error()


def test_argument_validation_of_the_fused_tail():
    lib = api.load_library()
    one = ctypes.c_void_p(8)  # never dereferenced: validation fails first
    br = (ctypes.c_int32 * 2)(2, 2)

    def call(d=128, V=500, K=4, dtype=1, B=2, T=8, gamma=2, max_depth=3, tp=None, tr=None, branching=br, T2=7,
             ws=one, ws_bytes=1 << 30, hidden=one):
        return lib.ss_lm_head_verify_draft(hidden, one, d, V, K, dtype, one, one, B, T, gamma, max_depth, tp, tr,
                                           branching, T2, one, one, one, one, one, one, None, None, ws, ws_bytes, None)

    assert call(T=65) == 2 and call(gamma=9) == 2 and call(max_depth=64) == 2 and call(K=9) == 2
    assert call(d=100) == 2                                  # bf16 needs d % 64 == 0
    assert call(T2=6) == 1 and b"7" in lib.ss_last_error()   # branching (2,2) has 7 nodes
    assert call(K=1) == 1                                    # branching 2 exceeds K = 1
    assert call(branching=None) == 1                         # neither template nor branching
    assert call(tp=one) == 1                                 # template given by half
    assert call(hidden=None) == 1
    assert call(ws_bytes=64) == 4 and b"workspace" in lib.ss_last_error()
    assert call(B=0, hidden=None, ws=None, ws_bytes=0) == 0  # empty batch: no-op


def test_attention_plan_query_is_host_only():
    # c4's shape: two splits merged inside the kernel (one kernel per call), two kernels with the knob off;
    # c3's 512 (sequence, head) items: unsplit; c2: more than two splits, so a merge kernel follows
    assert api.ss_msa_plan(4, 16, 4, 32, 32, 128, 4096 + 96, api.SS_BF16) == (2, 1)
    prev = api.ss_msa_set_merge_in_kernel(False)
    try:
        assert api.ss_msa_plan(4, 16, 4, 32, 32, 128, 4096 + 96, api.SS_BF16) == (2, 2)
    finally:
        api.ss_msa_set_merge_in_kernel(prev)
    assert api.ss_msa_plan(16, 16, 4, 32, 32, 128, 4096 + 96, api.SS_BF16) == (1, 1)
    n_splits, n_kernels = api.ss_msa_plan(1, 16, 4, 32, 32, 128, 2048 + 96, api.SS_BF16)
    assert n_splits > 2 and n_kernels == 2
    with pytest.raises(api.SSError):
        api.ss_msa_plan(1, 16, 4, 32, 32, 96, 2048, api.SS_BF16)     # head dim 96
    # the workspace query agrees: nothing but the header when unsplit
    assert api.ss_msa_workspace_bytes(16, 16, 4, 32, 32, 128, 4096 + 96, api.SS_BF16) == 256


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(api, "_lib", None)
    monkeypatch.setattr(api, "LIB_PATH", "/nonexistent/libss.so")
    with pytest.raises(RuntimeError, match="not built"):
        api.load_library()
