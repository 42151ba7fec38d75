"""Host logic of the launch plans (no GPU): how shapes are cut into splits, slices and workspaces."""
import ctypes

from paper_2402_11131_amd import api, synth


def _msa_plan(cfg, max_len):
    return api.ss_msa_plan(cfg.B, cfg.T, cfg.gamma, cfg.H, cfg.Hkv, cfg.D, max_len, api.SS_BF16 if cfg.dtype == "bf16" else api.SS_F32)


def test_attention_plans_of_the_five_workloads():
    c = synth.CONFIGS
    assert _msa_plan(c["c4"], 4096) == (2, 1)        # two splits, merged inside the attention kernel
    assert _msa_plan(c["c3"], 4096) == (1, 1)        # 512 (sequence, head) items: unsplit
    assert _msa_plan(c["c5"], 32768) == (4, 2)       # five row chunks of 128 rows x 64 KV heads x 4 splits = 5 whole rounds
    splits, kernels = _msa_plan(c["c2"], 2048)
    assert splits == 8 and kernels == 2              # one sequence: 8 splits and the merge kernel
    assert _msa_plan(c["c1"], 128)[1] in (1, 2)


def test_attention_workspace_grows_with_the_splits_and_holds_the_counters():
    c4 = synth.CONFIGS["c4"]
    lib = api.load_library()
    need = lib.ss_msa_workspace_bytes(c4.B, c4.T, c4.gamma, c4.H, c4.Hkv, c4.D, 4096, api.SS_BF16)
    partial_rows = c4.B * c4.H * 2 * c4.R                      # two splits
    assert need >= partial_rows * (c4.D + 1) * 4 + c4.B * c4.Hkv * 8 * 4
    assert lib.ss_msa_workspace_bytes(16, c4.T, c4.gamma, c4.H, c4.Hkv, c4.D, 4096, api.SS_BF16) <= 512   # c3: unsplit
    api.ss_msa_set_split_keys(1024)
    try:
        assert _msa_plan(c4, 4096) == (4, 2)                   # override: four splits go through the merge kernel
    finally:
        api.ss_msa_set_split_keys(0)
    assert _msa_plan(c4, 4096) == (2, 1)


def test_projection_slices():
    bf, f32 = api.SS_BF16, api.SS_F32
    assert api.ss_linear_rows_splits(320, 11008, 4096, bf) == 4     # down map: few outputs, many features
    assert api.ss_linear_rows_splits(320, 4096, 4096, bf) == 4      # output map
    for V in (12288, 22016, 32000):                                 # QKV, gate+up, LM-head-sized: many outputs
        assert api.ss_linear_rows_splits(320, 4096, V, bf) == 1
    assert api.ss_linear_rows_splits(320, 11008, 4096, f32) == 1    # the fp32 kernel is never cut
    assert api.ss_linear_rows_splits(64, 192, 4096, bf) == 1        # three feature blocks cannot be cut in two or four
    assert api.ss_linear_rows_splits(0, 4096, 4096, bf) == 1
    assert api.ss_linear_rows_splits(320, 100, 4096, bf) == 0       # d % 64 != 0: refused, message set
    assert b"64" in api.load_library().ss_last_error()


def test_projection_workspace_matches_the_slices():
    bf = api.SS_BF16
    for N, d, V in ((320, 11008, 4096), (320, 4096, 4096), (96, 2048, 250), (320, 4096, 12288), (1, 64, 8)):
        s = api.ss_linear_rows_splits(N, d, V, bf)
        need = api.ss_linear_rows_workspace_bytes(N, d, V, bf)
        assert need == (s * N * V * 4 + 256 if s > 1 else 256)
    lib = api.load_library()
    one = ctypes.c_void_p(256)  # never dereferenced: validation fails first
    assert lib.ss_linear_rows_ws(one, one, 320, 11008, 4096, bf, one, one, 1024, None) == 4      # SS_ERR_WORKSPACE
    assert b"workspace" in lib.ss_last_error()
    assert lib.ss_linear_rows_ws(one, one, 320, 11008, 4096, bf, one, None, 0, None) == 4
    assert lib.ss_linear_rows_ws(None, one, 320, 11008, 4096, bf, one, one, 1 << 30, None) == 1  # SS_ERR_INVALID_ARG


def test_attention_refuses_a_cache_beyond_its_page_offsets():
    # bf16 path: page offsets are kept in units of 256 bytes in 32 bits, i.e. up to 1 TiB per cache tensor; the
    # check runs on the host before anything is enqueued (the pointers are never dereferenced)
    lib = api.load_library()
    one = ctypes.c_void_p(256)
    pages = (1 << 40) // (32 * 64 * 128 * 2) + 1
    rc = lib.ss_msa_attention(one, one, one, one, one, one, 4, pages, one, one, 1, 4, 1, 32, 32, 128, 64, 0.1,
                              api.SS_BF16, 0, one, None, 0, None)
    assert rc == 2 and b"1 TiB" in lib.ss_last_error()   # SS_ERR_UNSUPPORTED
