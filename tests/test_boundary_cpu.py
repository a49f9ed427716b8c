"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the public header declares, sizes workspaces deterministically and rejects
bad arguments before touching the device."""
import ctypes
import os
import re

import pytest
import torch

from paper_2506_22694_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2506_22694_amd import build
        build.build_library()
    return binding.load_library()


def declared_functions():
    names = set()
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if fn.endswith(".h"):
            src = open(os.path.join(ROOT, "include", fn)).read()
            src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
            names |= set(re.findall(r"\b(vt_[a-z0-9_]+)\s*\(", src))
    return names


def test_library_exports_every_declared_symbol(lib):
    decl = declared_functions()
    assert decl == set(binding.EXPORTS)
    for name in decl:
        assert getattr(lib, name) is not None


def test_status_strings(lib):
    assert lib.vt_status_string(0) == b"VT_OK"
    for s in range(1, 7):
        assert lib.vt_status_string(s).startswith(b"VT_ERR_")
    assert b"unknown" in lib.vt_status_string(99)


def test_workspace_sizes_are_pure_host_functions(lib):
    a = lib.vt_draft_head_step_ws_bytes(8, 32768, 3072, 8)
    assert a > 0 and a % 256 == 0 and a == lib.vt_draft_head_step_ws_bytes(8, 32768, 3072, 8)
    assert lib.vt_draft_head_step_ws_bytes(1, 32768, 3072, 1) <= a
    assert lib.vt_draft_head_step_ws_bytes(0, 32768, 3072, 1) == 0
    assert lib.vt_draft_head_step_ws_bytes(1, 1 << 20, 3072, 1) == 0      # beyond the supported k
    c = lib.vt_count_tokens_ws_bytes(128256, 10_000_000)
    assert c >= 128256 * 4 and c % 256 == 0
    assert lib.vt_count_tokens_ws_bytes(128256, 100_000_000) == lib.vt_count_tokens_ws_bytes(128256, 10**9)
    assert lib.vt_build_trimmed_head_ws_bytes(128256, 3072, 32768) >= 1


VT_F32, VT_BF16 = binding.VT_F32, binding.VT_BF16
VT_ERR_NULL, VT_ERR_SHAPE, VT_ERR_DTYPE = 1, 2, 3      # as in include/vocabtrim.h


def _plan(lib, n, k, d, m, w_type=VT_BF16):
    buf = ctypes.create_string_buffer(256)
    lib.vt_draft_head_step_plan.argtypes = [ctypes.c_int32] * 4 + [ctypes.c_int, ctypes.c_char_p, ctypes.c_size_t]
    lib.vt_draft_head_step_plan.restype = ctypes.c_int
    rc = lib.vt_draft_head_step_plan(n, k, d, m, w_type, buf, 256)
    return rc, buf.value.decode()


def test_step_plan_is_a_pure_host_function_and_follows_the_head(lib):
    # (no device here: the planner assumes 256 CUs)
    # the benchmark's k: one tile of 128 rows per CU, eight waves
    assert _plan(lib, 8, 32768, 3072, 8) == (
        0, "head_mfma_kernel<1,8> workgroups=256 tile_rows=128 waves=8 column_split=1 + step_finalize_kernel")
    # the paper's own trimmed sizes: tiles of exactly ceil(k / 256) rows, still one per CU -- the extra rows shared
    # by the eight waves (rows a multiple of 1 KiB but not of 2 KiB), else nine waves
    for k, rows in ((32959, 129), (32975, 129), (33008, 129), (35010, 137)):
        for n, m in ((1, 1), (8, 8)):
            rc, text = _plan(lib, n, k, 3072, m)
            assert rc == 0 and f"head_mfma_kernel<1,8> workgroups=256 tile_rows={rows} waves=8" in text, text
        rc, text = _plan(lib, 8, k, 4096, 8)
        assert rc == 0 and "head_mfma_kernel<1,12>" in text and "tile_rows=144 waves=9" in text, text
        # more than 8 hidden rows: the same tiles, two or four groups of hidden rows (9 .. 16 rows run as two)
        for n, nt in ((9, 2), (16, 2), (32, 2), (33, 4), (64, 4)):
            rc, text = _plan(lib, n, k, 4096, 8)
            assert rc == 0 and f"head_mfma_kernel<{nt},8> workgroups=256 tile_rows={rows} waves=8" in text, text
    # below one tile per CU: five to seven waves of 16 rows for more than 8 hidden rows (where their threads can still
    # prefetch a chunk of h), smaller tiles with shared row groups for up to 8
    assert "head_mfma_kernel<4,7> workgroups=238 tile_rows=96 waves=6" in _plan(lib, 64, 22786, 4096, 8)[1]
    assert "head_mfma_kernel<2,7> workgroups=225 tile_rows=80 waves=5" in _plan(lib, 32, 18000, 4096, 8)[1]
    assert "head_mfma_kernel<4,8> workgroups=141 tile_rows=128" in _plan(lib, 64, 18000, 4096, 8)[1]
    assert "head_mfma_kernel<1,8> workgroups=179 tile_rows=128" in _plan(lib, 8, 22786, 3072, 8)[1]
    assert "head_mfma_kernel<1,12> workgroups=238 tile_rows=96 waves=6" in _plan(lib, 1, 22786, 3072, 1)[1]
    assert "tile_rows=32 waves=8 column_split=4" in _plan(lib, 8, 5000, 3072, 8)[1]
    # more tiles than CUs at 144 rows each: ten and twelve waves
    assert "tile_rows=160 waves=10" in _plan(lib, 8, 40000, 3072, 8)[1]
    assert "tile_rows=192 waves=12" in _plan(lib, 8, 49152, 3072, 8)[1]
    # beyond 256 x 192 rows, and fp32: the small-n kernel
    assert _plan(lib, 8, 65536, 3072, 8)[1].startswith("head_gemv_kernel<bf16,8,")
    assert _plan(lib, 4, 4096, 256, 4, VT_F32)[1].startswith("head_gemv_kernel<f32,4,")
    # many hidden rows, many tokens per row
    assert _plan(lib, 256, 32768, 8192, 16)[1] == (
        "pack_h_kernel + head_mfma_wide_kernel<2> workgroups=256 tile_rows=128 + row_select_kernel")
    # errors: shape, dtype, no buffer
    assert _plan(lib, 0, 32768, 3072, 8)[0] == VT_ERR_SHAPE
    assert _plan(lib, 8, 32768, 3072, 65)[0] == VT_ERR_SHAPE
    assert _plan(lib, 8, 32768, 3072, 8, 7)[0] == VT_ERR_DTYPE
    assert lib.vt_draft_head_step_plan(8, 32768, 3072, 8, VT_BF16, None, 0) == VT_ERR_NULL


def test_multi_head_step_plan_one_launch_or_head_by_head():
    plan = binding.draft_head_step_multi_plan
    # the general head beside a task head, four rows each: ten-wave tiles of 160 rows, 205 + 32 of them
    assert plan(8, 3072, [32768, 5000], [0, 0, 0, 0, 1, 1, 1, 1], 8) == (
        "head_mfma_kernel<1,12> heads=2 workgroups=237 tile_rows=160 waves=10 column_split=1 + step_finalize_kernel")
    # small heads: 32-row tiles, four waves per row group; heads without rows do not count
    assert plan(7, 1024, [1500, 700, 3000, 99999], [2, 0, 1, 1, 0, 2, 2], 5) == (
        "head_mfma_kernel<1,8> heads=3 workgroups=163 tile_rows=32 waves=8 column_split=4 + step_finalize_kernel")
    # too many rows for one tile per CU even at 192 rows, more than 8 hidden rows, one head only, fp32, many tokens
    assert plan(4, 3072, [33008, 32975], [0, 1, 1, 0], 8) == "head by head (2)"
    assert plan(12, 1024, [3000, 1500], [0, 1] * 6, 5) == "head by head (2)"
    assert plan(4, 512, [1000, 1200], [1, 1, 1, 1], 4) == "head by head (1)"
    assert plan(4, 512, [1000, 1200], [0, 1, 1, 0], 4, torch.float32) == "head by head (2)"
    assert plan(8, 4096, [16384, 16384], [0, 0, 0, 1, 1, 1, 1, 1], 12) == "head by head (2)"
    assert "heads=2 workgroups=256 tile_rows=128" in plan(8, 4096, [16384, 16384], [0, 0, 0, 1, 1, 1, 1, 1], 11)
    with pytest.raises(binding.VocabTrimError):
        plan(4, 512, [1000, 1200], [0, 2, 1, 0], 4)


A = ctypes.c_void_p(0x10000)      # a well-aligned fake device address; never dereferenced on these paths
ODD = ctypes.c_void_p(0x10004)


def test_count_tokens_argument_errors(lib):
    f = lib.vt_count_tokens
    assert f(A, 7, 10, 100, A, None, A, 1 << 30, None) == 3            # bad id type
    assert f(A, 0, 10, 0, A, None, A, 1 << 30, None) == 2              # V <= 0
    assert f(A, 0, -1, 100, A, None, A, 1 << 30, None) == 2            # negative length
    assert f(None, 0, 10, 100, A, None, A, 1 << 30, None) == 1         # ids NULL
    assert f(A, 0, 10, 100, None, None, A, 1 << 30, None) == 1         # counts NULL
    assert f(A, 0, 0, 100, A, None, None, 0, None) == 0                # empty stream: no-op
    assert f(None, 0, 0, 100, A, None, None, 0, None) == 0
    assert f(ctypes.c_void_p(0x10002), 0, 10, 100, A, None, A, 1 << 30, None) == 4   # ids not 4-byte aligned
    assert f(A, 0, 10, 100, ODD, None, A, 1 << 30, None) == 4          # counts not 8-byte aligned
    assert f(A, 0, 10, 100, A, None, None, 1 << 30, None) == 5         # ws NULL
    assert f(A, 0, 10, 100, A, None, A, 16, None) == 5                 # ws too small
    assert f(A, 0, 10, 100, A, None, ODD, 1 << 30, None) == 5          # ws misaligned


def test_build_trimmed_head_argument_errors(lib):
    f = lib.vt_build_trimmed_head
    ok_ws = (A, 1 << 20, None)
    assert f(A, 100, A, 5, 64, 10, A, A, *ok_ws) == 3                  # bad dtype
    assert f(A, 0, A, 1, 64, 10, A, A, *ok_ws) == 2                    # V <= 0
    assert f(A, 100, A, 1, 0, 10, A, A, *ok_ws) == 2                   # d <= 0
    assert f(A, 100, A, 1, 64, 0, A, A, *ok_ws) == 2                   # k < 1
    assert f(A, 100, A, 1, 64, 101, A, A, *ok_ws) == 2                 # k > V
    assert f(None, 100, A, 1, 64, 10, A, A, *ok_ws) == 1               # counts NULL
    assert f(A, 100, A, 1, 64, 10, None, A, *ok_ws) == 1               # map NULL
    assert f(A, 100, A, 1, 64, 10, A, None, *ok_ws) == 1               # W without W_trim
    assert f(A, 100, A, 1, 12, 10, A, A, *ok_ws) == 4                  # row of 24 bytes
    assert f(A, 100, ODD, 1, 64, 10, A, A, *ok_ws) == 4                # W misaligned
    assert f(A, 100, A, 1, 64, 10, A, A, None, 1 << 20, None) == 5     # ws NULL
    assert f(A, 100, A, 1, 64, 10, A, A, A, 0, None) == 5              # ws too small


def test_draft_head_step_argument_errors(lib):
    f = lib.vt_draft_head_step
    need = lib.vt_draft_head_step_ws_bytes(2, 1000, 512, 4)

    def call(h=A, ht=1, n=2, W=A, wt=1, k=1000, d=512, mp=A, m=4, oi=A, ol=A, lse=None, full=None, ws=A,
             wsb=need):
        return f(h, ht, n, W, wt, k, d, mp, m, oi, ol, lse, full, ws, wsb, None)

    assert call(ht=2) == 3 and call(wt=9) == 3
    assert call(ht=0, wt=1) == 3                                        # h and W must agree
    assert call(n=0) == 2 and call(k=0) == 2 and call(d=0) == 2
    assert call(m=0) == 2 and call(m=1001) == 2 and call(m=65) == 2
    assert call(k=1 << 20) == 2
    assert call(h=None) == 1 and call(W=None) == 1 and call(mp=None) == 1
    assert call(oi=None) == 1 and call(ol=None) == 1
    assert call(d=516) == 4                                             # row of 1032 bytes: not 16-byte rows
    assert call(h=ODD) == 4 and call(W=ODD) == 4
    assert call(ws=None) == 5 and call(wsb=need - 1) == 5 and call(ws=ODD) == 5
    assert lib.vt_draft_head_step_ws_init(None, 1024, None) == 5
    assert lib.vt_draft_head_step_ws_init(A, 8, None) == 5


def test_tree_selection_argument_errors(lib):
    f = lib.vt_tree_expand
    ok = (A, A, A, 8, 8, 8, A, A, A, None)
    for pos in (0, 1, 2, 6, 7, 8):
        bad = list(ok)
        bad[pos] = None
        assert f(*bad) == 1, pos
    assert f(A, A, A, 0, 8, 1, A, A, A, None) == 2
    assert f(A, A, A, 8, 0, 1, A, A, A, None) == 2
    assert f(A, A, A, 8, 8, 0, A, A, A, None) == 2
    assert f(A, A, A, 8, 8, 65, A, A, A, None) == 2          # K > n * m
    assert f(A, A, A, 257, 64, 8, A, A, A, None) == 2        # n * m above the limit
    g = lib.vt_tree_rerank
    assert g(None, 10, 5, A, None) == 1 and g(A, 10, 5, None, None) == 1
    assert g(A, 0, 1, A, None) == 2 and g(A, 10, 0, A, None) == 2 and g(A, 10, 11, A, None) == 2
    assert g(A, 16385, 8, A, None) == 2 and g(A, 4096, 1025, A, None) == 2


def test_choose_k_and_ranked_build_argument_errors(lib):
    f = lib.vt_choose_k
    big = 1 << 30
    assert f(A, 100, 2, 0.5, 0, A, A, big, None) == 3            # unknown mode
    assert f(A, 0, 0, 0.5, 0, A, A, big, None) == 2
    assert f(A, 100, 0, 1.5, 0, A, A, big, None) == 2            # p outside [0, 1]
    assert f(A, 100, 0, float("nan"), 0, A, A, big, None) == 2
    assert f(None, 100, 0, 0.5, 0, A, A, big, None) == 1 and f(A, 100, 0, 0.5, 0, None, A, big, None) == 1
    assert f(A, 100, 0, 0.5, 0, A, A, 16, None) == 5
    assert lib.vt_choose_k_ws_bytes(128256) >= 128256 * (4 + 8 + 24)
    g = lib.vt_build_trimmed_head_by_rank
    assert g(A, 100, A, 1, 64, 0, A, A, A, big, None) == 2
    assert g(A, 100, A, 1, 64, 10, None, A, A, big, None) == 1
    assert g(A, 100, A, 1, 64, 10, A, A, A, 256, None) == 5      # the sort needs room
    assert lib.vt_build_trimmed_head_ws_bytes(128256, 3072, 32768) >= 256 + 32768 * 28


def test_draft_tree_level_argument_errors(lib):
    f = lib.vt_draft_tree_level
    big = 1 << 30
    ok = [A, 1, 8, A, 1, 32768, 3072, A, 8, A, 8, A, A, A, A, A, A, big, None]
    assert f(*ok[:2], 0, *ok[3:]) == 2                          # n
    bad = list(ok); bad[10] = 0
    assert f(*bad) == 2                                         # K < 1
    bad = list(ok); bad[10] = 65
    assert f(*bad) == 2                                         # K > n * m
    for pos in (0, 3, 7, 9, 11, 12, 13, 14, 15):
        bad = list(ok); bad[pos] = None
        assert f(*bad) == 1, pos
    bad = list(ok); bad[1] = 0
    assert f(*bad) == 3                                         # h and W types differ
    bad = list(ok); bad[17] = 16
    assert f(*bad) == 5


def test_binding_refuses_host_tensors():
    import torch
    with pytest.raises(ValueError):
        binding.count_tokens(torch.zeros(4, dtype=torch.int32), 10)


def test_build_rejects_kernels_that_use_scratch_memory():
    # the draft-step kernels wait by hand for loads the compiler does not track, so a spilled register
    # could be saved before its value arrives: the build parses the compiler's resource remarks
    from paper_2506_22694_amd import build
    remarks = "\n".join([
        "a.hip:1:1: remark: Function Name: kernel_a [-Rpass-analysis=kernel-resource-usage]",
        "a.hip:1:1: remark:     VGPRs: 256 [-Rpass-analysis=kernel-resource-usage]",
        "a.hip:1:1: remark:     ScratchSize [bytes/lane]: 24 [-Rpass-analysis=kernel-resource-usage]",
        "a.hip:1:1: remark: Function Name: kernel_b [-Rpass-analysis=kernel-resource-usage]",
        "a.hip:1:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]",
    ])
    assert build._scratch_users(remarks) == [("kernel_a", 24)]
    assert any("vt_head_mfma.hip".startswith(p) for p in build.NO_SCRATCH)


_ASM_HEAD = """
\t.text
\t.globl\tkern
\t.type\tkern,@function
kern:
"""


def _lint(body):
    from paper_2506_22694_amd import inflight_lint
    bad, loads = inflight_lint.check_asm(_ASM_HEAD + body + "\ts_endpgm\n")
    return [(b[3]) for b in bad], loads


def test_inflight_lint_flags_touches_between_a_hand_issued_load_and_its_wait():
    load = "\t;;#ASMSTART\n\tglobal_load_dwordx4 v[4:7], v1, s[2:3] nt\n\t;;#ASMEND\n"
    load2 = "\t;;#ASMSTART\n\tglobal_load_dwordx4 v[8:11], v1, s[2:3] nt\n\t;;#ASMEND\n"
    wait = lambda n: f"\t;;#ASMSTART\n\ts_waitcnt vmcnt({n})\n\t;;#ASMEND\n"
    use = "\tds_write_b128 v20, v[4:7]\n"
    # clean: wait, then use; an unrelated instruction in between is fine
    assert _lint(load + "\tv_add_u32_e32 v30, v31, v32\n" + wait(0) + use) == ([], 1)
    # a copy before the wait reads a register that is still in flight
    assert _lint(load + "\tv_mov_b32_e32 v40, v5\n" + wait(0) + use)[0] == ["v_mov_b32_e32 v40, v5"]
    # vmcnt(1) with one younger load behind covers the first load, not the second
    assert _lint(load + load2 + wait(1) + use)[0] == []
    assert _lint(load + load2 + wait(1) + "\tds_write_b128 v20, v[8:11]\n")[0] == ["ds_write_b128 v20, v[8:11]"]
    # vmcnt(1) with nothing behind does not cover the load
    assert _lint(load + wait(1) + use)[0] == ["ds_write_b128 v20, v[4:7]"]
    # loads the compiler issued itself (outside the markers) are not followed but count as younger loads
    assert _lint("\tglobal_load_dword v9, v[2:3], off\n\tv_mov_b32_e32 v1, v9\n") == ([], 0)
    assert _lint(load + "\tglobal_load_dword v50, v[2:3], off\n" + wait(1) + use)[0] == []


def test_inflight_lint_reports_compiler_waits_that_drain_hand_issued_loads():
    from paper_2506_22694_amd import inflight_lint
    load = "\t;;#ASMSTART\n\tglobal_load_dwordx4 v[4:7], v1, s[2:3] nt\n\t;;#ASMEND\n"
    body = load + "\tglobal_load_dword v9, v[2:3], off\n\ts_waitcnt vmcnt(0)\n\tv_mov_b32_e32 v1, v9\n"
    drains = set()
    bad, _ = inflight_lint.check_asm(_ASM_HEAD + body + "\ts_endpgm\n", drains)
    assert bad == [] and [d[2] for d in drains] == ["s_waitcnt vmcnt(0)"]


def test_inflight_lint_follows_every_path():
    load = "\t;;#ASMSTART\n\tglobal_load_dwordx4 v[4:7], v1, s[2:3] nt\n\t;;#ASMEND\n"
    wait0 = "\t;;#ASMSTART\n\ts_waitcnt vmcnt(0)\n\t;;#ASMEND\n"
    # a branch around the wait: the path that skips it reaches the use with the load in flight
    body = load + "\ts_cbranch_scc1 .LBB0_2\n" + wait0 + ".LBB0_2:\n\tds_write_b128 v20, v[4:7]\n"
    assert _lint(body)[0] == ["ds_write_b128 v20, v[4:7]"]
    # a copy at the join of a branch that sits between the load and its wait
    body = (load + "\ts_cbranch_scc1 .LBB0_2\n\tv_mov_b32_e32 v30, 0\n.LBB0_2:\n\tv_mov_b32_e32 v40, v4\n" + wait0 +
            "\tds_write_b128 v20, v[40:43]\n")
    assert _lint(body)[0] == ["v_mov_b32_e32 v40, v4"]
    # a loop: the refill of the slot at the end of the body is waited for at the top of the next iteration
    loop = (".LBB0_1:\n" + wait0 + "\tds_write_b128 v20, v[4:7]\n" + load + "\ts_add_i32 s4, s4, 1\n\ts_cmp_lt_i32 s4, s5\n"
            "\ts_cbranch_scc1 .LBB0_1\n" + wait0)
    assert _lint(load + loop)[0] == []
    # the same loop with the staging write ahead of the wait
    loop_bad = (".LBB0_1:\n\tds_write_b128 v20, v[4:7]\n" + wait0 + load + "\ts_cmp_lt_i32 s4, s5\n"
                "\ts_cbranch_scc1 .LBB0_1\n" + wait0)
    assert _lint(load + loop_bad)[0] != []


def test_multi_head_argument_errors(lib):
    # validation happens on the host before any device call
    i32p = ctypes.c_int32 * 2
    ks = i32p(1000, 500)
    hor = (ctypes.c_int32 * 4)(0, 1, 0, 1)
    ptrs = (ctypes.c_void_p * 2)(0x1000, 0x2000)
    lib.vt_draft_head_step_multi.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int32, ctypes.c_int32,
                                             ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                             ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p,
                                             ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                             ctypes.c_void_p]
    lib.vt_draft_head_step_multi_ws_bytes.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32,
                                                      ctypes.c_int32]
    lib.vt_draft_head_step_multi_ws_bytes.restype = ctypes.c_size_t
    call = lambda **kw: lib.vt_draft_head_step_multi(
        kw.get("h", 0x1000), kw.get("ht", 1), kw.get("n", 4), kw.get("d", 256), kw.get("W", ptrs), kw.get("wt", 1),
        kw.get("k", ks), kw.get("map", ptrs), kw.get("H", 2), kw.get("hor", hor), kw.get("m", 4), 0x3000, 0x4000, None,
        kw.get("ws", 0x10000), kw.get("wsb", 1 << 30), None)
    assert call(h=None) == 1                      # VT_ERR_NULL
    assert call(hor=None) == 1
    assert call(n=0) == 2 and call(n=257) == 2    # VT_ERR_SHAPE
    assert call(H=0) == 2 and call(H=17) == 2
    assert call(hor=(ctypes.c_int32 * 4)(0, 2, 0, 1)) == 2      # head index out of range
    assert call(m=501) == 2                       # m beyond the smaller head that has rows
    assert call(m=65) == 2
    assert call(ht=0) == 3                        # VT_ERR_DTYPE: h and W differ
    assert call(h=0x1004) == 4                    # VT_ERR_ALIGN
    assert call(ws=None) == 5 and call(wsb=16) == 5
    need = lib.vt_draft_head_step_multi_ws_bytes(4, 256, ks, 2, 4)
    assert need > 0 and need % 256 == 0
    assert lib.vt_draft_head_step_multi_ws_bytes(0, 256, ks, 2, 4) == 0
    assert lib.vt_draft_head_step_multi_ws_bytes(4, 256, ks, 17, 4) == 0
    # an unused head's pointers are not looked at
    assert call(W=(ctypes.c_void_p * 2)(0x1000, None), hor=(ctypes.c_int32 * 4)(0, 0, 0, 0), wsb=16) == 5

    lib.vt_build_trimmed_heads.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int,
                                           ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                           ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    build = lambda **kw: lib.vt_build_trimmed_heads(kw.get("c", 0x1000), kw.get("V", 2000), kw.get("H", 2), None, 1, 256,
                                                    kw.get("k", ks), kw.get("map", ptrs), None, kw.get("ws", 0x10000),
                                                    kw.get("wsb", 1 << 30), None)
    assert build(c=None) == 1 and build(k=None) == 1 and build(map=None) == 1
    assert build(H=0) == 2 and build(H=17) == 2 and build(V=0) == 2
    assert build(V=900) == 2                      # k[0] = 1000 > V
    assert build(map=(ctypes.c_void_p * 2)(0x1000, None)) == 1
    assert build(wsb=16) == 5
