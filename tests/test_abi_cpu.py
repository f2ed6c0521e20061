"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, validates arguments before touching the device, and plans kernels sensibly."""
import ctypes
import os
import re
import subprocess

import pytest

from paper_2401_14110_amd import binding as lb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOOD_P = (5, 7, 15, 0)
GOOD_A = (4, 7, 7, 0)


def declared_functions():
    names = set()
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if fn.endswith(".h"):
            text = open(os.path.join(ROOT, "include", fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(lba_\w+)\s*\(", text))
    return names


def test_library_exports_every_declared_symbol():
    L = lb.lib()
    names = declared_functions()
    assert {"lba_gemm", "lba_gemm_bwd", "lba_mask_words", "lba_strerror", "lba_plan_query"} <= names
    for n in names:
        assert hasattr(L, n), n
        # the Python binding carries the same names
        assert hasattr(lb, n), n


def exported_functions():
    out = subprocess.run(["nm", "-D", "--defined-only", os.path.join(ROOT, "paper_2401_14110_amd", "liblba_hip.so")],
                         check=True, capture_output=True, text=True).stdout
    return {f[2] for f in (line.split() for line in out.splitlines()) if len(f) == 3 and f[1] in "TW" and f[2].startswith("lba_")}


def test_header_declares_every_exported_symbol():
    # the other direction: an exported entry point that the header does not declare cannot be reached from C
    exported = exported_functions()
    assert {"lba_gemm", "lba_gemm_bwd_chunked", "lba_mask_words_level2"} <= exported
    assert exported <= declared_functions(), exported - declared_functions()
    for n in exported:
        assert hasattr(lb, n), n


def test_a_c99_caller_compiles_against_the_header_and_links(tmp_path):
    exe = str(tmp_path / "c_caller")
    libdir = os.path.join(ROOT, "paper_2401_14110_amd")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "c_caller.c"), "-o", exe, "-L", libdir, "-llba_hip",
                    "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"], check=True)
    run = subprocess.run([exe], capture_output=True, text=True)
    assert run.returncode == 0, (run.returncode, run.stdout, run.stderr)
    assert "c caller ok" in run.stdout


def test_mask_word_counts_saturate_instead_of_wrapping():
    big = (1 << 62)
    assert lb.lba_mask_words(big, big, 64) == (1 << 64) - 1
    assert lb.lba_mask_words_level2(big, big, 1 << 40) == (1 << 64) - 1
    assert lb.lba_mask_words((1 << 30) - 64, 1 << 21, (1 << 31) - 64) == (1 << 64) - 1   # the largest admitted shape: 2^77 words
    assert lb.lba_mask_words(1 << 20, 1 << 20, (1 << 20) + 1) == ((1 << 15) + 1) << 40
    # a NULL plane with sizes whose product would overflow 64 bits is still a NULL error, not undefined behaviour
    A = ctypes.c_void_p(0x1000)
    assert lb.lba_gemm_bwd_diff(A, A, A, None, (1 << 30) - 64, 1 << 21, (1 << 31) - 64, GOOD_P, GOOD_A, 0, 0.5) == lb.ERR_NULL


def test_gradient_call_checks_every_pointer_before_launching():
    G = A = B = P = O = ctypes.c_void_p(0x1000)
    # dX and dW asked for, A missing: refused although the dX side alone would have been fine
    assert lb.lba_grad(G, None, B, P, None, O, O, 8, 8, 8, 1) == lb.ERR_NULL
    assert lb.lba_grad(G, A, None, P, None, O, O, 8, 8, 8, 1) == lb.ERR_NULL
    assert lb.lba_grad(G, A, B, None, None, O, O, 8, 8, 8, 1) == lb.ERR_NULL
    assert lb.lba_grad(G, A, B, P, None, O, O, 8, 8, 8, 2) == lb.ERR_NULL


def test_recompute_with_brick_maps_validates_before_launching():
    A = ctypes.c_void_p(0x1000)
    W = ctypes.c_void_p(0x2000)                                # 256-byte aligned
    need = lb.lba_grad_workspace_bytes(256, 64, 512)
    assert need >= 512
    args = (256, 64, 512, GOOD_P, GOOD_A)
    assert lb.lba_gemm_bwd_ws(A, A, A, None, A, *args, W, need) == lb.ERR_NULL        # the maps describe the OF plane
    assert lb.lba_gemm_bwd_ws(A, A, A, A, A, *args, None, need) == lb.ERR_NULL
    assert lb.lba_gemm_bwd_ws(A, A, A, A, A, *args, ctypes.c_void_p(0x2010), need) == lb.ERR_ALIGN
    assert lb.lba_gemm_bwd_ws(A, A, A, A, A, *args, W, need - 1) == lb.ERR_SHAPE
    assert lb.lba_gemm_bwd_ws(None, A, A, A, A, *args, W, need) == lb.ERR_NULL
    assert lb.lba_gemm_bwd_ws(A, A, A, A, A, 1 << 20, 1 << 11, 64, GOOD_P, GOOD_A, W, 1 << 30) == lb.ERR_SHAPE   # beyond lba_grad
    assert lb.lba_gemm_bwd_ws(A, A, A, A, A, 256, 64, 512, (9, 7, 15, 0), GOOD_A, W, need) == lb.ERR_FORMAT
    assert lb.lba_gemm_bwd_ws(A, A, A, A, A, 0, 64, 512, GOOD_P, GOOD_A, None, 0) == lb.OK            # nothing to do
    G = O = A
    assert lb.lba_grad_premapped(G, A, A, A, O, O, 256, 64, 512, None, need) == lb.ERR_NULL
    assert lb.lba_grad_premapped(G, A, A, A, O, O, 256, 64, 512, ctypes.c_void_p(0x2010), need) == lb.ERR_ALIGN
    assert lb.lba_grad_premapped(G, A, A, A, O, O, 256, 64, 512, W, need - 1) == lb.ERR_SHAPE
    assert lb.lba_grad_premapped(G, A, A, None, O, O, 256, 64, 512, W, need) == lb.ERR_NULL
    assert lb.lba_grad_premapped(None, A, A, A, O, O, 256, 64, 512, W, need) == lb.ERR_NULL


def test_status_texts():
    for code in range(0, 7):
        assert lb.strerror(code)
    assert lb.strerror(0) == "ok"
    assert "unknown" in lb.strerror(99)


def test_mask_words():
    assert lb.lba_mask_words(4, 5, 1) == 20
    assert lb.lba_mask_words(4, 5, 32) == 20
    assert lb.lba_mask_words(4, 5, 33) == 40
    assert lb.lba_mask_words(4096, 4096, 4096) == 128 * 4096 * 4096
    assert lb.lba_mask_words(0, 5, 33) == 0 and lb.lba_mask_words(4, 5, 0) == 0 and lb.lba_mask_words(-1, 5, 3) == 0
    assert lb.lba_mask_words_level2(4, 5, 1) == 20 and lb.lba_mask_words_level2(4, 5, 512) == 20
    assert lb.lba_mask_words_level2(4, 5, 513) == 40 and lb.lba_mask_words_level2(4, 0, 513) == 0


BAD_FMTS = [(4, 7, 7, 0x102), (4, 7, 7, 0x200), (4, 0, 7, 0), (4, 24, 7, 0), (1, 7, 0, 0), (8, 7, 7, 0), (4, 7, 127, 0), (4, 7, 7, 2), (4, 7, 7, -1),
            (7, 7, -1, 0), (4, 7, -113, 0)]


@pytest.mark.parametrize("bad", BAD_FMTS)
def test_format_limits_are_rejected_before_any_device_work(bad):
    # bogus non-null addresses: a call that got as far as the device would fault, so a clean
    # status proves validation comes first
    A = B = C = ctypes.c_void_p(0x1000)
    assert lb.lba_gemm(A, B, C, 8, 8, 8, bad, GOOD_A) == lb.ERR_FORMAT
    assert lb.lba_gemm(A, B, C, 8, 8, 8, GOOD_P, bad) == lb.ERR_FORMAT
    assert lb.lba_gemm_bwd(A, B, C, C, C, 8, 8, 8, bad, GOOD_A) == lb.ERR_FORMAT
    with pytest.raises(lb.LbaError):
        lb.lba_plan_query(8, 8, 8, bad, GOOD_A)


def test_edge_formats_are_accepted():
    for ok in [(4, 7, 126, 0), (7, 23, 0, 1), (2, 1, -124, 0), (7, 7, 64, 1), (4, 7, -112, 0),
               (4, 7, 7, 0x100), (4, 7, 7, 0x101)]:
        lb.lba_plan_query(8, 8, 8, ok, ok)


def test_shape_order_and_null_errors():
    A = B = C = ctypes.c_void_p(0x1000)
    assert lb.lba_gemm(A, B, C, -1, 8, 8, GOOD_P, GOOD_A) == lb.ERR_SHAPE
    assert lb.lba_gemm(A, B, C, 8, -1, 8, GOOD_P, GOOD_A) == lb.ERR_SHAPE
    assert lb.lba_gemm(A, B, C, 8, 8, -1, GOOD_P, GOOD_A) == lb.ERR_SHAPE
    assert lb.lba_gemm(A, B, C, 1 << 31, 8, 8, GOOD_P, GOOD_A) == lb.ERR_SHAPE
    assert lb.lba_gemm(A, B, C, 8, (1 << 21) + 1, 8, GOOD_P, GOOD_A) == lb.ERR_SHAPE
    # the largest M is 2^24 - 1 workgroups of 64 rows (a launch holds fewer than 2^32 lanes along x)
    assert lb.lba_gemm(A, B, C, (1 << 30) - 63, 8, 8, GOOD_P, GOOD_A) == lb.ERR_SHAPE
    assert lb.lba_plan_query((1 << 30) - 64, 8, 8, GOOD_P, GOOD_A)["grid_x"] == (1 << 24) - 1
    assert lb.lba_gemm(A, B, C, 8, 8, (1 << 31) - 63, GOOD_P, GOOD_A) == lb.ERR_SHAPE
    # one lane per output in the plane post-passes: M * N <= 2^31
    assert lb.lba_last_overflow(A, C, 1 << 20, (1 << 11) + 1, 8) == lb.ERR_SHAPE
    assert lb.lba_ste_plane(A, None, C, 1 << 20, (1 << 11) + 1, 8, 1, 0) == lb.ERR_SHAPE
    assert lb.lba_gemm(A, B, C, 8, 8, 8, GOOD_P, GOOD_A, order=5) == lb.ERR_UNSUPPORTED
    assert lb.lba_gemm(A, B, None, 8, 8, 8, GOOD_P, GOOD_A) == lb.ERR_NULL
    assert lb.lba_gemm(None, B, C, 8, 8, 8, GOOD_P, GOOD_A) == lb.ERR_NULL
    assert lb.lba_gemm(A, None, C, 8, 8, 8, GOOD_P, GOOD_A) == lb.ERR_NULL
    assert lb.lba_gemm_bwd(A, B, C, None, None, 8, 8, 8, GOOD_P, GOOD_A) == lb.ERR_NULL
    # empty outputs: nothing to do, pointers are not looked at
    assert lb.lba_gemm(None, None, None, 0, 8, 8, GOOD_P, GOOD_A) == lb.OK
    assert lb.lba_gemm(None, None, None, 8, 0, 8, GOOD_P, GOOD_A) == lb.OK


def test_diff_threshold_is_validated():
    A = B = C = D = ctypes.c_void_p(0x1000)
    call = lambda eps2, **kw: lb.lba_gemm_bwd_diff(A, B, C, D, kw.get("M", 0), 8, 8, GOOD_P, kw.get("qa", GOOD_A),
                                                   kw.get("order", 0), eps2)
    for ok in (0.0, 2.0 ** -32, 0.5, 0.75, 4095 * 2.0 ** -14, 16.0):
        assert call(ok) == lb.OK, ok                      # M = 0: validated, nothing launched
    for bad in (-0.5, 2.0 ** -33, 17.0, 4097 * 2.0 ** -14, 0.1, float("nan"), float("inf")):
        assert call(bad) == lb.ERR_FORMAT, bad
    assert call(0.5, qa=(4, 7, 200, 0)) == lb.ERR_FORMAT
    assert call(0.5, order=7) == lb.ERR_UNSUPPORTED
    assert call(0.5, order=1) == lb.OK
    assert lb.lba_gemm_bwd_diff(A, B, C, None, 8, 8, 8, GOOD_P, GOOD_A, 0, 0.5) == lb.ERR_NULL
    m4e3 = (3, 4, 3)
    assert lb.lba_gemm_bwd_diff_in(A, B, C, D, 0, 8, 8, m4e3, m4e3, GOOD_P, GOOD_A, 1, 0.5) == lb.OK
    assert lb.lba_gemm_bwd_diff_in(A, B, C, D, 0, 8, 8, m4e3, m4e3, GOOD_P, GOOD_A, 0, 0.3) == lb.ERR_FORMAT
    assert lb.lba_gemm_bwd_diff_in(A, B, C, D, 0, 8, 8, (3, 3, 3), m4e3, GOOD_P, GOOD_A, 0, 0.5) == lb.ERR_FORMAT
    assert lb.lba_gemm_bwd_diff_in(A, B, C, None, 8, 8, 8, m4e3, m4e3, GOOD_P, GOOD_A, 0, 0.5) == lb.ERR_NULL


def test_plan_picks_the_scaled_kernel_for_the_paper_formats():
    # 12-bit accumulator M7E4 with an M7E5 product format (Sec. 3.1), floor and nearest-even
    for rnd in (0, 1):
        for bp, ba in ((15, 7), (-1, -9), (12, 10), (9, 7)):
            p = lb.lba_plan_query(100352, 64, 576, (5, 7, bp, rnd), (4, 7, ba, rnd))
            assert p["kernel"] == 0 and p["round"] == rnd
            assert p["tile_m"] * p["grid_x"] >= 100352 and p["tile_n"] * p["grid_y"] >= 64
    # a product format that cannot alter any E4M3 product: fused multiply-add path
    assert lb.lba_plan_query(64, 64, 64, (6, 7, 20, 0), (4, 7, 7, 0))["prod_mode"] == 0
    assert lb.lba_plan_query(64, 64, 64, (5, 7, 15, 0), (4, 7, 7, 0))["prod_mode"] == 2   # can saturate
    assert lb.lba_plan_query(64, 64, 64, (5, 7, -1, 0), (4, 7, -9, 0))["prod_mode"] == 1  # can only flush


def test_tail_of_a_mixed_grid_is_cut_finer_where_it_runs_alone():
    # four rounds of 48 x 64 workgroups fill every slot of the chip, the 256 remaining rows follow on an empty chip:
    # 8 x 16 workgroups of 32 x 16 instead of 8 x 8 of 32 x 32 (forward call only)
    qp, qa = (5, 7, 15, 0), (4, 7, 7, 0)
    p = lb.lba_plan_query(12544, 256, 2304, qp, qa)
    assert (p["mid_blocks"], p["tail_blocks"], p["grid_x"]) == (1024, 128, 1152)
    assert lb.lba_plan_query(12544, 256, 2304, qp, qa, 0, 1)["tail_blocks"] == 64
    # twelve rounds of 64 x 64 and 256 tail workgroups: too many to double within one per CU
    assert lb.lba_plan_query(200704, 64, 576, qp, qa)["tail_blocks"] == 256
    # two rounds of 48 x 64 leave slots free: the tail runs beside them
    assert lb.lba_plan_query(3136, 512, 4608, qp, qa)["tail_blocks"] == 32


def test_kernel_names_for_other_operand_formats():
    # lba_plan_kernel_name_in mirrors the launchers: the mixed-grid kernels of the forward and the recompute call, the
    # 4 x 4 kernel on a plain grid, and lba_plan_kernel_name itself for E4M3
    fa, fb, qp, qa = (3, 4, 6), (4, 3, 9), (4, 7, 12, 0), (4, 7, 10, 0)
    assert lb.lba_plan_kernel_name_in(26897, 60, 40, fa, fb, qp, qa) == "lba_fast_in_mixed_kernel<32, 4, 0, 0>"
    assert lb.lba_plan_kernel_name_in(70, 50, 96, fa, fb, qp, qa, with_masks=1) == "lba_fast_bwd_in_mixed_kernel<4, 0, 2>"
    assert lb.lba_plan_kernel_name_in(26897, 60, 40, fa, fb, qp, qa, with_masks=3) == "lba_fast_bwd_in_mixed_kernel<4, 0, 0>"
    assert lb.lba_plan_kernel_name_in(60625, 64, 40, fa, fb, qp, qa, with_masks=1) == "lba_fast_bwd_kernel<4, 0, 0, 2, 1>"
    assert lb.lba_plan_kernel_name_in(4096, 768, 768, (3, 4, 3), (3, 4, 3), (5, 7, 15, 0), (4, 7, 7, 0)) == "lba_fast_kernel<4, 4, 32, 3, 0, 0, 1>"
    e4m3 = (4, 3, 7)
    assert lb.lba_plan_kernel_name_in(26897, 60, 40, e4m3, e4m3, (5, 7, 15, 0), (4, 7, 7, 0)) == \
        lb.lba_plan_kernel_name(26897, 60, 40, (5, 7, 15, 0), (4, 7, 7, 0))
    with pytest.raises(Exception):
        lb.lba_plan_kernel_name_in(64, 64, 64, (3, 3, 3), (3, 4, 3), (5, 7, 15, 0), (4, 7, 7, 0))


def test_plan_falls_back_to_the_general_kernel_when_the_fast_one_is_not_exact():
    q = lb.lba_plan_query
    # nearest-even where one FP32 rounding first would not be exact (M_acc < 7 with inexact sums below R_OF,
    # M_acc > 10, a saturated product off the grid): the scaled kernel's round-to-odd variant (two directed
    # sums, 4 slots more), up to M = 21; the general kernel beyond
    for qp, qa in (((5, 7, 15, 1), (5, 3, 15, 1)), ((5, 7, 15, 1), (4, 11, 7, 1)), ((5, 9, 15, 1), (5, 8, 15, 1)),
                   ((5, 7, 15, 1), (5, 21, 15, 1))):
        plan = q(64, 64, 64, qp, qa)
        assert plan["kernel"] == 0 and (plan["thread_m"], plan["thread_n"]) == (4, 4)
        assert plan["valu_per_mac_x100"] == q(64, 64, 64, qp, (4, 8, 7, 1))["valu_per_mac_x100"] + 400
    assert q(64, 64, 64, (5, 7, 15, 1), (5, 22, 15, 1))["kernel"] == 1
    assert q(64, 64, 64, (5, 7, 15, 1), (5, 3, 15, 1), with_masks=1)["kernel"] == 1
    assert q(64, 64, 64, (5, 9, 15, 1), (4, 8, 7, 1))["kernel"] == 0      # same product, but then every sum saturates
    assert q(64, 64, 64, (5, 7, 40, 1), (4, 7, -9, 1))["kernel"] == 1     # products far below R_UF of Q_acc
    assert q(64, 64, 64, (5, 4, 15, 1), (4, 7, 7, 1))["prod_mode"] == 6   # product mantissa rounded to nearest (and clamped): still the scaled kernel
    assert q(64, 64, 64, (5, 4, 15, 1), (4, 7, 7, 1), with_masks=1)["kernel"] == 1   # ... the recompute call: general kernel
    assert q(64, 64, 64, (5, 4, 15, 0), (4, 7, 7, 0), with_masks=1)["kernel"] == 0   # truncated products: scaled recompute kernel
    assert q(64, 64, 64, (5, 4, 15, 0), (4, 7, 7, 0), order=1, with_masks=1)["kernel"] == 1   # ... not for the chunked order
    assert q(64, 64, 64, (5, 4, 15, 0), (4, 7, 7, 0))["prod_mode"] == 4   # ... truncated (and clamped): a bit mask in the scaled kernel
    assert q(64, 64, 64, (6, 4, 20, 0), (4, 7, 7, 0))["prod_mode"] == 3   # ... truncated, cannot saturate
    assert q(64, 64, 64, (5, 7, 15, 0), (4, 3, 7, 0))["kernel"] == 0      # floor is exact at any M
    assert q(64, 64, 64, (5, 7, 15, 0), (7, 23, 64, 0))["kernel"] == 0
    # no-underflow flag: still the scaled kernel; a flagged Q_prod that cannot saturate is the identity
    assert q(64, 64, 64, (5, 7, -1, 0x100), (4, 7, -9, 0x100))["prod_mode"] == 0
    assert q(64, 64, 64, (5, 7, 15, 0x101), (4, 7, 7, 0x101))["kernel"] == 0
    # ... unless R_OF of the accumulator would be a denormal in the flag's fixed domain (2^-60): general kernel
    assert q(64, 64, 64, (5, 7, 15, 0), (4, 7, 90, 0x100))["kernel"] == 1
    assert q(64, 64, 64, (5, 7, 15, 0), (2, 7, 126, 0x100))["kernel"] == 1
    assert q(64, 64, 64, (5, 7, 15, 1), (4, 7, 90, 0x101), order=1)["kernel"] == 1
    assert q(64, 64, 64, (5, 7, 15, 0), (4, 7, 81, 0x100))["kernel"] == 0      # top exponent -66: still a normal there
    assert q(64, 64, 64, (5, 7, 15, 0), (4, 7, 82, 0x100))["kernel"] == 1
    # ... or a Q_prod that saturates every product at a value below 2^-66 would put the sums among them
    assert q(64, 64, 64, (4, 3, 101, 1), (4, 8, -57, 0x101), order=1)["kernel"] == 1
    assert q(64, 64, 64, (4, 3, 81, 0), (4, 8, -57, 0x100))["kernel"] == 0      # R_OF of Q_prod about 2^-65: fine
    assert q(64, 64, 64, (4, 3, 82, 0), (4, 8, -57, 0x100))["kernel"] == 1
    # recompute call: scaled-domain kernel for floor when Q_prod can underflow, else the general one
    assert q(64, 64, 64, (5, 7, 15, 0), (4, 7, 7, 0), with_masks=1)["kernel"] == 0
    assert q(64, 64, 64, (5, 7, 15, 1), (4, 7, 7, 1), with_masks=1)["kernel"] == 0      # nearest-even: where rounding twice is exact
    assert q(64, 64, 64, (5, 7, 15, 1), (4, 11, 7, 1), with_masks=1)["kernel"] == 1     # ... not beyond 10 mantissa bits
    assert q(64, 64, 64, (5, 7, 15, 1), (4, 7, 7, 1), with_masks=2)["kernel"] == 0      # the DIFF plane likewise
    assert q(64, 64, 64, (5, 7, 15, 1), (5, 3, 15, 1), with_masks=2)["kernel"] == 1
    assert q(64, 64, 64, (5, 7, 17, 0), (4, 7, -7, 0), with_masks=1)["kernel"] == 1     # products up to 2^24 below R_UF of Q_acc
    assert q(64, 64, 64, (5, 7, 17, 0), (4, 7, -6, 0), with_masks=1)["kernel"] == 0
    assert q(64, 64, 64, (6, 7, 20, 0), (4, 7, 7, 0), with_masks=1)["kernel"] == 1
    # chunked order, forward and recompute
    assert q(64, 64, 64, (5, 7, 15, 0), (4, 7, 7, 0), order=1)["kernel"] == 0
    assert q(64, 64, 64, (5, 7, 15, 1), (5, 3, 15, 1), order=1)["kernel"] == 0
    assert q(64, 64, 64, (5, 7, 15, 0), (4, 7, 7, 0), order=1, with_masks=1)["kernel"] == 0
    assert q(64, 64, 64, (5, 7, 15, 1), (4, 7, 7, 1), order=1, with_masks=1)["kernel"] == 0
    assert q(64, 64, 64, (5, 7, 15, 1), (5, 3, 15, 1), order=1, with_masks=1)["kernel"] == 1
    # nearest-even below 7 mantissa bits: scaled kernel only when every inexact FP32 sum overflows
    assert q(64, 64, 64, (5, 7, 15, 1), (4, 3, 7, 1))["kernel"] == 0
    assert q(64, 64, 64, (5, 7, 15, 1), (4, 6, 7, 1))["kernel"] == 0
    assert q(64, 64, 64, (5, 7, 15, 1), (5, 6, 15, 1))["valu_per_mac_x100"] == 1300     # round-to-odd variant
    assert q(64, 64, 64, (4, 9, 7, 1), (4, 6, 7, 1))["kernel"] == 0       # a saturated product has 10 bits: still clear of midpoints
    base = q(64, 64, 64, (4, 9, 7, 1), (4, 9, 7, 1))["valu_per_mac_x100"]
    assert q(64, 64, 64, (4, 12, 7, 1), (4, 9, 7, 1))["valu_per_mac_x100"] == base + 400   # 13 + 9 bits: an inexact sum could reach one
    with pytest.raises(lb.LbaError):
        q(64, 64, 64, (5, 7, 15, 0), (4, 7, 7, 0), order=2)


def test_workspace_sizes_of_the_gradient_calls():
    # host arithmetic only: the size from which split sums are combined in the workspace is the maps plus whole
    # slices, a multiple of 256, never below the minimum, equal to it where no sum is split, 0 where the minimum is 0
    for M, N, K in [(300, 200, 600), (3000, 24, 300), (40, 2100, 72), (1500, 64, 147), (50176, 512, 128), (802816, 64, 147),
                    (64, 1000, 2048), (130, 68, 260), (32, 28, 260), (4096, 4096, 4096), (1, 4, 1)]:
        small, fast = lb.lba_grad_workspace_bytes(M, N, K), lb.lba_grad_workspace_bytes_fast(M, N, K)
        assert small > 0 and fast >= small and fast % 256 == 0, (M, N, K, small, fast)
        extra = fast - small
        # slices of one product: a whole number (2 or more) of outputs-sized blocks of floats, rounded up to 256 bytes
        blocks = [extra // (4 * r * K) for r in (M, N) if extra >= 8 * r * K and (extra - 255 <= (extra // (4 * r * K)) * 4 * r * K <= extra)]
        assert extra == 0 or blocks, (M, N, K, extra)
    assert lb.lba_grad_workspace_bytes_fast(4096, 4096, 4096) == lb.lba_grad_workspace_bytes(4096, 4096, 4096)
    assert lb.lba_grad_workspace_bytes_fast(32, 28, 260) == lb.lba_grad_workspace_bytes(32, 28, 260)     # one step of s either way
    extra = lb.lba_grad_workspace_bytes_fast(50176, 512, 128) - lb.lba_grad_workspace_bytes(50176, 512, 128)
    assert extra > 0 and extra % (512 * 128 * 4) == 0          # whole slices of dW [512, 128]; dX [50176, 128] fills the chip uncut
    for bad in [(0, 8, 8), (8, 0, 8), (8, 8, 0), (-1, 8, 8), (1 << 31, 8, 8), (1 << 20, 1 << 11, 64)]:
        assert lb.lba_grad_workspace_bytes_fast(*bad) == 0 and lb.lba_grad_workspace_bytes(*bad) == 0
