"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol the public header declares, rejects bad arguments before launching
anything, and its host-side Eq. 2 agrees with the oracle bit for bit."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2505_20932_amd as P
from paper_2505_20932_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "cwac.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^(?:cwac_status|size_t|int32_t|const char \*)\s*\*?\s*(\w+)\s*\(", text, flags=re.M)
    return sorted(set(names))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2505_20932_amd import build
        build.build_library(verbose=False)
    return binding.lib()


def test_every_declared_symbol_is_exported(lib):
    declared = _declared_functions()
    assert "qlinear_cwac_forward" in declared and "cwac_calibrate_stats" in declared
    assert "cwac_solve" in declared and "cwac_fold" in declared
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in cwac.h but not exported"
    assert sorted(binding.EXPORTS) == declared
    for name in declared:                       # the Python binding carries the same names
        if name != "cwac_status_string":
            assert hasattr(P, name) or hasattr(binding, name)


def test_status_strings(lib):
    for code in range(0, -7, -1):
        s = lib.cwac_status_string(code)
        assert s and s != b"unknown status"
    assert lib.cwac_status_string(-99) == b"unknown status"


def test_struct_layout_matches_header():
    assert C.sizeof(binding.cwac_qparams) == 32
    assert binding.cwac_qparams.s_r.offset == 16 and binding.cwac_qparams.qmax.offset == 28


def test_sizes(lib):
    assert P.cwac_stats_bytes(1152) == 64 + 48 * 1152
    assert P.cwac_stats_bytes(0) == 0
    assert P.cwac_calibrate_stats_workspace(6304, 1152) >= 5 * 8 * 1152
    assert P.cwac_range_workspace(10) > 0


def test_argument_errors_launch_nothing(lib):
    qp = binding.make_qparams()
    null = None
    # NULL pointers
    assert lib.qlinear_cwac_forward(null, 16, null, 16, 1, 1, 16, C.byref(qp), null, null, null,
                                    null, 0, null, 1, null) == -1
    assert lib.cwac_calibrate_stats(null, 4, null, 4, 4, 4, null, null, 0, null) == -1
    assert lib.cwac_fold(null, null, null, null, null, 4, C.byref(qp), null, null, null, null,
                         null) == -1
    assert lib.cwac_solve(null, 4, 1e-12, null, null, null, null, null) == -1
    # shapes / alignment / modes are checked with fake (never dereferenced) addresses
    a = C.c_void_p(4096)
    assert lib.qlinear_cwac_forward(a, 24, a, 24, 4, 4, 24, C.byref(qp), a, a, null, null, 0, a, 4,
                                    null) == -2          # k % 16 != 0
    assert lib.qlinear_cwac_forward(a, 32, a, 32, 4, 4, 32, C.byref(qp), a, a, null, null, 7, a, 4,
                                    null) == -4          # unknown out_kind
    assert lib.qlinear_cwac_forward(C.c_void_p(4100), 32, a, 32, 4, 4, 32, C.byref(qp), a, a, null,
                                    null, 0, a, 4, null) == -3   # misaligned x_q
    assert lib.qlinear_cwac_forward(a, 32, a, 32, 4, 4, 65536, C.byref(qp), a, a, null, null, 0, a,
                                    4, null) == -2       # k too large for int32 accumulation
    bad = binding.make_qparams(mode=0, act_per_token=True)
    assert lib.cwac_fold(null, null, a, null, a, 4, C.byref(bad), a, a, null, null, null) == -4
    assert lib.cwac_calibrate_stats(a, 4, a, 4, 8, 4, a, null, 0, null) == -5   # no workspace
    assert lib.cwac_calibrate_stats(a, 4, a, 4, 0, 4, a, null, 0, null) == 0    # empty batch: no-op
    assert lib.cwac_calibrate_stats(a, 2, a, 4, 8, 4, a, a, 1 << 20, null) == -2  # ld < c_out


def test_argument_errors_of_the_widened_entry_points(lib):
    qp = binding.make_qparams()
    null = None
    a = C.c_void_p(4096)
    big = 1 << 30
    # fused calibration: NULLs, shapes outside the large-tile kernel, alignment, workspace
    f = lib.qlinear_cwac_calibrate_fused
    assert f(null, 128, a, 128, 256, 256, 128, a, null, null, null, a, 256, a, a, big, null) == -1
    assert f(a, 128, a, 128, 255, 256, 128, a, null, null, null, a, 256, a, a, big, null) == -2
    assert f(a, 128, a, 128, 256, 258, 128, a, null, null, null, a, 260, a, a, big, null) == -2  # n % 4
    assert f(a, 192, a, 192, 256, 256, 192, a, null, null, null, a, 256, a, a, big, null) == -2  # k % 128
    assert f(a, 128, a, 128, 256, 256, 128, a, null, null, null, a, 258, a, a, big, null) == -3  # ld_full % 4
    assert f(a, 128, a, 128, 256, 256, 128, a, null, null, null, a, 256, a, a, 64, null) == -5
    assert P.cwac_calibrate_fused_workspace(16384, 4096) == 64 * 5 * 4096 * 8 + 4096 * 4
    # integer-only form
    g = lib.cwac_fold_fixed_point
    assert g(null, null, null, null, null, 4, C.byref(qp), null, null, null, null, null) == -1
    per_token = binding.make_qparams(mode=1, act_per_token=True)
    assert g(null, null, a, null, a, 4, C.byref(per_token), a, a, a, null, null) == -4
    h = lib.qlinear_cwac_forward_fixed_point
    assert h(a, 32, a, 32, 4, 4, 32, C.byref(qp), null, a, null, a, 4, null) == -1   # no multiplier
    assert h(a, 24, a, 24, 4, 4, 24, C.byref(qp), a, a, null, a, 4, null) == -2      # k % 16
    assert h(a, 32, a, 32, 4, 4, 32, C.byref(qp), a, a, null, a, 2, null) == -2      # ldo < n
    # b-bit quantizers
    q = lib.cwac_quantize_act_bits
    assert q(a, 8, 4, 8, 1.0, 0, 9, a, 8, null) == -2          # bits out of range
    assert q(a, 8, 4, 8, 1.0, 8, 4, a, 8, null) == -2          # zero-point outside the 4-bit range
    assert q(a, 8, 0, 8, 1.0, 0, 4, a, 8, null) == 0           # no rows: no-op
    assert lib.cwac_quantize_rows_sym_bits(a, 8, 4, 8, 1, a, a, 8, null) == -2
    # diagnostic
    assert lib.cwac_mfma_probe(null, 10, 1, a, null) == -1
    assert lib.cwac_mfma_probe(a, 0, 1, a, null) == -2
    assert lib.cwac_hbm_read_probe(null, 4096, 1, a, null) == -1
    assert lib.cwac_hbm_read_probe(a, 8, 1, a, null) == -2
    assert lib.cwac_hbm_read_probe(C.c_void_p(4100), 4096, 1, a, null) == -3
    assert lib.cwac_mfma_probe_f16(null, 10, 1, a, null) == -1
    assert lib.cwac_mfma_probe_f16(a, 10, 0, a, null) == -2
    assert lib.cwac_mfma_probe_f16(C.c_void_p(4100), 10, 1, a, null) == -3


def test_argument_errors_of_the_weight_only_entry_points(lib):
    null = None
    a = C.c_void_p(4096)
    q = lib.cwac_w4_quantize_groupwise
    assert q(null, 128, 4, 128, a, a, a, null) == -1
    assert q(a, 192, 4, 192, a, a, a, null) == -2            # k % 128
    assert q(a, 64, 4, 128, a, a, a, null) == -2             # ldw < k
    assert q(C.c_void_p(4100), 128, 4, 128, a, a, a, null) == -3
    pk = lib.cwac_w4_pack
    assert pk(a, a, a, 48, 128, a, a, null) == -2            # n % 32
    assert pk(a, a, a, 64, 128, null, a, null) == -1
    assert pk(a, a, a, 64, 128, C.c_void_p(4104), a, null) == -3
    assert P.cwac_w4_packed_w_bytes(4096, 11008) == 4096 * 11008 // 2
    fo = lib.cwac_fold_weight_only
    assert fo(a, null, null, 8, a, a, null) == -4            # alpha without beta
    assert fo(null, null, null, 8, null, a, null) == -1
    f = lib.qlinear_w4a16_cwac_forward
    assert f(null, 128, a, a, 1, 256, 128, null, null, 3, a, 256, null) == -1
    assert f(a, 128, a, a, 1, 128, 128, null, null, 3, a, 128, null) == -2     # n < 256
    assert f(a, 128, a, a, 1, 272, 128, null, null, 3, a, 272, null) == -2     # n % 32
    assert f(a, 192, a, a, 1, 256, 192, null, null, 3, a, 256, null) == -2     # k % 128
    assert f(a, 128, a, a, 1, 256, 128, null, null, 0, a, 256, null) == -4     # int8 output: not this layer
    assert f(a, 132, a, a, 2, 256, 128, null, null, 3, a, 256, null) == -3     # ldx % 8
    assert f(a, 128, a, a, 2, 256, 128, null, null, 3, a, 260, null) == -3     # output pitch not 16-byte
    assert f(a, 128, a, a, 0, 256, 128, null, null, 3, a, 256, null) == -2     # no rows


def test_argument_errors_of_the_convolution_entry_point(lib):
    qp = binding.make_qparams(z_x=3)
    null = None
    a = C.c_void_p(4096)
    f = lib.qconv2d_cwac_forward
    ok_tail = (C.byref(qp), a, a, null, 0, a, 64, null)
    assert f(null, a, 1, 8, 8, 16, 64, 3, 3, 1, 1, *ok_tail) == -1
    assert f(a, a, 1, 8, 8, 24, 64, 3, 3, 1, 1, *ok_tail) == -2          # c_in % 16
    assert f(a, a, 1, 8, 8, 16, 64, 3, 3, 1, 3, *ok_tail) == -2          # pad >= kernel
    assert f(a, a, 1, 2, 2, 16, 64, 5, 5, 1, 1, *ok_tail) == -2          # image smaller than the window
    assert f(a, a, 1, 8, 8, 4096, 64, 3, 3, 1, 1, *ok_tail) == -2        # kh * kw * c_in > 32768
    assert f(a, a, 1, 8, 8, 16, 64, 3, 3, 0, 1, *ok_tail) == -2          # stride 0
    assert f(C.c_void_p(4100), a, 1, 8, 8, 16, 64, 3, 3, 1, 1, *ok_tail) == -3
    assert f(a, a, 1, 8, 8, 16, 64, 3, 3, 1, 1, C.byref(qp), a, a, null, 7, a, 64, null) == -4
    assert f(a, a, 1, 8, 8, 16, 64, 3, 3, 1, 1, C.byref(qp), a, a, null, 0, a, 32, null) == -2   # ldo < c_out
    per_token = binding.make_qparams(mode=1, act_per_token=True)
    assert f(a, a, 1, 8, 8, 16, 64, 3, 3, 1, 1, C.byref(per_token), a, a, a, 0, a, 64, null) == -4
    assert f(a, a, 1, 8, 8, 16, 64, 3, 3, 1, 1, null, a, a, null, 0, a, 64, null) == -1          # qp required


def test_mode_checks_of_the_forward(lib):
    """A qp that contradicts the vectors defining the epilogue is refused before any launch."""
    null = None
    a = C.c_void_p(4096)
    f = lib.qlinear_cwac_forward
    per_tensor = binding.make_qparams()
    per_token = binding.make_qparams(mode=1, act_per_token=True)
    fp_bias = binding.make_qparams(mode=1)
    #         x  ldx w ldw  m  n   k   qp                   mult off fbias sxrow kind out ldo
    assert f(a, 32, a, 32, 4, 4, 32, C.byref(per_token), a, a, a, null, 0, a, 4, null) == -4   # folded per token, no row scales
    assert f(a, 32, a, 32, 4, 4, 32, C.byref(per_tensor), a, a, null, a, 0, a, 4, null) == -4  # row scales, per-tensor qp
    assert f(a, 32, a, 32, 4, 4, 32, C.byref(fp_bias), a, a, null, null, 0, a, 4, null) == -4  # fp-bias fold, no fbias
    assert f(a, 32, a, 32, 4, 4, 32, C.byref(per_token), a, a, null, null, 1, a, 4, null) == -4  # fp32 output too
    h = lib.qlinear_cwac_forward_fixed_point
    assert h(a, 32, a, 32, 4, 4, 32, C.byref(per_token), a, a, null, a, 4, null) == -4
    assert h(a, 32, a, 32, 4, 4, 32, C.byref(fp_bias), a, a, null, a, 4, null) == -4
    ft = lib.qlinear_cwac_forward_table
    assert ft(a, 64, a, 64, 256, 256, 64, C.byref(per_token), a, null, a, a, 256, null) == -4


def test_tuning_is_validated_and_no_environment_variable_is_read(lib):
    null = None
    a = C.c_void_p(4096)
    qp = binding.make_qparams()
    for bad in (binding.make_tuning(kernel=7), binding.make_tuning(shape=7), binding.make_tuning(shape=-1),
                binding.make_tuning(stats_waves=3), binding.make_tuning(persist_loaders=2),
                binding.make_tuning(persist_loaders=16)):
        assert lib.qlinear_cwac_forward_ex(a, 32, a, 32, 4, 4, 32, C.byref(qp), a, a, null, null, 0, a, 4,
                                           C.byref(bad), null) == -4
        assert lib.cwac_forward_kernel_for(4, 4, 32, 32, 32, 0, C.byref(bad)) == -4
    for bad in (binding.make_tuning(w4_tile=64), binding.make_tuning(w4_tile=512), binding.make_tuning(w4_small_waves=16),
                binding.make_tuning(w4_small_depth=5), binding.make_tuning(w4_small_depth=1)):
        assert lib.qlinear_w4a16_cwac_forward_ex(a, 128, a, a, 1, 256, 128, null, null, 3, a, 256, C.byref(bad),
                                                 null) == -4
    # the dispatcher's choice is a function of sizes and the tuning argument alone
    want = binding.cwac_forward_kernel_for(16384, 4096, 4096, 4096, 4096)
    assert want == binding.CWAC_KERNEL_DIRECT_LDS
    os.environ["CWAC_FWD_TILE"] = "64"
    try:
        assert binding.cwac_forward_kernel_for(16384, 4096, 4096, 4096, 4096) == want
    finally:
        del os.environ["CWAC_FWD_TILE"]
    assert binding.cwac_forward_kernel_for(16384, 4096, 4096, 4096, 4096,
                                     tuning=binding.make_tuning(kernel=64)) == 64
    src = os.path.join(ROOT, "paper_2505_20932_amd", "csrc")
    for name in os.listdir(src):
        assert "getenv" not in open(os.path.join(src, name)).read(), name


def test_pitches_beyond_the_32_bit_lane_offsets_leave_the_direct_to_lds_kernel(lib):
    """The direct-to-LDS kernel forms row * pitch + chunk (rows < 256) in 32 bits; any pitch >= k is a
    legal argument, so pitches above 2^24 must take the generic kernel (64-bit row addresses)."""
    lds, g256 = binding.CWAC_KERNEL_DIRECT_LDS, binding.CWAC_KERNEL_GENERIC_256
    big = (1 << 24) + 16
    assert binding.cwac_forward_kernel_for(16384, 4096, 4096, 4096, 4096) == lds
    assert binding.cwac_forward_kernel_for(16384, 4096, 4096, 1 << 24, 1 << 24) == lds      # 255 * 2^24 + 128 < 2^32
    assert binding.cwac_forward_kernel_for(16384, 4096, 4096, big, 4096) == g256
    assert binding.cwac_forward_kernel_for(16384, 4096, 4096, 4096, big) == g256
    forced = binding.make_tuning(kernel=lds)
    assert binding.cwac_forward_kernel_for(16384, 4096, 4096, big, 4096, tuning=forced) == g256  # forcing cannot override it
    assert binding.cwac_forward_kernel_for(16384, 4096, 4096, 4096, 4096, tuning=forced) == lds
    # entry points that have no generic form refuse such pitches
    a = C.c_void_p(4096)
    null = None
    f = lib.qlinear_cwac_calibrate_fused
    assert f(a, big, a, 128, 256, 256, 128, a, null, null, null, a, 256, a, a, 1 << 30, null) == -2
    assert f(a, 128, a, big, 256, 256, 128, a, null, null, null, a, 256, a, a, 1 << 30, null) == -2
    assert f(a, 128, a, 128, 256, 256, 128, a, null, null, null, a, (1 << 26) + 4, a, a, 1 << 30, null) == -2
    # first-batch statistics: same checks as the accumulating call, and a first batch has rows
    g = lib.cwac_calibrate_stats_first
    assert g(null, 4, null, 4, 4, 4, null, null, 0, null) == -1
    assert g(a, 4, a, 4, 0, 4, a, a, 1 << 20, null) == -2
    assert g(a, 4, a, 4, 8, 4, a, null, 0, null) == -5


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_eq2_host_function_matches_oracle(orc, lib):
    x = synth.normal(5, 0, 1000).numpy()
    cases = [(-64.0, 191.0), (float(x.min()), float(x.max())), (0.0, 0.0), (-1e-3, 7.5),
             (3.0, 4.0), (-9.0, -2.0)]
    for bits in (4, 6, 8):
        for mn, mx in cases:
            s, z = P.cwac_qparams_from_range(mn, mx, bits)
            s0, z0 = orc.qparams_asym(mn, mx, bits)
            assert np.float32(s) == s0 and z == z0, (mn, mx, bits)


def test_argument_errors_of_the_block_glue_entry_points(lib):
    null = None
    a = C.c_void_p(4096)
    ln = lib.vit_residual_ln_quant
    #        h  ldh  r  ldr  s_r z_r h_out ldho gamma beta eps   s_x z_x x_q ldxq m  c
    assert ln(null, 64, a, 64, 1.0, 0, a, 64, a, a, 1e-6, 1.0, 0, a, 64, 4, 64, null) == -1
    assert ln(a, 64, null, 0, 1.0, 0, null, 0, a, a, 1e-6, 1.0, 0, null, 0, 4, 64, null) == -1  # nothing to do
    assert ln(a, 64, null, 0, 1.0, 0, null, 0, null, a, 1e-6, 1.0, 0, a, 64, 4, 64, null) == -1  # no gamma
    assert ln(a, 64, null, 0, 1.0, 0, a, 64, a, a, 1e-6, 1.0, 0, a, 64, 4, 64, null) == -4      # h_out without r
    assert ln(a, 64, a, 64, 1.0, 0, a, 64, a, a, 1e-6, 0.0, 0, a, 64, 4, 64, null) == -4        # s_x = 0
    assert ln(a, 60, a, 64, 1.0, 0, a, 64, a, a, 1e-6, 1.0, 0, a, 64, 4, 60, null) == -2        # c % 8
    assert ln(a, 4096, a, 4096, 1.0, 0, a, 4096, a, a, 1e-6, 1.0, 0, a, 4096, 4, 4096, null) == -2  # c > 2048
    assert ln(a, 32, a, 64, 1.0, 0, a, 64, a, a, 1e-6, 1.0, 0, a, 64, 4, 64, null) == -2        # ldh < c
    assert ln(a, 68, a, 64, 1.0, 0, a, 64, a, a, 1e-6, 1.0, 0, a, 64, 4, 64, null) == -3        # ldh % 8
    assert ln(a, 64, C.c_void_p(4100), 64, 1.0, 0, a, 64, a, a, 1e-6, 1.0, 0, a, 64, 4, 64, null) == -3
    gt = lib.vit_gelu_table
    assert gt(1.0, 0, 1.0, 0, null, null) == -1
    assert gt(0.0, 0, 1.0, 0, a, null) == -4
    tl = lib.vit_table_lookup
    assert tl(a, 64, null, a, 64, 4, 64, null) == -1
    assert tl(a, 64, a, a, 64, 4, 40, null) == -2            # n % 16
    assert tl(a, 64, a, a, 32, 4, 64, null) == -2            # ld_out < n
    assert tl(a, 72, a, a, 64, 4, 64, null) == -3            # ld_in % 16
    at = lib.vit_attention_int8
    #        r  ld   s    z  batch tokens heads d  bias ldb s_a z_a a  lda
    assert at(null, 192, 1.0, 0, 1, 16, 1, 64, null, 0, 1.0, 0, a, 64, null) == -1
    assert at(a, 192, 1.0, 0, 1, 4097, 1, 64, null, 0, 1.0, 0, a, 64, null) == -2   # more tokens than the longest sequence
    assert at(a, 192, 1.0, 0, 1, 16, 1, 48, null, 0, 1.0, 0, a, 64, null) == -2    # head width other than 64 or 32
    assert at(a, 128, 1.0, 0, 1, 16, 1, 64, null, 0, 1.0, 0, a, 64, null) == -2    # ld < 3 c
    assert at(a, 192, 1.0, 0, 1, 16, 1, 64, null, 0, 1.0, 0, a, 32, null) == -2    # lda < c
    assert at(a, 192, 1.0, 0, 1, 16, 1, 64, a, 16, 1.0, 0, a, 64, null) == -2      # bias rows not padded to a key tile
    assert at(a, 192, 1.0, 0, 1, 16, 1, 64, C.c_void_p(4100), 32, 1.0, 0, a, 64, null) == -3
    assert at(a, 192, 0.0, 0, 1, 16, 1, 64, null, 0, 1.0, 0, a, 64, null) == -4
    assert at(a, 192, 1.0, 200, 1, 16, 1, 64, null, 0, 1.0, 0, a, 64, null) == -4  # zero-point outside int8
    assert at(a, 196, 1.0, 0, 1, 16, 1, 64, null, 0, 1.0, 0, a, 64, null) == -3    # ld % 8
    assert at(a, 192, 1.0, 0, 1, 16, 1, 64, null, 0, 1.0, 0, C.c_void_p(4104), 64, null) == -3
    ft = lib.qlinear_cwac_forward_table
    qp = binding.make_qparams()
    assert ft(a, 64, a, 64, 256, 256, 64, C.byref(qp), a, null, null, a, 256, null) == -1     # no table
    assert ft(a, 64, a, 64, 256, 250, 64, C.byref(qp), a, null, a, a, 256, null) == -2        # n % 16
    assert ft(a, 64, a, 64, 256, 256, 64, C.byref(qp), a, null, a, a, 264, null) == -3        # ldo % 16
    assert ft(a, 64, a, 64, 256, 256, 64, C.byref(qp), a, null, C.c_void_p(4098), a, 256, null) == -3
    assert lib.vit_encoder_w8a8_forward(null, 1, a, a, a, 1 << 30, null) == -1
    bp = binding.vit_block_params()
    assert lib.vit_encoder_w8a8_forward(C.byref(bp), 0, a, a, a, 1 << 30, null) == -2   # no blocks
    assert lib.vit_encoder_w8a8_forward(C.byref(bp), 1, a, a, a, 1 << 30, null) == -1   # empty parameter block
