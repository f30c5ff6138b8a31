"""CPU-side checks of the C-ABI library: it loads, exports what the header declares, and
rejects bad arguments on the host before any launch (no GPU needed, no compute calls)."""
import ctypes as C
import os
import re

import pytest

import paper_2509_21302_amd as q

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "qvggt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qvggt_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = q.load_library()
    declared = _declared_symbols()
    assert declared, "no declarations found in include/qvggt.h"
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in qvggt.h but not exported"
    assert sorted(q.EXPORTS) == declared
    # every entry point has its C signature registered with ctypes: without it a 64-bit pointer would be passed as a C int
    for name in declared:
        assert getattr(lib, name).argtypes is not None, f"{name}: no argtypes in the binding"


def test_header_is_plain_c():
    """The boundary is a C header: no C++ or HIP types, nothing but <stddef.h> / <stdint.h>; a C99 compiler accepts it as it is."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c",
                        os.path.join(ROOT, "include", "qvggt.h")], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_status_strings():
    assert q.qvggt_status_string(0) == "QVGGT_OK"
    for s in range(1, 8):
        assert q.qvggt_status_string(s).startswith("QVGGT_ERR_")
    assert "unknown" in q.qvggt_status_string(99)


def test_workspace_bytes():
    assert q.qvggt_workspace_bytes(1374, 3072, 1024) >= 1374 * 512 + 1374 * 4
    assert q.qvggt_workspace_bytes(0, 3072, 1024) > 0
    assert q.qvggt_workspace_bytes(10, 3072, 1000) == 0      # K not a power of two
    assert q.qvggt_workspace_bytes(10, 3070, 1024) == 0      # N not a multiple of 16
    for K in (768, 1536, 3072, 6144, 1280, 2560, 5120, 1792, 3584):     # sizes 2^n * m with a Paley factor
        assert q.qvggt_workspace_bytes(10, 32, K) > 0
    for K in (1408, 2304, 7168, 384, 96):
        assert q.qvggt_workspace_bytes(10, 32, K) == 0
    assert q.qvggt_workspace_bytes(-1, 3072, 1024) == 0


OK, NULL, SHAPE, ALIGN, DTYPE, WORKSPACE, ARG = 0, 1, 2, 3, 4, 5, 6
P = 0x10000  # a fake, aligned, non-NULL device address: validation failures return before any use


def test_argument_validation_needs_no_gpu():
    lib = q.load_library()
    # shapes
    assert lib.qvggt_rotate_smooth_quant(P, 0, 4, 1000, None, None, P, P, None) == SHAPE
    assert lib.qvggt_rotate_smooth_quant(P, 0, 4, 64, None, None, P, P, None) == SHAPE
    assert lib.qvggt_rotate_smooth_quant(P, 0, 4, 16384, None, None, P, P, None) == SHAPE
    assert lib.qvggt_rotate_smooth_quant(P, 0, -1, 1024, None, None, P, P, None) == SHAPE
    assert lib.qvggt_w4a4_gemm(P, P, P, P, None, 4, 100, 1024, P, None, None) == SHAPE
    assert lib.qvggt_w4a4_gemm(P, P, P, P, None, 4, 0, 1024, P, None, None) == SHAPE
    assert lib.qvggt_prep_weights(P, 0, 24, 1024, None, None, C.c_float(0.5), P, P, P, None) == SHAPE
    # dtype
    assert lib.qvggt_rotate_smooth_quant(P, 7, 4, 1024, None, None, P, P, None) == DTYPE
    assert lib.qvggt_prep_weights(P, -1, 32, 1024, None, None, C.c_float(0.5), P, P, P, None) == DTYPE
    assert lib.qvggt_linear(P, 2, 4, 32, 1024, None, None, P, P, None, P, P, 1 << 20, None) == DTYPE
    # NULL pointers
    assert lib.qvggt_rotate_smooth_quant(None, 0, 4, 1024, None, None, P, P, None) == NULL
    assert lib.qvggt_rotate_smooth_quant(P, 0, 4, 1024, None, None, None, P, None) == NULL
    assert lib.qvggt_w4a4_gemm(P, None, P, P, None, 4, 32, 1024, P, None, None) == NULL
    assert lib.qvggt_prep_weights(P, 0, 32, 1024, None, None, C.c_float(0.5), P, None, P, None) == NULL
    assert lib.qvggt_linear(P, 0, 4, 32, 1024, None, None, P, P, None, P, None, 1 << 20, None) == NULL
    assert lib.qvggt_rotated_col_absmax(P, 0, 4, 1024, None, None, None) == NULL
    assert lib.qvggt_pack_int4(None, 4, 1024, P, None) == NULL
    # alignment
    assert lib.qvggt_rotate_smooth_quant(P + 2, 0, 4, 1024, None, None, P, P, None) == ALIGN
    assert lib.qvggt_w4a4_gemm(P, P, P, P, P + 8, 4, 32, 1024, P, None, None) == ALIGN
    assert lib.qvggt_unpack_int4(P, 4, 1024, P + 1, None) == ALIGN
    # alpha
    for bad in (-0.1, 1.5, float("nan"), float("inf")):
        assert lib.qvggt_prep_weights(P, 0, 32, 1024, None, None, C.c_float(bad), P, P, P, None) == ARG
    # static-step variant: same checks, plus the step pointer and the granularity flag
    st = lib.qvggt_rotate_smooth_quant_static
    assert st(P, 0, 4, 1000, None, None, P, 1, P, P, None) == SHAPE
    assert st(P, 9, 4, 1024, None, None, P, 1, P, P, None) == DTYPE
    assert st(P, 0, 4, 1024, None, None, None, 1, P, P, None) == NULL
    assert st(P, 0, 4, 1024, None, None, P, 0, None, P, None) == NULL
    assert st(P, 0, 4, 1024, None, None, P + 2, 0, P, P, None) == ALIGN
    for bad in (-1, 2, 7):
        assert st(P, 0, 4, 1024, None, None, P, bad, P, P, None) == ARG
    assert st(None, 0, 0, 1024, None, None, None, 1, None, None, None) == OK
    # LayerNorm in front: powers of two up to 4096, eps >= 0, optional gamma / beta aligned when given
    lnq = lib.qvggt_layernorm_rotate_smooth_quant
    e5 = C.c_float(1e-5)
    for badk in (1000, 768, 8192, 64):
        assert lnq(P, 0, 4, badk, None, None, e5, None, None, P, P, None) == SHAPE
    assert lnq(P, 7, 4, 1024, None, None, e5, None, None, P, P, None) == DTYPE
    assert lnq(None, 0, 4, 1024, None, None, e5, None, None, P, P, None) == NULL
    assert lnq(P, 0, 4, 1024, None, None, e5, None, None, P, None, None) == NULL
    assert lnq(P, 0, 4, 1024, P + 4, None, e5, None, None, P, P, None) == ALIGN
    assert lnq(P, 0, 4, 1024, None, P + 8, e5, None, None, P, P, None) == ALIGN
    for bad in (-1e-5, float("nan"), float("inf")):
        assert lnq(P, 0, 4, 1024, None, None, C.c_float(bad), None, None, P, P, None) == ARG
    assert lnq(None, 0, 0, 1024, None, None, e5, None, None, None, None, None) == OK
    # asymmetric setting: kernel 1 needs the zero-point buffer and a power-of-two K; the GEMM needs zero points and code sums
    rqa, cs, ga = lib.qvggt_rotate_smooth_quant_asym, lib.qvggt_weight_code_sums, lib.qvggt_w4a4_gemm_asym
    assert rqa(P, 0, 4, 768, None, None, P, P, P, None) == SHAPE
    assert rqa(P, 5, 4, 1024, None, None, P, P, P, None) == DTYPE
    assert rqa(P, 0, 4, 1024, None, None, P, P, None, None) == NULL
    assert rqa(P, 0, 4, 1024, None, None, P, P, P + 4, None) == ALIGN
    assert rqa(None, 0, 0, 1024, None, None, None, None, None, None) == OK
    assert cs(P, 16, 1000, P, None) == SHAPE and cs(P, -1, 1024, P, None) == SHAPE
    assert cs(None, 16, 1024, P, None) == NULL and cs(P, 16, 1024, P + 8, None) == ALIGN and cs(None, 0, 1024, None, None) == OK
    assert ga(P, P, P, P, P, P, None, 4, 100, 1024, P, None) == SHAPE
    assert ga(P, P, None, P, P, P, None, 4, 32, 1024, P, None) == NULL
    assert ga(P, P, P, P, P, None, None, 4, 32, 1024, P, None) == NULL
    assert ga(P, P, P, P, P, P + 4, None, 4, 32, 1024, P, None) == ALIGN
    assert ga(None, None, None, None, None, None, None, 0, 32, 1024, None, None) == OK
    # 6-bit floating-point matrix path: format size, converter, GEMM, direct kernel 1 (bf16, K = 1024 / 2048 / 4096 only)
    assert q.qvggt_e2m3_bytes(1, 1024) == 128 * 768 and q.qvggt_e2m3_bytes(129, 4096) == 256 * 3072 and q.qvggt_e2m3_bytes(5, 1000) == 0
    cv, eg, re, le = lib.qvggt_codes_to_e2m3, lib.qvggt_e2m3_gemm, lib.qvggt_rotate_smooth_quant_e2m3, lib.qvggt_linear_e2m3
    assert cv(P, 4, 1000, P, P, None) == SHAPE and cv(None, 4, 1024, P, P, None) == NULL and cv(P, 4, 1024, P + 4, P, None) == ALIGN
    assert cv(P, 4, 1024, P, None, None) == NULL and cv(None, 0, 1024, None, None, None) == NULL      # the counter of codes -8 is required
    assert cv(P, 4, 1024, P, P + 2, None) == ALIGN and cv(None, 0, 1024, None, P, None) == OK
    assert eg(P, P, P, P, None, 4, 100, 1024, P, None, None) == SHAPE
    assert eg(P, P, None, P, None, 4, 32, 1024, P, None, None) == NULL
    assert eg(P, P, P, P, P + 4, 4, 32, 1024, P, None, None) == ALIGN
    assert eg(None, None, None, None, None, 0, 32, 1024, None, None, None) == OK
    assert re(P, 0, 4, 512, None, None, P, P, None) == SHAPE and re(P, 1, 4, 1024, None, None, P, P, None) == DTYPE
    assert re(P, 0, 4, 1024, None, None, None, P, None) == NULL and re(None, 0, 0, 1024, None, None, None, None, None) == OK
    lne = lib.qvggt_layernorm_rotate_smooth_quant_e2m3
    e6 = C.c_float(1e-6)
    assert lne(P, 0, 4, 2048, None, None, e6, None, None, P, P, None) == SHAPE and lne(P, 1, 4, 1024, None, None, e6, None, None, P, P, None) == DTYPE
    assert lne(P, 0, 4, 1024, None, None, C.c_float(-1.0), None, None, P, P, None) == ARG
    assert lne(P, 0, 4, 1024, None, None, e6, None, None, None, P, None) == NULL and lne(None, 0, 0, 1024, None, None, e6, None, None, None, None, None) == OK
    ae, se, gs = lib.qvggt_rotate_smooth_quant_asym_e2m3, lib.qvggt_rotate_smooth_quant_static_e2m3, lib.qvggt_e2m3_gemm_shifted
    assert ae(P, 0, 4, 512, None, None, P, P, P, None) == SHAPE and ae(P, 1, 4, 1024, None, None, P, P, P, None) == DTYPE
    assert ae(P, 0, 4, 1024, None, None, P, P, None, None) == NULL and ae(None, 0, 0, 1024, None, None, None, None, None, None) == OK
    assert se(P, 0, 4, 1024, None, None, None, 1, P, P, P, None) == NULL and se(P, 0, 4, 1024, None, None, P, 2, P, P, P, None) == ARG
    assert se(P, 0, 4, 128, None, None, P, 1, P, P, P, None) == SHAPE and se(None, 0, 0, 1024, None, None, None, 1, None, None, None, None) == OK
    assert gs(P, P, P, P, P, P, None, 4, 100, 1024, P, None) == SHAPE and gs(P, P, None, P, P, P, None, 4, 32, 1024, P, None) == NULL
    assert gs(P, P, P, P, P, P + 4, None, 4, 32, 1024, P, None) == ALIGN and gs(None, None, None, None, None, None, None, 0, 32, 1024, None, None) == OK
    need6 = q.qvggt_workspace_bytes_e2m3(100, 32, 1024)
    assert need6 >= 128 * 768 + 400
    assert le(P, 0, 100, 32, 1024, None, None, P, P, None, P, P, need6 - 1, None) == WORKSPACE
    assert le(P, 0, 100, 32, 768, None, None, P, P, None, P, P, need6, None) == SHAPE
    assert le(P, 1, 100, 32, 1024, None, None, P, P, None, P, P, need6, None) == DTYPE
    # weight preparation with given factor and steps
    pg = lib.qvggt_prep_weights_given
    assert pg(P, 0, 24, 1024, None, None, None, 4, P, P, P, None) == SHAPE and pg(P, 3, 32, 1024, None, None, None, 4, P, P, P, None) == DTYPE
    assert pg(P, 0, 32, 1024, None, None, None, 3, P, P, P, None) == ARG and pg(P, 0, 32, 1024, None, None, None, 9, P, P, P, None) == ARG
    assert pg(P, 0, 32, 1024, None, None, None, 4, None, P, P, None) == NULL and pg(P, 0, 32, 1024, P + 4, None, None, 4, P, P, P, None) == ALIGN
    assert pg(P, 0, 32, 1024, None, None, P + 8, 4, P, P, P, None) == ALIGN
    # GELU fused into kernel 1: bf16, K = 1024 / 2048 / 4096 only
    for ge in (lib.qvggt_gelu_rotate_smooth_quant, lib.qvggt_gelu_rotate_smooth_quant_e2m3):
        assert ge(P, 0, 4, 512, None, None, P, P, P, None) == SHAPE and ge(P, 1, 4, 1024, None, None, P, P, P, None) == DTYPE
        assert ge(P, 0, 4, 1024, None, None, P, None, P, None) == NULL and ge(P, 0, 4, 1024, None, None, P, P, P + 4, None) == ALIGN
        assert ge(P, 0, 4, 1024, None, None, None, P, P, None) == NULL and ge(P, 0, 4, 1024, None, None, P + 8, P, P, None) == ALIGN     # the table
        assert ge(None, 0, 0, 1024, None, None, None, None, None, None) == OK
    gl = lib.qvggt_gelu_linear_e2m3
    assert gl(P, 0, 100, 32, 1024, None, None, P, P, P, None, P, P, q.qvggt_workspace_bytes_e2m3(100, 32, 1024) - 1, None) == WORKSPACE
    assert gl(P, 0, 100, 32, 768, None, None, P, P, P, None, P, P, 1 << 20, None) == SHAPE and gl(P, 1, 100, 32, 1024, None, None, P, P, P, None, P, P, 1 << 20, None) == DTYPE
    assert gl(P, 0, 100, 32, 1024, None, None, None, P, P, None, P, P, 1 << 20, None) == NULL
    assert lib.qvggt_gelu_table_bytes() == 16384 and lib.qvggt_gelu_table(None, None) == NULL and lib.qvggt_gelu_table(P + 4, None) == ALIGN
    # int8 blocks: format size, converter, direct kernel 1 (bf16, K = 1024 / 2048 / 4096 only), GEMM, whole path
    assert q.qvggt_i8b_bytes(1, 1024) == 128 * 1024 and q.qvggt_i8b_bytes(129, 4096) == 256 * 4096 and q.qvggt_i8b_bytes(5, 1000) == 0
    tb, rb, gb, lb = lib.qvggt_int8_to_blocks, lib.qvggt_rotate_smooth_quant_i8b, lib.qvggt_i8b_gemm, lib.qvggt_linear_i8b
    assert tb(P, 4, 1000, P, None) == SHAPE and tb(None, 4, 1024, P, None) == NULL and tb(P, 4, 1024, P + 4, None) == ALIGN
    assert tb(None, 0, 1024, None, None) == OK
    assert rb(P, 0, 4, 512, None, None, 8, P, P, None) == SHAPE and rb(P, 1, 4, 1024, None, None, 8, P, P, None) == DTYPE
    assert rb(P, 0, 4, 1024, None, None, 9, P, P, None) == ARG and rb(P, 0, 4, 1024, None, None, 8, None, P, None) == NULL
    assert rb(None, 0, 0, 1024, None, None, 8, None, None, None) == OK
    assert gb(P, P, P, P, None, 4, 100, 1024, P, None, None) == SHAPE and gb(P, P, None, P, None, 4, 32, 1024, P, None, None) == NULL
    assert gb(P, P, P, P, P + 4, 4, 32, 1024, P, None, None) == ALIGN and gb(None, None, None, None, None, 0, 32, 1024, None, None, None) == OK
    need8 = q.qvggt_workspace_bytes_i8b(100, 32, 1024)
    assert need8 >= 128 * 1024 + 400
    assert lb(P, 0, 100, 32, 1024, None, None, 8, P, P, None, P, P, need8 - 1, None) == WORKSPACE
    assert lb(P, 0, 100, 32, 768, None, None, 8, P, P, None, P, P, need8, None) == SHAPE
    assert lb(P, 1, 100, 32, 1024, None, None, 8, P, P, None, P, P, need8, None) == DTYPE
    assert lb(P, 0, 100, 32, 1024, None, None, 3, P, P, None, P, P, need8, None) == ARG
    # 8-bit / 6-bit entry points: the same checks, and the bit-width
    for bad in (3, 9, 0, -8):
        assert lib.qvggt_rotate_smooth_quant_i8(P, 0, 4, 1024, None, None, bad, P, P, None) == ARG
        assert lib.qvggt_prep_weights_i8(P, 0, 32, 1024, None, None, C.c_float(0.5), bad, P, P, P, None) == ARG
        assert lib.qvggt_linear_i8(P, 0, 4, 32, 1024, None, None, bad, P, P, None, P, P, 1 << 20, None) == ARG
    assert lib.qvggt_rotate_smooth_quant_i8(P, 0, 4, 1000, None, None, 8, P, P, None) == SHAPE
    assert lib.qvggt_rotate_smooth_quant_i8(P, 3, 4, 1024, None, None, 8, P, P, None) == DTYPE
    assert lib.qvggt_rotate_smooth_quant_i8(P, 0, 4, 1024, None, None, 6, None, P, None) == NULL
    assert lib.qvggt_prep_weights_i8(P, 0, 24, 1024, None, None, C.c_float(0.5), 8, P, P, P, None) == SHAPE
    assert lib.qvggt_prep_weights_i8(P, 0, 32, 1024, None, None, C.c_float(2.0), 8, P, P, P, None) == ARG
    assert lib.qvggt_i8_gemm(P, P, P, P, None, 4, 100, 1024, P, None, None) == SHAPE
    assert lib.qvggt_i8_gemm(P, P, None, P, None, 4, 32, 1024, P, None, None) == NULL
    assert lib.qvggt_i8_gemm(P, P, P, P, P + 4, 4, 32, 1024, P, None, None) == ALIGN
    assert lib.qvggt_i8_gemm(None, None, None, None, None, 0, 32, 1024, None, None, None) == OK
    need8 = q.qvggt_workspace_bytes_i8(100, 32, 1024)
    assert need8 >= 100 * 1024 + 100 * 4 and q.qvggt_workspace_bytes_i8(10, 30, 1024) == 0
    assert lib.qvggt_linear_i8(P, 0, 100, 32, 1024, None, None, 8, P, P, None, P, P, need8 - 1, None) == WORKSPACE
    assert lib.qvggt_layout_int8(P, 4, 1000, P, 1, None) == SHAPE
    assert lib.qvggt_layout_int8(P, 4, 1024, P, 2, None) == ARG
    assert lib.qvggt_layout_int8(P, 4, 1024, None, 1, None) == NULL
    assert lib.qvggt_layout_int8(None, 0, 1024, None, 0, None) == OK
    # workspace
    need = q.qvggt_workspace_bytes(100, 32, 1024)
    assert lib.qvggt_linear(P, 0, 100, 32, 1024, None, None, P, P, None, P, P, need - 1, None) == WORKSPACE
    # empty problems are accepted without touching anything
    assert lib.qvggt_rotate_smooth_quant(None, 0, 0, 1024, None, None, None, None, None) == OK
    assert lib.qvggt_w4a4_gemm(None, None, None, None, None, 0, 32, 1024, None, None, None) == OK
    assert lib.qvggt_linear(None, 0, 0, 32, 1024, None, None, None, None, None, None, None, 0, None) == OK
    assert lib.qvggt_pack_int4(None, 0, 1024, None, None) == OK


def test_own_workspace_entry_validates_without_a_gpu():
    """The entry point without a workspace argument: argument errors and the size limit are decided on the host."""
    lib = q.load_library()
    f = lib.qvggt_linear_e2m3_own_workspace
    limit = lib.qvggt_own_workspace_bytes()
    assert limit == 36 << 20
    assert f(P, 0, 4, 32, 1000, None, None, P, P, None, P, None) == SHAPE
    assert f(P, 0, 4, 32, 512, None, None, P, P, None, P, None) == SHAPE          # E2M3 kernel 1: K = 1024, 2048, 4096
    assert f(P, 1, 4, 32, 1024, None, None, P, P, None, P, None) == DTYPE
    assert f(None, 0, 4, 32, 1024, None, None, P, P, None, P, None) == NULL
    assert f(P, 0, 4, 32, 1024, None, None, P, P, None, None, None) == NULL
    assert f(P, 0, 4, 32, 1024, None, None, P + 4, P, None, P, None) == ALIGN
    assert f(None, 0, 0, 32, 1024, None, None, None, None, None, None, None) == OK
    # the limit: the largest token counts whose intermediate buffers fit, and one more
    for K, m_fit in ((4096, 12160), (1024, 48896)):
        assert lib.qvggt_workspace_bytes_e2m3(m_fit, 1024, K) <= limit < lib.qvggt_workspace_bytes_e2m3(m_fit + 1, 1024, K)
        assert f(P, 0, m_fit + 1, 1024, K, None, None, P, P, None, P, None) == WORKSPACE
    assert f(None, 0, 137400, 1024, 4096, None, None, None, None, None, None, None) == WORKSPACE     # size is checked before pointers
    # with no GPU the device set-up itself fails and is reported, nothing crashes
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:
        has_gpu = False
    if not has_gpu:
        assert lib.qvggt_init() == 7
        assert f(P, 0, 4, 32, 1024, None, None, P, P, None, P, None) == 7


def test_calibration_entry_points_validate_without_a_gpu():
    lib = q.load_library()
    rr, lg, ds = lib.qvggt_rotate_rows, lib.qvggt_calib_loss_grad, lib.qvggt_calib_descent_step
    assert rr(P, 0, 4, 1000, None, P, None) == SHAPE and rr(P, 0, 4, 768, None, P, None) == SHAPE and rr(P, 3, 4, 1024, None, P, None) == DTYPE
    assert rr(None, 0, 4, 1024, None, P, None) == NULL and rr(P, 0, 4, 1024, None, P + 4, None) == ALIGN and rr(None, 0, 0, 1024, None, None, None) == OK
    need = lib.qvggt_calib_workspace_bytes(100, 32, 1024)
    assert need >= 4 * (2 * 100 * 1024 + 2 * 32 * 1024 + 100 * 32) and lib.qvggt_calib_workspace_bytes(0, 32, 1024) == 0
    assert lib.qvggt_calib_workspace_bytes(100, 32, 1026) == 0
    args = lambda **kw: [kw.get("R", P), P, P, None, P, P, kw.get("xs", None), kw.get("T", 100), 32, kw.get("K", 1024), kw.get("bits", 4),
                         P, P, P, kw.get("gx", None), P, kw.get("wsb", need), None]
    assert lg(*args(T=0)) == SHAPE and lg(*args(K=1026)) == SHAPE and lg(*args(bits=3)) == ARG and lg(*args(bits=9)) == ARG
    assert lg(*args(R=None)) == NULL and lg(*args(R=P + 4)) == ALIGN and lg(*args(wsb=need - 1)) == WORKSPACE
    assert lg(*args(xs=P)) == NULL and lg(*args(gx=P)) == NULL            # a static step and its derivative come together
    assert ds(P, P, -1, C.c_float(0.1), C.c_float(1e-8), None) == SHAPE and ds(None, P, 4, C.c_float(0.1), C.c_float(1e-8), None) == NULL
    assert ds(P, P, 4, C.c_float(float("nan")), C.c_float(1e-8), None) == ARG and ds(P, P, 4, C.c_float(0.1), C.c_float(0.0), None) == ARG
    assert ds(P + 2, P, 4, C.c_float(0.1), C.c_float(1e-8), None) == ALIGN and ds(None, None, 0, C.c_float(0.1), C.c_float(1e-8), None) == OK


def test_binding_rejects_host_tensors():
    import torch
    x = torch.zeros(4, 1024, dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        q.qvggt_rotate_smooth_quant(x, None, None, torch.zeros(4, 512, dtype=torch.uint8), torch.zeros(4))


def test_nfds_argument_validation_needs_no_gpu():
    lib = q.load_library()
    dbl = C.c_double
    assert q.qvggt_nfds_workspace_bytes(8, 1 << 20, 0) > 0
    assert q.qvggt_nfds_workspace_bytes(8, 1001, 0) == 0            # a row must be whole 16-byte vectors
    assert q.qvggt_nfds_workspace_bytes(8, 1 << 20, 5) == 0
    need = q.qvggt_nfds_workspace_bytes(8, 1 << 20, 0)
    assert lib.qvggt_nfds_moments(P, 0, 8, 1001, P, P, P, need, None) == SHAPE
    assert lib.qvggt_nfds_moments(P, 7, 8, 1024, P, P, P, need, None) == DTYPE
    assert lib.qvggt_nfds_moments(None, 0, 8, 1024, P, P, P, need, None) == NULL
    assert lib.qvggt_nfds_moments(P + 4, 0, 8, 1024, P, P, P, need, None) == ALIGN
    assert lib.qvggt_nfds_moments(P, 0, 8, 1 << 20, P, P, P, need - 1, None) == WORKSPACE
    assert lib.qvggt_nfds_moments(None, 0, 0, 1024, None, None, None, 0, None) == OK
    assert lib.qvggt_nfds_frame_correlation(P, 0, 2, 1, 1024, P, P, need, None) == SHAPE     # needs at least two frames
    assert lib.qvggt_nfds_frame_correlation(P, 0, 2, 4, 1024, None, P, need, None) == NULL
    assert lib.qvggt_nfds_frame_correlation(P, 0, 2, 4, 1 << 20, P, P, 16, None) == WORKSPACE
    assert lib.qvggt_nfds_scores(P, P, 0, 4, dbl(1e-6), P, None) == SHAPE
    assert lib.qvggt_nfds_scores(P, P, 10, 4000, dbl(1e-6), P, None) == SHAPE
    assert lib.qvggt_nfds_scores(P, P, 10, 4, dbl(-1.0), P, None) == ARG
    assert lib.qvggt_nfds_scores(P, None, 10, 4, dbl(0.0), P, None) == NULL
    assert lib.qvggt_nfds_keep_lowest(P, 10, dbl(1.5), P, None) == ARG
    assert lib.qvggt_nfds_keep_lowest(P, 0, dbl(0.5), P, None) == SHAPE
    assert lib.qvggt_nfds_keep_lowest(P, 10, dbl(0.5), None, None) == NULL
    assert lib.qvggt_nfds_kmeans_step(P, 10, 3, 0, P, P + 64, P, None) == SHAPE
    assert lib.qvggt_nfds_kmeans_step(P, 10, 3, 2, P, P, P, None) == ARG                     # in-place centres
    assert lib.qvggt_nfds_kmeans_step(P, 10, 3, 2, P, P + 64, None, None) == NULL
    assert lib.qvggt_nfds_kmeans_step(P + 2, 10, 3, 2, P, P + 64, P, None) == ALIGN
