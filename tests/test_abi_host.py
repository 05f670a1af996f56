"""Host-only checks of the C ABI: the library loads, exports every symbol the header
declares, the size helpers agree with their definitions and every argument error is
reported before anything is launched (so these run without a GPU)."""
import os
import re

import pytest

from paper_1911_04477_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OK, NULL, SHAPE, STRIDE, ALIGN, WORKSPACE, HIP, UNSUPPORTED = range(8)


@pytest.fixture(scope="module")
def L():
    return B.lib()


def _declared_functions(header="bnn.h"):
    src = open(os.path.join(ROOT, "include", header)).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(bnn_[a-z0-9_]+)\s*\(", src)))


def test_every_declared_symbol_is_exported_and_bound(L):
    names = _declared_functions()
    assert len(names) >= 20
    for n in names:
        assert hasattr(L, n), n
    assert set(names) == set(B.SIGNATURES), set(names) ^ set(B.SIGNATURES)


def test_nothing_undeclared_is_exported(L):
    """The library is built with hidden visibility: its exported functions are exactly the
    two headers' declarations (the kernels' launch handles are data symbols, not functions)."""
    import subprocess
    out = subprocess.check_output(["nm", "-D", "--defined-only", B.LIB_PATH], text=True)
    funcs = {ln.split()[2] for ln in out.splitlines() if len(ln.split()) == 3 and ln.split()[1] == "T"}
    hooks = _declared_functions("bnn_testing.h")
    assert set(hooks) == set(B.TESTING_SIGNATURES), set(hooks) ^ set(B.TESTING_SIGNATURES)
    for n in hooks:
        assert hasattr(L, n), n
    assert funcs == set(_declared_functions()) | set(hooks), funcs ^ (set(_declared_functions()) | set(hooks))


def test_no_exported_writable_state():
    """What a call of bnn.h launches depends on its arguments only: the data symbols the library
    exports are the compiler's kernel launch handles and its per-file id bytes, nothing of the
    library's own, and none of the former process-wide switches exists."""
    import subprocess
    out = subprocess.check_output(["nm", "-D", "--defined-only", B.LIB_PATH], text=True)
    data = [ln.split()[2] for ln in out.splitlines() if len(ln.split()) == 3 and ln.split()[1] not in ("T", "t")]
    own = [n for n in data if not n.startswith(("__hip_cuid_", "__odr_asan_gen_", "__asan", "__ubsan"))
           and not re.match(r"_ZN3bnn\d+\w*_kernel", n)]
    assert own == [], own
    assert not any("internal" in ln or "force" in ln or "g_" in ln.split()[-1][:2] for ln in out.splitlines())


def test_status_strings(L):
    expect = ["BNN_OK", "BNN_ERR_NULL", "BNN_ERR_SHAPE", "BNN_ERR_STRIDE", "BNN_ERR_ALIGN", "BNN_ERR_WORKSPACE",
              "BNN_ERR_HIP", "BNN_ERR_UNSUPPORTED"]
    for i, s in enumerate(expect):
        assert L.bnn_status_str(i).decode() == s
    assert L.bnn_status_str(99).decode() == "BNN_ERR_UNKNOWN"


def test_size_helpers(L):
    for K, w in [(-1, 0), (0, 0), (1, 1), (63, 1), (64, 1), (65, 2), (200, 4), (256, 4), (4096, 64), (4608, 72)]:
        assert L.bnn_packed_words(K) == w
    assert L.bnn_conv_kwords(128, 3, 3) == 18
    assert L.bnn_conv_kwords(256, 3, 3) == 36
    assert L.bnn_conv_kwords(200, 1, 1) == 4
    assert L.bnn_conv_kwords(0, 3, 3) == 0
    assert L.bnn_conv_out_dim(32, 3, 1, 1) == 32
    assert L.bnn_conv_out_dim(56, 1, 2, 0) == 28
    assert L.bnn_conv_out_dim(7, 3, 2, 1) == 4
    assert L.bnn_conv_out_dim(2, 5, 1, 1) == 0
    assert L.bnn_conv_out_dim(5, 3, 0, 0) == 0
    # workspaces: packed NHWC image (+ patch matrix), each rounded up to 256 bytes
    img = 128 * 32 * 32 * 2 * 8
    assert L.bnn_im2col_workspace_bytes(128, 128, 32, 32, 3, 3, 1, 1, 1, 1) == img
    assert L.bnn_conv2d_workspace_bytes(128, 128, 32, 32, 3, 3, 1, 1, 1, 1) == img  # no patch matrix
    assert L.bnn_im2col_workspace_bytes(64, 200, 56, 56, 1, 1, 2, 2, 0, 0) == 0
    assert L.bnn_conv2d_workspace_bytes(64, 200, 56, 56, 1, 1, 2, 2, 0, 0) == 50176 * 4 * 8
    assert L.bnn_conv2d_workspace_bytes(1, 3, 2, 2, 5, 5, 1, 1, 0, 0) == 0  # invalid geometry


A16 = 4096  # a fake, 16-byte aligned, never dereferenced address
MIS = 4100  # misaligned


def test_encode_errors(L):
    assert L.bnn_encode(A16, -1, 8, 8, A16, 1, None) == SHAPE
    assert L.bnn_encode(A16, 4, 0, 8, A16, 1, None) == SHAPE
    assert L.bnn_encode(A16, 4, 65, 64, A16, 2, None) == STRIDE
    assert L.bnn_encode(A16, 4, 65, 65, A16, 1, None) == STRIDE
    assert L.bnn_encode(None, 0, 8, 8, None, 1, None) == OK  # empty: nothing to do
    assert L.bnn_encode(None, 4, 8, 8, A16, 1, None) == NULL
    assert L.bnn_encode(A16, 4, 8, 8, None, 1, None) == NULL
    assert L.bnn_encode(MIS, 4, 8, 8, A16, 1, None) == ALIGN
    assert L.bnn_encode(A16, 4, 8, 8, MIS, 1, None) == ALIGN


def test_pack_conv_weight_errors(L):
    assert L.bnn_pack_conv_weight(A16, 4, 0, 3, 3, A16, None) == SHAPE
    assert L.bnn_pack_conv_weight(A16, -1, 8, 3, 3, A16, None) == SHAPE
    assert L.bnn_pack_conv_weight(None, 0, 8, 3, 3, None, None) == OK
    assert L.bnn_pack_conv_weight(None, 4, 8, 3, 3, A16, None) == NULL
    assert L.bnn_pack_conv_weight(A16, 4, 8, 3, 3, MIS, None) == ALIGN


def test_gemm_errors(L):
    g = L.bnn_xnor_gemm
    assert g(A16, 4, A16, 4, A16, 8, 8, 8, 0, None) == SHAPE
    assert g(A16, 4, A16, 4, A16, 8, -1, 8, 256, None) == SHAPE
    assert g(A16, 3, A16, 4, A16, 8, 8, 8, 256, None) == STRIDE
    assert g(A16, 4, A16, 3, A16, 8, 8, 8, 256, None) == STRIDE
    assert g(A16, 4, A16, 4, A16, 7, 8, 8, 256, None) == STRIDE
    assert g(None, 4, None, 4, None, 8, 0, 8, 256, None) == OK
    assert g(None, 4, None, 4, None, 8, 8, 0, 256, None) == OK
    assert g(None, 4, A16, 4, A16, 8, 8, 8, 256, None) == NULL
    assert g(A16, 4, A16, 4, None, 8, 8, 8, 256, None) == NULL
    assert g(A16, 4, MIS, 4, A16, 8, 8, 8, 256, None) == ALIGN
    # column indices are ints computed on N rounded up to the tile width
    assert g(A16, 4, A16, 4, A16, 1 << 31, 8, (1 << 31) - 256, 256, None) == UNSUPPORTED
    e = L.bnn_xnor_gemm_epilogue
    assert e(A16, 4, A16, 4, 8, 8, 256, None, 8, None, 8, None, None, 0, None) == NULL  # no output at all
    assert e(A16, 4, A16, 4, 8, 8, 256, None, 8, A16, 8, None, A16, 1, None) == NULL  # Y without scale
    assert e(A16, 4, A16, 4, 8, 8, 256, None, 8, A16, 8, A16, A16, 0, None) == SHAPE  # Y needs an axis
    assert e(A16, 4, A16, 4, 8, 8, 256, None, 8, A16, 7, A16, A16, 1, None) == STRIDE
    assert e(A16, 4, A16, 4, 8, 8, 256, MIS, 8, A16, 8, A16, A16, 1, None) == ALIGN


def test_conv_and_im2col_errors(L):
    geo = (2, 8, 6, 6, 3, 3, 1, 1, 1, 1)
    need = L.bnn_conv2d_workspace_bytes(*geo)
    need_i = L.bnn_im2col_workspace_bytes(*geo)
    assert need == need_i > 0  # both hold the packed image; only im2col also writes the caller's patch matrix
    im = L.bnn_im2col_packed
    assert im(A16, 2, 8, 6, 6, 7, 7, 1, 1, 0, 0, A16, A16, 1 << 20, None) == SHAPE  # OH < 1
    assert im(A16, 2, 8, 6, 6, 3, 3, 0, 1, 1, 1, A16, A16, 1 << 20, None) == SHAPE  # stride 0
    assert im(A16, 2, 0, 6, 6, 3, 3, 1, 1, 1, 1, A16, A16, 1 << 20, None) == SHAPE
    assert im(None, 0, 8, 6, 6, 3, 3, 1, 1, 1, 1, None, None, 0, None) == OK
    assert im(None, *geo, A16, A16, need_i, None) == NULL
    assert im(A16, *geo, A16, None, need_i, None) == NULL
    assert im(A16, *geo, MIS, A16, need_i, None) == ALIGN
    assert im(A16, *geo, A16, A16, need_i - 1, None) == WORKSPACE
    cv = L.bnn_conv2d
    base = dict(x=A16, w=A16, oi=A16, of=None, sc=None, bi=None, ws=A16, wb=need)

    def call(D=4, g=geo, **kw):
        a = dict(base, **kw)
        N, C, H, W, kH, kW, sH, sW, pH, pW = g
        return cv(a["x"], a["w"], N, C, H, W, D, kH, kW, sH, sW, pH, pW, a["oi"], a["of"], a["sc"], a["bi"], a["ws"],
                  a["wb"], None)

    assert call(g=(2, 8, 6, 6, 3, 3, 1, 1, -1, 1)) == SHAPE
    assert call(D=-1) == SHAPE
    assert call(D=0) == OK
    assert call(x=None) == NULL
    assert call(oi=None) == NULL  # neither output
    assert call(of=A16) == NULL  # fp32 output without scale / bias
    assert call(ws=None) == NULL
    assert call(w=MIS) == ALIGN
    assert call(wb=need - 1) == WORKSPACE


def test_noalloc_conv_errors_need_no_device(L):
    """Size and argument checks of the entry point that allocates nothing run before any HIP call."""
    na = L.bnn_conv2d_noalloc
    assert L.bnn_conv2d_noalloc_max_bytes() == 8 << 20
    geo = (2, 8, 6, 6, 4, 3, 3, 1, 1, 1, 1)
    assert na(A16, A16, 128, 256, 56, 56, 256, 3, 3, 1, 1, 1, 1, A16, None, None, None, None) == WORKSPACE
    assert na(A16, A16, 2, 8, 6, 6, 4, 7, 7, 1, 1, 0, 0, A16, None, None, None, None) == SHAPE
    assert na(None, None, 0, 8, 6, 6, 4, 3, 3, 1, 1, 1, 1, None, None, None, None, None) == OK
    assert na(None, A16, *geo, A16, None, None, None, None) == NULL
    assert na(A16, A16, *geo, None, None, None, None, None) == NULL
    assert na(A16, A16, *geo, None, A16, None, None, None) == NULL  # fp32 output without scale / bias
    assert na(A16, MIS, *geo, A16, None, None, None, None) == ALIGN


def test_packed_conv_errors(L):
    cp = L.bnn_conv2d_packed
    geo = (2, 128, 8, 8, 64, 3, 3, 1, 1, 1, 1)

    def call(x=A16, w=A16, g=geo, pool=0, oi=None, of=None, op=A16, sc=A16, bi=A16):
        return cp(x, w, *g, pool, oi, of, op, sc, bi, None)

    assert call(pool=1) == SHAPE
    assert call(g=(2, 128, 7, 7, 64, 3, 3, 1, 1, 1, 1), pool=2) == SHAPE  # odd output size cannot pool
    assert call(g=(2, 128, 8, 8, -1, 3, 3, 1, 1, 1, 1)) == SHAPE
    assert call(g=(0, 128, 8, 8, 64, 3, 3, 1, 1, 1, 1)) == OK
    assert call(x=None) == NULL
    assert call(op=None) == NULL  # no output at all
    assert call(sc=None) == NULL  # packed output needs scale / bias
    assert call(oi=A16) == UNSUPPORTED  # one kind of output per call
    assert call(pool=2, op=None, oi=A16) == UNSUPPORTED  # pooling only in the packed epilogue
    assert call(w=MIS) == ALIGN
    # a reduction of 2^31 bits (8 x 8 taps of 2^25 channels) does not fit the kernel's int
    assert call(g=(1, 1 << 25, 8, 8, 1, 8, 8, 1, 1, 0, 0)) == UNSUPPORTED
    fs = L.bnn_conv2d_f32_sign
    assert fs(A16, A16, 2, 3, 8, 8, 128, 3, 3, 1, 1, 1, 1, None, A16, A16, None) == NULL
    assert fs(A16, A16, 2, 4, 8, 8, 128, 3, 3, 1, 1, 1, 1, A16, A16, A16, None) == UNSUPPORTED  # 36 taps > 32
    assert fs(A16, A16, 2, 3, 8, 8, 128, 9, 9, 1, 1, 0, 0, A16, A16, A16, None) == SHAPE
    pf = L.bnn_pack_fc_weight_nhwc
    assert pf(A16, 10, 0, 4, 4, A16, None) == SHAPE
    assert pf(None, 0, 64, 4, 4, None, None) == OK
    assert pf(None, 10, 64, 4, 4, A16, None) == NULL
    assert pf(A16, 10, 64, 4, 4, MIS, None) == ALIGN


def test_glue_errors(L):
    mp = L.bnn_maxpool2x2
    assert mp(A16, 2, 4, 5, 6, A16, None, None, None, None) == SHAPE  # odd H
    assert mp(A16, 2, 4, 6, 6, None, None, None, None, None) == NULL
    assert mp(A16, 2, 4, 6, 6, None, A16, None, None, None) == NULL
    assert mp(MIS, 2, 4, 6, 6, A16, None, None, None, None) == ALIGN
    assert mp(None, 0, 4, 6, 6, None, None, None, None, None) == OK
    cf = L.bnn_conv2d_f32
    assert cf(A16, A16, 2, 3, 8, 8, 4, 3, 3, 1, 1, 1, 1, A16, None, A16, None) == NULL  # scale without bias
    assert cf(A16, A16, 2, 3, 8, 8, 4, 9, 9, 1, 1, 0, 0, None, None, A16, None) == SHAPE
    assert cf(A16, None, 2, 3, 8, 8, 4, 3, 3, 1, 1, 1, 1, None, None, A16, None) == NULL
    fc = L.bnn_fc_f32
    assert fc(A16, A16, None, 4, 0, 4, 0, A16, None) == SHAPE
    assert fc(A16, A16, None, 4, 8, 4, 0, None, None) == NULL
    assert fc(A16, MIS, None, 4, 8, 4, 0, A16, None) == ALIGN
    assert L.bnn_valu_peak_probe(None, 4, 4, 0, None) == NULL
    assert L.bnn_valu_peak_probe(A16, -1, 4, 0, None) == SHAPE
    assert L.bnn_valu_peak_probe(A16, 4, 4, 3, None) == SHAPE  # no such kind
    assert L.bnn_copy_probe(A16, A16, 24, None) == SHAPE
    assert L.bnn_copy_probe(A16, None, 32, None) == NULL


def test_ablation_and_control_errors(L):
    for mf in (L.bnn_xnor_gemm_mfma_i8, L.bnn_xnor_gemm_mfma_fp4):
        assert mf(A16, 4, A16, 4, A16, 8, 8, 8, 0, None) == SHAPE          # K = 0
        assert mf(A16, 1, A16, 4, A16, 8, 8, 8, 200, None) == STRIDE       # lda < words
        assert mf(A16, 4, A16, 4, A16, 4, 8, 8, 200, None) == STRIDE       # ldc < N
        assert mf(A16, 4, A16, 4, None, 8, 8, 8, 200, None) == NULL
        assert mf(A16, 4, MIS, 4, A16, 8, 8, 8, 200, None) == ALIGN
        assert mf(None, 4, None, 4, None, 8, 0, 8, 200, None) == OK        # empty problem: nothing touched
    # the fp4 form counts in fp32: reductions of 2^24 bits and more are refused
    assert L.bnn_xnor_gemm_mfma_fp4(A16, 1 << 18, A16, 1 << 18, A16, 8, 8, 8, 1 << 24, None) == UNSUPPORTED
    # operands kept expanded in memory: strides in bytes, multiples of 16
    fx = L.bnn_xnor_gemm_mfma_fp4_expanded
    assert L.bnn_fp4_row_bytes(1) == 32 and L.bnn_fp4_row_bytes(64) == 32 and L.bnn_fp4_row_bytes(65) == 64
    assert L.bnn_fp4_row_bytes(0) == 0
    assert fx(A16, 128, A16, 128, A16, 8, 8, 8, 0, None) == SHAPE
    assert fx(A16, 96, A16, 128, A16, 8, 8, 8, 200, None) == STRIDE        # a row of 200 values takes 128 bytes
    assert fx(A16, 136, A16, 128, A16, 8, 8, 8, 200, None) == STRIDE       # not a multiple of 16
    assert fx(A16, 128, A16, 128, A16, 4, 8, 8, 200, None) == STRIDE       # ldc < N
    assert fx(A16, 128, A16, 128, None, 8, 8, 8, 200, None) == NULL
    assert fx(A16, 128, MIS, 128, A16, 8, 8, 8, 200, None) == ALIGN
    assert fx(None, 128, None, 128, None, 8, 0, 8, 200, None) == OK
    assert fx(A16, 1 << 23, A16, 1 << 23, A16, 8, 8, 8, 1 << 24, None) == UNSUPPORTED
    assert L.bnn_testing_xnor_gemm_mfma_fp4_expanded(A16, 128, A16, 128, A16, 8, 8, 8, 200, 3, None) == SHAPE  # no such tile
    ex = L.bnn_expand_fp4
    assert ex(A16, 4, 0, 4, A16, 128, None) == SHAPE
    assert ex(A16, 4, 200, 3, A16, 128, None) == STRIDE                    # source rows shorter than 4 words
    assert ex(A16, 4, 200, 4, A16, 96, None) == STRIDE
    assert ex(A16, 4, 200, 4, A16, 136, None) == STRIDE
    assert ex(A16, 4, 200, 4, None, 128, None) == NULL
    assert ex(MIS, 4, 200, 4, A16, 128, None) == ALIGN
    assert ex(None, 0, 200, 4, None, 128, None) == OK
    cx = L.bnn_conv2d_mfma_fp4_expanded
    assert cx(A16, A16, 2, 64, 8, 8, 4, 9, 9, 1, 1, 0, 0, A16, None) == SHAPE      # kernel larger than image
    assert cx(A16, A16, 2, 100, 8, 8, 4, 3, 3, 1, 1, 1, 1, A16, None) == UNSUPPORTED  # C not a multiple of 64
    assert cx(A16, None, 2, 64, 8, 8, 4, 3, 3, 1, 1, 1, 1, A16, None) == NULL
    assert cx(A16, A16, 2, 64, 8, 8, 4, 3, 3, 1, 1, 1, 1, MIS, None) == ALIGN
    assert cx(None, None, 0, 64, 8, 8, 4, 3, 3, 1, 1, 1, 1, None, None) == OK       # empty batch
    cc = L.bnn_control_conv2d_f32
    assert cc(A16, A16, 2, 3, 8, 8, 4, 9, 9, 1, 1, 0, 0, A16, None) == SHAPE   # kernel larger than image
    assert cc(A16, A16, 2, 3, 8, 8, -1, 3, 3, 1, 1, 1, 1, A16, None) == SHAPE
    assert cc(A16, None, 2, 3, 8, 8, 4, 3, 3, 1, 1, 1, 1, A16, None) == NULL
    assert cc(A16, A16, 2, 3, 8, 8, 4, 3, 3, 1, 1, 1, 1, MIS, None) == ALIGN
    assert cc(None, None, 0, 3, 8, 8, 4, 3, 3, 1, 1, 1, 1, None, None) == OK   # empty batch


def test_empty_problems_succeed_without_touching_anything(L):
    """Zero rows / columns / images / channels return OK before any pointer is looked at."""
    assert L.bnn_encode(None, 0, 64, 64, None, 1, None) == OK
    assert L.bnn_pack_conv_weight(None, 0, 3, 3, 3, None, None) == OK
    assert L.bnn_xnor_gemm(None, 4, None, 4, None, 8, 0, 8, 200, None) == OK
    assert L.bnn_xnor_gemm(None, 4, None, 4, None, 0, 8, 0, 200, None) == OK
    assert L.bnn_xnor_gemm_epilogue(None, 4, None, 4, 0, 8, 200, None, 8, None, 8, None, None, 1, None) == OK
    assert L.bnn_conv2d(None, None, 0, 3, 8, 8, 4, 3, 3, 1, 1, 1, 1, None, None, None, None, None, 0, None) == OK
    assert L.bnn_conv2d(None, None, 2, 3, 8, 8, 0, 3, 3, 1, 1, 1, 1, None, None, None, None, None, 0, None) == OK
    assert L.bnn_conv2d_f32_sign(None, None, 0, 3, 8, 8, 4, 3, 3, 1, 1, 1, 1, None, None, None, None) == OK
    assert L.bnn_pack_fc_weight_nhwc(None, 0, 4, 2, 2, None, None) == OK
    assert L.bnn_fc_f32(None, None, None, 0, 8, 4, 0, None, None) == OK


def test_prof_hook_is_inert_without_launches(L):
    assert L.bnn_prof_count() == 0
    assert L.bnn_prof_reset() == OK
    assert L.bnn_kernel_name(4).decode() == "xnor_gemm"
    assert L.bnn_kernel_name(1234).decode() == "unknown"


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU; asking the benchmark for more must say so and fail."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr
