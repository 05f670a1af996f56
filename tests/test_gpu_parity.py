"""GPU parity: every entry point of the C ABI against the CPU oracle, element by element,
on the same seeded host-generated inputs.  Integer / packed outputs must be bit-exact;
the fp32 epilogue must match within 1e-6 relative (it is in fact built to be bit-exact)."""
import numpy as np
import pytest
import torch

import oracle
from paper_1911_04477_amd import binding as B
from paper_1911_04477_amd import inputs

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def as_u64(t):
    return host(t).view("<u8")


def assert_f32_close(got, ref):
    assert got.shape == ref.shape
    # 1e-6 relative, as the contract asks; report bit-exactness too
    assert np.allclose(got, ref, rtol=1e-6, atol=1e-30), np.abs(got - ref).max()


# ---------------------------------------------------------------- encode (a1)
@pytest.mark.parametrize("rows,K", [(1, 1), (3, 31), (5, 64), (7, 65), (64, 256), (33, 200), (2, 4097), (130, 1152),
                                     (1000, 63), (17, 1024 + 13)])
def test_encode_matches_oracle(rows, K):
    print(f"encode rows={rows} K={K}", flush=True)
    rng = np.random.default_rng(rows * 100003 + K)
    x = inputs.inject_specials(rng.standard_normal((rows, K)).astype(np.float32), K, frac=0.01)
    got = as_u64(B.bnn_encode(dev(x)))
    assert np.array_equal(got, oracle.encode_rows(x))


def test_encode_strided_src_and_dst():
    print("encode strided", flush=True)
    rng = np.random.default_rng(5)
    rows, K, sld, dld = 37, 130, 140, 5
    big = rng.standard_normal((rows, sld)).astype(np.float32)
    src = dev(big)[:, :K]
    dst = torch.full((rows, dld), -1, dtype=torch.int64, device=DEV)
    B.bnn_encode(src, dst[:, :3])
    out = as_u64(dst)
    assert np.array_equal(out[:, :3], oracle.encode_rows(big[:, :K]))
    assert np.all(out[:, 3:] == np.uint64(0xFFFFFFFFFFFFFFFF))  # words past Kw untouched


def test_encode_cfg2_weights_full_size():
    print("encode cfg2 weights 4096x4096", flush=True)
    d = inputs.cfg2()
    got = as_u64(B.bnn_encode(dev(d["wt"])))
    assert np.array_equal(got, oracle.encode_rows(d["wt"]))


# ---------------------------------------------------------------- weight packing / im2col (a2)
CONV_CASES = [
    # N, C, H, W, D, kH, kW, sH, sW, pH, pW
    (2, 64, 6, 6, 5, 3, 3, 1, 1, 1, 1),
    (2, 128, 9, 7, 33, 3, 3, 1, 1, 1, 1),
    (3, 70, 8, 8, 9, 3, 3, 2, 2, 1, 1),
    (2, 200, 10, 10, 17, 1, 1, 2, 2, 0, 0),
    (1, 3, 12, 12, 4, 5, 5, 1, 1, 2, 2),
    (2, 256, 5, 6, 70, 3, 3, 1, 1, 0, 0),
    (1, 130, 7, 9, 3, 3, 1, 1, 2, 1, 0),
    (5, 192, 4, 4, 130, 1, 1, 1, 1, 0, 0),
    (1, 512, 8, 8, 12, 3, 3, 1, 1, 1, 1),
    (2, 32, 6, 5, 6, 2, 2, 1, 1, 1, 1),
    (1, 1, 3, 3, 1, 3, 3, 1, 1, 1, 1),
]


@pytest.mark.parametrize("case", CONV_CASES)
def test_pack_weight_and_im2col_match_oracle(case):
    print(f"im2col case={case}", flush=True)
    N, C, H, W, D, kH, kW, sH, sW, pH, pW = case
    rng = np.random.default_rng(sum(case))
    x = inputs.inject_specials(rng.standard_normal((N, C, H, W)).astype(np.float32), 1, frac=0.01)
    w = inputs.inject_specials(rng.standard_normal((D, C, kH, kW)).astype(np.float32), 2, frac=0.01)
    assert np.array_equal(as_u64(B.bnn_pack_conv_weight(dev(w))), oracle.pack_conv_weight(w))
    cols = as_u64(B.bnn_im2col_packed(dev(x), kH, kW, (sH, sW), (pH, pW)))
    assert np.array_equal(cols, oracle.im2col_packed(x, kH, kW, (sH, sW), (pH, pW)))


# ---------------------------------------------------------------- GEMM (a3)
def _gemm_case(M, N, K, seed, cfg=None):
    rng = np.random.default_rng(seed)
    A = inputs.inject_specials(rng.standard_normal((M, K)).astype(np.float32), seed, frac=0.002)
    Bm = inputs.inject_specials(rng.standard_normal((N, K)).astype(np.float32), seed + 1, frac=0.002)
    Ap, Bp = B.bnn_encode(dev(A)), B.bnn_encode(dev(Bm))
    got = host(B.bnn_xnor_gemm(Ap, Bp, K, cfg=cfg))
    assert np.array_equal(got, oracle.gemm_pm1(A, Bm))


# K = 130 / 192 (three-word rows: dword-at-a-time tail), 400 / 704 (4n + 3 words: window chunk at an odd word)
@pytest.mark.parametrize("K", [1, 31, 32, 33, 63, 64, 65, 130, 192, 200, 256, 257, 400, 511, 512, 544, 704, 1152,
                               2304 + 17])
@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 6, 7, 8, 9, 13, 14, 15, 16, 17, 18])
def test_gemm_k_sweep_all_tile_configs(K, cfg):
    print(f"gemm K={K} cfg={cfg}", flush=True)
    _gemm_case(37, 150, K, seed=K * 7 + cfg, cfg=cfg)


@pytest.mark.parametrize("M,N", [(1, 1), (1, 700), (65, 513), (64, 512), (130, 1030), (257, 64), (33, 65)])
@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 6, 7, 8, 9, 13, 14, 15, 16, 17, 18])
def test_gemm_ragged_tiles(M, N, cfg):
    print(f"gemm M={M} N={N} cfg={cfg}", flush=True)
    _gemm_case(M, N, 300, seed=M * 1000 + N + cfg, cfg=cfg)


@pytest.mark.parametrize("cfg", [1, 3])
@pytest.mark.parametrize("K", [1, 63, 64, 130, 192, 200, 256, 400, 512, 704, 1152, 2304 + 17])
def test_gemm_four_columns_per_lane_tiles_k_sweep(K, cfg):
    """N a multiple of 4: the 256-column tiles take four consecutive columns per lane and store 16 bytes
    (N = 150 in the sweep above takes the one-column form); every kind of K tail, one and several tiles."""
    print(f"gemm four-column tiles K={K} cfg={cfg}", flush=True)
    _gemm_case(37, 152, K, seed=K * 11 + cfg, cfg=cfg)
    _gemm_case(70, 516, K, seed=K * 13 + cfg, cfg=cfg)


@pytest.mark.parametrize("lean", [1, 0])
@pytest.mark.parametrize("cfg", [1, 3])
@pytest.mark.parametrize("case", [(3, 128, 8, 8, 40, 3, 3, 1, 1, 1, 1), (3, 128, 10, 10, 70, 3, 3, 1, 1, 1, 1),
                                  (2, 64, 7, 9, 33, 3, 3, 1, 1, 1, 1), (5, 192, 6, 6, 130, 3, 3, 2, 2, 1, 1),
                                  (4, 128, 12, 12, 64, 1, 1, 2, 2, 0, 0), (7, 256, 6, 6, 65, 3, 3, 1, 1, 1, 1)])
def test_conv2d_four_columns_per_lane_tiles(case, cfg, lean):
    """int32 and fp32 NCHW outputs of the 256-column tiles with both gathers: maps whose pixel count is a
    multiple of 4 (16-byte stores, four-pixel groups that must not straddle images: 64, 100 and 36 pixels
    per image against 256 columns per tile) and maps where it is not (63 and 9: one column per lane)."""
    print(f"conv2d four-column tiles case={case} cfg={cfg} lean={lean}", flush=True)
    N, C, H, W, D, kH, kW, sH, sW, pH, pW = case
    d = inputs.conv_inputs(inputs.ConvShape(*case), seed=sum(case) + 31)
    x = inputs.inject_specials(d["x"], 8, frac=0.01)
    xp = _u64dev(oracle.pack_nhwc(x))
    wp = B.bnn_pack_conv_weight(dev(d["w"]))
    sc, bi = dev(d["scale"]), dev(d["bias"])
    st, pd = (sH, sW), (pH, pW)
    ref = oracle.conv2d_pm1(x, d["w"], st, pd)
    assert np.array_equal(host(B.bnn_conv2d_packed(xp, wp, C, D, kH, kW, st, pd, out="i32", cfg=cfg, lean=lean)), ref)
    yref = oracle.scale_bias(ref, d["scale"], d["bias"], "nchw")
    got = host(B.bnn_conv2d_packed(xp, wp, C, D, kH, kW, st, pd, scale=sc, bias=bi, out="f32", cfg=cfg, lean=lean))
    assert np.array_equal(got, yref)
    oi, of = B.bnn_conv2d(dev(x), wp, D, kH, kW, st, pd, sc, bi, want_int=True, cfg=cfg, lean=lean)
    assert np.array_equal(host(oi), ref) and np.array_equal(host(of), yref)


@pytest.mark.parametrize("cfg", [-1, 10, 11, 12])
@pytest.mark.parametrize("M,N,K", [(37, 152, 200), (8, 4, 65), (64, 256, 256), (130, 1028, 193), (257, 516, 128),
                                   (33, 260, 100), (70, 2052, 255), (5, 64, 129)])
def test_gemm_short_rows_kernel(M, N, K, cfg):
    """Rows of two or four words with N a multiple of 4: the store-bound kernel (four consecutive
    columns per lane, 16-byte stores), 8 and 16 rows per wave, and whatever the heuristic picks;
    int32 alone, and int32 + fp32 with the channel along either axis, on padded leading dimensions."""
    print(f"gemm short rows M={M} N={N} K={K} cfg={cfg}", flush=True)
    c = None if cfg < 0 else cfg
    rng = np.random.default_rng(M * 31 + N + K)
    A = inputs.inject_specials(rng.standard_normal((M, K)).astype(np.float32), 1, frac=0.01)
    Bm = inputs.inject_specials(rng.standard_normal((N, K)).astype(np.float32), 2, frac=0.01)
    Ap, Bp = as_u64(B.bnn_encode(dev(A))).copy(), as_u64(B.bnn_encode(dev(Bm))).copy()
    tail = K % 64
    if tail:  # garbage past K in both operands must not count
        g = np.uint64((0xFFFFFFFFFFFFFFFF >> tail) << tail)
        Ap[:, -1] |= g & np.uint64(0x5A5A5A5A5A5A5A5A)
        Bp[:, -1] |= g & np.uint64(0xF0F0F0F00F0F0F0F)
    Ad, Bd = dev(Ap.view(np.int64)), dev(Bp.view(np.int64))
    ref = oracle.gemm_pm1(A, Bm)
    Cbig = torch.full((M, N + 8), -7, dtype=torch.int32, device=DEV)
    B.bnn_xnor_gemm(Ad, Bd, K, Cbig[:, :N], cfg=c)
    out = host(Cbig)
    assert np.array_equal(out[:, :N], ref) and np.all(out[:, N:] == -7)
    for axis in ("row", "col"):
        nch = M if axis == "row" else N
        sc = ((rng.random(nch) + 0.5) * rng.choice([-1.0, 1.0], nch)).astype(np.float32)
        bi = rng.standard_normal(nch).astype(np.float32)
        Ci, Y = B.bnn_xnor_gemm_epilogue(Ad, Bd, K, dev(sc), dev(bi), B.CH_ROW if axis == "row" else B.CH_COL,
                                         want_int=True, cfg=c)
        assert np.array_equal(host(Ci), ref)
        assert np.array_equal(host(Y), oracle.scale_bias(ref, sc, bi, axis))


@pytest.mark.parametrize("cfg", [-1, 10, 11, 12, 3])
@pytest.mark.parametrize("case", [(3, 200, 12, 12, 70, 1, 1, 2, 2, 0, 0),    # 36 pixels per image: short-row kernel
                                  (2, 200, 10, 10, 17, 1, 1, 2, 2, 0, 0),    # 25 pixels per image: not a multiple of 4
                                  (2, 128, 8, 8, 40, 1, 1, 1, 1, 0, 0),      # rows of two words, stride 1
                                  (5, 256, 6, 4, 130, 1, 1, 1, 2, 0, 0),
                                  (2, 100, 16, 16, 9, 1, 1, 2, 2, 0, 0),
                                  (2, 250, 9, 12, 33, 1, 1, 3, 2, 0, 0)])    # odd H, stride (3, 2)
def test_conv2d_pointwise_short_rows(case, cfg):
    """1x1 / pad-0 convolutions with at most 256 channels: the encode samples the strided pixels
    (8-byte loads on even rows with column stride 2) and the GEMM is the short-row kernel where the
    image size allows it; int32 and fp32 outputs against the oracle."""
    print(f"conv2d pointwise case={case} cfg={cfg}", flush=True)
    N, C, H, W, D, kH, kW, sH, sW, pH, pW = case
    shape = inputs.ConvShape(*case)
    d = inputs.conv_inputs(shape, seed=sum(case) + 21)
    x = inputs.inject_specials(d["x"], 9, frac=0.01)
    wp = B.bnn_pack_conv_weight(dev(d["w"]))
    oi, of = B.bnn_conv2d(dev(x), wp, D, 1, 1, (sH, sW), (0, 0), dev(d["scale"]), dev(d["bias"]), want_int=True,
                          cfg=None if cfg < 0 else cfg)
    ref = oracle.conv2d_pm1(x, d["w"], (sH, sW), (0, 0))
    assert np.array_equal(host(oi), ref)
    assert np.array_equal(host(of), oracle.scale_bias(ref, d["scale"], d["bias"], "nchw"))


def test_gemm_table1_truth_table():
    """Table 1 of the paper through encode + GEMM with K = 1 (63 masked tail bits)."""
    print("gemm truth table", flush=True)
    vals = np.array([[-1.0], [1.0]], dtype=np.float32)
    P = B.bnn_encode(dev(vals))
    assert as_u64(P).reshape(-1).tolist() == [0, 1]
    got = host(B.bnn_xnor_gemm(P, P, 1))
    assert got.tolist() == [[1, -1], [-1, 1]]


def test_gemm_masks_garbage_past_K():
    print("gemm tail garbage", flush=True)
    rng = np.random.default_rng(11)
    for K in (1, 33, 70, 200):
        A = rng.standard_normal((9, K)).astype(np.float32)
        Bm = rng.standard_normal((70, K)).astype(np.float32)
        Ap, Bp = as_u64(B.bnn_encode(dev(A))).copy(), as_u64(B.bnn_encode(dev(Bm))).copy()
        tail = K % 64
        garbage = np.uint64((0xFFFFFFFFFFFFFFFF >> tail) << tail) if tail else np.uint64(0)
        Ap[:, -1] |= garbage & np.uint64(0xA5A5A5A5A5A5A5A5)
        Bp[:, -1] |= garbage & np.uint64(0x0F0F0F0FF0F0F0F0)
        got = host(B.bnn_xnor_gemm(dev(Ap.view(np.int64)), dev(Bp.view(np.int64)), K))
        assert np.array_equal(got, oracle.gemm_pm1(A, Bm)), K


def test_gemm_leading_dimensions():
    print("gemm ld", flush=True)
    rng = np.random.default_rng(12)
    M, N, K = 20, 90, 330
    A = rng.standard_normal((M, K)).astype(np.float32)
    Bm = rng.standard_normal((N, K)).astype(np.float32)
    Kw = B.packed_words(K)
    Abig = torch.full((M, Kw + 3), 0x5555, dtype=torch.int64, device=DEV)
    Bbig = torch.full((N, Kw + 1), 0x3333, dtype=torch.int64, device=DEV)  # odd ldb: 8-byte load path
    B.bnn_encode(dev(A), Abig[:, :Kw])
    B.bnn_encode(dev(Bm), Bbig[:, :Kw])
    Cbig = torch.full((M, N + 5), -7, dtype=torch.int32, device=DEV)
    B.bnn_xnor_gemm(Abig[:, :Kw], Bbig[:, :Kw], K, Cbig[:, :N])
    out = host(Cbig)
    assert np.array_equal(out[:, :N], oracle.gemm_pm1(A, Bm))
    assert np.all(out[:, N:] == -7)


@pytest.mark.parametrize("axis", ["row", "col"])
@pytest.mark.parametrize("cfg", [-1, 1, 2, 3, 4, 6, 7, 8, 9, 13, 14, 15, 16, 17, 18])
@pytest.mark.parametrize("M,N,K", [(37, 150, 300), (130, 515, 1100), (8, 64, 64), (70, 200, 4096 + 77)])
def test_gemm_fp32_epilogue_both_axes(M, N, K, cfg, axis):
    """y = fma(scale[ch], float(acc), bias[ch]) with the channel along rows or columns, with and
    without the int32 result beside it, on every tile configuration."""
    print(f"gemm epilogue M={M} N={N} K={K} cfg={cfg} axis={axis}", flush=True)
    rng = np.random.default_rng(M + N + K + cfg)
    A = rng.standard_normal((M, K)).astype(np.float32)
    Bm = rng.standard_normal((N, K)).astype(np.float32)
    nch = M if axis == "row" else N
    sc = ((rng.random(nch) + 0.5) * rng.choice([-1.0, 1.0], nch)).astype(np.float32)
    bi = rng.standard_normal(nch).astype(np.float32)
    Ap, Bp = B.bnn_encode(dev(A)), B.bnn_encode(dev(Bm))
    ref = oracle.gemm_pm1(A, Bm)
    yref = oracle.scale_bias(ref, sc, bi, axis)
    ax = B.CH_ROW if axis == "row" else B.CH_COL
    C, Y = B.bnn_xnor_gemm_epilogue(Ap, Bp, K, dev(sc), dev(bi), ax, want_int=True, cfg=cfg)
    assert np.array_equal(host(C), ref)
    assert np.array_equal(host(Y), yref)
    C, Y = B.bnn_xnor_gemm_epilogue(Ap, Bp, K, dev(sc), dev(bi), ax, want_int=False, cfg=cfg)
    assert C is None and np.array_equal(host(Y), yref)


def test_gemm_deterministic_twice():
    print("gemm determinism", flush=True)
    d = inputs.cfg1()
    Ap, Bp = B.bnn_encode(dev(d["A"])), B.bnn_encode(dev(d["B"]))
    a = host(B.bnn_xnor_gemm(Ap, Bp, inputs.CFG1.K))
    b = host(B.bnn_xnor_gemm(Ap, Bp, inputs.CFG1.K))
    assert np.array_equal(a, b)


# ---------------------------------------------------------------- the five configurations
def test_cfg1_single_gemm():
    print("cfg1", flush=True)
    d = inputs.cfg1()
    A = inputs.inject_specials(d["A"], 1)
    Bm = inputs.inject_specials(d["B"], 2)
    Ap, Bp = B.bnn_encode(dev(A)), B.bnn_encode(dev(Bm))
    assert as_u64(Ap).view("<u4").shape == (64, 8)
    assert np.array_equal(host(B.bnn_xnor_gemm(Ap, Bp, 256)), oracle.gemm_pm1(A, Bm))


def test_cfg2_fc_layer_full_size():
    print("cfg2", flush=True)
    d = inputs.cfg2()
    act = inputs.inject_specials(d["act"], 3)
    Ap, Wp = B.bnn_encode(dev(act)), B.bnn_encode(dev(d["wt"]))
    C, Y = B.bnn_xnor_gemm_epilogue(Ap, Wp, inputs.CFG2.K, dev(d["scale"]), dev(d["bias"]), B.CH_COL, want_int=True)
    ref = oracle.gemm_pm1(act, d["wt"])
    assert np.array_equal(host(C), ref)
    yref = oracle.scale_bias(ref, d["scale"], d["bias"], "col")
    got = host(Y)
    assert_f32_close(got, yref)
    assert np.array_equal(got, yref)  # single-rounded fma on both sides: bit-exact


def _conv_parity(shape, data, with_epilogue=True):
    """bnn_conv2d against the oracle's direct convolution on EVERY output: int32 bit-exact, and the
    fp32 epilogue against oracle.scale_bias (1e-6 relative by contract, bit-exact by construction)."""
    x = inputs.inject_specials(data["x"], 7, frac=1e-4)
    w = data["w"]
    xd, wd = dev(x), dev(w)
    wp = B.bnn_pack_conv_weight(wd)
    st, pd = (shape.sH, shape.sW), (shape.pH, shape.pW)
    sc, bi = dev(data["scale"]), dev(data["bias"])
    oi, of = B.bnn_conv2d(xd, wp, shape.D, shape.kH, shape.kW, st, pd, sc if with_epilogue else None,
                          bi if with_epilogue else None, want_int=True)
    got = host(oi)
    assert got.shape == (x.shape[0], shape.D, shape.OH, shape.OW)
    ref = oracle.conv2d_pm1(x, w, st, pd)
    assert np.array_equal(got, ref)
    if with_epilogue:
        yref = oracle.scale_bias(ref, data["scale"], data["bias"], "nchw")
        assert_f32_close(host(of), yref)
        assert np.array_equal(host(of), yref)


def test_cfg3_cifar_conv_full_size():
    print("cfg3", flush=True)
    _conv_parity(inputs.CFG3, inputs.cfg3())


def test_cfg5a_imagenet_conv_full_size():
    """All 51.4 M int32 outputs and the fp32 epilogue of the ImageNet-shaped 3x3 convolution."""
    print("cfg5a", flush=True)
    _conv_parity(inputs.CFG5A, inputs.cfg5a())


def test_cfg5b_ragged_k_pointwise_stride2_full_size():
    print("cfg5b", flush=True)
    _conv_parity(inputs.CFG5B, inputs.cfg5b())


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv2d_small_cases(case):
    print(f"conv case={case}", flush=True)
    N, C, H, W, D, kH, kW, sH, sW, pH, pW = case
    shape = inputs.ConvShape(N, C, H, W, D, kH, kW, sH, sW, pH, pW)
    _conv_parity(shape, inputs.conv_inputs(shape, seed=sum(case)))


def test_conv2d_worked_examples():
    print("conv worked examples", flush=True)
    x = torch.full((1, 1, 3, 3), -1.0, device=DEV)
    w = torch.full((1, 1, 3, 3), 1.0, device=DEV)
    oi, _ = B.bnn_conv2d(x, B.bnn_pack_conv_weight(w), 1, 3, 3, (1, 1), (1, 1))
    assert host(oi)[0, 0].tolist() == [[1, -3, 1], [-3, -9, -3], [1, -3, 1]]
    x = torch.tensor([[[[1.0, -1.0], [-1.0, 1.0]]]], device=DEV)
    w = torch.tensor([[[[1.0, -1.0, 1.0], [-1.0, 1.0, -1.0], [1.0, -1.0, 1.0]]]], device=DEV)
    oi, _ = B.bnn_conv2d(x, B.bnn_pack_conv_weight(w), 1, 3, 3, (1, 1), (1, 1))
    assert host(oi)[0, 0].tolist() == [[5, -3], [-3, 5]]


# ---------------------------------------------------------------- glue (a6) and the stack (cfg 4)
def test_maxpool_and_f32_glue():
    print("glue", flush=True)
    rng = np.random.default_rng(21)
    a = rng.integers(-1152, 1153, size=(3, 5, 8, 6)).astype(np.int32)
    sc = (rng.random(5) + 0.5).astype(np.float32)
    bi = (rng.standard_normal(5) * 0.1).astype(np.float32)
    oi, of = B.bnn_maxpool2x2(dev(a), dev(sc), dev(bi), want_int=True)
    ref = oracle.maxpool2x2_i32(a)
    assert np.array_equal(host(oi), ref)
    assert np.array_equal(host(of), oracle.scale_bias(ref, sc, bi, "nchw"))
    x = rng.standard_normal((3, 3, 9, 8)).astype(np.float32)
    w = rng.standard_normal((5, 3, 3, 3)).astype(np.float32)
    got = host(B.bnn_conv2d_f32(dev(x), dev(w), (1, 1), (1, 1), dev(sc), dev(bi)))
    assert np.array_equal(got, oracle.conv2d_f32_seq(x, w, (1, 1), (1, 1), sc, bi))
    got = host(B.bnn_conv2d_f32(dev(x), dev(w), (2, 1), (0, 1)))
    assert np.array_equal(got, oracle.conv2d_f32_seq(x, w, (2, 1), (0, 1)))
    xf = rng.standard_normal((6, 100)).astype(np.float32)
    wf = rng.standard_normal((10, 100)).astype(np.float32)
    bf = rng.standard_normal(10).astype(np.float32)
    for sgn in (False, True):
        got = host(B.bnn_fc_f32(dev(xf), dev(wf), dev(bf), sign_input=sgn))
        assert np.array_equal(got, oracle.fc_f32_seq(xf, wf, bf, sign_input=sgn))


@pytest.mark.parametrize("M,K,N", [(256, 1024, 10), (6, 100, 10), (5, 1023, 3), (33, 2500, 37), (1, 4, 1),
                                   (4100, 64, 20), (300, 1030, 250)])
@pytest.mark.parametrize("sgn", [False, True])
def test_fc_f32_matches_oracle(M, K, N, sgn):
    """Both workgroup shapes (4 and 16 rows), rows of several LDS passes, K off the 16-byte grid,
    output counts off the group of 16; with and without bias."""
    print(f"fc_f32 M={M} K={K} N={N} sign={sgn}", flush=True)
    rng = np.random.default_rng(M * 7 + K + N)
    xf = inputs.inject_specials(rng.standard_normal((M, K)).astype(np.float32), 4, frac=0.002, with_nan=False)
    wf = rng.standard_normal((N, K)).astype(np.float32)
    bf = rng.standard_normal(N).astype(np.float32)
    got = host(B.bnn_fc_f32(dev(xf), dev(wf), dev(bf), sign_input=sgn))
    ref = oracle.fc_f32_seq(xf, wf, bf, sign_input=sgn)
    assert np.array_equal(got, ref, equal_nan=True)
    got = host(B.bnn_fc_f32(dev(xf), dev(wf), None, sign_input=sgn))
    assert np.array_equal(got, oracle.fc_f32_seq(xf, wf, None, sign_input=sgn), equal_nan=True)


@pytest.mark.parametrize("reading", ["A", "B"])
def test_cfg4_stack_small_batch_every_layer(reading):
    print(f"cfg4 stack batch 4 reading {reading}", flush=True)
    from paper_1911_04477_amd.stack import VggStack
    d = inputs.cfg4(batch=4, reading=reading)
    net = VggStack(d["layers"], d["params"], batch=4, device=DEV)
    out, acts = net.forward(dev(d["x"]), keep=True)
    ref = oracle.vgg_stack(d["x"], d["layers"], d["params"])
    for i, (g, r) in enumerate(zip(acts, ref["acts"])):
        assert np.array_equal(host(g).reshape(r.shape), r), f"layer {i} ({d['layers'][i].kind})"
    assert np.array_equal(host(out), ref["out"])


@pytest.fixture(scope="module")
def cfg4_b256():
    """Config 4 at the benchmarked batch with the oracle's activations of every layer, all 256
    images (computed once for the tests that use it)."""
    d = inputs.cfg4(batch=256)
    print("oracle: cfg4 stack, 256 images", flush=True)
    ref = oracle.vgg_stack(d["x"], d["layers"], d["params"])
    return d, ref


def test_cfg4_stack_full_batch_every_layer_every_image(cfg4_b256):
    """Batch 256 as benchmarked, through bnn_conv2d and the glue kernels: the activation of every
    layer and the logits of all 256 images against the oracle, bit for bit."""
    print("cfg4 stack batch 256", flush=True)
    from paper_1911_04477_amd.stack import VggStack
    d, ref = cfg4_b256
    net = VggStack(d["layers"], d["params"], batch=256, device=DEV)
    out, acts = net.forward(dev(d["x"]), keep=True)
    for i, (g, r) in enumerate(zip(acts, ref["acts"])):
        assert np.array_equal(host(g).reshape(r.shape), r), f"layer {i} ({d['layers'][i].kind})"
    out = host(out)
    assert np.array_equal(out, ref["out"])
    del acts
    out2 = host(net.forward(dev(d["x"])))
    assert np.array_equal(out, out2)


# ---------------------------------------------------------------- timing hook
def test_prof_hook_records_kernels():
    print("prof hook", flush=True)
    d = inputs.cfg1()
    B.prof_enable(True)
    try:
        Ap, Bp = B.bnn_encode(dev(d["A"])), B.bnn_encode(dev(d["B"]))
        B.bnn_xnor_gemm(Ap, Bp, 256)
        rec = B.prof_records()
        assert [r[0] for r in rec] == ["encode_rows", "encode_rows", "xnor_gemm_lowk"]  # K = 256: the short-row kernel
        assert all(0.0 < r[1] < 50.0 for r in rec)
        B.prof_reset()
        assert B.prof_records() == []
    finally:
        B.prof_enable(False)


# ---------------------------------------------------------------- packed activations between layers
def _u64dev(a):
    return dev(np.ascontiguousarray(a).view(np.int64))


@pytest.mark.parametrize("case", [(2, 3, 10, 9, 128, 3, 3, 1, 1, 1, 1), (3, 3, 8, 8, 70, 3, 3, 2, 2, 1, 1),
                                  (1, 1, 6, 6, 5, 5, 5, 1, 1, 2, 2), (2, 2, 7, 7, 200, 3, 3, 1, 1, 0, 0),
                                  (2, 3, 10, 9, 200, 3, 3, 1, 1, 1, 1),    # two channel chunks, the second partial
                                  (1, 3, 40, 37, 257, 3, 3, 1, 1, 1, 1),   # five words per pixel, 24 pixel groups
                                  (3, 3, 9, 11, 31, 3, 3, 1, 2, 0, 1),     # fewer than 32 channels
                                  (2, 3, 5, 5, 1, 3, 3, 1, 1, 1, 1)])      # one channel
def test_conv2d_f32_sign_matches_oracle(case):
    print(f"conv2d_f32_sign case={case}", flush=True)
    N, C, H, W, D, kH, kW, sH, sW, pH, pW = case
    shape = inputs.ConvShape(*case)
    d = inputs.conv_inputs(shape, seed=sum(case) + 1)
    x = inputs.inject_specials(d["x"], 3, frac=0.01, with_nan=False)
    got = as_u64(B.bnn_conv2d_f32_sign(dev(x), dev(d["w"]), dev(d["scale"]), dev(d["bias"]), (sH, sW), (pH, pW)))
    ref = oracle.pack_nhwc(oracle.conv2d_f32_seq(x, d["w"], (sH, sW), (pH, pW), d["scale"], d["bias"]))
    assert np.array_equal(got, ref)


PACKED_CASES = CONV_CASES + [
    (2, 128, 8, 8, 64, 3, 3, 1, 1, 1, 1),
    (3, 128, 12, 10, 130, 3, 3, 1, 1, 1, 1),
    (2, 256, 6, 6, 256, 3, 3, 1, 1, 1, 1),
    (1, 64, 4, 6, 10, 3, 3, 1, 1, 1, 1),
    (1, 320, 16, 16, 70, 3, 3, 1, 1, 1, 1),
    (2, 100, 7, 9, 33, 3, 3, 1, 1, 1, 1),     # two words per pixel, the second partial
    (1, 128, 6, 8, 16, 5, 5, 1, 1, 2, 2),     # 25 taps
    (1, 128, 10, 10, 8, 6, 6, 1, 1, 2, 2),    # 36 taps: more than the tap mask of the lean gather holds
    (2, 128, 9, 9, 20, 3, 3, 2, 2, 1, 1),     # stride 2
    (2, 128, 6, 6, 12, 1, 1, 1, 1, 0, 0),     # rows of two words: a half chunk only
    (2, 192, 6, 6, 12, 1, 1, 1, 1, 0, 0),     # rows of three words (odd: general gather)
]


@pytest.mark.parametrize("cfg", [1, 3, 4, 6, 9, 19, 20])
@pytest.mark.parametrize("case", PACKED_CASES[-11:] + PACKED_CASES[1:4])
def test_conv2d_packed_forced_tiles(case, cfg):
    """The binarizing epilogue on every tile shape it is written for (the pooled form only
    exists for the four-column tiles; other requests fall back to a legal tile, and 9, a
    configuration only the explicit GEMM has, to the heuristic)."""
    print(f"conv2d_packed forced cfg={cfg} case={case}", flush=True)
    N, C, H, W, D, kH, kW, sH, sW, pH, pW = case
    shape = inputs.ConvShape(*case)
    d = inputs.conv_inputs(shape, seed=sum(case) + 3)
    xp = _u64dev(oracle.pack_nhwc(d["x"]))
    wp = B.bnn_pack_conv_weight(dev(d["w"]))
    sc, bi = dev(d["scale"]), dev(d["bias"])
    st, pd = (sH, sW), (pH, pW)
    ref = oracle.conv2d_pm1(d["x"], d["w"], st, pd)
    got = as_u64(B.bnn_conv2d_packed(xp, wp, C, D, kH, kW, st, pd, scale=sc, bias=bi, out="packed", cfg=cfg))
    assert np.array_equal(got, oracle.pack_nhwc(oracle.scale_bias(ref, d["scale"], d["bias"], "nchw")))
    if shape.OH % 2 == 0 and shape.OW % 2 == 0:
        pref = oracle.scale_bias(oracle.maxpool2x2_i32(ref), d["scale"], d["bias"], "nchw")
        got = as_u64(B.bnn_conv2d_packed(xp, wp, C, D, kH, kW, st, pd, pool=2, scale=sc, bias=bi, out="packed",
                                         cfg=cfg))
        assert np.array_equal(got, oracle.pack_nhwc(pref))
    assert np.array_equal(host(B.bnn_conv2d_packed(xp, wp, C, D, kH, kW, st, pd, out="i32", cfg=cfg)), ref)
    # the same forced tile through bnn_conv2d (fp32 image in, int32 NCHW out)
    oi, _ = B.bnn_conv2d(dev(d["x"]), wp, D, kH, kW, st, pd, want_int=True, cfg=cfg)
    assert np.array_equal(host(oi), ref)


@pytest.mark.parametrize("lean", [1, 0])
@pytest.mark.parametrize("case", PACKED_CASES)
def test_conv2d_packed_all_output_kinds(case, lean):
    """lean = 0 forces the general implicit-GEMM gather also where the lean one applies."""
    print(f"conv2d_packed case={case} lean={lean}", flush=True)
    _conv2d_packed_all_output_kinds(case, lean=lean)


def _conv2d_packed_all_output_kinds(case, lean=None):
    N, C, H, W, D, kH, kW, sH, sW, pH, pW = case
    shape = inputs.ConvShape(*case)
    d = inputs.conv_inputs(shape, seed=sum(case) + 2)
    x = inputs.inject_specials(d["x"], 4, frac=0.01)
    xp = _u64dev(oracle.pack_nhwc(x))
    wp = B.bnn_pack_conv_weight(dev(d["w"]))
    sc, bi = dev(d["scale"]), dev(d["bias"])
    st, pd = (sH, sW), (pH, pW)
    ref = oracle.conv2d_pm1(x, d["w"], st, pd)
    assert np.array_equal(host(B.bnn_conv2d_packed(xp, wp, C, D, kH, kW, st, pd, out="i32", lean=lean)), ref)
    yref = oracle.scale_bias(ref, d["scale"], d["bias"], "nchw")
    assert np.array_equal(host(B.bnn_conv2d_packed(xp, wp, C, D, kH, kW, st, pd, scale=sc, bias=bi, out="f32", lean=lean)), yref)
    got = as_u64(B.bnn_conv2d_packed(xp, wp, C, D, kH, kW, st, pd, scale=sc, bias=bi, out="packed", lean=lean))
    assert np.array_equal(got, oracle.pack_nhwc(yref))
    if shape.OH % 2 == 0 and shape.OW % 2 == 0:
        pref = oracle.scale_bias(oracle.maxpool2x2_i32(ref), d["scale"], d["bias"], "nchw")
        got = as_u64(B.bnn_conv2d_packed(xp, wp, C, D, kH, kW, st, pd, pool=2, scale=sc, bias=bi, out="packed", lean=lean))
        assert np.array_equal(got, oracle.pack_nhwc(pref))


def _random_geometries(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        N = int(rng.integers(1, 4))
        C = int(rng.choice([1, 3, 17, 63, 64, 65, 100, 128, 129, 192, 200, 256]))
        H, W = int(rng.integers(3, 13)), int(rng.integers(3, 13))
        kH, kW = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        sH, sW = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        pH, pW = int(rng.integers(0, 3)), int(rng.integers(0, 3))
        D = int(rng.choice([1, 7, 31, 32, 33, 64, 65, 100, 130]))
        if H + 2 * pH < kH or W + 2 * pW < kW:
            continue
        out.append((N, C, H, W, D, kH, kW, sH, sW, pH, pW))
    return out


@pytest.mark.parametrize("case", _random_geometries(36, seed=20191104))
def test_conv_entry_points_on_random_geometries(case):
    """Seeded random shapes (kernel sizes 1..5, strides 1..3, pads 0..2, channel counts on and
    off the word grid) through bnn_conv2d, bnn_im2col_packed and every output kind of
    bnn_conv2d_packed."""
    print(f"random geometry case={case}", flush=True)
    N, C, H, W, D, kH, kW, sH, sW, pH, pW = case
    shape = inputs.ConvShape(*case)
    d = inputs.conv_inputs(shape, seed=sum(case) + 11)
    _conv_parity(shape, d)
    _conv2d_packed_all_output_kinds(case)
    x = inputs.inject_specials(d["x"], 5, frac=0.01)
    cols = as_u64(B.bnn_im2col_packed(dev(x), kH, kW, (sH, sW), (pH, pW)))
    assert np.array_equal(cols, oracle.im2col_packed(x, kH, kW, (sH, sW), (pH, pW)))


def test_conv2d_packed_negative_scale_and_pool_order():
    """With a negative scale the affine map is decreasing: pooling must act on the int32
    accumulators before the affine map, not on its result."""
    print("conv2d_packed negative scale", flush=True)
    shape = inputs.ConvShape(2, 128, 8, 8, 64, 3, 3, 1, 1, 1, 1)
    d = inputs.conv_inputs(shape, seed=77)
    scale = -d["scale"]
    xp = _u64dev(oracle.pack_nhwc(d["x"]))
    wp = B.bnn_pack_conv_weight(dev(d["w"]))
    ref = oracle.maxpool2x2_i32(oracle.conv2d_pm1(d["x"], d["w"], (1, 1), (1, 1)))
    pref = oracle.pack_nhwc(oracle.scale_bias(ref, scale, d["bias"], "nchw"))
    got = as_u64(B.bnn_conv2d_packed(xp, wp, 128, 64, 3, 3, (1, 1), (1, 1), pool=2, scale=dev(scale),
                                     bias=dev(d["bias"]), out="packed"))
    assert np.array_equal(got, pref)


def test_pack_fc_weight_nhwc_matches_oracle():
    print("pack_fc_weight_nhwc", flush=True)
    rng = np.random.default_rng(41)
    for (n_out, C, H, W) in [(10, 70, 2, 3), (33, 512, 4, 4), (4, 64, 1, 1)]:
        w = rng.standard_normal((n_out, C * H * W)).astype(np.float32)
        got = as_u64(B.bnn_pack_fc_weight_nhwc(dev(w), C, H, W))
        assert np.array_equal(got, oracle.pack_fc_weight_nhwc(w, C, H, W))


@pytest.mark.parametrize("reading", ["A", "B"])
def test_cfg4_fused_stack_small_batch_every_layer(reading):
    print(f"cfg4 fused stack batch 4 reading {reading}", flush=True)
    from paper_1911_04477_amd.stack import VggStackFused
    d = inputs.cfg4(batch=4, reading=reading)
    net = VggStackFused(d["layers"], d["params"], batch=4, device=DEV)
    out, acts = net.forward(dev(d["x"]), keep=True)
    ref = oracle.vgg_stack(d["x"], d["layers"], d["params"])
    for i, (L, g, r) in enumerate(zip(d["layers"], acts, ref["acts"])):
        if L.kind in ("conv_f32", "bconv"):
            assert np.array_equal(as_u64(g), oracle.pack_nhwc(r)), f"layer {i} ({L.kind})"
        else:
            assert np.array_equal(host(g), r), f"layer {i} ({L.kind})"
    assert np.array_equal(host(out), ref["out"])


def test_cfg4_fused_stack_full_batch_is_deterministic():
    """Twenty passes at the benchmark's batch size give the same bits every time, layer by layer
    (a race between waves would show up as a difference between passes)."""
    print("cfg4 fused stack batch 256, repeated passes", flush=True)
    from paper_1911_04477_amd.stack import VggStackFused
    d = inputs.cfg4(batch=256)
    net = VggStackFused(d["layers"], d["params"], batch=256, device=DEV)
    x = dev(d["x"])
    out0, acts0 = net.forward(x, keep=True)
    torch.cuda.synchronize()
    for rep in range(20):
        out, acts = net.forward(x, keep=True)
        for i, (a, b) in enumerate(zip(acts0, acts)):
            assert torch.equal(a, b), f"pass {rep}, layer {i}"
        assert torch.equal(out0, out), f"pass {rep}"


def test_cfg4_fused_stack_graph_replays_match_oracle():
    """The fused pass captured into a HIP graph: every replay (new input contents each time,
    eager work and synchronisations of this process in between) must give the oracle's result
    for the input it ran on."""
    print("cfg4 fused stack, graph replays", flush=True)
    from paper_1911_04477_amd.stack import VggStackFused
    batch = 4
    d = inputs.cfg4(batch=batch)
    net = VggStackFused(d["layers"], d["params"], batch=batch, device=DEV)
    xbuf = dev(d["x"]).clone()
    net.capture(xbuf)
    rng = np.random.default_rng(5)
    for rep in range(4):
        x = d["x"] if rep == 0 else rng.standard_normal(d["x"].shape).astype(np.float32)
        xbuf.copy_(dev(x))
        got = host(net.replay()).copy()
        ref = oracle.vgg_stack(x, d["layers"], d["params"])["out"]
        assert np.array_equal(got, ref), f"replay {rep}"
        # eager work between replays: the same pass outside the graph, and an unrelated GEMM
        assert np.array_equal(host(net.forward(xbuf)), ref), f"eager pass after replay {rep}"
        _gemm_case(9, 70, 200, seed=rep)


def test_cfg4_fused_stack_full_batch_every_layer_every_image(cfg4_b256):
    """The benchmark's default step (packed activations between layers, batch 256): every layer's
    packed activation and the logits of all 256 images against the oracle."""
    print("cfg4 fused stack batch 256", flush=True)
    from paper_1911_04477_amd.stack import VggStackFused
    d, ref = cfg4_b256
    net = VggStackFused(d["layers"], d["params"], batch=256, device=DEV)
    out, acts = net.forward(dev(d["x"]), keep=True)
    for i, (L, g, r) in enumerate(zip(d["layers"], acts, ref["acts"])):
        if L.kind in ("conv_f32", "bconv"):
            assert np.array_equal(as_u64(g), oracle.pack_nhwc(r)), f"layer {i} ({L.kind})"
        else:
            assert np.array_equal(host(g), r), f"layer {i} ({L.kind})"
    assert np.array_equal(host(out), ref["out"])


# ---------------------------------------------------------------- MFMA ablation
@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (37, 150, 300), (128, 128, 64), (130, 257, 1152), (64, 64, 256),
                                   (200, 333, 2304 + 17), (5, 700, 63),
                                   (300, 3300, 200), (513, 1650, 127)])
def test_mfma_ablation_matches_oracle(M, N, K):
    print(f"mfma M={M} N={N} K={K}", flush=True)
    rng = np.random.default_rng(M * 7919 + N * 31 + K)
    A = inputs.inject_specials(rng.standard_normal((M, K)).astype(np.float32), 1, frac=0.002)
    Bm = inputs.inject_specials(rng.standard_normal((N, K)).astype(np.float32), 2, frac=0.002)
    Ap, Bp = B.bnn_encode(dev(A)), B.bnn_encode(dev(Bm))
    ref = oracle.gemm_pm1(A, Bm)
    assert np.array_equal(host(B.bnn_xnor_gemm_mfma_i8(Ap, Bp, K)), ref)
    assert np.array_equal(host(B.bnn_xnor_gemm_mfma_fp4(Ap, Bp, K)), ref)


def test_mfma_ablation_equals_valu_path_at_cfg2():
    print("mfma cfg2", flush=True)
    d = inputs.cfg2()
    Ap, Wp = B.bnn_encode(dev(d["act"])), B.bnn_encode(dev(d["wt"]))
    a = host(B.bnn_xnor_gemm_mfma_i8(Ap, Wp, inputs.CFG2.K))
    b = host(B.bnn_xnor_gemm(Ap, Wp, inputs.CFG2.K))
    assert np.array_equal(a, b)
    assert np.array_equal(host(B.bnn_xnor_gemm_mfma_fp4(Ap, Wp, inputs.CFG2.K)), b)


def _e2m1_rows(x):
    """Rows of +-1 values as 4-bit floating-point codes, written out from the format's definition:
    +1.0 is 0x2, -1.0 is 0xA, value k in nibble k % 2 (low first) of byte k / 2, rows padded with
    0.0 (0x0) to a multiple of 64 values."""
    rows, K = x.shape
    Kp = (K + 63) // 64 * 64
    codes = np.zeros((rows, Kp), dtype=np.uint8)
    codes[:, :K] = np.where(x >= 0, 0x2, 0xA)
    return (codes[:, 0::2] | (codes[:, 1::2] << 4)).astype(np.uint8)


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (37, 150, 300), (128, 128, 64), (130, 257, 1152), (64, 64, 256),
                                   (200, 333, 2304 + 17), (5, 700, 63), (300, 3300, 200), (513, 1650, 127),
                                   (256, 1000, 128), (260, 129, 192)])
def test_mfma_fp4_expanded_ablation_matches_oracle(M, N, K):
    """Operands kept in memory as E2M1 +-1 rows: the expansion pass against the format's definition,
    the GEMM on every workgroup tile against the oracle."""
    print(f"mfma fp4 expanded M={M} N={N} K={K}", flush=True)
    rng = np.random.default_rng(M * 7919 + N * 31 + K + 5)
    A = inputs.inject_specials(rng.standard_normal((M, K)).astype(np.float32), 1, frac=0.002)
    Bm = inputs.inject_specials(rng.standard_normal((N, K)).astype(np.float32), 2, frac=0.002)
    A4, B4 = B.bnn_expand_fp4(B.bnn_encode(dev(A)), K), B.bnn_expand_fp4(B.bnn_encode(dev(Bm)), K)
    assert np.array_equal(host(A4), _e2m1_rows(A))
    assert np.array_equal(host(B4), _e2m1_rows(Bm))
    ref = oracle.gemm_pm1(A, Bm)
    for tile in (None, 0, 1, 2):
        assert np.array_equal(host(B.bnn_xnor_gemm_mfma_fp4_expanded(A4, B4, K, tile=tile)), ref), f"tile {tile}"


def test_mfma_fp4_expanded_strided_operands_and_output():
    """Leading dimensions larger than the rows: operands inside wider buffers, C inside a wider matrix."""
    print("mfma fp4 expanded strided", flush=True)
    M, N, K = 70, 200, 330
    rng = np.random.default_rng(77)
    A = rng.standard_normal((M, K)).astype(np.float32)
    Bm = rng.standard_normal((N, K)).astype(np.float32)
    rb = 32 * ((K + 63) // 64)
    A4w = torch.full((M, rb + 48), 0x77, dtype=torch.uint8, device="cuda")
    B4w = torch.full((N, rb + 16), 0x77, dtype=torch.uint8, device="cuda")
    B.bnn_expand_fp4(B.bnn_encode(dev(A)), K, out=A4w[:, :rb])
    B.bnn_expand_fp4(B.bnn_encode(dev(Bm)), K, out=B4w[:, :rb])
    assert np.array_equal(host(A4w[:, :rb]), _e2m1_rows(A)) and bool((A4w[:, rb:] == 0x77).all())
    Cw = torch.full((M, N + 24), -7, dtype=torch.int32, device="cuda")
    B.bnn_xnor_gemm_mfma_fp4_expanded(A4w[:, :rb], B4w[:, :rb], K, C=Cw[:, :N])
    assert np.array_equal(host(Cw[:, :N]), oracle.gemm_pm1(A, Bm))
    assert bool((Cw[:, N:] == -7).all())


@pytest.mark.parametrize("case", [(2, 64, 9, 7, 40, 3, 3, 1, 1, 1, 1), (3, 128, 12, 12, 130, 3, 3, 1, 1, 1, 1),
                                  (2, 192, 11, 10, 70, 3, 3, 2, 2, 1, 1), (1, 64, 8, 8, 300, 1, 1, 1, 1, 0, 0),
                                  (2, 128, 9, 9, 33, 5, 3, 1, 2, 2, 0), (2, 256, 14, 14, 256, 3, 3, 1, 1, 1, 1),
                                  (5, 64, 6, 6, 17, 2, 2, 1, 1, 1, 1)])
def test_conv2d_mfma_fp4_expanded_matches_oracle(case):
    """The matrix-core ablation as a convolution: patches gathered from the 4-bit NHWC image."""
    print(f"conv2d mfma fp4 expanded case={case}", flush=True)
    N, C, H, W, D, kH, kW, sH, sW, pH, pW = case
    d = inputs.conv_inputs(inputs.ConvShape(*case), seed=sum(case) + 23)
    x = inputs.inject_specials(d["x"], 7, frac=0.01)
    Cw = C // 64
    x4 = B.bnn_expand_fp4(_u64dev(oracle.pack_nhwc(x)).view(N * H * W, Cw), C).view(N, H, W, C // 2)
    assert np.array_equal(host(x4).reshape(N * H * W, C // 2), _e2m1_rows(x.transpose(0, 2, 3, 1).reshape(N * H * W, C)))
    w4 = B.bnn_expand_fp4(B.bnn_pack_conv_weight(dev(d["w"])), C * kH * kW)
    got = host(B.bnn_conv2d_mfma_fp4_expanded(x4, w4, C, D, kH, kW, (sH, sW), (pH, pW)))
    assert np.array_equal(got, oracle.conv2d_pm1(x, d["w"], (sH, sW), (pH, pW)))


# ---------------------------------------------------------------- fp32 control group (section 4.4)
@pytest.mark.parametrize("case", PACKED_CASES + [(1, 3, 5, 5, 130, 3, 3, 1, 1, 1, 1), (2, 40, 20, 20, 200, 3, 3, 2, 2, 0, 0)])
def test_control_group_conv_equals_binarized_result(case):
    """The real-valued GEMM on sign(x), sign(w) gives the same integers as the oracle (and so as
    the Xnor-Bitcount path), exactly: all partial sums are integers below 2^24."""
    print(f"control conv case={case}", flush=True)
    N, C, H, W, D, kH, kW, sH, sW, pH, pW = case
    shape = inputs.ConvShape(*case)
    d = inputs.conv_inputs(shape, seed=sum(case) + 5)
    x = inputs.inject_specials(d["x"], 6, frac=0.01)
    got = host(B.bnn_control_conv2d_f32(dev(x), dev(d["w"]), (sH, sW), (pH, pW)))
    ref = oracle.conv2d_pm1(x, d["w"], (sH, sW), (pH, pW))
    assert got.dtype == np.float32 and np.array_equal(got, ref.astype(np.float32))


def test_control_group_conv_cfg3_full_size():
    print("control conv cfg3", flush=True)
    d = inputs.cfg3()
    s = inputs.CFG3
    got = host(B.bnn_control_conv2d_f32(dev(d["x"]), dev(d["w"]), (s.sH, s.sW), (s.pH, s.pW)))
    ref = oracle.conv2d_pm1(d["x"], d["w"], (s.sH, s.sW), (s.pH, s.pW))
    assert np.array_equal(got, ref.astype(np.float32))


# ---------------------------------------------------------------- sizes far off the tile grid
def _popcount_rows(a_words, b_words, K):
    """K - 2 * popcount(a xor b) for every pair of packed rows, with numpy only: the identity the
    oracle's float GEMM is pinned against, usable where K >= 2^24 puts that fp32 sum out of its
    exact range."""
    x = a_words[:, None, :] ^ b_words[None, :, :]
    cnt = np.unpackbits(x.view(np.uint8), axis=-1).sum(axis=-1, dtype=np.int64)
    return (K - 2 * cnt).astype(np.int32)


@pytest.mark.parametrize("cfg", [-1, 3, 7, 9, 14, 15])
def test_gemm_very_long_rows(cfg):
    """K = 2^24 + 77 bits: 65536 full chunks and a ragged tail per row, accumulators in the millions."""
    print(f"gemm long K cfg={cfg}", flush=True)
    M, N, K = 3, 5, (1 << 24) + 77
    rng = np.random.default_rng(77)
    A = rng.standard_normal((M, K)).astype(np.float32)
    Bm = rng.standard_normal((N, K)).astype(np.float32)
    Bm[1] = A[0]            # one identical pair: C = K
    Bm[2] = -A[1]           # one opposite pair: C = -K (no zeros in a normal sample)
    Ap, Bp = B.bnn_encode(dev(A)), B.bnn_encode(dev(Bm))
    got = host(B.bnn_xnor_gemm(Ap, Bp, K, cfg=None if cfg < 0 else cfg))
    assert got[0, 1] == K and got[1, 2] == -K
    # rows encoded by the oracle, not by the GPU
    assert np.array_equal(got, _popcount_rows(oracle.encode_rows(A), oracle.encode_rows(Bm), K))
    # the first 2^24 - 1 columns through the float oracle, the rest by the identity
    K0 = (1 << 24) - 1
    head = oracle.gemm_pm1(np.ascontiguousarray(A[:, :K0]), np.ascontiguousarray(Bm[:, :K0]))
    tail = _popcount_rows(oracle.encode_rows(np.ascontiguousarray(A[:, K0:])),
                          oracle.encode_rows(np.ascontiguousarray(Bm[:, K0:])), K - K0)
    assert np.array_equal(got, head + tail)


def test_gemm_many_columns():
    """N = 1.5 million columns (grid far beyond 65535 workgroups), K = 100 (masked tail only)."""
    print("gemm many columns", flush=True)
    M, N, K = 9, 1_500_001, 100
    rng = np.random.default_rng(5)
    A = rng.standard_normal((M, K)).astype(np.float32)
    Bm = rng.standard_normal((N, K)).astype(np.float32)
    got = host(B.bnn_xnor_gemm(B.bnn_encode(dev(A)), B.bnn_encode(dev(Bm)), K))
    assert np.array_equal(got, oracle.gemm_pm1(A, Bm))


@pytest.mark.parametrize("N,C", [(255, 128), (510, 64)])
def test_conv2d_packed_largest_images(N, C):
    """Batches at the documented limit of N*C*H*W (2^33 values): 67 / 134 million pixels, a packed input of
    1 GiB; C = 128 takes the table-driven gather, C = 64 (one word per pixel) the general one.  The batch
    repeats three distinct images, so every image's result is known from the oracle's three."""
    print(f"conv2d_packed largest images N={N} C={C}", flush=True)
    H, W, D, st, pd = 512, 512, 8, (1, 1), (1, 1)
    d = inputs.conv_inputs(inputs.ConvShape(3, C, H, W, D, 3, 3, 1, 1, 1, 1), seed=N)
    x = inputs.inject_specials(d["x"], 6, frac=0.001)
    ref = oracle.conv2d_pm1(x, d["w"], st, pd)
    xp = _u64dev(oracle.pack_nhwc(x)).repeat(N // 3, 1, 1, 1)
    wp = B.bnn_pack_conv_weight(dev(d["w"]))
    # one image more is beyond the range: refused, nothing launched
    with pytest.raises(B.BnnError):
        B.bnn_conv2d_packed(torch.cat([xp, xp[:3]]), wp, C, D, 3, 3, st, pd, out="i32")
    out = B.bnn_conv2d_packed(xp, wp, C, D, 3, 3, st, pd, out="i32")
    torch.cuda.synchronize()
    assert torch.equal(out.view(N // 3, 3, D, H, W), dev(ref).expand(N // 3, 3, D, H, W))
    del out
    sc, bi = dev(d["scale"]), dev(d["bias"])
    pref = oracle.pack_nhwc(oracle.scale_bias(oracle.maxpool2x2_i32(ref), d["scale"], d["bias"], "nchw"))
    got = B.bnn_conv2d_packed(xp, wp, C, D, 3, 3, st, pd, pool=2, scale=sc, bias=bi, out="packed")
    torch.cuda.synchronize()
    assert torch.equal(got.view(N // 3, 3, H // 2, W // 2, 1), _u64dev(pref).expand(N // 3, 3, H // 2, W // 2, 1))
    del xp, got
    torch.cuda.empty_cache()
    if C == 128:
        # the same batch as fp32 NCHW (34 GB) through bnn_conv2d: its encode, then the same GEMM
        xf = dev(x).repeat(N // 3, 1, 1, 1)
        oi, _ = B.bnn_conv2d(xf, wp, D, 3, 3, st, pd)
        torch.cuda.synchronize()
        assert torch.equal(oi.view(N // 3, 3, D, H, W), dev(ref).expand(N // 3, 3, D, H, W))
        del xf, oi
        torch.cuda.empty_cache()


def _pm1_rows(packed, K):
    """Packed rows (uint64 words, element k in bit k % 64 of word k / 64, bit 1 = +1) as +-1 floats."""
    bits = np.unpackbits(np.ascontiguousarray(packed).view(np.uint8), axis=-1, bitorder="little")[:, :K]
    return np.where(bits == 1, 1.0, -1.0).astype(np.float32)


@pytest.mark.parametrize("N,K", [((1 << 31) - 257, 64), ((1 << 31) - 260, 128)])
def test_gemm_maximum_column_count(N, K):
    """The largest column count the header allows (2^31 - 257; the second case is the largest multiple of 4,
    which the short-row kernel takes): 17 / 34 GB of packed rows, 17 GB of output, checked on the first and
    last columns and on a random sample, against the oracle."""
    print(f"gemm max columns N={N} K={K}", flush=True)
    M, Kw = 2, K // 64
    g = torch.Generator(device="cuda").manual_seed(191104477)
    Bp = torch.randint(-2**63, 2**63 - 1, (N, Kw), dtype=torch.int64, device="cuda", generator=g)
    Ap = torch.randint(-2**63, 2**63 - 1, (M, Kw), dtype=torch.int64, device="cuda", generator=g)
    C = B.bnn_xnor_gemm(Ap, Bp, K)
    rng = np.random.default_rng(3)
    idx = np.unique(np.concatenate([np.arange(0, 1024), np.arange(N - 1024, N),
                                    rng.integers(0, N, size=200_000)])).astype(np.int64)
    it = torch.from_numpy(idx).cuda()
    got = host(C[:, it])
    rows = host(Bp[it]).view(np.uint64)
    ref = oracle.gemm_pm1(_pm1_rows(host(Ap).view(np.uint64), K), _pm1_rows(rows, K))
    assert np.array_equal(got, ref)
    del Bp, C
    torch.cuda.empty_cache()


def test_fused_stack_split_over_two_streams_matches_oracle():
    print("split batch over two streams", flush=True)
    from paper_1911_04477_amd.stack import SplitBatch
    d = inputs.cfg4(batch=6)
    sb = SplitBatch(d["layers"], d["params"], batch=6, parts=2, device=DEV)
    x = dev(d["x"])
    want = oracle.vgg_stack(d["x"], d["layers"], d["params"])["out"]
    for _ in range(3):  # replays reuse the per-slice buffers
        outs = sb.forward(x)
        got = np.concatenate([host(o) for o in outs], axis=0)
        assert np.array_equal(got, want)


def test_f32_glue_hand_worked_cases(golden_dir):
    """The hand-worked order / rounding cases of the real-valued layers, straight against the
    stored values (no oracle in between)."""
    import json
    import os
    with open(os.path.join(golden_dir, "f32_glue_order_examples.json")) as f:
        cases = json.load(f)
    f32 = lambda v: np.array([float(t) for t in v], dtype=np.float32)
    for c in cases["conv"]:
        print(f"conv2d_f32 hand-worked {c['name']}", flush=True)
        x, w = f32(c["x"]).reshape(c["x_shape"]), f32(c["w"]).reshape(c["w_shape"])
        args = (dev(x), dev(w), tuple(c["stride"]), tuple(c["pad"]))
        if "scale" in c:
            args += (dev(f32(c["scale"])), dev(f32(c["bias"])))
        got = host(B.bnn_conv2d_f32(*args)).ravel()
        assert np.array_equal(got, f32(c["out"]), equal_nan=True), (c["name"], got)
    for c in cases["fc"]:
        print(f"fc_f32 hand-worked {c['name']}", flush=True)
        x, w = np.array(c["x"], dtype=np.float32), np.array(c["w"], dtype=np.float32)
        got = host(B.bnn_fc_f32(dev(x), dev(w), dev(f32(c["bias"])), sign_input=c["sign_input"]))
        assert np.array_equal(got, np.array(c["out"], dtype=np.float32)), (c["name"], got)


@pytest.mark.parametrize("xs,ws", [(1e-25, 1e-15), (1e-38, 1.0), (1e18, 1e18), (1.0, 1e-44)])
def test_conv2d_f32_first_layer_chain_rounds_like_fmaf(xs, ws):
    """The 3x3x3 layer runs its (c, kh, kw) chain on the fp32 matrix cores, one reduction step
    per instruction; it must round exactly like the oracle's fmaf chain also where products or
    sums are subnormal, underflow to zero, or overflow."""
    case = (2, 3, 9, 8, 45, 3, 3, 1, 1, 1, 1)
    print(f"conv2d_f32 extreme magnitudes xs={xs} ws={ws}", flush=True)
    shape = inputs.ConvShape(*case)
    d = inputs.conv_inputs(shape, seed=77)
    x = (d["x"].astype(np.float64) * xs).astype(np.float32)
    w = (d["w"].astype(np.float64) * ws).astype(np.float32)
    got = host(B.bnn_conv2d_f32(dev(x), dev(w), (1, 1), (1, 1)))
    ref = oracle.conv2d_f32_seq(x, w, (1, 1), (1, 1))
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    assert np.array_equal(got.view(np.uint32)[~np.isnan(ref)], ref.view(np.uint32)[~np.isnan(ref)])
    sc = np.ones(45, np.float32)
    bi = np.zeros(45, np.float32)
    gp = as_u64(B.bnn_conv2d_f32_sign(dev(x), dev(w), dev(sc), dev(bi), (1, 1), (1, 1)))
    assert np.array_equal(gp, oracle.pack_nhwc(oracle.conv2d_f32_seq(x, w, (1, 1), (1, 1), sc, bi)))
    # an infinite filter tap: NaN wherever it meets a padding zero, on both sides
    w2 = w.copy()
    w2[0, 0, 0, 0] = np.inf
    w2[7, 2, 2, 1] = -np.inf
    got = host(B.bnn_conv2d_f32(dev(x), dev(w2), (1, 1), (1, 1)))
    ref = oracle.conv2d_f32_seq(x, w2, (1, 1), (1, 1))
    assert np.isnan(ref).any() and np.array_equal(np.isnan(got), np.isnan(ref))
    assert np.array_equal(got, ref, equal_nan=True)
    gp = as_u64(B.bnn_conv2d_f32_sign(dev(x), dev(w2), dev(sc), dev(bi), (1, 1), (1, 1)))
    assert np.array_equal(gp, oracle.pack_nhwc(oracle.conv2d_f32_seq(x, w2, (1, 1), (1, 1), sc, bi)))


@pytest.mark.parametrize("case", [(2, 3, 10, 9, 128, 3, 3, 1, 1, 1, 1), (3, 3, 8, 8, 70, 3, 3, 2, 2, 1, 1),
                                  (1, 3, 7, 5, 5, 3, 3, 1, 2, 0, 1), (2, 4, 6, 6, 9, 3, 3, 1, 1, 1, 1),
                                  (2, 3, 6, 6, 9, 5, 5, 1, 1, 2, 2), (1, 3, 20, 19, 161, 3, 3, 1, 1, 1, 1)])
@pytest.mark.parametrize("affine", [True, False])
def test_conv2d_f32_real_valued_layer(case, affine):
    """fp32 convolution with fp32 output: the 3-channel 3x3 form runs on the matrix-core kernel,
    other geometries on the general one; both follow the (c, kh, kw) fma order."""
    print(f"conv2d_f32 case={case} affine={affine}", flush=True)
    N, C, H, W, D, kH, kW, sH, sW, pH, pW = case
    shape = inputs.ConvShape(*case)
    d = inputs.conv_inputs(shape, seed=sum(case) + 9)
    x = inputs.inject_specials(d["x"], 8, frac=0.01, with_nan=False)
    if affine:
        got = host(B.bnn_conv2d_f32(dev(x), dev(d["w"]), (sH, sW), (pH, pW), dev(d["scale"]), dev(d["bias"])))
        ref = oracle.conv2d_f32_seq(x, d["w"], (sH, sW), (pH, pW), d["scale"], d["bias"])
    else:
        got = host(B.bnn_conv2d_f32(dev(x), dev(d["w"]), (sH, sW), (pH, pW)))
        ref = oracle.conv2d_f32_seq(x, d["w"], (sH, sW), (pH, pW))
    # injected infinities of both signs meet in some sums: NaN there on both sides
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    assert np.array_equal(got, ref, equal_nan=True)


# ---------------------------------------------------------------- whatever the size heuristic picks
def test_heuristic_kernel_selection_on_random_gemm_shapes():
    """Seeded random (M, N, K) on and off every grid through the entry points as an application
    calls them: the host chooses between the throughput, one-wave, split-K and short-row kernels."""
    rng = np.random.default_rng(1234)
    done = 0
    while done < 80:
        M = int(rng.choice([1, 3, 8, 31, 32, 33, 64, 100, 256, 300, 513]))
        N = int(rng.choice([1, 4, 60, 64, 68, 128, 200, 256, 1000, 1024, 4100]))
        K = int(rng.choice([1, 64, 65, 128, 200, 256, 257, 1000, 2048, 4096, 4100, 8192]))
        if M * N * K > 2e9:
            continue
        done += 1
        print(f"heuristic gemm M={M} N={N} K={K}", flush=True)
        A = rng.standard_normal((M, K)).astype(np.float32)
        Bm = rng.standard_normal((N, K)).astype(np.float32)
        sc = ((rng.random(N) + 0.5) * rng.choice([-1.0, 1.0], N)).astype(np.float32)
        bi = rng.standard_normal(N).astype(np.float32)
        C, Y = B.bnn_xnor_gemm_epilogue(B.bnn_encode(dev(A)), B.bnn_encode(dev(Bm)), K, dev(sc), dev(bi), B.CH_COL,
                                        want_int=True)
        ref = oracle.gemm_pm1(A, Bm)
        assert np.array_equal(host(C), ref), (M, N, K)
        assert np.array_equal(host(Y), oracle.scale_bias(ref, sc, bi, "col")), (M, N, K)


def test_heuristic_kernel_selection_on_random_packed_convs():
    """Seeded random layer shapes (few to many output pixels, scales of both signs) through
    bnn_conv2d_packed as the stack calls it: latency form, throughput tiles, short-row kernel."""
    rng = np.random.default_rng(4321)
    for it in range(60):
        N = int(rng.integers(1, 9))
        C = int(rng.choice([64, 128, 130, 192, 256, 512]))
        H, W = int(rng.choice([4, 6, 8, 10, 16])), int(rng.choice([4, 6, 8, 12, 16]))
        D = int(rng.choice([8, 31, 32, 33, 64, 100, 128, 256]))
        k = int(rng.choice([1, 3]))
        p = k // 2
        shape = inputs.ConvShape(N, C, H, W, D, k, k, 1, 1, p, p)
        print(f"heuristic conv {shape}", flush=True)
        d = inputs.conv_inputs(shape, seed=1000 + it)
        sc = (d["scale"] * rng.choice([-1.0, 1.0], D)).astype(np.float32)
        xp = _u64dev(oracle.pack_nhwc(d["x"]))
        wp = B.bnn_pack_conv_weight(dev(d["w"]))
        ref = oracle.conv2d_pm1(d["x"], d["w"], (1, 1), (p, p))
        assert np.array_equal(host(B.bnn_conv2d_packed(xp, wp, C, D, k, k, (1, 1), (p, p), out="i32")), ref)
        got = as_u64(B.bnn_conv2d_packed(xp, wp, C, D, k, k, (1, 1), (p, p), scale=dev(sc), bias=dev(d["bias"]),
                                         out="packed"))
        assert np.array_equal(got, oracle.pack_nhwc(oracle.scale_bias(ref, sc, d["bias"], "nchw")))
        got = as_u64(B.bnn_conv2d_packed(xp, wp, C, D, k, k, (1, 1), (p, p), pool=2, scale=dev(sc),
                                         bias=dev(d["bias"]), out="packed"))
        assert np.array_equal(got, oracle.pack_nhwc(oracle.scale_bias(oracle.maxpool2x2_i32(ref), sc, d["bias"], "nchw")))
