"""GPU parity: every step of the SwitchBack layer, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Bars: int8 codes, states and int32 accumulators bit-exact; dequantized outputs within 1 binary32
ulp before the bf16 cast (bf16 outputs must be the rounding of a value within that ulp); weight gradient
max-abs error <= 1e-2 * rms(dW) in binary32 output mode."""
import numpy as np
import pytest
import torch

from paper_2304_13013_amd import inputs as I
from paper_2304_13013_amd import switchback as sb

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def to_dev(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(DEV).view(torch.bfloat16)


def bits_of(t):
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def host(t):
    return t.detach().cpu().numpy()


def ulp(ref):
    return np.spacing(np.abs(ref).astype(np.float32))


def assert_bf16_is_rounding_within_one_ulp(got_bits, ref32, oracle):
    """The bf16 result must equal RNE(v) for some v in {ref - 1ulp, ref, ref + 1ulp}."""
    u = ulp(ref32)
    cands = [oracle.round_to_bf16(ref32), oracle.round_to_bf16(ref32 - u), oracle.round_to_bf16(ref32 + u)]
    ok = (got_bits == cands[0]) | (got_bits == cands[1]) | (got_bits == cands[2])
    assert ok.all(), "%d bf16 outputs are not the rounding of a value within 1 ulp" % int((~ok).sum())


def rand_bf16(rng, shape, scale=1.0):
    return I.f32_to_bf16_bits((rng.standard_normal(shape) * scale).astype(np.float32))


# ---------------------------------------------------------------------------------------------------------------
# quantizers
# ---------------------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("rows,cols", [
    (512, 256), (1, 8), (3, 64), (5, 520), (257, 1280), (66, 2048), (9, 2056), (130, 3072), (33, 5120),
    (7, 8192), (5, 12296), (6, 16384), (3, 16392), (2, 65536)])
def test_quantize_rowwise(oracle, rows, cols):
    x = rand_bf16(np.random.default_rng(rows * 131 + cols), (rows, cols), 2.0)
    if rows >= 8:
        I.plant_edge_rows(x)
    q, s = sb.quantize_rowwise(to_dev(x))
    torch.cuda.synchronize()
    qo, so = oracle.quantize_rowwise(x)
    np.testing.assert_array_equal(host(s).view(np.uint32), so.view(np.uint32))
    np.testing.assert_array_equal(host(q), qo)


def test_quantize_rowwise_empty():
    x = torch.empty((0, 64), dtype=torch.bfloat16, device=DEV)
    q, s = sb.quantize_rowwise(x)
    assert q.shape == (0, 64) and s.shape == (0,)


@pytest.mark.parametrize("rows,cols", [(1024, 256), (16, 16), (64, 64), (272, 144), (128, 128), (1280, 5120),
                                       (144, 4096 + 16)])
def test_quantize_tensorwise(oracle, rows, cols):
    w = rand_bf16(np.random.default_rng(rows + 7 * cols), (rows, cols), 0.05)
    q, q_t, s = sb.quantize_tensorwise(to_dev(w))
    torch.cuda.synchronize()
    qo, qto, so = oracle.quantize_tensorwise(w)
    assert host(s).view(np.uint32)[0] == np.float32(so).view(np.uint32)
    np.testing.assert_array_equal(host(q), qo)
    np.testing.assert_array_equal(host(q_t), qto)
    q2, none, s2 = sb.quantize_tensorwise(to_dev(w), transpose=False)
    torch.cuda.synchronize()
    assert none is None
    np.testing.assert_array_equal(host(q2), qo)


def test_quantize_tensorwise_degenerate(oracle):
    for w in (np.zeros((64, 64), np.uint16), I.f32_to_bf16_bits(np.full((32, 48), 1e-38, np.float32))):
        q, q_t, s = sb.quantize_tensorwise(to_dev(w))
        torch.cuda.synchronize()
        assert s.item() == 0 and not host(q).any() and not host(q_t).any()
    ties = np.zeros((16, 16), np.float32)
    ties[0, :9] = [1, 3, 5, 7, -1, -3, -5, -7, 254]
    q, _, s = sb.quantize_tensorwise(to_dev(I.f32_to_bf16_bits(ties)))
    torch.cuda.synchronize()
    assert s.item() == 254 and host(q)[0, :9].tolist() == [0, 2, 2, 4, 0, -2, -2, -4, 127]


# ---------------------------------------------------------------------------------------------------------------
# int8 product: raw accumulators, then dequantized
# ---------------------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("M,N,K", [(512, 1024, 256), (300, 320, 192), (1, 64, 64), (257, 64, 128),
                                   (700, 832, 448), (513, 256, 1280), (31, 576, 64)])
def test_int8_accumulators_bit_exact(oracle, M, N, K):
    rng = np.random.default_rng(M + N + K)
    a = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    b = rng.integers(-127, 128, size=(N, K)).astype(np.int8)
    acc = sb.matmul_int8_dequant(torch.from_numpy(a).to(DEV), None, torch.from_numpy(b).to(DEV), None,
                                 out_dtype=torch.int32)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(acc), oracle.matmul_int8(a, b))


def test_int8_accumulator_extremes(oracle):
    """Longest supported contraction with all codes at +-127: |acc| = 127^2 * 131072 still fits int32."""
    K = 131072
    a = np.full((64, K), 127, np.int8)
    a[1::2] = -127
    b = np.full((64, K), 127, np.int8)
    acc = host(sb.matmul_int8_dequant(torch.from_numpy(a).to(DEV), None, torch.from_numpy(b).to(DEV), None,
                                      out_dtype=torch.int32))
    assert (acc[0::2] == 16129 * K).all() and (acc[1::2] == -16129 * K).all()


@pytest.mark.parametrize("M,N,K", [(300, 320, 192), (512, 256, 1024)])
def test_dequantized_product(oracle, M, N, K):
    rng = np.random.default_rng(M * 3 + N)
    a = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    b = rng.integers(-127, 128, size=(N, K)).astype(np.int8)
    srow = (rng.random(M) * 4 + 1e-3).astype(np.float32)
    srow[M // 2] = 0.0
    sw = np.array([0.21875], np.float32)
    args = (torch.from_numpy(a).to(DEV), torch.from_numpy(srow).to(DEV), torch.from_numpy(b).to(DEV),
            torch.from_numpy(sw).to(DEV))
    y32 = host(sb.matmul_int8_dequant(*args, out_dtype=torch.float32))
    ybf = bits_of(sb.matmul_int8_dequant(*args, out_dtype=torch.bfloat16))
    ref = oracle.dequantize(oracle.matmul_int8(a, b), srow, sw[0])
    assert np.all(np.abs(y32 - ref) <= ulp(ref))
    assert not y32[M // 2].any()
    assert_bf16_is_rounding_within_one_ulp(ybf, ref, oracle)


# ---------------------------------------------------------------------------------------------------------------
# bias and layer-scale in the epilogue of the int8 product: gamma * (y + bias), bias first, one rounding each.  The
# kernel evaluates the oracle's operation sequence, so binary32 results are compared within one ulp of the dequantized
# value carried through the two operations, and must be bit-identical wherever the dequantized value is.
# ---------------------------------------------------------------------------------------------------------------

def assert_bias_layerscale(got32, got_bf16_bits, acc, srow, sw, bias, gamma, oracle):
    y = oracle.dequantize(acc, srow, np.float32(sw))
    ref = oracle.bias_layerscale(y, bias, gamma)
    g = np.ones(acc.shape[1], np.float32) if gamma is None else np.abs(gamma)
    tol = g[None, :].astype(np.float64) * ulp(y) + ulp(ref)         # 1 ulp of y through the multiply, then one rounding
    assert np.all(np.abs(got32.astype(np.float64) - ref) <= tol)
    assert np.array_equal(got32.view(np.uint32), ref.view(np.uint32))  # same operation order: the bits match
    np.testing.assert_array_equal(got_bf16_bits, oracle.round_to_bf16(ref))


@pytest.mark.parametrize("which", ["both", "bias", "gamma", "neither"])
@pytest.mark.parametrize("M,N,K", [(300, 320, 192), (512, 1024, 256), (4096, 2304, 256), (1000, 4160, 320)])
def test_bias_layerscale_product(oracle, M, N, K, which):
    """All three kernel instances: 64-byte k-steps (K = 192, 320), the 128x128 tile (8 large tiles), the 256x256 tile
    over more than one round of a 256-workgroup grid would need > 256 tiles; 144 tiles run one round."""
    rng = np.random.default_rng(M + N + K)
    a = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    b = rng.integers(-127, 128, size=(N, K)).astype(np.int8)
    srow = (rng.random(M) * 4 + 1e-3).astype(np.float32)
    srow[M // 3] = 0.0                                              # zero product row: output gamma * bias
    bias = (rng.standard_normal(N) * 3).astype(np.float32) if which in ("both", "bias") else None
    gamma = rng.standard_normal(N).astype(np.float32) if which in ("both", "gamma") else None
    if gamma is not None:
        gamma[5] = 0.0                                              # a zero-initialised layer-scale entry
    dev = lambda v: None if v is None else torch.from_numpy(v).to(DEV)
    args = (torch.from_numpy(a).to(DEV), dev(srow), torch.from_numpy(b).to(DEV), torch.tensor([0.21875], device=DEV),
            dev(bias), dev(gamma))
    o32 = host(sb.matmul_int8_dequant_bias_layerscale(*args, out_dtype=torch.float32))
    obf = bits_of(sb.matmul_int8_dequant_bias_layerscale(*args, out_dtype=torch.bfloat16))
    assert_bias_layerscale(o32, obf, oracle.matmul_int8(a, b), srow, 0.21875, bias, gamma, oracle)
    if gamma is not None:
        assert not o32[:, 5].any()
    if which == "neither":                                          # then it is the plain product, bit for bit
        np.testing.assert_array_equal(obf, bits_of(sb.matmul_int8_dequant(*args[:4])))


def test_bias_layerscale_layer(oracle):
    """The layer call on the tiny workload with edge rows, and on the ViT-H/14 output projection at full size (645
    tiles, three per workgroup) on one token row per 32-row block; a zero-initialised gamma gives an all-zero output."""
    d = I.make_layer_inputs("tiny")
    I.plant_edge_rows(d["x"])
    rng = np.random.default_rng(3)
    m = d["w"].shape[0]
    bias, gamma = rng.standard_normal(m).astype(np.float32), (rng.standard_normal(m) * 0.1).astype(np.float32)
    x, w = to_dev(d["x"]), to_dev(d["w"])
    bd, gd = torch.from_numpy(bias).to(DEV), torch.from_numpy(gamma).to(DEV)
    y32, bufs = sb.forward_bias_layerscale(x, w, bd, gd, y_dtype=torch.float32)
    ybf, _ = sb.forward_bias_layerscale(x, w, bd, gd, bufs=bufs)
    y0, _ = sb.forward_bias_layerscale(x, w, bd, torch.zeros_like(gd), bufs=bufs)
    f = oracle.forward(d["x"], d["w"])
    np.testing.assert_array_equal(host(bufs.xq), f["xq"])
    np.testing.assert_array_equal(host(bufs.wq_t), f["wq_t"])
    assert_bias_layerscale(host(y32), bits_of(ybf), f["acc"], f["state_x"], f["state_w"], bias, gamma, oracle)
    assert not (bits_of(y0) & 0x7fff).any()

    L = I.CONFIGS["vit_h14"].layers[1]
    d = I.make_layer_inputs("vit_h14", 1, which=("x", "w"))
    bias, gamma = rng.standard_normal(L.m).astype(np.float32), (rng.standard_normal(L.m) * 0.1).astype(np.float32)
    rows = one_row_per_block(L.b, 32, rng)
    idx = torch.from_numpy(rows).to(DEV)
    bd, gd = torch.from_numpy(bias).to(DEV), torch.from_numpy(gamma).to(DEV)
    x, w = to_dev(d["x"]), to_dev(d["w"])
    y32, bufs = sb.forward_bias_layerscale(x, w, bd, gd, y_dtype=torch.float32)
    ybf, _ = sb.forward_bias_layerscale(x, w, bd, gd, bufs=bufs)
    xq, sx = oracle.quantize_rowwise(d["x"][rows])
    wq, _, sw = oracle.quantize_tensorwise(d["w"])
    assert_bias_layerscale(host(y32[idx]), bits_of(ybf[idx]), oracle.matmul_int8(xq, wq), sx, sw, bias, gamma, oracle)


# ---------------------------------------------------------------------------------------------------------------
# SwitchBackM: row-wise dequantization (bit-exact) and the weight gradient built on it
# ---------------------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("rows,cols", [(512, 256), (1, 8), (3, 64), (37, 520), (257, 1280), (129, 5120), (5, 16392),
                                       (2, 65536)])
def test_dequantize_rowwise(oracle, rows, cols):
    rng = np.random.default_rng(rows * 17 + cols)
    q = rng.integers(-127, 128, size=(rows, cols)).astype(np.int8)
    s = np.abs(rng.standard_normal(rows)).astype(np.float32) * np.float32(3.0)
    s[0] = 0.0                                                 # a zero row's state
    if rows > 2:
        s[1], s[2] = np.float32(254.0), np.float32(2.0 ** -120)
    got = sb.dequantize_rowwise(torch.from_numpy(q).to(DEV), torch.from_numpy(s).to(DEV))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(bits_of(got), oracle.dequantize_rowwise(q, s))


def test_dequantize_rowwise_empty():
    q = torch.empty((0, 64), dtype=torch.int8, device=DEV)
    out = sb.dequantize_rowwise(q, torch.empty((0,), dtype=torch.float32, device=DEV))
    assert out.shape == (0, 64)


@pytest.mark.parametrize("shape", ["tiny", (197, 320, 64), (1000, 64, 256)])
def test_switchback_m_weight_gradient(oracle, shape):
    if shape == "tiny":
        d = I.make_layer_inputs("tiny")
        I.plant_edge_rows(d["x"])
    else:
        b, n, m = shape
        rng = np.random.default_rng(b + n + m)
        d = dict(x=rand_bf16(rng, (b, n)), w=rand_bf16(rng, (m, n), n ** -0.5), dy=rand_bf16(rng, (b, m), 0.1))
    x, w, dy = to_dev(d["x"]), to_dev(d["w"]), to_dev(d["dy"])
    _, bufs = sb.forward(x, w)                                 # fills xq, state_x: all the variant keeps of X
    dw32, x_hat = sb.backward_weight_m(dy, bufs, dw_dtype=torch.float32)
    dwbf, _ = sb.backward_weight_m(dy, bufs, dw_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    xq, sx = oracle.quantize_rowwise(d["x"])
    h = oracle.backward_weight_m(d["dy"], xq, sx)
    np.testing.assert_array_equal(bits_of(x_hat), h["x_hat"])
    rms = float(np.sqrt((h["dw64"] ** 2).mean()))
    got = host(dw32)
    assert np.abs(got.astype(np.float64) - h["dw64"]).max() <= 1e-2 * rms
    np.testing.assert_array_equal(bits_of(dwbf), oracle.round_to_bf16(got))


# ---------------------------------------------------------------------------------------------------------------
# SwitchBackQ: column-wise quantize-transpose (bit-exact), row-and-column dequantization, the two int8 passes
# ---------------------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("rows,cols", [(1024, 256), (16, 16), (64, 64), (272, 144), (1280, 5120), (5120, 1280),
                                       (144, 4096 + 16)])
def test_quantize_colwise_transpose(oracle, rows, cols):
    rng = np.random.default_rng(rows * 3 + cols)
    w = rand_bf16(rng, (rows, cols), 0.05)
    w[:, 0] = 0                                                # an all-zero column
    w[:, cols // 2] = I.f32_to_bf16_bits(I.bf16_bits_to_f32(w[:, cols // 2]) * np.float32(256.0))
    q_t, s = sb.quantize_colwise_transpose(to_dev(w))
    torch.cuda.synchronize()
    qo, so = oracle.quantize_colwise_transpose(w)
    np.testing.assert_array_equal(host(s).view(np.uint32), so.view(np.uint32))
    np.testing.assert_array_equal(host(q_t), qo)


@pytest.mark.parametrize("M,N,K", [(300, 320, 192), (512, 256, 1024), (257, 64, 128)])
def test_rowcol_dequantized_product(oracle, M, N, K):
    rng = np.random.default_rng(M + N + K)
    a = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    b = rng.integers(-127, 128, size=(N, K)).astype(np.int8)
    sa = (np.abs(rng.standard_normal(M)) + 0.01).astype(np.float32)
    sbv = (np.abs(rng.standard_normal(N)) * 0.1 + 0.001).astype(np.float32)
    sa[M // 2] = 0.0
    sbv[3] = 0.0
    args = (torch.from_numpy(a).to(DEV), torch.from_numpy(sa).to(DEV), torch.from_numpy(b).to(DEV),
            torch.from_numpy(sbv).to(DEV))
    y32 = host(sb.matmul_int8_dequant_rc(*args, out_dtype=torch.float32))
    ybf = bits_of(sb.matmul_int8_dequant_rc(*args, out_dtype=torch.bfloat16))
    ref = oracle.dequantize_rowcol(oracle.matmul_int8(a, b), sa, sbv)
    assert np.all(np.abs(y32 - ref) <= ulp(ref))
    assert not y32[M // 2].any() and not y32[:, 3].any()
    assert_bf16_is_rounding_within_one_ulp(ybf, ref, oracle)


def check_layer_q(oracle, d, rows=None):
    x, w, dy = to_dev(d["x"]), to_dev(d["w"]), to_dev(d["dy"])
    y32, bufs = sb.forward_q(x, w, y_dtype=torch.float32)
    ybf, _ = sb.forward_q(x, w, bufs=bufs, y_dtype=torch.bfloat16)
    dx32 = sb.backward_input_q(dy, w, bufs, dx_dtype=torch.float32)
    dxbf = sb.backward_input_q(dy, w, bufs, dx_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    xq, sx = oracle.quantize_rowwise(d["x"])
    wq, sw = oracle.quantize_rowwise(d["w"])
    gq, sg = oracle.quantize_rowwise(d["dy"])
    wq_t, swc = oracle.quantize_colwise_transpose(d["w"])
    for got, want in ((bufs.xq, xq), (bufs.wq, wq), (bufs.gq, gq), (bufs.wq_t, wq_t)):
        np.testing.assert_array_equal(host(got), want)
    for got, want in ((bufs.state_x, sx), (bufs.state_w_row, sw), (bufs.state_g, sg), (bufs.state_w_col, swc)):
        np.testing.assert_array_equal(host(got).view(np.uint32), want.view(np.uint32))
    rows = np.arange(d["x"].shape[0]) if rows is None else rows
    idx = torch.from_numpy(rows).to(DEV)
    ref = oracle.dequantize_rowcol(oracle.matmul_int8(xq[rows], wq), sx[rows], sw)
    assert np.all(np.abs(host(y32[idx]) - ref) <= ulp(ref))
    assert_bf16_is_rounding_within_one_ulp(bits_of(ybf[idx]), ref, oracle)
    ref = oracle.dequantize_rowcol(oracle.matmul_int8(gq[rows], wq_t), sg[rows], swc)
    assert np.all(np.abs(host(dx32[idx]) - ref) <= ulp(ref))
    assert_bf16_is_rounding_within_one_ulp(bits_of(dxbf[idx]), ref, oracle)


def test_switchback_q_tiny_with_edge_rows(oracle):
    d = I.make_layer_inputs("tiny")
    I.plant_edge_rows(d["x"])
    I.plant_edge_rows(d["dy"])
    d["w"][7] = 0                                              # an all-zero output feature
    check_layer_q(oracle, d)


@pytest.mark.parametrize("b,n,m", [(33, 192, 320), (300, 128, 576), (1000, 64, 256)])
def test_switchback_q_ragged_shapes(oracle, b, n, m):
    rng = np.random.default_rng(b + n + m + 1)
    d = dict(x=rand_bf16(rng, (b, n)), w=rand_bf16(rng, (m, n), n ** -0.5), dy=rand_bf16(rng, (b, m), 0.1))
    check_layer_q(oracle, d)


@pytest.mark.parametrize("config,layer", [("vit_b16", 0), ("vit_b16", 1), ("vit_l14", 0), ("vit_l14", 1), ("vit_l14", 2),
                                          ("vit_l14", 3), ("vit_h14", 0), ("vit_h14", 1), ("vit_h14", 2), ("vit_h14", 3),
                                          ("outlier", 0), ("outlier", 1)])
def test_switchback_q_full_size_sampled(oracle, config, layer):
    L = I.CONFIGS[config].layers[layer]
    d = I.make_layer_inputs(config, layer)
    check_layer_q(oracle, d, one_row_per_block(L.b, 32, np.random.default_rng(23)))


# ---------------------------------------------------------------------------------------------------------------
# the layer: tiny config, everything compared in full
# ---------------------------------------------------------------------------------------------------------------

def check_layer_full(oracle, d):
    x, w, dy = to_dev(d["x"]), to_dev(d["w"]), to_dev(d["dy"])
    y32, bufs = sb.forward(x, w, y_dtype=torch.float32)
    ybf, _ = sb.forward(x, w, bufs=bufs, y_dtype=torch.bfloat16)
    acc, _ = sb.forward(x, w, bufs=bufs, y_dtype=torch.int32)
    dx32 = sb.backward_input(dy, bufs, dx_dtype=torch.float32)
    dxbf = sb.backward_input(dy, bufs, dx_dtype=torch.bfloat16)
    dacc = sb.backward_input(dy, bufs, dx_dtype=torch.int32)
    dw32 = sb.backward_weight(dy, x, bufs, dw_dtype=torch.float32)
    dwbf = sb.backward_weight(dy, x, bufs, dw_dtype=torch.bfloat16)
    torch.cuda.synchronize()

    f = oracle.forward(d["x"], d["w"])
    np.testing.assert_array_equal(host(bufs.xq), f["xq"])
    np.testing.assert_array_equal(host(bufs.state_x).view(np.uint32), f["state_x"].view(np.uint32))
    np.testing.assert_array_equal(host(bufs.wq), f["wq"])
    np.testing.assert_array_equal(host(bufs.wq_t), f["wq_t"])
    assert host(bufs.state_w).view(np.uint32)[0] == np.float32(f["state_w"]).view(np.uint32)
    np.testing.assert_array_equal(host(acc), f["acc"])
    assert np.all(np.abs(host(y32) - f["y32"]) <= ulp(f["y32"]))
    assert_bf16_is_rounding_within_one_ulp(bits_of(ybf), f["y32"], oracle)

    g = oracle.backward_input(d["dy"], f["wq_t"], f["state_w"])
    np.testing.assert_array_equal(host(bufs.gq), g["gq"])
    np.testing.assert_array_equal(host(bufs.state_g).view(np.uint32), g["state_g"].view(np.uint32))
    np.testing.assert_array_equal(host(dacc), g["acc"])
    assert np.all(np.abs(host(dx32) - g["dx32"]) <= ulp(g["dx32"]))
    assert_bf16_is_rounding_within_one_ulp(bits_of(dxbf), g["dx32"], oracle)

    h = oracle.backward_weight(d["dy"], d["x"])
    rms = float(np.sqrt((h["dw64"] ** 2).mean()))
    got = host(dw32)
    assert np.abs(got.astype(np.float64) - h["dw64"]).max() <= 1e-2 * rms
    # bf16 mode: the rounding of the library's own binary32 result, hence within one bf16 ulp of the oracle's
    np.testing.assert_array_equal(bits_of(dwbf), oracle.round_to_bf16(got))
    return f, g, h


def test_layer_tiny_with_edge_rows(oracle):
    d = I.make_layer_inputs("tiny")
    I.plant_edge_rows(d["x"])
    I.plant_edge_rows(d["dy"])
    f, g, h = check_layer_full(oracle, d)
    assert not f["y32"][0].any() and not f["y32"][1].any()       # zero row and overflow row -> zero output


@pytest.mark.parametrize("b,n,m", [(1, 64, 64), (33, 192, 320), (197, 320, 64), (300, 128, 576), (1000, 64, 256)])
def test_layer_ragged_shapes(oracle, b, n, m):
    rng = np.random.default_rng(b + n + m)
    d = dict(x=rand_bf16(rng, (b, n)), w=rand_bf16(rng, (m, n), n ** -0.5), dy=rand_bf16(rng, (b, m), 0.1))
    check_layer_full(oracle, d)


def test_layer_empty_batch():
    w = to_dev(rand_bf16(np.random.default_rng(0), (64, 64), 0.1))
    x = torch.empty((0, 64), dtype=torch.bfloat16, device=DEV)
    y, bufs = sb.forward(x, w)
    dx = sb.backward_input(torch.empty((0, 64), dtype=torch.bfloat16, device=DEV), bufs)
    dw = sb.backward_weight(torch.empty((0, 64), dtype=torch.bfloat16, device=DEV), x, bufs, dw_dtype=torch.float32)
    torch.cuda.synchronize()
    assert y.shape == (0, 64) and dx.shape == (0, 64) and not host(dw).any()
    assert bufs.state_w.item() > 0                                # W is still quantized


def test_results_are_deterministic():
    d = I.make_layer_inputs("tiny")
    x, w, dy = to_dev(d["x"]), to_dev(d["w"]), to_dev(d["dy"])
    outs = []
    for _ in range(3):
        y, bufs = sb.forward(x, w)
        dx = sb.backward_input(dy, bufs)
        dw = sb.backward_weight(dy, x, bufs, dw_dtype=torch.float32)
        torch.cuda.synchronize()
        outs.append((bits_of(y), bits_of(dx), host(dw).copy()))
    for o in outs[1:]:
        assert all(np.array_equal(a, b) for a, b in zip(o, outs[0]))


# ---------------------------------------------------------------------------------------------------------------
# full-size configurations, in the launch configuration the benchmark times: quantizers compared in full,
# products on sampled rows the oracle computes one by one
# ---------------------------------------------------------------------------------------------------------------

FULL = [("vit_b16", 0), ("vit_b16", 1), ("vit_l14", 0), ("vit_l14", 1), ("vit_l14", 2), ("vit_l14", 3), ("vit_h14", 0),
        ("vit_h14", 1), ("vit_h14", 2), ("vit_h14", 3), ("outlier", 0), ("outlier", 1)]


def one_row_per_block(count, block, rng):
    """One index out of every `block` consecutive ones (each 32-row MFMA block of every tile contributes), plus the
    first and last rows and the rows on either side of the first and last tile edge."""
    base = np.arange(0, count, block)
    pick = np.minimum(base + rng.integers(0, block, base.size), count - 1)
    edges = [0, 1, 255, 256, count - 257, count - 256, count - 2, count - 1]
    return np.unique(np.concatenate([pick, [e for e in edges if 0 <= e < count]]))


@pytest.mark.parametrize("config,layer", FULL)
def test_layer_full_size_sampled(oracle, config, layer):
    L = I.CONFIGS[config].layers[layer]
    d = I.make_layer_inputs(config, layer)
    x, w, dy = to_dev(d["x"]), to_dev(d["w"]), to_dev(d["dy"])
    bufs = sb.LayerBuffers(L.b, L.n, L.m, DEV)
    rng = np.random.default_rng(17)
    rows = one_row_per_block(L.b, 32, rng)
    idx = torch.from_numpy(rows).to(DEV)
    take = lambda t: host(t[idx])
    yacc = take(sb.forward(x, w, bufs=bufs, y_dtype=torch.int32)[0])
    y32 = take(sb.forward(x, w, bufs=bufs, y_dtype=torch.float32)[0])
    ybf = bits_of(sb.forward(x, w, bufs=bufs, y_dtype=torch.bfloat16)[0][idx])
    dxacc = take(sb.backward_input(dy, bufs, dx_dtype=torch.int32))
    dx32 = take(sb.backward_input(dy, bufs, dx_dtype=torch.float32))
    dxbf = bits_of(sb.backward_input(dy, bufs, dx_dtype=torch.bfloat16)[idx])
    dw32 = sb.backward_weight(dy, x, bufs, dw_dtype=torch.float32)
    torch.cuda.synchronize()

    # quantizers: every element
    xq, sx = oracle.quantize_rowwise(d["x"])
    np.testing.assert_array_equal(host(bufs.state_x).view(np.uint32), sx.view(np.uint32))
    np.testing.assert_array_equal(host(bufs.xq), xq)
    wq, wq_t, sw = oracle.quantize_tensorwise(d["w"])
    assert host(bufs.state_w).view(np.uint32)[0] == np.float32(sw).view(np.uint32)
    np.testing.assert_array_equal(host(bufs.wq), wq)
    np.testing.assert_array_equal(host(bufs.wq_t), wq_t)
    gq, sg = oracle.quantize_rowwise(d["dy"])
    np.testing.assert_array_equal(host(bufs.state_g).view(np.uint32), sg.view(np.uint32))
    np.testing.assert_array_equal(host(bufs.gq), gq)

    # products: one token row out of every 32-row block of every tile row, all columns; raw accumulators bit-exact,
    # binary32 within one ulp, bf16 the rounding of such a value
    acc = oracle.matmul_int8(xq[rows], wq)
    np.testing.assert_array_equal(yacc, acc)
    ref = oracle.dequantize(acc, sx[rows], sw)
    assert np.all(np.abs(y32 - ref) <= ulp(ref))
    assert_bf16_is_rounding_within_one_ulp(ybf, ref, oracle)
    acc = oracle.matmul_int8(gq[rows], wq_t)
    np.testing.assert_array_equal(dxacc, acc)
    ref = oracle.dequantize(acc, sg[rows], sw)
    assert np.all(np.abs(dx32 - ref) <= ulp(ref))
    assert_bf16_is_rounding_within_one_ulp(dxbf, ref, oracle)

    # weight gradient: one dW row (column of dY) out of every 32-row block, full contraction, all columns
    jrows = one_row_per_block(L.m, 32, rng)
    dw_ref = oracle.weight_grad(np.ascontiguousarray(d["dy"][:, jrows]), d["x"])
    rms = float(np.sqrt((dw_ref ** 2).mean()))
    got = host(dw32[torch.from_numpy(jrows).to(DEV)]).astype(np.float64)
    assert np.abs(got - dw_ref).max() <= 1e-2 * rms

    # SwitchBackM: the dequantized X in full (bit-exact), its weight gradient on the same sampled rows
    dwm, x_hat = sb.backward_weight_m(dy, bufs, dw_dtype=torch.float32)
    torch.cuda.synchronize()
    xh = oracle.dequantize_rowwise(xq, sx)
    np.testing.assert_array_equal(bits_of(x_hat), xh)
    dwm_ref = oracle.weight_grad(np.ascontiguousarray(d["dy"][:, jrows]), xh)
    got = host(dwm[torch.from_numpy(jrows).to(DEV)]).astype(np.float64)
    assert np.abs(got - dwm_ref).max() <= 1e-2 * float(np.sqrt((dwm_ref ** 2).mean()))


# ---------------------------------------------------------------------------------------------------------------
# whole outputs at sizes where every workgroup of the persistent GEMM grids walks several tiles: the hand-over from
# one tile's last stage into the next tile's first, with the epilogue's stores in the wave's memory books, is compared
# with the oracle on EVERY element
# ---------------------------------------------------------------------------------------------------------------

def check_int8_product_whole(oracle, a, b, srow, sw):
    """aq [M,K], bq [N,K] int8 (host), srow [M] f32, sw f32 scalar: raw accumulators bit-exact, binary32 within one ulp,
    bf16 the rounding of such a value, every element."""
    ad, bd = torch.from_numpy(a).to(DEV), torch.from_numpy(b).to(DEV)
    srd, swd = torch.from_numpy(srow).to(DEV), torch.tensor([sw], dtype=torch.float32, device=DEV)
    acc_ref = oracle.matmul_int8(a, b)
    acc = host(sb.matmul_int8_dequant(ad, None, bd, None, out_dtype=torch.int32))
    np.testing.assert_array_equal(acc, acc_ref)
    del acc
    ref = oracle.dequantize(acc_ref, srow, np.float32(sw))
    del acc_ref
    y32 = host(sb.matmul_int8_dequant(ad, srd, bd, swd, out_dtype=torch.float32))
    assert np.all(np.abs(y32 - ref) <= ulp(ref))
    del y32
    ybf = bits_of(sb.matmul_int8_dequant(ad, srd, bd, swd, out_dtype=torch.bfloat16))
    assert_bf16_is_rounding_within_one_ulp(ybf, ref, oracle)


@pytest.mark.parametrize("M,N,K", [(4096, 4608, 128), (4096, 4608, 192), (32896, 1280, 192), (6304, 3072, 768),
                                   (2000, 9280, 320), (6304, 768, 3072), (3000, 1984, 256)])
def test_int8_product_whole_output_over_several_rounds(oracle, M, N, K):
    """288 to 645 output tiles on at most 256 workgroups: two to three tiles per workgroup, with both k-step
    instances (K a multiple of 128, and of 64 only), short and long contractions, ragged M.  The last two shapes have
    few large tiles (75 and 96) and take the 128x128-tile instance, two workgroups per compute unit, ragged M and N."""
    rng = np.random.default_rng(M + 3 * N + 7 * K)
    a = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    b = rng.integers(-127, 128, size=(N, K)).astype(np.int8)
    srow = (rng.random(M) * 4 + 1e-3).astype(np.float32)
    check_int8_product_whole(oracle, a, b, srow, 0.21875)


WHOLE = [("vit_h14", 1, True), ("vit_h14", 3, False), ("vit_l14", 1, True),
         ("vit_b16", 0, True), ("vit_b16", 1, True)]


@pytest.mark.parametrize("config,layer,with_dw", WHOLE, ids=["%s-%d" % (c, l) for c, l, _ in WHOLE])
def test_layer_whole_output(oracle, config, layer, with_dw):
    """Layers in the launch configuration the benchmark times, compared with the oracle on every element: Y and dX
    (raw accumulators, binary32, bf16) and, except for the largest, the whole dW.  ViT-H/14 proj (1280 -> 1280) and fc2
    (5120 -> 1280) run the 256 x 256-tile instances over several rounds of the persistent grids; ViT-L/14 proj and both
    layers of ViT-B/16 run the weight gradient, and ViT-B/16's 768-wide outputs also the int8 products, on the 128 x 128-tile
    instances."""
    L = I.CONFIGS[config].layers[layer]
    d = I.make_layer_inputs(config, layer)
    xq, sx = oracle.quantize_rowwise(d["x"])
    wq, wq_t, sw = oracle.quantize_tensorwise(d["w"])
    gq, sg = oracle.quantize_rowwise(d["dy"])
    # the layer calls, every element of the bf16 outputs and of the codes they are built from
    x, w, dy = to_dev(d["x"]), to_dev(d["w"]), to_dev(d["dy"])
    bufs = sb.LayerBuffers(L.b, L.n, L.m, DEV)
    ybf = bits_of(sb.forward(x, w, bufs=bufs)[0])
    dxbf = bits_of(sb.backward_input(dy, bufs))
    np.testing.assert_array_equal(host(bufs.xq), xq)
    np.testing.assert_array_equal(host(bufs.gq), gq)
    np.testing.assert_array_equal(host(bufs.wq_t), wq_t)
    ref = oracle.dequantize(oracle.matmul_int8(xq, wq), sx, sw)
    assert_bf16_is_rounding_within_one_ulp(ybf, ref, oracle)
    ref = oracle.dequantize(oracle.matmul_int8(gq, wq_t), sg, sw)
    assert_bf16_is_rounding_within_one_ulp(dxbf, ref, oracle)
    del ref, ybf, dxbf
    # the same two products through the product call: raw accumulators and binary32 as well
    check_int8_product_whole(oracle, xq, wq, sx, sw)
    check_int8_product_whole(oracle, gq, wq_t, sg, sw)
    if with_dw:
        dw32 = host(sb.backward_weight(dy, x, bufs, dw_dtype=torch.float32))
        dwbf = bits_of(sb.backward_weight(dy, x, bufs, dw_dtype=torch.bfloat16))
        dw_ref = oracle.weight_grad(d["dy"], d["x"])
        assert np.abs(dw32.astype(np.float64) - dw_ref).max() <= 1e-2 * float(np.sqrt((dw_ref ** 2).mean()))
        np.testing.assert_array_equal(dwbf, oracle.round_to_bf16(dw32))


@pytest.mark.parametrize("b,n,m", [(256, 4352, 4352), (1500, 2304, 2816), (4000, 1280, 1280)])
def test_weight_gradient_whole_output_over_several_rounds(oracle, b, n, m):
    """More work items than workgroups, so workgroups of the persistent grid take a second item: 289 large tiles
    without a split of the token range; 198 and 100 small tiles (the instance for short work items) with one.  dW
    compared with the oracle on every element."""
    rng = np.random.default_rng(b + n + m)
    dyb, xb = rand_bf16(rng, (b, m), 0.1), rand_bf16(rng, (b, n))
    dy, x = to_dev(dyb), to_dev(xb)
    dw32 = host(sb.backward_weight(dy, x, dw_dtype=torch.float32))
    dwbf = bits_of(sb.backward_weight(dy, x, dw_dtype=torch.bfloat16))
    dw_ref = oracle.weight_grad(dyb, xb)
    assert np.abs(dw32.astype(np.float64) - dw_ref).max() <= 1e-2 * float(np.sqrt((dw_ref ** 2).mean()))
    np.testing.assert_array_equal(dwbf, oracle.round_to_bf16(dw32))


def test_weight_gradient_large_tiles_with_splits(oracle):
    """Long token range, few tiles: the 256 x 256-tile instance with the token range cut into four pieces (64 tiles x 4
    splits, ragged last stage and ragged last tile row / column).  Every seventh row of dW (all residues modulo the
    32-row matrix-instruction block, every tile) compared on all columns."""
    b, n, m = 8600 + 37, 2048 - 128, 2048 - 64
    rng = np.random.default_rng(77)
    dyb, xb = rand_bf16(rng, (b, m), 0.1), rand_bf16(rng, (b, n))
    dy, x = to_dev(dyb), to_dev(xb)
    dw32 = host(sb.backward_weight(dy, x, dw_dtype=torch.float32))
    dwbf = bits_of(sb.backward_weight(dy, x, dw_dtype=torch.bfloat16))
    rows = np.arange(0, m, 7)
    dw_ref = oracle.weight_grad(np.ascontiguousarray(dyb[:, rows]), xb)
    assert np.abs(dw32[rows].astype(np.float64) - dw_ref).max() <= 1e-2 * float(np.sqrt((dw_ref ** 2).mean()))
    np.testing.assert_array_equal(dwbf, oracle.round_to_bf16(dw32))


# ---------------------------------------------------------------------------------------------------------------
# StableAdamW (the optimizer algorithm of the paper; per-tensor update clipping)
# ---------------------------------------------------------------------------------------------------------------

def adamw_case(count, seed, grad_bf16, first_step, spike):
    """Seeded optimizer state in the ranges of a transformer weight matrix mid-training: |theta| ~ 0.02, gradients
    ~ 1e-3 with a few exact zeros (dead coordinates keep u = v = 0), u ~ E[g^2]; `spike` multiplies the gradient by
    30 so that RMS_t > 1 and the learning rate is clipped."""
    rng = np.random.default_rng(seed)
    theta = (rng.standard_normal(count) * 0.02).astype(np.float32)
    g = (rng.standard_normal(count) * 1e-3 * (30.0 if spike else 1.0)).astype(np.float32)
    if first_step:
        v = np.zeros(count, np.float32)
        u = np.zeros(count, np.float32)
    else:
        v = (rng.standard_normal(count) * 3e-4).astype(np.float32)
        u = (rng.uniform(0.3, 3.0, count) * 1e-6).astype(np.float32)
    dead = rng.random(count) < 0.01
    g[dead] = 0.0
    v[dead] = 0.0
    u[dead] = 0.0
    if grad_bf16:
        g = I.f32_to_bf16_bits(g)
    return theta, v, u, g


# The C ABI takes the hyper-parameters as binary32; the oracle gets the same binary32 values (1 - 0.98f differs from
# 1 - 0.98 by 1e-6 relative, which is an input difference, not arithmetic).
ADAMW_HYPER = {k: float(np.float32(x)) for k, x in dict(alpha=2e-3, beta1=0.9, beta2=0.98, eps=1e-6, lam=0.2).items()}


def check_adamw(oracle, count, seed, grad_bf16, t, spike=False):
    h = ADAMW_HYPER
    theta, v, u, g = adamw_case(count, seed, grad_bf16, t == 1, spike)
    th_o, v_o, u_o, rms_o = oracle.stable_adamw_step(theta, v, u, g, h["alpha"], h["beta1"], h["beta2"], h["eps"],
                                                     h["lam"], t)
    th_d, v_d, u_d = (torch.from_numpy(a.copy()).to(DEV) for a in (theta, v, u))
    g_d = to_dev(g) if grad_bf16 else torch.from_numpy(g).to(DEV)
    rms_d = sb.stable_adamw_step(th_d, v_d, u_d, g_d, h["alpha"], h["beta1"], h["beta2"], h["eps"], h["lam"], t)
    torch.cuda.synchronize()
    rms = float(rms_d.item())
    assert abs(rms - rms_o) <= 2e-6 * rms_o + 1e-30, (rms, rms_o)
    if spike:
        assert rms_o > 2.0
    # Tolerances from the arithmetic: binary32 multiply-adds (2^-24 relative per rounding, decay rates rounded once).
    gf = (g.astype(np.uint32) << 16).view(np.float32).astype(np.float64) if grad_bf16 else g.astype(np.float64)
    b1 = h["beta1"] * (1 - h["beta1"] ** (t - 1)) / (1 - h["beta1"] ** t)
    e = 2.0 ** -24
    tol_v = 4 * e * (np.abs(b1 * v.astype(np.float64)) + np.abs((1 - b1) * gf)) + 1e-44
    assert (np.abs(host(v_d).astype(np.float64) - v_o) <= tol_v).all()
    assert (np.abs(host(u_d).astype(np.float64) - u_o) <= 8 * e * u_o.astype(np.float64) + 1e-44).all()
    eta = h["alpha"] / max(1.0, rms_o)
    den = np.sqrt(u_o.astype(np.float64)) + h["eps"]
    tol_th = (2 * np.spacing(np.abs(th_o)).astype(np.float64) + eta * tol_v / den
              + 4e-6 * np.abs(eta * v_o.astype(np.float64) / den) + 1e-6 * np.abs(eta * h["lam"] * theta))
    err = np.abs(host(th_d).astype(np.float64) - th_o)
    assert (err <= tol_th).all(), "theta off by up to %.3g (tolerance ratio %.2f)" % (err.max(), (err / tol_th).max())
    return err, tol_th


@pytest.mark.parametrize("count", [1, 3, 5, 1023, 4096, 4097, 70001, 1280 * 1280])
@pytest.mark.parametrize("grad_bf16", [True, False])
def test_stable_adamw_step(oracle, count, grad_bf16):
    check_adamw(oracle, count, 1000 + count % 997, grad_bf16, t=1)
    check_adamw(oracle, count, 2000 + count % 997, grad_bf16, t=7)
    check_adamw(oracle, count, 3000 + count % 997, grad_bf16, t=300, spike=True)


def test_stable_adamw_full_size_weight_and_grid_stride(oracle):
    """The benchmark's tensor (one MLP weight of ViT-H/14, 1280 x 5120) and one large enough that every workgroup
    loops (the grid is capped), with a count that leaves a tail."""
    check_adamw(oracle, 1280 * 5120, 77, True, t=12)
    check_adamw(oracle, 1280 * 5120, 78, False, t=12, spike=True)
    check_adamw(oracle, 20 * 1000 * 1000 + 3, 79, True, t=5)


def test_stable_adamw_batched_step_equals_per_tensor_steps(oracle):
    """Many tensors in two launches: every tensor is clipped by its own RMS, bit-identical to the per-tensor entry point
    (same workgroup partition), and within the per-tensor tolerance of the oracle."""
    h = ADAMW_HYPER
    counts = [1, 7, 1280, 3 * 1280, 4097, 1280 * 1280, 5, 70001, 1280 * 5120, 1024]
    cases = [adamw_case(c, 900 + i, True, False, spike=(i % 3 == 1)) for i, c in enumerate(counts)]
    batched, single = [], []
    for theta, v, u, g in cases:
        batched.append(tuple(torch.from_numpy(a.copy()).to(DEV) for a in (theta, v, u)) + (to_dev(g),))
        single.append(tuple(torch.from_numpy(a.copy()).to(DEV) for a in (theta, v, u)) + (to_dev(g),))
    plan = sb.AdamwPlan(batched)
    assert plan.total_blocks >= len(counts)
    rms = sb.stable_adamw_step_multi(plan, h["alpha"], h["beta1"], h["beta2"], h["eps"], h["lam"], 40)
    rms_single = [sb.stable_adamw_step(th, v, u, g, h["alpha"], h["beta1"], h["beta2"], h["eps"], h["lam"], 40)
                  for (th, v, u, g) in single]
    torch.cuda.synchronize()
    clipped = 0
    for i, ((theta, v, u, g), bt, st) in enumerate(zip(cases, batched, single)):
        for a, b in zip(bt[:3], st[:3]):
            np.testing.assert_array_equal(host(a).view(np.uint32), host(b).view(np.uint32))
        assert host(rms)[i].view(np.uint32) == host(rms_single[i])[0].view(np.uint32)
        th_o, v_o, u_o, rms_o = oracle.stable_adamw_step(theta, v, u, g, h["alpha"], h["beta1"], h["beta2"], h["eps"],
                                                         h["lam"], 40)
        assert abs(float(host(rms)[i]) - rms_o) <= 2e-6 * rms_o + 1e-30
        clipped += rms_o > 1.0
        np.testing.assert_allclose(host(bt[0]), th_o, rtol=1e-5, atol=1e-9)
    assert 0 < clipped < len(counts)                              # some tensors clipped, some not, in one launch


def test_stable_adamw_is_deterministic_and_leaves_grad_alone():
    theta, v, u, g = adamw_case(300001, 5, True, False, True)
    outs = []
    for _ in range(2):
        th_d, v_d, u_d = (torch.from_numpy(a.copy()).to(DEV) for a in (theta, v, u))
        g_d = to_dev(g)
        rms = sb.stable_adamw_step(th_d, v_d, u_d, g_d, 1e-3, 0.9, 0.95, 1e-6, 0.1, 9)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(bits_of(g_d), g)
        outs.append((host(th_d), host(v_d), host(u_d), host(rms)))
    for a, b in zip(*outs):
        np.testing.assert_array_equal(a.view(np.uint32), b.view(np.uint32))


# ---------------------------------------------------------------------------------------------------------------
# float8 SwitchBack (float8cast(x / absmax(x)) as the quantizer, real 8-bit float matrix instructions).  Codes and
# states bit-exact.  The product is compared with the oracle's exact sum under the error bound of the matrix
# instruction's arithmetic, which single-instruction probes with crafted operands show to be: the 64 products of one
# instruction are summed in groups of 8 consecutive k; inside a group every product is aligned to the largest one and
# TRUNCATED below 2^-13 of that product's power of two (a 14-bit window); group sums and the accumulator are then added
# at binary32 precision or better.  Hence per group an error below 7 * 2^-13 * max|a_k b_k|, in total below
# 7 * 2^-13 * sum_k |a_k b_k|, plus 2^-23 of that sum for each of the K/64 + 8 binary32 additions a result passes
# through.  (The paper's own float8 runs do this arithmetic in 16 bit, i.e. with 8 to 11 significant bits.)
# ---------------------------------------------------------------------------------------------------------------

def u8_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def f8_product_tolerance(abs_acc, r, K):
    return (7 * 2.0 ** -13 + (K / 64 + 8) * 2.0 ** -23) * abs_acc * np.abs(r.astype(np.float64))[:, None]


def assert_f8_outputs(got32, got_bf16_bits, acc, abs_acc, state_row, state_w, K, oracle):
    r = (state_row * np.float32(state_w)).astype(np.float32)
    y32, y64 = oracle.dequantize_f8(acc, state_row, state_w, want_f64=True)
    tol = f8_product_tolerance(abs_acc, r, K) + ulp(y32)
    if got32 is not None:
        err = np.abs(got32.astype(np.float64) - y64)
        assert (err <= tol).all(), "float8 product off by %.3g, %.2f of the tolerance" % (err.max(), (err / tol).max())
    if got_bf16_bits is not None:
        got = I.bf16_bits_to_f32(got_bf16_bits).astype(np.float64)
        half_bf16_ulp = np.abs(y64) * 2.0 ** -8 + 1e-45
        assert (np.abs(got - y64) <= tol + half_bf16_ulp).all()


@pytest.mark.parametrize("fmt", [0, 1])
@pytest.mark.parametrize("rows,cols", [(512, 256), (1, 8), (5, 520), (257, 1280), (9, 2056), (33, 5120), (5, 12296),
                                       (3, 16392), (2, 65536)])
def test_float8_quantize_rowwise(oracle, rows, cols, fmt):
    x = rand_bf16(np.random.default_rng(rows * 17 + cols + fmt), (rows, cols), 2.0)
    if rows >= 8:
        I.plant_edge_rows(x)
    codes, state = sb.quantize_rowwise_f8(to_dev(x), fmt)
    torch.cuda.synchronize()
    co, so = oracle.quantize_rowwise_f8(x, fmt)
    np.testing.assert_array_equal(host(state).view(np.uint32), so.view(np.uint32))
    np.testing.assert_array_equal(host(codes), co)


@pytest.mark.parametrize("fmt", [0, 1])
@pytest.mark.parametrize("rows,cols", [(1024, 256), (16, 16), (272, 144), (1280, 5120)])
def test_float8_quantize_tensorwise(oracle, rows, cols, fmt):
    w = rand_bf16(np.random.default_rng(rows + cols + fmt), (rows, cols), cols ** -0.5)
    w[rows // 2, cols // 3] = np.uint16(0xC000)                   # -2.0: the absmax, negative
    codes, codes_t, state = sb.quantize_tensorwise_f8(to_dev(w), fmt)
    torch.cuda.synchronize()
    co, cto, so = oracle.quantize_tensorwise_f8(w, fmt)
    assert host(state).view(np.uint32)[0] == np.float32(so).view(np.uint32)
    np.testing.assert_array_equal(host(codes), co)
    np.testing.assert_array_equal(host(codes_t), cto)


def layer_like_codes(rng, shape, fmt):
    """Random codes with |value| <= 1 (what the quantizers emit), all exponents of the format's [0, 1] range."""
    one = 0x38 if fmt == 0 else 0x3C
    mag = rng.integers(0, one + 1, shape).astype(np.uint8)
    return mag | (rng.integers(0, 2, shape).astype(np.uint8) << 7)


@pytest.mark.parametrize("fa,fb", [(0, 0), (1, 0), (0, 1), (1, 1)])
@pytest.mark.parametrize("M,N,K", [(300, 320, 256), (512, 256, 1024), (1, 64, 128), (257, 576, 384)])
def test_float8_product(oracle, M, N, K, fa, fb):
    rng = np.random.default_rng(M + N + K + 2 * fa + fb)
    a, b = layer_like_codes(rng, (M, K), fa), layer_like_codes(rng, (N, K), fb)
    sr = rng.uniform(0.5, 4.0, M).astype(np.float32)
    sw = np.float32(0.37)
    acc, abs_acc = oracle.matmul_f8(a, fa, b, fb, want_abs=True)
    sw_d = torch.tensor([sw], dtype=torch.float32, device=DEV)
    o32 = sb.matmul_f8_dequant(u8_dev(a), fa, u8_dev(sr), u8_dev(b), fb, sw_d, out_dtype=torch.float32)
    obf = sb.matmul_f8_dequant(u8_dev(a), fa, u8_dev(sr), u8_dev(b), fb, sw_d, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    assert_f8_outputs(host(o32), bits_of(obf), acc, abs_acc, sr, sw, K, oracle)


@pytest.mark.parametrize("fa,fb", [(0, 0), (1, 0)])
def test_float8_product_is_exact_when_binary32_can_hold_every_partial_sum(oracle, fa, fb):
    """Codes of 0, +-0.25, +-0.5, +-1: every product and partial sum is a small multiple of 1/16, exact in binary32
    in any order, so the result must equal the oracle's bit for bit -- each operand byte reaches the right k."""
    rng = np.random.default_rng(5 + fa)
    M, N, K = 333, 192, 640
    pick = {0: np.array([0x00, 0x28, 0x30, 0x38], np.uint8), 1: np.array([0x00, 0x34, 0x38, 0x3C], np.uint8)}
    a = pick[fa][rng.integers(0, 4, (M, K))] | (rng.integers(0, 2, (M, K)).astype(np.uint8) << 7)
    b = pick[fb][rng.integers(0, 4, (N, K))] | (rng.integers(0, 2, (N, K)).astype(np.uint8) << 7)
    a[:, ::7] = 0                                                   # break any symmetry between k positions
    sr = np.ones(M, np.float32)
    one = torch.ones(1, dtype=torch.float32, device=DEV)
    o32 = sb.matmul_f8_dequant(u8_dev(a), fa, u8_dev(sr), u8_dev(b), fb, one, out_dtype=torch.float32)
    torch.cuda.synchronize()
    acc = oracle.matmul_f8(a, fa, b, fb)
    assert np.abs(acc).max() > 10
    np.testing.assert_array_equal(host(o32).astype(np.float64), acc)


def test_float8_matrix_instruction_arithmetic_behind_the_tolerance(oracle):
    """The premises of f8_product_tolerance, checked through the product call with crafted operands (E4M3 codes 0x38 =
    1, 0x09 = 1.125 * 2^-6, 0x01 = 2^-9; one token row against one weight row, K = 128, everything else zero):
      * aligned groups of 8 consecutive k share one alignment step: a small product in the group of a large one is
        truncated below 2^-13 of the large product's power of two (1 + (1.125 * 2^-6)^2 = 1 + 2^-12 + 2^-14 + 2^-18
        comes back as 1 + 2^-12), so a group loses less than 7 * 2^-13 of its largest product;
      * the same small product in ANY other group of 8 is added exactly;
      * 1 + 63 * 2^-18 comes back as 1 + 56 * 2^-18: the seven tiny products sharing the group of the 1 vanish, the seven
        groups of eight tiny products are exact.
    Every case must also lie within the tolerance the parity tests use."""
    K = 128
    one = torch.ones(1, dtype=torch.float32, device=DEV)

    def product(a_row, b_row):
        a = np.zeros((1, K), np.uint8)
        b = np.zeros((64, K), np.uint8)
        a[0, :len(a_row)] = a_row
        b[0, :len(b_row)] = b_row
        got = host(sb.matmul_f8_dequant(u8_dev(a), 0, one, u8_dev(b), 0, one, out_dtype=torch.float32))
        acc, abs_acc = oracle.matmul_f8(a, 0, b, 0, want_abs=True)
        tol = f8_product_tolerance(abs_acc, np.ones(1, np.float32), K) + ulp(acc.astype(np.float32))
        assert (np.abs(got.astype(np.float64) - acc) <= tol).all()
        assert not got[0, 1:].any()
        return float(got[0, 0]), float(acc[0, 0])

    small = (1.125 * 2.0 ** -6) ** 2
    for pos in range(1, 8):                                    # same group of 8 as the large product: truncated
        row = [0x38] + [0] * (pos - 1) + [0x09]
        got, exact = product(row, row)
        assert exact == 1.0 + small
        assert got == 1.0 + 2.0 ** -12, (pos, got)
    for pos in (8, 9, 15, 16, 31, 32, 33, 63, 64, 127):        # any other group, either instruction: exact
        row = [0x38] + [0] * (pos - 1) + [0x09]
        got, exact = product(row, row)
        assert got == exact == 1.0 + small, (pos, got)
    row = [0x38] + [0x01] * 63
    got, exact = product(row, row)
    assert exact == 1.0 + 63 * 2.0 ** -18
    assert got == 1.0 + 56 * 2.0 ** -18, got
    row = [0x01] * 64                                           # no large product: nothing to align to, exact
    got, exact = product(row, row)
    assert got == exact == 64 * 2.0 ** -18


def check_layer_f8(oracle, d, rows=None):
    x, w, dy = to_dev(d["x"]), to_dev(d["w"]), to_dev(d["dy"])
    b, n = d["x"].shape
    m = d["w"].shape[0]
    bufs = sb.LayerBuffers(b, n, m, DEV)
    y32, _ = sb.forward_f8(x, w, bufs=bufs, y_dtype=torch.float32)
    ybf, _ = sb.forward_f8(x, w, bufs=bufs, y_dtype=torch.bfloat16)
    dx32 = sb.backward_input_f8(dy, bufs, dx_dtype=torch.float32)
    dxbf = sb.backward_input_f8(dy, bufs, dx_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    xq, sx = oracle.quantize_rowwise_f8(d["x"], oracle.E4M3)
    wq, wq_t, sw = oracle.quantize_tensorwise_f8(d["w"], oracle.E4M3)
    gq, sg = oracle.quantize_rowwise_f8(d["dy"], oracle.E5M2)
    as_u8 = lambda t: host(t).view(np.uint8)
    np.testing.assert_array_equal(as_u8(bufs.xq), xq)
    np.testing.assert_array_equal(host(bufs.state_x).view(np.uint32), sx.view(np.uint32))
    np.testing.assert_array_equal(as_u8(bufs.wq), wq)
    np.testing.assert_array_equal(as_u8(bufs.wq_t), wq_t)
    assert host(bufs.state_w).view(np.uint32)[0] == np.float32(sw).view(np.uint32)
    np.testing.assert_array_equal(as_u8(bufs.gq), gq)
    np.testing.assert_array_equal(host(bufs.state_g).view(np.uint32), sg.view(np.uint32))
    rows = np.arange(b) if rows is None else rows
    idx = torch.from_numpy(rows).to(DEV)
    acc, abs_acc = oracle.matmul_f8(xq[rows], oracle.E4M3, wq, oracle.E4M3, want_abs=True)
    assert_f8_outputs(host(y32[idx]), bits_of(ybf[idx]), acc, abs_acc, sx[rows], sw, n, oracle)
    acc, abs_acc = oracle.matmul_f8(gq[rows], oracle.E5M2, wq_t, oracle.E4M3, want_abs=True)
    assert_f8_outputs(host(dx32[idx]), bits_of(dxbf[idx]), acc, abs_acc, sg[rows], sw, m, oracle)
    return host(y32), host(dx32)


def test_float8_layer_tiny_with_edge_rows(oracle):
    d = I.make_layer_inputs("tiny")
    I.plant_edge_rows(d["x"])
    I.plant_edge_rows(d["dy"])
    y, dx = check_layer_f8(oracle, d)
    assert not y[0].any()                  # zero row -> zero output (1/1e-38 is finite: the tiny row is a live row here)


@pytest.mark.parametrize("b,n,m", [(1, 128, 128), (33, 256, 384), (300, 128, 640), (1000, 384, 256)])
def test_float8_layer_ragged_shapes(oracle, b, n, m):
    rng = np.random.default_rng(b + n + m)
    d = dict(x=rand_bf16(rng, (b, n)), w=rand_bf16(rng, (m, n), n ** -0.5), dy=rand_bf16(rng, (b, m), 0.1))
    check_layer_f8(oracle, d)


@pytest.mark.parametrize("config,layer", [("vit_b16", 0), ("vit_b16", 1), ("vit_l14", 0), ("vit_l14", 1), ("vit_l14", 2),
                                          ("vit_l14", 3), ("vit_h14", 0), ("vit_h14", 1), ("vit_h14", 2), ("vit_h14", 3),
                                          ("outlier", 0), ("outlier", 1)])
def test_float8_layer_full_size_sampled(oracle, config, layer):
    L = I.CONFIGS[config].layers[layer]
    d = I.make_layer_inputs(config, layer)
    check_layer_f8(oracle, d, one_row_per_block(L.b, 32, np.random.default_rng(29)))


def test_float8_layer_is_deterministic_and_rejects_unsupported_widths():
    d = I.make_layer_inputs("tiny")
    x, w = to_dev(d["x"]), to_dev(d["w"])
    a, _ = sb.forward_f8(x, w)
    b, _ = sb.forward_f8(x, w)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(bits_of(a), bits_of(b))
    with pytest.raises(sb.SwitchBackError):
        sb.forward_f8(x[:, :192].contiguous(), w[:, :192].contiguous())     # n % 128 != 0


# ---------------------------------------------------------------------------------------------------------------
# seeded random shapes: ragged M, every multiple-of-64 width class, all kernel instances (which one runs depends on
# K % 128 and on the tile count), every output mode, whole outputs
# ---------------------------------------------------------------------------------------------------------------

def random_shapes(seed, count, max_m, max_n, max_k):
    rng = np.random.default_rng(seed)
    return [(int(rng.integers(1, max_m + 1)), 64 * int(rng.integers(1, max_n // 64 + 1)),
             64 * int(rng.integers(1, max_k // 64 + 1))) for _ in range(count)]


@pytest.mark.parametrize("M,N,K", random_shapes(101, 16, 2500, 1536, 1024) + random_shapes(102, 6, 12000, 6144, 384))
def test_int8_product_random_shapes(oracle, M, N, K):
    rng = np.random.default_rng(M * 7 + N * 3 + K)
    a = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    b = rng.integers(-127, 128, size=(N, K)).astype(np.int8)
    srow = (rng.random(M) * 2 + 0.25).astype(np.float32)
    check_int8_product_whole(oracle, a, b, srow, 0.4375)
    bias, gamma = rng.standard_normal(N).astype(np.float32), rng.standard_normal(N).astype(np.float32)
    dev = lambda v: torch.from_numpy(v).to(DEV)
    args = (dev(a), dev(srow), dev(b), torch.tensor([0.4375], device=DEV), dev(bias), dev(gamma))
    o32 = host(sb.matmul_int8_dequant_bias_layerscale(*args, out_dtype=torch.float32))
    obf = bits_of(sb.matmul_int8_dequant_bias_layerscale(*args, out_dtype=torch.bfloat16))
    assert_bias_layerscale(o32, obf, oracle.matmul_int8(a, b), srow, 0.4375, bias, gamma, oracle)


@pytest.mark.parametrize("b,n,m", [(mm, nn, kk) for (mm, nn, kk) in random_shapes(103, 10, 5000, 1024, 1024)])
def test_weight_gradient_random_shapes(oracle, b, n, m):
    rng = np.random.default_rng(b + 5 * n + 11 * m)
    dyb, xb = rand_bf16(rng, (b, m), 0.1), rand_bf16(rng, (b, n))
    dw32 = host(sb.backward_weight(to_dev(dyb), to_dev(xb), dw_dtype=torch.float32))
    dw_ref = oracle.weight_grad(dyb, xb)
    assert np.abs(dw32.astype(np.float64) - dw_ref).max() <= 1e-2 * float(np.sqrt((dw_ref ** 2).mean()))


# ---------------------------------------------------------------------------------------------------------------
# maximum sizes: operands that end just below the 4 GiB reach of the kernels' 32-bit buffer offsets
# ---------------------------------------------------------------------------------------------------------------

def test_int8_product_at_the_largest_operand(oracle):
    """aq of (M + 256) * K = 2^32 - 4096 bytes: the last tile's addresses, including the rows past M that must read as
    zero, end just below 2^32.  Inputs are drawn on the GPU (seeded); the oracle gets the sampled rows."""
    M, N, K = 1048319, 64, 4096
    assert (M + 256) * K < 2 ** 32 <= (M + 257) * K
    g = torch.Generator(device=DEV)
    g.manual_seed(41)
    a = torch.randint(-127, 128, (M, K), generator=g, device=DEV, dtype=torch.int8)
    b = torch.randint(-127, 128, (N, K), generator=g, device=DEV, dtype=torch.int8)
    sr = torch.rand(M, generator=g, device=DEV) + 0.5
    sw = torch.tensor([0.731], device=DEV)
    acc = sb.matmul_int8_dequant(a, None, b, None, out_dtype=torch.int32)
    ybf = sb.matmul_int8_dequant(a, sr, b, sw, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    rng = np.random.default_rng(42)
    rows = np.unique(np.concatenate([[0, 255, 256, M - 256 - 63, M - 64, M - 2, M - 1], rng.integers(0, M, 40)]))
    idx = torch.from_numpy(rows).to(DEV)
    ref = oracle.matmul_int8(host(a[idx]), host(b))
    np.testing.assert_array_equal(host(acc[idx]), ref)
    y = oracle.dequantize(ref, host(sr[idx]), np.float32(0.731))
    assert_bf16_is_rounding_within_one_ulp(bits_of(ybf[idx]), y, oracle)
    # one more row would not be addressable: the boundary says so instead of launching
    with pytest.raises(sb.SwitchBackError):
        sb.matmul_int8_dequant(torch.empty((M + 1, K), dtype=torch.int8, device=DEV), sr, b, sw)


def test_weight_gradient_at_the_largest_operand(oracle):
    """X of (b + 256) * n * 2 bytes just below 2^32 (bf16): split-K over a million tokens, ragged last token tile."""
    b, n, m = 1048319, 2048, 64
    assert (b + 256) * n * 2 < 2 ** 32 <= (b + 257) * n * 2
    g = torch.Generator(device=DEV)
    g.manual_seed(43)
    x = torch.randn((b, n), generator=g, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    dy = (torch.randn((b, m), generator=g, device=DEV, dtype=torch.float32) * 0.1).to(torch.bfloat16)
    dw = sb.backward_weight(dy, x, dw_dtype=torch.float32)
    torch.cuda.synchronize()
    jrows = np.array([0, 31, 63])
    ref = oracle.weight_grad(np.ascontiguousarray(bits_of(dy)[:, jrows]), bits_of(x))
    rms = float(np.sqrt((ref ** 2).mean()))
    got = host(dw)[jrows].astype(np.float64)
    assert np.abs(got - ref).max() <= 1e-2 * rms


# ---------------------------------------------------------------------------------------------------------------
# repeatability at full size: the GEMM kernels order their memory traffic with hand-counted waits, so the same launch
# is repeated many times on the benchmark's shapes and every result must equal the first bit for bit
# ---------------------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("config,layer", [("vit_h14", 1), ("vit_h14", 2), ("vit_h14", 3), ("vit_l14", 1),
                                          ("vit_b16", 0), ("vit_b16", 1)])
def test_products_are_repeatable_at_full_size(config, layer):
    """ViT-H/14: the 256 x 256-tile instances; ViT-L/14 proj and ViT-B/16: the 128 x 128-tile instances of the weight
    gradient (and, for ViT-B/16's 768-wide outputs, of the 8-bit products)."""
    L = I.CONFIGS[config].layers[layer]
    g = torch.Generator(device=DEV)
    g.manual_seed(50 + layer)
    x = torch.randn((L.b, L.n), generator=g, device=DEV).to(torch.bfloat16)
    w = (torch.randn((L.m, L.n), generator=g, device=DEV) * L.n ** -0.5).to(torch.bfloat16)
    dy = (torch.randn((L.b, L.m), generator=g, device=DEV) * 0.1).to(torch.bfloat16)
    bufs = sb.LayerBuffers(L.b, L.n, L.m, DEV)
    y0, _ = sb.forward(x, w, bufs=bufs)
    dx0 = sb.backward_input(dy, bufs)
    dw0 = sb.backward_weight(dy, x, bufs)
    y, dx, dw = torch.empty_like(y0), torch.empty_like(dx0), torch.empty_like(dw0)
    for rep in range(25):
        y.fill_(1.0), dx.fill_(1.0), dw.fill_(1.0)
        sb.matmul_int8_dequant(bufs.xq, bufs.state_x, bufs.wq, bufs.state_w, out=y)
        sb.matmul_int8_dequant(bufs.gq, bufs.state_g, bufs.wq_t, bufs.state_w, out=dx)
        sb.backward_weight(dy, x, bufs, dw=dw)
        assert torch.equal(y, y0) and torch.equal(dx, dx0) and torch.equal(dw, dw0), "repetition %d differs" % rep
    y8, _ = sb.forward_f8(x, w, bufs=bufs)
    y8b = torch.empty_like(y8)
    u8 = lambda q: q.view(torch.uint8)
    for rep in range(25):
        y8b.fill_(1.0)
        sb.matmul_f8_dequant(u8(bufs.xq), sb.SB_E4M3, bufs.state_x, u8(bufs.wq), sb.SB_E4M3, bufs.state_w, out=y8b)
        assert torch.equal(y8b, y8), "float8 repetition %d differs" % rep
