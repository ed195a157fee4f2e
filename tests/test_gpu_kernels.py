"""GPU parity, kernel by kernel: each C-ABI call against the fp64 CPU oracle on the same
seeded inputs, element by element (sizes the oracle finishes in seconds, spanning several
tiles and ragged tails)."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2109_12191_amd as dp
from gpu_util import BF16_TOL, F32_TOL, assert_close, dev, host
from workloads import Layer, conv, dense, gn_affine, to_bf16_grid

pytestmark = pytest.mark.gpu


def _inputs(layer, n, seed, dtype, x_abs=False, dy_std=0.05):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((n,) + tuple(layer.x_shape)).astype(np.float32)
    if x_abs:
        x = np.abs(x)
    dy = (rng.standard_normal((n,) + tuple(layer.dy_shape)) * dy_std).astype(np.float32)
    if dtype == "bf16":
        x, dy = to_bf16_grid(x), to_bf16_grid(dy)
    return x, dy


def _oracle_grads(layer, x, dy):
    gw, gb, n2 = [], [], []
    for i in range(x.shape[0]):
        w, b = oracle.example_grad(layer, x[i], dy[i])
        gw.append(w.reshape(-1))
        gb.append(b if b is not None else np.zeros(0))
        n2.append(oracle.sqnorm(w) + (oracle.sqnorm(b) if b is not None else 0.0))
    return np.stack(gw), np.stack(gb), np.array(n2)


def _run_per_example(layer, x, dy, dtype, materialise=True, g_stride=0):
    n = x.shape[0]
    d = dp.make_desc(layer, n, dtype)
    pw, pb = dp.dp_weight_count(d), dp.dp_bias_count(d)
    assert (pw, pb) == (layer.pw, layer.pb)
    ws = torch.empty(max(16, dp.dp_workspace_bytes(d)), dtype=torch.uint8, device="cuda:0")
    sq = torch.full((n,), -1.0, device="cuda:0")
    xd, dyd = dev(x, dtype), dev(dy, dtype)
    if not materialise:
        dp.dp_per_example_grad(d, xd, dyd, None, None, sq, ws)
        torch.cuda.synchronize()
        return None, None, host(sq)
    if g_stride:
        g = torch.full((n, g_stride), 7.0, device="cuda:0")
        off_b = (pw + 3) & ~3
        dp.dp_per_example_grad(d, xd, dyd, g.data_ptr(), g[:, off_b:].data_ptr() if pb else None, sq, ws,
                               g_stride=g_stride)
        torch.cuda.synchronize()
        gh = host(g)
        assert np.all(gh[:, off_b + pb:] == 7.0) and np.all(gh[:, pw:off_b] == 7.0)   # nothing else touched
        return gh[:, :pw], gh[:, off_b:off_b + pb], host(sq)
    gw = torch.full((n, pw), 7.0, device="cuda:0")
    gb = torch.full((n, max(pb, 1)), 7.0, device="cuda:0")
    dp.dp_per_example_grad(d, xd, dyd, gw, gb if pb else None, sq, ws)
    torch.cuda.synchronize()
    return host(gw), host(gb)[:, :pb], host(sq)


CONV_CASES = [
    # name, layer, n
    ("3x3 s1 ragged tiles", Layer("conv", 20, 70, 12, 12, 3, 3, 1, 1, False), 3),
    ("3x3 s1 bias small", Layer("conv", 3, 16, 10, 9, 3, 3, 1, 1, True), 4),
    ("3x3 s2 big", Layer("conv", 40, 200, 15, 15, 3, 3, 2, 1, False), 2),
    ("1x1 s1 direct S=196", conv(150, 130, 1, 1, 14), 3),
    ("1x1 s1 direct S=49 bias", conv(96, 72, 1, 1, 7, bias=True), 3),
    ("1x1 s1 direct S=225 odd", conv(33, 65, 1, 1, 15), 2),
    ("1x1 s2", conv(48, 80, 1, 2, 14), 2),
    ("7x7 s2 cin3", conv(3, 64, 7, 2, 32), 2),
    ("5x3 rect nopad", Layer("conv", 6, 9, 11, 13, 5, 3, 1, 0, True), 2),
    ("long K several chunks", conv(8, 24, 3, 1, 40, bias=True), 2),
    ("256 x 64 output", conv(40, 200, 1, 1, 12), 3),
    ("64 x 256 output", conv(30, 48, 3, 1, 12, bias=True), 3),
    ("3x3 long K sliced", conv(24, 64, 3, 1, 56), 1),
    ("many examples per workgroup", conv(8, 8, 1, 1, 4, bias=True), 1700),
    ("256 x 128 tiles eight waves short K with tail", conv(256, 256, 1, 1, 10), 64),
    ("whole rows in blocks of 32, 14 x 14 maps", conv(256, 512, 1, 1, 14), 64),
    ("whole rows in blocks of 32, two column ranges", conv(512, 256, 1, 1, 14), 64),
    ("whole rows in blocks of 32, rows of 204", Layer("conv", 256, 256, 12, 17, 1, 1, 1, 0, False), 128),
    ("3x3 s1 odd width 7", conv(72, 136, 3, 1, 7), 5),
    ("3x3 s2 odd width 15->8", conv(16, 80, 3, 2, 15), 3),
    ("stride 3", Layer("conv", 6, 10, 14, 17, 3, 3, 3, 1, False), 2),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("name,layer,n", CONV_CASES, ids=[c[0] for c in CONV_CASES])
def test_conv_per_example_grad_and_norm(name, layer, n, dtype):
    tol = F32_TOL if dtype == "f32" else BF16_TOL
    x, dy = _inputs(layer, n, 101, dtype)
    ref_w, ref_b, ref_n2 = _oracle_grads(layer, x, dy)
    gw, gb, sq = _run_per_example(layer, x, dy, dtype)
    for i in range(n):
        assert_close(gw[i], ref_w[i], tol, f"{name} dW[{i}]")
        if layer.pb:
            assert_close(gb[i], ref_b[i], tol, f"{name} db[{i}]")
    assert np.allclose(sq, ref_n2, rtol=tol, atol=0), (sq, ref_n2)
    # norms-only call gives the same norms bit for bit (same kernel, no store)
    _, _, sq2 = _run_per_example(layer, x, dy, dtype, materialise=False)
    assert np.array_equal(sq, sq2)


# 3x3 stride-1 pad-1 bf16 layers with >= 64 channels run in the raw-row kernel: every supported
# row width, ragged channel counts, image heights that leave a partial last chunk, K sliced over
# workgroups (few tiles) and unsliced (many).
ROWS_CASES = [
    ("w56 three chunks sliced", Layer("conv", 64, 64, 10, 56, 3, 3, 1, 1, False), 2, None),
    ("w28 ragged channels", Layer("conv", 80, 72, 28, 28, 3, 3, 1, 1, False), 2, None),
    ("w14 one chunk", Layer("conv", 130, 64, 14, 14, 3, 3, 1, 1, False), 3, None),
    ("w16 short image", Layer("conv", 64, 96, 9, 16, 3, 3, 1, 1, False), 2, None),
    ("w32 two chunks", Layer("conv", 64, 64, 12, 32, 3, 3, 1, 1, False), 2, None),
    ("w8 one chunk", Layer("conv", 64, 64, 8, 8, 3, 3, 1, 1, False), 3, None),
    ("w7 tall image", Layer("conv", 64, 70, 19, 7, 3, 3, 1, 1, False), 2, None),
    ("w8 two chunks unsliced many examples", Layer("conv", 64, 64, 11, 8, 3, 3, 1, 1, False), 520, [0, 1, 259, 518, 519]),
    # stride 2 (rows of X split by column parity first): output widths 28, 14 and 7
    ("s2 28->14 ragged channels", Layer("conv", 80, 72, 28, 28, 3, 3, 2, 1, False), 3, None),
    ("s2 14->7", Layer("conv", 128, 64, 14, 14, 3, 3, 2, 1, False), 3, None),
    ("s2 short image 12x28 -> 6x14", Layer("conv", 64, 96, 12, 28, 3, 3, 2, 1, False), 2, None),
    ("s2 14->7 unsliced many examples", Layer("conv", 64, 64, 14, 14, 3, 3, 2, 1, False), 515, [0, 1, 300, 513, 514]),
    ("s2 56->28 last chunk of one row", Layer("conv", 64, 96, 20, 56, 3, 3, 2, 1, False), 3, None),
    ("s2 56->28 ragged channels", Layer("conv", 80, 72, 56, 56, 3, 3, 2, 1, False), 3, None),
]


@pytest.mark.parametrize("name,layer,n,sample", ROWS_CASES, ids=[c[0] for c in ROWS_CASES])
def test_conv3x3_raw_row_kernel(name, layer, n, sample):
    d = dp.make_desc(layer, n, "bf16")
    assert dp.dp_kernel_variant(d, dp.DP_WS_PER_EXAMPLE_GRAD).startswith("conv3x3_rows")
    x, dy = _inputs(layer, n, 211, "bf16")
    gw, _, sq = _run_per_example(layer, x, dy, "bf16")
    _, _, sq2 = _run_per_example(layer, x, dy, "bf16", materialise=False)
    assert np.array_equal(sq, sq2)
    for i in (sample if sample is not None else range(n)):
        w, _ = oracle.example_grad(layer, x[i], dy[i])
        assert_close(gw[i], w.reshape(-1), BF16_TOL, f"{name} dW[{i}]")
        assert math.isclose(sq[i], oracle.sqnorm(w), rel_tol=BF16_TOL), (i, sq[i], oracle.sqnorm(w))


# The network's first convolution (7x7, stride 2, pad 3, 64 output channels, a few input channels, bf16) has a kernel of
# its own: output rows split over workgroups two at a time (odd last range), one to three input channels, wide and narrow maps.
STEM_CASES = [
    ("64x64 three channels", conv(3, 64, 7, 2, 64), 3),
    ("224x224 three channels", conv(3, 64, 7, 2, 224), 2),
    ("38x96 last range of one row", Layer("conv", 3, 64, 38, 96, 7, 7, 2, 3, False), 2),
    ("one channel 32x32", conv(1, 64, 7, 2, 32), 5),
    ("two channels 8x32 one range", Layer("conv", 2, 64, 8, 32, 7, 7, 2, 3, False), 4),
]


@pytest.mark.parametrize("name,layer,n", STEM_CASES, ids=[c[0] for c in STEM_CASES])
def test_conv_stem_kernel(name, layer, n):
    d = dp.make_desc(layer, n, "bf16")
    assert dp.dp_kernel_variant(d, dp.DP_WS_PER_EXAMPLE_GRAD) == "conv_stem7x7<bf16,per_example>"
    x, dy = _inputs(layer, n, 223, "bf16")
    gw, _, sq = _run_per_example(layer, x, dy, "bf16")
    _, _, sq2 = _run_per_example(layer, x, dy, "bf16", materialise=False)
    assert np.array_equal(sq, sq2)
    gws, _, sq3 = _run_per_example(layer, x, dy, "bf16", g_stride=layer.pw + 12)
    assert np.array_equal(gws, gw) and np.array_equal(sq3, sq)
    for i in range(n):
        w, _ = oracle.example_grad(layer, x[i], dy[i])
        assert_close(gw[i], w.reshape(-1), BF16_TOL, f"{name} dW[{i}]")
        assert math.isclose(sq[i], oracle.sqnorm(w), rel_tol=BF16_TOL), (i, sq[i], oracle.sqnorm(w))


def test_conv_strided_gradient_matrix_layout():
    layer = Layer("conv", 5, 9, 8, 8, 3, 3, 1, 1, True)
    x, dy = _inputs(layer, 3, 103, "f32")
    ref_w, ref_b, ref_n2 = _oracle_grads(layer, x, dy)
    gw, gb, sq = _run_per_example(layer, x, dy, "f32", g_stride=432)   # 405 -> pad 408, +9 bias, slack
    assert_close(gw, ref_w, F32_TOL, "strided dW")
    assert_close(gb, ref_b, F32_TOL, "strided db")
    assert np.allclose(sq, ref_n2, rtol=F32_TOL)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("layer", [dense(784, 256), dense(256, 10), dense(300, 37, tokens=3), dense(5, 3, bias=False)],
                         ids=["784x256", "256x10", "300x37xT3", "5x3nobias"])
def test_dense_per_example_grad_and_norm(layer, dtype):
    tol = F32_TOL if dtype == "f32" else BF16_TOL
    x, dy = _inputs(layer, 5, 107, dtype)
    ref_w, ref_b, ref_n2 = _oracle_grads(layer, x, dy)
    gw, gb, sq = _run_per_example(layer, x, dy, dtype)
    assert_close(gw, ref_w, tol, "dense dW")
    if layer.pb:
        assert_close(gb, ref_b, tol, "dense db")
    assert np.allclose(sq, ref_n2, rtol=tol)
    _, _, sq2 = _run_per_example(layer, x, dy, dtype, materialise=False)
    if layer.h == 1:
        # one token per example: the norm-only call uses |dy|^2 |x|^2 (+ |dy|^2), the same number
        # up to fp32 rounding order
        assert np.allclose(sq2, ref_n2, rtol=F32_TOL), (sq2, ref_n2)
    else:
        assert np.array_equal(sq, sq2)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("c,hw,groups", [(16, 32, 8), (64, 8, 8), (24, 5, 3), (32, 7, 32), (64, 56, 32), (600, 3, 2)])
def test_groupnorm_affine_grad_and_norm(c, hw, groups, dtype):
    tol = F32_TOL if dtype == "f32" else BF16_TOL
    layer = gn_affine(c, hw, groups)
    x, dy = _inputs(layer, 4, 109, dtype)
    x = x * 1.5 + 0.25
    if dtype == "bf16":
        x = to_bf16_grid(x)
    ref_w, ref_b, ref_n2 = _oracle_grads(layer, x, dy)
    gw, gb, sq = _run_per_example(layer, x, dy, dtype)
    assert_close(gw, ref_w, tol, "dgamma")
    assert_close(gb, ref_b, tol, "dbeta")
    assert np.allclose(sq, ref_n2, rtol=tol)


def test_norms_and_clip_factors():
    rng = np.random.default_rng(5)
    L, n, G = 7, 37, 3
    layer_sq = rng.uniform(0.0, 4.0, (L, n)).astype(np.float32)
    layer_sq[:, 5] = 0.0
    grp = np.array([0, 2, 1, 1, 0, 2, 2], dtype=np.int32)
    out = torch.full((G, n), -1.0, device="cuda:0")
    dp.dp_norms(dev(layer_sq), torch.from_numpy(grp).cuda(), L, n, G, out)
    got = host(out)
    ref = np.stack([layer_sq[grp == g].astype(np.float64).sum(0) for g in range(G)])
    assert np.allclose(got, ref, rtol=1e-6)
    for c in (0.5, 1.7, math.inf):
        f = torch.empty(n, device="cuda:0")
        dp.dp_clip_factors(out[1], c, n, f)
        ref_f = np.array([oracle.clip_factor(v, c) for v in got[1]])
        assert np.allclose(host(f), ref_f, rtol=1e-6)
        assert host(f)[5] == 1.0


@pytest.mark.parametrize("n,p,stride", [(16, 36928, 0), (5, 1001, 0), (33, 4096, 4100), (3, 7, 8), (1100, 64, 0)])
def test_clip_accumulate_materialised(n, p, stride):
    rng = np.random.default_rng(11)
    s = stride or p
    g = rng.standard_normal((n, s)).astype(np.float32)
    n2 = (rng.uniform(0.2, 3.0, n) ** 2).astype(np.float32)
    n2[0] = 0.0
    acc0 = rng.standard_normal(p).astype(np.float32)
    c = 1.0
    f = np.array([oracle.clip_factor(float(v), c) for v in n2])
    ref = acc0.astype(np.float64) + (f[:, None] * g[:, :p].astype(np.float64)).sum(0)
    acc = dev(acc0)
    dp.dp_clip_accumulate(dev(g), dev(n2), c, n, p, acc, g_stride=stride)
    assert_close(host(acc), ref, F32_TOL, "clip_accumulate")
    # twice the same call from the same start gives the same bits (fixed summation order)
    acc2 = dev(acc0)
    dp.dp_clip_accumulate(dev(g), dev(n2), c, n, p, acc2, g_stride=stride)
    assert torch.equal(acc, acc2)


RECOMPUTE_CASES = [
    ("conv 3x3 bias", Layer("conv", 20, 70, 12, 12, 3, 3, 1, 1, True), 9),
    ("conv 1x1 S=49", conv(96, 136, 1, 1, 7), 6),
    ("conv 3x3 s2", conv(24, 40, 3, 2, 14), 5),
    ("conv small long K", conv(8, 24, 3, 1, 40, bias=True), 3),
    ("conv many examples", conv(64, 200, 1, 1, 7), 40),
    ("conv 3x3 biased small", conv(30, 48, 3, 1, 12, bias=True), 6),
    ("conv 1x1 cout 200", conv(40, 200, 1, 1, 12), 6),
    ("dense", dense(300, 37, tokens=2), 7),
    ("dense fc", dense(784, 256), 6),
    ("gn", gn_affine(16, 9, 4), 6),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("name,layer,n", RECOMPUTE_CASES, ids=[c[0] for c in RECOMPUTE_CASES])
def test_clip_accumulate_recompute(name, layer, n, dtype):
    tol = F32_TOL if dtype == "f32" else BF16_TOL
    x, dy = _inputs(layer, n, 113, dtype)
    rng = np.random.default_rng(17)
    n2 = (rng.uniform(0.3, 2.5, n) ** 2).astype(np.float32)     # both branches of the clip
    n2[1] = 0.0
    c = 1.0
    f = np.array([oracle.clip_factor(float(v), c) for v in n2])
    acc0_w = rng.standard_normal(layer.pw).astype(np.float32) * 0.01
    acc0_b = rng.standard_normal(max(layer.pb, 1)).astype(np.float32) * 0.01
    ref_w = acc0_w.astype(np.float64) + oracle.weighted_sum_elems(layer, x, dy, f, np.arange(layer.pw))
    d = dp.make_desc(layer, n, dtype)
    ws = torch.empty(max(16, dp.dp_workspace_bytes(d, dp.DP_WS_RECOMPUTE)), dtype=torch.uint8, device="cuda:0")
    aw, ab = dev(acc0_w), dev(acc0_b)
    dp.dp_clip_accumulate_recompute(d, dev(x, dtype), dev(dy, dtype), dev(n2), c, aw, ab if layer.pb else None, ws)
    # compare the increment (the part the call computes) as well as the total
    assert_close(host(aw) - acc0_w, ref_w - acc0_w, tol, f"{name} acc_w increment")
    if layer.pb:
        ref_b = acc0_b[:layer.pb].astype(np.float64) + oracle.weighted_sum_elems(layer, x, dy, f, np.arange(layer.pb),
                                                                                  bias=True)
        assert_close(host(ab)[:layer.pb] - acc0_b[:layer.pb], ref_b - acc0_b[:layer.pb], tol, f"{name} acc_b increment")


ROWS_WEIGHTED_CASES = [
    # name, layer, n  (raw-row kernel in its clip-weighted mode: example ranges through the workspace, or one range)
    ("w7 ranges", Layer("conv", 128, 128, 7, 7, 3, 3, 1, 1, False), 9),
    ("w14 ragged channels ranges", Layer("conv", 80, 72, 14, 14, 3, 3, 1, 1, False), 5),
    ("w28 two chunks", Layer("conv", 64, 64, 10, 28, 3, 3, 1, 1, False), 3),
    ("w56 short image", Layer("conv", 64, 64, 6, 56, 3, 3, 1, 1, False), 2),
    ("w8 many tiles one range", Layer("conv", 1024, 1024, 8, 8, 3, 3, 1, 1, False), 2),
]


@pytest.mark.parametrize("name,layer,n", ROWS_WEIGHTED_CASES, ids=[c[0] for c in ROWS_WEIGHTED_CASES])
def test_conv3x3_raw_row_kernel_weighted(name, layer, n):
    d = dp.make_desc(layer, n, "bf16")
    assert dp.dp_kernel_variant(d, dp.DP_WS_RECOMPUTE).startswith("conv3x3_rows")
    x, dy = _inputs(layer, n, 223, "bf16")
    rng = np.random.default_rng(19)
    n2 = (rng.uniform(0.3, 2.5, n) ** 2).astype(np.float32)
    n2[1] = 0.0
    f = np.array([oracle.clip_factor(float(v), 1.0) for v in n2])
    acc0 = rng.standard_normal(layer.pw).astype(np.float32) * 0.01
    idx = np.arange(layer.pw) if layer.pw <= 200_000 else rng.choice(layer.pw, size=20_000, replace=False)
    ref = oracle.weighted_sum_elems(layer, x, dy, f, idx)
    ws = torch.empty(max(16, dp.dp_workspace_bytes(d, dp.DP_WS_RECOMPUTE)), dtype=torch.uint8, device="cuda:0")
    aw = dev(acc0)
    dp.dp_clip_accumulate_recompute(d, dev(x, "bf16"), dev(dy, "bf16"), dev(n2), 1.0, aw, None, ws)
    got = host(aw)
    assert_close(got[idx] - acc0[idx], ref, BF16_TOL, f"{name} increment")
    # same call again from the same start: same bits
    aw2 = dev(acc0)
    dp.dp_clip_accumulate_recompute(d, dev(x, "bf16"), dev(dy, "bf16"), dev(n2), 1.0, aw2, None, ws)
    assert torch.equal(aw, aw2)


def test_philox_integer_stream_is_bit_exact():
    for seed, step, tid, p in [(0, 0, 0, 1), (0, 0, 0, 3), (0, 0, 1, 1027), (0x123456789ABCDEF, 0x100000005, 77, 4096),
                               (2**64 - 1, 2**40 + 3, 2**32 - 1, 65537), (42, 7, 3, 1_000_001)]:
        raw = torch.zeros(p, dtype=torch.int32, device="cuda:0")
        dp.dp_philox_raw(raw, p, seed, step, tid)
        got = raw.cpu().numpy().view(np.uint32)
        assert np.array_equal(got, oracle.noise_raw(seed, step, tid, p)), (seed, step, tid, p)


@pytest.mark.parametrize("p", [1, 6, 4099, 203_530])
def test_noise_finalize_matches_oracle(p):
    rng = np.random.default_rng(19)
    acc = rng.standard_normal(p).astype(np.float32)
    sigma, c, b, seed, step, tid = 1.1, 1.5, 256, 9, 4, 6
    ref = oracle.noise_finalize(acc.astype(np.float64), sigma, c, b, seed, step, tid)
    a = dev(acc)
    out = torch.empty(p, device="cuda:0")
    dp.dp_add_noise_finalize(a, out, p, sigma, c, b, seed, step, tid)
    assert_close(host(out), ref, F32_TOL, "finalize")
    # noise alone (acc = 0): the normals themselves
    z = torch.zeros(p, device="cuda:0")
    dp.dp_add_noise_finalize(z, z, p, 1.0, 1.0, 1, seed, step, tid)       # in place
    assert_close(host(z), oracle.noise_normal(seed, step, tid, p), F32_TOL, "normals")
    # sigma = 0: plain division
    out0 = torch.empty(p, device="cuda:0")
    dp.dp_add_noise_finalize(a, out0, p, 0.0, c, b, seed, step, tid)
    assert_close(host(out0), acc.astype(np.float64) / b, 1e-6, "sigma=0")


def test_noise_moments_match_sigma_c_within_one_percent():
    p = 2_000_000
    sigma, c, b = 1.1, 1.0, 32
    out = torch.empty(p, device="cuda:0")
    dp.dp_add_noise_finalize(torch.zeros(p, device="cuda:0"), out, p, sigma, c, b, 0, 0, 0)
    z = host(out) * b
    assert abs(z.std() / (sigma * c) - 1.0) < 0.01
    assert abs(z.mean()) < 0.01 * sigma * c
    assert abs(np.mean(z ** 2) / (sigma * c) ** 2 - 1.0) < 0.01


PARTIAL_CASES = [
    ("generic conv, one tile row", conv(24, 40, 3, 1, 12, bias=True), 3, "f32"),
    ("generic conv, K sliced", conv(24, 64, 3, 1, 56), 1, "bf16"),
    ("1x1 flat", conv(150, 130, 1, 1, 14), 3, "bf16"),
    ("raw-row 3x3 unsliced", Layer("conv", 130, 64, 14, 14, 3, 3, 1, 1, False), 3, "bf16"),
    ("raw-row 3x3 sliced", Layer("conv", 64, 64, 10, 56, 3, 3, 1, 1, False), 2, "bf16"),
    ("dense one token", dense(300, 37), 5, "bf16"),
    ("dense three tokens", dense(300, 37, tokens=3), 4, "f32"),
    ("groupnorm", gn_affine(24, 5, 3), 4, "f32"),
]


@pytest.mark.parametrize("materialise", [False, True], ids=["norm_only", "materialise"])
@pytest.mark.parametrize("name,layer,n,dtype", PARTIAL_CASES, ids=[c[0] for c in PARTIAL_CASES])
def test_partial_norm_path_matches_reduced_norms(name, layer, n, dtype, materialise):
    """dp_per_example_grad_partials + dp_norms_from_partials give the norms dp_per_example_grad gives
    (two layers share a group here, so the reduction over layers is exercised too)."""
    x, dy = _inputs(layer, n, 307, dtype)
    if layer.kind == "gn":
        x = x * 1.5 + 0.25
        if dtype == "bf16":
            x = to_bf16_grid(x)
    d = dp.make_desc(layer, n, dtype)
    xd, dyd = dev(x, dtype), dev(dy, dtype)
    nbytes = max(16, dp.dp_workspace_bytes(d))
    sq = torch.zeros(n, device="cuda:0")
    ws0 = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    gw = torch.empty((n, layer.pw), device="cuda:0") if materialise else None
    gb = torch.empty((n, max(layer.pb, 1)), device="cuda:0") if materialise else None
    dp.dp_per_example_grad(d, xd, dyd, gw, gb if (materialise and layer.pb) else None, sq, ws0)
    wss = [torch.empty(nbytes, dtype=torch.uint8, device="cuda:0") for _ in range(2)]
    gw2 = torch.empty((n, layer.pw), device="cuda:0") if materialise else None
    for ws in wss:
        dp.dp_per_example_grad_partials(d, xd, dyd, gw2, gb if (materialise and layer.pb) else None, ws)
    count = dp.dp_norm_partial_count(d, materialise)
    table = dp.PartialTable([w.data_ptr() for w in wss], [count, count], [0, 0])
    out = torch.full((1, n), -1.0, device="cuda:0")
    dp.dp_norms_from_partials(table, n, 1, out)
    torch.cuda.synchronize()
    assert np.allclose(host(out)[0], 2.0 * host(sq), rtol=1e-5, atol=0), (host(out)[0], host(sq))
    if materialise:
        assert torch.equal(gw, gw2)


@pytest.mark.parametrize("p,sigma,momentum,with_out", [(4099, 1.1, 0.9, True), (6, 0.0, 0.0, False), (203_530, 0.7, 0.5, False),
                                                       (1024, 1.0, 0.0, True)])
def test_fused_noise_finalize_and_sgd_update(p, sigma, momentum, with_out):
    """dp_add_noise_finalize_update against the oracle: finalize in fp64, then its SGD step; two steps in a
    row so the momentum buffer is carried."""
    rng = np.random.default_rng(p)
    theta = rng.standard_normal(p).astype(np.float32)
    vel = (rng.standard_normal(p) * 0.1).astype(np.float32)
    use_v = momentum != 0.0 or p == 1024          # a buffer with momentum 0 is legal too
    th_d, v_d = dev(theta), dev(vel) if use_v else None
    th_ref, v_ref = theta.astype(np.float64), (vel.astype(np.float64) if use_v else None)
    for step in range(2):
        acc = (rng.standard_normal(p) * 3.0).astype(np.float32)
        out_d = torch.zeros(p, device="cuda:0") if with_out else None
        lr = 0.1 / (step + 1)
        dp.dp_add_noise_finalize_update(dev(acc), th_d, v_d, out_d, p, sigma, 1.5, 64, 42, step, 9, lr, momentum)
        g_ref = oracle.noise_finalize(acc, sigma, 1.5, 64, 42, step, 9)
        th_ref, v_ref = oracle.sgd_update(g_ref, th_ref, v_ref, lr, momentum)
        if with_out:
            assert_close(host(out_d), g_ref, F32_TOL, f"g step {step}")
            sep = torch.zeros(p, device="cuda:0")
            dp.dp_add_noise_finalize(dev(acc), sep, p, sigma, 1.5, 64, 42, step, 9)
            assert torch.equal(out_d, sep)             # the fused call forms the same gradient bits
        assert_close(host(th_d), th_ref, F32_TOL, f"theta step {step}")
        if use_v:
            assert_close(host(v_d), v_ref, F32_TOL, f"velocity step {step}")


@pytest.mark.parametrize("p,first,count,batch", [(4099, 0, 8, 8), (6, 3, 2, 16), (203_530, 32, 32, 256)])
def test_per_example_noise_form(p, first, count, batch):
    """dp_add_example_noise against the oracle: the sum of the per-example draws lands on the accumulator."""
    rng = np.random.default_rng(p)
    acc0 = (rng.standard_normal(p) * 0.5).astype(np.float32)
    acc = dev(acc0)
    dp.dp_add_example_noise(acc, p, 1.1, 0.9, batch, 0xABCDEF0123, 3, 5, first, count)
    ref = oracle.add_example_noise(acc0, 1.1, 0.9, batch, 0xABCDEF0123, 3, 5, first, count)
    assert_close(host(acc) - acc0, ref - acc0, F32_TOL, "per-example noise increment")
    # moments of what was added (count examples of variance sigma^2 C^2 / batch each)
    if p > 100_000:
        inc = host(acc) - acc0
        target = 1.1 * 0.9 * math.sqrt(count / batch)
        assert abs(inc.mean()) < 0.01 * target and abs(inc.std() / target - 1.0) < 0.01
    # sigma = 0 leaves the accumulator alone
    acc2 = dev(acc0)
    dp.dp_add_example_noise(acc2, p, 0.0, 0.9, batch, 1, 1, 1, first, count)
    assert torch.equal(acc2, dev(acc0))


@pytest.mark.parametrize("c,hw,groups", [(16, 12, 4), (520, 6, 2)], ids=["one sweep", "groups of 260 channels"])
def test_groupnorm_affine_with_a_large_mean_and_small_spread(c, hw, groups):
    """Statistics are taken about a shift (the group's first element), so a group whose values sit far from zero
    keeps its variance: the stated fp32 tolerance holds on both GroupNorm kernels."""
    layer = gn_affine(c, hw, groups)
    rng = np.random.default_rng(5)
    x = (rng.standard_normal((3,) + tuple(layer.x_shape)) * 0.05 + 40.0).astype(np.float32)
    dy = (rng.standard_normal((3,) + tuple(layer.dy_shape)) * 0.05).astype(np.float32)
    ref_w, ref_b, ref_n2 = _oracle_grads(layer, x, dy)
    gw, gb, sq = _run_per_example(layer, x, dy, "f32")
    assert_close(gw, ref_w, F32_TOL, "dgamma")
    assert_close(gb, ref_b, F32_TOL, "dbeta")
    assert np.allclose(sq, ref_n2, rtol=F32_TOL, atol=0)


GRAM_CASES = [
    ("512->2048 7x7", conv(512, 2048, 1, 1, 7), 5),
    ("2048->512 7x7", conv(2048, 512, 1, 1, 7), 3),
    ("384->640 7x7 ragged channel blocks", conv(384, 640, 1, 1, 7), 4),
    ("512->1024 8x8 (S = 64)", conv(512, 1024, 1, 1, 8), 2),
    ("512->512 4x4", conv(512, 512, 1, 1, 4), 33),
    ("3x3 512->512 7x7", conv(512, 512, 3, 1, 7), 3),
    ("3x3 stride 2 14->7 ragged", conv(320, 264, 3, 2, 14), 4),
    ("3x3 6x8 rectangular", Layer("conv", 128, 256, 6, 8, 3, 3, 1, 1, False), 3),
]


@pytest.mark.parametrize("name,layer,n", GRAM_CASES, ids=[c[0] for c in GRAM_CASES])
def test_gram_route_norms(name, layer, n):
    """Norm-only calls of 1x1 convs on small maps go through two Gram matrices: same norms as the oracle's
    sum of squares and as the materialising call's."""
    d = dp.make_desc(layer, n, "bf16")
    assert dp.dp_kernel_variant(d, dp.DP_WS_PER_EXAMPLE_GRAD) == "conv_gram_norm<bf16>"
    count = dp.dp_norm_partial_count(d, False)
    x, dy = _inputs(layer, n, 401, "bf16", x_abs=True)
    _, _, sq_mat = _run_per_example(layer, x, dy, "bf16")
    _, _, sq = _run_per_example(layer, x, dy, "bf16", materialise=False)
    assert np.allclose(sq, sq_mat, rtol=2e-5, atol=0), (sq, sq_mat)
    for i in range(n):                              # every example against the oracle's sum of squares
        w, _ = oracle.example_grad(layer, x[i], dy[i])
        assert math.isclose(sq[i], oracle.sqnorm(w), rel_tol=1e-4), (i, sq[i], oracle.sqnorm(w))
    # the partial-norm entry point leaves the same numbers at the start of the workspace
    ws = torch.empty(dp.dp_workspace_bytes(d), dtype=torch.uint8, device="cuda:0")
    dp.dp_per_example_grad_partials(d, dev(x, "bf16"), dev(dy, "bf16"), None, None, ws)
    torch.cuda.synchronize()
    parts = host(ws[: 4 * n * count].view(torch.float32)).reshape(n, count)
    assert np.allclose(parts.sum(axis=1), sq, rtol=1e-5)


def test_clip_accumulate_segments_matches_one_call_per_segment():
    """Several clipping groups in one launch: same bits as a dp_clip_accumulate call per segment, and the oracle's sum."""
    rng = np.random.default_rng(31)
    n, sizes, groups = 7, [36, 4, 1028, 260, 8, 4096], [0, 0, 1, 2, 2, 1]
    begins = np.concatenate([[0], np.cumsum(sizes)[:-1]])
    p = int(sum(sizes))
    stride = p + 8
    g = rng.standard_normal((n, stride)).astype(np.float32)
    n2 = (rng.uniform(0.3, 2.5, (3, n)) ** 2).astype(np.float32)
    n2[1, 2] = 0.0
    clips = [0.7, 0.7, 1.3, 2.0, 2.0, 1.3]
    acc0 = rng.standard_normal(p).astype(np.float32)
    acc = dev(acc0)
    table = dp.SegmentTable(begins, groups, clips)
    dp.dp_clip_accumulate_segments(dev(g), dev(n2), 3, table, n, p, acc, g_stride=stride)
    ref_dev = dev(acc0)
    gd, n2d = dev(g), dev(n2)
    ref = acc0.astype(np.float64)
    for b, sz, grp, c in zip(begins, sizes, groups, clips):
        dp.dp_clip_accumulate(gd[:, b:].data_ptr(), n2d[grp], c, n, sz, ref_dev[b:].data_ptr(), g_stride=stride)
        f = np.array([oracle.clip_factor(float(v), c) for v in n2[grp]])
        ref[b: b + sz] += (f[:, None] * g[:, b: b + sz].astype(np.float64)).sum(axis=0)
    torch.cuda.synchronize()
    assert torch.equal(acc, ref_dev)
    assert_close(host(acc) - acc0, ref - acc0, F32_TOL, "segments increment")


@pytest.mark.parametrize("with_update", [False, True])
def test_flat_finalize_gives_the_bits_of_one_call_per_tensor(with_update):
    """dp_add_noise_finalize_flat: several tensors of a flat vector in one launch (ragged sizes, padding between
    tensors, a tensor longer than several workgroups), same counters and bits as a call per tensor; the step
    taken from a device word; the oracle's values."""
    rng = np.random.default_rng(77)
    sizes = [10, 4096, 1, 5003, 1024, 300_001, 7]
    ids = [0, 1, 9, 4, 5, 106, 107]
    begins, pos = [], 0
    for sz in sizes:
        begins.append(pos)
        pos += (sz + 3) // 4 * 4 + (8 if sz == 1 else 0)        # tensors start on 4-float boundaries, one extra gap
    p_total = pos
    acc0 = (rng.standard_normal(p_total) * 0.3).astype(np.float32)
    acc = dev(acc0)
    table = dp.TensorTable(begins, sizes, ids)
    sigma, clip, batch, seed, step = 0.9, 1.3, 48, 0x1234_5678_9ABC, 6
    step_dev = torch.tensor([step], dtype=torch.int64, device="cuda:0")
    out = torch.full((p_total,), -5.0, device="cuda:0")
    want = torch.full((p_total,), -5.0, device="cuda:0")
    if not with_update:
        dp.dp_add_noise_finalize_flat(acc, out, table, sigma, clip, batch, seed, step=999, step_dev=step_dev)
        for b, sz, tid in zip(begins, sizes, ids):
            dp.dp_add_noise_finalize(acc[b:].data_ptr(), want[b:].data_ptr(), sz, sigma, clip, batch, seed, step, tid)
        torch.cuda.synchronize()
        assert torch.equal(out, want)                              # padding untouched (-5), tensors bit-equal
        for b, sz, tid in zip(begins, sizes, ids):
            ref = oracle.noise_finalize(acc0[b: b + sz], sigma, clip, batch, seed, step, tid)
            assert_close(host(out[b: b + sz]), ref, F32_TOL, f"tensor {tid}")
        # the host-side step argument is used when no device word is given
        out2 = torch.full((p_total,), -5.0, device="cuda:0")
        dp.dp_add_noise_finalize_flat(acc, out2, table, sigma, clip, batch, seed, step=step)
        assert torch.equal(out2, want)
        # sigma = 0: plain division, no draws
        dp.dp_add_noise_finalize_flat(acc, out2, table, 0.0, clip, batch, seed, step=step)
        for b, sz in zip(begins, sizes):
            assert torch.equal(out2[b: b + sz], acc[b: b + sz] * (1.0 / batch))
    else:
        th0 = rng.standard_normal(p_total).astype(np.float32)
        v0 = (rng.standard_normal(p_total) * 0.1).astype(np.float32)
        th, v = dev(th0), dev(v0)
        thw, vw = dev(th0), dev(v0)
        dp.dp_add_noise_finalize_flat(acc, out, table, sigma, clip, batch, seed, step_dev=step_dev, theta=th, velocity=v,
                                      lr=0.05, momentum=0.9)
        for b, sz, tid in zip(begins, sizes, ids):
            dp.dp_add_noise_finalize_update(acc[b:].data_ptr(), thw[b:].data_ptr(), vw[b:].data_ptr(), want[b:].data_ptr(),
                                            sz, sigma, clip, batch, seed, step, tid, 0.05, 0.9)
        torch.cuda.synchronize()
        assert torch.equal(out, want) and torch.equal(th, thw) and torch.equal(v, vw)
        # without a gradient output and without momentum
        th2 = dev(th0)
        dp.dp_add_noise_finalize_flat(acc, None, table, sigma, clip, batch, seed, step=step, theta=th2, lr=0.05)
        g = host(want)
        for b, sz in zip(begins, sizes):
            assert_close(host(th2[b: b + sz]), th0[b: b + sz].astype(np.float64) - 0.05 * g[b: b + sz], F32_TOL, "theta")


NHWC_CASES = [
    ("1x1 aligned rows bf16", conv(64, 160, 1, 1, 12), "bf16"),
    ("3x3 raw rows bf16", conv(64, 64, 3, 1, 14), "bf16"),
    ("3x3 stride 2 bias fp32", conv(12, 20, 3, 2, 11, bias=True), "f32"),
    ("7x7 stem bf16", conv(3, 32, 7, 2, 30), "bf16"),
    ("groupnorm fp32", gn_affine(32, 10, 8), "f32"),
    ("dense bf16 (no channel axis to move)", dense(100, 36), "bf16"),
]


@pytest.mark.parametrize("name,layer,dtype", NHWC_CASES, ids=[c[0] for c in NHWC_CASES])
def test_channels_last_inputs_give_the_bits_of_channels_first(name, layer, dtype):
    """DP_NHWC: x [n, h, w, cin], dy [n, oh, ow, cout].  Per-example gradients, norms, the recomputing clipped sum and
    unit sums: the oracle's values, and the very bits of the channels-first call on the same numbers."""
    n = 4
    tol = F32_TOL if dtype == "f32" else BF16_TOL
    x, dy = _inputs(layer, n, 8800, dtype)
    last = (lambda a: np.ascontiguousarray(np.moveaxis(a, 1, -1))) if layer.kind != "dense" else (lambda a: a)
    ref_w, ref_b, ref_n2 = _oracle_grads(layer, x, dy)
    results = []
    for layout, xs, dys in ((dp.DP_NCHW, x, dy), (dp.DP_NHWC, last(x), last(dy))):
        d = dp.make_desc(layer, n, dtype, layout=layout)
        xd, dyd = dev(xs, dtype), dev(dys, dtype)
        ws = torch.empty(max(16, dp.dp_workspace_bytes(d), dp.dp_workspace_bytes(d, dp.DP_WS_RECOMPUTE),
                             dp.dp_unit_workspace_bytes(d, 2)), dtype=torch.uint8, device="cuda:0")
        gw = torch.full((n, layer.pw), 7.0, device="cuda:0")
        gb = torch.full((n, max(layer.pb, 1)), 7.0, device="cuda:0")
        sq = torch.full((n,), -1.0, device="cuda:0")
        dp.dp_per_example_grad(d, xd, dyd, gw, gb if layer.pb else None, sq, ws)
        sq_only = torch.full((n,), -1.0, device="cuda:0")
        dp.dp_per_example_grad(d, xd, dyd, None, None, sq_only, ws)
        acc_w = torch.zeros(layer.pw, device="cuda:0")
        acc_b = torch.zeros(max(layer.pb, 1), device="cuda:0")
        n2 = dev((np.array([0.5, 1.0, 1.5, 2.0]) ** 2 * float(ref_n2.mean())).astype(np.float32))
        dp.dp_clip_accumulate_recompute(d, xd, dyd, n2, math.sqrt(float(ref_n2.mean())), acc_w, acc_b if layer.pb else None, ws)
        uw = torch.zeros((n // 2, layer.pw), device="cuda:0")
        ub = torch.zeros((n // 2, max(layer.pb, 1)), device="cuda:0")
        usq = torch.zeros(n // 2, device="cuda:0")
        dp.dp_unit_grad(d, 2, xd, dyd, uw, ub if layer.pb else None, usq, ws)
        torch.cuda.synchronize()
        results.append((gw, gb, sq, sq_only, acc_w, acc_b, uw, ub, usq))
    for a, b in zip(*results):
        assert torch.equal(a, b)
    gw, gb, sq = results[1][:3]
    assert np.allclose(host(sq), ref_n2, rtol=tol, atol=0)
    for i in range(n):
        assert_close(host(gw[i]), ref_w[i], tol, f"{name} dW[{i}]")
        if layer.pb:
            assert_close(host(gb[i, :layer.pb]), ref_b[i], tol, f"{name} db[{i}]")


BATCH_LAYERS = [
    conv(64, 256, 1, 1, 28), conv(256, 64, 1, 1, 28), conv(64, 64, 1, 1, 28),          # 1x1, aligned rows
    conv(160, 136, 1, 1, 28), conv(130, 200, 1, 1, 14),                               # 128x128 tiles when the launch is shared
    conv(96, 72, 1, 1, 7, bias=True), conv(33, 65, 1, 1, 15),                          # odd S: gather loader, bias
    conv(64, 64, 3, 1, 28), conv(64, 128, 3, 1, 28), conv(128, 64, 3, 1, 14),          # raw-row 3x3 kernels
    conv(48, 80, 1, 2, 14), conv(128, 128, 3, 2, 28), conv(3, 64, 7, 2, 64),           # strided, long K
    conv(256, 512, 1, 1, 7), conv(512, 256, 3, 1, 7),                                  # Gram-route norms
    conv(64, 64, 3, 1, 56), conv(64, 64, 3, 2, 56),                                    # raw-row 3x3: 56-wide rows, stride 2 onto 28-wide rows
    dense(100, 36), gn_affine(32, 10, 8),
]


@pytest.mark.parametrize("n", [1, 5])
@pytest.mark.parametrize("materialise", [False, True])
def test_batch_call_matches_the_single_layer_calls_and_the_oracle(n, materialise):
    """dp_per_example_grad_batch: many layers in one call (layers of one kernel share a launch, tiling chosen for a
    shared launch): every layer's gradients and norms against the single-layer call and against the oracle."""
    dtype = "bf16"
    ins = [_inputs(l, n, 900 + k, dtype) for k, l in enumerate(BATCH_LAYERS)]
    descs = [dp.make_desc(l, n, dtype) for l in BATCH_LAYERS]
    xs = [dev(x, dtype) for x, _ in ins]
    dys = [dev(dy, dtype) for _, dy in ins]
    wss = [torch.empty(max(16, dp.dp_workspace_bytes(d)), dtype=torch.uint8, device="cuda:0") for d in descs]
    sq = torch.full((len(descs), n), -1.0, device="cuda:0")
    gws = [torch.full((n, l.pw), 7.0, device="cuda:0") for l in BATCH_LAYERS]
    gbs = [torch.full((n, max(l.pb, 1)), 7.0, device="cuda:0") for l in BATCH_LAYERS]
    batch = dp.LayerBatch(descs, [w.data_ptr() for w in wss], [w.numel() for w in wss])
    for rep in range(2):                                   # twice: same bits on every call
        dp.dp_per_example_grad_batch(batch, batch.ptrs([t.data_ptr() for t in xs]), batch.ptrs([t.data_ptr() for t in dys]),
                                     batch.ptrs([t.data_ptr() for t in gws]) if materialise else None,
                                     batch.ptrs([t.data_ptr() if l.pb else None for t, l in zip(gbs, BATCH_LAYERS)]) if materialise else None,
                                     batch.ptrs([sq[k].data_ptr() for k in range(len(descs))]))
        torch.cuda.synchronize()
        if rep == 0:
            first = (sq.clone(), [g.clone() for g in gws])
        else:
            assert torch.equal(sq, first[0]) and all(torch.equal(a, b) for a, b in zip(gws, first[1]))
    for k, l in enumerate(BATCH_LAYERS):
        x, dy = ins[k]
        ref_w, ref_b, ref_n2 = _oracle_grads(l, x, dy)
        assert np.allclose(host(sq[k]), ref_n2, rtol=BF16_TOL, atol=0), (k, l, host(sq[k]), ref_n2)
        gw1, gb1, sq1 = _run_per_example(l, x, dy, dtype, materialise=materialise)
        assert np.allclose(host(sq[k]), sq1, rtol=3e-5, atol=0), (k, l)
        if materialise:
            for i in range(n):
                assert_close(host(gws[k][i]), ref_w[i], BF16_TOL, f"layer {k} dW[{i}]")
                if l.pb:
                    assert_close(host(gbs[k][i, :l.pb]), ref_b[i], BF16_TOL, f"layer {k} db[{i}]")
            assert_close(host(gws[k]), gw1, 2e-5, f"layer {k} against the single-layer call")


@pytest.mark.parametrize("materialise", [False, True])
def test_batch_call_of_whole_row_blocks_with_a_ragged_last_group_of_examples(materialise):
    """Two 1x1 layers on 14x14 maps in one batch call: the kernel that moves whole rows in blocks of 32, several examples
    per workgroup (66 examples: the last group is short), gradients and norms against the oracle."""
    dtype, n = "bf16", 66
    layers = [conv(256, 512, 1, 1, 14), conv(512, 256, 1, 1, 14)]
    descs = [dp.make_desc(l, n, dtype) for l in layers]
    for d in descs:
        assert dp.dp_kernel_variant(d, dp.DP_WS_PER_EXAMPLE_GRAD | dp.DP_VARIANT_SHARED) == "conv_contract<bf16,256x256rows,per_example>"
    ins = [_inputs(l, n, 1300 + k, dtype) for k, l in enumerate(layers)]
    xs = [dev(x, dtype) for x, _ in ins]
    dys = [dev(dy, dtype) for _, dy in ins]
    wss = [torch.empty(max(16, dp.dp_workspace_bytes(d)), dtype=torch.uint8, device="cuda:0") for d in descs]
    sq = torch.full((2, n), -1.0, device="cuda:0")
    gws = [torch.full((n, l.pw), 7.0, device="cuda:0") for l in layers]
    batch = dp.LayerBatch(descs, [w.data_ptr() for w in wss], [w.numel() for w in wss])
    dp.dp_per_example_grad_batch(batch, batch.ptrs([t.data_ptr() for t in xs]), batch.ptrs([t.data_ptr() for t in dys]),
                                 batch.ptrs([t.data_ptr() for t in gws]) if materialise else None, None,
                                 batch.ptrs([sq[k].data_ptr() for k in range(2)]))
    torch.cuda.synchronize()
    for k, l in enumerate(layers):
        ref_w, _, ref_n2 = _oracle_grads(l, *ins[k])
        assert np.allclose(host(sq[k]), ref_n2, rtol=BF16_TOL, atol=0), (k, host(sq[k]), ref_n2)
        if materialise:
            for i in (0, 3, 4, 63, 64, 65):
                assert_close(host(gws[k][i]), ref_w[i], BF16_TOL, f"layer {k} dW[{i}]")
        else:
            assert torch.all(gws[k] == 7.0)


def test_gram_route_norms_in_a_batch_call_with_several_blocks_per_workgroup():
    """Norm-only batch call on 7x7 maps with a dozen examples: the Gram-route kernel takes four blocks of 256 channels
    per workgroup there (one block when a layer is alone); the norms against the oracle and against the single calls."""
    dtype, n = "bf16", 12
    layers = [conv(2048, 512, 1, 1, 7), conv(512, 1280, 1, 1, 7), conv(512, 256, 3, 1, 7), conv(256, 256, 3, 2, 14)]
    descs = [dp.make_desc(l, n, dtype) for l in layers]
    for d in descs:
        assert dp.dp_kernel_variant(d, dp.DP_WS_PER_EXAMPLE_GRAD) == "conv_gram_norm<bf16>"
    ins = [_inputs(l, n, 1500 + k, dtype) for k, l in enumerate(layers)]
    xs = [dev(x, dtype) for x, _ in ins]
    dys = [dev(dy, dtype) for _, dy in ins]
    wss = [torch.empty(max(16, dp.dp_workspace_bytes(d)), dtype=torch.uint8, device="cuda:0") for d in descs]
    sq = torch.full((len(layers), n), -1.0, device="cuda:0")
    batch = dp.LayerBatch(descs, [w.data_ptr() for w in wss], [w.numel() for w in wss])
    dp.dp_per_example_grad_batch(batch, batch.ptrs([t.data_ptr() for t in xs]), batch.ptrs([t.data_ptr() for t in dys]), None, None,
                                 batch.ptrs([sq[k].data_ptr() for k in range(len(layers))]))
    torch.cuda.synchronize()
    for k, l in enumerate(layers):
        ref_n2 = _oracle_grads(l, *ins[k])[2]
        assert np.allclose(host(sq[k]), ref_n2, rtol=BF16_TOL, atol=0), (k, host(sq[k]), ref_n2)
        sq1 = _run_per_example(l, *ins[k], dtype, materialise=False)[2]
        assert np.allclose(host(sq[k]), sq1, rtol=3e-5, atol=0), k


@pytest.mark.parametrize("n", [1, 5])
def test_batch_calls_with_the_reduction_left_to_one_launch(n):
    """Two batch calls that leave their partial sums in the workspaces (sqnorm NULL), then ONE
    dp_layer_norms_from_partials over the layers of both: the norms of the oracle, and the bits of the batch call
    that reduces by itself."""
    dtype = "bf16"
    ins = [_inputs(l, n, 900 + k, dtype) for k, l in enumerate(BATCH_LAYERS)]
    descs = [dp.make_desc(l, n, dtype) for l in BATCH_LAYERS]
    xs = [dev(x, dtype) for x, _ in ins]
    dys = [dev(dy, dtype) for _, dy in ins]
    wss = [torch.empty(max(16, dp.dp_workspace_bytes(d)), dtype=torch.uint8, device="cuda:0") for d in descs]
    L = len(descs)
    halves = [list(range(0, L, 2)), list(range(1, L, 2))]
    sq = torch.full((L, n), -1.0, device="cuda:0")
    sq_own = torch.full((L, n), -2.0, device="cuda:0")
    import ctypes
    counts = (ctypes.c_int32 * L)()
    for ids in halves:
        batch = dp.LayerBatch([descs[i] for i in ids], [wss[i].data_ptr() for i in ids], [wss[i].numel() for i in ids])
        args = (batch, batch.ptrs([xs[i].data_ptr() for i in ids]), batch.ptrs([dys[i].data_ptr() for i in ids]), None, None)
        dp.dp_per_example_grad_batch(*args, batch.ptrs([sq_own[i].data_ptr() for i in ids]))
        torch.cuda.synchronize()
        dp.dp_per_example_grad_batch(*args, None)
        for k, i in enumerate(ids):
            counts[i] = batch.partial_counts[k]
            assert counts[i] >= 1
    dp.dp_layer_norms_from_partials((ctypes.c_void_p * L)(*[w.data_ptr() for w in wss]), counts,
                                    (ctypes.c_void_p * L)(*[sq[i].data_ptr() for i in range(L)]), L, n)
    torch.cuda.synchronize()
    assert torch.equal(sq, sq_own)
    for k, l in enumerate(BATCH_LAYERS):
        ref_n2 = _oracle_grads(l, *ins[k])[2]
        assert np.allclose(host(sq[k]), ref_n2, rtol=BF16_TOL, atol=0), (k, l, host(sq[k]), ref_n2)


@pytest.mark.parametrize("n", [1, 6])
def test_recompute_batch_call_matches_the_single_layer_calls_and_the_oracle(n):
    dtype = "bf16"
    rng = np.random.default_rng(61)
    layers = BATCH_LAYERS
    ins = [_inputs(l, n, 950 + k, dtype) for k, l in enumerate(layers)]
    descs = [dp.make_desc(l, n, dtype) for l in layers]
    xs = [dev(x, dtype) for x, _ in ins]
    dys = [dev(dy, dtype) for _, dy in ins]
    wss = [torch.empty(max(16, dp.dp_workspace_bytes(d, dp.DP_WS_RECOMPUTE)), dtype=torch.uint8, device="cuda:0") for d in descs]
    n2 = (rng.uniform(0.4, 2.0, (len(layers), n)) ** 2).astype(np.float32)          # both clip branches
    n2d = dev(n2)
    clips = [1.0 + 0.1 * (k % 3) for k in range(len(layers))]
    acc0 = [rng.standard_normal(l.pw).astype(np.float32) * 1e-3 for l in layers]
    accb0 = [rng.standard_normal(max(l.pb, 1)).astype(np.float32) * 1e-3 for l in layers]
    acc_w = [dev(a) for a in acc0]
    acc_b = [dev(a) for a in accb0]
    batch = dp.LayerBatch(descs, [w.data_ptr() for w in wss], [w.numel() for w in wss])
    dp.dp_clip_accumulate_recompute_batch(batch, batch.ptrs([t.data_ptr() for t in xs]), batch.ptrs([t.data_ptr() for t in dys]),
                                          batch.ptrs([n2d[k].data_ptr() for k in range(len(layers))]), batch.floats(clips),
                                          batch.ptrs([t.data_ptr() for t in acc_w]),
                                          batch.ptrs([t.data_ptr() if l.pb else None for t, l in zip(acc_b, layers)]))
    torch.cuda.synchronize()
    for k, l in enumerate(layers):
        x, dy = ins[k]
        f = np.array([oracle.clip_factor(float(v), clips[k]) for v in n2[k]])
        ref_w, ref_b, _ = _oracle_grads(l, x, dy)
        want = (f[:, None] * ref_w).sum(axis=0)
        assert_close(host(acc_w[k]) - acc0[k], want, BF16_TOL, f"layer {k} {l} weighted sum")
        if l.pb:
            assert_close(host(acc_b[k])[:l.pb] - accb0[k][:l.pb], (f[:, None] * ref_b).sum(axis=0), BF16_TOL, f"layer {k} bias")
        # the single-layer call
        one = dev(acc0[k])
        oneb = dev(accb0[k])
        dp.dp_clip_accumulate_recompute(descs[k], xs[k], dys[k], n2d[k], clips[k], one, oneb if l.pb else None, wss[k])
        torch.cuda.synchronize()
        assert_close(host(acc_w[k]) - acc0[k], host(one) - acc0[k], 1e-4, f"layer {k} against the single-layer call")
