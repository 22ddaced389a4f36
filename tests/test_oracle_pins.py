"""Pins for the CPU oracle: it is checked against things other than itself.

The paper prints no worked numerical example, so the pins are hand-computed
cases (tests/golden/hand_conv_cases.txt), closed forms, invariants, special
cases that reduce to an independent library routine (numpy einsum, torch CPU
float64 ops) and a brute-force scatter formulation written here in Python.
None of these tests needs a GPU.
"""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_conv_cases.txt")


def _rng(seed):
    return np.random.default_rng(seed)


def _rand(rng, *shape):
    return rng.standard_normal(shape).astype(np.float32)


# --------------------------------------------------------------------------- P1
def _golden_cases():
    cases, cur = [], {}
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if not line:
            continue
        key, val = line.split(":", 1)
        if key == "case" and cur:
            cases.append(cur)
            cur = {}
        cur[key] = val.strip()
    cases.append(cur)
    return cases


@pytest.mark.parametrize("case", _golden_cases(), ids=lambda c: c["case"])
def test_hand_computed_cases(case):
    dims = dict(kv.split("=") for kv in case["shape"].split())
    d = {k: int(v) for k, v in dims.items()}
    x = np.array(case["in"].split(), dtype=np.float32).reshape(d["N"], d["Cin"], d["H"], d["W"])
    w = np.array(case["w"].split(), dtype=np.float32).reshape(d["Cout"], d["Cin"], d["K"], d["K"])
    b = np.array(case["b"].split(), dtype=np.float32)
    want = np.array(case["out"].split(), dtype=np.float32)
    got = oracle.conv2d(x, w, b, stride=d["S"], pad=d["P"], relu=bool(d["relu"]))
    assert got.size == want.size
    np.testing.assert_array_equal(got.ravel(), want)


# --------------------------------------------------------------------------- P2
def test_1x1_conv_is_matrix_product():
    rng = _rng(10)
    x = _rand(rng, 2, 7, 5, 6)
    w = _rand(rng, 4, 7, 1, 1)
    b = _rand(rng, 4)
    got = oracle.conv2d(x, w, b)
    want = np.einsum("mc,nchw->nmhw", w[:, :, 0, 0].astype(np.float64), x.astype(np.float64))
    want += b.astype(np.float64)[None, :, None, None]
    np.testing.assert_allclose(got, want.astype(np.float32), rtol=0, atol=0)


# --------------------------------------------------------------------------- P3
@pytest.mark.parametrize("pad", [0, 1, 2, 3])
def test_delta_kernel_is_identity(pad):
    rng = _rng(11)
    C, K = 3, 2 * pad + 1
    x = _rand(rng, 2, C, 6, 7)
    w = np.zeros((C, C, K, K), np.float32)
    for c in range(C):
        w[c, c, pad, pad] = 1.0
    np.testing.assert_array_equal(oracle.conv2d(x, w, None, 1, pad), x)


# --------------------------------------------------------------------------- P4
def test_translation_equivariance_stride1():
    rng = _rng(12)
    K, P = 3, 1
    core = _rand(rng, 1, 2, 5, 5)
    w = _rand(rng, 3, 2, K, K)
    big = np.zeros((1, 2, 16, 16), np.float32)
    big[:, :, 3:8, 4:9] = core
    shifted = np.zeros_like(big)
    dy, dx = 4, 3
    shifted[:, :, 3 + dy:8 + dy, 4 + dx:9 + dx] = core
    a = oracle.conv2d(big, w, None, 1, P)
    bb = oracle.conv2d(shifted, w, None, 1, P)
    np.testing.assert_array_equal(a[:, :, 1:11, 1:12], bb[:, :, 1 + dy:11 + dy, 1 + dx:12 + dx])
    assert np.abs(a).sum() > 0


# --------------------------------------------------------------------------- P5
@pytest.mark.parametrize("K,P,S", [(3, 1, 1), (7, 2, 2), (1, 0, 1), (5, 2, 1), (3, 0, 2)])
def test_all_ones_counts_in_bounds_taps(K, P, S):
    Cin, H, W = 4, 9, 11
    x = np.ones((1, Cin, H, W), np.float32)
    w = np.ones((2, Cin, K, K), np.float32)
    got = oracle.conv2d(x, w, None, S, P)
    Ho, Wo = (H + 2 * P - K) // S + 1, (W + 2 * P - K) // S + 1
    assert got.shape == (1, 2, Ho, Wo)
    for oh in range(Ho):
        rows = sum(0 <= oh * S + i - P < H for i in range(K))
        for ow in range(Wo):
            cols = sum(0 <= ow * S + j - P < W for j in range(K))
            assert got[0, 0, oh, ow] == Cin * rows * cols
            assert got[0, 1, oh, ow] == Cin * rows * cols
    if (K, P, S) == (3, 1, 1):
        assert got[0, 0, 0, 0] == 4 * Cin and got[0, 0, 0, 1] == 6 * Cin and got[0, 0, 1, 1] == 9 * Cin


# --------------------------------------------------------------------------- P6
@pytest.mark.parametrize("S", [2, 3])
def test_stride_is_subsampling_of_stride1(S):
    rng = _rng(13)
    x = _rand(rng, 2, 3, 12, 13)
    w = _rand(rng, 4, 3, 3, 3)
    b = _rand(rng, 4)
    dense = oracle.conv2d(x, w, b, 1, 1)
    strided = oracle.conv2d(x, w, b, S, 1)
    np.testing.assert_array_equal(strided, dense[:, :, ::S, ::S][:, :, :strided.shape[2], :strided.shape[3]])


# --------------------------------------------------------------------------- P7
def test_linearity_bias_once_and_relu_after_bias():
    rng = _rng(14)
    x = _rand(rng, 1, 3, 8, 8)
    y = _rand(rng, 1, 3, 8, 8)
    w = _rand(rng, 5, 3, 3, 3)
    b = _rand(rng, 5)
    a = np.float32(0.5)  # exact in binary, so a*x is exact
    lhs = oracle.conv2d(a * x + y, w, b, 1, 1)
    rhs = (a * oracle.conv2d(x, w, None, 1, 1).astype(np.float64)
           + oracle.conv2d(y, w, None, 1, 1).astype(np.float64) + b[None, :, None, None])
    np.testing.assert_allclose(lhs, rhs, rtol=0, atol=2e-6)
    relu_on = oracle.conv2d(x, w, b, 1, 1, relu=True)
    relu_off = oracle.conv2d(x, w, b, 1, 1, relu=False)
    np.testing.assert_array_equal(relu_on, np.maximum(relu_off, 0))
    assert (relu_off < 0).any()
    # a zero input leaves exactly the bias (added once, not once per input layer)
    zero = oracle.conv2d(np.zeros_like(x), w, b, 1, 1)
    np.testing.assert_array_equal(zero, np.broadcast_to(b[None, :, None, None], zero.shape))


# ------------------------------------------------------------- library pin: conv
@pytest.mark.parametrize("N,Cin,H,W,Cout,K,S,P", [
    (2, 3, 23, 19, 5, 7, 2, 2), (1, 5, 9, 9, 4, 3, 1, 1), (2, 6, 7, 8, 3, 1, 1, 0),
    (1, 2, 10, 12, 3, 5, 3, 2), (1, 4, 6, 6, 2, 3, 2, 0), (1, 1, 4, 4, 1, 4, 1, 0),
    (1, 2, 5, 7, 2, 3, 1, 2)])
def test_conv_matches_torch_float64(N, Cin, H, W, Cout, K, S, P):
    rng = _rng(15)
    x, w, b = _rand(rng, N, Cin, H, W), _rand(rng, Cout, Cin, K, K), _rand(rng, Cout)
    got = oracle.conv2d(x, w, b, S, P, relu=False)
    want = F.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                    torch.from_numpy(b).double(), stride=S, padding=P).numpy()
    assert got.shape == want.shape
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-6 * (1 + np.abs(want).max()))
    # a non-square, multi-layer case distinguishes every axis: check a transposed
    # kernel or swapped H/W would not pass
    if K > 1 and H != W:
        wrong = F.conv2d(torch.from_numpy(x).double(),
                         torch.from_numpy(w).double().transpose(2, 3).contiguous(),
                         torch.from_numpy(b).double(), stride=S, padding=P).numpy()
        assert np.abs(got - wrong).max() > 1e-3


# --------------------------------------------------------------------------- P11
def _scatter_conv(x, w, b, S, P):
    """Scatter form: walk the *input* pixels and add each one's contribution into
    every output it touches.  Deliberately a different loop structure."""
    N, Cin, H, W = x.shape
    Cout, _, K, _ = w.shape
    Ho, Wo = (H + 2 * P - K) // S + 1, (W + 2 * P - K) // S + 1
    out = np.zeros((N, Cout, Ho, Wo), np.float64)
    if b is not None:
        out += b.astype(np.float64)[None, :, None, None]
    for n in range(N):
        for c in range(Cin):
            for ih in range(H):
                for iw in range(W):
                    v = float(x[n, c, ih, iw])
                    for i in range(K):
                        t = ih + P - i
                        if t < 0 or t % S:
                            continue
                        oh = t // S
                        if oh >= Ho:
                            continue
                        for j in range(K):
                            u = iw + P - j
                            if u < 0 or u % S:
                                continue
                            ow = u // S
                            if ow >= Wo:
                                continue
                            out[n, :, oh, ow] += v * w[:, c, i, j].astype(np.float64)
    return out


@pytest.mark.parametrize("K,S,P", [(3, 1, 1), (3, 2, 0), (2, 2, 1), (1, 1, 0), (4, 3, 2)])
def test_scatter_formulation_agrees(K, S, P):
    rng = _rng(16)
    x, w, b = _rand(rng, 1, 2, 6, 7), _rand(rng, 3, 2, K, K), _rand(rng, 3)
    got = oracle.conv2d(x, w, b, S, P)
    want = _scatter_conv(x, w, b, S, P)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-6)
    # the double accumulator agrees to 1e-12 relative before the final rounding
    assert np.abs(got.astype(np.float64) - want).max() <= 6e-8 * (1 + np.abs(want).max())


# --------------------------------------------------------------------------- P8
@pytest.mark.parametrize("K,S,H,W", [(3, 2, 111, 111), (3, 2, 10, 12), (2, 2, 8, 8), (3, 1, 5, 6), (2, 3, 9, 7)])
def test_maxpool_of_ramp_closed_form(K, S, H, W):
    ramp = (np.arange(H)[:, None] * W + np.arange(W)[None, :]).astype(np.float32)
    x = np.stack([ramp, -ramp])[None]          # layer 1 decreasing: max is the window's first tap
    got = oracle.maxpool(x, K, S)
    Ho, Wo = (H - K) // S + 1, (W - K) // S + 1
    assert got.shape == (1, 2, Ho, Wo)
    oh, ow = np.arange(Ho)[:, None], np.arange(Wo)[None, :]
    np.testing.assert_array_equal(got[0, 0], (oh * S + K - 1) * W + ow * S + K - 1)
    np.testing.assert_array_equal(got[0, 1], -((oh * S) * W + ow * S))


def test_maxpool_matches_torch_and_handles_negatives():
    rng = _rng(17)
    x = _rand(rng, 2, 3, 13, 15) - 5.0          # all negative: a zero-initialised max would fail
    want = F.max_pool2d(torch.from_numpy(x), 3, 2).numpy()
    np.testing.assert_array_equal(oracle.maxpool(x, 3, 2), want)


def test_avgpool_closed_forms():
    H, W = 13, 13
    const = np.full((2, 3, H, W), 2.5, np.float32)
    np.testing.assert_array_equal(oracle.avgpool_global(const), np.full((2, 3), 2.5, np.float32))
    ramp = np.arange(H * W, dtype=np.float32).reshape(1, 1, H, W)
    assert oracle.avgpool_global(ramp)[0, 0] == np.float32((H * W - 1) / 2)
    rng = _rng(18)
    x = _rand(rng, 2, 4, 5, 7)
    np.testing.assert_allclose(oracle.avgpool_global(x), x.astype(np.float64).mean(axis=(2, 3)), atol=1e-7)


def test_softmax_properties():
    rng = _rng(19)
    x = _rand(rng, 4, 1000) * 3
    y = oracle.softmax(x)
    assert np.abs(y.astype(np.float64).sum(1) - 1).max() <= 1e-6
    np.testing.assert_allclose(y, torch.softmax(torch.from_numpy(x).double(), 1).numpy(), atol=1e-9)
    np.testing.assert_allclose(oracle.softmax(np.zeros((2, 10), np.float32)), 0.1, atol=1e-8)
    np.testing.assert_allclose(oracle.softmax(x + np.float32(8.0)), y, atol=1e-6)   # shift invariance
    big = np.array([[1e4, -1e4, 0, 1e4]], np.float32)
    yb = oracle.softmax(big)
    assert np.isfinite(yb).all()
    np.testing.assert_allclose(yb, [[0.5, 0, 0, 0.5]], atol=1e-12)
    assert (np.argmax(x, 1) == np.argmax(y, 1)).all()


# --------------------------------------------------------------------------- P9
def test_fire_is_composition_and_concat_order():
    rng = _rng(20)
    x = _rand(rng, 2, 6, 7, 9)
    w_sq, b_sq = _rand(rng, 4, 6, 1, 1), _rand(rng, 4)
    w_e1, b_e1 = _rand(rng, 5, 4, 1, 1), _rand(rng, 5)
    w_e3, b_e3 = _rand(rng, 3, 4, 3, 3), _rand(rng, 3)
    out = oracle.fire(x, w_sq, b_sq, w_e1, b_e1, w_e3, b_e3)
    assert out.shape == (2, 8, 7, 9)
    s = oracle.conv2d(x, w_sq, b_sq, 1, 0, relu=True)
    np.testing.assert_array_equal(out[:, :5], oracle.conv2d(s, w_e1, b_e1, 1, 0, relu=True))
    np.testing.assert_array_equal(out[:, 5:], oracle.conv2d(s, w_e3, b_e3, 1, 1, relu=True))
    # independent library version in float64
    xt = torch.from_numpy(x).double()
    st = F.relu(F.conv2d(xt, torch.from_numpy(w_sq).double(), torch.from_numpy(b_sq).double()))
    e1 = F.relu(F.conv2d(st, torch.from_numpy(w_e1).double(), torch.from_numpy(b_e1).double()))
    e3 = F.relu(F.conv2d(st, torch.from_numpy(w_e3).double(), torch.from_numpy(b_e3).double(), padding=1))
    np.testing.assert_allclose(out, torch.cat([e1, e3], 1).numpy(), atol=2e-5)


def test_fire_padding_is_zero_not_relu_of_squeeze_bias():
    # Squeeze weights zero and squeeze bias +2: the squeeze map is the constant 2
    # inside the image.  The 3x3 expand must see 0 outside the image, so with
    # all-ones 3x3 weights a corner sums 4 taps, an edge 6, the interior 9.
    Cin, Csq, H, W = 3, 2, 5, 6
    x = np.ones((1, Cin, H, W), np.float32)
    w_sq, b_sq = np.zeros((Csq, Cin, 1, 1), np.float32), np.full(Csq, 2.0, np.float32)
    w_e1, b_e1 = np.ones((1, Csq, 1, 1), np.float32), np.zeros(1, np.float32)
    w_e3, b_e3 = np.ones((1, Csq, 3, 3), np.float32), np.zeros(1, np.float32)
    out = oracle.fire(x, w_sq, b_sq, w_e1, b_e1, w_e3, b_e3)
    assert (out[0, 0] == 2.0 * Csq).all()
    e3 = out[0, 1]
    assert e3[0, 0] == 4 * 2 * Csq and e3[0, 2] == 6 * 2 * Csq and e3[2, 3] == 9 * 2 * Csq
    assert e3[H - 1, W - 1] == 4 * 2 * Csq and e3[H - 1, 2] == 6 * 2 * Csq


# --------------------------------------------------------------------------- P10
def test_shape_chain_mac_and_parameter_counts():
    layers = synth.conv_layers()
    assert len(layers) == 26
    macs = params = 0
    for name, cin, cout, k, s, p, h in layers:
        ho = (h + 2 * p - k) // s + 1
        macs += cout * ho * ho * cin * k * k
        params += cout * cin * k * k + cout
    assert macs == 832_667_936
    assert params == 1_248_424
    h = (224 + 2 * 2 - 7) // 2 + 1
    chain = [h]
    for _ in range(3):
        h = (h - 3) // 2 + 1
        chain.append(h)
    assert chain == [111, 55, 27, 13]


def _torch_squeezenet(x, params):
    t = [torch.from_numpy(p).double() for p in params]
    a = F.relu(F.conv2d(torch.from_numpy(x).double(), t[0], t[1], stride=2, padding=2))
    taps = {"conv1": a}
    a = F.max_pool2d(a, 3, 2)
    taps["pool1"] = a
    p = 2
    for f in range(2, 10):
        s = F.relu(F.conv2d(a, t[p], t[p + 1]))
        a = torch.cat([F.relu(F.conv2d(s, t[p + 2], t[p + 3])),
                       F.relu(F.conv2d(s, t[p + 4], t[p + 5], padding=1))], 1)
        p += 6
        taps[f"fire{f}"] = a
        if f in (4, 8):
            a = F.max_pool2d(a, 3, 2)
            taps[f"pool{f}"] = a
    a = F.relu(F.conv2d(a, t[50], t[51]))
    taps["conv10"] = a
    m = a.mean(dim=(2, 3))
    taps["means"] = m
    taps["probs"] = torch.softmax(m, 1)
    return taps


def test_squeezenet_wiring_against_torch_float64():
    cfg = synth.config_squeezenet(seed=2, n=1)
    probs, taps = oracle.squeezenet(cfg["x"], cfg["params"], want_taps=True)
    want = _torch_squeezenet(cfg["x"], cfg["params"])
    assert set(taps) == set(want)
    for name in oracle.TAP_NAMES:
        w = want[name].numpy()
        assert taps[name].shape == w.shape, name
        # the oracle rounds to float between layers, the float64 chain does not
        err = np.abs(taps[name] - w).max()
        assert err <= 2e-5 * (1 + np.abs(w).max()), (name, err)
    np.testing.assert_array_equal(probs, taps["probs"])
    assert abs(float(probs.astype(np.float64).sum()) - 1) < 1e-6
    assert taps["conv1"].shape == (1, 96, 111, 111) and taps["fire9"].shape == (1, 512, 13, 13)


def test_conv1_variant_227_no_pad_has_same_output_shape():
    cfg = synth.config_conv1(seed=1, n=1, size=227)
    out = oracle.conv2d(cfg["x"], cfg["w"], cfg["b"], 2, cfg["pad"], relu=True)
    assert out.shape == (1, 96, 111, 111)
    assert oracle.maxpool(out, 3, 2).shape == (1, 96, 55, 55)


# --------------------------------------------------------------------------- P12
def test_paper_index_maps_are_bijections():
    """Equations for (w, h, m) from the thread index x, row-major and in the
    four-layer-stacked order (sections "Parallel Computation of Output Elements"
    and "Zero-overhead Vectorization")."""
    Wo, Ho, M = 5, 3, 8
    n = Wo * Ho * M
    seen = set()
    for x in range(n):
        w, h, m = x % Wo, (x // Wo) % Ho, x // (Wo * Ho)
        assert (m * Ho + h) * Wo + w == x
        seen.add((m, h, w))
    assert len(seen) == n
    seen = set()
    for x in range(n):
        w, h = (x // 4) % Wo, (x // (4 * Wo)) % Ho
        m = (x % 4) + (x // (4 * Wo * Ho)) * 4
        assert 0 <= m < M
        # position of (m,h,w) in the stacked layout [M/4][H][W][4]
        assert (((m // 4) * Ho + h) * Wo + w) * 4 + m % 4 == x
        seen.add((m, h, w))
    assert len(seen) == n


def test_granularity_rule_matches_table_of_optimal_g():
    """Thread granularity g must leave numOutputLayers / g divisible by four
    (section "Optimizing Thread Granularity"); every g the paper's table of
    optimal granularities prints obeys it for that layer's output count."""
    table = {96: (6, 12), 64: (4, 8, 16), 128: (4, 8, 32), 192: (6, 12, 16)}
    for cout, gs in table.items():
        for g in gs:
            assert cout % g == 0 and (cout // g) % 4 == 0


def test_oracle_rejects_bad_arguments():
    x = np.zeros((1, 1, 2, 2), np.float32)
    w = np.zeros((1, 1, 3, 3), np.float32)
    with pytest.raises(ValueError):
        oracle.conv2d(x, w, None, 1, 0)      # window larger than the image
    with pytest.raises(ValueError):
        oracle.conv2d(x, np.zeros((1, 2, 1, 1), np.float32))
