"""Parity of the reduced-precision path (bfloat16 feature maps and kernels, fp32 sums,
blocked layout [N][C/8][H][W][8]) with the CPU oracle, through the C boundary.

Two bars per layer:
  * the stated one -- the oracle is fed the UNROUNDED fp32 tensors and the result must
    be within 2e-2 * (1 + |ref|);
  * a tight one -- the oracle is fed the same bfloat16-rounded inputs and kernels the
    GPU sees, so only the summation order and the final rounding of the result to
    bfloat16 (relative 2^-9) differ: 4e-3 * (1 + |ref|).  A wrong tap, kernel or layer
    fails this one by orders of magnitude.
The layout conversion on the host side of these tests is plain torch indexing on the
CPU; it shares nothing with the library.
"""
import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu

BF16_TOL = 2e-2
TIGHT_TOL = 4e-3


@pytest.fixture(scope="module")
def sq():
    import paper_1611_07151_amd as m
    return m


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t if dtype is None else t.to(dtype)


def rounded(a):
    """fp32 array rounded to bfloat16 (nearest even) and widened again."""
    return torch.from_numpy(np.ascontiguousarray(a)).to(torch.bfloat16).float().numpy()


def to_blocked(x):
    """NCHW fp32 array -> CPU bfloat16 tensor [N][ceil(C/8)][H][W][8], zero filled past C."""
    n, c, h, w = x.shape
    cb = (c + 7) // 8
    full = np.zeros((n, cb * 8, h, w), dtype=np.float32)
    full[:, :c] = x
    t = torch.from_numpy(full).reshape(n, cb, 8, h, w).permute(0, 1, 3, 4, 2).contiguous()
    return t.to(torch.bfloat16)


def from_blocked(m, c):
    """bfloat16 tensor [N][CB][H][W][8] (any device) -> NCHW fp32 array with c layers."""
    m = m.detach().float().cpu()
    n, cb, h, w, _ = m.shape
    return m.permute(0, 1, 4, 2, 3).reshape(n, cb * 8, h, w)[:, :c].contiguous().numpy()


def assert_close(got, ref, tol, what=""):
    got = np.asarray(got)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.isfinite(got).all(), what
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    bound = tol * (1 + np.abs(ref.astype(np.float64)))
    bad = err > bound
    assert not bad.any(), (f"{what}: {int(bad.sum())} of {bad.size} outside tolerance; worst "
                           f"{float((err / bound).max()):.3g}x at {np.unravel_index(np.argmax(err / bound), err.shape)}")


# ------------------------------------------------------------------------------ layout
@pytest.mark.parametrize("shape", [(2, 16, 5, 7), (1, 3, 9, 4), (3, 20, 13, 13), (1, 1000, 2, 3), (2, 32, 55, 55), (3, 20, 27, 29),
                                   (1, 8, 23, 22), (2, 9, 1, 1)])
def test_pack_and_unpack_match_the_layout_definition(sq, shape):
    rng = np.random.default_rng(11)
    x = synth.normal01(rng, shape)
    want = to_blocked(x)
    got = sq.sq_blocked_pack(dev(x))
    assert got.shape == want.shape
    assert torch.equal(got.cpu().view(torch.int16), want.view(torch.int16))          # same rounding, same places
    got_b = sq.sq_blocked_pack(dev(x, torch.bfloat16))                                # bfloat16 NCHW in (16-byte pieces through LDS)
    assert torch.equal(got_b.cpu().view(torch.int16), want.view(torch.int16))
    shifted = torch.empty(x.size + 1, device="cuda", dtype=torch.bfloat16)[1:].view(shape)   # two bytes off: element by element
    shifted.copy_(dev(x, torch.bfloat16))
    assert shifted.data_ptr() % 16 != 0
    assert torch.equal(sq.sq_blocked_pack(shifted).cpu().view(torch.int16), want.view(torch.int16))
    back = sq.sq_blocked_unpack(got, shape[1])
    assert np.array_equal(back.cpu().numpy(), rounded(x))


# ------------------------------------------------------------------------- convolution
BLOCKED_CASES = [
    # N, Cin, H,  W,  Cout, K
    (2, 96, 55, 55, 16, 1),      # squeeze: fewer layers than one MFMA block
    (2, 16, 55, 55, 64, 1),      # expand1x1: a single step
    (2, 16, 55, 55, 64, 3),      # expand3x3
    (2, 32, 55, 55, 128, 3),
    (3, 256, 27, 27, 48, 1),     # 48 layers: one and a half blocks
    (2, 48, 27, 27, 192, 3),
    (3, 64, 13, 13, 256, 3),     # tiles straddle images
    (2, 512, 13, 13, 64, 1),
    (2, 512, 13, 13, 1000, 1),   # conv10: 1000 = 31.25 blocks of 32
    (1, 16, 1, 1, 8, 1),         # one pixel
    (1, 16, 5, 7, 24, 3),        # nothing fills a tile
    (1, 32, 9, 11, 40, 5),       # 5x5
    (5, 16, 8, 8, 32, 3),        # 320 pixels: exactly five tiles
]


@pytest.mark.parametrize("case", BLOCKED_CASES, ids=lambda c: "x".join(map(str, c)))
@pytest.mark.parametrize("relu", [True, False])
def test_blocked_conv_matches_oracle(sq, case, relu):
    N, Cin, H, W, Cout, K = case
    P = (K - 1) // 2
    rng = np.random.default_rng(200 + Cin * K + Cout)
    x = synth.normal01(rng, (N, Cin, H, W))
    w, b = synth.conv_params(rng, Cout, Cin, K)
    ref = oracle.conv2d(x, w, b, 1, P, relu)                         # unrounded inputs: the stated bar
    ref_r = oracle.conv2d(rounded(x), rounded(w), b, 1, P, relu)     # what the GPU was given: the tight bar
    m = to_blocked(x).cuda()
    for wd in (dev(w), dev(w, torch.bfloat16)):
        wp = sq.sq_blocked_pack_kernels(wd)
        out = sq.sq_blocked_conv2d_forward(m, wp, dev(b), Cin, Cout, K, P, relu)
        got = from_blocked(out, Cout)
        assert_close(got, ref, BF16_TOL, "stated tolerance")
        assert_close(got, ref_r, TIGHT_TOL, "same rounded operands")
    out0 = sq.sq_blocked_conv2d_forward(m, wp, None, Cin, Cout, K, P, relu)
    assert_close(from_blocked(out0, Cout), oracle.conv2d(rounded(x), rounded(w), None, 1, P, relu), TIGHT_TOL, "no bias")


CONV7_CASES = [
    # N, H,   W,   Cout, P
    (1, 224, 224, 96, 2),       # conv1 at full size
    (1, 227, 227, 96, 0),       # the other reading of conv1 (227, no padding)
    (2, 37, 41, 96, 2),         # odd sizes, ragged tiles
    (3, 21, 19, 40, 3),         # fewer layers, wide padding
    (1, 7, 7, 8, 0),            # a single output pixel
]


@pytest.mark.parametrize("case", CONV7_CASES, ids=lambda c: "x".join(map(str, c)))
@pytest.mark.parametrize("relu", [True, False])
def test_blocked_conv7s2_matches_oracle(sq, case, relu):
    N, H, W, Cout, P = case
    rng = np.random.default_rng(300 + H + Cout)
    x = synth.uniform01(rng, (N, 3, H, W))
    w, b = synth.conv_params(rng, Cout, 3, 7)
    ref = oracle.conv2d(x, w, b, 2, P, relu)
    ref_r = oracle.conv2d(rounded(x), rounded(w), b, 2, P, relu)
    for xd in (dev(x), dev(x, torch.bfloat16)):
        for wd in (dev(w), dev(w, torch.bfloat16)):
            out = sq.sq_blocked_conv7s2_forward(xd, sq.sq_blocked_pack_kernels7(wd), dev(b), Cout, P, relu)
            got = from_blocked(out, Cout)
            assert_close(got, ref, BF16_TOL, "stated tolerance")
            assert_close(got, ref_r, TIGHT_TOL, "same rounded operands")
    out = torch.full((N, 13, ref.shape[2], ref.shape[3], 8), -7.0, device="cuda", dtype=torch.bfloat16)   # 104 layers
    sq.sq_blocked_conv7s2_forward(dev(x), sq.sq_blocked_pack_kernels7(dev(w)), None, Cout, P, relu, out=out, c_offset=8)
    full = from_blocked(out, 104)
    assert_close(full[:, 8:8 + Cout], oracle.conv2d(rounded(x), rounded(w), None, 2, P, relu), TIGHT_TOL, "offset, no bias")
    assert (full[:, :8] == -7.0).all() and (full[:, 8 + Cout:] == -7.0).all()


@pytest.mark.parametrize("k", [1, 3])
def test_blocked_conv_channel_offset_leaves_other_layers_untouched(sq, k):
    rng = np.random.default_rng(9)
    x = synth.normal01(rng, (2, 16, 27, 27))
    w, b = synth.conv_params(rng, 64, 16, k)
    ref_r = oracle.conv2d(rounded(x), rounded(w), b, 1, k // 2, True)
    out = torch.full((2, 12, 27, 27, 8), -7.0, device="cuda", dtype=torch.bfloat16)    # 96 layers
    sq.sq_blocked_conv2d_forward(to_blocked(x).cuda(), sq.sq_blocked_pack_kernels(dev(w)), dev(b), 16, 64, k, k // 2,
                                 True, out=out, c_offset=24)
    full = from_blocked(out, 96)
    assert_close(full[:, 24:88], ref_r, TIGHT_TOL, "written layers")
    assert (full[:, :24] == -7.0).all() and (full[:, 88:] == -7.0).all()


@pytest.mark.parametrize("shape", [(2, 96, 55, 16, 64), (2, 128, 55, 32, 128), (3, 256, 27, 48, 192), (2, 384, 27, 64, 256),
                                   (5, 512, 13, 64, 256), (1, 32, 6, 16, 24)])
def test_blocked_fire_matches_oracle(sq, shape):
    """Squeeze, then both expands in one launch -- and the whole layer in one launch -- against the oracle's fire
    layer; also with a large positive squeeze bias, so that a padded tap that saw relu(bias) instead of zero
    would show."""
    N, Cin, H, Csq, Ce = shape
    rng = np.random.default_rng(400 + Cin + Ce)
    x = synth.normal01(rng, (N, Cin, H, H))
    (w_sq, b_sq), (w_e1, b_e1), (w_e3, b_e3) = (synth.conv_params(rng, Csq, Cin, 1), synth.conv_params(rng, Ce, Csq, 1),
                                                synth.conv_params(rng, Ce, Csq, 3))
    packed = [sq.sq_blocked_pack_kernels(dev(w)) for w in (w_sq, w_e1, w_e3)]
    for bias_shift in (0.0, 3.0):
        bs = (b_sq + bias_shift).astype(np.float32)
        ref = oracle.fire(x, w_sq, bs, w_e1, b_e1, w_e3, b_e3)
        ws = torch.empty(sq.sq_blocked_map_bytes(N, Csq, H, H), device="cuda", dtype=torch.uint8)

        def run():
            return sq.sq_blocked_fire_forward(to_blocked(x).cuda(), Cin, packed[0], dev(bs), packed[1], dev(b_e1), packed[2],
                                              dev(b_e3), Csq, Ce, Ce, workspace=ws)
        try:
            sq.lib.sq_tune_fire_one_launch(0)          # squeeze into the workspace, then both expands in one launch
            out = run()
            s_gpu = from_blocked(ws.view(torch.bfloat16).view(N, Csq // 8, H, H, 8), Csq)
            sq.lib.sq_tune_fire_one_launch(1)          # the whole layer in one launch, squeeze map in LDS
            sq.sq_profile_begin(8)
            out1 = run()
            stages = [r["name"] for r in sq.sq_profile_end()]
        finally:
            sq.lib.sq_tune_fire_one_launch(-1)
        assert len(stages) == 1 and stages[0].startswith("fire|fire1_bf16"), stages
        assert torch.equal(out.view(torch.int16), out1.view(torch.int16)), "one launch and two launches differ"
        got = from_blocked(out, 2 * Ce)
        # the stated tolerance is per convolution: the squeeze map (left in the workspace) against the oracle,
        # then the expands against the oracle applied to that squeeze map
        if bias_shift == 0.0:   # (a squeeze map with mean 3 is outside the value range the tolerance is stated for)
            assert_close(s_gpu, oracle.conv2d(x, w_sq, bs, 1, 0, True), BF16_TOL, "squeeze")
            ref_e = np.concatenate([oracle.conv2d(s_gpu, w_e1, b_e1, 1, 0, True), oracle.conv2d(s_gpu, w_e3, b_e3, 1, 1, True)],
                                   axis=1)
            assert_close(got, ref_e, BF16_TOL, "expands")
            assert_close(got, ref, 2 * BF16_TOL, "whole fire layer (two roundings)")
        # tight bar, convolution by convolution, each on exactly the operands the GPU had (the squeeze map is
        # taken from the GPU: where the two sides' sums straddle a rounding boundary it differs by one ulp)
        assert_close(s_gpu, oracle.conv2d(rounded(x), rounded(w_sq), bs, 1, 0, True), TIGHT_TOL, f"squeeze, shift {bias_shift}")
        ref_r = np.concatenate([oracle.conv2d(s_gpu, rounded(w_e1), b_e1, 1, 0, True),
                                oracle.conv2d(s_gpu, rounded(w_e3), b_e3, 1, 1, True)], axis=1)
        assert_close(got, ref_r, TIGHT_TOL, f"expands, shift {bias_shift}")


def test_blocked_conv_refuses_what_it_does_not_cover(sq):
    m = torch.zeros((1, 1, 4, 4, 8), device="cuda", dtype=torch.bfloat16)
    wp = torch.zeros(sq.sq_blocked_kernel_bytes(8, 8, 1), device="cuda", dtype=torch.uint8)
    with pytest.raises(sq.SqError) as e:
        sq.sq_blocked_conv2d_forward(m, wp, None, 8, 8, 1, 0)          # Cin not a multiple of 16
    assert e.value.status == -3
    m2 = torch.zeros((1, 2, 4, 4, 8), device="cuda", dtype=torch.bfloat16)
    wp2 = torch.zeros(sq.sq_blocked_kernel_bytes(8, 16, 3), device="cuda", dtype=torch.uint8)
    with pytest.raises(sq.SqError) as e:
        sq.sq_blocked_conv2d_forward(m2, wp2, None, 16, 8, 3, 0)       # 3x3 without its padding
    assert e.value.status == -3


# ----------------------------------------------------------------------------- pooling
@pytest.mark.parametrize("shape,k,s", [((2, 96, 111, 111), 3, 2), ((2, 256, 55, 55), 3, 2), ((3, 512, 27, 27), 3, 2),
                                       ((1, 12, 7, 9), 2, 1), ((1, 8, 3, 3), 3, 2)])
def test_blocked_maxpool_is_exact(sq, shape, k, s):
    rng = np.random.default_rng(5)
    x = synth.normal01(rng, shape)
    ref = oracle.maxpool(rounded(x), k, s)             # the maximum of bfloat16 values is one of them
    got = from_blocked(sq.sq_blocked_maxpool(to_blocked(x).cuda(), shape[1], k, s), shape[1])
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("case", [(2, 96, 111, 111, 16), (2, 256, 55, 55, 32), (3, 512, 27, 27, 64), (1, 16, 3, 3, 8),
                                  (2, 48, 10, 7, 40), (1, 16, 4, 9, 72)])
@pytest.mark.parametrize("relu", [True, False])
def test_pooling_inside_the_convolution_launch(sq, case, relu):
    """3x3 stride-2 max pooling fused into the 1x1 convolution that reads it: equal bit for bit to the two
    separate launches, and to the oracle (pooling exact, convolution at the tight bar); inputs of both signs."""
    N, Cin, Hin, Win, Cout = case
    rng = np.random.default_rng(500 + Cin + Cout)
    x = synth.normal01(rng, (N, Cin, Hin, Win))
    w, b = synth.conv_params(rng, Cout, Cin, 1)
    m = to_blocked(x).cuda()
    wp = sq.sq_blocked_pack_kernels(dev(w))
    fused = sq.sq_blocked_pool_conv2d_forward(m, wp, dev(b), Cin, Cout, relu)
    two = sq.sq_blocked_conv2d_forward(sq.sq_blocked_maxpool(m, Cin, 3, 2), wp, dev(b), Cin, Cout, 1, 0, relu)
    assert fused.shape == two.shape
    assert torch.equal(fused.view(torch.int16), two.view(torch.int16))
    pooled = oracle.maxpool(rounded(x), 3, 2)
    assert_close(from_blocked(fused, Cout), oracle.conv2d(pooled, rounded(w), b, 1, 0, relu), TIGHT_TOL, "pool + 1x1")
    assert_close(from_blocked(fused, Cout), oracle.conv2d(oracle.maxpool(x, 3, 2), w, b, 1, 0, relu), BF16_TOL, "stated tolerance")
    # into a wider map at an offset
    out = torch.full((N, Cout // 8 + 2, two.shape[2], two.shape[3], 8), -7.0, device="cuda", dtype=torch.bfloat16)
    sq.sq_blocked_pool_conv2d_forward(m, wp, dev(b), Cin, Cout, relu, out=out, c_offset=8)
    assert torch.equal(out[:, 1:-1].contiguous().view(torch.int16), two.view(torch.int16))
    assert (out[:, 0] == -7.0).all() and (out[:, -1] == -7.0).all()


# planes of 1, 20, 64, 128, 169 and 256 pixels take the forms with the loads issued up front, 272 and 900 the loop
@pytest.mark.parametrize("shape", [(2, 1000, 13, 13), (3, 20, 5, 4), (1, 8, 1, 1), (2, 24, 8, 8), (1, 16, 8, 16), (2, 9, 16, 16),
                                   (1, 40, 16, 17), (2, 12, 30, 30)])
def test_blocked_avgpool_matches_oracle(sq, shape):
    rng = np.random.default_rng(6)
    x = synth.normal01(rng, shape)
    ref = oracle.avgpool_global(rounded(x))
    got = sq.sq_blocked_avgpool_global(to_blocked(x).cuda(), shape[1]).cpu().numpy()
    assert_close(got, ref, 1e-5, "class means")


# ----------------------------------------------------------------------------- network
def _network(sq, cfg, x_dev):
    params = [dev(p) for p in cfg["params"]]
    packed = sq.sq_squeezenet_bf16_pack_params(params)
    probs, taps = sq.sq_squeezenet_forward_bf16(x_dev, params, packed, want_taps=True)
    plain = sq.sq_squeezenet_forward_bf16(x_dev, params, packed)     # without taps the pools run inside the squeeze launches
    assert torch.equal(plain, probs)
    return params, probs, taps


def test_network_stage_by_stage_on_the_previous_stage_output(sq):
    """Every stage of the reduced-precision network against the oracle applied to the GPU's own
    previous stage (so that each comparison sees one layer's error, not the accumulated one)."""
    cfg = synth.config_squeezenet(seed=2, n=1)
    P = cfg["params"]
    _, probs, taps = _network(sq, cfg, dev(cfg["x"]))
    t = {k: v.cpu().numpy() for k, v in taps.items()}
    assert_close(t["conv1"], oracle.conv2d(cfg["x"], P[0], P[1], 2, 2, True), BF16_TOL, "conv1")
    assert np.array_equal(t["pool1"], oracle.maxpool(t["conv1"], 3, 2))
    prev = "pool1"
    for f, name in enumerate(("fire2", "fire3", "fire4", "fire5", "fire6", "fire7", "fire8", "fire9")):
        p = 2 + 6 * f
        # the squeeze map is rounded to bfloat16 between the squeeze and the expands
        ref = oracle.fire(t[prev], *P[p:p + 6])
        assert_close(t[name], ref, BF16_TOL, name)
        prev = name
        if name in ("fire4", "fire8"):
            pool = "pool4" if name == "fire4" else "pool8"
            assert np.array_equal(t[pool], oracle.maxpool(t[name], 3, 2))
            prev = pool
    assert_close(t["conv10"], oracle.conv2d(t["fire9"], P[50], P[51], 1, 0, True), BF16_TOL, "conv10")
    assert_close(t["means"], oracle.avgpool_global(t["conv10"]), 1e-5, "class means")
    assert_close(t["probs"], oracle.softmax(t["means"]), 1e-5, "probabilities")
    assert abs(float(probs.sum()) - 1.0) < 1e-4


def test_network_end_to_end_against_the_fp32_oracle_and_fp32_gpu(sq):
    """Accumulated error of the reduced-precision network over all 26 convolutions, and agreement of
    the predicted class with the fp32 network (the paper's check of its relaxed-precision mode:
    same top-1 class, section "Imprecise computing")."""
    n = 8
    cfg = synth.config_squeezenet(seed=3, n=n)
    x = dev(cfg["x"])
    params, probs, taps = _network(sq, cfg, x)
    probs32, taps32 = sq.sq_squeezenet_forward(x, params, want_taps=True)
    # class means: the quantity the prediction is read from.  Error of the bfloat16 pipeline
    # relative to the spread of the means over the classes.
    m16, m32 = taps["means"].cpu().numpy().astype(np.float64), taps32["means"].cpu().numpy().astype(np.float64)
    spread = m32.std(axis=1, keepdims=True)
    rel = np.abs(m16 - m32) / spread
    # measured: maximum 3-6 % of the spread, rms 0.6 %; the bounds are twice the worst seen
    assert rel.max() < 0.12, rel.max()
    assert np.sqrt((rel ** 2).mean()) < 0.02
    ref_p, ref_t = oracle.squeezenet(cfg["x"][:1], cfg["params"], want_taps=True)
    assert_close(taps["means"][:1].cpu().numpy(), ref_t["means"], 5e-2, "class means of image 0 against the oracle")
    # top-1: wherever the fp32 winner leads the runner-up by more than the measured error, both agree
    top16, top32 = m16.argmax(axis=1), m32.argmax(axis=1)
    srt = np.sort(m32, axis=1)
    clear = (srt[:, -1] - srt[:, -2]) > 2 * np.abs(m16 - m32).max(axis=1)
    assert (top16[clear] == top32[clear]).all()
    assert (top16 == top32).mean() >= 0.5
    # a bfloat16 image gives the same network as its fp32 widening
    xb = x.to(torch.bfloat16)
    packed = sq.sq_squeezenet_bf16_pack_params(params)
    pb = sq.sq_squeezenet_forward_bf16(xb, params, packed)
    pf = sq.sq_squeezenet_forward_bf16(xb.float(), params, packed)
    assert_close(pb.cpu().numpy(), pf.cpu().numpy(), 2e-2, "bfloat16 image vs its fp32 widening")


@pytest.mark.parametrize("n", [3, 33])
def test_networks_at_odd_batch_sizes(sq, n):
    """Batches that fill no tile evenly (and sit on both sides of the fusion policies): the fp32 network
    against the oracle on the first and last image, the reduced-precision network against the fp32 one."""
    cfg = synth.config_squeezenet(seed=7, n=n)
    x = dev(cfg["x"])
    params = [dev(p) for p in cfg["params"]]
    probs32, taps32 = sq.sq_squeezenet_forward(x, params, want_taps=True)
    assert torch.equal(sq.sq_squeezenet_forward(x, params), probs32)
    for i in (0, n - 1):
        ref_p, ref_t = oracle.squeezenet(cfg["x"][i:i + 1], cfg["params"], want_taps=True)
        assert_close(taps32["means"][i:i + 1].cpu().numpy(), ref_t["means"], 1e-4, f"fp32 class means, image {i}")
        assert_close(probs32[i:i + 1].cpu().numpy(), ref_p, 1e-4, f"fp32 probabilities, image {i}")
    _, probs16, taps16 = _network(sq, cfg, x)
    m16, m32 = taps16["means"].cpu().numpy().astype(np.float64), taps32["means"].cpu().numpy().astype(np.float64)
    rel = np.abs(m16 - m32) / m32.std(axis=1, keepdims=True)
    assert rel.max() < 0.12 and np.sqrt((rel ** 2).mean()) < 0.02, (rel.max(), np.sqrt((rel ** 2).mean()))
    assert abs(float(probs16.sum()) - n) < 1e-3


def test_network_largest_batch(sq):
    """907 images, the largest batch the reduced-precision network call takes (conv1's bfloat16 output just under
    2^31 bytes): three distinct images repeated; every copy must give what its image gives at the front of the
    batch, and the front ones must agree with the fp32 oracle as at any batch.  One image more is refused."""
    assert sq.SQ_SQUEEZENET_BF16_MAX_BATCH == 907
    cfg = synth.config_squeezenet(seed=8, n=3)
    params = [dev(p) for p in cfg["params"]]
    packed = sq.sq_squeezenet_bf16_pack_params(params)
    x3 = dev(cfg["x"])
    x = torch.cat([x3.repeat(302, 1, 1, 1), x3[:1]])         # image i is cfg["x"][i % 3]
    assert x.shape[0] == 907
    probs = sq.sq_squeezenet_forward_bf16(x, params, packed).cpu().numpy()
    assert np.isfinite(probs).all() and np.abs(probs.sum(1) - 1).max() < 1e-4
    spread = np.abs(probs[:906].reshape(302, 3, 1000) - probs[:3][None]).max()
    assert spread <= 1e-6 and np.abs(probs[906] - probs[0]).max() <= 1e-6, spread
    ref = oracle.squeezenet(cfg["x"], cfg["params"])
    assert (probs[:3].argmax(1) == ref.argmax(1)).all()
    assert np.abs(probs[:3] - ref).max() < 0.25 * ref.max()
    with pytest.raises(sq.SqError) as e:
        sq.sq_squeezenet_forward_bf16(torch.empty((908, 3, 224, 224), device="cuda"), params, packed)
    assert e.value.status == -3
