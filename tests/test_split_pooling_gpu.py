"""The kernels of the split max pooling one at a time (section "Pooling and Softmax": 3x3 window, stride 2): a layer
that pools the columns of its result as it writes it, and the 1x1 layer behind that pools the rows as it reads.

The format of the map between the two is stated in include/sq_tuning.h; `positions` below restates it.  A maximum
picks one of its arguments, so every comparison of pooled values is for equal bits; the convolution behind is
compared with the oracle (fp32 tolerance) and, bit for bit, with sq_maxpool_conv2d_forward in the same tiling.
"""
import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu

FP32_TOL = 1e-4


@pytest.fixture(scope="module")
def sq():
    import paper_1611_07151_amd as m
    return m


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def positions(geometry, n, row, Wp):
    """Column-pooled map: position of pooled column x in `row` of image n, and whether a seam slot follows it."""
    shift, slots_row, slots_image, _ = geometry
    q0 = n * slots_image + (row // 2) * slots_row
    x = np.arange(Wp)
    return x + ((q0 + x) >> shift) - (q0 >> shift), ((q0 + x) & ((1 << shift) - 1)) == (1 << shift) - 1


def check_column_pooled(hp, full, geometry, what):
    """hp: the map a kernel wrote (before ReLU); full: the layer's plain result (after ReLU)."""
    hp = np.maximum(hp.cpu().numpy(), 0)      # NaN (never written) stays NaN and fails the comparison where it is used
    full = full.cpu().numpy()
    N, C, Ho, Wo = full.shape
    Wp = (Wo - 3) // 2 + 1
    x = np.arange(Wp)
    for n in range(N):
        for r in range(Ho):
            pos, seam = positions(geometry, n, r, Wp)
            row, got = full[n][:, r, :], hp[n][:, r, :]                     # [layers][columns]
            two = np.maximum(row[:, 2 * x], row[:, 2 * x + 1])
            want = np.where(seam, two, np.maximum(two, row[:, 2 * x + 2]))
            assert np.array_equal(got[:, pos], want), f"{what}: image {n} row {r}"
            assert np.array_equal(got[:, pos[seam] + 1], row[:, 2 * x[seam] + 2]), f"{what}: seams of image {n} row {r}"


def column_pooled_on_host(full, geometry, rng):
    """The map a producer would write for `full` (values before ReLU: negative entries stay), NaN where nothing is written."""
    N, C, Ho, Wo = full.shape
    Wp = (Wo - 3) // 2 + 1
    hp = np.full((N, C, Ho, geometry[3]), np.nan, np.float32)
    x = np.arange(Wp)
    for n in range(N):
        for r in range(Ho):
            pos, seam = positions(geometry, n, r, Wp)
            row, dst = full[n][:, r, :], hp[n][:, r, :]                     # views: [layers][columns]
            two = np.maximum(row[:, 2 * x], row[:, 2 * x + 1])
            dst[:, pos] = np.where(seam, two, np.maximum(two, row[:, 2 * x + 2]))
            dst[:, pos[seam] + 1] = row[:, 2 * x[seam] + 2]
    return hp


# conv1-type layer: tiles of 2 x 16 pixels; widths that end inside a tile, in its first column, on its last
@pytest.mark.parametrize("n,h,w,pad", [(2, 224, 224, 2), (1, 37, 75, 2), (3, 21, 41, 0), (1, 224, 134, 3), (2, 19, 11, 1)])
def test_conv1_writes_column_pooled_map(sq, n, h, w, pad):
    rng = np.random.default_rng(31 + h)
    x = synth.uniform01(rng, (n, 3, h, w))
    wt = synth.he_normal(rng, 96, 3, 7)
    b = synth.bias(rng, 96)
    # the plain map from a conv1-type kernel too (they all add up in the same order; other tilings of the layer do not)
    names = [sq.sq_conv_variant_name(v) for v in range(sq.sq_conv_variant_count())]
    full = sq.sq_conv2d_forward_ex(dev(x), dev(wt), dev(b), 2, pad, True, algo=sq.SQ_ALGO_VARIANT0 + names.index("k7s2c3_waves8"))
    hp, g = sq.sq_tune_conv2d_forward_poolcols(dev(x), dev(wt), dev(b), pad)
    assert g[0] == 3 and g[1] == 8 * ((full.shape[3] + 15) // 16)
    check_column_pooled(hp, full, g, "conv1")


# fire layer through the expand pair of autonomous wavefronts: tile groups of 16 tiles run across rows and images
@pytest.mark.parametrize("n,cin,h,w,csq,ce", [(3, 128, 55, 55, 32, 128), (4, 64, 27, 27, 64, 256), (3, 32, 9, 14, 16, 32),
                                              (5, 16, 7, 3, 16, 32), (3, 48, 12, 33, 32, 64), (7, 16, 5, 8, 16, 32)])
def test_fire_writes_column_pooled_map(sq, n, cin, h, w, csq, ce):
    rng = np.random.default_rng(41 + h * w)
    x = synth.uniform01(rng, (n, cin, h, w))
    p = [synth.he_normal(rng, csq, cin, 1), synth.bias(rng, csq), synth.he_normal(rng, ce, csq, 1), synth.bias(rng, ce),
         synth.he_normal(rng, ce, csq, 3), synth.bias(rng, ce)]
    d = [dev(a) for a in p]
    sq.lib.sq_tune_expand_pair(3)       # the plain map from the same form of the expand pair: same order of additions
    try:
        full = sq.sq_fire_forward(dev(x), *d)
    finally:
        sq.lib.sq_tune_expand_pair(-1)
    hp, g = sq.sq_tune_fire_forward_poolcols(dev(x), *d)
    assert g[:3] == [4, (w + 1) // 2, ((w + 1) // 2) * ((h + 1) // 2)]
    check_column_pooled(hp, full, g, "fire")
    # and the squeeze behind it, from the map the kernel wrote: the bits of pooling inside that squeeze
    wn = synth.he_normal(rng, 32, 2 * ce, 1)
    bn = synth.bias(rng, 32)
    if h >= 3:
        for v in range(sq.sq_conv_variant_count()):
            try:
                inside = sq.sq_maxpool_conv2d_forward(full, dev(wn), dev(bn), algo=sq.SQ_ALGO_VARIANT0 + v)
            except sq.SqError:
                continue
            split = sq.sq_tune_poolrows_conv2d_forward(hp, w, dev(wn), dev(bn), g, algo=sq.SQ_ALGO_VARIANT0 + v)
            assert torch.equal(split, inside), sq.sq_conv_variant_name(v)


def test_fire_without_a_column_pooling_kernel_is_refused(sq):
    rng = np.random.default_rng(5)
    x = dev(synth.uniform01(rng, (2, 32, 9, 9)))     # two images: the expand pair starts at three
    d = [dev(a) for a in (synth.he_normal(rng, 16, 32, 1), synth.bias(rng, 16), synth.he_normal(rng, 32, 16, 1), synth.bias(rng, 32),
                          synth.he_normal(rng, 32, 16, 3), synth.bias(rng, 32))]
    with pytest.raises(sq.SqError) as e:
        sq.sq_tune_fire_forward_poolcols(x, *d)
    assert e.value.status == -3


# the reader alone, on maps laid out on the host: group sizes and row lengths no producer here has, negative values
# (the producer's ReLU is the reader's), NaN in every slot a producer would not write
@pytest.mark.parametrize("n,cin,h,w,cout,shift,slack", [(2, 32, 13, 13, 16, 2, 0), (3, 16, 9, 40, 48, 3, 3), (1, 64, 27, 27, 64, 4, 0),
                                                        (2, 16, 3, 3, 16, 1, 1), (5, 16, 8, 7, 32, 4, 0), (1, 96, 111, 111, 16, 3, 1)])
def test_reader_of_column_pooled_maps(sq, n, cin, h, w, cout, shift, slack):
    rng = np.random.default_rng(51 + w)
    full = synth.normal01(rng, (n, cin, h, w))                      # before ReLU
    wt = synth.he_normal(rng, cout, cin, 1)
    b = synth.bias(rng, cout)
    Wp = (w - 3) // 2 + 1
    slots_row = (w + 1) // 2 + slack
    g = [shift, slots_row, slots_row * ((h + 1) // 2) + slack, Wp + (Wp >> shift) + 2 + slack]
    hp = column_pooled_on_host(full, g, rng)
    got = sq.sq_tune_poolrows_conv2d_forward(dev(hp), w, dev(wt), dev(b), g)
    relu = np.maximum(full, 0)
    ref = oracle.conv2d(oracle.maxpool(relu, 3, 2), wt, b, 1, 0, True)
    np.testing.assert_allclose(got.cpu().numpy(), ref, rtol=0, atol=FP32_TOL * max(1.0, float(np.abs(ref).max())))
    inside = sq.sq_maxpool_conv2d_forward(dev(relu), dev(wt), dev(b))
    assert torch.equal(got, inside)


def test_reader_rejects_geometry_that_cannot_hold_the_map(sq):
    x = torch.zeros((1, 16, 9, 8), device="cuda")
    w = torch.zeros((16, 16, 1, 1), device="cuda")
    for g in ([4, 3, 30, 8], [4, 6, 10, 8], [4, 6, 30, 5], [0, 6, 30, 8]):     # row slots, image slots, row stride, shift
        with pytest.raises(sq.SqError) as e:
            sq.sq_tune_poolrows_conv2d_forward(x[..., :g[3]].contiguous(), 11, w, None, g)
        assert e.value.status == -2
