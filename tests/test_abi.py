"""The C boundary on a machine without a GPU: the library loads, exports every
symbol the header declares, and rejects bad arguments before touching HIP."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "sq.h")
TUNING_HEADER = os.path.join(ROOT, "include", "sq_tuning.h")
LIB = os.path.join(ROOT, "paper_1611_07151_amd", "libsq.so")


@pytest.fixture(scope="module")
def lib():
    assert os.path.exists(LIB), "build the library first: python paper_1611_07151_amd/build.py"
    l = ctypes.CDLL(LIB)
    l.sq_strerror.restype = ctypes.c_char_p
    l.sq_fire_workspace_bytes.restype = ctypes.c_size_t
    l.sq_squeezenet_workspace_bytes.restype = ctypes.c_size_t
    l.sq_conv_variant_name.restype = ctypes.c_char_p
    return l


def _declared(header=HEADER):
    text = open(header).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sq_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared()
    assert {"sq_conv2d_forward", "sq_maxpool", "sq_fire_forward", "sq_squeezenet_forward", "sq_set_dtype",
            "sq_pack_weights", "sq_set_stream", "sq_strerror"} <= set(names)
    for n in names + _declared(TUNING_HEADER):
        assert hasattr(lib, n), n


def test_every_exported_symbol_is_declared_in_a_header():
    """No undeclared entry points: what the shared library exports under the sq_ prefix is exactly what the
    two headers under include/ declare."""
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", LIB], capture_output=True, text=True, check=True).stdout
    exported = {line.split()[-1] for line in out.splitlines() if line.split() and line.split()[-1].startswith("sq_")}
    declared = set(_declared()) | set(_declared(TUNING_HEADER))
    assert exported - declared == set(), sorted(exported - declared)
    assert declared - exported == set(), sorted(declared - exported)
    assert all(n.startswith("sq_tune_") for n in _declared(TUNING_HEADER))
    assert not any(n.startswith("sq_tune_") for n in _declared())


def test_strerror_covers_all_codes(lib):
    seen = {lib.sq_strerror(c) for c in range(0, -6, -1)}
    assert len(seen) == 6 and b"unknown status" not in seen
    assert lib.sq_strerror(-99) == b"unknown status"


FAKE = ctypes.c_void_p(0x1000)   # never dereferenced: validation fails first
NULL = ctypes.c_void_p(0)


def test_conv_rejects_bad_arguments_before_any_gpu_call(lib):
    f = lib.sq_conv2d_forward
    good = [1, 3, 8, 8, 4, 3, 1, 1, 1]
    assert f(NULL, FAKE, FAKE, FAKE, *good) == -1
    assert f(FAKE, NULL, FAKE, FAKE, *good) == -1
    assert f(FAKE, FAKE, FAKE, NULL, *good) == -1
    for idx, bad in [(0, 0), (1, -1), (2, 0), (3, 0), (4, 0), (5, 0), (6, 0), (7, -1)]:
        args = list(good)
        args[idx] = bad
        assert f(FAKE, FAKE, FAKE, FAKE, *args) == -2, (idx, bad)
    # window larger than the padded image
    assert f(FAKE, FAKE, FAKE, FAKE, 1, 3, 4, 4, 4, 7, 1, 1, 0) == -2
    g = lib.sq_conv2d_forward_ex
    assert g(FAKE, FAKE, FAKE, FAKE, *good, 4, 1, 0, 0) == -2      # c_offset + Cout > out_channels
    assert g(FAKE, FAKE, FAKE, FAKE, *good, 4, -1, 0, 0) == -2
    assert g(FAKE, FAKE, FAKE, FAKE, *good, 4, 0, 7, 0) == -3      # unknown dtype
    assert g(FAKE, FAKE, FAKE, FAKE, *good, 4, 0, 0, 2 + lib.sq_conv_variant_count()) == -3


def test_conv_workspace_entry_point_checks_its_scratch(lib):
    sz = ctypes.c_size_t
    lib.sq_conv2d_workspace_bytes.restype = sz
    need = lib.sq_conv2d_workspace_bytes(32, 128, 3, 1, 1)
    # transformed kernels: 16 values per (layer, input layer), in two orders: layers rounded up to 64, and layers as they are
    assert need == 16 * 128 * 32 * 4 + 16 * 128 * 32 * 4
    assert lib.sq_conv2d_workspace_bytes(32, 96, 3, 1, 1) == 16 * 128 * 32 * 4 + 16 * 96 * 32 * 4
    assert lib.sq_conv2d_workspace_bytes(32, 128, 3, 2, 1) == 0     # stride 2: no algorithm needs scratch
    assert lib.sq_conv2d_workspace_bytes(32, 128, 1, 1, 0) == 0
    # space-to-depth form of a strided layer: the copy [N][Cin*S*S][Ho+K'-1][Wo+K'-1] and the regrouped kernels, fp32
    lib.sq_conv2d_strided_workspace_bytes.restype = sz
    up = lambda v: (v + 255) // 256 * 256
    assert lib.sq_conv2d_strided_workspace_bytes(64, 3, 227, 227, 96, 11, 4, 0) == up(64 * 48 * 57 * 57 * 4) + up(96 * 48 * 9 * 4)
    assert lib.sq_conv2d_strided_workspace_bytes(2, 8, 21, 23, 24, 5, 2, 2) == up(2 * 32 * 13 * 14 * 4) + up(24 * 32 * 9 * 4)
    assert lib.sq_conv2d_strided_workspace_bytes(2, 16, 27, 27, 64, 3, 1, 1) == 0      # stride 1: nothing to regroup
    assert lib.sq_conv2d_strided_workspace_bytes(0, 3, 227, 227, 96, 11, 4, 0) == 0
    assert lib.sq_conv2d_strided_workspace_bytes(1, 3, 8, 8, 96, 11, 4, 0) == 0        # kernel larger than the image
    assert lib.sq_conv2d_workspace_bytes(30, 128, 3, 1, 1) == 0     # input layers not a multiple of 8
    assert lib.sq_conv2d_workspace_bytes(0, 128, 3, 1, 1) == 0
    h = lib.sq_conv2d_forward_ws
    good = [1, 32, 8, 8, 128, 3, 1, 1, 1, 128, 0, 0, 0]
    assert h(NULL, FAKE, FAKE, FAKE, *good, FAKE, sz(need)) == -1
    assert h(FAKE, FAKE, FAKE, FAKE, *good, ctypes.c_void_p(0x1010), sz(need)) == -4   # misaligned scratch
    bad = list(good); bad[9] = 100                                   # out_channels < Cout
    assert h(FAKE, FAKE, FAKE, FAKE, *bad, FAKE, sz(need)) == -2
    # the scratch-needing algorithm is refused when the scratch is missing or too small
    names = [lib.sq_conv_variant_name(i).decode() for i in range(lib.sq_conv_variant_count())]
    wino = 2 + [i for i, n in enumerate(names) if "f2x2" in n][0]
    sel = list(good); sel[12] = wino
    assert h(FAKE, FAKE, FAKE, FAKE, *sel, NULL, sz(0)) == -3
    assert h(FAKE, FAKE, FAKE, FAKE, *sel, FAKE, sz(need - 1)) == -3
    assert lib.sq_conv2d_forward_ex(FAKE, FAKE, FAKE, FAKE, *sel) == -3


def test_pool_and_softmax_reject_bad_arguments(lib):
    assert lib.sq_maxpool(NULL, FAKE, 1, 1, 8, 8, 3, 2) == -1
    assert lib.sq_maxpool(FAKE, FAKE, 1, 1, 2, 8, 3, 2) == -2
    assert lib.sq_maxpool(FAKE, FAKE, 1, 1, 8, 8, 3, 0) == -2
    f = lib.sq_maxpool_conv2d_forward     # in, w, b, out, N, Cin, H, W, Cout, relu, out_channels, c_offset, algo
    assert f(NULL, FAKE, FAKE, FAKE, 1, 16, 9, 9, 8, 1, 8, 0, 0) == -1
    assert f(FAKE, FAKE, NULL, FAKE, 1, 16, 2, 9, 8, 1, 8, 0, 0) == -2      # no 3x3 window fits
    assert f(FAKE, FAKE, NULL, FAKE, 1, 16, 9, 9, 8, 1, 8, 1, 0) == -2      # layers past the end of out
    assert f(FAKE, FAKE, NULL, FAKE, 1, 16, 9, 9, 8, 1, 8, 0, 1) == -3      # the one-thread-per-output kernel cannot
    assert f(FAKE, FAKE, NULL, FAKE, 1, 24, 9, 9, 8, 1, 8, 0, 0) == -3      # no tiling's input-layer chunk divides 24
    assert lib.sq_avgpool_global(FAKE, NULL, 1, 1, 8, 8) == -1
    assert lib.sq_avgpool_global(FAKE, FAKE, 1, 0, 8, 8) == -2
    assert lib.sq_softmax(NULL, FAKE, 1, 10) == -1
    assert lib.sq_softmax(FAKE, FAKE, 1, 0) == -2


def test_fire_and_network_check_workspace(lib):
    need = lib.sq_fire_workspace_bytes(2, 55, 55, 16, 64)
    assert need >= 2 * 16 * 55 * 55 * 4 and need % 256 == 0
    sz = ctypes.c_size_t
    fire = lambda ws, nbytes, n=2: lib.sq_fire_forward(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE,
                                                       n, 96, 55, 55, 16, 64, 64, ws, sz(nbytes))
    assert fire(NULL, need) == -4
    assert fire(FAKE, need - 1) == -4
    assert fire(ctypes.c_void_p(0x1004), need) == -4       # misaligned
    assert fire(FAKE, need, n=0) == -2
    assert lib.sq_fire_forward(NULL, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 2, 96, 55, 55, 16, 64, 64,
                               FAKE, sz(need)) == -1

    wsb = lib.sq_squeezenet_workspace_bytes(1)
    assert wsb >= (96 * 111 * 111 + 256 * 55 * 55) * 4
    assert lib.sq_squeezenet_workspace_bytes(0) == 0
    params = (ctypes.c_void_p * 52)(*[0x1000] * 52)
    net = lib.sq_squeezenet_forward
    assert net(FAKE, params, FAKE, 1, FAKE, sz(wsb - 1), None) == -4
    assert net(FAKE, params, FAKE, 0, FAKE, sz(wsb), None) == -2
    assert net(NULL, params, FAKE, 1, FAKE, sz(wsb), None) == -1
    # a batch whose conv1 output the 32-bit offsets of the kernels cannot address is refused up front
    assert (453 * 96 * 111 * 111) < 2 ** 29 <= (454 * 96 * 111 * 111)
    assert net(FAKE, params, FAKE, 454, FAKE, sz(lib.sq_squeezenet_workspace_bytes(454)), None) == -3
    assert net(FAKE, params, FAKE, 453, FAKE, sz(lib.sq_squeezenet_workspace_bytes(453) - 1), None) == -4
    params[17] = None
    assert net(FAKE, params, FAKE, 1, FAKE, sz(wsb), None) == -1


def test_variant_names(lib):
    n = lib.sq_conv_variant_count()
    assert n >= 0
    names = [lib.sq_conv_variant_name(i) for i in range(n)]
    assert all(names) and len(set(names)) == n
    assert lib.sq_conv_variant_name(n) == b""
    assert lib.sq_conv_variant_name(-1) == b""


def test_product_package_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_1611_07151_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath:
            continue
        for fn in files:
            if fn.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, fn)).read()
                assert "oracle" not in text.lower(), os.path.join(dirpath, fn)


def test_division_by_multiplication_is_exact(lib):
    """The kernels divide by runtime constants with a precomputed multiplier; the host
    twin of that routine must agree with integer division over the ranges in use."""
    f = lib.sq_tune_fastdiv_mismatches
    f.restype = ctypes.c_longlong
    f.argtypes = [ctypes.c_uint, ctypes.c_uint]
    for d in (1, 2, 3, 5, 7, 13, 15, 16, 27, 29, 55, 57, 111, 169, 227, 392, 729, 3025, 12321, 65536, 1000003):
        assert f(d, 3_000_000) == 0, d
    for d in (3, 111, 12321, 2_000_003):
        assert f(d, 40_000_000) == 0, d


def test_tuned_table_names_exist(lib):
    names = {lib.sq_conv_variant_name(i).decode() for i in range(lib.sq_conv_variant_count())}
    inc = os.path.join(ROOT, "paper_1611_07151_amd", "csrc", "tuned_table.inc")
    rows = re.findall(r'^\{[^"]*"([^"]+)", "([^"]+)"\},', open(inc).read(), flags=re.M)
    assert rows, "tuned table is empty"
    used = {n for row in rows for n in row}
    assert used <= names, used - names


def test_reduced_precision_entry_points_validate_before_any_gpu_call(lib):
    """Blocked bfloat16 maps: size queries, and every refusal that needs no GPU."""
    sz = ctypes.c_size_t
    for name in ("sq_blocked_map_bytes", "sq_blocked_kernel_bytes", "sq_blocked_kernel7_bytes",
                 "sq_squeezenet_bf16_packed_bytes", "sq_squeezenet_bf16_workspace_bytes"):
        getattr(lib, name).restype = sz
    # [N][ceil(C/8)][H][W][8] two-byte elements; kernels [Cout/32][K*K][Cin/16][64][8]
    assert lib.sq_blocked_map_bytes(2, 20, 5, 7) == 2 * 3 * 5 * 7 * 16
    assert lib.sq_blocked_map_bytes(0, 8, 5, 7) == 0
    assert lib.sq_blocked_kernel_bytes(48, 32, 3) == 2 * 9 * 2 * 64 * 16
    assert lib.sq_blocked_kernel7_bytes() == 3 * 11 * 64 * 16
    assert lib.sq_squeezenet_bf16_packed_bytes() % 256 == 0
    assert lib.sq_squeezenet_bf16_packed_bytes() >= 2 * 1_248_424 - 2 * (96 * 147) - 2 * 1200   # all kernels, two bytes each
    assert lib.sq_squeezenet_bf16_workspace_bytes(0) == 0
    assert 2 * lib.sq_squeezenet_bf16_workspace_bytes(3) < lib.sq_squeezenet_workspace_bytes(3) + 4096 * 3 + 4 * 3000 * 2

    conv = lib.sq_blocked_conv2d_forward
    good = [1, 16, 8, 8, 32, 3, 1, 1, 32, 0]      # N Cin H W Cout K P relu ldc c_offset
    assert conv(NULL, FAKE, FAKE, FAKE, *good) == -1
    assert conv(FAKE, NULL, FAKE, FAKE, *good) == -1
    assert conv(FAKE, FAKE, FAKE, NULL, *good) == -1
    for idx, bad in [(0, 0), (1, 0), (2, 0), (3, -1), (4, 0), (5, 0), (6, -1)]:
        args = list(good)
        args[idx] = bad
        assert conv(FAKE, FAKE, FAKE, FAKE, *args) == -2, (idx, bad)
    assert conv(FAKE, FAKE, FAKE, FAKE, 1, 16, 8, 8, 32, 3, 1, 1, 24, 0) == -2     # output map too narrow
    assert conv(FAKE, FAKE, FAKE, FAKE, 1, 16, 8, 8, 32, 3, 1, 1, 64, 40) == -2    # offset + Cout past the map
    for args in ([1, 8, 8, 8, 32, 3, 1, 1, 32, 0],      # Cin not a multiple of 16
                 [1, 16, 8, 8, 12, 3, 1, 1, 16, 0],     # Cout not a multiple of 8
                 [1, 16, 8, 8, 32, 3, 0, 1, 32, 0],     # 3x3 without its padding
                 [1, 16, 8, 8, 32, 2, 0, 1, 32, 0],     # even kernel size
                 [1, 16, 8, 8, 32, 7, 3, 1, 32, 0],     # kernel size beyond 5
                 [1, 16, 8, 8, 32, 3, 1, 1, 36, 4],     # offset not a multiple of 8
                 [1, 4096, 8, 8, 32, 3, 1, 1, 32, 0]):  # kernels of 32 layers beyond half the LDS
        assert conv(FAKE, FAKE, FAKE, FAKE, *args) == -3, args
    assert conv(ctypes.c_void_p(0x1004), FAKE, FAKE, FAKE, *good) == -3             # maps are 16-byte aligned

    c7 = lib.sq_blocked_conv7s2_forward
    assert c7(NULL, 0, FAKE, FAKE, FAKE, 1, 224, 224, 96, 2, 1, 96, 0) == -1
    assert c7(FAKE, 0, FAKE, FAKE, FAKE, 1, 4, 224, 96, 0, 1, 96, 0) == -2          # window larger than the image
    assert c7(FAKE, 0, FAKE, FAKE, FAKE, 1, 224, 224, 96, 2, 1, 64, 0) == -2         # map too narrow
    assert c7(FAKE, 5, FAKE, FAKE, FAKE, 1, 224, 224, 96, 2, 1, 96, 0) == -3         # unknown image type
    assert c7(FAKE, 0, FAKE, FAKE, FAKE, 1, 224, 224, 104, 2, 1, 104, 0) == -3       # more than 96 layers
    assert c7(FAKE, 0, FAKE, FAKE, FAKE, 1, 224, 224, 20, 2, 1, 24, 0) == -3         # not a multiple of 8

    assert lib.sq_blocked_pack(NULL, 0, FAKE, 1, 8, 4, 4) == -1
    assert lib.sq_blocked_pack(FAKE, 0, FAKE, 1, 0, 4, 4) == -2
    assert lib.sq_blocked_pack(FAKE, 7, FAKE, 1, 8, 4, 4) == -3
    assert lib.sq_blocked_unpack(FAKE, NULL, 1, 8, 4, 4) == -1
    assert lib.sq_blocked_pack_kernels(FAKE, 0, ctypes.c_void_p(0x1008), 8, 16, 1) == -3
    assert lib.sq_blocked_pack_kernels7(FAKE, 0, FAKE, 0) == -2
    assert lib.sq_blocked_maxpool(FAKE, FAKE, 1, 8, 2, 9, 3, 2) == -2
    assert lib.sq_blocked_avgpool_global(FAKE, NULL, 1, 8, 4, 4) == -1

    fire = lib.sq_blocked_fire_forward
    fire.argtypes = [ctypes.c_void_p] * 8 + [ctypes.c_int] * 7 + [ctypes.c_void_p, sz]
    ws = ctypes.c_void_p(0x2000)
    need = lib.sq_blocked_map_bytes(1, 16, 8, 8)
    assert fire(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, NULL, 1, 96, 8, 8, 16, 64, 64, ws, need) == -1
    assert fire(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1, 96, 8, 8, 16, 64, 64, ws, need - 1) == -4
    assert fire(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1, 96, 8, 8, 16, 64, 64, ctypes.c_void_p(0x2010), need) == -4
    assert fire(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1, 96, 8, 8, 0, 64, 64, ws, need) == -2
    assert fire(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1, 100, 8, 8, 16, 64, 64, ws, need) == -3   # Cin % 16

    net = lib.sq_squeezenet_forward_bf16
    net.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(ctypes.c_void_p), ctypes.c_void_p, ctypes.c_void_p,
                    ctypes.c_int, ctypes.c_void_p, sz, ctypes.POINTER(ctypes.c_void_p)]
    params = (ctypes.c_void_p * 52)(*([0x1000] * 52))
    big = lib.sq_squeezenet_bf16_workspace_bytes(1)
    assert net(NULL, 0, params, FAKE, FAKE, 1, ws, big, None) == -1
    assert net(FAKE, 0, params, FAKE, FAKE, 0, ws, big, None) == -2
    assert net(FAKE, 3, params, FAKE, FAKE, 1, ws, big, None) == -3
    assert net(FAKE, 0, params, ctypes.c_void_p(0x1000), FAKE, 1, ws, big - 1, None) == -4
    assert net(FAKE, 0, params, ctypes.c_void_p(0x1010), FAKE, 1, ws, big, None) == -4        # packed kernels 256-byte aligned
    # conv1's bfloat16 output of 908 images passes 2^31 bytes: refused before anything is enqueued
    assert 907 * 96 * 111 * 111 * 2 < 2 ** 31 <= 908 * 96 * 111 * 111 * 2
    assert net(FAKE, 0, params, FAKE, FAKE, 908, ws, lib.sq_squeezenet_bf16_workspace_bytes(908), None) == -3
    assert net(FAKE, 0, params, FAKE, FAKE, 907, ws, lib.sq_squeezenet_bf16_workspace_bytes(907) - 1, None) == -4
    holes = (ctypes.c_void_p * 52)(*([0x1000] * 51 + [None]))
    assert net(FAKE, 0, holes, FAKE, FAKE, 1, ws, big, None) == -1
    pk = lib.sq_squeezenet_bf16_pack_params
    pk.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_void_p, sz]
    assert pk(params, ctypes.c_void_p(0x1000), lib.sq_squeezenet_bf16_packed_bytes() - 1) == -4
    assert pk(holes, ctypes.c_void_p(0x1000), lib.sq_squeezenet_bf16_packed_bytes()) == -1


def test_dtype_setter_and_packed_entry_points_validate_before_any_gpu_call(lib):
    sz = ctypes.c_size_t
    lib.sq_packed_weights_bytes.restype = sz
    lib.sq_fire_packed_bytes.restype = sz
    lib.sq_squeezenet_bf16_packed_bytes.restype = sz
    assert lib.sq_set_dtype(0) == 0 and lib.sq_set_dtype(7) == -3
    # fp32: the sixteen-value transforms of the eight expand3x3 kernel sets (output layers in blocks of 64)
    fires = [(16, 64), (16, 64), (32, 128), (32, 128), (48, 192), (48, 192), (64, 256), (64, 256)]
    assert lib.sq_packed_weights_bytes(0) == sum(16 * 4 * sq * ((e + 63) // 64 * 64) + 16 * 4 * sq * e for sq, e in fires)
    assert lib.sq_packed_weights_bytes(1) == lib.sq_squeezenet_bf16_packed_bytes()
    assert lib.sq_packed_weights_bytes(5) == 0
    assert lib.sq_fire_packed_bytes(16, 64) == 2 * 16 * 4 * 16 * 64
    assert lib.sq_fire_packed_bytes(12, 64) == 0 and lib.sq_fire_packed_bytes(16, 0) == 0
    params = (ctypes.c_void_p * 52)(*([0x1000] * 52))
    pk = lib.sq_pack_weights
    pk.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_void_p, sz]
    need = lib.sq_packed_weights_bytes(0)
    assert pk(params, 0, NULL, need) == -1
    assert pk(params, 0, ctypes.c_void_p(0x1010), need) == -4
    assert pk(params, 0, FAKE, need - 1) == -4
    assert pk(params, 9, FAKE, need) == -3
    holes = (ctypes.c_void_p * 52)(*([0x1000] * 30 + [None] + [0x1000] * 21))
    assert pk(holes, 0, FAKE, need) == -1
    fp = lib.sq_fire_pack_weights
    fp.argtypes = [ctypes.c_void_p, ctypes.c_void_p, sz, ctypes.c_int, ctypes.c_int]
    assert fp(NULL, FAKE, 131072, 16, 64) == -1
    assert fp(FAKE, FAKE, 131071, 16, 64) == -4
    assert fp(FAKE, FAKE, 131072, 12, 64) == -3
    assert fp(FAKE, FAKE, 131072, 0, 64) == -2
    net = lib.sq_squeezenet_forward_packed
    net.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
                    ctypes.c_void_p, sz, ctypes.POINTER(ctypes.c_void_p)]
    lib.sq_squeezenet_workspace_bytes.restype = sz
    wsb = lib.sq_squeezenet_workspace_bytes(1)
    ws = ctypes.c_void_p(0x2000)
    assert net(FAKE, params, NULL, FAKE, 1, ws, wsb, None) == -1
    assert net(FAKE, params, ctypes.c_void_p(0x1010), FAKE, 1, ws, wsb, None) == -4
    assert net(FAKE, params, FAKE, FAKE, 0, ws, wsb, None) == -2
    assert net(FAKE, params, FAKE, FAKE, 1, ws, wsb - 1, None) == -4
    ff = lib.sq_fire_forward_packed
    ff.argtypes = [ctypes.c_void_p] * 9 + [ctypes.c_int] * 7 + [ctypes.c_void_p, sz]
    mapb = (2 * 16 * 55 * 55 * 4 + 255) // 256 * 256
    good = [2, 96, 55, 55, 16, 64, 64]
    assert ff(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, NULL, FAKE, *good, ws, mapb) == -1
    assert ff(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, *good, ws, mapb - 1) == -4
    assert ff(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 2, 96, 55, 55, 12, 64, 64, ws, mapb) == -3
    # reduced precision is a mode of the calling thread: the fp32-only calls refuse it, and say so before anything else
    assert lib.sq_set_dtype(1) == 0
    try:
        assert ff(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, *good, ws, mapb) == -3
        plain = lib.sq_squeezenet_forward
        plain.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p), ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, sz,
                          ctypes.POINTER(ctypes.c_void_p)]
        assert plain(FAKE, params, FAKE, 1, ws, wsb, None) == -3
        # packed network in reduced precision: the checks of the reduced-precision network apply (batch limit 907)
        assert net(FAKE, params, FAKE, FAKE, 908, ws, sz(1 << 40), None) == -3
        assert net(FAKE, params, FAKE, FAKE, 454, ws, 16, None) == -4
    finally:
        assert lib.sq_set_dtype(0) == 0


def test_two_host_threads_call_entry_points_at_once(lib):
    """Stream, arithmetic mode and last error belong to the calling thread; size queries and argument checks
    run concurrently without sharing anything that is written."""
    import threading
    sz = ctypes.c_size_t
    lib.sq_fire_workspace_bytes.restype = sz
    lib.sq_squeezenet_workspace_bytes.restype = sz
    fire = lib.sq_fire_forward
    fire.argtypes = [ctypes.c_void_p] * 8 + [ctypes.c_int] * 7 + [ctypes.c_void_p, sz]
    need = lib.sq_fire_workspace_bytes(2, 55, 55, 16, 64)
    errors, barrier = [], threading.Barrier(2)

    def worker(mode):
        try:
            barrier.wait()
            assert lib.sq_set_dtype(mode) == 0
            assert lib.sq_set_stream(ctypes.c_void_p(0)) == 0
            for i in range(2000):
                # the other thread keeps the other mode: this thread's answer never changes
                rc = fire(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 2, 96, 55, 55, 16, 64, 64, NULL, need)
                assert rc == (-4 if mode == 0 else -3), (mode, i, rc)
                assert lib.sq_squeezenet_workspace_bytes(1 + i % 7) > 0
                assert lib.sq_conv2d_forward(FAKE, FAKE, FAKE, FAKE, 1, 3, 8, 8, 4, 3, 0, 1, 1) == -2
                assert lib.sq_maxpool(FAKE, FAKE, 1, 1, 2, 8, 3, 2) == -2
                assert lib.sq_last_hip_error() == 0
        except Exception as e:       # noqa: BLE001 - reported by the main thread
            errors.append(e)
        finally:
            lib.sq_set_dtype(0)

    threads = [threading.Thread(target=worker, args=(m,)) for m in (0, 1)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors


# ---- split pooling (sq_tuning.h): the map format's own arithmetic, and argument checks without a GPU ----------

def _row_stride(Wo, shift):
    Wp = (Wo - 3) // 2 + 1
    return Wp + (Wp >> shift) + 2


def test_column_pooled_rows_hold_every_seam_slot():
    """Position of pooled column x = x + (group ends before it); the reader also loads the slot behind it.  For every
    width, group size and alignment of a row's first slot both must lie inside the row, positions must not collide, and
    a seam slot must sit exactly between the last column of a group and the first of the next."""
    for shift in range(1, 7):
        gm = (1 << shift) - 1
        for Wo in list(range(3, 140)) + [223, 224, 511]:
            Wp = (Wo - 3) // 2 + 1
            rs = _row_stride(Wo, shift)
            for q0 in range(0, 3 << shift):
                pos = [x + ((q0 + x) >> shift) - (q0 >> shift) for x in range(Wp)]
                assert pos[0] == 0 and pos[-1] + 1 <= rs - 1, (shift, Wo, q0)
                for x in range(1, Wp):
                    step = pos[x] - pos[x - 1]
                    assert step == (2 if ((q0 + x - 1) & gm) == gm else 1), (shift, Wo, q0, x)
                # the writer of the tile after the row's last pooled column puts its first column one slot before
                # the position that tile's own pooled column would have: still inside the row
                after = Wp + ((q0 + Wp) >> shift) - (q0 >> shift)
                assert after - 1 <= rs - 1


def test_split_pooling_hooks_validate_before_any_gpu_call(lib):
    f = ctypes.c_void_p(256)          # never dereferenced on the host
    geo = (ctypes.c_int * 4)()
    conv = lib.sq_tune_conv2d_forward_poolcols
    conv.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_int] * 8 + [ctypes.POINTER(ctypes.c_int)]
    assert conv(None, f, f, f, 1, 3, 224, 224, 96, 7, 2, 2, geo) == -1
    assert conv(f, f, f, f, 1, 3, 224, 224, 96, 7, 2, 2, None) == -1
    assert conv(f, f, f, f, 0, 3, 224, 224, 96, 7, 2, 2, geo) == -2
    assert conv(f, f, f, f, 1, 3, 224, 224, 64, 7, 2, 2, geo) == -3      # only the conv1-type layer has the form
    assert conv(f, f, f, f, 1, 3, 224, 224, 96, 3, 1, 1, geo) == -3
    assert conv(f, f, f, f, 1, 3, 5, 224, 96, 7, 2, 0, geo) == -2        # kernel does not fit
    assert conv(f, f, f, f, 1, 3, 224, 9, 96, 7, 2, 0, geo) == -2        # fewer than three result columns: nothing to pool
    fire = lib.sq_tune_fire_forward_poolcols
    fire.argtypes = [ctypes.c_void_p] * 8 + [ctypes.c_int] * 7 + [ctypes.c_void_p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_int)]
    assert fire(f, f, f, f, f, f, f, None, 3, 32, 9, 9, 16, 32, 32, f, 1 << 30, geo) == -1
    assert fire(f, f, f, f, f, f, f, f, 3, 32, 9, 2, 16, 32, 32, f, 1 << 30, geo) == -2
    assert fire(f, f, f, f, f, f, f, f, 3, 32, 9, 9, 16, 32, 32, None, 0, geo) == -4
    assert fire(f, f, f, f, f, f, f, f, 3, 32, 9, 9, 16, 32, 32, f, 16, geo) == -4
    assert fire(f, f, f, f, f, f, f, f, 2, 32, 9, 9, 16, 32, 32, f, 1 << 30, geo) == -3   # no expand pair below three images
    rows = lib.sq_tune_poolrows_conv2d_forward
    rows.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_int] * 9 + [ctypes.POINTER(ctypes.c_int)]
    ok = (ctypes.c_int * 4)(4, 6, 30, _row_stride(11, 4))
    assert rows(None, f, f, f, 1, 16, 9, 11, 16, 1, 16, 0, 0, ok) == -1
    assert rows(f, f, f, f, 1, 16, 2, 11, 16, 1, 16, 0, 0, ok) == -2
    assert rows(f, f, f, f, 1, 16, 9, 11, 16, 1, 8, 0, 0, ok) == -2       # layer range outside the output tensor
    assert rows(f, f, f, f, 1, 16, 9, 11, 16, 1, 16, 0, 1, ok) == -3      # the one-thread-per-output kernel has no such form
    for bad in ((0, 6, 30, 8), (4, 3, 30, 8), (4, 6, 29, 8), (4, 6, 30, _row_stride(11, 4) - 1)):
        assert rows(f, f, f, f, 1, 16, 9, 11, 16, 1, 16, 0, 0, (ctypes.c_int * 4)(*bad)) == -2, bad
