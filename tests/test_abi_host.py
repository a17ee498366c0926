"""Host-side tests of the C ABI: the library loads, exports every symbol the header
declares, rejects bad arguments before touching the GPU, and its tile mapping is a
bijection.  No compute call needs a GPU here."""
import ctypes
import os
import re

import pytest

from paper_2205_00618_amd import binding as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
P = 4096  # a fake, non-null device address: validation never dereferences it


def _has_gpu():
    import torch
    return torch.cuda.is_available()


def header_symbols():
    names = []
    inc = os.path.join(ROOT, "include")
    for header in sorted(os.listdir(inc)):
        if not header.endswith(".h"):
            continue
        text = open(os.path.join(inc, header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"\b([A-Za-z_][A-Za-z0-9_]*)\s*\(", text)
    return names


def test_library_exports_every_declared_symbol():
    lib = b.load()
    declared = set(header_symbols())
    assert declared == set(b.SYMBOLS)
    for name in declared:
        assert hasattr(lib, name), name
    assert b.version() >= 141


def test_strerror_covers_all_codes():
    seen = {b.strerror(c) for c in range(0, -8, -1)}
    assert len(seen) == 8 and "unknown status" not in seen
    assert b.strerror(-99) == "unknown status"


@pytest.mark.parametrize("fn", [b.sgemm, b.igemm_s8s32])
def test_gemm_validation(fn):
    assert fn(-1, 4, 4, P, 4, P, 4, P, 4) == b.ERR_DIM
    assert fn(4, -1, 4, P, 4, P, 4, P, 4) == b.ERR_DIM
    assert fn(4, 4, -1, P, 4, P, 4, P, 4) == b.ERR_DIM
    assert fn(4, 4, 8, P, 7, P, 4, P, 4) == b.ERR_LD      # lda < K
    assert fn(4, 8, 4, P, 4, P, 7, P, 8) == b.ERR_LD      # ldb < N
    assert fn(4, 8, 4, P, 4, P, 8, P, 7) == b.ERR_LD      # ldc < N
    assert fn(4, 4, 4, P, 0, P, 4, P, 4) == b.ERR_LD
    assert fn(4, 4, 4, 0, 4, P, 4, P, 4) == b.ERR_NULL
    assert fn(4, 4, 4, P, 4, 0, 4, P, 4) == b.ERR_NULL
    assert fn(4, 4, 4, P, 4, P, 4, 0, 4) == b.ERR_NULL
    assert fn(2**31, 4, 4, P, 4, P, 4, P, 4) == b.ERR_TOO_LARGE
    assert fn(4, 4, 4, P, 2**31, P, 4, P, 4) == b.ERR_TOO_LARGE
    # empty problems succeed without a device and without looking at the pointers
    assert fn(0, 4, 4, 0, 4, 0, 4, 0, 4) == b.OK
    assert fn(4, 0, 4, 0, 4, 0, 1, 0, 1) == b.OK
    assert fn(4, 4, 0, 0, 1, 0, 4, 0, 4) == b.OK


def test_gemm_bt_validation():
    fn = b.igemm_s8s32_bt   # Bt is N x K: ldbt is checked against K
    assert fn(-1, 4, 4, P, 4, P, 4, P, 4) == b.ERR_DIM
    assert fn(4, 4, 8, P, 7, P, 8, P, 4) == b.ERR_LD      # lda < K
    assert fn(4, 2, 8, P, 8, P, 7, P, 2) == b.ERR_LD      # ldbt < K
    assert fn(4, 8, 2, P, 2, P, 2, P, 7) == b.ERR_LD      # ldc < N
    if not _has_gpu():
        assert fn(4, 8, 2, P, 2, P, 2, P, 8) == b.ERR_NO_DEVICE   # ldbt < N is fine: reaches the device check
    assert fn(4, 4, 4, P, 4, 0, 4, P, 4) == b.ERR_NULL
    assert fn(4, 4, 4, P, 4, P, 2**31, P, 4) == b.ERR_TOO_LARGE
    assert fn(4, 4, 0, 0, 1, 0, 1, 0, 4) == b.OK
    assert fn(0, 4, 4, 0, 4, 0, 4, 0, 4) == b.OK


def test_conv_validation():
    ok = dict(N=1, H=8, W=8, C=4, K=4, R=3, S=3, stride=1, pad=1)

    def call(**kw):
        a = dict(ok, **kw)
        return b.conv2d_nhwc(a["N"], a["H"], a["W"], a["C"], a["K"], a["R"], a["S"], a["stride"],
                             a["pad"], a.get("inp", P), a.get("w", P), a.get("out", P))

    for key in ("C", "K", "R", "S", "stride"):
        assert call(**{key: 0}) == b.ERR_DIM, key
    for key in ("N", "H", "W", "pad"):
        assert call(**{key: -1}) == b.ERR_DIM, key
    assert call(H=1, pad=0) == b.ERR_DIM            # filter taller than the padded image
    assert call(W=2, R=3, S=5, pad=1) == b.ERR_DIM
    assert call(w=0) == b.ERR_NULL
    assert call(out=0) == b.ERR_NULL
    assert call(inp=0) == b.ERR_NULL
    assert call(N=2**20, H=2**10, W=2**10) == b.ERR_TOO_LARGE
    assert call(K=2**31) == b.ERR_TOO_LARGE
    assert call(N=0, inp=0, w=0, out=0) == b.OK


def test_dwconv_validation():
    ok = dict(N=1, H=8, W=8, C=4, R=3, S=3, stride=1, pad=1)

    def call(**kw):
        a = dict(ok, **kw)
        return b.dwconv2d_nhwc_fused(a["N"], a["H"], a["W"], a["C"], a["R"], a["S"], a["stride"], a["pad"],
                                     a.get("inp", P), a.get("w", P), a.get("out", P), a.get("bias"),
                                     a.get("post", b.POST_NONE))

    for key in ("C", "R", "S", "stride"):
        assert call(**{key: 0}) == b.ERR_DIM, key
    for key in ("N", "H", "W", "pad"):
        assert call(**{key: -1}) == b.ERR_DIM, key
    assert call(H=1, pad=0) == b.ERR_DIM
    assert call(post=7) == b.ERR_OP
    assert call(w=0) == b.ERR_NULL
    assert call(out=0) == b.ERR_NULL
    assert call(inp=0) == b.ERR_NULL
    assert call(N=2**20, H=2**10, W=2**10) == b.ERR_TOO_LARGE
    assert call(C=2**31) == b.ERR_TOO_LARGE
    assert call(stride=2**31) == b.ERR_TOO_LARGE
    assert call(N=0, inp=0, w=0, out=0) == b.OK
    assert b.dwconv2d_nhwc(1, 8, 8, 4, 3, 3, 0, 1, P, P, P) == b.ERR_DIM
    assert b.dwconv2d_nhwc(0, 8, 8, 4, 3, 3, 1, 1, 0, 0, 0) == b.OK


@pytest.mark.parametrize("fn", [b.tensor_copy_f32, b.tensor_copy_s8])
def test_tensor_copy_validation(fn):
    if not _has_gpu():   # never launch on the fake address
        assert fn(2, 2, 2, 2, 8, 4, 2, 1, P, P) == b.ERR_NO_DEVICE   # valid: reaches the device check
    assert fn(-1, 2, 2, 2, 8, 4, 2, 1, P, P) == b.ERR_DIM
    assert fn(2, 2, 2, 2, 8, 4, -2, 1, P, P) == b.ERR_DIM
    assert fn(2, 2, 2, 2, 8, 4, 2, 1, 0, P) == b.ERR_NULL
    assert fn(2, 2, 2, 2, 8, 4, 2, 1, P, 0) == b.ERR_NULL
    assert fn(0, 2, 2, 2, 8, 4, 2, 1, 0, 0) == b.OK
    assert fn(2, 2, 0, 2, 8, 4, 2, 1, 0, 0) == b.OK
    assert fn(2**31, 1, 1, 1, 0, 0, 0, 0, P, P) == b.ERR_TOO_LARGE
    assert fn(2**16, 2**16, 1, 1, 0, 0, 0, 0, P, P) == b.ERR_TOO_LARGE     # 2^32 elements
    assert fn(2, 1, 1, 1, 2**31, 0, 0, 0, P, P) == b.ERR_TOO_LARGE
    assert fn(2**20, 1, 1, 1, 2**20, 0, 0, 0, P, P) == b.ERR_TOO_LARGE     # last offset ~2^40


def test_fused_validation():
    assert b.sgemm_fused(4, 4, 4, P, 4, P, 4, P, 4, None, 9, 0) == b.ERR_OP
    assert b.sgemm_fused(4, 4, 4, P, 4, P, 4, P, 4, None, 0, 9) == b.ERR_OP
    assert b.sgemm_fused(4, 4, 4, P, 4, P, 4, P, 4, None, b.PRE_BIAS, b.POST_RELU) == b.ERR_NULL
    assert b.sgemm_fused(-1, 4, 4, P, 4, P, 4, P, 4, None, 0, 0) == b.ERR_DIM
    assert b.sgemm_fused(4, 4, 4, P, 3, P, 4, P, 4, None, 0, 0) == b.ERR_LD
    assert b.sgemm_fused(0, 4, 4, 0, 4, 0, 4, 0, 4, None, b.PRE_ZERO, b.POST_RELU) == b.OK
    assert b.sgemm_fused(4, 4, 0, 0, 1, 0, 4, 0, 4, None, 0, 0) == b.OK        # plain form, K = 0: no-op
    assert b.sgemm_fused(4, 4, 0, 0, 1, 0, 4, 0, 4, None, b.PRE_ZERO, 0) == b.ERR_NULL  # must write C
    assert b.conv2d_nhwc_fused(1, 8, 8, 4, 4, 3, 3, 1, 1, P, P, P, None, 5) == b.ERR_OP
    assert b.conv2d_nhwc_fused(0, 8, 8, 4, 4, 3, 3, 1, 1, 0, 0, 0, None, b.POST_RELU) == b.OK


def test_no_device_is_reported_not_crashed():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    assert b.sgemm(4, 4, 4, P, 4, P, 4, P, 4) == b.ERR_NO_DEVICE
    assert b.last_hip_error() != 0


def test_tuning_and_variant_table():
    names = b.variant_names()
    assert len(names) >= 2 and all(n.startswith("sgemm_") for n in names)
    assert b.set_tuning(len(names), 0) == b.ERR_DIM
    assert b.set_tuning(-2, 0) == b.ERR_DIM
    assert b.set_tuning(0, -1) == b.ERR_DIM
    assert b.set_tuning(0, 3) == b.OK
    assert b.set_tuning(-1, 0) == b.OK
    assert b.set_stream(None) == b.OK
    assert b.set_conv_tuning(99) == b.ERR_DIM
    assert b.set_conv_tuning(-2) == b.ERR_DIM
    assert b.set_conv_tuning(0) == b.OK
    assert b.set_conv_tuning(-1) == b.OK
    assert b.set_igemm_tuning(len(b.igemm_variant_names())) == b.ERR_DIM
    assert b.set_igemm_tuning(-2) == b.ERR_DIM
    assert b.set_igemm_tuning(2) == b.OK
    assert b.set_igemm_tuning(-1) == b.OK
    assert b.igemm_variant_names()[:2] == ["igemm_128x128x64", "igemm_64x64x64"]
    assert b.set_conv_split(-1) == b.ERR_DIM
    assert b.set_conv_split(4) == b.OK
    assert b.set_conv_split(0) == b.OK
    assert b.set_conv_tail(-2) == b.ERR_DIM
    assert b.set_conv_tail(3) == b.OK
    assert b.set_conv_tail(-1) == b.OK
    assert len(b.conv_variant_names()) >= 9 and all(n.startswith("conv2d_") for n in b.conv_variant_names())
    assert b.set_dwconv_tuning(len(b.dwconv_variant_names()), 0) == b.ERR_DIM
    assert b.dwconv_variant_names()[4:6] == ["dwconv_direct_vec4", "dwconv_direct_scalar"]
    assert b.set_dwconv_tile(-1, 0, 0) == b.ERR_DIM
    assert b.set_dwconv_tile(0, 0, 3) == b.ERR_DIM
    assert b.set_dwconv_tile(7, 8, 2) == b.OK
    assert b.set_dwconv_tile(0, 0, 0) == b.OK
    assert b.set_dwconv_tuning(-2, 0) == b.ERR_DIM
    assert b.set_dwconv_tuning(0, -1) == b.ERR_DIM
    assert b.set_dwconv_tuning(5, 8) == b.OK
    assert b.set_dwconv_tuning(-1, 0) == b.OK


@pytest.mark.parametrize("tm,tn,group", [(1, 1, 8), (32, 32, 8), (33, 2, 8), (8, 8, 3), (5, 7, 8),
                                         (1, 100, 8), (100, 1, 8), (3, 3, 1), (17, 13, 4)])
def test_tile_mapping_is_a_bijection(tm, tn, group):
    seen = set()
    for wg in range(tm * tn):
        r, c = b.tile_of_workgroup(wg, tm, tn, group)
        assert 0 <= r < tm and 0 <= c < tn
        seen.add((r, c))
    assert len(seen) == tm * tn
    with pytest.raises(b.LsmiError):
        b.tile_of_workgroup(tm * tn, tm, tn, group)


def test_tile_mapping_keeps_an_xcd_on_neighbouring_tiles():
    # 32 x 32 tiles, bands of 8 rows: the 128 workgroups of one XCD (ids = xcd mod 8)
    # cover an 8 x 16 block, i.e. 8 A panels and 16 B panels instead of 32 + 32
    tiles = [b.tile_of_workgroup(wg, 32, 32, 8) for wg in range(0, 1024, 8)]
    rows = {r for r, _ in tiles}
    cols = {c for _, c in tiles}
    assert len(rows) == 8 and len(cols) == 16


def test_build_reports_spilling_kernels():
    from paper_2205_00618_amd import build
    report = """a.hip:1:1: remark: Function Name: kernel_a [-Rpass-analysis=kernel-resource-usage]
a.hip:1:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]
a.hip:9:1: remark: Function Name: kernel_b [-Rpass-analysis=kernel-resource-usage]
a.hip:9:1: remark:     ScratchSize [bytes/lane]: 384 [-Rpass-analysis=kernel-resource-usage]"""
    assert build.spilling_kernels(report) == [("kernel_b", 384)]


def test_division_by_multiplication_is_exact():
    """The kernels' division by a launch-time divisor against Python's integer division: small
    and large divisors, powers of two and their neighbours, numerators at the 32-bit edges."""
    import random
    rng = random.Random(7)
    divisors = [1, 2, 3, 5, 7, 8, 9, 56, 3136, 64, 63, 65, 255, 256, 257, 1000, 4096, 4097, 65535, 65536,
                65537, 2**31 - 1, 2**31, 2**31 + 1, 2**32 - 1] + [rng.randrange(1, 2**32) for _ in range(200)]
    for d in divisors:
        edge = [0, 1, d - 1, d, d + 1, 2 * d - 1, 2 * d, 2**31 - 1, 2**31, 2**32 - 1, (2**32 - 1) // d * d,
                (2**32 - 1) // d * d - 1]
        for n in edge + [rng.randrange(0, 2**32) for _ in range(50)]:
            if 0 <= n < 2**32:
                assert b.fast_divide(n, d) == n // d, (n, d)


def test_tile_walk_of_the_kernels_matches_the_plain_definition():
    # lsmi_tile_of_workgroup runs the kernels' form (launch-time divisors); the walk's definition:
    # ids are dealt to 8 XCDs round-robin, every XCD owns a contiguous range of the logical order,
    # which runs down bands of group_m tile rows, column by column
    for tiles_m, tiles_n, group_m in [(1, 1, 8), (7, 3, 8), (32, 32, 8), (33, 5, 8), (9, 16, 4), (1568, 1, 1), (5, 1, 1)]:
        nt = tiles_m * tiles_n
        order = []
        for g in range(0, tiles_m, group_m):
            rows = min(group_m, tiles_m - g)
            order += [(g + r, c) for c in range(tiles_n) for r in range(rows)]
        q, rem = divmod(nt, 8)
        for wg in range(nt):
            xcd, idx = wg % 8, wg // 8
            logical = xcd * q + min(xcd, rem) + idx
            assert b.tile_of_workgroup(wg, tiles_m, tiles_n, group_m) == order[logical], (wg, tiles_m, tiles_n)
