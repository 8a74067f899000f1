"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and validates descriptors before touching the device."""
import os
import re

import pytest

from paper_1704_04428_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_1704_04428_amd import build
        build.build()
    return B.lib()


def _declared_symbols():
    with open(os.path.join(ROOT, "include", "conv_mcmk.h")) as f:
        text = f.read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(conv_mcmk_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_symbols()
    assert set(names) == set(B.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def test_strerror_covers_all_codes(lib):
    texts = [B.strerror(c) for c in range(7)]
    assert texts[0] == "ok" and len(set(texts)) == 7
    assert "unknown" in B.strerror(99)


def test_check_accepts_benchmark_layers(lib):
    from paper_1704_04428_amd import workloads as wl
    for L in wl.LAYERS.values():
        d = B.desc(L.n, L.c, L.h, L.w, L.m, L.k, L.pad)
        for v in (B.KN2ROW, B.KN2ROW_2PASS, B.IM2COL, B.DIRECT, B.KN2COL, B.IM2ROW):
            assert B.conv_mcmk_check(d, v) == B.OK, (L.name, v)


def test_check_rejects_bad_descriptors(lib):
    ok = dict(n=1, c=4, h=8, w=8, m=4, k=3, pad=1)
    for field in ("n", "c", "h", "w", "m", "k"):
        bad = dict(ok, **{field: 0})
        assert B.conv_mcmk_check(B.desc(**bad), B.KN2ROW_2PASS) == B.ERR_SHAPE, field
    assert B.conv_mcmk_check(B.desc(**dict(ok, pad=-1)), B.KN2ROW) == B.ERR_SHAPE
    assert B.conv_mcmk_check(B.desc(**dict(ok, h=2, w=2, k=5, pad=0)), B.IM2COL) == B.ERR_SHAPE   # empty output
    # strides are a generalisation (section II-A treats unit stride): fused kernels take 1 and 2, the rest any
    assert B.conv_mcmk_check(B.desc(**ok, stride=0), B.IM2COL) == B.ERR_SHAPE
    assert B.conv_mcmk_check(B.desc(**ok, stride=2), B.KN2ROW) == B.OK
    assert B.conv_mcmk_check(B.desc(**ok, stride=3), B.KN2ROW) == B.ERR_UNSUPPORTED
    assert B.conv_mcmk_check(B.desc(**ok, stride=3), B.KN2COL) == B.ERR_UNSUPPORTED
    for v in (B.KN2ROW_2PASS, B.IM2COL, B.IM2ROW, B.DIRECT):
        assert B.conv_mcmk_check(B.desc(**ok, stride=3), v) == B.OK
    assert B.conv_mcmk_check(B.desc(**ok, dtype=7), B.KN2ROW) == B.ERR_UNSUPPORTED
    assert B.conv_mcmk_check(B.desc(**ok), 9) == B.ERR_UNSUPPORTED
    for k in range(1, 8):                                                                         # fused: k = 1 .. 7
        assert B.conv_mcmk_check(B.desc(**dict(ok, k=k, pad=3)), B.KN2ROW) == B.OK
        assert B.conv_mcmk_check(B.desc(**dict(ok, k=k, pad=3)), B.KN2COL) == B.OK
    assert B.conv_mcmk_check(B.desc(**dict(ok, k=8, pad=4)), B.KN2ROW) == B.ERR_UNSUPPORTED
    assert B.conv_mcmk_check(B.desc(**dict(ok, k=8, pad=4)), B.KN2COL) == B.ERR_UNSUPPORTED
    assert B.conv_mcmk_check(B.desc(**dict(ok, k=8, pad=4)), B.KN2ROW_2PASS) == B.OK
    assert B.conv_mcmk_check(B.desc(**dict(ok, c=12), dtype=B.BF16), B.KN2COL) == B.ERR_UNSUPPORTED   # octets
    assert B.conv_mcmk_check(B.desc(**dict(ok, c=16), dtype=B.BF16), B.KN2COL) == B.OK
    assert B.conv_mcmk_check(B.desc(**dict(ok, c=12)), B.KN2COL) == B.OK
    assert B.conv_mcmk_check(B.desc(**dict(ok, c=6)), B.KN2COL) == B.ERR_UNSUPPORTED                   # quads
    assert B.conv_mcmk_check(B.desc(**dict(ok, h=70000, w=70000)), B.DIRECT) == B.ERR_SHAPE      # >= 2^31 per image
    assert lib.conv_mcmk_check(None, B.KN2ROW) == B.ERR_NULL
    # bf16 [C][H][W] input is staged two positions at a time: a one-element plane is refused
    one = dict(n=1, c=8, h=1, w=1, m=4, k=1, pad=0)
    assert B.conv_mcmk_check(B.desc(**one), B.KN2ROW) == B.OK
    assert B.conv_mcmk_check(B.desc(**one, dtype=B.BF16), B.KN2ROW) == B.ERR_UNSUPPORTED
    assert B.conv_mcmk_check(B.desc(**one, dtype=B.BF16), B.KN2ROW_2PASS) == B.ERR_UNSUPPORTED
    assert B.conv_mcmk_check(B.desc(**one, dtype=B.BF16), B.IM2COL) == B.ERR_UNSUPPORTED
    assert B.conv_mcmk_check(B.desc(**one, dtype=B.BF16), B.KN2COL) == B.OK
    assert B.conv_mcmk_check(B.desc(**dict(one, w=2), dtype=B.BF16), B.KN2ROW) == B.OK
    # the patch matrix of one image must stay addressable with 32-bit byte offsets: 512 x 25 x 224 x 224 elements does not
    big = B.desc(1, 512, 224, 224, 64, 5, 2)
    assert B.conv_mcmk_check(big, B.KN2ROW) == B.OK
    assert B.conv_mcmk_check(big, B.KN2ROW_2PASS) == B.OK
    assert B.conv_mcmk_check(big, B.IM2COL) == B.ERR_SHAPE
    assert B.conv_mcmk_check(big, B.IM2ROW) == B.ERR_SHAPE
    assert B.conv_mcmk_select(big)[0] == B.KN2ROW


def test_sizes(lib):
    d = B.desc(2, 20, 9, 11, 35, 3, 1)
    q, p = 9, 11

    def patch_workspace(desc, variant, matrix_bytes, result_floats):
        # the patch matrix, alone or followed (at the next multiple of 256 bytes) by 2, 4, 8 or 16 copies of the result
        total = B.conv_mcmk_workspace_bytes(desc, variant)
        copies = (result_floats + 3) // 4 * 4 * 4
        assert total in [matrix_bytes] + [(matrix_bytes + 255) // 256 * 256 + parts * copies for parts in (2, 4, 8, 16)]
        return total
    assert B.conv_mcmk_workspace_bytes(d, B.KN2ROW) == 0
    assert B.conv_mcmk_workspace_bytes(d, B.DIRECT) == 0
    assert B.conv_mcmk_workspace_bytes(d, B.KN2ROW_2PASS) == 2 * 9 * 35 * 9 * 11 * 4     # k^2 x the output
    patch_workspace(d, B.IM2COL, 2 * 20 * 9 * q * p * 4, 2 * 35 * q * p)                  # k^2 x the input
    # stride 2: Q = floor((9 + 2 - 3) / 2) + 1 = 5, P = floor((11 + 2 - 3) / 2) + 1 = 6; the patch matrix shrinks,
    # the two-pass product (all H x W positions of every tap) does not
    ds = B.desc(2, 20, 9, 11, 35, 3, 1, 2)
    patch_workspace(ds, B.IM2COL, 2 * 20 * 9 * 5 * 6 * 4, 2 * 35 * 5 * 6)
    patch_workspace(ds, B.IM2ROW, 2 * 20 * 9 * 5 * 6 * 4, 2 * 35 * 5 * 6)
    assert B.conv_mcmk_workspace_bytes(ds, B.KN2ROW_2PASS) == 2 * 9 * 35 * 9 * 11 * 4
    assert B.conv_mcmk_packed_kernel_bytes(ds, B.KN2ROW) == B.conv_mcmk_packed_kernel_bytes(d, B.KN2ROW)
    mb, cg = 3, 2      # ceil(35/16), ceil(20/16)
    assert B.conv_mcmk_packed_kernel_bytes(d, B.KN2ROW) == 9 * mb * cg * 256 * 4
    assert B.conv_mcmk_packed_kernel_bytes(d, B.KN2ROW_2PASS) == 9 * mb * cg * 256 * 4
    assert B.conv_mcmk_packed_kernel_bytes(d, B.KN2COL) == 9 * mb * cg * 256 * 4
    assert B.conv_mcmk_workspace_bytes(d, B.KN2COL) == 0
    patch_workspace(d, B.IM2ROW, 2 * 20 * 9 * q * p * 4, 2 * 35 * q * p)
    assert B.conv_mcmk_packed_kernel_bytes(d, B.IM2ROW) == B.conv_mcmk_packed_kernel_bytes(d, B.IM2COL)
    assert B.conv_mcmk_check(B.desc(2, 21, 9, 11, 35, 3, 1), B.IM2ROW) == B.ERR_UNSUPPORTED      # channel vectors
    assert B.conv_mcmk_packed_kernel_bytes(d, B.IM2COL) == mb * 12 * 256 * 4              # ceil(180/16) = 12
    assert B.conv_mcmk_packed_kernel_bytes(d, B.DIRECT) == 0
    assert B.conv_mcmk_workspace_bytes(B.desc(0, 1, 1, 1, 1, 1, 0), B.IM2COL) == 0
    # bf16 operands: 32-channel groups, 2-byte elements; the two-pass product stays fp32
    db = B.desc(2, 20, 9, 11, 35, 3, 1, 1, B.BF16)
    assert B.conv_mcmk_packed_kernel_bytes(db, B.KN2ROW) == 9 * mb * 1 * 512 * 2
    assert B.conv_mcmk_packed_kernel_bytes(db, B.IM2COL) == mb * 6 * 512 * 2                  # ceil(180/32) = 6
    patch_workspace(db, B.IM2COL, 2 * 20 * 9 * q * p * 2, 2 * 35 * q * p)
    assert B.conv_mcmk_workspace_bytes(db, B.KN2ROW_2PASS) == 2 * 9 * 35 * 9 * 11 * 4
    assert B.conv_mcmk_check(db, B.DIRECT) == B.ERR_UNSUPPORTED


def test_compute_calls_validate_before_launch(lib):
    """NULL pointers and bad descriptors are refused on the host: no device is touched."""
    import ctypes
    d = B.desc(1, 4, 8, 8, 4, 3, 1)
    null = ctypes.c_void_p(0)
    for name in ("conv_mcmk_kn2row", "conv_mcmk_kn2row_2pass", "conv_mcmk_im2col", "conv_mcmk_direct",
                 "conv_mcmk_kn2col", "conv_mcmk_im2row"):
        fn = getattr(lib, name)
        assert fn(ctypes.byref(d), null, null, null, null, 0, null) == B.ERR_NULL
        bad = B.desc(1, 4, 8, 8, 4, 3, 1, dtype=5)
        assert fn(ctypes.byref(bad), null, null, null, null, 0, null) == B.ERR_UNSUPPORTED
        bad = B.desc(1, 4, 8, 8, 4, 3, 1, stride=0)
        assert fn(ctypes.byref(bad), null, null, null, null, 0, null) == B.ERR_SHAPE
    fake = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1004)
    assert lib.conv_mcmk_kn2row(ctypes.byref(d), odd, fake, fake, null, 0, null) == B.ERR_ALIGN
    assert lib.conv_mcmk_im2col(ctypes.byref(d), fake, fake, fake, null, 0, null) == B.ERR_WORKSPACE
    assert lib.conv_mcmk_kn2row_2pass(ctypes.byref(d), fake, fake, fake, fake, 16, null) == B.ERR_WORKSPACE
    assert lib.conv_mcmk_prepack(ctypes.byref(d), B.KN2ROW, null, null, null) == B.ERR_NULL
    assert lib.conv_mcmk_prepack(ctypes.byref(d), B.DIRECT, fake, fake, null) == B.ERR_UNSUPPORTED
    assert lib.conv_mcmk_cvt_f32_bf16(null, null, 4, null) == B.ERR_NULL
    # the epilogue and 1 x 1 entry points validate the same way
    for name in ("conv_mcmk_kn2row_bias_relu", "conv_mcmk_kn2col_bias_relu"):
        fn = getattr(lib, name)
        assert fn(ctypes.byref(d), null, null, null, 1, null, null) == B.ERR_NULL
        assert fn(ctypes.byref(d), fake, fake, ctypes.c_void_p(0x1002), 1, fake, null) == B.ERR_ALIGN      # bias: 4-byte aligned
        assert fn(ctypes.byref(B.desc(1, 4, 8, 8, 4, 3, 1, stride=3)), fake, fake, null, 0, fake, null) == B.ERR_UNSUPPORTED
    assert lib.conv_mcmk_1x1(ctypes.byref(d), fake, fake, fake, null) == B.ERR_UNSUPPORTED               # k = 3
    d1 = B.desc(1, 4, 8, 8, 4, 1, 0)
    assert lib.conv_mcmk_1x1(ctypes.byref(d1), null, fake, fake, null) == B.ERR_NULL
    assert lib.conv_mcmk_1x1(ctypes.byref(d1), fake, odd, fake, null) == B.ERR_ALIGN


def test_plan_selection_for_benchmark_layers(lib, monkeypatch):
    """The per-layer choice of the fused kernel (host logic only): the shapes measured fastest on
    the benchmark layers."""
    from paper_1704_04428_amd import workloads as wl
    B.conv_mcmk_force_tile(-1)
    want = {
        # single small images: quarter tiles, so that 4 x 16 (tiles x row blocks) becomes 256 workgroups
        "cfg3_alexnet_conv2": "tile 7x7, waves 1x4, row blocks 1, channel groups 1, channel split 1, 256 workgroups",
        "cfg2_googlenet5x5": "tile 7x7, waves 1x4, row blocks 1, channel groups 1, channel split 1, 96 workgroups",
        # one large image of few channels: single 14 x 14 tiles (36.9 us; the pair of tiles with two channel groups measures
        # 35.4 us but writes 1.6 x the output's bytes, and the estimate fitted to all layers puts the single tiles ahead)
        "cfg4_vgg_early": "tile 14x14, waves 4x2, row blocks 1, channel groups 1, channel split 1, 256 workgroups",
        # 56 x 56 images: pairs of tiles under sixteen waves, one workgroup per compute unit, 2 % padding instead of 6 %
        "cfg5a_vgg_deep56": "tile 14x28, waves 4x4, row blocks 1, channel groups 1, channel split 1, 256 workgroups",
        # 28 x 28 images: too few pairs for 64-row workgroups, so 32 rows and two channel groups of eight waves
        "cfg5b_vgg_deep28": "tile 14x28, waves 2x4, row blocks 1, channel groups 2, channel split 1, 256 workgroups",
        # 14x14 images: 64 tiles of 64 kernels cannot fill 256 CUs, so the contraction is split four ways
        "cfg5c_vgg_deep14": "tile 14x14, waves 1x4, row blocks 1, channel groups 4, channel split 1, 256 workgroups",
    }
    for name, text in want.items():
        L = wl.LAYERS[name]
        plan = B.conv_mcmk_describe_plan(B.desc(L.n, L.c, L.h, L.w, L.m, L.k, L.pad), B.KN2ROW)
        assert text in plan, (name, plan)
    # few channels, many tiles: every further workgroup of a CU costs a prologue and a closing write, so few
    # large workgroups beat many small ones (measured 241 us against 271 us, and 38.8 us against 42.4 us)
    assert "tile 14x28, waves 4x4" in B.conv_mcmk_describe_plan(B.desc(8, 64, 224, 224, 64, 3, 1), B.KN2ROW)
    assert "tile 14x14, waves 2x4, row blocks 1, channel groups 1, channel split 1, 256 workgroups" in \
        B.conv_mcmk_describe_plan(B.desc(1, 128, 112, 112, 128, 3, 1), B.KN2ROW)
    # a 1 x 1 kernel on 16 x 16 tiles: one position per staging thread (measured 16.9 us against 18.5 us on 14 x 14 tiles)
    assert "tile 16x16, waves 2x4" in B.conv_mcmk_describe_plan(B.desc(8, 256, 56, 56, 64, 1, 0), B.KN2ROW)
    # an RGB first layer: the instantiation with one channel quad (fp32, [C][H][W], k = 3 / 5 / 7, unit stride)
    assert "one channel quad" in B.conv_mcmk_describe_plan(B.desc(8, 3, 224, 224, 64, 7, 3), B.KN2ROW)
    assert "one channel quad" not in B.conv_mcmk_describe_plan(B.desc(8, 5, 224, 224, 64, 7, 3), B.KN2ROW)
    assert "one channel quad" in B.conv_mcmk_describe_plan(B.desc(8, 3, 224, 224, 64, 7, 3, stride=2), B.KN2ROW)
    assert "one channel quad" not in B.conv_mcmk_describe_plan(B.desc(8, 3, 224, 224, 64, 6, 3, stride=2), B.KN2ROW)
    assert "one channel quad" not in B.conv_mcmk_describe_plan(B.desc(8, 4, 224, 224, 64, 7, 3), B.KN2COL)
    d = B.desc(1, 8, 10, 10, 8, 3, 1)
    assert "shift-add" in B.conv_mcmk_describe_plan(d, B.KN2ROW_2PASS)
    assert "patch matrix [72 x 100]" in B.conv_mcmk_describe_plan(d, B.IM2COL)
    assert "800 outputs" in B.conv_mcmk_describe_plan(d, B.DIRECT)
    assert "patch matrix [100 x 72]" in B.conv_mcmk_describe_plan(d, B.IM2ROW)
    assert B.conv_mcmk_describe_plan(d, B.KN2COL).startswith("kn2col fused f32")
    with pytest.raises(B.ConvMcmkError):
        B.conv_mcmk_describe_plan(B.desc(1, 8, 10, 10, 8, 3, 1, stride=3), B.KN2ROW)
    # stride 2: 14 x 14 output tiles only, Q = P = 5 here
    assert "tile 14x14" in B.conv_mcmk_describe_plan(B.desc(1, 8, 10, 10, 8, 3, 1, stride=2), B.KN2ROW)
    B.conv_mcmk_force_tile(5)
    assert "tile 16x16, waves 1x4, row blocks 1, channel groups 1, channel split 1" in B.conv_mcmk_describe_plan(d, B.KN2ROW)
    assert "tile 14x14" in B.conv_mcmk_describe_plan(B.desc(1, 8, 10, 10, 8, 3, 1, stride=2), B.KN2ROW)   # 16 x 16: not with a stride
    B.conv_mcmk_force_tile(6)
    assert "channel groups 4" in B.conv_mcmk_describe_plan(d, B.KN2ROW)
    # bf16 operands on the deep 56 x 56 layer: two row blocks per wave; whole image rows for the [M][Q][P] output
    L = wl.LAYERS["cfg5a_vgg_deep56"]
    B.conv_mcmk_force_tile(-1)
    db = B.desc(L.n, L.c, L.h, L.w, L.m, L.k, L.pad, 1, B.BF16)
    assert "tile 4x56, waves 4x2, row blocks 2" in B.conv_mcmk_describe_plan(db, B.KN2ROW)
    assert "tile 14x14, waves 4x2, row blocks 2" in B.conv_mcmk_describe_plan(db, B.KN2COL)
    # a 1 x 1 layer with many tiles: no channel groups (they measured 24 us against 9.9 us on 16 x 16 tiles)
    plan = B.conv_mcmk_describe_plan(B.desc(8, 256, 56, 56, 64, 1, 0, 1, B.BF16), B.KN2ROW)
    assert "tile 16x16" in plan and "channel groups 1" in plan, plan
    B.conv_mcmk_force_tile(6)
    assert "channel groups 4" in B.conv_mcmk_describe_plan(B.desc(1, 8, 10, 10, 8, 3, 1, 1, B.BF16), B.KN2ROW)
    # an entry the kernel side does not have is ignored: the selector's own choice stands
    assert "channel groups 1" in B.conv_mcmk_describe_plan(B.desc(1, 8, 10, 10, 8, 5, 2), B.KN2ROW)


def test_image_size_limit_of_the_32_bit_offsets(lib):
    """The tile kernels address one image through 32-bit byte offsets and mark "outside the image" with an offset of
    2 GiB, to which a staging slot's channel (below 32) and the first chunk beyond the data (below C + 32) are still
    added: (C + 64) H W must stay below 2^29 elements, for every variant (the staged ones run their matrix product on
    the same kernels), and likewise (C k k + 64) Q P for the patch matrices."""
    at_limit = dict(n=1, c=64, h=2048, w=2048, m=1, k=3, pad=1)            # (64 + 64) * 2^22 == 2^29
    below = dict(at_limit, h=2047)
    for variant in (B.KN2ROW, B.KN2COL, B.KN2ROW_2PASS, B.DIRECT):
        assert B.conv_mcmk_check(B.desc(**at_limit), variant) == B.ERR_SHAPE, variant
        assert B.conv_mcmk_check(B.desc(**below), variant) == B.OK, variant
    patch_at_limit = dict(n=1, c=64, h=916, w=916, m=1, k=3, pad=1)        # (576 + 64) * 916^2 >= 2^29
    patch_below = dict(patch_at_limit, h=915)
    assert (576 + 64) * 916 * 916 >= 2 ** 29 > (576 + 64) * 915 * 916
    for variant in (B.IM2COL, B.IM2ROW):
        assert B.conv_mcmk_check(B.desc(**patch_at_limit), variant) == B.ERR_SHAPE, variant
        assert B.conv_mcmk_check(B.desc(**patch_below), variant) == B.OK, variant
    assert B.conv_mcmk_check(B.desc(**patch_at_limit), B.KN2ROW) == B.OK


def test_output_dims_entry_point(lib):
    """conv_mcmk_output_dims is where callers get Q and P from (the binding computes no sizes of its own)."""
    assert B.conv_mcmk_output_dims(B.desc(1, 3, 224, 224, 8, 7, 3, 2)) == (112, 112)
    assert B.conv_mcmk_output_dims(B.desc(2, 5, 9, 11, 7, 3, 0)) == (7, 9)
    assert B.conv_mcmk_output_dims(B.desc(1, 1, 5, 5, 1, 2, 1, 3)) == (2, 2)
    with pytest.raises(B.ConvMcmkError) as e:
        B.conv_mcmk_output_dims(B.desc(1, 1, 2, 2, 1, 5, 0))
    assert e.value.code == B.ERR_SHAPE
    assert lib.conv_mcmk_output_dims(None, None, None) == B.ERR_NULL


def test_kernel_register_budget():
    """The compiler's per-kernel report of the last build: no loop spills to scratch, and the 8-wave
    tile kernels stay within 128 vector registers (two workgroups per compute unit need that)."""
    from paper_1704_04428_amd import build
    usage = build.resource_usage()
    if not usage:
        pytest.skip("no compiler resource report beside the objects (library built elsewhere)")
    # register-to-register spills are fine, and so are a few registers' worth of scratch in the prologue of the
    # kernels that sit at the 256-register limit; anything beyond 64 bytes per lane means a loop is spilling
    spilling = {k: v for k, v in usage.items() if v.get("ScratchSize", 0) > 64}
    assert not spilling, spilling
    wide = [v for k, v in usage.items() if "kn2row_tile_f32ILi3ELi14ELi14ELi4ELi2ELi16E" in k and k.endswith("Li1ELi1ELi4ELb0EEEvNS_8TileArgsE")]
    assert len(wide) == 2                                   # unit stride, one channel group, all four channel quads: NCHW and channels-last
    assert all(v["VGPRs"] + v.get("AGPRs", 0) <= 128 for v in wide), wide


def test_variant_selection(lib, monkeypatch):
    """The per-layer choice among algorithms (host logic): the fused kernel wherever it applies, a
    staged variant where it does not, the workspace limit honoured."""
    import ctypes
    from paper_1704_04428_amd import workloads as wl
    B.conv_mcmk_force_tile(-1)
    for L in list(wl.LAYERS.values()) + list(wl.GENERALISED_LAYERS.values()):
        d = B.desc(L.n, L.c, L.h, L.w, L.m, L.k, L.pad, L.stride)
        variant, est = B.conv_mcmk_select(d)
        assert variant == B.KN2ROW and est > 0, L.name
        assert B.conv_mcmk_select(d, ws_limit_bytes=0)[0] == B.KN2ROW                # needs no workspace
        if L.c % 4 == 0:
            assert B.conv_mcmk_select(d, channels_last=True)[0] == B.KN2COL
    # a first-layer-like 11 x 11 kernel with stride 4: outside the fused kernels, so a staged variant;
    # the patch matrix is small (stride 4), the two-pass product is not
    big = B.desc(1, 3, 227, 227, 96, 11, 0, 4)
    assert B.conv_mcmk_select(big)[0] == B.IM2COL
    assert B.conv_mcmk_select(big, ws_limit_bytes=B.conv_mcmk_workspace_bytes(big, B.IM2COL) - 1)[0] == B.DIRECT
    assert B.conv_mcmk_select(B.desc(1, 4, 227, 227, 96, 11, 0, 4), channels_last=True)[0] == B.IM2ROW
    # bf16 operands, k = 9, no workspace allowed: nothing can run it
    with pytest.raises(B.ConvMcmkError) as e:
        B.conv_mcmk_select(B.desc(1, 8, 30, 30, 8, 9, 4, 1, B.BF16), ws_limit_bytes=0)
    assert e.value.code == B.ERR_WORKSPACE
    with pytest.raises(B.ConvMcmkError) as e:
        B.conv_mcmk_select(B.desc(1, 8, 0, 30, 8, 3, 1))
    assert e.value.code == B.ERR_SHAPE
    with pytest.raises(B.ConvMcmkError) as e:
        B.conv_mcmk_select(B.desc(1, 6, 30, 30, 8, 3, 1), channels_last=True)            # channel vectors of 4
    assert e.value.code == B.ERR_UNSUPPORTED
    out = ctypes.c_int(0)
    assert lib.conv_mcmk_select(None, 0, 0, ctypes.byref(out), None) == B.ERR_NULL
    assert lib.conv_mcmk_select(ctypes.byref(big), 0, 0, None, None) == B.ERR_NULL
    null = ctypes.c_void_p(0)
    assert lib.conv_mcmk_run(ctypes.byref(big), 17, null, null, null, null, 0, null) == B.ERR_UNSUPPORTED
    assert lib.conv_mcmk_run(ctypes.byref(big), B.IM2COL, null, null, null, null, 0, null) == B.ERR_NULL


def test_patch_workspace_follows_the_split_of_the_product(lib):
    """im2col / im2row ask for their patch matrix and, where the plan splits the contraction of their matrix product,
    for one copy of the result per part behind it (at the next multiple of 256 bytes); the two-pass form and the fused
    variants never ask for copies.  Host logic only: sizes against the plan text, over a few hundred layers."""
    import numpy as np
    rng = np.random.default_rng(77)
    seen_split = seen_plain = 0
    for _ in range(300):
        n = int(rng.choice([1, 2, 8])); c = int(rng.choice([8, 16, 64, 96, 256, 512])); m = int(rng.choice([16, 35, 64, 256, 512]))
        h = int(rng.choice([7, 13, 14, 28, 56])); w = int(rng.choice([7, 14, 27, 56])); k = int(rng.choice([1, 3, 5])); pad = k // 2
        for dtype, elt in ((B.F32, 4), (B.BF16, 2)):
            d = B.desc(n, c, h, w, m, k, pad, 1, dtype)
            for variant in (B.IM2COL, B.IM2ROW):
                if B.conv_mcmk_check(d, variant) != B.OK:
                    continue
                plan = B.conv_mcmk_describe_plan(d, variant)
                parts = int(plan.split("channel split ")[1].split(",")[0])
                matrix = n * c * k * k * h * w * elt
                copies = (n * m * h * w + 3) // 4 * 16
                want = matrix if parts == 1 else (matrix + 255) // 256 * 256 + parts * copies
                assert B.conv_mcmk_workspace_bytes(d, variant) == want, (plan, want)
                seen_split += parts > 1
                seen_plain += parts == 1
            if B.conv_mcmk_check(d, B.KN2ROW_2PASS) == B.OK:
                assert B.conv_mcmk_workspace_bytes(d, B.KN2ROW_2PASS) == n * k * k * m * h * w * 4
            assert B.conv_mcmk_workspace_bytes(d, B.KN2ROW) == 0
    assert seen_split > 50 and seen_plain > 50, (seen_split, seen_plain)
