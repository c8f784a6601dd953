"""CPU-side checks of the C ABI: the library loads, exports every symbol the header
declares, and rejects bad arguments before launching anything (no GPU needed)."""
import ctypes
import os
import re

import pytest

from paper_2601_11660_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_symbols():
    txt = open(os.path.join(ROOT, "include", "mbu.h")).read()
    txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
    return sorted(set(re.findall(r"\b(mbu_[a-z0-9_]+)\s*\(", txt)))


def test_library_exports_every_declared_symbol():
    L = B.lib()
    syms = header_symbols()
    assert len(syms) >= 25
    for s in syms:
        assert hasattr(L, s), s
    assert sorted(B.EXPORTS) == syms


def test_null_and_alignment_errors():
    L = B.lib()
    assert L.mbu_pack_act(None, 0, 1, 4, 4, 32, None, None) == B.MBU_ERR_NULL
    assert "NULL" in B.last_error()
    fake, fake2 = 0x10000, 0x20000    # never dereferenced: validation fails first
    assert L.mbu_pack_act(fake, 0, 1, 4, 4, 32, fake2 + 4, None) == B.MBU_ERR_ALIGN
    assert L.mbu_pack_act(fake, 7, 1, 4, 4, 32, fake2, None) == B.MBU_ERR_ARG
    assert L.mbu_pack_act(fake, 0, 0, 4, 4, 32, fake2, None) == B.MBU_ERR_SHAPE
    assert L.mbu_maxpool2x2_bits(fake, 1, 1, 4, 32, fake2, None) == B.MBU_ERR_SHAPE
    assert L.mbu_maxpool2x2_bits(fake, 1, 4, 4, 32, None, None) == B.MBU_ERR_NULL
    assert L.mbu_upsample2x_bits(None, 1, 4, 4, 32, fake2, None) == B.MBU_ERR_NULL
    assert L.mbu_concat_bits(fake, 48, fake2, 32, 1, 4, 4, fake, None) == B.MBU_ERR_SHAPE
    assert L.mbu_pack_weights(None, 64, 64, fake, None) == B.MBU_ERR_NULL
    assert L.mbu_pack_weights(fake, 48, 64, fake2, None) == B.MBU_ERR_SHAPE


def test_conv_argument_validation():
    L = B.lib()
    a, w, t, o = 0x10000, 0x20000, 0x30000, 0x40000
    f = L.mbu_conv3x3_masked_binary
    assert f(a, 1, 8, 8, 64, w, 64, t, None, None, None) == B.MBU_ERR_NULL
    assert f(a, 1, 8, 8, 64, w, 48, t, o, None, None) == B.MBU_ERR_SHAPE
    assert f(a, 1, 8, 0, 64, w, 64, t, o, None, None) == B.MBU_ERR_SHAPE
    assert f(a, 1, 8, 8, 64, w, 64, t, a, None, None) == B.MBU_ERR_ARG
    assert f(a, 1, 8, 8, 64, w, 64, t + 8, o, None, None) == B.MBU_ERR_ALIGN
    assert f(None, 1, 8, 8, 64, w, 64, t, o, None, None) == B.MBU_ERR_NULL


def test_fused_conv_argument_validation():
    L = B.lib()
    a, lo, w, t, o, p = 0x10000, 0x20000, 0x30000, 0x40000, 0x50000, 0x60000
    f = L.mbu_conv3x3_masked_binary_fused
    assert f(a, 64, lo, 128, 1, 8, 8, w, 64, t, None, None, None) == B.MBU_ERR_NULL
    assert f(a, 64, None, 128, 1, 8, 8, w, 64, t, o, None, None) == B.MBU_ERR_SHAPE
    assert f(a, 64, lo, 0, 1, 8, 8, w, 64, t, o, None, None) == B.MBU_ERR_SHAPE
    assert f(a, 48, lo, 128, 1, 8, 8, w, 64, t, o, None, None) == B.MBU_ERR_SHAPE
    assert f(a, 64, lo, 128, 1, 1, 8, w, 64, t, o, None, None) == B.MBU_ERR_SHAPE
    assert f(a, 64, None, 0, 1, 1, 8, w, 64, t, o, p, None) == B.MBU_ERR_SHAPE     # no 2x2 window
    assert f(a, 64, None, 0, 1, 8, 1, w, 64, t, o, p, None) == B.MBU_ERR_SHAPE
    assert f(a, 64, lo, 128, 1, 8, 8, w, 64, t, lo, None, None) == B.MBU_ERR_ARG
    assert f(a, 64, lo + 4, 128, 1, 8, 8, w, 64, t, o, None, None) == B.MBU_ERR_ALIGN


def test_tconv_and_concat_argument_validation():
    L = B.lib()
    a, b, w, t, o = 0x10000, 0x20000, 0x30000, 0x40000, 0x50000
    f = L.mbu_tconv2x2_masked_binary
    assert f(a, 1, 4, 4, 64, w, 64, t, None, None, None) == B.MBU_ERR_NULL
    assert f(a, 1, 4, 4, 64, w, 48, t, o, None, None) == B.MBU_ERR_SHAPE
    assert f(a, 1, 0, 4, 64, w, 64, t, o, None, None) == B.MBU_ERR_SHAPE
    assert f(a, 1, 4, 4, 64, w, 64, t, a, None, None) == B.MBU_ERR_ARG
    assert f(a, 1, 4, 4, 64, w + 2, 64, t, o, None, None) == B.MBU_ERR_ALIGN
    n = ctypes.c_size_t()
    assert L.mbu_packed_tconv_weights_bytes(64, 128, ctypes.byref(n)) == 0
    assert n.value >= 4 * 64 * 128 // 2
    assert L.mbu_packed_tconv_weights_bytes(40, 128, ctypes.byref(n)) == B.MBU_ERR_SHAPE
    assert L.mbu_pack_tconv_weights(None, 64, 64, o, None) == B.MBU_ERR_NULL
    g = L.mbu_conv3x3_masked_binary_concat
    assert g(a, 64, None, 64, 1, 8, 8, w, 64, t, o, None, None) == B.MBU_ERR_NULL
    assert g(a, 48, b, 64, 1, 8, 8, w, 64, t, o, None, None) == B.MBU_ERR_SHAPE
    assert g(a, 64, b, 64, 1, 8, 8, w, 64, t, b, None, None) == B.MBU_ERR_ARG
    assert g(a, 64, b, 0, 1, 8, 8, w, 64, t, o, None, None) == B.MBU_ERR_SHAPE
    h = L.mbu_conv3x3_masked_binary_two_inputs
    assert h(a, 64, None, 64, 4, 4, 1, 1, 9, 9, w, 64, t, o, None, None) == B.MBU_ERR_NULL
    assert h(a, 64, b, 64, 5, 4, 1, 1, 9, 9, w, 64, t, o, None, None) == B.MBU_ERR_SHAPE   # 2*5 > 9
    assert h(a, 64, b, 64, 9, 10, 0, 1, 9, 9, w, 64, t, o, None, None) == B.MBU_ERR_SHAPE
    assert h(a, 64, b, 64, 0, 4, 1, 1, 9, 9, w, 64, t, o, None, None) == B.MBU_ERR_SHAPE
    assert h(a, 64, b, 64, 4, 4, 2, 1, 9, 9, w, 64, t, o, None, None) == B.MBU_ERR_ARG
    assert h(a, 48, b, 64, 4, 4, 1, 1, 9, 9, w, 64, t, o, None, None) == B.MBU_ERR_SHAPE
    assert h(a, 64, b, 64, 1, 1, 0, 1, 1, 9, w, 64, t, o, a + 64, None) == B.MBU_ERR_SHAPE  # pool, H = 1
    assert h(a, 64, b, 64, 4, 4, 1, 1, 9, 9, w, 64, t, b, None, None) == B.MBU_ERR_ARG


def test_unet_plan_with_transposed_decoder():
    from paper_2601_11660_amd import synth
    plan = synth.unet_channel_plan(64, 4, transposed=True)
    d = _desc(convs=[(ci, co) for _, ci, co, _ in plan])
    ups = (B.ConvLayer * 4)()
    for i, c in enumerate((512, 256, 128, 64)):
        ups[i].cin, ups[i].cout = 2 * c, c
        ups[i].packed_w, ups[i].thresh = 0x10000, 0x20000
    d.up_convs = ups
    L = B.lib()
    assert L.mbu_unet_num_steps(ctypes.byref(d)) == 32
    n = ctypes.c_size_t()
    assert L.mbu_unet_workspace_bytes(ctypes.byref(d), 1, 64, 128, ctypes.byref(n)) == 0
    names = []
    for s in range(32):
        name = ctypes.c_char_p()
        assert L.mbu_unet_step_info(ctypes.byref(d), 1, 64, 128, s, ctypes.byref(name), None, None,
                                    None, None) == 0
        names.append(name.value.decode())
    assert names[15:19] == ["up4", "cat4", "dec4a", "dec4b"]
    ups[1].cin = 300
    assert L.mbu_unet_workspace_bytes(ctypes.byref(d), 1, 64, 128, ctypes.byref(n)) == B.MBU_ERR_SHAPE


def test_packed_weight_size_and_path_switch():
    assert B.packed_weights_bytes(64, 64) > 2 * 9 * 64 * 64 // 8
    # optional sections: each one adds its size, the matrix fragments are always there
    full = B.packed_weights_bytes(512, 1536)
    lean = B.packed_weights_bytes(512, 1536, B.BLOB_MATRIX)
    assert B.packed_weights_bytes(512, 1536, 0) == lean and B.packed_weights_bytes(512, 1536, B.BLOB_ALL) == full
    planes = B.packed_weights_bytes(512, 1536, B.BLOB_BIT_PLANES) - lean
    taps = B.packed_weights_bytes(512, 1536, B.BLOB_SUMMED_TAPS) - lean
    assert planes >= 2 * 9 * 1536 * 512 // 8 and taps >= 16 * 1536 * 512 // 2 and lean + planes + taps == full
    assert lean >= 9 * 1536 * 512 // 2 and lean < 0.4 * full
    n_ = ctypes.c_size_t()
    assert B.lib().mbu_packed_weights_bytes_sections(64, 64, 8, ctypes.byref(n_)) == B.MBU_ERR_ARG
    assert B.lib().mbu_pack_weights_sections(0x10000, 64, 64, 16, 0x20000, None) == B.MBU_ERR_ARG
    with pytest.raises(B.MbuError):
        B.packed_weights_bytes(40, 64)
    n = ctypes.c_size_t()
    assert B.lib().mbu_packed_weights_bytes(64, 64, None) == B.MBU_ERR_NULL
    assert B.lib().mbu_set_conv_path(9) == B.MBU_ERR_ARG
    assert B.lib().mbu_set_conv_tuning(5, 0) == B.MBU_ERR_ARG
    assert B.lib().mbu_set_conv_tuning(3, 1) == B.MBU_ERR_ARG
    for k in (1, 3, 6, 7, 8, 9):
        assert B.lib().mbu_set_conv_tuning(k, 0) == 0
    assert B.lib().mbu_set_conv_tuning(10, 0) == B.MBU_ERR_ARG
    assert B.lib().mbu_set_conv_tuning(0, 0) == 0
    B.set_conv_path(B.PATH_VALU)
    assert B.get_conv_path() == B.PATH_VALU
    B.set_conv_path(B.PATH_AUTO)


def _desc(levels=4, base=64, convs=None):
    d = B.UNetDesc(levels=levels, base=base, in_channels=3, n_classes=19)
    if convs is not None:
        arr = (B.ConvLayer * len(convs))()
        for i, (ci, co) in enumerate(convs):
            arr[i].cin, arr[i].cout = ci, co
            arr[i].packed_w, arr[i].thresh = 0x10000, 0x20000
        d.convs = arr
        d._keep = arr
    return d


def test_unet_plan_validation_and_workspace():
    from paper_2601_11660_amd import synth
    plan = synth.unet_channel_plan(64, 4)
    d = _desc(convs=[(ci, co) for _, ci, co, _ in plan])
    L = B.lib()
    assert L.mbu_unet_num_steps(ctypes.byref(d)) == 28
    n = ctypes.c_size_t()
    assert L.mbu_unet_workspace_bytes(ctypes.byref(d), 1, 64, 128, ctypes.byref(n)) == 0
    # every step's packed output, 256-byte aligned regions
    expect = 0
    names = []
    for s in range(27):
        name = ctypes.c_char_p()
        off = ctypes.c_size_t()
        h, w, c = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
        assert L.mbu_unet_step_info(ctypes.byref(d), 1, 64, 128, s, ctypes.byref(name),
                                    ctypes.byref(off), ctypes.byref(h), ctypes.byref(w),
                                    ctypes.byref(c)) == 0
        assert off.value == expect
        expect += (h.value * w.value * (c.value // 32) * 4 + 255) // 256 * 256
        names.append(name.value.decode())
    assert n.value == expect
    assert names[:4] == ["stem", "enc1a", "enc1b", "pool1"] and names[15:19] == ["cat4", "dec4a", "dec4b", "cat3"]
    # sizes that are not multiples of 16: pooling rounds down, the decoder pads back up
    assert L.mbu_unet_workspace_bytes(ctypes.byref(d), 1, 75, 131, ctypes.byref(n)) == 0
    sizes = {}
    for s in range(28):
        name = ctypes.c_char_p()
        h, w = ctypes.c_int(), ctypes.c_int()
        assert L.mbu_unet_step_info(ctypes.byref(d), 1, 75, 131, s, ctypes.byref(name), None,
                                    ctypes.byref(h), ctypes.byref(w), None) == 0
        sizes[name.value.decode()] = (h.value, w.value)
    assert sizes["pool1"] == (37, 65) and sizes["pool2"] == (18, 32) and sizes["pool4"] == (4, 8)
    assert sizes["cat4"] == (9, 16) and sizes["cat2"] == (37, 65) and sizes["classifier"] == (75, 131)
    assert L.mbu_unet_workspace_bytes(ctypes.byref(d), 1, 15, 128, ctypes.byref(n)) == B.MBU_ERR_SHAPE
    # which kernel a step launches, and which steps launch none (no GPU needed: nothing runs)
    d.fuse = 1
    kern = {}
    for s in range(28):
        k = ctypes.c_char_p()
        assert L.mbu_unet_step_kernel(ctypes.byref(d), 1, 1024, 2048, s, ctypes.byref(k)) == 0
        kern[names[s] if s < 27 else "classifier"] = k.value.decode()
    assert kern["stem"] == "stem_rows_kernel" and kern["classifier"].startswith("classifier_kernel")
    assert kern["enc1a"] == "conv_mfma_rows_kernel" and kern["dec1a"] == "conv_mfma_upcat_kernel"
    assert kern["enc4b"] == "conv_mfma_block_kernel" and kern["cat1"] == "" and kern["pool1"] == ""
    k = ctypes.c_char_p()
    assert L.mbu_unet_step_kernel(ctypes.byref(d), 1, 75, 131, 25, ctypes.byref(k)) == 0   # dec1a, padded
    assert k.value.decode() == "conv_mfma_block_kernel"
    assert L.mbu_unet_step_kernel(ctypes.byref(d), 1, 64, 128, 99, ctypes.byref(k)) == B.MBU_ERR_ARG
    d.fuse = 0
    # inconsistent channel plan
    bad = [(ci, co) for _, ci, co, _ in plan]
    bad[10] = (1024, 512)
    d2 = _desc(convs=bad)
    assert L.mbu_unet_workspace_bytes(ctypes.byref(d2), 1, 64, 128, ctypes.byref(n)) == B.MBU_ERR_SHAPE
    assert "layer 10" in B.last_error()
    # forward: workspace too small / NULL image are caught before any launch
    assert L.mbu_unet_forward(ctypes.byref(d), None, 1, 64, 128, 0x50000, 0x60000, 1 << 40, None) == B.MBU_ERR_NULL
    d.stem_w, d.cls_w, d.cls_b = 0x70000, 0x80000, 0x90000
    assert L.mbu_unet_forward(ctypes.byref(d), 0x40000, 1, 64, 128, 0x50000, 0x60000, 16, None) == B.MBU_ERR_WORKSPACE


def test_stem_and_classifier_argument_validation():
    L = B.lib()
    img, w, o, p = 0x10000, 0x20000, 0x30000, 0x40000
    f = L.mbu_stem_fp32
    assert f(None, 1, 3, 8, 8, w, 64, o, None, None) == B.MBU_ERR_NULL
    assert f(img, 1, 3, 8, 8, w, 64, None, p, None) == B.MBU_ERR_NULL
    assert f(img, 1, 2, 8, 8, w, 64, o, None, None) == B.MBU_ERR_SHAPE
    assert f(img, 1, 3, 8, 8, w, 48, o, None, None) == B.MBU_ERR_SHAPE
    assert f(img, 1, 3, 0, 8, w, 64, o, None, None) == B.MBU_ERR_SHAPE
    assert f(img, 1, 3, 8, 8, w, 64, o, p + 4, None) == B.MBU_ERR_ALIGN
    assert f(img, 64, 3, 4096, 4096, w, 64, o, None, None) == B.MBU_ERR_SHAPE     # > 2 GiB image
    assert L.mbu_set_stem_path(9) == B.MBU_ERR_ARG
    assert L.mbu_set_stem_path(B.STEM_VALU) == B.MBU_OK and L.mbu_get_stem_path() == B.STEM_VALU
    assert L.mbu_set_stem_path(B.STEM_MFMA_GATHER) == B.MBU_OK and L.mbu_get_stem_path() == B.STEM_MFMA_GATHER
    assert L.mbu_set_stem_path(B.STEM_AUTO) == B.MBU_OK
    g = L.mbu_classifier_fp32
    a, b = 0x50000, 0x60000
    assert g(None, 1, 8, 8, 64, w, b, 19, o, None) == B.MBU_ERR_NULL
    assert g(a, 1, 8, 8, 96, w, b, 19, o, None) == B.MBU_ERR_SHAPE
    assert g(a, 1, 8, 8, 64, w, b, 33, o, None) == B.MBU_ERR_SHAPE
    assert g(a, 1, 8, 8, 64, w, b + 4, 19, o, None) == B.MBU_ERR_ALIGN
