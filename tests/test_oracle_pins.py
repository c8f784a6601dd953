"""Pins for the CPU oracle: everything here runs without a GPU and checks the oracle
against things other than itself - brute force in a different formulation, the paper's
bit identities (Eq. 1, Eq. 2 / Algorithm 1), closed forms, invariants and PyTorch-CPU
float64 library routines."""
import itertools

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import oracle as O
from paper_2601_11660_amd import synth
from tests import bitref


def rand_case(seed, N, H, W, Cin, Cout, keep=0.6):
    c = synth.conv_case(99, seed, N, H, W, Cin, Cout, keep)
    return c.a, c.w, c.theta


# ---------------------------------------------------------------- brute force
def scatter_conv(a, w):
    """Independent formulation: explicit zero-padded input, and every (input pixel,
    weight) pair *scatters* its product to the output it belongs to (pure Python)."""
    N, H, W, Cin = a.shape
    Cout = w.shape[0]
    out = np.zeros((N, H, W, Cout), np.int64)
    for n in range(N):
        for yi in range(H):
            for xi in range(W):
                for ky in range(3):
                    for kx in range(3):
                        yo, xo = yi - (ky - 1), xi - (kx - 1)
                        if 0 <= yo < H and 0 <= xo < W:
                            for o in range(Cout):
                                for c in range(Cin):
                                    out[n, yo, xo, o] += int(w[o, ky, kx, c]) * int(a[n, yi, xi, c])
    return out


def test_bruteforce_all_activation_patterns_3x3_single_channel():
    rng = np.random.default_rng(1)
    ws = rng.integers(-1, 2, size=(6, 1, 3, 3, 1), dtype=np.int8)
    for bits in itertools.product((-1, 1), repeat=9):
        a = np.array(bits, np.int8).reshape(1, 3, 3, 1)
        for w in ws[:2]:
            assert np.array_equal(O.conv3x3(a, w), scatter_conv(a, w))
    # all 3^9 ternary kernels against one fixed activation pattern, centre output
    a = np.array([1, -1, 1, 1, 1, -1, -1, 1, -1], np.int8).reshape(1, 3, 3, 1)
    for k in itertools.product((-1, 0, 1), repeat=9):
        w = np.array(k, np.int8).reshape(1, 3, 3, 1)
        expect = sum(int(x) * int(y) for x, y in zip(k, a.ravel()))
        assert int(O.conv3x3(a, w)[0, 1, 1, 0]) == expect


@pytest.mark.parametrize("H,W,Cin,Cout", [(4, 5, 3, 2), (3, 3, 2, 1), (1, 1, 5, 3),
                                          (2, 7, 1, 4), (5, 1, 2, 2)])
def test_bruteforce_small_ragged(H, W, Cin, Cout):
    for seed in range(3):
        a, w, _ = rand_case(seed, 2, H, W, Cin, Cout)
        assert np.array_equal(O.conv3x3(a, w), scatter_conv(a, w))


# ------------------------------------------------ library special case (torch)
@pytest.mark.parametrize("N,H,W,Cin,Cout", [(1, 17, 23, 40, 24), (2, 8, 8, 64, 64),
                                            (1, 33, 9, 96, 32)])
def test_conv_equals_torch_float64(N, H, W, Cin, Cout):
    a, w, _ = rand_case(5, N, H, W, Cin, Cout)
    ref = F.conv2d(torch.from_numpy(a).double().permute(0, 3, 1, 2),
                   torch.from_numpy(w).double().permute(0, 3, 1, 2), padding=1)
    ref = ref.permute(0, 2, 3, 1).numpy()
    acc = O.conv3x3(a, w)
    assert np.array_equal(acc.astype(np.float64), ref)


def test_points_equal_full():
    a, w, _ = rand_case(6, 2, 9, 11, 32, 8)
    acc = O.conv3x3(a, w)
    rng = np.random.default_rng(0)
    pts = np.stack([rng.integers(0, 2, 200), rng.integers(0, 9, 200),
                    rng.integers(0, 11, 200), rng.integers(0, 8, 200)], 1).astype(np.int32)
    got = O.conv3x3_points(a, w, pts)
    assert np.array_equal(got, acc[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]])


# ------------------------------------------------------ orientation / indexing
def test_single_tap_is_a_shifted_copy():
    """One non-zero weight at (o, ky, kx, c) = s  =>  out[..., o] is channel c shifted
    by (ky-1, kx-1) and scaled by s, zero where the source is outside the image.
    Pins cross-correlation orientation and the OHWI index order."""
    a, _, _ = rand_case(7, 1, 6, 7, 5, 3)
    for (o, ky, kx, c, s) in [(0, 0, 0, 1, 1), (1, 2, 1, 4, -1), (2, 1, 2, 0, 1), (0, 2, 0, 3, -1)]:
        w = np.zeros((3, 3, 3, 5), np.int8)
        w[o, ky, kx, c] = s
        acc = O.conv3x3(a, w)
        exp = np.zeros((6, 7), np.int32)
        for y in range(6):
            for x in range(7):
                yy, xx = y + ky - 1, x + kx - 1
                if 0 <= yy < 6 and 0 <= xx < 7:
                    exp[y, x] = s * a[0, yy, xx, c]
        assert np.array_equal(acc[0, :, :, o], exp)
        others = [k for k in range(3) if k != o]
        assert not acc[0][:, :, others].any()


# ------------------------------------------------------------ paper identities
def test_eq1_xnor_popcount_all_small_vectors():
    for n in range(1, 7):
        for abits in range(1 << n):
            for bbits in range(1 << n):
                a = [1 if (abits >> i) & 1 else -1 for i in range(n)]
                b = [1 if (bbits >> i) & 1 else -1 for i in range(n)]
                assert bitref.dot_xnor(abits, bbits, n) == sum(x * y for x, y in zip(a, b))


def test_eq2_two_plane_identity_and_its_constant():
    """Eq. 2: with b = b_pos - b_neg the dot product is popc(a'^b_neg) - popc(a'^b_pos),
    as Algorithm 1 computes it (R = C_neg - C_pos, no additive n).  The printed closed
    form carries an extra '+ n'; this test shows that reading is off by exactly n."""
    for n in range(1, 5):
        for abits in range(1 << n):
            for tern in itertools.product((-1, 0, 1), repeat=n):
                a = [1 if (abits >> i) & 1 else -1 for i in range(n)]
                pos = bitref.to_int([t == 1 for t in tern])
                neg = bitref.to_int([t == -1 for t in tern])
                true = sum(x * y for x, y in zip(a, tern))
                assert bitref.dot_two_planes(abits, pos, neg) == true
                assert n + bitref.dot_two_planes(abits, pos, neg) == true + n
                # sign/mask form: W = pos plane, M = pos | neg
                assert bitref.dot_sign_mask(abits, pos, pos | neg) == true


def packed_conv_reference(a, w):
    """Evaluate the layer through the bit formulas (Eq. 2 / sign-mask form) on packed
    words with out-of-image taps removed from the mask."""
    N, H, W, Cin = a.shape
    Cout = w.shape[0]
    A = bitref.pack_pm1(a)
    pos = bitref.pack_pm1(np.where(w == 1, 1, -1))
    neg = bitref.pack_pm1(np.where(w == -1, 1, -1))
    out = np.zeros((N, H, W, Cout), np.int64)
    for n in range(N):
        for y in range(H):
            for x in range(W):
                for o in range(Cout):
                    s = 0
                    for ky in range(3):
                        for kx in range(3):
                            yy, xx = y + ky - 1, x + kx - 1
                            if not (0 <= yy < H and 0 <= xx < W):
                                continue
                            for k in range(A.shape[-1]):
                                av, p, g = int(A[n, yy, xx, k]), int(pos[o, ky, kx, k]), int(neg[o, ky, kx, k])
                                m = p | g
                                v1 = bitref.popc(m) - 2 * bitref.popc((p ^ av) & m)
                                v2 = bitref.popc((av ^ g) & m) - bitref.popc((av ^ p) & m)
                                assert v1 == v2
                                s += v1
                    out[n, y, x, o] = s
    return out


@pytest.mark.parametrize("Cin", [32, 40, 64, 96])
def test_popcount_identity_matches_plain_sum(Cin):
    a, w, _ = rand_case(11, 1, 4, 5, Cin, 3, keep=0.5)
    assert np.array_equal(O.conv3x3(a, w), packed_conv_reference(a, w))


# ------------------------------------------------------------------ invariants
def test_all_zero_mask_gives_zero_and_threshold_of_zero():
    a, w, th = rand_case(12, 1, 8, 8, 64, 16)
    acc, out = O.masked_binary_layer(a, np.zeros_like(w), th)
    assert not acc.any()
    assert np.array_equal(out[0, 0, 0], np.where(0 >= th, 1, -1))


def test_full_mask_reduces_to_xnor_popcount():
    rng = np.random.default_rng(3)
    a = synth.pm1_bits(rng, (1, 6, 6, 64))
    w = synth.pm1_bits(rng, (4, 3, 3, 64))
    acc = O.conv3x3(a, w)
    A, Wb = bitref.pack_pm1(a), bitref.pack_pm1(w)
    for (y, x) in [(0, 0), (3, 3), (5, 2), (0, 5)]:
        for o in range(4):
            s = 0
            for ky in range(3):
                for kx in range(3):
                    yy, xx = y + ky - 1, x + kx - 1
                    if 0 <= yy < 6 and 0 <= xx < 6:
                        for k in range(2):
                            s += bitref.dot_xnor(int(A[0, yy, xx, k]), int(Wb[o, ky, kx, k]), 32)
            assert acc[0, y, x, o] == s


def test_negation_additivity_parity_and_bound():
    a, w, _ = rand_case(13, 1, 7, 9, 48, 8, keep=0.5)
    acc = O.conv3x3(a, w)
    assert np.array_equal(O.conv3x3(-a, w), -acc)
    assert np.array_equal(O.conv3x3(a, -w), -acc)
    # additivity over disjoint masks
    rng = np.random.default_rng(4)
    split = rng.random(w.shape) < 0.5
    w1, w2 = w * split, w * ~split
    assert np.array_equal(O.conv3x3(a, w1.astype(np.int8)) + O.conv3x3(a, w2.astype(np.int8)), acc)
    # |acc| <= number of kept in-image taps, same parity
    ones = np.ones_like(a)
    kept = O.conv3x3(ones, np.abs(w).astype(np.int8))
    assert (np.abs(acc) <= kept).all()
    assert ((acc - kept) % 2 == 0).all()
    # a layer of all-(+1) weights on all-(+1) input counts in-image taps: 4/6/9 * Cin
    cnt = O.conv3x3(ones, np.ones_like(w))
    assert cnt[0, 0, 0, 0] == 4 * 48 and cnt[0, 0, 3, 0] == 6 * 48 and cnt[0, 3, 3, 0] == 9 * 48


def test_interior_translation_equivariance():
    a, w, _ = rand_case(14, 1, 10, 12, 32, 4)
    acc = O.conv3x3(a, w)
    a2 = np.roll(a, (2, 3), axis=(1, 2))
    acc2 = O.conv3x3(a2, w)
    assert np.array_equal(acc2[0, 4:9, 5:11], acc[0, 2:7, 2:8])


def test_threshold_tie_goes_to_plus_one():
    a, w, _ = rand_case(15, 1, 5, 5, 32, 6)
    acc = O.conv3x3(a, w)
    th = acc[0, 2, 2].copy()
    out = O.threshold(acc, th)
    assert (out[0, 2, 2] == 1).all()
    out2 = O.threshold(acc, th + 1)
    assert (out2[0, 2, 2] == -1).all()
    assert np.array_equal(out, np.where(acc >= th, 1, -1))


def test_fast_packing_helper_equals_the_plain_one():
    """tests/bitref.pack_pm1_fast (numpy packbits, used on full-size tensors) gives the words of
    pack_pm1 (explicit sum of bit * 2^i), including on hand-built words."""
    rng = np.random.default_rng(3)
    for C in (32, 64, 96, 512):
        a = synth.pm1_bits(rng, (2, 3, 5, C))
        assert np.array_equal(bitref.pack_pm1_fast(a), bitref.pack_pm1(a))
    one = -np.ones((1, 64), np.int8)
    one[0, 0] = one[0, 31] = one[0, 33] = 1
    assert bitref.pack_pm1_fast(one).tolist() == [[0x80000001, 0x00000002]]


# ------------------------------------------------------------------------ glue
def test_pool_upsample_concat_match_torch():
    rng = np.random.default_rng(5)
    a = synth.pm1_bits(rng, (2, 6, 8, 40))
    b = synth.pm1_bits(rng, (2, 6, 8, 24))
    t = torch.from_numpy(a).double().permute(0, 3, 1, 2)
    assert np.array_equal(O.maxpool2x2(a),
                          F.max_pool2d(t, 2).permute(0, 2, 3, 1).numpy().astype(np.int8))
    assert np.array_equal(O.upsample2x(a),
                          F.interpolate(t, scale_factor=2, mode="nearest").permute(0, 2, 3, 1).numpy().astype(np.int8))
    assert np.array_equal(O.concat(a, b), np.concatenate([a, b], -1))


def test_pool_is_or_on_bits_all_16_cases():
    for bits in itertools.product((-1, 1), repeat=4):
        a = np.array(bits, np.int8).reshape(1, 2, 2, 1)
        assert O.maxpool2x2(a)[0, 0, 0, 0] == (1 if any(b == 1 for b in bits) else -1)


# ---------------------------------------------------------------- float layers
def test_stem_against_float64():
    rng = np.random.default_rng(6)
    img = rng.standard_normal((2, 3, 9, 13), dtype=np.float32)
    w = rng.standard_normal((8, 3, 3, 3), dtype=np.float32)
    pre, sgn = O.stem(img, w)
    wt = torch.from_numpy(w).double().permute(0, 3, 1, 2)
    ref = F.conv2d(torch.from_numpy(img).double(), wt, padding=1).permute(0, 2, 3, 1).numpy()
    mag = F.conv2d(torch.from_numpy(img).double().abs(), wt.abs(), padding=1).permute(0, 2, 3, 1).numpy()
    assert (np.abs(pre - ref) <= 1e-6 * mag + 1e-30).all()
    assert np.allclose(pre, ref, rtol=1e-4, atol=1e-5)
    clear = np.abs(ref) > 1e-5 * mag
    assert np.array_equal(sgn[clear], np.where(ref >= 0, 1, -1)[clear])
    assert np.array_equal(sgn, np.where(pre >= 0, 1, -1))
    # exact tie: a zero image gives pre == 0 everywhere and binarises to +1
    _, s0 = O.stem(np.zeros_like(img), w)
    assert (s0 == 1).all()


def test_classifier_against_float64():
    rng = np.random.default_rng(7)
    a = synth.pm1_bits(rng, (2, 5, 6, 64))
    w = (rng.standard_normal((19, 64), dtype=np.float32) / np.float32(8))
    b = rng.standard_normal((19,), dtype=np.float32)
    out = O.classifier(a, w, b)
    ref = F.conv2d(torch.from_numpy(a).double().permute(0, 3, 1, 2),
                   torch.from_numpy(w).double()[:, :, None, None],
                   torch.from_numpy(b).double()).numpy()
    assert out.shape == (2, 19, 5, 6)
    assert (np.abs(out - ref) <= 1e-4 * np.maximum(1.0, np.abs(ref))).all()


# ----------------------------------------------------------------------- U-Net
def torch_unet(case):
    """The same network recomposed from PyTorch-CPU float64 library ops."""
    def t(a):
        return torch.from_numpy(np.ascontiguousarray(a)).double()
    x = F.conv2d(t(case.image), t(case.stem_w).permute(0, 3, 1, 2), padding=1)
    x = torch.where(x >= 0, 1.0, -1.0).double()
    it = iter(case.convs)

    def dconv(x):
        for _ in range(2):
            w, th = next(it)
            acc = F.conv2d(x, t(w).permute(0, 3, 1, 2), padding=1)
            x = torch.where(acc >= t(th)[None, :, None, None], 1.0, -1.0).double()
        return x
    skips = []
    for _ in range(case.levels):
        x = dconv(x)
        skips.append(x)
        x = F.max_pool2d(x, 2)
    x = dconv(x)
    for l in range(case.levels, 0, -1):
        x = F.interpolate(x, scale_factor=2, mode="nearest")
        x = torch.cat([skips[l - 1], x], 1)
        x = dconv(x)
    last = x
    logits = F.conv2d(x, t(case.cls_w)[:, :, None, None], t(case.cls_b))
    return logits.numpy(), last.permute(0, 2, 3, 1).numpy().astype(np.int8)


def test_unet_matches_torch_composition():
    case = synth.unet_case(2, 0, 1, 32, 48, base=32, levels=2, n_classes=5)
    # the float64 stem may disagree with the float32 one only where |pre| is tiny; make
    # sure this seed has no such pixel so the whole cascade can be compared exactly
    pre, _ = O.stem(case.image, case.stem_w)
    assert np.abs(pre).min() > 2e-5
    logits, taps = O.unet_forward(case.image, case.stem_w, case.convs, case.cls_w,
                                  case.cls_b, levels=2)
    ref_logits, ref_last = torch_unet(case)
    assert [n for n, _ in taps] == ["stem", "enc1a", "enc1b", "pool1", "enc2a", "enc2b", "pool2",
                                    "mida", "midb", "up2", "cat2", "dec2a", "dec2b",
                                    "up1", "cat1", "dec1a", "dec1b"]
    assert np.array_equal(taps[-1][1], ref_last)
    assert (np.abs(logits - ref_logits) <= 1e-4 * np.maximum(1.0, np.abs(ref_logits))).all()
    shapes = {n: t.shape for n, t in taps}
    assert shapes["cat2"] == (1, 16, 24, 64 + 128) and shapes["cat1"] == (1, 32, 48, 32 + 64)


def test_channel_plan_and_mac_count():
    plan = synth.unet_channel_plan(64, 4)
    assert len(plan) == 18
    assert plan[10] == ("dec4a", 1536, 512, 4) and plan[16] == ("dec1a", 192, 64, 1)
    assert synth.unet_conv_macs(plan, 1, 1024, 2048) == 1855425871872


def test_config0_regression_fixture():
    """The stored summary of the oracle's config-0 output (written by
    tests/golden/make_golden.py from the oracle alone) still matches."""
    import os
    from tests.golden.make_golden import config0_summary
    path = os.path.join(os.path.dirname(__file__), "golden", "config0_oracle.txt")
    with open(path) as f:
        stored = f.read().splitlines()
    assert stored == config0_summary()


# ------------------------------------------------------- transposed layer (decoder)
def test_tconv_equals_torch_conv_transpose_and_brute_force():
    rng = np.random.default_rng(21)
    a = synth.pm1_bits(rng, (2, 5, 7, 40))
    w = synth.ternary_tconv_weights(99, 0, 0, 24, 40, 0.6)
    acc = O.tconv2x2(a, w)
    assert acc.shape == (2, 10, 14, 24)
    # library special case: ConvTranspose2d weight is [Cin][Cout][kh][kw]
    wt = torch.from_numpy(w).double().permute(3, 0, 1, 2)
    ref = F.conv_transpose2d(torch.from_numpy(a).double().permute(0, 3, 1, 2), wt, stride=2)
    assert np.array_equal(acc.astype(np.float64), ref.permute(0, 2, 3, 1).numpy())
    # brute force in scatter form on a tiny case
    a2, w2 = a[:1, :2, :3, :5], w[:3, :, :, :5]
    out = np.zeros((1, 4, 6, 3), np.int64)
    for y in range(2):
        for x in range(3):
            for dy in range(2):
                for dx in range(2):
                    for o in range(3):
                        out[0, 2 * y + dy, 2 * x + dx, o] = sum(
                            int(w2[o, dy, dx, c]) * int(a2[0, y, x, c]) for c in range(5))
    assert np.array_equal(O.tconv2x2(np.ascontiguousarray(a2), np.ascontiguousarray(w2)), out)


def test_tconv_single_tap_and_invariants():
    rng = np.random.default_rng(22)
    a = synth.pm1_bits(rng, (1, 3, 4, 6))
    for (o, dy, dx, c, sgn) in [(0, 0, 0, 2, 1), (1, 1, 0, 5, -1), (2, 0, 1, 0, 1), (1, 1, 1, 3, -1)]:
        w = np.zeros((3, 2, 2, 6), np.int8)
        w[o, dy, dx, c] = sgn
        acc = O.tconv2x2(a, w)
        exp = np.zeros((6, 8), np.int32)
        exp[dy::2, dx::2] = sgn * a[0, :, :, c]
        assert np.array_equal(acc[0, :, :, o], exp)
        assert not acc[0][:, :, [k for k in range(3) if k != o]].any()
    w = synth.ternary_tconv_weights(99, 1, 0, 4, 6, 0.5)
    acc = O.tconv2x2(a, w)
    assert np.array_equal(O.tconv2x2(-a, w), -acc)
    kept = O.tconv2x2(np.ones_like(a), np.abs(w).astype(np.int8))
    assert (np.abs(acc) <= kept).all() and ((acc - kept) % 2 == 0).all()
    assert not O.tconv2x2(a, np.zeros_like(w)).any()


def test_unet_with_transposed_decoder_matches_torch():
    case = synth.unet_case(5, 0, 1, 16, 32, base=32, levels=2, n_classes=3, transposed=True)
    pre, _ = O.stem(case.image, case.stem_w)
    assert np.abs(pre).min() > 2e-5
    logits, taps = O.unet_forward(case.image, case.stem_w, case.convs, case.cls_w, case.cls_b,
                                  levels=2, up_convs=case.up_convs)

    def t(a):
        return torch.from_numpy(np.ascontiguousarray(a)).double()
    x = F.conv2d(t(case.image), t(case.stem_w).permute(0, 3, 1, 2), padding=1)
    x = torch.where(x >= 0, 1.0, -1.0).double()
    it = iter(case.convs)

    def dconv(x):
        for _ in range(2):
            w, th = next(it)
            acc = F.conv2d(x, t(w).permute(0, 3, 1, 2), padding=1)
            x = torch.where(acc >= t(th)[None, :, None, None], 1.0, -1.0).double()
        return x
    skips = []
    for _ in range(2):
        x = dconv(x)
        skips.append(x)
        x = F.max_pool2d(x, 2)
    x = dconv(x)
    for j, l in enumerate((2, 1)):
        wu, tu = case.up_convs[j]
        acc = F.conv_transpose2d(x, t(wu).permute(3, 0, 1, 2), stride=2)
        x = torch.where(acc >= t(tu)[None, :, None, None], 1.0, -1.0).double()
        x = torch.cat([skips[l - 1], x], 1)
        x = dconv(x)
    assert np.array_equal(taps[-1][1], x.permute(0, 2, 3, 1).numpy().astype(np.int8))
    shapes = {n: v.shape for n, v in taps}
    assert shapes["up2"] == (1, 8, 16, 64) and shapes["cat2"] == (1, 8, 16, 128)
    assert shapes["cat1"] == (1, 16, 32, 64)


# ------------------------------------------------------------ threshold folding, cost ranking
def test_batchnorm_sign_against_torch_and_closed_forms():
    """Pins of the oracle's batch norm + sign step (what Algorithm 1's threshold stands for,
    Sec. 3.2.2): the library routine in float64, and hand-solvable cases."""
    rng = np.random.default_rng(21)
    C = 24
    acc = rng.integers(-300, 301, size=(2, 5, 7, C))
    g = rng.standard_normal(C)
    b = rng.standard_normal(C) * 3
    m = rng.standard_normal(C) * 20
    v = rng.uniform(0.5, 40.0, C)
    bias = rng.standard_normal(C)
    y, s = O.batchnorm_sign(acc, g, b, m, v, 1e-5, bias)
    x = torch.from_numpy((acc + bias).astype(np.float64)).permute(0, 3, 1, 2)
    ref = F.batch_norm(x, torch.from_numpy(m), torch.from_numpy(v), torch.from_numpy(g),
                       torch.from_numpy(b), training=False, eps=1e-5).permute(0, 2, 3, 1).numpy()
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-12)
    assert np.array_equal(s, np.where(ref >= 0, 1, -1))
    # identity batch norm: the bit is (acc + bias >= 0); a tie gives +1
    one, zero = np.ones(3), np.zeros(3)
    _, s = O.batchnorm_sign(np.array([[-1, 0, 1]]), one, zero, zero, one, 0.0, np.array([0.0, 0.0, -1.0]))
    assert s.tolist() == [[-1, 1, 1]]
    # a negative scale reverses the comparison, a zero scale leaves the sign of beta
    _, s = O.batchnorm_sign(np.array([[5, 5, 5]]), np.array([-1.0, 0.0, 0.0]), np.array([0.0, -2.0, 2.0]),
                            zero, one, 0.0)
    assert s.tolist() == [[-1, -1, 1]]


def test_cost_scores_properties():
    """Sec. 3.1.2's score: range, weights, order."""
    rng = np.random.default_rng(23)
    ops = rng.uniform(1e6, 1e11, 12)
    par = rng.uniform(1e3, 1e7, 12)
    for w_op in (0.0, 0.3, 0.5, 1.0):
        s, order = O.cost_scores(ops, par, w_op)
        assert s.min() >= 0 and s.max() <= 1 and (np.diff(s[order]) >= 0).all()
    # w_op = 1 ranks by operations alone, w_op = 0 by parameters alone
    assert np.array_equal(O.cost_scores(ops, par, 1.0)[1], np.argsort(ops, kind="stable"))
    assert np.array_equal(O.cost_scores(ops, par, 0.0)[1], np.argsort(par, kind="stable"))
    # the cheapest layer in both counts scores 0, the dearest in both scores 1
    s, _ = O.cost_scores([1, 5, 9], [2, 3, 7], 0.25)
    assert s[0] == 0.0 and s[2] == 1.0 and abs(s[1] - (0.25 * 0.5 + 0.75 * 0.2)) < 1e-15
    # the paper's observation (Sec. 3.1.2): grouped as its twelve configurable layers (double
    # convolutions, transposed convolutions), the transposed layers of a U-Net cost far fewer
    # operations than the others and therefore head the priority list
    plan = synth.unet_channel_plan(64, 4, transposed=True)
    h = w = 512
    conv_ops = [2.0 * (h >> (lv - 1)) * (w >> (lv - 1)) * 9 * ci * co for _, ci, co, lv in plan]
    conv_par = [9.0 * ci * co for _, ci, co, _ in plan]
    pairs = [(conv_ops[i] + conv_ops[i + 1], conv_par[i] + conv_par[i + 1]) for i in range(2, len(plan), 2)]
    ups = [(2.0 * (h >> l) * (w >> l) * (128 << l) * (64 << l), 4.0 * (128 << l) * (64 << l))
           for l in range(4)]                       # up1..up4: one tap per output pixel
    layers = pairs + ups
    _, order = O.cost_scores([o for o, _ in layers], [p for _, p in layers], 1.0)
    assert set(order[:4].tolist()) == set(range(len(pairs), len(pairs) + 4))
    assert 5 * max(o for o, _ in ups) <= min(o for o, _ in pairs)
    # Appendix A.4 (cost scores with w_op = w_param = 0.5): ranks 1-4 are the four transposed
    # layers, ordered from the full-resolution one (fewest parameters, rank 1) to the deepest
    # (rank 4); their operation counts are equal, so the parameter count decides.  This plan
    # reproduces that order and the scores' magnitudes (all four below 0.13, as printed); the
    # scores of the double convolutions depend on the channel plan of the missing architecture
    # figure and are not reproduced.
    s, order = O.cost_scores([o for o, _ in layers], [p for _, p in layers], 0.5)
    n = len(pairs)
    assert order[:4].tolist() == [n + 0, n + 1, n + 2, n + 3]      # up1 (full resolution) ... up4 (deepest)
    assert (np.diff(s[n:n + 4]) > 0).all() and s[n + 3] < 0.13 and s[n] < 0.02
    assert s[n + 3] < s[:n].min()


def test_upsampled_channels_collapse_to_2x2_kernels_at_low_resolution():
    """Identity the decoder kernel of the library relies on (a property of the definitions of
    nearest up-sampling and of the zero-padded 3x3 layer, Sec. 2.1 / Sec. 3.1.1): the layer on
    the up-sampled tensor equals, for every output parity class (dy, dx), a 2x2 kernel over the
    low-resolution tensor whose entries are sums of the 3x3 taps that fall on the same low pixel
    (rows {Y-1, Y, Y} for dy = 0, {Y, Y, Y+1} for dy = 1), with zero padding of the low tensor.
    Checked on the oracle's accumulators, borders included; the summed entries stay in -4..4."""
    rng = np.random.default_rng(5)
    N, Hl, Wl, C, Co = 2, 3, 5, 6, 4
    low = synth.pm1_bits(rng, (N, Hl, Wl, C))
    w = rng.integers(-1, 2, size=(Co, 3, 3, C)).astype(np.int8)
    acc, _ = O.masked_binary_layer(O.upsample2x(low), w, np.zeros(Co, np.int32))
    taps = {0: ([0], [1, 2]), 1: ([0, 1], [2])}     # parity -> 3x3 indices on low offset 0 / 1
    pad = np.zeros((N, Hl + 2, Wl + 2, C), np.int64)
    pad[:, 1:-1, 1:-1] = low
    for dy in (0, 1):
        for dx in (0, 1):
            k2 = np.zeros((Co, 2, 2, C), np.int64)
            for a in (0, 1):
                for b in (0, 1):
                    for ky in taps[dy][a]:
                        for kx in taps[dx][b]:
                            k2[:, a, b] += w[:, ky, kx]
            assert np.abs(k2).max() <= 4
            got = np.zeros((N, Hl, Wl, Co), np.int64)
            for a in (0, 1):
                for b in (0, 1):
                    # low pixel (Y - 1 + dy + a, X - 1 + dx + b), in padded coordinates + 1
                    win = pad[:, dy + a:dy + a + Hl, dx + b:dx + b + Wl]
                    got += np.einsum("nyxc,oc->nyxo", win, k2[:, a, b])
            assert np.array_equal(got, acc[:, dy::2, dx::2]), (dy, dx)


def test_bit_valued_activations_with_half_valued_padding_reproduce_the_layer():
    """Identity the matrix-path kernels of the library rely on (a property of Eq. 1 with zero
    padding, Sec. 3.1.1): with a' = (a + 1) / 2 - the packed bit itself, and 1/2 for a pixel
    outside the image, whose value 0 lies half way between -1 and +1 - the accumulator is
    sum w a = 2 sum w a' - sum w, the last sum over ALL taps and channels of the output channel,
    borders included.  All terms are multiples of 1/2 and every partial sum is exactly
    representable, so a threshold comparison R >= theta is the sign test of
    sum w a' - (theta + sum w) / 2.  Checked on the oracle's accumulators."""
    rng = np.random.default_rng(9)
    N, H, W, C, Co = 2, 4, 5, 7, 6
    a = synth.pm1_bits(rng, (N, H, W, C))
    w = rng.integers(-1, 2, size=(Co, 3, 3, C)).astype(np.int8)
    theta = rng.integers(-10, 11, size=Co).astype(np.int32)
    acc, out = O.masked_binary_layer(a, w, theta)
    half = np.full((N, H + 2, W + 2, C), 0.5)
    half[:, 1:-1, 1:-1] = (a.astype(np.float64) + 1.0) / 2.0
    got = np.zeros((N, H, W, Co))
    for ky in range(3):
        for kx in range(3):
            got += np.einsum("nyxc,oc->nyxo", half[:, ky:ky + H, kx:kx + W], w[:, ky, kx].astype(np.float64))
    wsum = w.astype(np.int64).reshape(Co, -1).sum(1)
    assert np.array_equal(2.0 * got - wsum, acc.astype(np.float64))
    start = -(theta.astype(np.float64) + wsum) / 2.0
    assert np.array_equal(np.where(got + start >= 0, 1, -1), out)


# ------------------------------------------------- frame sizes that are not multiples of 2^levels
def test_floor_pooling_and_zero_padding_match_torch():
    """Odd sizes (Appendix A.3 lists 959-pixel-wide frames): pooling drops the last row / column
    like the library routine's default (floor) mode, and the decoder's padding is the library's
    constant padding with the difference split floor(d/2) before, the rest after."""
    rng = np.random.default_rng(31)
    for H, W in ((7, 9), (6, 9), (7, 8), (2, 5), (3, 3)):
        a = synth.pm1_bits(rng, (2, H, W, 5))
        t = torch.from_numpy(a).double().permute(0, 3, 1, 2)
        ref = F.max_pool2d(t, 2).permute(0, 2, 3, 1).numpy().astype(np.int8)
        got = O.maxpool2x2(a)
        assert got.shape == (2, H // 2, W // 2, 5) and np.array_equal(got, ref)
    a = synth.pm1_bits(rng, (2, 4, 6, 3))
    t = torch.from_numpy(a).double().permute(0, 3, 1, 2)
    for Ho, Wo in ((4, 6), (5, 6), (4, 7), (5, 7), (7, 9)):
        dy, dx = Ho - 4, Wo - 6
        ref = F.pad(t, [dx // 2, dx - dx // 2, dy // 2, dy - dy // 2]).permute(0, 2, 3, 1).numpy()
        assert np.array_equal(O.zero_pad_to(a, Ho, Wo), ref.astype(np.int8))
    # one missing row / column: the padding is the last row / column, all zeros
    p = O.zero_pad_to(a, 5, 7)
    assert np.array_equal(p[:, :4, :6], a) and not p[:, 4].any() and not p[:, :, 6].any()


def test_layer_on_zero_padded_activations():
    """A padded element (value 0) adds nothing: the layer on a tensor with zero-valued elements
    equals the library convolution in float64 and the scatter-form brute force, and equals the
    layer with the weights that meet those elements masked."""
    rng = np.random.default_rng(32)
    a = synth.pm1_bits(rng, (1, 4, 5, 6))
    a[:, :, 4, 3:] = 0          # last column of the last three channels was padded
    a[:, 3, :, 3:] = 0
    w = synth.ternary_weights(98, 0, 0, 4, 6, 0.7)
    acc = O.conv3x3(a, w)
    ref = F.conv2d(torch.from_numpy(a).double().permute(0, 3, 1, 2),
                   torch.from_numpy(w).double().permute(0, 3, 1, 2), padding=1).permute(0, 2, 3, 1).numpy()
    assert np.array_equal(acc.astype(np.float64), ref)
    assert np.array_equal(acc, scatter_conv(a, w))
    # same sums when the zero elements are replaced by +1 and excluded through the image border
    # instead: rows 0..2, columns 0..3 of the padded channels as an image of their own
    lo = O.conv3x3(a[:, :3, :4, 3:], w[..., 3:])
    hi = O.conv3x3(a[..., :3], w[..., :3])
    assert np.array_equal(acc[:, :3, :4], hi[:, :3, :4] + lo)


def torch_unet_any_size(case):
    """The network recomposed from PyTorch-CPU float64 library ops for any frame size: floor
    pooling, decoder feature padded to the skip feature's size before the concatenation."""
    def t(a):
        return torch.from_numpy(np.ascontiguousarray(a)).double()
    x = F.conv2d(t(case.image), t(case.stem_w).permute(0, 3, 1, 2), padding=1)
    x = torch.where(x >= 0, 1.0, -1.0).double()
    it = iter(case.convs)

    def dconv(x):
        for _ in range(2):
            w, th = next(it)
            acc = F.conv2d(x, t(w).permute(0, 3, 1, 2), padding=1)
            x = torch.where(acc >= t(th)[None, :, None, None], 1.0, -1.0).double()
        return x
    skips = []
    for _ in range(case.levels):
        x = dconv(x)
        skips.append(x)
        x = F.max_pool2d(x, 2)
    x = dconv(x)
    for j, l in enumerate(range(case.levels, 0, -1)):
        if case.up_convs is None:
            x = F.interpolate(x, scale_factor=2, mode="nearest")
        else:
            wu, tu = case.up_convs[j]
            acc = F.conv_transpose2d(x, t(wu).permute(3, 0, 1, 2), stride=2)
            x = torch.where(acc >= t(tu)[None, :, None, None], 1.0, -1.0).double()
        sk = skips[l - 1]
        dy, dx = sk.shape[2] - x.shape[2], sk.shape[3] - x.shape[3]
        x = F.pad(x, [dx // 2, dx - dx // 2, dy // 2, dy - dy // 2])
        x = torch.cat([sk, x], 1)
        x = dconv(x)
    logits = F.conv2d(x, t(case.cls_w)[:, :, None, None], t(case.cls_b))
    return logits.numpy(), x.permute(0, 2, 3, 1).numpy().astype(np.int8)


@pytest.mark.parametrize("transposed", [False, True])
@pytest.mark.parametrize("H,W,levels", [(21, 27, 2), (23, 38, 3), (16, 31, 2)])
def test_unet_on_odd_frame_sizes_matches_torch(H, W, levels, transposed):
    for seed in range(4):
        case = synth.unet_case(13, seed, 1, H, W, base=32, levels=levels, n_classes=2,
                               transposed=transposed)
        pre, _ = O.stem(case.image, case.stem_w)
        if np.abs(pre).min() > 2e-5:      # float64 and float32 first layers agree on every sign
            break
    else:
        raise AssertionError("no seed without a near-zero first-layer sum")
    logits, taps = O.unet_forward(case.image, case.stem_w, case.convs, case.cls_w, case.cls_b,
                                  levels=levels, up_convs=case.up_convs)
    ref_logits, ref_last = torch_unet_any_size(case)
    assert np.array_equal(taps[-1][1], ref_last)
    assert (np.abs(logits - ref_logits) <= 1e-4 * np.maximum(1.0, np.abs(ref_logits))).all()
    shapes = {n: v.shape[1:3] for n, v in taps}
    assert shapes[f"pool{levels}"] == (H >> levels, W >> levels)
    assert shapes["up1"] == (2 * (H // 2), 2 * (W // 2)) and shapes["cat1"] == (H, W)
    if W % 2:
        assert not taps[[n for n, _ in taps].index("cat1")][1][0, :, W - 1, 32:].any()
