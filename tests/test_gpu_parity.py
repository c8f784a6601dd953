"""GPU parity: the HIP library (through the C ABI) against the CPU oracle, element by
element on the same seeded inputs.  Integer accumulators and packed bits must be
bit-exact; the float32 classifier within 1e-4 relative."""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_2601_11660_amd import binding as B
from paper_2601_11660_amd import synth
from tests import bitref
from tests.gpu_util import check_conv_rows, dev, host, host_u32, say

pytestmark = pytest.mark.gpu

PATHS = [(B.PATH_VALU, "valu"), (B.PATH_MFMA, "mfma")]


@pytest.fixture(autouse=True)
def _auto_path():
    yield
    B.set_conv_path(B.PATH_AUTO)
    B.set_conv_tuning(0)
    torch.cuda.synchronize()


# ------------------------------------------------------------------------ packing
@pytest.mark.parametrize("C", [1, 31, 32, 40, 64, 96, 100, 512])
def test_pack_act_int8_and_float(C):
    say(f"pack_act C={C}")
    rng = np.random.default_rng(C)
    a = synth.pm1_bits(rng, (2, 5, 7, C))
    got = host_u32(B.pack_act(dev(a)))
    assert np.array_equal(got, bitref.pack_pm1(a))
    f = rng.standard_normal((2, 5, 7, C)).astype(np.float32)
    f.ravel()[::5] = 0.0
    f.ravel()[1::7] = -0.0
    got = host_u32(B.pack_act(dev(f)))
    assert np.array_equal(got, bitref.pack_pm1(np.where(f >= 0, 1, -1)))


def run_layer(case, path, want_acc=True):
    B.set_conv_path(path)
    N, H, W, Cin = case.a.shape
    Cout = case.w.shape[0]
    act = B.pack_act(dev(case.a))
    blob = B.pack_weights(dev(case.w))
    theta = dev(case.theta)
    # bits-only call first (the production kernel), then, if asked, the call that also
    # returns the accumulators; both must give the same packed bits
    bits, _ = B.conv3x3_masked_binary(act, Cin, blob, Cout, theta, True, False)
    torch.cuda.synchronize()
    bits = host_u32(bits)
    acc = None
    if want_acc:
        bits2, acc = B.conv3x3_masked_binary(act, Cin, blob, Cout, theta, True, True)
        torch.cuda.synchronize()
        assert np.array_equal(host_u32(bits2), bits), "bits differ between the two kernels"
        acc = host(acc)
    return bits, acc


SMALL_SHAPES = [
    # N, H, W, Cin, Cout, keep
    (1, 64, 64, 64, 64, 0.6),      # the smallest workload
    (2, 13, 37, 96, 32, 0.5),      # ragged tile edges, Cin = 1.5 matrix steps, half channel tile
    (1, 9, 70, 64, 128, 0.3),      # two channel tiles, three column tiles
    (1, 8, 32, 32, 64, 0.7),       # one packed word per pixel
    (1, 20, 33, 40, 96, 0.6),      # Cin not a multiple of 32
    (3, 5, 5, 128, 64, 0.6),       # tiny images, batch
    (1, 1, 1, 64, 64, 0.6),        # single pixel: every tap but the centre is padding
    (1, 2, 3, 256, 32, 0.5),
    (1, 17, 65, 192, 64, 0.6),     # decoder-like Cin = 3*64
    (1, 16, 16, 512, 256, 0.6),
    (1, 3, 130, 160, 160, 0.4),
]


@pytest.mark.parametrize("path,pname", PATHS)
@pytest.mark.parametrize("shape", SMALL_SHAPES)
def test_conv_matches_oracle_elementwise(shape, path, pname):
    N, H, W, Cin, Cout, keep = shape
    say(f"conv {pname} N={N} H={H} W={W} Cin={Cin} Cout={Cout} keep={keep}")
    tb = 8 if shape == SMALL_SHAPES[0] else None
    case = synth.conv_case(0 if tb else 7, 0, N, H, W, Cin, Cout, keep, theta_bound=tb)
    acc_ref, out_ref = O.masked_binary_layer(case.a, case.w, case.theta)
    bits, acc = run_layer(case, path)
    assert np.array_equal(acc, acc_ref)
    assert np.array_equal(bits, bitref.pack_pm1(out_ref))


@pytest.mark.parametrize("path,pname", PATHS)
def test_conv_bits_only_and_acc_only(path, pname):
    say(f"conv outputs optional {pname}")
    B.set_conv_path(path)
    case = synth.conv_case(7, 1, 1, 11, 40, 64, 64, 0.6)
    acc_ref, out_ref = O.masked_binary_layer(case.a, case.w, case.theta)
    act, blob, th = B.pack_act(dev(case.a)), B.pack_weights(dev(case.w)), dev(case.theta)
    bits, acc = B.conv3x3_masked_binary(act, 64, blob, 64, th, True, False)
    assert acc is None and np.array_equal(host_u32(bits), bitref.pack_pm1(out_ref))
    bits, acc = B.conv3x3_masked_binary(act, 64, blob, 64, th, False, True)
    assert bits is None and np.array_equal(host(acc), acc_ref)


@pytest.mark.parametrize("path,pname", PATHS)
def test_conv_degenerate_masks_and_ties(path, pname):
    say(f"conv degenerate {pname}")
    case = synth.conv_case(7, 2, 1, 12, 34, 64, 64, 0.6)
    # all-zero mask: accumulator 0 everywhere, bit = (0 >= theta)
    zero = synth.ConvCase(case.a, np.zeros_like(case.w), case.theta, 0.0)
    bits, acc = run_layer(zero, path)
    assert not acc.any()
    exp = bitref.pack_pm1(np.broadcast_to(np.where(0 >= case.theta, 1, -1), (1, 12, 34, 64)))
    assert np.array_equal(bits, exp)
    # full mask: plain XNOR-popcount layer (Eq. 1)
    full = synth.ConvCase(case.a, np.where(case.w == 0, 1, case.w).astype(np.int8), case.theta, 1.0)
    acc_ref, out_ref = O.masked_binary_layer(full.a, full.w, full.theta)
    bits, acc = run_layer(full, path)
    assert np.array_equal(acc, acc_ref) and np.array_equal(bits, bitref.pack_pm1(out_ref))
    # ties: theta equal to the accumulators of one pixel -> all +1 there; theta+1 -> all -1
    acc_ref, _ = O.masked_binary_layer(case.a, case.w, case.theta)
    for th in (acc_ref[0, 5, 17].copy(), acc_ref[0, 5, 17] + 1, acc_ref[0, 0, 0].copy()):
        tie = synth.ConvCase(case.a, case.w, th.astype(np.int32), 0.6)
        bits, _ = run_layer(tie, path)
        assert np.array_equal(bits, bitref.pack_pm1(O.threshold(acc_ref, th.astype(np.int32))))
    # extreme thresholds
    for v in (-(2 ** 31), 2 ** 31 - 1, 9 * 64, -9 * 64, 9 * 64 + 1):
        th = np.full(64, v, np.int32)
        bits, _ = run_layer(synth.ConvCase(case.a, case.w, th, 0.6), path)
        assert np.array_equal(bits, bitref.pack_pm1(O.threshold(acc_ref, th)))


@pytest.mark.parametrize("kernel", [1, 3, 6, 7, 8, 9])
@pytest.mark.parametrize("shape", SMALL_SHAPES + [(1, 100, 100, 128, 128, 0.6), (2, 31, 67, 64, 192, 0.5)])
def test_every_matrix_kernel_variant_matches_oracle(shape, kernel):
    """The library picks a kernel variant per layer shape; each variant must be exact on
    every shape (single and multiple input steps, ragged tiles, odd word counts)."""
    N, H, W, Cin, Cout, keep = shape
    say(f"conv mfma kernel={kernel} N={N} H={H} W={W} Cin={Cin} Cout={Cout}")
    case = synth.conv_case(8, 0, N, H, W, Cin, Cout, keep)
    _, out_ref = O.masked_binary_layer(case.a, case.w, case.theta)
    B.set_conv_tuning(kernel)
    bits, _ = run_layer(case, B.PATH_MFMA, want_acc=False)
    assert np.array_equal(bits, bitref.pack_pm1(out_ref))


ROWS_SHAPES = [
    # N, H, W, Cin, Cout: single 64-channel input step
    (1, 64, 64, 64, 64),
    (2, 38, 70, 64, 128),      # ragged strip, two output tiles, two images
    (1, 2, 2, 32, 32),         # one word in, half an output tile
    (1, 130, 34, 40, 96),      # Cin not a multiple of 32, many row segments
    (3, 6, 200, 64, 64),
    (1, 256, 512, 64, 64),     # every wave slot of the chip busy
    # wide enough that a wave's row segment is longer than the six-row loop body: segments of
    # 10 (6 + 4), 8 (6 + 2) and 6 rows with two waves per SIMD, 20, 14 and 12 with one
    (1, 160, 2048, 64, 128),
    (1, 110, 2048, 40, 128),
    (1, 96, 2048, 64, 128),
    # odd sizes: the pooled output rounds down (the last row / column is in no window)
    (1, 37, 71, 64, 64),
    (2, 9, 33, 40, 96),
    (1, 3, 3, 64, 32),
]


@pytest.mark.parametrize("kernel", [7, 8])
@pytest.mark.parametrize("shape", ROWS_SHAPES)
def test_row_streaming_kernel_with_pooled_output(shape, kernel):
    """The row-streaming kernel of the single-step layers (one or two waves per SIMD): packed
    output and the 2x2-pooled output written from the same pass (Sec. 2.1) against the oracle."""
    N, H, W, Cin, Cout = shape
    say(f"conv rows kernel={kernel} N={N} H={H} W={W} Cin={Cin} Cout={Cout}")
    case = synth.conv_case(11, 0, N, H, W, Cin, Cout, 0.6)
    _, out_ref = O.masked_binary_layer(case.a, case.w, case.theta)
    B.set_conv_tuning(kernel)
    pa = B.pack_act(dev(case.a))
    blob = B.pack_weights(dev(case.w))
    bits, pool = B.conv3x3_masked_binary_fused(pa, Cin, None, 0, blob, Cout, dev(case.theta), True, True)
    torch.cuda.synchronize()
    assert np.array_equal(host_u32(bits), bitref.pack_pm1(out_ref))
    assert np.array_equal(host_u32(pool), bitref.pack_pm1(O.maxpool2x2(out_ref)))
    bits2, _ = run_layer(case, B.PATH_MFMA, want_acc=False)
    assert np.array_equal(bits2, bitref.pack_pm1(out_ref))


ROWS2K_SHAPES = [
    # N, H, W, Cin, Cout: two 64-channel input steps (three or four words per pixel)
    (1, 64, 64, 128, 128),
    (2, 38, 70, 128, 64),      # ragged strip, two images
    (1, 2, 2, 96, 32),         # three words in, one output tile
    (1, 130, 34, 100, 96),     # Cin not a multiple of 32, many row segments, odd tile count
    (3, 6, 200, 128, 128),
    (1, 160, 2048, 128, 128),  # row segments of 20 rows (6-row loop body + remainder)
    (1, 110, 2048, 96, 64),    # ... 8 rows
    (1, 39, 65, 128, 128),     # odd sizes: pooled output rounds down
    (2, 7, 35, 100, 64),
]


@pytest.mark.parametrize("shape", ROWS2K_SHAPES)
def test_row_streaming_kernel_for_two_input_steps(shape):
    """The row-streaming kernel for layers with 65..128 input channels (32 output channels per
    wave): packed output and the 2x2-pooled output of the same pass against the oracle."""
    N, H, W, Cin, Cout = shape
    say(f"conv rows2k N={N} H={H} W={W} Cin={Cin} Cout={Cout}")
    case = synth.conv_case(12, 0, N, H, W, Cin, Cout, 0.6)
    _, out_ref = O.masked_binary_layer(case.a, case.w, case.theta)
    B.set_conv_tuning(9)
    pa = B.pack_act(dev(case.a))
    blob = B.pack_weights(dev(case.w))
    bits, pool = B.conv3x3_masked_binary_fused(pa, Cin, None, 0, blob, Cout, dev(case.theta), True, True)
    torch.cuda.synchronize()
    assert np.array_equal(host_u32(bits), bitref.pack_pm1(out_ref))
    assert np.array_equal(host_u32(pool), bitref.pack_pm1(O.maxpool2x2(out_ref)))
    bits2, _ = run_layer(case, B.PATH_MFMA, want_acc=False)
    assert np.array_equal(bits2, bitref.pack_pm1(out_ref))


FUSED_SHAPES = [
    # N, H, W, Ca, Clow, Cout
    (1, 16, 64, 64, 128, 64),      # decoder level 1 shape in miniature
    (2, 12, 38, 96, 160, 96),      # odd word counts on both sides, ragged tiles
    (1, 8, 34, 32, 32, 64),        # one word each: a step straddles the two sources
    (1, 20, 40, 128, 256, 256),
    (1, 6, 10, 64, 40, 32),        # low channels not a multiple of 32
    (1, 4, 4, 512, 1024, 128),
    (1, 13, 37, 96, 160, 96),      # odd sizes: low is 6 x 18, its up-sampling is zero-padded; pool rounds down
    (2, 9, 35, 128, 128, 256),
]


@pytest.mark.parametrize("shape", FUSED_SHAPES)
def test_fused_concat_upsample_pool(shape):
    """mbu_conv3x3_masked_binary_fused against the oracle's separate up-sample, concat,
    layer and pooling."""
    N, H, W, Ca, Clow, Cout = shape
    say(f"conv fused N={N} H={H} W={W} Ca={Ca} Clow={Clow} Cout={Cout}")
    rng = np.random.default_rng(Ca + Clow)
    skip = synth.pm1_bits(rng, (N, H, W, Ca))
    low = synth.pm1_bits(rng, (N, H // 2, W // 2, Clow))
    w = synth.ternary_weights(9, 0, 0, Cout, Ca + Clow, 0.6)
    th = synth.thresholds(9, 0, 0, Cout, (9 * (Ca + Clow)) // 16)
    x = O.concat(skip, O.zero_pad_to(O.upsample2x(low), H, W))
    _, out_ref = O.masked_binary_layer(x, w, th)
    pool_ref = O.maxpool2x2(out_ref)
    blob = B.pack_weights(dev(w))
    pa, pl = B.pack_act(dev(skip)), B.pack_act(dev(low))
    bits, pool = B.conv3x3_masked_binary_fused(pa, Ca, pl, Clow, blob, Cout, dev(th), True, True)
    torch.cuda.synchronize()
    assert np.array_equal(host_u32(bits), bitref.pack_pm1(out_ref))
    assert np.array_equal(host_u32(pool), bitref.pack_pm1(pool_ref))
    # pooled output alone; plain input with pooled output
    _, pool2 = B.conv3x3_masked_binary_fused(pa, Ca, pl, Clow, blob, Cout, dev(th), False, True)
    assert np.array_equal(host_u32(pool2), bitref.pack_pm1(pool_ref))
    w1 = synth.ternary_weights(9, 1, 0, Cout, Ca, 0.6)
    _, o1 = O.masked_binary_layer(skip, w1, th)
    b1, p1 = B.conv3x3_masked_binary_fused(pa, Ca, None, 0, B.pack_weights(dev(w1)), Cout, dev(th),
                                           True, True)
    assert np.array_equal(host_u32(b1), bitref.pack_pm1(o1))
    assert np.array_equal(host_u32(p1), bitref.pack_pm1(O.maxpool2x2(o1)))


UPCAT_SHAPES = [
    # N, H, W, Ca, Clow, Cout, keep: skip channels % 64 == 0 and low channels % 128 == 0
    (1, 16, 128, 64, 128, 64, 0.6),
    (2, 10, 140, 64, 128, 96, 1.0),     # ragged tiles both ways, no zero weights: sums reach +-4
    (1, 2, 2, 64, 128, 32, 0.6),        # one low pixel
    (1, 36, 132, 128, 256, 64, 0.3),
    (1, 8, 8, 256, 1024, 128, 0.9),     # many low steps
    (3, 6, 66, 192, 128, 64, 0.6),      # more skip than low channels
]


@pytest.mark.parametrize("shape", UPCAT_SHAPES)
def test_upsampled_decoder_kernel_matches_oracle(shape):
    """Decoder layer over [skip | 2x up-sampled low] (Sec. 2.1) with the up-sampled channels
    contracted at low resolution (summed taps): bit-exact against the oracle's up-sample,
    concatenation and layer, and against the library's kernel that reads the window at full
    resolution."""
    N, H, W, Ca, Clow, Cout, keep = shape
    say(f"conv upcat N={N} H={H} W={W} Ca={Ca} Clow={Clow} Cout={Cout} keep={keep}")
    rng = np.random.default_rng(Ca + Clow + H)
    skip = synth.pm1_bits(rng, (N, H, W, Ca))
    low = synth.pm1_bits(rng, (N, H // 2, W // 2, Clow))
    w = synth.ternary_weights(12, 0, 0, Cout, Ca + Clow, keep)
    th = synth.thresholds(12, 0, 0, Cout, (9 * (Ca + Clow)) // 16)
    _, out_ref = O.masked_binary_layer(O.concat(skip, O.upsample2x(low)), w, th)
    blob = B.pack_weights(dev(w))
    pa, pl = B.pack_act(dev(skip)), B.pack_act(dev(low))
    bits, _ = B.conv3x3_masked_binary_fused(pa, Ca, pl, Clow, blob, Cout, dev(th), True, False)
    torch.cuda.synchronize()
    assert np.array_equal(host_u32(bits), bitref.pack_pm1(out_ref))
    B.set_conv_tuning(1)     # the block-cooperative kernel on the same call
    bits1, _ = B.conv3x3_masked_binary_fused(pa, Ca, pl, Clow, blob, Cout, dev(th), True, False)
    torch.cuda.synchronize()
    assert np.array_equal(host_u32(bits1), host_u32(bits))
    if keep == 1.0:
        # every summed tap at its extreme (+4 / -4 in the corners of the 2x2 kernels)
        for sgn in (1, -1):
            w1 = np.full_like(w, sgn)
            _, ref1 = O.masked_binary_layer(O.concat(skip, O.upsample2x(low)), w1, th)
            b1, _ = B.conv3x3_masked_binary_fused(pa, Ca, pl, Clow, B.pack_weights(dev(w1)), Cout, dev(th),
                                                  True, False)
            torch.cuda.synchronize()
            assert np.array_equal(host_u32(b1), bitref.pack_pm1(ref1))


TCONV_SHAPES = [
    # N, H, W, Cin, Cout
    (1, 8, 32, 128, 64),
    (2, 5, 37, 96, 32),       # ragged pixel groups, odd word count, half channel tile
    (1, 3, 70, 64, 128),
    (1, 1, 1, 32, 64),
    (1, 6, 9, 40, 96),        # Cin not a multiple of 32
    (1, 16, 16, 1024, 512),
    (2, 5, 37, 256, 96),      # four input steps: weights-resident kernel, ragged groups, two images
    (1, 7, 70, 512, 64),      # eight steps, groups of two rows
    (1, 9, 33, 128, 128),     # two steps, groups of four rows with a ragged last group
]


@pytest.mark.parametrize("shape", TCONV_SHAPES)
def test_tconv_matches_oracle_elementwise(shape):
    N, H, W, Cin, Cout = shape
    say(f"tconv N={N} H={H} W={W} Cin={Cin} Cout={Cout}")
    rng = np.random.default_rng(Cin + Cout)
    a = synth.pm1_bits(rng, (N, H, W, Cin))
    w = synth.ternary_tconv_weights(10, 0, 0, Cout, Cin, 0.6)
    th = synth.thresholds(10, 0, 0, Cout, max(1, Cin // 8))
    acc_ref, out_ref = O.masked_binary_tconv_layer(a, w, th)
    act, blob, thd = B.pack_act(dev(a)), B.pack_tconv_weights(dev(w)), dev(th)
    bits, _ = B.tconv2x2_masked_binary(act, Cin, blob, Cout, thd, True, False)
    bits2, acc = B.tconv2x2_masked_binary(act, Cin, blob, Cout, thd, True, True)
    torch.cuda.synchronize()
    assert np.array_equal(host(acc), acc_ref)
    assert np.array_equal(host_u32(bits), bitref.pack_pm1(out_ref))
    assert np.array_equal(host_u32(bits2), bitref.pack_pm1(out_ref))
    # ties and a zero mask
    th2 = acc_ref[0, 0, 0].astype(np.int32).copy()
    b3, _ = B.tconv2x2_masked_binary(act, Cin, blob, Cout, dev(th2), True, False)
    assert np.array_equal(host_u32(b3), bitref.pack_pm1(O.threshold(acc_ref, th2)))
    bz, az = B.tconv2x2_masked_binary(act, Cin, B.pack_tconv_weights(dev(np.zeros_like(w))), Cout,
                                      thd, True, True)
    assert not host(az).any()


@pytest.mark.parametrize("shape", [(1, 12, 40, 64, 64, 64), (2, 9, 33, 96, 160, 96),
                                   (1, 8, 34, 32, 40, 64)])
def test_conv_on_plain_concatenation(shape):
    N, H, W, Ca, Cb, Cout = shape
    say(f"conv concat N={N} H={H} W={W} Ca={Ca} Cb={Cb} Cout={Cout}")
    rng = np.random.default_rng(Ca * 7 + Cb)
    a = synth.pm1_bits(rng, (N, H, W, Ca))
    b = synth.pm1_bits(rng, (N, H, W, Cb))
    w = synth.ternary_weights(11, 0, 0, Cout, Ca + Cb, 0.6)
    th = synth.thresholds(11, 0, 0, Cout, (9 * (Ca + Cb)) // 16)
    _, out_ref = O.masked_binary_layer(O.concat(a, b), w, th)
    bits, _ = B.conv3x3_masked_binary_concat(B.pack_act(dev(a)), Ca, B.pack_act(dev(b)), Cb,
                                             B.pack_weights(dev(w)), Cout, dev(th))
    torch.cuda.synchronize()
    assert np.array_equal(host_u32(bits), bitref.pack_pm1(out_ref))


@pytest.mark.parametrize("shape", [(1, 38, 70, 64, None, None), (2, 7, 33, 96, None, None), (1, 64, 64, 128, None, None),
                                   (1, 9, 13, 64, 8, 12), (2, 21, 67, 32, 20, 66), (1, 12, 40, 64, 3, 5)])
def test_row_streaming_kernel_on_two_inputs(shape):
    """The two-step row-streaming kernel reading [64 channels | 64 channels] of two tensors in
    place (first layer of the last decoder level behind a transposed layer, Sec. 2.1), the
    second tensor possibly smaller than the frame; with the pooled second output where the
    sizes allow; accumulators recovered through thresholds for one shape."""
    N, H, W, Cout, Hb, Wb = shape
    say(f"conv rows2k two inputs {shape}")
    rng = np.random.default_rng(H * W + Cout)
    a = synth.pm1_bits(rng, (N, H, W, 64))
    b = synth.pm1_bits(rng, (N, Hb or H, Wb or W, 64))
    w = synth.ternary_weights(17, 0, 0, Cout, 128, 0.6)
    th = synth.thresholds(17, 0, 0, Cout, 72)
    pad = np.zeros((N, H, W, 64), np.int8)
    pad[:, :b.shape[1], :b.shape[2]] = b
    acc_ref, out_ref = O.masked_binary_layer(O.concat(a, pad), w, th)
    pa, pb, blob = B.pack_act(dev(a)), B.pack_act(dev(b)), B.pack_weights(dev(w))
    B.set_conv_tuning(9)
    if Hb is None:
        bits, pool = B.conv3x3_masked_binary_concat(pa, 64, pb, 64, blob, Cout, dev(th), want_pool=True)
        assert np.array_equal(host_u32(pool), bitref.pack_pm1(O.maxpool2x2(out_ref)))
    else:
        bits, _ = B.conv3x3_masked_binary_two_inputs(pa, 64, pb, 64, False, blob, Cout, dev(th))
    torch.cuda.synchronize()
    assert np.array_equal(host_u32(bits), bitref.pack_pm1(out_ref))
    B.set_conv_tuning(1)      # the block kernel on the same call
    if Hb is None:
        bits1, _ = B.conv3x3_masked_binary_concat(pa, 64, pb, 64, blob, Cout, dev(th))
    else:
        bits1, _ = B.conv3x3_masked_binary_two_inputs(pa, 64, pb, 64, False, blob, Cout, dev(th))
    assert np.array_equal(host_u32(bits1), host_u32(bits))
    if shape[1] == 9:
        B.set_conv_tuning(9)
        got = recover_acc(lambda t: B.conv3x3_masked_binary_two_inputs(pa, 64, pb, 64, False, blob, Cout, t)[0],
                          acc_ref, Cout)
        assert np.array_equal(got, acc_ref)


@pytest.mark.parametrize("fuse", [True, False])
def test_unet_transposed_decoder_small_all_layers(fuse):
    """The paper-shaped decoder: masked transposed 2x2 layers instead of nearest up-sampling."""
    say(f"unet transposed small fuse={fuse}")
    case = synth.unet_case(6, 0, 2, 32, 64, base=32, levels=2, n_classes=5, transposed=True)
    compare_unet_all_taps(case, 2, 32, 64, fuse)
    case = synth.unet_case(6, 1, 1, 64, 96, base=64, levels=3, n_classes=19, transposed=True)
    compare_unet_all_taps(case, 1, 64, 96, fuse)


def test_unet_transposed_decoder_1024x2048_by_induction():
    say("unet transposed 1024x2048 induction")
    case = synth.unet_case(6, 2, 1, 1024, 2048, keep=0.6, transposed=True)
    check_unet_by_induction(case, 1, 1024, 2048)


def test_paths_agree_and_are_deterministic():
    say("conv paths agree")
    case = synth.conv_case(7, 3, 2, 40, 72, 128, 128, 0.5)
    b1, a1 = run_layer(case, B.PATH_VALU)
    b2, a2 = run_layer(case, B.PATH_MFMA)
    b3, a3 = run_layer(case, B.PATH_MFMA)
    assert np.array_equal(b1, b2) and np.array_equal(a1, a2)
    assert np.array_equal(b2, b3) and np.array_equal(a2, a3)


# --------------------------------------------- layer sweep at full size (512 x 512)
@pytest.mark.parametrize("C", [64, 128, 256, 512])
@pytest.mark.parametrize("keep", [0.3, 0.5, 0.7])
def test_layer_sweep_full_size(C, keep):
    say(f"layer sweep C={C} keep={keep}")
    case = synth.conv_case(1, 0, 1, 512, 512, C, C, keep)
    act = host_u32(B.pack_act(dev(case.a)))
    assert np.array_equal(act[0, 100], bitref.pack_pm1(case.a[0, 100]))
    outs = {}
    for path, pname in PATHS:
        bits, _ = run_layer(case, path, want_acc=False)
        outs[pname] = bits
    assert np.array_equal(outs["valu"], outs["mfma"])
    bits = outs["mfma"]
    # the whole tensor against the oracle for every shape of the sweep
    _, out_ref = O.masked_binary_layer(case.a, case.w, case.theta)
    exp = bitref.pack_pm1_fast(out_ref)
    bad = int((bits != exp).sum())
    assert bad == 0, f"C={C} keep={keep}: {bad} packed words differ"


# --------------------------------------------------------------------------- glue
@pytest.mark.parametrize("C", [32, 64, 96, 128, 192, 512, 40])
def test_pool_upsample_concat(C):
    say(f"glue C={C}")
    rng = np.random.default_rng(C)
    a = synth.pm1_bits(rng, (2, 6, 10, C))
    pa = B.pack_act(dev(a))
    assert np.array_equal(host_u32(B.maxpool2x2_bits(pa, C)), bitref.pack_pm1(O.maxpool2x2(a)))
    assert np.array_equal(host_u32(B.upsample2x_bits(pa, C)), bitref.pack_pm1(O.upsample2x(a)))
    if C % 32 == 0:
        for Cb in (32, 64, 40, C):
            b = synth.pm1_bits(rng, (2, 6, 10, Cb))
            got = host_u32(B.concat_bits(pa, C, B.pack_act(dev(b)), Cb))
            assert np.array_equal(got, bitref.pack_pm1(O.concat(a, b)))


# ------------------------------------------------------------------------ network
def build_unet(case, fuse=True):
    ups = None if case.up_convs is None else [(dev(w), dev(t)) for w, t in case.up_convs]
    return B.UNet(dev(case.stem_w), [(dev(w), dev(t)) for w, t in case.convs],
                  dev(case.cls_w), dev(case.cls_b), levels=case.levels, fuse=fuse, up_convs=ups)


def compare_unet_all_taps(case, N, H, W, fuse=True, images=None):
    """Every element of every step's output and of the logits against the oracle's network.
    images: which images of the batch to compare (default all); the oracle runs on those
    images only, the GPU on the whole batch (images are independent)."""
    net = build_unet(case, fuse)
    fused_away = fuse and B.get_conv_path() != B.PATH_VALU
    logits = net.forward(dev(case.image))
    torch.cuda.synchronize()
    got_logits = host(logits)
    pack = bitref.pack_pm1_fast if case.base % 32 == 0 else bitref.pack_pm1
    for n in (range(N) if images is None else images):
        ref_logits, taps = O.unet_forward(case.image[n:n + 1], case.stem_w, case.convs, case.cls_w,
                                          case.cls_b, levels=case.levels, up_convs=case.up_convs)
        taps = dict(taps)
        for s in range(net.num_steps - 1):
            name, _, h, w, c = net.step_info(N, H, W, s)
            ref = taps.pop(name)
            assert ref.shape == (1, h, w, c), name
            if name.startswith("cat") and (fused_away or (ref == 0).any()):
                continue      # folded into the layer that reads it (always, when the up-sampled
                              # part had to be zero-padded); never written
            got = host_u32(net.step_output(N, H, W, s)[n:n + 1])
            bad = int((got != pack(ref)).sum())
            assert bad == 0, f"image {n} step {s} ({name}): {bad} packed words differ"
            del ref
        err = np.abs(got_logits[n:n + 1] - ref_logits)
        assert (err <= 1e-4 * np.maximum(1.0, np.abs(ref_logits))).all(), float(err.max())


@pytest.mark.parametrize("fuse", [True, False])
@pytest.mark.parametrize("path,pname", PATHS)
def test_unet_small_all_layers(path, pname, fuse):
    say(f"unet small {pname} fuse={fuse}")
    B.set_conv_path(path)
    case = synth.unet_case(2, 1, 2, 32, 48, base=32, levels=2, n_classes=5)
    compare_unet_all_taps(case, 2, 32, 48, fuse)
    case = synth.unet_case(2, 2, 1, 64, 96, base=64, levels=3, n_classes=19)
    compare_unet_all_taps(case, 1, 64, 96, fuse)


@pytest.mark.parametrize("fuse", [True, False])
def test_unet_512_all_layers(fuse):
    """Full U-Net forward at 1x3x512x512, per-layer keep probability in [0.4,0.8]:
    every layer's packed bits exactly, logits within 1e-4 relative."""
    say(f"unet 512x512 all layers fuse={fuse}")
    case = synth.unet_case(2, 0, 1, 512, 512)
    compare_unet_all_taps(case, 1, 512, 512, fuse)


def check_unet_by_induction(case, N, H, W, rows_per_layer=3, fuse=True):
    """Full-size check without running the whole oracle: every step's GPU output is
    checked against the oracle applied to that step's GPU *input* (sampled row strips
    for the convolutions, everything for the cheap steps), so the chain is exact by
    induction from the image."""
    net = build_unet(case, fuse)
    logits = net.forward(dev(case.image))
    torch.cuda.synchronize()
    outs = {}
    infos = [net.step_info(N, H, W, s) for s in range(net.num_steps)]
    for s, (name, _, h, w, c) in enumerate(infos[:-1]):
        outs[name] = host_u32(net.step_output(N, H, W, s))
    # stem, on sampled rows of image 0 and the last image
    for n in sorted({0, N - 1}):
        for r0 in (0, H // 2 - 1, H - 2):
            c0, c1 = max(0, r0 - 1), min(H, r0 + 3)
            _, sg = O.stem(case.image[n:n + 1, :, c0:c1], case.stem_w)
            assert np.array_equal(outs["stem"][n, r0:r0 + 2],
                                  bitref.pack_pm1(sg[0, r0 - c0:r0 - c0 + 2])), "stem"
    prev = "stem"
    ci = 0
    skips = {}
    for s, (name, _, h, w, c) in enumerate(infos[:-1]):
        if name == "stem":
            continue
        if name.startswith("pool"):
            l = int(name[4:])
            skips[l] = prev
            x = outs[prev]
            exp = x[:, 0::2, 0::2] | x[:, 1::2, 0::2] | x[:, 0::2, 1::2] | x[:, 1::2, 1::2]
            # OR of packed words is the max of +-1 values (checked against the oracle's
            # pooling in the small-shape glue test); spot check through the oracle too
            a = bitref.unpack_pm1(x[:1, :4], c)
            assert np.array_equal(bitref.pack_pm1(O.maxpool2x2(a)), outs[name][:1, :2]), name
            assert np.array_equal(exp, outs[name]), name
        elif name.startswith("up"):
            # transposed layer: sampled input rows -> two output rows each
            j = case.levels - int(name[2:])
            wu, tu = case.up_convs[j]
            xin = outs[prev]
            hh = xin.shape[1]
            for n in sorted({0, N - 1}):
                for r0 in sorted({0, hh // 2, hh - 1}):
                    a = bitref.unpack_pm1(xin[n:n + 1, r0:r0 + 1], wu.shape[3])
                    _, o = O.masked_binary_tconv_layer(a, wu, tu)
                    assert np.array_equal(outs[name][n:n + 1, 2 * r0:2 * r0 + 2], bitref.pack_pm1(o)), name
        elif name.startswith("cat"):
            l = int(name[3:])
            sk, lo = outs[skips[l]], outs[prev]
            up = lo if case.up_convs is not None else np.repeat(np.repeat(lo, 2, axis=1), 2, axis=2)
            cat = np.concatenate([sk, up], -1)
            if fuse:
                outs[name] = cat      # never materialised on the GPU: the next layer reads
            else:                     # skip and low in place, so check it against this
                assert np.array_equal(cat, outs[name]), name
        else:
            wgt, th = case.convs[ci]
            ci += 1
            cin = wgt.shape[3]
            hh = outs[prev].shape[1]
            starts = sorted({0, max(0, hh // 2 - 1), max(0, hh - rows_per_layer)})
            for n in sorted({0, N - 1}):
                for r0 in starts:
                    check_conv_rows(outs[prev], cin, wgt, th, outs[name], n, r0,
                                    min(hh, r0 + rows_per_layer), name)
        prev = name
    # classifier on sampled rows
    got = host(logits)
    last = outs[prev]
    for n in sorted({0, N - 1}):
        for r0 in (0, H // 2, H - 2):
            a = bitref.unpack_pm1(last[n:n + 1, r0:r0 + 2], case.base)
            ref = O.classifier(a, case.cls_w, case.cls_b)
            g = got[n:n + 1, :, r0:r0 + 2]
            assert (np.abs(g - ref) <= 1e-4 * np.maximum(1.0, np.abs(ref))).all(), "classifier"


@pytest.mark.parametrize("fuse", [True, False])
def test_unet_1024x2048_by_induction(fuse):
    """The high-resolution shape the benchmark times: batch 1, 3x1024x2048, keep 0.6."""
    say(f"unet 1024x2048 induction fuse={fuse}")
    case = synth.unet_case(3, 0, 1, 1024, 2048, keep=0.6)
    check_unet_by_induction(case, 1, 1024, 2048, fuse=fuse)


def test_unet_1024x2048_every_element():
    """The shape the benchmark times (batch 1, 3x1024x2048, keep 0.6, glue folded into the
    layers as in the timed run): every element of every layer's output and every logit against
    the oracle's whole-network forward pass."""
    say("unet 1024x2048 every element")
    case = synth.unet_case(3, 0, 1, 1024, 2048, keep=0.6)
    compare_unet_all_taps(case, 1, 1024, 2048, True)


def wide_case(mean_zero, n, h, w):
    plan = synth.unet_channel_plan(128, 4)
    zf = synth.cost_aware_zero_fractions(plan, 1024, 1024, mean_zero)
    return synth.unet_case(4, 0, n, h, w, base=128, keeps=[1.0 - z for z in zf])


@pytest.mark.parametrize("mean_zero", [0.2, 0.4, 0.6, 0.8])
def test_unet_wide_batch_by_induction(mean_zero):
    """Sparsity-stress network (channels widened 2x, cost-aware per-layer zero fractions) on a
    small batch: ragged row strips, two images."""
    say(f"unet wide mean_zero={mean_zero}")
    check_unet_by_induction(wide_case(mean_zero, 2, 256, 256), 2, 256, 256)


@pytest.mark.parametrize("mean_zero", [0.2, 0.4, 0.6, 0.8])
def test_unet_wide_batch8_full_size(mean_zero):
    """The sparsity-stress workload at its full size: batch 8, 3x1024x1024, channels widened
    2x (128..2048, decoder inputs 384..3072), cost-aware zero pattern around each of the four
    mean zero fractions.  Checked by induction on sampled rows of the first and the last image."""
    say(f"unet wide batch 8 at 1024x1024 mean_zero={mean_zero}")
    check_unet_by_induction(wide_case(mean_zero, 8, 1024, 1024), 8, 1024, 1024, rows_per_layer=2)


def test_unet_wide_batch8_first_and_last_image_every_element():
    """The same batch-8 run at mean zero fraction 0.4: every element of every layer and every
    logit of image 0 against the oracle's forward pass of that image (the batch's images are
    independent), and of image 7 the same (the last tiles of the persistent kernels' walk)."""
    say("unet wide batch 8 at 1024x1024 mean_zero=0.4, images 0 and 7 every element")
    compare_unet_all_taps(wide_case(0.4, 8, 1024, 1024), 8, 1024, 1024, True, images=(0, 7))


# ---------------------------------- the production kernels' accumulators, seen through the bits
def recover_acc(run_bits, acc_ref, cout):
    """R of Algorithm 1 as the bits-only (production) kernels compute it: the call is repeated
    with every threshold from min(R) - 1 to max(R) + 1 (the same value for all channels); an
    output is 1 exactly for the thresholds <= its R, so counting the ones gives R itself."""
    lo, hi = int(acc_ref.min()) - 1, int(acc_ref.max()) + 1
    sh = torch.arange(32, dtype=torch.int32, device="cuda")
    count = None
    for t in range(lo, hi + 1):
        bits = run_bits(torch.full((cout,), t, dtype=torch.int32, device="cuda"))
        ones = ((bits.unsqueeze(-1) >> sh) & 1).flatten(-2)[..., :cout]
        count = ones if count is None else count + ones
    torch.cuda.synchronize()
    return host(count) + (lo - 1)


ACC_CASES = [
    # label, kernel variant (mbu_set_conv_tuning), N, H, W, Cin, Cout
    ("rows, two waves per SIMD", 7, 1, 12, 70, 64, 64),
    ("rows, one wave per SIMD", 8, 2, 9, 40, 40, 96),
    ("rows, two input steps", 9, 1, 10, 40, 128, 64),
    ("block, waves over rows", 1, 1, 18, 40, 192, 64),
    ("block, waves over rows and channels", 1, 1, 9, 40, 96, 128),
    ("block, waves over channels", 1, 1, 8, 34, 128, 256),
    ("wave-private, 3 rows", 3, 1, 7, 40, 96, 64),
    ("wave-private, 6 rows", 6, 1, 13, 33, 64, 32),
    ("automatic choice", 0, 1, 16, 16, 512, 256),
]


@pytest.mark.parametrize("case", ACC_CASES, ids=[c[0] for c in ACC_CASES])
def test_production_kernel_accumulators_through_thresholds(case):
    """Every accumulator of the bits-only kernels is pinned to its exact value (not only to the
    side of one threshold it lies on): an error of the sum that crosses no sampled threshold
    would otherwise go unseen."""
    label, kernel, N, H, W, Cin, Cout = case
    say(f"accumulators through thresholds: {label} N={N} H={H} W={W} Cin={Cin} Cout={Cout}")
    c = synth.conv_case(15, 0, N, H, W, Cin, Cout, 0.6)
    acc_ref = O.conv3x3(c.a, c.w)
    B.set_conv_path(B.PATH_MFMA)
    B.set_conv_tuning(kernel)
    act, blob = B.pack_act(dev(c.a)), B.pack_weights(dev(c.w))
    got = recover_acc(lambda th: B.conv3x3_masked_binary(act, Cin, blob, Cout, th)[0], acc_ref, Cout)
    assert np.array_equal(got, acc_ref)


def test_decoder_kernel_accumulators_through_thresholds():
    """The same for the two-input forms: the low-resolution decoder kernel (summed taps), the
    block kernel reading [skip | up-sampled low] in place, and a second input that covers less
    than the frame (zeros where it has no pixel)."""
    say("accumulators through thresholds: two-input kernels")
    rng = np.random.default_rng(77)
    N, H, W, Ca, Cb, Cout = 1, 8, 72, 64, 128, 64
    skip = synth.pm1_bits(rng, (N, H, W, Ca))
    low = synth.pm1_bits(rng, (N, H // 2, W // 2, Cb))
    w = synth.ternary_weights(15, 1, 0, Cout, Ca + Cb, 0.6)
    acc_ref = O.conv3x3(O.concat(skip, O.upsample2x(low)), w)
    pa, pl, blob = B.pack_act(dev(skip)), B.pack_act(dev(low)), B.pack_weights(dev(w))
    for kernel in (0, 1):     # low-resolution kernel, block kernel
        B.set_conv_tuning(kernel)
        got = recover_acc(lambda th: B.conv3x3_masked_binary_fused(pa, Ca, pl, Cb, blob, Cout, th, True, False)[0],
                          acc_ref, Cout)
        assert np.array_equal(got, acc_ref), f"kernel variant {kernel}"
    B.set_conv_tuning(0)
    H2, W2 = 9, 13
    skip = synth.pm1_bits(rng, (N, H2, W2, 64))
    b = synth.pm1_bits(rng, (N, 8, 12, 96))
    w = synth.ternary_weights(15, 2, 0, 64, 160, 0.6)
    acc_ref = O.conv3x3(O.concat(skip, O.zero_pad_to(b, H2, W2)), w)
    pa, pb, blob = B.pack_act(dev(skip)), B.pack_act(dev(b)), B.pack_weights(dev(w))
    got = recover_acc(lambda th: B.conv3x3_masked_binary_two_inputs(pa, 64, pb, 96, False, blob, 64, th)[0],
                      acc_ref, 64)
    assert np.array_equal(got, acc_ref)


@pytest.mark.parametrize("shape", [(1, 6, 40, 128, 64), (1, 5, 33, 512, 64), (2, 4, 37, 96, 64),
                                   (1, 3, 70, 64, 128)],
                         ids=["weights resident, 2 steps", "weights resident, 8 steps", "streamed weights",
                              "single step"])
def test_transposed_kernel_accumulators_through_thresholds(shape):
    N, H, W, Cin, Cout = shape
    say(f"accumulators through thresholds: transposed layer N={N} H={H} W={W} Cin={Cin} Cout={Cout}")
    rng = np.random.default_rng(Cin * 3 + Cout)
    a = synth.pm1_bits(rng, (N, H, W, Cin))
    w = synth.ternary_tconv_weights(15, 3, 0, Cout, Cin, 0.6)
    acc_ref = O.tconv2x2(a, w)
    act, blob = B.pack_act(dev(a)), B.pack_tconv_weights(dev(w))
    got = recover_acc(lambda th: B.tconv2x2_masked_binary(act, Cin, blob, Cout, th, True, False)[0], acc_ref, Cout)
    assert np.array_equal(got, acc_ref)


# ------------------------------------------- frame sizes that are not multiples of 2^levels
PADDED_SHAPES = [
    # N, H, W, Ca, Cb, Cout, upsample
    (1, 9, 13, 64, 64, 64, 0),        # b is 8 x 12: one row and one column of zeros
    (2, 11, 35, 96, 160, 96, 0),      # odd word counts, ragged tiles, two images
    (1, 8, 33, 32, 40, 64, 0),        # only the column is missing; a step straddles the sources
    (1, 9, 13, 64, 128, 64, 1),       # nearest up-sampling of a 4 x 6 tensor to 8 x 12 of 9 x 13
    (2, 7, 70, 64, 128, 128, 1),
    (1, 37, 65, 128, 256, 64, 1),
    (1, 16, 64, 64, 128, 64, 1),      # nothing missing: the general entry point on a full extent
    (1, 9, 70, 64, 64, 64, 0, 2, 3),  # a second input far smaller than the frame: 2 x 3 pixels
    (2, 12, 40, 32, 96, 32, 1, 1, 1), # ... one pixel, up-sampled to 2 x 2
]


@pytest.mark.parametrize("shape", PADDED_SHAPES)
def test_two_input_layer_with_padded_second_input(shape):
    """Decoder layer of a frame whose size is not a multiple of 2^levels (Appendix A.3): the
    second input covers the top left of the frame, the rest of its channels are zeros."""
    N, H, W, Ca, Cb, Cout, ups = shape[:7]
    say(f"conv two inputs {shape}")
    rng = np.random.default_rng(Ca + Cb + H + W)
    Hb, Wb = shape[7:] if len(shape) > 7 else (H // 2, W // 2) if ups else (H - (H & 1), W - (W & 1))
    a = synth.pm1_bits(rng, (N, H, W, Ca))
    b = synth.pm1_bits(rng, (N, Hb, Wb, Cb))
    w = synth.ternary_weights(14, 0, 0, Cout, Ca + Cb, 0.6)
    th = synth.thresholds(14, 0, 0, Cout, (9 * (Ca + Cb)) // 16)
    bb = O.upsample2x(b) if ups else b
    # the second input sits at the top left of the frame: zeros below and to the right of it
    pad = np.zeros((N, H, W, Cb), np.int8)
    pad[:, :bb.shape[1], :bb.shape[2]] = bb
    if len(shape) == 7:
        assert np.array_equal(pad, O.zero_pad_to(bb, H, W))     # the decoder's padding is this placement
    x = O.concat(a, pad)
    _, out_ref = O.masked_binary_layer(x, w, th)
    bits, _ = B.conv3x3_masked_binary_two_inputs(B.pack_act(dev(a)), Ca, B.pack_act(dev(b)), Cb, bool(ups),
                                                 B.pack_weights(dev(w)), Cout, dev(th))
    torch.cuda.synchronize()
    assert np.array_equal(host_u32(bits), bitref.pack_pm1(out_ref))
    if ups and len(shape) == 7:
        # the fused entry point takes the same layer for odd sizes (low = floor(H/2) x floor(W/2))
        bits2, _ = B.conv3x3_masked_binary_fused(B.pack_act(dev(a)), Ca, B.pack_act(dev(b)), Cb,
                                                 B.pack_weights(dev(w)), Cout, dev(th), True, False)
        torch.cuda.synchronize()
        assert np.array_equal(host_u32(bits2), bitref.pack_pm1(out_ref))


@pytest.mark.parametrize("C", [32, 64, 96, 40])
def test_pool_rounds_odd_sizes_down(C):
    say(f"pool odd sizes C={C}")
    rng = np.random.default_rng(C + 1)
    for H, W in ((7, 9), (6, 9), (7, 8), (3, 2)):
        a = synth.pm1_bits(rng, (2, H, W, C))
        got = host_u32(B.maxpool2x2_bits(B.pack_act(dev(a)), C))
        assert np.array_equal(got, bitref.pack_pm1(O.maxpool2x2(a)))


@pytest.mark.parametrize("fuse", [True, False])
@pytest.mark.parametrize("transposed", [False, True])
def test_unet_odd_frame_sizes_small_all_layers(transposed, fuse):
    say(f"unet odd sizes transposed={transposed} fuse={fuse}")
    case = synth.unet_case(13, 0, 2, 37, 51, base=32, levels=2, n_classes=2, transposed=transposed)
    compare_unet_all_taps(case, 2, 37, 51, fuse)
    case = synth.unet_case(13, 1, 1, 75, 131, base=64, levels=4, n_classes=19, transposed=transposed)
    compare_unet_all_taps(case, 1, 75, 131, fuse)
    case = synth.unet_case(13, 2, 1, 70, 100, base=64, levels=3, n_classes=2, transposed=transposed)
    compare_unet_all_taps(case, 1, 70, 100, fuse)


def test_unet_odd_frame_sizes_are_refused_on_the_vector_path():
    say("unet odd sizes valu path")
    case = synth.unet_case(13, 0, 1, 37, 51, base=32, levels=2, n_classes=2)
    B.set_conv_path(B.PATH_VALU)
    net = build_unet(case, True)
    with pytest.raises(B.MbuError) as e:
        net.forward(dev(case.image))
    assert e.value.code == B.MBU_ERR_SHAPE


def test_unet_paper_frame_640x959_every_element():
    """The paper's Carvana frame (Appendix A.3: 959 wide, 640 high), network with the paper's
    transposed decoder and two classes, synthetic data: every element of every layer and every
    logit against the oracle."""
    say("unet 640x959 transposed decoder, 2 classes, every element")
    case = synth.unet_case(7, 0, 1, 640, 959, keep=0.6, transposed=True, n_classes=2)
    compare_unet_all_taps(case, 1, 640, 959, True)


# ------------------------------------------------------------------------ float32 ends
STEM_PATHS = [(B.STEM_VALU, "valu"), (B.STEM_MFMA, "mfma"), (B.STEM_MFMA_GATHER, "mfma-gather")]
STEM_KAPPA = 2.0 ** -17      # the matrix path's documented error budget


def _stem_norm_bound(image, w):
    """||w_o||_2 * ||patch(n,y,x)||_2 for every output, float64 [N,H,W,Co]."""
    x2 = torch.from_numpy(image.astype(np.float64) ** 2).sum(1, keepdim=True)
    p2 = torch.nn.functional.conv2d(x2, torch.ones(1, 1, 3, 3, dtype=torch.float64), padding=1)
    pn = np.sqrt(p2.numpy()[:, 0])                                    # [N,H,W]
    wn = np.sqrt((w.astype(np.float64) ** 2).reshape(w.shape[0], -1).sum(1))
    return pn[..., None] * wn[None, None, None, :]


def check_stem(image, w, path, pname, label):
    say(f"stem {label} path={pname} image={image.shape} Co={w.shape[0]}")
    B.set_stem_path(path)
    try:
        bits, _ = B.stem_fp32(dev(image), dev(w))
        bits2, pre = B.stem_fp32(dev(image), dev(w), want_pre=True)
        torch.cuda.synchronize()
    finally:
        B.set_stem_path(B.STEM_AUTO)
    ref_pre, ref_sgn = O.stem(image, w)
    exp = bitref.pack_pm1(ref_sgn)
    got, got2, pre = host_u32(bits), host_u32(bits2), host(pre)
    assert np.array_equal(got, exp), f"{label}: {int((got != exp).sum())} packed words differ"
    assert np.array_equal(got2, exp), f"{label}: bits differ when pre-activations are requested"
    return pre, ref_pre


STEM_SHAPES = [  # N, Ci, H, W, Co
    (1, 3, 37, 45, 64), (2, 3, 64, 100, 64), (1, 1, 33, 70, 32), (1, 3, 130, 257, 128),
    (3, 3, 16, 16, 96), (1, 3, 1, 1, 64), (1, 1, 2, 31, 64), (1, 3, 3, 32, 32),
    (1, 3, 6200, 40, 64),    # tall: the row-walking kernel's segments are several rows long
]


@pytest.mark.parametrize("path,pname", STEM_PATHS)
@pytest.mark.parametrize("shape", STEM_SHAPES)
def test_stem_matches_oracle(shape, path, pname):
    N, Ci, H, W, Co = shape
    rng = np.random.default_rng([11, N, Ci, H, W, Co])
    image = rng.standard_normal((N, Ci, H, W), dtype=np.float32)
    w = rng.standard_normal((Co, 3, 3, Ci), dtype=np.float32)
    pre, ref = check_stem(image, w, path, pname, "normal")
    if path == B.STEM_VALU:
        # same rounding sequence on both sides: the values themselves are identical, which
        # more than meets the layer's stated accuracy of 1e-4 relative
        assert np.array_equal(pre, ref)
        assert (np.abs(pre - ref) <= 1e-4 * np.maximum(1.0, np.abs(ref))).all()
    else:
        err = np.abs(pre.astype(np.float64) - ref.astype(np.float64))
        bound = STEM_KAPPA * _stem_norm_bound(image, w)
        assert (err <= bound).all(), f"estimate outside its error budget, worst {float((err / bound).max()):.3f}"


@pytest.mark.parametrize("path,pname", STEM_PATHS)
def test_stem_degenerate_inputs(path, pname):
    """Sums that are exactly zero or cancel almost completely, zero regions, extreme scales:
    the cases in which only the sequential chain defines the sign."""
    rng = np.random.default_rng(5)
    H, W, Co = 40, 70, 64
    # small integers: many sums are exactly 0 (tie -> +1) and all are exactly representable
    img = rng.integers(-2, 3, size=(1, 3, H, W)).astype(np.float32)
    w = rng.integers(-2, 3, size=(Co, 3, 3, 3)).astype(np.float32)
    pre, ref = check_stem(img, w, path, pname, "integers")
    assert (ref == 0).sum() > 1000 and np.array_equal(pre, ref)
    # all-zero image, and an image with zero regions and signed zeros
    check_stem(np.zeros((1, 3, H, W), np.float32), w, path, pname, "zero image")
    img = rng.standard_normal((1, 3, H, W), dtype=np.float32)
    img[:, :, 10:25, 20:50] = 0.0
    img[:, :, 12:14, 22:40] = -0.0
    check_stem(img, rng.standard_normal((Co, 3, 3, 3), dtype=np.float32), path, pname, "zero regions")
    # output channels whose weights are all zero: y = +0 everywhere (bit 1), and it must not cost
    # a sequential sum per pixel
    w = rng.standard_normal((Co, 3, 3, 3), dtype=np.float32)
    w[5] = 0.0
    w[40] = -0.0
    check_stem(rng.standard_normal((1, 3, H, W), dtype=np.float32), w, path, pname, "zero weight rows")
    # nearly cancelling sums: two copies of a channel with opposite weights plus a tiny third
    img = rng.standard_normal((1, 3, H, W), dtype=np.float32)
    img[:, 1] = img[:, 0]
    img[:, 2] *= np.float32(1e-7)
    w = rng.standard_normal((Co, 3, 3, 3), dtype=np.float32)
    w[..., 1] = -w[..., 0]
    check_stem(img, w, path, pname, "cancellation")
    # extreme but finite scales, mixed inside one image
    for scale_i, scale_w in ((1e30, 1e-3), (1e-30, 1.0), (1e-25, 1e-20), (1e18, 1e18)):
        img = rng.standard_normal((1, 3, H, W), dtype=np.float32) * np.float32(scale_i)
        img[:, :, :, 35:] *= np.float32(1e-6)
        w = rng.standard_normal((Co, 3, 3, 3), dtype=np.float32) * np.float32(scale_w)
        check_stem(img, w, path, pname, f"scale {scale_i:g} x {scale_w:g}")
    # magnitudes that differ from pixel to pixel by up to 2^40, and from row to row: patches that
    # are tiny against their neighbours (the row-walking kernel shares one scale per window)
    img = rng.standard_normal((1, 3, H, W), dtype=np.float32)
    img *= np.exp2(rng.integers(-20, 21, size=(1, 1, H, W))).astype(np.float32)
    check_stem(img, rng.standard_normal((Co, 3, 3, 3), dtype=np.float32), path, pname, "per-pixel scales")
    img = rng.standard_normal((1, 3, H, W), dtype=np.float32)
    img *= np.exp2(rng.integers(-30, 31, size=(1, 1, H, 1))).astype(np.float32)
    check_stem(img, rng.standard_normal((Co, 3, 3, 3), dtype=np.float32), path, pname, "per-row scales")
    # non-finite pixels: the comparison "sum >= 0" is false for NaN on both sides
    img = rng.standard_normal((1, 3, H, W), dtype=np.float32)
    img[0, 1, 5, 7] = np.nan
    img[0, 0, 20, 60] = np.inf
    img[0, 2, 30, 3] = -np.inf
    check_stem(img, rng.standard_normal((Co, 3, 3, 3), dtype=np.float32), path, pname, "non-finite")


def test_stem_full_size_frame():
    """All 134 M outputs of the benchmark frame's first layer against the oracle."""
    case = synth.unet_case(3, 0, 1, 1024, 2048, keep=0.6)
    pre, ref = check_stem(case.image, case.stem_w, B.STEM_MFMA, "mfma", "1024x2048")
    err = np.abs(pre.astype(np.float64) - ref.astype(np.float64))
    bound = STEM_KAPPA * _stem_norm_bound(case.image, case.stem_w)
    worst = float((err / bound).max())
    undecided = float((np.abs(pre) <= bound).mean())
    say(f"stem 1024x2048: worst |estimate - chain| / budget = {worst:.3f}; "
        f"fraction of outputs inside the budget (recomputed) <= {undecided:.2e}")
    assert worst <= 1.0


@pytest.mark.parametrize("shape", [(1, 9, 33, 32, 5), (2, 16, 40, 64, 19), (1, 7, 100, 128, 32),
                                   (1, 64, 64, 64, 1),
                                   (3, 5, 7, 64, 19), (4, 3, 5, 32, 3), (5, 1, 1, 64, 19),    # 32-pixel groups across images
                                   # few classes (table look-up kernel): all widths, strides across images
                                   (2, 33, 70, 64, 2), (1, 600, 700, 64, 2), (3, 40, 50, 128, 4), (1, 9, 9, 32, 1),
                                   (7, 11, 13, 128, 3), (1, 1100, 1900, 64, 1)])
def test_classifier_matches_oracle(shape):
    N, H, W, C, K = shape
    say(f"classifier {shape}")
    rng = np.random.default_rng([12, N, H, W, C, K])
    a = synth.pm1_bits(rng, (N, H, W, C))
    w = (rng.standard_normal((K, C), dtype=np.float32) / np.float32(8.0))
    b = rng.standard_normal((K,), dtype=np.float32)
    got = host(B.classifier_fp32(B.pack_act(dev(a)), C, dev(w), dev(b)))
    ref = O.classifier(a, w, b)
    assert (np.abs(got - ref) <= 1e-4 * np.maximum(1.0, np.abs(ref))).all()


# ------------------------------------------------------------- deployment flow around the layer
@pytest.mark.parametrize("shape", [(1, 20, 40, 64, 96), (2, 9, 33, 160, 64)])
def test_layer_with_folded_batchnorm(shape):
    """Batch norm + bias + sign after the layer (Sec. 3.2.2) folded into integer thresholds by
    the library, channels with a negative scale handled by negating their weights: the GPU
    layer's bits against the oracle's convolution followed by float64 batch norm and sign."""
    N, H, W, Cin, Cout = shape
    say(f"folded batch norm {shape}")
    case = synth.conv_case(8, 0, N, H, W, Cin, Cout, 0.5)
    rng = np.random.default_rng([14, Cin, Cout])
    g = rng.standard_normal(Cout)
    g[3::11] = 0.0
    beta = rng.standard_normal(Cout)
    mean = rng.standard_normal(Cout) * 6
    var = rng.uniform(0.5, 60.0, Cout)
    bias = rng.standard_normal(Cout)
    eps = 1e-5
    thresh, flip = B.fold_batchnorm(g, beta, mean, var, eps, bias, 9 * Cin)
    assert flip.sum() > 0 and (flip == 0).sum() > 0
    w_dev = np.where(flip[:, None, None, None] != 0, -case.w, case.w).astype(np.int8)
    bits, _ = B.conv3x3_masked_binary(B.pack_act(dev(case.a)), Cin, B.pack_weights(dev(w_dev)), Cout,
                                      dev(thresh))
    torch.cuda.synchronize()
    acc = O.conv3x3(case.a, case.w)
    y, s = O.batchnorm_sign(acc, g, beta, mean, var, eps, bias)
    got = bitref.unpack_pm1(host_u32(bits), Cout)
    sure = np.abs(y) > 1e-9
    assert sure.mean() > 0.999 and np.array_equal(got[sure], s[sure])


@pytest.mark.parametrize("fuse", [True, False])
def test_unet_smallest_frames_and_one_image_channel(fuse):
    """Degenerate sizes of the network: a frame of exactly 2^levels pixels a side (the bottleneck
    is a single pixel, every tap but the centre is padding), the same plus one (every level
    odd), and a one-channel image."""
    say(f"unet smallest frames fuse={fuse}")
    for H, W in ((16, 16), (17, 19), (16, 48)):
        case = synth.unet_case(16, H, 2, H, W, base=32, levels=4, n_classes=3)
        compare_unet_all_taps(case, 2, H, W, fuse)
    case = synth.unet_case(16, 1, 1, 40, 56, base=64, levels=2, n_classes=2)
    case.image = np.ascontiguousarray(case.image[:, :1])
    case.stem_w = np.ascontiguousarray(case.stem_w[..., :1])
    compare_unet_all_taps(case, 1, 40, 56, fuse)


def test_two_frames_in_flight_on_two_streams():
    """Two handles on one network (shared weights, own workspace) with forward passes
    interleaved on two streams: the same logits and layer outputs as one frame at a time."""
    say("two frames in flight")
    case = synth.unet_case(2, 4, 1, 128, 192, base=64, levels=3, n_classes=7)
    rng = np.random.default_rng(9)
    img2 = rng.standard_normal(case.image.shape, dtype=np.float32)
    net = build_unet(case, True)
    ref1 = host(net.forward(dev(case.image)))
    last1 = host_u32(net.step_output(1, 128, 192, net.num_steps - 2)).copy()
    ref2 = host(net.forward(dev(img2)))
    twin = net.clone_for_stream()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    i1, i2 = dev(case.image), dev(img2)
    o1 = torch.empty((1, 7, 128, 192), dtype=torch.float32, device="cuda")
    o2 = torch.empty_like(o1)
    torch.cuda.synchronize()
    for _ in range(20):
        with torch.cuda.stream(s1):
            net.forward(i1, o1)
        with torch.cuda.stream(s2):
            twin.forward(i2, o2)
    torch.cuda.synchronize()
    assert np.array_equal(host(o1), ref1) and np.array_equal(host(o2), ref2)
    assert np.array_equal(host_u32(net.step_output(1, 128, 192, net.num_steps - 2)), last1)
    assert twin.workspace.data_ptr() != net.workspace.data_ptr()


def test_forward_passes_from_two_host_threads():
    """The entry points are re-entrant: two host threads, each with its own handle, stream and
    workspace, run forward passes at the same time (ctypes releases the interpreter lock during
    the calls) while a third thread keeps re-writing the process-wide settings with the values
    they already have; every pass gives the single-threaded result."""
    import threading
    say("forward passes from two host threads")
    case = synth.unet_case(2, 5, 1, 96, 160, base=64, levels=3, n_classes=4)
    imgs = [case.image, np.random.default_rng(10).standard_normal(case.image.shape, dtype=np.float32)]
    net = build_unet(case, True)
    refs = [host(net.forward(dev(im))).copy() for im in imgs]
    handles = [net, net.clone_for_stream()]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    d_imgs = [dev(im) for im in imgs]
    outs = [torch.empty((1, 4, 96, 160), dtype=torch.float32, device="cuda") for _ in imgs]
    torch.cuda.synchronize()
    errors, stop = [], threading.Event()

    def worker(i):
        try:
            torch.cuda.set_device(0)
            for _ in range(60):
                with torch.cuda.stream(streams[i]):
                    handles[i].forward(d_imgs[i], outs[i])
                streams[i].synchronize()
                if not np.array_equal(host(outs[i]), refs[i]):
                    errors.append(f"thread {i}: logits differ")
                    return
        except Exception as e:          # noqa: BLE001 - reported through the list
            errors.append(f"thread {i}: {e!r}")

    def setter():
        while not stop.is_set():
            B.set_conv_path(B.PATH_AUTO)
            B.set_conv_tuning(0)
            B.set_stem_path(B.STEM_AUTO)

    ts = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    st = threading.Thread(target=setter)
    st.start()
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    stop.set()
    st.join()
    assert not errors, errors


def test_blob_sections():
    """Blobs packed with only the sections a layer's place in the network reads: the network
    object packs them that way by default; same bits as with complete blobs; a blob without the
    bit planes is refused by the vector-ALU path instead of being read out of bounds."""
    say("blob sections")
    case = synth.unet_case(2, 3, 1, 64, 96, base=64, levels=2, n_classes=5)
    lean = build_unet(case, True)
    assert lean.sections == [B.BLOB_MATRIX] * 6 + [B.BLOB_MATRIX | B.BLOB_SUMMED_TAPS, B.BLOB_MATRIX] * 2
    assert [lean.step_kernel(1, 64, 96, s) for s in (10, 13)] == ["conv_mfma_upcat_kernel"] * 2
    full = B.UNet(dev(case.stem_w), [(dev(w), dev(t)) for w, t in case.convs], dev(case.cls_w),
                  dev(case.cls_b), levels=2, all_sections=True)
    assert sum(b.numel() for b in lean.blobs) < 0.5 * sum(b.numel() for b in full.blobs)
    a, b = lean.forward(dev(case.image)), full.forward(dev(case.image))
    torch.cuda.synchronize()
    assert np.array_equal(host(a), host(b))
    for s in range(lean.num_steps - 1):
        if not lean.step_info(1, 64, 96, s)[0].startswith("cat"):
            assert np.array_equal(host_u32(lean.step_output(1, 64, 96, s)), host_u32(full.step_output(1, 64, 96, s)))
    # without the summed taps the decoder layers fall back to the 9-tap kernel: same bits
    none = build_unet(case, True)
    keep = [B.pack_weights(dev(w), B.BLOB_MATRIX) for w, _ in case.convs]
    for i, blob in enumerate(keep):
        none._layers[i].sections = B.BLOB_MATRIX
        none._layers[i].packed_w = blob.data_ptr()
    assert none.step_kernel(1, 64, 96, 10) == "conv_mfma_block_kernel"
    c = none.forward(dev(case.image))
    torch.cuda.synchronize()
    assert np.array_equal(host(c), host(b))
    B.set_conv_path(B.PATH_VALU)
    with pytest.raises(B.MbuError) as e:
        lean.forward(dev(case.image))
    assert e.value.code == B.MBU_ERR_ARG


def test_unet_with_cost_ranked_binary_and_masked_layers():
    """The deployment of Sec. 3.1.2 / 3.2.1: layers are masked in ascending cost-score order,
    the rest stay pure binary (no zero weights); every layer of the mixed network is bit-exact.
    On the matrix path a binary layer is the masked layer with an empty mask."""
    say("unet with cost-ranked masked layers")
    N, H, W = 1, 64, 96
    plan = synth.unet_channel_plan(64, 3)
    ops = [2.0 * (H >> (lv - 1)) * (W >> (lv - 1)) * 9 * ci * co for _, ci, co, lv in plan]
    par = [9.0 * ci * co for _, ci, co, _ in plan]
    _, order = B.cost_rank(ops, par, 0.5)
    masked = set(order[:len(plan) // 2].tolist())          # the cheaper half gets the zero state
    keeps = [0.5 if i in masked else 1.0 for i in range(len(plan))]
    case = synth.unet_case(9, 0, N, H, W, base=64, levels=3, keeps=keeps)
    for i, (wt, _) in enumerate(case.convs):
        assert ((wt == 0).any()) == (i in masked)
    compare_unet_all_taps(case, N, H, W, True)
