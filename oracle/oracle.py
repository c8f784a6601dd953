"""numpy front end of the C oracle (oracle/mbu_oracle.c) plus the U-Net composition.

TEST INFRASTRUCTURE ONLY.  The HIP library and its Python binding never import this
module; only tests, the smoke check and the benchmark's cpu_baseline leg do.  All
values are unpacked: activations int8 in {-1,+1} (NHWC), weights int8 in {-1,0,+1}
(OHWI), thresholds int32, images/logits float32 NCHW.

The network walk in `unet_forward` follows the encoder / decoder description of
Sec. 2.1 (double convolutions, down-sampling, up-sampling, skip concatenation) with
full-precision first and last layers (Sec. 4.1); every inner layer is the masked
layer of Sec. 3.1.1 followed by Algorithm 1's threshold step.
"""
import ctypes
import os

import numpy as np

from .build_oracle import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(_build())
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _chk(a, dtype, ndim=None):
    a = np.ascontiguousarray(a, dtype=dtype)
    if ndim is not None and a.ndim != ndim:
        raise ValueError(f"expected {ndim} dims, got {a.shape}")
    return a


def conv3x3(a, w):
    """acc[n,y,x,o] = sum_{ky,kx,c} w[o,ky,kx,c] * a[n,y+ky-1,x+kx-1,c]; taps outside
    the image add nothing (masked layer, Sec. 3.1.1; R of Algorithm 1)."""
    a = _chk(a, np.int8, 4)
    w = _chk(w, np.int8, 4)
    N, H, W, Cin = a.shape
    Cout = w.shape[0]
    assert w.shape == (Cout, 3, 3, Cin)
    acc = np.empty((N, H, W, Cout), np.int32)
    lib().orc_conv3x3(_p(a), N, H, W, Cin, _p(w), Cout, _p(acc))
    return acc


def conv3x3_points(a, w, pts):
    """The same sum at the listed outputs only; pts is [K,4] rows of (n,y,x,o)."""
    a = _chk(a, np.int8, 4)
    w = _chk(w, np.int8, 4)
    pts = _chk(pts, np.int32, 2)
    N, H, W, Cin = a.shape
    Cout = w.shape[0]
    assert pts.shape[1] == 4
    assert (pts >= 0).all() and (pts < np.array([N, H, W, Cout])).all()
    acc = np.empty(pts.shape[0], np.int32)
    lib().orc_conv3x3_points(_p(a), N, H, W, Cin, _p(w), Cout, _p(pts),
                             ctypes.c_long(pts.shape[0]), _p(acc))
    return acc


def threshold(acc, theta):
    """+1 where acc >= theta[o], else -1 (Algorithm 1, threshold comparison)."""
    acc = _chk(acc, np.int32)
    theta = _chk(theta, np.int32, 1)
    C = acc.shape[-1]
    assert theta.shape[0] == C
    out = np.empty(acc.shape, np.int8)
    lib().orc_threshold(_p(acc), _p(theta), ctypes.c_long(acc.size // C), C, _p(out))
    return out


def masked_binary_layer(a, w, theta):
    """One masked layer: dot products then threshold. Returns (acc, +-1 output)."""
    acc = conv3x3(a, w)
    return acc, threshold(acc, theta)


def tconv2x2(a, w):
    """Masked transposed convolution, kernel 2x2 stride 2 (up-sampling layer of the decoder,
    Sec. 2.1): acc[n,2y+dy,2x+dx,o] = sum_c w[o,dy,dx,c] * a[n,y,x,c].  w is [Cout,2,2,Cin]."""
    a = _chk(a, np.int8, 4)
    w = _chk(w, np.int8, 4)
    N, H, W, Cin = a.shape
    Cout = w.shape[0]
    assert w.shape == (Cout, 2, 2, Cin)
    acc = np.empty((N, 2 * H, 2 * W, Cout), np.int32)
    lib().orc_tconv2x2(_p(a), N, H, W, Cin, _p(w), Cout, _p(acc))
    return acc


def masked_binary_tconv_layer(a, w, theta):
    """Transposed layer followed by the threshold step (the quantised network adds batch
    norm + binary activation after the transposed convolution, Appendix A.1; both fold into
    the integer threshold as in Algorithm 1).  Returns (acc, +-1 output)."""
    acc = tconv2x2(a, w)
    return acc, threshold(acc, theta)


def maxpool2x2(a):
    """2x2 stride-2 max pooling; an odd last row / column is dropped (floor)."""
    a = _chk(a, np.int8, 4)
    N, H, W, C = a.shape
    out = np.empty((N, H // 2, W // 2, C), np.int8)
    lib().orc_maxpool2x2(_p(a), N, H, W, C, _p(out))
    return out


def upsample2x(a):
    a = _chk(a, np.int8, 4)
    N, H, W, C = a.shape
    out = np.empty((N, 2 * H, 2 * W, C), np.int8)
    lib().orc_upsample2x(_p(a), N, H, W, C, _p(out))
    return out


def zero_pad_to(a, Ho, Wo):
    """Pads a feature map with zeros to Ho x Wo, splitting the difference like the usual U-Net
    decoder does: floor(d/2) rows on top / columns on the left, the rest at the bottom / right
    (with floor pooling d is 0 or 1, so the padding sits at the bottom and on the right)."""
    a = _chk(a, np.int8, 4)
    N, H, W, C = a.shape
    assert Ho >= H and Wo >= W
    out = np.empty((N, Ho, Wo, C), np.int8)
    lib().orc_zero_pad(_p(a), N, H, W, C, (Ho - H) // 2, (Wo - W) // 2, Ho, Wo, _p(out))
    return out


def concat(a, b):
    a = _chk(a, np.int8, 4)
    b = _chk(b, np.int8, 4)
    assert a.shape[:3] == b.shape[:3]
    N, H, W, Ca = a.shape
    Cb = b.shape[3]
    out = np.empty((N, H, W, Ca + Cb), np.int8)
    lib().orc_concat(_p(a), Ca, _p(b), Cb, ctypes.c_long(N * H * W), _p(out))
    return out


def stem(img, w):
    """float32 3x3 first layer (Sec. 4.1), then sign with 0 -> +1.
    img NCHW, w [Co,3,3,Ci]. Returns (pre-activation NHWC float32, +-1 NHWC int8)."""
    img = _chk(img, np.float32, 4)
    w = _chk(w, np.float32, 4)
    N, Ci, H, W = img.shape
    Co = w.shape[0]
    assert w.shape == (Co, 3, 3, Ci)
    pre = np.empty((N, H, W, Co), np.float32)
    sgn = np.empty((N, H, W, Co), np.int8)
    lib().orc_stem(_p(img), N, Ci, H, W, _p(w), Co, _p(pre), _p(sgn))
    return pre, sgn


def classifier(a, w, b):
    """float32 1x1 last layer (Sec. 4.1) on +-1 features. a NHWC, w [K,C], b [K].
    Returns logits NCHW float32."""
    a = _chk(a, np.int8, 4)
    w = _chk(w, np.float32, 2)
    b = _chk(b, np.float32, 1)
    N, H, W, C = a.shape
    K = w.shape[0]
    assert w.shape == (K, C) and b.shape == (K,)
    out = np.empty((N, K, H, W), np.float32)
    lib().orc_classifier(_p(a), N, H, W, C, _p(w), _p(b), K, _p(out))
    return out


def unet_forward(image, stem_w, convs, cls_w, cls_b, levels=4, up_convs=None):
    """Whole network on unpacked values.

    up_convs: None = the decoder up-samples by 2x nearest neighbour.  Otherwise a list of
    (w [Cout,2,2,Cin], theta) per decoder level, deepest first: the decoder up-samples with a
    masked transposed convolution + threshold (Sec. 2.1, Appendix A.1) instead.

    convs: list of (w, theta) in execution order: two per encoder level (level 1 ..
    `levels`), two for the bottleneck, two per decoder level (`levels` .. 1);
    2*(2*levels+1) entries.  Down-sampling is 2x2 max pooling (floor), up-sampling is 2x
    nearest neighbour, and the skip feature is placed before the up-sampled one, which is
    zero-padded to the skip feature's size when the two differ (odd frame sizes; the padded
    elements are 0, not +-1, and add nothing to the next layer's sums).
    Returns (logits, taps) where taps is the list of every intermediate +-1 tensor
    in execution order as (name, array).
    """
    assert len(convs) == 2 * (2 * levels + 1)
    taps = []
    it = iter(convs)

    def double_conv(x, tag):
        for half in "ab":
            w, th = next(it)
            _, x = masked_binary_layer(x, w, th)
            taps.append((f"{tag}{half}", x))
        return x

    _, x = stem(image, stem_w)
    taps.append(("stem", x))
    skips = []
    for l in range(1, levels + 1):
        x = double_conv(x, f"enc{l}")
        skips.append(x)
        x = maxpool2x2(x)
        taps.append((f"pool{l}", x))
    x = double_conv(x, "mid")
    for l in range(levels, 0, -1):
        if up_convs is None:
            x = upsample2x(x)
        else:
            wu, tu = up_convs[levels - l]
            _, x = masked_binary_tconv_layer(x, wu, tu)
        taps.append((f"up{l}", x))
        sk = skips[l - 1]
        if x.shape[1:3] != sk.shape[1:3]:
            # frame size not a multiple of 2^levels: pooling dropped a row / column on the way
            # down, the up-sampled tensor is padded with zeros to the skip feature's size
            x = zero_pad_to(x, sk.shape[1], sk.shape[2])
        x = concat(sk, x)
        taps.append((f"cat{l}", x))
        x = double_conv(x, f"dec{l}")
    logits = classifier(x, cls_w, cls_b)
    return logits, taps


def batchnorm_sign(acc, gamma, beta, mean, var, eps, bias=None):
    """What the integer threshold of Algorithm 1 stands for (Sec. 3.2.2: it covers batch norm,
    bias and the binary activation): the layer's integer sums go through bias, inference-mode
    batch norm and the sign activation, all in float64, channel = last axis.
    Returns (y float64, +-1 int8 with y >= 0 -> +1)."""
    acc = np.asarray(acc, dtype=np.float64)
    g, b, m, v = (np.asarray(t, dtype=np.float64) for t in (gamma, beta, mean, var))
    z = acc if bias is None else acc + np.asarray(bias, dtype=np.float64)
    y = g * (z - m) / np.sqrt(v + eps) + b
    return y, np.where(y >= 0, 1, -1).astype(np.int8)


def cost_scores(n_ops, n_params, w_op):
    """Weighted cost score of every layer (Sec. 3.1.2): w_op * ops^ + (1 - w_op) * params^
    with the operation and parameter counts scaled to [0, 1] over the layers (smallest count
    -> 0, largest -> 1).  Returns (scores, indices by ascending score; ties by index)."""
    o = np.asarray(n_ops, dtype=np.float64)
    p = np.asarray(n_params, dtype=np.float64)

    def unit(v):
        span = v.max() - v.min()
        return (v - v.min()) / span if span > 0 else np.zeros_like(v)

    s = w_op * unit(o) + (1.0 - w_op) * unit(p)
    return s, np.argsort(s, kind="stable")
