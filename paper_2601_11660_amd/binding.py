"""Thin ctypes binding over the C ABI declared in include/mbu.h.

Argument marshalling only: every step of the path runs in the HIP kernels of
libmbu_hip.so.  PyTorch supplies device memory and the current stream, nothing else.
There is no CPU fallback: if the library has not been built, importing the entry
points raises.
"""
import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmbu_hip.so")

MBU_OK = 0
MBU_ERR_NULL, MBU_ERR_SHAPE, MBU_ERR_ALIGN, MBU_ERR_WORKSPACE, MBU_ERR_HIP, MBU_ERR_ARG = -1, -2, -3, -4, -5, -6
PATH_AUTO, PATH_VALU, PATH_MFMA = 0, 1, 2
STEM_AUTO, STEM_VALU, STEM_MFMA, STEM_MFMA_GATHER = 0, 1, 2, 3
STATIC_WORKSPACE_BYTES = 32 << 20
BLOB_BIT_PLANES, BLOB_SUMMED_TAPS, BLOB_MATRIX, BLOB_ALL = 1, 2, 4, 7

EXPORTS = [
    "mbu_last_error", "mbu_set_conv_path", "mbu_get_conv_path", "mbu_set_conv_tuning", "mbu_pack_act",
    "mbu_set_stem_path", "mbu_get_stem_path", "mbu_stem_fp32", "mbu_classifier_fp32",
    "mbu_fold_batchnorm", "mbu_cost_rank",
    "mbu_packed_weights_bytes", "mbu_pack_weights", "mbu_conv3x3_masked_binary",
    "mbu_packed_weights_bytes_sections", "mbu_pack_weights_sections",
    "mbu_conv3x3_masked_binary_fused", "mbu_conv3x3_masked_binary_concat",
    "mbu_conv3x3_masked_binary_two_inputs", "mbu_unet_step_kernel",
    "mbu_packed_tconv_weights_bytes", "mbu_pack_tconv_weights", "mbu_tconv2x2_masked_binary",
    "mbu_maxpool2x2_bits", "mbu_upsample2x_bits", "mbu_concat_bits", "mbu_unet_num_steps",
    "mbu_unet_step_info", "mbu_unet_step_launches", "mbu_unet_workspace_bytes", "mbu_unet_forward",
    "mbu_unet_forward_static",
    "mbu_event_create", "mbu_event_destroy", "mbu_event_record", "mbu_event_elapsed_ms",
]


class MbuError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"mbu error {code}: {msg}")
        self.code = code


class ConvLayer(ctypes.Structure):
    _fields_ = [("packed_w", ctypes.c_void_p), ("thresh", ctypes.c_void_p),
                ("cin", ctypes.c_int), ("cout", ctypes.c_int), ("sections", ctypes.c_int)]


class UNetDesc(ctypes.Structure):
    _fields_ = [("levels", ctypes.c_int), ("base", ctypes.c_int),
                ("in_channels", ctypes.c_int), ("n_classes", ctypes.c_int),
                ("stem_w", ctypes.c_void_p), ("convs", ctypes.POINTER(ConvLayer)),
                ("cls_w", ctypes.c_void_p), ("cls_b", ctypes.c_void_p),
                ("step_events", ctypes.POINTER(ctypes.c_void_p)), ("fuse", ctypes.c_int),
                ("up_convs", ctypes.POINTER(ConvLayer))]


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it first "
                               "(python -m paper_2601_11660_amd.build); there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        L.mbu_last_error.restype = ctypes.c_char_p
        vp, ci = ctypes.c_void_p, ctypes.c_int
        L.mbu_pack_act.argtypes = [vp, ci, ci, ci, ci, ci, vp, vp]
        L.mbu_packed_weights_bytes.argtypes = [ci, ci, ctypes.POINTER(ctypes.c_size_t)]
        L.mbu_pack_weights.argtypes = [vp, ci, ci, vp, vp]
        L.mbu_packed_weights_bytes_sections.argtypes = [ci, ci, ci, ctypes.POINTER(ctypes.c_size_t)]
        L.mbu_pack_weights_sections.argtypes = [vp, ci, ci, ci, vp, vp]
        L.mbu_conv3x3_masked_binary.argtypes = [vp, ci, ci, ci, ci, vp, ci, vp, vp, vp, vp]
        L.mbu_conv3x3_masked_binary_fused.argtypes = [vp, ci, vp, ci, ci, ci, ci, vp, ci, vp, vp, vp, vp]
        L.mbu_conv3x3_masked_binary_concat.argtypes = [vp, ci, vp, ci, ci, ci, ci, vp, ci, vp, vp, vp, vp]
        L.mbu_conv3x3_masked_binary_two_inputs.argtypes = [vp, ci, vp, ci, ci, ci, ci, ci, ci, ci, vp, ci,
                                                           vp, vp, vp, vp]
        L.mbu_packed_tconv_weights_bytes.argtypes = [ci, ci, ctypes.POINTER(ctypes.c_size_t)]
        L.mbu_pack_tconv_weights.argtypes = [vp, ci, ci, vp, vp]
        L.mbu_tconv2x2_masked_binary.argtypes = [vp, ci, ci, ci, ci, vp, ci, vp, vp, vp, vp]
        L.mbu_stem_fp32.argtypes = [vp, ci, ci, ci, ci, vp, ci, vp, vp, vp]
        L.mbu_classifier_fp32.argtypes = [vp, ci, ci, ci, ci, vp, vp, ci, vp, vp]
        dp = ctypes.POINTER(ctypes.c_double)
        L.mbu_fold_batchnorm.argtypes = [dp, dp, dp, dp, ctypes.c_double, dp, ci, ci,
                                         ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int8)]
        L.mbu_cost_rank.argtypes = [dp, dp, ci, ctypes.c_double, dp, ctypes.POINTER(ci)]
        L.mbu_maxpool2x2_bits.argtypes = [vp, ci, ci, ci, ci, vp, vp]
        L.mbu_upsample2x_bits.argtypes = [vp, ci, ci, ci, ci, vp, vp]
        L.mbu_concat_bits.argtypes = [vp, ci, vp, ci, ci, ci, ci, vp, vp]
        L.mbu_unet_num_steps.argtypes = [ctypes.POINTER(UNetDesc)]
        L.mbu_unet_step_info.argtypes = [ctypes.POINTER(UNetDesc), ci, ci, ci, ci,
                                         ctypes.POINTER(ctypes.c_char_p),
                                         ctypes.POINTER(ctypes.c_size_t),
                                         ctypes.POINTER(ci), ctypes.POINTER(ci), ctypes.POINTER(ci)]
        L.mbu_unet_step_launches.argtypes = [ctypes.POINTER(UNetDesc), ci, ci, ci, ci]
        L.mbu_unet_step_kernel.argtypes = [ctypes.POINTER(UNetDesc), ci, ci, ci, ci,
                                           ctypes.POINTER(ctypes.c_char_p)]
        L.mbu_unet_workspace_bytes.argtypes = [ctypes.POINTER(UNetDesc), ci, ci, ci,
                                               ctypes.POINTER(ctypes.c_size_t)]
        L.mbu_unet_forward.argtypes = [ctypes.POINTER(UNetDesc), vp, ci, ci, ci, vp, vp,
                                       ctypes.c_size_t, vp]
        L.mbu_unet_forward_static.argtypes = [ctypes.POINTER(UNetDesc), vp, ci, ci, ci, vp, vp]
        L.mbu_event_create.argtypes = [ctypes.POINTER(vp)]
        L.mbu_event_destroy.argtypes = [vp]
        L.mbu_event_record.argtypes = [vp, vp]
        L.mbu_event_elapsed_ms.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_float)]
        _lib = L
    return _lib


def last_error() -> str:
    return lib().mbu_last_error().decode()


def check(rc: int) -> None:
    if rc != MBU_OK:
        raise MbuError(rc, last_error())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, dtypes) -> int:
    if not t.is_cuda:
        raise ValueError("expected a device tensor")
    if t.dtype not in dtypes:
        raise ValueError(f"expected dtype in {dtypes}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError("expected a contiguous tensor")
    return t.data_ptr()


def set_conv_path(path: int) -> None:
    check(lib().mbu_set_conv_path(path))


def get_conv_path() -> int:
    return lib().mbu_get_conv_path()


def set_conv_tuning(kernel: int = 0) -> None:
    """mbu_set_conv_tuning: 0 automatic, 1 block-cooperative, 3 / 6 wave-private variants."""
    check(lib().mbu_set_conv_tuning(kernel, 0))


def set_stem_path(path: int) -> None:
    check(lib().mbu_set_stem_path(path))


def get_stem_path() -> int:
    return lib().mbu_get_stem_path()


def stem_fp32(image: torch.Tensor, w: torch.Tensor, want_pre: bool = False
              ) -> Tuple[torch.Tensor, Optional[torch.Tensor]]:
    """mbu_stem_fp32: image float32 NCHW, w float32 [Co,3,3,Ci] -> (packed bits [N,H,W,Co/32],
    float32 NHWC pre-activations or None)."""
    N, Ci, H, W = image.shape
    Co = w.shape[0]
    bits = torch.empty((N, H, W, Co // 32), dtype=torch.int32, device=image.device)
    pre = torch.empty((N, H, W, Co), dtype=torch.float32, device=image.device) if want_pre else None
    check(lib().mbu_stem_fp32(_dev(image, (torch.float32,)), N, Ci, H, W, _dev(w, (torch.float32,)),
                              Co, bits.data_ptr(), pre.data_ptr() if pre is not None else None,
                              _stream()))
    return bits, pre


def classifier_fp32(act: torch.Tensor, c: int, w: torch.Tensor, b: torch.Tensor) -> torch.Tensor:
    """mbu_classifier_fp32: packed bits [N,H,W,C/32], w [K,C], b [K] -> float32 logits NCHW."""
    N, H, W, _ = act.shape
    K = w.shape[0]
    out = torch.empty((N, K, H, W), dtype=torch.float32, device=act.device)
    check(lib().mbu_classifier_fp32(_dev(act, (torch.int32,)), N, H, W, c, _dev(w, (torch.float32,)),
                                    _dev(b, (torch.float32,)), K, out.data_ptr(), _stream()))
    return out


def fold_batchnorm(gamma, beta, mean, var, eps: float, bias, fan_in: int):
    """mbu_fold_batchnorm on host arrays -> (int32 thresholds, int8 flip flags) as numpy arrays."""
    import numpy as np

    def arr(a):
        return np.ascontiguousarray(a, dtype=np.float64)

    g, b, m, v = arr(gamma), arr(beta), arr(mean), arr(var)
    C = g.shape[0]
    bs = arr(bias) if bias is not None else None
    thresh = np.empty(C, np.int32)
    flip = np.empty(C, np.int8)
    dp = ctypes.POINTER(ctypes.c_double)

    def ptr(a):
        return a.ctypes.data_as(dp)

    check(lib().mbu_fold_batchnorm(ptr(g), ptr(b), ptr(m), ptr(v), float(eps),
                                   ptr(bs) if bs is not None else None, C, int(fan_in),
                                   thresh.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                   flip.ctypes.data_as(ctypes.POINTER(ctypes.c_int8))))
    return thresh, flip


def cost_rank(n_ops, n_params, w_op: float = 0.5):
    """mbu_cost_rank on host arrays -> (scores float64, order int32) as numpy arrays."""
    import numpy as np
    o = np.ascontiguousarray(n_ops, dtype=np.float64)
    p = np.ascontiguousarray(n_params, dtype=np.float64)
    L = o.shape[0]
    score = np.empty(L, np.float64)
    order = np.empty(L, np.int32)
    dp = ctypes.POINTER(ctypes.c_double)
    check(lib().mbu_cost_rank(o.ctypes.data_as(dp), p.ctypes.data_as(dp), L, float(w_op),
                              score.ctypes.data_as(dp), order.ctypes.data_as(ctypes.POINTER(ctypes.c_int))))
    return score, order


# Packed words are stored in int32 tensors (same bits as the ABI's uint32).
def pack_act(x: torch.Tensor) -> torch.Tensor:
    """mbu_pack_act: NHWC int8 (bit = v > 0) or float32 (bit = v >= 0) -> [N,H,W,ceil(C/32)]."""
    N, H, W, C = x.shape
    dt = 0 if x.dtype == torch.int8 else 1
    out = torch.empty((N, H, W, (C + 31) // 32), dtype=torch.int32, device=x.device)
    check(lib().mbu_pack_act(_dev(x, (torch.int8, torch.float32)), dt, N, H, W, C,
                             out.data_ptr(), _stream()))
    return out


def packed_weights_bytes(cout: int, cin: int, sections: int = BLOB_ALL) -> int:
    n = ctypes.c_size_t(0)
    check(lib().mbu_packed_weights_bytes_sections(cout, cin, sections, ctypes.byref(n)))
    return n.value


def pack_weights(w_ohwi: torch.Tensor, sections: int = BLOB_ALL) -> torch.Tensor:
    """mbu_pack_weights(_sections): device int8 [Cout,3,3,Cin] in {-1,0,+1} -> opaque blob
    (uint8 tensor) holding the given sections."""
    cout, kh, kw, cin = w_ohwi.shape
    assert kh == 3 and kw == 3
    blob = torch.empty(packed_weights_bytes(cout, cin, sections), dtype=torch.uint8, device=w_ohwi.device)
    check(lib().mbu_pack_weights_sections(_dev(w_ohwi, (torch.int8,)), cout, cin, sections,
                                          blob.data_ptr(), _stream()))
    return blob


def conv3x3_masked_binary(act: torch.Tensor, cin: int, packed_w: torch.Tensor, cout: int,
                          thresh: torch.Tensor, want_bits: bool = True, want_acc: bool = False,
                          out_bits: Optional[torch.Tensor] = None,
                          out_acc: Optional[torch.Tensor] = None
                          ) -> Tuple[Optional[torch.Tensor], Optional[torch.Tensor]]:
    """mbu_conv3x3_masked_binary -> (packed bits [N,H,W,Cout/32] or None, int32 acc NHWC or None)."""
    N, H, W, _ = act.shape
    if want_bits and out_bits is None:
        out_bits = torch.empty((N, H, W, cout // 32), dtype=torch.int32, device=act.device)
    if want_acc and out_acc is None:
        out_acc = torch.empty((N, H, W, cout), dtype=torch.int32, device=act.device)
    check(lib().mbu_conv3x3_masked_binary(
        _dev(act, (torch.int32,)), N, H, W, cin, _dev(packed_w, (torch.uint8,)), cout,
        _dev(thresh, (torch.int32,)),
        out_bits.data_ptr() if out_bits is not None else None,
        out_acc.data_ptr() if out_acc is not None else None, _stream()))
    return out_bits, out_acc


def conv3x3_masked_binary_fused(act: torch.Tensor, ca: int, low: Optional[torch.Tensor], clow: int,
                                packed_w: torch.Tensor, cout: int, thresh: torch.Tensor,
                                want_bits: bool = True, want_pool: bool = False
                                ) -> Tuple[Optional[torch.Tensor], Optional[torch.Tensor]]:
    """mbu_conv3x3_masked_binary_fused -> (packed bits or None, 2x2-pooled packed bits or None)."""
    N, H, W, _ = act.shape
    out_bits = (torch.empty((N, H, W, cout // 32), dtype=torch.int32, device=act.device)
                if want_bits else None)
    out_pool = (torch.empty((N, H // 2, W // 2, cout // 32), dtype=torch.int32, device=act.device)
                if want_pool else None)
    check(lib().mbu_conv3x3_masked_binary_fused(
        _dev(act, (torch.int32,)), ca, _dev(low, (torch.int32,)) if low is not None else None, clow,
        N, H, W, _dev(packed_w, (torch.uint8,)), cout, _dev(thresh, (torch.int32,)),
        out_bits.data_ptr() if out_bits is not None else None,
        out_pool.data_ptr() if out_pool is not None else None, _stream()))
    return out_bits, out_pool


def conv3x3_masked_binary_concat(a: torch.Tensor, ca: int, b: torch.Tensor, cb: int,
                                 packed_w: torch.Tensor, cout: int, thresh: torch.Tensor,
                                 want_pool: bool = False):
    """mbu_conv3x3_masked_binary_concat -> (packed bits, pooled packed bits or None)."""
    N, H, W, _ = a.shape
    out_bits = torch.empty((N, H, W, cout // 32), dtype=torch.int32, device=a.device)
    out_pool = (torch.empty((N, H // 2, W // 2, cout // 32), dtype=torch.int32, device=a.device)
                if want_pool else None)
    check(lib().mbu_conv3x3_masked_binary_concat(
        _dev(a, (torch.int32,)), ca, _dev(b, (torch.int32,)), cb, N, H, W,
        _dev(packed_w, (torch.uint8,)), cout, _dev(thresh, (torch.int32,)), out_bits.data_ptr(),
        out_pool.data_ptr() if out_pool is not None else None, _stream()))
    return out_bits, out_pool


def conv3x3_masked_binary_two_inputs(a: torch.Tensor, ca: int, b: torch.Tensor, cb: int,
                                     upsample: bool, packed_w: torch.Tensor, cout: int,
                                     thresh: torch.Tensor, want_pool: bool = False):
    """mbu_conv3x3_masked_binary_two_inputs: b [N,Hb,Wb,ceil(cb/32)] may cover less than the
    frame of a -> (packed bits, pooled packed bits or None)."""
    N, H, W, _ = a.shape
    out_bits = torch.empty((N, H, W, cout // 32), dtype=torch.int32, device=a.device)
    out_pool = (torch.empty((N, H // 2, W // 2, cout // 32), dtype=torch.int32, device=a.device)
                if want_pool else None)
    check(lib().mbu_conv3x3_masked_binary_two_inputs(
        _dev(a, (torch.int32,)), ca, _dev(b, (torch.int32,)), cb, b.shape[1], b.shape[2],
        1 if upsample else 0, N, H, W, _dev(packed_w, (torch.uint8,)), cout,
        _dev(thresh, (torch.int32,)), out_bits.data_ptr(),
        out_pool.data_ptr() if out_pool is not None else None, _stream()))
    return out_bits, out_pool


def pack_tconv_weights(w: torch.Tensor) -> torch.Tensor:
    """mbu_pack_tconv_weights: device int8 [Cout,2,2,Cin] -> opaque blob (uint8 tensor)."""
    cout, kh, kw, cin = w.shape
    assert kh == 2 and kw == 2
    n = ctypes.c_size_t(0)
    check(lib().mbu_packed_tconv_weights_bytes(cout, cin, ctypes.byref(n)))
    blob = torch.empty(n.value, dtype=torch.uint8, device=w.device)
    check(lib().mbu_pack_tconv_weights(_dev(w, (torch.int8,)), cout, cin, blob.data_ptr(), _stream()))
    return blob


def tconv2x2_masked_binary(act: torch.Tensor, cin: int, packed_w: torch.Tensor, cout: int,
                           thresh: torch.Tensor, want_bits: bool = True, want_acc: bool = False):
    """mbu_tconv2x2_masked_binary -> (packed bits [N,2H,2W,Cout/32] or None, int32 acc or None)."""
    N, H, W, _ = act.shape
    out_bits = (torch.empty((N, 2 * H, 2 * W, cout // 32), dtype=torch.int32, device=act.device)
                if want_bits else None)
    out_acc = (torch.empty((N, 2 * H, 2 * W, cout), dtype=torch.int32, device=act.device)
               if want_acc else None)
    check(lib().mbu_tconv2x2_masked_binary(
        _dev(act, (torch.int32,)), N, H, W, cin, _dev(packed_w, (torch.uint8,)), cout,
        _dev(thresh, (torch.int32,)), out_bits.data_ptr() if out_bits is not None else None,
        out_acc.data_ptr() if out_acc is not None else None, _stream()))
    return out_bits, out_acc


def maxpool2x2_bits(x: torch.Tensor, c: int) -> torch.Tensor:
    N, H, W, Cw = x.shape
    out = torch.empty((N, H // 2, W // 2, Cw), dtype=torch.int32, device=x.device)
    check(lib().mbu_maxpool2x2_bits(_dev(x, (torch.int32,)), N, H, W, c, out.data_ptr(), _stream()))
    return out


def upsample2x_bits(x: torch.Tensor, c: int) -> torch.Tensor:
    N, H, W, Cw = x.shape
    out = torch.empty((N, 2 * H, 2 * W, Cw), dtype=torch.int32, device=x.device)
    check(lib().mbu_upsample2x_bits(_dev(x, (torch.int32,)), N, H, W, c, out.data_ptr(), _stream()))
    return out


def concat_bits(a: torch.Tensor, ca: int, b: torch.Tensor, cb: int) -> torch.Tensor:
    N, H, W, Caw = a.shape
    out = torch.empty((N, H, W, Caw + b.shape[3]), dtype=torch.int32, device=a.device)
    check(lib().mbu_concat_bits(_dev(a, (torch.int32,)), ca, _dev(b, (torch.int32,)), cb, N, H, W,
                                out.data_ptr(), _stream()))
    return out


class Event:
    """HIP event recorded on a given stream through the library's helpers."""

    def __init__(self):
        h = ctypes.c_void_p()
        check(lib().mbu_event_create(ctypes.byref(h)))
        self.handle = h

    def record(self, stream: Optional[int] = None):
        check(lib().mbu_event_record(self.handle, _stream() if stream is None else stream))

    def elapsed_ms(self, stop: "Event") -> float:
        ms = ctypes.c_float()
        check(lib().mbu_event_elapsed_ms(self.handle, stop.handle, ctypes.byref(ms)))
        return ms.value

    def __del__(self):
        try:
            lib().mbu_event_destroy(self.handle)
        except Exception:
            pass


class EventSet:
    """Events plus the host array of their handles that the descriptor points to."""

    def __init__(self, n: int):
        self.events = [Event() for _ in range(n)]
        self.array = (ctypes.c_void_p * n)(*[e.handle.value for e in self.events])


class UNet:
    """Owner of the device tensors and the host descriptor for mbu_unet_forward."""

    def __init__(self, stem_w: torch.Tensor, convs: Sequence[Tuple[torch.Tensor, torch.Tensor]],
                 cls_w: torch.Tensor, cls_b: torch.Tensor, levels: int = 4, fuse: bool = True,
                 up_convs: Optional[Sequence[Tuple[torch.Tensor, torch.Tensor]]] = None,
                 all_sections: bool = False):
        """stem_w float32 [base,3,3,Ci]; convs: (w int8 OHWI, theta int32) device tensors in
        execution order; cls_w float32 [K,base]; cls_b float32 [K].  Every layer's blob holds
        only the sections its place in the network reads (the bit planes when the vector-ALU
        path is selected at construction, the summed taps for the first layer of a decoder level
        that up-samples nearest-neighbour) unless all_sections is set."""
        self.levels = levels
        self.base = stem_w.shape[0]
        self.in_channels = stem_w.shape[3]
        self.n_classes = cls_w.shape[0]
        self.stem_w = stem_w.contiguous()
        self.cls_w = cls_w.contiguous()
        self.cls_b = cls_b.contiguous()
        self.blobs: List[torch.Tensor] = []
        self.thetas: List[torch.Tensor] = []
        self.shapes: List[Tuple[int, int]] = []
        self.sections: List[int] = []
        planes = BLOB_BIT_PLANES if get_conv_path() == PATH_VALU else 0
        for i, (w, th) in enumerate(convs):
            first_of_decoder_level = i >= 2 * levels + 2 and i % 2 == 0
            sec = BLOB_ALL if all_sections else (
                BLOB_MATRIX | planes | (BLOB_SUMMED_TAPS if first_of_decoder_level and up_convs is None else 0))
            self.sections.append(sec)
            self.blobs.append(pack_weights(w.contiguous(), sec))
            self.thetas.append(th.contiguous())
            self.shapes.append((w.shape[3], w.shape[0]))
        n = len(self.blobs)
        self._layers = (ConvLayer * n)()
        for i in range(n):
            self._layers[i].packed_w = self.blobs[i].data_ptr()
            self._layers[i].thresh = self.thetas[i].data_ptr()
            self._layers[i].cin, self._layers[i].cout = self.shapes[i]
            self._layers[i].sections = self.sections[i]
        self._up_layers = None
        self.up_blobs: List[torch.Tensor] = []
        self.up_thetas: List[torch.Tensor] = []
        if up_convs is not None:
            # transposed decoder: (w int8 [Cout,2,2,Cin], theta int32) per level, deepest first
            assert len(up_convs) == levels
            self._up_layers = (ConvLayer * levels)()
            for i, (w, th) in enumerate(up_convs):
                self.up_blobs.append(pack_tconv_weights(w.contiguous()))
                self.up_thetas.append(th.contiguous())
                self._up_layers[i].packed_w = self.up_blobs[i].data_ptr()
                self._up_layers[i].thresh = self.up_thetas[i].data_ptr()
                self._up_layers[i].cin, self._up_layers[i].cout = w.shape[3], w.shape[0]
        self.desc = UNetDesc(levels=levels, base=self.base, in_channels=self.in_channels,
                             n_classes=self.n_classes, stem_w=self.stem_w.data_ptr(),
                             convs=self._layers, cls_w=self.cls_w.data_ptr(),
                             cls_b=self.cls_b.data_ptr(), step_events=None,
                             fuse=1 if fuse else 0, up_convs=self._up_layers)
        self.num_steps = lib().mbu_unet_num_steps(ctypes.byref(self.desc))
        if self.num_steps < 0:
            check(self.num_steps)
        self._events: Optional[EventSet] = None
        self.workspace: Optional[torch.Tensor] = None

    def clone_for_stream(self) -> "UNet":
        """A second handle on the same network for another frame in flight: shares the weight
        blobs, thresholds and float weights (read-only), owns its descriptor, events and
        workspace.  Forward passes of the two handles may overlap on different streams."""
        import copy
        other = copy.copy(self)
        other.desc = UNetDesc(levels=self.levels, base=self.base, in_channels=self.in_channels,
                              n_classes=self.n_classes, stem_w=self.stem_w.data_ptr(),
                              convs=self._layers, cls_w=self.cls_w.data_ptr(),
                              cls_b=self.cls_b.data_ptr(), step_events=None,
                              fuse=self.desc.fuse, up_convs=self._up_layers)
        other._events = None
        other.workspace = None
        return other

    def workspace_bytes(self, N: int, H: int, W: int) -> int:
        n = ctypes.c_size_t(0)
        check(lib().mbu_unet_workspace_bytes(ctypes.byref(self.desc), N, H, W, ctypes.byref(n)))
        return n.value

    def new_event_set(self) -> "EventSet":
        """A fresh set of num_steps+1 events for one forward pass."""
        return EventSet(self.num_steps + 1)

    def use_event_set(self, es: Optional["EventSet"]) -> None:
        """Make the next forward passes record their per-step events into `es`
        (None switches event recording off)."""
        self._events = es
        self.desc.step_events = (ctypes.cast(es.array, ctypes.POINTER(ctypes.c_void_p))
                                 if es is not None else None)

    def enable_step_events(self, on: bool = True) -> None:
        self.use_event_set(self.new_event_set() if on else None)

    def step_launches(self, N: int, H: int, W: int, step: int) -> bool:
        rc = lib().mbu_unet_step_launches(ctypes.byref(self.desc), N, H, W, step)
        if rc < 0:
            check(rc)
        return rc == 1

    def step_kernel(self, N: int, H: int, W: int, step: int) -> str:
        """Name of the kernel the step launches for this shape ("" if it launches none)."""
        name = ctypes.c_char_p()
        check(lib().mbu_unet_step_kernel(ctypes.byref(self.desc), N, H, W, step, ctypes.byref(name)))
        return name.value.decode()

    def step_times_ms(self, N: int, H: int, W: int, es: Optional["EventSet"] = None) -> List[float]:
        """Per-step durations of the last forward pass recorded into `es`; steps folded into
        a neighbouring layer report 0."""
        es = es if es is not None else self._events
        assert es is not None
        live = [i for i in range(self.num_steps) if self.step_launches(N, H, W, i)]
        out = [0.0] * self.num_steps
        for a, b in zip(live, live[1:] + [self.num_steps]):
            out[a] = es.events[a].elapsed_ms(es.events[b])
        return out

    def step_info(self, N: int, H: int, W: int, step: int):
        name = ctypes.c_char_p()
        off = ctypes.c_size_t()
        h, w, c = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
        check(lib().mbu_unet_step_info(ctypes.byref(self.desc), N, H, W, step, ctypes.byref(name),
                                       ctypes.byref(off), ctypes.byref(h), ctypes.byref(w),
                                       ctypes.byref(c)))
        return name.value.decode(), off.value, h.value, w.value, c.value

    def forward(self, image: torch.Tensor, logits: Optional[torch.Tensor] = None) -> torch.Tensor:
        N, Ci, H, W = image.shape
        need = self.workspace_bytes(N, H, W)
        if self.workspace is None or self.workspace.numel() < need:
            self.workspace = torch.empty(need, dtype=torch.uint8, device=image.device)
        if logits is None:
            logits = torch.empty((N, self.n_classes, H, W), dtype=torch.float32, device=image.device)
        check(lib().mbu_unet_forward(ctypes.byref(self.desc), _dev(image, (torch.float32,)), N, H, W,
                                     logits.data_ptr(), self.workspace.data_ptr(),
                                     self.workspace.numel(), _stream()))
        return logits

    def forward_static(self, image: torch.Tensor, logits: torch.Tensor) -> torch.Tensor:
        """mbu_unet_forward_static: the forward pass on the library's own fixed workspace.
        Nothing is allocated here either: the caller passes the logits tensor."""
        N, Ci, H, W = image.shape
        if tuple(logits.shape) != (N, self.n_classes, H, W):
            raise ValueError("logits must be [N, n_classes, H, W]")
        check(lib().mbu_unet_forward_static(ctypes.byref(self.desc), _dev(image, (torch.float32,)),
                                            N, H, W, _dev(logits, (torch.float32,)), _stream()))
        return logits

    def step_output(self, N: int, H: int, W: int, step: int) -> torch.Tensor:
        """Packed output of a step of the last forward pass, as an int32 view [N,h,w,c/32]."""
        _, off, h, w, c = self.step_info(N, H, W, step)
        n = N * h * w * (c // 32) * 4
        return self.workspace[off:off + n].view(torch.int32).view(N, h, w, c // 32)
