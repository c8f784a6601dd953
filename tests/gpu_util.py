"""Helpers for the GPU parity tests (host <-> device copies, strip checks)."""
import sys

import numpy as np
import torch

from oracle import oracle as O
from tests import bitref


def say(msg):
    """Name the case before touching the GPU, flushed, so a fault can be attributed."""
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host_u32(t):
    return t.detach().cpu().numpy().view(np.uint32)


def host(t):
    return t.detach().cpu().numpy()


def check_conv_rows(in_packed, cin, w, theta, out_packed, n, r0, r1, label=""):
    """Compare rows [r0,r1) of image n of a GPU layer output (packed, host uint32 array
    [N,H,W,Cout/32]) with the oracle run on the unpacked rows it depends on."""
    N, H, W, _ = in_packed.shape
    c0, c1 = max(0, r0 - 1), min(H, r1 + 1)
    a = bitref.unpack_pm1(in_packed[n:n + 1, c0:c1], cin)
    # the strip is treated by the oracle as an image of its own; rows r0..r1 see the same
    # neighbours as in the full image because the context rows are included (or are the
    # true image border).
    _, out = O.masked_binary_layer(a, w, theta)
    exp = bitref.pack_pm1(out[:, r0 - c0:r1 - c0])
    got = out_packed[n:n + 1, r0:r1]
    bad = int((exp != got).sum())
    assert bad == 0, f"{label}: {bad} packed words differ in rows {r0}..{r1} of image {n}"
