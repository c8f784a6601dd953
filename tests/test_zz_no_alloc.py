"""The entry point that allocates nothing (mbu_unet_forward_static: the workspace is a fixed
device array inside the library) against mbu_unet_forward on the same inputs and against the
oracle, on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_2601_11660_amd import binding as B
from paper_2601_11660_amd import synth
from tests.gpu_util import dev, host, say

pytestmark = pytest.mark.gpu


def _net(case):
    return B.UNet(dev(case.stem_w), [(dev(w), dev(t)) for w, t in case.convs], dev(case.cls_w),
                  dev(case.cls_b), levels=case.levels)


def test_static_workspace_forward_matches_the_caller_workspace_forward():
    B.set_conv_path(B.PATH_AUTO)
    B.set_conv_tuning(0)
    # first the largest shape that fits (the 512 x 512 network), then a smaller odd-sized one:
    # the second call finds the first call's data in the array
    shapes = [(1, 512, 512, 4), (2, 70, 101, 3)]
    for N, H, W, levels in shapes:
        say(f"static workspace forward N={N} H={H} W={W} levels={levels}")
        case = synth.unet_case(2, 0, N, H, W, levels=levels)
        net = _net(case)
        assert net.workspace_bytes(N, H, W) <= B.STATIC_WORKSPACE_BYTES
        image = dev(case.image)
        ref = net.forward(image)
        out = torch.full((N, case.n_classes, H, W), float("nan"), dtype=torch.float32, device="cuda")
        got = net.forward_static(image, out)
        torch.cuda.synchronize()
        assert got.data_ptr() == out.data_ptr()
        got, ref = host(got), host(ref)
        assert np.array_equal(got, ref), "differs from mbu_unet_forward"
        ref_logits, _ = O.unet_forward(case.image, case.stem_w, case.convs, case.cls_w, case.cls_b,
                                       levels=levels)
        err = np.abs(got - ref_logits)
        assert (err <= 1e-4 * np.maximum(1.0, np.abs(ref_logits))).all(), float(err.max())


def test_static_workspace_forward_rejects_shapes_beyond_its_maximum():
    say("static workspace forward: too large")
    case = synth.unet_case(2, 0, 1, 64, 64, levels=4)
    net = _net(case)
    big = torch.zeros((1, 3, 1024, 1024), dtype=torch.float32, device="cuda")
    out = torch.zeros((1, case.n_classes, 1024, 1024), dtype=torch.float32, device="cuda")
    with pytest.raises(B.MbuError) as e:
        net.forward_static(big, out)
    assert e.value.code == B.MBU_ERR_WORKSPACE
