"""The entry point that allocates nothing (mpcnn_seg_forward_static: the workspace is a fixed
array in the library's device image) against mpcnn_seg_forward on a caller-owned workspace:
same kernels, same plan, so the probabilities must agree bit for bit.  Two calls in a row, the
second on a smaller input (the array keeps the first call's contents), then a size it refuses."""
import numpy as np
import pytest
import torch

from paper_1302_1690_amd import mpcnn, workloads as wl

pytestmark = pytest.mark.gpu


def test_static_workspace_forward_matches_seg_forward():
    cfg = wl.CONFIGS[1]
    params = wl.make_params(cfg)
    net = mpcnn.Net(cfg.layers, cfg.in_channels, cfg.patch)
    net.set_params(params)
    for batch, h, w in ((2, 200, 231), (1, 97, 64)):
        c = wl.crop(cfg, batch, h, w)
        img, _ = wl.make_inputs(c)
        d_img = torch.from_numpy(img).cuda()
        assert net.workspace_bytes(batch, h, w, False) <= mpcnn.STATIC_WORKSPACE_BYTES
        want = net.seg_forward(d_img).cpu().numpy()
        got = torch.full((batch, cfg.n_classes, c.out_h, c.out_w), -1.0, dtype=torch.float32, device="cuda")
        before = torch.cuda.memory_allocated()
        net.seg_forward_static(d_img, got)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        print("static workspace forward %dx%dx%d" % (batch, h, w), flush=True)
        np.testing.assert_array_equal(got.cpu().numpy(), want)
    # a batch whose activations do not fit the fixed array is refused, nothing is launched
    big = wl.crop(cfg, 4, 600, 600)
    assert net.workspace_bytes(4, 600, 600, False) > mpcnn.STATIC_WORKSPACE_BYTES
    d_img = torch.zeros((4, 1, 600, 600), device="cuda")
    out = torch.zeros((4, cfg.n_classes, big.out_h, big.out_w), device="cuda")
    with pytest.raises(mpcnn.MpcnnError) as e:
        net.seg_forward_static(d_img, out)
    assert e.value.status == 3
    net.close()
