"""A training step (forward + backward + SGD) recorded into a HIP graph by the caller and replayed:
the step's entry points only launch kernels on the stream they are given (no allocation, no copy, no
memset, no wait), so a capture of that stream holds the whole step.  Every replay is checked against
the same steps made eagerly on a second net, bit for bit (the kernels' summation orders are fixed),
with eager work and synchronisation between the replays."""
import numpy as np
import pytest
import torch

from paper_1302_1690_amd import mpcnn, workloads as wl

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_training_step_replayed_from_a_graph(dtype):
    cfg = wl.crop(wl.CONFIGS[1], 2, 120, 109)
    lr, scale, n_steps = 0.05, 1.0 / cfg.valid_pixels, 4
    img, lab = wl.make_inputs(cfg)
    params = wl.make_params(cfg)
    d_img = torch.from_numpy(img).cuda()
    d_lab = torch.from_numpy(lab).cuda()
    shape = (cfg.batch, cfg.n_classes, cfg.out_h, cfg.out_w)
    store = mpcnn.BF16 if dtype == "bf16" else mpcnn.F32

    def fresh():
        net = mpcnn.Net(cfg.layers, cfg.in_channels, cfg.patch, dtype=store)
        net.set_params(params)
        probs = torch.zeros(shape, dtype=torch.float32, device="cuda")
        loss = torch.zeros(1, dtype=torch.float64, device="cuda")
        ws = net.alloc_workspace(cfg.batch, cfg.height, cfg.width, True)
        return net, probs, loss, ws

    # ---- eager: n_steps steps, parameters and loss after each
    net, probs, loss, ws = fresh()
    want = []
    for _ in range(n_steps):
        net.seg_backward(d_img, d_lab, None, probs, loss, ws=ws)
        net.sgd_step(lr, scale)
        torch.cuda.synchronize()
        want.append((net.get_params(), float(loss.item()), probs.cpu().numpy()))
    net.close()
    assert np.abs(want[-1][0] - params).max() > 1e-4          # the steps do move the parameters

    # ---- graph: the first step eagerly (plans made, weight packs out of date as after any update),
    # then one step recorded and replayed for the others
    net, probs, loss, ws = fresh()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        net.seg_backward(d_img, d_lab, None, probs, loss, ws=ws)
        net.sgd_step(lr, scale)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(net.get_params(), want[0][0])
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        net.seg_backward(d_img, d_lab, None, probs, loss, ws=ws)
        net.sgd_step(lr, scale)
    np.testing.assert_array_equal(net.get_params(), want[0][0])    # recording runs nothing
    for k in range(1, n_steps):
        graph.replay()
        torch.cuda.synchronize()
        print("graph replay %d (%s)" % (k, dtype), flush=True)
        np.testing.assert_array_equal(net.get_params(), want[k][0])
        assert float(loss.item()) == want[k][1]
        np.testing.assert_array_equal(probs.cpu().numpy(), want[k][2])
        # eager work of the program's own between the replays
        junk = (d_img * 2.0).sum().item()
        assert np.isfinite(junk)
    net.close()
