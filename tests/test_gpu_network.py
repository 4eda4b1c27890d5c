"""GPU parity of the chained networks (ResNet-18-, AlexNet- and VGG-16-shaped): every node's packed codes and
the int32 logits bit-exact against the chained oracle."""
import numpy as np
import pytest
import torch

from oracle import network as onet
from paper_2106_12169_amd import binding as B
from paper_2106_12169_amd import workloads as wl
from paper_2106_12169_amd.network import PackedNet
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def _check_all_nodes(layers, net, want, batch):
    for L in layers:
        got = hp.words_u32(net.buf[L.name])
        if L.kind == "fc":
            assert np.array_equal(net.buf[L.name].cpu().numpy(), want[L.name]), L.name
        elif L.kind == "sumpool" and L.name == net.fused_tail:
            continue                                    # computed inside the last layer's launch: no buffer of its own
        elif L.kind == "sumpool":
            codes, pad = hp.unpack_matrix(got, batch, L.Cout, L.q_out)
            assert np.array_equal(codes, want[L.name]) and pad == 0, L.name
        else:
            div = 2 if (L.kind == "conv" and L.pool) else 1
            codes, pad = hp.unpack_fmap(got, batch, L.Ho // div, L.Wo // div, L.Cout, L.q_out)
            assert codes.shape == want[L.name].shape, L.name
            assert np.array_equal(codes, want[L.name]) and pad == 0, L.name


@pytest.mark.parametrize("fuse_tail", [False, True])
def test_small_network_every_node(fuse_tail):
    layers = wl.resnet18_layers(image_hw=64, num_classes=100, widths=(32, 64, 96, 128))
    params = wl.network_params(layers, seed=1)
    img = wl.image_batch(3, 2, 64)
    net = PackedNet(layers, params, 2, fuse_tail=fuse_tail)
    assert (net.fused_tail is not None) == fuse_tail
    net.forward(torch.from_numpy(img).cuda())
    torch.cuda.synchronize()
    _check_all_nodes(layers, net, onet.run(layers, params, img), 2)


def test_resnet18_shape_batch8_logits_and_graph_replay():
    """Configuration 4 at full size, eagerly and as a HIP-graph replay."""
    layers = wl.resnet18_layers()
    params = wl.network_params(layers)
    img = wl.image_batch(2004, 8, 224)
    net = PackedNet(layers, params, 8)
    d_img = torch.from_numpy(img).cuda()
    logits = net.forward(d_img).clone()
    torch.cuda.synchronize()
    want = onet.run(layers, params, img)
    _check_all_nodes(layers, net, want, 8)
    assert np.array_equal(logits.cpu().numpy(), want["fc"])
    # graph capture of the same launches; replays must reproduce the eager result
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        net.forward(d_img)
    torch.cuda.current_stream().wait_stream(s)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        net.forward(d_img)
    for _ in range(3):
        net.buf["fc"].zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(net.buf["fc"].cpu().numpy(), want["fc"])


def test_resnet18_shape_batch32_every_node():
    """A larger batch takes other kernel variants (one tile per wave instead of K split over a block's waves, no
    paired launches for the early stages): every node against the chained oracle again."""
    layers = wl.resnet18_layers()
    params = wl.network_params(layers)
    img = wl.image_batch(2005, 32, 224)
    net = PackedNet(layers, params, 32, fuse_tail=False)
    logits = net.forward(torch.from_numpy(img).cuda())
    torch.cuda.synchronize()
    want = onet.run(layers, params, img)
    _check_all_nodes(layers, net, want, 32)
    assert np.array_equal(logits.cpu().numpy(), want["fc"])


@pytest.mark.parametrize("make,kw,hw,batch", [
    (wl.alexnet_layers, dict(num_classes=50, widths=(32, 64, 96, 64, 64), fc_width=128), 99, 3),
    (wl.vgg16_layers, dict(num_classes=50, widths=(64, 64, 128, 128, 128), fc_width=128), 32, 3),
    (wl.vgg16_layers, dict(num_classes=10, widths=(64, 64, 64, 64, 64), fc_width=64), 70, 1),   # odd frames: pooling drops a row and a column
])
def test_small_plain_chains_every_node(make, kw, hw, batch):
    """AlexNet- and VGG-shaped chains (11 x 11 / 4 input layer, 3 x 3 / 2 pooling on codes, 2 x 2 pooling fused into
    the convolution, fully connected layers as full-frame and 1 x 1 convolutions), reduced sizes, every node."""
    layers = make(image_hw=hw, **kw)
    params = wl.network_params(layers, seed=2)
    img = wl.image_batch(7, batch, hw)
    net = PackedNet(layers, params, batch)
    net.forward(torch.from_numpy(img).cuda())
    torch.cuda.synchronize()
    want = onet.run(layers, params, img)
    _check_all_nodes(layers, net, want, batch)
    for L in layers:                                    # the synthetic parameters keep every layer on all four codes
        if L.kind == "conv":
            hist = np.bincount(want[L.name].ravel(), minlength=4) / want[L.name].size
            assert hist.min() > 0.003, (L.name, hist)


@pytest.mark.parametrize("make,batch", [(wl.alexnet_layers, 8), (wl.vgg16_layers, 2)])
def test_plain_chains_full_size(make, batch):
    layers = make()
    params = wl.network_params(layers)
    img = wl.image_batch(2006, batch, 224)
    net = PackedNet(layers, params, batch)
    logits = net.forward(torch.from_numpy(img).cuda())
    torch.cuda.synchronize()
    want = onet.run(layers, params, img)
    _check_all_nodes(layers, net, want, batch)
    assert np.array_equal(logits.cpu().numpy(), want[layers[-1].name])


@pytest.mark.parametrize("make,kw,hw", [
    (wl.resnet18_layers, dict(num_classes=100, widths=(32, 64, 96, 128)), 64),
    (wl.vgg16_layers, dict(num_classes=10, widths=(64, 64, 64, 64, 64), fc_width=64), 38),
])
def test_small_networks_on_the_literal_kernel(make, kw, hw):
    """Every convolution and fully connected layer on the AND + popcount kernel (MFMA override 0): residual blocks,
    shortcut convolutions, fused 2 x 2 pooling, full-frame and 1 x 1 classifier layers; only the 8-bit input layer
    keeps its own kernel.  Same codes and logits as the oracle, node by node."""
    B.apnn_debug_force("MFMA", 0)
    layers = make(image_hw=hw, **kw)
    params = wl.network_params(layers, seed=4)
    img = wl.image_batch(9, 2, hw)
    net = PackedNet(layers, params, 2, fuse_tail=False)
    net.forward(torch.from_numpy(img).cuda())
    torch.cuda.synchronize()
    _check_all_nodes(layers, net, onet.run(layers, params, img), 2)
