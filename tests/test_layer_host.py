"""Host-side behaviour of the drop-in layer: construction, argument checks, conversion of a network,
and a loud refusal to estimate without a GPU (there is no CPU fallback)."""
import pytest
import torch

from paper_2106_06998_amd.layer import SignReLU, XConv2d, XConv3d, convert_net


def test_layer_is_a_conv2d_with_the_probing_arguments():
    layer = XConv2d(8, 4, 3, r=4, stride=2, padding=1, probe="gaussian", mode="multi")
    assert isinstance(layer, torch.nn.Conv2d) and layer.weight.shape == (4, 8, 3, 3)
    assert "r=4" in repr(layer) and "mode=multi" in repr(layer)
    for bad in (dict(mode="other"), dict(probe="uniform"), dict(dilation=2), dict(groups=2), dict(padding="same"),
                dict(padding_mode="reflect")):
        with pytest.raises(ValueError):
            XConv2d(8, 4, 3, r=4, **bad)


def test_layer_is_a_plain_convolution_when_no_weight_gradient_is_needed():
    layer = XConv2d(8, 4, 3, r=4, padding=1)
    x = torch.randn(2, 8, 6, 6)
    want = torch.nn.functional.conv2d(x, layer.weight, layer.bias, 1, 1)
    layer.eval()
    assert torch.equal(layer(x), want)
    layer.train()
    with torch.no_grad():
        assert torch.equal(layer(x), want)
    layer.weight.requires_grad_(False)
    assert torch.equal(layer(x), want)
    assert layer.last_seed is None


def test_layer_refuses_to_estimate_on_the_cpu():
    layer = XConv2d(8, 4, 3, r=4, padding=1)
    with pytest.raises(RuntimeError, match="GPU only"):
        layer(torch.randn(2, 8, 6, 6))


def test_convert_net_replaces_only_what_the_layer_supports():
    net = torch.nn.Sequential(
        torch.nn.Conv2d(3, 32, 3, padding=1),                 # fewer input channels than probing vectors
        torch.nn.Sequential(torch.nn.Conv2d(32, 16, 3, padding=1, bias=False), torch.nn.ReLU()),
        torch.nn.Conv2d(16, 16, 3, padding=2, dilation=2),
        torch.nn.Conv2d(16, 16, 1, groups=4),
        torch.nn.Conv2d(16, 8, 3, stride=2, padding=1))
    params = list(net.parameters())
    net, n = convert_net(net, r=8, probe="gaussian")
    assert n == 2
    assert isinstance(net[1][0], XConv2d) and net[1][0].bias is None and net[1][0].probe == "gaussian" and net[1][0].r == 8
    assert isinstance(net[4], XConv2d) and net[4].stride == (2, 2)
    assert [type(net[i]) for i in (0, 2, 3)] == [torch.nn.Conv2d] * 3
    assert all(a is b for a, b in zip(params, net.parameters()))
    assert net[1][0].base_seed != net[4].base_seed             # layers draw different probes in the same iteration
    _, again = convert_net(net, r=8)
    assert again == 0                                           # already converted layers are left alone
    net2, n2 = convert_net(torch.nn.Sequential(torch.nn.Conv2d(3, 8, 3)), r=8, mode="multi")
    assert n2 == 1                                              # probes over pixels and channels pay off for any channel count


def test_volumetric_layer_and_its_conversion():
    layer = XConv3d(32, 8, 3, r=8, padding=1)
    assert isinstance(layer, torch.nn.Conv3d) and "r=8" in repr(layer)
    with pytest.raises(ValueError):
        XConv3d(32, 8, 3, r=8, dilation=2)
    with pytest.raises(RuntimeError, match="GPU only"):
        layer(torch.randn(1, 32, 4, 4, 4))
    layer.eval()
    x = torch.randn(1, 32, 4, 4, 4)
    assert torch.equal(layer(x), torch.nn.functional.conv3d(x, layer.weight, layer.bias, 1, 1))
    net = torch.nn.Sequential(torch.nn.Conv3d(32, 8, 3, padding=1),
                              torch.nn.Conv3d(32, 8, 3, padding=3),     # depth padding beyond the kernel depth: kept
                              torch.nn.Conv3d(4, 8, 3, padding=1))      # fewer channels than probing vectors: kept
    net, n = convert_net(net, r=8)
    assert n == 1 and isinstance(net[0], XConv3d) and type(net[1]) is torch.nn.Conv3d and type(net[2]) is torch.nn.Conv3d
    _, m = convert_net(torch.nn.Sequential(torch.nn.Conv3d(32, 8, 3, padding=1)), r=8, mode="multi")
    assert m == 0                                                       # volumetric layers take channel probes only


def test_sign_relu_module_on_the_host():
    m = SignReLU()
    x = torch.tensor([-1.0, 0.0, 2.0])
    assert torch.equal(m(x), torch.tensor([0.0, 0.0, 2.0]))                # no gradient needed: a plain ReLU
    with pytest.raises(RuntimeError, match="GPU only"):
        m(x.clone().requires_grad_(True))
    net = torch.nn.Sequential(torch.nn.Conv2d(32, 8, 3), torch.nn.ReLU(), torch.nn.Sequential(torch.nn.ReLU(inplace=True)))
    net, n = convert_net(net, r=8, relu=True)
    assert n == 1 and isinstance(net[1], SignReLU) and isinstance(net[2][0], SignReLU)
    net, n = convert_net(torch.nn.Sequential(torch.nn.Conv2d(32, 8, 3), torch.nn.ReLU()), r=8)
    assert type(net[1]) is torch.nn.ReLU                                    # only on request

