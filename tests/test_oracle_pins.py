"""Pins for the fp64 CPU oracle: each check ties an oracle function to something other
than itself -- a closed form, an invariant, brute force written differently, or a
library routine used as a special case -- so that a dropped term, a wrong sign or
index, or a transposed operand fails at least one of them.

The paper prints no numeric example for any operator (Table 3 gives names, Table 4
shapes), hence no paper-value fixtures.
"""
import itertools

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import xenos_oracle as xo
from workloads import cnn_graphs as wg

RNG = np.random.default_rng(7)


def rnd(*shape):
    return RNG.standard_normal(shape)


# --------------------------------------------------------------------------- conv
@pytest.mark.parametrize("R", [1, 3, 5, 7])
def test_conv_centre_delta_is_identity(R):
    C = 3
    x = rnd(2, C, 9, 11)
    w = np.zeros((C, C, R, R))
    for c in range(C):
        w[c, c, R // 2, R // 2] = 1.0
    y = xo.conv2d(x, w, stride=1, pad=R // 2)
    assert np.array_equal(y, x)


def test_conv_offcentre_delta_shifts_with_zero_fill():
    x = rnd(1, 2, 6, 7)
    for (r, s) in itertools.product(range(3), range(3)):
        w = np.zeros((2, 2, 3, 3))
        w[0, 0, r, s] = w[1, 1, r, s] = 1.0
        y = xo.conv2d(x, w, pad=1)
        # y[oh, ow] = x[oh + r - 1, ow + s - 1], zero outside
        ref = np.zeros_like(x)
        for oh in range(6):
            for ow in range(7):
                ih, iw = oh + r - 1, ow + s - 1
                if 0 <= ih < 6 and 0 <= iw < 7:
                    ref[:, :, oh, ow] = x[:, :, ih, iw]
        assert np.array_equal(y, ref), (r, s)


def test_conv_delta_picks_channel_not_transposed():
    # w[k=1, c=0] = 1 only: output channel 1 must copy INPUT channel 0 (catches a K/C transposition)
    x = rnd(1, 2, 4, 4)
    w = np.zeros((2, 2, 1, 1))
    w[1, 0, 0, 0] = 1.0
    y = xo.conv2d(x, w)
    assert np.array_equal(y[0, 1], x[0, 0]) and not y[0, 0].any()


def test_conv_all_ones_counts_taps():
    C = 5
    x = np.ones((1, C, 6, 8))
    w = np.ones((2, C, 3, 3))
    y = xo.conv2d(x, w, pad=1)
    assert (y[:, :, 1:-1, 1:-1] == 9 * C).all()
    assert (y[:, :, 0, 1:-1] == 6 * C).all() and (y[:, :, 1:-1, -1] == 6 * C).all()
    assert y[0, 0, 0, 0] == 4 * C and y[0, 1, -1, -1] == 4 * C


def test_conv_bias_is_added_once_per_output():
    x = np.zeros((2, 3, 5, 5))
    w = rnd(4, 3, 3, 3)
    b = rnd(4)
    y = xo.conv2d(x, w, b, pad=1)
    assert np.array_equal(y, np.broadcast_to(b[None, :, None, None], y.shape))


def test_conv1x1_is_matrix_product():
    x = rnd(2, 6, 5, 4)
    w = rnd(7, 6, 1, 1)
    y = xo.conv2d(x, w)
    ref = np.einsum("kc,nchw->nkhw", w[:, :, 0, 0], x)
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-13)
    ref2 = (w[:, :, 0, 0] @ x.reshape(2, 6, 20)).reshape(2, 7, 5, 4)
    np.testing.assert_allclose(y, ref2, rtol=0, atol=1e-13)


def test_conv_linearity():
    x1, x2 = rnd(1, 3, 7, 7), rnd(1, 3, 7, 7)
    w1, w2 = rnd(4, 3, 3, 3), rnd(4, 3, 3, 3)
    a, b = 0.75, -2.5
    np.testing.assert_allclose(xo.conv2d(a * x1 + b * x2, w1, stride=2, pad=1),
                               a * xo.conv2d(x1, w1, stride=2, pad=1) + b * xo.conv2d(x2, w1, stride=2, pad=1),
                               atol=1e-12)
    np.testing.assert_allclose(xo.conv2d(x1, a * w1 + b * w2, pad=1),
                               a * xo.conv2d(x1, w1, pad=1) + b * xo.conv2d(x1, w2, pad=1), atol=1e-12)


@pytest.mark.parametrize("s", [2, 3])
def test_conv_stride_subsamples_stride1(s):
    x, w = rnd(1, 2, 11, 13), rnd(3, 2, 3, 3)
    y1 = xo.conv2d(x, w, stride=1, pad=1)
    ys = xo.conv2d(x, w, stride=s, pad=1)
    assert np.array_equal(ys, y1[:, :, ::s, ::s][:, :, :ys.shape[2], :ys.shape[3]])


def test_depthwise_is_independent_single_channel_convs():
    C = 5
    x, w = rnd(2, C, 8, 8), rnd(C, 1, 3, 3)
    y = xo.conv2d(x, w, stride=2, pad=1, groups=C)
    for c in range(C):
        yc = xo.conv2d(x[:, c:c + 1], w[c:c + 1], stride=2, pad=1)
        assert np.array_equal(y[:, c:c + 1], yc)


def test_grouped_conv_blocks():
    x, w = rnd(1, 6, 5, 5), rnd(4, 3, 3, 3)          # groups = 2: out 0-1 read in 0-2, out 2-3 read in 3-5
    y = xo.conv2d(x, w, pad=1, groups=2)
    assert np.array_equal(y[:, :2], xo.conv2d(x[:, :3], w[:2], pad=1))
    assert np.array_equal(y[:, 2:], xo.conv2d(x[:, 3:], w[2:], pad=1))


def _im2col_conv(x, w, stride, pad):
    """Second, independently written formulation: explicit patch matrix times weight matrix."""
    n, c, h, wd = x.shape
    k, _, r, s = w.shape
    xp = np.zeros((n, c, h + 2 * pad, wd + 2 * pad))
    xp[:, :, pad:pad + h, pad:pad + wd] = x
    oh, ow = (h + 2 * pad - r) // stride + 1, (wd + 2 * pad - s) // stride + 1
    cols = np.empty((n, oh * ow, c * r * s))
    for i in range(oh):
        for j in range(ow):
            cols[:, i * ow + j, :] = xp[:, :, i * stride:i * stride + r, j * stride:j * stride + s].reshape(n, -1)
    return (cols @ w.reshape(k, -1).T).transpose(0, 2, 1).reshape(n, k, oh, ow)


@pytest.mark.parametrize("R,stride,pad", [(r, s, p) for r in (1, 3, 7) for s in (1, 2) for p in (0, 1, 3)])
def test_conv_brute_force_and_library(R, stride, pad):
    if 7 + 2 * pad < R:
        pytest.skip("kernel larger than padded map")
    x, w, b = rnd(2, 4, 7, 7), rnd(3, 4, R, R), rnd(3)
    y = xo.conv2d(x, w, b, stride=stride, pad=pad)
    ref = _im2col_conv(x, w, stride, pad) + b[None, :, None, None]
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-12)
    lib = F.conv2d(torch.from_numpy(x), torch.from_numpy(w), torch.from_numpy(b), stride=stride, padding=pad)
    np.testing.assert_allclose(y, lib.numpy(), rtol=0, atol=1e-12)


def test_conv_nonsquare_map_library():
    x, w = rnd(1, 3, 9, 14), rnd(5, 3, 3, 3)
    y = xo.conv2d(x, w, stride=2, pad=1)
    lib = F.conv2d(torch.from_numpy(x), torch.from_numpy(w), stride=2, padding=1).numpy()
    np.testing.assert_allclose(y, lib, atol=1e-12)


# --------------------------------------------------------------------------- BN / bias / ReLU
def test_bn_identity_stats():
    x = rnd(2, 3, 4, 4)
    eps = 1e-5
    y = xo.bn(x, np.ones(3), np.zeros(3), np.zeros(3), np.full(3, 1 - eps), eps)
    np.testing.assert_allclose(y, x, rtol=4e-16, atol=0)


def test_bn_constant_closed_form():
    g, b, m, v = np.array([2.0, 0.5]), np.array([0.1, -0.3]), np.array([1.0, -1.0]), np.array([3.0, 0.25])
    x = np.stack([np.full((3, 3), 4.0), np.full((3, 3), -2.0)])[None]
    y = xo.bn(x, g, b, m, v, eps=0.0)
    assert np.allclose(y[0, 0], 2.0 * (4.0 - 1.0) / np.sqrt(3.0) + 0.1, rtol=1e-15)
    assert np.allclose(y[0, 1], 0.5 * (-2.0 + 1.0) / 0.5 - 0.3, rtol=1e-15)


def test_bn_library():
    x = rnd(2, 4, 5, 5)
    g, b, m, v = rnd(4), rnd(4), rnd(4), RNG.random(4) + 0.5
    y = xo.bn(x, g, b, m, v, 1e-5)
    lib = F.batch_norm(torch.from_numpy(x), torch.from_numpy(m), torch.from_numpy(v), torch.from_numpy(g),
                       torch.from_numpy(b), training=False, eps=1e-5).numpy()
    np.testing.assert_allclose(y, lib, atol=1e-13)


@pytest.mark.parametrize("bias_first", [True, False])
def test_bn_folding_identity_both_orders(bias_first):
    # the CBR group lists Conv, Bn, Bias, Relu (Section 4.3); either order of Bn and Bias must fold into
    # one per-channel scale and shift applied to the bias-free convolution
    x, w, b = rnd(1, 3, 6, 6), rnd(4, 3, 3, 3), rnd(4)
    g, be, m, v = RNG.random(4) + 0.5, rnd(4), rnd(4), RNG.random(4) + 0.5
    eps = 1e-5
    scale = g / np.sqrt(v + eps)
    if bias_first:
        y = xo.bn(xo.bias_add(xo.conv2d(x, w, pad=1), b), g, be, m, v, eps)
        shift = be + (b - m) * scale
    else:
        y = xo.bias_add(xo.bn(xo.conv2d(x, w, pad=1), g, be, m, v, eps), b)
        shift = be - m * scale + b
    folded = xo.conv2d(x, w * scale[:, None, None, None], pad=1) + shift[None, :, None, None]
    np.testing.assert_allclose(y, folded, atol=1e-13)


def test_relu_and_bias():
    x = np.array([-1.5, -0.0, 0.0, 2.0, -1e-300, 1e-300])
    assert np.array_equal(xo.relu(x), np.array([0.0, 0.0, 0.0, 2.0, 0.0, 1e-300]))
    t = rnd(2, 3, 2, 2)
    b = rnd(3)
    assert np.array_equal(xo.bias_add(t, b), t + b[None, :, None, None])


# --------------------------------------------------------------------------- pooling
def test_maxpool_relu_commute():
    x = rnd(2, 3, 9, 9)
    assert np.array_equal(xo.pool(xo.relu(x), 3, 2, 1), xo.relu(xo.pool(x, 3, 2, 1)))
    assert np.array_equal(xo.pool(xo.relu(x), 2, 2), xo.relu(xo.pool(x, 2, 2)))


def test_maxpool_ramp_takes_last_in_range_element():
    h = w = 7
    x = np.arange(h * w, dtype=np.float64).reshape(1, 1, h, w)
    for (k, s, p, ceil) in [(2, 2, 0, 0), (3, 2, 1, 0), (3, 2, 0, 1), (3, 1, 1, 0)]:
        y = xo.pool(x, k, s, p, ceil)
        for oh in range(y.shape[2]):
            for ow in range(y.shape[3]):
                ih, iw = min(oh * s - p + k - 1, h - 1), min(ow * s - p + k - 1, w - 1)
                assert y[0, 0, oh, ow] == x[0, 0, ih, iw]


def test_maxpool_padding_never_wins():
    x = -np.ones((1, 1, 4, 4)) * 5.0
    assert (xo.pool(x, 3, 2, 1) == -5.0).all()


def test_avgpool_constant_and_partition():
    x = np.full((1, 2, 6, 6), 3.25)
    assert (xo.pool(x, 3, 2, 1, avg=True) == 3.25).all()          # divisor = in-range count
    z = rnd(2, 3, 8, 6)
    y = xo.pool(z, 2, 2, avg=True)
    np.testing.assert_allclose(y.sum(axis=(2, 3)) * 4, z.sum(axis=(2, 3)), atol=1e-12)
    np.testing.assert_allclose(xo.gap(z)[:, :, 0, 0], z.sum(axis=(2, 3)) / 48, atol=1e-14)
    np.testing.assert_allclose(xo.gap(z[:, :, :6, :6]), xo.pool(z[:, :, :6, :6], 6, 6, avg=True), atol=1e-14)


@pytest.mark.parametrize("k,s,p,ceil", [(2, 2, 0, 0), (3, 2, 1, 0), (3, 2, 0, 1), (3, 1, 1, 0), (2, 2, 0, 1)])
@pytest.mark.parametrize("hw", [(7, 7), (8, 11), (13, 13)])
def test_pool_library(k, s, p, ceil, hw):
    x = rnd(2, 3, *hw)
    t = torch.from_numpy(x)
    y = xo.pool(x, k, s, p, ceil)
    np.testing.assert_array_equal(y, F.max_pool2d(t, k, s, p, ceil_mode=bool(ceil)).numpy())
    for cip in (0, 1):
        ya = xo.pool(x, k, s, p, ceil, avg=True, count_include_pad=cip)
        lib = F.avg_pool2d(t, k, s, p, ceil_mode=bool(ceil), count_include_pad=bool(cip)).numpy()
        np.testing.assert_allclose(ya, lib, atol=1e-13)


def test_pool_out_sizes_of_the_workloads():
    assert xo.pool_out(112, 3, 2, 1, 0) == 56                 # ResNet stem
    assert [xo.pool_out(n, 3, 2, 0, 1) for n in (111, 55, 27)] == [55, 27, 13]   # SqueezeNet ceil mode
    assert xo.pool_out(224, 2, 2, 0, 0) == 112


# --------------------------------------------------------------------------- FC / flatten / add / concat
def test_fc_is_1x1_conv_on_1x1_map():
    # Table 4 writes FullyConnected as a 1x1xI map with a 1x1xIxO kernel
    x, w, b = rnd(3, 10, 1, 1), rnd(6, 10), rnd(6)
    np.testing.assert_allclose(xo.fc(x, w, b), xo.conv2d(x, w[:, :, None, None], b), atol=1e-13)
    np.testing.assert_allclose(xo.fc(x, w, b)[:, :, 0, 0], x[:, :, 0, 0] @ w.T + b, atol=1e-13)


def test_fc_flatten_order_one_hot():
    C, H, W = 3, 2, 4
    w = rnd(5, C * H * W)
    for (c, h, wd) in itertools.product(range(C), range(H), range(W)):
        x = np.zeros((1, C, H, W))
        x[0, c, h, wd] = 1.0
        y = xo.fc(x, w)
        assert np.array_equal(y[0, :, 0, 0], w[:, c * H * W + h * W + wd])


def test_fc_equals_full_map_conv():
    x, w = rnd(2, 3, 4, 4), rnd(5, 48)
    np.testing.assert_allclose(xo.fc(x, w), xo.conv2d(x, w.reshape(5, 3, 4, 4)), atol=1e-13)


def test_k_split_identity_eq1():
    # Eq. 1: y = Wx + B splits over output channels into y1 = W1 x + B1, y2 = W2 x + B2,
    # which join without any layout transformation: exact equality in the oracle
    x, w, b = rnd(2, 4, 6, 6), rnd(7, 4, 3, 3), rnd(7)
    y = xo.conv2d(x, w, b, pad=1)
    y1, y2 = xo.conv2d(x, w[:3], b[:3], pad=1), xo.conv2d(x, w[3:], b[3:], pad=1)
    assert np.array_equal(y, xo.concat([y1, y2]))
    assert np.array_equal(xo.concat([y1, y2]), np.concatenate([y1, y2], axis=1))
    assert np.array_equal(xo.add(y1, y1), 2 * y1)


def test_channel_slice_is_the_inverse_of_concat():
    x = rnd(2, 7, 3, 4)
    a, b, c = xo.channel_slice(x, 0, 2), xo.channel_slice(x, 2, 4), xo.channel_slice(x, 6, 1)
    assert np.array_equal(xo.concat([a, b, c]), x)
    assert np.array_equal(b, x[:, 2:6])
    with pytest.raises(AssertionError):
        xo.channel_slice(x, 5, 3)


@pytest.mark.parametrize("c,g", [(6, 2), (6, 3), (12, 4), (8, 1), (8, 8), (10, 5)])
def test_channel_shuffle_closed_forms(c, g):
    # every channel holds its own index: the shuffled tensor lists, group-interleaved, 0, m, 2m, ..., 1, m+1, ...
    m = c // g
    x = np.broadcast_to(np.arange(c, dtype=np.float64)[None, :, None, None], (2, c, 3, 2)).copy()
    y = xo.channel_shuffle(x, g)
    want = [j * m + i for i in range(m) for j in range(g)]
    assert np.array_equal(y[1, :, 2, 1], np.array(want, np.float64))
    assert sorted(y[0, :, 0, 0].tolist()) == list(range(c))            # a permutation of the channels
    # shuffling with g groups and then with C / g groups is the identity (the two transposes cancel)
    z = rnd(2, c, 3, 2)
    assert np.array_equal(xo.channel_shuffle(xo.channel_shuffle(z, g), m), z)
    # one group, or one channel per group, moves nothing
    if g == 1 or g == c:
        assert np.array_equal(xo.channel_shuffle(z, g), z)
    # the reshape / transpose form of the same definition, and the library routine
    assert np.array_equal(xo.channel_shuffle(z, g), z.reshape(2, g, m, 3, 2).transpose(0, 2, 1, 3, 4).reshape(2, c, 3, 2))
    assert np.array_equal(xo.channel_shuffle(z, g), F.channel_shuffle(torch.from_numpy(z), g).numpy())
    # with two groups the shuffle of concat(a, b) interleaves a and b
    if g == 2:
        a, b = z[:, :m], z[:, m:]
        assert np.array_equal(y := xo.channel_shuffle(xo.concat([a, b]), 2), y) and np.array_equal(y[:, 0::2], a) and np.array_equal(y[:, 1::2], b)


def test_spatial_split_identity():
    # inH split needs boundary rows (Section 4.2.1): rows 0-3 of the output depend on input rows 0-4 only
    x, w = rnd(1, 2, 8, 8), rnd(3, 2, 3, 3)
    y = xo.conv2d(x, w, pad=1)
    top = xo.conv2d(x[:, :, :5], w, pad=1)[:, :, :4]
    assert np.array_equal(y[:, :, :4], top)


# --------------------------------------------------------------------------- whole graphs
def _cfg0_pure_python(g):
    """Config 0 by brute force in pure Python floats, written against the definitions only."""
    conv, bnop = g.ops[0], g.ops[1]
    x = g.x.astype(np.float64)
    w = conv.params["weight"].astype(np.float64)
    _, C, H, W = x.shape
    K = w.shape[0]
    gm, bt, mu, var = (bnop.params[k].astype(np.float64) for k in ("gamma", "beta", "mean", "var"))
    act = np.empty((K, H, W))
    for k in range(K):
        for oh in range(H):
            for ow in range(W):
                acc = 0.0
                for c in range(C):
                    for r in range(3):
                        for s in range(3):
                            ih, iw = oh + r - 1, ow + s - 1
                            if 0 <= ih < H and 0 <= iw < W:
                                acc += x[0, c, ih, iw] * w[k, c, r, s]
                v = gm[k] * (acc - mu[k]) / np.sqrt(var[k] + 1e-5) + bt[k]
                act[k, oh, ow] = max(v, 0.0)
    out = np.empty((1, K, H // 2, W // 2))
    for k in range(K):
        for ph in range(H // 2):
            for pw in range(W // 2):
                out[0, k, ph, pw] = max(act[k, 2 * ph, 2 * pw], act[k, 2 * ph, 2 * pw + 1],
                                        act[k, 2 * ph + 1, 2 * pw], act[k, 2 * ph + 1, 2 * pw + 1])
    return out


def test_cfg0_graph_brute_force():
    g = wg.single_chain(batch=1, hw=16)
    y = xo.forward(g)
    assert y.shape == (1, 16, 8, 8)
    np.testing.assert_allclose(y, _cfg0_pure_python(g), atol=1e-13)


def _torch_forward(g):
    """Library cross-check of the graph runner: the same graph through torch float64 CPU ops."""
    t = {0: torch.from_numpy(g.x.astype(np.float64))}
    for i, op in enumerate(g.ops):
        a, p = op.attrs, {k: torch.from_numpy(v.astype(np.float64)) for k, v in op.params.items()}
        ins = [t[j] for j in op.inputs]
        if op.kind == "conv":
            y = F.conv2d(ins[0], p["weight"], p.get("bias"), a["stride"], a["pad"], 1, a["groups"])
        elif op.kind == "bn":
            y = F.batch_norm(ins[0], p["mean"], p["var"], p["gamma"], p["beta"], False, 0.0, a["eps"])
        elif op.kind == "bias":
            y = ins[0] + p["bias"][None, :, None, None]
        elif op.kind == "relu":
            y = F.relu(ins[0])
        elif op.kind == "maxpool":
            y = F.max_pool2d(ins[0], a["k"], a["stride"], a["pad"], ceil_mode=bool(a.get("ceil", 0)))
        elif op.kind == "gap":
            y = ins[0].mean(dim=(2, 3), keepdim=True)
        elif op.kind == "add":
            y = ins[0] + ins[1]
        elif op.kind == "concat":
            y = torch.cat(ins, 1)
        elif op.kind == "fc":
            y = F.linear(ins[0].flatten(1), p["weight"], p.get("bias"))[:, :, None, None]
        elif op.kind == "slice":
            y = torch.narrow(ins[0], 1, a["c_begin"], a["out_c"])
        elif op.kind == "shuffle":
            y = F.channel_shuffle(ins[0], a["groups"])
        else:
            raise ValueError(op.kind)
        t[i + 1] = y
    return t[g.output].numpy()


@pytest.mark.parametrize("builder,kw", [
    (wg.mobilenet_v1, dict(hw=32, width=0.25, classes=10)),
    (wg.resnet18, dict(hw=32, width=0.125, classes=10)),
    (wg.vgg16, dict(hw=32, width=0.125, fc_dim=32, classes=10)),
    (wg.squeezenet11, dict(hw=63, classes=10)),
    (wg.shufflenet_v2, dict(hw=64, channels=(16, 24, 48), repeats=(2, 3, 2), stem=8, last=64, classes=10)),
])
def test_graph_runner_against_library_and_batch_independence(builder, kw):
    g = builder(batch=2, seed=11, nonzero_bias=True, **kw)
    y = xo.forward(g)
    ref = _torch_forward(g)
    scale = np.abs(ref).max()
    assert np.abs(y - ref).max() <= 1e-12 * scale
    # images in a batch are independent
    y0 = xo.forward(g, g.x[1:2])
    np.testing.assert_array_equal(y0[0], y[1])


def test_oracle_is_deterministic():
    g = wg.single_chain(batch=2)
    assert np.array_equal(xo.forward(g), xo.forward(g))


# ------------------------------------------------------------------------------------------ x.matmul (Table 3; Table 1 MatmulX -> MatmulY)
def test_matmul_against_numpy_and_row_structure():
    r = np.random.default_rng(77)
    m, k, n = 9, 13, 7
    x, w, b = r.standard_normal((m, k, 1, 1)), r.standard_normal((n, k)), r.standard_normal(n)
    y = xo.matmul(x, w, b)
    assert y.shape == (m, n, 1, 1)
    want = np.matmul(x.reshape(m, k), w.T) + b                         # library routine, float64
    np.testing.assert_allclose(y.reshape(m, n), want, rtol=0, atol=1e-12)
    # a transposed operand fails this: W is [out][in], rows of X are independent
    np.testing.assert_allclose(xo.matmul(x[3:4], w, b), y[3:4], rtol=0, atol=0)
    eye = np.eye(k)
    np.testing.assert_array_equal(xo.matmul(x, eye), x)                # identity weights
    onehot = np.zeros((k, k, 1, 1)); onehot[np.arange(k), np.arange(k)] = 1.0
    np.testing.assert_array_equal(xo.matmul(onehot, w).reshape(k, n), w.T)   # one-hot row i selects column i of W^T = W[:, i]
    # the same operator as a fully connected layer on a 1x1 map and as a 1x1 convolution
    np.testing.assert_allclose(y, xo.fc(x, w, b), rtol=0, atol=0)
    np.testing.assert_allclose(y, xo.conv2d(x, w.reshape(n, k, 1, 1), b), rtol=0, atol=1e-12)


def test_matmul_chain_graph_against_library():
    # MatmulX -> MatmulY with ReLU between and a shortcut around (the feed-forward block of a small transformer)
    g = wg.matmul_chain(rows=11, widths=(24, 40, 24), seed=5)
    y = xo.forward(g)
    t = torch.from_numpy(g.x.astype(np.float64)).reshape(11, 24)
    p = g.ops[0].params
    x0 = torch.relu((t - torch.from_numpy(p["mean"].astype(np.float64))) / torch.sqrt(torch.from_numpy(p["var"].astype(np.float64)) + float(np.float32(1e-5)))
                    * torch.from_numpy(p["gamma"].astype(np.float64)) + torch.from_numpy(p["beta"].astype(np.float64)))
    mm = [op for op in g.ops if op.kind == "matmul"]
    h = torch.relu(x0 @ torch.from_numpy(mm[0].params["weight"].astype(np.float64)).T + torch.from_numpy(mm[0].params["bias"].astype(np.float64)))
    out = h @ torch.from_numpy(mm[1].params["weight"].astype(np.float64)).T + torch.from_numpy(mm[1].params["bias"].astype(np.float64)) + x0
    np.testing.assert_allclose(y.reshape(11, 24), out.numpy(), rtol=0, atol=1e-12)
    # without the shortcut: widths that differ, three matmuls
    g3 = wg.matmul_chain(rows=5, widths=(16, 8, 32, 12), seed=6, residual=False)
    assert [op.kind for op in g3.ops] == ["matmul", "relu", "matmul", "relu", "matmul"] and xo.forward(g3).shape == (5, 12, 1, 1)
