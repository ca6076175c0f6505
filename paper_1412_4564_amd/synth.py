"""Seeded synthetic inputs shaped like the workloads of the MatConvNet manual.

This module holds NO arithmetic of the method: it only names layer shapes and
draws Gaussian tensors.  Both the GPU tests/benchmark and the CPU oracle's
tests take their inputs from here; output shapes are passed in by the caller
(each side computes them with its own code).

Memory convention: the manual's H x W x D x N arrays are first-index-fastest
(Sec. 2.3.1, vec() order).  A C-contiguous array of shape (N, D, W, H) has that
memory order, and that is what is returned.

Shapes: the layers are those of the networks the manual trains and times
(Sec. 1.2-1.4: a CIFAR-sized LeNet-style stack, the first two layers of the
Krizhevsky-style network including its two-group layer, three depths of the
VGG-VD 3x3 stack, a first fully-connected layer run as a 6x6 convolution, a
1x1 layer, and one deliberately irregular layer).  The datasets and trained
weights themselves are not used: x ~ N(0,1), dzdy ~ N(0,1),
w ~ N(0, 2/(H'W'D')) (second argument is the variance), b ~ N(0, 0.01).
"""
from __future__ import annotations

from collections import OrderedDict

import torch

BASE_SEED = 14124564


def _layer(x, w, stride=(1, 1), pad=(0, 0, 0, 0), group=0, index=0):
    H, W, D, N = x
    Hf, Wf, Df, K = w
    return dict(H=H, W=W, D=D, N=N, Hf=Hf, Wf=Wf, Df=Df, K=K,
                stride=tuple(stride), pad=tuple(pad), config=group, index=index)


# name -> layer.  'config' is the 1-based index of the workload group, 'index'
# the layer within it; both only feed the seed.
LAYERS = OrderedDict([
    ("1",  _layer((32, 32, 3, 8),      (5, 5, 3, 32),      (1, 1), (2, 2, 2, 2), 1, 0)),
    ("2a", _layer((32, 32, 3, 100),    (5, 5, 3, 32),      (1, 1), (2, 2, 2, 2), 2, 0)),
    ("2b", _layer((16, 16, 32, 100),   (5, 5, 32, 32),     (1, 1), (2, 2, 2, 2), 2, 1)),
    ("2c", _layer((8, 8, 32, 100),     (5, 5, 32, 64),     (1, 1), (2, 2, 2, 2), 2, 2)),
    ("3a", _layer((227, 227, 3, 128),  (11, 11, 3, 96),    (4, 4), (0, 0, 0, 0), 3, 0)),
    ("3b", _layer((27, 27, 96, 128),   (5, 5, 48, 256),    (1, 1), (2, 2, 2, 2), 3, 1)),
    ("4a", _layer((224, 224, 64, 32),  (3, 3, 64, 64),     (1, 1), (1, 1, 1, 1), 4, 0)),
    ("4b", _layer((56, 56, 256, 32),   (3, 3, 256, 256),   (1, 1), (1, 1, 1, 1), 4, 1)),
    ("4c", _layer((14, 14, 512, 32),   (3, 3, 512, 512),   (1, 1), (1, 1, 1, 1), 4, 2)),
    ("5a", _layer((6, 6, 256, 256),    (6, 6, 256, 4096),  (1, 1), (0, 0, 0, 0), 5, 0)),
    ("5b", _layer((28, 28, 512, 64),   (1, 1, 512, 128),   (1, 1), (0, 0, 0, 0), 5, 1)),
    ("5c", _layer((37, 53, 16, 4),     (3, 5, 16, 24),     (2, 3), (1, 0, 2, 1), 5, 2)),
])


def with_batch(layer, n):
    """The same layer at another batch size (for bounded CPU timing and quick tests)."""
    out = dict(layer)
    out["N"] = int(n)
    return out


def _gen(layer, tensor_index, extra=0):
    g = torch.Generator(device="cpu")
    g.manual_seed(BASE_SEED + 1000 * int(extra) + 100 * layer["config"] + 10 * layer["index"] + tensor_index)
    return g


def x_shape(layer):
    return (layer["N"], layer["D"], layer["W"], layer["H"])


def w_shape(layer):
    return (layer["K"], layer["Df"], layer["Wf"], layer["Hf"])


def make_x(layer, seed=0):
    return torch.randn(x_shape(layer), generator=_gen(layer, 0, seed), dtype=torch.float32)


def make_w(layer, seed=0):
    fan = layer["Hf"] * layer["Wf"] * layer["Df"]
    w = torch.randn(w_shape(layer), generator=_gen(layer, 1, seed), dtype=torch.float32)
    return w * float((2.0 / fan) ** 0.5)


def make_b(layer, seed=0):
    return torch.randn((layer["K"],), generator=_gen(layer, 2, seed), dtype=torch.float32) * 0.1


def make_dzdy(layer, Ho, Wo, seed=0):
    """dzdy ~ N(0,1) of shape (N, K, Wo, Ho); Ho, Wo come from the caller."""
    return torch.randn((layer["N"], layer["K"], int(Wo), int(Ho)), generator=_gen(layer, 3, seed),
                       dtype=torch.float32)


# ---- convolution transpose (Sec. 4.2) ------------------------------------------------------
# The manual names two uses of the block: decoders / deconvolutional networks that run a
# convolution backwards, and learnable interpolation.  The shapes below are of those two kinds
# (a stride-1 "deconvnet" mirror of a VGG 3x3 layer, a 2x upsampling decoder layer, 2x and 32x
# per-class interpolation of score maps with one group per class, and one irregular layer).
# Layer fields: x is H x W x D x N, f is H' x W' x K' x D, `groups` groups, y has groups*K'
# channels.  Same distributions as above; f ~ N(0, 2/(H'W'D/groups)).
def _tlayer(x, f, groups=1, up=(1, 1), crop=(0, 0, 0, 0), index=0):
    H, W, D, N = x
    Hf, Wf, Kf, Df = f
    assert Df == D
    return dict(H=H, W=W, D=D, N=N, Hf=Hf, Wf=Wf, Kf=Kf, groups=groups,
                up=tuple(up), crop=tuple(crop), config=6, index=index)


CONVT_LAYERS = OrderedDict([
    ("t1", _tlayer((56, 56, 256, 32),  (3, 3, 256, 256),   1,  (1, 1),   (1, 1, 1, 1),     0)),
    ("t2", _tlayer((28, 28, 256, 32),  (4, 4, 128, 256),   1,  (2, 2),   (1, 1, 1, 1),     1)),
    ("t3", _tlayer((34, 34, 21, 8),    (4, 4, 21, 21),     1,  (2, 2),   (0, 0, 0, 0),     2)),
    ("t4", _tlayer((16, 16, 21, 4),    (64, 64, 1, 21),    21, (32, 32), (16, 16, 16, 16), 3)),
    ("t5", _tlayer((7, 5, 6, 3),       (5, 3, 4, 6),       2,  (3, 2),   (2, 0, 1, 3),     4)),
])


def tx_shape(layer):
    return (layer["N"], layer["D"], layer["W"], layer["H"])


def tf_shape(layer):
    return (layer["D"], layer["Kf"], layer["Wf"], layer["Hf"])


def make_tx(layer, seed=0):
    return torch.randn(tx_shape(layer), generator=_gen(layer, 0, seed), dtype=torch.float32)


def make_tf(layer, seed=0):
    fan = layer["Hf"] * layer["Wf"] * (layer["D"] // layer["groups"])
    f = torch.randn(tf_shape(layer), generator=_gen(layer, 1, seed), dtype=torch.float32)
    return f * float((2.0 / fan) ** 0.5)


def make_tb(layer, seed=0):
    return torch.randn((layer["groups"] * layer["Kf"],), generator=_gen(layer, 2, seed), dtype=torch.float32) * 0.1


def make_tdzdy(layer, Ho, Wo, seed=0):
    """dzdy ~ N(0,1) of shape (N, groups*K', Wo, Ho); Ho, Wo come from the caller."""
    return torch.randn((layer["N"], layer["groups"] * layer["Kf"], int(Wo), int(Ho)),
                       generator=_gen(layer, 3, seed), dtype=torch.float32)


# ---- spatial pooling (Sec. 4.3) --------------------------------------------------------------
# Pooling layers of the same networks: the 3x3/stride-2 pools of the CIFAR-sized stack (32 -> 16 -> 8,
# bottom/right pad 1, the second one an average), the 3x3/stride-2 pools of the Krizhevsky-style network
# (55 -> 27, 13 -> 6), the 2x2/stride-2 pool after the first VGG block, and one irregular layer.
def _player(x, window, stride, pad, method, index):
    H, W, D, N = x
    return dict(H=H, W=W, D=D, N=N, window=tuple(window), stride=tuple(stride), pad=tuple(pad), method=method,
                config=11, index=index)


POOL_LAYERS = OrderedDict([
    ("p1", _player((32, 32, 32, 100),   (3, 3), (2, 2), (0, 1, 0, 1), "max", 0)),
    ("p2", _player((16, 16, 32, 100),   (3, 3), (2, 2), (0, 1, 0, 1), "avg", 1)),
    ("p3", _player((55, 55, 96, 128),   (3, 3), (2, 2), (0, 0, 0, 0), "max", 2)),
    ("p4", _player((224, 224, 64, 32),  (2, 2), (2, 2), (0, 0, 0, 0), "max", 3)),
    ("p5", _player((13, 13, 256, 128),  (3, 3), (2, 2), (0, 0, 0, 0), "max", 4)),
    ("p6", _player((37, 53, 16, 4),     (3, 5), (2, 3), (1, 0, 2, 1), "avg", 5)),
])


def make_px(layer, seed=0):
    return torch.randn((layer["N"], layer["D"], layer["W"], layer["H"]), generator=_gen(layer, 0, seed),
                       dtype=torch.float32)


def make_pdzdy(layer, Ho, Wo, seed=0):
    return torch.randn((layer["N"], layer["D"], int(Wo), int(Ho)), generator=_gen(layer, 3, seed), dtype=torch.float32)
