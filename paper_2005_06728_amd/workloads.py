"""Seeded synthetic workloads for the OD-SGD update path.

This module holds *only* input generation: parameter-set shapes, hyper-parameter
values and the random recipes for weights and gradients.  It contains none of
the method's arithmetic and is the one module that both the GPU tests and the
CPU oracle tests draw inputs from.

The five parameter sets stand in for the networks the method is trained on
(Section 4.1 trains MobileNet, ResNet-18/20 and ResNet-50 on MNIST, CIFAR-10 and
ImageNet); no dataset is used -- gradients are random tensors with a stated
distribution.  "N(0, x)" means standard deviation x.
"""
import math
from collections import namedtuple

import torch

BASE_SEED = 200506728

Tensor = namedtuple("Tensor", "name shape kind")  # kind: conv | fc | bn_scale | bias
Hyper = namedtuple("Hyper", "lr local_lr momentum weight_decay grad_scale")
Workload = namedtuple(
    "Workload",
    "name index tensors num_workers hyper iterations weight_init weight_std "
    "grad_std grad_tail_prob grad_tail_scale grad_zero_prob")


def _conv(name, cout, cin, k):
    return Tensor(name + ".weight", (cout, cin, k, k), "conv")


def _bn(name, c):
    return [Tensor(name + ".scale", (c,), "bn_scale"), Tensor(name + ".bias", (c,), "bias")]


def _fc(name, cout, cin):
    return [Tensor(name + ".weight", (cout, cin), "fc"), Tensor(name + ".bias", (cout,), "bias")]


def _conv_b(name, cout, cin, k):
    return [_conv(name, cout, cin, k), Tensor(name + ".bias", (cout,), "bias")]


def _lenet5():
    t = []
    t += _conv_b("conv1", 6, 1, 5)
    t += _conv_b("conv2", 16, 6, 5)
    t += _fc("fc1", 120, 400)
    t += _fc("fc2", 84, 120)
    t += _fc("fc3", 10, 84)
    return t


def _resnet20():
    """CIFAR ResNet-20 with projection (1x1 conv) shortcuts where the width changes."""
    t = [_conv("stem", 16, 3, 3)] + _bn("stem.bn", 16)
    cin = 16
    for stage, c in enumerate((16, 32, 64)):
        for block in range(3):
            p = "s%d.b%d" % (stage, block)
            t += [_conv(p + ".conv1", c, cin, 3)] + _bn(p + ".bn1", c)
            t += [_conv(p + ".conv2", c, c, 3)] + _bn(p + ".bn2", c)
            if cin != c:
                t += [_conv(p + ".proj", c, cin, 1)] + _bn(p + ".proj.bn", c)
            cin = c
    t += _fc("fc", 10, 64)
    return t


def _resnet50():
    t = [_conv("stem", 64, 3, 7)] + _bn("stem.bn", 64)
    cin = 64
    for stage, (mid, blocks) in enumerate(((64, 3), (128, 4), (256, 6), (512, 3))):
        cout = 4 * mid
        for block in range(blocks):
            p = "s%d.b%d" % (stage, block)
            t += [_conv(p + ".conv1", mid, cin, 1)] + _bn(p + ".bn1", mid)
            t += [_conv(p + ".conv2", mid, mid, 3)] + _bn(p + ".bn2", mid)
            t += [_conv(p + ".conv3", cout, mid, 1)] + _bn(p + ".bn3", cout)
            if block == 0:
                t += [_conv(p + ".proj", cout, cin, 1)] + _bn(p + ".proj.bn", cout)
            cin = cout
    t += _fc("fc", 1000, 2048)
    return t


def _alexnet():
    t = []
    t += _conv_b("conv1", 64, 3, 11)
    t += _conv_b("conv2", 192, 64, 5)
    t += _conv_b("conv3", 384, 192, 3)
    t += _conv_b("conv4", 256, 384, 3)
    t += _conv_b("conv5", 256, 256, 3)
    t += _fc("fc6", 4096, 9216)
    t += _fc("fc7", 4096, 4096)
    t += _fc("fc8", 1000, 4096)
    return t


def _vgg16():
    t = []
    cin = 3
    for i, c in enumerate((64, 64, 128, 128, 256, 256, 256, 512, 512, 512, 512, 512, 512)):
        t += _conv_b("conv%d" % (i + 1), c, cin, 3)
        cin = c
    t += _fc("fc14", 4096, 25088)
    t += _fc("fc15", 4096, 4096)
    t += _fc("fc16", 1000, 4096)
    return t


# hyper-parameter values: ones the paper runs with where it names them
#   lenet5   : local SGD with the global updater's lr (Section 4.2); wd as listed for this set
#   resnet20 : global 0.4 + local 0.5 (Section 4.6, warm-up study)
#   resnet50 : global 1.6 + local 0.2, momentum 0.9, wd 1e-4 (Section 4.4, lr grid)
WORKLOADS = {}
for _i, _w in enumerate([
    Workload("lenet5", 0, _lenet5(), 4, Hyper(0.01, 0.01, 0.9, 5e-4, 0.0), 10,
             "normal", 0.05, 1e-3, 0.0, 1.0, 0.0),
    Workload("resnet20", 1, _resnet20(), 8, Hyper(0.4, 0.5, 0.9, 1e-4, 0.0), 100,
             "he", None, 1e-3, 0.01, 100.0, 0.0),
    Workload("resnet50", 2, _resnet50(), 8, Hyper(1.6, 0.2, 0.9, 1e-4, 0.0), 50,
             "he", None, 1e-4, 0.0, 1.0, 0.0),
    Workload("alexnet", 3, _alexnet(), 16, Hyper(0.01, 0.01, 0.9, 5e-4, 0.0), 20,
             "normal", 0.01, 1e-4, 0.0, 1.0, 0.0),
    Workload("vgg16", 4, _vgg16(), 16, Hyper(0.01, 0.01, 0.9, 5e-4, 0.0), 10,
             "normal", 0.01, 1e-4, 0.0, 1.0, 1e-3),
]):
    WORKLOADS[_w.name] = _w


def numels(wl):
    return [math.prod(t.shape) for t in wl.tensors]


def total_params(wl):
    return sum(numels(wl))


def _seed(wl, role, iteration=0, worker=0):
    """Independent sub-stream per (workload, role, iteration, worker)."""
    x = BASE_SEED
    for part in (wl.index, role, iteration, worker):
        x = (x * 1000003 + part + 1) % (2 ** 63 - 1)
    return x


def _generator(device, seed):
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    return gen


def fill_weights_(bufs, wl, device=None):
    """Fill the K weight buffers (flat fp32 tensors) in place."""
    device = bufs[0].device if device is None else device
    gen = _generator(device, _seed(wl, 1))
    for buf, t in zip(bufs, wl.tensors):
        if wl.weight_init == "normal":
            buf.normal_(0.0, wl.weight_std, generator=gen)
        elif t.kind in ("conv", "fc"):
            fan_in = math.prod(t.shape[1:])
            buf.normal_(0.0, math.sqrt(2.0 / fan_in), generator=gen)
        elif t.kind == "bn_scale":
            buf.fill_(1.0)
        else:
            buf.zero_()


def fill_grads_(bufs, wl, iteration, worker):
    """Fill worker `worker`'s K gradient buffers in place for one iteration."""
    device = bufs[0].device
    gen = _generator(device, _seed(wl, 2, iteration, worker))
    for buf in bufs:
        buf.normal_(0.0, wl.grad_std, generator=gen)
        if wl.grad_tail_prob > 0.0:
            mask = torch.rand(buf.shape, generator=gen, device=device) < wl.grad_tail_prob
            buf.mul_(torch.where(mask, wl.grad_tail_scale, 1.0))
        if wl.grad_zero_prob > 0.0:
            mask = torch.rand(buf.shape, generator=gen, device=device) < wl.grad_zero_prob
            buf.masked_fill_(mask, 0.0)


def _arena_views(ns, streams, device, skew_bytes, align_elems=4):
    """One allocation holding `streams` flat buckets.  Inside a bucket the K
    tensors are packed at offsets aligned to align_elems floats; bucket j starts
    at j * (bucket size rounded up to 2 MiB + skew_bytes), so that equal element
    offsets in different buckets do not share their low address bits."""
    offs, o = [], 0
    for n in ns:
        offs.append(o)
        o += (n + align_elems - 1) // align_elems * align_elems
    bucket = (o * 4 + (1 << 21) - 1) // (1 << 21) * (1 << 21) + skew_bytes
    assert bucket % 16 == 0
    arena = torch.empty(bucket * streams // 4, dtype=torch.float32, device=device)
    views = [[arena[j * (bucket // 4) + a: j * (bucket // 4) + a + n] for a, n in zip(offs, ns)]
             for j in range(streams)]
    return arena, views


def allocate(wl, device, num_workers=None, layout="separate", skew_bytes=12288, align_elems=4):
    """Allocate the full resident state for a workload: one flat fp32 tensor per
    parameter tensor per role.  Returns dict(w, v, g, u) with w, v: [K] and
    g, u: [W][K].  Momentum is zero, local weights start as a copy of w_0
    (workers pull the initial weights before the first iteration, Alg. 2).

    layout="separate": every tensor is its own torch allocation.
    layout="arena":    2 + 2W flat buckets (w, v, g_0.., u_0..) in one allocation,
                       consecutive buckets staggered by skew_bytes."""
    W = wl.num_workers if num_workers is None else num_workers
    ns = numels(wl)
    if layout == "arena":
        arena, views = _arena_views(ns, 2 + 2 * W, device, skew_bytes, align_elems)
        st = {"w": views[0], "v": views[1], "g": views[2:2 + W], "u": views[2 + W:], "arena": arena}
    else:
        mk = lambda: [torch.empty(n, dtype=torch.float32, device=device) for n in ns]
        st = {"w": mk(), "v": mk(), "g": [mk() for _ in range(W)], "u": [mk() for _ in range(W)]}
    fill_weights_(st["w"], wl)
    for b in st["v"]:
        b.zero_()
    for m in range(W):
        for k in range(len(ns)):
            st["u"][m][k].copy_(st["w"][k])
    return st


def fill_all_grads_(st, wl, iteration):
    for m in range(len(st["g"])):
        fill_grads_(st["g"][m], wl, iteration, m)
