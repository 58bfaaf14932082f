"""Seeded synthetic inputs: model-shaped parameter sets and gradient buffers.

This module serves both the HIP path and the CPU oracle and therefore holds
none of the method's arithmetic: only tensor shapes (public architecture
arithmetic of CIFAR ResNet-20/56, ImageNet ResNet-50/152 and VGG-16), initial
weights and random gradients.  They stand in for the CIFAR-10 / ImageNet
training runs of the paper's evaluation (Sec. 4.1): the update pipeline is
element-wise and does not depend on where a gradient came from.
"""
import math
from collections import namedtuple

import torch

TensorSpec = namedtuple("TensorSpec", "name shape kind fan_in")
Workload = namedtuple(
    "Workload",
    "name tensors K k W steps lr momentum wd grad_sigma grad_fan_in_scale "
    "outlier_p outlier_mul seed")


def _numel(shape):
    n = 1
    for s in shape:
        n *= s
    return n


def _conv(out, name, cin, cout, ks, bn=True, bias=False):
    out.append(TensorSpec(name + ".weight", (cout, cin, ks, ks), "conv",
                          cin * ks * ks))
    if bias:
        out.append(TensorSpec(name + ".bias", (cout,), "bias", cin * ks * ks))
    if bn:
        out.append(TensorSpec(name + ".bn.gamma", (cout,), "bn_gamma", cout))
        out.append(TensorSpec(name + ".bn.beta", (cout,), "bn_beta", cout))


def _fc(out, name, cin, cout):
    out.append(TensorSpec(name + ".weight", (cout, cin), "fc", cin))
    out.append(TensorSpec(name + ".bias", (cout,), "bias", cin))


def cifar_resnet(blocks_per_stage):
    """CIFAR ResNet-(6n+2): 3x3 stem, 3 stages of n basic blocks at 16/32/64
    channels, a 1x1 projection where the width changes, BN after each conv,
    fc 64->10."""
    t = []
    _conv(t, "stem", 3, 16, 3)
    cin = 16
    for s, c in enumerate((16, 32, 64)):
        for b in range(blocks_per_stage):
            p = "s%d.b%d" % (s, b)
            _conv(t, p + ".conv1", cin, c, 3)
            _conv(t, p + ".conv2", c, c, 3)
            if cin != c:
                _conv(t, p + ".proj", cin, c, 1)
            cin = c
    _fc(t, "fc", 64, 10)
    return t


def imagenet_resnet(stages):
    """Bottleneck ResNet: 7x7 stem, stages of 1x1/3x3/1x1 blocks with widths
    64/128/256/512 (x4 out), a 1x1 projection at each stage entry, BN after
    each conv, fc 2048->1000."""
    t = []
    _conv(t, "stem", 3, 64, 7)
    cin = 64
    for s, (nb, c) in enumerate(zip(stages, (64, 128, 256, 512))):
        for b in range(nb):
            p = "s%d.b%d" % (s, b)
            _conv(t, p + ".conv1", cin, c, 1)
            _conv(t, p + ".conv2", c, c, 3)
            _conv(t, p + ".conv3", c, 4 * c, 1)
            if b == 0:
                _conv(t, p + ".proj", cin, 4 * c, 1)
            cin = 4 * c
    _fc(t, "fc", 2048, 1000)
    return t


def vgg16():
    """VGG-16: thirteen 3x3 convs with biases, then fc 25088-4096-4096-1000."""
    t = []
    cin = 3
    for i, c in enumerate((64, 64, 128, 128, 256, 256, 256, 512, 512, 512,
                           512, 512, 512)):
        _conv(t, "conv%d" % i, cin, c, 3, bn=False, bias=True)
        cin = c
    _fc(t, "fc6", 512 * 7 * 7, 4096)
    _fc(t, "fc7", 4096, 4096)
    _fc(t, "fc8", 4096, 1000)
    return t


def alexnet():
    """AlexNet (single-tower form): five convs with biases, fc 9216-4096-4096-1000."""
    t = []
    for i, (cin, cout, ks) in enumerate(((3, 64, 11), (64, 192, 5), (192, 384, 3), (384, 256, 3),
                                         (256, 256, 3))):
        _conv(t, "conv%d" % i, cin, cout, ks, bn=False, bias=True)
    _fc(t, "fc6", 256 * 6 * 6, 4096)
    _fc(t, "fc7", 4096, 4096)
    _fc(t, "fc8", 4096, 1000)
    return t


def vgg11():
    """VGG-11: eight 3x3 convs with biases, then fc 25088-4096-4096-1000."""
    t = []
    cin = 3
    for i, c in enumerate((64, 128, 256, 256, 512, 512, 512, 512)):
        _conv(t, "conv%d" % i, cin, c, 3, bn=False, bias=True)
        cin = c
    _fc(t, "fc6", 512 * 7 * 7, 4096)
    _fc(t, "fc7", 4096, 4096)
    _fc(t, "fc8", 4096, 1000)
    return t


def _wl(name, tensors, K, k, steps, **kw):
    d = dict(W=2, lr=0.1, momentum=0.9, wd=1e-4, grad_sigma=1e-2,
             grad_fan_in_scale=False, outlier_p=0.0, outlier_mul=1.0, seed=0)
    d.update(kw)
    return Workload(name=name, tensors=tensors, K=K, k=k, steps=steps, **d)


def workload(name):
    """The five benchmark configurations (and the delay sweep of the fifth)."""
    if name == "resnet20":
        return _wl(name, cifar_resnet(3), 4, 4, 10, seed=101)
    if name == "resnet56":
        return _wl(name, cifar_resnet(9), 8, 4, 50, grad_fan_in_scale=True,
                   seed=102)
    if name == "resnet50":
        return _wl(name, imagenet_resnet((3, 4, 6, 3)), 8, 5, 20, seed=103)
    if name == "vgg16":
        return _wl(name, vgg16(), 8, 4, 20, outlier_p=0.01, outlier_mul=100.0,
                   seed=104)
    if name.startswith("resnet152"):
        k = int(name.split("_k")[1]) if "_k" in name else 4
        return _wl(name, imagenet_resnet((3, 8, 36, 3)), 16, k, 20, seed=105)
    # the communication-intensive models of the paper's Sec. 4.5 (4 workers, 5-step delay)
    if name == "alexnet":
        return _wl(name, alexnet(), 4, 5, 20, seed=106)
    if name == "vgg11":
        return _wl(name, vgg11(), 4, 5, 20, seed=107)
    # any CIFAR ResNet-(6n+2), e.g. cifar_resnet110: sizes between the benchmark
    # configurations, for sweeps (K = 8, k = 4 like the ResNet-56 one)
    if name.startswith("cifar_resnet"):
        depth = int(name[len("cifar_resnet"):])
        if depth < 8 or (depth - 2) % 6:
            raise KeyError(name)
        return _wl(name, cifar_resnet((depth - 2) // 6), 8, 4, 20, grad_fan_in_scale=True, seed=108)
    # one flat tensor of N elements, e.g. flat138357544: a model without layer
    # structure, for sweeps (K = 8, k = 4)
    if name.startswith("flat"):
        n = int(name[len("flat"):])
        if n < 1:
            raise KeyError(name)
        return _wl(name, [TensorSpec("flat.weight", (n,), "fc", 1024)], 8, 4, 20, seed=109)
    raise KeyError(name)


WORKLOAD_NAMES = ("resnet20", "resnet56", "resnet50", "vgg16", "resnet152_k2",
                  "resnet152_k4", "resnet152_k8")


def numels(tensors):
    return [_numel(t.shape) for t in tensors]


def layout(tensors, align=64, shift=0):
    """Element offsets of the tensors inside one flat buffer: each start is
    rounded up to `align` elements and then moved by `shift` elements (a
    non-zero shift gives deliberately misaligned tensors).  Returns
    (offsets, total)."""
    offs, cur = [], 0
    for t in tensors:
        cur = (cur + align - 1) // align * align
        offs.append(cur + shift)
        cur += _numel(t.shape) + shift
    return offs, cur


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def initial_weights(wl, device="cpu", align=64, shift=0):
    """One flat fp32 buffer holding w_0: conv/fc ~ N(0, sqrt(2/fan_in)), BN
    gamma 1, BN beta and biases 0.  Returns (flat, offsets)."""
    offs, total = layout(wl.tensors, align, shift)
    flat = torch.zeros(total, dtype=torch.float32, device=device)
    g = _gen(device, wl.seed * 1000003 + 1)
    for t, o in zip(wl.tensors, offs):
        n = _numel(t.shape)
        v = flat[o:o + n]
        if t.kind in ("conv", "fc"):
            v.normal_(0.0, math.sqrt(2.0 / t.fan_in), generator=g)
        elif t.kind == "bn_gamma":
            v.fill_(1.0)
    return flat, offs


def gradient_set(wl, set_index, device="cpu", align=64, shift=0, skew=0, dtype=torch.float32):
    """Gradients of all K workers for one iteration: a list of K flat
    buffers laid out like the weights.  Each tensor ~ N(0, grad_sigma),
    optionally times 1/sqrt(fan_in) per layer, optionally with a seeded
    Bernoulli(outlier_p) mask of elements multiplied by outlier_mul.  Drawn
    in fp32; a 16-bit `dtype` rounds the drawn values to that type, as a
    mixed-precision backward pass would hand them over."""
    offs, total = layout(wl.tensors, align, shift)
    out = []
    for i in range(wl.K):
        g = _gen(device, (wl.seed * 1000003 + 7919 * (set_index + 1)) * 64 + i)
        # skew: worker i's buffer starts i*skew elements into its allocation,
        # so that the K buffers do not share one address alignment
        flat = torch.empty(total + i * skew, dtype=torch.float32, device=device)[i * skew:]
        flat.normal_(0.0, wl.grad_sigma, generator=g)
        if wl.grad_fan_in_scale:
            for t, o in zip(wl.tensors, offs):
                flat[o:o + _numel(t.shape)].mul_(1.0 / math.sqrt(t.fan_in))
        if wl.outlier_p > 0.0:
            m = torch.empty(total, dtype=torch.float32, device=device)
            m.uniform_(0.0, 1.0, generator=g)
            flat.mul_(torch.where(m < wl.outlier_p,
                                  torch.tensor(wl.outlier_mul, device=device),
                                  torch.tensor(1.0, device=device)))
            del m
        if dtype != torch.float32:
            # same element offsets; keep the skew in elements of the new type
            q = torch.empty(total + i * skew, dtype=dtype, device=device)[i * skew:]
            q.copy_(flat)
            flat = q
        out.append(flat)
    return out


def views(flat, tensors, offs):
    """Per-tensor 1-D views of a flat buffer."""
    return [flat[o:o + _numel(t.shape)] for t, o in zip(tensors, offs)]
