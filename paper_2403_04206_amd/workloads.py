"""Seeded synthetic workloads: layer lists with the shapes of the models the paper
trains (Sec. 6: ResNet-20, WideResNet, ResNet-50 ...) and random parameter / gradient
arrays with a chosen per-(worker, layer) gradient scale.

This module holds NO arithmetic of the GRAWA update.  It only says how big the
layers are and draws the inputs; both the GPU library's tests and the CPU checker's
tests call it so that they see the same arrays.  No dataset, trained weight or real
gradient is involved: only the public architectures' tensor shapes are used, and
values are Gaussian.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np
import torch


# ----------------------------------------------------------------------------
# layer lists (sizes in elements, network order)
# ----------------------------------------------------------------------------

def _conv(cin, cout, k):
    return cin * cout * k * k


def resnet20_layers(grouped: bool = True):
    """CIFAR ResNet-20 (3 stages x 3 basic blocks, widths 16/32/64, identity shortcuts,
    FC 64x10).  grouped=True: each conv with its BN scale+shift is one segment and the FC
    weight+bias is one (20 segments); grouped=False: one segment per tensor (59)."""
    segs = []

    def conv_bn(cin, cout):
        if grouped:
            segs.append(_conv(cin, cout, 3) + 2 * cout)
        else:
            segs.extend([_conv(cin, cout, 3), cout, cout])

    conv_bn(3, 16)
    cin = 16
    for width in (16, 32, 64):
        for _ in range(3):
            conv_bn(cin, width)
            conv_bn(width, width)
            cin = width
    if grouped:
        segs.append(64 * 10 + 10)
    else:
        segs.extend([64 * 10, 10])
    return segs


def _resnet_imagenet(block, counts, num_classes=1000):
    """Per-tensor sizes of the ImageNet ResNets (7x7 stem, four stages, FC)."""
    segs = [_conv(3, 64, 7), 64, 64]
    cin = 64
    for stage, (width, n) in enumerate(zip((64, 128, 256, 512), counts)):
        for b in range(n):
            stride = 2 if (b == 0 and stage > 0) else 1
            if block == "basic":
                cout = width
                segs += [_conv(cin, width, 3), width, width, _conv(width, width, 3), width, width]
            else:
                cout = 4 * width
                segs += [_conv(cin, width, 1), width, width, _conv(width, width, 3), width, width,
                         _conv(width, cout, 1), cout, cout]
            if stride != 1 or cin != cout:
                segs += [_conv(cin, cout, 1), cout, cout]
            cin = cout
    segs += [cin * num_classes, num_classes]
    return segs


def resnet18_layers():
    return _resnet_imagenet("basic", (2, 2, 2, 2))


def resnet50_layers():
    return _resnet_imagenet("bottleneck", (3, 4, 6, 3))


def wrn28_10_layers(num_classes=100):
    """WideResNet-28-10, pre-activation blocks: per block BN, conv3x3, BN, conv3x3 and a
    1x1 shortcut conv where the width changes; final BN and FC."""
    segs = [_conv(3, 16, 3)]
    cin = 16
    for width in (160, 320, 640):
        for _ in range(4):
            segs += [cin, cin, _conv(cin, width, 3), width, width, _conv(width, width, 3)]
            if cin != width:
                segs.append(_conv(cin, width, 1))
            cin = width
    segs += [640, 640, 640 * num_classes, num_classes]
    return segs


def transformer_350m_layers(vocab=50_000, d=1024, ffn=4096, blocks=24):
    """Decoder-only transformer: token embedding, `blocks` x {LN, QKV+bias, proj+bias, LN,
    FC1+bias, FC2+bias}, final LN.  No position table."""
    segs = [vocab * d]
    for _ in range(blocks):
        segs += [d, d, d * 3 * d, 3 * d, d * d, d, d, d, d * ffn, ffn, ffn * d, d]
    segs += [d, d]
    return segs


# ----------------------------------------------------------------------------
# the five benchmark configurations
# ----------------------------------------------------------------------------

@dataclass
class Workload:
    name: str
    K: int
    layers: list
    grad_dtype: str = "f32"            # "f32" or "bf16"
    lam: float = 0.1
    lr: float | None = None            # set where the configuration includes a local SGD step
    variants: tuple = ("mgrawa", "lgrawa")
    fused_sgd: bool = False
    log10_scale: tuple = (-3.0, 1.0)   # gradient std s = 10^U(lo, hi) per (worker, layer)
    tiny_worker: int | None = None     # this worker's gradients get std 1e-6 on every layer
    scale_table: np.ndarray | None = None   # explicit [K, L] gradient stds (replaces the random draw)
    seed: tuple = (0, 0)
    offsets: np.ndarray = field(init=False)

    def __post_init__(self):
        self.offsets = np.concatenate([[0], np.cumsum(self.layers)]).astype(np.int64)

    @property
    def P(self):
        return int(self.offsets[-1])

    @property
    def L(self):
        return len(self.layers)

    @property
    def grad_bytes(self):
        return 2 if self.grad_dtype == "bf16" else 4

    def update_bytes(self):
        """Minimum HBM traffic of one distributed phase: read g once for the norms, read and
        write x once; with the fused SGD step g is read a second time."""
        per = self.grad_bytes + 8 + (self.grad_bytes if self.fused_sgd else 0)
        return self.K * self.P * per


def config(i: int) -> Workload:
    if i == 0:
        return Workload("cfg0_resnet20_K4", 4, resnet20_layers(True), lam=0.1, seed=(0, 0))
    if i == 1:
        return Workload("cfg1_resnet18_K4", 4, resnet18_layers(), lam=0.1, lr=0.1, seed=(0, 1))
    if i == 2:
        return Workload("cfg2_wrn28x10_K16", 16, wrn28_10_layers(), lam=0.05, variants=("lgrawa",), seed=(0, 2))
    if i == 3:
        return Workload("cfg3_transformer350m_K8_bf16g", 8, transformer_350m_layers(), grad_dtype="bf16",
                        lam=0.1, log10_scale=(-4.0, 0.0), seed=(0, 3))
    if i == 4:
        return Workload("cfg4_resnet50_K32_fused_sgd", 32, resnet50_layers(), lam=0.1, lr=0.1,
                        variants=("lgrawa",), fused_sgd=True, tiny_worker=0, seed=(0, 4))
    raise ValueError("configs are numbered 0..4")


N_CONFIGS = 5


# ----------------------------------------------------------------------------
# input arrays
# ----------------------------------------------------------------------------

ROW_ALIGN = 256   # elements: 1 KiB pitch granularity for fp32 rows, 512 B for bf16 rows


def round_up(n, m):
    return (n + m - 1) // m * m


def grad_scales(w: Workload) -> np.ndarray:
    """s[k, l]: standard deviation of worker k's gradient in layer l."""
    if w.scale_table is not None:
        s = np.asarray(w.scale_table, dtype=np.float64)
        if s.shape != (w.K, w.L):
            raise ValueError("scale_table must be [K, L]")
        return s
    rng = np.random.default_rng(list(w.seed) + [17])
    s = 10.0 ** rng.uniform(w.log10_scale[0], w.log10_scale[1], size=(w.K, w.L))
    if w.tiny_worker is not None:
        s[w.tiny_worker, :] = 1e-6
    return s


def make_inputs(w: Workload, device="cpu", ld_pad: int = 0, param_std: float = 0.05):
    """Draw x ~ N(0, param_std^2) (float32 [K, ld]) and g[k, layer l] ~ N(0, s[k,l]^2)
    (float32, or bfloat16 rounded to nearest even from float32).  The row pitch ld is P
    rounded up to ROW_ALIGN elements (so that every row starts on a cache-line boundary, the
    layout the library is fastest on) plus ld_pad (to break that alignment on purpose).
    Returns torch tensors on `device`; the padding columns hold a large sentinel so that a
    kernel that touches them is noticed."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(int(w.seed[0]) * 1_000_003 + int(w.seed[1]) * 7919 + 12345)
    P, K = w.P, w.K
    ld = round_up(P, ROW_ALIGN) + ld_pad
    s = torch.from_numpy(grad_scales(w)).to(torch.float32).to(dev)
    sizes = torch.from_numpy(np.diff(w.offsets)).to(dev)
    x = torch.empty((K, ld), dtype=torch.float32, device=dev)
    g = torch.empty((K, ld), dtype=torch.bfloat16 if w.grad_dtype == "bf16" else torch.float32, device=dev)
    for k in range(K):
        x[k, :P] = torch.randn(P, generator=gen, device=dev, dtype=torch.float32) * param_std
        row = torch.randn(P, generator=gen, device=dev, dtype=torch.float32)
        row *= torch.repeat_interleave(s[k], sizes)
        g[k, :P] = row.to(g.dtype)
        del row
    if ld > P:
        x[:, P:] = 7.0e7
        g[:, P:] = 3.0e4
    return x, g


def make_small(seed: int, K: int, sizes, grad_dtype="f32", ld_pad=0, device="cpu",
               log10_scale=(-3.0, 1.0)):
    """An ad-hoc workload for edge-case tests: arbitrary (ragged, unaligned) layer sizes."""
    w = Workload("small_seed%d" % seed, K, [int(v) for v in sizes], grad_dtype=grad_dtype,
                 log10_scale=log10_scale, seed=(1, seed))
    x, g = make_inputs(w, device=device, ld_pad=ld_pad)
    return w, x, g


def to_numpy_params(x: torch.Tensor) -> np.ndarray:
    return np.ascontiguousarray(x.detach().cpu().numpy())


def to_numpy_grads(g: torch.Tensor) -> np.ndarray:
    """float32 as is; bfloat16 as its uint16 bit patterns."""
    g = g.detach().cpu()
    if g.dtype == torch.bfloat16:
        return np.ascontiguousarray(g.view(torch.int16).numpy().view(np.uint16))
    return np.ascontiguousarray(g.numpy())
