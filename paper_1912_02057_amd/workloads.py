"""Seeded synthetic inputs for the RTN ternary conv/GEMM path.

This module only *draws inputs* (tensors, thresholds, scale/offset parameters,
layer shapes).  It holds none of the method's arithmetic -- no ternarization,
no packing, no contraction, no epilogue -- so that the HIP library and the CPU
oracle can both be fed the same bits without sharing code.  It imports neither.

Everything is generated with numpy's PCG64 on the host from an explicit seed,
as float32/float64, and handed out as numpy arrays.

Stand-ins: the paper trains and evaluates on ImageNet / CIFAR-10 with learned
weights; neither is available, so the tensors here have ResNet-18's shapes and
random values (N(0,1) activations, He-initialised weights), thresholds from the
TWN-style rule  Delta = 0.7 * mean|.|  and alpha/beta drawn from U(0.5,1.5) /
U(-0.2,0.2), or from the value ranges of the paper's Table 4.
"""
from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class ConvShape:
    name: str
    C: int       # input channels
    H: int       # input height (= width)
    O: int       # output channels
    k: int       # kernel size (k x k)
    stride: int
    pad: int

    @property
    def OH(self):
        return (self.H + 2 * self.pad - self.k) // self.stride + 1

    @property
    def K(self):
        return self.C * self.k * self.k

    def macs(self, batch):
        """Dense MAC count (padded taps included), the usual framework convention."""
        return batch * self.OH * self.OH * self.O * self.K


def resnet18_ternary_layers():
    """The 19 ternary convs of ResNet-18 (layer names as in the paper's Table 4;
    the stem conv and the FC layer stay full precision and are not listed)."""
    L = []
    L += [ConvShape("layer1.%d.conv%d" % (b, c), 64, 56, 64, 3, 1, 1) for b in (0, 1) for c in (1, 2)]
    for stage, (cin, cout, hin) in enumerate([(64, 128, 56), (128, 256, 28), (256, 512, 14)], start=2):
        hout = hin // 2
        L.append(ConvShape("layer%d.0.conv1" % stage, cin, hin, cout, 3, 2, 1))
        L.append(ConvShape("layer%d.0.conv2" % stage, cout, hout, cout, 3, 1, 1))
        L.append(ConvShape("layer%d.0.downsample.0" % stage, cin, hin, cout, 1, 2, 0))
        L.append(ConvShape("layer%d.1.conv1" % stage, cout, hout, cout, 3, 1, 1))
        L.append(ConvShape("layer%d.1.conv2" % stage, cout, hout, cout, 3, 1, 1))
    return L


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def twn_threshold(x, axis=None):
    """Delta = 0.7 * mean|x| (mean in float64, rounded once to float32).
    axis=None: one scalar; axis=0: one per leading index (per filter / per row)."""
    a = np.abs(x.astype(np.float64))
    if axis is None:
        return np.float32(0.7 * a.mean())
    return (0.7 * a.reshape(a.shape[0], -1).mean(axis=1)).astype(np.float32)


def scale_offset(rng, n=None, table4=False):
    """alpha ~ U(0.5,1.5), beta ~ U(-0.2,0.2); with table4=True the wider ranges
    the paper reports for trained ResNet-18 layers (gamma in [0.77,2.47],
    beta in [-0.23,1.48])."""
    size = () if n is None else (n,)
    if table4:
        a = rng.uniform(0.77, 2.47, size=size)
        b = rng.uniform(-0.23, 1.48, size=size)
    else:
        a = rng.uniform(0.5, 1.5, size=size)
        b = rng.uniform(-0.2, 0.2, size=size)
    return np.float32(a) if n is None else a.astype(np.float32), \
        np.float32(b) if n is None else b.astype(np.float32)


def ternary_matrix(rng, rows, cols, p_zero):
    """i.i.d. values in {-1,0,+1} as float32: P(0)=p_zero, P(+1)=P(-1)=(1-p_zero)/2."""
    u = rng.random((rows, cols), dtype=np.float32)
    half = np.float32((1.0 - p_zero) / 2.0)
    out = np.zeros((rows, cols), dtype=np.float32)
    out[u < half] = -1.0
    out[u >= np.float32(1.0) - half] = 1.0
    return out


def gemm_case(M, N, K, p_zero=0.4, seed=1, table4=False):
    """GEMM workload: activations [M,K] and weights [N,K] drawn directly as
    ternary values stored in float32 (to be ternarized at Delta = 0.5), per-row
    alpha_a/beta_a and per-column alpha_w/beta_w."""
    rng = _rng(seed)
    xa = ternary_matrix(rng, M, K, p_zero)
    xw = ternary_matrix(rng, N, K, p_zero)
    aa, ba = scale_offset(rng, M, table4)
    aw, bw = scale_offset(rng, N, table4)
    return dict(xa=xa, xw=xw, delta_a=np.float32(0.5), delta_w=np.float32(0.5),
                alpha_a=aa, beta_a=ba, alpha_w=aw, beta_w=bw, M=M, N=N, K=K)


def gemm_case_real(M, N, K, seed=1):
    """GEMM workload with real-valued inputs N(0,1) and TWN thresholds (per
    tensor for activations, per row for weights); exercises thresholding on
    non-trivial floats, including exact ties planted at the threshold."""
    rng = _rng(seed)
    xa = rng.standard_normal((M, K), dtype=np.float32)
    xw = rng.standard_normal((N, K), dtype=np.float32)
    da = twn_threshold(xa)
    dw = twn_threshold(xw, axis=0)
    # plant exact ties: |x| == Delta must ternarize to 0 (strict inequality)
    xa[0, 0] = da
    xa[-1, -1] = -da
    xw[0, 0] = dw[0]
    aa, ba = scale_offset(rng, M)
    aw, bw = scale_offset(rng, N)
    return dict(xa=xa, xw=xw, delta_a=da, delta_w=dw, alpha_a=aa, beta_a=ba,
                alpha_w=aw, beta_w=bw, M=M, N=N, K=K)


def conv_case(shape, batch, seed=0, per_channel=True, delta_a=None, table4=False, bn=False,
              Hx=None, Wx=None):
    """One ternary conv layer: x [B,C,H,W] ~ N(0,1); W [O,C,k,k] ~ N(0, sqrt(2/(C k k)))
    (He init); Delta_a = 0.7*mean|x| (one per tensor) unless given; Delta_w per
    filter (per_channel) or one per layer; alpha_a/beta_a layer-wise scalars;
    alpha_w/beta_w per output channel (per_channel) or scalars; optional BN
    affine (scale, shift) from random running statistics."""
    rng = _rng(seed)
    H = shape.H if Hx is None else Hx
    W = shape.H if Wx is None else Wx
    x = rng.standard_normal((batch, shape.C, H, W), dtype=np.float32)
    std = np.float32(np.sqrt(2.0 / shape.K))
    w = rng.standard_normal((shape.O, shape.C, shape.k, shape.k), dtype=np.float32) * std
    da = twn_threshold(x) if delta_a is None else np.float32(delta_a)
    dw = twn_threshold(w, axis=0) if per_channel else twn_threshold(w)
    aa, ba = scale_offset(rng, None, table4)
    aw, bw = scale_offset(rng, shape.O if per_channel else None, table4=False)
    out = dict(x=x, w=w, delta_a=da, delta_w=dw, alpha_a=aa, beta_a=ba, alpha_w=aw, beta_w=bw,
               shape=shape, batch=batch, H=H, W=W)
    if bn:
        mean = rng.normal(0.0, 0.1, shape.O)
        var = rng.uniform(0.5, 1.5, shape.O)
        g = rng.uniform(0.5, 1.5, shape.O)
        b = rng.normal(0.0, 0.1, shape.O)
        scale = g / np.sqrt(var + 1e-5)
        out["bn_scale"] = scale.astype(np.float32)
        out["bn_shift"] = (b - mean * scale).astype(np.float32)
    return out


# The single-layer case: 3x3, stride 1, pad 1, batch 1, 64->64 @ 56x56,
# Delta_a = 0.5, per-layer scalars.
CONFIG1_SHAPE = ConvShape("config1", 64, 56, 64, 3, 1, 1)


def config1_case():
    return conv_case(CONFIG1_SHAPE, batch=1, seed=0, per_channel=False, delta_a=0.5)


def resnet18_block_topology():
    """(conv1, conv2, downsample or None) indices into resnet18_ternary_layers() of the 8
    residual blocks, in forward order."""
    blocks = [(0, 1, None), (2, 3, None)]
    for s in range(3):
        b = 4 + 5 * s
        blocks += [(b, b + 1, b + 2), (b + 3, b + 4, None)]
    return blocks


def resnet18_network_params(seed=0, num_classes=1000):
    """Random-init parameters of the whole network of the full-forward configuration: the
    fp32 stem (7x7/2 conv 3->64 + BN), the 19 ternary convs (He-init weights, per-filter
    TWN thresholds, layer-wise activation scale/offset, per-filter weight scale/offset, BN
    affine from random running statistics) and the fp32 classifier (512 -> num_classes)."""
    rng = _rng(seed)
    stem_w = rng.standard_normal((64, 3, 7, 7), dtype=np.float32) * np.float32(np.sqrt(2.0 / (3 * 49)))
    g = rng.uniform(0.5, 1.5, 64)
    var = rng.uniform(0.5, 1.5, 64)
    stem_scale = (g / np.sqrt(var + 1e-5)).astype(np.float32)
    stem_shift = (rng.normal(0.0, 0.1, 64) - rng.normal(0.0, 0.1, 64) * stem_scale).astype(np.float32)
    layers = []
    for i, sh in enumerate(resnet18_ternary_layers()):
        c = conv_case(sh, batch=1, seed=seed * 1000 + 700 + i, per_channel=True, bn=True)
        layers.append(dict(sh=sh, w=c["w"], dw=c["delta_w"], aa=c["alpha_a"], ba=c["beta_a"], aw=c["alpha_w"],
                           bw=c["beta_w"], bs=c["bn_scale"], bh=c["bn_shift"]))
    fc_w = rng.standard_normal((num_classes, 512), dtype=np.float32) * np.float32(np.sqrt(1.0 / 512))
    fc_b = (rng.standard_normal(num_classes) * 0.01).astype(np.float32)
    return dict(stem_w=stem_w, stem_scale=stem_scale, stem_shift=stem_shift, layers=layers, fc_w=fc_w, fc_b=fc_b,
                delta_a=np.float32(0.5))
