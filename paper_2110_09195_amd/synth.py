"""Seeded synthetic inputs for the sub-bit convolution path.

Holds no arithmetic of the method: it only draws tensors (activations, subsets of the 512
binary kernels, index maps, scales, real-valued kernels) with the shapes and value
structure of the paper's networks.  The CPU oracle and the HIP library both consume the
arrays produced here; neither is imported by this module.

The paper's CIFAR10 / ImageNet data, trained weights and learnt subsets are not available,
so every workload is a stand-in:
  * activations: N(0,1) fp32 (their sign is the +-1 activation);
  * subset P of a layer: K codes drawn without replacement from [0, 512) (Sec. 4.2, random
    layer-specific sampling; distinct as Sec. 4.3 requires);
  * indices: i.i.d. uniform over [0, K), or Zipf(1.1)-skewed as a stand-in for the clustered
    kernel frequencies of Figs. 1 and 3;
  * alpha: U(0.5, 1.5) fp32 per output channel;
  * real-valued kernels for projection: N(0,1) fp32.
"""
from dataclasses import dataclass

import numpy as np

BASE_SEED = 20211009


@dataclass(frozen=True)
class Layer:
    name: str
    N: int
    C_in: int
    C_out: int
    H: int
    W: int
    stride: int = 1
    K: int = 32
    act: str = "bin"          # "bin" or "f32"
    index_dist: str = "uniform"  # "uniform" or "zipf"

    @property
    def H_out(self):
        return (self.H - 1) // self.stride + 1

    @property
    def W_out(self):
        return (self.W - 1) // self.stride + 1

    @property
    def pixels(self):
        return self.N * self.H_out * self.W_out

    @property
    def dense_ops(self):
        """2 * 9 * C_in * C_out * N * H_out * W_out: the dense convolution this layer equals."""
        return 2 * 9 * self.C_in * self.C_out * self.pixels


def rng(config, layer=0):
    return np.random.Generator(np.random.PCG64(BASE_SEED + 1000 * config + layer))


def activations(g, N, C, H, W):
    return g.standard_normal((N, C, H, W), dtype=np.float32)


def codebook(g, K):
    """K distinct 9-bit codes."""
    return np.sort(g.choice(512, size=K, replace=False)).astype(np.uint16)


def indices(g, C_out, C_in, K, dist="uniform"):
    if dist == "uniform":
        return g.integers(0, K, size=(C_out, C_in), dtype=np.int64).astype(np.uint16)
    if dist == "zipf":
        p = np.arange(1, K + 1, dtype=np.float64) ** -1.1
        p /= p.sum()
        rank_to_entry = g.permutation(K)
        ranks = g.choice(K, size=(C_out, C_in), p=p)
        return rank_to_entry[ranks].astype(np.uint16)
    raise ValueError(dist)


def alpha(g, C_out):
    return g.uniform(0.5, 1.5, size=C_out).astype(np.float32)


def real_kernels(g, n):
    return g.standard_normal((n, 9), dtype=np.float32)


def layer_inputs(layer, config, layer_no=0):
    """Everything one sub-bit layer needs: x fp32 NCHW, codebook, idx, alpha."""
    g = rng(config, layer_no)
    x = activations(g, layer.N, layer.C_in, layer.H, layer.W)
    cb = codebook(g, layer.K)
    idx = indices(g, layer.C_out, layer.C_in, layer.K, layer.index_dist)
    a = alpha(g, layer.C_out)
    return x, cb, idx, a


# ---- the five workloads -------------------------------------------------------------

CFG1 = Layer("resnet20-stage1", N=8, C_in=16, C_out=16, H=32, W=32, K=32, act="bin")
CFG2 = Layer("resnet20-stage3-f32", N=256, C_in=64, C_out=64, H=8, W=8, K=32, act="f32")
CFG3 = Layer("resnet18-stage3", N=128, C_in=256, C_out=256, H=14, W=14, K=32, act="bin",
             index_dist="zipf")


def cfg4(K):
    return Layer("resnet34-stage4-K%d" % K, N=256, C_in=512, C_out=512, H=7, W=7, K=K, act="bin")


def resnet18_stack(N=64, K=32):
    """The sixteen 3x3 convolutions of ResNet-18 after the stem at 224x224 input (stride-2
    layers are the first of stages 2-4).  This list reproduces the 1-bit Bit-OPs entry of
    Table 2 under the Sec. 4.5 count, which is how it was fixed."""
    spec = [(64, 64, 56, 1)] * 4 + \
           [(64, 128, 56, 2)] + [(128, 128, 28, 1)] * 3 + \
           [(128, 256, 28, 2)] + [(256, 256, 14, 1)] * 3 + \
           [(256, 512, 14, 2)] + [(512, 512, 7, 1)] * 3
    return [Layer("resnet18-conv%02d" % i, N=N, C_in=ci, C_out=co, H=hw, W=hw, stride=s, K=K)
            for i, (ci, co, hw, s) in enumerate(spec)]


def resnet34_stack(N=64, K=32):
    spec = [(64, 64, 56, 1)] * 6 + \
           [(64, 128, 56, 2)] + [(128, 128, 28, 1)] * 7 + \
           [(128, 256, 28, 2)] + [(256, 256, 14, 1)] * 11 + \
           [(256, 512, 14, 2)] + [(512, 512, 7, 1)] * 5
    return [Layer("resnet34-conv%02d" % i, N=N, C_in=ci, C_out=co, H=hw, W=hw, stride=s, K=K)
            for i, (ci, co, hw, s) in enumerate(spec)]


def resnet20_stack(N=1, K=32):
    """The eighteen 3x3 convolutions of CIFAR ResNet-20 after the stem (32x32 input)."""
    spec = [(16, 16, 32, 1)] * 6 + \
           [(16, 32, 32, 2)] + [(32, 32, 16, 1)] * 5 + \
           [(32, 64, 16, 2)] + [(64, 64, 8, 1)] * 5
    return [Layer("resnet20-conv%02d" % i, N=N, C_in=ci, C_out=co, H=hw, W=hw, stride=s, K=K)
            for i, (ci, co, hw, s) in enumerate(spec)]
