"""The five synthetic workloads (shapes, distributions, seeds) and smaller siblings of
the same recipe for parity tests. Only input tensors are produced here; no operator
is evaluated. ``N(m, v)`` is read as mean m, variance v throughout.
"""
from __future__ import annotations

from dataclasses import dataclass
import numpy as np

from . import rng


@dataclass(frozen=True)
class SoftmaxWorkload:
    """Row-wise softmax, fp32 rows x cols, entries N(0, var 4)."""
    rows: int = 256
    cols: int = 1024
    config: int = 1

    def make(self, set_index: int = 0):
        x = rng.normal(rng.tensor_seed(self.config, 0, set_index), (self.rows, self.cols), 0.0, 4.0)
        return {"x": x}

    def bytes_moved(self) -> int:
        return 8 * self.rows * self.cols


@dataclass(frozen=True)
class LayerNormWorkload:
    """LayerNorm over the last dim: bf16 x ~ N(1, var 3); fp32 gamma ~ U[0.5,1.5],
    beta ~ N(0, var 0.1); eps 1e-5; bf16 output."""
    rows: int = 8192
    cols: int = 4096
    eps: float = 1e-5
    config: int = 2

    def make(self, set_index: int = 0):
        x = rng.normal(rng.tensor_seed(self.config, 0, set_index), (self.rows, self.cols), 1.0, 3.0)
        gamma = rng.uniform(rng.tensor_seed(self.config, 1, set_index), (self.cols,), 0.5, 1.5)
        beta = rng.normal(rng.tensor_seed(self.config, 2, set_index), (self.cols,), 0.0, 0.1)
        return {"x_bf16": rng.f32_to_bf16_bits(x), "gamma": gamma, "beta": beta}

    def bytes_moved(self) -> int:
        return 4 * self.rows * self.cols


@dataclass(frozen=True)
class GemmWorkload:
    """C = A*B, bf16 A (M x K row-major) and B (K x N column-major, i.e. stored N x K),
    entries U[-1,1], fp32 C row-major."""
    M: int = 4096
    N: int = 4096
    K: int = 4096
    config: int = 3

    def make(self, set_index: int = 0):
        a = rng.uniform(rng.tensor_seed(self.config, 0, set_index), (self.M, self.K), -1.0, 1.0)
        b = rng.uniform(rng.tensor_seed(self.config, 1, set_index), (self.N, self.K), -1.0, 1.0)
        return {"a_bf16": rng.f32_to_bf16_bits(a), "b_bf16": rng.f32_to_bf16_bits(b)}

    def flops(self) -> int:
        return 2 * self.M * self.N * self.K


@dataclass(frozen=True)
class AttnScoreWorkload:
    """Batched Q K^T scaled by alpha, then row softmax: batch = B*heads matrices,
    Q and K each [batch][seq][d] row-major bf16 with entries N(0,1)."""
    batch: int = 32 * 16
    seq: int = 512
    d: int = 64
    alpha: float = 0.125
    config: int = 4

    def make(self, set_index: int = 0):
        q = rng.normal(rng.tensor_seed(self.config, 0, set_index), (self.batch, self.seq, self.d), 0.0, 1.0)
        k = rng.normal(rng.tensor_seed(self.config, 1, set_index), (self.batch, self.seq, self.d), 0.0, 1.0)
        return {"q_bf16": rng.f32_to_bf16_bits(q), "k_bf16": rng.f32_to_bf16_bits(k)}

    def flops(self) -> int:
        return 2 * self.batch * self.seq * self.seq * self.d


@dataclass(frozen=True)
class ConvWorkload:
    """conv2d, NHWC bf16 activations ~ U[0,1], KRSC bf16 weights ~ N(0, var 2/(R*S*C))."""
    N: int = 32
    H: int = 56
    W: int = 56
    C: int = 64
    K: int = 128
    R: int = 3
    S: int = 3
    stride: int = 1
    pad: int = 1
    config: int = 5

    @property
    def P(self) -> int:
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Q(self) -> int:
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    def make(self, set_index: int = 0):
        x = rng.uniform(rng.tensor_seed(self.config, 0, set_index), (self.N, self.H, self.W, self.C), 0.0, 1.0)
        w = rng.normal(rng.tensor_seed(self.config, 1, set_index), (self.K, self.R, self.S, self.C),
                       0.0, 2.0 / (self.R * self.S * self.C))
        return {"x_bf16": rng.f32_to_bf16_bits(x), "w_bf16": rng.f32_to_bf16_bits(w)}

    def flops(self) -> int:
        return 2 * self.N * self.P * self.Q * self.K * self.R * self.S * self.C


CONFIG1 = SoftmaxWorkload()
CONFIG1_LARGE = SoftmaxWorkload(rows=131072, cols=1024)
CONFIG2 = LayerNormWorkload()
CONFIG3 = GemmWorkload()
CONFIG4 = AttnScoreWorkload()
CONFIG5 = ConvWorkload()


# Shapes of the paper's own operator table (Section 4.3) for the four operator kinds built
# here, with this module's recipes (same distributions and seeds, config numbers 11..17).
# The table gives extents only; the readings used: layernorm / softmax rows x cols (fp32);
# matmul 768x1024x1024 = M x K x N; bmm 192x256x128x256 = batch x M x K x N; conv
# N x K_out x C_in x H x W x filter, stride 1, "same" zero padding.
PAPER_SOFTMAX = SoftmaxWorkload(rows=24576, cols=512, config=11)
PAPER_LAYERNORM_1 = LayerNormWorkload(rows=16384, cols=1024, config=12)
PAPER_LAYERNORM_2 = LayerNormWorkload(rows=4096, cols=4096, config=13)
PAPER_MATMUL = GemmWorkload(M=768, N=1024, K=1024, config=14)
PAPER_BMM_BATCH = 192
PAPER_BMM = GemmWorkload(M=256, N=256, K=128, config=15)          # per matrix; PAPER_BMM_BATCH of them
PAPER_CONV_1 = ConvWorkload(N=8, H=512, W=512, C=3, K=10, R=5, S=5, pad=2, config=16)
PAPER_CONV_2 = ConvWorkload(N=8, H=56, W=56, C=64, K=64, R=3, S=3, pad=1, config=17)
