"""Seeded synthetic workloads shaped like the paper's pruned VGG-16 / ResNet-50 layers.

This module only *draws inputs*: layer shapes, sparsity patterns, weight and activation values,
and the host-side quantisation that turns the fp32 draws into the integer arrays both the GPU
library and the CPU oracle receive.  It contains none of the convolution arithmetic and imports
neither the HIP binding nor the oracle, so both sides can be fed from it.

Recipe (stands in for the paper's trained-and-pruned CIFAR / ImageNet models, Tables 6 and 7 of
the paper's GPU-results subsection, which are not available offline):
  * per output channel, ``n = max(1, floor((1 - sparsity) * K + 0.5))`` distinct positions out of
    ``K = C*R*S`` drawn uniformly at random and sorted (the "unified" per-channel non-zero count
    the paper's sparse-convolution section prescribes);
  * kept weights ~ N(0, sigma = 0.05) in fp32, activations ~ U(-1, 1) in fp32;
  * fp16 variants are round-to-nearest-even casts of the same draws;
  * int8: symmetric, per-output-channel weight scale ``max|w| / 127``, per-tensor activation
    scale ``max|x| / 127``;
  * 4-bit codebook: 16 centroids at the N(0, 0.05) quantiles ``(k + 1/2) / 16`` quantised to
    int8, every kept weight mapped to the nearest centroid (ties to the lower index);
  * 4-bit codebook with sixteen-bit centroids (the paper's 4b/16b configuration): the same 16
    centroids and the same assignment, the centroids rounded to fp16, activations fp16.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional, Tuple

import numpy as np

BASE_SEED = 21121545


@dataclasses.dataclass(frozen=True)
class Layer:
    """One convolution layer of a workload (NCHW activations, OIHW-flattened weights)."""
    name: str
    C: int
    D: int
    H: int
    W: int
    R: int = 3
    S: int = 3
    stride_h: int = 1
    stride_w: int = 1
    pad_h: int = 1
    pad_w: int = 1
    N: int = 1
    sparsity: float = 0.9
    dtype: str = "f32"          # f32 | f16 | i8 | cb4 | cb4h
    seed: int = BASE_SEED

    @property
    def K(self) -> int:
        return self.C * self.R * self.S

    @property
    def Hp(self) -> int:
        return self.H + 2 * self.pad_h

    @property
    def Wp(self) -> int:
        return self.W + 2 * self.pad_w

    @property
    def P(self) -> int:
        return (self.Hp - self.R) // self.stride_h + 1

    @property
    def Q(self) -> int:
        return (self.Wp - self.S) // self.stride_w + 1

    @property
    def n(self) -> int:
        """Stored entries per output channel for the nominal sparsity."""
        return nnz_per_channel(self.K, self.sparsity)

    @property
    def useful_macs(self) -> int:
        return self.N * self.D * self.P * self.Q * self.n

    def elem_sizes(self) -> Tuple[float, int, float]:
        """(e_x, e_y, e_w) in bytes for this layer's dtype."""
        return {"f32": (4, 4, 4.0), "f16": (2, 2, 2.0), "i8": (1, 4, 1.0), "cb4": (1, 4, 0.5),
                "cb4h": (2, 2, 0.5)}[self.dtype]

    def algorithmic_bytes(self) -> float:
        """Bytes the method must move once: input + output + stored weights and offsets."""
        ex, ey, ew = self.elem_sizes()
        b = self.N * (self.C * self.H * self.W * ex + self.D * self.P * self.Q * ey)
        b += self.D * self.n * (ew + 4)
        if self.dtype in ("i8", "cb4"):
            b += self.D * 4
        if self.dtype == "cb4":
            b += 16
        if self.dtype == "cb4h":
            b += 32
        return float(b)

    def replace(self, **kw) -> "Layer":
        return dataclasses.replace(self, **kw)


def nnz_per_channel(K: int, sparsity: float) -> int:
    return max(1, int(math.floor((1.0 - sparsity) * K + 0.5)))


# --------------------------------------------------------------------------------------------
# the five workload configurations
# --------------------------------------------------------------------------------------------

VGG_WIDTHS = [(3, 64), (64, 64), (64, 128), (128, 128), (128, 256), (256, 256), (256, 256),
              (256, 512), (512, 512), (512, 512), (512, 512), (512, 512), (512, 512)]
VGG_SPATIAL = [32, 32, 16, 16, 8, 8, 8, 4, 4, 4, 2, 2, 2]
VGG_SPARSITY = [0.70, 0.80, 0.85, 0.85, 0.90, 0.90, 0.90, 0.92, 0.92, 0.92, 0.95, 0.95, 0.95]


def config1() -> List[Layer]:
    return [Layer("cfg1_conv3x3_64x64_32", 64, 64, 32, 32, N=1, sparsity=0.9, dtype="f32",
                  seed=BASE_SEED + 1000)]


def _vgg(config: int, dtype: str, sparsities: List[float], N: int = 64) -> List[Layer]:
    out = []
    for i, ((c, d), hw, s) in enumerate(zip(VGG_WIDTHS, VGG_SPATIAL, sparsities)):
        out.append(Layer(f"vgg{i + 1}_{c}x{d}_{hw}", c, d, hw, hw, N=N, sparsity=s, dtype=dtype,
                         seed=BASE_SEED + 1000 * config + i))
    return out


def config2() -> List[Layer]:
    return _vgg(2, "f32", VGG_SPARSITY)


def resnet50_shapes() -> List[Layer]:
    """The 15 distinct bottleneck conv shapes of a ResNet-50 at 224x224 (no batch/sparsity)."""
    shapes = []
    for stage, (hw, w) in enumerate([(56, 64), (28, 128), (14, 256), (7, 512)]):
        tag = f"s{hw}"
        shapes.append(Layer(f"{tag}_reduce1x1", 4 * w, w, hw, hw, 1, 1, 1, 1, 0, 0))
        if stage > 0:
            shapes.append(Layer(f"{tag}_conv3x3_s2", w, w, 2 * hw, 2 * hw, 3, 3, 2, 2, 1, 1))
        shapes.append(Layer(f"{tag}_conv3x3", w, w, hw, hw, 3, 3, 1, 1, 1, 1))
        shapes.append(Layer(f"{tag}_expand1x1", w, 4 * w, hw, hw, 1, 1, 1, 1, 0, 0))
    return shapes


def _resnet(config: int, dtype: str, sparsities: List[float], N: int = 32) -> List[Layer]:
    out = []
    for i, sh in enumerate(resnet50_shapes()):
        for s in sparsities:
            out.append(sh.replace(name=f"{sh.name}_sp{int(round(s * 100))}", N=N, sparsity=s,
                                  dtype=dtype, seed=BASE_SEED + 1000 * config + i))
    return out


def config3() -> List[Layer]:
    return _resnet(3, "f32", [0.80, 0.90])


def config4() -> List[Layer]:
    return _resnet(4, "f16", [0.50, 0.70, 0.80, 0.90, 0.95])


def config5() -> List[Layer]:
    return _vgg(5, "i8", [0.9] * 13) + [l.replace(name=l.name + "_cb4") for l in _vgg(5, "cb4", [0.9] * 13)]


def config6() -> List[Layer]:
    """The 1-D convolution workload (Table 8 of the paper: "CNN 1D for input 300x64", kernel sizes
    2x1 and 3x1, sparsities 77 / 83 / 87.5 %, batch 128, float and half).  Reading taken: 300 input
    channels (embedding width), sequence length 64, 64 output channels, the kernel running along
    the sequence; laid out as H = 1, W = 64, R = 1, S = 2 or 3."""
    out = []
    for di, dtype in enumerate(("f32", "f16")):
        for ki, k in enumerate((2, 3)):
            for si, sp in enumerate((0.77, 0.83, 0.875)):
                pct = ("%g" % (sp * 100)).replace(".", "p")
                out.append(Layer(f"cnn1d_300x64_k{k}_sp{pct}" + ("_f16" if dtype == "f16" else ""),
                                 300, 64, 1, 64, 1, k, 1, 1, 0, 0, N=128, sparsity=sp, dtype=dtype,
                                 seed=BASE_SEED + 6000 + 100 * di + 10 * ki + si))
    return out


def config7() -> List[Layer]:
    """The paper's 4b/16b quantisation on the VGG-16-shaped stack at 90 %: weights as 4-bit indices
    into 16 sixteen-bit centroids, half-precision activations (its quantisation-results table)."""
    return [l.replace(name=l.name + "_cb4h") for l in _vgg(7, "cb4h", [0.9] * 13)]


CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5, 6: config6, 7: config7}


def headline_layer() -> Layer:
    """Largest ResNet-50-shaped layer (by bytes moved) at 90 % sparsity, fp32, batch 32."""
    for l in config3():
        if l.name == "s56_reduce1x1_sp90":
            return l
    raise AssertionError


# --------------------------------------------------------------------------------------------
# draws
# --------------------------------------------------------------------------------------------

def draw_weights_csr(layer: Layer, n: Optional[int] = None, ragged: bool = False
                     ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """CSR (rowptr[D+1] i32, colidx[nnz] i32 ascending per row, values[nnz] f32).

    ``ragged=True`` draws a different count per row (between 0 and n) to exercise row padding.
    """
    rng = np.random.default_rng(layer.seed)
    K, D = layer.K, layer.D
    n = layer.n if n is None else n
    if not 0 <= n <= K:
        raise ValueError("n out of range")
    counts = np.full(D, n, dtype=np.int64)
    if ragged:
        counts = rng.integers(0, n + 1, size=D)
        counts[rng.integers(0, D)] = n
    rowptr = np.zeros(D + 1, dtype=np.int32)
    rowptr[1:] = np.cumsum(counts)
    colidx = np.empty(int(rowptr[-1]), dtype=np.int32)
    for d in range(D):
        cnt = int(counts[d])
        if cnt == K:
            cols = np.arange(K)
        else:
            cols = np.sort(rng.choice(K, size=cnt, replace=False))
        colidx[rowptr[d]:rowptr[d + 1]] = cols
    values = rng.normal(0.0, 0.05, size=colidx.shape[0]).astype(np.float32)
    return rowptr, colidx, values


def draw_input(layer: Layer, N: Optional[int] = None) -> np.ndarray:
    """Activations U(-1, 1), fp32, NCHW."""
    rng = np.random.default_rng(layer.seed + 500)
    N = layer.N if N is None else N
    x = rng.random((N, layer.C, layer.H, layer.W), dtype=np.float32)
    x *= 2.0
    x -= 1.0
    return x


# --------------------------------------------------------------------------------------------
# host-side quantisation of the draws (input preparation, shared by both sides)
# --------------------------------------------------------------------------------------------

def quantise_weights_int8(rowptr: np.ndarray, values: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Symmetric per-output-channel int8: returns (q[nnz] int8, scale[D] f32)."""
    D = rowptr.shape[0] - 1
    q = np.zeros(values.shape[0], dtype=np.int8)
    scale = np.ones(D, dtype=np.float32)
    for d in range(D):
        v = values[rowptr[d]:rowptr[d + 1]].astype(np.float64)
        if v.size == 0:
            continue
        m = float(np.max(np.abs(v)))
        sc = m / 127.0 if m > 0 else 1.0
        scale[d] = sc
        q[rowptr[d]:rowptr[d + 1]] = np.clip(np.rint(v / sc), -127, 127).astype(np.int8)
    return q, scale


def quantise_activations_int8(x: np.ndarray) -> Tuple[np.ndarray, float]:
    m = float(np.max(np.abs(x))) if x.size else 0.0
    sc = m / 127.0 if m > 0 else 1.0
    q = np.clip(np.rint(x.astype(np.float64) / sc), -127, 127).astype(np.int8)
    return q, sc


def _norm_ppf(p: np.ndarray) -> np.ndarray:
    from scipy.special import ndtri
    return ndtri(p)


def codebook16(sigma: float = 0.05) -> Tuple[np.ndarray, np.ndarray, float]:
    """(centroids f64[16] sorted, centroids int8[16], scale) for the 4-bit non-linear quantiser."""
    k = np.arange(16, dtype=np.float64)
    c = sigma * _norm_ppf((k + 0.5) / 16.0)
    sc = float(np.max(np.abs(c))) / 127.0
    cb = np.clip(np.rint(c / sc), -127, 127).astype(np.int8)
    return c, cb, sc


def assign_codebook(values: np.ndarray, centroids: np.ndarray) -> np.ndarray:
    """Index (uint8 in [0,16)) of the nearest centroid for each value; ties go to the lower index."""
    d = np.abs(values.astype(np.float64)[:, None] - centroids[None, :])
    return np.argmin(d, axis=1).astype(np.uint8)


def prepare(layer: Layer, N: Optional[int] = None, n: Optional[int] = None, ragged: bool = False
            ) -> Dict[str, object]:
    """Everything both sides need for one layer, in the dtype the layer names.

    Returns a dict with rowptr, colidx, values (f32 | f16 | i8 | u8 indices), x (f32 | f16 | i8),
    scales (f32[D] or None), codebook (i8[16] | f16[16] or None), x_scale (float or None).
    """
    rowptr, colidx, w = draw_weights_csr(layer, n=n, ragged=ragged)
    x = draw_input(layer, N)
    out: Dict[str, object] = {"layer": layer, "rowptr": rowptr, "colidx": colidx, "scales": None,
                              "codebook": None, "x_scale": None}
    if layer.dtype == "f32":
        out["values"], out["x"] = w, x
    elif layer.dtype == "f16":
        out["values"], out["x"] = w.astype(np.float16), x.astype(np.float16)
    elif layer.dtype == "i8":
        q, sc = quantise_weights_int8(rowptr, w)
        xq, xs = quantise_activations_int8(x)
        out.update(values=q, scales=sc, x=xq, x_scale=xs)
    elif layer.dtype == "cb4":
        cent, cb, sc = codebook16()
        idx = assign_codebook(w, cent)
        xq, xs = quantise_activations_int8(x)
        out.update(values=idx, scales=np.full(layer.D, sc, dtype=np.float32), codebook=cb, x=xq,
                   x_scale=xs)
    elif layer.dtype == "cb4h":
        cent, _, _ = codebook16()
        idx = assign_codebook(w, cent)
        out.update(values=idx, codebook=cent.astype(np.float16), x=x.astype(np.float16))
    else:
        raise ValueError(layer.dtype)
    return out
