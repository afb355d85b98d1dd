"""Seeded synthetic inputs for the 2:4 masked convolution: layer shapes and tensors only.

This module holds no arithmetic of the method (no compression, no convolution): it draws
weights, activations, biases and 2:4 masks with the shapes and value distributions of the CNN
workloads the paper evaluates (ResNet-50 and ConvNeXt-T from torchvision, Sec. 4
"Architectures"), which stand in for ImageNet activations and pretrained weights.  Both the GPU
path and the CPU oracle are fed from here, so they see identical bits.

Recipe: numpy Generator(PCG64(seed)); float32 draws in the fixed order W, x, bias, mask logits;
W ~ N(0, 2/K) (He fan-in) drawn as [cout, cin, kh, kw]; x = ReLU(N(0,1)) (or N(0,1) for an
image-like input) as [N, H, W, cin]; bias ~ N(0, 0.01) (variance); then cast to the 16-bit
storage type with round-to-nearest-even.  Masks are 2-of-4 along the flattened reduction index
(Sec. 3.1, Eq. 2): either the two largest |w| of each block ("top2", ties to the lower
position) or the argmax over six N(0,1) logits per block ("logits"), mimicking a learned mask.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace

import numpy as np

F16, BF16, I8, F8 = 0, 1, 2, 3
K_CRS, K_RSC = 0, 1
ACT_NONE, ACT_RELU, ACT_GELU = 0, 1, 2

# The six 2-of-4 patterns in lexicographic order of the kept positions (pattern matrix D of Eq. 2).
PATTERNS = np.array([[1, 1, 0, 0], [1, 0, 1, 0], [1, 0, 0, 1],
                     [0, 1, 1, 0], [0, 1, 0, 1], [0, 0, 1, 1]], dtype=np.uint8)


@dataclass(frozen=True)
class Layer:
    name: str
    N: int
    H: int
    W: int
    cin: int
    cout: int
    kh: int
    kw: int
    stride: int = 1
    pad: int = 0
    dtype: int = F16
    korder: int = K_CRS
    act: int = ACT_NONE
    mask: str = "top2"          # "top2" | "logits" | "none" (layer stays dense)
    relu_input: bool = True     # x = ReLU(N(0,1)) vs plain N(0,1)
    seed: int = 0
    count: int = 1              # occurrences in the network (for stack totals)

    @property
    def K(self) -> int:
        return self.cin * self.kh * self.kw

    @property
    def Ho(self) -> int:
        return (self.H + 2 * self.pad - self.kh) // self.stride + 1

    @property
    def Wo(self) -> int:
        return (self.W + 2 * self.pad - self.kw) // self.stride + 1

    @property
    def P(self) -> int:
        return self.N * self.Ho * self.Wo

    @property
    def dense_equiv_flop(self) -> int:
        return 2 * self.cout * self.P * self.K

    def algorithmic_bytes(self, sparse: bool = True) -> int:
        """x read once + y written once + weights (+ indices) + bias."""
        if self.dtype in (I8, F8):     # 8-bit operands, 16-bit output, fp32 scale and bias per channel
            xb = self.N * self.H * self.W * self.cin
            wb = (self.cout * self.K // 2 + self.cout * self.K // 8) if sparse else self.cout * self.K
            return xb + 2 * self.P * self.cout + wb + 8 * self.cout
        xb = 2 * self.N * self.H * self.W * self.cin
        yb = 2 * self.P * self.cout
        wb = (self.cout * self.K + self.cout * self.K // 8) if sparse else 2 * self.cout * self.K
        return xb + yb + wb + 4 * self.cout


def to_bits(a: np.ndarray, dtype: int) -> np.ndarray:
    """float32 array -> 16-bit storage patterns (uint16), round-to-nearest-even."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == F16:
        return a.astype(np.float16).view(np.uint16)
    u = a.view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def from_bits(b: np.ndarray, dtype: int) -> np.ndarray:
    """16-bit storage patterns -> float32 (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    if dtype == F16:
        return b.view(np.float16).astype(np.float32)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def flatten_weight(w_oihw: np.ndarray, korder: int) -> np.ndarray:
    """[cout, cin, kh, kw] -> [cout, K] in the given flattening of (c, r, t)."""
    cout = w_oihw.shape[0]
    if korder == K_CRS:
        return np.ascontiguousarray(w_oihw.reshape(cout, -1))
    return np.ascontiguousarray(w_oihw.transpose(0, 2, 3, 1).reshape(cout, -1))


def mask_top2(W_bits: np.ndarray, dtype: int) -> np.ndarray:
    """Keep the two largest |w| of every block of 4; ties go to the lower position."""
    cout, K = W_bits.shape
    mag = np.abs(from_bits(W_bits, dtype)).reshape(cout, K // 4, 4)
    order = np.argsort(-mag, axis=-1, kind="stable")
    M = np.zeros((cout, K // 4, 4), dtype=np.uint8)
    np.put_along_axis(M, order[..., :2], 1, axis=-1)
    return M.reshape(cout, K)


def mask_from_logits(logits: np.ndarray) -> np.ndarray:
    """[cout, K/4, 6] logits -> mask via argmax over the six patterns (ties to the lowest id)."""
    cout, G, _ = logits.shape
    return PATTERNS[np.argmax(logits, axis=-1)].reshape(cout, 4 * G)


def make_inputs(L: Layer) -> dict:
    """Draw (W_bits [cout,K], M [cout,K] or None, x_bits NHWC, bias fp32) for a layer."""
    rng = np.random.Generator(np.random.PCG64(L.seed))
    w = rng.standard_normal((L.cout, L.cin, L.kh, L.kw), dtype=np.float32) * np.float32(np.sqrt(2.0 / L.K))
    x = rng.standard_normal((L.N, L.H, L.W, L.cin), dtype=np.float32)
    if L.relu_input:
        np.maximum(x, 0, out=x)
    bias = rng.standard_normal(L.cout, dtype=np.float32) * np.float32(0.1)
    W_bits = flatten_weight(to_bits(w, L.dtype), L.korder)
    if L.mask == "none":
        M = None
    elif L.mask == "top2":
        M = mask_top2(W_bits, L.dtype)
    elif L.mask == "logits":
        M = mask_from_logits(rng.standard_normal((L.cout, L.K // 4, 6), dtype=np.float32))
    else:
        raise ValueError(L.mask)
    return {"W": W_bits, "M": M, "x": to_bits(x, L.dtype), "bias": bias}


def make_inputs_q8(L: Layer) -> dict:
    """The 8-bit integer variant of a layer: (W int8 [cout,K], M, x int8 NHWC, scale fp32, bias fp32).

    Draw order W, x, bias, mask logits as above; weights are the He-normal draws quantised symmetrically per output
    channel (step = max|w| / 127), activations ReLU(N(0,1)) (or N(0,1)) quantised with one step for the tensor
    (4 / 127, i.e. clipped at four standard deviations); `scale` is the product of the two steps, so that
    scale * integer sum approximates the real-valued convolution."""
    rng = np.random.Generator(np.random.PCG64(L.seed))
    w = rng.standard_normal((L.cout, L.cin, L.kh, L.kw), dtype=np.float32) * np.float32(np.sqrt(2.0 / L.K))
    x = rng.standard_normal((L.N, L.H, L.W, L.cin), dtype=np.float32)
    if L.relu_input:
        np.maximum(x, 0, out=x)
    bias = rng.standard_normal(L.cout, dtype=np.float32) * np.float32(0.1)
    w_step = np.abs(w).reshape(L.cout, -1).max(axis=1) / np.float32(127.0)
    w_step = np.where(w_step > 0, w_step, np.float32(1.0)).astype(np.float32)
    Wq = np.clip(np.rint(w / w_step[:, None, None, None]), -127, 127).astype(np.int8)
    x_step = np.float32(4.0 / 127.0)
    xq = np.clip(np.rint(x / x_step), -127, 127).astype(np.int8)
    Wq = flatten_weight(Wq, L.korder)
    if L.mask == "none":
        M = None
    elif L.mask == "top2":
        mag = np.abs(Wq.astype(np.int32)).reshape(L.cout, L.K // 4, 4)
        order = np.argsort(-mag, axis=-1, kind="stable")
        M = np.zeros((L.cout, L.K // 4, 4), dtype=np.uint8)
        np.put_along_axis(M, order[..., :2], 1, axis=-1)
        M = M.reshape(L.cout, L.K)
    elif L.mask == "logits":
        M = mask_from_logits(rng.standard_normal((L.cout, L.K // 4, 6), dtype=np.float32))
    else:
        raise ValueError(L.mask)
    return {"W": Wq, "M": M, "x": xq, "scale": (w_step * x_step).astype(np.float32), "bias": bias}


def to_e4m3(a: np.ndarray) -> np.ndarray:
    """float32 array -> OCP FP8 E4M3 bytes (uint8), round-to-nearest-even, saturating at +-448 (a storage cast of the
    inputs, done by the tensor library)."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).clamp_(-448.0, 448.0)
    return t.to(torch.float8_e4m3fn).view(torch.uint8).numpy()


def make_inputs_f8(L: Layer) -> dict:
    """The FP8 (E4M3) variant of a layer: (W bytes [cout,K], M, x bytes NHWC, scale fp32, bias fp32).

    Same draws as make_inputs; weights are divided per output channel by max|w| / 448 and activations by 4 / 448
    (four standard deviations map to the format's largest value) before the cast; `scale` is the product of the two
    divisors.  "top2" masks rank the magnitudes of the cast bytes (sign bit dropped: E4M3 is monotone in the rest)."""
    rng = np.random.Generator(np.random.PCG64(L.seed))
    w = rng.standard_normal((L.cout, L.cin, L.kh, L.kw), dtype=np.float32) * np.float32(np.sqrt(2.0 / L.K))
    x = rng.standard_normal((L.N, L.H, L.W, L.cin), dtype=np.float32)
    if L.relu_input:
        np.maximum(x, 0, out=x)
    bias = rng.standard_normal(L.cout, dtype=np.float32) * np.float32(0.1)
    w_step = np.abs(w).reshape(L.cout, -1).max(axis=1) / np.float32(448.0)
    w_step = np.where(w_step > 0, w_step, np.float32(1.0)).astype(np.float32)
    Wb = flatten_weight(to_e4m3(w / w_step[:, None, None, None]), L.korder)
    x_step = np.float32(4.0 / 448.0)
    xb = to_e4m3(x / x_step)
    if L.mask == "none":
        M = None
    elif L.mask == "top2":
        mag = (Wb & 0x7F).astype(np.int32).reshape(L.cout, L.K // 4, 4)
        order = np.argsort(-mag, axis=-1, kind="stable")
        M = np.zeros((L.cout, L.K // 4, 4), dtype=np.uint8)
        np.put_along_axis(M, order[..., :2], 1, axis=-1)
        M = M.reshape(L.cout, L.K)
    elif L.mask == "logits":
        M = mask_from_logits(rng.standard_normal((L.cout, L.K // 4, 6), dtype=np.float32))
    else:
        raise ValueError(L.mask)
    return {"W": Wb, "M": M, "x": xb, "scale": (w_step * x_step).astype(np.float32), "bias": bias}


def make_weights(L: Layer, scale: float = 1.0) -> dict:
    """Only (W_bits, M, bias) of a layer, for a chained stack whose activations come from the layer before.
    `scale` multiplies the He-normal weights (the last convolution of a residual branch is drawn smaller so that
    the un-normalised sum of sixteen branches stays in range)."""
    rng = np.random.Generator(np.random.PCG64(L.seed))
    w = rng.standard_normal((L.cout, L.cin, L.kh, L.kw), dtype=np.float32) * np.float32(scale * np.sqrt(2.0 / L.K))
    bias = rng.standard_normal(L.cout, dtype=np.float32) * np.float32(0.1)
    W_bits = flatten_weight(to_bits(w, L.dtype), L.korder)
    M = None if L.mask == "none" else mask_top2(W_bits, L.dtype)
    return {"W": W_bits, "M": M, "bias": bias}


def make_small_int_inputs(L: Layer, seed: int = 0) -> dict:
    """Small-integer tensors (w in {-1,0,1}, x in {0,1,2}, integer bias) for which no rounding
    occurs anywhere as long as every partial sum stays below the storage type's exact-integer
    range: the GPU result must then equal the oracle bit for bit."""
    rng = np.random.Generator(np.random.PCG64(seed))
    w = rng.integers(-1, 2, size=(L.cout, L.cin, L.kh, L.kw)).astype(np.float32)
    x = rng.integers(0, 3, size=(L.N, L.H, L.W, L.cin)).astype(np.float32)
    bias = rng.integers(-2, 3, size=L.cout).astype(np.float32)
    W_bits = flatten_weight(to_bits(w, L.dtype), L.korder)
    M = mask_from_logits(rng.standard_normal((L.cout, L.K // 4, 6), dtype=np.float32))
    return {"W": W_bits, "M": M, "x": to_bits(x, L.dtype), "bias": bias}


# --------------------------------------------------------------------------------------------
# Benchmark configurations
# --------------------------------------------------------------------------------------------

CONFIG0 = Layer("cfg0_3x3_64_16x16_f16", N=1, H=16, W=16, cin=64, cout=64, kh=3, kw=3, stride=1, pad=1,
                dtype=F16, act=ACT_NONE, mask="top2", seed=0)
CONFIG1 = Layer("cfg1_3x3_256_14x14_n32_f16", N=32, H=14, W=14, cin=256, cout=256, kh=3, kw=3, stride=1,
                pad=1, dtype=F16, act=ACT_RELU, mask="logits", seed=0)
CONFIG2 = Layer("cfg2_1x1_1024_256_14x14_n64_bf16", N=64, H=14, W=14, cin=1024, cout=256, kh=1, kw=1,
                dtype=BF16, act=ACT_RELU, mask="top2", seed=0)


def resnet50_layers(batch: int = 64, dtype: int = BF16) -> list[Layer]:
    """The 53 convolutions of torchvision's ResNet-50 (stride on the 3x3) at 224x224, as 24
    unique shapes with occurrence counts.  The 7x7 stem (cin=3) and the four downsample
    shortcuts stay dense; everything else carries a top-2 mask along cin*kh*kw.  BN is folded
    into the bias.  ReLU follows conv1/conv2 of a bottleneck; conv3 and shortcuts have none."""
    out: list[Layer] = []

    def add(name, H, cin, cout, k, s, mask, act, count, relu_input=True):
        idx = len(out)
        out.append(Layer(name, N=batch, H=H, W=H, cin=cin, cout=cout, kh=k, kw=k, stride=s, pad=k // 2,
                         dtype=dtype, act=act, mask=mask, relu_input=relu_input,
                         seed=3000 + idx, count=count))

    add("stem_7x7_3_64_s2", 224, 3, 64, 7, 2, "none", ACT_RELU, 1, relu_input=False)
    # stage 1 (56x56), width 64 -> 256
    add("s1_c1_1x1_64_64", 56, 64, 64, 1, 1, "top2", ACT_RELU, 1)
    add("s1_c2_3x3_64_64", 56, 64, 64, 3, 1, "top2", ACT_RELU, 3)
    add("s1_c3_1x1_64_256", 56, 64, 256, 1, 1, "top2", ACT_NONE, 3)
    add("s1_ds_1x1_64_256", 56, 64, 256, 1, 1, "none", ACT_NONE, 1)
    add("s1_c1_1x1_256_64", 56, 256, 64, 1, 1, "top2", ACT_RELU, 2)
    # stage 2 (28x28), width 128 -> 512
    add("s2_c1_1x1_256_128", 56, 256, 128, 1, 1, "top2", ACT_RELU, 1)
    add("s2_c2_3x3_128_128_s2", 56, 128, 128, 3, 2, "top2", ACT_RELU, 1)
    add("s2_c3_1x1_128_512", 28, 128, 512, 1, 1, "top2", ACT_NONE, 4)
    add("s2_ds_1x1_256_512_s2", 56, 256, 512, 1, 2, "none", ACT_NONE, 1)
    add("s2_c1_1x1_512_128", 28, 512, 128, 1, 1, "top2", ACT_RELU, 3)
    add("s2_c2_3x3_128_128", 28, 128, 128, 3, 1, "top2", ACT_RELU, 3)
    # stage 3 (14x14), width 256 -> 1024
    add("s3_c1_1x1_512_256", 28, 512, 256, 1, 1, "top2", ACT_RELU, 1)
    add("s3_c2_3x3_256_256_s2", 28, 256, 256, 3, 2, "top2", ACT_RELU, 1)
    add("s3_c3_1x1_256_1024", 14, 256, 1024, 1, 1, "top2", ACT_NONE, 6)
    add("s3_ds_1x1_512_1024_s2", 28, 512, 1024, 1, 2, "none", ACT_NONE, 1)
    add("s3_c1_1x1_1024_256", 14, 1024, 256, 1, 1, "top2", ACT_RELU, 5)
    add("s3_c2_3x3_256_256", 14, 256, 256, 3, 1, "top2", ACT_RELU, 5)
    # stage 4 (7x7), width 512 -> 2048
    add("s4_c1_1x1_1024_512", 14, 1024, 512, 1, 1, "top2", ACT_RELU, 1)
    add("s4_c2_3x3_512_512_s2", 14, 512, 512, 3, 2, "top2", ACT_RELU, 1)
    add("s4_c3_1x1_512_2048", 7, 512, 2048, 1, 1, "top2", ACT_NONE, 3)
    add("s4_ds_1x1_1024_2048_s2", 14, 1024, 2048, 1, 2, "none", ACT_NONE, 1)
    add("s4_c1_1x1_2048_512", 7, 2048, 512, 1, 1, "top2", ACT_RELU, 2)
    add("s4_c2_3x3_512_512", 7, 512, 512, 3, 1, "top2", ACT_RELU, 2)
    assert sum(l.count for l in out) == 53
    return out


def convnext_t_stage1_layers(batch: int = 128, dtype: int = BF16) -> list[Layer]:
    """Masked convolutions of ConvNeXt-T stage 1 at 56x56: the pointwise expansion 96->384 and
    contraction 384->96 of each of the 3 blocks (2:4 along cin, argmax-of-logits masks) and the
    2x2 stride-2 downsample 96->192 (K=384).  The 7x7 depthwise convolution is grouped and stays
    dense (Sec. 4 "Architectures"); it is outside this library's boundary."""
    return [
        Layer("cnx_pw_96_384", N=batch, H=56, W=56, cin=96, cout=384, kh=1, kw=1, dtype=dtype,
              act=ACT_NONE, mask="logits", relu_input=False, seed=4000, count=3),
        Layer("cnx_pw_384_96", N=batch, H=56, W=56, cin=384, cout=96, kh=1, kw=1, dtype=dtype,
              act=ACT_NONE, mask="logits", relu_input=False, seed=4001, count=3),
        Layer("cnx_ds_2x2_96_192_s2", N=batch, H=56, W=56, cin=96, cout=192, kh=2, kw=2, stride=2, pad=0,
              dtype=dtype, act=ACT_NONE, mask="logits", relu_input=False, seed=4002, count=1),
    ]


def with_batch(L: Layer, N: int) -> Layer:
    return replace(L, N=N, name=f"{L.name}@N{N}")
