"""Shapes of the five benchmark workloads and their seeded synthetic tensors.

This module holds NO arithmetic of the method: it only lists layer shapes (copied from the public
architectures the paper evaluates on, Section 5.1) and draws seeded random tensors.  It is the one module
shared by the HIP-path tests/bench and the CPU oracle: both sides receive the same bytes.

The paper's datasets and pre-trained weights are not available; tensors here stand in for them and copy
only shapes, batch sizes and value distributions:
  cfg 0  one linear layer 512 -> 256, 64 tokens, fp32, N(0,1)
  cfg 1  WideResNet-28-10 conv stack, batch 200, 32x32 inputs, fp32; conv inputs are post-ReLU
         (max(0, N(0,1)), ~50 % exact zeros), the stem input is U(0,1) + N(0, 0.1^2)
  cfg 2  ResNet-50 conv stack, batch 64, 224x224 inputs, bf16, post-ReLU inputs, stem U(0,1) + N(0, 0.2^2)
  cfg 3  ViT-B/16 encoder linears, batch 64 x 197 tokens, bf16, N(0,1)
  cfg 4  hierarchical segmentation transformer linears (4 stages, channels 64/128/320/512), batch 2,
         1024x512 inputs, bf16, N(0,1)
"""
from dataclasses import dataclass, replace
from typing import List

import torch


@dataclass(frozen=True)
class Layer:
    name: str
    kind: str            # "linear" | "conv2d"
    dtype: str           # "f32" | "bf16"
    group_len: int       # selection scope used on the performance path
    dist: str = "normal"  # distribution of the cached activation: "normal" | "relu" | "image01" | "image02"
    # linear: A [M, K], dY [M, N], dW [N, K]
    M: int = 0
    K: int = 0
    N: int = 0
    # conv2d: A [Nb, Ci, H, W], dY [Nb, Co, OH, OW], dW [Co, Ci, kh, kw]
    Nb: int = 0
    Ci: int = 0
    H: int = 0
    W: int = 0
    Co: int = 0
    kh: int = 1
    kw: int = 1
    stride: int = 1
    pad: int = 0

    @property
    def OH(self):
        return (self.H + 2 * self.pad - self.kh) // self.stride + 1

    @property
    def OW(self):
        return (self.W + 2 * self.pad - self.kw) // self.stride + 1

    @property
    def a_shape(self):
        return (self.M, self.K) if self.kind == "linear" else (self.Nb, self.Ci, self.H, self.W)

    @property
    def dy_shape(self):
        return (self.M, self.N) if self.kind == "linear" else (self.Nb, self.Co, self.OH, self.OW)

    @property
    def dw_shape(self):
        return (self.N, self.K) if self.kind == "linear" else (self.Co, self.Ci, self.kh, self.kw)

    @property
    def n(self):
        s = 1
        for d in self.a_shape:
            s *= d
        return s

    @property
    def n_dy(self):
        s = 1
        for d in self.dy_shape:
            s *= d
        return s

    @property
    def n_w(self):
        s = 1
        for d in self.dw_shape:
            s *= d
        return s

    @property
    def elem_bytes(self):
        return 4 if self.dtype == "f32" else 2

    @property
    def dense_flops(self):
        """Dense-equivalent flops of the weight gradient (2 per multiply-add)."""
        if self.kind == "linear":
            return 2 * self.M * self.K * self.N
        return 2 * self.Nb * self.OH * self.OW * self.Co * self.Ci * self.kh * self.kw


def _conv(name, dtype, nb, ci, hw, co, k, stride, dist="relu"):
    return Layer(name=name, kind="conv2d", dtype=dtype, group_len=4096, dist=dist, Nb=nb, Ci=ci, H=hw, W=hw, Co=co,
                 kh=k, kw=k, stride=stride, pad=k // 2)


def _lin(name, dtype, m, k, n, dist="normal"):
    return Layer(name=name, kind="linear", dtype=dtype, group_len=k, dist=dist, M=m, K=k, N=n)


def cfg0_single_linear() -> List[Layer]:
    return [_lin("fc", "f32", 64, 512, 256)]


def cfg1_wideresnet28_10(batch=200) -> List[Layer]:
    """28 convolutions: stem, 3 stages x 4 basic blocks x two 3x3 convs, one 1x1 shortcut per stage."""
    L = [_conv("stem", "f32", batch, 3, 32, 16, 3, 1, dist="image01")]
    cin, hw = 16, 32
    for s, width in enumerate((160, 320, 640)):
        for b in range(4):
            stride = 2 if (s > 0 and b == 0) else 1
            L.append(_conv(f"s{s+1}b{b+1}.conv1", "f32", batch, cin, hw, width, 3, stride))
            hw_out = hw // stride
            L.append(_conv(f"s{s+1}b{b+1}.conv2", "f32", batch, width, hw_out, width, 3, 1))
            if b == 0:
                L.append(_conv(f"s{s+1}b{b+1}.shortcut", "f32", batch, cin, hw, width, 1, stride))
            cin, hw = width, hw_out
    assert len(L) == 28
    return L


def cfg2_resnet50(batch=64, image=224) -> List[Layer]:
    """53 convolutions: 7x7/2 stem, bottlenecks [3,4,6,3], stride on the 3x3, 1x1 downsample per stage."""
    L = [_conv("stem", "bf16", batch, 3, image, 64, 7, 2, dist="image02")]
    hw = image // 4  # stem stride 2, then 3x3/2 max-pool
    cin = 64
    for s, (width, blocks) in enumerate(zip((64, 128, 256, 512), (3, 4, 6, 3))):
        for b in range(blocks):
            stride = 2 if (s > 0 and b == 0) else 1
            L.append(_conv(f"s{s+1}b{b+1}.conv1", "bf16", batch, cin, hw, width, 1, 1))
            L.append(_conv(f"s{s+1}b{b+1}.conv2", "bf16", batch, width, hw, width, 3, stride))
            hw_out = hw // stride
            L.append(_conv(f"s{s+1}b{b+1}.conv3", "bf16", batch, width, hw_out, 4 * width, 1, 1))
            if b == 0:
                L.append(_conv(f"s{s+1}b{b+1}.downsample", "bf16", batch, cin, hw, 4 * width, 1, stride))
            cin, hw = 4 * width, hw_out
    assert len(L) == 53
    return L


def cfg3_vit_b16(batch=64, tokens=197) -> List[Layer]:
    """48 linears: 12 blocks x {qkv, proj, fc1, fc2}."""
    m = batch * tokens
    L = []
    for b in range(12):
        L += [_lin(f"blk{b}.qkv", "bf16", m, 768, 2304), _lin(f"blk{b}.proj", "bf16", m, 768, 768),
              _lin(f"blk{b}.fc1", "bf16", m, 768, 3072), _lin(f"blk{b}.fc2", "bf16", m, 3072, 768)]
    return L


def cfg4_segformer_like(batch=2, height=1024, width=512) -> List[Layer]:
    """266 linears of a 4-stage hierarchical encoder (depths 3/6/40/3) and an all-MLP decoder."""
    chans, depths, strides = (64, 128, 320, 512), (3, 6, 40, 3), (4, 8, 16, 32)
    kv_tokens = batch * (height // 32) * (width // 32)  # spatially reduced keys/values
    L = []
    for s, (c, d, st) in enumerate(zip(chans, depths, strides)):
        t = batch * (height // st) * (width // st)
        for b in range(d):
            p = f"st{s+1}b{b+1}."
            L += [_lin(p + "q", "bf16", t, c, c), _lin(p + "kv", "bf16", kv_tokens, c, 2 * c),
                  _lin(p + "proj", "bf16", t, c, c), _lin(p + "fc1", "bf16", t, c, 4 * c),
                  _lin(p + "fc2", "bf16", t, 4 * c, c)]
    for s, (c, st) in enumerate(zip(chans, strides)):
        L.append(_lin(f"dec.proj{s+1}", "bf16", batch * (height // st) * (width // st), c, 768))
    t0 = batch * (height // 4) * (width // 4)
    L += [_lin("dec.fuse", "bf16", t0, 3072, 768), _lin("dec.cls", "bf16", t0, 768, 19)]
    assert len(L) == 266
    return L


# intervals the per-layer ratios are mapped into, per config (cfg 0 uses the fixed r = 0.5)
RATIO_RANGE = {0: (0.5, 0.5), 1: (0.3, 0.9), 2: (0.5, 0.95), 3: (0.5, 0.9), 4: (0.6, 0.95)}
IMPORTANCE_PASS_RATIO = 0.9  # static ratio of the extra forward-backward pass (Section 4.2, strategy (ii))


def config_layers(cfg: int, **kw) -> List[Layer]:
    return (cfg0_single_linear, cfg1_wideresnet28_10, cfg2_resnet50, cfg3_vit_b16, cfg4_segformer_like)[cfg](**kw)


def shrink(layer: Layer, batch_div: int) -> Layer:
    """The same layer at a smaller batch (fewer tokens / images) for parity tests the oracle can finish."""
    if layer.kind == "linear":
        return replace(layer, M=max(1, layer.M // batch_div))
    return replace(layer, Nb=max(1, layer.Nb // batch_div))


def distinct_shapes(layers: List[Layer]) -> List[Layer]:
    """First layer of every distinct (shape, dtype) in the list."""
    seen, out = set(), []
    for l in layers:
        key = (l.kind, l.dtype, l.a_shape, l.dy_shape, l.kh, l.kw, l.stride, l.pad)
        if key not in seen:
            seen.add(key)
            out.append(l)
    return out


_ROLES = {"A": 1, "dY": 2}


def tensor_seed(cfg: int, layer_index: int, role: str, base_seed: int = 0) -> int:
    return (base_seed * 1_000_003 + cfg * 100_003 + layer_index * 101 + _ROLES[role]) & 0x7FFFFFFF


def _torch_dtype(dtype: str):
    return torch.float32 if dtype == "f32" else torch.bfloat16


def draw(shape, dist: str, dtype: str, seed: int, device="cpu") -> torch.Tensor:
    """Seeded synthetic tensor.  Drawn in fp32 on `device`, then rounded to the storage dtype."""
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    if dist == "normal":
        t = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    elif dist == "relu":
        t = torch.randn(shape, generator=g, device=device, dtype=torch.float32).clamp_(min=0.0)
    elif dist in ("image01", "image02"):
        sigma = 0.1 if dist == "image01" else 0.2
        t = torch.rand(shape, generator=g, device=device, dtype=torch.float32)
        t += sigma * torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    else:
        raise ValueError(dist)
    return t.to(_torch_dtype(dtype)).contiguous()


def layer_tensors(cfg: int, layer_index: int, layer: Layer, device="cpu", base_seed: int = 0):
    """(A, dY) for one layer, seeded by (config, layer, role)."""
    A = draw(layer.a_shape, layer.dist, layer.dtype, tensor_seed(cfg, layer_index, "A", base_seed), device)
    dY = draw(layer.dy_shape, "normal", layer.dtype, tensor_seed(cfg, layer_index, "dY", base_seed), device)
    return A, dY


def to_numpy_bits(t: torch.Tensor):
    """Host numpy view of a tensor for the oracle: float32 as is, bfloat16 as its uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view("uint16")
    return t.numpy()
