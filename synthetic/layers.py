"""Layer-shape tables (shapes only: no weights, no data) and the benchmark
configurations built from them.

The three architectures are listed as flat sequences of convolution / FC
shapes with the spatial size each layer sees; pooling, activation, residual
adds and concatenations are not layers of the block-sparse path and appear
only through the spatial sizes and channel counts they imply.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Iterator, List, Tuple

from .gen import LayerCase, draw_layer, seed_for


@dataclass(frozen=True)
class ConvSpec:
    name: str
    I: int
    O: int
    H: int
    K: int
    L: int            # input height seen by the layer
    J: int            # input width
    stride: Tuple[int, int] = (1, 1)
    pad: Tuple[int, int] = (0, 0)

    @property
    def M(self) -> int:
        return (self.L + 2 * self.pad[0] - self.H) // self.stride[0] + 1

    @property
    def N(self) -> int:
        return (self.J + 2 * self.pad[1] - self.K) // self.stride[1] + 1

    def dense_flops(self, B: int) -> int:
        return 2 * B * self.M * self.N * self.O * self.I * self.H * self.K


def _c(name, I, O, k, size, s=1, p=0) -> ConvSpec:
    kh, kw = (k, k) if isinstance(k, int) else k
    ph, pw = (p, p) if isinstance(p, int) else p
    sh, sw = (s, s) if isinstance(s, int) else s
    L, J = (size, size) if isinstance(size, int) else size
    return ConvSpec(name, I, O, kh, kw, L, J, (sh, sw), (ph, pw))


def resnet50_layers() -> List[ConvSpec]:
    """53 convolutions + the 2048->1000 FC; stride of a downsampling
    bottleneck sits on its 3x3."""
    out = [_c("conv1", 3, 64, 7, 224, s=2, p=3)]
    size = 56                     # after the 3x3/2 max pool
    inp = 64
    for stage, (width, blocks) in enumerate([(64, 3), (128, 4), (256, 6), (512, 3)], 1):
        for b in range(blocks):
            s = 2 if (b == 0 and stage > 1) else 1
            pre = f"layer{stage}.{b}"
            out.append(_c(f"{pre}.conv1", inp, width, 1, size))
            out.append(_c(f"{pre}.conv2", width, width, 3, size, s=s, p=1))
            osize = size // s
            out.append(_c(f"{pre}.conv3", width, 4 * width, 1, osize))
            if b == 0:
                out.append(_c(f"{pre}.downsample", inp, 4 * width, 1, size, s=s))
            inp = 4 * width
            size = osize
    out.append(_c("fc", 2048, 1000, 1, 1))
    return out


def vgg16_layers() -> List[ConvSpec]:
    """13 3x3 convolutions + FC 25088->4096->4096->1000."""
    out = []
    cfg = [(64, 2, 224), (128, 2, 112), (256, 3, 56), (512, 3, 28), (512, 3, 14)]
    inp = 3
    for gi, (ch, n, size) in enumerate(cfg, 1):
        for j in range(n):
            out.append(_c(f"conv{gi}_{j + 1}", inp, ch, 3, size, p=1))
            inp = ch
    out.append(_c("fc6", 25088, 4096, 1, 1))
    out.append(_c("fc7", 4096, 4096, 1, 1))
    out.append(_c("fc8", 4096, 1000, 1, 1))
    return out


def inception_v3_layers() -> List[ConvSpec]:
    """94 convolutions of the 299x299 Inception-v3 + FC 2048->1000."""
    out = [
        _c("stem.1a_3x3", 3, 32, 3, 299, s=2),
        _c("stem.2a_3x3", 32, 32, 3, 149),
        _c("stem.2b_3x3", 32, 64, 3, 147, p=1),
        _c("stem.3b_1x1", 64, 80, 1, 73),
        _c("stem.4a_3x3", 80, 192, 3, 73),
    ]

    def block_a(pre, inp, pool):
        z = 35
        out.extend([
            _c(f"{pre}.b1x1", inp, 64, 1, z),
            _c(f"{pre}.b5x5_1", inp, 48, 1, z),
            _c(f"{pre}.b5x5_2", 48, 64, 5, z, p=2),
            _c(f"{pre}.b3x3dbl_1", inp, 64, 1, z),
            _c(f"{pre}.b3x3dbl_2", 64, 96, 3, z, p=1),
            _c(f"{pre}.b3x3dbl_3", 96, 96, 3, z, p=1),
            _c(f"{pre}.pool", inp, pool, 1, z),
        ])
        return 64 + 64 + 96 + pool

    ch = block_a("mixed5b", 192, 32)
    ch = block_a("mixed5c", ch, 64)
    ch = block_a("mixed5d", ch, 64)

    out.extend([
        _c("mixed6a.b3x3", ch, 384, 3, 35, s=2),
        _c("mixed6a.b3x3dbl_1", ch, 64, 1, 35),
        _c("mixed6a.b3x3dbl_2", 64, 96, 3, 35, p=1),
        _c("mixed6a.b3x3dbl_3", 96, 96, 3, 35, s=2),
    ])
    ch = 384 + 96 + ch

    def block_c(pre, inp, c7):
        z = 17
        out.extend([
            _c(f"{pre}.b1x1", inp, 192, 1, z),
            _c(f"{pre}.b7x7_1", inp, c7, 1, z),
            _c(f"{pre}.b7x7_2", c7, c7, (1, 7), z, p=(0, 3)),
            _c(f"{pre}.b7x7_3", c7, 192, (7, 1), z, p=(3, 0)),
            _c(f"{pre}.b7x7dbl_1", inp, c7, 1, z),
            _c(f"{pre}.b7x7dbl_2", c7, c7, (7, 1), z, p=(3, 0)),
            _c(f"{pre}.b7x7dbl_3", c7, c7, (1, 7), z, p=(0, 3)),
            _c(f"{pre}.b7x7dbl_4", c7, c7, (7, 1), z, p=(3, 0)),
            _c(f"{pre}.b7x7dbl_5", c7, 192, (1, 7), z, p=(0, 3)),
            _c(f"{pre}.pool", inp, 192, 1, z),
        ])
        return 768

    for nm, c7 in (("mixed6b", 128), ("mixed6c", 160), ("mixed6d", 160), ("mixed6e", 192)):
        ch = block_c(nm, ch, c7)

    out.extend([
        _c("mixed7a.b3x3_1", ch, 192, 1, 17),
        _c("mixed7a.b3x3_2", 192, 320, 3, 17, s=2),
        _c("mixed7a.b7x7x3_1", ch, 192, 1, 17),
        _c("mixed7a.b7x7x3_2", 192, 192, (1, 7), 17, p=(0, 3)),
        _c("mixed7a.b7x7x3_3", 192, 192, (7, 1), 17, p=(3, 0)),
        _c("mixed7a.b7x7x3_4", 192, 192, 3, 17, s=2),
    ])
    ch = 320 + 192 + ch

    def block_e(pre, inp):
        z = 8
        out.extend([
            _c(f"{pre}.b1x1", inp, 320, 1, z),
            _c(f"{pre}.b3x3_1", inp, 384, 1, z),
            _c(f"{pre}.b3x3_2a", 384, 384, (1, 3), z, p=(0, 1)),
            _c(f"{pre}.b3x3_2b", 384, 384, (3, 1), z, p=(1, 0)),
            _c(f"{pre}.b3x3dbl_1", inp, 448, 1, z),
            _c(f"{pre}.b3x3dbl_2", 448, 384, 3, z, p=1),
            _c(f"{pre}.b3x3dbl_3a", 384, 384, (1, 3), z, p=(0, 1)),
            _c(f"{pre}.b3x3dbl_3b", 384, 384, (3, 1), z, p=(1, 0)),
            _c(f"{pre}.pool", inp, 192, 1, z),
        ])
        return 320 + 768 + 768 + 192

    ch = block_e("mixed7b", ch)
    ch = block_e("mixed7c", ch)
    out.append(_c("fc", ch, 1000, 1, 1))
    return out


def _case_from_spec(spec: ConvSpec, *, B: int, cfg: int, idx: int, bo=8, bi=8,
                    dtype="bf16", density=0.5, mask_kind="exact",
                    w_std=None, draw_x=True) -> LayerCase:
    return draw_layer(spec.name, B=B, L=spec.L, J=spec.J, I=spec.I, O=spec.O,
                      H=spec.H, K=spec.K, stride=spec.stride, pad=spec.pad,
                      bo=bo, bi=bi, dtype=dtype, mask_kind=mask_kind,
                      density=density, seed=seed_for(cfg, idx), w_std=w_std,
                      draw_x=draw_x)


def config_cases(cfg: int, *, batch: int | None = None,
                 draw_x: bool = True) -> Iterator[LayerCase]:
    """Yield the layers of benchmark configuration ``cfg`` (0..4).

    0  FC fp32 64x256 -> 256, 8x8, Bernoulli(0.5)
    1  3x3 conv s1 p1 bf16, X 32x56x56x64, W 64x3x3x64, 8x8, exactly half kept
    2  1x1 conv 256->1024 at 14x14, batch 32, bf16; 8x8 / 4x16 / 16x4 at block
       densities 0.25, 0.5, 0.75, 1.0
    3  ResNet50-shaped stack, batch 32, bf16, 8x8, half kept per layer
    4  VGG16- and InceptionV3-shaped stacks, batch 16, same masks
    Every X here is an independent N(0,1) draw; callers that chain a stack feed
    their own activations and pass ``draw_x=False``.
    """
    if cfg == 0:
        yield draw_layer("c0.fc", B=batch or 64, L=1, J=1, I=256, O=256,
                         dtype="f32", mask_kind="bernoulli", density=0.5,
                         seed=seed_for(0), w_std=0.02, draw_x=draw_x)
    elif cfg == 1:
        yield draw_layer("c1.conv3x3", B=batch or 32, L=56, J=56, I=64, O=64,
                         H=3, K=3, stride=1, pad=1, dtype="bf16",
                         mask_kind="exact", density=0.5, seed=seed_for(1),
                         w_std=0.05, draw_x=draw_x)
    elif cfg == 2:
        idx = 0
        for bo, bi in ((8, 8), (4, 16), (16, 4)):
            for d in (0.25, 0.5, 0.75, 1.0):
                yield draw_layer(f"c2.conv1x1.{bo}x{bi}.d{d}", B=batch or 32,
                                 L=14, J=14, I=256, O=1024, dtype="bf16",
                                 bo=bo, bi=bi, mask_kind="exact", density=d,
                                 seed=seed_for(2, idx), w_std=0.05,
                                 draw_x=draw_x)
                idx += 1
    elif cfg == 3:
        for idx, spec in enumerate(resnet50_layers()):
            c = _case_from_spec(spec, B=batch or 32, cfg=3, idx=idx, draw_x=draw_x)
            c.meta["net"] = "resnet50"
            yield c
    elif cfg == 4:
        for idx, spec in enumerate(vgg16_layers()):
            c = _case_from_spec(spec, B=batch or 16, cfg=4, idx=idx, draw_x=draw_x)
            c.meta["net"] = "vgg16"
            yield c
        for idx, spec in enumerate(inception_v3_layers()):
            c = _case_from_spec(spec, B=batch or 16, cfg=4, idx=100 + idx, draw_x=draw_x)
            c.meta["net"] = "inception_v3"
            yield c
    else:
        raise ValueError(cfg)
