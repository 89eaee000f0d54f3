"""Parameter-shape lists, in registration order (the order of
``net.parameters()`` that Algorithm 1 of the paper reverses when it fills
buckets).  Names are informational; only the order and the element counts
matter to the gradient-synchronization path.
"""
from __future__ import annotations

from math import prod
from typing import List, Tuple

Shape = Tuple[str, Tuple[int, ...]]


def tiny_shapes() -> List[Shape]:
    """Eight small fp32 tensors (14,042 elements).  The 10-element tensor
    makes bucket offsets that are not multiples of 16 bytes and the
    [128, 64] tensor alone exceeds a 16 KiB cap."""
    dims = [(64, 32), (64,), (128, 64), (128,), (10, 128), (10,),
            (3, 3, 16, 16), (16,)]
    return [(f"t{i}", d) for i, d in enumerate(dims)]


def resnet50_shapes() -> List[Shape]:
    """ResNet-50 parameter list: stem, four stages of (3, 4, 6, 3)
    bottleneck blocks (planes 64/128/256/512, expansion 4), and the
    2048 -> 1000 classifier.  Within a block the 1x1 / 3x3 / 1x1
    convolutions each come with their batch-norm scale and shift; the
    projection shortcut of a stage's first block is registered after them.
    161 tensors, 25,557,032 elements."""
    out: List[Shape] = [("conv1.w", (64, 3, 7, 7)), ("bn1.g", (64,)),
                        ("bn1.b", (64,))]
    inplanes = 64
    for stage, (planes, blocks) in enumerate(
            zip((64, 128, 256, 512), (3, 4, 6, 3)), start=1):
        for blk in range(blocks):
            pre = f"layer{stage}.{blk}."
            wide = planes * 4
            out += [(pre + "conv1.w", (planes, inplanes, 1, 1)),
                    (pre + "bn1.g", (planes,)), (pre + "bn1.b", (planes,)),
                    (pre + "conv2.w", (planes, planes, 3, 3)),
                    (pre + "bn2.g", (planes,)), (pre + "bn2.b", (planes,)),
                    (pre + "conv3.w", (wide, planes, 1, 1)),
                    (pre + "bn3.g", (wide,)), (pre + "bn3.b", (wide,))]
            if blk == 0:
                out += [(pre + "down.conv.w", (wide, inplanes, 1, 1)),
                        (pre + "down.bn.g", (wide,)),
                        (pre + "down.bn.b", (wide,))]
            inplanes = wide
    out += [("fc.w", (1000, 2048)), ("fc.b", (1000,))]
    return out


def bert_large_shapes() -> List[Shape]:
    """BERT-large parameter list: 24 layers, hidden 1024, feed-forward
    4096, vocabulary 30,522, 512 positions, 2 token types, pooler; no
    separate output head (it would share the word embedding).  391 tensors,
    335,141,888 elements."""
    h, ff = 1024, 4096
    out: List[Shape] = [("emb.word", (30522, h)), ("emb.pos", (512, h)),
                        ("emb.type", (2, h)), ("emb.ln.g", (h,)),
                        ("emb.ln.b", (h,))]
    for layer in range(24):
        pre = f"layer{layer}."
        for proj in ("q", "k", "v", "attn_out"):
            out += [(pre + proj + ".w", (h, h)), (pre + proj + ".b", (h,))]
        out += [(pre + "attn_ln.g", (h,)), (pre + "attn_ln.b", (h,)),
                (pre + "ffn_in.w", (ff, h)), (pre + "ffn_in.b", (ff,)),
                (pre + "ffn_out.w", (h, ff)), (pre + "ffn_out.b", (h,)),
                (pre + "out_ln.g", (h,)), (pre + "out_ln.b", (h,))]
    out += [("pooler.w", (h, h)), ("pooler.b", (h,))]
    return out


def uniform_shapes(count: int = 40, elems: int = 25 * (1 << 20) // 4) -> List[Shape]:
    """Diagnostic list: `count` equal tensors of `elems` elements (25 MiB of
    fp32 each by default), so that every bucket is one plain contiguous run."""
    return [(f"u{i}", (elems,)) for i in range(count)]


def numel_of(shapes: List[Shape]) -> List[int]:
    return [int(prod(d)) for _, d in shapes]


WORKLOAD_SHAPES = {
    "tiny": tiny_shapes,
    "resnet50": resnet50_shapes,
    "bert_large": bert_large_shapes,
    "uniform": uniform_shapes,
}
