"""Parameter-set shapes of the workloads the paper evaluates (Section 5.2, Table 2).

Only the *shapes* are used: tensors are filled with seeded synthetic values.  The
layer lists are the public, standard architecture definitions (ResNet-50 bottleneck
network; BERT-large encoder), written out here as tensor shapes.
"""
from __future__ import annotations

from dataclasses import dataclass
from math import prod
from typing import List, Sequence, Tuple


@dataclass(frozen=True)
class ParamSet:
    """An ordered list of named tensor shapes; one replica holds one of each."""
    name: str
    names: Tuple[str, ...]
    shapes: Tuple[Tuple[int, ...], ...]

    @property
    def numel(self) -> List[int]:
        return [prod(s) for s in self.shapes]

    @property
    def n_tensors(self) -> int:
        return len(self.shapes)

    @property
    def P(self) -> int:
        return sum(self.numel)

    @property
    def offsets(self) -> List[int]:
        """Start of each tensor in the unpadded concatenation (length n_tensors + 1)."""
        out, acc = [0], 0
        for n in self.numel:
            acc += n
            out.append(acc)
        return out

    def fan_in(self, t: int) -> int:
        """Fan-in used for Kaiming-normal init: product of all dims but the first;
        for 1-D tensors (normalisation scales, biases) the element count."""
        s = self.shapes[t]
        return prod(s[1:]) if len(s) >= 2 else s[0]


def flat_param_set(P: int, name: str = "flat") -> ParamSet:
    return ParamSet(name, ("w",), ((int(P),),))


def custom_param_set(numel: Sequence[int], name: str = "custom") -> ParamSet:
    return ParamSet(name, tuple(f"t{i}" for i in range(len(numel))),
                    tuple((int(n),) for n in numel))


def resnet50_param_set() -> ParamSet:
    """ResNet-50: 161 tensors, 25,557,032 parameters (53 convolutions, 53 normalisation
    scale/shift pairs, one fully connected layer with bias)."""
    names: List[str] = []
    shapes: List[Tuple[int, ...]] = []

    def conv_bn(tag: str, cout: int, cin: int, k: int) -> None:
        names.append(f"{tag}.conv.weight"); shapes.append((cout, cin, k, k))
        names.append(f"{tag}.bn.weight");   shapes.append((cout,))
        names.append(f"{tag}.bn.bias");     shapes.append((cout,))

    conv_bn("stem", 64, 3, 7)
    cin = 64
    for stage, (blocks, width) in enumerate([(3, 64), (4, 128), (6, 256), (3, 512)], start=1):
        for b in range(blocks):
            tag = f"layer{stage}.{b}"
            conv_bn(f"{tag}.a", width, cin, 1)
            conv_bn(f"{tag}.b", width, width, 3)
            conv_bn(f"{tag}.c", 4 * width, width, 1)
            if b == 0:
                conv_bn(f"{tag}.downsample", 4 * width, cin, 1)
            cin = 4 * width
    names.append("fc.weight"); shapes.append((1000, 2048))
    names.append("fc.bias");   shapes.append((1000,))
    return ParamSet("resnet50", tuple(names), tuple(shapes))


def bert_large_param_set() -> ParamSet:
    """BERT-large encoder: 24 layers, hidden 1024, FFN 4096, vocabulary 30522, 512 positions;
    391 tensors, 335,141,888 parameters."""
    H, F, V, L, NPOS = 1024, 4096, 30522, 24, 512
    names: List[str] = []
    shapes: List[Tuple[int, ...]] = []

    def add(n: str, *s: int) -> None:
        names.append(n); shapes.append(tuple(s))

    add("emb.word", V, H); add("emb.position", NPOS, H); add("emb.token_type", 2, H)
    add("emb.ln.weight", H); add("emb.ln.bias", H)
    for l in range(L):
        p = f"layer{l}"
        for proj in ("q", "k", "v", "o"):
            add(f"{p}.attn.{proj}.weight", H, H); add(f"{p}.attn.{proj}.bias", H)
        add(f"{p}.attn.ln.weight", H); add(f"{p}.attn.ln.bias", H)
        add(f"{p}.ffn.in.weight", F, H); add(f"{p}.ffn.in.bias", F)
        add(f"{p}.ffn.out.weight", H, F); add(f"{p}.ffn.out.bias", H)
        add(f"{p}.ffn.ln.weight", H); add(f"{p}.ffn.ln.bias", H)
    add("pooler.weight", H, H); add("pooler.bias", H)
    return ParamSet("bert_large", tuple(names), tuple(shapes))
