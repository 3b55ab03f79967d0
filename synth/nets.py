"""Layer-list descriptions of the benchmark networks (pure data, no arithmetic).

A network is a list of dicts.  Every layer has

  op    : "linear" | "conv" | "relu" | "maxpool2" | "bn" | "add" | "gap"
  src   : index of the layer whose output it consumes (-1 = the network input)
  src2  : second operand, only for "add"

plus shape fields.  Activations are channels-last: [rows, H, W, C]; a "linear"
layer sees its input flattened in (h, w, c) order.  Parameters are one flat
fp32 vector in layer order: weight then bias for linear/conv, gamma then beta
for bn.  Linear weights are [out][in]; conv weights are [cout][kh][kw][cin].
"""
from __future__ import annotations

from typing import Dict, List, Tuple

LayerList = List[Dict]


def _shape_after(layers: LayerList, in_shape: Tuple[int, int, int]) -> List[Tuple[int, int, int]]:
    """Output (H, W, C) of every layer."""
    shapes: List[Tuple[int, int, int]] = []

    def shp(i):
        return in_shape if i < 0 else shapes[i]

    for L in layers:
        h, w, c = shp(L["src"])
        op = L["op"]
        if op == "linear":
            assert h * w * c == L["cin"], (h, w, c, L)
            shapes.append((1, 1, L["cout"]))
        elif op == "conv":
            assert c == L["cin"], (c, L)
            k, s, p = L["k"], L["stride"], L["pad"]
            shapes.append(((h + 2 * p - k) // s + 1, (w + 2 * p - k) // s + 1, L["cout"]))
        elif op in ("relu", "bn"):
            shapes.append((h, w, c))
        elif op == "maxpool2":
            assert h % 2 == 0 and w % 2 == 0
            shapes.append((h // 2, w // 2, c))
        elif op == "add":
            assert shp(L["src2"]) == (h, w, c)
            shapes.append((h, w, c))
        elif op == "gap":
            shapes.append((1, 1, c))
        else:
            raise ValueError(op)
    return shapes


def layer_shapes(layers: LayerList, in_shape):
    return _shape_after(layers, tuple(in_shape))


def param_slices(layers: LayerList) -> List[Dict[str, Tuple[int, int]]]:
    """Per layer: name -> (start, stop) in the flat parameter vector."""
    out = []
    pos = 0
    for L in layers:
        d: Dict[str, Tuple[int, int]] = {}
        if L["op"] == "linear":
            n = L["cout"] * L["cin"]
            d["w"] = (pos, pos + n); pos += n
            if L["bias"]:
                d["b"] = (pos, pos + L["cout"]); pos += L["cout"]
        elif L["op"] == "conv":
            n = L["cout"] * L["k"] * L["k"] * L["cin"]
            d["w"] = (pos, pos + n); pos += n
            if L["bias"]:
                d["b"] = (pos, pos + L["cout"]); pos += L["cout"]
        elif L["op"] == "bn":
            d["gamma"] = (pos, pos + L["c"]); pos += L["c"]
            d["beta"] = (pos, pos + L["c"]); pos += L["c"]
        out.append(d)
    return out


def param_count(layers: LayerList) -> int:
    sl = param_slices(layers)
    last = 0
    for d in sl:
        for (_, e) in d.values():
            last = max(last, e)
    return last


def mlp(dims) -> LayerList:
    """Fully connected net dims[0] -> ... -> dims[-1], ReLU between layers, biases on."""
    layers: LayerList = []
    for i in range(len(dims) - 1):
        layers.append(dict(op="linear", src=len(layers) - 1, cin=dims[i], cout=dims[i + 1], bias=True))
        if i < len(dims) - 2:
            layers.append(dict(op="relu", src=len(layers) - 1))
    return layers


def cnn3(num_classes: int = 10, hw: int = 32, chans=(3, 32, 64, 128)) -> LayerList:
    """Three 3x3 stride-1 pad-1 convolutions with bias, each followed by ReLU and a
    2x2 stride-2 max-pool, then one fully connected layer."""
    layers: LayerList = []
    s = hw
    for i in range(len(chans) - 1):
        layers.append(dict(op="conv", src=len(layers) - 1, cin=chans[i], cout=chans[i + 1],
                           k=3, stride=1, pad=1, bias=True))
        layers.append(dict(op="relu", src=len(layers) - 1))
        layers.append(dict(op="maxpool2", src=len(layers) - 1))
        s //= 2
    layers.append(dict(op="linear", src=len(layers) - 1, cin=s * s * chans[-1], cout=num_classes, bias=True))
    return layers


def resnet18(num_classes: int = 100, widths=(64, 128, 256, 512), blocks=(2, 2, 2, 2), cin: int = 3) -> LayerList:
    """ResNet-18-shaped net for 32x32 inputs: 3x3 stem (no pool), four stages of
    basic blocks, stride-2 first block in stages 2-4 with a 1x1 stride-2
    conv+bn shortcut, global average pool, fully connected classifier.
    Convolutions carry no bias; every conv is followed by batch norm."""
    layers: LayerList = []

    def add(**kw):
        layers.append(kw)
        return len(layers) - 1

    x = add(op="conv", src=-1, cin=cin, cout=widths[0], k=3, stride=1, pad=1, bias=False)
    x = add(op="bn", src=x, c=widths[0])
    x = add(op="relu", src=x)
    c_prev = widths[0]
    for si, (wd, nb) in enumerate(zip(widths, blocks)):
        for bi in range(nb):
            stride = 2 if (si > 0 and bi == 0) else 1
            y = add(op="conv", src=x, cin=c_prev, cout=wd, k=3, stride=stride, pad=1, bias=False)
            y = add(op="bn", src=y, c=wd)
            y = add(op="relu", src=y)
            y = add(op="conv", src=y, cin=wd, cout=wd, k=3, stride=1, pad=1, bias=False)
            y = add(op="bn", src=y, c=wd)
            if stride != 1 or c_prev != wd:
                sc = add(op="conv", src=x, cin=c_prev, cout=wd, k=1, stride=stride, pad=0, bias=False)
                sc = add(op="bn", src=sc, c=wd)
            else:
                sc = x
            y = add(op="add", src=y, src2=sc)
            x = add(op="relu", src=y)
            c_prev = wd
    x = add(op="gap", src=x)
    add(op="linear", src=x, cin=c_prev, cout=num_classes, bias=True)
    return layers
