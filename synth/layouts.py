"""Tensor-list layouts with transformer-layer shapes.

The paper trains GPT-NeoX-style Pythia models (Sec. 5, "Evaluation Task");
the server state is the flattened list of that model's parameter tensors.
Only shapes matter here: every server-side step is elementwise.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple

import numpy as np


@dataclass(frozen=True)
class Layout:
    """An ordered list of parameter tensors.

    names[i]   human-readable tensor name
    shapes[i]  its shape (row-major, contiguous)
    fan_in[i]  the fan-in used to scale synthetic deltas: the first
               dimension of a weight matrix stored as (in, out); 1 for
               vectors and for the input embedding (a lookup table)
    """
    names: Tuple[str, ...]
    shapes: Tuple[Tuple[int, ...], ...]
    fan_in: Tuple[int, ...]

    @property
    def n_tensors(self) -> int:
        return len(self.shapes)

    @property
    def numel(self) -> np.ndarray:
        return np.array([int(np.prod(s)) for s in self.shapes], dtype=np.int64)

    @property
    def offsets(self) -> np.ndarray:
        """Start of each tensor in the packed flat index space (length n+1)."""
        off = np.zeros(self.n_tensors + 1, dtype=np.int64)
        np.cumsum(self.numel, out=off[1:])
        return off

    @property
    def total(self) -> int:
        return int(self.numel.sum())

    def tensor_of(self, flat_index: np.ndarray) -> np.ndarray:
        """Index of the tensor that holds each packed flat index."""
        return np.searchsorted(self.offsets, flat_index, side="right") - 1


def flat_layout(n: int) -> Layout:
    """One tensor of n elements (the Tiny workload)."""
    return Layout(("flat",), ((int(n),),), (1,))


def gpt_layout(d_model: int, n_layers: int, vocab: int = 50304, d_ff: int | None = None) -> Layout:
    """GPT-NeoX-style decoder: untied input/output embeddings, biases on every
    linear layer, two LayerNorms per block and a final LayerNorm.

    With vocab 50304 this gives 70,426,624 parameters for (512, 6),
    162,322,944 for (768, 12), 405,334,016 for (1024, 24) and
    1,011,781,632 for (2048, 16) -- the Pythia-70M/160M/410M/1B sizes.
    """
    d = int(d_model)
    ff = int(d_ff) if d_ff is not None else 4 * d
    names: List[str] = []
    shapes: List[Tuple[int, ...]] = []
    fan: List[int] = []

    def add(name, shape, fan_in):
        names.append(name)
        shapes.append(tuple(int(x) for x in shape))
        fan.append(int(fan_in))

    add("embed_in.weight", (vocab, d), 1)
    for i in range(n_layers):
        p = f"layers.{i}."
        add(p + "ln1.weight", (d,), 1)
        add(p + "ln1.bias", (d,), 1)
        add(p + "attn.qkv.weight", (d, 3 * d), d)
        add(p + "attn.qkv.bias", (3 * d,), 1)
        add(p + "attn.out.weight", (d, d), d)
        add(p + "attn.out.bias", (d,), 1)
        add(p + "ln2.weight", (d,), 1)
        add(p + "ln2.bias", (d,), 1)
        add(p + "mlp.up.weight", (d, ff), d)
        add(p + "mlp.up.bias", (ff,), 1)
        add(p + "mlp.down.weight", (ff, d), ff)
        add(p + "mlp.down.bias", (d,), 1)
    add("final_ln.weight", (d,), 1)
    add("final_ln.bias", (d,), 1)
    add("embed_out.weight", (d, vocab), d)
    return Layout(tuple(names), tuple(shapes), tuple(fan))
