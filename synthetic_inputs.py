"""Seeded synthetic workloads for the redistribution path (inputs only).

This module holds no redistribution arithmetic: it names meshes, writes
distributed types as text, and draws seeded global arrays.  Both the CPU
oracle's tests and the GPU harness take their inputs from here; neither side's
code is imported.

The five workloads mirror the shapes deep-learning redistributions have
(activations switching between batch- and hidden-sharded layouts, weight axis
swaps, gathers to full replicas, attention tensors resharded at random), which
is also how the paper samples its own evaluation problems (random problems,
each mesh axis either replicated or partitioning one dimension, Sec. 8).
bf16 data is carried as raw uint16 bit patterns: the path moves bytes only.
"""
from __future__ import annotations

import random
from math import prod

import numpy as np

BASE_SEED = 211201075

# name -> dtype tag, bytes per element, global shape, mesh (declaration order), list of (src, dst) types
WORKLOADS = {
    "c1_int32_2x2": {
        "dtype": "int32", "elem_size": 4, "gshape": (64, 48), "mesh": {"a": 2, "b": 2},
        "pairs": [("[32{a}64, 24{b}48]", "[16{a,b}64, 48]"),
                  ("[16{a,b}64, 48]", "[32{a}64, 24{b}48]")],
    },
    "c2_bf16_act_1x8": {
        "dtype": "bf16", "elem_size": 2, "gshape": (4096, 8192), "mesh": {"x": 8},
        "pairs": [("[512{x}4096, 8192]", "[4096, 1024{x}8192]"),
                  ("[4096, 1024{x}8192]", "[512{x}4096, 8192]")],
    },
    "c3_fp32_weight_4x2": {
        "dtype": "fp32", "elem_size": 4, "gshape": (8192, 32768), "mesh": {"x": 4, "y": 2},
        "pairs": [("[2048{x}8192, 16384{y}32768]", "[4096{y}8192, 8192{x}32768]")],
    },
    "c4_bf16_act_2x4x4": {
        "dtype": "bf16", "elem_size": 2, "gshape": (64, 2048, 4096), "mesh": {"x": 2, "y": 4, "z": 4},
        "pairs": [("[32{x}64, 512{y}2048, 1024{z}4096]", "[8{x,y}64, 2048, 1024{z}4096]"),
                  ("[8{x,y}64, 2048, 1024{z}4096]", "[64, 2048, 4096]")],
    },
    "c5_bf16_attn_8x8": {
        "dtype": "bf16", "elem_size": 2, "gshape": (16, 32, 2048, 128), "mesh": {"p": 8, "q": 8},
        "pairs": None,   # 50 sampled pairs: sample_pairs("c5_bf16_attn_8x8")
    },
}

_NP_DTYPE = {"int32": np.int32, "fp32": np.float32, "bf16": np.uint16}
_ORDER = list(WORKLOADS)


def np_dtype(tag):
    return _NP_DTYPE[tag]


def type_text(gshape, mesh, axes_per_dim):
    """Write a distributed type as text from the axes tiling each dimension."""
    parts = []
    for n, axes in zip(gshape, axes_per_dim):
        if not axes:
            parts.append(str(n))
        else:
            k = prod(mesh[a] for a in axes)
            if n % k:
                raise ValueError("tiling does not divide the dimension")
            parts.append("%d{%s}%d" % (n // k, ",".join(axes), n))
    return "[" + ", ".join(parts) + "]"


def sample_pairs(name, count=50, seed=None):
    """Random (src, dst) type pairs: every mesh axis is either replicated or tiles
    one dimension; a draw whose tiling does not divide the dimension is rejected;
    two axes on one dimension get a coin-flipped order; src != dst."""
    w = WORKLOADS[name]
    gshape, mesh = w["gshape"], w["mesh"]
    rng = random.Random(BASE_SEED + 50 if seed is None else seed)

    def one():
        while True:
            per_dim = [[] for _ in gshape]
            for ax in mesh:
                pick = rng.randrange(-1, len(gshape))
                if pick >= 0:
                    per_dim[pick].append(ax)
            for lst in per_dim:
                if len(lst) > 1:
                    rng.shuffle(lst)
            try:
                return type_text(gshape, mesh, per_dim)
            except ValueError:
                continue

    pairs = []
    while len(pairs) < count:
        a, b = one(), one()
        if a != b:
            pairs.append((a, b))
    return pairs


# ---- the paper's own evaluation shape (Sec. 8): 3 mesh axes, arrays of up to 6 dimensions, global sizes
# 64 MB - 800 MB, every axis either replicated or partitioning one dimension.  The paper's 1000 sampled
# problems are not published; these are drawn the same way from a fixed seed.
PAPER_MESH = {"a": 2, "b": 2, "c": 2}
PAPER_ELEM_SIZE = 4
_PAPER_DIMS = [4, 8, 16, 24, 32, 36, 40, 48, 64, 72, 74, 80, 90, 96, 128, 156, 160, 180, 184, 256, 296, 312, 320, 360,
               368, 512, 1024, 2048]


# The four problems the paper prints in its Table "adversarial" (Sec. 8; 2x2x2 mesh, 4-byte elements,
# 162 / 113 / 127 / 64 MB), as (name, source type, target type).
ADVERSARIAL_PROBLEMS = [
    ("P1", "[360, 184{c}368, 320]", "[90{c,a}360, 368, 160{b}320]"),
    ("P2", "[80, 40{c}80, 72, 64]", "[40{b}80, 80, 36{c}72, 64]"),
    ("P3", "[296, 360, 156{c}312]", "[74{b,c}296, 180{a}360, 312]"),
    ("P4", "[8{c}16, 16, 16, 8{a}16, 16, 8{b}16]", "[16, 16, 16, 16, 16, 8{a}16]"),
]


def sample_paper_problems(count=1000, seed=None, min_mb=64, max_mb=800):
    """[(global shape, src type, dst type)]: rank 2..6, 4-byte elements, global size within [min_mb, max_mb] MiB."""
    rng = random.Random(BASE_SEED + 1000 if seed is None else seed)
    mesh = PAPER_MESH
    out = []
    while len(out) < count:
        rank = rng.randint(2, 6)
        gshape = tuple(rng.choice(_PAPER_DIMS) for _ in range(rank))
        mb = prod(gshape) * PAPER_ELEM_SIZE / 2 ** 20
        if not (min_mb <= mb <= max_mb):
            continue

        def one():
            for _ in range(100):
                per_dim = [[] for _ in gshape]
                for ax in mesh:
                    pick = rng.randrange(-1, rank)
                    if pick >= 0:
                        per_dim[pick].append(ax)
                for lst in per_dim:
                    rng.shuffle(lst)
                try:
                    return type_text(gshape, mesh, per_dim)
                except ValueError:
                    continue
            return None

        a, b = one(), one()
        if a is None or b is None or a == b:
            continue
        out.append((gshape, a, b))
    return out


def pairs_of(name):
    w = WORKLOADS[name]
    return w["pairs"] if w["pairs"] is not None else sample_pairs(name)


def global_array(name, pattern="seeded", gshape=None):
    """The global array of a workload.  pattern: "seeded" (the workload's value
    distribution) or "iota" (element = its global linear index, wrapped to the
    element width) which makes any misplaced element visible."""
    w = WORKLOADS[name]
    gshape = tuple(gshape or w["gshape"])
    dt = np_dtype(w["dtype"])
    n = prod(gshape)
    if pattern == "iota":
        return (np.arange(n, dtype=np.uint64) & np.uint64((1 << (8 * w["elem_size"])) - 1)).astype(
            {2: np.uint16, 4: np.uint32}[w["elem_size"]]).view(dt).reshape(gshape)
    rng = np.random.default_rng(BASE_SEED + _ORDER.index(name) + 1)
    if w["dtype"] == "int32":
        return rng.integers(np.iinfo(np.int32).min, np.iinfo(np.int32).max, size=gshape, dtype=np.int32, endpoint=True)
    if w["dtype"] == "fp32":
        return rng.uniform(-1.0, 1.0, size=gshape).astype(np.float32)
    # bf16 N(0,1): draw fp32 in blocks, keep the upper 16 bits (round to nearest even)
    out = np.empty(n, dtype=np.uint16)
    step = 1 << 24
    for lo in range(0, n, step):
        f = rng.standard_normal(min(step, n - lo), dtype=np.float32).view(np.uint32)
        f = f + np.uint32(0x7FFF) + ((f >> np.uint32(16)) & np.uint32(1))
        out[lo:lo + f.size] = (f >> np.uint32(16)).astype(np.uint16)
    return out.reshape(gshape)


def random_bytes_array(gshape, elem_size, seed):
    """Opaque elements of any width (1, 2, 4, 8 or 16 bytes) as a uint8 array with a
    trailing axis of length elem_size."""
    rng = np.random.default_rng(seed)
    return rng.integers(0, 256, size=tuple(gshape) + (elem_size,), dtype=np.uint8)
