"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

Nothing in this module belongs to the method: it holds tensor-shape lists, the packed
layout, neighbour lists for the topologies the workloads use, and random draws.  The
HIP path and the CPU oracle both receive what is generated here; neither generates
inputs of its own.

Workloads (tensor *shapes* only - no weights, no data sets):

* GPT-2 style decoder (L layers, width w): token embedding 50257 x w, position
  embedding 1024 x w, per layer two layer norms, fused QKV, attention projection, and
  a 4w MLP, a final layer norm, output head tied to the embedding.
* ResNet-50: 7x7 stem, bottleneck stages [3, 4, 6, 3], batch-norm scale and shift after
  every convolution, 1000-way classifier.

Topologies: ring, static exponential graph (hops 2^k), one-peer exponential graph
(one hop per iteration), complete graph, identity, permutation; each returned as the
CSR rows of the mixing matrix with uniform weights 1/|N_i| stored as float32.
"""

from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Sequence, Tuple

import numpy as np

BASE_SEED = 241011998


# --------------------------------------------------------------------------------------
# tensor shape lists
# --------------------------------------------------------------------------------------

def gpt2_shapes(n_layer: int, width: int, vocab: int = 50257, n_pos: int = 1024) -> List[Tuple[str, Tuple[int, ...]]]:
    w = width
    out = [("wte", (vocab, w)), ("wpe", (n_pos, w))]
    for l in range(n_layer):
        p = f"h{l}."
        out += [
            (p + "ln1.g", (w,)), (p + "ln1.b", (w,)),
            (p + "attn.qkv.w", (w, 3 * w)), (p + "attn.qkv.b", (3 * w,)),
            (p + "attn.proj.w", (w, w)), (p + "attn.proj.b", (w,)),
            (p + "ln2.g", (w,)), (p + "ln2.b", (w,)),
            (p + "mlp.fc.w", (w, 4 * w)), (p + "mlp.fc.b", (4 * w,)),
            (p + "mlp.proj.w", (4 * w, w)), (p + "mlp.proj.b", (w,)),
        ]
    out += [("lnf.g", (w,)), ("lnf.b", (w,))]
    return out


def resnet50_shapes(n_class: int = 1000) -> List[Tuple[str, Tuple[int, ...]]]:
    out = [("conv1", (64, 3, 7, 7)), ("bn1.g", (64,)), ("bn1.b", (64,))]
    inplanes = 64
    for si, (planes, blocks) in enumerate(zip((64, 128, 256, 512), (3, 4, 6, 3))):
        for bi in range(blocks):
            p = f"layer{si + 1}.{bi}."
            out += [
                (p + "conv1", (planes, inplanes, 1, 1)), (p + "bn1.g", (planes,)), (p + "bn1.b", (planes,)),
                (p + "conv2", (planes, planes, 3, 3)), (p + "bn2.g", (planes,)), (p + "bn2.b", (planes,)),
                (p + "conv3", (planes * 4, planes, 1, 1)), (p + "bn3.g", (planes * 4,)), (p + "bn3.b", (planes * 4,)),
            ]
            if bi == 0:
                out += [(p + "down.conv", (planes * 4, inplanes, 1, 1)),
                        (p + "down.bn.g", (planes * 4,)), (p + "down.bn.b", (planes * 4,))]
            inplanes = planes * 4
    out += [("fc.w", (n_class, 2048)), ("fc.b", (n_class,))]
    return out


def odd_shapes() -> List[Tuple[str, Tuple[int, ...]]]:
    """Test-only layout with sizes that are not multiples of the vector width."""
    sizes = [1, 3, 17, 1001, 255, 257, 1023, 1025, 4097, 2, 5, 64, 31]
    return [(f"odd{i}", (s,)) for i, s in enumerate(sizes)]


def numel(shape: Sequence[int]) -> int:
    n = 1
    for s in shape:
        n *= int(s)
    return n


@dataclass
class PackedLayout:
    """Tensors laid end to end in definition order; every tensor starts at a multiple
    of ``align_elems`` elements (16 bytes in the narrowest dtype that will use the
    layout).  ``d`` is the packed length including padding."""
    names: List[str]
    offsets: np.ndarray   # uint64 [n_tensors]
    numels: np.ndarray    # uint64 [n_tensors]
    d: int


def pack(shapes: Sequence[Tuple[str, Tuple[int, ...]]], align_elems: int = 8) -> PackedLayout:
    names, offs, nums = [], [], []
    cur = 0
    for name, shp in shapes:
        n = numel(shp)
        names.append(name)
        offs.append(cur)
        nums.append(n)
        cur += -(-n // align_elems) * align_elems
    return PackedLayout(names, np.asarray(offs, dtype=np.uint64), np.asarray(nums, dtype=np.uint64), int(cur))


# --------------------------------------------------------------------------------------
# topologies  ->  (row_ptr int32[R+1], col int32[nnz], w float32[nnz])
# --------------------------------------------------------------------------------------

def _uniform_rows(neigh: Sequence[Sequence[int]]):
    row_ptr = [0]
    col: List[int] = []
    w: List[float] = []
    for nb in neigh:
        col += list(nb)
        w += [np.float32(1.0) / np.float32(len(nb))] * len(nb)
        row_ptr.append(len(col))
    return (np.asarray(row_ptr, dtype=np.int32), np.asarray(col, dtype=np.int32),
            np.asarray(w, dtype=np.float32))


def ring(n: int):
    """Each replica with its two ring neighbours and itself; weights 1/3 (1/2 for n=2,
    1 for n=1)."""
    neigh = []
    for i in range(n):
        nb = [i]
        for j in ((i - 1) % n, (i + 1) % n):
            if j not in nb:
                nb.append(j)
        neigh.append(nb)
    return _uniform_rows(neigh)


def static_exponential(n: int):
    """Replica i listens to itself and to i + 2^k (mod n) for every 2^k < n."""
    neigh = []
    for i in range(n):
        nb = [i]
        h = 1
        while h < n:
            j = (i + h) % n
            if j not in nb:
                nb.append(j)
            h *= 2
        neigh.append(nb)
    return _uniform_rows(neigh)


def one_peer_exponential(n: int, slot: int):
    """Replica i averages with replica i + 2^slot (mod n), weights 1/2 each."""
    hop = (1 << slot) % n
    neigh = [[i, (i + hop) % n] if hop else [i] for i in range(n)]
    return _uniform_rows(neigh)


def one_peer_slots(n: int) -> int:
    """Number of distinct hops 2^k < n."""
    k = 0
    while (1 << k) < n:
        k += 1
    return max(k, 1)


def one_peer_ring(n: int, slot: int):
    """One-peer ring (appendix figure of the same name): two alternating perfect matchings of
    the ring.  Even slots pair (0,1), (2,3), ...; odd slots pair (1,2), (3,4), ..., (n-1,0).
    Weights 1/2."""
    assert n % 2 == 0
    shift = slot % 2
    neigh = [None] * n
    for a in range(shift, n + shift, 2):
        i, j = a % n, (a + 1) % n
        neigh[i] = [i, j]
        neigh[j] = [j, i]
    return _uniform_rows(neigh)


def aer_groups(per_node: int, phase: int):
    """Alternating Exponential Ring for four nodes (appendix figure of that name).  Every drawn
    loop is an All-Reduce (a plain average) over its members.  In each of the four phases one pair
    of nodes forms a common loop and the other two nodes average internally; the pairs are, in
    order, nodes (2,3), (0,1), (0,2), (1,3) - ring hops 1, 1, 2, 2."""
    pair = [(2, 3), (0, 1), (0, 2), (1, 3)][phase % 4]
    node = lambda a: list(range(a * per_node, (a + 1) * per_node))
    groups = [node(pair[0]) + node(pair[1])]
    groups += [node(a) for a in range(4) if a not in pair]
    return groups


def aer(per_node: int, phase: int):
    """Rows of the mixing matrix of one AER phase: uniform weights over the row's loop."""
    n = 4 * per_node
    neigh = [None] * n
    for grp in aer_groups(per_node, phase):
        for i in grp:
            neigh[i] = [i] + [j for j in grp if j != i]
    return _uniform_rows(neigh)


def complete(n: int):
    return _uniform_rows([list(range(n)) for _ in range(n)])


def identity(n: int):
    return _uniform_rows([[i] for i in range(n)])


def permutation(perm: Sequence[int]):
    return _uniform_rows([[int(p)] for p in perm])


def node_share_ring():
    """One node's row of a ring: source buffer 0 is the node's own parameters, buffers
    1 and 2 are the receive buffers of its two neighbours; weights 1/3."""
    return _uniform_rows([[0, 1, 2]])


# --------------------------------------------------------------------------------------
# random draws
# --------------------------------------------------------------------------------------

def seed_for(cfg: int, stream: int) -> int:
    """One seed per (configuration, stream).  Streams: 0 parameters, 1 receive buffers,
    2 + t gradients of iteration t."""
    return BASE_SEED + 1000 * cfg + stream


def normal_np(seed: int, shape, std: float, dtype=np.float32) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(size=shape) * std).astype(dtype)


def normal_torch(seed: int, shape, std: float, device, dtype=None):
    """Normal draws from torch's generator on ``device`` (values differ between
    devices; a run generates once and hands copies to whoever needs them)."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    out = torch.empty(shape, device=device, dtype=torch.float32)
    out.normal_(0.0, std, generator=g)
    return out if dtype is None or dtype == torch.float32 else out.to(dtype)


# --------------------------------------------------------------------------------------
# the five configurations
# --------------------------------------------------------------------------------------

@dataclass
class Workload:
    name: str
    cfg: int
    n_rows: int
    n_cols: int
    shapes: List[Tuple[str, Tuple[int, ...]]]
    param_dtype: str      # "f32" | "bf16"
    grad_dtype: str
    s: int
    steps: int
    grad_std: float
    topology: str         # "ring" | "static_exp" | "one_peer_exp" | "node_share"
    param_std: float = 0.02
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8

    def layout(self) -> PackedLayout:
        return pack(self.shapes)

    def n_slots(self) -> int:
        return one_peer_slots(self.n_rows) if self.topology == "one_peer_exp" else 1

    def csr(self, slot: int = 0):
        if self.topology == "ring":
            return ring(self.n_rows)
        if self.topology == "static_exp":
            return static_exponential(self.n_rows)
        if self.topology == "one_peer_exp":
            return one_peer_exponential(self.n_rows, slot)
        if self.topology == "node_share":
            return node_share_ring()
        raise ValueError(self.topology)

    def slot_of_step(self, t: int) -> int:
        """Iteration t of a time-varying topology uses slot t mod n_slots: configuration 4 pairs replica i
        with i + 2^(t mod 6) at step t.  Any log2(n) consecutive iterations visit every hop once."""
        return t % self.n_slots()

    def bytes_per_replica_param(self) -> float:
        """Algorithmic HBM bytes per updated element, averaged over an accumulation
        loop: every distinct input read once and every output written once.
        x read + x written + g + m_hat + v_hat + b read + b written, receive buffers
        on top, plus 8 bytes of moment write-back on the one fold iteration of a loop,
        minus the 4-byte read of b on the loop's first iteration."""
        px = 2 if self.param_dtype == "bf16" else 4
        pg = 2 if self.grad_dtype == "bf16" else 4
        base = px * (self.n_cols / self.n_rows) + px + pg + 4 + 4 + 4 + 4
        if self.s == 1:           # Algorithm 1: no accumulator, moments written every time
            return px * (self.n_cols / self.n_rows) + px + pg + 8 + 8
        return base + 4.0 / self.s


def scaled(shapes, div: int):
    """The same tensor list with every dimension larger than 8 divided by ``div`` (at
    least 8 kept): small copies of the big layouts for tests the oracle can run whole."""
    out = []
    for name, shp in shapes:
        out.append((name, tuple(max(8, int(x) // div) if x > 8 else int(x) for x in shp)))
    return out


def workload(cfg: int, scale_div: int = 1) -> Workload:
    if cfg == 1:
        wl = Workload("cfg1_ring4_flat1M", 1, 4, 4, [("flat", (1048576,))], "f32", "f32", 2, 10, 1e-2, "ring")
    elif cfg == 2:
        wl = Workload("cfg2_exp16_gpt2small", 2, 16, 16, gpt2_shapes(12, 768), "f32", "f32", 4, 20, 1e-3, "static_exp")
    elif cfg == 3:
        wl = Workload("cfg3_nodeshare_gpt2medium", 3, 1, 3, gpt2_shapes(24, 1024), "f32", "f32", 8, 50, 1e-3, "node_share")
    elif cfg == 4:
        wl = Workload("cfg4_onepeer64_resnet50", 4, 64, 64, resnet50_shapes(), "f32", "f32", 2, 30, 1e-2, "one_peer_exp")
    elif cfg == 5:
        wl = Workload("cfg5_ring8_gpt2large_bf16", 5, 8, 8, gpt2_shapes(36, 1280), "bf16", "bf16", 4, 10, 1e-3, "ring")
    else:
        raise ValueError(f"unknown configuration {cfg}")
    if scale_div > 1:
        wl.shapes = scaled(wl.shapes, scale_div)
        wl.name += f"_div{scale_div}"
    return wl
