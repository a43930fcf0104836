"""Seeded synthetic inputs for the Cerberus verify step.

This module only *draws inputs*: model shapes, random-init weights, static candidate
trees, KV prefixes, candidate tables and gate states.  It holds none of the method's
arithmetic (no norms, attention, heads, entropy, acceptance); the CPU oracle and the
HIP library each implement those on their own and are both fed from here, so a value
produced here reaches both sides unchanged.

Shapes follow the LLaMA family the paper evaluates on (Section 5.1, "Models") and the
head layout of Section 5.1, "Training": 4 decoding heads, each four Resblocks and one
fully connected layer.  The trained weights, the evaluation set and the hand-picked
tree-path lists of the paper are not available; everything here is random-init and
seeded, and stands in for them.
"""
from __future__ import annotations

import itertools
from typing import Dict, List, Sequence, Tuple

import torch

# --------------------------------------------------------------------------------------
# model shapes
# --------------------------------------------------------------------------------------

_BASE = dict(n_resblocks=4, special_block=1, rms_eps=1e-6, rope_theta=10000.0,
             entropy_threshold=float("inf"))

CONFIGS: Dict[str, dict] = {
    # parity-sized decoder
    "tiny": dict(_BASE, n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ffn=688,
                 vocab=1024, n_cerb_heads=4, topk=4),
    # LLaMA-7B shape (Vicuna-7B is a fine-tune of it; Section 5.1 "Models")
    "7b": dict(_BASE, n_layers=32, d_model=4096, n_heads=32, head_dim=128, d_ffn=11008,
               vocab=32000, n_cerb_heads=4, topk=6),
    # LLaMA-13B shape, five decoding heads
    "13b": dict(_BASE, n_layers=40, d_model=5120, n_heads=40, head_dim=128, d_ffn=13824,
                vocab=32000, n_cerb_heads=5, topk=6),
}


def make_config(name: str, **overrides) -> dict:
    cfg = dict(CONFIGS[name])
    cfg.update(overrides)
    return cfg


def head_block_widths(cfg: dict) -> List[List[int]]:
    """Width (= rows = columns of W) of every Resblock of every decoding head.

    Head 0 has no predecessor and stays at the model width.  For head i >= 1 the block
    at index `special_block` takes the concatenation of two width-d vectors, so it and
    every later block of that head are 2d wide (Section 4.1, the special Resblock adds
    the concatenated input back as the residual).  special_block < 0 switches the link
    off: every block of every head is d wide (independent heads, Section 4.1 first
    paragraphs).
    """
    d, sb = cfg["d_model"], cfg["special_block"]
    out = []
    for i in range(cfg["n_cerb_heads"]):
        row = []
        for s in range(cfg["n_resblocks"]):
            wide = (i >= 1 and sb >= 0 and s >= sb)
            row.append(2 * d if wide else d)
        out.append(row)
    return out


def head_fc_width(cfg: dict, i: int) -> int:
    return head_block_widths(cfg)[i][-1]


# --------------------------------------------------------------------------------------
# random tensors
# --------------------------------------------------------------------------------------

def _gen(seed: int, tensor_id: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1_000_003 + int(tensor_id) * 7919 + 12345) % (2 ** 63 - 1))
    return g


def _normal(shape, std, mean, seed, tensor_id, device, dtype) -> torch.Tensor:
    g = _gen(seed, tensor_id, device)
    t = torch.empty(shape, dtype=torch.float32, device=device)
    t.normal_(0.0, 1.0, generator=g)
    t.mul_(std).add_(mean)
    return t.to(dtype).contiguous()


def make_weights(cfg: dict, seed: int = 0, dtype=torch.float32, device="cpu",
                 std: float = 0.02) -> dict:
    """Random-init base model and decoding heads, stored in `dtype`.

    Matrices are [out, in] row-major and drawn N(0, std); norm gains 1 + N(0, std);
    Resblock biases N(0, std).  Values are rounded to `dtype` here, once, so both
    consumers see the same representable numbers.
      wqkv      [3d, d]   rows 0..d-1 = Q, d..2d-1 = K, 2d..3d-1 = V
      w_gate_up [2F, d]   rows 0..F-1 = gate, F..2F-1 = up
    """
    d, F, V = cfg["d_model"], cfg["d_ffn"], cfg["vocab"]
    tid = itertools.count()

    def mat(o, i):
        return _normal((o, i), std, 0.0, seed, next(tid), device, dtype)

    def gain(n):
        return _normal((n,), std, 1.0, seed, next(tid), device, dtype)

    def bias(n):
        return _normal((n,), std, 0.0, seed, next(tid), device, dtype)

    W = {"embed": mat(V, d), "final_norm": gain(d), "lm_head": mat(V, d), "layers": []}
    for _ in range(cfg["n_layers"]):
        W["layers"].append({
            "attn_norm": gain(d), "wqkv": mat(3 * d, d), "wo": mat(d, d),
            "ffn_norm": gain(d), "w_gate_up": mat(2 * F, d), "w_down": mat(d, F),
        })
    widths = head_block_widths(cfg)
    W["heads"] = []
    for i in range(cfg["n_cerb_heads"]):
        blocks = [{"w": mat(w, w), "b": bias(w)} for w in widths[i]]
        W["heads"].append({"blocks": blocks, "fc": mat(V, widths[i][-1])})
    return W


def make_heads(cfg: dict, seed: int, dtype=torch.float32, device="cpu", std: float = 0.02) -> list:
    """Decoding heads alone (same recipe as in make_weights, tensor ids of their own), for a second
    head layout over a base model that is already there."""
    tid = itertools.count(1 << 20)
    widths = head_block_widths(cfg)
    heads = []
    for i in range(cfg["n_cerb_heads"]):
        blocks = [{"w": _normal((w, w), std, 0.0, seed, next(tid), device, dtype),
                   "b": _normal((w,), std, 0.0, seed, next(tid), device, dtype)} for w in widths[i]]
        heads.append({"blocks": blocks, "fc": _normal((cfg["vocab"], widths[i][-1]), std, 0.0, seed, next(tid), device, dtype)})
    return heads


def make_kv_prefix(cfg: dict, batch: int, capacity: int, seed: int, dtype, device) -> torch.Tensor:
    """Synthetic N(0,1) KV slab [n_layers][2][batch][n_heads][capacity][head_dim]."""
    shape = (cfg["n_layers"], 2, batch, cfg["n_heads"], capacity, cfg["head_dim"])
    return _normal(shape, 1.0, 0.0, seed, 900_001, device, dtype)


def make_token_ids(n: int, vocab: int, seed: int, tensor_id: int = 0) -> torch.Tensor:
    g = _gen(seed, 800_000 + tensor_id, "cpu")
    return torch.randint(0, vocab, (n,), generator=g, dtype=torch.int64).to(torch.int32)


def make_candidates(cfg: dict, batch: int, seed: int) -> torch.Tensor:
    """[batch][Hc][topk] distinct random ids per (sequence, head)."""
    Hc, K, V = cfg["n_cerb_heads"], cfg["topk"], cfg["vocab"]
    g = _gen(seed, 700_001, "cpu")
    out = torch.empty((batch, Hc, K), dtype=torch.int32)
    for b in range(batch):
        for i in range(Hc):
            out[b, i] = torch.randperm(V, generator=g)[:K].to(torch.int32)
    return out


def make_gate_states(n: int, d: int, seed: int, lo: float = 0.5, hi: float = 4.0) -> torch.Tensor:
    """n hidden-state stand-ins h_s = alpha_s * z_s, z ~ N(0,1)^d, alpha ~ U(lo, hi).

    Random-init hidden states all have nearly the same entropy, so the scale alpha is
    drawn to spread the entropies on both sides of a threshold.
    """
    g = _gen(seed, 600_001, "cpu")
    z = torch.empty((n, d), dtype=torch.float32).normal_(0.0, 1.0, generator=g)
    a = torch.empty((n, 1), dtype=torch.float32).uniform_(lo, hi, generator=g)
    return (a * z).contiguous()


# --------------------------------------------------------------------------------------
# static candidate trees (Section 5.1, "Tree Settings": a hand-picked subset of the
# k + k^2 + ... rank-prefix paths; the paper does not list its subsets)
# --------------------------------------------------------------------------------------

Path = Tuple[int, ...]

TINY_TREE_PATHS: Tuple[Path, ...] = (
    (), (0,), (1,), (2,), (3,), (0, 0), (0, 1), (1, 0), (1, 1), (2, 0), (2, 1), (3, 0),
    (0, 0, 0), (0, 1, 0), (1, 0, 0), (0, 0, 0, 0),
)


def count_all_paths(n_heads: int, k: int) -> int:
    """Size of the full solution space k + k^2 + ... + k^n_heads."""
    return sum(k ** i for i in range(1, n_heads + 1))


def select_paths(n_heads: int, n_paths: int, k: int = 10) -> List[Path]:
    """Deterministic stand-in for a hand-picked path list.

    Every rank tuple of depth 1..n_heads with ranks < k gets the integer cost
    sum_i (5 + i + 8 * r_i) (i = 1-based depth of the element); the n_paths cheapest
    are kept (ties: shallower first, then lexicographic).  A prefix or a lower-ranked
    sibling always costs less, so the selection is prefix- and sibling-closed.
    Returned with the root () first, ordered by (depth, tuple).
    """
    scored = []
    for depth in range(1, n_heads + 1):
        for tup in itertools.product(range(k), repeat=depth):
            cost = sum(5 + (i + 1) + 8 * r for i, r in enumerate(tup))
            scored.append((cost, depth, tup))
    scored.sort()
    chosen = [t for _, _, t in scored[:n_paths]]
    chosen.sort(key=lambda t: (len(t), t))
    return [()] + chosen


def paths_to_tree(paths: Sequence[Path]) -> Tuple[List[int], List[int]]:
    """Rank tuples -> (parent[], rank[]) with node 0 = root, parent[n] < n."""
    index = {p: n for n, p in enumerate(paths)}
    parent, rank = [], []
    for p in paths:
        if len(p) == 0:
            parent.append(-1)
            rank.append(0)
        else:
            parent.append(index[p[:-1]])
            rank.append(p[-1])
    return parent, rank


def make_tree(name: str, n_heads: int = 4) -> Tuple[List[int], List[int]]:
    """'tiny' = the fixed 16-node tree; 'p63' = 63 generated paths + root = 64 nodes;
    'chain<k>' = a single path of k nodes below the root (rank 0 everywhere); 'bfs<k>x<n>' = the
    first n nodes of the k-ary tree in breadth-first order; 'rand<n>s<seed>k<k>' = a seeded random
    tree of n nodes with at most k children per node (children take ranks 0, 1, ... in order)."""
    if name == "tiny":
        return paths_to_tree(TINY_TREE_PATHS)
    if name == "root":
        return [-1], [0]
    if name.startswith("chain"):
        k = int(name[5:])
        return paths_to_tree([tuple([0] * i) for i in range(k + 1)])
    if name.startswith("rand"):                     # 'rand<n>s<seed>k<k>': n nodes, random shape, at most k children per node
        n, rest = name[4:].split("s")
        seed, k = rest.split("k")
        n, seed, k = int(n), int(seed), int(k)
        g = _gen(seed, 600_001, "cpu")
        paths: List[Path] = [()]
        while len(paths) < n:
            p = paths[int(torch.randint(0, len(paths), (1,), generator=g))]
            kids = sum(1 for q in paths if len(q) == len(p) + 1 and q[:-1] == p)
            if len(p) < n_heads and kids < k:
                paths.append(p + (kids,))
        paths.sort(key=lambda t: (len(t), t))
        return paths_to_tree(paths)
    if name.startswith("bfs"):                      # 'bfs<k>x<n>': the first n nodes of the k-ary tree in breadth-first order
        k, n = (int(v) for v in name[3:].split("x"))
        paths, level = [()], [()]
        while len(paths) < n:
            level = [p + (r,) for p in level for r in range(k)]
            paths += level
        return paths_to_tree(paths[:n])
    if name.startswith("p"):
        return paths_to_tree(select_paths(n_heads, int(name[1:])))
    raise KeyError(name)


# --------------------------------------------------------------------------------------
# host views of the same tensors (for CPU consumers)
# --------------------------------------------------------------------------------------

def to_host_f32(obj):
    """Recursively turn tensors into float32 numpy arrays holding the same values."""
    if isinstance(obj, torch.Tensor):
        if obj.is_floating_point():
            return obj.detach().to("cpu", torch.float32).numpy()
        return obj.detach().cpu().numpy()
    if isinstance(obj, dict):
        return {k: to_host_f32(v) for k, v in obj.items()}
    if isinstance(obj, (list, tuple)):
        return [to_host_f32(v) for v in obj]
    return obj


class LazyHostLayers:
    """Sequence view over W["layers"] that converts one layer to host float32 on access,
    so a 7B-shaped model never has to sit in host memory as a whole."""

    def __init__(self, layers, on_access=None):
        self._layers = layers
        self._on_access = on_access

    def __len__(self):
        return len(self._layers)

    def __getitem__(self, l):
        if self._on_access is not None:
            self._on_access(l)
        return to_host_f32(self._layers[l])


def to_host_lazy(W: dict, on_access=None) -> dict:
    out = {k: to_host_f32(v) for k, v in W.items() if k != "layers"}
    out["layers"] = LazyHostLayers(W["layers"], on_access)
    return out
