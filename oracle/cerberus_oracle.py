"""CPU oracle for one Cerberus decoding step.  TEST INFRASTRUCTURE ONLY.

A plain, slow, float64 numpy implementation of what the per-step tree-verification
decode pass computes, written from the paper (Cerberus: Algorithm 1, Section 4.1 for the
decoding heads, Section 4.2 for the entropy gate, Section 5.1 "Tree Settings" for the
candidate tree).  It exists so that the HIP library can be compared against it.  It shares
no code with the HIP path and must never be imported by it: only tests, the smoke check
and the benchmark's CPU-baseline leg may call anything in this file.

Arithmetic is float64 throughout (the paper fixes no precision); weights arrive as
float32 arrays holding exactly the values the GPU stores (bf16- or fp32-representable)
and are widened on use.  Matrix products use numpy's matmul as a library step; there is
no blocking, fusion or reordering beyond what the step definitions state.

Where the paper is silent the following readings are taken (each listed in the design
notes of the repository):
  * decoder layer internals: LLaMA family (Section 5.1 "Models"): pre-norm RMSNorm,
    multi-head attention with rotary embedding (half-split pairing), SwiGLU FFN, no
    biases, untied LM head.                                         [parity unpinned:
    eps, RoPE pairing and pre/post-norm choice of h_last come from this reading]
  * h_last of Algorithm 1 is the output of the final RMSNorm, the vector the LM head
    multiplies; the same vector feeds the gate and the decoding heads.
  * tree attention (named in Sections 1 and 5.1, not defined): node n sees the whole
    committed prefix and its ancestors-or-self in the tree; its position is
    prefix_length + depth(n).
  * acceptance (Section 3.1 speaks of "the final tokens to be accepted", gives no rule):
    greedy exact match, longest prefix from the root.
  * Cerberus heads (Section 4.1; the figure is not available): one special Resblock per
    head i >= 1 at index `special_block`, fed Concat(own state, state of head i-1), both
    taken before that stage; output width 2d because the printed residual adds the
    concatenation back.  Numeric values of this wiring: parity unpinned (reading).
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence

import numpy as np

F64 = np.float64


def _f(a) -> np.ndarray:
    return np.asarray(a, dtype=F64)


# --------------------------------------------------------------------------------------
# static tree (Section 5.1 "Tree Settings")
# --------------------------------------------------------------------------------------

def tree_tables(parent: Sequence[int]):
    """depth[n] and anc[n, m] = (m is n or an ancestor of n).  Node 0 is the root."""
    T = len(parent)
    depth = np.zeros(T, dtype=np.int64)
    anc = np.zeros((T, T), dtype=bool)
    assert parent[0] == -1
    for n in range(T):
        p = parent[n]
        if n > 0:
            assert 0 <= p < n, "nodes must be listed parents-first"
            depth[n] = depth[p] + 1
            anc[n] = anc[p]
        anc[n, n] = True
    return depth, anc


def tree_tokens(root: int, cand: np.ndarray, parent: Sequence[int], rank: Sequence[int]) -> np.ndarray:
    """Token carried by every node: the root carries the pending LM-head token, a node at
    depth delta >= 1 carries candidate `rank[n]` of decoding head delta-1 (Algorithm 1,
    the Candidates tuple: LM head first, then head 0, 1, ...)."""
    depth, _ = tree_tables(parent)
    tok = np.zeros(len(parent), dtype=np.int64)
    tok[0] = int(root)
    for n in range(1, len(parent)):
        tok[n] = int(cand[depth[n] - 1][rank[n]])
    return tok


# --------------------------------------------------------------------------------------
# decoder building blocks (LLaMA family; Algorithm 1 lines 1-5)
# --------------------------------------------------------------------------------------

def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    x = _f(x)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x * _f(gain) / np.sqrt(ms + eps)


def rope(x: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotary embedding on x[rows, heads, dh]: pair (j, j + dh/2) is rotated by the angle
    pos * theta^(-2j/dh)."""
    x = _f(x)
    dh = x.shape[-1]
    half = dh // 2
    j = np.arange(half, dtype=F64)
    ang = _f(pos)[:, None] * np.power(F64(theta), -2.0 * j / dh)[None, :]   # [rows, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, a * s + b * c], axis=-1)


def silu(z: np.ndarray) -> np.ndarray:
    z = _f(z)
    return z / (1.0 + np.exp(-z))


def new_kv(cfg: dict, capacity: int) -> list:
    shape = (cfg["n_heads"], capacity, cfg["head_dim"])
    return [(np.zeros(shape, F64), np.zeros(shape, F64)) for _ in range(cfg["n_layers"])]


def decoder_rows(cfg: dict, W: dict, tok: np.ndarray, pos: np.ndarray, vis: np.ndarray,
                 kv: list, L: int, probe=None):
    """Run the base decoder over `rows` new tokens against a cache holding L committed rows.

    Row r sees cache rows 0..L-1 and new row m wherever vis[r, m].  K/V of new row r are
    written to cache row L + r.  Returns (h_last[rows, d], logits[rows, V]).

    `probe(name, layer, value) -> value`, if given, is shown every named intermediate and
    may replace it (diagnostics only: recording activations, or emulating a storage
    precision); with probe=None the arithmetic is exactly as written.
    """
    if probe is None:
        probe = lambda name, layer, value: value
    d, nH, dh, F = cfg["d_model"], cfg["n_heads"], cfg["head_dim"], cfg["d_ffn"]
    eps, theta = cfg["rms_eps"], cfg["rope_theta"]
    rows = len(tok)
    vis = np.asarray(vis, dtype=bool)
    allowed = np.concatenate([np.ones((rows, L), dtype=bool), vis], axis=1)   # [rows, L+rows]
    x = _f(W["embed"][np.asarray(tok, dtype=np.int64)])
    layers = W["layers"]
    for l in range(cfg["n_layers"]):
        lw = layers[l]
        m = probe("attn_in", l, rmsnorm(x, lw["attn_norm"], eps))
        qkv = m @ _f(lw["wqkv"]).T
        q = probe("q", l, rope(qkv[:, :d].reshape(rows, nH, dh), pos, theta))
        k = probe("k", l, rope(qkv[:, d:2 * d].reshape(rows, nH, dh), pos, theta))
        v = probe("v", l, qkv[:, 2 * d:].reshape(rows, nH, dh))
        K, V = kv[l]
        K[:, L:L + rows, :] = np.transpose(k, (1, 0, 2))
        V[:, L:L + rows, :] = np.transpose(v, (1, 0, 2))
        o = np.zeros((rows, nH, dh), F64)
        for h in range(nH):
            s = (q[:, h, :] @ K[h, :L + rows, :].T) / math.sqrt(dh)
            s = np.where(allowed, s, -np.inf)
            s = s - np.max(s, axis=1, keepdims=True)
            e = np.exp(s)
            p = probe("p", l, e / np.sum(e, axis=1, keepdims=True))
            o[:, h, :] = p @ V[h, :L + rows, :]
        o = probe("attn_out", l, o)
        x = x + o.reshape(rows, d) @ _f(lw["wo"]).T
        m2 = probe("ffn_in", l, rmsnorm(x, lw["ffn_norm"], eps))
        gu = m2 @ _f(lw["w_gate_up"]).T
        act = probe("ffn_act", l, silu(gu[:, :F]) * gu[:, F:])
        x = probe("x", l, x + act @ _f(lw["w_down"]).T)
    h_last = probe("h_last", -1, rmsnorm(x, W["final_norm"], eps))
    logits = h_last @ _f(W["lm_head"]).T
    return h_last, logits


def argmax_lowest(v: np.ndarray) -> np.ndarray:
    """Index of the maximum along the last axis; the lowest index wins a tie."""
    return np.argmax(_f(v), axis=-1)


# --------------------------------------------------------------------------------------
# acceptance and cache compaction (tree verification, Algorithm 1 line 13)
# --------------------------------------------------------------------------------------

def accept_path(g: Sequence[int], tok: Sequence[int], parent: Sequence[int]) -> List[int]:
    """Walk down from the root: at node `cur` the base model's own next token is g[cur];
    descend into the lowest-numbered child that carries exactly that token, stop when no
    child does.  The root is always accepted."""
    T = len(parent)
    path = [0]
    cur = 0
    while True:
        nxt = -1
        for c in range(cur + 1, T):
            if parent[c] == cur and int(tok[c]) == int(g[cur]):
                nxt = c
                break
        if nxt < 0:
            return path
        path.append(nxt)
        cur = nxt


def compact_kv(kv: list, L: int, path: Sequence[int]) -> None:
    """Move the accepted nodes' K/V rows so that they follow the prefix contiguously:
    row L + path[j] -> row L + j, j ascending.  Rows past L + len(path) are don't-care."""
    for K, V in kv:
        for j in range(1, len(path)):
            K[:, L + j, :] = K[:, L + path[j], :]
            V[:, L + j, :] = V[:, L + path[j], :]


# --------------------------------------------------------------------------------------
# entropy gate (Section 4.2; Algorithm 1 lines 6-8)
# --------------------------------------------------------------------------------------

def entropy_bits(h: np.ndarray) -> float:
    """S = -sum_i P_i log2 P_i with P = softmax(h) over the components of one hidden
    vector; terms with P_i = 0 contribute 0."""
    h = _f(h)
    z = h - np.max(h)
    e = np.exp(z)
    P = e / np.sum(e)
    if np.any(np.isnan(P)):
        return float("nan")
    nz = P > 0
    return float(-np.sum(P[nz] * np.log2(P[nz])))


def gate(h: np.ndarray, threshold: float):
    """Returns (S, flag); flag 1 = auto-regressive step, chosen when S > threshold.
    Equality keeps the parallel path; a NaN entropy takes the auto-regressive one."""
    S = entropy_bits(h)
    flag = 0 if S <= threshold else 1
    return S, flag


# --------------------------------------------------------------------------------------
# decoding heads (Section 4.1)
# --------------------------------------------------------------------------------------

def resblock(Wm: np.ndarray, b: np.ndarray, x: np.ndarray) -> np.ndarray:
    """Output = SiLU((W x + b) + x), as printed in Section 4.1."""
    x = _f(x)
    return silu((_f(Wm) @ x + _f(b)) + x)


def cerberus_heads(cfg: dict, heads: list, h: np.ndarray) -> List[np.ndarray]:
    """Vocabulary logits of every decoding head for one hidden vector h.

    All heads advance one Resblock per stage, together.  At stage `special_block` head
    i >= 1 feeds its block Concat(state_i, state_{i-1}), both states as they stood before
    this stage, so no head ever waits for another head's later blocks.  special_block < 0:
    independent heads (no link).
    """
    Hc, R, sb = cfg["n_cerb_heads"], cfg["n_resblocks"], cfg["special_block"]
    state = [_f(h) for _ in range(Hc)]
    for s in range(R):
        before = state
        after = []
        for i in range(Hc):
            blk = heads[i]["blocks"][s]
            if s == sb and i >= 1:
                inp = np.concatenate([before[i], before[i - 1]])
            else:
                inp = before[i]
            after.append(resblock(blk["w"], blk["b"], inp))
        state = after
    return [_f(heads[i]["fc"]) @ state[i] for i in range(Hc)]


def topk_ids(v: np.ndarray, k: int) -> np.ndarray:
    """Ids of the k largest entries, largest first; equal values: lower id first."""
    v = _f(v)
    order = np.lexsort((np.arange(v.shape[0]), -v))
    return order[:k].astype(np.int64)


# --------------------------------------------------------------------------------------
# the step (Algorithm 1 in streaming form)
# --------------------------------------------------------------------------------------

def new_state(kv: list, L: int, root: int, cand: np.ndarray, flag: int) -> dict:
    return {"kv": kv, "L": int(L), "root": int(root), "cand": np.array(cand, dtype=np.int64),
            "flag": int(flag)}


def verify_step(cfg: dict, W: dict, parent: Sequence[int], rank: Sequence[int], st: dict,
                force_ar: bool = False, forced_node_argmax: Optional[np.ndarray] = None,
                forced_gate_hidden: Optional[np.ndarray] = None, probe=None) -> dict:
    """One decoding step for one sequence; updates `st` in place and returns everything
    the step computed.

    The gate and the heads run at the end of a forward pass, on the hidden state of the
    last accepted node, and choose the shape of the next pass: that is Algorithm 1 with
    Tree_Verify recognised as the next base-model forward.  st["flag"] = 1 (or force_ar)
    makes this pass a plain one-token step (tree of size 1).
    """
    if st["flag"] or force_ar:
        parent_s, rank_s = [-1], [0]
    else:
        parent_s, rank_s = list(parent), list(rank)
    T = len(parent_s)
    depth, anc = tree_tables(parent_s)
    L = st["L"]
    tok = tree_tokens(st["root"], st["cand"], parent_s, rank_s)
    pos = L + depth
    h_last, logits = decoder_rows(cfg, W, tok, pos, anc, st["kv"], L, probe)
    g = argmax_lowest(logits)
    if forced_node_argmax is not None:
        g = np.asarray(forced_node_argmax, dtype=np.int64)[:T]
    path = accept_path(g, tok, parent_s)
    a = len(path)
    committed = tok[path]
    new_root = int(g[path[-1]])
    compact_kv(st["kv"], L, path)
    h = h_last[path[-1]]
    gate_in = h if forced_gate_hidden is None else _f(forced_gate_hidden)
    S, flag = gate(gate_in, cfg["entropy_threshold"])
    head_logits = None
    cand = st["cand"]
    if flag == 0:
        head_logits = cerberus_heads(cfg, W["heads"], h)
        cand = np.stack([topk_ids(hl, cfg["topk"]) for hl in head_logits])
    st.update(L=L + a, root=new_root, cand=cand, flag=flag)
    return {"T": T, "tok": tok, "pos": pos, "h_last": h_last, "logits": logits, "g": g,
            "path": path, "accept_len": a, "committed": committed, "root": new_root,
            "entropy": S, "flag": flag, "head_logits": head_logits, "cand": cand,
            "L_before": L, "L_after": L + a}


def prefill(cfg: dict, W: dict, tokens: Sequence[int], capacity: int) -> dict:
    """Causal forward of a whole prompt from an empty cache, then the gate and the heads
    on its last position: the state a first decoding step starts from."""
    n = len(tokens)
    kv = new_kv(cfg, capacity)
    vis = np.tril(np.ones((n, n), dtype=bool))
    h_last, logits = decoder_rows(cfg, W, np.asarray(tokens), np.arange(n), vis, kv, 0)
    root = int(argmax_lowest(logits[-1]))
    S, flag = gate(h_last[-1], cfg["entropy_threshold"])
    K = cfg["topk"]
    cand = np.zeros((cfg["n_cerb_heads"], K), dtype=np.int64)
    if flag == 0:
        cand = np.stack([topk_ids(hl, K) for hl in cerberus_heads(cfg, W["heads"], h_last[-1])])
    return new_state(kv, n, root, cand, flag)


def greedy_decode(cfg: dict, W: dict, kv: list, L: int, root: int, n_tokens: int) -> List[int]:
    """Plain auto-regressive greedy decoding: feed the pending token, take the argmax,
    repeat.  Returns the n_tokens tokens fed (i.e. committed), starting with `root`."""
    out = []
    t = int(root)
    for _ in range(n_tokens):
        out.append(t)
        _, logits = decoder_rows(cfg, W, np.array([t]), np.array([L]), np.ones((1, 1), bool), kv, L)
        L += 1
        t = int(argmax_lowest(logits[0]))
    return out
