"""Are the oracle's pins sharp?  Every entry below plants one plausible mistake in a copy of the
oracle's source (a dropped term, a wrong sign or index, a swapped operand, an off-by-one), on the
CPU, and the pins of test_oracle_pins.py are run against the copy: at least one of them has to fail.
A mistake that no pin notices would mean the oracle could carry it unseen.

The mistakes are text edits, so each also checks that the text it replaces is still there exactly
once: an edit of the oracle that removes it fails here until the entry is brought up to date.
"""
import inspect
import types

import pytest

from oracle import cerberus_oracle as orc
from tests import test_oracle_pins as pins

# (name, text in the oracle, replacement)
MUTANTS = [
    ("rmsnorm: eps outside the root", "np.sqrt(ms + eps)", "(np.sqrt(ms) + eps)"),
    ("rmsnorm: sum instead of mean", "ms = np.mean(x * x, axis=-1, keepdims=True)", "ms = np.sum(x * x, axis=-1, keepdims=True)"),
    ("rmsnorm: gain dropped", "return x * _f(gain) / np.sqrt(ms + eps)", "return x / np.sqrt(ms + eps)"),
    ("rope: rotation sign", "[a * c - b * s, a * s + b * c]", "[a * c + b * s, b * c - a * s]"),
    ("rope: frequency exponent", "-2.0 * j / dh", "-1.0 * j / dh"),
    ("rope: pairs (2j, 2j+1) instead of (j, j+dh/2)", "a, b = x[..., :half], x[..., half:]", "a, b = x[..., 0::2], x[..., 1::2]"),
    ("silu: sign of the exponent", "return z / (1.0 + np.exp(-z))", "return z / (1.0 + np.exp(z))"),
    ("attention: 1/sqrt(dh) dropped", "/ math.sqrt(dh)\n", "\n"),
    ("attention: mask dropped", "s = np.where(allowed, s, -np.inf)", "s = s + 0.0"),
    ("attention: prefix rows hidden from the tree rows", "np.ones((rows, L), dtype=bool), vis]", "np.zeros((rows, L), dtype=bool), vis]"),
    ("attention: V rows written from k", "V[:, L:L + rows, :] = np.transpose(v, (1, 0, 2))", "V[:, L:L + rows, :] = np.transpose(k, (1, 0, 2))"),
    ("attention: K/V rows one row late", "K[:, L:L + rows, :] = np.transpose(k, (1, 0, 2))", "K[:, L + 1:L + rows + 1, :] = np.transpose(k, (1, 0, 2))"),
    ("attention: v gets the rotary embedding", 'v = probe("v", l, qkv[:, 2 * d:].reshape(rows, nH, dh))', 'v = probe("v", l, rope(qkv[:, 2 * d:].reshape(rows, nH, dh), pos, theta))'),
    ("attention: k without the rotary embedding", 'k = probe("k", l, rope(qkv[:, d:2 * d].reshape(rows, nH, dh), pos, theta))', 'k = probe("k", l, qkv[:, d:2 * d].reshape(rows, nH, dh))'),
    ("decoder: attention residual dropped", "x = x + o.reshape(rows, d) @ _f(lw[\"wo\"]).T", "x = o.reshape(rows, d) @ _f(lw[\"wo\"]).T"),
    ("decoder: gate and up swapped", "silu(gu[:, :F]) * gu[:, F:]", "gu[:, :F] * silu(gu[:, F:])"),
    ("decoder: FFN reads the attention norm's gain", 'rmsnorm(x, lw["ffn_norm"], eps)', 'rmsnorm(x, lw["attn_norm"], eps)'),
    ("decoder: final norm dropped", 'rmsnorm(x, W["final_norm"], eps))', 'x)'),
    ("decoder: weight not transposed in the LM head", 'logits = h_last @ _f(W["lm_head"]).T', 'logits = h_last @ _f(W["lm_head"])[:, :h_last.shape[1]].T[:h_last.shape[1]].T @ np.eye(h_last.shape[1], _f(W["lm_head"]).shape[0])'),
    ("tree: ancestors not inherited", "anc[n] = anc[p]", "anc[n, p] = True"),
    ("tree: siblings visible", "anc[n, n] = True", "anc[n, n] = True; anc[n, [m for m in range(n) if n > 0 and parent[m] == parent[n]]] = True"),
    ("tree tokens: head index off by one", "cand[depth[n] - 1][rank[n]]", "cand[min(depth[n], len(cand) - 1)][rank[n]]"),
    ("tree tokens: rank ignored", "cand[depth[n] - 1][rank[n]]", "cand[depth[n] - 1][0]"),
    ("step: positions by row instead of by depth", "pos = L + depth", "pos = L + np.arange(T)"),
    ("accept: highest child wins", "for c in range(cur + 1, T):", "for c in range(T - 1, cur, -1):"),
    ("accept: compares with the child's own argmax", "int(tok[c]) == int(g[cur])", "int(tok[c]) == int(g[c])"),
    ("accept: any node with the token, not only a child", "parent[c] == cur and int(tok[c])", "int(tok[c])"),
    ("accept: stops one level early", "        path.append(nxt)\n        cur = nxt", "        cur = nxt\n        if any(parent[c] == cur for c in range(T)):\n            path.append(nxt)\n        else:\n            return path"),
    ("compaction: destination off by one", "K[:, L + j, :] = K[:, L + path[j], :]", "K[:, L + j - 1, :] = K[:, L + path[j], :]"),
    ("compaction: V left behind", "            V[:, L + j, :] = V[:, L + path[j], :]\n", ""),
    ("compaction: node index used as destination", "K[:, L + j, :] = K[:, L + path[j], :]", "K[:, L + path[j], :] = K[:, L + j, :]"),
    ("entropy: natural logarithm", "np.log2(P[nz])", "np.log(P[nz])"),
    ("entropy: sign", "return float(-np.sum(P[nz] * np.log2(P[nz])))", "return float(np.sum(P[nz] * np.log2(P[nz])))"),
    ("entropy: softmax without normalisation", "P = e / np.sum(e)", "P = e"),
    ("gate: polarity", "flag = 0 if S <= threshold else 1", "flag = 1 if S <= threshold else 0"),
    ("gate: equality goes auto-regressive", "flag = 0 if S <= threshold else 1", "flag = 0 if S < threshold else 1"),
    ("resblock: skip connection dropped", "return silu((_f(Wm) @ x + _f(b)) + x)", "return silu(_f(Wm) @ x + _f(b))"),
    ("resblock: bias dropped", "return silu((_f(Wm) @ x + _f(b)) + x)", "return silu(_f(Wm) @ x + x)"),
    ("resblock: transposed weight", "return silu((_f(Wm) @ x + _f(b)) + x)", "return silu((_f(Wm).T @ x + _f(b)) + x)"),
    ("resblock: activation before the skip", "return silu((_f(Wm) @ x + _f(b)) + x)", "return silu(_f(Wm) @ x + _f(b)) + x"),
    ("heads: concat order", "np.concatenate([before[i], before[i - 1]])", "np.concatenate([before[i - 1], before[i]])"),
    ("heads: link reads the neighbour's new state", "np.concatenate([before[i], before[i - 1]])", "np.concatenate([before[i], after[i - 1]])"),
    ("heads: link from head 0 for everyone", "np.concatenate([before[i], before[i - 1]])", "np.concatenate([before[i], before[0]])"),
    ("heads: link at the wrong block", "if s == sb and i >= 1:", "if s == sb + 1 and i >= 1:"),
    ("heads: vocabulary projection of the neighbour", 'return [_f(heads[i]["fc"]) @ state[i] for i in range(Hc)]', 'return [_f(heads[i]["fc"]) @ state[max(i - 1, 0)] if _f(heads[i]["fc"]).shape[1] == state[max(i - 1, 0)].shape[0] else _f(heads[i]["fc"]) @ state[i] for i in range(Hc)]'),
    ("top-k: ascending", "order = np.lexsort((np.arange(v.shape[0]), -v))", "order = np.lexsort((np.arange(v.shape[0]), v))"),
    ("top-k: ties to the higher id", "order = np.lexsort((np.arange(v.shape[0]), -v))", "order = np.lexsort((-np.arange(v.shape[0]), -v))"),
    ("argmax: ties to the higher id", "return np.argmax(_f(v), axis=-1)", "return _f(v).shape[-1] - 1 - np.argmax(_f(v)[..., ::-1], axis=-1)"),
    ("step: next root from the root's argmax", "new_root = int(g[path[-1]])", "new_root = int(g[path[0]])"),
    ("step: gate and heads on the root's hidden state", "h = h_last[path[-1]]", "h = h_last[0]"),
    ("step: cache not compacted", "    compact_kv(st[\"kv\"], L, path)\n", ""),
    ("step: length advanced by the tree size", "st.update(L=L + a,", "st.update(L=L + T,"),
    ("step: heads run although the gate said auto-regressive", "    if flag == 0:\n        head_logits = cerberus_heads(cfg, W[\"heads\"], h)", "    if True:\n        head_logits = cerberus_heads(cfg, W[\"heads\"], h)"),
    ("step: gate flag ignored when shaping the pass", "if st[\"flag\"] or force_ar:", "if force_ar:"),
    ("decoder: FFN residual dropped", 'x = probe("x", l, x + act @ _f(lw["w_down"]).T)', 'x = probe("x", l, act @ _f(lw["w_down"]).T)'),
    ("attention: visibility transposed", "allowed = np.concatenate([np.ones((rows, L), dtype=bool), vis], axis=1)", "allowed = np.concatenate([np.ones((rows, L), dtype=bool), vis.T | np.eye(rows, dtype=bool)], axis=1)"),
    ("attention: q and k slices swapped", 'q = probe("q", l, rope(qkv[:, :d].reshape(rows, nH, dh), pos, theta))\n        k = probe("k", l, rope(qkv[:, d:2 * d].reshape(rows, nH, dh), pos, theta))', 'k = probe("q", l, rope(qkv[:, :d].reshape(rows, nH, dh), pos, theta))\n        q = probe("k", l, rope(qkv[:, d:2 * d].reshape(rows, nH, dh), pos, theta))'),
    ("attention: heads share head 0's keys", "s = (q[:, h, :] @ K[h, :L + rows, :].T)", "s = (q[:, h, :] @ K[0, :L + rows, :].T)"),
    ("tree tokens: root replaced by the first candidate", "tok[0] = int(root)", "tok[0] = int(cand[0][0])"),
    ("step: commits the argmax instead of the node tokens", "committed = tok[path]", "committed = g[path]"),
    ("step: gate on the logits instead of the hidden state", "gate_in = h if forced_gate_hidden is None", "gate_in = logits[path[-1]] if forced_gate_hidden is None"),
    ("step: argmax of the parent row", "g = argmax_lowest(logits)\n", "g = argmax_lowest(logits)[np.maximum(np.asarray(parent_s), 0)]\n"),
    ("prefill: gate on the first position", 'S, flag = gate(h_last[-1], cfg["entropy_threshold"])', 'S, flag = gate(h_last[0], cfg["entropy_threshold"])'),
    ("prefill: heads on the first position", 'cerberus_heads(cfg, W["heads"], h_last[-1])])', 'cerberus_heads(cfg, W["heads"], h_last[0])])'),
    ("greedy reference: position not advanced", "        L += 1\n", "        L += 0\n"),
    ("rope: positions off by one", "ang = _f(pos)[:, None] *", "ang = (_f(pos)[:, None] + 1.0) *"),
    ("rope: q rotated, k rotated the other way", 'k = probe("k", l, rope(qkv[:, d:2 * d].reshape(rows, nH, dh), pos, theta))', 'k = probe("k", l, rope(qkv[:, d:2 * d].reshape(rows, nH, dh), -np.asarray(pos), theta))'),
    ("attention: softmax over the queries", "s = s - np.max(s, axis=1, keepdims=True)\n            e = np.exp(s)\n            p = probe(\"p\", l, e / np.sum(e, axis=1, keepdims=True))", "s = s - np.max(s)\n            e = np.exp(s)\n            p = probe(\"p\", l, e / np.sum(e, axis=0, keepdims=True))"),
    ("attention: values of head 0 for every head", "o[:, h, :] = p @ V[h, :L + rows, :]", "o[:, h, :] = p @ V[0, :L + rows, :]"),
    ("attention: output heads in reverse order", "x = x + o.reshape(rows, d) @", "x = x + o[:, ::-1, :].reshape(rows, d) @"),
    ("embedding: row of the next token id", 'x = _f(W["embed"][np.asarray(tok, dtype=np.int64)])', 'x = _f(W["embed"][(np.asarray(tok, dtype=np.int64) + 1) % len(W["embed"])])'),
    ("decoder: layers in reverse order", "lw = layers[l]", "lw = layers[cfg[\"n_layers\"] - 1 - l]"),
    ("decoder: K/V of layer 0 for every layer", "K, V = kv[l]", "K, V = kv[0]"),
    ("compaction: K and V swapped", "K[:, L + j, :] = K[:, L + path[j], :]\n            V[:, L + j, :] = V[:, L + path[j], :]", "K[:, L + j, :] = V[:, L + path[j], :]\n            V[:, L + j, :] = K[:, L + path[j], :]"),
    ("compaction: only the first layer", "    for K, V in kv:\n        for j in range(1, len(path)):", "    for K, V in kv[:1]:\n        for j in range(1, len(path)):"),
    ("step: committed tokens exclude the root", "committed = tok[path]", "committed = tok[path[1:]]"),
    ("heads: every head gets head 0's blocks", 'blk = heads[i]["blocks"][s]', 'blk = heads[i if s == sb else 0]["blocks"][s] if len(heads[0]["blocks"][s]["b"]) == len(heads[i]["blocks"][s]["b"]) else heads[i]["blocks"][s]'),
    ("top-k: k+1 entries", "return order[:k].astype(np.int64)", "return order[:k + 1].astype(np.int64)"),
    ("prefill: root from the first position", "root = int(argmax_lowest(logits[-1]))", "root = int(argmax_lowest(logits[0]))"),
    ("prefill: full visibility instead of causal", "vis = np.tril(np.ones((n, n), dtype=bool))", "vis = np.ones((n, n), dtype=bool)"),
]


def _pin_calls():
    """Every pin as a zero-argument callable (parametrised pins once per parameter; the tree-pass
    fixture is computed afresh, against whatever oracle is current)."""
    calls = []
    for name, fn in sorted(vars(pins).items(), key=lambda kv: getattr(kv[1], "__code__", None) and kv[1].__code__.co_firstlineno or 0):
        if not name.startswith("test_") or not callable(fn):
            continue
        params = inspect.signature(fn).parameters
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        if marks:
            (argname, values), = [(m.args[0], m.args[1]) for m in marks]
            for v in values:
                calls.append((f"{name}[{v}]", lambda fn=fn, argname=argname, v=v: fn(**{argname: v})))
        elif "tiny_tree_pass" in params:
            calls.append((name, lambda fn=fn: fn(pins.make_tiny_tree_pass())))
        else:
            assert not params, f"pin {name} takes arguments this runner does not know: {list(params)}"
            calls.append((name, fn))
    return calls


def _first_failing_pin():
    for name, call in _pin_calls():
        try:
            call()
        except Exception as e:      # an assertion, or the mistake made the oracle itself raise
            return name, e
    return None, None


def test_pins_pass_on_the_oracle_as_it_stands():
    name, err = _first_failing_pin()
    assert name is None, f"{name}: {err!r}"


@pytest.mark.parametrize("mutant", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_some_pin(mutant, monkeypatch):
    label, old, new = mutant
    src = inspect.getsource(orc)
    assert src.count(old) == 1, f"'{old}' occurs {src.count(old)} times in the oracle: bring this entry up to date"
    mod = types.ModuleType("cerberus_oracle_mutant")
    mod.__dict__["__name__"] = "cerberus_oracle_mutant"
    exec(compile(src.replace(old, new), "<oracle with: %s>" % label, "exec"), mod.__dict__)
    for k, v in vars(mod).items():
        if callable(v) and getattr(v, "__module__", None) == "cerberus_oracle_mutant" and hasattr(orc, k):
            monkeypatch.setattr(orc, k, v)
    name, err = _first_failing_pin()
    assert name is not None, f"no pin notices: {label}"
