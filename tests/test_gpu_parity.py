"""GPU parity tests: the HIP library, called through its C ABI, against the CPU oracle on the
same seeded inputs.  Run with `-m gpu` on an MI355X."""
import copy
import dataclasses
import sys

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import cerberus_oracle as orc
from paper_2410_13344_amd import binding as B
from paper_2410_13344_amd import synth
from tests import harness as H

F32, BF16 = B.CERBERUS_F32, B.CERBERUS_BF16


def say(msg):
    print(msg, flush=True)


@pytest.fixture(scope="module")
def tiny_pairs():
    cache = {}

    def get(dtype, **kw):
        key = (dtype, tuple(sorted(kw.items())))
        if key not in cache:
            cache[key] = H.Pair("tiny", dtype, "tiny", seed=0, max_batch=1, kv_capacity=256, **kw)
        return cache[key]

    return get


def _prefilled(pair, n_prompt=128, seed=1):
    prompt = synth.make_token_ids(n_prompt, pair.cfg["vocab"], seed=seed).numpy()
    return orc.prefill(pair.cfg, pair.W, prompt, capacity=pair.kv_capacity)


def _run_forced_steps(pair, n_steps, cand_mode, attn_mfma, gate_states=None):
    """Teacher-forced steps: before every step the device state is loaded from the oracle's."""
    cfg, dtype = pair.cfg, pair.dtype
    pair.engine.set_param("attn_mfma", attn_mfma)
    taps = pair.taps(forced_gate=gate_states is not None)
    st = pair.engine.new_state()
    ost = _prefilled(pair)
    greedy = None
    if cand_mode in ("planted", "adversarial"):
        ref = _prefilled(pair)
        greedy = orc.greedy_decode(cfg, pair.W, ref["kv"], ref["L"], ref["root"], 5 * n_steps + 8)
    rng = np.random.default_rng(7)
    done = 0
    reports = []
    for step in range(n_steps):
        if greedy is not None:
            cand = rng.integers(0, cfg["vocab"], size=(cfg["n_cerb_heads"], cfg["topk"]))
            depth = int(rng.integers(0, cfg["n_cerb_heads"] + 1))
            for i in range(depth):
                r = 0 if cand_mode == "planted" else cfg["topk"] - 1
                cand[i, r] = greedy[done + 1 + i]
            ost["cand"], ost["flag"] = cand, 0
        forced = None
        if gate_states is not None:
            forced = gate_states[step]
            taps.forced_gate_hidden[0] = torch.from_numpy(forced).cuda()
        H.round_oracle_kv(ost, dtype)
        H.upload_sequence(st, 0, ost, dtype)
        out = pair.oracle_step(ost, forced_gate_hidden=forced)
        pair.engine.verify_step(st, 1)
        torch.cuda.synchronize()
        rep = H.compare_step(cfg, out, st, taps, 0, pair.T, dtype, ost,
                             tol=H.TOL_BF16_TINY if dtype == BF16 else None)
        say(f"  step {step}: T={out['T']} a={out['accept_len']} flag={out['flag']} logit_err={rep.max_logit_err:.2e} "
            f"h_err={rep.max_hidden_err:.2e} head_err={rep.max_head_logit_err:.2e} S_err={rep.entropy_err:.2e} "
            f"argmax {rep.argmax_checked}/{rep.argmax_checked + rep.argmax_skipped} cand {rep.cand_checked}/"
            f"{rep.cand_checked + rep.cand_skipped}")
        assert not rep.failures, f"step {step}: " + "; ".join(rep.failures)
        reports.append((out, rep))
        done += out["accept_len"]
    return reports


@pytest.mark.parametrize("dtype,attn_mfma", [(F32, 0), (BF16, 0), (BF16, 1)])
@pytest.mark.parametrize("cand_mode", ["heads", "planted", "adversarial"])
def test_tiny_steps_match_oracle(tiny_pairs, dtype, attn_mfma, cand_mode):
    say(f"tiny steps dtype={dtype} attn_mfma={attn_mfma} cand={cand_mode}")
    reps = _run_forced_steps(tiny_pairs(dtype), 8, cand_mode, attn_mfma)
    lens = [o["accept_len"] for o, _ in reps]
    assert sum(r.accept_checked for _, r in reps) >= 6
    if cand_mode == "planted":
        assert max(lens) >= 3            # deep acceptances and their compaction were exercised
    assert sum(r.argmax_checked for _, r in reps) > 0


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_tiny_medusa_heads_mode(tiny_pairs, dtype):
    """special_block = -1 switches the link between the heads off: every head is a stack of d-wide
    Resblocks on h_last alone (the Medusa heads the paper compares with, Section 4.1).  Same step,
    same checks; the heads' candidates and logits must match the oracle's independent heads."""
    say(f"tiny steps, independent heads, dtype={dtype}")
    pair = tiny_pairs(dtype, special_block=-1)
    assert all(w == pair.cfg["d_model"] for ws in synth.head_block_widths(pair.cfg) for w in ws)
    reps = _run_forced_steps(pair, 4, "heads", 1)
    assert sum(r.cand_checked for _, r in reps) > 0


@pytest.mark.parametrize("shape", [
    dict(special_block=0), dict(special_block=2), dict(special_block=3),           # the link at the first, a middle, the last block
    dict(special_block=0, n_resblocks=1), dict(n_cerb_heads=1), dict(n_cerb_heads=8, special_block=2),
    dict(n_resblocks=16, special_block=15),
])
@pytest.mark.parametrize("dtype", [F32, BF16])
def test_tiny_head_layouts(dtype, shape):
    """Where the special Resblock sits decides which blocks of heads 1.. are 2d wide and at which
    stage a head reads its neighbour (Section 4.1): every position, a single block, a single head,
    the largest head count and block count the library takes."""
    say(f"tiny steps, head layout {shape}, dtype={dtype}")
    pair = H.Pair("tiny", dtype, "tiny" if shape.get("n_cerb_heads", 4) >= 4 else "chain1", seed=3, max_batch=1, kv_capacity=256, **shape)
    reps = _run_forced_steps(pair, 2, "heads", 1)
    assert sum(r.cand_checked for _, r in reps) > 0
    pair.engine.close()


@pytest.mark.parametrize("limit", ["vocab", "d_model"])
def test_limit_shapes(limit):
    """The largest vocabulary (65536: sixteen top-k slices, the full id range of the argmax) and the
    largest model width (8192: both column groups of the one-workgroup-per-row kernels, eight blocks
    per row in the residual kernel) the library accepts, bf16, MFMA attention."""
    if limit == "vocab":
        over = dict(vocab=65536)
    else:
        over = dict(d_model=8192, n_heads=64, head_dim=128, n_layers=1, d_ffn=1024, vocab=1024, n_cerb_heads=2,
                    n_resblocks=1, special_block=0)
    say(f"limit shape {over}")
    pair = H.Pair("tiny", BF16, "tiny" if limit == "vocab" else "chain2", seed=5, max_batch=2, kv_capacity=256, **over)
    cfg = pair.cfg
    taps = pair.taps()
    st = pair.engine.new_state()
    osts = []
    for b, n_prompt in enumerate((70, 9)):
        prompt = synth.make_token_ids(n_prompt, cfg["vocab"], seed=90 + b).numpy()
        osts.append(orc.prefill(cfg, pair.W, prompt, capacity=pair.kv_capacity))
    for step in range(2):
        for b, ost in enumerate(osts):
            ost["flag"] = 0
            H.round_oracle_kv(ost, BF16)
            H.upload_sequence(st, b, ost, BF16)
        outs = [pair.oracle_step(ost) for ost in osts]
        pair.engine.verify_step(st, 2)
        torch.cuda.synchronize()
        assert int(st.status[0]) == 0
        for b, (ost, out) in enumerate(zip(osts, outs)):
            rep = H.compare_step(cfg, out, st, taps, b, pair.T, BF16, ost, tol=H.TOL_BF16)
            say(f"  step {step} seq {b}: logit_err={rep.max_logit_err:.2e} head_err={rep.max_head_logit_err:.2e} "
                f"argmax {rep.argmax_checked} cand {rep.cand_checked}")
            assert not rep.failures, f"{limit} step {step} seq {b}: " + "; ".join(rep.failures)
    pair.engine.close()


@pytest.mark.parametrize("tree", ["p120", "p150"])
@pytest.mark.parametrize("dtype,attn_mfma", [(F32, 0), (BF16, 0), (BF16, 1)])
def test_tiny_large_trees(dtype, attn_mfma, tree):
    """Trees of 120 and 150 paths (Section 5.1 "Tree Settings"; 121 / 151 nodes, ranks up to 9):
    ancestor masks of two and three words, several row blocks, query blocks and tree chunks.  Every
    node's logits, token and argmax are compared, so every mask word and block is exercised."""
    say(f"tiny steps, tree {tree}, dtype={dtype} attn_mfma={attn_mfma}")
    pair = H.Pair("tiny", dtype, tree, seed=0, max_batch=1, kv_capacity=512, topk=10)
    assert pair.T == int(tree[1:]) + 1
    reps = _run_forced_steps(pair, 3, "planted", attn_mfma)
    assert sum(r.argmax_checked for _, r in reps) > 0
    pair.engine.close()


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_tiny_gated_steps_take_both_paths(tiny_pairs, dtype):
    """configs[0]: threshold at the median entropy of 64 random states; the gate input of every
    step is one of those states, so auto-regressive and tree steps alternate."""
    states = synth.make_gate_states(64, 256, seed=0).numpy()
    S = np.sort([orc.entropy_bits(h) for h in states])
    thr = float((S[31] + S[32]) / 2)
    pair = tiny_pairs(dtype, entropy_threshold=thr)
    say(f"tiny gated dtype={dtype} threshold={thr:.4f}")
    reps = _run_forced_steps(pair, 32, "heads", 1 if dtype == BF16 else 0, gate_states=states)
    Ts = [o["T"] for o, _ in reps]
    assert 1 in Ts and 16 in Ts
    assert all(o["accept_len"] == 1 for o, _ in reps if o["T"] == 1)
    assert sum(r.flag_checked for _, r in reps) >= 24


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_ar_step_entry_point(tiny_pairs, dtype):
    pair = tiny_pairs(dtype)
    taps = pair.taps()
    st = pair.engine.new_state()
    ost = _prefilled(pair, seed=3)
    ost["flag"] = 0                          # the entry point must ignore the flag
    for step in range(3):
        H.round_oracle_kv(ost, dtype)
        H.upload_sequence(st, 0, ost, dtype)
        out = pair.oracle_step(ost, force_ar=True)
        pair.engine.ar_step(st, 1)
        torch.cuda.synchronize()
        rep = H.compare_step(pair.cfg, out, st, taps, 0, pair.T, dtype, ost)
        assert out["T"] == 1 and not rep.failures, "; ".join(rep.failures)


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_decode_chains_steps_on_the_device_and_logs_tokens(tiny_pairs, dtype):
    """The multi-step driver: n steps enqueued in one call, the device-side gate flag choosing each
    next step's shape, committed tokens appended to a device log.  Free-running on both sides (no
    teacher forcing is possible inside the call), so the comparison stops at the first decision of
    the oracle whose margin is within the tolerance; the threshold is set between the entropies a
    dry oracle run produces, so both kinds of step occur."""
    n_steps = 14
    tol = H.TOL_F32 if dtype == F32 else H.TOL_BF16_TINY
    base = tiny_pairs(dtype)
    dry = _prefilled(base)
    H.round_oracle_kv(dry, dtype)
    ent = sorted(base.oracle_step(dry)["entropy"] for _ in range(n_steps))
    thr = 0.5 * (ent[n_steps // 2 - 1] + ent[n_steps // 2])
    pair = tiny_pairs(dtype, entropy_threshold=float(thr))
    pair.engine.set_param("attn_mfma", 1)
    pair.engine.set_taps(None)
    ost = _prefilled(pair)
    H.round_oracle_kv(ost, dtype)
    st = pair.engine.new_state()
    H.upload_sequence(st, 0, ost, dtype)
    L0 = ost["L"]
    log = torch.full((1, 64), -1, dtype=torch.int32, device="cuda")
    count = torch.zeros(1, dtype=torch.int32, device="cuda")
    pair.engine.decode(st, 1, n_steps, log, count)
    torch.cuda.synchronize()
    assert int(st.status[0]) == 0
    got = log[0, :int(count[0])].cpu().tolist()
    assert int(st.kv_len[0]) == L0 + len(got)

    want, kinds, clear = [], [], True
    for step in range(n_steps):
        out = pair.oracle_step(ost)
        srt = -np.sort(-out["logits"][out["path"]], axis=1)
        margin = float(np.min(srt[:, 0] - srt[:, 1]))
        if margin <= 2 * tol.logits or abs(out["entropy"] - thr) <= 2 * tol.entropy:
            clear = False
            say(f"  step {step}: oracle margin {margin:.2e}, entropy gap {abs(out['entropy'] - thr):.2e}: comparison ends here")
            break
        want += [int(t) for t in out["committed"]]
        kinds.append(out["T"])
    say(f"  {len(kinds)} steps compared, tree sizes {kinds}, {len(want)} tokens")
    assert got[:len(want)] == want
    assert len(kinds) >= 6 and 1 in kinds and pair.T in kinds        # both kinds of step ran
    if clear:
        assert len(got) == len(want) and int(st.gate_flag[0]) == ost["flag"] and int(st.root_token[0]) == ost["root"]

    # a log too short for the tokens: the sequence keeps decoding, the log stops, the status says so
    st2 = pair.engine.new_state()
    ost2 = _prefilled(pair)
    H.round_oracle_kv(ost2, dtype)
    H.upload_sequence(st2, 0, ost2, dtype)
    short = torch.full((1, 3), -1, dtype=torch.int32, device="cuda")
    count2 = torch.zeros(1, dtype=torch.int32, device="cuda")
    pair.engine.decode(st2, 1, 5, short, count2)
    torch.cuda.synchronize()
    assert int(count2[0]) == 3 and short[0].cpu().tolist() == got[:3]
    assert int(st2.status[0]) == B.CERBERUS_DEV_LOG_FULL and int(st2.kv_len[0]) >= L0 + 5


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_generate_from_prompts_equals_greedy_decoding(dtype):
    """End to end, nothing injected: prompt phase and chained steps on the device for two sequences,
    against plain greedy auto-regressive decoding in the oracle (the method is lossless: whatever
    the heads propose, the committed stream is the base model's greedy stream).  Compared up to the
    first token whose top-2 margin in the oracle is within the tolerance."""
    pair = H.Pair("tiny", dtype, "tiny", seed=4, max_batch=2, kv_capacity=256)
    cfg = pair.cfg
    tol = H.TOL_F32 if dtype == F32 else H.TOL_BF16_TINY
    st = pair.engine.new_state()
    prompts = [synth.make_token_ids(n, cfg["vocab"], seed=300 + n) for n in (45, 17)]
    n_steps = 12
    got = pair.engine.generate(st, prompts, n_steps)
    assert int(st.status[0]) == 0
    for b, p in enumerate(prompts):
        ost = orc.prefill(cfg, pair.W, p.numpy(), capacity=pair.kv_capacity)
        assert len(got[b]) >= n_steps and int(st.kv_len[b]) == len(p) + len(got[b])
        L, t, n_ok = ost["L"], ost["root"], 0
        for k in range(len(got[b])):
            if got[b][k] != t:
                break
            _, logits = orc.decoder_rows(cfg, pair.W, np.array([t]), np.array([L]), np.ones((1, 1), bool), ost["kv"], L)
            L += 1
            n_ok += 1
            srt = -np.sort(-logits[0])
            if srt[0] - srt[1] <= 2 * tol.logits:      # the next token is not decided within the tolerance
                say(f"  seq {b}: margin {srt[0] - srt[1]:.2e} after {n_ok} tokens: comparison ends here")
                n_ok = len(got[b])
                break
            t = int(orc.argmax_lowest(logits[0]))
        say(f"  seq {b}: {len(got[b])} tokens generated, greedy stream matched")
        assert n_ok == len(got[b]), f"seq {b}: token {n_ok} is {got[b][n_ok]}, greedy decoding gives {t}"
    pair.engine.close()


@pytest.mark.parametrize("n_prompt", [100, 230])
@pytest.mark.parametrize("dtype", [F32, BF16])
def test_prefill_seeds_the_first_step(tiny_pairs, dtype, n_prompt):
    """Algorithm 1 lines 1-5: the prompt's causal forward from an empty cache, in passes of up to 192
    rows (100 tokens: one pass; 230: a full pass and one of 38), then LM head, gate and heads on the last position.
    Compared with the oracle's one-shot causal prefill: every K/V row, the logits of the last pass,
    the pending token, entropy and flag, the candidates; then one decoding step taken from the seeded
    state on both sides."""
    # bf16: the rows of earlier passes are read back from the bf16 cache while the oracle keeps them
    # in float64, so the bar is the general bf16 one, not the teacher-forced tiny-shape one
    tol = H.TOL_F32 if dtype == F32 else H.TOL_BF16
    pair = tiny_pairs(dtype)
    cfg, T = pair.cfg, pair.T
    pair.engine.set_param("attn_mfma", 1)
    taps = pair.taps()
    prompt = synth.make_token_ids(n_prompt, cfg["vocab"], seed=21)
    st = pair.engine.new_state()
    st.kv_len[0] = 0
    st.gate_flag[0] = 1                       # must be overwritten by the gate
    pair.engine.prefill(st, 1, 0, prompt.cuda())
    torch.cuda.synchronize()
    assert int(st.status[0]) == 0 and int(st.kv_len[0]) == n_prompt and int(st.accept_len[0]) == 0

    # the oracle's prefill, once for the state and once step by step for the intermediate values
    ost = orc.prefill(cfg, pair.W, prompt.numpy(), capacity=pair.kv_capacity)
    kv2 = orc.new_kv(cfg, pair.kv_capacity)
    h_last, logits = orc.decoder_rows(cfg, pair.W, prompt.numpy(), np.arange(n_prompt),
                                      np.tril(np.ones((n_prompt, n_prompt), dtype=bool)), kv2, 0)
    for l in range(cfg["n_layers"]):
        for kvi in (0, 1):
            got = st.kv[l, kvi, 0, :, :n_prompt].double().cpu().numpy()
            want = ost["kv"][l][kvi][:, :n_prompt]
            mm = H.kv_mismatch(got, want, tol)
            assert mm is None, (l, kvi, mm)
    P = B.CERBERUS_MAX_TREE                    # rows of a full pass
    n_last = n_prompt % P or P                 # rows of the last pass: the taps hold its first T rows at slots 0..
    k, first = min(n_last, T), n_prompt - n_last
    err = float(np.max(np.abs(taps.logits[:k].double().cpu().numpy() - logits[first:first + k])))
    herr = float(np.max(np.abs(taps.h_last[:k].double().cpu().numpy() - h_last[first:first + k])))
    say(f"  prefill: last pass of {n_last} rows, first {k} tapped, logits err {err:.2e}, h_last err {herr:.2e}")
    assert err <= tol.logits and herr <= tol.hidden
    srt = -np.sort(-logits[-1])
    if srt[0] - srt[1] > 2 * tol.logits:
        assert int(st.root_token[0]) == ost["root"]
    S, flag = orc.gate(h_last[-1], cfg["entropy_threshold"])
    assert abs(float(st.entropy[0]) - S) <= tol.entropy and int(st.gate_flag[0]) == flag == 0
    want_hl = np.stack(orc.cerberus_heads(cfg, pair.W["heads"], h_last[-1]))
    hl = taps.head_logits[0].double().cpu().numpy()
    checked = 0
    for i in range(cfg["n_cerb_heads"]):
        tol_i = H.head_logit_tol(tol, want_hl[i])
        assert float(np.max(np.abs(hl[i] - want_hl[i]))) <= tol_i
        srt_i = -np.sort(-want_hl[i])[:cfg["topk"] + 1]
        for j in range(cfg["topk"]):
            if H._margin_ok(srt_i, j, tol_i):
                checked += 1
                assert int(st.cand[0, i, j]) == int(ost["cand"][i, j]), (i, j)
    assert checked > 0

    # a second sequence's slot is untouched by a prefill of the first: covered by batch = 1 here; the
    # decoding step that follows runs from the seeded state on both sides
    if int(st.root_token[0]) == ost["root"] and np.array_equal(st.cand[0].cpu().numpy(), ost["cand"]):
        out = pair.oracle_step(ost)
        pair.engine.verify_step(st, 1)
        torch.cuda.synchronize()
        rep = H.compare_step(cfg, out, st, taps, 0, T, dtype, ost, tol=tol)
        say(f"  first step after prefill: logits err {rep.max_logit_err:.2e}, accept {out['accept_len']}")
        assert not rep.failures, "; ".join(rep.failures)

    # a prompt that does not fit: status bit, nothing committed beyond what fitted
    st3 = pair.engine.new_state()
    st3.kv_len[0] = pair.kv_capacity - 20
    pair.engine.prefill(st3, 1, 0, prompt[:40].cuda())
    torch.cuda.synchronize()
    assert int(st3.status[0]) & B.CERBERUS_DEV_KV_OVERFLOW
    assert int(st3.kv_len[0]) == pair.kv_capacity - 20           # the one pass of 40 rows did not fit: nothing committed
    with pytest.raises(RuntimeError):
        pair.engine.prefill(st3, 1, 1, prompt.cuda())             # sequence index out of range


def test_prefill_of_one_sequence_leaves_the_others_alone():
    """Batch of four: sequences 0, 1 and 3 hold decoding states, sequence 2 gets its prompt.  Nothing
    of the others may change, and the next launch decodes all four against the oracle."""
    dtype = F32
    pair = H.Pair("tiny", dtype, "tiny", seed=0, max_batch=4, kv_capacity=256)
    cfg = pair.cfg
    taps = pair.taps()
    st = pair.engine.new_state()
    osts = {}
    for b, n_prompt in ((0, 33), (1, 90), (3, 17)):
        prompt = synth.make_token_ids(n_prompt, cfg["vocab"], seed=60 + b).numpy()
        osts[b] = orc.prefill(cfg, pair.W, prompt, capacity=pair.kv_capacity)
        H.upload_sequence(st, b, osts[b], dtype)
    st.kv_len[2] = 0
    before = {k: getattr(st, k).clone() for k in ("kv", "kv_len", "root_token", "cand", "gate_flag", "entropy", "accept_len")}
    prompt2 = synth.make_token_ids(45, cfg["vocab"], seed=62)
    pair.engine.prefill(st, 4, 2, prompt2.cuda())
    torch.cuda.synchronize()
    assert int(st.status[0]) == 0 and int(st.kv_len[2]) == 45
    others = [0, 1, 3]
    for k, v in before.items():
        got = getattr(st, k)
        if k == "kv":
            assert torch.equal(got[:, :, others], v[:, :, others])
        else:
            assert torch.equal(got[others], v[others]), k
    osts[2] = orc.prefill(cfg, pair.W, prompt2.numpy(), capacity=pair.kv_capacity)
    assert int(st.root_token[2]) == osts[2]["root"] and np.array_equal(st.cand[2].cpu().numpy(), osts[2]["cand"])
    outs = {b: pair.oracle_step(osts[b]) for b in range(4)}
    pair.engine.verify_step(st, 4)
    torch.cuda.synchronize()
    for b in range(4):
        rep = H.compare_step(cfg, outs[b], st, taps, b, pair.T, dtype, osts[b])
        assert not rep.failures, f"seq {b}: " + "; ".join(rep.failures)
    pair.engine.close()


def test_gate_entry_point_matches_oracle(tiny_pairs):
    states = synth.make_gate_states(64, 256, seed=0)
    S = np.array([orc.entropy_bits(h) for h in states.numpy()])
    srt = np.sort(S)
    thr = float((srt[31] + srt[32]) / 2)
    pair = tiny_pairs(F32, entropy_threshold=thr)
    ent = torch.zeros(64, dtype=torch.float32, device="cuda")
    flag = torch.full((64,), -1, dtype=torch.int32, device="cuda")
    B.cerberus_gate(pair.engine.ctx, states.cuda(), ent, flag)
    torch.cuda.synchronize()
    assert np.max(np.abs(ent.cpu().numpy() - S)) < 1e-4
    clear = np.abs(S - thr) > 1e-3
    assert clear.sum() >= 60
    assert np.array_equal(flag.cpu().numpy()[clear], (S > thr).astype(np.int32)[clear])
    assert 20 <= int(flag.sum()) <= 44
    # closed forms: uniform state -> log2(d); one dominant component -> 0; NaN -> auto-regressive
    special = torch.zeros((3, 256), dtype=torch.float32)
    special[0] = 2.5
    special[1, 17] = 1e4
    special[2, 3] = float("nan")
    B.cerberus_gate(pair.engine.ctx, special.cuda(), ent[:3], flag[:3])
    torch.cuda.synchronize()
    e = ent[:3].cpu().numpy()
    assert abs(e[0] - 8.0) < 1e-5 and e[1] == 0.0 and np.isnan(e[2])
    assert flag[:3].cpu().numpy().tolist() == [int(8.0 > thr), 0, 1]


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_accept_entry_point_is_bit_exact(tiny_pairs, dtype):
    pair = tiny_pairs(dtype)
    cfg, T = pair.cfg, pair.T
    st = pair.engine.new_state()
    g = torch.Generator().manual_seed(5)
    L = 37
    tok = torch.arange(100, 100 + T, dtype=torch.int32)
    cases = {
        "none": {},                                   # nothing matches: only the root
        "hazard": {0: 2, 2: 7, 7: 14},                # path 0,2,7,14: row L+2 is a source and a later destination
        "deep": {0: 1, 1: 5, 5: 12, 12: 15},          # full depth
        "dup": {0: 2},
    }
    for name, chain in cases.items():
        kv = torch.randn(st.kv.shape, generator=g).to(st.kv.dtype)
        st.kv.copy_(kv.cuda())
        st.kv_len[0] = L
        tk = tok.clone()
        if name == "dup":
            tk[1] = tk[2]                              # duplicate siblings: lower index wins
        gg = torch.full((T,), -1, dtype=torch.int32)
        for a, b in chain.items():
            if b is not None:
                gg[a] = tk[b]
        want_path = orc.accept_path(gg.numpy(), tk.numpy(), pair.parent)
        ref = [(kv[l, 0, 0].double().numpy().copy(), kv[l, 1, 0].double().numpy().copy()) for l in range(cfg["n_layers"])]
        orc.compact_kv(ref, L, want_path)
        B.cerberus_accept(pair.engine.ctx, gg.cuda(), tk.cuda(), st.struct, 1)
        torch.cuda.synchronize()
        a = int(st.accept_len[0])
        assert st.accepted_nodes[0, :a].cpu().tolist() == want_path, name
        assert st.accepted_tokens[0, :a].cpu().tolist() == [int(tk[n]) for n in want_path]
        assert int(st.kv_len[0]) == L + a and int(st.root_token[0]) == int(gg[want_path[-1]])
        got = st.kv.cpu()
        for l in range(cfg["n_layers"]):
            for kvi in (0, 1):
                want = torch.from_numpy(ref[l][kvi]).to(st.kv.dtype)
                # rows below L + a are defined and must be bit-identical copies; rows above are don't-care
                assert torch.equal(got[l, kvi, 0, :, :L + a], want[:, :L + a]), (name, l, kvi)
        if name == "dup":
            assert want_path == [0, 1]
    assert int(st.status[0]) == 0


def test_capacity_overflow_sets_status_and_skips(tiny_pairs):
    pair = tiny_pairs(F32)
    st = pair.engine.new_state()
    st.kv_len[0] = pair.kv_capacity - 3              # the 16-node tree no longer fits
    st.gate_flag[0] = 0
    before = st.kv.clone()
    pair.engine.verify_step(st, 1)
    torch.cuda.synchronize()
    assert int(st.status[0]) & B.DEV_KV_OVERFLOW
    assert int(st.accept_len[0]) == 0 and int(st.kv_len[0]) == pair.kv_capacity - 3
    assert torch.equal(before, st.kv)


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_tree_that_exactly_fills_the_cache(dtype):
    """A capacity that is no multiple of the attention chunk (333 rows), and a prefix that leaves
    room for exactly the 16 rows of the tree: the last cache row is written and read, nothing beyond."""
    pair = H.Pair("tiny", dtype, "tiny", seed=2, max_batch=1, kv_capacity=333)
    cfg = pair.cfg
    taps = pair.taps()
    st = pair.engine.new_state()
    prompt = synth.make_token_ids(333 - pair.T, cfg["vocab"], seed=33).numpy()
    ost = orc.prefill(cfg, pair.W, prompt, capacity=pair.kv_capacity)
    ost["flag"] = 0
    H.round_oracle_kv(ost, dtype)
    H.upload_sequence(st, 0, ost, dtype)
    out = pair.oracle_step(ost)
    pair.engine.verify_step(st, 1)
    torch.cuda.synchronize()
    assert int(st.status[0]) == 0
    rep = H.compare_step(cfg, out, st, taps, 0, pair.T, dtype, ost, tol=H.TOL_BF16_TINY if dtype == BF16 else None)
    assert not rep.failures, "; ".join(rep.failures)
    # one more row of prefix and the same tree no longer fits
    st.kv_len[0] = 333 - pair.T + 1
    st.gate_flag[0] = 0
    pair.engine.verify_step(st, 1)
    torch.cuda.synchronize()
    assert int(st.status[0]) & B.DEV_KV_OVERFLOW
    pair.engine.close()


def test_bad_arguments_are_rejected(tiny_pairs):
    pair = tiny_pairs(F32)
    st = pair.engine.new_state()
    with pytest.raises(B.CerberusError):
        pair.engine.verify_step(st, 2)               # batch > max_batch
    with pytest.raises(B.CerberusError):
        pair.engine.set_param("no_such_knob", 1)


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_tiny_batch_mixed_ar_and_tree_in_one_launch(dtype):
    """Four independent sequences with different prefix lengths and gate decisions share one launch:
    rows are packed per sequence, a flagged sequence contributes a single row."""
    pair = H.Pair("tiny", dtype, "tiny", seed=0, max_batch=4, kv_capacity=256)
    cfg = pair.cfg
    taps = pair.taps()
    st = pair.engine.new_state()
    tol = H.TOL_BF16_TINY if dtype == BF16 else None
    osts = []
    for b, (n_prompt, flag) in enumerate(((40, 0), (77, 1), (128, 0), (100, 1))):
        prompt = synth.make_token_ids(n_prompt, cfg["vocab"], seed=20 + b).numpy()
        ost = orc.prefill(cfg, pair.W, prompt, capacity=pair.kv_capacity)
        if flag:
            ost["flag"] = 1
        osts.append(ost)
    for step in range(4):
        for b, ost in enumerate(osts):
            H.round_oracle_kv(ost, dtype)
            H.upload_sequence(st, b, ost, dtype)
        outs = [pair.oracle_step(ost) for ost in osts]
        pair.engine.verify_step(st, 4)
        torch.cuda.synchronize()
        assert int(st.status[0]) == 0
        for b, (ost, out) in enumerate(zip(osts, outs)):
            rep = H.compare_step(cfg, out, st, taps, b, pair.T, dtype, ost, tol=tol)
            say(f"  step {step} seq {b}: T={out['T']} L={out['L_before']} a={out['accept_len']} logit_err={rep.max_logit_err:.2e}")
            assert not rep.failures, f"step {step} seq {b}: " + "; ".join(rep.failures)
        if step == 1:                      # flip the gate decisions for the next launch
            for ost in osts:
                ost["flag"] = 1 - ost["flag"]
    # a batch smaller than max_batch and the forced one-token entry point
    for b, ost in enumerate(osts[:3]):
        H.round_oracle_kv(ost, dtype)
        H.upload_sequence(st, b, ost, dtype)
    outs = [pair.oracle_step(ost, force_ar=True) for ost in osts[:3]]
    pair.engine.ar_step(st, 3)
    torch.cuda.synchronize()
    for b, (ost, out) in enumerate(zip(osts[:3], outs)):
        rep = H.compare_step(cfg, out, st, taps, b, pair.T, dtype, ost, tol=tol)
        assert out["T"] == 1 and not rep.failures, f"ar seq {b}: " + "; ".join(rep.failures)


@pytest.mark.parametrize("target_wgs,chunk", [(1, 128), (8, 128), (16, 128), (4096, 128), (1, 256), (4096, 256)])
def test_tiny_attention_work_list(target_wgs, chunk):
    """The MFMA attention kernel walks a work list built from the sequences' present lengths: with a small
    workgroup target a cache range of several chunks is one item (running softmax over its rounds, the last
    round ragged), with a large one every chunk is its own item; three sequences of different lengths, one
    of them on the one-token path, share the launch.  Either way the step matches the oracle."""
    pair = H.Pair("tiny", BF16, "p63", seed=0, max_batch=3, kv_capacity=640, topk=6)
    pair.engine.set_param("attn_chunk", chunk)
    pair.engine.set_param("attn_target_wgs", target_wgs)
    cfg = pair.cfg
    taps = pair.taps()
    st = pair.engine.new_state()
    osts = []
    for b, (n_prompt, flag) in enumerate(((531, 0), (300, 1), (129, 0))):     # 5, 3 and 2 chunks of 128 rows
        prompt = synth.make_token_ids(n_prompt, cfg["vocab"], seed=60 + b).numpy()
        ost = orc.prefill(cfg, pair.W, prompt, capacity=pair.kv_capacity)
        ost["flag"] = flag
        H.round_oracle_kv(ost, BF16)
        H.upload_sequence(st, b, ost, BF16)
        osts.append(ost)
    outs = [pair.oracle_step(ost) for ost in osts]
    pair.engine.verify_step(st, 3)
    torch.cuda.synchronize()
    assert int(st.status[0]) == 0
    for b, (ost, out) in enumerate(zip(osts, outs)):
        rep = H.compare_step(cfg, out, st, taps, b, pair.T, BF16, ost, tol=H.TOL_BF16_TINY)
        say(f"  target {target_wgs} chunk {chunk} seq {b}: L={out['L_before']} logit_err={rep.max_logit_err:.2e}")
        assert not rep.failures, f"seq {b}: " + "; ".join(rep.failures)
    pair.engine.close()


@pytest.mark.parametrize("tree", ["root", "chain4", "rand17s1k4", "rand33s2k4", "rand65s3k4", "rand100s4k4", "rand129s5k4"])
def test_tiny_odd_tree_shapes(tree):
    """Tree sizes that are no multiple of anything (a lone root, a single chain, random shapes around
    the 16-, 32-, 64- and 128-row boundaries), bf16 MFMA path, two sequences with different prefixes:
    every node's token, logits and argmax, acceptance, gate, candidates against the oracle."""
    pair = H.Pair("tiny", BF16, tree, seed=0, max_batch=2, kv_capacity=384)
    cfg = pair.cfg
    taps = pair.taps()
    st = pair.engine.new_state()
    osts = []
    for b, n_prompt in enumerate((131, 58)):
        prompt = synth.make_token_ids(n_prompt, cfg["vocab"], seed=70 + b).numpy()
        osts.append(orc.prefill(cfg, pair.W, prompt, capacity=pair.kv_capacity))
    for step in range(2):
        for b, ost in enumerate(osts):
            ost["flag"] = 0
            H.round_oracle_kv(ost, BF16)
            H.upload_sequence(st, b, ost, BF16)
        outs = [pair.oracle_step(ost) for ost in osts]
        pair.engine.verify_step(st, 2)
        torch.cuda.synchronize()
        assert int(st.status[0]) == 0
        for b, (ost, out) in enumerate(zip(osts, outs)):
            rep = H.compare_step(cfg, out, st, taps, b, pair.T, BF16, ost, tol=H.TOL_BF16_TINY)
            assert not rep.failures, f"{tree} step {step} seq {b}: " + "; ".join(rep.failures)
    say(f"  tree {tree}: {pair.T} nodes ok")
    pair.engine.close()


@pytest.mark.parametrize("seed", list(range(10)))
def test_tiny_random_launches(seed):
    """Seeded random launches: tree shape, batch, prefix lengths (down to a single committed row),
    which sequences take the one-token step, and per-sequence candidates planted to a random depth
    on a random child rank, so that acceptance, compaction and packing meet in combinations the
    hand-written cases do not list.  Three chained launches per case; every sequence is compared."""
    rng = np.random.default_rng(1000 + seed)
    dtype = F32 if seed % 5 == 4 else BF16
    tree = ["tiny", "p63", f"rand{int(rng.integers(20, 60))}s{seed}k4", f"rand{int(rng.integers(66, 140))}s{seed}k4",
            "chain4", "p63", "tiny", f"rand{int(rng.integers(2, 16))}s{seed}k4", "p63", "bfs3x40"][seed]
    max_batch = int(rng.integers(1, 6))
    batch = int(rng.integers(1, max_batch + 1))
    pair = H.Pair("tiny", dtype, tree, seed=seed, max_batch=max_batch, kv_capacity=384, **({"topk": 6} if tree == "p63" else {}))
    cfg = pair.cfg
    Hc, K = cfg["n_cerb_heads"], cfg["topk"]
    taps = pair.taps()
    st = pair.engine.new_state()
    tol = H.TOL_BF16_TINY if dtype == BF16 else None
    osts, greedy, done = [], [], []
    for b in range(batch):
        n_prompt = int(rng.choice([1, 2, 3, 17, 64, 127, 128, 129, 200])) if rng.random() < 0.6 else int(rng.integers(1, 230))
        prompt = synth.make_token_ids(n_prompt, cfg["vocab"], seed=500 + 10 * seed + b).numpy()
        osts.append(orc.prefill(cfg, pair.W, prompt, capacity=pair.kv_capacity))
        ref = orc.prefill(cfg, pair.W, prompt, capacity=pair.kv_capacity)
        greedy.append(orc.greedy_decode(cfg, pair.W, ref["kv"], ref["L"], ref["root"], 3 * (Hc + 1) + 2))
        done.append(0)
    say(f"  seed {seed}: tree {tree} ({pair.T} nodes), dtype {dtype}, batch {batch}/{max_batch}, prefixes {[o['L'] for o in osts]}")
    for step in range(3):
        for b, ost in enumerate(osts):
            cand = rng.integers(0, cfg["vocab"], size=(Hc, K))
            for i in range(int(rng.integers(0, Hc + 1))):
                cand[i, int(rng.integers(0, K))] = greedy[b][done[b] + 1 + i]
            ost["cand"] = cand
            ost["flag"] = int(rng.random() < 0.3)
            H.round_oracle_kv(ost, dtype)
            H.upload_sequence(st, b, ost, dtype)
        outs = [pair.oracle_step(ost) for ost in osts]
        pair.engine.verify_step(st, batch)
        torch.cuda.synchronize()
        assert int(st.status[0]) == 0
        for b, (ost, out) in enumerate(zip(osts, outs)):
            rep = H.compare_step(cfg, out, st, taps, b, pair.T, dtype, ost, tol=tol)
            assert not rep.failures, f"seed {seed} step {step} seq {b} (T={out['T']}, L={out['L_before']}, a={out['accept_len']}): " + "; ".join(rep.failures)
            done[b] += out["accept_len"]
    pair.engine.close()


@pytest.mark.parametrize("dtype,attn_mfma", [(F32, 0), (BF16, 1)])
def test_tiny_head_dim_128_full_tree(dtype, attn_mfma):
    """The 7B/13B head size (128) and the 64-node tree at a width the oracle can afford for every
    node: two heads of 128, all 64 rows compared (the full-size tests compare one sampled path)."""
    say(f"tiny with head_dim 128, 64-node tree, dtype={dtype}")
    pair = H.Pair("tiny", dtype, "p63", seed=0, max_batch=1, kv_capacity=384, n_heads=2, head_dim=128, topk=6)
    assert pair.cfg["n_heads"] * pair.cfg["head_dim"] == pair.cfg["d_model"] and pair.T == 64
    reps = _run_forced_steps(pair, 3, "planted", attn_mfma)
    assert sum(r.argmax_checked for _, r in reps) > 0
    pair.engine.close()


def test_graph_replay_equals_eager_launch(tiny_pairs):
    """bench.py times a HIP-graph replay of the step.  The same step captured once and replayed
    several times, with eager work and synchronisations between the replays, must reproduce the
    eager launch bit for bit every time (the library enqueues kernels only, no memset nodes)."""
    pair = tiny_pairs(BF16)
    pair.engine.set_param("attn_mfma", 1)
    taps = pair.taps()
    ost = _prefilled(pair)
    H.round_oracle_kv(ost, BF16)
    st = pair.engine.new_state()
    H.upload_sequence(st, 0, ost, BF16)
    snap = {k: getattr(st, k).clone() for k in ("kv", "kv_len", "root_token", "cand", "gate_flag")}

    def restore():
        for k, v in snap.items():
            getattr(st, k).copy_(v)

    pair.engine.verify_step(st, 1)
    torch.cuda.synchronize()
    names = ("kv", "kv_len", "root_token", "cand", "gate_flag", "entropy", "accept_len", "accepted_tokens", "accepted_nodes")
    eager = {k: getattr(st, k).clone() for k in names}
    eager_logits = taps.logits.clone()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        restore()
        pair.engine.verify_step(st, 1, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    restore()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        pair.engine.verify_step(st, 1, stream=torch.cuda.current_stream())
    for rep in range(4):
        restore()
        taps.logits.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in names:
            assert torch.equal(getattr(st, k), eager[k]), (rep, k)
        assert torch.equal(taps.logits, eager_logits), rep
        _ = (taps.logits.sum() + st.kv.float().sum()).item()      # eager library work between replays
    assert int(st.status[0]) == 0


@pytest.mark.parametrize("params", [
    {"gemm_nsub": 4}, {"gemm_target_wgs": 64}, {"gemm_target_wgs": 4096, "gemm_max_split": 16}, {"gemm_max_split": 1},
    {"act_split": 0}, {"act_split": 0, "gemm_nsub": 4, "attn_mfma": 0}, {"attn_chunk": 256}, {"attn_chunk": 128},
    {"gemm_wg_slots": 0}, {"gemm_wg_slots": 40}, {"gemm_uneven_split": 1, "gemm_target_wgs": 100, "gemm_wg_slots": 0},
    {"gemm_fused": 0}, {"gemm_fused": 1},
])
def test_tiny_tuning_knobs_do_not_change_results(params):
    """Every value of the tuning knobs selects another tiling, split or kernel instance of the same
    arithmetic (one activation plane instead of two with act_split = 0: bf16-rounded GEMM inputs, still
    well inside the bf16 bar at this depth)."""
    pair = H.Pair("tiny", BF16, "p63", seed=0, max_batch=1, kv_capacity=384, topk=6)
    for k, v in params.items():
        pair.engine.set_param(k, v)
    cfg = pair.cfg
    taps = pair.taps()
    st = pair.engine.new_state()
    ost = orc.prefill(cfg, pair.W, synth.make_token_ids(77, cfg["vocab"], seed=80).numpy(), capacity=pair.kv_capacity)
    ost["flag"] = 0
    H.round_oracle_kv(ost, BF16)
    H.upload_sequence(st, 0, ost, BF16)
    out = pair.oracle_step(ost)
    pair.engine.verify_step(st, 1)
    torch.cuda.synchronize()
    tol = H.TOL_BF16
    if params.get("act_split") == 0:
        # one bf16 plane: a GEMM input carries 8 significant bits instead of 16, so a new cache row is off
        # by up to 2^-9 relative before its own rounding to bf16: up to two rounding steps apart
        tol = dataclasses.replace(tol, kv_atol=1e-2, kv_rtol=1.6e-2)
    rep = H.compare_step(cfg, out, st, taps, 0, pair.T, BF16, ost, tol=tol)
    say(f"  {params}: logits err {rep.max_logit_err:.2e}")
    assert not rep.failures, f"{params}: " + "; ".join(rep.failures)
    pair.engine.close()


@pytest.mark.parametrize("nsub_rows,team", [(4, 3), (2, 1), (2, 0)])
def test_tiny_maximum_batch_and_tree(nsub_rows, team):
    """The largest launch the library takes: 16 sequences, a 192-node tree (three mask words, three
    query blocks and tree chunks), 13 of them running the whole tree and 3 a single row: 2499 packed
    rows, 40 row blocks in every GEMM (with either instance of the GEMM for several row blocks; gate/up,
    QKV and the LM head on the team kernel, 23 row blocks of 112 rows, only gate/up, or everything on
    the same kernel).  Every row of every sequence is compared."""
    pair = H.Pair("tiny", BF16, "bfs4x192", seed=0, max_batch=16, kv_capacity=384)
    pair.engine.set_param("gemm_nsub_rows", nsub_rows)
    pair.engine.set_param("gemm_team", team)
    cfg = pair.cfg
    assert pair.T == B.CERBERUS_MAX_TREE and pair.max_batch == B.CERBERUS_MAX_BATCH
    taps = pair.taps()
    st = pair.engine.new_state()
    osts = []
    for b in range(16):
        prompt = synth.make_token_ids(8 + 11 * b, cfg["vocab"], seed=40 + b).numpy()     # prefixes 8 .. 173
        ost = orc.prefill(cfg, pair.W, prompt, capacity=pair.kv_capacity)
        ost["flag"] = 1 if b in (3, 8, 15) else 0
        H.round_oracle_kv(ost, BF16)
        H.upload_sequence(st, b, ost, BF16)
        osts.append(ost)
    outs = [pair.oracle_step(ost) for ost in osts]
    pair.engine.verify_step(st, 16)
    torch.cuda.synchronize()
    assert int(st.status[0]) == 0
    worst = 0.0
    for b, (ost, out) in enumerate(zip(osts, outs)):
        rep = H.compare_step(cfg, out, st, taps, b, pair.T, BF16, ost, tol=H.TOL_BF16_TINY)
        worst = max(worst, rep.max_logit_err)
        assert not rep.failures, f"seq {b}: " + "; ".join(rep.failures)
    say(f"  16 sequences, {sum(o['T'] for o in outs)} rows: worst logits err {worst:.2e}")
    pair.engine.close()


@pytest.mark.parametrize("flags", [(0, 0, 0), (1, 0, 1), (1, 1, 1), (0, 1, 0)])
def test_tiny_row_counts_below_the_launch_bound(flags):
    """The launches of a step are planned for batch x tree rows (3 x 192 = 576 here); how many rows there are
    is decided on the device by the gate flags: 576, 194, 3 or 385.  The GEMM for many rows forms its row
    blocks and teams from that count, and its consumers sum the planned number of partial planes whatever
    it is.  Every row of every sequence is compared."""
    pair = H.Pair("tiny", BF16, "bfs4x192", seed=0, max_batch=3, kv_capacity=384)
    cfg = pair.cfg
    taps = pair.taps()
    st = pair.engine.new_state()
    osts = []
    for b in range(3):
        prompt = synth.make_token_ids(20 + 37 * b, cfg["vocab"], seed=70 + b).numpy()
        ost = orc.prefill(cfg, pair.W, prompt, capacity=pair.kv_capacity)
        ost["flag"] = flags[b]
        H.round_oracle_kv(ost, BF16)
        H.upload_sequence(st, b, ost, BF16)
        osts.append(ost)
    outs = [pair.oracle_step(ost) for ost in osts]
    pair.engine.verify_step(st, 3)
    torch.cuda.synchronize()
    assert int(st.status[0]) == 0
    worst = 0.0
    for b, (ost, out) in enumerate(zip(osts, outs)):
        rep = H.compare_step(cfg, out, st, taps, b, pair.T, BF16, ost, tol=H.TOL_BF16_TINY)
        worst = max(worst, rep.max_logit_err)
        assert not rep.failures, f"flags {flags}, seq {b}: " + "; ".join(rep.failures)
    say(f"  flags {flags}, {sum(o['T'] for o in outs)} rows of 576: worst logits err {worst:.2e}")
    pair.engine.close()


# ---------------------------------------------------------------------------------------------
# full size: the 7B and 13B shapes in the launch configurations bench.py times (bf16, prefix 1024 /
# 2048).  The oracle runs the WHOLE candidate tree (a 64-node 7B step takes it a few seconds), so
# every row's logits, hidden state and argmax, the forced depth-4 acceptance and its compaction in
# every layer, the gate, all heads' logits and the candidates are compared.
# ---------------------------------------------------------------------------------------------
@pytest.fixture(scope="module")
def pair_7b():
    say("7B: building weights and engine")
    return H.Pair("7b", BF16, "p63", seed=0, max_batch=1, kv_capacity=1280, lazy_host=True)


@pytest.mark.parametrize("gemm_fused", [1, 0])
def test_7b_full_size_whole_tree_matches_oracle(pair_7b, gemm_fused):
    """The headline configuration, with the whole-K fused QKV / gate-up launches (the default for up to 64
    rows) and with the split-K GEMMs and separate RoPE / SwiGLU launches."""
    pair_7b.engine.set_param("gemm_fused", gemm_fused)
    try:
        _full_size_step(pair_7b, 1024, 1280)
    finally:
        pair_7b.engine.set_param("gemm_fused", 1)


def test_7b_120_path_tree_whole_tree_matches_oracle(pair_7b):
    """The tree size of the paper's main table (Section 5.1: 120 paths, top-10 per head): 121 nodes,
    so two 64-row blocks in every GEMM, two query blocks and two tree chunks in attention, two mask
    words per node."""
    pair = H.Pair("7b", BF16, "p120", max_batch=1, kv_capacity=1280, share=pair_7b, topk=10)
    assert pair.T == 121 and max(pair.rank) < 10
    _full_size_step(pair, 1024, 1280)
    pair.engine.close()


def test_7b_150_path_tree_whole_tree_matches_oracle(pair_7b):
    """The largest tree of Section 5.1 (150 paths): 151 nodes, three row blocks, three mask words."""
    pair = H.Pair("7b", BF16, "p150", max_batch=1, kv_capacity=1280, share=pair_7b, topk=10)
    assert pair.T == 151
    _full_size_step(pair, 1024, 1280)
    pair.engine.close()


def test_7b_step_is_bitwise_reproducible(pair_7b):
    """Split-K partials are summed in a fixed order and nothing uses atomics on floats, so the same
    state gives the same bits: logits of all 64 nodes, hidden states, candidates, entropy, on three
    launches of the full-size step (a race between workgroups would show here)."""
    pair = pair_7b
    cfg, cap, L = pair.cfg, pair.kv_capacity, 1024
    taps = pair.taps()
    st = pair.engine.new_state()
    kv0 = synth.make_kv_prefix(cfg, 1, cap, seed=0, dtype=torch.bfloat16, device="cuda")
    cand = synth.make_candidates(cfg, 1, seed=3)[0].cuda()
    root = int(synth.make_token_ids(1, cfg["vocab"], seed=2)[0])
    ref = None
    for rep in range(3):
        st.kv.copy_(kv0)
        st.kv_len[0], st.root_token[0], st.gate_flag[0] = L, root, 0
        st.cand[0] = cand
        pair.engine.verify_step(st, 1)
        torch.cuda.synchronize()
        got = (taps.logits.clone(), taps.h_last.clone(), taps.head_logits.clone(), st.cand.clone(), st.entropy.clone(),
               st.kv[:, :, :, :, L:L + 8].clone())
        if ref is None:
            ref = got
        else:
            for a, b in zip(ref, got):
                assert torch.equal(a, b), rep
    assert int(st.status[0]) == 0


def test_7b_ar_step_reached_through_the_gate_matches_oracle(pair_7b):
    """A sequence whose gate flag says auto-regressive, run by cerberus_verify_step: the launches are
    sized for the whole tree but carry one row (the kernels' paths for partly filled row tiles).
    Nothing forced: logits, argmax, committed token, cache row, gate and the heads' candidates for the
    next step against the oracle's one-row step."""
    pair = pair_7b
    cfg, cap, L, tol = pair.cfg, pair.kv_capacity, 1024, H.TOL_BF16
    taps = pair.taps()
    st = pair.engine.new_state()
    st.kv.copy_(synth.make_kv_prefix(cfg, 1, cap, seed=0, dtype=torch.bfloat16, device="cuda"))
    root = int(synth.make_token_ids(1, cfg["vocab"], seed=2)[0])
    cand = synth.make_candidates(cfg, 1, seed=3)[0]
    st.kv_len[0], st.root_token[0], st.gate_flag[0] = L, root, 1
    st.cand[0] = cand.cuda()
    kv_host = [(st.kv[l, 0, 0].double().cpu().numpy(), st.kv[l, 1, 0].double().cpu().numpy()) for l in range(cfg["n_layers"])]
    pair.engine.verify_step(st, 1)
    torch.cuda.synchronize()
    ost = orc.new_state(kv_host, L, root, cand.numpy(), 1)
    out = orc.verify_step(cfg, pair.W, pair.parent, pair.rank, ost)
    assert out["T"] == 1
    rep = H.compare_step(cfg, out, st, taps, 0, pair.T, BF16, ost, tol=tol)
    say(f"7B AR step through the gate: logits err {rep.max_logit_err:.3e}, h_last err {rep.max_hidden_err:.3e}, "
        f"head logits err {rep.max_head_logit_err:.3e}, entropy err {rep.entropy_err:.2e}, candidates {rep.cand_checked} checked")
    assert not rep.failures, "; ".join(rep.failures)
    assert rep.accept_checked and rep.flag_checked and rep.cand_checked > 0


def test_13b_full_size_whole_tree_matches_oracle():
    """configs[3]: 40 layers, d 5120, 40 heads, FFN 13824, five decoding heads, prefix 2048."""
    say("13B: building weights and engine")
    pair = H.Pair("13b", BF16, "p63", seed=0, max_batch=1, kv_capacity=2304, lazy_host=True)
    _full_size_step(pair, 2048, 2304)
    pair.engine.close()


def _deepest_path(pair):
    """Root-to-leaf node list ending in the deepest leaf with the largest index."""
    depth, _ = orc.tree_tables(pair.parent)
    leaf = max(n for n in range(pair.T) if depth[n] == max(depth))
    nodes = []
    n = leaf
    while n >= 0:
        nodes.append(n)
        n = pair.parent[n]
    return nodes[::-1]


def _full_size_step(pair, L, cap):
    cfg, T, tol = pair.cfg, pair.T, H.TOL_BF16
    tag = f"{cfg['n_layers']}x{cfg['d_model']} T={T}"
    st = pair.engine.new_state()
    st.kv.copy_(synth.make_kv_prefix(cfg, 1, cap, seed=0, dtype=torch.bfloat16, device="cuda"))
    root = int(synth.make_token_ids(1, cfg["vocab"], seed=2)[0])
    cand = synth.make_candidates(cfg, 1, seed=3)[0]
    st.kv_len[0], st.root_token[0], st.gate_flag[0] = L, root, 0
    st.cand[0] = cand.cuda()

    # force the acceptance down the deepest path on both sides (random-init heads never get a
    # candidate accepted), so that a full-depth commit and its compaction are exercised at full
    # size; 777 is the (forced) next root, -1 (no token) everywhere off the path
    nodes = _deepest_path(pair)
    taps = pair.taps(forced_argmax=True)
    tok_full = orc.tree_tokens(root, cand.numpy(), pair.parent, pair.rank)
    forced = np.full(T, -1, dtype=np.int64)
    for j, n in enumerate(nodes):
        forced[n] = int(tok_full[nodes[j + 1]]) if j + 1 < len(nodes) else 777
    taps.forced_node_argmax.copy_(torch.from_numpy(forced).to(torch.int32).cuda())

    kv_before = st.kv.clone()
    pair.engine.verify_step(st, 1)
    torch.cuda.synchronize()
    assert int(st.status[0]) == 0
    say(tag + ": device step done; running the oracle on the whole tree")

    kv_host = [(kv_before[l, 0, 0].double().cpu().numpy(), kv_before[l, 1, 0].double().cpu().numpy())
               for l in range(cfg["n_layers"])]
    W_lazy = pair.W
    W_lazy["layers"]._on_access = lambda l: say(f"  oracle layer {l}") if l % 8 == 0 else None
    ost = orc.new_state(kv_host, L, root, cand.numpy(), 0)
    out = orc.verify_step(cfg, W_lazy, pair.parent, pair.rank, ost, forced_node_argmax=forced)
    assert out["T"] == T and out["path"] == nodes

    rep = H.compare_step(cfg, out, st, taps, 0, T, BF16, ost, forced_argmax=True, tol=tol)
    say(f"{tag}: all {T} rows: logits max-abs err {rep.max_logit_err:.3e} (std of logits {out['logits'].std():.3f}), h_last err "
        f"{rep.max_hidden_err:.3e}, real argmax checked {rep.argmax_checked}/{T}, entropy err {rep.entropy_err:.2e}, head logits err "
        f"{rep.max_head_logit_err:.3e}, candidates checked {rep.cand_checked}/{rep.cand_checked + rep.cand_skipped}")
    assert not rep.failures, "; ".join(rep.failures)
    assert rep.accept_checked and rep.flag_checked and rep.cand_checked > 0 and rep.argmax_checked > T // 2
    assert int(st.accept_len[0]) == len(nodes) and int(st.root_token[0]) == 777
    assert torch.equal(st.kv[:, :, :, :, :L], kv_before[:, :, :, :, :L])       # committed rows untouched


# ---------------------------------------------------------------------------------------------
# The widened rows at full size: independent heads, the multi-step driver, the prompt phase.
# ---------------------------------------------------------------------------------------------
def test_7b_independent_heads_step_matches_oracle(pair_7b):
    """special_block = -1 at the 7B shape: four d-wide heads over the shared base model.  The step
    runs the whole tree; the acceptance is forced to stop at the root on both sides, so the oracle
    needs the root's row only (a tree of size 1 gives the same row 0 as any tree pass) and then
    runs its heads on that row's hidden state."""
    pair = H.Pair("7b", BF16, "p63", max_batch=1, kv_capacity=1280, share=pair_7b, heads_seed=9, special_block=-1)
    cfg, T, L, tol = pair.cfg, pair.T, 1024, H.TOL_BF16
    assert all(w == cfg["d_model"] for ws in synth.head_block_widths(cfg) for w in ws)
    st = pair.engine.new_state()
    st.kv.copy_(synth.make_kv_prefix(cfg, 1, pair.kv_capacity, seed=0, dtype=torch.bfloat16, device="cuda"))
    root = int(synth.make_token_ids(1, cfg["vocab"], seed=2)[0])
    cand = synth.make_candidates(cfg, 1, seed=3)[0]
    st.kv_len[0], st.root_token[0], st.gate_flag[0] = L, root, 0
    st.cand[0] = cand.cuda()
    taps = pair.taps(forced_argmax=True)
    forced = np.full(T, -1, dtype=np.int64)
    forced[0] = 777                                   # no child carries it: the walk stops at the root
    taps.forced_node_argmax.copy_(torch.from_numpy(forced).to(torch.int32).cuda())
    kv_host = [(st.kv[l, 0, 0].double().cpu().numpy(), st.kv[l, 1, 0].double().cpu().numpy()) for l in range(cfg["n_layers"])]
    pair.engine.verify_step(st, 1)
    torch.cuda.synchronize()
    ost = orc.new_state(kv_host, L, root, cand.numpy(), 0)
    out = orc.verify_step(cfg, pair.W, [-1], [0], ost, forced_node_argmax=forced[:1])
    rep = H.compare_step(cfg, out, st, taps, 0, T, BF16, ost, forced_argmax=True, tol=tol)
    say(f"7B independent heads: logits err {rep.max_logit_err:.3e}, head logits err {rep.max_head_logit_err:.3e}, "
        f"candidates checked {rep.cand_checked}/{rep.cand_checked + rep.cand_skipped}")
    assert not rep.failures, "; ".join(rep.failures)
    assert rep.accept_checked and rep.flag_checked and rep.cand_checked > 0
    pair.engine.close()


def test_7b_decode_two_chained_steps_match_oracle(pair_7b):
    """cerberus_decode at the 7B shape, nothing forced: two steps enqueued in one call, the second
    one drafted by the first one's heads.  The oracle runs the same two whole-tree steps; the token
    log is compared up to the first decision whose margin is within the tolerance, and the second
    step's rows (the taps hold the last step's) are compared like any single step."""
    pair = pair_7b
    cfg, T, L, tol = pair.cfg, pair.T, 1024, H.TOL_BF16
    taps = pair.taps()
    st = pair.engine.new_state()
    st.kv.copy_(synth.make_kv_prefix(cfg, 1, pair.kv_capacity, seed=0, dtype=torch.bfloat16, device="cuda"))
    root = int(synth.make_token_ids(1, cfg["vocab"], seed=2)[0])
    cand = synth.make_candidates(cfg, 1, seed=3)[0]
    st.kv_len[0], st.root_token[0], st.gate_flag[0] = L, root, 0
    st.cand[0] = cand.cuda()
    kv_host = [(st.kv[l, 0, 0].double().cpu().numpy(), st.kv[l, 1, 0].double().cpu().numpy()) for l in range(cfg["n_layers"])]
    log = torch.full((1, 16), -1, dtype=torch.int32, device="cuda")
    count = torch.zeros(1, dtype=torch.int32, device="cuda")
    pair.engine.decode(st, 1, 2, log, count)
    torch.cuda.synchronize()
    assert int(st.status[0]) == 0
    got = log[0, :int(count[0])].cpu().tolist()
    assert int(st.kv_len[0]) == L + len(got)

    ost = orc.new_state(kv_host, L, root, cand.numpy(), 0)
    depth, _ = orc.tree_tables(pair.parent)
    want, clear = [], True
    for step in range(2):
        if step == 1:                                # the device's second step read bf16 cache rows
            H.round_oracle_kv(ost, BF16)
        out = orc.verify_step(cfg, pair.W, pair.parent, pair.rank, ost)
        srt = -np.sort(-out["logits"][out["path"]], axis=1)
        margin = float(np.min(srt[:, 0] - srt[:, 1]))
        say(f"  7B decode step {step}: accept {out['accept_len']}, argmax margin {margin:.2e}")
        if margin <= 2 * tol.logits:
            clear = False
            break
        want += [int(t) for t in out["committed"]]
        if step == 0:
            # The second step's tree carries the first step's candidates.  Where two head logits of the
            # oracle lie within the tolerance their order is not decided, so the device's own choice is
            # read back from its second step's node tokens, checked wherever the margin is clear, and
            # the oracle continues from it.
            tok2 = taps.node_token[:T].cpu().numpy()
            assert int(tok2[0]) == out["root"]
            cand_dev = np.array(ost["cand"])
            checked = 0
            for n in range(1, T):
                i, j = depth[n] - 1, pair.rank[n]
                s_i = -np.sort(-out["head_logits"][i])[:cfg["topk"] + 1]
                if H._margin_ok(s_i, j, tol.logits):
                    checked += 1
                    assert int(tok2[n]) == int(ost["cand"][i, j]), (n, i, j)
                cand_dev[i, j] = int(tok2[n])
            say(f"  7B decode: {checked}/{T - 1} tree tokens of the second step checked against the oracle's candidates")
            assert checked > 0
            ost["cand"] = cand_dev
    assert got[:len(want)] == want and len(want) >= 1
    if clear:
        assert len(got) == len(want)
        rep = H.compare_step(cfg, out, st, taps, 0, T, BF16, ost, tol=tol)
        say(f"  7B decode, second step: logits err {rep.max_logit_err:.3e}, head logits err {rep.max_head_logit_err:.3e}")
        assert not rep.failures, "; ".join(rep.failures)
    else:
        say("  7B decode: an argmax of the committed path sits within the tolerance; compared the log up to it")


def test_7b_prefill_two_passes_matches_oracle(pair_7b):
    """cerberus_prefill at the 7B shape: 230 prompt tokens from an empty cache (a pass of 192 rows and
    one of 38), against the oracle's one-shot causal prefill: cache rows, the last pass's logits and
    hidden states, pending token, gate, the heads' logits and candidates."""
    pair = pair_7b
    cfg, T, tol, n_prompt = pair.cfg, pair.T, H.TOL_BF16, 230
    taps = pair.taps()
    prompt = synth.make_token_ids(n_prompt, cfg["vocab"], seed=21)
    st = pair.engine.new_state()
    st.kv_len[0] = 0
    st.gate_flag[0] = 1
    pair.engine.prefill(st, 1, 0, prompt.cuda())
    torch.cuda.synchronize()
    assert int(st.status[0]) == 0 and int(st.kv_len[0]) == n_prompt
    # The oracle takes the same two passes, its cache rounded to bf16 between them: the device's
    # second pass reads the first pass's rows from the bf16 cache, and the storage type of the cache
    # is part of the configuration, not an error of the path (that passes and a one-shot forward
    # agree is pinned on the oracle itself).
    say("7B prefill: device done; oracle's causal forward over 192 + 38 rows")
    P = B.CERBERUS_MAX_TREE
    ost = {"kv": orc.new_kv(cfg, n_prompt)}
    kv = ost["kv"]
    hs, ls = [], []
    for off in range(0, n_prompt, P):
        n = min(P, n_prompt - off)
        h_p, l_p = orc.decoder_rows(cfg, pair.W, prompt.numpy()[off:off + n], np.arange(off, off + n),
                                    np.tril(np.ones((n, n), dtype=bool)), kv, off)
        hs.append(h_p)
        ls.append(l_p)
        if off + n < n_prompt:
            H.round_oracle_kv(ost, BF16)
            kv = ost["kv"]
    h_last, logits = np.concatenate(hs), np.concatenate(ls)
    for l in (0, cfg["n_layers"] // 2, cfg["n_layers"] - 1):
        for kvi in (0, 1):
            got = st.kv[l, kvi, 0, :, :n_prompt].double().cpu().numpy()
            want = kv[l][kvi][:, :n_prompt]
            mm = H.kv_mismatch(got, want, tol)
            assert mm is None, (l, kvi, mm)
    n_last = n_prompt % P or P
    k, first = min(n_last, T), n_prompt - n_last
    err = float(np.max(np.abs(taps.logits[:k].double().cpu().numpy() - logits[first:first + k])))
    herr = float(np.max(np.abs(taps.h_last[:k].double().cpu().numpy() - h_last[first:first + k])))
    say(f"7B prefill: last pass of {n_last} rows, {k} tapped: logits err {err:.3e}, h_last err {herr:.3e}")
    assert err <= tol.logits and herr <= tol.hidden
    srt = -np.sort(-logits[-1])
    if srt[0] - srt[1] > 2 * tol.logits:
        assert int(st.root_token[0]) == int(orc.argmax_lowest(logits[-1]))
    S, flag = orc.gate(h_last[-1], cfg["entropy_threshold"])
    assert abs(float(st.entropy[0]) - S) <= tol.entropy and int(st.gate_flag[0]) == flag == 0
    want_hl = np.stack(orc.cerberus_heads(cfg, pair.W["heads"], h_last[-1]))
    hl = taps.head_logits[0].double().cpu().numpy()
    herr2 = float(np.max(np.abs(hl - want_hl)))
    say(f"7B prefill: head logits err {herr2:.3e}")
    assert herr2 <= tol.logits
    checked = 0
    for i in range(cfg["n_cerb_heads"]):
        srt_i = -np.sort(-want_hl[i])[:cfg["topk"] + 1]
        ids = orc.topk_ids(want_hl[i], cfg["topk"])
        for j in range(cfg["topk"]):
            if H._margin_ok(srt_i, j, tol.logits):
                checked += 1
                assert int(st.cand[0, i, j]) == int(ids[j]), (i, j)
    assert checked > 0


# ---------------------------------------------------------------------------------------------
# configs[2]: 256 consecutive steps at the 7B shape with the gate active.  The oracle cannot run
# 256 full-size steps, so the schedule is driven through the taps (forced gate input, forced
# per-node argmax) and everything that is decided by small integer logic is checked against the
# oracle's own functions on the same forced inputs: the gate decision of every step, the tree size
# each step ran with, accepted path, committed tokens, next root and the growth of the cache length.
# ---------------------------------------------------------------------------------------------
def test_7b_gated_256_step_schedule(pair_7b):
    L0, cap, n_steps, thr = 1024, 2560, 256, 9.0
    pair = H.Pair("7b", BF16, "p63", max_batch=1, kv_capacity=cap, share=pair_7b, entropy_threshold=thr)
    cfg, T, Hc = pair.cfg, pair.T, pair.cfg["n_cerb_heads"]
    d = cfg["d_model"]
    taps = pair.taps(logits=False, forced_argmax=True, forced_gate=True)
    st = pair.engine.new_state()
    st.kv.copy_(synth.make_kv_prefix(cfg, 1, cap, seed=0, dtype=torch.bfloat16, device="cuda"))
    st.kv_len[0] = L0
    st.root_token[0] = int(synth.make_token_ids(1, cfg["vocab"], seed=2)[0])
    st.cand[0] = synth.make_candidates(cfg, 1, seed=3)[0].cuda()
    st.gate_flag[0] = 0
    rng = np.random.default_rng(11)
    z = synth.make_gate_states(n_steps, d, seed=5, lo=1.0, hi=1.0).numpy()       # unit-scale states
    depth, _ = orc.tree_tables(pair.parent)
    children = {n: [c for c in range(T) if pair.parent[c] == n] for n in range(T)}
    L, flag = L0, 0
    n_ar = n_tree = committed = 0
    for step in range(n_steps):
        ar_next = rng.random() < 0.3                    # ~30 % of the steps hand over to an AR step
        alpha = 0.5 if ar_next else 3.0                 # entropy ~11.8 bits vs ~5.5 bits around T = 9
        hidden = (alpha * z[step]).astype(np.float32)
        S_want, flag_want = orc.gate(hidden, thr)
        assert flag_want == int(ar_next)
        a_want = int(rng.integers(1, Hc + 2))           # accepted length drawn uniformly from 1..Hc+1
        T_step = 1 if flag else T
        # plant a path of that depth in the forced argmax (clipped to what this step's tree has)
        tok = taps.node_token                           # filled by the step itself; read after the step
        path = [0]
        while len(path) < a_want and T_step > 1 and children[path[-1]]:
            path.append(int(rng.choice(children[path[-1]])))
        # the forced argmax needs the node tokens, which depend only on state known before the step
        cand_now = st.cand[0].cpu().numpy()
        root_now = int(st.root_token[0])
        tok_now = orc.tree_tokens(root_now, cand_now, pair.parent if T_step > 1 else [-1], pair.rank if T_step > 1 else [0])
        forced = np.full(T, -1, dtype=np.int64)
        for j, n in enumerate(path):
            forced[n] = tok_now[path[j + 1]] if j + 1 < len(path) else (1000 + step) % cfg["vocab"]
        # a forced token may collide with a sibling's token; the oracle's walk is the arbiter
        want_path = orc.accept_path(forced[:T_step], tok_now, (pair.parent if T_step > 1 else [-1]))
        taps.forced_node_argmax.copy_(torch.from_numpy(forced).to(torch.int32).cuda())
        taps.forced_gate_hidden[0] = torch.from_numpy(hidden).cuda()
        pair.engine.verify_step(st, 1)
        torch.cuda.synchronize()
        a = int(st.accept_len[0])
        assert taps.node_token[:T_step].cpu().numpy().tolist() == tok_now.tolist(), step
        assert st.accepted_nodes[0, :a].cpu().tolist() == want_path, (step, want_path)
        assert st.accepted_tokens[0, :a].cpu().tolist() == [int(tok_now[n]) for n in want_path]
        assert int(st.root_token[0]) == int(forced[want_path[-1]])
        L += len(want_path)
        assert int(st.kv_len[0]) == L
        assert abs(float(st.entropy[0]) - S_want) < 1e-3 and int(st.gate_flag[0]) == flag_want, step
        n_ar += T_step == 1
        n_tree += T_step > 1
        committed += a
        flag = flag_want
    assert int(st.status[0]) == 0 and L <= cap - T
    say(f"7B schedule: {n_tree} tree steps, {n_ar} AR steps, {committed} tokens committed, final L {L}")
    assert n_ar > 40 and n_tree > 120
    pair.engine.close()


# ---------------------------------------------------------------------------------------------
# configs[4]: eight independent 7B-shape sequences, prefixes drawn from 512..4096, per-sequence
# gate decisions drawn Bernoulli(0.3), one launch.  For every one of the eight sequences the oracle
# runs one root-to-leaf path of a tree sequence as a chain tree (a node's result depends only on the
# prefix and its ancestors, so the chain's rows must equal those rows of the full tree pass), or the
# single row of an auto-regressive one.
# ---------------------------------------------------------------------------------------------
def test_7b_batch8_mixed_launch(pair_7b):
    Bn, cap = 8, 4224
    pair = H.Pair("7b", BF16, "p63", max_batch=Bn, kv_capacity=cap, share=pair_7b)
    cfg, T, tol = pair.cfg, pair.T, H.TOL_BF16
    rng = np.random.default_rng(21)
    Ls = rng.integers(512, 4097, size=Bn)
    flags = (rng.random(Bn) < 0.3).astype(np.int32)
    flags[0], flags[1] = 0, 1                       # at least one of each kind
    st = pair.engine.new_state()
    st.kv.copy_(synth.make_kv_prefix(cfg, Bn, cap, seed=4, dtype=torch.bfloat16, device="cuda"))
    roots = synth.make_token_ids(Bn, cfg["vocab"], seed=6)
    cands = synth.make_candidates(cfg, Bn, seed=7)
    st.kv_len.copy_(torch.from_numpy(Ls.astype(np.int32)).cuda())
    st.root_token.copy_(roots.cuda())
    st.cand.copy_(cands.cuda())
    st.gate_flag.copy_(torch.from_numpy(flags).cuda())
    taps = pair.taps()
    pair.engine.verify_step(st, Bn)
    torch.cuda.synchronize()
    assert int(st.status[0]) == 0
    rows = int(np.sum(np.where(flags == 1, 1, T)))
    say(f"7B batch 8: prefixes {Ls.tolist()} (sum {int(Ls.sum())}), flags {flags.tolist()}, {rows} packed rows")
    # a different root-to-leaf path per tree sequence: the leaves in turn, deepest first
    depth, _ = orc.tree_tables(pair.parent)
    leaves = sorted((n for n in range(T) if n not in set(pair.parent)), key=lambda n: (-depth[n], -n))
    worst = 0.0
    for b in range(Bn):
        nodes = []
        n = leaves[(5 * b) % len(leaves)] if flags[b] == 0 else 0
        while n >= 0:
            nodes.append(n)
            n = pair.parent[n]
        nodes.reverse()
        chain_parent = [-1] + list(range(len(nodes) - 1))
        chain_rank = [pair.rank[n] for n in nodes]
        Lb = int(Ls[b])
        kv_host = []
        for l in range(cfg["n_layers"]):              # the step leaves the committed rows 0..L-1 as they were
            K = np.zeros((cfg["n_heads"], Lb + len(nodes), cfg["head_dim"]))
            V = np.zeros_like(K)
            K[:, :Lb] = st.kv[l, 0, b, :, :Lb].double().cpu().numpy()
            V[:, :Lb] = st.kv[l, 1, b, :, :Lb].double().cpu().numpy()
            kv_host.append((K, V))
        ost = orc.new_state(kv_host, Lb, int(roots[b]), cands[b].numpy(), 0)
        out = orc.verify_step(cfg, pair.W, chain_parent, chain_rank, ost)
        idx = torch.tensor([b * T + n for n in nodes])
        assert np.array_equal(taps.node_token[idx].cpu().numpy(), out["tok"])
        err = float(np.max(np.abs(taps.logits[idx].double().cpu().numpy() - out["logits"])))
        herr = float(np.max(np.abs(taps.h_last[idx].double().cpu().numpy() - out["h_last"])))
        worst = max(worst, err)
        say(f"7B batch 8 seq {b} (L={Lb}, flag={flags[b]}): logits max-abs err {err:.3e}, h_last err {herr:.3e} on nodes {nodes}")
        assert err <= tol.logits and herr <= tol.hidden
        srt = -np.sort(-out["logits"], axis=1)
        safe = (srt[:, 0] - srt[:, 1]) > 2 * tol.logits
        assert np.array_equal(taps.node_argmax[idx].cpu().numpy()[safe], np.argmax(out["logits"], axis=1)[safe])
        # random candidates never match the model's own token: only the root is accepted
        if safe[0]:
            assert int(st.accept_len[b]) == 1 == out["accept_len"]
            assert int(st.kv_len[b]) == Lb + 1 and int(st.root_token[b]) == out["root"]
            assert abs(float(st.entropy[b]) - out["entropy"]) <= tol.entropy
            # the committed row of every layer
            for l in (0, cfg["n_layers"] // 2, cfg["n_layers"] - 1):
                for kvi in (0, 1):
                    got = st.kv[l, kvi, b, :, Lb].double().cpu().numpy()
                    want = ost["kv"][l][kvi][:, Lb]
                    mm = H.kv_mismatch(got, want, tol)
                    assert mm is None, (b, l, kvi, mm)
    say(f"7B batch 8: all {Bn} sequences compared, worst logits err {worst:.3e}")
    pair.engine.close()
