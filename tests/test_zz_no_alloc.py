"""The allocation-free acceptance entry point against cerberus_accept, through the C ABI."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import cerberus_oracle as orc
from paper_2410_13344_amd import binding as B
from tests import harness as H


def _run(pair, entry, kv, L, gg, tk, batch):
    """One call of `entry` on a fresh state holding `kv`, lengths L, per-node arrays gg / tk."""
    st = pair.engine.new_state()
    st.kv.copy_(kv)
    st.kv_len[:batch] = torch.tensor(L, dtype=torch.int32).cuda()
    entry(pair.engine.ctx, gg.cuda(), tk.cuda(), st.struct, batch)
    torch.cuda.synchronize()
    return st


def _same(a, b, batch):
    for k in ("accept_len", "accepted_tokens", "accepted_nodes", "root_token", "kv_len", "status"):
        x, y = getattr(a, k), getattr(b, k)
        assert torch.equal(x[:batch] if x.shape[0] >= batch and k != "status" else x, y[:batch] if y.shape[0] >= batch and k != "status" else y), k
    assert torch.equal(a.kv, b.kv)


@pytest.mark.parametrize("dtype", [B.CERBERUS_F32, B.CERBERUS_BF16])
def test_accept_noalloc_equals_accept_on_two_calls_in_a_row(dtype):
    pair = H.Pair("tiny", dtype, "tiny", seed=0, max_batch=3, kv_capacity=256)
    cfg, T = pair.cfg, pair.T
    g = torch.Generator().manual_seed(11)
    kv = torch.randn(pair.engine.new_state().kv.shape, generator=g).to(H.torch_dtype(dtype)).cuda()
    tok = torch.arange(100, 100 + 3 * T, dtype=torch.int32)
    chains = [{0: 2, 2: 7, 7: 14}, {0: 1, 1: 5, 5: 12, 12: 15}, {}]     # per sequence: node -> accepted child
    gg = torch.full((3 * T,), -1, dtype=torch.int32)
    for b, chain in enumerate(chains):
        for a, c in chain.items():
            gg[b * T + a] = tok[b * T + c]
    # first call: three sequences; second call, right after it on the same GPU: one sequence (a smaller
    # input over an array that still holds the first call's contents)
    for batch, L in ((3, [37, 90, 5]), (1, [64])):
        ref = _run(pair, B.cerberus_accept, kv, L, gg, tok, batch)
        got = _run(pair, B.cerberus_accept_noalloc, kv, L, gg, tok, batch)
        _same(got, ref, batch)
        assert int(got.status[0]) == 0
        for b in range(batch):                     # and both agree with the oracle's walk
            want = orc.accept_path(gg[b * T:(b + 1) * T].numpy(), tok[b * T:(b + 1) * T].numpy(), pair.parent)
            a = int(got.accept_len[b])
            assert got.accepted_nodes[b, :a].cpu().tolist() == want, (batch, b)
    # a sequence that does not fit sits the call out; the others still read their own rows b*T..
    L = [256 - 3, 40, 7]
    ref = _run(pair, B.cerberus_accept, kv, L, gg, tok, 3)
    got = _run(pair, B.cerberus_accept_noalloc, kv, L, gg, tok, 3)
    _same(got, ref, 3)
    assert int(got.status[0]) & B.CERBERUS_DEV_KV_OVERFLOW and int(got.accept_len[0]) == 0
    for b in (1, 2):
        want = orc.accept_path(gg[b * T:(b + 1) * T].numpy(), tok[b * T:(b + 1) * T].numpy(), pair.parent)
        a = int(got.accept_len[b])
        assert got.accepted_nodes[b, :a].cpu().tolist() == want, b
        assert int(got.kv_len[b]) == L[b] + a
    pair.engine.close()


def test_accept_noalloc_rejects_what_does_not_fit():
    """1024 tree rows in all is the limit of the static array: 16 sequences of a 65-node tree are 1040."""
    pair = H.Pair("tiny", B.CERBERUS_F32, "rand65s3k4", seed=0, max_batch=16, kv_capacity=128)
    st = pair.engine.new_state()
    z = torch.zeros(16 * pair.T, dtype=torch.int32, device="cuda")
    with pytest.raises(B.CerberusError) as e:
        B.cerberus_accept_noalloc(pair.engine.ctx, z, z, st.struct, 16)
    assert e.value.code == -3 and "1024" in str(e.value)
    B.cerberus_accept_noalloc(pair.engine.ctx, z, z, st.struct, 15)       # 975 rows fit
    torch.cuda.synchronize()
    pair.engine.close()
