"""lc_decode_step_static (the decode step on the library's own static scratch array, for callers
that cannot allocate) against lc_decode_step, through the C ABI: two calls in a row, the second on
a smaller input, then the size limit."""
import numpy as np
import pytest

import lc_workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2603_08453_amd import binding as lc
    lc.lib()
    from tests import gpu_common
    return gpu_common


def _both(G, case, qb, budget):
    """(ids, out, lse) of lc_decode_step and of lc_decode_step_static on the same inputs."""
    import torch
    from paper_2603_08453_amd import binding as lc
    w = case.w
    q = G.to_bf16_tensor(qb)
    res = []
    for static in (False, True):
        ids = torch.full((w.B, w.H_kv, case.cap), -1, dtype=torch.int32, device="cuda")
        counts = torch.full((w.B, w.H_kv), -1, dtype=torch.int32, device="cuda")
        out = torch.full((w.B, w.H_q, w.d), float("nan"), dtype=torch.float32, device="cuda")
        lse = torch.full((w.B, w.H_q), float("nan"), dtype=torch.float32, device="cuda")
        if static:
            lc.lc_decode_step_static(case.idx, q, case.K, case.V, budget, out, lse=lse, chunk_ids=ids, counts=counts)
        else:
            lc.lc_decode_step(case.idx, q, case.K, case.V, budget, out, case.ws, lse=lse, chunk_ids=ids, counts=counts)
        torch.cuda.synchronize()
        ih, ch = ids.cpu().numpy(), counts.cpu().numpy()
        res.append(([[ih[b, h, : ch[b, h]].copy() for h in range(w.H_kv)] for b in range(w.B)],
                    out.cpu().numpy(), lse.cpu().numpy()))
    return res


def _check_same(G, case, qb, budget, tag):
    from oracle import lychee_oracle as orc
    from tests import helpers as H
    w = case.w
    (ids_a, out_a, lse_a), (ids_s, out_s, lse_s) = _both(G, case, qb, budget)
    for b in range(w.B):
        for h in range(w.H_kv):
            assert ids_s[b][h].tolist() == ids_a[b][h].tolist(), (tag, b, h)
            # and both against the oracle, so that the comparison cannot pass on two wrong answers
            oi = case.oidx[b][h]
            q = wl.bf16_bits_to_f64(qb[b, h * w.G:(h + 1) * w.G])
            H.accept_ids(ids_s[b][h], orc.node_scores(oi, 0, q), oi.lens(), budget)
            ref, ref_lse = orc.sparse_decode(q, case.Kf(b, h), case.Vf(b, h), oi.bounds, oi.T, ids_s[b][h])
            mx, rel = G.attention_errors(out_s[b, h * w.G:(h + 1) * w.G], ref)
            assert mx <= 1e-2 and rel <= 2e-3, (tag, b, h, mx, rel)
    mx, rel = G.attention_errors(out_s, out_a.astype(np.float64))
    assert mx <= 1e-2 and rel <= 2e-3, (tag, mx, rel)
    fin = np.isfinite(lse_a)
    assert np.array_equal(fin, np.isfinite(lse_s)), tag
    assert np.allclose(lse_s[fin], lse_a[fin], atol=1e-3), tag


def test_static_scratch_step_equals_the_workspace_step(G):
    from paper_2603_08453_amd import binding as lc
    assert lc.lc_static_workspace_bytes() == 16 << 20
    # first call: two ragged sequences, four levels deep walk, an open tail
    w1 = wl.tiny("na-big", B=2, H_q=8, H_kv=2, levels=3, fanout=6, T=6000, chunk_lo=8, chunk_hi=48, budget=900)
    c1 = G.make_case(w1, tails=[5, 0], extra_tokens=4, extra_chunks=4)
    assert 0 < lc.lc_decode_workspace_bytes(c1.cfg, w1.B, w1.H_q, w1.H_kv) <= lc.lc_static_workspace_bytes()
    q1 = np.stack([s.Q[0] for s in c1.seqs])
    _check_same(G, c1, q1, w1.budget, "first call")
    # second call, right behind it, on a smaller input: whatever the first call left in the array must not matter
    w2 = wl.tiny("na-small", B=1, H_q=4, H_kv=1, levels=2, fanout=4, T=700, chunk_lo=4, chunk_hi=20, budget=128)
    c2 = G.make_case(w2, tails=[2], extra_tokens=4, extra_chunks=4)
    q2 = np.stack([s.Q[0] for s in c2.seqs])
    _check_same(G, c2, q2, w2.budget, "second, smaller call")
    # and the first input once more
    _check_same(G, c1, q1, w1.budget, "third call")


def test_static_scratch_step_rejects_what_does_not_fit(G):
    """A configuration whose decode workspace exceeds the array is refused before anything is enqueued."""
    import torch
    from paper_2603_08453_amd import binding as lc
    w = wl.tiny("na-cap", B=4, H_q=16, H_kv=8, levels=2, fanout=4, T=300, chunk_lo=4, chunk_hi=20, budget=64)
    # capacity for 24 thousand chunks in each of 32 (sequence, head) pairs: 25 bytes of step workspace per chunk
    case = G.make_case(w, extra_tokens=24000, extra_chunks=24000)
    assert lc.lc_decode_workspace_bytes(case.cfg, w.B, w.H_q, w.H_kv) > lc.lc_static_workspace_bytes()
    q = G.to_bf16_tensor(np.stack([s.Q[0] for s in case.seqs]))
    out = torch.full((w.B, w.H_q, w.d), 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(lc.LycheeError) as e:
        lc.lc_decode_step_static(case.idx, q, case.K, case.V, w.budget, out)
    assert e.value.code == lc.LC_ERR_CAPACITY
    torch.cuda.synchronize()
    assert float(out.min()) == 7.0 and float(out.max()) == 7.0
