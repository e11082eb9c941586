"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same
seeded inputs and the identical stored index.

Bars (written here, derived in the design notes):
  * chunk-id sets: identical to the oracle's, except that chunks whose oracle score
    lies within 1e-5 (relative, logit units) of the cutoff may differ; ties by lower id.
  * chunk scores: float32 vs float64, |diff| <= 2e-5 * max(1, |score|).
  * attention: bf16 inputs, float32 accumulation: max abs error <= 1e-2 and
    relative L2 error <= 2e-3 against the float64 oracle.
"""
import math
from dataclasses import replace

import numpy as np
import pytest

import lc_workloads as wl
from oracle import lychee_oracle as orc
from tests import helpers as H

pytestmark = pytest.mark.gpu

ATTN_MAX_ABS = 1e-2
ATTN_REL_L2 = 2e-3
SCORE_REL = 2e-5


@pytest.fixture(scope="module")
def G():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from tests import gpu_common
    return gpu_common


def _say(msg):
    print(f"[case] {msg}", flush=True)


def _q_group(case, qi, b, h):
    g = case.w.G
    return wl.bf16_bits_to_f64(case.seqs[b].Q[qi, h * g:(h + 1) * g])


def _q_batch(case, qi):
    return np.stack([s.Q[qi] for s in case.seqs])


def _check_retrieve(G, case, qbits, budget, policy=orc.POLICY_EXACT, beam=None, sink=0, tag=""):
    from paper_2603_08453_amd import binding as lc
    w = case.w
    lc.lc_set_policy(case.idx, policy, beam, sink)
    ids, scores, _ = G.gpu_retrieve(case, qbits, budget)
    for b in range(w.B):
        for h in range(w.H_kv):
            oi = case.oidx[b][h]
            q = wl.bf16_bits_to_f64(qbits[b, h * w.G:(h + 1) * w.G])
            s_ref = orc.node_scores(oi, 0, q)
            pinned = orc.pinned_chunks(oi, sink)
            where = f"{tag} b={b} h={h} budget={budget} policy={policy} sink={sink}"
            if policy == orc.POLICY_EXACT:
                H.accept_ids(ids[b][h], s_ref, oi.lens(), budget, pinned=pinned)
                ref = orc.retrieve_flat(oi, q, budget, sink)
                if len(ref) != len(ids[b][h]) or np.any(ref != ids[b][h]):
                    _say(f"in-band difference at {where}: oracle {len(ref)} ids, gpu {len(ids[b][h])}")
            else:
                st = {}
                ref = orc.retrieve_beam(oi, q, budget, beam, sink, st)
                assert ids[b][h].tolist() == ref.tolist(), where
            # scores: every chunk the GPU scored must agree with the oracle; selected chunks must be scored
            sg = scores[b, h, : oi.M]
            scored = np.isfinite(sg)
            assert np.all(np.abs(sg[scored] - s_ref[scored]) <= SCORE_REL * np.maximum(1.0, np.abs(s_ref[scored]))), where
            free = np.setdiff1d(ids[b][h], pinned)
            assert np.all(scored[free]), where
    return ids


def _check_decode(G, case, qbits, ids_per_bh, tag=""):
    w = case.w
    out, lse = G.gpu_decode(case, qbits, ids_per_bh)
    ref = np.zeros((w.B, w.H_q, w.d))
    ref_lse = np.zeros((w.B, w.H_q))
    for b in range(w.B):
        for h in range(w.H_kv):
            oi = case.oidx[b][h]
            q = wl.bf16_bits_to_f64(qbits[b, h * w.G:(h + 1) * w.G])
            o, l = orc.sparse_decode(q, case.Kf(b, h), case.Vf(b, h), oi.bounds, oi.T, ids_per_bh[b][h])
            ref[b, h * w.G:(h + 1) * w.G] = o
            ref_lse[b, h * w.G:(h + 1) * w.G] = l
    mx, rel = G.attention_errors(out, ref)
    _say(f"{tag}: attention max|err| {mx:.2e}, rel L2 {rel:.2e}")
    assert np.all(np.isfinite(out))
    assert mx <= ATTN_MAX_ABS and rel <= ATTN_REL_L2, (tag, mx, rel)
    fin = np.isfinite(ref_lse)
    assert np.array_equal(fin, np.isfinite(lse))
    assert np.all(lse[~fin] == -np.inf)
    assert np.all(np.abs(lse[fin] - ref_lse[fin]) <= 1e-3), tag
    return out


def _check_step(G, case, qbits, budget, policy=orc.POLICY_EXACT, beam=None, sink=0, tag=""):
    """The fused entry point against the two separate calls: same chunk lists, same attention, bit
    for bit (the separate calls are checked against the oracle by the other helpers)."""
    from paper_2603_08453_amd import binding as lc
    w = case.w
    lc.lc_set_policy(case.idx, policy, beam, sink)
    ids, _, _ = G.gpu_retrieve(case, qbits, budget)
    out, lse = G.gpu_decode(case, qbits, ids)
    ids_f, out_f, lse_f = G.gpu_step(case, qbits, budget)
    where = f"{tag} budget={budget} policy={policy} sink={sink}"
    for b in range(w.B):
        for h in range(w.H_kv):
            assert ids_f[b][h].tolist() == ids[b][h].tolist(), f"{where} b={b} h={h}"
    assert np.array_equal(out_f, out), where
    assert np.array_equal(lse_f, lse), where
    _, out_n, lse_n = G.gpu_step(case, qbits, budget, with_ids=False)
    assert np.array_equal(out_n, out) and np.array_equal(lse_n, lse), where + " (no id output)"


# ----------------------------------------------------------------- C1: the reference config

@pytest.fixture(scope="module")
def c1(G):
    _say("building C1 (4K tokens, 8 KV heads, L=2, F=16)")
    return G.make_case(wl.C1)


def test_c1_retrieve_exact(G, c1):
    for budget in (1024, 300, 17):
        _check_retrieve(G, c1, _q_batch(c1, 0), budget, tag="C1")


def test_c1_decode_with_oracle_ids(G, c1):
    qb = _q_batch(c1, 0)
    ids = [[orc.retrieve_flat(c1.oidx[0][h], _q_group(c1, 0, 0, h), 1024) for h in range(8)]]
    _check_decode(G, c1, qb, ids, tag="C1 budget 1024")


def test_c1_end_to_end_own_ids(G, c1):
    qb = _q_batch(c1, 0)
    ids = _check_retrieve(G, c1, qb, 1024, tag="C1 e2e")
    _check_decode(G, c1, qb, ids, tag="C1 e2e (gpu ids)")


def test_c1_full_budget_is_dense_attention(G, c1):
    """Budget >= context: every chunk selected and the output equals dense softmax attention
    computed by library routines (not by the oracle)."""
    qb = _q_batch(c1, 0)
    ids = _check_retrieve(G, c1, qb, 4096, tag="C1 dense")
    M = c1.oidx[0][0].M
    assert all(ids[0][h].tolist() == list(range(M)) for h in range(8))
    out, lse = G.gpu_decode(c1, qb, ids)
    for h in range(8):
        ref, ref_lse = H.dense_attention_library(_q_group(c1, 0, 0, h), c1.Kf(0, h), c1.Vf(0, h))
        mx, rel = G.attention_errors(out[0, 4 * h:4 * h + 4], ref)
        assert mx <= ATTN_MAX_ABS and rel <= ATTN_REL_L2
        assert np.all(np.abs(lse[0, 4 * h:4 * h + 4] - ref_lse) <= 1e-3)


def test_c1_edge_budgets_and_zero_query(G, c1):
    qb = _q_batch(c1, 0)
    ids = _check_retrieve(G, c1, qb, 0, tag="C1 budget 0")
    assert all(len(ids[0][h]) == 0 for h in range(8))
    out, lse = G.gpu_decode(c1, qb, ids)                  # nothing selected, no open tail
    assert np.all(out == 0) and np.all(lse == -np.inf)
    q0 = np.zeros_like(qb)
    ids = _check_retrieve(G, c1, q0, 200, tag="C1 q=0")
    lens = c1.oidx[0][0].lens()
    k = int(np.searchsorted(np.cumsum(lens), 200, side="right"))
    assert all(ids[0][h].tolist() == list(range(k)) for h in range(8))     # lowest ids first on ties
    out, _ = G.gpu_decode(c1, q0, ids)                    # equal logits: plain mean of the attended V
    for h in range(8):
        rows = np.arange(c1.oidx[0][h].bounds[k])
        want = c1.Vf(0, h)[rows].mean(axis=0)
        assert np.abs(out[0, 4 * h] - want).max() <= 1e-3


def test_c1_sink_and_beam(G, c1):
    qb = _q_batch(c1, 0)
    _check_retrieve(G, c1, qb, 512, sink=16, tag="C1 sink")
    _check_retrieve(G, c1, qb, 512, sink=100, tag="C1 sink100")
    _check_retrieve(G, c1, qb, 1024, policy=orc.POLICY_BEAM, beam=[0, 3], tag="C1 beam top-3")
    _check_retrieve(G, c1, qb, 1024, policy=orc.POLICY_BEAM, beam=[12, 2], tag="C1 beam leaf 12")
    _check_retrieve(G, c1, qb, 1024, policy=orc.POLICY_BEAM, beam=[0, 0], sink=40, tag="C1 beam unbounded")
    from paper_2603_08453_amd import binding as lc
    lc.lc_set_policy(c1.idx, lc.LC_POLICY_EXACT, None, 0)


def test_c1_repeatable(G, c1):
    """Two runs give bit-identical ids and outputs (no order-dependent atomics)."""
    qb = _q_batch(c1, 0)
    a, sa, _ = G.gpu_retrieve(c1, qb, 1024)
    b, sb, _ = G.gpu_retrieve(c1, qb, 1024)
    assert all(np.array_equal(x, y) for x, y in zip(a[0], b[0]))
    assert np.array_equal(sa, sb, equal_nan=True)
    o1, l1 = G.gpu_decode(c1, qb, a)
    o2, l2 = G.gpu_decode(c1, qb, a)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)


def test_c1_fused_step_equals_separate_calls(G, c1):
    from paper_2603_08453_amd import binding as lc
    qb = _q_batch(c1, 0)
    for budget in (0, 1, 200, 1024, 4096, 10 ** 6):
        _check_step(G, c1, qb, budget, tag="C1 step")
    _check_step(G, c1, np.zeros_like(qb), 200, tag="C1 step q=0")
    _check_step(G, c1, qb, 512, sink=16, tag="C1 step sink")
    _check_step(G, c1, qb, 512, sink=100, tag="C1 step sink100")
    _check_step(G, c1, qb, 1024, policy=orc.POLICY_BEAM, beam=[0, 3], tag="C1 step beam top-3")
    _check_step(G, c1, qb, 1024, policy=orc.POLICY_BEAM, beam=[12, 2], tag="C1 step beam leaf 12")
    _check_step(G, c1, qb, 1024, policy=orc.POLICY_BEAM, beam=[0, 0], sink=40, tag="C1 step beam unbounded")
    lc.lc_set_policy(c1.idx, lc.LC_POLICY_EXACT, None, 0)
    for mode in (lc.LC_PRUNE_NEVER, lc.LC_PRUNE_AUTO, lc.LC_PRUNE_ALWAYS):
        lc.lc_set_prune(c1.idx, mode)
        _check_step(G, c1, qb, 777, tag=f"C1 step prune={mode}")
    # and against the oracle directly, end to end
    ids_f, out_f, _ = G.gpu_step(c1, qb, 1024)
    for h in range(8):
        oi = c1.oidx[0][h]
        q = wl.bf16_bits_to_f64(qb[0, 4 * h:4 * h + 4])
        H.accept_ids(ids_f[0][h], orc.node_scores(oi, 0, q), oi.lens(), 1024, pinned=orc.pinned_chunks(oi, 0))
        ref, _ = orc.sparse_decode(q, c1.Kf(0, h), c1.Vf(0, h), oi.bounds, oi.T, ids_f[0][h])
        mx, rel = G.attention_errors(out_f[0, 4 * h:4 * h + 4], ref)
        assert mx <= ATTN_MAX_ABS and rel <= ATTN_REL_L2


def test_fused_step_falls_back_with_many_chunks(G):
    """About ten thousand chunks per sequence: the call runs the kernels of the two separate entry
    points (repeating the selection per workgroup would cost more) and must give the same results."""
    w = wl.tiny("many-chunks", levels=2, fanout=16, T=20000, chunk_lo=1, chunk_hi=3, H_q=4, H_kv=1, budget=500)
    case = G.make_case(w)
    assert case.oidx[0][0].M > 9500
    qb = _q_batch(case, 0)
    for budget in (0, 500, 10 ** 6):
        _check_step(G, case, qb, budget, tag="many-chunks")
    ids = _check_retrieve(G, case, qb, 500, tag="many-chunks")
    _check_decode(G, case, qb, ids, tag="many-chunks")


@pytest.mark.parametrize("T,Hq", [(1100, 4), (2200, 4), (3000, 8), (4600, 4), (7200, 4), (7200, 8)])
def test_fused_step_at_every_selection_width(G, T, Hq):
    """Chunk counts on both sides of each width of the in-register selection (2, 4, 6, 10 and 16
    chunks per lane of a 256-thread workgroup), up to just below the 4096 chunks where the step
    changes to the separate kernels; the ragged last wavefront is partly empty in each."""
    w = wl.tiny(f"width-{T}", levels=2, fanout=16, T=T, chunk_lo=1, chunk_hi=3, H_q=Hq, H_kv=1, budget=300)
    case = G.make_case(w)
    _say(f"{w.name}: {case.oidx[0][0].M} chunks, G = {Hq}")
    assert case.oidx[0][0].M <= 4096
    qb = _q_batch(case, 0)
    ids = _check_retrieve(G, case, qb, 300, tag=w.name)                    # the separate calls against the oracle,
    _check_decode(G, case, qb, ids, tag=w.name)                            # then the step against the separate calls
    for budget in (0, 300, 10 ** 6):
        _check_step(G, case, qb, budget, tag=w.name)
    _check_step(G, case, qb, 64, sink=7, tag=w.name + " sink")
    _check_step(G, case, np.zeros_like(qb), 200, tag=w.name + " q=0")      # one tie group: the overflow path


def test_more_chunks_than_the_select_can_stage_in_lds(G):
    """About twenty thousand chunks: the scoring kernel's last workgroup stages keys and lengths in
    global scratch instead of LDS, and the fused step falls back to the separate kernels."""
    from paper_2603_08453_amd import binding as lc
    w = wl.tiny("huge-M", levels=3, fanout=16, T=40000, chunk_lo=1, chunk_hi=3, H_q=2, H_kv=1, budget=700)
    case = G.make_case(w)
    assert case.oidx[0][0].M > 19000
    qb = _q_batch(case, 0)
    for prune in (lc.LC_PRUNE_NEVER, lc.LC_PRUNE_ALWAYS):
        lc.lc_set_prune(case.idx, prune)
        for budget in (0, 700, 10 ** 6):
            ids = _check_retrieve(G, case, qb, budget, tag=f"huge-M prune={prune}")
            _check_step(G, case, qb, budget, tag=f"huge-M step prune={prune}")
    _check_retrieve(G, case, np.zeros_like(qb), 5000, tag="huge-M q=0")        # one tie group of 20000 chunks
    _check_retrieve(G, case, qb, 700, sink=50, tag="huge-M sink")
    ids = _check_retrieve(G, case, qb, 700, tag="huge-M")
    _check_decode(G, case, qb, ids, tag="huge-M")


# ----------------------------------------------------------------- small, ragged, tails, deep trees

@pytest.mark.parametrize("name,kw,tails", [
    ("tiny-L1", dict(levels=1, fanout=4), None),
    ("tiny-L3-tail", dict(levels=3, fanout=3, T=700), [9]),
    ("tiny-L4-G1", dict(levels=4, fanout=2, H_q=2, H_kv=2, T=900), [1]),
    ("tiny-G8", dict(levels=2, fanout=5, H_q=8, H_kv=1, T=600), [0]),
    ("ragged-G7", dict(B=3, H_q=14, H_kv=2, levels=3, fanout=4, T=0, T_range=(300, 1500), chunk_lo=2, chunk_hi=40),
     [0, 33, 5]),
    ("one-chunk", dict(levels=2, fanout=4, T=20, chunk_lo=20, chunk_hi=20), None),
])
def test_small_cases(G, name, kw, tails):
    w = wl.tiny(name, **kw)
    _say(f"{name}: {w}")
    case = G.make_case(w, tails=tails)
    qb = _q_batch(case, 0)
    for budget in (0, 1, 50, w.budget, 10 ** 6):
        ids = _check_retrieve(G, case, qb, budget, tag=name)
        _check_decode(G, case, qb, ids, tag=f"{name} budget {budget}")
        _check_step(G, case, qb, budget, tag=name + " step")
    if w.levels > 1:
        beam = [0] + [2] * (w.levels - 1)
        _check_retrieve(G, case, qb, w.budget, policy=orc.POLICY_BEAM, beam=beam, tag=name + " beam")
        _check_step(G, case, qb, w.budget, policy=orc.POLICY_BEAM, beam=beam, tag=name + " step beam")
    _check_retrieve(G, case, qb, 64, sink=7, tag=name + " sink")
    _check_step(G, case, qb, 64, sink=7, tag=name + " step sink")


def test_pruning_happens_and_stays_exact(G):
    """Tightly clustered keys: the level-by-level pass skips most chunks (their scores come
    back as -inf = never computed) and the selection still equals the flat scan."""
    w = wl.tiny("tight", levels=3, fanout=4, T=4000, chunk_lo=4, chunk_hi=12, budget=60, H_q=4, H_kv=2)
    case = G.make_case(w, offset_std=3.0, noise_std=0.02)
    qb = _q_batch(case, 0)
    _check_retrieve(G, case, qb, 60, tag="tight")
    _, scores, _ = G.gpu_retrieve(case, qb, 60)
    M = case.oidx[0][0].M
    scored = np.isfinite(scores[0, :, :M]).sum(axis=1)
    _say(f"tight clusters: scored {scored.tolist()} of {M} chunks per head")
    assert np.all(scored < M)


def test_select_with_a_large_tie_group(G):
    """q = 0 makes every chunk score equal: several hundred chunks tie at the cutoff, more than the
    selection's short list holds, so the cut is made in id order by a scan."""
    w = wl.tiny("ties", levels=2, fanout=8, T=4000, chunk_lo=4, chunk_hi=12, H_q=4, H_kv=2, budget=1000)
    case = G.make_case(w)
    M = case.oidx[0][0].M
    assert M > 300
    q0 = np.zeros_like(_q_batch(case, 0))
    lens = case.oidx[0][0].lens()
    for budget in (0, 7, 1000, 2500, 10 ** 6):
        ids = _check_retrieve(G, case, q0, budget, tag="ties")
        k = int(np.searchsorted(np.cumsum(lens), budget, side="right"))
        assert all(ids[0][h].tolist() == list(range(k)) for h in range(w.H_kv)), budget
    # a chunk-count limit cuts the same tie group
    ids = _check_retrieve(G, case, q0, 10 ** 6, policy=orc.POLICY_BEAM, beam=[300, 0], tag="ties beam")
    assert all(ids[0][h].tolist() == list(range(300)) for h in range(w.H_kv))
    ids = _check_retrieve(G, case, q0, 600, policy=orc.POLICY_BEAM, beam=[300, 0], sink=30, tag="ties beam sink")
    _check_step(G, case, q0, 600, policy=orc.POLICY_BEAM, beam=[300, 0], sink=30, tag="ties step beam sink")
    for budget in (7, 1000, 2500):
        _check_step(G, case, q0, budget, tag="ties step")
    from paper_2603_08453_amd import binding as lc
    lc.lc_set_policy(case.idx, lc.LC_POLICY_EXACT, None, 0)


def test_select_with_a_crowded_score_range(G):
    """One chunk with a very negative score stretches the score range so far that thousands of
    chunks share a few histogram bins: the bin holding the cutoff must be split again."""
    w = wl.tiny("crowded", levels=2, fanout=8, T=9000, chunk_lo=2, chunk_hi=4, H_q=2, H_kv=1, budget=600)

    def outlier(seqs):
        for s in seqs:
            q = wl.bf16_bits_to_f64(s.Q[0])                                  # [H_q][d]
            u = -(q / np.linalg.norm(q, axis=1, keepdims=True)).sum(axis=0)
            c = (len(s.bounds) - 1) // 2
            rows = slice(int(s.bounds[c]), int(s.bounds[c + 1]))
            s.K[0, rows] = wl.f32_to_bf16_bits((40.0 * u).astype(np.float32))[None, :]

    case = G.make_case(w, mutate=outlier)
    qb = _q_batch(case, 0)
    oi = case.oidx[0][0]
    s_ref = orc.node_scores(oi, 0, wl.bf16_bits_to_f64(qb[0]))
    pos = s_ref[s_ref > 0]
    _say(f"crowded: M={oi.M}, min score {s_ref.min():.2f}, positive scores {pos.min():.3f}..{pos.max():.3f}")
    assert s_ref.min() < -1.0 and len(pos) > 2500 and pos.max() / pos.min() < 16.0
    for prune in (0, 2):
        from paper_2603_08453_amd import binding as lc
        lc.lc_set_prune(case.idx, prune)
        for budget in (3, 600, 5000, 10 ** 6):
            ids = _check_retrieve(G, case, qb, budget, tag=f"crowded prune={prune}")
            _check_step(G, case, qb, budget, tag=f"crowded step prune={prune}")
        _check_decode(G, case, qb, ids, tag="crowded")


def test_paper_literal_algorithm1(G):
    """The paper's own configuration of Algorithm 1: unit-norm representatives with radius 0
    (PAPER_UNIT), top-k_g coarse units then top-k_c fine clusters (BEAM), *all* chunks of the kept
    fine clusters attended (no chunk-level limit: budget = everything), attention sink of 16 tokens,
    chunks of 8..16 tokens, 2 chunks per fine cluster on average."""
    from paper_2603_08453_amd import binding as lc
    w = wl.tiny("paper", levels=3, fanout=2, T=3000, chunk_lo=8, chunk_hi=16, H_q=8, H_kv=2)
    case = G.make_case(w, geometry=orc.PAPER_UNIT)
    qb = _q_batch(case, 0)
    k_c, k_g = 12, 6
    beam = [0, k_c, k_g]
    ids = _check_retrieve(G, case, qb, 10 ** 9, policy=orc.POLICY_BEAM, beam=beam, sink=16, tag="paper-literal")
    for h in range(w.H_kv):
        oi = case.oidx[0][h]
        kept_clusters = set(oi.parent[0][ids[0][h]].tolist())
        pinned = set(orc.pinned_chunks(oi, 16).tolist())
        free_clusters = set(oi.parent[0][[j for j in ids[0][h] if j not in pinned]].tolist())
        assert len(free_clusters) <= k_c
        # every chunk of a kept fine cluster is there
        for c in free_clusters:
            assert set(np.nonzero(oi.parent[0] == c)[0].tolist()) - pinned <= set(ids[0][h].tolist())
    _check_decode(G, case, qb, ids, tag="paper-literal attention")
    lc.lc_set_policy(case.idx, lc.LC_POLICY_EXACT, None, 0)


def test_prune_modes_give_the_same_ids(G, c1):
    """The level walk is an optimisation of EXACT retrieval: always / never / auto agree bit for bit."""
    from paper_2603_08453_amd import binding as lc
    qb = _q_batch(c1, 0)
    got = []
    for mode in (lc.LC_PRUNE_ALWAYS, lc.LC_PRUNE_NEVER, lc.LC_PRUNE_AUTO):
        lc.lc_set_prune(c1.idx, mode)
        ids, _, _ = G.gpu_retrieve(c1, qb, 777)
        got.append(ids)
    lc.lc_set_prune(c1.idx, lc.LC_PRUNE_ALWAYS)
    for h in range(8):
        assert got[0][0][h].tolist() == got[1][0][h].tolist() == got[2][0][h].tolist()


def test_split_count_does_not_change_the_result(G):
    w = wl.tiny("splits", levels=2, fanout=4, T=3000, chunk_lo=4, chunk_hi=32, budget=1500)
    outs = []
    for splits in (1, 3, 16):
        case = G.make_case(w, decode_splits=splits, tails=[5])
        qb = _q_batch(case, 0)
        ids = [[orc.retrieve_flat(case.oidx[0][h], _q_group(case, 0, 0, h), 1500) for h in range(w.H_kv)]]
        outs.append(_check_decode(G, case, qb, ids, tag=f"splits={splits}"))
    assert np.abs(outs[0] - outs[1]).max() <= 1e-4 and np.abs(outs[0] - outs[2]).max() <= 1e-4


# ----------------------------------------------------------------- index build on the GPU

# shapes of the build: levels small enough to be clustered whole in one workgroup; a batch whose
# chunk level straddles that kernel's limit (224 points, 64 clusters) so that the level takes the
# tiled kernels and the one above it the small one; chunks of 1..200 tokens, i.e. pooling with
# one, several and partly filled batches of rows
BUILD_SHAPES = {
    "small-levels": dict(B=2, levels=3, fanout=4, T=0, T_range=(800, 1600), chunk_lo=3, chunk_hi=30),
    "straddle": dict(B=2, levels=3, fanout=3, T=0, T_range=(2900, 4600), chunk_lo=4, chunk_hi=24),
    "long-chunks": dict(B=1, levels=3, fanout=4, T=9000, chunk_lo=1, chunk_hi=200),
}


@pytest.mark.parametrize("shape", list(BUILD_SHAPES))
@pytest.mark.parametrize("geometry", [orc.TOKEN_BALL, orc.PAPER_UNIT])
def test_build_index_matches_oracle(G, geometry, shape):
    from paper_2603_08453_amd import binding as lc
    w = wl.tiny("build-" + shape, **BUILD_SHAPES[shape])
    case = G.make_case(w, tails=[4, 0][:w.B], geometry=geometry, build_on="gpu")
    _say(f"build {shape}: chunks per sequence {[case.oidx[b][0].M for b in range(w.B)]}")
    blob = lc.unpack_blob(lc.lc_index_export(case.idx))
    tally = {}
    for b in range(w.B):
        s = blob["seqs"][b]
        assert s["T"] == case.seqs[b].T and np.array_equal(s["bounds"], case.seqs[b].bounds)
        for h in range(w.H_kv):
            oi = case.oidx[b][h]
            gi = G.levels_to_oracle_index(s["heads"][h], s["bounds"], s["T"], w.fanout, geometry)
            assert [gi.n(l) for l in range(w.levels)] == [oi.n(l) for l in range(w.levels)]
            # level 0 never depends on clustering: direct parity
            assert np.allclose(gi.center[0], oi.center[0], rtol=2e-6, atol=2e-6)
            assert np.all(gi.radius[0] >= oi.radius[0] * (1 - 1e-6))
            assert np.all(gi.radius[0] <= oi.radius[0] * (1 + 2e-5) + 1e-7)
            # invariants of the GPU-built index, by brute force
            H.check_covering_invariant(gi, case.Kf(b, h), slack=1e-6)
            H.check_counts(gi)
            if H.same_topology_or_near_tie(gi, oi, w.levels - 1, f"build b{b} h{h}", tally):
                for l in range(1, w.levels):
                    live = oi.nchunk[l] > 0
                    assert np.allclose(gi.center[l][live], oi.center[l][live], rtol=1e-5, atol=1e-5)
                    assert np.all(gi.radius[l][live] >= oi.radius[l][live] * (1 - 1e-6))
                    assert np.all(gi.radius[l][live] <= oi.radius[l][live] * (1 + 5e-5) + 1e-6)
    _say(f"build geometry={geometry}: {tally.get('same', 0)}/{w.B * w.H_kv} (seq, head) trees have the oracle's topology, "
         f"{tally.get('near_tie', 0)} differ behind a near-tie of the oracle's clustering")
    # retrieval on the GPU-built index is exact with respect to its own stored values
    qb = _q_batch(case, 0)
    ids, scores, _ = G.gpu_retrieve(case, qb, w.budget)
    for b in range(w.B):
        s = blob["seqs"][b]
        for h in range(w.H_kv):
            gi = G.levels_to_oracle_index(s["heads"][h], s["bounds"], s["T"], w.fanout, geometry)
            q = wl.bf16_bits_to_f64(qb[b, h * w.G:(h + 1) * w.G])
            H.accept_ids(ids[b][h], orc.node_scores(gi, 0, q), gi.lens(), w.budget)


@pytest.mark.parametrize("seed", list(range(int(__import__("os").environ.get("LC_RANDOM_BUILDS", "8")))))
def test_random_builds(G, seed):
    """Seeded random shapes built on the GPU: level 0 against the oracle directly, the levels above
    wherever the oracle's clustering has no near-tie, the covering invariant by brute force."""
    from paper_2603_08453_amd import binding as lc
    r = np.random.default_rng(5000 + seed)
    h_kv = int(r.integers(1, 4))
    B = int(r.integers(1, 4))
    levels = int(r.integers(2, 5))
    fanout = int(r.integers(2, 12))
    lo = int(r.integers(1, 12))
    hi = lo + int(r.integers(0, 90))
    t_lo = int(r.integers(200, 5000))
    geometry = orc.TOKEN_BALL if r.random() < 0.7 else orc.PAPER_UNIT
    w = wl.tiny(f"rbuild{seed}", cfg_id=5000 + seed, B=B, H_q=h_kv, H_kv=h_kv, levels=levels, fanout=fanout, T=0,
                T_range=(t_lo, t_lo + int(r.integers(1, 3000))), chunk_lo=lo, chunk_hi=hi)
    # (float32 chunk centers: with bfloat16 ones a mean next to a rounding boundary may round the other
    # way in float32 than in float64, which the dedicated bfloat16 build test allows for)
    case = G.make_case(w, tails=[int(x) for x in r.integers(0, 20, size=B)], geometry=geometry, build_on="gpu")
    _say(f"build seed {seed}: B={B} H_kv={h_kv} L={levels} F={fanout} chunks {lo}..{hi} "
         f"M={[case.oidx[b][0].M for b in range(B)]} geometry {geometry}")
    blob = lc.unpack_blob(lc.lc_index_export(case.idx))
    tally = {}
    for b in range(B):
        sq = blob["seqs"][b]
        for h in range(h_kv):
            oi = case.oidx[b][h]
            gi = G.levels_to_oracle_index(sq["heads"][h], sq["bounds"], sq["T"], w.fanout, geometry)
            assert [gi.n(l) for l in range(levels)] == [oi.n(l) for l in range(levels)]
            assert np.allclose(gi.center[0], oi.center[0], rtol=2e-6, atol=2e-6)
            assert np.all(gi.radius[0] >= oi.radius[0] * (1 - 1e-6))
            H.check_covering_invariant(gi, case.Kf(b, h), slack=1e-6)
            H.check_counts(gi)
            if H.same_topology_or_near_tie(gi, oi, levels - 1, f"rbuild{seed} b{b} h{h}", tally):
                for l in range(1, levels):
                    live = oi.nchunk[l] > 0
                    assert np.allclose(gi.center[l][live], oi.center[l][live], rtol=1e-5, atol=1e-5)
                    assert np.all(gi.radius[l][live] >= oi.radius[l][live] * (1 - 1e-6))
    _say(f"  {tally.get('same', 0)} trees with the oracle's topology, {tally.get('near_tie', 0)} behind a near-tie")


def _bf16_ulp(x):
    """Spacing of bfloat16 values at |x| (8 significant bits)."""
    _, e = np.frexp(np.abs(x))
    return np.ldexp(1.0, e - 8)


def test_bf16_chunk_centers_imported_index(G):
    """An index whose chunk centers are stored as bfloat16: import/export keeps every value, and
    retrieval (flat, level walk, top-k per level), attention and the fused step match the oracle
    on the same stored values."""
    from paper_2603_08453_amd import binding as lc
    w = wl.tiny("half", B=2, H_q=8, H_kv=2, levels=3, fanout=4, T=0, T_range=(1500, 2500), chunk_lo=3, chunk_hi=30)
    case = G.make_case(w, tails=[6, 0], center_dtype=lc.LC_CENTER_BF16)
    blob = lc.unpack_blob(lc.lc_index_export(case.idx))
    assert blob["center_dtype"] == lc.LC_CENTER_BF16
    for b in range(w.B):
        for h in range(w.H_kv):
            oi = case.oidx[b][h]
            for l in range(w.levels):
                assert np.array_equal(blob["seqs"][b]["heads"][h][l]["center"].astype(np.float64), oi.center[l]), (b, h, l)
            assert np.array_equal(orc.store_bf16(oi.center[0]), oi.center[0])
    qb = _q_batch(case, 0)
    for prune in (lc.LC_PRUNE_NEVER, lc.LC_PRUNE_ALWAYS):
        lc.lc_set_prune(case.idx, prune)
        for budget in (0, 90, 700, 10 ** 6):
            ids = _check_retrieve(G, case, qb, budget, tag=f"half prune={prune}")
            _check_decode(G, case, qb, ids, tag=f"half budget {budget}")
            _check_step(G, case, qb, budget, tag=f"half step prune={prune}")
    _check_retrieve(G, case, qb, 500, sink=20, tag="half sink")
    beam = [0, 6, 2]
    _check_retrieve(G, case, qb, 600, policy=orc.POLICY_BEAM, beam=beam, tag="half beam")
    _check_step(G, case, qb, 600, policy=orc.POLICY_BEAM, beam=beam, tag="half step beam")
    lc.lc_set_policy(case.idx, lc.LC_POLICY_EXACT, None, 0)
    # a blob written for float32 centers is refused: its radii were measured from other centers
    f32_cfg = lc.lc_config_default(levels=w.levels, fanout=w.fanout, max_chunks=case.cfg.max_chunks,
                                   max_tokens=case.cfg.max_tokens)
    import torch
    buf = torch.zeros(lc.lc_index_bytes(f32_cfg, w.B, w.H_kv), dtype=torch.uint8, device="cuda")
    with pytest.raises(lc.LycheeError) as e:
        lc.lc_index_import(f32_cfg, lc.lc_index_export(case.idx), buf)
    assert e.value.code == lc.LC_ERR_BAD_BLOB


@pytest.mark.parametrize("geometry", [orc.TOKEN_BALL, orc.PAPER_UNIT])
def test_bf16_chunk_centers_built_on_gpu(G, geometry):
    """lc_build_index with bfloat16 chunk centers: the stored centers are bfloat16 values, equal to the
    oracle's except where the float32 mean falls on the other side of a rounding boundary (then one
    bfloat16 step away); the radii cover the tokens around the stored centers; retrieval on the
    built index is exact with respect to its own stored values."""
    from paper_2603_08453_amd import binding as lc
    w = wl.tiny("halfbuild", B=2, levels=3, fanout=4, T=0, T_range=(800, 1600), chunk_lo=3, chunk_hi=30)
    case = G.make_case(w, tails=[4, 0], geometry=geometry, build_on="gpu", center_dtype=lc.LC_CENTER_BF16)
    blob = lc.unpack_blob(lc.lc_index_export(case.idx))
    n_el = n_diff = 0
    tally = {}
    for b in range(w.B):
        s = blob["seqs"][b]
        for h in range(w.H_kv):
            oi = case.oidx[b][h]
            gi = G.levels_to_oracle_index(s["heads"][h], s["bounds"], s["T"], w.fanout, geometry)
            assert [gi.n(l) for l in range(w.levels)] == [oi.n(l) for l in range(w.levels)]
            assert np.array_equal(orc.store_bf16(gi.center[0]), gi.center[0])
            diff = np.abs(gi.center[0] - oi.center[0])
            assert np.all(diff <= _bf16_ulp(oi.center[0]) * 1.0000001)
            n_el += diff.size
            n_diff += int((diff > 0).sum())
            exact_rows = np.all(diff == 0, axis=1)
            assert np.all(gi.radius[0][exact_rows] >= oi.radius[0][exact_rows] * (1 - 1e-6))
            assert np.all(gi.radius[0][exact_rows] <= oi.radius[0][exact_rows] * (1 + 2e-5) + 1e-7)
            H.check_covering_invariant(gi, case.Kf(b, h), slack=1e-6)
            H.check_counts(gi)
            H.same_topology_or_near_tie(gi, oi, w.levels - 1, f"bf16 build b{b} h{h}", tally)
    _say(f"bf16 build geometry={geometry}: {n_diff} of {n_el} chunk-center elements one bfloat16 step from the "
         f"oracle's; {tally.get('same', 0)}/{w.B * w.H_kv} trees have the oracle's topology, {tally.get('near_tie', 0)} differ behind a near-tie")
    assert n_diff <= 0.002 * n_el
    qb = _q_batch(case, 0)
    ids, scores, _ = G.gpu_retrieve(case, qb, w.budget)
    ids_f, out_f, _ = G.gpu_step(case, qb, w.budget)
    out, _ = G.gpu_decode(case, qb, ids)
    assert np.array_equal(out, out_f)
    for b in range(w.B):
        s = blob["seqs"][b]
        for h in range(w.H_kv):
            gi = G.levels_to_oracle_index(s["heads"][h], s["bounds"], s["T"], w.fanout, geometry)
            q = wl.bf16_bits_to_f64(qb[b, h * w.G:(h + 1) * w.G])
            H.accept_ids(ids[b][h], orc.node_scores(gi, 0, q), gi.lens(), w.budget)
            assert ids_f[b][h].tolist() == ids[b][h].tolist()


def test_bf16_chunk_centers_append_stream(G):
    """Lazy update with bfloat16 chunk centers: every new chunk's stored center is a bfloat16 value, its
    radius covers its tokens, the path above it is updated as in the oracle, and re-clustering
    afterwards starts from the stored (rounded) chunk centers."""
    import torch
    from paper_2603_08453_amd import binding as lc
    steps, L = 120, 3
    w = wl.tiny("halfstream", B=2, levels=L, fanout=4, T=0, T_range=(300, 500), chunk_lo=3, chunk_hi=20,
                stream_close_lo=3, stream_close_hi=17)
    case = G.make_case(w, tails=[2, 0], extra_tokens=steps, extra_chunks=steps, center_dtype=lc.LC_CENTER_BF16)
    streams = [wl.make_stream(w, b, steps) for b in range(w.B)]
    Kf = [[np.vstack([case.Kf(b, h), np.zeros((steps, w.d))]) for h in range(w.H_kv)] for b in range(w.B)]
    for t in range(steps):
        k_bits = np.stack([st.k[t] for st in streams])
        v_bits = np.stack([st.v[t] for st in streams])
        close = [int(st.close[t]) for st in streams]
        lc.lc_append(case.idx, case.K, case.V, G.to_bf16_tensor(k_bits), G.to_bf16_tensor(v_bits), close, case.ws)
        for b in range(w.B):
            for h in range(w.H_kv):
                oi = case.oidx[b][h]
                Kf[b][h][oi.T] = wl.bf16_bits_to_f64(k_bits[b, h])
                orc.append_token(oi)
                if close[b]:
                    orc.close_chunk(oi, Kf[b][h])
    torch.cuda.synchronize()
    blob = lc.unpack_blob(lc.lc_index_export(case.idx))
    n_el = n_diff = 0
    for b in range(w.B):
        s = blob["seqs"][b]
        for h in range(w.H_kv):
            oi = case.oidx[b][h]
            gi = G.levels_to_oracle_index(s["heads"][h], s["bounds"], s["T"], w.fanout, orc.TOKEN_BALL)
            assert gi.M == oi.M and gi.M > len(case.seqs[b].bounds) - 1
            assert np.array_equal(orc.store_bf16(gi.center[0]), gi.center[0])
            diff = np.abs(gi.center[0] - oi.center[0])
            assert np.all(diff <= _bf16_ulp(oi.center[0]) * 1.0000001)
            n_el += diff.size
            n_diff += int((diff > 0).sum())
            H.check_covering_invariant(gi, Kf[b][h], slack=1e-6)
            H.check_counts(gi)
            assert np.array_equal(gi.parent[0], oi.parent[0])
            if np.all(diff == 0):
                for l in range(1, L):
                    live = oi.nchunk[l] > 0
                    assert np.allclose(gi.center[l][live], oi.center[l][live], rtol=2e-5, atol=2e-5)
                    assert np.all(gi.radius[l][live] >= oi.radius[l][live] * (1 - 1e-6))
                    assert np.all(gi.radius[l][live] <= oi.radius[l][live] * (1 + 1e-3) + 1e-5)
    _say(f"bf16 append: {n_diff} of {n_el} chunk-center elements one bfloat16 step from the oracle's")
    assert n_diff <= 0.002 * n_el
    lc.lc_recluster(case.idx, case.ws)
    torch.cuda.synchronize()
    after = lc.unpack_blob(lc.lc_index_export(case.idx))
    qb = np.stack([st.q[steps - 1] for st in streams])
    ids, _, _ = G.gpu_retrieve(case, qb, 150)
    for b in range(w.B):
        sa = after["seqs"][b]
        for h in range(w.H_kv):
            gi = G.levels_to_oracle_index(sa["heads"][h], sa["bounds"], sa["T"], w.fanout, orc.TOKEN_BALL)
            assert np.array_equal(gi.center[0].astype(np.float32), blob["seqs"][b]["heads"][h][0]["center"])
            H.check_covering_invariant(gi, Kf[b][h], slack=1e-6)
            q = wl.bf16_bits_to_f64(qb[b, h * w.G:(h + 1) * w.G])
            H.accept_ids(ids[b][h], orc.node_scores(gi, 0, q), gi.lens(), 150)


def test_per_level_fanouts_built_on_gpu(G):
    """The paper's tiers (Appendix A): 2 chunks per fine cluster, many fine clusters per coarse unit.
    lc_build_index sizes every level by its own fan-out; the tree matches the oracle's and retrieval
    (level walk and top-k per level) works on it."""
    from paper_2603_08453_amd import binding as lc
    w = wl.tiny("tiers", B=2, H_q=8, H_kv=2, levels=3, fanout=16, T=0, T_range=(1500, 2500), chunk_lo=8, chunk_hi=16)
    fan = [0, 2, 22]
    case = G.make_case(w, tails=[5, 0], build_on="gpu", fanouts=fan)
    blob = lc.unpack_blob(lc.lc_index_export(case.idx))
    assert blob["fanouts"][:3] == fan
    tally = {}
    for b in range(w.B):
        s = blob["seqs"][b]
        T, M, n_lev = case.idx.info(b)
        assert list(n_lev[:3]) == [M, -(-M // 2), -(-(-(-M // 2)) // 22)]
        for h in range(w.H_kv):
            oi = case.oidx[b][h]
            gi = G.levels_to_oracle_index(s["heads"][h], s["bounds"], s["T"], w.fanout, orc.TOKEN_BALL)
            assert [gi.n(l) for l in range(3)] == [oi.n(l) for l in range(3)]
            H.check_covering_invariant(gi, case.Kf(b, h), slack=1e-6)
            H.check_counts(gi)
            H.same_topology_or_near_tie(gi, oi, 2, f"tiers b{b} h{h}", tally)
    _say(f"tiers: {tally.get('same', 0)}/{w.B * w.H_kv} trees have the oracle's topology, {tally.get('near_tie', 0)} differ behind a near-tie")
    # a blob of this index is refused by a configuration with other fan-outs
    import torch
    other = lc.lc_config_default(levels=3, fanout=16, fanouts=[0, 2, 8], max_chunks=case.cfg.max_chunks,
                                 max_tokens=case.cfg.max_tokens)
    buf = torch.zeros(lc.lc_index_bytes(other, w.B, w.H_kv), dtype=torch.uint8, device="cuda")
    with pytest.raises(lc.LycheeError) as e:
        lc.lc_index_import(other, lc.lc_index_export(case.idx), buf)
    assert e.value.code == lc.LC_ERR_BAD_BLOB
    # retrieval on the imported oracle index of the same shape: exact policy and top-k per level
    case2 = G.make_case(w, tails=[5, 0], fanouts=fan)
    qb = _q_batch(case2, 0)
    for budget in (100, 700):
        ids = _check_retrieve(G, case2, qb, budget, tag="tiers")
        _check_decode(G, case2, qb, ids, tag=f"tiers budget {budget}")
        _check_step(G, case2, qb, budget, tag="tiers step")
    beam = [0, 20, 3]
    _check_retrieve(G, case2, qb, 10 ** 9, policy=orc.POLICY_BEAM, beam=beam, sink=16, tag="tiers beam")
    _check_step(G, case2, qb, 10 ** 9, policy=orc.POLICY_BEAM, beam=beam, sink=16, tag="tiers step beam")
    lc.lc_set_policy(case2.idx, lc.LC_POLICY_EXACT, None, 0)


# ----------------------------------------------------------------- lazy update

@pytest.mark.parametrize("geometry,L", [(orc.TOKEN_BALL, 3), (orc.TOKEN_BALL, 1), (orc.PAPER_UNIT, 2)])
def test_append_stream_matches_oracle(G, geometry, L):
    import torch
    from paper_2603_08453_amd import binding as lc
    steps = 150
    w = wl.tiny("stream", B=2, levels=L, fanout=4, T=0, T_range=(300, 500), chunk_lo=3, chunk_hi=20,
                stream_close_lo=3, stream_close_hi=17)
    case = G.make_case(w, tails=[2, 0], geometry=geometry, extra_tokens=steps, extra_chunks=steps)
    streams = [wl.make_stream(w, b, steps) for b in range(w.B)]
    Kf = [[np.vstack([case.Kf(b, h), np.zeros((steps, w.d))]) for h in range(w.H_kv)] for b in range(w.B)]
    Vf = [[np.vstack([case.Vf(b, h), np.zeros((steps, w.d))]) for h in range(w.H_kv)] for b in range(w.B)]
    parent_mismatch = 0
    for t in range(steps):
        k_bits = np.stack([st.k[t] for st in streams])
        v_bits = np.stack([st.v[t] for st in streams])
        close = [int(st.close[t]) for st in streams]
        if t % 2 == 1:
            close[1] = 0                       # sequences close at different times
        lc.lc_append(case.idx, case.K, case.V, G.to_bf16_tensor(k_bits), G.to_bf16_tensor(v_bits), close, case.ws)
        for b in range(w.B):
            for h in range(w.H_kv):
                oi = case.oidx[b][h]
                Kf[b][h][oi.T] = wl.bf16_bits_to_f64(k_bits[b, h])
                Vf[b][h][oi.T] = wl.bf16_bits_to_f64(v_bits[b, h])
                orc.append_token(oi)
                if close[b]:
                    orc.close_chunk(oi, Kf[b][h])
        if t % 50 == 49 or t == steps - 1:
            torch.cuda.synchronize()
            blob = lc.unpack_blob(lc.lc_index_export(case.idx))
            for b in range(w.B):
                s = blob["seqs"][b]
                T, M, _ = case.idx.info(b)
                assert (T, M) == (case.oidx[b][0].T, case.oidx[b][0].M) == (s["T"], len(s["bounds"]) - 1)
                assert np.array_equal(s["bounds"], case.oidx[b][0].bounds)
                for h in range(w.H_kv):
                    oi = case.oidx[b][h]
                    gi = G.levels_to_oracle_index(s["heads"][h], s["bounds"], s["T"], w.fanout, geometry)
                    H.check_covering_invariant(gi, Kf[b][h], slack=1e-6)
                    H.check_counts(gi)
                    if L > 1 and not np.array_equal(gi.parent[0], oi.parent[0]):
                        parent_mismatch += 1
                        continue
                    for l in range(L):
                        live = oi.nchunk[l] > 0
                        assert np.allclose(gi.center[l][live], oi.center[l][live], rtol=2e-5, atol=2e-5), (t, b, h, l)
                        assert np.all(gi.radius[l][live] >= oi.radius[l][live] * (1 - 1e-6))
                        assert np.all(gi.radius[l][live] <= oi.radius[l][live] * (1 + 1e-3) + 1e-5)
    _say(f"append L={L} geometry={geometry}: parent choice differed from the oracle in {parent_mismatch} checks")
    assert parent_mismatch == 0
    # the cache rows were written, and retrieval + attention over the grown index agree
    for b in range(w.B):
        for h in range(w.H_kv):
            T = case.oidx[b][h].T
            got = case.K[b, h, :T].float().cpu().numpy()
            assert np.array_equal(got, Kf[b][h][:T].astype(np.float32))
    qb = np.stack([st.q[steps - 1] for st in streams])
    lc.lc_set_policy(case.idx, lc.LC_POLICY_EXACT, None, 0)
    ids, scores, _ = G.gpu_retrieve(case, qb, 120)
    out, lse = G.gpu_decode(case, qb, ids)
    for b in range(w.B):
        for h in range(w.H_kv):
            oi = case.oidx[b][h]
            q = wl.bf16_bits_to_f64(qb[b, h * w.G:(h + 1) * w.G])
            H.accept_ids(ids[b][h], orc.node_scores(oi, 0, q), oi.lens(), 120)
            ref, _ = orc.sparse_decode(q, Kf[b][h], Vf[b][h], oi.bounds, oi.T, ids[b][h])
            mx, rel = G.attention_errors(out[b, h * w.G:(h + 1) * w.G], ref)
            assert mx <= ATTN_MAX_ABS and rel <= ATTN_REL_L2


def test_recluster_after_a_stream_equals_a_fresh_build(G):
    """Drift control: after many lazy appends lc_recluster rebuilds the levels above the chunks;
    the result must be what the oracle builds from scratch on the sequence as it stands."""
    import torch
    from paper_2603_08453_amd import binding as lc
    steps, L, F = 400, 3, 4
    w = wl.tiny("drift", B=2, levels=L, fanout=F, T=0, T_range=(300, 500), chunk_lo=3, chunk_hi=20,
                stream_close_lo=3, stream_close_hi=17)
    case = G.make_case(w, tails=[2, 0], extra_tokens=steps, extra_chunks=steps)
    streams = [wl.make_stream(w, b, steps) for b in range(w.B)]
    Kf = [[np.vstack([case.Kf(b, h), np.zeros((steps, w.d))]) for h in range(w.H_kv)] for b in range(w.B)]
    for t in range(steps):
        k_bits = np.stack([st.k[t] for st in streams])
        v_bits = np.stack([st.v[t] for st in streams])
        close = [int(st.close[t]) for st in streams]
        lc.lc_append(case.idx, case.K, case.V, G.to_bf16_tensor(k_bits), G.to_bf16_tensor(v_bits), close, case.ws)
        for b in range(w.B):
            for h in range(w.H_kv):
                oi = case.oidx[b][h]
                Kf[b][h][oi.T] = wl.bf16_bits_to_f64(k_bits[b, h])
                orc.append_token(oi)
                if close[b]:
                    orc.close_chunk(oi, Kf[b][h])
    torch.cuda.synchronize()
    before = lc.unpack_blob(lc.lc_index_export(case.idx))
    # how far the radii have drifted since the build, against the oracle's definition on its own
    # lazily updated tree (same parent choices on both sides, so the same nodes grew)
    triggered = 0
    for level in range(1, L):
        drift = lc.lc_index_drift(case.idx, level, case.ws)
        for b in range(w.B):
            for h in range(w.H_kv):
                oi = case.oidx[b][h]
                gb = G.levels_to_oracle_index(before["seqs"][b]["heads"][h], before["seqs"][b]["bounds"],
                                              before["seqs"][b]["T"], F, orc.TOKEN_BALL)
                then, now, grow, n = orc.radius_drift(oi, level)
                got = drift[b, h]
                assert got[3] == n and got[1] >= got[0] and got[2] >= 0.0, (level, b, h, got)
                if np.array_equal(gb.parent[0], oi.parent[0]):
                    # (the GPU inflates every updated radius by a few 1e-6 to stay on the safe side of its
                    # float32 rounding; over some thirty updates of a node that adds up to a few 1e-4)
                    assert np.allclose(got[:3], [then, now, grow], rtol=1e-3, atol=1e-4), (level, b, h, got, then, now, grow)
                    assert got[1] >= now * (1 - 1e-6) and got[2] >= grow * (1 - 1e-6) - 1e-6
                triggered += int(level == 1 and got[1] > 1.02 * got[0])
        if level == 1:
            _say(f"drift of level 1 before re-clustering: sum of radii now / at build = "
                 f"{drift[..., 1].sum() / drift[..., 0].sum():.4f}, largest growth of one node {drift[..., 2].max():.3f}")
    assert triggered > 0                     # 400 streamed tokens did inflate some tree's fine clusters
    lc.lc_recluster(case.idx, case.ws)
    torch.cuda.synchronize()
    for level in range(1, L):                # a re-clustered index starts from a fresh baseline
        drift = lc.lc_index_drift(case.idx, level, case.ws)
        assert np.array_equal(drift[..., 0], drift[..., 1]) and np.all(drift[..., 2] == 0.0)
    after = lc.unpack_blob(lc.lc_index_export(case.idx))
    tally = {}
    for b in range(w.B):
        sb, sa = before["seqs"][b], after["seqs"][b]
        assert sa["T"] == sb["T"] and np.array_equal(sa["bounds"], sb["bounds"])
        T, M, n_lev = case.idx.info(b)
        for h in range(w.H_kv):
            lazy = case.oidx[b][h]
            assert (T, M) == (lazy.T, lazy.M)
            fresh = orc.build_index(Kf[b][h][:T], lazy.bounds, T, L, F)
            gi = G.levels_to_oracle_index(sa["heads"][h], sa["bounds"], sa["T"], F, orc.TOKEN_BALL)
            gb = G.levels_to_oracle_index(sb["heads"][h], sb["bounds"], sb["T"], F, orc.TOKEN_BALL)
            assert [gi.n(l) for l in range(L)] == [fresh.n(l) for l in range(L)] == list(n_lev[:L])
            assert gi.n(1) > gb.n(1)                               # the tree grew with the sequence
            # the chunk nodes are untouched
            assert np.array_equal(gi.center[0], gb.center[0]) and np.array_equal(gi.radius[0], gb.radius[0])
            H.check_covering_invariant(gi, Kf[b][h], slack=1e-6)
            H.check_counts(gi)
            if H.same_topology_or_near_tie(gi, fresh, L - 1, f"recluster b{b} h{h}", tally):
                for l in range(1, L):
                    live = fresh.nchunk[l] > 0
                    assert np.allclose(gi.center[l][live], fresh.center[l][live], rtol=1e-5, atol=1e-5)
                    assert np.all(gi.radius[l][live] >= fresh.radius[l][live] * (1 - 1e-6))
                    assert np.all(gi.radius[l][live] <= fresh.radius[l][live] * (1 + 5e-5) + 1e-6)
            if b == 0 and h == 0:
                _say(f"drift: mean level-1 radius {gb.radius[1][gb.nchunk[1] > 0].mean():.3f} over {gb.n(1)} nodes "
                     f"before, {gi.radius[1].mean():.3f} over {gi.n(1)} nodes after re-clustering")
    _say(f"recluster: {tally.get('same', 0)}/{w.B * w.H_kv} (seq, head) trees have the topology of the oracle's fresh build, "
         f"{tally.get('near_tie', 0)} differ behind a near-tie")
    # retrieval and attention on the re-clustered index (level walk on) agree with the oracle on it
    qb = np.stack([st.q[steps - 1] for st in streams])
    ids, _, _ = G.gpu_retrieve(case, qb, 150)
    for b in range(w.B):
        sa = after["seqs"][b]
        for h in range(w.H_kv):
            gi = G.levels_to_oracle_index(sa["heads"][h], sa["bounds"], sa["T"], F, orc.TOKEN_BALL)
            q = wl.bf16_bits_to_f64(qb[b, h * w.G:(h + 1) * w.G])
            H.accept_ids(ids[b][h], orc.node_scores(gi, 0, q), gi.lens(), 150)


def test_capacity_errors(G):
    from paper_2603_08453_amd import binding as lc
    w = wl.tiny("cap", levels=2, fanout=4, T=100)
    case = G.make_case(w)              # no room for more tokens or chunks
    k = G.to_bf16_tensor(np.zeros((1, w.H_kv, w.d), dtype=np.uint16))
    with pytest.raises(lc.LycheeError) as e:
        lc.lc_append(case.idx, case.K, case.V, k, k, [0], case.ws)
    assert e.value.code == lc.LC_ERR_CAPACITY
    import torch
    ids = torch.zeros((1, w.H_kv, 2), dtype=torch.int32, device="cuda")
    counts = torch.zeros((1, w.H_kv), dtype=torch.int32, device="cuda")
    q = G.to_bf16_tensor(case.seqs[0].Q[0][None])
    with pytest.raises(lc.LycheeError) as e:
        lc.lc_retrieve(case.idx, q, 64, ids, counts, case.ws)
    assert e.value.code == lc.LC_ERR_CAPACITY
    out = torch.zeros((1, w.H_q, w.d), dtype=torch.float32, device="cuda")
    with pytest.raises(lc.LycheeError) as e:          # the same capacity rule when the fused step is asked for ids
        lc.lc_decode_step(case.idx, q, case.K, case.V, 64, out, case.ws, chunk_ids=ids, counts=counts)
    assert e.value.code == lc.LC_ERR_CAPACITY
    with pytest.raises(lc.LycheeError) as e:          # ids and counts come together or not at all
        lc.lc_decode_step(case.idx, q, case.K, case.V, 64, out, case.ws, chunk_ids=ids)
    assert e.value.code == lc.LC_ERR_INVALID_ARG
    lc.lc_decode_step(case.idx, q, case.K, case.V, 64, out, case.ws)        # without ids no capacity is needed
    torch.cuda.synchronize()
    assert torch.isfinite(out).all()


def test_index_with_no_closed_chunk_yet(G):
    """A stream's very beginning: every token is still in the open tail.  Retrieval returns nothing,
    attention is dense attention over the tail (checked with library routines), and the first closed
    chunk is grafted into the empty tree."""
    import torch
    from paper_2603_08453_amd import binding as lc
    w = wl.tiny("empty", levels=3, fanout=4, T=50, H_q=4, H_kv=2)
    s = wl.make_sequence(w, 0, 50)
    cfg = lc.lc_config_default(levels=3, fanout=4, max_chunks=8, max_tokens=80)
    K = torch.zeros((1, 2, 80, w.d), dtype=torch.bfloat16, device="cuda")
    V = torch.zeros_like(K)
    K[0, :, :50] = G.to_bf16_tensor(s.K)
    V[0, :, :50] = G.to_bf16_tensor(s.V)
    ib = torch.zeros(lc.lc_index_bytes(cfg, 1, 2), dtype=torch.uint8, device="cuda")
    ws = torch.zeros(lc.lc_workspace_bytes(cfg, 1, 4, 2), dtype=torch.uint8, device="cuda")
    idx = lc.lc_build_index(cfg, K, [50], [[0]], ib, ws)
    assert idx.info(0)[:2] == (50, 0)
    q = G.to_bf16_tensor(s.Q[0][None])
    ids = torch.full((1, 2, 8), -1, dtype=torch.int32, device="cuda")
    counts = torch.full((1, 2), -1, dtype=torch.int32, device="cuda")
    out = torch.zeros((1, 4, w.d), dtype=torch.float32, device="cuda")
    lse = torch.zeros((1, 4), dtype=torch.float32, device="cuda")
    for fused in (False, True):
        out.fill_(float("nan"))
        if fused:
            lc.lc_decode_step(idx, q, K, V, 64, out, ws, lse=lse, chunk_ids=ids, counts=counts)
        else:
            lc.lc_retrieve(idx, q, 64, ids, counts, ws)
            lc.lc_sparse_decode(idx, q, K, V, ids, counts, out, ws, lse=lse)
        torch.cuda.synchronize()
        assert counts.cpu().numpy().tolist() == [[0, 0]]
        for h in range(2):
            ref, ref_lse = H.dense_attention_library(wl.bf16_bits_to_f64(s.Q[0][2 * h:2 * h + 2]),
                                                     wl.bf16_bits_to_f64(s.K[h]), wl.bf16_bits_to_f64(s.V[h]))
            mx, rel = G.attention_errors(out[0, 2 * h:2 * h + 2].cpu().numpy(), ref)
            assert mx <= ATTN_MAX_ABS and rel <= ATTN_REL_L2, (fused, h, mx, rel)
            assert np.all(np.abs(lse[0, 2 * h:2 * h + 2].cpu().numpy() - ref_lse) <= 1e-3)
    # the first chunk closes: 51 tokens become chunk 0, and it can be retrieved
    st = wl.make_stream(w, 0, 2)
    lc.lc_append(idx, K, V, G.to_bf16_tensor(st.k[0][None]), G.to_bf16_tensor(st.v[0][None]), [1], ws)
    lc.lc_append(idx, K, V, G.to_bf16_tensor(st.k[1][None]), G.to_bf16_tensor(st.v[1][None]), [0], ws)
    torch.cuda.synchronize()
    assert idx.info(0)[:2] == (52, 1)
    lc.lc_decode_step(idx, q, K, V, 64, out, ws, lse=lse, chunk_ids=ids, counts=counts)
    torch.cuda.synchronize()
    assert counts.cpu().numpy().tolist() == [[1, 1]] and ids[0, :, 0].cpu().numpy().tolist() == [0, 0]
    assert torch.isfinite(out).all()
    lc.lc_retrieve(idx, q, 40, ids, counts, ws)                      # the only chunk is longer than this budget
    torch.cuda.synchronize()
    assert counts.cpu().numpy().tolist() == [[0, 0]]


def test_chunker_bounds_feed_the_index(G):
    """The host chunker's boundaries are a valid chunk_bounds argument: build on them, and one decode
    step over everything equals dense attention."""
    import torch
    from paper_2603_08453_amd import binding as lc
    r = np.random.default_rng(5)
    vocab = ["the", " cat", ".", ",", "\n", "\n\n", "}", " ", "x", "foo ", ":", "y", " sat", " on", " mat"]
    T = 600
    toks = [vocab[i] for i in r.integers(0, len(vocab), size=T)]
    bounds = lc.lc_chunk_tokens(toks, 8, 16)
    lens = np.diff(bounds)
    assert bounds[0] == 0 and bounds[-1] == T and lens.max() <= 16 and lens[:-1].min() >= 8
    w = wl.tiny("chunked", levels=2, fanout=4, T=T, H_q=4, H_kv=2)
    s = wl.make_sequence(w, 0, T)
    cfg = lc.lc_config_default(levels=2, fanout=4, max_chunks=len(lens) + 4, max_tokens=T + 8)
    K = torch.zeros((1, 2, T + 8, w.d), dtype=torch.bfloat16, device="cuda")
    V = torch.zeros_like(K)
    K[0, :, :T] = G.to_bf16_tensor(s.K)
    V[0, :, :T] = G.to_bf16_tensor(s.V)
    ib = torch.zeros(lc.lc_index_bytes(cfg, 1, 2), dtype=torch.uint8, device="cuda")
    ws = torch.zeros(lc.lc_workspace_bytes(cfg, 1, 4, 2), dtype=torch.uint8, device="cuda")
    idx = lc.lc_build_index(cfg, K, [T], [bounds], ib, ws)
    assert idx.info(0)[:2] == (T, len(lens))
    out = torch.zeros((1, 4, w.d), dtype=torch.float32, device="cuda")
    lc.lc_decode_step(idx, G.to_bf16_tensor(s.Q[0][None]), K, V, T, out, ws)
    torch.cuda.synchronize()
    for h in range(2):
        ref, _ = H.dense_attention_library(wl.bf16_bits_to_f64(s.Q[0][2 * h:2 * h + 2]),
                                           wl.bf16_bits_to_f64(s.K[h]), wl.bf16_bits_to_f64(s.V[h]))
        mx, rel = G.attention_errors(out[0, 2 * h:2 * h + 2].cpu().numpy(), ref)
        assert mx <= ATTN_MAX_ABS and rel <= ATTN_REL_L2


@pytest.mark.parametrize("seed", list(range(int(__import__("os").environ.get("LC_RANDOM_CONFIGS", "24")))))
def test_random_small_configurations(G, seed):
    """Seeded random shapes: group size 1..8, 1..4 levels, odd fan-outs, ragged batches, open tails,
    sinks, both policies -- retrieval, attention and the fused step against the oracle."""
    from paper_2603_08453_amd import binding as lc
    r = np.random.default_rng(1000 + seed)
    g = int(r.integers(1, 9))
    h_kv = int(r.integers(1, 4))
    B = int(r.integers(1, 4))
    levels = int(r.integers(1, 5))
    fanout = int(r.integers(2, 9))
    lo = int(r.integers(1, 9))
    hi = lo + int(r.integers(0, 40))
    t_lo = int(r.integers(40, 600))
    w = wl.tiny(f"rand{seed}", cfg_id=1000 + seed, B=B, H_q=g * h_kv, H_kv=h_kv, levels=levels, fanout=fanout, T=0,
                T_range=(t_lo, t_lo + int(r.integers(1, 1500))), chunk_lo=lo, chunk_hi=hi)
    tails = [int(x) for x in r.integers(0, 30, size=B)]
    geometry = orc.TOKEN_BALL if r.random() < 0.7 else orc.PAPER_UNIT
    _say(f"seed {seed}: G={g} H_kv={h_kv} B={B} L={levels} F={fanout} chunks {lo}..{hi} tails {tails} geometry {geometry}")
    r2 = np.random.default_rng(7000 + seed)
    splits = int(r2.choice([0, 0, 1, 2, 7]))                      # 0 = the library's choice
    center_dtype = int(r2.integers(0, 2))                          # float32 / bfloat16 chunk centers
    case = G.make_case(w, tails=tails, geometry=geometry, prune=int(r.integers(0, 3)), decode_splits=splits,
                       center_dtype=center_dtype)
    qb = _q_batch(case, 0)
    for budget in (int(r.integers(0, 40)), int(r.integers(40, 400)), int(r.integers(400, 3000))):
        sink = int(r.integers(0, 30)) if r.random() < 0.4 else 0
        ids = _check_retrieve(G, case, qb, budget, sink=sink, tag=f"rand{seed}")
        _check_decode(G, case, qb, ids, tag=f"rand{seed} budget {budget}")
        _check_step(G, case, qb, budget, sink=sink, tag=f"rand{seed} step")
    if levels > 1:
        beam = [int(r.integers(0, 12))] + [int(r.integers(1, 6)) for _ in range(levels - 1)]
        budget = int(r.integers(50, 2000))
        _check_retrieve(G, case, qb, budget, policy=orc.POLICY_BEAM, beam=beam, tag=f"rand{seed} beam {beam}")
        _check_step(G, case, qb, budget, policy=orc.POLICY_BEAM, beam=beam, tag=f"rand{seed} step beam")
    lc.lc_set_policy(case.idx, lc.LC_POLICY_EXACT, None, 0)


@pytest.mark.parametrize("seed", list(range(int(__import__("os").environ.get("LC_RANDOM_MEDIUM_CONFIGS", "4")))))
def test_random_medium_configurations(G, seed):
    """Seeded random shapes with tens of thousands of tokens and hundreds to thousands of chunks per
    head (both sides of the chunk count at which lc_decode_step changes its kernels), forced small
    split counts (several tiles per split) and budgets of thousands of tokens."""
    from paper_2603_08453_amd import binding as lc
    r = np.random.default_rng(3000 + seed)
    g = int(r.integers(1, 9))
    h_kv = int(r.integers(1, 3))
    B = int(r.integers(1, 3))
    levels = int(r.integers(2, 5))
    fanout = int(r.integers(8, 33))
    lo = int(r.integers(4, 17))
    hi = lo + int(r.integers(0, 49))
    t_lo = int(r.integers(20000, 60000))
    w = wl.tiny(f"med{seed}", cfg_id=3000 + seed, B=B, H_q=g * h_kv, H_kv=h_kv, levels=levels, fanout=fanout, T=0,
                T_range=(t_lo, t_lo + int(r.integers(1, 30000))), chunk_lo=lo, chunk_hi=hi)
    tails = [int(x) for x in r.integers(0, 70, size=B)]
    splits = int(r.choice([0, 0, 1, 3, 8]))
    _say(f"medium seed {seed}: G={g} H_kv={h_kv} B={B} L={levels} F={fanout} chunks {lo}..{hi} tails {tails} splits {splits}")
    case = G.make_case(w, tails=tails, prune=int(r.integers(0, 3)), decode_splits=splits, center_dtype=seed % 2)
    _say(f"  chunks per sequence {[len(s.bounds) - 1 for s in case.seqs]}, tokens {[s.T for s in case.seqs]}")
    qb = _q_batch(case, 0)
    for budget in (int(r.integers(500, 3000)), int(r.integers(3000, 9000))):
        sink = int(r.integers(0, 40)) if r.random() < 0.4 else 0
        ids = _check_retrieve(G, case, qb, budget, sink=sink, tag=f"med{seed}")
        _check_decode(G, case, qb, ids, tag=f"med{seed} budget {budget}")
        _check_step(G, case, qb, budget, sink=sink, tag=f"med{seed} step")
    beam = [int(r.integers(0, 200))] + [int(r.integers(2, 20)) for _ in range(levels - 1)]
    budget = int(r.integers(1000, 5000))
    _check_retrieve(G, case, qb, budget, policy=orc.POLICY_BEAM, beam=beam, tag=f"med{seed} beam {beam}")
    _check_step(G, case, qb, budget, policy=orc.POLICY_BEAM, beam=beam, tag=f"med{seed} step beam")
    lc.lc_set_policy(case.idx, lc.LC_POLICY_EXACT, None, 0)


def test_read_sweep_reads_every_word_once(G):
    """The bandwidth probe folds (xor) exactly the words of the buffer, whatever its length."""
    import torch
    from paper_2603_08453_amd import binding as lc
    r = np.random.default_rng(11)
    for n_words in (4, 4 * 1000, 4 * (256 * 2048 * 4 + 77), 4 * 3_000_001):
        host = r.integers(0, 2 ** 31, size=n_words, dtype=np.int64).astype(np.int32)
        src = torch.from_numpy(host).cuda()
        sink = torch.full((2048,), 123, dtype=torch.int32, device="cuda")
        lc.lc_bench_read_sweep(src, sink)
        torch.cuda.synchronize()
        assert int(np.bitwise_xor.reduce(sink.cpu().numpy())) == int(np.bitwise_xor.reduce(host)), n_words


def test_graph_replays_equal_eager(G, c1):
    """The retrieval + attention calls captured in a HIP graph: every replay, with eager work and
    synchronisations in between, reproduces the eager results bit for bit (nothing in the kernels'
    cross-workgroup hand-off may depend on state left by an earlier launch)."""
    import torch
    from paper_2603_08453_amd import binding as lc
    w = c1.w
    lc.lc_set_policy(c1.idx, lc.LC_POLICY_EXACT, None, 0)
    lc.lc_set_prune(c1.idx, lc.LC_PRUNE_ALWAYS)
    qs = [G.to_bf16_tensor(np.stack([wl.make_queries(w, b, c1.seqs[b].offsets, 1, stream=200 + i)[0][0]
                                     for b in range(w.B)])) for i in range(3)]
    ids = [torch.zeros((w.B, w.H_kv, c1.cap), dtype=torch.int32, device="cuda") for _ in range(3)]
    counts = [torch.zeros((w.B, w.H_kv), dtype=torch.int32, device="cuda") for _ in range(3)]
    outs = [torch.zeros((w.B, w.H_q, w.d), dtype=torch.float32, device="cuda") for _ in range(6)]

    def work():
        for i in range(3):
            lc.lc_retrieve(c1.idx, qs[i], 700, ids[i], counts[i], c1.ws)
            lc.lc_sparse_decode(c1.idx, qs[i], c1.K, c1.V, ids[i], counts[i], outs[i], c1.ws)
            lc.lc_decode_step(c1.idx, qs[i], c1.K, c1.V, 700, outs[3 + i], c1.ws)

    work()
    torch.cuda.synchronize()
    want = [o.clone() for o in outs]
    want_ids = [(a.clone(), c.clone()) for a, c in zip(ids, counts)]
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        work()
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            work()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for rep in range(4):
        for o in outs:
            o.fill_(float("nan"))
        for a in ids:
            a.fill_(-7)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for o, ref in zip(outs, want):
            assert torch.equal(o, ref), rep
        for (a, c), (ra, rc) in zip(zip(ids, counts), want_ids):
            assert torch.equal(c, rc)
            for b in range(w.B):
                for h in range(w.H_kv):
                    n = int(c[b, h])
                    assert torch.equal(a[b, h, :n], ra[b, h, :n])
        # eager work of the same kind between the replays
        lc.lc_decode_step(c1.idx, qs[rep % 3], c1.K, c1.V, 300 + rep, outs[0], c1.ws)
        torch.cuda.synchronize()
    lc.lc_set_prune(c1.idx, lc.LC_PRUNE_ALWAYS)
