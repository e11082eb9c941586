"""Benchmark of the LycheeCluster decode hot path on one MI355X.

A step = one decode step of one attention layer over the whole batch: Eq. 2 scoring of the
chunks (with pruning when the index is large), budget selection, split-K attention over the
selected chunks and the merge -- by default through lc_decode_step (two kernels, the second one
selects and attends), with --separate through lc_retrieve followed by lc_sparse_decode.
Inputs are seeded synthetic tensors, resident in HBM before the timed region.
To keep the numbers honest about HBM, consecutive steps walk over several
replicas of (K, V, index) whose total footprint exceeds the 256 MB last-level
cache several times, and use a different query each step.

Prints one JSON line: metric/value/unit, config, roofline (dominant kernel vs HBM peak), cpu_baseline, extra.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import lc_workloads as wl  # noqa: E402

HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="C3-128K", choices=sorted(wl.WORKLOADS))
    ap.add_argument("--replicas", type=int, default=0, help="0 = 32 (or as many as fit in 64 GiB)")
    ap.add_argument("--queries", type=int, default=16)
    ap.add_argument("--policy", default="exact", choices=["exact", "beam"])
    ap.add_argument("--splits", type=int, default=0)
    ap.add_argument("--centers", default="f32", choices=["f32", "bf16"], help="storage of the chunk-level centers")
    ap.add_argument("--separate", action="store_true", help="time lc_retrieve + lc_sparse_decode instead of lc_decode_step")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--stream-steps", type=int, default=0, help="streaming workload: decode steps (0 = the workload's own)")
    ap.add_argument("--pmc-mode", action="store_true",
                    help="for rocprofv3 --pmc runs: eager steps only, then a plain device copy of known size "
                         "(2 x 256 MiB) that calibrates the byte counters")
    return ap.parse_args()



def bench_stream(args, w):
    """The streaming configuration: a prefill, then `w.stream_steps` real decode steps, each of them
    lc_append (one new token; the open chunk closes at the drawn lengths and is grafted lazily)
    followed by lc_decode_step on the grown sequence.  Four passes, each on an index of its own:
    append + decode and append alone, launched eagerly and replayed from one HIP graph that holds
    every step of the stream as its own nodes (the close decisions are by-value kernel arguments, so
    each step keeps its own).  One (K, V, index) per pass, 143 MB: the rows stay in the last-level cache
    between steps, as they would in a real stream."""
    import torch
    from paper_2603_08453_amd import binding as lc
    lc.lib()
    dev = torch.device("cuda:0")
    G, steps = w.G, (w.stream_steps if args.stream_steps <= 0 else args.stream_steps)
    s0 = wl.make_sequence(w, 0, w.T)
    st = wl.make_stream(w, 0, steps)
    M0 = len(s0.bounds) - 1
    n_close = int(st.close.sum())
    cfg = lc.lc_config_default(levels=w.levels, fanout=w.fanout, max_chunks=M0 + n_close + 8,
                               max_tokens=w.T + steps + 8, decode_splits=args.splits)
    to_t = lambda bits: torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16)
    k_dev, v_dev, q_dev = to_t(st.k).to(dev), to_t(st.v).to(dev), to_t(st.q).to(dev)
    K0 = torch.zeros((1, w.H_kv, cfg.max_tokens, w.d), dtype=torch.bfloat16, device=dev)
    V0 = torch.zeros_like(K0)
    K0[0, :, : s0.T] = to_t(s0.K).to(dev)
    V0[0, :, : s0.T] = to_t(s0.V).to(dev)
    out = torch.zeros((1, w.H_q, w.d), dtype=torch.float32, device=dev)

    def fresh():
        K, V = K0.clone(), V0.clone()
        ib = torch.zeros(lc.lc_index_bytes(cfg, 1, w.H_kv), dtype=torch.uint8, device=dev)
        ws = torch.zeros(lc.lc_workspace_bytes(cfg, 1, w.H_q, w.H_kv), dtype=torch.uint8, device=dev)
        idx = lc.lc_build_index(cfg, K, [s0.T], [s0.bounds], ib, ws)
        torch.cuda.synchronize()
        return dict(K=K, V=V, ib=ib, ws=ws, idx=idx)

    def run(rp, with_decode, lo, hi):
        for t in range(lo, hi):
            lc.lc_append(rp["idx"], rp["K"], rp["V"], k_dev[t:t + 1], v_dev[t:t + 1], [int(st.close[t])], rp["ws"])
            if with_decode:
                lc.lc_decode_step(rp["idx"], q_dev[t:t + 1], rp["K"], rp["V"], w.budget, out, rp["ws"])

    def eager(with_decode):
        rp = fresh()
        run(rp, with_decode, 0, args.warmup)              # warm-up steps are part of the stream, untimed
        torch.cuda.synchronize()
        t = time.perf_counter()
        run(rp, with_decode, args.warmup, steps)
        torch.cuda.synchronize()
        return (time.perf_counter() - t) / (steps - args.warmup) * 1e6, rp

    def graphed(with_decode):
        rp = fresh()
        side = torch.cuda.Stream()
        run(rp, with_decode, 0, args.warmup)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                run(rp, with_decode, args.warmup, steps)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        g.replay()                                        # once: a second replay would append the stream again
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (steps - args.warmup), rp

    step_eager, rp_e = eager(True)
    app_eager, _ = eager(False)
    step_graph = app_graph = None
    rp_g = None
    if not args.no_graph:
        step_graph, rp_g = graphed(True)
        app_graph, _ = graphed(False)
    # both full passes must end in the same state and give the same last output
    T_e, M_e, _ = rp_e["idx"].info(0)
    assert (T_e, M_e) == (w.T + steps, M0 + n_close), (T_e, M_e)
    if rp_g is not None:
        assert rp_g["idx"].info(0)[:2] == (T_e, M_e)
        a = lc.unpack_blob(lc.lc_index_export(rp_e["idx"]))["seqs"][0]
        b = lc.unpack_blob(lc.lc_index_export(rp_g["idx"]))["seqs"][0]
        assert all(np.array_equal(a["heads"][h][l]["center"], b["heads"][h][l]["center"])
                   for h in range(w.H_kv) for l in range(w.levels)), "graph replay and eager stream diverged"

    # the dominant kernel (selection + attention of lc_decode_step) alone, on the final state
    rp = rp_e
    q_last = q_dev[steps - 1:steps]
    ids = torch.zeros((1, w.H_kv, w.budget + 8), dtype=torch.int32, device=dev)
    counts = torch.zeros((1, w.H_kv), dtype=torch.int32, device=dev)
    lc.lc_decode_step(rp["idx"], q_last, rp["K"], rp["V"], w.budget, out, rp["ws"], chunk_ids=ids, counts=counts)
    torch.cuda.synchronize()
    blob = lc.unpack_blob(lc.lc_index_export(rp["idx"]))["seqs"][0]
    lens = np.diff(blob["bounds"].astype(np.int64))
    ih, ch = ids.cpu().numpy(), counts.cpu().numpy()
    tok = sum(int(lens[ih[0, h, : ch[0, h]]].sum()) + (T_e - int(blob["bounds"][-1])) for h in range(w.H_kv))
    dom_bytes = tok * 4 * w.d + w.H_q * w.d * 6 + M_e * w.H_kv * 12
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        lc.lc_bench_select_attend(rp["idx"], q_last, rp["K"], rp["V"], w.budget, out, rp["ws"])
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            for _ in range(200):
                lc.lc_bench_select_attend(rp["idx"], q_last, rp["K"], rp["V"], w.budget, out, rp["ws"])
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    g.replay()
    torch.cuda.synchronize()
    e0.record()
    g.replay()
    e1.record()
    torch.cuda.synchronize()
    dom_us = e0.elapsed_time(e1) * 1e3 / 200
    best = min(x for x in (step_eager, step_graph) if x is not None)
    res = {
        "metric": "us per decode step per layer (append + retrieve + attend), streaming",
        "value": round(best, 2), "unit": "us/step", "n_gpus": 1, "steps": steps - args.warmup, "warmup": args.warmup,
        "ms_per_step": round(best * 1e-3, 5), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 in, f32 accumulate", "data": "synthetic (seeded; clustered keys, drifting stream)",
        "config": {"workload": w.name, "batch": 1, "q_heads": w.H_q, "kv_heads": w.H_kv, "head_dim": w.d,
                   "prefill": w.T, "stream_steps": steps, "chunks_at_start": M0, "chunks_closed": n_close,
                   "levels": w.levels, "fanout": w.fanout, "budget": w.budget,
                   "launch": "hip-graph" if best == step_graph else "eager"},
        "roofline": {"bound": "hbm", "achieved": round(dom_bytes / (dom_us * 1e-6) / 1e9, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(dom_bytes / (dom_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4), "traffic": None,
                     "kernel": f"lc_decode_kernel<{G}, true, ...>", "bytes_per_launch": round(dom_bytes),
                     "us_per_launch": round(dom_us, 2),
                     "note": "one replica, rows resident in the last-level cache: bytes served, not HBM bytes"},
        "cpu_baseline": None,
        "extra": {"step_us_eager": round(step_eager, 2), "step_us_graph": None if step_graph is None else round(step_graph, 2),
                  "append_us_eager": round(app_eager, 2), "append_us_graph": None if app_graph is None else round(app_graph, 2),
                  "append_share_of_step_graph": None if step_graph is None else round(app_graph / step_graph, 3),
                  "tokens_attended_last_step": tok},
    }
    print(json.dumps(res), flush=True)


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build targets one GPU; --gpus must be 1 (no collectives, no sharding).",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2603_08453_amd import binding as lc
    lc.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    w = wl.WORKLOADS[args.workload]
    G = w.G
    if w.stream_steps > 0:
        bench_stream(args, w)
        return

    # ------------------------------------------------------------- inputs
    t0 = time.time()
    lens = wl.seq_lengths(w)
    seqs = [wl.make_sequence(w, b, lens[b]) for b in range(w.B)]
    Tmax = max(s.T for s in seqs)
    Mmax = max(len(s.bounds) - 1 for s in seqs)
    extra = 64
    tiers = {} if w.fanouts is None else {"fanouts": list(w.fanouts)}
    cfg = lc.lc_config_default(levels=w.levels, fanout=w.fanout, max_chunks=Mmax + extra, max_tokens=Tmax + extra,
                               decode_splits=args.splits,
                               center_dtype=lc.LC_CENTER_BF16 if args.centers == "bf16" else lc.LC_CENTER_F32, **tiers)
    # top-k per level: the workload's own beam, else 4 nodes kept at each internal level but 16 at level 1
    beam_cfg = [0] * lc.LC_MAX_LEVELS
    for l in range(1, w.levels):
        beam_cfg[l] = (w.beam[l] if w.beam is not None else (4 if l >= 2 else 16))
    if args.policy == "beam":
        cfg.policy = lc.LC_POLICY_BEAM
        for i, v in enumerate(beam_cfg):
            cfg.beam[i] = v
    to_t = lambda bits: torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16)
    K0 = torch.zeros((w.B, w.H_kv, Tmax + extra, w.d), dtype=torch.bfloat16, device=dev)
    V0 = torch.zeros_like(K0)
    for b, s in enumerate(seqs):
        K0[b, :, : s.T] = to_t(s.K).to(dev)
        V0[b, :, : s.T] = to_t(s.V).to(dev)
    nq = args.queries
    Qs = []
    for i in range(nq):
        qb = np.stack([wl.make_queries(w, b, seqs[b].offsets, 1, stream=100 + i)[0][0] for b in range(w.B)])
        Qs.append(to_t(qb).to(dev))
    index_bytes = lc.lc_index_bytes(cfg, w.B, w.H_kv)
    ws_bytes = lc.lc_workspace_bytes(cfg, w.B, w.H_q, w.H_kv)
    kv_bytes = 2 * K0.numel() * 2
    # one replica per "layer": 32 of them (as in a 32-layer model) unless that exceeds 64 GiB;
    # 32 x the index alone already exceeds the 256 MB last-level cache at the headline config
    R = args.replicas or max(2, min(32, int((64 << 30) // (kv_bytes + index_bytes))))
    gen_s = time.time() - t0

    reps = []
    build_ms = []
    for r in range(R):
        K = K0 if r == 0 else K0.clone()
        V = V0 if r == 0 else V0.clone()
        ib = torch.zeros(index_bytes, dtype=torch.uint8, device=dev)
        ws = torch.zeros(ws_bytes, dtype=torch.uint8, device=dev)
        torch.cuda.synchronize()
        tb = time.perf_counter()
        idx = lc.lc_build_index(cfg, K, [s.T for s in seqs], [s.bounds for s in seqs], ib, ws)
        torch.cuda.synchronize()
        build_ms.append((time.perf_counter() - tb) * 1e3)
        reps.append(dict(K=K, V=V, ib=ib, ws=ws, idx=idx))
    cap = int(min(Mmax + extra, w.budget + 8))
    ids_q = [torch.zeros((w.B, w.H_kv, cap), dtype=torch.int32, device=dev) for _ in range(nq)]
    counts_q = [torch.zeros((w.B, w.H_kv), dtype=torch.int32, device=dev) for _ in range(nq)]
    out = torch.zeros((w.B, w.H_q, w.d), dtype=torch.float32, device=dev)

    def retrieve(i):
        rp = reps[i % R]
        lc.lc_retrieve(rp["idx"], Qs[i % nq], w.budget, ids_q[i % nq], counts_q[i % nq], rp["ws"])

    def attend(i):
        rp = reps[i % R]
        lc.lc_sparse_decode(rp["idx"], Qs[i % nq], rp["K"], rp["V"], ids_q[i % nq], counts_q[i % nq], out, rp["ws"])

    def step_separate(i):
        retrieve(i)
        attend(i)

    def step_fused(i):
        rp = reps[i % R]
        lc.lc_decode_step(rp["idx"], Qs[i % nq], rp["K"], rp["V"], w.budget, out, rp["ws"])

    step = step_separate if args.separate else step_fused

    # ------------------------------------------------------------- algorithmic bytes
    # attended tokens per query (the index replicas are identical, so one pass over the queries suffices)
    tok_per_q, chunks_per_q, scored_per_q = [], [], []
    scores = torch.zeros((w.B, w.H_kv, cfg.max_chunks), dtype=torch.float32, device=dev)
    bounds_np = [s.bounds.astype(np.int64) for s in seqs]
    for i in range(nq):
        scores.fill_(float("nan"))          # entries past a sequence's last chunk are never written: not "scored"
        lc.lc_retrieve(reps[0]["idx"], Qs[i], w.budget, ids_q[i], counts_q[i], reps[0]["ws"], scores=scores)
        torch.cuda.synchronize()
        ih, ch, sh = ids_q[i].cpu().numpy(), counts_q[i].cpu().numpy(), scores.cpu().numpy()
        tok = 0
        for b in range(w.B):
            ln = np.diff(bounds_np[b])
            for h in range(w.H_kv):
                tok += int(ln[ih[b, h, : ch[b, h]]].sum()) + (seqs[b].T - int(bounds_np[b][-1]))
        tok_per_q.append(tok)
        chunks_per_q.append(int(ch.sum()))
        scored_per_q.append(int(np.isfinite(sh[:, :, :Mmax]).sum()))
    io_small = w.B * w.H_q * w.d * (2 + 4)
    attend_bytes = float(np.mean(tok_per_q)) * 4 * w.d + io_small
    n_upper = sum(sum(reps[0]["idx"].info(b)[2][1:]) for b in range(w.B)) * w.H_kv
    node_bytes = w.d * 4 + 4 + 4
    chunk_node_bytes = w.d * (2 if args.centers == "bf16" else 4) + 4 + 4
    retrieve_bytes = float(np.mean(scored_per_q)) * chunk_node_bytes + n_upper * node_bytes \
        + sum(len(bn) - 1 for bn in bounds_np) * w.H_kv * 8 + w.B * w.H_q * w.d * 2 + float(np.mean(chunks_per_q)) * 4

    # ------------------------------------------------------------- timing
    def timed(fn, n, start=0):
        torch.cuda.synchronize()
        t = time.perf_counter()
        for i in range(start, start + n):
            fn(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t) / n

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    eager_s = timed(step, args.steps)
    if args.pmc_mode:
        timed(step_separate if step is step_fused else step_fused, args.steps)     # the other entry points' kernels too
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"pmc_mode": True, "eager_us": round(eager_s * 1e6, 2), "calibration_copy_bytes": 256 << 20,
                          "attend_bytes": round(attend_bytes), "retrieve_bytes": round(retrieve_bytes)}), flush=True)
        return

    # HIP graphs: launch overhead out of the way.  K steps = full graphs of `unit` steps + one remainder graph.
    side = torch.cuda.Stream()

    def capture(fn, n):
        g = torch.cuda.CUDAGraph()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for i in range(4):
                fn(i)
            side.synchronize()
            with torch.cuda.graph(g, stream=side):
                for i in range(n):
                    fn(i)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        return g

    def graph_us_per_launch(fn, total):
        """Average time per call of fn over exactly `total` calls replayed from graphs, by HIP events
        recorded on the stream the graphs are launched on."""
        unit = min(total, 256)
        full, rem = divmod(total, unit)
        g_full = capture(fn, unit)
        g_rem = capture(fn, rem) if rem else None
        g_full.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t = time.perf_counter()
        e0.record()
        for _ in range(full):
            g_full.replay()
        if g_rem is not None:
            g_rem.replay()
        e1.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t) / total
        return e0.elapsed_time(e1) * 1e3 / total, wall

    graph_s = attend_us = retrieve_us = separate_s = None
    if not args.no_graph:
        try:
            _, graph_s = graph_us_per_launch(step, args.steps)
            _, separate_s = graph_us_per_launch(step_separate, args.steps)
            attend_us, _ = graph_us_per_launch(attend, args.steps)
            retrieve_us, _ = graph_us_per_launch(retrieve, args.steps)
            for i in range(nq):           # leave ids consistent with the queries again
                retrieve(i)
        except Exception as e:       # graph capture only optimises the launch path
            print(f"bench.py: HIP graph capture failed ({e}); falling back to eager event timing", file=sys.stderr)
            graph_s = None
    if attend_us is None:
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(min(args.steps, 512))]
        for i, (e0, e1) in enumerate(ev):
            retrieve(i)
            e0.record()
            attend(i)
            e1.record()
        torch.cuda.synchronize()
        attend_us = float(np.mean([e0.elapsed_time(e1) for e0, e1 in ev])) * 1e3
        for i, (e0, e1) in enumerate(ev):
            e0.record()
            retrieve(i)
            e1.record()
            attend(i)
        torch.cuda.synchronize()
        retrieve_us = float(np.mean([e0.elapsed_time(e1) for e0, e1 in ev])) * 1e3

    # The second kernel of lc_decode_step (selection + attention) by itself: back-to-back launches from
    # a graph through the measurement aid lc_bench_select_attend -- every replica's workspace still
    # holds the score keys of the query it is paired with here (replica r with query r mod nq).
    def step_fused_paired(i):
        rp = reps[i % R]
        lc.lc_decode_step(rp["idx"], Qs[(i % R) % nq], rp["K"], rp["V"], w.budget, out, rp["ws"])

    def second_kernel_paired(i):
        rp = reps[i % R]
        lc.lc_bench_select_attend(rp["idx"], Qs[(i % R) % nq], rp["K"], rp["V"], w.budget, out, rp["ws"])

    fused_us = None
    if not args.separate and not args.no_graph:
        for i in range(R):
            step_fused_paired(i)
        torch.cuda.synchronize()
        try:
            second_kernel_paired(0)
            fused_us, _ = graph_us_per_launch(second_kernel_paired, args.steps)
        except lc.LycheeError as e:          # the step does not run as score + select/attend here (too many chunks, or top-k per level)
            if e.code != lc.LC_ERR_CAPACITY:
                raise
    two_kernel_step = fused_us is not None
    if fused_us is None:
        fused_us = attend_us

    # the same step with the level-by-level walk forced on (EXACT: same ids, more kernels), and with the
    # paper's per-level top-k (BEAM: 4 nodes kept at each internal level but 16 at level 1)
    walk_us = beam_us = None
    if graph_s is not None and args.policy == "exact" and w.levels > 1:
        try:
            try:
                for rp in reps:
                    lc.lc_set_prune(rp["idx"], lc.LC_PRUNE_ALWAYS)
                step(0)
                _, t_walk = graph_us_per_launch(step, args.steps)
                walk_us = t_walk * 1e6
            except lc.LycheeError as e:      # more internal nodes than the exact walk holds on chip
                if e.code != lc.LC_ERR_CAPACITY:
                    raise
            for rp in reps:
                lc.lc_set_policy(rp["idx"], lc.LC_POLICY_BEAM, beam_cfg, 0)
            _, t_beam = graph_us_per_launch(step, args.steps)
            beam_us = t_beam * 1e6
        finally:
            for rp in reps:
                lc.lc_set_policy(rp["idx"], lc.LC_POLICY_EXACT, None, 0)
                lc.lc_set_prune(rp["idx"], lc.LC_PRUNE_AUTO)
            for i in range(nq):
                retrieve(i)
            torch.cuda.synchronize()

    # the same step on indices whose chunk-level centers are stored as bfloat16 (half the index bytes)
    half_us = None
    if graph_s is not None and args.centers == "f32" and args.policy == "exact":
        cfg_half = lc.lc_config_default(levels=w.levels, fanout=w.fanout, max_chunks=Mmax + extra,
                                        max_tokens=Tmax + extra, decode_splits=args.splits,
                                        center_dtype=lc.LC_CENTER_BF16, **tiers)
        half = []
        for rp in reps:
            ibh = torch.zeros(lc.lc_index_bytes(cfg_half, w.B, w.H_kv), dtype=torch.uint8, device=dev)
            half.append((ibh, lc.lc_build_index(cfg_half, rp["K"], [s.T for s in seqs], [s.bounds for s in seqs],
                                               ibh, rp["ws"])))
        torch.cuda.synchronize()

        def step_half(i):
            rp = reps[i % R]
            lc.lc_decode_step(half[i % R][1], Qs[i % nq], rp["K"], rp["V"], w.budget, out, rp["ws"])

        _, t_half = graph_us_per_launch(step_half, args.steps)
        half_us = t_half * 1e6
        del half

    # warm (cache-resident) figure: one replica, one query
    def step_warm(i):
        rp = reps[0]
        if args.separate:
            lc.lc_retrieve(rp["idx"], Qs[0], w.budget, ids_q[0], counts_q[0], rp["ws"])
            lc.lc_sparse_decode(rp["idx"], Qs[0], rp["K"], rp["V"], ids_q[0], counts_q[0], out, rp["ws"])
        else:
            lc.lc_decode_step(rp["idx"], Qs[0], rp["K"], rp["V"], w.budget, out, rp["ws"])
    for i in range(20):
        step_warm(i)
    warm_s = timed(step_warm, min(args.steps, 500))

    # append (lazy update), timed separately: one token per step, a chunk closes every 32 tokens
    st = wl.make_stream(w, 0, extra)
    kn = [to_t(np.stack([st.k[t]] * w.B)).to(dev) for t in range(extra)]
    vn = [to_t(np.stack([st.v[t]] * w.B)).to(dev) for t in range(extra)]
    torch.cuda.synchronize()
    ta = time.perf_counter()
    n_app = extra - 2
    for t in range(n_app):
        lc.lc_append(reps[0]["idx"], reps[0]["K"], reps[0]["V"], kn[t], vn[t],
                     [1 if (t % 32 == 31) else 0] * w.B, reps[0]["ws"])
    torch.cuda.synchronize()
    append_us = (time.perf_counter() - ta) / n_app * 1e6

    # what a plain device copy reaches on this machine (read + written bytes per second), as context for the 8 TB/s figure
    cp_src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
    cp_dst = torch.empty_like(cp_src)
    cp_dst.copy_(cp_src)
    ce0, ce1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ce0.record()
    for _ in range(5):
        cp_dst.copy_(cp_src)
    ce1.record()
    torch.cuda.synchronize()
    copy_gbps = 5 * 2 * (1 << 30) / (ce0.elapsed_time(ce1) * 1e-3) / 1e9
    # and a plain streaming read of 2 GiB (the decode path only reads)
    del cp_dst
    rd_src = torch.empty(2 << 30, dtype=torch.uint8, device=dev).fill_(1)
    rd_sink = torch.zeros(2048, dtype=torch.int32, device=dev)
    lc.lc_bench_read_sweep(rd_src, rd_sink)
    ce0.record()
    for _ in range(5):
        lc.lc_bench_read_sweep(rd_src, rd_sink)
    ce1.record()
    torch.cuda.synchronize()
    read_gbps = 5 * (2 << 30) / (ce0.elapsed_time(ce1) * 1e-3) / 1e9
    del cp_src, rd_src

    best_s = graph_s if (graph_s is not None and graph_s < eager_s) else eager_s
    step_bytes = attend_bytes + retrieve_bytes

    # ------------------------------------------------------------- CPU baseline (the oracle, as it stands)
    # Two figures on this machine's host cores: one thread, and all the cores this process may run on
    # (the affinity mask), with one (KV head) task per worker thread and the BLAS pool held at one
    # thread per worker.  The oracle is float64 numpy; nothing in it is tuned for this.
    cpu = None
    if not args.no_cpu_baseline:
        from concurrent.futures import ThreadPoolExecutor
        from oracle import lychee_oracle as orc
        from threadpoolctl import threadpool_limits
        n_aff = len(os.sched_getaffinity(0))
        b0 = 0
        s0 = seqs[b0]
        heads = list(range(w.H_kv))
        tb = time.perf_counter()
        oidx, Kf, Vf = {}, {}, {}
        for h in heads:
            Kf[h] = wl.bf16_bits_to_f64(s0.K[h])
            Vf[h] = wl.bf16_bits_to_f64(s0.V[h])
            oidx[h] = orc.build_index(Kf[h], s0.bounds, s0.T, w.levels,
                                      w.fanout if w.fanouts is None else [f if f > 0 else w.fanout for f in w.fanouts],
                                      center_dtype=orc.CENTER_BF16 if args.centers == "bf16" else orc.CENTER_F32)
            if time.perf_counter() - tb > 60 and len(oidx) >= 2:
                break
        heads = sorted(oidx)
        cpu_build_s = (time.perf_counter() - tb) / len(heads)
        qcache = [wl.bf16_bits_to_f64(wl.make_queries(w, b0, s0.offsets, 1, stream=100 + i)[0][0]) for i in range(nq)]

        def head_step(task):
            i, h = task
            q = qcache[i % nq][h * G:(h + 1) * G]
            sel = orc.retrieve_flat(oidx[h], q, w.budget)
            orc.sparse_decode(q, Kf[h], Vf[h], oidx[h].bounds, oidx[h].T, sel)

        def run(workers, seconds):
            """Seconds per decode step of one sequence (all its KV heads), and the steps that were run."""
            n_done, tc = 0, time.perf_counter()
            with threadpool_limits(limits=1):
                if workers == 1:
                    while time.perf_counter() - tc < seconds:
                        for h in heads:
                            head_step((n_done, h))
                        n_done += 1
                else:
                    with ThreadPoolExecutor(max_workers=workers) as pool:
                        while time.perf_counter() - tc < seconds:
                            batch = max(1, -(-workers // len(heads)))         # steps in flight: enough tasks for every worker
                            list(pool.map(head_step, [(n_done + k, h) for k in range(batch) for h in heads]))
                            n_done += batch
            return (time.perf_counter() - tc) / n_done * (w.H_kv / len(heads)), n_done

        one_s, one_n = run(1, args.cpu_seconds / 2)
        all_s, all_n = run(n_aff, args.cpu_seconds / 2)
        sample = (f"decode steps (flat-scan retrieve + attend) of sequence 0, {len(heads)} of {w.H_kv} KV heads, "
                  f"scaled to {w.B} sequence(s) x {w.H_kv} heads; {one_n} steps on one thread, {all_n} steps on "
                  f"{n_aff} threads (affinity mask; one head per task); oracle index build {cpu_build_s:.1f} s "
                  f"per (sequence, head), not included")
        cpu = {"value": round(all_s * w.B * 1e6, 1), "unit": "us/step", "cores": int(n_aff), "kind": "oracle",
               "sample": sample,
               "single_thread": {"value": round(one_s * w.B * 1e6, 1), "unit": "us/step", "cores": 1}}

    # dominant kernel: the attention kernel (of lc_decode_step: it also repeats the selection, whose
    # algorithmic input is one key and one boundary pair per chunk and head)
    if args.separate or not two_kernel_step:
        dom_name, dom_us, dom_bytes = f"lc_decode_kernel<{G}, false", attend_us, attend_bytes
    else:
        select_bytes = sum(len(bn) - 1 for bn in bounds_np) * w.H_kv * 12
        dom_name, dom_us, dom_bytes = f"lc_decode_kernel<{G}, true", fused_us, attend_bytes + select_bytes
    # HBM traffic of that kernel: hardware counters cannot be read from inside this process, so the figure
    # is the one of the committed rocprofv3 --pmc summary of this workload (null if there is none)
    traffic, traffic_src = None, None
    prof = os.path.join("profiles", f"lc_decode_step_{w.name}_hbm_traffic.md")
    if os.path.exists(os.path.join(ROOT, prof)):
        for ln in open(os.path.join(ROOT, prof)):
            cells = [c.strip() for c in ln.split("|")]
            if len(cells) > 7 and cells[1].startswith(dom_name) and "=" in cells[7]:
                traffic, traffic_src = int(float(cells[7].split("=")[-1])), prof
                dom_name = cells[1]
                break
    if not dom_name.endswith(">"):
        dom_name += ", 1>" if (args.separate or not two_kernel_step) else ", ...>"
    res = {
        "metric": "us per decode step per layer (retrieve+attend), 128K ctx" if w.name.startswith("C3") else
                  "us per decode step per layer (retrieve+attend)",
        "value": round(best_s * 1e6, 2),
        "unit": "us/step",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(best_s * 1e3, 5),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16 in, f32 accumulate",
        "data": "synthetic (seeded; clustered keys, queries biased to 3 chunks)",
        "config": {"workload": w.name, "batch": w.B, "q_heads": w.H_q, "kv_heads": w.H_kv, "head_dim": w.d,
                   "context": Tmax, "chunks": Mmax, "levels": w.levels, "fanout": w.fanout, "budget": w.budget,
                   "policy": args.policy, "chunk_centers": args.centers, "replicas": R, "queries": nq,
                   "entry": "lc_retrieve+lc_sparse_decode" if args.separate else "lc_decode_step",
                   "launch": "hip-graph" if best_s == graph_s else "eager"},
        "roofline": {"bound": "hbm", "achieved": round(dom_bytes / (dom_us * 1e-6) / 1e9, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(dom_bytes / (dom_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                     "traffic": traffic, "traffic_source": traffic_src, "kernel": dom_name,
                     "bytes_per_launch": round(dom_bytes), "us_per_launch": round(dom_us, 2)},
        "cpu_baseline": cpu,
        "extra": {
            "eager_us": round(eager_s * 1e6, 2),
            "graph_us": None if graph_s is None else round(graph_s * 1e6, 2),
            "warm_cache_us": round(warm_s * 1e6, 2),
            "level_walk_forced_us": None if walk_us is None else round(walk_us, 2),
            "beam_policy_us": None if beam_us is None else round(beam_us, 2),
            "bf16_chunk_centers_us": None if half_us is None else round(half_us, 2),
            "entry_points": "lc_retrieve + lc_sparse_decode" if args.separate else "lc_decode_step",
            "separate_calls_us": None if separate_s is None else round(separate_s * 1e6, 2),
            "select_attend_kernel_us_event": round(fused_us, 2),
            "retrieve_us_event": round(retrieve_us, 2),
            "attend_us_event": round(attend_us, 2),
            "attend_kernel_alone_frac_of_hbm_peak": round(attend_bytes / (attend_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
            "append_us": round(append_us, 2),
            "build_ms": round(float(np.median(build_ms)), 2),
            "device_copy_GBps": round(copy_gbps, 1),
            "device_read_GBps": round(read_gbps, 1),
            "step_bytes": round(step_bytes),
            "retrieve_bytes": round(retrieve_bytes),
            "attend_bytes": round(attend_bytes),
            "step_GBps": round(step_bytes / best_s / 1e9, 1),
            "step_frac_of_hbm_peak": round(step_bytes / best_s / 1e9 / HBM_PEAK_GBS, 4),
            "tokens_attended_per_step": round(float(np.mean(tok_per_q)), 1),
            "chunks_selected_per_step": round(float(np.mean(chunks_per_q)), 1),
            "chunks_scored_per_step": round(float(np.mean(scored_per_q)), 1),
            "input_gen_s": round(gen_s, 1),
        },
    }
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
