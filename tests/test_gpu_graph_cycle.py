"""A captured HIP graph of decode steps against the same steps launched on the stream.

A decode step takes its launch geometry and (for small batches) the pool lengths from the host's
mirror, so a captured step is only valid for the pool sizes of the moment it was captured at.  In
steady state those sizes are periodic: after one whole eviction cycle (trigger - budget + 1 steps,
or spare slots + 1 steps with deferred compaction) they are back where they were.  A graph that
holds one whole cycle of mkv_decode_step_static calls -- the entry point that allocates nothing --
can therefore be replayed cycle after cycle.  Here such a graph is replayed several times, with
ordinary stream launches and synchronisations in between, and after every replay its outputs,
scores, positions, liveness and (at the end) its K/V rows must equal, bit for bit, those of a twin
context that took the same steps through mkv_decode_step on the stream.  The twin's path is the
one the other GPU tests hold against the CPU oracle; sequence 0 of the chunked bf16 case is held
against it here as well.
"""
import numpy as np
import pytest
import torch

from paper_2605_29873_amd import inputs as X
from tests.harness import make_ctx, oracle_state, to_device, from_device, OUT_TOL, SCORE_RTOL, SCORE_ATOL

pytestmark = pytest.mark.gpu

BF16 = dict(n_q_heads=8, n_kv_heads=2, head_dim=128, dtype="bf16", n_layers=1)

CASES = {
    # matrix-core kernels, selection kernel + row mover once per cycle of 8 steps
    "chunked-bf16": (X.Workload("graph-chunked", batch=3, prefill_min=150, prefill_max=400, decode_budget=48,
                                evict_trigger=55, recent_window=4, alpha=0.9, steps=0, hh_prob=0.05, **BF16), None),
    # the paper's cadence with deferred compaction: a slot marked per step, rows compacted every
    # spare + 1 = 9 steps (decode_capacity 0 = the library's default, which turns it on)
    "cadence-deferred-bf16": (X.Workload("graph-cadence", batch=2, prefill_min=90, prefill_max=200, decode_budget=40,
                                         evict_trigger=40, recent_window=0, alpha=0.8, steps=0, hh_prob=0.05, **BF16), 0),
    # vector-ALU kernels (fp32, 64-wide heads), the paper's cadence with immediate compaction
    "cadence-f32": (X.Workload("graph-f32", batch=2, n_layers=1, n_q_heads=8, n_kv_heads=2, head_dim=64, dtype="f32",
                               prefill_min=40, prefill_max=70, decode_budget=12, evict_trigger=12, recent_window=2,
                               alpha=0.9, steps=0), None),
}


@pytest.mark.parametrize("case", list(CASES))
def test_a_captured_eviction_cycle_replays_like_the_stream_launches(mkv, case):
    wl, capacity = CASES[case]
    deferred = capacity == 0
    cycle = 9 if deferred else wl.evict_trigger - wl.decode_budget + 1
    if cycle == 1:
        cycle = 4            # every step evicts one token: any number of steps is a whole number of cycles
    tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        eager = make_ctx(mkv, wl, manual_evict=False, stream=side.cuda_stream, decode_capacity=capacity)
        graph = make_ctx(mkv, wl, manual_evict=False, stream=side.cuda_stream, decode_capacity=capacity)
        st = oracle_state(wl) if case == "chunked-bf16" else None
        try:
            for s in range(wl.batch):
                k, v = X.prefill_kv(wl, 0, s)
                dk, dv = to_device(k, wl.dtype), to_device(v, wl.dtype)
                for c in (eager, graph):
                    mkv.mkv_prefill_append(c, 0, s, dk.data_ptr(), dv.data_ptr(), k.shape[0])
                if st is not None and s == 0:
                    st.prefill_append(k, v)
            # the step inputs of one cycle, fed again in every cycle (a graph holds their addresses)
            host = [X.step_batch(wl, 0, i) for i in range(cycle)]
            bank = [tuple(to_device(a, wl.dtype) for a in trio) for trio in host]
            out_e = torch.zeros((cycle, wl.batch, wl.n_q_heads, wl.head_dim), dtype=tdt, device="cuda")
            out_g = torch.zeros_like(out_e)
            t = 0

            def eager_step(ctx, static, out):
                q, k, v = bank[t % cycle]
                fn = mkv.mkv_decode_step_static if static else mkv.mkv_decode_step
                fn(ctx, 0, q.data_ptr(), k.data_ptr(), v.data_ptr(), out[t % cycle].data_ptr())

            def oracle_step():
                """Sequence 0 on the CPU; at an eviction the oracle removes what the device removed
                (that the device's choice is the rule's is the subject of other tests)."""
                q, k, v = host[t % cycle]
                ref, _ = st.decode_step(q[0], k[0], v[0], auto_evict=False)
                return ref

            # into steady state, both contexts on the stream: past the first eviction and a cycle more
            refs = {}
            for _ in range(wl.evict_trigger + 1 + 2 * cycle + 3):
                eager_step(eager, False, out_e)
                eager_step(graph, True, out_g)
                if st is not None:
                    oracle_step()
                    if st.n_decode > wl.evict_trigger:
                        torch.cuda.synchronize()
                        _, pos = mkv.mkv_read_scores(eager, 0, 0)
                        st.remove(0, np.nonzero(~np.isin(st.pos[0], pos))[0])
                t += 1
            torch.cuda.synchronize()
            assert torch.equal(out_e, out_g)
            t0 = t
            lens0 = [mkv.mkv_read_slots(graph, 0, s, wl.capacity + 80)[0].size for s in range(wl.batch)]

            # one whole cycle captured (nothing runs yet; the host mirror walks through the cycle)
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                for i in range(cycle):
                    eager_step(graph, True, out_g)
                    t += 1
            t = t0
            assert [mkv.mkv_read_slots(graph, 0, s, wl.capacity + 80)[0].size for s in range(wl.batch)] == lens0, \
                "the pool sizes did not recur after the captured cycle"

            rtol, atol = OUT_TOL[wl.dtype]
            for rep in range(4):
                out_g.zero_()
                g.replay()
                for i in range(cycle):
                    eager_step(eager, False, out_e)
                    if st is not None:
                        refs[t % cycle] = oracle_step()
                        if st.n_decode > wl.evict_trigger:
                            torch.cuda.synchronize()
                            _, pos = mkv.mkv_read_scores(eager, 0, 0)
                            st.remove(0, np.nonzero(~np.isin(st.pos[0], pos))[0])
                    t += 1
                torch.cuda.synchronize()
                assert torch.equal(out_e, out_g), f"{case} replay {rep}: Att of the replayed cycle differs from the stream launches"
                for s in range(wl.batch):
                    se, pe, le, pend_e = mkv.mkv_read_slots(eager, 0, s, wl.capacity + 80)
                    sg, pg, lg, pend_g = mkv.mkv_read_slots(graph, 0, s, wl.capacity + 80)
                    assert np.array_equal(pe, pg) and np.array_equal(le, lg) and pend_e == pend_g, \
                        f"{case} replay {rep} seq {s}: pool layout differs"
                    assert np.array_equal(se.view(np.uint32), sg.view(np.uint32)), f"{case} replay {rep} seq {s}: scores differ"
                if st is not None:
                    got = from_device(out_g)
                    for i in range(cycle):      # slot i of the bank, wherever in the cycle the capture began
                        err = np.abs(got[i, 0] - refs[i])
                        assert np.all(err <= atol + rtol * np.abs(refs[i])), f"{case} replay {rep} step {i}: Att off the oracle"
                    ss, ps = mkv.mkv_read_scores(graph, 0, 0)
                    assert np.array_equal(ps, st.pos[0].astype(np.int32))
                    e = np.abs(ss.astype(np.float64) - st.I[0])
                    assert np.all(e <= SCORE_RTOL * np.abs(st.I[0]) + SCORE_ATOL), f"{case} replay {rep}: scores off the oracle"
                # the program's own work between two replays: a few kernels and a synchronisation
                junk = torch.randn(1 << 16, device="cuda").sum()
                torch.cuda.synchronize()
                assert torch.isfinite(junk)
            # at the end the readers that compact: K/V rows, scores, positions
            dt = mkv.MKV_BF16 if wl.dtype == "bf16" else mkv.MKV_F32
            for s in range(wl.batch):
                se, pe = mkv.mkv_read_scores(eager, 0, s)
                sg, pg = mkv.mkv_read_scores(graph, 0, s)
                assert np.array_equal(pe, pg) and np.array_equal(se.view(np.uint32), sg.view(np.uint32))
                assert pe.size == wl.decode_budget or not deferred
                for h in range(wl.n_kv_heads):
                    ke, ve = mkv.mkv_read_kv(eager, 0, s, 0, h, wl.head_dim, dt)
                    kg, vg = mkv.mkv_read_kv(graph, 0, s, 0, h, wl.head_dim, dt)
                    assert np.array_equal(ke, kg) and np.array_equal(ve, vg), f"{case} seq {s} head {h}: rows differ"
        finally:
            torch.cuda.synchronize()
            mkv.mkv_destroy(eager)
            mkv.mkv_destroy(graph)
