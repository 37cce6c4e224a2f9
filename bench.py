#!/usr/bin/env python3
"""Benchmark of the Moment-KV decode hot path on one MI355X.

A "step" is one pass of the whole hot path -- append, split-K attention with logit emission,
split merge + head mean + momentum update, and (when the decode pool exceeds its trigger) selection
and in-place compaction -- for every sequence of every layer of the workload, on synthetic inputs
that are resident in HBM before the timed region starts.  bf16 layers with 128-wide heads run the
matrix-core attention kernel (attn_mq_kernel), the others the vector-ALU one (attn_split_kernel).

Prints ONE JSON line.  `value` = microseconds per decode step per layer (lower is better), with
tokens/s and the whole-step algorithmic GB/s beside it; `roofline` covers the attention kernel,
timed with start/stop HIP events attached to every launch in a second pass of the same steps; `cpu_baseline` is the
CPU oracle timed on a bounded sample of the same workload.

The metric is the step *with* its share of evictions in steady state, so the timed region always
consists of whole eviction cycles: --steps is rounded up to a multiple of the workload's eviction
cycle (64 steps for the Llama-shaped layers, 65 with deferred compaction for the Qwen-shaped one), for
the single-layer workloads to at least sixteen cycles (1024 steps and more; the mean over the whole
region is `value`, the median over its cycles is reported beside it), and the count actually timed
is reported as `steps_timed`.  Any such window holds the same number of evictions wherever it starts.  The
warm-up is --warmup steps but at least one whole cycle (reported as `warmup_run`), so that the
first eviction of the process and the first calls through the binding lie in front of the timed
region: a 64-step window (4.5 ms) right after five warm-up calls read 1-3 us per step high.
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

HBM_PEAK_GBPS = 8000.0
# Single-layer workloads: whole eviction cycles timed at least (16 cycles of 64 steps = 1024 steps).
kMinCycles = 16

# Kernel arguments in device memory: the default of this ROCm release, stated here because the
# kernels' start-up depends on it (with the arguments in host memory every launch waits for them
# across the bus: +10 us per step on every workload).  Read by the HIP runtime when it starts.
os.environ.setdefault("HIP_FORCE_DEV_KERNARG", "1")


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=80)
    ap.add_argument("--min-cycles", type=int, default=kMinCycles,
                    help="single-layer workloads time at least this many whole eviction cycles (counter runs under "
                         "rocprofv3 use 1: every kernel is serialised there)")
    ap.add_argument("--workload", default="cfg3", help="cfg1..cfg5 (default cfg3: the HBM-bound Llama-3.1-8B-shaped layer)")
    ap.add_argument("--also", default="cfg2,cfg4,cfg5", help="comma list of further workloads reported under 'others' ('' = none)")
    ap.add_argument("--split-keys", type=int, default=0)
    ap.add_argument("--attn-variant", type=int, default=0)
    ap.add_argument("--groups-per-cu", type=int, default=0)
    ap.add_argument("--q-len", type=int, default=0,
                    help="tokens per sequence and call: 0 = mkv_decode_step (the headline path); N >= 1 = "
                         "mkv_decode_step_multi with N query rows (matrix-core kernel), reported under 'multi_query'")
    ap.add_argument("--producer-hidden", type=int, default=0,
                    help="also time the step with the fused k/v producer (mkv_project_append, hidden size N) in "
                         "front of it, reported under 'producer'")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--variants", action="store_true",
                    help="also time score-rule variants of the main workload (same kernels, other parameters)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB elementwise pass (for scaling rocprofv3's FETCH_SIZE/WRITE_SIZE)")
    ap.add_argument("--cpu-seconds", type=float, default=16.0, help="CPU time budget of the oracle baseline (two legs)")
    ap.add_argument("--cpu-leg", default="", help="internal: 'seq,seconds,threads' -- run one worker leg of the CPU "
                                                  "baseline on that sequence and print [steps, wall s, cpu s]")
    return ap.parse_args()


def to_device(torch, X, x, dtype):
    if dtype == "bf16":
        return torch.from_numpy(X.bf16_bits(x).view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()


class Job:
    """One workload resident on the GPU: pools filled, decode pools at the budget, a bank of step
    inputs on the device."""

    BANK = 64

    def __init__(self, wl, split_keys=0, variant=0, gpc=0, q_len=0):
        import torch
        import paper_2605_29873_amd.binding as mkv
        from paper_2605_29873_amd import inputs as X
        self.torch, self.mkv, self.X, self.wl = torch, mkv, X, wl
        self.q_len = q_len
        self.tdtype = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
        self.lens = [X.prefill_len(wl, s) for s in range(wl.batch)]
        cfg = mkv.make_config(
            n_layers=wl.n_layers, batch=wl.batch, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads,
            head_dim=wl.head_dim, dtype=mkv.MKV_BF16 if wl.dtype == "bf16" else mkv.MKV_F32,
            max_prefill=wl.prefill_max, decode_budget=wl.decode_budget, evict_trigger=wl.evict_trigger,
            # single-query steps: the library's default capacity (one append past the trigger, plus
            # the spare slots of deferred compaction where that applies)
            decode_capacity=(wl.capacity + q_len - 1) if q_len else 0, recent_window=wl.recent_window, alpha=wl.alpha,
            softmax_scale=0.0, score_mode=0, split_keys=split_keys, attn_variant=variant, groups_per_cu=gpc,
            max_q_len=q_len,
            stream=torch.cuda.current_stream().cuda_stream)
        self.arena_bytes = mkv.mkv_required_bytes(cfg)
        self.ctx = mkv.mkv_create(cfg)
        self._fill()
        self._bank()
        self.t = 0

    def _fill(self):
        """Prefill pools and budget-full decode pools: N(0,1) values drawn on the device (torch's
        seeded generator), scores of the magnitude a momentum-accumulated attention share has."""
        torch, mkv, wl = self.torch, self.mkv, self.wl
        gen = torch.Generator(device="cuda")
        gen.manual_seed(wl.seed)
        rng = np.random.default_rng(wl.seed)
        t_now = 4 * wl.capacity
        shape_d = (wl.decode_budget, wl.n_kv_heads, wl.head_dim)
        for layer in range(wl.n_layers):
            for s in range(wl.batch):
                m = self.lens[s]
                if m:
                    k = torch.randn((m, wl.n_kv_heads, wl.head_dim), generator=gen, device="cuda", dtype=torch.float32).to(self.tdtype)
                    v = torch.randn((m, wl.n_kv_heads, wl.head_dim), generator=gen, device="cuda", dtype=torch.float32).to(self.tdtype)
                    mkv.mkv_prefill_append(self.ctx, layer, s, k.data_ptr(), v.data_ptr(), m)
                kd = torch.randn(shape_d, generator=gen, device="cuda", dtype=torch.float32).to(self.tdtype)
                vd = torch.randn(shape_d, generator=gen, device="cuda", dtype=torch.float32).to(self.tdtype)
                pos = np.sort(rng.choice(t_now, wl.decode_budget, replace=False)).astype(np.int32)
                sc = (rng.random(wl.decode_budget, dtype=np.float32) * 1e-3).astype(np.float32)
                mkv.mkv_load_decode(self.ctx, layer, s, kd.data_ptr(), vd.data_ptr(), sc, pos, t_now)
        torch.cuda.synchronize()

    def _bank(self):
        """BANK consecutive steps of the workload's seeded step inputs, per layer, on the device."""
        torch, X, wl = self.torch, self.X, self.wl
        layers = range(wl.n_layers)
        # layers beyond the first few reuse a rotated copy of the drawn inputs: drawing 32 x BANK x batch
        # Philox streams on the host would take minutes and adds nothing to a timing run
        drawn = min(wl.n_layers, 2)
        per_layer = []
        for layer in range(drawn):
            qs, ks, vs = zip(*(X.step_batch(wl, layer, 4 * wl.capacity + t) for t in range(self.BANK)))
            per_layer.append((to_device(torch, X, np.stack(qs), wl.dtype), to_device(torch, X, np.stack(ks), wl.dtype),
                              to_device(torch, X, np.stack(vs), wl.dtype)))
        if self.q_len:   # [BANK, B, heads, D] -> [BANK / q_len, B, q_len, heads, D]
            n = self.q_len
            per_layer = [tuple(a[:self.BANK // n * n].view(self.BANK // n, n, *a.shape[1:]).transpose(1, 2).contiguous()
                               for a in trio) for trio in per_layer]
        self.q = [per_layer[l % drawn][0] for l in layers]
        self.k = [per_layer[l % drawn][1] for l in layers]
        self.v = [per_layer[l % drawn][2] for l in layers]
        self.shift = [l // drawn for l in layers]
        self.out = torch.empty((wl.batch, max(1, self.q_len), wl.n_q_heads, wl.head_dim), dtype=self.tdtype, device="cuda")
        torch.cuda.synchronize()

    def close(self):
        self.mkv.mkv_destroy(self.ctx)


def run_steps(job: Job, n: int):
    mkv, ctx, wl = job.mkv, job.ctx, job.wl
    out_ptr = job.out.data_ptr()
    for _ in range(n):
        for layer in range(wl.n_layers):
            i = (job.t + job.shift[layer]) % job.q[layer].shape[0]
            if job.q_len:
                mkv.mkv_decode_step_multi(ctx, layer, job.q_len, job.q[layer][i].data_ptr(), job.k[layer][i].data_ptr(),
                                          job.v[layer][i].data_ptr(), out_ptr)
            else:
                mkv.mkv_decode_step(ctx, layer, job.q[layer][i].data_ptr(), job.k[layer][i].data_ptr(),
                                    job.v[layer][i].data_ptr(), out_ptr)
        job.t += 1


def pool_sizes(job: Job):
    """Decode pool size per sequence of layer 0 (all layers move in step)."""
    return [job.mkv.mkv_get_lens(job.ctx, 0, s)[1] for s in range(job.wl.batch)]


def algorithmic_bytes(job: Job, n_d_before: list[int]):
    """Bytes the method must move in one decode step of ONE layer, given each sequence's decode
    pool size before the step: (whole step, attention kernel).  The rows an eviction moves depend
    on the scores and are left out of the numerator, which is therefore conservative."""
    wl = job.wl
    b = wl.itemsize
    nq = max(1, job.q_len)                                # tokens appended per sequence and call
    row = wl.n_kv_heads * wl.head_dim * b * 2            # K and V bytes of one token of one layer
    attn = 0
    rest = 0
    for m, n0 in zip(job.lens, n_d_before):
        n1 = n0 + nq
        attn += (m + n1) * row                            # K, V read once
        attn += nq * wl.n_q_heads * wl.head_dim * b       # q read
        attn += nq * row                                  # append write
        rest += nq * wl.n_q_heads * wl.head_dim * b       # out write
        rest += nq * n1 * wl.n_kv_heads * 4 * 2           # decode-slice probabilities per KV group, write + read
        rest += n1 * 4 * 2                                # I read + write
    return attn + rest, attn


def time_region(job: Job, steps: int, window: int = 0):
    """Times `steps` steps between two events on the library's stream.  window > 0: an event is
    also recorded after every `window` steps (whole eviction cycles), and the per-window times come
    back as microseconds per step per layer (one event per cycle: well under 0.1 us per step)."""
    torch = job.torch
    n_win = steps // window if window and steps % window == 0 else 1
    per = steps // n_win
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(n_win + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    evs[0].record()
    for w in range(n_win):
        run_steps(job, per)
        evs[w + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    windows = [evs[w].elapsed_time(evs[w + 1]) * 1e3 / (per * job.wl.n_layers) for w in range(n_win)]
    return evs[0].elapsed_time(evs[-1]) * 1e-3, wall, windows


def deferred_compaction(wl, q_len=0, variant=0):
    """Whether the library defers compaction for this workload at its default capacity (the rule
    of include/mkv.h: trigger == budget, bf16 x 128, single-query steps, default kernel variant),
    and the spare slots it then adds."""
    on = (wl.evict_trigger == wl.decode_budget and wl.dtype == "bf16" and wl.head_dim == 128 and q_len == 0
          and variant == 0)
    return on, min(64, max(8, wl.decode_budget // 8))


def whole_cycles(wl, steps, q_len=0, variant=0):
    """`steps` rounded up to whole eviction cycles of the workload (calls, when a call appends
    q_len tokens): the pools return to the budget every `chunk` appended tokens.  With deferred
    compaction the cycle is the compaction's: spare slots + 1 steps."""
    if wl.evict_trigger >= 2**31 - 1:
        return steps
    chunk = wl.evict_trigger - wl.decode_budget + 1
    nq = max(1, q_len)
    cycle = -(-chunk // nq)                     # calls per cycle (the last call of a cycle crosses the trigger)
    deferred, spare = deferred_compaction(wl, q_len, variant)
    if deferred:
        cycle = spare + 1
    return -(-max(1, steps) // cycle) * cycle


def simulate(job, n_now, steps):
    """Algorithmic bytes and evicting steps over `steps` calls from the pool sizes n_now
    (deterministic: + q_len per call, back to the budget once above the trigger).  Returns
    (whole-step bytes, attention bytes, evicting steps, pool sizes afterwards)."""
    wl, nq = job.wl, max(1, job.q_len)
    total_bytes = attn_bytes = evict_steps = 0
    sim = list(n_now)
    for _ in range(steps):
        tb, ab = algorithmic_bytes(job, sim)
        total_bytes += tb
        attn_bytes += ab
        sim = [n + nq for n in sim]
        if any(n > wl.evict_trigger for n in sim):
            evict_steps += 1
        sim = [wl.decode_budget if n > wl.evict_trigger else n for n in sim]
    return total_bytes, attn_bytes, evict_steps, sim


def measure(wl, steps, warmup, split_keys=0, variant=0, gpc=0, q_len=0, evicts=True, min_cycles=kMinCycles):
    """evicts=False: a setting that is meant never to reach its trigger (the full-cache variant);
    its window is timed as given."""
    job = Job(wl, split_keys, variant, gpc, q_len)
    nq = max(1, q_len)
    requested = steps
    warmup_run = warmup
    if evicts:
        steps = whole_cycles(wl, steps, q_len, variant)
        if wl.n_layers == 1:
            # steady state (cf. the docstring): the warm-up passes the first eviction, and the timed
            # region is at least min_cycles whole cycles -- a window of a few milliseconds right after a
            # handful of warm-up calls mostly measures the host getting up to speed
            cycle = whole_cycles(wl, 1, q_len, variant)
            steps = max(steps, min_cycles * cycle) if cycle >= 16 else max(steps, whole_cycles(wl, 64 * min_cycles, q_len, variant))
            warmup_run = max(warmup, cycle + 8)
    try:
        run_steps(job, warmup_run)
        n_now = pool_sizes(job)
        total_bytes, _, evict_steps, n_after = simulate(job, n_now, steps)
        cycle = whole_cycles(wl, 1, q_len, variant) if evicts else 0
        gpu_s, wall_s, windows = time_region(job, steps, cycle if cycle >= 16 else 0)
        assert pool_sizes(job) == n_after, "the pools did not move as the byte count assumes"
        # second pass of the same number of steps with per-kernel events; its attention bytes are
        # counted for the pool sizes of that pass
        _, attn_bytes, evict_steps2, _ = simulate(job, n_after, steps)
        job.mkv.mkv_set_profiling(job.ctx, True)
        run_steps(job, steps)
        prof, psteps, pevict = job.mkv.mkv_read_profile(job.ctx)
        job.mkv.mkv_set_profiling(job.ctx, False)
        n_launch = steps * wl.n_layers
        assert psteps == n_launch
        finite = evicts and wl.evict_trigger < 2**31 - 1
        deferred, spare = deferred_compaction(wl, q_len, variant)
        # launches that moved rows: every evicting step, or one compaction per spare + 1 steps
        moved = steps // (spare + 1) * wl.n_layers if deferred else evict_steps2 * wl.n_layers
        assert not finite or (evict_steps > 0 and pevict == moved > 0), \
            "a timed window of a workload that evicts must contain its evictions' row moves"
        res = {
            "workload": wl.name,
            "steps_requested": requested,
            "steps_timed": steps,
            "warmup_run": warmup_run,
            "evicting_steps_in_timed_window": evict_steps,
            "deferred_compaction": bool(deferred and finite),
            "us_per_step_per_layer": gpu_s * 1e6 / n_launch,
            # the same region cut into whole eviction cycles: median, fastest and slowest cycle
            "cycle_windows": len(windows),
            "us_per_step_per_layer_median_cycle": float(np.median(windows)),
            "us_per_step_per_layer_cycle_range": [float(min(windows)), float(max(windows))],
            "ms_per_step": gpu_s * 1e3 / steps,
            "wall_ms_per_step": wall_s * 1e3 / steps,
            "tokens_per_s": wl.batch * nq * steps / gpu_s,
            "step_algorithmic_GBps": total_bytes * wl.n_layers / gpu_s / 1e9,
            "step_frac_of_hbm_peak": total_bytes * wl.n_layers / gpu_s / 1e9 / HBM_PEAK_GBPS,
            "attn_kernel_us": prof["attn_us"] / n_launch,
            "finish_kernel_us": prof["finish_us"] / n_launch,
            "evict_us_per_evicting_launch": (prof["evict_us"] / pevict) if pevict else None,
            "evicting_launches": int(pevict),
            "evict_us_per_step_amortised": prof["evict_us"] / n_launch,   # the eviction kernels' share of a step
            "attn_algorithmic_bytes_per_launch": attn_bytes / steps,
            "attn_GBps": (attn_bytes / steps) / (prof["attn_us"] / n_launch * 1e-6) / 1e9,
            "arena_GB": job.arena_bytes / 1e9,
            "pool_tokens_per_layer": int(sum(job.lens) + sum(n_now)),
        }
        return res
    finally:
        job.close()


def measure_producer(wl, hidden, steps, warmup):
    """The decode step fed by mkv_project_append (k/v projection + rotary encoding written into the
    pool) against the same step fed with ready-made k_new / v_new."""
    job = Job(wl)
    try:
        torch, mkv = job.torch, job.mkv
        n = wl.n_kv_heads * wl.head_dim
        gen = torch.Generator(device="cuda")
        gen.manual_seed(wl.seed + 1)
        draw = lambda *shape: torch.randn(shape, generator=gen, device="cuda", dtype=torch.float32)
        wk = (draw(n, hidden) / hidden ** 0.5).to(torch.bfloat16)
        wv = (draw(n, hidden) / hidden ** 0.5).to(torch.bfloat16)
        xs = draw(job.BANK, wl.batch, hidden).to(torch.bfloat16)
        pos = torch.tensor([job.lens[s] + 4 * wl.capacity for s in range(wl.batch)], dtype=torch.int32, device="cuda")
        out_ptr = job.out.data_ptr()

        def run(n_steps, fused):
            for _ in range(n_steps):
                i = job.t % job.BANK
                if fused:
                    mkv.mkv_project_append(job.ctx, 0, xs[i].data_ptr(), wk.data_ptr(), wv.data_ptr(), hidden,
                                           pos.data_ptr(), 500000.0)
                    mkv.mkv_decode_step(job.ctx, 0, job.q[0][i].data_ptr(), None, None, out_ptr)
                else:
                    mkv.mkv_decode_step(job.ctx, 0, job.q[0][i].data_ptr(), job.k[0][i].data_ptr(),
                                        job.v[0][i].data_ptr(), out_ptr)
                job.t += 1
        res = {}
        for fused in (False, True):
            run(warmup, fused)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            run(steps, fused)
            e1.record()
            torch.cuda.synchronize()
            res["fused_us_per_step" if fused else "plain_us_per_step"] = e0.elapsed_time(e1) * 1e3 / steps
        wbytes = 2 * n * hidden * 2
        res.update({"hidden": hidden, "weight_bytes": wbytes,
                    "producer_us": res["fused_us_per_step"] - res["plain_us_per_step"],
                    "note": "layer 0 only; producer_us = fused step - plain step (two launches: partial products, rotate+store)"})
        res["producer_weight_GBps"] = wbytes / (res["producer_us"] * 1e-6) / 1e9
        return res
    finally:
        job.close()


def _oracle_leg(job):
    """One timed leg of the CPU baseline (also the body of a worker process): the oracle as it
    stands on one sequence of the workload, from a budget-full decode pool, for about `seconds`,
    with the BLAS/OpenMP pools of numpy limited to `threads`.  Returns (steps, wall s, cpu s)."""
    wl, seq, seconds, threads = job
    from threadpoolctl import threadpool_limits
    from oracle import momentkv_oracle as O
    from paper_2605_29873_amd import inputs as X
    with threadpool_limits(limits=threads):
        st = O.MomentKVState(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.decode_budget, wl.alpha,
                             wl.evict_trigger, wl.recent_window)
        st.prefill_append(*X.prefill_kv(wl, 0, seq))
        t_now = 4 * wl.capacity
        st.load_decode(*X.decode_snapshot(wl, 0, seq, wl.decode_budget, t_now), t_now)
        inputs = [X.step_inputs(wl, 0, seq, t_now + t) for t in range(8)]
        n = 0
        c0, t0 = time.process_time(), time.perf_counter()
        while time.perf_counter() - t0 < seconds and n < 4096:
            st.decode_step(*inputs[n % len(inputs)])
            n += 1
        return n, time.perf_counter() - t0, time.process_time() - c0


def cpu_baseline(wl, seconds):
    """The oracle as it stands, timed on this machine's host cores in two forms, each for about
    half of `seconds`: (a) one thread, sequence 0; (b) all cores this process may use -- the
    sequences of the batch are independent, so min(batch, cores) worker processes take one sequence
    each and share the cores' threads between them.  Both are scaled to one decode step of the whole
    batch of one layer.  Runs before anything touches the GPU (the workers are fresh processes)."""
    import subprocess
    from paper_2605_29873_amd import inputs as X
    share = len(os.sched_getaffinity(0))
    for var in ("OMP_NUM_THREADS",):               # a machine's stated CPU share, where it sets one
        if os.environ.get(var, "").isdigit():
            share = max(1, min(share, int(os.environ[var])))
    n1, wall1, _ = _oracle_leg((wl, 0, seconds / 2, 1))
    single_us = wall1 / n1 * 1e6 * wl.batch
    workers = max(1, min(wl.batch, share))
    threads = max(1, share // workers)
    # one child process per worker, each this script again with --cpu-leg (prints its three numbers)
    key = next(k for k, w in X.workloads().items() if w == wl)
    procs = [subprocess.Popen([sys.executable, os.path.abspath(__file__), "--workload", key,
                               "--cpu-leg", f"{s},{seconds / 2},{threads}"], stdout=subprocess.PIPE, text=True)
             for s in range(workers)]
    legs = []
    for p in procs:
        out, _ = p.communicate()
        if p.returncode != 0:
            raise RuntimeError("a CPU-baseline worker failed")
        n, wall, cpu_s = json.loads(out.strip().splitlines()[-1])
        legs.append((n, wall, cpu_s))
    rate = sum(n / wall for n, wall, _ in legs)                   # sequence-steps per second, all workers
    used = sum(cpu / wall for _, wall, cpu in legs)
    return {"value": wl.batch / rate * 1e6, "unit": "us per decode step per layer",
            "cores": max(1, int(round(used))), "kind": "oracle",
            "sample": f"layer 0 from budget-full decode pools, numpy fp64; all cores: {workers} worker processes x "
                      f"{threads} threads on sequences 0..{workers - 1} for {seconds / 2:.0f} s "
                      f"({sum(n for n, _, _ in legs)} sequence-steps), scaled to batch {wl.batch}; single thread: "
                      f"sequence 0 (prefill {X.prefill_len(wl, 0)}), {n1} steps",
            "single_thread": {"value": single_us, "unit": "us per decode step per layer", "cores": 1},
            "nproc": os.cpu_count(), "cpu_share": share}


def variant_workloads(wl):
    """Parameter settings of the same kernels that mimic the comparison systems the paper times in
    its throughput figure (their cache rules only, not the systems): all at the decode position
    where the budgeted pools are full and a never-evicting cache holds `steps` tokens."""
    from paper_2605_29873_amd import inputs as X
    chunk = wl.evict_trigger - wl.decode_budget + 1
    full_len = min(wl.steps, 12288)
    return {
        "moment-kv (alpha, window as configured)": wl,
        "moment-kv, paper cadence (evict 1 per step, no window)":
            X.scaled(wl, evict_trigger=wl.decode_budget, recent_window=0),
        "cumulative scores + recent window (alpha=1)": X.scaled(wl, alpha=1.0),
        "instantaneous scores + recent window (alpha=0)": X.scaled(wl, alpha=0.0),
        "sliding window only (window = budget)": X.scaled(wl, recent_window=wl.decode_budget),
        f"full cache (no eviction, {full_len} decode tokens held)":
            X.scaled(wl, decode_budget=full_len, evict_trigger=full_len + 16 * chunk, recent_window=0),
    }


def attn_kernel_name(wl, variant: int) -> str:
    mfma = wl.dtype == "bf16" and wl.head_dim == 128 and (variant == 0 or variant >= 16)
    return "attn_mq_kernel" if mfma else "attn_split_kernel"


def measured_traffic(workload_key: str):
    """HBM bytes per attention launch from the committed rocprofv3 counter summary, if there is one."""
    path = os.path.join(ROOT, "profiles", f"{workload_key}_pmc.txt")
    try:
        for ln in open(path):
            if ln.startswith("traffic_bytes_per_launch:"):
                return float(ln.split(":")[1])
    except OSError:
        pass
    return None


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    from paper_2605_29873_amd import inputs as X
    wls = X.workloads()
    wl = wls[args.workload]
    if args.cpu_leg:
        seq, seconds, threads = args.cpu_leg.split(",")
        print(json.dumps(_oracle_leg((wl, int(seq), float(seconds), int(threads)))))
        return
    cpu = None if args.no_cpu_baseline else cpu_baseline(wl, args.cpu_seconds)   # before the GPU is touched
    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    import paper_2605_29873_amd.binding as mkv
    mkv.load()
    if args.calibrate_copy:   # a plain elementwise pass of known size: 1 GiB read + 1 GiB written
        src = torch.ones(256 * 1024 * 1024, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.mul(src, 2.0, out=dst)      # shows up as one elementwise kernel of 2^28 elements
        torch.cuda.synchronize()
        del src, dst
    main_res = measure(wl, args.steps, args.warmup, args.split_keys, args.attn_variant, args.groups_per_cu,
                       min_cycles=args.min_cycles)
    others = {}
    for name in [n for n in args.also.split(",") if n and n != args.workload]:
        w = wls[name]
        # many-layer jobs: one whole eviction cycle (measure() rounds up to whole cycles)
        steps = args.steps if w.n_layers == 1 else 1
        warm = args.warmup if w.n_layers == 1 else 8
        try:
            others[name] = measure(w, steps, warm, args.split_keys, args.attn_variant, args.groups_per_cu,
                                   min_cycles=args.min_cycles)
        except Exception as e:  # a side measurement must not lose the main line
            others[name] = {"error": repr(e)}
    line = {
        "metric": "\u00b5s per decode step per layer (attn+score+evict) + achieved HBM GB/s vs peak",
        "value": main_res["us_per_step_per_layer"],
        "unit": "us",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "steps_timed": main_res["steps_timed"],      # --steps rounded up to whole eviction cycles, at least sixteen
        "warmup_run": main_res["warmup_run"],        # --warmup, at least one whole eviction cycle
        "ms_per_step": main_res["ms_per_step"],
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if wl.dtype == "f32" else "bf16",   # bf16 operands, fp32 accumulation and scores
        "data": "synthetic",
        "config": {"workload": wl.name, "batch": wl.batch, "layers": wl.n_layers,
                   "heads": f"{wl.n_q_heads}q/{wl.n_kv_heads}kv x {wl.head_dim}",
                   "prefill": f"{wl.prefill_min}..{wl.prefill_max}", "decode_budget": wl.decode_budget,
                   "evict_chunk": wl.evict_trigger - wl.decode_budget + 1,
                   "recent_window": wl.recent_window, "alpha": wl.alpha},
        "tokens_per_s": main_res["tokens_per_s"],
        "hbm_GBps_whole_step": main_res["step_algorithmic_GBps"],
        "hbm_frac_whole_step": main_res["step_frac_of_hbm_peak"],
        "roofline": {"bound": "hbm", "kernel": attn_kernel_name(wl, args.attn_variant),
                     "achieved": main_res["attn_GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": main_res["attn_GBps"] / HBM_PEAK_GBPS, "traffic": measured_traffic(args.workload),
                     # the counters' bytes over the same launch time, beside the algorithmic figure
                     "traffic_GBps": (measured_traffic(args.workload) / (main_res["attn_kernel_us"] * 1e-6) / 1e9
                                      if measured_traffic(args.workload) else None),
                     "traffic_source": f"profiles/{args.workload}_pmc.txt (rocprofv3 FETCH_SIZE/WRITE_SIZE, bytes per launch)",
                     "algorithmic_bytes_per_launch": main_res["attn_algorithmic_bytes_per_launch"],
                     "avg_launch_us": main_res["attn_kernel_us"],
                     "timing": "start/stop HIP events attached to every launch, second pass of the same steps"},
        "detail": main_res,
        "others": others,
    }
    if args.q_len:
        r = measure(wl, args.steps, args.warmup, args.split_keys, args.attn_variant, args.groups_per_cu, args.q_len)
        r["q_len"] = args.q_len
        r["note"] = "one call = q_len tokens per sequence; us_per_step_per_layer is per call"
        line["multi_query"] = r
    if args.producer_hidden:
        line["producer"] = measure_producer(wl, args.producer_hidden, min(args.steps, 128), 16)
    if args.variants:
        line["variants"] = {}
        for name, w in variant_workloads(wl).items():
            r = measure(w, min(args.steps, 128), 8, args.split_keys, args.attn_variant, args.groups_per_cu,
                        evicts=not name.startswith("full cache"))
            line["variants"][name] = {k: r[k] for k in ("us_per_step_per_layer", "steps_timed", "tokens_per_s", "attn_kernel_us",
                                                         "finish_kernel_us", "evict_us_per_evicting_launch",
                                                         "evicting_launches", "pool_tokens_per_layer")}
    if cpu is not None:
        line["cpu_baseline"] = cpu
    print(json.dumps(line))


if __name__ == "__main__":
    main()
