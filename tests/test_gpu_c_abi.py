"""The C ABI driven from a plain C99 program (tests/abi_gpu_driver.c, built next to the library by
the package's build step): device memory from hipMalloc, no Python and no PyTorch in that process.
The inputs come from the seeded generators through a file, the program's outputs come back through
a file and are held against the CPU oracle: Att of every step at the output tolerance, the pool
sizes after every step exactly, and at the end the retained positions exactly and the scores at
the score tolerance.  The inputs are fixed, so the run is the same every time."""
import os
import subprocess

import numpy as np
import pytest

from paper_2605_29873_amd import inputs as X
from paper_2605_29873_amd.build import C_DRIVER_PATH
from tests.harness import oracle_state, OUT_TOL, SCORE_RTOL, SCORE_ATOL

pytestmark = pytest.mark.gpu

CASES = {
    # the matrix-core kernels: bf16, 128-wide heads, chunks of 8 leave
    "bf16-chunked": (X.Workload("c-abi-bf16", batch=3, n_layers=1, n_q_heads=8, n_kv_heads=2, head_dim=128, dtype="bf16",
                                prefill_min=60, prefill_max=260, decode_budget=24, evict_trigger=31, recent_window=3,
                                alpha=0.9, steps=70, hh_prob=0.05), 0),
    # the vector-ALU kernels: fp32, 64-wide heads; the step that allocates nothing
    "f32-static-scratch": (X.Workload("c-abi-f32", batch=2, n_layers=1, n_q_heads=8, n_kv_heads=2, head_dim=64, dtype="f32",
                                      prefill_min=30, prefill_max=90, decode_budget=16, evict_trigger=20, recent_window=2,
                                      alpha=0.8, steps=50, hh_prob=0.05), 1),
    # the paper's cadence on the matrix-core kernels (the library defers compaction by itself)
    "bf16-paper-cadence": (X.Workload("c-abi-cadence", batch=2, n_layers=1, n_q_heads=14, n_kv_heads=2, head_dim=128,
                                      dtype="bf16", prefill_min=50, prefill_max=120, decode_budget=40, evict_trigger=40,
                                      recent_window=0, alpha=0.8, steps=75, hh_prob=0.05), 0),
}


@pytest.mark.parametrize("case", list(CASES))
def test_decode_loop_from_plain_c_matches_the_oracle(mkv, tmp_path, case):
    wl, static = CASES[case]
    assert os.path.exists(C_DRIVER_PATH), f"{C_DRIVER_PATH} is missing: run __graft_entry__.build() first"
    B, H, Hkv, D = wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim
    lens = [X.prefill_len(wl, s) for s in range(B)]
    f_in, f_out = tmp_path / "in.bin", tmp_path / "out.bin"
    oracles = []
    with open(f_in, "wb") as fh:
        np.array([B, H, Hkv, D, int(wl.dtype == "bf16"), wl.decode_budget, wl.evict_trigger, wl.recent_window,
                  wl.steps, static], dtype=np.int32).tofile(fh)
        np.array([wl.alpha], dtype=np.float32).tofile(fh)
        np.array(lens, dtype=np.int32).tofile(fh)
        for s in range(B):
            k, v = X.prefill_kv(wl, 0, s)
            k.astype(np.float32).tofile(fh)
            v.astype(np.float32).tofile(fh)
            st = oracle_state(wl)
            st.prefill_append(k, v)
            oracles.append(st)
        steps = [X.step_batch(wl, 0, t) for t in range(wl.steps)]
        for q, k, v in steps:
            for a in (q, k, v):
                a.astype(np.float32).tofile(fh)
    run = subprocess.run([C_DRIVER_PATH, str(f_in), str(f_out)], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0 and run.stdout.strip().endswith("ok"), run.stdout[-2000:] + run.stderr[-2000:]

    raw = np.fromfile(f_out, dtype=np.uint8)
    off = 0

    def take(n, dtype):
        nonlocal off
        a = raw[off:off + n * 4].view(dtype)
        off += n * 4
        return a

    rtol, atol = OUT_TOL[wl.dtype]
    evictions = 0
    for t, (q, k, v) in enumerate(steps):
        got = take(B * H * D, np.float32).reshape(B, H, D)
        sizes = take(B, np.int32)
        for s, st in enumerate(oracles):
            ref, _ = st.decode_step(q[s], k[s], v[s], auto_evict=True)      # Algorithm 1, capacity check included
            err = np.abs(got[s] - ref)
            assert np.all(err <= atol + rtol * np.abs(ref)), f"{case} step {t} seq {s}: Att off by {err.max():.3e}"
            assert sizes[s] == st.n_decode, f"{case} step {t} seq {s}: pool size {sizes[s]}, oracle {st.n_decode}"
            evictions += int(st.n_decode == wl.decode_budget and t >= wl.decode_budget)
    for s, st in enumerate(oracles):
        n = int(take(1, np.int32)[0])
        scores, pos = take(n, np.float32), take(n, np.int32)
        assert np.array_equal(pos, st.pos[0].astype(np.int32)), f"{case} seq {s}: retained positions differ from the oracle's"
        e = np.abs(scores.astype(np.float64) - st.I[0])
        assert np.all(e <= SCORE_RTOL * np.abs(st.I[0]) + SCORE_ATOL), f"{case} seq {s}: scores off the oracle"
    assert off == raw.size
    assert evictions >= 4 * B
