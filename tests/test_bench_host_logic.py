"""Host-side arithmetic of bench.py (no GPU): which step counts it times, how it counts the
algorithmic bytes, and that the timed window of every workload that evicts holds evictions."""
import types

import numpy as np
import pytest

import bench
from paper_2605_29873_amd import inputs as X

WL = X.workloads()


def test_timed_steps_are_whole_eviction_cycles():
    # chunks of 64 (cfg2, cfg3, cfg5), the deferred compaction's 64 spare slots + 1 (cfg4), cfg1's chunk of 9
    assert bench.whole_cycles(WL["cfg3"], 20) == 64
    assert bench.whole_cycles(WL["cfg3"], 65) == 128
    assert bench.whole_cycles(WL["cfg2"], 1) == 64
    assert bench.whole_cycles(WL["cfg5"], 1) == 64
    assert bench.whole_cycles(WL["cfg4"], 20) == 65
    assert bench.whole_cycles(WL["cfg1"], 20) == 27
    # several tokens per call: a cycle is chunk / q_len calls, rounded up; no deferral with q_len > 0
    assert bench.whole_cycles(WL["cfg3"], 1, q_len=4) == 16
    assert bench.whole_cycles(WL["cfg4"], 1, q_len=2) == 1
    # a context that never evicts is timed as asked
    never = X.scaled(WL["cfg3"], evict_trigger=X.NEVER)
    assert bench.whole_cycles(never, 20) == 20


def test_deferred_compaction_rule_mirrors_the_library_default():
    on, spare = bench.deferred_compaction(WL["cfg4"])
    assert on and spare == 64                       # budget 512 / 8
    assert not bench.deferred_compaction(WL["cfg3"])[0]          # chunked eviction
    assert not bench.deferred_compaction(WL["cfg4"], q_len=2)[0]
    assert not bench.deferred_compaction(WL["cfg4"], variant=15)[0]
    assert bench.deferred_compaction(X.scaled(WL["cfg4"], decode_budget=40, evict_trigger=40))[1] == 8


def _job(wl, lens, q_len=0):
    return types.SimpleNamespace(wl=wl, lens=lens, q_len=q_len)


def test_algorithmic_bytes_follow_the_kv_footprint():
    # one Llama-shaped token of one layer is 4096 bytes of K and V (tests/golden/kv_footprint.txt)
    wl = WL["cfg3"]
    job = _job(wl, [1000, 3000])
    total, attn = bench.algorithmic_bytes(job, [2048, 2100])
    keys = (1000 + 2049) + (3000 + 2101)
    q_and_append = 2 * (32 * 128 * 2 + 4096)
    assert attn == keys * 4096 + q_and_append
    rest = 2 * 32 * 128 * 2 + (2049 + 2101) * (8 * 4 * 2 + 4 * 2)
    assert total == attn + rest
    # four tokens per call: the pool is read once for all four
    job4 = _job(wl, [1000, 3000], q_len=4)
    _, attn4 = bench.algorithmic_bytes(job4, [2048, 2100])
    assert attn4 == ((1000 + 2052) + (3000 + 2104)) * 4096 + 4 * q_and_append


@pytest.mark.parametrize("name", ["cfg2", "cfg3", "cfg5"])
def test_any_window_of_whole_cycles_holds_the_same_evictions(name):
    wl = WL[name]
    job = _job(wl, [wl.prefill_max] * wl.batch)
    steps = bench.whole_cycles(wl, 100)
    counts = set()
    for start in (wl.decode_budget, wl.decode_budget + 1, wl.decode_budget + 40, wl.evict_trigger):
        _, _, evict_steps, after = bench.simulate(job, [start] * wl.batch, steps)
        counts.add(evict_steps)
        assert after == [start] * wl.batch          # a whole number of cycles brings the pools back
    assert counts == {steps // 64}


def test_gpus_above_one_are_refused(monkeypatch, capsys):
    monkeypatch.setattr("sys.argv", ["bench.py", "--gpus", "2"])
    with pytest.raises(SystemExit) as e:
        bench.main()
    assert e.value.code == 2
    assert "one GPU" in capsys.readouterr().err
