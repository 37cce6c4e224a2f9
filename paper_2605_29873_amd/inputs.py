"""Seeded synthetic inputs for the Moment-KV decode loop.

This module only *draws numbers*: it holds none of the method's arithmetic (no softmax, no
score update, no selection).  Both the CPU oracle's tests and the HIP library's tests/bench take
their inputs from here so that the two sides see identical bits.

The paper evaluates on long-generation benchmarks with trained Llama-3.1-8B / Mistral-7B weights
(Experiments, "Implementation Details").  Neither the data nor the weights exist here, so the
workloads below only borrow the *shapes* (GQA 32/8 x 128 heads, decode budgets 512/1024,
multi-thousand-token generations) and the *structure* the paper's attention heat-map shows
(Observations, "Temporal Nature of Attention": sustained heavy hitters, temporary dips, bursts),
with Gaussian values.

Every stream is a counter-based Philox generator keyed by (seed, layer, seq) with the step index
and the role in the counter, so any (layer, seq, step) can be drawn independently and in any order.
Values are rounded once to the storage dtype (bf16 by round-to-nearest-even) and returned as
float32 arrays that hold exactly those values.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from functools import lru_cache
import numpy as np

_ROLE_PREFILL_K = 0
_ROLE_PREFILL_V = 1
_ROLE_STEP = 2
_ROLE_DIRECTION = 3
_ROLE_LAYOUT = 4
_ROLE_SNAPSHOT = 5
_ROLE_WEIGHT = 6
_ROLE_HIDDEN = 7

NEVER = 2**31 - 1


@dataclass(frozen=True)
class Workload:
    """One synthetic configuration (shapes + the structure of its attention pattern)."""
    name: str
    batch: int
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str                 # "f32" or "bf16": storage type of Q/K/V/out
    prefill_min: int           # per-sequence prefill length is drawn uniformly in
    prefill_max: int           # [prefill_min, prefill_max] (equal => fixed length)
    decode_budget: int         # B_d
    evict_trigger: int         # T_e: evict back to B_d when n_d > T_e  (T_e = B_d is the paper)
    recent_window: int         # W: newest W decode tokens are never candidates (0 is the paper)
    alpha: float               # momentum factor
    steps: int                 # decode steps of the full run
    hh_mode: str = "bernoulli"  # "designated": hh_count steps among the first hh_among; else i.i.d.
    hh_prob: float = 0.0
    hh_count: int = 0
    hh_among: int = 0
    hh_shift: float = 3.0      # heavy-hitter keys are shifted by hh_shift * u
    q_align: float = 0.5       # every query carries q_align * u
    burst_period: int = 0      # every burst_period steps ...
    burst_keys: int = 32       # ... the burst_keys keys appended just before carry +hh_shift * v_b
    burst_len: int = 16        # ... and the next burst_len queries carry burst_gain * v_b
    burst_gain: float = 2.0
    dip_period: int = 0        # q_align drops to 0 for the first dip_len of every dip_period steps
    dip_len: int = 0
    seed: int = 20260529

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def capacity(self) -> int:
        """Largest decode length ever held: one append past the trigger."""
        return self.evict_trigger + 1

    @property
    def itemsize(self) -> int:
        return 2 if self.dtype == "bf16" else 4


def workloads() -> dict:
    """The five configurations of the build, keyed cfg1..cfg5."""
    llama = dict(n_q_heads=32, n_kv_heads=8, head_dim=128, dtype="bf16")
    return {
        "cfg1": Workload("cfg1-tiny-f32", batch=1, n_layers=1, n_q_heads=8, n_kv_heads=2,
                         head_dim=64, dtype="f32", prefill_min=256, prefill_max=256,
                         decode_budget=64, evict_trigger=72, recent_window=8, alpha=0.9,
                         steps=200, hh_mode="designated", hh_count=4, hh_among=64),
        "cfg2": Workload("cfg2-llama8b-layer-b1", batch=1, n_layers=1, **llama,
                         prefill_min=4096, prefill_max=4096, decode_budget=1024,
                         evict_trigger=1024 + 63, recent_window=64, alpha=0.9, steps=4096,
                         hh_prob=0.01, burst_period=512),
        "cfg3": Workload("cfg3-llama8b-layer-b16-ragged", batch=16, n_layers=1, **llama,
                         prefill_min=2048, prefill_max=8192, decode_budget=2048,
                         evict_trigger=2048 + 63, recent_window=64, alpha=0.95, steps=8192,
                         hh_prob=0.01, burst_period=512),
        "cfg4": Workload("cfg4-qwen7b-layer-b8-chunk1", batch=8, n_layers=1, n_q_heads=28,
                         n_kv_heads=4, head_dim=128, dtype="bf16", prefill_min=8192,
                         prefill_max=8192, decode_budget=512, evict_trigger=512,
                         recent_window=32, alpha=0.8, steps=16384, hh_prob=0.005,
                         dip_period=128, dip_len=8),
        "cfg5": Workload("cfg5-llama8b-32layer-b32", batch=32, n_layers=32, **llama,
                         prefill_min=16384, prefill_max=16384, decode_budget=4096,
                         evict_trigger=4096 + 63, recent_window=128, alpha=0.9, steps=32768,
                         hh_prob=0.01, burst_period=512),
    }


def scaled(wl: Workload, **changes) -> Workload:
    """A copy of a workload with some fields replaced (smaller shapes for quick parity cases)."""
    return replace(wl, **changes)


# ----------------------------------------------------------------------------------------------
# storage rounding
# ----------------------------------------------------------------------------------------------

def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result is float32."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    b = (b + 0x7FFF + ((b >> 16) & 1)) & 0xFFFF0000
    return b.astype(np.uint32).view(np.float32).reshape(np.shape(x))


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of values that are already bf16-representable float32."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    assert not np.any(b & 0xFFFF), "value is not representable in bfloat16"
    return (b >> 16).astype(np.uint16).reshape(np.shape(x))


def bf16_from_bits(u: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(u, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def to_storage_values(x: np.ndarray, dtype: str) -> np.ndarray:
    x = np.asarray(x, dtype=np.float32)
    return round_bf16(x) if dtype == "bf16" else x


def storage_array(x: np.ndarray, dtype: str) -> np.ndarray:
    """The bytes handed to the device: float32, or uint16 bf16 patterns."""
    return bf16_bits(x) if dtype == "bf16" else np.ascontiguousarray(x, dtype=np.float32)


# ----------------------------------------------------------------------------------------------
# streams
# ----------------------------------------------------------------------------------------------

def _gen(wl: Workload, layer: int, seq: int, role: int, index: int = 0) -> np.random.Generator:
    key = [wl.seed & (2**64 - 1), ((layer & 0xFFFFFFFF) << 32) | (seq & 0xFFFFFFFF)]
    return np.random.Generator(np.random.Philox(key=key, counter=[0, 0, index, role]))


def prefill_len(wl: Workload, seq: int) -> int:
    """Prompt length of a sequence (same for every layer)."""
    if wl.prefill_min == wl.prefill_max:
        return wl.prefill_max
    g = _gen(wl, 0, seq, _ROLE_LAYOUT, 0)
    return int(g.integers(wl.prefill_min, wl.prefill_max + 1))


@lru_cache(maxsize=256)
def direction(wl: Workload, index: int = 0) -> np.ndarray:
    """Unit vector in R^D: index 0 is the shared heavy-hitter direction u, b>=1 the burst v_b."""
    g = _gen(wl, 0, 0, _ROLE_DIRECTION, index)
    v = g.standard_normal(wl.head_dim)
    return (v / np.linalg.norm(v)).astype(np.float32)


def prefill_kv(wl: Workload, layer: int, seq: int, n_tokens: int | None = None):
    """K, V of the prompt: iid N(0,1), shape [M, Hkv, D], storage-rounded float32."""
    m = prefill_len(wl, seq) if n_tokens is None else n_tokens
    shape = (m, wl.n_kv_heads, wl.head_dim)
    k = _gen(wl, layer, seq, _ROLE_PREFILL_K).standard_normal(shape, dtype=np.float32)
    v = _gen(wl, layer, seq, _ROLE_PREFILL_V).standard_normal(shape, dtype=np.float32)
    return to_storage_values(k, wl.dtype), to_storage_values(v, wl.dtype)


@lru_cache(maxsize=4096)
def heavy_hitter_steps(wl: Workload, layer: int, seq: int) -> np.ndarray:
    """Designated mode only: the decode steps whose keys are heavy hitters."""
    g = _gen(wl, layer, seq, _ROLE_LAYOUT, 1)
    return np.sort(g.choice(wl.hh_among, size=wl.hh_count, replace=False))


def is_heavy_hitter(wl: Workload, layer: int, seq: int, t: int) -> bool:
    if wl.hh_mode == "designated":
        return bool(t in set(heavy_hitter_steps(wl, layer, seq).tolist()))
    if wl.hh_prob <= 0.0:
        return False
    g = _gen(wl, layer, seq, _ROLE_LAYOUT, 2 + t)
    return bool(g.random() < wl.hh_prob)


def step_inputs(wl: Workload, layer: int, seq: int, t: int):
    """q [H,D], k_new [Hkv,D], v_new [Hkv,D] of decode step t (0-based), storage-rounded."""
    g = _gen(wl, layer, seq, _ROLE_STEP, t)
    q = g.standard_normal((wl.n_q_heads, wl.head_dim), dtype=np.float32)
    k = g.standard_normal((wl.n_kv_heads, wl.head_dim), dtype=np.float32)
    v = g.standard_normal((wl.n_kv_heads, wl.head_dim), dtype=np.float32)
    u = direction(wl, 0)
    beta = wl.q_align
    if wl.dip_period and (t % wl.dip_period) < wl.dip_len:
        beta = 0.0
    q = q + np.float32(beta) * u
    if is_heavy_hitter(wl, layer, seq, t):
        k = k + np.float32(wl.hh_shift) * u
    if wl.burst_period:
        b_next = t // wl.burst_period + 1           # keys just before burst b_next
        if b_next * wl.burst_period - wl.burst_keys <= t < b_next * wl.burst_period:
            k = k + np.float32(wl.hh_shift) * direction(wl, b_next)
        b_cur = t // wl.burst_period                 # queries just after burst b_cur
        if b_cur >= 1 and t - b_cur * wl.burst_period < wl.burst_len:
            q = q + np.float32(wl.burst_gain) * direction(wl, b_cur)
    return (to_storage_values(q, wl.dtype), to_storage_values(k, wl.dtype),
            to_storage_values(v, wl.dtype))


def step_batch(wl: Workload, layer: int, t: int):
    """Step inputs of every sequence: q [B,H,D], k [B,Hkv,D], v [B,Hkv,D]."""
    qs, ks, vs = zip(*(step_inputs(wl, layer, s, t) for s in range(wl.batch)))
    return np.stack(qs), np.stack(ks), np.stack(vs)


def decode_snapshot(wl: Workload, layer: int, seq: int, n_d: int, t_now: int):
    """A synthetic mid-run decode pool, so that a parity case can start near an eviction
    without replaying thousands of steps: n_d keys/values drawn like step inputs, strictly
    increasing original positions below t_now, and positive scores of the magnitude a
    momentum-accumulated attention share has.  Returns (K [n_d,Hkv,D], V, scores f32, pos i32)."""
    g = _gen(wl, layer, seq, _ROLE_SNAPSHOT, n_d)
    shape = (n_d, wl.n_kv_heads, wl.head_dim)
    k = to_storage_values(g.standard_normal(shape, dtype=np.float32), wl.dtype)
    v = to_storage_values(g.standard_normal(shape, dtype=np.float32), wl.dtype)
    pos = np.sort(g.choice(t_now, size=n_d, replace=False)).astype(np.int32)
    scores = (g.random(n_d, dtype=np.float32) * np.float32(1e-3)).astype(np.float32)
    return k, v, scores, pos


def projection_weights(wl: Workload, layer: int, hidden: int):
    """W_k, W_v [Hkv*D, hidden] of one layer (one row per output feature), N(0, 1/hidden) so that
    the projected rows have unit variance like the other synthetic keys; storage-rounded."""
    g = _gen(wl, layer, 0, _ROLE_WEIGHT, hidden)
    n = wl.n_kv_heads * wl.head_dim
    sd = np.float32(1.0 / np.sqrt(hidden))
    wk = g.standard_normal((n, hidden), dtype=np.float32) * sd
    wv = g.standard_normal((n, hidden), dtype=np.float32) * sd
    return to_storage_values(wk, wl.dtype), to_storage_values(wv, wl.dtype)


def step_hidden(wl: Workload, layer: int, t: int, hidden: int) -> np.ndarray:
    """The layer input x_t of every sequence at decode step t: [B, hidden], N(0,1), storage-rounded."""
    rows = [_gen(wl, layer, s, _ROLE_HIDDEN, t).standard_normal(hidden, dtype=np.float32)
            for s in range(wl.batch)]
    return to_storage_values(np.stack(rows), wl.dtype)
