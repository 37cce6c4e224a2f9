"""CPU oracle of the Moment-KV decode loop.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 numpy statement of what one decode step computes, written from the paper:
Algorithm 1 ("Decoding with Moment-KV"), the attention of the KV-cache preliminaries (Eq. 2), the
head-mean (Eq. 4), the momentum update (Eq. 5), the new-token rule (Eq. 6), the capacity check
(Eq. 7), the selection (Eq. 8) and the removal (Eq. 9).  The steps are taken in the paper's order;
nothing is blocked, fused, split or reordered.  numpy's matmul/exp/lexsort serve as steps.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this file.  It
shares no code with the HIP library and imports nothing from it.

Readings taken where the paper is silent or ambiguous (each also listed in the design notes):
  R1  softmax scale is 1/sqrt(head_dim): the paper's sqrt(d) is written for a single head.
  R2  under grouped-query attention query head h reads KV head h // (H/Hkv); "mean over heads"
      (Eq. 4) runs over all H *query* heads, so there is ONE score per decode token per
      (layer, sequence) and a token leaves every KV head together.
  R3  the softmax runs over the whole pool (prefill + decode, including the token appended in
      this step); the decode slice is NOT renormalised, so sum_i abar_i = 1 - prefill mass.
  R4  the step's attention sees the cache before this step's eviction (Alg. 1 orders
      append, attend, update, evict).
  R5  eviction cadence generalised: evict iff n_d > T_e, back to exactly B_d.  T_e = B_d is the
      paper (one token per step once full).
  R6  optional recent window W: the W newest decode tokens are not candidates.  W = 0 is the
      paper: Eq. 8 draws its candidates from the whole decode pool, with no recency term.
  R7  Eq. 8 leaves ties open (any minimal-sum subset); one choice is pinned: lower score first,
      equal scores -> the older token (smaller original position) goes first.
  R8  removal is stable: survivors keep their order of generation.
  R9  the selection compares scores in the precision the caller hands in; the parity harness
      hands in float32 (the precision the device keeps scores in), the state itself stays fp64.
  R10 score_mode "per_kv_head" (a variant, not the paper): each KV head keeps its own score
      vector, averaged over its own G query heads, and evicts independently.
  R11 Alg. 1 starts from ComputeQKV(x_t) and leaves the projections and the positional encoding
      to the model.  project_kv() states the usual choice for the models the paper runs: linear
      maps k = W_k x, v = W_v x and a rotary encoding of k in the rotate-half layout -- feature i
      of a head pairs with feature i + D/2, angle pos * theta^(-2i/D).
  R12 the paper fixes no precision.  Everything is fp64 by default; `accumulate=np.float32` on
      attention_weights / attention_output (and on MomentKVState) takes the same steps with every
      product, sum and exponential in float32 -- the device's accumulation width -- so that a test
      can say how much of a device-vs-oracle gap is rounding.  Same code, other dtype.

Pins: tests/test_oracle_*.py (closed forms, invariants, a library SDPA, exhaustive subset
search).  The multi-step trajectory as a whole is "parity unpinned" against any published
number: the paper prints no worked example; it is pinned piecewise by those tests.
"""
from __future__ import annotations

import numpy as np


# ----------------------------------------------------------------------------------------------
# Alg. 1, first line: the token's key and value (R11)
# ----------------------------------------------------------------------------------------------

def rotary(k: np.ndarray, pos: int, theta: float) -> np.ndarray:
    """Rotary encoding of k [..., D] at position pos, rotate-half layout: for i < D/2 the pair
    (k[i], k[i + D/2]) is turned by the angle pos * theta**(-2i/D)."""
    k = np.asarray(k, dtype=np.float64)
    D = k.shape[-1]
    half = D // 2
    ang = float(pos) * np.power(float(theta), -2.0 * np.arange(half) / D)
    c, s_ = np.cos(ang), np.sin(ang)
    lo, hi = k[..., :half], k[..., half:]
    return np.concatenate([lo * c - hi * s_, hi * c + lo * s_], axis=-1)


def project_kv(x: np.ndarray, Wk: np.ndarray, Wv: np.ndarray, pos: int, theta: float, n_kv_heads: int):
    """k [Hkv, D] = rotary(W_k x), v [Hkv, D] = W_v x for one token (Alg. 1 ComputeQKV, the K and V
    part).  x [hidden]; Wk, Wv [Hkv*D, hidden], feature = kv_head * D + i."""
    x = np.asarray(x, dtype=np.float64)
    k = (np.asarray(Wk, dtype=np.float64) @ x).reshape(n_kv_heads, -1)
    v = (np.asarray(Wv, dtype=np.float64) @ x).reshape(n_kv_heads, -1)
    return rotary(k, pos, theta), v


# ----------------------------------------------------------------------------------------------
# Eq. 2: attention of one query over the pool
# ----------------------------------------------------------------------------------------------

def attention_weights(q: np.ndarray, K: np.ndarray, scale: float, accumulate=np.float64) -> np.ndarray:
    """A[h, j] = softmax_j(scale * <q[h], K[j, h // G]>)  (Eq. 2; Alg. 1 softmax line).

    q [H, D]; K [N, Hkv, D] (pool order: prefill tokens first, then decode tokens).
    accumulate: dtype of every product, sum and exponential (R12); fp64 unless asked otherwise.
    """
    q = np.asarray(q, dtype=accumulate)
    K = np.asarray(K, dtype=accumulate)
    H, D = q.shape
    N, Hkv, _ = K.shape
    G = H // Hkv
    A = np.empty((H, N), dtype=accumulate)
    for h in range(H):
        s = accumulate(scale) * (K[:, h // G, :] @ q[h])          # logits over the whole pool
        e = np.exp(s - s.max())
        A[h] = e / e.sum(dtype=accumulate)
    return A


def attention_output(A: np.ndarray, V: np.ndarray, accumulate=np.float64) -> np.ndarray:
    """Att[h] = sum_j A[h, j] * V[j, h // G]  (Eq. 2).  A [H, N]; V [N, Hkv, D] -> [H, D]."""
    A = np.asarray(A, dtype=accumulate)
    V = np.asarray(V, dtype=accumulate)
    H, N = A.shape
    Hkv = V.shape[1]
    G = H // Hkv
    out = np.empty((H, V.shape[2]), dtype=accumulate)
    for h in range(H):
        out[h] = A[h] @ V[:, h // G, :]
    return out


# ----------------------------------------------------------------------------------------------
# Eq. 4-6: head mean, momentum
# ----------------------------------------------------------------------------------------------

def head_mean(A_dec: np.ndarray) -> np.ndarray:
    """abar_i = (1/H) sum_h a^h[i] over the rows handed in  (Eq. 4)."""
    return np.asarray(A_dec, dtype=np.float64).sum(axis=0) / A_dec.shape[0]


def momentum_update(I: np.ndarray, abar: np.ndarray, alpha: float) -> np.ndarray:
    """I_i(t) = alpha * I_i(t-1) + abar_i(t)  (Eq. 5; Eq. 6 is the case I_i(t-1) = 0)."""
    return alpha * np.asarray(I, dtype=np.float64) + np.asarray(abar, dtype=np.float64)


# ----------------------------------------------------------------------------------------------
# Eq. 7-9: capacity, selection, removal
# ----------------------------------------------------------------------------------------------

def overflow(n_d: int, budget: int) -> int:
    """overflow = max(0, |decode pool| - B_d)  (Eq. 7)."""
    return max(0, n_d - budget)


def select_evict(scores: np.ndarray, pos: np.ndarray, n_evict: int, window: int = 0) -> np.ndarray:
    """Slots of the n_evict lowest-score candidates (Eq. 8), ascending slot order.

    Candidates are the slots [0, n - window) (R6).  Order: score, then original position (R7).
    Scores are compared exactly as given (R9).
    """
    scores = np.asarray(scores)
    n = scores.shape[0]
    n_cand = n - window
    if n_evict <= 0:
        return np.empty(0, dtype=np.int64)
    if n_evict > n_cand:
        raise ValueError("more evictions than candidates")
    order = np.lexsort((np.asarray(pos)[:n_cand], scores[:n_cand]))   # last key is primary
    return np.sort(order[:n_evict]).astype(np.int64)


def survivors(n: int, evicted: np.ndarray) -> np.ndarray:
    """Slots that stay, in their old order (Eq. 9 with R8)."""
    keep = np.ones(n, dtype=bool)
    keep[evicted] = False
    return np.nonzero(keep)[0]


# ----------------------------------------------------------------------------------------------
# Algorithm 1 for one (layer, sequence)
# ----------------------------------------------------------------------------------------------

class MomentKVState:
    """Cache pools and importance vector of one (layer, sequence), stepped by Algorithm 1."""

    def __init__(self, n_q_heads: int, n_kv_heads: int, head_dim: int, decode_budget: int,
                 alpha: float, evict_trigger: int | None = None, recent_window: int = 0,
                 softmax_scale: float | None = None, score_mode: str = "layer_mean",
                 decision_dtype=np.float32, accumulate=np.float64):
        assert n_q_heads % n_kv_heads == 0
        self.H, self.Hkv, self.D = n_q_heads, n_kv_heads, head_dim
        self.G = n_q_heads // n_kv_heads
        self.budget = decode_budget
        self.trigger = decode_budget if evict_trigger is None else evict_trigger   # R5
        self.window = recent_window                                                 # R6
        self.alpha = float(alpha)
        self.scale = 1.0 / np.sqrt(head_dim) if softmax_scale is None else float(softmax_scale)  # R1
        self.score_mode = score_mode
        self.decision_dtype = decision_dtype                                        # R9
        self.accumulate = accumulate                                                # R12
        self.Kp = np.zeros((0, n_kv_heads, head_dim))
        self.Vp = np.zeros((0, n_kv_heads, head_dim))
        self.frozen = False
        n_vec = 1 if score_mode == "layer_mean" else n_kv_heads
        # one pool per score vector: layer_mean -> a single pool of all KV heads (R2);
        # per_kv_head -> Hkv pools, pool g holding KV head g only (R10)
        self.Kd = [np.zeros((0, n_kv_heads if n_vec == 1 else 1, head_dim)) for _ in range(n_vec)]
        self.Vd = [np.zeros_like(k) for k in self.Kd]
        self.I = [np.zeros(0) for _ in range(n_vec)]
        self.pos = [np.zeros(0, dtype=np.int64) for _ in range(n_vec)]
        self.t = 0
        self.last_evicted = [np.empty(0, dtype=np.int64) for _ in range(n_vec)]

    # -- prefill pool (frozen once decoding starts) --------------------------------------------
    def prefill_append(self, K: np.ndarray, V: np.ndarray) -> None:
        if self.frozen:
            raise RuntimeError("prefill pool is frozen once decoding has started")
        self.Kp = np.concatenate([self.Kp, np.asarray(K, dtype=np.float64)])
        self.Vp = np.concatenate([self.Vp, np.asarray(V, dtype=np.float64)])

    def load_decode(self, K, V, scores, pos, t: int) -> None:
        """Restore a decode pool (layer_mean mode): the state a run would hold mid-way."""
        assert self.score_mode == "layer_mean"
        self.Kd[0] = np.asarray(K, dtype=np.float64).copy()
        self.Vd[0] = np.asarray(V, dtype=np.float64).copy()
        self.I[0] = np.asarray(scores, dtype=np.float64).copy()
        self.pos[0] = np.asarray(pos, dtype=np.int64).copy()
        self.t = int(t)

    @property
    def n_prefill(self) -> int:
        return self.Kp.shape[0]

    @property
    def n_decode(self) -> int:
        return self.I[0].shape[0]

    # -- Algorithm 1 ---------------------------------------------------------------------------
    def decode_step(self, q, k_new, v_new, auto_evict: bool = True):
        """One pass of Algorithm 1.  Returns (Att [H, D], abar) where abar is the head-mean
        decode-slice attention of this step (a list of Hkv vectors in per_kv_head mode)."""
        self.frozen = True
        q = np.asarray(q, dtype=np.float64)
        k_new = np.asarray(k_new, dtype=np.float64)
        v_new = np.asarray(v_new, dtype=np.float64)
        M = self.n_prefill
        # Alg. 1: pool_d <- pool_d U {(K_t, V_t)};  I <- I U {0}
        if self.score_mode == "layer_mean":
            self.Kd[0] = np.concatenate([self.Kd[0], k_new[None]])
            self.Vd[0] = np.concatenate([self.Vd[0], v_new[None]])
        else:
            for g in range(self.Hkv):
                self.Kd[g] = np.concatenate([self.Kd[g], k_new[None, g:g + 1]])
                self.Vd[g] = np.concatenate([self.Vd[g], v_new[None, g:g + 1]])
        for v in range(len(self.I)):
            self.I[v] = np.concatenate([self.I[v], [0.0]])
            self.pos[v] = np.concatenate([self.pos[v], [self.t]])
        self.t += 1

        if self.score_mode == "layer_mean":
            # pool <- prefill U decode;  A <- softmax(q K^T / sqrt(d));  Att = A V
            K = np.concatenate([self.Kp, self.Kd[0]])
            V = np.concatenate([self.Vp, self.Vd[0]])
            A = attention_weights(q, K, self.scale, self.accumulate)
            out = attention_output(A, V, self.accumulate)
            # Abar <- mean over heads;  a_dec <- Abar[|prefill|:]
            abar = head_mean(A)[M:]
            # I_i(t) <- alpha I_i(t-1) + abar_i(t) for every decode token (new one included)
            self.I[0] = momentum_update(self.I[0], abar, self.alpha)
            abar_ret = abar
        else:
            out = np.empty((self.H, self.D))
            abar_ret = []
            for g in range(self.Hkv):
                K = np.concatenate([self.Kp[:, g:g + 1], self.Kd[g]])
                V = np.concatenate([self.Vp[:, g:g + 1], self.Vd[g]])
                qg = q[g * self.G:(g + 1) * self.G]
                A = attention_weights(qg, K, self.scale, self.accumulate)
                out[g * self.G:(g + 1) * self.G] = attention_output(A, V, self.accumulate)
                abar = head_mean(A)[M:]
                self.I[g] = momentum_update(self.I[g], abar, self.alpha)
                abar_ret.append(abar)
        # if |pool_d| > trigger: evict
        if auto_evict and self.n_decode > self.trigger:
            self.evict()
        return out, abar_ret

    def evict(self) -> None:
        """Alg. 1 eviction branch: overflow (Eq. 7), selection (Eq. 8), removal (Eq. 9)."""
        for v in range(len(self.I)):
            n = self.I[v].shape[0]
            ov = overflow(n, self.budget)
            if ov == 0:
                self.last_evicted[v] = np.empty(0, dtype=np.int64)
                continue
            decision_scores = self.I[v].astype(self.decision_dtype)
            self.remove(v, select_evict(decision_scores, self.pos[v], ov, self.window))

    def remove(self, v: int, evicted: np.ndarray) -> None:
        """Eq. 9 for score vector v: the given slots leave, the survivors keep their order (R8).
        evict() calls it with its own selection; a test whose two sides split on a near-tie
        calls it with the other side's (checked) selection so that the runs stay comparable."""
        E = np.asarray(evicted, dtype=np.int64)
        keep = survivors(self.I[v].shape[0], E)
        self.last_evicted[v] = self.pos[v][E]
        self.Kd[v] = self.Kd[v][keep]
        self.Vd[v] = self.Vd[v][keep]
        self.I[v] = self.I[v][keep]
        self.pos[v] = self.pos[v][keep]
