"""CPU oracle for the ZSMerge budgeted KV-cache step.  TEST INFRASTRUCTURE ONLY.

Plain, slow NumPy written from the paper; it is the yardstick the HIP path is compared
with and shares no code with it.  Only the tests, the smoke check and the benchmark's
CPU-baseline leg may import this module; the product path never does.

What is implemented, per (layer, sequence, KV head) "unit":

  * compensated attention of one query per query head over the retained slots and the
    incoming token                                            (Eq. 4, Sec. 3.5)
  * decayed contribution scores                               (Eq. 3, Sec. 3.3)
  * the online cache update: append to the proximity set, demote its oldest token to
    the context set, evict the context token of lowest score, absorb it into the
    residual set                                              (Alg. 1)
  * residual absorption: slot choice by largest key dot product, incremental mean of
    key and value, fusion count                               (Eq. 5, Eq. 6, Sec. 3.4)
  * one-shot prefill compression: score every prompt token from the last W prompt
    queries, keep the latest B_p and the top-B_c, absorb the rest in position order
                                       (Sec. 3.2; appendix "Implementation Details")
  * Alg. 1 run literally from an empty cache (`online_prefill`), kept for tiny inputs.

Arithmetic is fp64.  *Stored* state is rounded to its storage type at every store:
token slots hold copies of input rows (already in the K/V storage dtype), residual
keys/values and scores are fp32, counts and positions are integers.  A decision that
depends on a stored float (lowest score, largest dot product) is therefore taken on the
same fp32/fp16 values the device holds.

Readings of the paper that this file fixes (each is restated where it is used):
  R1  a decode step attends over the cache *and* the incoming token itself (Eq. 1 sums
      i = 1..T although Alg. 1 appends k_T after the attention line);
  R2  the score update uses the compensated probabilities of Eq. 4;
  R3  the eviction looks at scores after this step's update (Alg. 1 writes s^(T));
  R4  ties: lowest (score, position) is evicted, highest (score, -position) is kept by
      the prefill selection, lowest residual index wins Eq. 5;
  R6  prefill is one-shot; the tokens it does not keep are absorbed by the residual set;
  R9  grouped queries: every query head has its own softmax and output, the score
      update uses the mean over the group;
  R11 an unused residual slot (w = 0) takes no part in the softmax, for every alpha.

Parity pins: tests/test_oracle_pins.py checks this file against full attention
(B >= T), a separately written eviction-only policy (B_r = 0), the arithmetic mean
(B_r = 1), closed forms of the score sums, Thm. 1, brute-force subset enumeration for
the selection, and the literal Alg. 1 trace.  `prefill_compress` (one-shot) versus
`online_prefill` (Alg. 1 from an empty cache) are different procedures and are not
expected to agree: parity unpinned between those two; only the one-shot form is the
contract.
"""
from __future__ import annotations

from collections import deque
from dataclasses import dataclass
from typing import List, Optional

import numpy as np

f32 = np.float32


def _store32(x):
    """Round to the fp32 storage type, keep carrying the value as fp64."""
    return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)


@dataclass
class StepInfo:
    """What one decode step decided (slot indices are physical slot numbers)."""
    write_slot: int        # token slot that received the incoming token
    evicted_pos: int       # original position of the evicted token, -1 if none was evicted
    merged_slot: int       # residual slot that absorbed it, -1 if none (no eviction or B_r = 0)
    cand_slots: np.ndarray  # context-set candidates the eviction chose among (after demotion)
    cand_s: np.ndarray      # their stored scores (fp32 values)
    cand_pos: np.ndarray


class UnitCache:
    """Compressed cache of one unit: K_B = [K_r | K_c | K_p] with B = B_r + B_c + B_p slots.

    Physical slots: [0, B_r) are residual slots, [B_r, B) token slots.  Which token slot
    belongs to the proximity or the context set is bookkeeping (`Kp`, `Kc`), as in Alg. 1;
    a slot freed by an eviction is reused by the incoming token.
    """

    def __init__(self, d: int, G: int, B_p: int, B_c: int, B_r: int,
                 lam: float = 0.98, alpha: float = 1.0, scale: Optional[float] = None):
        if B_p < 1:
            raise ValueError("B_p >= 1 required (the incoming token must not evict itself)")
        self.d, self.G = d, G
        self.B_p, self.B_c, self.B_r = B_p, B_c, B_r
        self.B = B_p + B_c + B_r
        self.lam, self.alpha = float(lam), float(alpha)
        self.scale = float(scale) if scale else 1.0 / np.sqrt(d)
        B = self.B
        self.K = np.zeros((B, d))
        self.V = np.zeros((B, d))
        self.pos = np.full(B, -1, dtype=np.int64)
        self.w = np.zeros(B, dtype=np.int64)       # fusion count, 0 = empty slot
        self.s = np.zeros(B)                        # stored scores (fp32 values)
        self.n_seen = 0                             # T: tokens seen so far
        self.Kp: deque = deque()                    # proximity set, oldest first (slot ids)
        self.Kc: List[int] = []                     # context set (slot ids)
        self.Kr: List[int] = []                     # residual slots in use (slot ids)

    # -- helpers ---------------------------------------------------------------------
    def _free_token_slot(self) -> int:
        for j in range(self.B_r, self.B):
            if self.w[j] == 0:
                return j
        raise AssertionError("no free token slot")

    def _absorb(self, k, v, pos, s) -> int:
        """Alg. 1, residual branch: open a residual slot while one is unused, otherwise
        Eq. 5 (largest raw dot product, lowest index on ties) then Eq. 6."""
        if self.B_r == 0:
            return -1
        if len(self.Kr) + 1 <= self.B_r:
            r = len(self.Kr)                       # residual slots are opened in index order
            self.Kr.append(r)
            self.K[r], self.V[r] = _store32(k), _store32(v)
            self.w[r], self.pos[r], self.s[r] = 1, pos, s
            return r
        dots = self.K[self.Kr] @ k
        r = self.Kr[int(np.argmax(dots))]          # argmax returns the first maximum
        w = float(self.w[r])
        self.K[r] = _store32((w * self.K[r] + k) / (w + 1.0))
        self.V[r] = _store32((w * self.V[r] + v) / (w + 1.0))
        self.w[r] += 1
        return r

    # -- decode ----------------------------------------------------------------------
    def decode_step(self, q, k_new, v_new):
        """One pass of Alg. 1's loop body for the token at position T = n_seen.

        q [G, d], k_new [d], v_new [d] (values representable in the K/V storage dtype).
        Returns (out [G, d] fp64, StepInfo).
        """
        q = np.asarray(q, dtype=np.float64).reshape(self.G, self.d)
        k_new = np.asarray(k_new, dtype=np.float64)
        v_new = np.asarray(v_new, dtype=np.float64)
        T = self.n_seen
        occ = np.flatnonzero(self.w > 0)                       # R11

        # Eq. 4 with the incoming token as the last entry (R1); w = 1 adds log 1 = 0
        z = np.empty((self.G, occ.size + 1))
        z[:, :-1] = (q @ self.K[occ].T) * self.scale + self.alpha * np.log(self.w[occ].astype(np.float64))
        z[:, -1] = (q @ k_new) * self.scale
        z -= z.max(axis=1, keepdims=True)
        e = np.exp(z)
        a = e / e.sum(axis=1, keepdims=True)
        out = a[:, :-1] @ self.V[occ] + a[:, -1:] * v_new[None, :]

        # Eq. 3 on the pooled probabilities (R2, R9); a new token starts from s = 0
        self.last_occ, self.last_a = occ, a                    # kept for inspection by tests
        abar = a.mean(axis=0)
        self.s[occ] = _store32(self.lam * self.s[occ] + abar[:-1])
        s_new = float(_store32(abar[-1]))

        # Alg. 1: the token joins the proximity set ...
        NEW = -2
        self.Kp.append(NEW)
        freed = None
        evicted_pos, merged = -1, -1
        cand = np.zeros(0, dtype=np.int64)
        if len(self.Kp) > self.B_p:
            old = self.Kp.popleft()                            # ... its oldest member is demoted ...
            self.Kc.append(old)
            if len(self.Kc) > self.B_c:                        # ... and the context set overflows
                cand = np.array(self.Kc, dtype=np.int64)
                c_hat = min(self.Kc, key=lambda j: (self.s[j], self.pos[j]))   # R3, R4
                self.Kc.remove(c_hat)
                evicted_pos = int(self.pos[c_hat])
                merged = self._absorb(self.K[c_hat].copy(), self.V[c_hat].copy(),
                                      evicted_pos, self.s[c_hat])
                freed = c_hat
        if freed is None:
            freed = self._free_token_slot()
        info = StepInfo(freed, evicted_pos, merged, cand, self.s[cand].copy(), self.pos[cand].copy())
        self.K[freed], self.V[freed] = k_new, v_new
        self.pos[freed], self.w[freed], self.s[freed] = T, 1, s_new
        self.Kp[-1] = freed
        self.n_seen = T + 1
        return out, info

    # -- prefill ---------------------------------------------------------------------
    def prefill_compress(self, Qw, K, V):
        """One-shot compression of a T-token prompt into an empty cache (R6).

        Qw [G, W, d]: the last W prompt queries (positions T-W .. T-1), W <= T; W = T
        gives the full-history score initialisation.  K, V [T, d].
        Returns the prompt scores s[T] (fp32 values) for inspection.
        """
        assert self.n_seen == 0 and not self.Kp and not self.Kc and not self.Kr
        K = np.asarray(K, dtype=np.float64)
        V = np.asarray(V, dtype=np.float64)
        T = K.shape[0]
        Qw = np.asarray(Qw, dtype=np.float64).reshape(self.G, -1, self.d)
        W = Qw.shape[1]
        assert W <= T
        s = prompt_scores(Qw, K, self.lam, self.scale)

        n_tok = self.B_p + self.B_c
        if T <= n_tok:
            keep = list(range(T))
            n_p = min(T, self.B_p)
            ctx, prox = keep[:T - n_p], keep[T - n_p:]
        else:
            prox = list(range(T - self.B_p, T))                # latest B_p tokens
            head = np.arange(T - self.B_p)
            # top-B_c by score; among equal scores the earlier position is kept (R4)
            order = sorted(head.tolist(), key=lambda t: (-s[t], t))
            ctx = sorted(order[:self.B_c])
        kept = set(ctx) | set(prox)

        j = self.B_r
        for t in ctx:
            self._put_token(j, K[t], V[t], t, s[t]); self.Kc.append(j); j += 1
        for t in prox:
            self._put_token(j, K[t], V[t], t, s[t]); self.Kp.append(j); j += 1
        for t in range(T):                                      # the rest, in position order
            if t not in kept:
                self._absorb(K[t], V[t], t, s[t])
        self.n_seen = T
        return s

    def _put_token(self, j, k, v, pos, s):
        self.K[j], self.V[j] = k, v
        self.pos[j], self.w[j], self.s[j] = pos, 1, s

    def online_prefill(self, Q, K, V):
        """Alg. 1 run literally from the empty cache over the whole prompt: one
        decode_step per prompt token.  Q [G, T, d].  Returns outputs [T, G, d]."""
        Q = np.asarray(Q, dtype=np.float64).reshape(self.G, -1, self.d)
        outs = []
        for t in range(K.shape[0]):
            o, _ = self.decode_step(Q[:, t], K[t], V[t])
            outs.append(o)
        return np.stack(outs)

    # -- state exchange (parity hook) -----------------------------------------------
    def export_state(self):
        return dict(K=self.K.copy(), V=self.V.copy(), pos=self.pos.copy(), w=self.w.copy(),
                    s=self.s.copy(), n_seen=self.n_seen)

    def import_state(self, K, V, pos, w, s, n_seen):
        """Adopt a state given slot by slot.  The set bookkeeping of Alg. 1 is rebuilt
        from the positions: the proximity set is the B_p most recent token slots (it is
        a FIFO of arrivals and positions only grow), the context set the other ones."""
        self.K[:], self.V[:] = K, V
        self.pos[:], self.w[:], self.s[:] = pos, w, s
        self.n_seen = int(n_seen)
        tok = [j for j in range(self.B_r, self.B) if self.w[j] > 0]
        tok.sort(key=lambda j: self.pos[j])
        n_p = min(len(tok), self.B_p)
        self.Kc = tok[:len(tok) - n_p]
        self.Kp = deque(tok[len(tok) - n_p:])
        self.Kr = [r for r in range(self.B_r) if self.w[r] > 0]


def prompt_scores(Qw, K, lam, scale):
    """Scores of the T prompt tokens after the prompt (Eq. 3 unrolled over the last W
    query steps, grouped queries pooled by their mean): fp32 values, shape [T].

    Query row i' of Qw is the query at position i = T - W + i'; it attends causally to
    positions t <= i (Eq. 1); its probabilities enter with weight lam**(T-1-i)."""
    G, W, d = Qw.shape
    T = K.shape[0]
    s = np.zeros(T)
    for ip in range(W):
        i = T - W + ip
        z = (Qw[:, ip, :] @ K[:i + 1].T) * scale                # [G, i+1]
        z -= z.max(axis=1, keepdims=True)
        e = np.exp(z)
        a = (e / e.sum(axis=1, keepdims=True)).mean(axis=0)
        s[:i + 1] = lam * s[:i + 1] + a                          # Eq. 3, step by step
    return _store32(s)


def full_attention_row(q, K, V, scale):
    """Eq. 1 for one query over all T keys (textbook softmax(q K^T / sqrt d) V)."""
    z = (K @ q) * scale
    z -= z.max()
    e = np.exp(z)
    a = e / e.sum()
    return a @ V, a
