"""Seeded synthetic workloads for the budgeted KV-cache step (inputs only).

This module produces the inputs that both the HIP path and the CPU oracle consume:
Llama-shaped Q/K/V with skewed attention, and the table of workload shapes.  It holds
none of the method's arithmetic (no attention, no scores, no merging) and imports
neither the HIP binding nor the oracle.

Generator.  Every value is a pure function of
(master seed, tensor id, layer, sequence, head, position, channel): a 64-bit integer
hash (splitmix64 finaliser) gives two uniforms, a Box-Muller step in fp64 gives one
N(0,1) draw, which is then rounded to the storage dtype.  Any slice can therefore be
regenerated in isolation and on either device.  (CPU and GPU transcendental functions
may differ in the last bit, so a parity test always hands the *same bytes* to both
sides: it generates once and copies.)

Structure of the data (stand-in for the efficiency runs' undisclosed synthetic
prompts; experiment section, "Benchmark Diversity"):
  * K, V, Q rows are i.i.d. N(0,1);
  * per (layer, KV head) a unit direction u and four outlier channels;
  * positions 0..3 are attention sinks (strength 4), every other position is a heavy
    hitter with probability 0.02 (strength 3): k += c * d**0.25 * u;
  * every query gets q += d**0.25 * u, so a boosted key's logit is shifted by about +c
    while the others stay about N(0,1);
  * workloads 1..4 multiply the four outlier channels of K by 8 (after the boost).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import torch

MASTER_SEED = 20250310

_M64 = (1 << 64) - 1
_GOLD = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB

TID_K, TID_V, TID_Q, TID_DIR, TID_OUTLIER, TID_HEAVY, TID_LEN = 1, 2, 3, 4, 5, 6, 7
TID_DK, TID_DV, TID_DQ, TID_DHEAVY = 11, 12, 13, 16


def _mix_py(x: int) -> int:
    x &= _M64
    x ^= x >> 30
    x = (x * _C1) & _M64
    x ^= x >> 27
    x = (x * _C2) & _M64
    x ^= x >> 31
    return x


def key_of(*parts: int) -> int:
    """Chain the integer parts into one 64-bit stream key (host side)."""
    h = 0
    for p in parts:
        h = _mix_py((h + _GOLD + (p & _M64)) & _M64)
    return h


def _signed(x: int) -> int:
    return x - (1 << 64) if x >= (1 << 63) else x


def _lsr(x: torch.Tensor, k: int) -> torch.Tensor:
    return (x >> k) & ((1 << (64 - k)) - 1)


def _mix_t(x: torch.Tensor) -> torch.Tensor:
    x = x ^ _lsr(x, 30)
    x = x * _signed(_C1)
    x = x ^ _lsr(x, 27)
    x = x * _signed(_C2)
    x = x ^ _lsr(x, 31)
    return x


def uniform01(keys: torch.Tensor, counters: torch.Tensor, lane: int) -> torch.Tensor:
    """Uniform in (0,1] from the top 53 bits of hash(key, counter, lane); fp64."""
    x = keys + counters * _signed(_GOLD) + _signed((lane * 0xD1B54A32D192ED03) & _M64)
    bits = _lsr(_mix_t(x), 11)
    return (bits.to(torch.float64) + 1.0) * (1.0 / 9007199254740992.0)


def normal(keys: torch.Tensor, counters: torch.Tensor) -> torch.Tensor:
    """One N(0,1) draw per (key, counter), fp64 (Box-Muller, cosine branch)."""
    u1 = uniform01(keys, counters, 0)
    u2 = uniform01(keys, counters, 1)
    return torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)


_TORCH_DTYPE = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def torch_dtype(name: str) -> torch.dtype:
    return _TORCH_DTYPE[name]


def to_storage(x64: torch.Tensor, dtype: str) -> torch.Tensor:
    """fp64 -> fp32 -> storage dtype (both steps round to nearest even)."""
    return x64.to(torch.float32).to(_TORCH_DTYPE[dtype])


@dataclass
class Workload:
    """One workload shape.  T is the prompt length (per sequence: see seq_lens)."""
    name: str
    n_layers: int
    n_seqs: int
    n_kv_heads: int
    q_per_kv: int          # G
    head_dim: int          # d
    dtype: str             # "f32" | "f16" | "bf16"
    prompt_len: int        # T_max
    budget: int            # B at prompt_len (slot stride); see budgets()
    decode_steps: int
    window: int            # W query rows used to initialise scores; 0 = full history
    outliers: bool
    ragged: Optional[Tuple[int, int]] = None   # inclusive range of T_b
    budget_ratio: Optional[float] = None       # B_b = ceil(ratio * T_b) when ragged
    n_residual: int = 1
    prox: Optional[int] = None                 # B_p override (default: half of the budget)
    lam: float = 0.98
    alpha: float = 1.0
    seed: int = MASTER_SEED
    k_gain: float = 1.0    # every key (prompt and decode) is multiplied by this: widens the spread of the logits
    layer0: int = 0        # first layer id (for slicing a deep workload)
    seq0: int = 0
    head0: int = 0

    @property
    def n_units(self) -> int:
        return self.n_layers * self.n_seqs * self.n_kv_heads

    def seq_lens(self) -> List[int]:
        if self.ragged is None:
            return [self.prompt_len] * self.n_seqs
        lo, hi = self.ragged
        return [lo + key_of(self.seed, TID_LEN, self.seq0 + b) % (hi - lo + 1)
                for b in range(self.n_seqs)]

    def budgets(self) -> Tuple[List[int], List[int], int]:
        """Per-sequence (B_p, B_c) and the shared B_r.

        Tail ratio B_p/B = 0.5 (hyper-parameter section, practical recommendations);
        the remaining B - B_p - B_r slots are context slots.
        """
        bp, bc = [], []
        for t in self.seq_lens():
            b = self.budget if self.budget_ratio is None else int(math.ceil(self.budget_ratio * t - 1e-9))
            p = b // 2 if self.prox is None else self.prox
            bp.append(p)
            bc.append(b - p - self.n_residual)
        return bp, bc, self.n_residual

    @property
    def slot_capacity(self) -> int:
        bp, bc, br = self.budgets()
        return max(p + c for p, c in zip(bp, bc)) + br

    def sliced(self, **kw) -> "Workload":
        """Same generator streams, smaller extent (e.g. fewer layers / sequences)."""
        d = dict(self.__dict__)
        d.update(kw)
        return Workload(**d)


def workload(i: int) -> Workload:
    """The five benchmark workloads, numbered as in the benchmark definition."""
    if i == 0:
        return Workload("tiny-fp32", 1, 1, 4, 1, 64, "f32", 512, 64, 64, 0, False)
    if i == 1:
        return Workload("llama2-7b-1layer-4k", 1, 1, 32, 1, 128, "f16", 4096, 205, 256, 32, True)
    if i == 2:
        return Workload("llama2-7b-54k-5pct", 32, 1, 32, 1, 128, "f16", 54000, 2700, 512, 32, True)
    if i == 3:
        return Workload("batched-ragged-16k-10pct", 32, 64, 32, 1, 128, "f16", 16384, 1639, 256, 32, True,
                        ragged=(8192, 16384), budget_ratio=0.10)
    if i == 4:
        return Workload("gqa-llama3-8b-32k", 32, 16, 8, 4, 128, "bf16", 32768, 1024, 512, 32, True)
    raise ValueError(f"no workload {i}")


# ----------------------------------------------------------------------------------
# per-(layer, head) structure
# ----------------------------------------------------------------------------------

def head_direction(wl: Workload, layer: int, head: int, device="cpu") -> torch.Tensor:
    """Unit vector u[d] (fp64) shared by the boosted keys and all queries of a KV head."""
    k = torch.tensor(_signed(key_of(wl.seed, TID_DIR, layer, head)), dtype=torch.int64, device=device)
    c = torch.arange(wl.head_dim, dtype=torch.int64, device=device)
    g = normal(k, c)
    return g / torch.linalg.vector_norm(g)


def outlier_channels(wl: Workload, layer: int, head: int) -> List[int]:
    """Four distinct channel indices (host ints)."""
    out: List[int] = []
    n = 0
    while len(out) < 4:
        c = key_of(wl.seed, TID_OUTLIER, layer, head, n) % wl.head_dim
        n += 1
        if c not in out:
            out.append(c)
    return out


_CACHE: dict = {}     # small per-(layer, heads) tensors that every call for the same layer needs again


def _cached(key, make):
    if key not in _CACHE:
        if len(_CACHE) > 4096:
            _CACHE.clear()
        _CACHE[key] = make()
    return _CACHE[key]


def _keys(wl: Workload, tid: int, layer: int, seqs: Sequence[int], heads: Sequence[int], device) -> torch.Tensor:
    def make():
        ks = [[_signed(key_of(wl.seed, tid, layer, b, h)) for h in heads] for b in seqs]
        return torch.tensor(ks, dtype=torch.int64, device=device)
    return _cached(("keys", wl.seed, tid, layer, tuple(seqs), tuple(heads), str(device)), make)


def _boost_strength(wl: Workload, tid: int, layer: int, seqs, heads, pos: torch.Tensor, device) -> torch.Tensor:
    """c[S,H,P]: 4 at sink positions 0..3, 3 at heavy hitters (p = 0.02), else 0.  pos is [S,P]."""
    hk = _keys(wl, tid, layer, seqs, heads, device)[:, :, None]
    u = uniform01(hk, pos[:, None, :], 2)
    c = torch.where(u < 0.02, 3.0, 0.0).to(torch.float64)
    c = torch.where((pos[:, None, :] < 4).expand_as(c), torch.full_like(c, 4.0), c)
    return c


def _dir_and_outliers(wl: Workload, layer: int, heads, device):
    def make():
        u = torch.stack([head_direction(wl, layer, h, device) for h in heads])          # [H,d]
        mult = torch.ones(len(heads), wl.head_dim, dtype=torch.float64, device=device)
        if wl.outliers:
            for i, h in enumerate(heads):
                for c in outlier_channels(wl, layer, h):
                    mult[i, c] = 8.0
        return u, mult
    return _cached(("dir", wl.seed, layer, tuple(heads), wl.head_dim, wl.outliers, str(device)), make)


def _pos2d(pos: torch.Tensor, n_seqs: int, device) -> torch.Tensor:
    """Positions as [S,P]: a 1-D tensor means the same positions for every sequence."""
    pos = pos.to(device=device, dtype=torch.int64)
    return pos[None, :].expand(n_seqs, -1) if pos.dim() == 1 else pos


def kv_rows(wl: Workload, layer: int, pos: torch.Tensor, *, decode: bool = False,
            seqs: Optional[Sequence[int]] = None, heads: Optional[Sequence[int]] = None,
            device="cpu") -> Tuple[torch.Tensor, torch.Tensor]:
    """K, V rows at the given positions: [S, H, P, d] in the storage dtype.

    `pos` is an int64 tensor of absolute token positions, [P] (the same for every
    sequence) or [S,P] (per sequence).  Prompt tokens and decode-step tokens come from
    different streams (decode=True), both indexed by absolute position, so a row does not
    depend on how the call was sliced.
    """
    seqs = list(range(wl.seq0, wl.seq0 + wl.n_seqs)) if seqs is None else list(seqs)
    heads = list(range(wl.head0, wl.head0 + wl.n_kv_heads)) if heads is None else list(heads)
    layer = wl.layer0 + layer
    d = wl.head_dim
    pos = _pos2d(pos, len(seqs), device)
    ctr = pos[:, :, None] * d + torch.arange(d, dtype=torch.int64, device=device)[None, None, :]   # [S,P,d]
    kk = _keys(wl, TID_DK if decode else TID_K, layer, seqs, heads, device)[:, :, None, None]
    vk = _keys(wl, TID_DV if decode else TID_V, layer, seqs, heads, device)[:, :, None, None]
    K = normal(kk, ctr[:, None])
    V = normal(vk, ctr[:, None])
    u, mult = _dir_and_outliers(wl, layer, heads, device)
    c = _boost_strength(wl, TID_DHEAVY if decode else TID_HEAVY, layer, seqs, heads, pos, device)
    if decode:
        # sinks exist only at the start of the prompt
        c = torch.where(c == 4.0, torch.zeros_like(c), c)
    K = K + (c[..., None] * (d ** 0.25)) * u[None, :, None, :]
    K = K * mult[None, :, None, :]
    if wl.k_gain != 1.0:
        K = K * wl.k_gain
    return to_storage(K, wl.dtype), to_storage(V, wl.dtype)


def q_rows(wl: Workload, layer: int, pos: torch.Tensor, *, decode: bool = False,
           seqs: Optional[Sequence[int]] = None, heads: Optional[Sequence[int]] = None,
           device="cpu") -> torch.Tensor:
    """Query rows at the given positions ([P] or per sequence [S,P]): [S, H, G, P, d] in the storage dtype."""
    seqs = list(range(wl.seq0, wl.seq0 + wl.n_seqs)) if seqs is None else list(seqs)
    heads = list(range(wl.head0, wl.head0 + wl.n_kv_heads)) if heads is None else list(heads)
    layer = wl.layer0 + layer
    d, G = wl.head_dim, wl.q_per_kv
    pos = _pos2d(pos, len(seqs), device)
    ctr = pos[:, :, None] * d + torch.arange(d, dtype=torch.int64, device=device)[None, None, :]   # [S,P,d]
    tid = TID_DQ if decode else TID_Q

    def make():
        ks = [[[_signed(key_of(wl.seed, tid, layer, b, h * G + g)) for g in range(G)] for h in heads] for b in seqs]
        return torch.tensor(ks, dtype=torch.int64, device=device)
    qk = _cached(("qkeys", wl.seed, tid, layer, tuple(seqs), tuple(heads), G, str(device)), make)[..., None, None]   # [S,H,G,1,1]
    Q = normal(qk, ctr[:, None, None])
    u, _ = _dir_and_outliers(wl, layer, heads, device)
    Q = Q + (d ** 0.25) * u[None, :, None, None, :]
    return to_storage(Q, wl.dtype)


def prompt(wl: Workload, layer: int, *, seqs=None, heads=None, device="cpu"):
    """Prompt tensors of one layer.

    Returns (Q, K, V, seq_lens): K, V [S, H, T_max, d]; Q [S, H, G, Wq, d] with
    Wq = window (or T_max for full history).  Row r of Q for sequence b is the query
    at position T_b - min(Wq, T_b) + r; rows past min(Wq, T_b) are padding.  K/V rows
    past T_b are padding (generated, never read).
    """
    seqs_l = list(range(wl.seq0, wl.seq0 + wl.n_seqs)) if seqs is None else list(seqs)
    all_lens = dict(zip(range(wl.seq0, wl.seq0 + wl.n_seqs), wl.seq_lens()))
    lens = [all_lens[b] for b in seqs_l]
    T = wl.prompt_len
    K, V = kv_rows(wl, layer, torch.arange(T), seqs=seqs_l, heads=heads, device=device)
    Wq = T if wl.window == 0 else min(wl.window, T)
    first = torch.tensor([tb - min(Wq, tb) for tb in lens])                       # position of each sequence's query row 0
    pos = first[:, None] + torch.arange(Wq)[None, :]                              # [S,Wq]; the tail rows are padding
    Q = q_rows(wl, layer, pos, seqs=seqs_l, heads=heads, device=device)
    return Q, K, V, lens


def decode_inputs(wl: Workload, layer: int, step: int, *, seqs=None, heads=None, device="cpu"):
    """Inputs of decode step `step` (0-based) for one layer.

    Returns q [S, H, G, d], k_new, v_new [S, H, d]; sequence b's token sits at
    absolute position T_b + step.
    """
    seqs_l = list(range(wl.seq0, wl.seq0 + wl.n_seqs)) if seqs is None else list(seqs)
    all_lens = dict(zip(range(wl.seq0, wl.seq0 + wl.n_seqs), wl.seq_lens()))
    pos = torch.tensor([[all_lens[b] + step] for b in seqs_l])            # [S,1]: every sequence at its own position
    k, v = kv_rows(wl, layer, pos, decode=True, seqs=seqs_l, heads=heads, device=device)
    q = q_rows(wl, layer, pos, decode=True, seqs=seqs_l, heads=heads, device=device)
    return q[:, :, :, 0].contiguous(), k[:, :, 0].contiguous(), v[:, :, 0].contiguous()


def decode_inputs_uniform(wl: Workload, layers: Sequence[int], steps: Sequence[int], device="cpu"):
    """Decode inputs for several layers and steps of a workload whose sequences all
    have the same length: q [n_steps, L, S, H, G, d], k_new/v_new [n_steps, L, S, H, d]."""
    assert wl.ragged is None
    pos = torch.tensor([wl.prompt_len + s for s in steps])
    qs, ks, vs = [], [], []
    for l in layers:
        k, v = kv_rows(wl, l, pos, decode=True, device=device)            # [S,H,P,d]
        q = q_rows(wl, l, pos, decode=True, device=device)                # [S,H,G,P,d]
        ks.append(k.permute(2, 0, 1, 3)); vs.append(v.permute(2, 0, 1, 3))
        qs.append(q.permute(3, 0, 1, 2, 4))
    return (torch.stack(qs, 1).contiguous(), torch.stack(ks, 1).contiguous(), torch.stack(vs, 1).contiguous())
