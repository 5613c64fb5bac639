"""Seeded synthetic inputs for the SqueezeAttention hot path.

This module only *makes inputs*: it holds none of the method's arithmetic (no
cosine, no clustering, no softmax, no selection).  Both the HIP path and the
CPU oracle are fed from here, so both see identical bytes.

The paper measures on real prompts (Sec. 5.1, Table 1: CNN/DailyMail, XSUM,
SAMSUM, NarrativeQA, TriviaQA) with trained checkpoints; neither is available,
so these generators stand in for them with the same *shapes* (prompt 256-8k,
generation 16-1024, batch 1-224, budgets 15-30 %, p 0.3-0.4; Sec. 4.2.1,
Tables 2-3) and with the qualitative layer-importance pattern of Fig. 2
(first/last layers change the hidden state most).

Random numbers come from a counter-based integer hash (a splitmix64-style
finaliser keyed by (seed, tensor id, layer) and the flat element index), turned
into an approximately standard normal by summing twelve 10-bit fields of the
hash (Irwin-Hall, variance exactly 1 after scaling).  Only integer operations
and one multiplication by a constant are involved, so the same bytes come out
on the CPU and on the GPU, and any element can be regenerated on its own.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Tuple

import torch

BASE_SEED = 20240404

# tensor ids (one stream of random numbers per id and layer)
TID_H_IN, TID_H_NOISE, TID_K, TID_V, TID_Q_PROMPT = 1, 2, 3, 4, 5
TID_Q_DECODE, TID_K_NEW, TID_V_NEW, TID_U, TID_HH_MASK, TID_A_JITTER = 6, 7, 8, 9, 10, 11

_MASK64 = (1 << 64) - 1


def _s64(x: int) -> int:
    """Python int (mod 2^64) -> the signed value an int64 holds for those bits."""
    x &= _MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


_M1 = _s64(0xBF58476D1CE4E5B9)
_M2 = _s64(0x94D049BB133111EB)
_GOLD = _s64(0x9E3779B97F4A7C15)


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix(x: torch.Tensor) -> torch.Tensor:
    x = (x ^ _lsr(x, 30)) * _M1
    x = (x ^ _lsr(x, 27)) * _M2
    return x ^ _lsr(x, 31)


def _mix_int(x: int) -> int:
    x &= _MASK64
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & _MASK64
    return x ^ (x >> 31)


def _key(seed: int, tid: int, layer: int) -> int:
    k = _mix_int(seed)
    k = _mix_int(k ^ (tid * 0xD6E8FEB86659FD93))
    k = _mix_int(k ^ ((layer + 1) * 0xCA5A826395121157))
    return _s64(k)


_IH_MEAN = 12 * 1023 / 2.0                      # 6138.0
_IH_INV_STD = 1.0 / math.sqrt(1024.0 ** 2 - 1.0)  # var of 12 uniform{0..1023} summed
_CHUNK = 1 << 25


def _hash_pair(key: int, start: int, n: int, device) -> Tuple[torch.Tensor, torch.Tensor]:
    i = torch.arange(start, start + n, dtype=torch.int64, device=device)
    h1 = _mix(i * _GOLD + key)
    h2 = _mix(h1 + _GOLD)
    return h1, h2


def normal(tid: int, layer: int, shape, device="cpu", seed: int = BASE_SEED) -> torch.Tensor:
    """fp32 tensor of approximately N(0,1) values; element with flat index i
    depends only on (seed, tid, layer, i)."""
    n = 1
    for s in shape:
        n *= int(s)
    out = torch.empty(n, dtype=torch.float32, device=device)
    key = _key(seed, tid, layer)
    for start in range(0, n, _CHUNK):
        m = min(_CHUNK, n - start)
        h1, h2 = _hash_pair(key, start, m, device)
        acc = torch.zeros(m, dtype=torch.int64, device=device)
        for h in (h1, h2):
            for j in range(6):
                acc += _lsr(h, 10 * j) & 1023
        out[start:start + m] = ((acc.to(torch.float64) - _IH_MEAN) * _IH_INV_STD).to(torch.float32)
    return out.view(*shape)


def bernoulli(tid: int, layer: int, shape, prob: float, device="cpu", seed: int = BASE_SEED) -> torch.Tensor:
    n = 1
    for s in shape:
        n *= int(s)
    key = _key(seed, tid, layer)
    h1, _ = _hash_pair(key, 0, n, device)
    thr = int(prob * float(1 << 53))
    return (_lsr(h1, 11) < thr).view(*shape)


# --------------------------------------------------------------------------
# workloads
# --------------------------------------------------------------------------

@dataclass(frozen=True)
class Workload:
    name: str
    L: int            # attention layers
    Hq: int           # query heads
    Hkv: int          # key/value heads
    D: int            # head dimension
    hidden: int       # model width (length of a hidden-state row)
    B: int            # batch
    P: int            # prompt tokens
    S: int            # decode steps
    dtype: str        # "f32" | "bf16"  (storage type of q, K, V, hidden states)
    policy: str       # "h2o" | "streaming" | "sliding"
    budget_pct: int   # b_init as a percentage of the prompt length
    p: float          # share of b_init that an unimportant layer keeps
    cos_pattern: str  # which layer-importance pattern the hidden states follow
    n_sink: int = 4
    hh_prob: float = 0.02
    hh_boost: float = 3.0

    @property
    def g(self) -> int:
        return self.Hq // self.Hkv

    @property
    def b_init(self) -> int:
        return self.P * self.budget_pct // 100

    @property
    def total_budget(self) -> int:
        return self.L * self.b_init

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2


WORKLOADS = {
    "tiny": Workload("tiny", 4, 4, 4, 64, 256, 1, 256, 16, "f32", "h2o", 20, 0.35, "tiny"),
    "llama2_7b": Workload("llama2_7b", 32, 32, 32, 128, 4096, 8, 2048, 256, "bf16", "h2o", 20, 0.35, "ends4"),
    "mistral_7b": Workload("mistral_7b", 32, 32, 8, 128, 4096, 32, 4096, 512, "bf16", "streaming", 30, 0.3, "mistral"),
    "llama2_70b": Workload("llama2_70b", 80, 64, 8, 128, 8192, 16, 8192, 256, "bf16", "sliding", 15, 0.4, "ends70b"),
    "stress_7b": Workload("stress_7b", 32, 32, 32, 128, 4096, 224, 512, 1024, "bf16", "h2o", 20, 0.35, "ends4"),
}


def scaled(wl: Workload, **kw) -> Workload:
    """A copy of a workload with some sizes replaced (used for reduced parity cases)."""
    d = {f: getattr(wl, f) for f in wl.__dataclass_fields__}
    d.update(kw)
    return Workload(**d)


def cos_targets(wl: Workload) -> List[float]:
    """Target mean cosine per layer (the pattern of Fig. 2: first and last
    layers low, the rest high).  Returns L floats."""
    L = wl.L
    z = normal(TID_A_JITTER, 0, (L,), "cpu").clamp(-2.0, 2.0).tolist()
    uni = [(x + 2.0) / 4.0 for x in z]          # in [0,1], only used for spread
    if wl.cos_pattern == "tiny":
        a = [2.0, 0.3, 0.3, 1.5]
        return [1.0 / math.sqrt(1.0 + x * x) for x in (a * ((L + 3) // 4))[:L]]
    if wl.cos_pattern == "ends4":
        c = [0.90 + 0.015 * z[l] for l in range(L)]
        low = {0: 0.35, 1: 0.45, L - 2: 0.55, L - 1: 0.50}
        for l, v in low.items():
            c[l] = v
        return c
    if wl.cos_pattern == "mistral":
        c = []
        for l in range(L):
            if l in (0, 1, L - 1):
                c.append({0: 0.40, 1: 0.45, L - 1: 0.50}[l])
            elif l < L // 2:
                c.append(0.75 + 0.01 * z[l])
            else:
                c.append(0.93 + 0.005 * z[l])
        return c
    if wl.cos_pattern == "ends70b":
        low = set(range(0, L // 8)) | set(range(L - L // 10, L)) | {L * 37 // 80, L * 53 // 80}
        return [0.35 + 0.25 * uni[l] if l in low else 0.90 + 0.0075 * z[l] for l in range(L)]
    raise ValueError(wl.cos_pattern)


def noise_scales(wl: Workload) -> List[float]:
    """a_l with h_out = h_in + a_l * noise, so that E[cos] ~ 1/sqrt(1+a_l^2)."""
    return [math.sqrt(1.0 / (c * c) - 1.0) for c in cos_targets(wl)]


def hidden_states(wl: Workload, layer: int, device="cpu", n_tokens: int | None = None):
    """(h_in, h_out) of one layer: [T, hidden] each, storage dtype."""
    T = wl.B * wl.P if n_tokens is None else n_tokens
    a = noise_scales(wl)[layer]
    h_in = normal(TID_H_IN, layer, (T, wl.hidden), device)
    noise = normal(TID_H_NOISE, layer, (T, wl.hidden), device)
    noise *= a                     # separate multiply and add: each rounded once
    h_out = h_in + noise
    dt = wl.torch_dtype
    return h_in.to(dt), h_out.to(dt)


def unit_dirs(wl: Workload) -> torch.Tensor:
    """Heavy-hitter direction u per (layer, kv head): [L, Hkv, D] fp32, unit
    norm.  Always made on the CPU (fp64 normalisation) and then shipped."""
    u = normal(TID_U, 0, (wl.L, wl.Hkv, wl.D), "cpu").to(torch.float64)
    u = u / u.norm(dim=-1, keepdim=True)
    return u.to(torch.float32)


def hh_mask(wl: Workload, device="cpu") -> torch.Tensor:
    """[B, P+S] bool: which positions are heavy hitters (shared by all layers
    and heads of a sequence)."""
    return bernoulli(TID_HH_MASK, 0, (wl.B, wl.P + wl.S), wl.hh_prob, device)


def prompt_kv(wl: Workload, layer: int, device="cpu", u=None, mask=None):
    """Prompt keys and values of one layer: [B, Hkv, P, D] each, storage dtype."""
    u = unit_dirs(wl) if u is None else u
    mask = hh_mask(wl, device) if mask is None else mask
    shape = (wl.B, wl.Hkv, wl.P, wl.D)
    K = normal(TID_K, layer, shape, device)
    V = normal(TID_V, layer, shape, device)
    boost = (wl.hh_boost * u[layer]).to(device)                       # [Hkv, D]
    m = mask[:, :wl.P].to(torch.float32)                              # [B, P]
    K = K + m[:, None, :, None] * boost[None, :, None, :]
    dt = wl.torch_dtype
    return K.to(dt), V.to(dt)


def prompt_q(wl: Workload, layer: int, device="cpu", u=None):
    """Prompt queries of one layer: [B, Hq, P, D] storage dtype."""
    u = unit_dirs(wl) if u is None else u
    Q = normal(TID_Q_PROMPT, layer, (wl.B, wl.Hq, wl.P, wl.D), device)
    boost = (wl.hh_boost * u[layer]).to(device).repeat_interleave(wl.g, dim=0)  # [Hq, D]
    Q = Q + boost[None, :, None, :]
    return Q.to(wl.torch_dtype)


def decode_qkv(wl: Workload, layer: int, device="cpu", u=None, mask=None, steps: int | None = None):
    """Decode-time inputs of one layer for all steps:
    q [S, B, Hq, D], k_new [S, B, Hkv, D], v_new [S, B, Hkv, D], storage dtype.
    Step t (0-based) appends the token at position P + t."""
    S = wl.S if steps is None else steps
    u = unit_dirs(wl) if u is None else u
    mask = hh_mask(wl, device) if mask is None else mask
    q = normal(TID_Q_DECODE, layer, (S, wl.B, wl.Hq, wl.D), device)
    k = normal(TID_K_NEW, layer, (S, wl.B, wl.Hkv, wl.D), device)
    v = normal(TID_V_NEW, layer, (S, wl.B, wl.Hkv, wl.D), device)
    boost = (wl.hh_boost * u[layer]).to(device)                       # [Hkv, D]
    q = q + boost.repeat_interleave(wl.g, dim=0)[None, None]
    m = mask[:, wl.P:wl.P + S].to(torch.float32).transpose(0, 1)      # [S, B]
    k = k + m[:, :, None, None] * boost[None, None]
    dt = wl.torch_dtype
    return q.to(dt), k.to(dt), v.to(dt)


# -- byte accounting (what the method must move; Sec. 2.1 KV size model) ---------------------------

def kv_bytes_per_token(wl: Workload) -> int:
    """Sec. 2.1: every token adds one K and one V vector per layer and KV head --
    2 * n_layer * n_kv_head * d_head elements (0.5 MB for Llama-2-7B in 16 bits: 2 * 32 * 4096 * 2 B)."""
    return 2 * wl.L * wl.Hkv * wl.D * wl.elem_bytes


def full_cache_bytes_per_sequence(wl: Workload) -> int:
    """An uncompressed cache sized for the whole generation: P + S tokens per sequence."""
    return (wl.P + wl.S) * kv_bytes_per_token(wl)


def resident_cache_bytes(wl: Workload, slots_per_layer) -> int:
    """Bytes the compact caches of this library hold resident: slots_per_layer[l] slots in layer l (over all
    sequences and KV heads), each a K row and a V row plus the token's position (4 bytes) and, under H2O,
    its accumulated score (4 bytes)."""
    per_slot = 2 * wl.D * wl.elem_bytes + (8 if wl.policy == "h2o" else 4)
    return sum(int(n) * per_slot for n in slots_per_layer)


def squeezed_cache_bytes(wl: Workload, budgets) -> int:
    """resident_cache_bytes of a batch whose layer l keeps min(budget_l, P + S) slots per sequence and KV head."""
    return resident_cache_bytes(wl, [wl.B * wl.Hkv * min(b, wl.P + wl.S) for b in budgets])


def equal_memory_batch(wl: Workload, squeezed_bytes: int) -> int:
    """Sec. 5.4 (Table 3) read at attention level: the largest batch whose UNCOMPRESSED cache, sized for
    the whole generation of `wl` (P + S tokens per sequence, Sec. 2.1 size model), fits in the bytes the
    squeezed run's caches occupy."""
    return int(squeezed_bytes // full_cache_bytes_per_sequence(wl))


def decode_bytes_per_step(wl: Workload, budgets) -> list:
    """Algorithmic HBM bytes of each of the S decode steps over all layers: every kept K and V row read
    once (n_l = min(P + t + 1, b_l) tokens per unit after the append / eviction), 8 bytes of accumulated
    score per kept token under H2O (one read, one write), the appended K and V rows written, q read and
    out written."""
    e, row = wl.elem_bytes, wl.D * wl.elem_bytes
    units = wl.B * wl.Hkv
    out = []
    for t in range(wl.S):
        tot = 0
        for b in budgets:
            n = min(wl.P + t + 1, b)
            tot += units * (n * 2 * row + (8 * n if wl.policy == "h2o" else 0) + 2 * row)
        tot += wl.L * wl.B * wl.Hq * wl.D * e * 2
        out.append(tot)
    return out


def decode_bytes_per_step_ragged(wl: Workload, budget_seq, prompt_len) -> list:
    """The same count for a ragged batch: budget_seq[l][b] is layer l's budget for sequence b,
    prompt_len[b] its prompt length (its step-t token has position prompt_len[b] + t)."""
    e, row = wl.elem_bytes, wl.D * wl.elem_bytes
    out = []
    for t in range(wl.S):
        tot = 0
        for per_seq in budget_seq:
            for b, budget in enumerate(per_seq):
                n = min(prompt_len[b] + t + 1, budget)
                tot += wl.Hkv * (n * 2 * row + (8 * n if wl.policy == "h2o" else 0) + 2 * row)
        tot += wl.L * wl.B * wl.Hq * wl.D * e * 2
        out.append(tot)
    return out
