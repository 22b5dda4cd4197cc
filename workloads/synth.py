"""Seeded synthetic inputs for the chunk-eviction hot path.

This module only makes inputs: shapes, a counter-based random generator and
the value recipe of each workload.  It contains none of the method's
arithmetic (no attention, scoring, selection or gathering) and is the one
module that both the tests of the CPU oracle and the callers of the HIP
library may import.

Recipe (stands in for post-RoPE Q/K/V of Mistral-7B / Llama-2 shaped layers on
long documents, which are not available offline):

* every element of Q, K, V and of the instruction queries Q_I is
  z * head_dim**-0.5 with z ~ N(0, 1) i.i.d., rounded to the workload dtype;
* keys at document positions 0..3 are multiplied by ``sink_scale`` (4);
* each other document position is, with probability ``heavy_prob``, a heavy
  hitter whose key is multiplied by ``heavy_scale`` (2.5); the draw is per
  (document, position) and shared by all layers and heads;
* ``peaked`` variants leave Q, K and Q_I unscaled so that logits have unit
  spread and the importance scores are far from uniform (parity only).

Every element is a pure function of (seed, tensor id, b, l, head, position,
dim): a 64-bit counter goes through a splitmix64-style mixer, its two 32-bit
halves become two uniforms and Box-Muller turns them into one normal.  The
same torch integer/float64 ops run on the CPU and on the GPU, so any slice
can be regenerated anywhere.
"""

from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Dict, Optional

import torch

CACHE_INSTR, CACHE_SHARED, CACHE_DUAL = 0, 1, 2
SELECT_PER_KV_HEAD, SELECT_PER_LAYER = 0, 1

_TID_Q, _TID_K, _TID_V, _TID_QI, _TID_HEAVY = 1, 2, 3, 4, 5

_MASK64 = (1 << 64) - 1


def _s64(c: int) -> int:
    """Python int -> the signed 64-bit value with the same bit pattern."""
    c &= _MASK64
    return c - (1 << 64) if c >= (1 << 63) else c


_GOLDEN = _s64(0x9E3779B97F4A7C15)
_M1 = _s64(0xBF58476D1CE4E5B9)
_M2 = _s64(0x94D049BB133111EB)


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str                 # "f32" | "bf16"
    batch: int
    layers: int
    q_heads: int
    kv_heads: int
    head_dim: int
    doc_len: int               # T
    chunk_len: int             # l_s
    budget: int                # k
    instr_len: int             # n_i
    cache_mode: int = CACHE_INSTR
    select_mode: int = SELECT_PER_KV_HEAD
    budget_lm: int = 0
    start_size: int = 0        # leading document states that are never evicted (0 = plain selection)
    lm_ordering: int = 0       # DUAL only: 0 = score after append, 1 = evict, then append (Section 4.1's order)
    score_mode: int = 0        # 0 = this step's score decides, 1 = accumulated scores (H2O's rule)
    position_shift: int = 0    # 1 = tensors are taken as un-rotated, positions are cache slots (Section 5.3)
    rope_base: float = 0.0     # 0 -> 10000
    sink_scale: float = 4.0
    heavy_prob: float = 0.0
    heavy_scale: float = 2.5
    peaked: bool = False
    seed: int = 1234

    @property
    def n_chunks(self) -> int:
        return (self.doc_len + self.chunk_len - 1) // self.chunk_len

    @property
    def group(self) -> int:
        return self.q_heads // self.kv_heads

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    def chunk_bounds(self, i: int):
        lo = i * self.chunk_len
        return lo, min(self.doc_len, lo + self.chunk_len)

    def cache_len_before(self, i: int, budget: Optional[int] = None) -> int:
        """Cache length when chunk i arrives: min(k, tokens so far)."""
        b = self.budget if budget is None else budget
        return min(b, i * self.chunk_len)


WORKLOADS: Dict[str, Workload] = {
    # tiny fp32 run the oracle finishes in seconds
    "cfg1_tiny_f32": Workload("cfg1_tiny_f32", "f32", 1, 1, 4, 1, 64, 512, 32, 64, 8, seed=1235),
    # Mistral-7B shape, the configuration the headline metric is quoted on
    "cfg2_mistral7b": Workload("cfg2_mistral7b", "bf16", 1, 32, 32, 8, 128, 16384, 512, 768, 64,
                               heavy_prob=0.02, seed=1236),
    # Llama-2-7B shape (MHA), shared cache, batch 4
    "cfg3_llama2_7b_shared": Workload("cfg3_llama2_7b_shared", "bf16", 4, 32, 32, 32, 128, 32768, 1024, 1024, 128,
                                      cache_mode=CACHE_SHARED, seed=1237),
    # dual cache, Mistral-7B shape, batch 8
    "cfg4_dual": Workload("cfg4_dual", "bf16", 8, 32, 32, 8, 128, 65536, 512, 768, 64,
                          cache_mode=CACHE_DUAL, budget_lm=768, heavy_prob=0.02, seed=1238),
    # large-layer run, one GPU's share
    "cfg5_large": Workload("cfg5_large", "bf16", 4, 80, 64, 8, 128, 131072, 2048, 4096, 256,
                           heavy_prob=0.01, seed=1239),
}


def peaked(w: Workload) -> Workload:
    return replace(w, name=w.name + "_peaked", peaked=True)


def scaled_down(w: Workload, **kw) -> Workload:
    """A smaller instance of the same recipe (fewer layers, shorter document…)."""
    return replace(w, name=w.name + "_small", **kw)


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix64(x: torch.Tensor) -> torch.Tensor:
    z = x + _GOLDEN
    z = (z ^ _lsr(z, 30)) * _M1
    z = (z ^ _lsr(z, 27)) * _M2
    return z ^ _lsr(z, 31)


def _stream_key(seed: int, tensor_id: int) -> int:
    # scalar mixing done in Python integers
    z = (seed * 0x9E3779B97F4A7C15 + tensor_id * 0xD1B54A32D192ED03 + 0x2545F4914F6CDD1D) & _MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return _s64(z ^ (z >> 31))


def _uniform_pair(counter: torch.Tensor, key: int):
    h = _mix64(_mix64(counter ^ key))
    hi = _lsr(h, 32).to(torch.float64)
    lo = (h & 0xFFFFFFFF).to(torch.float64)
    return (hi + 0.5) / 4294967296.0, (lo + 0.5) / 4294967296.0


def _normal(counter: torch.Tensor, key: int) -> torch.Tensor:
    u1, u2 = _uniform_pair(counter, key)
    return torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)


def _counter(w: Workload, heads: int, span: int, b, l, h, pos, device) -> torch.Tensor:
    """Linear element index of [B, L, heads, span, d] for the index vectors given."""
    d = w.head_dim
    bb = torch.as_tensor(b, dtype=torch.int64, device=device).view(-1, 1, 1, 1, 1)
    ll = torch.as_tensor(l, dtype=torch.int64, device=device).view(1, -1, 1, 1, 1)
    hh = torch.as_tensor(h, dtype=torch.int64, device=device).view(1, 1, -1, 1, 1)
    pp = torch.as_tensor(pos, dtype=torch.int64, device=device).view(1, 1, 1, -1, 1)
    dd = torch.arange(d, dtype=torch.int64, device=device).view(1, 1, 1, 1, -1)
    return (((bb * w.layers + ll) * heads + hh) * span + pp) * d + dd


def heavy_mask(w: Workload, b, pos, device) -> torch.Tensor:
    """[len(b), len(pos)] bool: which document positions carry a heavy-hitter key."""
    bb = torch.as_tensor(b, dtype=torch.int64, device=device).view(-1, 1)
    pp = torch.as_tensor(pos, dtype=torch.int64, device=device).view(1, -1)
    if w.heavy_prob <= 0.0:
        return torch.zeros((bb.shape[0], pp.shape[1]), dtype=torch.bool, device=device)
    u, _ = _uniform_pair(bb * w.doc_len + pp, _stream_key(w.seed, _TID_HEAVY))
    return (u < w.heavy_prob) & (pp >= 4)


def key_multiplier(w: Workload, b, pos, device) -> torch.Tensor:
    """[len(b), len(pos)] float64 factor applied to the keys of each position."""
    pp = torch.as_tensor(pos, dtype=torch.int64, device=device).view(1, -1)
    m = torch.ones((len(b), pp.shape[1]), dtype=torch.float64, device=device)
    m = torch.where(heavy_mask(w, b, pos, device), torch.full_like(m, w.heavy_scale), m)
    return torch.where(pp < 4, torch.full_like(m, w.sink_scale), m)


def gen_tensor(w: Workload, which: str, positions, device="cpu", b=None, l=None, h=None,
               chunk_index: int = 0) -> torch.Tensor:
    """Values of one input tensor on a sub-grid.

    ``which`` is "q", "k", "v" (document tensors; ``positions`` are document
    positions) or "q_instr" (``positions`` are instruction rows 0..n_i-1 and
    ``chunk_index`` selects the per-chunk re-encoding).  ``b``, ``l``, ``h``
    default to all documents, layers and heads.  Returns [len(b), len(l),
    len(h), len(positions), d] in the workload dtype.
    """
    heads = w.kv_heads if which in ("k", "v") else w.q_heads
    b = list(range(w.batch)) if b is None else list(b)
    l = list(range(w.layers)) if l is None else list(l)
    h = list(range(heads)) if h is None else list(h)
    positions = torch.as_tensor(positions, dtype=torch.int64, device=device)
    if which == "q_instr":
        span = w.instr_len * w.n_chunks
        ctr = _counter(w, heads, span, b, l, h, chunk_index * w.instr_len + positions, device)
        tid = _TID_QI
    else:
        ctr = _counter(w, heads, w.doc_len, b, l, h, positions, device)
        tid = {"q": _TID_Q, "k": _TID_K, "v": _TID_V}[which]
    z = _normal(ctr, _stream_key(w.seed, tid))
    unscaled = w.peaked and which in ("q", "k", "q_instr")
    if not unscaled:
        z = z * (float(w.head_dim) ** -0.5)
    if which == "k":
        z = z * key_multiplier(w, b, positions, device).view(len(b), 1, 1, -1, 1)
    return z.to(w.torch_dtype)


def make_chunk(w: Workload, i: int, device="cpu", b=None, l=None) -> Dict[str, torch.Tensor]:
    """Inputs of chunk step i: q [B,L,Hq,c_i,d], k/v [B,L,Hkv,c_i,d], q_instr [B,L,Hq,n_i,d]."""
    lo, hi = w.chunk_bounds(i)
    pos = torch.arange(lo, hi, dtype=torch.int64, device=device)
    rows = torch.arange(w.instr_len, dtype=torch.int64, device=device)
    return {
        "q": gen_tensor(w, "q", pos, device, b, l),
        "k": gen_tensor(w, "k", pos, device, b, l),
        "v": gen_tensor(w, "v", pos, device, b, l),
        "q_instr": gen_tensor(w, "q_instr", rows, device, b, l, chunk_index=i),
    }


def make_chunk_sliced(w: Workload, i: int, device="cpu", b=None, l=None, max_elems: int = 1 << 27,
                      out: Optional[Dict[str, torch.Tensor]] = None) -> Dict[str, torch.Tensor]:
    """make_chunk for shapes whose 64-bit temporaries would not fit at once: the same values, generated one
    (document, group of layers) slice at a time (at most about max_elems elements of q per slice) and written
    into ``out`` (allocated here if not given)."""
    b = list(range(w.batch)) if b is None else list(b)
    l = list(range(w.layers)) if l is None else list(l)
    lo, hi = w.chunk_bounds(i)
    c, d, dt = hi - lo, w.head_dim, w.torch_dtype
    if out is None:
        out = {"q": torch.empty((len(b), len(l), w.q_heads, c, d), dtype=dt, device=device),
               "k": torch.empty((len(b), len(l), w.kv_heads, c, d), dtype=dt, device=device),
               "v": torch.empty((len(b), len(l), w.kv_heads, c, d), dtype=dt, device=device),
               "q_instr": torch.empty((len(b), len(l), w.q_heads, w.instr_len, d), dtype=dt, device=device)}
    per_layer = w.q_heads * max(c, w.instr_len) * d
    lg = max(1, min(len(l), max_elems // per_layer))
    for bi, bb in enumerate(b):
        for l0 in range(0, len(l), lg):
            part = make_chunk(w, i, device, b=[bb], l=l[l0:l0 + lg])
            for name in ("q", "k", "v", "q_instr"):
                out[name][bi:bi + 1, l0:l0 + lg, :, :part[name].shape[3]] = part[name]
            del part
    return out


def make_document(w: Workload, device="cpu", b=None, l=None) -> Dict[str, torch.Tensor]:
    """Whole-document tensors, generated chunk by chunk to bound temporaries:
    q [B,L,Hq,T,d], k/v [B,L,Hkv,T,d], q_instr [n_chunks,B,L,Hq,n_i,d]."""
    nb = w.batch if b is None else len(list(b))
    nl = w.layers if l is None else len(list(l))
    dt, d = w.torch_dtype, w.head_dim
    q = torch.empty((nb, nl, w.q_heads, w.doc_len, d), dtype=dt, device=device)
    k = torch.empty((nb, nl, w.kv_heads, w.doc_len, d), dtype=dt, device=device)
    v = torch.empty_like(k)
    qi = torch.empty((w.n_chunks, nb, nl, w.q_heads, w.instr_len, d), dtype=dt, device=device)
    for i in range(w.n_chunks):
        lo, hi = w.chunk_bounds(i)
        ch = make_chunk(w, i, device, b, l)
        q[:, :, :, lo:hi] = ch["q"]
        k[:, :, :, lo:hi] = ch["k"]
        v[:, :, :, lo:hi] = ch["v"]
        qi[i] = ch["q_instr"]
    return {"q": q, "k": k, "v": v, "q_instr": qi}
