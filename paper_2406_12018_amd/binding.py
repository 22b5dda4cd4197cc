"""ctypes binding of libcitrus.so (the C ABI in include/citrus.h).

Argument marshalling only: every step of the hot path runs in the HIP kernels
behind the C entry points of the same names.  torch is used for device memory
and for the current HIP stream, nothing else.  There is no CPU fallback: if the
library is missing or an entry point fails, an exception is raised.
"""

from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Callable, Optional, Sequence

import torch

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libcitrus.so")

F32, BF16 = 0, 1
CACHE_INSTR, CACHE_SHARED, CACHE_DUAL, CACHE_STANDARD = 0, 1, 2, 3
SELECT_PER_KV_HEAD, SELECT_PER_LAYER = 0, 1
LM_SCORE_AFTER_APPEND, LM_EVICT_THEN_APPEND = 0, 1
SCORE_PER_STEP, SCORE_ACCUMULATED = 0, 1

EVENTS_PER_STEP = 8

OK, ERR_NULL, ERR_SHAPE, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_DEVICE, ERR_PROVIDER = range(7)

EXPORTS = (
    "citrus_abi_version", "citrus_status_string", "citrus_workspace_bytes", "citrus_chunk_attn",
    "citrus_instr_score", "citrus_cache_score", "citrus_evict_cache", "citrus_evict_cache_static",
    "citrus_static_scratch_bytes", "citrus_decode_step", "citrus_rope", "citrus_score_accumulate", "citrus_score_gather", "citrus_topk_select", "citrus_kv_compact", "citrus_resident_provider",
    "citrus_process_document", "citrus_probe_mfma",
)


class CitrusError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib().citrus_status_string(status).decode() if _LIB is not None else "?"
        super().__init__(f"{where}: status {status} ({msg})")


class CConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "batch", "layers", "q_heads", "kv_heads", "head_dim", "chunk_len", "budget", "budget_lm", "instr_len",
        "cache_capacity", "dtype", "cache_mode", "select_mode", "start_size", "lm_ordering", "score_mode", "position_shift")] + [
            ("rope_base", C.c_float), ("softmax_scale", C.c_float)]


class CSideStream(C.Structure):
    _fields_ = [("stream", C.c_void_p), ("fork_event", C.c_void_p), ("join_event", C.c_void_p)]


class CTensor(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("stride_b", C.c_int64), ("stride_l", C.c_int64), ("stride_h", C.c_int64),
                ("stride_s", C.c_int64)]


class CChunkIO(C.Structure):
    _fields_ = [("q", CTensor), ("k", CTensor), ("v", CTensor), ("q_instr", CTensor), ("out", CTensor),
                ("chunk_len", C.c_int32)]


class CResidentDoc(C.Structure):
    _fields_ = [("q", CTensor), ("k", CTensor), ("v", CTensor), ("out", CTensor), ("q_instr", CTensor),
                ("q_instr_stride_chunk", C.c_int64), ("doc_len", C.c_int32), ("chunk_len", C.c_int32),
                ("dtype", C.c_int32)]


PROVIDER = C.CFUNCTYPE(C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.POINTER(CChunkIO))

_LIB = None


def _lib():
    """Load libcitrus.so (built in-tree by paper_2406_12018_amd.build)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -m paper_2406_12018_amd.build); "
                           "there is no fallback path")
    lib = C.CDLL(LIB_PATH)
    P, I, V, S = C.POINTER, C.c_int32, C.c_void_p, C.c_size_t
    lib.citrus_abi_version.restype = I
    lib.citrus_status_string.restype = C.c_char_p
    lib.citrus_status_string.argtypes = [I]
    lib.citrus_workspace_bytes.restype = S
    lib.citrus_workspace_bytes.argtypes = [P(CConfig)]
    lib.citrus_chunk_attn.restype = I
    lib.citrus_chunk_attn.argtypes = [P(CConfig), CTensor, CTensor, CTensor, I, CTensor, CTensor, I, CTensor, V, V, V, V, S, V]
    lib.citrus_instr_score.restype = I
    lib.citrus_instr_score.argtypes = [P(CConfig), CTensor, CTensor, I, CTensor, I, V, V, S, V]
    lib.citrus_cache_score.restype = I
    lib.citrus_cache_score.argtypes = [P(CConfig), CTensor, I, CTensor, I, V, V, V, S, V]
    lib.citrus_evict_cache.restype = I
    lib.citrus_evict_cache.argtypes = [P(CConfig), CTensor, I, CTensor, CTensor, I, I, CTensor, CTensor, V, V, S, V]
    lib.citrus_evict_cache_static.restype = I
    lib.citrus_evict_cache_static.argtypes = [P(CConfig), CTensor, I, CTensor, CTensor, I, I, CTensor, CTensor, V, V]
    lib.citrus_static_scratch_bytes.restype = S
    lib.citrus_static_scratch_bytes.argtypes = []
    lib.citrus_decode_step.restype = I
    lib.citrus_decode_step.argtypes = [P(CConfig), CTensor, CTensor, CTensor, CTensor, CTensor, I, CTensor, V, S, V]
    lib.citrus_rope.restype = I
    lib.citrus_rope.argtypes = [P(CConfig), CTensor, I, I, I, CTensor, V]
    lib.citrus_score_accumulate.restype = I
    lib.citrus_score_accumulate.argtypes = [P(CConfig), V, I, V, I, V]
    lib.citrus_score_gather.restype = I
    lib.citrus_score_gather.argtypes = [P(CConfig), V, I, V, I, I, V, V]
    lib.citrus_topk_select.restype = I
    lib.citrus_topk_select.argtypes = [P(CConfig), V, I, I, V, V, S, V]
    lib.citrus_kv_compact.restype = I
    lib.citrus_kv_compact.argtypes = [P(CConfig), CTensor, CTensor, I, CTensor, CTensor, I, V, I, I, CTensor, CTensor, V]
    lib.citrus_resident_provider.restype = I
    lib.citrus_resident_provider.argtypes = [V, I, V, P(CChunkIO)]
    lib.citrus_process_document.restype = I
    lib.citrus_process_document.argtypes = [P(CConfig), V, V, I, I, P(CTensor), P(CTensor), P(CTensor), P(CTensor),
                                            P(I), P(I), P(I), P(I), P(V), V, V, P(I), V, V, S, V, P(CSideStream)]
    lib.citrus_probe_mfma.restype = I
    lib.citrus_probe_mfma.argtypes = [I, V, S, P(C.c_int64), V]
    _LIB = lib
    return lib


@dataclass
class Config:
    batch: int
    layers: int
    q_heads: int
    kv_heads: int
    head_dim: int
    chunk_len: int
    budget: int
    instr_len: int
    dtype: int = BF16
    cache_mode: int = CACHE_INSTR
    select_mode: int = SELECT_PER_KV_HEAD
    budget_lm: int = 0
    cache_capacity: int = 0          # 0 -> the smallest capacity the configuration needs
    softmax_scale: float = 0.0
    start_size: int = 0              # leading document states that are never evicted
    lm_ordering: int = LM_SCORE_AFTER_APPEND
    score_mode: int = SCORE_PER_STEP
    position_shift: int = 0          # 1: inputs come without rotary embedding, positions are cache slots
    rope_base: float = 0.0           # 0 -> 10000

    def __post_init__(self):
        if self.cache_capacity == 0:
            # a cache run in the printed order keeps the whole previous chunk until the next eviction
            held = self.chunk_len if self.lm_ordering == LM_EVICT_THEN_APPEND else 0
            if self.cache_mode == CACHE_DUAL:
                self.cache_capacity = max(self.budget, self.budget_lm + held)
            elif self.cache_mode == CACHE_STANDARD:
                self.cache_capacity = self.budget + held
            else:
                self.cache_capacity = max(self.budget, self.budget_lm)

    def c(self) -> CConfig:
        return CConfig(self.batch, self.layers, self.q_heads, self.kv_heads, self.head_dim, self.chunk_len,
                       self.budget, self.budget_lm, self.instr_len, self.cache_capacity, self.dtype,
                       self.cache_mode, self.select_mode, self.start_size, self.lm_ordering, self.score_mode, self.position_shift, self.rope_base,
                       self.softmax_scale)

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == F32 else torch.bfloat16

    @property
    def sel_heads(self) -> int:
        return 1 if self.select_mode == SELECT_PER_LAYER else self.kv_heads

    @staticmethod
    def from_workload(w, **overrides) -> "Config":
        kw = dict(batch=w.batch, layers=w.layers, q_heads=w.q_heads, kv_heads=w.kv_heads, head_dim=w.head_dim,
                  chunk_len=w.chunk_len, budget=w.budget, instr_len=w.instr_len,
                  dtype=F32 if w.dtype == "f32" else BF16, cache_mode=w.cache_mode, select_mode=w.select_mode,
                  budget_lm=w.budget_lm, start_size=getattr(w, "start_size", 0),
                  lm_ordering=getattr(w, "lm_ordering", 0), score_mode=getattr(w, "score_mode", 0),
                  position_shift=getattr(w, "position_shift", 0), rope_base=getattr(w, "rope_base", 0.0))
        kw.update(overrides)
        return Config(**kw)


def tensor(t: Optional[torch.Tensor]) -> CTensor:
    """[B, L, H, S, d] torch tensor (d contiguous) -> citrus_tensor."""
    if t is None:
        return CTensor(None, 0, 0, 0, 0)
    if t.dim() != 5 or t.stride(4) != 1:
        raise ValueError("expected a [B, L, H, S, d] tensor with contiguous last axis")
    return CTensor(t.data_ptr(), t.stride(0), t.stride(1), t.stride(2), t.stride(3))


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _check(status: int, where: str):
    if status != OK:
        raise CitrusError(status, where)


def abi_version() -> int:
    return _lib().citrus_abi_version()


def status_string(status: int) -> str:
    return _lib().citrus_status_string(status).decode()


def workspace_bytes(cfg: Config) -> int:
    cc = cfg.c()
    return int(_lib().citrus_workspace_bytes(C.byref(cc)))


def alloc_workspace(cfg: Config, device="cuda") -> torch.Tensor:
    n = workspace_bytes(cfg)
    if n == 0:
        raise CitrusError(ERR_SHAPE, "citrus_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def citrus_chunk_attn(cfg: Config, q, k_cache, v_cache, cache_len: int, k_chunk, v_chunk, out=None, lse=None,
                      lm_score=None, workspace=None, stream=None, chunk_len: Optional[int] = None, lse_cache=None):
    chunk_len = q.shape[3] if chunk_len is None else chunk_len
    if out is None:
        out = torch.empty_like(q)
    cc = cfg.c()
    st = _lib().citrus_chunk_attn(C.byref(cc), tensor(q), tensor(k_cache), tensor(v_cache), cache_len,
                                  tensor(k_chunk), tensor(v_chunk), chunk_len, tensor(out), _ptr(lse), _ptr(lse_cache),
                                  _ptr(lm_score), _ptr(workspace), 0 if workspace is None else workspace.numel(),
                                  _stream(stream))
    _check(st, "citrus_chunk_attn")
    return out


def citrus_instr_score(cfg: Config, q_instr, k_cache, cache_len: int, k_chunk, score=None, workspace=None,
                       stream=None, chunk_len: Optional[int] = None):
    chunk_len = k_chunk.shape[3] if chunk_len is None else chunk_len
    if score is None:
        score = torch.empty((cfg.batch, cfg.layers, cfg.kv_heads, cache_len + chunk_len), dtype=torch.float32,
                            device=q_instr.device)
    cc = cfg.c()
    st = _lib().citrus_instr_score(C.byref(cc), tensor(q_instr), tensor(k_cache), cache_len, tensor(k_chunk),
                                   chunk_len, _ptr(score), _ptr(workspace),
                                   0 if workspace is None else workspace.numel(), _stream(stream))
    _check(st, "citrus_instr_score")
    return score


def citrus_cache_score(cfg: Config, q, k_cache, cache_len: int, score=None, workspace=None, stream=None,
                       rows: Optional[int] = None, lse_cache=None):
    rows = q.shape[3] if rows is None else rows
    if score is None:
        score = torch.empty((cfg.batch, cfg.layers, cfg.kv_heads, cache_len), dtype=torch.float32, device=q.device)
    cc = cfg.c()
    st = _lib().citrus_cache_score(C.byref(cc), tensor(q), rows, tensor(k_cache), cache_len, _ptr(lse_cache),
                                   _ptr(score), _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream(stream))
    _check(st, "citrus_cache_score")
    return score


def citrus_evict_cache(cfg: Config, q, k_cache, v_cache, cache_len: int, k: int, k_new, v_new, idx=None,
                       workspace=None, stream=None, rows: Optional[int] = None) -> int:
    """Returns the number of states kept, min(k, cache_len)."""
    rows = q.shape[3] if rows is None else rows
    cc = cfg.c()
    st = _lib().citrus_evict_cache(C.byref(cc), tensor(q), rows, tensor(k_cache), tensor(v_cache), cache_len, k,
                                   tensor(k_new), tensor(v_new), _ptr(idx), _ptr(workspace),
                                   0 if workspace is None else workspace.numel(), _stream(stream))
    _check(st, "citrus_evict_cache")
    return min(k, cache_len)


def static_scratch_bytes() -> int:
    return int(_lib().citrus_static_scratch_bytes())


def citrus_evict_cache_static(cfg: Config, q, k_cache, v_cache, cache_len: int, k: int, k_new, v_new, idx=None,
                              stream=None, rows: Optional[int] = None) -> int:
    """citrus_evict_cache without a workspace: scratch lives in the library's static device array."""
    rows = q.shape[3] if rows is None else rows
    cc = cfg.c()
    st = _lib().citrus_evict_cache_static(C.byref(cc), tensor(q), rows, tensor(k_cache), tensor(v_cache), cache_len, k,
                                          tensor(k_new), tensor(v_new), _ptr(idx), _stream(stream))
    _check(st, "citrus_evict_cache_static")
    return min(k, cache_len)


def citrus_decode_step(cfg: Config, q, k_new, v_new, k_cache, v_cache, cache_len: int, out=None, workspace=None,
                       stream=None):
    """Appends the token's state to row cache_len of the cache (in place) and returns the attention output."""
    if out is None:
        out = torch.empty_like(q)
    cc = cfg.c()
    st = _lib().citrus_decode_step(C.byref(cc), tensor(q), tensor(k_new), tensor(v_new), tensor(k_cache),
                                   tensor(v_cache), cache_len, tensor(out), _ptr(workspace),
                                   0 if workspace is None else workspace.numel(), _stream(stream))
    _check(st, "citrus_decode_step")
    return out


def citrus_rope(cfg: Config, x, pos0: int, y=None, stream=None, rows: Optional[int] = None):
    """Rotary embedding of x [B, L, H, rows, d] at positions pos0, pos0 + 1, ...; y=x rotates in place."""
    rows = x.shape[3] if rows is None else rows
    if y is None:
        y = torch.empty_like(x)
    cc = cfg.c()
    st = _lib().citrus_rope(C.byref(cc), tensor(x), x.shape[2], rows, pos0, tensor(y), _stream(stream))
    _check(st, "citrus_rope")
    return y


def citrus_score_accumulate(cfg: Config, score, acc, cache_len: int, stream=None, n: Optional[int] = None):
    """score[..., j] += acc[..., j] for j < cache_len (in place)."""
    n = score.shape[-1] if n is None else n
    cc = cfg.c()
    st = _lib().citrus_score_accumulate(C.byref(cc), _ptr(score), n, _ptr(acc), cache_len, _stream(stream))
    _check(st, "citrus_score_accumulate")
    return score


def citrus_score_gather(cfg: Config, score, idx, m: int, acc_new, stream=None, n: Optional[int] = None,
                        idx_pitch: Optional[int] = None):
    n = score.shape[-1] if n is None else n
    idx_pitch = idx.shape[-1] if idx_pitch is None else idx_pitch
    cc = cfg.c()
    st = _lib().citrus_score_gather(C.byref(cc), _ptr(score), n, _ptr(idx), idx_pitch, m, _ptr(acc_new), _stream(stream))
    _check(st, "citrus_score_gather")
    return acc_new


def citrus_topk_select(cfg: Config, score, k: int, idx=None, stream=None, n: Optional[int] = None):
    n = score.shape[-1] if n is None else n
    if idx is None:
        idx = torch.full((cfg.batch, cfg.layers, cfg.sel_heads, k), -1, dtype=torch.int32, device=score.device)
    cc = cfg.c()
    st = _lib().citrus_topk_select(C.byref(cc), _ptr(score), n, k, _ptr(idx), None, 0, _stream(stream))
    _check(st, "citrus_topk_select")
    return idx


def citrus_kv_compact(cfg: Config, k_cache, v_cache, cache_len: int, k_chunk, v_chunk, idx, m: int, k_new, v_new,
                      stream=None, chunk_len: Optional[int] = None, idx_pitch: Optional[int] = None):
    chunk_len = k_chunk.shape[3] if chunk_len is None else chunk_len
    idx_pitch = idx.shape[-1] if idx_pitch is None else idx_pitch
    cc = cfg.c()
    st = _lib().citrus_kv_compact(C.byref(cc), tensor(k_cache), tensor(v_cache), cache_len, tensor(k_chunk),
                                  tensor(v_chunk), chunk_len, _ptr(idx), idx_pitch, m, tensor(k_new), tensor(v_new),
                                  _stream(stream))
    _check(st, "citrus_kv_compact")
    return k_new, v_new


def probe_mfma(iters: int, sink: torch.Tensor, stream=None) -> int:
    """Launches the MFMA-only probe kernel; returns the number of MFMA instructions it issues (32768 flop each)."""
    count = C.c_int64(0)
    st = _lib().citrus_probe_mfma(iters, _ptr(sink), sink.numel(), C.byref(count), _stream(stream))
    _check(st, "citrus_probe_mfma")
    return count.value


@dataclass
class DocumentState:
    """Ping-pong cache buffers and the host-side bookkeeping of the chunk loop."""
    k_cache: Sequence[torch.Tensor]
    v_cache: Sequence[torch.Tensor]
    cache_len: int = 0
    buffer_index: int = 0
    k_cache_lm: Optional[Sequence[torch.Tensor]] = None
    v_cache_lm: Optional[Sequence[torch.Tensor]] = None
    cache_len_lm: int = 0
    buffer_index_lm: int = 0
    acc_score: Optional[Sequence[torch.Tensor]] = None   # SCORE_ACCUMULATED: sums of the cache rows, ping-pong

    @staticmethod
    def allocate(cfg: Config, device="cuda") -> "DocumentState":
        shape = (cfg.batch, cfg.layers, cfg.kv_heads, cfg.cache_capacity, cfg.head_dim)
        mk = lambda: [torch.zeros(shape, dtype=cfg.torch_dtype, device=device) for _ in range(2)]
        st = DocumentState(mk(), mk())
        if cfg.cache_mode == CACHE_DUAL:
            st.k_cache_lm, st.v_cache_lm = mk(), mk()
        if cfg.score_mode == SCORE_ACCUMULATED:
            st.acc_score = [torch.zeros((cfg.batch, cfg.layers, cfg.kv_heads, cfg.cache_capacity), dtype=torch.float32,
                                        device=device) for _ in range(2)]
        return st

    def current(self):
        return (self.k_cache[self.buffer_index][:, :, :, :self.cache_len],
                self.v_cache[self.buffer_index][:, :, :, :self.cache_len])

    def current_lm(self):
        return (self.k_cache_lm[self.buffer_index_lm][:, :, :, :self.cache_len_lm],
                self.v_cache_lm[self.buffer_index_lm][:, :, :, :self.cache_len_lm])


def resident_doc(cfg: Config, q, k, v, q_instr, out, doc_len: Optional[int] = None) -> CResidentDoc:
    """q [B,L,Hq,T,d], k/v [B,L,Hkv,T,d], out like q, q_instr [n_chunks,B,L,Hq,n_i,d] or [B,L,Hq,n_i,d]."""
    if q_instr.dim() == 6:
        qi0, stride_chunk = q_instr[0], q_instr.stride(0)
    else:
        qi0, stride_chunk = q_instr, 0
    return CResidentDoc(tensor(q), tensor(k), tensor(v), tensor(out), tensor(qi0), stride_chunk,
                        q.shape[3] if doc_len is None else doc_len, cfg.chunk_len, cfg.dtype)


class SideStream:
    """A second stream and the two events citrus_process_document needs to run a step's selection and
    gather next to its chunk attention.  The events are plain HIP events without timing."""

    def __init__(self, device=None):
        self.stream = torch.cuda.Stream(device=device)
        self._hip = C.CDLL("libamdhip64.so")
        self._hip.hipEventCreateWithFlags.argtypes = [C.POINTER(C.c_void_p), C.c_uint]
        self._hip.hipEventDestroy.argtypes = [C.c_void_p]
        self._events = []
        with torch.cuda.device(self.stream.device):
            for _ in range(2):
                ev = C.c_void_p()
                rc = self._hip.hipEventCreateWithFlags(C.byref(ev), 0x2)  # hipEventDisableTiming
                if rc != 0:
                    raise RuntimeError(f"hipEventCreateWithFlags failed: {rc}")
                self._events.append(ev)
        self.c = CSideStream(C.c_void_p(self.stream.cuda_stream), self._events[0], self._events[1])

    def __del__(self):
        for ev in getattr(self, "_events", []):
            self._hip.hipEventDestroy(ev)


def citrus_process_document(cfg: Config, state: DocumentState, workspace, *, doc: Optional[CResidentDoc] = None,
                            provider: Optional[Callable] = None, first_chunk: int = 0, max_chunks: int = -1,
                            idx_history=None, idx_history_lm=None, phase_events=None, stream=None,
                            side: Optional[SideStream] = None) -> int:
    """Run the chunk loop.  Either ``doc`` (a resident document, served by the
    library's own provider) or ``provider`` (a Python callable
    ``(chunk_index, io: CChunkIO) -> 0 | 1 | negative``) supplies the chunks.
    ``phase_events`` is an optional ctypes array of hipEvent_t handles
    (EVENTS_PER_STEP per step).  ``side``: an optional SideStream; the single-cache
    modes then run selection and gather next to the chunk attention.  Updates
    ``state`` in place and returns the number of chunks processed."""
    lib = _lib()
    if (doc is None) == (provider is None):
        raise ValueError("give exactly one of doc / provider")
    if doc is not None:
        fn = C.cast(lib.citrus_resident_provider, C.c_void_p)
        user = C.cast(C.pointer(doc), C.c_void_p)
        keep = doc
    else:
        def _cb(_user, index, _stream_ptr, io_ptr):
            try:
                return int(provider(index, io_ptr.contents))
            except Exception:  # never let an exception cross the C boundary
                return -1
        keep = PROVIDER(_cb)
        fn = C.cast(keep, C.c_void_p)
        user = None
    arr = lambda ts: (CTensor * 2)(tensor(ts[0]), tensor(ts[1]))
    kc, vc = arr(state.k_cache), arr(state.v_cache)
    dual = state.k_cache_lm is not None
    kl = arr(state.k_cache_lm) if dual else None
    vl = arr(state.v_cache_lm) if dual else None
    n_c, n_c_lm = C.c_int32(state.cache_len), C.c_int32(state.cache_len_lm)
    cur, cur_lm = C.c_int32(state.buffer_index), C.c_int32(state.buffer_index_lm)
    done = C.c_int32(0)
    cc = cfg.c()
    acc = None
    if state.acc_score is not None:
        acc = (C.c_void_p * 2)(state.acc_score[0].data_ptr(), state.acc_score[1].data_ptr())
    st = lib.citrus_process_document(C.byref(cc), fn, user, first_chunk, max_chunks, kc, vc, kl, vl,
                                     C.byref(n_c), C.byref(n_c_lm), C.byref(cur), C.byref(cur_lm), acc,
                                     _ptr(idx_history), _ptr(idx_history_lm), C.byref(done), phase_events, _ptr(workspace),
                                     0 if workspace is None else workspace.numel(), _stream(stream),
                                     None if side is None else C.byref(side.c))
    del keep
    state.cache_len, state.buffer_index = n_c.value, cur.value
    if dual:
        state.cache_len_lm, state.buffer_index_lm = n_c_lm.value, cur_lm.value
    _check(st, "citrus_process_document")
    return done.value
