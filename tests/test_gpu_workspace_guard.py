"""Nothing may be written outside the workspace: every entry point that takes one is called with a block of
exactly citrus_workspace_bytes() bytes cut out of a larger buffer, over call shapes on both sides of every
boundary at which the library changes kernels (the scorers choose by the CALL's candidate and row counts, the
block is sized by the CONFIGURATION's maxima), and the bytes in front of and behind the block must keep their
pattern.  Score mass is checked on the way, so a kernel that quietly lost its scratch would show as well.
Needs an MI355X."""

import numpy as np
import pytest
import torch

import paper_2406_12018_amd as api

pytestmark = pytest.mark.gpu
DEV = "cuda"
GUARD = 1 << 16
PATTERN = 0xA5


def rand(shape, dt, seed, scale=0.3):
    g = torch.Generator().manual_seed(int(seed))
    return (torch.randn(shape, generator=g) * scale).to(dt).to(DEV)


class Guarded:
    def __init__(self, cfg):
        self.n = api.workspace_bytes(cfg)
        self.buf = torch.full((self.n + 2 * GUARD,), PATTERN, dtype=torch.uint8, device=DEV)
        self.ws = self.buf[GUARD:GUARD + self.n]

    def check(self, what):
        torch.cuda.synchronize()
        front = bool((self.buf[:GUARD] == PATTERN).all())
        back = bool((self.buf[GUARD + self.n:] == PATTERN).all())
        assert front and back, f"{what}: bytes outside the workspace were overwritten (front ok {front}, back ok {back})"


CASES = {
    # name: (config, cache lengths to call with, row counts for the calls that take `rows`)
    "g8_one_unit_up_to_2600": (dict(B=1, L=1, Hq=8, Hkv=1, c=64, n_i=64, cap=2600, dtype="bf16"),
                               [0, 1, 31, 32, 1215, 1216, 1217, 2495, 2496, 2497, 2536], [1, 33, 64]),
    "g4_512_rows_two_layers": (dict(B=1, L=2, Hq=8, Hkv=2, c=64, n_i=128, cap=2500, dtype="bf16"),
                               [0, 64, 1216, 1217, 2400, 2436], [1, 64, 128]),
    "many_units_past_the_small_launch_bound": (dict(B=2, L=40, Hq=8, Hkv=8, c=32, n_i=32, cap=1300, dtype="bf16"),
                                               [0, 700, 1248, 1268], [32]),
    "wide_groups_two_launch": (dict(B=1, L=2, Hq=16, Hkv=1, c=128, n_i=40, cap=900, dtype="bf16"),
                               [0, 100, 640, 772], [1, 40]),
    "dual_paper_order_chunk_rows": (dict(B=1, L=2, Hq=8, Hkv=2, c=128, n_i=16, cap=1500, dtype="bf16", dual=True),
                                    [64, 1152, 1153, 1372], [1, 16, 17, 64, 128]),
    "f32_small": (dict(B=2, L=1, Hq=4, Hkv=2, c=32, n_i=8, cap=200, dtype="f32", d=64), [0, 5, 64, 168], [1, 8]),
}


@pytest.mark.parametrize("name", list(CASES))
def test_workspace_is_never_overrun(name):
    spec, cache_lens, row_counts = CASES[name]
    d = spec.get("d", 128)
    dt = torch.bfloat16 if spec["dtype"] == "bf16" else torch.float32
    B, L, Hq, Hkv, c, n_i, cap = (spec[k] for k in ("B", "L", "Hq", "Hkv", "c", "n_i", "cap"))
    G = Hq // Hkv
    extra = dict(cache_mode=api.CACHE_DUAL, budget_lm=cap - c, lm_ordering=api.LM_EVICT_THEN_APPEND) if spec.get("dual") else {}
    cfg = api.Config(batch=B, layers=L, q_heads=Hq, kv_heads=Hkv, head_dim=d, chunk_len=c, budget=cap - c, instr_len=n_i,
                     dtype=api.BF16 if spec["dtype"] == "bf16" else api.F32, cache_capacity=cap, **extra)
    g = Guarded(cfg)
    q, qi = rand((B, L, Hq, c, d), dt, 1), rand((B, L, Hq, n_i, d), dt, 2)
    kc, vc = rand((B, L, Hkv, cap, d), dt, 3), rand((B, L, Hkv, cap, d), dt, 4, 1.0)
    k, v = rand((B, L, Hkv, c, d), dt, 5), rand((B, L, Hkv, c, d), dt, 6, 1.0)
    kn, vn = torch.empty_like(kc), torch.empty_like(vc)
    dq, dk, dv = rand((B, L, Hq, 1, d), dt, 7), rand((B, L, Hkv, 1, d), dt, 8), rand((B, L, Hkv, 1, d), dt, 9, 1.0)
    tol = 5e-3 if spec["dtype"] == "bf16" else 1e-5
    for n_c in cache_lens:
        assert n_c + c <= cap
        print(f"{name}: cache {n_c}", flush=True)
        n = n_c + c
        lm = torch.empty((B, L, Hkv, n), dtype=torch.float32, device=DEV)
        api.citrus_chunk_attn(cfg, q, kc if n_c else None, vc if n_c else None, n_c, k, v, lm_score=lm, workspace=g.ws)
        g.check(f"chunk_attn n_c={n_c}")
        np.testing.assert_allclose(lm.sum(-1).cpu().numpy(), c * G, rtol=tol)
        sc = api.citrus_instr_score(cfg, qi, kc, n_c, k, workspace=g.ws)
        g.check(f"instr_score n_c={n_c}")
        np.testing.assert_allclose(sc.sum(-1).cpu().numpy(), n_i * G, rtol=tol)
        if n_c == 0:
            continue
        for rows in row_counts:
            text = qi if rows <= n_i else q  # rows above the instruction length come from the chunk's queries
            cs = api.citrus_cache_score(cfg, text, kc, n_c, workspace=g.ws, rows=rows)
            g.check(f"cache_score n_c={n_c} rows={rows}")
            np.testing.assert_allclose(cs.sum(-1).cpu().numpy(), rows * G, rtol=tol)
            kept = api.citrus_evict_cache(cfg, text, kc, vc, n_c, min(8, cap - c), kn, vn, workspace=g.ws, rows=rows)
            g.check(f"evict_cache n_c={n_c} rows={rows}")
            assert kept == min(8, n_c)
        if n_c + 1 <= cap:
            kc2, vc2 = kc.clone(), vc.clone()
            api.citrus_decode_step(cfg, dq, dk, dv, kc2, vc2, n_c, workspace=g.ws)
            g.check(f"decode_step n_c={n_c}")


# ----------------------------------------------------------------------------
# the chunk loop: workspace, outputs, both cache pairs, accumulated sums and the index history between guards
# ----------------------------------------------------------------------------

from test_gpu_layouts import Padded  # noqa: E402
from test_gpu_parity import DOC_CASES  # noqa: E402  (the document configurations of the parity tests)
from workloads import make_document  # noqa: E402

GUARD_ELEMS = 4096


class GuardedTensor:
    """A tensor cut out of the middle of a larger buffer whose ends hold a pattern."""

    def __init__(self, shape, dtype, pattern):
        n = int(np.prod(shape))
        self.flat = torch.full((n + 2 * GUARD_ELEMS,), pattern, dtype=dtype, device=DEV)
        self.flat[GUARD_ELEMS:GUARD_ELEMS + n] = 0
        self.t = self.flat[GUARD_ELEMS:GUARD_ELEMS + n].view(shape)
        self.n, self.pattern = n, pattern

    def intact(self):
        return bool((self.flat[:GUARD_ELEMS] == self.pattern).all()) and bool((self.flat[GUARD_ELEMS + self.n:] == self.pattern).all())


GUARDED_DOCS = ["cfg1_ragged", "cfg1_per_layer", "cfg1_dual", "cfg1_chunk_gt_budget", "cfg1_dual_paper_order", "cfg2_small",
                "cfg3_small_shared_mha", "cfg4_small_dual", "cfg4_small_dual_paper_order", "cfg5_small_g8",
                "cfg2_small_accumulated", "cfg2_small_position_shift", "cfg4_small_dual_position_shift",
                "cfg4_small_dual_paper_order_position_shift", "cfg2_small_standard_paper_order", "degenerate_bf16_c64_k1",
                "degenerate_bf16_doc_shorter_than_chunk", "degenerate_bf16_dual_paper_order_c5"]


@pytest.mark.parametrize("name", [n for n in GUARDED_DOCS if n in DOC_CASES])
def test_document_loop_writes_only_what_it_owns(name):
    w = DOC_CASES[name]
    cfg = api.Config.from_workload(w)
    doc = make_document(w, DEV)
    guards = {}

    def g(key, shape, dtype, pattern):
        guards[key] = GuardedTensor(shape, dtype, pattern)
        return guards[key].t

    fpat = 3.0
    cshape = (cfg.batch, cfg.layers, cfg.kv_heads, cfg.cache_capacity, cfg.head_dim)
    state = api.DocumentState([g("k0", cshape, cfg.torch_dtype, fpat), g("k1", cshape, cfg.torch_dtype, fpat)],
                              [g("v0", cshape, cfg.torch_dtype, fpat), g("v1", cshape, cfg.torch_dtype, fpat)])
    if cfg.cache_mode == api.CACHE_DUAL:
        state.k_cache_lm = [g("kl0", cshape, cfg.torch_dtype, fpat), g("kl1", cshape, cfg.torch_dtype, fpat)]
        state.v_cache_lm = [g("vl0", cshape, cfg.torch_dtype, fpat), g("vl1", cshape, cfg.torch_dtype, fpat)]
    if cfg.score_mode == api.SCORE_ACCUMULATED:
        ashape = (cfg.batch, cfg.layers, cfg.kv_heads, cfg.cache_capacity)
        state.acc_score = [g("a0", ashape, torch.float32, fpat), g("a1", ashape, torch.float32, fpat)]
    out = g("out", tuple(doc["q"].shape), cfg.torch_dtype, fpat)
    hist = g("hist", (w.n_chunks, w.batch, w.layers, cfg.sel_heads, w.budget), torch.int32, -77)
    hist_lm = None
    if cfg.cache_mode == api.CACHE_DUAL:
        hist_lm = g("hist_lm", (w.n_chunks, w.batch, w.layers, cfg.sel_heads, w.budget_lm), torch.int32, -77)
    gw = Guarded(cfg)
    rd = api.resident_doc(cfg, doc["q"], doc["k"], doc["v"], doc["q_instr"], out)
    done = api.citrus_process_document(cfg, state, gw.ws, doc=rd, idx_history=hist, idx_history_lm=hist_lm)
    assert done == w.n_chunks
    gw.check(f"{name}: workspace")
    for key, gt in guards.items():
        assert gt.intact(), f"{name}: bytes next to `{key}` were overwritten"

    # the same document read through views with NaN elements around every axis (the ragged last chunk ends where
    # the document ends: one row further is NaN) gives the same bits
    padded = Padded()
    state3 = api.DocumentState.allocate(cfg, DEV)
    out3 = torch.zeros_like(doc["q"])
    rd3 = api.resident_doc(cfg, padded(doc["q"]), padded(doc["k"]), padded(doc["v"]), doc["q_instr"], out3)
    api.citrus_process_document(cfg, state3, api.alloc_workspace(cfg, DEV), doc=rd3)
    torch.cuda.synchronize()
    assert torch.equal(out3, out), f"{name}: elements outside the document's views were read"
    assert padded.untouched()

    # the same document with ordinary allocations gives the same bits
    state2 = api.DocumentState.allocate(cfg, DEV)
    out2 = torch.zeros_like(doc["q"])
    ws2 = api.alloc_workspace(cfg, DEV)
    rd2 = api.resident_doc(cfg, doc["q"], doc["k"], doc["v"], doc["q_instr"], out2)
    api.citrus_process_document(cfg, state2, ws2, doc=rd2)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)
    assert state.cache_len == state2.cache_len and state.buffer_index == state2.buffer_index
    ka, kb = state.current()[0], state2.current()[0]
    assert torch.equal(ka, kb)
