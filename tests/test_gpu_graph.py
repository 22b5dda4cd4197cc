"""The chunk loop under HIP graph capture: citrus_process_document allocates nothing, never synchronises and
takes its chunks from a resident document, so a whole document can be recorded into one graph and replayed.
Every replay (with the program's own eager work and synchronisations in between) must give the bits of the
eager run.  Needs an MI355X."""

import pytest
import torch

import paper_2406_12018_amd as api
from workloads import WORKLOADS, make_document, scaled_down

pytestmark = pytest.mark.gpu
DEV = "cuda"

BASE = dict(layers=2, q_heads=8, kv_heads=2, doc_len=1500, chunk_len=192, budget=256, instr_len=16)
CASES = {
    "single_cache": dict(),
    "dual": dict(cache_mode=api.CACHE_DUAL, budget_lm=192),
    "dual_evict_then_append": dict(cache_mode=api.CACHE_DUAL, budget_lm=192, lm_ordering=api.LM_EVICT_THEN_APPEND),
    "position_shift": dict(position_shift=1),
    "accumulated_per_layer": dict(score_mode=api.SCORE_ACCUMULATED, select_mode=api.SELECT_PER_LAYER),
    "standard": dict(cache_mode=api.CACHE_STANDARD),
    # selection and gather beside the attention launch: the second stream joins the capture at every step's fork
    # event and leaves it at the join event
    "single_cache_second_stream": dict(),
}


def reset(state):
    state.cache_len = state.cache_len_lm = 0
    state.buffer_index = state.buffer_index_lm = 0


def snapshot(state, out, hist):
    kc, vc = state.current()
    parts = [out.clone(), hist.clone(), kc.clone(), vc.clone()]
    if state.k_cache_lm is not None:
        parts += [t.clone() for t in state.current_lm()]
    return parts


@pytest.mark.parametrize("case", sorted(CASES))
def test_document_loop_replays_from_a_graph(case):
    w = scaled_down(WORKLOADS["cfg2_mistral7b"], **BASE, **CASES[case])
    print(f"graph case {case}: {w}", flush=True)
    cfg = api.Config.from_workload(w)
    doc = make_document(w, DEV)
    state = api.DocumentState.allocate(cfg, DEV)
    ws = api.alloc_workspace(cfg, DEV)
    out = torch.zeros_like(doc["q"])
    hist = torch.full((w.n_chunks, w.batch, w.layers, cfg.sel_heads, w.budget), -1, dtype=torch.int32, device=DEV)
    rd = api.resident_doc(cfg, doc["q"], doc["k"], doc["v"], doc["q_instr"], out)

    side = api.SideStream(DEV) if case.endswith("second_stream") else None

    def run():
        reset(state)
        done = api.citrus_process_document(cfg, state, ws, doc=rd, idx_history=hist, side=side)
        assert done == w.n_chunks

    run()  # eager; also raises the kernels' dynamic-LDS limits, which a capture must not do
    torch.cuda.synchronize()
    want = snapshot(state, out, hist)
    lens = (state.cache_len, state.cache_len_lm, state.buffer_index, state.buffer_index_lm)

    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        run()  # warm-up on the capture stream
    stream.synchronize()
    with torch.cuda.graph(graph, stream=stream):
        run()
    assert (state.cache_len, state.cache_len_lm, state.buffer_index, state.buffer_index_lm) == lens
    for replay in range(3):
        # eager work between the replays: outputs, histories and both cache buffers are wiped
        out.zero_()
        hist.fill_(-1)
        for t in list(state.k_cache) + list(state.v_cache) + list(state.k_cache_lm or []) + list(state.v_cache_lm or []):
            t.zero_()
        if state.acc_score is not None:
            for t in state.acc_score:
                t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = snapshot(state, out, hist)
        for i, (a, b) in enumerate(zip(got, want)):
            assert torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a,
                               b.view(torch.int16) if b.dtype == torch.bfloat16 else b), (case, replay, i)


def test_final_eviction_and_decoding_replay_from_a_graph():
    """What follows a document in a serving loop, recorded as one graph: the instruction evicts the cache once more
    through the entry point that allocates nothing (the one meant for callers under capture), then four tokens are
    decoded over the retained states."""
    B, L, Hq, Hkv, d, n, k, rows, steps = 1, 4, 32, 8, 128, 832, 768, 64, 4
    cfg = api.Config(batch=B, layers=L, q_heads=Hq, kv_heads=Hkv, head_dim=d, chunk_len=64, budget=k, instr_len=rows,
                     dtype=api.BF16, cache_capacity=n)
    g = torch.Generator(device="cpu").manual_seed(77)
    mk = lambda *shape, scale=1.0: (torch.randn(shape, generator=g) * scale).bfloat16().to(DEV)
    q_i = mk(B, L, Hq, rows, d, scale=1.5)
    kc, vc = mk(B, L, Hkv, n, d, scale=1.5 * d ** -0.5), mk(B, L, Hkv, n, d)
    q_t, k_t, v_t = mk(steps, B, L, Hq, 1, d), mk(steps, B, L, Hkv, 1, d, scale=d ** -0.5), mk(steps, B, L, Hkv, 1, d)
    ws = api.alloc_workspace(cfg, DEV)
    k_new, v_new = torch.zeros((B, L, Hkv, n, d), dtype=torch.bfloat16, device=DEV), torch.zeros((B, L, Hkv, n, d), dtype=torch.bfloat16, device=DEV)
    idx = torch.full((B, L, Hkv, k), -1, dtype=torch.int32, device=DEV)
    outs = torch.zeros((steps, B, L, Hq, 1, d), dtype=torch.bfloat16, device=DEV)

    def run():
        assert api.citrus_evict_cache_static(cfg, q_i, kc, vc, n, k, k_new, v_new, idx=idx) == k
        for t in range(steps):
            api.citrus_decode_step(cfg, q_t[t], k_t[t], v_t[t], k_new, v_new, k + t, out=outs[t], workspace=ws)

    run()  # eager: looks up the static array's address and raises the dynamic-LDS limits
    torch.cuda.synchronize()
    want = [t.clone() for t in (k_new, v_new, idx, outs)]
    assert (idx[..., 1:] > idx[..., :-1]).all() and outs.float().abs().sum() > 0
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        run()
    stream.synchronize()
    with torch.cuda.graph(graph, stream=stream):
        run()
    for replay in range(3):
        for t in (k_new, v_new, outs):
            t.zero_()
        idx.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(zip((k_new, v_new, idx, outs), want)):
            assert torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a,
                               b.view(torch.int16) if b.dtype == torch.bfloat16 else b), (replay, i)
