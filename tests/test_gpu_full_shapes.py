"""Parity with the oracle at the STATED shapes of the Llama-2 MHA (shared cache), dual-cache and large-layer
configurations: key ranges of 2048 and 6144 candidates, 64- to 128-chunk trajectories, 128 to 320
(document, layer) units per launch, and the provider path of citrus_process_document with chunks generated
from the seeded recipe on the stream.  Needs an MI355X.

Two tests per configuration:
  document  a whole document at the configuration's per-unit shape (T, c, k, n_i, heads, cache mode) for one
            document and two layers, fed by a provider that generates chunk i when the loop asks for it.  The
            oracle replays the selection history (integer gathers) and, at sampled steps, checks outputs,
            log-sum-exp, scores, the band rule and the exact top-k of the GPU's own scores; the final caches
            are compared bit for bit.
  step      one steady-state step at the configuration's full batch x layers through the four entry points,
            three units checked against the oracle.
The oracle works on a subset of the KV groups where a unit is large (its attention is 344 GFLOP per unit and
step at the large-layer shape)."""

import numpy as np
import pytest
import torch

import paper_2406_12018_amd as api
from oracle import citrus_oracle as orc
from workloads import WORKLOADS, make_chunk_sliced, peaked

from helpers import assert_close, bits, check_selection, np64

pytestmark = pytest.mark.gpu
DEV = "cuda"


def say(msg):
    print(msg, flush=True)


# name -> (workload, layers of document 0 that the document test runs, sampled steps, KV groups the oracle covers)
FULL_SHAPES = {
    "cfg3": (WORKLOADS["cfg3_llama2_7b_shared"], (0, 31), (0, 1, 2, 17, 31), (0, 13, 31)),
    "cfg4": (WORKLOADS["cfg4_dual"], (0, 31), (0, 1, 2, 64, 127), (0, 3, 7)),
    "cfg5": (WORKLOADS["cfg5_large"], (0, 79), (0, 2, 3, 33, 63), (0, 7)),
}


def heads_of(w, groups):
    g = w.group
    return [h for kv in groups for h in range(kv * g, (kv + 1) * g)]


def gather_rows(doc_blg, pos):
    """doc_blg [Hkv, T, d] (device), pos [Hkv, n] (host int64) -> [Hkv, n, d] on the device."""
    p = torch.from_numpy(pos).to(doc_blg.device)
    return torch.stack([doc_blg[g][p[g]] for g in range(doc_blg.shape[0])])


def check_unit_step(w, what, groups, q, qi, kc, vc, k_ch, v_ch, idx_doc, out_doc, lm=None):
    """One (document, layer) unit at one step, stand-alone through the entry points on the replayed cache.

    q [Hq, c, d], qi [Hq, n_i, d], kc / vc [Hkv, n_c, d] (the instruction or only cache), k_ch / v_ch [Hkv, c, d],
    idx_doc [Hkv, m]: what the document run selected, out_doc [Hq, c, d]: what it wrote.
    lm (DUAL): dict(kc, vc, idx_doc, budget) of the language-modelling cache, which the chunk attends over."""
    one = api.Config.from_workload(w, batch=1, layers=1)
    ws = api.alloc_workspace(one, DEV)
    u5 = lambda t: t[None, None]
    c, n_c = q.shape[1], kc.shape[1]
    n = n_c + c
    att_k, att_v = (lm["kc"], lm["vc"]) if lm is not None else (kc, vc)
    n_att = att_k.shape[1]
    lse = torch.empty((1, 1, w.q_heads, c), dtype=torch.float32, device=DEV)
    score_lm = None
    if lm is not None:
        score_lm = torch.empty((1, 1, w.kv_heads, n_att + c), dtype=torch.float32, device=DEV)
    out = api.citrus_chunk_attn(one, u5(q), u5(att_k), u5(att_v), n_att, u5(k_ch), u5(v_ch), lse=lse, lm_score=score_lm,
                                workspace=ws)
    score = api.citrus_instr_score(one, u5(qi), u5(kc), n_c, u5(k_ch), workspace=ws)
    idx = api.citrus_topk_select(one, score, w.budget)
    torch.cuda.synchronize()
    m = min(w.budget, n)
    # the batched document run and the stand-alone step do the same arithmetic per unit
    assert torch.equal(out[0, 0], out_doc), f"{what}: output differs from the stand-alone step"
    assert torch.equal(idx[0, 0, :, :m].cpu(), torch.from_numpy(idx_doc[:, :m]).to(torch.int32)), f"{what}: selection"
    hs = heads_of(w, groups)
    gl = list(groups)
    kcat = np.concatenate([np64(att_k[gl]), np64(k_ch[gl])], axis=1)
    vcat = np.concatenate([np64(att_v[gl]), np64(v_ch[gl])], axis=1)
    q64 = np64(q[hs])
    o_ref, lse_ref, _ = orc.chunk_attn(q64, kcat, vcat, n_att)
    assert_close(np64(out[0, 0][hs]), o_ref, w.dtype, f"{what}: out")
    assert_close(np64(lse[0, 0][hs]), lse_ref, w.dtype, f"{what}: lse")
    fracs = []
    if lm is not None:
        s_lm_ref = orc.lm_score(q64, kcat, n_att)
        assert_close(np64(score_lm[0, 0][gl]), s_lm_ref, w.dtype, f"{what}: lm_score")
        np.testing.assert_allclose(np64(score_lm[0, 0]).sum(-1), c * w.group, rtol=2e-3)
        idx_lm = api.citrus_topk_select(one, score_lm, lm["budget"])
        m_lm = min(lm["budget"], n_att + c)
        assert torch.equal(idx_lm[0, 0, :, :m_lm].cpu(), torch.from_numpy(lm["idx_doc"][:, :m_lm]).to(torch.int32))
        for x, g in enumerate(gl):
            fracs.append(check_selection(lm["idx_doc"][g], score_lm[0, 0, g].cpu().numpy(), s_lm_ref[x], lm["budget"],
                                         w.dtype, f"{what}: lm select g{g}"))
        kcat = np.concatenate([np64(kc[gl]), np64(k_ch[gl])], axis=1)
    s_ref = orc.instr_score(np64(qi[hs]), kcat)
    assert_close(np64(score[0, 0][gl]), s_ref, w.dtype, f"{what}: score")
    np.testing.assert_allclose(np64(score[0, 0]).sum(-1), w.instr_len * w.group, rtol=2e-3)
    for x, g in enumerate(gl):
        fracs.append(check_selection(idx_doc[g], score[0, 0, g].cpu().numpy(), s_ref[x], w.budget, w.dtype,
                                     f"{what}: select g{g}"))
    return fracs


@pytest.mark.parametrize("name", list(FULL_SHAPES), ids=list(FULL_SHAPES))
def test_full_shape_document_through_seeded_provider(name):
    w, layers, sample_steps, groups = FULL_SHAPES[name]
    say(f"full-shape document {w.name}: T {w.doc_len} c {w.chunk_len} k {w.budget} n_i {w.instr_len} "
        f"{w.q_heads}/{w.kv_heads} heads, document 0, layers {layers}")
    dual = w.cache_mode == api.CACHE_DUAL
    L = len(layers)
    cfg = api.Config.from_workload(w, batch=1, layers=L)
    state = api.DocumentState.allocate(cfg, DEV)
    ws = api.alloc_workspace(cfg, DEV)
    hist = torch.full((w.n_chunks, 1, L, w.kv_heads, w.budget), -1, dtype=torch.int32, device=DEV)
    hist_lm = torch.full((w.n_chunks, 1, L, w.kv_heads, w.budget_lm), -1, dtype=torch.int32, device=DEV) if dual else None
    chunks = []

    def provider(i, io):   # chunk i of the seeded recipe, generated on the stream when the loop asks for it
        if i >= w.n_chunks:
            return 1
        ch = make_chunk_sliced(w, i, DEV, b=[0], l=list(layers))
        ch["out"] = torch.zeros_like(ch["q"])
        chunks.append(ch)
        io.q, io.k, io.v = api.binding.tensor(ch["q"]), api.binding.tensor(ch["k"]), api.binding.tensor(ch["v"])
        io.q_instr, io.out = api.binding.tensor(ch["q_instr"]), api.binding.tensor(ch["out"])
        io.chunk_len = ch["q"].shape[3]
        return 0

    done = api.citrus_process_document(cfg, state, ws, provider=provider, idx_history=hist, idx_history_lm=hist_lm)
    torch.cuda.synchronize()
    assert done == w.n_chunks == len(chunks)
    assert state.cache_len == w.budget and (not dual or state.cache_len_lm == w.budget_lm)
    k_doc = torch.cat([ch["k"] for ch in chunks], dim=3)[0]   # [L, Hkv, T, d]
    v_doc = torch.cat([ch["v"] for ch in chunks], dim=3)[0]
    hist_h = hist.cpu().numpy().astype(np.int64)
    hist_lm_h = hist_lm.cpu().numpy().astype(np.int64) if dual else None
    fracs = []
    for li, layer in enumerate(layers):
        pos = np.zeros((w.kv_heads, 0), dtype=np.int64)
        pos_lm = np.zeros((w.kv_heads, 0), dtype=np.int64)
        for i in range(w.n_chunks):
            lo, hi = w.chunk_bounds(i)
            new = np.broadcast_to(np.arange(lo, hi), (w.kv_heads, hi - lo))
            cand = np.concatenate([pos, new], axis=1)
            m = min(w.budget, cand.shape[1])
            idx = hist_h[i, 0, li][:, :m]
            assert (np.diff(idx, axis=1) > 0).all() and idx.min() >= 0 and idx.max() < cand.shape[1], f"step {i}"
            if dual:
                cand_lm = np.concatenate([pos_lm, new], axis=1)
                m_lm = min(w.budget_lm, cand_lm.shape[1])
                idx_lm = hist_lm_h[i, 0, li][:, :m_lm]
                assert (np.diff(idx_lm, axis=1) > 0).all() and idx_lm.min() >= 0 and idx_lm.max() < cand_lm.shape[1]
            if i in sample_steps:
                ch = chunks[i]
                lm = None
                if dual:
                    lm = dict(kc=gather_rows(k_doc[li], pos_lm), vc=gather_rows(v_doc[li], pos_lm), idx_doc=idx_lm,
                              budget=w.budget_lm)
                fracs += check_unit_step(w, f"{w.name} layer {layer} step {i}", groups, ch["q"][0, li], ch["q_instr"][0, li],
                                         gather_rows(k_doc[li], pos), gather_rows(v_doc[li], pos), ch["k"][0, li],
                                         ch["v"][0, li], idx, ch["out"][0, li], lm)
            pos = np.stack([cand[g][idx[g]] for g in range(w.kv_heads)])
            if dual:
                pos_lm = np.stack([cand_lm[g][idx_lm[g]] for g in range(w.kv_heads)])
        # the caches the document run left behind hold exactly the replayed document rows
        kc_gpu, vc_gpu = state.current()
        assert torch.equal(kc_gpu[0, li], gather_rows(k_doc[li], pos)) and torch.equal(vc_gpu[0, li], gather_rows(v_doc[li], pos))
        if dual:
            kl_gpu, vl_gpu = state.current_lm()
            assert torch.equal(kl_gpu[0, li], gather_rows(k_doc[li], pos_lm))
            assert torch.equal(vl_gpu[0, li], gather_rows(v_doc[li], pos_lm))
    say(f"{w.name}: mean in-band fraction of the selection band rule = {np.mean(fracs):.3f}")


STEP_CASES = {
    "cfg3": (WORKLOADS["cfg3_llama2_7b_shared"], ((0, 0), (1, 17), (3, 31)), (0, 13, 31)),
    "cfg4": (WORKLOADS["cfg4_dual"], ((0, 0), (4, 9), (7, 31)), (0, 3, 7)),
    "cfg5": (WORKLOADS["cfg5_large"], ((0, 0), (2, 41), (3, 79)), (0, 7)),
    "cfg5_peaked": (peaked(WORKLOADS["cfg5_large"]), ((0, 0), (3, 79)), (5,)),
    "cfg2_peaked": (peaked(WORKLOADS["cfg2_mistral7b"]), ((0, 0), (0, 9), (0, 31)), tuple(range(8))),
}


@pytest.mark.parametrize("name", list(STEP_CASES), ids=list(STEP_CASES))
def test_full_shape_steady_state_step(name):
    """All batch x layers units of the configuration in one launch per entry point; a few units checked."""
    w, units, groups = STEP_CASES[name]
    say(f"full-shape step {w.name}: B {w.batch} L {w.layers} c {w.chunk_len} cache {w.budget} n_i {w.instr_len}")
    dual = w.cache_mode == api.CACHE_DUAL
    cfg = api.Config.from_workload(w)
    ws = api.alloc_workspace(cfg, DEV)
    i_step = (w.budget + w.chunk_len - 1) // w.chunk_len + 1          # a chunk that meets a full cache
    ch = make_chunk_sliced(w, i_step, DEV)
    gen = torch.Generator(device=DEV).manual_seed(w.seed)
    kscale = 1.0 if w.peaked else w.head_dim ** -0.5

    def cache(budget, scale):   # a full cache with the workload's plain value distribution
        t = torch.empty((w.batch, w.layers, w.kv_heads, budget, w.head_dim), dtype=w.torch_dtype, device=DEV)
        for b in range(w.batch):
            t[b] = (torch.randn(t.shape[1:], generator=gen, device=DEV, dtype=torch.float32) * scale).to(w.torch_dtype)
        return t

    kc, vc = cache(w.budget, kscale), cache(w.budget, w.head_dim ** -0.5)
    n_c = w.budget
    att_k, att_v, n_att = kc, vc, n_c
    score_lm = None
    if dual:
        att_k, att_v, n_att = cache(w.budget_lm, kscale), cache(w.budget_lm, w.head_dim ** -0.5), w.budget_lm
        score_lm = torch.empty((w.batch, w.layers, w.kv_heads, n_att + w.chunk_len), dtype=torch.float32, device=DEV)
    lse = torch.empty((w.batch, w.layers, w.q_heads, w.chunk_len), dtype=torch.float32, device=DEV)
    out = api.citrus_chunk_attn(cfg, ch["q"], att_k, att_v, n_att, ch["k"], ch["v"], lse=lse, lm_score=score_lm, workspace=ws)
    score = api.citrus_instr_score(cfg, ch["q_instr"], kc, n_c, ch["k"], workspace=ws)
    idx = api.citrus_topk_select(cfg, score, w.budget)
    kn, vn = torch.zeros_like(kc), torch.zeros_like(vc)
    api.citrus_kv_compact(cfg, kc, vc, n_c, ch["k"], ch["v"], idx, w.budget, kn, vn)
    if dual:
        idx_lm = api.citrus_topk_select(cfg, score_lm, w.budget_lm)
        kn_lm, vn_lm = torch.zeros_like(att_k), torch.zeros_like(att_v)
        api.citrus_kv_compact(cfg, att_k, att_v, n_att, ch["k"], ch["v"], idx_lm, w.budget_lm, kn_lm, vn_lm)
    torch.cuda.synchronize()
    np.testing.assert_allclose(np64(score).sum(-1), w.instr_len * w.group, rtol=2e-3)
    hs, gl = heads_of(w, groups), list(groups)
    fracs = []
    for (b, l) in units:
        what = f"{w.name} unit {(b, l)}"
        kcat = np.concatenate([np64(att_k[b, l][gl]), np64(ch["k"][b, l][gl])], axis=1)
        vcat = np.concatenate([np64(att_v[b, l][gl]), np64(ch["v"][b, l][gl])], axis=1)
        q64 = np64(ch["q"][b, l][hs])
        o_ref, lse_ref, _ = orc.chunk_attn(q64, kcat, vcat, n_att)
        assert_close(np64(out[b, l][hs]), o_ref, w.dtype, f"{what}: out")
        assert_close(np64(lse[b, l][hs]), lse_ref, w.dtype, f"{what}: lse")
        if dual:
            s_lm_ref = orc.lm_score(q64, kcat, n_att)
            assert_close(np64(score_lm[b, l][gl]), s_lm_ref, w.dtype, f"{what}: lm_score")
            for x, g in enumerate(gl):
                fracs.append(check_selection(idx_lm[b, l, g].cpu().numpy(), score_lm[b, l, g].cpu().numpy(), s_lm_ref[x],
                                             w.budget_lm, w.dtype, f"{what}: lm select g{g}"))
            kb = np.concatenate([bits(att_k[b, l]), bits(ch["k"][b, l])], axis=1)
            vb = np.concatenate([bits(att_v[b, l]), bits(ch["v"][b, l])], axis=1)
            k_ref, v_ref = orc.kv_compact(kb, vb, idx_lm[b, l].cpu().numpy())
            np.testing.assert_array_equal(bits(kn_lm[b, l]), k_ref)
            np.testing.assert_array_equal(bits(vn_lm[b, l]), v_ref)
            kcat = np.concatenate([np64(kc[b, l][gl]), np64(ch["k"][b, l][gl])], axis=1)
        s_ref = orc.instr_score(np64(ch["q_instr"][b, l][hs]), kcat)
        assert_close(np64(score[b, l][gl]), s_ref, w.dtype, f"{what}: score")
        for x, g in enumerate(gl):
            fracs.append(check_selection(idx[b, l, g].cpu().numpy(), score[b, l, g].cpu().numpy(), s_ref[x], w.budget,
                                         w.dtype, f"{what}: select g{g}"))
        kb = np.concatenate([bits(kc[b, l]), bits(ch["k"][b, l])], axis=1)
        vb = np.concatenate([bits(vc[b, l]), bits(ch["v"][b, l])], axis=1)
        k_ref, v_ref = orc.kv_compact(kb, vb, idx[b, l].cpu().numpy())
        np.testing.assert_array_equal(bits(kn[b, l]), k_ref)
        np.testing.assert_array_equal(bits(vn[b, l]), v_ref)
    say(f"{w.name}: mean in-band fraction of the selection band rule = {np.mean(fracs):.3f}")
