"""Shared helpers of the GPU parity tests: tolerances, conversions, the
selection band rule, and a step-by-step driver of the four entry points."""

from __future__ import annotations

import numpy as np
import torch

from oracle import citrus_oracle as orc

TOL = {"f32": (1e-5, 1e-5), "bf16": (2e-2, 1e-2)}   # (atol, rtol): |gpu - ref| <= atol + rtol*|ref|


def np64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def bits(t: torch.Tensor) -> np.ndarray:
    """Raw bit pattern of a tensor (bf16 -> int16, f32 -> int32) on the host."""
    t = t.detach().to("cpu").contiguous()
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32).numpy()


def assert_close(gpu, ref, dtype: str, what: str = ""):
    atol, rtol = TOL[dtype]
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert gpu.shape == ref.shape, (what, gpu.shape, ref.shape)
    err = np.abs(gpu - ref)
    bound = atol + rtol * np.abs(ref)
    bad = err > bound
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside tolerance, max err {err.max():.3e}"
    assert np.isfinite(gpu).all(), what


def check_selection(gpu_idx, gpu_score, ref_score, k: int, dtype: str, what: str = "", start_size: int = 0):
    """The two selection checks for one score vector.

    1. Exact: the GPU's indices are exactly the top-k (lower index wins ties,
       ascending output; the first start_size candidates always kept) of the
       GPU's OWN f32 score vector.
    2. Band rule: against the oracle's selection on the oracle's scores, the
       sets may differ only at positions whose oracle score lies within the
       tolerance of the oracle's last kept score (among the candidates that
       are not kept unconditionally).
    Returns the fraction of positions inside the band.
    """
    gpu_idx = np.asarray(gpu_idx)
    n = ref_score.shape[0]
    m = min(k, n)
    own = orc.topk_select_1d(np.asarray(gpu_score, dtype=np.float32), k, start_size)
    np.testing.assert_array_equal(gpu_idx[:m], own, err_msg=f"{what}: not the exact top-k of its own scores")
    ref_idx = orc.topk_select_1d(ref_score, k, start_size)
    if n <= k:
        np.testing.assert_array_equal(gpu_idx[:m], ref_idx)
        return 0.0
    atol, rtol = TOL[dtype]
    s0 = min(start_size, k)
    if s0 == k:
        np.testing.assert_array_equal(gpu_idx[:m], ref_idx)
        return 0.0
    boundary = np.sort(ref_score[s0:])[::-1][k - s0 - 1]
    band = np.abs(ref_score - boundary) <= atol + rtol * abs(boundary)
    band[:s0] = False  # the unconditional ones can never differ
    diff = np.setxor1d(gpu_idx[:m], ref_idx)
    assert band[diff].all(), f"{what}: selection differs outside the tolerance band at {diff[~band[diff]][:8]}"
    return float(band.mean())


class StepwiseRun:
    """Drives chunk_attn / instr_score / topk_select / kv_compact one chunk at
    a time through the binding, keeping every intermediate for comparison."""

    def __init__(self, api, cfg, device="cuda"):
        self.api, self.cfg = api, cfg
        self.state = api.DocumentState.allocate(cfg, device)
        self.ws = api.alloc_workspace(cfg, device)
        self.steps = []

    def _chunk_evicted_step(self, q, k, v, k_pair, v_pair, n_old, cur, budget):
        """One step of a cache that the document's own chunks evict (the second cache of DUAL, the only
        cache of STANDARD), in the configured ordering, through the public entry points.  Returns the
        intermediates and the cache length after the step; the result is in buffer cur ^ 1."""
        api, cfg = self.api, self.cfg
        c = q.shape[3]
        kl, vl, kl_new, vl_new = k_pair[cur], v_pair[cur], k_pair[cur ^ 1], v_pair[cur ^ 1]
        lse = torch.empty((cfg.batch, cfg.layers, cfg.q_heads, c), dtype=torch.float32, device=q.device)
        # what the attention and the chunk's scores read: with the position shift, copies rotated to the slots
        # of THIS cache; the gathers keep moving the unrotated keys
        q_att, kl_att, k_att = q, kl, k
        if cfg.position_shift:
            k_rot = torch.empty((cfg.batch, cfg.layers, cfg.kv_heads, n_old + c, cfg.head_dim), dtype=q.dtype, device=q.device)
            if n_old > 0:
                api.citrus_rope(cfg, kl, 0, y=k_rot, rows=n_old)
            api.citrus_rope(cfg, k, n_old, y=k_rot[:, :, :, n_old:])
            q_att = api.citrus_rope(cfg, q, n_old)
            kl_att, k_att = k_rot, k_rot[:, :, :, n_old:]
        if cfg.lm_ordering == api.LM_EVICT_THEN_APPEND:
            # Section 4.1's order: encode given the cache, evict the cache by the chunk's attention to it,
            # then append the whole chunk
            kept = min(budget, n_old)
            # when something has to go, the attention launch also returns each row's normaliser over the
            # cache alone, and the cache score is then a single pass over the keys
            lse_cache = None
            if n_old > budget:
                lse_cache = torch.empty((cfg.batch, cfg.layers, cfg.q_heads, c), dtype=torch.float32, device=q.device)
            out = api.citrus_chunk_attn(cfg, q_att, kl_att, vl, n_old, k_att, v, lse=lse, lse_cache=lse_cache)
            score = idx = None
            if n_old > 0:
                if n_old > budget:
                    score = api.citrus_cache_score(cfg, q_att, kl_att, n_old, lse_cache=lse_cache)
                    idx = api.citrus_topk_select(cfg, score, budget)
                else:  # everything stays: the selection does not read the scores
                    unread = torch.zeros((cfg.batch, cfg.layers, cfg.kv_heads, n_old), dtype=torch.float32, device=q.device)
                    idx = api.citrus_topk_select(cfg, unread, budget)
                api.citrus_kv_compact(cfg, kl, vl, n_old, k, v, idx, kept, kl_new, vl_new)
            tail = torch.arange(n_old, n_old + c, dtype=torch.int32, device=q.device).expand(
                cfg.batch, cfg.layers, cfg.sel_heads, c).contiguous()
            api.citrus_kv_compact(cfg, kl, vl, n_old, k, v, tail, c, kl_new[:, :, :, kept:], vl_new[:, :, :, kept:])
            return dict(out=out, lse=lse, score=score, idx=idx, kept=kept, new_len=kept + c)
        n_new = n_old + c
        score = torch.empty((cfg.batch, cfg.layers, cfg.kv_heads, n_new), dtype=torch.float32, device=q.device)
        out = api.citrus_chunk_attn(cfg, q_att, kl_att, vl, n_old, k_att, v, lse=lse, lm_score=score, workspace=self.ws)
        idx = api.citrus_topk_select(cfg, score, budget)
        kept = min(budget, n_new)
        api.citrus_kv_compact(cfg, kl, vl, n_old, k, v, idx, kept, kl_new, vl_new)
        return dict(out=out, lse=lse, score=score, idx=idx, kept=kept, new_len=kept)

    def step(self, q, k, v, q_instr):
        api, cfg, st = self.api, self.cfg, self.state
        dual = cfg.cache_mode == api.CACHE_DUAL
        c = q.shape[3]
        rec = {"n_c": st.cache_len}
        if cfg.cache_mode == api.CACHE_STANDARD:
            r = self._chunk_evicted_step(q, k, v, st.k_cache, st.v_cache, st.cache_len, st.buffer_index, cfg.budget)
            st.buffer_index ^= 1
            st.cache_len = r["new_len"]
            rec.update(out=r["out"], lse=r["lse"], score=r["score"], idx=r["idx"], m=r["kept"])
            self.steps.append(rec)
            return rec
        kc, vc = st.k_cache[st.buffer_index], st.v_cache[st.buffer_index]
        n = st.cache_len + c
        # what attention and scores read: with the position shift, copies rotated to this step's positions
        q_att, qi_att, kc_att, k_att = q, q_instr, kc, k
        if cfg.position_shift:
            n_c = st.cache_len
            k_rot = torch.empty((cfg.batch, cfg.layers, cfg.kv_heads, n, cfg.head_dim), dtype=q.dtype, device=q.device)
            if n_c > 0:
                api.citrus_rope(cfg, kc, 0, y=k_rot, rows=n_c)
            api.citrus_rope(cfg, k, n_c, y=k_rot[:, :, :, n_c:])
            if not dual:   # DUAL: the chunk attends over the other cache, at that cache's positions
                q_att = api.citrus_rope(cfg, q, n_c)
            qi_att = api.citrus_rope(cfg, q_instr, n)
            kc_att, k_att = k_rot, k_rot[:, :, :, n_c:]
        if dual:
            r = self._chunk_evicted_step(q, k, v, st.k_cache_lm, st.v_cache_lm, st.cache_len_lm, st.buffer_index_lm,
                                         cfg.budget_lm)
            rec.update(n_c_lm=st.cache_len_lm, score_lm=r["score"], idx_lm=r["idx"], m_lm=r["kept"], lse=r["lse"])
            out = r["out"]
            st.buffer_index_lm ^= 1
            st.cache_len_lm = r["new_len"]
        else:
            lse = torch.empty((cfg.batch, cfg.layers, cfg.q_heads, c), dtype=torch.float32, device=q.device)
            out = api.citrus_chunk_attn(cfg, q_att, kc_att, vc, st.cache_len, k_att, v, lse=lse)
            rec["lse"] = lse
        score = api.citrus_instr_score(cfg, qi_att, kc_att, st.cache_len, k_att, workspace=self.ws)
        accumulated = cfg.score_mode == api.SCORE_ACCUMULATED
        if accumulated:  # a cache state's sum so far joins this step's score
            api.citrus_score_accumulate(cfg, score, st.acc_score[st.buffer_index], st.cache_len)
        idx = api.citrus_topk_select(cfg, score, cfg.budget)
        m = min(cfg.budget, n)
        api.citrus_kv_compact(cfg, kc, vc, st.cache_len, k, v, idx, m, st.k_cache[st.buffer_index ^ 1],
                              st.v_cache[st.buffer_index ^ 1])
        if accumulated:  # and the kept states carry their sums on
            api.citrus_score_gather(cfg, score, idx, m, st.acc_score[st.buffer_index ^ 1])
        st.buffer_index ^= 1
        st.cache_len = m
        rec.update(out=out, score=score, idx=idx, m=m)
        self.steps.append(rec)
        return rec
