"""Pins of the CPU oracle against things other than itself: a hand-evaluated
example, closed forms, invariants, brute force in pure Python, and torch's CPU
attention routine as a library special case.  CPU only."""

import json
import math
import os

import numpy as np
import pytest
import torch

from oracle import citrus_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "eq1_two_key_example.json")


def rng(seed):
    return np.random.default_rng(seed)


# ----------------------------------------------------------------------------
# hand-evaluated example (Eq. (1), Section 4.1 step 1)
# ----------------------------------------------------------------------------

def _golden_keys(g):
    a = 2.0 * math.log(3.0)
    k = np.zeros((g["kv_heads"], 2, g["head_dim"]))
    for h, row in enumerate(g["key_first_coord"]):
        for j, s in enumerate(row):
            k[h, j, 0] = a if s == "2ln3" else 0.0
    return k


def test_golden_instr_score():
    g = json.load(open(GOLDEN))
    k = _golden_keys(g)
    qi = np.zeros((g["q_heads"], 2, g["head_dim"]))
    qi[:, :, 0] = np.array(g["instr_query_first_coord"], dtype=float)
    s = orc.instr_score(qi, k)
    np.testing.assert_allclose(s, np.array(g["instr_score_expected"]), rtol=0, atol=1e-14)
    assert abs(s[0].sum() - g["instr_score_mass"]) < 1e-14


def test_golden_chunk_attn_and_lm_score():
    g = json.load(open(GOLDEN))
    k = _golden_keys(g)
    v = np.zeros_like(k)
    v[:, 0, 0] = 1.0
    v[:, 1, 1] = 1.0
    q = np.zeros((g["q_heads"], 1, g["head_dim"]))
    q[:, 0, 0] = np.array(g["chunk_attn"]["query_first_coord"], dtype=float)
    out, lse, probs = orc.chunk_attn(q, k, v, n_c=1)
    np.testing.assert_allclose(out[:, 0, :], np.array(g["chunk_attn"]["out_expected"], dtype=float), atol=1e-14)
    np.testing.assert_allclose(orc.lm_score(q, k, n_c=1), np.array(g["chunk_attn"]["lm_score_expected"]), atol=1e-14)
    # lse of head 0: log(3 + 1)
    assert abs(lse[0, 0] - math.log(4.0)) < 1e-14


def test_golden_causal_two_token_chunk():
    g = json.load(open(GOLDEN))
    k = _golden_keys(g)[:1]
    v = np.zeros_like(k)
    v[0, 0, 0] = 1.0
    v[0, 1, 1] = 1.0
    q = np.zeros((1, 2, 4))
    q[0, :, 0] = 1.0
    out, _, _ = orc.chunk_attn(q, k, v, n_c=0)
    np.testing.assert_allclose(out[0], np.array(g["causal_two_token_chunk"]["out_expected"], dtype=float), atol=1e-14)
    np.testing.assert_allclose(orc.lm_score(q, k, n_c=0)[0], g["causal_two_token_chunk"]["lm_score_expected"], atol=1e-14)


# ----------------------------------------------------------------------------
# brute force in pure Python (no numpy arithmetic) on tiny shapes
# ----------------------------------------------------------------------------

def _py_attention(q, kc, vc, n_c, scale):
    """Nested-loop causal attention for one (query head, kv head) pair."""
    c, d = len(q), len(q[0])
    out, probs = [], []
    for t in range(c):
        last = n_c + t
        logits = [scale * sum(q[t][x] * kc[j][x] for x in range(d)) for j in range(last + 1)]
        m = max(logits)
        e = [math.exp(s - m) for s in logits]
        z = sum(e)
        p = [x / z for x in e] + [0.0] * (len(kc) - last - 1)
        probs.append(p)
        out.append([sum(p[j] * vc[j][x] for j in range(last + 1)) for x in range(d)])
    return out, probs


@pytest.mark.parametrize("hq,hkv,c,n_c,d", [(4, 2, 5, 3, 8), (3, 3, 4, 0, 4), (6, 2, 1, 7, 8)])
def test_chunk_attn_and_scores_vs_python_loops(hq, hkv, c, n_c, d):
    r = rng(hq * 100 + c)
    n = n_c + c
    q = r.normal(size=(hq, c, d))
    k = r.normal(size=(hkv, n, d))
    v = r.normal(size=(hkv, n, d))
    qi = r.normal(size=(hq, 3, d))
    out, lse, probs = orc.chunk_attn(q, k, v, n_c)
    g_size = hq // hkv
    scale = 1.0 / math.sqrt(d)
    lm = [[0.0] * n for _ in range(hkv)]
    ins = [[0.0] * n for _ in range(hkv)]
    for h in range(hq):
        g = h // g_size
        o_py, p_py = _py_attention(q[h].tolist(), k[g].tolist(), v[g].tolist(), n_c, scale)
        np.testing.assert_allclose(out[h], np.array(o_py), atol=1e-12)
        for t in range(c):
            for j in range(n):
                lm[g][j] += p_py[t][j]
        # instruction rows: no mask, softmax over all n keys
        for u in range(3):
            logits = [scale * sum(qi[h, u, x] * k[g, j, x] for x in range(d)) for j in range(n)]
            z = sum(math.exp(s) for s in logits)
            for j in range(n):
                ins[g][j] += math.exp(logits[j]) / z
    np.testing.assert_allclose(orc.lm_score(q, k, n_c), np.array(lm), atol=1e-12)
    np.testing.assert_allclose(orc.instr_score(qi, k), np.array(ins), atol=1e-12)


def _py_topk(score, k):
    """Repeatedly remove the best remaining candidate (highest score, then
    lowest index)."""
    n = len(score)
    if n <= k:
        return list(range(n))
    alive = list(range(n))
    chosen = []
    for _ in range(k):
        best = alive[0]
        for j in alive[1:]:
            if score[j] > score[best]:
                best = j
        alive.remove(best)
        chosen.append(best)
    return sorted(chosen)


@pytest.mark.parametrize("n,k,levels", [(17, 5, None), (64, 64, None), (40, 39, 3), (33, 1, 2), (50, 20, 4), (9, 30, None)])
def test_topk_vs_bruteforce(n, k, levels):
    r = rng(n * 1000 + k)
    for _ in range(20):
        s = r.random(n) if levels is None else r.integers(0, levels, n).astype(np.float64)
        assert orc.topk_select_1d(s, k).tolist() == _py_topk(s.tolist(), k)


def test_topk_equals_full_sort_set():
    r = rng(5)
    s = r.random(300)
    idx = orc.topk_select_1d(s, 100)
    assert set(idx.tolist()) == set(np.argsort(s)[::-1][:100].tolist())
    assert np.all(np.diff(idx) > 0)


def _py_topk_start(score, k, s0):
    """The appendix variant written out on its own: the first s0 candidates are taken, then the best
    remaining candidate (highest score, then lowest index) is taken k - s0 times."""
    n = len(score)
    if n <= k:
        return list(range(n))
    chosen = list(range(min(s0, k)))
    alive = [j for j in range(n) if j not in chosen]
    while len(chosen) < k:
        best = alive[0]
        for j in alive[1:]:
            if score[j] > score[best]:
                best = j
        chosen.append(best)
        alive.remove(best)
    return sorted(chosen)


@pytest.mark.parametrize("n,k,s0,levels", [(17, 5, 2, None), (40, 39, 4, 3), (33, 4, 4, 2), (50, 20, 1, 4), (9, 30, 3, None),
                                          (25, 6, 0, None)])
def test_topk_with_start_size_vs_bruteforce(n, k, s0, levels):
    r = rng(n * 977 + k + s0)
    for _ in range(20):
        s = r.random(n) if levels is None else r.integers(0, levels, n).astype(np.float64)
        got = orc.topk_select_1d(s, k, s0).tolist()
        assert got == _py_topk_start(s.tolist(), k, s0)
        if n > k:
            assert got[:min(s0, k)] == list(range(min(s0, k)))
    # start_size = 0 is the plain selection
    s = r.random(30)
    assert orc.topk_select_1d(s, 7, 0).tolist() == _py_topk(s.tolist(), 7)


def test_start_size_changes_nothing_when_the_first_states_win_anyway():
    r = rng(77)
    s = r.random(60)
    s[:4] += 10.0  # the first four are the four best
    np.testing.assert_array_equal(orc.topk_select_1d(s, 12, 4), orc.topk_select_1d(s, 12))
    s[:4] -= 20.0  # now the four worst: forced in, and the eight best of the rest beside them
    forced = orc.topk_select_1d(s, 12, 4)
    np.testing.assert_array_equal(forced[:4], np.arange(4))
    np.testing.assert_array_equal(forced[4:], 4 + orc.topk_select_1d(s[4:], 8))
    assert not set(range(4)) & set(orc.topk_select_1d(s, 12).tolist())


@pytest.mark.parametrize("mode", [orc.CACHE_INSTR, orc.CACHE_DUAL])
def test_document_start_size_keeps_the_first_states(mode):
    """Keys at document positions 0..3 are made repulsive for every query, so that plain eviction drops
    them; with start_size = 4 they stay at the front of every cache, the rest follows the usual rule."""
    hq, hkv, t, d, chunk, budget = 4, 2, 64, 8, 8, 12
    q, k, v, qi = _doc(91, hq, hkv, t, d, 3, chunk)
    q, qi = np.abs(q), [np.abs(x) for x in qi]
    k[:, :4] = -3.0 * np.abs(k[:, :4]) - 1.0   # all logits against positive queries strongly negative
    plain = orc.process_document(q, k, v, qi, chunk, budget, cache_mode=mode, budget_lm=budget)
    kept = orc.process_document(q, k, v, qi, chunk, budget, cache_mode=mode, budget_lm=budget, start_size=4)
    assert not (plain.positions < 4).any()
    np.testing.assert_array_equal(kept.positions[:, :4], np.tile(np.arange(4), (hkv, 1)))
    np.testing.assert_array_equal(kept.k_cache[:, :4], k[:, :4])
    assert np.all(np.diff(kept.positions, axis=1) > 0) and kept.positions.shape == (hkv, budget)
    if mode == orc.CACHE_DUAL:
        np.testing.assert_array_equal(kept.positions_lm[:, :4], np.tile(np.arange(4), (hkv, 1)))
    # every step's selection: the first four candidates, then the plain rule on the rest with k - 4 places
    for tr in kept.trace:
        if tr.idx.shape[1] < tr.score.shape[1]:
            for g in range(hkv):
                np.testing.assert_array_equal(tr.idx[g, :4], np.arange(4))
                np.testing.assert_array_equal(tr.idx[g, 4:], 4 + orc.topk_select_1d(tr.score[g, 4:], budget - 4))


def test_topk_per_layer_sums_heads():
    s = np.array([[0.9, 0.1, 0.5, 0.0], [0.0, 0.2, 0.6, 0.3]])
    # per head: top-2 are {0,2} and {2,3}; layer-wise sums are .9 .3 1.1 .3 -> {0,2}
    np.testing.assert_array_equal(orc.topk_select(s, 2), [[0, 2], [2, 3]])
    np.testing.assert_array_equal(orc.topk_select(s, 2, orc.SELECT_PER_LAYER), [[0, 2]])
    # layer-wise tie between positions 1 and 3 (sum .3 each): the lower index wins
    np.testing.assert_array_equal(orc.topk_select(s, 3, orc.SELECT_PER_LAYER), [[0, 1, 2]])


# ----------------------------------------------------------------------------
# invariants and closed forms
# ----------------------------------------------------------------------------

def test_softmax_rows_sum_to_one_and_mass():
    r = rng(11)
    hq, hkv, c, n_c, d, n_i = 8, 2, 16, 24, 16, 5
    q = r.normal(size=(hq, c, d)) * 3
    k = r.normal(size=(hkv, n_c + c, d)) * 3
    v = r.normal(size=(hkv, n_c + c, d))
    qi = r.normal(size=(hq, n_i, d)) * 3
    _, _, probs = orc.chunk_attn(q, k, v, n_c)
    np.testing.assert_allclose(probs.sum(axis=-1), 1.0, atol=1e-12)
    # masked entries are exactly zero
    for t in range(c):
        assert np.all(probs[:, t, n_c + t + 1:] == 0.0)
    g_size = hq // hkv
    np.testing.assert_allclose(orc.instr_score(qi, k).sum(axis=1), n_i * g_size, atol=1e-11)
    np.testing.assert_allclose(orc.lm_score(q, k, n_c).sum(axis=1), c * g_size, atol=1e-11)


def test_zero_instruction_queries_give_uniform_scores():
    r = rng(3)
    k = r.normal(size=(2, 37, 8))
    s = orc.instr_score(np.zeros((4, 6, 8)), k)
    np.testing.assert_allclose(s, 6 * 2 / 37.0, atol=1e-13)


def test_identical_keys_give_equal_scores_and_lowest_indices():
    r = rng(4)
    key = r.normal(size=(8,))
    k = np.broadcast_to(key, (2, 50, 8)).copy()
    qi = r.normal(size=(4, 6, 8))
    s = orc.instr_score(qi, k)
    np.testing.assert_allclose(s, 6 * 2 / 50.0, atol=1e-13)
    # all-equal scores (exactly equal by construction here): lowest indices win
    np.testing.assert_array_equal(orc.topk_select(np.full((2, 50), 0.24), 7), np.tile(np.arange(7), (2, 1)))


def test_dominant_key_takes_all_mass():
    r = rng(6)
    d = 8
    k = r.normal(size=(1, 20, d)) * 0.01
    k[0, 13] = 100.0
    qi = np.abs(r.normal(size=(2, 4, d))) + 0.5
    s = orc.instr_score(qi, k)
    assert abs(s[0, 13] - 8.0) < 1e-9 and s[0].sum() == pytest.approx(8.0)


def test_instr_score_permutation_equivariance_and_head_grouping():
    r = rng(8)
    hq, hkv, n, d = 6, 3, 29, 8
    k = r.normal(size=(hkv, n, d))
    qi = r.normal(size=(hq, 4, d))
    perm = r.permutation(n)
    np.testing.assert_allclose(orc.instr_score(qi, k[:, perm]), orc.instr_score(qi, k)[:, perm], atol=1e-13)
    # contiguous grouping: zeroing heads 0,1 (group 0) makes only KV head 0 uniform
    qz = qi.copy()
    qz[0:2] = 0.0
    s = orc.instr_score(qz, k)
    np.testing.assert_allclose(s[0], 4 * 2 / n, atol=1e-13)
    assert np.std(s[1]) > 1e-3 and np.std(s[2]) > 1e-3


def test_tova_special_case_single_token_chunk():
    """A chunk of one token with one query head per KV head: the chunk score
    is that token's attention row (TOVA as CSE with l_s = 1, Section 5.2)."""
    r = rng(9)
    d, n_c = 16, 30
    q = r.normal(size=(2, 1, d))
    k = r.normal(size=(2, n_c + 1, d))
    s = orc.lm_score(q, k, n_c)
    for h in range(2):
        row = torch.softmax(torch.from_numpy(q[h, 0] @ k[h].T / math.sqrt(d)), dim=0).numpy()
        np.testing.assert_allclose(s[h], row, atol=1e-13)


def test_custom_scale_is_used():
    r = rng(10)
    q = r.normal(size=(1, 2, 4)); k = r.normal(size=(1, 5, 4)); v = r.normal(size=(1, 5, 4))
    o1, _, _ = orc.chunk_attn(q, k, v, 3, scale=0.5)      # 1/sqrt(4)
    o2, _, _ = orc.chunk_attn(q, k, v, 3)
    o3, _, _ = orc.chunk_attn(q, k, v, 3, scale=0.25)
    np.testing.assert_allclose(o1, o2, atol=1e-15)
    assert np.max(np.abs(o1 - o3)) > 1e-3


# ----------------------------------------------------------------------------
# library special case: torch's CPU attention
# ----------------------------------------------------------------------------

def _sdpa(q, k, v, mask=None, causal=False, group=1):
    tq = torch.from_numpy(q)[None]
    tk = torch.from_numpy(np.repeat(k, group, axis=0))[None]
    tv = torch.from_numpy(np.repeat(v, group, axis=0))[None]
    m = None if mask is None else torch.from_numpy(mask)
    return torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=m, is_causal=causal)[0].numpy()


def _doc(seed, hq, hkv, t, d, n_i, chunk):
    r = rng(seed)
    n_chunks = (t + chunk - 1) // chunk
    return (r.normal(size=(hq, t, d)), r.normal(size=(hkv, t, d)), r.normal(size=(hkv, t, d)),
            [r.normal(size=(hq, n_i, d)) for _ in range(n_chunks)])


def test_chunk_attn_vs_torch_sdpa():
    hq, hkv, t, d = 4, 2, 24, 8
    q, k, v, _ = _doc(21, hq, hkv, t, d, 2, 8)
    np.testing.assert_allclose(orc.full_causal_attention(q, k, v), _sdpa(q, k, v, causal=True, group=2), atol=1e-12)


@pytest.mark.parametrize("mode", [orc.CACHE_INSTR, orc.CACHE_SHARED, orc.CACHE_DUAL])
def test_budget_at_least_document_is_full_attention(mode):
    hq, hkv, t, d, chunk = 4, 2, 45, 8, 8          # ragged last chunk of 5
    q, k, v, qi = _doc(22, hq, hkv, t, d, 3, chunk)
    res = orc.process_document(q, k, v, qi, chunk, budget=64, cache_mode=mode, budget_lm=64)
    out = np.concatenate([tr.out for tr in res.trace], axis=1)
    np.testing.assert_allclose(out, _sdpa(q, k, v, causal=True, group=2), atol=1e-12)
    assert res.k_cache.shape[1] == t
    np.testing.assert_array_equal(res.positions, np.tile(np.arange(t), (hkv, 1)))
    np.testing.assert_array_equal(res.k_cache, k)


def test_sliding_window_replay_matches_banded_attention():
    """Forcing 'keep the most recent k candidates' turns the loop into
    sliding-window attention, which torch computes with a band mask: pins the
    cache/chunk concatenation, n_c bookkeeping and the gather."""
    hq, hkv, t, d, chunk, budget = 2, 1, 40, 8, 6, 9
    q, k, v, qi = _doc(23, hq, hkv, t, d, 2, chunk)
    n_chunks = (t + chunk - 1) // chunk
    forced, n_c = [], 0
    for i in range(n_chunks):
        c = min(chunk, t - i * chunk)
        n = n_c + c
        keep = min(budget, n)
        forced.append(np.arange(n - keep, n)[None, :])
        n_c = keep
    res = orc.process_document(q, k, v, qi, chunk, budget, forced_idx=forced)
    out = np.concatenate([tr.out for tr in res.trace], axis=1)
    # row t (chunk i starting at lo) sees positions max(0, lo - budget) .. t
    mask = np.zeros((t, t), dtype=bool)
    for row in range(t):
        lo = (row // chunk) * chunk
        mask[row, max(0, lo - budget):row + 1] = True
    np.testing.assert_allclose(out, _sdpa(q, k, v, mask=mask, group=2), atol=1e-12)
    np.testing.assert_array_equal(res.positions[0], np.arange(t - budget, t))
    np.testing.assert_array_equal(res.v_cache[0], v[0, t - budget:])


def test_process_document_invariants_and_cache_contents():
    hq, hkv, t, d, chunk, budget = 4, 2, 70, 8, 16, 24
    q, k, v, qi = _doc(24, hq, hkv, t, d, 3, chunk)
    res = orc.process_document(q, k, v, qi, chunk, budget)
    tokens = 0
    for i, tr in enumerate(res.trace):
        assert tr.n_c == min(budget, tokens)
        c = min(chunk, t - i * chunk)
        tokens += c
        assert tr.idx.shape == (hkv, min(budget, tr.n_c + c))
        assert np.all(np.diff(tr.idx, axis=1) > 0)
        np.testing.assert_allclose(tr.score.sum(axis=1), 3 * 2, atol=1e-11)
    assert res.positions.shape == (hkv, budget)
    assert np.all(np.diff(res.positions, axis=1) > 0)
    for g in range(hkv):
        np.testing.assert_array_equal(res.k_cache[g], k[g, res.positions[g]])
        np.testing.assert_array_equal(res.v_cache[g], v[g, res.positions[g]])
    # the two single-cache modes are the same computation
    res2 = orc.process_document(q, k, v, qi, chunk, budget, cache_mode=orc.CACHE_SHARED)
    np.testing.assert_array_equal(res.positions, res2.positions)
    # layer-wise selection: every KV head keeps the same positions
    res3 = orc.process_document(q, k, v, qi, chunk, budget, select_mode=orc.SELECT_PER_LAYER)
    np.testing.assert_array_equal(res3.positions[0], res3.positions[1])
    assert res3.trace[-1].idx.shape[0] == 1


def test_dual_mode_threads_are_separate():
    """Chunk attention reads the LM cache, the instruction score reads the
    instruction cache: force the LM cache to a sliding window and the
    instruction cache to 'oldest positions' and check each against torch."""
    hq, hkv, t, d, chunk, budget = 2, 1, 30, 8, 5, 7
    q, k, v, qi = _doc(25, hq, hkv, t, d, 2, chunk)
    n_chunks = t // chunk
    f_lm, f_in, n_c = [], [], 0
    for i in range(n_chunks):
        n = n_c + chunk
        keep = min(budget, n)
        f_lm.append(np.arange(n - keep, n)[None, :])
        f_in.append(np.arange(keep)[None, :])
        n_c = keep
    res = orc.process_document(q, k, v, qi, chunk, budget, cache_mode=orc.CACHE_DUAL, budget_lm=budget,
                               forced_idx=f_in, forced_idx_lm=f_lm)
    out = np.concatenate([tr.out for tr in res.trace], axis=1)
    mask = np.zeros((t, t), dtype=bool)
    for row in range(t):
        lo = (row // chunk) * chunk
        mask[row, max(0, lo - budget):row + 1] = True
    np.testing.assert_allclose(out, _sdpa(q, k, v, mask=mask, group=2), atol=1e-12)
    np.testing.assert_array_equal(res.positions[0], np.arange(budget))
    np.testing.assert_array_equal(res.positions_lm[0], np.arange(t - budget, t))
    # last step's instruction score: softmax over [positions 0..6 ; last chunk]
    cand = np.concatenate([np.arange(budget), np.arange(t - chunk, t)])
    logits = torch.from_numpy(qi[n_chunks - 1] @ k[0, cand].T / math.sqrt(d))
    expect = torch.softmax(logits, dim=-1).sum(dim=(0, 1)).numpy()
    np.testing.assert_allclose(res.trace[-1].score[0], expect, atol=1e-12)
    # LM score of the last step sums the causal probabilities over [window ; chunk]
    np.testing.assert_allclose(res.trace[-1].score_lm.sum(), chunk * hq, atol=1e-11)


def test_kv_compact_is_a_bit_copy_and_broadcasts():
    r = rng(30)
    k = r.normal(size=(3, 10, 4)).astype(np.float32)
    v = r.normal(size=(3, 10, 4)).astype(np.float32)
    idx = np.array([[1, 4, 9]])
    kn, vn = orc.kv_compact(k, v, idx)
    assert kn.dtype == np.float32
    for g in range(3):
        np.testing.assert_array_equal(kn[g], k[g, [1, 4, 9]])
        np.testing.assert_array_equal(vn[g], v[g, [1, 4, 9]])
    kn, _ = orc.kv_compact(k, v, np.tile(np.arange(10), (3, 1)))
    np.testing.assert_array_equal(kn, k)


# ----------------------------------------------------------------------------
# the language-modelling cache in the order Section 4.1 prints (evict, then append)
# ----------------------------------------------------------------------------

def _importance_by_hand(q_rows, k, cache):
    """Eq. (1) with plain loops for one head: mean over the text's tokens of the softmax over the cache alone."""
    d = k.shape[1]
    imp = [0.0] * len(cache)
    for qt in q_rows:
        logit = [sum(qt[x] * k[j][x] for x in range(d)) / math.sqrt(d) for j in cache]
        mx = max(logit)
        w = [math.exp(a - mx) for a in logit]
        z = sum(w)
        for a in range(len(cache)):
            imp[a] += w[a] / z / len(q_rows)
    return imp


def _standard_cse_by_hand(q, k, v, chunk, budget, q_final=None):
    """Standard chunked state eviction for ONE head, written with plain loops from the three steps of
    Section 4.1: encode the chunk given the cache; evict the cache by Eq. (1) (s = chunk, normalised over
    the cache states); put the chunk into the cache.  With ``q_final`` (the instruction's queries) the cache
    is evicted once more by the instruction when the document has ended.
    Returns (outputs [T, d], final cache positions)."""
    t_total, d = q.shape
    cache = []                                   # document positions, in order
    outs = np.zeros((t_total, v.shape[1]))
    for lo in range(0, t_total, chunk):
        hi = min(t_total, lo + chunk)
        # step 1: token t attends to the cache and to the chunk tokens up to itself
        for t in range(lo, hi):
            cand = cache + list(range(lo, t + 1))
            logit = [sum(q[t][x] * k[j][x] for x in range(d)) / math.sqrt(d) for j in cand]
            mx = max(logit)
            w = [math.exp(a - mx) for a in logit]
            z = sum(w)
            for x in range(v.shape[1]):
                outs[t][x] = sum(w[a] * v[cand[a]][x] for a in range(len(cand))) / z
        # step 2: importance of every cache state = mean over chunk tokens of the softmax over the cache alone
        if len(cache) > budget:
            imp = [0.0] * len(cache)
            for t in range(lo, hi):
                logit = [sum(q[t][x] * k[j][x] for x in range(d)) / math.sqrt(d) for j in cache]
                mx = max(logit)
                w = [math.exp(a - mx) for a in logit]
                z = sum(w)
                for a in range(len(cache)):
                    imp[a] += w[a] / z / (hi - lo)
            order = sorted(range(len(cache)), key=lambda a: (-imp[a], a))[:budget]
            cache = [cache[a] for a in sorted(order)]
        # step 3
        cache = cache + list(range(lo, hi))
    if q_final is not None and len(cache) > budget:
        imp = _importance_by_hand(q_final, k, cache)
        order = sorted(range(len(cache)), key=lambda a: (-imp[a], a))[:budget]
        cache = [cache[a] for a in sorted(order)]
    return outs, cache


def test_lm_evict_then_append_vs_hand_written_standard_cse():
    hq, hkv, t, d, chunk, budget = 1, 1, 37, 4, 5, 7
    q, k, v, qi = _doc(131, hq, hkv, t, d, 2, chunk)
    res = orc.process_document(q, k, v, qi, chunk, budget=6, cache_mode=orc.CACHE_DUAL, budget_lm=budget,
                               lm_ordering=orc.LM_EVICT_THEN_APPEND)
    outs, cache = _standard_cse_by_hand(q[0], k[0], v[0], chunk, budget)
    np.testing.assert_allclose(np.concatenate([tr.out for tr in res.trace], axis=1)[0], outs, atol=1e-12)
    assert res.positions_lm[0].tolist() == cache
    np.testing.assert_array_equal(res.k_cache_lm[0], k[0][cache])


def test_lm_evict_then_append_invariants():
    hq, hkv, t, d, chunk, budget, budget_lm = 4, 2, 75, 8, 16, 20, 24
    q, k, v, qi = _doc(132, hq, hkv, t, d, 3, chunk)
    res = orc.process_document(q, k, v, qi, chunk, budget, cache_mode=orc.CACHE_DUAL, budget_lm=budget_lm,
                               lm_ordering=orc.LM_EVICT_THEN_APPEND)
    ref = orc.process_document(q, k, v, qi, chunk, budget, cache_mode=orc.CACHE_DUAL, budget_lm=budget_lm)
    held = 0
    for i, tr in enumerate(res.trace):
        c = min(chunk, t - i * chunk)
        assert tr.n_c_lm == held                       # the cache still holds the whole previous chunk
        assert tr.score_lm.shape == (hkv, held)        # only cache states are scored
        if held:
            np.testing.assert_allclose(tr.score_lm.sum(axis=1), c * 2, atol=1e-10)   # each row's softmax over the cache sums to 1
        assert tr.idx_lm.shape[1] == min(held, budget_lm)
        held = min(held, budget_lm) + c
        # the instruction cache does not depend on the ordering of the other cache
        np.testing.assert_array_equal(tr.idx, ref.trace[i].idx)
    assert res.positions_lm.shape == (hkv, held)
    last = t - (t - 1) // chunk * chunk
    np.testing.assert_array_equal(res.positions_lm[:, -last:], np.tile(np.arange(t - last, t), (hkv, 1)))
    assert np.all(np.diff(res.positions_lm, axis=1) > 0)
    np.testing.assert_array_equal(res.positions, ref.positions)


def test_lm_evict_then_append_with_large_budget_is_full_attention():
    hq, hkv, t, d, chunk = 4, 2, 45, 8, 8
    q, k, v, qi = _doc(133, hq, hkv, t, d, 3, chunk)
    res = orc.process_document(q, k, v, qi, chunk, budget=64, cache_mode=orc.CACHE_DUAL, budget_lm=64,
                               lm_ordering=orc.LM_EVICT_THEN_APPEND)
    out = np.concatenate([tr.out for tr in res.trace], axis=1)
    np.testing.assert_allclose(out, _sdpa(q, k, v, causal=True, group=2), atol=1e-12)
    np.testing.assert_array_equal(res.k_cache_lm, k)


# ----------------------------------------------------------------------------
# Standard CSE on its own, and the extra eviction by the instruction at the end
# ----------------------------------------------------------------------------

def test_standard_cse_vs_hand_written_loop_with_final_instruction_eviction():
    hq, hkv, t, d, chunk, budget = 1, 1, 43, 4, 6, 8
    q, k, v, qi = _doc(141, hq, hkv, t, d, 3, chunk)
    res = orc.standard_cse(q, k, v, chunk, budget, q_instr_final=qi[-1])
    outs, cache_before = _standard_cse_by_hand(q[0], k[0], v[0], chunk, budget)
    _, cache_after = _standard_cse_by_hand(q[0], k[0], v[0], chunk, budget, q_final=qi[-1][0])
    np.testing.assert_allclose(res.out[0], outs, atol=1e-12)
    assert res.positions[0].tolist() == cache_before
    assert res.positions_final[0].tolist() == cache_after and len(cache_after) == budget
    np.testing.assert_array_equal(res.k_final[0], k[0][cache_after])
    np.testing.assert_array_equal(res.v_final[0], v[0][cache_after])
    # the hand-written importance is the mean, the oracle's score the sum over the text's tokens
    imp = _importance_by_hand(qi[-1][0], k[0], cache_before)
    np.testing.assert_allclose(res.score_final[0] / qi[-1].shape[1], imp, atol=1e-12)


def _append_then_evict_by_hand(q, k, chunk, budget):
    """The other ordering for ONE head with plain loops: the chunk's states are appended, the chunk's own
    causal attention over [cache ; chunk] is summed per state, the best ``budget`` stay."""
    t_total, d = q.shape
    cache = []
    for lo in range(0, t_total, chunk):
        hi = min(t_total, lo + chunk)
        cand = cache + list(range(lo, hi))
        imp = [0.0] * len(cand)
        for t in range(lo, hi):
            seen = len(cache) + (t - lo) + 1
            logit = [sum(q[t][x] * k[j][x] for x in range(d)) / math.sqrt(d) for j in cand[:seen]]
            mx = max(logit)
            w = [math.exp(a - mx) for a in logit]
            z = sum(w)
            for a in range(seen):
                imp[a] += w[a] / z
        order = sorted(range(len(cand)), key=lambda a: (-imp[a], a))[:budget]
        cache = [cand[a] for a in sorted(order)]
    return cache


def test_standard_cse_score_after_append_vs_hand_written_loop_and_dual_lm_thread():
    hq, hkv, t, d, chunk, budget = 1, 1, 41, 4, 7, 9
    q, k, v, qi = _doc(142, hq, hkv, t, d, 2, chunk)
    res = orc.standard_cse(q, k, v, chunk, budget, lm_ordering=orc.LM_SCORE_AFTER_APPEND)
    assert res.positions[0].tolist() == _append_then_evict_by_hand(q[0], k[0], chunk, budget)
    # several heads: the language-modelling thread of the dual design is the same process
    hq, hkv = 4, 2
    q, k, v, qi = _doc(143, hq, hkv, t, d, 2, chunk)
    for ordering in (orc.LM_SCORE_AFTER_APPEND, orc.LM_EVICT_THEN_APPEND):
        for mode in (orc.SELECT_PER_KV_HEAD, orc.SELECT_PER_LAYER):
            alone = orc.standard_cse(q, k, v, chunk, budget, lm_ordering=ordering, select_mode=mode, start_size=2)
            dual = orc.process_document(q, k, v, qi, chunk, budget=5, cache_mode=orc.CACHE_DUAL, budget_lm=budget,
                                        select_mode=mode, start_size=2, lm_ordering=ordering)
            np.testing.assert_array_equal(alone.positions, dual.positions_lm)
            np.testing.assert_allclose(alone.out, np.concatenate([tr.out for tr in dual.trace], axis=1), atol=1e-12)


def test_evict_cache_one_token_one_head_keeps_the_largest_dot_products():
    """A text of one token and one head: softmax is monotone, so the kept states are those with the k largest
    q.k, whatever the normalisation; a transposed operand or a wrong sign would choose others."""
    rng = np.random.default_rng(144)
    n, d, keep = 23, 6, 5
    qt, kc, vc = rng.standard_normal((1, 1, d)), rng.standard_normal((1, n, d)), rng.standard_normal((1, n, d))
    k_new, v_new, idx, score = orc.evict_cache(qt, kc, vc, keep)
    dots = [float(sum(qt[0, 0, x] * kc[0, j, x] for x in range(d))) for j in range(n)]
    want = sorted(sorted(range(n), key=lambda j: -dots[j])[:keep])
    assert idx[0].tolist() == want
    np.testing.assert_array_equal(k_new[0], kc[0][want])
    np.testing.assert_array_equal(v_new[0], vc[0][want])
    np.testing.assert_allclose(score.sum(), 1.0, atol=1e-12)


def test_evict_cache_invariants_and_small_cache():
    rng = np.random.default_rng(145)
    hq, hkv, n, d, rows = 4, 2, 30, 8, 5
    qt, kc, vc = rng.standard_normal((hq, rows, d)), rng.standard_normal((hkv, n, d)), rng.standard_normal((hkv, n, d))
    k_new, v_new, idx, score = orc.evict_cache(qt, kc, vc, 12, start_size=3)
    np.testing.assert_allclose(score.sum(axis=1), rows * (hq // hkv), atol=1e-10)
    assert idx.shape == (hkv, 12) and np.all(np.diff(idx, axis=1) > 0) and np.all(idx[:, :3] == np.arange(3))
    for g in range(hkv):
        np.testing.assert_array_equal(k_new[g], kc[g][idx[g]])
    # a cache that fits the budget stays whole
    k_all, v_all, idx_all, _ = orc.evict_cache(qt, kc, vc, 64)
    np.testing.assert_array_equal(k_all, kc)
    np.testing.assert_array_equal(idx_all, np.tile(np.arange(n), (hkv, 1)))


# ----------------------------------------------------------------------------
# one decoding step over the retained cache
# ----------------------------------------------------------------------------

def test_decode_step_vs_torch_sdpa_and_token_by_token_equals_causal_attention():
    hq, hkv, n, d = 4, 2, 19, 8
    r = rng(151)
    q, kn, vn = r.normal(size=(hq, d)), r.normal(size=(hkv, d)), r.normal(size=(hkv, d))
    kc, vc = r.normal(size=(hkv, n, d)), r.normal(size=(hkv, n, d))
    out, k2, v2 = orc.decode_step(q, kn, vn, kc, vc)
    np.testing.assert_array_equal(k2[:, :n], kc)
    np.testing.assert_array_equal(k2[:, n], kn)
    np.testing.assert_array_equal(v2[:, n], vn)
    np.testing.assert_allclose(out, _sdpa(q[:, None, :], k2, v2, group=2)[:, 0], atol=1e-12)
    # generating a sequence token by token from an empty cache is causal attention over it
    t = 11
    qs, ks, vs = r.normal(size=(hq, t, d)), r.normal(size=(hkv, t, d)), r.normal(size=(hkv, t, d))
    kc, vc = np.zeros((hkv, 0, d)), np.zeros((hkv, 0, d))
    rows = []
    for i in range(t):
        o, kc, vc = orc.decode_step(qs[:, i], ks[:, i], vs[:, i], kc, vc)
        rows.append(o)
    np.testing.assert_allclose(np.stack(rows, axis=1), _sdpa(qs, ks, vs, causal=True, group=2), atol=1e-12)


def test_decode_step_closed_forms():
    hq, hkv, n, d = 2, 1, 6, 4
    r = rng(152)
    vc, vn = r.normal(size=(hkv, n, d)), r.normal(size=(hkv, d))
    # a zero query weighs all n + 1 states equally: the output is the mean of their values
    out, _, v2 = orc.decode_step(np.zeros((hq, d)), r.normal(size=(hkv, d)), vn, r.normal(size=(hkv, n, d)), vc)
    np.testing.assert_allclose(out, np.tile(v2[0].mean(axis=0), (hq, 1)), atol=1e-12)
    # a key that dominates takes all the weight, the token's own key included
    q = np.zeros((hq, d)); q[:, 0] = 50.0
    kc = np.zeros((hkv, n, d)); kc[0, 3, 0] = 40.0
    out, _, _ = orc.decode_step(q, np.zeros((hkv, d)), vn, kc, vc)
    np.testing.assert_allclose(out, np.tile(vc[0, 3], (hq, 1)), atol=1e-9)
    kn = np.zeros((hkv, d)); kn[0, 0] = 80.0
    out, _, _ = orc.decode_step(q, kn, vn, kc, vc)
    np.testing.assert_allclose(out, np.tile(vn[0], (hq, 1)), atol=1e-9)
    # custom scale: doubling the scale equals doubling the query
    a, _, _ = orc.decode_step(r.normal(size=(hq, d)) * 0 + 1.0, kn * 0.01, vn, kc * 0.01, vc, scale=0.6)
    b, _, _ = orc.decode_step(np.full((hq, d), 2.0), kn * 0.01, vn, kc * 0.01, vc, scale=0.3)
    np.testing.assert_allclose(a, b, atol=1e-12)


# ----------------------------------------------------------------------------
# accumulated scores (the H2O rule on the instruction-aware cache)
# ----------------------------------------------------------------------------

def _accumulated_by_hand(k, q_instr, chunk, budget):
    """ONE head, plain loops: every state carries the sum of the instruction-attention mass it has received
    in the steps since it entered the cache; after each step the ``budget`` largest sums stay."""
    t_total, d = k.shape
    cache, total = [], {}
    step = 0
    for lo in range(0, t_total, chunk):
        hi = min(t_total, lo + chunk)
        cand = cache + list(range(lo, hi))
        for qt in q_instr[step]:
            logit = [sum(qt[x] * k[j][x] for x in range(d)) / math.sqrt(d) for j in cand]
            mx = max(logit)
            w = [math.exp(a - mx) for a in logit]
            z = sum(w)
            for a, j in enumerate(cand):
                total[j] = total.get(j, 0.0) + w[a] / z
        keep = sorted(sorted(cand, key=lambda j: (-total[j], j))[:budget])
        total = {j: total[j] for j in keep}     # an evicted state and its sum are gone for good
        cache = keep
        step += 1
    return cache, total


def test_accumulated_scores_vs_hand_written_loop():
    hq, hkv, t, d, chunk, budget = 1, 1, 47, 4, 6, 9
    q, k, v, qi = _doc(161, hq, hkv, t, d, 3, chunk)
    res = orc.process_document(q, k, v, qi, chunk, budget, score_mode=orc.SCORE_ACCUMULATED)
    cache, total = _accumulated_by_hand(k[0], [x[0] for x in qi], chunk, budget)
    assert res.positions[0].tolist() == cache
    np.testing.assert_allclose(res.acc_score[0], [total[j] for j in cache], atol=1e-12)
    # the rule matters: the plain per-step rule keeps a different set on this document
    plain = orc.process_document(q, k, v, qi, chunk, budget)
    assert plain.positions[0].tolist() != cache


def test_accumulated_scores_invariants():
    hq, hkv, t, d, chunk, budget = 4, 2, 60, 8, 8, 12
    q, k, v, qi = _doc(162, hq, hkv, t, d, 3, chunk)
    for mode in (orc.SELECT_PER_KV_HEAD, orc.SELECT_PER_LAYER):
        res = orc.process_document(q, k, v, qi, chunk, budget, select_mode=mode, score_mode=orc.SCORE_ACCUMULATED,
                                   start_size=2)
        plain = orc.process_document(q, k, v, qi, chunk, budget, select_mode=mode, start_size=2)
        # the first step has nothing to add to: same selection; outputs of step 0 and 1 are those of the plain rule
        np.testing.assert_array_equal(res.trace[0].idx, plain.trace[0].idx)
        np.testing.assert_allclose(res.trace[1].out, plain.trace[1].out, atol=1e-12)
        # a kept state's sum is at least its latest score, and the sums of a step add up to the mass received
        # by the kept states over their life time, which is at most steps * rows * heads per KV head
        assert res.acc_score.shape == (hkv, budget) and np.all(res.acc_score > 0)
        assert np.all(res.acc_score.sum(axis=1) <= len(res.trace) * 3 * 2 + 1e-9)
        assert np.all(np.diff(res.positions, axis=1) > 0) and np.all(res.positions[:, :2] == np.arange(2))
    # a budget that holds the whole document never evicts: the cache is the document, the sums are the
    # column sums over all steps a state has seen
    res = orc.process_document(q, k, v, qi, chunk, budget=64, score_mode=orc.SCORE_ACCUMULATED)
    np.testing.assert_array_equal(res.k_cache, k)
    want = np.zeros((hkv, t))
    for i, tr in enumerate(res.trace):
        n = min(t, (i + 1) * chunk)
        want[:, :n] += orc.instr_score(qi[i], k[:, :n])
    np.testing.assert_allclose(res.acc_score, want, atol=1e-10)


# ----------------------------------------------------------------------------
# rotary embedding at cache positions (position shift)
# ----------------------------------------------------------------------------

def test_rope_worked_examples_and_properties():
    # d = 2: one pair, frequency 1: a plane rotation by `position` radians
    x = np.array([[[1.0, 0.0], [0.0, 2.0], [3.0, 4.0]]])
    y = orc.rope(x, [0, math.pi / 2, 1.0])
    np.testing.assert_allclose(y[0, 0], [1.0, 0.0], atol=1e-15)                     # position 0: untouched
    np.testing.assert_allclose(y[0, 1], [-2.0, 0.0], atol=1e-12)                    # quarter turn of (0, 2)
    np.testing.assert_allclose(y[0, 2], [3 * math.cos(1) - 4 * math.sin(1), 4 * math.cos(1) + 3 * math.sin(1)], atol=1e-12)
    # d = 4, base 100: pairs (0, 2) and (1, 3) with frequencies 1 and 100^(-1/2) = 0.1
    x = np.array([[[1.0, 1.0, 0.0, 0.0]]])
    y = orc.rope(x, [5], base=100.0)
    np.testing.assert_allclose(y[0, 0], [math.cos(5), math.cos(0.5), math.sin(5), math.sin(0.5)], atol=1e-12)
    # norms are kept, and q.k depends on the distance of the two positions only
    r = rng(171)
    q, k = r.normal(size=(2, 7, 16)), r.normal(size=(2, 7, 16))
    pos = np.array([0, 3, 4, 10, 11, 50, 700])
    np.testing.assert_allclose(np.linalg.norm(orc.rope(q, pos), axis=-1), np.linalg.norm(q, axis=-1), atol=1e-12)
    a = np.einsum("hsd,htd->hst", orc.rope(q, pos), orc.rope(k, pos))
    b = np.einsum("hsd,htd->hst", orc.rope(q, pos + 123), orc.rope(k, pos + 123))
    np.testing.assert_allclose(a, b, atol=1e-10)
    # the same rotation written the way the model code writes it (cos/sin tables and a rotate-half), in torch
    t = torch.from_numpy(q)
    inv = 1.0 / (10000.0 ** (torch.arange(0, 16, 2, dtype=torch.float64) / 16))
    ang = torch.from_numpy(pos.astype(np.float64))[:, None] * inv[None, :]
    emb = torch.cat([ang, ang], dim=-1)
    rot = torch.cat([-t[..., 8:], t[..., :8]], dim=-1)
    np.testing.assert_allclose(orc.rope(q, pos), (t * emb.cos() + rot * emb.sin()).numpy(), atol=1e-12)


def _rot_by_hand(x, pos, base):
    d = len(x)
    y = [0.0] * d
    for i in range(d // 2):
        a = pos * base ** (-2.0 * i / d)
        y[i] = x[i] * math.cos(a) - x[i + d // 2] * math.sin(a)
        y[i + d // 2] = x[i + d // 2] * math.cos(a) + x[i] * math.sin(a)
    return y


def _position_shift_by_hand(q, k, v, q_instr, chunk, budget, base):
    """ONE head, plain loops: the cache holds unrotated keys; whenever a candidate is attended to it is rotated
    to its place in [cache ; chunk], a chunk token to the place of its own state, an instruction token to the
    places behind all candidates.  Returns (outputs, final cache positions)."""
    t_total, d = q.shape
    cache, outs, step = [], np.zeros((t_total, v.shape[1])), 0
    for lo in range(0, t_total, chunk):
        hi = min(t_total, lo + chunk)
        cand = cache + list(range(lo, hi))
        krot = [_rot_by_hand(k[j], slot, base) for slot, j in enumerate(cand)]
        for t in range(lo, hi):
            seen = len(cache) + (t - lo) + 1
            qr = _rot_by_hand(q[t], len(cache) + (t - lo), base)
            logit = [sum(qr[x] * krot[a][x] for x in range(d)) / math.sqrt(d) for a in range(seen)]
            mx = max(logit)
            w = [math.exp(a - mx) for a in logit]
            z = sum(w)
            for x in range(v.shape[1]):
                outs[t][x] = sum(w[a] * v[cand[a]][x] for a in range(seen)) / z
        imp = [0.0] * len(cand)
        for u, qt in enumerate(q_instr[step]):
            qr = _rot_by_hand(qt, len(cand) + u, base)
            logit = [sum(qr[x] * krot[a][x] for x in range(d)) / math.sqrt(d) for a in range(len(cand))]
            mx = max(logit)
            w = [math.exp(a - mx) for a in logit]
            z = sum(w)
            for a in range(len(cand)):
                imp[a] += w[a] / z
        keep = sorted(sorted(range(len(cand)), key=lambda a: (-imp[a], a))[:budget])
        cache = [cand[a] for a in keep]
        step += 1
    return outs, cache


def test_position_shift_vs_hand_written_loop():
    hq, hkv, t, d, chunk, budget = 1, 1, 33, 4, 5, 8
    q, k, v, qi = _doc(172, hq, hkv, t, d, 3, chunk)
    res = orc.process_document(q, k, v, qi, chunk, budget, position_shift=True, rope_base=50.0)
    outs, cache = _position_shift_by_hand(q[0], k[0], v[0], [x[0] for x in qi], chunk, budget, 50.0)
    np.testing.assert_allclose(np.concatenate([tr.out for tr in res.trace], axis=1)[0], outs, atol=1e-12)
    assert res.positions[0].tolist() == cache
    np.testing.assert_array_equal(res.k_cache[0], k[0][cache])       # the cache keeps the unrotated keys
    # positions matter: without the shift the same tensors give another result
    plain = orc.process_document(q, k, v, qi, chunk, budget)
    assert not np.allclose(np.concatenate([tr.out for tr in plain.trace], axis=1)[0], outs)


def test_position_shift_without_eviction_is_rope_at_document_positions():
    hq, hkv, t, d, chunk = 4, 2, 29, 8, 6
    q, k, v, qi = _doc(173, hq, hkv, t, d, 2, chunk)
    res = orc.process_document(q, k, v, qi, chunk, budget=64, position_shift=True)
    out = np.concatenate([tr.out for tr in res.trace], axis=1)
    pos = np.arange(t)
    np.testing.assert_allclose(out, _sdpa(orc.rope(q, pos), orc.rope(k, pos), v, causal=True, group=2), atol=1e-12)


def _dual_position_shift_by_hand(q, k, v, q_instr, chunk, budget, budget_lm, base, paper_order):
    """ONE head, plain loops, two caches with their own slots (Section 4.2 individual cache with the position
    shift of Section 5.3).  The chunk attends over [LM cache ; chunk] rotated to the LM cache's slots and scores
    it (its own causal column sums, or, in the printed order, Eq. (1) over the cache states alone before the
    chunk is appended); the instruction scores [instruction cache ; chunk] rotated to that cache's slots from
    the places behind its candidates.  Returns (outputs, LM cache positions, instruction cache positions)."""
    t_total, d = q.shape
    lm, ic, outs, step = [], [], np.zeros((t_total, v.shape[1])), 0
    sm = lambda logit: [math.exp(a - max(logit)) / sum(math.exp(b - max(logit)) for b in logit) for a in logit]
    dot = lambda a, b: sum(a[x] * b[x] for x in range(d)) / math.sqrt(d)
    for lo in range(0, t_total, chunk):
        hi = min(t_total, lo + chunk)
        cand = lm + list(range(lo, hi))
        krot = [_rot_by_hand(k[j], slot, base) for slot, j in enumerate(cand)]
        imp_lm = [0.0] * len(cand)
        imp_cache = [0.0] * len(lm)
        for t in range(lo, hi):
            seen = len(lm) + (t - lo) + 1
            qr = _rot_by_hand(q[t], len(lm) + (t - lo), base)
            w = sm([dot(qr, krot[a]) for a in range(seen)])
            for x in range(v.shape[1]):
                outs[t][x] = sum(w[a] * v[cand[a]][x] for a in range(seen))
            for a in range(seen):
                imp_lm[a] += w[a]
            if lm:   # Eq. (1) as printed: softmax over the cache states alone
                wc = sm([dot(qr, krot[a]) for a in range(len(lm))])
                for a in range(len(lm)):
                    imp_cache[a] += wc[a]
        if paper_order:
            keep = sorted(sorted(range(len(lm)), key=lambda a: (-imp_cache[a], a))[:budget_lm])
            lm = [lm[a] for a in keep] + list(range(lo, hi))
        else:
            keep = sorted(sorted(range(len(cand)), key=lambda a: (-imp_lm[a], a))[:budget_lm])
            lm = [cand[a] for a in keep]
        cand_i = ic + list(range(lo, hi))
        krot_i = [_rot_by_hand(k[j], slot, base) for slot, j in enumerate(cand_i)]
        imp = [0.0] * len(cand_i)
        for u, qt in enumerate(q_instr[step]):
            w = sm([dot(_rot_by_hand(qt, len(cand_i) + u, base), krot_i[a]) for a in range(len(cand_i))])
            for a in range(len(cand_i)):
                imp[a] += w[a]
        keep = sorted(sorted(range(len(cand_i)), key=lambda a: (-imp[a], a))[:budget])
        ic = [cand_i[a] for a in keep]
        step += 1
    return outs, lm, ic


@pytest.mark.parametrize("paper_order", [False, True])
def test_dual_position_shift_vs_hand_written_loop(paper_order):
    hq, hkv, t, d, chunk, budget, budget_lm = 1, 1, 31, 4, 5, 7, 6
    q, k, v, qi = _doc(181, hq, hkv, t, d, 3, chunk)
    res = orc.process_document(q, k, v, qi, chunk, budget, cache_mode=orc.CACHE_DUAL, budget_lm=budget_lm,
                               position_shift=True, rope_base=50.0,
                               lm_ordering=orc.LM_EVICT_THEN_APPEND if paper_order else orc.LM_SCORE_AFTER_APPEND)
    outs, lm, ic = _dual_position_shift_by_hand(q[0], k[0], v[0], [x[0] for x in qi], chunk, budget, budget_lm, 50.0,
                                                paper_order)
    np.testing.assert_allclose(np.concatenate([tr.out for tr in res.trace], axis=1)[0], outs, atol=1e-12)
    assert res.positions_lm[0].tolist() == lm and res.positions[0].tolist() == ic
    np.testing.assert_array_equal(res.k_cache_lm[0], k[0][lm])     # both caches keep the unrotated keys
    np.testing.assert_array_equal(res.k_cache[0], k[0][ic])
    # the two caches hold different states at different slots, and the positions matter
    assert lm != ic
    plain = orc.process_document(q, k, v, qi, chunk, budget, cache_mode=orc.CACHE_DUAL, budget_lm=budget_lm,
                                 lm_ordering=orc.LM_EVICT_THEN_APPEND if paper_order else orc.LM_SCORE_AFTER_APPEND)
    assert not np.allclose(np.concatenate([tr.out for tr in plain.trace], axis=1)[0], outs)
