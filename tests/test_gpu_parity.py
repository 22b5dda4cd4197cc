"""Parity of the HIP path (through the C ABI) with the CPU oracle, entry point
by entry point and over whole documents.  Needs an MI355X."""

import numpy as np
import pytest
import torch

import paper_2406_12018_amd as api
from oracle import citrus_oracle as orc
from workloads import WORKLOADS, make_chunk, make_document, peaked, scaled_down
from workloads.synth import Workload

from helpers import TOL, StepwiseRun, assert_close, bits, check_selection, np64

pytestmark = pytest.mark.gpu
DEV = "cuda"


def say(msg):
    print(msg, flush=True)


def rand(shape, dtype, seed, scale=1.0):
    g = torch.Generator(device="cpu").manual_seed(seed)
    return (torch.randn(shape, generator=g, dtype=torch.float32) * scale).to(dtype).to(DEV)


def make_cfg(dtype, B=1, L=2, Hq=4, Hkv=2, d=64, c=32, k=64, n_i=8, **kw):
    return api.Config(batch=B, layers=L, q_heads=Hq, kv_heads=Hkv, head_dim=d, chunk_len=c, budget=k, instr_len=n_i,
                      dtype=api.F32 if dtype == "f32" else api.BF16, **kw)


def tdt(dtype):
    return torch.float32 if dtype == "f32" else torch.bfloat16


# ----------------------------------------------------------------------------
# compaction: bit-exact
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("dtype,d", [("f32", 64), ("bf16", 128), ("bf16", 64), ("f32", 128)])
@pytest.mark.parametrize("per_layer", [False, True])
def test_kv_compact_bit_exact(dtype, d, per_layer):
    B, L, Hkv, n_c, c, m = 2, 3, 2, 37, 21, 29
    cfg = make_cfg(dtype, B=B, L=L, Hkv=Hkv, d=d, c=32, k=64,
                   select_mode=api.SELECT_PER_LAYER if per_layer else api.SELECT_PER_KV_HEAD)
    say(f"compact {dtype} d={d} per_layer={per_layer}")
    # strided sources: cache has capacity 64, chunk is a slice of a longer document tensor
    kc, vc = rand((B, L, Hkv, 64, d), tdt(dtype), 1), rand((B, L, Hkv, 64, d), tdt(dtype), 2)
    kdoc, vdoc = rand((B, L, Hkv, 100, d), tdt(dtype), 3), rand((B, L, Hkv, 100, d), tdt(dtype), 4)
    kch, vch = kdoc[:, :, :, 40:40 + c], vdoc[:, :, :, 40:40 + c]
    hs = 1 if per_layer else Hkv
    r = np.random.default_rng(5)
    idx_np = np.stack([np.sort(r.choice(n_c + c, m, replace=False)) for _ in range(B * L * hs)]).reshape(B, L, hs, m)
    idx = torch.full((B, L, hs, 40), -7, dtype=torch.int32, device=DEV)
    idx[..., :m] = torch.from_numpy(idx_np).to(DEV)
    kn = torch.full((B, L, Hkv, 64, d), 9.0, dtype=tdt(dtype), device=DEV)
    vn = torch.full_like(kn, 9.0)
    api.citrus_kv_compact(cfg, kc, vc, n_c, kch, vch, idx, m, kn, vn)
    torch.cuda.synchronize()
    for b in range(B):
        for l in range(L):
            kcat = np.concatenate([bits(kc[b, l, :, :n_c]), bits(kch[b, l])], axis=1)
            vcat = np.concatenate([bits(vc[b, l, :, :n_c]), bits(vch[b, l])], axis=1)
            k_ref, v_ref = orc.kv_compact(kcat, vcat, idx_np[b, l])
            np.testing.assert_array_equal(bits(kn[b, l, :, :m]), k_ref)
            np.testing.assert_array_equal(bits(vn[b, l, :, :m]), v_ref)
    # rows beyond m are untouched
    assert (kn[:, :, :, m:] == 9.0).all() and (vn[:, :, :, m:] == 9.0).all()


def test_kv_compact_identity():
    cfg = make_cfg("bf16", d=128, c=16, k=64)
    kc, vc = rand((1, 2, 2, 64, 128), torch.bfloat16, 1), rand((1, 2, 2, 64, 128), torch.bfloat16, 2)
    kch, vch = rand((1, 2, 2, 16, 128), torch.bfloat16, 3), rand((1, 2, 2, 16, 128), torch.bfloat16, 4)
    idx = torch.arange(56, dtype=torch.int32, device=DEV).expand(1, 2, 2, 56).contiguous()
    kn, vn = torch.zeros_like(kc), torch.zeros_like(vc)
    api.citrus_kv_compact(cfg, kc, vc, 40, kch, vch, idx, 56, kn, vn)
    assert torch.equal(kn[:, :, :, :40], kc[:, :, :, :40]) and torch.equal(kn[:, :, :, 40:56], kch)
    assert torch.equal(vn[:, :, :, :40], vc[:, :, :, :40]) and torch.equal(vn[:, :, :, 40:56], vch)


# ----------------------------------------------------------------------------
# selection: exact
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("n,k,levels", [(96, 64, None), (1280, 768, None), (1280, 768, 7), (6144, 4096, None),
                                        (2048, 1024, 2), (300, 300, None), (5, 64, None), (1, 1, None),
                                        (1000, 1, None), (1000, 999, 3), (257, 128, None), (40096, 5000, None),
                                        (40096, 40095, 5), (100000, 3, 2),
                                        # both sides of the sizes at which the kernel that keeps a unit's keys in
                                        # registers (8, then 24 per thread) hands over to the next one; few levels:
                                        # the threshold's ties span every 256-candidate row and wave
                                        (2048, 1500, 3), (2049, 1500, 3), (2049, 7, None), (6144, 3000, 2), (6145, 3000, 2),
                                        (6145, 6144, None), (1793, 1792, 4), (255, 3, 2), (513, 512, None)])
@pytest.mark.parametrize("per_layer", [False, True])
def test_topk_select_exact(n, k, levels, per_layer):
    B, L, Hkv = 2, 2, 4
    cfg = make_cfg("f32", B=B, L=L, Hq=4, Hkv=Hkv, k=k,
                   select_mode=api.SELECT_PER_LAYER if per_layer else api.SELECT_PER_KV_HEAD)
    say(f"topk n={n} k={k} levels={levels} per_layer={per_layer}")
    r = np.random.default_rng(n * 7 + k)
    s = r.random((B, L, Hkv, n)).astype(np.float32) if levels is None else \
        (r.integers(0, levels, (B, L, Hkv, n)) * 0.125 - 0.25).astype(np.float32)
    idx = api.citrus_topk_select(cfg, torch.from_numpy(s).to(DEV), k).cpu().numpy()
    m = min(n, k)
    for b in range(B):
        for l in range(L):
            if per_layer:
                layer = s[b, l, 0].copy()
                for g in range(1, Hkv):
                    layer = (layer + s[b, l, g]).astype(np.float32)   # same f32 order as the kernel
                np.testing.assert_array_equal(idx[b, l, 0, :m], orc.topk_select_1d(layer, k))
            else:
                ref = orc.topk_select(s[b, l], k)
                np.testing.assert_array_equal(idx[b, l, :, :m], ref)
    assert (idx[..., m:] == -1).all()


@pytest.mark.parametrize("n,k,start,levels", [(300, 100, 4, None), (1280, 768, 4, None), (97, 5, 5 - 1, 3), (600, 64, 1, 2),
                                              (50, 80, 4, None)])
@pytest.mark.parametrize("per_layer", [False, True])
def test_topk_select_with_start_size_exact(n, k, start, levels, per_layer):
    """The first start_size candidates are always kept, also when their scores are the lowest."""
    B, L, Hkv = 2, 1, 2
    cfg = make_cfg("f32", B=B, L=L, Hq=2, Hkv=Hkv, k=k, start_size=start,
                   select_mode=api.SELECT_PER_LAYER if per_layer else api.SELECT_PER_KV_HEAD)
    say(f"topk start_size n={n} k={k} start={start} levels={levels} per_layer={per_layer}")
    r = np.random.default_rng(n * 13 + k + start)
    s = r.random((B, L, Hkv, n)).astype(np.float32) if levels is None else \
        (r.integers(0, levels, (B, L, Hkv, n)) * 0.125).astype(np.float32)
    s[..., :start] = -5.0  # worst of all: plain selection would drop them
    idx = api.citrus_topk_select(cfg, torch.from_numpy(s).to(DEV), k).cpu().numpy()
    m = min(n, k)
    for b in range(B):
        for l in range(L):
            if per_layer:
                layer = s[b, l, 0].copy()
                for g in range(1, Hkv):
                    layer = (layer + s[b, l, g]).astype(np.float32)
                np.testing.assert_array_equal(idx[b, l, 0, :m], orc.topk_select_1d(layer, k, start))
            else:
                np.testing.assert_array_equal(idx[b, l, :, :m], orc.topk_select(s[b, l], k, start_size=start))
    if n > k:
        assert (idx[..., :start] == np.arange(start)).all()


def test_topk_all_equal_scores_keep_lowest_indices():
    cfg = make_cfg("f32", B=1, L=1, Hq=2, Hkv=2, k=100)
    s = torch.full((1, 1, 2, 333), 0.2, device=DEV)
    idx = api.citrus_topk_select(cfg, s, 100).cpu().numpy()
    np.testing.assert_array_equal(idx[0, 0], np.tile(np.arange(100), (2, 1)))


# ----------------------------------------------------------------------------
# instruction score and chunk attention
# ----------------------------------------------------------------------------

SHAPES = [
    # dtype, B, L, Hq, Hkv, d,  c,  n_c, n_i, qk_scale
    ("f32", 1, 1, 4, 1, 64, 32, 64, 8, 1.0 / 8),
    ("f32", 2, 2, 4, 2, 64, 19, 45, 5, 1.0),
    ("f32", 1, 2, 2, 2, 128, 32, 0, 3, 0.5),
    ("bf16", 1, 2, 8, 2, 128, 96, 160, 24, 0.09),
    ("bf16", 1, 1, 32, 8, 128, 512, 768, 64, 0.09),
    ("bf16", 2, 1, 4, 4, 128, 70, 131, 33, 1.0),
    ("bf16", 1, 1, 16, 2, 128, 130, 0, 64, 1.0),
    ("bf16", 1, 2, 4, 2, 64, 50, 77, 9, 0.5),
    ("bf16", 1, 1, 2, 1, 128, 1, 300, 1, 1.0),
    ("bf16", 1, 2, 8, 2, 128, 45, 83, 37, 0.3),
    ("bf16", 1, 1, 8, 2, 128, 200, 1150, 40, 0.09),
    ("bf16", 1, 2, 8, 2, 128, 300, 1280, 16, 0.09),
    ("bf16", 2, 1, 4, 1, 128, 45, 96, 8, 0.5),
    # chunk and instruction lengths that are multiples of the column-sum kernel's 128-row staging chunk (its
    # pointer-stepping instance), with group sizes 1, 2 and 8, ragged caches, and instruction groups wide enough
    # for the two-launch scorer with several key ranges merged per row
    ("bf16", 1, 2, 8, 1, 128, 128, 333, 128, 0.3),
    ("bf16", 2, 1, 2, 2, 128, 256, 77, 256, 0.5),
    ("bf16", 1, 1, 4, 2, 128, 384, 1500, 384, 0.09),
    # the edges of the single-product scorer's range: 2560 candidates and 512 instruction rows per KV group are
    # the last shapes it takes, one more of either goes to the two-pass kernels; 1280 / 1281 candidates switch
    # its strip height
    ("bf16", 1, 1, 8, 1, 128, 64, 2496, 64, 0.3),
    ("bf16", 1, 1, 8, 1, 128, 64, 2497, 64, 0.3),
    ("bf16", 1, 1, 1, 1, 128, 32, 1000, 513, 0.3),
    ("bf16", 1, 2, 4, 2, 128, 64, 1216, 48, 0.3),
    ("bf16", 1, 2, 4, 2, 128, 64, 1217, 48, 0.3),
    # a cache far longer than any configuration's: 627 key tiles per row block, scores that no longer fit a
    # workgroup's LDS (two-launch scorer with eight key ranges)
    ("bf16", 1, 1, 8, 2, 128, 96, 40000, 24, 0.09),
]


def step_inputs(dtype, B, L, Hq, Hkv, d, c, n_c, n_i, s, seed=0):
    t = tdt(dtype)
    cap = max(n_c, 1) + 3
    return dict(q=rand((B, L, Hq, c, d), t, seed + 1, s), qi=rand((B, L, Hq, n_i, d), t, seed + 2, s),
                kc=rand((B, L, Hkv, cap, d), t, seed + 3, s), vc=rand((B, L, Hkv, cap, d), t, seed + 4),
                k=rand((B, L, Hkv, c, d), t, seed + 5, s), v=rand((B, L, Hkv, c, d), t, seed + 6))


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "-".join(str(x) for x in s[:9]))
def test_instr_score_parity(shape):
    dtype, B, L, Hq, Hkv, d, c, n_c, n_i, s = shape
    say(f"instr_score {shape}")
    x = step_inputs(*shape)
    cfg = make_cfg(dtype, B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, c=c, k=max(n_c, 1) + 3, n_i=n_i)
    ws = api.alloc_workspace(cfg)
    score = api.citrus_instr_score(cfg, x["qi"], x["kc"], n_c, x["k"], workspace=ws)
    torch.cuda.synchronize()
    got = np64(score)
    for b in range(B):
        for l in range(L):
            kcat = np.concatenate([np64(x["kc"][b, l, :, :n_c]), np64(x["k"][b, l])], axis=1)
            ref = orc.instr_score(np64(x["qi"][b, l]), kcat)
            assert_close(got[b, l], ref, dtype, f"score b{b} l{l}")
    # total mass = instruction rows x heads per KV head
    np.testing.assert_allclose(got.sum(-1), n_i * (Hq // Hkv), rtol=2e-3 if dtype == "bf16" else 1e-5)
    # run-to-run bit identical
    again = api.citrus_instr_score(cfg, x["qi"], x["kc"], n_c, x["k"], workspace=ws)
    assert torch.equal(score, again)


# Launches with more (document, layer, KV head) units than the single-product scorer takes: the two-pass kernels,
# which the small shapes above no longer reach.  One case per kernel the launcher can pick, on ragged row and
# candidate counts; three sampled (document, layer) pairs against the oracle, every unit by its mass and by a
# second run.
MANY_UNITS = [
    # B, L, Hq, Hkv, c, n_c, n_i   -> kernel
    (2, 40, 8, 8, 19, 45, 37),       # 37 rows per KV head: four waves, one round
    (2, 40, 32, 8, 33, 700, 50),     # 200 rows, 733 candidates: key tiles stay in registers between the passes
    (2, 40, 32, 8, 77, 1500, 50),    # 200 rows, 1577 candidates: sixteen waves, keys read twice
    (2, 40, 32, 8, 40, 900, 70),     # 280 rows: two launches, key ranges merged per row
    (3, 30, 16, 8, 64, 2497, 64),    # 128 rows, 2561 candidates: one past the single-product scorer's range
]


@pytest.mark.parametrize("shape", MANY_UNITS, ids=lambda s: "-".join(str(x) for x in s))
def test_instr_score_two_pass_kernels(shape):
    B, L, Hq, Hkv, c, n_c, n_i = shape
    say(f"instr_score, many units {shape}")
    d, t, s = 128, torch.bfloat16, 0.3
    cfg = make_cfg("bf16", B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, c=c, k=n_c + 3, n_i=n_i)
    ws = api.alloc_workspace(cfg)
    qi = rand((B, L, Hq, n_i, d), t, 11, s)
    kc, k = rand((B, L, Hkv, n_c + 3, d), t, 12, s), rand((B, L, Hkv, c, d), t, 13, s)
    score = api.citrus_instr_score(cfg, qi, kc, n_c, k, workspace=ws)
    again = api.citrus_instr_score(cfg, qi, kc, n_c, k, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(score, again)
    got = np64(score)
    np.testing.assert_allclose(got.sum(-1), n_i * (Hq // Hkv), rtol=2e-3)
    for b, l in ((0, 0), (B - 1, L // 2), (B // 2, L - 1)):
        kcat = np.concatenate([np64(kc[b, l, :, :n_c]), np64(k[b, l])], axis=1)
        assert_close(got[b, l], orc.instr_score(np64(qi[b, l]), kcat), "bf16", f"score b{b} l{l}")


@pytest.mark.parametrize("shape", [s for s in SHAPES if s[7] > 0], ids=lambda s: "-".join(str(x) for x in s[:9]))
def test_cache_score_parity(shape):
    """Eq. (1) as printed, with the chunk's queries: softmax over the cache states alone, no mask."""
    dtype, B, L, Hq, Hkv, d, c, n_c, n_i, s = shape
    say(f"cache_score {shape}")
    x = step_inputs(*shape, seed=200)
    cfg = make_cfg(dtype, B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, c=c, k=8, n_i=n_i, cache_mode=api.CACHE_DUAL, budget_lm=4,
                   lm_ordering=api.LM_EVICT_THEN_APPEND, cache_capacity=n_c + c + 3)
    ws = api.alloc_workspace(cfg)
    for rows in sorted({c, max(1, c // 3)}):
        score = api.citrus_cache_score(cfg, x["q"], x["kc"], n_c, workspace=ws, rows=rows)
        torch.cuda.synchronize()
        got = np64(score)
        for b in range(B):
            for l in range(L):
                ref = orc.instr_score(np64(x["q"][b, l, :, :rows]), np64(x["kc"][b, l, :, :n_c]))
                assert_close(got[b, l], ref, dtype, f"cache score rows {rows} b{b} l{l}")
        np.testing.assert_allclose(got.sum(-1), rows * (Hq // Hkv), rtol=2e-3 if dtype == "bf16" else 1e-5)
        again = api.citrus_cache_score(cfg, x["q"], x["kc"], n_c, workspace=ws, rows=rows)
        assert torch.equal(score, again)
    # the normaliser over the cache as a by-product of the chunk's attention (aligned caches: the same
    # launch; others: a pass of its own), and the single-pass score that takes it
    lse_c = torch.empty((B, L, Hq, c), dtype=torch.float32, device=DEV)
    kch, vch = rand((B, L, Hkv, c, d), tdt(dtype), 251, s), rand((B, L, Hkv, c, d), tdt(dtype), 252)
    out_a = api.citrus_chunk_attn(cfg, x["q"], x["kc"], x["vc"], n_c, kch, vch, lse_cache=lse_c)
    out_b = api.citrus_chunk_attn(cfg, x["q"], x["kc"], x["vc"], n_c, kch, vch)
    assert torch.equal(out_a, out_b)
    one_pass = api.citrus_cache_score(cfg, x["q"], x["kc"], n_c, lse_cache=lse_c)
    torch.cuda.synchronize()
    scale = 1.0 / np.sqrt(d)
    for b in range(B):
        for l in range(L):
            ref = orc.instr_score(np64(x["q"][b, l]), np64(x["kc"][b, l, :, :n_c]))
            assert_close(np64(one_pass[b, l]), ref, dtype, f"single-pass cache score b{b} l{l}")
            kc64, q64 = np64(x["kc"][b, l, :, :n_c]), np64(x["q"][b, l])
            # the oracle's own normaliser of the rows over the cache states alone
            lse_ref = np.stack([orc.softmax_rows(q64[h] @ kc64[h // (Hq // Hkv)].T * scale)[1] for h in range(Hq)])
            assert_close(np64(lse_c[b, l]), lse_ref, dtype, f"cache-only log-sum-exp b{b} l{l}")
    # a configuration without such a cache has workspace for instr_len rows only
    plain = make_cfg(dtype, B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, c=c, k=n_c + 3, n_i=n_i)
    ws_plain = api.alloc_workspace(plain)
    if c > n_i:
        with pytest.raises(api.CitrusError):
            api.citrus_cache_score(plain, x["q"], x["kc"], n_c, workspace=ws_plain)
    few = api.citrus_cache_score(plain, x["q"], x["kc"], n_c, workspace=ws_plain, rows=min(c, n_i))
    ref = orc.instr_score(np64(x["q"][0, 0, :, :min(c, n_i)]), np64(x["kc"][0, 0, :, :n_c]))
    assert_close(np64(few[0, 0]), ref, dtype, "cache score, instruction-sized text")


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "-".join(str(x) for x in s[:9]))
def test_chunk_attn_parity(shape):
    dtype, B, L, Hq, Hkv, d, c, n_c, n_i, s = shape
    say(f"chunk_attn {shape}")
    x = step_inputs(*shape, seed=100)
    cfg = make_cfg(dtype, B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, c=c, k=max(n_c, 1) + 3, n_i=n_i)
    ws = api.alloc_workspace(cfg)
    lse = torch.empty((B, L, Hq, c), dtype=torch.float32, device=DEV)
    lm = torch.empty((B, L, Hkv, n_c + c), dtype=torch.float32, device=DEV)
    kc = x["kc"] if n_c > 0 else None
    vc = x["vc"] if n_c > 0 else None
    out = api.citrus_chunk_attn(cfg, x["q"], kc, vc, n_c, x["k"], x["v"], lse=lse, lm_score=lm, workspace=ws)
    torch.cuda.synchronize()
    for b in range(B):
        for l in range(L):
            kcat = np.concatenate([np64(x["kc"][b, l, :, :n_c]), np64(x["k"][b, l])], axis=1)
            vcat = np.concatenate([np64(x["vc"][b, l, :, :n_c]), np64(x["v"][b, l])], axis=1)
            o_ref, lse_ref, _ = orc.chunk_attn(np64(x["q"][b, l]), kcat, vcat, n_c)
            assert_close(np64(out[b, l]), o_ref, dtype, f"out b{b} l{l}")
            assert_close(np64(lse[b, l]), lse_ref, dtype, f"lse b{b} l{l}")
            assert_close(np64(lm[b, l]), orc.lm_score(np64(x["q"][b, l]), kcat, n_c), dtype, f"lm_score b{b} l{l}")
    # lm_score without a caller lse goes through the workspace and gives the same bits
    lm2 = torch.empty_like(lm)
    out2 = api.citrus_chunk_attn(cfg, x["q"], kc, vc, n_c, x["k"], x["v"], lm_score=lm2, workspace=ws)
    assert torch.equal(out, out2) and torch.equal(lm, lm2)


@pytest.mark.parametrize("direction", ["rising", "falling", "spike"])
def test_chunk_attn_moving_row_maximum(direction):
    """Logits whose row maximum keeps moving from tile to tile (rising), never moves after the first tile
    (falling), or jumps once by a large amount in the middle of the keys (spike): the running maximum is
    updated lazily and the accumulators, row sums and pending probabilities are rescaled on the way."""
    dtype, B, L, Hq, Hkv, d, c, n_c = "bf16", 1, 2, 8, 2, 128, 160, 416
    say(f"chunk_attn moving maximum {direction}")
    x = step_inputs(dtype, B, L, Hq, Hkv, d, c, n_c, 8, 1.0, seed=300)
    n = n_c + c
    pos = torch.arange(n, device=DEV, dtype=torch.float32)
    if direction == "rising":
        gain = 0.5 + 6.0 * pos / n
    elif direction == "falling":
        gain = 6.5 - 6.0 * pos / n
    else:
        gain = torch.where((pos >= 301) & (pos < 304), 12.0, 1.0)
    # keys share a direction with the queries so that the gain moves the logits, not only their spread
    bias = rand((1, 1, 1, 1, d), torch.bfloat16, 777, 1.0)
    kc = ((x["kc"][..., :n_c, :].float() + bias.float()) * gain[:n_c, None]).to(torch.bfloat16)
    kk = ((x["k"].float() + bias.float()) * gain[n_c:, None]).to(torch.bfloat16)
    q = (x["q"].float() + bias.float()).to(torch.bfloat16)
    cfg = make_cfg(dtype, B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, c=c, k=n_c, n_i=8)
    lse = torch.empty((B, L, Hq, c), dtype=torch.float32, device=DEV)
    out = api.citrus_chunk_attn(cfg, q, kc, x["vc"][..., :n_c, :], n_c, kk, x["v"], lse=lse)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all() and torch.isfinite(lse).all()
    for l in range(L):
        kcat = np.concatenate([np64(kc[0, l]), np64(kk[0, l])], axis=1)
        vcat = np.concatenate([np64(x["vc"][0, l, :, :n_c]), np64(x["v"][0, l])], axis=1)
        o_ref, lse_ref, _ = orc.chunk_attn(np64(q[0, l]), kcat, vcat, n_c)
        assert_close(np64(out[0, l]), o_ref, dtype, f"out l{l}")
        np.testing.assert_allclose(np64(lse[0, l]), lse_ref, rtol=1e-2, atol=2e-2)


def test_chunk_attn_strided_views_and_short_chunk():
    """Chunk tensors that are slices of document tensors; chunk shorter than cfg.chunk_len."""
    dtype, B, L, Hq, Hkv, d = "bf16", 1, 2, 8, 2, 128
    cfg = make_cfg(dtype, B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, c=64, k=128, n_i=8)
    qd, kd, vd = (rand((B, L, h, 200, d), torch.bfloat16, s) for h, s in ((Hq, 1), (Hkv, 2), (Hkv, 3)))
    kc, vc = rand((B, L, Hkv, 128, d), torch.bfloat16, 4), rand((B, L, Hkv, 128, d), torch.bfloat16, 5)
    outd = torch.zeros_like(qd)
    lo, hi = 150, 187
    api.citrus_chunk_attn(cfg, qd[:, :, :, lo:hi], kc, vc, 100, kd[:, :, :, lo:hi], vd[:, :, :, lo:hi],
                          out=outd[:, :, :, lo:hi])
    torch.cuda.synchronize()
    assert (outd[:, :, :, :lo] == 0).all() and (outd[:, :, :, hi:] == 0).all()
    for l in range(L):
        kcat = np.concatenate([np64(kc[0, l, :, :100]), np64(kd[0, l, :, lo:hi])], axis=1)
        vcat = np.concatenate([np64(vc[0, l, :, :100]), np64(vd[0, l, :, lo:hi])], axis=1)
        o_ref, _, _ = orc.chunk_attn(np64(qd[0, l, :, lo:hi]), kcat, vcat, 100)
        assert_close(np64(outd[0, l, :, lo:hi]), o_ref, dtype, f"strided out l{l}")


def test_custom_softmax_scale():
    cfg = make_cfg("f32", B=1, L=1, Hq=2, Hkv=1, d=64, c=16, k=32, n_i=4, softmax_scale=0.3)
    x = step_inputs("f32", 1, 1, 2, 1, 64, 16, 20, 4, 1.0)
    out = api.citrus_chunk_attn(cfg, x["q"], x["kc"], x["vc"], 20, x["k"], x["v"])
    kcat = np.concatenate([np64(x["kc"][0, 0, :, :20]), np64(x["k"][0, 0])], axis=1)
    vcat = np.concatenate([np64(x["vc"][0, 0, :, :20]), np64(x["v"][0, 0])], axis=1)
    o_ref, _, _ = orc.chunk_attn(np64(x["q"][0, 0]), kcat, vcat, 20, scale=0.3)
    assert_close(np64(out[0, 0]), o_ref, "f32", "scaled out")


# ----------------------------------------------------------------------------
# whole documents: step-by-step, teacher-forced against the oracle
# ----------------------------------------------------------------------------

def run_document_stepwise(w: Workload, sample_units=None, check_every=1):
    """Run the four entry points chunk by chunk; at every checked step replay
    the GPU's selections in the oracle (so one near-tie cannot change later
    steps) and compare outputs, scores, selections and the compacted cache."""
    cfg = api.Config.from_workload(w)
    doc = make_document(w, DEV)
    run = StepwiseRun(api, cfg, DEV)
    dual = w.cache_mode == api.CACHE_DUAL
    paper_lm = dual and w.lm_ordering == api.LM_EVICT_THEN_APPEND
    accumulated = w.score_mode == api.SCORE_ACCUMULATED
    units = sample_units or [(b, l) for b in range(w.batch) for l in range(w.layers)]
    hs = cfg.sel_heads
    # oracle-side state per unit: document positions held by each cache row
    pos = {u: np.zeros((w.kv_heads, 0), dtype=np.int64) for u in units}
    pos_lm = {u: np.zeros((w.kv_heads, 0), dtype=np.int64) for u in units}
    acc_ref = {u: np.zeros((w.kv_heads, 0)) for u in units}   # oracle-side accumulated scores of the cache rows
    host = {name: t.cpu() for name, t in doc.items()}
    band_fracs = []
    for i in range(w.n_chunks):
        lo, hi = w.chunk_bounds(i)
        rec = run.step(doc["q"][:, :, :, lo:hi], doc["k"][:, :, :, lo:hi], doc["v"][:, :, :, lo:hi], doc["q_instr"][i])
        torch.cuda.synchronize()
        c = hi - lo
        chunk_pos = np.broadcast_to(np.arange(lo, hi), (w.kv_heads, c))
        for (b, l) in units:
            kd, vd = np64(host["k"][b, l]), np64(host["v"][b, l])
            qd = np64(host["q"][b, l, :, lo:hi])
            qi = np64(host["q_instr"][i, b, l])
            # the cache the GPU should hold = document rows at the replayed positions
            cand = np.concatenate([pos[(b, l)], chunk_pos], axis=1)
            kcat = np.stack([kd[g, cand[g]] for g in range(w.kv_heads)])
            vcat = np.stack([vd[g, cand[g]] for g in range(w.kv_heads)])
            n_c = pos[(b, l)].shape[1]
            assert n_c == rec["n_c"]
            base = w.rope_base or 10000.0
            if w.position_shift:
                # the tensors are un-rotated; every step rotates them to the positions of the cache
                kcat = orc.rope(kcat, np.arange(n_c + c), base)
                if not dual:
                    qd = orc.rope(qd, n_c + np.arange(c), base)
                qi = orc.rope(qi, n_c + c + np.arange(qi.shape[1]), base)
            idx = rec["idx"][b, l].cpu().numpy()[:, :rec["m"]]
            check = (i % check_every == 0) or i == w.n_chunks - 1
            if dual:
                cand_lm = np.concatenate([pos_lm[(b, l)], chunk_pos], axis=1)
                kcat_lm = np.stack([kd[g, cand_lm[g]] for g in range(w.kv_heads)])
                vcat_lm = np.stack([vd[g, cand_lm[g]] for g in range(w.kv_heads)])
                n_c_lm = pos_lm[(b, l)].shape[1]
                assert n_c_lm == rec["n_c_lm"]
                if w.position_shift:   # the language-modelling cache has its own slots
                    kcat_lm = orc.rope(kcat_lm, np.arange(n_c_lm + c), base)
                    qd = orc.rope(qd, n_c_lm + np.arange(c), base)
                if check:
                    o_ref, lse_ref, _ = orc.chunk_attn(qd, kcat_lm, vcat_lm, n_c_lm)
                if paper_lm:
                    # the chunk's queries score the cache states alone; the kept ones stay in order and
                    # the whole chunk goes in behind them
                    kept = pos_lm[(b, l)]
                    if n_c_lm > 0:
                        idx_lm = rec["idx_lm"][b, l].cpu().numpy()[:, :rec["m_lm"]]
                        if check and n_c_lm > w.budget_lm:
                            s_lm_ref = orc.instr_score(qd, kcat_lm[:, :n_c_lm])
                            assert_close(np64(rec["score_lm"][b, l]), s_lm_ref, w.dtype,
                                         f"cache score step {i} unit {(b, l)}")
                            for g in range(hs):
                                ref_vec = s_lm_ref.sum(0) if hs == 1 else s_lm_ref[g]
                                gpu_vec = (layer_sum_f32(rec["score_lm"][b, l]) if hs == 1
                                           else rec["score_lm"][b, l, g].cpu().numpy())
                                band_fracs.append(check_selection(idx_lm[g], gpu_vec, ref_vec, w.budget_lm, w.dtype,
                                                                  f"lm cache select step {i}", w.start_size))
                        elif check:
                            np.testing.assert_array_equal(idx_lm, np.tile(np.arange(n_c_lm), (hs, 1)))
                        kept = np.stack([kept[g][idx_lm[g % hs]] for g in range(w.kv_heads)])
                    pos_lm[(b, l)] = np.concatenate([kept, chunk_pos], axis=1)
                else:
                    idx_lm = rec["idx_lm"][b, l].cpu().numpy()[:, :rec["m_lm"]]
                    if check:
                        s_lm_ref = orc.lm_score(qd, kcat_lm, n_c_lm)
                        assert_close(np64(rec["score_lm"][b, l]), s_lm_ref, w.dtype, f"lm_score step {i} unit {(b, l)}")
                        for g in range(hs):
                            ref_vec = s_lm_ref.sum(0) if hs == 1 else s_lm_ref[g]
                            gpu_vec = (layer_sum_f32(rec["score_lm"][b, l]) if hs == 1
                                       else rec["score_lm"][b, l, g].cpu().numpy())
                            band_fracs.append(check_selection(idx_lm[g], gpu_vec, ref_vec, w.budget_lm, w.dtype,
                                                              f"lm select step {i}", w.start_size))
                    pos_lm[(b, l)] = np.stack([cand_lm[g][idx_lm[g % hs]] for g in range(w.kv_heads)])
            elif check:
                o_ref, lse_ref, _ = orc.chunk_attn(qd, kcat, vcat, n_c)
            if check or accumulated:
                s_ref = orc.instr_score(qi, kcat)
                if accumulated:   # sums follow the replayed selections, like the positions
                    s_ref = s_ref + np.concatenate([acc_ref[(b, l)], np.zeros((w.kv_heads, c))], axis=1)
                    acc_ref[(b, l)] = np.stack([s_ref[g][idx[g % hs]] for g in range(w.kv_heads)])
            if check:
                assert_close(np64(rec["out"][b, l]), o_ref, w.dtype, f"out step {i} unit {(b, l)}")
                assert_close(np64(rec["lse"][b, l]), lse_ref, w.dtype, f"lse step {i} unit {(b, l)}")
                assert_close(np64(rec["score"][b, l]), s_ref, w.dtype, f"score step {i} unit {(b, l)}")
                for g in range(hs):
                    ref_vec = s_ref.sum(0) if hs == 1 else s_ref[g]
                    gpu_vec = layer_sum_f32(rec["score"][b, l]) if hs == 1 else rec["score"][b, l, g].cpu().numpy()
                    band_fracs.append(check_selection(idx[g], gpu_vec, ref_vec, w.budget, w.dtype, f"select step {i}",
                                                      w.start_size))
            pos[(b, l)] = np.stack([cand[g][idx[g % hs]] for g in range(w.kv_heads)])
            if check:
                # compaction bit-exact: cache row r holds document row pos[r]
                st = run.state
                kc_gpu, vc_gpu = st.current()
                for g in range(w.kv_heads):
                    p = torch.from_numpy(pos[(b, l)][g])
                    np.testing.assert_array_equal(bits(kc_gpu[b, l, g]), bits(host["k"][b, l, g][p]))
                    np.testing.assert_array_equal(bits(vc_gpu[b, l, g]), bits(host["v"][b, l, g][p]))
                if accumulated:
                    # the sums the kept states carry: copies of the GPU's own scores, close to the oracle's
                    acc_gpu = st.acc_score[st.buffer_index][b, l, :, :st.cache_len]
                    for g in range(w.kv_heads):
                        own = rec["score"][b, l, g][torch.from_numpy(idx[g % hs]).to(DEV).long()]
                        assert torch.equal(acc_gpu[g], own)
                    assert_close(np64(acc_gpu), acc_ref[(b, l)], w.dtype, f"accumulated score step {i} unit {(b, l)}")
                if dual:
                    kl_gpu, vl_gpu = st.current_lm()
                    for g in range(w.kv_heads):
                        p = torch.from_numpy(pos_lm[(b, l)][g])
                        np.testing.assert_array_equal(bits(kl_gpu[b, l, g]), bits(host["k"][b, l, g][p]))
                        np.testing.assert_array_equal(bits(vl_gpu[b, l, g]), bits(host["v"][b, l, g][p]))
    say(f"{w.name}: mean in-band fraction of the selection band rule = {np.mean(band_fracs):.3f}")
    if w.start_size and w.doc_len > w.budget:
        # the initial states are never evicted: the first rows of every cache are the first document rows
        for u in units:
            np.testing.assert_array_equal(pos[u][:, :w.start_size], np.tile(np.arange(w.start_size), (w.kv_heads, 1)))
            if dual:
                np.testing.assert_array_equal(pos_lm[u][:, :w.start_size],
                                              np.tile(np.arange(w.start_size), (w.kv_heads, 1)))
    return run, doc


def layer_sum_f32(score_blg: torch.Tensor) -> np.ndarray:
    s = score_blg.cpu().numpy()
    acc = s[0].copy()
    for g in range(1, s.shape[0]):
        acc = (acc + s[g]).astype(np.float32)
    return acc


DOC_CASES = {
    "cfg1": WORKLOADS["cfg1_tiny_f32"],
    "cfg1_peaked": peaked(WORKLOADS["cfg1_tiny_f32"]),
    "cfg1_ragged": scaled_down(WORKLOADS["cfg1_tiny_f32"], doc_len=499, layers=2, kv_heads=2, batch=2),
    "cfg1_per_layer": scaled_down(peaked(WORKLOADS["cfg1_tiny_f32"]), layers=2, kv_heads=2, doc_len=200,
                                  select_mode=api.SELECT_PER_LAYER),
    "cfg1_dual": scaled_down(peaked(WORKLOADS["cfg1_tiny_f32"]), doc_len=256, cache_mode=api.CACHE_DUAL, budget_lm=48),
    "cfg1_chunk_gt_budget": scaled_down(WORKLOADS["cfg1_tiny_f32"], doc_len=300, chunk_len=80, budget=50),
    "cfg1_start4": scaled_down(peaked(WORKLOADS["cfg1_tiny_f32"]), doc_len=256, layers=2, kv_heads=2, start_size=4),
    "cfg1_dual_start4": scaled_down(peaked(WORKLOADS["cfg1_tiny_f32"]), doc_len=256, cache_mode=api.CACHE_DUAL,
                                    budget_lm=48, start_size=4),
    "cfg1_dual_paper_order": scaled_down(peaked(WORKLOADS["cfg1_tiny_f32"]), doc_len=301, cache_mode=api.CACHE_DUAL,
                                         budget_lm=48, lm_ordering=api.LM_EVICT_THEN_APPEND),
    "cfg1_dual_paper_order_start4_per_layer": scaled_down(
        peaked(WORKLOADS["cfg1_tiny_f32"]), doc_len=256, layers=2, kv_heads=2, cache_mode=api.CACHE_DUAL, budget_lm=20,
        start_size=4, select_mode=api.SELECT_PER_LAYER, lm_ordering=api.LM_EVICT_THEN_APPEND),
    "cfg1_accumulated": scaled_down(peaked(WORKLOADS["cfg1_tiny_f32"]), doc_len=300, layers=2, kv_heads=2,
                                    score_mode=api.SCORE_ACCUMULATED),
    "cfg1_accumulated_per_layer_start4": scaled_down(peaked(WORKLOADS["cfg1_tiny_f32"]), doc_len=256, layers=2, kv_heads=2,
                                                     score_mode=api.SCORE_ACCUMULATED, start_size=4,
                                                     select_mode=api.SELECT_PER_LAYER),
    "cfg2_small_accumulated": scaled_down(WORKLOADS["cfg2_mistral7b"], layers=2, doc_len=2300,
                                          score_mode=api.SCORE_ACCUMULATED),
    "cfg1_position_shift": scaled_down(peaked(WORKLOADS["cfg1_tiny_f32"]), doc_len=301, layers=2, kv_heads=2,
                                       position_shift=1),
    "cfg1_position_shift_accumulated_per_layer": scaled_down(
        peaked(WORKLOADS["cfg1_tiny_f32"]), doc_len=256, layers=2, kv_heads=2, position_shift=1, rope_base=500.0,
        score_mode=api.SCORE_ACCUMULATED, select_mode=api.SELECT_PER_LAYER, start_size=2),
    "cfg2_small_position_shift": scaled_down(WORKLOADS["cfg2_mistral7b"], layers=2, doc_len=2300, position_shift=1),
    "cfg1_dual_position_shift": scaled_down(peaked(WORKLOADS["cfg1_tiny_f32"]), doc_len=301, layers=2, kv_heads=2,
                                            cache_mode=api.CACHE_DUAL, budget_lm=48, position_shift=1, rope_base=500.0),
    "cfg1_dual_paper_order_position_shift": scaled_down(peaked(WORKLOADS["cfg1_tiny_f32"]), doc_len=256,
                                                        cache_mode=api.CACHE_DUAL, budget_lm=40, position_shift=1,
                                                        lm_ordering=api.LM_EVICT_THEN_APPEND),
    "cfg4_small_dual_position_shift": scaled_down(peaked(WORKLOADS["cfg4_dual"]), batch=2, layers=1, q_heads=8, kv_heads=2,
                                                  doc_len=1500, chunk_len=256, budget=320, budget_lm=384, position_shift=1),
    "cfg4_small_dual_paper_order_position_shift": scaled_down(
        WORKLOADS["cfg4_dual"], batch=1, layers=2, q_heads=8, kv_heads=2, doc_len=1300, chunk_len=256, budget=320,
        budget_lm=256, position_shift=1, lm_ordering=api.LM_EVICT_THEN_APPEND),
    "cfg2_small": scaled_down(WORKLOADS["cfg2_mistral7b"], layers=2, doc_len=2560),
    "cfg2_small_start4": scaled_down(WORKLOADS["cfg2_mistral7b"], layers=2, doc_len=2560, start_size=4),
    "cfg2_small_peaked": scaled_down(peaked(WORKLOADS["cfg2_mistral7b"]), layers=1, doc_len=2000),
    "cfg3_small_shared_mha": scaled_down(WORKLOADS["cfg3_llama2_7b_shared"], batch=2, layers=1, q_heads=4, kv_heads=4,
                                         doc_len=2100, chunk_len=256, budget=384, instr_len=32),
    "cfg4_small_dual": scaled_down(peaked(WORKLOADS["cfg4_dual"]), batch=2, layers=1, q_heads=8, kv_heads=2,
                                   doc_len=1536, chunk_len=256, budget=320, budget_lm=384),
    "cfg4_small_dual_paper_order": scaled_down(peaked(WORKLOADS["cfg4_dual"]), batch=2, layers=1, q_heads=8, kv_heads=2,
                                               doc_len=1500, chunk_len=256, budget=320, budget_lm=384,
                                               lm_ordering=api.LM_EVICT_THEN_APPEND),
    "cfg5_small_g8": scaled_down(WORKLOADS["cfg5_large"], batch=1, layers=1, q_heads=16, kv_heads=2, doc_len=2048,
                                 chunk_len=512, budget=640, instr_len=96),
    # degenerate sizes: one-token chunks, budget 1, one instruction token, a document shorter than a chunk
    "degenerate_f32_c1_k1_ni1": scaled_down(WORKLOADS["cfg1_tiny_f32"], doc_len=7, chunk_len=1, budget=1, instr_len=1),
    "degenerate_bf16_c1_k1_ni1": scaled_down(WORKLOADS["cfg2_mistral7b"], layers=1, doc_len=6, chunk_len=1, budget=1,
                                             instr_len=1),
    "degenerate_bf16_c64_k1": scaled_down(WORKLOADS["cfg2_mistral7b"], layers=1, doc_len=300, chunk_len=64, budget=1),
    "degenerate_bf16_doc_shorter_than_chunk": scaled_down(WORKLOADS["cfg2_mistral7b"], layers=1, doc_len=100),
    "degenerate_bf16_dual_c1": scaled_down(peaked(WORKLOADS["cfg2_mistral7b"]), layers=1, doc_len=9, chunk_len=1, budget=2,
                                           budget_lm=3, instr_len=3, cache_mode=api.CACHE_DUAL),
    "degenerate_bf16_dual_paper_order_c5": scaled_down(peaked(WORKLOADS["cfg2_mistral7b"]), layers=1, doc_len=40,
                                                       chunk_len=5, budget=4, budget_lm=3, instr_len=3,
                                                       cache_mode=api.CACHE_DUAL, lm_ordering=api.LM_EVICT_THEN_APPEND),
    "degenerate_bf16_position_shift_c7": scaled_down(peaked(WORKLOADS["cfg2_mistral7b"]), layers=1, doc_len=50,
                                                     chunk_len=7, budget=9, instr_len=3, position_shift=1),
}


@pytest.mark.parametrize("case", list(DOC_CASES), ids=list(DOC_CASES))
def test_document_stepwise_teacher_forced(case):
    say(f"document {case}")
    run_document_stepwise(DOC_CASES[case])


# ----------------------------------------------------------------------------
# Standard CSE on its own, and the extra eviction by the instruction after the last chunk
# ----------------------------------------------------------------------------

STANDARD_CASES = {
    "cfg1_standard_paper_order": scaled_down(peaked(WORKLOADS["cfg1_tiny_f32"]), doc_len=301,
                                             cache_mode=api.CACHE_STANDARD, lm_ordering=api.LM_EVICT_THEN_APPEND),
    "cfg1_standard_after_append_per_layer_start2": scaled_down(
        peaked(WORKLOADS["cfg1_tiny_f32"]), doc_len=256, layers=2, kv_heads=2, cache_mode=api.CACHE_STANDARD,
        select_mode=api.SELECT_PER_LAYER, start_size=2),
    "cfg2_small_standard_paper_order": scaled_down(WORKLOADS["cfg2_mistral7b"], layers=1, doc_len=2300,
                                                   cache_mode=api.CACHE_STANDARD, lm_ordering=api.LM_EVICT_THEN_APPEND),
    "cfg2_small_standard_paper_order_per_layer": scaled_down(
        peaked(WORKLOADS["cfg2_mistral7b"]), layers=2, doc_len=1700, cache_mode=api.CACHE_STANDARD,
        lm_ordering=api.LM_EVICT_THEN_APPEND, select_mode=api.SELECT_PER_LAYER, start_size=4),
}


def _selection_checks(idx_gpu, score_gpu_blg, score_ref, k, w, what):
    """Band rule and exactness for every selection head of one (document, layer)."""
    hs = idx_gpu.shape[0]
    for g in range(hs):
        ref_vec = score_ref.sum(0) if hs == 1 else score_ref[g]
        gpu_vec = layer_sum_f32(score_gpu_blg) if hs == 1 else score_gpu_blg[g].cpu().numpy()
        check_selection(idx_gpu[g], gpu_vec, ref_vec, k, w.dtype, what, w.start_size)


@pytest.mark.parametrize("case", list(STANDARD_CASES), ids=list(STANDARD_CASES))
def test_standard_cse_document_and_final_instruction_eviction(case):
    w = STANDARD_CASES[case]
    say(f"standard CSE {case}")
    cfg = api.Config.from_workload(w)
    doc = make_document(w, DEV)
    run = StepwiseRun(api, cfg, DEV)
    outs = []
    for i in range(w.n_chunks):
        lo, hi = w.chunk_bounds(i)
        outs.append(run.step(doc["q"][:, :, :, lo:hi], doc["k"][:, :, :, lo:hi], doc["v"][:, :, :, lo:hi], None)["out"])
    torch.cuda.synchronize()
    out_gpu = torch.cat(outs, dim=3)
    st = run.state
    hs = cfg.sel_heads
    # the extra eviction with the instruction as the text, into the other buffer of the pair
    qi = doc["q_instr"][w.n_chunks - 1]
    idx_f = torch.full((w.batch, w.layers, hs, w.budget), -1, dtype=torch.int32, device=DEV)
    k_cur, v_cur = st.k_cache[st.buffer_index], st.v_cache[st.buffer_index]
    k_fin, v_fin = st.k_cache[st.buffer_index ^ 1], st.v_cache[st.buffer_index ^ 1]
    kept = api.citrus_evict_cache(cfg, qi, k_cur, v_cur, st.cache_len, w.budget, k_fin, v_fin, idx=idx_f, workspace=run.ws)
    score_f = api.citrus_cache_score(cfg, qi, k_cur, st.cache_len, workspace=run.ws)
    torch.cuda.synchronize()
    assert kept == min(w.budget, st.cache_len)
    host = {name: t.cpu() for name, t in doc.items()}
    for b in range(w.batch):
        for l in range(w.layers):
            # the oracle follows the GPU's selections, so one near-tie cannot change the later steps
            forced = [np.zeros((hs, 0), dtype=np.int64) if rec["idx"] is None
                      else rec["idx"][b, l].cpu().numpy()[:, :rec["m"]].astype(np.int64) for rec in run.steps]
            idx_f_bl = idx_f[b, l].cpu().numpy()[:, :kept].astype(np.int64)
            res = orc.standard_cse(np64(host["q"][b, l]), np64(host["k"][b, l]), np64(host["v"][b, l]), w.chunk_len,
                                   w.budget, lm_ordering=w.lm_ordering, select_mode=w.select_mode,
                                   start_size=w.start_size, q_instr_final=np64(host["q_instr"][w.n_chunks - 1, b, l]),
                                   forced_idx=forced, forced_idx_final=idx_f_bl)
            assert_close(np64(out_gpu[b, l]), res.out, w.dtype, f"out unit {(b, l)}")
            for i, rec in enumerate(run.steps):
                if rec["score"] is None:
                    continue   # nothing had to be evicted at this step
                assert_close(np64(rec["score"][b, l]), res.score[i], w.dtype, f"score step {i} unit {(b, l)}")
                _selection_checks(forced[i], rec["score"][b, l], res.score[i], w.budget, w, f"select step {i}")
            # cache when the document has ended: bit copies of the document rows the oracle holds
            assert res.positions.shape[1] == st.cache_len
            for g in range(w.kv_heads):
                p = torch.from_numpy(res.positions[g])
                np.testing.assert_array_equal(bits(k_cur[b, l, g, :st.cache_len]), bits(host["k"][b, l, g][p]))
                np.testing.assert_array_equal(bits(v_cur[b, l, g, :st.cache_len]), bits(host["v"][b, l, g][p]))
            # final eviction by the instruction
            if st.cache_len > w.budget:
                assert_close(np64(score_f[b, l]), res.score_final, w.dtype, f"final score unit {(b, l)}")
                _selection_checks(idx_f_bl, score_f[b, l], res.score_final, w.budget, w, "final select")
            else:
                np.testing.assert_array_equal(idx_f_bl, np.tile(np.arange(kept), (hs, 1)))
            for g in range(w.kv_heads):
                p = torch.from_numpy(res.positions_final[g])
                np.testing.assert_array_equal(bits(k_fin[b, l, g, :kept]), bits(host["k"][b, l, g][p]))
                np.testing.assert_array_equal(bits(v_fin[b, l, g, :kept]), bits(host["v"][b, l, g][p]))
    if w.start_size:
        assert (idx_f[..., :w.start_size].cpu() == torch.arange(w.start_size)).all()


# ----------------------------------------------------------------------------
# rotary embedding at explicit positions
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("dtype,B,L,H,rows,d,pos0,base", [
    ("bf16", 1, 2, 8, 70, 128, 0, 0.0), ("bf16", 2, 1, 3, 33, 128, 777, 1e6), ("bf16", 1, 1, 32, 512, 128, 768, 0.0),
    ("bf16", 1, 2, 2, 19, 64, 5, 500.0), ("f32", 1, 2, 4, 45, 64, 1300, 0.0), ("f32", 2, 1, 2, 7, 128, 4000, 1e6),
])
def test_rope_parity(dtype, B, L, H, rows, d, pos0, base):
    say(f"rope {dtype} B{B} L{L} H{H} rows{rows} d{d} pos0 {pos0} base {base}")
    cfg = make_cfg(dtype, B=B, L=L, Hq=H, Hkv=H, d=d, c=32, k=64, n_i=8, rope_base=base)
    buf = rand((B, L, H, rows + 6, d), tdt(dtype), 501)
    x = buf[:, :, :, 3:3 + rows]                     # a strided view
    before = buf.clone()
    y = api.citrus_rope(cfg, x, pos0)
    torch.cuda.synchronize()
    assert torch.equal(buf, before)
    for b in range(B):
        for l in range(L):
            ref = orc.rope(np64(x[b, l]), pos0 + np.arange(rows), base or 10000.0)
            assert_close(np64(y[b, l]), ref, dtype, f"rope b{b} l{l}")
    # in place gives the same bits and leaves the rows around the view alone
    api.citrus_rope(cfg, x, pos0, y=x)
    torch.cuda.synchronize()
    assert torch.equal(x, y)
    assert torch.equal(buf[:, :, :, :3], before[:, :, :, :3]) and torch.equal(buf[:, :, :, 3 + rows:], before[:, :, :, 3 + rows:])


# ----------------------------------------------------------------------------
# decoding steps over the retained cache
# ----------------------------------------------------------------------------

DECODE_SHAPES = [
    # dtype, B, L, Hq, Hkv, d, cache_len, qk_scale
    ("bf16", 1, 2, 8, 2, 128, 0, 1.0),
    ("bf16", 1, 1, 4, 4, 128, 31, 1.0),
    ("bf16", 2, 1, 8, 2, 128, 32, 0.5),
    ("bf16", 1, 2, 32, 8, 128, 832, 0.09),
    ("bf16", 1, 1, 16, 2, 128, 1201, 0.3),
    ("bf16", 1, 1, 64, 2, 128, 300, 0.3),
    ("bf16", 3, 2, 4, 1, 128, 4500, 0.09),
    ("bf16", 4, 8, 16, 8, 128, 100, 0.3),
    ("bf16", 1, 1, 8, 2, 128, 40000, 0.09),   # two units, keys split over eight workgroups each
    ("bf16", 2, 40, 8, 8, 128, 1203, 0.3),    # 640 units: more than the chip takes at once, no split
    ("bf16", 1, 2, 4, 2, 64, 77, 0.5),
    ("f32", 2, 1, 4, 2, 64, 45, 1.0),
    ("f32", 1, 1, 2, 2, 128, 130, 0.5),
]


@pytest.mark.parametrize("shape", DECODE_SHAPES, ids=lambda s: "-".join(str(x) for x in s[:7]))
def test_decode_step_parity(shape):
    dtype, B, L, Hq, Hkv, d, n, s = shape
    say(f"decode_step {shape}")
    t = tdt(dtype)
    steps = 3
    cap = n + steps + 2
    cfg = make_cfg(dtype, B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, c=16, k=max(n, 1), n_i=4, cache_capacity=cap)
    ws = api.alloc_workspace(cfg)
    # the cache is a view with a longer row pitch than its capacity (strides are honoured)
    kbuf, vbuf = rand((B, L, Hkv, cap + 5, d), t, 401, s), rand((B, L, Hkv, cap + 5, d), t, 402)
    kc, vc = kbuf[:, :, :, :cap], vbuf[:, :, :, :cap]
    k_before, v_before = kc.clone(), vc.clone()
    ref_k = [[np64(kc[b, l, :, :n]) for l in range(L)] for b in range(B)]
    ref_v = [[np64(vc[b, l, :, :n]) for l in range(L)] for b in range(B)]
    for i in range(steps):
        q = rand((B, L, Hq, 1, d), t, 410 + i, s)
        kn, vn = rand((B, L, Hkv, 1, d), t, 420 + i, s), rand((B, L, Hkv, 1, d), t, 430 + i)
        out = api.citrus_decode_step(cfg, q, kn, vn, kc, vc, n + i, workspace=ws)
        torch.cuda.synchronize()
        assert torch.equal(kc[:, :, :, n + i], kn[:, :, :, 0]) and torch.equal(vc[:, :, :, n + i], vn[:, :, :, 0])
        for b in range(B):
            for l in range(L):
                o_ref, ref_k[b][l], ref_v[b][l] = orc.decode_step(np64(q[b, l, :, 0]), np64(kn[b, l, :, 0]),
                                                                  np64(vn[b, l, :, 0]), ref_k[b][l], ref_v[b][l])
                assert_close(np64(out[b, l, :, 0]), o_ref, dtype, f"decode step {i} b{b} l{l}")
    # nothing but the appended rows changed, inside the view and outside
    assert torch.equal(kc[:, :, :, :n], k_before[:, :, :, :n]) and torch.equal(vc[:, :, :, :n], v_before[:, :, :, :n])
    assert torch.equal(kc[:, :, :, n + steps:], k_before[:, :, :, n + steps:])
    assert torch.equal(vc[:, :, :, n + steps:], v_before[:, :, :, n + steps:])
    # a full cache is refused
    with pytest.raises(api.CitrusError):
        api.citrus_decode_step(cfg, q, kn, vn, kc, vc, cap, workspace=ws)


def test_decode_step_repeats_bit_identically_and_matches_chunk_attention_of_one_token():
    """The same step twice gives the same bits; a chunk of one token through citrus_chunk_attn is the same
    computation by another kernel (agreement within the bf16 tolerance)."""
    B, L, Hq, Hkv, d, n = 1, 2, 32, 8, 128, 832
    cfg = make_cfg("bf16", B=B, L=L, Hq=Hq, Hkv=Hkv, d=d, c=16, k=n, n_i=4, cache_capacity=n + 4)
    ws = api.alloc_workspace(cfg)
    kc, vc = rand((B, L, Hkv, n + 4, d), torch.bfloat16, 441, 0.09), rand((B, L, Hkv, n + 4, d), torch.bfloat16, 442)
    q = rand((B, L, Hq, 1, d), torch.bfloat16, 443, 0.09)
    kn, vn = rand((B, L, Hkv, 1, d), torch.bfloat16, 444, 0.09), rand((B, L, Hkv, 1, d), torch.bfloat16, 445)
    by_chunk = api.citrus_chunk_attn(cfg, q, kc, vc, n, kn, vn)
    a = api.citrus_decode_step(cfg, q, kn, vn, kc, vc, n, workspace=ws)
    b = api.citrus_decode_step(cfg, q, kn, vn, kc, vc, n, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    np.testing.assert_allclose(np64(a), np64(by_chunk), atol=2e-2, rtol=1e-2)


# ----------------------------------------------------------------------------
# the chunk loop entry point
# ----------------------------------------------------------------------------

def run_process_document(w, doc, split_at=None, use_python_provider=False, use_side_stream=False):
    cfg = api.Config.from_workload(w)
    state = api.DocumentState.allocate(cfg, DEV)
    ws = api.alloc_workspace(cfg, DEV)
    out = torch.zeros_like(doc["q"])
    hist = torch.full((w.n_chunks, w.batch, w.layers, cfg.sel_heads, w.budget), -1, dtype=torch.int32, device=DEV)
    hist_lm = None
    if w.cache_mode == api.CACHE_DUAL:
        hist_lm = torch.full((w.n_chunks, w.batch, w.layers, cfg.sel_heads, w.budget_lm), -1, dtype=torch.int32, device=DEV)
    rd = api.resident_doc(cfg, doc["q"], doc["k"], doc["v"], doc["q_instr"], out)
    side = api.SideStream(DEV) if use_side_stream else None
    if use_side_stream:
        # selection and gather next to the attention (single-cache modes); twice in a row, so that a second call
        # starts while the side stream may still hold work of the first
        done = api.citrus_process_document(cfg, state, ws, doc=rd, idx_history=hist, idx_history_lm=hist_lm, side=side)
        state.cache_len = state.cache_len_lm = 0
        state.buffer_index = state.buffer_index_lm = 0
        done = api.citrus_process_document(cfg, state, ws, doc=rd, idx_history=hist, idx_history_lm=hist_lm, side=side)
    elif use_python_provider:
        def provider(i, io):
            lo, hi = w.chunk_bounds(i)
            if lo >= w.doc_len:
                return 1
            io.q = api.binding.tensor(doc["q"][:, :, :, lo:hi])
            io.k = api.binding.tensor(doc["k"][:, :, :, lo:hi])
            io.v = api.binding.tensor(doc["v"][:, :, :, lo:hi])
            io.out = api.binding.tensor(out[:, :, :, lo:hi])
            io.q_instr = api.binding.tensor(doc["q_instr"][i])
            io.chunk_len = hi - lo
            return 0
        done = api.citrus_process_document(cfg, state, ws, provider=provider, idx_history=hist, idx_history_lm=hist_lm)
    elif split_at is None:
        done = api.citrus_process_document(cfg, state, ws, doc=rd, idx_history=hist, idx_history_lm=hist_lm)
    else:
        d1 = api.citrus_process_document(cfg, state, ws, doc=rd, max_chunks=split_at, idx_history=hist,
                                         idx_history_lm=hist_lm)
        torch.cuda.synchronize()
        d2 = api.citrus_process_document(cfg, state, ws, doc=rd, first_chunk=split_at, idx_history=hist[split_at:],
                                         idx_history_lm=None if hist_lm is None else hist_lm[split_at:])
        done = d1 + d2
    torch.cuda.synchronize()
    assert done == w.n_chunks
    return state, out, hist, hist_lm


@pytest.mark.parametrize("case", ["cfg1", "cfg1_ragged", "cfg1_dual", "cfg1_dual_start4", "cfg1_dual_paper_order",
                                  "cfg1_dual_paper_order_start4_per_layer", "cfg2_small", "cfg2_small_start4",
                                  "cfg4_small_dual", "cfg4_small_dual_paper_order", "cfg1_position_shift", "cfg1_dual_position_shift",
                                  "cfg1_dual_paper_order_position_shift", "cfg4_small_dual_position_shift",
                                  "cfg4_small_dual_paper_order_position_shift",
                                  "cfg1_position_shift_accumulated_per_layer", "cfg2_small_position_shift", "cfg1_accumulated",
                                  "cfg1_accumulated_per_layer_start4", "cfg2_small_accumulated", "cfg1_standard_paper_order",
                                  "cfg1_standard_after_append_per_layer_start2", "cfg2_small_standard_paper_order"])
def test_process_document_equals_stepwise_and_resumes(case):
    say(f"process_document {case}")
    check_process_document_equals_stepwise(DOC_CASES.get(case) or STANDARD_CASES[case])


def check_process_document_equals_stepwise(w):
    cfg = api.Config.from_workload(w)
    doc = make_document(w, DEV)
    # stepwise reference run on the GPU (itself checked against the oracle above)
    run = StepwiseRun(api, cfg, DEV)
    outs = []
    for i in range(w.n_chunks):
        lo, hi = w.chunk_bounds(i)
        outs.append(run.step(doc["q"][:, :, :, lo:hi], doc["k"][:, :, :, lo:hi], doc["v"][:, :, :, lo:hi],
                             doc["q_instr"][i])["out"])
    torch.cuda.synchronize()
    out_step = torch.cat(outs, dim=3)
    state, out, hist, hist_lm = run_process_document(w, doc)
    assert torch.equal(out, out_step)
    assert state.cache_len == run.state.cache_len and state.cache_len_lm == run.state.cache_len_lm
    if not (w.cache_mode == api.CACHE_STANDARD and w.lm_ordering == api.LM_EVICT_THEN_APPEND):
        assert state.cache_len == min(w.budget, w.doc_len)
    for a, b in zip(state.current(), run.state.current()):
        assert torch.equal(a, b)
    for i, rec in enumerate(run.steps):
        if rec["idx"] is not None:  # None: first chunk of the evict-then-append order
            assert torch.equal(hist[i][..., :rec["m"]], rec["idx"][..., :rec["m"]])
        if hist_lm is not None and rec["idx_lm"] is not None:  # None: first chunk of the evict-then-append order
            assert torch.equal(hist_lm[i][..., :rec["m_lm"]], rec["idx_lm"][..., :rec["m_lm"]])
    if hist_lm is not None:
        for a, b in zip(state.current_lm(), run.state.current_lm()):
            assert torch.equal(a, b)
    if w.score_mode == api.SCORE_ACCUMULATED:
        assert torch.equal(state.acc_score[state.buffer_index][..., :state.cache_len],
                           run.state.acc_score[run.state.buffer_index][..., :run.state.cache_len])
    # resume: two calls give the same bits as one; so does a second full run, a Python provider, and a run with a side stream
    for kw in (dict(split_at=max(1, w.n_chunks // 3)), dict(), dict(use_python_provider=True), dict(use_side_stream=True)):
        state2, out2, hist2, _ = run_process_document(w, doc, **kw)
        assert torch.equal(out2, out) and torch.equal(hist2, hist), kw
        for a, b in zip(state2.current(), state.current()):
            assert torch.equal(a, b)


def test_budget_at_least_document_is_full_causal_attention():
    w = scaled_down(WORKLOADS["cfg2_mistral7b"], layers=1, q_heads=8, kv_heads=2, doc_len=700, chunk_len=128,
                    budget=1024, instr_len=16)
    doc = make_document(w, DEV)
    state, out, hist, _ = run_process_document(w, doc)
    assert state.cache_len == 700
    kc, vc = state.current()
    assert torch.equal(kc, doc["k"]) and torch.equal(vc, doc["v"])
    ref = orc.full_causal_attention(np64(doc["q"][0, 0]), np64(doc["k"][0, 0]), np64(doc["v"][0, 0]))
    assert_close(np64(out[0, 0]), ref, "bf16", "full causal")


# ----------------------------------------------------------------------------
# full-size run in the launch configuration bench.py times (sampled checks)
# ----------------------------------------------------------------------------

def test_full_size_cfg2_sampled_against_oracle():
    """The whole Mistral-7B-shaped document through citrus_process_document, as
    bench.py runs it.  The oracle replays the GPU's selection history for a few
    (document, layer) units (integer gathers only) and checks, at sampled
    steps, the attention output, the selection against the oracle's scores
    (band rule) and, at the end, the compacted cache bit for bit."""
    w = WORKLOADS["cfg2_mistral7b"]
    say(f"full size {w.name}")
    cfg = api.Config.from_workload(w)
    doc = make_document(w, DEV)
    state, out, hist, _ = run_process_document(w, doc)
    assert state.cache_len == w.budget
    units = [(0, 0), (0, 13), (0, 31)]
    steps = {0, 1, 2, 17, 31}
    hist_h = hist.cpu().numpy()
    kc_gpu, vc_gpu = state.current()
    in_band = []
    for (b, l) in units:
        kd, vd = np64(doc["k"][b, l]), np64(doc["v"][b, l])
        pos = np.zeros((w.kv_heads, 0), dtype=np.int64)
        for i in range(w.n_chunks):
            lo, hi = w.chunk_bounds(i)
            cand = np.concatenate([pos, np.broadcast_to(np.arange(lo, hi), (w.kv_heads, hi - lo))], axis=1)
            m = min(w.budget, cand.shape[1])
            idx = hist_h[i, b, l][:, :m]
            assert (np.diff(idx, axis=1) > 0).all() and idx.min() >= 0 and idx.max() < cand.shape[1]
            if i in steps:
                kcat = np.stack([kd[g, cand[g]] for g in range(w.kv_heads)])
                vcat = np.stack([vd[g, cand[g]] for g in range(w.kv_heads)])
                o_ref, _, _ = orc.chunk_attn(np64(doc["q"][b, l, :, lo:hi]), kcat, vcat, pos.shape[1])
                assert_close(np64(out[b, l, :, lo:hi]), o_ref, w.dtype, f"out unit {(b, l)} step {i}")
                s_ref = orc.instr_score(np64(doc["q_instr"][i, b, l]), kcat)
                np.testing.assert_allclose(s_ref.sum(axis=1), w.instr_len * w.group, rtol=1e-9)
                if cand.shape[1] > w.budget:
                    atol, rtol = TOL[w.dtype]
                    for g in range(w.kv_heads):
                        ref_idx = orc.topk_select_1d(s_ref[g], w.budget)
                        boundary = np.sort(s_ref[g])[::-1][w.budget - 1]
                        band = np.abs(s_ref[g] - boundary) <= atol + rtol * abs(boundary)
                        diff = np.setxor1d(idx[g], ref_idx)
                        assert band[diff].all()
                        in_band.append(band.mean())
            pos = np.stack([cand[g][idx[g]] for g in range(w.kv_heads)])
        for g in range(w.kv_heads):
            p = torch.from_numpy(pos[g])
            np.testing.assert_array_equal(bits(kc_gpu[b, l, g]), bits(doc["k"][b, l, g].cpu()[p]))
            np.testing.assert_array_equal(bits(vc_gpu[b, l, g]), bits(doc["v"][b, l, g].cpu()[p]))
    say(f"full size: fraction of positions inside the selection tolerance band = {np.mean(in_band):.3f}")


def test_full_size_single_step_all_checks():
    """One steady-state step of the Mistral-7B-shaped configuration through the
    four entry points, all (document, layer) units launched, three checked:
    outputs, log-sum-exp, scores, exact selection, bit-exact compaction."""
    w = WORKLOADS["cfg2_mistral7b"]
    cfg = api.Config.from_workload(w)
    ch = make_chunk(w, 5, DEV)
    n_c = w.budget
    kc = rand((w.batch, w.layers, w.kv_heads, n_c, w.head_dim), torch.bfloat16, 11, w.head_dim ** -0.5)
    vc = rand((w.batch, w.layers, w.kv_heads, n_c, w.head_dim), torch.bfloat16, 12, w.head_dim ** -0.5)
    ws = api.alloc_workspace(cfg)
    lse = torch.empty((w.batch, w.layers, w.q_heads, w.chunk_len), dtype=torch.float32, device=DEV)
    out = api.citrus_chunk_attn(cfg, ch["q"], kc, vc, n_c, ch["k"], ch["v"], lse=lse)
    score = api.citrus_instr_score(cfg, ch["q_instr"], kc, n_c, ch["k"], workspace=ws)
    idx = api.citrus_topk_select(cfg, score, w.budget)
    kn, vn = torch.zeros_like(kc), torch.zeros_like(vc)
    api.citrus_kv_compact(cfg, kc, vc, n_c, ch["k"], ch["v"], idx, w.budget, kn, vn)
    torch.cuda.synchronize()
    for l in (0, 9, 31):
        kcat = np.concatenate([np64(kc[0, l]), np64(ch["k"][0, l])], axis=1)
        vcat = np.concatenate([np64(vc[0, l]), np64(ch["v"][0, l])], axis=1)
        o_ref, lse_ref, _ = orc.chunk_attn(np64(ch["q"][0, l]), kcat, vcat, n_c)
        assert_close(np64(out[0, l]), o_ref, "bf16", f"out l{l}")
        assert_close(np64(lse[0, l]), lse_ref, "bf16", f"lse l{l}")
        s_ref = orc.instr_score(np64(ch["q_instr"][0, l]), kcat)
        assert_close(np64(score[0, l]), s_ref, "bf16", f"score l{l}")
        kb = np.concatenate([bits(kc[0, l]), bits(ch["k"][0, l])], axis=1)
        vb = np.concatenate([bits(vc[0, l]), bits(ch["v"][0, l])], axis=1)
        for g in range(w.kv_heads):
            check_selection(idx[0, l, g].cpu().numpy(), score[0, l, g].cpu().numpy(), s_ref[g], w.budget, "bf16")
        k_ref, v_ref = orc.kv_compact(kb, vb, idx[0, l].cpu().numpy())
        np.testing.assert_array_equal(bits(kn[0, l]), k_ref)
        np.testing.assert_array_equal(bits(vn[0, l]), v_ref)
