"""Parity of the entry points with the CPU oracle over seeded random shapes: ragged chunk and
cache lengths, every GQA group size the kernels special-case, both head dims and both dtypes.
The shapes are drawn from a seeded generator, so a failing case is named by its index.  Needs an
MI355X."""

import numpy as np
import pytest
import torch

import paper_2406_12018_amd as api
from oracle import citrus_oracle as orc

from helpers import assert_close, np64

pytestmark = pytest.mark.gpu
DEV = "cuda"
CASES = 48


def rand(shape, dt, seed, scale=1.0):
    g = torch.Generator().manual_seed(int(seed))
    return (torch.randn(shape, generator=g) * scale).to(dt).to(DEV)


def draw_shape(case):
    rng = np.random.default_rng(7000 + case)
    dtype = "bf16" if rng.random() < 0.85 else "f32"
    d = 128 if rng.random() < 0.8 else 64
    B, L = int(rng.integers(1, 3)), int(rng.integers(1, 3))
    Hkv = int(rng.choice([1, 2, 4]))
    G = int(rng.choice([1, 2, 3, 4, 8, 16, 32]))
    c = int(rng.integers(1, 560))
    # an empty cache, any length, or a multiple of the 32-key half tile (the fused cache normaliser's case)
    n_c = int(rng.choice([0, int(rng.integers(1, 1500)), 32 * int(rng.integers(1, 44))]))
    n_i = int(rng.integers(1, 140))
    scale = float(rng.choice([0.09, 0.3, 1.0, 3.0]))  # flat to sharply peaked attention rows (logits of a few tens)
    return dtype, d, B, L, Hkv, G, c, n_c, n_i, scale


@pytest.mark.parametrize("case", range(CASES))
def test_random_shape(case):
    dtype, d, B, L, Hkv, G, c, n_c, n_i, s = draw_shape(case)
    Hq = Hkv * G
    print(f"case {case}: {dtype} d{d} B{B} L{L} Hq{Hq} Hkv{Hkv} c{c} n_c{n_c} n_i{n_i} scale{s}", flush=True)
    dt = torch.bfloat16 if dtype == "bf16" else torch.float32
    cap = n_c + c + 8
    cfg = api.Config(batch=B, layers=L, q_heads=Hq, kv_heads=Hkv, head_dim=d, chunk_len=c, budget=max(4, n_c),
                     instr_len=n_i, dtype=api.BF16 if dtype == "bf16" else api.F32, cache_mode=api.CACHE_STANDARD,
                     lm_ordering=api.LM_EVICT_THEN_APPEND, cache_capacity=cap)
    ws = api.alloc_workspace(cfg)
    seed = 100 * case
    q, qi = rand((B, L, Hq, c, d), dt, seed + 1, s), rand((B, L, Hq, n_i, d), dt, seed + 2, s)
    kc, vc = rand((B, L, Hkv, cap, d), dt, seed + 3, s), rand((B, L, Hkv, cap, d), dt, seed + 4)
    k, v = rand((B, L, Hkv, c, d), dt, seed + 5, s), rand((B, L, Hkv, c, d), dt, seed + 6)
    lse = torch.empty((B, L, Hq, c), dtype=torch.float32, device=DEV)
    lm = torch.empty((B, L, Hkv, n_c + c), dtype=torch.float32, device=DEV)
    lse_c = torch.empty((B, L, Hq, c), dtype=torch.float32, device=DEV) if n_c > 0 else None
    out = api.citrus_chunk_attn(cfg, q, kc if n_c else None, vc if n_c else None, n_c, k, v, lse=lse, lm_score=lm,
                                workspace=ws, lse_cache=lse_c)
    sc = api.citrus_instr_score(cfg, qi, kc, n_c, k, workspace=ws)
    cs = api.citrus_cache_score(cfg, q, kc, n_c, workspace=ws) if n_c > 0 else None
    cs1 = api.citrus_cache_score(cfg, q, kc, n_c, lse_cache=lse_c) if n_c > 0 else None
    # one decoding step over the cache, in place on a copy
    kc2, vc2 = kc.clone(), vc.clone()
    dq, dk = rand((B, L, Hq, 1, d), dt, seed + 7, s), rand((B, L, Hkv, 1, d), dt, seed + 8, s)
    dv = rand((B, L, Hkv, 1, d), dt, seed + 9)
    dout = api.citrus_decode_step(cfg, dq, dk, dv, kc2, vc2, n_c, workspace=ws)
    torch.cuda.synchronize()
    for b in range(B):
        for l in range(L):
            kcat = np.concatenate([np64(kc[b, l, :, :n_c]), np64(k[b, l])], axis=1)
            vcat = np.concatenate([np64(vc[b, l, :, :n_c]), np64(v[b, l])], axis=1)
            o_ref, lse_ref, _ = orc.chunk_attn(np64(q[b, l]), kcat, vcat, n_c)
            assert_close(np64(out[b, l]), o_ref, dtype, "out")
            assert_close(np64(lse[b, l]), lse_ref, dtype, "lse")
            assert_close(np64(lm[b, l]), orc.lm_score(np64(q[b, l]), kcat, n_c), dtype, "lm_score")
            assert_close(np64(sc[b, l]), orc.instr_score(np64(qi[b, l]), kcat), dtype, "instr_score")
            if n_c > 0:
                ref = orc.instr_score(np64(q[b, l]), np64(kc[b, l, :, :n_c]))
                assert_close(np64(cs[b, l]), ref, dtype, "cache_score")
                assert_close(np64(cs1[b, l]), ref, dtype, "cache_score from the attention launch's normaliser")
            d_ref, _, _ = orc.decode_step(np64(dq[b, l, :, 0]), np64(dk[b, l, :, 0]), np64(dv[b, l, :, 0]),
                                          np64(kc[b, l, :, :n_c]), np64(vc[b, l, :, :n_c]))
            assert_close(np64(dout[b, l, :, 0]), d_ref, dtype, "decode")
    # the token's K/V row was appended behind the retained states, bit for bit
    assert torch.equal(kc2[:, :, :, n_c], dk[:, :, :, 0]) and torch.equal(vc2[:, :, :, n_c], dv[:, :, :, 0])
    assert torch.equal(kc2[:, :, :, :n_c], kc[:, :, :, :n_c])
