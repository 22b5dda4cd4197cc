"""citrus_evict_cache_static (scratch in the library's static device array, nothing allocated) against
citrus_evict_cache (caller's workspace): same kernels, so every output must agree bit for bit.  Each case
makes two calls in a row, the second on a smaller input, so that the array still holds the first call's
partial sums, scores and positions when the second one runs.  Needs an MI355X."""

import pytest
import torch

import paper_2406_12018_amd as api

pytestmark = pytest.mark.gpu
DEV = "cuda"


def rand(shape, dtype, seed, scale=1.0):
    g = torch.Generator(device="cpu").manual_seed(seed)
    return (torch.randn(shape, generator=g, dtype=torch.float32) * scale).to(dtype).to(DEV)


def one_call(dtype, B, L, Hq, Hkv, d, rows, n, k, seed, per_layer=False, explicit_idx=True, start_size=0):
    """Both entry points on the same inputs; returns nothing, asserts bit equality."""
    print(f"evict_cache_static {dtype} B{B} L{L} {Hq}/{Hkv} d{d} rows{rows} n{n} k{k} per_layer={per_layer} "
          f"idx={'given' if explicit_idx else 'scratch'}", flush=True)
    t = torch.float32 if dtype == "f32" else torch.bfloat16
    cfg = api.Config(batch=B, layers=L, q_heads=Hq, kv_heads=Hkv, head_dim=d, chunk_len=64, budget=k, instr_len=rows,
                     dtype=api.F32 if dtype == "f32" else api.BF16, cache_capacity=max(n, k), start_size=start_size,
                     select_mode=api.SELECT_PER_LAYER if per_layer else api.SELECT_PER_KV_HEAD)
    q = rand((B, L, Hq, rows, d), t, seed, 1.5)
    kc, vc = rand((B, L, Hkv, n, d), t, seed + 1, 1.5 * d ** -0.5), rand((B, L, Hkv, n, d), t, seed + 2)
    ws = api.alloc_workspace(cfg, DEV)
    hs = cfg.sel_heads
    m = min(k, n)
    k_ref, v_ref = torch.full((B, L, Hkv, k, d), 7.0, dtype=t, device=DEV), torch.full((B, L, Hkv, k, d), 7.0, dtype=t, device=DEV)
    k_new, v_new = torch.full_like(k_ref, 7.0), torch.full_like(v_ref, 7.0)
    idx_ref = torch.full((B, L, hs, k), -1, dtype=torch.int32, device=DEV)
    idx_new = torch.full_like(idx_ref, -1) if explicit_idx else None
    assert api.citrus_evict_cache(cfg, q, kc, vc, n, k, k_ref, v_ref, idx=idx_ref, workspace=ws) == m
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    assert api.citrus_evict_cache_static(cfg, q, kc, vc, n, k, k_new, v_new, idx=idx_new) == m
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(k_new, k_ref) and torch.equal(v_new, v_ref)
    if explicit_idx:
        assert torch.equal(idx_new, idx_ref)
    # the reference itself did something: m rows written, the rest untouched, positions ascending
    assert (k_ref[:, :, :, m:] == 7.0).all() and not (k_ref[:, :, :, :m] == 7.0).all()
    assert (idx_ref[..., 1:m] > idx_ref[..., :m - 1]).all()


CASES = {
    # bf16 d=128: two-launch scorer (384 query rows per KV group: partial (max, sum) pairs in the scratch), then
    # the one-launch scorer on a smaller input
    "bf16_two_launch_then_fused": [dict(dtype="bf16", B=2, L=3, Hq=8, Hkv=2, d=128, rows=96, n=1100, k=700, seed=1),
                                   dict(dtype="bf16", B=1, L=2, Hq=8, Hkv=2, d=128, rows=24, n=333, k=200, seed=2)],
    # Mistral-7B-shaped final eviction by the instruction (as after a document), then a smaller cache
    "bf16_cfg2_shape_then_smaller": [dict(dtype="bf16", B=1, L=32, Hq=32, Hkv=8, d=128, rows=64, n=832, k=768, seed=3),
                                     dict(dtype="bf16", B=1, L=8, Hq=32, Hkv=8, d=128, rows=64, n=800, k=300, seed=4,
                                          explicit_idx=False)],
    # generic kernels (f32, d=64), layer-wise selection, positions kept in the scratch
    "f32_generic_per_layer": [dict(dtype="f32", B=2, L=2, Hq=4, Hkv=2, d=64, rows=8, n=200, k=64, seed=5, per_layer=True,
                                   explicit_idx=False, start_size=4),
                              dict(dtype="f32", B=1, L=1, Hq=4, Hkv=2, d=64, rows=3, n=70, k=33, seed=6, per_layer=True)],
    # a cache that already fits: copied whole, no score is computed
    "bf16_cache_fits": [dict(dtype="bf16", B=1, L=2, Hq=4, Hkv=4, d=128, rows=16, n=500, k=400, seed=7),
                        dict(dtype="bf16", B=1, L=2, Hq=4, Hkv=4, d=128, rows=16, n=100, k=400, seed=8)],
}


@pytest.mark.parametrize("case", list(CASES), ids=list(CASES))
def test_evict_cache_static_equals_evict_cache_twice_in_a_row(case):
    assert api.static_scratch_bytes() == 16 << 20
    for kw in CASES[case]:
        one_call(**kw)


def test_evict_cache_static_refuses_what_does_not_fit():
    cfg = api.Config(batch=4, layers=32, q_heads=32, kv_heads=8, head_dim=128, chunk_len=64, budget=768, instr_len=128,
                     dtype=api.BF16, cache_capacity=832)
    q = torch.zeros((4, 32, 32, 128, 128), dtype=torch.bfloat16, device=DEV)
    kc = torch.zeros((4, 32, 8, 832, 128), dtype=torch.bfloat16, device=DEV)
    kn = torch.zeros((4, 32, 8, 768, 128), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(api.CitrusError) as e:
        api.citrus_evict_cache_static(cfg, q, kc, kc.clone(), 832, 768, kn, kn.clone())
    assert e.value.status == api.binding.ERR_WORKSPACE
