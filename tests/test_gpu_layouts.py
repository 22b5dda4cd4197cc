"""The C ABI takes element strides: every entry point gives the same bits on token-major tensors
(storage [B, L, S, H, d], passed as a [B, L, H, S, d] view with stride_h = d) and on views with unused
elements around every axis (all NaN: never read, never written) as on head-major ones, whose results the
other GPU tests check against the oracle.  Needs an MI355X."""

import pytest
import torch

import paper_2406_12018_amd as api

pytestmark = pytest.mark.gpu
DEV = "cuda"


def rand(shape, dt, seed, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(shape, generator=g) * scale).to(dt).to(DEV)


def token_major(t):
    """Same values, storage order [B, L, S, H, d]."""
    return t.permute(0, 1, 3, 2, 4).contiguous().permute(0, 1, 3, 2, 4)


class Padded:
    """Same values inside a larger allocation: every axis has unused elements in front of and behind the view
    (rows stay 16-byte aligned), all of them NaN.  A kernel that read them would poison its results; one that
    wrote them is caught by untouched()."""

    def __init__(self):
        self.made = []

    def __call__(self, t):
        B, L, H, S, d = t.shape
        big = torch.full((B + 1, L + 2, H + 3, S + 5, d + 24), float("nan"), dtype=t.dtype, device=t.device)
        view = big[1:, 1:L + 1, 2:H + 2, 3:S + 3, 8:8 + d]
        view.copy_(t)
        self.made.append((big, view))
        return view

    def untouched(self):
        for big, view in self.made:
            mask = torch.ones(big.shape, dtype=torch.bool, device=big.device)
            B, L, H, S, d = view.shape
            mask[1:, 1:L + 1, 2:H + 2, 3:S + 3, 8:8 + d] = False
            if not bool(torch.isnan(big[mask]).all()):
                return False
        return True


@pytest.mark.parametrize("dtype,d,Hq,Hkv,c,n_c,n_i", [("bf16", 128, 8, 2, 200, 320, 40), ("bf16", 128, 4, 4, 65, 0, 7),
                                                     ("bf16", 64, 4, 2, 50, 77, 9), ("f32", 64, 4, 1, 33, 40, 5)])
def test_token_major_equals_head_major(dtype, d, Hq, Hkv, c, n_c, n_i):
    print(f"layouts {dtype} d{d} Hq{Hq} Hkv{Hkv} c{c} n_c{n_c} n_i{n_i}", flush=True)
    dt = torch.bfloat16 if dtype == "bf16" else torch.float32
    B, L = 2, 2
    cap = n_c + c + 4
    cfg = api.Config(batch=B, layers=L, q_heads=Hq, kv_heads=Hkv, head_dim=d, chunk_len=c, budget=max(4, n_c),
                     instr_len=n_i, dtype=api.BF16 if dtype == "bf16" else api.F32, cache_mode=api.CACHE_STANDARD,
                     lm_ordering=api.LM_EVICT_THEN_APPEND, cache_capacity=cap)
    ws = api.alloc_workspace(cfg)
    s = d ** -0.25
    q, qi = rand((B, L, Hq, c, d), dt, 1, s), rand((B, L, Hq, n_i, d), dt, 2, s)
    kc, vc = rand((B, L, Hkv, cap, d), dt, 3, s), rand((B, L, Hkv, cap, d), dt, 4)
    k, v = rand((B, L, Hkv, c, d), dt, 5, s), rand((B, L, Hkv, c, d), dt, 6)
    dq0, dk0, dv0 = rand((B, L, Hq, 1, d), dt, 7, s), rand((B, L, Hkv, 1, d), dt, 8, s), rand((B, L, Hkv, 1, d), dt, 9)
    m = min(n_c + c, 37)
    idx = torch.arange(0, 2 * m, 2, dtype=torch.int32, device=DEV).clamp(max=n_c + c - 1).repeat(B, L, Hkv, 1).contiguous()
    results = []
    padded = Padded()
    for layout in (lambda t: t, token_major, padded):
        Q, QI, KC, VC, K, V = layout(q), layout(qi), layout(kc.clone()), layout(vc.clone()), layout(k), layout(v)
        lse = torch.empty((B, L, Hq, c), dtype=torch.float32, device=DEV)
        lm = torch.empty((B, L, Hkv, n_c + c), dtype=torch.float32, device=DEV)
        lse_c = torch.empty((B, L, Hq, c), dtype=torch.float32, device=DEV) if n_c >= 32 and n_c % 32 == 0 else None
        out = layout(torch.zeros_like(q))
        api.citrus_chunk_attn(cfg, Q, KC if n_c else None, VC if n_c else None, n_c, K, V, out=out, lse=lse, lm_score=lm,
                              workspace=ws, lse_cache=lse_c)
        sc = api.citrus_instr_score(cfg, QI, KC, n_c, K, workspace=ws)
        cs = api.citrus_cache_score(cfg, Q, KC, n_c, workspace=ws) if n_c else None
        kn = layout(torch.zeros((B, L, Hkv, m, d), dtype=dt, device=DEV))
        vn = layout(torch.zeros((B, L, Hkv, m, d), dtype=dt, device=DEV))
        api.citrus_kv_compact(cfg, KC, VC, n_c, K, V, idx, m, kn, vn)
        dout = api.citrus_decode_step(cfg, layout(dq0), layout(dk0), layout(dv0), KC, VC, n_c, workspace=ws)
        y = layout(torch.zeros_like(k))
        api.citrus_rope(cfg, K, 5, y=y)
        torch.cuda.synchronize()
        results.append(dict(out=out.contiguous(), lse=lse, lm_score=lm, instr_score=sc, cache_score=cs, k_new=kn.contiguous(),
                            v_new=vn.contiguous(), decode_out=dout.contiguous(), rope=y.contiguous(),
                            cache_after_decode=KC.contiguous()[:, :, :, :n_c + 1]))
    for name, a in results[0].items():
        if a is not None:
            assert torch.equal(a, results[1][name]), name
            assert torch.equal(a, results[2][name]), f"{name} (padded strides)"
    assert padded.untouched(), "elements outside a padded view were written"
