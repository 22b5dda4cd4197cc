"""The synthetic input generator: deterministic, sliceable, right statistics. CPU only."""

import torch

from workloads import WORKLOADS, gen_tensor, heavy_mask, make_chunk, make_chunk_sliced, make_document, peaked, scaled_down


def test_named_workloads_match_their_shapes():
    w = WORKLOADS["cfg2_mistral7b"]
    assert (w.batch, w.layers, w.q_heads, w.kv_heads, w.head_dim) == (1, 32, 32, 8, 128)
    assert (w.doc_len, w.chunk_len, w.budget, w.instr_len, w.n_chunks) == (16384, 512, 768, 64, 32)
    assert WORKLOADS["cfg1_tiny_f32"].n_chunks == 16
    assert WORKLOADS["cfg5_large"].group == 8
    assert w.cache_len_before(0) == 0 and w.cache_len_before(1) == 512 and w.cache_len_before(2) == 768


def test_document_is_deterministic_and_sliceable():
    w = WORKLOADS["cfg1_tiny_f32"]
    d1, d2 = make_document(w), make_document(w)
    for key in d1:
        assert torch.equal(d1[key], d2[key])
    ch = make_chunk(w, 3)
    lo, hi = w.chunk_bounds(3)
    assert torch.equal(ch["k"], d1["k"][:, :, :, lo:hi])
    assert torch.equal(ch["q_instr"], d1["q_instr"][3])
    one = gen_tensor(w, "q", [100, 7], h=[2])
    assert torch.equal(one[0, 0, 0, 0], d1["q"][0, 0, 2, 100]) and torch.equal(one[0, 0, 0, 1], d1["q"][0, 0, 2, 7])
    assert not torch.equal(d1["q_instr"][0], d1["q_instr"][1])


def test_value_recipe():
    w = scaled_down(WORKLOADS["cfg2_mistral7b"], layers=2, doc_len=4096)
    d = make_document(w)
    assert d["q"].dtype == torch.bfloat16
    s = w.head_dim ** 0.5
    assert abs(d["q"].double().std().item() * s - 1.0) < 0.01
    assert abs(d["v"].double().std().item() * s - 1.0) < 0.01
    assert abs(d["v"].double().mean().item()) < 1e-3
    hm = heavy_mask(w, [0], range(w.doc_len), "cpu")[0]
    assert 0.01 < hm.float().mean().item() < 0.03 and not hm[:4].any()
    k = d["k"].double()
    assert abs(k[:, :, :, :4].std().item() * s - 4.0) < 0.2
    assert abs(k[:, :, :, hm].std().item() * s - 2.5) < 0.1
    plain = ~hm
    plain[:4] = False
    assert abs(k[:, :, :, plain].std().item() * s - 1.0) < 0.01
    # heavy hitters are per position, shared by layers and heads
    ratio = (k[:, :, :, hm].abs().mean(dim=(0, 4)) * s)
    assert ratio.min() > 1.5


def test_peaked_variant_leaves_logit_inputs_unscaled():
    w = peaked(WORKLOADS["cfg1_tiny_f32"])
    d = make_document(w)
    assert abs(d["q"].double().std().item() - 1.0) < 0.02
    assert abs(d["v"].double().std().item() * 8 - 1.0) < 0.02


def test_sliced_chunk_generation_gives_the_same_values():
    w = scaled_down(WORKLOADS["cfg2_mistral7b"], batch=2, layers=3, q_heads=4, kv_heads=2, doc_len=300, chunk_len=64,
                    instr_len=8)
    for i in (0, 4):   # a full chunk and the short last one
        whole = make_chunk(w, i)
        parts = make_chunk_sliced(w, i, max_elems=4 * 64 * 128 * 2)   # two layers per slice
        for name in whole:
            assert torch.equal(whole[name], parts[name])
        sub = make_chunk_sliced(w, i, b=[1], l=[2, 0], max_elems=1)
        assert torch.equal(sub["k"][0, 0], whole["k"][1, 2]) and torch.equal(sub["q"][0, 1], whole["q"][1, 0])
