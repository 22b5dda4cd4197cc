"""The C-ABI library loads, exports every symbol the header declares, and turns
bad arguments into error codes on the host without touching a device.  CPU only."""

import ctypes as C
import os
import re

import pytest

from paper_2406_12018_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "citrus.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(citrus_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B._lib()
    names = declared_symbols()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None
    header = open(os.path.join(ROOT, "include", "citrus.h")).read()
    assert B.abi_version() == int(re.search(r"#define\s+CITRUS_ABI_VERSION\s+(\d+)", header).group(1)) == 10


def test_struct_layouts_match_the_header():
    assert C.sizeof(B.CConfig) == 19 * 4
    assert C.sizeof(B.CTensor) == 5 * 8
    assert C.sizeof(B.CChunkIO) == 5 * 40 + 8
    assert C.sizeof(B.CResidentDoc) == 5 * 40 + 8 + 16


def cfg(**kw):
    base = dict(batch=1, layers=1, q_heads=4, kv_heads=2, head_dim=64, chunk_len=32, budget=64, instr_len=8, dtype=B.F32)
    base.update(kw)
    return B.Config(**base)


def test_status_strings():
    for s in range(7):
        assert B.status_string(s) not in ("", "unknown status")
    assert B.status_string(99) == "unknown status"


@pytest.mark.parametrize("kw,ok", [
    ({}, True), ({"q_heads": 3}, False), ({"head_dim": 96}, False), ({"budget": 0}, False), ({"dtype": 7}, False),
    ({"cache_mode": B.CACHE_DUAL}, False), ({"cache_mode": B.CACHE_DUAL, "budget_lm": 16}, True),
    ({"cache_capacity": 8}, False), ({"softmax_scale": -1.0}, False), ({"select_mode": 5}, False),
    ({"batch": 70000}, False), ({"lm_ordering": 2}, False),
    # the largest launch (8 workgroups per 32 rows of every head) has to stay a 31-bit grid
    ({"batch": 64, "layers": 1000, "q_heads": 4096, "kv_heads": 512, "chunk_len": 64}, False),
    ({"batch": 64, "layers": 1000, "q_heads": 2048, "kv_heads": 512, "chunk_len": 64}, True),
    ({"cache_mode": B.CACHE_DUAL, "budget_lm": 16, "lm_ordering": B.LM_EVICT_THEN_APPEND}, True),
    # the evict-then-append cache keeps a whole chunk beside the budget
    ({"cache_mode": B.CACHE_DUAL, "budget_lm": 48, "lm_ordering": B.LM_EVICT_THEN_APPEND, "cache_capacity": 64}, False),
    ({"cache_mode": B.CACHE_STANDARD}, True), ({"cache_mode": B.CACHE_STANDARD, "lm_ordering": B.LM_EVICT_THEN_APPEND}, True),
    ({"cache_mode": B.CACHE_STANDARD, "lm_ordering": B.LM_EVICT_THEN_APPEND, "cache_capacity": 64}, False),
    ({"cache_mode": 4}, False), ({"score_mode": B.SCORE_ACCUMULATED}, True), ({"score_mode": 2}, False),
    ({"score_mode": B.SCORE_ACCUMULATED, "cache_mode": B.CACHE_STANDARD}, False),
    ({"position_shift": 1}, True), ({"position_shift": 2}, False), ({"position_shift": 1, "rope_base": 0.5}, False),
    ({"position_shift": 1, "rope_base": 1e6}, True), ({"position_shift": 1, "cache_mode": B.CACHE_STANDARD}, False),
    ({"score_mode": B.SCORE_ACCUMULATED, "cache_mode": B.CACHE_DUAL, "budget_lm": 16}, False),
    ({"position_shift": 1, "cache_mode": B.CACHE_DUAL, "budget_lm": 16}, True),
    ({"position_shift": 1, "cache_mode": B.CACHE_DUAL, "budget_lm": 16, "lm_ordering": B.LM_EVICT_THEN_APPEND}, True),
])
def test_workspace_bytes_validates_config(kw, ok):
    assert (B.workspace_bytes(cfg(**kw)) > 0) == ok


def test_workspace_never_shrinks_when_the_configuration_grows():
    """A call may use any cache length up to the capacity and the entry points that take `rows` any row count
    up to the configured one, and the scorer picks its kernel by the call's own shape: a workspace sized for a
    larger configuration must cover every smaller call.  (A size that followed only the largest shape once
    dropped the single-product scorer's partial sums at 2561 candidates and left the 2560-candidate call
    writing past its block.)"""
    base = dict(batch=1, layers=1, q_heads=8, kv_heads=1, head_dim=128, chunk_len=64, budget=64, instr_len=64, dtype=B.BF16)
    sizes = [B.workspace_bytes(cfg(**base, cache_capacity=cap)) for cap in range(64, 3200, 13)]
    assert all(b >= a for a, b in zip(sizes, sizes[1:]))
    by_rows = [B.workspace_bytes(cfg(**{**base, "instr_len": r}, cache_capacity=2496)) for r in range(1, 700, 7)]
    assert all(b >= a for a, b in zip(by_rows, by_rows[1:]))
    # the block of the 2560-candidate call: 16 strips x 2 partial columns x 2560 floats
    need = 16 * 2 * 2560 * 4
    assert B.workspace_bytes(cfg(**base, cache_capacity=2496)) >= need
    assert B.workspace_bytes(cfg(**base, cache_capacity=2499)) >= need


def fake(ptr=0x1000, s=64):
    return B.CTensor(ptr, s * 1024, s * 512, s * 128, s)


def test_entry_points_reject_bad_arguments_before_any_launch():
    lib = B._lib()
    c = cfg().c()
    null = B.CTensor(None, 0, 0, 0, 0)
    ws = C.c_void_p(0x10000)
    big = 1 << 30
    # NULL config
    assert lib.citrus_chunk_attn(None, fake(), fake(), fake(), 0, fake(), fake(), 8, fake(), None, None, None, None, 0, None) == B.ERR_NULL
    # NULL q
    assert lib.citrus_chunk_attn(C.byref(c), null, fake(), fake(), 0, fake(), fake(), 8, fake(), None, None, None, None, 0, None) == B.ERR_NULL
    # NULL cache with cache_len > 0
    assert lib.citrus_chunk_attn(C.byref(c), fake(), null, null, 4, fake(), fake(), 8, fake(), None, None, None, None, 0, None) == B.ERR_NULL
    # chunk_len out of range, cache_len above capacity
    assert lib.citrus_chunk_attn(C.byref(c), fake(), fake(), fake(), 0, fake(), fake(), 33, fake(), None, None, None, None, 0, None) == B.ERR_SHAPE
    assert lib.citrus_chunk_attn(C.byref(c), fake(), fake(), fake(), 65, fake(), fake(), 8, fake(), None, None, None, None, 0, None) == B.ERR_SHAPE
    # misaligned pointer / stride
    assert lib.citrus_chunk_attn(C.byref(c), fake(0x1004), fake(), fake(), 0, fake(), fake(), 8, fake(), None, None, None, None, 0, None) == B.ERR_SHAPE
    assert lib.citrus_chunk_attn(C.byref(c), fake(s=66), fake(), fake(), 0, fake(), fake(), 8, fake(), None, None, None, None, 0, None) == B.ERR_SHAPE
    # lm_score without lse needs a workspace
    assert lib.citrus_chunk_attn(C.byref(c), fake(), fake(), fake(), 0, fake(), fake(), 8, fake(), None, None, C.c_void_p(0x2000), None, 0, None) == B.ERR_WORKSPACE
    # instr_score: NULL score, missing / short workspace
    assert lib.citrus_instr_score(C.byref(c), fake(), fake(), 0, fake(), 8, None, ws, big, None) == B.ERR_NULL
    assert lib.citrus_instr_score(C.byref(c), fake(), fake(), 0, fake(), 8, C.c_void_p(0x2000), None, 0, None) == B.ERR_WORKSPACE
    assert lib.citrus_instr_score(C.byref(c), fake(), fake(), 0, fake(), 8, C.c_void_p(0x2000), ws, 16, None) == B.ERR_WORKSPACE
    # topk: NULLs, n/k < 1
    assert lib.citrus_topk_select(C.byref(c), None, 8, 4, C.c_void_p(0x2000), None, 0, None) == B.ERR_NULL
    assert lib.citrus_topk_select(C.byref(c), C.c_void_p(0x2000), 0, 4, C.c_void_p(0x3000), None, 0, None) == B.ERR_SHAPE
    assert lib.citrus_topk_select(C.byref(c), C.c_void_p(0x2000), 8, 0, C.c_void_p(0x3000), None, 0, None) == B.ERR_SHAPE
    # compact: NULL idx, m out of range, pitch < m, destination aliasing a source
    assert lib.citrus_kv_compact(C.byref(c), fake(), fake(), 4, fake(), fake(), 8, None, 8, 8, fake(0x9000), fake(0xA000), None) == B.ERR_NULL
    assert lib.citrus_kv_compact(C.byref(c), fake(), fake(), 4, fake(), fake(), 8, C.c_void_p(0x2000), 8, 0, fake(0x9000), fake(0xA000), None) == B.ERR_SHAPE
    assert lib.citrus_kv_compact(C.byref(c), fake(), fake(), 4, fake(), fake(), 8, C.c_void_p(0x2000), 4, 8, fake(0x9000), fake(0xA000), None) == B.ERR_SHAPE
    assert lib.citrus_kv_compact(C.byref(c), fake(), fake(), 4, fake(), fake(), 8, C.c_void_p(0x2000), 8, 8, fake(), fake(0xA000), None) == B.ERR_SHAPE
    # start_size must leave room for at least one scored state
    for bad_start in (-1, cfg().budget):
        bs = cfg(start_size=bad_start).c()
        assert lib.citrus_topk_select(C.byref(bs), C.c_void_p(0x2000), 8, 4, C.c_void_p(0x3000), None, 0, None) == B.ERR_SHAPE
    # cache_score: the rows must fit the workspace (instr_len rows, or chunk_len rows for a configuration
    # that runs a cache in the evict-then-append order)
    sc = C.c_void_p(0x2000)
    assert lib.citrus_cache_score(C.byref(c), fake(), 9, fake(), 8, None, sc, ws, big, None) == B.ERR_SHAPE
    for mode_kw in (dict(cache_mode=B.CACHE_DUAL, budget_lm=16), dict(cache_mode=B.CACHE_STANDARD)):
        e = cfg(lm_ordering=B.LM_EVICT_THEN_APPEND, **mode_kw).c()
        assert lib.citrus_cache_score(C.byref(e), null, 8, fake(), 8, None, sc, ws, big, None) == B.ERR_NULL
        assert lib.citrus_cache_score(C.byref(e), fake(), 8, fake(), 8, None, None, ws, big, None) == B.ERR_NULL
        assert lib.citrus_cache_score(C.byref(e), fake(), 0, fake(), 8, None, sc, ws, big, None) == B.ERR_SHAPE
        assert lib.citrus_cache_score(C.byref(e), fake(), 33, fake(), 8, None, sc, ws, big, None) == B.ERR_SHAPE
        assert lib.citrus_cache_score(C.byref(e), fake(), 8, fake(), 0, None, sc, ws, big, None) == B.ERR_SHAPE
        assert lib.citrus_cache_score(C.byref(e), fake(), 8, fake(), 97, None, sc, ws, big, None) == B.ERR_SHAPE
        assert lib.citrus_cache_score(C.byref(e), fake(), 8, fake(), 8, None, sc, None, 0, None) == B.ERR_WORKSPACE
        assert lib.citrus_cache_score(C.byref(e), fake(), 8, fake(), 8, None, sc, ws, 16, None) == B.ERR_WORKSPACE
    # a given normaliser makes the workspace unnecessary; a cache-only normaliser needs a cache
    assert lib.citrus_cache_score(C.byref(c), null, 8, fake(), 8, C.c_void_p(0x7000), sc, None, 0, None) == B.ERR_NULL
    assert lib.citrus_chunk_attn(C.byref(c), fake(), fake(), fake(), 0, fake(), fake(), 8, fake(), None, C.c_void_p(0x7000),
                                 None, None, 0, None) == B.ERR_SHAPE
    # evict_cache: rows as above, k within the budget, destinations distinct from the sources
    ev = lambda cc, rows=8, n=40, k=16, kn=fake(0x9000), vn=fake(0xA000), w=ws, wb=big: lib.citrus_evict_cache(
        C.byref(cc), fake(), rows, fake(0x5000), fake(0x6000), n, k, kn, vn, None, w, wb, None)
    assert ev(c, rows=9) == B.ERR_SHAPE
    assert ev(c, n=0) == B.ERR_SHAPE and ev(c, n=65) == B.ERR_SHAPE
    assert ev(c, k=0) == B.ERR_SHAPE and ev(c, k=65) == B.ERR_SHAPE
    assert ev(c, kn=fake(0x5000)) == B.ERR_SHAPE and ev(c, vn=fake(0x6000)) == B.ERR_SHAPE
    assert ev(c, kn=null) == B.ERR_NULL
    assert ev(c, w=None, wb=0) == B.ERR_WORKSPACE
    # decode_step: the cache needs a free row; the token's tensors must not be the cache itself
    dec = lambda n=8, kn=fake(0x7000), w=ws, wb=big, qq=fake(): lib.citrus_decode_step(
        C.byref(c), qq, kn, fake(0x8000), fake(0x5000), fake(0x6000), n, fake(0x9000), w, wb, None)
    assert dec(n=-1) == B.ERR_SHAPE and dec(n=64) == B.ERR_SHAPE
    assert dec(kn=fake(0x5000)) == B.ERR_SHAPE
    assert dec(qq=null) == B.ERR_NULL
    assert dec(w=None, wb=0) == B.ERR_WORKSPACE
    # accumulated scores: NULLs, lengths
    p1, p2, p3 = C.c_void_p(0x2000), C.c_void_p(0x3000), C.c_void_p(0x4000)
    assert lib.citrus_score_accumulate(C.byref(c), None, 8, p2, 4, None) == B.ERR_NULL
    assert lib.citrus_score_accumulate(C.byref(c), p1, 8, None, 4, None) == B.ERR_NULL
    assert lib.citrus_score_accumulate(C.byref(c), p1, 0, p2, 0, None) == B.ERR_SHAPE
    assert lib.citrus_score_accumulate(C.byref(c), p1, 97, p2, 4, None) == B.ERR_SHAPE
    assert lib.citrus_score_accumulate(C.byref(c), p1, 8, p2, 9, None) == B.ERR_SHAPE
    assert lib.citrus_score_accumulate(C.byref(c), p1, 90, p2, 65, None) == B.ERR_SHAPE
    assert lib.citrus_score_gather(C.byref(c), p1, 8, None, 4, 4, p3, None) == B.ERR_NULL
    assert lib.citrus_score_gather(C.byref(c), p1, 8, p2, 4, 0, p3, None) == B.ERR_SHAPE
    assert lib.citrus_score_gather(C.byref(c), p1, 8, p2, 3, 4, p3, None) == B.ERR_SHAPE
    assert lib.citrus_score_gather(C.byref(c), p1, 8, p2, 80, 65, p3, None) == B.ERR_SHAPE
    # rope: heads, rows, positions
    assert lib.citrus_rope(C.byref(c), null, 4, 8, 0, fake(), None) == B.ERR_NULL
    assert lib.citrus_rope(C.byref(c), fake(), 0, 8, 0, fake(), None) == B.ERR_SHAPE
    assert lib.citrus_rope(C.byref(c), fake(), 4, -1, 0, fake(), None) == B.ERR_SHAPE
    assert lib.citrus_rope(C.byref(c), fake(), 4, 8, -1, fake(), None) == B.ERR_SHAPE
    assert lib.citrus_rope(C.byref(c), fake(), 4, 0, 0, fake(), None) == B.OK      # nothing to do, nothing launched
    # unsupported head_dim
    bad = cfg(head_dim=96).c()
    assert lib.citrus_topk_select(C.byref(bad), C.c_void_p(0x2000), 8, 4, C.c_void_p(0x3000), None, 0, None) == B.ERR_UNSUPPORTED


def test_process_document_validation_and_provider_protocol():
    lib = B._lib()
    c = cfg().c()
    two = (B.CTensor * 2)(fake(0x10000), fake(0x20000))
    two_v = (B.CTensor * 2)(fake(0x30000), fake(0x40000))
    same = (B.CTensor * 2)(fake(0x10000), fake(0x10000))
    n_c, cur, done = C.c_int32(0), C.c_int32(0), C.c_int32(-1)
    ws, big = C.c_void_p(0x100000), 1 << 30
    calls = []

    def provider(_u, i, _s, _io):
        calls.append(i)
        return 1          # "no more chunks" before anything would be launched

    cb = B.PROVIDER(provider)
    fn = C.cast(cb, C.c_void_p)
    run = lambda **o: lib.citrus_process_document(
        o.get("cfg", C.byref(c)), o.get("fn", fn), None, o.get("first", 3), -1, o.get("k", two), two_v, None, None,
        C.byref(o.get("n_c", n_c)), None, C.byref(cur), None, o.get("acc", None), None, None, C.byref(done), None,
        o.get("ws", ws),
        o.get("ws_bytes", big), None, o.get("side", None))
    assert run() == B.OK and calls == [3] and done.value == 0
    # a side stream needs its stream and both events
    half_side = B.CSideStream(C.c_void_p(0x70000), C.c_void_p(0x71000), None)
    assert run(side=C.byref(half_side)) == B.ERR_NULL
    full_side = B.CSideStream(C.c_void_p(0x70000), C.c_void_p(0x71000), C.c_void_p(0x72000))
    assert run(side=C.byref(full_side)) == B.OK
    assert run(fn=None) == B.ERR_NULL
    assert run(k=same) == B.ERR_SHAPE
    assert run(n_c=C.c_int32(65)) == B.ERR_SHAPE
    assert run(first=-1) == B.ERR_SHAPE
    assert run(ws=None) == B.ERR_WORKSPACE
    assert run(ws_bytes=100) == B.ERR_WORKSPACE
    # accumulated scores need their two buffers
    ca = cfg(score_mode=B.SCORE_ACCUMULATED).c()
    assert run(cfg=C.byref(ca)) == B.ERR_NULL
    same_acc = (C.c_void_p * 2)(0x50000, 0x50000)
    assert run(cfg=C.byref(ca), acc=same_acc) == B.ERR_SHAPE
    assert run(cfg=C.byref(ca), acc=(C.c_void_p * 2)(0x50000, 0x60000)) == B.OK
    # a provider that aborts
    cb2 = B.PROVIDER(lambda _u, i, _s, _io: -5)
    assert run(fn=C.cast(cb2, C.c_void_p)) == B.ERR_PROVIDER
    # a provider that hands over an invalid chunk length: rejected before any launch
    def bad_len(_u, i, _s, io):
        io.contents.chunk_len = 1000
        return 0
    cb3 = B.PROVIDER(bad_len)
    assert run(fn=C.cast(cb3, C.c_void_p)) == B.ERR_SHAPE
    # DUAL needs the LM buffers
    d = cfg(cache_mode=B.CACHE_DUAL, budget_lm=32).c()
    assert run(cfg=C.byref(d)) == B.ERR_NULL


def test_resident_provider_slices_the_document():
    lib = B._lib()
    doc = B.CResidentDoc(fake(0x100000), fake(0x200000), fake(0x300000), fake(0x400000), fake(0x500000),
                         4096, 70, 32, B.BF16)
    io = B.CChunkIO()
    assert lib.citrus_resident_provider(C.byref(doc), 0, None, C.byref(io)) == 0 and io.chunk_len == 32
    assert io.q.ptr == 0x100000 and io.q_instr.ptr == 0x500000
    assert lib.citrus_resident_provider(C.byref(doc), 2, None, C.byref(io)) == 0 and io.chunk_len == 6
    assert io.k.ptr == 0x200000 + 64 * 64 * 2 and io.out.ptr == 0x400000 + 64 * 64 * 2
    assert io.q_instr.ptr == 0x500000 + 2 * 4096 * 2
    assert lib.citrus_resident_provider(C.byref(doc), 3, None, C.byref(io)) == 1
    assert lib.citrus_resident_provider(None, 0, None, C.byref(io)) < 0


def test_unit_span_of_two_gib_or_more_is_rejected_before_any_launch():
    """The kernels address the rows of one (b, l, h) unit with 32-bit byte offsets: every entry point refuses a
    tensor whose touched rows span 2 GiB or more, on the host."""
    lib = B._lib()
    c = cfg(dtype=B.BF16, head_dim=128, chunk_len=512, budget=768, instr_len=64).c()
    wide = lambda rows: B.CTensor(0x1000, 1 << 40, 1 << 38, 1 << 36, (((1 << 31) // 2 - 128) // (rows - 1)) // 8 * 8 + 8)
    ok = lambda rows: B.CTensor(0x1000, 1 << 40, 1 << 38, 1 << 36, (((1 << 31) // 2 - 128) // (rows - 1)) // 8 * 8 - 8)
    attn = lambda q, kc: lib.citrus_chunk_attn(C.byref(c), q, kc, fake(), 0, fake(), fake(), 512, fake(), None, None,
                                                None, None, 0, None)
    assert attn(wide(512), fake()) == B.ERR_SHAPE
    assert attn(B.CTensor(0x1000, 0, 0, 0, 1 << 31), fake()) == B.ERR_SHAPE
    # the same stride is fine for fewer rows: the bound is on what the call touches (checked up to the next
    # validation step, which needs no device either: a missing workspace)
    sc, ws = C.c_void_p(0x2000), C.c_void_p(0x10000)
    score = lambda qi: lib.citrus_instr_score(C.byref(c), qi, fake(), 0, fake(), 8, sc, None, 0, None)
    assert score(wide(64)) == B.ERR_SHAPE
    assert score(ok(64)) == B.ERR_WORKSPACE
    assert lib.citrus_kv_compact(C.byref(c), fake(), fake(), 4, fake(), fake(), 8, C.c_void_p(0x2000), 768, 768,
                                 wide(768), fake(0xA000), None) == B.ERR_SHAPE
    assert lib.citrus_rope(C.byref(c), wide(100), 4, 100, 0, fake(), None) == B.ERR_SHAPE


def test_evict_cache_static_validates_like_evict_cache_and_bounds_its_scratch():
    lib = B._lib()
    assert B.static_scratch_bytes() == 16 << 20
    c = cfg().c()
    null = B.CTensor(None, 0, 0, 0, 0)
    ev = lambda cc, rows=8, n=40, k=16, kn=fake(0x9000), vn=fake(0xA000), q=fake(): lib.citrus_evict_cache_static(
        C.byref(cc), q, rows, fake(0x5000), fake(0x6000), n, k, kn, vn, None, None)
    assert lib.citrus_evict_cache_static(None, fake(), 8, fake(), fake(), 40, 16, fake(), fake(), None, None) == B.ERR_NULL
    assert ev(c, rows=0) == B.ERR_SHAPE
    assert ev(c, n=0) == B.ERR_SHAPE and ev(c, n=65) == B.ERR_SHAPE
    assert ev(c, k=0) == B.ERR_SHAPE and ev(c, k=65) == B.ERR_SHAPE
    assert ev(c, kn=fake(0x5000)) == B.ERR_SHAPE and ev(c, vn=fake(0x6000)) == B.ERR_SHAPE
    assert ev(c, kn=null) == B.ERR_NULL and ev(c, q=null) == B.ERR_NULL
    # a request beyond the fixed array is refused on the host: 64 B per query row alone is 32 MiB here
    big = cfg(dtype=B.BF16, head_dim=128, batch=4, layers=32, q_heads=32, kv_heads=8, chunk_len=512, budget=768,
              instr_len=128).c()
    assert lib.citrus_evict_cache_static(C.byref(big), fake(), 128, fake(0x5000), fake(0x6000), 768, 700, fake(0x9000),
                                         fake(0xA000), None, None) == B.ERR_WORKSPACE


def test_concurrent_host_threads_get_the_same_codes():
    """Entry points keep no unsynchronised state: many threads validating at once all see the codes a single
    thread sees."""
    import threading
    lib = B._lib()
    c = cfg().c()
    null = B.CTensor(None, 0, 0, 0, 0)
    sc, ws = C.c_void_p(0x2000), C.c_void_p(0x10000)

    def calls():
        return [
            lib.citrus_chunk_attn(C.byref(c), null, fake(), fake(), 0, fake(), fake(), 8, fake(), None, None, None, None, 0, None),
            lib.citrus_chunk_attn(C.byref(c), fake(), fake(), fake(), 65, fake(), fake(), 8, fake(), None, None, None, None, 0, None),
            lib.citrus_instr_score(C.byref(c), fake(), fake(), 0, fake(), 8, sc, ws, 16, None),
            lib.citrus_topk_select(C.byref(c), sc, 0, 4, C.c_void_p(0x3000), None, 0, None),
            lib.citrus_evict_cache_static(C.byref(c), fake(), 8, fake(0x5000), fake(0x6000), 40, 0, fake(0x9000), fake(0xA000), None, None),
            lib.citrus_rope(C.byref(c), fake(), 4, 0, 0, fake(), None),
            int(lib.citrus_workspace_bytes(C.byref(c)) > 0),
        ]

    expected = calls()
    assert expected == [B.ERR_NULL, B.ERR_SHAPE, B.ERR_WORKSPACE, B.ERR_SHAPE, B.ERR_SHAPE, B.OK, 1]
    results, errors = [], []

    def worker():
        try:
            for _ in range(200):
                results.append(calls())
        except Exception as e:  # pragma: no cover
            errors.append(e)

    threads = [threading.Thread(target=worker) for _ in range(8)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors and len(results) == 1600 and all(r == expected for r in results)
