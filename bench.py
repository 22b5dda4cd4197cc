#!/usr/bin/env python3
"""Benchmark of the CItruS chunk-eviction hot path on one MI355X.

One step = one whole document through citrus_process_document (chunk
attention, instruction score, top-k selection, K/V compaction for every chunk,
all layers and heads).  Inputs are synthetic, seeded, and resident in HBM before
the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]

    python bench.py --decode [--steps K] [--warmup W] [--workload NAME]
        a secondary measurement: K decoding steps (citrus_decode_step) over the cache the document loop
        leaves behind (budget + instr_len states, growing by one per step), as its own JSON line.
"""

from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_MFMA_TFLOPS = 2500.0   # MI355X dense bf16
PEAK_HBM_GBS = 8000.0

# HBM bytes per chunk-attention launch measured offline with rocprofv3 --pmc
# (FETCH_SIZE and WRITE_SIZE runs, scaled by a copy kernel of known size); see
# profiles/.  None until a measurement for that workload exists.
MEASURED_TRAFFIC_BYTES = {"cfg2_mistral7b": 562.0e6}


class HipEvents:
    """A flat array of hipEvent_t created through the HIP runtime (timing enabled)."""

    def __init__(self, count: int, wanted=None):
        """count slots; only slots i with wanted(i) true get an event, the others stay NULL (the library
        skips NULL entries: every recorded event costs a few microseconds of stream time)."""
        self.hip = C.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.hip.hipEventDestroy.argtypes = [C.c_void_p]
        self.arr = (C.c_void_p * count)()
        for i in range(count):
            if wanted is not None and not wanted(i):
                continue
            ev = C.c_void_p()
            rc = self.hip.hipEventCreate(C.byref(ev))
            if rc != 0:
                raise RuntimeError(f"hipEventCreate failed: {rc}")
            self.arr[i] = ev

    def elapsed_ms(self, i: int, j: int) -> float:
        ms = C.c_float()
        rc = self.hip.hipEventElapsedTime(C.byref(ms), self.arr[i], self.arr[j])
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
        return ms.value

    def destroy(self):
        for ev in self.arr:
            if ev:
                self.hip.hipEventDestroy(ev)


def attn_flops_per_launch(w, i: int, budget: int, holds_previous_chunk: bool = False) -> float:
    """Algorithmic (causal-masked) flops of chunk i's attention launch:
    4 * d * Hq * B * L * sum_t (n_c + t + 1).  A cache run in the evict-then-append order still holds the
    whole previous chunk next to its budget."""
    lo, hi = w.chunk_bounds(i)
    c = hi - lo
    if holds_previous_chunk:
        n_c = 0
        for j in range(i):
            n_c = min(n_c, budget) + (w.chunk_bounds(j)[1] - w.chunk_bounds(j)[0])
    else:
        n_c = w.cache_len_before(i, budget)
    return 4.0 * w.head_dim * w.q_heads * w.batch * w.layers * (c * n_c + c * (c + 1) / 2.0)


def cpu_baseline(w, target_seconds: float = 15.0):
    """The CPU oracle, as it stands, timed on steady-state chunk steps of one
    (document, layer) unit of the same workload; scaled to the metric's unit."""
    import numpy as np
    import torch
    from oracle import citrus_oracle as orc
    from workloads import make_chunk

    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    f64 = lambda t: t.to(torch.float64).numpy()
    first = min(w.n_chunks - 1, (w.budget + w.chunk_len - 1) // w.chunk_len)   # first steady-state chunk
    n_c = w.cache_len_before(first)
    rng = np.random.default_rng(0)
    ch = make_chunk(w, first, "cpu", b=[0], l=[0])
    # a steady-state cache: budget rows with the workload's plain value distribution
    kc = f64((torch.from_numpy(rng.standard_normal((w.kv_heads, n_c, w.head_dim))) * w.head_dim ** -0.5).to(w.torch_dtype))
    vc = f64((torch.from_numpy(rng.standard_normal((w.kv_heads, n_c, w.head_dim))) * w.head_dim ** -0.5).to(w.torch_dtype))
    q, k, v, qi = (f64(ch[x][0, 0]) for x in ("q", "k", "v", "q_instr"))
    steps, t0 = 0, time.perf_counter()
    while True:
        k_cat = np.concatenate([kc, k], axis=1)
        v_cat = np.concatenate([vc, v], axis=1)
        orc.chunk_attn(q, k_cat, v_cat, n_c)
        s = orc.instr_score(qi, k_cat)
        idx = orc.topk_select(s, w.budget)
        kc, vc = orc.kv_compact(k_cat, v_cat, idx)
        steps += 1
        dt = time.perf_counter() - t0
        if dt > target_seconds or steps >= 128:
            break
    per_unit_step = dt / steps                       # seconds per (document, layer) chunk step
    tok_s = w.chunk_len / (per_unit_step * w.batch * w.layers)
    return {"value": tok_s, "unit": "document tokens/s per layer-stack", "cores": threads, "kind": "oracle",
            "sample": f"{steps} steady-state chunk steps (cache {n_c} + chunk {w.chunk_len}) of one (document, layer) "
                      f"unit, {dt:.1f} s, scaled by batch*layers={w.batch * w.layers}; numpy float64, BLAS threads={threads}"}


def score_bytes_per_launch(w, i: int) -> float:
    """Algorithmic bytes of chunk i's instruction-score launch: every candidate key and every instruction query
    read once, the f32 scores written: ((n*Hkv + n_i*Hq)*d*e + 4*n*Hkv) * B * L."""
    e = 4 if w.dtype == "f32" else 2
    n = w.cache_len_before(i) + (w.chunk_bounds(i)[1] - w.chunk_bounds(i)[0])
    return float(w.batch * w.layers) * ((n * w.kv_heads + w.instr_len * w.q_heads) * w.head_dim * e + 4 * n * w.kv_heads)


def score_flops_per_launch(w, i: int) -> float:
    """Flops of Eq. (1) with the instruction as the text: one QK^T over the candidates, 2 * d * n_i * n * Hq * B * L."""
    n = w.cache_len_before(i) + (w.chunk_bounds(i)[1] - w.chunk_bounds(i)[0])
    return 2.0 * w.head_dim * w.instr_len * n * w.q_heads * w.batch * w.layers


def compact_bytes_per_launch(w, i: int) -> float:
    """Algorithmic bytes of chunk i's gather: the kept K and V rows read once and written once:
    4 * m * Hkv * d * e * B * L with m = min(k, n)."""
    e = 4 if w.dtype == "f32" else 2
    n = w.cache_len_before(i) + (w.chunk_bounds(i)[1] - w.chunk_bounds(i)[0])
    return float(w.batch * w.layers) * 4 * min(w.budget, n) * w.kv_heads * w.head_dim * e


def measured_peaks(torch, api, dev):
    """What this machine reaches on the two roofs, measured here and now: a plain 1 GiB device-to-device copy (read +
    write bytes per second) and a kernel of back-to-back bf16 MFMAs without memory traffic (citrus_probe_mfma)."""
    src = torch.empty(1 << 29, dtype=torch.bfloat16, device=dev).fill_(1.0)
    dst = torch.empty_like(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    best_copy = 0.0
    for it in range(4):
        e0.record()
        dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        if it > 0:
            best_copy = max(best_copy, 2.0 * src.numel() * 2 / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    del src, dst
    sink = torch.empty(1024 * 1024, dtype=torch.float32, device=dev)
    best_mfma = 0.0
    for it in range(4):
        e0.record()
        count = api.binding.probe_mfma(4000, sink)
        e1.record()
        torch.cuda.synchronize()
        if it > 0:
            best_mfma = max(best_mfma, count * 32768.0 / (e0.elapsed_time(e1) * 1e-3) / 1e12)
    return {"copy_GBs": round(best_copy, 1), "mfma_only_bf16_TFLOPs": round(best_mfma, 1),
            "note": "best of 3: 1 GiB device copy (read+write bytes); 16 waves per CU issuing independent 32x32x16 bf16 "
                    "MFMAs back to back, no memory traffic"}


def calibrate_copy(torch, dev):
    """A plain elementwise copy of known size (256 MiB read + 256 MiB written), three times: the reference
    for scaling rocprofv3's HBM counters."""
    src = torch.ones(128 * 1024 * 1024, dtype=torch.bfloat16, device=dev)
    dst = torch.empty_like(src)
    for _ in range(3):
        torch.add(src, 0, out=dst)
    torch.cuda.synchronize()
    del src, dst


def decode_mode(args, w, api, torch):
    """K decoding steps of one token (all layers) over budget + instr_len retained states."""
    dev = "cuda:0"
    n0 = w.budget + w.instr_len
    total = args.warmup + args.steps
    cfg = api.Config.from_workload(w, cache_capacity=n0 + total)
    ws = api.alloc_workspace(cfg, dev)
    g = torch.Generator(device="cpu").manual_seed(w.seed)
    mk = lambda shape, scale: (torch.randn(shape, generator=g) * scale).to(w.torch_dtype).to(dev)
    ksc = w.head_dim ** -0.25
    kc = mk((w.batch, w.layers, w.kv_heads, n0 + total, w.head_dim), ksc)
    vc = mk((w.batch, w.layers, w.kv_heads, n0 + total, w.head_dim), 1.0)
    # a few distinct tokens, cycled
    toks = [(mk((w.batch, w.layers, w.q_heads, 1, w.head_dim), ksc), mk((w.batch, w.layers, w.kv_heads, 1, w.head_dim), ksc),
             mk((w.batch, w.layers, w.kv_heads, 1, w.head_dim), 1.0)) for _ in range(4)]
    out = torch.empty_like(toks[0][0])
    torch.cuda.synchronize()
    if args.calibrate_copy:
        calibrate_copy(torch, dev)
    for i in range(args.warmup):
        q, kn, vn = toks[i % 4]
        api.citrus_decode_step(cfg, q, kn, vn, kc, vc, n0 + i, out=out, workspace=ws)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(args.warmup, total):
        q, kn, vn = toks[i % 4]
        api.citrus_decode_step(cfg, q, kn, vn, kc, vc, n0 + i, out=out, workspace=ws)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    dev_ms = e0.elapsed_time(e1) / args.steps
    esize = 4 if w.dtype == "f32" else 2
    n_avg = n0 + args.warmup + (args.steps - 1) / 2.0 + 1      # states read per step, the token's own included
    byt = w.batch * w.layers * esize * w.head_dim * (2 * w.kv_heads * n_avg + 2 * w.q_heads + 4 * w.kv_heads)
    print(json.dumps({
        "metric": "decoding steps/s over the retained cache (one token through all layers)",
        "value": round(1e3 / wall_ms, 1), "unit": "steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name + " decode", "batch": w.batch, "layers": w.layers, "q_heads": w.q_heads,
                   "kv_heads": w.kv_heads, "head_dim": w.head_dim, "cache_states": n0, "grows_by": 1},
        "roofline": {"kernel": "decode_attn_kernel", "bound": "hbm", "achieved": round(byt / (dev_ms * 1e-3) / 1e9, 1),
                     "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(byt / (dev_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                     "traffic": None, "avg_launch_ms": round(dev_ms, 5), "algorithmic_bytes_per_launch": byt},
    }), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg2_mistral7b")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--position-shift", action="store_true",
                    help="treat the synthetic tensors as un-rotated and apply the position shift (rotary embedding "
                         "at cache positions) in every step")
    ap.add_argument("--decode", action="store_true",
                    help="measure decoding steps over the retained cache instead of the document loop")
    ap.add_argument("--cache-mode", choices=["instr", "shared", "dual", "standard"], default=None,
                    help="override the workload's cache design (dual needs a workload with budget_lm)")
    ap.add_argument("--lm-ordering", choices=["score-after-append", "evict-then-append"], default=None,
                    help="override how the chunk-evicted cache of dual / standard is run")
    ap.add_argument("--layers", type=int, default=0,
                    help="override the workload's layer count (e.g. 1: the small launches of a model whose layers "
                         "run one after the other)")
    ap.add_argument("--ring", type=int, default=0,
                    help="stream the document through a ring of this many pre-staged chunk buffers (a provider "
                         "callback cycles through them) instead of keeping the whole document resident; chosen "
                         "automatically when the resident document would not fit")
    ap.add_argument("--overlap", action="store_true",
                    help="single-cache modes: run selection and gather next to the chunk attention on a second stream "
                         "(2-3 %% more tokens/s; the attention launch itself then shares the chip and takes 9 %% longer)")
    ap.add_argument("--graph", action="store_true",
                    help="record one document's launches into a HIP graph and time its replays (resident documents); "
                         "the chunk-attention launch duration then comes from untimed eager documents")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch a plain elementwise copy of known size (256 MiB read + 256 MiB written) three "
                         "times before the warm-up, as the reference for scaling rocprofv3 HBM counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2406_12018_amd as api
    from workloads import WORKLOADS, make_chunk, make_document

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the hot path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = WORKLOADS[args.workload]
    if args.decode:
        decode_mode(args, w, api, torch)
        return
    mode_names = ["instr", "shared", "dual", "standard"]
    if args.cache_mode is not None or args.lm_ordering is not None or args.position_shift or args.layers > 0:
        from dataclasses import replace
        over = {"position_shift": 1} if args.position_shift else {}
        if args.layers > 0:
            over["layers"] = args.layers
        if args.cache_mode is not None:
            over["cache_mode"] = mode_names.index(args.cache_mode)
        if args.lm_ordering is not None:
            over["lm_ordering"] = ["score-after-append", "evict-then-append"].index(args.lm_ordering)
        w = replace(w, **over)
        if w.cache_mode == api.CACHE_DUAL and w.budget_lm < 1:
            w = replace(w, budget_lm=w.budget)
    cfg = api.Config.from_workload(w)
    dual = w.cache_mode == api.CACHE_DUAL
    standard = w.cache_mode == api.CACHE_STANDARD
    chunk_evicted = dual or standard            # a cache evicted by the document's own chunks exists
    paper_order = chunk_evicted and w.lm_ordering == api.LM_EVICT_THEN_APPEND

    esize = 4 if w.dtype == "f32" else 2
    resident_bytes = esize * w.head_dim * w.batch * w.layers * (
        2 * w.q_heads * w.doc_len + 2 * w.kv_heads * w.doc_len + w.q_heads * w.instr_len * w.n_chunks)
    ring = args.ring if args.ring > 0 else (0 if resident_bytes < 150e9 else 2)
    state = api.DocumentState.allocate(cfg, dev)
    ws = api.alloc_workspace(cfg, dev)
    if ring == 0:
        doc = make_document(w, dev)
        out = torch.empty_like(doc["q"])
        rd = api.resident_doc(cfg, doc["q"], doc["k"], doc["v"], doc["q_instr"], out)
        provider = None
    else:
        # pre-staged ring of chunk buffers (inputs of chunks 0..ring-1 of the same recipe, generated in
        # slices to bound temporaries); chunk i is served from slot i % ring, generation is outside the timing
        slots = []
        for i in range(min(ring, w.n_chunks)):
            slot = {"q": torch.empty((w.batch, w.layers, w.q_heads, w.chunk_len, w.head_dim), dtype=w.torch_dtype, device=dev),
                    "k": torch.empty((w.batch, w.layers, w.kv_heads, w.chunk_len, w.head_dim), dtype=w.torch_dtype, device=dev),
                    "q_instr": torch.empty((w.batch, w.layers, w.q_heads, w.instr_len, w.head_dim), dtype=w.torch_dtype, device=dev)}
            slot["v"] = torch.empty_like(slot["k"])
            slot["out"] = torch.empty_like(slot["q"])
            per_layer = w.q_heads * w.chunk_len * w.head_dim
            lg = max(1, min(w.layers, (1 << 27) // per_layer))
            for b in range(w.batch):
                for l0 in range(0, w.layers, lg):
                    ls = list(range(l0, min(w.layers, l0 + lg)))
                    part = make_chunk(w, i, dev, b=[b], l=ls)
                    for name in ("q", "k", "v", "q_instr"):
                        slot[name][b:b + 1, l0:l0 + len(ls)] = part[name]
                    del part
            slots.append({name: (t, api.binding.tensor(t)) for name, t in slot.items()})
        rd = None

        def provider(i, io):
            if i >= w.n_chunks:
                return 1
            sl = slots[i % len(slots)]
            io.q, io.k, io.v, io.q_instr, io.out = sl["q"][1], sl["k"][1], sl["v"][1], sl["q_instr"][1], sl["out"][1]
            io.chunk_len = w.chunk_bounds(i)[1] - w.chunk_bounds(i)[0]
            return 0
    torch.cuda.synchronize()

    E = api.binding.EVENTS_PER_STEP
    # timed region: only the two events that bracket the chunk-attention launch of every step; the
    # per-phase breakdown comes from one more, untimed, document with all events
    # Single-cache modes: a step's selection and gather run on a second stream next to its chunk attention
    # (the library then scores the instruction first; events 5 and 1 bracket the attention launch).
    overlap = args.overlap and not dual and not standard
    side = api.SideStream(dev) if overlap else None
    attn_begin = 5 if overlap else 0
    events = HipEvents(args.steps * w.n_chunks * E, wanted=lambda i: i % E in (attn_begin, 1))
    phase_events = HipEvents(w.n_chunks * E)

    def one_document(ev_offset=None, ev=None):
        ev = events if ev is None else ev
        state.cache_len = state.cache_len_lm = 0
        state.buffer_index = state.buffer_index_lm = 0
        pe = None
        if ev_offset is not None:
            pe = C.cast(C.byref(ev.arr, ev_offset * C.sizeof(C.c_void_p)), C.c_void_p)
        done = api.citrus_process_document(cfg, state, ws, doc=rd, provider=provider, phase_events=pe, side=side)
        assert done == w.n_chunks

    if args.calibrate_copy:
        calibrate_copy(torch, dev)

    graph = None
    if args.graph:
        if ring != 0:
            print("bench.py: --graph takes a resident document (no --ring)", file=sys.stderr)
            sys.exit(2)
        # the library allocates nothing and never synchronises, so a document's launches can be recorded as they
        # are; one eager document first (it raises the kernels' dynamic-LDS limits, which a capture must not do)
        capture_stream = torch.cuda.Stream()
        with torch.cuda.stream(capture_stream):
            one_document()
        capture_stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=capture_stream):
            one_document()

    for _ in range(args.warmup):
        graph.replay() if graph else one_document()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        graph.replay() if graph else one_document(s * w.n_chunks * E)
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens = w.batch * w.doc_len
    value = tokens / (ms_per_step * 1e-3)
    # untimed: all eight events of every step, over a few documents (per-phase times and the launch durations
    # of the instruction score and the gather)
    PHASE_DOCS = 3 if ms_per_step < 100.0 else 1
    phase_sets = [phase_events] + [HipEvents(w.n_chunks * E) for _ in range(PHASE_DOCS - 1)]
    for pe_set in phase_sets:
        one_document(0, pe_set)
    torch.cuda.synchronize()

    # chunk-attention launch durations from the events recorded inside the timed region
    attn_ms, attn_fl = [], []
    for s in range(0 if graph else args.steps):
        for i in range(w.n_chunks):
            base = (s * w.n_chunks + i) * E
            attn_ms.append(events.elapsed_ms(base + attn_begin, base + 1))
            attn_fl.append(attn_flops_per_launch(w, i, w.budget_lm if dual else w.budget, paper_order))
    if graph:  # no events inside the replayed graph: the untimed eager documents bracket the same launch (0 -> 1)
        for pe_set in phase_sets:
            for i in range(w.n_chunks):
                attn_ms.append(pe_set.elapsed_ms(i * E + attn_begin, i * E + 1))
                attn_fl.append(attn_flops_per_launch(w, i, w.budget_lm if dual else w.budget, paper_order))
    events.destroy()
    # per-phase device time of the extra document
    names = {1: "chunk_attn", 2: "lm_score", 3: "lm_select", 4: "lm_compact", 5: "instr_score", 6: "select", 7: "compact"}
    phase_ms = {v: 0.0 for v in names.values()}
    # launch durations of the instruction score (events 4 -> 5; 0 -> 5 with --overlap) and of the gather
    # (6 -> 7), every chunk of the untimed documents, with the algorithmic bytes of the same launches
    score_ms, score_by, compact_ms, compact_by, select_ms = [], [], [], [], []
    if not standard:
        for pe_set in phase_sets:
            for i in range(w.n_chunks):
                score_ms.append(pe_set.elapsed_ms(i * E + (0 if overlap else 4), i * E + 5))
                score_by.append(score_bytes_per_launch(w, i))
                select_ms.append(pe_set.elapsed_ms(i * E + 5, i * E + 6))
                compact_ms.append(pe_set.elapsed_ms(i * E + 6, i * E + 7))
                compact_by.append(compact_bytes_per_launch(w, i))
    for pe_set in phase_sets[1:]:
        pe_set.destroy()
    for i in range(w.n_chunks):
        if overlap:
            # order on the main stream: 0 step start, instruction score, 5, chunk attention, 1; on the side
            # stream, behind event 5: selection, 6, gather, 7 (these two phases run next to the attention)
            for name, (e0, e1) in {"instr_score": (0, 5), "chunk_attn": (5, 1), "select": (5, 6), "compact": (6, 7)}.items():
                phase_ms[name] += phase_events.elapsed_ms(i * E + e0, i * E + e1)
            continue
        for p, name in names.items():
            if (not chunk_evicted and p in (2, 3, 4)) or (standard and p in (5, 6, 7)):
                continue
            phase_ms[name] += phase_events.elapsed_ms(i * E + p - 1, i * E + p)
    phase_events.destroy()
    phase_ms = {k: round(v, 4) for k, v in phase_ms.items()
                if (chunk_evicted or not k.startswith("lm_")) and not (standard and k in ("instr_score", "select", "compact"))}
    avg_ms = sum(attn_ms) / len(attn_ms)
    avg_fl = sum(attn_fl) / len(attn_fl)
    achieved = avg_fl / (avg_ms * 1e-3) / 1e12
    overridden = args.cache_mode is not None or args.lm_ordering is not None or args.position_shift or args.layers > 0
    traffic = None if overridden else MEASURED_TRAFFIC_BYTES.get(w.name)

    def hbm_entry(kernel, step, ms, by, note=None):
        a_ms, a_by = sum(ms) / len(ms), sum(by) / len(by)
        gbs = a_by / (a_ms * 1e-3) / 1e9
        e = {"kernel": kernel, "step": step, "bound": "hbm", "algorithmic_bytes_per_launch": a_by,
             "avg_launch_ms": round(a_ms, 5), "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
             "frac": round(gbs / PEAK_HBM_GBS, 4)}
        if note:
            e["note"] = note
        return e

    roofline_other = []
    if score_ms:
        # which roof bounds the instruction score depends on the shape: flops of Eq. (1) per byte it must move
        sc_flops = sum(score_flops_per_launch(w, i) for i in range(w.n_chunks)) / w.n_chunks
        ent = hbm_entry("instr_score kernels (instruction score)", "a2", score_ms, score_by,
                        "launch duration = HIP events around the instruction-score launch(es) of every chunk of "
                        f"{PHASE_DOCS} untimed documents (includes the event gap of a few microseconds)")
        a_ms = sum(score_ms) / len(score_ms)
        ent["algorithmic_flops_per_launch"] = sc_flops
        ent["achieved_TFLOPs"] = round(sc_flops / (a_ms * 1e-3) / 1e12, 1)
        ent["frac_of_bf16_mfma_peak"] = round(sc_flops / (a_ms * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS, 4)
        ent["frac_of_hbm_peak"] = ent["frac"]
        # the roof that bounds it: flops per algorithmic byte against the machine balance (312 flop per byte)
        if sc_flops / ent["algorithmic_bytes_per_launch"] > PEAK_BF16_MFMA_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
            ent.update(bound="mfma", achieved=ent["achieved_TFLOPs"], peak=PEAK_BF16_MFMA_TFLOPS, unit="TFLOP/s",
                       frac=ent["frac_of_bf16_mfma_peak"])
        roofline_other.append(ent)
        roofline_other.append(hbm_entry("compact_kernel (K/V gather)", "a4", compact_ms, compact_by,
                                        "same events, around the gather launch"))
        roofline_other.append({"kernel": "topk_regs{6,8,24}_kernel / topk_kernel (selection)", "step": "a3", "bound": "latency",
                               "avg_launch_ms": round(sum(select_ms) / len(select_ms), 5),
                               "note": "a chain of barrier-separated LDS passes over a few KB per unit: no roofline fraction"})

    # the same fractions against what this machine reaches in this run (a device copy, an MFMA-only loop)
    peaks = measured_peaks(torch, api, dev)
    for ent in roofline_other:
        if "achieved" in ent:
            reached = peaks["mfma_only_bf16_TFLOPs"] if ent["unit"] == "TFLOP/s" else peaks["copy_GBs"]
            ent["frac_of_measured_peak"] = round(ent["achieved"] / reached, 4) if reached > 0 else None

    result = {
        "metric": "document tokens/sec per layer-stack + % HBM/MFMA peak, Mistral-7B shape",
        "value": round(value, 1), "unit": "document tokens/s per layer-stack",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "layers": w.layers, "q_heads": w.q_heads,
                   "kv_heads": w.kv_heads, "head_dim": w.head_dim, "doc_len": w.doc_len, "chunk_len": w.chunk_len,
                   "budget": w.budget, "instr_len": w.instr_len,
                   "cache_mode": mode_names[w.cache_mode],
                   "lm_ordering": ["score_after_append", "evict_then_append"][w.lm_ordering] if chunk_evicted else None,
                   "select": "per_kv_head", "position_shift": bool(w.position_shift),
                   "inputs": "resident document" if ring == 0 else
                   f"ring of {ring} pre-staged chunk buffers holding chunks 0..{ring - 1} of the recipe, replayed for the whole "
                   "document (dense timing; not the document's own values)",
                   "streams": "selection + gather next to the chunk attention on a second stream" if overlap else "one",
                   "launch": "one HIP graph per document, replayed" if graph else "eager"},
        "roofline": {"kernel": ("attn_pipe_kernel_w8_rotq + the rope launches of the step (the events bracket both)"
                                if w.position_shift else "attn_pipe_kernel_w8 (chunk attention)"), "bound": "mfma",
                     "achieved": round(achieved, 2), "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / PEAK_BF16_MFMA_TFLOPS, 4),
                     "frac_of_measured_peak": (round(achieved / peaks["mfma_only_bf16_TFLOPs"], 4)
                                               if peaks["mfma_only_bf16_TFLOPs"] > 0 else None),
                     "traffic": traffic,
                     "traffic_source": None if traffic is None else
                     "constant from an offline rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE run of this command "
                     "(profiles/bench_cfg2_mistral7b_hbm_traffic.md), not measured in this run",
                     "avg_launch_ms": round(avg_ms, 5), "algorithmic_flops_per_launch": avg_fl},
        "roofline_other": roofline_other,
        "peaks_measured": peaks,
        "phase_ms_per_step": phase_ms,
        "phase_note": "phases: one extra untimed document with all events; roofline: events around every chunk-attention "
                      + ("launch of the untimed eager documents (the timed region replays a graph without events)" if graph
                         else "launch of the timed region") + ("; select and compact run concurrently with chunk_attn (their times "
                                                      "are not additive)" if overlap else ""),
    }
    if not args.no_cpu_baseline and not overridden:
        # (the baseline times the default step sequence; it is not reported for overridden designs)
        result["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
