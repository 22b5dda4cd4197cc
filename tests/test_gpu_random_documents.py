"""The chunk loop over seeded random configurations: cache mode, ordering of the chunk-evicted cache, selection
granularity, accumulated scores, start size, position shift, GQA group, ragged document, chunk and budget sizes are
drawn together, so that combinations no hand-written case names are reached.  Each document is checked step by
step against the CPU oracle (teacher-forced, as the named cases are) and citrus_process_document against the same
steps issued one entry point at a time (bit-exact, with resume, a Python provider and a side stream).
A second family draws larger chunks, budgets and instructions (the sizes at which kernels change).
A failing case is named by its index.  Needs an MI355X."""

import numpy as np
import pytest

import paper_2406_12018_amd as api
from workloads import Workload

from test_gpu_parity import check_process_document_equals_stepwise, run_document_stepwise

pytestmark = pytest.mark.gpu
CASES = 48


def draw_workload(case):
    r = np.random.default_rng(9100 + case)
    bf16 = r.random() < 0.6
    d = 128 if (bf16 and r.random() < 0.8) else 64
    hkv = int(r.choice([1, 2, 4]))
    group = int(r.choice([1, 2, 4, 8]))
    chunk = int(r.choice([int(r.integers(1, 12)), int(r.integers(12, 70)), int(r.integers(70, 140))]))
    budget = int(r.choice([int(r.integers(2, 10)), int(r.integers(10, 90)), int(r.integers(90, 200))]))
    n_chunks = int(r.integers(2, 9))
    doc_len = max(2, chunk * n_chunks - int(r.integers(0, chunk)))
    mode = int(r.choice([api.CACHE_INSTR, api.CACHE_SHARED, api.CACHE_DUAL, api.CACHE_DUAL, api.CACHE_STANDARD]))
    kw = dict(cache_mode=mode, select_mode=int(r.integers(0, 2)))
    if mode in (api.CACHE_DUAL, api.CACHE_STANDARD):
        kw["lm_ordering"] = int(r.integers(0, 2))
    if mode == api.CACHE_DUAL:
        kw["budget_lm"] = int(r.choice([int(r.integers(2, 10)), int(r.integers(10, 120))]))
    if mode in (api.CACHE_INSTR, api.CACHE_SHARED) and r.random() < 0.4:
        kw["score_mode"] = api.SCORE_ACCUMULATED
    smallest = min(budget, kw.get("budget_lm", budget))
    if r.random() < 0.4 and smallest > 1:
        kw["start_size"] = int(r.integers(1, min(5, smallest)))
    if mode != api.CACHE_STANDARD and r.random() < 0.4:
        kw["position_shift"] = 1
    return Workload(f"random_{case}", "bf16" if bf16 else "f32", int(r.integers(1, 3)), int(r.integers(1, 3)), hkv * group, hkv,
                    d, doc_len, chunk, budget, int(r.integers(1, 25)), peaked=bool(r.random() < 0.5), seed=9100 + case, **kw)


@pytest.mark.parametrize("case", range(CASES))
def test_random_document(case):
    w = draw_workload(case)
    print(f"case {case}: {w}", flush=True)
    if w.cache_mode != api.CACHE_STANDARD:  # Standard CSE alone has a document test of its own form
        run_document_stepwise(w)
    check_process_document_equals_stepwise(w)


BIG_CASES = 16


def draw_big_workload(case):
    """Chunks to 640, budgets to 1600, up to 300 instruction rows: the sizes at which the scorer, the selection and
    the attention launcher change kernels, reached from inside the loop."""
    r = np.random.default_rng(77000 + case)
    bf16 = r.random() < 0.85
    d = 128 if (bf16 and r.random() < 0.9) else 64
    hkv = int(r.choice([1, 2]))
    group = int(r.choice([1, 2, 4, 8]))
    chunk = int(r.choice([64, 128, 192, 256, 320, 512, int(r.integers(33, 640))]))
    budget = int(r.choice([128, 256, 768, 1024, int(r.integers(100, 1600))]))
    n_chunks = int(r.integers(2, 6))
    doc_len = max(2, chunk * n_chunks - int(r.integers(0, chunk)))
    mode = int(r.choice([api.CACHE_INSTR, api.CACHE_DUAL, api.CACHE_DUAL, api.CACHE_STANDARD]))
    kw = dict(cache_mode=mode, select_mode=int(r.integers(0, 2)))
    if mode in (api.CACHE_DUAL, api.CACHE_STANDARD):
        kw["lm_ordering"] = int(r.integers(0, 2))
    if mode == api.CACHE_DUAL:
        kw["budget_lm"] = int(r.choice([96, 256, int(r.integers(50, 900))]))
    if mode == api.CACHE_INSTR and r.random() < 0.3:
        kw["score_mode"] = api.SCORE_ACCUMULATED
    if r.random() < 0.3:
        kw["start_size"] = int(r.integers(1, 5))
    if mode != api.CACHE_STANDARD and r.random() < 0.4:
        kw["position_shift"] = 1
    n_i = int(r.choice([16, 64, 128, 256, int(r.integers(1, 300))]))
    return Workload(f"random_big_{case}", "bf16" if bf16 else "f32", 1, int(r.integers(1, 3)), hkv * group, hkv, d, doc_len,
                    chunk, budget, n_i, peaked=bool(r.random() < 0.5), seed=77000 + case, **kw)


@pytest.mark.parametrize("case", range(BIG_CASES))
def test_random_big_document(case):
    w = draw_big_workload(case)
    print(f"big case {case}: {w}", flush=True)
    if w.cache_mode != api.CACHE_STANDARD:
        run_document_stepwise(w)
    check_process_document_equals_stepwise(w)

