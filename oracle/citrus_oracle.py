"""CPU oracle for the CItruS chunk-eviction hot path (arXiv 2406.12018).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition the HIP
library is checked against.  Nothing in the product path may import it: only
tests, the smoke check and the benchmark's cpu_baseline leg do.  It shares no
code with the HIP path and never reads a value the HIP path produced.

Everything is computed in float64 with numpy.  Inputs are whatever values the
caller hands over (for bf16 runs: the bf16-rounded values widened exactly to
float64); no result is rounded back to a narrower type.

What each function follows in the paper:

* ``softmax_rows``, ``chunk_attn``: step 1 of the Standard CSE process
  (Section 4.1, "Overall process"): encode the chunk given the cache, i.e.
  ordinary causal softmax attention with the 1/sqrt(d_k) scaling that Eq. (1)
  writes out.
* ``instr_score``: Eq. (1) with the instruction text I in the role of the
  chunk s (Section 4.2, Imp(I, c^I) for the individual cache and Imp(I, c)
  for the shared cache).
* ``lm_score``: Eq. (1) with the document chunk itself as s (Section 4.1).
* ``topk_select``: Eq. (2)-(3), the k highest importance scores form the
  selection set; layer-wise granularity is the last paragraph of Section 4.1.
* ``kv_compact``: Eq. (3)/(5), the evicted cache keeps exactly the selected
  states.
* ``process_document``: the chunk loop of Section 4.1 / 4.3 with the cache
  designs of Section 4.2 (individual, shared) and the dual form
  (language-modelling cache next to the instruction cache).
* ``evict_cache``: one eviction of a cache by a text (Section 4.1 step 2, and
  the extra eviction by the instruction after the last chunk that the same
  paragraph describes): Eq. (1) over the cache states alone, Eq. (2)-(3).
* ``standard_cse``: the Standard CSE process of Section 4.1 on its own (one
  cache, evicted by the document chunks), ending with that extra eviction.
* ``rope`` and ``position_shift`` in ``process_document``: the position shift
  mechanism of Section 5.3 ("Hyperparameters"): the cache always uses the same
  positional embeddings, i.e. a state's position is its slot in the cache, not
  its place in the document.  Keys are kept without rotary embedding and are
  rotated by their slot index whenever they are attended to.
* ``decode_step``: one step of generating the response from the retained
  states (Section 4.3): the new token's state joins the cache and its query
  attends over all of it, the same softmax attention as in Eq. (1).

Readings taken where the paper is silent (all listed again in the design
notes of the repository):

* Eq. (1) has a mean over the chunk's tokens; the functions here return the
  SUM over tokens and over the query heads that share a KV head.  The mean is
  that sum divided by a constant, so the selection is unchanged, and the sum
  has a checkable total mass (rows x heads).
* Query head h reads KV head h // G (contiguous groups, G = Hq / Hkv).
* The softmax of Eq. (1) runs over all candidate states [cache ; chunk]: the
  chunk's states are appended first and the eviction then keeps k of the
  n = n_c + c candidates.  For an instruction-scored cache this is the
  paper's evict-then-append order hoisted by one step.
* Instruction rows carry no causal mask (the instruction follows the whole
  document) and the instruction's own keys are not part of the softmax.
* Ties: the lower index wins; retained states keep ascending original order.
* n <= k keeps every candidate (the first chunk enters the cache whole).

Pins (tests/test_oracle_pins.py): softmax rows sum to one; total score mass;
budget >= document length reproduces one-shot full causal attention
(cross-checked against torch's scaled_dot_product_attention on the CPU);
selection against a brute-force pure-Python ordering, with duplicates; the
closed forms for Q_I = 0, all-equal keys and a dominant key; the TOVA special
case (chunk of one token); a hand-computed two-key example stored under
tests/golden/.  Parity of Imp values or selected sets on real text is
unpinned: it needs trained weights and the paper's datasets.
"""

from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

LM_SCORE_AFTER_APPEND = 0   # the chunk's own causal attention scores [LM cache ; chunk] right away
LM_EVICT_THEN_APPEND = 1    # Section 4.1 as printed: evict the cache by the chunk's attention to it, then append

SCORE_PER_STEP = 0      # Eq. (1) of the current step decides (the paper's method)
SCORE_ACCUMULATED = 1   # the sum of the scores a state received since it entered the cache decides (H2O's rule)

SELECT_PER_KV_HEAD = 0
SELECT_PER_LAYER = 1

CACHE_INSTR = 0
CACHE_SHARED = 1
CACHE_DUAL = 2


def _f64(x) -> np.ndarray:
    return np.asarray(x, dtype=np.float64)


def softmax_rows(logits: np.ndarray, valid: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Row softmax (the fraction inside Eq. (1)).

    ``logits`` is [rows, n]; ``valid`` an optional boolean [rows, n] mask of the
    states a row may see (False entries get probability exactly 0).  Returns
    (p, lse) with p [rows, n] and lse [rows] = log sum_j exp(logit_j) over the
    valid entries.
    """
    s = _f64(logits)
    if valid is not None:
        s = np.where(valid, s, -np.inf)
    m = np.max(s, axis=1, keepdims=True)
    e = np.exp(s - m)
    z = np.sum(e, axis=1, keepdims=True)
    return e / z, (m + np.log(z))[:, 0]


def _scale(d: int, scale: Optional[float]) -> float:
    return 1.0 / math.sqrt(d) if (scale is None or scale == 0.0) else float(scale)


def _causal_valid(c: int, n_c: int, n: int) -> np.ndarray:
    """Row t of the chunk sees every cache state and chunk states 0..t."""
    j = np.arange(n)[None, :]
    t = np.arange(c)[:, None]
    return j <= (n_c + t)


def rope(x, positions, base: float = 10000.0) -> np.ndarray:
    """Rotary position embedding in the convention of the Llama / Mistral
    models the paper runs (pairs (i, i + d/2); angle = position * base^(-2i/d)).

    x [H, S, d]; positions [S] (any integers or floats).  Returns the rotated
    array: y_i = x_i cos - x_{i+d/2} sin,  y_{i+d/2} = x_{i+d/2} cos + x_i sin.
    """
    x = _f64(x)
    h, s_len, d = x.shape
    half = d // 2
    pos = np.asarray(positions, dtype=np.float64).reshape(s_len)
    inv_freq = base ** (-np.arange(half, dtype=np.float64) * 2.0 / d)
    ang = pos[:, None] * inv_freq[None, :]               # [S, d/2]
    cos, sin = np.cos(ang)[None], np.sin(ang)[None]
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * cos - hi * sin, hi * cos + lo * sin], axis=-1)


def chunk_attn(q, k_cat, v_cat, n_c: int, scale: Optional[float] = None):
    """Encode a chunk given the cache (Section 4.1, step 1).

    q [Hq, c, d]; k_cat, v_cat [Hkv, n, d] with n = n_c + c: the first n_c
    rows are the retained cache, the rest the chunk's own states.  Row t
    attends to cache rows 0..n_c-1 and chunk rows 0..t.

    Returns (out [Hq, c, d], lse [Hq, c], probs [Hq, c, n]).
    """
    q, k_cat, v_cat = _f64(q), _f64(k_cat), _f64(v_cat)
    hq, c, d = q.shape
    hkv, n, _ = k_cat.shape
    assert n == n_c + c and hq % hkv == 0
    g_size = hq // hkv
    sc = _scale(d, scale)
    valid = _causal_valid(c, n_c, n)
    out = np.zeros((hq, c, d))
    lse = np.zeros((hq, c))
    probs = np.zeros((hq, c, n))
    for h in range(hq):
        g = h // g_size
        logits = (q[h] @ k_cat[g].T) * sc
        p, l = softmax_rows(logits, valid)
        probs[h] = p
        lse[h] = l
        out[h] = p @ v_cat[g]
    return out, lse, probs


def instr_score(q_instr, k_cat, scale: Optional[float] = None) -> np.ndarray:
    """Instruction-aware importance, summed form of Eq. (1) with s = I.

    q_instr [Hq, n_i, d]; k_cat [Hkv, n, d].  score[g, j] = sum over the query
    heads h of group g and over the instruction rows u of
    softmax_j(q_instr[h, u] . k_cat[g, j] / sqrt(d)).  No mask.
    Imp(I, c_j) = score[g, j] / (n_i * G).
    """
    q_instr, k_cat = _f64(q_instr), _f64(k_cat)
    hq, n_i, d = q_instr.shape
    hkv, n, _ = k_cat.shape
    assert hq % hkv == 0
    g_size = hq // hkv
    sc = _scale(d, scale)
    score = np.zeros((hkv, n))
    for h in range(hq):
        g = h // g_size
        p, _ = softmax_rows((q_instr[h] @ k_cat[g].T) * sc)
        score[g] += p.sum(axis=0)
    return score


def lm_score(q, k_cat, n_c: int, scale: Optional[float] = None) -> np.ndarray:
    """Chunk-scored importance, summed form of Eq. (1) with s = the chunk.

    Uses the same causal probabilities as ``chunk_attn`` (masked entries count
    as zero).  score[g, j] = sum_{h in g} sum_t p[h, t, j].
    """
    q = _f64(q)
    k_cat = _f64(k_cat)
    hq, c, d = q.shape
    hkv, n, _ = k_cat.shape
    g_size = hq // hkv
    sc = _scale(d, scale)
    valid = _causal_valid(c, n_c, n)
    score = np.zeros((hkv, n))
    for h in range(hq):
        g = h // g_size
        p, _ = softmax_rows((q[h] @ k_cat[g].T) * sc, valid)
        score[g] += p.sum(axis=0)
    return score


def topk_select_1d(score: np.ndarray, k: int, start_size: int = 0) -> np.ndarray:
    """Eq. (2)-(3) for one score vector: positions of the min(k, n) highest
    scores, ties to the lower index, returned in ascending position order.

    ``start_size`` > 0 is the variant of the appendix "Analysis on initial
    tokens": the first start_size candidates are always preserved and the
    remaining k - start_size places go to the best of the others."""
    score = np.asarray(score)
    n = score.shape[0]
    if n <= k:
        return np.arange(n, dtype=np.int64)
    s0 = min(start_size, k)
    # stable sort on the negated score: equal scores keep ascending index order
    order = s0 + np.argsort(-score[s0:], kind="stable")
    return np.sort(np.concatenate([np.arange(s0), order[:k - s0]])).astype(np.int64)


def topk_select(score, k: int, select_mode: int = SELECT_PER_KV_HEAD, start_size: int = 0) -> np.ndarray:
    """score [Hkv, n] -> idx [Hkv, min(k, n)] (per KV head) or [1, min(k, n)]
    (layer-wise: the scores of all heads are added first, Section 4.1 last
    paragraph)."""
    score = np.asarray(score)
    if select_mode == SELECT_PER_LAYER:
        return topk_select_1d(score.sum(axis=0), k, start_size)[None, :]
    return np.stack([topk_select_1d(score[g], k, start_size) for g in range(score.shape[0])])


def kv_compact(k_cat, v_cat, idx):
    """Eq. (3)/(5): the cache after eviction holds exactly the selected rows.

    k_cat, v_cat [Hkv, n, d] (any dtype, copied untouched); idx [Hsel, m] with
    Hsel = Hkv or 1 (broadcast).  Returns (k_new, v_new) [Hkv, m, d].
    """
    k_cat = np.asarray(k_cat)
    v_cat = np.asarray(v_cat)
    idx = np.asarray(idx)
    hkv = k_cat.shape[0]
    k_new = np.stack([k_cat[g][idx[g % idx.shape[0]]] for g in range(hkv)])
    v_new = np.stack([v_cat[g][idx[g % idx.shape[0]]] for g in range(hkv)])
    return k_new, v_new


@dataclass
class ChunkTrace:
    """Everything one chunk step produced, for step-by-step comparison."""
    n_c: int
    out: np.ndarray                      # [Hq, c, d]
    lse: np.ndarray                      # [Hq, c]
    score: np.ndarray                    # [Hkv, n]  instruction score
    idx: np.ndarray                      # [Hsel, m]
    n_c_lm: int = 0
    score_lm: Optional[np.ndarray] = None
    idx_lm: Optional[np.ndarray] = None


@dataclass
class DocumentResult:
    k_cache: np.ndarray                  # [Hkv, n_c, d]
    v_cache: np.ndarray
    positions: np.ndarray                # [Hkv, n_c] original document positions held
    k_cache_lm: Optional[np.ndarray] = None
    v_cache_lm: Optional[np.ndarray] = None
    positions_lm: Optional[np.ndarray] = None
    trace: List[ChunkTrace] = field(default_factory=list)
    acc_score: Optional[np.ndarray] = None   # [Hkv, n_c] accumulated scores of the kept states (SCORE_ACCUMULATED)


def process_document(q, k, v, q_instr: Sequence[np.ndarray], chunk_len: int, budget: int,
                     cache_mode: int = CACHE_INSTR, select_mode: int = SELECT_PER_KV_HEAD,
                     budget_lm: Optional[int] = None, scale: Optional[float] = None,
                     forced_idx: Optional[Sequence[np.ndarray]] = None,
                     forced_idx_lm: Optional[Sequence[np.ndarray]] = None,
                     keep_trace: bool = True, start_size: int = 0,
                     lm_ordering: int = LM_SCORE_AFTER_APPEND,
                     score_mode: int = SCORE_PER_STEP,
                     position_shift: bool = False, rope_base: float = 10000.0) -> DocumentResult:
    """The chunk loop for one (document, layer).

    q [Hq, T, d]; k, v [Hkv, T, d]; q_instr: one [Hq, n_i, d] array per chunk
    (the instruction re-encoded against the current cache).  Per chunk:
    candidates = [cache ; chunk]; the chunk attends causally over them
    (Section 4.1 step 1); the instruction scores them (Eq. (1), s = I); the k
    best stay (Eq. (2)-(5)).  INSTR and SHARED run the same sequence on the
    single cache.  DUAL keeps a second, language-modelling cache of budget
    ``budget_lm`` that the chunk attends over and scores with its own
    attention (Eq. (1), s = chunk), next to the instruction cache that only
    the instruction scores; both receive the chunk's states (Section 4.2,
    individual cache).

    ``forced_idx`` replays a given selection history instead of the oracle's
    own (the per-step scores are still computed), so a trajectory can be
    compared step by step without one near-tie changing all later steps.
    ``lm_ordering`` (DUAL only) chooses how the language-modelling cache is
    evicted.  LM_SCORE_AFTER_APPEND: as described above.  LM_EVICT_THEN_APPEND
    is the three steps of Section 4.1 in the order printed: the chunk is
    encoded given the cache C (which still holds the whole previous chunk, up
    to budget_lm + chunk_len states), the states of C are scored by Eq. (1)
    with s = the chunk and the softmax normalised over the states of C only,
    the budget_lm best stay, and then all states of the chunk are put into
    the cache.  (The instruction cache is the same computation in both
    orderings, hoisted by one step.)
    ``start_size``: the first start_size states of the document are never
    evicted (appendix "Analysis on initial tokens"); they are the first
    candidates of every step because retained states keep their order.
    ``score_mode`` = SCORE_ACCUMULATED is the accumulative-attention rule that
    Section 5.2 ("Baselines", H2O and "H2O + Shared Cache") pairs with the
    instruction-aware cache: a state's importance is the sum of the Eq. (1)
    scores it has received from the instruction in every step since it entered
    the cache (a new state starts at its first score); the k largest sums stay
    and carry their sums on.  Only the instruction-scored cache uses it.
    ``position_shift``: q, k and q_instr are given WITHOUT rotary embedding
    and positions are those of the cache (Section 5.3): in every step
    candidate j of [cache ; chunk] is rotated to position j, chunk query t to
    n_c + t, instruction query u to n + u (the instruction follows the
    candidates); the cache itself keeps the unrotated keys.  With DUAL each
    cache has its own slots: the chunk attends over (and scores) the
    language-modelling cache at that cache's positions, the instruction scores
    the instruction cache at its own.
    """
    q, k, v = _f64(q), _f64(k), _f64(v)
    hq, t_total, d = q.shape
    hkv = k.shape[0]
    n_chunks = (t_total + chunk_len - 1) // chunk_len
    assert len(q_instr) >= n_chunks
    budget_lm = budget if budget_lm is None else budget_lm
    dual = cache_mode == CACHE_DUAL

    kc = np.zeros((hkv, 0, d)); vc = np.zeros((hkv, 0, d))
    pos = np.zeros((hkv, 0), dtype=np.int64)
    kc_lm = np.zeros((hkv, 0, d)); vc_lm = np.zeros((hkv, 0, d))
    pos_lm = np.zeros((hkv, 0), dtype=np.int64)
    acc = np.zeros((hkv, 0))             # accumulated score of every cache state (SCORE_ACCUMULATED)
    trace: List[ChunkTrace] = []

    for i in range(n_chunks):
        lo, hi = i * chunk_len, min(t_total, (i + 1) * chunk_len)
        c = hi - lo
        qs, ks, vs = q[:, lo:hi], k[:, lo:hi], v[:, lo:hi]
        chunk_pos = np.broadcast_to(np.arange(lo, hi, dtype=np.int64), (hkv, c))

        n_c = kc.shape[1]
        k_cat = np.concatenate([kc, ks], axis=1)
        v_cat = np.concatenate([vc, vs], axis=1)
        pos_cat = np.concatenate([pos, chunk_pos], axis=1)

        tr_lm = {}
        if dual:
            n_c_lm = kc_lm.shape[1]
            k_cat_lm = np.concatenate([kc_lm, ks], axis=1)
            v_cat_lm = np.concatenate([vc_lm, vs], axis=1)
            pos_cat_lm = np.concatenate([pos_lm, chunk_pos], axis=1)
            q_att_lm, k_att_lm = qs, k_cat_lm
            if position_shift:
                # this cache has its own slots: its state j sits at position j, chunk token t at n_c_lm + t
                k_att_lm = rope(k_cat_lm, np.arange(n_c_lm + c), rope_base)
                q_att_lm = rope(qs, n_c_lm + np.arange(c), rope_base)
            out, lse, probs = chunk_attn(q_att_lm, k_att_lm, v_cat_lm, n_c_lm, scale)
            g_size = hq // hkv
            if lm_ordering == LM_EVICT_THEN_APPEND:
                # step 2 of Section 4.1: Eq. (1) with s = chunk over the states of the cache alone
                # (every chunk token sees the whole cache, so there is no mask)
                if n_c_lm > 0:
                    s_lm = instr_score(q_att_lm, k_att_lm[:, :n_c_lm], scale)
                    idx_lm = (np.asarray(forced_idx_lm[i]) if forced_idx_lm is not None
                              else topk_select(s_lm, budget_lm, select_mode, start_size))
                else:
                    s_lm = np.zeros((hkv, 0))
                    idx_lm = np.zeros((1 if select_mode == SELECT_PER_LAYER else hkv, 0), dtype=np.int64)
                kept_k, kept_v = (kv_compact(kc_lm, vc_lm, idx_lm) if n_c_lm > 0 else (kc_lm, vc_lm))
                kept_pos = (np.stack([pos_lm[g][idx_lm[g % idx_lm.shape[0]]] for g in range(hkv)])
                            if n_c_lm > 0 else pos_lm)
                # step 3: all states of the chunk enter the cache
                kc_lm = np.concatenate([kept_k, ks], axis=1)
                vc_lm = np.concatenate([kept_v, vs], axis=1)
                pos_lm = np.concatenate([kept_pos, chunk_pos], axis=1)
            else:
                s_lm = probs.reshape(hkv, g_size, c, -1).sum(axis=(1, 2))
                idx_lm = (np.asarray(forced_idx_lm[i]) if forced_idx_lm is not None
                          else topk_select(s_lm, budget_lm, select_mode, start_size))
                kc_lm, vc_lm = kv_compact(k_cat_lm, v_cat_lm, idx_lm)
                pos_lm = np.stack([pos_cat_lm[g][idx_lm[g % idx_lm.shape[0]]] for g in range(hkv)])
            tr_lm = dict(n_c_lm=n_c_lm, score_lm=s_lm, idx_lm=idx_lm)
        elif position_shift:
            n = n_c + c
            k_att = rope(k_cat, np.arange(n), rope_base)
            out, lse, _ = chunk_attn(rope(qs, n_c + np.arange(c), rope_base), k_att, v_cat, n_c, scale)
        else:
            out, lse, _ = chunk_attn(qs, k_cat, v_cat, n_c, scale)

        if position_shift:
            n = n_c + c
            if dual:   # the instruction cache's own slots
                k_att = rope(k_cat, np.arange(n), rope_base)
            s_in = instr_score(rope(q_instr[i], n + np.arange(np.asarray(q_instr[i]).shape[1]), rope_base), k_att, scale)
        else:
            s_in = instr_score(q_instr[i], k_cat, scale)
        if score_mode == SCORE_ACCUMULATED:
            s_in = s_in + np.concatenate([acc, np.zeros((hkv, c))], axis=1)
        idx = (np.asarray(forced_idx[i]) if forced_idx is not None
               else topk_select(s_in, budget, select_mode, start_size))
        if score_mode == SCORE_ACCUMULATED:
            acc = np.stack([s_in[g][idx[g % idx.shape[0]]] for g in range(hkv)])
        kc, vc = kv_compact(k_cat, v_cat, idx)
        pos = np.stack([pos_cat[g][idx[g % idx.shape[0]]] for g in range(hkv)])
        if keep_trace:
            trace.append(ChunkTrace(n_c=n_c, out=out, lse=lse, score=s_in, idx=idx, **tr_lm))

    return DocumentResult(k_cache=kc, v_cache=vc, positions=pos,
                          k_cache_lm=kc_lm if dual else None,
                          v_cache_lm=vc_lm if dual else None,
                          positions_lm=pos_lm if dual else None, trace=trace,
                          acc_score=acc if score_mode == SCORE_ACCUMULATED else None)


def evict_cache(q_text, k_cache, v_cache, k: int, select_mode: int = SELECT_PER_KV_HEAD, start_size: int = 0,
                scale: Optional[float] = None, forced_idx: Optional[np.ndarray] = None):
    """One eviction of a cache by a text (Section 4.1, step 2; with the
    instruction as the text it is the additional eviction after the last
    chunk that removes the bias towards that chunk).

    q_text [Hq, rows, d]: queries of the text's tokens; k_cache, v_cache
    [Hkv, n, d].  The states are scored by Eq. (1), the softmax running over
    the n states of the cache alone (every token of the text sees the whole
    cache); the k best stay in their order (Eq. (2)-(3)).
    Returns (k_new, v_new, idx, score).
    """
    score = instr_score(q_text, k_cache, scale)
    idx = np.asarray(forced_idx) if forced_idx is not None else topk_select(score, k, select_mode, start_size)
    k_new, v_new = kv_compact(k_cache, v_cache, idx)
    return k_new, v_new, idx, score


@dataclass
class StandardCseResult:
    out: np.ndarray                      # [Hq, T, d] chunk outputs over the whole document
    k_cache: np.ndarray                  # [Hkv, n_c, d] cache when the document ends (before a final eviction)
    v_cache: np.ndarray
    positions: np.ndarray                # [Hkv, n_c]
    idx: List[np.ndarray]                # per chunk: kept positions among that step's candidates
    score: List[np.ndarray]              # per chunk: the scores they were chosen by
    k_final: Optional[np.ndarray] = None  # after the eviction by the instruction, if one was asked for
    v_final: Optional[np.ndarray] = None
    positions_final: Optional[np.ndarray] = None
    idx_final: Optional[np.ndarray] = None
    score_final: Optional[np.ndarray] = None


def standard_cse(q, k, v, chunk_len: int, budget: int, lm_ordering: int = LM_EVICT_THEN_APPEND,
                 select_mode: int = SELECT_PER_KV_HEAD, start_size: int = 0, scale: Optional[float] = None,
                 q_instr_final=None, forced_idx: Optional[Sequence[np.ndarray]] = None,
                 forced_idx_final: Optional[np.ndarray] = None) -> StandardCseResult:
    """Standard CSE alone (Section 4.1, "Overall process"): one cache, evicted
    by the document's own chunks, no instruction during encoding.

    LM_EVICT_THEN_APPEND is the printed order: encode the chunk given the
    cache, evict the cache down to ``budget`` states by the chunk's attention
    to it (Eq. (1) over the cache states alone), put all states of the chunk
    in; the first chunk just enters.  LM_SCORE_AFTER_APPEND is this
    repository's other reading: the chunk's states are appended first and the
    chunk's own causal attention over [cache ; chunk] decides which ``budget``
    of them stay.
    If ``q_instr_final`` [Hq, n_i, d] is given, the cache is evicted one more
    time with the instruction as the text once the document has ended, down to
    ``budget`` states (the end of the same paragraph).
    """
    q, k, v = _f64(q), _f64(k), _f64(v)
    hq, t_total, d = q.shape
    hkv = k.shape[0]
    n_chunks = (t_total + chunk_len - 1) // chunk_len
    kc = np.zeros((hkv, 0, d)); vc = np.zeros((hkv, 0, d))
    pos = np.zeros((hkv, 0), dtype=np.int64)
    outs, idxs, scores = [], [], []
    for i in range(n_chunks):
        lo, hi = i * chunk_len, min(t_total, (i + 1) * chunk_len)
        qs, ks, vs = q[:, lo:hi], k[:, lo:hi], v[:, lo:hi]
        chunk_pos = np.broadcast_to(np.arange(lo, hi, dtype=np.int64), (hkv, hi - lo))
        n_c = kc.shape[1]
        forced = None if forced_idx is None else forced_idx[i]
        # step 1: encode the chunk given the cache
        out, _, _ = chunk_attn(qs, np.concatenate([kc, ks], axis=1), np.concatenate([vc, vs], axis=1), n_c, scale)
        outs.append(out)
        if lm_ordering == LM_EVICT_THEN_APPEND:
            if n_c > 0:
                # step 2: the chunk evicts the cache
                kc, vc, idx, sc = evict_cache(qs, kc, vc, budget, select_mode, start_size, scale, forced)
                pos = np.stack([pos[g][idx[g % idx.shape[0]]] for g in range(hkv)])
            else:
                idx, sc = np.zeros((1 if select_mode == SELECT_PER_LAYER else hkv, 0), dtype=np.int64), np.zeros((hkv, 0))
            # step 3: the chunk's states enter
            kc = np.concatenate([kc, ks], axis=1)
            vc = np.concatenate([vc, vs], axis=1)
            pos = np.concatenate([pos, chunk_pos], axis=1)
        else:
            k_cat, v_cat = np.concatenate([kc, ks], axis=1), np.concatenate([vc, vs], axis=1)
            pos_cat = np.concatenate([pos, chunk_pos], axis=1)
            sc = lm_score(qs, k_cat, n_c, scale)
            idx = np.asarray(forced) if forced is not None else topk_select(sc, budget, select_mode, start_size)
            kc, vc = kv_compact(k_cat, v_cat, idx)
            pos = np.stack([pos_cat[g][idx[g % idx.shape[0]]] for g in range(hkv)])
        idxs.append(idx)
        scores.append(sc)
    res = StandardCseResult(out=np.concatenate(outs, axis=1), k_cache=kc, v_cache=vc, positions=pos, idx=idxs,
                            score=scores)
    if q_instr_final is not None:
        res.k_final, res.v_final, res.idx_final, res.score_final = evict_cache(
            _f64(q_instr_final), kc, vc, budget, select_mode, start_size, scale, forced_idx_final)
        res.positions_final = np.stack([pos[g][res.idx_final[g % res.idx_final.shape[0]]] for g in range(hkv)])
    return res


def decode_step(q_new, k_new, v_new, k_cache, v_cache, scale: Optional[float] = None):
    """One generation step over the retained cache (Section 4.3: the k states
    left by the last eviction encode the instruction and the response).

    q_new [Hq, d]; k_new, v_new [Hkv, d]: the new token; k_cache, v_cache
    [Hkv, n, d].  The token's own state is appended (nothing is evicted while
    the response is generated) and its query attends over all n + 1 states.
    Returns (out [Hq, d], k_cache' [Hkv, n + 1, d], v_cache').
    """
    q_new, k_new, v_new = _f64(q_new), _f64(k_new), _f64(v_new)
    k_all = np.concatenate([_f64(k_cache), k_new[:, None, :]], axis=1)
    v_all = np.concatenate([_f64(v_cache), v_new[:, None, :]], axis=1)
    hq, d = q_new.shape
    hkv = k_all.shape[0]
    g_size = hq // hkv
    sc = _scale(d, scale)
    out = np.zeros((hq, d))
    for h in range(hq):
        g = h // g_size
        p, _ = softmax_rows((k_all[g] @ q_new[h])[None, :] * sc)
        out[h] = p[0] @ v_all[g]
    return out, k_all, v_all


def full_causal_attention(q, k, v, scale: Optional[float] = None) -> np.ndarray:
    """Textbook causal attention over a whole document in one shot; what the
    chunk loop must reproduce when the budget is at least the document
    length."""
    out, _, _ = chunk_attn(q, k, v, 0, scale)
    return out
