// Host side of the C ABI declared in include/citrus.h: argument validation,
// kernel dispatch, and the chunk loop of the paper's "Overall process"
// (Section 4.1, Section 4.3).  No device memory is allocated here and no call
// synchronises with the device.
#include <math.h>
#include <string.h>

#include "citrus_internal.h"

using namespace citrus;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

int elem_bytes(int dtype) { return dtype == CITRUS_F32 ? 4 : 2; }

citrus_status check_config(const citrus_config* c) {
  if (c == nullptr) return CITRUS_ERR_NULL;
  if (c->batch < 1 || c->layers < 1 || c->q_heads < 1 || c->kv_heads < 1) return CITRUS_ERR_SHAPE;
  if (c->q_heads % c->kv_heads != 0) return CITRUS_ERR_SHAPE;
  if (c->chunk_len < 1 || c->budget < 1 || c->instr_len < 1) return CITRUS_ERR_SHAPE;
  if (static_cast<int64_t>(c->batch) * c->layers > 65535 || c->q_heads > 65535) return CITRUS_ERR_SHAPE;
  {
    // the largest launch has one workgroup per (document, layer, query head, 32-row tile, range of key tiles):
    // its count, like every unit count formed in 32 bits below, has to stay under 2^31
    const int64_t rows_max = c->chunk_len > c->instr_len ? c->chunk_len : c->instr_len;
    const int64_t blocks = static_cast<int64_t>(c->batch) * c->layers * c->q_heads * ((rows_max + 31) / 32) * kMaxKeySplits;
    if (blocks >= (int64_t{1} << 31)) return CITRUS_ERR_SHAPE;
  }
  if (c->cache_mode != CITRUS_CACHE_INSTR && c->cache_mode != CITRUS_CACHE_SHARED &&
      c->cache_mode != CITRUS_CACHE_DUAL && c->cache_mode != CITRUS_CACHE_STANDARD)
    return CITRUS_ERR_UNSUPPORTED;
  if (c->select_mode != CITRUS_SELECT_PER_KV_HEAD && c->select_mode != CITRUS_SELECT_PER_LAYER)
    return CITRUS_ERR_UNSUPPORTED;
  if (c->dtype != CITRUS_F32 && c->dtype != CITRUS_BF16) return CITRUS_ERR_UNSUPPORTED;
  if (c->head_dim != 64 && c->head_dim != 128) return CITRUS_ERR_UNSUPPORTED;
  if (c->cache_mode == CITRUS_CACHE_DUAL && c->budget_lm < 1) return CITRUS_ERR_SHAPE;
  const int need = c->cache_mode == CITRUS_CACHE_DUAL && c->budget_lm > c->budget ? c->budget_lm : c->budget;
  if (c->cache_capacity < need) return CITRUS_ERR_SHAPE;
  if (c->start_size < 0 || c->start_size >= c->budget) return CITRUS_ERR_SHAPE;
  if (c->lm_ordering != CITRUS_LM_SCORE_AFTER_APPEND && c->lm_ordering != CITRUS_LM_EVICT_THEN_APPEND)
    return CITRUS_ERR_UNSUPPORTED;
  if (c->lm_ordering == CITRUS_LM_EVICT_THEN_APPEND) {
    // the cache the chunk evicts still holds the whole previous chunk
    if (c->cache_mode == CITRUS_CACHE_DUAL && c->cache_capacity < c->budget_lm + c->chunk_len) return CITRUS_ERR_SHAPE;
    if (c->cache_mode == CITRUS_CACHE_STANDARD && c->cache_capacity < c->budget + c->chunk_len) return CITRUS_ERR_SHAPE;
  }
  if (c->cache_mode == CITRUS_CACHE_DUAL && c->start_size >= c->budget_lm) return CITRUS_ERR_SHAPE;
  if (!(c->softmax_scale >= 0.0f) || isinf(c->softmax_scale)) return CITRUS_ERR_SHAPE;
  if (c->score_mode != CITRUS_SCORE_PER_STEP && c->score_mode != CITRUS_SCORE_ACCUMULATED) return CITRUS_ERR_UNSUPPORTED;
  if (c->score_mode == CITRUS_SCORE_ACCUMULATED && c->cache_mode != CITRUS_CACHE_INSTR &&
      c->cache_mode != CITRUS_CACHE_SHARED)
    return CITRUS_ERR_UNSUPPORTED;
  if (c->position_shift != 0 && c->position_shift != 1) return CITRUS_ERR_UNSUPPORTED;
  if (c->position_shift && c->cache_mode == CITRUS_CACHE_STANDARD) return CITRUS_ERR_UNSUPPORTED;
  if (!(c->rope_base >= 0.0f) || isinf(c->rope_base) || (c->rope_base > 0.0f && c->rope_base < 1.0f))
    return CITRUS_ERR_SHAPE;
  return CITRUS_OK;
}

Dims dims_of(const citrus_config* c) {
  Dims d;
  d.B = c->batch; d.L = c->layers; d.Hq = c->q_heads; d.Hkv = c->kv_heads; d.G = c->q_heads / c->kv_heads;
  d.D = c->head_dim;
  d.scale = c->softmax_scale > 0.0f ? c->softmax_scale : 1.0f / sqrtf(static_cast<float>(c->head_dim));
  return d;
}

float rope_base_of(const citrus_config* c) { return c->rope_base > 0.0f ? c->rope_base : 10000.0f; }

// 16-byte row alignment: pointer and every stride.  `rows`: the sequence rows of a (b, l, h) unit the call may
// touch; they must span less than 2 GiB, because the kernels address a unit's rows with 32-bit byte offsets.
citrus_status check_tensor(const citrus_config* c, const citrus_tensor& t, int64_t rows, bool may_be_null) {
  if (t.ptr == nullptr) return may_be_null ? CITRUS_OK : CITRUS_ERR_NULL;
  const int esz = elem_bytes(c->dtype);
  const int64_t q = 16 / esz;
  if (reinterpret_cast<uintptr_t>(t.ptr) % 16 != 0) return CITRUS_ERR_SHAPE;
  if (t.stride_b % q || t.stride_l % q || t.stride_h % q || t.stride_s % q) return CITRUS_ERR_SHAPE;
  if (t.stride_s <= 0) return CITRUS_ERR_SHAPE;
  constexpr int64_t kUnitSpan = int64_t{1} << 31;
  if (t.stride_s >= kUnitSpan) return CITRUS_ERR_SHAPE;
  if (rows > 0 && ((rows - 1) * t.stride_s + c->head_dim) * esz >= kUnitSpan) return CITRUS_ERR_SHAPE;
  return CITRUS_OK;
}

#define CITRUS_TRY(expr)                         \
  do {                                           \
    const citrus_status st__ = (expr);           \
    if (st__ != CITRUS_OK) return st__;          \
  } while (0)

citrus_status check_lengths(const citrus_config* c, int cache_len, int chunk_len) {
  if (cache_len < 0 || cache_len > c->cache_capacity) return CITRUS_ERR_SHAPE;
  if (chunk_len < 1 || chunk_len > c->chunk_len) return CITRUS_ERR_SHAPE;
  return CITRUS_OK;
}

// A block of float scratch and what it holds: the scorer picks its kernel by what fits.
struct Scratch {
  float* ptr;
  size_t floats;
};

// Workspace layout (all blocks kAlign-aligned).
struct Workspace {
  size_t lse_chunk, lse_instr, lse_cache, score, score_lm, idx, idx_lm, iota, decode, k_rot, k_rot_lm, q_rot, qi_rot, total;
};

// A cache evicted by the document's own chunks exists (DUAL's second cache, or the only one of STANDARD)
// and is run in the order Section 4.1 prints.
bool evict_then_append(const citrus_config* c) {
  return (c->cache_mode == CITRUS_CACHE_DUAL || c->cache_mode == CITRUS_CACHE_STANDARD) &&
         c->lm_ordering == CITRUS_LM_EVICT_THEN_APPEND;
}

// floats of the partial-softmax block that serves up to `rows` query rows per head over up to cache_capacity +
// chunk_len candidates
size_t score_scratch_floats(const citrus_config* c, int rows) {
  const size_t n_max = static_cast<size_t>(c->cache_capacity) + c->chunk_len;
  return instr_score_mfma_workspace_floats(dims_of(c), rows, static_cast<int>(n_max));
}

Workspace workspace_layout(const citrus_config* c) {
  Workspace w;
  const size_t units_q = static_cast<size_t>(c->batch) * c->layers * c->q_heads;
  const size_t units_kv = static_cast<size_t>(c->batch) * c->layers * c->kv_heads;
  const size_t n_max = static_cast<size_t>(c->cache_capacity) + c->chunk_len;
  const bool dual = c->cache_mode == CITRUS_CACHE_DUAL;
  size_t off = 0;
  w.lse_chunk = off; off += align_up(units_q * c->chunk_len * sizeof(float));
  // scratch of the instruction score: partial (max, sum) pairs x 8 key ranges, or partial column sums per row strip
  w.lse_instr = off; off += align_up(score_scratch_floats(c, c->instr_len) * sizeof(float));
  w.lse_cache = off; off += evict_then_append(c) ? align_up(score_scratch_floats(c, c->chunk_len) * sizeof(float)) : 0;  // same, chunk rows
  w.score = off;     off += align_up(units_kv * n_max * sizeof(float));
  w.score_lm = off;  off += dual ? align_up(units_kv * n_max * sizeof(float)) : 0;
  w.idx = off;       off += align_up(units_kv * c->budget * sizeof(int32_t));
  w.idx_lm = off;    off += dual ? align_up(units_kv * c->budget_lm * sizeof(int32_t)) : 0;
  w.iota = off;      off += align_up(c->chunk_len * sizeof(int32_t));
  {
    const Dims dm = dims_of(c);
    w.decode = off;  off += decode_mfma_supported(c->dtype, dm) ? align_up(decode_mfma_workspace_floats(dm) * sizeof(float)) : 0;
  }
  // position shift: rotated copies of the candidates' keys, the chunk's and the instruction's queries
  const size_t esz = static_cast<size_t>(elem_bytes(c->dtype)) * c->head_dim;
  w.k_rot = off;   off += c->position_shift ? align_up(units_kv * n_max * esz) : 0;
  w.k_rot_lm = off; off += c->position_shift && dual ? align_up(units_kv * n_max * esz) : 0;  // each cache has its own slots
  w.q_rot = off;   off += c->position_shift ? align_up(units_q * c->chunk_len * esz) : 0;
  w.qi_rot = off;  off += c->position_shift ? align_up(units_q * c->instr_len * esz) : 0;
  w.total = off;
  return w;
}

citrus_status check_workspace(const citrus_config* c, const void* ws, size_t bytes) {
  if (ws == nullptr || bytes < workspace_layout(c).total) return CITRUS_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(ws) % 16 != 0) return CITRUS_ERR_WORKSPACE;
  return CITRUS_OK;
}

// ---- dispatch: MFMA kernels where they apply, generic kernels otherwise ----

hipError_t run_attn(const citrus_config* c, const Dims& dm, View q, int rows, Segments ks, Segments vs, int causal,
                    View out, float* lse, hipStream_t st) {
  if (mfma_path_supported(c->dtype, dm))
    return launch_attn_mfma(dm, q, rows, ks, vs, causal, out, lse, nullptr, 1, nullptr, st);
  return launch_attn_generic(c->dtype, dm, q, rows, ks, vs, causal, out, lse, st);
}

hipError_t run_colsum(const citrus_config* c, const Dims& dm, View q, int rows, Segments ks, int causal,
                      const float* lse, float* score, hipStream_t st) {
  if (mfma_path_supported(c->dtype, dm))
    return launch_colsum_mfma(dm, q, rows, ks, causal, lse, 1, nullptr, score, st);
  return launch_colsum_generic(c->dtype, dm, q, rows, ks, causal, lse, score, st);
}

// Unchecked bodies shared by the public entry points and the chunk loop.

// lse_cache (optional, needs ks.n_c > 0): each row's log-sum-exp over the cache states alone, the
// normaliser of Eq. (1) as printed.  A by-product of the MFMA attention kernel when the cache ends on
// a 32-key boundary; a pass of its own over the cache otherwise.
// q_rope_pos0 >= 0 (MFMA path only, see attn_rotates_queries): q is unrotated and the kernel rotates it.
citrus_status do_chunk_attn(const citrus_config* c, const Dims& dm, const citrus_tensor& q, Segments ks, Segments vs,
                            const citrus_tensor& out, float* lse, float* lm_score, float* lse_cache, hipStream_t st,
                            int q_rope_pos0 = -1) {
  const bool mfma = mfma_path_supported(c->dtype, dm);
  if (q_rope_pos0 >= 0 && !mfma) return CITRUS_ERR_UNSUPPORTED;
  const bool fused_lse = lse_cache != nullptr && mfma && attn_mfma_emits_cache_lse(ks, 1, make_view(out));
  // in-kernel query rotation together with a cache-only normaliser that needs a pass of its own: not
  // combined by any caller (decided before anything is launched)
  if (q_rope_pos0 >= 0 && lse_cache != nullptr && !fused_lse) return CITRUS_ERR_UNSUPPORTED;
  if (fused_lse || q_rope_pos0 >= 0) {
    CITRUS_TRY(hip_status(launch_attn_mfma(dm, make_view(q), ks.c, ks, vs, /*causal=*/1, make_view(out), lse,
                                           fused_lse ? lse_cache : nullptr, 1, nullptr, st, q_rope_pos0,
                                           rope_base_of(c))));
  } else {
    CITRUS_TRY(hip_status(run_attn(c, dm, make_view(q), ks.c, ks, vs, /*causal=*/1, make_view(out), lse, st)));
    if (lse_cache != nullptr) {
      Segments only = ks;  // the cache as the only key segment
      only.chunk = ks.cache;
      only.c = ks.n_c;
      only.n_c = 0;
      View none{nullptr, 0, 0, 0, 0};
      CITRUS_TRY(hip_status(run_attn(c, dm, make_view(q), ks.c, only, only, /*causal=*/0, none, lse_cache, st)));
    }
  }
  if (lm_score != nullptr)
    CITRUS_TRY(hip_status(run_colsum(c, dm, make_view(q), ks.c, ks, /*causal=*/1, lse, lm_score, st)));
  return CITRUS_OK;
}

citrus_status do_instr_score(const citrus_config* c, const Dims& dm, const citrus_tensor& q_instr, Segments ks,
                             Scratch scratch, float* score, hipStream_t st) {
  float* const lse_ws = scratch.ptr;
  if (mfma_path_supported(c->dtype, dm))
    return hip_status(launch_instr_score_mfma(dm, make_view(q_instr), c->instr_len, ks, lse_ws, scratch.floats, score, st));
  View none{nullptr, 0, 0, 0, 0};
  // pass 1: row normalisers (log-sum-exp over all n candidates, no mask)
  CITRUS_TRY(hip_status(run_attn(c, dm, make_view(q_instr), c->instr_len, ks, ks, /*causal=*/0, none, lse_ws, st)));
  // pass 2: probabilities summed down the rows of each KV group
  CITRUS_TRY(hip_status(run_colsum(c, dm, make_view(q_instr), c->instr_len, ks, /*causal=*/0, lse_ws, score, st)));
  return CITRUS_OK;
}

// A cache as the only key segment (the kernels take [cache ; chunk]; the chunk part is empty here and
// the cache is passed as the "chunk" so that every row index is a chunk row index).
Segments cache_only(const citrus_tensor& cache, int cache_len) {
  Segments s;
  s.cache = make_view(cache);
  s.chunk = make_view(cache);
  s.n_c = 0;
  s.c = cache_len;
  return s;
}

// Eq. (1) as printed: the rows of q score the states of one cache, softmax over those states alone.
// The cache is handed to the kernels as the only key segment.
citrus_status do_cache_score(const citrus_config* c, const Dims& dm, const citrus_tensor& q, int rows,
                             const citrus_tensor& k_cache, int cache_len, const float* lse_given, Scratch scratch,
                             float* score, hipStream_t st) {
  float* const lse_ws = scratch.ptr;
  const Segments ks = cache_only(k_cache, cache_len);
  if (lse_given != nullptr)  // the normalisers are known: only the column sums are left
    return hip_status(run_colsum(c, dm, make_view(q), rows, ks, /*causal=*/0, lse_given, score, st));
  if (mfma_path_supported(c->dtype, dm))
    return hip_status(launch_instr_score_mfma(dm, make_view(q), rows, ks, lse_ws, scratch.floats, score, st));
  View none{nullptr, 0, 0, 0, 0};
  CITRUS_TRY(hip_status(run_attn(c, dm, make_view(q), rows, ks, ks, /*causal=*/0, none, lse_ws, st)));
  CITRUS_TRY(hip_status(run_colsum(c, dm, make_view(q), rows, ks, /*causal=*/0, lse_ws, score, st)));
  return CITRUS_OK;
}

int sel_heads(const citrus_config* c) { return c->select_mode == CITRUS_SELECT_PER_LAYER ? 1 : c->kv_heads; }

citrus_status do_topk(const citrus_config* c, const float* score, int n, int k, int32_t* idx, hipStream_t st) {
  const bool per_layer = c->select_mode == CITRUS_SELECT_PER_LAYER;
  const int units = c->batch * c->layers * (per_layer ? 1 : c->kv_heads);
  return hip_status(launch_topk(score, units, per_layer ? c->kv_heads : 1, n, k, c->start_size, idx, st));
}

citrus_status do_compact(const citrus_config* c, const Dims& dm, Segments ks, Segments vs, const int32_t* idx,
                         int idx_pitch, int m, const citrus_tensor& k_new, const citrus_tensor& v_new,
                         hipStream_t st) {
  return hip_status(launch_compact(elem_bytes(c->dtype), dm, ks, vs, idx, idx_pitch, sel_heads(c), m,
                                   make_view(k_new), make_view(v_new), st));
}

// A dense [B, L, heads, rows, d] tensor at `ptr`.
citrus_tensor dense_tensor(void* ptr, int64_t layers, int64_t heads, int64_t rows, int64_t d) {
  citrus_tensor t;
  t.ptr = ptr;
  t.stride_s = d;
  t.stride_h = rows * d;
  t.stride_l = heads * rows * d;
  t.stride_b = layers * heads * rows * d;
  return t;
}

// The same tensor starting at sequence row `row`.
citrus_tensor rows_from(citrus_tensor t, int64_t row, int dtype) {
  t.ptr = static_cast<char*>(t.ptr) + row * t.stride_s * elem_bytes(dtype);
  return t;
}

Segments segments(const citrus_tensor& cache, int cache_len, const citrus_tensor& chunk, int chunk_len) {
  Segments s;
  s.cache = make_view(cache);
  s.chunk = make_view(chunk);
  s.n_c = cache_len;
  s.c = chunk_len;
  if (cache_len == 0) s.cache = s.chunk;  // never dereferenced, but keep it a valid pointer
  return s;
}

// Partial-softmax block of the workspace that fits `rows` query rows, or a NULL block.
Scratch cache_score_block(const citrus_config* c, void* workspace, int rows) {
  const Workspace wl = workspace_layout(c);
  char* ws = static_cast<char*>(workspace);
  if (rows <= c->instr_len) return Scratch{reinterpret_cast<float*>(ws + wl.lse_instr), score_scratch_floats(c, c->instr_len)};
  if (evict_then_append(c) && rows <= c->chunk_len)
    return Scratch{reinterpret_cast<float*>(ws + wl.lse_cache), score_scratch_floats(c, c->chunk_len)};
  return Scratch{nullptr, 0};
}

// Argument checks shared by the two forms of the eviction of a cache by a text.
citrus_status check_evict_args(const citrus_config* cfg, const citrus_tensor& q, int rows, const citrus_tensor& k_cache,
                               const citrus_tensor& v_cache, int cache_len, int k, const citrus_tensor& k_new,
                               const citrus_tensor& v_new) {
  CITRUS_TRY(check_config(cfg));
  if (rows < 1 || cache_len < 1 || cache_len > cfg->cache_capacity || k < 1 || k > cfg->budget) return CITRUS_ERR_SHAPE;
  CITRUS_TRY(check_tensor(cfg, q, rows, false));
  CITRUS_TRY(check_tensor(cfg, k_cache, cache_len, false));
  CITRUS_TRY(check_tensor(cfg, v_cache, cache_len, false));
  CITRUS_TRY(check_tensor(cfg, k_new, k, false));
  CITRUS_TRY(check_tensor(cfg, v_new, k, false));
  if (k_new.ptr == k_cache.ptr || v_new.ptr == v_cache.ptr) return CITRUS_ERR_SHAPE;
  return CITRUS_OK;
}

// Score of the cache by the rows of q, selection, gather.  scratch: partial-softmax block for `rows` query rows;
// score: B*L*Hkv*cache_len floats; idx: B*L*Hsel*k positions.  A cache that fits stays whole: the selection is
// then the identity and reads no score.
citrus_status do_evict_cache(const citrus_config* cfg, const citrus_tensor& q, int rows, const citrus_tensor& k_cache,
                             const citrus_tensor& v_cache, int cache_len, int k, const citrus_tensor& k_new,
                             const citrus_tensor& v_new, int32_t* idx, Scratch scratch, float* score, hipStream_t st) {
  const Dims dm = dims_of(cfg);
  const int m = cache_len < k ? cache_len : k;
  if (cache_len > k) CITRUS_TRY(do_cache_score(cfg, dm, q, rows, k_cache, cache_len, nullptr, scratch, score, st));
  CITRUS_TRY(do_topk(cfg, score, cache_len, k, idx, st));
  const Segments ks = cache_only(k_cache, cache_len), vs = cache_only(v_cache, cache_len);
  return do_compact(cfg, dm, ks, vs, idx, k, m, k_new, v_new, st);
}

// ---- device scratch that lives in the library's own image, for callers that cannot allocate ----
// One copy per GPU, held from the moment the library's code is loaded on that GPU until the process ends.
// `scratch` is only a host-side name for the array: its device address differs per GPU and is looked up once
// per device (hipGetSymbolAddress) and kept; host code passes that address, never the name, to kernels.
constexpr size_t kStaticScratchBytes = size_t{16} << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
std::atomic<char*> g_scratch_base[kMaxDevices] = {};

citrus_status static_scratch_base(char** base) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return CITRUS_ERR_DEVICE;
  if (dev < 0 || dev >= kMaxDevices) return CITRUS_ERR_UNSUPPORTED;
  char* p = g_scratch_base[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    void* sym = nullptr;
    if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || sym == nullptr) return CITRUS_ERR_DEVICE;
    p = static_cast<char*>(sym);
    g_scratch_base[dev].store(p, std::memory_order_release);  // two threads racing here store the same address
  }
  *base = p;
  return CITRUS_OK;
}

// What citrus_evict_cache_static keeps in the array, sized by the call's own arguments.
struct StaticEvictLayout {
  size_t lse, score, idx, total;
};
StaticEvictLayout static_evict_layout(const citrus_config* c, int rows, int cache_len, int k) {
  const size_t units_kv = static_cast<size_t>(c->batch) * c->layers * c->kv_heads;
  const size_t units_sel = static_cast<size_t>(c->batch) * c->layers * sel_heads(c);
  StaticEvictLayout s;
  size_t off = 0;
  // partial (max, sum) pairs x 8 key ranges, or partial column sums per row strip
  s.lse = off;   off += align_up(instr_score_mfma_workspace_floats(dims_of(c), rows, cache_len) * sizeof(float));
  s.score = off; off += align_up(units_kv * cache_len * sizeof(float));
  s.idx = off;   off += align_up(units_sel * k * sizeof(int32_t));
  s.total = off;
  return s;
}

}  // namespace

extern "C" {

int32_t citrus_abi_version(void) { return CITRUS_ABI_VERSION; }

const char* citrus_status_string(int32_t status) {
  switch (status) {
    case CITRUS_OK: return "ok";
    case CITRUS_ERR_NULL: return "a required pointer is NULL";
    case CITRUS_ERR_SHAPE: return "sizes or strides are inconsistent or out of range";
    case CITRUS_ERR_UNSUPPORTED: return "dtype, head_dim or mode not supported";
    case CITRUS_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case CITRUS_ERR_DEVICE: return "HIP runtime error at kernel launch";
    case CITRUS_ERR_PROVIDER: return "chunk provider reported an error";
    default: return "unknown status";
  }
}

size_t citrus_workspace_bytes(const citrus_config* cfg) {
  if (check_config(cfg) != CITRUS_OK) return 0;
  return workspace_layout(cfg).total;
}

int32_t citrus_chunk_attn(const citrus_config* cfg, citrus_tensor q, citrus_tensor k_cache, citrus_tensor v_cache,
                          int32_t cache_len, citrus_tensor k_chunk, citrus_tensor v_chunk, int32_t chunk_len,
                          citrus_tensor out, float* lse, float* lse_cache, float* lm_score, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
  CITRUS_TRY(check_config(cfg));
  CITRUS_TRY(check_lengths(cfg, cache_len, chunk_len));
  if (lse_cache != nullptr && cache_len == 0) return CITRUS_ERR_SHAPE;
  CITRUS_TRY(check_tensor(cfg, q, chunk_len, false));
  CITRUS_TRY(check_tensor(cfg, out, chunk_len, false));
  CITRUS_TRY(check_tensor(cfg, k_chunk, chunk_len, false));
  CITRUS_TRY(check_tensor(cfg, v_chunk, chunk_len, false));
  CITRUS_TRY(check_tensor(cfg, k_cache, cache_len, cache_len == 0));
  CITRUS_TRY(check_tensor(cfg, v_cache, cache_len, cache_len == 0));
  if (lm_score != nullptr && lse == nullptr) {
    CITRUS_TRY(check_workspace(cfg, workspace, workspace_bytes));
    lse = reinterpret_cast<float*>(static_cast<char*>(workspace) + workspace_layout(cfg).lse_chunk);
  }
  const Dims dm = dims_of(cfg);
  return do_chunk_attn(cfg, dm, q, segments(k_cache, cache_len, k_chunk, chunk_len),
                       segments(v_cache, cache_len, v_chunk, chunk_len), out, lse, lm_score, lse_cache,
                       static_cast<hipStream_t>(hip_stream));
}

int32_t citrus_instr_score(const citrus_config* cfg, citrus_tensor q_instr, citrus_tensor k_cache, int32_t cache_len,
                           citrus_tensor k_chunk, int32_t chunk_len, float* score, void* workspace,
                           size_t workspace_bytes, void* hip_stream) {
  CITRUS_TRY(check_config(cfg));
  CITRUS_TRY(check_lengths(cfg, cache_len, chunk_len));
  if (score == nullptr) return CITRUS_ERR_NULL;
  CITRUS_TRY(check_tensor(cfg, q_instr, cfg->instr_len, false));
  CITRUS_TRY(check_tensor(cfg, k_chunk, chunk_len, false));
  CITRUS_TRY(check_tensor(cfg, k_cache, cache_len, cache_len == 0));
  CITRUS_TRY(check_workspace(cfg, workspace, workspace_bytes));
  const Dims dm = dims_of(cfg);
  const Scratch scratch{reinterpret_cast<float*>(static_cast<char*>(workspace) + workspace_layout(cfg).lse_instr),
                        score_scratch_floats(cfg, cfg->instr_len)};
  return do_instr_score(cfg, dm, q_instr, segments(k_cache, cache_len, k_chunk, chunk_len), scratch, score,
                        static_cast<hipStream_t>(hip_stream));
}

int32_t citrus_cache_score(const citrus_config* cfg, citrus_tensor q, int32_t rows, citrus_tensor k_cache,
                           int32_t cache_len, const float* lse_cache, float* score, void* workspace,
                           size_t workspace_bytes, void* hip_stream) {
  CITRUS_TRY(check_config(cfg));
  if (rows < 1 || cache_len < 1 || cache_len > cfg->cache_capacity) return CITRUS_ERR_SHAPE;
  if (score == nullptr) return CITRUS_ERR_NULL;
  CITRUS_TRY(check_tensor(cfg, q, rows, false));
  CITRUS_TRY(check_tensor(cfg, k_cache, cache_len, false));
  if (lse_cache != nullptr) {  // no workspace needed: the rows' normalisers are given
    if (rows > cfg->chunk_len && rows > cfg->instr_len) return CITRUS_ERR_SHAPE;
    return do_cache_score(cfg, dims_of(cfg), q, rows, k_cache, cache_len, lse_cache, Scratch{nullptr, 0}, score,
                          static_cast<hipStream_t>(hip_stream));
  }
  CITRUS_TRY(check_workspace(cfg, workspace, workspace_bytes));
  const Scratch scratch = cache_score_block(cfg, workspace, rows);
  if (scratch.ptr == nullptr) return CITRUS_ERR_SHAPE;
  return do_cache_score(cfg, dims_of(cfg), q, rows, k_cache, cache_len, nullptr, scratch, score,
                        static_cast<hipStream_t>(hip_stream));
}

int32_t citrus_evict_cache(const citrus_config* cfg, citrus_tensor q, int32_t rows, citrus_tensor k_cache,
                           citrus_tensor v_cache, int32_t cache_len, int32_t k, citrus_tensor k_new,
                           citrus_tensor v_new, int32_t* idx, void* workspace, size_t workspace_bytes,
                           void* hip_stream) {
  CITRUS_TRY(check_evict_args(cfg, q, rows, k_cache, v_cache, cache_len, k, k_new, v_new));
  CITRUS_TRY(check_workspace(cfg, workspace, workspace_bytes));
  const Scratch scratch = cache_score_block(cfg, workspace, rows);
  if (scratch.ptr == nullptr) return CITRUS_ERR_SHAPE;
  const Workspace wl = workspace_layout(cfg);
  char* ws = static_cast<char*>(workspace);
  float* score = reinterpret_cast<float*>(ws + wl.score);
  if (idx == nullptr) idx = reinterpret_cast<int32_t*>(ws + wl.idx);
  return do_evict_cache(cfg, q, rows, k_cache, v_cache, cache_len, k, k_new, v_new, idx, scratch, score,
                        static_cast<hipStream_t>(hip_stream));
}

size_t citrus_static_scratch_bytes(void) { return kStaticScratchBytes; }

int32_t citrus_evict_cache_static(const citrus_config* cfg, citrus_tensor q, int32_t rows, citrus_tensor k_cache,
                                  citrus_tensor v_cache, int32_t cache_len, int32_t k, citrus_tensor k_new,
                                  citrus_tensor v_new, int32_t* idx, void* hip_stream) {
  CITRUS_TRY(check_evict_args(cfg, q, rows, k_cache, v_cache, cache_len, k, k_new, v_new));
  const StaticEvictLayout sl = static_evict_layout(cfg, rows, cache_len, k);
  if (sl.total > kStaticScratchBytes) return CITRUS_ERR_WORKSPACE;  // beyond the fixed array: use citrus_evict_cache
  char* base = nullptr;
  CITRUS_TRY(static_scratch_base(&base));
  if (idx == nullptr) idx = reinterpret_cast<int32_t*>(base + sl.idx);
  const Scratch scratch{reinterpret_cast<float*>(base + sl.lse),
                        instr_score_mfma_workspace_floats(dims_of(cfg), rows, cache_len)};
  return do_evict_cache(cfg, q, rows, k_cache, v_cache, cache_len, k, k_new, v_new, idx, scratch,
                        reinterpret_cast<float*>(base + sl.score), static_cast<hipStream_t>(hip_stream));
}

int32_t citrus_rope(const citrus_config* cfg, citrus_tensor x, int32_t heads, int32_t rows, int32_t pos0,
                    citrus_tensor y, void* hip_stream) {
  CITRUS_TRY(check_config(cfg));
  if (heads < 1 || heads > 65535 || rows < 0 || pos0 < 0) return CITRUS_ERR_SHAPE;
  CITRUS_TRY(check_tensor(cfg, x, rows, false));
  CITRUS_TRY(check_tensor(cfg, y, rows, false));
  return hip_status(launch_rope(cfg->dtype, dims_of(cfg), make_view(x), make_view(y), heads, rows, pos0,
                                rope_base_of(cfg), static_cast<hipStream_t>(hip_stream)));
}

int32_t citrus_decode_step(const citrus_config* cfg, citrus_tensor q, citrus_tensor k_new, citrus_tensor v_new,
                           citrus_tensor k_cache, citrus_tensor v_cache, int32_t cache_len, citrus_tensor out,
                           void* workspace, size_t workspace_bytes, void* hip_stream) {
  CITRUS_TRY(check_config(cfg));
  if (cache_len < 0 || cache_len >= cfg->cache_capacity) return CITRUS_ERR_SHAPE;
  CITRUS_TRY(check_tensor(cfg, q, 1, false));
  CITRUS_TRY(check_tensor(cfg, k_new, 1, false));
  CITRUS_TRY(check_tensor(cfg, v_new, 1, false));
  CITRUS_TRY(check_tensor(cfg, k_cache, cache_len + 1, false));
  CITRUS_TRY(check_tensor(cfg, v_cache, cache_len + 1, false));
  CITRUS_TRY(check_tensor(cfg, out, 1, false));
  if (k_new.ptr == k_cache.ptr || v_new.ptr == v_cache.ptr) return CITRUS_ERR_SHAPE;
  CITRUS_TRY(check_workspace(cfg, workspace, workspace_bytes));
  const Dims dm = dims_of(cfg);
  const Workspace wl = workspace_layout(cfg);
  char* ws = static_cast<char*>(workspace);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  // candidates: the cache rows, then the new token's own state
  Segments ks = segments(k_cache, cache_len, k_new, 1), vs = segments(v_cache, cache_len, v_new, 1);
  ks.cache = make_view(k_cache);  // also when it is empty: row cache_len of it is written
  vs.cache = make_view(v_cache);
  // the token's state also becomes row cache_len of the cache (nothing is evicted while the response is
  // generated): inside the same launch on the MFMA path, by a one-row gather otherwise
  if (decode_mfma_supported(cfg->dtype, dm))
    return hip_status(launch_decode_mfma(dm, make_view(q), ks, vs, make_view(out),
                                         reinterpret_cast<float*>(ws + wl.decode), /*append_token=*/1, st));
  CITRUS_TRY(hip_status(run_attn(cfg, dm, make_view(q), 1, ks, vs, /*causal=*/1, make_view(out), nullptr, st)));
  int32_t* one = reinterpret_cast<int32_t*>(ws + wl.iota);
  CITRUS_TRY(hip_status(launch_iota(one, cache_len, 1, st)));
  return hip_status(launch_compact(elem_bytes(cfg->dtype), dm, ks, vs, one, /*idx_pitch=*/0, /*idx_heads=*/1, 1,
                                   make_view(rows_from(k_cache, cache_len, cfg->dtype)),
                                   make_view(rows_from(v_cache, cache_len, cfg->dtype)), st));
}

int32_t citrus_score_accumulate(const citrus_config* cfg, float* score, int32_t n, const float* acc,
                                int32_t cache_len, void* hip_stream) {
  CITRUS_TRY(check_config(cfg));
  if (score == nullptr || acc == nullptr) return CITRUS_ERR_NULL;
  if (n < 1 || n > cfg->cache_capacity + cfg->chunk_len) return CITRUS_ERR_SHAPE;
  if (cache_len < 0 || cache_len > n || cache_len > cfg->cache_capacity) return CITRUS_ERR_SHAPE;
  return hip_status(launch_score_add(dims_of(cfg), score, acc, n, cache_len, cfg->cache_capacity,
                                     static_cast<hipStream_t>(hip_stream)));
}

int32_t citrus_score_gather(const citrus_config* cfg, const float* score, int32_t n, const int32_t* idx,
                            int32_t idx_pitch, int32_t m, float* acc_new, void* hip_stream) {
  CITRUS_TRY(check_config(cfg));
  if (score == nullptr || idx == nullptr || acc_new == nullptr) return CITRUS_ERR_NULL;
  if (n < 1 || n > cfg->cache_capacity + cfg->chunk_len) return CITRUS_ERR_SHAPE;
  if (m < 1 || m > cfg->cache_capacity || idx_pitch < m) return CITRUS_ERR_SHAPE;
  return hip_status(launch_score_gather(dims_of(cfg), score, idx, acc_new, n, m, idx_pitch, sel_heads(cfg),
                                        cfg->cache_capacity, static_cast<hipStream_t>(hip_stream)));
}

int32_t citrus_topk_select(const citrus_config* cfg, const float* score, int32_t n, int32_t k, int32_t* idx,
                           void* workspace, size_t workspace_bytes, void* hip_stream) {
  (void)workspace;
  (void)workspace_bytes;
  CITRUS_TRY(check_config(cfg));
  if (score == nullptr || idx == nullptr) return CITRUS_ERR_NULL;
  if (n < 1 || k < 1) return CITRUS_ERR_SHAPE;
  return do_topk(cfg, score, n, k, idx, static_cast<hipStream_t>(hip_stream));
}

int32_t citrus_kv_compact(const citrus_config* cfg, citrus_tensor k_cache, citrus_tensor v_cache, int32_t cache_len,
                          citrus_tensor k_chunk, citrus_tensor v_chunk, int32_t chunk_len, const int32_t* idx,
                          int32_t idx_pitch, int32_t m, citrus_tensor k_new, citrus_tensor v_new, void* hip_stream) {
  CITRUS_TRY(check_config(cfg));
  CITRUS_TRY(check_lengths(cfg, cache_len, chunk_len));
  if (idx == nullptr) return CITRUS_ERR_NULL;
  if (m < 1 || m > cfg->cache_capacity || idx_pitch < m) return CITRUS_ERR_SHAPE;
  CITRUS_TRY(check_tensor(cfg, k_chunk, chunk_len, false));
  CITRUS_TRY(check_tensor(cfg, v_chunk, chunk_len, false));
  CITRUS_TRY(check_tensor(cfg, k_cache, cache_len, cache_len == 0));
  CITRUS_TRY(check_tensor(cfg, v_cache, cache_len, cache_len == 0));
  CITRUS_TRY(check_tensor(cfg, k_new, m, false));
  CITRUS_TRY(check_tensor(cfg, v_new, m, false));
  if (k_new.ptr == k_cache.ptr || v_new.ptr == v_cache.ptr || k_new.ptr == k_chunk.ptr || v_new.ptr == v_chunk.ptr)
    return CITRUS_ERR_SHAPE;
  const Dims dm = dims_of(cfg);
  return do_compact(cfg, dm, segments(k_cache, cache_len, k_chunk, chunk_len),
                    segments(v_cache, cache_len, v_chunk, chunk_len), idx, idx_pitch, m, k_new, v_new,
                    static_cast<hipStream_t>(hip_stream));
}

int32_t citrus_resident_provider(void* user, int32_t chunk_index, void* hip_stream, citrus_chunk_io* io) {
  (void)hip_stream;
  if (user == nullptr || io == nullptr || chunk_index < 0) return -1;
  const citrus_resident_doc* d = static_cast<const citrus_resident_doc*>(user);
  if (d->chunk_len < 1 || d->doc_len < 0) return -1;
  const int64_t lo = static_cast<int64_t>(chunk_index) * d->chunk_len;
  if (lo >= d->doc_len) return 1;
  const int64_t hi = lo + d->chunk_len < d->doc_len ? lo + d->chunk_len : d->doc_len;
  if (d->dtype != CITRUS_F32 && d->dtype != CITRUS_BF16) return -1;
  const int esize = elem_bytes(d->dtype);
  auto advance = [](citrus_tensor t, int64_t rows, int esz) {
    t.ptr = static_cast<char*>(t.ptr) + rows * t.stride_s * esz;
    return t;
  };
  io->q = advance(d->q, lo, esize);
  io->k = advance(d->k, lo, esize);
  io->v = advance(d->v, lo, esize);
  io->out = advance(d->out, lo, esize);
  io->q_instr = d->q_instr;
  io->q_instr.ptr = static_cast<char*>(d->q_instr.ptr) + static_cast<int64_t>(chunk_index) * d->q_instr_stride_chunk * esize;
  io->chunk_len = static_cast<int32_t>(hi - lo);
  return 0;
}

int32_t citrus_process_document(const citrus_config* cfg, citrus_chunk_provider next, void* user,
                                int32_t first_chunk, int32_t max_chunks, const citrus_tensor* k_cache,
                                const citrus_tensor* v_cache, const citrus_tensor* k_cache_lm,
                                const citrus_tensor* v_cache_lm, int32_t* cache_len, int32_t* cache_len_lm,
                                int32_t* buffer_index, int32_t* buffer_index_lm, float* const* acc_score,
                                int32_t* idx_history,
                                int32_t* idx_history_lm, int32_t* chunks_done, void* const* phase_events,
                                void* workspace, size_t workspace_bytes, void* hip_stream,
                                const citrus_side_stream* side) {
  CITRUS_TRY(check_config(cfg));
  if (side != nullptr && (side->stream == nullptr || side->fork_event == nullptr || side->join_event == nullptr))
    return CITRUS_ERR_NULL;
  if (next == nullptr || k_cache == nullptr || v_cache == nullptr || cache_len == nullptr || buffer_index == nullptr)
    return CITRUS_ERR_NULL;
  const bool dual = cfg->cache_mode == CITRUS_CACHE_DUAL;
  const bool standard = cfg->cache_mode == CITRUS_CACHE_STANDARD;
  if (dual && (k_cache_lm == nullptr || v_cache_lm == nullptr || cache_len_lm == nullptr || buffer_index_lm == nullptr))
    return CITRUS_ERR_NULL;
  const bool accumulated = cfg->score_mode == CITRUS_SCORE_ACCUMULATED;
  if (accumulated && (acc_score == nullptr || acc_score[0] == nullptr || acc_score[1] == nullptr)) return CITRUS_ERR_NULL;
  if (accumulated && acc_score[0] == acc_score[1]) return CITRUS_ERR_SHAPE;
  if (first_chunk < 0) return CITRUS_ERR_SHAPE;
  for (int i = 0; i < 2; ++i) {
    CITRUS_TRY(check_tensor(cfg, k_cache[i], cfg->cache_capacity, false));
    CITRUS_TRY(check_tensor(cfg, v_cache[i], cfg->cache_capacity, false));
    if (dual) {
      CITRUS_TRY(check_tensor(cfg, k_cache_lm[i], cfg->cache_capacity, false));
      CITRUS_TRY(check_tensor(cfg, v_cache_lm[i], cfg->cache_capacity, false));
    }
  }
  if (k_cache[0].ptr == k_cache[1].ptr || v_cache[0].ptr == v_cache[1].ptr) return CITRUS_ERR_SHAPE;
  // a cache run in the printed order still holds the previous chunk between two steps
  const bool paper_order = evict_then_append(cfg);
  const int held = paper_order ? cfg->chunk_len : 0;
  if (*cache_len < 0 || *cache_len > cfg->budget + (standard ? held : 0) || (*buffer_index != 0 && *buffer_index != 1))
    return CITRUS_ERR_SHAPE;
  if (dual && (*cache_len_lm < 0 || *cache_len_lm > cfg->budget_lm + held ||
               (*buffer_index_lm != 0 && *buffer_index_lm != 1)))
    return CITRUS_ERR_SHAPE;
  CITRUS_TRY(check_workspace(cfg, workspace, workspace_bytes));

  const Dims dm = dims_of(cfg);
  const Workspace wl = workspace_layout(cfg);
  char* ws = static_cast<char*>(workspace);
  float* lse_chunk = reinterpret_cast<float*>(ws + wl.lse_chunk);
  const Scratch lse_instr{reinterpret_cast<float*>(ws + wl.lse_instr), score_scratch_floats(cfg, cfg->instr_len)};
  float* lse_cache = reinterpret_cast<float*>(ws + wl.lse_cache);
  int32_t* iota_ws = reinterpret_cast<int32_t*>(ws + wl.iota);
  float* score = reinterpret_cast<float*>(ws + wl.score);
  float* score_lm = reinterpret_cast<float*>(ws + wl.score_lm);
  int32_t* idx_ws = reinterpret_cast<int32_t*>(ws + wl.idx);
  int32_t* idx_lm_ws = reinterpret_cast<int32_t*>(ws + wl.idx_lm);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const size_t units_sel = static_cast<size_t>(cfg->batch) * cfg->layers * sel_heads(cfg);

  int n_c = *cache_len, cur = *buffer_index;
  int n_c_lm = dual ? *cache_len_lm : 0, cur_lm = dual ? *buffer_index_lm : 0;
  int done = 0;
  citrus_status status = CITRUS_OK;
  // selection and gather of the single-cache modes next to the chunk attention, on the caller's second stream
  const bool overlap = side != nullptr && !dual && !standard;
  hipStream_t st_side = overlap ? static_cast<hipStream_t>(side->stream) : st;
  auto mark_on = [&](hipStream_t stream, int step, int phase) {
    if (phase_events != nullptr && phase_events[step * CITRUS_EVENTS_PER_STEP + phase] != nullptr)
      (void)hipEventRecord(static_cast<hipEvent_t>(phase_events[step * CITRUS_EVENTS_PER_STEP + phase]), stream);
  };
  auto mark = [&](int step, int phase) { mark_on(st, step, phase); };

  // One step of a cache that the document's own chunks evict (Section 4.1): the second cache of DUAL, the
  // only cache of STANDARD.  Marks phases 1..4.
  struct ChunkEvicted {
    const citrus_tensor *k, *v;  // ping-pong pair
    int* len;
    int* cur;
    int budget;
    float* score;
    int32_t* idx;  // where this step's selection goes (pitch = budget)
  };
  auto chunk_evicted_step = [&](const ChunkEvicted& t, const citrus_chunk_io& io_in, int c) -> citrus_status {
    const int n_old = *t.len, from = *t.cur, to = from ^ 1;
    const Segments kl = segments(t.k[from], n_old, io_in.k, c), vl = segments(t.v[from], n_old, io_in.v, c);
    // What the chunk's attention and its scores read.  With the position shift: copies rotated to the
    // positions of THIS cache (its state j -> j, chunk token t -> n_old + t); the gathers below keep moving
    // the unrotated keys.
    citrus_chunk_io io = io_in;
    Segments kl_att = kl;
    citrus_tensor k_cache_att = t.k[from];
    if (cfg->position_shift) {
      const float base = rope_base_of(cfg);
      const int n_all = n_old + c;
      const citrus_tensor k_rot = dense_tensor(ws + wl.k_rot_lm, cfg->layers, cfg->kv_heads, n_all, cfg->head_dim);
      const citrus_tensor k_rot_chunk = rows_from(k_rot, n_old, cfg->dtype);
      io.q = dense_tensor(ws + wl.q_rot, cfg->layers, cfg->q_heads, c, cfg->head_dim);
      const RopeJob jobs[3] = {{kl.cache, make_view(k_rot), cfg->kv_heads, n_old, 0},  // skipped while the cache is empty
                               {kl.chunk, make_view(k_rot_chunk), cfg->kv_heads, c, n_old},
                               {make_view(io_in.q), make_view(io.q), cfg->q_heads, c, n_old}};
      CITRUS_TRY(hip_status(launch_rope_batch(cfg->dtype, dm, jobs, 3, base, st)));
      kl_att = segments(k_rot, n_old, k_rot_chunk, c);
      k_cache_att = k_rot;
    }
    if (paper_order) {
      // the order Section 4.1 prints: encode the chunk given the cache (it still holds the whole previous
      // chunk), evict the cache by the chunk's attention to it, then put the chunk in
      const int kept = n_old < t.budget ? n_old : t.budget;
      const bool evicts = n_old > t.budget;
      // the rows' normalisers over the cache alone come out of the attention launch
      CITRUS_TRY(do_chunk_attn(cfg, dm, io.q, kl_att, vl, io.out, nullptr, nullptr, evicts ? lse_cache : nullptr, st));
      mark(done, 1);
      if (evicts) CITRUS_TRY(do_cache_score(cfg, dm, io.q, c, k_cache_att, n_old, lse_cache, Scratch{nullptr, 0}, t.score, st));
      mark(done, 2);
      if (n_old > 0) CITRUS_TRY(do_topk(cfg, t.score, n_old, t.budget, t.idx, st));
      mark(done, 3);
      // kept cache states first, then the chunk's states behind them (positions n_old .. of the candidates)
      if (kept > 0) CITRUS_TRY(do_compact(cfg, dm, kl, vl, t.idx, t.budget, kept, t.k[to], t.v[to], st));
      CITRUS_TRY(hip_status(launch_iota(iota_ws, n_old, c, st)));
      CITRUS_TRY(hip_status(launch_compact(elem_bytes(cfg->dtype), dm, kl, vl, iota_ws, /*idx_pitch=*/0,
                                           /*idx_heads=*/1, c, make_view(rows_from(t.k[to], kept, cfg->dtype)),
                                           make_view(rows_from(t.v[to], kept, cfg->dtype)), st)));
      mark(done, 4);
      *t.len = kept + c;
    } else {
      // the chunk attends over [cache ; chunk] and scores all of it itself; eviction in the same step
      const int n_new = n_old + c;
      const int kept = n_new < t.budget ? n_new : t.budget;
      CITRUS_TRY(do_chunk_attn(cfg, dm, io.q, kl_att, vl, io.out, lse_chunk, nullptr, nullptr, st));
      mark(done, 1);
      CITRUS_TRY(hip_status(run_colsum(cfg, dm, make_view(io.q), c, kl_att, /*causal=*/1, lse_chunk, t.score, st)));
      mark(done, 2);
      CITRUS_TRY(do_topk(cfg, t.score, n_new, t.budget, t.idx, st));
      mark(done, 3);
      CITRUS_TRY(do_compact(cfg, dm, kl, vl, t.idx, t.budget, kept, t.k[to], t.v[to], st));
      mark(done, 4);
      *t.len = kept;
    }
    *t.cur = to;
    return CITRUS_OK;
  };

  for (; max_chunks < 0 || done < max_chunks; ++done) {
    citrus_chunk_io io;
    memset(&io, 0, sizeof(io));
    const int32_t rc = next(user, first_chunk + done, hip_stream, &io);
    if (rc == 1) break;
    if (rc != 0) { status = CITRUS_ERR_PROVIDER; break; }
    const int c = io.chunk_len;
    if (c < 1 || c > cfg->chunk_len) { status = CITRUS_ERR_SHAPE; break; }
    if ((status = check_tensor(cfg, io.q, c, false)) != CITRUS_OK) break;
    if ((status = check_tensor(cfg, io.k, c, false)) != CITRUS_OK) break;
    if ((status = check_tensor(cfg, io.v, c, false)) != CITRUS_OK) break;
    if ((status = check_tensor(cfg, io.q_instr, cfg->instr_len, /*may_be_null=*/standard)) != CITRUS_OK) break;
    if ((status = check_tensor(cfg, io.out, c, false)) != CITRUS_OK) break;

    mark(done, 0);
    if (standard) {
      // Standard CSE alone: the instruction takes no part in the encoding of the document
      int32_t* idx = idx_history ? idx_history + static_cast<size_t>(done) * units_sel * cfg->budget : idx_ws;
      const ChunkEvicted t{k_cache, v_cache, &n_c, &cur, cfg->budget, score, idx};
      if ((status = chunk_evicted_step(t, io, c)) != CITRUS_OK) break;
      for (int p = 5; p <= 7; ++p) mark(done, p);
      continue;
    }

    // instruction (or only) cache: candidates [cache ; chunk]
    const Segments ks = segments(k_cache[cur], n_c, io.k, c), vs = segments(v_cache[cur], n_c, io.v, c);
    const int n = n_c + c;
    const int m = n < cfg->budget ? n : cfg->budget;
    // What attention and scores read.  With the position shift: copies rotated to this step's
    // positions (candidate j -> j, chunk query t -> n_c + t, instruction query u -> n + u); the
    // selection still gathers the unrotated keys.
    Segments ks_att = ks;
    citrus_tensor q_att = io.q, qi_att = io.q_instr;
    // (DUAL: the chunk attends over the language-modelling cache, so its queries are rotated to that cache's
    // positions inside chunk_evicted_step)
    const int q_rope_pos0 = cfg->position_shift && !dual && mfma_path_supported(cfg->dtype, dm) ? n_c : -1;
    if (cfg->position_shift) {
      const float base = rope_base_of(cfg);
      const citrus_tensor k_rot = dense_tensor(ws + wl.k_rot, cfg->layers, cfg->kv_heads, n, cfg->head_dim);
      q_att = dense_tensor(ws + wl.q_rot, cfg->layers, cfg->q_heads, c, cfg->head_dim);
      qi_att = dense_tensor(ws + wl.qi_rot, cfg->layers, cfg->q_heads, cfg->instr_len, cfg->head_dim);
      const citrus_tensor k_rot_chunk = rows_from(k_rot, n_c, cfg->dtype);
      // one launch for the step's rotations; the MFMA attention kernel rotates its query rows itself while they
      // are staged in LDS, and with two caches the chunk's queries belong to the other cache's thread
      const bool rotate_q_here = !dual && q_rope_pos0 < 0;
      const RopeJob jobs[4] = {{ks.cache, make_view(k_rot), cfg->kv_heads, n_c, 0},  // skipped while the cache is empty
                               {ks.chunk, make_view(k_rot_chunk), cfg->kv_heads, c, n_c},
                               {make_view(io.q_instr), make_view(qi_att), cfg->q_heads, cfg->instr_len, n},
                               {make_view(io.q), make_view(q_att), cfg->q_heads, rotate_q_here ? c : 0, n_c}};
      if ((status = hip_status(launch_rope_batch(cfg->dtype, dm, jobs, 4, base, st))) != CITRUS_OK) break;
      if (!rotate_q_here) q_att = io.q;
      ks_att = segments(k_rot, n_c, k_rot_chunk, c);
    }
    int32_t* idx = idx_history ? idx_history + static_cast<size_t>(done) * units_sel * cfg->budget : idx_ws;
    // instruction score, selection and gather of the instruction (or only) cache; the last two on `sel_st`
    auto score_step = [&]() -> citrus_status {
      CITRUS_TRY(do_instr_score(cfg, dm, qi_att, ks_att, lse_instr, score, st));
      if (accumulated) CITRUS_TRY(hip_status(launch_score_add(dm, score, acc_score[cur], n, n_c, cfg->cache_capacity, st)));
      mark(done, 5);
      return CITRUS_OK;
    };
    auto select_gather_step = [&](hipStream_t sel_st) -> citrus_status {
      CITRUS_TRY(do_topk(cfg, score, n, cfg->budget, idx, sel_st));
      mark_on(sel_st, done, 6);
      CITRUS_TRY(do_compact(cfg, dm, ks, vs, idx, cfg->budget, m, k_cache[cur ^ 1], v_cache[cur ^ 1], sel_st));
      if (accumulated)
        CITRUS_TRY(hip_status(launch_score_gather(dm, score, idx, acc_score[cur ^ 1], n, m, cfg->budget, sel_heads(cfg),
                                                  cfg->cache_capacity, sel_st)));
      mark_on(sel_st, done, 7);
      return CITRUS_OK;
    };
    if (overlap) {
      if ((status = score_step()) != CITRUS_OK) break;
      if ((status = hip_status(hipEventRecord(static_cast<hipEvent_t>(side->fork_event), st))) != CITRUS_OK) break;
      if ((status = hip_status(hipStreamWaitEvent(st_side, static_cast<hipEvent_t>(side->fork_event), 0))) != CITRUS_OK) break;
      // From here on the side stream may hold work of this step.  Whatever fails below, hip_stream is ordered
      // behind that work before the call returns: the next step, and whatever the caller enqueues after the
      // call, reads the buffer the gather fills.
      status = select_gather_step(st_side);
      const hipError_t joined = hipEventRecord(static_cast<hipEvent_t>(side->join_event), st_side);
      if (status == CITRUS_OK) {
        status = do_chunk_attn(cfg, dm, q_att, ks_att, vs, io.out, nullptr, nullptr, nullptr, st, q_rope_pos0);
        for (int p = 1; p <= 4; ++p) mark(done, p);
      }
      hipError_t ordered = joined;
      if (ordered == hipSuccess) ordered = hipStreamWaitEvent(st, static_cast<hipEvent_t>(side->join_event), 0);
      if (ordered != hipSuccess) {
        // the event could not order the two streams: drain the side stream on the host (error path only)
        (void)hipStreamSynchronize(st_side);
        if (status == CITRUS_OK) status = CITRUS_ERR_DEVICE;
      }
      if (status != CITRUS_OK) break;
    } else {
      if (dual) {
        int32_t* idx_lm = idx_history_lm ? idx_history_lm + static_cast<size_t>(done) * units_sel * cfg->budget_lm : idx_lm_ws;
        const ChunkEvicted t{k_cache_lm, v_cache_lm, &n_c_lm, &cur_lm, cfg->budget_lm, score_lm, idx_lm};
        if ((status = chunk_evicted_step(t, io, c)) != CITRUS_OK) break;
      } else {
        if ((status = do_chunk_attn(cfg, dm, q_att, ks_att, vs, io.out, nullptr, nullptr, nullptr, st, q_rope_pos0)) !=
            CITRUS_OK)
          break;
        for (int p = 1; p <= 4; ++p) mark(done, p);
      }
      if ((status = score_step()) != CITRUS_OK) break;
      if ((status = select_gather_step(st)) != CITRUS_OK) break;
    }
    cur ^= 1;
    n_c = m;
  }
  *cache_len = n_c;
  *buffer_index = cur;
  if (dual) {
    *cache_len_lm = n_c_lm;
    *buffer_index_lm = cur_lm;
  }
  if (chunks_done != nullptr) *chunks_done = done;
  return status;
}

}  // extern "C"
