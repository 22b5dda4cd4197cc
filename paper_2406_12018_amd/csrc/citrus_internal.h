// Internal declarations shared by the translation units of libcitrus.so.
// Not part of the public ABI (see include/citrus.h for that).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "citrus.h"

namespace citrus {

// A strided [B, L, H, S, d] view in element units; d is contiguous.
struct View {
  const void* ptr;
  int64_t sb, sl, sh, ss;
};

inline View make_view(const citrus_tensor& t) { return View{t.ptr, t.stride_b, t.stride_l, t.stride_h, t.stride_s}; }

// Problem sizes every kernel launcher receives.
struct Dims {
  int B, L, Hq, Hkv, G, D;
  float scale;  // softmax scale (already resolved, never 0)
};

// The candidate keys/values of a step: cache rows then chunk rows.
struct Segments {
  View cache;   // [B, L, Hkv, >= n_c, d]
  View chunk;   // [B, L, Hkv, c, d]
  int n_c;      // valid cache rows
  int c;        // chunk rows
};

inline citrus_status hip_status(hipError_t e) { return e == hipSuccess ? CITRUS_OK : CITRUS_ERR_DEVICE; }

// ---- generic VALU kernels (f32 and bf16 element types), attn_generic.hip ----
// rows: number of query rows per head; causal != 0 -> row t sees candidates j <= n_c + t.
// out may be NULL (log-sum-exp only); lse may be NULL.
hipError_t launch_attn_generic(int dtype, const Dims& dm, View q, int rows, Segments kseg, Segments vseg, int causal,
                               View out, float* lse, hipStream_t st);
// score[b,l,g,j] = sum_{h in g} sum_{t<rows} exp(scale*q.k - lse[b,l,h,t]) (0 where masked)
hipError_t launch_colsum_generic(int dtype, const Dims& dm, View q, int rows, Segments kseg, int causal,
                                 const float* lse, float* score, hipStream_t st);

// ---- bf16 MFMA kernels (head_dim 128), attn_mfma.hip ----
bool mfma_path_supported(int dtype, const Dims& dm);
// key_splits > 1: log-sum-exp only, one partial (log2-domain maximum, sum) pair per key range
// and row in part[split][B*L*Hq*rows]; key_splits == 1: out and/or lse (natural log) as given.
// lse_cache (optional): per row, the log-sum-exp over the cache states alone, a by-product of the
// causal kernel with output when attn_mfma_emits_cache_lse() holds (cache ends on a 32-key boundary).
bool attn_mfma_emits_cache_lse(const Segments& kseg, int causal, View out);
// q_rope_pos0 >= 0 (kernel with output only): the query rows are given without rotary embedding and are
// rotated to positions q_rope_pos0 + row inside the kernel, with the bits launch_rope would give.
hipError_t launch_attn_mfma(const Dims& dm, View q, int rows, Segments kseg, Segments vseg, int causal, View out,
                            float* lse, float* lse_cache, int key_splits, float2* part, hipStream_t st,
                            int q_rope_pos0 = -1, float rope_base = 0.f);
// normaliser per row from lse (natural log) or, if part != NULL, merged from key_splits partial pairs
hipError_t launch_colsum_mfma(const Dims& dm, View q, int rows, Segments kseg, int causal, const float* lse,
                              int key_splits, const float2* part, float* score, hipStream_t st);
// Most ranges of key tiles a two-launch score splits the keys of a row into (one workgroup per range).
constexpr int kMaxKeySplits = 8;
// Floats of scratch that cover every launch_instr_score_mfma call with at most `rows` query rows per head over
// at most n keys (the launcher picks its kernel by the call's own shape, and the kernels' needs do not grow
// together: a block sized for the largest shape alone could be too small for a smaller one).
size_t instr_score_mfma_workspace_floats(const Dims& dm, int rows, int n);
// `workspace_floats`: what the block behind `workspace` holds; a kernel whose scratch does not fit is not
// chosen, and hipErrorInvalidValue comes back if none fits.
hipError_t launch_instr_score_mfma(const Dims& dm, View q, int rows, Segments kseg, float* workspace,
                                   size_t workspace_floats, float* score, hipStream_t st);

// ---- instruction score with one q.k product per (row, key): row strips kept on chip, instr_strip.hip ----
// taken for this shape, given a scratch block of workspace_floats floats?
bool instr_strip_supported(const Dims& dm, const View& q, int rows, const Segments& kseg, size_t workspace_floats);
// largest scratch any supported launch with at most `rows` rows and at most n keys writes (0: none is supported)
size_t instr_strip_workspace_floats(const Dims& dm, int rows, int n);
hipError_t launch_instr_strip(const Dims& dm, View q, int rows, Segments kseg, float* workspace, size_t workspace_floats,
                              float* score, hipStream_t st);

// ---- bf16 MFMA decoding step (head_dim 128), decode_attn.hip ----
bool decode_mfma_supported(int dtype, const Dims& dm);
size_t decode_mfma_workspace_floats(const Dims& dm);
// One query row per head over [cache ; the new token's row] (kseg.c == 1); workspace holds the partial
// results of the key ranges (decode_mfma_workspace_floats).  append_token != 0: the token's K/V row is
// also written to row kseg.n_c of the cache tensors (which must have room for it).
hipError_t launch_decode_mfma(const Dims& dm, View q, Segments kseg, Segments vseg, View out, float* workspace,
                              int append_token, hipStream_t st);

// ---- rotary embedding at explicit positions, rope.hip ----
// y[b,l,h,s,:] = RoPE(x[b,l,h,s,:], pos0 + s) for h < heads, s < rows; y may be x itself.
hipError_t launch_rope(int dtype, const Dims& dm, View x, View y, int heads, int rows, int pos0, float base,
                       hipStream_t st);
// Up to kMaxRopeJobs rotations in one launch (bf16; f32 takes one launch each): the keys and queries of a step.
// A job with rows <= 0 is skipped.
constexpr int kMaxRopeJobs = 4;
struct RopeJob {
  View x, y;
  int heads, rows, pos0;
};
hipError_t launch_rope_batch(int dtype, const Dims& dm, const RopeJob* jobs, int count, float base, hipStream_t st);

// Kernels that take more than 64 KB of dynamic LDS need their limit raised once per device.  `state` is a
// static object next to the launch; the current device's slot remembers the largest size granted.  The
// slots are atomics (relaxed order is enough: the value only saves a repeated hipFuncSetAttribute, which
// the runtime serialises itself), so host threads may call the launchers concurrently.  Every launcher
// asks for ONE size per kernel (its maximum), so two threads can never lower each other's limit.
constexpr int kMaxDevices = 64;
struct LdsLimit {
  std::atomic<int> granted[kMaxDevices] = {};
};
inline hipError_t raise_lds_limit(LdsLimit& state, const void* kernel, int bytes) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool tracked = dev >= 0 && dev < kMaxDevices;
  if (tracked && state.granted[dev].load(std::memory_order_relaxed) >= bytes) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess && tracked) {
    int seen = state.granted[dev].load(std::memory_order_relaxed);
    while (seen < bytes && !state.granted[dev].compare_exchange_weak(seen, bytes, std::memory_order_relaxed)) {
    }
  }
  return e;
}

// ---- selection and compaction, select_compact.hip ----
// units = B*L*Hsel; score rows are [units*(per_layer?Hkv:1)] x n.
hipError_t launch_topk(const float* score, int units, int heads_to_sum, int n, int k, int forced, int32_t* idx,
                       hipStream_t st);
// p[i] = base + i for i < count
hipError_t launch_iota(int32_t* p, int base, int count, hipStream_t st);
// score [B*L*Hkv][n] += acc [B*L*Hkv][acc_pitch] on the first n_c candidates
hipError_t launch_score_add(const Dims& dm, float* score, const float* acc, int n, int n_c, int acc_pitch,
                            hipStream_t st);
// acc_new [B*L*Hkv][acc_pitch]: row r < m takes score[idx[r]] (idx as in launch_compact)
hipError_t launch_score_gather(const Dims& dm, const float* score, const int32_t* idx, float* acc_new, int n, int m,
                               int idx_pitch, int idx_heads, int acc_pitch, hipStream_t st);
hipError_t launch_compact(int elem_bytes, const Dims& dm, Segments kseg, Segments vseg, const int32_t* idx,
                          int idx_pitch, int idx_heads, int m, View k_new, View v_new, hipStream_t st);

}  // namespace citrus
