// Selection (Eq. (2)-(3): keep the k highest importance scores) and compaction
// (Eq. (3), (5): the evicted cache holds exactly the selected states).
#include "citrus_internal.h"

namespace citrus {
namespace {

constexpr int kSelThreads = 256;
constexpr int kSelWaves = kSelThreads / 64;

// Order-preserving map float -> uint32 (larger float <=> larger key).  -0 is
// folded onto +0 first so that equal values get equal keys.
__device__ inline uint32_t order_key(float f) {
  f += 0.0f;
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// The value a selection unit ranks for candidate j: one head's score, or the
// sum over the layer's KV heads taken in head order (layer-wise eviction).
__device__ inline float unit_score(const float* base, int heads_to_sum, int n, int j) {
  float s = base[j];
  for (int g = 1; g < heads_to_sum; ++g) s += base[static_cast<int64_t>(g) * n + j];
  return s;
}

// The key candidate j is ranked by.  The first `forced` candidates (the initial document states
// that are never evicted) rank above every score.
__device__ inline uint32_t unit_key(const float* base, int heads_to_sum, int n, int forced, int j) {
  return j < forced ? 0xffffffffu : order_key(unit_score(base, heads_to_sum, n, j));
}

// One workgroup per selection unit.  A radix select over the 32-bit order keys
// (4 passes of 8 bits, integer LDS histograms) finds the k-th largest key T;
// then one ordered pass emits, in ascending position, every candidate with
// key > T and the first (k - count(key > T)) candidates with key == T.  The
// result is exactly the top-k under (score descending, position ascending).
__global__ __launch_bounds__(kSelThreads) void topk_kernel(const float* score, int heads_to_sum, int n, int k,
                                                          int forced, int32_t* idx) {
  __shared__ int hist[256];
  __shared__ uint32_t s_prefix;
  __shared__ int s_need;
  __shared__ int wave_tot[2][kSelWaves];
  const int unit = blockIdx.x, tid = threadIdx.x;
  const float* base = score + static_cast<int64_t>(unit) * heads_to_sum * n;
  int32_t* out = idx + static_cast<int64_t>(unit) * k;

  if (n <= k) {  // nothing to evict: keep every candidate
    for (int j = tid; j < n; j += kSelThreads) out[j] = j;
    return;
  }

  uint32_t prefix = 0;  // bits of T fixed so far (high bits)
  int need = k;         // rank of T among the keys that match the prefix
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    hist[tid] = 0;  // kSelThreads == 256 bins
    __syncthreads();
    const uint32_t hi_mask = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
    for (int j = tid; j < n; j += kSelThreads) {
      const uint32_t key = unit_key(base, heads_to_sum, n, forced, j);
      if ((key & hi_mask) == prefix) atomicAdd(&hist[(key >> shift) & 0xff], 1);
    }
    __syncthreads();
    // Find the bin where the count of keys in higher bins first reaches `need`: thread t owns bin t,
    // computes the number of keys in bins above it with a suffix scan (wave shuffles + one LDS hop),
    // and the one bin with above < need <= above + own announces itself.
    {
      const int own = hist[tid];
      int incl = own;  // inclusive suffix sum within the wave: bins tid .. end of wave
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int v = __shfl_down(incl, o, 64);
        if ((tid % 64) + o < 64) incl += v;
      }
      if (tid % 64 == 0) wave_tot[0][tid / 64] = incl;  // total of this wave's 64 bins
      __syncthreads();
      int above = incl - own;
      for (int x = tid / 64 + 1; x < kSelWaves; ++x) above += wave_tot[0][x];
      if (above < need && need <= above + own) {
        s_prefix = prefix | (static_cast<uint32_t>(tid) << shift);
        s_need = need - above;
      }
    }
    __syncthreads();
    prefix = s_prefix;
    need = s_need;
    __syncthreads();
  }
  const uint32_t thr = prefix;  // key of the k-th best candidate
  // `need` = how many candidates with key == thr are kept (lowest positions first)

  const int lane = tid % 64, w = tid / 64;
  int kept_before = 0, eq_before = 0;
  for (int j0 = 0; j0 < n; j0 += kSelThreads) {
    const int j = j0 + tid;
    uint32_t key = 0;
    bool in = j < n;
    if (in) key = unit_key(base, heads_to_sum, n, forced, j);
    const bool gt = in && key > thr, eq = in && key == thr;
    const uint64_t eq_ballot = __ballot(eq);
    const uint64_t below = (1ull << lane) - 1ull;
    if (lane == 0) wave_tot[0][w] = __popcll(eq_ballot);
    __syncthreads();
    int eq_rank = eq_before + __popcll(eq_ballot & below);
    int eq_total = 0;
    for (int x = 0; x < kSelWaves; ++x) {
      if (x < w) eq_rank += wave_tot[0][x];
      eq_total += wave_tot[0][x];
    }
    const bool keep = gt || (eq && eq_rank < need);
    const uint64_t keep_ballot = __ballot(keep);
    if (lane == 0) wave_tot[1][w] = __popcll(keep_ballot);
    __syncthreads();
    int pos = kept_before + __popcll(keep_ballot & below);
    int keep_total = 0;
    for (int x = 0; x < kSelWaves; ++x) {
      if (x < w) pos += wave_tot[1][x];
      keep_total += wave_tot[1][x];
    }
    if (keep) out[pos] = j;
    kept_before += keep_total;
    eq_before += eq_total;
    __syncthreads();
  }
}

// The same selection for a unit whose keys fit the workgroup's registers (n <= ITEMS * THREADS): the scores
// are read once (candidate i * THREADS + tid is item i of thread tid), the four radix passes run on the
// registers with three barriers each (two histograms take turns, so clearing one needs no barrier of its own;
// the first 256 threads own the bins), and the ordered emission takes two barriers in all: per row of THREADS
// candidates and wave, the number of threshold-equal and then of kept candidates goes to LDS, and a
// candidate's rank is the sum of the counts in front of it.  Exactly the result of topk_kernel.
template <int ITEMS, int THREADS>
__device__ __forceinline__ void topk_regs_body(const float* score, int heads_to_sum, int n, int k, int forced,
                                               int32_t* idx) {
  constexpr int WAVES = THREADS / 64, kBins = 256, kBinWaves = kBins / 64;
  static_assert(THREADS >= kBins && ITEMS <= 32, "thread t < 256 owns bin t; one bit per item");
  __shared__ int hist[2][kBins];
  __shared__ uint32_t s_prefix;
  __shared__ int s_need;
  __shared__ int wave_tot[kBinWaves];
  __shared__ int row_cnt[2][ITEMS][WAVES];
  const int unit = blockIdx.x, tid = threadIdx.x, lane = tid % 64, w = tid / 64;
  const float* base = score + static_cast<int64_t>(unit) * heads_to_sum * n;
  int32_t* out = idx + static_cast<int64_t>(unit) * k;

  if (n <= k) {  // nothing to evict: keep every candidate
    for (int j = tid; j < n; j += THREADS) out[j] = j;
    return;
  }

  uint32_t key[ITEMS];
#pragma unroll
  for (int i = 0; i < ITEMS; ++i) {
    const int j = i * THREADS + tid;
    key[i] = j < n ? unit_key(base, heads_to_sum, n, forced, j) : 0u;
  }
  if (tid < kBins) hist[0][tid] = 0;
  __syncthreads();

  uint32_t prefix = 0;  // bits of T fixed so far (high bits)
  int need = k;         // rank of T among the keys that match the prefix
#pragma unroll
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    int* h = hist[pass & 1];
    if (tid < kBins) hist[(pass + 1) & 1][tid] = 0;  // the next pass's histogram; its last readers passed two barriers ago
    const uint32_t hi_mask = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
#pragma unroll
    for (int i = 0; i < ITEMS; ++i)
      if (i * THREADS + tid < n && (key[i] & hi_mask) == prefix) atomicAdd(&h[(key[i] >> shift) & 0xff], 1);
    __syncthreads();
    // thread t < 256 owns bin t: keys in higher bins = suffix sum (wave shuffles + one LDS hop)
    int own = 0, incl = 0;
    if (w < kBinWaves) {  // wave-uniform
      own = h[tid];
      incl = own;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int v = __shfl_down(incl, o, 64);
        if (lane + o < 64) incl += v;
      }
      if (lane == 0) wave_tot[w] = incl;
    }
    __syncthreads();
    if (w < kBinWaves) {
      int above = incl - own;
      for (int x = w + 1; x < kBinWaves; ++x) above += wave_tot[x];
      if (above < need && need <= above + own) {  // exactly one bin
        s_prefix = prefix | (static_cast<uint32_t>(tid) << shift);
        s_need = need - above;
      }
    }
    __syncthreads();
    prefix = s_prefix;
    need = s_need;
  }
  const uint32_t thr = prefix;  // key of the k-th best candidate; `need` of the candidates with that key are kept

  // set bits of a ballot below this lane (v_mbcnt: no per-lane mask to keep in registers)
  auto lanes_below = [](uint64_t ballot) {
    return static_cast<int>(__builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(ballot >> 32),
                                                      __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(ballot), 0u)));
  };
  // candidates of the same row and wave in front of this one (threshold-equal first, then kept): 0 .. 63, a byte each
  uint32_t rank_in_row[(ITEMS + 3) / 4] = {};
  auto set_rank = [&](int i, int r) { rank_in_row[i / 4] = (rank_in_row[i / 4] & ~(0xffu << (8 * (i % 4)))) | (static_cast<uint32_t>(r) << (8 * (i % 4))); };
  auto get_rank = [&](int i) { return static_cast<int>((rank_in_row[i / 4] >> (8 * (i % 4))) & 0xffu); };
#pragma unroll
  for (int i = 0; i < ITEMS; ++i) {
    if (i * THREADS >= n) break;  // block-uniform
    const bool eq = i * THREADS + tid < n && key[i] == thr;
    const uint64_t ballot = __ballot(eq);
    set_rank(i, lanes_below(ballot));
    if (lane == 0) row_cnt[0][i][w] = __popcll(ballot);
  }
  __syncthreads();
  uint32_t keep_bits = 0;
  int eq_before = 0;
#pragma unroll
  for (int i = 0; i < ITEMS; ++i) {
    if (i * THREADS >= n) break;
    int eq_rank = eq_before + get_rank(i);
#pragma unroll
    for (int x = 0; x < WAVES; ++x) {
      const int c = row_cnt[0][i][x];
      if (x < w) eq_rank += c;
      eq_before += c;
    }
    const bool in = i * THREADS + tid < n;
    const bool keep = in && (key[i] > thr || (key[i] == thr && eq_rank < need));
    const uint64_t ballot = __ballot(keep);
    set_rank(i, lanes_below(ballot));
    if (lane == 0) row_cnt[1][i][w] = __popcll(ballot);
    keep_bits |= keep ? (1u << i) : 0u;
    __builtin_amdgcn_sched_barrier(0);  // one row's counts in registers at a time (see the register budget below)
  }
  __syncthreads();
  int kept_before = 0;
#pragma unroll
  for (int i = 0; i < ITEMS; ++i) {
    if (i * THREADS >= n) break;
    int pos = kept_before + get_rank(i);
#pragma unroll
    for (int x = 0; x < WAVES; ++x) {
      const int c = row_cnt[1][i][x];
      if (x < w) pos += c;
      kept_before += c;
    }
    if (keep_bits & (1u << i)) out[pos] = i * THREADS + tid;
    __builtin_amdgcn_sched_barrier(0);
  }
}

// Six keys per thread (up to 1536 candidates: the Mistral-7B shape's 1280) fit 32 registers with one wave per
// SIMD: next to two waves of the chunk-attention kernel (240 registers each) a SIMD has 32 left, and with them
// these workgroups run beside an attention launch (the second-stream form of the chunk loop) instead of waiting
// for a compute unit of their own.  Eight keys need 34.
__global__ __launch_bounds__(kSelThreads) void topk_regs6_kernel(const float* score, int heads_to_sum, int n, int k,
                                                                int forced, int32_t* idx) {
  topk_regs_body<6, kSelThreads>(score, heads_to_sum, n, k, forced, idx);
}
__global__ __launch_bounds__(kSelThreads) void topk_regs8_kernel(const float* score, int heads_to_sum, int n, int k,
                                                                int forced, int32_t* idx) {
  topk_regs_body<8, kSelThreads>(score, heads_to_sum, n, k, forced, idx);
}
__global__ __launch_bounds__(kSelThreads) void topk_regs24_kernel(const float* score, int heads_to_sum, int n, int k,
                                                                 int forced, int32_t* idx) {
  topk_regs_body<24, kSelThreads>(score, heads_to_sum, n, k, forced, idx);
}

__global__ void iota_kernel(int32_t* p, int base, int count) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) p[i] = base + i;
}

// Accumulated scores: the sum a cache state carries is added to this step's score of the same candidate
// (chunk candidates start at their first score) ...
__global__ __launch_bounds__(256) void score_add_kernel(float* score, const float* acc, int n, int n_c, int acc_pitch,
                                                        int heads) {
  const int64_t u = static_cast<int64_t>(blockIdx.z) * heads + blockIdx.y;
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j < n_c) score[u * n + j] += acc[u * acc_pitch + j];
}
// ... and the kept states take their sums along: acc_new[r] = score[idx[r]].
__global__ __launch_bounds__(256) void score_gather_kernel(const float* score, const int32_t* idx, float* acc_new, int n,
                                                           int m, int idx_pitch, int idx_heads, int acc_pitch,
                                                           int heads) {
  const int g = blockIdx.y;
  const int64_t u = static_cast<int64_t>(blockIdx.z) * heads + g;
  const int r = blockIdx.x * 256 + threadIdx.x;
  if (r >= m) return;
  const int gi = idx_heads == 1 ? 0 : g;
  int j = idx[(static_cast<int64_t>(blockIdx.z) * idx_heads + gi) * idx_pitch + r];
  j = max(0, min(j, n - 1));  // a bad index must never become an out-of-bounds read
  acc_new[u * acc_pitch + r] = score[u * n + j];
}

// Row gather: every thread moves 16 bytes of a K row and 16 bytes of a V row.
template <int ROW_BYTES>
__global__ __launch_bounds__(256) void compact_kernel(Dims dm, Segments ks, Segments vs, int elem_bytes,
                                                      const int32_t* idx, int idx_pitch, int idx_heads, int m,
                                                      View k_new, View v_new) {
  constexpr int kLanesPerRow = ROW_BYTES / 16;
  constexpr int kRowsPerBlock = 256 / kLanesPerRow;
  const int g = blockIdx.y, b = blockIdx.z / dm.L, l = blockIdx.z % dm.L;
  const int r = blockIdx.x * kRowsPerBlock + threadIdx.x / kLanesPerRow;
  const int seg = threadIdx.x % kLanesPerRow;
  if (r >= m) return;
  const int gi = idx_heads == 1 ? 0 : g;
  int j = idx[(static_cast<int64_t>(blockIdx.z) * idx_heads + gi) * idx_pitch + r];
  j = max(0, min(j, ks.n_c + ks.c - 1));  // a bad index must never become an out-of-bounds read
  const int64_t unit_cache_k = b * ks.cache.sb + l * ks.cache.sl + g * ks.cache.sh;
  const int64_t unit_chunk_k = b * ks.chunk.sb + l * ks.chunk.sl + g * ks.chunk.sh;
  const int64_t unit_cache_v = b * vs.cache.sb + l * vs.cache.sl + g * vs.cache.sh;
  const int64_t unit_chunk_v = b * vs.chunk.sb + l * vs.chunk.sl + g * vs.chunk.sh;
  const char* ksrc;
  const char* vsrc;
  if (j < ks.n_c) {
    ksrc = static_cast<const char*>(ks.cache.ptr) + (unit_cache_k + static_cast<int64_t>(j) * ks.cache.ss) * elem_bytes;
    vsrc = static_cast<const char*>(vs.cache.ptr) + (unit_cache_v + static_cast<int64_t>(j) * vs.cache.ss) * elem_bytes;
  } else {
    const int jc = j - ks.n_c;
    ksrc = static_cast<const char*>(ks.chunk.ptr) + (unit_chunk_k + static_cast<int64_t>(jc) * ks.chunk.ss) * elem_bytes;
    vsrc = static_cast<const char*>(vs.chunk.ptr) + (unit_chunk_v + static_cast<int64_t>(jc) * vs.chunk.ss) * elem_bytes;
  }
  char* kdst = static_cast<char*>(const_cast<void*>(k_new.ptr)) +
               (b * k_new.sb + l * k_new.sl + g * k_new.sh + static_cast<int64_t>(r) * k_new.ss) * elem_bytes;
  char* vdst = static_cast<char*>(const_cast<void*>(v_new.ptr)) +
               (b * v_new.sb + l * v_new.sl + g * v_new.sh + static_cast<int64_t>(r) * v_new.ss) * elem_bytes;
  const uint4 kv = reinterpret_cast<const uint4*>(ksrc)[seg];
  const uint4 vv = reinterpret_cast<const uint4*>(vsrc)[seg];
  reinterpret_cast<uint4*>(kdst)[seg] = kv;
  reinterpret_cast<uint4*>(vdst)[seg] = vv;
}

template <int ROW_BYTES>
hipError_t compact_launch(int elem_bytes, const Dims& dm, Segments ks, Segments vs, const int32_t* idx,
                          int idx_pitch, int idx_heads, int m, View k_new, View v_new, hipStream_t st) {
  constexpr int kRowsPerBlock = 256 / (ROW_BYTES / 16);
  dim3 grid((m + kRowsPerBlock - 1) / kRowsPerBlock, dm.Hkv, dm.B * dm.L);
  hipLaunchKernelGGL((compact_kernel<ROW_BYTES>), grid, dim3(256), 0, st, dm, ks, vs, elem_bytes, idx, idx_pitch,
                     idx_heads, m, k_new, v_new);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_topk(const float* score, int units, int heads_to_sum, int n, int k, int forced, int32_t* idx,
                       hipStream_t st) {
  forced = min(forced, k);
  if (n <= 6 * kSelThreads)
    hipLaunchKernelGGL(topk_regs6_kernel, dim3(units), dim3(kSelThreads), 0, st, score, heads_to_sum, n, k, forced, idx);
  else if (n <= 8 * kSelThreads)
    hipLaunchKernelGGL(topk_regs8_kernel, dim3(units), dim3(kSelThreads), 0, st, score, heads_to_sum, n, k, forced, idx);
  else if (n <= 24 * kSelThreads)
    hipLaunchKernelGGL(topk_regs24_kernel, dim3(units), dim3(kSelThreads), 0, st, score, heads_to_sum, n, k, forced, idx);
  else
    hipLaunchKernelGGL(topk_kernel, dim3(units), dim3(kSelThreads), 0, st, score, heads_to_sum, n, k, forced, idx);
  return hipGetLastError();
}

hipError_t launch_iota(int32_t* p, int base, int count, hipStream_t st) {
  hipLaunchKernelGGL(iota_kernel, dim3((count + 255) / 256), dim3(256), 0, st, p, base, count);
  return hipGetLastError();
}

hipError_t launch_score_add(const Dims& dm, float* score, const float* acc, int n, int n_c, int acc_pitch,
                            hipStream_t st) {
  if (n_c <= 0) return hipSuccess;
  hipLaunchKernelGGL(score_add_kernel, dim3((n_c + 255) / 256, dm.Hkv, dm.B * dm.L), dim3(256), 0, st, score, acc, n,
                     n_c, acc_pitch, dm.Hkv);
  return hipGetLastError();
}

hipError_t launch_score_gather(const Dims& dm, const float* score, const int32_t* idx, float* acc_new, int n, int m,
                               int idx_pitch, int idx_heads, int acc_pitch, hipStream_t st) {
  hipLaunchKernelGGL(score_gather_kernel, dim3((m + 255) / 256, dm.Hkv, dm.B * dm.L), dim3(256), 0, st, score, idx,
                     acc_new, n, m, idx_pitch, idx_heads, acc_pitch, dm.Hkv);
  return hipGetLastError();
}

hipError_t launch_compact(int elem_bytes, const Dims& dm, Segments ks, Segments vs, const int32_t* idx,
                          int idx_pitch, int idx_heads, int m, View k_new, View v_new, hipStream_t st) {
  const int row_bytes = dm.D * elem_bytes;
  switch (row_bytes) {
    case 128: return compact_launch<128>(elem_bytes, dm, ks, vs, idx, idx_pitch, idx_heads, m, k_new, v_new, st);
    case 256: return compact_launch<256>(elem_bytes, dm, ks, vs, idx, idx_pitch, idx_heads, m, k_new, v_new, st);
    case 512: return compact_launch<512>(elem_bytes, dm, ks, vs, idx, idx_pitch, idx_heads, m, k_new, v_new, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace citrus
