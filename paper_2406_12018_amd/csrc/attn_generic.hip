// Generic (vector-ALU) attention kernels for f32 and bf16 element types.
//
// These are the kernels of the f32 mode (tiny parity configuration) and the
// fallback for bf16 shapes the MFMA kernels do not cover.  They follow the same
// definitions as the fast path: softmax attention with the 1/sqrt(d_k) scaling
// of Eq. (1) (Section 4.1 step 1), and the summed form of Eq. (1) for the
// importance scores.
#include "citrus_internal.h"

namespace citrus {
namespace {

constexpr int kWave = 64;
constexpr int kRowsPerBlock = 4;  // one wavefront per query row

// Logit: the type the q.k products are accumulated and the maximum / normaliser subtracted in.  The f32
// mode promises 1e-5 against an f64 reference: with logits of a few tens an f32 dot product and subtraction
// alone leave a relative error of that order in the probability, so f32 inputs use f64 there.
template <typename T> struct Elem;
template <> struct Elem<float> {
  typedef double Logit;
  static constexpr int kVec = 4;  // elements per 16-byte load
  __device__ static void load16(const float* p, float* dst) {
    float4 v = *reinterpret_cast<const float4*>(p);
    dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
  }
  __device__ static float load1(const float* p) { return *p; }
  __device__ static void store1(float* p, float v) { *p = v; }
};
template <> struct Elem<uint16_t> {  // bf16 as raw bits
  typedef float Logit;
  static constexpr int kVec = 8;
  __device__ static float cvt(uint16_t b) { return __uint_as_float(static_cast<uint32_t>(b) << 16); }
  __device__ static void load16(const uint16_t* p, float* dst) {
    uint4 v = *reinterpret_cast<const uint4*>(p);
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      dst[2 * i] = __uint_as_float(w[i] << 16);
      dst[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  __device__ static float load1(const uint16_t* p) { return cvt(*p); }
  __device__ static void store1(uint16_t* p, float v) {  // round to nearest even
    uint32_t u = __float_as_uint(v);
    u += 0x7fffu + ((u >> 16) & 1u);
    *p = static_cast<uint16_t>(u >> 16);
  }
};

template <typename T>
__device__ inline const T* row_ptr(const View& v, int b, int l, int h, int s) {
  return static_cast<const T*>(v.ptr) + (b * v.sb + l * v.sl + h * v.sh + static_cast<int64_t>(s) * v.ss);
}

// candidate j -> its row in the cache or the chunk segment
template <typename T>
__device__ inline const T* cand_ptr(const Segments& sg, int b, int l, int g, int j) {
  return j < sg.n_c ? row_ptr<T>(sg.cache, b, l, g, j) : row_ptr<T>(sg.chunk, b, l, g, j - sg.n_c);
}

__device__ inline float mad(float a, float b, float c) { return fmaf(a, b, c); }
__device__ inline double mad(double a, double b, double c) { return fma(a, b, c); }

__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// One wavefront per query row; lanes split the keys of a 64-key tile for the
// logits and split head_dim for the output accumulation.
template <typename T, int D>
__global__ __launch_bounds__(kWave* kRowsPerBlock) void attn_generic_kernel(Dims dm, View q, int rows, Segments ks,
                                                                           Segments vs, int causal, View out,
                                                                           float* lse) {
  __shared__ float q_s[kRowsPerBlock][D];
  __shared__ float p_s[kRowsPerBlock][kWave];
  const int lane = threadIdx.x % kWave, w = threadIdx.x / kWave;
  const int h = blockIdx.y, b = blockIdx.z / dm.L, l = blockIdx.z % dm.L, g = h / dm.G;
  const int n = ks.n_c + ks.c;
  const int t_raw = blockIdx.x * kRowsPerBlock + w;
  const bool row_ok = t_raw < rows;
  const int t = row_ok ? t_raw : rows - 1;
  const int limit = causal ? ks.n_c + t : n - 1;  // last visible candidate
  const int t_blk_last = min(rows - 1, blockIdx.x * kRowsPerBlock + kRowsPerBlock - 1);
  const int blk_limit = causal ? ks.n_c + t_blk_last : n - 1;
  constexpr int E = D / kWave;  // output dims per lane

  const T* qp = row_ptr<T>(q, b, l, h, t);
  for (int e = lane; e < D; e += kWave) q_s[w][e] = Elem<T>::load1(qp + e);
  __syncthreads();

  float m = -INFINITY, lsum = 0.f, acc[E];
#pragma unroll
  for (int e = 0; e < E; ++e) acc[e] = 0.f;

  for (int j0 = 0; j0 <= blk_limit; j0 += kWave) {
    const int j = j0 + lane;
    const bool valid = j <= limit;
    typedef typename Elem<T>::Logit Logit;
    Logit s = -INFINITY;
    if (valid) {
      const T* kp = cand_ptr<T>(ks, b, l, g, j);
      Logit dot = 0;
#pragma unroll 4
      for (int e = 0; e < D; e += Elem<T>::kVec) {
        float kv[Elem<T>::kVec];
        Elem<T>::load16(kp + e, kv);
#pragma unroll
        for (int x = 0; x < Elem<T>::kVec; ++x) dot = mad(static_cast<Logit>(q_s[w][e + x]), static_cast<Logit>(kv[x]), dot);
      }
      s = dot * static_cast<Logit>(dm.scale);
    }
    // the running maximum is an f32 value; it only has to be the same number wherever it is subtracted
    const float m_new = fmaxf(m, wave_max(static_cast<float>(s)));
    // tile 0 always holds candidate 0, which every row sees, so m_new is finite
    const float p = valid ? expf(static_cast<float>(s - static_cast<Logit>(m_new))) : 0.f;
    const float corr = expf(m - m_new);
    lsum = lsum * corr + wave_sum(p);
    m = m_new;
    p_s[w][lane] = p;
    __syncthreads();
    if (out.ptr != nullptr) {
#pragma unroll
      for (int e = 0; e < E; ++e) acc[e] *= corr;
      const int cnt = min(kWave, limit + 1 - j0);  // may be <= 0 for rows that see nothing here
      for (int jj = 0; jj < cnt; ++jj) {
        const T* vp = cand_ptr<T>(vs, b, l, g, j0 + jj);
        const float pj = p_s[w][jj];
#pragma unroll
        for (int e = 0; e < E; ++e) acc[e] = fmaf(pj, Elem<T>::load1(vp + lane + e * kWave), acc[e]);
      }
    }
    __syncthreads();
  }

  if (!row_ok) return;
  if (out.ptr != nullptr) {
    T* op = const_cast<T*>(row_ptr<T>(out, b, l, h, t));
    const float inv = 1.f / lsum;
#pragma unroll
    for (int e = 0; e < E; ++e) Elem<T>::store1(op + lane + e * kWave, acc[e] * inv);
  }
  if (lse != nullptr && lane == 0)
    lse[(static_cast<int64_t>(blockIdx.z) * dm.Hq + h) * rows + t] = m + logf(lsum);
}

constexpr int kColsumThreads = 256;
constexpr int kColsumQTile = 16;

// One thread per candidate key; the query rows of the KV group stream through
// LDS.  The sum runs in a fixed order (heads, then rows), so it is reproducible.
template <typename T, int D>
__global__ __launch_bounds__(kColsumThreads) void colsum_generic_kernel(Dims dm, View q, int rows, Segments ks,
                                                                       int causal, const float* lse, float* score) {
  __shared__ float q_s[kColsumQTile][D];
  __shared__ float lse_s[kColsumQTile];
  const int g = blockIdx.y, b = blockIdx.z / dm.L, l = blockIdx.z % dm.L;
  const int n = ks.n_c + ks.c;
  const int j = blockIdx.x * kColsumThreads + threadIdx.x;
  const bool key_ok = j < n;

  float kreg[D];
  {
    const T* kp = cand_ptr<T>(ks, b, l, g, key_ok ? j : n - 1);
#pragma unroll
    for (int e = 0; e < D; e += Elem<T>::kVec) Elem<T>::load16(kp + e, kreg + e);
  }
  // first chunk row that sees candidate j (cache candidates are seen by every row)
  const int t_first = (causal && j >= ks.n_c) ? j - ks.n_c : 0;

  float sum = 0.f;
  for (int hh = 0; hh < dm.G; ++hh) {
    const int h = g * dm.G + hh;
    const float* lse_h = lse + (static_cast<int64_t>(blockIdx.z) * dm.Hq + h) * rows;
    for (int t0 = 0; t0 < rows; t0 += kColsumQTile) {
      const int tn = min(kColsumQTile, rows - t0);
      __syncthreads();
      for (int x = threadIdx.x; x < tn * D; x += kColsumThreads)
        q_s[x / D][x % D] = Elem<T>::load1(row_ptr<T>(q, b, l, h, t0 + x / D) + x % D);
      if (threadIdx.x < tn) lse_s[threadIdx.x] = lse_h[t0 + threadIdx.x];
      __syncthreads();
      for (int tt = 0; tt < tn; ++tt) {
        typedef typename Elem<T>::Logit Logit;
        Logit dot = 0;
#pragma unroll
        for (int e = 0; e < D; ++e) dot = mad(static_cast<Logit>(q_s[tt][e]), static_cast<Logit>(kreg[e]), dot);
        const float p = expf(static_cast<float>(dot * static_cast<Logit>(dm.scale) - static_cast<Logit>(lse_s[tt])));
        if (t0 + tt >= t_first) sum += p;
      }
    }
  }
  if (key_ok) score[(static_cast<int64_t>(blockIdx.z) * dm.Hkv + g) * n + j] = sum;
}

template <typename T, int D>
hipError_t attn_launch_t(const Dims& dm, View q, int rows, Segments ks, Segments vs, int causal, View out,
                         float* lse, hipStream_t st) {
  dim3 grid((rows + kRowsPerBlock - 1) / kRowsPerBlock, dm.Hq, dm.B * dm.L);
  hipLaunchKernelGGL((attn_generic_kernel<T, D>), grid, dim3(kWave * kRowsPerBlock), 0, st, dm, q, rows, ks, vs,
                     causal, out, lse);
  return hipGetLastError();
}

template <typename T, int D>
hipError_t colsum_launch_t(const Dims& dm, View q, int rows, Segments ks, int causal, const float* lse,
                           float* score, hipStream_t st) {
  const int n = ks.n_c + ks.c;
  dim3 grid((n + kColsumThreads - 1) / kColsumThreads, dm.Hkv, dm.B * dm.L);
  hipLaunchKernelGGL((colsum_generic_kernel<T, D>), grid, dim3(kColsumThreads), 0, st, dm, q, rows, ks, causal, lse,
                     score);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_generic(int dtype, const Dims& dm, View q, int rows, Segments ks, Segments vs, int causal,
                               View out, float* lse, hipStream_t st) {
  if (dtype == CITRUS_F32) {
    return dm.D == 64 ? attn_launch_t<float, 64>(dm, q, rows, ks, vs, causal, out, lse, st)
                      : attn_launch_t<float, 128>(dm, q, rows, ks, vs, causal, out, lse, st);
  }
  return dm.D == 64 ? attn_launch_t<uint16_t, 64>(dm, q, rows, ks, vs, causal, out, lse, st)
                    : attn_launch_t<uint16_t, 128>(dm, q, rows, ks, vs, causal, out, lse, st);
}

hipError_t launch_colsum_generic(int dtype, const Dims& dm, View q, int rows, Segments ks, int causal,
                                 const float* lse, float* score, hipStream_t st) {
  if (dtype == CITRUS_F32) {
    return dm.D == 64 ? colsum_launch_t<float, 64>(dm, q, rows, ks, causal, lse, score, st)
                      : colsum_launch_t<float, 128>(dm, q, rows, ks, causal, lse, score, st);
  }
  return dm.D == 64 ? colsum_launch_t<uint16_t, 64>(dm, q, rows, ks, causal, lse, score, st)
                    : colsum_launch_t<uint16_t, 128>(dm, q, rows, ks, causal, lse, score, st);
}

}  // namespace citrus
