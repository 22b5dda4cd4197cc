// Rotary position embedding at explicit positions: the position shift of Section 5.3
// ("Hyperparameters"), where a cached state's position is its slot in the cache.  The cache keeps
// unrotated keys; before every step the candidates, the chunk's queries and the instruction's
// queries are rotated to their positions of that step.
//
// Convention of the Llama / Mistral models: pairs (i, i + d/2), angle = position * base^(-2 i / d).
// HBM-bound elementwise work: a thread owns eight pairs of one sequence row, computes their sines
// and cosines once and applies them to that row of EVERY head of the (document, layer): the
// angle does not depend on the head, and the transcendental work per byte drops by the head count.
// (The chunk-attention kernel can rotate its query rows itself, in registers: rope_math.h.)
#include "citrus_internal.h"
#include "rope_math.h"

namespace citrus {
namespace {

// Heads that share one thread's sines and cosines.  More would save transcendental work, fewer give
// more workgroups: the instruction's queries are 64 rows only.
constexpr int kHeadsPerThread = 4;

// bf16: 16-byte accesses = 8 elements; thread (row, part) owns elements 8 part .. +7 of the low half
// and the same of the high half.  f32 math.  (block_x, block_z): the workgroup's place in the grid of its own
// rotation, also when several rotations share one launch.
__device__ inline void rope_bf16_block(const View& x, const View& y, int heads, int rows, int d, int pos0,
                                       float log2_base, int L, int block_x, int block_z) {
  const int parts = d / 16;  // 8-element groups per half row
  const int e = block_x * 256 + threadIdx.x;
  const int row = e / parts, part = e % parts;
  if (row >= rows) return;
  const int b = blockIdx.y / L, l = blockIdx.y % L;
  float cs[8], sn[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) rope_sincos_bf16(pos0 + row, 8 * part + i, d, log2_base, sn[i], cs[i]);
  const int half = d / 2;
  const int h_begin = block_z * kHeadsPerThread, h_count = min(kHeadsPerThread, heads - h_begin);
  for (int hh = 0; hh < h_count; ++hh) {
    // workgroups start at different heads: head strides are often large powers of two, and all
    // workgroups walking the heads in step would keep hitting the same memory channels
    const int h = h_begin + (hh + block_x) % h_count;
    const uint16_t* xp = static_cast<const uint16_t*>(x.ptr) + (b * x.sb + l * x.sl + h * x.sh + row * x.ss) + 8 * part;
    uint16_t* yp = static_cast<uint16_t*>(const_cast<void*>(y.ptr)) + (b * y.sb + l * y.sl + h * y.sh + row * y.ss) + 8 * part;
    const uint4 lo = *reinterpret_cast<const uint4*>(xp);
    const uint4 hi = *reinterpret_cast<const uint4*>(xp + half);
    const uint32_t lw[4] = {lo.x, lo.y, lo.z, lo.w}, hw[4] = {hi.x, hi.y, hi.z, hi.w};
    uint32_t lo_out[4], hi_out[4];
#pragma unroll
    for (int p = 0; p < 4; ++p)
      rope_rotate_words(lw[p], hw[p], cs[2 * p], sn[2 * p], cs[2 * p + 1], sn[2 * p + 1], lo_out[p], hi_out[p]);
    *reinterpret_cast<uint4*>(yp) = make_uint4(lo_out[0], lo_out[1], lo_out[2], lo_out[3]);
    *reinterpret_cast<uint4*>(yp + half) = make_uint4(hi_out[0], hi_out[1], hi_out[2], hi_out[3]);
  }
}

__global__ __launch_bounds__(256) void rope_bf16_kernel(View x, View y, int heads, int rows, int d, int pos0,
                                                        float log2_base, int L) {
  rope_bf16_block(x, y, heads, rows, d, pos0, log2_base, L, blockIdx.x, blockIdx.z);
}

// Several rotations of one step (candidates' keys, chunk keys, queries) in ONE launch: the workgroups of
// rotation j follow those of rotation j - 1 along x; a rotation's head groups are folded into x as well.
struct RopeBatch {
  View x[kMaxRopeJobs], y[kMaxRopeJobs];
  int heads[kMaxRopeJobs], rows[kMaxRopeJobs], pos0[kMaxRopeJobs];
  int first_block[kMaxRopeJobs + 1];  // along x; job j owns [first_block[j], first_block[j + 1])
  int blocks_x[kMaxRopeJobs];         // of a job's own grid: row blocks (its head groups make up the rest)
  int count;
};
__global__ __launch_bounds__(256) void rope_bf16_batch_kernel(RopeBatch jobs, int d, float log2_base, int L) {
  int j = 0;
  while (j + 1 < jobs.count && static_cast<int>(blockIdx.x) >= jobs.first_block[j + 1]) ++j;  // block-uniform
  const int local = blockIdx.x - jobs.first_block[j];
  rope_bf16_block(jobs.x[j], jobs.y[j], jobs.heads[j], jobs.rows[j], d, jobs.pos0[j], log2_base, L, local % jobs.blocks_x[j],
                  local / jobs.blocks_x[j]);
}

// f32: 16-byte accesses = 4 elements; angles, sines and cosines in double so that the f32 results are
// correctly rounded to within the f32 tolerance at positions in the thousands.
__global__ __launch_bounds__(256) void rope_f32_kernel(View x, View y, int heads, int rows, int d, int pos0,
                                                       double log2_base, int L) {
  const int parts = d / 8;  // 4-element groups per half row
  const int e = blockIdx.x * 256 + threadIdx.x;
  const int row = e / parts, part = e % parts;
  if (row >= rows) return;
  const int b = blockIdx.y / L, l = blockIdx.y % L;
  double cs[4], sn[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const double inv_freq = exp2(-static_cast<double>(2 * (4 * part + i)) / static_cast<double>(d) * log2_base);
    sincos(static_cast<double>(pos0 + row) * inv_freq, &sn[i], &cs[i]);
  }
  const int half = d / 2;
  const int h_begin = blockIdx.z * kHeadsPerThread, h_count = min(kHeadsPerThread, heads - h_begin);
  for (int hh = 0; hh < h_count; ++hh) {
    // workgroups start at different heads: head strides are often large powers of two, and all
    // workgroups walking the heads in step would keep hitting the same memory channels
    const int h = h_begin + (hh + blockIdx.x) % h_count;
    const float* xp = static_cast<const float*>(x.ptr) + (b * x.sb + l * x.sl + h * x.sh + row * x.ss) + 4 * part;
    float* yp = static_cast<float*>(const_cast<void*>(y.ptr)) + (b * y.sb + l * y.sl + h * y.sh + row * y.ss) + 4 * part;
    const float4 lo = *reinterpret_cast<const float4*>(xp);
    const float4 hi = *reinterpret_cast<const float4*>(xp + half);
    const float lv[4] = {lo.x, lo.y, lo.z, lo.w}, hv[4] = {hi.x, hi.y, hi.z, hi.w};
    float lo_out[4], hi_out[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      lo_out[i] = static_cast<float>(lv[i] * cs[i] - hv[i] * sn[i]);
      hi_out[i] = static_cast<float>(hv[i] * cs[i] + lv[i] * sn[i]);
    }
    *reinterpret_cast<float4*>(yp) = make_float4(lo_out[0], lo_out[1], lo_out[2], lo_out[3]);
    *reinterpret_cast<float4*>(yp + half) = make_float4(hi_out[0], hi_out[1], hi_out[2], hi_out[3]);
  }
}

}  // namespace

hipError_t launch_rope(int dtype, const Dims& dm, View x, View y, int heads, int rows, int pos0, float base,
                       hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  if (dtype == CITRUS_BF16) {
    const int threads = rows * (dm.D / 16);
    hipLaunchKernelGGL(rope_bf16_kernel, dim3((threads + 255) / 256, dm.B * dm.L, (heads + kHeadsPerThread - 1) / kHeadsPerThread),
                       dim3(256), 0, st, x, y, heads, rows, dm.D, pos0, log2f(base), dm.L);
  } else {
    const int threads = rows * (dm.D / 8);
    hipLaunchKernelGGL(rope_f32_kernel, dim3((threads + 255) / 256, dm.B * dm.L, (heads + kHeadsPerThread - 1) / kHeadsPerThread),
                       dim3(256), 0, st, x, y, heads, rows, dm.D, pos0, log2(static_cast<double>(base)), dm.L);
  }
  return hipGetLastError();
}

hipError_t launch_rope_batch(int dtype, const Dims& dm, const RopeJob* jobs, int count, float base, hipStream_t st) {
  if (count < 1 || count > kMaxRopeJobs) return hipErrorInvalidValue;
  if (dtype != CITRUS_BF16 || count == 1) {  // f32 (the tiny configuration): one launch per rotation
    for (int j = 0; j < count; ++j) {
      const hipError_t e = launch_rope(dtype, dm, jobs[j].x, jobs[j].y, jobs[j].heads, jobs[j].rows, jobs[j].pos0, base, st);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }
  RopeBatch b;
  b.count = 0;
  int blocks = 0;
  for (int j = 0; j < count; ++j) {
    if (jobs[j].rows <= 0) continue;
    const int k = b.count++;
    b.x[k] = jobs[j].x; b.y[k] = jobs[j].y;
    b.heads[k] = jobs[j].heads; b.rows[k] = jobs[j].rows; b.pos0[k] = jobs[j].pos0;
    b.blocks_x[k] = (jobs[j].rows * (dm.D / 16) + 255) / 256;
    b.first_block[k] = blocks;
    blocks += b.blocks_x[k] * ((jobs[j].heads + kHeadsPerThread - 1) / kHeadsPerThread);
  }
  if (b.count == 0) return hipSuccess;
  b.first_block[b.count] = blocks;
  for (int k = b.count; k < kMaxRopeJobs; ++k) {  // unused slots: defined values
    b.x[k] = b.x[0]; b.y[k] = b.y[0];
    b.heads[k] = b.rows[k] = b.pos0[k] = 0; b.blocks_x[k] = 1;
    b.first_block[k + 1] = blocks;
  }
  hipLaunchKernelGGL(rope_bf16_batch_kernel, dim3(blocks, dm.B * dm.L, 1), dim3(256), 0, st, b, dm.D, log2f(base), dm.L);
  return hipGetLastError();
}

}  // namespace citrus
