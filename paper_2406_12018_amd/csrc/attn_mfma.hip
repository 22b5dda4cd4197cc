// bf16 MFMA kernels for head_dim 128 on gfx950 (CDNA4).
//
//  attn_pipe_kernel_w8 flash-style chunk attention (Section 4.1 step 1; softmax
//                      with the 1/sqrt(d_k) scaling of Eq. (1)): online softmax
//                      over 64-key tiles staged in LDS, S^T = K.Q^T and
//                      O^T = V^T.P^T on v_mfma_f32_32x32x16_bf16.
//  lse_mfma_kernel     the rows' log-sum-exp alone (first pass of the two-pass
//                      importance scores).
//  colsum_mfma_kernel  summed form of Eq. (1): probabilities exp(s - lse)
//                      added down the query rows of a KV group, per key.
//
// Layout facts used throughout (wave64, v_mfma_f32_32x32x16_bf16):
//   A operand: lane l holds row (l % 32), contraction slots 8*(l / 32) .. +7
//   B operand: lane l holds column (l % 32), the same contraction slots
//   C/D:       lane l, register i holds column (l % 32),
//              row 8*(i / 4) + 4*(l / 32) + (i % 4)
// Computing S^T (keys x queries) puts one query per lane, so softmax row
// reductions are in-lane plus one exchange with lane l ^ 32, and the S^T
// accumulators are directly the B operand (P^T) of the second product.
#include <type_traits>

#include "citrus_internal.h"
#include "rope_math.h"


namespace citrus {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) short i16x4;

constexpr int D = 128;
constexpr int kWaves = 4;               // one wave per SIMD and block; two or more blocks share a CU
constexpr int kThreads = kWaves * 64;
constexpr int kRowsPerWave = 32;        // one 32-query column tile per wave
constexpr int kTileN = 64;              // keys per LDS tile
constexpr int kXcds = 8;
constexpr int kBufferFlags = 0x00020000;  // raw buffer resource word 3 on CDNA: 32-bit data format, no swizzle
constexpr int kPitchK = D + 8;          // padded LDS row pitch in bf16 (272 B) of the column-sum kernel's Q chunk
constexpr int kRowBytes = 2 * D;        // K/V tile rows in LDS are unpadded (256 B) and XOR-swizzled
constexpr int kTileBytes = kTileN * kRowBytes;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kMaxSlack = 8.0f;  // probabilities stay below 2^8: exact in f32, same relative rounding in bf16

union Pack8 {
  bf16x8 v;
  uint4 u;
  uint32_t w[4];
  i16x4 h[2];
};

__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
  f32x2 f = {lo, hi};
  bf16x2 b = __builtin_convertvector(f, bf16x2);  // round to nearest even
  return __builtin_bit_cast(uint32_t, b);
}

__device__ inline const uint16_t* unit_ptr(const View& v, int b, int l, int h) {
  return static_cast<const uint16_t*>(v.ptr) + (b * v.sb + l * v.sl + h * v.sh);
}

// LDS transpose read (ds_read_b64_tr_b16).  Within each group of 16 lanes, lane s passes the
// address of 4 consecutive bf16 and lane i receives element (i % 4) of lanes i/4, 4 + i/4,
// 8 + i/4, 12 + i/4.  With lane s pointing at &V[key(s / 4)][d0 + 4 (s % 4)], lane i gets
// V[key(0..3)][d0 + i]: four keys of one head_dim column, i.e. half of an MFMA A operand of V^T.
__device__ inline i16x4 lds_read_tr16(const char* p) {
  typedef i16x4 __attribute__((address_space(3))) * lds_ptr;
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
}

// Instructions whose issue ORDER matters (a software pipeline that overlaps the matrix pipe with
// the exponentials inside one wave) are written as volatile asm statements: the compiler keeps
// volatile statements in source order and allocates their registers, but does not see inside
// them, so the software-managed hazards are handled here: v_exp_f32 is followed by the one wait
// state a non-transcendental consumer needs, and no vector instruction may read an MFMA result
// sooner than the MFMA takes to complete (callers keep a whole MFMA group in between).
typedef __attribute__((ext_vector_type(4))) int i32x4;
__device__ inline void mfma_pinned(f32x16& acc, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0"
               : "+v"(acc)
               : "v"(__builtin_bit_cast(i32x4, a)), "v"(__builtin_bit_cast(i32x4, b)));
}
__device__ inline f32x16 mfma_pinned_first(const bf16x8& a, const bf16x8& b) {  // accumulator starts at zero
  f32x16 d;
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0"
               : "=&v"(d)
               : "v"(__builtin_bit_cast(i32x4, a)), "v"(__builtin_bit_cast(i32x4, b)));
  return d;
}
__device__ inline float exp2_pinned(float x) {
  float y;
  asm volatile("v_exp_f32 %0, %1\n\ts_nop 0" : "=v"(y) : "v"(x));
  return y;
}

__device__ inline float max3_pinned(float a, float b, float c) {
  float y;
  asm volatile("v_max3_f32 %0, %1, %2, %3" : "=v"(y) : "v"(a), "v"(b), "v"(c));
  return y;
}
// v_exp_f32 followed by an MFMA that does not read its result: the MFMA is the wait state.
__device__ inline float exp2_then_mfma(float x, f32x16& acc, const bf16x8& a, const bf16x8& b) {
  float y;
  asm volatile("v_exp_f32 %0, %2\n\tv_mfma_f32_32x32x16_bf16 %1, %3, %4, %1"
               : "=&v"(y), "+v"(acc)
               : "v"(x), "v"(__builtin_bit_cast(i32x4, a)), "v"(__builtin_bit_cast(i32x4, b)));
  return y;
}

// Small fences for the optimiser, as functions so that kernel templates hold no asm of their own.
__device__ inline void hide_loop_invariance(int& a, int& b) { asm volatile("" : "+v"(a), "+v"(b)); }
__device__ inline void keep_values_here(uint32_t (&p)[8], float& l) {
  asm volatile("" : "+v"(p[0]), "+v"(p[1]), "+v"(p[2]), "+v"(p[3]), "+v"(p[4]), "+v"(p[5]), "+v"(p[6]), "+v"(p[7]), "+v"(l));
}
__device__ inline void no_memory_motion() { asm volatile("" ::: "memory"); }
// enough wait states for every MFMA issued through the pinned helpers above to have written its result
__device__ inline void wait_for_pinned_mfmas() { asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory"); }

// Barrier that publishes tiles streamed into LDS by buffer_load ... lds.  Those writes are tracked
// by the issuing wave's vector-memory counter only, and the fence inside __syncthreads() covers
// ordinary LDS traffic: every wave has to drain its own loads before it arrives.
__device__ inline void barrier_after_lds_fill() {
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0), nothing else
  __syncthreads();
}

// How the waves of a block split (head, 32-row tile) tasks inside one KV group.
struct TaskShape {
  int heads_per_block;  // 4, 2 or 1 query heads of the group
  int tiles_per_block;  // kWaves / heads_per_block row tiles of 32
};
__host__ __device__ inline TaskShape task_shape(int G, int waves = kWaves) {
  const int hpb = (G % 4 == 0) ? 4 : ((G % 2 == 0) ? 2 : 1);
  return TaskShape{hpb, waves / hpb};
}

// Row normalisers only (no values, no output): the log-sum-exp of every query row over the keys it sees,
// or, with key_splits > 1, one partial (running maximum, sum) pair per key range and row.  First pass of the
// two-pass importance scores and of a cache-only normaliser that the attention launch could not emit.
__global__ __launch_bounds__(kThreads, 2) void lse_mfma_kernel(Dims dm, View q, int rows, Segments ks, int causal,
                                                              float* lse, int key_splits, float2* part) {
  __shared__ __attribute__((aligned(1024))) char k_s[2 * kTileBytes];  // double-buffered tiles

  const int tid = threadIdx.x, lane = tid % 64, w = tid / 64;
  const int col = lane % 32, grp = lane / 32;
  const TaskShape ts = task_shape(dm.G);
  const int head_groups = dm.G / ts.heads_per_block;
  const int rows_per_block = ts.tiles_per_block * kRowsPerWave;
  const int row_blocks = (rows + rows_per_block - 1) / rows_per_block;
  // Workgroups are handed to the 8 XCDs round-robin by their linear id.  Remap so that the
  // workgroups of one (document, layer, KV head), which read the same K/V, land on ONE XCD and
  // share its L2; within a unit the row blocks with the longest causal range come first.
  int logical = blockIdx.x;
  const int total = gridDim.x;
  if (total % kXcds == 0) logical = (blockIdx.x % kXcds) * (total / kXcds) + blockIdx.x / kXcds;
  // With key_splits > 1 each workgroup covers one contiguous range of key
  // tiles and writes a partial (running maximum, sum) pair per row; the consumer merges them.
  const int sp = logical % key_splits;
  logical /= key_splits;
  // Causal attention: a workgroup takes the row block with the longest key range still free and then
  // its mirror image (the shortest), so every workgroup does the same number of key tiles.
  const bool paired = causal != 0 && key_splits == 1;
  const int rb_slots = paired ? (row_blocks + 1) / 2 : row_blocks;
  const int rb_first = row_blocks - 1 - logical % rb_slots;
  const int rb_second = row_blocks - 1 - rb_first;
  const int passes = (paired && rb_second != rb_first) ? 2 : 1;
  const int hg = (logical / rb_slots) % head_groups;
  const int g = (logical / (rb_slots * head_groups)) % dm.Hkv;
  const int bl = logical / (rb_slots * head_groups * dm.Hkv);
  const int b = bl / dm.L, l = bl % dm.L;
  const int h = g * dm.G + hg * ts.heads_per_block + (w % ts.heads_per_block);
  const int n_c = ks.n_c;
  const int n = n_c + ks.c;

  // ---- global -> LDS staging of one 64-key tile, without a stop in registers ----
  // buffer_load ... lds: a wave-level instruction moves 64 x 16 B from per-lane global addresses
  // to 1 KB of consecutive LDS, i.e. four unpadded 256-byte rows.  Bank conflicts of the column
  // reads below are avoided by an XOR swizzle instead of padding: the 16-byte segment `seg` of
  // tile row `row` lives at segment position seg ^ f(row), f(row) = 2 (row % 8) ^ ((row / 8) % 2),
  // which the loading lane realises by fetching global segment (its LDS position) ^ f(row).
  // Wave w fills rows 16 w + 4 i .. + 3 with instruction i = 0..3.  Rows that fall outside the
  // candidates re-read the last row (finite values; their logits are masked).
  const int k_ss_cache = static_cast<int>(ks.cache.ss), k_ss_chunk = static_cast<int>(ks.chunk.ss);
  auto seg_bytes = [](int rows_, int ss_) { return rows_ > 0 ? ((rows_ - 1) * ss_ + D) * 2 : 0; };
  const __amdgpu_buffer_rsrc_t k_rs_cache = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(unit_ptr(ks.cache, b, l, g)), 0, seg_bytes(n_c, k_ss_cache), kBufferFlags);
  const __amdgpu_buffer_rsrc_t k_rs_chunk = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(unit_ptr(ks.chunk, b, l, g)), 0, seg_bytes(ks.c, k_ss_chunk), kBufferFlags);
  const int wu = __builtin_amdgcn_readfirstlane(w);
  const int fill_row = 16 * wu + lane / 16;                       // tile row this lane fills with instruction 0
  const int fill_seg16 = ((lane % 16) ^ (2 * (lane / 16))) * 16;  // byte offset of its global segment, before ^ c_i
  typedef __attribute__((address_space(3))) void* lds_void_ptr;
  auto fill4 = [&](char* lds_tile, __amdgpu_buffer_rsrc_t rs_cache, __amdgpu_buffer_rsrc_t rs_chunk, int ss_cache,
                   int ss_chunk, int j0) {
    const bool simple = (j0 + kTileN <= n_c) || (j0 >= n_c && j0 + kTileN <= n);  // block-uniform
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int ci16 = ((8 * (i & 1)) | (i >> 1)) * 16;
      lds_void_ptr dst = (lds_void_ptr)(lds_tile + (16 * wu + 4 * i) * kRowBytes);
      if (simple) {
        const bool in_cache = j0 < n_c;
        const int ss = in_cache ? ss_cache : ss_chunk;
        const int r0 = in_cache ? j0 : j0 - n_c;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(in_cache ? rs_cache : rs_chunk, dst, 16,
                                                 fill_row * ss * 2 + (fill_seg16 ^ ci16), (r0 + 4 * i) * ss * 2, 0, 0);
      } else {  // the tile straddles the cache / chunk boundary or the end of the candidates
        const int j = min(j0 + fill_row + 4 * i, n - 1);
        if (j < n_c)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_cache, dst, 16, j * ss_cache * 2 + (fill_seg16 ^ ci16), 0, 0, 0);
        else
          __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_chunk, dst, 16, (j - n_c) * ss_chunk * 2 + (fill_seg16 ^ ci16),
                                                   0, 0, 0);
      }
    }
  };
  auto fetch_tile = [&](int j0_, int buf_) {
    fill4(k_s + buf_ * kTileBytes, k_rs_cache, k_rs_chunk, k_ss_cache, k_ss_chunk, j0_);
  };

  // per-lane LDS read offsets (bytes inside a tile buffer), swizzle included
  // A operand of S^T: key row `col`, head_dim segment 2 kk + grp
  const int f_col = (2 * (col & 7)) ^ ((col >> 3) & 1);
  int k_off[8];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) k_off[kk] = col * kRowBytes + (((2 * kk + grp) ^ f_col) * 16);
  for (int pass = 0; pass < passes; ++pass) {
  const int rb = pass == 0 ? rb_first : rb_second;
  const int row0 = (rb * ts.tiles_per_block + w / ts.heads_per_block) * kRowsPerWave;

  // last candidate any row of this block / this wave can see
  const int blk_row_last = min(rows, (rb + 1) * rows_per_block) - 1;
  const int blk_limit = causal ? n_c + blk_row_last : n - 1;
  const int all_tiles = blk_limit / kTileN + 1;
  const int tiles_per_split = (all_tiles + key_splits - 1) / key_splits;
  const int t_begin = sp * tiles_per_split;
  const int t_end = min(all_tiles, t_begin + tiles_per_split);
  const bool wave_active = row0 < rows;
  const int wave_row_last = min(rows, row0 + kRowsPerWave) - 1;
  const int wave_limit_max = causal ? n_c + wave_row_last : n - 1;  // beyond it the wave sees nothing
  const int wave_limit_min = causal ? n_c + row0 : n - 1;           // up to it every row sees everything

  // ---- Q^T operand, kept in registers: q_op[kk] = Q[row0 + col][16 kk + 8 grp ..+7] ----
  bf16x8 q_op[8];
  const int t_lane = max(min(row0 + col, rows - 1), 0);
  {
    const uint16_t* qp = unit_ptr(q, b, l, h) + static_cast<int64_t>(t_lane) * q.ss + 8 * grp;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      Pack8 p;
      p.u = *reinterpret_cast<const uint4*>(qp + 16 * kk);
      q_op[kk] = p.v;
    }
  }
  const int limit_lane = causal ? n_c + t_lane : n - 1;

  // ---- running softmax state: one query per lane ----
  const float c2 = dm.scale * kLog2e;  // logits are kept in the log2 domain
  float m_run = -INFINITY, l_run = 0.f;

  if (t_begin < t_end) {  // block-uniform
  fetch_tile(t_begin * kTileN, 0);
  barrier_after_lds_fill();  // also: the Q operand loads have landed

  for (int jt = t_begin; jt < t_end; ++jt) {
    const int j0 = jt * kTileN;
    const int buf = (jt - t_begin) & 1;
    const char* k_t = k_s + buf * kTileBytes;
    // The other buffer was last read one iteration ago and every wave has passed the barrier that
    // ended that iteration: the next tile can stream into it while this one is computed.
    if (jt + 1 < t_end) fetch_tile(j0 + kTileN, buf ^ 1);

    if (wave_active && j0 <= wave_limit_max) {
      // S^T = K . Q^T for 64 keys x 32 queries
      f32x16 s_acc[2];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) s_acc[mt][i] = 0.f;
#pragma unroll
      for (int kh = 0; kh < 2; ++kh) {  // the two 32-key halves are independent MFMA chains: interleave them
        Pack8 a[2][4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
          for (int mt = 0; mt < 2; ++mt)
            a[mt][kk].u = *reinterpret_cast<const uint4*>(k_t + 32 * mt * kRowBytes + k_off[4 * kh + kk]);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
          for (int mt = 0; mt < 2; ++mt)
            s_acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mt][kk].v, q_op[4 * kh + kk], s_acc[mt], 0, 0, 0);
      }

      if (j0 + kTileN - 1 > wave_limit_min) {  // wave-uniform: only tiles that touch the causal edge / the tail
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int j = j0 + 32 * mt + 8 * (i / 4) + 4 * grp + (i % 4);
            if (j > limit_lane) s_acc[mt][i] = -INFINITY;
          }
      }
      // Running maximum, kept lazily: softmax is invariant to the subtracted value, so m_run only has
      // to stay within kMaxSlack (log2 units) of the true row maximum to keep exp2 in range.  The fast
      // path looks at this lane's own 32 logits only; the exchange with lane l ^ 32, the update of
      // m_run and the rescale of the running sum happen only when some row needs them.
      float mx = s_acc[0][0];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s_acc[mt][i]);
      if (__any(mx * c2 > m_run + kMaxSlack)) {  // wave-uniform and rare after the first tiles
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run, mx * c2);
        // 0 on a row's first visible tile (m_run = -inf); 1 for a row that has seen nothing yet
        const float alpha = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(m_run - m_new);
        l_run *= alpha;
        m_run = m_new;
      }
      float psum = 0.f;
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) psum += __builtin_amdgcn_exp2f(fmaf(s_acc[mt][i], c2, -m_run));
      l_run += psum;
    }

    barrier_after_lds_fill();  // publishes the tile that streamed in; everyone is done with this one
  }
  }

  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const int t = row0 + col;
  if (wave_active && t < rows) {
  const int64_t row_id = (static_cast<int64_t>(bl) * dm.Hq + h) * rows + t;
  if (part != nullptr && grp == 0)  // log2 domain; an empty or fully masked range leaves (-inf, 0)
    part[static_cast<int64_t>(sp) * dm.B * dm.L * dm.Hq * rows + row_id] = make_float2(m_run, l_tot);
  if (lse != nullptr && grp == 0) lse[row_id] = (m_run + log2f(l_tot)) * kLn2;
  }  // row valid
  }  // pass
}

// The same attention, with output, as a software pipeline over half tiles of 32 keys: in step h the
// MFMAs of S^T(h + 1) = K.Q^T and of O^T += V^T.P^T(h - 1) are issued between the exponentials of
// half tile h, so that inside ONE wave the matrix pipe, the vector pipe and the LDS reads run at
// the same time instead of taking turns (the order is fixed with volatile asm statements, see above).
// K tiles are fetched one 64-key tile further ahead than V tiles; one barrier per 64 keys.
template <int WAVES, bool ROTATE_Q>
__device__ __forceinline__ void attn_pipe_body(const Dims& dm, const View& q, int rows, const Segments& ks,
                                               const Segments& vs, int causal, const View& out, float* lse,
                                               float* lse_cache, int q_rope_pos0, float rope_log2_base) {
  constexpr bool HAS_PV = true;
  constexpr int key_splits = 1;
  float2* const part = nullptr;
  __shared__ __attribute__((aligned(1024))) char k_s[2 * kTileBytes];  // double-buffered tiles
  __shared__ __attribute__((aligned(1024))) char v_s[HAS_PV ? 2 * kTileBytes : 16];
  extern __shared__ __attribute__((aligned(1024))) char q_stage[];  // [WAVES][32 rows][256 B], dynamic

  const int tid = threadIdx.x, lane = tid % 64, w = tid / 64;
  const int col = lane % 32, grp = lane / 32;
  constexpr int kFillRows = kTileN / WAVES;  // rows of a tile each wave fetches: 4 per instruction
  constexpr int kFillInstr = kFillRows / 4;
  const TaskShape ts = task_shape(dm.G, WAVES);
  const int head_groups = dm.G / ts.heads_per_block;
  const int rows_per_block = ts.tiles_per_block * kRowsPerWave;
  const int row_blocks = (rows + rows_per_block - 1) / rows_per_block;
  // Workgroups are handed to the 8 XCDs round-robin by their linear id.  Remap so that the
  // workgroups of one (document, layer, KV head), which read the same K/V, land on ONE XCD and
  // share its L2; within a unit the row blocks with the longest causal range come first.
  int logical = blockIdx.x;
  const int total = gridDim.x;
  if (total % kXcds == 0) logical = (blockIdx.x % kXcds) * (total / kXcds) + blockIdx.x / kXcds;
  // With key_splits > 1 (log-sum-exp only) each workgroup covers one contiguous range of key
  // tiles and writes a partial (running maximum, sum) pair per row; the consumer merges them.
  const int sp = logical % key_splits;
  logical /= key_splits;
  // Causal attention: a workgroup takes the row block with the longest key range still free and then
  // its mirror image (the shortest), so every workgroup does the same number of key tiles.
  const bool paired = causal != 0 && key_splits == 1;
  const int rb_slots = paired ? (row_blocks + 1) / 2 : row_blocks;
  const int rb_first = row_blocks - 1 - logical % rb_slots;
  const int rb_second = row_blocks - 1 - rb_first;
  const int passes = (paired && rb_second != rb_first) ? 2 : 1;
  const int hg = (logical / rb_slots) % head_groups;
  const int g = (logical / (rb_slots * head_groups)) % dm.Hkv;
  const int bl = logical / (rb_slots * head_groups * dm.Hkv);
  const int b = bl / dm.L, l = bl % dm.L;
  const int wu = __builtin_amdgcn_readfirstlane(w);  // the wave's index as a scalar: what depends on it stays scalar
  const int h = g * dm.G + hg * ts.heads_per_block + (wu % ts.heads_per_block);
  const int n_c = ks.n_c;
  const int n = n_c + ks.c;

  // ---- global -> LDS staging of one 64-key tile, without a stop in registers ----
  // buffer_load ... lds: a wave-level instruction moves 64 x 16 B from per-lane global addresses
  // to 1 KB of consecutive LDS, i.e. four unpadded 256-byte rows.  Bank conflicts of the column
  // reads below are avoided by an XOR swizzle instead of padding: the 16-byte segment `seg` of
  // tile row `row` lives at segment position seg ^ f(row), f(row) = 2 (row % 8) ^ ((row / 8) % 2),
  // which the loading lane realises by fetching global segment (its LDS position) ^ f(row).
  // Wave w fills rows 16 w + 4 i .. + 3 with instruction i = 0..3.  Rows that fall outside the
  // candidates re-read the last row (finite values; their logits are masked).
  const int k_ss_cache = static_cast<int>(ks.cache.ss), k_ss_chunk = static_cast<int>(ks.chunk.ss);
  const int v_ss_cache = static_cast<int>(vs.cache.ss), v_ss_chunk = static_cast<int>(vs.chunk.ss);
  auto seg_bytes = [](int rows_, int ss_) { return rows_ > 0 ? ((rows_ - 1) * ss_ + D) * 2 : 0; };
  const __amdgpu_buffer_rsrc_t k_rs_cache = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(unit_ptr(ks.cache, b, l, g)), 0, seg_bytes(n_c, k_ss_cache), kBufferFlags);
  const __amdgpu_buffer_rsrc_t k_rs_chunk = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(unit_ptr(ks.chunk, b, l, g)), 0, seg_bytes(ks.c, k_ss_chunk), kBufferFlags);
  const __amdgpu_buffer_rsrc_t v_rs_cache = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(unit_ptr(HAS_PV ? vs.cache : ks.cache, b, l, g)), 0, seg_bytes(n_c, v_ss_cache), kBufferFlags);
  const __amdgpu_buffer_rsrc_t v_rs_chunk = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(unit_ptr(HAS_PV ? vs.chunk : ks.chunk, b, l, g)), 0, seg_bytes(ks.c, v_ss_chunk), kBufferFlags);
  const int fill_row_c = kFillRows * wu + lane / 16;                // tile row this lane fills with instruction 0
  const int fill_seg16_c = ((lane % 16) ^ (2 * (lane / 16))) * 16;  // byte offset of its global segment, before ^ c_i
  // instruction i covers rows r = kFillRows wu + 4 i .. + 3; the lane-independent part of f(row)
  auto swz16 = [&](int i) {
    const int r = kFillRows * wu + 4 * i;
    return ((2 * (r % 8)) ^ ((r / 8) % 2)) * 16;
  };
  typedef __attribute__((address_space(3))) void* lds_void_ptr;
  auto fill4 = [&](char* lds_tile, __amdgpu_buffer_rsrc_t rs_cache, __amdgpu_buffer_rsrc_t rs_chunk, int ss_cache,
                   int ss_chunk, int j0) {
    const bool simple = (j0 + kTileN <= n_c) || (j0 >= n_c && j0 + kTileN <= n);  // block-uniform
    // the per-lane offsets are recomputed at every fill: hoisted out of the loop they would occupy
    // registers the pipeline needs (the empty asm hides their loop invariance from the optimiser)
    int fill_row = fill_row_c, fill_seg16 = fill_seg16_c;
    hide_loop_invariance(fill_row, fill_seg16);
    if (simple) {  // the whole tile lies in one segment: one resource, scalar row offsets
      const bool in_cache = j0 < n_c;
      const __amdgpu_buffer_rsrc_t rs = in_cache ? rs_cache : rs_chunk;
      const int ss2 = (in_cache ? ss_cache : ss_chunk) * 2;
      const int r0 = in_cache ? j0 : j0 - n_c;
      const int row_off = fill_row * ss2;
#pragma unroll
      for (int i = 0; i < kFillInstr; ++i)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void_ptr)(lds_tile + (kFillRows * wu + 4 * i) * kRowBytes), 16,
                                                 row_off + (fill_seg16 ^ swz16(i)), (r0 + 4 * i) * ss2, 0, 0);
    } else {  // the tile straddles the cache / chunk boundary or the end of the candidates
#pragma unroll
      for (int i = 0; i < kFillInstr; ++i) {
        lds_void_ptr dst = (lds_void_ptr)(lds_tile + (kFillRows * wu + 4 * i) * kRowBytes);
        const int seg = fill_seg16 ^ swz16(i);
        const int j = min(j0 + fill_row + 4 * i, n - 1);
        if (j < n_c)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_cache, dst, 16, j * ss_cache * 2 + seg, 0, 0, 0);
        else
          __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_chunk, dst, 16, (j - n_c) * ss_chunk * 2 + seg, 0, 0, 0);
      }
    }
  };

  // per-lane LDS read offsets (bytes inside a tile buffer), swizzle included
  // A operand of S^T: key row `col`, head_dim segment 2 kk + grp
  const int f_col = (2 * (col & 7)) ^ ((col >> 3) & 1);
  // k_off(kk) = col * kRowBytes + ((2 kk + grp) ^ f_col) * 16 = k_off0 ^ (32 kk): one register instead of eight
  const int k_off0 = col * kRowBytes + ((grp ^ f_col) * 16);
  auto k_off = [&](int kk) { return k_off0 ^ (32 * kk); };
  // V^T operand through transpose reads.  The 16-lane group q16 = lane / 16 serves MFMA rows
  // 16 (q16 % 2) .. +15 for contraction lane group q16 / 2; output row c' of tile r is head_dim
  // 16 r + (c' % 16) + 64 (c' / 16).  Source lane s16 points at 4 consecutive head_dim values of key
  // row 4 (q16 / 2) + s16 / 4 (+ 8 rd + 16 half + 32 mt): segment 2 r + 8 (q16 % 2) + (s16 % 4) / 2.
  const int s16 = lane % 16, q16 = lane / 16;
  const int v_cl = (8 * (q16 % 2) + (s16 % 4) / 2) ^ (8 * (q16 / 2) + 2 * (s16 / 4));
  // v_off(e), e = 2 r + rd (f(row) of read rd differs from read 0 by ^ rd), = v_off0 ^ (16 e)
  const int v_off0 = (4 * (q16 / 2) + s16 / 4) * kRowBytes + (v_cl * 16) + 8 * (s16 % 2);
  auto v_off = [&](int e) { return v_off0 ^ (16 * e); };

  // The first step of a row block multiplies p_prev = 0 with the second half of V buffer 1, which nothing has
  // filled yet in the first row block: zero it once (0 x garbage could be NaN).  Published by the barrier
  // in front of the first operand reads.
  *reinterpret_cast<uint4*>(v_s + kTileBytes + 32 * kRowBytes + 16 * tid) = make_uint4(0u, 0u, 0u, 0u);
  static_assert(WAVES * 64 * 16 == 32 * kRowBytes, "one 16-byte store per thread covers the half tile");

  for (int pass = 0; pass < passes; ++pass) {
  const int rb = pass == 0 ? rb_first : rb_second;
  const int row0 = (rb * ts.tiles_per_block + wu / ts.heads_per_block) * kRowsPerWave;

  // last candidate any row of this block / this wave can see
  const int blk_row_last = min(rows, (rb + 1) * rows_per_block) - 1;
  const int blk_limit = causal ? n_c + blk_row_last : n - 1;
  const int all_tiles = blk_limit / kTileN + 1;
  const int tiles_per_split = (all_tiles + key_splits - 1) / key_splits;
  const int t_begin = sp * tiles_per_split;
  const int t_end = min(all_tiles, t_begin + tiles_per_split);
  const bool wave_active = row0 < rows;
  const int wave_limit_min = causal ? n_c + row0 : n - 1;           // up to it every row sees everything

  // ---- Q^T operand, kept in registers: q_op[kk] = Q[row0 + col][16 kk + 8 grp ..+7] ----
  // (loaded further down, behind the requests for the first tiles: a lane reads 16-byte pieces of its
  // own row, 64 scattered pieces per instruction, which keep the address path busy for a while)
  bf16x8 q_op[8];
  const int t_lane = max(min(row0 + col, rows - 1), 0);
  const int limit_lane = causal ? n_c + t_lane : n - 1;

  // ---- running softmax state: one query per lane ----
  const float c2 = dm.scale * kLog2e;  // logits are kept in the log2 domain
  float m_run = -INFINITY, l_run = 0.f;
  // Optional by-product: each row's log-sum-exp over the cache states alone, i.e. the running
  // (maximum, sum) pair at the moment the last cache half tile has been added.  Needs the cache to end
  // on a half-tile boundary (the launcher checks); every row sees every cache state.
  const int snap_h = lse_cache != nullptr ? n_c / 32 - 1 : -1;
  float m_snap = -INFINITY, l_snap = 0.f;
  f32x16 o_acc[4];
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int i = 0; i < 16; ++i) o_acc[r][i] = 0.f;

  // fetch of one 64-key tile of K or of V into buffer (tile - t_begin) % 2
  auto fetch_k = [&](int tile) {
    fill4(k_s + ((tile - t_begin) & 1) * kTileBytes, k_rs_cache, k_rs_chunk, k_ss_cache, k_ss_chunk, tile * kTileN);
  };
  auto fetch_v = [&](int tile) {
    fill4(v_s + ((tile - t_begin) & 1) * kTileBytes, v_rs_cache, v_rs_chunk, v_ss_cache, v_ss_chunk, tile * kTileN);
  };
  // A tile that lies inside one segment is fetched with four instructions that differ only in
  // scalar operands; such fetches can be issued one by one between the MFMAs of a step.
  struct FillPlan {
    __amdgpu_buffer_rsrc_t rs;
    char* lds;    // first row this wave fills
    int soff;     // byte offset of instruction 0's first row inside the segment
    int ss8;      // bytes between the rows of consecutive instructions (4 rows)
    int row_off;  // per lane: its row inside the instruction's four rows, in bytes
    int seg16;    // per lane: byte offset of its 16-byte segment before the per-instruction swizzle term
  };
  // At most two tiles are not: the one that holds the cache / chunk boundary and the one that holds
  // the end of the candidates.
  const int straddle_tile = (n_c % kTileN) ? n_c / kTileN : -1;
  const int ragged_tile = (n % kTileN) ? n / kTileN : -1;
  auto tile_is_simple = [&](int tile) { return tile != straddle_tile && tile != ragged_tile; };
  auto plan_fill = [&](char* buffer, int tile, __amdgpu_buffer_rsrc_t rs_cache, __amdgpu_buffer_rsrc_t rs_chunk,
                       int ss_cache, int ss_chunk) {  // `buffer`: the tile buffer of the right parity
    const int j0 = tile * kTileN;
    const bool in_cache = j0 < n_c;
    const int ss2 = (in_cache ? ss_cache : ss_chunk) * 2;
    int fill_row = lane / 16, fill_seg16 = fill_seg16_c;
    hide_loop_invariance(fill_row, fill_seg16);  // formed per fetch: see fill4
    FillPlan fp;
    fp.rs = in_cache ? rs_cache : rs_chunk;
    fp.lds = buffer + kFillRows * wu * kRowBytes;
    fp.soff = ((in_cache ? j0 : j0 - n_c) + kFillRows * wu) * ss2;
    fp.ss8 = 4 * ss2;
    fp.row_off = fill_row * ss2;
    fp.seg16 = fill_seg16;
    return fp;
  };
  auto fill_one = [&](const FillPlan& fp, int i) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(fp.rs, (lds_void_ptr)(fp.lds + 4 * i * kRowBytes), 16,
                                             fp.row_off + (fp.seg16 ^ swz16(i)),
                                             fp.soff + i * fp.ss8, 0, 0);
  };

  const int h_first = 2 * t_begin, h_last = 2 * t_end - 1;  // half tiles of 32 keys (block-uniform)
  f32x16 s_cur;            // logits of the half tile whose probabilities are computed next
  uint32_t p_prev[8];      // bf16 probabilities of the half tile before it, not yet multiplied with V
  Pack8 ka[8];             // K operand of the next logit product, read one step ahead
  float mx_cur = 0.f;      // this lane's maximum over s_cur (before masking)
#pragma unroll
  for (int x = 0; x < 8; ++x) p_prev[x] = 0u;
  auto read_k_ops = [&](int hn_raw) {  // half tile hn_raw, clamped to the last one
    const int hn = min(hn_raw, h_last);
    const char* k_t = k_s + (((hn >> 1) - t_begin) & 1) * kTileBytes + (hn & 1) * 32 * kRowBytes;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) ka[kk].u = *reinterpret_cast<const uint4*>(k_t + k_off(kk));
  };

  // The same with the buffer parity and the half tile as constants: inside the key loop (unrolled over the
  // two parities) every LDS address is then a per-lane register plus an immediate offset.  No clamp: what is
  // read past the last tile feeds logits that are never used.
  auto read_k_ops_at = [&](auto parity, auto half) {
    const char* k_t = k_s + decltype(parity)::value * kTileBytes + decltype(half)::value * 32 * kRowBytes;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) ka[kk].u = *reinterpret_cast<const uint4*>(k_t + k_off(kk));
  };

  // One step: finish the softmax of half tile h (logits in s_cur) while the logits of h + 1 and the
  // product P(h - 1).V run on the matrix pipe.  Past either end the neighbour is clamped: the
  // logits computed past the end are never used, and p_prev is zero before the first step.
  // With fill_k / fill_v the four fetch instructions of that plan are issued between the MFMAs.
  // v_t: the V half tile that belongs to half tile hc - 1.
  auto half_step = [&](int hc, const char* v_t, bool fill_k, bool fill_v, const FillPlan& fk, const FillPlan& fv) {
    const int jb = 32 * hc;
    if (jb + 31 > wave_limit_min) {  // wave-uniform: the causal edge and the ragged end only
      const int lim_rel = limit_lane - jb - 4 * grp;
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if (8 * (i / 4) + (i % 4) > lim_rel) s_cur[i] = -INFINITY;
      mx_cur = s_cur[0];
#pragma unroll
      for (int i = 1; i < 16; ++i) mx_cur = fmaxf(mx_cur, s_cur[i]);
    }
    // Running maximum, kept lazily: softmax is invariant to the subtracted value, so m_run only has
    // to stay within kMaxSlack (log2 units) of the true row maximum to keep exp2 in range.  The
    // lane's maximum over the half tile was taken at the end of the previous step.
    float mx = mx_cur;
    if (__any(mx * c2 > m_run + kMaxSlack)) {  // wave-uniform and rare after the first tiles
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m_run, mx * c2);
      // 0 on a row's first visible tile (m_run = -inf); 1 for a row that has seen nothing yet
      const float alpha = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(m_run - m_new);
      l_run *= alpha;
      // the last P.V MFMAs of the previous step may still be in flight and the compiler cannot see them
      wait_for_pinned_mfmas();
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int i = 0; i < 16; ++i) o_acc[r][i] *= alpha;
      // the probabilities still waiting for their product with V were taken against the old maximum
#pragma unroll
      for (int x = 0; x < 8; ++x) {
        const float lo = __uint_as_float(p_prev[x] << 16), hi = __uint_as_float(p_prev[x] & 0xffff0000u);
        p_prev[x] = pack_bf16x2(lo * alpha, hi * alpha);
      }
      m_run = m_new;
    }
    const float m_sub = m_run == -INFINITY ? 0.f : m_run;  // a row that has seen nothing yet: exp2(-inf) = 0
    __builtin_amdgcn_sched_barrier(0);

    // O^T += V^T . P^T: contraction step `half` covers keys 16 half .. +15 of the half tile in the slot
    // order the S^T accumulators have: slot i of lane group grp is key 8 (i / 4) + 4 grp + (i % 4) of
    // the step, so slots 0..3 / 4..7 are two transpose reads.
    // The V^T operands of the second contraction step are read once half of the K operands are
    // spent (the empty asm with a memory clobber keeps the reads from being hoisted above it):
    // all sixteen up front would not fit the register budget.
    Pack8 va[2][4];
    auto read_v_ops = [&](int half) {
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int rd = 0; rd < 2; ++rd)
          va[half][r].h[rd] = lds_read_tr16(v_t + (16 * half + 8 * rd) * kRowBytes + v_off(2 * r + rd));
    };
    read_v_ops(0);
    // sixteen MFMAs; the exponential of logit x of half tile h is issued right before MFMA x + 1
    float p[16];
    float mx_nxt = 0.f;
    f32x16 s_nxt = mfma_pinned_first(ka[0].v, q_op[0]);
#pragma unroll
    for (int kk = 1; kk < 8; ++kk) {
      p[kk - 1] = exp2_then_mfma(fmaf(s_cur[kk - 1], c2, -m_sub), s_nxt, ka[kk].v, q_op[kk]);
      if ((kk & 1) && kk / 2 < kFillInstr && fill_k) fill_one(fk, kk / 2);  // block-uniform
      if (kk == 4) {
        no_memory_motion();
        read_v_ops(1);
      }
    }
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      Pack8 pb;
#pragma unroll
      for (int x = 0; x < 4; ++x) pb.w[x] = p_prev[4 * half + x];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int x = 7 + 4 * half + r;
        p[x] = exp2_then_mfma(fmaf(s_cur[x], c2, -m_sub), o_acc[r], va[half][r].v, pb.v);
        if ((r & 1) && 2 * half + r / 2 < kFillInstr && fill_v) fill_one(fv, 2 * half + r / 2);  // block-uniform
        // The lane's maximum of the next half tile's logits, one v_max3 per MFMA slot.  s_nxt was
        // completed by the eighth MFMA of the step; three further MFMAs have been issued since.
        const int y = 4 * half + r - 2;  // 0 .. 5
        if (y == 0) mx_nxt = max3_pinned(s_nxt[0], s_nxt[1], s_nxt[2]);
        if (y > 0) mx_nxt = max3_pinned(mx_nxt, s_nxt[2 * y + 1], s_nxt[2 * y + 2]);
      }
    }
    p[15] = exp2_pinned(fmaf(s_cur[15], c2, -m_sub));
    mx_nxt = max3_pinned(mx_nxt, s_nxt[13], s_nxt[14]);
    mx_nxt = fmaxf(mx_nxt, s_nxt[15]);
    // the row sum is taken over the bf16-rounded probabilities, the values P.V uses: one v_dot2
    // with (1, 1) adds a pair
    uint32_t p_cur[8];
    float psum = 0.f;
#pragma unroll
    for (int x = 0; x < 8; ++x) {
      p_cur[x] = pack_bf16x2(p[2 * x], p[2 * x + 1]);
      psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, p_cur[x]),
                                             __builtin_bit_cast(bf16x2, 0x3f803f80u), psum, false);
    }
    l_run += psum;
    if (hc == snap_h) {  // block-uniform
      m_snap = m_run;
      l_snap = l_run;
    }
    // keep the probabilities in this block: without a use here the optimiser sinks the exponentials
    // to their first use in the next step, behind the MFMAs they are meant to overlap with
    keep_values_here(p_cur, l_run);
    __builtin_amdgcn_sched_barrier(0);
    s_cur = s_nxt;
    mx_cur = mx_nxt;
#pragma unroll
    for (int x = 0; x < 8; ++x) p_prev[x] = p_cur[x];
  };
  const FillPlan no_plan{};

  if (t_begin < t_end) {  // block-uniform
  fetch_k(t_begin);
  fetch_v(t_begin);
  if (t_begin + 1 < t_end) fetch_k(t_begin + 1);
  // The wave's 32 query rows come in through LDS as well: whole 256-byte rows, four per load
  // instruction, into the wave's own 8 KB (same swizzle as a key tile), from where the B operand is
  // read like a key operand.  Loading them straight into the operand layout would put 64 scattered
  // 16-byte pieces into every load instruction.
  {
    const int q_ss2 = static_cast<int>(q.ss) * 2;
    const __amdgpu_buffer_rsrc_t q_rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>(unit_ptr(q, b, l, h)), 0, ((rows - 1) * static_cast<int>(q.ss) + D) * 2, kBufferFlags);
    int r_in = lane / 16, pos = lane % 16;
    hide_loop_invariance(r_in, pos);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = 4 * i + r_in;
      const int f = (2 * (r % 8)) ^ ((r / 8) % 2);
      const int row = min(row0 + r, rows - 1);  // rows past the end repeat the last one; never stored
      __builtin_amdgcn_raw_ptr_buffer_load_lds(q_rs, (lds_void_ptr)(q_stage + (32 * wu + 4 * i) * kRowBytes), 16,
                                               max(row, 0) * q_ss2 + ((pos ^ f) * 16), 0, 0, 0);
    }
  }
  barrier_after_lds_fill();  // also: the query rows have landed
  // Position shift: the query rows arrive without rotary embedding and are rotated here, in the staging
  // region, to position q_rope_pos0 + row, before the operands are read (only a few registers are live at
  // this point; rotating the operands in registers pushed the whole kernel over its register budget).
  // Element i of a row pairs with element i + 64: 16-byte segment sg with segment sg + 8.  A lane takes
  // one (row, sg) of the wave's 32 x 8 per round; the wave touches only its own rows, so no barrier.
  if (ROTATE_Q) {
    char* q_t = q_stage + 32 * wu * kRowBytes;
#pragma unroll 1
    for (int round = 0; round < 4; ++round) {
      const int r = 8 * round + lane / 8, sg = lane % 8;
      const int f = (2 * (r % 8)) ^ ((r / 8) % 2);
      uint4* lo_p = reinterpret_cast<uint4*>(q_t + r * kRowBytes + ((sg ^ f) * 16));
      uint4* hi_p = reinterpret_cast<uint4*>(q_t + r * kRowBytes + (((sg + 8) ^ f) * 16));
      Pack8 lo, hi;
      lo.u = *lo_p;
      hi.u = *hi_p;
      const int pos = q_rope_pos0 + max(min(row0 + r, rows - 1), 0);
#pragma unroll
      for (int wd = 0; wd < 4; ++wd) {
        const int i0 = 8 * sg + 2 * wd;
        float s0, c0, s1, c1;
        rope_sincos_bf16(pos, i0, D, rope_log2_base, s0, c0);
        rope_sincos_bf16(pos, i0 + 1, D, rope_log2_base, s1, c1);
        rope_rotate_words(lo.w[wd], hi.w[wd], c0, s0, c1, s1, lo.w[wd], hi.w[wd]);
      }
      *lo_p = lo.u;
      *hi_p = hi.u;
    }
  }
  {
    const char* q_t = q_stage + 32 * wu * kRowBytes;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      Pack8 p;
      p.u = *reinterpret_cast<const uint4*>(q_t + k_off(kk));
      q_op[kk] = p.v;
    }
  }
  read_k_ops(h_first);
#pragma unroll
  for (int i = 0; i < 16; ++i) s_cur[i] = 0.f;
#pragma unroll
  for (int kk = 0; kk < 8; ++kk)  // logits of the first half tile
    s_cur = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[kk].v, q_op[kk], s_cur, 0, 0, 0);
  mx_cur = s_cur[0];
#pragma unroll
  for (int i = 1; i < 16; ++i) mx_cur = fmaxf(mx_cur, s_cur[i]);
  read_k_ops(h_first + 1);
  // One 64-key tile per call; `parity` is the tile's buffer (t_begin = 0 in this kernel: tile jt lives in
  // buffer jt % 2), so the loop below alternates two copies of the step whose LDS offsets are constants.
  static_assert(key_splits == 1, "the tile buffers are addressed by jt % 2");
  auto tile_step = [&](auto parity, int jt) {
    constexpr int P = decltype(parity)::value;
    // P.V of the second half of tile jt - 1 (before the first tile: p_prev = 0 times the zeros written at
    // kernel start, or times stale finite data in later row blocks)
    half_step(2 * jt, v_s + (1 - P) * kTileBytes + 32 * kRowBytes, false, false, no_plan, no_plan);
    // Every wave has read the second half of K tile jt and the last of V tile jt - 1: their buffers
    // take K tile jt + 2 and V tile jt + 1, which are first read after the next barrier.
    barrier_after_lds_fill();
    read_k_ops_at(std::integral_constant<int, 1 - P>{}, std::integral_constant<int, 0>{});  // K tile jt + 1, first half
    // Tiles inside one segment are fetched from within the step, one instruction between two
    // MFMAs (plans of tiles that are not wanted are formed but never used); the others here.
    const bool want_k = jt + 2 < t_end, want_v = jt + 1 < t_end;
    const bool k_inside = want_k && tile_is_simple(jt + 2), v_inside = want_v && tile_is_simple(jt + 1);
    if (want_k && !k_inside) fetch_k(jt + 2);
    if (want_v && !v_inside) fetch_v(jt + 1);
    const FillPlan fk = plan_fill(k_s + P * kTileBytes, jt + 2, k_rs_cache, k_rs_chunk, k_ss_cache, k_ss_chunk);
    const FillPlan fv = plan_fill(v_s + (1 - P) * kTileBytes, jt + 1, v_rs_cache, v_rs_chunk, v_ss_cache, v_ss_chunk);
    half_step(2 * jt + 1, v_s + P * kTileBytes, k_inside, v_inside, fk, fv);
    read_k_ops_at(std::integral_constant<int, 1 - P>{}, std::integral_constant<int, 1>{});  // K tile jt + 1, second half
  };
  for (int jt = t_begin; jt < t_end; jt += 2) {
    tile_step(std::integral_constant<int, 0>{}, jt);
    if (jt + 1 < t_end) tile_step(std::integral_constant<int, 1>{}, jt + 1);
  }
  {  // the product of the last half tile
    const char* v_t = v_s + ((t_end - 1 - t_begin) & 1) * kTileBytes + 32 * kRowBytes;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      Pack8 va[4];
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int rd = 0; rd < 2; ++rd)
          va[r].h[rd] = lds_read_tr16(v_t + (16 * half + 8 * rd) * kRowBytes + v_off(2 * r + rd));
      Pack8 pb;
#pragma unroll
      for (int x = 0; x < 4; ++x) pb.w[x] = p_prev[4 * half + x];
#pragma unroll
      for (int r = 0; r < 4; ++r) o_acc[r] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[r].v, pb.v, o_acc[r], 0, 0, 0);
    }
  }
  __syncthreads();  // the buffers are free for the next row block
  }

  const float l_snap_tot = l_snap + __shfl_xor(l_snap, 32, 64);
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const int t = row0 + col;
  if (wave_active && t < rows) {
  const int64_t row_id = (static_cast<int64_t>(bl) * dm.Hq + h) * rows + t;
  if (part != nullptr && grp == 0)  // log2 domain; an empty or fully masked range leaves (-inf, 0)
    part[static_cast<int64_t>(sp) * dm.B * dm.L * dm.Hq * rows + row_id] = make_float2(m_run, l_tot);
  if (lse_cache != nullptr && grp == 0) lse_cache[row_id] = (m_snap + log2f(l_snap_tot)) * kLn2;
  if (lse != nullptr && grp == 0) lse[row_id] = (m_run + log2f(l_tot)) * kLn2;
  }  // row valid
  // The output tile leaves through LDS: a lane holds 4-element pieces of ONE query row (256 bytes
  // between neighbouring lanes), so direct stores put 64 scattered 8-byte pieces into every store
  // instruction and keep the compute unit's address path busy for microseconds per row block.  Each
  // wave parks its 32 x 128 tile in its own 8 KB of the tile buffers (free after the barrier above;
  // 16-byte segments XOR-swizzled by the row so that the column-wise writes spread over the banks)
  // and stores it back as whole 256-byte rows.
  {
    int colx = col, lanex = lane;
    hide_loop_invariance(colx, lanex);  // offsets are formed here, per row block, not kept in registers
    char* o_s = (wu < 4 ? k_s : v_s) + (wu % 4) * (32 * kRowBytes) + colx * kRowBytes;
    // A lane pair (col, col + 32) shares every 16-byte segment.  The LDS has 32 banks of 4 bytes, so segment
    // positions p and p + 8 of a row meet in the same banks, and 16 lanes go through per cycle: the two 8-byte
    // halves of a segment are kept swapped where (p / 8) ^ (row / 16) is odd, which gives the 16 lanes of a
    // cycle 16 different 8-byte slots of the 128 bytes the banks span.
    const int c16 = colx % 16, half0 = grp ^ (colx / 16);
    const float inv = 1.f / l_tot;
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        // registers 4 i4 .. +3 are rows c' = 8 i4 + 4 grp + 0..3 -> head_dim 16 r + (c' % 16) + 64 (c' / 16):
        // 16-byte segment 2 r + (i4 % 2) + 8 (i4 / 2), its half `grp`
        const int sg = 2 * r + (i4 % 2) + 8 * (i4 / 2);
        uint2 wds;
        wds.x = pack_bf16x2(o_acc[r][4 * i4] * inv, o_acc[r][4 * i4 + 1] * inv);
        wds.y = pack_bf16x2(o_acc[r][4 * i4 + 2] * inv, o_acc[r][4 * i4 + 3] * inv);
        const int p = sg ^ c16;  // segment position
        *reinterpret_cast<uint2*>(o_s + p * 16 + 8 * (half0 ^ (p >> 3))) = wds;
      }
    const char* o_r = (wu < 4 ? k_s : v_s) + (wu % 4) * (32 * kRowBytes) + lanex * 16;  // row lanex / 16 of a 4-row group
    const int r_in = lanex / 16, pos = lanex % 16;
    uint16_t* ob = const_cast<uint16_t*>(unit_ptr(out, b, l, h));
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = 4 * i + r_in;
      uint4 piece = *reinterpret_cast<const uint4*>(o_r + 4 * i * kRowBytes);
      if (((pos >> 3) ^ (i >> 2)) & 1) piece = make_uint4(piece.z, piece.w, piece.x, piece.y);  // halves back in order
      if (wave_active && row0 + r < rows)
        *reinterpret_cast<uint4*>(ob + static_cast<int64_t>(row0 + r) * out.ss + 8 * (pos ^ (r % 16))) = piece;
    }
  }
  __syncthreads();  // the parked tiles have been read back: the next row block may fill the buffers
  }  // pass
}

// Eight waves per workgroup: two 32-row tiles of the four heads of a KV group (or the equivalent
// split for smaller groups) share every K/V tile, which halves the fetch traffic per MFMA
// against four waves; one workgroup per CU, two waves per SIMD.
__global__ __launch_bounds__(512, 1) void attn_pipe_kernel_w8(Dims dm, View q, int rows, Segments ks, Segments vs,
                                                             int causal, View out, float* lse, float* lse_cache) {
  attn_pipe_body<8, false>(dm, q, rows, ks, vs, causal, out, lse, lse_cache, -1, 0.f);
}
// The same kernel for query rows that arrive without rotary embedding (position shift): they are rotated
// in the LDS staging region before the operands are read.  An instance of its own, so that the kernel
// above does not carry the extra prologue.
__global__ __launch_bounds__(512, 1) void attn_pipe_kernel_w8_rotq(Dims dm, View q, int rows, Segments ks, Segments vs,
                                                                  int causal, View out, float* lse, float* lse_cache,
                                                                  int q_rope_pos0, float rope_log2_base) {
  attn_pipe_body<8, true>(dm, q, rows, ks, vs, causal, out, lse, lse_cache, q_rope_pos0, rope_log2_base);
}

// Brings the per-range (maximum, sum) pairs of a row, part[s * rows_total + row], to one normaliser,
// left in part[row] as (log-sum-exp in the log2 domain, 1): a pair that the column-sum kernel reads like
// any single range.  Done once per row here rather than by every workgroup of the column-sum launch
// (one per 256 keys), each of which walked the ranges with dependent loads in front of every chunk.
__global__ __launch_bounds__(256) void merge_partials_kernel(float2* part, int key_splits, int64_t rows_total) {
  const int64_t row = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (row >= rows_total) return;
  float2 ps[kMaxKeySplits];
#pragma unroll
  for (int s = 0; s < kMaxKeySplits; ++s)  // independent loads; an absent range counts as (-inf, 0)
    ps[s] = s < key_splits ? part[s * rows_total + row] : make_float2(-INFINITY, 0.f);
  float m = -INFINITY;
#pragma unroll
  for (int s = 0; s < kMaxKeySplits; ++s) m = fmaxf(m, ps[s].x);
  float lsum = 0.f;
#pragma unroll
  for (int s = 0; s < kMaxKeySplits; ++s)
    if (s < key_splits) lsum += ps[s].y * exp2f(ps[s].x - m);
  part[row] = make_float2(m + log2f(lsum), 1.f);
}

// Summed form of Eq. (1): score[g, j] = sum over the query rows of the KV group of
// exp(s - lse).  One wave per 32 candidate keys, which stay in registers as the A operand; the
// group's query rows (all its heads, flattened) are staged through LDS in chunks of 128 rows and
// stream by as B operands.  Per-lane partial sums are reduced across the 32 query lanes once at
// the end, in a fixed order: no atomics, bit-reproducible.
constexpr int kColsumWaves = 8;
constexpr int kColsumKeyTiles = 1;  // 32-key tiles per wave: a workgroup covers 256 keys per staged Q chunk
constexpr int kColsumQRows = 128;   // query rows per LDS chunk
// STEPWISE: rows is a multiple of kColsumQRows, so every chunk of staged rows is full and lies inside one
// head (an instance of its own: both address paths in one kernel cost the registers that two workgroups
// per compute unit need).
template <bool STEPWISE>
__global__ __launch_bounds__(kColsumWaves * 64, 4) void colsum_mfma_kernel(Dims dm, View q, int rows, Segments ks,
                                                                        int causal, const float* lse, int key_splits,
                                                                        const float2* part, float* score) {
  // two staging buffers of query rows and their normalisers (log2 domain, +inf for padding rows)
  extern __shared__ __attribute__((aligned(16))) char colsum_smem[];
  uint16_t* const q_sb = reinterpret_cast<uint16_t*>(colsum_smem);                        // [2][kColsumQRows][kPitchK]
  float* const lse_sb = reinterpret_cast<float*>(q_sb + 2 * kColsumQRows * kPitchK);      // [2][kColsumQRows]
  const int tid = threadIdx.x, lane = tid % 64, w = tid / 64;
  const int col = lane % 32, grp = lane / 32;
  const int g = blockIdx.y, bl = blockIdx.z, b = bl / dm.L, l = bl % dm.L;
  const int n_c = ks.n_c, n = n_c + ks.c;
  const int j0 = (blockIdx.x * kColsumWaves + w) * (32 * kColsumKeyTiles);
  const bool wave_has_keys = j0 < n;
  const int j_last = j0 + 32 * kColsumKeyTiles - 1;

  bf16x8 k_op[kColsumKeyTiles][8];
  // bases and strides are read once: a per-lane choice between the two structs' fields would compile to a
  // per-lane load of the chosen field from the argument block
  const uint16_t* const k_cache_u = unit_ptr(ks.cache, b, l, g) + 8 * grp;
  const uint16_t* const k_chunk_u = unit_ptr(ks.chunk, b, l, g) + 8 * grp;
  const int64_t k_ss_cache = ks.cache.ss, k_ss_chunk = ks.chunk.ss;
#pragma unroll
  for (int kt = 0; kt < kColsumKeyTiles; ++kt) {
    const int j = min(j0 + 32 * kt + col, n - 1);
    const bool in_cache = j < n_c;
    const int64_t off = in_cache ? j * k_ss_cache : (j - n_c) * k_ss_chunk;
    const uint16_t* kp = (in_cache ? k_cache_u : k_chunk_u) + off;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      Pack8 p;
      p.u = *reinterpret_cast<const uint4*>(kp + 16 * kk);
      k_op[kt][kk] = p.v;
    }
  }
  const float c2 = dm.scale * kLog2e;
  float acc[kColsumKeyTiles][16];
#pragma unroll
  for (int kt = 0; kt < kColsumKeyTiles; ++kt)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[kt][i] = 0.f;

  const int total_rows = dm.G * rows;  // flattened (head in group, row)
  const int64_t part_stride = static_cast<int64_t>(dm.B) * dm.L * dm.Hq * rows;
  // The rows of chunk c + 1 are requested (into registers) before the products of chunk c start and
  // written to the other buffer afterwards: one barrier per chunk, no exposed load latency.
  // A thread stages 16 bytes of rows tid / 16 + 32 x of a chunk.  STEPWISE: every chunk lies inside one head
  // and is full, so its first row is a wave-uniform pointer that moves on by adds, and a thread's part of the
  // address never changes; dividing the flattened row index by `rows` for every load cost more vector
  // instructions per chunk than three of its four products.
  constexpr int kStageLoads = kColsumQRows / (kColsumWaves * 4);  // 16 threads per row, 16 bytes each
  constexpr int kStageStep = kColsumWaves * 4;                     // rows between a thread's loads
  i32x4 q_in[kStageLoads];
  float lse_in = INFINITY;
  const int64_t lse_row0 = (static_cast<int64_t>(bl) * dm.Hq + g * dm.G) * rows;  // the group's heads are consecutive
  const uint32_t q_thread_off = ((tid / 16) * static_cast<uint32_t>(q.ss) + 8 * (tid % 16)) * 2;  // bytes; a head's rows span < 2 GiB
  int stage_head = 0, stage_row = 0;  // where the next requested chunk starts (block-uniform)
  auto request_chunk = [&](int f0) {
    if constexpr (STEPWISE) {
      const uint16_t* const base = unit_ptr(q, b, l, g * dm.G + stage_head) + static_cast<int64_t>(stage_row) * q.ss;
#pragma unroll
      for (int x = 0; x < kStageLoads; ++x) {  // scalar base per load + one 32-bit per-thread byte offset
        const char* const base_x = reinterpret_cast<const char*>(base + x * kStageStep * q.ss);
        q_in[x] = *reinterpret_cast<const i32x4*>(base_x + q_thread_off);
      }
      stage_row += kColsumQRows;
      if (stage_row == rows) {
        stage_row = 0;
        ++stage_head;
      }
    } else {
#pragma unroll
      for (int x = 0; x < kStageLoads; ++x) {
        const int f = min(f0 + tid / 16 + x * kStageStep, total_rows - 1);
        const int hh = f / rows, t = f % rows;
        q_in[x] = *reinterpret_cast<const i32x4*>(unit_ptr(q, b, l, g * dm.G + hh) + static_cast<int64_t>(t) * q.ss +
                                                  8 * (tid % 16));
      }
    }
    float v = INFINITY;  // padding rows contribute exp2(-inf) = 0
    if (tid < kColsumQRows && f0 + tid < total_rows) {
      const int64_t row_id = lse_row0 + f0 + tid;
      if (part != nullptr) {  // merge the per-range (maximum, sum) pairs
        float m = -INFINITY;
        for (int s = 0; s < key_splits; ++s) m = fmaxf(m, part[s * part_stride + row_id].x);
        float lsum = 0.f;
        for (int s = 0; s < key_splits; ++s) {
          const float2 ps = part[s * part_stride + row_id];
          lsum += ps.y * exp2f(ps.x - m);
        }
        v = m + log2f(lsum);
      } else {
        v = lse[row_id] * kLog2e;
      }
    }
    lse_in = v;
  };
  request_chunk(0);
  int buf = 0;
  int chunk_row = 0;  // STEPWISE: row of its head at which the chunk being multiplied starts
  for (int f0 = 0; f0 < total_rows; f0 += kColsumQRows, buf ^= 1) {
    const int f_cnt = min(kColsumQRows, total_rows - f0);
    uint16_t* const q_s = q_sb + buf * (kColsumQRows * kPitchK);
    float* const lse_s = lse_sb + buf * kColsumQRows;
    // this buffer was last read two chunks ago, and every wave has passed the previous chunk's barrier since
#pragma unroll
    for (int x = 0; x < kStageLoads; ++x)
      *reinterpret_cast<i32x4*>(&q_s[(tid / 16 + x * kStageStep) * kPitchK + 8 * (tid % 16)]) = q_in[x];
    if (tid < kColsumQRows) lse_s[tid] = lse_in;
    if (f0 + kColsumQRows < total_rows) request_chunk(f0 + kColsumQRows);  // block-uniform
    __syncthreads();
    if (wave_has_keys) {
      for (int qt = 0; qt * 32 < f_cnt; ++qt) {
        const int tile_row = STEPWISE ? chunk_row + 32 * qt : (f0 + 32 * qt) % rows;  // wave-uniform
        if (causal) {  // wave-uniform: skip query tiles none of whose rows sees any key of this wave
          const int t_first = tile_row;
          const int t_last = t_first + 31 >= rows ? rows - 1 : t_first + 31;  // a tile that wraps reaches a head's end
          if (n_c + t_last < j0) continue;
        }
        Pack8 qb[8];
        const uint16_t* qrow = &q_s[(32 * qt + col) * kPitchK + 8 * grp];
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) qb[kk].u = *reinterpret_cast<const uint4*>(qrow + 16 * kk);
        const float lse2 = lse_s[32 * qt + col];
        // A mask is needed only where a key of this wave can be invisible to a row of this tile:
        // past the last candidate, or (causal) a chunk key later than the tile's first row.  The
        // flattened rows of one 32-row tile span at most two heads; t_lo is the smallest chunk row.
        const int f_first = f0 + 32 * qt;
        int t_lo = tile_row;
        if (t_lo + 31 >= rows) t_lo = 0;                            // tile wraps into the next head
        const bool need_mask = (j_last >= n) || (causal && j_last > n_c + t_lo);
        int limit = n - 1;
        if (need_mask && causal) limit = n_c + (STEPWISE ? tile_row + col : (f_first + col) % rows);
#pragma unroll
        for (int kt = 0; kt < kColsumKeyTiles; ++kt) {
          f32x16 s_t;
#pragma unroll
          for (int i = 0; i < 16; ++i) s_t[i] = 0.f;
#pragma unroll
          for (int kk = 0; kk < 8; ++kk)
            s_t = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k_op[kt][kk], qb[kk].v, s_t, 0, 0, 0);
          if (need_mask) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int j = j0 + 32 * kt + 8 * (i / 4) + 4 * grp + (i % 4);
              const float p = __builtin_amdgcn_exp2f(fmaf(s_t[i], c2, -lse2));
              acc[kt][i] += (j <= limit) ? p : 0.f;
            }
          } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[kt][i] += __builtin_amdgcn_exp2f(fmaf(s_t[i], c2, -lse2));
          }
        }
      }
    }
    if (STEPWISE) {
      chunk_row += kColsumQRows;
      if (chunk_row == rows) chunk_row = 0;
    }
  }
  if (!wave_has_keys) return;
#pragma unroll
  for (int kt = 0; kt < kColsumKeyTiles; ++kt)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      float v = acc[kt][i];
#pragma unroll
      for (int o = 16; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
      const int j = j0 + 32 * kt + 8 * (i / 4) + 4 * grp + (i % 4);
      if (col == 0 && j < n) score[(static_cast<int64_t>(bl) * dm.Hkv + g) * n + j] = v;
    }
}

// Sum of 16 per-lane values over the 32 lanes that share lane / 32, in 16 exchanges: each step
// halves the values a lane still carries (the lane keeps the half its own bit selects and takes
// the partner's partial sum of the same half).  On return lane c holds, for value index c / 2,
// the total over its 32 lanes.
__device__ inline float reduce16_over32(const float (&v)[16], int col) {
  float a[8], b[4], c[2];
  const bool u16 = col & 16, u8 = col & 8, u4 = col & 4, u2 = col & 2;
#pragma unroll
  for (int x = 0; x < 8; ++x) a[x] = (u16 ? v[x + 8] : v[x]) + __shfl_xor(u16 ? v[x] : v[x + 8], 16, 64);
#pragma unroll
  for (int x = 0; x < 4; ++x) b[x] = (u8 ? a[x + 4] : a[x]) + __shfl_xor(u8 ? a[x] : a[x + 4], 8, 64);
#pragma unroll
  for (int x = 0; x < 2; ++x) c[x] = (u4 ? b[x + 2] : b[x]) + __shfl_xor(u4 ? b[x] : b[x + 2], 4, 64);
  const float d = (u2 ? c[1] : c[0]) + __shfl_xor(u2 ? c[0] : c[1], 2, 64);
  return d + __shfl_xor(d, 1, 64);
}

// Instruction score (Eq. (1), summed form) in ONE launch for KV groups whose query rows
// (instruction rows x heads of the group, flattened) fit one LDS chunk: a workgroup owns one
// (document, layer, KV head).  All its query rows sit in LDS; wave (kw, qh) walks key tiles
// kw, kw + KW, ... (32 keys, in registers as the A operand) against q-tiles of its share qh:
//   pass 1  per-lane online (maximum, sum) over the wave's keys  -> merged over waves in LDS into
//           the row normaliser (log2 domain);
//   pass 2  the same products again, exp2(s - normaliser) summed down the query rows per key.
// Partial column sums of the q shares meet in LDS and are added in a fixed order: no atomics.
// With KREG > 0 a wave keeps its (at most KREG) key tiles in registers from the first pass to the
// second: K is read from memory once, and all its loads are in flight together at the start.
template <int QT_TOTAL, int Q_SPLIT, int WAVES, int KREG>
__global__ __launch_bounds__(WAVES * 64) void instr_fused_kernel(Dims dm, View q, int rows, Segments ks,
                                                                 float* score) {
  constexpr int KW = WAVES / Q_SPLIT;         // waves that share the key tiles
  constexpr int QT_PER = QT_TOTAL / Q_SPLIT;  // q-tiles per wave
  constexpr int QROWS = QT_TOTAL * 32;
  extern __shared__ __attribute__((aligned(16))) char fused_smem[];
  uint16_t* q_s = reinterpret_cast<uint16_t*>(fused_smem);              // [QROWS][kPitchK]
  float2* stats_s = reinterpret_cast<float2*>(q_s + QROWS * kPitchK);   // [KW][QROWS]
  float* lse_s = reinterpret_cast<float*>(stats_s + KW * QROWS);        // [QROWS]
  float* part_s = lse_s + QROWS;                                        // [Q_SPLIT][32 * tiles]

  const int tid = threadIdx.x, lane = tid % 64, w = tid / 64;
  const int col = lane % 32, grp = lane / 32;
  const int kw = w / Q_SPLIT, qh = w % Q_SPLIT;
  const int g = blockIdx.x % dm.Hkv, bl = blockIdx.x / dm.Hkv, b = bl / dm.L, l = bl % dm.L;
  const int n_c = ks.n_c, n = n_c + ks.c;
  const int tiles = (n + 31) / 32;
  const int total_rows = dm.G * rows;  // <= QROWS (the launcher guarantees it)
  const float c2 = dm.scale * kLog2e;

  const uint16_t* k_cache_u = unit_ptr(ks.cache, b, l, g) + 8 * grp;
  const uint16_t* k_chunk_u = unit_ptr(ks.chunk, b, l, g) + 8 * grp;
  // the strides are read here, once: a per-lane choice between the two struct fields inside the loader
  // would compile to a per-lane LOAD of the chosen field from the argument block, in front of every tile
  const int64_t k_ss_cache = ks.cache.ss, k_ss_chunk = ks.chunk.ss;
  auto load_keys = [&](int kt, bf16x8 (&k_op)[8]) {
    const int j = min(32 * kt + col, n - 1);
    const bool in_cache = j < n_c;
    const int64_t off = in_cache ? j * k_ss_cache : (j - n_c) * k_ss_chunk;
    const uint16_t* kp = (in_cache ? k_cache_u : k_chunk_u) + off;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      Pack8 p;
      p.u = *reinterpret_cast<const uint4*>(kp + 16 * kk);
      k_op[kk] = p.v;
    }
  };
  auto logits = [&](const bf16x8 (&k_op)[8], int qt) {  // S^T tile: 32 keys x the 32 rows of q-tile qt
    Pack8 qb[8];
    const uint16_t* qrow = &q_s[(32 * qt + col) * kPitchK + 8 * grp];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) qb[kk].u = *reinterpret_cast<const uint4*>(qrow + 16 * kk);
    f32x16 s_t;
#pragma unroll
    for (int i = 0; i < 16; ++i) s_t[i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) s_t = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k_op[kk], qb[kk].v, s_t, 0, 0, 0);
    return s_t;
  };

  // The query rows go through LDS.  They are requested first and waited for BEFORE the bulk of the key
  // loads is issued: every workgroup of the launch starts at the same moment, and behind 80+ MB of key
  // requests the query rows of the slowest wave (all of them are needed before the first product) arrive
  // when the whole burst is nearly through.  Loads return in order and the compiler counts them, so the
  // first pass then starts on a wave's first key tile while its later ones are still arriving.
  constexpr int kQLoads = QROWS / (WAVES * 4);  // 16 threads per row, 16 bytes each
  i32x4 q_in[kQLoads];
#pragma unroll
  for (int x = 0; x < kQLoads; ++x) {
    const int f = min(tid / 16 + x * WAVES * 4, total_rows - 1);  // padding rows repeat the last row; never summed
    const int hh = f / rows, t = f % rows;
    q_in[x] = *reinterpret_cast<const i32x4*>(unit_ptr(q, b, l, g * dm.G + hh) + static_cast<int64_t>(t) * q.ss +
                                              8 * (tid % 16));
  }
  __builtin_amdgcn_sched_barrier(0);  // keep the issue order
  bf16x8 k_res[KREG > 0 ? KREG : 1][8];
  if constexpr (KREG > 0) load_keys(min(kw, tiles - 1), k_res[0]);  // the launcher guarantees tiles <= KW * KREG
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int x = 0; x < kQLoads; ++x)
    *reinterpret_cast<i32x4*>(&q_s[(tid / 16 + x * WAVES * 4) * kPitchK + 8 * (tid % 16)]) = q_in[x];
  __syncthreads();

  // With resident key tiles the first pass requests tile i + 1 when it starts on tile i: a compute unit
  // can only keep so many requests in flight, so issuing all of a wave's key loads up front would hold
  // the wave (and with it the barrier above) until most of the keys have arrived.
  auto for_my_tiles = [&](auto first_pass, auto&& tile_fn) {
    if constexpr (KREG > 0) {
#pragma unroll
      for (int i = 0; i < KREG; ++i) {
        if constexpr (decltype(first_pass)::value) {
          __builtin_amdgcn_sched_barrier(0);
          if (i + 1 < KREG) load_keys(min(kw + KW * (i + 1), tiles - 1), k_res[i + 1]);
          __builtin_amdgcn_sched_barrier(0);
        }
        if (kw + KW * i < tiles) tile_fn(k_res[i], kw + KW * i);  // wave-uniform
      }
    } else {
      for (int kt = kw; kt < tiles; kt += KW) {
        bf16x8 k_op[8];
        load_keys(kt, k_op);
        tile_fn(k_op, kt);
      }
    }
  };

  // ---- pass 1: row normalisers ----
  float m_run[QT_PER], l_run[QT_PER];
#pragma unroll
  for (int x = 0; x < QT_PER; ++x) {
    m_run[x] = -INFINITY;
    l_run[x] = 0.f;
  }
  for_my_tiles(std::true_type{}, [&](const bf16x8 (&k_op)[8], int kt) {
    const int valid = n - 32 * kt;  // keys of the tile that exist (wave-uniform)
#pragma unroll
    for (int x = 0; x < QT_PER; ++x) {
      const int qt = qh * QT_PER + x;
      if (32 * qt >= total_rows) continue;  // wave-uniform
      f32x16 s_t = logits(k_op, qt);
      if (valid < 32) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (8 * (i / 4) + 4 * grp + (i % 4) >= valid) s_t[i] = -INFINITY;
      }
      float mx = s_t[0];
#pragma unroll
      for (int i = 1; i < 16; ++i) mx = fmaxf(mx, s_t[i]);
      const float m_new = fmaxf(m_run[x], mx * c2);  // -inf only while the lane has seen no key at all
      const float alpha = (m_new == m_run[x]) ? 1.f : __builtin_amdgcn_exp2f(m_run[x] - m_new);
      const float m_sub = m_new == -INFINITY ? 0.f : m_new;
      float psum = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) psum += __builtin_amdgcn_exp2f(fmaf(s_t[i], c2, -m_sub));
      l_run[x] = fmaf(l_run[x], alpha, psum);
      m_run[x] = m_new;
    }
  });
#pragma unroll
  for (int x = 0; x < QT_PER; ++x) {  // the two lane halves saw different keys of every tile
    const float m_o = __shfl_xor(m_run[x], 32, 64), l_o = __shfl_xor(l_run[x], 32, 64);
    const float mm = fmaxf(m_run[x], m_o);
    const float lt = l_run[x] * (m_run[x] == mm ? 1.f : __builtin_amdgcn_exp2f(m_run[x] - mm)) +
                     l_o * (m_o == mm ? 1.f : __builtin_amdgcn_exp2f(m_o - mm));
    if (grp == 0) stats_s[kw * QROWS + 32 * (qh * QT_PER + x) + col] = make_float2(mm, lt);
  }
  __syncthreads();
  if (tid < QROWS) {
    float v = INFINITY;  // padding rows contribute exp2(-inf) = 0
    if (tid < total_rows) {
      float mm = -INFINITY;
#pragma unroll
      for (int x = 0; x < KW; ++x) mm = fmaxf(mm, stats_s[x * QROWS + tid].x);
      float lsum = 0.f;
#pragma unroll
      for (int x = 0; x < KW; ++x) {
        const float2 ps = stats_s[x * QROWS + tid];
        lsum += ps.y * (ps.x == mm ? 1.f : exp2f(ps.x - mm));
      }
      v = mm + log2f(lsum);
    }
    lse_s[tid] = v;
  }
  __syncthreads();

  // ---- pass 2: column sums of exp2(s - normaliser) ----
  float lse2[QT_PER];
#pragma unroll
  for (int x = 0; x < QT_PER; ++x) lse2[x] = lse_s[32 * (qh * QT_PER + x) + col];
  for_my_tiles(std::false_type{}, [&](const bf16x8 (&k_op)[8], int kt) {
    float acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
    for (int x = 0; x < QT_PER; ++x) {
      const int qt = qh * QT_PER + x;
      if (32 * qt >= total_rows) continue;  // wave-uniform
      const f32x16 s_t = logits(k_op, qt);
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[i] += __builtin_amdgcn_exp2f(fmaf(s_t[i], c2, -lse2[x]));
    }
    const float tot = reduce16_over32(acc, col);  // value index col / 2 -> key 8 (i / 4) + 4 grp + (i % 4)
    const int i = col >> 1;
    if ((col & 1) == 0) part_s[qh * 32 * tiles + 32 * kt + 8 * (i / 4) + 4 * grp + (i % 4)] = tot;
  });
  __syncthreads();
  float* dst = score + (static_cast<int64_t>(bl) * dm.Hkv + g) * n;
  for (int j = tid; j < n; j += WAVES * 64) {
    float v = part_s[j];
#pragma unroll
    for (int x = 1; x < Q_SPLIT; ++x) v += part_s[x * 32 * tiles + j];
    dst[j] = v;
  }
}

constexpr size_t kFusedLdsBudget = 150 * 1024;  // of the CU's 160 KB
constexpr int kFusedKeyTilesInRegs = 5;           // 160 of a wave's 256 registers

template <int QT_TOTAL, int Q_SPLIT, int WAVES>
size_t instr_fused_lds_bytes(int n) {
  constexpr int QROWS = QT_TOTAL * 32;
  const int tiles = (n + 31) / 32;
  return static_cast<size_t>(QROWS) * kPitchK * 2 + static_cast<size_t>(WAVES / Q_SPLIT) * QROWS * 8 + QROWS * 4 +
         static_cast<size_t>(Q_SPLIT) * 32 * tiles * 4;
}

template <int QT_TOTAL, int Q_SPLIT, int WAVES, int KREG>
hipError_t instr_fused_launch(const Dims& dm, View q, int rows, Segments ks, float* score, hipStream_t st) {
  const size_t lds = instr_fused_lds_bytes<QT_TOTAL, Q_SPLIT, WAVES>(ks.n_c + ks.c);
  auto kern = instr_fused_kernel<QT_TOTAL, Q_SPLIT, WAVES, KREG>;
  static LdsLimit limit;
  const hipError_t e = raise_lds_limit(limit, reinterpret_cast<const void*>(kern), static_cast<int>(kFusedLdsBudget));
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(dm.B * dm.L * dm.Hkv), dim3(WAVES * 64), lds, st, dm, q, rows, ks, score);
  return hipGetLastError();
}


}  // namespace

bool mfma_path_supported(int dtype, const Dims& dm) { return dtype == CITRUS_BF16 && dm.D == D; }

static bool fits_i32(const View& v, int rows) {
  return v.ss > 0 && v.ss * static_cast<int64_t>(rows > 0 ? rows : 1) < (int64_t{1} << 31);
}

bool attn_mfma_emits_cache_lse(const Segments& ks, int causal, View out) {
  return out.ptr != nullptr && causal != 0 && ks.n_c > 0 && ks.n_c % 32 == 0;
}

hipError_t launch_attn_mfma(const Dims& dm, View q, int rows, Segments ks, Segments vs, int causal, View out,
                            float* lse, float* lse_cache, int key_splits, float2* part, hipStream_t st,
                            int q_rope_pos0, float rope_base) {
  if (lse_cache != nullptr && !attn_mfma_emits_cache_lse(ks, causal, out)) return hipErrorInvalidValue;
  if (q_rope_pos0 >= 0 && out.ptr == nullptr) return hipErrorInvalidValue;  // only the kernel with output rotates
  if (!fits_i32(ks.cache, ks.n_c) || !fits_i32(ks.chunk, ks.c) || !fits_i32(vs.cache, vs.n_c) ||
      !fits_i32(vs.chunk, vs.c))
    return hipErrorInvalidValue;
  if (key_splits < 1 || (key_splits > 1 && (out.ptr != nullptr || part == nullptr))) return hipErrorInvalidValue;
  constexpr int kPipeWaves = 8;
  const bool pipe = out.ptr != nullptr;
  const TaskShape ts = task_shape(dm.G, pipe ? kPipeWaves : kWaves);
  const int rows_per_block = ts.tiles_per_block * kRowsPerWave;
  const int row_blocks = (rows + rows_per_block - 1) / rows_per_block;
  const int rb_slots = (causal && key_splits == 1) ? (row_blocks + 1) / 2 : row_blocks;  // paired row blocks
  dim3 grid(rb_slots * (dm.G / ts.heads_per_block) * dm.Hkv * dm.B * dm.L * key_splits);
  constexpr int kQStageBytes = kPipeWaves * 32 * kRowBytes;  // dynamic LDS next to the 64 KB of static tiles
  if (pipe) {
    static LdsLimit limit, limit_rotq;
    hipError_t e = raise_lds_limit(limit, reinterpret_cast<const void*>(attn_pipe_kernel_w8), kQStageBytes);
    if (e == hipSuccess) e = raise_lds_limit(limit_rotq, reinterpret_cast<const void*>(attn_pipe_kernel_w8_rotq), kQStageBytes);
    if (e != hipSuccess) return e;
  }
  if (pipe && q_rope_pos0 >= 0)
    hipLaunchKernelGGL(attn_pipe_kernel_w8_rotq, grid, dim3(kPipeWaves * 64), kQStageBytes, st, dm, q, rows, ks, vs, causal, out, lse,
                       lse_cache, q_rope_pos0, log2f(rope_base));
  else if (pipe)
    hipLaunchKernelGGL(attn_pipe_kernel_w8, grid, dim3(kPipeWaves * 64), kQStageBytes, st, dm, q, rows, ks, vs, causal, out, lse,
                       lse_cache);
  else
    hipLaunchKernelGGL(lse_mfma_kernel, grid, dim3(kThreads), 0, st, dm, q, rows, ks, causal, lse, key_splits, part);
  return hipGetLastError();
}

hipError_t launch_colsum_mfma(const Dims& dm, View q, int rows, Segments ks, int causal, const float* lse,
                              int key_splits, const float2* part, float* score, hipStream_t st) {
  const int n = ks.n_c + ks.c;
  constexpr int kKeysPerBlock = 32 * kColsumKeyTiles * kColsumWaves;
  dim3 grid((n + kKeysPerBlock - 1) / kKeysPerBlock, dm.Hkv, dm.B * dm.L);
  constexpr int kLdsBytes = 2 * kColsumQRows * (kPitchK * 2 + 4);  // two buffers of rows and normalisers: 70 KB
  static LdsLimit limit_stepwise, limit_any;
  const bool stepwise = rows % kColsumQRows == 0;
  const auto kern = stepwise ? colsum_mfma_kernel<true> : colsum_mfma_kernel<false>;
  const hipError_t e = raise_lds_limit(stepwise ? limit_stepwise : limit_any, reinterpret_cast<const void*>(kern), kLdsBytes);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, grid, dim3(kColsumWaves * 64), kLdsBytes, st, dm, q, rows, ks, causal, lse, key_splits, part,
                     score);
  return hipGetLastError();
}

// Instruction score in two launches: partial log-sum-exp over ranges of key tiles (enough
// workgroups to fill the chip although there are few instruction rows), then the column sums.
size_t instr_score_mfma_workspace_floats(const Dims& dm, int rows, int n) {
  const size_t two_launch = static_cast<size_t>(2) * kMaxKeySplits * dm.B * dm.L * dm.Hq * rows;
  const size_t strips = instr_strip_workspace_floats(dm, rows, n);
  return two_launch > strips ? two_launch : strips;
}

hipError_t launch_instr_score_mfma(const Dims& dm, View q, int rows, Segments ks, float* workspace,
                                   size_t workspace_floats, float* score, hipStream_t st) {
  const int n = ks.n_c + ks.c;
  // a short text over a candidate set that a workgroup's registers can hold one row strip of: one product
  // per (row, key)
  if (instr_strip_supported(dm, q, rows, ks, workspace_floats))
    return launch_instr_strip(dm, q, rows, ks, workspace, workspace_floats, score, st);
  // otherwise two passes over the keys; few query rows per KV group: one fused launch
  const int total_rows = dm.G * rows;
  const int tiles32 = (n + 31) / 32;
  if (total_rows <= 128 && instr_fused_lds_bytes<4, 1, 8>(n) <= kFusedLdsBudget)
    return instr_fused_launch<4, 1, 8, 0>(dm, q, rows, ks, score, st);
  if (total_rows <= 256 && tiles32 <= 8 * kFusedKeyTilesInRegs && instr_fused_lds_bytes<8, 1, 8>(n) <= kFusedLdsBudget)
    return instr_fused_launch<8, 1, 8, kFusedKeyTilesInRegs>(dm, q, rows, ks, score, st);
  if (total_rows <= 256 && instr_fused_lds_bytes<8, 2, 16>(n) <= kFusedLdsBudget)
    return instr_fused_launch<8, 2, 16, 0>(dm, q, rows, ks, score, st);
  const int tiles = (n + kTileN - 1) / kTileN;
  int splits = (tiles + 3) / 4;  // about four key tiles per workgroup
  splits = splits < 1 ? 1 : (splits > kMaxKeySplits ? kMaxKeySplits : splits);
  const int64_t rows_total = static_cast<int64_t>(dm.B) * dm.L * dm.Hq * rows;
  if (static_cast<size_t>(2) * splits * rows_total > workspace_floats) return hipErrorInvalidValue;
  float2* part = reinterpret_cast<float2*>(workspace);
  View none{nullptr, 0, 0, 0, 0};
  hipError_t e = launch_attn_mfma(dm, q, rows, ks, ks, /*causal=*/0, none, nullptr, nullptr, splits, part, st);
  if (e != hipSuccess) return e;
  if (splits > 1) {  // one normaliser per row, in place of the first range's pairs
    hipLaunchKernelGGL(merge_partials_kernel, dim3(static_cast<unsigned>((rows_total + 255) / 256)), dim3(256), 0, st, part,
                       splits, rows_total);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return launch_colsum_mfma(dm, q, rows, ks, /*causal=*/0, nullptr, 1, part, score, st);
}

}  // namespace citrus
