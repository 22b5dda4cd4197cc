// One decoding step over the retained cache (Section 4.3: the k states kept by the last eviction,
// followed by the instruction and the tokens generated so far), bf16, head_dim 128, gfx950.
//
// A single query per head reads every key and value once: the step is bound by HBM, not by
// arithmetic.  The kernel is therefore organised around the stream of K/V bytes:
//   * a workgroup owns one (document, layer, KV head) and one contiguous range of keys; the query
//     heads of the GQA group share every K/V byte that is fetched;
//   * each of its four waves streams its own 32-key tiles from global memory straight into a
//     private, double-buffered LDS region (buffer_load ... lds) and waits on its own vector-memory
//     counter only: there is no barrier in the key loop;
//   * the arithmetic runs on the matrix pipe although only G of its 32 query columns carry data:
//     S^T = K.Q^T and O^T = V^T.P^T on v_mfma_f32_32x32x16_bf16 take 16 MFMAs per 16 KB tile,
//     about a tenth of the time the tile needs to arrive, and the operand layouts are the ones the
//     chunk-attention kernels use (one query per lane, transpose reads for V^T);
//   * the waves' partial (maximum, sum, output) triples are merged through LDS at the end; with
//     more than one key range per unit a small second kernel merges the ranges.
#include "citrus_internal.h"

namespace citrus {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) short i16x4;

constexpr int D = 128;
constexpr int kTileKeys = 32;             // keys per wave tile = rows of one MFMA
constexpr int kRowBytes = 2 * D;          // unpadded, XOR-swizzled rows
constexpr int kTileBytes = kTileKeys * kRowBytes;          // 8 KB of K, the same of V
constexpr int kWaveLdsBytes = 4 * kTileBytes;              // {K, V} x two buffers
constexpr int kBufferFlags = 0x00020000;  // raw buffer resource word 3 on CDNA: 32-bit data format, no swizzle
constexpr int kLoadsPerTile = 2 * kTileKeys / 4;           // 16 instructions of 1 KB
constexpr int kMaxSplits = 8;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kMaxSlack = 8.0f;

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

typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(2))) int i32x2;

// LDS reads of a tile, written as asm: the compiler drains the vector-memory counter in front of every
// LDS read it can see while LDS-direct loads are in flight (it cannot tell that they fill the OTHER
// buffer), which would make each wave wait for the tile it has just requested.  Each block waits for
// its own reads, so nothing the compiler does not know about is left pending.
// The eight 16-byte A operands (32 keys x 16 head_dim values each) of S^T = K.Q^T:
__device__ inline void lds_read_k_operands(Pack8 (&a)[8], const uint32_t (&addr)[8]) {
  i32x4 r0, r1, r2, r3, r4, r5, r6, r7;
  asm volatile(
      "ds_read_b128 %0, %8\n\t"
      "ds_read_b128 %1, %9\n\t"
      "ds_read_b128 %2, %10\n\t"
      "ds_read_b128 %3, %11\n\t"
      "ds_read_b128 %4, %12\n\t"
      "ds_read_b128 %5, %13\n\t"
      "ds_read_b128 %6, %14\n\t"
      "ds_read_b128 %7, %15\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(r0), "=&v"(r1), "=&v"(r2), "=&v"(r3), "=&v"(r4), "=&v"(r5), "=&v"(r6), "=&v"(r7)
      : "v"(addr[0]), "v"(addr[1]), "v"(addr[2]), "v"(addr[3]), "v"(addr[4]), "v"(addr[5]), "v"(addr[6]), "v"(addr[7])
      : "memory");
  a[0].v = __builtin_bit_cast(bf16x8, r0); a[1].v = __builtin_bit_cast(bf16x8, r1);
  a[2].v = __builtin_bit_cast(bf16x8, r2); a[3].v = __builtin_bit_cast(bf16x8, r3);
  a[4].v = __builtin_bit_cast(bf16x8, r4); a[5].v = __builtin_bit_cast(bf16x8, r5);
  a[6].v = __builtin_bit_cast(bf16x8, r6); a[7].v = __builtin_bit_cast(bf16x8, r7);
}
// The four A operands of one 16-key contraction step of O^T = V^T.P^T through transpose reads
// (ds_read_b64_tr_b16; lane mapping as in the chunk-attention kernels): operand r = head_dim tile r,
// read rd = keys 8 rd .. +7 of the step, which lie 8 rows = 2048 bytes further on.
__device__ inline void lds_read_v_operands(Pack8 (&a)[4], const uint32_t (&addr)[8]) {
  i32x2 r0, r1, r2, r3, r4, r5, r6, r7;
  asm volatile(
      "ds_read_b64_tr_b16 %0, %8\n\t"
      "ds_read_b64_tr_b16 %1, %9 offset:2048\n\t"
      "ds_read_b64_tr_b16 %2, %10\n\t"
      "ds_read_b64_tr_b16 %3, %11 offset:2048\n\t"
      "ds_read_b64_tr_b16 %4, %12\n\t"
      "ds_read_b64_tr_b16 %5, %13 offset:2048\n\t"
      "ds_read_b64_tr_b16 %6, %14\n\t"
      "ds_read_b64_tr_b16 %7, %15 offset:2048\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(r0), "=&v"(r1), "=&v"(r2), "=&v"(r3), "=&v"(r4), "=&v"(r5), "=&v"(r6), "=&v"(r7)
      : "v"(addr[0]), "v"(addr[1]), "v"(addr[2]), "v"(addr[3]), "v"(addr[4]), "v"(addr[5]), "v"(addr[6]), "v"(addr[7])
      : "memory");
  a[0].h[0] = __builtin_bit_cast(i16x4, r0); a[0].h[1] = __builtin_bit_cast(i16x4, r1);
  a[1].h[0] = __builtin_bit_cast(i16x4, r2); a[1].h[1] = __builtin_bit_cast(i16x4, r3);
  a[2].h[0] = __builtin_bit_cast(i16x4, r4); a[2].h[1] = __builtin_bit_cast(i16x4, r5);
  a[3].h[0] = __builtin_bit_cast(i16x4, r6); a[3].h[1] = __builtin_bit_cast(i16x4, r7);
}

// The tile whose loads were issued before the newest kLoadsPerTile ones has landed in LDS.  LDS-direct
// loads complete in order and are counted by the issuing wave's vector-memory counter.  The waits are
// the compiler's own builtin, so that its counter bookkeeping knows about them (a wait hidden in an asm
// statement leaves it believing that the query loads are still pending, and it then drains the counter
// in front of the first LDS read of every iteration, prefetched tile included); the empty asm with a
// memory clobber keeps the LDS reads of the tile behind the wait.
// s_waitcnt immediate on gfx9: vmcnt[3:0] = bits 3:0, expcnt = bits 6:4, lgkmcnt = bits 11:8, vmcnt[5:4] = bits 15:14.
__device__ inline void wait_all_but_newest_tile() {
  __builtin_amdgcn_s_waitcnt(0x4F70);  // vmcnt(16), nothing else
  asm volatile("" ::: "memory");
}
__device__ inline void wait_all_loads() {
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0), nothing else
  asm volatile("" ::: "memory");
}
// keeps two predicated regions from being merged into one with per-lane operands
__device__ inline void keep_apart() { asm volatile("" ::: "memory"); }
static_assert(kLoadsPerTile == 16, "the wait above counts one tile's load instructions");

// Partial results per (key range, document, layer, query head): {m, l} in the log2 domain and the
// unnormalised output row.
struct Partials {
  float2* ml;  // [splits][B*L*Hq]
  float* o;    // [splits][B*L*Hq][D]
};

template <int WAVES>
__device__ __forceinline__ void decode_attn_body(const Dims& dm, const View& q, const Segments& ks, const Segments& vs,
                                                 const View& out, int key_splits, const Partials& part,
                                                 int append_token) {
  constexpr int kWaves = WAVES;
  constexpr int kThreads = kWaves * 64;
  extern __shared__ __attribute__((aligned(1024))) char lds[];

  const int tid = threadIdx.x, lane = tid % 64;
  const int wu = __builtin_amdgcn_readfirstlane(tid / 64);
  const int col = lane % 32, grp = lane / 32;
  const int sp = blockIdx.x % key_splits;
  const int unit = blockIdx.x / key_splits;  // (b, l, g)
  const int g = unit % dm.Hkv;
  const int bl = unit / dm.Hkv;
  const int b = bl / dm.L, l = bl % dm.L;
  const int n_c = ks.n_c;
  const int n = n_c + ks.c;

  // key tiles of this workgroup's range, dealt round-robin to its waves
  const int all_tiles = (n + kTileKeys - 1) / kTileKeys;
  const int tiles_per_split = (all_tiles + key_splits - 1) / key_splits;
  const int t_begin = sp * tiles_per_split;
  const int t_end = min(all_tiles, t_begin + tiles_per_split);

  // ---- global -> LDS staging of one 32-key tile by ONE wave: 8 instructions of 4 rows each ----
  // The 16-byte segment `seg` of tile row `row` lives at position seg ^ f(row),
  // f(row) = 2 (row % 8) ^ ((row / 8) % 2): both read patterns below are free of bank conflicts.
  const int k_ss_cache = static_cast<int>(ks.cache.ss), k_ss_chunk = static_cast<int>(ks.chunk.ss);
  const int v_ss_cache = static_cast<int>(vs.cache.ss), v_ss_chunk = static_cast<int>(vs.chunk.ss);
  auto seg_bytes = [](int rows_, int ss_) { return rows_ > 0 ? ((rows_ - 1) * ss_ + D) * 2 : 0; };
  const __amdgpu_buffer_rsrc_t k_rs_cache = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(unit_ptr(ks.cache, b, l, g)), 0, seg_bytes(n_c, k_ss_cache), kBufferFlags);
  const __amdgpu_buffer_rsrc_t k_rs_chunk = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(unit_ptr(ks.chunk, b, l, g)), 0, seg_bytes(ks.c, k_ss_chunk), kBufferFlags);
  const __amdgpu_buffer_rsrc_t v_rs_cache = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(unit_ptr(vs.cache, b, l, g)), 0, seg_bytes(n_c, v_ss_cache), kBufferFlags);
  const __amdgpu_buffer_rsrc_t v_rs_chunk = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(unit_ptr(vs.chunk, b, l, g)), 0, seg_bytes(ks.c, v_ss_chunk), kBufferFlags);
  typedef __attribute__((address_space(3))) void* lds_void_ptr;
  char* const wave_lds = lds + wu * kWaveLdsBytes;  // [buffer][K | V][tile]
  typedef __attribute__((address_space(3))) char* lds_char_ptr;
  const uint32_t wave_lds_addr = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_char_ptr)wave_lds));
  const int fill_row = lane / 16;                   // row inside the 4-row group of one instruction
  const int fill_pos = lane % 16;                   // 16-byte position inside the LDS row
  auto fill_tile = [&](int tile, int buf) {
    const int j0 = tile * kTileKeys;
    char* k_t = wave_lds + buf * 2 * kTileBytes;
    char* v_t = k_t + kTileBytes;
    const bool in_cache = j0 + kTileKeys <= n_c;  // wave-uniform: every row of the tile is a cache row
#pragma unroll
    for (int i = 0; i < kTileKeys / 4; ++i) {
      const int row = 4 * i + fill_row;
      const int f = (2 * (row % 8)) ^ ((row / 8) % 2);
      const int seg = (fill_pos ^ f) * 16;
      lds_void_ptr kd = (lds_void_ptr)(k_t + 4 * i * kRowBytes);
      lds_void_ptr vd = (lds_void_ptr)(v_t + 4 * i * kRowBytes);
      if (in_cache) {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(k_rs_cache, kd, 16, (j0 + row) * k_ss_cache * 2 + seg, 0, 0, 0);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(v_rs_cache, vd, 16, (j0 + row) * v_ss_cache * 2 + seg, 0, 0, 0);
      } else {
        // The tile holds the end of the cache, the new token's row, or rows past the end (they re-read
        // the last row: finite values, masked in the logits).  Two separately predicated loads, each
        // with ONE buffer resource: a resource chosen per lane would be loaded in a serialising loop.
        const int j = min(j0 + row, n - 1);
        if (j < n_c) {
          __builtin_amdgcn_raw_ptr_buffer_load_lds(k_rs_cache, kd, 16, j * k_ss_cache * 2 + seg, 0, 0, 0);
          __builtin_amdgcn_raw_ptr_buffer_load_lds(v_rs_cache, vd, 16, j * v_ss_cache * 2 + seg, 0, 0, 0);
        }
        keep_apart();
        if (j >= n_c) {
          __builtin_amdgcn_raw_ptr_buffer_load_lds(k_rs_chunk, kd, 16, (j - n_c) * k_ss_chunk * 2 + seg, 0, 0, 0);
          __builtin_amdgcn_raw_ptr_buffer_load_lds(v_rs_chunk, vd, 16, (j - n_c) * v_ss_chunk * 2 + seg, 0, 0, 0);
        }
        keep_apart();
      }
    }
  };

  // per-lane LDS read offsets inside a tile, swizzle included (same scheme as the chunk-attention kernels)
  const int f_col = (2 * (col & 7)) ^ ((col >> 3) & 1);
  int k_off[8];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) k_off[kk] = col * kRowBytes + (((2 * kk + grp) ^ f_col) * 16);
  const int s16 = lane % 16, q16 = lane / 16;
  const int v_cl = (8 * (q16 % 2) + (s16 % 4) / 2) ^ (8 * (q16 / 2) + 2 * (s16 / 4));
  int v_off[8];
#pragma unroll
  for (int e = 0; e < 8; ++e)
    v_off[e] = (4 * (q16 / 2) + s16 / 4) * kRowBytes + ((e ^ v_cl) * 16) + 8 * (s16 % 2);

  // ---- Q^T operand: column `col` is query head g*G + col (columns >= G repeat the last head; unused) ----
  const int h_lane = g * dm.G + min(col, dm.G - 1);
  bf16x8 q_op[8];
  {
    const uint16_t* qp = unit_ptr(q, b, l, h_lane) + 8 * grp;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      Pack8 p;
      p.u = *reinterpret_cast<const uint4*>(qp + 16 * kk);
      q_op[kk] = p.v;
    }
  }

  // The token's own state becomes row n_c of the cache.  Candidates j >= n_c are always read from the
  // token's tensors, never from the cache, so no workgroup reads the row that is written here.
  if (append_token && sp == key_splits - 1 && wu == kWaves - 1 && lane < 32) {
    const int part16 = lane % 16;  // 16 x 16 bytes per row; lanes 0..15 copy K, lanes 16..31 copy V
    const bool is_v = lane >= 16;
    const uint16_t* src = is_v ? unit_ptr(vs.chunk, b, l, g) : unit_ptr(ks.chunk, b, l, g);
    const View& cv = is_v ? vs.cache : ks.cache;
    uint16_t* dst = const_cast<uint16_t*>(unit_ptr(cv, b, l, g)) + static_cast<int64_t>(n_c) * cv.ss;
    *reinterpret_cast<uint4*>(dst + 8 * part16) = *reinterpret_cast<const uint4*>(src + 8 * part16);
  }
  wait_all_loads();  // the query operand has landed before the first tile is requested

  const float c2 = dm.scale * kLog2e;  // logits in the log2 domain
  float m_run = -INFINITY, l_run = 0.f;
  f32x16 o_acc[4];
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int i = 0; i < 16; ++i) o_acc[r][i] = 0.f;

  int tile = t_begin + wu;
  if (tile < t_end) fill_tile(tile, 0);
  for (int it = 0; tile < t_end; tile += kWaves, ++it) {
    const int buf = it & 1;
    // the other buffer was last read in the previous iteration, whose reads have all returned
    if (tile + kWaves < t_end) {
      fill_tile(tile + kWaves, buf ^ 1);
      wait_all_but_newest_tile();
    } else {
      wait_all_loads();
    }
    const uint32_t k_t = wave_lds_addr + buf * 2 * kTileBytes;  // LDS byte addresses
    const uint32_t v_t = k_t + kTileBytes;
    const int j0 = tile * kTileKeys;

    // S^T = K . Q^T for 32 keys x 32 query columns
    f32x16 s_acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) s_acc[i] = 0.f;
    Pack8 a[8];
    {
      uint32_t addr[8];
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) addr[kk] = k_t + k_off[kk];
      lds_read_k_operands(a, addr);
    }
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) s_acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk].v, q_op[kk], s_acc, 0, 0, 0);

    if (j0 + kTileKeys > n) {  // wave-uniform: the last tile
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int j = j0 + 8 * (i / 4) + 4 * grp + (i % 4);
        if (j >= n) s_acc[i] = -INFINITY;
      }
    }
    // running maximum, updated only when some column moved by more than kMaxSlack (log2 units)
    float mx = s_acc[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) mx = fmaxf(mx, s_acc[i]);
    if (__any(mx * c2 > m_run + kMaxSlack)) {
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m_run, mx * c2);  // finite: every tile holds at least one real key
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);  // 0 on the first tile
      l_run *= alpha;
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int i = 0; i < 16; ++i) o_acc[r][i] *= alpha;
      m_run = m_new;
    }
    uint32_t p_pk[8];
    float psum = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float p0 = __builtin_amdgcn_exp2f(fmaf(s_acc[2 * i], c2, -m_run));
      const float p1 = __builtin_amdgcn_exp2f(fmaf(s_acc[2 * i + 1], c2, -m_run));
      p_pk[i] = pack_bf16x2(p0, p1);
      // the row sum is taken over the bf16-rounded probabilities, the values P.V uses
      psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, p_pk[i]),
                                             __builtin_bit_cast(bf16x2, 0x3f803f80u), psum, false);
    }
    l_run += psum;

    // O^T += V^T . P^T, two contraction steps of 16 keys
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      Pack8 av[4];
      {
        uint32_t addr[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) addr[e] = v_t + 16 * half * kRowBytes + v_off[e];
        lds_read_v_operands(av, addr);
      }
      Pack8 pb;
#pragma unroll
      for (int x = 0; x < 4; ++x) pb.w[x] = p_pk[4 * half + x];
#pragma unroll
      for (int r = 0; r < 4; ++r) o_acc[r] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[r].v, pb.v, o_acc[r], 0, 0, 0);
    }
  }

  // ---- merge the four waves through LDS (the tile buffers are free once every wave is here) ----
  const float l_wave = l_run + __shfl_xor(l_run, 32, 64);
  __syncthreads();
  float* o_s = reinterpret_cast<float*>(lds);                   // [wave][32 columns][D]
  float2* ml_s = reinterpret_cast<float2*>(lds + kWaves * 32 * D * 4);  // [wave][32]
  if (col < dm.G) {
    if (grp == 0) ml_s[wu * 32 + col] = make_float2(m_run, l_wave);
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        // registers 4 i4 .. +3 are rows c' = 8 i4 + 4 grp + 0..3 -> head_dim 16 r + (c' % 16) + 64 (c' / 16)
        const int c0 = 8 * i4 + 4 * grp;
        const int d0 = 16 * r + (c0 % 16) + 64 * (c0 / 16);
        *reinterpret_cast<float4*>(o_s + (wu * 32 + col) * D + d0) =
            make_float4(o_acc[r][4 * i4], o_acc[r][4 * i4 + 1], o_acc[r][4 * i4 + 2], o_acc[r][4 * i4 + 3]);
      }
  }
  __syncthreads();
  for (int e = tid; e < dm.G * D; e += kThreads) {
    const int hq = e / D, d = e % D;
    float m_all = -INFINITY;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) m_all = fmaxf(m_all, ml_s[w * 32 + hq].x);
    float l_all = 0.f, o_all = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float2 ml = ml_s[w * 32 + hq];
      const float wgt = ml.x == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ml.x - m_all);  // a wave without tiles
      l_all = fmaf(ml.y, wgt, l_all);
      o_all = fmaf(o_s[(w * 32 + hq) * D + d], wgt, o_all);
    }
    const int h = g * dm.G + hq;
    if (key_splits == 1) {
      uint16_t* op = const_cast<uint16_t*>(unit_ptr(out, b, l, h));
      const uint32_t pk = pack_bf16x2(o_all / l_all, 0.f);
      op[d] = static_cast<uint16_t>(pk & 0xffffu);
    } else {
      const int64_t row = static_cast<int64_t>(sp) * dm.B * dm.L * dm.Hq + static_cast<int64_t>(bl) * dm.Hq + h;
      part.o[row * D + d] = o_all;
      if (d == 0) part.ml[row] = make_float2(m_all, l_all);
    }
  }
}

// Four waves per workgroup and 32 KB of LDS per wave: one workgroup per compute unit.  Narrower
// workgroups (one or two waves, 5 or 2 of them per compute unit) were measured 2 to 7 % slower at every
// shape tried, so this is the only instance.
constexpr int kWaves = 4;
__global__ __launch_bounds__(64 * kWaves) void decode_attn_kernel(Dims dm, View q, Segments ks, Segments vs, View out,
                                                                 int key_splits, Partials part, int append_token) {
  decode_attn_body<kWaves>(dm, q, ks, vs, out, key_splits, part, append_token);
}

// Merge of the key ranges: one thread per (document, layer, query head, head_dim element).
__global__ __launch_bounds__(256) void decode_merge_kernel(Dims dm, View out, int key_splits, Partials part) {
  const int64_t rows = static_cast<int64_t>(dm.B) * dm.L * dm.Hq;
  const int64_t e = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (e >= rows * D) return;
  const int64_t row = e / D;
  const int d = static_cast<int>(e % D);
  float m_all = -INFINITY;
  for (int s = 0; s < key_splits; ++s) m_all = fmaxf(m_all, part.ml[s * rows + row].x);
  float l_all = 0.f, o_all = 0.f;
  for (int s = 0; s < key_splits; ++s) {
    const float2 ml = part.ml[s * rows + row];
    const float wgt = ml.x == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ml.x - m_all);
    l_all = fmaf(ml.y, wgt, l_all);
    o_all = fmaf(part.o[(s * rows + row) * D + d], wgt, o_all);
  }
  const int h = static_cast<int>(row % dm.Hq);
  const int bl = static_cast<int>(row / dm.Hq);
  uint16_t* op = const_cast<uint16_t*>(unit_ptr(out, bl / dm.L, bl % dm.L, h));
  op[d] = static_cast<uint16_t>(pack_bf16x2(o_all / l_all, 0.f) & 0xffffu);
}

// Key ranges per unit.  A unit's keys are split over several workgroups only when there are fewer units
// than compute units (a second launch merges the ranges; measured slower whenever one workgroup per
// unit already fills the chip), and only while every wave keeps at least two tiles.
int choose_splits(int units, int n) {
  const int tiles = (n + kTileKeys - 1) / kTileKeys;
  int splits = 1;
  while (splits < kMaxSplits && units * splits < 256 && tiles / (2 * splits) >= 2 * kWaves) splits *= 2;
  const int per = (tiles + splits - 1) / splits;
  return (tiles + per - 1) / per;  // no empty key range
}

}  // namespace

bool decode_mfma_supported(int dtype, const Dims& dm) { return dtype == CITRUS_BF16 && dm.D == D && dm.G <= 32; }

size_t decode_mfma_workspace_floats(const Dims& dm) {
  return static_cast<size_t>(kMaxSplits) * dm.B * dm.L * dm.Hq * (D + 2);
}

hipError_t launch_decode_mfma(const Dims& dm, View q, Segments ks, Segments vs, View out, float* workspace,
                              int append_token, hipStream_t st) {
  if (ks.c != 1) return hipErrorInvalidValue;  // one new token
  const int units = dm.B * dm.L * dm.Hkv;
  const int n = ks.n_c + ks.c;
  const int splits = choose_splits(units, n);
  const int64_t rows = static_cast<int64_t>(dm.B) * dm.L * dm.Hq;
  Partials part;
  part.ml = reinterpret_cast<float2*>(workspace);
  part.o = workspace + 2 * static_cast<size_t>(kMaxSplits) * rows;
  constexpr int kLdsBytes = kWaves * kWaveLdsBytes;  // 128 KB
  static LdsLimit limit;
  hipError_t e = raise_lds_limit(limit, reinterpret_cast<const void*>(decode_attn_kernel), kLdsBytes);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(decode_attn_kernel, dim3(units * splits), dim3(64 * kWaves), kLdsBytes, st, dm, q, ks, vs, out,
                     splits, part, append_token);
  e = hipGetLastError();
  if (e != hipSuccess || splits == 1) return e;
  const int64_t elems = rows * D;
  hipLaunchKernelGGL(decode_merge_kernel, dim3(static_cast<unsigned>((elems + 255) / 256)), dim3(256), 0, st, dm, out,
                     splits, part);
  return hipGetLastError();
}

}  // namespace citrus
