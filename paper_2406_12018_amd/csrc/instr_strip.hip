// Instruction score (Eq. (1) with the instruction as the text, Section 4.2; summed form) with ONE product
// q.k per (instruction row, candidate key), bf16, head_dim 128, gfx950.
//
// The score of a key is a sum over instruction rows of softmax weights, and every row has its own
// normaliser, which is known only after the row has seen all keys.  Instead of a second pass over the
// keys, a workgroup keeps the un-normalised weights of a STRIP of instruction rows on chip:
//   * a workgroup owns one (document, layer, KV head) and one strip of 64 (or 32) of the group's
//     instruction rows (heads x rows, flattened); its eight waves split the candidate keys, each wave
//     streaming its own 32-key tiles from global memory straight into a private double-buffered LDS
//     region (buffer_load ... lds) and waiting on its own vector-memory counter: no barrier in the key loop;
//   * S^T = K.Q^T on v_mfma_f32_32x32x16_bf16 puts one instruction row per lane; the lane keeps a lazy
//     reference (within 2^8 of its running maximum), turns the logits into weights exp2(s - reference)
//     right away, rounds them to bf16 and keeps them in registers (a strip of 64 rows x 1280 keys is 80
//     registers per lane over the 512 lanes), together with the reference each key tile was taken against;
//   * the rows' sums over a tile come from the matrix pipe too (a product of the rounded weights with a
//     matrix of ones), so the vector pipe is left with the maximum, one multiply-add, the exponential and
//     the rounding per weight;
//   * when the keys are through, the waves' (reference, sum) pairs meet in LDS and give each row's
//     normaliser; the column sums  sum_rows weight[row][key] * 2^(reference - row maximum) / row sum  are
//     a product that contracts over the rows: every stored tile goes through the wave's LDS region once
//     (written row-major, read back with transpose reads as the A operand) and meets a B operand that holds
//     the rows' factors, split into two bf16 parts (16 significant bits) in two columns;
//   * each strip writes its two partial columns; a second, tiny kernel adds the partial sums of a KV head
//     in a fixed order.  No atomics: bit-reproducible.
// Against two passes over the keys this halves the matrix and the exponential work, the strips of a KV head
// run at the same time on one XCD, so that its keys come from HBM once, and a KV head is spread over several
// compute units.  What it pays for that is a fixed cost per workgroup (first tile and instruction rows,
// normaliser exchange, the transposed product) of about two thirds of its run time at 1280 keys, and keys
// that cross the L2 -> compute unit path once per strip.  Measured at 32/8 heads, 64 instruction rows, 1280
// keys: 19.5 us against 39 us for the two-pass kernel with up to 64 (document, layer, KV head) units in a
// launch (one workgroup per compute unit), 36 against 42 us with 128 units, 68 against 52 us with 256: the
// launcher takes this kernel while its workgroups fit the chip twice, i.e. for the small launches that a
// model whose layers run one after the other makes, and the two-pass kernels for the large batched ones.
#include "citrus_internal.h"

namespace citrus {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) int i32x4;

constexpr int D = 128;
constexpr int kTileKeys = 32;
constexpr int kRowBytes = 2 * D;
constexpr int kTileBytes = kTileKeys * kRowBytes;  // 8 KB
constexpr int kWaves = 8;
constexpr int kThreads = kWaves * 64;
constexpr int kXcds = 8;
constexpr int kLoadsPerTile = kTileKeys / 4;  // 8 instructions of 1 KB
constexpr int kBufferFlags = 0x00020000;      // raw buffer resource word 3 on CDNA: 32-bit data format, no swizzle
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kMaxSlack = 8.0f;  // weights stay below 2^8

union Pack8 {
  bf16x8 v;
  uint4 u;
};

__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
  f32x2 f = {lo, hi};
  bf16x2 b = __builtin_convertvector(f, bf16x2);  // round to nearest even
  return __builtin_bit_cast(uint32_t, b);
}
__device__ inline float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ inline float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ inline const uint16_t* unit_ptr(const View& v, int b, int l, int h) {
  return static_cast<const uint16_t*>(v.ptr) + (b * v.sb + l * v.sl + h * v.sh);
}

// The eight 16-byte A operands of a key tile, read from the wave's own LDS region.  Written as asm: while
// LDS-direct loads are in flight the compiler drains the vector-memory counter in front of every LDS read
// it can see (it cannot tell that they fill the OTHER buffer).  The block waits for its own reads.
template <int OFFSET>
__device__ inline void lds_read_k_operands(bf16x8 (&a)[8], const uint32_t (&addr)[8]) {
  i32x4 r0, r1, r2, r3, r4, r5, r6, r7;
  asm volatile(
      "ds_read_b128 %0, %8 offset:%16\n\t"
      "ds_read_b128 %1, %9 offset:%16\n\t"
      "ds_read_b128 %2, %10 offset:%16\n\t"
      "ds_read_b128 %3, %11 offset:%16\n\t"
      "ds_read_b128 %4, %12 offset:%16\n\t"
      "ds_read_b128 %5, %13 offset:%16\n\t"
      "ds_read_b128 %6, %14 offset:%16\n\t"
      "ds_read_b128 %7, %15 offset:%16\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(r0), "=&v"(r1), "=&v"(r2), "=&v"(r3), "=&v"(r4), "=&v"(r5), "=&v"(r6), "=&v"(r7)
      : "v"(addr[0]), "v"(addr[1]), "v"(addr[2]), "v"(addr[3]), "v"(addr[4]), "v"(addr[5]), "v"(addr[6]), "v"(addr[7]),
        "n"(OFFSET)
      : "memory");
  a[0] = __builtin_bit_cast(bf16x8, r0); a[1] = __builtin_bit_cast(bf16x8, r1);
  a[2] = __builtin_bit_cast(bf16x8, r2); a[3] = __builtin_bit_cast(bf16x8, r3);
  a[4] = __builtin_bit_cast(bf16x8, r4); a[5] = __builtin_bit_cast(bf16x8, r5);
  a[6] = __builtin_bit_cast(bf16x8, r6); a[7] = __builtin_bit_cast(bf16x8, r7);
}

// LDS-direct loads complete in order and are counted by the issuing wave's vector-memory counter.  The
// waits are the compiler's own builtin so that its counter bookkeeping knows about them; the empty asm
// with a memory clobber keeps the LDS reads of the tile behind the wait.
// s_waitcnt immediate on gfx9: vmcnt[3:0] = bits 3:0, expcnt = bits 6:4, lgkmcnt = bits 11:8, vmcnt[5:4] = bits 15:14.
__device__ inline void wait_all_but_newest_tile() {
  __builtin_amdgcn_s_waitcnt(0x0F78);  // vmcnt(8), nothing else
  asm volatile("" ::: "memory");
}
__device__ inline void wait_all_loads() {
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0), nothing else
  asm volatile("" ::: "memory");
}
__device__ inline void keep_apart() { asm volatile("" ::: "memory"); }
static_assert(kLoadsPerTile == 8, "the wait above counts one tile's load instructions");

// LDS transpose read (ds_read_b64_tr_b16).  Within each group of 16 lanes, lane s passes the address of 4
// consecutive bf16 and lane i receives element (i % 4) of lanes i/4, 4 + i/4, 8 + i/4, 12 + i/4.
typedef __attribute__((ext_vector_type(4))) short i16x4;
__device__ inline i16x4 lds_read_tr16(const char* p) {
  typedef i16x4 __attribute__((address_space(3))) * lds_ptr;
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
}
union PackA {
  bf16x8 v;
  i16x4 h[2];
  uint32_t w[4];
  uint4 u;
};

// ROW_TILES: 32-row tiles per strip (1 or 2); TPW: key tiles a wave can hold (n <= 8 * TPW * 32).
template <int ROW_TILES, int TPW>
__global__ __launch_bounds__(kThreads, 1) void instr_strip_kernel(Dims dm, View q, int rows, Segments ks, int strips,
                                                                 float* part) {
  constexpr int kStripRows = 32 * ROW_TILES;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  char* const q_s = smem;                                            // [ROW_TILES][32 rows][256 B], swizzled
  char* const k_s = smem + ROW_TILES * kTileBytes;                   // [kWaves][2][8 KB]
  float2* const stats_s = reinterpret_cast<float2*>(k_s + kWaves * 2 * kTileBytes);  // [kWaves][ROW_TILES][32]

  const int tid = threadIdx.x, lane = tid % 64;
  const int wu = __builtin_amdgcn_readfirstlane(tid / 64);
  const int col = lane % 32, grp = lane / 32;
  // Workgroups go to the 8 XCDs round-robin by their linear id.  Remap so that the strips of one
  // (document, layer, KV head), which stream the same keys, are neighbours on ONE XCD and share its L2.
  int logical = blockIdx.x;
  const int total = gridDim.x;
  if (total % kXcds == 0) logical = (blockIdx.x % kXcds) * (total / kXcds) + blockIdx.x / kXcds;
  const int strip = logical % strips;
  const int unit = logical / strips;  // (b, l, g)
  const int g = unit % dm.Hkv, bl = unit / dm.Hkv, b = bl / dm.L, l = bl % dm.L;
  const int n_c = ks.n_c, n = n_c + ks.c;
  const int tiles = (n + kTileKeys - 1) / kTileKeys;
  const int total_rows = dm.G * rows;  // instruction rows of the KV group, flattened (head, row)
  const float c2 = dm.scale * kLog2e;  // logits in the log2 domain

  // ---- global -> LDS staging of one 32-key tile by ONE wave: 8 instructions of 4 rows each ----
  // The 16-byte segment `seg` of tile row `row` lives at position seg ^ f(row),
  // f(row) = 2 (row % 8) ^ ((row / 8) % 2): the operand reads below are free of bank conflicts.
  // For instruction i a lane fills row 4 i + lane / 16: f = 2 (lane / 16) ^ (8 (i % 2) | (i / 2) % 2), so the
  // lane's byte offset is (its row offset) + ((its segment term) ^ (a constant of the instruction)).
  const int k_ss_cache = static_cast<int>(ks.cache.ss), k_ss_chunk = static_cast<int>(ks.chunk.ss);
  auto seg_bytes = [](int rows_, int ss_) { return rows_ > 0 ? ((rows_ - 1) * ss_ + D) * 2 : 0; };
  const __amdgpu_buffer_rsrc_t k_rs_cache = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(unit_ptr(ks.cache, b, l, g)), 0, seg_bytes(n_c, k_ss_cache), kBufferFlags);
  const __amdgpu_buffer_rsrc_t k_rs_chunk = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(unit_ptr(ks.chunk, b, l, g)), 0, seg_bytes(ks.c, k_ss_chunk), kBufferFlags);
  typedef __attribute__((address_space(3))) void* lds_void_ptr;
  typedef __attribute__((address_space(3))) char* lds_char_ptr;
  char* const wave_lds = k_s + wu * 2 * kTileBytes;
  const uint32_t wave_lds_addr = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_char_ptr)wave_lds));
  const int fill_row = lane / 16;  // row inside the 4-row group of one instruction
  const int fill_pos = lane % 16;  // 16-byte position inside the LDS row
  const int fill_seg = (fill_pos ^ (2 * fill_row)) * 16;
  auto fill_tile = [&](int tile, int buf) {
    const int j0 = tile * kTileKeys;
    char* k_t = wave_lds + buf * kTileBytes;
    const bool in_cache = j0 + kTileKeys <= n_c;             // wave-uniform: every row is a cache row
    const bool in_chunk = j0 >= n_c && j0 + kTileKeys <= n;  // wave-uniform: every row is a chunk row
    if (in_cache || in_chunk) {  // one resource, scalar row offsets
      const __amdgpu_buffer_rsrc_t rs = in_cache ? k_rs_cache : k_rs_chunk;
      const int ss2 = (in_cache ? k_ss_cache : k_ss_chunk) * 2;
      const int r0 = in_cache ? j0 : j0 - n_c;
      const int row_off = fill_row * ss2;
#pragma unroll
      for (int i = 0; i < kLoadsPerTile; ++i) {
        const int ci = ((8 * (i % 2)) | ((i / 2) % 2)) * 16;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void_ptr)(k_t + 4 * i * kRowBytes), 16, row_off + (fill_seg ^ ci),
                                                 (r0 + 4 * i) * ss2, 0, 0);
      }
    } else {
      // The tile holds the cache / chunk boundary or the end of the candidates (rows past the end re-read
      // the last row: finite values, masked in the logits).  Two separately predicated loads, each with
      // ONE buffer resource: a resource chosen per lane would be loaded in a serialising loop.  Such a
      // tile takes 8 to 16 load instructions; the wait in the key loop counts 8 for the newest tile, so
      // behind such a tile it waits for more than it needs, never for less.
#pragma unroll
      for (int i = 0; i < kLoadsPerTile; ++i) {
        const int ci = ((8 * (i % 2)) | ((i / 2) % 2)) * 16;
        const int seg = fill_seg ^ ci;
        lds_void_ptr kd = (lds_void_ptr)(k_t + 4 * i * kRowBytes);
        const int j = min(j0 + 4 * i + fill_row, n - 1);
        if (j < n_c) __builtin_amdgcn_raw_ptr_buffer_load_lds(k_rs_cache, kd, 16, j * k_ss_cache * 2 + seg, 0, 0, 0);
        keep_apart();
        if (j >= n_c)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(k_rs_chunk, kd, 16, (j - n_c) * k_ss_chunk * 2 + seg, 0, 0, 0);
        keep_apart();
      }
    }
  };

  // ---- the strip's instruction rows: whole 256-byte rows into LDS, four per load instruction ----
  // Flattened row fl = strip * kStripRows + r is row fl % rows of head fl / rows of the group; rows past the
  // end repeat the last one and are given weight 0 at the end.
  {
    const __amdgpu_buffer_rsrc_t q_rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>(unit_ptr(q, b, l, g * dm.G)), 0,
        static_cast<int>(((dm.G - 1) * q.sh + (rows - 1) * q.ss + D) * 2), kBufferFlags);
    constexpr int kQInstr = kStripRows / 4;  // load instructions for the strip
#pragma unroll
    for (int x = 0; x < (kQInstr + kWaves - 1) / kWaves; ++x) {
      const int i = wu + kWaves * x;  // wave-uniform
      if (i < kQInstr) {
        const int r = 4 * i + fill_row;
        const int f = (2 * (r % 8)) ^ ((r / 8) % 2);
        const int fl = min(strip * kStripRows + r, total_rows - 1);
        const int hh = fl / rows, t = fl - hh * rows;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(q_rs, (lds_void_ptr)(q_s + 4 * i * kRowBytes), 16,
                                                 static_cast<int>((hh * q.sh + t * q.ss) * 2) + ((fill_pos ^ f) * 16), 0, 0,
                                                 0);
      }
    }
  }
  if (wu < tiles) fill_tile(wu, 0);
  wait_all_loads();
  __syncthreads();  // every wave's part of the strip has landed

  // per-lane LDS read addresses of the eight A operands of a key tile in buffer 0 of the wave's region
  // (swizzle included); buffer 1 is an immediate offset
  const int f_col = (2 * (col & 7)) ^ ((col >> 3) & 1);
  uint32_t k_addr[8];
  int q_off[8];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) {
    q_off[kk] = col * kRowBytes + (((2 * kk + grp) ^ f_col) * 16);
    k_addr[kk] = wave_lds_addr + q_off[kk];
  }

  // Q^T operands: q_op[rt][kk] = row (32 rt + col) of the strip, head_dim 16 kk + 8 grp .. + 7
  bf16x8 q_op[ROW_TILES][8];
#pragma unroll
  for (int rt = 0; rt < ROW_TILES; ++rt)
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      Pack8 p;
      p.u = *reinterpret_cast<const uint4*>(q_s + rt * kTileBytes + q_off[kk]);
      q_op[rt][kk] = p.v;
    }
  PackA ones;  // eight bf16 1.0: the A operand that adds a tile's weights along the keys
#pragma unroll
  for (int x = 0; x < 4; ++x) ones.w[x] = 0x3f803f80u;

  // ---- the key loop: un-normalised weights of the wave's tiles, kept in registers ----
  // e_pk[i][rt][x]: weights of key slots (2x, 2x + 1) of the lane's row in row tile rt, key tile i (bf16 pairs:
  // the B operand layout of a product that contracts over the keys)
  uint32_t e_pk[TPW][ROW_TILES][8];
  float ref[TPW][ROW_TILES];    // the reference the weights of a tile were taken against (log2 domain)
  float m_run[ROW_TILES], l_run[ROW_TILES];
#pragma unroll
  for (int rt = 0; rt < ROW_TILES; ++rt) {
    m_run[rt] = -INFINITY;
    l_run[rt] = 0.f;
  }
#pragma unroll
  for (int i = 0; i < TPW; ++i) {
    const int kt = wu + kWaves * i;  // wave-uniform
#pragma unroll
    for (int rt = 0; rt < ROW_TILES; ++rt) {
      ref[i][rt] = -INFINITY;
#pragma unroll
      for (int x = 0; x < 8; ++x) e_pk[i][rt][x] = 0u;
    }
    if (kt >= tiles) continue;
    // the other buffer was last read in the previous iteration, whose reads have all returned
    if (i + 1 < TPW && kt + kWaves < tiles) {
      fill_tile(kt + kWaves, (i & 1) ^ 1);
      wait_all_but_newest_tile();
    } else {
      wait_all_loads();
    }
    bf16x8 ka[8];
    if (i & 1)
      lds_read_k_operands<kTileBytes>(ka, k_addr);
    else
      lds_read_k_operands<0>(ka, k_addr);
    const int valid = n - kTileKeys * kt;  // keys of the tile that exist (wave-uniform)
#pragma unroll
    for (int rt = 0; rt < ROW_TILES; ++rt) {
      f32x16 s;
#pragma unroll
      for (int x = 0; x < 16; ++x) s[x] = 0.f;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[kk], q_op[rt][kk], s, 0, 0, 0);
      if (valid < kTileKeys) {
#pragma unroll
        for (int x = 0; x < 16; ++x)
          if (8 * (x / 4) + 4 * grp + (x % 4) >= valid) s[x] = -INFINITY;
      }
      float mx = __builtin_fmaxf(__builtin_fmaxf(s[0], s[1]), s[2]);
#pragma unroll
      for (int x = 3; x < 15; x += 2) mx = __builtin_fmaxf(__builtin_fmaxf(mx, s[x]), s[x + 1]);
      mx = __builtin_fmaxf(mx, s[15]) * c2;
      // Lazy reference, one per row (the two lanes of a row see different keys of the tile and share it): it
      // only has to stay within kMaxSlack of the row's running maximum, so the exchange with the other lane
      // happens in the rare branch alone.
      if (__any(mx > m_run[rt] + kMaxSlack)) {  // wave-uniform; rare after the first tile
        const float mxr = fmaxf(mx, __shfl_xor(mx, 32, 64));
        if (mxr > m_run[rt] + kMaxSlack) {
          l_run[rt] *= __builtin_amdgcn_exp2f(m_run[rt] - mxr);  // 0 when nothing was seen before
          m_run[rt] = mxr;
        }
      }
      const float m_sub = m_run[rt] == -INFINITY ? 0.f : m_run[rt];  // a row whose keys are all masked so far
      ref[i][rt] = m_run[rt];
      PackA pb[2];
#pragma unroll
      for (int x = 0; x < 8; ++x) {
        const float e0 = __builtin_amdgcn_exp2f(fmaf(s[2 * x], c2, -m_sub));
        const float e1 = __builtin_amdgcn_exp2f(fmaf(s[2 * x + 1], c2, -m_sub));
        const uint32_t w = pack_bf16x2(e0, e1);
        e_pk[i][rt][x] = w;
        pb[x / 4].w[x % 4] = w;
      }
      // the row's sum over the tile's 32 keys (both lanes of the row get it), of the rounded weights: a
      // product with a matrix of ones on the matrix pipe instead of sixteen vector additions
      f32x16 lacc;
#pragma unroll
      for (int x = 0; x < 16; ++x) lacc[x] = 0.f;
      lacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones.v, pb[0].v, lacc, 0, 0, 0);
      lacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones.v, pb[1].v, lacc, 0, 0, 0);
      l_run[rt] += lacc[0];
    }
  }

  // ---- row normalisers: the (reference, sum) pairs of the eight waves ----
  if (grp == 0) {
#pragma unroll
    for (int rt = 0; rt < ROW_TILES; ++rt) stats_s[(wu * ROW_TILES + rt) * 32 + col] = make_float2(m_run[rt], l_run[rt]);
  }
  __syncthreads();
  float m_row[ROW_TILES], inv_row[ROW_TILES];
#pragma unroll
  for (int rt = 0; rt < ROW_TILES; ++rt) {
    float mm = -INFINITY;
#pragma unroll
    for (int x = 0; x < kWaves; ++x) mm = fmaxf(mm, stats_s[(x * ROW_TILES + rt) * 32 + col].x);
    float lsum = 0.f;
#pragma unroll
    for (int x = 0; x < kWaves; ++x) {  // fixed order: every lane of the row gets the same bits
      const float2 ps = stats_s[(x * ROW_TILES + rt) * 32 + col];
      lsum += ps.x == -INFINITY ? 0.f : ps.y * __builtin_amdgcn_exp2f(ps.x - mm);
    }
    m_row[rt] = mm;
    const bool real_row = strip * kStripRows + 32 * rt + col < total_rows;
    inv_row[rt] = real_row ? 1.f / lsum : 0.f;  // padding rows carry no weight
  }

  // ---- column sums of the strip, on the matrix pipe ----
  // score[key] = sum over the strip's rows of weight[row][key] * factor[row], factor = 2^(reference - row
  // maximum) / row sum: a product that contracts over the ROWS.  The weights sit in registers with the
  // keys in the contraction slots, so each tile goes through the wave's own (now idle) LDS region once:
  // written row-major [row][key] and read back with transpose reads as the A operand (keys x rows).  The B
  // operand holds the factors in its first two columns: the bf16 head of each factor in column 0 and the
  // bf16 rest in column 1 (together 16 significant bits); the two columns are added by the strip sum.
  constexpr int kEPitch = 72;                      // bytes per row of the [32 rows][32 keys] bf16 tile (18 banks:
                                                   // rows r and r + 16 share banks, the others do not)
  char* const e_t = wave_lds;                      // 2.25 KB
  char* const f_t = wave_lds + 32 * kEPitch;       // [2][32] bf16 factors: heads, rests
  const int s16 = lane % 16, q16 = lane / 16;
  const char* const a_rd = e_t + (8 * (q16 / 2) + s16 / 4) * kEPitch + (16 * (q16 % 2) + 4 * (s16 % 4)) * 2;
  float* const dst = part + ((static_cast<int64_t>(unit) * strips + strip) * 2 + col) * n;  // col < 2 only
#pragma unroll
  for (int i = 0; i < TPW; ++i) {
    const int kt = wu + kWaves * i;  // wave-uniform
    if (kt >= tiles) continue;
    f32x16 acc;
#pragma unroll
    for (int x = 0; x < 16; ++x) acc[x] = 0.f;
#pragma unroll
    for (int rt = 0; rt < ROW_TILES; ++rt) {
      const float f = ref[i][rt] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ref[i][rt] - m_row[rt]) * inv_row[rt];
      const uint32_t f_hi = pack_bf16x2(f, 0.f);
      const uint32_t f_lo = pack_bf16x2(f - bf16_lo(f_hi), 0.f);
#pragma unroll
      for (int x = 0; x < 4; ++x)  // key slots 4 x .. + 3 of the lane = keys 8 x + 4 grp .. + 3 of the tile
        *reinterpret_cast<uint2*>(e_t + col * kEPitch + (8 * x + 4 * grp) * 2) =
            make_uint2(e_pk[i][rt][2 * x], e_pk[i][rt][2 * x + 1]);
      if (grp == 0) {
        *reinterpret_cast<uint16_t*>(f_t + 2 * col) = static_cast<uint16_t>(f_hi);
        *reinterpret_cast<uint16_t*>(f_t + 64 + 2 * col) = static_cast<uint16_t>(f_lo);
      }
      __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the wave's own LDS writes are done
      asm volatile("" ::: "memory");
#pragma unroll
      for (int st = 0; st < 2; ++st) {  // two contraction steps of 16 rows
        PackA a, fb;
        a.h[0] = lds_read_tr16(a_rd + (16 * st) * kEPitch);
        a.h[1] = lds_read_tr16(a_rd + (16 * st + 4) * kEPitch);
        fb.u = make_uint4(0u, 0u, 0u, 0u);
        if (col < 2) fb.u = *reinterpret_cast<const uint4*>(f_t + 64 * col + (16 * st + 8 * grp) * 2);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, fb.v, acc, 0, 0, 0);
      }
      asm volatile("" ::: "memory");  // the next tile's writes stay behind these reads
    }
    if (col < 2) {
#pragma unroll
      for (int x = 0; x < 16; ++x) {
        const int j = kTileKeys * kt + 8 * (x / 4) + 4 * grp + (x % 4);
        if (j < n) dst[j] = acc[x];
      }
    }
  }
}

// score[u][j] = sum over the strips' partial columns s (ascending) of part[u][s][j]
__global__ __launch_bounds__(256) void strip_sum_kernel(const float* __restrict__ part, int strips, int n, int64_t total,
                                                       float* __restrict__ score) {
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int64_t u = idx / n;
  const int j = static_cast<int>(idx - u * n);
  const float* p = part + u * (2 * strips) * n + j;  // two partial columns per strip
  float v = p[0];
  for (int s = 1; s < 2 * strips; ++s) v += p[static_cast<int64_t>(s) * n];
  score[idx] = v;
}

template <int ROW_TILES>
constexpr int strip_lds_bytes() {
  return ROW_TILES * kTileBytes + kWaves * 2 * kTileBytes + kWaves * ROW_TILES * 32 * 8;
}

template <int ROW_TILES, int TPW>
hipError_t strip_launch(const Dims& dm, View q, int rows, Segments ks, float* part, float* score, hipStream_t st) {
  const int n = ks.n_c + ks.c;
  const int strips = (dm.G * rows + 32 * ROW_TILES - 1) / (32 * ROW_TILES);
  const int units = dm.B * dm.L * dm.Hkv;
  constexpr int lds = strip_lds_bytes<ROW_TILES>();
  auto kern = instr_strip_kernel<ROW_TILES, TPW>;
  static LdsLimit limit;
  hipError_t e = raise_lds_limit(limit, reinterpret_cast<const void*>(kern), lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(units * strips), dim3(kThreads), lds, st, dm, q, rows, ks, strips, part);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int64_t total = static_cast<int64_t>(units) * n;
  hipLaunchKernelGGL(strip_sum_kernel, dim3(static_cast<unsigned>((total + 255) / 256)), dim3(256), 0, st, part, strips, n,
                     total, score);
  return hipGetLastError();
}

constexpr int kStripMaxKeysShort = kWaves * 5 * kTileKeys;   // 1280: 64-row strips, five key tiles per wave
constexpr int kStripMaxKeysLong = kWaves * 10 * kTileKeys;   // 2560: 32-row strips, ten key tiles per wave
constexpr int kStripMaxRows = 512;  // instruction rows per KV group: bounds the partial sums to 16 strips per KV head
constexpr int kStripMaxGroups = 608;  // workgroups per launch: twice the compute units of the largest gfx9 part (304)

}  // namespace

// compute units of the current device, looked up once per device
static int compute_units() {
  static std::atomic<int> cached[kMaxDevices] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
  int cus = cached[dev].load(std::memory_order_relaxed);
  if (cus == 0) {
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
    cached[dev].store(cus, std::memory_order_relaxed);
  }
  return cus;
}

// Floats of partial column sums a launch writes: two columns per strip; counted for the finer strip height,
// which bounds both.
static size_t strip_partial_floats(const Dims& dm, int rows, int n) {
  const size_t units = static_cast<size_t>(dm.B) * dm.L * dm.Hkv;
  const size_t strips = (static_cast<size_t>(dm.G) * rows + 31) / 32;
  return units * strips * 2 * n;
}

bool instr_strip_supported(const Dims& dm, const View& q, int rows, const Segments& ks, size_t workspace_floats) {
  const int n = ks.n_c + ks.c;
  if (n < 1 || n > kStripMaxKeysLong || rows < 1 || dm.G * rows > kStripMaxRows) return false;
  // worth it while the workgroups (one per KV head and strip) fit the chip twice; see the top of this file
  const int strip_rows = (n <= kStripMaxKeysShort && dm.G * rows > 32) ? 64 : 32;
  const int64_t groups = static_cast<int64_t>(dm.B) * dm.L * dm.Hkv * ((dm.G * rows + strip_rows - 1) / strip_rows);
  if (groups > 2 * compute_units() || groups > kStripMaxGroups) return false;
  if (strip_partial_floats(dm, rows, n) > workspace_floats) return false;  // the caller's block was sized for less
  // per-lane byte offsets into the group's instruction rows and into a key segment are 32-bit
  constexpr int64_t kSpan = int64_t{1} << 31;
  if (q.sh < 0 || q.ss <= 0 || ((dm.G - 1) * q.sh + (rows - 1) * q.ss + D) * 2 >= kSpan) return false;
  auto fits = [&](const View& v, int r) { return v.ss > 0 && ((r > 0 ? r - 1 : 0) * v.ss + D) * 2 < kSpan; };
  return fits(ks.cache, ks.n_c) && fits(ks.chunk, ks.c);
}

size_t instr_strip_workspace_floats(const Dims& dm, int rows, int n) {
  // The largest shape (r <= rows, m <= n) the launcher may hand to this kernel: G r <= kStripMaxRows, and no more
  // workgroups than any chip takes twice even with the taller strips (a bound that needs no device query: the
  // size of a workspace must not depend on where it is asked for); m <= kStripMaxKeysLong.  The need grows with
  // both, so the largest admissible pair bounds every smaller call.
  const size_t units = static_cast<size_t>(dm.B) * dm.L * dm.Hkv;
  if (units < 1 || units > kStripMaxGroups || dm.G < 1 || dm.G > kStripMaxRows || rows < 1 || n < 1) return 0;
  const size_t tall_strips = kStripMaxGroups / units;                       // 64-row strips per KV head, at most
  size_t r = static_cast<size_t>(kStripMaxRows) / dm.G;                     // G r <= kStripMaxRows
  if (64 * tall_strips / dm.G < r) r = 64 * tall_strips / dm.G;            // ceil(G r / 64) <= tall_strips
  if (static_cast<size_t>(rows) < r) r = rows;
  if (r < 1) return 0;
  const int m = n < kStripMaxKeysLong ? n : kStripMaxKeysLong;
  return strip_partial_floats(dm, static_cast<int>(r), m);
}

hipError_t launch_instr_strip(const Dims& dm, View q, int rows, Segments ks, float* workspace, size_t workspace_floats,
                              float* score, hipStream_t st) {
  const int n = ks.n_c + ks.c;
  if (!instr_strip_supported(dm, q, rows, ks, workspace_floats)) return hipErrorInvalidValue;
  if (n <= kStripMaxKeysShort && dm.G * rows > 32) return strip_launch<2, 5>(dm, q, rows, ks, workspace, score, st);
  if (n <= kStripMaxKeysShort) return strip_launch<1, 5>(dm, q, rows, ks, workspace, score, st);
  return strip_launch<1, 10>(dm, q, rows, ks, workspace, score, st);
}

}  // namespace citrus
