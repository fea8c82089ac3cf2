// Device code of the FDA monitor for gfx950 (wave64): shared definitions and the streaming
// state kernel (Algorithm 1 line 6).  The other kernels are in fda_small_kernels.hpp.
//
// The hash of a coordinate (bucket and sign per sketch row) depends on the coefficients and on
// j only -- not on the worker, not on the step.  Evaluating two cubics mod p per sketch row
// costs more vector-ALU work per coordinate than the whole rest of the pass is allowed at the
// HBM roofline, so it is evaluated once per context into a table in HBM which the state pass
// streams next to the slab: one record per coordinate holding, for every sketch row of a row
// group, a field of FB bits (bucket in the low FB-1 bits, top bit set for sign -1), fields packed
// back to back and the record padded to whole 16-bit words -- 10 bytes per coordinate for a
// 7 x 1000 sketch, 8 for 5 x 500 and 5 x 250 (FB = 11), 2 bytes per row for wider sketches
// (FB = 16).  A lane's V = 4 coordinates are 4 consecutive records: a few wide loads.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "fda.h"

namespace fda {

constexpr uint32_t kPrime = 0x7fffffffu;     // 2^31 - 1
constexpr int kStateThreads = 512;           // 8 waves per workgroup
constexpr int kMaxKC = 8;                    // worker slots of one workgroup
constexpr int kSmallThreads = 256;

struct HashCoef {
  uint32_t c[FDA_MAX_SKETCH_ROWS][2][4];     // [row][bucket|sign][power of j]
};

// Which kind of LDS sketch cell a state kernel accumulates into.
enum CellKind { kCellI32 = 0, kCellI64 = 1, kCellF64 = 2 };

// Fixed-point scales of one fda_local_state call, chosen on the device from a sample of the
// drifts (scale_kernel) and read by the state and merge kernels, and the flags that send a
// call from the 32-bit integer cells to the 64-bit ones and from those to fp64 cells.
struct ScaleInfo {
  double S64, invS64;     // 64-bit cells: a drift u is added as the integer round(u * S64)
  double invS32;
  float S32;              // 32-bit cells: round(u * S32)
  float bound32;          // every |u| must stay below this for the 32-bit cells to be valid
  float bound64;          // ... and below this for the 64-bit cells
  int flag32;             // set: the 32-bit result is void (range, or a cell wrapped) -> 64-bit pass
  int overflow64;         // set: the 64-bit cells cannot hold the drifts either -> fp64 pass
  int flagm;              // mean-state kernel: set when a drift reached boundm -> its fp64 pass
  double invSm;
  float Sm;               // mean-state kernel: a drift u enters as the integer round(u * Sm)
  float boundm;           // ... and every |u| must stay below this
};

struct StateParams {
  const void* w;
  const float* w_t0;
  const float* xi;
  long long row_stride;
  long long d;
  long long chunk;        // coordinates per partition (multiple of the tile)
  int K;
  int l;
  int m;
  int G;                  // worker groups
  int R;                  // sketch-row groups (workgroups of one worker group share the data)
  int P;                  // coordinate partitions
  int stride;             // 8-byte-cell passes: LDS cells per bucket (>= worker slots of the group, odd)
  int do_lin;
  int do_sk;
  int vec_ok;             // whole-vector loads and stores may be used (pointers are element-aligned)
  double* part_np;        // [P][K][2]
  void* part_sk;          // [P][K][l*m] 8-byte words: int64 (integer cells) or double (fp64 cells)
  ScaleInfo* scale;
  const uint16_t* table;  // [R][dpad] records of the tabulated hash (32-bit-cell pass only)
  long long dpad;
  int grp;                // rows per placement group of the table (1: a field is a bucket of its own row)
  HashCoef coef;          // the fallback passes evaluate the hash themselves
};

struct bf16_t { uint16_t bits; };

// Vectors of 2 or 4 dwords that only promise the alignment of the element they are made of (4 bytes
// for fp32 data, 2 for bf16).  gfx950 executes 8- and 16-byte global loads and stores at any such
// address, so a slab whose rows start off the 16-byte grid (d not a multiple of the vector width,
// odd strides) still moves whole vectors.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4), aligned(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2), aligned(4)));
typedef float f32x4 __attribute__((ext_vector_type(4), aligned(4)));
typedef uint32_t u32x4_h __attribute__((ext_vector_type(4), aligned(2)));     // 8 bf16
typedef uint32_t u32x2_h __attribute__((ext_vector_type(2), aligned(2)));     // 4 bf16

// Streaming loads.  Every byte of the slab is read exactly once per pass, so its loads carry the
// nontemporal hint: on this chip a read-only pass of plain 16-byte loads reaches about 6.3 TB/s, the
// same pass with the hint about 7.1 TB/s (the library's calibration kernels measure both).  w_t0, xi
// and the hash table are read by every worker group of a coordinate range; hinting them too cost the
// passes with several worker groups up to a tenth, so they keep plain loads.
#ifndef FDA_NT_SLAB
#define FDA_NT_SLAB 1
#endif
#ifndef FDA_NT_SHARED
#define FDA_NT_SHARED 0
#endif
template <typename VecT, bool NT>
__device__ __forceinline__ VecT load_vec_hint(const void* p) {
  if constexpr (NT) return __builtin_nontemporal_load(reinterpret_cast<const VecT*>(p));
  else return *reinterpret_cast<const VecT*>(p);
}
typedef uint32_t u32x2_a8 __attribute__((ext_vector_type(2)));                // 8-byte aligned pair (table words)
constexpr bool kNtSlab = FDA_NT_SLAB != 0;
constexpr bool kNtShared = FDA_NT_SHARED != 0;

// ---- slab element access ---------------------------------------------------------------
template <typename T> struct Slab;
template <> struct Slab<float> {
  static constexpr int V = 4;                // elements per 16-byte load
  static __device__ __forceinline__ void load_vec(const float* p, float (&x)[4]) {
    const f32x4 t = *reinterpret_cast<const f32x4*>(p);
    x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
  }
  static __device__ __forceinline__ float load_one(const float* p) { return *p; }
  static __device__ __forceinline__ void store_vec(float* p, const float (&x)[4]) {
    const f32x4 t = {x[0], x[1], x[2], x[3]};
    *reinterpret_cast<f32x4*>(p) = t;
  }
  static __device__ __forceinline__ void store_one(float* p, float x) { *p = x; }
};
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;   // NaN stays NaN
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;                   // ties to even
}
template <> struct Slab<bf16_t> {
  static constexpr int V = 8;
  static __device__ __forceinline__ void load_vec(const bf16_t* p, float (&x)[8]) {
    const u32x4_h t = *reinterpret_cast<const u32x4_h*>(p);
    x[0] = __uint_as_float(t.x << 16); x[1] = __uint_as_float(t.x & 0xffff0000u);
    x[2] = __uint_as_float(t.y << 16); x[3] = __uint_as_float(t.y & 0xffff0000u);
    x[4] = __uint_as_float(t.z << 16); x[5] = __uint_as_float(t.z & 0xffff0000u);
    x[6] = __uint_as_float(t.w << 16); x[7] = __uint_as_float(t.w & 0xffff0000u);
  }
  static __device__ __forceinline__ float load_one(const bf16_t* p) {
    return __uint_as_float((uint32_t)p->bits << 16);
  }
  static __device__ __forceinline__ void store_vec(bf16_t* p, const float (&x)[8]) {
    u32x4_h t;
    t.x = f32_to_bf16_rne(x[0]) | (f32_to_bf16_rne(x[1]) << 16);
    t.y = f32_to_bf16_rne(x[2]) | (f32_to_bf16_rne(x[3]) << 16);
    t.z = f32_to_bf16_rne(x[4]) | (f32_to_bf16_rne(x[5]) << 16);
    t.w = f32_to_bf16_rne(x[6]) | (f32_to_bf16_rne(x[7]) << 16);
    *reinterpret_cast<u32x4_h*>(p) = t;
  }
  static __device__ __forceinline__ void store_one(bf16_t* p, float x) {
    p->bits = (uint16_t)f32_to_bf16_rne(x);
  }
};

template <int V, bool NT = false>
__device__ __forceinline__ void load_f32_vec(const float* p, float (&x)[V]) {
#pragma unroll
  for (int q = 0; q < V; q += 4) {
    const f32x4 t = load_vec_hint<f32x4, NT>(p + q);
    x[q] = t.x; x[q + 1] = t.y; x[q + 2] = t.z; x[q + 3] = t.w;
  }
}
template <int V>
__device__ __forceinline__ void store_f32_vec(float* p, const float (&x)[V]) {
#pragma unroll
  for (int q = 0; q < V; q += 4) {
    const f32x4 t = {x[q], x[q + 1], x[q + 2], x[q + 3]};
    *reinterpret_cast<f32x4*>(p + q) = t;
  }
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
  return v;                                   // valid in lane 0
}

// Sum over the workgroup in a fixed shape; result valid in thread 0.  `scratch` holds one
// double per wave.  Ends with a barrier so scratch can be reused.
__device__ __forceinline__ double block_sum(double v, double* scratch) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  v = wave_sum(v);
  if (lane == 0) scratch[wave] = v;
  __syncthreads();
  double r = 0.0;
  if (threadIdx.x == 0)
    for (int t = 0; t < nw; ++t) r += scratch[t];
  __syncthreads();
  return r;
}

// Split of K workers into G nearly equal groups.
__device__ __host__ inline void group_range(int K, int G, int g, int* start, int* count) {
  int base = K / G, rem = K % G;
  *count = base + (g < rem ? 1 : 0);
  *start = g * base + (g < rem ? g : rem);
}

constexpr double kRoundMagic = 6755399441055744.0;       // 1.5 * 2^52

// ---- arithmetic modulo the Mersenne prime 2^31 - 1 (operands already reduced) --------
__device__ __forceinline__ uint32_t addmod(uint32_t a, uint32_t b) {
  uint32_t s = a + b;                        // < 2^32
  return min(s, s - kPrime);                 // s - p wraps to a huge value when s < p
}
__device__ __forceinline__ uint32_t mulmod(uint32_t a, uint32_t b) {
  uint64_t t = (uint64_t)a * b;              // < 2^62
  uint32_t lo = (uint32_t)t & kPrime;
  uint32_t hi = (uint32_t)(t >> 31);         // 2^31 = 1 (mod p)
  uint32_t s = lo + hi;                      // <= 2p - 1
  return min(s, s - kPrime);
}
// c[3] j^3 + c[2] j^2 + c[1] j + c[0] mod p
__device__ __forceinline__ uint32_t poly3(const uint32_t* c, uint32_t j) {
  uint32_t g = c[3];
  g = addmod(mulmod(g, j), c[2]);
  g = addmod(mulmod(g, j), c[1]);
  g = addmod(mulmod(g, j), c[0]);
  return g;
}
// bucket = floor(g_b(j) * m / 2^31) in bits 0..14, bit 15 set when g_s(j) is odd (sign -1)
__device__ __forceinline__ uint32_t hash_entry(const HashCoef& hc, int row, uint32_t j, uint32_t m) {
  const uint32_t gb = poly3(hc.c[row][0], j);
  const uint32_t gs = poly3(hc.c[row][1], j);
  return __umulhi(gb << 1, m) | ((gs & 1u) << 15);
}

// ---- the tabulated hash: geometry of a record and of a lane's share of a tile -----------
constexpr int kDummyCells = 64;              // cells of the dummy region (power of two)
// field width for a sketch of m columns (a field is below 2 m): 11 bits while m <= 1024, else 16
__host__ __device__ constexpr int field_bits_for(int m) { return m <= 1024 ? 11 : 16; }
template <int LR, int FB>
struct RecGeom {
  static constexpr int kWords = (LR * FB + 15) / 16;        // 16-bit words per coordinate record
  static constexpr int kDwords = 2 * kWords;                // dwords of a lane's 4 consecutive records
  static constexpr uint32_t kFieldMask = (1u << FB) - 1u;
};
// A field of the table is s = bucket + m * (1 when the sign is -1), below 2 m.
// The table is stored in blocks of 256 coordinates: the share of one wave of one tile (64 lanes x 4
// consecutive coordinates).  A lane's 4 records are N = RecGeom::kDwords dwords, which it loads in the
// widest pieces: N / 4 of 16 bytes, then one of 8, then one of 4.  Inside a block the dwords are laid
// out piece by piece, lane after lane within a piece, so every load instruction of the wave reads one
// dense run of 64 x 16 (8, 4) bytes.  (Records laid one after the other would make each instruction
// touch every line of the block for a part of its bytes.)
constexpr int kRecBlockCoords = 256;
// the N dwords of `lane` from the block starting at blk (16-byte aligned)
template <int N, bool NT>
__device__ __forceinline__ void load_rec_block(const uint32_t* blk, int lane, uint32_t (&out)[N]) {
  constexpr int n4 = N / 4, n2 = (N % 4) / 2, n1 = N % 2;
#pragma unroll
  for (int q = 0; q < n4; ++q) {
    const u32x4 t = load_vec_hint<u32x4, NT>(blk + (q * 64 + lane) * 4);
    out[4 * q] = t.x; out[4 * q + 1] = t.y; out[4 * q + 2] = t.z; out[4 * q + 3] = t.w;
  }
  if constexpr (n2 == 1) {
    const u32x2 t = load_vec_hint<u32x2, NT>(blk + n4 * 256 + lane * 2);
    out[4 * n4] = t.x; out[4 * n4 + 1] = t.y;
  }
  if constexpr (n1 == 1) out[N - 1] = load_vec_hint<uint32_t, NT>(blk + n4 * 256 + n2 * 128 + lane);
}
// the FB-bit field of sketch-row slot i of the lane's coordinate v (both known after unrolling:
// word index and shift fold to constants); bits above FB are garbage, callers mask
template <int LR, int FB>
__device__ __forceinline__ uint32_t rec_field(const uint32_t (&rec)[RecGeom<LR, FB>::kDwords], int v, int i) {
  const int bit = v * 16 * RecGeom<LR, FB>::kWords + i * FB;
  const int dw = bit >> 5, sh = bit & 31;
  if (sh + FB <= 32) return rec[dw] >> sh;
  return __builtin_amdgcn_alignbit(rec[dw + 1 < RecGeom<LR, FB>::kDwords ? dw + 1 : dw], rec[dw], sh);
}

// the same field, exactly (nothing above its FB bits): one bit-field extract where the field lies inside a
// dword (when it ends at bit 32 the shift alone), a funnel shift and an extract where it straddles two.
// (Written as the instruction: from the plain expression the compiler makes a shift and a mask and then
// cannot fold the scaling of the field into the address computation.)
template <int WIDTH>
__device__ __forceinline__ uint32_t bit_field(uint32_t x, uint32_t off) {     // off: the same in every lane
  uint32_t r;
  asm("v_bfe_u32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "s"(off), "n"(WIDTH));
  __builtin_assume(r < (1u << WIDTH));
  return r;
}
template <int LR, int FB>
__device__ __forceinline__ uint32_t rec_field_exact(const uint32_t (&rec)[RecGeom<LR, FB>::kDwords], int v, int i) {
  const int bit = v * 16 * RecGeom<LR, FB>::kWords + i * FB;
  const int dw = bit >> 5, sh = bit & 31;
  if (sh + FB == 32) return rec[dw] >> sh;
  if (sh + FB < 32) return bit_field<FB>(rec[dw], (uint32_t)sh);
  return bit_field<FB>(__builtin_amdgcn_alignbit(rec[dw + 1 < RecGeom<LR, FB>::kDwords ? dw + 1 : dw], rec[dw], sh), 0u);
}

// One lane's share of a tile, as loaded: V coordinates of w_t0, xi, of each worker's row and
// the V hash records.
constexpr int kStateV = 4;       // coordinates a lane owns per tile (fp32: 16 bytes, bf16: 8 bytes)
template <typename T, int KC, int LR, int FB>
struct TileRaw {
  static constexpr int V = kStateV;
  static constexpr int kWords = V * (int)sizeof(T) / 4;
  float w0[V];
  float x[V];
  uint32_t w[KC][kWords];                       // V elements of row k: 4 fp32 or 4 bf16
  uint32_t rec[RecGeom<LR, FB>::kDwords];       // the V records of the tabulated hash
};
__device__ __forceinline__ float raw_elem(const uint32_t (&r)[4], int v) {      // fp32
  return __uint_as_float(r[v]);
}
__device__ __forceinline__ float raw_elem(const uint32_t (&r)[2], int v) {      // bf16
  return __uint_as_float((v & 1) ? (r[v >> 1] & 0xffff0000u) : (r[v >> 1] << 16));
}

// ----------------------------------------------------------------------------------------
// Algorithm 1 line 6.  Workgroup (p, g, r) streams coordinates [p*chunk, (p+1)*chunk) of the
// workers of group g exactly once and owns the sketch rows of row group r.  Per tile every
// lane owns V consecutive coordinates: it loads w_t0 (and xi) once, then the V elements of
// each of its KC workers and the V table entries of each of its LR sketch rows, forms the
// drifts in registers, accumulates ||u||^2 and <xi,u> (fp32 within the tile, fp64 across
// tiles; row group 0 only) and adds sign*u into the workgroup's private LDS sketch, laid out
// [row][bucket][worker].  The loads of the next tile are issued
// before the current one is consumed.
//
// KC and LR are compile-time and the loops over them carry no tests: a group with fewer than
// KC workers re-reads its last worker into the spare slots, whose LDS columns are never
// flushed; a group with fewer than LR rows sends the spare rows' additions to a small dummy
// region behind the sketch.  (Tests inside the unrolled loops cost more scalar branching
// than the whole useful work.)
//
// How the sketch cells accumulate is dictated by the LDS of gfx950.  Measured per CU and clock
// on random cells: ds_add_f32 0.33 lanes, ds_add_f64 2.8, ds_add_u64 5.5, ds_add_rtn_u32 10.4.
// So the cells are integers and a drift u is added as round(u * 2^e), with 2^e chosen per call
// from a sample of the drifts (scale_kernel).  Integer addition is exact: the result
// does not depend on the order in which lanes and workgroups add, run-to-run bit-identical.
//   kCellI32  32-bit cells holding sum + 2^30; every add is below 2^30 in magnitude and returns
//             the old value, which must lie in [0, 2^31) -- top bit clear, i.e. the sum so far in
//             [-2^30, 2^30): then no add can have wrapped (the final values are held to the same
//             band when they are flushed).
//             The mean sampled |u| maps to about 2^18.  Runs on every call and also produces
//             the scalar components.  A value outside the band, or a drift at or above
//             ScaleInfo::bound32, raises ScaleInfo::flag32.
//             With an even number of worker slots the cells of slots 2t and 2t+1 of a bucket are
//             the low and the high half of one 8-byte word and receive q_lo + 2^32 * q_hi (as a
//             64-bit two's-complement number) in ONE ds_add_rtn_u64: half the LDS instructions,
//             measured 1.07 to 1.15 times faster.  While the low half stays inside its band it
//             neither borrows from nor carries into the high half, so both halves hold exactly
//             what two 32-bit additions would have left; once it leaves the band its top bit is
//             seen (by the next addition to the word or by the flush) and the pass is void anyway.
//   kCellI64  64-bit cells, sketch only, runs only when flag32 is set.  The sampled maximum
//             maps to qbits - 13 bits, qbits chosen from the exact largest number of terms
//             of a cell so that no cell can overflow.  A drift at or above bound64 raises
//             ScaleInfo::overflow64 (noticed by the first pass, which sees every drift).
//   kCellF64  fp64 cells (ds_add_f64), sketch only, runs only when overflow64 is set.
// ----------------------------------------------------------------------------------------
constexpr uint32_t kCellBias = 0x40000000u;   // a 32-bit cell holds its sum plus 2^30

// Where the 32-bit cells of a workgroup sit in LDS: [row slot][bucket][worker slot], KC words per
// bucket.  With an even KC two neighbouring worker slots are one 8-byte word and take one 64-bit
// addition (below); a bucket stride that is a multiple of 16 bytes would put every bucket on the
// same few banks, so when KC is a multiple of 4 two words are skipped after every 8 buckets.
// (An odd KC spreads the buckets over the banks by itself.)
__host__ __device__ constexpr bool cells32_skewed(int KC) { return KC % 4 == 0; }
__host__ __device__ constexpr uint32_t cells32_bucket_word(uint32_t b, int KC) {   // first word of bucket b in its row
  return b * (uint32_t)KC + (cells32_skewed(KC) ? ((b >> 3) << 1) : 0u);
}
// buckets a row of m takes up: with the skew a whole number of groups of 8, so that the offset of bucket
// number r * (that) + b of a run of rows is the r-th row's base plus the offset of b in its row
__host__ __device__ constexpr int cells32_row_buckets(int m, int KC) {
  return cells32_skewed(KC) ? (m + 7) / 8 * 8 : m;
}
__host__ __device__ constexpr uint32_t cells32_row_words(int m, int KC) {          // words of one row of m buckets
  return cells32_bucket_word((uint32_t)cells32_row_buckets(m, KC), KC);            // even whenever KC is
}
__host__ __device__ constexpr uint32_t cells32_words(int rows, int m, int KC) {    // rows plus the dummy region
  return (uint32_t)rows * cells32_row_words(m, KC) + cells32_row_words(kDummyCells, KC);
}
// A table with PLACED rows (sign-split LDS rows of 2 m buckets, an even number of worker slots): the row
// slots of a record come in groups of `grp` consecutive rows, and inside a group the builder of the table
// decides per coordinate which slot holds which row (a rotation).  A field is then (row within the group)
// * (buckets a row takes up, cells32_row_buckets) + s, the bucket index counted from the group's first row,
// in kPlacedFieldBits bits; the state kernel adds the group's base and never learns the row.  What the
// builder gains by it: the 64-bit LDS additions of one instruction are served 16 lanes at a time, lanes
// whose 8-byte words lie 128 bytes apart one after the other, and with a choice of slots part of those
// collisions can be avoided (measured: 8.2 to 8.7 LDS clocks per addition instead of 12.3).
constexpr int kPlacedFieldBits = 13;
__host__ __device__ constexpr int placed_group_rows(int rows, int m, int KC) {     // 0: no placement
  const int fit = (1 << kPlacedFieldBits) / cells32_row_buckets(2 * m, KC);
  const int g = rows < fit ? rows : fit;
  return g >= 2 ? g : 0;
}
// Sign-split rows (SPLIT): a row has 2 m buckets, the table field s itself is the bucket index -- terms
// of sign -1 are ADDED to bucket m + b, and the flush takes (bucket b) - (bucket m + b).  The pass then
// needs neither the negated terms nor a select per addition; it needs twice the LDS.

// floor(x + 0.5) as an integer in one instruction (|x| < 2^31): the fixed-point term of a scaled drift,
// at most half a unit from it
__device__ __forceinline__ int round_half_up(float x) {
  int q;
  asm("v_cvt_rpi_i32_f32 %0, %1" : "=v"(q) : "v"(x));
  return q;
}

template <typename T, int KC, int LR, int CELL, int FB, bool SPLIT = false>
__global__ void __launch_bounds__(kStateThreads)
state_kernel(const StateParams prm) {
  static_assert(!SPLIT || CELL == kCellI32, "sign-split rows: 32-bit cells only");
  constexpr int V = kStateV;
  constexpr long long kTile = (long long)kStateThreads * V;
  // only the 32-bit-cell pass streams the table; the fallback passes evaluate the hash
  constexpr bool kTabulated = CELL == kCellI32;
  using Geom = RecGeom<LR, FB>;
  using Tile = TileRaw<T, KC, LR, FB>;        // the fallback passes leave its records unloaded
  extern __shared__ __align__(16) unsigned char lds_raw[];
  constexpr int kCellBytes = (CELL == kCellI32) ? 4 : 8;
  if constexpr (CELL == kCellI64) {
    if (prm.scale->flag32 == 0 || prm.scale->overflow64 != 0) return;
  }
  if constexpr (CELL == kCellF64) {
    if (prm.scale->overflow64 == 0) return;
  }

  // XCD-aware placement: consecutive workgroup ids go round-robin over the 8 XCDs, so the
  // G*R workgroups that read the same coordinates (and share w_t0 / xi / slab rows / table
  // rows) get ids that land on one XCD and its L2.
  // (Partitions beyond the last multiple of 8 take the ids that are left, in order: their workgroups are
  // spread over the XCDs and fill the CUs that whole groups of 8 partitions would leave idle.)
  const int b = blockIdx.x;
  const int GR = prm.G * prm.R;
  const int aligned = (prm.P & ~7) * GR;               // workgroups of the XCD-aligned partitions
  int gr, p;
  if (b < aligned) {
    const int xcd = b & 7, slot = b >> 3;
    gr = slot % GR;
    p = (slot / GR) * 8 + xcd;
  } else {
    const int e = b - aligned;
    gr = e % GR;
    p = (prm.P & ~7) + e / GR;
  }
  const int g = gr / prm.R, r = gr - g * prm.R;
  int kstart, kcnt, rstart = 0, rcnt = 0;
  group_range(prm.K, prm.G, g, &kstart, &kcnt);
  if (prm.do_sk) group_range(prm.l, prm.R, r, &rstart, &rcnt);
  const bool scalars = (CELL == kCellI32) && (r == 0);
  bool sketch = prm.do_sk != 0;
  if constexpr (CELL == kCellI32) {
    // a later pass will redo every sketch partial: only the scalar components are left to do
    if (sketch && prm.scale->flag32 != 0) {
      if (!scalars) return;
      sketch = false;
    }
  }

  // 32-bit cells: cells32_* layout, KC words per bucket; 8-byte cells: prm.stride cells per bucket
  constexpr bool kPaired = CELL == kCellI32 && KC % 2 == 0;
  constexpr bool kSkewed = CELL == kCellI32 && cells32_skewed(KC);
  const uint32_t stride_bytes = CELL == kCellI32 ? 4u * KC : (uint32_t)prm.stride * kCellBytes;
  const int cells = rcnt * prm.m;                      // cells this workgroup owns
  const int mrow = SPLIT ? 2 * prm.m : prm.m;          // buckets of one LDS row
  const uint32_t row_words32 = cells32_row_words(mrow, KC);
  const uint32_t dummy_base = CELL == kCellI32 ? (uint32_t)rcnt * row_words32 * 4u : (uint32_t)cells * stride_bytes;
  const int lds_cells = !sketch ? 0
                        : CELL == kCellI32 ? (int)cells32_words(rcnt, mrow, KC) : (cells + kDummyCells) * prm.stride;
  double* red = reinterpret_cast<double*>(lds_raw + (((size_t)lds_cells * kCellBytes + 15) & ~(size_t)15));

  const int tid = threadIdx.x;
  if constexpr (CELL == kCellI32) {
    uint32_t* c32 = reinterpret_cast<uint32_t*>(lds_raw);
    for (int t = tid; t < lds_cells; t += kStateThreads) c32[t] = kCellBias;     // sum 0
  } else {
    unsigned long long* c64 = reinterpret_cast<unsigned long long*>(lds_raw);
    for (int t = tid; t < lds_cells; t += kStateThreads) c64[t] = 0ull;         // integer 0 and 0.0
  }
  __syncthreads();

  double dn[KC], dp[KC];
#pragma unroll
  for (int k = 0; k < KC; ++k) { dn[k] = 0.0; dp[k] = 0.0; }

  // per worker slot: its slab row (spare slots repeat the last worker);
  // per row slot: its LDS base (spare slots: the dummy region, whose table fields -- and, in the
  // fallback passes, masked buckets -- stay below kDummyCells)
  const T* wrow[KC];
#pragma unroll
  for (int k = 0; k < KC; ++k)
    wrow[k] = reinterpret_cast<const T*>(prm.w) +
              (long long)(kstart + (k < kcnt ? k : kcnt - 1)) * prm.row_stride;
  uint32_t rowbase[LR];
#pragma unroll
  for (int i = 0; i < LR; ++i) {
    // (placed rows: the base of the slot's group, the field counts buckets from there)
    if constexpr (CELL == kCellI32) rowbase[i] = i < rcnt ? (uint32_t)(i / prm.grp * prm.grp) * row_words32 * 4u : dummy_base;
    else rowbase[i] = i < rcnt ? (uint32_t)(i * prm.m) * stride_bytes : dummy_base;
  }
  // this row group's records: [r][dpad] records of Geom::kWords 16-bit words
  const uint32_t* const recs =
      reinterpret_cast<const uint32_t*>(prm.table + (size_t)r * prm.dpad * Geom::kWords);

  const long long cbeg = (long long)p * prm.chunk;
  long long cend = cbeg + prm.chunk;
  if (cend > prm.d) cend = prm.d;
  const long long dlim = prm.d;
  const bool lin = prm.do_lin && scalars;
  const float* const w0p = prm.w_t0;
  const float* const xip = lin ? prm.xi : prm.w_t0;   // without LinearFDA: any readable vector

  double S64 = 1.0;
  float S32 = 1.0f, amax = 0.0f;
  uint32_t seen_or = 0u;            // OR of every 32-bit cell value this lane's adds returned
  if (prm.do_sk) { S64 = prm.scale->S64; S32 = prm.scale->S32; }

  // SC: this workgroup also produces the scalar components; SK: it accumulates sketch rows.
  auto run = [&](auto sc_tag, auto sk_tag) {
    constexpr bool SC = decltype(sc_tag)::value;
    constexpr bool SK = decltype(sk_tag)::value;

    // whole vectors, no tests: for tiles that lie entirely inside the chunk
    auto load_fast = [&](Tile& t, long long j0) {
      load_f32_vec<V, kNtShared>(w0p + j0, t.w0);
      if constexpr (SC) load_f32_vec<V, kNtShared>(xip + j0, t.x);
#pragma unroll
      for (int k = 0; k < KC; ++k) {
        if constexpr (sizeof(T) == 4) {
          const u32x4 q = load_vec_hint<u32x4, kNtSlab>(wrow[k] + j0);
          t.w[k][0] = q.x; t.w[k][1] = q.y; t.w[k][2] = q.z; t.w[k][3] = q.w;
        } else {
          const u32x2_h q = load_vec_hint<u32x2_h, kNtSlab>(wrow[k] + j0);
          t.w[k][0] = q.x; t.w[k][1] = q.y;
        }
      }
      if constexpr (SK && kTabulated)
        load_rec_block<Geom::kDwords, kNtShared>(recs + (j0 >> 8) * (64 * Geom::kDwords), (int)(j0 >> 2) & 63, t.rec);
    };
    // element by element, every access tested: ragged tails and slabs without dword alignment
    auto load_slow = [&](Tile& t, long long j0) {
#pragma unroll
      for (int v = 0; v < V; ++v) {
        const bool in = (j0 + v < dlim);
        t.w0[v] = in ? w0p[j0 + v] : 0.0f;
        if constexpr (SC) t.x[v] = in ? xip[j0 + v] : 0.0f;
      }
#pragma unroll
      for (int k = 0; k < KC; ++k) {
        const T* row = wrow[k] + j0;
        if constexpr (sizeof(T) == 4) {
#pragma unroll
          for (int v = 0; v < 4; ++v)
            t.w[k][v] = (j0 + v < dlim) ? __float_as_uint(Slab<T>::load_one(row + v)) : 0u;
        } else {
#pragma unroll
          for (int v = 0; v < 4; v += 2) {
            const uint16_t* h = reinterpret_cast<const uint16_t*>(row);
            const uint32_t lo = (j0 + v < dlim) ? (uint32_t)h[v] : 0u;
            const uint32_t hi = (j0 + v + 1 < dlim) ? (uint32_t)h[v + 1] : 0u;
            t.w[k][v >> 1] = lo | (hi << 16);
          }
        }
      }
      // the table is padded to dpad (whole blocks of 256 coordinates): always whole records
      if constexpr (SK && kTabulated)
        load_rec_block<Geom::kDwords, false>(recs + (j0 >> 8) * (64 * Geom::kDwords), (int)(j0 >> 2) & 63, t.rec);
    };

    // fp32 partial sums of the scalar components: kept over kScalarTiles tiles (that many times V
    // terms each), then added to the fp64 sums -- the fp64 conversions and additions are the most
    // expensive instructions of the loop, and 16 fp32 terms stay well inside the tolerance
    constexpr int kScalarTiles = 4;
    float sn[KC], sp[KC];
#pragma unroll
    for (int k = 0; k < KC; ++k) { sn[k] = 0.0f; sp[k] = 0.0f; }
    int held = 0;                             // tiles whose scalar partials are still in sn / sp
    auto widen = [&]() {
      if constexpr (SC) {
#pragma unroll
        for (int k = 0; k < KC; ++k) {
          dn[k] += (double)sn[k]; dp[k] += (double)sp[k];
          sn[k] = 0.0f; sp[k] = 0.0f;
        }
      }
      held = 0;
    };

    auto consume = [&](const Tile& t, long long j0) {
      uint32_t pend_old[KC];                  // 32-bit cells: the last batch not yet examined
      bool have_pending = false;
#pragma unroll
      for (int v = 0; v < V; ++v) {
        // The 32-bit-cell pass works on u * S32 throughout: S32 is a power of two, so
        // fma(w, S32, -w_t0 * S32) is exactly (w - w_t0 as fp32 rounds it) * S32, the scalar
        // sums come out multiplied by S32^2 and S32 (undone exactly at the end), and the
        // fixed-point term is one conversion away.  (The fallback passes keep the plain drift.)
        float u[KC];
        const float w0s = (CELL == kCellI32) ? t.w0[v] * S32 : t.w0[v];
#pragma unroll
        for (int k = 0; k < KC; ++k) {
          if constexpr (CELL == kCellI32) u[k] = fmaf(raw_elem(t.w[k], v), S32, -w0s);
          else u[k] = raw_elem(t.w[k], v) - w0s;
          if constexpr (SC) {
            sn[k] = fmaf(u[k], u[k], sn[k]);
            sp[k] = fmaf(t.x[v], u[k], sp[k]);
            amax = fmaxf(amax, fabsf(u[k]));
          }
        }
        if constexpr (SK && CELL == kCellI32) {
          uint32_t q[KC], nq[KC];
#pragma unroll
          for (int k = 0; k < KC; ++k) {
            q[k] = (uint32_t)round_half_up(u[k]);
            nq[k] = SPLIT ? 0u : 0u - q[k];
          }
          // paired slots: the high half of q_lo + 2^32 * q_hi is q_hi minus one when q_lo is negative
          uint32_t qh[KC / 2 + 1], nqh[KC / 2 + 1];
          if constexpr (kPaired) {
#pragma unroll
            for (int k = 0; k < KC; k += 2) {
              qh[k / 2] = q[k + 1] + (uint32_t)((int)q[k] >> 31);
              nqh[k / 2] = SPLIT ? 0u : nq[k + 1] + (uint32_t)((int)nq[k] >> 31);
            }
          }
#pragma unroll
          for (int i = 0; i < LR; ++i) {
            const uint32_t s = rec_field_exact<LR, FB>(t.rec, v, i);
            // sign-split rows add the term itself to bucket s; otherwise s >= m means sign -1, bucket s - m
            const bool neg = !SPLIT && s >= (uint32_t)prm.m;
            const uint32_t bucket = neg ? s - (uint32_t)prm.m : s;
            // skewed: 8 more bytes after every 8 buckets, bucket * stride + (bucket & ~7) -- the same as
            // bucket * (stride + 1) with its low three bits cleared (stride and row bases: multiples of 8)
            const uint32_t off = kSkewed ? ((__umul24(bucket, stride_bytes + 1u) + rowbase[i]) & ~7u)
                                         : __umul24(bucket, stride_bytes) + rowbase[i];
            uint32_t old[KC];
            if constexpr (kPaired) {
              unsigned long long* cell = reinterpret_cast<unsigned long long*>(lds_raw + off);
#pragma unroll
              for (int k = 0; k < KC; k += 2) {
                const uint32_t lo = neg ? nq[k] : q[k], hi = neg ? nqh[k / 2] : qh[k / 2];
                const unsigned long long o = atomicAdd(cell + k / 2, ((unsigned long long)hi << 32) | lo);
                old[k] = (uint32_t)o;
                old[k + 1] = (uint32_t)(o >> 32);
              }
            } else {
              uint32_t* cell = reinterpret_cast<uint32_t*>(lds_raw + off);
#pragma unroll
              for (int k = 0; k < KC; ++k) old[k] = atomicAdd(cell + k, neg ? nq[k] : q[k]);
            }
            // Every add is below 2^30 in magnitude (ScaleInfo::bound32) and a cell holds its sum
            // plus 2^30, so a cell cannot wrap in an add that found it below 2^31 (sum so far in
            // [-2^30, 2^30)): if the top bit of every value ever returned was clear, no cell
            // wrapped.  The returned values are OR-ed together (a three-operand OR takes two of
            // them: half an instruction per add).  The values of the row before are examined only
            // now, with this row's adds already on their way, so the LDS round trip hides behind
            // the next batch.
            if (have_pending) {
#pragma unroll
              for (int k = 0; k < KC; ++k) seen_or |= pend_old[k];
            }
#pragma unroll
            for (int k = 0; k < KC; ++k) pend_old[k] = old[k];
            have_pending = true;
          }
        }
        if constexpr (SK && CELL != kCellI32) {
          // fallback passes: the hash is evaluated here (two cubics mod p per row and coordinate)
          unsigned long long q[KC], nq[KC];
          if constexpr (CELL == kCellI64) {
#pragma unroll
            for (int k = 0; k < KC; ++k) {
              const double y = fma((double)u[k], S64, kRoundMagic);           // round to integer
              q[k] = (unsigned long long)(__double_as_longlong(y) - __double_as_longlong(kRoundMagic));
              nq[k] = 0ull - q[k];
            }
          }
          const long long j = j0 + v;
          const uint32_t key = j < dlim ? (uint32_t)j : 0u;                  // past the end the drift is zero
#pragma unroll
          for (int i = 0; i < LR; ++i) {
            const bool live = i < rcnt;
            const uint32_t h = hash_entry(prm.coef, rstart + (live ? i : 0), key, (uint32_t)prm.m);
            const uint32_t bucket = live ? (h & 0x7fffu) : (h & (uint32_t)(kDummyCells - 1));
            const uint32_t off = __umul24(bucket, stride_bytes) + rowbase[i];
            const bool neg = (h & 0x8000u) != 0u;
            if constexpr (CELL == kCellI64) {
              unsigned long long* cell = reinterpret_cast<unsigned long long*>(lds_raw + off);
#pragma unroll
              for (int k = 0; k < KC; ++k) atomicAdd(cell + k, neg ? nq[k] : q[k]);
            } else {
              double* cell = reinterpret_cast<double*>(lds_raw + off);
#pragma unroll
              for (int k = 0; k < KC; ++k) atomicAdd(cell + k, neg ? -(double)u[k] : (double)u[k]);
            }
          }
        }
      }
      if constexpr (SK && CELL == kCellI32) {
        if (have_pending) {
#pragma unroll
          for (int k = 0; k < KC; ++k) seen_or |= pend_old[k];
        }
      }
      if constexpr (SC) {
        if (++held == kScalarTiles) widen();
      }
    };

    // tiles that lie wholly inside the chunk (every lane has a whole vector): software
    // pipelined, the next tile's loads in flight while the current tile is consumed
    const long long nfast = prm.vec_ok ? (cend > cbeg ? (cend - cbeg) / kTile : 0) : 0;
    long long j0 = cbeg + (long long)tid * V;
    if (nfast > 0) {
      Tile cur;
      load_fast(cur, j0);
      for (long long it = 1; it < nfast; ++it) {
        Tile nxt;
        load_fast(nxt, j0 + kTile);
        consume(cur, j0);
        cur = nxt;
        j0 += kTile;
      }
      consume(cur, j0);
      j0 += kTile;
    }
    // what is left: at most one ragged tile, or everything when vectors are not possible
    for (; j0 < cend; j0 += kTile) {
      Tile t;
      load_slow(t, j0);
      consume(t, j0);
    }
    widen();
  };
  if (scalars) {
    if (sketch) run(std::true_type{}, std::true_type{});
    else run(std::true_type{}, std::false_type{});
  } else {
    run(std::false_type{}, std::true_type{});
  }

  if constexpr (CELL == kCellI32) {
    if (prm.do_sk) {
      if (scalars) {
        // drifts the integer cells cannot hold (any drift at all when the sample saw none)
        const float b32 = prm.scale->bound32, b64 = prm.scale->bound64;
        amax = amax * (1.0f / S32);              // back to the drift's own unit (exact: a power of two)
        const bool bad32 = b32 > 0.0f ? !(amax < b32) : (amax > 0.0f);
        const bool bad64 = b64 > 0.0f ? !(amax < b64) : (amax > 0.0f);
        if (bad32 || bad64) prm.scale->flag32 = 1;
        if (bad64) prm.scale->overflow64 = 1;
      }
      if ((seen_or & 0x80000000u) != 0u) prm.scale->flag32 = 1;
    }
  }

  // ---- workgroup reduction of the scalar components (fixed shape) ---------------------
  const int lane = tid & 63, wave = tid >> 6;
  constexpr int kWaves = kStateThreads / 64;
  if (scalars) {
#pragma unroll
    for (int k = 0; k < KC; ++k) {
      double a = wave_sum(dn[k]);
      double c = wave_sum(dp[k]);
      if (lane == 0) { red[(wave * KC + k) * 2] = a; red[(wave * KC + k) * 2 + 1] = c; }
    }
  }
  __syncthreads();
  if (scalars && tid < 2 * kcnt) {
    const int k = tid >> 1, q = tid & 1;
    double s = 0.0;
    for (int wv = 0; wv < kWaves; ++wv) s += red[(wv * KC + k) * 2 + q];
    if (q == 1 && !lin) s = 0.0;               // no LinearFDA: the projection slot stays zero
    // the sums were formed on drifts scaled by S32 (a power of two: exact to undo)
    const double inv = 1.0 / (double)S32;
    prm.part_np[((size_t)p * prm.K + kstart + k) * 2 + q] = s * (q == 0 ? inv * inv : inv);
  }
  // ---- flush the LDS sketch to this workgroup's slice of the partial buffer -----------
  if (sketch) {
    const int allcells = prm.l * prm.m;
    unsigned long long* out = reinterpret_cast<unsigned long long*>(prm.part_sk);
    bool left_band = false;
    if constexpr (CELL == kCellI32) {
      // a wave takes one (row, worker) at a time, its lanes the buckets: no divisions per cell
      const uint32_t* words = reinterpret_cast<const uint32_t*>(lds_raw);
      for (int combo = wave; combo < rcnt * kcnt; combo += kWaves) {
        const int i = combo / kcnt, k = combo - i * kcnt;
        const uint32_t* row = words + (size_t)i * row_words32 + k;
        unsigned long long* dst = out + ((size_t)p * prm.K + kstart + k) * allcells + (size_t)(rstart + i) * prm.m;
        for (int bkt = lane; bkt < prm.m; bkt += 64) {
          const uint32_t word = row[cells32_bucket_word((uint32_t)bkt, KC)];
          left_band = left_band || (word & 0x80000000u) != 0u;      // the last additions are examined here
          long long sum = (long long)(int)(word - kCellBias);
          if constexpr (SPLIT) {
            const uint32_t minus = row[cells32_bucket_word((uint32_t)(bkt + prm.m), KC)];
            left_band = left_band || (minus & 0x80000000u) != 0u;
            sum -= (long long)(int)(minus - kCellBias);
          }
          dst[bkt] = (unsigned long long)sum;
        }
      }
    } else {
      for (int t = tid; t < kcnt * cells; t += kStateThreads) {
        const int k = t / cells, c = t - k * cells;
        out[((size_t)p * prm.K + kstart + k) * allcells + (size_t)rstart * prm.m + c] =
            reinterpret_cast<const unsigned long long*>(lds_raw)[(size_t)c * prm.stride + k];
      }
    }
    if constexpr (CELL == kCellI32) {
      if (left_band) prm.scale->flag32 = 1;
    }
  }
}

}  // namespace fda
