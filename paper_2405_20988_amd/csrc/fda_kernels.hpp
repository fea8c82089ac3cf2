// Device code of the FDA monitor for gfx950 (wave64).  Included by fda_api.hip only.
//
// Kernels
//   state_kernel     Algorithm 1 line 6: one streaming pass over the [K,d] slab that forms
//                    the drifts in registers and reduces them to per-workgroup partial
//                    states (squared norm, <xi,u>, AMS sketch in LDS).
//   merge_kernel     fixed-order fp64 sum of the per-workgroup partials -> state[K][S].
//   estimate_kernel  Algorithm 1 lines 7-8: mean state, M2, H (Thm 1, Thm 2), decision.
//   sync_kernel      Algorithm 1 line 9: fused mean over workers + broadcast to all rows.
//   xi_norm_kernel / xi_scale_kernel   Section 3.2: the normalized model difference.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fda.h"

namespace fda {

constexpr uint32_t kPrime = 0x7fffffffu;     // 2^31 - 1
constexpr int kStateThreads = 512;           // 8 waves per workgroup
constexpr int kMaxKC = 16;                   // workers handled by one workgroup
constexpr int kSmallThreads = 256;

struct HashCoef {
  uint32_t c[FDA_MAX_SKETCH_ROWS][2][4];     // [row][bucket|sign][power of j]
};

// Fixed-point scale of one fda_local_state call, chosen on the device from a sample of the
// drifts (scale_*_kernel) and read by the state and merge kernels.
struct ScaleInfo {
  double S;               // 2^e: a drift u enters the sketch as the integer round(u * S)
  double invS;            // 2^-e
  float bound;            // every |u| must stay below this for the integer path to be valid
  int overflow;           // set by the integer path when some |u| did not; selects the fp64 path
  int pad[2];
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
  int P;                  // coordinate partitions, multiple of 8
  int stride;             // LDS 8-byte words per sketch cell (>= workers of the group)
  int do_lin;
  int do_sk;
  int vec_ok;             // all pointers / strides allow 16-byte loads
  double* part_np;        // [P][K][2]
  void* part_sk;          // [P][K][l*m] 8-byte words: int64 (integer path) or double (fp64 path)
  ScaleInfo* scale;
};

struct bf16_t { uint16_t bits; };

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

// ---- slab element access ---------------------------------------------------------------
template <typename T> struct Slab;
template <> struct Slab<float> {
  static constexpr int V = 4;                // elements per 16-byte load
  static __device__ __forceinline__ void load_vec(const float* p, float (&x)[4]) {
    float4 t = *reinterpret_cast<const float4*>(p);
    x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
  }
  static __device__ __forceinline__ float load_one(const float* p) { return *p; }
  static __device__ __forceinline__ void store_vec(float* p, const float (&x)[4]) {
    *reinterpret_cast<float4*>(p) = make_float4(x[0], x[1], x[2], x[3]);
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
    uint4 t = *reinterpret_cast<const uint4*>(p);
    x[0] = __uint_as_float(t.x << 16); x[1] = __uint_as_float(t.x & 0xffff0000u);
    x[2] = __uint_as_float(t.y << 16); x[3] = __uint_as_float(t.y & 0xffff0000u);
    x[4] = __uint_as_float(t.z << 16); x[5] = __uint_as_float(t.z & 0xffff0000u);
    x[6] = __uint_as_float(t.w << 16); x[7] = __uint_as_float(t.w & 0xffff0000u);
  }
  static __device__ __forceinline__ float load_one(const bf16_t* p) {
    return __uint_as_float((uint32_t)p->bits << 16);
  }
  static __device__ __forceinline__ void store_vec(bf16_t* p, const float (&x)[8]) {
    uint4 t;
    t.x = f32_to_bf16_rne(x[0]) | (f32_to_bf16_rne(x[1]) << 16);
    t.y = f32_to_bf16_rne(x[2]) | (f32_to_bf16_rne(x[3]) << 16);
    t.z = f32_to_bf16_rne(x[4]) | (f32_to_bf16_rne(x[5]) << 16);
    t.w = f32_to_bf16_rne(x[6]) | (f32_to_bf16_rne(x[7]) << 16);
    *reinterpret_cast<uint4*>(p) = t;
  }
  static __device__ __forceinline__ void store_one(bf16_t* p, float x) {
    p->bits = (uint16_t)f32_to_bf16_rne(x);
  }
};

template <int V>
__device__ __forceinline__ void load_f32_vec(const float* p, float (&x)[V]) {
#pragma unroll
  for (int q = 0; q < V; q += 4) {
    float4 t = *reinterpret_cast<const float4*>(p + q);
    x[q] = t.x; x[q + 1] = t.y; x[q + 2] = t.z; x[q + 3] = t.w;
  }
}
template <int V>
__device__ __forceinline__ void store_f32_vec(float* p, const float (&x)[V]) {
#pragma unroll
  for (int q = 0; q < V; q += 4)
    *reinterpret_cast<float4*>(p + q) = make_float4(x[q], x[q + 1], x[q + 2], x[q + 3]);
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

// ---- the hash along a lane's coordinate sequence, by forward differences ---------------
// A lane visits coordinates j0, j0+1, .., j0+V-1, then the same V offsets from j0+S, j0+2S, ..
// (S = coordinates per tile).  A cubic's values on such a lattice follow from additions only:
//   inside a tile   g(j+1) = g(j) + D1(j),  D1(j+1) = D1(j) + D2(j),  D2(j+1) = D2(j) + D3
//   tile to tile    g(j+S) = g(j) + E1(j),  E1(j+S) = E1(j) + E2(j),  E2(j+S) = E2(j) + E3
//                   D1(j+S) = D1(j) + F1(j), F1(j+S) = F1(j) + F2,    D2(j+S) = D2(j) + G
// all modulo p, where D3, E3, F2, G are constants of the polynomial and of S.  Every value is
// the exact residue, so buckets and signs are those of direct evaluation.
struct Chain { uint32_t g, e1, e2, d1, f1, d2; };         // per lane
struct ChainConst { uint32_t e3, f2, gg, d3; };           // same in every lane

__device__ __forceinline__ uint32_t submod(uint32_t a, uint32_t b) {
  uint32_t s = a - b;                        // wraps when a < b
  return min(s, s + kPrime);
}
__device__ __forceinline__ uint32_t reduce_key(uint32_t x) { return min(x, x - kPrime); }  // x < 2p

__device__ __forceinline__ void chain_init(const uint32_t* c, uint32_t j, uint32_t S, Chain& ch,
                                           ChainConst& cc) {
  const uint32_t g00 = poly3(c, reduce_key(j)), g01 = poly3(c, reduce_key(j + 1));
  const uint32_t g02 = poly3(c, reduce_key(j + 2)), g03 = poly3(c, reduce_key(j + 3));
  const uint32_t g10 = poly3(c, reduce_key(j + S)), g11 = poly3(c, reduce_key(j + S + 1));
  const uint32_t g12 = poly3(c, reduce_key(j + S + 2));
  const uint32_t g20 = poly3(c, reduce_key(j + 2 * S)), g21 = poly3(c, reduce_key(j + 2 * S + 1));
  const uint32_t g30 = poly3(c, reduce_key(j + 3 * S));
  ch.g = g00;
  ch.e1 = submod(g10, g00);
  const uint32_t e1_s = submod(g20, g10), e1_2s = submod(g30, g20);
  ch.e2 = submod(e1_s, ch.e1);
  cc.e3 = submod(submod(e1_2s, e1_s), ch.e2);
  ch.d1 = submod(g01, g00);
  const uint32_t d1_s = submod(g11, g10), d1_2s = submod(g21, g20);
  ch.f1 = submod(d1_s, ch.d1);
  cc.f2 = submod(submod(d1_2s, d1_s), ch.f1);
  const uint32_t d1_1 = submod(g02, g01), d1_2 = submod(g03, g02);
  ch.d2 = submod(d1_1, ch.d1);
  cc.gg = submod(submod(submod(g12, g11), d1_s), ch.d2);
  cc.d3 = submod(submod(d1_2, d1_1), ch.d2);
}
__device__ __forceinline__ void chain_next_tile(Chain& ch, const ChainConst& cc) {
  ch.g = addmod(ch.g, ch.e1);
  ch.e1 = addmod(ch.e1, ch.e2);
  ch.e2 = addmod(ch.e2, cc.e3);
  ch.d1 = addmod(ch.d1, ch.f1);
  ch.f1 = addmod(ch.f1, cc.f2);
  ch.d2 = addmod(ch.d2, cc.gg);
}
__device__ __forceinline__ uint32_t uniform(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }

constexpr double kRoundMagic = 6755399441055744.0;       // 1.5 * 2^52

// ----------------------------------------------------------------------------------------
// Algorithm 1 line 6.  Workgroup (p, g, r) streams coordinates [p*chunk, (p+1)*chunk) of the
// workers of group g exactly once and owns the sketch rows of row group r.  Per tile every
// lane owns V consecutive coordinates: it loads w_t0 (and xi) once, then the V elements of
// each of its <= KC workers, forms the drifts in registers, accumulates ||u||^2 and <xi,u>
// (fp32 within the tile, fp64 across tiles; row group 0 only) and adds sign*u into the
// workgroup's private LDS sketch, laid out [row][bucket][worker] with an odd worker stride.
// The hash of a coordinate is evaluated once and reused by all workers of the group.
//
// How the sketch cells accumulate is dictated by the LDS of gfx950, measured per CU and
// clock on random cells: ds_add_f32 0.33 lanes, ds_add_f64 2.8, ds_add_u64 5.5.  So:
//   FX = true   the cells are 64-bit integers: u is added as round(u * 2^e) (ds_add_u64),
//               with 2^e chosen per call from a sample of the drifts so that the unit is at
//               most 2^-28 of the sampled maximum.  Integer addition is exact, so the result
//               does not depend on the order in which lanes and workgroups add: run-to-run
//               bit-identical.  A drift at or above 2^13 times the sampled maximum cannot be
//               represented; the lane that meets one raises ScaleInfo::overflow.
//   FX = false  the same pass with fp64 cells (ds_add_f64) and direct hash evaluation; it runs
//               only when ScaleInfo::overflow is set and then replaces the sketch partials.
// ----------------------------------------------------------------------------------------
template <typename T, int KC, int LR, bool FX>
__global__ void __launch_bounds__(kStateThreads)
state_kernel(const StateParams prm, const HashCoef hc) {
  constexpr int V = Slab<T>::V;
  constexpr uint32_t kTile = kStateThreads * V;
  extern __shared__ __align__(16) unsigned char lds_raw[];
  if constexpr (!FX) {
    if (prm.scale->overflow == 0) return;
  }

  // XCD-aware placement: consecutive workgroup ids go round-robin over the 8 XCDs, so the
  // G*R workgroups that read the same coordinates (and share w_t0 / xi / slab rows) get ids
  // that land on one XCD and its L2.
  const int b = blockIdx.x;
  const int xcd = b & 7, slot = b >> 3;
  const int GR = prm.G * prm.R;
  const int gr = slot % GR;
  const int p = (slot / GR) * 8 + xcd;
  const int g = gr / prm.R, r = gr - g * prm.R;
  int kstart, kcnt, rstart = 0, rcnt = 0;
  group_range(prm.K, prm.G, g, &kstart, &kcnt);
  if (prm.do_sk) group_range(prm.l, prm.R, r, &rstart, &rcnt);
  const bool scalars = FX && (r == 0);
  if constexpr (FX) {
    // the fp64 pass will redo every sketch partial: only the scalar components are left to do
    if (prm.do_sk && prm.scale->overflow != 0) {
      if (!scalars) return;
      rcnt = 0;
    }
  }

  const int cells = rcnt * prm.m;                      // cells this workgroup owns
  unsigned long long* sk = reinterpret_cast<unsigned long long*>(lds_raw);
  const size_t sk_bytes = ((size_t)cells * prm.stride * 8 + 15) & ~(size_t)15;
  double* red = reinterpret_cast<double*>(lds_raw + sk_bytes);     // [waves][KC][2]

  const int tid = threadIdx.x;
  for (int t = tid; t < cells * prm.stride; t += kStateThreads) sk[t] = 0ull;   // 0 and 0.0
  __syncthreads();

  double dn[KC], dp[KC];
#pragma unroll
  for (int k = 0; k < KC; ++k) { dn[k] = 0.0; dp[k] = 0.0; }

  const T* wbase = reinterpret_cast<const T*>(prm.w) + (long long)kstart * prm.row_stride;
  const long long cbeg = (long long)p * prm.chunk;
  long long cend = cbeg + prm.chunk;
  if (cend > prm.d) cend = prm.d;
  const bool lin = prm.do_lin && scalars;
  const uint32_t stride_bytes = (uint32_t)prm.stride * 8u;

  double S = 1.0;
  float bound = 0.0f, amax = 0.0f;
  if (FX && rcnt > 0) { S = prm.scale->S; bound = prm.scale->bound; }

  Chain ch[LR][2];
  ChainConst cc[LR][2];
  if constexpr (FX) {
#pragma unroll
    for (int i = 0; i < LR; ++i)
      if (i < rcnt) {
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          ChainConst t;
          chain_init(hc.c[rstart + i][c], (uint32_t)(cbeg + (long long)tid * V), kTile, ch[i][c], t);
          cc[i][c].e3 = uniform(t.e3); cc[i][c].f2 = uniform(t.f2);
          cc[i][c].gg = uniform(t.gg); cc[i][c].d3 = uniform(t.d3);
        }
      }
  }

  for (long long j0 = cbeg + (long long)tid * V; j0 < cend; j0 += (long long)kTile) {
    float w0[V], x[V], u[KC][V];
    const bool full = prm.vec_ok && (j0 + V <= prm.d);
    if (full) {
      load_f32_vec<V>(prm.w_t0 + j0, w0);
      if (lin) load_f32_vec<V>(prm.xi + j0, x);
#pragma unroll
      for (int k = 0; k < KC; ++k)
        if (k < kcnt) Slab<T>::load_vec(wbase + (long long)k * prm.row_stride + j0, u[k]);
    } else {
#pragma unroll
      for (int v = 0; v < V; ++v) {
        const bool in = (j0 + v < prm.d);
        w0[v] = in ? prm.w_t0[j0 + v] : 0.0f;
        if (lin) x[v] = in ? prm.xi[j0 + v] : 0.0f;
#pragma unroll
        for (int k = 0; k < KC; ++k)
          if (k < kcnt)
            u[k][v] = in ? Slab<T>::load_one(wbase + (long long)k * prm.row_stride + j0 + v) : 0.0f;
      }
    }
    if (!lin) {
#pragma unroll
      for (int v = 0; v < V; ++v) x[v] = 0.0f;
    }
#pragma unroll
    for (int k = 0; k < KC; ++k) {
      if (k < kcnt) {
        float sn = 0.0f, sp = 0.0f;
#pragma unroll
        for (int v = 0; v < V; ++v) {
          u[k][v] -= w0[v];
          sn = fmaf(u[k][v], u[k][v], sn);
          sp = fmaf(x[v], u[k][v], sp);
          if (FX) amax = fmaxf(amax, fabsf(u[k][v]));
        }
        if (scalars) {
          dn[k] += (double)sn;
          dp[k] += (double)sp;
        }
      }
    }
    if constexpr (FX) {
      // byte offset of the cell of (row, coordinate) in bits 0..30, the sign in bit 31
      uint32_t where[LR][V];
#pragma unroll
      for (int i = 0; i < LR; ++i)
        if (i < rcnt) {
          uint32_t gb[V], gs[V];
#pragma unroll
          for (int c = 0; c < 2; ++c) {
            uint32_t a = ch[i][c].g, d1 = ch[i][c].d1, d2 = ch[i][c].d2;
#pragma unroll
            for (int v = 0; v < V; ++v) {
              if (c == 0) gb[v] = a; else gs[v] = a;
              if (v + 1 < V) {
                a = addmod(a, d1);
                if (v + 2 < V) { d1 = addmod(d1, d2); d2 = addmod(d2, cc[i][c].d3); }
              }
            }
            chain_next_tile(ch[i][c], cc[i][c]);
          }
          const uint32_t rowbase = (uint32_t)(i * prm.m) * stride_bytes;
#pragma unroll
          for (int v = 0; v < V; ++v) {
            const uint32_t bucket = __umulhi(gb[v] << 1, (uint32_t)prm.m);   // floor(gb*m/2^31)
            where[i][v] = (bucket * stride_bytes + rowbase) | (gs[v] << 31);
          }
        }
#pragma unroll
      for (int k = 0; k < KC; ++k)
        if (k < kcnt) {
#pragma unroll
          for (int v = 0; v < V; ++v) {
            const double y = fma((double)u[k][v], S, kRoundMagic);          // round to integer
            const long long q = __double_as_longlong(y) - __double_as_longlong(kRoundMagic);
            const long long nq = -q;
#pragma unroll
            for (int i = 0; i < LR; ++i)
              if (i < rcnt) {
                const uint32_t wv = where[i][v];
                unsigned long long* cell = reinterpret_cast<unsigned long long*>(
                    lds_raw + (wv & 0x7fffffffu)) + k;
                atomicAdd(cell, (unsigned long long)(((int32_t)wv < 0) ? nq : q));
              }
          }
        }
    } else {
      double* skd = reinterpret_cast<double*>(lds_raw);
      for (int i = 0; i < rcnt; ++i) {
        const uint32_t* cb = hc.c[rstart + i][0];
        const uint32_t* cs = hc.c[rstart + i][1];
        const int rowoff = i * prm.m;
#pragma unroll
        for (int v = 0; v < V; ++v) {
          const uint32_t j = (uint32_t)(j0 + v);
          const uint32_t gb = poly3(cb, j);
          const uint32_t gs = poly3(cs, j);
          const uint32_t bucket = __umulhi(gb << 1, (uint32_t)prm.m);
          const bool neg = (gs & 1u) != 0;                                    // odd -> -1
          double* cell = skd + (size_t)(rowoff + bucket) * prm.stride;
#pragma unroll
          for (int k = 0; k < KC; ++k)
            if (k < kcnt) atomicAdd(cell + k, (double)(neg ? -u[k][v] : u[k][v]));
        }
      }
    }
  }

  if (FX && rcnt > 0) {
    // a drift the integer cells cannot hold (or any drift at all when the sample saw none)
    const bool bad = bound > 0.0f ? !(amax < bound) : (amax > 0.0f);
    if (bad) prm.scale->overflow = 1;
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
    prm.part_np[((size_t)p * prm.K + kstart + k) * 2 + q] = s;
  }
  // ---- flush the LDS sketch to this workgroup's slice of the partial buffer -----------
  const int allcells = prm.l * prm.m;
  unsigned long long* out = reinterpret_cast<unsigned long long*>(prm.part_sk);
  for (int t = tid; t < kcnt * cells; t += kStateThreads) {
    const int k = t / cells, c = t - k * cells;
    out[((size_t)p * prm.K + kstart + k) * allcells + (size_t)rstart * prm.m + c] =
        sk[(size_t)c * prm.stride + k];
  }
}

// ---- how many coordinates can meet in one cell of one workgroup ------------------------
// Depends only on the hash, d and the partitioning, so it is counted once per context: the
// exact maximum, over workgroups, rows and buckets, of the number of coordinates of the
// workgroup's chunk that fall into the bucket.  It bounds the number of terms of any LDS cell.
__global__ void __launch_bounds__(kStateThreads)
cell_count_kernel(const HashCoef hc, int l, int m, long long d, long long chunk,
                  unsigned int* __restrict__ nmax) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  unsigned int* cnt = reinterpret_cast<unsigned int*>(lds_raw);
  __shared__ unsigned int shmax[kStateThreads / 64];
  const int p = blockIdx.x / l, i = blockIdx.x - p * l;
  for (int t = threadIdx.x; t < m; t += kStateThreads) cnt[t] = 0u;
  __syncthreads();
  const long long cbeg = (long long)p * chunk;
  long long cend = cbeg + chunk;
  if (cend > d) cend = d;
  for (long long j = cbeg + threadIdx.x; j < cend; j += kStateThreads) {
    const uint32_t gb = poly3(hc.c[i][0], (uint32_t)j);
    atomicAdd(cnt + __umulhi(gb << 1, (uint32_t)m), 1u);
  }
  __syncthreads();
  unsigned int mx = 0u;
  for (int t = threadIdx.x; t < m; t += kStateThreads) mx = max(mx, cnt[t]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mx = max(mx, (unsigned int)__shfl_down((int)mx, o, 64));
  if ((threadIdx.x & 63) == 0) shmax[threadIdx.x >> 6] = mx;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int t = 1; t < kStateThreads / 64; ++t) mx = max(mx, shmax[t]);
    atomicMax(nmax, mx);
  }
}
__global__ void clear_u32_kernel(unsigned int* p) { if (threadIdx.x == 0 && blockIdx.x == 0) *p = 0u; }

// ---- the per-call fixed-point scale ----------------------------------------------------
// Largest and mean |w_kj - w_t0_j| over an evenly spaced sample of coordinates of every worker.
template <typename T>
__global__ void __launch_bounds__(kSmallThreads)
scale_sample_kernel(const T* __restrict__ w, const float* __restrict__ w_t0, int K, long long d,
                    long long row_stride, int samples, float* __restrict__ part_max,
                    double* __restrict__ part_sum) {
  __shared__ float sh[kSmallThreads / 64];
  __shared__ double scratch[kSmallThreads / 64];
  float m = 0.0f;
  double sum = 0.0;
  const long long total = (long long)K * samples;
  for (long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x; t < total;
       t += (long long)gridDim.x * blockDim.x) {
    const int k = (int)(t / samples);
    const long long j = (t - (long long)k * samples) * d / samples;
    const float u = fabsf(Slab<T>::load_one(w + (long long)k * row_stride + j) - w_t0[j]);
    m = fmaxf(m, u);                           // fmaxf drops NaN
    if (u == u && u < 3.0e38f) sum += (double)u;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_down(m, o, 64));
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = m;
  const double tot = block_sum(sum, scratch);  // has the barriers sh needs
  if (threadIdx.x == 0) {
    for (int t = 1; t < kSmallThreads / 64; ++t) m = fmaxf(m, sh[t]);
    part_max[blockIdx.x] = m;
    part_sum[blockIdx.x] = tot;
  }
}

// The unit 2^-e of the integer cells.  With at most nmax terms per cell, |q| < 2^qbits keeps
// every cell below 2^62.  Drifts up to 2^12..2^13 times the sampled maximum are allowed for
// (the sample can miss the tail), which leaves qbits - 13 bits below the sampled maximum.  If
// the mean sampled magnitude would still get fewer than 17 of them, or the sample saw nothing
// usable, the call is sent down the fp64 path right away.
__global__ void scale_finalize_kernel(const float* __restrict__ part_max,
                                      const double* __restrict__ part_sum, int n, long long nsamples,
                                      const unsigned int* __restrict__ nmax,
                                      ScaleInfo* __restrict__ out) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  float amax = 0.0f;
  double sum = 0.0;
  for (int t = 0; t < n; ++t) { amax = fmaxf(amax, part_max[t]); sum += part_sum[t]; }
  ScaleInfo s;
  s.S = 1.0; s.invS = 1.0; s.bound = 0.0f; s.overflow = 0; s.pad[0] = 0; s.pad[1] = 0;
  if (amax > 0.0f && isfinite(amax)) {
    unsigned int terms = *nmax;
    int cb = 0;
    while (cb < 32 && (1ull << cb) <= (unsigned long long)terms) ++cb;    // terms < 2^cb
    int qbits = 62 - cb;
    if (qbits > 50) qbits = 50;                // the rounding trick needs |u * 2^e| < 2^51
    const int head = 13;
    const int ex = ilogbf(amax);               // 2^ex <= amax < 2^(ex+1)
    const int e = qbits - (ex + head);         // |u| < 2^(ex+head)  =>  |u * 2^e| < 2^qbits
    s.S = ldexp(1.0, e);
    s.invS = ldexp(1.0, -e);
    s.bound = (ex + head > 127) ? 3.0e38f : ldexpf(1.0f, ex + head);
    const double mean = sum / (double)nsamples;
    if (!(mean * s.S >= 131072.0)) s.overflow = 1;     // fewer than 17 bits for a typical drift
  }
  *out = s;
}

// state[k][s] = sum over partitions, in partition order, in fp64 (the integer partials are
// exact, so for them the order would not matter anyway).
__global__ void __launch_bounds__(kSmallThreads)
merge_kernel(const double* __restrict__ part_np, const void* __restrict__ part_sk,
             const ScaleInfo* __restrict__ scale, float* __restrict__ state, int K, int cells,
             int P) {
  const int S = 2 + cells;
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long long)K * S) return;
  const int k = (int)(idx / S), s = (int)(idx - (long long)k * S);
  double acc = 0.0;
  if (s < 2) {
    for (int p = 0; p < P; ++p) acc += part_np[((size_t)p * K + k) * 2 + s];
  } else {
    const int c = s - 2;
    if (scale->overflow == 0) {
      const long long* pi = reinterpret_cast<const long long*>(part_sk);
      for (int p = 0; p < P; ++p) acc += (double)pi[((size_t)p * K + k) * cells + c];
      acc *= scale->invS;
    } else {
      const double* pd = reinterpret_cast<const double*>(part_sk);
      for (int p = 0; p < P; ++p) acc += pd[((size_t)p * K + k) * cells + c];
    }
  }
  state[idx] = (float)acc;
}

// ----------------------------------------------------------------------------------------
// Algorithm 1 lines 7-8, one workgroup, all in fp64:
//   mean_k of the states;  row norms of the mean sketch;  M2 = their median (Section 3.1);
//   H_sketch = n - M2/(1+eps) (Thm 1);  H_linear = n - p^2 (Thm 2);  sync = H > theta.
// ----------------------------------------------------------------------------------------
__global__ void __launch_bounds__(1024)
estimate_kernel(const float* __restrict__ state, int K, int l, int m, int variants, double eps,
                double theta, double tie_tol, fda_estimate* __restrict__ out) {
  __shared__ double scratch[16];
  __shared__ double rows[FDA_MAX_SKETCH_ROWS];
  const int cells = (variants & FDA_VARIANT_SKETCH) ? l * m : 0;
  const int S = 2 + cells;
  const int tid = threadIdx.x;
  double vn = 0.0, vp = 0.0;
  for (int k = tid; k < K; k += blockDim.x) {
    vn += (double)state[(size_t)k * S];
    vp += (double)state[(size_t)k * S + 1];
  }
  const double sn = block_sum(vn, scratch);
  const double sp = block_sum(vp, scratch);
  if (cells) {
    for (int i = 0; i < l; ++i) {
      double acc = 0.0;
      for (int bkt = tid; bkt < m; bkt += blockDim.x) {
        double c = 0.0;
        for (int k = 0; k < K; ++k) c += (double)state[(size_t)k * S + 2 + i * m + bkt];
        c /= (double)K;
        acc += c * c;
      }
      const double r = block_sum(acc, scratch);
      if (tid == 0) rows[i] = r;
    }
  }
  if (tid == 0) {
    fda_estimate e;
    e.mean_sqnorm = sn / (double)K;
    e.mean_proj = 0.0; e.m2 = 0.0; e.h_linear = 0.0; e.h_sketch = 0.0;
    e.sync_linear = 0; e.sync_sketch = 0; e.near_tie_linear = 0; e.near_tie_sketch = 0;
    e.nonfinite = 0; e.reserved = 0;
    const double band = tie_tol * fmax(e.mean_sqnorm, fabs(theta));
    if (variants & FDA_VARIANT_LINEAR) {
      e.mean_proj = sp / (double)K;
      e.h_linear = e.mean_sqnorm - e.mean_proj * e.mean_proj;
      if (isfinite(e.h_linear)) {
        e.sync_linear = e.h_linear > theta ? 1 : 0;
        e.near_tie_linear = fabs(e.h_linear - theta) <= band ? 1 : 0;
      } else {
        e.sync_linear = 1; e.nonfinite = 1;
      }
    }
    if (cells) {
      // median of l values: insertion sort, then middle (even l: mean of the two middle)
      double r[FDA_MAX_SKETCH_ROWS];
      for (int i = 0; i < l; ++i) {
        double v = rows[i];
        int q = i;
        while (q > 0 && !(r[q - 1] <= v)) { r[q] = r[q - 1]; --q; }
        r[q] = v;
      }
      e.m2 = (l & 1) ? r[l / 2] : 0.5 * (r[l / 2 - 1] + r[l / 2]);
      e.h_sketch = e.mean_sqnorm - e.m2 / (1.0 + eps);
      if (isfinite(e.h_sketch)) {
        e.sync_sketch = e.h_sketch > theta ? 1 : 0;
        e.near_tie_sketch = fabs(e.h_sketch - theta) <= band ? 1 : 0;
      } else {
        e.sync_sketch = 1; e.nonfinite = 1;
      }
    }
    *out = e;
  }
}

// ----------------------------------------------------------------------------------------
// Algorithm 1 line 9: read the K rows once, average in fp32 in worker order, write the
// average to every row, to w_t0, and the old w_t0 to w_prev.
// ----------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(kSmallThreads)
sync_kernel(T* __restrict__ w, float* __restrict__ w_t0, float* __restrict__ w_prev,
            const int32_t* __restrict__ pred, int K, long long d, long long row_stride, int vec_ok) {
  constexpr int V = Slab<T>::V;
  if (pred != nullptr && *pred == 0) return;
  const float kf = (float)K;
  const long long nvec = (d + V - 1) / V;
  for (long long vi = (long long)blockIdx.x * blockDim.x + threadIdx.x; vi < nvec;
       vi += (long long)gridDim.x * blockDim.x) {
    const long long j0 = vi * V;
    float acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = 0.0f;
    if (vec_ok && j0 + V <= d) {
#pragma unroll 4
      for (int k = 0; k < K; ++k) {
        float x[V];
        Slab<T>::load_vec(w + (long long)k * row_stride + j0, x);
#pragma unroll
        for (int v = 0; v < V; ++v) acc[v] += x[v];
      }
#pragma unroll
      for (int v = 0; v < V; ++v) acc[v] = acc[v] / kf;
      if (w_prev != nullptr) {
        float old[V];
        load_f32_vec<V>(w_t0 + j0, old);
        store_f32_vec<V>(w_prev + j0, old);
      }
      store_f32_vec<V>(w_t0 + j0, acc);
#pragma unroll 4
      for (int k = 0; k < K; ++k) Slab<T>::store_vec(w + (long long)k * row_stride + j0, acc);
    } else {
      for (int v = 0; v < V; ++v) {
        const long long j = j0 + v;
        if (j >= d) break;
        float a = 0.0f;
        for (int k = 0; k < K; ++k) a += Slab<T>::load_one(w + (long long)k * row_stride + j);
        a = a / kf;
        if (w_prev != nullptr) w_prev[j] = w_t0[j];
        w_t0[j] = a;
        for (int k = 0; k < K; ++k) Slab<T>::store_one(w + (long long)k * row_stride + j, a);
      }
    }
  }
}

// ----------------------------------------------------------------------------------------
// Section 3.2: xi = (w_t0 - w_prev) / ||w_t0 - w_prev||.  Pass 1: per-workgroup partial of
// the squared norm; pass 2: every workgroup re-sums the partials in the same fixed order
// and scales its share of the difference.
// ----------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kSmallThreads)
xi_norm_kernel(const float* __restrict__ w_t0, const float* __restrict__ w_prev,
               const int32_t* __restrict__ pred, long long d, double* __restrict__ partial) {
  __shared__ double scratch[kSmallThreads / 64];
  if (pred != nullptr && *pred == 0) return;
  double acc = 0.0;
  const long long step = (long long)gridDim.x * blockDim.x;
  long long j = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  while (j < d) {
    float part = 0.0f;                       // a short fp32 run, then fp64
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      if (j < d) { const float df = w_t0[j] - w_prev[j]; part = fmaf(df, df, part); }
      j += step;
    }
    acc += (double)part;
  }
  const double s = block_sum(acc, scratch);
  if (threadIdx.x == 0) partial[blockIdx.x] = s;
}

__global__ void __launch_bounds__(kSmallThreads)
xi_scale_kernel(const float* __restrict__ w_t0, const float* __restrict__ w_prev,
                float* __restrict__ xi, const int32_t* __restrict__ pred, long long d,
                const double* __restrict__ partial, int npartial) {
  __shared__ double scratch[kSmallThreads / 64];
  __shared__ float scale_sh;
  if (pred != nullptr && *pred == 0) return;
  double acc = 0.0;
  for (int t = threadIdx.x; t < npartial; t += blockDim.x) acc += partial[t];
  const double tot = block_sum(acc, scratch);
  if (threadIdx.x == 0) {
    const double nrm = sqrt(tot);
    scale_sh = (nrm > 0.0 && isfinite(nrm)) ? (float)(1.0 / nrm) : 0.0f;
  }
  __syncthreads();
  const float scale = scale_sh;
  for (long long j = (long long)blockIdx.x * blockDim.x + threadIdx.x; j < d;
       j += (long long)gridDim.x * blockDim.x) {
    const float df = w_t0[j] - w_prev[j];
    xi[j] = (scale == 0.0f) ? 0.0f : df * scale;
  }
}

}  // namespace fda
