// Device code of the FDA monitor for gfx950 (wave64): everything except the state kernel.
// Included by fda_api.hip only.
//
//   hash_table_kernel, cell_count_kernel   once per context: the tabulated hash and the largest
//                    number of coordinates a workgroup can put into one sketch cell
//   scale_kernel     per call: the fixed-point unit of the integer sketch cells
//   merge_kernel     fixed-order fp64 sum of the per-workgroup partials -> state[K][S]
//   merge_mean_kernel  the same for the partials of mean_state_kernel -> mean_state[S]
//   estimate_kernel  Algorithm 1 lines 7-8: mean state, M2, H (Thm 1, Thm 2), decision
//   sync_kernel      Algorithm 1 line 9: fused mean over workers + broadcast to all rows (+ the squared
//                    norm of the model change, for the refresh of xi)
//   sync_from_mean_kernel  the same from an average model that is already there, with xi
//   xi_norm_kernel / xi_scale_kernel   Section 3.2: the normalized model difference
#pragma once
#include "fda_kernels.hpp"

namespace fda {

// ---- the hash, tabulated once per context (Section 3.1 sketch; hash family: two cubics mod 2^31 - 1
// per row).  Per row group r and coordinate j one record of `words` 16-bit words; a record packs,
// lowest bits first, one field of `fb` bits per row slot of the group: bucket + m for sign -1, bucket
// for sign +1 (below 2 m, which fits: field_bits_for).  Slots past the group's last row (and whole
// records past d) hold a value below kDummyCells: the state kernels send those additions to a dummy
// region (whatever bucket and sign they decode from it, the bucket stays below kDummyCells).
// Layout [row group][block of 256 coordinates][dwords in load order]: the 2 * words dwords of the 4
// records that a lane of the state kernels loads together are placed where load_rec_block() reads
// them.  One thread writes one lane's share; a workgroup of kSmallThreads covers 4 blocks.
//
// grp >= 2: placed rows (see kPlacedFieldBits) for a state kernel of KC worker slots.  The rows of the
// group come in placement groups of grp; slot a of a placement group of n rows holds row (a + rot) % n of
// it, field = that row's number in the group times the buckets a row takes up (cells32_row_buckets) plus
// the plain field, and rot is chosen per coordinate so that the additions one instruction of the state
// kernel issues collide as little as the choice allows.  The model: the 16 lanes 16 g .. 16 g + 15 of a
// wave are served together, instruction (v, slot) takes coordinate 4 lane + v of the block from each, and
// two of them collide when the 8-byte words they address lie a multiple of 128 bytes apart: the word
// index of a field (cells32_bucket_word / 2) modulo 16 is its class.  Cost of an instruction = the largest number of lanes in one class; per (16 lanes, v,
// placement group) one thread places the 16 coordinates one after the other where the sum over the
// slots grows least, then revisits each twice.  The result depends only on the hash and the shape.
constexpr int kPlaceSweeps = 3;
__global__ void __launch_bounds__(kSmallThreads)
hash_table_kernel(const HashCoef hc, int l, int R, int slots, int m, int fb, int words, int grp, int KC,
                  long long d, long long dpad, uint16_t* __restrict__ table) {
  __shared__ uint16_t fld[kSmallThreads][4][8];                // plain fields, by thread, coordinate, row
  __shared__ uint8_t rotsel[kSmallThreads][4][4];              // chosen rotation, by thread, coordinate, placement group
  __shared__ uint8_t hist[kSmallThreads / 64][16][8][16];      // by wave, (16 lanes, v), slot, class
  const int r = blockIdx.y;
  const int tid = threadIdx.x;
  const long long j4 = ((long long)blockIdx.x * blockDim.x + tid) * 4;
  int rstart, rcnt;
  group_range(l, R, r, &rstart, &rcnt);
  const bool placed = grp >= 2;
  const uint32_t mrow = placed ? (uint32_t)cells32_row_buckets(2 * m, KC) : 0u;   // buckets per LDS row, as a field counts them
  for (int q = 0; q < 4; ++q) {
    const long long j = j4 + q;
    for (int i = 0; i < slots; ++i) {
      uint32_t f = (uint32_t)(j + 17 * i) & (uint32_t)(kDummyCells - 1);
      if (i < rcnt && j < d) {
        const uint32_t h = hash_entry(hc, rstart + i, (uint32_t)j, (uint32_t)m);
        f = (h & 0x7fffu) + (h >> 15) * (uint32_t)m;           // bucket + m * (sign is -1)
      }
      fld[tid][q][i] = (uint16_t)f;
    }
  }
  if (placed) {                                                // (uniform over the workgroup)
    const int ngroups = (rcnt + grp - 1) / grp;                // at most 4: grp >= 2, at most 8 rows
    for (int q = 0; q < 4; ++q)
      for (int g = 0; g < 4; ++g) rotsel[tid][q][g] = 0;
    __syncthreads();
    const int wave = tid >> 6, lane = tid & 63;
    // problem (16 lanes gi, coordinate v) = lane & 15; placement groups lane >> 4, lane >> 4 + 4, ...
    const int prob = lane & 15, gi = prob >> 2, v = prob & 3;
    for (int g = lane >> 4; g < ngroups; g += 4) {
      const int g0 = g * grp, n = rcnt - g0 < grp ? rcnt - g0 : grp;
      if (n < 2) continue;
      uint8_t (*h)[16] = &hist[wave][prob][g0];                // n slots of 16 classes
      for (int a = 0; a < n; ++a)
        for (int c = 0; c < 16; ++c) h[a][c] = 0;
      const int member0 = wave * 64 + gi * 16;
      // class of member t's entry of row `row` (within the placement group)
      auto cls = [&](int t, int row) {
        const uint32_t field = (uint32_t)row * mrow + fld[member0 + t][v][g0 + row];
        return (int)((cells32_bucket_word(field, KC) >> 1) & 15u);
      };
      for (int sweep = 0; sweep < kPlaceSweeps; ++sweep) {
        for (int t = 0; t < 16; ++t) {
          if (sweep > 0) {
            const int cur = rotsel[member0 + t][v][g];
            for (int a = 0; a < n; ++a) { int row = a + cur; if (row >= n) row -= n; h[a][cls(t, row)] -= 1; }
          }
          int mx[8];
          for (int a = 0; a < n; ++a) {
            int top = 0;
            for (int c = 0; c < 16; ++c) top = h[a][c] > top ? h[a][c] : top;
            mx[a] = top;
          }
          int best = 1 << 30, brot = 0;
          for (int rot = 0; rot < n; ++rot) {
            int cost = 0;
            for (int a = 0; a < n; ++a) {
              int row = a + rot; if (row >= n) row -= n;
              const int after = h[a][cls(t, row)] + 1;
              cost += after > mx[a] ? after : mx[a];
            }
            if (cost < best) { best = cost; brot = rot; }
          }
          rotsel[member0 + t][v][g] = (uint8_t)brot;
          for (int a = 0; a < n; ++a) { int row = a + brot; if (row >= n) row -= n; h[a][cls(t, row)] += 1; }
        }
      }
    }
    __syncthreads();
  }
  if (j4 >= dpad) return;
  uint32_t dw[16];                                             // 4 records of at most 8 words
  for (int t = 0; t < 16; ++t) dw[t] = 0u;
  for (int q = 0; q < 4; ++q) {
    unsigned long long bits[3] = {0ull, 0ull, 0ull};          // slots * fb <= 8 * 16 bits
    for (int i = 0; i < slots; ++i) {
      unsigned long long f = fld[tid][q][i];
      if (placed && i < rcnt) {
        const int g = i / grp, g0 = g * grp, n = rcnt - g0 < grp ? rcnt - g0 : grp;
        int row = i - g0 + rotsel[tid][q][g]; if (row >= n) row -= n;
        f = (unsigned long long)((uint32_t)row * mrow + fld[tid][q][g0 + row]);
      }
      const int pos = i * fb, idx = pos >> 6, sh = pos & 63;
      bits[idx] |= f << sh;
      if (sh + fb > 64) bits[idx + 1] |= f >> (64 - sh);
    }
    for (int t = 0; t < words; ++t) {
      const uint32_t w16 = (uint32_t)(bits[t >> 2] >> (16 * (t & 3))) & 0xffffu;
      const int w = q * words + t;                             // 16-bit word of the lane's share
      dw[w >> 1] |= w16 << (16 * (w & 1));
    }
  }
  const int N = 2 * words, n4 = N / 4, n2 = (N % 4) / 2;
  const int lane = (int)(j4 >> 2) & 63;
  uint32_t* blk = reinterpret_cast<uint32_t*>(table) +
                  ((size_t)r * (size_t)(dpad / kRecBlockCoords) + (size_t)(j4 / kRecBlockCoords)) * (size_t)(64 * N);
  for (int t = 0; t < N; ++t) {
    int off;
    if (t < 4 * n4) off = ((t >> 2) * 64 + lane) * 4 + (t & 3);
    else if (t < 4 * n4 + 2 * n2) off = n4 * 256 + lane * 2 + (t - 4 * n4);
    else off = n4 * 256 + n2 * 128 + lane;
    blk[off] = dw[t];
  }
}

// ---- how many coordinates can meet in one cell of one workgroup ------------------------
// Depends only on the hash, d and the partitioning, so it is counted once per context: the
// exact maximum, over workgroups, rows and buckets, of the number of coordinates of the
// workgroup's chunk that fall into the bucket.  It bounds the number of terms of any LDS cell.
__global__ void __launch_bounds__(kStateThreads)
cell_count_kernel(const HashCoef hc, int l, int m, int split, long long d, long long chunk,
                  unsigned int* __restrict__ nmax) {   // nmax: the entry to raise
  // split: the pass keeps the two signs of a bucket in cells of their own (sign-split rows)
  extern __shared__ __align__(16) unsigned char lds_raw[];
  unsigned int* cnt = reinterpret_cast<unsigned int*>(lds_raw);
  __shared__ unsigned int shmax[kStateThreads / 64];
  const int p = blockIdx.x / l, i = blockIdx.x - p * l;
  const int ncell = split ? 2 * m : m;
  for (int t = threadIdx.x; t < ncell; t += kStateThreads) cnt[t] = 0u;
  __syncthreads();
  const long long cbeg = (long long)p * chunk;
  long long cend = cbeg + chunk;
  if (cend > d) cend = d;
  for (long long j = cbeg + threadIdx.x; j < cend; j += kStateThreads) {
    const uint32_t h = hash_entry(hc, i, (uint32_t)j, (uint32_t)m);
    atomicAdd(cnt + (h & 0x7fffu) + ((split && (h >> 15)) ? m : 0), 1u);
  }
  __syncthreads();
  unsigned int mx = 0u;
  for (int t = threadIdx.x; t < ncell; t += kStateThreads) mx = max(mx, cnt[t]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mx = max(mx, (unsigned int)__shfl_down((int)mx, o, 64));
  if ((threadIdx.x & 63) == 0) shmax[threadIdx.x >> 6] = mx;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int t = 1; t < kStateThreads / 64; ++t) mx = max(mx, shmax[t]);
    atomicMax(nmax, mx);
  }
}
__global__ void clear_u32_kernel(unsigned int* p, int n) {
  if (blockIdx.x == 0 && (int)threadIdx.x < n) p[threadIdx.x] = 0u;
}

// ---- the per-call fixed-point scale ----------------------------------------------------
// The units of the integer cells.
// 64-bit cells: with at most nmax[1] terms per cell, |q| < 2^qbits keeps every cell below 2^62.
// Drifts up to 2^12..2^13 times the sampled maximum are allowed for (the sample can miss the
// tail), which leaves qbits - 13 bits below the sampled maximum.  If the mean sampled magnitude
// would still get fewer than 17 of them, or the sample saw nothing usable, the call is sent
// down the fp64 path right away.
// 32-bit cells: the mean sampled magnitude maps to [2^18, 2^19) -- every term is rounded by at
// most 2^-19 of the mean |u| -- and single drifts may reach 2^30, i.e. 2048..4096 times the mean
// (a Student-t(3) tail over 3e9 draws reaches about 1400 times).  A cell wraps only if its sum
// leaves (-2^31, 2^31), which for sums of up to a few thousand such terms does not happen, and
// if it does it is noticed.  Cells that can collect more than 4096 terms get one bit less;
// beyond 16384 terms the call goes to the 64-bit pass.
__device__ inline ScaleInfo choose_scale(float amax, double mean, const unsigned int* nmax) {
  ScaleInfo s;
  s.S64 = 1.0; s.invS64 = 1.0; s.invS32 = 1.0; s.S32 = 1.0f;
  s.bound32 = 0.0f; s.bound64 = 0.0f; s.flag32 = 0; s.overflow64 = 0;
  s.flagm = 0; s.invSm = 1.0; s.Sm = 1.0f; s.boundm = 0.0f;
  if (amax > 0.0f && isfinite(amax) && mean > 0.0) {
    // ---- 64-bit cells
    int cb = 0;
    while (cb < 32 && (1ull << cb) <= (unsigned long long)nmax[1]) ++cb;   // terms < 2^cb
    int qbits = 62 - cb;
    if (qbits > 50) qbits = 50;                // the rounding trick needs |u * 2^e| < 2^51
    const int head = 13;
    const int ex = ilogbf(amax);               // 2^ex <= amax < 2^(ex+1)
    const int e = qbits - (ex + head);         // |u| < 2^(ex+head)  =>  |u * 2^e| < 2^qbits
    s.S64 = ldexp(1.0, e);
    s.invS64 = ldexp(1.0, -e);
    s.bound64 = (ex + head > 127) ? 3.0e38f : ldexpf(1.0f, ex + head);
    if (!(mean * s.S64 >= 131072.0)) { s.overflow64 = 1; s.flag32 = 1; }   // < 17 bits for a typical drift
    // ---- 32-bit cells
    int cb32 = 0;
    while (cb32 < 32 && (1ull << cb32) <= (unsigned long long)nmax[0]) ++cb32;
    const int shrink = cb32 > 12 ? (cb32 - 12 + 1) / 2 : 0;
    const int em = ilogb(mean);                // 2^em <= mean < 2^(em+1)
    // ---- mean-state kernel: 32-bit terms, 64-bit sums, the mean magnitude at [2^18, 2^19)
    const int emn = 18 - em;
    if (emn > 120 || emn < -120) {
      s.flagm = 1;
    } else {
      s.Sm = ldexpf(1.0f, emn);
      s.invSm = ldexp(1.0, -emn);
      s.boundm = (30 - emn > 127) ? 3.0e38f : ldexpf(1.0f, 30 - emn);
      if (!(amax < s.boundm)) s.flagm = 1;
    }
    const int e32 = 18 - shrink - em;
    if (e32 > 120 || e32 < -120 || shrink > 1) {
      s.flag32 = 1;
    } else {
      s.S32 = ldexpf(1.0f, e32);
      s.invS32 = ldexp(1.0, -e32);
      s.bound32 = (30 - e32 > 127) ? 3.0e38f : ldexpf(1.0f, 30 - e32);
      if (!(amax < s.bound32)) s.flag32 = 1;   // the sample already holds a drift too large
    }
  }
  return s;
}

// Largest and mean |w_kj - w_t0_j| over `samples` coordinates of every worker: evenly spaced runs
// of 8 consecutive coordinates (a run shares its cache lines, so the scattered reads cost an
// eighth of what single coordinates would).  A thread takes one sampled coordinate and every
// slices-th worker (the loads of one thread are independent HBM misses: about eight per thread,
// several in flight); per-workgroup maximum and sum;
// the workgroup that finishes last combines the per-workgroup results in a fixed order, chooses
// the scales and clears the flags.  `ticket` counts finished workgroups and is left at zero.
constexpr int kScaleMaxSlices = 8;          // a sampled coordinate's workers are split over 1..8 threads

template <typename T>
__global__ void __launch_bounds__(kSmallThreads)
scale_kernel(const T* __restrict__ w, const float* __restrict__ w_t0, int K, long long d,
             long long row_stride, int samples, int slices, float* __restrict__ part_max,
             double* __restrict__ part_sum, unsigned int* __restrict__ ticket,
             const unsigned int* __restrict__ nmax, ScaleInfo* __restrict__ out) {
  __shared__ float sh[kSmallThreads / 64];
  __shared__ double scratch[kSmallThreads / 64];
  __shared__ int last;
  float m = 0.0f;
  double sum = 0.0;
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  const int smp = t / slices, slice = t - smp * slices;
  if (smp < samples) {
    // samples is a multiple of 8 and at most d, or equal to d (then every coordinate is taken)
    const long long j = (samples & 7) ? (long long)smp
                                      : (long long)(smp >> 3) * (d / (samples >> 3)) + (smp & 7);
    const float base = w_t0[j];
    float part = 0.0f;
#pragma unroll 4
    for (int k = slice; k < K; k += slices) {
      const float u = fabsf(Slab<T>::load_one(w + (long long)k * row_stride + j) - base);
      m = fmaxf(m, u);                         // fmaxf drops NaN
      if (u == u && u < 3.0e38f) part += u;
    }
    sum = (double)part;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_down(m, o, 64));
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = m;
  const double tot = block_sum(sum, scratch);  // has the barriers sh needs
  if (threadIdx.x == 0) {
    for (int q = 1; q < kSmallThreads / 64; ++q) m = fmaxf(m, sh[q]);
    part_max[blockIdx.x] = m;
    part_sum[blockIdx.x] = tot;
    __threadfence();
    last = (atomicAdd(ticket, 1u) == gridDim.x - 1) ? 1 : 0;
  }
  __syncthreads();
  if (!last) return;
  __threadfence();
  if (threadIdx.x < 64) {                      // lane q takes partials q, q + 64, ...
    float am = 0.0f;
    double sm = 0.0;
    for (int q = threadIdx.x; q < (int)gridDim.x; q += 64) {
      am = fmaxf(am, reinterpret_cast<volatile float*>(part_max)[q]);
      sm += reinterpret_cast<volatile double*>(part_sum)[q];
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) am = fmaxf(am, __shfl_down(am, o, 64));
    sm = wave_sum(sm);
    if (threadIdx.x == 0) {
      *out = choose_scale(am, sm / ((double)samples * K), nmax);
      *ticket = 0u;
    }
  }
}

// state[k][s] = sum over the partitions in fp64.  A workgroup handles 32 consecutive state
// entries; eight lanes per entry each sum every eighth partition and the eight sums are added
// in slice order: a fixed shape (and the integer partials are exact anyway).  The scalar
// components always come from the first pass (P32 partitions); the sketch partials from
// whichever pass was the last to run.
__global__ void __launch_bounds__(kSmallThreads)
merge_kernel(const double* __restrict__ part_np, const void* __restrict__ part_sk,
             const ScaleInfo* __restrict__ scale, float* __restrict__ state, int K, int cells,
             int P32, int P64) {
  __shared__ double sh[8][32];
  const int S = 2 + cells;
  const int o = threadIdx.x & 31, slice = threadIdx.x >> 5;
  const long long idx = (long long)blockIdx.x * 32 + o;
  const bool live = idx < (long long)K * S;
  double acc = 0.0, unit = 1.0;
  if (live) {
    const int k = (int)(idx / S), s = (int)(idx - (long long)k * S);
    if (s < 2) {
#pragma unroll 8
      for (int p = slice; p < P32; p += 8) acc += part_np[((size_t)p * K + k) * 2 + s];
    } else {
      const int c = s - 2;
      if (scale->overflow64 != 0) {
        const double* pd = reinterpret_cast<const double*>(part_sk);
#pragma unroll 8
        for (int p = slice; p < P64; p += 8) acc += pd[((size_t)p * K + k) * cells + c];
      } else {
        const bool narrow = scale->flag32 == 0;
        const int P = narrow ? P32 : P64;
        unit = narrow ? scale->invS32 : scale->invS64;
        const long long* pi = reinterpret_cast<const long long*>(part_sk);
#pragma unroll 8
        for (int p = slice; p < P; p += 8) acc += (double)pi[((size_t)p * K + k) * cells + c];
      }
    }
  }
  sh[slice][o] = acc;
  __syncthreads();
  if (live && slice == 0) {
    double t = 0.0;
#pragma unroll
    for (int q = 0; q < 8; ++q) t += sh[q][o];
    state[idx] = (float)(t * unit);
  }
}

// mean_state[s] = (sum over the partitions) / K, for the partials of mean_state_kernel: the two
// scalar sums in fp64, the sketch cells as 64-bit integers in units of 1/Sm (or fp64 when the
// call went down the fp64 path).  Same fixed shape as merge_kernel.  One entry past the state,
// the summed squared norm of the model change goes to *dnorm (for fda_sync_from_mean).
__global__ void __launch_bounds__(kSmallThreads)
merge_mean_kernel(const double* __restrict__ part_np, const void* __restrict__ part_sk,
                  const ScaleInfo* __restrict__ scale, float* __restrict__ mean_state,
                  double* __restrict__ dnorm, int K, int cells, int P) {
  __shared__ double sh[8][32];
  const int S = 2 + cells;
  const int o = threadIdx.x & 31, slice = threadIdx.x >> 5;
  const int s = blockIdx.x * 32 + o;
  const bool live = s <= S;
  double acc = 0.0, unit = 1.0;
  if (live) {
    if (s < 2 || s == S) {
      const int q = s < 2 ? s : 2;
#pragma unroll 8
      for (int p = slice; p < P; p += 8) acc += part_np[(size_t)p * 3 + q];
    } else {
      const int c = s - 2;
      if (scale->flagm != 0) {
        const double* pd = reinterpret_cast<const double*>(part_sk);
#pragma unroll 8
        for (int p = slice; p < P; p += 8) acc += pd[(size_t)p * cells + c];
      } else {
        unit = scale->invSm;
        const long long* pi = reinterpret_cast<const long long*>(part_sk);
        long long isum = 0;                       // exact
#pragma unroll 8
        for (int p = slice; p < P; p += 8) isum += pi[(size_t)p * cells + c];
        acc = (double)isum;
      }
    }
  }
  sh[slice][o] = acc;
  __syncthreads();
  if (live && slice == 0) {
    double t = 0.0;
#pragma unroll
    for (int q = 0; q < 8; ++q) t += sh[q][o];
    if (s == S) *dnorm = t;
    else mean_state[s] = (float)(t * unit / (double)K);
  }
}

// ----------------------------------------------------------------------------------------
// Algorithm 1 lines 7-8, all in fp64:
//   mean_k of the states;  row norms of the mean sketch;  M2 = their median (Section 3.1);
//   H_sketch = n - M2/(1+eps) (Thm 1);  H_linear = n - p^2 (Thm 2);  sync = H > theta.
// Workgroup b takes 256 consecutive cells of one sketch row (one cell per thread: mean over the
// K workers, squared, summed over the workgroup); workgroup 0 also takes the scalar components.
// The workgroup that finishes last adds the per-workgroup sums of every row in workgroup order,
// takes the median and writes the result.  `ticket` counts finished workgroups and is left at 0.
// ----------------------------------------------------------------------------------------
constexpr int kEstCols = kSmallThreads;      // cells per workgroup

__global__ void __launch_bounds__(kSmallThreads)
estimate_kernel(const float* __restrict__ state, int K, int l, int m, int variants, double eps,
                double theta, double tie_tol, double* __restrict__ part, unsigned int* __restrict__ ticket,
                const ScaleInfo* __restrict__ scale, int mean_mode, fda_estimate* __restrict__ out) {
  __shared__ double scratch[kSmallThreads / 64];
  __shared__ int last;
  const int cells = (variants & FDA_VARIANT_SKETCH) ? l * m : 0;
  const int S = 2 + cells;
  const int bpr = (m + kEstCols - 1) / kEstCols;     // workgroups per sketch row
  const int tid = threadIdx.x;
  // part[0], part[1]: sums of the two scalar components; part[2 + b]: workgroup b's row sum
  if (cells) {
    const int i = blockIdx.x / bpr, col = (blockIdx.x - i * bpr) * kEstCols + tid;
    double sq = 0.0;
    if (col < m) {
      double c = 0.0;
#pragma unroll 8
      for (int k = 0; k < K; ++k) c += (double)state[(size_t)k * S + 2 + i * m + col];
      c /= (double)K;
      sq = c * c;
    }
    const double r = block_sum(sq, scratch);
    if (tid == 0) part[2 + blockIdx.x] = r;
  }
  if (blockIdx.x == 0) {
    double vn = 0.0, vp = 0.0;
    for (int k = tid; k < K; k += blockDim.x) {
      vn += (double)state[(size_t)k * S];
      vp += (double)state[(size_t)k * S + 1];
    }
    const double sn = block_sum(vn, scratch);
    const double sp = block_sum(vp, scratch);
    if (tid == 0) { part[0] = sn; part[1] = sp; }
  }
  if (tid == 0) {
    __threadfence();
    last = (atomicAdd(ticket, 1u) == gridDim.x - 1) ? 1 : 0;
  }
  __syncthreads();
  if (!last || tid != 0) return;
  __threadfence();
  const volatile double* vpart = part;
  fda_estimate e;
  e.mean_sqnorm = vpart[0] / (double)K;
  e.mean_proj = 0.0; e.m2 = 0.0; e.h_linear = 0.0; e.h_sketch = 0.0;
  e.sync_linear = 0; e.sync_sketch = 0; e.near_tie_linear = 0; e.near_tie_sketch = 0;
  e.nonfinite = 0;
  // which kind of sketch cell the last state pass used (scale: its record, or NULL)
  e.state_path = -1;
  if (cells && scale != nullptr)
    e.state_path = mean_mode ? (scale->flagm ? 1 : 0) : (scale->overflow64 ? 2 : (scale->flag32 ? 1 : 0));
  const double band = tie_tol * fmax(e.mean_sqnorm, fabs(theta));
  if (variants & FDA_VARIANT_LINEAR) {
    e.mean_proj = vpart[1] / (double)K;
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
      double v = 0.0;
      for (int b = 0; b < bpr; ++b) v += vpart[2 + i * bpr + b];
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
  *ticket = 0u;
}

// ----------------------------------------------------------------------------------------
// Algorithm 1 line 9: read the K rows once, average in fp32 in worker order, write the
// average to every row, to w_t0, and the old w_t0 to w_prev.
//
// A lane owns 4 consecutive coordinates (16 bytes of fp32, 8 bytes of bf16), so every load and store
// instruction of a wave covers whole cache lines, and workgroup b owns the contiguous range of such
// vectors [b * per, (b + 1) * per), a few trips long (the host launches one workgroup per 1024
// vectors): workgroups that run at the same time work on neighbouring addresses of every row, which
// is what keeps the K + 2 interleaved read and write streams efficient in DRAM (ranges of hundreds
// of KiB per workgroup cost a bf16 slab's pass a third of its rate).  STREAM: every byte is read once
// and written once, so loads and stores carry the nontemporal hint -- chosen by the host for slabs
// too large to stay in the memory-side cache, where it gains 3-8 %; small slabs lose by it.  (With 8
// coordinates per lane the fp32 vectors of a bf16 slab's pass become two 16-byte accesses 32 bytes
// apart: half cache lines per instruction, which the hinted stores pay for twice.)
// ----------------------------------------------------------------------------------------
constexpr bool kSyncContiguous = true;
constexpr int kSyncV = 4;                    // coordinates per lane in the synchronization kernels

template <typename VecT, bool NT>
__device__ __forceinline__ void store_vec_hint(void* p, VecT v) {
  if constexpr (NT) __builtin_nontemporal_store(v, reinterpret_cast<VecT*>(p));
  else *reinterpret_cast<VecT*>(p) = v;
}
// 4 slab elements at p as floats, and back
template <bool NT>
__device__ __forceinline__ void load_slab4(const float* p, float (&x)[4]) {
  const f32x4 t = load_vec_hint<f32x4, NT>(p);
  x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
}
template <bool NT>
__device__ __forceinline__ void load_slab4(const bf16_t* p, float (&x)[4]) {
  const u32x2_h t = load_vec_hint<u32x2_h, NT>(p);
  x[0] = __uint_as_float(t.x << 16); x[1] = __uint_as_float(t.x & 0xffff0000u);
  x[2] = __uint_as_float(t.y << 16); x[3] = __uint_as_float(t.y & 0xffff0000u);
}
template <bool NT>
__device__ __forceinline__ void store_f32x4(float* p, const float (&x)[4]) {
  const f32x4 t = {x[0], x[1], x[2], x[3]};
  store_vec_hint<f32x4, NT>(p, t);
}
// what a slab row stores for 4 averaged values: the fp32 values, or their bf16 roundings (packed)
struct RowVec4 { uint32_t w[4]; };
__device__ __forceinline__ RowVec4 pack_row4(const float (&x)[4], const float*) {
  RowVec4 r;
  r.w[0] = __float_as_uint(x[0]); r.w[1] = __float_as_uint(x[1]);
  r.w[2] = __float_as_uint(x[2]); r.w[3] = __float_as_uint(x[3]);
  return r;
}
__device__ __forceinline__ RowVec4 pack_row4(const float (&x)[4], const bf16_t*) {
  RowVec4 r;
  r.w[0] = f32_to_bf16_rne(x[0]) | (f32_to_bf16_rne(x[1]) << 16);
  r.w[1] = f32_to_bf16_rne(x[2]) | (f32_to_bf16_rne(x[3]) << 16);
  r.w[2] = 0u; r.w[3] = 0u;
  return r;
}
template <bool NT>
__device__ __forceinline__ void store_row4(float* p, const RowVec4& r) {
  const u32x4 t = {r.w[0], r.w[1], r.w[2], r.w[3]};
  store_vec_hint<u32x4, NT>(p, t);
}
template <bool NT>
__device__ __forceinline__ void store_row4(bf16_t* p, const RowVec4& r) {
  const u32x2_h t = {r.w[0], r.w[1]};
  store_vec_hint<u32x2_h, NT>(p, t);
}

// the range of vectors a workgroup walks, and its stride
struct SyncRange { long long beg, end, step; };
__device__ __forceinline__ SyncRange sync_range(long long nvec) {
  SyncRange r;
  if (kSyncContiguous) {
    const long long per = (nvec + gridDim.x - 1) / gridDim.x;
    r.beg = (long long)blockIdx.x * per;
    r.end = r.beg + per < nvec ? r.beg + per : nvec;
    r.step = blockDim.x;
  } else {
    r.beg = (long long)blockIdx.x * blockDim.x;
    r.end = nvec;
    r.step = (long long)gridDim.x * blockDim.x;
  }
  return r;
}

template <typename T, bool STREAM>
__global__ void __launch_bounds__(kSmallThreads)
sync_kernel(T* __restrict__ w, float* __restrict__ w_t0, float* __restrict__ w_prev,
            const int32_t* __restrict__ pred, int K, long long d, long long row_stride, int vec_ok,
            double* __restrict__ norm_part) {
  // norm_part != NULL: entry [workgroup] receives the workgroup's share of ||new w_t0 - old w_t0||^2
  // (fp32 squares of four coordinates, then fp64), which saves the refresh of xi its pass over both vectors
  constexpr int V = kSyncV;
  __shared__ double scratch[kSmallThreads / 64];
  if (pred != nullptr && *pred == 0) return;
  double nacc = 0.0;
  const float kf = (float)K;
  const SyncRange rg = sync_range((d + V - 1) / V);
  for (long long vi = rg.beg + threadIdx.x; vi < rg.end; vi += rg.step) {
    const long long j0 = vi * V;
    float acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = 0.0f;
    if (vec_ok && j0 + V <= d) {
#pragma unroll 8
      for (int k = 0; k < K; ++k) {
        float x[V];
        load_slab4<STREAM>(w + (long long)k * row_stride + j0, x);
#pragma unroll
        for (int v = 0; v < V; ++v) acc[v] += x[v];
      }
#pragma unroll
      for (int v = 0; v < V; ++v) acc[v] = acc[v] / kf;
      if (w_prev != nullptr || norm_part != nullptr) {
        float old[V];
        load_f32_vec<V, STREAM>(w_t0 + j0, old);
        if (w_prev != nullptr) store_f32x4<STREAM>(w_prev + j0, old);
        if (norm_part != nullptr) {
          const float dx = acc[0] - old[0], dy = acc[1] - old[1], dz = acc[2] - old[2], dw = acc[3] - old[3];
          nacc += (double)fmaf(dx, dx, fmaf(dy, dy, fmaf(dz, dz, dw * dw)));
        }
      }
      store_f32x4<STREAM>(w_t0 + j0, acc);
      const RowVec4 row = pack_row4(acc, static_cast<const T*>(nullptr));
#pragma unroll 8
      for (int k = 0; k < K; ++k) store_row4<STREAM>(w + (long long)k * row_stride + j0, row);
    } else {
      for (int v = 0; v < V; ++v) {
        const long long j = j0 + v;
        if (j >= d) break;
        float a = 0.0f;
        for (int k = 0; k < K; ++k) a += Slab<T>::load_one(w + (long long)k * row_stride + j);
        a = a / kf;
        const float o = w_t0[j];
        if (w_prev != nullptr) w_prev[j] = o;
        if (norm_part != nullptr) nacc += (double)((a - o) * (a - o));
        w_t0[j] = a;
        for (int k = 0; k < K; ++k) Slab<T>::store_one(w + (long long)k * row_stride + j, a);
      }
    }
  }
  if (norm_part != nullptr) {
    const double s = block_sum(nacc, scratch);
    if (threadIdx.x == 0) norm_part[blockIdx.x] = s;
  }
}
// n partial sums -> gridDim.x sums of contiguous slices, out[workgroup], each in a fixed order
__global__ void __launch_bounds__(kSmallThreads)
sum_partials_kernel(const double* __restrict__ part, long long n, const int32_t* __restrict__ pred,
                    double* __restrict__ out) {
  __shared__ double scratch[kSmallThreads / 64];
  if (pred != nullptr && *pred == 0) return;
  const long long per = (n + gridDim.x - 1) / gridDim.x;
  const long long beg = (long long)blockIdx.x * per;
  const long long end = beg + per < n ? beg + per : n;
  double acc = 0.0;
  for (long long t = beg + threadIdx.x; t < end; t += kSmallThreads) acc += part[t];
  const double s = block_sum(acc, scratch);
  if (threadIdx.x == 0) out[blockIdx.x] = s;
}

// Algorithm 1 line 9 when the average model is already there (w_bar from mean_state_kernel):
// every row <- w_bar, w_prev <- w_t0, w_t0 <- w_bar, and (xi != NULL) the xi of Section 3.2,
// (w_bar - old w_t0) / ||w_bar - old w_t0||, with the squared norm taken from *dnorm.
template <typename T, bool STREAM>
__global__ void __launch_bounds__(kSmallThreads)
sync_from_mean_kernel(T* __restrict__ w, float* __restrict__ w_t0, float* __restrict__ w_prev,
                      float* __restrict__ xi, const float* __restrict__ w_bar,
                      const double* __restrict__ dnorm, const int32_t* __restrict__ pred, int K,
                      long long d, long long row_stride, int vec_ok) {
  constexpr int V = kSyncV;
  if (pred != nullptr && *pred == 0) return;
  float scale = 0.0f;
  if (xi != nullptr) {
    const double nrm = sqrt(*dnorm);
    scale = (nrm > 0.0 && isfinite(nrm)) ? (float)(1.0 / nrm) : 0.0f;
  }
  const SyncRange rg = sync_range((d + V - 1) / V);
  for (long long vi = rg.beg + threadIdx.x; vi < rg.end; vi += rg.step) {
    const long long j0 = vi * V;
    if (vec_ok && j0 + V <= d) {
      float nb[V], old[V];
      load_f32_vec<V, STREAM>(w_bar + j0, nb);
      load_f32_vec<V, STREAM>(w_t0 + j0, old);
      if (w_prev != nullptr) store_f32x4<STREAM>(w_prev + j0, old);
      store_f32x4<STREAM>(w_t0 + j0, nb);
      if (xi != nullptr) {
        float x[V];
#pragma unroll
        for (int v = 0; v < V; ++v) x[v] = (scale == 0.0f) ? 0.0f : (nb[v] - old[v]) * scale;
        store_f32x4<STREAM>(xi + j0, x);
      }
      const RowVec4 row = pack_row4(nb, static_cast<const T*>(nullptr));
#pragma unroll 8
      for (int k = 0; k < K; ++k) store_row4<STREAM>(w + (long long)k * row_stride + j0, row);
    } else {
      for (int v = 0; v < V; ++v) {
        const long long j = j0 + v;
        if (j >= d) break;
        const float a = w_bar[j], o = w_t0[j];
        if (w_prev != nullptr) w_prev[j] = o;
        w_t0[j] = a;
        if (xi != nullptr) xi[j] = (scale == 0.0f) ? 0.0f : (a - o) * scale;
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
               const int32_t* __restrict__ pred, long long d, int vec_ok, double* __restrict__ partial) {
  __shared__ double scratch[kSmallThreads / 64];
  if (pred != nullptr && *pred == 0) return;
  double acc = 0.0;
  const long long step = (long long)gridDim.x * blockDim.x;
  const long long t0 = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long nvec = vec_ok ? d / 4 : 0;             // whole 16-byte vectors
  for (long long v = t0; v < nvec; v += step) {
    const f32x4 a = reinterpret_cast<const f32x4*>(w_t0)[v];
    const f32x4 b = reinterpret_cast<const f32x4*>(w_prev)[v];
    const float dx = a.x - b.x, dy = a.y - b.y, dz = a.z - b.z, dw = a.w - b.w;
    acc += (double)fmaf(dx, dx, fmaf(dy, dy, fmaf(dz, dz, dw * dw)));   // a short fp32 run, then fp64
  }
  for (long long j = nvec * 4 + t0; j < d; j += step) {  // the tail, or everything without vectors
    const float df = w_t0[j] - w_prev[j];
    acc += (double)(df * df);
  }
  const double s = block_sum(acc, scratch);
  if (threadIdx.x == 0) partial[blockIdx.x] = s;
}

__global__ void __launch_bounds__(kSmallThreads)
xi_scale_kernel(const float* __restrict__ w_t0, const float* __restrict__ w_prev,
                float* __restrict__ xi, const int32_t* __restrict__ pred, long long d, int vec_ok,
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
  const long long step = (long long)gridDim.x * blockDim.x;
  const long long t0 = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long nvec = vec_ok ? d / 4 : 0;
  for (long long v = t0; v < nvec; v += step) {
    const f32x4 a = reinterpret_cast<const f32x4*>(w_t0)[v];
    const f32x4 b = reinterpret_cast<const f32x4*>(w_prev)[v];
    f32x4 o = {0.0f, 0.0f, 0.0f, 0.0f};
    if (scale != 0.0f) o = (a - b) * scale;
    reinterpret_cast<f32x4*>(xi)[v] = o;
  }
  for (long long j = nvec * 4 + t0; j < d; j += step) {
    const float df = w_t0[j] - w_prev[j];
    xi[j] = (scale == 0.0f) ? 0.0f : df * scale;
  }
}

}  // namespace fda
