// Device code of the FDA monitor for gfx950 (wave64): the mean-state kernel.
//
// Algorithm 1 line 7 needs only the average state.  With all K workers in one address space the
// linearity of the AMS sketch (Section 3.1: sk(a u + b v) = a sk(u) + b sk(v)) gives it
// directly:  mean_k sk(u_k) = sk(mean_k u_k),  mean_k <xi,u_k> = <xi, mean_k u_k>,  so the
// sketch costs l LDS additions per coordinate instead of l*K and the pass is bound by the HBM
// stream again.  (The per-worker states of Algorithm 1 line 6 stay with state_kernel.)
//
// Workgroup (p, r) streams coordinates [p*chunk, (p+1)*chunk) of ALL K workers exactly once, in
// batches of KB slab rows, and owns the sketch rows of row group r (R > 1 only when l*m 8-byte
// cells do not fit in LDS; then every row group repeats the loads).  Per tile a lane owns V
// consecutive coordinates; for each it sums the K drifts, accumulates sum_k u^2 and <xi,u>
// (fp32 within the tile, fp64 across tiles; row group 0 only), and at the end of the tile adds
// sign * (sum of the K drifts) into the LDS sketch [row][bucket] once per sketch row.
// On request (w_bar != NULL) row group 0 also writes the average model w_t0 + mean_k u_k and
// accumulates the squared norm of what fda_sync_from_mean will see as the model change,
// (w_bar - w_t0) as rounded to fp32 -- Algorithm 1 line 9 and the xi of Section 3.2 then need
// no second pass over the slab.
//
//   kCellI64  a drift enters as the integer round(u * Sm) (Sm = ScaleInfo::Sm, the mean sampled
//             |u| maps to about 2^18, every |u| must stay below boundm = 2^30 / Sm); the K
//             integers of a coordinate are summed in 64 bits and added to 64-bit cells.  All of
//             it is exact, so the result does not depend on the order of additions or on the
//             partitioning.  |sum of a cell| < K * chunk * 2^30, which the host keeps below 2^63.
//             A drift at or above boundm raises ScaleInfo::flagm.
//   kCellF64  fp64 sums and ds_add_f64 cells; runs only when flagm is set.
#pragma once
#include "fda_kernels.hpp"

namespace fda {

struct MeanParams {
  const void* w;
  const float* w_t0;
  const float* xi;
  long long row_stride;
  long long d;
  long long chunk;        // coordinates per partition (multiple of the tile)
  int K;
  int l;
  int m;
  int R;                  // sketch-row groups
  int P;                  // coordinate partitions, multiple of 8
  int do_lin;
  int do_sk;
  int vec_ok;             // all pointers / strides allow whole-vector loads
  float* w_bar;           // [d] or NULL: receives w_t0 + mean_k u_k
  double* part_np;        // [P][3]: sum_k ||u_k||^2, sum_k <xi,u_k>, ||w_bar - w_t0||^2 of the partition
  void* part_sk;          // [P][l*m] 8-byte words: int64 (integer cells) or double (fp64 cells)
  ScaleInfo* scale;
  const uint16_t* table;  // [R][dpad] records of the tabulated hash, one field per row slot
  long long dpad;
};

template <typename T, int KB>
struct MeanBatch {
  static constexpr int kWords = kStateV * (int)sizeof(T) / 4;
  uint32_t w[KB][kWords];       // V elements of each of KB slab rows
};
template <int LR, int FB>
struct MeanHead {
  float w0[kStateV];
  float x[kStateV];
  uint32_t rec[RecGeom<LR, FB>::kDwords];      // the V records of the tabulated hash
};

template <typename T, int KB, int LR, int CELL, int FB>
__global__ void __launch_bounds__(kStateThreads)
mean_state_kernel(const MeanParams prm) {
  static_assert(CELL == kCellI64 || CELL == kCellF64, "8-byte cells only");
  constexpr int V = kStateV;
  constexpr long long kTile = (long long)kStateThreads * V;
  using Batch = MeanBatch<T, KB>;
  using Geom = RecGeom<LR, FB>;
  using Head = MeanHead<LR, FB>;
  extern __shared__ __align__(16) unsigned char lds_raw[];
  if constexpr (CELL == kCellF64) {
    if (prm.do_sk == 0 || prm.scale->flagm == 0) return;
  }

  // consecutive workgroup ids go round-robin over the 8 XCDs: the R workgroups that read the
  // same coordinates get ids on one XCD and its L2
  const int b = blockIdx.x;
  const int xcd = b & 7, slot = b >> 3;
  const int r = slot % prm.R;
  const int p = (slot / prm.R) * 8 + xcd;
  int rstart = 0, rcnt = 0;
  if (prm.do_sk) group_range(prm.l, prm.R, r, &rstart, &rcnt);
  const bool scalars = (CELL == kCellI64) && (r == 0);
  bool sketch = prm.do_sk != 0;
  if constexpr (CELL == kCellI64) {
    // the fp64 pass will redo the sketch: only the scalar components are left to do
    if (sketch && prm.scale->flagm != 0) {
      if (!scalars) return;
      sketch = false;
    }
  }

  const int cells = rcnt * prm.m;
  const uint32_t dummy_base = (uint32_t)cells * 8u;
  const int lds_cells = sketch ? cells + kDummyCells : 0;
  double* red = reinterpret_cast<double*>(lds_raw + (size_t)lds_cells * 8);
  const int tid = threadIdx.x;
  {
    unsigned long long* c64 = reinterpret_cast<unsigned long long*>(lds_raw);
    for (int t = tid; t < lds_cells; t += kStateThreads) c64[t] = 0ull;     // integer 0 and 0.0
  }
  __syncthreads();

  // spare row slots: their table fields hold buckets below kDummyCells, sent to the dummy region
  uint32_t rowbase[LR];
#pragma unroll
  for (int i = 0; i < LR; ++i) rowbase[i] = i < rcnt ? (uint32_t)(i * prm.m) * 8u : dummy_base;
  const uint32_t* const recs =
      reinterpret_cast<const uint32_t*>(prm.table + (size_t)r * prm.dpad * Geom::kWords);

  const long long cbeg = (long long)p * prm.chunk;
  long long cend = cbeg + prm.chunk;
  if (cend > prm.d) cend = prm.d;
  const long long dlim = prm.d;
  const bool lin = prm.do_lin && scalars;
  const float* const w0p = prm.w_t0;
  const float* const xip = lin ? prm.xi : prm.w_t0;     // without LinearFDA: any readable vector
  const T* const wbase = reinterpret_cast<const T*>(prm.w);
  const long long rs = prm.row_stride;
  const int K = prm.K;
  const int NB = (K + KB - 1) / KB;                     // batches of slab rows per tile
  const int tail = K - (NB - 1) * KB;                   // rows of the last batch, 1..KB
  const float Sm = prm.do_sk ? prm.scale->Sm : 1.0f;
  float* const wbp = scalars ? prm.w_bar : nullptr;
  const float kf = (float)K;

  double dn = 0.0, dp = 0.0, dd = 0.0;
  float amax = 0.0f;

  // SC: this workgroup also produces the scalar components; SK: it accumulates sketch rows.
  auto run = [&](auto sc_tag, auto sk_tag) {
    constexpr bool SC = decltype(sc_tag)::value;
    constexpr bool SK = decltype(sk_tag)::value;
    long long acc[V];         // integer cells: sum over the workers of round(u * Sm)
    double us[V];             // fp64 cells: sum over the workers of u
    float um[V];              // scalar workgroups: sum over the workers of u, for the average model
    float sn = 0.0f, sp = 0.0f;
#pragma unroll
    for (int v = 0; v < V; ++v) { acc[v] = 0; us[v] = 0.0; um[v] = 0.0f; }

    // slab rows k0 .. k0+KB-1 (rows past the last worker repeat it; consume() drops them)
    auto load_batch_fast = [&](Batch& bt, long long j0, int k0) {
#pragma unroll
      for (int k = 0; k < KB; ++k) {
        const int row = (k0 + k < K) ? k0 + k : K - 1;
        const T* src = wbase + (long long)row * rs + j0;
        if constexpr (sizeof(T) == 4) {
          const u32x4 q = load_vec_hint<u32x4, kNtSlab>(src);
          bt.w[k][0] = q.x; bt.w[k][1] = q.y; bt.w[k][2] = q.z; bt.w[k][3] = q.w;
        } else {
          const u32x2_h q = load_vec_hint<u32x2_h, kNtSlab>(src);
          bt.w[k][0] = q.x; bt.w[k][1] = q.y;
        }
      }
    };
    auto load_batch_slow = [&](Batch& bt, long long j0, int k0) {
#pragma unroll
      for (int k = 0; k < KB; ++k) {
        const int row = (k0 + k < K) ? k0 + k : K - 1;
        const T* src = wbase + (long long)row * rs + j0;
        if constexpr (sizeof(T) == 4) {
#pragma unroll
          for (int v = 0; v < 4; ++v)
            bt.w[k][v] = (j0 + v < dlim) ? __float_as_uint(Slab<T>::load_one(src + v)) : 0u;
        } else {
          const uint16_t* h = reinterpret_cast<const uint16_t*>(src);
#pragma unroll
          for (int v = 0; v < 4; v += 2) {
            const uint32_t lo = (j0 + v < dlim) ? (uint32_t)h[v] : 0u;
            const uint32_t hi = (j0 + v + 1 < dlim) ? (uint32_t)h[v + 1] : 0u;
            bt.w[k][v >> 1] = lo | (hi << 16);
          }
        }
      }
    };
    auto load_table = [&](Head& h, long long j0) {
      // the table is padded to dpad (whole blocks of 256 coordinates): always whole records
      if constexpr (SK)
        load_rec_block<Geom::kDwords, kNtSlab>(recs + (j0 >> 8) * (64 * Geom::kDwords), (int)(j0 >> 2) & 63, h.rec);
    };
    auto load_head_fast = [&](Head& h, long long j0) {
      load_f32_vec<V, kNtShared>(w0p + j0, h.w0);
      if constexpr (SC) load_f32_vec<V, kNtShared>(xip + j0, h.x);
      load_table(h, j0);
    };
    auto load_head_slow = [&](Head& h, long long j0) {
#pragma unroll
      for (int v = 0; v < V; ++v) {
        const bool in = (j0 + v < dlim);
        h.w0[v] = in ? w0p[j0 + v] : 0.0f;
        if constexpr (SC) h.x[v] = in ? xip[j0 + v] : 0.0f;
      }
      load_table(h, j0);
    };

    // one batch of rows; `live` of its KB rows are workers (the others contribute nothing)
    auto consume = [&](const Batch& bt, const Head& h, auto tail_tag, int live) {
      constexpr bool TAIL = decltype(tail_tag)::value;
#pragma unroll
      for (int k = 0; k < KB; ++k) {
#pragma unroll
        for (int v = 0; v < V; ++v) {
          float u = raw_elem(bt.w[k], v) - h.w0[v];
          if constexpr (TAIL) u = (k < live) ? u : 0.0f;
          if constexpr (SC) {
            sn = fmaf(u, u, sn);
            sp = fmaf(h.x[v], u, sp);
            amax = fmaxf(amax, fabsf(u));
            um[v] += u;
          }
          if constexpr (SK && CELL == kCellI64) acc[v] += (long long)round_half_up(u * Sm);
          if constexpr (SK && CELL == kCellF64) us[v] += (double)u;
        }
      }
    };

    // end of a tile: the scalar partials go to fp64, the V sums into the sketch rows
    auto finish = [&](const Head& h, long long j0, bool whole) {
      if constexpr (SC) {
        dn += (double)sn; dp += (double)sp;
        sn = 0.0f; sp = 0.0f;
        if (wbp != nullptr) {
          float wb[V], sd = 0.0f;
#pragma unroll
          for (int v = 0; v < V; ++v) {
            wb[v] = h.w0[v] + um[v] / kf;
            const float df = wb[v] - h.w0[v];        // the model change as fp32 storage keeps it
            sd = fmaf(df, df, sd);
          }
          if (whole) {
            store_f32_vec<V>(wbp + j0, wb);
            dd += (double)sd;
          } else {
            sd = 0.0f;
#pragma unroll
            for (int v = 0; v < V; ++v)
              if (j0 + v < dlim) {
                wbp[j0 + v] = wb[v];
                const float df = wb[v] - h.w0[v];
                sd = fmaf(df, df, sd);
              }
            dd += (double)sd;
          }
        }
#pragma unroll
        for (int v = 0; v < V; ++v) um[v] = 0.0f;
      }
      if constexpr (SK) {
#pragma unroll
        for (int v = 0; v < V; ++v) {
#pragma unroll
          for (int i = 0; i < LR; ++i) {
            const uint32_t hw = rec_field<LR, FB>(h.rec, v, i);
            const uint32_t sb = hw & Geom::kFieldMask;                     // bucket + m * (sign is -1)
            const bool neg = sb >= (uint32_t)prm.m;
            const uint32_t off = ((neg ? sb - (uint32_t)prm.m : sb) << 3) + rowbase[i];
            if constexpr (CELL == kCellI64) {
              const unsigned long long q = (unsigned long long)acc[v];
              atomicAdd(reinterpret_cast<unsigned long long*>(lds_raw + off), neg ? 0ull - q : q);
            } else {
              atomicAdd(reinterpret_cast<double*>(lds_raw + off), neg ? -us[v] : us[v]);
            }
          }
          acc[v] = 0; us[v] = 0.0;
        }
      }
    };

    // tiles that lie wholly inside the chunk: software pipelined over (tile, batch), the next
    // batch's loads (and, before a tile's last batch, the next tile's w_t0 / xi / table) in
    // flight while the current batch is consumed
    const long long nfast = prm.vec_ok ? (cend > cbeg ? (cend - cbeg) / kTile : 0) : 0;
    long long j0 = cbeg + (long long)tid * V;
    if (nfast > 0) {
      Head hc;
      Batch bc;
      load_head_fast(hc, j0);
      load_batch_fast(bc, j0, 0);
      for (long long it = 0; it < nfast; ++it) {
        for (int bi = 1; bi < NB; ++bi) {
          Batch bn;
          load_batch_fast(bn, j0, bi * KB);
          consume(bc, hc, std::false_type{}, KB);
          bc = bn;
        }
        const long long jn = (it + 1 < nfast) ? j0 + kTile : j0;   // the last prefetch re-reads, unused
        Head hn;
        Batch bn;
        load_head_fast(hn, jn);
        load_batch_fast(bn, jn, 0);
        if (tail < KB) consume(bc, hc, std::true_type{}, tail);
        else consume(bc, hc, std::false_type{}, KB);
        finish(hc, j0, true);
        hc = hn;
        bc = bn;
        j0 += kTile;
      }
    }
    // what is left: at most one ragged tile, or everything when vectors are not possible
    for (; j0 < cend; j0 += kTile) {
      Head h;
      load_head_slow(h, j0);
      for (int bi = 0; bi < NB; ++bi) {
        Batch bt;
        load_batch_slow(bt, j0, bi * KB);
        if (bi == NB - 1 && tail < KB) consume(bt, h, std::true_type{}, tail);
        else consume(bt, h, std::false_type{}, KB);
      }
      finish(h, j0, false);
    }
  };
  if (scalars) {
    if (sketch) run(std::true_type{}, std::true_type{});
    else run(std::true_type{}, std::false_type{});
  } else {
    run(std::false_type{}, std::true_type{});
  }

  if constexpr (CELL == kCellI64) {
    if (prm.do_sk && scalars) {
      // drifts the integers cannot hold (any drift at all when the sample saw none)
      const float bm = prm.scale->boundm;
      const bool bad = bm > 0.0f ? !(amax < bm) : (amax > 0.0f);
      if (bad) prm.scale->flagm = 1;
    }
  }

  // ---- workgroup reduction of the scalar components (fixed shape) ---------------------
  const int lane = tid & 63, wave = tid >> 6;
  constexpr int kWaves = kStateThreads / 64;
  if (scalars) {
    const double a = wave_sum(dn);
    const double c = wave_sum(dp);
    const double e = wave_sum(dd);
    if (lane == 0) { red[wave * 3] = a; red[wave * 3 + 1] = c; red[wave * 3 + 2] = e; }
  }
  __syncthreads();
  if (scalars && tid < 3) {
    double s = 0.0;
    for (int wv = 0; wv < kWaves; ++wv) s += red[wv * 3 + tid];
    if (tid == 1 && !lin) s = 0.0;               // no LinearFDA: the projection slot stays zero
    prm.part_np[(size_t)p * 3 + tid] = s;
  }
  // ---- flush the LDS sketch to this workgroup's slice of the partial buffer -----------
  if (sketch) {
    const int allcells = prm.l * prm.m;
    unsigned long long* out = reinterpret_cast<unsigned long long*>(prm.part_sk);
    const unsigned long long* c64 = reinterpret_cast<const unsigned long long*>(lds_raw);
    for (int t = tid; t < cells; t += kStateThreads)
      out[(size_t)p * allcells + (size_t)rstart * prm.m + t] = c64[t];
  }
}

}  // namespace fda
