// C ABI of the FDA monitor (include/fda.h): argument checks, launch planning, kernel
// launches.  Everything the path computes runs in the kernels of fda_kernels.hpp.
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstddef>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>

#include "fda.h"
#include "fda_small_kernels.hpp"
#include "fda_state_launch.hpp"
#include "fda_mean_launch.hpp"

// Scratch of fda_estimate_variance_static: the per-workgroup partial sums of estimate_kernel
// (2 + FDA_MAX_SKETCH_ROWS * 128 doubles) and, 256-aligned behind them, its finished-workgroup
// counter.  Every GPU the library runs on holds its own copy until the process ends.  In host code
// this name is only a handle for hipGetSymbolAddress: the address kernels are given is the one
// static_scratch() looked up for the current device.
constexpr size_t kStaticPartDoubles = 2 + (size_t)FDA_MAX_SKETCH_ROWS * 128;
constexpr size_t kStaticTicketOffset = (kStaticPartDoubles * 8 + 255) / 256 * 256;
constexpr size_t kStaticScratchBytes = kStaticTicketOffset + 256;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

#define FDA_HIP(call)                                                                  \
  do {                                                                                 \
    hipError_t e_ = (call);                                                            \
    if (e_ != hipSuccess)                                                              \
      return fail(FDA_EHIP, "%s failed: %s", #call, hipGetErrorString(e_));            \
  } while (0)

constexpr int64_t kLdsReserve = 1536;      // reduction scratch (8 waves x 8 worker slots x 2 doubles) + slack
constexpr int kMaxRounds = 4;              // at most this many rounds of resident workgroups per launch
constexpr int64_t kMaxTermsPlanned = 12000;    // terms per 32-bit cell and workgroup the planner allows for
constexpr int64_t kMaxTermsPlannedSplit = 3500;   // ... per cell of a sign-split row
constexpr double kWorkgroupOverheadTiles = 6.0;   // what a state workgroup costs besides its tiles, in tiles
// the planner's cost model, in vector-ALU instructions per coordinate
constexpr double kElementCost = 6.5;       // load / unpack / drift / fixed point / scalar sums of one slab element
constexpr double kNegateCost = 2.0;        // ... its negated term, when the rows are not sign-split
constexpr double kDecodeCost = 2.5;        // one table field into an LDS address
constexpr double kSignCost = 3.0;          // ... and into a sign and a bucket, when the rows are not sign-split
constexpr double kSelectCost = 1.0;        // choosing the term or its negative for one 32-bit cell
constexpr double kAtomicCost = 7.5;        // one 32-bit LDS addition and the OR of what it returned
constexpr double kPairAddCost = 13.0;      // one 64-bit LDS addition (two cells) and the OR of what it returned
constexpr double kPlacedPairAddCost = 9.5; // ... when the table's row slots are placed against LDS collisions
constexpr double kSharedByteCost = 0.25;   // per byte of w_t0 / xi / table read by one more workgroup
constexpr int kMaxEstBlocksPerRow = 128;   // 32768 / 256: workgroups of estimate_kernel per sketch row
constexpr int kScaleSamples = 16384;       // sampled coordinates per worker for the scale
constexpr int kScaleBlocks = kScaleSamples * fda::kScaleMaxSlices / fda::kSmallThreads;   // its workgroups, at most
constexpr int kXiBlocks = 4096;
constexpr int kSyncNormSlices = 64;   // the synchronization kernel's partial norms are condensed to this many
constexpr long long kSyncVectorsPerBlock = 4 * fda::kSmallThreads;   // four trips per workgroup
constexpr long long kStreamBytes = 512ll << 20;   // slabs beyond this are synchronized with streaming hints
constexpr int64_t kAlign = 256;

int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

// How one state pass is spread over the chip for a given sketch-cell size.
struct Split {
  int G, R, kcnt_max, rcnt_max, KC, LR, P, stride;
  int split;        // 32-bit cells: sign-split LDS rows (2 m buckets per row)
  int64_t chunk, lds_bytes;
};
// How one mean-state pass is spread over the chip.
struct MeanSplit {
  int R, rcnt_max, P, occ;
  int64_t chunk, lds_bytes;
};
struct Plan {
  Split narrow;     // 32-bit cells: the pass every call runs
  Split wide;       // 8-byte cells: the 64-bit integer and fp64 passes
  MeanSplit mean;   // fda_mean_state
  int vec;          // elements per 16-byte slab load
  int fb;           // bits per field of the tabulated hash
  int narrow_fb;    // ... of the table the 32-bit-cell pass streams (kPlacedFieldBits with placed rows)
  int grp;          // rows per placement group of that table (1: rows keep their slots)
  int words;        // 16-bit words per record of the table the 32-bit-cell pass streams
  int mean_words;   // ... and of the mean-state pass's table
  bool shared_table;  // both passes split the rows alike and stream one table
  int64_t cells, S, dpad;
  int64_t off_np, off_sk, off_xi, off_syncnorm, off_scale, off_smax, off_ssum, off_nmax, off_dnorm, off_est, off_ticket, off_table,
      off_mean_table, ws_bytes;
};

int validate(const fda_desc* d) {
  if (d == nullptr) return fail(FDA_EINVAL, "desc is NULL");
  if (d->K < 1) return fail(FDA_EINVAL, "K must be >= 1 (got %d)", d->K);
  if (d->d < 1) return fail(FDA_EINVAL, "d must be >= 1");
  if (d->d >= (int64_t)FDA_HASH_PRIME - 64)
    return fail(FDA_ERANGE, "d must be below 2^31 - 1 - 64: coordinates are hash keys modulo 2^31 - 1");
  if (d->row_stride < d->d) return fail(FDA_EINVAL, "row_stride must be >= d");
  if (d->dtype != FDA_F32 && d->dtype != FDA_BF16) return fail(FDA_EINVAL, "unknown dtype %d", d->dtype);
  if ((d->flags & ~FDA_DESC_PLAIN_TABLE) != 0) return fail(FDA_EINVAL, "unknown flags");
  if ((d->variants & ~(FDA_VARIANT_LINEAR | FDA_VARIANT_SKETCH)) != 0 || d->variants == 0)
    return fail(FDA_EINVAL, "variants must be a non-empty mask of FDA_VARIANT_LINEAR | FDA_VARIANT_SKETCH");
  if (d->variants & FDA_VARIANT_SKETCH) {
    if (d->l < 1 || d->l > FDA_MAX_SKETCH_ROWS)
      return fail(FDA_EINVAL, "l must be in 1..%d (got %d)", FDA_MAX_SKETCH_ROWS, d->l);
    if (d->m < 1) return fail(FDA_EINVAL, "m must be >= 1");
    if (d->m > 32767) return fail(FDA_ERANGE, "m must be below 32768 (bucket indices are tabulated in 15 bits)");
    if ((int64_t)d->l * d->m > (int64_t)1 << 24) return fail(FDA_ERANGE, "l*m too large");
    if (!(d->eps > -1.0)) return fail(FDA_EINVAL, "eps must be > -1");
    if (d->hash_coef == nullptr) return fail(FDA_EINVAL, "hash_coef is NULL");
    for (int t = 0; t < d->l * 8; ++t)
      if (d->hash_coef[t] >= FDA_HASH_PRIME)
        return fail(FDA_ERANGE, "hash_coef[%d] is not below 2^31 - 1", t);
  }
  return FDA_OK;
}

int make_split(const fda_desc* d, int cus, int64_t lds_cu, int cell_bytes, Split* sp) {
  const bool sk = (d->variants & FDA_VARIANT_SKETCH) != 0;
  const int64_t cells = sk ? (int64_t)d->l * d->m : 0;
  const int vec = fda::kStateV;
  // Split the K workers into G groups and the l sketch rows into R groups so that one
  // workgroup's sketch (rows x m cells x worker slots) fits in LDS.  The kernel has KC worker
  // slots and LR row slots (compile-time); slots a group does not fill still execute.  Every
  // row group repeats the loads and the fixed-point conversion of its workers' elements; every
  // workgroup decodes its rows' table entries and re-reads w_t0 / xi / table (through L2).
  // Pick the split with the least estimated vector-ALU work per coordinate.
  const int l = sk ? d->l : 1;
  double best = -1.0;
  int bestG = 0, bestR = 0, bestKC = 0, bestLR = 0, bestSplit = 0;
  const bool narrow = cell_bytes == 4;
  for (int G = 1; G <= d->K; ++G) {
    const int kc = (d->K + G - 1) / G;
    {
      int KC = 0;                                            // the smallest kernel that holds kc workers
      if (narrow) {
        for (int c : fda::kKCSet)
          if (c >= kc) { KC = c; break; }
      } else {
        for (int c : fda::kWideKCSet)
          if (c >= kc) { KC = c; break; }
      }
      if (KC == 0) continue;
      const int stride = (KC == 1) ? 1 : (KC | 1);
      // sign-split rows (32-bit cells, even slot counts): no negated terms, no select per addition, twice the LDS
      // (without a sketch either kind of kernel does the same)
      for (int split = (narrow && KC % 2 == 0) ? 1 : 0; split >= 0; --split) {
        if (narrow && !fda::narrow_kernel_exists(KC, split != 0)) continue;
        for (int R = 1; R <= l; ++R) {
          const int rc = (l + R - 1) / R;
          int LR = 0;                                        // row slots of the kernel that would run
          if (narrow) {
            if (rc <= fda::kMaxLR && KC * rc <= fda::kMaxSlots) LR = rc;
          } else {
            for (int c : fda::kWideLRSet)
              if (c >= rc) { LR = c; break; }
          }
          if (LR == 0) continue;
          const int64_t need = !cells ? 0
                               : narrow ? (int64_t)fda::cells32_words(rc, split ? 2 * d->m : d->m, KC) * 4
                                        : ((int64_t)rc * d->m + fda::kDummyCells) * stride * cell_bytes;
          if (need + kLdsReserve > lds_cu) continue;
          // Estimated cost per coordinate, in vector-ALU instructions (an LDS addition counted as what it
          // keeps the compute unit from issuing): per element slot the load / drift / fixed-point work
          // (with the negated terms unless the rows are sign-split), per row slot the table field, per
          // addition the select (unless split), the overflow OR and the LDS instruction itself.
          const double wg = (double)G * R;
          const double pairs = (KC % 2 == 0 && narrow) ? KC / 2 : KC;           // LDS instructions per row slot
          // (a table with placed rows avoids about a third of the LDS collisions)
          const bool placed = narrow && split && cells && fda::placed_kernel_exists(KC) &&
                              !(d->flags & FDA_DESC_PLAIN_TABLE) && fda::placed_group_rows(rc, d->m, KC) >= 2;
          const double per_add = (KC % 2 == 0 && narrow) ? (placed ? kPlacedPairAddCost
                                                            : split ? kPairAddCost : kPairAddCost + 2.0 * kSelectCost)
                                                         : kAtomicCost + kSelectCost;
          const double cost = wg * KC * (split ? kElementCost : kElementCost + kNegateCost) +
                              wg * LR * (split ? kDecodeCost : kDecodeCost + kSignCost) +
                              wg * LR * pairs * per_add +
                              wg * (8 + 2 * LR) * kSharedByteCost + 1e-3 * wg;
          if (best < 0.0 || cost < best) {
            best = cost; bestG = G; bestR = R; bestKC = KC; bestLR = LR; bestSplit = split;
          }
          break;   // a larger R only costs more for this G
        }
      }
    }
  }
  if (bestG == 0)
    return fail(FDA_ERANGE, "one row of an m = %d sketch does not fit in %lld bytes of LDS", d->m,
                (long long)lds_cu);
  sp->G = bestG;
  sp->R = bestR;
  sp->split = bestSplit;
  sp->kcnt_max = (d->K + bestG - 1) / bestG;
  sp->rcnt_max = (l + bestR - 1) / bestR;
  sp->KC = bestKC;
  sp->LR = bestLR;
  sp->stride = (sp->KC == 1) ? 1 : (sp->KC | 1);
  const int64_t sk_bytes = !cells ? 0
                           : narrow ? (int64_t)fda::cells32_words(sp->rcnt_max, sp->split ? 2 * d->m : d->m, sp->KC) * 4
                                    : ((int64_t)sp->rcnt_max * d->m + fda::kDummyCells) * sp->stride * cell_bytes;
  sp->lds_bytes = round_up(sk_bytes, 16) + kLdsReserve;
  // one workgroup per CU: the kernels hold more registers than two resident workgroups would allow
  const int occ = 1;
  const int64_t tile = (int64_t)fda::kStateThreads * vec;
  // Partitions: all workgroups do the same amount of work, so the launch should fill the resident
  // slots a whole number of times; and a workgroup costs its set-up, reductions and flush on top of
  // its tiles (measured: about six tiles' worth).  Among the first few feasible numbers of rounds of
  // resident workgroups keep the cheapest: rounds x (tiles per workgroup + overhead).
  // Feasible: 32-bit cells take up to 16384 terms (scale_kernel sends fuller ones to the 64-bit pass), so
  // a chunk should put about 12000 into a cell at most.  The cells of sign-split rows take the terms of one
  // hash sign each, which do not cancel when the drifts themselves lean one way: they are kept at about
  // 3500 expected terms (a term of mean magnitude is 2^18..2^19 units: the band of 2^30 then holds unless
  // more than about half of a cell's mass leans one way -- such a call finishes on the 64-bit cells).
  const int64_t slots = (int64_t)cus * occ, gr = (int64_t)bestG * bestR;
  const int64_t tiles = (d->d + tile - 1) / tile;
  int64_t pmin = 1;
  if (narrow && cells) {
    const int64_t per_row = (int64_t)d->m * (bestSplit ? 2 : 1);
    const int64_t terms = bestSplit ? kMaxTermsPlannedSplit : kMaxTermsPlanned;
    pmin = (d->d + per_row * terms - 1) / (per_row * terms);
    if (pmin > tiles) pmin = tiles;
  }
  int64_t P = 0;
  double best_time = -1.0;
  int tried = 0;
  for (int64_t rounds = 1; tried < kMaxRounds; ++rounds) {
    int64_t cand = slots * rounds / gr;                 // (whole groups of 8 partitions share an XCD each)
    if (cand < 1) cand = 1;
    if (cand > tiles) cand = tiles;
    if (cand < pmin) continue;                          // more rounds are needed: cand grows with them
    ++tried;
    const int64_t wgs = cand * gr;
    const double est = (double)((wgs + slots - 1) / slots) * ((double)((tiles + cand - 1) / cand) + kWorkgroupOverheadTiles);
    if (best_time < 0.0 || est < best_time * 0.98) { best_time = est; P = cand; }
    if (cand == tiles) break;                           // one tile per workgroup: nothing finer
  }
  sp->P = (int)P;
  sp->chunk = round_up((d->d + P - 1) / P, tile);
  return FDA_OK;
}

int make_mean_split(const fda_desc* d, int cus, int64_t lds_cu, MeanSplit* ms) {
  const bool sk = (d->variants & FDA_VARIANT_SKETCH) != 0;
  const int l = sk ? d->l : 1;
  // every workgroup reads all K workers; its sketch rows (8-byte cells) must fit in LDS, and the
  // fewer row groups the better, since each repeats all the loads
  int R = 0, rc = 0;
  int64_t bytes = 0;
  for (int cand = 1; cand <= l; ++cand) {
    rc = (l + cand - 1) / cand;
    if (rc > fda::kMeanMaxLR) continue;
    bytes = (sk ? ((int64_t)rc * d->m + fda::kDummyCells) * 8 : 0) + kLdsReserve;
    if (bytes <= lds_cu) { R = cand; break; }
  }
  if (R == 0)
    return fail(FDA_ERANGE, "one row of an m = %d sketch does not fit in %lld bytes of LDS", d->m,
                (long long)lds_cu);
  ms->R = R;
  ms->rcnt_max = rc;
  ms->lds_bytes = bytes;
  // Two workgroups per CU when the LDS allows and a workgroup alone does not keep enough loads in flight:
  // with 16-byte loads per lane and row (fp32 slabs) one workgroup per CU does, and half as many, longer
  // workgroups measured 3-6 % faster; with 8-byte loads (bf16) two per CU measured 3 % faster.
  ms->occ = (2 * bytes <= lds_cu && d->dtype == FDA_BF16) ? 2 : 1;
  const int64_t tile = (int64_t)fda::kStateThreads * fda::kStateV;
  const int64_t tiles = (d->d + tile - 1) / tile;
  int64_t P = (int64_t)cus * ms->occ / R / 8 * 8;  // one round of resident workgroups
  if (P < 8) P = 8;
  if (P > round_up(tiles, 8)) P = round_up(tiles, 8);
  ms->P = (int)P;
  ms->chunk = round_up((d->d + P - 1) / P, tile);
  return FDA_OK;
}

int make_plan(const fda_desc* d, int cus, int64_t lds_cu, Plan* pl) {
  if (cus < 1 || lds_cu < 16384) return fail(FDA_EINVAL, "bad device description");
  const bool sk = (d->variants & FDA_VARIANT_SKETCH) != 0;
  pl->cells = sk ? (int64_t)d->l * d->m : 0;
  pl->S = 2 + pl->cells;
  pl->vec = d->dtype == FDA_F32 ? 4 : 8;
  int rc = make_split(d, cus, lds_cu, 8, &pl->wide);     // the stricter one first: its error message
  if (rc != FDA_OK) return rc;
  rc = make_split(d, cus, lds_cu, 4, &pl->narrow);
  if (rc != FDA_OK) return rc;
  rc = make_mean_split(d, cus, lds_cu, &pl->mean);
  if (rc != FDA_OK) return rc;
  // the per-workgroup partials of fda_local_state and of fda_mean_state share one region
  const int64_t Pmax = pl->narrow.P > pl->wide.P ? pl->narrow.P : pl->wide.P;
  int64_t np_bytes = (int64_t)pl->narrow.P * d->K * 2 * 8, sk_bytes = Pmax * d->K * pl->cells * 8;
  if (np_bytes < (int64_t)pl->mean.P * 3 * 8) np_bytes = (int64_t)pl->mean.P * 3 * 8;
  if (sk_bytes < (int64_t)pl->mean.P * pl->cells * 8) sk_bytes = (int64_t)pl->mean.P * pl->cells * 8;
  pl->off_np = 0;
  pl->off_sk = round_up(pl->off_np + np_bytes, kAlign);
  pl->off_xi = round_up(pl->off_sk + sk_bytes, kAlign);
  // one partial norm per workgroup of the synchronization kernel, and their sum
  const int64_t sync_blocks = ((d->d + fda::kSyncV - 1) / fda::kSyncV + kSyncVectorsPerBlock - 1) / kSyncVectorsPerBlock;
  pl->off_syncnorm = round_up(pl->off_xi + kXiBlocks * 8, kAlign);
  pl->off_scale = round_up(pl->off_syncnorm + (sync_blocks + kSyncNormSlices) * 8, kAlign);
  pl->off_smax = round_up(pl->off_scale + 2 * (int64_t)sizeof(fda::ScaleInfo), kAlign);
  pl->off_ssum = round_up(pl->off_smax + kScaleBlocks * 4, kAlign);
  pl->off_nmax = round_up(pl->off_ssum + kScaleBlocks * 8, kAlign);
  pl->off_dnorm = round_up(pl->off_nmax + 8, kAlign);
  pl->off_est = round_up(pl->off_dnorm + 8, kAlign);
  pl->off_ticket = round_up(pl->off_est + (2 + (int64_t)FDA_MAX_SKETCH_ROWS * kMaxEstBlocksPerRow) * 8, kAlign);
  pl->off_table = round_up(pl->off_ticket + 8, kAlign);
  pl->dpad = round_up(d->d, fda::kRecBlockCoords);      // the table comes in whole blocks
  // the tabulated hash: per row group one record per coordinate with a field per row slot
  pl->fb = fda::field_bits_for(sk ? d->m : 1);
  // placed rows (slots chosen against LDS collisions): sign-split rows in an unskewed layout, when a
  // placement group of at least two rows fits the wider field
  pl->grp = 1;
  pl->narrow_fb = pl->fb;
  if (sk && pl->narrow.split && fda::placed_kernel_exists(pl->narrow.KC) &&
      !(d->flags & FDA_DESC_PLAIN_TABLE)) {
    const int g = fda::placed_group_rows(pl->narrow.rcnt_max, d->m, pl->narrow.KC);
    if (g >= 2) { pl->grp = g; pl->narrow_fb = fda::kPlacedFieldBits; }
  }
  pl->words = (pl->narrow.LR * pl->narrow_fb + 15) / 16;
  pl->mean_words = (pl->mean.rcnt_max * pl->fb + 15) / 16;
  pl->shared_table = pl->grp == 1 && pl->narrow.R == pl->mean.R && pl->narrow.LR == pl->mean.rcnt_max;
  const int64_t table_bytes = sk ? (int64_t)pl->narrow.R * pl->dpad * pl->words * 2 : 0;
  const int64_t mean_table_bytes =
      sk && !pl->shared_table ? (int64_t)pl->mean.R * pl->dpad * pl->mean_words * 2 : 0;
  pl->off_mean_table = pl->shared_table ? pl->off_table : round_up(pl->off_table + table_bytes, kAlign);
  pl->ws_bytes = round_up(pl->off_mean_table + mean_table_bytes + (pl->shared_table ? table_bytes : 0), kAlign);
  return FDA_OK;
}

void export_plan(const Plan& pl, fda_plan_info* out) {
  out->worker_groups = pl.narrow.G;
  out->row_groups = pl.narrow.R;
  out->rows_per_group = pl.narrow.rcnt_max;
  out->workers_per_group = pl.narrow.kcnt_max;
  out->partitions = pl.narrow.P;
  out->threads = fda::kStateThreads;
  out->chunk = pl.narrow.chunk;
  out->lds_bytes = pl.narrow.lds_bytes;
  out->workspace_bytes = pl.ws_bytes;
  out->state_floats = pl.S;
  out->mean_row_groups = pl.mean.R;
  out->mean_rows_per_group = pl.mean.rcnt_max;
  out->mean_partitions = pl.mean.P;
  out->mean_workgroups_per_cu = pl.mean.occ;
  out->mean_chunk = pl.mean.chunk;
  out->mean_lds_bytes = pl.mean.lds_bytes;
  out->sign_split_rows = pl.narrow.split;
  out->worker_slots = pl.narrow.KC;
  out->placed_row_group = pl.grp >= 2 ? pl.grp : 0;
  out->reserved = 0;
}

int device_shape(int* cus, int64_t* lds) {
  int dev = 0;
  FDA_HIP(hipGetDevice(&dev));
  int v = 0;
  FDA_HIP(hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev));
  *cus = v;
  FDA_HIP(hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev));
  *lds = v;
  return FDA_OK;
}

// Whole-vector loads and stores only need the alignment of the element type, which every entry point
// checks of its pointers: the vector path is always available (the element-wise path of the kernels
// serves the ragged end of a vector).
constexpr int kVecOk = 1;

// Route a launch (or, with prm == nullptr, the LDS-limit setup) to the translation unit that
// holds the kernel for this slab type, cell kind and shape.
int dispatch_any(int dtype, int cell, const Split& sp, int FB, const fda::StateParams* prm, hipStream_t st) {
  const int KC = sp.KC, LR = sp.LR;
  const size_t lds = (size_t)sp.lds_bytes;
  hipError_t e = hipErrorInvalidValue;
  if (cell == fda::kCellI32) {
#define FDA_CASE(t, kc) case kc: e = fda::launch_narrow_##t##_kc##kc(LR, FB, sp.split, prm, lds, st); break
    if (dtype == FDA_F32) {
      switch (KC) { FDA_CASE(f32, 1); FDA_CASE(f32, 2); FDA_CASE(f32, 4); FDA_CASE(f32, 6); FDA_CASE(f32, 8); }
    } else {
      switch (KC) { FDA_CASE(bf16, 1); FDA_CASE(bf16, 2); FDA_CASE(bf16, 4); FDA_CASE(bf16, 6); FDA_CASE(bf16, 8); }
    }
#undef FDA_CASE
  } else if (dtype == FDA_F32) {
    e = cell == fda::kCellI64 ? fda::launch_wide_f32_i64(KC, LR, prm, lds, st)
                              : fda::launch_wide_f32_f64(KC, LR, prm, lds, st);
  } else {
    e = cell == fda::kCellI64 ? fda::launch_wide_bf16_i64(KC, LR, prm, lds, st)
                              : fda::launch_wide_bf16_f64(KC, LR, prm, lds, st);
  }
  if (e == hipErrorInvalidValue)
    return fail(FDA_EINVAL, "internal: no state kernel for %d workers x %d rows per workgroup", KC, LR);
  if (e != hipSuccess) return fail(FDA_EHIP, "state kernel launch failed: %s", hipGetErrorString(e));
  return FDA_OK;
}

int dispatch_mean(int dtype, int cell, const MeanSplit& ms, int FB, const fda::MeanParams* prm, hipStream_t st) {
  const size_t lds = (size_t)ms.lds_bytes;
  hipError_t e;
  if (dtype == FDA_F32)
    e = cell == fda::kCellI64 ? fda::launch_mean_f32_i64(ms.rcnt_max, FB, prm, lds, st)
                              : fda::launch_mean_f32_f64(ms.rcnt_max, FB, prm, lds, st);
  else
    e = cell == fda::kCellI64 ? fda::launch_mean_bf16_i64(ms.rcnt_max, FB, prm, lds, st)
                              : fda::launch_mean_bf16_f64(ms.rcnt_max, FB, prm, lds, st);
  if (e == hipErrorInvalidValue)
    return fail(FDA_EINVAL, "internal: no mean-state kernel for %d rows per workgroup", ms.rcnt_max);
  if (e != hipSuccess) return fail(FDA_EHIP, "mean-state kernel launch failed: %s", hipGetErrorString(e));
  return FDA_OK;
}

constexpr int kProfSlots = 64;

// Device address of `scratch` on the current device, looked up once per device (with that device
// current) and kept: each GPU has its own copy of the array at its own address.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[kMaxDevices] = {};

int static_scratch(unsigned char** out) {
  int dev = -1;
  FDA_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(FDA_ERANGE, "device ordinal %d is beyond %d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    FDA_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (p == nullptr) return fail(FDA_EHIP, "hipGetSymbolAddress returned a null address");
    g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
  }
  *out = g_scratch_ptr[dev];
  return FDA_OK;
}

}  // namespace

struct fda_ctx {
  fda_desc desc;
  fda::HashCoef coef;
  Plan plan;
  unsigned char* ws;
  int device;
  int cus;
  bool counted = false;       // cell_count_kernel has been enqueued for this context
  bool table_built = false;       // the hash table of the 32-bit-cell pass has been enqueued
  bool mean_table_built = false;  // ... of the mean-state pass (the same table when the plan shares it)
  bool tickets_cleared = false;
  // optional timing of the state kernel (fda_profile_enable)
  bool prof_on = false;
  hipEvent_t prof_start[kProfSlots] = {};
  hipEvent_t prof_stop[kProfSlots] = {};
  int prof_pending = 0;       // recorded pairs not yet read
  double prof_ms = 0.0;
  int64_t prof_launches = 0;
};

namespace {
// The finished-workgroup counters of scale_kernel and estimate_kernel start at zero and are left
// at zero by every launch; the workspace arrives uninitialised, so they are cleared once.
int clear_tickets_once(fda_ctx* c, hipStream_t st) {
  if (c->tickets_cleared) return FDA_OK;
  hipLaunchKernelGGL(fda::clear_u32_kernel, dim3(1), dim3(64), 0, st,
                     reinterpret_cast<unsigned int*>(c->ws + c->plan.off_ticket), 2);
  FDA_HIP(hipGetLastError());
  // ... and so are the two scale records, whose flags an estimate may report before any state pass ran
  static_assert(2 * sizeof(fda::ScaleInfo) <= 64 * 4, "clear_u32_kernel clears at most 64 words");
  hipLaunchKernelGGL(fda::clear_u32_kernel, dim3(1), dim3(64), 0, st,
                     reinterpret_cast<unsigned int*>(c->ws + c->plan.off_scale),
                     (int)(2 * sizeof(fda::ScaleInfo) / 4));
  FDA_HIP(hipGetLastError());
  c->tickets_cleared = true;
  return FDA_OK;
}

// Fold the recorded event pairs into the running totals (waits for them).
int prof_drain(fda_ctx* c) {
  for (int t = 0; t < c->prof_pending; ++t) {
    FDA_HIP(hipEventSynchronize(c->prof_stop[t]));
    float ms = 0.0f;
    FDA_HIP(hipEventElapsedTime(&ms, c->prof_start[t], c->prof_stop[t]));
    c->prof_ms += ms;
    c->prof_launches += 1;
  }
  c->prof_pending = 0;
  return FDA_OK;
}

// Start / stop of one timed kernel (fda_profile_enable); slot < 0: timing is off.
int prof_begin(fda_ctx* c, hipStream_t st, int* slot) {
  *slot = -1;
  if (!c->prof_on) return FDA_OK;
  if (c->prof_pending == kProfSlots) {
    int rc = prof_drain(c);
    if (rc != FDA_OK) return rc;
  }
  *slot = c->prof_pending;
  FDA_HIP(hipEventRecord(c->prof_start[*slot], st));
  return FDA_OK;
}
int prof_end(fda_ctx* c, hipStream_t st, int slot) {
  if (slot < 0) return FDA_OK;
  FDA_HIP(hipEventRecord(c->prof_stop[slot], st));
  c->prof_pending = slot + 1;
  return FDA_OK;
}

// Before the first sketch of a context: the hash table and the cell counts.  Then, per call, the
// fixed-point units from a sample of the drifts (this also clears the flags in *scale).
int build_table(fda_ctx* ctx, int R, int slots, int fb, int words, int grp, int KC, int64_t off, hipStream_t st) {
  const fda_desc& d = ctx->desc;
  const Plan& pl = ctx->plan;
  const long long groups = pl.dpad / 4;
  // what the kernel's arrays assume: at most 8 row slots, records of at most 8 words, placement groups of 2..8 rows
  if (slots < 1 || slots > 8 || words < 1 || words > 8 || grp < 1 || grp > 8 || slots * fb > words * 16)
    return fail(FDA_EINVAL, "table shape out of range: %d slots of %d bits in %d words, groups of %d", slots, fb, words, grp);
  hipLaunchKernelGGL(fda::hash_table_kernel,
                     dim3((unsigned)((groups + fda::kSmallThreads - 1) / fda::kSmallThreads), (unsigned)R),
                     dim3(fda::kSmallThreads), 0, st, ctx->coef, d.l, R, slots, d.m, fb, words, grp, KC,
                     (long long)d.d, (long long)pl.dpad, reinterpret_cast<uint16_t*>(ctx->ws + off));
  FDA_HIP(hipGetLastError());
  return FDA_OK;
}

// for_mean: the call is fda_mean_state (else fda_local_state): which table must exist
int prepare_sketch(fda_ctx* ctx, const void* w, const float* w_t0, fda::ScaleInfo* scale, bool for_mean,
                   hipStream_t st) {
  const fda_desc& d = ctx->desc;
  const Plan& pl = ctx->plan;
  int rc0 = clear_tickets_once(ctx, st);
  if (rc0 != FDA_OK) return rc0;
  float* smax = reinterpret_cast<float*>(ctx->ws + pl.off_smax);
  double* ssum = reinterpret_cast<double*>(ctx->ws + pl.off_ssum);
  unsigned int* nmax = reinterpret_cast<unsigned int*>(ctx->ws + pl.off_nmax);
  if (!ctx->counted) {
    // once per context: the largest number of coordinates any workgroup puts in one cell,
    // for the partitioning of the 32-bit pass ([0]) and of the 8-byte passes ([1]) ...
    hipLaunchKernelGGL(fda::clear_u32_kernel, dim3(1), dim3(64), 0, st, nmax, 2);
    FDA_HIP(hipGetLastError());
    hipLaunchKernelGGL(fda::cell_count_kernel, dim3(pl.narrow.P * d.l), dim3(fda::kStateThreads),
                       (size_t)d.m * 4 * (pl.narrow.split ? 2 : 1), st, ctx->coef, d.l, d.m, pl.narrow.split,
                       (long long)d.d, (long long)pl.narrow.chunk, nmax);
    FDA_HIP(hipGetLastError());
    hipLaunchKernelGGL(fda::cell_count_kernel, dim3(pl.wide.P * d.l), dim3(fda::kStateThreads),
                       (size_t)d.m * 4, st, ctx->coef, d.l, d.m, 0, (long long)d.d,
                       (long long)pl.wide.chunk, nmax + 1);
    FDA_HIP(hipGetLastError());
    ctx->counted = true;
  }
  // ... and the hash of every (row, coordinate), tabulated for the pass that is about to run
  if (!for_mean && !ctx->table_built) {
    int rc = build_table(ctx, pl.narrow.R, pl.narrow.LR, pl.narrow_fb, pl.words, pl.grp, pl.narrow.KC, pl.off_table, st);
    if (rc != FDA_OK) return rc;
    ctx->table_built = true;
    if (pl.shared_table) ctx->mean_table_built = true;
  }
  if (for_mean && !ctx->mean_table_built) {
    int rc = build_table(ctx, pl.mean.R, pl.mean.rcnt_max, pl.fb, pl.mean_words, 1, 1, pl.off_mean_table, st);
    if (rc != FDA_OK) return rc;
    ctx->mean_table_built = true;
    if (pl.shared_table) ctx->table_built = true;
  }
  const int samples = (int)(d.d < kScaleSamples ? d.d : kScaleSamples);
  int slices = (d.K + 7) / 8;                 // about eight workers per thread
  if (slices > fda::kScaleMaxSlices) slices = fda::kScaleMaxSlices;
  const int sblocks = (samples * slices + fda::kSmallThreads - 1) / fda::kSmallThreads;
  unsigned int* ticket = reinterpret_cast<unsigned int*>(ctx->ws + pl.off_ticket);
  if (d.dtype == FDA_F32)
    hipLaunchKernelGGL(fda::scale_kernel<float>, dim3(sblocks), dim3(fda::kSmallThreads), 0, st,
                       static_cast<const float*>(w), w_t0, d.K, (long long)d.d, (long long)d.row_stride,
                       samples, slices, smax, ssum, ticket, nmax, scale);
  else
    hipLaunchKernelGGL(fda::scale_kernel<fda::bf16_t>, dim3(sblocks), dim3(fda::kSmallThreads), 0, st,
                       static_cast<const fda::bf16_t*>(w), w_t0, d.K, (long long)d.d,
                       (long long)d.row_stride, samples, slices, smax, ssum, ticket, nmax, scale);
  FDA_HIP(hipGetLastError());
  return FDA_OK;
}

// Launches go to the current device: it must be the one the context (and its workspace) lives on.
int check_device(const fda_ctx* ctx) {
  int dev = -1;
  FDA_HIP(hipGetDevice(&dev));
  if (dev != ctx->device)
    return fail(FDA_EINVAL, "the context was created on device %d but device %d is current", ctx->device, dev);
  return FDA_OK;
}

// The argument checks fda_local_state and fda_mean_state share.
int check_state_args(const fda_ctx* ctx, const void* w, const float* w_t0, const float* xi, const float* out) {
  if (ctx == nullptr || w == nullptr || w_t0 == nullptr || out == nullptr)
    return fail(FDA_EINVAL, "NULL argument");
  int rcd = check_device(ctx);
  if (rcd != FDA_OK) return rcd;
  const fda_desc& d = ctx->desc;
  if ((d.variants & FDA_VARIANT_LINEAR) && xi == nullptr)
    return fail(FDA_EINVAL, "xi is NULL but FDA_VARIANT_LINEAR is requested");
  const int esz = d.dtype == FDA_F32 ? 4 : 2;
  if (reinterpret_cast<uintptr_t>(w) % esz != 0 || reinterpret_cast<uintptr_t>(w_t0) % 4 != 0 ||
      reinterpret_cast<uintptr_t>(out) % 4 != 0 || (xi && reinterpret_cast<uintptr_t>(xi) % 4 != 0))
    return fail(FDA_EINVAL, "pointer not aligned to its element type");
  return FDA_OK;
}
}  // namespace

extern "C" {

const char* fda_strerror(int code) {
  switch (code) {
    case FDA_OK: return "success";
    case FDA_EINVAL: return "invalid argument";
    case FDA_ERANGE: return "value out of the supported range";
    case FDA_ENOMEM: return "workspace too small";
    case FDA_EHIP: return "HIP runtime error";
  }
  return "unknown error code";
}

const char* fda_last_error(void) { return g_err; }

int fda_plan(const fda_desc* desc, int32_t compute_units, int64_t lds_bytes_per_cu,
             fda_plan_info* out) {
  if (out == nullptr) return fail(FDA_EINVAL, "out is NULL");
  int rc = validate(desc);
  if (rc != FDA_OK) return rc;
  Plan pl;
  rc = make_plan(desc, compute_units, lds_bytes_per_cu, &pl);
  if (rc != FDA_OK) return rc;
  export_plan(pl, out);
  return FDA_OK;
}

int fda_workspace_bytes(const fda_desc* desc, size_t* bytes) {
  if (bytes == nullptr) return fail(FDA_EINVAL, "bytes is NULL");
  int rc = validate(desc);
  if (rc != FDA_OK) return rc;
  int cus = 0;
  int64_t lds = 0;
  rc = device_shape(&cus, &lds);
  if (rc != FDA_OK) return rc;
  Plan pl;
  rc = make_plan(desc, cus, lds, &pl);
  if (rc != FDA_OK) return rc;
  *bytes = (size_t)pl.ws_bytes;
  return FDA_OK;
}

int fda_create(fda_ctx** ctx, const fda_desc* desc, void* workspace, size_t workspace_bytes) {
  if (ctx == nullptr) return fail(FDA_EINVAL, "ctx is NULL");
  *ctx = nullptr;
  int rc = validate(desc);
  if (rc != FDA_OK) return rc;
  if (workspace == nullptr) return fail(FDA_EINVAL, "workspace is NULL");
  if (reinterpret_cast<uintptr_t>(workspace) % kAlign != 0)
    return fail(FDA_EINVAL, "workspace must be 256-byte aligned");
  int cus = 0;
  int64_t lds = 0;
  rc = device_shape(&cus, &lds);
  if (rc != FDA_OK) return rc;
  Plan pl;
  rc = make_plan(desc, cus, lds, &pl);
  if (rc != FDA_OK) return rc;
  if ((int64_t)workspace_bytes < pl.ws_bytes)
    return fail(FDA_ENOMEM, "workspace has %zu bytes, %lld needed", workspace_bytes, (long long)pl.ws_bytes);
  fda_ctx* c = new (std::nothrow) fda_ctx;
  if (c == nullptr) return fail(FDA_ENOMEM, "out of host memory");
  c->desc = *desc;
  c->desc.hash_coef = nullptr;
  std::memset(&c->coef, 0, sizeof(c->coef));
  if (desc->variants & FDA_VARIANT_SKETCH)
    std::memcpy(&c->coef, desc->hash_coef, sizeof(uint32_t) * 8 * desc->l);
  c->plan = pl;
  c->ws = static_cast<unsigned char*>(workspace);
  c->cus = cus;
  if (hipGetDevice(&c->device) != hipSuccess) {
    delete c;
    return fail(FDA_EHIP, "hipGetDevice failed");
  }
  // The dynamic-LDS limit of a kernel is one setting per process: raise it to everything the
  // device allows, so that a context created later with a smaller sketch cannot lower it under
  // what an earlier context's launches need.
  Split narrow_max = pl.narrow, wide_max = pl.wide;
  MeanSplit mean_max = pl.mean;
  narrow_max.lds_bytes = wide_max.lds_bytes = mean_max.lds_bytes = lds;
  rc = dispatch_any(desc->dtype, fda::kCellI32, narrow_max, pl.narrow_fb, nullptr, nullptr);
  if (rc == FDA_OK) rc = dispatch_mean(desc->dtype, fda::kCellI64, mean_max, pl.fb, nullptr, nullptr);
  if (rc == FDA_OK && (desc->variants & FDA_VARIANT_SKETCH))
    rc = dispatch_mean(desc->dtype, fda::kCellF64, mean_max, pl.fb, nullptr, nullptr);
  if (rc == FDA_OK && (desc->variants & FDA_VARIANT_SKETCH)) {
    rc = dispatch_any(desc->dtype, fda::kCellI64, wide_max, pl.fb, nullptr, nullptr);
    if (rc == FDA_OK) rc = dispatch_any(desc->dtype, fda::kCellF64, wide_max, pl.fb, nullptr, nullptr);
    if (rc == FDA_OK &&
        hipFuncSetAttribute(reinterpret_cast<const void*>(fda::cell_count_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds - 1024) != hipSuccess)   // the kernel also has a little static LDS
      rc = fail(FDA_EHIP, "hipFuncSetAttribute(cell_count_kernel) failed");
  }
  if (rc != FDA_OK) {
    delete c;
    return rc;
  }
  *ctx = c;
  return FDA_OK;
}

int fda_destroy(fda_ctx* ctx) {
  if (ctx == nullptr) return FDA_OK;
  for (int t = 0; t < kProfSlots; ++t) {
    if (ctx->prof_start[t]) (void)hipEventDestroy(ctx->prof_start[t]);
    if (ctx->prof_stop[t]) (void)hipEventDestroy(ctx->prof_stop[t]);
  }
  delete ctx;
  return FDA_OK;
}

int fda_last_state_path(fda_ctx* ctx, int32_t* path, void* stream) {
  if (ctx == nullptr || path == nullptr) return fail(FDA_EINVAL, "NULL argument");
  if (!(ctx->desc.variants & FDA_VARIANT_SKETCH)) { *path = -1; return FDA_OK; }
  hipStream_t st = static_cast<hipStream_t>(stream);
  fda::ScaleInfo info;
  FDA_HIP(hipMemcpyAsync(&info, ctx->ws + ctx->plan.off_scale, sizeof(info), hipMemcpyDeviceToHost, st));
  FDA_HIP(hipStreamSynchronize(st));
  *path = info.overflow64 ? 2 : (info.flag32 ? 1 : 0);
  return FDA_OK;
}

int fda_last_mean_state_path(fda_ctx* ctx, int32_t* path, void* stream) {
  if (ctx == nullptr || path == nullptr) return fail(FDA_EINVAL, "NULL argument");
  if (!(ctx->desc.variants & FDA_VARIANT_SKETCH)) { *path = -1; return FDA_OK; }
  hipStream_t st = static_cast<hipStream_t>(stream);
  fda::ScaleInfo info;
  FDA_HIP(hipMemcpyAsync(&info, ctx->ws + ctx->plan.off_scale + sizeof(fda::ScaleInfo), sizeof(info),
                         hipMemcpyDeviceToHost, st));
  FDA_HIP(hipStreamSynchronize(st));
  *path = info.flagm ? 1 : 0;
  return FDA_OK;
}

int fda_profile_enable(fda_ctx* ctx, int on) {
  if (ctx == nullptr) return fail(FDA_EINVAL, "ctx is NULL");
  if (on && ctx->prof_start[0] == nullptr) {
    for (int t = 0; t < kProfSlots; ++t) {
      FDA_HIP(hipEventCreate(&ctx->prof_start[t]));
      FDA_HIP(hipEventCreate(&ctx->prof_stop[t]));
    }
  }
  if (!on) {
    int rc = prof_drain(ctx);
    if (rc != FDA_OK) return rc;
  }
  ctx->prof_on = on != 0;
  return FDA_OK;
}

int fda_profile_read(fda_ctx* ctx, double* state_kernel_ms, int64_t* launches, int reset) {
  if (ctx == nullptr || state_kernel_ms == nullptr || launches == nullptr)
    return fail(FDA_EINVAL, "NULL argument");
  int rc = prof_drain(ctx);
  if (rc != FDA_OK) return rc;
  *state_kernel_ms = ctx->prof_ms;
  *launches = ctx->prof_launches;
  if (reset) { ctx->prof_ms = 0.0; ctx->prof_launches = 0; }
  return FDA_OK;
}

int fda_state_floats(const fda_ctx* ctx, int64_t* S) {
  if (ctx == nullptr || S == nullptr) return fail(FDA_EINVAL, "NULL argument");
  *S = ctx->plan.S;
  return FDA_OK;
}

int fda_get_plan(const fda_ctx* ctx, fda_plan_info* out) {
  if (ctx == nullptr || out == nullptr) return fail(FDA_EINVAL, "NULL argument");
  export_plan(ctx->plan, out);
  return FDA_OK;
}

int fda_local_state(fda_ctx* ctx, const void* w, const float* w_t0, const float* xi,
                    float* state, void* stream) {
  int rc = check_state_args(ctx, w, w_t0, xi, state);
  if (rc != FDA_OK) return rc;
  const fda_desc& d = ctx->desc;
  const Plan& pl = ctx->plan;
  const bool lin = (d.variants & FDA_VARIANT_LINEAR) != 0;
  const bool sk = (d.variants & FDA_VARIANT_SKETCH) != 0;
  hipStream_t st = static_cast<hipStream_t>(stream);

  auto params_for = [&](const Split& sp) {
    fda::StateParams prm;
    prm.w = w; prm.w_t0 = w_t0; prm.xi = xi;
    prm.row_stride = d.row_stride; prm.d = d.d; prm.chunk = sp.chunk;
    prm.K = d.K; prm.l = sk ? d.l : 0; prm.m = sk ? d.m : 0;
    prm.G = sp.G; prm.R = sp.R; prm.P = sp.P; prm.stride = sp.stride;
    prm.do_lin = lin; prm.do_sk = sk;
    prm.vec_ok = kVecOk;
    prm.part_np = reinterpret_cast<double*>(ctx->ws + pl.off_np);
    prm.part_sk = ctx->ws + pl.off_sk;
    prm.scale = reinterpret_cast<fda::ScaleInfo*>(ctx->ws + pl.off_scale);
    prm.table = reinterpret_cast<const uint16_t*>(ctx->ws + pl.off_table);
    prm.dpad = pl.dpad;
    prm.grp = &sp == &pl.narrow ? pl.grp : 1;
    prm.coef = ctx->coef;
    return prm;
  };
  const fda::StateParams prm32 = params_for(pl.narrow);
  const fda::StateParams prm64 = params_for(pl.wide);

  if (sk) {
    rc = prepare_sketch(ctx, w, w_t0, prm32.scale, false, st);
    if (rc != FDA_OK) return rc;
  }
  int slot = -1;
  rc = prof_begin(ctx, st, &slot);
  if (rc != FDA_OK) return rc;
  rc = dispatch_any(d.dtype, fda::kCellI32, pl.narrow, pl.narrow_fb, &prm32, st);
  if (rc != FDA_OK) return rc;
  rc = prof_end(ctx, st, slot);
  if (rc != FDA_OK) return rc;
  if (sk) {
    // these two return at once unless the pass before them could not represent the drifts
    rc = dispatch_any(d.dtype, fda::kCellI64, pl.wide, pl.fb, &prm64, st);
    if (rc != FDA_OK) return rc;
    rc = dispatch_any(d.dtype, fda::kCellF64, pl.wide, pl.fb, &prm64, st);
    if (rc != FDA_OK) return rc;
  }

  const long long total = (long long)d.K * pl.S;
  const int blocks = (int)((total + 31) / 32);
  hipLaunchKernelGGL(fda::merge_kernel, dim3(blocks), dim3(fda::kSmallThreads), 0, st,
                     prm32.part_np, prm32.part_sk, prm32.scale, state, d.K, (int)pl.cells,
                     pl.narrow.P, pl.wide.P);
  FDA_HIP(hipGetLastError());
  return FDA_OK;
}

int fda_mean_state(fda_ctx* ctx, const void* w, const float* w_t0, const float* xi,
                   float* mean_state, float* w_bar, void* stream) {
  int rc = check_state_args(ctx, w, w_t0, xi, mean_state);
  if (rc != FDA_OK) return rc;
  const fda_desc& d = ctx->desc;
  const Plan& pl = ctx->plan;
  const MeanSplit& ms = pl.mean;
  const bool lin = (d.variants & FDA_VARIANT_LINEAR) != 0;
  const bool sk = (d.variants & FDA_VARIANT_SKETCH) != 0;
  // a cell's integer sum stays below K * chunk * 2^30 in magnitude
  if (sk && (double)d.K * (double)ms.chunk >= 8589934592.0)
    return fail(FDA_ERANGE, "K * coordinates per workgroup must stay below 2^33");
  if (w_bar != nullptr && reinterpret_cast<uintptr_t>(w_bar) % 4 != 0)
    return fail(FDA_EINVAL, "pointer not aligned to its element type");
  hipStream_t st = static_cast<hipStream_t>(stream);

  fda::MeanParams prm;
  prm.w = w; prm.w_t0 = w_t0; prm.xi = xi;
  prm.row_stride = d.row_stride; prm.d = d.d; prm.chunk = ms.chunk;
  prm.K = d.K; prm.l = sk ? d.l : 0; prm.m = sk ? d.m : 0;
  prm.R = ms.R; prm.P = ms.P;
  prm.do_lin = lin; prm.do_sk = sk;
  prm.vec_ok = kVecOk;
  prm.w_bar = w_bar;
  prm.part_np = reinterpret_cast<double*>(ctx->ws + pl.off_np);
  prm.part_sk = ctx->ws + pl.off_sk;
  prm.scale = reinterpret_cast<fda::ScaleInfo*>(ctx->ws + pl.off_scale) + 1;
  prm.table = reinterpret_cast<const uint16_t*>(ctx->ws + pl.off_mean_table);
  prm.dpad = pl.dpad;

  if (sk) {
    rc = prepare_sketch(ctx, w, w_t0, prm.scale, true, st);
    if (rc != FDA_OK) return rc;
  }
  int slot = -1;
  rc = prof_begin(ctx, st, &slot);
  if (rc != FDA_OK) return rc;
  rc = dispatch_mean(d.dtype, fda::kCellI64, ms, pl.fb, &prm, st);
  if (rc != FDA_OK) return rc;
  rc = prof_end(ctx, st, slot);
  if (rc != FDA_OK) return rc;
  if (sk) {
    // returns at once unless a drift was too large for the integers
    rc = dispatch_mean(d.dtype, fda::kCellF64, ms, pl.fb, &prm, st);
    if (rc != FDA_OK) return rc;
  }
  const int blocks = (int)((pl.S + 1 + 31) / 32);
  hipLaunchKernelGGL(fda::merge_mean_kernel, dim3(blocks), dim3(fda::kSmallThreads), 0, st,
                     prm.part_np, prm.part_sk, prm.scale, mean_state,
                     reinterpret_cast<double*>(ctx->ws + pl.off_dnorm), d.K, (int)pl.cells, ms.P);
  FDA_HIP(hipGetLastError());
  return FDA_OK;
}

static int estimate_rows(fda_ctx* ctx, const float* state, int rows, int mean_mode, double theta, double tie_tol,
                         fda_estimate* out_dev, fda_estimate* out_host, void* stream) {
  if (ctx == nullptr || state == nullptr || out_dev == nullptr)
    return fail(FDA_EINVAL, "NULL argument");
  if (reinterpret_cast<uintptr_t>(out_dev) % 8 != 0) return fail(FDA_EINVAL, "out_dev must be 8-byte aligned");
  int rcd = check_device(ctx);
  if (rcd != FDA_OK) return rcd;
  if (!(tie_tol >= 0.0)) return fail(FDA_EINVAL, "tie_tol must be >= 0");
  const fda_desc& d = ctx->desc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool sk = (d.variants & FDA_VARIANT_SKETCH) != 0;
  const int bpr = (d.m + fda::kEstCols - 1) / fda::kEstCols;
  const int eblocks = sk ? d.l * bpr : 1;
  int rc = clear_tickets_once(ctx, st);
  if (rc != FDA_OK) return rc;
  const fda::ScaleInfo* scale =
      reinterpret_cast<const fda::ScaleInfo*>(ctx->ws + ctx->plan.off_scale) + (mean_mode ? 1 : 0);
  hipLaunchKernelGGL(fda::estimate_kernel, dim3(eblocks), dim3(fda::kSmallThreads), 0, st, state, rows,
                     sk ? d.l : 0, sk ? d.m : 1, d.variants, d.eps, theta, tie_tol,
                     reinterpret_cast<double*>(ctx->ws + ctx->plan.off_est),
                     reinterpret_cast<unsigned int*>(ctx->ws + ctx->plan.off_ticket) + 1, scale, mean_mode,
                     out_dev);
  FDA_HIP(hipGetLastError());
  if (out_host != nullptr) {
    FDA_HIP(hipMemcpyAsync(out_host, out_dev, sizeof(fda_estimate), hipMemcpyDeviceToHost, st));
    FDA_HIP(hipStreamSynchronize(st));
  }
  return FDA_OK;
}

int fda_estimate_variance(fda_ctx* ctx, const float* state, double theta, double tie_tol,
                          fda_estimate* out_dev, fda_estimate* out_host, void* stream) {
  return estimate_rows(ctx, state, ctx ? ctx->desc.K : 0, 0, theta, tie_tol, out_dev, out_host, stream);
}

int fda_estimate_variance_mean(fda_ctx* ctx, const float* mean_state, double theta, double tie_tol,
                               fda_estimate* out_dev, fda_estimate* out_host, void* stream) {
  return estimate_rows(ctx, mean_state, 1, 1, theta, tie_tol, out_dev, out_host, stream);
}

int fda_estimate_variance_static(const float* state, int32_t K, int32_t l, int32_t m, int32_t variants,
                                 double eps, double theta, double tie_tol, fda_estimate* out_dev,
                                 void* stream) {
  if (state == nullptr || out_dev == nullptr) return fail(FDA_EINVAL, "NULL argument");
  if (reinterpret_cast<uintptr_t>(state) % 4 != 0 || reinterpret_cast<uintptr_t>(out_dev) % 8 != 0)
    return fail(FDA_EINVAL, "state must be 4-byte and out_dev 8-byte aligned");
  if (K < 1) return fail(FDA_EINVAL, "K must be >= 1 (got %d)", K);
  if ((variants & ~(FDA_VARIANT_LINEAR | FDA_VARIANT_SKETCH)) != 0 || variants == 0)
    return fail(FDA_EINVAL, "variants must be a non-empty mask of FDA_VARIANT_LINEAR | FDA_VARIANT_SKETCH");
  if (!(tie_tol >= 0.0)) return fail(FDA_EINVAL, "tie_tol must be >= 0");
  const bool sk = (variants & FDA_VARIANT_SKETCH) != 0;
  if (sk) {
    if (l < 1 || l > FDA_MAX_SKETCH_ROWS)
      return fail(FDA_ERANGE, "l must be in 1..%d (got %d): the static scratch holds no more rows", FDA_MAX_SKETCH_ROWS, l);
    if (m < 1 || m > FDA_STATIC_MAX_M)
      return fail(FDA_ERANGE, "m must be in 1..%d (got %d): the static scratch holds no wider rows", FDA_STATIC_MAX_M, m);
    if (!(eps > -1.0)) return fail(FDA_EINVAL, "eps must be > -1");
  }
  const int bpr = sk ? (m + fda::kEstCols - 1) / fda::kEstCols : 1;
  const int eblocks = sk ? l * bpr : 1;
  if ((size_t)(2 + eblocks) > kStaticPartDoubles)
    return fail(FDA_ERANGE, "internal: %d partial sums do not fit the static scratch", 2 + eblocks);
  unsigned char* base = nullptr;
  int rc = static_scratch(&base);
  if (rc != FDA_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  unsigned int* ticket = reinterpret_cast<unsigned int*>(base + kStaticTicketOffset);
  // the counter must start at zero whatever an earlier call left (a fill kernel, not a memset node)
  hipLaunchKernelGGL(fda::clear_u32_kernel, dim3(1), dim3(64), 0, st, ticket, 1);
  FDA_HIP(hipGetLastError());
  hipLaunchKernelGGL(fda::estimate_kernel, dim3(eblocks), dim3(fda::kSmallThreads), 0, st, state, K,
                     sk ? l : 0, sk ? m : 1, variants, eps, theta, tie_tol,
                     reinterpret_cast<double*>(base), ticket, static_cast<const fda::ScaleInfo*>(nullptr), 0,
                     out_dev);
  FDA_HIP(hipGetLastError());
  return FDA_OK;
}

namespace {
int sync_impl(fda_ctx* ctx, void* w, float* w_t0, float* w_prev, float* xi, const int32_t* pred_dev,
              void* stream);
}
int fda_sync(fda_ctx* ctx, void* w, float* w_t0, float* w_prev, const int32_t* pred_dev,
             void* stream) {
  return sync_impl(ctx, w, w_t0, w_prev, nullptr, pred_dev, stream);
}
int fda_sync_xi(fda_ctx* ctx, void* w, float* w_t0, float* w_prev, float* xi, const int32_t* pred_dev,
                void* stream) {
  if (w_prev == nullptr || xi == nullptr) return fail(FDA_EINVAL, "NULL argument");
  if (reinterpret_cast<uintptr_t>(xi) % 4 != 0) return fail(FDA_EINVAL, "pointer not aligned to its element type");
  return sync_impl(ctx, w, w_t0, w_prev, xi, pred_dev, stream);
}
namespace {
// xi != NULL: the synchronization kernel also leaves the squared norm of the model change, and xi is
// written by the scaling pass of fda_update_xi alone
int sync_impl(fda_ctx* ctx, void* w, float* w_t0, float* w_prev, float* xi, const int32_t* pred_dev,
              void* stream) {
  if (ctx == nullptr || w == nullptr || w_t0 == nullptr) return fail(FDA_EINVAL, "NULL argument");
  int rcd = check_device(ctx);
  if (rcd != FDA_OK) return rcd;
  const fda_desc& d = ctx->desc;
  const uintptr_t esz = d.dtype == FDA_F32 ? 4 : 2;
  if (reinterpret_cast<uintptr_t>(w) % esz != 0 || reinterpret_cast<uintptr_t>(w_t0) % 4 != 0 ||
      (w_prev && reinterpret_cast<uintptr_t>(w_prev) % 4 != 0))
    return fail(FDA_EINVAL, "pointer not aligned to its element type");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int vec_ok = kVecOk;
  const int V = fda::kSyncV;
  const long long nvec = (d.d + V - 1) / V;
  const long long blocks = (nvec + kSyncVectorsPerBlock - 1) / kSyncVectorsPerBlock;
  const bool hinted = (long long)d.K * d.d * (d.dtype == FDA_F32 ? 4 : 2) > kStreamBytes;
  const dim3 grid((unsigned)blocks), block(fda::kSmallThreads);
  double* norm_part = xi != nullptr ? reinterpret_cast<double*>(ctx->ws + ctx->plan.off_syncnorm) : nullptr;
#define FDA_SYNC_LAUNCH(T, S)                                                                          \
  hipLaunchKernelGGL((fda::sync_kernel<T, S>), grid, block, 0, st, static_cast<T*>(w), w_t0, w_prev,   \
                     pred_dev, d.K, (long long)d.d, (long long)d.row_stride, vec_ok, norm_part)
  if (d.dtype == FDA_F32) { if (hinted) FDA_SYNC_LAUNCH(float, true); else FDA_SYNC_LAUNCH(float, false); }
  else { if (hinted) FDA_SYNC_LAUNCH(fda::bf16_t, true); else FDA_SYNC_LAUNCH(fda::bf16_t, false); }
#undef FDA_SYNC_LAUNCH
  FDA_HIP(hipGetLastError());
  if (xi != nullptr) {
    // the partial norms -> a few (fixed order), then the scaling pass: xi = (w_t0 - w_prev) / norm
    double* total = norm_part + blocks;
    hipLaunchKernelGGL(fda::sum_partials_kernel, dim3(kSyncNormSlices), dim3(fda::kSmallThreads), 0, st,
                       norm_part, blocks, pred_dev, total);
    FDA_HIP(hipGetLastError());
    const long long items = vec_ok ? (d.d + 3) / 4 : d.d;
    long long sblocks = (items + fda::kSmallThreads - 1) / fda::kSmallThreads;
    const long long cap = (long long)ctx->cus * 16;
    if (sblocks > cap) sblocks = cap;
    if (sblocks < 1) sblocks = 1;
    hipLaunchKernelGGL(fda::xi_scale_kernel, dim3((unsigned)sblocks), dim3(fda::kSmallThreads), 0, st,
                       w_t0, w_prev, xi, pred_dev, (long long)d.d, vec_ok, total, kSyncNormSlices);
    FDA_HIP(hipGetLastError());
  }
  return FDA_OK;
}
}  // namespace

int fda_sync_from_mean(fda_ctx* ctx, void* w, float* w_t0, float* w_prev, float* xi,
                       const float* w_bar, const int32_t* pred_dev, void* stream) {
  if (ctx == nullptr || w == nullptr || w_t0 == nullptr || w_bar == nullptr)
    return fail(FDA_EINVAL, "NULL argument");
  int rcd = check_device(ctx);
  if (rcd != FDA_OK) return rcd;
  const fda_desc& d = ctx->desc;
  const uintptr_t esz = d.dtype == FDA_F32 ? 4 : 2;
  if (reinterpret_cast<uintptr_t>(w) % esz != 0 || reinterpret_cast<uintptr_t>(w_t0) % 4 != 0 ||
      reinterpret_cast<uintptr_t>(w_bar) % 4 != 0 || (w_prev && reinterpret_cast<uintptr_t>(w_prev) % 4 != 0) ||
      (xi && reinterpret_cast<uintptr_t>(xi) % 4 != 0))
    return fail(FDA_EINVAL, "pointer not aligned to its element type");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int vec_ok = kVecOk;
  const int V = fda::kSyncV;
  const long long nvec = (d.d + V - 1) / V;
  const long long blocks = (nvec + kSyncVectorsPerBlock - 1) / kSyncVectorsPerBlock;
  const bool hinted = (long long)d.K * d.d * (d.dtype == FDA_F32 ? 4 : 2) > kStreamBytes;
  const dim3 grid((unsigned)blocks), block(fda::kSmallThreads);
  const double* dnorm = reinterpret_cast<const double*>(ctx->ws + ctx->plan.off_dnorm);
#define FDA_SYNC_LAUNCH(T, S)                                                                          \
  hipLaunchKernelGGL((fda::sync_from_mean_kernel<T, S>), grid, block, 0, st, static_cast<T*>(w), w_t0, \
                     w_prev, xi, w_bar, dnorm, pred_dev, d.K, (long long)d.d, (long long)d.row_stride, vec_ok)
  if (d.dtype == FDA_F32) { if (hinted) FDA_SYNC_LAUNCH(float, true); else FDA_SYNC_LAUNCH(float, false); }
  else { if (hinted) FDA_SYNC_LAUNCH(fda::bf16_t, true); else FDA_SYNC_LAUNCH(fda::bf16_t, false); }
#undef FDA_SYNC_LAUNCH
  FDA_HIP(hipGetLastError());
  return FDA_OK;
}

int fda_update_xi(fda_ctx* ctx, const float* w_t0, const float* w_prev, float* xi,
                  const int32_t* pred_dev, void* stream) {
  if (ctx == nullptr || w_t0 == nullptr || w_prev == nullptr || xi == nullptr)
    return fail(FDA_EINVAL, "NULL argument");
  int rcd = check_device(ctx);
  if (rcd != FDA_OK) return rcd;
  const fda_desc& d = ctx->desc;
  if (reinterpret_cast<uintptr_t>(w_t0) % 4 != 0 || reinterpret_cast<uintptr_t>(w_prev) % 4 != 0 ||
      reinterpret_cast<uintptr_t>(xi) % 4 != 0)
    return fail(FDA_EINVAL, "pointer not aligned to its element type");
  hipStream_t st = static_cast<hipStream_t>(stream);
  double* partial = reinterpret_cast<double*>(ctx->ws + ctx->plan.off_xi);
  const int vec_ok = kVecOk;
  const long long items = vec_ok ? (d.d + 3) / 4 : d.d;       // what one thread takes per loop trip
  long long blocks = (items + fda::kSmallThreads * 4 - 1) / (fda::kSmallThreads * 4);
  if (blocks > kXiBlocks) blocks = kXiBlocks;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(fda::xi_norm_kernel, dim3((unsigned)blocks), dim3(fda::kSmallThreads), 0, st,
                     w_t0, w_prev, pred_dev, (long long)d.d, vec_ok, partial);
  FDA_HIP(hipGetLastError());
  long long sblocks = (items + fda::kSmallThreads - 1) / fda::kSmallThreads;
  const long long cap = (long long)ctx->cus * 16;
  if (sblocks > cap) sblocks = cap;
  if (sblocks < 1) sblocks = 1;
  hipLaunchKernelGGL(fda::xi_scale_kernel, dim3((unsigned)sblocks), dim3(fda::kSmallThreads), 0, st,
                     w_t0, w_prev, xi, pred_dev, (long long)d.d, vec_ok, partial, (int)blocks);
  FDA_HIP(hipGetLastError());
  return FDA_OK;
}

int fda_step(fda_ctx* ctx, void* w, float* w_t0, float* w_prev, float* xi, float* state, float* w_bar,
             double theta, double tie_tol, int32_t decide_by, int32_t flags, fda_estimate* out_dev,
             fda_estimate* out_host, void* stream) {
  if (ctx == nullptr || out_dev == nullptr) return fail(FDA_EINVAL, "NULL argument");
  if ((decide_by != FDA_VARIANT_LINEAR && decide_by != FDA_VARIANT_SKETCH) ||
      !(ctx->desc.variants & decide_by))
    return fail(FDA_EINVAL, "decide_by must be one of the context's variants");
  if ((flags & ~FDA_STEP_MEAN_STATE) != 0) return fail(FDA_EINVAL, "unknown flags");
  if (xi != nullptr && w_prev == nullptr) return fail(FDA_EINVAL, "w_prev is required when xi is given");
  const bool mean = (flags & FDA_STEP_MEAN_STATE) != 0;
  if (!mean && w_bar != nullptr) return fail(FDA_EINVAL, "w_bar needs FDA_STEP_MEAN_STATE");
  const int32_t* pred = reinterpret_cast<const int32_t*>(
      reinterpret_cast<const unsigned char*>(out_dev) +
      (decide_by == FDA_VARIANT_LINEAR ? offsetof(fda_estimate, sync_linear)
                                       : offsetof(fda_estimate, sync_sketch)));
  int rc;
  if (mean) {
    rc = fda_mean_state(ctx, w, w_t0, xi, state, w_bar, stream);
    if (rc != FDA_OK) return rc;
    rc = fda_estimate_variance_mean(ctx, state, theta, tie_tol, out_dev, nullptr, stream);
  } else {
    rc = fda_local_state(ctx, w, w_t0, xi, state, stream);
    if (rc != FDA_OK) return rc;
    rc = fda_estimate_variance(ctx, state, theta, tie_tol, out_dev, nullptr, stream);
  }
  if (rc != FDA_OK) return rc;
  if (w_bar != nullptr) {
    rc = fda_sync_from_mean(ctx, w, w_t0, w_prev, xi, w_bar, pred, stream);
  } else {
    rc = xi != nullptr ? fda_sync_xi(ctx, w, w_t0, w_prev, xi, pred, stream)
                       : fda_sync(ctx, w, w_t0, w_prev, pred, stream);
  }
  if (rc != FDA_OK) return rc;
  if (out_host != nullptr) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    FDA_HIP(hipMemcpyAsync(out_host, out_dev, sizeof(fda_estimate), hipMemcpyDeviceToHost, st));
    FDA_HIP(hipStreamSynchronize(st));
  }
  return FDA_OK;
}

}  // extern "C"
