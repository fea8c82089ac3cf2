/* A plain C caller of the FDA library: no C++, no Python, no torch.  It builds a small [K][d]
 * slab with a fixed arithmetic pattern, runs Algorithm 1 lines 6-9 once through the C ABI
 * (fda_local_state, fda_estimate_variance, fda_sync, fda_update_xi) and once through
 * fda_mean_state, and prints what it got, one "name value" pair per line, so that a test can
 * compare the numbers with the CPU oracle's on the same pattern.
 *
 *   fda_c_example K d l m theta
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "fda.h"

#define HIP_OK(call)                                                                   \
  do {                                                                                 \
    hipError_t e_ = (call);                                                            \
    if (e_ != hipSuccess) {                                                            \
      fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));                \
      return 2;                                                                        \
    }                                                                                  \
  } while (0)
#define FDA_CALL(call)                                                                 \
  do {                                                                                 \
    int rc_ = (call);                                                                  \
    if (rc_ != FDA_OK) {                                                               \
      fprintf(stderr, "%s failed: %s (%s)\n", #call, fda_strerror(rc_), fda_last_error()); \
      return 3;                                                                        \
    }                                                                                  \
  } while (0)

/* the input pattern: small integers scaled by powers of two (exact in fp32) */
static float pattern_w_t0(long long j) { return (float)((j * 7 + 3) % 33 - 16) / 64.0f; }
static float pattern_u(int k, long long j) { return (float)((j * 5 + k * 11 + 1) % 17 - 8) / 1024.0f; }
static float pattern_xi(long long j) { return (float)((j * 3 + 2) % 9 - 4) / 8.0f; }
static uint32_t pattern_coef(int t) { return (uint32_t)((1103515245ull * (unsigned long long)(t + 1) + 12345ull) % 2147483647ull); }

int main(int argc, char** argv) {
  if (argc != 6) {
    fprintf(stderr, "usage: %s K d l m theta\n", argv[0]);
    return 1;
  }
  const int K = atoi(argv[1]);
  const long long d = atoll(argv[2]);
  const int l = atoi(argv[3]), m = atoi(argv[4]);
  const double theta = atof(argv[5]);

  uint32_t coef[FDA_MAX_SKETCH_ROWS * 8];
  for (int t = 0; t < l * 8; ++t) coef[t] = pattern_coef(t);
  fda_desc desc;
  desc.K = K; desc.d = d; desc.row_stride = d; desc.dtype = FDA_F32;
  desc.variants = FDA_VARIANT_LINEAR | FDA_VARIANT_SKETCH;
  desc.l = l; desc.m = m; desc.flags = 0; desc.eps = 0.06; desc.hash_coef = coef;

  float* hw = (float*)malloc(sizeof(float) * (size_t)K * (size_t)d);
  float* h0 = (float*)malloc(sizeof(float) * (size_t)d);
  float* hx = (float*)malloc(sizeof(float) * (size_t)d);
  if (!hw || !h0 || !hx) return 4;
  for (long long j = 0; j < d; ++j) {
    h0[j] = pattern_w_t0(j);
    hx[j] = pattern_xi(j);
    for (int k = 0; k < K; ++k) hw[(size_t)k * d + j] = h0[j] + pattern_u(k, j);
  }

  size_t ws_bytes = 0;
  FDA_CALL(fda_workspace_bytes(&desc, &ws_bytes));
  void *ws, *w, *w_t0, *w_prev, *xi, *state, *mean_state, *est_dev;
  HIP_OK(hipMalloc(&ws, ws_bytes));
  HIP_OK(hipMalloc(&w, sizeof(float) * (size_t)K * d));
  HIP_OK(hipMalloc(&w_t0, sizeof(float) * d));
  HIP_OK(hipMalloc(&w_prev, sizeof(float) * d));
  HIP_OK(hipMalloc(&xi, sizeof(float) * d));
  HIP_OK(hipMalloc(&est_dev, sizeof(fda_estimate)));
  HIP_OK(hipMemcpy(w, hw, sizeof(float) * (size_t)K * d, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(w_t0, h0, sizeof(float) * d, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(xi, hx, sizeof(float) * d, hipMemcpyHostToDevice));

  fda_ctx* ctx = NULL;
  FDA_CALL(fda_create(&ctx, &desc, ws, ws_bytes));
  int64_t S = 0;
  FDA_CALL(fda_state_floats(ctx, &S));
  HIP_OK(hipMalloc(&state, sizeof(float) * (size_t)K * S));
  HIP_OK(hipMalloc(&mean_state, sizeof(float) * (size_t)S));

  fda_estimate est, est_mean;
  FDA_CALL(fda_local_state(ctx, w, (const float*)w_t0, (const float*)xi, (float*)state, NULL));
  FDA_CALL(fda_estimate_variance(ctx, (const float*)state, theta, 1e-5, (fda_estimate*)est_dev, &est, NULL));
  FDA_CALL(fda_mean_state(ctx, w, (const float*)w_t0, (const float*)xi, (float*)mean_state, NULL, NULL));
  FDA_CALL(fda_estimate_variance_mean(ctx, (const float*)mean_state, theta, 1e-5, (fda_estimate*)est_dev,
                                      &est_mean, NULL));
  /* synchronize if the sketch variant says so (the device-side decision sits in est_dev) */
  const int32_t* pred = (const int32_t*)((const char*)est_dev + offsetof(fda_estimate, sync_sketch));
  FDA_CALL(fda_sync(ctx, w, (float*)w_t0, (float*)w_prev, pred, NULL));
  FDA_CALL(fda_update_xi(ctx, (const float*)w_t0, (const float*)w_prev, (float*)xi, pred, NULL));
  HIP_OK(hipDeviceSynchronize());

  float* hs = (float*)malloc(sizeof(float) * (size_t)K * S);
  if (!hs) return 4;
  HIP_OK(hipMemcpy(hs, state, sizeof(float) * (size_t)K * S, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(h0, w_t0, sizeof(float) * d, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(hx, xi, sizeof(float) * d, hipMemcpyDeviceToHost));
  double xin = 0.0, w0sum = 0.0;
  for (long long j = 0; j < d; ++j) { xin += (double)hx[j] * hx[j]; w0sum += h0[j]; }

  printf("state_floats %lld\n", (long long)S);
  for (int k = 0; k < K; ++k) printf("sqnorm_%d %.9g\nproj_%d %.9g\n", k, hs[(size_t)k * S], k, hs[(size_t)k * S + 1]);
  printf("sketch_0_0_0 %.9g\n", hs[2]);
  printf("mean_sqnorm %.17g\nmean_proj %.17g\nm2 %.17g\nh_linear %.17g\nh_sketch %.17g\n", est.mean_sqnorm,
         est.mean_proj, est.m2, est.h_linear, est.h_sketch);
  printf("sync_linear %d\nsync_sketch %d\nnonfinite %d\n", est.sync_linear, est.sync_sketch, est.nonfinite);
  printf("mean_mode_h_linear %.17g\nmean_mode_h_sketch %.17g\nmean_mode_sync_sketch %d\n", est_mean.h_linear,
         est_mean.h_sketch, est_mean.sync_sketch);
  printf("xi_sqnorm_after %.9g\nw_t0_sum_after %.9g\n", xin, w0sum);

  FDA_CALL(fda_destroy(ctx));
  hipFree(ws); hipFree(w); hipFree(w_t0); hipFree(w_prev); hipFree(xi); hipFree(state);
  hipFree(mean_state); hipFree(est_dev);
  free(hw); free(h0); free(hx); free(hs);
  return 0;
}
