/*
 * Plain-C use of the update-undo library (no Python, no torch): an AdamW step on two tensors, digests
 * before and after, the per-tensor mask derived from the digests, and the undo of the marked tensors.
 *
 * Built by `python -m paper_2302_06173_amd.build` next to the library (plain gcc; the HIP runtime is
 * used for device memory only).
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "swift_undo.h"

#define HIP_OK(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { \
  fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_)); return 2; } } while (0)
#define SWIFT_OK_OR_DIE(call) do { int rc_ = (call); if (rc_ != SWIFT_OK) { \
  fprintf(stderr, "%s: error %d: %s\n", #call, rc_, swift_last_error()); return 3; } } while (0)

static uint32_t lcg(uint32_t *s) { *s = *s * 1664525u + 1013904223u; return *s; }
static float uniform(uint32_t *s, float scale) { return scale * ((float)(lcg(s) >> 8) / 8388608.0f - 1.0f); }

int main(void) {
  enum { NT = 2 };
  const int64_t numel[NT] = {300007, 4096};
  float *h[NT][4], *d[NT][4];               /* theta, g, m, v */
  uint32_t seed = 12345u;
  for (int t = 0; t < NT; ++t)
    for (int k = 0; k < 4; ++k) {
      const size_t bytes = (size_t)numel[t] * sizeof(float);
      h[t][k] = (float *)malloc(bytes);
      if (!h[t][k]) return 1;
      const float scale = k == 0 ? 0.05f : k == 1 ? 2e-3f : k == 2 ? 2e-4f : 2e-6f;
      for (int64_t i = 0; i < numel[t]; ++i) h[t][k][i] = k == 3 ? fabsf(uniform(&seed, scale)) : uniform(&seed, scale);
      HIP_OK(hipMalloc((void **)&d[t][k], bytes));
      HIP_OK(hipMemcpy(d[t][k], h[t][k], bytes, hipMemcpyHostToDevice));
    }
  void *param[NT], *m[NT], *v[NT];
  const void *grad[NT];
  const void *state[3 * NT];
  int64_t state_numel[3 * NT];
  for (int t = 0; t < NT; ++t) {
    param[t] = d[t][0]; grad[t] = d[t][1]; m[t] = d[t][2]; v[t] = d[t][3];
    for (int k = 0; k < 3; ++k) { state[k * NT + t] = d[t][k == 0 ? 0 : k + 1]; state_numel[k * NT + t] = numel[t]; }
  }
  const swift_tensor_list list = {NT, param, grad, m, v, numel, NULL};
  const swift_hparams hp = {SWIFT_ADAMW, SWIFT_F32, 100, 6e-4, 0.1, 0.0, 0.0, 0.9, 0.95, 1e-8, 0, 0};
  const uint8_t only_first[NT] = {1, 0};     /* the update reached tensor 0 before the failure */
  uint64_t *dig0, *dig1;
  uint8_t *dmask, hmask[NT];
  HIP_OK(hipMalloc((void **)&dig0, 3 * NT * sizeof(uint64_t)));
  HIP_OK(hipMalloc((void **)&dig1, 3 * NT * sizeof(uint64_t)));
  HIP_OK(hipMalloc((void **)&dmask, NT));

  SWIFT_OK_OR_DIE(swift_state_digest(3 * NT, state, state_numel, 0, dig0, NULL));
  SWIFT_OK_OR_DIE(swift_opt_step(&list, &hp, only_first, NULL));
  SWIFT_OK_OR_DIE(swift_state_digest(3 * NT, state, state_numel, 0, dig1, NULL));
  SWIFT_OK_OR_DIE(swift_mask_from_digests(NT, 3, dig0, dig1, dmask, NULL));
  SWIFT_OK_OR_DIE(swift_opt_undo_dmask(&list, &hp, dmask, NULL));
  HIP_OK(hipDeviceSynchronize());
  HIP_OK(hipMemcpy(hmask, dmask, NT, hipMemcpyDeviceToHost));
  if (hmask[0] != 1 || hmask[1] != 0) { fprintf(stderr, "mask from digests is %d %d, expected 1 0\n", hmask[0], hmask[1]); return 4; }

  double worst = 0.0;
  for (int t = 0; t < NT; ++t)
    for (int k = 0; k < 4; ++k) {
      const size_t bytes = (size_t)numel[t] * sizeof(float);
      float *back = (float *)malloc(bytes);
      if (!back) return 1;
      HIP_OK(hipMemcpy(back, d[t][k], bytes, hipMemcpyDeviceToHost));
      for (int64_t i = 0; i < numel[t]; ++i) {
        const double a = back[i], b = h[t][k][i], err = fabs(a - b);
        if ((t == 1 || k == 1) && a != b) { fprintf(stderr, "tensor %d stream %d changed at %lld\n", t, k, (long long)i); return 5; }
        if (err > fmax(1e-5 * fabs(b), 1e-8)) { fprintf(stderr, "tensor %d stream %d element %lld: %g vs %g\n", t, k, (long long)i, a, b); return 6; }
        if (b != 0.0 && err / fabs(b) > worst) worst = err / fabs(b);
      }
      free(back);
    }
  printf("ok: step on tensor 0, digest-derived mask {1, 0}, undo; worst relative round-trip error %.3g\n", worst);
  SWIFT_OK_OR_DIE(swift_shutdown());
  return 0;
}
