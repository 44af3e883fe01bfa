// Measurement aid for gfx950: issue cost of the vector instructions that the digest mixer and the
// binary64 update arithmetic are made of, each relative to v_add_u32.  Every kernel runs eight
// independent dependency chains per lane, eight wavefronts per SIMD, no memory traffic.
//   alu_issue_rates [iterations per chain, default 2000]      (400000 gives about 45 ms per instruction)
// Result on MI355X: 32-bit multiplies, v_mad_u64_u32, 64-bit shifts and adds, binary64 FMA and the
// conversions all issue at the full rate (one wavefront instruction per 4 cycles); only the binary64
// reciprocal, reciprocal square root and square root take 16 cycles (binary32 rsq: 8).  The rate does
// not drop over 45 ms of pure arithmetic, so the lower shader clock seen under the digest kernels
// (counters: 1.8-1.9 GHz against 2.3 GHz) comes from arithmetic and HBM streaming together.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>

#define CK(x)                                                     \
  do {                                                            \
    hipError_t e_ = (x);                                          \
    if (e_ != hipSuccess) {                                       \
      printf("%s: %s\n", #x, hipGetErrorString(e_));              \
      return 1;                                                   \
    }                                                             \
  } while (0)

constexpr int kChains = 8;

template <int OP>
__global__ void __launch_bounds__(256) chain_kernel(uint64_t *out, uint32_t kk, int iters) {
  uint32_t a[kChains];
  uint64_t z[kChains];
  double d[kChains];
  for (int c = 0; c < kChains; ++c) {
    a[c] = threadIdx.x * 77u + c;
    z[c] = ((uint64_t)a[c] << 32) | (c * 13u + 1);
    d[c] = 1.0 + c;
  }
  const uint64_t k64 = ((uint64_t)kk << 32) | 0x9E3779B9u;
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int c = 0; c < kChains; ++c) {
      if constexpr (OP == 0) asm volatile("v_add_u32 %0, %0, %1" : "+v"(a[c]) : "s"(kk));
      if constexpr (OP == 1) asm volatile("v_mul_lo_u32 %0, %0, %1" : "+v"(a[c]) : "s"(kk));
      if constexpr (OP == 2) asm volatile("v_mad_u64_u32 %0, vcc, %1, %2, %0" : "+v"(z[c]) : "v"(a[c]), "s"(kk) : "vcc");
      if constexpr (OP == 3) asm volatile("v_lshrrev_b64 %0, 1, %0" : "+v"(z[c]));
      if constexpr (OP == 4) asm volatile("v_lshl_add_u64 %0, %0, 0, %1" : "+v"(z[c]) : "s"(k64));
      if constexpr (OP == 5) asm volatile("v_mul_hi_u32 %0, %0, %1" : "+v"(a[c]) : "s"(kk));
      if constexpr (OP == 6) asm volatile("v_xor_b32 %0, %0, %1" : "+v"(a[c]) : "s"(kk));
      if constexpr (OP == 7) asm volatile("v_add3_u32 %0, %0, %1, %1" : "+v"(a[c]) : "s"(kk));
      if constexpr (OP == 8) asm volatile("v_fma_f64 %0, %0, %0, %0" : "+v"(d[c]));
      if constexpr (OP == 9) asm volatile("v_mul_f64 %0, %0, %0" : "+v"(d[c]));
      if constexpr (OP == 10) asm volatile("v_cvt_f64_f32 %0, %1" : "=v"(d[c]) : "v"(a[c]));
      if constexpr (OP == 11) asm volatile("v_cvt_f32_f64 %0, %1" : "=v"(a[c]) : "v"(d[c]));
      if constexpr (OP == 12) asm volatile("v_rcp_f64 %0, %0" : "+v"(d[c]));
      if constexpr (OP == 13) asm volatile("v_rsq_f64 %0, %0" : "+v"(d[c]));
      if constexpr (OP == 14) asm volatile("v_sqrt_f64 %0, %0" : "+v"(d[c]));
      if constexpr (OP == 15) asm volatile("v_rsq_f32 %0, %0" : "+v"(a[c]));
      if constexpr (OP == 16) asm volatile("v_div_scale_f64 %0, vcc, %0, %0, %0" : "+v"(d[c])::"vcc");
      if constexpr (OP == 17) asm volatile("v_div_fmas_f64 %0, %0, %0, %0" : "+v"(d[c])::"vcc");
      if constexpr (OP == 18) asm volatile("v_div_fixup_f64 %0, %0, %0, %0" : "+v"(d[c]));
      if constexpr (OP == 19) asm volatile("v_mov_b32_dpp %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf" : "+v"(a[c]));
    }
  }
  uint64_t s = 0;
  for (int c = 0; c < kChains; ++c) s += a[c] + z[c] + (uint64_t)d[c];
  if (s == 0x1234567) out[0] = s;     // keeps the chains alive; practically never true
}

static double g_ref_ns = 1.0;

template <int OP>
int run(const char *name, uint64_t *out, int iters) {
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  int cus = 0;
  CK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, 0));
  const int grid = cus * 8;           // 8 workgroups of 4 wavefronts per CU = 8 wavefronts per SIMD
  hipLaunchKernelGGL(chain_kernel<OP>, dim3(grid), dim3(256), 0, 0, out, 0x6A09E667u, 16);
  CK(hipDeviceSynchronize());
  float best = 1e30f;
  for (int r = 0; r < 3; ++r) {
    CK(hipEventRecord(e0));
    hipLaunchKernelGGL(chain_kernel<OP>, dim3(grid), dim3(256), 0, 0, out, 0x6A09E667u, iters);
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms = 0;
    CK(hipEventElapsedTime(&ms, e0, e1));
    if (ms < best) best = ms;
  }
  const double per_simd = (double)grid * 4 / (cus * 4) * iters * kChains;     // wavefront instructions per SIMD
  const double ns = best * 1e6 / per_simd;
  if (OP == 0) g_ref_ns = ns;
  printf("%-18s %9.3f ms  %6.3f ns per wavefront instruction = %5.2f x v_add_u32  (%5.2f cycles at 2.4 GHz)\n", name, best,
         ns, ns / g_ref_ns, ns * 2.4);
  fflush(stdout);
  CK(hipEventDestroy(e0));
  CK(hipEventDestroy(e1));
  return 0;
}

int main(int argc, char **argv) {
  const int iters = argc > 1 ? atoi(argv[1]) : 2000;
  if (iters < 1 || iters > 4000000) {
    printf("iterations must be in [1, 4000000]\n");
    return 2;
  }
  uint64_t *out = nullptr;
  CK(hipMalloc(&out, 64));
  int rc = 0;
  rc |= run<0>("v_add_u32", out, iters);
  rc |= run<1>("v_mul_lo_u32", out, iters);
  rc |= run<2>("v_mad_u64_u32", out, iters);
  rc |= run<3>("v_lshrrev_b64", out, iters);
  rc |= run<4>("v_lshl_add_u64", out, iters);
  rc |= run<5>("v_mul_hi_u32", out, iters);
  rc |= run<6>("v_xor_b32", out, iters);
  rc |= run<7>("v_add3_u32", out, iters);
  rc |= run<8>("v_fma_f64", out, iters);
  rc |= run<9>("v_mul_f64", out, iters);
  rc |= run<10>("v_cvt_f64_f32", out, iters);
  rc |= run<11>("v_cvt_f32_f64", out, iters);
  rc |= run<12>("v_rcp_f64", out, iters);
  rc |= run<13>("v_rsq_f64", out, iters);
  rc |= run<14>("v_sqrt_f64", out, iters);
  rc |= run<15>("v_rsq_f32", out, iters);
  rc |= run<16>("v_div_scale_f64", out, iters);
  rc |= run<17>("v_div_fmas_f64", out, iters);
  rc |= run<18>("v_div_fixup_f64", out, iters);
  rc |= run<19>("v_mov_b32_dpp", out, iters);
  (void)hipFree(out);
  return rc;
}
