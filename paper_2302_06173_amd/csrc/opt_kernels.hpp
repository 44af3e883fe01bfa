// Optimizer step / update-undo kernels for gfx950 (one multi-tensor launch per call).
//
// What is computed: Alg. 1 and Alg. 2 of the paper (SGD with momentum and its undo) and the
// Adam / AdamW pairs of App. A.  How: every workgroup walks a flat chunk table with a grid
// stride; a chunk is a run of up to `chunk_elems` elements of one tensor.  Each lane moves 16
// bytes per stream per access (theta, g, m, v in; theta, m, v out), widens to binary64, applies
// the update lines with explicit FMAs and rounds once on the way out.  The path is HBM-bound
// (28 bytes per element for Adam with fp32 gradients), so there is no LDS staging and no MFMA.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace swift {

constexpr int kSGDM = 0, kADAM = 1, kADAMW = 2;
constexpr int kThreads = 256;           // 4 wavefronts of 64
#ifndef SWIFT_UNROLL
#define SWIFT_UNROLL 2                  // 16-byte accesses in flight per lane and stream
#endif
#ifndef SWIFT_NT
#define SWIFT_NT 1                      // non-temporal (streaming) loads and stores
#endif

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct TensorDesc {        // one per tensor, 48 bytes, device resident
  float *x;                // theta, in/out
  const void *g;           // gradient, fp32 or bf16, read only
  float *m;                // momentum buffer / first moment, in/out
  float *v;                // second moment, in/out (unused for SGDM)
  int64_t numel;
  uint32_t vec_ok;         // 1: all pointers aligned for the 128-bit path
  uint32_t pad;
};

struct ChunkRef {          // one per chunk, 8 bytes, device resident
  uint32_t tensor;         // index into the descriptor table
  uint32_t chunk;          // chunk number inside the tensor: elements [chunk*CE, chunk*CE+CE)
};

// Scalars derived on the host in binary64 from the hyper-parameters (never as 1.0f - float(beta)).
struct OptConsts {
  double eta, lam;
  double mu, omt, inv_mu;                 // SGDM: mu, 1-tau, 1/mu
  double b1, b2, c1, c2, inv_b1, inv_b2;  // beta, 1-beta, 1/beta
  double rbc1, rbc2;                      // 1/(1-beta1^t), 1/(1-beta2^t)
  double eps;
  double inv_oml;                         // 1/(1 - eta*lambda)   (AdamW undo)
  int32_t mu_is_zero;
  int32_t pad;
};

// Tensor pointers come out of a descriptor table, so the compiler cannot tell their address
// space; the explicit cast makes every access a global_load / global_store instead of a flat one.
#define SWIFT_GLOBAL __attribute__((address_space(1)))
template <bool NT, typename T>
__device__ __forceinline__ T ld(const T *p) {
  const SWIFT_GLOBAL T *q = (const SWIFT_GLOBAL T *)p;
  if constexpr (NT) return __builtin_nontemporal_load(q);
  else return *q;
}
template <bool NT, typename T>
__device__ __forceinline__ void st(T *p, T val) {
  SWIFT_GLOBAL T *q = (SWIFT_GLOBAL T *)p;
  if constexpr (NT) __builtin_nontemporal_store(val, q);
  else *q = val;
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t hi16) { return __uint_as_float(hi16 << 16); }

// One element.  The vector body and the scalar head/tail path both call this, so an element's
// result bits do not depend on where it falls in a chunk or on pointer alignment.
// u = m^ / (sqrt(v^) + eps) with m^ = m/(1-beta1^t), v^ = v/(1-beta2^t)   (App. A).
template <int KIND, bool UNDO>
__device__ __forceinline__ void update_elem(float &xf, float gf, float &mf, float &vf, const OptConsts &c) {
  const double x = (double)xf, g = (double)gf, m = (double)mf;
  if constexpr (KIND == kSGDM) {
    if constexpr (!UNDO) {                          // Alg. 1
      const double gp = fma(c.lam, x, g);
      const double mt = fma(c.mu, m, c.omt * gp);
      mf = (float)mt;
      xf = (float)fma(-c.eta, mt, x);
    } else {                                        // Alg. 2
      const double xt = fma(c.eta, m, x);
      xf = (float)xt;
      if (!c.mu_is_zero) {
        const double gp = fma(c.lam, xt, g);
        mf = (float)(fma(-c.omt, gp, m) * c.inv_mu);
      }
    }
  } else {
    const double v = (double)vf;
    if constexpr (!UNDO) {                          // App. A "Adam" / "AdamW"
      const double gp = (KIND == kADAM) ? fma(c.lam, x, g) : g;
      const double mt = fma(c.b1, m, c.c1 * gp);
      const double vt = fma(c.b2, v, c.c2 * (gp * gp));
      const double u = (mt * c.rbc1) / (sqrt(vt * c.rbc2) + c.eps);
      mf = (float)mt;
      vf = (float)vt;
      if constexpr (KIND == kADAM) xf = (float)fma(-c.eta, u, x);
      else xf = (float)fma(-c.eta, fma(c.lam, x, u), x);
    } else {                                        // App. A "Undo Adam" / "Undo AdamW"
      const double u = (m * c.rbc1) / (sqrt(v * c.rbc2) + c.eps);
      double xt = fma(c.eta, u, x);
      if constexpr (KIND == kADAMW) xt *= c.inv_oml;
      const double gp = (KIND == kADAM) ? fma(c.lam, xt, g) : g;
      xf = (float)xt;
      mf = (float)(fma(-c.c1, gp, m) * c.inv_b1);
      vf = (float)(fma(-c.c2, gp * gp, v) * c.inv_b2);
    }
  }
}

template <int KIND, bool UNDO>
__device__ __forceinline__ void update_vec4(f32x4 &x, const f32x4 &g, f32x4 &m, f32x4 &v, const OptConsts &c) {
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    float xe = x[k], me = m[k], ve = (KIND == kSGDM) ? 0.f : v[k];
    update_elem<KIND, UNDO>(xe, g[k], me, ve, c);
    x[k] = xe;
    m[k] = me;
    if constexpr (KIND != kSGDM) v[k] = ve;
  }
}

template <bool BF16G, bool NT>
__device__ __forceinline__ f32x4 load_grad4(const void *g, int64_t i4) {
  if constexpr (BF16G) {
    const u32x2 raw = ld<NT>(reinterpret_cast<const u32x2 *>(g) + i4);   // 4 bf16 = 8 bytes
    f32x4 r;
    r[0] = bf16_bits_to_f32(raw[0] & 0xFFFFu);
    r[1] = bf16_bits_to_f32(raw[0] >> 16);
    r[2] = bf16_bits_to_f32(raw[1] & 0xFFFFu);
    r[3] = bf16_bits_to_f32(raw[1] >> 16);
    return r;
  } else {
    return ld<NT>(reinterpret_cast<const f32x4 *>(g) + i4);
  }
}

template <bool BF16G>
__device__ __forceinline__ float load_grad1(const void *g, int64_t i) {
  if constexpr (BF16G) return bf16_bits_to_f32(ld<false>(reinterpret_cast<const uint16_t *>(g) + i));
  else return ld<false>(reinterpret_cast<const float *>(g) + i);
}

// Grid-stride over the chunk table.  `dmask` (nullable) holds one byte per tensor in device
// memory: chunks of tensors whose byte is zero are skipped.
template <int KIND, bool UNDO, bool BF16G, bool NT, int U>
__global__ void __launch_bounds__(kThreads)
opt_kernel(const TensorDesc *__restrict__ descs, const ChunkRef *__restrict__ chunks, uint32_t n_chunks,
           uint32_t chunk_elems, const uint8_t *__restrict__ dmask, const OptConsts c) {
  constexpr bool HASV = (KIND != kSGDM);
  const uint32_t tid = threadIdx.x;
  for (uint32_t ci = blockIdx.x; ci < n_chunks; ci += gridDim.x) {
    const ChunkRef ch = chunks[ci];
    if (dmask != nullptr && dmask[ch.tensor] == 0) continue;
    const TensorDesc d = descs[ch.tensor];
    const int64_t base = (int64_t)ch.chunk * chunk_elems;
    const int64_t left = d.numel - base;
    const uint32_t len = left < (int64_t)chunk_elems ? (uint32_t)left : chunk_elems;
    float *__restrict__ xp = d.x + base;
    float *__restrict__ mp = d.m + base;
    float *__restrict__ vp = HASV ? d.v + base : nullptr;
    const void *gp = BF16G ? (const void *)(reinterpret_cast<const uint16_t *>(d.g) + base)
                           : (const void *)(reinterpret_cast<const float *>(d.g) + base);
    if (d.vec_ok) {
      // chunk_elems is a multiple of 4, so `base` keeps the 16-byte alignment of the tensor
      f32x4 *x4 = reinterpret_cast<f32x4 *>(xp);
      f32x4 *m4 = reinterpret_cast<f32x4 *>(mp);
      f32x4 *v4 = reinterpret_cast<f32x4 *>(vp);
      const uint32_t n4 = len >> 2;
      uint32_t i = 0;
      for (; i + U * kThreads <= n4; i += U * kThreads) {       // full tiles: no predicates
        f32x4 xr[U], gr[U], mr[U], vr[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const uint32_t j = i + u * kThreads + tid;
          xr[u] = ld<NT>(x4 + j);
          gr[u] = load_grad4<BF16G, NT>(gp, j);
          mr[u] = ld<NT>(m4 + j);
          if constexpr (HASV) vr[u] = ld<NT>(v4 + j);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const uint32_t j = i + u * kThreads + tid;
          update_vec4<KIND, UNDO>(xr[u], gr[u], mr[u], vr[u], c);
          st<NT>(x4 + j, xr[u]);
          st<NT>(m4 + j, mr[u]);
          if constexpr (HASV) st<NT>(v4 + j, vr[u]);
        }
      }
      for (uint32_t j = i + tid; j < n4; j += kThreads) {       // ragged end of the chunk
        f32x4 xr = ld<NT>(x4 + j), gr = load_grad4<BF16G, NT>(gp, j), mr = ld<NT>(m4 + j), vr;
        if constexpr (HASV) vr = ld<NT>(v4 + j);
        update_vec4<KIND, UNDO>(xr, gr, mr, vr, c);
        st<NT>(x4 + j, xr);
        st<NT>(m4 + j, mr);
        if constexpr (HASV) st<NT>(v4 + j, vr);
      }
      const uint32_t e = (n4 << 2) + tid;                        // last numel % 4 elements
      if (e < len) {
        float xe = ld<false>(xp + e), me = ld<false>(mp + e), ve = 0.f;
        if constexpr (HASV) ve = ld<false>(vp + e);
        update_elem<KIND, UNDO>(xe, load_grad1<BF16G>(gp, e), me, ve, c);
        st<false>(xp + e, xe);
        st<false>(mp + e, me);
        if constexpr (HASV) st<false>(vp + e, ve);
      }
    } else {
      for (uint32_t e = tid; e < len; e += kThreads) {           // unaligned tensor: 4-byte accesses
        float xe = ld<false>(xp + e), me = ld<false>(mp + e), ve = 0.f;
        if constexpr (HASV) ve = ld<false>(vp + e);
        update_elem<KIND, UNDO>(xe, load_grad1<BF16G>(gp, e), me, ve, c);
        st<false>(xp + e, xe);
        st<false>(mp + e, me);
        if constexpr (HASV) st<false>(vp + e, ve);
      }
    }
  }
}

// Plain copy with the optimizer kernels' access pattern (16 bytes per lane, grid stride over
// tiles of U*256 vectors): the practical HBM ceiling and the calibration run for byte counters.
template <bool NT, int U>
__global__ void __launch_bounds__(kThreads)
copy_kernel(u32x4 *__restrict__ dst, const u32x4 *__restrict__ src, uint64_t n16) {
  const uint64_t tile = (uint64_t)U * kThreads;
  const uint64_t n_tiles = (n16 + tile - 1) / tile;
  for (uint64_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
    const uint64_t i0 = t * tile + threadIdx.x;
    u32x4 r[U];
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (i0 + (uint64_t)u * kThreads < n16) r[u] = ld<NT>(src + i0 + (uint64_t)u * kThreads);
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (i0 + (uint64_t)u * kThreads < n16) st<NT>(dst + i0 + (uint64_t)u * kThreads, r[u]);
  }
}

}  // namespace swift
