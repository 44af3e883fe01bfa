// Optimizer step / update-undo kernels for gfx950 (one multi-tensor launch per call).
//
// What is computed: Alg. 1 and Alg. 2 of the paper (SGD with momentum and its undo) and the
// SGD / Adam / AdamW pairs of App. A.  How: the tensor list is cut into a flat table of chunks (runs of
// one tensor's elements); one 64-lane workgroup handles one tile of a chunk.  Each lane moves 16
// bytes per stream (theta, g, m, v in; theta, m, v out), widens to binary64, applies the update
// lines with explicit FMAs and rounds once on the way out.  The path is HBM-bound (28 bytes per
// element for Adam with fp32 gradients, 0.7 flop per byte), so there is no LDS staging and no MFMA;
// what matters is the order and the number of memory requests in flight (see opt_kernel below).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace swift {

constexpr int kSGDM = 0, kADAM = 1, kADAMW = 2, kSGD = 3;   // kSGD: App. A's plain SGD, no optimizer state
constexpr int kThreads = 256;           // 4 wavefronts of 64
// Launch shapes of the optimizer kernels that get compiled: X(U, BLOCK) = 16-byte vectors per lane,
// lanes per workgroup.  The product builds the measured best only; -DSWIFT_SWEEP_SHAPES adds the
// shapes that sweeps compare it with (SWIFT_TILE_U / SWIFT_TILE_BLOCK select among them).
#ifndef SWIFT_SHAPES
#ifdef SWIFT_SWEEP_SHAPES
#define SWIFT_SHAPES(X) X(1, 64) X(2, 64) X(4, 64) X(1, 256)
#else
#define SWIFT_SHAPES(X) X(1, 64)
#endif
#endif
// Tuning defaults, all measured on MI355X with the 7 B-parameter list (wavefronts per compute unit
// are enforced through unused dynamic LDS).  Each can be overridden on the compiler's command line.
#ifndef SWIFT_DIGEST_WAVES_PER_CU
#define SWIFT_DIGEST_WAVES_PER_CU 0     // digest kernel: residency cap (0 = none)
#endif
#ifndef SWIFT_DIGEST_CHUNK
#define SWIFT_DIGEST_CHUNK 65536        // digest kernel: words per workgroup (large inputs)
#endif
#ifndef SWIFT_DEFAULT_U
#define SWIFT_DEFAULT_U 1
#endif
#ifndef SWIFT_DEFAULT_BLOCK
#define SWIFT_DEFAULT_BLOCK 64
#endif
#ifndef SWIFT_DEFAULT_WAVES_PER_CU
#define SWIFT_DEFAULT_WAVES_PER_CU 11
#endif
#ifndef SWIFT_DEFAULT_WAVES_PER_CU_SGDM
#define SWIFT_DEFAULT_WAVES_PER_CU_SGDM 14
#endif
#ifndef SWIFT_DEFAULT_WAVES_PER_CU_SGD
#define SWIFT_DEFAULT_WAVES_PER_CU_SGD 24   // plain SGD: 2 streams in, 1 out (7B list: 6.34 TB/s at 14, 6.73 at 18, 6.82 at 24, 6.72 at 28)
#endif
#ifndef SWIFT_FUSED_U
#define SWIFT_FUSED_U 1                 // step/undo fused with the digest: vectors per lane
#endif
#ifndef SWIFT_FUSED_WAVES_PER_CU
#define SWIFT_FUSED_WAVES_PER_CU 20     // step/undo fused with the digest
#endif
#ifndef SWIFT_LAMB_U1
#define SWIFT_LAMB_U1 1                 // LAMB pass 1: vectors per lane (tile = U * 256 elements, one partial sum pair per tile)
#endif
#ifndef SWIFT_LAMB_U3
#define SWIFT_LAMB_U3 1                 // LAMB pass 3
#endif
#ifndef SWIFT_LAMB_WAVES_P1
#define SWIFT_LAMB_WAVES_P1 14          // LAMB pass 1 (U = 1): wavefronts per CU
#endif
#ifndef SWIFT_LAMB_WAVES_P3
#define SWIFT_LAMB_WAVES_P3 20          // LAMB pass 3 (3 streams in, 1 out)
#endif
#ifndef SWIFT_DEFAULT_DMASK_WGS_PER_CU
#define SWIFT_DEFAULT_DMASK_WGS_PER_CU 16384
#endif
#ifndef SWIFT_DMASK_QUEUE
#define SWIFT_DMASK_QUEUE 1             // device-mask launches: 1 = resident wavefronts drawing tiles from counters, 0 = capped strided grid
#endif
#ifndef SWIFT_DMASK_COUNTERS
#define SWIFT_DMASK_COUNTERS 64         // tile counters of the queue mode (a power of two, at most 256): 32 and 128 are slower
#endif
#ifndef SWIFT_DMASK_QUEUE_WAVES_PER_CU
#define SWIFT_DMASK_QUEUE_WAVES_PER_CU 10 // resident wavefronts per CU in queue mode
#endif
#ifndef SWIFT_COPY_U
#define SWIFT_COPY_U 1                  // copy kernel: 16-byte vectors per lane
#endif
#ifndef SWIFT_COPY_WAVES_PER_CU
#define SWIFT_COPY_WAVES_PER_CU 0       // copy kernel: residency cap (0 = none: measured best, 6.7 TB/s)
#endif
#ifndef SWIFT_NT
#define SWIFT_NT 1                      // non-temporal (streaming) loads and stores
#endif

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct ChunkDesc {         // one per chunk of the optimizer kernels, 64 bytes, device resident
  float *x;                // theta of the chunk's first element, in/out
  const void *g;           // gradient, fp32 or bf16, read only
  float *m;                // momentum buffer / first moment, in/out (null for plain SGD)
  float *v;                // second moment, in/out (null for SGDM and plain SGD)
  uint16_t *xb;            // bfloat16 copy of theta, out only (null if the caller keeps none)
  uint32_t len;            // elements in this chunk (the last chunk of a tensor is short)
  uint32_t tensor;         // index of the tensor in the caller's list (for the device mask)
  uint32_t vec_ok;         // 1: every pointer is aligned for the 128-bit path
  uint32_t elem0;          // index of the chunk's first element inside its tensor (mod 2^32)
  uint64_t pad;
};

struct ChunkRef {          // digest kernel: one per chunk, 8 bytes, device resident
  uint32_t tensor;         // index into the descriptor table
  uint32_t chunk;          // chunk number inside the buffer
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
  int32_t clamp_v;                        // undo: store a recovered v below zero as +0
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

// Streaming accesses of the 128-bit path go through buffer instructions: the chunk's base pointer
// is wave-uniform, the byte range of the chunk is the buffer's extent (the hardware drops
// anything outside it), and the cache-policy bits can be chosen per access.  Measured on MI355X
// for the 4-read/3-write stream: loads `nt`; stores `sc0 sc1 nt` (2-3 % above `nt` alone,
// 9 % above default stores).
#ifndef SWIFT_LOAD_AUX
#define SWIFT_LOAD_AUX 2                // nt
#endif
#ifndef SWIFT_STORE_AUX
#define SWIFT_STORE_AUX 19              // sc0 (1) | nt (2) | sc1 (16)
#endif
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00027000);
}
__device__ __forceinline__ f32x4 buf_ld4(__amdgpu_buffer_rsrc_t r, uint32_t byte_off) {
  return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, SWIFT_LOAD_AUX));
}
__device__ __forceinline__ void buf_st4(__amdgpu_buffer_rsrc_t r, uint32_t byte_off, f32x4 val) {
  __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, val), r, (int)byte_off, 0, SWIFT_STORE_AUX);
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t hi16) { return __uint_as_float(hi16 << 16); }

// Nearest bfloat16 (the upper half of binary32) of a binary32 value, ties to even, overflow to
// infinity, every NaN to the quiet NaN 0x7FC0.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  const uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// Square root of a binary64 that is at least 2^-767 or zero, negative, infinite or NaN -- which holds
// for every second moment here: a binary32 value, or beta2 * binary32 + (1-beta2) * (binary32)^2, times
// 1/(1-beta2^t) >= 1.  It is the compiler's own binary64 expansion (reciprocal-root seed, two coupled
// Newton steps, two residual corrections; 0 and +inf pass through, negative gives NaN) without the
// rescaling of arguments below 2^-767 that cannot occur here: same result bits, five instructions fewer.
__device__ __forceinline__ double sqrt_moment(double x) {
  const double y = __builtin_amdgcn_rsq(x);
  double g = x * y;
  double h = y * 0.5;
  const double r = fma(-h, g, 0.5);
  g = fma(g, r, g);
  h = fma(h, r, h);
  double d = fma(-g, g, x);
  g = fma(d, h, g);
  d = fma(-g, g, x);
  g = fma(d, h, g);
  return __builtin_amdgcn_class(x, 0x260) ? x : g;                 // +-0 and +inf: the argument itself
}

// One element.  The vector body and the scalar head/tail path both call this, so an element's
// result bits do not depend on where it falls in a chunk or on pointer alignment.
// u = m^ / (sqrt(v^) + eps) with m^ = m/(1-beta1^t), v^ = v/(1-beta2^t)   (App. A).
template <int KIND, bool UNDO>
__device__ __forceinline__ void update_elem(float &xf, float gf, float &mf, float &vf, const OptConsts &c) {
  const double x = (double)xf, g = (double)gf, m = (double)mf;
  if constexpr (KIND == kSGD) {                     // App. A "SGD" / "Undo SGD": theta only
    if constexpr (!UNDO) xf = (float)fma(-c.eta, fma(c.lam, x, g), x);
    else xf = (float)(fma(c.eta, g, x) * c.inv_oml);
  } else if constexpr (KIND == kSGDM) {
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
      // coupled decay can make g' = g + lambda x arbitrarily small in binary64 (an absurdly small lambda), so
      // Adam's step keeps the general root; with the raw binary32 gradient the argument is in sqrt_moment's range
      const double root = (KIND == kADAM) ? sqrt(vt * c.rbc2) : sqrt_moment(vt * c.rbc2);
      const double u = (mt * c.rbc1) / (root + c.eps);
      mf = (float)mt;
      vf = (float)vt;
      if constexpr (KIND == kADAM) xf = (float)fma(-c.eta, u, x);
      else xf = (float)fma(-c.eta, fma(c.lam, x, u), x);
    } else {                                        // App. A "Undo Adam" / "Undo AdamW"
      const double u = (m * c.rbc1) / (sqrt_moment(v * c.rbc2) + c.eps);
      double xt = fma(c.eta, u, x);
      if constexpr (KIND == kADAMW) xt *= c.inv_oml;
      const double gp = (KIND == kADAM) ? fma(c.lam, xt, g) : g;
      xf = (float)xt;
      mf = (float)(fma(-c.c1, gp, m) * c.inv_b1);
      double vt = fma(-c.c2, gp * gp, v) * c.inv_b2;
      if (c.clamp_v && vt < 0.0) vt = 0.0;          // optional, not in the paper: see SWIFT_CLAMP_V
      vf = (float)vt;
    }
  }
}

// An "op" tells process_tile which streams a kernel moves and what to do with one element:
//   kLoadG, kHasM, kHasV   gradient / first moment (momentum buffer) / second moment are read
//   kStoreX, kStoreM, kStoreV   streams written back
//   kStoreXB               the bfloat16 copy of the new theta is written too
//   elem(i, x, g, m, v)    the arithmetic of element i of the chunk (may also accumulate into
//                          members of the op)
//   kPost, post(i, x, m, v)  if kPost: called for element i with the values that were stored, AFTER the
//                          stores of its vector have been issued (work that only reads the results runs
//                          while the stores are on their way)
template <int KIND, bool UNDO, bool XB = false>
struct OptOp {             // optimizer step or undo of one element
  static constexpr bool kLoadG = true, kHasM = (KIND != kSGD), kHasV = (KIND == kADAM || KIND == kADAMW);
  static constexpr bool kStoreX = true, kStoreM = kHasM, kStoreV = kHasV, kStoreXB = XB;
  static constexpr bool kPost = false;
  const OptConsts &c;
  __device__ __forceinline__ void elem(uint32_t, float &x, float g, float &m, float &v) {
    update_elem<KIND, UNDO>(x, g, m, v, c);
  }
};

template <typename Op>
__device__ __forceinline__ void update_vec4(Op &op, uint32_t j, f32x4 &x, const f32x4 &g, f32x4 &m, f32x4 &v) {
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    float xe = x[k], me = Op::kHasM ? m[k] : 0.f, ve = Op::kHasV ? v[k] : 0.f;
    op.elem(4u * j + k, xe, Op::kLoadG ? g[k] : 0.f, me, ve);
    x[k] = xe;
    if constexpr (Op::kHasM) m[k] = me;
    if constexpr (Op::kHasV) v[k] = ve;
  }
}

template <typename Op>
__device__ __forceinline__ void post_vec4(Op &op, uint32_t j, const f32x4 &x, const f32x4 &m, const f32x4 &v) {
#pragma unroll
  for (int k = 0; k < 4; ++k) op.post(4u * j + k, x[k], Op::kHasM ? m[k] : 0.f, Op::kHasV ? v[k] : 0.f);
}

// The bfloat16 copy of vector j (4 consecutive elements): 8 bytes.
__device__ __forceinline__ void buf_st_bf16x4(__amdgpu_buffer_rsrc_t r, uint32_t j, const f32x4 &val) {
  u32x2 packed;
  packed[0] = f32_to_bf16_bits(val[0]) | (f32_to_bf16_bits(val[1]) << 16);
  packed[1] = f32_to_bf16_bits(val[2]) | (f32_to_bf16_bits(val[3]) << 16);
  __builtin_amdgcn_raw_buffer_store_b64(packed, r, (int)(j * 8u), 0, SWIFT_STORE_AUX);
}

// Vector j (4 consecutive elements) of the chunk's gradient, widened to fp32.
template <bool BF16G>
__device__ __forceinline__ f32x4 load_grad4(__amdgpu_buffer_rsrc_t rg, uint32_t j) {
  if constexpr (BF16G) {
    const u32x2 raw = __builtin_amdgcn_raw_buffer_load_b64(rg, (int)(j * 8u), 0, SWIFT_LOAD_AUX);   // 4 bf16
    f32x4 r;
    r[0] = bf16_bits_to_f32(raw[0] & 0xFFFFu);
    r[1] = bf16_bits_to_f32(raw[0] >> 16);
    r[2] = bf16_bits_to_f32(raw[1] & 0xFFFFu);
    r[3] = bf16_bits_to_f32(raw[1] >> 16);
    return r;
  } else {
    return buf_ld4(rg, j * 16u);
  }
}

template <bool BF16G>
__device__ __forceinline__ float load_grad1(const void *g, int64_t i) {
  if constexpr (BF16G) return bf16_bits_to_f32(ld<false>(reinterpret_cast<const uint16_t *>(g) + i));
  else return ld<false>(reinterpret_cast<const float *>(g) + i);
}

// One element through 4-byte accesses (ragged tails and unaligned tensors).
template <typename Op, bool BF16G>
__device__ __forceinline__ void process_scalar(Op &op, const ChunkDesc &d, uint32_t e) {
  float xe = ld<false>(d.x + e), me = 0.f, ve = 0.f, ge = 0.f;
  if constexpr (Op::kHasM) me = ld<false>(d.m + e);
  if constexpr (Op::kHasV) ve = ld<false>(d.v + e);
  if constexpr (Op::kLoadG) ge = load_grad1<BF16G>(d.g, e);
  op.elem(e, xe, ge, me, ve);
  if constexpr (Op::kStoreX) st<false>(d.x + e, xe);
  if constexpr (Op::kStoreXB) st<false>(d.xb + e, (uint16_t)f32_to_bf16_bits(xe));
  if constexpr (Op::kStoreM) st<false>(d.m + e, me);
  if constexpr (Op::kStoreV) st<false>(d.v + e, ve);
  if constexpr (Op::kPost) op.post(e, xe, me, ve);
}

// A hook lets a kernel slip one more memory request in behind a tile's loads, while they are in flight.
struct NoHook {
  __device__ __forceinline__ void after_loads() {}
};

// One tile: U*BLOCK 16-byte vectors (U*BLOCK*4 elements) of one chunk, starting at element
// ti * U*BLOCK*4 of the chunk (the caller has checked that this is inside the chunk).
template <typename Op, bool BF16G, int U, int BLOCK, typename Hook = NoHook>
__device__ __forceinline__ void process_tile(Op &op, const ChunkDesc &d, uint32_t ti, uint32_t tid, Hook hook = Hook()) {
  constexpr bool HASV = Op::kHasV, HASM = Op::kHasM;
  const f32x4 zero4{0.f, 0.f, 0.f, 0.f};
  constexpr uint32_t TILE4 = U * BLOCK;                          // vectors per tile
  const uint32_t len = d.len;
  if (d.vec_ok) {
    // chunk starts are multiples of 4 elements, so chunks keep their tensor's 16-byte alignment
    const uint32_t n4 = len >> 2;
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(d.x, n4 * 16u), rm = make_rsrc(d.m, HASM ? n4 * 16u : 0u);
    const __amdgpu_buffer_rsrc_t rv = make_rsrc(d.v, HASV ? n4 * 16u : 0u);
    const __amdgpu_buffer_rsrc_t rg = make_rsrc(d.g, Op::kLoadG ? n4 * (BF16G ? 8u : 16u) : 0u);
    const __amdgpu_buffer_rsrc_t rxb = make_rsrc(d.xb, Op::kStoreXB ? n4 * 8u : 0u);
    const uint32_t j0 = ti * TILE4;
    if (j0 + TILE4 <= n4) {                                      // full tile: no predicates
      f32x4 xr[U], gr[U], mr[U], vr[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t j = j0 + u * BLOCK + tid;
        xr[u] = buf_ld4(rx, j * 16u);
        gr[u] = Op::kLoadG ? load_grad4<BF16G>(rg, j) : zero4;
        mr[u] = HASM ? buf_ld4(rm, j * 16u) : zero4;
        vr[u] = HASV ? buf_ld4(rv, j * 16u) : zero4;
      }
      // Every load of the tile goes out before anything waits for one of them.  Left alone, the scheduler put the
      // last load of the undo kernels with bf16 gradients behind the wait for the first (a full memory latency per
      // tile: GPT-2 list, undo 6.56 against 6.14 ms for the step at the same residency).
      __builtin_amdgcn_sched_barrier(0);
      hook.after_loads();
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t j = j0 + u * BLOCK + tid;
        update_vec4(op, j, xr[u], gr[u], mr[u], vr[u]);
        if constexpr (Op::kStoreX) buf_st4(rx, j * 16u, xr[u]);
        if constexpr (Op::kStoreXB) buf_st_bf16x4(rxb, j, xr[u]);
        if constexpr (Op::kStoreM) buf_st4(rm, j * 16u, mr[u]);
        if constexpr (Op::kStoreV) buf_st4(rv, j * 16u, vr[u]);
      }
      if constexpr (Op::kPost) {
#pragma unroll
        for (int u = 0; u < U; ++u) post_vec4(op, j0 + u * BLOCK + tid, xr[u], mr[u], vr[u]);
      }
    } else {                                                     // ragged end of a tensor
      hook.after_loads();
      for (uint32_t j = j0 + tid; j < n4; j += BLOCK) {
        f32x4 xr = buf_ld4(rx, j * 16u), mr = HASM ? buf_ld4(rm, j * 16u) : zero4;
        f32x4 gr = Op::kLoadG ? load_grad4<BF16G>(rg, j) : zero4;
        f32x4 vr = HASV ? buf_ld4(rv, j * 16u) : zero4;
        update_vec4(op, j, xr, gr, mr, vr);
        if constexpr (Op::kStoreX) buf_st4(rx, j * 16u, xr);
        if constexpr (Op::kStoreXB) buf_st_bf16x4(rxb, j, xr);
        if constexpr (Op::kStoreM) buf_st4(rm, j * 16u, mr);
        if constexpr (Op::kStoreV) buf_st4(rv, j * 16u, vr);
        if constexpr (Op::kPost) post_vec4(op, j, xr, mr, vr);
      }
      const uint32_t e = (n4 << 2) + tid;                        // last numel % 4 elements
      if (e < len) process_scalar<Op, BF16G>(op, d, e);          // (they start inside this tile)
    }
  } else {                                                       // unaligned tensor: 4-byte accesses
    hook.after_loads();
    const uint32_t e0 = ti * (TILE4 * 4u);
    const uint32_t e1 = (e0 + TILE4 * 4u < len) ? e0 + TILE4 * 4u : len;
    for (uint32_t e = e0 + tid; e < e1; e += BLOCK) process_scalar<Op, BF16G>(op, d, e);
  }
}

// A whole 64-byte table entry in one scalar load (the table is not written while a kernel that
// reads it runs, which is what the constant address space requires).  Field by field the compiler
// fetches the length first and the pointers in later rounds, each a scalar-cache round trip.
__device__ __forceinline__ ChunkDesc fetch_desc(const ChunkDesc *p) {
  typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));
  typedef const __attribute__((address_space(4))) u32x16 *const_u32x16_ptr;
  static_assert(sizeof(ChunkDesc) == sizeof(u32x16), "table entry is 64 bytes");
  const u32x16 raw = *(const_u32x16_ptr)p;
  ChunkDesc d;
  __builtin_memcpy(&d, &raw, sizeof d);
  return d;
}

// The tiles of one workgroup: slot w = blockIdx.x, then every gridDim.x-th slot below `end`.  A
// chunk is up to chunk_elems consecutive elements of one tensor (the last chunk of a tensor is
// short) and spans 2^tpc_shift tile slots, so slot w is tile (w & (tpc-1)) of chunk (w >> tpc_shift).
// The chunk table holds ready-made pointers, so a wavefront is two rounds of scalar loads (kernel
// arguments, table entry) away from issuing its vector loads; nothing else may sit in front of the
// first entry fetch (one more dependent scalar load there cost the lightest kernel, SGDM with bf16
// gradients, 7 %).  The host launches at most as many workgroups as the table has slots, so the
// first pass needs no bounds test.
template <int KIND, bool UNDO, bool BF16G, bool XB, int U, int BLOCK, bool DRAIN>
__device__ __forceinline__ void opt_tiles(const ChunkDesc *__restrict__ chunks, uint64_t end, uint32_t tpc_shift,
                                          const OptConsts &c) {
  constexpr uint32_t TILE = U * BLOCK * 4u;                      // elements per tile
  OptOp<KIND, UNDO, XB> op{c};
  uint64_t w = blockIdx.x;
  do {
    const ChunkDesc d = fetch_desc(chunks + (w >> tpc_shift));
    const uint32_t ti = (uint32_t)w & ((1u << tpc_shift) - 1u);
    if (ti * TILE >= d.len) continue;                            // slot past the end of a short chunk
    process_tile<OptOp<KIND, UNDO, XB>, BF16G, U, BLOCK>(op, d, ti, threadIdx.x);
    // A workgroup that goes round again first lets its stores drain (s_waitcnt vmcnt(0)), as a
    // retiring workgroup would before its slot is reused: measured 1-3 % faster for strided launches.
    if constexpr (DRAIN) __builtin_amdgcn_s_waitcnt(0x0F70);
  } while ((w += gridDim.x) < end);
}

// One workgroup per tile: the grid equals the number of slots, and the hardware dispatcher hands
// tiles out in address order as wavefronts retire, which keeps the window of HBM pages in flight
// narrow (a persistent grid-stride loop lets workgroups drift apart and measured 10-20 % slower
// for this 4-read/3-write pattern; so did several tiles per workgroup).  The launch passes dynamic
// LDS that is never touched: it only caps how many workgroups share a compute unit, because more
// than ~11 wavefronts per CU in flight lowers the achieved HBM bandwidth of the mixed read/write
// stream.
template <int KIND, bool UNDO, bool BF16G, bool XB, int U, int BLOCK>
__global__ void __launch_bounds__(BLOCK)
opt_kernel(const ChunkDesc *__restrict__ chunks, uint64_t n_slots, uint32_t tpc_shift, const OptConsts c) {
  opt_tiles<KIND, UNDO, BF16G, XB, U, BLOCK, false>(chunks, n_slots, tpc_shift, c);
}

// The same update over a table that compact_chunks_kernel packed from a device-resident mask: only
// the device knows how many slots it holds (*n_slots_dev; entries past that count are empty), so
// the grid is capped by the host, workgroups stride over the slots and stop at the count.
template <int KIND, bool UNDO, bool BF16G, bool XB, int U, int BLOCK>
__global__ void __launch_bounds__(BLOCK)
opt_packed_kernel(const ChunkDesc *__restrict__ chunks, const uint64_t *__restrict__ n_slots_dev, uint32_t tpc_shift,
                  const OptConsts c) {
  typedef const __attribute__((address_space(4))) uint64_t *const_u64_ptr;   // uniform address: scalar load
  opt_tiles<KIND, UNDO, BF16G, XB, U, BLOCK, true>(chunks, *(const_u64_ptr)n_slots_dev, tpc_shift, c);
}

// The packed table again, but with a fixed grid of resident wavefronts that ask for their tiles: the
// wavefronts of counter c (blockIdx mod n_counters) draw j = 0, 1, 2, ... from it and take slot
// j * n_counters + c, so slots are handed out in address order, as the dispatcher does for one tile
// per workgroup, and a launch costs time in proportion to the marked tiles only -- no workgroup is
// dispatched for nothing, whatever the mask's density.  The request for the next index goes out
// behind the current tile's loads and comes back while the tile is processed.  Every wavefront ends:
// the counters only grow, and a wavefront leaves as soon as its slot is at or beyond the count.
// counters: one 32-bit counter per 128 bytes, zero when the kernel starts (compact_chunks_kernel clears them).
struct NextTile {
  unsigned int *counter;
  uint32_t *next;
  __device__ __forceinline__ void after_loads() {
    if (threadIdx.x == 0) *next = atomicAdd(counter, 1u);
  }
};

template <int KIND, bool UNDO, bool BF16G, bool XB, int U, int BLOCK>
__global__ void __launch_bounds__(BLOCK)
opt_queue_kernel(const ChunkDesc *__restrict__ chunks, const uint64_t *__restrict__ n_slots_dev, uint32_t tpc_shift,
                 const OptConsts c, unsigned int *__restrict__ counters, uint32_t log2_counters) {
  typedef const __attribute__((address_space(4))) uint64_t *const_u64_ptr;
  constexpr uint32_t TILE = U * BLOCK * 4u;
  const uint32_t lane_c = blockIdx.x & ((1u << log2_counters) - 1u);
  unsigned int *ctr = counters + lane_c * 32u;
  const uint64_t end = *(const_u64_ptr)n_slots_dev;
  uint32_t j = 0;
  if (threadIdx.x == 0) j = atomicAdd(ctr, 1u);
  j = (uint32_t)__builtin_amdgcn_readfirstlane((int)j);
  OptOp<KIND, UNDO, XB> op{c};
  for (;;) {
    const uint64_t w = ((uint64_t)j << log2_counters) + lane_c;
    if (w >= end) break;
    const ChunkDesc d = fetch_desc(chunks + (w >> tpc_shift));
    const uint32_t ti = (uint32_t)w & ((1u << tpc_shift) - 1u);
    uint32_t nxt = 0;
    NextTile hook{ctr, &nxt};
    if (ti * TILE < d.len) process_tile<OptOp<KIND, UNDO, XB>, BF16G, U, BLOCK, NextTile>(op, d, ti, threadIdx.x, hook);
    else hook.after_loads();
    // The wavefront lets its stores drain before it takes its next tile, as a retiring workgroup would before its
    // slot is reused (6.35 against 6.04 TB/s without); by then the next index has arrived as well.  Fetching the next
    // tile's table entry one tile ahead (two indices in flight) was measured too and is slower (6.08).
    __builtin_amdgcn_s_waitcnt(0x0F70);
    j = (uint32_t)__builtin_amdgcn_readfirstlane((int)nxt);
  }
}

// Plain copy with the same launch shape (one tile of U*BLOCK 16-byte vectors per workgroup): the
// practical HBM ceiling of a 1-read/1-write stream and the calibration run for byte counters.
template <int U, int BLOCK>
__global__ void __launch_bounds__(BLOCK)
copy_kernel(u32x4 *__restrict__ dst, const u32x4 *__restrict__ src, uint64_t n16) {
  constexpr bool NT = SWIFT_NT != 0;
  const uint64_t tile = (uint64_t)U * BLOCK;
  const uint64_t n_tiles = (n16 + tile - 1) / tile;
  for (uint64_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
    const uint64_t i0 = t * tile + threadIdx.x;
    u32x4 r[U];
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (i0 + (uint64_t)u * BLOCK < n16) r[u] = ld<NT>(src + i0 + (uint64_t)u * BLOCK);
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (i0 + (uint64_t)u * BLOCK < n16) st<NT>(dst + i0 + (uint64_t)u * BLOCK, r[u]);
  }
}

}  // namespace swift
