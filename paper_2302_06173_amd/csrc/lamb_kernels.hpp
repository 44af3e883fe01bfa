// LAMB step and its saved-norm undo for gfx950.
//
// LAMB is Adam's elementwise arithmetic plus one non-invertible operator, a sum: the L2 norms
// behind the per-tensor trust ratio (paper, Table 1 and section "Update-undo").  The paper's
// remedy is to save the norm at step time; the undo is then elementwise again.  Per tensor:
//   m_t, v_t as AdamW;  r = m^/(sqrt(v^)+eps);  u = r + lambda x_t;
//   q = ||x_t|| / ||u||  (1 if either norm is 0);  x_{t+1} = x_t - eta q u
//   undo: x_t = (x_{t+1} + eta q r) / (1 - eta q lambda);  m, v as "Undo AdamW" (App. A).
// The step is three launches: (1) moments + per-tile partial sums of x^2 and u^2 (reads theta,
// g, m, v; writes m, v: 24 B per element), (2) a fixed-order reduction of the partials to the two
// norms of every tensor, (3) the parameter update (reads theta, m, v; writes theta: 16 B per
// element, 18 with a bfloat16 copy of theta).  Partial sums are combined in a fixed order (lane tree, then strided sums, then an
// LDS tree), so the saved norms -- and with them every replica's parameters -- are bit-identical
// from run to run.  The undo is one launch with AdamW-undo traffic (28 B per element).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "opt_kernels.hpp"
#include "digest_kernels.hpp"

namespace swift {

struct TensorSpan {        // one per tensor of the caller's list, device resident
  uint64_t first_slot;     // first tile slot of the tensor in the partial-sum array
  uint64_t n_slots;        // tile slots that hold a partial sum (0 for empty or unmarked tensors)
  uint32_t active;         // 1: the tensor takes part in this call
  uint32_t pad;
};

// Two sums over the 64 lanes at once, in a fixed order: afterwards lane 0 holds the sum of a and lane 1 the sum
// of b (every even lane holds a sum of a, every odd lane one of b, formed in lane-dependent but fixed order).
// In the first exchange a lane keeps one of its two values and hands the other to its partner, which keeps that
// one; from then on a single register moves, and the rows are combined by lane swaps instead of lane reads.
__device__ __forceinline__ double wave_sum2_f64(double a, double b) {
  const bool odd = (threadIdx.x & 1u) != 0;
  auto bits = [](double x) { return (uint64_t)__double_as_longlong(x); };
  auto dbl = [](uint64_t x) { return __longlong_as_double((long long)x); };
  double r = (odd ? b : a) + dbl(dpp_fetch_u64<0xB1>(bits(odd ? a : b)));   // lane ^ 1
  r += dbl(dpp_fetch_u64<0x4E>(bits(r)));                                    // lane ^ 2
  r += dbl(dpp_fetch_u64<0x124>(bits(r)));                                   // row_ror:4 (keeps the lane's parity)
  r += dbl(dpp_fetch_u64<0x128>(bits(r)));                                   // row_ror:8 -> sums over the row
  // rows: v_permlane16_swap gives {row0, row0, row2, row2} and {row1, row1, row3, row3}, v_permlane32_swap the halves
  uint32_t lo = (uint32_t)bits(r), hi = (uint32_t)(bits(r) >> 32);
  auto pl = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
  auto ph = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
  r = dbl(((uint64_t)ph[0] << 32) | pl[0]) + dbl(((uint64_t)ph[1] << 32) | pl[1]);
  lo = (uint32_t)bits(r);
  hi = (uint32_t)(bits(r) >> 32);
  pl = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
  ph = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
  return dbl(((uint64_t)ph[0] << 32) | pl[0]) + dbl(((uint64_t)ph[1] << 32) | pl[1]);
}

// Pass 1 of the step: the moment recurrences (written back) and the running sums for the norms.
struct LambMomentsOp {
  static constexpr bool kLoadG = true, kHasM = true, kHasV = true, kStoreX = false, kStoreM = true, kStoreV = true, kStoreXB = false;
  static constexpr bool kPost = false;
  const OptConsts &c;
  double sx = 0.0, su = 0.0;
  __device__ __forceinline__ void elem(uint32_t, float &xf, float gf, float &mf, float &vf) {
    const double x = (double)xf, g = (double)gf;
    const double mt = fma(c.b1, (double)mf, c.c1 * g);
    const double vt = fma(c.b2, (double)vf, c.c2 * (g * g));
    const double r = (mt * c.rbc1) / (sqrt_moment(vt * c.rbc2) + c.eps);
    const double u = fma(c.lam, x, r);
    mf = (float)mt;
    vf = (float)vt;
    sx = fma(x, x, sx);
    su = fma(u, u, su);
  }
};

// Pass 3 of the step: x <- x - (eta q)(r + lambda x), r from the stored new moments.
template <bool XB>
struct LambApplyOp {
  static constexpr bool kLoadG = false, kHasM = true, kHasV = true, kStoreX = true, kStoreM = false, kStoreV = false, kStoreXB = XB;
  static constexpr bool kPost = false;
  const OptConsts &c;
  double eta_q;
  __device__ __forceinline__ void elem(uint32_t, float &xf, float, float &mf, float &vf) {
    const double x = (double)xf;
    const double r = ((double)mf * c.rbc1) / (sqrt_moment((double)vf * c.rbc2) + c.eps);
    xf = (float)fma(-eta_q, fma(c.lam, x, r), x);
  }
};

// Trust ratio from the two saved norms.
__device__ __forceinline__ double lamb_ratio(const double *norms, uint32_t tensor) {
  typedef const __attribute__((address_space(4))) double *const_f64_ptr;     // uniform address: scalar loads
  const double nx = ((const_f64_ptr)norms)[2 * (uint64_t)tensor], nu = ((const_f64_ptr)norms)[2 * (uint64_t)tensor + 1];
  return (nx > 0.0 && nu > 0.0) ? nx / nu : 1.0;
}

// One workgroup (one wavefront: BLOCK is 64) per tile; partial[slot] = {sum x^2, sum u^2} of the tile.
template <bool BF16G, int U, int BLOCK>
__global__ void __launch_bounds__(BLOCK)
lamb_moments_kernel(const ChunkDesc *__restrict__ chunks, uint64_t n_slots, uint32_t tpc_shift, const OptConsts c,
                    double2 *__restrict__ partial) {
  static_assert(BLOCK == 64, "the partial sum of a tile is a single-wavefront reduction");
  constexpr uint32_t TILE = U * BLOCK * 4u;
  uint64_t w = blockIdx.x;
  do {
    const ChunkDesc d = fetch_desc(chunks + (w >> tpc_shift));
    const uint32_t ti = (uint32_t)w & ((1u << tpc_shift) - 1u);
    if (ti * TILE >= d.len) continue;          // slot past the end of a short chunk
    LambMomentsOp op{c};
    process_tile<LambMomentsOp, BF16G, U, BLOCK>(op, d, ti, threadIdx.x);
    const double sum = wave_sum2_f64(op.sx, op.su);           // lane 0: sum x^2, lane 1: sum u^2
    if (threadIdx.x < 2) reinterpret_cast<double *>(partial)[2 * w + threadIdx.x] = sum;
  } while ((w += gridDim.x) < n_slots);
}

// One workgroup per tensor: norms[2i] = ||x||, norms[2i+1] = ||u|| from the tensor's partial sums,
// which occupy consecutive slots (only a tensor's last chunk is short).  Fixed summation order.
__global__ void __launch_bounds__(kThreads)
lamb_norms_kernel(const TensorSpan *__restrict__ spans, const double2 *__restrict__ partial, double *__restrict__ norms) {
  __shared__ double sh[2][kThreads];
  const TensorSpan sp = spans[blockIdx.x];
  if (!sp.active) return;
  double sx = 0.0, su = 0.0;
  for (uint64_t k = threadIdx.x; k < sp.n_slots; k += kThreads) {
    const double2 p = partial[sp.first_slot + k];
    sx += p.x;
    su += p.y;
  }
  sh[0][threadIdx.x] = sx;
  sh[1][threadIdx.x] = su;
  __syncthreads();
  for (uint32_t half = kThreads / 2; half > 0; half >>= 1) {
    if (threadIdx.x < half) {
      sh[0][threadIdx.x] += sh[0][threadIdx.x + half];
      sh[1][threadIdx.x] += sh[1][threadIdx.x + half];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    norms[2 * (uint64_t)blockIdx.x] = sqrt(sh[0][0]);
    norms[2 * (uint64_t)blockIdx.x + 1] = sqrt(sh[1][0]);
  }
}

// Pass 3 of the step: one workgroup per tile.
template <bool XB, int U, int BLOCK>
__global__ void __launch_bounds__(BLOCK)
lamb_apply_kernel(const ChunkDesc *__restrict__ chunks, uint64_t n_slots, uint32_t tpc_shift, const OptConsts c,
                  const double *__restrict__ norms) {
  constexpr uint32_t TILE = U * BLOCK * 4u;
  uint64_t w = blockIdx.x;
  do {
    const ChunkDesc d = fetch_desc(chunks + (w >> tpc_shift));
    const uint32_t ti = (uint32_t)w & ((1u << tpc_shift) - 1u);
    if (ti * TILE >= d.len) continue;
    LambApplyOp<XB> op{c, c.eta * lamb_ratio(norms, d.tensor)};
    process_tile<LambApplyOp<XB>, false, U, BLOCK>(op, d, ti, threadIdx.x);
  } while ((w += gridDim.x) < n_slots);
}

// Undo: AdamW's undo with eta q in place of eta (q from the saved norms), one workgroup per tile.
template <bool BF16G, bool XB, int U, int BLOCK>
__global__ void __launch_bounds__(BLOCK)
lamb_undo_kernel(const ChunkDesc *__restrict__ chunks, uint64_t n_slots, uint32_t tpc_shift, const OptConsts c,
                 const double *__restrict__ norms) {
  constexpr uint32_t TILE = U * BLOCK * 4u;
  uint64_t w = blockIdx.x;
  do {
    const ChunkDesc d = fetch_desc(chunks + (w >> tpc_shift));
    const uint32_t ti = (uint32_t)w & ((1u << tpc_shift) - 1u);
    if (ti * TILE >= d.len) continue;
    OptConsts cq = c;
    cq.eta = c.eta * lamb_ratio(norms, d.tensor);
    cq.inv_oml = 1.0 / (1.0 - cq.eta * c.lam);
    OptOp<kADAMW, true, XB> op{cq};
    process_tile<OptOp<kADAMW, true, XB>, BF16G, U, BLOCK>(op, d, ti, threadIdx.x);
  } while ((w += gridDim.x) < n_slots);
}

}  // namespace swift
