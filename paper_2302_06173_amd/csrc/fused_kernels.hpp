// Optimizer step / undo fused with the digest of the state it leaves behind (gfx950).
//
// A training loop that wants to recognise stepped tensors after a failure needs the digests of
// the state at the last completed iteration.  Computing them in a pass of their own re-reads
// theta, m and v (12 bytes per parameter, 45 % on top of an Adam step); here the kernel that
// writes the new state also mixes the words it writes, so the reference digests cost no HBM
// traffic beyond 24 bytes per chunk.  Per tile the three lane sums are combined by DPP and added
// to the chunk's three slots with 64-bit atomics (order-free: the digest is a sum mod 2^64); a
// second small kernel adds each tensor's chunk slots into the per-tensor digests, which equal
// what swift_state_digest returns for the same buffers with one shard per buffer.
// Measured on MI355X (7B list): the mixer's 32-bit integer multiplies run at half rate, so the
// digest arithmetic alone sustains about 1.75 T words/s; fused into the update it makes the kernel
// ALU-bound (step 35.3 ms, undo 36.1 ms) instead of HBM-bound, against 28.6 + 12.7 ms for the
// two separate passes: a gain of 13-14 %, not the 30 % the saved traffic alone would give.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "opt_kernels.hpp"
#include "digest_kernels.hpp"
#include "lamb_kernels.hpp"

namespace swift {

template <int KIND, bool UNDO, bool XB>
struct OptDigestOp {       // step or undo of one element + digest contributions of its new words
  static constexpr bool kLoadG = true, kHasV = (KIND != kSGDM);
  static constexpr bool kStoreX = true, kStoreM = true, kStoreV = kHasV, kStoreXB = XB;
  const OptConsts &c;
  uint32_t elem0;          // index of the chunk's first element inside its tensor
  uint64_t dx = 0, dm = 0, dv = 0;
  __device__ __forceinline__ void elem(uint32_t i, float &x, float g, float &m, float &v) {
    update_elem<KIND, UNDO>(x, g, m, v, c);
    const uint32_t idx = elem0 + i;
    dx += digest_mix(idx, __float_as_uint(x));
    dm += digest_mix(idx, __float_as_uint(m));
    if constexpr (kHasV) dv += digest_mix(idx, __float_as_uint(v));
  }
};

// One workgroup (one wavefront) per tile; chunk_digest[3c + k] accumulates theta, m, v of chunk c.
template <int KIND, bool UNDO, bool BF16G, bool XB, int U, int BLOCK>
__global__ void __launch_bounds__(BLOCK)
opt_digest_kernel(const ChunkDesc *__restrict__ chunks, uint64_t n_slots, uint32_t tpc_shift, const OptConsts c,
                  unsigned long long *__restrict__ chunk_digest) {
  static_assert(BLOCK == 64, "the tile digest is a single-wavefront reduction");
  constexpr uint32_t TILE = U * BLOCK * 4u;
  uint64_t w = blockIdx.x;
  do {
    const uint64_t ci = w >> tpc_shift;
    const ChunkDesc d = fetch_desc(chunks + ci);
    const uint32_t ti = (uint32_t)w & ((1u << tpc_shift) - 1u);
    if (ti * TILE >= d.len) continue;
    OptDigestOp<KIND, UNDO, XB> op{c, d.elem0};
    process_tile<OptDigestOp<KIND, UNDO, XB>, BF16G, U, BLOCK>(op, d, ti, threadIdx.x);
    const uint64_t sx = wave_sum_u64(op.dx), sm = wave_sum_u64(op.dm);
    const uint64_t sv = (KIND != kSGDM) ? wave_sum_u64(op.dv) : 0;
    if (threadIdx.x == 0) {
      atomicAdd(chunk_digest + 3 * ci, (unsigned long long)sx);
      atomicAdd(chunk_digest + 3 * ci + 1, (unsigned long long)sm);
      if constexpr (KIND != kSGDM) atomicAdd(chunk_digest + 3 * ci + 2, (unsigned long long)sv);
    }
  } while ((w += gridDim.x) < n_slots);
}

// One wavefront per tensor: out[g * n_tensors + i] = sum of the tensor's chunk slots of group g
// (g = 0 theta, 1 m, 2 v).  spans[i] holds the tensor's first chunk and chunk count.
__global__ void __launch_bounds__(64)
digest_gather_kernel(const TensorSpan *__restrict__ spans, const unsigned long long *__restrict__ chunk_digest,
                     uint32_t n_tensors, uint32_t n_groups, uint64_t *__restrict__ out) {
  const TensorSpan sp = spans[blockIdx.x];
  if (!sp.active) return;
  for (uint32_t g = 0; g < n_groups; ++g) {
    uint64_t acc = 0;
    for (uint64_t k = threadIdx.x; k < sp.n_slots; k += 64) acc += chunk_digest[3 * (sp.first_slot + k) + g];
    const uint64_t total = wave_sum_u64(acc);
    if (threadIdx.x == 0) out[(uint64_t)g * n_tensors + blockIdx.x] = total;
  }
}

}  // namespace swift
