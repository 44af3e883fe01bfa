// Optimizer step / undo fused with the digest of the state it leaves behind (gfx950).
//
// A training loop that wants to recognise stepped tensors after a failure needs the digests of
// the state at the last completed iteration.  Computing them in a pass of their own re-reads
// theta, m and v (12 bytes per parameter, 45 % on top of an Adam step); here the kernel that
// writes the new state also mixes the words it writes, so the reference digests cost no HBM
// traffic beyond 24 bytes per tile.  Per tile the three lane sums are combined in one pass of lane
// exchanges (DPP inside the rows, lane swaps across them) and stored in the tile's slot; two small kernels then add the tile slots of each chunk and the
// chunk sums of each tensor (order-free: the digest is a sum mod 2^64).  The results equal what
// swift_state_digest returns for the same buffers with one shard per buffer.
// The kernel is bound by instruction issue, not by HBM: about 48 vector instructions of update
// arithmetic plus 3 x 16 of mixing per element, at a shader clock that the chip lowers under this
// load; see the instruction-rate and counter notes that come with the benchmarks.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "opt_kernels.hpp"
#include "digest_kernels.hpp"
#include "lamb_kernels.hpp"

namespace swift {

template <int KIND, bool UNDO, bool XB>
struct OptDigestOp {       // step or undo of one element + digest contributions of its new words
  static constexpr bool kLoadG = true, kHasM = (KIND != kSGD), kHasV = (KIND == kADAM || KIND == kADAMW);
  static constexpr bool kStoreX = true, kStoreM = kHasM, kStoreV = kHasV, kStoreXB = XB;
  static constexpr bool kPost = true;      // the words are mixed after their stores have been issued
  const OptConsts &c;
  uint32_t base;           // index of the chunk's first element inside its tensor, plus the mixer's K1.hi
  uint64_t dx = 0, dm = 0, dv = 0;
  __device__ __forceinline__ void elem(uint32_t, float &x, float g, float &m, float &v) {
    update_elem<KIND, UNDO>(x, g, m, v, c);
  }
  __device__ __forceinline__ void post(uint32_t i, float x, float m, float v) {
    const uint32_t idx = base + i;
    dx += digest_mix_pre(idx, __float_as_uint(x));
    if constexpr (kHasM) dm += digest_mix_pre(idx, __float_as_uint(m));
    if constexpr (kHasV) dv += digest_mix_pre(idx, __float_as_uint(v));
  }
};

// One workgroup (one wavefront) per tile; tile_digest[3w + k] receives the theta, m, v sums of tile
// slot w (k = 0, 1, 2) with plain stores.  Atomic adds into per-chunk slots were measured first and
// bound the kernel: the 256 tiles of a chunk are in flight together and their atomics serialise on a
// few cache lines, and a wavefront cannot retire before its atomics are acknowledged (35 ms for the 7B
// list with three single-lane atomics per tile, 48 ms with one 12-lane atomic instruction).
template <int KIND, bool UNDO, bool BF16G, bool XB, int U, int BLOCK>
__global__ void __launch_bounds__(BLOCK)
opt_digest_kernel(const ChunkDesc *__restrict__ chunks, uint64_t n_slots, uint32_t tpc_shift, const OptConsts c,
                  uint64_t *__restrict__ tile_digest) {
  static_assert(BLOCK == 64, "the tile digest is a single-wavefront reduction");
  constexpr uint32_t TILE = U * BLOCK * 4u;
  uint64_t w = blockIdx.x;
  do {
    const ChunkDesc d = fetch_desc(chunks + (w >> tpc_shift));
    const uint32_t ti = (uint32_t)w & ((1u << tpc_shift) - 1u);
    if (ti * TILE >= d.len) continue;
    OptDigestOp<KIND, UNDO, XB> op{c, d.elem0 + (uint32_t)(kK1 >> 32)};
    process_tile<OptDigestOp<KIND, UNDO, XB>, BF16G, U, BLOCK>(op, d, ti, threadIdx.x);
    // lanes 0, 1, 2 end with the theta, m and v sums and store them side by side
    const uint64_t sum = wave_sum3_u64(op.dx, op.dm, op.dv);
    constexpr uint32_t kGroups = (KIND == kSGD) ? 1u : (KIND == kSGDM ? 2u : 3u);   // theta [, m [, v]]
    if (threadIdx.x < kGroups) st<false>(tile_digest + 3 * w + threadIdx.x, sum);
  } while ((w += gridDim.x) < n_slots);
}

// One workgroup per chunk: chunk_digest[3c + g] = sum of the chunk's tile sums of group g (only
// the tiles that exist: a tensor's last chunk is short, and the slots behind it were never written).
__global__ void __launch_bounds__(kThreads)
chunk_digest_kernel(const ChunkDesc *__restrict__ chunks, uint32_t tpc_shift, uint32_t tile_elems, uint32_t n_groups,
                    const uint64_t *__restrict__ tile_digest, uint64_t *__restrict__ chunk_digest) {
  __shared__ uint64_t part[3][kThreads / 64];
  const uint32_t ci = blockIdx.x, tid = threadIdx.x;
  const uint32_t n_tiles = (chunks[ci].len + tile_elems - 1) / tile_elems;
  const uint64_t *slots = tile_digest + 3 * ((uint64_t)ci << tpc_shift);
  uint64_t acc[3] = {0, 0, 0};
  for (uint32_t t = tid; t < n_tiles; t += kThreads)
    for (uint32_t g = 0; g < n_groups; ++g) acc[g] += slots[3 * (uint64_t)t + g];
#pragma unroll
  for (int g = 0; g < 3; ++g) {
    const uint64_t s = wave_sum_u64(acc[g]);
    if ((tid & 63u) == 0) part[g][tid >> 6] = s;
  }
  __syncthreads();
  if (tid < n_groups) {
    uint64_t t = 0;
#pragma unroll
    for (int wv = 0; wv < kThreads / 64; ++wv) t += part[tid][wv];
    chunk_digest[3 * (uint64_t)ci + tid] = t;
  }
}

// One wavefront per tensor: out[g * n_tensors + i] = sum of the tensor's chunk slots of group g
// (g = 0 theta, 1 m, 2 v).  spans[i] holds the tensor's first chunk and chunk count.
__global__ void __launch_bounds__(64)
digest_gather_kernel(const TensorSpan *__restrict__ spans, const uint64_t *__restrict__ chunk_digest,
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
