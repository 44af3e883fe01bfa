// State-digest kernels for gfx950.
//
// The digest of a shard is the modulo-2^64 sum of a bijectively mixed (index, word) pair per
// 32-bit word, so partial sums can be combined in any order: lanes accumulate privately, a
// wavefront combines its 64 lanes with DPP row operations and cross-row lane reads, the four
// wavefronts of a workgroup meet in LDS, and a second small kernel adds the chunk sums of a shard.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "opt_kernels.hpp"

namespace swift {

struct DigestDesc {        // one per buffer, 24 bytes, device resident
  const uint32_t *w;       // raw 32-bit words
  int64_t numel;
  uint64_t first_out;      // index of this buffer's first shard in the output array
};

constexpr uint64_t kK1 = 0x9E3779B97F4A7C15ull;
constexpr uint64_t kK2 = 0x6A09E667F3BCC909ull;
constexpr uint64_t kK3 = 0xBB67AE8584CAA73Bull;

// z = (i << 32) | w;  z += K1;  z ^= z >> 32;  z *= K2;  z ^= z >> 29;  z *= K3;  z ^= z >> 32
// The first two steps are written on the 32-bit halves: the low half is w + K1.lo, the high half
// i + K1.hi + carry (one add-with-carry pair, and when i is a register plus a constant the constant
// folds into K1.hi), and after z ^= z >> 32 the low half is lo ^ hi.  Every instruction of the mixer
// issues at full rate on gfx950 (32-bit multiplies and 64-bit shifts included); 16 per word is the
// floor: a 64 x 64 -> 64 bit multiply takes two 32-bit multiplies, one 32 x 32 -> 64 and a 3-input add.
// digest_mix_pre takes i + K1.hi (mod 2^32), which a loop over consecutive words keeps in a register.
__device__ __forceinline__ uint64_t digest_mix_pre(uint32_t i_plus_k1hi, uint32_t w) {
  uint32_t lo;
  const uint32_t carry = __builtin_uadd_overflow(w, (uint32_t)kK1, &lo) ? 1u : 0u;
  const uint32_t hi = i_plus_k1hi + carry;
  uint64_t z = ((uint64_t)hi << 32) | (uint64_t)(lo ^ hi);
  z *= kK2;
  z ^= z >> 29;
  z *= kK3;
  z ^= z >> 32;
  return z;
}

__device__ __forceinline__ uint64_t digest_mix(uint32_t i, uint32_t w) {
  return digest_mix_pre(i + (uint32_t)(kK1 >> 32), w);
}

// The four words of one 16-byte vector whose first word has index e: pass e + K1.hi.
__device__ __forceinline__ uint64_t digest_mix4_pre(uint32_t e_plus_k1hi, const u32x4 &r) {
  return (digest_mix_pre(e_plus_k1hi, r[0]) + digest_mix_pre(e_plus_k1hi + 1u, r[1])) +
         (digest_mix_pre(e_plus_k1hi + 2u, r[2]) + digest_mix_pre(e_plus_k1hi + 3u, r[3]));
}

// Lane exchange inside a row of 16 lanes through the DPP data path.
template <int CTRL>
__device__ __forceinline__ uint64_t dpp_fetch_u64(uint64_t s) {
  const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)s, CTRL, 0xF, 0xF, true);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(s >> 32), CTRL, 0xF, 0xF, true);
  return ((uint64_t)hi << 32) | lo;
}

// Sum of `s` over each row of 16 lanes (mod 2^64): afterwards every lane holds its row's sum.
__device__ __forceinline__ uint64_t row_sum_u64(uint64_t s) {
  s += dpp_fetch_u64<0xB1>(s);    // quad_perm [1,0,3,2]: lane ^ 1
  s += dpp_fetch_u64<0x4E>(s);    // quad_perm [2,3,0,1]: lane ^ 2   -> every lane holds its quad's sum
  s += dpp_fetch_u64<0x141>(s);   // row_half_mirror: lane i <-> 7-i   -> sum of 8
  s += dpp_fetch_u64<0x140>(s);   // row_mirror:      lane i <-> 15-i  -> sum of the row of 16
  return s;
}

// Sum of `s` over the 64 lanes of the wavefront (mod 2^64); the result is wave-uniform.
__device__ __forceinline__ uint64_t wave_sum_u64(uint64_t s) {
  s = row_sum_u64(s);
  uint64_t total = 0;
#pragma unroll
  for (int row = 0; row < 4; ++row) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)s, row * 16);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(s >> 32), row * 16);
    total += ((uint64_t)hi << 32) | lo;
  }
  return total;
}

// The same value summed over the four rows: every lane ends with the sum of lanes l, l^16, l^32 and l^48.
// v_permlane16_swap exchanges the odd rows of its first operand with the even rows of its second, so with both
// operands equal to r the two results are {row0, row0, row2, row2} and {row1, row1, row3, row3};
// v_permlane32_swap does the same with the two halves of the wavefront.
__device__ __forceinline__ uint64_t rows_sum_u64(uint64_t r) {
  uint32_t lo = (uint32_t)r, hi = (uint32_t)(r >> 32);
  auto pl = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
  auto ph = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
  const uint64_t s = (((uint64_t)ph[0] << 32) | pl[0]) + (((uint64_t)ph[1] << 32) | pl[1]);
  lo = (uint32_t)s;
  hi = (uint32_t)(s >> 32);
  pl = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
  ph = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
  return (((uint64_t)ph[0] << 32) | pl[0]) + (((uint64_t)ph[1] << 32) | pl[1]);
}

// Three sums over the wavefront at once (mod 2^64): afterwards lane l holds the sum of a if l % 4 == 0, of b if
// l % 4 == 1, of c otherwise.  Summing each value on its own takes 3 x 4 exchanges inside the rows; here the first
// two exchanges also halve the number of live values (a lane keeps one value and sends the other one to its
// partner, which keeps that one), so the remaining exchanges move a single register: 7 exchanges instead of 12,
// and one pass over the rows instead of three.
__device__ __forceinline__ uint64_t wave_sum3_u64(uint64_t a, uint64_t b, uint64_t c) {
  const uint32_t lane = threadIdx.x & 63u;
  const bool odd = (lane & 1u) != 0, upper = (lane & 2u) != 0;
  const uint64_t ab = (odd ? b : a) + dpp_fetch_u64<0xB1>(odd ? a : b);   // lane ^ 1: even lanes a, odd lanes b
  const uint64_t cc = c + dpp_fetch_u64<0xB1>(c);
  uint64_t r = (upper ? cc : ab) + dpp_fetch_u64<0x4E>(upper ? ab : cc);  // lane ^ 2: a, b, c, c within each quad
  r += dpp_fetch_u64<0x124>(r);                                           // row_ror:4  (keeps lane % 4)
  r += dpp_fetch_u64<0x128>(r);                                           // row_ror:8  -> sums over the row
  return rows_sum_u64(r);
}

__global__ void __launch_bounds__(kThreads) fill_u64_kernel(uint64_t *p, uint64_t n, uint64_t value) {
  for (uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += (uint64_t)gridDim.x * kThreads)
    p[i] = value;
}

// One workgroup per chunk (the grid equals the chunk count; the loop only covers a capped grid).
// Chunk numbering inside a buffer: a full shard spans cps = ceil(S / chunk_elems) chunk numbers,
// chunk = shard * cps + k covers words [shard*S + k*CE, ...) of the buffer, i.e. shard-relative
// indices [k*CE, min(k*CE + CE, shard length)).  S = shard_elems, or numel when shard_elems = 0.
// The chunk's sum goes to partial[ci] if `partial` is given (digest_reduce_kernel then adds the
// chunks of each shard; atomic adds of hundreds of chunks into one output serialise and cost a
// mid-size buffer most of its time), else straight to out[shard]: the host passes no `partial`
// only when every shard is a single chunk.
__global__ void __launch_bounds__(kThreads)
digest_kernel(const DigestDesc *__restrict__ descs, const ChunkRef *__restrict__ chunks, uint32_t n_chunks,
              uint32_t chunk_elems, uint64_t shard_elems, uint64_t *__restrict__ partial, uint64_t *__restrict__ out) {
  constexpr bool NT = SWIFT_NT != 0;
  __shared__ uint64_t wave_part[kThreads / 64];
  const uint32_t tid = threadIdx.x;
  for (uint32_t ci = blockIdx.x; ci < n_chunks; ci += gridDim.x) {
    const ChunkRef ch = chunks[ci];
    const DigestDesc d = descs[ch.tensor];
    const uint64_t S = shard_elems ? shard_elems : (uint64_t)d.numel;
    const uint32_t cps = (uint32_t)((S + chunk_elems - 1) / chunk_elems);
    const uint32_t shard = ch.chunk / cps;
    const uint32_t k = ch.chunk - shard * cps;
    const uint64_t shard_off = (uint64_t)shard * S;
    const uint64_t rest = (uint64_t)d.numel - shard_off;
    const uint64_t shard_len = rest < S ? rest : S;
    const uint32_t idx0 = k * chunk_elems;                       // shard-relative index of the chunk's first word
    const uint64_t left = shard_len - idx0;
    const uint32_t len = left < chunk_elems ? (uint32_t)left : chunk_elems;
    const uint32_t *__restrict__ p = d.w + shard_off + idx0;

    // head: words before the first 16-byte boundary; body: 16-byte vectors; tail: the rest
    uint32_t head = (uint32_t)(((16u - (uint32_t)((uintptr_t)p & 15u)) & 15u) >> 2);
    if (head > len) head = len;
    const uint32_t n4 = (len - head) >> 2;
    const uint32_t tail0 = head + (n4 << 2);
    const u32x4 *__restrict__ p4 = reinterpret_cast<const u32x4 *>(p + head);
    const uint32_t ib = idx0 + head;                             // shard-relative index of the body's first word

    uint64_t acc = 0;
    if (tid < head) acc += digest_mix(idx0 + tid, ld<false>(p + tid));
    // One 16-byte load per lane and round, mixed as soon as it arrives.  The kernel is bound by
    // instruction issue (about 16 vector instructions per word, at a shader clock the chip lowers
    // under this load), not by load latency: issuing the next round's load ahead of the mixing
    // (software pipelining) and several loads per lane were measured and are slower.
    uint32_t ek = ib + (tid << 2) + (uint32_t)(kK1 >> 32);       // index of this lane's next vector, + K1.hi
    uint32_t i = 0;
    for (; i + kThreads <= n4; i += kThreads, ek += kThreads * 4u) acc += digest_mix4_pre(ek, ld<NT>(p4 + i + tid));   // full rounds: no predicate
    if (i + tid < n4) acc += digest_mix4_pre(ek, ld<NT>(p4 + i + tid));
    if (tail0 + tid < len) acc += digest_mix(idx0 + tail0 + tid, ld<false>(p + tail0 + tid));

    const uint64_t wsum = wave_sum_u64(acc);
    if ((tid & 63u) == 0) wave_part[tid >> 6] = wsum;
    __syncthreads();
    if (tid == 0) {
      uint64_t t = 0;
#pragma unroll
      for (int wv = 0; wv < kThreads / 64; ++wv) t += wave_part[wv];
      if (partial) partial[ci] = t;
      else out[d.first_out + shard] = t;
    }
    __syncthreads();                                             // wave_part is reused by the next chunk
  }
}

// Where the chunk sums of one output (one shard) sit in the partial array: consecutive entries.
struct DigestSpan {
  uint64_t first;
  uint64_t count;            // 0: an empty buffer digested as one shard; its digest is 0
};

// out[o] = sum of the chunk sums of output o.  WG = false: one wavefront per output (many outputs of a few
// chunks each); WG = true: one workgroup per output (few outputs of hundreds of chunks: the loads of one
// wavefront alone would be a chain of memory latencies).  Four loads are in flight per lane.
template <bool WG>
__global__ void __launch_bounds__(kThreads)
digest_reduce_kernel(const DigestSpan *__restrict__ spans, const uint64_t *__restrict__ partial, uint64_t n_out,
                     uint64_t *__restrict__ out) {
  constexpr uint32_t L = WG ? kThreads : 64;
  const uint64_t o = WG ? (uint64_t)blockIdx.x : (uint64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  if (o >= n_out) return;                                        // whole wavefronts leave together; never taken if WG
  const DigestSpan sp = spans[o];
  const uint64_t *p = partial + sp.first;
  uint64_t a0 = 0, a1 = 0, a2 = 0, a3 = 0;
  uint64_t k = WG ? threadIdx.x : (threadIdx.x & 63u);
  for (; k + 3 * L < sp.count; k += 4 * L) {
    a0 += p[k];
    a1 += p[k + L];
    a2 += p[k + 2 * L];
    a3 += p[k + 3 * L];
  }
  for (; k < sp.count; k += L) a0 += p[k];
  const uint64_t wsum = wave_sum_u64((a0 + a1) + (a2 + a3));
  if constexpr (WG) {
    __shared__ uint64_t wave_part[kThreads / 64];
    if ((threadIdx.x & 63u) == 0) wave_part[threadIdx.x >> 6] = wsum;
    __syncthreads();
    if (threadIdx.x == 0) {
      uint64_t t = 0;
      for (int wv = 0; wv < kThreads / 64; ++wv) t += wave_part[wv];
      out[o] = t;
    }
  } else {
    if ((threadIdx.x & 63u) == 0) out[o] = wsum;
  }
}

// mask[i] = 1 if tensor i's digest differs in any of the n_groups group-major digest rows.
__global__ void __launch_bounds__(kThreads)
mask_from_digests_kernel(uint32_t n_tensors, uint32_t n_groups, const uint64_t *__restrict__ before,
                         const uint64_t *__restrict__ after, uint8_t *__restrict__ mask) {
  for (uint32_t i = blockIdx.x * kThreads + threadIdx.x; i < n_tensors; i += gridDim.x * kThreads) {
    uint8_t changed = 0;
    for (uint32_t gI = 0; gI < n_groups; ++gI) {
      const uint64_t j = (uint64_t)gI * n_tensors + i;
      changed |= (before[j] != after[j]) ? 1 : 0;
    }
    mask[i] = changed;
  }
}

// Where a tensor's chunks sit in the optimizer chunk table.
struct TensorChunks {
  uint32_t first, count;
};

// Packs an optimizer chunk table by a device-resident mask (one byte per tensor, nonzero = marked),
// so that a launch over the packed table touches marked tensors only without the host ever seeing
// the mask.  One workgroup per tensor.  With A = chunks of marked tensors before this one, I =
// chunks of unmarked tensors before it and T = chunks of all marked tensors, a marked tensor's
// entries are copied to packed[A ...) (list order is kept) and an unmarked tensor writes empty
// entries to packed[T + I ...): every entry of `packed` is written, so nothing of an earlier call
// survives.  *n_slots_out = T << tpc_shift, the number of tile slots the packed table holds.  The
// kernel also clears the n_counters (at most kThreads) tile counters that opt_queue_kernel draws from.
__global__ void __launch_bounds__(kThreads)
compact_chunks_kernel(const ChunkDesc *__restrict__ chunks, const TensorChunks *__restrict__ spans, uint32_t n_tensors,
                      const uint8_t *__restrict__ mask, uint32_t tpc_shift, ChunkDesc *__restrict__ packed,
                      uint64_t *__restrict__ n_slots_out, unsigned int *__restrict__ counters, uint32_t n_counters) {
  __shared__ uint64_t part[3][kThreads / 64];
  const uint32_t t = blockIdx.x, tid = threadIdx.x;
  uint64_t marked_before = 0, unmarked_before = 0, marked_total = 0;
  for (uint32_t j = tid; j < n_tensors; j += kThreads) {
    const uint64_t cnt = spans[j].count;
    if (mask[j] != 0) {
      marked_total += cnt;
      if (j < t) marked_before += cnt;
    } else if (j < t) {
      unmarked_before += cnt;
    }
  }
  const uint64_t s0 = wave_sum_u64(marked_before), s1 = wave_sum_u64(unmarked_before), s2 = wave_sum_u64(marked_total);
  if ((tid & 63u) == 0) {
    part[0][tid >> 6] = s0;
    part[1][tid >> 6] = s1;
    part[2][tid >> 6] = s2;
  }
  __syncthreads();
  uint64_t sum[3] = {0, 0, 0};
#pragma unroll
  for (int k = 0; k < 3; ++k)
#pragma unroll
    for (int wv = 0; wv < kThreads / 64; ++wv) sum[k] += part[k][wv];
  const bool marked = mask[t] != 0;
  const TensorChunks sp = spans[t];
  const uint64_t dst = marked ? sum[0] : sum[2] + sum[1];
  ChunkDesc empty;
  empty.x = nullptr; empty.g = nullptr; empty.m = nullptr; empty.v = nullptr; empty.xb = nullptr;
  empty.len = 0; empty.tensor = t; empty.vec_ok = 0; empty.elem0 = 0; empty.pad = 0;
  for (uint32_t k = tid; k < sp.count; k += kThreads) packed[dst + k] = marked ? chunks[sp.first + k] : empty;
  if (t == 0 && tid == 0) *n_slots_out = sum[2] << tpc_shift;
  if (t == 0 && tid < n_counters) counters[tid * 32u] = 0;       // the tile counters of opt_queue_kernel, 128 bytes apart
}

}  // namespace swift
