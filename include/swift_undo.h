/*
 * swift_undo.h -- C ABI of the update-undo library for one MI355X (gfx950).
 *
 * The library implements the data-parallel hot path of Swift's replication-based recovery
 * (arXiv 2302.06173, section "Update-undo"): a fused optimizer step over a list of tensors, the
 * closed-form elementwise inverse of that step, which rolls the parameters and the optimizer
 * moments of a replica back from iteration t+1 to iteration t using the cached gradient g_t, and a
 * 64-bit digest of raw state bits that tells which tensors already hold the stepped state.
 *
 * General rules
 *   - Plain C types only.  Every pointer is marked HOST or DEVICE below.  DEVICE pointers must
 *     be ordinary device allocations of the GPU that is current (hipSetDevice) during the call.
 *   - The caller owns every buffer it passes.  The library allocates only internal tables (tensor
 *     descriptors and chunk lists, 64 bytes per 16 Ki or 64 Ki elements, plus the per-list scratch the
 *     LAMB, fused-digest and device-mask calls describe), cached per distinct tensor list -- distinct
 *     meaning: same pointers, sizes, gradient type and host mask.  The first call on a list builds its
 *     tables (an allocation and synchronous copies: about 2 ms for a few hundred tensors); later calls
 *     find them.  Tables are NEVER freed as a side effect of another call: only swift_cache_trim (the
 *     caller decides when) and swift_shutdown free them.  swift_cache_stats tells how much is held.
 *   - HIP graphs: a call on a list whose tables exist consists of kernel launches only and may be
 *     captured.  A call that would have to build tables (a list, or a kind of call on it, that has not
 *     been made before) while its stream is capturing returns SWIFT_EINVAL: make the same call once
 *     before the capture.  A captured graph holds pointers into the tables it was recorded with; such
 *     tables survive swift_cache_trim, and swift_shutdown must not be called while a graph that was
 *     captured over library calls may still be replayed.
 *   - Pointer checks (device memory of the current GPU, numel elements inside one allocation, no
 *     overlap) are made in full when a list's tables are built.  Later calls on the same list look up
 *     its first buffer again and rebuild the tables if the allocation behind it has changed; a caller
 *     that frees tensors and allocates others at the same addresses gets no further checking.
 *   - HOST arrays (pointer arrays, numel, masks, hyper-parameters) are read during the call only.
 *   - Work is enqueued on `hip_stream` (a hipStream_t; NULL = the default stream) and the call
 *     returns without waiting for it.  Order with respect to other work -- including update
 *     kernels that were launched before a failure was noticed and must still run to completion
 *     (paper, Implementation, "Update-undo") -- is stream order.
 *   - Every entry point returns SWIFT_OK (0) or a negative swift_status and swift_last_error()
 *     describes the problem.  No exceptions, no aborts.  SWIFT_EINVAL and SWIFT_ENOTINVERTIBLE are
 *     reported before anything is enqueued.  SWIFT_EHIP from a kernel launch can leave earlier
 *     launches of the same call on the stream (the LAMB step, the fused-digest and the device-mask
 *     calls are two or three launches): the state is then undefined, as after any failed launch.
 *   - theta, m and v are IEEE binary32; gradients are binary32 or bfloat16.  Arithmetic inside
 *     the kernels is binary64 with one rounding to binary32 at each store.  NaN/Inf propagate;
 *     denormals are kept; nothing is clamped.
 *   - No two tensors of a list may overlap, and no other work may touch them while a call's
 *     kernels run.
 */
#ifndef SWIFT_UNDO_H
#define SWIFT_UNDO_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SWIFT_OK = 0,
  SWIFT_EINVAL = -1,         /* bad argument: null pointer, negative count, step < 1, unknown kind or
                                dtype, non-finite or out-of-range hyper-parameter, missing v array,
                                pointer that is not device memory of the current GPU or whose
                                allocation is shorter than numel elements, misaligned pointer */
  SWIFT_ENOTINVERTIBLE = -2, /* undo only: the inverse divides by zero (beta1 = 0, beta2 = 0, or
                                eta*lambda = 1 for AdamW and plain SGD) */
  SWIFT_EHIP = -3            /* a HIP runtime call failed (the message carries its error name), or the
                                library could not get host memory; no C++ exception leaves the library */
} swift_status;

typedef enum {
  SWIFT_SGDM = 0,  /* Alg. 1 / Alg. 2: SGD with momentum mu, dampening tau, coupled decay lambda.
                      mu = 0 is App. A's plain SGD with the damped gradient left in the m buffer. */
  SWIFT_ADAM = 1,  /* App. A "Adam" / "Undo Adam": decay coupled into the gradient, g' = g + lambda x */
  SWIFT_ADAMW = 2, /* App. A "AdamW" / "Undo AdamW": decoupled decay, alpha = 1 */
  SWIFT_LAMB = 3,  /* LAMB with saved norms ("Update-undo" section, Table 1); swift_lamb_* entry points only */
  SWIFT_SGD = 4    /* App. A "SGD" / "Undo SGD": no optimizer state, theta and the gradient only (12 bytes per
                      parameter); the undo solves the update line for x_t instead of reading a buffer */
} swift_opt_kind;

typedef enum { SWIFT_F32 = 0, SWIFT_BF16 = 1 } swift_dtype; /* gradients only */

/* Bits of swift_hparams.flags. */
typedef enum {
  SWIFT_CLAMP_V = 1 /* undo of Adam, AdamW and LAMB: a recovered second moment below zero is stored as
                       +0.  "Undo Adam" (App. A) solves v_t = beta2 v_{t-1} + (1-beta2) g'^2 for
                       v_{t-1}; since the step rounded v_t, the solution can come out slightly
                       negative where v_{t-1} was almost zero, and a caller that does anything with
                       v but re-apply step t with the same gradient would take the root of a negative
                       number.  The paper applies no clamp, so this is off by default; the test
                       v < 0 is made on the binary64 value, NaN stays NaN. */
} swift_flags;

/* Hyper-parameters in the paper's notation (Alg. 1, Alg. 2, App. A).  `step` is the t of m_t and
 * of the bias corrections 1 - beta^t; a step and the undo of that step use the same value. */
typedef struct {
  int32_t kind;         /* swift_opt_kind */
  int32_t grad_dtype;   /* swift_dtype */
  int64_t step;         /* t >= 1 */
  double lr;            /* eta_t, finite */
  double weight_decay;  /* lambda >= 0 */
  double momentum;      /* mu in [0, 1]   (SGDM) */
  double dampening;     /* tau in [0, 1]  (SGDM) */
  double beta1, beta2;  /* in [0, 1)      (Adam, AdamW) */
  double eps;           /* >= 0           (Adam, AdamW) */
  int32_t flags;        /* swift_flags, 0 for the paper's algorithms as printed */
  int32_t reserved;     /* must be 0 */
} swift_hparams;

/* A list of n tensors (0 <= n < 2^24).  All arrays are HOST arrays of length n; the pointers they hold are
 * DEVICE pointers to contiguous 1-D storage of numel[i] elements.  param, m, v: binary32,
 * 4-byte aligned, updated in place.  grad: binary32 (4-byte aligned) or bfloat16 (2-byte
 * aligned), NEVER written -- the undo needs it intact (paper, "Update-undo": only the latest
 * gradient is cached, no extra memory).  16-byte alignment of all of a tensor's pointers
 * (8-byte for bfloat16 buffers) selects the 128-bit access path; results are bit-identical either way.
 * v may be NULL for SWIFT_SGDM and SWIFT_SGD, m for SWIFT_SGD (neither is looked at then).  Tensors with
 * numel 0 are allowed and skipped.
 * Placement advice (throughput only, never correctness): on MI355X the kernels run 2-10 % faster when
 * param[i], grad[i], m[i], v[i] of a tensor do NOT all start at the same address modulo 8 KiB, e.g. when
 * consecutive buffers of an arena are an odd multiple of 2 KiB apart; allocators that hand out buffers at
 * 2 MiB granularity produce the slow case.  swift_arena_layout computes such a placement.
 * param_bf16 (nullable array; not from the paper): mixed-precision training keeps a bfloat16 copy of
 * the parameters next to the binary32 master weights.  If the array is given, swift_opt_step and
 * swift_opt_undo (host- and device-mask forms) also write, for every tensor they touch, the bfloat16
 * nearest to each new binary32 parameter (ties to even, NaN -> 0x7FC0) into param_bf16[i] (2-byte
 * aligned, numel[i] elements, write only): 2 more bytes of traffic per parameter instead of a cast pass.
 * So do the LAMB and fused-digest entry points (the digests cover theta, m and v, not the copy). */
typedef struct {
  int64_t n;
  void *const *param;
  const void *const *grad;
  void *const *m;
  void *const *v;
  const int64_t *numel;
  void *const *param_bf16;
} swift_tensor_list;

/* Optimizer step t: (x_t, g_t, m_{t-1}, v_{t-1}) -> (x_{t+1}, m_t, v_t) in place, for every
 * tensor whose mask entry is non-zero (all tensors if the mask is NULL).
 *   SGD   (App. A "SGD"):    x <- x - eta (g + lambda x)
 *   SGDM  (Alg. 1):          g' = g + lambda x;  m <- mu m + (1-tau) g';  x <- x - eta m
 *   Adam  (App. A "Adam"):   g' = g + lambda x;  m <- beta1 m + (1-beta1) g';
 *                            v <- beta2 v + (1-beta2) g'^2;
 *                            x <- x - eta (m/(1-beta1^t)) / (sqrt(v/(1-beta2^t)) + eps)
 *   AdamW (App. A "AdamW"):  moments from the raw g;  x <- x - eta (u + lambda x), u as above.
 * host_mask: HOST, n bytes, nullable. */
int swift_opt_step(const swift_tensor_list *list, const swift_hparams *hp,
                   const uint8_t *host_mask, void *hip_stream);

/* Undo of step t: (x_{t+1}, g_t, m_t, v_t) -> (x_t, m_{t-1}, v_{t-1}) in place, for every tensor
 * marked as updated (mask entry non-zero; all if NULL).  The parameter is recovered first, from
 * the new moments; coupled decay is rebuilt from the recovered parameter.
 *   SGD   (App. A "Undo SGD"):   x <- (x + eta g) / (1 - eta lambda)
 *   SGDM  (Alg. 2):              x <- x + eta m;  m <- (m - (1-tau)(g + lambda x)) / mu
 *                                (mu = 0: the m buffer is left as it is)
 *   Adam  (App. A "Undo Adam"):  x <- x + eta u;  g' = g + lambda x;
 *                                m <- (m - (1-beta1) g')/beta1;  v <- (v - (1-beta2) g'^2)/beta2
 *   AdamW (App. A "Undo AdamW"): x <- (x + eta u)/(1 - eta lambda);  m, v as Adam with raw g.
 * Because the step rounds to binary32, the result equals the pre-step state only up to
 * floating-point error (paper, "Update-undo"); it matches a binary64 evaluation of the same
 * formulas on the same input bits to within binary32 rounding.
 * Returns SWIFT_ENOTINVERTIBLE as described at swift_status. */
int swift_opt_undo(const swift_tensor_list *list, const swift_hparams *hp,
                   const uint8_t *host_mask, void *hip_stream);

/* The same two operations with the "updated" marks in DEVICE memory (n bytes, not nullable, left
 * unchanged), read on the device when the call's kernels run: the mask can be produced by
 * swift_mask_from_digests on the same stream with no host round trip.  A small kernel packs the
 * work list by the mask into scratch memory the library keeps for this tensor list (allocated on
 * the first such call); calls on the same list must not overlap, as for any call that writes the
 * same tensors.  Since the host cannot size the launch to the marked tensors, a fixed number of
 * resident wavefronts draws the marked tiles from counters on the device: the time follows the
 * marked elements whatever the mask's density, at about 6 % less bandwidth than the host-mask
 * calls; prefer those when the host knows the marks. */
int swift_opt_step_dmask(const swift_tensor_list *list, const swift_hparams *hp,
                         const uint8_t *device_mask, void *hip_stream);
int swift_opt_undo_dmask(const swift_tensor_list *list, const swift_hparams *hp,
                         const uint8_t *device_mask, void *hip_stream);

/* swift_opt_undo_dmask for callers that cannot allocate device memory: code under HIP graph capture
 * whose list has no tables yet, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same result bits.  The call makes no allocation and no copy: its chunk table, packed table and
 * counters live in a device array that is part of the library's code object (4.1 MiB per GPU, held
 * from the first use of the library on that GPU until the process ends), and the table is written by
 * kernels from descriptors passed in their arguments, so nothing is cached per list either.  Limits:
 * at most SWIFT_NOALLOC_MAX_TENSORS tensors, and the list must fit SWIFT_NOALLOC_MAX_CHUNKS chunks of
 * at most 4 Mi elements (about 137 G elements in long tensors; every tensor takes at least one chunk);
 * beyond that, and if list->param_bf16 is given, the call returns SWIFT_EINVAL.  All calls on one GPU
 * share the one array: two such calls that overlap in time on a GPU race, whatever their lists and
 * streams; on one stream they are ordered.  The first library call on a GPU performs one-time set-up
 * (code loading, symbol lookup); make it outside a capture.  Pointers are checked in full on every call. */
#define SWIFT_NOALLOC_MAX_TENSORS 4096
#define SWIFT_NOALLOC_MAX_CHUNKS 32768
int swift_opt_undo_dmask_noalloc(const swift_tensor_list *list, const swift_hparams *hp,
                                 const uint8_t *device_mask, void *hip_stream);

/* swift_opt_step / swift_opt_undo that also return the digests of the state they leave behind, at no
 * extra HBM traffic: digests_device[g * n + i] is the digest of tensor i's theta (g = 0), m (g = 1) and
 * v (g = 2; SGDM has g = 0, 1 only, plain SGD g = 0 only), one shard per tensor, identical to what swift_state_digest writes
 * for the buffer order theta_0..theta_{n-1}, m_0.., v_0.. with shard_elems = 0.  A training loop keeps
 * the digests of the last completed iteration this way; after a failure one swift_state_digest pass and
 * swift_mask_from_digests tell which tensors hold stepped bits (the role of the paper's per-parameter
 * "updated" flag, Implementation, "Update-undo").  Entries of unmarked tensors are left alone.  Every
 * tensor must have fewer than 2^32 elements.  digests_device: DEVICE, 3n (2n for SGDM, n for SGD) entries, 8-byte
 * aligned.  The call keeps per-list scratch (24 bytes per 256 elements): calls on one list must not overlap. */
int swift_opt_step_digest(const swift_tensor_list *list, const swift_hparams *hp, const uint8_t *host_mask,
                          uint64_t *digests_device, void *hip_stream);
int swift_opt_undo_digest(const swift_tensor_list *list, const swift_hparams *hp, const uint8_t *host_mask,
                          uint64_t *digests_device, void *hip_stream);

/* LAMB.  The paper (section "Update-undo", Table 1) notes that LAMB adds a sum -- the L2 norms behind
 * its per-tensor trust ratio -- to Adam's invertible elementwise operators, and that saving the norm
 * (a scalar) at step time makes the step invertible; it prints no algorithm.  The step here is the
 * published LAMB update (You et al. 2019) with phi = identity, per tensor of the list:
 *   m, v as AdamW;  r = m^/(sqrt(v^)+eps);  u = r + lambda x;  q = ||x|| / ||u|| (1 if either norm is 0);
 *   x <- x - eta q u
 * swift_lamb_step writes norms_device[2i] = ||x_t||, norms_device[2i+1] = ||u|| (binary64) for every
 * participating tensor i (entries of unmarked tensors are left alone; the sums are formed in a fixed
 * order, so the values are reproducible bit for bit).  swift_lamb_undo takes those saved norms back:
 *   x <- (x + eta q r)/(1 - eta q lambda);  m, v as "Undo AdamW" (App. A).
 * hp->kind must be SWIFT_LAMB; beta1, beta2, eps as for Adam.  norms_device: DEVICE, 2*n doubles, 8-byte
 * aligned.  If 1 - eta q lambda happens to be 0 for a tensor the undo yields Inf/NaN there (q lives on
 * the device, so the host cannot refuse the call).  The step keeps per-list scratch for the partial
 * sums (16 bytes per 256 elements): calls on the same list must not overlap in time. */
int swift_lamb_step(const swift_tensor_list *list, const swift_hparams *hp, const uint8_t *host_mask,
                    double *norms_device, void *hip_stream);
int swift_lamb_undo(const swift_tensor_list *list, const swift_hparams *hp, const uint8_t *host_mask,
                    const double *norms_device, void *hip_stream);

/* 64-bit digests of raw 32-bit words.  This stands in for the paper's per-parameter "marked as
 * updated" flag (Implementation, "Update-undo"): a shard whose digest differs from the digest
 * recorded at iteration t holds stepped bits.  For a shard of words w_0..w_{k-1} (k < 2^32), with
 * i the index inside the shard and all arithmetic modulo 2^64:
 *   z = (i << 32) | w_i;  z += K1;  z ^= z >> 32;  z *= K2;  z ^= z >> 29;  z *= K3;  z ^= z >> 32
 *   digest = sum_i z                       (empty shard: 0)
 *   K1 = 0x9E3779B97F4A7C15, K2 = 0x6A09E667F3BCC909, K3 = 0xBB67AE8584CAA73B
 * buf: HOST array of n_buf DEVICE pointers to 4-byte elements (4-byte aligned); numel: HOST.
 * shard_elems = 0: one shard per buffer (numel < 2^32 required); otherwise 0 < shard_elems < 2^32
 * and a buffer is cut into consecutive shards of that many words, the last one short.
 * out_device: DEVICE, swift_digest_count(...) entries, buffer-major; fully overwritten.
 * Shards longer than the kernel's chunk (4 Ki to 64 Ki words, by total size) are summed in two launches
 * through per-list scratch (8 bytes per chunk): calls on the same buffer list must not overlap in time. */
int swift_state_digest(int64_t n_buf, const void *const *buf, const int64_t *numel,
                       int64_t shard_elems, uint64_t *out_device, void *hip_stream);

/* Number of digests swift_state_digest writes: sum_i ceil(numel_i / shard_elems), or n_buf when
 * shard_elems = 0.  Pure host arithmetic.  Returns a negative swift_status on bad arguments. */
int64_t swift_digest_count(int64_t n_buf, const int64_t *numel, int64_t shard_elems);

/* Selective undo: derive the per-tensor "updated" marks from two digest arrays.  Both arrays are
 * DEVICE arrays of n_groups * n_tensors digests laid out group-major (e.g. the per-tensor digests
 * of all theta, then all m, then all v, as swift_state_digest writes them for that buffer order
 * with shard_elems = 0).  mask_device[i] = 1 if any group's digest of tensor i differs, else 0.
 * mask_device: DEVICE, n_tensors bytes, fully overwritten. */
int swift_mask_from_digests(int64_t n_tensors, int64_t n_groups, const uint64_t *before_device,
                            const uint64_t *after_device, uint8_t *mask_device, void *hip_stream);

/* Update tracker: the paper's own bookkeeping (Implementation, "Update-undo").  In data-parallel
 * training the update of a tensor is launched as soon as its gradient is final (after that tensor's
 * all-reduce), and the tensor is then marked as updated; after a failure the survivors let the kernels
 * already launched finish and undo exactly the marked tensors.  The tracker is host state (the marks and the
 * streams that carried this iteration's launches); ids refer to the positions of the tensors in the caller's
 * full list.  A stream given to swift_tracker_step must stay alive until the iteration's swift_tracker_undo or
 * swift_tracker_marks has returned or the next swift_tracker_begin.
 *   swift_tracker_create   n_tensors >= 0; *out receives the handle (HOST, owned by the library).
 *   swift_tracker_begin    starts iteration `step` (>= 1) and drops the marks of the previous one.
 *   swift_tracker_step     `group` is a sub-list of the full list, tensor_ids[k] (HOST, group->n entries)
 *                          the position of group tensor k in the full list.  If grad_ready_event (a
 *                          hipEvent_t, nullable) is given, the stream waits for it first; then
 *                          swift_opt_step(group, hp, NULL, stream) is enqueued and the ids are marked.
 *                          hp->step must equal the iteration in progress; an id already marked in this
 *                          iteration is an error (SWIFT_EINVAL) and nothing is enqueued.
 *   swift_tracker_marks    waits (on the host) until the streams that carried this iteration's tracked
 *                          launches have drained, then copies the marks (HOST, n_tensors bytes, 1 = updated).
 *   swift_tracker_undo     enqueues swift_opt_undo(list, hp, marks, stream) on the FULL list (list->n must
 *                          equal n_tensors) behind every tracked launch of the iteration: by stream order
 *                          where they share `stream`, else through an event that `stream` waits for on the
 *                          device.  The host does not wait.  The marks are cleared: once the stream has run,
 *                          the replica is back at the start of the iteration.
 *   swift_tracker_destroy  frees the handle (NULL is allowed); launches in flight are not affected.
 * One tracker serves one GPU and one training loop; its calls are serialised by an internal lock. */
typedef struct swift_tracker swift_tracker;
int swift_tracker_create(int64_t n_tensors, swift_tracker **out);
int swift_tracker_begin(swift_tracker *tracker, int64_t step);
int swift_tracker_step(swift_tracker *tracker, const swift_tensor_list *group, const int64_t *tensor_ids,
                       const swift_hparams *hp, void *grad_ready_event, void *hip_stream);
int swift_tracker_marks(swift_tracker *tracker, uint8_t *host_mask_out);
int swift_tracker_undo(swift_tracker *tracker, const swift_tensor_list *list, const swift_hparams *hp,
                       void *hip_stream);
int swift_tracker_destroy(swift_tracker *tracker);

/* Measurement aid: a plain device-to-device copy of `bytes` bytes (a multiple of 16; both pointers
 * 16-byte aligned, DEVICE) written with the same access pattern as the optimizer kernels.  It
 * gives the practical HBM ceiling of this access pattern and calibrates profiler byte counters. */
int swift_stream_copy(void *dst_device, const void *src_device, int64_t bytes, void *hip_stream);

/* Machine grouping for selective logging (paper, section "Selective Logging"); host arithmetic only,
 * no GPU call.  N machines host consecutive pipeline stages; logging keeps the messages between
 * groups of machines, and a failure rolls back the failed machine's whole group.  Starting from one
 * group per machine, the adjacent pair with the smallest dR/dM is merged while the logging data of one
 * checkpoint interval, T * (bytes on the links between groups), exceeds storage_limit, with
 *   R(G_i,G_{i+1}) = R(G_i) + R(G_{i+1}) + M(G_i,G_{i+1})/B,   dM = M(G_i,G_{i+1}) T,
 *   dR = R(G_i,G_{i+1})(|G_i|+|G_{i+1}|)/N - R(G_i)|G_i|/N - R(G_{i+1})|G_{i+1}|/N,
 * and, if parallel_recovery is non-zero, every R(G) in dR divided by floor(N/|G|).  Ties go to the
 * pair with the lowest index; a link with M = 0 is merged only when no other is left.
 * compute_time: HOST, n_machines entries, R of each machine (finite, >= 0).  message_bytes: HOST,
 * n_machines - 1 entries, M between machine i and i+1 (finite, >= 0; may be NULL for one machine).
 * checkpoint_interval: T > 0 iterations.  bandwidth: B > 0 bytes per time unit of R (infinity allowed).
 * group_of: HOST, n_machines entries out: group index of each machine, groups numbered from 0 in
 * pipeline order.  storage_out / recovery_out (nullable): T * bytes on the remaining inter-group links,
 * and the expected recovery time sum_G R(G)|G|/N of the result.  O(n_machines log n_machines) time: the result is
 * that of the paper's loop, found with a priority queue instead of a scan per merge. */
int swift_logging_groups(int64_t n_machines, const double *compute_time, const double *message_bytes,
                         double checkpoint_interval, double bandwidth, double storage_limit, int parallel_recovery,
                         int32_t *group_of, double *storage_out, double *recovery_out);

/* Placement helper, host arithmetic only: byte offsets for the state of n tensors inside ONE device allocation
 * (the caller allocates total_bytes, 256-byte aligned, and carves the buffers out of it), laid out so that the
 * kernels reach their best bandwidth.  offsets[i * S + k] is the offset of stream k of tensor i, with S = 4
 * streams (theta, gradient, m, v) if with_v is positive, 3 (theta, gradient, m) if it is 0, 2 (theta, gradient:
 * plain SGD) if it is negative; the buffers of a
 * tensor are adjacent, tensor after tensor.  A buffer of 1 MiB or more occupies its size rounded up to 8 KiB plus
 * 2 KiB, so that consecutive buffers start an odd multiple of 2 KiB apart and theta, g, m, v of a tensor begin in
 * four different quarters of an 8 KiB window; smaller buffers are rounded up to 256 bytes.  Why: a tile of the
 * update kernels reads the same offset of all four buffers at once, and when these start at the same address
 * modulo 8 KiB (what an allocator with 2 MiB granularity produces) MI355X serves them 2-10 % slower.  Every
 * offset is a multiple of 256.  numel, offsets: HOST (offsets: n * S entries); total_bytes: HOST, nullable. */
int swift_arena_layout(int64_t n, const int64_t *numel, int32_t grad_dtype, int32_t with_v, int64_t *offsets,
                       int64_t *total_bytes);

/* What the library holds: number of cached lists and bytes of device memory behind them (either
 * pointer may be NULL).  HOST. */
int swift_cache_stats(int64_t *n_lists, int64_t *device_bytes);

/* Frees cached tables, least recently used first, until at most max_device_bytes remain (0: all that
 * can go).  Tables that a captured graph may use are kept.  Freeing synchronises the device.  The
 * only call besides swift_shutdown that frees tables: a training loop whose lists keep changing
 * (fresh host masks, re-allocated tensors) calls it when it sees fit. */
int swift_cache_trim(int64_t max_device_bytes);

/* Frees every cached table on every device (synchronises those devices first), including tables that
 * captured graphs use: do not replay such graphs afterwards. */
int swift_shutdown(void);

/* Message of the last error on the calling thread ("" if none).  HOST, owned by the library. */
const char *swift_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SWIFT_UNDO_H */
