/*
 * tt_emb.h - C ABI of the MI355X (gfx950) tensor-train embedding library.
 *
 * The library implements the minibatch hot path of TT-compressed node embeddings:
 *   forward          ids -> rows of the table W, W[i,:] = G1[i1] G2[i2] G3[i3]
 *                    (paper: Section 3, Eq. "tt-embedding" and the paragraph after it that
 *                    evaluates a row by d-1 = 2 matrix products over unfolded core slices;
 *                    Section 4.2 for the split i1 = i/(n2 n3), i2 = (i/n3) mod n2, i3 = i mod n3)
 *   backward_update  dL/drows -> gradients of the three cores, summed over the batch, followed by
 *                    the parameter update on the device (paper: Section 5, the "bwd" and "upd"
 *                    phases of the timing breakdown; the paper prints no formula and names no
 *                    optimiser, so this is the chain rule through the two products and plain SGD)
 *
 * Naming.  The table has N = n1*n2*n3 rows (paper: M = m1 m2 m3) of D = d1*d2*d3 floats
 * (paper: N = n1 n2 n3); the TT ranks are (1, r1, r2, 1) (paper: R_0..R_3 with R_0 = R_3 = 1).
 *
 * Core storage (defined by this library).  fp32, each slice contiguous and stored as the
 * unfolding matrix that the row construction multiplies:
 *   g1[n1][d1][r1]        G1[i1] is d1 x r1            paper G_1(0, i1, j1, a)
 *   g2[n2][r1][d2][r2]    G2[i2] is r1 x (d2*r2)       paper G_2(a, i2, j2, b)
 *   g3[n3][r2][d3]        G3[i3] is r2 x d3            paper G_3(b, i3, j3, 0)
 * Output column order is j = (j1*d2 + j2)*d3 + j3 (Eq. "tt-embedding").
 *
 * Memory.  Every pointer named "device" is HIP device memory owned by the caller; the library
 * borrows it and never allocates or frees device memory.  Cores must be 16-byte aligned, ids
 * 8-byte aligned, out and grad_out 16-byte aligned for the shapes that run on the matrix-core
 * kernels (see TT_EMB_FLAG_GENERIC_KERNELS) and 4-byte aligned otherwise (TT_EMB_EINVAL if not).
 * The handle owns host bookkeeping only.
 * All calls are asynchronous on the given HIP stream unless stated otherwise (tt_emb_prepare also
 * uses two internal streams of default priority, created on its first call).  A handle must not
 * be used from two threads or two streams at once.
 *
 * Graph capture.  forward, forward_eval, materialize and backward_update only enqueue kernels on
 * hip_stream and may be captured into a HIP graph, as long as the handle has never been given to
 * tt_emb_prepare: a handle that has orders its index sets through events on streams of its own,
 * which a capture cannot contain, so every call on it (tt_emb_prepare included) returns
 * TT_EMB_ESTATE while hip_stream is being captured.  Use a second handle for captured steps.
 *
 * Errors.  Every function returns TT_EMB_OK (0) or a negative code and never aborts.
 */
#ifndef TT_EMB_H
#define TT_EMB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tt_emb* tt_emb_t; /* opaque handle */

enum {
  TT_EMB_OK = 0,
  TT_EMB_EINVAL = -1,    /* null pointer, non-positive factor, unsupported size, B < 0          */
  TT_EMB_ENOSPC = -2,    /* B > max_batch, or the workspace is smaller than workspace_bytes()   */
  TT_EMB_ESTATE = -3,    /* backward_update without a pending forward; a call that the handle's
                            state does not allow (see the functions)                            */
  TT_EMB_EHIP = -4,      /* a HIP call failed; tt_emb_strerror(code) carries HIP's message      */
  TT_EMB_ERANGE = -5,    /* get_stats only: some id of the last batch was outside [0, N)        */
  TT_EMB_EINTERNAL = -6  /* get_stats only: a kernel met an index it could not have produced    */
};

enum {
  TT_EMB_FLAG_CHECK_RANGE = 1u,    /* get_stats returns TT_EMB_ERANGE when an id was out of range */
  TT_EMB_FLAG_IDS_READY = 4u,      /* the ids given to tt_emb_prepare are complete in device memory
                                      when the call is made: the library then need not order its
                                      index stream after what hip_stream holds, only after its own
                                      earlier use of the index set (a pipeline can start a step
                                      earlier, and the caller's stream carries one event less)  */
  TT_EMB_FLAG_GENERIC_KERNELS = 2u /* use the any-shape vector-ALU kernels even for shapes that
                                      have matrix-core kernels (d1 in {4,8,...,32}, d2 = 4,
                                      r1 = r2 in {8,16,32,64,128}, d3 in {4,8}); for comparison and
                                      testing                                                    */
};

typedef struct {
  int64_t n[3];      /* node factors n1,n2,n3 (paper m_k); N = n1*n2*n3 must be below 2^31;
                        n2 and n3 at most 2048                                                  */
  int32_t d[3];      /* embedding-dimension factors d1,d2,d3 (paper n_k); D = d1*d2*d3 <= 4096.
                        d1 = 8, 12, ... 32 with d2 = 4, d3 in {4,8}, r1 = r2 in {8,...,128} also
                        runs on the matrix-core kernels: G1[i1] is treated as d1/4 slabs of
                        4 x r1 (a table with d1/4 times the first-core slices and quarter-height
                        rows over the same memory); this needs (d1/4)*N < 2^31 and
                        (d1/4)*max_batch < 2^30, enlarges the workspace accordingly and is
                        invisible at this interface                                             */
  int32_t r[2];      /* inner TT ranks r1, r2 (paper R_1, R_2)                                  */
  int64_t max_batch; /* upper bound on B, sizes the workspace; 1 <= max_batch < 2^30            */
  int32_t device;    /* HIP device ordinal the buffers live on                                  */
  uint32_t flags;    /* TT_EMB_FLAG_*                                                           */
} tt_emb_config;

/* Bytes of device workspace that tt_emb_create needs for this configuration (Section 3: the
 * factorisations and ranks of cfg fix the sizes of the cores and of every intermediate). */
int tt_emb_workspace_bytes(const tt_emb_config* cfg, size_t* bytes);

/*
 * Creates a handle for the table that three TT cores define (Section 3, Eq. "tt-matrix": a matrix
 * with N = n1*n2*n3 rows and D = d1*d2*d3 columns held as cores of ranks (1, r1, r2, 1); cfg gives
 * the two factorisations and the ranks) over caller-owned cores (device, layout above, updated in
 * place by backward_update) and a caller-owned workspace (device, at least workspace_bytes(),
 * 256-byte aligned).  Both must stay alive until tt_emb_destroy.  Host-only: enqueues nothing.
 * Returns TT_EMB_EINVAL for a null pointer, a misaligned buffer or a configuration outside the
 * limits stated at tt_emb_config, TT_EMB_ENOSPC when workspace_bytes is too small.
 */
int tt_emb_create(tt_emb_t* out, const tt_emb_config* cfg, float* g1, float* g2, float* g3,
                  void* workspace, size_t workspace_bytes);

/*
 * Forward (Section 3, Eq. "tt-embedding"; Section 4.2).  ids: device int64[B]; out: device
 * fp32[B][D], row-major.  Row b receives the embedding of ids[b]; repeated ids give repeated rows;
 * an id outside [0, N) gives a zero row and takes no part in the backward pass.  0 <= B <=
 * max_batch; B = 0 is a no-op.  The index structures and prefix products G1[i1] G2[i2] of this
 * batch are kept in the workspace for the next backward_update; ids may be released once the
 * stream has passed this call.  hip_stream is a hipStream_t (0 = the null stream).
 */
int tt_emb_forward(tt_emb_t h, const int64_t* ids, int64_t B, float* out, void* hip_stream);

/*
 * Lookup only (evaluation, inference): as tt_emb_forward, but the batch does not stay pending, so no
 * backward_update can follow it.  Returns TT_EMB_ESTATE while a forward is pending (its cached
 * products share the workspace).
 */
int tt_emb_forward_eval(tt_emb_t h, const int64_t* ids, int64_t B, float* out, void* hip_stream);

/*
 * Lookup for callers that cannot allocate device memory or keep a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Computes what tt_emb_forward_eval
 * computes (same kernels, bit-identical rows) without a handle and without a caller workspace: the
 * index structures and prefix products of the batch go to a 64 MiB device array that is part of
 * the library's code object (every GPU the library runs on holds its own copy until the process
 * ends).  Nothing is allocated or freed, on the device or through any library, by this call.
 *   cfg      shape, ranks and flags as for tt_emb_create (no re-indexing table, no slab-split
 *            restrictions beyond those of tt_emb_config); cfg->device must be the current device;
 *            cfg->max_batch only bounds B
 *   g1..g3   device, the cores (read only)          ids   device int64[B]
 *   out      device fp32[B][D]                      B     0 <= B <= cfg->max_batch
 * The scratch need grows with the batch: about 100 bytes per id plus 4*d1*d2*r2 bytes per distinct
 * (i1,i2) prefix the batch could hold (min(B, n1*n2) of them) plus tables of a few n2, n3 words;
 * a batch that needs more than 64 MiB returns TT_EMB_ENOSPC (a 136 x 136 x 136 table at rank 32
 * has 18,496 prefixes of 2 KiB and fits batches of up to about 250,000 ids; a 480 x 480 x 482
 * table at rank 16 can meet a new 1 KiB prefix with every id and fits about 55,000).  TT_EMB_EINVAL for null or misaligned pointers, a bad configuration, or a current
 * device other than cfg->device.  The first call on a device looks the array's address up
 * (hipGetSymbolAddress); make that call outside graph capture - a call with B = 0 does only that.
 * All calls on one GPU share the one array, which keeps the last call's contents (every kernel
 * clears what it needs cleared): calls that overlap on one GPU - two streams, two threads - race
 * and must be serialised by the caller; calls on one stream are ordered by the stream.
 */
int tt_emb_lookup_static(const tt_emb_config* cfg, const float* g1, const float* g2, const float* g3,
                         const int64_t* ids, int64_t B, float* out, void* hip_stream);

/*
 * Writes the rows first_row .. first_row+count-1 of the table W itself (Section 3, Eq. "tt-matrix":
 * the dense matrix the cores stand for) to out, device fp32[count][D]; count may exceed max_batch
 * (the rows are produced max_batch at a time).  Row numbers are table rows: a re-indexing table is
 * not applied.  0 <= first_row, first_row + count <= N.  TT_EMB_ESTATE while a forward is pending.
 */
int tt_emb_materialize(tt_emb_t h, int64_t first_row, int64_t count, float* out, void* hip_stream);

/*
 * Node re-indexing (Section 4.2: nodes are renumbered, e.g. by graph partition, so that nodes that
 * are drawn together get neighbouring table rows and share (i1,i2) prefixes).  new_id_of: device
 * int32[n_ids], borrowed until replaced or the handle is destroyed; every later prepare / forward /
 * forward_eval looks up row new_id_of[id] for id in [0, n_ids) and treats any other id, and any
 * entry outside [0, N), as out of range.  new_id_of = NULL (n_ids = 0) removes the table.  Host-only;
 * prepared batches are dropped.  TT_EMB_ESTATE while a forward is pending.
 */
int tt_emb_set_reindex(tt_emb_t h, const int32_t* new_id_of, int64_t n_ids);

/*
 * Update rule of backward_update (the paper names no optimiser; plain SGD is the default).  With
 * three state arrays - device fp32, shaped and aligned like g1, g2, g3, zeroed by the caller before
 * the first step, borrowed until replaced or the handle is destroyed - every later backward_update
 * applies row-sparse Adagrad to the slices the batch touches:
 *   S[s] <- S[s] + dG[s]^2 ;  G[s] <- G[s] - lr * dG[s] / (sqrt(S[s]) + eps)      (elementwise)
 * with dG the same batch-summed gradient as for SGD; untouched slices and their state are not
 * written.  eps > 0.  Three null pointers return to SGD.  Host-only.
 */
int tt_emb_set_adagrad(tt_emb_t h, float* s1, float* s2, float* s3, float eps);

/*
 * The same for Adam in its row-sparse ("lazy") form: six state arrays (first moments m1..m3, second
 * moments v1..v3; device fp32, shaped and aligned like the cores, borrowed), and for the slices a
 * batch touches, with t = steps_done + 1, + 2, ... counting the backward_update calls that had a
 * non-empty batch:
 *   m <- beta1 m + (1 - beta1) dG ;  v <- beta2 v + (1 - beta2) dG^2
 *   G <- G - lr * (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps)          (elementwise)
 * Untouched slices keep core and moments (their moments do not decay).  0 <= beta < 1, eps > 0;
 * steps_done is 0 for zeroed moments, or the step count the moments were saved at.  Six null
 * pointers return to SGD; tt_emb_set_adagrad and tt_emb_set_adam replace each other.  Host-only.
 */
int tt_emb_set_adam(tt_emb_t h, float* m1, float* m2, float* m3, float* v1, float* v2, float* v3,
                    float beta1, float beta2, float eps, int64_t steps_done);

/*
 * Optional flow control for loops that never synchronise: blocks the calling host thread until the
 * backward_update made `age` calls before the latest one (age 0: the latest, at most 2) has
 * finished on the device.  Only calls made on a handle with TT_EMB_FLAG_IDS_READY after
 * tt_emb_prepare has been used are tracked (they are the ones that leave an event behind);
 * anything else returns at once.  Calling it with age 1 before every step keeps the host at most
 * two steps ahead of the device, which is when tt_emb_forward finds the pipeline of its prepared
 * batch finished and need not put a wait for it on the caller's stream.  Enqueues nothing.
 */
int tt_emb_wait_backward(tt_emb_t h, int age);

/*
 * Optional: builds the index structures (split, sort, unique ids and prefixes: the part of
 * Section 4.2's sharing that depends on the ids only) of a COMING batch ahead of time, on a stream
 * of the library's own that starts once everything enqueued so far on hip_stream has run.  A later
 * tt_emb_forward with the same ids pointer and the same B finds them ready, waits for them on its
 * own stream and skips that work (the oldest such batch if two match); a prepared batch that no
 * forward asks for is eventually overwritten (the oldest first).  The workspace holds four index
 * sets, which take turns on the library's two streams: one set may be in use by a forward/backward
 * pair while two others are filled, so up to two batches can be ahead, and an index pipeline that is
 * started two steps early has two steps to finish.  Typical use, once per step, anywhere around
 * the calls of the current batch: forward(ids); prepare(ids of the batch after next); ...;
 * backward_update(...) - the index
 * work of coming batches then overlaps this batch's arithmetic (minibatch samplers know the next
 * ids early).  An ids buffer must keep its contents until the forward that uses it has been enqueued.
 * Results are identical with or without it.  tt_emb_get_stats refers to the latest forward only
 * until the next tt_emb_prepare.
 */
int tt_emb_prepare(tt_emb_t h, const int64_t* ids, int64_t B, void* hip_stream);

/*
 * Backward and update (Section 5, phases "bwd" and "upd").  grad_out: device fp32[B][D] for the
 * batch of the latest forward.  Forms dG1, dG2, dG3 of L = sum_b <grad_out[b], out[b]> from the
 * cores as they are when the call starts (all positions add, no averaging), then applies
 * Gk[s] <- Gk[s] - lr*dGk[s] to every slice s the batch touches; other slices are not written.
 * Sums are formed in a fixed order: the same inputs give bit-identical cores.  Consumes the
 * pending forward (a second call without a new forward returns TT_EMB_ESTATE); a call that is
 * rejected for its arguments (TT_EMB_EINVAL) leaves the forward pending.
 */
int tt_emb_backward_update(tt_emb_t h, const float* grad_out, float lr, void* hip_stream);

/*
 * Counters of the latest forward: U = distinct in-range ids, Q = distinct (i1,i2) prefixes,
 * out_of_range = number of ids outside [0, N).  Any pointer may be null.  Synchronises the stream
 * of that forward.  Returns TT_EMB_ERANGE (flag CHECK_RANGE set and out_of_range > 0) or
 * TT_EMB_EINTERNAL after filling the outputs.
 */
int tt_emb_get_stats(tt_emb_t h, int64_t* U, int64_t* Q, int64_t* out_of_range);

/*
 * Per-kernel timing for benchmarks.  While enabled, every kernel launch is bracketed by a pair of
 * HIP events on the launch stream (this slows a step down; never enable it inside a throughput
 * measurement).  tt_emb_profile_read synchronises, then reports for kernel slot k (0 <= k < n,
 * n = return value of tt_emb_profile_slots) its name, the number of launches and their summed
 * duration in milliseconds since profiling was enabled or last read; it then resets the sums.
 * The last slot, "event_pair", is an event pair with no launch between, recorded once per
 * backward_update: its average is what the bracketing itself adds to every other slot.
 */
int tt_emb_profile_enable(tt_emb_t h, int enable);
int tt_emb_profile_slots(void);
int tt_emb_profile_read(tt_emb_t h, int slot, const char** name, int64_t* launches, double* ms);

/*
 * Device calibration for roofline figures (not part of the path), best of five launches each:
 *   copy    a plain streaming copy of the first half of device_buf onto its second half; bytes
 *           read + written per second (the larger the buffer, the closer to the HBM rate)
 *   mfma    a register-resident loop of fp32 matrix-core instructions on every compute unit; flop
 *           per second
 *   gather  1 KiB records fetched from pseudo-random places of a 1 MiB table (resident in every
 *           L2), eight in flight per wavefront, no reuse in the vector L1: bytes per second that
 *           the path L2 -> L1 -> registers delivers to per-id operand gathers
 *   far_gather  the same gathers from a 64 MiB table (beyond the L2s, inside the Infinity Cache):
 *           what the fabric behind the L2s delivers to them; 0 when device_buf is below 66 MiB
 * device_buf: caller-owned, 256-byte aligned, at least 8 MiB.  Synchronises hip_stream; overwrites
 * device_buf.
 */
int tt_emb_profile_peaks(void* device_buf, size_t bytes, void* hip_stream, double* copy_bytes_per_s,
                         double* mfma_flops_per_s, double* gather_bytes_per_s,
                         double* far_gather_bytes_per_s);

/* Frees the handle (host memory only). */
int tt_emb_destroy(tt_emb_t h);

/* Static description of a code; for TT_EMB_EHIP the text of the most recent HIP failure. */
const char* tt_emb_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* TT_EMB_H */
