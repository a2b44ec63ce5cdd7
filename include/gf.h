/*
 * gf.h -- C ABI of the MI355X (gfx950) implementation of one worker's
 * gradient-aggregation path of GradientFlow (arxiv 1902.06855).
 *
 * Notation (the paper's): m gradient tensors with IDs 1..m, produced by the
 * backward pass in the order m..1; N = total elements; P = number of workers
 * ("GPUs" in the paper; here P buffers resident in one GPU's memory); theta =
 * lazy-allreduce threshold; C = gradients per chunk; k = number of important
 * chunks; S = loss scale; hg = historical gradient (Algorithm 1).
 *
 * Conventions for every call
 *   - "device" pointers are HIP device memory owned by the caller; "host"
 *     pointers are ordinary host memory.  Pointer *tables* (arrays of
 *     pointers) passed to the compute calls are themselves device arrays.
 *   - The library owns only the plan (host tables + a few KB of device
 *     tables) and the fixed scratch array of gf_fuse_pack_static, which is part
 *     of its code object.  Compute calls allocate nothing, never synchronise with the
 *     host, and are enqueued on `stream` (a hipStream_t passed as void*;
 *     NULL = the default stream).
 *   - Data pointers need only their natural alignment (4 bytes for fp32,
 *     2 bytes for fp16); 16-byte aligned tensors take the 128-bit path.
 *   - Errors are return codes; nothing throws.  Arguments are validated on
 *     the host before anything is launched.  Non-finite inputs are not
 *     detected: infinities and NaNs propagate by IEEE rules.
 *   - fp16 means IEEE binary16; every fp32->fp16 conversion rounds to nearest
 *     even, keeps subnormals and overflows to infinity.
 *   - A call's outputs must not overlap its inputs unless stated.
 */
#ifndef GF_H
#define GF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GF_OK = 0,
    GF_EINVAL = 1,   /* bad argument (null where required, out of range, wrong mode) */
    GF_ENOMEM = 2,   /* host or device allocation failed (plan calls only)          */
    GF_EHIP = 3,     /* a HIP runtime call or kernel launch failed                  */
    GF_ESTATE = 4,   /* plan in the wrong state: device tables missing (call
                        gf_plan_to_device), already uploaded for a setter that
                        must run before, or uploaded to another GPU than the one
                        that is current at a compute call                           */
    GF_ELIMIT = 5    /* the plan needs more scratch than the fixed array of
                        gf_fuse_pack_static holds (use gf_fuse_pack)                */
} gf_status;

/* Element type of what travels between workers (Section 2.5: fp16 gradients go
 * into allreduce under mixed precision; Section 2.3: fp32 in the baseline). */
typedef enum { GF_WIRE_F16 = 0, GF_WIRE_F32 = 1 } gf_wire;

typedef struct gf_plan gf_plan;
typedef void *gf_stream;             /* hipStream_t */

/* phase bits of gf_fuse_pack */
#define GF_PHASE_ACCUM 1u            /* g + hg, chunk norms                        */
#define GF_PHASE_PACK  2u            /* cast, scale, pack, historical-gradient rule */
/* modifiers, for callers that run the four calls back to back on one workspace   */
#define GF_PHASE_SLOTS 4u            /* the workspace already holds the slot map of
                                        sel_idx (gf_chunk_score_select left it)    */
#define GF_PHASE_DEFER_NORMS 8u      /* leave the chunk norms in the workspace for
                                        gf_chunk_score_select to finish            */

const char *gf_status_string(gf_status s);

/* ------------------------------------------------------------------ planning
 * Section 3.1 (lazy allreduce) and Section 3.2 (chunk partition), host only:
 *   - pool layout: tensor j occupies [sum_{i>j} numel_i, sum_{i>=j} numel_i);
 *   - buckets: walking j = m..1, a bucket closes after the tensor that makes
 *     the waited size strictly greater than theta_elems; the rest is flushed
 *     after tensor 1; buckets hold whole tensors only;
 *   - chunks: chunk c = pool [c*C, min(N,(c+1)*C)), n_chunks = ceil(N/C).
 * tensor_numel: host array [m], ID order 1..m, every entry >= 1.
 * theta_elems >= 0 in wire elements.  chunk_elems = 0 makes a dense-only plan
 * (no sparsification; compute calls then work on internal fixed-size tiles and
 * the ring is run per bucket); chunk_elems >= 1 makes a CSC plan (the packed
 * buffer is reduced bucket-wise, see gf_ring_reduce_sim), at most 2^28.
 * 1 <= P <= 4096.
 * gf_plan_create touches no GPU.  Returns GF_EINVAL / GF_ENOMEM on failure and
 * leaves *out NULL. */
gf_status gf_plan_create(gf_plan **out, const int64_t *tensor_numel, int32_t m,
                         int64_t theta_elems, int32_t chunk_elems, int32_t P, gf_wire wire);

/* Element type of the gradients handed to gf_fuse_pack (Section 3.1: the
 * memory pool manages FP32 or FP16 gradients; Section 2.5: mixed-precision
 * backward produces FP16 gradients).  Default GF_WIRE_F32.  With GF_WIRE_F16
 * every pointer in `grads` / `pools` addresses IEEE binary16 values, which are
 * widened to fp32 exactly before anything else is done to them.  Host only;
 * may be changed between calls. */
gf_status gf_plan_set_grad_type(gf_plan *plan, gf_wire type);

/* Order of the simulated allreduce (Section 2.4).  M = 0 or M = P: the flat
 * ring over all P ranks (the default).  Otherwise the hierarchical allreduce
 * with M groups of G = P / M consecutive ranks (P must be a multiple of M), the
 * lowest rank of a group being its master:
 *   1. ring-based reduce inside each group: the partial sum travels along the
 *      chain that starts at the rank after the master and ends on the master,
 *      y_g = x_{gG+1} + x_{gG+2} + ... + x_{gG+G-1} + x_{gG}, rounded to the
 *      wire type at every hop;
 *   2. ring allreduce among the M masters: the buffer (or bucket) is cut into M
 *      segments of roundup(ceil(len / M), 16 bytes) elements and segment s ends
 *      as y_s + y_{s+1} + ... + y_{s-1} (indices mod M);
 *   3. broadcast inside each group (copies, no arithmetic).
 * gf_ring_reduce_sim, gf_plan_ring_segment and the bucket rule are otherwise
 * unchanged.  Host only; must be called before gf_plan_to_device (GF_ESTATE
 * afterwards).  GF_EINVAL if M does not divide P. */
gf_status gf_plan_set_reduce_groups(gf_plan *plan, int32_t M);

/* Copies the plan's tables to the current HIP device (allocates; synchronous).
 * Required once before any compute call; idempotent.  Compute calls must be
 * made with that same device current (GF_ESTATE otherwise). */
gf_status gf_plan_to_device(gf_plan *plan);

/* Frees host and device tables.  NULL is allowed. */
void gf_plan_destroy(gf_plan *plan);

/* Any output pointer may be NULL.  n_chunks is 0 for a dense-only plan. */
gf_status gf_plan_info(const gf_plan *plan, int64_t *N, int32_t *n_chunks, int32_t *n_buckets);

/* Host copies of the layout: tensor_off [m] (ID order), bucket_lo/hi [n_buckets]
 * (pool element ranges, generation order).  Any pointer may be NULL. */
gf_status gf_plan_layout(const gf_plan *plan, int64_t *tensor_off, int64_t *bucket_lo,
                         int64_t *bucket_hi);

/* Ring segment length (elements) for a message of L elements: the L elements
 * are cut into P equal segments (Section 2.4) of roundup(ceil(L/P), 16 bytes)
 * elements; trailing segments may be short or empty.  Returns -1 on bad input. */
int64_t gf_plan_ring_segment(const gf_plan *plan, int64_t L);

/* Number of work tiles (= n_chunks for a CSC plan) and the pieces of tensors
 * that make up tile `tile`, in pool order: piece i is `len[i]` elements of
 * tensor `tensor[i]` (0-based ID index) starting at element `src_off[i]` of
 * that tensor.  Returns the piece count (pieces beyond `cap` are not written),
 * or -1 on bad input.  For tests of the fusion tables. */
int32_t gf_plan_tiles(const gf_plan *plan);
int32_t gf_plan_tile_pieces(const gf_plan *plan, int32_t tile, int32_t cap,
                            int32_t *tensor, int64_t *src_off, int32_t *len);

/* Bytes of device scratch the compute calls need (pass it as `workspace`,
 * 256-byte aligned).  Its contents carry nothing from one call to the next,
 * except for the two hand-overs a caller may ask for explicitly: the slot map
 * that gf_chunk_score_select leaves for gf_fuse_pack (GF_PHASE_SLOTS) and the
 * unfinished chunk norms that gf_fuse_pack leaves for gf_chunk_score_select
 * (GF_PHASE_DEFER_NORMS).  Calls that may run at the same time must not share a
 * workspace, except gf_fuse_pack_range calls over disjoint chunk ranges that
 * all pass GF_PHASE_SLOTS. */
size_t gf_plan_workspace_bytes(const gf_plan *plan);

/* Warm-up dense training (Section 3.2): over the first `warmup_iterations`
 * iterations the sparsity ratio ramps linearly from zero to its final value
 * 1 - final_density.  Returns the number of important chunks for 0-based
 * iteration `iteration` of a CSC plan, computed in double precision as
 *     s = (1 - final_density) * min(iteration, warmup_iterations) / warmup_iterations
 *     k = ceil((1 - s) * n_chunks - 1e-9), clamped to [1, n_chunks]
 * (warmup_iterations = 0: the final value from the start).  Host only.
 * Returns -1 on bad input (dense plan, final_density outside (0, 1],
 * negative counts). */
int32_t gf_plan_warmup_k(const gf_plan *plan, double final_density, int64_t iteration,
                         int64_t warmup_iterations);

/* --------------------------------------------------------------- gf_fuse_pack
 * Lazy-allreduce fusion (Section 3.1), the allreduce-preprocess step of
 * Algorithm 1, the local chunk norms of Section 3.2, and the cast / pack of
 * Sections 2.5 and 3.2, for all P workers in one pass.
 *
 * Gradients come either as `grads`, a device table [P*m] of device pointers
 * (entry p*m + j = worker p's tensor with 0-based ID index j, numel_j fp32
 * values, anywhere in memory: the fusion is folded into the read), or as
 * `pools`, a device table [P] of N-element fp32 pools already laid out as
 * above (the paper's zero-copy design).  Exactly one of the two is non-NULL
 * when GF_PHASE_ACCUM is set; both are ignored otherwise.
 *
 * residual: device table [P] of N-element fp32 historical-gradient pools,
 *   read and written in place; NULL = dense path (acc = g, phase must be
 *   ACCUM|PACK, sel_idx must be NULL).
 * sel_idx:  device array [k], ascending chunk indices of the important
 *   chunks; NULL = every chunk (k ignored).  Requires a CSC plan.
 * sendbuf:  device table [P] of wire-typed buffers.  The j-th selected chunk
 *   is written at element j*C (chunks in ascending order, the short last chunk
 *   of the pool, if selected, comes last and is written at its real length);
 *   with sel_idx NULL the buffer is the whole pool, N elements.
 * chunk_l1: device [P*n_chunks] fp32 out (worker-major), or NULL; written
 *   when GF_PHASE_ACCUM is set: sum of |acc| over the chunk's real elements,
 *   accumulated in fp64, rounded once to fp32.  CSC plans only.
 *
 * phase = ACCUM          acc = g + hg (fp32), hg <- acc, norms out.
 * phase = PACK           acc = hg as left by ACCUM.  Selected chunks:
 *                        send = wire(acc * S), hg <- +0.  Others: hg <- mu*acc.
 * phase = ACCUM | PACK   both in a single pass over the data (sel_idx is
 *                        already known: the paper's schedule, or the dense path).
 * mu is Algorithm 1's "momentum" applied to the historical gradient.
 * workspace (gf_plan_workspace_bytes, 256-byte aligned) is needed when sel_idx
 * is given together with GF_PHASE_PACK, when chunk_l1 is asked for on a plan
 * whose chunks are longer than 8192 elements (partial norms are combined
 * there), and with either modifier bit; GF_EINVAL if it is missing then.  It may
 * be NULL otherwise.
 *
 * Modifier bits (Section 3.2: the important chunks of an iteration are chosen
 * at the end of the one before, so a steady-state iteration is this call, the
 * allreduce, the unpack and the selection, back to back on one workspace):
 *   GF_PHASE_SLOTS        with sel_idx and GF_PHASE_PACK: sel_idx / k are the
 *     selection the last gf_chunk_score_select on this workspace produced and
 *     nothing has written the workspace's slot map since; the call then does
 *     not rebuild it (one small launch fewer).
 *   GF_PHASE_DEFER_NORMS  with GF_PHASE_ACCUM on a CSC plan: the chunk norms
 *     stay in the workspace as per-sub-tile partial sums, chunk_l1 is ignored
 *     (may be NULL), and the next gf_chunk_score_select on this workspace, called
 *     with chunk_l1 NULL, finishes them (same values, same order of additions). */
gf_status gf_fuse_pack(const gf_plan *plan, uint32_t phase,
                       const void *const *grads, const float *const *pools,
                       float *const *residual,
                       const int32_t *sel_idx, int32_t k,
                       float loss_scale, float mu,
                       void *const *sendbuf, float *chunk_l1,
                       void *workspace, gf_stream stream);

/* --------------------------------------------------------- gf_fuse_pack_range
 * gf_fuse_pack over the chunks [chunk_lo, chunk_hi) only, for a caller that
 * packs the important chunks while backward is still filling the pool
 * (Section 3.2: an important chunk is copied into the packed buffer as soon as
 * backward has filled it, and the buffer is handed to allreduce whenever what
 * waits in it exceeds the threshold; Section 3.1, enable-overlap setting): once
 * the gradients of pool elements [chunk_lo * C, min(N, chunk_hi * C)) exist, this
 * call does for
 * those chunks exactly what gf_fuse_pack does for all of them -- sel_idx / k
 * are still the whole selection, the j-th selected chunk still lands at
 * element j*C of the send buffers, chunk_l1 entries outside the range are not
 * touched -- so that calls over ranges that tile [0, n_chunks) leave the same
 * bytes everywhere as one gf_fuse_pack.  CSC plans only; phase must include
 * GF_PHASE_ACCUM; 0 <= chunk_lo <= chunk_hi <= n_chunks (an empty range does
 * nothing).  Without GF_PHASE_SLOTS every call rebuilds the whole slot map. */
gf_status gf_fuse_pack_range(const gf_plan *plan, uint32_t phase,
                             const void *const *grads, const float *const *pools,
                             float *const *residual,
                             const int32_t *sel_idx, int32_t k,
                             float loss_scale, float mu,
                             void *const *sendbuf, float *chunk_l1,
                             int32_t chunk_lo, int32_t chunk_hi,
                             void *workspace, gf_stream stream);

/* -------------------------------------------------------- gf_fuse_pack_static
 * gf_fuse_pack for callers that can neither allocate device memory nor hand a
 * workspace over: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, same kernels and bit-identical
 * results; the scratch (slot map, partial chunk norms) lives in a fixed device
 * array of GF_STATIC_SCRATCH_BYTES that is part of the library's code object
 * (every GPU the library runs on holds one copy until the process ends).  The
 * call allocates nothing and frees nothing.
 * GF_ELIMIT if gf_plan_workspace_bytes(plan) > GF_STATIC_SCRATCH_BYTES (nothing
 * is launched); GF_EINVAL for the two modifier bits (the array is private to
 * this entry point); other errors as gf_fuse_pack.  All calls on one GPU share that
 * GPU's array, which keeps the previous call's contents (every entry a call
 * reads is written by that call first): two calls that overlap in time on one
 * GPU, on different streams or from different threads, race. */
#define GF_STATIC_SCRATCH_BYTES (4u << 20)
gf_status gf_fuse_pack_static(const gf_plan *plan, uint32_t phase,
                              const void *const *grads, const float *const *pools,
                              float *const *residual,
                              const int32_t *sel_idx, int32_t k,
                              float loss_scale, float mu,
                              void *const *sendbuf, float *chunk_l1, gf_stream stream);

/* ------------------------------------------------------ gf_chunk_score_select
 * Section 3.2, important-chunk selection.  What the paper does with a small
 * allreduce of the norm vector is here a sum over the P rows of chunk_l1.
 *
 * score[c] = sum_p chunk_l1[p][c]  (p ascending, fp64, rounded to fp32) for a
 * chunk that was not sent this iteration; for prev_sel[j] (the chunks that went
 * through this iteration's allreduce) score = sum_p (reduced_l1[j] / P): every
 * GPU holds the same reduced values and divides its norm by the GPU count.
 * prev_sel NULL (k_prev ignored) scores every chunk by the first rule.
 * The k chunks with the largest score are chosen, equal scores going to the
 * lower chunk index.  A score that is not a number ranks above every number
 * (such chunks tie among themselves); -0 equals +0.
 *
 * chunk_l1 [P*n_chunks], reduced_l1 [k_prev], prev_sel [k_prev] ascending:
 *   device, in.   scores [n_chunks] fp32, sel_idx [k] int32 ascending,
 *   mask [n_chunks] bytes (1 = chosen), packed_len [1] int64 (number of
 *   elements the chosen chunks hold): device, out; scores, mask and
 *   packed_len may be NULL.  sel_idx may be the same buffer as prev_sel.
 * chunk_l1 NULL: the norms are those the last gf_fuse_pack on this workspace
 *   left there (GF_PHASE_DEFER_NORMS).
 * workspace: needed when scores or chunk_l1 is NULL.  Whenever it is given the
 *   call also leaves the slot map of the new selection in it (rank of every
 *   chosen chunk, -1 elsewhere) for a gf_fuse_pack with GF_PHASE_SLOTS.
 * 1 <= k <= n_chunks.  CSC plans only. */
gf_status gf_chunk_score_select(const gf_plan *plan, const float *chunk_l1,
                                const float *reduced_l1, const int32_t *prev_sel, int32_t k_prev,
                                int32_t k, float *scores, int32_t *sel_idx, uint8_t *mask,
                                int64_t *packed_len, void *workspace, gf_stream stream);

/* --------------------------------------------------------- gf_ring_reduce_sim
 * The arithmetic of ring allreduce (Section 2.4) over P send buffers that all
 * live in this GPU's memory.  Element i of segment s ends up as the left fold
 *     x_s[i] + x_{s+1}[i] + ... + x_{s-1}[i]      (worker indices mod P)
 * rounded to the wire type after every addition, which is what P-1
 * reduce-scatter hops produce when rank r first sends its segment r to rank
 * r+1; the all-gather hops are copies.  After gf_plan_set_reduce_groups the
 * order is the hierarchical one described there (group chains, then the ring
 * over the masters, M segments instead of P).
 *
 * sendbuf: device table [P] of wire-typed buffers of L elements, only read
 *   (for a dense plan on an fp16 wire they may be the workers' fp16 gradient
 *   pools themselves: Section 3.1's allreduce directly on the memory pool).
 * CSC plan: the packed buffer [0, L) is reduced bucket by bucket, each bucket
 *   a ring of its own (Section 3.2: CSC starts an allreduce once the buffer
 *   holds more than theta): packed chunks are taken in order and a bucket
 *   closes after the chunk that makes the waited size strictly greater than
 *   theta_elems; the rest is flushed.  With theta_elems >= L that is one ring
 *   over [0, L).  If L_dev is non-NULL it points to a device int64 holding the
 *   actual length (0 <= *L_dev <= L) and L only sizes the launch; this lets
 *   the length come straight from gf_chunk_score_select.
 * Dense plan: L must be N, L_dev NULL; every lazy-allreduce bucket is reduced
 *   as a ring of its own (its own segments), all in one launch.
 * reduced: device, L wire elements out.  allgather_out: NULL, or a device
 *   table [P] of buffers that each also receive the L reduced elements. */
gf_status gf_ring_reduce_sim(const gf_plan *plan, const void *const *sendbuf, int64_t L,
                             const int64_t *L_dev, void *reduced, void *const *allgather_out,
                             void *workspace, gf_stream stream);

/* ------------------------------------------------------- gf_ring_reduce_range
 * gf_ring_reduce_sim for a CSC plan whose packed buffer is filled range by
 * range (gf_fuse_pack_range) while backward is still running: reduces exactly
 * those lazy-allreduce buckets of the packed buffer whose last chunk lies in
 * [chunk_lo, chunk_hi) -- the buckets that the sweep over that range completed
 * (Section 3.2: the allreduce of a bucket starts once the buffer holds more
 * than theta).  Which buckets those are is decided on the device from sel_idx
 * (the selection the buffer was packed with, k entries); the host needs no
 * copy of it, so a whole iteration can be recorded in a graph.  Calls over
 * ranges that tile [0, n_chunks) together leave the same bytes in `reduced`
 * as one gf_ring_reduce_sim.  L must be k * C (the buffer's capacity); L_dev as
 * in gf_ring_reduce_sim.  The caller orders the call after the gf_fuse_pack_range
 * calls of this and all earlier ranges. */
gf_status gf_ring_reduce_range(const gf_plan *plan, const void *const *sendbuf, int64_t L,
                               const int64_t *L_dev, const int32_t *sel_idx, int32_t k,
                               int32_t chunk_lo, int32_t chunk_hi, void *reduced,
                               void *const *allgather_out, void *workspace, gf_stream stream);

/* ------------------------------------------------------------ gf_unpack_apply
 * Second cast of Section 2.5 and the write-back of Section 3.2:
 *     out[c*C + i] = fp32(reduced[j*C + i]) * alpha     for c = sel_idx[j]
 * (alpha = 1/S gives back summed gradients in unscaled units).  Positions of
 * chunks that were not sent are not written.  sel_idx NULL = all N elements.
 * out_pool: device N-element fp32 pool, or NULL.  out_tensors: NULL, or a
 *   device table [m] of per-tensor fp32 destinations (0-based ID index); at
 *   least one of the two must be given, both may be.
 * reduced_l1: NULL, or device [k] fp32 out: sum of |out| over the j-th
 *   selected chunk (fp64 accumulation, one rounding); needs sel_idx.
 * L: elements in `reduced` (CSC: (k-1)*C < L <= k*C; dense: N). */
gf_status gf_unpack_apply(const gf_plan *plan, const void *reduced, int64_t L,
                          const int32_t *sel_idx, int32_t k, float alpha,
                          float *out_pool, void *const *out_tensors,
                          float *reduced_l1, void *workspace, gf_stream stream);

/* ------------------------------------------------------------ gf_unpack_range
 * gf_unpack_apply for the chunks of the packed buckets that
 * gf_ring_reduce_range reduces for the same [chunk_lo, chunk_hi): the other
 * selected chunks (and their reduced_l1 entries) are left for the calls whose
 * range completes their bucket.  Other arguments as in gf_unpack_apply. */
gf_status gf_unpack_range(const gf_plan *plan, const void *reduced, int64_t L,
                          const int32_t *sel_idx, int32_t k, int32_t chunk_lo, int32_t chunk_hi,
                          float alpha, float *out_pool, void *const *out_tensors,
                          float *reduced_l1, void *workspace, gf_stream stream);

/* ------------------------------------------------------------ gf_csc_iteration
 * One steady-state iteration of coarse-grained sparse communication in the
 * paper's schedule (Section 3.2: the important chunks of an iteration are chosen
 * at the end of the one before; Algorithm 1), issued by one host call as
 *     gf_fuse_pack (accumulate, chunk norms, pack, historical gradient)
 *  -> gf_ring_reduce_sim -> gf_unpack_apply -> gf_chunk_score_select
 * back to back on `stream`, with the chunk norms handed from the first call to
 * the last through the workspace.  Every buffer ends with the bytes the four
 * calls leave when made one by one.
 *
 * sel_idx [max(k, k_next)], device, in/out: in, the k important chunks of this
 *   iteration (ascending); out, the k_next chunks chosen for the next one.
 * packed_len, device int64, in/out: in, the number of elements the k chunks hold
 *   (as gf_chunk_score_select wrote it for them); out, the same for the next
 *   selection.
 * reduced_l1 [k] device out (the norms of the reduced chunks, which the selection
 *   consumes); scores [n_chunks] and mask [n_chunks]: device out, may be NULL.
 * modifiers: 0, or GF_PHASE_SLOTS when sel_idx / k are what the last
 *   gf_chunk_score_select or gf_csc_iteration on this workspace produced (the slot
 *   map is then not rebuilt).  The call always leaves the new selection's slot map
 *   in the workspace, so iterations chained on one workspace pass GF_PHASE_SLOTS.
 * Other arguments as in the four calls; workspace is required.  The first
 * iteration of a job has no selection yet and is made of the single calls
 * (accumulate, select, pack, ...).  CSC plans only.  Everything is validated
 * before the first launch. */
gf_status gf_csc_iteration(const gf_plan *plan, uint32_t modifiers,
                           const void *const *grads, const float *const *pools,
                           float *const *residual,
                           int32_t *sel_idx, int32_t k, int32_t k_next, int64_t *packed_len,
                           float loss_scale, float mu, void *const *sendbuf,
                           void *reduced, void *const *allgather_out,
                           float alpha, float *out_pool, void *const *out_tensors,
                           float *reduced_l1, float *scores, uint8_t *mask,
                           void *workspace, gf_stream stream);

/* ------------------------------------------------------- gf_unpack_sgd_update
 * gf_unpack_apply plus the SGD-update step of Algorithm 1 (momentum SGD
 * correction) in the same pass.  With g = fp32(reduced) * alpha, at every
 * element of an important chunk
 *     hu = momentum * hu + learning_rate * g      (historical update)
 *     w  = w + hu                                 (the update u_t is hu_t)
 * each product and sum rounded to fp32 on its own; elsewhere hu and w are not
 * touched (hu_t = hu_{t-1}, no update).  The sign convention is the paper's:
 * the caller passes a negative learning_rate for descent.
 * w / hu come either as N-element fp32 pools in the plan's layout (w_pool,
 * hu_pool) or as device tables [m] of per-tensor fp32 buffers (w_tensors,
 * hu_tensors); exactly one of the two forms.
 * w_half_pool / w_half_tensors: NULL, or the FP16 copy of the weights that
 *   forward and backward use under mixed precision (Section 2.5: FP16
 *   parameters there, FP32 values in the update), in the same form as w (an
 *   N-element binary16 pool, or a device table [m] of per-tensor binary16
 *   buffers; GF_EINVAL if the form differs).  Wherever a weight is updated its
 *   FP16 copy is rewritten from the new fp32 value (one conversion); the other
 *   elements are not touched.
 * out_pool (optional) also receives g as gf_unpack_apply would write it.  Other
 * arguments as in gf_unpack_apply. */
gf_status gf_unpack_sgd_update(const gf_plan *plan, const void *reduced, int64_t L,
                               const int32_t *sel_idx, int32_t k, float alpha,
                               float momentum, float learning_rate,
                               float *w_pool, float *hu_pool,
                               void *const *w_tensors, void *const *hu_tensors,
                               void *w_half_pool, void *const *w_half_tensors,
                               float *out_pool, float *reduced_l1,
                               void *workspace, gf_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* GF_H */
