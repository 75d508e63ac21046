/*
 * marsit.h -- C ABI of the MI355X (gfx950) library for the one-bit synchronisation pass of
 * Marsit ("Sign Bit is Enough: A Learning Synchronization Framework for Multi-hop All-reduce with
 * Ultimate Compression", arXiv 2204.06787).
 *
 * Conventions shared by every entry point
 *   - Return value: MARSIT_OK (0) or a negative marsit_status.  Nothing throws.
 *   - Pointers named g, c, x, update*, bits*, recv, local, out are DEVICE pointers owned by the
 *     caller.  The library never allocates, frees or synchronises; work is enqueued on `stream`
 *     (a hipStream_t passed as void*; NULL is the default stream) and the call returns at once.
 *     Apart from the marsit_pipeline_* calls an entry point only launches kernels on `stream`, so
 *     it may be recorded into a HIP graph; scalar arguments (seed, t, scale) are then fixed in it.
 *   - Host threads: the library keeps no mutable state between calls (the error slots below are per
 *     thread), so threads may call it at the same time on their own streams and buffers.  The
 *     exceptions are stated where they apply: one marsit_pipeline object is used by one thread at
 *     a time, marsit_exchange_step_sim_static shares one workspace per GPU, and
 *     marsit_set_fused_waves_per_cu changes a process-wide setting.
 *   - fp32 vectors are plain arrays of IEEE-754 binary32.  Arithmetic is fp32 with one
 *     round-to-nearest-even operation per step of Algorithm 1; denormals are kept.
 *   - Sign bitmaps: 64-bit words; element e sits in word e/64 at bit e%64 (least significant
 *     first); bit 1 means +1, i.e. the IEEE sign bit is clear (+0 -> +1, -0 -> -1); bits at
 *     positions >= d of the last word are written as 0.  Bitmap pointers must be 8-byte aligned,
 *     fp32 pointers 4-byte aligned (MARSIT_EALIGN otherwise).  That is all the 128-bit accesses of
 *     the kernels need; but rows that start on 128-byte boundaries (128-byte aligned bases, row
 *     stride ld a multiple of 32 elements) are faster, because a wavefront's 1 KB access then
 *     covers 8 whole cache lines instead of straddling 9 (77-80 % against 69-74 % of the HBM peak
 *     for the fused pass): a caller that owns the layout should pad ld to a multiple of 32.
 *   - Random merge masks: counter-based Philox4x32-10.  The 32-bit word that decides bit j of
 *     packed word w at hop id h is output (j mod 4) of Philox with key = (seed low, seed high) and
 *     counter = (j / 4, h, w low, w high).  With fold count m the local sign is taken where that
 *     word is < floor(2^32 / m)  (probability 1/m; m = 1: always).
 *   - d == 0 or n_words == 0: success, nothing is launched.
 *   - NaN inputs: the sign bit of whatever the fp32 add produces is used; bit-for-bit agreement
 *     with another machine is not promised for NaN.
 */
#ifndef MARSIT_H
#define MARSIT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MARSIT_MAX_WORKERS 64u

/* Largest number of elements per vector (d, n) any entry point takes: 2^34 - 1024.  Every kernel
 * covers its vector with one launch, at most one work-item per 4 elements in whole workgroups of
 * 256, and a launch must stay below 2^32 work-items.  Larger sizes return MARSIT_EINVAL; split the
 * vector (the random stream is keyed by the global word index, see word_begin). */
#define MARSIT_MAX_ELEMENTS 17179868160ull

typedef enum marsit_status {
    MARSIT_OK = 0,
    MARSIT_EINVAL = -1,   /* NULL required pointer, M == 0, M > MARSIT_MAX_WORKERS, fold == 0, ld < d,
                             grid_x does not divide M, non-finite scale, K == 0, more than
                             MARSIT_MAX_ELEMENTS elements */
    MARSIT_EALIGN = -2,   /* a pointer is not aligned to its element size */
    MARSIT_EHIP = -3,     /* a HIP call failed; marsit_last_hip_error() has the raw hipError_t */
    MARSIT_ESCRATCH = -4  /* marsit_exchange_step_sim_static only: the input needs more workspace than
                             MARSIT_STATIC_SCRATCH_WORDS */
} marsit_status;

/* Library version: major * 10000 + minor * 100 + patch. */
int marsit_version(void);

/* Raw hipError_t of the last failed HIP call made by this library on the calling thread (0: none). */
int marsit_last_hip_error(void);

/* Static, NUL-terminated description of a status code. */
const char *marsit_status_string(int status);

/* Host-side.  Work-items in x of the widest launch any entry point makes for a vector of d elements
 * (columns of 4 elements in whole workgroups of 256); 0 if d is 0 or exceeds MARSIT_MAX_ELEMENTS.
 * Always below 2^32, the most one launch may have. */
uint64_t marsit_grid_work_items(uint64_t d);

/*
 * Host-side Philox4x32-10 (Salmon et al., SC'11), the generator behind the merge masks.
 * All three arrays are HOST memory.  For tests and for callers that want to replay a mask.
 */
void marsit_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/*
 * Host-side.  "Split into M parts" (the split step of Algorithm 1) on packed words, as the schedules use it.
 * Writes M + 1 non-decreasing word indices to bounds_out (HOST memory); part f covers words
 * [bounds_out[f], bounds_out[f+1]).
 *   ring (grid_x == 0 or grid_x == M): part i = [floor(i*W/M), floor((i+1)*W/M)); its chain
 *     starts at worker i.
 *   torus (X = grid_x columns, Y = M / X rows): the W words are split in X row-parts by the same
 *     rule and every row-part again in Y sub-parts; part f = a*Y + b is sub-part b of row-part a.
 * Returns MARSIT_EINVAL for M == 0, M > MARSIT_MAX_WORKERS, grid_x not dividing M, NULL bounds_out.
 */
int marsit_split_bounds(uint64_t n_words, uint32_t M, uint32_t grid_x, uint64_t *bounds_out);

/*
 * Algorithm 1, compensated gradient and sign step for one worker:  bit e of bits_out = sgn(g[e] + c[e]).
 *   g, c     [d] fp32; c may be NULL (taken as 0).
 *   bits_out [ceil(d/64)] 64-bit words.
 */
int marsit_compress(const float *g, const float *c, uint64_t *bits_out, uint64_t d, void *stream);

/*
 * Algorithm 1, merge step (the operator of Section 4.1.1) for one hop and a run of packed words:
 *     out = (recv AND local) OR ((recv XOR local) AND v),  v drawn by Eq. 2 of Section 4.1.1
 * which is the same as: take the local bit where the Bernoulli(1/fold) draw succeeds, else keep
 * the received bit.
 *   recv       [n_words] bitmap received from the previous worker of the chain.
 *   local      [n_words] this worker's own sign bitmap (torus column phase: its row's result).
 *   out        [n_words]; may be the same buffer as recv or as local.
 *   word_begin global index of word 0 of these arrays in the whole bitmap (it keys the stream).
 *   fold       how many workers `out` stands for, this one included (>= 1); hop h of a ring: h+1.
 *   hop_id     Philox counter word 1.  Ring: h.  Torus: row phase (y << 8) | h for row y,
 *              column phase (1 << 16) | k.
 */
int marsit_hop_merge(const uint64_t *recv, const uint64_t *local, uint64_t *out,
                     uint64_t word_begin, uint64_t n_words, uint32_t fold, uint32_t hop_id,
                     uint64_t seed, void *stream);

/*
 * The sign step and one merge in one launch, for a worker that folds its own signs of a part into
 * the segment it received (Algorithm 1, sign step followed by the merge of the same part): the result equals
 * marsit_compress(g, c, tmp, n) followed by marsit_hop_merge(recv, tmp, out, word_begin,
 * ceil(n/64), fold, hop_id, seed), without storing the local bitmap.
 *   recv  [ceil(n/64)] received segment (may be NULL when fold == 1);  out may alias recv.
 *   g, c  [n] the worker's gradient and compensation FROM THE FIRST ELEMENT OF THE PART (element
 *         64 * word_begin of its vector); c may be NULL.  n: elements of the part (a ragged last
 *         word is allowed; its bits past n are written as 0).
 */
int marsit_compress_hop_merge(const uint64_t *recv, const float *g, const float *c, uint64_t *out,
                              uint64_t word_begin, uint64_t n, uint32_t fold, uint32_t hop_id,
                              uint64_t seed, void *stream);

/*
 * marsit_hop_merge with the seed read from DEVICE memory (one 64-bit word, 8-byte aligned) when
 * the kernel runs, not when it is enqueued: a HIP graph that a caller captures around such launches
 * can be replayed with a new seed.  marsit_set_device_seed writes that word with a one-thread kernel on `stream`
 * (no memcpy, so it may sit next to a graph launch).
 */
int marsit_hop_merge_device_seed(const uint64_t *recv, const uint64_t *local, uint64_t *out,
                                 uint64_t word_begin, uint64_t n_words, uint32_t fold, uint32_t hop_id,
                                 const uint64_t *seed_device, void *stream);
int marsit_set_device_seed(uint64_t *seed_device, uint64_t seed, void *stream);

/*
 * Algorithm 1, global update and compensation update for one worker, from the final bitmap every worker holds after the
 * gather period:   update_out[e] = bit ? +scale : -scale;   c_out[e] = (g[e] + c[e]) - update_out[e].
 *   bits       [ceil(d/64)].
 *   g, c       [d]; c may be NULL (taken as 0).
 *   scale      global step size eta_s; finite.
 *   update_out [d] or NULL (not written).
 *   c_out      [d]; may be the same buffer as c.
 */
int marsit_decode_compensate(const uint64_t *bits, const float *g, const float *c, float scale,
                             float *update_out, float *c_out, uint64_t d, void *stream);

/*
 * marsit_decode_compensate with the model update of Algorithm 2 in the same pass:
 * x[e] <- x[e] - update[e].  This is what one worker runs after the gather period: its gradient,
 * compensation and model are each read once, compensation and model written once (20 bytes per
 * element instead of 28 for the two separate passes).  x [d] must not alias the outputs;
 * update_out may be NULL.  Results equal marsit_decode_compensate followed by marsit_apply_update.
 */
int marsit_decode_compensate_apply(const uint64_t *bits, const float *g, const float *c, float scale,
                                   float *x, float *update_out, float *c_out, uint64_t d, void *stream);

/*
 * The whole one-bit pass (Algorithm 1, the branch mod(t,K) != 0) for M workers simulated inside one
 * device, fused in one kernel: compensate, sign, the M-1 merges of every part's chain, decode,
 * global compensation.  Results are bit-identical to chaining marsit_compress, marsit_hop_merge
 * and marsit_decode_compensate along the same schedule.
 *   g          [M][ld] gradients, already multiplied by the local step size (as Algorithm 2 passes them).
 *   c          [M][ld] compensation; read as c_t, overwritten with c_{t+1}.  Columns >= d untouched.
 *   update_out [d] global update g_t (the same for every worker).
 *   bits_out   [ceil(d/64)] final merged bitmap, or NULL.
 *   M          1..MARSIT_MAX_WORKERS.   ld >= d.
 *   grid_x     0 or M: ring; part i starts at worker i and hop h folds worker (i+h) mod M.
 *              Otherwise a torus with X = grid_x columns and Y = M/X rows, worker (y,x) = y*X + x:
 *              rows first (in every row the chain of row-part a starts at column a), then columns
 *              over the Y row results (the chain of sub-part b starts at row b).
 */
int marsit_ring_step_sim(const float *g, float *c, float *update_out, uint64_t *bits_out,
                         uint32_t M, uint64_t d, uint64_t ld, float scale, uint64_t seed,
                         uint32_t grid_x, void *stream);

/*
 * Tuning hook, host-side, process-wide.  The compiled kernels of marsit_ring_step_sim (and of the
 * entry points built on them) limit how many of their one-wavefront workgroups share a compute unit
 * -- about 21 / M, never fewer than 3 -- because HBM delivers most when the window of addresses in
 * flight is compact.  waves = 2..32 forces that count for every compiled ring and torus schedule,
 * 0 restores the built-in choice; anything else is MARSIT_EINVAL.  Results do not depend on it.
 * bench.py --fused-waves uses it to reproduce the occupancy sweep behind the built-in choice.
 */
int marsit_set_fused_waves_per_cu(uint32_t waves);

/*
 * Other multi-hop schedules (Section 5 names tree all-reduce and others as easy extensions, without
 * detail).  Reading taken: when the two operands of a merge stand for different numbers of workers,
 * Eq. 2 is used with the local share in place of 1/m, i.e. the local sign is kept with probability
 * w_local / (w_recv + w_local), decided by u < floor(2^32 * w_local / (w_recv + w_local)).
 * marsit_hop_merge(fold) is marsit_hop_merge_weighted(w_recv = fold - 1, w_local = 1).
 *   w_local >= 1; w_recv = 0: out = local.  Other arguments as in marsit_hop_merge.
 */
int marsit_hop_merge_weighted(const uint64_t *recv, const uint64_t *local, uint64_t *out,
                              uint64_t word_begin, uint64_t n_words, uint32_t w_recv,
                              uint32_t w_local, uint32_t hop_id, uint64_t seed, void *stream);

/*
 * The one-bit pass over a binary reduction tree, fused in one kernel: whole vectors, no split in
 * parts; at level l (stride 2^l) worker k = 0, 2*2^l, 4*2^l, ... receives the sign vector of worker
 * k + 2^l and folds it into its own, each side weighted by the workers of its subtree (so any M
 * works, not only powers of two); after ceil(log2 M) levels worker 0 holds the final vector.
 * hop id of a merge: (2 << 16) | (level << 8) | receiver.  A hierarchical ("segmented") ring of
 * groups is the torus schedule of marsit_ring_step_sim with grid_x = group size.
 * Arguments as in marsit_ring_step_sim.
 */
int marsit_tree_step_sim(const float *g, float *c, float *update_out, uint64_t *bits_out,
                         uint32_t M, uint64_t d, uint64_t ld, float scale, uint64_t seed,
                         void *stream);

/* marsit_tree_step_sim with the model update x[e] <- x[e] - g_t[e] in the same pass (as
 * marsit_step_apply does for the ring and the torus); update_out may be NULL, x must not alias it. */
int marsit_tree_step_apply(const float *g, float *c, float *x, float *update_out, uint64_t *bits_out,
                           uint32_t M, uint64_t d, uint64_t ld, float scale, uint64_t seed, void *stream);

/*
 * The one-bit pass over a torus whose last row may be short (any 1 <= grid_x <= M; Section 5 names
 * further all-reduce layouts without detail): X = grid_x columns, Y = ceil(M / X) rows, worker
 * (y, x) = y*X + x; the last row has M - (Y-1)*X workers.  Row phase as in marsit_ring_step_sim
 * with every row's own length (the chain of row-part a starts at column a mod X_y); the column
 * merges are weighted by the number of workers each side stands for, as in
 * marsit_hop_merge_weighted, with hop id (1 << 16) | k.  If grid_x divides M this is
 * marsit_ring_step_sim (same results, same kernels).  Other arguments as there; the _apply form
 * also updates the model, as marsit_step_apply does.
 */
int marsit_ragged_torus_step_sim(const float *g, float *c, float *update_out, uint64_t *bits_out,
                                 uint32_t M, uint64_t d, uint64_t ld, float scale, uint64_t seed,
                                 uint32_t grid_x, void *stream);
int marsit_ragged_torus_step_apply(const float *g, float *c, float *x, float *update_out,
                                   uint64_t *bits_out, uint32_t M, uint64_t d, uint64_t ld, float scale,
                                   uint64_t seed, uint32_t grid_x, void *stream);

/*
 * The same pass as marsit_ring_step_sim, hop by hop, as a real transport would run it: one
 * marsit_compress per worker, then for every part the chain of M-1 marsit_hop_merge launches over
 * that part's words (row chains, then column chains on a torus), then one marsit_decode_compensate
 * per worker.  All launches go to `stream` in order.  Results are bit-identical to the fused pass;
 * it moves about 20*M*d bytes instead of 12*M*d and exists to show what the fusion buys and as the
 * skeleton for a transport between the hops.
 *   workspace  device scratch owned by the caller, marsit_chain_workspace_words(M, d, grid_x)
 *              64-bit words: the M per-worker bitmaps, then (torus only) the Y row results.
 *   bits_out   [ceil(d/64)] final merged bitmap; required here (the chains are built in it).
 * Other arguments as in marsit_ring_step_sim.
 */
int marsit_chain_step_sim(const float *g, float *c, float *update_out, uint64_t *bits_out,
                          uint64_t *workspace, uint32_t M, uint64_t d, uint64_t ld, float scale,
                          uint64_t seed, uint32_t grid_x, void *stream);

/*
 * The whole chain of one part in one launch, for a deployment that exchanges the sign segments
 * all-to-all instead of passing them round the ring (Section 4's reduce period collapsed into one
 * exchange step: every worker sends the owner of a part its own signs of that part, the owner
 * folds them, the gather period follows): out = the chain that starts with operand `first` and
 * folds operand (first + h) mod K at hop h = 1..K-1 with fold count h + 1 and hop id hop_base | h.
 * Bit-identical to the K - 1 marsit_hop_merge calls of that chain.
 *   maps          operand k's segment starts at maps + k * stride_words ([n_words] each).
 *   K             1..MARSIT_MAX_WORKERS operands;  first < K.
 *   hop_base      low 8 bits zero: 0 for a ring, (y << 8) for row y of a torus, (1 << 16) for the
 *                 column phase.
 *   out           [n_words]; must not overlap the operands.
 */
int marsit_fold_segments(const uint64_t *maps, uint64_t stride_words, uint32_t K, uint32_t first,
                         uint64_t *out, uint64_t word_begin, uint64_t n_words, uint32_t hop_base,
                         uint64_t seed, void *stream);

/*
 * The one-bit pass of M simulated workers as that one exchange step: M marsit_compress, one
 * marsit_fold_segments per part (rows, then columns on a torus), M marsit_decode_compensate, all
 * on `stream`.  Arguments, workspace (marsit_chain_workspace_words) and results as in
 * marsit_chain_step_sim; 3M launches on a ring instead of M*M + M.
 */
int marsit_exchange_step_sim(const float *g, float *c, float *update_out, uint64_t *bits_out,
                             uint64_t *workspace, uint32_t M, uint64_t d, uint64_t ld, float scale,
                             uint64_t seed, uint32_t grid_x, void *stream);

/* Host-side: size of the workspace of marsit_chain_step_sim in 64-bit words (0 for bad arguments). */
uint64_t marsit_chain_workspace_words(uint32_t M, uint64_t d, uint32_t grid_x);

/*
 * marsit_exchange_step_sim for callers that cannot allocate device memory or carry a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The call
 * allocates nothing and frees nothing; its workspace is a static device array inside the library of
 * MARSIT_STATIC_SCRATCH_WORDS 64-bit words (32 MiB, held by every GPU the library is used on until
 * the process ends).  Inputs, outputs and results exactly as marsit_exchange_step_sim.
 *   - Inputs with marsit_chain_workspace_words(M, d, grid_x) > MARSIT_STATIC_SCRATCH_WORDS are
 *     rejected with MARSIT_ESCRATCH before anything is launched (ring of M workers: M * ceil(d/64)
 *     words, so d <= 33 554 432 at M = 8; the 25.6 M-element, 8-worker workload fits).
 *   - The first call on a device looks the array's device address up (hipGetSymbolAddress, no
 *     allocation); make that first call outside a graph capture.
 *   - Every call on one GPU uses that GPU's one array.  Nothing in it has to start at zero (each
 *     word that is read was written earlier in the same call), so earlier calls leave no trace in
 *     the results; but two calls that overlap in time on one GPU (different streams, or graphs
 *     replayed concurrently) race on it and must be ordered by the caller.
 */
#define MARSIT_STATIC_SCRATCH_WORDS 4194304u
int marsit_exchange_step_sim_static(const float *g, float *c, float *update_out, uint64_t *bits_out,
                                    uint32_t M, uint64_t d, uint64_t ld, float scale, uint64_t seed,
                                    uint32_t grid_x, void *stream);

/*
 * The ring of Section 4 / Fig. 3 with one HIP stream per worker: every hop of every part is its own
 * launch and waits only for what a real ring waits for -- the segment from the previous worker
 * and the release of its own send buffer.  A worker computes the signs of the part it starts before
 * anything arrives (Algorithm 1: receive in parallel with the sign step); every later hop is one
 * marsit_compress_hop_merge launch.  The gather period is simulated: the last holder of a part writes it to bits_out, which
 * every worker reads.  marsit_pipeline_step takes grid_x as marsit_ring_step_sim does: on a torus each
 * row runs its ring first; the row result of row-part a ends at column (a + X - 1) mod X, whose Y
 * workers then run the column ring over the Y sub-parts of that row-part.  marsit_pipeline_ring_step
 * is marsit_pipeline_step with grid_x = 0.  Results are bit-identical to marsit_ring_step_sim.
 *
 * marsit_pipeline_create makes the M streams (default priority) and the events; this is the only
 * call of the library that creates runtime objects, marsit_pipeline_destroy releases them (after
 * synchronising the worker streams).  marsit_pipeline_step allocates nothing; it returns when
 * everything is enqueued, and `stream` is made to wait for the workers, so work enqueued on
 * `stream` afterwards sees the results.  One step at a time per pipeline object.
 *   workspace  device scratch owned by the caller, marsit_pipeline_workspace_words(M, d, grid_x)
 *              64-bit words (0 for an invalid shape): the M per-worker bitmaps and two send
 *              buffers per worker, on a torus also the Y row results and two column-phase send
 *              buffers per worker.
 */
typedef struct marsit_pipeline marsit_pipeline;
int marsit_pipeline_create(marsit_pipeline **out, uint32_t M);
int marsit_pipeline_destroy(marsit_pipeline *p);
uint64_t marsit_pipeline_workspace_words(uint32_t M, uint64_t d, uint32_t grid_x);
int marsit_pipeline_step(marsit_pipeline *p, const float *g, float *c, float *update_out,
                         uint64_t *bits_out, uint64_t *workspace, uint64_t d, uint64_t ld, float scale,
                         uint64_t seed, uint32_t grid_x, void *stream);
int marsit_pipeline_ring_step(marsit_pipeline *p, const float *g, float *c, float *update_out,
                              uint64_t *bits_out, uint64_t *workspace, uint64_t d, uint64_t ld,
                              float scale, uint64_t seed, void *stream);
/* Raw hipError_t of the last failed HIP call of the marsit_pipeline_* functions on this thread. */
int marsit_pipeline_last_hip_error(void);

/*
 * Algorithm 1, the branch mod(t,K) == 0 (the full-precision round) for M simulated workers:
 *     update_out[e] = (1/M) * sum_m (g[m][e] + c[m][e]);   c[m][e] = 0.
 * Each g + c is one fp32 add; their sum (m = 0..M-1, in that order, starting from +0) and the
 * division by M are done in double precision, and the quotient is rounded once to fp32.
 */
int marsit_full_sync(const float *g, float *c, float *update_out, uint32_t M, uint64_t d,
                     uint64_t ld, void *stream);

/*
 * Algorithm 1 as a whole: the one-bit pass when t mod K != 0, the full-precision round when
 * t mod K == 0.  K == 0 is MARSIT_EINVAL.  Round t = 0 satisfies t mod K == 0 for every K, so it is
 * always a full-precision round (and leaves bits_out unwritten): a run of one-bit rounds only
 * starts at t >= 1 with K > t_max, or calls marsit_ring_step_sim directly.  bits_out is left
 * untouched by a full-precision round.  Other arguments as in marsit_ring_step_sim.
 */
int marsit_step(uint64_t t, uint64_t K, const float *g, float *c, float *update_out,
                uint64_t *bits_out, uint32_t M, uint64_t d, uint64_t ld, float scale,
                uint64_t seed, uint32_t grid_x, void *stream);

/*
 * One round of Algorithm 2 in one pass: marsit_step and the model update x[e] <- x[e] - g_t[e] in
 * the same kernels (x is read and written once; the separate marsit_apply_update pass and, if
 * update_out is NULL, the write of g_t are saved).  Results equal marsit_step followed by
 * marsit_apply_update bit for bit.
 *   x           [d] the model, device memory, updated in place; must not alias update_out.
 *   update_out  [d] or NULL.
 * Other arguments as in marsit_step.
 */
int marsit_step_apply(uint64_t t, uint64_t K, const float *g, float *c, float *x, float *update_out,
                      uint64_t *bits_out, uint32_t M, uint64_t d, uint64_t ld, float scale,
                      uint64_t seed, uint32_t grid_x, void *stream);

/*
 * One round of Algorithm 1 with the schedule as an argument, and of Algorithm 2 when the model is
 * given: the whole decision "which branch, which schedule" is taken here, so a training loop makes
 * this one call per round.
 *   t mod K == 0 : the full-precision round (the same for every schedule; bits_out untouched);
 *   otherwise    : the one-bit pass over `schedule`:
 *     MARSIT_SCHEDULE_RING   grid_x must be 0 (or M);                 as marsit_ring_step_sim
 *     MARSIT_SCHEDULE_TORUS  1 <= grid_x <= M columns; the last row is short when grid_x does not
 *                            divide M;                                as marsit_ragged_torus_step_sim
 *     MARSIT_SCHEDULE_TREE   grid_x must be 0;                        as marsit_tree_step_sim
 *   x           [d] the model, updated in place (x <- x - g_t) in the same pass, or NULL for the
 *               synchronisation alone; must not alias update_out.
 *   update_out  [d] the global update g_t, or NULL when x is given.
 * Results equal the entry points named above (followed by marsit_apply_update) bit for bit.
 */
typedef enum marsit_schedule {
    MARSIT_SCHEDULE_RING = 0,
    MARSIT_SCHEDULE_TORUS = 1,
    MARSIT_SCHEDULE_TREE = 2
} marsit_schedule;
int marsit_round(uint64_t t, uint64_t K, int schedule, uint32_t grid_x, const float *g, float *c,
                 float *x, float *update_out, uint64_t *bits_out, uint32_t M, uint64_t d, uint64_t ld,
                 float scale, uint64_t seed, void *stream);

/*
 * Diagnostics of Section 3.2.2 / Fig. 2(b).  The matching rate of a sign vector is the share of
 * elements whose sign equals the sign of the non-compressed aggregate.
 *
 * marsit_aggregate_sign: bit e of bits_out = sgn(sum_m (g[m][e] + c[m][e])); every term is the fp32
 *   compensated gradient of Algorithm 1, the sum over m runs in double, in worker order.
 * marsit_majority_vote: bit e = 1 where at least as many workers have a + sign as a - sign
 *   (signSGD with majority vote; a tie counts as +).
 * marsit_count_matching: *count_out (DEVICE memory, one 64-bit word, overwritten) = number of
 *   positions e < d at which the two bitmaps agree.
 * g, c [M][ld]; bits_out, bits_a, bits_b [ceil(d/64)].
 */
int marsit_aggregate_sign(const float *g, const float *c, uint64_t *bits_out, uint32_t M, uint64_t d,
                          uint64_t ld, void *stream);
int marsit_majority_vote(const float *g, const float *c, uint64_t *bits_out, uint32_t M, uint64_t d,
                         uint64_t ld, void *stream);
int marsit_count_matching(const uint64_t *bits_a, const uint64_t *bits_b, uint64_t d,
                          uint64_t *count_out, void *stream);

/*
 * The strawman of Section 3.2 -- a comparison point, NOT part of Marsit: SSDM's stochastic sign
 * Q(.) (Appendix A: +1 with probability 1/2 + v_j / (2 ||v||)) and cascading compression
 * (receive, recover, aggregate, compress, send).
 *
 * marsit_ssdm_cascade_hop, one hop on a run of n elements (element 0 = bit 0 of bits word 0):
 *     t[e]    = (recv_bits ? (+-*recv_norm by the received sign) : 0) + (g[e] + c[e])       fp32
 *     *norm_out = sqrtf((float) sum_e (double)t[e]^2)
 *     bit e of bits_out = (double)u_e < (double)(0.5f + t[e] / (2.0f * *norm_out)) * 2^32
 *   u_e from the Philox stream of (seed, hop_id, word_begin + e/64), position e%64; p = 0.5 when the
 *   norm is 0.  recv_bits == NULL: the first holder (t = g + c).  bits_out may be recv_bits;
 *   norm_out must not be recv_norm.  recv_norm, norm_out: DEVICE floats.
 *   workspace: DEVICE scratch of MARSIT_CASCADE_WORKSPACE_BYTES bytes, 8-byte aligned.
 *
 * marsit_cascade_ring_step_sim, the whole strawman over the ring of M workers: part i of the
 * word-aligned split starts at worker i as Q(s^(i)) and takes M-1 cascade hops (hop id (3<<16)|h);
 * update_out[e] = (+-final norm of the part) / M; norms_out [M] (DEVICE) final norm per part.
 * c is read (s = g + c) but not updated: the strawman has no compensation step.
 */
#define MARSIT_CASCADE_WORKSPACE_BYTES 8256u
int marsit_ssdm_cascade_hop(const uint64_t *recv_bits, const float *recv_norm, const float *g,
                            const float *c, uint64_t *bits_out, float *norm_out, void *workspace,
                            uint64_t word_begin, uint64_t n, uint32_t hop_id, uint64_t seed,
                            void *stream);
int marsit_cascade_ring_step_sim(const float *g, const float *c, float *update_out, uint64_t *bits_out,
                                 float *norms_out, void *workspace, uint32_t M, uint64_t d, uint64_t ld,
                                 uint64_t seed, void *stream);

/*
 * Local momentum of the M workers before a synchronisation (Section 5, optimizers: the image runs
 * use Momentum; heavy-ball form):  buf <- beta * buf + grad;  g_out <- eta_l * buf,  each operation
 * rounded once in fp32.  g_out is what Algorithm 2 passes to the synchronisation as the scaled
 * gradient.  All three arrays are [M][ld] device memory, columns >= d untouched; g_out may be the
 * same array as grad, buf may not alias either.  beta, eta_l finite.
 */
int marsit_local_momentum(float *buf, const float *grad, float *g_out, uint32_t M, uint64_t d,
                          uint64_t ld, float beta, float eta_l, void *stream);

/*
 * Local Adam of the M workers before a synchronisation (Section 5, optimizers: the sentiment-analysis
 * runs use Adam; the paper prints no formula, the optimizer's published form with bias correction is
 * taken).  With first moment p = mom1, second moment q = mom2 and gradient a = grad:
 *     p <- beta1 * p + (1 - beta1) * a;     q <- beta2 * q + (1 - beta2) * (a * a);
 *     g_out <- eta_l * ((p / bias1) / (sqrt(q / bias2) + eps)),
 * each operation rounded once in fp32 in the order written (1 - beta is rounded once).  bias1 and
 * bias2 are the caller's 1 - beta1^t and 1 - beta2^t for the round t >= 1 being taken (they depend
 * on t only); both must be finite and non-zero.  g_out is what Algorithm 2 passes to the
 * synchronisation as the scaled gradient.  All four arrays are [M][ld] device memory, columns >= d
 * untouched; g_out may be the same array as grad, the moments may alias nothing.  A zero second
 * moment with eps = 0 gives 0/0 = NaN, as the formula says.
 */
int marsit_local_adam(float *mom1, float *mom2, const float *grad, float *g_out, uint32_t M, uint64_t d,
                      uint64_t ld, float beta1, float beta2, float eps, float eta_l, float bias1,
                      float bias2, void *stream);

/* Algorithm 2, the model update:  x[e] <- x[e] - update[e]. */
int marsit_apply_update(float *x, const float *update, uint64_t d, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MARSIT_H */
