/*
 * libslimdp -- the per-iteration communication-set path of Slim-DP
 * (Sun, Chen, Bian, Liu, Liu: "Slim-DP: A Light Communication Data Parallelism
 * for DNN", AAAI-18) as hand-written HIP kernels for gfx950 behind a C ABI.
 *
 * One context serves one global model of n binary32 parameters and up to
 * max_workers logical workers whose buffers all live on ONE GPU.
 *
 * General rules
 *  - Every pointer marked [dev] is device memory owned by the caller; every pointer
 *    marked [host] is host memory that is read (or written) during the call and not
 *    retained.  "table" = a host array of device pointers, one per worker.
 *  - Every call returns SLIMDP_OK or a negative SLIMDP_ERR_* code; on error nothing has
 *    been launched and slimdp_last_error() describes the cause.  Nothing aborts, throws
 *    or prints.
 *  - Calls are asynchronous on the HIP stream given to slimdp_create and never
 *    synchronise the host; every output size is known from the arguments.  Conditions
 *    only the device can detect (see slimdp_synchronize) are reported there.  The only
 *    work that may run elsewhere: an announced explorer draw (option "explore_hint_mode" = 1)
 *    and explorer requests (option "explore_async" = 1) on the library's own side stream; the
 *    calls that need their results make the caller's stream wait for them.
 *  - The library allocates device memory in slimdp_create, once more when the option
 *    "speculative_pack" is first switched on (slimdp_capture_bytes), and once more on the first
 *    explorer request that needs the large key buffer (see slimdp_capture_bytes); never otherwise.
 *  - Same inputs give the same output bits, whatever the launch geometry.
 *  - Indices are 0-based uint32 (the paper counts from 1); n <= SLIMDP_MAX_N = 2^31 (indices and loop counters are
 *    32-bit and no loop steps by 2^31 or more, so none can wrap).
 *
 * Tiles.  The index range is cut into tiles of at most SLIMDP_TILE consecutive
 * parameters that never cross a segment boundary (flat model: tile t is
 * [t*SLIMDP_TILE, (t+1)*SLIMDP_TILE)).  Every ascending index list the library writes
 * comes with its "tile offsets": off[t] = number of list entries below the start of tile
 * t, off[T] = list length (T = slimdp_num_tiles).  pack / merge / pull take those
 * offsets back so that no kernel has to search the lists.
 */
#ifndef SLIMDP_H
#define SLIMDP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SLIMDP_TILE 4096u
#define SLIMDP_MAX_WORKERS 32u
#define SLIMDP_MAX_SEGMENTS 65536u
#define SLIMDP_MAX_N (1ull << 31)

enum {
    SLIMDP_OK = 0,
    SLIMDP_ERR_INVALID_ARG = -1,   /* null pointer, zero size, unsorted segment offsets, W out of range */
    SLIMDP_ERR_OUT_OF_RANGE = -2,  /* k_s > n_s, m_s > n_s - k_s, counts that do not add up */
    SLIMDP_ERR_STALE_CORE = -3,    /* core_epoch is not the epoch of the context's current core */
    SLIMDP_ERR_WORKSPACE = -4,     /* device allocation failed in slimdp_create */
    SLIMDP_ERR_HIP = -5,           /* a HIP runtime call failed */
    SLIMDP_ERR_DEVICE_STATUS = -6  /* slimdp_synchronize: a kernel flagged an impossible request */
};

/* slimdp_select_core flags */
#define SLIMDP_SELECT_REUSE_HISTOGRAM 1u
/* slimdp_pack flags */
#define SLIMDP_PACK_UPDATES_AS_SCORED 1u

typedef struct slimdp_ctx slimdp_ctx;

/* ---------------------------------------------------------------------------------- */
/* Context                                                                             */
/* ---------------------------------------------------------------------------------- */

/* Creates a context for n parameters in n_seg segments.
 *   seg_off [host, n_seg+1]: seg_off[0]=0 < ... < seg_off[n_seg]=n (strictly increasing).
 *                            n_seg=1 is the flat model (global ranking, section 3.2 of the paper).
 *   seed: key of the counter-based generator used by slimdp_sample_explore.
 *   hip_stream: a hipStream_t (NULL = the default stream); all work is enqueued there.
 * Allocates slimdp_workspace_bytes(...) of device memory on the current device. */
int slimdp_create(slimdp_ctx** out, uint64_t n, uint32_t max_workers, uint32_t n_seg,
                  const uint64_t* seg_off, uint64_t seed, void* hip_stream);
int slimdp_destroy(slimdp_ctx* ctx);

/* Device bytes slimdp_create allocates; 0 if the arguments are invalid.  Pure host function. */
uint64_t slimdp_workspace_bytes(uint64_t n, uint32_t max_workers, uint32_t n_seg,
                                const uint64_t* seg_off);
/* Device bytes that switching option "speculative_pack" on allocates on top; 0 if the arguments are invalid.
 * Explorer requests whose candidates do not fit the small per-sub-tile slots (m_seg at least a quarter of what lies
 * outside the core, or segments so small that the candidate zone, about 12 sqrt(m_seg) + 64 words wide, covers more
 * than a few parameters in a thousand) allocate once more, 4 * max_workers * (n rounded up to tiles + one tile)
 * bytes, on their first occurrence.  Pure host function. */
uint64_t slimdp_capture_bytes(uint64_t n, uint32_t max_workers, uint32_t n_seg, const uint64_t* seg_off);
/* Number of tiles T; 0 if the arguments are invalid.  Pure host function. */
uint64_t slimdp_num_tiles(uint64_t n, uint32_t n_seg, const uint64_t* seg_off);
/* tile_start [host, T+1]: start index of every tile, tile_start[T] = n. */
int slimdp_tile_starts(const slimdp_ctx* ctx, uint32_t* tile_start);

/* Message for the last error returned on this context ("" if none).  ctx may be NULL:
 * then the message of the last failed slimdp_create on this thread. */
const char* slimdp_last_error(const slimdp_ctx* ctx);

/* Waits for the context's stream and returns SLIMDP_ERR_DEVICE_STATUS if a kernel since
 * the previous slimdp_synchronize met a request it could not satisfy (an explorer larger
 * than the number of non-core parameters of its segment, index lists whose length does
 * not match).  The only call that blocks the host. */
int slimdp_synchronize(slimdp_ctx* ctx);

/* Options.  Known names:
 *   "speculative_pack" (0/1, default 0): slimdp_score additionally keeps the update values of
 *       every parameter whose significance reaches the threshold of the previous
 *       slimdp_select_core less a small margin, up to a quarter of every 1024 parameters (own device
 *       allocation of about W*n bytes, made by this call: slimdp_capture_bytes); if the following slimdp_select_core(..REUSE_HISTOGRAM) finds its
 *       threshold at or above that bound, the next slimdp_pack takes the core values from
 *       there instead of scanning the update vectors again, PROVIDED that call carries the
 *       flag SLIMDP_PACK_UPDATES_AS_SCORED (see slimdp_pack); without the flag a pack always
 *       reads the vectors it is given.  Results are bit-identical either way (the same slow
 *       drift of the core that the paper's key caching relies on, section 3.3).  One capture
 *       serves one pack.
 *       Before the first selection of a context there is no earlier threshold: the scoring pass
 *       then estimates the coming one from a sample of its own significances (flat model, at
 *       least 64 whole tiles), provided it knows the size of the coming core: from an announced
 *       draw (slimdp_explore_hint), from option "expected_core", or from the last selection.
 *   "expected_core" (-1 = unknown, default; else k of the next slimdp_select_core, flat model).
 *   "explore_hint_mode" (0/1, default 0): where an announced explorer draw runs: 0 inside
 *       the next slimdp_score, 1 at once on a side stream of the library (default priority),
 *       beside whatever runs on the context's stream.
 *   "explore_async" (0/1, default 0): slimdp_sample_explore runs on the library's side stream, beside whatever is
 *       enqueued on the context's stream AFTER the call (its many small kernels are bound by latency, not by memory).
 *       It starts once everything enqueued before the call is done.  slimdp_pack, slimdp_merge and slimdp_pull wait
 *       for the requests that write the lists they are given (and do not wait for requests into other arrays);
 *       slimdp_select_core, slimdp_import_core, a synchronous slimdp_sample_explore, a slimdp_score that carries an
 *       announced draw, and slimdp_synchronize wait for all of them.  Other work on the context's stream must not
 *       touch the lists before one of those calls.  A pack that takes kept values
 *       (SLIMDP_PACK_UPDATES_AS_SCORED) extracts the core values meanwhile.  With cached core keys the request for
 *       iteration t+1 can be issued before the pack of iteration t (other output arrays) and then runs beside pack
 *       and merge.
 *   "side_blocks" (1..8): blocks per compute unit of a side-stream draw.
 *   "pull_kernel" (0/1, default 1): how slimdp_pull patches local models (1: a pass that streams them; 0: scattered
 *       writes); results do not depend on it.
 *   "pack_kernel" (0/1, default 1), "pack_nbuf" (1/2): which form of the general pack kernel runs (1: loading and
 *       storing waves apart; 0: one set of waves, with pack_nbuf tiles in LDS); results do not depend on them.
 *   "explore_force_fallback" (0/1/2), "explore_per_tile_tail" (0/1): test switches: make
 *       the explorer's first zones miss (1: too few candidates, 2: sure zone too large) so
 *       that the exact rerun runs; never take the short-list tail.
 *   "core_predict" (0/1/2, default 1): flat models with 16-byte aligned arrays: slimdp_score also sorts every whole tile
 *       against the threshold bin of the previous selection, so that slimdp_select_core(..REUSE_HISTOGRAM) need not read
 *       the scores again when its histogram confirms that bin (otherwise it does, as without the option).  0 switches
 *       that off; 2 is a test switch that makes the prediction always wrong.
 *   "capture_estimate_bias" (test switch): added to a sampled capture bound, in units of the last place.
 *   "score_pipeline" (0/1), "strided_tiles" (0/1), "build_blocks" (1..64), "pack_core_blocks" (0..64): which scoring
 *       kernel serves a flat model and launch shapes; results do not depend on them.
 * An unknown name or a value outside the stated range is SLIMDP_ERR_INVALID_ARG. */
int slimdp_set_option(slimdp_ctx* ctx, const char* name, int64_t value);

/* ---------------------------------------------------------------------------------- */
/* The path                                                                            */
/* ---------------------------------------------------------------------------------- */

/* Significance, equation (1) of section 3.2:  score_i = |w_i| + c * |g_i|, with
 * g_i = ((g_0[i] + g_1[i]) + ...) + g_{W-1}[i] in binary32 in worker order (the summed
 * update the server holds, section 3.3 steps 3 and 6) and ONE fused multiply-add
 * fma(c, |g_i|, |w_i|).  A NaN result is stored as the quiet NaN 0x7FC00000.
 *   w [dev, n], g [host table of W dev pointers, n each], c >= 0 finite,
 *   score [dev, n] fully overwritten.  1 <= W <= SLIMDP_MAX_WORKERS.
 * Also accumulates, per segment, the histogram of the leading bits of every score, which
 * the next slimdp_select_core may reuse (SLIMDP_SELECT_REUSE_HISTOGRAM). */
int slimdp_score(slimdp_ctx* ctx, const float* w, const float* const* g, uint32_t W, float c,
                 float* score);

/* The last iteration before a reselection (algorithm 1, the branch (t+1) % q == 0; section
 * 3.3 steps 3 and 6): every worker has pushed its WHOLE update, the server applies all of
 * them and ranks the new core with the new model and these updates, in one pass:
 *     acc_i = ((+0 + g_0[i]) + g_1[i]) + ...           binary32, worker order (as slimdp_merge)
 *     w_i  <- fma(-lr, acc_i, w_i)                     every i, in place
 *     score_i = fma(c, |acc_i|, |w_i (new)|)           equation (1), quiet NaN as in slimdp_score
 * Arguments as slimdp_score, w is read and written; lr finite; score must not alias w.
 * Leaves the same histogram behind as slimdp_score for slimdp_select_core to reuse, and
 * serves an announced explorer draw the same way. */
int slimdp_dense_update_score(slimdp_ctx* ctx, float* w, const float* const* g, uint32_t W, float lr,
                              float c, float* score);

/* Core-Selection operator T_S (section 3.1 item 1; section 3.2, the ranking after equation (1);
 * section 3.3 step 6): per segment s the k_seg[s] parameters that come first when ranked
 * by (score bit pattern as uint32, descending; index, ascending).  For scores >= +0 that
 * is the numeric order with ties going to the lower index; NaN ranks above +infinity.
 *   score    [dev, n]
 *   k_seg    [host, n_seg], k_seg[s] <= size of segment s
 *   flags    SLIMDP_SELECT_REUSE_HISTOGRAM: score is the buffer the last slimdp_score on
 *            this context wrote and has not been modified since (otherwise the library
 *            spends one more pass over score to count); error if no such histogram is pending.
 *   core_idx [dev, sum k_seg]  chosen global indices, ascending
 *   core_bits[dev, ceil(n/32)] bit (i mod 32) of word (i div 32) set iff i is in the core
 *   core_off [dev, T+1]        tile offsets of core_idx
 *   core_epoch [host, 1]       identifier of this core, the library's stand-in for what both
 *            ends of the key-caching filter hold (section 3.5); pack/merge/pull made for
 *            another core are refused with SLIMDP_ERR_STALE_CORE. */
int slimdp_select_core(slimdp_ctx* ctx, const float* score, const uint64_t* k_seg, uint32_t flags,
                       uint32_t* core_idx, uint32_t* core_bits, uint32_t* core_off,
                       uint64_t* core_epoch);

/* Resuming from a checkpoint.  The state of the path between two iterations is the global model, the cached core
 * keys, the iteration number and the seed (the explorers are functions of seed, iteration, worker and the core).  A
 * new context (same n, segments and seed) adopts the saved keys with this call and continues as if it had selected
 * them: it rebuilds the bitmap and the tile offsets from the list and issues a core epoch of its own.
 *   core_idx [dev, sum k_seg] ascending, k_seg[s] of them inside segment s (as slimdp_select_core wrote them; not
 *   re-checked); core_bits [dev, ceil(n/32)], core_off [dev, T+1], core_epoch [host, 1]: outputs. */
int slimdp_import_core(slimdp_ctx* ctx, const uint32_t* core_idx, const uint64_t* k_seg, uint32_t* core_bits,
                       uint32_t* core_off, uint64_t* core_epoch);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): the same selection as slimdp_select_core for a flat model (one segment) without a context.
 * Calls no hipMalloc / hipFree: the workspace is a fixed array of 5 MiB inside the library's device image (every GPU
 * the library runs on holds its own copy until the process ends), which serves n <= SLIMDP_STATIC_MAX_N
 * parameters; a larger n is refused with SLIMDP_ERR_OUT_OF_RANGE.  Runs on the current device, asynchronously on
 * hip_stream (NULL = the default stream).  All calls on one GPU share that GPU's array: calls that overlap in time
 * on one GPU (different streams or threads) race; serialise them.  Nothing else is shared with contexts.
 *   score [dev, n]; k <= n; core_idx [dev, k] ascending; core_bits [dev, ceil(n/32)];
 *   core_off [dev, slimdp_num_tiles(n, 1, {0, n}) + 1].  Errors: message via slimdp_last_error(NULL).
 * Conditions only the device could detect are not reported (there is no context to ask). */
#define SLIMDP_STATIC_MAX_N (1u << 20)
int slimdp_select_core_static(const float* score, uint64_t n, uint64_t k, uint32_t* core_idx, uint32_t* core_bits,
                              uint32_t* core_off, void* hip_stream);

/* Exploration operator T_R^k (section 3.1 item 2; section 3.3 step 2) for the workers
 * worker0 .. worker0+n_workers-1: each draws, per segment s, m_seg[s] parameters uniformly
 * without replacement from those outside the core, afresh for every (worker, iteration).
 * Realisation: parameter i gets the random word r = word (i mod 4) of Philox4x32-10 with
 * counter (i div 4, worker, iteration low 32, iteration high 32) and key (seed low, seed
 * high); the m_seg[s] non-core parameters with the smallest (r, i) are taken.
 *   core_bits [dev, ceil(n/32)] as written by slimdp_select_core
 *   k_seg     [host, n_seg]  number of core parameters per segment in core_bits (bounds m_seg
 *             and sizes the candidate search; a wrong value costs time, not correctness)
 *   m_seg     [host, n_seg], m_seg[s] <= n_s - k_seg[s]
 *   expl_idx  [host table, n_workers] of [dev, sum m_seg]: chosen global indices, ascending
 *   expl_off  [host table, n_workers] of [dev, T+1]: their tile offsets
 * If core_bits holds more core parameters than k_seg says and m_seg cannot be met, the
 * affected list is left partly unwritten and slimdp_synchronize reports it. */
int slimdp_sample_explore(slimdp_ctx* ctx, const uint32_t* core_bits, const uint64_t* k_seg,
                          uint32_t worker0, uint32_t n_workers, uint64_t iteration,
                          const uint64_t* m_seg, uint32_t* const* expl_idx,
                          uint32_t* const* expl_off);

/* Optional announcement of the explorer draw that a coming
 * slimdp_sample_explore(ctx, core_bits, k_seg, worker0, n_workers, iteration, m_seg, ...)
 * will need (the arguments must then be identical, else the draw is simply redone).  The
 * random words do not depend on the core or on any data, so their generation -- the only
 * step of the path bound by integer arithmetic rather than by memory -- can hide under
 * memory-bound work, as the paper notes for its worker side (section 3.5, the paragraph on
 * time efficiency): by default the next slimdp_score on this context draws while it streams
 * the model; with option "explore_hint_mode" = 1 the draw starts at once on a side stream.
 * Purely a performance hint: results are bit-identical with or without it.  Host arrays as
 * in slimdp_sample_explore; k_seg is the core size the coming slimdp_select_core will use. */
int slimdp_explore_hint(slimdp_ctx* ctx, const uint64_t* k_seg, uint32_t worker0, uint32_t n_workers,
                        uint64_t iteration, const uint64_t* m_seg);

/* Tile offsets of any ascending index list (for lists that did not come from the two
 * calls above).  idx [dev, count] ascending, all < n; off [dev, T+1]. */
int slimdp_tile_offsets(slimdp_ctx* ctx, const uint32_t* idx, uint64_t count, uint32_t* off);

/* Push, worker side (section 3.3 step 3; wire format of section 3.5): for each of the
 * n_workers workers extract its update at the communication set T_C = core U explorer.
 * Core: values only (the keys are cached under core_epoch); explorer: <key, value> with
 * the keys being expl_idx itself.  Bit copies:
 *   core_val[q][j] = g[q][core_idx[j]],  expl_val[q][j] = g[q][expl_idx[q][j]].
 *   g [host table, n_workers] of [dev, n]; core_idx [dev, k]; core_off [dev, T+1];
 *   expl_idx / expl_off [host tables]; m_w [host, n_workers] explorer sizes;
 *   core_val [host table] of [dev, k]; expl_val [host table] of [dev, m_w[q]].
 *   flags    SLIMDP_PACK_UPDATES_AS_SCORED: the caller states that g is the very table of
 *            arrays, unmodified since, that the last slimdp_score on this context read, and
 *            that core_idx came from the slimdp_select_core(..REUSE_HISTOGRAM) that followed
 *            it.  With option "speculative_pack" on, the pack may then take values the scoring
 *            pass kept instead of reading g again.  Never set it after refilling the update
 *            buffers (the steady iterations of algorithm 1 pack updates no scoring pass has
 *            seen): the library cannot detect changed contents, only a different table
 *            (SLIMDP_ERR_INVALID_ARG).  Without the flag nothing kept is ever used.
 * Words on the wire per worker: k + 2*m_w[q], the (2*alpha - beta)*n of section 3.5. */
int slimdp_pack(slimdp_ctx* ctx, uint32_t n_workers, const float* const* g,
                const uint32_t* core_idx, const uint32_t* core_off, uint64_t k,
                const uint32_t* const* expl_idx, const uint32_t* const* expl_off,
                const uint64_t* m_w, float* const* core_val, float* const* expl_val,
                uint64_t core_epoch, uint32_t flags);

/* Update, server side (section 3.3 step 3):  w_i <- w_i - lr * sum_q T_C(delta_q)_i.
 * For every index i some worker sent: acc = +0; for q ascending over the workers whose
 * communication set holds i: acc += value; then w_i = fma(-lr, acc, w_i).  Indices nobody
 * sent keep their bits.  No atomics; the result does not depend on scheduling.
 * Requires each explorer list to be disjoint from the core (as slimdp_sample_explore
 * guarantees); otherwise the core contributions to an index are added before the
 * explorer ones, those again in worker order.
 *   w [dev, n] in place; the other arguments as in slimdp_pack (values are inputs). */
int slimdp_merge(slimdp_ctx* ctx, float* w, float lr, uint64_t core_epoch, uint32_t n_workers,
                 const uint32_t* core_idx, const uint32_t* core_off, uint64_t k,
                 const float* const* core_val, const uint32_t* const* expl_idx,
                 const uint32_t* const* expl_off, const float* const* expl_val,
                 const uint64_t* m_w);

/* Pull and local Merge (section 3.3 steps 4 and 5): each worker reads the global model
 * at its communication set, core_out[q][j] = w[core_idx[j]], expl_out[q][j] =
 * w[expl_idx[q][j]]; if w_local is not NULL and w_local[q] is not NULL the worker's local
 * model is overwritten at those indices and left alone elsewhere.
 *   w [dev, n]; core_out [host table] of [dev, k]; expl_out [host table] of [dev, m_w[q]];
 *   w_local NULL or [host table] of (NULL or [dev, n]). */
int slimdp_pull(slimdp_ctx* ctx, const float* w, uint64_t core_epoch, uint32_t n_workers,
                const uint32_t* core_idx, const uint32_t* core_off, uint64_t k,
                const uint32_t* const* expl_idx, const uint32_t* const* expl_off,
                const uint64_t* m_w, float* const* core_out, float* const* expl_out,
                float* const* w_local);

/* LocalTrain, worker side (section 3.3 step 1; first line of the worker loop of algorithm 1): one mini-batch step
 * of every worker on its LOCAL model, and the accumulation of the update that the next push extracts from:
 *     w_local[q][i] <- fma(-eta, grad[q][i], w_local[q][i])
 *     delta[q][i]   <- grad[q][i]                      with SLIMDP_LOCAL_FIRST (first mini-batch after a communication)
 *     delta[q][i]   <- delta[q][i] + grad[q][i]        otherwise: the sum over the p mini-batches in binary32, in order
 * The gradient is an input (the library trains no network).  delta[q] is what slimdp_pack takes as g[q]; after the
 * push, slimdp_pull overwrites w_local[q] at the communication set (steps 4 and 5) and leaves the rest to diverge
 * from the global model, which is what the explorer is for (section 3.1).
 *   w_local, grad, delta [host tables, n_workers] of [dev, n], pairwise distinct per worker; eta finite. */
#define SLIMDP_LOCAL_FIRST 1u
int slimdp_local_step(slimdp_ctx* ctx, uint32_t n_workers, float* const* w_local, const float* const* grad,
                      float* const* delta, float eta, uint32_t flags);

/* LocalTrain and Push in one pass (section 3.3 steps 1 and 3): the last mini-batch step before a communication
 * together with the extraction of what the push sends.  Same results, bit for bit, as
 *     slimdp_local_step(ctx, n_workers, w_local, grad, delta, eta, flags) followed by
 *     slimdp_pack(ctx, n_workers, delta, core_idx, ..., core_val, expl_val, core_epoch, 0),
 * but the accumulated updates are not read a second time: the extraction's own scan of the update vectors (the full
 * scan that section 3.5 counts per extraction) rides on the pass that writes them.  Arguments as in those two
 * calls; the explorer lists of the coming push must exist (they depend on seed, iteration, worker and the core only:
 * slimdp_sample_explore can run before the local steps). */
int slimdp_local_step_pack(slimdp_ctx* ctx, uint32_t n_workers, float* const* w_local, const float* const* grad,
                           float* const* delta, float eta, uint32_t flags, const uint32_t* core_idx,
                           const uint32_t* core_off, uint64_t k, const uint32_t* const* expl_idx,
                           const uint32_t* const* expl_off, const uint64_t* m_w, float* const* core_val,
                           float* const* expl_val, uint64_t core_epoch);

/* Pull, local Merge and the first LocalTrain step of the next round in one pass (section 3.3 steps 4 and 5, then step 1):
 * every worker's local model is overwritten with the global one at its communication set, then stepped.  Same
 * results, bit for bit, as
 *     slimdp_pull(ctx, w, core_epoch, n_workers, core_idx, ..., w_local)      (its value outputs aside) followed by
 *     slimdp_local_step(ctx, n_workers, w_local, grad, delta, eta, flags),
 * but the local models are streamed once instead of being patched by scattered writes and then streamed.
 *   w [dev, n] the global model after the merge; lists as in slimdp_pull; w_local, grad, delta, eta, flags as in
 *   slimdp_local_step (SLIMDP_LOCAL_FIRST is the usual case: a new accumulation starts after a communication). */
int slimdp_pull_local_step(slimdp_ctx* ctx, const float* w, uint64_t core_epoch, uint32_t n_workers,
                           const uint32_t* core_idx, const uint32_t* core_off, uint64_t k,
                           const uint32_t* const* expl_idx, const uint32_t* const* expl_off, const uint64_t* m_w,
                           float* const* w_local, const float* const* grad, float* const* delta, float eta,
                           uint32_t flags);

/* Quantised wire values: the method composes with gradient quantisation (section 2.2, last sentences); the
 * comparison of section 4.2 uses random quantisation with 8 bits and buckets of 512, after Alistarh et al. (QSGD).
 * Applied to the packed values of workers worker0 .. worker0+n_workers-1 (kind 0: core_val, kind 1: expl_val):
 * per bucket of 512 consecutive list entries one binary32 scale = the bucket's largest magnitude; per value one
 * byte = sign bit | level, the level in 0..127 on the grid scale * level / 127, rounded up with probability equal
 * to the fraction (unbiased): y = (|v| / scale) * 127, level = floor(y) + (u < y - floor(y)), all in binary32,
 * u = (word >> 8) * 2^-24, word = word (j mod 4) of Philox4x32-10 with counter (j div 4, worker, iteration low,
 * iteration high) and key (seed low ^ 0x51534744, seed high ^ kind) for list entry j.  Values must be finite.
 * Bytes on the wire per worker: k + 4 ceil(k/512) for the core, 5 m + 4 ceil(m/512) for the explorer (its keys
 * stay 32-bit), against the 4 (k + 2m) of section 3.5.
 *   val [host table] of [dev, count[q]]; count [host, n_workers] <= n;
 *   code [host table] of [dev, count[q]] bytes; scale [host table] of [dev, ceil(count[q] / 512)]. */
int slimdp_quantize(slimdp_ctx* ctx, uint32_t n_workers, uint32_t worker0, const float* const* val, const uint64_t* count,
                    uint32_t kind, uint64_t iteration, uint8_t* const* code, float* const* scale);
/* The receiver's side: val[q][j] = sign * ((scale * level) / 127), two binary32 roundings.  The result feeds
 * slimdp_merge like unquantised packs. */
int slimdp_dequantize(slimdp_ctx* ctx, uint32_t n_workers, const uint8_t* const* code, const float* const* scale,
                      const uint64_t* count, float* const* val);

/* Signature of the cached core keys (section 3.5, communication efficiency: for the core only the values
 * travel, together with a signature of the cached keys): the two sides of a link compare it instead of the key
 * list.  The paper does not fix the function; here: sum over list positions j of mix(core_idx[j] + 2^32 * j) modulo 2^64, mix being
 * the output function of SplitMix64 (Steele, Lea, Flood, OOPSLA 2014).
 *   core_idx [dev, k], sig [dev, one uint64, 8-byte aligned] overwritten. */
int slimdp_core_signature(slimdp_ctx* ctx, const uint32_t* core_idx, uint64_t k, uint64_t* sig);

/* The raw random words slimdp_sample_explore attaches to the indices i0 .. i0+count-1 for
 * (worker, iteration) under the context's seed.  out [dev, count]. */
int slimdp_debug_philox(slimdp_ctx* ctx, uint64_t iteration, uint32_t worker, uint32_t i0,
                        uint64_t count, uint32_t* out);

#ifdef __cplusplus
}
#endif
#endif /* SLIMDP_H */
