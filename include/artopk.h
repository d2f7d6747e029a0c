/*
 * artopk.h -- C ABI of the MI355X (gfx950) AR-Topk gradient compressor.
 *
 * One call of artopk_step() performs, for W data-parallel workers whose
 * gradients all live on one GPU, the loop body of Alg. 1 of "Flexible
 * Communication for Optimal Distributed Learning over Unpredictable Networks"
 * (AR-Topk compression, Sec. III-A/III-B) together with the error feedback of
 * Sec. II-C:
 *
 *     acc_w   = g_w + residual_w                       (EF equations, Alg. 1)
 *     leader  = step mod W            (STAR-Topk)   or
 *               first argmax_w var(acc_w)  (VAR-Topk)  (Sec. III-B)
 *     idx     = the k positions of largest |acc_leader| (Sec. III-A, Topk)
 *     vals_w  = acc_w[idx]                             (Alg. 1, gather)
 *     sum     = ((vals_0 + vals_1) + ...) + vals_{W-1}  (stand-in for AllReduce)
 *     update  = zeros(N); update[idx] = sum            (input of the SGD update)
 *     residual_w = acc_w with the idx positions set to +0.0
 *
 * Conventions
 *   - W is the paper's cluster size N, N here is the number of gradient
 *     elements (the paper's G), k = ceil(c * N) is computed by the caller.
 *   - All data buffers are caller-owned DEVICE memory, float32 / int32 /
 *     float64 as typed, 16-byte aligned.  A buffer that a call writes must not
 *     overlap any other buffer of that call (checked on the host: ARTOPK_EINVAL);
 *     buffers that are only read may overlap each other.  Arrays of pointers
 *     (g, residual, acc, x) and the segment tables are HOST memory and are
 *     read before the call returns.
 *   - Work is enqueued on the stream given to artopk_create(); calls return
 *     without synchronising.  Outputs are valid once that stream has been
 *     synchronised by the caller.  Calls on one context must not overlap.
 *   - The library allocates device memory only inside artopk_create().
 *   - Return value: ARTOPK_OK or a negative error code; on ARTOPK_EINVAL
 *     nothing has been enqueued.  No exception or abort crosses this boundary.
 *   - Magnitudes are ordered by the raw 31 magnitude bits of the float32, so
 *     +x and -x tie, denormals keep their order, Inf > finite, NaN > Inf.
 *     Among equal magnitudes the lowest index wins.  idx is ascending.
 *   - N < 2^31, 1 <= k <= N, 1 <= W <= ARTOPK_MAX_WORKERS.
 */
#ifndef ARTOPK_H
#define ARTOPK_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct artopk_ctx artopk_ctx;

enum {
  ARTOPK_OK = 0,
  ARTOPK_EINVAL = -1, /* bad argument; nothing enqueued                        */
  ARTOPK_ENOMEM = -2, /* device allocation failed in artopk_create             */
  ARTOPK_EHIP = -3,   /* a HIP runtime call failed; see artopk_last_error      */
  ARTOPK_ESTATE = -4  /* a kernel reported an internal inconsistency           */
};

/* Leader rule (Sec. III-B).  FIXED takes the leader from the caller.  VAR uses
 * the population variance of the dense error-fed vector.  VAR_TOPK is Alg. 1
 * taken literally: every worker runs Top-k on its own vector and the worker
 * whose k values have the largest squared norm leads (first maximum); its
 * cost is W selections instead of one.  VAR_G reads "largest gradient
 * variance" as the variance of the raw gradient g_w, before the residual is
 * added; everything else is as in VAR (same kernels, same cost).
 * STAR_COUNTER is the round-robin rule of STAR with the iteration counter kept
 * in the context's device memory: leader = counter mod W, and every step (every
 * replay of a recorded one) advances the counter by one.  The leader is then
 * not known to the host, so the step takes the route of the variance rules
 * (every worker's pass prepares the selection) without their statistics. */
enum {
  ARTOPK_STAR = 0, ARTOPK_VAR = 1, ARTOPK_FIXED = 2, ARTOPK_VAR_TOPK = 3, ARTOPK_VAR_G = 4,
  ARTOPK_STAR_COUNTER = 5
};

/* Element type of the gradients handed to artopk_step_g16. */
enum { ARTOPK_G_F32 = 0, ARTOPK_G_BF16 = 1, ARTOPK_G_F16 = 2 };

#define ARTOPK_MAX_WORKERS 64

/* Stages whose duration artopk_get_profile() reports (milliseconds).  With the
 * leader known up front (STAR / FIXED) the step runs the leader's
 * pass and the selection first and then ONE fused pass over the other W-1
 * workers; that pass is reported as ARTOPK_PROF_GATHER. */
enum {
  ARTOPK_PROF_PASS_A = 0, /* fused EF add + variance partials + histograms
                             (VAR: all workers; leader known: the leader only)  */
  ARTOPK_PROF_SELECT = 1, /* everything between pass A and the final idx       */
  ARTOPK_PROF_GATHER = 2, /* VAR: gather + ordered sum + residual zeroing;
                             leader known: fused EF add + gather + zeroing of
                             the W-1 other workers                              */
  ARTOPK_PROF_UPDATE = 3, /* (leader zeroing, ordered sum,) dense update fill  */
  ARTOPK_PROF_TOTAL = 4,  /* whole call                                        */
  ARTOPK_PROF_COUNT = 5
};

/*
 * Create a context bound to `hip_stream` (a hipStream_t; NULL = the default
 * stream) on the current device and allocate its scratch for problems up to
 * max_w workers, max_n elements, max_k kept entries and max_segments segments.
 * *out is set only on success.  A context serialises nothing by itself: calls
 * on one context must not overlap (its scratch is shared between them), and
 * all of them are enqueued on the one stream it was created with.  Scratch size: about 16.4 MiB per worker plus
 * 64 KiB per segment plus
 * 8 (max_k + max(max_n / 8, 2^22)) bytes of survivor list plus 8 max_w max_k bytes plus
 * max_n / 8 bytes per worker of survivor bit masks plus 1.5 max_n bytes in which a
 * leader's fused pass stages list entries tile by tile.  The library reads no environment
 * variable and keeps no state outside its contexts (artopk_variance_static's fixed
 * scratch excepted, see there).
 */
int artopk_create(artopk_ctx** out, int32_t max_w, int64_t max_n, int64_t max_k,
                  int32_t max_segments, void* hip_stream);

/*
 * Bytes of device memory that artopk_create would allocate for these limits (host
 * arithmetic only: no device is touched), or -1 if artopk_create would refuse them.
 */
int64_t artopk_scratch_bytes(int32_t max_w, int64_t max_n, int64_t max_k, int32_t max_segments);

/*
 * Switches between routes that give identical results (for tests and tuning; the
 * defaults are what the measurements chose).  Takes effect from the next call on
 * the context.  ARTOPK_EINVAL for an unknown key or a value outside its range.
 *   ARTOPK_OPT_GUESS_MIN_N        shortest flat vector that gets the sampled
 *                                 threshold guess before its fused pass (and
 *                                 shortest segmented vector whose fused pass
 *                                 walks the tiles in the same striding order);
 *                                 1 .. 2^31 (2^31 = never), default 33554432
 *   ARTOPK_OPT_UPDATE_TILES_MIN_N shortest vector whose dense update is
 *                                 streamed tile by tile with the values stored
 *                                 behind the zeros, shorter ones are built
 *                                 chunk by chunk in on-chip memory; 1 .. 2^31,
 *                                 default 4194304
 *   ARTOPK_OPT_LEADER_FIRST       1 (default): with a leader known up front run
 *                                 its pass and the selection first, then one
 *                                 fused pass over the other workers; 0: the
 *                                 fused pass over all workers first and an
 *                                 entry-by-entry gather, as under the variance rule
 *   ARTOPK_OPT_NONTEMPORAL        1 (default): non-temporal loads and stores in
 *                                 the streaming passes; 0: ordinary ones
 *   ARTOPK_OPT_STAGE_TILES        on the guess route with a leader known up
 *                                 front, the leader's fused pass can hand the
 *                                 elements that reach the guessed bound on as
 *                                 list entries, tile by tile, instead of leaving
 *                                 only the bit mask (from which the list is
 *                                 built by fetching the marked values one by
 *                                 one).  1 (default): for selections of one
 *                                 element in 256 or denser (beyond one in 32
 *                                 the alternative is the histogram route);
 *                                 2: for every selection; 0: never
 */
enum {
  ARTOPK_OPT_GUESS_MIN_N = 0,
  ARTOPK_OPT_UPDATE_TILES_MIN_N = 1,
  ARTOPK_OPT_LEADER_FIRST = 2,
  ARTOPK_OPT_NONTEMPORAL = 3,
  ARTOPK_OPT_STAGE_TILES = 4
};
int artopk_set_option(artopk_ctx* ctx, int32_t key, int64_t value);
int artopk_get_option(const artopk_ctx* ctx, int32_t key, int64_t* value_out);

/* Free the scratch.  The caller must have synchronised the stream. */
int artopk_destroy(artopk_ctx* ctx);

/* Text of the last error on this context (never NULL); with ctx = NULL the text of the
 * calling thread's last failed call that takes no context. */
const char* artopk_last_error(const artopk_ctx* ctx);

/*
 * Synchronise the context's stream and report whether any kernel since the
 * last call flagged an internal error (ARTOPK_ESTATE) -- e.g. a bounded wait
 * that expired.  Returns ARTOPK_OK otherwise.  The error word is sticky: while it
 * is set the selection kernels of later calls return at once, so every output
 * produced between the failing kernel and the artopk_status call that reports
 * (and clears) it is unspecified.
 */
int artopk_status(artopk_ctx* ctx);

/*
 * Per-worker variance used by the VAR-Topk leader rule (Sec. III-B; Alg. 1,
 * worker-selection branch): population variance (divide by N) of each of the W
 * vectors, accumulated in float64.
 *   x          host array of W device pointers, each N float32 (read only)
 *   var_out    device, W float64
 *   argmax_out device int32, lowest w attaining the maximum; may be NULL
 */
int artopk_variance(artopk_ctx* ctx, const float* const* x, int32_t w, int64_t n,
                    double* var_out, int32_t* argmax_out);

/*
 * artopk_variance for callers that cannot allocate device memory: code that is being
 * recorded into a HIP graph, tight serving loops, harnesses that forbid hipMalloc.  It
 * takes no context (creating one allocates): its kernels' scratch -- the per-block
 * partial results, 1.5 MiB -- is a fixed array inside the library's device code, which
 * every GPU the library runs on holds until the process ends.  The call allocates and
 * frees nothing, on the device or through any library.  Limits: 1 <= W <=
 * ARTOPK_MAX_WORKERS (what the fixed array holds) and 1 <= N < 2^31; anything beyond is
 * ARTOPK_EINVAL with nothing enqueued (text: artopk_last_error(NULL)).
 *   x, var_out, argmax_out   as for artopk_variance; results are the same bits
 *   hip_stream               the hipStream_t to enqueue on (NULL = the default stream)
 * All calls on one GPU share that GPU's array, whatever their stream: calls whose
 * kernels may overlap on one GPU race and must be ordered by the caller.  Nothing in
 * the array needs clearing between calls (every word read is written first).
 */
int artopk_variance_static(const float* const* x, int32_t w, int64_t n, double* var_out,
                           int32_t* argmax_out, void* hip_stream);

/*
 * Exact Top-k by magnitude (Sec. II-C "largest k%", Sec. III-A, Alg. 1 Topk).
 *   acc      device, N float32 (read only)
 *   nseg     number of segments; 1 with seg_off = seg_k = NULL selects k
 *            entries of the whole vector
 *   seg_off  host, nseg+1 int64, ascending, seg_off[0] = 0, seg_off[nseg] = N
 *   seg_k    host, nseg int64, 1 <= seg_k[s] <= size of segment s; their sum
 *            must equal k
 *   idx_out  device, k int32: global indices, ascending
 */
int artopk_select_topk(artopk_ctx* ctx, const float* acc, int64_t n, int32_t nseg,
                       const int64_t* seg_off, const int64_t* seg_k, int64_t k,
                       int32_t* idx_out);

/*
 * Gather every worker's values at the shared indices and add them in worker
 * order 0..W-1 in float32 (Alg. 1: G[ix] on every worker, then AllReduce).
 *   acc      host array of W device pointers, each N float32 (read only)
 *   idx      device, k int32, ascending, each in [0, N)
 *   vals_out device, W*k float32 row-major [w][m]; may be NULL
 *   sum_out  device, k float32
 */
int artopk_gather_sum(artopk_ctx* ctx, const float* const* acc, int32_t w, int64_t n,
                      const int32_t* idx, int64_t k, float* vals_out, float* sum_out);

/*
 * Residual rewrite and dense update (Alg. 1: residual = G - g~, and the update
 * that consumes the reduced values; second EF equation of Sec. II-C).
 *   residual host array of W device pointers; each holds acc_w on entry and on
 *            exit differs only at the idx positions, which become +0.0
 *   idx      device, k int32, strictly ascending, each in [0, N) (as the
 *            selection writes them); a list that is not leaves update
 *            unspecified and is reported by artopk_status as ARTOPK_ESTATE
 *            where a kernel notices it
 *   sum      device, k float32
 *   update   device, N float32, fully overwritten: zeros, and sum[m] at idx[m]
 */
int artopk_scatter_residual(artopk_ctx* ctx, float* const* residual, int32_t w, int64_t n,
                            const int32_t* idx, int64_t k, const float* sum, float* update);

/*
 * One whole step (Alg. 1 loop body for all W workers).
 *   g            host array of W device pointers, N float32 each, read only
 *   residual     host array of W device pointers, N float32 each, updated in
 *                place (holds residual_{i-1} on entry, residual_i on exit)
 *   nseg/seg_off/seg_k/k  as in artopk_select_topk (one leader per step even
 *                when the selection is per segment)
 *   mode         ARTOPK_STAR (leader = step mod W), ARTOPK_VAR, ARTOPK_FIXED,
 *                ARTOPK_VAR_TOPK, ARTOPK_VAR_G or ARTOPK_STAR_COUNTER (see the enum)
 *   step         the paper's iteration counter i (ignored by ARTOPK_STAR_COUNTER,
 *                which counts on the device: artopk_set_step_counter)
 *   fixed_leader used by ARTOPK_FIXED only
 *   leader_out   device int32 (may be NULL)
 *   var_out      device W float64 (may be NULL): the per-worker variances in VAR
 *                mode, the squared norms of each worker's own Top-k values in
 *                VAR_TOPK mode; untouched otherwise
 *   idx_out      device k int32
 *   vals_out     device W*k float32 (may be NULL)
 *   sum_out      device k float32
 *   update_out   device N float32 (may be NULL: the dense update is then not
 *                written, for callers that take (idx_out, sum_out) to
 *                artopk_apply_update instead)
 * The call only enqueues kernels on the context's stream: it allocates nothing,
 * issues no memset and does not synchronise (a segmented layout is copied to
 * the device the first time it is seen, so make one call with it before
 * recording).  With stage timing off it can therefore be recorded into a HIP
 * graph and replayed; in VAR mode the leader is taken on the device at every
 * replay, in STAR / FIXED mode the recorded leader is replayed, and in
 * STAR_COUNTER mode every replay takes the next leader of the round.
 */
int artopk_step(artopk_ctx* ctx, const float* const* g, float* const* residual, int32_t w,
                int64_t n, int32_t nseg, const int64_t* seg_off, const int64_t* seg_k,
                int64_t k, int32_t mode, uint64_t step, int32_t fixed_leader,
                int32_t* leader_out, double* var_out, int32_t* idx_out, float* vals_out,
                float* sum_out, float* update_out);

/*
 * Sets the iteration counter that ARTOPK_STAR_COUNTER steps read and advance
 * (Alg. 1, STAR branch: leader = i mod W).  A new context starts at 0.  The
 * value is written by a kernel on the context's stream, in order with the
 * steps around it; nothing is allocated or synchronised.
 */
int artopk_set_step_counter(artopk_ctx* ctx, uint64_t value);

/*
 * artopk_step for gradients stored in 16 bits (the residual, and everything
 * derived from it, stays float32: the error-feedback state of Sec. II-C must
 * not lose what compression leaves behind).  Each gradient value is widened
 * exactly to float32 -- bfloat16: its bits become the upper half of the
 * float32; float16: the IEEE conversion, subnormals included -- and the step is
 * then the one artopk_step defines, bit for bit.  The fused pass reads 2 bytes
 * per gradient element instead of 4.
 *   g       host array of W device pointers, each N 16-bit elements, 8-byte aligned
 *   g_type  ARTOPK_G_BF16 or ARTOPK_G_F16
 * All other arguments, outputs and errors as for artopk_step.
 */
int artopk_step_g16(artopk_ctx* ctx, const void* const* g, int32_t g_type, float* const* residual,
                    int32_t w, int64_t n, int32_t nseg, const int64_t* seg_off,
                    const int64_t* seg_k, int64_t k, int32_t mode, uint64_t step,
                    int32_t fixed_leader, int32_t* leader_out, double* var_out, int32_t* idx_out,
                    float* vals_out, float* sum_out, float* update_out);

/*
 * Every worker's own exact Top-k (Alg. 1 calls Topk on each worker before the
 * leader is chosen; the AllGather exchange of Sec. II-C sends exactly these
 * values and indices).  Same ordering rules as artopk_select_topk.
 *   acc        host array of W device pointers, each N float32 (read only)
 *   idx_out    device W*k int32 row-major [w][m], each row ascending
 *   vals_out   device W*k float32, vals_out[w][m] = acc_w[idx_out[w][m]]; may be NULL
 *   sqnorm_out device W float64, sum of squares of each worker's k values
 *              (the quantity Alg. 1 writes for the VAR leader); may be NULL
 *   argmax_out device int32, first worker with the largest squared norm; may be NULL
 */
int artopk_topk_workers(artopk_ctx* ctx, const float* const* acc, int32_t w, int64_t n, int64_t k,
                        int32_t* idx_out, float* vals_out, double* sqnorm_out, int32_t* argmax_out);

/*
 * Compression gain of every worker for the step just taken (the heuristic the
 * paper quotes in Sec. II-C, "Statistical Efficiency in Gradient Compression":
 * ||g_c||^2 / ||g_e||^2 with g_e the error-fed and g_c the compressed gradient).
 * Because g_e = g_c + residual with disjoint supports, it is computed from the
 * step's outputs as V / (V + R), V = sum vals_w^2, R = sum residual_w^2, in
 * float64.  Reads 4*W*N + 4*W*k bytes.
 *   residual host array of W device pointers: the residuals AFTER artopk_step
 *   vals     device W*k float32, the step's vals_out
 *   gain_out device W float64
 */
int artopk_compression_gain(artopk_ctx* ctx, const float* const* residual, int32_t w, int64_t n,
                            const float* vals, int64_t k, double* gain_out);

/*
 * Sparse form of the model update of Alg. 1 (w <- w - eta * g~): only the k
 * reduced positions change, weights[idx[m]] -= eta * sum[m] in float32 (one
 * multiply, one subtract).  A caller that applies the update this way does not
 * need the dense update_out of artopk_step.
 *   weights device N float32, updated in place; idx, sum as produced by the step
 */
int artopk_apply_update(artopk_ctx* ctx, float* weights, int64_t n, const int32_t* idx,
                        const float* sum, int64_t k, float eta);

/*
 * Stage timing.  enable = 1 records two HIP events on the context's stream
 * directly around the launch of the dominant kernel of every artopk_step (the
 * fused pass over all workers, reported as PASS_A; or, when the leader is known
 * up front, the fused pass over the other workers, reported as GATHER) and
 * nothing else; enable = 2 records an event at every stage boundary; 0
 * switches it off.  artopk_get_profile synchronises the stream and writes up
 * to `count` stage durations in milliseconds (order: the ARTOPK_PROF_* enum;
 * stages that did not run, or were not bracketed, report 0), each averaged
 * over the calls made since profiling was enabled (at most the 64 most recent).
 */
int artopk_set_profile(artopk_ctx* ctx, int32_t enable);
int artopk_get_profile(artopk_ctx* ctx, float* ms_out, int32_t count);

/*
 * How the last artopk_step ran its selection (Sec. III-B leaves the Top-k
 * method open; this only reports which of the library's equivalent routes was
 * taken, for tests and tuning).  Synchronises the stream and writes up to
 * `count` host int32 values:
 *   [0] 1 if the step sampled a threshold guess before its fused pass
 *   [1] 1 if the survivor list was then written from the fused pass' bit mask
 *       (0 with [0] = 1: the guess did not hold and the full route was taken)
 *   [2] entries in the survivor list
 *   [3] 1 if the list was written after the first radix digit (or from the
 *       mask), 0 if that did not fit and the deeper array passes wrote it
 *   [4] workers the dominant streaming kernel covered (W, or W-1 when the
 *       leader is known up front)
 * Flat (one-segment) steps only; segmented steps report [0] = [1] = 0.
 */
int artopk_select_info(artopk_ctx* ctx, int32_t* info_out, int32_t count);

/* Library version, major*10000 + minor*100 + patch. */
int32_t artopk_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ARTOPK_H */
