/*
 * rps.h -- C ABI of the MI355X (gfx950) library for the lossy partitioned
 * model-averaging round of RPS, the algorithm of "Distributed Learning over
 * Unreliable Networks" (arXiv 1810.07766), simulated for n workers held as one
 * [n, N] array on a single GPU.
 *
 * One round (Alg. 1 of the paper):
 *   1. local SGD step           v_i = x_i - gamma * g_i                (Sec. 4.1; Alg. 1 steps 3-5)
 *   2. partition                every v_i is cut into the same n blocks (Sec. 4.1 eq. (dividev))
 *   3. Reduce-Scatter w/ drops  the server b(j) of block j averages the copies of block j that
 *                               reach it; each copy is lost independently with probability p,
 *                               the server's own copy never is        (Sec. 3; Sec. 4.1 RS step;
 *                                                                      supplement, Lemma 7 proof)
 *   4. All-Gather w/ drops      worker i overwrites block j with that average iff the reply
 *                               reaches it (lost with probability p), else keeps v_i's block
 *                                                                     (Sec. 4.1 AG step, eq. (dividex))
 * The server b(j) is a fresh uniform permutation every round (Alg. 1 step 6).
 *
 * Conventions
 *   - X and G are CALLER-OWNED DEVICE memory: contiguous row-major [n, N] (worker-major), fp32
 *     or bf16 -- or tile-major, see RPS_FLAG_LAYOUT_TILED.  The library never allocates, frees or
 *     keeps them.  A 16-byte aligned base with N % 4 == 0 (fp32) or N % 8 == 0 (bf16; any N in
 *     the tiled layout) takes the 128-bit load/store path; anything else is handled by a slower
 *     element-wise path with identical results.
 *   - All device work is enqueued on the HIP stream given at creation; no call synchronises
 *     except where stated.  Results are valid in stream order.  rps_local_step, rps_lossy_average,
 *     rps_round, rps_round_gradient_averaging and rps_convert_layout enqueue kernels only (no
 *     allocation, no synchronisation, no memset): a caller may capture them in a HIP graph; the
 *     `step` argument is then part of the captured launch.  Launches recorded during capture draw
 *     the network outcome of their step into a table of their own that no eager call uses, so
 *     replays and eager calls may be mixed in any order on the context's stream and every call
 *     still sees the outcome of exactly (seed, its step) (Alg. 1 steps 6-7).  A captured launch
 *     always uses the generated outcome: capturing while a mask override is in force returns
 *     RPS_EUNSUPPORTED (nothing is recorded), and an override set later does not reach a graph.
 *   - Every function returns RPS_OK (0) or a negative error code; nothing aborts or throws.
 *     An error detected before launch leaves X untouched.
 *   - The round's randomness is a pure function of (seed, step): the caller supplies `step`,
 *     so a run can be checkpointed and resumed by storing (X, step).  step < 2^56.
 *   - A context is not thread-safe; distinct contexts are independent.
 */
#ifndef RPS_H
#define RPS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rps_ctx rps_ctx;

enum {
    RPS_OK = 0,
    RPS_EINVAL = -1,        /* bad argument (see each function) */
    RPS_ENOMEM = -2,        /* host or device allocation failed */
    RPS_EHIP = -3,          /* a HIP call failed; see rps_last_hip_error() */
    RPS_EUNSUPPORTED = -4,  /* valid request this build does not implement (a forced network outcome
                               inside a stream capture) */
    RPS_ETOOBIG = -5        /* rps_consensus_static: n or N beyond the maximum its fixed scratch serves */
};

enum { RPS_DTYPE_F32 = 0, RPS_DTYPE_BF16 = 1 };

/* rps_create flags */
enum {
    /* Worker j serves block j in every round: the simplification the paper uses when it
       explains the algorithm (Sec. 4.1).  Default is Alg. 1's per-round random permutation. */
    RPS_FLAG_SERVER_IDENTITY = 1u,
    /* X and G are stored tile-major instead of row-major: the model is cut into tiles of
       RPS_TILE_BYTES per worker (32 fp32 or 64 bf16 columns) and the n workers' segments of a
       tile are adjacent, i.e. element (worker i, column c) lives at ((c / T) * n + i) * T + c % T
       with T = RPS_TILE_BYTES / sizeof(element).  The array holds ceil(N / T) * n * T elements
       (rps_storage_elems); the columns of the last tile beyond N are padding that is never read
       or written.  All n values of a column then sit within n * 128 bytes of each other, and a
       round streams through memory in address order, reading only a few KB before it writes
       them back -- measured 19 % faster than row-major on the benchmark's headline workload.
       Results are those of the row-major layout up to the summation order of the fp64 column
       sums (still fixed, and the same for every receiver of a block).  Worker i's model is the
       strided view [:, i, :].  Every entry point accepts either layout; not available with
       external servers. */
    RPS_FLAG_LAYOUT_TILED = 2u
};

#define RPS_TILE_BYTES 128

/* Number of elements an X or G array must hold for n workers, N columns, the dtype and the
   layout chosen by `flags` (n * N for row-major).  Returns -1 for invalid arguments. */
int64_t rps_storage_elems(int32_t n, int64_t N, int32_t dtype, uint32_t flags);

/*
 * Create a context for n workers with N parameters each (problem statement, Sec. 3; inputs
 * of Alg. 1: step size gamma; the network is characterised by n and the drop probability p).
 *   out            receives the handle (host pointer; untouched on error)
 *   n              workers = blocks = servers, 1..64
 *   N              parameters per worker, n <= N <= 2^34
 *   block_offsets  HOST array of n+1 int64 with off[0] = 0 < off[1] < ... < off[n] = N, block j
 *                  being columns [off[j], off[j+1]); or NULL for the paper's equally-sized
 *                  blocks, which needs N % n == 0.  Copied; the caller keeps ownership.
 *   p              drop probability of every worker<->server message, 0 <= p <= 1
 *   gamma          step size of the local SGD step
 *   seed           64-bit key of the counter-based random numbers
 *   dtype          RPS_DTYPE_F32 or RPS_DTYPE_BF16 (storage; arithmetic is fp32, sums fp64)
 *   flags          RPS_FLAG_* (server assignment, storage layout)
 *   hip_stream     hipStream_t on which all work is enqueued (NULL = the default stream)
 * Allocates a fixed ~100 KB of device memory -- six tables of the O(n^2) delivery bits packed as one
 * 64-bit word per block and direction (3 KB each: two for eager calls, one each for queries, stream
 * capture, a forced outcome and the outcome "nothing arrives"), 32 KB of reduction scratch for rps_consensus / rps_estimate_mixing,
 * 48 KB of noise cells for the synthetic gradient -- and two pinned host staging buffers (3 KB,
 * 16 KB); nothing proportional to N.  Errors: RPS_EINVAL, RPS_ENOMEM, RPS_EHIP.
 */
int rps_create(rps_ctx **out, int32_t n, int64_t N, const int64_t *block_offsets, double p,
               float gamma, uint64_t seed, int32_t dtype, uint32_t flags, void *hip_stream);

/*
 * Same, for `servers` external parameter servers that are not workers (the paper's Fig. 1
 * draws three servers and four workers and notes that the analysis extends to any numbers):
 * the model is cut into `servers` blocks (1..64; block_offsets has servers+1 entries, or NULL
 * for equal blocks with N % servers == 0), every one of the n x servers uplinks and downlinks
 * is lossy -- there is no reliable self link -- and a server that received no copy sends
 * nothing, so every worker keeps its v for that block (the paper does not treat this case).
 * Masks of such a context are [worker * servers + block]; rps_get_masks reports server = -1.
 */
int rps_create_external(rps_ctx **out, int32_t n, int32_t servers, int64_t N, const int64_t *block_offsets,
                        double p, float gamma, uint64_t seed, int32_t dtype, void *hip_stream);

/* End of a run (Alg. 1's output is the workers' models, which stay in the caller's X): frees the
   context's tables.  Synchronises the stream first.  NULL is a no-op. */
int rps_destroy(rps_ctx *ctx);

/*
 * Synthetic stochastic gradient used when G == NULL:  g = weight_decay * x + sigma * z, with z
 * standard Gaussian noise generated in registers from (seed, step, worker, column).  Stands in
 * for Alg. 1 steps 3-4 (sampling data and computing a stochastic gradient).  Default 0, 0.
 * A change of sigma rewrites the context's 16 KB device table of noise radii (sigma * r) in
 * stream order and synchronises the stream; not to be called during a stream capture.
 */
int rps_set_synthetic_grad(rps_ctx *ctx, float sigma, float weight_decay);

/*
 * Row-major layout only: the rows of X and G (one worker's model each, Sec. 4.1) are `pitch` elements
 * apart instead of N (N <= pitch <= 2^35), i.e. element (worker i, column c) lives at i * pitch + c and
 * the pitch - N elements after every row are padding that is never read or written.  Applies to every
 * following call.  Why one would: a wavefront reads the same columns of all n rows at once, and when
 * the row size is a multiple of 32 KB those n addresses fall on the same memory channel (measured at
 * n = 8, N = 2^22 fp32 with a gradient buffer: 0.60-0.65 of the HBM peak at pitch = N, 0.72 at
 * rps_recommended_row_pitch).  A pitch that is a multiple of 16 bytes keeps the 128-bit path.
 * RPS_EINVAL for a tiled context or a pitch out of range.
 */
int rps_set_row_pitch(rps_ctx *ctx, int64_t pitch);

/* Smallest pitch >= N (in elements) whose size in bytes is 4 KB past a multiple of 64 KB; -1 for
   invalid arguments. */
int64_t rps_recommended_row_pitch(int64_t N, int32_t dtype);

/* Change the step size (the paper notes a decayed step size reaches a critical point, Sec. 5). */
int rps_set_gamma(rps_ctx *ctx, float gamma);

/*
 * Local SGD step (Sec. 4.1; Alg. 1 step 5), in place:  X <- X - gamma * G.
 *   X   device [n, N], context dtype
 *   G   device [n, N], same dtype; or NULL for the synthetic gradient
 * v is rounded to the storage dtype (what is stored is what would travel).
 */
int rps_local_step(rps_ctx *ctx, void *X, const void *G, uint64_t step);

/*
 * One Reduce-Scatter + All-Gather round with drops (Sec. 4.1; Alg. 1 steps 6-8), in place on
 * the intermediate models V held in X, with the network outcome of (seed, step) or the
 * override set by rps_set_mask_override.  Rows whose reply was lost are left untouched.
 */
int rps_lossy_average(rps_ctx *ctx, void *X, uint64_t step);

/*
 * Fused round -- one iteration of Alg. 1 (steps 3-8; Sec. 4.1: local step, Reduce-Scatter and
 * All-Gather with drops) for all n workers: same result, bit for bit, as rps_local_step followed by
 * rps_lossy_average, in one pass over X (each element read at most once and written once).
 * Arguments as for those two calls.
 */
int rps_round(rps_ctx *ctx, void *X, const void *G, uint64_t step);

/*
 * Gradient averaging under loss -- the comparison the paper runs in Sec. 6 (averaging gradients
 * instead of models under message drops converges worse): the Reduce-Scatter / All-Gather with
 * drops of (seed, step) is applied to G instead of V, then every worker takes its local step with
 * what it holds:   x'[i] = x[i] - gamma * (reply for block j reached i ? average of the gradient
 * copies that reached the server : its own g[i]),  the average rounded to the storage dtype.
 *   X   device [n, N], updated in place;   G   device [n, N] (required), read only
 * Worker models drift apart under this scheme (nothing ever pulls them together again), which
 * rps_consensus makes visible.
 */
int rps_round_gradient_averaging(rps_ctx *ctx, void *X, const void *G, uint64_t step);

/*
 * Test hook: the network outcome (Sec. 3: every message between a worker and a server is lost
 * independently with probability p; Alg. 1 step 6: the servers are a fresh uniform permutation of
 * the workers) that the DEVICE generates for `step`, copied to HOST arrays.
 *   up, down   n*B bytes each (B = number of blocks), index [worker * B + block]; 1 = delivered
 *   server     B int32, server[j] = worker that averages block j (-1: external server)
 * Any pointer may be NULL.  Ignores a mask override.  Synchronises the stream.
 */
int rps_get_masks(rps_ctx *ctx, uint64_t step, uint8_t *up, uint8_t *down, int32_t *server);

/*
 * The same outcome computed on the HOST by the library's own host copy of the generator (no GPU, no
 * context; same specification as the device kernel, separate code): what rps_get_masks must return
 * for a context created with these n, p, seed and flags -- or, with servers > 0, for an
 * rps_create_external context with that many servers (flags must then be 0; servers = 0 means the
 * workers are the servers).  Output arrays as in rps_get_masks; any may be NULL.
 * Errors: RPS_EINVAL (n or servers outside 1..64, p outside [0, 1], step >= 2^56, unknown flags).
 */
int rps_masks_host(int32_t n, int32_t servers, double p, uint64_t seed, uint32_t flags, uint64_t step, uint8_t *up,
                   uint8_t *down, int32_t *server);

/*
 * Test hook: force the network outcome of every following round -- any pattern of lost messages the
 * network model of Sec. 3 allows, e.g. every uplink lost, or one worker cut off (HOST arrays, layout as in
 * rps_get_masks; copied).  Every block must have at least one delivered uplink (a server
 * always holds its own copy).  Passing all three NULL restores the generated masks.
 * Synchronises the stream.
 */
int rps_set_mask_override(rps_ctx *ctx, const uint8_t *up, const uint8_t *down, const int32_t *server);

/*
 * Consensus statistics of the state in one streaming read of X (supplement, Lemma 1: the
 * disagreement sum_i ||x_i - xbar||^2 = ||X (I - A_n)||_F^2 that the convergence proof bounds):
 *   distance  HOST double, receives sum over workers of ||x_i - xbar||^2   (may be NULL)
 *   mean_sq   HOST double, receives ||xbar||^2, xbar = (1/n) sum_i x_i       (may be NULL)
 * fp64 accumulation in a fixed order (deterministic).  Uses a fixed 32 KB reduction scratch
 * allocated by rps_create.  Synchronises the stream.
 */
int rps_consensus(rps_ctx *ctx, const void *X, double *distance, double *mean_sq);

/*
 * rps_consensus for callers that cannot allocate or synchronise: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Needs no context; calls no hipMalloc / hipFree or
 * any allocating routine, does not synchronise, and only enqueues kernels on `hip_stream`.
 *   X           device array of n workers x N columns, dtype and layout (flags: 0 or
 *               RPS_FLAG_LAYOUT_TILED) as for rps_consensus; caller-owned, read only
 *   out         DEVICE array of 2 doubles, caller-owned: out[0] receives sum_i ||x_i - xbar||^2,
 *               out[1] receives ||xbar||^2, valid in stream order.  Same kernels, same fixed
 *               reduction order and therefore the same bits as rps_consensus.
 *   hip_stream  hipStream_t to enqueue on (NULL = the default stream)
 * The per-workgroup partial sums go to a reduction scratch that is part of the library's code
 * object: a fixed 32 KB (2 x 2048 doubles) on every GPU the library runs on, held until the process
 * ends.  It serves 1 <= n <= 64 and 1 <= N <= 2^34; anything larger is rejected with RPS_ETOOBIG
 * before anything is enqueued.  Every call on a GPU shares that GPU's scratch (each call overwrites
 * all the entries it later reads, so nothing needs clearing): calls whose kernels may overlap on one
 * GPU -- different streams, concurrent graph launches -- race and must be ordered by the caller.
 * The first call on a GPU (or rps_create on it) looks up the scratch's device address; do that once
 * outside a capture.  Errors: RPS_EINVAL (NULL or non-device X, bad dtype / flags / sizes),
 * RPS_ETOOBIG, RPS_EHIP.
 */
int rps_consensus_static(const void *X, int32_t n, int64_t N, int32_t dtype, uint32_t flags, double *out,
                         void *hip_stream);

/*
 * Monte-Carlo estimate of the constants alpha1 and alpha2 of the mixing matrix W_t of
 * X_{t+1} = V_t W_t (Sec. 4.2, eqs. (def_alpha1), (def_alpha2):  E[W W^T] = alpha1 I + (1-alpha1) A_n,
 * E[W A_n W^T] = alpha2 I + (1-alpha2) A_n;  Fig. 2 plots alpha2 and Fig. 3 beta = alpha1 - alpha2 over
 * n and p) from the network outcomes the device generates for the `rounds` steps starting at
 * first_step (every block of every round is one sample of W; no model data is touched):
 *   alpha1 = (n e1 - 1)/(n - 1),  e1 = mean over samples and rows m of sum_k W_mk^2     (supplement, Lemma 7)
 *   alpha2 = (e2 - 1)/(n - 1),    e2 = mean over samples and rows m of (sum_k W_mk)^2   (supplement, Lemma 8)
 *   alpha1, alpha2   HOST doubles (either may be NULL);   1 <= rounds <= 2^24;   n >= 2
 * Ignores a mask override.  fp64, fixed summation order (deterministic).  Uses the context's
 * reduction scratch; synchronises the stream.  Errors: RPS_EINVAL, RPS_EHIP.
 */
int rps_estimate_mixing(rps_ctx *ctx, uint64_t first_step, int64_t rounds, double *alpha1, double *alpha2);

/*
 * Copy the state between the two layouts (any context of matching n, N and dtype; its own layout
 * flag does not matter):  to_tiled != 0: src is row-major [n, N], dst receives the tile-major
 * arrangement (rps_storage_elems elements; padding columns are written as zeros);  to_tiled == 0:
 * the reverse.  The row-major side has the context's row pitch (rps_set_row_pitch; N by default).  dst and src are device arrays that must not overlap.  One streaming pass, enqueued
 * on the context's stream.
 */
int rps_convert_layout(rps_ctx *ctx, void *dst, const void *src, int32_t to_tiled);

/*
 * Launch shape of the round kernel, for tuning sweeps; results never depend on it.
 *   rows_in_flight       rows per load chunk (a wavefront keeps two chunks in flight): 2 or 4
 *   waves_per_workgroup  1..16 (a workgroup's wavefronts own adjacent tiles and, with the
 *                        in-register gradient, share one LDS copy of the noise cells); rounded up to
 *                        the nearest width the kernel in question is built for (in-register
 *                        gradient: 4, 8, 12, 14 tile-major and 2, 4, 8 row-major; otherwise 1, or
 *                        4 row-major; always 8 for fp32 tile-major with 57 or more workers, where
 *                        pairs of wavefronts share a tile)
 *   max_waves_per_cu     cap on resident wavefronts per compute unit (0 = no cap); rounded down to whole
 *                        workgroups, and never below two workgroups (a workgroup holds at most 64 KB
 *                        of the compute unit's 160 KB of LDS); rps_query_occupancy shows the outcome
 *   tiles_per_wave       tiles a wavefront works through with the in-register gradient, 1..64
 *                        (0 = chosen per launch)
 * Until this is called every launch takes the measured best shape for its worker count, dtype
 * and gradient source (none / buffer / in-register).  RPS_EINVAL for other values.
 */
int rps_set_launch_tuning(rps_ctx *ctx, int32_t rows_in_flight, int32_t waves_per_workgroup,
                          int32_t max_waves_per_cu, int32_t tiles_per_wave);

/*
 * Test hook for the launch shape: how many wavefronts of the round kernel one compute unit can hold
 * with the launch shape this context would use for the given gradient source (0 = none, i.e.
 * rps_lossy_average; 1 = gradient buffer; 2 = in-register gradient) -- the answer of the HIP
 * runtime's occupancy calculator for that kernel, its workgroup size and the LDS it is launched
 * with.  Nothing is launched.  The library caps occupancy through an LDS allocation it never touches
 * (max_waves_per_cu of rps_set_launch_tuning and the built-in defaults); this call lets a test
 * check that the cap arrives.  Errors: RPS_EINVAL, RPS_EHIP.
 */
int rps_query_occupancy(rps_ctx *ctx, int32_t gradient_source, int32_t *waves_per_cu);

/*
 * Test hook: the cell values of the synthetic gradient noise as the library computes them on the
 * host (no GPU needed): radius[4096] = sqrt(-2 ln((k + 1/2)/4096)), cos_sin[2 * 4096] = the
 * interleaved (cos, sin) of 2 pi (a + 1/2)/4096, each the nearest fp32.  HOST arrays.
 */
int rps_noise_cells(float *radius, float *cos_sin);

/*
 * Kernel timing for benchmarks: while enabled, every rps_round / rps_lossy_average /
 * rps_local_step / rps_round_gradient_averaging / rps_consensus / rps_convert_layout brackets its
 * kernel(s) (not the small mask kernel) with HIP events on the context's stream.  rps_get_kernel_time synchronises the stream, returns the accumulated
 * kernel milliseconds and launch count since enabling, and resets both.  At most 4096
 * launches are recorded between two reads.
 */
int rps_set_profiling(rps_ctx *ctx, int32_t enable);
int rps_get_kernel_time(rps_ctx *ctx, double *total_ms, int64_t *launches);
/* Same, per launch: ms[k] receives the duration of the k-th recorded launch (HOST array of `capacity`
   doubles; launches beyond it are counted in *launches but not stored). */
int rps_get_kernel_times(rps_ctx *ctx, double *ms, int64_t capacity, int64_t *launches);

/* hipError_t of the last failing HIP call in this context (0 = none); with ctx == NULL: of the last
   failing HIP call of this host thread that had no context yet (inside rps_create). */
int rps_last_hip_error(const rps_ctx *ctx);

/* Static description of an error code. */
const char *rps_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* RPS_H */
