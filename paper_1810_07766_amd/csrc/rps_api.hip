// C ABI of the RPS library (see include/rps.h for the contract of every entry point).
// Host-side only: argument validation, the O(n) device table, launches on the caller's stream.
#include "../../include/rps.h"
#include "rps_internal.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <utility>
#include <vector>

using rps::RoundParams;
using rps::RoundTable;

struct rps_ctx {
    int32_t n = 0;
    int32_t nb = 0;                   // blocks: n, or the number of external servers
    bool external = false;
    int64_t N = 0;
    int64_t pitch = 0;                // row-major: elements between consecutive workers' rows (>= N)
    double p = 0.0;
    uint64_t threshold = 0;     // a message is lost iff its hash word < threshold = floor(p 2^32)
    float gamma = 0.0f, sigma = 0.0f, lambda = 0.0f;
    uint64_t seed = 0;
    int32_t dtype = 0;
    uint32_t flags = 0;
    hipStream_t stream = nullptr;
    int device = 0;
    int64_t max_block_cols = 0;
    std::vector<int64_t> off;
    RoundTable *tab_base = nullptr;   // device allocation: six tables + the reduction scratch
    // The two tables of the eager calls: only launches that execute at once ever write them, so what
    // the host believes about them (cur_step / next_step) stays true whatever else happens.
    RoundTable *tab = nullptr;        // device: table the averaging kernels read (outcome of cur_step if cur_valid)
    RoundTable *tab_other = nullptr;  // device: outcome of next_step if next_valid, prepared by the previous kernel
    RoundTable *tab_query = nullptr;  // device: scratch table for rps_get_masks
    RoundTable *tab_capture = nullptr;   // device: the only table launches recorded during stream capture write and read
    RoundTable *tab_override = nullptr;  // device: the forced outcome of rps_set_mask_override
    RoundTable *tab_nothing = nullptr;   // device: the outcome "no message arrives" (all masks zero), never rewritten: with
                                         // it the round kernel performs exactly the local step
    bool cur_valid = false, next_valid = false;
    uint64_t cur_step = 0, next_step = 0;
    RoundTable *staging = nullptr;    // pinned host copy (create, override, query)
    double *partials = nullptr;       // device: 2 * kMaxPartials + 2 doubles (consensus reduction scratch + result)
    float *noise_cells = nullptr;     // device: sigma * radius[kNoiseGrid], then the (cos, sin) pairs of the angle cells
    float *radius_staging = nullptr;  // pinned host: sigma * radius on its way to the device
    bool override_on = false;
    bool profiling = false;
    std::vector<hipEvent_t> ev_start, ev_stop;
    size_t ev_used = 0;
    int last_hip = 0;
    bool tune_set = false;             // rps_set_launch_tuning was called: `tune` replaces the defaults
    rps::LaunchTuning tune{2, 1, 8, 0};
};

// Cell values of the synthetic gradient noise (a Box-Muller pair per hash word on a grid of
// kNoiseGrid radius cells x kNoiseGrid angle cells): the nearest fp32 to the real values, from
// 80-bit extended arithmetic (64-bit significand: far below half an fp32 ulp of error, so the
// rounding is the correct one wherever the real value is not within 1e-18 of a tie).
void rps::build_noise_cells(float *radius, float *cos_sin) {
    const long double grid = (long double)rps::kNoiseGrid;
    const long double two_pi = 6.283185307179586476925286766559005768L;
    for (int k = 0; k < rps::kNoiseGrid; ++k) {
        radius[k] = (float)sqrtl(-2.0L * logl(((long double)k + 0.5L) / grid));
        const long double phi = two_pi * (((long double)k + 0.5L) / grid);
        cos_sin[2 * k] = (float)cosl(phi);
        cos_sin[2 * k + 1] = (float)sinl(phi);
    }
}

namespace {

constexpr size_t kMaxProfiledLaunches = 4096;

// hipError_t of the last failing HIP call that had no context to record it in (rps_create,
// rps_consensus_static), per host thread.
thread_local int g_last_hip_without_ctx = 0;

int hip_fail(rps_ctx *ctx, hipError_t e) {
    if (ctx)
        ctx->last_hip = (int)e;
    else
        g_last_hip_without_ctx = (int)e;
    return RPS_EHIP;
}
#define RPS_HIP(ctx, call)                                  \
    do {                                                    \
        hipError_t e_ = (call);                             \
        if (e_ != hipSuccess) return hip_fail((ctx), e_);   \
    } while (0)

bool step_ok(uint64_t step) { return step < (1ull << 56); }

// Row-major launch shapes, from sweeps over rows per chunk, workgroup width and occupancy cap at 2-64
// workers in both dtypes and for each gradient source (fractions of the HBM peak in the comments).  The
// in-place update mixes n read streams with n write streams, and a wavefront's tile is n KB: the memory
// system handles that best with few wavefronts resident -- fewer still when a gradient buffer doubles
// the loads in flight -- but a compute unit wants some 40-70 KB in flight, so small n takes more of them.
rps::LaunchTuning default_tuning(int32_t n, int32_t dtype, int grad_mode) {
    const bool bf16 = dtype == RPS_DTYPE_BF16;
    if (grad_mode == rps::kGradNone) {
        // averaging alone: single wavefronts under a cap (fixed at 5 this ran at 0.59 instead of 0.86 at 4
        // workers, 0.71 / 0.85 at 6, 0.78 / 0.84 at 12); bf16 takes more from 32 workers on (n = 64 0.54 -> 0.63)
        if (n <= 2) return rps::LaunchTuning{2, 4, 0, 0};
        int cap = n <= 4 ? 12 : (n <= 7 ? 8 : (n <= 12 ? 6 : 5));
        if (bf16) cap = n >= 48 ? 12 : (n >= 32 ? 8 : std::max(cap, 6));
        return rps::LaunchTuning{4, 1, cap, 0};
    }
    if (grad_mode == rps::kGradBuffer) {
        if (n <= 2) return bf16 ? rps::LaunchTuning{2, 4, 0, 0} : rps::LaunchTuning{2, 1, 12, 0};   // 0.51-0.55 -> 0.82
        if (n <= 4) return rps::LaunchTuning{2, 1, n == 3 ? 12 : 8, 0};                             // 0.63-0.78 -> 0.81-0.82
        if (n < 12) return rps::LaunchTuning{2, 1, 6, 0};                                           // fp32 n = 8 0.72 -> 0.75
        if (bf16 && n >= 32) return rps::LaunchTuning{2, 4, 0, 0};                                  // n = 64 0.48 -> 0.60
        return rps::LaunchTuning{2, 1, 5, 0};
    }
    // in-register gradient: the workgroup's wavefronts share the LDS copy of the noise cells
    if (bf16) return n <= 4 ? rps::LaunchTuning{n <= 2 ? 2 : 4, 8, 0, 0} : rps::LaunchTuning{2, 4, 0, 0};   // n = 4 0.69 -> 0.73
    if (n <= 8) return rps::LaunchTuning{2, 8, n <= 3 ? 0 : 12, 0};   // n = 4 0.62 -> 0.77, n = 6 0.68 -> 0.77, n = 8 0.70 -> 0.72
    return n >= 24 ? rps::LaunchTuning{2, 2, 0, 0} : rps::LaunchTuning{4, 4, 12, 0};
}

// Tile-major launch shapes, from sweeps over 1-64 workers in both dtypes at equal state size (fractions of
// the HBM peak in the comments).  Two things decide: how many bytes a wavefront step covers (a tile is
// n x 128 bytes and 8 / lane_groups tiles share a wavefront) and how full its row slots are.
rps::LaunchTuning tiled_tuning(int n, bool bf16, int grad_mode) {
    const int elem = bf16 ? 2 : 4;
    const bool noise = grad_mode == rps::kGradSynthetic, buffer = grad_mode == rps::kGradBuffer;
    if (rps::narrow_split(n, elem))   // pairs of wavefronts per tile, workgroups of 8: two per compute unit
        return rps::LaunchTuning{4, 8, noise ? 0 : 16, 0};
    if (n > 32) {   // the chunked kernel
        // in-register gradient: one row pair per chunk keeps the registers at four or more wavefronts per SIMD;
        // fp32 (74 registers): two workgroups of 12 (+1-3 % over one of 14), bf16: two of 8
        // (bf16 below 62 workers: workgroups of 4, n = 40 0.68 -> 0.70, n = 56 0.72 -> 0.74; not at 64)
        if (noise) return rps::LaunchTuning{2, bf16 ? (n < 62 ? 4 : 8) : 12, 0, 0};
        // gradient buffer: single wavefronts -- bf16 below 62 workers (185 registers; n = 33 0.66 -> 0.79,
        // n = 44 0.73 -> 0.78, n = 56 0.75 -> 0.77; n = 64 0.79 -> 0.77: not there), fp32 with one row pair
        // per chunk (n = 36 0.75 -> 0.78, n = 56 0.73 -> 0.77)
        if (buffer)
            return bf16 ? (n < 62 ? rps::LaunchTuning{4, 1, 10, 0} : rps::LaunchTuning{4, 8, 16, 0})
                        : rps::LaunchTuning{2, 1, n < 40 ? 10 : 8, 0};
        // averaging alone: from 52 workers on one row pair per chunk (bf16 n = 64 0.81 -> 0.86, fp32 n = 56 0.80 -> 0.83)
        return rps::LaunchTuning{n >= 52 ? 2 : 4, 1, n >= 48 ? 8 : 10, 0};
    }
    const rps::NarrowShape shape = rps::narrow_shape(n, elem);
    const int slots = 2 * shape.lane_groups * shape.row_pairs;   // rows a tile's lanes can hold
    const bool three = shape.row_pairs == 3;
    // Single wavefronts: as many per compute unit as put about 44 KB in flight (4 KB steps: 11; 3 KB,
    // e.g. 12 or 24 workers: 14, measured 0.80 -> 0.84 and 0.77 -> 0.84 against 10; 2 KB, 2 workers: 22,
    // 0.75 -> 0.87; 6 KB, bf16 on three row pairs: 8; 1 KB, 1 worker: no cap, 0.37 -> 0.66)
    const int step_bytes = (8 / shape.lane_groups) * n * RPS_TILE_BYTES;
    const int fit = 45056 / step_bytes;
    const rps::LaunchTuning singles{4, 1, fit >= 32 ? 0 : std::max(fit, 8), 0};
    if (!noise && !buffer) return singles;   // averaging alone
    if (buffer) {
        // nothing is shared between wavefronts; a wide workgroup (its wavefronts start together on adjacent
        // tiles of their XCD) is still 2-4 % faster where the row slots are full, single wavefronts are
        // where they are not (fp32 n = 12 0.75 -> 0.78, n = 5 0.73 -> 0.76; bf16 n = 10 0.72 -> 0.78,
        // n = 20 0.72 -> 0.77, n = 28 0.74 -> 0.78)
        if (bf16) {
            if (!three && n == slots && n >= 4 && n <= 16) return rps::LaunchTuning{4, 14, 0, 0};   // 4, 8, 16 workers
            if (three && (shape.lane_groups == 1 || n == slots)) return rps::LaunchTuning{4, 8, 16, 0};   // 5, 6, 12, 24
            return singles;
        }
        if (n > 2 && 100 * n > 85 * slots) return rps::LaunchTuning{4, n >= 16 ? 14 : 12, 0, 0};
        return singles;
    }
    // in-register gradient: the workgroup's wavefronts share one LDS copy of the noise cells.  fp32 (81-90
    // registers): one workgroup of 14 per compute unit (12 below 16 workers; also 12 at 23-31 workers, whose
    // tiles leave row slots idle: n = 24 0.73 -> 0.76, n = 28 0.76 -> 0.78); three row pairs (125
    // registers): two workgroups of 8 (n = 18 0.72 -> 0.77, n = 20 0.74 -> 0.77).  bf16 (112-128 registers,
    // 150 on three row pairs): two workgroups of 8; up to 16 workers one of 12, two of 8 or four of 4 as
    // the tile takes 1, 2 or 4 lane groups; workgroups of 4 on three row pairs
    // Steps per wavefront (0 = the launcher's default: 1 for fp32, 2 for bf16): more where a step is well under
    // 4 KB, so that a workgroup's copy of the noise cells is spread over enough data (fp32 n = 1 0.52 -> 0.70,
    // n = 2 0.79 -> 0.82, n = 5 0.71 -> 0.75)
    const int per_4k = std::min(4, (4096 + step_bytes / 2) / step_bytes);
    const int steps = per_4k > (bf16 ? 2 : 1) ? per_4k : 0;
    if (three) return rps::LaunchTuning{4, bf16 ? 4 : 8, 0, steps};
    if (bf16) return rps::LaunchTuning{4, n > 16 ? 8 : (shape.lane_groups == 4 ? 4 : (shape.lane_groups == 2 ? 8 : 12)), 0, steps};   // up to 16 workers: 119-120 registers
    return rps::LaunchTuning{4, n >= 16 && (n < 23 || n == 32) ? 14 : 12, 0, steps};
}

// Occupancy cap of the gradient averaging (it reads X and G: twice the bytes of the averaging alone per
// wavefront step), from a sweep over 2-64 workers.  Tile-major: single wavefronts with about 34 KB of X in
// flight per compute unit (8 for 4 KB steps: n = 8 0.80 -> 0.84 of the HBM peak, n = 16 0.82 -> 0.85 against a
// fixed 12; 6 for the 6-8 KB steps above 32 workers: n = 64 0.78 -> 0.83, bf16 0.73 -> 0.82); fp32 at 28-32
// (and up to 2) workers: no cap, i.e. one workgroup of 14.  Row-major (workgroups of 4, never fewer than two per compute
// unit): more of them for the short tiles of few workers (n = 3 0.67 -> 0.80, fp32 n = 6 0.70 -> 0.77), no cap
// from 48 workers on (fp32 n = 48 0.51 -> 0.61).
int gradavg_cap(const rps_ctx *ctx) {
    const int n = ctx->n;
    if (ctx->flags & RPS_FLAG_LAYOUT_TILED) {
        if (ctx->dtype == RPS_DTYPE_F32 && (n <= 2 || (n >= 28 && n <= 32))) return 0;
        const int step_bytes = (8 / rps::gradavg_lane_groups(n)) * n * RPS_TILE_BYTES;
        return std::min(16, std::max(6, (34816 + step_bytes / 2) / step_bytes));
    }
    return n <= 3 ? 24 : (n <= 6 && ctx->dtype == RPS_DTYPE_F32 ? 16 : (n >= 48 ? 0 : 8));
}

rps::LaunchTuning tuning_for(const rps_ctx *ctx, int grad_mode) {
    if (ctx->tune_set) return ctx->tune;
    if (ctx->flags & RPS_FLAG_LAYOUT_TILED) return tiled_tuning(ctx->n, ctx->dtype == RPS_DTYPE_BF16, grad_mode);
    return default_tuning(ctx->n, ctx->dtype, grad_mode);
}

RoundParams make_params(const rps_ctx *ctx, const void *X, const void *G, uint64_t step) {
    RoundParams prm;
    prm.N = ctx->N;
    prm.n = ctx->n;
    prm.blocks = ctx->nb;
    const int64_t vec = ctx->dtype == RPS_DTYPE_F32 ? 4 : 8;   // elements per 16 bytes
    const bool aligned = ((uintptr_t)X % 16 == 0) && (G == nullptr || (uintptr_t)G % 16 == 0);
    prm.tiled = (ctx->flags & RPS_FLAG_LAYOUT_TILED) ? 1 : 0;
    prm.stride = prm.tiled ? (RPS_TILE_BYTES / 16) * vec : ctx->pitch;   // tiled: every tile row is one short segment, whatever N is
    prm.vec_ok = (aligned && (prm.tiled || ctx->pitch % vec == 0)) ? 1 : 0;  // every row starts on a 16-byte boundary
    prm.gamma = ctx->gamma;
    prm.sigma = ctx->sigma;
    prm.lambda = ctx->lambda;
    prm.seed_lo = (uint32_t)ctx->seed;
    prm.seed_hi = (uint32_t)(ctx->seed >> 32);
    prm.step_lo = (uint32_t)step;
    prm.step_hi24 = (uint32_t)((step >> 32) & 0xFFFFFFu);
    prm.next_tab = nullptr;
    prm.threshold = ctx->threshold;
    prm.server_mode = 0;
    prm.next_step_lo = prm.next_step_hi24 = 0;
    prm.noise_cells = ctx->noise_cells;
    prm.tiles_per_wave = 1;
    return prm;
}

// Brackets `launch` with events when profiling is on.
template <typename F>
int timed_launch(rps_ctx *ctx, F launch) {
    const bool rec = ctx->profiling && ctx->ev_used < kMaxProfiledLaunches;
    if (rec) {
        if (ctx->ev_used == ctx->ev_start.size()) {
            hipEvent_t a, b;
            RPS_HIP(ctx, hipEventCreate(&a));
            hipError_t e = hipEventCreate(&b);
            if (e != hipSuccess) {
                (void)hipEventDestroy(a);
                return hip_fail(ctx, e);
            }
            try {   // no exception may cross the C boundary
                ctx->ev_start.push_back(a);
                ctx->ev_stop.push_back(b);
            } catch (...) {
                if (ctx->ev_start.size() > ctx->ev_stop.size()) ctx->ev_start.pop_back();
                (void)hipEventDestroy(a);
                (void)hipEventDestroy(b);
                return RPS_ENOMEM;
            }
        }
        RPS_HIP(ctx, hipEventRecord(ctx->ev_start[ctx->ev_used], ctx->stream));
    }
    RPS_HIP(ctx, launch());
    if (rec) {
        RPS_HIP(ctx, hipEventRecord(ctx->ev_stop[ctx->ev_used], ctx->stream));
        ++ctx->ev_used;
    }
    return RPS_OK;
}

int server_mode(const rps_ctx *ctx) {
    return ctx->external ? 2 : ((ctx->flags & RPS_FLAG_SERVER_IDENTITY) ? 1 : 0);
}

// Makes ctx->tab hold the network outcome of `step` and asks the averaging kernel about to be
// launched to prepare the outcome of step + 1 in the other table (rounds usually come with
// consecutive steps; a call whose step is already in one of the two tables needs no mask launch).
// What a table holds is tracked on the host by step number, so results never depend on this.
// Launches recorded while the stream is being captured into a graph run later, any number of times,
// between eager calls the host cannot foresee: they are self-contained (their own mask launch) and
// touch only the capture table, which no eager call reads or writes, so a replay can never change
// a table whose step the host tracks.  `use` receives the table the averaging kernel must read.
int prepare_outcome(rps_ctx *ctx, uint64_t step, RoundParams &prm, const RoundTable *&use) {
    prm.next_tab = nullptr;
    prm.threshold = ctx->threshold;
    prm.server_mode = server_mode(ctx);
    prm.next_step_lo = prm.next_step_hi24 = 0;
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    bool capturing = true;
    if (hipStreamIsCapturing(ctx->stream, &cs) == hipSuccess)
        capturing = cs != hipStreamCaptureStatusNone;
    else
        (void)hipGetLastError();
    if (capturing) {
        // a forced outcome lives in host-written memory that a later rps_set_mask_override changes:
        // a graph cannot pin it
        if (ctx->override_on) return RPS_EUNSUPPORTED;
        use = ctx->tab_capture;
        RPS_HIP(ctx, rps::launch_masks(ctx->tab_capture, ctx->n, ctx->nb, ctx->seed, step, ctx->threshold,
                                       server_mode(ctx), ctx->stream));
        return RPS_OK;
    }
    if (ctx->override_on) {   // the override table holds the forced outcome
        use = ctx->tab_override;
        return RPS_OK;
    }
    if (ctx->next_valid && ctx->next_step == step) {
        std::swap(ctx->tab, ctx->tab_other);
    } else if (!(ctx->cur_valid && ctx->cur_step == step)) {
        ctx->cur_valid = false;
        RPS_HIP(ctx, rps::launch_masks(ctx->tab, ctx->n, ctx->nb, ctx->seed, step, ctx->threshold, server_mode(ctx),
                                       ctx->stream));
    }
    ctx->cur_valid = true;
    ctx->cur_step = step;
    ctx->next_valid = false;
    if (step_ok(step + 1)) {
        prm.next_tab = ctx->tab_other;
        prm.next_step_lo = (uint32_t)(step + 1);
        prm.next_step_hi24 = (uint32_t)(((step + 1) >> 32) & 0xFFFFFFu);
    }
    use = ctx->tab;
    return RPS_OK;
}

// After the averaging kernel was enqueued (rc == RPS_OK) the other table will hold step + 1.
int commit_outcome(rps_ctx *ctx, uint64_t step, const RoundParams &prm, int rc) {
    if (rc != RPS_OK) {
        ctx->cur_valid = ctx->next_valid = false;
    } else if (prm.next_tab != nullptr) {
        ctx->next_valid = true;
        ctx->next_step = step + 1;
    }
    return rc;
}

// The cell values of the synthetic gradient noise, computed once per process.
const float *noise_cells_host() {
    static const std::vector<float> cells = [] {
        std::vector<float> v(3 * (size_t)rps::kNoiseGrid);
        rps::build_noise_cells(v.data(), v.data() + rps::kNoiseGrid);
        return v;
    }();
    return cells.data();
}

// The device copy of the radius cells carries sigma: sigma * r rounded to fp32 once, here on the
// host (the same IEEE multiplication the oracle does per sample).  In stream order after the work
// already enqueued; synchronises so that the staging buffer can be reused.
hipError_t upload_scaled_radii(rps_ctx *ctx) {
    hipError_t e = hipStreamSynchronize(ctx->stream);   // an earlier upload may still be reading the staging buffer
    if (e != hipSuccess) return e;
    const float *radius = noise_cells_host();
    for (int k = 0; k < rps::kNoiseGrid; ++k) ctx->radius_staging[k] = ctx->sigma * radius[k];
    e = hipMemcpyAsync(ctx->noise_cells, ctx->radius_staging, (size_t)rps::kNoiseGrid * sizeof(float),
                       hipMemcpyHostToDevice, ctx->stream);
    if (e != hipSuccess) return e;
    return hipStreamSynchronize(ctx->stream);
}

// ---------------------------------------------------------------------------------------
// Host copy of the network-outcome generator (Sec. 3; Alg. 1 steps 6-7), written on its own: the
// same specification the mask kernel implements on the device -- Philox4x32-10 keyed by the seed,
// counter (worker, block, step low word, domain << 24 | step high 24 bits); domains 0 uplink,
// 1 downlink, 2 server sort key -- evaluated here with plain 64-bit integer arithmetic, so that
// the device table can be checked against something that never ran on the GPU.
// ---------------------------------------------------------------------------------------
uint32_t host_hash_word0(uint64_t seed, uint64_t step, uint32_t a, uint32_t b, uint32_t domain) {
    uint32_t x0 = a, x1 = b, x2 = (uint32_t)step, x3 = (domain << 24) | (uint32_t)((step >> 32) & 0xFFFFFFu);
    uint32_t ka = (uint32_t)seed, kb = (uint32_t)(seed >> 32);
    for (int round = 0; round < 10; ++round) {
        const uint64_t left = 0xD2511F53ull * x0, right = 0xCD9E8D57ull * x2;
        const uint32_t y0 = (uint32_t)(right >> 32) ^ x1 ^ ka, y2 = (uint32_t)(left >> 32) ^ x3 ^ kb;
        x1 = (uint32_t)right;
        x3 = (uint32_t)left;
        x0 = y0;
        x2 = y2;
        ka += 0x9E3779B9u;
        kb += 0xBB67AE85u;
    }
    return x0;
}

// Fills a RoundTable's outcome fields (not the offsets) for `step`.
void host_outcome(RoundTable &t, int n, int nb, uint64_t seed, uint64_t step, uint64_t threshold, int mode) {
    int32_t server_of[rps::kMaxWorkers];
    if (mode == 0) {
        // block j goes to the worker whose sort key has rank j among (key, worker index)
        std::pair<uint32_t, int> keyed[rps::kMaxWorkers];
        for (int i = 0; i < n; ++i) keyed[i] = {host_hash_word0(seed, step, (uint32_t)i, 0u, 2u), i};
        std::sort(keyed, keyed + n);
        for (int j = 0; j < nb; ++j) server_of[j] = keyed[j].second;
    } else {
        for (int j = 0; j < nb; ++j) server_of[j] = mode == 1 ? j : -1;
    }
    for (int j = 0; j < nb; ++j) {
        uint64_t u = 0, d = 0;
        for (int i = 0; i < n; ++i) {
            const bool self = i == server_of[j];   // not a network message
            if (self || (uint64_t)host_hash_word0(seed, step, (uint32_t)i, (uint32_t)j, 0u) >= threshold) u |= 1ull << i;
            if (self || (uint64_t)host_hash_word0(seed, step, (uint32_t)i, (uint32_t)j, 1u) >= threshold) d |= 1ull << i;
        }
        t.ucol[j] = u;
        t.dcol_drawn[j] = d;
        t.dcol[j] = u ? d : 0;
        t.cnt[j] = __builtin_popcountll(u);
        t.inv_cnt[j] = u ? 1.0 / (double)t.cnt[j] : 0.0;
        t.server[j] = server_of[j];
    }
}

void unpack_outcome(const RoundTable &t, int n, int nb, uint8_t *up, uint8_t *down, int32_t *server) {
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < nb; ++j) {
            if (up) up[i * nb + j] = (uint8_t)((t.ucol[j] >> i) & 1);
            if (down) down[i * nb + j] = (uint8_t)((t.dcol_drawn[j] >> i) & 1);
        }
    if (server)
        for (int j = 0; j < nb; ++j) server[j] = t.server[j];
}

struct DeviceGuard {   // make the context's device current for the duration of a call
    int prev = -1;
    bool ok = false;
    explicit DeviceGuard(int dev) {
        if (hipGetDevice(&prev) == hipSuccess) ok = (prev == dev) || hipSetDevice(dev) == hipSuccess;
    }
    ~DeviceGuard() {
        int cur = -1;
        if (prev >= 0 && hipGetDevice(&cur) == hipSuccess && cur != prev) (void)hipSetDevice(prev);
    }
};

}  // namespace

extern "C" {

static int create_impl(rps_ctx **out, int32_t n, int32_t nb, bool external, int64_t N, const int64_t *block_offsets,
                       double p, float gamma, uint64_t seed, int32_t dtype, uint32_t flags, void *hip_stream) {
    if (!out) return RPS_EINVAL;
    if (n < 1 || n > rps::kMaxWorkers) return RPS_EINVAL;
    if (nb < 1 || nb > rps::kMaxWorkers) return RPS_EINVAL;
    if (N < nb || N > (1ll << 34)) return RPS_EINVAL;
    if (!(p >= 0.0 && p <= 1.0)) return RPS_EINVAL;   // also rejects NaN
    if (!std::isfinite(gamma)) return RPS_EINVAL;
    if (dtype != RPS_DTYPE_F32 && dtype != RPS_DTYPE_BF16) return RPS_EINVAL;
    if (flags & ~(uint32_t)(RPS_FLAG_SERVER_IDENTITY | RPS_FLAG_LAYOUT_TILED)) return RPS_EINVAL;

    rps_ctx *ctx = new (std::nothrow) rps_ctx;
    if (!ctx) return RPS_ENOMEM;
    try {   // no exception may cross the C boundary
        ctx->off.resize((size_t)nb + 1);
    } catch (...) {
        delete ctx;
        return RPS_ENOMEM;
    }
    if (block_offsets) {
        for (int j = 0; j <= nb; ++j) ctx->off[j] = block_offsets[j];
        bool ok = ctx->off[0] == 0 && ctx->off[nb] == N;
        for (int j = 0; j < nb && ok; ++j) ok = ctx->off[j] < ctx->off[j + 1];
        if (!ok) {
            delete ctx;
            return RPS_EINVAL;
        }
    } else {
        if (N % nb != 0) {   // the paper's blocks are equally sized
            delete ctx;
            return RPS_EINVAL;
        }
        for (int j = 0; j <= nb; ++j) ctx->off[j] = (N / nb) * j;
    }
    for (int j = 0; j < nb; ++j)
        if (ctx->off[j + 1] - ctx->off[j] > ctx->max_block_cols) ctx->max_block_cols = ctx->off[j + 1] - ctx->off[j];

    ctx->n = n;
    ctx->nb = nb;
    ctx->external = external;
    ctx->N = N;
    ctx->pitch = N;
    ctx->p = p;
    ctx->threshold = (uint64_t)std::floor(p * 4294967296.0);
    ctx->gamma = gamma;
    ctx->seed = seed;
    ctx->dtype = dtype;
    ctx->flags = flags;
    ctx->stream = (hipStream_t)hip_stream;

    hipError_t e = hipGetDevice(&ctx->device);
    if (e == hipSuccess) {   // set-up is the place to resolve this GPU's static scratch (rps_consensus_static)
        double *unused = nullptr;
        e = rps::static_scratch(ctx->device, &unused);
    }
    const size_t scratch_bytes = (2 * (size_t)rps::kMaxPartials + 2) * sizeof(double);
    const size_t cells_at = (6 * sizeof(RoundTable) + scratch_bytes + 255) & ~(size_t)255;
    const size_t cells_bytes = 3 * (size_t)rps::kNoiseGrid * sizeof(float);
    if (e == hipSuccess) e = hipMalloc((void **)&ctx->tab_base, cells_at + cells_bytes);
    if (e == hipSuccess) {
        ctx->noise_cells = reinterpret_cast<float *>(reinterpret_cast<char *>(ctx->tab_base) + cells_at);
        e = hipMemcpyAsync(ctx->noise_cells, noise_cells_host(), cells_bytes, hipMemcpyHostToDevice, ctx->stream);
    }
    if (e == hipSuccess)
        e = hipHostMalloc((void **)&ctx->radius_staging, (size_t)rps::kNoiseGrid * sizeof(float), hipHostMallocDefault);
    if (e == hipSuccess) e = upload_scaled_radii(ctx);   // sigma = 0 until rps_set_synthetic_grad
    if (e == hipSuccess) {
        ctx->tab = ctx->tab_base;
        ctx->tab_other = ctx->tab_base + 1;
        ctx->tab_query = ctx->tab_base + 2;
        ctx->tab_capture = ctx->tab_base + 3;
        ctx->tab_override = ctx->tab_base + 4;
        ctx->tab_nothing = ctx->tab_base + 5;
        ctx->partials = reinterpret_cast<double *>(ctx->tab_base + 6);
        e = hipHostMalloc((void **)&ctx->staging, sizeof(RoundTable), hipHostMallocDefault);
    }
    if (e == hipSuccess) {
        std::memset(ctx->staging, 0, sizeof(RoundTable));
        for (int j = 0; j <= nb; ++j) ctx->staging->off[j] = ctx->off[j];
        for (int k = 0; k < 6 && e == hipSuccess; ++k)   // every table carries the block offsets; all masks start at zero
            e = hipMemcpyAsync(ctx->tab_base + k, ctx->staging, sizeof(RoundTable), hipMemcpyHostToDevice, ctx->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    }
    if (e != hipSuccess) {
        const bool oom = (e == hipErrorOutOfMemory);
        g_last_hip_without_ctx = (int)e;
        if (ctx->tab_base) (void)hipFree(ctx->tab_base);
        if (ctx->staging) (void)hipHostFree(ctx->staging);
        if (ctx->radius_staging) (void)hipHostFree(ctx->radius_staging);
        delete ctx;
        return oom ? RPS_ENOMEM : RPS_EHIP;
    }
    *out = ctx;
    return RPS_OK;
}

int rps_create(rps_ctx **out, int32_t n, int64_t N, const int64_t *block_offsets, double p, float gamma,
               uint64_t seed, int32_t dtype, uint32_t flags, void *hip_stream) {
    return create_impl(out, n, n, false, N, block_offsets, p, gamma, seed, dtype, flags, hip_stream);
}

int64_t rps_storage_elems(int32_t n, int64_t N, int32_t dtype, uint32_t flags) {
    if (n < 1 || n > rps::kMaxWorkers || N < 1 || N > (1ll << 34)) return -1;
    if (dtype != RPS_DTYPE_F32 && dtype != RPS_DTYPE_BF16) return -1;
    if (!(flags & RPS_FLAG_LAYOUT_TILED)) return (int64_t)n * N;
    const int64_t T = RPS_TILE_BYTES / (dtype == RPS_DTYPE_F32 ? 4 : 2);
    return ((N + T - 1) / T) * n * T;
}

int rps_create_external(rps_ctx **out, int32_t n, int32_t servers, int64_t N, const int64_t *block_offsets, double p,
                        float gamma, uint64_t seed, int32_t dtype, void *hip_stream) {
    return create_impl(out, n, servers, true, N, block_offsets, p, gamma, seed, dtype, 0u, hip_stream);
}

int rps_destroy(rps_ctx *ctx) {
    if (!ctx) return RPS_OK;
    DeviceGuard guard(ctx->device);
    int rc = RPS_OK;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) rc = RPS_EHIP;
    for (hipEvent_t ev : ctx->ev_start) (void)hipEventDestroy(ev);
    for (hipEvent_t ev : ctx->ev_stop) (void)hipEventDestroy(ev);
    if (ctx->tab_base && hipFree(ctx->tab_base) != hipSuccess) rc = RPS_EHIP;
    if (ctx->staging && hipHostFree(ctx->staging) != hipSuccess) rc = RPS_EHIP;
    if (ctx->radius_staging && hipHostFree(ctx->radius_staging) != hipSuccess) rc = RPS_EHIP;
    delete ctx;
    return rc;
}

int rps_set_synthetic_grad(rps_ctx *ctx, float sigma, float weight_decay) {
    if (!ctx || !std::isfinite(sigma) || sigma < 0.0f || !std::isfinite(weight_decay)) return RPS_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return RPS_EHIP;
    const float before = ctx->sigma;
    ctx->sigma = sigma;
    if (sigma != before) {
        const hipError_t e = upload_scaled_radii(ctx);
        if (e != hipSuccess) {
            ctx->sigma = before;   // the device table still holds the old radii (or is rewritten by the next call)
            return hip_fail(ctx, e);
        }
    }
    ctx->lambda = weight_decay;
    return RPS_OK;
}

int rps_set_row_pitch(rps_ctx *ctx, int64_t pitch) {
    if (!ctx || (ctx->flags & RPS_FLAG_LAYOUT_TILED)) return RPS_EINVAL;
    if (pitch < ctx->N || pitch > (1ll << 35)) return RPS_EINVAL;
    ctx->pitch = pitch;
    return RPS_OK;
}

int64_t rps_recommended_row_pitch(int64_t N, int32_t dtype) {
    if (N < 1 || N > (1ll << 34) || (dtype != RPS_DTYPE_F32 && dtype != RPS_DTYPE_BF16)) return -1;
    const int64_t elem = dtype == RPS_DTYPE_F32 ? 4 : 2;
    // smallest pitch >= N whose byte size is 4 KB past a multiple of 64 KB
    const int64_t bytes = N * elem;
    int64_t base = (bytes / 65536) * 65536 + 4096;
    if (base < bytes) base += 65536;
    return base / elem;
}

int rps_set_gamma(rps_ctx *ctx, float gamma) {
    if (!ctx || !std::isfinite(gamma)) return RPS_EINVAL;
    ctx->gamma = gamma;
    return RPS_OK;
}

int rps_local_step(rps_ctx *ctx, void *X, const void *G, uint64_t step) {
    if (!ctx || !X || !step_ok(step)) return RPS_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return RPS_EHIP;
    const RoundParams prm = make_params(ctx, X, G, step);
    const int mode = G ? rps::kGradBuffer : rps::kGradSynthetic;
    // Tile-major layout, in-register gradient: the round kernel under the outcome "no message arrives"
    // is the local step (no row enters a sum, every row keeps its own v), and its lanes own both rows of
    // a worker pair, so the noise of a (4 columns x 2 workers) patch is generated once.
    if ((ctx->flags & RPS_FLAG_LAYOUT_TILED) && mode == rps::kGradSynthetic)
        return timed_launch(ctx, [&] {
            return rps::launch_round(ctx->dtype, mode, X, nullptr, ctx->tab_nothing, prm, ctx->max_block_cols,
                                     tuning_for(ctx, mode), ctx->stream);
        });
    return timed_launch(ctx, [&] { return rps::launch_local_step(ctx->dtype, mode, X, G, prm, ctx->tune_set ? ctx->tune.tiles_per_wave : 0, ctx->stream); });
}

int rps_lossy_average(rps_ctx *ctx, void *X, uint64_t step) {
    if (!ctx || !X || !step_ok(step)) return RPS_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return RPS_EHIP;
    RoundParams prm = make_params(ctx, X, nullptr, step);
    const RoundTable *tab = nullptr;
    const int rc = prepare_outcome(ctx, step, prm, tab);
    if (rc != RPS_OK) return rc;
    return commit_outcome(ctx, step, prm, timed_launch(ctx, [&] {
        return rps::launch_round(ctx->dtype, rps::kGradNone, X, nullptr, tab, prm, ctx->max_block_cols,
                                 tuning_for(ctx, rps::kGradNone), ctx->stream);
    }));
}

int rps_round(rps_ctx *ctx, void *X, const void *G, uint64_t step) {
    if (!ctx || !X || !step_ok(step)) return RPS_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return RPS_EHIP;
    RoundParams prm = make_params(ctx, X, G, step);
    const int mode = G ? rps::kGradBuffer : rps::kGradSynthetic;
    const RoundTable *tab = nullptr;
    const int rc = prepare_outcome(ctx, step, prm, tab);
    if (rc != RPS_OK) return rc;
    return commit_outcome(ctx, step, prm, timed_launch(ctx, [&] {
        return rps::launch_round(ctx->dtype, mode, X, G, tab, prm, ctx->max_block_cols, tuning_for(ctx, mode),
                                 ctx->stream);
    }));
}

int rps_round_gradient_averaging(rps_ctx *ctx, void *X, const void *G, uint64_t step) {
    if (!ctx || !X || !G || !step_ok(step)) return RPS_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return RPS_EHIP;
    RoundParams prm = make_params(ctx, X, G, step);
    const RoundTable *tab = nullptr;
    const int rc = prepare_outcome(ctx, step, prm, tab);
    if (rc != RPS_OK) return rc;
    return commit_outcome(ctx, step, prm, timed_launch(ctx, [&] {
        const int cap = ctx->tune_set ? ctx->tune.max_waves_per_cu : gradavg_cap(ctx);
        return rps::launch_gradavg(ctx->dtype, X, G, tab, prm, ctx->max_block_cols, cap, ctx->stream);
    }));
}

int rps_get_masks(rps_ctx *ctx, uint64_t step, uint8_t *up, uint8_t *down, int32_t *server) {
    if (!ctx || !step_ok(step)) return RPS_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return RPS_EHIP;
    RPS_HIP(ctx, rps::launch_masks(ctx->tab_query, ctx->n, ctx->nb, ctx->seed, step, ctx->threshold, server_mode(ctx),
                                   ctx->stream));
    RPS_HIP(ctx, hipMemcpyAsync(ctx->staging, ctx->tab_query, sizeof(RoundTable), hipMemcpyDeviceToHost, ctx->stream));
    RPS_HIP(ctx, hipStreamSynchronize(ctx->stream));
    unpack_outcome(*ctx->staging, ctx->n, ctx->nb, up, down, server);
    return RPS_OK;
}

int rps_masks_host(int32_t n, int32_t servers, double p, uint64_t seed, uint32_t flags, uint64_t step, uint8_t *up,
                   uint8_t *down, int32_t *server) {
    if (n < 1 || n > rps::kMaxWorkers || servers < 0 || servers > rps::kMaxWorkers) return RPS_EINVAL;
    if (!(p >= 0.0 && p <= 1.0) || !step_ok(step)) return RPS_EINVAL;
    if (flags & ~(uint32_t)(RPS_FLAG_SERVER_IDENTITY | RPS_FLAG_LAYOUT_TILED)) return RPS_EINVAL;
    if (servers > 0 && flags != 0) return RPS_EINVAL;   // as rps_create_external: no flags
    const int nb = servers > 0 ? servers : n;
    const int mode = servers > 0 ? 2 : ((flags & RPS_FLAG_SERVER_IDENTITY) ? 1 : 0);
    RoundTable t;
    std::memset(&t, 0, sizeof(t));
    host_outcome(t, n, nb, seed, step, (uint64_t)std::floor(p * 4294967296.0), mode);
    unpack_outcome(t, n, nb, up, down, server);
    return RPS_OK;
}

int rps_set_mask_override(rps_ctx *ctx, const uint8_t *up, const uint8_t *down, const int32_t *server) {
    if (!ctx) return RPS_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return RPS_EHIP;
    if (!up && !down && !server) {   // the eager tables were not touched: what the host tracks still holds
        RPS_HIP(ctx, hipStreamSynchronize(ctx->stream));
        ctx->override_on = false;
        return RPS_OK;
    }
    if (!up || !down || !server) return RPS_EINVAL;
    const int n = ctx->n, nb = ctx->nb;
    RoundTable t;
    std::memset(&t, 0, sizeof(t));
    for (int j = 0; j <= nb; ++j) t.off[j] = ctx->off[j];
    for (int j = 0; j < nb; ++j) {
        if (!ctx->external && (server[j] < 0 || server[j] >= n)) return RPS_EINVAL;
        uint64_t u = 0, d = 0;
        for (int i = 0; i < n; ++i) {
            if (up[i * nb + j]) u |= 1ull << i;
            if (down[i * nb + j]) d |= 1ull << i;
        }
        if (u == 0 && !ctx->external) return RPS_EINVAL;   // a worker-server always holds its own copy
        t.ucol[j] = u;
        t.dcol_drawn[j] = d;
        t.dcol[j] = u ? d : 0;
        t.cnt[j] = __builtin_popcountll(u);
        t.inv_cnt[j] = u ? 1.0 / (double)t.cnt[j] : 0.0;
        t.server[j] = ctx->external ? -1 : server[j];
    }
    RPS_HIP(ctx, hipStreamSynchronize(ctx->stream));   // staging may still be in flight
    *ctx->staging = t;
    RPS_HIP(ctx, hipMemcpyAsync(ctx->tab_override, ctx->staging, sizeof(RoundTable), hipMemcpyHostToDevice, ctx->stream));
    RPS_HIP(ctx, hipStreamSynchronize(ctx->stream));
    ctx->override_on = true;
    return RPS_OK;
}

int rps_consensus(rps_ctx *ctx, const void *X, double *distance, double *mean_sq) {
    if (!ctx || !X) return RPS_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return RPS_EHIP;
    const RoundParams prm = make_params(ctx, X, nullptr, 0);
    double *out = ctx->partials + 2 * rps::kMaxPartials;
    const int rc = timed_launch(ctx, [&] {
        return rps::launch_consensus(ctx->dtype, X, prm, ctx->partials, rps::kMaxPartials, out, ctx->stream);
    });
    if (rc != RPS_OK) return rc;
    double host[2] = {0.0, 0.0};
    RPS_HIP(ctx, hipMemcpyAsync(host, out, sizeof(host), hipMemcpyDeviceToHost, ctx->stream));
    RPS_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (distance) *distance = host[0];
    if (mean_sq) *mean_sq = host[1];
    return RPS_OK;
}

int rps_consensus_static(const void *X, int32_t n, int64_t N, int32_t dtype, uint32_t flags, double *out,
                         void *hip_stream) {
    if (!X || !out) return RPS_EINVAL;
    if (dtype != RPS_DTYPE_F32 && dtype != RPS_DTYPE_BF16) return RPS_EINVAL;
    if (flags & ~(uint32_t)RPS_FLAG_LAYOUT_TILED) return RPS_EINVAL;
    if (n < 1 || N < 1) return RPS_EINVAL;
    if (n > rps::kMaxWorkers || N > (1ll << 34)) return RPS_ETOOBIG;   // beyond what the fixed scratch is laid out for
    // the GPU that holds X: its copy of the scratch is the one to use
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, X) != hipSuccess) {
        (void)hipGetLastError();
        return RPS_EINVAL;
    }
    if (attr.type != hipMemoryTypeDevice) return RPS_EINVAL;
    DeviceGuard guard(attr.device);
    if (!guard.ok) return RPS_EHIP;
    double *partials = nullptr;
    if (rps::static_scratch(attr.device, &partials) != hipSuccess) return RPS_EHIP;
    RoundParams prm{};
    prm.N = N;
    prm.n = n;
    prm.blocks = n;
    const int64_t vec = dtype == RPS_DTYPE_F32 ? 4 : 8;
    prm.tiled = (flags & RPS_FLAG_LAYOUT_TILED) ? 1 : 0;
    prm.stride = prm.tiled ? (RPS_TILE_BYTES / 16) * vec : N;
    prm.vec_ok = ((uintptr_t)X % 16 == 0 && (prm.tiled || N % vec == 0)) ? 1 : 0;
    if (rps::launch_consensus(dtype, X, prm, partials, rps::kMaxPartials, out, (hipStream_t)hip_stream) != hipSuccess)
        return RPS_EHIP;
    return RPS_OK;
}

int rps_estimate_mixing(rps_ctx *ctx, uint64_t first_step, int64_t rounds, double *alpha1, double *alpha2) {
    if (!ctx || rounds < 1 || rounds > (1ll << 24) || ctx->n < 2) return RPS_EINVAL;
    if (!step_ok(first_step) || !step_ok(first_step + (uint64_t)rounds - 1)) return RPS_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return RPS_EHIP;
    const int groups = (int)std::min<int64_t>(rounds, rps::kMaxPartials);
    std::vector<double> host;
    try {   // no exception may cross the C boundary; nothing is enqueued yet
        host.resize(2 * (size_t)groups);
    } catch (...) {
        return RPS_ENOMEM;
    }
    RPS_HIP(ctx, rps::launch_mixing_moments(ctx->partials, groups, rounds, ctx->n, ctx->nb, ctx->seed, first_step,
                                            ctx->threshold, server_mode(ctx), ctx->stream));
    RPS_HIP(ctx, hipMemcpyAsync(host.data(), ctx->partials, 2 * (size_t)groups * sizeof(double), hipMemcpyDeviceToHost,
                                ctx->stream));
    RPS_HIP(ctx, hipStreamSynchronize(ctx->stream));
    double sq = 0.0, sum_sq = 0.0;
    for (int w = 0; w < groups; ++w) {
        sq += host[2 * w];
        sum_sq += host[2 * w + 1];
    }
    // means over rounds, blocks and the n rows of W: E[(W W^T)_mm] and n E[(W A_n W^T)_mm]
    const double n = (double)ctx->n, samples = (double)rounds * (double)ctx->nb * n;
    if (alpha1) *alpha1 = (n * (sq / samples) - 1.0) / (n - 1.0);
    if (alpha2) *alpha2 = (sum_sq / samples - 1.0) / (n - 1.0);
    return RPS_OK;
}

int rps_convert_layout(rps_ctx *ctx, void *dst, const void *src, int32_t to_tiled) {
    if (!ctx || !dst || !src || dst == src) return RPS_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return RPS_EHIP;
    const int64_t vec = ctx->dtype == RPS_DTYPE_F32 ? 4 : 8;
    const bool aligned = (uintptr_t)dst % 16 == 0 && (uintptr_t)src % 16 == 0 && ctx->pitch % vec == 0;
    return timed_launch(ctx, [&] {
        return rps::launch_convert_layout(ctx->dtype, dst, src, ctx->N, ctx->pitch, ctx->n, to_tiled != 0, aligned,
                                          ctx->stream);
    });
}

int rps_set_launch_tuning(rps_ctx *ctx, int32_t rows_in_flight, int32_t waves_per_workgroup, int32_t max_waves_per_cu,
                          int32_t tiles_per_wave) {
    if (!ctx) return RPS_EINVAL;
    if (rows_in_flight != 2 && rows_in_flight != 4) return RPS_EINVAL;
    if (waves_per_workgroup < 1 || waves_per_workgroup > 16) return RPS_EINVAL;
    if (max_waves_per_cu < 0 || tiles_per_wave < 0 || tiles_per_wave > 64) return RPS_EINVAL;
    ctx->tune = rps::LaunchTuning{rows_in_flight, waves_per_workgroup, max_waves_per_cu, tiles_per_wave};
    ctx->tune_set = true;
    return RPS_OK;
}

int rps_query_occupancy(rps_ctx *ctx, int32_t gradient_source, int32_t *waves_per_cu) {
    if (!ctx || !waves_per_cu) return RPS_EINVAL;
    if (gradient_source != rps::kGradNone && gradient_source != rps::kGradBuffer && gradient_source != rps::kGradSynthetic)
        return RPS_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return RPS_EHIP;
    // no array is touched: any aligned address serves to pick the 128-bit kernels
    const RoundParams prm = make_params(ctx, nullptr, nullptr, 0);
    rps::LaunchTuning tune = tuning_for(ctx, gradient_source);
    int waves = 0;
    tune.occupancy_query = &waves;
    RPS_HIP(ctx, rps::launch_round(ctx->dtype, gradient_source, nullptr, nullptr, nullptr, prm, ctx->max_block_cols, tune,
                                   ctx->stream));
    *waves_per_cu = waves;
    return RPS_OK;
}

int rps_set_profiling(rps_ctx *ctx, int32_t enable) {
    if (!ctx) return RPS_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return RPS_EHIP;
    RPS_HIP(ctx, hipStreamSynchronize(ctx->stream));
    ctx->profiling = enable != 0;
    ctx->ev_used = 0;
    return RPS_OK;
}

int rps_get_kernel_times(rps_ctx *ctx, double *ms, int64_t capacity, int64_t *launches) {
    if (!ctx || !launches || capacity < 0 || (capacity > 0 && !ms)) return RPS_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return RPS_EHIP;
    RPS_HIP(ctx, hipStreamSynchronize(ctx->stream));
    const size_t count = std::min<size_t>(ctx->ev_used, (size_t)capacity);
    for (size_t k = 0; k < count; ++k) {
        float t = 0.0f;
        RPS_HIP(ctx, hipEventElapsedTime(&t, ctx->ev_start[k], ctx->ev_stop[k]));
        ms[k] = (double)t;
    }
    *launches = (int64_t)ctx->ev_used;
    ctx->ev_used = 0;
    return RPS_OK;
}

int rps_get_kernel_time(rps_ctx *ctx, double *total_ms, int64_t *launches) {
    if (!ctx || !total_ms || !launches) return RPS_EINVAL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return RPS_EHIP;
    RPS_HIP(ctx, hipStreamSynchronize(ctx->stream));
    double sum = 0.0;
    for (size_t k = 0; k < ctx->ev_used; ++k) {
        float ms = 0.0f;
        RPS_HIP(ctx, hipEventElapsedTime(&ms, ctx->ev_start[k], ctx->ev_stop[k]));
        sum += (double)ms;
    }
    *total_ms = sum;
    *launches = (int64_t)ctx->ev_used;
    ctx->ev_used = 0;
    return RPS_OK;
}

int rps_noise_cells(float *radius, float *cos_sin) {
    if (!radius || !cos_sin) return RPS_EINVAL;
    const float *cells = noise_cells_host();
    std::memcpy(radius, cells, (size_t)rps::kNoiseGrid * sizeof(float));
    std::memcpy(cos_sin, cells + rps::kNoiseGrid, 2 * (size_t)rps::kNoiseGrid * sizeof(float));
    return RPS_OK;
}

int rps_last_hip_error(const rps_ctx *ctx) { return ctx ? ctx->last_hip : g_last_hip_without_ctx; }

const char *rps_strerror(int code) {
    switch (code) {
        case RPS_OK: return "success";
        case RPS_EINVAL: return "invalid argument";
        case RPS_ENOMEM: return "out of memory";
        case RPS_EHIP: return "HIP runtime error (see rps_last_hip_error)";
        case RPS_EUNSUPPORTED: return "not supported";
        case RPS_ETOOBIG: return "size beyond the maximum of the allocation-free entry point";
        default: return "unknown error code";
    }
}

}  // extern "C"
