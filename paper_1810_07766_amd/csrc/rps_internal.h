// Internal declarations shared by the kernel file and the C-ABI file of the HIP library.
// (Not installed; the public interface is include/rps.h.)
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rps {

constexpr int kMaxWorkers = 64;          // one 64-bit lane mask per block and direction
constexpr int kNoiseGrid = 4096;         // radius cells = angle cells of the synthetic gradient noise

// Device-resident description of one round's network outcome plus the block partition.
// Written by the mask kernel (or copied from the host for a mask override), read by the
// round kernels through wave-uniform (scalar) loads.
struct RoundTable {
    uint64_t ucol[kMaxWorkers];     // bit i of ucol[j]: worker i's copy of block j reached server[j]
    uint64_t dcol[kMaxWorkers];     // bit i of dcol[j]: server[j]'s reply reached worker i (0 if it had nothing to send)
    uint64_t dcol_drawn[kMaxWorkers];   // the downlink bits as drawn (what rps_get_masks reports)
    double inv_cnt[kMaxWorkers];    // 1 / popcount(ucol[j])
    int64_t off[kMaxWorkers + 1];   // block j = columns [off[j], off[j+1])
    int32_t cnt[kMaxWorkers];       // popcount(ucol[j]) >= 1
    int32_t server[kMaxWorkers];    // worker that averages block j
};

struct RoundParams {
    int64_t N;            // columns (parameters per worker)
    int64_t stride;       // storage distance between consecutive rows of a tile: N (row-major) or the tile width (tiled: 128 bytes of elements)
    int32_t tiled;        // 1: storage is [tiles][n][tile width] (rps.h, RPS_FLAG_LAYOUT_TILED)
    int32_t n;            // workers
    int32_t blocks;       // blocks (= n unless the servers are external)
    int32_t vec_ok;       // 1: every full 8-column group may use 128-bit accesses
    float gamma;
    float sigma;          // synthetic gradient: noise std
    float lambda;         // synthetic gradient: weight decay
    uint32_t seed_lo, seed_hi;
    uint32_t step_lo, step_hi24;
    // Outcome of the following step, prepared by the averaging kernels (nullptr: not wanted)
    RoundTable *next_tab;
    uint64_t threshold;     // a message is lost iff its hash word < threshold
    int32_t server_mode;
    uint32_t next_step_lo, next_step_hi24;
    // Synthetic gradient noise: the cell values radius[kNoiseGrid], then (cos, sin) of the angle
    // cells (the kernels use the kNoiseGrid / 2 below pi; device memory owned by the context), and
    // how many steps a wavefront takes (set by the launchers)
    const float *noise_cells;
    int32_t tiles_per_wave;
};

enum GradMode { kGradNone = 0, kGradBuffer = 1, kGradSynthetic = 2 };

constexpr int kLdsBytesPerCu = 160 * 1024;

// Launch shape of the round kernel (see rps_set_launch_tuning in rps.h).
struct LaunchTuning {
    int rows_in_flight;        // rows per load chunk (two chunks are in flight): 2 or 4
    int waves_per_workgroup;   // wavefronts per workgroup (adjacent tiles): 1, 2, 4, 8 or 16 (rounded to what the kernel offers)
    int max_waves_per_cu;      // occupancy cap; 0 or >= 32: none
    int tiles_per_wave;        // steps per wavefront in kernels that generate noise; 0: chosen by the launcher
    int *occupancy_query = nullptr;   // non-null: launch_round launches nothing and stores here the wavefronts per compute
                                      // unit that the chosen kernel and launch shape allow
};

// Tile-major round: how the n rows of a 128-byte tile are dealt to a wavefront's 8 lane groups.  A tile
// takes 1, 2, 4 or 8 of them (8, 4, 2 or 1 tiles share the wavefront); each group's lanes hold 1, 2 or 3
// row pairs, or walk more in chunks (row_pairs == 0, more than 32 workers).  Two pairs per lane is the
// rule; three go where the worker count is far enough off a power of two that two would leave row slots
// (i.e. loads, and for bf16 the noise arithmetic, which every slot pays) idle:
//   fp32: only where over 30 % were idle (9-10 and 17-22 workers: 0.60-0.69 -> 0.72-0.76 of the HBM peak
//         at equal state size; it measured 4 % slower at 6 and 12 workers, +-1 % at 24);
//   bf16: wherever fewer slots result (5-6, 9-12, 17-24 workers: 0.45-0.57 -> 0.62-0.75).
// Three pairs on all 8 groups (33-48 workers) are not used: 187-200 registers per lane halve the occupancy.
struct NarrowShape {
    int lane_groups;
    int row_pairs;
};
inline NarrowShape narrow_shape(int n, int elem_bytes) {
    const int pairs = (n + 1) / 2;
    if (pairs > 16) return {8, 0};
    const int need = (pairs + 1) / 2;
    const int pg = need > 4 ? 8 : (need > 2 ? 4 : (need > 1 ? 2 : 1));
    const int cp = pairs <= pg ? 1 : 2;
    const int need3 = (pairs + 2) / 3;
    const int pg3 = need3 > 4 ? 8 : (need3 > 2 ? 4 : (need3 > 1 ? 2 : 1));
    const int slots = pg * cp, slots3 = pg3 * 3;
    const bool three = pg3 <= 4 && slots3 < slots && (elem_bytes == 2 || (pg3 >= 2 && 10 * pairs < 7 * slots));
    return three ? NarrowShape{pg3, 3} : NarrowShape{pg, cp};
}

// Tile-major round above 32 workers: the chunked kernel (one wavefront per tile of n x 128 bytes), or
// round_kernel_split (a pair of wavefronts per tile, half the row pairs each, column sums exchanged
// through LDS).  The split pays once each half nearly fills a wavefront's 32 row slots; measured at equal
// state size, fp32, fraction of the HBM peak, chunked -> split (fused round / averaging alone / round on
// a gradient buffer): n = 64 0.77 -> 0.80 / 0.82 -> 0.85 / 0.78 -> 0.80, n = 60 0.73 -> 0.76 / 0.79 -> 0.83
// / 0.71 -> 0.76, n = 56 0.75 -> 0.75 / 0.80 -> 0.78 / 0.74 -> 0.76, n = 48 0.76 -> 0.71 / 0.84 -> 0.83 /
// 0.76 -> 0.77.  bf16, where the fused round is bound by the noise arithmetic, loses with it (n = 64:
// 0.75 -> 0.69 fused, 0.79 -> 0.74 on a gradient buffer; only the averaging alone gains, 0.82 -> 0.84),
// and all entry points of one dtype must share one summation order (fused == unfused bit for bit).
inline bool narrow_split(int n, int elem_bytes) { return elem_bytes == 4 && n >= 57; }

// Tile-major gradient averaging: lane groups per tile (a lane holds up to two row pairs, or walks more).
inline int gradavg_lane_groups(int n) {
    const int pairs = (n + 1) / 2, need = (pairs + 1) / 2;
    return need > 4 ? 8 : (need > 2 ? 4 : (need > 1 ? 2 : 1));
}

// Host side of the synthetic gradient noise: the kNoiseGrid radius values sqrt(-2 ln((k + 1/2)/kNoiseGrid))
// and the kNoiseGrid (cos, sin) pairs of 2 pi (a + 1/2)/kNoiseGrid, each the nearest fp32.
void build_noise_cells(float *radius, float *cos_sin);

// Launchers (rps_kernels.hip).  All enqueue on `stream` and return the launch status.
// server_mode: 0 = per-round random permutation of the workers, 1 = worker j serves block j,
// 2 = external servers (no reliable self link; blocks may differ from n)
hipError_t launch_masks(RoundTable *tab, int n, int blocks, uint64_t seed, uint64_t step, uint64_t threshold,
                        int server_mode, hipStream_t stream);
// Mixing-matrix moments of the outcomes of steps first_step .. first_step+rounds-1: out = device
// array of 2*workgroups doubles, workgroup w's sums (over its rounds, all blocks, all rows m of W)
// of sum_k W_mk^2 and of (sum_k W_mk)^2.
hipError_t launch_mixing_moments(double *out, int workgroups, int64_t rounds, int n, int blocks, uint64_t seed,
                                 uint64_t first_step, uint64_t threshold, int server_mode, hipStream_t stream);
hipError_t launch_round(int dtype, int grad_mode, void *X, const void *G, const RoundTable *tab,
                        const RoundParams &prm, int64_t max_block_cols, const LaunchTuning &tune, hipStream_t stream);
// tiles_per_wave: 1 KB steps per wavefront with the in-register gradient; 0: chosen by the launcher
hipError_t launch_local_step(int dtype, int grad_mode, void *X, const void *G,
                             const RoundParams &prm, int tiles_per_wave, hipStream_t stream);

hipError_t launch_gradavg(int dtype, void *X, const void *G, const RoundTable *tab, const RoundParams &prm,
                          int64_t max_block_cols, int max_waves_per_cu, hipStream_t stream);

// Copy between the row-major [n, N] (rows `pitch` elements apart) and the tile-major arrangement of the
// same state (aligned: both bases 16-byte aligned and the pitch a multiple of the 16-byte group, so whole
// groups move at once).
hipError_t launch_convert_layout(int dtype, void *dst, const void *src, int64_t N, int64_t pitch, int n, bool to_tiled,
                                 bool aligned, hipStream_t stream);

// Consensus statistics: partials = device scratch of 2*max_partials doubles, out = 2 device doubles.
constexpr int kMaxPartials = 2048;
hipError_t launch_consensus(int dtype, const void *X, const RoundParams &prm, double *partials, int max_partials,
                            double *out, hipStream_t stream);
// Device address, on GPU `device` (which must be current), of the library's statically allocated
// reduction scratch of 2*kMaxPartials doubles; resolved once per GPU, no allocation.
hipError_t static_scratch(int device, double **out);

}  // namespace rps
