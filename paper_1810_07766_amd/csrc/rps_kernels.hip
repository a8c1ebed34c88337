// HIP kernels (gfx950 / CDNA4, wave64) of the RPS lossy model-averaging round of
// "Distributed Learning over Unreliable Networks" (arXiv 1810.07766), Sec. 4.1 / Alg. 1.
//
// Compile with -ffp-contract=off: the local step and the synthetic-gradient noise are specified as
// exact sequences of IEEE fp32 operations and every fused multiply-add is written explicitly.
//
// Kernels
//   masks_kernel      network outcome of one round: server permutation, uplink and downlink
//                     delivery bits (Sec. 3; Alg. 1 steps 6-7), n workgroups of one wavefront
//                     (the averaging kernels also prepare the following step's outcome)
//   mixing_moments_kernel  Monte-Carlo sums for the constants alpha1, alpha2 of the mixing matrix
//                     (Sec. 4.2), one wavefront per simulated round
//   round_kernel      local SGD step + Reduce-Scatter average + All-Gather write-back in one
//                     pass; every wavefront owns one tile (64 lanes x 16 bytes) of one block
//                     and walks all n rows of it; no data is staged in LDS (the only LDS use is
//                     the shared copy of the noise cells, the only barrier the one that ends it)
//   round_kernel_narrow  the same round on the tile-major layout: a wavefront owns the contiguous
//                     n x 128 bytes of a 128-byte-wide tile, 8 rows per instruction
//   local_step_kernel the local SGD step alone, one row per wavefront (contiguous streams);
//                     local_step_tiled_kernel: the same on the tile-major layout with a gradient
//                     buffer (with the in-register gradient: round_kernel_narrow, nothing delivered)
//   gradavg_kernel    the gradient-averaging comparison of Sec. 6 (same masks applied to G);
//                     gradavg_kernel_narrow: the same on the tile-major layout
//   convert_layout_kernel  copy of a state between the row-major and the tile-major arrangement
//   consensus_kernel  sum_i ||x_i - xbar||^2 and ||xbar||^2 in one streaming read (Lemma 1's quantity)
// The path is a streaming reduction with < 0.5 flop per byte: it is bound by HBM bandwidth
// (with the in-register Gaussian generator also by the LDS gathers of the noise cells and plain
// vector ALU work on the bf16 workloads), never by a dense contraction, so there is no MFMA here.
#include "rps_internal.h"

#include <atomic>
#include <type_traits>

namespace rps {
namespace {

// ---------------------------------------------------------------------------------------
// Counter-based hash: Philox4x32 (Salmon et al., SC'11).  32x32->64 products map to
// v_mad_u64_u32 on gfx9.
// ---------------------------------------------------------------------------------------
template <int ROUNDS>
__device__ __forceinline__ void philox4x32(uint32_t c[4], uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
        if (r > 0) {
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        const uint64_t p0 = (uint64_t)0xD2511F53u * c[0];
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c[2];
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c[1] ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c[3] ^ k1;
        c[1] = (uint32_t)p1;
        c[3] = (uint32_t)p0;
        c[0] = n0;
        c[2] = n2;
    }
}

// A launch dimension holds fewer than 2^32 work-items, so long 1-D ranges of workgroups are folded
// into (x, z): workgroup index = blockIdx.z * gridDim.x + blockIdx.x.
constexpr unsigned kMaxGridX = 1u << 20;
__device__ __forceinline__ int64_t linear_block() { return (int64_t)blockIdx.z * gridDim.x + blockIdx.x; }
__device__ __forceinline__ int64_t linear_blocks() { return (int64_t)gridDim.z * gridDim.x; }
// Index of the unit of work (tile, chunk) that wavefront `wave` of a workgroup of `wpb` wavefronts
// takes in its step `it`.  Workgroups are handed to the 8 XCDs of the chip in turn, and the memory
// system is at its best when CONSECUTIVE units are in flight on DIFFERENT XCDs (measured with an
// in-place copy of 4 KB units: 6.0 TB/s when unit u runs on XCD u mod 8, 5.0 TB/s when every XCD
// works on runs of 16 units).  With one wavefront per workgroup that comes by itself; a workgroup
// of several wavefronts therefore takes units 8 apart -- the units u = 8 q + x of its own XCD x --
// so that unit u still runs on XCD u mod 8 (the launchers round the grid to a multiple of 8
// workgroups).  A wavefront's next step lies a whole grid further on: the chip then works on a few
// compact, forward-moving windows of memory.
__device__ __forceinline__ int64_t unit_index(int it, int wpb, int wave) {
    const int64_t lb = (int64_t)it * linear_blocks() + linear_block();
    return (((lb >> 3) * wpb + wave) << 3) + (lb & 7);
}
inline dim3 folded_grid(int64_t workgroups, unsigned y) {
    const int64_t gx = workgroups < (int64_t)kMaxGridX ? (workgroups > 0 ? workgroups : 1) : (int64_t)kMaxGridX;
    return dim3((unsigned)gx, y, (unsigned)((workgroups + gx - 1) / gx));
}

// For kernels that place their units with unit_index(): a multiple of 8 workgroups.
inline dim3 folded_grid8(int64_t workgroups, unsigned y) { return folded_grid((workgroups + 7) & ~(int64_t)7, y); }

constexpr uint32_t kDomainUplink = 0u << 24, kDomainDownlink = 1u << 24, kDomainServer = 2u << 24,
                   kDomainNoise = 3u << 24;
constexpr int kMaskRounds = 10;   // network outcome: the generator's standard round count
constexpr int kNoiseRounds = 7;   // gradient noise: the smallest count its authors report as passing BigCrush

// ---------------------------------------------------------------------------------------
// Network outcome (Sec. 3: every message lost independently with probability p; Alg. 1
// step 6: servers drawn uniformly without replacement).  Workgroup j = block j, lane i =
// worker i.  The permutation is a rank sort of per-worker hash keys: natively parallel,
// n compare steps through wavefront shuffles.
// ---------------------------------------------------------------------------------------
// Server of block j for this lane's round: the worker whose hash key has rank j (lane i = worker i).
__device__ __forceinline__ int draw_server(int n, int i, int j, uint32_t key) {
    int rank = 0;
    for (int k = 0; k < n; ++k) {
        const uint32_t other = __shfl(key, k, 64);
        rank += (other < key || (other == key && k < i)) ? 1 : 0;
    }
    const uint64_t hit = __ballot(i < n && rank == j);
    return __ffsll((long long)hit) - 1;   // exactly one lane has rank j
}

__device__ __forceinline__ uint32_t server_key(int i, uint32_t seed_lo, uint32_t seed_hi, uint32_t step_lo,
                                               uint32_t step_hi24) {
    uint32_t c[4] = {(uint32_t)i, 0u, step_lo, kDomainServer | step_hi24};
    philox4x32<kMaskRounds>(c, seed_lo, seed_hi);
    return c[0];
}

// Delivery bits of block j (one bit per worker) with server s (-1: external, no reliable link).
__device__ __forceinline__ void draw_links(int n, int i, int j, int s, uint32_t seed_lo, uint32_t seed_hi,
                                           uint32_t step_lo, uint32_t step_hi24, uint64_t threshold,
                                           uint64_t &ucol, uint64_t &dcol) {
    const bool active = i < n;
    uint32_t cu[4] = {(uint32_t)i, (uint32_t)j, step_lo, kDomainUplink | step_hi24};
    philox4x32<kMaskRounds>(cu, seed_lo, seed_hi);
    uint32_t cd[4] = {(uint32_t)i, (uint32_t)j, step_lo, kDomainDownlink | step_hi24};
    philox4x32<kMaskRounds>(cd, seed_lo, seed_hi);
    // a worker's link to itself is not a network message: forced after the draw
    ucol = __ballot(active && ((uint64_t)cu[0] >= threshold || i == s));
    dcol = __ballot(active && ((uint64_t)cd[0] >= threshold || i == s));
}

// Outcome of block j for one round, computed by one full wavefront (lane i = worker i) and written
// to `tab` by lane 0.
__device__ __forceinline__ void write_block_outcome(RoundTable *__restrict__ tab, int n, int j, int i, uint32_t seed_lo,
                                                    uint32_t seed_hi, uint32_t step_lo, uint32_t step_hi24,
                                                    uint64_t threshold, int server_mode) {
    // external parameter servers (the paper's Fig. 1) are not workers: no lane is the server
    int s = server_mode == 2 ? -1 : j;
    if (server_mode == 0) s = draw_server(n, i, j, server_key(i, seed_lo, seed_hi, step_lo, step_hi24));

    uint64_t ucol, dcol;
    draw_links(n, i, j, s, seed_lo, seed_hi, step_lo, step_hi24, threshold, ucol, dcol);
    if (i == 0) {
        const int cnt = __popcll(ucol);
        tab->ucol[j] = ucol;
        tab->dcol_drawn[j] = dcol;
        // an external server that received nothing has nothing to send: nobody overwrites
        tab->dcol[j] = cnt > 0 ? dcol : 0;
        tab->cnt[j] = cnt;
        tab->inv_cnt[j] = cnt > 0 ? 1.0 / (double)cnt : 0.0;
        tab->server[j] = s;
    }
}

__global__ __launch_bounds__(64) void masks_kernel(RoundTable *__restrict__ tab, int n, uint32_t seed_lo,
                                                   uint32_t seed_hi, uint32_t step_lo, uint32_t step_hi24,
                                                   uint64_t threshold, int server_mode) {
    write_block_outcome(tab, n, blockIdx.x, threadIdx.x, seed_lo, seed_hi, step_lo, step_hi24, threshold, server_mode);
}

// The averaging kernels also prepare the NEXT round's outcome (rounds usually come with consecutive
// steps): the first wavefront of every block's grid row writes block j's outcome for step + 1 into
// the other table, so that the next call needs no separate mask launch.  prm.next_tab == nullptr:
// not wanted.  `first` must be wave-uniform and true for exactly one full wavefront per block.
__device__ __forceinline__ void prepare_next_outcome(const RoundParams &prm, bool first, int j, int lane) {
    if (prm.next_tab != nullptr && first)
        write_block_outcome(prm.next_tab, prm.n, j, lane, prm.seed_lo, prm.seed_hi, prm.next_step_lo, prm.next_step_hi24,
                            prm.threshold, prm.server_mode);
}

// ---------------------------------------------------------------------------------------
// Monte-Carlo moments of the mixing matrix W of X_{t+1} = V_t W_t (Sec. 4.2): entry (m,k) of
// a block's W is the weight of v_m in x'_k, i.e. 1/c if m reached the server and the reply
// reached k, plus 1 on the diagonal if the reply did not reach k.  Row m therefore has
//   sum_k W_mk   = U_m d / c + (1 - D_m),      sum_k W_mk^2 = U_m d / c^2 + (1 - D_m)
// with c copies received and d replies delivered.  Lane m = worker m; workgroup w takes rounds
// first_step + w, + w + gridDim.x, ... and writes out[2w] = its sum over rounds, blocks and rows
// of sum_k W_mk^2, out[2w+1] = of (sum_k W_mk)^2.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void mixing_moments_kernel(double *__restrict__ out, int64_t rounds, int n,
                                                            int blocks, uint32_t seed_lo, uint32_t seed_hi,
                                                            uint64_t first_step, uint64_t threshold,
                                                            int server_mode) {
    const int m = threadIdx.x;
    double sq = 0.0, sum_sq = 0.0;
    for (int64_t r = blockIdx.x; r < rounds; r += gridDim.x) {
        const uint64_t step = first_step + (uint64_t)r;
        const uint32_t step_lo = (uint32_t)step, step_hi24 = (uint32_t)((step >> 32) & 0xFFFFFFu);
        const uint32_t key = server_mode == 0 ? server_key(m, seed_lo, seed_hi, step_lo, step_hi24) : 0u;
        for (int j = 0; j < blocks; ++j) {
            int s = server_mode == 2 ? -1 : j;
            if (server_mode == 0) s = draw_server(n, m, j, key);
            uint64_t ucol, dcol;
            draw_links(n, m, j, s, seed_lo, seed_hi, step_lo, step_hi24, threshold, ucol, dcol);
            const int c = __popcll(ucol);
            if (c == 0) dcol = 0;   // nothing to send: W = I for this block
            const double d = (double)__popcll(dcol);
            const double um = (double)((ucol >> m) & 1), keep = 1.0 - (double)((dcol >> m) & 1);
            const double inv = c > 0 ? 1.0 / (double)c : 0.0;
            const double row_sum = um * d * inv + keep;
            if (m < n) {
                sq += um * d * inv * inv + keep;
                sum_sq += row_sum * row_sum;
            }
        }
    }
    for (int o = 32; o > 0; o >>= 1) {
        sq += __shfl_xor(sq, o, 64);
        sum_sq += __shfl_xor(sum_sq, o, 64);
    }
    if (m == 0) {
        out[2 * (size_t)blockIdx.x] = sq;
        out[2 * (size_t)blockIdx.x + 1] = sum_sq;
    }
}

// ---------------------------------------------------------------------------------------
// Synthetic gradient noise: a Box-Muller pair per 32-bit hash word on a 4096 x 4096 grid of
// (radius, angle) cells.  The cell values (correctly rounded fp32 of sqrt(-2 ln((k + 1/2)/4096)),
// cos and sin of 2 pi (a + 1/2)/4096) come from a table the host computes, the radii multiplied by
// sigma (one more rounding) when sigma is set; every workgroup of a kernel that generates noise
// copies it into LDS, so that a pair costs one mask, one shift-and-mask, one bit-field insert, two
// LDS gathers and two multiplies.
//   word bits 2..13  -> radius cell (one 4-byte LDS read)
//   word bits 17..27 -> angle cell within the half turn (one 8-byte LDS read of the (cos, sin) entry:
//                       the table is an aligned float2 array so that the compiler emits ds_read_b64,
//                       not two dword reads that each pay their own bank conflicts: +1.2 % on the
//                       bf16 / 64-worker round);  bit 31 adds the half turn, i.e. flips the sign of
//                       both members: LDS holds only the 2048 cells of the first half turn, and the
//                       bit is copied into the sign of sigma * r >= 0 by one bit-field insert
// ---------------------------------------------------------------------------------------
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct alignas(16) NoiseLds {
    float radius[kNoiseGrid];        // sigma * r, rounded once
    float2 dir[kNoiseGrid / 2];      // (cos, sin) of the kNoiseGrid / 2 angle cells below pi: one 8-byte read per pair
};
struct NoNoiseLds {
    float unused;
};
template <int GRAD>
struct LdsFor {
    using type = NoNoiseLds;
};
template <>
struct LdsFor<kGradSynthetic> {
    using type = NoiseLds;
};

// Copy of the context's 32 KB of cells (sigma * radius[4096], then the (cos, sin) pairs of the 2048
// angle cells below pi) into the workgroup's LDS by LDS-direct loads: a wavefront instruction moves
// 64 lanes x 16 bytes from global memory straight into 1 KB of LDS (no registers), the 32
// instructions are dealt out to the workgroup's wavefronts.  begin() only issues them; end() waits
// for this wavefront's share and ends with the workgroup barrier, so what a wavefront issues in
// between -- the loads of its first tile -- is in flight during the copy.  Every wavefront of the
// workgroup must pass begin() and end() exactly once.
template <int WPB>
__device__ __forceinline__ void noise_fill_begin(NoiseLds &lds, const float *__restrict__ cells, int wave, int lane) {
    constexpr int kPieces = (int)(sizeof(NoiseLds) / 1024);
    float *dst = reinterpret_cast<float *>(&lds);
#pragma unroll
    for (int c = 0; c < (kPieces + WPB - 1) / WPB; ++c) {
        const int piece = c * WPB + wave;   // wave-uniform
        if (piece < kPieces)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(cells + piece * 256 + lane * 4),
                                             (__attribute__((address_space(3))) void *)(dst + piece * 256), 16, 0, 0);
    }
}
// PENDING = vector memory instructions this wavefront has issued since noise_fill_begin() (its first
// tile's loads): the memory counter retires in order, so waiting until only PENDING operations are
// outstanding waits for the copy and leaves those loads in flight -- the workgroup barrier then
// does not line the wavefronts up on their tile loads, and the noise of the first tile is computed
// under their latency like that of every later one.  (A __syncthreads() here makes the compiler
// drain the whole memory queue first.)
template <int PENDING>
__device__ __forceinline__ void noise_fill_end(NoiseLds &) {
    static_assert(PENDING >= 0 && PENDING < 64, "the counter holds 6 bits");
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(PENDING) : "memory");
}
template <int WPB>
__device__ __forceinline__ void noise_fill_begin(NoNoiseLds &, const float *, int, int) {}
template <int PENDING>
__device__ __forceinline__ void noise_fill_end(NoNoiseLds &) {}

__device__ __forceinline__ void box_muller_pair(uint32_t word, const NoiseLds &lds, float &even, float &odd) {
    const float r = lds.radius[(word >> 2) & (kNoiseGrid - 1)];
    const float2 d = lds.dir[(word >> 17) & (kNoiseGrid / 2 - 1)];
    // sign bit from the word, the rest from r (v_bfi_b32): -(r * c) is the rounded r * -c exactly
    const float rs = __uint_as_float((__float_as_uint(r) & 0x7FFFFFFFu) | (word & 0x80000000u));
    even = rs * d.x;
    odd = rs * d.y;
}

// One hash call serves a 4-column x 2-worker patch: words 0,1 -> worker 2*pair, words 2,3 ->
// worker 2*pair+1, columns 4*quad..4*quad+3 (16 bytes of fp32 per row: one lane's vector).  The
// counter is (quad >> 7, (quad & 127) | pair << 7, step, domain): the callers pass quad >> 7 as
// quad_hi -- wave-uniform wherever a wavefront's columns lie inside one aligned run of 512, so
// that the first hash rounds are partly scalar work -- and the low seven bits as quad_lo.
__device__ __forceinline__ void noise_patch(const RoundParams &prm, const NoiseLds &lds, int pair, uint32_t quad_hi,
                                            uint32_t quad_lo, float za[4], float zb[4]) {
    uint32_t c[4] = {quad_hi, quad_lo | ((uint32_t)pair << 7), prm.step_lo, kDomainNoise | prm.step_hi24};
    philox4x32<kNoiseRounds>(c, prm.seed_lo, prm.seed_hi);
    box_muller_pair(c[0], lds, za[0], za[1]);
    box_muller_pair(c[1], lds, za[2], za[3]);
    box_muller_pair(c[2], lds, zb[0], zb[1]);
    box_muller_pair(c[3], lds, zb[2], zb[3]);
}
__device__ __forceinline__ void noise_patch(const RoundParams &, const NoNoiseLds &, int, uint32_t, uint32_t, float *,
                                            float *) {}

// ---------------------------------------------------------------------------------------
// Storage formats: fp32, or bf16 bit patterns with round-to-nearest-even on every store.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x0040u;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// 128-bit accesses carry the non-temporal hint: the state is far larger than the caches and
// every element is touched once per round, so nothing is gained by keeping lines resident.
// One lane's vector is 16 bytes (Raw): 4 fp32 columns or 8 bf16 columns.  Rows wait in
// registers in Raw form and are unpacked to fp32 only when they are processed.
template <typename ST>
struct Storage;

template <>
struct Storage<float> {
    static constexpr int VEC = 4;
    using Raw = f32x4;
    using Acc = double;   // column sums of fp32 values are taken in fp64
    static __device__ __forceinline__ float round(float v) { return v; }
    static __device__ __forceinline__ void unpack(Raw a, float x[VEC]) {
        x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
    }
    static __device__ __forceinline__ Raw pack(const float x[VEC]) {
        const Raw a = {x[0], x[1], x[2], x[3]};
        return a;
    }
    // round x to storage in place and return it packed (fp32: nothing to round)
    static __device__ __forceinline__ Raw round_vec(float x[VEC]) { return pack(x); }
    static __device__ __forceinline__ float load1(const float *p) { return *p; }
    static __device__ __forceinline__ void store1(float *p, float v) { *p = v; }
};

template <>
struct Storage<uint16_t> {
    static constexpr int VEC = 8;
    using Raw = u32x4;
    using Acc = double;   // the same for bf16 values: an fp32 sum is under 1 % faster on the 64-worker workload (measured),
                          // and its rounding flips about one stored bf16 result in 1e5 against the fp64 definition
    static __device__ __forceinline__ float round(float v) { return bf16_bits_to_f32(f32_to_bf16_bits(v)); }
    static __device__ __forceinline__ void unpack(Raw a, float x[VEC]) {
        x[0] = __uint_as_float(a.x << 16); x[1] = __uint_as_float(a.x & 0xFFFF0000u);
        x[2] = __uint_as_float(a.y << 16); x[3] = __uint_as_float(a.y & 0xFFFF0000u);
        x[4] = __uint_as_float(a.z << 16); x[5] = __uint_as_float(a.z & 0xFFFF0000u);
        x[6] = __uint_as_float(a.w << 16); x[7] = __uint_as_float(a.w & 0xFFFF0000u);
    }
    // for values that are already bf16-representable (rounded by round()): a truncation
    static __device__ __forceinline__ Raw pack(const float x[VEC]) {
        Raw a;
        a.x = (__float_as_uint(x[0]) >> 16) | (__float_as_uint(x[1]) & 0xFFFF0000u);
        a.y = (__float_as_uint(x[2]) >> 16) | (__float_as_uint(x[3]) & 0xFFFF0000u);
        a.z = (__float_as_uint(x[4]) >> 16) | (__float_as_uint(x[5]) & 0xFFFF0000u);
        a.w = (__float_as_uint(x[6]) >> 16) | (__float_as_uint(x[7]) & 0xFFFF0000u);
        return a;
    }
    // round x to bf16 (nearest even) in place and return the packed bits: one hardware
    // conversion (v_cvt_pk_bf16_f32) per pair of values, then re-widened for the fp64 sums
    static __device__ __forceinline__ Raw round_vec(float x[VEC]) {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        uint32_t w[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const f32x2 v = {x[2 * k], x[2 * k + 1]};
            const bf16x2 r = __builtin_convertvector(v, bf16x2);
            __builtin_memcpy(&w[k], &r, 4);
            x[2 * k] = __uint_as_float(w[k] << 16);
            x[2 * k + 1] = __uint_as_float(w[k] & 0xFFFF0000u);
        }
        const Raw a = {w[0], w[1], w[2], w[3]};
        return a;
    }
    static __device__ __forceinline__ float load1(const uint16_t *p) { return bf16_bits_to_f32(*p); }
    static __device__ __forceinline__ void store1(uint16_t *p, float v) { *p = (uint16_t)(__float_as_uint(v) >> 16); }
};

// Where one lane works: VEC columns [c0, c0+VEC) of the column range [lo, hi), c0 = tile0 + loff
// with tile0 wave-uniform and loff = lane * VEC.  Row pointers handed to load_raw / store_raw
// already include tile0 (wave-uniform base + 32-bit lane offset: no per-lane 64-bit address
// arithmetic).  In a FULL wavefront every lane's vector lies inside the range and is 16-byte
// aligned: one 128-bit access per row and no per-lane test (keeps all loads of a row chunk in
// one basic block, in flight together).  Otherwise (block edges, unaligned pitch) lanes touch
// only their own columns inside the range, element by element.
struct LaneCols {
    int64_t tile0, lo, hi;
    uint32_t loff;
    __device__ __forceinline__ int64_t c0() const { return tile0 + loff; }
    // noise counter of the lane's first quad: tile0 is a multiple of the wavefront's tile width (at
    // most 512 columns, a divisor of 512), so the high part is wave-uniform
    __device__ __forceinline__ uint32_t quad_hi() const { return (uint32_t)(tile0 >> 9); }
    __device__ __forceinline__ uint32_t quad_lo() const { return ((uint32_t)(tile0 >> 2) & 127u) + (loff >> 2); }
};

template <typename ST, bool FULL>
__device__ __forceinline__ typename Storage<ST>::Raw load_raw(const ST *tile_row, const LaneCols &lc) {
    using S = Storage<ST>;
    if (FULL) {
        return __builtin_nontemporal_load(reinterpret_cast<const typename S::Raw *>(tile_row + lc.loff));
    } else {
        float x[S::VEC];
#pragma unroll
        for (int e = 0; e < S::VEC; ++e) {
            const int64_t c = lc.c0() + e;
            x[e] = (c >= lc.lo && c < lc.hi) ? S::load1(tile_row + lc.loff + e) : 0.0f;
        }
        return S::pack(x);
    }
}
template <typename ST, bool FULL>
__device__ __forceinline__ void store_raw(ST *tile_row, const LaneCols &lc, typename Storage<ST>::Raw v) {
    using S = Storage<ST>;
    if (FULL) {
        // Streaming store with the "sc1 nt" cache policy, measured 1.5 % faster on the in-place
        // row walk than the plain non-temporal global store.  Only buffer stores let the policy
        // be chosen from C++: the row's 1 KB tile segment is described by a raw buffer resource
        // (wave-uniform base, hardware bounds check at 64 lanes x 16 bytes) + the lane offset.
        constexpr int kAuxSc1Nt = (1 << 4) | (1 << 1);
        const __amdgpu_buffer_rsrc_t rsrc =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<ST *>(tile_row), 0, 64 * 16, 0x00020000);
        u32x4 bits;
        __builtin_memcpy(&bits, &v, sizeof(bits));
        __builtin_amdgcn_raw_buffer_store_b128(bits, rsrc, (int)(lc.loff * (uint32_t)sizeof(ST)), 0, kAuxSc1Nt);
    } else {
        float x[S::VEC];
        S::unpack(v, x);
#pragma unroll
        for (int e = 0; e < S::VEC; ++e) {
            const int64_t c = lc.c0() + e;
            if (c >= lc.lo && c < lc.hi) S::store1(tile_row + lc.loff + e, x[e]);
        }
    }
}

// Noise of the lane's VEC columns for the worker pair (2*pair, 2*pair+1).
template <int VEC, typename LDS>
__device__ __forceinline__ void noise_rows(const RoundParams &prm, const LDS &lds, int pair, uint32_t quad_hi,
                                           uint32_t quad_lo, float za[VEC], float zb[VEC]) {
#pragma unroll
    for (int q = 0; q < VEC / 4; ++q) noise_patch(prm, lds, pair, quad_hi, quad_lo + q, za + 4 * q, zb + 4 * q);
}

// v = x - gamma * g, rounded to storage (Alg. 1 step 5); g = the caller's gradient or
// lambda * x + noise.  x is overwritten by v; the packed form of v is returned.
template <typename ST, int GRAD>
__device__ __forceinline__ typename Storage<ST>::Raw sgd_step(const RoundParams &prm, const float *g_or_z,
                                                              float x[Storage<ST>::VEC]) {
    constexpr int VEC = Storage<ST>::VEC;
    if (GRAD == kGradSynthetic && prm.lambda != 0.0f) {   // fma(0, x, z) == z for finite x: skipped without decay
#pragma unroll
        for (int e = 0; e < VEC; ++e)
            x[e] = __builtin_fmaf(-prm.gamma, __builtin_fmaf(prm.lambda, x[e], g_or_z[e]), x[e]);
    } else if (GRAD != kGradNone) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) x[e] = __builtin_fmaf(-prm.gamma, g_or_z[e], x[e]);
    }
    if (GRAD == kGradNone) return Storage<ST>::pack(x);   // loaded from storage: already representable
    return Storage<ST>::round_vec(x);
}

// ---------------------------------------------------------------------------------------
// Fused round.  grid = (ceil(tiles of the largest block / WPB), n blocks); a workgroup is WPB
// independent wavefronts, each owning one tile of 64 x VEC columns of block j (tiles sit on
// absolute multiples of the tile width, so every wavefront access is one aligned 1 KB segment
// whatever the block offsets are, and lanes coincide with 16-byte segments and noise quads;
// the first and last tile of a block may be partial).  The wavefront walks the n rows of its tile:
//   pass 1  read x[i, tile], form v (Alg. 1 step 5); if worker i's copy reached the server
//           (uplink bit) add it to the fp64 column sums; if the reply will not reach worker i
//           (downlink bit clear) its final value is v: store it now
//   pass 2  vt = sum / |N_j| once per column; store vt to every row whose downlink bit is set
// Every element is read once and written once; no state data is staged in LDS (only the noise cells
// live there, and the one barrier of a workgroup is the one that ends their copy).
// Delivery tests are wave-uniform scalar branches (row index and mask words live in SGPRs).
// All receivers get the same registers, so they hold identical bits.
// ---------------------------------------------------------------------------------------

// Running position of the loads: the next row to load and its tile pointer(s).  Rows past n
// repeat row n-1 (loaded, never used), so every load of a chunk is unconditional.
template <typename ST>
struct LoadCursor {
    const ST *x, *g;
    int row;
};

template <typename ST, int GRAD, int R, bool FULL>
__device__ __forceinline__ void load_chunk(LoadCursor<ST> &cur, const RoundParams &prm, const LaneCols &lc,
                                           typename Storage<ST>::Raw x[R],
                                           typename Storage<ST>::Raw g[GRAD == kGradBuffer ? R : 1]) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
        x[r] = load_raw<ST, FULL>(cur.x, lc);
        if (GRAD == kGradBuffer) g[r] = load_raw<ST, FULL>(cur.g, lc);
        if (cur.row + 1 < prm.n) {   // scalar
            ++cur.row;
            cur.x += prm.stride;
            if (GRAD == kGradBuffer) cur.g += prm.stride;
        }
    }
}

// Pass 1 for the chunk of rows i0..i0+R-1: v for every row that needs it, column sums, and
// the final value of the rows that will not receive the reply.
template <typename ST, int GRAD, int R, bool FULL, typename LDS>
__device__ __forceinline__ void process_chunk(ST *__restrict__ Xt, const RoundParams &prm, const LDS &lds,
                                              const LaneCols &lc, uint64_t ucol, uint64_t dcol, int i0,
                                              const typename Storage<ST>::Raw xr[R],
                                              const typename Storage<ST>::Raw gr[GRAD == kGradBuffer ? R : 1],
                                              typename Storage<ST>::Acc acc[Storage<ST>::VEC]) {
    using S = Storage<ST>;
    using Acc = typename S::Acc;
    constexpr int VEC = S::VEC;
    const int n = prm.n;
#pragma unroll
    for (int r = 0; r < R; r += 2) {   // worker pairs (i0 is even)
        const int ia = i0 + r, ib = ia + 1;
        if (ia < n) {
            const bool ua = (ucol >> ia) & 1, da = (dcol >> ia) & 1;
            const bool ub = ib < n && ((ucol >> ib) & 1), db = ib >= n || ((dcol >> ib) & 1);
            // v is needed if it enters the average or stays as the worker's own value
            const bool need_a = ua || (GRAD != kGradNone && !da);
            const bool need_b = ub || (GRAD != kGradNone && !db);
            if (need_a || need_b) {
                float za[VEC], zb[VEC];
                if (GRAD == kGradSynthetic) noise_rows<VEC>(prm, lds, ia >> 1, lc.quad_hi(), lc.quad_lo(), za, zb);
                if (need_a) {
                    float v[VEC];
                    S::unpack(xr[r], v);
                    if (GRAD == kGradBuffer) S::unpack(gr[GRAD == kGradBuffer ? r : 0], za);
                    const typename S::Raw vr = sgd_step<ST, GRAD>(prm, za, v);
                    if (ua) {
#pragma unroll
                        for (int e = 0; e < VEC; ++e) acc[e] += (Acc)v[e];
                    }
                    if (GRAD != kGradNone && !da) store_raw<ST, FULL>(Xt + (int64_t)ia * prm.stride, lc, vr);
                }
                if (need_b) {
                    float v[VEC];
                    S::unpack(xr[r + 1], v);
                    if (GRAD == kGradBuffer) S::unpack(gr[GRAD == kGradBuffer ? r + 1 : 0], zb);
                    const typename S::Raw vr = sgd_step<ST, GRAD>(prm, zb, v);
                    if (ub) {
#pragma unroll
                        for (int e = 0; e < VEC; ++e) acc[e] += (Acc)v[e];
                    }
                    if (GRAD != kGradNone && !db) store_raw<ST, FULL>(Xt + (int64_t)ib * prm.stride, lc, vr);
                }
            }
        }
    }
    // A row that was skipped above has never been waited for.  Consume every register of the
    // chunk here, so that no load is still pending on them when the caller's loop issues the
    // next loads into the same registers (otherwise the compiler must drain the whole memory
    // queue at the loop head, which serialises the prefetch).
#pragma unroll
    for (int r = 0; r < R; ++r) asm volatile("" ::"v"(xr[r]));
    if (GRAD == kGradBuffer) {
#pragma unroll
        for (int r = 0; r < R; ++r) asm volatile("" ::"v"(gr[r]));
    }
}

// One tile, all n rows.  The row loop is software-pipelined by hand: the loads of chunk k+1
// are issued before chunk k is processed, so a wavefront overlaps its own memory latency with
// its own arithmetic and few resident wavefronts suffice.
// after_first_loads(count) is called once the first chunk's loads are issued, with their number
// (see noise_fill_end).
template <typename ST, int GRAD, int R, bool FULL, typename LDS, typename F>
__device__ __forceinline__ void round_tile(ST *__restrict__ X, const ST *__restrict__ G, const RoundParams &prm,
                                           const LDS &lds, const LaneCols &lc, uint64_t ucol, uint64_t dcol, double inv,
                                           const F &after_first_loads) {
    using S = Storage<ST>;
    using Acc = typename S::Acc;
    using Raw = typename S::Raw;
    constexpr int VEC = S::VEC;
    constexpr int RG = GRAD == kGradBuffer ? R : 1;
    const int n = prm.n;
    ST *Xt = X + lc.tile0;   // row 0 of the tile (wave-uniform)

    Acc acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0;

    LoadCursor<ST> cur;
    cur.x = Xt;
    cur.g = GRAD == kGradBuffer ? G + lc.tile0 : nullptr;
    cur.row = 0;
    Raw xa[R], xb[R], ga[RG], gb[RG];
    load_chunk<ST, GRAD, R, FULL>(cur, prm, lc, xa, ga);
    after_first_loads(std::integral_constant<int, FULL ? (GRAD == kGradBuffer ? 2 : 1) * R : 0>{});
    int i0 = 0;
    // steady state: every load is unconditional, so the number of requests in flight at each
    // point is static and the waits inserted by the compiler leave the prefetch outstanding
    for (; i0 + 2 * R < n; i0 += 2 * R) {
        load_chunk<ST, GRAD, R, FULL>(cur, prm, lc, xb, gb);
        process_chunk<ST, GRAD, R, FULL>(Xt, prm, lds, lc, ucol, dcol, i0, xa, ga, acc);
        load_chunk<ST, GRAD, R, FULL>(cur, prm, lc, xa, ga);
        process_chunk<ST, GRAD, R, FULL>(Xt, prm, lds, lc, ucol, dcol, i0 + R, xb, gb, acc);
    }
    if (i0 + R < n) {   // two chunks left
        load_chunk<ST, GRAD, R, FULL>(cur, prm, lc, xb, gb);
        process_chunk<ST, GRAD, R, FULL>(Xt, prm, lds, lc, ucol, dcol, i0, xa, ga, acc);
        process_chunk<ST, GRAD, R, FULL>(Xt, prm, lds, lc, ucol, dcol, i0 + R, xb, gb, acc);
    } else {            // one chunk left
        process_chunk<ST, GRAD, R, FULL>(Xt, prm, lds, lc, ucol, dcol, i0, xa, ga, acc);
    }

    float vt[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) vt[e] = (float)(acc[e] * (Acc)inv);
    const Raw vt_raw = S::round_vec(vt);
    ST *row = Xt;
    for (int i = 0; i < n; ++i, row += prm.stride)
        if ((dcol >> i) & 1) store_raw<ST, FULL>(row, lc, vt_raw);
}

template <typename ST, int GRAD, int R, int WPB>
__global__ __launch_bounds__(WPB * 64) void round_kernel(ST *__restrict__ X, const ST *__restrict__ G,
                                                         const RoundTable *__restrict__ tab, const RoundParams prm) {
    constexpr int VEC = Storage<ST>::VEC;
    constexpr int TILE = 64 * VEC;
    __shared__ typename LdsFor<GRAD>::type lds;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int j = blockIdx.y;
    // the noise cells travel to LDS while the first tile's loads are in flight (as in
    // round_kernel_narrow): every wavefront passes the copy's barrier exactly once
    noise_fill_begin<WPB>(lds, prm.noise_cells, wave, lane);
    bool fill_pending = true;
    const auto finish_fill = [&](auto pending) {
        if (fill_pending) noise_fill_end<decltype(pending)::value>(lds);
        fill_pending = false;
    };
    const int64_t lo = tab->off[j], hi = tab->off[j + 1];
    const uint64_t ucol = tab->ucol[j], dcol = tab->dcol[j];
    const double inv = tab->inv_cnt[j];
    // a wavefront takes tiles_per_wave tiles, a whole grid apart (the workgroup's wavefronts stay on
    // adjacent tiles): the LDS copy of the noise cells is paid once per WPB * tiles_per_wave tiles
    for (int it = 0; it < prm.tiles_per_wave; ++it) {
        const int64_t tile0 = (lo / TILE) * TILE + unit_index(it, WPB, wave) * TILE;
        if (tile0 >= hi) break;   // wave-uniform: this block has fewer tiles than the largest one
        LaneCols lc;
        lc.tile0 = tile0;
        lc.loff = (uint32_t)lane * VEC;
        lc.lo = lo;
        lc.hi = hi;
        if (prm.vec_ok && tile0 >= lo && tile0 + TILE <= hi)   // wave-uniform
            round_tile<ST, GRAD, R, true>(X, G, prm, lds, lc, ucol, dcol, inv, finish_fill);
        else
            round_tile<ST, GRAD, 2, false>(X, G, prm, lds, lc, ucol, dcol, inv, finish_fill);
    }
    finish_fill(std::integral_constant<int, 0>{});
    prepare_next_outcome(prm, linear_block() == 0 && wave == 0, j, lane);
}

// ---------------------------------------------------------------------------------------
// Narrow tiles (the tile-major layout): the same round with LPR = 8 lanes per row segment.  A tile
// is LPR x 16 = 128 bytes wide and its n rows are adjacent in memory; one wavefront instruction
// covers 64 / LPR = 8 row segments (lane group = lane / LPR), and a lane owns row pairs of its
// 16-byte column group, so that the noise hash of a (4 columns x 2 rows) patch still serves one
// lane.  A wavefront then reads only about 4 KB of consecutive memory before it writes it back
// (one tile of 32 workers, or several adjacent tiles of fewer), against 32 KB spread over 32 rows
// in the row-major kernel -- which is what the memory system rewards.  Column sums: every lane
// group sums its own rows in ascending order, the groups of a tile are then combined by a
// butterfly over the lanes (a fixed order, the same for every receiver, but not the plain
// ascending order of the row-major kernel).
// ---------------------------------------------------------------------------------------
constexpr int kTiledLanes = 8;   // lanes per row segment of the tiled layout: 8 x 16 B = 128 B (RPS_TILE_BYTES)

// Access to the lane's 16-byte group of one row segment: `base` is wave-uniform, `eoff` the lane's
// element offset from it.  FULL: one 128-bit access through a raw buffer resource of `limit` bytes
// built on `base` (SGPR base + 32-bit VGPR offset: no per-lane 64-bit address arithmetic; the
// hardware drops accesses at or beyond `limit`: loads return 0, stores do nothing; loads
// non-temporal, stores with the sc1 nt streaming policy).  Otherwise element by element inside
// [lo, hi).
template <typename ST, bool FULL>
__device__ __forceinline__ typename Storage<ST>::Raw load_seg(const ST *base, uint32_t eoff, uint32_t limit, int64_t c0,
                                                              int64_t lo, int64_t hi) {
    using S = Storage<ST>;
    if (FULL) {
        constexpr int kAuxNt = 1 << 1;
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<ST *>(base), 0, (int)limit, 0x00020000);
        const u32x4 bits = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)(eoff * (uint32_t)sizeof(ST)), 0, kAuxNt);
        typename S::Raw v;
        __builtin_memcpy(&v, &bits, sizeof(v));
        return v;
    } else {
        const ST *p = base + eoff;
        float x[S::VEC];
#pragma unroll
        for (int e = 0; e < S::VEC; ++e) x[e] = (c0 + e >= lo && c0 + e < hi) ? S::load1(p + e) : 0.0f;
        return S::pack(x);
    }
}
template <typename ST, bool FULL>
__device__ __forceinline__ void store_seg(ST *base, uint32_t eoff, uint32_t limit, int64_t c0, int64_t lo, int64_t hi,
                                          typename Storage<ST>::Raw v) {
    using S = Storage<ST>;
    if (FULL) {
        constexpr int kAuxSc1Nt = (1 << 4) | (1 << 1);
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(base, 0, (int)limit, 0x00020000);
        u32x4 bits;
        __builtin_memcpy(&bits, &v, sizeof(bits));
        __builtin_amdgcn_raw_buffer_store_b128(bits, rsrc, (int)(eoff * (uint32_t)sizeof(ST)), 0, kAuxSc1Nt);
    } else {
        ST *p = base + eoff;
        float x[S::VEC];
        S::unpack(v, x);
#pragma unroll
        for (int e = 0; e < S::VEC; ++e)
            if (c0 + e >= lo && c0 + e < hi) S::store1(p + e, x[e]);
    }
}

// Sum of a double over the PG lane groups (of 8 lanes each) that share a tile, left in every one of
// them -- the same additions in the same order as a butterfly of __shfl_xor steps over lane distances
// 8, 16 and 32 (a + b for the pair of groups, whichever lane computes it), but through the
// cross-lane VALU paths instead of three dependent LDS permutes per 32-bit half:
//   distance 8   DPP row rotate by 8 within each row of 16 lanes
//   distance 16  v_permlane16_swap(x, x): rows 0,1 <- (row 0, row 1), rows 2,3 <- (row 2, row 3)
//   distance 32  v_permlane32_swap(x, x): both halves <- (lanes 0-31, lanes 32-63)
// Used where the kernel also keeps the LDS busy with noise gathers (bf16, 64 workers: +2.5 %; it
// is not faster where the LDS is otherwise idle).
__device__ __forceinline__ double pair_to_double(uint32_t lo, uint32_t hi) {
    const uint64_t b = ((uint64_t)hi << 32) | lo;
    double d;
    __builtin_memcpy(&d, &b, 8);
    return d;
}
template <int PG>
__device__ __forceinline__ double sum_lane_groups(double a) {
    uint64_t b;
    if (PG >= 2) {
        __builtin_memcpy(&b, &a, 8);
        constexpr int kRowRotate8 = 0x128;
        const uint32_t lo = __builtin_amdgcn_update_dpp(0u, (uint32_t)b, kRowRotate8, 0xf, 0xf, false);
        const uint32_t hi = __builtin_amdgcn_update_dpp(0u, (uint32_t)(b >> 32), kRowRotate8, 0xf, 0xf, false);
        a += pair_to_double(lo, hi);
    }
    if (PG >= 4) {
        __builtin_memcpy(&b, &a, 8);
        const auto lo = __builtin_amdgcn_permlane16_swap((uint32_t)b, (uint32_t)b, false, false);
        const auto hi = __builtin_amdgcn_permlane16_swap((uint32_t)(b >> 32), (uint32_t)(b >> 32), false, false);
        a = pair_to_double(lo[0], hi[0]) + pair_to_double(lo[1], hi[1]);
    }
    if (PG >= 8) {
        __builtin_memcpy(&b, &a, 8);
        const auto lo = __builtin_amdgcn_permlane32_swap((uint32_t)b, (uint32_t)b, false, false);
        const auto hi = __builtin_amdgcn_permlane32_swap((uint32_t)(b >> 32), (uint32_t)(b >> 32), false, false);
        a = pair_to_double(lo[0], hi[0]) + pair_to_double(lo[1], hi[1]);
    }
    return a;
}

// PG = lane groups per tile (8, 4, 2 or 1).  With 16 or more workers a tile takes all 8 lane groups
// of the wavefront; with fewer, 8 / PG adjacent tiles share the wavefront (lane group lgw serves
// tile lgw / PG as group lgw % PG), so that no lane group idles and the wavefront still moves 1 KB
// per instruction.
template <typename ST, int GRAD, int LPR, int PG, int CP, bool FULL>
struct NarrowTile {
    using S = Storage<ST>;
    using Acc = typename S::Acc;
    using LDS = typename LdsFor<GRAD>::type;
    using Raw = typename S::Raw;
    static constexpr int VEC = S::VEC;
    static constexpr int GROUPS = PG;            // lane groups of one tile = its rows per wavefront instruction
    static constexpr int TPW = (64 / LPR) / PG;  // tiles per wavefront
    static constexpr uint32_t STRIDE = LPR * VEC;   // elements between consecutive rows of a tile (tiled layout)
    // CP = row pairs per lane and load chunk (2 * CP rows in flight per chunk): 2, or 1 when the
    // workers give a lane a single pair
    static constexpr int CG = GRAD == kGradBuffer ? 2 * CP : 1;

    const RoundParams &prm;
    const LDS &lds;
    uint32_t quad_hi, quad_lo;   // noise counter of the lane's first quad; quad_hi is wave-uniform
    ST *Xt;            // the wavefront's first tile: wave-uniform base, every access adds a 32-bit lane offset
    const ST *Gt;
    uint32_t sub_off;  // this lane's tile inside the wavefront's run + its columns inside a row segment
    int64_t c0, lo, hi;   // c0: the lane's first column
    int lg;            // the lane's group inside its tile
    int n;             // rows this wavefront walks: all prm.n workers, or its half of them (round_kernel_split)
    int pair0;         // worker pair of its first row (0, or 16 for the upper half): the noise counter
    // The lane's rows are 2*lg + 2*GROUPS*k + r (pair k, r = 0, 1): bit 2*GROUPS*k + r of these words
    // (the masks shifted down by 2*lg) says whether that row's copy reached the server (sum),
    // whether its reply arrived (gets the average), whether it keeps its own v -- rows >= n: none.
    uint64_t sum_bits, avg_bits, own_bits;
    uint32_t limit;    // bytes of the wavefront's tiles: the buffer resource's bound

    // lgw = lane / LPR, col_off = (lane % LPR) * VEC, first = first column of the wavefront's first tile
    __device__ __forceinline__ NarrowTile(const RoundParams &prm_, const LDS &lds_, ST *Xt_, const ST *Gt_,
                                          uint32_t col_off, int64_t first, int64_t lo_, int64_t hi_, uint64_t ucol,
                                          uint64_t dcol, int lgw, int rows, int pair0_)
        : prm(prm_), lds(lds_), Xt(Xt_), Gt(Gt_), lo(lo_), hi(hi_), lg(lgw % PG), n(rows), pair0(pair0_) {
        const int tw = lgw / PG;   // the lane's tile among the wavefront's
        sub_off = (uint32_t)tw * (uint32_t)prm.n * STRIDE + col_off;
        c0 = first + (int64_t)tw * (LPR * VEC) + col_off;
        // `first` is a multiple of the wavefront's width, which divides 512 columns
        quad_hi = (uint32_t)(first >> 9);
        quad_lo = ((uint32_t)(first >> 2) & 127u) + (((uint32_t)tw * (LPR * VEC) + col_off) >> 2);
        const uint64_t valid = n >= 64 ? ~0ull : ((1ull << n) - 1);
        sum_bits = (ucol & valid) >> (2 * lg);
        avg_bits = (dcol & valid) >> (2 * lg);
        own_bits = (~dcol & valid) >> (2 * lg);
        limit = (uint32_t)TPW * (uint32_t)n * STRIDE * (uint32_t)sizeof(ST);
    }

    // bit of pair k, row r of that pair
    static __device__ __forceinline__ bool bit(uint64_t w, int k, int r) { return (w >> (2 * GROUPS * k + r)) & 1; }
    // rows of the lane's k-th pair
    __device__ __forceinline__ int row_a(int k) const { return 2 * (lg + GROUPS * k); }
    __device__ __forceinline__ uint32_t off(int i) const { return (uint32_t)i * STRIDE + sub_off; }

    __device__ __forceinline__ void load_chunk(int k0, Raw x[2 * CP], Raw g[CG]) const {
        const int last = n - 1;
#pragma unroll
        for (int q = 0; q < CP; ++q) {
            int ia = row_a(k0 + q), ib = ia + 1;
            if (!FULL) {   // rows past n repeat row n-1, unused (FULL: the buffer bound returns zeros)
                ia = ia < last ? ia : last;
                ib = ib < last ? ib : last;
            }
            x[2 * q] = load_seg<ST, FULL>(Xt, off(ia), limit, c0, lo, hi);
            x[2 * q + 1] = load_seg<ST, FULL>(Xt, off(ib), limit, c0, lo, hi);
            if (GRAD == kGradBuffer) {
                g[GRAD == kGradBuffer ? 2 * q : 0] = load_seg<ST, FULL>(Gt, off(ia), limit, c0, lo, hi);
                g[GRAD == kGradBuffer ? 2 * q + 1 : 0] = load_seg<ST, FULL>(Gt, off(ib), limit, c0, lo, hi);
            }
        }
    }

    __device__ __forceinline__ void row(int k, int r, Raw xr, Raw gr, const float *z, Acc acc[VEC]) const {
        const bool u = bit(sum_bits, k, r), own = GRAD != kGradNone && bit(own_bits, k, r);
        if (!(u || own)) return;
        float v[VEC], g[VEC];
        S::unpack(xr, v);
        if (GRAD == kGradBuffer) S::unpack(gr, g);
        const Raw vr = sgd_step<ST, GRAD>(prm, GRAD == kGradBuffer ? g : z, v);
        if (u) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] += (Acc)v[e];
        }
        if (own) store_seg<ST, FULL>(Xt, off(row_a(k) + r), limit, c0, lo, hi, vr);
    }

    __device__ __forceinline__ void process_chunk(int k0, const Raw x[2 * CP], const Raw g[CG], Acc acc[VEC]) const {
        if (GRAD == kGradSynthetic && sizeof(ST) == 2 && (CP >= 3 || (CP == 2 && PG < 8))) {
            // bf16 (8 values per lane and row, bound by this arithmetic rather than by the loads) on three row pairs,
            // or on two with fewer than 8 lane groups: pair by pair, so that only one pair's noise is live -- 200 -> 150
            // and 139 -> 119 registers per lane, i.e. 12 instead of 8 and 16 instead of 12 wavefronts per compute
            // unit (n = 18 0.57 -> 0.64 of the HBM peak, n = 20 0.62 -> 0.67, n = 16 0.73 -> 0.76); the first pair's
            // noise still runs under the loads' latency.  (Two pairs on all 8 lane groups, 17-32 workers, already fit
            // 128 registers and are 3 % faster with all the noise first.)
#pragma unroll
            for (int q = 0; q < CP; ++q) {
                float za[VEC], zb[VEC];
                noise_rows<VEC>(prm, lds, pair0 + (row_a(k0 + q) >> 1), quad_hi, quad_lo, za, zb);
                row(k0 + q, 0, x[2 * q], g[0], za, acc);
                row(k0 + q, 1, x[2 * q + 1], g[0], zb, acc);
            }
        } else {
            // the noise does not depend on the loaded values: all of it first, under the loads' latency
            float za[CP][VEC], zb[CP][VEC];
            if (GRAD == kGradSynthetic) {
#pragma unroll
                for (int q = 0; q < CP; ++q)
                    noise_rows<VEC>(prm, lds, pair0 + (row_a(k0 + q) >> 1), quad_hi, quad_lo, za[q], zb[q]);
            }
#pragma unroll
            for (int q = 0; q < CP; ++q) {
                row(k0 + q, 0, x[2 * q], g[GRAD == kGradBuffer ? 2 * q : 0], za[q], acc);
                row(k0 + q, 1, x[2 * q + 1], g[GRAD == kGradBuffer ? 2 * q + 1 : 0], zb[q], acc);
            }
        }
#pragma unroll
        for (int q = 0; q < 2 * CP; ++q) asm volatile("" ::"v"(x[q]));   // see process_chunk of the wide kernel
        if (GRAD == kGradBuffer) {
#pragma unroll
            for (int q = 0; q < CG; ++q) asm volatile("" ::"v"(g[q]));
        }
    }

    template <typename C>
    __device__ __forceinline__ void finish(Acc acc[VEC], double inv, int steps, const C &combine) const {
        // combine the lane groups: after the butterfly every lane of a column group holds the same sum
        if (GRAD == kGradSynthetic && LPR == 8) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] = sum_lane_groups<PG>(acc[e]);
        } else {
#pragma unroll
            for (int o = LPR; o < LPR * PG; o <<= 1) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[e] += __shfl_xor(acc[e], o, 64);
            }
        }
        combine(acc);   // round_kernel_split: plus the other half's sums
        float vt[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) vt[e] = (float)(acc[e] * (Acc)inv);
        const Raw vt_raw = S::round_vec(vt);
        __builtin_amdgcn_s_setprio(3);
        for (int q = 0; q < steps; ++q) {
            if (bit(avg_bits, q, 0)) store_seg<ST, FULL>(Xt, off(row_a(q)), limit, c0, lo, hi, vt_raw);
            if (bit(avg_bits, q, 1)) store_seg<ST, FULL>(Xt, off(row_a(q) + 1), limit, c0, lo, hi, vt_raw);
        }
    }

    // SINGLE: the launcher guarantees n <= 2 * GROUPS * CP, i.e. the lane's rows are one load chunk
    // and every row index is a compile-time constant (the general loop is then not even compiled
    // in: having both in one kernel costs registers).
    // after_first_loads() is called once the first chunk's loads are issued (see noise_fill_begin)
    template <bool SINGLE, typename F, typename C>
    __device__ __forceinline__ void run(double inv, const F &after_first_loads, const C &combine) const {
        const int steps = ((n + 1) / 2 + GROUPS - 1) / GROUPS;   // row pairs per lane (wave-uniform)
        Acc acc[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] = 0;
        Raw xa[2 * CP], xb[2 * CP], ga[CG], gb[CG];
        // a wavefront that is about to issue its loads, or to store its results, goes before the
        // ones that are busy with arithmetic: the memory queue stays fed
        __builtin_amdgcn_s_setprio(3);
        load_chunk(0, xa, ga);
        __builtin_amdgcn_s_setprio(0);
        // vector loads just issued (the element-wise path issues many small ones: it waits for all)
        after_first_loads(std::integral_constant<int, FULL ? (GRAD == kGradBuffer ? 4 : 2) * CP : 0>{});
        if constexpr (SINGLE) {
            process_chunk(0, xa, ga, acc);
            finish(acc, inv, steps, combine);
            return;
        }
        int k = 0;
        for (; k + 2 * CP < steps; k += 2 * CP) {
            load_chunk(k + CP, xb, gb);
            process_chunk(k, xa, ga, acc);
            load_chunk(k + 2 * CP, xa, ga);
            process_chunk(k + CP, xb, gb, acc);
        }
        if (k + CP < steps) {
            load_chunk(k + CP, xb, gb);
            process_chunk(k, xa, ga, acc);
            process_chunk(k + CP, xb, gb, acc);
        } else {
            process_chunk(k, xa, ga, acc);
        }
        finish(acc, inv, steps, combine);
    }
};

// Tiled layout only: the tile [tile0, tile0 + LPR * VEC) of all n workers is the contiguous run of
// n * LPR * 16 bytes at element offset tile0 * n; a wavefront takes 8 / PG adjacent tiles at a time,
// tiles_per_wave times, WPB such runs apart (the wavefronts of a workgroup stay next to each other).
//
// Register budget (second launch bound: wavefronts per SIMD the compiler has to leave room for; 0 = its
// own choice).  bf16, in-register gradient, 17-32 workers on two row pairs: 130 registers per lane by
// itself, i.e. three wavefronts per SIMD and one workgroup of 8 per compute unit; held to 128 (no
// spills) two workgroups fit: 0.69 -> 0.78 of the HBM peak at 32 workers.  The variants that need
// spills for it (two pairs on fewer lane groups: 139 registers; three pairs: 200) are slower with it.
template <typename ST, int GRAD, int PG, int CP, bool SINGLE>
constexpr int narrow_min_waves_per_simd() {
    return sizeof(ST) == 2 && GRAD == kGradSynthetic && SINGLE && PG == 8 && CP == 2 ? 4 : 0;
}

template <typename ST, int GRAD, int LPR, int PG, int CP, bool SINGLE, int WPB>
__global__ __launch_bounds__(WPB * 64, (narrow_min_waves_per_simd<ST, GRAD, PG, CP, SINGLE>())) void round_kernel_narrow(
    ST *__restrict__ X, const ST *__restrict__ G, const RoundTable *__restrict__ tab, const RoundParams prm) {
    constexpr int VEC = Storage<ST>::VEC;
    constexpr int WIDTH = ((64 / LPR) / PG) * LPR * VEC;   // columns per wavefront and step
    __shared__ typename LdsFor<GRAD>::type lds;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int j = blockIdx.y;
    // the noise cells travel to LDS while the first tile's loads are in flight: the copy is issued
    // here, the wait and the workgroup barrier follow the first tile's loads -- or the loop, for a
    // wavefront that has no tile: every wavefront passes the barrier exactly once
    noise_fill_begin<WPB>(lds, prm.noise_cells, wave, lane);
    bool fill_pending = true;
    const auto finish_fill = [&](auto pending) {
        if (fill_pending) noise_fill_end<decltype(pending)::value>(lds);
        fill_pending = false;
    };
    const int64_t lo = tab->off[j], hi = tab->off[j + 1];
    const uint64_t ucol = tab->ucol[j], dcol = tab->dcol[j];
    const double inv = tab->inv_cnt[j];
    const uint32_t col_off = (uint32_t)(lane % LPR) * VEC;
    const auto nothing = [](auto) {};
    for (int it = 0; it < prm.tiles_per_wave; ++it) {
        const int64_t first = (lo / WIDTH) * WIDTH + unit_index(it, WPB, wave) * WIDTH;
        if (first >= hi) break;   // wave-uniform
        ST *Xt = X + first * prm.n;
        const ST *Gt = G ? G + first * prm.n : nullptr;
        const bool full = prm.vec_ok && first >= lo && first + WIDTH <= hi;   // wave-uniform
        if (full) {
            const NarrowTile<ST, GRAD, LPR, PG, CP, true> t(prm, lds, Xt, Gt, col_off, first, lo, hi, ucol, dcol, lane / LPR,
                                                            prm.n, 0);
            t.template run<SINGLE>(inv, finish_fill, nothing);
        } else {
            const NarrowTile<ST, GRAD, LPR, PG, CP, false> t(prm, lds, Xt, Gt, col_off, first, lo, hi, ucol, dcol, lane / LPR,
                                                             prm.n, 0);
            t.template run<SINGLE>(inv, finish_fill, nothing);
        }
    }
    finish_fill(std::integral_constant<int, 0>{});
    prepare_next_outcome(prm, linear_block() == 0 && wave == 0, j, lane);
}

// More than 32 workers, tiled layout: a tile (n x 128 bytes, up to 8 KB) is shared by a PAIR of
// wavefronts of the workgroup -- wavefront 2q takes the lower half of the row pairs (rounded up),
// wavefront 2q+1 the rest, each as a single load chunk like a tile of up to 32 workers -- and the two
// exchange their column sums through LDS before either writes the average back.  What this buys is
// the memory behaviour of the 4 KB tile: an in-place walk is the slower the more data lies between a
// read and its write-back.
// Used for fp32 from 57 workers on (narrow_split() has the measurements); bf16 is not built.
// Barriers: every wavefront of the workgroup executes exactly one for the noise-cell copy (at its
// first step, whether or not it has a tile) and exactly one per step for the exchange (whether or
// not it has a tile), so their counts agree however the tiles run out; the two wavefronts of a pair
// always share their tile and hence take the same path.  The exchange slots alternate between two
// buffers: a wavefront rewrites a slot two steps later, after a barrier that its partner reaches
// only once it has used the values read from it.
template <typename ST, int GRAD, int LPR, int WPB>
__global__ __launch_bounds__(WPB * 64, (narrow_min_waves_per_simd<ST, GRAD, 8, 2, true>())) void round_kernel_split(
    ST *__restrict__ X, const ST *__restrict__ G, const RoundTable *__restrict__ tab, const RoundParams prm) {
    static_assert(WPB % 2 == 0 && 64 / LPR == 8, "pairs of wavefronts; a tile takes all 8 lane groups");
    constexpr int VEC = Storage<ST>::VEC;
    constexpr int WIDTH = LPR * VEC;   // columns per pair of wavefronts and step: one tile
    constexpr uint32_t STRIDE = LPR * VEC;
    using Acc = typename Storage<ST>::Acc;
    __shared__ typename LdsFor<GRAD>::type lds;
    __shared__ Acc exchange[2][WPB][LPR][VEC];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int upper = wave & 1;
    const int j = blockIdx.y;
    noise_fill_begin<WPB>(lds, prm.noise_cells, wave, lane);
    bool fill_pending = true;
    const auto finish_fill = [&](auto pending) {
        if (fill_pending) noise_fill_end<decltype(pending)::value>(lds);
        fill_pending = false;
    };
    const int64_t lo = tab->off[j], hi = tab->off[j + 1];
    const int kHalf = ((prm.n + 3) / 4) * 2;   // rows of the lower half: half the row pairs, rounded up (wave-uniform)
    const uint64_t ucol = tab->ucol[j] >> (upper * kHalf), dcol = tab->dcol[j] >> (upper * kHalf);
    const double inv = tab->inv_cnt[j];
    const int rows = upper ? prm.n - kHalf : kHalf;   // the launcher guarantees 32 < n <= 64: both halves hold 1..32 rows
    const uint32_t col_off = (uint32_t)(lane % LPR) * VEC;
    for (int it = 0; it < prm.tiles_per_wave; ++it) {
        const int64_t first = (lo / WIDTH) * WIDTH + unit_index(it, WPB / 2, wave >> 1) * WIDTH;
        Acc(*const mine)[VEC] = exchange[it & 1][wave], (*const theirs)[VEC] = exchange[it & 1][wave ^ 1];
        const auto exchange_barrier = [] { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };
        const auto add_other_half = [&](Acc acc[VEC]) {
            if (lane < LPR) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) mine[lane][e] = acc[e];
            }
            exchange_barrier();
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] += theirs[lane % LPR][e];
        };
        if (first >= hi) {   // wave-uniform, and the same for both wavefronts of a pair
            finish_fill(std::integral_constant<int, 0>{});
            exchange_barrier();
            continue;
        }
        ST *Xt = X + first * prm.n + upper * (kHalf * STRIDE);
        const ST *Gt = G ? G + first * prm.n + upper * (kHalf * STRIDE) : nullptr;
        const bool full = prm.vec_ok && first >= lo && first + WIDTH <= hi;   // wave-uniform
        if (full) {
            const NarrowTile<ST, GRAD, LPR, 8, 2, true> t(prm, lds, Xt, Gt, col_off, first, lo, hi, ucol, dcol, lane / LPR, rows,
                                                          upper * (kHalf / 2));
            t.template run<true>(inv, finish_fill, add_other_half);
        } else {
            const NarrowTile<ST, GRAD, LPR, 8, 2, false> t(prm, lds, Xt, Gt, col_off, first, lo, hi, ucol, dcol, lane / LPR, rows,
                                                           upper * (kHalf / 2));
            t.template run<true>(inv, finish_fill, add_other_half);
        }
    }
    finish_fill(std::integral_constant<int, 0>{});   // only if the loop had no step at all
    prepare_next_outcome(prm, linear_block() == 0 && wave == 0, j, lane);
}

// Local SGD step alone: grid = (runs of vector chunks, workers); a lane owns one 16-byte vector of
// one row per chunk.  One row per wavefront keeps every access stream contiguous (measured 0.80 of
// the HBM peak against 0.74 when a lane served both rows of a worker pair); the price is that the
// noise hash of a (4 columns x 2 workers) patch is evaluated by both rows' lanes, each keeping
// its half.  A wavefront step covers U adjacent chunks of 1 KB (all loads first, then the
// arithmetic and the stores); it takes tiles_per_wave steps.
template <typename ST, int GRAD, bool FULL, int U, typename LDS, typename F>
__device__ __forceinline__ void local_step_chunks(ST *__restrict__ X, const ST *__restrict__ G, const RoundParams &prm,
                                                  const LDS &lds, LaneCols lc, int i, int chunks, const F &after_loads) {
    using S = Storage<ST>;
    constexpr int VEC = S::VEC;
    constexpr int TILE = 64 * VEC;
    ST *row = X + (int64_t)i * prm.stride + lc.tile0;
    const ST *grow = GRAD == kGradBuffer ? G + (int64_t)i * prm.stride + lc.tile0 : nullptr;
    typename S::Raw xr[U], gr[GRAD == kGradBuffer ? U : 1];
    const int64_t tile0 = lc.tile0;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (u < chunks) {   // wave-uniform
            lc.tile0 = tile0 + u * TILE;
            xr[u] = load_raw<ST, FULL>(row + u * TILE, lc);
            if (GRAD == kGradBuffer) gr[GRAD == kGradBuffer ? u : 0] = load_raw<ST, FULL>(grow + u * TILE, lc);
        }
    }
    after_loads(std::integral_constant<int, FULL ? (GRAD == kGradBuffer ? 2 : 1) * U : 0>{});   // FULL: chunks == U
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (u < chunks) {
            lc.tile0 = tile0 + u * TILE;
            float x[VEC], g[VEC], other[VEC];
            S::unpack(xr[u], x);
            if (GRAD == kGradBuffer) {
                S::unpack(gr[GRAD == kGradBuffer ? u : 0], g);
            } else if (i & 1) {
                noise_rows<VEC>(prm, lds, i >> 1, lc.quad_hi(), lc.quad_lo(), other, g);
            } else {
                noise_rows<VEC>(prm, lds, i >> 1, lc.quad_hi(), lc.quad_lo(), g, other);
            }
            store_raw<ST, FULL>(row + u * TILE, lc, sgd_step<ST, GRAD>(prm, g, x));
        }
    }
}

template <typename ST, int GRAD, int WPB>
__global__ __launch_bounds__(WPB * 64) void local_step_kernel(ST *__restrict__ X, const ST *__restrict__ G,
                                                              const RoundParams prm) {
    constexpr int VEC = Storage<ST>::VEC;
    constexpr int TILE = 64 * VEC;
    constexpr int U = GRAD == kGradSynthetic ? 4 : 1;
    __shared__ typename LdsFor<GRAD>::type lds;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int row = blockIdx.y;
    noise_fill_begin<WPB>(lds, prm.noise_cells, wave, lane);
    bool fill_pending = true;
    const auto finish_fill = [&](auto pending) {
        if (fill_pending) noise_fill_end<decltype(pending)::value>(lds);
        fill_pending = false;
    };
    for (int it = 0; it < prm.tiles_per_wave; ++it) {
        const int64_t tile0 = unit_index(it, WPB, wave) * (U * TILE);
        if (tile0 >= prm.N) break;   // wave-uniform
        LaneCols lc;
        lc.tile0 = tile0;
        lc.loff = (uint32_t)lane * VEC;
        lc.lo = 0;
        lc.hi = prm.N;
        const int64_t left = (prm.N - tile0 + TILE - 1) / TILE;
        const int chunks = (int)(left < U ? left : U);
        if (prm.vec_ok && tile0 + U * TILE <= prm.N)
            local_step_chunks<ST, GRAD, true, U>(X, G, prm, lds, lc, row, U, finish_fill);
        else
            local_step_chunks<ST, GRAD, false, U>(X, G, prm, lds, lc, row, chunks, finish_fill);
    }
    finish_fill(std::integral_constant<int, 0>{});
}

// Local step on the tiled layout with a gradient buffer: the storage is one run of (tile, worker)
// segments of kTiledLanes x 16 bytes, and x - gamma * g needs no coordinates, so a wavefront takes
// 1 KB of it in storage order (8 segments) and the pass is a plain sequential stream over X and G.
// Lane -> segment s = 8 * k + lane / 8 of KB k -> tile s / n; only the padding columns of the last
// tile need care.  (With the in-register gradient the local step runs through round_kernel_narrow
// under the outcome "no message arrives".)
template <typename ST, int WPB>
__global__ __launch_bounds__(WPB * 64) void local_step_tiled_kernel(ST *__restrict__ X, const ST *__restrict__ G,
                                                                    const RoundParams prm) {
    using S = Storage<ST>;
    using Raw = typename S::Raw;
    constexpr int VEC = S::VEC;
    constexpr int LPR = kTiledLanes, TILE = LPR * VEC, SEGS = 64 / LPR;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t tiles = (prm.N + TILE - 1) / TILE;
    const int64_t kb = unit_index(0, WPB, wave);
    const int64_t seg0 = kb * SEGS;                   // first segment of this KB: scalar division
    int64_t tile = seg0 / prm.n;
    int i = (int)(seg0 % prm.n) + lane / LPR;         // the lane's segment lies at most 64 / LPR rows further
    while (i >= prm.n) {
        i -= prm.n;
        ++tile;
    }
    const int64_t seg = seg0 + lane / LPR;
    if (tile >= tiles) return;                        // past the last tile
    const int64_t c0 = tile * TILE + (lane % LPR) * VEC;
    if (c0 >= prm.N) return;                          // padding columns of the last tile
    ST *px = X + seg * TILE + (lane % LPR) * VEC;     // plain global accesses: measured faster here than the
    const ST *pg = G + (px - X);                      // buffer form the round kernels use
    float x[VEC], g[VEC];
    if (prm.vec_ok && c0 + VEC <= prm.N) {
        const Raw xr = __builtin_nontemporal_load(reinterpret_cast<const Raw *>(px));
        const Raw gr = __builtin_nontemporal_load(reinterpret_cast<const Raw *>(pg));
        S::unpack(xr, x);
        S::unpack(gr, g);
        __builtin_nontemporal_store(sgd_step<ST, kGradBuffer>(prm, g, x), reinterpret_cast<Raw *>(px));
    } else {
        S::unpack(load_seg<ST, false>(px, 0, 0, c0, 0, prm.N), x);
        S::unpack(load_seg<ST, false>(pg, 0, 0, c0, 0, prm.N), g);
        store_seg<ST, false>(px, 0, 0, c0, 0, prm.N, sgd_step<ST, kGradBuffer>(prm, g, x));
    }
}

// Launch shapes.  The memory system of this GPU is at its best when the chip-wide footprint of
// requests in flight is a few MB: occupancy is therefore capped through the LDS a workgroup holds --
// the noise cells where a kernel generates noise, plus a dynamic allocation that is never touched.
// Returns the dynamic LDS bytes that leave room for max_waves_per_cu / wpb workgroups per compute
// unit (0 or >= 32 waves: no cap), given the kernel's static LDS.
size_t occupancy_pad(int max_waves_per_cu, int wpb, size_t static_lds) {
    if (max_waves_per_cu <= 0 || max_waves_per_cu >= 32) return 0;
    int wgs = max_waves_per_cu / wpb;
    if (wgs < 1) wgs = 1;
    size_t per = ((size_t)kLdsBytesPerCu / wgs) & ~(size_t)255;
    if (per > 65536) per = 65536;   // the default per-workgroup limit
    return per > static_lds ? per - static_lds : 0;
}

template <int GRAD>
constexpr size_t static_lds_bytes() {
    return sizeof(typename LdsFor<GRAD>::type);
}

// Steps a wavefront takes in a kernel that generates noise (each workgroup first copies the 32 KB
// of noise cells into LDS, which has to be spread over enough work -- but every further step of a
// wavefront costs more than a fresh wavefront would, so few): up to `most`, fewer while the grid
// would otherwise not fill the chip.  Other kernels: 1.
int steps_per_wave(int grad_mode, int64_t wave_steps_per_row, int wpb, int64_t rows, int wanted, int most) {
    if (grad_mode != kGradSynthetic) return 1;
    if (wanted > 0) return wanted;
    int t = most;
    while (t > 1 && ((wave_steps_per_row + (int64_t)wpb * t - 1) / ((int64_t)wpb * t)) * rows < 4096) t >>= 1;
    return t;
}

// Launches the round kernel `kernel` -- or, when the tuning carries an occupancy query, launches
// nothing and reports how many wavefronts of this kernel, workgroup size and dynamic LDS size the
// runtime's occupancy calculator lets one compute unit hold (what the occupancy cap above is meant
// to control).
template <typename K, typename ST>
hipError_t launch_or_query(K kernel, dim3 grid, int wpb, size_t lds, hipStream_t stream, const LaunchTuning &tune, ST *X,
                           const ST *G, const RoundTable *tab, const RoundParams &prm) {
    if (tune.occupancy_query != nullptr) {
        int wgs = 0;
        const hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&wgs, kernel, wpb * 64, lds);
        *tune.occupancy_query = wgs * wpb;
        return e;
    }
    hipLaunchKernelGGL(kernel, grid, dim3(wpb * 64), lds, stream, X, G, tab, prm);
    return hipGetLastError();
}

template <typename ST, int GRAD, int R, int WPB>
hipError_t launch_round_v(ST *X, const ST *G, const RoundTable *tab, RoundParams prm, int64_t max_block_cols,
                          const LaunchTuning &tune, hipStream_t stream) {
    constexpr int TILE = 64 * Storage<ST>::VEC;
    // tiles sit on absolute multiples of TILE columns: a block may overhang one tile on each side
    const int64_t tiles = (max_block_cols + 2 * TILE - 2) / TILE;
    prm.tiles_per_wave = steps_per_wave(GRAD, tiles, WPB, prm.blocks, tune.tiles_per_wave, 1);
    const int64_t per_wg = (int64_t)WPB * prm.tiles_per_wave;
    const dim3 grid = folded_grid8((tiles + per_wg - 1) / per_wg, (unsigned)prm.blocks);
    const size_t lds = occupancy_pad(tune.max_waves_per_cu, WPB, static_lds_bytes<GRAD>());
    return launch_or_query(round_kernel<ST, GRAD, R, WPB>, grid, WPB, lds, stream, tune, X, G, tab, prm);
}

template <typename ST, int GRAD, int LPR, int WPB>
hipError_t launch_round_narrow(ST *X, const ST *G, const RoundTable *tab, RoundParams prm, int64_t max_block_cols,
                               const LaunchTuning &tune, hipStream_t stream) {
    constexpr int TILE = LPR * Storage<ST>::VEC;
    constexpr int GROUPS = 64 / LPR;
    const NarrowShape shape = narrow_shape(prm.n, (int)sizeof(ST));
    const int pg = shape.lane_groups;
    const int64_t width = (int64_t)(GROUPS / pg) * TILE;   // columns per wavefront and step
    const int64_t steps = (max_block_cols + 2 * width - 2) / width;
    // fp32: one step (about 4 KB) per wavefront is best at every worker count (n = 8 / 16 / 32: +2-3 %
    // over two); bf16: two
    prm.tiles_per_wave = steps_per_wave(GRAD, steps, WPB, prm.blocks, tune.tiles_per_wave, sizeof(ST) == 4 ? 1 : 2);
    const int64_t per_wg = (int64_t)WPB * prm.tiles_per_wave;
    const dim3 grid = folded_grid8((steps + per_wg - 1) / per_wg, (unsigned)prm.blocks);
    const size_t lds = occupancy_pad(tune.max_waves_per_cu, WPB, static_lds_bytes<GRAD>());
#define RPS_N(PG, CP, SINGLE) \
    return launch_or_query(round_kernel_narrow<ST, GRAD, LPR, PG, CP, SINGLE, WPB>, grid, WPB, lds, stream, tune, X, G, tab, prm)
    switch (shape.row_pairs * 8 + pg) {
        case 1 * 8 + 1: RPS_N(1, 1, true);
        case 1 * 8 + 2: RPS_N(2, 1, true);
        case 1 * 8 + 4: RPS_N(4, 1, true);
        case 1 * 8 + 8: RPS_N(8, 1, true);
        case 2 * 8 + 1: RPS_N(1, 2, true);
        case 2 * 8 + 2: RPS_N(2, 2, true);
        case 2 * 8 + 4: RPS_N(4, 2, true);
        case 2 * 8 + 8: RPS_N(8, 2, true);
        case 3 * 8 + 2: RPS_N(2, 3, true);
        case 3 * 8 + 4: RPS_N(4, 3, true);
        case 3 * 8 + 1:
            if constexpr (sizeof(ST) == 2) RPS_N(1, 3, true);
            return hipErrorInvalidValue;
        default: break;
    }
    if (shape.row_pairs != 0) return hipErrorInvalidValue;
    // more than 32 workers: chunks of one or two row pairs
    if (tune.rows_in_flight <= 2) RPS_N(8, 1, false);
    RPS_N(8, 2, false);
#undef RPS_N
}

template <typename ST, int GRAD, int LPR, int WPB>
hipError_t launch_round_split(ST *X, const ST *G, const RoundTable *tab, RoundParams prm, int64_t max_block_cols,
                              const LaunchTuning &tune, hipStream_t stream) {
    constexpr int TILE = LPR * Storage<ST>::VEC;
    if (prm.n <= 32 || prm.n > 64) return hipErrorInvalidValue;   // each half must hold 1..32 rows
    const int64_t steps = (max_block_cols + 2 * TILE - 2) / TILE;
    prm.tiles_per_wave = steps_per_wave(GRAD, steps, WPB / 2, prm.blocks, tune.tiles_per_wave, sizeof(ST) == 4 ? 1 : 2);
    const int64_t per_wg = (int64_t)(WPB / 2) * prm.tiles_per_wave;
    const dim3 grid = folded_grid8((steps + per_wg - 1) / per_wg, (unsigned)prm.blocks);
    const size_t fixed = static_lds_bytes<GRAD>() + sizeof(typename Storage<ST>::Acc) * 2 * WPB * LPR * Storage<ST>::VEC;
    const size_t lds = occupancy_pad(tune.max_waves_per_cu, WPB, fixed);
    return launch_or_query(round_kernel_split<ST, GRAD, LPR, WPB>, grid, WPB, lds, stream, tune, X, G, tab, prm);
}

// Workgroup widths.  Tile-major: kernels that generate noise share the LDS copy of the noise cells
// among 4, 8, 12 or 14 wavefronts: with 81-88 registers per lane one workgroup of 12 or 14 is all a
// compute unit holds, which is both the occupancy this memory system likes best for the in-place
// walk and the fewest copies of the cells (n = 32 fp32: 0.823 of the HBM peak with 2 x 8, 0.834
// with 12, 0.838 with 14, 0.827 with 16).  The round on a gradient buffer shares nothing, and is
// still 3-4 % faster in workgroups of 12 or 14 than in single wavefronts (a workgroup's wavefronts
// start together on adjacent tiles of their XCD); the averaging alone is fastest in single
// wavefronts under its occupancy cap.  Row-major, where a tile is n KB: 2, 4 or 8 wavefronts share
// the cells; the others keep one wavefront per workgroup, or 4 (bf16 on a gradient buffer from 32 workers on).
template <typename ST, int GRAD>
hipError_t launch_round_t(ST *X, const ST *G, const RoundTable *tab, const RoundParams &prm, int64_t max_block_cols,
                          const LaunchTuning &tune, hipStream_t stream) {
    const int r = tune.rows_in_flight, w = tune.waves_per_workgroup;
    if (prm.tiled) {
        if constexpr (sizeof(ST) == 4) {
            if (narrow_split(prm.n, 4)) return launch_round_split<ST, GRAD, kTiledLanes, 8>(X, G, tab, prm, max_block_cols, tune, stream);
        }
#define RPS_T(W) launch_round_narrow<ST, GRAD, kTiledLanes, W>(X, G, tab, prm, max_block_cols, tune, stream)
        // (if constexpr: only the widths a gradient source is launched with are compiled)
        if constexpr (GRAD == kGradNone)
            return RPS_T(1);
        else if constexpr (GRAD == kGradBuffer)
            return w <= 1 ? RPS_T(1) : (w <= 8 ? RPS_T(8) : (w <= 12 ? RPS_T(12) : RPS_T(14)));
        else
            return w <= 4 ? RPS_T(4) : (w <= 8 ? RPS_T(8) : (w <= 12 ? RPS_T(12) : RPS_T(14)));
#undef RPS_T
    }
#define RPS_V(R, W) launch_round_v<ST, GRAD, R, W>(X, G, tab, prm, max_block_cols, tune, stream)
    if constexpr (GRAD == kGradSynthetic) {
        if (w <= 2) return r <= 2 ? RPS_V(2, 2) : RPS_V(4, 2);
        if (w <= 4) return r <= 2 ? RPS_V(2, 4) : RPS_V(4, 4);
        return r <= 2 ? RPS_V(2, 8) : RPS_V(4, 8);
    } else {
        if (w == 1) return r <= 2 ? RPS_V(2, 1) : RPS_V(4, 1);
        return r <= 2 ? RPS_V(2, 4) : RPS_V(4, 4);
    }
#undef RPS_V
}

template <typename ST>
hipError_t launch_round_g(int grad_mode, ST *X, const ST *G, const RoundTable *tab, const RoundParams &prm,
                          int64_t max_block_cols, const LaunchTuning &tune, hipStream_t stream) {
    switch (grad_mode) {
        case kGradNone: return launch_round_t<ST, kGradNone>(X, G, tab, prm, max_block_cols, tune, stream);
        case kGradBuffer: return launch_round_t<ST, kGradBuffer>(X, G, tab, prm, max_block_cols, tune, stream);
        default: return launch_round_t<ST, kGradSynthetic>(X, G, tab, prm, max_block_cols, tune, stream);
    }
}

template <typename ST>
hipError_t launch_local_step_g(int grad_mode, ST *X, const ST *G, RoundParams prm, int wanted_steps, hipStream_t stream) {
    constexpr int VEC = Storage<ST>::VEC;
    constexpr int WS = 8;   // wavefronts per workgroup where noise is generated (they share the LDS cells)
    if (prm.tiled) {
        if (grad_mode != kGradBuffer) return hipErrorInvalidValue;   // the in-register gradient goes through launch_round
        const int64_t tiles = (prm.N + kTiledLanes * VEC - 1) / (kTiledLanes * VEC);
        const int64_t kb = (tiles * prm.n * kTiledLanes + 63) / 64;   // wavefronts: 1 KB of storage each
        prm.tiles_per_wave = 1;
        hipLaunchKernelGGL((local_step_tiled_kernel<ST, 4>), folded_grid8((kb + 3) / 4, 1), dim3(256), 0, stream, X, G, prm);
        return hipGetLastError();
    }
    const int64_t tiles = (prm.N + 64 * VEC - 1) / (64 * VEC);
    if (grad_mode == kGradBuffer) {
        prm.tiles_per_wave = 1;
        hipLaunchKernelGGL((local_step_kernel<ST, kGradBuffer, 4>), folded_grid8((tiles + 3) / 4, (unsigned)prm.n), dim3(256),
                           0, stream, X, G, prm);
    } else {
        const int64_t units = (tiles + 3) / 4;   // a wavefront step is 4 chunks here
        prm.tiles_per_wave = steps_per_wave(kGradSynthetic, units, WS, prm.n, wanted_steps, 1);
        const int64_t per_wg = (int64_t)WS * prm.tiles_per_wave;
        hipLaunchKernelGGL((local_step_kernel<ST, kGradSynthetic, WS>),
                           folded_grid8((units + per_wg - 1) / per_wg, (unsigned)prm.n), dim3(WS * 64), 0, stream, X, G, prm);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Gradient averaging under loss (the baseline of Sec. 6 that the paper shows converging worse
// than model averaging): the same Reduce-Scatter / All-Gather with drops is applied to the
// GRADIENTS, and each worker then takes its local step with what it ended up holding:
//   gt[c]    = (1/|N_j|) sum_{i : U[i,j]} g[i,c]         (rounded to storage: it travels)
//   x'[i,c]  = x[i,c] - gamma * (D[i,j] ? gt[c] : g[i,c])
// Pass 1 walks the rows of G (column sums), pass 2 walks the rows of X (a worker whose reply
// was lost re-reads its own gradient row).  12 B fp32 per worker-param: G once, X read + write.
// ---------------------------------------------------------------------------------------
template <typename ST, bool FULL>
__device__ __forceinline__ void gradavg_tile(ST *__restrict__ X, const ST *__restrict__ G, const RoundParams &prm,
                                             const LaneCols &lc, uint64_t ucol, uint64_t dcol, double inv) {
    using S = Storage<ST>;
    using Acc = typename S::Acc;
    using Raw = typename S::Raw;
    constexpr int VEC = S::VEC;
    constexpr int R = 4;
    const int n = prm.n;

    Acc acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0;
    const ST *grow = G + lc.tile0;
    for (int i0 = 0; i0 < n; i0 += R) {
        Raw g[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {   // rows past n repeat row n-1, unused
            g[r] = load_raw<ST, FULL>(grow, lc);
            if (i0 + r + 1 < n) grow += prm.stride;
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int i = i0 + r;
            if (i < n && ((ucol >> i) & 1)) {
                float v[VEC];
                S::unpack(g[r], v);
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[e] += (Acc)v[e];
            }
        }
    }
    float gt[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) gt[e] = (float)(acc[e] * (Acc)inv);
    (void)S::round_vec(gt);

    ST *xrow = X + lc.tile0;
    for (int i0 = 0; i0 < n; i0 += R) {
        Raw x[R];
        const ST *ld = xrow;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            x[r] = load_raw<ST, FULL>(ld, lc);
            if (i0 + r + 1 < n) ld += prm.stride;
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int i = i0 + r;
            if (i < n) {
                float v[VEC], own[VEC];
                S::unpack(x[r], v);
                const float *gsrc = gt;
                if (!((dcol >> i) & 1)) {   // reply lost: the worker applies its own gradient
                    S::unpack(load_raw<ST, FULL>(G + lc.tile0 + (int64_t)i * prm.stride, lc), own);
                    gsrc = own;
                }
#pragma unroll
                for (int e = 0; e < VEC; ++e) v[e] = __builtin_fmaf(-prm.gamma, gsrc[e], v[e]);
                store_raw<ST, FULL>(xrow, lc, S::round_vec(v));
                xrow += prm.stride;
            }
        }
    }
}

template <typename ST>
__global__ __launch_bounds__(256) void gradavg_kernel(ST *__restrict__ X, const ST *__restrict__ G,
                                                      const RoundTable *__restrict__ tab, const RoundParams prm) {
    constexpr int VEC = Storage<ST>::VEC;
    constexpr int TILE = 64 * VEC;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int j = blockIdx.y;
    prepare_next_outcome(prm, linear_block() == 0 && wave == 0, j, lane);
    const int64_t lo = tab->off[j], hi = tab->off[j + 1];
    const int64_t tile0 = (lo / TILE) * TILE + (linear_block() * 4 + wave) * TILE;
    if (tile0 >= hi) return;   // wave-uniform
    LaneCols lc;
    lc.tile0 = tile0;
    lc.loff = (uint32_t)lane * VEC;
    lc.lo = lo;
    lc.hi = hi;
    if (prm.vec_ok && tile0 >= lo && tile0 + TILE <= hi)
        gradavg_tile<ST, true>(X, G, prm, lc, tab->ucol[j], tab->dcol[j], tab->inv_cnt[j]);
    else
        gradavg_tile<ST, false>(X, G, prm, lc, tab->ucol[j], tab->dcol[j], tab->inv_cnt[j]);
}

// Gradient averaging on the tiled layout, lane groups as in round_kernel_narrow: PG lane groups per
// 128-byte-wide tile (8 with more than 16 workers; with fewer, 8 / PG adjacent tiles share the
// wavefront so that no lane group idles).  A lane has at most 8 rows (n <= 64), at most 4 below
// PG = 8: its gradient segments stay in registers between the column sums and the update, so G is
// read once.
template <typename ST, int PG, bool FULL>
__device__ __forceinline__ void gradavg_tile_narrow(ST *__restrict__ Xt, const ST *__restrict__ Gt, const RoundParams &prm,
                                                    uint32_t col_off, int64_t first, int64_t lo, int64_t hi, uint64_t ucol,
                                                    uint64_t dcol, double inv, int lgw) {
    using S = Storage<ST>;
    using Acc = typename S::Acc;
    using Raw = typename S::Raw;
    constexpr int VEC = S::VEC;
    constexpr int LPR = kTiledLanes, TPW = (64 / LPR) / PG;
    constexpr uint32_t STRIDE = LPR * VEC;
    constexpr int ROWS = PG == 8 ? 2 * ((kMaxWorkers / 2 + PG - 1) / PG) : 4;   // rows per lane at most
    const int n = prm.n;
    const int tw = lgw / PG, lg = lgw % PG;   // the lane's tile among the wavefront's, its group inside that tile
    const uint32_t sub_off = (uint32_t)tw * (uint32_t)n * STRIDE + col_off;
    const int64_t c0 = first + (int64_t)tw * (LPR * VEC) + col_off;
    const uint32_t limit = (uint32_t)TPW * (uint32_t)n * STRIDE * (uint32_t)sizeof(ST);
    Raw g[ROWS], x[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {   // lane's row r: pair lg + PG * (r / 2); rows past n repeat row n-1, unused
        const int i = 2 * (lg + PG * (r >> 1)) + (r & 1);
        const uint32_t o = (uint32_t)(i < n ? i : n - 1) * STRIDE + sub_off;
        g[r] = load_seg<ST, FULL>(Gt, o, limit, c0, lo, hi);
        x[r] = load_seg<ST, FULL>(Xt, o, limit, c0, lo, hi);
    }
    Acc acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0;
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        const int i = 2 * (lg + PG * (r >> 1)) + (r & 1);
        if (i < n && ((ucol >> i) & 1)) {
            float v[VEC];
            S::unpack(g[r], v);
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] += (Acc)v[e];
        }
    }
#pragma unroll
    for (int o = LPR; o < LPR * PG; o <<= 1) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] += __shfl_xor(acc[e], o, 64);
    }
    float gt[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) gt[e] = (float)(acc[e] * (Acc)inv);
    (void)S::round_vec(gt);   // the average travels in the storage format
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        const int i = 2 * (lg + PG * (r >> 1)) + (r & 1);
        if (i < n) {
            float v[VEC], own[VEC];
            S::unpack(x[r], v);
            S::unpack(g[r], own);
            const bool d = (dcol >> i) & 1;   // reply lost: the worker applies its own gradient
#pragma unroll
            for (int e = 0; e < VEC; ++e) v[e] = __builtin_fmaf(-prm.gamma, d ? gt[e] : own[e], v[e]);
            store_seg<ST, FULL>(Xt, (uint32_t)i * STRIDE + sub_off, limit, c0, lo, hi, S::round_vec(v));
        }
    }
}

// WPB wavefronts per workgroup, on adjacent units of their XCD (see unit_index): as for the round on a
// gradient buffer, a workgroup of 14 is a few per cent faster than single wavefronts at 32 workers.
template <typename ST, int PG, int WPB>
__global__ __launch_bounds__(WPB * 64) void gradavg_kernel_narrow(ST *__restrict__ X, const ST *__restrict__ G,
                                                                  const RoundTable *__restrict__ tab,
                                                                  const RoundParams prm) {
    constexpr int VEC = Storage<ST>::VEC;
    constexpr int WIDTH = ((64 / kTiledLanes) / PG) * kTiledLanes * VEC;   // columns per wavefront
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int j = blockIdx.y;
    prepare_next_outcome(prm, linear_block() == 0 && wave == 0, j, lane);
    const int64_t lo = tab->off[j], hi = tab->off[j + 1];
    const int64_t first = (lo / WIDTH) * WIDTH + unit_index(0, WPB, wave) * WIDTH;
    if (first >= hi) return;   // wave-uniform
    const uint32_t col_off = (uint32_t)(lane % kTiledLanes) * VEC;
    ST *Xt = X + first * prm.n;
    const ST *Gt = G + first * prm.n;
    if (prm.vec_ok && first >= lo && first + WIDTH <= hi)
        gradavg_tile_narrow<ST, PG, true>(Xt, Gt, prm, col_off, first, lo, hi, tab->ucol[j], tab->dcol[j], tab->inv_cnt[j],
                                          lane / kTiledLanes);
    else
        gradavg_tile_narrow<ST, PG, false>(Xt, Gt, prm, col_off, first, lo, hi, tab->ucol[j], tab->dcol[j], tab->inv_cnt[j],
                                           lane / kTiledLanes);
}

// ---------------------------------------------------------------------------------------
// Consensus statistics (supplement, Lemma 1: the quantity sum_i ||x_i - xbar||^2 =
// ||X (I - A_n)||_F^2 that the proof bounds) and ||xbar||^2.  One streaming read of X: a
// wavefront walks the n rows of a tile with row 0 as pivot (y_i = x_i - x_0 in fp64, so that
// sum y^2 - (sum y)^2 / n does not cancel when the workers nearly agree), tiles are taken
// grid-stride, and the reduction order is fixed: lanes (butterfly), the four wavefronts of a
// workgroup, then one workgroup over the per-workgroup partials.
// ---------------------------------------------------------------------------------------
template <typename ST, bool FULL>
__device__ __forceinline__ void consensus_tile(const ST *__restrict__ X, const RoundParams &prm, const LaneCols &lc,
                                               double &dist, double &msq) {
    using S = Storage<ST>;
    constexpr int VEC = S::VEC;
    constexpr int R = 8;
    const int n = prm.n;
    const ST *row = X + lc.tile0;
    float p[VEC];
    S::unpack(load_raw<ST, FULL>(row, lc), p);
    double s1[VEC], s2[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) s1[e] = s2[e] = 0.0;
    row += prm.stride;
    for (int i = 1; i < n; i += R, row += (int64_t)R * prm.stride) {   // chunks of up to R rows: loads first
        typename S::Raw x[R];
#pragma unroll
        for (int r = 0; r < R; ++r)
            if (i + r < n) x[r] = load_raw<ST, FULL>(row + (int64_t)r * prm.stride, lc);   // wave-uniform
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (i + r < n) {
                float v[VEC];
                S::unpack(x[r], v);
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const double y = (double)v[e] - (double)p[e];
                    s1[e] += y;
                    s2[e] = __builtin_fma(y, y, s2[e]);
                }
            }
        }
    }
    const double inv_n = 1.0 / (double)n;
#pragma unroll
    for (int e = 0; e < VEC; ++e) {   // columns outside [lo, hi) were loaded as 0 and add 0
        const double m = s1[e] * inv_n;
        dist += s2[e] - s1[e] * m;
        const double mean = (double)p[e] + m;
        msq = __builtin_fma(mean, mean, msq);
    }
}

// The same statistics on the tiled layout with 1 or 2 workers.  A wavefront step is U units; in a unit a
// tile takes PG of the 8 lane groups (8 / PG adjacent tiles share it); lane group lg of a tile holds rows
// lg, lg + PG, ... (ROWS of them) of its 16-byte column group, all U * ROWS loads are issued up front
// (4 KB in flight per wavefront).  The pivot row 0 is what the tile's first lane group loaded: the others
// get it by a lane shuffle.  Per column, sum_i y_i^2 needs no exchange (every lane adds its own rows'
// share to its running total), sum_i y_i is combined over the tile's lane groups on the cross-lane VALU
// paths and the lanes of its first group carry the column's -(sum y)^2 / n and mean^2.  (With more
// workers this arrangement -- rows dealt over lane groups -- paid a shuffle, a cross-group sum and the
// closing arithmetic per tile of 1-4 KB: 0.44-0.58 of the HBM peak at 6-8 fp32 workers, 0.21-0.51 for
// bf16 up to 32; consensus_tiles_by_column below replaced it there.)
template <typename ST, bool FULL, int PG, int ROWS, int U>
__device__ __forceinline__ void consensus_tiles_tiled(const ST *__restrict__ X, const RoundParams &prm, int64_t tile_index,
                                                      int lane, double &dist, double &msq) {
    using S = Storage<ST>;
    using Raw = typename S::Raw;
    constexpr int VEC = S::VEC;
    constexpr int LPR = kTiledLanes, TILE = LPR * VEC;
    constexpr int TPU = (64 / LPR) / PG;   // tiles that share the wavefront in one of its U units
    const int n = prm.n;
    const int lgw = lane / LPR, sub = lane % LPR;
    const int lg = lgw % PG, tw = lgw / PG;   // the lane's group inside its tile, its tile inside the unit
    const ST *Xt = X + tile_index * TILE * n;   // wave-uniform: first tile of the step
    const uint32_t tile_elems = (uint32_t)n * TILE;
    const int64_t ntiles = (prm.N + TILE - 1) / TILE;
    int tiles = (int)(ntiles - tile_index < U * TPU ? ntiles - tile_index : U * TPU);   // wave-uniform
    const uint32_t limit = (uint32_t)tiles * tile_elems * (uint32_t)sizeof(ST);
    Raw x[U][ROWS];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int t = u * TPU + tw;   // the lane's tile among the step's
        const int64_t c0 = (tile_index + t) * TILE + sub * VEC;
#pragma unroll
        for (int k = 0; k < ROWS; ++k) {
            const int i = lg + PG * k;
            // rows past n and tiles past the last one: an offset at the buffer's bound (FULL: the
            // hardware returns zeros without touching memory) / an empty column range (element-wise)
            const bool live = i < n && t < tiles;
            const uint32_t off = live ? (uint32_t)t * tile_elems + (uint32_t)i * TILE + sub * VEC : limit / (uint32_t)sizeof(ST);
            x[u][k] = load_seg<ST, FULL>(Xt, FULL || live ? off : 0u, limit, c0, 0, live ? prm.N : 0);
        }
    }
    const double inv_n = 1.0 / (double)n;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (u * TPU < tiles) {   // wave-uniform; a lane whose own tile lies past the last one holds zeros and adds 0
            float p[VEC], v[VEC];
            u32x4 bits;
            __builtin_memcpy(&bits, &x[u][0], sizeof(bits));
            const int pivot = tw * PG * LPR + sub;   // the lane of the tile's first group: row 0
            bits.x = __shfl(bits.x, pivot, 64); bits.y = __shfl(bits.y, pivot, 64);
            bits.z = __shfl(bits.z, pivot, 64); bits.w = __shfl(bits.w, pivot, 64);
            Raw praw;
            __builtin_memcpy(&praw, &bits, sizeof(praw));
            S::unpack(praw, p);                 // row 0 of this lane's column group
            double s1[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) s1[e] = 0.0;
#pragma unroll
            for (int k = 0; k < ROWS; ++k) {
                if (lg + PG * k < n) {
                    S::unpack(x[u][k], v);
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {   // columns outside [0, N) were loaded as 0, their pivot too
                        const double y = (double)v[e] - (double)p[e];
                        s1[e] += y;
                        dist = __builtin_fma(y, y, dist);
                    }
                }
            }
            // over the tile's lane groups on the cross-lane VALU paths (no LDS permutes: a tile of few workers is
            // 1 KB or less, and this is its fixed cost)
#pragma unroll
            for (int e = 0; e < VEC; ++e) s1[e] = sum_lane_groups<PG>(s1[e]);
            if (lg == 0) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const double m = s1[e] * inv_n;
                    dist = __builtin_fma(-s1[e], m, dist);
                    const double mean = (double)p[e] + m;
                    msq = __builtin_fma(mean, mean, msq);
                }
            }
        }
    }
}

// The tiled layout walked by columns: a wavefront step is 8 adjacent tiles, lane group lane / 8 takes
// one of them and its 8 lanes the tile's eight 16-byte column groups, and every lane walks ALL n rows of
// its own columns (R loads in flight, 128 bytes apart) -- so a column's sums stay in one lane: no pivot
// shuffle, no sum across lane groups, and the per-column closing arithmetic is paid once per n rows.  A
// wavefront load instruction fetches eight whole 128-byte segments n * 128 bytes apart; over the n rows
// the wavefront covers one contiguous run of 8 * n * 128 bytes.
template <typename ST, bool FULL>
__device__ __forceinline__ void consensus_tiles_by_column(const ST *__restrict__ X, const RoundParams &prm, int64_t tile_index,
                                                          int lane, double &dist, double &msq) {
    using S = Storage<ST>;
    using Raw = typename S::Raw;
    constexpr int VEC = S::VEC;
    constexpr int LPR = kTiledLanes, TILE = LPR * VEC, STEP = 64 / LPR, R = 8;
    const int n = prm.n;
    const int tw = lane / LPR, sub = lane % LPR;
    const ST *Xt = X + tile_index * TILE * n;   // wave-uniform: first tile of the step
    const uint32_t tile_elems = (uint32_t)n * TILE;
    const int64_t ntiles = (prm.N + TILE - 1) / TILE;
    const int tiles = (int)(ntiles - tile_index < STEP ? ntiles - tile_index : STEP);   // wave-uniform
    const uint32_t limit = (uint32_t)tiles * tile_elems * (uint32_t)sizeof(ST);
    const bool live = tw < tiles;   // a lane whose tile lies past the last one loads zeros and adds 0
    const int64_t c0 = (tile_index + tw) * TILE + sub * VEC;
    const uint32_t base = (uint32_t)tw * tile_elems + sub * VEC;
    const auto load = [&](int i) {
        // tiles past the last one: an offset at the buffer's bound (FULL: the hardware returns zeros
        // without touching memory) / an empty column range (element-wise)
        const uint32_t off = live ? base + (uint32_t)i * TILE : limit / (uint32_t)sizeof(ST);
        return load_seg<ST, FULL>(Xt, FULL || live ? off : 0u, limit, c0, 0, live ? prm.N : 0);
    };
    float p[VEC], v[VEC];
    S::unpack(load(0), p);   // row 0 is the pivot of the lane's columns
    double s1[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) s1[e] = 0.0;
    for (int i = 1; i < n; i += R) {   // chunks of up to R rows, all of a chunk's loads issued before the arithmetic
        Raw x[R];
#pragma unroll
        for (int r = 0; r < R; ++r)
            if (i + r < n) x[r] = load(i + r);   // wave-uniform
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (i + r < n) {
                S::unpack(x[r], v);
#pragma unroll
                for (int e = 0; e < VEC; ++e) {   // columns outside [0, N) were loaded as 0, their pivot too
                    const double y = (double)v[e] - (double)p[e];
                    s1[e] += y;
                    dist = __builtin_fma(y, y, dist);
                }
            }
        }
    }
    const double inv_n = 1.0 / (double)n;
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        const double m = s1[e] * inv_n;
        dist = __builtin_fma(-s1[e], m, dist);
        const double mean = (double)p[e] + m;
        msq = __builtin_fma(mean, mean, msq);
    }
}

template <typename ST>
__device__ __forceinline__ void consensus_walk_by_column(const ST *__restrict__ X, const RoundParams &prm, int wave, int lane,
                                                         double &dist, double &msq) {
    constexpr int TILE = kTiledLanes * Storage<ST>::VEC;
    constexpr int STEP = 64 / kTiledLanes;
    const int64_t ntiles = (prm.N + TILE - 1) / TILE;
    for (int it = 0;; ++it) {
        const int64_t t = unit_index(it, 4, wave) * STEP;
        if (t >= ntiles) break;   // wave-uniform; later steps lie further on
        if (prm.vec_ok && (t + STEP) * TILE <= prm.N)
            consensus_tiles_by_column<ST, true>(X, prm, t, lane, dist, msq);
        else
            consensus_tiles_by_column<ST, false>(X, prm, t, lane, dist, msq);
    }
}

template <typename ST, int PG, int ROWS, int U>
__device__ __forceinline__ void consensus_walk_tiled(const ST *__restrict__ X, const RoundParams &prm, int wave, int lane,
                                                     double &dist, double &msq) {
    constexpr int TILE = kTiledLanes * Storage<ST>::VEC;
    constexpr int STEP = U * ((64 / kTiledLanes) / PG);   // tiles per wavefront step
    const int64_t ntiles = (prm.N + TILE - 1) / TILE;
    for (int it = 0;; ++it) {
        const int64_t t = unit_index(it, 4, wave) * STEP;
        if (t >= ntiles) break;   // wave-uniform; later steps lie further on
        if (prm.vec_ok && (t + STEP) * TILE <= prm.N)
            consensus_tiles_tiled<ST, true, PG, ROWS, U>(X, prm, t, lane, dist, msq);
        else
            consensus_tiles_tiled<ST, false, PG, ROWS, U>(X, prm, t, lane, dist, msq);
    }
}

template <typename ST>
__global__ __launch_bounds__(256) void consensus_kernel(const ST *__restrict__ X, const RoundParams prm,
                                                        double *__restrict__ partials) {
    constexpr int VEC = Storage<ST>::VEC;
    __shared__ double red[4][2];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    double dist = 0.0, msq = 0.0;
    if (prm.tiled) {
        // from 3 workers on every lane walks all rows of its own columns; with 1 or 2 workers that would be 1-2 KB
        // per wavefront step, and a tile is dealt to 1 or 2 lane groups instead (4 units of 8 or 4 tiles: 4 KB)
        if (prm.n <= 1)
            consensus_walk_tiled<ST, 1, 1, 4>(X, prm, wave, lane, dist, msq);
        else if (prm.n <= 2)
            consensus_walk_tiled<ST, 2, 1, 4>(X, prm, wave, lane, dist, msq);
        else
            consensus_walk_by_column<ST>(X, prm, wave, lane, dist, msq);
    } else {
        constexpr int TILE = 64 * VEC;
        const int64_t ntiles = (prm.N + TILE - 1) / TILE;
        for (int it = 0;; ++it) {
            const int64_t t = unit_index(it, 4, wave);
            if (t >= ntiles) break;   // wave-uniform
            LaneCols lc;
            lc.tile0 = t * TILE;
            lc.loff = (uint32_t)lane * VEC;
            lc.lo = 0;
            lc.hi = prm.N;
            if (prm.vec_ok && lc.tile0 + TILE <= prm.N)
                consensus_tile<ST, true>(X, prm, lc, dist, msq);
            else
                consensus_tile<ST, false>(X, prm, lc, dist, msq);
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        dist += __shfl_xor(dist, off, 64);
        msq += __shfl_xor(msq, off, 64);
    }
    if (lane == 0) {
        red[wave][0] = dist;
        red[wave][1] = msq;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        partials[2 * blockIdx.x + 0] = (red[0][0] + red[1][0]) + (red[2][0] + red[3][0]);
        partials[2 * blockIdx.x + 1] = (red[0][1] + red[1][1]) + (red[2][1] + red[3][1]);
    }
}

// One workgroup: fixed-order sum of the per-workgroup partials -> out[0] = distance, out[1] = ||xbar||^2.
__global__ __launch_bounds__(256) void consensus_final_kernel(const double *__restrict__ partials, int count,
                                                              double *__restrict__ out) {
    __shared__ double red[256][2];
    double d = 0.0, m = 0.0;
    for (int k = threadIdx.x; k < count; k += 256) {
        d += partials[2 * k];
        m += partials[2 * k + 1];
    }
    red[threadIdx.x][0] = d;
    red[threadIdx.x][1] = m;
    __syncthreads();
    for (int half = 128; half >= 1; half >>= 1) {
        if ((int)threadIdx.x < half) {
            red[threadIdx.x][0] += red[threadIdx.x + half][0];
            red[threadIdx.x][1] += red[threadIdx.x + half][1];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        out[0] = red[0][0];
        out[1] = red[0][1];
    }
}

}  // namespace

hipError_t launch_masks(RoundTable *tab, int n, int blocks, uint64_t seed, uint64_t step, uint64_t threshold,
                        int server_mode, hipStream_t stream) {
    hipLaunchKernelGGL(masks_kernel, dim3((unsigned)blocks), dim3(64), 0, stream, tab, n, (uint32_t)seed,
                       (uint32_t)(seed >> 32), (uint32_t)step, (uint32_t)((step >> 32) & 0xFFFFFFu), threshold,
                       server_mode);
    return hipGetLastError();
}

hipError_t launch_mixing_moments(double *out, int workgroups, int64_t rounds, int n, int blocks, uint64_t seed,
                                 uint64_t first_step, uint64_t threshold, int server_mode, hipStream_t stream) {
    hipLaunchKernelGGL(mixing_moments_kernel, dim3((unsigned)workgroups), dim3(64), 0, stream, out, rounds, n, blocks,
                       (uint32_t)seed, (uint32_t)(seed >> 32), first_step, threshold, server_mode);
    return hipGetLastError();
}

hipError_t launch_round(int dtype, int grad_mode, void *X, const void *G, const RoundTable *tab,
                        const RoundParams &prm, int64_t max_block_cols, const LaunchTuning &tune, hipStream_t stream) {
    if (dtype == 0)
        return launch_round_g<float>(grad_mode, (float *)X, (const float *)G, tab, prm, max_block_cols, tune, stream);
    return launch_round_g<uint16_t>(grad_mode, (uint16_t *)X, (const uint16_t *)G, tab, prm, max_block_cols, tune,
                                    stream);
}

hipError_t launch_local_step(int dtype, int grad_mode, void *X, const void *G, const RoundParams &prm,
                             int tiles_per_wave, hipStream_t stream) {
    if (dtype == 0) return launch_local_step_g<float>(grad_mode, (float *)X, (const float *)G, prm, tiles_per_wave, stream);
    return launch_local_step_g<uint16_t>(grad_mode, (uint16_t *)X, (const uint16_t *)G, prm, tiles_per_wave, stream);
}

hipError_t launch_gradavg(int dtype, void *X, const void *G, const RoundTable *tab, const RoundParams &prm,
                          int64_t max_block_cols, int max_waves_per_cu, hipStream_t stream) {
    const int vec = dtype == 0 ? 4 : 8;
    if (prm.tiled) {
        // lane groups per tile as in launch_round_narrow: a lane gets two row pairs where the workers allow it
        const int pg = gradavg_lane_groups(prm.n);
        const int64_t width = (int64_t)(8 / pg) * kTiledLanes * vec;   // columns per wavefront
        const int64_t steps = (max_block_cols + 2 * width - 2) / width;
        // no cap asked for (the default for fp32 with 24 or more workers: +3 % there, nothing or a loss with
        // fewer): one workgroup of 14 wavefronts; otherwise single wavefronts under the cap
        const int wpb = (dtype == 0 && max_waves_per_cu == 0) ? 14 : 1;
        const dim3 grid = folded_grid8((steps + wpb - 1) / wpb, (unsigned)prm.blocks);
        size_t lds = 0;
        if (max_waves_per_cu > 0 && max_waves_per_cu < 32) {
            lds = ((size_t)kLdsBytesPerCu / max_waves_per_cu) & ~(size_t)255;
            if (lds > 65536) lds = 65536;
        }
#define RPS_GA(ST, PG)                                                                                                  \
    do {                                                                                                                \
        if (wpb == 14)                                                                                                  \
            hipLaunchKernelGGL((gradavg_kernel_narrow<ST, PG, 14>), grid, dim3(14 * 64), lds, stream, (ST *)X, (const ST *)G, \
                               tab, prm);                                                                               \
        else                                                                                                            \
            hipLaunchKernelGGL((gradavg_kernel_narrow<ST, PG, 1>), grid, dim3(64), lds, stream, (ST *)X, (const ST *)G, tab,  \
                               prm);                                                                                    \
    } while (0)
        if (dtype == 0) {
            if (pg == 8) RPS_GA(float, 8); else if (pg == 4) RPS_GA(float, 4); else if (pg == 2) RPS_GA(float, 2); else RPS_GA(float, 1);
        } else {
            if (pg == 8) RPS_GA(uint16_t, 8); else if (pg == 4) RPS_GA(uint16_t, 4); else if (pg == 2) RPS_GA(uint16_t, 2); else RPS_GA(uint16_t, 1);
        }
#undef RPS_GA
        return hipGetLastError();
    }
    const int64_t tile = 64 * vec;
    const int64_t tiles = (max_block_cols + 2 * tile - 2) / tile;
    const dim3 grid = folded_grid((tiles + 3) / 4, (unsigned)prm.blocks);
    size_t lds = 0;
    if (max_waves_per_cu > 0 && max_waves_per_cu < 32) {
        int wgs = max_waves_per_cu / 4;
        if (wgs < 1) wgs = 1;
        lds = ((size_t)kLdsBytesPerCu / wgs) & ~(size_t)255;
        if (lds > 65536) lds = 65536;
    }
    if (dtype == 0)
        hipLaunchKernelGGL(gradavg_kernel<float>, grid, dim3(256), lds, stream, (float *)X, (const float *)G, tab, prm);
    else
        hipLaunchKernelGGL(gradavg_kernel<uint16_t>, grid, dim3(256), lds, stream, (uint16_t *)X, (const uint16_t *)G,
                           tab, prm);
    return hipGetLastError();
}

constexpr int kConvertUnits = 4;
// Re-arrangement between the two layouts.  A wavefront unit is 1 KB of the tile-major array in storage
// order (8 segments of 128 bytes: lane / 8 -> segment, lane % 8 -> 16-byte group) and the matching
// 128-byte pieces of up to 8 rows of the row-major array.  TO_TILED: padding columns of the last
// tile are written as zeros.  Byte-wise copy: ELEM is the element size.
template <int ELEM, bool TO_TILED>
__global__ __launch_bounds__(256) void convert_layout_kernel(void *__restrict__ dst, const void *__restrict__ src, int64_t N,
                                                             int64_t pitch, int n, int aligned) {
    constexpr int LPR = kTiledLanes, VEC = 16 / ELEM, TILE = LPR * VEC;
    constexpr int U = kConvertUnits;   // 1 KB units per wavefront, adjacent in the tile-major array: all loads, then all stores
    const int64_t q0 = (linear_block() * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6)) * U;
    const int lane = threadIdx.x & 63;
    char *d = (char *)dst;
    const char *sp = (const char *)src;
    int64_t t_off[U], r_off[U], c0[U];
    bool live[U], whole[U];
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t seg0 = (q0 + u) * (64 / LPR);
        int64_t tile = seg0 / n;
        int i = (int)(seg0 % n) + lane / LPR;
        while (i >= n) {
            i -= n;
            ++tile;
        }
        c0[u] = tile * TILE + (lane % LPR) * VEC;
        live[u] = tile * TILE < N;   // not past the last tile
        whole[u] = live[u] && aligned && c0[u] + VEC <= N;
        t_off[u] = ((seg0 + lane / LPR) * TILE + (lane % LPR) * VEC) * ELEM;   // bytes, tile-major array
        r_off[u] = ((int64_t)i * pitch + c0[u]) * ELEM;                         // bytes, row-major array
        if (whole[u]) v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(sp + (TO_TILED ? r_off[u] : t_off[u])));
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (whole[u]) {
            __builtin_nontemporal_store(v[u], reinterpret_cast<u32x4 *>(d + (TO_TILED ? t_off[u] : r_off[u])));
        } else if (live[u]) {
            for (int e = 0; e < VEC; ++e) {
                for (int b = 0; b < ELEM; ++b) {
                    if (TO_TILED)
                        d[t_off[u] + e * ELEM + b] = c0[u] + e < N ? sp[r_off[u] + e * ELEM + b] : (char)0;
                    else if (c0[u] + e < N)
                        d[r_off[u] + e * ELEM + b] = sp[t_off[u] + e * ELEM + b];
                }
            }
        }
    }
}

hipError_t launch_convert_layout(int dtype, void *dst, const void *src, int64_t N, int64_t pitch, int n, bool to_tiled,
                                 bool aligned, hipStream_t stream) {
    const int elem = dtype == 0 ? 4 : 2;
    const int64_t T = kTiledLanes * (16 / elem);
    const int64_t tiles = (N + T - 1) / T;
    const int64_t kb = (tiles * n * kTiledLanes + 63) / 64;   // 1 KB units
    const dim3 grid = folded_grid((kb + 4 * kConvertUnits - 1) / (4 * kConvertUnits), 1);
    if (dtype == 0) {
        if (to_tiled)
            hipLaunchKernelGGL((convert_layout_kernel<4, true>), grid, dim3(256), 0, stream, dst, src, N, pitch, n, (int)aligned);
        else
            hipLaunchKernelGGL((convert_layout_kernel<4, false>), grid, dim3(256), 0, stream, dst, src, N, pitch, n, (int)aligned);
    } else {
        if (to_tiled)
            hipLaunchKernelGGL((convert_layout_kernel<2, true>), grid, dim3(256), 0, stream, dst, src, N, pitch, n, (int)aligned);
        else
            hipLaunchKernelGGL((convert_layout_kernel<2, false>), grid, dim3(256), 0, stream, dst, src, N, pitch, n, (int)aligned);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Reduction scratch for callers that cannot allocate: one array per GPU, living in the code
// object's global segment, as large as the scratch a context allocates (the consensus kernels
// are launched with at most kMaxPartials workgroups, so it serves every width the interface
// accepts).  `scratch` below is a host-side stand-in for the symbol, NOT a device address:
// host code must go through the pointer resolved per device by static_scratch().
// ---------------------------------------------------------------------------------------
namespace {
static __device__ __align__(256) double scratch[2 * kMaxPartials];
constexpr int kMaxDevices = 64;
std::atomic<double *> g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU, resolved on first use
}  // namespace

hipError_t static_scratch(int device, double **out) {
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    double *p = g_scratch_ptr[device].load(std::memory_order_acquire);
    if (p == nullptr) {   // `device` is current (the caller's guard); every GPU has its own copy at its own address
        int cur = -1;
        hipError_t e = hipGetDevice(&cur);
        if (e != hipSuccess) return e;
        if (cur != device) return hipErrorInvalidDevice;
        void *addr = nullptr;
        e = hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (addr == nullptr) return hipErrorInvalidSymbol;
        p = static_cast<double *>(addr);
        g_scratch_ptr[device].store(p, std::memory_order_release);   // racing first calls resolve the same address
    }
    *out = p;
    return hipSuccess;
}

hipError_t launch_consensus(int dtype, const void *X, const RoundParams &prm, double *partials, int max_partials,
                            double *out, hipStream_t stream) {
    // units of one wavefront step: a tile of 64 lanes x 16 bytes (row-major), or 32 / 16 / 8 tiles of 128 bytes (tiled)
    int64_t tile = dtype == 0 ? 256 : 512;
    if (prm.tiled) tile = (tile / 8) * (prm.n <= 1 ? 32 : (prm.n <= 2 ? 16 : 8));   // as consensus_kernel deals them out
    const int64_t ntiles = (prm.N + tile - 1) / tile;
    int64_t wgs = ((ntiles + 3) / 4 + 7) & ~(int64_t)7;   // unit_index(): a multiple of 8 workgroups
    if (wgs > max_partials) wgs = max_partials;
    if (dtype == 0)
        hipLaunchKernelGGL(consensus_kernel<float>, dim3((unsigned)wgs), dim3(256), 0, stream, (const float *)X, prm,
                           partials);
    else
        hipLaunchKernelGGL(consensus_kernel<uint16_t>, dim3((unsigned)wgs), dim3(256), 0, stream,
                           (const uint16_t *)X, prm, partials);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(consensus_final_kernel, dim3(1), dim3(256), 0, stream, partials, (int)wgs, out);
    return hipGetLastError();
}

}  // namespace rps
