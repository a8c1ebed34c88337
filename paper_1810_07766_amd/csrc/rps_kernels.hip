// HIP kernels (gfx950 / CDNA4, wave64) of the RPS lossy model-averaging round of
// "Distributed Learning over Unreliable Networks" (arXiv 1810.07766), Sec. 4.1 / Alg. 1.
//
// Compile with -ffp-contract=off: the synthetic-gradient noise is specified as an exact
// sequence of IEEE fp32 operations and every fused multiply-add is written explicitly.
//
// Kernels
//   masks_kernel      network outcome of one round: server permutation, uplink and downlink
//                     delivery bits (Sec. 3; Alg. 1 steps 6-7), n workgroups of one wavefront
//   round_kernel      local SGD step + Reduce-Scatter average + All-Gather write-back in one
//                     pass; one workgroup per tile of 512 columns of one block, rows split
//                     over the workgroup's wavefronts
//   local_step_kernel the local SGD step alone
// The path is a streaming reduction with < 0.5 flop per byte: it is bound by HBM bandwidth
// (and, with the in-register Gaussian generator, by plain vector ALU work), never by a dense
// contraction, so there is no MFMA here.
#include "rps_internal.h"

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

constexpr uint32_t kDomainUplink = 0u << 24, kDomainDownlink = 1u << 24, kDomainServer = 2u << 24,
                   kDomainNoise = 3u << 24;
constexpr int kMaskRounds = 10, kNoiseRounds = 10;

// ---------------------------------------------------------------------------------------
// Network outcome (Sec. 3: every message lost independently with probability p; Alg. 1
// step 6: servers drawn uniformly without replacement).  Workgroup j = block j, lane i =
// worker i.  The permutation is a rank sort of per-worker hash keys: natively parallel,
// n compare steps through wavefront shuffles.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void masks_kernel(RoundTable *__restrict__ tab, int n, uint32_t seed_lo,
                                                   uint32_t seed_hi, uint32_t step_lo, uint32_t step_hi24,
                                                   uint64_t threshold, int identity_server) {
    const int j = blockIdx.x;
    const int i = threadIdx.x;
    const bool active = i < n;

    int s = j;
    if (!identity_server) {
        uint32_t c[4] = {(uint32_t)i, 0u, step_lo, kDomainServer | step_hi24};
        philox4x32<kMaskRounds>(c, seed_lo, seed_hi);
        const uint32_t key = c[0];
        int rank = 0;
        for (int k = 0; k < n; ++k) {
            const uint32_t other = __shfl(key, k, 64);
            rank += (other < key || (other == key && k < i)) ? 1 : 0;
        }
        const uint64_t hit = __ballot(active && rank == j);
        s = __ffsll((long long)hit) - 1;   // exactly one lane has rank j
    }

    uint32_t cu[4] = {(uint32_t)i, (uint32_t)j, step_lo, kDomainUplink | step_hi24};
    philox4x32<kMaskRounds>(cu, seed_lo, seed_hi);
    uint32_t cd[4] = {(uint32_t)i, (uint32_t)j, step_lo, kDomainDownlink | step_hi24};
    philox4x32<kMaskRounds>(cd, seed_lo, seed_hi);
    // a worker's link to itself is not a network message: forced after the draw
    const bool up = active && ((uint64_t)cu[0] >= threshold || i == s);
    const bool down = active && ((uint64_t)cd[0] >= threshold || i == s);
    const uint64_t ucol = __ballot(up);
    const uint64_t dcol = __ballot(down);
    if (i == 0) {
        const int cnt = __popcll(ucol);
        tab->ucol[j] = ucol;
        tab->dcol[j] = dcol;
        tab->cnt[j] = cnt;
        tab->inv_cnt[j] = 1.0 / (double)cnt;
        tab->server[j] = s;
    }
}

// ---------------------------------------------------------------------------------------
// Synthetic gradient noise: one hash call -> eight values sigma*z for columns 8g..8g+7 of one
// worker.  Each word gives a Box-Muller pair: 16-bit radius index (low half), 16-bit angle
// index (high half).  Every operation below is an exactly rounded fp32 operation in a fixed
// order, so the bits do not depend on the machine.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ void box_muller_pair(uint32_t word, float sigma, float &even, float &odd) {
    // u1 = a / 2^17 (a odd);  -log2 u1 = lz + (1 - log2 m),  m in [1,2),  w = 2 - m
    const uint32_t a = ((word & 0xFFFFu) << 1) | 1u;
    const int nlz = __builtin_clz(a);   // 15..31
    const float m = __uint_as_float((a << (nlz - 8)) + 0x3F000000u);
    const float w = 2.0f - m;
    const float lzf = (float)(nlz - 15);
    float q = __builtin_fmaf(w, 0x1.767762p-5f, -0x1.6ad1d8p-8f);
    q = __builtin_fmaf(w, q, 0x1.9117f8p-4f);
    q = __builtin_fmaf(w, q, 0x1.fc1588p-3f);
    q = __builtin_fmaf(w, q, 0x1.000288p+0f);
    const float t = w * q;                                        // -2 ln(1 - w/2)
    const float L = __builtin_fmaf(lzf, 0x1.62e430p+0f, t);       // -2 ln u1
    // r = L * rsqrt(L): bit-trick seed and two Newton steps
    const float h = 0.5f * L;
    float y = __uint_as_float(0x5F3759DFu - (__float_as_uint(L) >> 1));
    y = y * __builtin_fmaf(-h, y * y, 1.5f);
    y = y * __builtin_fmaf(-h, y * y, 1.5f);
    const float rs = sigma * (L * y);
    // angle x = (2f+1) pi/65536 with f the signed 15-bit field [30:16]; bit 31 adds pi
    const int32_t f = (int32_t)(word << 1) >> 17;
    const float x = (float)(2 * f + 1) * 0x1.921fb6p-15f;
    const float x2 = x * x;
    float sp = __builtin_fmaf(x2, -0x1.8b3e4ep-13f, 0x1.10c46cp-7f);
    sp = __builtin_fmaf(x2, sp, -0x1.5554aep-3f);
    const float sn = __builtin_fmaf(x * x2, sp, x);
    float cp = __builtin_fmaf(x2, -0x1.54c10ap-10f, 0x1.54aa20p-5f);
    cp = __builtin_fmaf(x2, cp, -0x1.fffd12p-2f);
    const float cs = __builtin_fmaf(x2, cp, 1.0f);
    const float rsgn = __uint_as_float(__float_as_uint(rs) | (word & 0x80000000u));
    even = rsgn * cs;
    odd = rsgn * sn;
}

__device__ __forceinline__ void noise8(const RoundParams &prm, int worker, int64_t group, float z[8]) {
    uint32_t c[4] = {(uint32_t)group, (uint32_t)worker, prm.step_lo, kDomainNoise | prm.step_hi24};
    philox4x32<kNoiseRounds>(c, prm.seed_lo, prm.seed_hi);
#pragma unroll
    for (int q = 0; q < 4; ++q) box_muller_pair(c[q], prm.sigma, z[2 * q], z[2 * q + 1]);
}

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

template <typename ST>
struct Storage;

template <>
struct Storage<float> {
    static __device__ __forceinline__ float round(float v) { return v; }
    static __device__ __forceinline__ void load8(const float *p, float x[8]) {
        const float4 a = reinterpret_cast<const float4 *>(p)[0];
        const float4 b = reinterpret_cast<const float4 *>(p)[1];
        x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
        x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
    }
    static __device__ __forceinline__ void store8(float *p, const float x[8]) {
        reinterpret_cast<float4 *>(p)[0] = make_float4(x[0], x[1], x[2], x[3]);
        reinterpret_cast<float4 *>(p)[1] = make_float4(x[4], x[5], x[6], x[7]);
    }
    static __device__ __forceinline__ float load1(const float *p) { return *p; }
    static __device__ __forceinline__ void store1(float *p, float v) { *p = v; }
};

template <>
struct Storage<uint16_t> {
    static __device__ __forceinline__ float round(float v) { return bf16_bits_to_f32(f32_to_bf16_bits(v)); }
    static __device__ __forceinline__ void load8(const uint16_t *p, float x[8]) {
        const uint4 a = *reinterpret_cast<const uint4 *>(p);
        x[0] = __uint_as_float(a.x << 16); x[1] = __uint_as_float(a.x & 0xFFFF0000u);
        x[2] = __uint_as_float(a.y << 16); x[3] = __uint_as_float(a.y & 0xFFFF0000u);
        x[4] = __uint_as_float(a.z << 16); x[5] = __uint_as_float(a.z & 0xFFFF0000u);
        x[6] = __uint_as_float(a.w << 16); x[7] = __uint_as_float(a.w & 0xFFFF0000u);
    }
    // values are already bf16-representable (rounded by round()): packing is a truncation
    static __device__ __forceinline__ void store8(uint16_t *p, const float x[8]) {
        uint4 a;
        a.x = (__float_as_uint(x[0]) >> 16) | (__float_as_uint(x[1]) & 0xFFFF0000u);
        a.y = (__float_as_uint(x[2]) >> 16) | (__float_as_uint(x[3]) & 0xFFFF0000u);
        a.z = (__float_as_uint(x[4]) >> 16) | (__float_as_uint(x[5]) & 0xFFFF0000u);
        a.w = (__float_as_uint(x[6]) >> 16) | (__float_as_uint(x[7]) & 0xFFFF0000u);
        *reinterpret_cast<uint4 *>(p) = a;
    }
    static __device__ __forceinline__ float load1(const uint16_t *p) { return bf16_bits_to_f32(*p); }
    static __device__ __forceinline__ void store1(uint16_t *p, float v) { *p = (uint16_t)(__float_as_uint(v) >> 16); }
};

// Load / store the lane's eight columns [c0, c0+8) of one row; `full` lanes use 128-bit
// accesses, ragged lanes touch only columns inside [lo, hi).
template <typename ST>
__device__ __forceinline__ void load_cols(const ST *row, int64_t c0, int64_t lo, int64_t hi, bool full, float x[8]) {
    if (full) {
        Storage<ST>::load8(row + c0, x);
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int64_t c = c0 + e;
            x[e] = (c >= lo && c < hi) ? Storage<ST>::load1(row + c) : 0.0f;
        }
    }
}
template <typename ST>
__device__ __forceinline__ void store_cols(ST *row, int64_t c0, int64_t lo, int64_t hi, bool full, const float x[8]) {
    if (full) {
        Storage<ST>::store8(row + c0, x);
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int64_t c = c0 + e;
            if (c >= lo && c < hi) Storage<ST>::store1(row + c, x[e]);
        }
    }
}

// v = x - gamma * g, rounded to storage (Alg. 1 step 5).  x holds the row's eight values on
// entry and v on exit.
template <typename ST, int GRAD>
__device__ __forceinline__ void sgd_step(const RoundParams &prm, const ST *Grow, int worker, int64_t c0, int64_t lo,
                                         int64_t hi, bool full, float x[8]) {
    if (GRAD == kGradBuffer) {
        float g[8];
        load_cols<ST>(Grow, c0, lo, hi, full, g);
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = Storage<ST>::round(__builtin_fmaf(-prm.gamma, g[e], x[e]));
    } else if (GRAD == kGradSynthetic) {
        float z[8];
        noise8(prm, worker, c0 >> 3, z);
        if (prm.lambda != 0.0f) {   // fma(0, x, z) == z for finite x: skipped when there is no decay
#pragma unroll
            for (int e = 0; e < 8; ++e) z[e] = __builtin_fmaf(prm.lambda, x[e], z[e]);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = Storage<ST>::round(__builtin_fmaf(-prm.gamma, z[e], x[e]));
    }
}

// ---------------------------------------------------------------------------------------
// Fused round.  grid = (tiles of the largest block, n blocks); workgroup = W wavefronts.
// Lane l of every wavefront owns columns base + (tile*64 + l)*8 .. +8 of block j, where base
// is the block start rounded down to a multiple of 8 (so lanes coincide with noise groups and
// 128-bit segments).  Wavefront w owns rows w, w+W, ...: the "is this copy delivered" tests
// are wave-uniform scalar branches.  Partial column sums are accumulated in fp64, exchanged
// through LDS once per tile, and every wavefront forms the same average in the same order
// (so all receivers hold identical bits).  Each element is read at most once and written at
// most once; a row that neither contributes (uplink lost) nor keeps its own value (reply
// received) is not read at all.
// ---------------------------------------------------------------------------------------
template <typename ST, int GRAD, int W, int RPW>
__global__ __launch_bounds__(W * 64) void round_kernel(ST *__restrict__ X, const ST *__restrict__ G,
                                                       const RoundTable *__restrict__ tab, const RoundParams prm) {
    __shared__ double2 part[W][4][64];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int j = blockIdx.y;
    const int64_t lo = tab->off[j], hi = tab->off[j + 1];
    const int64_t base = lo & ~(int64_t)7;
    const int64_t tile0 = base + (int64_t)blockIdx.x * kTileCols;
    if (tile0 >= hi) return;   // uniform: this block has fewer tiles than the largest one
    const uint64_t ucol = tab->ucol[j], dcol = tab->dcol[j];
    const double inv = tab->inv_cnt[j];

    const int64_t c0 = tile0 + (int64_t)lane * kColsPerLane;
    const bool any = c0 < hi;   // (c0 + 8 > lo always holds)
    const bool full = prm.vec_ok && c0 >= lo && c0 + kColsPerLane <= hi;

    float v[RPW][8];
    double acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.0;

#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        const int i = wave + r * W;
        if (i < prm.n) {
            const bool u = (ucol >> i) & 1, d = (dcol >> i) & 1;
            if ((u || (!d && GRAD != kGradNone)) && any) {
                const ST *row = X + (int64_t)i * prm.N;
                load_cols<ST>(row, c0, lo, hi, full, v[r]);
                sgd_step<ST, GRAD>(prm, G ? G + (int64_t)i * prm.N : nullptr, i, c0, lo, hi, full, v[r]);
                if (u) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[e] += (double)v[r][e];
                }
            }
        }
    }

#pragma unroll
    for (int k = 0; k < 4; ++k) part[wave][k][lane] = make_double2(acc[2 * k], acc[2 * k + 1]);
    __syncthreads();
    float vt[8];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        double2 t = part[0][k][lane];
#pragma unroll
        for (int w = 1; w < W; ++w) {
            const double2 o = part[w][k][lane];
            t.x += o.x;
            t.y += o.y;
        }
        vt[2 * k] = Storage<ST>::round((float)(t.x * inv));
        vt[2 * k + 1] = Storage<ST>::round((float)(t.y * inv));
    }

#pragma unroll
    for (int r = 0; r < RPW; ++r) {
        const int i = wave + r * W;
        if (i < prm.n && any) {
            ST *row = X + (int64_t)i * prm.N;
            if ((dcol >> i) & 1)
                store_cols<ST>(row, c0, lo, hi, full, vt);
            else if (GRAD != kGradNone)
                store_cols<ST>(row, c0, lo, hi, full, v[r]);
        }
    }
}

// Local SGD step alone: grid = (column-group chunks, n rows), lane = one 8-column group.
template <typename ST, int GRAD>
__global__ __launch_bounds__(256) void local_step_kernel(ST *__restrict__ X, const ST *__restrict__ G,
                                                         const RoundParams prm) {
    const int i = blockIdx.y;
    const int64_t c0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * kColsPerLane;
    if (c0 >= prm.N) return;
    const bool full = prm.vec_ok && c0 + kColsPerLane <= prm.N;
    ST *row = X + (int64_t)i * prm.N;
    float x[8];
    load_cols<ST>(row, c0, 0, prm.N, full, x);
    sgd_step<ST, GRAD>(prm, G ? G + (int64_t)i * prm.N : nullptr, i, c0, 0, prm.N, full, x);
    store_cols<ST>(row, c0, 0, prm.N, full, x);
}

template <typename ST, int GRAD>
hipError_t launch_round_t(ST *X, const ST *G, const RoundTable *tab, const RoundParams &prm,
                          int64_t max_block_cols, hipStream_t stream) {
    // a block that starts off an 8-column boundary may need one extra tile
    const int64_t tiles = (max_block_cols + 7 + kTileCols - 1) / kTileCols;
    const dim3 grid((unsigned)tiles, (unsigned)prm.n, 1);
    const int n = prm.n;
    if (n <= 4)
        hipLaunchKernelGGL((round_kernel<ST, GRAD, 4, 1>), grid, dim3(256), 0, stream, X, G, tab, prm);
    else if (n <= 8)
        hipLaunchKernelGGL((round_kernel<ST, GRAD, 4, 2>), grid, dim3(256), 0, stream, X, G, tab, prm);
    else if (n <= 16)
        hipLaunchKernelGGL((round_kernel<ST, GRAD, 4, 4>), grid, dim3(256), 0, stream, X, G, tab, prm);
    else if (n <= 32)
        hipLaunchKernelGGL((round_kernel<ST, GRAD, 4, 8>), grid, dim3(256), 0, stream, X, G, tab, prm);
    else
        hipLaunchKernelGGL((round_kernel<ST, GRAD, 8, 8>), grid, dim3(512), 0, stream, X, G, tab, prm);
    return hipGetLastError();
}

template <typename ST>
hipError_t launch_round_g(int grad_mode, ST *X, const ST *G, const RoundTable *tab, const RoundParams &prm,
                          int64_t max_block_cols, hipStream_t stream) {
    switch (grad_mode) {
        case kGradNone: return launch_round_t<ST, kGradNone>(X, G, tab, prm, max_block_cols, stream);
        case kGradBuffer: return launch_round_t<ST, kGradBuffer>(X, G, tab, prm, max_block_cols, stream);
        default: return launch_round_t<ST, kGradSynthetic>(X, G, tab, prm, max_block_cols, stream);
    }
}

template <typename ST>
hipError_t launch_local_step_g(int grad_mode, ST *X, const ST *G, const RoundParams &prm, hipStream_t stream) {
    const int64_t groups = (prm.N + kColsPerLane - 1) / kColsPerLane;
    const dim3 grid((unsigned)((groups + 255) / 256), (unsigned)prm.n, 1);
    if (grad_mode == kGradBuffer)
        hipLaunchKernelGGL((local_step_kernel<ST, kGradBuffer>), grid, dim3(256), 0, stream, X, G, prm);
    else
        hipLaunchKernelGGL((local_step_kernel<ST, kGradSynthetic>), grid, dim3(256), 0, stream, X, G, prm);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_masks(RoundTable *tab, int n, uint64_t seed, uint64_t step, uint64_t threshold,
                        int identity_server, hipStream_t stream) {
    hipLaunchKernelGGL(masks_kernel, dim3((unsigned)n), dim3(64), 0, stream, tab, n, (uint32_t)seed,
                       (uint32_t)(seed >> 32), (uint32_t)step, (uint32_t)((step >> 32) & 0xFFFFFFu), threshold,
                       identity_server);
    return hipGetLastError();
}

hipError_t launch_round(int dtype, int grad_mode, void *X, const void *G, const RoundTable *tab,
                        const RoundParams &prm, int64_t max_block_cols, hipStream_t stream) {
    if (dtype == 0)
        return launch_round_g<float>(grad_mode, (float *)X, (const float *)G, tab, prm, max_block_cols, stream);
    return launch_round_g<uint16_t>(grad_mode, (uint16_t *)X, (const uint16_t *)G, tab, prm, max_block_cols, stream);
}

hipError_t launch_local_step(int dtype, int grad_mode, void *X, const void *G, const RoundParams &prm,
                             hipStream_t stream) {
    if (dtype == 0) return launch_local_step_g<float>(grad_mode, (float *)X, (const float *)G, prm, stream);
    return launch_local_step_g<uint16_t>(grad_mode, (uint16_t *)X, (const uint16_t *)G, prm, stream);
}

}  // namespace rps
