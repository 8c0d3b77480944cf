// All-pairs inner products of up to 64 micro-gradients in one read of the data
// (Eq. 4 needs g_i . g_j for every pair; Fig. 1c/d logs the resulting distances).
//
// G = X X^T with X the (rows x P) matrix whose rows are the gradients. The
// contraction runs over P, so it maps onto the matrix cores with P as the K
// dimension. Rows are taken in groups of 16; for every pair of groups (a <= b)
// one 16x16 accumulator tile is kept per wavefront:
//   binary32 rows: v_mfma_f32_16x16x4_f32   (lane l supplies row l%16, k = l/16)
//   bfloat16 rows: v_mfma_f32_16x16x32_bf16 (lane l supplies row l%16, k = 8*(l/16)..+7)
// Both operands of either instruction use the same lane layout and the sum runs
// over all k, so a register loaded from memory serves as A or as B unchanged.
// Four groups (64 rows) need 10 tiles; the symmetric half is never computed.
//
// Per wavefront step every lane reads 32 contiguous bytes of its row (two
// 16-byte nontemporal loads), four lanes cover one 128-byte line of the row, and
// the loads of the next step are issued before the MFMAs of the current one.
// Tiles accumulate in binary32 inside the matrix core and are flushed every
// kGramFlush steps into binary64 totals that live in LDS, one private region
// per wavefront (keeping them in registers pushed the 10-tile kernel past 256
// VGPRs, i.e. down to one wavefront per SIMD).
#pragma once
#include "gaf_device.hpp"

namespace gaf {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

constexpr int kGramGroups = 4;          // row groups per launch
constexpr int kGramRows = 16 * kGramGroups;
constexpr int kGramFlush = 16;          // steps between binary32 -> binary64 flushes
constexpr int kGramThreads = 128;       // 2 wavefronts per workgroup (LDS totals: 2 x 20 KB at 10 tiles)
constexpr int kGramWaves = kGramThreads / 64;
constexpr int kGramBlocks = 1024;       // workgroups per launch (fixed: the summation order depends on it)
constexpr int kGramTile = 16 * 16;      // entries per tile
constexpr int kGramMaxTiles = 10;       // 4 groups: 4 diagonal + 6 off-diagonal tiles

// Which tiles a launch computes.
//   kFull : every pair (a <= b) of the NG groups               -> NG (NG + 1) / 2 tiles
//   kCross: groups {0,1} against groups {2,3} (NG must be 4)   -> 4 tiles
enum GramMode { kFull = 0, kCross = 1 };

// Tiles are numbered so that the first NG (NG + 1) / 2 of them are exactly the
// pairs among the first NG groups: (0,0) (0,1) (1,1) (0,2) (1,2) (2,2) (0,3) ...
template <int NG, int kMode>
struct TileList {
    static constexpr int count = kMode == kFull ? NG * (NG + 1) / 2 : 4;
    // tile t -> (row group, column group)
    __host__ __device__ static constexpr int ga(int t)
    {
        constexpr int full[kGramMaxTiles] = {0, 0, 1, 0, 1, 2, 0, 1, 2, 3};
        constexpr int cross[4] = {0, 0, 1, 1};
        return kMode == kFull ? full[t] : cross[t];
    }
    __host__ __device__ static constexpr int gb(int t)
    {
        constexpr int full[kGramMaxTiles] = {0, 1, 1, 2, 2, 2, 3, 3, 3, 3};
        constexpr int cross[4] = {2, 3, 2, 3};
        return kMode == kFull ? full[t] : cross[t];
    }
};

struct GramArgs {
    const void *rows[kGramRows];  // DEVICE pointers, group g = rows[16 g .. 16 g + 15]; never NULL: rows past
                                  // the last gradient alias a real one and their tile entries are dropped
    size_t P;
    double *ws;                   // [kGramBlocks][kGramMaxTiles][kGramTile] per-workgroup tiles
};

// ---- one step's worth of one row for one lane: 32 bytes --------------------
template <typename T> struct GramTraits;
template <> struct GramTraits<float> {
    static constexpr int kLane = 8;                 // elements per lane per step
    typedef f32x4_t raw;
};
template <> struct GramTraits<bf16_t> {
    static constexpr int kLane = 16;
    typedef u32x4_t raw;
};

template <typename T>
__device__ __forceinline__ void gram_load(const T *row, size_t p, typename GramTraits<T>::raw (&v)[2])
{
    typedef typename GramTraits<T>::raw raw;
    constexpr int half = GramTraits<T>::kLane / 2;
    v[0] = __builtin_nontemporal_load(reinterpret_cast<const raw *>(row + p));
    v[1] = __builtin_nontemporal_load(reinterpret_cast<const raw *>(row + p + half));
}
__device__ __forceinline__ void gram_load_guarded(const float *row, size_t p, size_t P, f32x4_t (&v)[2])
{
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const size_t q = p + 4 * h + e;
            v[h][e] = q < P ? row[q] : 0.f;
        }
}
__device__ __forceinline__ void gram_load_guarded(const bf16_t *row, size_t p, size_t P, u32x4_t (&v)[2])
{
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const size_t q = p + 8 * h + 2 * e;
            const uint32_t lo = q < P ? row[q] : 0u, hi = q + 1 < P ? row[q + 1] : 0u;
            v[h][e] = lo | (hi << 16);
        }
}

__device__ __forceinline__ void gram_mma(const f32x4_t (&x)[2], const f32x4_t (&y)[2], floatx4 &acc, int h, int e)
{
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(x[h][e], y[h][e], acc, 0, 0, 0);
}
__device__ __forceinline__ void gram_mma(const u32x4_t (&x)[2], const u32x4_t (&y)[2], floatx4 &acc, int h, int)
{
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, x[h]),
                                                  __builtin_bit_cast(bf16x8_t, y[h]), acc, 0, 0, 0);
}

template <typename T, int NG, int kMode>
__global__ __launch_bounds__(kGramThreads) void gram_kernel(GramArgs a)
{
    typedef TileList<NG, kMode> Tiles;
    typedef typename GramTraits<T>::raw raw;
    constexpr int NT = Tiles::count;
    constexpr int kLane = GramTraits<T>::kLane;
    constexpr int kStep = 4 * kLane;                    // elements of each row per wavefront step (128 bytes)
    constexpr int kInner = sizeof(T) == 4 ? 4 : 1;      // MFMAs per 16-byte register

    __shared__ double tot_lds[kGramWaves][NT * kGramTile];   // per-wavefront binary64 totals, <= 40 KB

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 15, kq = lane >> 4;

    // this lane's row in each group, selected with compile-time indices so the
    // pointer table stays in the kernel-argument segment
    const T *row[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        row[g] = nullptr;
#pragma unroll
        for (int k = 0; k < 16; ++k)
            if (r == k) row[g] = static_cast<const T *>(a.rows[16 * g + k]);
    }

    const size_t P = a.P;
    const size_t nwaves = size_t(gridDim.x) * kGramWaves;
    const size_t gw = size_t(blockIdx.x) * kGramWaves + wave;

    // Tile entry in accumulator register v of lane l: row i = 4*(l/16) + v, column j = l%16.
    double *tot = &tot_lds[wave][(4 * kq) * 16 + r];   // + t*kGramTile + v*16
    floatx4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int v = 0; v < 4; ++v) tot[t * kGramTile + v * 16] = 0.0;
    }

    // Hot-loop loads are unconditional (absent rows alias a real row on the host
    // side and their tile entries are dropped later), so the compiler keeps all
    // of a step's loads in flight behind one counter wait.
    auto load_step = [&](size_t s, raw (&x)[NG][2]) {
        const size_t p = s * kStep + size_t(kq) * kLane;
#pragma unroll
        for (int g = 0; g < NG; ++g) gram_load(row[g], p, x[g]);
    };
    auto compute = [&](const raw (&x)[NG][2]) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int e = 0; e < kInner; ++e)
#pragma unroll
                for (int t = 0; t < NT; ++t) gram_mma(x[Tiles::ga(t)], x[Tiles::gb(t)], acc[t], h, e);
    };
    auto flush = [&]() {
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                tot[t * kGramTile + v * 16] += (double)acc[t][v];   // this lane's own LDS slot
                acc[t][v] = 0.f;
            }
    };

    // Full steps, two register buffers: the loads of step k+1 are in flight while
    // step k is multiplied. The steady-state loop has no conditional loads.
    const size_t nfull = P / kStep;
    raw x0[NG][2], x1[NG][2];
    int since_flush = 0;
    auto after_step = [&]() {
        if (++since_flush == kGramFlush) {
            since_flush = 0;
            flush();
        }
    };
    size_t s = gw;
    if (s < nfull) {
        load_step(s, x0);
        while (s + 2 * nwaves < nfull) {
            load_step(s + nwaves, x1);
            compute(x0);
            after_step();
            load_step(s + 2 * nwaves, x0);
            compute(x1);
            after_step();
            s += 2 * nwaves;
        }
        if (s + nwaves < nfull) {
            load_step(s + nwaves, x1);
            compute(x0);
            compute(x1);
        } else {
            compute(x0);
        }
    }
    // ragged tail (P not a multiple of the step): one wavefront, element-wise guarded loads
    if (nfull * kStep < P && gw == nfull % nwaves) {
        const size_t p = nfull * kStep + size_t(kq) * kLane;
#pragma unroll
        for (int g = 0; g < NG; ++g) gram_load_guarded(row[g], p, P, x0[g]);
        compute(x0);
    }
    flush();

    // the workgroup's tile = its wavefronts' totals added in wavefront order
    __syncthreads();
    double *out = a.ws + size_t(blockIdx.x) * kGramMaxTiles * kGramTile;
    for (int e = threadIdx.x; e < NT * kGramTile; e += kGramThreads) {
        double v = tot_lds[0][e];
#pragma unroll
        for (int w = 1; w < kGramWaves; ++w) v += tot_lds[w][e];
        out[e] = v;
    }
}

// Adds the per-workgroup tiles in workgroup order and scatters them into the
// full symmetric matrix of inner products (binary64, leading dimension N).
struct GramFinalArgs {
    const double *ws;
    int nblocks;
    int ntiles;
    int tile_ga[kGramMaxTiles], tile_gb[kGramMaxTiles];  // local group of each tile's rows / columns
    int group_row[kGramGroups];                          // first global row of each local group
    double *gram;   // [N][N]
    int N;
};

// One workgroup handles 16 consecutive tile entries; thread (slice, entry) adds
// the workgroups of its slice in order, then the 16 slice sums are added in
// slice order: a fixed tree, so the result is reproducible.
__global__ __launch_bounds__(kBlock) void gram_finalize_kernel(GramFinalArgs a)
{
    __shared__ double part[16][16];
    const int el = threadIdx.x & 15, slice = threadIdx.x >> 4;
    const int e = blockIdx.x * 16 + el;
    const bool live = e < a.ntiles * kGramTile;
    const int per = (a.nblocks + 15) / 16;
    double s = 0.0;
    if (live) {
        const int b1 = (slice + 1) * per < a.nblocks ? (slice + 1) * per : a.nblocks;
        for (int b = slice * per; b < b1; ++b) s += a.ws[size_t(b) * kGramMaxTiles * kGramTile + e];
    }
    part[slice][el] = s;
    __syncthreads();
    if (slice != 0 || !live) return;
    s = part[0][el];
#pragma unroll
    for (int k = 1; k < 16; ++k) s += part[k][el];
    const int t = e / kGramTile, i = (e % kGramTile) / 16, j = e % 16;
    const int gi = a.group_row[a.tile_ga[t]] + i, gj = a.group_row[a.tile_gb[t]] + j;
    if (gi >= a.N || gj >= a.N) return;
    a.gram[size_t(gi) * a.N + gj] = s;
    if (a.tile_ga[t] != a.tile_gb[t]) a.gram[size_t(gj) * a.N + gi] = s;
}

// Eq. 4 for every pair from the matrix of inner products.
__global__ void gram_to_distance_kernel(const double *gram, int N, float *D, double *gram_out)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= N * N) return;
    const int i = idx / N, j = idx % N;
    const double gij = gram[i <= j ? idx : j * N + i];   // upper triangle: D comes out exactly symmetric
    if (gram_out) gram_out[idx] = gij;
    D[idx] = (i == j) ? 0.f
                      : (float)distance_from_sums(gij, gram[size_t(i) * N + i], gram[size_t(j) * N + j]);
}

}  // namespace gaf
