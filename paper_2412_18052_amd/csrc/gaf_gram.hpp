// All-pairs inner products of up to 64 micro-gradients in one read of the data,
// for the cosine-distance diagnostic (Eq. 4 over every pair; Fig. 1c/d).
//
// G = X X^T with X the (rows x P) matrix whose rows are the gradients. The
// contraction runs over P, so it maps onto the matrix cores with P as the K
// dimension: one v_mfma_f32_32x32x2_f32 multiplies a 32x2 slab of one 32-row
// group with the 2x32 slab of another and adds into a 32x32 accumulator tile.
// The 64 rows form two groups A and B; three tiles (AA, AB, BB) cover the
// symmetric matrix. Both operands of the instruction want "lane l holds row
// l%32, k = l/32", so one register loaded from memory serves as either operand.
#pragma once
#include "gaf_device.hpp"

namespace gaf {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kGramRows = 64;          // rows per launch: two groups of 32
constexpr int kGramStep = 32;          // P-elements consumed per wavefront step (2 lanes x 16 per row)
constexpr int kGramFlush = 64;         // steps between binary32 -> binary64 flushes of the tiles
constexpr int kGramBlocks = 512;       // workgroups per launch (fixed: summation order depends on it)
constexpr int kGramTile = 32 * 32;     // entries per tile

struct GramArgs {
    const void *rows[kGramRows];  // DEVICE pointers; NULL rows read as zero
    size_t P;
    double *ws;                   // [kGramBlocks][3][kGramTile] per-workgroup tiles
    int do_aa, do_ab, do_bb;      // which tiles this launch computes
    int use_b;                    // group B present
};

// 16 consecutive elements of one row, widened, as four float4. p is a multiple of 16.
__device__ __forceinline__ void load16(const float *row, size_t p, float4 (&v)[4])
{
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = *reinterpret_cast<const float4 *>(row + p + 4 * j);
}
__device__ __forceinline__ void load16(const bf16_t *row, size_t p, float4 (&v)[4])
{
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const uint4 r = *reinterpret_cast<const uint4 *>(row + p + 8 * j);
        v[2 * j] = make_float4(__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xffff0000u),
                               __uint_as_float(r.y << 16), __uint_as_float(r.y & 0xffff0000u));
        v[2 * j + 1] = make_float4(__uint_as_float(r.z << 16), __uint_as_float(r.z & 0xffff0000u),
                                   __uint_as_float(r.w << 16), __uint_as_float(r.w & 0xffff0000u));
    }
}
template <typename T>
__device__ __forceinline__ void load16_guarded(const T *row, size_t p, size_t P, float4 (&v)[4])
{
    float e[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) e[k] = (p + k < P) ? load1(row, p + k) : 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = make_float4(e[4 * j], e[4 * j + 1], e[4 * j + 2], e[4 * j + 3]);
}

__device__ __forceinline__ void mfma16(const float4 (&x)[4], const float4 (&y)[4], floatx16 &acc)
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(x[j].x, y[j].x, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(x[j].y, y[j].y, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(x[j].z, y[j].z, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(x[j].w, y[j].w, acc, 0, 0, 0);
    }
}

template <typename T>
__global__ __launch_bounds__(kBlock) void gram_kernel(GramArgs a)
{
    __shared__ double tile_lds[3 * kGramTile];     // 24 KB: cross-wavefront combine

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 31, h = lane >> 5;

    // this lane's row of each group, picked with compile-time indices so the
    // pointer table stays in the kernel-argument segment
    const T *row_a = nullptr, *row_b = nullptr;
#pragma unroll
    for (int k = 0; k < 32; ++k) {
        if (r == k) {
            row_a = static_cast<const T *>(a.rows[k]);
            row_b = static_cast<const T *>(a.rows[32 + k]);
        }
    }
    const bool use_b = a.use_b != 0;

    const size_t P = a.P;
    const size_t nsteps = (P + kGramStep - 1) / kGramStep;
    const size_t nwaves = size_t(gridDim.x) * kWaves;
    const size_t gw = size_t(blockIdx.x) * kWaves + wave;

    floatx16 acc_aa = {0}, acc_ab = {0}, acc_bb = {0};
    double tot_aa[16], tot_ab[16], tot_bb[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) tot_aa[v] = tot_ab[v] = tot_bb[v] = 0.0;

    int since_flush = 0;
    for (size_t s = gw; s < nsteps; s += nwaves) {
        const size_t p = s * kGramStep + size_t(h) * 16;
        float4 xa[4], xb[4];
        const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int j = 0; j < 4; ++j) xa[j] = xb[j] = zero4;
        if ((s + 1) * kGramStep <= P) {
            if (row_a) load16(row_a, p, xa);
            if (use_b && row_b) load16(row_b, p, xb);
        } else {
            if (row_a) load16_guarded(row_a, p, P, xa);
            if (use_b && row_b) load16_guarded(row_b, p, P, xb);
        }
        if (a.do_aa) mfma16(xa, xa, acc_aa);
        if (a.do_ab) mfma16(xa, xb, acc_ab);
        if (a.do_bb) mfma16(xb, xb, acc_bb);
        if (++since_flush == kGramFlush) {
            since_flush = 0;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                tot_aa[v] += (double)acc_aa[v];
                tot_ab[v] += (double)acc_ab[v];
                tot_bb[v] += (double)acc_bb[v];
                acc_aa[v] = acc_ab[v] = acc_bb[v] = 0.f;
            }
        }
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        tot_aa[v] += (double)acc_aa[v];
        tot_ab[v] += (double)acc_ab[v];
        tot_bb[v] += (double)acc_bb[v];
    }

    // Tile entry held in accumulator register v of lane l: row i = 8*(v/4) + 4*(l/32) + v%4,
    // column j = l%32. Wavefronts add their tiles into LDS one after the other.
    for (int w = 0; w < kWaves; ++w) {
        if (wave == w) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int i = 8 * (v / 4) + 4 * h + (v % 4);
                const int e = i * 32 + r;
                if (w == 0) {
                    tile_lds[0 * kGramTile + e] = tot_aa[v];
                    tile_lds[1 * kGramTile + e] = tot_ab[v];
                    tile_lds[2 * kGramTile + e] = tot_bb[v];
                } else {
                    tile_lds[0 * kGramTile + e] += tot_aa[v];
                    tile_lds[1 * kGramTile + e] += tot_ab[v];
                    tile_lds[2 * kGramTile + e] += tot_bb[v];
                }
            }
        }
        __syncthreads();
    }
    double *out = a.ws + size_t(blockIdx.x) * 3 * kGramTile;
    for (int e = threadIdx.x; e < 3 * kGramTile; e += kBlock) out[e] = tile_lds[e];
}

// Adds the per-workgroup tiles in workgroup order and scatters the three tiles
// into the full symmetric matrix of inner products (binary64, ld = N).
struct GramFinalArgs {
    const double *ws;
    int nblocks;
    double *gram;   // [N][N]
    int N;
    int row_a, row_b;   // first global row of group A / group B
    int do_aa, do_ab, do_bb;
};

__global__ __launch_bounds__(kBlock) void gram_finalize_kernel(GramFinalArgs a)
{
    const int e = blockIdx.x * kBlock + threadIdx.x;   // 0 .. 3*1024-1
    if (e >= 3 * kGramTile) return;
    const int tile = e / kGramTile, i = (e % kGramTile) / 32, j = e % 32;
    if ((tile == 0 && !a.do_aa) || (tile == 1 && !a.do_ab) || (tile == 2 && !a.do_bb)) return;
    double s = 0.0;
    for (int b = 0; b < a.nblocks; ++b) s += a.ws[size_t(b) * 3 * kGramTile + e];
    const int gi = (tile == 2 ? a.row_b : a.row_a) + i;
    const int gj = (tile == 0 ? a.row_a : a.row_b) + j;
    if (gi >= a.N || gj >= a.N) return;
    a.gram[size_t(gi) * a.N + gj] = s;
    if (tile == 1) a.gram[size_t(gj) * a.N + gi] = s;
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
