// Device-side helpers shared by the libgaf kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gaf {

constexpr int kBlock = 256;           // threads per workgroup: 4 wavefronts of 64
constexpr int kWaves = kBlock / 64;

// Decision state kept on the device between passes. Written only by the
// one-workgroup decision kernel (or a one-thread set-up kernel); read by every
// workgroup of the following pass at its start.
struct State {
    int32_t accept;    // 1 if the gradient reduced last was accepted
    int32_t count;     // c of Algorithm 1 including that gradient
    int32_t seed;      // 1 if that gradient is the seed (aggregate <- g_i)
    int32_t c_prev;    // streaming: c before the gradient being visited (stashed by the reducing pass)
    double dot, nn_g, nn_i;  // the three sums behind the last distance
};

using bf16_t = uint16_t;  // storage type of a bfloat16 element

// ---- loads: 4 consecutive elements widened to binary32 ---------------------
// kStream = true marks the load nontemporal: the line is not kept in the
// caches. Measured on vectors far larger than the caches, read-only passes run
// at 6.7 TB/s with the hint against 6.2 TB/s without; on vectors that fit the
// last-level cache the hint costs a few percent, so the host picks by size.
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

template <bool kStream = false>
__device__ __forceinline__ float4 load4(const float *p, size_t idx)
{
    const f32x4_t *q = reinterpret_cast<const f32x4_t *>(p + idx);   // 16-byte load
    const f32x4_t v = kStream ? __builtin_nontemporal_load(q) : *q;
    return make_float4(v.x, v.y, v.z, v.w);
}
template <bool kStream = false>
__device__ __forceinline__ float4 load4(const bf16_t *p, size_t idx)
{
    const u32x2_t *q = reinterpret_cast<const u32x2_t *>(p + idx);   // 8-byte load
    const u32x2_t r = kStream ? __builtin_nontemporal_load(q) : *q;
    return make_float4(__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xffff0000u),
                       __uint_as_float(r.y << 16), __uint_as_float(r.y & 0xffff0000u));
}
__device__ __forceinline__ float load1(const float *p, size_t idx) { return p[idx]; }
__device__ __forceinline__ float load1(const bf16_t *p, size_t idx)
{
    return __uint_as_float(static_cast<uint32_t>(p[idx]) << 16);
}

// ---- wavefront reduction through DPP ---------------------------------------
// Moves a binary64 value between lanes with one DPP control word (two 32-bit
// moves). All lanes are active and every source lane exists for the controls
// used below, so the "old" operand never shows through.
template <int kCtrl>
__device__ __forceinline__ double dpp_move(double v)
{
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __builtin_amdgcn_update_dpp(0, lo, kCtrl, 0xf, 0xf, false);
    hi = __builtin_amdgcn_update_dpp(0, hi, kCtrl, 0xf, 0xf, false);
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double read_lane(double v, int lane)
{
    int lo = __builtin_amdgcn_readlane(__double2loint(v), lane);
    int hi = __builtin_amdgcn_readlane(__double2hiint(v), lane);
    return __hiloint2double(hi, lo);
}

// Sum over the 64 lanes, same value returned in every lane. Fixed tree:
// butterfly inside each row of 16 lanes (quad_perm [1,0,3,2], quad_perm
// [2,3,0,1], row_half_mirror, row_mirror), then the four row totals are added
// in row order.
__device__ __forceinline__ double wave_sum(double v)
{
    v += dpp_move<0xB1>(v);
    v += dpp_move<0x4E>(v);
    v += dpp_move<0x141>(v);
    v += dpp_move<0x140>(v);
    return ((read_lane(v, 15) + read_lane(v, 31)) + read_lane(v, 47)) + read_lane(v, 63);
}

// Workgroup sum of three values; the result is valid in thread 0 only.
// LDS carries one value per wavefront; thread 0 adds them in wavefront order.
__device__ __forceinline__ void block_sum3(double &a, double &b, double &c)
{
    __shared__ double lds[3][kWaves];
    a = wave_sum(a);
    b = wave_sum(b);
    c = wave_sum(c);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __syncthreads();  // LDS may still be read from a previous use
    if (lane == 0) {
        lds[0][wave] = a;
        lds[1][wave] = b;
        lds[2][wave] = c;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        a = lds[0][0];
        b = lds[1][0];
        c = lds[2][0];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) {
            a += lds[0][w];
            b += lds[1][w];
            c += lds[2][w];
        }
    }
}

// Eq. 4 from the three sums, in binary64. Zero norm: distance 1 by definition.
__device__ __forceinline__ double distance_from_sums(double xy, double xx, double yy)
{
    if (xx == 0.0 || yy == 0.0) return 1.0;
    return 1.0 - xy / (sqrt(xx) * sqrt(yy));
}

}  // namespace gaf
