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

// Every gradient and aggregate lives in global memory, but a pointer that reaches a kernel by
// way of a table in LDS is "generic" to the compiler, and an access through a generic pointer
// becomes a flat_ instruction: it counts against the LDS counter as well as the vector-memory
// one, so that every wait for an LDS read also waits for it and the two can no longer be
// pipelined apart. The loaders therefore say where the data is.
#define GAF_GLOBAL __attribute__((address_space(1)))
template <typename V>
__device__ __forceinline__ const GAF_GLOBAL V *as_global(const void *p)
{
    return (const GAF_GLOBAL V *)p;
}
template <typename V>
__device__ __forceinline__ GAF_GLOBAL V *as_global(void *p)
{
    return (GAF_GLOBAL V *)p;
}

template <bool kStream = false>
__device__ __forceinline__ float4 load4(const float *p, size_t idx)
{
    const GAF_GLOBAL f32x4_t *q = as_global<f32x4_t>(p + idx);   // 16-byte load
    const f32x4_t v = kStream ? __builtin_nontemporal_load(q) : *q;
    return make_float4(v.x, v.y, v.z, v.w);
}
template <bool kStream = false>
__device__ __forceinline__ float4 load4(const bf16_t *p, size_t idx)
{
    const GAF_GLOBAL u32x2_t *q = as_global<u32x2_t>(p + idx);   // 8-byte load
    const u32x2_t r = kStream ? __builtin_nontemporal_load(q) : *q;
    return make_float4(__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xffff0000u),
                       __uint_as_float(r.y << 16), __uint_as_float(r.y & 0xffff0000u));
}
__device__ __forceinline__ float load1(const float *p, size_t idx) { return p[idx]; }
__device__ __forceinline__ float load1(const bf16_t *p, size_t idx)
{
    return __uint_as_float(static_cast<uint32_t>(p[idx]) << 16);
}

// ---- write windows -----------------------------------------------------------
// A pass that mostly reads but also writes pays far more for its written bytes than a pass that
// only writes: measured on vectors of a GiB, one 1 KB store per 8 KB of loads costs 0.57 ms per
// GiB written against 0.22 ms per GiB for stores alone, wherever in the loop the store is issued,
// in bursts or not, temporal or not -- the memory turns around between reading and writing for
// every small group of writes. What does help is making the WHOLE chip write at the same time.
// The constant 100 MHz clock (s_memrealtime) reads the same in every compute unit, so it can
// serve as the conductor without any communication: time is cut into periods of `period` ticks
// whose first `win` ticks are the write window. A workgroup keeps its results on chip, writes them out
// when it finds the window open, and then idles until the window closes, so that for a few
// microseconds the memory sees (nearly) nothing but writes and for the rest of the period nothing
// but reads (measured on the same mix: 1.81 -> 1.45 ms, 6.7 TB/s in total).
// Results never depend on it: the same values go to the same addresses, only later. Waiting is
// bounded by the clock and, should the clock not move, by a spin limit.
struct WriteGate {
    unsigned period, win;    // period and window length in 10 ns ticks; win == 0: never open
    unsigned base;           // start of the period the last look at the clock fell into
    // (the low 32 bits of the clock are enough: they wrap every 43 s, which costs one odd period)
    __device__ __forceinline__ WriteGate(unsigned period_, unsigned win_) : period(period_ ? period_ : 1u), win(win_)
    {
        const unsigned t = unsigned(__builtin_amdgcn_s_memrealtime());
        base = t - t % period;          // the one division; afterwards the period is tracked by subtraction
    }
    __device__ __forceinline__ bool open()
    {
        if (win == 0) return false;
        unsigned d = unsigned(__builtin_amdgcn_s_memrealtime()) - base;
        if (d >= period) {
            const unsigned n = d >= 2 * period ? d / period : 1u;      // more than a period since the last look: rare
            base += n * period;
            d -= n * period;
        }
        return d < win;
    }
    __device__ __forceinline__ void wait_closed()
    {
        for (int spin = 0; spin < 4096 && open(); ++spin) __builtin_amdgcn_s_sleep(4);
    }
};

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
