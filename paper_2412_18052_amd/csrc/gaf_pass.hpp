// Streaming passes of the GAF filter (Algorithm 1's inner loop, Eq. 4, Eq. 5).
//
// One pass walks the P-long vectors once. Per element it (optionally) forms the
// new value m of the running mean, (optionally) stores it, and (optionally)
// accumulates the three sums of Eq. 4 against the next gradient n:
//     dot += m*n,  nn_g += m*m,  nn_i += n*n            (binary64 accumulators)
// Each workgroup leaves its three partial sums in device memory; a one-workgroup
// kernel launched right behind adds them in index order, forms the distance,
// compares it with tau and leaves the decision in device memory for the
// following pass. Nothing returns to the host. (Electing the last workgroup
// with a ticket inside the reducing kernel was measured first: the device-scope
// fences it needs cost about 75 ns per workgroup, serialised -- 100 us per pass
// at 1370 workgroups -- against about 3 us for the extra launch.)
#pragma once
#include "gaf_device.hpp"

namespace gaf {

constexpr int kUnroll = 4;                                  // 16-byte units per thread per tile
constexpr size_t kTile = size_t(kBlock) * kUnroll * 4;      // elements per workgroup per tile
constexpr int kMaxBlocks = 2048;                            // partial-sum slots per sum

// How the running mean m is obtained for an element.
enum Mode {
    kKeep = 0,     // m = aggregate as stored; nothing is written
    kUpdate = 1,   // m = a + (g - a) / c with g = the pending accepted gradient; written
    kAdopt = 2     // m = g widened (g is the seed); written
};

struct PassArgs {
    const float *acc;        // aggregate as stored (kKeep, kUpdate)
    const void *pend;        // pending gradient: accepted-but-not-yet-applied (kUpdate) or seed (kAdopt)
    const void *next;        // gradient to take the distance to (reducing passes)
    float *dst;              // where m is stored (kUpdate, kAdopt); may equal acc
    size_t P;
    State *st;
    double *partials;        // [3][kMaxBlocks]
    const int32_t *count_in; // c before this gradient; NULL means 1
    float tau;
    float *cos_out;          // D for `next` (nullable)
    uint8_t *mask_out;       // decision for `next` (nullable)
    int32_t *count_out;      // receives c (nullable)
    int seed_outputs;        // also write cos_out[-1] = 0, mask_out[-1] = 1 (first pass of a batch)
};

template <typename T, int kMode, bool kReduce>
__device__ __forceinline__ void element(float a, float g, float n, float inv_c, float &m,
                                        double &dot, double &nn_g, double &nn_i)
{
    if (kMode == kKeep) m = a;
    else if (kMode == kUpdate) m = __builtin_fmaf(g - a, inv_c, a);
    else m = g;
    if (kReduce) {
        const double md = (double)m, nd = (double)n;
        dot = __builtin_fma(md, nd, dot);
        nn_g = __builtin_fma(md, md, nn_g);
        nn_i = __builtin_fma(nd, nd, nn_i);
    }
}

// The walk over the vectors, shared by all passes. Tiles are handed to
// workgroups round-robin so that the workgroups running at any moment read one
// contiguous window of memory.
template <typename T, int kMode, bool kReduce, bool kStream>
__device__ __forceinline__ void walk(const PassArgs &a, float inv_c, double &dot, double &nn_g,
                                     double &nn_i)
{
    const float *acc = a.acc;
    const T *pend = static_cast<const T *>(a.pend);
    const T *next = static_cast<const T *>(a.next);
    float *dst = a.dst;
    const size_t P = a.P;
    const size_t ntiles = (P + kTile - 1) / kTile;
    const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);

    for (size_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const size_t base = t * kTile + size_t(threadIdx.x) * 4;
        if ((t + 1) * kTile <= P) {
            float4 va[kUnroll], vg[kUnroll], vn[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const size_t idx = base + size_t(u) * kBlock * 4;
                va[u] = (kMode != kAdopt) ? load4(acc, idx) : zero4;
                vg[u] = (kMode != kKeep) ? load4<kStream>(pend, idx) : zero4;
                vn[u] = kReduce ? load4<kStream>(next, idx) : zero4;
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const size_t idx = base + size_t(u) * kBlock * 4;
                float4 m;
                element<T, kMode, kReduce>(va[u].x, vg[u].x, vn[u].x, inv_c, m.x, dot, nn_g, nn_i);
                element<T, kMode, kReduce>(va[u].y, vg[u].y, vn[u].y, inv_c, m.y, dot, nn_g, nn_i);
                element<T, kMode, kReduce>(va[u].z, vg[u].z, vn[u].z, inv_c, m.z, dot, nn_g, nn_i);
                element<T, kMode, kReduce>(va[u].w, vg[u].w, vn[u].w, inv_c, m.w, dot, nn_g, nn_i);
                if (kMode != kKeep) *reinterpret_cast<float4 *>(dst + idx) = m;
            }
        } else {
            // ragged last tile: whole 4-element units while they fit, then single elements
#pragma unroll 1
            for (int u = 0; u < kUnroll; ++u) {
                const size_t idx = base + size_t(u) * kBlock * 4;
                if (idx + 4 <= P) {
                    const float4 va = (kMode != kAdopt) ? load4(acc, idx) : zero4;
                    const float4 vg = (kMode != kKeep) ? load4(pend, idx) : zero4;
                    const float4 vn = kReduce ? load4(next, idx) : zero4;
                    float4 m;
                    element<T, kMode, kReduce>(va.x, vg.x, vn.x, inv_c, m.x, dot, nn_g, nn_i);
                    element<T, kMode, kReduce>(va.y, vg.y, vn.y, inv_c, m.y, dot, nn_g, nn_i);
                    element<T, kMode, kReduce>(va.z, vg.z, vn.z, inv_c, m.z, dot, nn_g, nn_i);
                    element<T, kMode, kReduce>(va.w, vg.w, vn.w, inv_c, m.w, dot, nn_g, nn_i);
                    if (kMode != kKeep) *reinterpret_cast<float4 *>(dst + idx) = m;
                } else {
                    for (size_t e = idx; e < P; ++e) {
                        const float va = (kMode != kAdopt) ? acc[e] : 0.f;
                        const float vg = (kMode != kKeep) ? load1(pend, e) : 0.f;
                        const float vn = kReduce ? load1(next, e) : 0.f;
                        float m;
                        element<T, kMode, kReduce>(va, vg, vn, inv_c, m, dot, nn_g, nn_i);
                        if (kMode != kKeep) dst[e] = m;
                    }
                }
            }
        }
    }
}

// Leaves this workgroup's sums in its slot of the partial-sum table.
__device__ __forceinline__ void publish_partials(const PassArgs &a, double dot, double nn_g,
                                                 double nn_i)
{
    block_sum3(dot, nn_g, nn_i);
    if (threadIdx.x == 0) {
        a.partials[0 * kMaxBlocks + blockIdx.x] = dot;
        a.partials[1 * kMaxBlocks + blockIdx.x] = nn_g;
        a.partials[2 * kMaxBlocks + blockIdx.x] = nn_i;
    }
}

// One workgroup: adds the nb partial sums of the reducing pass that has just
// finished in index order (strided per thread, then the fixed wavefront and
// workgroup trees), forms the distance of Eq. 4 and takes the decision of
// Algorithm 1 (accept iff D <= tau; NaN compares false). No floating-point
// atomics anywhere, so the result does not depend on scheduling.
// Streaming use: *count_in == 0 means the gradient is the seed and no reduction
// was run for it.
__global__ __launch_bounds__(kBlock) void decide_kernel(PassArgs a, int nb)
{
    const int32_t c_prev = a.count_in ? *a.count_in : 1;
    State *st = a.st;
    if (c_prev == 0) {
        if (threadIdx.x == 0) {
            st->accept = 1;
            st->count = 1;
            st->seed = 1;
            if (a.cos_out) a.cos_out[0] = 0.f;
            if (a.mask_out) a.mask_out[0] = 1;
            if (a.count_out) a.count_out[0] = 1;
        }
        return;
    }
    double s0 = 0.0, s1 = 0.0, s2 = 0.0;
    for (int b = threadIdx.x; b < nb; b += kBlock) {
        s0 += a.partials[0 * kMaxBlocks + b];
        s1 += a.partials[1 * kMaxBlocks + b];
        s2 += a.partials[2 * kMaxBlocks + b];
    }
    block_sum3(s0, s1, s2);
    if (threadIdx.x == 0) {
        const double D = distance_from_sums(s0, s1, s2);
        const int accept = (D <= (double)a.tau) ? 1 : 0;   // false for NaN
        st->accept = accept;
        st->count = c_prev + accept;
        st->seed = 0;
        st->dot = s0;
        st->nn_g = s1;
        st->nn_i = s2;
        if (a.cos_out) a.cos_out[0] = (float)D;
        if (a.mask_out) a.mask_out[0] = (uint8_t)accept;
        if (a.count_out) a.count_out[0] = c_prev + accept;
        if (a.seed_outputs) {
            a.cos_out[-1] = 0.f;
            a.mask_out[-1] = 1;
        }
    }
}

// In all pass kernels kStream selects nontemporal loads for the gradient
// streams (the aggregate itself is always loaded normally: it is about to be
// rewritten or re-read).
//
// First pass of a batch: the seed g_1 becomes the aggregate (stored widened to
// binary32) while the sums for g_2 are taken in the same walk.
template <typename T, bool kStream>
__global__ __launch_bounds__(kBlock) void seed_reduce_kernel(PassArgs a)
{
    double dot = 0.0, nn_g = 0.0, nn_i = 0.0;
    walk<T, kAdopt, true, kStream>(a, 0.f, dot, nn_g, nn_i);
    publish_partials(a, dot, nn_g, nn_i);
}

// Reducing pass. If a pending accepted gradient exists (a.pend non-null and the
// previous decision was "accept") its running-mean update is applied and stored
// on the way; the sums are taken on the updated aggregate.
// Streaming use passes count_in = the caller's counter: zero there means the
// incoming gradient is the seed, so there is nothing to compare it with.
template <typename T, bool kStream>
__global__ __launch_bounds__(kBlock) void reduce_kernel(PassArgs a)
{
    const int32_t c_prev = a.count_in ? *a.count_in : 1;
    // streaming: the caller's counter is rewritten by the pass that follows, so that pass reads it from here
    if (blockIdx.x == 0 && threadIdx.x == 0) a.st->c_prev = c_prev;
    if (c_prev == 0) return;   // seed: nothing to compare with
    const bool apply = (a.pend != nullptr) && (a.st->accept != 0);
    double dot = 0.0, nn_g = 0.0, nn_i = 0.0;
    if (apply)
        walk<T, kUpdate, true, kStream>(a, 1.0f / (float)c_prev, dot, nn_g, nn_i);
    else
        walk<T, kKeep, true, kStream>(a, 0.f, dot, nn_g, nn_i);
    publish_partials(a, dot, nn_g, nn_i);
}

// Streaming with one step of look-ahead: the visit of g_i first applies what the previous visit
// decided about ITS gradient (a.pend; the decision is in the device state: rejected, accepted, or
// accepted as the seed) and takes the sums for g_i on the aggregate as it then stands -- one walk
// instead of an updating walk plus a reducing one. The decision about g_i itself is left pending
// in turn. a.count_in is the caller's counter: c including the pending gradient; zero there
// means g_i is the seed and there is nothing to compare it with.
template <typename T, bool kStream>
__global__ __launch_bounds__(kBlock) void step_reduce_kernel(PassArgs a)
{
    const int32_t c_prev = *a.count_in;
    if (blockIdx.x == 0 && threadIdx.x == 0) a.st->c_prev = c_prev;
    if (c_prev == 0) return;
    const bool apply = (a.pend != nullptr) && (a.st->accept != 0);
    const bool seed = apply && (a.st->seed != 0);
    double dot = 0.0, nn_g = 0.0, nn_i = 0.0;
    if (seed)
        walk<T, kAdopt, true, kStream>(a, 0.f, dot, nn_g, nn_i);
    else if (apply)
        walk<T, kUpdate, true, kStream>(a, 1.0f / (float)c_prev, dot, nn_g, nn_i);
    else
        walk<T, kKeep, true, kStream>(a, 0.f, dot, nn_g, nn_i);
    publish_partials(a, dot, nn_g, nn_i);
}

// Non-reducing pass: applies the pending decision and nothing else. A rejected
// gradient costs no memory traffic (every workgroup leaves at once).
template <typename T, bool kStream>
__global__ __launch_bounds__(kBlock) void update_kernel(PassArgs a)
{
    const State *st = a.st;
    const int accept = st->accept, seed = st->seed, c = st->count;
    if (blockIdx.x == 0 && threadIdx.x == 0 && a.count_out) a.count_out[0] = c;
    if (!accept) return;
    double d0 = 0.0, d1 = 0.0, d2 = 0.0;
    if (seed)
        walk<T, kAdopt, false, kStream>(a, 0.f, d0, d1, d2);
    else
        walk<T, kUpdate, false, kStream>(a, 1.0f / (float)c, d0, d1, d2);
}

// Streaming: decision and update in ONE launch. Every workgroup re-derives the
// decision from the nb partial sums of the reducing pass (same fixed summation
// order everywhere, so all workgroups agree bit for bit), then rejected
// gradients cost nothing more and accepted ones are folded in. Workgroup 0 also
// publishes distance, mask, count and state. Saves the separate decision launch,
// which is worth ~15 % of a streaming visit at P = 11 M. The reducing pass is
// launched with at most kStepBlocks workgroups so that the redundant re-reduction
// stays a few MB of L2 reads in total.
constexpr int kStepBlocks = 512;

template <typename T, bool kStream>
__global__ __launch_bounds__(kBlock) void decide_update_kernel(PassArgs a, int nb)
{
    __shared__ int s_accept;
    State *st = a.st;
    const int32_t c_prev = st->c_prev;
    const bool seed = c_prev == 0;
    double s0 = 0.0, s1 = 0.0, s2 = 0.0;
    if (!seed) {
        for (int b = threadIdx.x; b < nb; b += kBlock) {
            s0 += a.partials[0 * kMaxBlocks + b];
            s1 += a.partials[1 * kMaxBlocks + b];
            s2 += a.partials[2 * kMaxBlocks + b];
        }
        block_sum3(s0, s1, s2);
    }
    if (threadIdx.x == 0) {
        const double D = seed ? 0.0 : distance_from_sums(s0, s1, s2);
        const int accept = seed ? 1 : ((D <= (double)a.tau) ? 1 : 0);   // false for NaN
        s_accept = accept;
        if (blockIdx.x == 0) {
            st->accept = accept;
            st->count = c_prev + accept;
            st->seed = seed ? 1 : 0;
            st->dot = s0;
            st->nn_g = s1;
            st->nn_i = s2;
            if (a.cos_out) a.cos_out[0] = (float)D;
            if (a.mask_out) a.mask_out[0] = (uint8_t)accept;
            if (a.count_out) a.count_out[0] = c_prev + accept;
        }
    }
    __syncthreads();
    if (!s_accept) return;
    double d0 = 0.0, d1 = 0.0, d2 = 0.0;
    if (seed)
        walk<T, kAdopt, false, kStream>(a, 0.f, d0, d1, d2);
    else
        walk<T, kUpdate, false, kStream>(a, 1.0f / (float)(c_prev + 1), d0, d1, d2);
}

// One-thread set-up for a batch of a single gradient (N == 1): the seed is the result.
__global__ void init_single_kernel(State *st, float *cos_out, uint8_t *mask_out)
{
    st->accept = 1;
    st->count = 1;
    st->seed = 1;
    cos_out[0] = 0.f;
    mask_out[0] = 1;
}

}  // namespace gaf
