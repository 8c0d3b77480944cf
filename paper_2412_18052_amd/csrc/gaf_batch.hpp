// Gram-first schedule of the batch aggregation.
//
// The decisions of Algorithm 1 depend on the gradients only through inner
// products. With A the set accepted before g_i is visited and G_jk = g_j . g_k:
//     g_i . sum_A g_j = sum_{j in A} G_ij,   |sum_A g_j|^2 = sum_{j,k in A} G_jk,
//     |g_i|^2 = G_ii,
// so Eq. 4 for every visit, and hence the whole accept mask, follows from the
// N x N Gram matrix. The batch then costs one read of every gradient (Gram
// kernel), an O(N^2) scalar scan (filter_kernel below), and one read of the
// accepted gradients plus one write of the result (mean_kernel, Eq. 5) --
// instead of one read of the aggregate per visit and a rewrite per acceptance.
// Same mask, distances and macro-gradient as the sequential schedule up to
// rounding. For batches of up to 8 gradients the inner products are binary64 sums
// of exact products; for larger ones they come from the matrix cores (binary32
// sums over at most 8 stages, then binary64: about 1e-7 relative at worst).
//
// The second read of the accepted gradients is only needed because the accept
// set is unknown while the Gram pass has the data on chip. Where it pays, the
// set is therefore guessed beforehand (from a sample of the vectors, or from
// the previous call), the Gram pass writes the mean of the guess as it goes
// (kMean variants), the filter launch on the full matrix verifies the guess
// and keeps a record of hits and misses, and the mean kernel only runs when
// the guess was wrong or not used: see Prediction, filter_kernel, mean_kernel.
// Whatever is guessed, the results are those of the two-pass form bit for bit.
#pragma once
#include "gaf_device.hpp"
#include "gaf_gram.hpp"
#include "gaf_pass.hpp"

namespace gaf {

constexpr int kBatchMaxN = 64;   // gradients the Gram-first schedule handles (one Gram launch)

// One wavefront. Visits the gradients in ring order behind the seed
// (seed, seed+1, .., N-1, 0, .., seed-1; seed = 0 is the plain array order)
// exactly as Algorithm 1 does, with the three sums of Eq. 4 taken from the
// Gram matrix. Lane k carries the k-th accepted index; the dot product is a
// fixed-tree wavefront sum. Outputs are indexed by gradient index.
// Runs on ONE full wavefront (all 64 lanes active). Returns c.
// *closest (optional) receives the smallest |D - tau| over the visited gradients: how close the
// run came to deciding otherwise.
// |running sum|^2 is carried as nn_g + 2 dot + nn_i. When the accepted gradients nearly cancel
// (an anti-aligned gradient admitted with tau near 2) that expression can round to a value that
// is tiny next to its terms, or negative. Below the resolution of the inner products -- 2^-40 of
// the sum of the accepted |g_j|^2 for the binary64 sums of small batches (N <= 8), 2^-18 for the
// matrix-core sums, whose tiles spend up to eight stages in binary32 -- it is rounding noise, and
// the running sum is treated as the zero vector (distance 1 by definition) rather than letting
// sqrt(< 0) or a random cosine decide about everything that follows.
__device__ __forceinline__ int run_filter(const double *gram, int N, int seed, float tau,
                                          uint8_t *mask, float *cos_dist, int32_t *accepted_list,
                                          double *closest = nullptr)
{
    const int lane = threadIdx.x & 63;
    int my_index = lane == 0 ? seed : -1;   // lane k < c holds the k-th accepted gradient
    int c = 1;
    double nn_g = gram[size_t(seed) * N + seed];   // |running sum|^2
    double nn_terms = nn_g;                        // sum of the accepted |g_j|^2
    const double cancel_eps = N <= 8 ? 0x1p-40 : 0x1p-18;
    double near = 4.0;
    if (lane == 0) {
        mask[seed] = 1;
        cos_dist[seed] = 0.f;
        accepted_list[0] = seed;
    }
    for (int k = 1; k < N; ++k) {
        const int i = seed + k < N ? seed + k : seed + k - N;
        const double term = my_index >= 0 ? gram[size_t(my_index) * N + i] : 0.0;
        const double dot = wave_sum(term);
        const double nn_i = gram[size_t(i) * N + i];
        const double D = distance_from_sums(dot, nn_g, nn_i);
        const bool accept = D <= (double)tau;      // false for NaN
        const double gap = fabs(D - (double)tau);
        if (gap != gap) near = 0.0;                // a NaN distance counts as "as close as it gets"
        else if (gap < near) near = gap;
        if (lane == 0) {
            mask[i] = accept ? 1 : 0;
            cos_dist[i] = (float)D;
        }
        if (accept) {
            if (lane == c) my_index = i;
            if (lane == 0) accepted_list[c] = i;
            nn_g = nn_g + 2.0 * dot + nn_i;
            nn_terms += nn_i;
            if (nn_g <= cancel_eps * nn_terms) nn_g = 0.0;
            ++c;
        }
    }
    if (closest) *closest = near;
    return c;
}

// A guess made from a sample is acted on only if every sampled distance kept this far from tau
// (four standard errors of a cosine estimated from 2^22 elements): in training the distances crowd
// around tau (Fig. 1), and a guess that is a coin toss costs a wasted write of the whole result.
constexpr double kSpecMargin = 2e-3;

// What a filter launch does with the context's Prediction.
enum : int { kSpecNone = 0, kSpecGuess = 1, kSpecVerify = 2, kSpecVerifyCarried = 3 };

// kSpecGuess (run on the inner products of a sample; accepted_list = pred->list): records the
// guessed accept set and decides whether this call's Gram pass writes its mean -- only if the
// guess names at least min_count gradients (below that the stand-alone mean is cheaper than
// mixing writes into the reading pass) and no backoff from an earlier wrong guess is running.
// kSpecVerify / kSpecVerifyCarried (run on the full inner products): compares the guess with the
// accept set just computed, tells the mean kernel whether the result is already in place, and
// keeps the record: a written guess that was wrong stops writing for `penalty` calls and doubles
// the penalty, a right one halves it; a call that did not write counts the backoff down. The
// carried form then stores the accept set just computed as the next call's guess. All on the
// device, so a caller whose gradients sit close to the threshold stops paying for wrong guesses
// without ever synchronising.
// The body, run by one full wavefront (threadIdx.x = lane).
__device__ __forceinline__ void filter_body(const double *gram, int N, float tau, State *st, uint8_t *mask,
                                            float *cos_dist, int32_t *count, int32_t *accepted_list, int spec,
                                            Prediction *pred, int min_count)
{
    if (spec == kSpecGuess && pred->backoff > 0) {
        // backing off: the sampling launch did not run either, there is no guess
        if (threadIdx.x == 0) {
            pred->count = 0;
            pred->write = 0;
            pred->valid = 0;
            pred->n = N;
        }
        return;
    }
    double closest = 0.0;
    const int c = run_filter(gram, N, 0, tau, mask, cos_dist, accepted_list, &closest);
    if (threadIdx.x == 0) {
        count[0] = c;
        st->count = c;
        st->accept = 0;
        st->seed = 0;
    }
    if (spec == kSpecGuess) {
        if (threadIdx.x == 0) {
            // a guess is written only if no decision of the sampled run was a close call: a
            // cosine estimated from the sample is off by about 1 / sqrt(sample size) = 5e-4
            pred->write = (c >= min_count && pred->backoff == 0 && closest >= kSpecMargin) ? 1 : 0;
            pred->valid = 0;
            pred->n = N;
        }
    } else if (spec == kSpecVerify || spec == kSpecVerifyCarried) {
        if (threadIdx.x == 0) {      // the thread that wrote accepted_list above
            const bool carried = spec == kSpecVerifyCarried;
            const bool wrote = carried ? carried_guess_writes(pred, N, min_count) : pred->write != 0;
            bool same = pred->count == c;
            for (int k = 0; same && k < c; ++k) same = pred->list[k] == accepted_list[k];
            int penalty = pred->penalty < 1 ? 1 : pred->penalty;
            if (wrote) {
                if (same) {
                    penalty = penalty > 1 ? penalty / 2 : 1;
                } else {
                    pred->backoff = penalty;
                    penalty = 2 * penalty < kSpecMaxPenalty ? 2 * penalty : kSpecMaxPenalty;
                }
            } else if (pred->backoff > 0) {
                pred->backoff -= 1;
            }
            pred->penalty = penalty;
            pred->write = wrote ? 1 : 0;
            pred->valid = (wrote && same) ? 1 : 0;
            if (pred->notify)
                __hip_atomic_store(pred->notify, pred->valid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            pred->next_tile = 0;             // tile counter of the mean launch that follows
            if (carried) {
                pred->n = N;
                pred->count = c;
                for (int k = 0; k < c; ++k) pred->list[k] = accepted_list[k];
            }
        }
    }
}

__global__ __launch_bounds__(64) void filter_kernel(const double *gram, int N, float tau, State *st,
                                                    uint8_t *mask, float *cos_dist, int32_t *count,
                                                    int32_t *accepted_list, int spec = kSpecNone,
                                                    Prediction *pred = nullptr, int min_count = 0)
{
    filter_body(gram, N, tau, st, mask, cos_dist, count, accepted_list, spec, pred, min_count);
}

// Forgets the record of earlier guesses (a fresh context, or the schedule was set anew).
__global__ void prediction_reset_kernel(Prediction *pred)
{
    pred->count = 0;
    pred->n = 0;
    pred->write = 0;
    pred->valid = 0;
    pred->backoff = 0;
    pred->penalty = 1;
}

// Order-indifferent variant (Sec. 3.1, last paragraph): workgroup s replays the
// filter with g_s as the seed and the others in ring order behind it, all from
// the same Gram matrix; results go to per-seed rows of a workspace.
struct SeedWs {
    uint8_t mask[kBatchMaxN][kBatchMaxN];
    float dist[kBatchMaxN][kBatchMaxN];
    int32_t list[kBatchMaxN][kBatchMaxN];
    int32_t count[kBatchMaxN];
};

__global__ __launch_bounds__(64) void seed_runs_kernel(const double *gram, int N, float tau, SeedWs *ws)
{
    const int s = blockIdx.x;
    const int c = run_filter(gram, N, s, tau, ws->mask[s], ws->dist[s], ws->list[s]);
    if (threadIdx.x == 0) ws->count[s] = c;
}

// Keeps the run with the most accepted gradients (ties: the lowest seed index).
__global__ __launch_bounds__(64) void seed_select_kernel(const SeedWs *ws, int N, State *st, uint8_t *mask,
                                                         float *cos_dist, int32_t *count, int32_t *seed_out,
                                                         int32_t *accepted_list)
{
    int best = 0;
    for (int s = 1; s < N; ++s)
        if (ws->count[s] > ws->count[best]) best = s;
    const int i = threadIdx.x;
    if (i < N) {
        mask[i] = ws->mask[best][i];
        cos_dist[i] = ws->dist[best][i];
        accepted_list[i] = ws->list[best][i];
    }
    if (i == 0) {
        count[0] = ws->count[best];
        seed_out[0] = best;
        st->count = ws->count[best];
        st->accept = 0;
        st->seed = 0;
    }
}

// ---- small batches (N <= 8): inner products on the vector ALU in binary64 ----
// With few rows the matrix-core tiles would be mostly padding (a 16-row group
// is the smallest unit), while N (N + 1) / 2 <= 36 binary64 accumulators fit in
// registers. Products of widened binary32/bfloat16 values are exact in binary64,
// every load is a fully coalesced 16-byte (8-byte for bf16) load, and at 8 TB/s
// the FMAs need under a third of the binary64 issue rate.
constexpr int kMeanClaim = 4;            // tiles a workgroup of the mean kernel claims per counter access
constexpr int kMeanQueueBlocks = 2048;   // workgroups of a mean launch that claims its tiles
constexpr size_t kMeanQueueMinTiles = 32768;   // ... used from this many tiles up (one workgroup per tile below)
constexpr int kSmallMaxN = 8;            // (run_filter's resolution rule assumes this 8)
constexpr int kSmallMaxPairs = kSmallMaxN * (kSmallMaxN + 1) / 2;
constexpr int kSmallBlocks = 512;       // workgroups of the small-batch Gram kernel (<= kMaxBlocks)

struct SmallGramArgs {
    const void *rows[kSmallMaxN];
    size_t P;
    double *partials;     // [pairs][kMaxBlocks]
    const Prediction *pred;   // kMean only
    float *mean_out;
    int carry_n, min_count;   // kMean only: see GramArgs
    size_t chunk_stride;      // non-zero: sampling launch, see gram_small_range
};

// Units of four elements per thread per tile: four, except for five and more binary32 rows, where the loaded
// values alone would take 128 registers (bfloat16 rows are held packed, two registers per unit; with four units
// in flight 8 x 1e9 bf16 runs 6 % faster than with two: 2.70 -> 2.53 ms).
__host__ __device__ constexpr int small_gram_unroll(int n, int elem_bytes) { return n <= 4 || elem_bytes == 2 ? 4 : 2; }
__host__ __device__ constexpr size_t small_gram_tile(int n, int elem_bytes)
{
    return size_t(kBlock) * small_gram_unroll(n, elem_bytes) * 4;
}

// Inner products of all pairs of N rows over the element range [lo, hi), for the
// tiles first, first + stride, ... of that range; the workgroup's sums end up in
// out[pair] for pair = 0 .. N(N+1)/2 - 1 (row-major upper triangle), written by
// the first N(N+1)/2 threads. lo must be a multiple of 8 elements.
// kMean: the mean (Eq. 5) of the gradients a Prediction names is written to
// mean_out from the registers that already hold the loaded values (see the
// matrix-core Gram kernel for the idea); the plain filter visits in index order,
// so adding the predicted rows in index order reproduces the stand-alone mean
// kernel bit for bit.
// kHalves = 2: the workgroup is two halves of kBlock threads, each a virtual workgroup of its
// own (`first`, `out` and the tiles belong to the calling half) that share only a barrier per
// tile, which keeps the two from drifting apart (two separate workgroups on a compute unit were
// seen to finish far apart when the kernel also writes: the older one is served first).
template <typename T, int N, bool kStream, bool kMean = false, int kHalves = 1>
__device__ __forceinline__ void gram_small_range(const void *const (&rows)[kSmallMaxN], size_t lo, size_t hi,
                                                 size_t first, size_t stride, double *out, size_t out_stride,
                                                 const Prediction *pred = nullptr, float *mean_out = nullptr,
                                                 size_t chunk_stride = 0, int carry_n = 0, int min_count = 0)
{
    constexpr int NP = N * (N + 1) / 2;
    constexpr int U = small_gram_unroll(N, sizeof(T));
    constexpr size_t tile = small_gram_tile(N, sizeof(T));
    constexpr size_t kTilesPerChunk = kSampleChunk / tile;
    static_assert(kSampleChunk % tile == 0, "a sample run is a whole number of tiles");
    static_assert(kHalves == 1 || kHalves == 2, "one or two virtual workgroups per workgroup");
    __shared__ double lds_all[kHalves][NP][kWaves];
    const int half = kHalves == 1 ? 0 : int(threadIdx.x) / kBlock;
    const int tid = kHalves == 1 ? int(threadIdx.x) : int(threadIdx.x) % kBlock;
    double(*const lds)[kWaves] = lds_all[half];

    const T *row[N];
#pragma unroll
    for (int i = 0; i < N; ++i) row[i] = static_cast<const T *>(rows[i]);
    double acc[NP];
#pragma unroll
    for (int k = 0; k < NP; ++k) acc[k] = 0.0;

    bool take[N];                    // kMean: is row i in the predicted accept set (uniform)
    float inv_c = 0.f;
#pragma unroll
    for (int i = 0; i < N; ++i) take[i] = false;
    const bool write_mean =
        kMean && (carry_n ? carried_guess_writes(pred, carry_n, min_count) : pred->write != 0);
    if (kMean && write_mean) {
        const int c = pred->count;
        inv_c = 1.0f / (float)c;
        for (int k = 0; k < c; ++k) {
            const int idx = pred->list[k];
#pragma unroll
            for (int i = 0; i < N; ++i) take[i] = take[i] || idx == i;
        }
    }

    auto add = [&](const float (&x)[N]) {
        double d[N];
#pragma unroll
        for (int i = 0; i < N; ++i) d[i] = (double)x[i];
        int k = 0;
#pragma unroll
        for (int i = 0; i < N; ++i)
#pragma unroll
            for (int j = i; j < N; ++j, ++k) acc[k] = __builtin_fma(d[i], d[j], acc[k]);
    };

    const size_t ntiles = (hi - lo + tile - 1) / tile;
    // tiles first, first + stride, ...; with two halves both run the trip count of the first half
    // (it has the lower `first`), and a half without a tile left only joins the barrier
    const size_t first0 = first - size_t(half);
    const size_t n_trip = ntiles > first0 ? (ntiles - first0 + stride - 1) / stride : 0;
    for (size_t trip = 0; trip < n_trip; ++trip) {
        const size_t t = first + trip * stride;
        if (kHalves > 1) {
            __syncthreads();
            if (t >= ntiles) continue;
        }
        // sampling launch (chunk_stride != 0): [lo, hi) indexes the sample, whose run r of
        // kSampleChunk elements starts at element r * chunk_stride of the vectors
        const size_t tile_at = chunk_stride ? (t / kTilesPerChunk) * chunk_stride + (t % kTilesPerChunk) * tile
                                            : t * tile;
        const size_t base = lo + tile_at + size_t(tid) * 4;
        if (lo + (t + 1) * tile <= hi) {
            float4 v[U][N];
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int i = 0; i < N; ++i) v[u][i] = load4<kStream>(row[i], base + size_t(u) * kBlock * 4);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float x[N];
#pragma unroll
                for (int i = 0; i < N; ++i) x[i] = v[u][i].x;
                add(x);
#pragma unroll
                for (int i = 0; i < N; ++i) x[i] = v[u][i].y;
                add(x);
#pragma unroll
                for (int i = 0; i < N; ++i) x[i] = v[u][i].z;
                add(x);
#pragma unroll
                for (int i = 0; i < N; ++i) x[i] = v[u][i].w;
                add(x);
                if (kMean && write_mean) {
                    f32x4_t m = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int i = 0; i < N; ++i)
                        if (take[i]) {
                            m.x += v[u][i].x;
                            m.y += v[u][i].y;
                            m.z += v[u][i].z;
                            m.w += v[u][i].w;
                        }
                    const f32x4_t o = {m.x * inv_c, m.y * inv_c, m.z * inv_c, m.w * inv_c};
                    f32x4_t *dst = reinterpret_cast<f32x4_t *>(mean_out + base + size_t(u) * kBlock * 4);
                    if (kStream) __builtin_nontemporal_store(o, dst);
                    else *dst = o;
                }
            }
        } else {
            for (int u = 0; u < U; ++u)
                for (int e = 0; e < 4; ++e) {
                    const size_t idx = base + size_t(u) * kBlock * 4 + e;
                    if (idx >= hi) continue;
                    float x[N];
#pragma unroll
                    for (int i = 0; i < N; ++i) x[i] = load1(row[i], idx);
                    add(x);
                    if (kMean && write_mean) {
                        float m = 0.f;
#pragma unroll
                        for (int i = 0; i < N; ++i)
                            if (take[i]) m += x[i];
                        mean_out[idx] = m * inv_c;
                    }
                }
        }
    }
    // workgroup sums: DPP tree per wavefront, wavefronts added in order
    const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int k = 0; k < NP; ++k) {
        const double v = wave_sum(acc[k]);
        if (lane == 0) lds[k][wave] = v;
    }
    __syncthreads();
    if (tid < NP) {
        double v = lds[tid][0];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) v += lds[tid][w];
        out[size_t(tid) * out_stride] = v;
    }
}

template <typename T, int N, bool kStream, bool kMean = false, int kHalves = 1>
__global__ __launch_bounds__(kBlock *kHalves) void gram_small_kernel(SmallGramArgs a)
{
    // a sampling launch has nothing to do while a backoff runs: no guess will be written
    if (a.chunk_stride != 0 && a.pred->backoff > 0) return;
    // partials laid out [pair][kMaxBlocks], one column per virtual workgroup
    const size_t vblock = size_t(blockIdx.x) * kHalves + (kHalves == 1 ? 0 : threadIdx.x / kBlock);
    gram_small_range<T, N, kStream, kMean, kHalves>(a.rows, 0, a.P, vblock, size_t(gridDim.x) * kHalves,
                                                    a.partials + vblock, kMaxBlocks, a.pred, a.mean_out,
                                                    a.chunk_stride, a.carry_n, a.min_count);
}

// One workgroup per pair (i <= j): adds that pair's per-workgroup partial inner
// products (strided per thread, then the fixed wavefront and workgroup trees)
// and writes both mirror entries of the Gram matrix (leading dimension N).
// (A single workgroup doing all pairs in turn was measured at 50-70 us for 36
// pairs x 1370 partials: one memory round trip per pair, serialised.)
__global__ __launch_bounds__(kBlock) void gram_small_finalize_kernel(const double *partials, int nb, int N,
                                                                     double *gram)
{
    const int k = blockIdx.x;
    double s = 0.0, z0 = 0.0, z1 = 0.0;
    for (int b = threadIdx.x; b < nb; b += kBlock) s += partials[size_t(k) * kMaxBlocks + b];
    block_sum3(s, z0, z1);
    if (threadIdx.x == 0) {
        int i = 0, left = k;              // pair index k -> (i, j), j >= i, row-major upper triangle
        while (left >= N - i) {
            left -= N - i;
            ++i;
        }
        const int j = i + left;
        gram[i * N + j] = s;
        gram[j * N + i] = s;
    }
}

// Small batches with few partial sums (N (N + 1) / 2 * nb <= kFinalizeFilterMax): the ordered
// combine of the small-batch Gram kernel's partials and the filter replay in ONE launch of one
// workgroup -- at these sizes the launches are what a call costs (P = 1e6, N = 4: four launches of
// 5-6 us; the paper's own N = 2 at P = 11 M: 42-53 us in all). Each pair gets S threads (S = the
// largest power of two with pairs * S <= 256); thread (pair, slice) adds the partials slice,
// slice + S, ... in order, then the S slice sums are added by halving (slice k takes slice
// k + S/2, ...): a fixed tree, but not the one of gram_small_finalize_kernel -- the last bits of
// the inner products may differ between entry points that take the one route or the other. The
// matrix goes to LDS for the filter and to `gram` for whoever reads it later.
constexpr int kFinalizeFilterMax = 8192;

// The combine: red[kBlock] and g[kSmallMaxN^2] are the workgroup's LDS; `gram` (nullable) also
// receives the matrix. Ends with a barrier: g is complete for every thread.
__device__ __forceinline__ void finalize_partials(const double *partials, int nb, int N, double *red, double *g,
                                                  double *gram)
{
    const int np = N * (N + 1) / 2;
    int S = 1;
    while (2 * S * np <= kBlock) S *= 2;
    const int pair = threadIdx.x / S, slice = threadIdx.x % S;
    double s = 0.0;
    if (pair < np) {
        // eight loads in flight at a time, added in index order (one memory round trip per eight
        // values instead of one per value: this sum sits on the critical path of a 10 us call)
        const double *src = partials + size_t(pair) * kMaxBlocks;
        for (int b0 = slice; b0 < nb; b0 += 8 * S) {
            double v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = b0 + k * S < nb ? src[b0 + k * S] : 0.0;
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (b0 + k * S < nb) s += v[k];
        }
    }
    red[threadIdx.x] = s;
    for (int h = S / 2; h >= 1; h /= 2) {
        __syncthreads();
        if (pair < np && slice < h) red[threadIdx.x] += red[threadIdx.x + h];
    }
    __syncthreads();
    if (int(threadIdx.x) < np) {
        const double v = red[threadIdx.x * S];
        int i = 0, left = threadIdx.x;    // pair index -> (i, j), j >= i, row-major upper triangle
        while (left >= N - i) {
            left -= N - i;
            ++i;
        }
        const int j = i + left;
        g[i * N + j] = v;
        g[j * N + i] = v;
        if (gram) {
            gram[i * N + j] = v;
            gram[j * N + i] = v;
        }
    }
    __syncthreads();
}

__global__ __launch_bounds__(kBlock) void finalize_filter_kernel(const double *partials, int nb, double *gram,
                                                                 int N, float tau, State *st, uint8_t *mask,
                                                                 float *cos_dist, int32_t *count,
                                                                 int32_t *accepted_list, int spec,
                                                                 Prediction *pred, int min_count)
{
    __shared__ double red[kBlock];
    __shared__ double g[kSmallMaxN * kSmallMaxN];
    finalize_partials(partials, nb, N, red, g, gram);
    if (threadIdx.x < 64)
        filter_body(g, N, tau, st, mask, cos_dist, count, accepted_list, spec, pred, min_count);
}

struct MeanArgs {
    const void *rows[kBatchMaxN];   // DEVICE pointers of all N gradients
    int N;
    const int32_t *accepted_list;   // DEVICE, indices of the accepted gradients in visiting order
    const State *st;                // st->count = c
    float *out;                     // may be NULL in the fused-optimizer form
    size_t P;
    Prediction *pred;               // non-NULL: if pred->valid, `out` already holds the result (written by
                                    // the Gram pass for a guessed accept set that proved right)
    int claim_tiles;                // workgroups claim their tiles from pred->next_tile (see mean_kernel)
    // fused GAF-SGD step (kSgd): parameters and momentum buffer, in place
    float *theta, *vel;
    float lr, mu, wd;
};

// The optimizer step the experiments use (Sec. 4.1: SGD with momentum, weight
// decay as L2 term) applied to one element of the macro-gradient g (Eq. 6):
//     d = g + wd * theta;  v <- mu * v + d;  theta <- theta - lr * v
__device__ __forceinline__ void sgd_element(float g, float &theta, float &v, float lr, float mu, float wd)
{
    const float d = __builtin_fmaf(wd, theta, g);
    v = __builtin_fmaf(mu, v, d);
    theta = __builtin_fmaf(-lr, v, theta);
}

// Eq. 5: out = (sum of the accepted gradients) / c, accumulated in binary32 in
// visiting order. Reads c gradients once, writes the result once.
// kSgd: the GAF-SGD update is applied in the same pass (one read and one write
// of parameters and momentum, no separate optimizer pass); with c == 1 there is
// no consensus and parameters and optimizer state are left untouched
// (Algorithm 1's skip).
// Mean of the accepted gradients (and, with kSgd, the fused optimizer step) over
// the element range [lo, hi), tiles first, first + stride, ... of that range.
// table/list live in LDS: pointers of all gradients, indices of the accepted ones.
template <typename T, bool kStream, bool kSgd>
__device__ __forceinline__ void mean_range(const MeanArgs &a, const void *const *table, const int32_t *list,
                                           int c, size_t lo, size_t hi, size_t first, size_t stride,
                                           size_t tile_end = ~size_t(0))
{
    const float inv_c = 1.0f / (float)c;
    const size_t all_tiles = (hi - lo + kTile - 1) / kTile;
    const size_t ntiles = all_tiles < tile_end ? all_tiles : tile_end;
    float *out = a.out;
    const bool step = kSgd && c > 1;
    if (kSgd && !step && !out) return;      // skipped step, nothing else asked for

    for (size_t t = first; t < ntiles; t += stride) {
        const size_t base = lo + t * kTile + size_t(threadIdx.x) * 4;
        if (lo + (t + 1) * kTile <= hi) {
            float4 sum[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) sum[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            auto add4 = [&](const float4 (&v)[kUnroll]) {
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    sum[u].x += v[u].x;
                    sum[u].y += v[u].y;
                    sum[u].z += v[u].z;
                    sum[u].w += v[u].w;
                }
            };
            int k = 0;
            for (; k + 1 < c; k += 2) {      // two gradients' loads in flight together
                const T *g0 = static_cast<const T *>(table[list[k]]);
                const T *g1 = static_cast<const T *>(table[list[k + 1]]);
                float4 v0[kUnroll], v1[kUnroll];
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) v0[u] = load4<kStream>(g0, base + size_t(u) * kBlock * 4);
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) v1[u] = load4<kStream>(g1, base + size_t(u) * kBlock * 4);
                add4(v0);
                add4(v1);
            }
            if (k < c) {
                const T *g0 = static_cast<const T *>(table[list[k]]);
                float4 v0[kUnroll];
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) v0[u] = load4<kStream>(g0, base + size_t(u) * kBlock * 4);
                add4(v0);
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const size_t idx = base + size_t(u) * kBlock * 4;
                const f32x4_t o = {sum[u].x * inv_c, sum[u].y * inv_c, sum[u].z * inv_c, sum[u].w * inv_c};
                if (!kSgd || out) {
                    f32x4_t *dst = reinterpret_cast<f32x4_t *>(out + idx);
                    // out-of-cache sizes: the result is written once and not read back here (+5 % measured)
                    if (kStream) __builtin_nontemporal_store(o, dst);
                    else *dst = o;
                }
                if (step) {
                    f32x4_t th = *reinterpret_cast<const f32x4_t *>(a.theta + idx);
                    f32x4_t ve = *reinterpret_cast<const f32x4_t *>(a.vel + idx);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float t1 = th[e], v1 = ve[e];
                        sgd_element(o[e], t1, v1, a.lr, a.mu, a.wd);
                        th[e] = t1;
                        ve[e] = v1;
                    }
                    *reinterpret_cast<f32x4_t *>(a.theta + idx) = th;
                    *reinterpret_cast<f32x4_t *>(a.vel + idx) = ve;
                }
            }
        } else {
            // ragged last tile, element-wise
            for (int u = 0; u < kUnroll; ++u)
                for (int e = 0; e < 4; ++e) {
                    const size_t idx = base + size_t(u) * kBlock * 4 + e;
                    if (idx >= hi) continue;
                    float sum = 0.f;
                    for (int k = 0; k < c; ++k) sum += load1(static_cast<const T *>(table[list[k]]), idx);
                    const float o = sum * inv_c;
                    if (!kSgd || out) out[idx] = o;
                    if (step) sgd_element(o, a.theta[idx], a.vel[idx], a.lr, a.mu, a.wd);
                }
        }
    }
}

template <typename T, bool kStream, bool kSgd>
__global__ __launch_bounds__(kBlock) void mean_kernel(MeanArgs a)
{
    __shared__ const void *table[kBatchMaxN];
    __shared__ int32_t list[kBatchMaxN];
    const int c = a.st->count;
    if (a.pred && a.pred->valid) return;      // the fused pass already wrote exactly this mean
    if (threadIdx.x < kBatchMaxN) {
        table[threadIdx.x] = a.rows[threadIdx.x];
        list[threadIdx.x] = int(threadIdx.x) < c ? a.accepted_list[threadIdx.x] : 0;
    }
    __syncthreads();
    if (!a.claim_tiles) {
        mean_range<T, kStream, kSgd>(a, table, list, c, 0, a.P, blockIdx.x, gridDim.x);
        return;
    }
    // Long vectors after a guess: a bounded grid (a launch that finds the result in place must
    // stay cheap, and a workgroup per tile would cost 50 us just to dispatch at 1e9 elements)
    // whose workgroups claim kMeanClaim tiles at a time from a counter -- no sums cross tiles,
    // so which workgroup takes which tile does not change a bit of the result, and the
    // dispatcher-like balance is worth 10-15 % over a fixed split. The counter was cleared by
    // the filter launch that verified the guess.
    __shared__ unsigned claimed;
    const size_t ntiles = (a.P + kTile - 1) / kTile;
    for (;;) {
        if (threadIdx.x == 0) claimed = atomicAdd(&a.pred->next_tile, (unsigned)kMeanClaim);
        __syncthreads();
        const size_t t0 = claimed;
        __syncthreads();
        if (t0 >= ntiles) return;       // every workgroup gets here once the tiles run out
        mean_range<T, kStream, kSgd>(a, table, list, c, 0, a.P, t0, 1, t0 + kMeanClaim);
    }
}

// Short vectors, small batches: combine, filter and mean in ONE launch behind the Gram kernel.
// Every workgroup of the mean redoes the combine of the Gram kernel's partial sums and the
// replay of Algorithm 1 for itself (same code and summation order as finalize_filter_kernel, so
// all workgroups agree bit for bit with it and with each other), then takes its tile of Eq. 5;
// workgroup 0 also publishes matrix, mask, distances, count and state. Saves a dependent launch
// (6 to 9 us, a third of a call at P = 1e6); the host uses it only where the partial sums that
// all the workgroups re-read stay a few MB in total. With nb == 0 the matrix has been combined
// by a launch of its own and only the replay is redone per workgroup (small batches of any
// length below the guessing threshold: still one launch fewer).
struct FilterOut {
    double *gram;
    State *st;
    uint8_t *mask;
    float *cos_dist;
    int32_t *count;
    int32_t *accepted_list;
};

template <typename T, bool kStream>
__global__ __launch_bounds__(kBlock) void mean_filter_kernel(MeanArgs a, const double *partials, int nb, float tau,
                                                             FilterOut o)
{
    __shared__ double red[kBlock];
    __shared__ double g[kSmallMaxN * kSmallMaxN];
    __shared__ const void *table[kBatchMaxN];
    __shared__ int32_t list[kBatchMaxN];
    __shared__ uint8_t l_mask[kSmallMaxN];
    __shared__ float l_dist[kSmallMaxN];
    __shared__ int l_count;
    const int N = a.N;
    if (threadIdx.x < kBatchMaxN) {
        table[threadIdx.x] = a.rows[threadIdx.x];
        list[threadIdx.x] = 0;
    }
    if (nb > 0) {
        finalize_partials(partials, nb, N, red, g, blockIdx.x == 0 ? o.gram : nullptr);
    } else {                                   // the matrix is already combined: o.gram is the input
        if (int(threadIdx.x) < N * N) g[threadIdx.x] = o.gram[threadIdx.x];
        __syncthreads();
    }
    if (threadIdx.x < 64) {
        const int c = run_filter(g, N, 0, tau, l_mask, l_dist, list);
        if (threadIdx.x == 0) l_count = c;
    }
    __syncthreads();
    const int c = l_count;
    if (blockIdx.x == 0) {
        if (int(threadIdx.x) < N) {
            o.mask[threadIdx.x] = l_mask[threadIdx.x];
            o.cos_dist[threadIdx.x] = l_dist[threadIdx.x];
        }
        if (int(threadIdx.x) < c) o.accepted_list[threadIdx.x] = list[threadIdx.x];
        if (threadIdx.x == 0) {
            o.count[0] = c;
            o.st->count = c;
            o.st->accept = 0;
            o.st->seed = 0;
        }
    }
    mean_range<T, kStream, false>(a, table, list, c, 0, a.P, blockIdx.x, gridDim.x);
}

// ---- bucketed filtering in three launches (small batches) -------------------
// Bucket b covers elements [off[b], off[b+1]) and is served by workgroups
// [blk[b], blk[b+1]) of the Gram and of the mean launch; both tables travel in
// the kernel-argument segment.
constexpr int kSegMaxBuckets = 256;
constexpr int kSegMaxBlocks = 32768;     // workgroups over all buckets (size of the partial-sum table)

struct SegTable {
    unsigned long long off[kSegMaxBuckets + 1];
    int32_t blk[kSegMaxBuckets + 1];
    int B;
};

struct SegWs {                           // per-bucket outcome of the filter, read by the mean launch
    int32_t list[kSegMaxBuckets][kSmallMaxN];
    int32_t count[kSegMaxBuckets];
};

__device__ __forceinline__ int seg_bucket_of(const SegTable &tab, int wg)
{
    int lo = 0, hi = tab.B - 1;          // largest b with blk[b] <= wg
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (tab.blk[mid] <= wg) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

struct SegGramArgs {
    const void *rows[kSmallMaxN];
    SegTable tab;
    double *partials;                    // [workgroup][kSmallMaxPairs]
};

template <typename T, int N, bool kStream>
__global__ __launch_bounds__(kBlock) void gram_seg_kernel(SegGramArgs a)
{
    const int b = seg_bucket_of(a.tab, blockIdx.x);
    const int first = a.tab.blk[b], nblk = a.tab.blk[b + 1] - first;
    gram_small_range<T, N, kStream>(a.rows, a.tab.off[b], a.tab.off[b + 1], blockIdx.x - first, nblk,
                                    a.partials + size_t(blockIdx.x) * kSmallMaxPairs, 1);
}

// One workgroup per bucket: ordered sum of the bucket's partial inner products
// (thread = (pair, slice of the bucket's workgroups); slices added in order),
// then Algorithm 1 replayed on the bucket's Gram matrix by the first wavefront.
__global__ __launch_bounds__(kBlock) void seg_filter_kernel(const double *partials, SegTable tab, int N, float tau,
                                                            uint8_t *mask, float *cos_dist, int32_t *count,
                                                            SegWs *ws)
{
    __shared__ double red[kWaves][64];
    __shared__ double g[kSmallMaxN * kSmallMaxN];
    const int b = blockIdx.x;
    const int first = tab.blk[b], last = tab.blk[b + 1];
    const int np = N * (N + 1) / 2;
    const int pair = threadIdx.x & 63, slice = threadIdx.x >> 6;
    double s = 0.0;
    if (pair < np)
        for (int w = first + slice; w < last; w += kWaves) s += partials[size_t(w) * kSmallMaxPairs + pair];
    red[slice][pair] = s;
    __syncthreads();
    if (int(threadIdx.x) < np) {
        double v = red[0][pair];
#pragma unroll
        for (int k = 1; k < kWaves; ++k) v += red[k][pair];
        int i = 0, left = pair;           // pair index -> (i, j), j >= i, row-major upper triangle
        while (left >= N - i) {
            left -= N - i;
            ++i;
        }
        const int j = i + left;
        g[i * N + j] = v;
        g[j * N + i] = v;
    }
    __syncthreads();
    if (threadIdx.x < 64) {
        const int c = run_filter(g, N, 0, tau, mask + size_t(b) * N, cos_dist + size_t(b) * N, ws->list[b]);
        if (threadIdx.x == 0) {
            count[b] = c;
            ws->count[b] = c;
        }
    }
}

struct SegMeanArgs {
    MeanArgs m;                          // rows, out (P, accepted_list, st unused)
    SegTable tab;
    const SegWs *ws;
};

static_assert(sizeof(SegMeanArgs) <= 4096 && sizeof(SegGramArgs) <= 4096, "kernel arguments must fit 4 KB");

template <typename T, bool kStream>
__global__ __launch_bounds__(kBlock) void mean_seg_kernel(SegMeanArgs a)
{
    __shared__ const void *table[kBatchMaxN];
    __shared__ int32_t list[kBatchMaxN];
    const int b = seg_bucket_of(a.tab, blockIdx.x);
    const int first = a.tab.blk[b], nblk = a.tab.blk[b + 1] - first;
    const int c = a.ws->count[b];
    if (threadIdx.x < kBatchMaxN) {
        table[threadIdx.x] = a.m.rows[threadIdx.x];
        list[threadIdx.x] = int(threadIdx.x) < c ? a.ws->list[b][threadIdx.x] : 0;
    }
    __syncthreads();
    mean_range<T, kStream, false>(a.m, table, list, c, a.tab.off[b], a.tab.off[b + 1], blockIdx.x - first, nblk);
}

}  // namespace gaf
