// libgaf: host side of the C ABI declared in include/gaf.h. Validates
// arguments, sizes the launches (a fixed function of P, so results are
// reproducible) and enqueues kernels on the caller's stream. It never
// synchronises and never reads a device result.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/gaf.h"
#include "gaf_batch.hpp"
#include "gaf_gram.hpp"
#include "gaf_pass.hpp"

using namespace gaf;

struct gaf_ctx {
    int device;
    size_t max_P;
    int max_N;
    State *st;           // device
    double *partials;    // device, [3][kMaxBlocks]
    double *gram_ws;     // device, [kGramBlocks][kGramMaxTiles][kGramTile]
    double *gram_full;   // device, [max_N][max_N]
    int32_t *accepted;   // device, [max_N] indices of accepted gradients (Gram-first schedule)
    SeedWs *seed_ws;     // device, per-seed filter runs (order-indifferent variant)
    SegWs *seg_ws;       // device, per-bucket filter outcomes (bucketed filtering)
    Prediction *pred;    // device, accept set predicted from a sample (fused mean) and the record of earlier guesses
    volatile int32_t *guess_note;   // pinned host memory (null in the context that allocates nothing): whether the
                                    // last verified guess left the result in place, written by the device
    bool pred_reset;     // that record is to be cleared by the next call that guesses
    gaf_schedule schedule;
    // streaming with look-ahead: the gradient whose decision (in `st`) has not been applied yet
    const void *pend_g;
    float *pend_accum;
    int32_t *pend_count;
    size_t pend_P;
    gaf_dtype pend_dt;
    // launch timing (off unless gaf_profile_begin was called)
    bool prof_on;
    int prof_cap;
    std::vector<hipEvent_t> prof_ev;   // start/stop pairs
    std::vector<int32_t> prof_id;
};

namespace {

inline bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// Workgroups for a streaming pass over P elements: every workgroup gets the
// same number of tiles (to within one), at most kMaxBlocks workgroups.
inline int pass_blocks(size_t P, int cap = kMaxBlocks)
{
    const size_t ntiles = (P + kTile - 1) / kTile;
    const size_t iters = (ntiles + cap - 1) / cap;
    return static_cast<int>((ntiles + iters - 1) / iters);
}

// Workgroups for a pass that writes and has no sums to combine afterwards (masked mean,
// update, copy): one per tile. Measured on 1 and 4 GiB copies and 2..9-stream sums, workgroups
// that take one tile and end run 7-19 % faster than 2048 workgroups looping over the tiles
// (6.0-6.5 against 5.0-5.9 TB/s; the longer the vectors the larger the gap): the dispatcher
// evens out what a fixed split cannot. Passes that leave partial sums keep the bounded grid
// above (their summation order is tied to it).
inline int tile_blocks(size_t P)
{
    const size_t ntiles = (P + kTile - 1) / kTile;
    return static_cast<int>(ntiles < (size_t(1) << 22) ? ntiles : (size_t(1) << 22));
}

gaf_status check_ctx(const gaf_ctx *ctx)
{
    if (!ctx) return GAF_EINVAL;
    int cur = -1;
    if (hipGetDevice(&cur) != hipSuccess) return GAF_EHIP;
    if (cur != ctx->device) return GAF_EDEVICE;
    return GAF_OK;
}

inline gaf_status launched()
{
    return hipGetLastError() == hipSuccess ? GAF_OK : GAF_EHIP;
}

// Brackets one kernel launch with a pair of events when launch timing is on.
struct Timed {
    gaf_ctx *ctx;
    hipStream_t s;
    bool live;
    Timed(gaf_ctx *c, hipStream_t st, gaf_kernel_id id) : ctx(c), s(st), live(false)
    {
        // (gaf_profile_begin reserved room for prof_cap records: no allocation, nothing to throw, here)
        if (!c->prof_on || static_cast<int>(c->prof_id.size()) >= c->prof_cap) return;
        hipEvent_t a, b;
        if (hipEventCreate(&a) != hipSuccess) return;
        if (hipEventCreate(&b) != hipSuccess) {
            (void)hipEventDestroy(a);
            return;
        }
        c->prof_ev.push_back(a);
        c->prof_ev.push_back(b);
        c->prof_id.push_back(static_cast<int32_t>(id));
        (void)hipEventRecord(a, s);
        live = true;
    }
    ~Timed()
    {
        if (live) (void)hipEventRecord(ctx->prof_ev.back(), s);
    }
};

// Gradient streams are loaded nontemporally when one pass touches more than the
// last-level cache can hold (256 MiB on MI355X); below that, later passes find
// the gradients still cached and the hint would throw that away.
inline bool stream_loads(size_t P, size_t elem_bytes)
{
    return (4 + 2 * elem_bytes) * P > (size_t(256) << 20);
}

template <typename T, bool kStream>
gaf_status aggregate_impl(gaf_ctx *ctx, const void *const *grads, int N, size_t P, float tau,
                          float *out, uint8_t *mask, float *cos_dist, int32_t *count,
                          hipStream_t s)
{
    const dim3 grid(pass_blocks(P)), block(kBlock);
    PassArgs a{};
    a.P = P;
    a.st = ctx->st;
    a.partials = ctx->partials;
    a.tau = tau;
    a.dst = out;

    if (N == 1) {
        {
            Timed t(ctx, s, GAF_K_INIT);
            init_single_kernel<<<1, 1, 0, s>>>(ctx->st, cos_dist, mask);
        }
        if (launched() != GAF_OK) return GAF_EHIP;
        a.pend = grads[0];
        a.count_out = count;
        {
            Timed t(ctx, s, GAF_K_UPDATE);
            update_kernel<T, kStream><<<tile_blocks(P), block, 0, s>>>(a);
        }
        return launched();
    }

    // pass 1: adopt the seed, reduce against grads[1]
    a.pend = grads[0];
    a.next = grads[1];
    a.cos_out = cos_dist + 1;
    a.mask_out = mask + 1;
    a.count_out = count;
    a.seed_outputs = 1;
    {
        Timed t(ctx, s, GAF_K_SEED_REDUCE);
        seed_reduce_kernel<T, kStream><<<grid, block, 0, s>>>(a);
    }
    if (launched() != GAF_OK) return GAF_EHIP;
    {
        Timed t(ctx, s, GAF_K_DECIDE);
        decide_kernel<<<1, block, 0, s>>>(a, grid.x);
    }
    if (launched() != GAF_OK) return GAF_EHIP;

    // passes 2..N-1: apply the decision on grads[i-1] while reducing against grads[i]
    a.acc = out;
    a.seed_outputs = 0;
    a.count_in = &ctx->st->count;
    for (int i = 2; i < N; ++i) {
        a.pend = grads[i - 1];
        a.next = grads[i];
        a.cos_out = cos_dist + i;
        a.mask_out = mask + i;
        {
            Timed t(ctx, s, GAF_K_REDUCE);
            reduce_kernel<T, kStream><<<grid, block, 0, s>>>(a);
        }
        if (launched() != GAF_OK) return GAF_EHIP;
        {
            Timed t(ctx, s, GAF_K_DECIDE);
            decide_kernel<<<1, block, 0, s>>>(a, grid.x);
        }
        if (launched() != GAF_OK) return GAF_EHIP;
    }

    // tail: apply the decision on the last gradient (no traffic if it was rejected)
    a.pend = grads[N - 1];
    a.next = nullptr;
    a.cos_out = nullptr;
    a.mask_out = nullptr;
    a.count_out = nullptr;
    {
        Timed t(ctx, s, GAF_K_UPDATE);
        update_kernel<T, kStream><<<tile_blocks(P), block, 0, s>>>(a);
    }
    return launched();
}

// Streaming visits of vectors from this length on take three launches (reduce, decide, update)
// instead of two (reduce, decide+update).
constexpr size_t kStepSplitMinP = size_t(1) << 26;

template <typename T, bool kStream>
gaf_status step_impl(gaf_ctx *ctx, float *accum, int32_t *count, const void *g_i, size_t P,
                     float tau, float *cos_out, uint8_t *acc_out, hipStream_t s)
{
    // Long vectors: the update runs one workgroup per tile (see tile_blocks), which is worth more
    // than the decision launch it would otherwise absorb; the reducing pass then uses the full grid.
    const bool long_vector = P >= kStepSplitMinP;
    const dim3 grid(pass_blocks(P, long_vector ? kMaxBlocks : kStepBlocks)), block(kBlock);
    PassArgs a{};
    a.P = P;
    a.st = ctx->st;
    a.partials = ctx->partials;
    a.tau = tau;
    a.acc = accum;
    a.dst = accum;
    a.next = g_i;
    a.count_in = count;
    {
        Timed t(ctx, s, GAF_K_REDUCE);
        reduce_kernel<T, kStream><<<grid, block, 0, s>>>(a);
    }
    if (launched() != GAF_OK) return GAF_EHIP;
    a.cos_out = cos_out;
    a.mask_out = acc_out;
    if (long_vector) {
        {
            Timed t(ctx, s, GAF_K_DECIDE);
            decide_kernel<<<1, block, 0, s>>>(a, grid.x);     // reads *count: 0 means g_i seeds
        }
        if (launched() != GAF_OK) return GAF_EHIP;
    }
    a.pend = g_i;
    a.next = nullptr;
    a.count_in = nullptr;
    a.count_out = count;
    {
        Timed t(ctx, s, GAF_K_UPDATE);
        if (long_vector) {
            a.cos_out = nullptr;
            a.mask_out = nullptr;
            update_kernel<T, kStream><<<tile_blocks(P), block, 0, s>>>(a);
        } else {
            decide_update_kernel<T, kStream><<<grid, block, 0, s>>>(a, grid.x);
        }
    }
    return launched();
}

// Applies the update a look-ahead visit left pending (no memory traffic if that gradient was
// rejected) and forgets it.
template <typename T, bool kStream>
gaf_status flush_impl(gaf_ctx *ctx, hipStream_t s)
{
    PassArgs a{};
    a.P = ctx->pend_P;
    a.st = ctx->st;
    a.partials = ctx->partials;
    a.acc = ctx->pend_accum;
    a.dst = ctx->pend_accum;
    a.pend = ctx->pend_g;
    {
        Timed t(ctx, s, GAF_K_UPDATE);
        update_kernel<T, kStream><<<tile_blocks(a.P), kBlock, 0, s>>>(a);
    }
    return launched();
}

gaf_status flush_pending(gaf_ctx *ctx, hipStream_t s)
{
    if (!ctx->pend_g) return GAF_OK;
    const size_t P = ctx->pend_P;
    const gaf_status rc =
        ctx->pend_dt == GAF_F32
            ? (stream_loads(P, 4) ? flush_impl<float, true>(ctx, s) : flush_impl<float, false>(ctx, s))
            : (stream_loads(P, 2) ? flush_impl<bf16_t, true>(ctx, s) : flush_impl<bf16_t, false>(ctx, s));
    ctx->pend_g = nullptr;
    return rc;
}

// One visit with look-ahead: two launches (update of the pending gradient + sums for g_i in one
// walk; decision). The update for g_i stays pending.
template <typename T, bool kStream>
gaf_status step_lookahead_impl(gaf_ctx *ctx, float *accum, int32_t *count, const void *g_i, size_t P,
                               float tau, float *cos_out, uint8_t *acc_out, hipStream_t s)
{
    // the launch shape of gaf_step's reducing pass: same partial sums, same distances, bit for bit
    const dim3 grid(pass_blocks(P, P >= kStepSplitMinP ? kMaxBlocks : kStepBlocks)), block(kBlock);
    PassArgs a{};
    a.P = P;
    a.st = ctx->st;
    a.partials = ctx->partials;
    a.tau = tau;
    a.acc = accum;
    a.dst = accum;
    a.pend = ctx->pend_g;
    a.next = g_i;
    a.count_in = count;
    {
        Timed t(ctx, s, GAF_K_REDUCE);
        step_reduce_kernel<T, kStream><<<grid, block, 0, s>>>(a);
    }
    if (launched() != GAF_OK) return GAF_EHIP;
    a.cos_out = cos_out;
    a.mask_out = acc_out;
    a.count_out = count;
    {
        Timed t(ctx, s, GAF_K_DECIDE);
        decide_kernel<<<1, block, 0, s>>>(a, grid.x);     // reads *count: 0 means g_i seeds
    }
    return launched();
}

// Smallest predicted accept count for which the Gram pass writes the mean itself. Writing the
// 4 P bytes from inside the reading pass (in write windows) added 0.9 to 1.2 ms to the measured
// calls (batches of 32 GB), independent of the count c, while the stand-alone mean costs
// (c s + 4) P bytes at about 5.9 TB/s; below these break-even counts (smallest c at which the
// whole call was measured faster with the fused write, 32 GB batches) the stand-alone mean is the
// cheaper one (by at most 7% of the call).
// groups = 0 means the small-batch (N <= 8) kernel.
template <typename T>
constexpr int fused_min_count(int groups)
{
    constexpr int bf16_min[5] = {2, 2, 2, 4, 4};
    constexpr int f32_min[5] = {1, 2, 4, 4, 4};
    return sizeof(T) == 2 ? bf16_min[groups] : f32_min[groups];
}
// The same for a batch of N gradients. A guess carried over from the previous call is used on
// shorter vectors, where the small-batch kernel gains from writing even a one-gradient "mean"
// (the stand-alone pass would cost a launch and a second read of that gradient).
template <typename T>
int spec_min_count(int N, bool carried)
{
    if (N <= kSmallMaxN) return carried ? 1 : fused_min_count<T>(0);
    return fused_min_count<T>((N + 15) / 16);
}

// Enqueues the Gram kernel for up to four 16-row groups (global group indices in
// `groups`, -1 = absent) and the ordered combine of its per-workgroup tiles into
// ctx->gram_full (leading dimension N).
// With `mean_out` the launch also writes the mean of ctx->pred's accept set there (kFull only).
// With `chunk_stride` the launch reads a sample instead: P / kSampleChunk runs of kSampleChunk
// elements, run r starting at element r * chunk_stride of every gradient.
// Write windows of a pass that reads `read_bytes` and writes `write_bytes` in all (see WriteGate):
// period and window length in ticks of the 100 MHz clock. The window's share of the period is the
// share of the pass's time that the writing needs at the rates measured on MI355X (7.0 TB/s
// reading, 5.5 TB/s writing, 6.5 TB/s for the pass as a whole; on 16 x 1e9 bf16 a sweep of period
// and window put the best window at 0.136 of the period, this formula gives 0.137). A workgroup
// looks at the clock once per stage, so a window is at least 1.15 stages long; its ring holds
// `hold_stages` stages' results, so the period is 0.8 of the time those take -- unless the
// window's minimum length asks for a longer one (then results are also written when the ring is
// full: few bytes in that case).
struct GateParams {
    unsigned period, win;
};
// GAF_WRITE_WINDOWS in the environment (read once): "0" switches the windows off (results are
// then written whenever a ring is full), "PERIOD:WINDOW" in 10 ns ticks replaces the formula below;
// anything else, or nothing, leaves the formula in charge. Timing only: no result depends on it.
inline bool gate_override(GateParams &gp)
{
    static const GateParams fixed = [] {
        GateParams g{~0u, 0u};                          // period ~0: no override
        if (const char *e = std::getenv("GAF_WRITE_WINDOWS")) {
            unsigned p = 0, w = 0;
            if (std::sscanf(e, "%u:%u", &p, &w) == 2 && p > 0 && w < p) g = {p, w};
            else if (e[0] == '0' && e[1] == 0) g = {0u, 0u};
        }
        return g;
    }();
    if (fixed.period == ~0u) return false;
    gp = fixed;
    return true;
}
inline GateParams gate_params(double read_bytes, double write_bytes, double stage_bytes, int hold_stages)
{
    GateParams forced;
    if (gate_override(forced)) return forced;
    const double t_write = write_bytes / 5.5e12, t_total = read_bytes / 7.0e12 + t_write;
    const double share = t_write / t_total;
    const double stage_ticks = stage_bytes * kGramBlocks / 6.5e12 * 1e8;
    const double win_min = 1.15 * stage_ticks;
    double period = 0.8 * hold_stages * stage_ticks;                 // what the ring covers, with a margin
    if (share * period < win_min) period = win_min / share;          // ... or what the window needs
    if (period > 30000.0) period = 30000.0;
    return {(unsigned)period, (unsigned)(share * period)};
}

template <typename T, int NG, int kMode>
gaf_status gram_launch(gaf_ctx *ctx, const void *const *grads, int N, size_t P, const int (&groups)[4],
                       hipStream_t s, gaf_kernel_id id = GAF_K_GRAM, float *mean_out = nullptr,
                       size_t chunk_stride = 0, int carry_n = 0)
{
    constexpr size_t kStagesPerChunk = kSampleChunk / (size_t(256) * gram_stage_m(NG) / sizeof(T));
    static_assert(kStagesPerChunk >= 1 && (kStagesPerChunk & (kStagesPerChunk - 1)) == 0, "power of two");
    if (chunk_stride && (mean_out || P % kSampleChunk)) return GAF_EINVAL;
    typedef TileList<NG, kMode> Tiles;
    GramArgs g{};
    GramFinalArgs f{};
    for (int k = 0; k < NG; ++k) {
        for (int r = 0; r < 16; ++r) {
            const int i = groups[k] * 16 + r;
            g.rows[16 * k + r] = (groups[k] >= 0 && i < N) ? grads[i] : grads[0];   // alias: result dropped
        }
        f.group_row[k] = groups[k] >= 0 ? groups[k] * 16 : N;   // absent group: rows >= N are dropped
    }
    g.P = P;
    g.ws = ctx->gram_ws;
    g.pred = ctx->pred;
    g.out = mean_out;
    g.carry_n = carry_n;
    g.min_count = spec_min_count<T>(N, carry_n != 0);
    g.chunk_shift = 62;
    if (chunk_stride)
        for (g.chunk_shift = 0; (size_t(1) << g.chunk_shift) < kStagesPerChunk;) ++g.chunk_shift;
    g.chunk_stride = chunk_stride;
    if (mean_out) {
        const double stage_bytes = 16.0 * NG * 256 * gram_stage_m(NG);
        const GateParams gp = gate_params(double(N) * sizeof(T) * P, 4.0 * P, stage_bytes,
                                          gram_hold_stages<T>(NG));
        g.gate_period = gp.period;
        g.gate_win = gp.win;
    }
    {
        Timed t(ctx, s, id);
        if (mean_out && kMode == kFull)
            gram_kernel<T, NG, kFull, true><<<kGramBlocks, kBlock, 0, s>>>(g);
        else
            gram_kernel<T, NG, kMode><<<kGramBlocks, kBlock, 0, s>>>(g);
    }
    if (launched() != GAF_OK) return GAF_EHIP;
    f.ws = ctx->gram_ws;
    f.nblocks = kGramBlocks;
    f.ntiles = Tiles::count;
    for (int t = 0; t < Tiles::count; ++t) {
        f.tile_ga[t] = Tiles::ga(t);
        f.tile_gb[t] = Tiles::gb(t);
    }
    f.gram = ctx->gram_full;
    f.N = N;
    {
        Timed t(ctx, s, GAF_K_GRAM_FINALIZE);
        gram_finalize_kernel<<<(Tiles::count * kGramTile + 15) / 16, kBlock, 0, s>>>(f);
    }
    return launched();
}

// Inner products of all pairs into ctx->gram_full. N <= 64: one launch, every
// gradient read once. Larger N: 64-row panels, then the tiles between 32-row
// halves of different panels.
// `mean_out` (N <= 64 only): see gram_launch.
template <typename T>
gaf_status gram_all_pairs(gaf_ctx *ctx, const void *const *grads, int N, size_t P, hipStream_t s,
                          gaf_kernel_id id = GAF_K_GRAM, float *mean_out = nullptr, size_t chunk_stride = 0,
                          int carry_n = 0)
{
    const int ng = (N + 15) / 16;
    for (int g0 = 0; g0 < ng; g0 += 4) {
        const int n = ng - g0 < 4 ? ng - g0 : 4;
        const int groups[4] = {g0, n > 1 ? g0 + 1 : -1, n > 2 ? g0 + 2 : -1, n > 3 ? g0 + 3 : -1};
        gaf_status rc = GAF_OK;
        switch (n) {
        case 1: rc = gram_launch<T, 1, kFull>(ctx, grads, N, P, groups, s, id, mean_out, chunk_stride, carry_n); break;
        case 2: rc = gram_launch<T, 2, kFull>(ctx, grads, N, P, groups, s, id, mean_out, chunk_stride, carry_n); break;
        case 3: rc = gram_launch<T, 3, kFull>(ctx, grads, N, P, groups, s, id, mean_out, chunk_stride, carry_n); break;
        default: rc = gram_launch<T, 4, kFull>(ctx, grads, N, P, groups, s, id, mean_out, chunk_stride, carry_n); break;
        }
        if (rc != GAF_OK) return rc;
    }
    const int nh = (ng + 1) / 2;   // 32-row halves
    for (int ha = 0; ha < nh; ++ha)
        for (int hb = ha + 1; hb < nh; ++hb) {
            if (ha / 2 == hb / 2) continue;   // same panel: done above
            const int groups[4] = {2 * ha, 2 * ha + 1 < ng ? 2 * ha + 1 : -1, 2 * hb,
                                   2 * hb + 1 < ng ? 2 * hb + 1 : -1};
            const gaf_status rc = gram_launch<T, 4, kCross>(ctx, grads, N, P, groups, s);
            if (rc != GAF_OK) return rc;
        }
    return GAF_OK;
}

// Gram-first schedule: Gram matrix, scalar filter, masked mean. N <= kBatchMaxN.
// N <= kSmallMaxN: binary64 vector-ALU inner products into ctx->gram_full.
template <typename T, bool kStream, int N>
gaf_status gram_small_launch(const SmallGramArgs &g, int nb, hipStream_t s)
{
    // two barrier-coupled halves per workgroup where measured faster when the kernel also writes
    // the mean: binary32 rows from N = 5 up (-6 to -16 %); neutral or slower elsewhere
    constexpr int kHalves = sizeof(T) == 4 && N >= 5 ? 2 : 1;
    if (g.mean_out && nb % kHalves == 0)
        gram_small_kernel<T, N, kStream, true, kHalves><<<nb / kHalves, kBlock * kHalves, 0, s>>>(g);
    else if (g.mean_out)
        gram_small_kernel<T, N, kStream, true><<<nb, kBlock, 0, s>>>(g);
    else
        gram_small_kernel<T, N, kStream><<<nb, kBlock, 0, s>>>(g);
    return launched();
}

// With `mean_out` the launch also writes the mean of ctx->pred's accept set there.
// `merge_nb` non-null: if the partial sums are few enough for the filter launch to combine them
// itself (finalize_filter_kernel), the combine launch is left out and *merge_nb receives the
// number of workgroups whose partials are waiting; otherwise *merge_nb = 0.
template <typename T, bool kStream>
gaf_status gram_small(gaf_ctx *ctx, const void *const *grads, int N, size_t P, hipStream_t s,
                      gaf_kernel_id id = GAF_K_GRAM, float *mean_out = nullptr, size_t chunk_stride = 0,
                      int carry_n = 0, int *merge_nb = nullptr)
{
    if (chunk_stride && (mean_out || P % kSampleChunk)) return GAF_EINVAL;
    SmallGramArgs g{};
    for (int i = 0; i < kSmallMaxN; ++i) g.rows[i] = grads[i < N ? i : 0];
    g.P = P;
    g.partials = ctx->gram_ws;
    g.pred = ctx->pred;
    g.mean_out = mean_out;
    g.chunk_stride = chunk_stride;
    g.carry_n = carry_n;
    g.min_count = spec_min_count<T>(N, carry_n != 0);
    // at most two workgroups per CU: few partial sums to combine afterwards, and the widest
    // variant (N = 8) does not fit more anyway
    const int nb = pass_blocks(P) < kSmallBlocks ? pass_blocks(P) : kSmallBlocks;
    gaf_status rc = GAF_OK;
    {
        Timed t(ctx, s, id);
        switch (N) {
        case 1: rc = gram_small_launch<T, kStream, 1>(g, nb, s); break;
        case 2: rc = gram_small_launch<T, kStream, 2>(g, nb, s); break;
        case 3: rc = gram_small_launch<T, kStream, 3>(g, nb, s); break;
        case 4: rc = gram_small_launch<T, kStream, 4>(g, nb, s); break;
        case 5: rc = gram_small_launch<T, kStream, 5>(g, nb, s); break;
        case 6: rc = gram_small_launch<T, kStream, 6>(g, nb, s); break;
        case 7: rc = gram_small_launch<T, kStream, 7>(g, nb, s); break;
        default: rc = gram_small_launch<T, kStream, 8>(g, nb, s); break;
        }
    }
    if (rc != GAF_OK) return rc;
    if (merge_nb) {
        *merge_nb = (N * (N + 1) / 2) * nb <= kFinalizeFilterMax ? nb : 0;
        if (*merge_nb) return GAF_OK;
    }
    {
        Timed t(ctx, s, GAF_K_GRAM_FINALIZE);
        gram_small_finalize_kernel<<<N * (N + 1) / 2, kBlock, 0, s>>>(ctx->gram_ws, nb, N, ctx->gram_full);
    }
    return launched();
}

// Fused mean (see gram_kernel's kMean): used from this vector length up, with the accept set
// guessed from a sample of this many elements of every gradient, taken as evenly spaced runs of
// kSampleChunk elements (the parts of a model's gradient differ, so a prefix would be a poor
// sample). The guess costs N * kSpecSample elements of extra reading (under 1 % at kSpecMinP);
// a wrong guess costs one stand-alone mean pass.
constexpr size_t kSpecSample = size_t(1) << 22;
constexpr size_t kSpecMinP = size_t(1) << 26;
// Shorter vectors down to this length guess "the accept set of the previous call" instead
// (no sample: it would cost too large a share); below it the calls are launch-bound and a
// writing Gram pass gains nothing.
constexpr size_t kCarryMinP = size_t(1) << 21;
// ... and only for batches of two, the setting of the paper's own experiments, where the guess is
// "the second gradient was accepted last time (or was not)": measured on batches of 8 gradients of
// 11.2 M elements drawn independently, the exact accept set of the previous call was never this
// call's (0 of 20), so larger batches do not guess on short vectors.
constexpr int kCarryN = 2;
constexpr size_t kMergeMeanMaxBytes = size_t(8) << 20;   // partial sums re-read by all workgroups of a merged mean launch

// Distance in elements between the starts of consecutive runs of the sample for vectors of
// length P >= kSpecMinP: the runs spread over the whole vector, the last one ends inside it.
constexpr size_t spec_chunk_stride(size_t P)
{
    return P / (kSpecSample / kSampleChunk) / kSampleChunk * kSampleChunk;
}

// Variations of the Gram-first batch call.
struct BatchOptions {
    const double *gram = nullptr;   // caller's matrix of inner products: the Gram pass is skipped
    int32_t *best_seed = nullptr;   // non-null: order-indifferent variant, receives the winning seed
    float *theta = nullptr;         // non-null: fused GAF-SGD step on (theta, vel)
    float *vel = nullptr;
    float lr = 0.f, mu = 0.f, wd = 0.f;
    float *dist_matrix = nullptr;   // non-null: also write the N x N distance matrix (and gram_out if non-null)
    double *gram_out = nullptr;
};

template <typename T, bool kStream>
gaf_status aggregate_gram_impl(gaf_ctx *ctx, const void *const *grads, int N, size_t P, float tau,
                               const BatchOptions &opt, float *out, uint8_t *mask, float *cos_dist,
                               int32_t *count, hipStream_t s)
{
    const double *gram = opt.gram;
    // AUTO: the Gram pass writes the mean of a guessed accept set while it holds the data on chip,
    // and the guess is checked afterwards. Long vectors: guessed from a sample. Shorter ones:
    // the previous call's accept set.
    const bool speculate = !gram && !opt.best_seed && !opt.theta && ctx->schedule == GAF_SCHEDULE_AUTO &&
                           (P >= kSpecMinP || (P >= kCarryMinP && N == kCarryN));
    const bool carried = speculate && P < kSpecMinP;
    const bool small = N <= kSmallMaxN;
    if (speculate && ctx->pred_reset) {
        prediction_reset_kernel<<<1, 1, 0, s>>>(ctx->pred);
        if (launched() != GAF_OK) return GAF_EHIP;
        ctx->pred_reset = false;
    }
    // Small batches whose filter launch can combine the Gram kernel's partial sums itself (the
    // plain call only: the matrix and best-seed forms keep the separate combine, and with it the
    // bits of gaf_pairwise).
    const bool may_merge = small && !gram && !opt.best_seed && !opt.dist_matrix;
    int merge_nb = 0;
    if (speculate && !carried) {
        const size_t cs = spec_chunk_stride(P);
        gaf_status rc = small ? gram_small<T, false>(ctx, grads, N, kSpecSample, s, GAF_K_GRAM_SAMPLE, nullptr, cs, 0,
                                                     may_merge ? &merge_nb : nullptr)
                              : gram_all_pairs<T>(ctx, grads, N, kSpecSample, s, GAF_K_GRAM_SAMPLE, nullptr, cs);
        if (rc != GAF_OK) return rc;
        {
            Timed t(ctx, s, GAF_K_FILTER);
            if (merge_nb)
                finalize_filter_kernel<<<1, kBlock, 0, s>>>(ctx->gram_ws, merge_nb, ctx->gram_full, N, tau, ctx->st,
                                                            &ctx->seed_ws->mask[0][0], &ctx->seed_ws->dist[0][0],
                                                            &ctx->pred->count, ctx->pred->list, kSpecGuess,
                                                            ctx->pred, spec_min_count<T>(N, false));
            else
                filter_kernel<<<1, 64, 0, s>>>(ctx->gram_full, N, tau, ctx->st, &ctx->seed_ws->mask[0][0],
                                               &ctx->seed_ws->dist[0][0], &ctx->pred->count, ctx->pred->list,
                                               kSpecGuess, ctx->pred, spec_min_count<T>(N, false));
        }
        if (launched() != GAF_OK) return GAF_EHIP;
    }
    merge_nb = 0;
    if (speculate) {
        const int carry_n = carried ? N : 0;
        const gaf_status rc = small ? gram_small<T, kStream>(ctx, grads, N, P, s, GAF_K_GRAM, out, 0, carry_n,
                                                             may_merge ? &merge_nb : nullptr)
                                    : gram_all_pairs<T>(ctx, grads, N, P, s, GAF_K_GRAM, out, 0, carry_n);
        if (rc != GAF_OK) return rc;
        gram = ctx->gram_full;
    } else if (!gram) {
        const gaf_status rc = small ? gram_small<T, kStream>(ctx, grads, N, P, s, GAF_K_GRAM, nullptr, 0, 0,
                                                             may_merge ? &merge_nb : nullptr)
                                    : gram_all_pairs<T>(ctx, grads, N, P, s);
        if (rc != GAF_OK) return rc;
        gram = ctx->gram_full;
    }
    // Short vectors: the mean launch does the combine and the filter as well, every workgroup for
    // itself -- as long as what they all re-read of the Gram kernel's partial sums stays small.
    const bool merge_mean = merge_nb != 0 && !speculate && !opt.theta && out &&
                            size_t(tile_blocks(P)) * size_t(merge_nb) * (N * (N + 1) / 2) * sizeof(double) <= kMergeMeanMaxBytes;
    // ... and otherwise, for small batches, at least the filter replay (from the combined matrix)
    const bool merge_replay = !merge_mean && small && !speculate && !opt.theta && !opt.best_seed && out;
    if (opt.best_seed) {
        {
            Timed t(ctx, s, GAF_K_FILTER);
            seed_runs_kernel<<<N, 64, 0, s>>>(gram, N, tau, ctx->seed_ws);
        }
        if (launched() != GAF_OK) return GAF_EHIP;
        {
            Timed t(ctx, s, GAF_K_FILTER);
            seed_select_kernel<<<1, 64, 0, s>>>(ctx->seed_ws, N, ctx->st, mask, cos_dist, count,
                                                opt.best_seed, ctx->accepted);
        }
    } else if (merge_mean || (merge_replay && !merge_nb)) {
        // combine and filter, or the filter alone, ride in the mean launch below
    } else {
        const int spec = !speculate ? kSpecNone : carried ? kSpecVerifyCarried : kSpecVerify;
        Timed t(ctx, s, GAF_K_FILTER);
        if (merge_nb)
            finalize_filter_kernel<<<1, kBlock, 0, s>>>(ctx->gram_ws, merge_nb, ctx->gram_full, N, tau, ctx->st, mask,
                                                        cos_dist, count, ctx->accepted, spec, ctx->pred,
                                                        spec_min_count<T>(N, carried));
        else
            filter_kernel<<<1, 64, 0, s>>>(gram, N, tau, ctx->st, mask, cos_dist, count, ctx->accepted, spec,
                                           ctx->pred, spec_min_count<T>(N, carried));
    }
    if (launched() != GAF_OK) return GAF_EHIP;
    if (opt.dist_matrix) {
        Timed t(ctx, s, GAF_K_DISTANCE);
        gram_to_distance_kernel<<<(N * N + kBlock - 1) / kBlock, kBlock, 0, s>>>(gram, N, opt.dist_matrix,
                                                                                 opt.gram_out);
    }
    if (opt.dist_matrix && launched() != GAF_OK) return GAF_EHIP;
    MeanArgs m{};
    for (int i = 0; i < kBatchMaxN; ++i) m.rows[i] = grads[i < N ? i : 0];
    m.N = N;
    m.accepted_list = ctx->accepted;
    m.st = ctx->st;
    m.out = out;
    m.P = P;
    m.pred = speculate ? ctx->pred : nullptr;
    m.theta = opt.theta;
    m.vel = opt.vel;
    m.lr = opt.lr;
    m.mu = opt.mu;
    m.wd = opt.wd;
    {
        // long vectors after a guess: the launch may have nothing to do, so a bounded grid that
        // claims its tiles from a counter
        // ... unless the last guess the host has heard of did not leave the result in place (declined,
        // wrong, or backing off): then the launch will most likely have all the work to do, and one
        // workgroup per tile does that 8 % faster. The note may be a call or two old; either grid is
        // correct whatever happens.
        const bool expect_in_place = !ctx->guess_note || *ctx->guess_note != 0;
        m.claim_tiles = speculate && expect_in_place && size_t(tile_blocks(P)) >= kMeanQueueMinTiles;
        const int nb = m.claim_tiles ? kMeanQueueBlocks : tile_blocks(P);
        Timed t(ctx, s, GAF_K_MEAN);
        if (merge_mean)
            mean_filter_kernel<T, kStream><<<nb, kBlock, 0, s>>>(
                m, ctx->gram_ws, merge_nb, tau, FilterOut{ctx->gram_full, ctx->st, mask, cos_dist, count, ctx->accepted});
        else if (merge_replay && !merge_nb)
            mean_filter_kernel<T, kStream><<<nb, kBlock, 0, s>>>(
                m, nullptr, 0, tau,
                FilterOut{const_cast<double *>(gram), ctx->st, mask, cos_dist, count, ctx->accepted});
        else if (opt.theta)
            mean_kernel<T, kStream, true><<<nb, kBlock, 0, s>>>(m);
        else
            mean_kernel<T, kStream, false><<<nb, kBlock, 0, s>>>(m);
    }
    return launched();
}

template <typename T>
gaf_status pairwise_impl(gaf_ctx *ctx, const void *const *grads, int N, size_t P, float *D,
                         double *gram_out, hipStream_t s)
{
    gaf_status rc;
    if (N <= kSmallMaxN)
        rc = (size_t(N) * sizeof(T) * P > (size_t(256) << 20))
                 ? gram_small<T, true>(ctx, grads, N, P, s)
                 : gram_small<T, false>(ctx, grads, N, P, s);
    else
        rc = gram_all_pairs<T>(ctx, grads, N, P, s);
    if (rc != GAF_OK) return rc;
    const int n2 = N * N;
    {
        Timed t(ctx, s, GAF_K_DISTANCE);
        gram_to_distance_kernel<<<(n2 + kBlock - 1) / kBlock, kBlock, 0, s>>>(ctx->gram_full, N, D,
                                                                             gram_out);
    }
    return launched();
}

gaf_status gram_first_dispatch(gaf_ctx *ctx, const void *const *grads, int N, size_t P, gaf_dtype dt,
                               float tau, const BatchOptions &gram, float *out, uint8_t *mask,
                               float *cos_dist, int32_t *count, hipStream_t s)
{
    if (flush_pending(ctx, s) != GAF_OK) return GAF_EHIP;
    // the masked mean reads up to N gradients of s bytes and writes 4 bytes per element
    const bool st = (size_t(N) * (dt == GAF_F32 ? 4 : 2) + 4) * P > (size_t(256) << 20);
    if (dt == GAF_F32)
        return st ? aggregate_gram_impl<float, true>(ctx, grads, N, P, tau, gram, out, mask, cos_dist, count, s)
                  : aggregate_gram_impl<float, false>(ctx, grads, N, P, tau, gram, out, mask, cos_dist, count, s);
    return st ? aggregate_gram_impl<bf16_t, true>(ctx, grads, N, P, tau, gram, out, mask, cos_dist, count, s)
              : aggregate_gram_impl<bf16_t, false>(ctx, grads, N, P, tau, gram, out, mask, cos_dist, count, s);
}

static_assert(size_t(kSegMaxBlocks) * kSmallMaxPairs <= size_t(kGramBlocks) * kGramMaxTiles * kGramTile,
              "the bucketed partial-sum table reuses the Gram workspace");

template <typename T, bool kStream, int N>
gaf_status gram_seg_launch(const SegGramArgs &g, int nblocks, hipStream_t s)
{
    gram_seg_kernel<T, N, kStream><<<nblocks, kBlock, 0, s>>>(g);
    return launched();
}

// Bucketed filtering for small batches in three launches whatever the number of
// buckets: segmented Gram, one filter workgroup per bucket, segmented mean.
template <typename T, bool kStream>
gaf_status bucketed_seg_impl(gaf_ctx *ctx, const void *const *grads, int N, float tau, int B,
                             const size_t *off, float *out, uint8_t *mask, float *cos_dist,
                             int32_t *count, hipStream_t s)
{
    SegGramArgs g{};
    for (int i = 0; i < kSmallMaxN; ++i) g.rows[i] = grads[i < N ? i : 0];
    g.tab.B = B;
    g.partials = ctx->gram_ws;
    // workgroups per bucket: one per tile of the Gram kernel, capped so that all buckets together
    // stay within the partial-sum table
    const size_t tile = small_gram_tile(N, sizeof(T));
    const int cap = kSegMaxBlocks / B < 256 ? kSegMaxBlocks / B : 256;
    int total = 0;
    for (int b = 0; b < B; ++b) {
        const size_t ntiles = (off[b + 1] - off[b] + tile - 1) / tile;
        g.tab.off[b] = off[b];
        g.tab.blk[b] = total;
        total += ntiles < size_t(cap) ? static_cast<int>(ntiles) : cap;
    }
    g.tab.off[B] = off[B];
    g.tab.blk[B] = total;
    gaf_status rc = GAF_OK;
    {
        Timed t(ctx, s, GAF_K_GRAM);
        switch (N) {
        case 1: rc = gram_seg_launch<T, kStream, 1>(g, total, s); break;
        case 2: rc = gram_seg_launch<T, kStream, 2>(g, total, s); break;
        case 3: rc = gram_seg_launch<T, kStream, 3>(g, total, s); break;
        case 4: rc = gram_seg_launch<T, kStream, 4>(g, total, s); break;
        case 5: rc = gram_seg_launch<T, kStream, 5>(g, total, s); break;
        case 6: rc = gram_seg_launch<T, kStream, 6>(g, total, s); break;
        case 7: rc = gram_seg_launch<T, kStream, 7>(g, total, s); break;
        default: rc = gram_seg_launch<T, kStream, 8>(g, total, s); break;
        }
    }
    if (rc != GAF_OK) return rc;
    {
        Timed t(ctx, s, GAF_K_FILTER);
        seg_filter_kernel<<<B, kBlock, 0, s>>>(ctx->gram_ws, g.tab, N, tau, mask, cos_dist, count,
                                               ctx->seg_ws);
    }
    if (launched() != GAF_OK) return GAF_EHIP;
    SegMeanArgs m{};
    for (int i = 0; i < kBatchMaxN; ++i) m.m.rows[i] = grads[i < N ? i : 0];
    m.m.N = N;
    m.m.out = out;
    m.m.P = off[B];
    m.tab = g.tab;
    m.ws = ctx->seg_ws;
    {
        Timed t(ctx, s, GAF_K_MEAN);
        mean_seg_kernel<T, kStream><<<total, kBlock, 0, s>>>(m);
    }
    return launched();
}

// Schedule selection of the plain batch call (arguments already validated).
gaf_status aggregate_dispatch(gaf_ctx *ctx, const void *const *grads, int N, size_t P, gaf_dtype dt,
                              float tau, float *out, uint8_t *accept_mask, float *cos_dist,
                              int32_t *count, hipStream_t s)
{
    if (ctx->schedule == GAF_SCHEDULE_GRAM && (N < 2 || N > kBatchMaxN)) return GAF_EUNSUPPORTED;
    if (flush_pending(ctx, s) != GAF_OK) return GAF_EHIP;
    const bool gram_first = ctx->schedule == GAF_SCHEDULE_GRAM ||
                            (ctx->schedule == GAF_SCHEDULE_AUTO && N >= 2 && N <= kBatchMaxN);
    if (gram_first)
        return gram_first_dispatch(ctx, grads, N, P, dt, tau, BatchOptions{}, out, accept_mask, cos_dist, count, s);
    if (dt == GAF_F32)
        return stream_loads(P, 4)
                   ? aggregate_impl<float, true>(ctx, grads, N, P, tau, out, accept_mask, cos_dist, count, s)
                   : aggregate_impl<float, false>(ctx, grads, N, P, tau, out, accept_mask, cos_dist, count, s);
    return stream_loads(P, 2)
               ? aggregate_impl<bf16_t, true>(ctx, grads, N, P, tau, out, accept_mask, cos_dist, count, s)
               : aggregate_impl<bf16_t, false>(ctx, grads, N, P, tau, out, accept_mask, cos_dist, count, s);
}

// Checks shared by the batch entry points. `out` may be NULL where the caller allows it.
gaf_status check_batch(const gaf_ctx *ctx, const void *const *grads, int N, size_t P, gaf_dtype dt,
                       const float *out, bool out_required)
{
    gaf_status rc = check_ctx(ctx);
    if (rc != GAF_OK) return rc;
    if (!grads || N < 1 || P == 0 || (out_required && !out)) return GAF_EINVAL;
    if (N > ctx->max_N || P > ctx->max_P) return GAF_EINVAL;
    if (dt != GAF_F32 && dt != GAF_BF16) return GAF_EUNSUPPORTED;
    if (out && misaligned(out)) return GAF_EALIGN;
    for (int i = 0; i < N; ++i) {
        if (!grads[i] || (out && grads[i] == static_cast<const void *>(out))) return GAF_EINVAL;
        if (misaligned(grads[i])) return GAF_EALIGN;
    }
    return GAF_OK;
}

// ---- the entry point that allocates nothing -----------------------------------------------
// Its workspace is a fixed array in every device's global memory instead of a context's
// allocations: the same blocks a context holds, laid out back to back. Host code never uses the
// array's name as an address (in host code that name is only a handle for the runtime): the device
// address is asked for once per device and kept.
constexpr size_t align256(size_t n) { return (n + 255) / 256 * 256; }
constexpr size_t kStOffState = 0;
constexpr size_t kStOffPartials = kStOffState + align256(sizeof(State));
constexpr size_t kStOffGramWs = kStOffPartials + align256(sizeof(double) * 3 * kMaxBlocks);
constexpr size_t kStOffGramFull = kStOffGramWs + align256(sizeof(double) * size_t(kGramBlocks) * kGramMaxTiles * kGramTile);
constexpr size_t kStOffAccepted = kStOffGramFull + align256(sizeof(double) * GAF_STATIC_MAX_N * GAF_STATIC_MAX_N);
constexpr size_t kStOffSeedWs = kStOffAccepted + align256(sizeof(int32_t) * GAF_STATIC_MAX_N);
constexpr size_t kStOffSegWs = kStOffSeedWs + align256(sizeof(SeedWs));
constexpr size_t kStOffPred = kStOffSegWs + align256(sizeof(SegWs));
constexpr size_t kStaticScratchBytes = kStOffPred + align256(sizeof(Prediction));
static_assert(GAF_STATIC_MAX_N == kBatchMaxN, "the fixed workspace serves the Gram-first schedule's batch sizes");
static_assert(kStaticScratchBytes <= (size_t(11) << 20), "the fixed workspace is meant to stay modest (about 10.6 MB)");

static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kStaticScratchBytes];

constexpr int kStaticMaxDevices = 64;
std::mutex g_static_mutex;
gaf_ctx g_static_ctx[kStaticMaxDevices];      // pointers into each device's copy of `scratch`
bool g_static_ready[kStaticMaxDevices];
bool g_static_cleared[kStaticMaxDevices];     // the clearing kernel has been enqueued once

// Zeroes the parts of the fixed workspace that a context gets zeroed at creation (decision state,
// Gram matrix, record of guesses). A kernel rather than a memset, so that a caller may capture it.
struct StaticClear {
    unsigned char *base;
    size_t off[3], bytes[3];
};
__global__ void static_clear_kernel(StaticClear c)
{
    for (int r = 0; r < 3; ++r)
        for (size_t b = size_t(blockIdx.x) * blockDim.x + threadIdx.x; b < c.bytes[r] / 4;
             b += size_t(gridDim.x) * blockDim.x)
            reinterpret_cast<uint32_t *>(c.base + c.off[r])[b] = 0u;
}

// The current device's fixed-workspace context, set up on first use: the device address of this
// device's copy of `scratch` is looked up (the only runtime query; no allocation) and the
// context's pointers are set into it.
gaf_status static_context(gaf_ctx **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return GAF_EHIP;
    if (dev < 0 || dev >= kStaticMaxDevices) return GAF_ELIMIT;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    gaf_ctx *c = &g_static_ctx[dev];
    if (!g_static_ready[dev]) {
        unsigned char *base = nullptr;
        if (hipGetSymbolAddress(reinterpret_cast<void **>(&base), HIP_SYMBOL(scratch)) != hipSuccess || !base) {
            (void)hipGetLastError();
            return GAF_EHIP;
        }
        c->device = dev;
        c->max_P = GAF_STATIC_MAX_P;
        c->max_N = GAF_STATIC_MAX_N;
        c->st = reinterpret_cast<State *>(base + kStOffState);
        c->partials = reinterpret_cast<double *>(base + kStOffPartials);
        c->gram_ws = reinterpret_cast<double *>(base + kStOffGramWs);
        c->gram_full = reinterpret_cast<double *>(base + kStOffGramFull);
        c->accepted = reinterpret_cast<int32_t *>(base + kStOffAccepted);
        c->seed_ws = reinterpret_cast<SeedWs *>(base + kStOffSeedWs);
        c->seg_ws = reinterpret_cast<SegWs *>(base + kStOffSegWs);
        c->pred = reinterpret_cast<Prediction *>(base + kStOffPred);
        c->pred_reset = false;
        c->guess_note = nullptr;
        c->pend_g = nullptr;
        c->schedule = GAF_SCHEDULE_AUTO;
        c->prof_on = false;
        c->prof_cap = 0;
        g_static_ready[dev] = true;
    }
    *out = c;
    return GAF_OK;
}

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

const char *gaf_strerror(gaf_status status)
{
    switch (status) {
    case GAF_OK: return "ok";
    case GAF_EINVAL: return "invalid argument";
    case GAF_EALIGN: return "device vector pointer is not 16-byte aligned";
    case GAF_ENOMEM: return "out of device memory";
    case GAF_EHIP: return "HIP runtime call or kernel launch failed";
    case GAF_EUNSUPPORTED: return "unsupported element type, or batch size outside the range of the requested form";
    case GAF_EDEVICE: return "context's device is not the current device";
    case GAF_ELIMIT: return "size beyond the fixed limits of the entry point that allocates nothing";
    }
    return "unknown status";
}

gaf_status gaf_create(gaf_ctx **out_ctx, int device, size_t max_P, int max_N)
{
    if (!out_ctx || max_P == 0 || max_N < 1) return GAF_EINVAL;
    *out_ctx = nullptr;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess) return GAF_EHIP;
    if (device < 0 || device >= ndev) return GAF_EINVAL;
    int prev = 0;
    if (hipGetDevice(&prev) != hipSuccess) return GAF_EHIP;
    if (hipSetDevice(device) != hipSuccess) return GAF_EHIP;

    gaf_ctx *ctx = new (std::nothrow) gaf_ctx();
    if (!ctx) {
        (void)hipSetDevice(prev);
        return GAF_ENOMEM;
    }
    ctx->device = device;
    ctx->max_P = max_P;
    ctx->max_N = max_N;
    ctx->prof_on = false;
    ctx->prof_cap = 0;
    ctx->schedule = GAF_SCHEDULE_AUTO;
    ctx->pred_reset = false;
    ctx->guess_note = nullptr;
    ctx->pend_g = nullptr;
    const size_t gram_ws_bytes = sizeof(double) * size_t(kGramBlocks) * kGramMaxTiles * kGramTile;
    const size_t gram_full_bytes = sizeof(double) * size_t(max_N) * size_t(max_N);
    bool ok = hipMalloc(reinterpret_cast<void **>(&ctx->st), sizeof(State)) == hipSuccess &&
              hipMalloc(reinterpret_cast<void **>(&ctx->partials),
                        sizeof(double) * 3 * kMaxBlocks) == hipSuccess &&
              hipMalloc(reinterpret_cast<void **>(&ctx->gram_ws), gram_ws_bytes) == hipSuccess &&
              hipMalloc(reinterpret_cast<void **>(&ctx->gram_full), gram_full_bytes) == hipSuccess &&
              hipMalloc(reinterpret_cast<void **>(&ctx->accepted),
                        sizeof(int32_t) * size_t(max_N < kBatchMaxN ? kBatchMaxN : max_N)) == hipSuccess &&
              hipMalloc(reinterpret_cast<void **>(&ctx->seed_ws), sizeof(SeedWs)) == hipSuccess &&
              hipMalloc(reinterpret_cast<void **>(&ctx->seg_ws), sizeof(SegWs)) == hipSuccess &&
              hipMalloc(reinterpret_cast<void **>(&ctx->pred), sizeof(Prediction)) == hipSuccess;
    ok = ok && hipMemset(ctx->st, 0, sizeof(State)) == hipSuccess;
    ok = ok && hipMemset(ctx->gram_full, 0, gram_full_bytes) == hipSuccess;
    ok = ok && hipMemset(ctx->pred, 0, sizeof(Prediction)) == hipSuccess;
    {
        // the note the verifying filter leaves for the host (pinned host memory, written by the device)
        void *note = nullptr, *note_dev = nullptr;
        ok = ok && hipHostMalloc(&note, 64, hipHostMallocDefault) == hipSuccess;
        if (ok) {
            ctx->guess_note = static_cast<volatile int32_t *>(note);
            *ctx->guess_note = 1;
            ok = hipHostGetDevicePointer(&note_dev, note, 0) == hipSuccess &&
                 hipMemcpy(&ctx->pred->notify, &note_dev, sizeof note_dev, hipMemcpyHostToDevice) == hipSuccess;
        }
    }
    ok = ok && hipDeviceSynchronize() == hipSuccess;
    (void)hipSetDevice(prev);
    if (!ok) {
        (void)hipGetLastError();
        gaf_destroy(ctx);
        return GAF_ENOMEM;
    }
    *out_ctx = ctx;
    return GAF_OK;
}

gaf_status gaf_destroy(gaf_ctx *ctx)
{
    if (!ctx) return GAF_EINVAL;
    int prev = 0;
    const bool have_prev = hipGetDevice(&prev) == hipSuccess;
    (void)hipSetDevice(ctx->device);
    if (ctx->st) (void)hipFree(ctx->st);
    if (ctx->partials) (void)hipFree(ctx->partials);
    if (ctx->gram_ws) (void)hipFree(ctx->gram_ws);
    if (ctx->gram_full) (void)hipFree(ctx->gram_full);
    if (ctx->accepted) (void)hipFree(ctx->accepted);
    if (ctx->seed_ws) (void)hipFree(ctx->seed_ws);
    if (ctx->seg_ws) (void)hipFree(ctx->seg_ws);
    if (ctx->pred) (void)hipFree(ctx->pred);
    if (ctx->guess_note) (void)hipHostFree(const_cast<int32_t *>(ctx->guess_note));
    for (hipEvent_t e : ctx->prof_ev) (void)hipEventDestroy(e);
    if (have_prev) (void)hipSetDevice(prev);
    delete ctx;
    return GAF_OK;
}

gaf_status gaf_profile_begin(gaf_ctx *ctx, int max_launches)
{
    gaf_status rc = check_ctx(ctx);
    if (rc != GAF_OK) return rc;
    if (max_launches < 1) return GAF_EINVAL;
    for (hipEvent_t e : ctx->prof_ev) (void)hipEventDestroy(e);
    ctx->prof_ev.clear();
    ctx->prof_id.clear();
    try {
        ctx->prof_ev.reserve(2 * static_cast<size_t>(max_launches));
        ctx->prof_id.reserve(static_cast<size_t>(max_launches));
    } catch (...) {
        ctx->prof_on = false;
        return GAF_ENOMEM;
    }
    ctx->prof_cap = max_launches;
    ctx->prof_on = true;
    return GAF_OK;
}

gaf_status gaf_profile_end(gaf_ctx *ctx, gaf_launch_time *out, int cap, int *n)
{
    gaf_status rc = check_ctx(ctx);
    if (rc != GAF_OK) return rc;
    if (!out || !n || cap < 0) return GAF_EINVAL;
    ctx->prof_on = false;
    const int have = static_cast<int>(ctx->prof_id.size());
    const int take = have < cap ? have : cap;
    rc = GAF_OK;
    for (int k = 0; k < take; ++k) {
        float ms = 0.f;
        if (hipEventSynchronize(ctx->prof_ev[2 * k + 1]) != hipSuccess ||
            hipEventElapsedTime(&ms, ctx->prof_ev[2 * k], ctx->prof_ev[2 * k + 1]) != hipSuccess)
            rc = GAF_EHIP;
        out[k].kernel = ctx->prof_id[k];
        out[k].ms = ms;
    }
    *n = take;
    for (hipEvent_t e : ctx->prof_ev) (void)hipEventDestroy(e);
    ctx->prof_ev.clear();
    ctx->prof_id.clear();
    return rc;
}

gaf_status gaf_aggregate(gaf_ctx *ctx, const void *const *grads, int N, size_t P, gaf_dtype dt,
                         float tau, float *out, uint8_t *accept_mask, float *cos_dist,
                         int32_t *count, void *stream)
{
    gaf_status rc = check_ctx(ctx);
    if (rc != GAF_OK) return rc;
    if (!grads || N < 1 || P == 0 || !out || !accept_mask || !cos_dist || !count) return GAF_EINVAL;
    if (N > ctx->max_N || P > ctx->max_P) return GAF_EINVAL;
    if (dt != GAF_F32 && dt != GAF_BF16) return GAF_EUNSUPPORTED;
    if (misaligned(out)) return GAF_EALIGN;
    for (int i = 0; i < N; ++i) {
        if (!grads[i] || grads[i] == static_cast<const void *>(out)) return GAF_EINVAL;
        if (misaligned(grads[i])) return GAF_EALIGN;
    }
    return aggregate_dispatch(ctx, grads, N, P, dt, tau, out, accept_mask, cos_dist, count,
                              static_cast<hipStream_t>(stream));
}

gaf_status gaf_aggregate_with_gram(gaf_ctx *ctx, const void *const *grads, int N, size_t P,
                                   gaf_dtype dt, float tau, const double *gram, float *out,
                                   uint8_t *accept_mask, float *cos_dist, int32_t *count, void *stream)
{
    gaf_status rc = check_ctx(ctx);
    if (rc != GAF_OK) return rc;
    if (!grads || N < 1 || P == 0 || !gram || !out || !accept_mask || !cos_dist || !count)
        return GAF_EINVAL;
    if (N > ctx->max_N || P > ctx->max_P) return GAF_EINVAL;
    if (dt != GAF_F32 && dt != GAF_BF16) return GAF_EUNSUPPORTED;
    if (N > kBatchMaxN) return GAF_EUNSUPPORTED;
    if (misaligned(out)) return GAF_EALIGN;
    for (int i = 0; i < N; ++i) {
        if (!grads[i] || grads[i] == static_cast<const void *>(out)) return GAF_EINVAL;
        if (misaligned(grads[i])) return GAF_EALIGN;
    }
    BatchOptions opt;
    opt.gram = gram;
    return gram_first_dispatch(ctx, grads, N, P, dt, tau, opt, out, accept_mask, cos_dist, count,
                               static_cast<hipStream_t>(stream));
}

gaf_status gaf_aggregate_with_matrix(gaf_ctx *ctx, const void *const *grads, int N, size_t P,
                                     gaf_dtype dt, float tau, float *out, uint8_t *accept_mask,
                                     float *cos_dist, int32_t *count, float *D, double *gram, void *stream)
{
    gaf_status rc = check_batch(ctx, grads, N, P, dt, out, true);
    if (rc != GAF_OK) return rc;
    if (!accept_mask || !cos_dist || !count || !D) return GAF_EINVAL;
    if (N > kBatchMaxN) return GAF_EUNSUPPORTED;
    BatchOptions opt;
    opt.dist_matrix = D;
    opt.gram_out = gram;
    return gram_first_dispatch(ctx, grads, N, P, dt, tau, opt, out, accept_mask, cos_dist, count,
                               static_cast<hipStream_t>(stream));
}

gaf_status gaf_aggregate_best_seed(gaf_ctx *ctx, const void *const *grads, int N, size_t P,
                                   gaf_dtype dt, float tau, float *out, uint8_t *accept_mask,
                                   float *cos_dist, int32_t *count, int32_t *seed, void *stream)
{
    gaf_status rc = check_batch(ctx, grads, N, P, dt, out, true);
    if (rc != GAF_OK) return rc;
    if (!accept_mask || !cos_dist || !count || !seed) return GAF_EINVAL;
    if (N > kBatchMaxN) return GAF_EUNSUPPORTED;
    BatchOptions opt;
    opt.best_seed = seed;
    return gram_first_dispatch(ctx, grads, N, P, dt, tau, opt, out, accept_mask, cos_dist, count,
                               static_cast<hipStream_t>(stream));
}

gaf_status gaf_aggregate_sgd(gaf_ctx *ctx, const void *const *grads, int N, size_t P, gaf_dtype dt,
                             float tau, float *params, float *momentum_buf, float lr, float momentum,
                             float weight_decay, float *out, uint8_t *accept_mask, float *cos_dist,
                             int32_t *count, void *stream)
{
    gaf_status rc = check_batch(ctx, grads, N, P, dt, out, false);
    if (rc != GAF_OK) return rc;
    if (!params || !momentum_buf || !accept_mask || !cos_dist || !count) return GAF_EINVAL;
    if (params == momentum_buf || params == out || momentum_buf == out) return GAF_EINVAL;
    if (misaligned(params) || misaligned(momentum_buf)) return GAF_EALIGN;
    for (int i = 0; i < N; ++i)
        if (grads[i] == static_cast<const void *>(params) || grads[i] == static_cast<const void *>(momentum_buf))
            return GAF_EINVAL;
    if (N > kBatchMaxN) return GAF_EUNSUPPORTED;
    BatchOptions opt;
    opt.theta = params;
    opt.vel = momentum_buf;
    opt.lr = lr;
    opt.mu = momentum;
    opt.wd = weight_decay;
    return gram_first_dispatch(ctx, grads, N, P, dt, tau, opt, out, accept_mask, cos_dist, count,
                               static_cast<hipStream_t>(stream));
}

gaf_status gaf_aggregate_bucketed(gaf_ctx *ctx, const void *const *grads, int N, size_t P,
                                  gaf_dtype dt, float tau, int B, const size_t *bucket_offsets,
                                  float *out, uint8_t *accept_mask, float *cos_dist, int32_t *count,
                                  void *stream)
{
    gaf_status rc = check_batch(ctx, grads, N, P, dt, out, true);
    if (rc != GAF_OK) return rc;
    if (!accept_mask || !cos_dist || !count || B < 1 || !bucket_offsets) return GAF_EINVAL;
    if (bucket_offsets[0] != 0 || bucket_offsets[B] != P) return GAF_EINVAL;
    for (int b = 0; b < B; ++b) {
        if (bucket_offsets[b + 1] <= bucket_offsets[b]) return GAF_EINVAL;
        if (bucket_offsets[b] % 8 != 0) return GAF_EALIGN;   // keeps every slice 16-byte aligned
    }
    if (ctx->schedule == GAF_SCHEDULE_GRAM && (N < 2 || N > kBatchMaxN)) return GAF_EUNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (flush_pending(ctx, st) != GAF_OK) return GAF_EHIP;
    if (N <= kSmallMaxN && B <= kSegMaxBuckets && ctx->schedule != GAF_SCHEDULE_SEQUENTIAL) {
        const bool big = (size_t(N) * (dt == GAF_F32 ? 4 : 2) + 4) * P > (size_t(256) << 20);
        if (dt == GAF_F32)
            return big ? bucketed_seg_impl<float, true>(ctx, grads, N, tau, B, bucket_offsets, out, accept_mask, cos_dist, count, st)
                       : bucketed_seg_impl<float, false>(ctx, grads, N, tau, B, bucket_offsets, out, accept_mask, cos_dist, count, st);
        return big ? bucketed_seg_impl<bf16_t, true>(ctx, grads, N, tau, B, bucket_offsets, out, accept_mask, cos_dist, count, st)
                   : bucketed_seg_impl<bf16_t, false>(ctx, grads, N, tau, B, bucket_offsets, out, accept_mask, cos_dist, count, st);
    }
    const size_t es = dt == GAF_F32 ? 4 : 2;
    const void **slice = new (std::nothrow) const void *[static_cast<size_t>(N)];
    if (!slice) return GAF_ENOMEM;
    for (int b = 0; b < B && rc == GAF_OK; ++b) {
        const size_t lo = bucket_offsets[b], len = bucket_offsets[b + 1] - lo;
        for (int i = 0; i < N; ++i) slice[i] = static_cast<const char *>(grads[i]) + lo * es;
        rc = aggregate_dispatch(ctx, slice, N, len, dt, tau, out + lo, accept_mask + size_t(b) * N,
                                cos_dist + size_t(b) * N, count + b, static_cast<hipStream_t>(stream));
    }
    delete[] slice;
    return rc;
}

gaf_status gaf_set_schedule(gaf_ctx *ctx, gaf_schedule schedule)
{
    if (!ctx) return GAF_EINVAL;
    if (schedule != GAF_SCHEDULE_AUTO && schedule != GAF_SCHEDULE_SEQUENTIAL &&
        schedule != GAF_SCHEDULE_GRAM)
        return GAF_EINVAL;
    ctx->schedule = schedule;
    ctx->pred_reset = true;
    return GAF_OK;
}

gaf_status gaf_fused_mean_record(gaf_ctx *ctx, int32_t record[4])
{
    gaf_status rc = check_ctx(ctx);
    if (rc != GAF_OK) return rc;
    if (!record) return GAF_EINVAL;
    Prediction h;
    if (hipDeviceSynchronize() != hipSuccess ||
        hipMemcpy(&h, ctx->pred, sizeof h, hipMemcpyDeviceToHost) != hipSuccess) {
        (void)hipGetLastError();
        return GAF_EHIP;
    }
    if (ctx->pred_reset) h.write = h.valid = h.backoff = h.penalty = 0;   // cleared, not yet on the device
    record[0] = h.write;
    record[1] = h.valid;
    record[2] = h.backoff;
    record[3] = h.penalty < 1 ? 1 : h.penalty;
    return GAF_OK;
}

gaf_status gaf_step(gaf_ctx *ctx, float *accum, int32_t *count, const void *g_i, size_t P,
                    gaf_dtype dt, float tau, float *cos_dist_out, uint8_t *accepted_out,
                    void *stream)
{
    gaf_status rc = check_ctx(ctx);
    if (rc != GAF_OK) return rc;
    if (!accum || !count || !g_i || P == 0 || g_i == static_cast<const void *>(accum))
        return GAF_EINVAL;
    if (P > ctx->max_P) return GAF_EINVAL;
    if (dt != GAF_F32 && dt != GAF_BF16) return GAF_EUNSUPPORTED;
    if (misaligned(accum) || misaligned(g_i)) return GAF_EALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (flush_pending(ctx, s) != GAF_OK) return GAF_EHIP;
    if (dt == GAF_F32)
        return stream_loads(P, 4)
                   ? step_impl<float, true>(ctx, accum, count, g_i, P, tau, cos_dist_out, accepted_out, s)
                   : step_impl<float, false>(ctx, accum, count, g_i, P, tau, cos_dist_out, accepted_out, s);
    return stream_loads(P, 2)
               ? step_impl<bf16_t, true>(ctx, accum, count, g_i, P, tau, cos_dist_out, accepted_out, s)
               : step_impl<bf16_t, false>(ctx, accum, count, g_i, P, tau, cos_dist_out, accepted_out, s);
}

gaf_status gaf_step_lookahead(gaf_ctx *ctx, float *accum, int32_t *count, const void *g_i, size_t P,
                              gaf_dtype dt, float tau, float *cos_dist_out, uint8_t *accepted_out,
                              void *stream)
{
    gaf_status rc = check_ctx(ctx);
    if (rc != GAF_OK) return rc;
    if (!accum || !count || !g_i || P == 0 || g_i == static_cast<const void *>(accum))
        return GAF_EINVAL;
    if (P > ctx->max_P) return GAF_EINVAL;
    if (dt != GAF_F32 && dt != GAF_BF16) return GAF_EUNSUPPORTED;
    if (misaligned(accum) || misaligned(g_i)) return GAF_EALIGN;
    // a pending gradient belongs to one running aggregate: the same (accum, count, P, dtype)
    if (ctx->pend_g && (ctx->pend_accum != accum || ctx->pend_count != count || ctx->pend_P != P ||
                        ctx->pend_dt != dt || ctx->pend_g == g_i))
        return GAF_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dt == GAF_F32)
        rc = stream_loads(P, 4)
                 ? step_lookahead_impl<float, true>(ctx, accum, count, g_i, P, tau, cos_dist_out, accepted_out, s)
                 : step_lookahead_impl<float, false>(ctx, accum, count, g_i, P, tau, cos_dist_out, accepted_out, s);
    else
        rc = stream_loads(P, 2)
                 ? step_lookahead_impl<bf16_t, true>(ctx, accum, count, g_i, P, tau, cos_dist_out, accepted_out, s)
                 : step_lookahead_impl<bf16_t, false>(ctx, accum, count, g_i, P, tau, cos_dist_out, accepted_out, s);
    if (rc != GAF_OK) {
        ctx->pend_g = nullptr;
        return rc;
    }
    ctx->pend_g = g_i;
    ctx->pend_accum = accum;
    ctx->pend_count = count;
    ctx->pend_P = P;
    ctx->pend_dt = dt;
    return GAF_OK;
}

gaf_status gaf_flush(gaf_ctx *ctx, void *stream)
{
    gaf_status rc = check_ctx(ctx);
    if (rc != GAF_OK) return rc;
    return flush_pending(ctx, static_cast<hipStream_t>(stream));
}

gaf_status gaf_pairwise(gaf_ctx *ctx, const void *const *grads, int N, size_t P, gaf_dtype dt,
                        float *D, double *gram, void *stream)
{
    gaf_status rc = check_ctx(ctx);
    if (rc != GAF_OK) return rc;
    if (!grads || N < 1 || P == 0 || !D) return GAF_EINVAL;
    if (N > ctx->max_N || P > ctx->max_P) return GAF_EINVAL;
    if (dt != GAF_F32 && dt != GAF_BF16) return GAF_EUNSUPPORTED;
    for (int i = 0; i < N; ++i) {
        if (!grads[i]) return GAF_EINVAL;
        if (misaligned(grads[i])) return GAF_EALIGN;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    return dt == GAF_F32 ? pairwise_impl<float>(ctx, grads, N, P, D, gram, s)
                         : pairwise_impl<bf16_t>(ctx, grads, N, P, D, gram, s);
}

gaf_status gaf_static_init(void)
{
    gaf_ctx *ctx = nullptr;
    return static_context(&ctx);
}

gaf_status gaf_aggregate_static(const void *const *grads, int N, size_t P, gaf_dtype dt, float tau,
                                float *out, uint8_t *accept_mask, float *cos_dist, int32_t *count,
                                void *stream)
{
    if (!grads || N < 1 || P == 0 || !out || !accept_mask || !cos_dist || !count) return GAF_EINVAL;
    if (N > GAF_STATIC_MAX_N || P > GAF_STATIC_MAX_P) return GAF_ELIMIT;
    if (dt != GAF_F32 && dt != GAF_BF16) return GAF_EUNSUPPORTED;
    if (misaligned(out)) return GAF_EALIGN;
    for (int i = 0; i < N; ++i) {
        if (!grads[i] || grads[i] == static_cast<const void *>(out)) return GAF_EINVAL;
        if (misaligned(grads[i])) return GAF_EALIGN;
    }
    gaf_ctx *ctx = nullptr;
    const gaf_status rc = static_context(&ctx);
    if (rc != GAF_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    {
        // first call on this device: the workspace starts from zero like a fresh context's
        std::lock_guard<std::mutex> lock(g_static_mutex);
        if (!g_static_cleared[ctx->device]) {
            StaticClear c{reinterpret_cast<unsigned char *>(ctx->st),
                          {kStOffState, kStOffGramFull, kStOffPred},
                          {sizeof(State), sizeof(double) * GAF_STATIC_MAX_N * GAF_STATIC_MAX_N, sizeof(Prediction)}};
            static_clear_kernel<<<8, kBlock, 0, s>>>(c);
            if (launched() != GAF_OK) return GAF_EHIP;
            g_static_cleared[ctx->device] = true;
        }
    }
    return aggregate_dispatch(ctx, grads, N, P, dt, tau, out, accept_mask, cos_dist, count, s);
}

}  // extern "C"
#pragma GCC visibility pop
