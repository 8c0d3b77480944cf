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
// over all k, so one register serves as A or as B unchanged. Four groups (64
// rows) need 10 tiles; the symmetric half is never computed.
//
// Memory side. The matrix-core layout wants 16 different rows in 16 adjacent
// lanes. Loading global memory that way (each lane 32 bytes of its own row) was
// measured at 2.6 TB/s with the MFMAs removed -- every 16-lane group of a load
// touches 16 different cache lines. So global loads are made fully coalesced
// instead (16 adjacent lanes read 256 contiguous bytes of ONE row, a wavefront
// load covers 4 rows) and the tile of the matrix is turned through LDS:
//   stage = (16 NG rows) x (256 M bytes); each of the 4 wavefronts loads a
//   quarter of the rows, stores its 16-byte pieces to LDS (row stride padded by
//   16 bytes: conflict-free), and after one barrier reads back, for EVERY row,
//   its own quarter of the stage's columns in matrix-core layout.
// Two LDS stages alternate (one, with a second barrier, in the kernels that also write
// the mean); the global loads of stage k+1 are issued before the MFMAs of stage k. Tiles accumulate in binary32 inside the matrix core and are
// flushed into binary64 registers every kGramFlush stages.
#pragma once
#include <type_traits>

#include "gaf_device.hpp"

namespace gaf {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

constexpr int kGramGroups = 4;          // row groups per launch
constexpr int kGramRows = 16 * kGramGroups;
constexpr int kGramFlush = 8;           // stages between binary32 -> binary64 flushes
constexpr int kGramBlocks = 512;        // (virtual) workgroups per launch (fixed: the summation order depends on it)
constexpr int kGramTile = 16 * 16;      // entries per tile
constexpr int kGramMaxTiles = 10;       // 4 groups: 4 diagonal + 6 off-diagonal tiles
constexpr int kGramPad = 4;             // LDS row padding, 32-bit words
constexpr size_t kSampleChunk = size_t(1) << 14;   // elements per contiguous run of a sampling launch

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

// Stage width in units of 256 bytes per row, by number of row groups: 16 KB per stage with one
// or two groups, 32 KB with three or four, i.e. 32-64 KB of loads in flight per compute unit.
// (Measured with plain streaming loops: 16-32 KB in flight per compute unit already saturate the
// memory system; beyond 64 KB the queues in front of it only get longer.) The width is the same
// for every variant of a group count, so that all of them add the columns in the same order.
__host__ __device__ constexpr int gram_stage_m(int ng) { return ng == 1 ? 4 : 2; }

// An accept set guessed before the full inner products are known: which gradients
// Algorithm 1 will probably accept, in visiting order, and what is done with the guess.
// Two sources of guesses: for long vectors a filter run on a sample of the vectors
// (it also decides `write`); for shorter ones, where a sample would cost too large a share,
// the accept set of the previous call with the same N (agreement rates drift slowly over
// training; with the two micro-batches of the paper's experiments the guess is simply
// "as last time"). Lives in device memory for the context's lifetime: the fields from `n` on
// carry the record from call to call.
struct Prediction {
    int32_t count;
    int32_t list[kGramRows];
    int32_t write;     // this call's Gram pass writes the mean of the guess
    int32_t valid;     // ... and the guess was right: the result is in place (set by the full filter)
    int32_t n;         // batch size the guess belongs to
    int32_t backoff;   // calls left during which no guess is written, after a wrong one
    int32_t penalty;   // backoff imposed by the next wrong guess: doubles per miss up to kSpecMaxPenalty,
                       // halves per hit; 0 = never used, treated as 1
    uint32_t next_tile;  // work counter of the mean launch after a guess (cleared by the verifying filter)
    int32_t *notify;   // host memory the device can write, or null: receives `valid` of every verified guess,
                       // so that the host can size the next call's mean launch for what is likely to come
                       // (a hint only: no result depends on it). Set once when the context is created.
};

// Guess carried over from the previous call (carry_n = this call's N): is it usable, and does
// this call's Gram pass therefore write its mean? Evaluated identically by every workgroup of
// the Gram pass and, afterwards, by the filter that verifies the guess; the record is not
// modified in between.
__device__ __forceinline__ bool carried_guess_writes(const Prediction *p, int carry_n, int min_count)
{
    return p->n == carry_n && p->count >= min_count && p->count <= carry_n && p->backoff == 0;
}
constexpr int kSpecMaxPenalty = 64;

struct GramArgs {
    const void *rows[kGramRows];  // DEVICE pointers, group g = rows[16 g .. 16 g + 15]; never NULL: rows past
                                  // the last gradient alias a real one and their tile entries are dropped
    size_t P;
    double *ws;                   // [kGramBlocks][kGramMaxTiles][kGramTile] per-workgroup tiles
    // kMean only: the mean of the predicted accept set is formed from the staged data and written here
    const Prediction *pred;
    float *out;
    // kMean launches write the mean only if pred->write says so (carry_n == 0: guess from a sample)
    // or if carried_guess_writes(pred, carry_n, min_count) (guess carried over from the last call).
    int carry_n, min_count;
    // Sampling launches read runs of 2^chunk_shift stages, run r starting at element r * chunk_stride;
    // an ordinary launch has chunk_shift = 62 (one run that never ends) and chunk_stride = 0.
    int chunk_shift;
    size_t chunk_stride;
    // kMean only: write windows (see WriteGate): period and length of the window in ticks of the
    // constant 100 MHz clock; gate_win = 0: no windows.
    unsigned gate_period, gate_win;
};

// 16 bytes of a row starting at element p, element-wise and zero past the end.
__device__ __forceinline__ u32x4_t gram_load_guarded(const GAF_GLOBAL float *row, size_t p, size_t P)
{
    u32x4_t v;
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = p + e < P ? __float_as_uint(row[p + e]) : 0u;
    return v;
}
__device__ __forceinline__ u32x4_t gram_load_guarded(const GAF_GLOBAL bf16_t *row, size_t p, size_t P)
{
    u32x4_t v;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const size_t q = p + 2 * e;
        const uint32_t lo = q < P ? row[q] : 0u, hi = q + 1 < P ? row[q + 1] : 0u;
        v[e] = lo | (hi << 16);
    }
    return v;
}

template <typename T>
__device__ __forceinline__ void gram_mma(const u32x4_t &x, const u32x4_t &y, floatx4 &acc, int e)
{
    if (sizeof(T) == 4)
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(x[e]), __uint_as_float(y[e]), acc, 0, 0, 0);
    else
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, x),
                                                      __builtin_bit_cast(bf16x8_t, y), acc, 0, 0, 0);
}

// Splits 8 binary32 values into three bfloat16 vectors with x = hi + mid + lo
// (each step rounds to nearest even and subtracts exactly, so the residuals have
// no preferred sign). hi*hi + hi*mid + mid*hi + mid*mid + hi*lo + lo*hi then
// reproduces x*y to about 2^-23 relative -- binary32 product accuracy -- with six
// bfloat16 MFMAs that together take 3/8 of the time of the binary32 MFMAs they
// replace. Converted two values at a time (one packed conversion instruction per pair).
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void split3(const u32x4_t &w0, const u32x4_t &w1, bf16x8_t &hi, bf16x8_t &mid,
                                       bf16x8_t &lo)
{
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
        const f32x2_t x = {__uint_as_float(e < 4 ? w0[e & 3] : w1[e & 3]),
                           __uint_as_float(e < 4 ? w0[(e + 1) & 3] : w1[(e + 1) & 3])};
        const bf16x2_t h = __builtin_convertvector(x, bf16x2_t);
        const f32x2_t r1 = x - __builtin_convertvector(h, f32x2_t);
        const bf16x2_t m = __builtin_convertvector(r1, bf16x2_t);
        const f32x2_t r2 = r1 - __builtin_convertvector(m, f32x2_t);
        const bf16x2_t l = __builtin_convertvector(r2, bf16x2_t);
        hi[e] = h[0];
        hi[e + 1] = h[1];
        mid[e] = m[0];
        mid[e + 1] = m[1];
        lo[e] = l[0];
        lo[e + 1] = l[1];
    }
}

__device__ __forceinline__ void mma_bf16(const bf16x8_t &x, const bf16x8_t &y, floatx4 &acc)
{
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, y, acc, 0, 0, 0);
}

// kMean: while a stage sits in LDS, the mean (Eq. 5) of the gradients a
// Prediction names is formed from it and written to a.out -- same summation
// order and arithmetic as the stand-alone mean kernel, so the values are
// bit-identical to what that kernel would write for the same accept set. If the
// prediction turns out right (checked on the device once the full inner
// products are known) the accepted gradients are never read a second time.
//
// kSplit (binary32 rows only): multiply through the three-way bfloat16 split
// instead of binary32 MFMAs. Used where the binary32 matrix rate would bind
// (three or four row groups); with one or two groups the kernel is memory bound
// either way and the split would only add vector-ALU work.
//
constexpr int kLdsPerBlock = 79 * 1024;   // bytes of LDS a workgroup may use: two workgroups per compute unit (160 KB)

// Geometry of a writing (kMean) kernel's LDS, by element size and number of row groups: words per
// stage buffer (16 NG rows and the zero row, each padded), bytes of one stage's piece of the mean,
// and how many such pieces the ring behind the stage buffer holds.
__host__ __device__ constexpr int gram_mean_stage_words(int ng) { return (16 * ng + 1) * (64 * gram_stage_m(ng) + kGramPad); }
__host__ __device__ constexpr int gram_piece_bytes(int elem_bytes, int ng) { return 256 * gram_stage_m(ng) / elem_bytes * 4; }
// (A writing kernel stages through ONE LDS buffer -- a second barrier per stage instead of a second
// buffer -- so that the ring gets the space: with 64 rows two buffers would leave it 12 KB, far
// less than a write window's worth. Measured against two buffers: 64 x 2.5e8 bf16 5.87 -> 5.33 ms,
// 64 x 1.24e8 binary32 5.86 -> 5.77, 32 x 5e8 bf16 5.44 -> 5.34, 16 x 1e9 bf16 5.66 -> 5.60.)
__host__ __device__ constexpr int gram_mean_bufs(int) { return 1; }
__host__ __device__ constexpr int gram_hold_stages_for(int elem_bytes, int ng)
{
    const int n = (kLdsPerBlock - gram_mean_bufs(ng) * gram_mean_stage_words(ng) * 4) / gram_piece_bytes(elem_bytes, ng);
    return n < 64 ? n : 64;
}
template <typename T>
constexpr int gram_hold_stages(int ng) { return gram_hold_stages_for(int(sizeof(T)), ng); }

template <typename T, int NG, int kMode, bool kMean = false, bool kSplit = (sizeof(T) == 4 && NG >= 3)>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(2))) void gram_kernel(GramArgs a)
{
    // Lane from the execution mask and wavefront index as a scalar, so that nothing in the loops
    // depends on the register the thread index arrives in (the compiler was seen to spill that
    // register and to reload it inside the stage loop, behind a wait for every load in flight).
    const int lane = int(__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)));
    const int wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 6);
    const int tid = wave * 64 + lane;
    const size_t vblock = blockIdx.x;
    // a sampling launch has nothing to do while a backoff runs: no guess will be written
    if (a.chunk_stride != 0 && a.pred->backoff > 0) return;
    typedef TileList<NG, kMode> Tiles;
    constexpr int NT = Tiles::count;
    constexpr int M = gram_stage_m(NG);
    constexpr int kRows = 16 * NG;
    constexpr int kRowWords = 64 * M + kGramPad;            // LDS words per row of a stage
    // kMean: one more row per stage buffer, all zeros, stands in for "no gradient" (see mean_piece)
    constexpr int kStageWords = (kRows + (kMean ? 1 : 0)) * kRowWords;
    constexpr int kElem16 = 16 / sizeof(T);                 // elements per 16-byte piece
    constexpr size_t kStageElems = size_t(256) * M / sizeof(T);   // elements of each row per stage
    constexpr int kInner = sizeof(T) == 4 ? 4 : 1;          // MFMAs per 16-byte register
    constexpr int kBufs = kMean ? gram_mean_bufs(NG) : 2;   // stage buffers in LDS

    // kMean: the first kQuads threads each own four consecutive columns of a stage (16-byte stores;
    // 8-byte ones by twice the threads measured 2 % slower), and a ring of finished pieces of the
    // mean (one piece = the stage's kStageElems binary32 results) waits in LDS for the next write
    // window: whatever a workgroup's share of the LDS (two workgroups per compute unit) leaves
    // after the stage buffer.
    constexpr int kQuads = int(kStageElems) / 4;
    static_assert(kQuads <= kBlock, "at most one quad of a stage per thread");
    constexpr int kPieceBytes = int(kStageElems) * 4;
    constexpr int kHoldStages = kMean ? gram_hold_stages<T>(NG) : 0;
    static_assert(!kMean || (kHoldStages >= 8 && kStageWords == gram_mean_stage_words(NG) && kPieceBytes == gram_piece_bytes(sizeof(T), NG)),
                  "ring geometry");
    constexpr int kHoldWords = kHoldStages * kPieceBytes / 4;
    __shared__ __attribute__((aligned(16))) uint32_t stage[kBufs * kStageWords + kHoldWords];
    static_assert((kBufs * kStageWords + kHoldWords) * 4 >= NT * kGramTile * 8, "the LDS is reused for the final combine");
    __shared__ const void *row_table[kGramRows];
    __shared__ int gate_flag[2];

    const int l16 = lane & 15, sub = lane >> 4;

    // pointer table into LDS, read with compile-time indices so that it stays in
    // the kernel-argument segment
    if (threadIdx.x < kRows) {
        const void *p = nullptr;
#pragma unroll
        for (int k = 0; k < kRows; ++k)
            if (int(threadIdx.x) == k) p = a.rows[k];
        row_table[threadIdx.x] = p;
    }
    // kMean: LDS word offset, within a stage buffer, of the k-th gradient of the guessed accept set
    // (visiting order); entries past the guess point at the zero row. The table lives in LDS; a
    // stage's mean reads it back four entries at a time (the same address in every lane) and moves
    // them to scalar registers, so that the row reads that follow are "scalar offset plus the
    // thread's columns" and no register is tied up between stages.
    __shared__ __attribute__((aligned(16))) int32_t pred_off[kGramRows];
    int c_pred = 0;
    bool write_mean = false;
    if (kMean) {
        c_pred = a.pred->count;
        write_mean = a.carry_n ? carried_guess_writes(a.pred, a.carry_n, a.min_count) : a.pred->write != 0;
        if (!write_mean) c_pred = 0;
        if (c_pred > kRows) c_pred = kRows;
        if (tid < kRows) {
            const int r = tid < c_pred ? a.pred->list[tid] : -1;
            pred_off[tid] = (r >= 0 && r < kRows ? r : kRows) * kRowWords;
        }
        for (int w = tid; w < kRowWords; w += kBlock)
            stage[kRows * kRowWords + w] = stage[(kBufs - 1) * kStageWords + kRows * kRowWords + w] = 0u;
    }
    __syncthreads();

    // loading role: this wavefront owns rows [4 NG wave, 4 NG (wave+1)); lane = (row sub, 16-byte piece l16)
    const GAF_GLOBAL T *lrow[NG];
    int lword[NG];
#pragma unroll
    for (int j = 0; j < NG; ++j) {
        const int rr = 4 * NG * wave + 4 * j + sub;
        lrow[j] = as_global<T>(row_table[rr]);
        lword[j] = rr * kRowWords + l16 * 4;
    }
    // computing role: this wavefront owns columns [16 M wave, 16 M (wave+1)) words of every row;
    // lane = (row l16 of each group, k-slot sub)
    const int cword = l16 * kRowWords + wave * 16 * M + sub * 4;

    const size_t P = a.P;
    const size_t nfull = P / kStageElems;
    const size_t G = gridDim.x;

    floatx4 acc[NT];
    double tot[NT][4];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int v = 0; v < 4; ++v) tot[t][v] = 0.0;
    }

    const int chunk_shift = a.chunk_shift;
    const size_t chunk_stride = a.chunk_stride;
    auto stage_base = [&](size_t s) {      // first element of stage s (uniform)
        return (s >> chunk_shift) * chunk_stride + (s & ((size_t(1) << chunk_shift) - 1)) * kStageElems;
    };
    u32x4_t pre[NG][M];
    auto gload = [&](size_t s) {
        const size_t e0 = stage_base(s) + size_t(l16) * kElem16;
#pragma unroll
        for (int j = 0; j < NG; ++j)
#pragma unroll
            for (int m = 0; m < M; ++m)
                pre[j][m] = __builtin_nontemporal_load(
                    reinterpret_cast<const GAF_GLOBAL u32x4_t *>(lrow[j] + e0 + size_t(m) * 16 * kElem16));
    };
    auto gload_guarded = [&](size_t s) {
        const size_t e0 = s * kStageElems + size_t(l16) * kElem16;
#pragma unroll
        for (int j = 0; j < NG; ++j)
#pragma unroll
            for (int m = 0; m < M; ++m)
                pre[j][m] = gram_load_guarded(lrow[j], e0 + size_t(m) * 16 * kElem16, P);
    };
    auto lstore = [&](int buf) {
#pragma unroll
        for (int j = 0; j < NG; ++j)
#pragma unroll
            for (int m = 0; m < M; ++m)
                *reinterpret_cast<u32x4_t *>(&stage[buf * kStageWords + lword[j] + m * 64]) = pre[j][m];
    };
    auto compute = [&](int buf) {
        if (kSplit) {
            // Group g + 1 is read and split (vector ALU) while the tiles whose later group is g are
            // multiplied (matrix core): the tile list is ordered by later group, so the two streams
            // of instructions are independent and can be issued side by side.
            static_assert(M % 2 == 0, "the split path consumes 32 columns per MFMA");
#pragma unroll
            for (int c = 0; c < M / 2; ++c) {
                bf16x8_t hi[NG], mid[NG], lo[NG];
                auto fetch = [&](int g) {
                    const uint32_t *src = &stage[buf * kStageWords + (g * 16 + l16) * kRowWords +
                                                 wave * 16 * M + c * 32 + sub * 8];
                    split3(*reinterpret_cast<const u32x4_t *>(src), *reinterpret_cast<const u32x4_t *>(src + 4),
                           hi[g], mid[g], lo[g]);
                };
                fetch(0);
                // Phase g: the tiles whose later group is g (6 (g + 1) MFMAs), with the split of
                // group g + 1 (about 48 vector-ALU instructions) dealt out between them; left to
                // itself the scheduler puts all splits first and all MFMAs behind them, and the two
                // pipes take turns instead of running side by side.
#define GAF_GRAM_PHASE(g)                                                                         \
    if (g < NG) {                                                                                 \
        if (g + 1 < NG) fetch(g + 1);                                                             \
        _Pragma("unroll") for (int t = 0; t < NT; ++t)                                            \
        {                                                                                         \
            const int ga = Tiles::ga(t), gb = Tiles::gb(t);                                       \
            if (kMode == kFull ? gb != g : (g != NG - 1)) continue;                               \
            mma_bf16(hi[ga], hi[gb], acc[t]);                                                     \
            mma_bf16(hi[ga], mid[gb], acc[t]);                                                    \
            mma_bf16(mid[ga], hi[gb], acc[t]);                                                    \
            mma_bf16(mid[ga], mid[gb], acc[t]);                                                   \
            mma_bf16(hi[ga], lo[gb], acc[t]);                                                     \
            mma_bf16(lo[ga], hi[gb], acc[t]);                                                     \
        }                                                                                         \
        if (kMode == kFull && g + 1 < NG) {                                                       \
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);                                    \
            _Pragma("unroll") for (int i = 0; i < 6 * (g + 1); ++i)                               \
            {                                                                                     \
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                \
                __builtin_amdgcn_sched_group_barrier(0x002, (48 + 6 * (g + 1) - 1) / (6 * (g + 1)), 0); \
            }                                                                                     \
        }                                                                                         \
        __builtin_amdgcn_sched_barrier(0);                                                        \
    }
                GAF_GRAM_PHASE(0)
                GAF_GRAM_PHASE(1)
                GAF_GRAM_PHASE(2)
                GAF_GRAM_PHASE(3)
#undef GAF_GRAM_PHASE
            }
            return;
        }
#pragma unroll
        for (int c = 0; c < M; ++c) {
            u32x4_t x[NG];
#pragma unroll
            for (int g = 0; g < NG; ++g)
                x[g] = *reinterpret_cast<const u32x4_t *>(
                    &stage[buf * kStageWords + g * 16 * kRowWords + cword + c * 16]);
#pragma unroll
            for (int e = 0; e < kInner; ++e)
#pragma unroll
                for (int t = 0; t < NT; ++t) gram_mma<T>(x[Tiles::ga(t)], x[Tiles::gb(t)], acc[t], e);
        }
    };
    // Eq. 5 over the guessed accept set for the stage in buffer `buf`: a thread adds, for each of
    // its four columns, the guessed rows in visiting order, a batch of rows' reads issued at once;
    // rows past the guess read the zero row, and adding +0 changes no bit of a sum that started
    // from +0.
    const float inv_c = 1.0f / (float)(c_pred > 0 ? c_pred : 1);
    constexpr int kMeanBatch = 8;      // rows read at once
    auto mean_piece = [&](int buf) {
        f32x4_t sum = {0.f, 0.f, 0.f, 0.f};
        if (tid < kQuads) {
            const uint32_t *src = &stage[buf * kStageWords + (sizeof(T) == 4 ? 4 : 2) * tid];
            typedef int32_t i32x4_t __attribute__((ext_vector_type(4)));
            for (int k0 = 0; k0 < c_pred; k0 += 16) {      // uniform trip count
                // sixteen offsets in one go (one LDS round trip), then the rows in batches
                i32x4_t offv[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) offv[q] = *reinterpret_cast<const i32x4_t *>(&pred_off[k0 + 4 * q]);
                int o[16];
#pragma unroll
                for (int k = 0; k < 16; ++k) o[k] = __builtin_amdgcn_readfirstlane(offv[k / 4][k % 4]);
#pragma unroll
                for (int b0 = 0; b0 < 16; b0 += kMeanBatch) {
                    if (k0 + b0 >= c_pred) break;          // uniform
                    if (sizeof(T) == 4) {
                        u32x4_t w[kMeanBatch];
#pragma unroll
                        for (int k = 0; k < kMeanBatch; ++k) w[k] = *reinterpret_cast<const u32x4_t *>(src + o[b0 + k]);
#pragma unroll
                        for (int k = 0; k < kMeanBatch; ++k) {
                            sum.x += __uint_as_float(w[k].x);
                            sum.y += __uint_as_float(w[k].y);
                            sum.z += __uint_as_float(w[k].z);
                            sum.w += __uint_as_float(w[k].w);
                        }
                    } else {
                        u32x2_t w[kMeanBatch];
#pragma unroll
                        for (int k = 0; k < kMeanBatch; ++k) w[k] = *reinterpret_cast<const u32x2_t *>(src + o[b0 + k]);
#pragma unroll
                        for (int k = 0; k < kMeanBatch; ++k) {
                            sum.x += __uint_as_float(w[k].x << 16);
                            sum.y += __uint_as_float(w[k].x & 0xffff0000u);
                            sum.z += __uint_as_float(w[k].y << 16);
                            sum.w += __uint_as_float(w[k].y & 0xffff0000u);
                        }
                    }
                }
            }
        }
        return f32x4_t{sum.x * inv_c, sum.y * inv_c, sum.z * inv_c, sum.w * inv_c};
    };
    // The mean of full stage s: one 16-byte store per thread, 4 KB or less, contiguous.
    GAF_GLOBAL float *const mean_out = as_global<float>(a.out);
    auto mean_store = [&](const f32x4_t &o, size_t s) {
        if (tid < kQuads)
            __builtin_nontemporal_store(o, reinterpret_cast<GAF_GLOBAL f32x4_t *>(mean_out + s * kStageElems + size_t(tid) * 4));
    };
    // ragged last stage: element-wise guarded
    auto mean_store_guarded = [&](const f32x4_t &o, size_t s) {
        const size_t idx = s * kStageElems + size_t(tid) * 4;
        if (tid < kQuads)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (idx + e < P) mean_out[idx + e] = o[e];
    };
    // Pieces of the mean wait in the LDS ring (each thread reads back only what it wrote itself).
    f32x4_t *const hold = reinterpret_cast<f32x4_t *>(stage + kBufs * kStageWords);
    auto hold_put = [&](int slot, const f32x4_t &o) {
        if (tid < kQuads) hold[slot * kQuads + tid] = o;
    };
    // writes out the `n` held pieces, which belong to stages s0, s0 + G, ...
    // (LDS reads in batches, so that the stores of a flush leave within a fraction of a window)
    constexpr int kFlushBatch = 8;
    auto hold_flush = [&](int n, size_t s0) {
        if (tid < kQuads)
            for (int j0 = 0; j0 < n; j0 += kFlushBatch) {
                f32x4_t v[kFlushBatch];
#pragma unroll
                for (int j = 0; j < kFlushBatch; ++j) v[j] = hold[((j0 + j < n) ? j0 + j : j0) * kQuads + tid];
#pragma unroll
                for (int j = 0; j < kFlushBatch; ++j)
                    if (j0 + j < n) mean_store(v[j], s0 + size_t(j0 + j) * G);
            }
    };
    auto flush = [&]() {
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                tot[t][v] += (double)acc[t][v];
                acc[t][v] = 0.f;
            }
    };

    // This workgroup takes stages blockIdx.x, blockIdx.x + G, ...: n_mine of them. All but the last
    // have a successor to prefetch; they run as a loop without a condition around its loads, so
    // that the compiler can count them: the wait before the LDS stores then covers the prefetching
    // loads and nothing younger.
    const size_t n_mine = nfull > vblock ? (nfull - vblock + G - 1) / G : 0;
    const size_t n_steady = n_mine > 0 ? n_mine - 1 : 0;
    int buf = 0, since_flush = 0;
    auto run = [&](auto with_mean) {
        constexpr bool kWrite = kMean && decltype(with_mean)::value;
        if (n_mine > 0) {
            gload(vblock);
            lstore(0);
        }
        __syncthreads();
        size_t k = 0;
        if (n_steady > 0) {
            size_t s = vblock;
            WriteGate gate(a.gate_period, a.gate_win);
            int held = 0, parity = 0;          // pieces in the ring; which of the two flags this stage uses
            size_t held_from = s;              // stage of the oldest piece
            for (; k < n_steady; ++k, s += G) {
                gload(s + G);              // in flight during the MFMAs below
                compute(buf);
                if (kWrite) {
                    hold_put(held, mean_piece(buf));
                    ++held;
                    // one thread looks at the clock; the whole workgroup acts on what it saw, after
                    // the barrier below (flags alternate: the next look may come before a slow
                    // wavefront has read this one)
                    if (wave == 0 && lane == 0) gate_flag[parity] = gate.open() ? 1 : 0;
                }
                if (++since_flush == kGramFlush) {
                    since_flush = 0;
                    flush();
                }
                if (kBufs == 2) {
                    lstore(buf ^ 1);       // the other buffer was last read before the previous barrier
                    __syncthreads();
                    buf ^= 1;
                } else {                   // one buffer: everyone must be done reading it first
                    __syncthreads();
                    lstore(0);
                    __syncthreads();
                }
                if (kWrite) {
                    const bool open = gate_flag[parity] != 0;
                    parity ^= 1;
                    // window open: out with everything held, then no loads until it closes;
                    // ring full: cannot wait for a window
                    if (open || held == kHoldStages) {
                        hold_flush(held, held_from);
                        held = 0;
                        held_from = s + G;
                        if (open) gate.wait_closed();
                    }
                }
            }
            if (kWrite) hold_flush(held, held_from);
        }
        if (k < n_mine) {              // the last full stage
            compute(buf);
            if (kWrite) mean_store(mean_piece(buf), vblock + k * G);
        }
        // ragged tail (P not a multiple of the stage width): one workgroup, element-wise guarded loads
        if (nfull * kStageElems < P && vblock == nfull % G) {
            __syncthreads();
            gload_guarded(nfull);
            lstore(0);
            __syncthreads();
            compute(0);
            if (kWrite) mean_store_guarded(mean_piece(0), nfull);
        }
    };
    if (kMean && write_mean) run(std::true_type{});
    else run(std::false_type{});
    flush();

    // Tile entry in accumulator register v of lane l: row i = 4*(l/16) + v, column j = l%16.
    // Wavefronts add their tiles (their column quarters) into LDS one after the other.
    double *comb = reinterpret_cast<double *>(stage);
    for (int w = 0; w < kWaves; ++w) {
        __syncthreads();
        if (wave == w) {
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int e = t * kGramTile + (4 * sub + v) * 16 + l16;
                    if (w == 0) comb[e] = tot[t][v];
                    else comb[e] += tot[t][v];
                }
        }
    }
    __syncthreads();
    double *out = a.ws + vblock * kGramMaxTiles * kGramTile;
    for (int e = tid; e < NT * kGramTile; e += kBlock) out[e] = comb[e];
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
