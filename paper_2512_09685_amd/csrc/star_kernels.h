// Launch interface between the C-ABI layer (host) and the gfx950 kernels.
#pragma once

#include <hip/hip_runtime_api.h>

#include <cstdint>

#include "star.h"

namespace star {

constexpr int kBlock = 256;          // threads per workgroup: 4 wave64
constexpr int kFewRows = 6;          // up to this many rows the Gram matrix behind the norms stays in vector registers
constexpr int kGridCap = 1024;       // most workgroups a norm-reducing launch uses (sizes the partial buffer)

// Work queue of one launch: the next tile nobody has claimed yet and the number of workgroups that
// have left the kernel.  16 bytes of device memory, all zero between launches: the last workgroup
// to leave clears it, so no fill is needed before the next launch (stream order does the rest).
struct TileQueue {
    unsigned long long next;
    unsigned int done;
    unsigned int pad;
};

// Tiles handed to a workgroup per claim.  Never a power of two: with 2, 4 or 8 tiles every claim starts
// on an 8/16/32 KB boundary of every row, all workgroups then hit the same memory channels at the same
// moments, and the update measured 5-8 % slower than with 3.  Light tiles (few rows: a thread moves less
// than 96 bytes per tile, state included) are finished so quickly that claims of 3 come faster than the
// one counter serves them (it sustains about 80 M atomics/s); 5 measured 15-40 % faster there (one fp32
// row and the state: 0.37 against 0.48 ms on 110 M elements), 6, 7 and 9 slower again.
constexpr int kClaim = 3;
constexpr int kClaimLight = 5;
// What a launch does to memory decides how much work a claim should cover.  A claim's round trip to the
// counter is hidden only if the workgroup has several microseconds of tiles left when it asks, and a
// kernel that only reads gets through a tile much faster than one that also writes the state back:
//   Update   reads the rows, reads and writes the state: 3 tiles, 5 when light (see above), 2 when very heavy;
//   ReadOnly the norms alone, the Gram matrix: about 200 KB per claim (16 bf16 rows, 32 KB a tile: 6 or 7
//            tiles run 0.83-0.86 of the HBM peak against 0.68-0.71 with 3; 8 bf16 rows: 13 tiles 0.82
//            against 0.61 with 5; 16 fp32 rows stay at 3);
//   Reduce   reads the rows, writes one output row per group: about 140 KB per claim (16 bf16 rows: 4
//            tiles 0.75 against 0.71 with 3; 16 fp32 rows: 2 tiles 0.74 against 0.72).
enum class Traffic { Update, ReadOnly, Reduce };
inline int queue_claim(int thread_bytes, Traffic traffic = Traffic::Update) {
    const int tile = (thread_bytes < 1 ? 1 : thread_bytes) * kBlock;
    if (traffic == Traffic::ReadOnly) {
        const int c = (200 * 1024 + tile / 2) / tile;
        return c < 3 ? 3 : (c > 16 ? 16 : c);
    }
    if (traffic == Traffic::Reduce) {
        const int c = (140 * 1024 + tile / 2) / tile;
        return c < 2 ? 2 : (c > 9 ? 9 : c);
    }
    // very heavy tiles (20 to 32 fp32 rows: 90-140 KB a tile): two tiles a claim, 2-4 % ahead of three
    if (thread_bytes >= 320) return 2;
    return thread_bytes < 96 ? kClaimLight : kClaim;
}

// Shards shorter than this many elements keep the static mapping (and need no queue): with few tiles
// per workgroup the claims' round trips show (1 Mi elements: 15 against 7.5 us); from 16 Mi on the
// queue order wins (+12 % with 8 fp32 rows).
constexpr int64_t kQueueMinElements = 16 << 20;
// Shards shorter than this take their norms from direct sums whatever the stream (see decide()).
constexpr int64_t kTinyShardElements = 4096;

// First round of claims (see for_each_claimed_tile): workgroup b of G gets 1 + b % claim tiles, laid out
// one after the other from tile 0; the queue's counter hands out the tiles from `base` on.
// A negative `claim` is the short-shard form: first claims that split all `ntile` tiles evenly between
// the workgroups (consecutive tiles each, counts differ by at most one), so that nothing is left for
// the counter and no workgroup waits for it.  With 2 to 8 tiles per workgroup the unequal first claims
// and their granularity would leave some workgroups with twice the work of others, and a kernel of a
// few microseconds would spend one or two of them on the counter's round trips.
struct FirstClaim {
    int64_t t0;                // first tile of the workgroup's first claim
    int n;                     // tiles in it
    unsigned long long base;   // tiles covered by all first claims together
};
__host__ __device__ inline FirstClaim first_claim_of(const int64_t b, const int64_t G, const int claim,
                                                     const int64_t ntile = 0) {
    if (claim < 0) {   // short shard: the tiles split evenly, workgroup b gets [b ntile / G, (b+1) ntile / G)
        FirstClaim e;
        e.t0 = b * ntile / G;
        e.n = (int)((b + 1) * ntile / G - e.t0);
        e.base = (unsigned long long)ntile;
        return e;
    }
    const int64_t per_group = (int64_t)claim * (claim + 1) / 2;   // tiles taken by `claim` consecutive workgroups
    const int64_t r = b % claim, rg = G % claim;
    FirstClaim f;
    f.t0 = (b / claim) * per_group + r * (r + 1) / 2;
    f.n = (int)r + 1;
    f.base = (unsigned long long)((G / claim) * per_group + rg * (rg + 1) / 2);
    return f;
}

struct RowPtrs {
    const void* p[STAR_MAX_WORKERS];
};

// Coefficients of the collapsed map, passed by value in the kernel arguments
// so that they live in scalar registers:
//   p' = p + (dp*p + m01*v + sum_w b0[w] g_w),   v' = m10*p + m11*v + sum_w b1[w] g_w
struct AffCoef {
    float dp, m01, m10, m11;
    float b0[STAR_MAX_WORKERS];
    float b1[STAR_MAX_WORKERS];
};

// Row counts the kernels are instantiated for; a plan with Wc rows runs on
// padded_rows(Wc) >= Wc rows, the extra ones carrying zero coefficients.
int padded_rows(int Wc);

// Small group tables travel in the kernel arguments instead of through a
// host-to-device copy: a call with one or a few updates (the un-queued
// parameter-server case) is then a single enqueue.
constexpr int kInlineUpdates = 32;
constexpr int kInlineCoef = 256;
struct InlineTables {
    float coef[kInlineCoef];        // [U][Wp]
    float lr[kInlineUpdates];
    uint32_t mask[kInlineUpdates];
    void* out[kInlineUpdates];      // output rows (aggregation only)
};
inline bool tables_fit_inline(int U, int Wp) { return U <= kInlineUpdates && U * Wp <= kInlineCoef; }

struct SeqArgs {
    float* params;
    float* momentum;
    RowPtrs rows;
    const float* coef;     // device [U][Wp], or null: the tables are in `inl`
    const float* lr;       // device [U]
    const uint32_t* mask;  // device [U]
    const InlineTables* inl;  // host; used when coef is null
    const AffCoef* cf;     // host, or null; not null: the update is applied once, as this map (17-32 fp32 rows, update + norms)
    int32_t U;             // updates in this launch
    float mu, wd;
    int64_t P;
    int32_t vec_ok;        // all buffers 16-byte aligned
    void* publish;         // device copy of the new params (P elements), or null
    int32_t publish_dtype; // star_dtype of that copy
    double* partials;      // device [U][grid] sums of gbar^2 per block (norms only)
    TileQueue* queue;      // device, zeroed; null: fixed assignment of tiles to workgroups
};

// Which launches take their tiles from the queue when the caller hands one in (the matrix-core kernel
// always does): the step-by-step kernel for one or two updates (longer streams are bound by arithmetic
// and keep the fixed assignment with as many waves as fit), the collapsed one unless it carries the
// register-heavy Gram accumulators of more than kFewRows rows.
inline bool seq_takes_queue(int updates_in_launch) { return updates_in_launch <= 2; }
// Collapsed update with direct norms (step-by-step kernel's norm walk): for 17 to 32 fp32 rows, when the
// stream's direct norm sums cost at most this many multiply-adds per element.  Measured against the Gram
// matrix on the matrix cores, 2 Mi and 64 Mi elements, 6 to 16 updates: the walk wins by 5-14 % up to about
// 130 / 145 / 160 / 175 multiply-adds with 20 / 24 / 28 / 32 rows and loses beyond (at twice that by a third);
// the limit grows with the rows because the matrix-core kernel's time does.
inline double direct_norm_fma_limit(int Wp) { return 4.0 * Wp + 48.0; }
// Which Gram launches of the collapsed kernel use the few-rows form (double fold slots in LDS after every
// chunk, tiles from the queue on long shards): up to kFewRows rows -- except the Gram matrix alone on exactly
// kFewRows fp32 rows, whose 21 slot updates per chunk are not hidden by 96 bytes of loads (32 to 96 Mi
// elements: 0.57-0.65 of the HBM peak, against 0.82 with 5 rows and 0.85 with 7); that one takes the form
// of the larger row counts (fp32 slots folded every kGramFold tiles, fixed assignment).
constexpr bool gram_few_rows_form(int Wp, bool f32_rows, bool update) {
    return Wp <= kFewRows && !(Wp == kFewRows && f32_rows && !update);
}
inline bool aff_takes_queue(bool gram, int Wp, bool f32_rows, bool update) {
    return !gram || gram_few_rows_form(Wp, f32_rows, update);
}

// Largest number of updates one launch of the step-by-step kernel accepts
// (bounded by the LDS tables and, with norms, the per-thread accumulators).
int seq_max_updates(int Wp, bool norms);

// Step-by-step evaluation.  Returns the grid used in *grid_out (needed to
// reduce the partials).  grid_cap bounds it.
hipError_t launch_seq(int Wp, int dtype, bool update, bool norms, const SeqArgs& a, int num_cu, int grid_cap,
                      int* grid_out, hipStream_t s);

struct AffArgs {
    float* params;
    float* momentum;
    RowPtrs rows;
    AffCoef cf;
    int64_t P;
    int32_t vec_ok;
    void* publish;          // device copy of the new params (P elements), or null
    int32_t publish_dtype;  // star_dtype of that copy
    double* partials;  // device [Wp(Wp+1)/2][grid] pairwise-product sums per block (gram only)
    TileQueue* queue;  // device, zeroed; null: fixed assignment of tiles to workgroups (not for the matrix-core kernel)
};

// Collapsed evaluation, optionally accumulating the Gram matrix of the rows.
hipError_t launch_affine(int Wp, int dtype, bool update, bool gram, const AffArgs& a, int num_cu, int grid_cap,
                         int* grid_out, hipStream_t s);

// The same with the Gram matrix formed on the matrix cores (any Wp up to 32; `gram` is implied).
hipError_t launch_affine_mfma(int Wp, int dtype, bool update, const AffArgs& a, int num_cu, int grid_cap,
                              int* grid_out, hipStream_t s);

// out[e] = sum_b partials[e*grid + b] in a fixed order; sums_out (double) and
// sqrt_out (float, square root of the sum) are each optional.
hipError_t launch_reduce(const double* partials, int n_out, int grid, double* sums_out, float* sqrt_out,
                         hipStream_t s);

// norms_out[u] = sqrt( c_u^T Gamma c_u ), Gamma upper-triangular packed [Wp(Wp+1)/2], coef [U][Wp] doubles.
hipError_t launch_gram_norms(const double* gamma, const double* coef, int U, int Wp, float* norms_out,
                             hipStream_t s);

// Packed upper triangle over Wp rows [Wp(Wp+1)/2] -> full symmetric [W][W], W <= Wp (all zero when gamma is null).
hipError_t launch_gram_unpack(const double* gamma, int Wp, int W, double* out, hipStream_t s);

hipError_t launch_fill(float* dst, int64_t n, float value, hipStream_t s);

// ---- the fixed device workspace of the entry point that allocates nothing
// One array of kScratchBytes per GPU, part of the library's device code (no hipMalloc behind it):
//   [0, 256)                                   the tile queue
//   [256, 256 + kScratchTableBytes)            group tables
//   [256 + kScratchTableBytes, kScratchBytes)  per-workgroup partial sums and the reduced Gram matrix
constexpr int kScratchMaxUpdates = 256;                       // longest stream that entry point accepts
constexpr size_t kScratchTableBytes = 128 * 1024;             // tables of 256 updates over 32 rows: 100 KB
constexpr size_t kScratchPartialDoubles = 528 * (size_t)kGridCap + 528;   // Gram partials of 32 rows
constexpr size_t kScratchBytes = 4608 * 1024;                 // 4.5 MiB
static_assert(256 + kScratchTableBytes + kScratchPartialDoubles * sizeof(double) <= kScratchBytes,
              "the three parts fit in the array");

// Device address of the array on the current device (resolved once per device, then cached).
hipError_t scratch_address(void** out);

// dst[0..bytes) = src[0..bytes): host data carried to the device in kernel arguments, a few KB per
// launch -- no copy engine, no staging buffer, nothing allocated.  dst 16-byte aligned.
hipError_t launch_upload(void* dst_dev, const void* src_host, size_t bytes, hipStream_t s);

// Puts a tile queue back to "no tile claimed, nobody left".
hipError_t launch_queue_clear(TileQueue* q, hipStream_t s);

// ---- aggregation without the optimizer step (star_group_reduce)
struct ReduceArgs {
    RowPtrs rows;
    const float* coef;       // device [U][Wp], or null: the tables are in `inl`
    const uint32_t* mask;    // device [U]
    void* const* out;        // device array of U output row pointers
    const InlineTables* inl; // host; used when coef is null
    int32_t U;               // groups in this launch
    int32_t out_dtype;       // star_dtype of the outputs
    int64_t P;
    int32_t vec_ok;          // every row and every output 16-byte aligned
    int32_t norms;           // also accumulate sum of squares per group
    double* partials;        // device [U][grid] (norms only)
    TileQueue* queue;        // device, zeroed; null: fixed assignment of tiles to workgroups
};

int reduce_max_updates(int Wp, bool norms);

hipError_t launch_group_reduce(int Wp, int dtype, const ReduceArgs& a, int num_cu, int grid_cap, int* grid_out,
                               hipStream_t s);

}  // namespace star
