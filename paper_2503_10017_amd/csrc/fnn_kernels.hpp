// Host-side declarations of the kernel launchers that the C entry points are built from.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <mutex>

#include "../../include/fnn.h"

namespace fnn {

typedef unsigned long long u64;

// A launch shape that depends on the device (how many workgroups of a kernel it holds, how much
// LDS it grants): computed once per device by the first call made with that device current, under
// a lock, so that host threads and devices may make their first calls concurrently.
struct DeviceCache {
    static constexpr int MAX_DEVICES = 64;
    std::mutex mu;
    bool filled[MAX_DEVICES] = {};
    long long value[MAX_DEVICES] = {};
    // compute(device) returns the value, negative = failed (reported, not cached)
    template <typename F>
    long long get(F&& compute) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess) return -1;
        if (dev < 0 || dev >= MAX_DEVICES) return compute(dev);
        std::lock_guard<std::mutex> lock(mu);
        if (!filled[dev]) {
            const long long v = compute(dev);
            if (v < 0) return v;
            value[dev] = v;
            filled[dev] = true;
        }
        return value[dev];
    }
};

// Padded channel count of a prepared map: 16-bit formats use one K=16 matrix instruction,
// a K=16 and a K=8 one (24 channels, no padding for the paper's d = 24) or two K=16 ones;
// fp32 uses K=2 instructions on channel pairs.
constexpr int padded_d(int d, int compute) {
    if (compute == FNN_F32) return (d + 7) / 8 * 8;
    return d <= 16 ? 16 : (d <= 24 ? 24 : (d + 15) / 16 * 16);
}
// Channels of a prepared row that carry data: the descriptor plus, for the L2 score, the
// norm terms and their unit partners (two 16-bit halves each, or one fp32 value each).
inline int l2_extra_channels(int compute) { return compute == FNN_F32 ? 2 : 4; }
// ... or, for the two-term fp16 representation (FNN_FLAG_SPLIT), three copies of the descriptor's
// channels: [hi, hi, lo] in image 1 and [hi, lo, hi] in image 2.
inline int effective_d(int d, int compute, bool l2, bool split = false) {
    return split ? 3 * d : (l2 ? d + l2_extra_channels(compute) : d);
}
constexpr int MAX_ROW_CHANNELS = 96;  // widest prepared row (16-bit formats; fp32 rows hold at most 32)
inline int elem_size(int dtype) { return dtype == FNN_F32 ? 4 : 2; }
inline int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

// ---- prepare: convert / pad the caller's maps into the workspace ------------------------
struct PrepSide {
    const void* src[FNN_MAX_BATCH];  // device pointers, one per pair
    int64_t n;                       // valid pixels
    int64_t n_pad;                   // rows written per pair (multiple of 32; rows >= n are zero)
    int32_t segment_major;           // 1: rows are stored in the dense kernel's segment-major order
    int64_t row_stride;              // source row stride, elements
    int32_t dtype;                   // source storage format
    int32_t second_image;            // L2 score: 0 = rows [x, 1.., -|x|^2/2..], 1 = rows [x, -|x|^2/2.., 1..]
    void* dst;                       // [batch][n_pad][dp] in the compute format
};
// Small initialisations that ride along with the prepare launch instead of costing launches
// of their own: clearing key tables / bitmaps, and step 1 of the FastNN iteration (U^0).
struct PrepExtra {
    u64* zero_ptr;          // range of 64-bit words to clear (NULL: none)
    int64_t zero_count;
    const int32_t* seeds;   // [batch][n_seeds] (NULL: no seed initialisation)
    int32_t* cur_u;         // [batch][n_seeds] <- seeds
    int32_t* seed_id;       // [batch][n_seeds] <- 0, 1, 2, ...
    int32_t* n_active;      // [batch] <- n_seeds
    int32_t n_seeds;
};
struct PrepArgs {
    PrepExtra extra;
    PrepSide side[2];
    int32_t n_sides;  // 1 or 2
    int32_t batch;
    int32_t d;
    int32_t dp;
    int32_t compute;
    int32_t normalize;  // divide every descriptor by its Euclidean norm first (FNN_FLAG_NORMALIZE)
    int32_t l2;         // append the norm channels of the L2 score (FNN_FLAG_L2)
    int32_t split;      // rows hold the two-term fp16 representation (FNN_FLAG_SPLIT); d is the source's
};
hipError_t launch_prep(const PrepArgs& a, hipStream_t s);
// "no neighbour": idx = -1, score = -inf (score may be NULL)
hipError_t launch_fill_i32f32(int32_t* idx, float* score, int64_t count, hipStream_t s);

// ---- one-directional search ------------------------------------------------------------
struct SearchArgs {
    const char* src;        // prepared map the queries are rows of, [batch][*][dp]
    int64_t src_bstride;    // bytes per pair
    int32_t src_rows;       // rows per pair in src (row indices are clamped to it)
    const int32_t* q_idx;   // [batch][nq] rows of src, or NULL
    const u64* q_keys;      // [batch][nq] keys whose index field names the row, or NULL
    const int32_t* nq_active;  // [batch] or NULL
    int32_t nq;
    const char* tgt;        // prepared candidate map [batch][m_tiles*32][dp]
    int64_t tgt_bstride;
    int32_t m;              // valid candidates
    int32_t m_tiles;
    u64* out_keys;          // [batch][nq], must hold 0 (or earlier partial results)
};
// Pass 1: out_keys receive (best score, tile of 32 candidates holding it).
hipError_t launch_search(const SearchArgs& a, int batch, int compute, int dp, hipStream_t s);

// The first searches of a call whose maps are still the caller's fp32 arrays (24 channels, a
// 16-bit compute format, every query live): the candidates are read from the caller's map,
// rounded on the way, staged through LDS once per workgroup, and written to the prepared map
// `s.tgt` as a by-product, so no separate prepare pass over that map is needed.
struct RawMaps {
    const float* map[FNN_MAX_BATCH];  // caller's map of every pair (16-byte aligned rows)
    int64_t row_stride;               // floats per row (a multiple of 4)
};
struct FirstSearchArgs {
    SearchArgs s;      // s.tgt: prepared candidate map to WRITE; s.nq_active is ignored (all nq queries are live)
    RawMaps raw_tgt;   // candidates
    RawMaps raw_src;   // queries, when raw_queries != 0 (else they are rows of the prepared map s.src)
    int32_t raw_queries;
};
// true if this shape should take the staged first search: enough queries to fill the workgroups'
// four waves and, with `batch` pairs sharing the device, chunks of m candidates long enough
bool first_search_applies(int64_t nq, int64_t m, int batch);
hipError_t launch_search_first(const FirstSearchArgs& a, int batch, int compute, hipStream_t s);
// launch_resolve with the queries still in the caller's fp32 map
hipError_t launch_resolve_raw(const FirstSearchArgs& a, int batch, int compute, int32_t* out_idx, float* out_score, hipStream_t s);
// Pass 2: out_keys become (best score, lowest candidate index); optionally also stored to
// out_idx / out_score (either may be NULL).  Queries without any candidate get -1 / -inf.
hipError_t launch_resolve(const SearchArgs& a, int batch, int compute, int dp, int32_t* out_idx, float* out_score,
                          hipStream_t s);

// ---- the paper's blocked schedules with a materialised score block (contrast experiment) ----
struct BlockedArgs {
    const char* src;        // prepared query map (one pair)
    int32_t src_rows;
    const int32_t* q_idx;   // [nq] or NULL
    int32_t nq;
    const char* tgt;        // prepared candidate map
    int32_t m;
    float* dists;           // [block_rows][ld] score block in device memory
    int64_t ld;             // columns of the score block (multiple of 32)
    int32_t* out_idx;       // [nq]
    float* out_score;       // [nq] (required: it holds the running best between blocks)
    int32_t half_accumulate;  // FNN_FLAG_HALF_ACCUMULATE: fp16 products and fp16 sums on the vector ALU
};
// block_cols == 0: Algorithm 2 (whole B per block of A); otherwise Algorithm 1 (double loop).
hipError_t run_blocked(const BlockedArgs& a, int compute, int d, int dp, int block_rows, int block_cols, hipStream_t s);

// ---- reciprocal iteration bookkeeping ----------------------------------------------------
struct RecipState {
    int32_t* cur_u[2];   // [batch][n_seeds] ping-pong: U^t of the seeds still moving
    int32_t* seed_id[2]; // [batch][n_seeds] which seed sits in each slot
    int32_t* n_active;   // [batch]
    u64* keys_f;         // [batch][n_seeds] result of the search into image 2 (V^t)
    u64* keys_b;         // [batch][n_seeds] result of the search back into image 1 (U^{t+1})
    uint32_t* bitmap;    // [batch][n_words] one bit per pixel of image 1, for the final sort
    int32_t* word_rank;  // [batch][n_words] rank of the first bit of each bitmap word
    int64_t n_words;
};
// mode 0: ordinary iteration t; 1: last iteration (survivors are reported as unconverged);
// 2: no iteration at all (max_iter == 0): every seed is reported unconverged with (U^0, V^0).
hipError_t launch_recip_step(const RecipState& st, int which, int32_t n_seeds, int batch, int t, int mode,
                             int32_t* seed_i, int32_t* seed_j, int32_t* seed_iter, hipStream_t s);
hipError_t launch_recip_dedup(const RecipState& st, int32_t n_seeds, int batch,
                              const int32_t* seed_i, const int32_t* seed_j, const int32_t* seed_iter,
                              int32_t* pairs, int32_t* n_pairs, hipStream_t s);

// ---- dense mutual nearest neighbours -----------------------------------------------------
constexpr int DENSE_J = 4;      // candidate tiles resident per wave
constexpr int DENSE_WAVES = 4;  // waves per workgroup
constexpr int DENSE_TILES_PER_GROUP = DENSE_J * DENSE_WAVES;
struct DenseArgs {
    const char* d1;        // prepared queries, segment-major, [batch][n_sb*32*DENSE_S][dp]
    int64_t d1_bstride;
    const char* d2;        // prepared candidates, natural order, [batch][m_tiles*32][dp]
    int64_t d2_bstride;
    int32_t n, m;
    int32_t n_sb;          // super-blocks of queries (32*DENSE_S pixels each)
    int32_t m_tiles;       // 32-pixel tiles of candidates
    u64* row_keys;         // [batch][n] zero-initialised; (best score, group of DENSE_J tiles)
    u64* col_keys;         // [batch][m] zero-initialised; (best score, run of DENSE_S queries)
    int32_t sb_per_wg;     // super-blocks swept by one workgroup
    int32_t groups_per_wg; // candidate groups (DENSE_WAVES x DENSE_J tiles) per workgroup
    // pass 2: pixels bucketed by their winning unit
    int32_t row_units;     // groups of DENSE_J candidate tiles
    int32_t col_units;     // runs of DENSE_S queries (n_sb * 32)
    int64_t rows_cap;      // list positions for the queries: round_up(n, 32) + 32 * row_units
    int64_t cols_cap;      // list positions for the candidates: round_up(m, 32) + 32 * col_units
    int32_t* unit_counts;  // [batch][row_units + col_units] zero-initialised
    int32_t* unit_cursor;  // [batch][row_units + col_units] next free list position (after the fill: end) of a bucket
    int32_t* lists;        // [batch][rows_cap + cols_cap] pixels grouped by unit, buckets start on multiples of 32
    int32_t* chunk_unit;   // [batch][(rows_cap + cols_cap) / 32] unit of every chunk of 32 list positions
    int32_t* chunk_totals; // [batch][2] chunks in use per side
};
// Pass 1 (both maxima with coarse locations) and pass 2 (exact indices and scores into
// nn12/s12/nn21/s21; s12, s21 may be NULL).
hipError_t launch_dense(const DenseArgs& a, int batch, int compute, int dp, int32_t* nn12, float* s12, int32_t* nn21,
                        float* s21, hipStream_t s);

struct DenseFinalArgs {
    int32_t n, m;
    const int32_t* nn12;
    const int32_t* nn21;
    int32_t* pairs;       // [batch][min(n,m)][2]
    int32_t* n_pairs;     // [batch]
    int32_t* block_counts;  // [batch][ceil(max(n,m)/1024)] scratch
};
hipError_t launch_dense_final(const DenseFinalArgs& a, int batch, hipStream_t s);

// ---- matches as pixel coordinates, confidence filter -------------------------------------
struct PixelArgs {
    const int32_t* pairs;    // [batch][max_pairs][2] flat pixel ids (i in image 1, j in image 2)
    const int32_t* n_pairs;  // [batch]
    int64_t max_pairs;
    int64_t n, m;            // pixels per image
    int32_t width1, width2;
    const float* conf1;      // [batch][n] or NULL
    const float* conf2;      // [batch][m] or NULL
    float min_conf1, min_conf2;
    int32_t* out_xy;         // [batch][max_pairs][4]
    int32_t* out_count;      // [batch]
};
hipError_t launch_pairs_to_pixels(const PixelArgs& a, int batch, hipStream_t s);

}  // namespace fnn
