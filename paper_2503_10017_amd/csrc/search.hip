// One-directional nearest-neighbour search: the single loop of Algorithm 2 ("FastNN-Lite",
// section 3.4.3) with its distance block fused away.  Each wave keeps a few 32-query blocks
// resident in registers, streams candidate tiles past them, forms every 32x32 block of
// scores with matrix instructions (fp32 accumulation, Algorithm 3) and folds it at once into
// a per-query running best, so no score ever leaves the register file and memory traffic is
// one pass over the candidate map per resident query group.
//
// The search runs in two passes: pass 1 finds, per query, the best score and the tile of 32
// candidates that holds it, at roughly 0.6 vector operations per score; pass 2 recomputes
// that one tile per query to name the lowest candidate index attaining the score.
//
// Work split (decided on the device from the live query count, so the host never needs to
// read it back): the queries form row groups of G*R*32, the candidate tiles are cut into
// chunks, one wave takes one (row group, chunk) unit -- every candidate tile it loads meets
// G groups of R query blocks, a group past the live queries is skipped -- and merges its
// result into the packed keys with a 64-bit atomic max (score first, lowest index on ties).
#include <type_traits>

#include "fnn_device.hpp"
#include "fnn_kernels.hpp"
#include "trace.hpp"

namespace fnn {

constexpr int SEARCH_R = 4;           // 32-query blocks whose products are in flight together
// A wave keeps G groups of R query blocks resident (G = 1, 2 or 4, chosen per launch), so every
// candidate tile it loads meets G*R query blocks.
constexpr int SEARCH_WIDE_MIN_TILES = 128;  // a wave takes more groups only while its chunk stays at least this long
// Shortest chunk worth a wave.  Every chunk ends in 64-bit atomic max operations on the keys of
// the live queries, and atomics on one address are served one after the other (about 13 ns
// each here): with few live queries and few pairs, 4-tile chunks and one atomic per wave meant
// 1536 of them per key and 21-34 us per search of a 512x384 map.  8-tile chunks together with
// the workgroup-level merge in the kernel take 8-12 us (4 and 16 measured slower).
constexpr int SEARCH_MIN_TILES = 8;
constexpr int SEARCH_WAVES = 4;       // waves per workgroup
constexpr int SEARCH_P = 4;           // candidate tiles in flight per wave

__device__ __forceinline__ float max3(float a, float b, float c) { return __builtin_fmaxf(__builtin_fmaxf(a, b), c); }

// Largest of `seed` and the 16 scores of one result fragment: eight 3-input max operations.
__device__ __forceinline__ float fold16(float seed, const f32x16& x) {
    const float t0 = max3(x[0], x[1], x[2]);
    const float t1 = max3(x[3], x[4], x[5]);
    const float t2 = max3(x[6], x[7], x[8]);
    const float t3 = max3(x[9], x[10], x[11]);
    const float t4 = max3(x[12], x[13], x[14]);
    const float t5 = max3(t0, t1, t2);
    const float t6 = max3(t3, t4, x[15]);
    return max3(seed, t5, t6);
}

__device__ __forceinline__ int64_t query_row(const SearchArgs& a, int64_t qbase, int slot) {
    int64_t row;
    if (a.q_keys) row = (int64_t)(0xFFFFFFFFu - (uint32_t)(a.q_keys[qbase + slot] & 0xFFFFFFFFull));
    else if (a.q_idx) row = a.q_idx[qbase + slot];
    else row = slot;
    return min(max(row, (int64_t)0), (int64_t)a.src_rows - 1);  // never read outside the map
}

// One unit of pass 1: the query blocks of slots [slot0, slot0 + 32*R*G) against the candidate
// tiles [t0, t1).  Per query the best score and the 32-candidate TILE that holds it: a lane only
// keeps a running maximum (3-input max) and, once per tile, notes the tile when the maximum
// rose -- strictly, so the lowest tile wins among equal scores.  The key carries the tile
// number in its index field; pass 2 turns it into the candidate index.  With `combine` the
// keys go to the workgroup's table in LDS (slot0 is 0 then), else to the global table.
// P candidate tiles are always in flight towards the registers; a slot is refilled as soon
// as its tile has been handed to the matrix cores.  EXACT: loads past the end of the chunk are
// skipped (for chunks that may be shorter than the ring); otherwise they re-read the chunk's
// last tile, which keeps the loop free of branches around the loads.
template <int CT, int DP, int R, int P, int G, bool EXACT>
__device__ __forceinline__ void search_unit(const SearchArgs& a, const char* src, const char* tgt, int64_t qbase,
                                            int n_act, int slot0, int t0, int t1, bool combine, u64* wg_keys, int c, int h) {
    using O = Ops<CT, DP>;
    using Frag = typename O::Frag;
    const float ninf = -__builtin_inff();
    // The first P loads are issued before the (dependent) query fetch so that both latencies
    // overlap.
    Frag ring[P];
#pragma unroll
    for (int p = 0; p < P; ++p) {
        if (!EXACT) ring[p] = O::load_tile(tgt + (int64_t)min(t0 + p, t1 - 1) * (32 * O::ROW_BYTES), c, h);
        else if (p == 0 || t0 + p < t1)  // uniform; a slot past the end is never used
            ring[p] = O::load_tile(tgt + (int64_t)(t0 + p) * (32 * O::ROW_BYTES), c, h);
    }

    // blocks past the live queries of the last row group are computed on row 0 and dropped;
    // a whole group of R blocks past them is skipped
    Frag q[G][R];
    float best[G][R];
    int best_tile[G][R];
    bool live[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        live[g] = slot0 + g * 32 * R < n_act;  // uniform
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int slot = slot0 + (g * R + r) * 32 + c;
            const int64_t row = slot < n_act ? query_row(a, qbase, slot) : 0;
            q[g][r] = O::load(src + row * O::ROW_BYTES, h);
            best[g][r] = ninf;
            best_tile[g][r] = 0x7FFFFFFF;
        }
    }

    for (int tb = t0; tb < t1; tb += P) {
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const int t = tb + p;
            if (t < t1) {  // uniform
                const Frag cur = ring[p];
                if (!EXACT) ring[p] = O::load_tile(tgt + (int64_t)min(t + P, t1 - 1) * (32 * O::ROW_BYTES), c, h);
                else if (t + P < t1) ring[p] = O::load_tile(tgt + (int64_t)(t + P) * (32 * O::ROW_BYTES), c, h);
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    if (live[g]) {
                        f32x16 acc[R];
#pragma unroll
                        for (int r = 0; r < R; ++r) acc[r] = O::mma(cur, q[g][r]);
                        if (t * 32 + 32 > a.m) {  // only the last tile of the map can be partial
                            // candidate t*32 + tile_row(v, h) lies past the map; tested against one
                            // lane-dependent bound so that no per-register constants stay resident
                            const int bound = a.m - t * 32 - 4 * h;
#pragma unroll
                            for (int r = 0; r < R; ++r)
#pragma unroll
                                for (int v = 0; v < 16; ++v)
                                    if (tile_row(v, 0) >= bound) acc[r][v] = ninf;
                        }
#pragma unroll
                        for (int r = 0; r < R; ++r) {
                            const float top = fold16(best[g][r], acc[r]);
                            if (top > best[g][r]) best_tile[g][r] = t;
                            best[g][r] = top;
                        }
                    }
                }
            }
        }
    }

#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float ob = __shfl_xor(best[g][r], 32);
            const int ot = __shfl_xor(best_tile[g][r], 32);
            if (ob > best[g][r] || (ob == best[g][r] && ot < best_tile[g][r])) {
                best[g][r] = ob;
                best_tile[g][r] = ot;
            }
            const int slot = slot0 + (g * R + r) * 32 + c;
            if (h == 0 && slot < n_act) {
                const u64 key = pack_key(best[g][r], best_tile[g][r]);
                if (combine) atomicMax(&wg_keys[slot], key);
                else atomicMax(&a.out_keys[qbase + slot], key);
            }
        }
}

// Candidate tiles a wave keeps in flight when a pair has at most 32*R live queries (NB = blocks
// that hold one).  Such a search is bound by streaming the candidate map, not by arithmetic,
// and what limits a stream is the number of bytes on their way: the registers that the resident
// query blocks of the wide variants would occupy hold a longer ring instead.  Rows wider than
// 96 bytes keep the ordinary ring (their fragments leave no room).
template <int CT, int DP, int NB>
constexpr int stream_ring() {
    constexpr int frag_regs = Ops<CT, DP>::ROW_BYTES / 8;
    constexpr int fit = (NB <= 2 ? 96 : 72) / frag_regs;
    constexpr int base = Ops<CT, DP>::ROW_BYTES > 128 ? 2 : SEARCH_P;
    return frag_regs > 12 ? base : (fit > 16 ? 16 : (fit < base ? base : fit));
}

// Pass 1 kernel.  (waves_per_eu >= 2 caps the kernel at 256 registers, which lets the matrix
// instructions write their results straight into ordinary vector registers.)
template <int CT, int DP, int R, int P, int G>
__global__ __launch_bounds__(SEARCH_WAVES * 64) __attribute__((amdgpu_waves_per_eu(2)))
void search_kernel(SearchArgs a) {
    const int lane = threadIdx.x & 63, c = lane & 31, h = lane >> 5;
    // Workgroups are dealt to the 8 XCDs round-robin by their linear id, and each XCD has
    // its own L2.  Renumber them so that every XCD owns one contiguous run of (pair, unit)
    // work: the row groups that sweep the same candidate chunk then share one L2 instead
    // of fetching the chunk from HBM once per XCD.
    const int n_wgs = gridDim.x * gridDim.y;
    int wg = blockIdx.y * gridDim.x + blockIdx.x;
    if ((n_wgs & 7) == 0) wg = (wg & 7) * (n_wgs >> 3) + (wg >> 3);
    const int b = wg / gridDim.x;
    const int wave = (wg % gridDim.x) * SEARCH_WAVES + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n_waves = gridDim.x * SEARCH_WAVES;

    int n_act = a.nq;
    if (a.nq_active) n_act = min(max(a.nq_active[b], 0), a.nq);
    if (n_act <= 0 || a.m_tiles <= 0) return;

    const int row_groups = (n_act + 32 * R * G - 1) / (32 * R * G);
    int chunks = max(1, n_waves / row_groups);
    int tiles_per_chunk = max((a.m_tiles + chunks - 1) / chunks, SEARCH_MIN_TILES);
    chunks = (a.m_tiles + tiles_per_chunk - 1) / tiles_per_chunk;

    const char* src = a.src + (int64_t)b * a.src_bstride;
    const char* tgt = a.tgt + (int64_t)b * a.tgt_bstride;
    const int64_t qbase = (int64_t)b * a.nq;

    // With a single row group every unit of this pair serves the same queries, so the waves of
    // a workgroup first merge their results in LDS and the workgroup sends one atomic per query
    // instead of one per wave: atomics on one address are served serially, and with few live
    // queries that chain is what the search waits for.  (row_groups is the same for the whole
    // workgroup, so the barriers below are uniform.)
    __shared__ u64 wg_keys[32 * R * G];
    const bool combine = row_groups == 1;
    if (combine) {
        for (int i = threadIdx.x; i < 32 * R * G; i += SEARCH_WAVES * 64) wg_keys[i] = 0;
        __syncthreads();
    }

    const int64_t units = (int64_t)row_groups * chunks;
    for (int64_t unit = wave; unit < units; unit += n_waves) {
        const int chunk = (int)(unit / row_groups);
        const int rg = (int)(unit % row_groups);
        const int slot0 = rg * 32 * R * G;
        const int t0 = chunk * tiles_per_chunk;
        const int t1 = min(t0 + tiles_per_chunk, a.m_tiles);
        if (n_act <= 32 * R) {
            // few live queries (one row group, so combine is set): only the blocks that hold a
            // live query are multiplied, and the ring is as long as the registers allow
            if (n_act <= 32)
                search_unit<CT, DP, 1, stream_ring<CT, DP, 1>(), 1, true>(a, src, tgt, qbase, n_act, 0, t0, t1, true, wg_keys, c, h);
            else if (n_act <= 64)
                search_unit<CT, DP, 2, stream_ring<CT, DP, 2>(), 1, true>(a, src, tgt, qbase, n_act, 0, t0, t1, true, wg_keys, c, h);
            else
                search_unit<CT, DP, R, stream_ring<CT, DP, R>(), 1, true>(a, src, tgt, qbase, n_act, 0, t0, t1, true, wg_keys, c, h);
        } else {
            search_unit<CT, DP, R, P, G, false>(a, src, tgt, qbase, n_act, slot0, t0, t1, combine, wg_keys, c, h);
        }
    }
    if (combine) {
        __syncthreads();
        for (int i = threadIdx.x; i < min(n_act, 32 * R * G); i += SEARCH_WAVES * 64) {
            const u64 key = wg_keys[i];
            if (key != 0) atomicMax(&a.out_keys[qbase + i], key);
        }
    }
}

// ---- the first searches of a call, on maps that are not prepared yet -----------------------
// Same arithmetic and same keys as search_kernel, for the case "every query live, candidates
// still in the caller's fp32 map" (the first forward and the first backward search of the
// FastNN iteration).  A workgroup's four waves take four row groups of ONE candidate chunk:
// each turn every wave fetches one 32-pixel tile of the caller's map, rounds it to the compute
// format in registers (the cast of Algorithm 3), puts the fragment into the workgroup's LDS
// ring and -- first row-group quad only -- stores it to the prepared map; after a barrier all
// four waves read the four staged tiles from LDS and multiply them with their resident query
// blocks.  The map is thus read once per quad instead of once per wave, the raw tiles of the
// next two turns are always in flight, and the separate prepare pass over the map disappears.
constexpr int FIRST_G = 3;        // groups of R query blocks per wave: 3072 queries = 8 row groups = 2 quads
constexpr int FIRST_TURN = SEARCH_WAVES;  // tiles staged per turn (one per wave)
constexpr int FIRST_AHEAD = 2;    // turns whose raw tiles are in flight
constexpr int FIRST_MIN_CHUNK = 32;  // tiles a chunk must hold for the staged kernel to be worth its start-up

// A candidate tile on its way to the LDS ring: the 12 fp32 values of the caller's row (RAWT), or
// the fragment of an already prepared map.
template <int CT, bool RAWT>
struct FirstTile {
    using O = Ops<CT, 24>;
    using Pending = std::conditional_t<RAWT, typename O::Raw, typename O::Frag>;
    static __device__ __forceinline__ Pending fetch(const FirstSearchArgs& fa, const char* tgt, int b, int t, int t1, int c, int h) {
        if constexpr (RAWT) {
            const int64_t pixel = (int64_t)t * 32 + c;
            if (t < t1 && pixel < fa.s.m) return O::load_raw(fa.raw_tgt.map[b] + pixel * fa.raw_tgt.row_stride, h);
            return O::zero_raw();  // padding rows of the prepared map are zero
        } else {
            return O::load_tile(tgt + (int64_t)min(t, t1 - 1) * (32 * O::ROW_BYTES), c, h);
        }
    }
    static __device__ __forceinline__ typename O::Frag fragment(const Pending& p) {
        if constexpr (RAWT) return O::round_raw(p);
        else return p;
    }
};

template <int CT, int G, bool RAWT>
__global__ __launch_bounds__(SEARCH_WAVES * 64) __attribute__((amdgpu_waves_per_eu(2)))
void search_first_kernel(FirstSearchArgs fa) {
    using O = Ops<CT, 24>;
    using Frag = typename O::Frag;
    using Tile = FirstTile<CT, RAWT>;
    constexpr int R = SEARCH_R;
    const SearchArgs& a = fa.s;
    __shared__ uint4 stage_lo[2][FIRST_TURN][64];
    __shared__ uint2 stage_hi[2][FIRST_TURN][64];
    const int lane = threadIdx.x & 63, c = lane & 31, h = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // one XCD owns a contiguous run of (pair, unit) work, see search_kernel
    const int n_wgs = gridDim.x * gridDim.y;
    int wg = blockIdx.y * gridDim.x + blockIdx.x;
    if ((n_wgs & 7) == 0) wg = (wg & 7) * (n_wgs >> 3) + (wg >> 3);
    const int b = wg / gridDim.x;
    const int wgi = wg % gridDim.x;
    const int n_act = a.nq;
    if (n_act <= 0 || a.m_tiles <= 0) return;

    const int row_groups = (n_act + 32 * R * G - 1) / (32 * R * G);
    const int quads = (row_groups + SEARCH_WAVES - 1) / SEARCH_WAVES;
    int chunks = max(1, (int)gridDim.x / quads);
    int tiles_per_chunk = (a.m_tiles + chunks - 1) / chunks;
    tiles_per_chunk = (tiles_per_chunk + FIRST_TURN - 1) / FIRST_TURN * FIRST_TURN;
    chunks = (a.m_tiles + tiles_per_chunk - 1) / tiles_per_chunk;

    const char* src = a.src + (int64_t)b * a.src_bstride;
    char* tgt = const_cast<char*>(a.tgt) + (int64_t)b * a.tgt_bstride;
    const int64_t qbase = (int64_t)b * a.nq;
    const float ninf = -__builtin_inff();

    const int units = quads * chunks;
    for (int unit = wgi; unit < units; unit += gridDim.x) {  // uniform in the workgroup
        const int chunk = unit / quads, quad = unit % quads;
        const int slot0 = (quad * SEARCH_WAVES + wave) * 32 * R * G;
        const int t0 = chunk * tiles_per_chunk;
        const int t1 = min(t0 + tiles_per_chunk, a.m_tiles);
        const int n_turns = (t1 - t0 + FIRST_TURN - 1) / FIRST_TURN;

        static_assert(FIRST_AHEAD == 2, "the turn loop below is unrolled by the two ring slots");
        typename Tile::Pending raw[FIRST_AHEAD];
#pragma unroll
        for (int p = 0; p < FIRST_AHEAD; ++p) raw[p] = Tile::fetch(fa, tgt, b, t0 + p * FIRST_TURN + wave, t1, c, h);

        // The running best of a query block lives in two registers that trade places from tile to
        // tile (the tiles of a turn are unrolled, so which one is current is known at compile time):
        // the fold writes the new best beside the old one, which the "did it rise" test still needs,
        // instead of into a scratch register that then has to be copied.
        static_assert(FIRST_TURN % 2 == 0, "after a turn the current best is in best[0] again");
        Frag q[G][R];
        float best[2][G][R];
        int best_tile[G][R];
        bool live[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            live[g] = slot0 + g * 32 * R < n_act;  // uniform in the wave
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int slot = slot0 + (g * R + r) * 32 + c;
                const int64_t row = slot < n_act ? query_row(a, qbase, slot) : 0;
                if (fa.raw_queries) q[g][r] = O::round_raw(O::load_raw(fa.raw_src.map[b] + row * fa.raw_src.row_stride, h));
                else q[g][r] = O::load(src + row * O::ROW_BYTES, h);
                best[0][g][r] = ninf;
                best[1][g][r] = ninf;
                best_tile[g][r] = 0x7FFFFFFF;
            }
        }

        // one turn: stage my tile of the turn, then multiply the four staged tiles
        auto turn = [&](int k, auto slot_tag) {
            constexpr int SLOT = decltype(slot_tag)::value;
            const int mine = t0 + k * FIRST_TURN + wave;
            const Frag f = Tile::fragment(raw[SLOT]);
            stage_lo[SLOT][wave][lane] = f.lo;
            stage_hi[SLOT][wave][lane] = f.hi;
            if (RAWT && quad == 0 && mine < t1) O::store_tile(tgt + (int64_t)mine * (32 * O::ROW_BYTES), c, h, f);
            raw[SLOT] = Tile::fetch(fa, tgt, b, mine + FIRST_AHEAD * FIRST_TURN, t1, c, h);
            __syncthreads();
#pragma unroll
            for (int j = 0; j < FIRST_TURN; ++j) {
                const int t = t0 + k * FIRST_TURN + j;
                const int now = j & 1, then = now ^ 1;
                if (t < t1) {  // uniform
                    Frag cur;
                    cur.lo = stage_lo[SLOT][j][lane];
                    cur.hi = stage_hi[SLOT][j][lane];
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        if (live[g]) {
                            f32x16 acc[R];
#pragma unroll
                            for (int r = 0; r < R; ++r) acc[r] = O::mma(cur, q[g][r]);
                            if (t * 32 + 32 > a.m) {  // only the last tile of the map can be partial
                                const int bound = a.m - t * 32 - 4 * h;
#pragma unroll
                                for (int r = 0; r < R; ++r)
#pragma unroll
                                    for (int v = 0; v < 16; ++v)
                                        if (tile_row(v, 0) >= bound) acc[r][v] = ninf;
                            }
#pragma unroll
                            for (int r = 0; r < R; ++r) {
                                const float top = fold16(best[now][g][r], acc[r]);
                                if (top > best[now][g][r]) best_tile[g][r] = t;
                                best[then][g][r] = top;
                            }
                        }
                    }
                } else {  // past the chunk's last tile: the best just moves on
#pragma unroll
                    for (int g = 0; g < G; ++g)
#pragma unroll
                        for (int r = 0; r < R; ++r) best[then][g][r] = best[now][g][r];
                }
            }
        };
        for (int k = 0; k < n_turns; k += 2) {
            turn(k, std::integral_constant<int, 0>{});
            if (k + 1 < n_turns) turn(k + 1, std::integral_constant<int, 1>{});  // uniform
        }

#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int r = 0; r < R; ++r) {
                float mine = best[0][g][r];
                const float ob = __shfl_xor(mine, 32);
                const int ot = __shfl_xor(best_tile[g][r], 32);
                if (ob > mine || (ob == mine && ot < best_tile[g][r])) {
                    mine = ob;
                    best_tile[g][r] = ot;
                }
                const int slot = slot0 + (g * R + r) * 32 + c;
                if (h == 0 && slot < n_act) atomicMax(&a.out_keys[qbase + slot], pack_key(mine, best_tile[g][r]));
            }
        __syncthreads();  // the next unit's first turn reuses ring slot 0
    }
}

// Pass 2: one wave per query recomputes the 32 scores of the winning tile with the same
// matrix instruction (the query replicated into every column, so each score has the bits
// pass 1 saw) and picks the lowest candidate that attains the maximum.  The key is
// rewritten with the candidate index; optionally index and score are stored as well.
// load_query(b, row, h) supplies the query fragment.
template <int CT, int DP, typename LoadQuery>
__device__ __forceinline__ void resolve_body(const SearchArgs& a, int32_t* out_idx, float* out_score, LoadQuery load_query) {
    using O = Ops<CT, DP>;
    using Frag = typename O::Frag;
    const int lane = threadIdx.x & 63, c = lane & 31, h = lane >> 5;
    const int wave = blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n_waves = gridDim.x * 4;
    const int b = blockIdx.y;
    int n_act = a.nq;
    if (a.nq_active) n_act = min(max(a.nq_active[b], 0), a.nq);
    const char* tgt = a.tgt + (int64_t)b * a.tgt_bstride;
    const int64_t qbase = (int64_t)b * a.nq;
    const float ninf = -__builtin_inff();

    for (int slot = wave; slot < n_act; slot += n_waves) {
        const u64 key = a.out_keys[qbase + slot];
        int32_t idx = -1;
        float score = ninf;
        if (key != 0) {
            const int tile = min(key_index(key), a.m_tiles - 1);
            const Frag qf = load_query(b, query_row(a, qbase, slot), h);
            const Frag cand = O::load(tgt + ((int64_t)tile * 32 + c) * O::ROW_BYTES, h);
            f32x16 acc = O::mma(cand, qf);
            if (tile * 32 + 32 > a.m) {
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    if (tile * 32 + tile_row(v, h) >= a.m) acc[v] = ninf;
            }
            float top = fold16(ninf, acc);
            top = __builtin_fmaxf(top, __shfl_xor(top, 32));
            int row = 64;
#pragma unroll
            for (int v = 15; v >= 0; --v)
                if (acc[v] == top) row = tile_row(v, h);
            row = min(row, __shfl_xor(row, 32));
            idx = tile * 32 + row;
            score = top;
            if (lane == 0) a.out_keys[qbase + slot] = pack_key(score, idx);
        }
        if (lane == 0 && out_idx) {
            out_idx[qbase + slot] = idx;
            if (out_score) out_score[qbase + slot] = score;
        }
    }
}

template <int CT, int DP>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2)))
void resolve_kernel(SearchArgs a, int32_t* out_idx, float* out_score) {
    using O = Ops<CT, DP>;
    resolve_body<CT, DP>(a, out_idx, out_score, [&](int b, int64_t row, int h) {
        return O::load(a.src + (int64_t)b * a.src_bstride + row * O::ROW_BYTES, h);
    });
}

// The same with the queries still in the caller's fp32 map (rounded on the way, like the
// fused first search rounds them).
template <int CT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2)))
void resolve_raw_kernel(FirstSearchArgs fa, int32_t* out_idx, float* out_score) {
    using O = Ops<CT, 24>;
    resolve_body<CT, 24>(fa.s, out_idx, out_score, [&](int b, int64_t row, int h) {
        return O::round_raw(O::load_raw(fa.raw_src.map[b] + row * fa.raw_src.row_stride, h));
    });
}

// One resident wave per hardware slot: the grid is exactly what the chip holds at once
// (workgroups per CU from the occupancy calculator x CUs), split evenly between the pairs, so
// there is no partial last round and the per-wave start-up cost and the final key merges are
// paid once per slot.  Two waves per SIMD are what the widest variant fits and what measured
// best for the narrower ones too, so the widest variant's occupancy sizes every launch.
// Candidate tiles in flight: rows wider than 128 bytes (the two-term fp16 representation) take
// a shorter ring so that ring, query fragments and accumulators still fit the register file.
template <int CT, int DP>
constexpr int search_ring() {
    return Ops<CT, DP>::ROW_BYTES > 128 ? 2 : SEARCH_P;
}
template <int CT, int DP>
constexpr int search_g_limit() {
    // a query fragment is ROW_BYTES / 8 registers per lane and G*R of them are resident
    constexpr int frag_regs = Ops<CT, DP>::ROW_BYTES / 8;
    return frag_regs <= 6 ? 4 : (frag_regs <= 12 ? 2 : 1);
}
template <int CT, int DP>
static int search_wgs_per_pair(int batch) {
    static DeviceCache resident_wgs;  // workgroups of the widest variant the current device holds at once
    const long long resident = resident_wgs.get([](int dev) -> long long {
        int per_cu = 0;
        hipDeviceProp_t prop;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu,
                                                         search_kernel<CT, DP, SEARCH_R, search_ring<CT, DP>(), search_g_limit<CT, DP>()>,
                                                         SEARCH_WAVES * 64, 0) != hipSuccess ||
            hipGetDeviceProperties(&prop, dev) != hipSuccess)
            return -1;
        return (long long)(per_cu > 0 ? per_cu : 1) * prop.multiProcessorCount;
    });
    if (resident <= 0) return 0;
    int wgs = (int)resident / batch;
    if (wgs >= 8) wgs &= ~7;  // a multiple of 8 per pair keeps the XCD renumbering a bijection
    return wgs < 1 ? 1 : wgs;
}

// Tiles per chunk if the launch used row groups of G*R blocks.
template <int CT, int DP, int G>
static int search_chunk_tiles(const SearchArgs& a, int batch) {
    const int n_waves = search_wgs_per_pair<CT, DP>(batch) * SEARCH_WAVES;
    const int row_groups = (a.nq + 32 * SEARCH_R * G - 1) / (32 * SEARCH_R * G);
    const int chunks = n_waves / row_groups > 0 ? n_waves / row_groups : 1;
    return a.m_tiles / chunks;
}

template <int CT, int DP, int G>
static hipError_t launch_search_g(const SearchArgs& a, int batch, hipStream_t s) {
    int wgs = search_wgs_per_pair<CT, DP>(batch);
    if (wgs == 0) return hipErrorUnknown;
    const int64_t max_units = (int64_t)((a.nq + 32 * SEARCH_R * G - 1) / (32 * SEARCH_R * G)) *
                              ((a.m_tiles + SEARCH_MIN_TILES - 1) / SEARCH_MIN_TILES);
    const int64_t need = (max_units + SEARCH_WAVES - 1) / SEARCH_WAVES;
    if (need < wgs) wgs = (int)(need > 0 ? need : 1);
    return launch_detail(TK_SEARCH, G, search_kernel<CT, DP, SEARCH_R, search_ring<CT, DP>(), G>, dim3(wgs, batch), dim3(SEARCH_WAVES * 64), 0, s, a);
}

template <int CT, int DP>
static hipError_t launch_search_t(const SearchArgs& a, int batch, hipStream_t s) {
    // Wider row groups (more query blocks per loaded candidate tile) pay off while the chunks
    // stay long -- with many waves per pair (few pairs) short chunks would mostly pay
    // start-up -- and while the resident query fragments fit the register file.
    constexpr int G_LIMIT = search_g_limit<CT, DP>();
    if constexpr (G_LIMIT >= 4)
        if (search_chunk_tiles<CT, DP, 4>(a, batch) >= SEARCH_WIDE_MIN_TILES) return launch_search_g<CT, DP, 4>(a, batch, s);
    if constexpr (G_LIMIT >= 2)
        if (search_chunk_tiles<CT, DP, 2>(a, batch) >= SEARCH_WIDE_MIN_TILES) return launch_search_g<CT, DP, 2>(a, batch, s);
    return launch_search_g<CT, DP, 1>(a, batch, s);
}

hipError_t launch_search(const SearchArgs& a, int batch, int compute, int dp, hipStream_t s) {
    if (a.nq <= 0 || batch <= 0) return hipSuccess;
    if (compute == FNN_F16) {
        if (dp == 16) return launch_search_t<CT_F16, 16>(a, batch, s);
        if (dp == 24) return launch_search_t<CT_F16, 24>(a, batch, s);
        if (dp == 32) return launch_search_t<CT_F16, 32>(a, batch, s);
        // rows of the two-term representation (three copies of the channels)
        if (dp == 48) return launch_search_t<CT_F16, 48>(a, batch, s);
        if (dp == 64) return launch_search_t<CT_F16, 64>(a, batch, s);
        if (dp == 80) return launch_search_t<CT_F16, 80>(a, batch, s);
        if (dp == 96) return launch_search_t<CT_F16, 96>(a, batch, s);
    } else if (compute == FNN_BF16) {
        if (dp == 16) return launch_search_t<CT_BF16, 16>(a, batch, s);
        if (dp == 24) return launch_search_t<CT_BF16, 24>(a, batch, s);
        if (dp == 32) return launch_search_t<CT_BF16, 32>(a, batch, s);
    } else {
        if (dp == 8) return launch_search_t<CT_F32, 8>(a, batch, s);
        if (dp == 16) return launch_search_t<CT_F32, 16>(a, batch, s);
        if (dp == 24) return launch_search_t<CT_F32, 24>(a, batch, s);
        if (dp == 32) return launch_search_t<CT_F32, 32>(a, batch, s);
    }
    return hipErrorInvalidValue;
}

// ---- fused first search: launch shape ------------------------------------------------------
// Workgroups of the staged kernel that the current device holds at once (0: unknown).
static int first_search_resident_wgs() {
    static DeviceCache resident_wgs;
    const long long resident = resident_wgs.get([](int dev) -> long long {
        int per_cu = 0;
        hipDeviceProp_t prop;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, search_first_kernel<CT_F16, FIRST_G, true>, SEARCH_WAVES * 64, 0) != hipSuccess ||
            hipGetDeviceProperties(&prop, dev) != hipSuccess)
            return -1;
        return (long long)(per_cu > 0 ? per_cu : 1) * prop.multiProcessorCount;
    });
    return resident > 0 ? (int)resident : 0;
}
static int first_search_wgs_per_pair(int batch) {
    int wgs = first_search_resident_wgs() / batch;
    if (wgs >= 8) wgs &= ~7;
    return wgs < 1 ? 1 : wgs;
}

bool first_search_applies(int64_t nq, int64_t m, int batch) {
    // at least one full quad of row groups, so that the four waves of a workgroup all have queries ...
    if (nq < (int64_t)SEARCH_WAVES * 32 * SEARCH_R * FIRST_G || nq > 0x7FFFFFFF) return false;
    // ... and chunks of at least FIRST_MIN_CHUNK tiles: one pair alone spreads over so many workgroups
    // that a chunk would be a few turns long and mostly start-up (measured: a single 512x384 pair is
    // 1.5 % slower with the staged kernel, two pairs are 2.5 % faster)
    const int64_t row_groups = (nq + 32 * SEARCH_R * FIRST_G - 1) / (32 * SEARCH_R * FIRST_G);
    const int64_t quads = (row_groups + SEARCH_WAVES - 1) / SEARCH_WAVES;
    const int64_t chunks = first_search_wgs_per_pair(batch) / quads > 0 ? first_search_wgs_per_pair(batch) / quads : 1;
    return (m + 31) / 32 / chunks >= FIRST_MIN_CHUNK;
}

template <int CT, bool RAWT>
static hipError_t launch_search_first_t(const FirstSearchArgs& a, int batch, hipStream_t s) {
    if (first_search_resident_wgs() <= 0) return hipErrorUnknown;
    int wgs = first_search_wgs_per_pair(batch);
    const int row_groups = (a.s.nq + 32 * SEARCH_R * FIRST_G - 1) / (32 * SEARCH_R * FIRST_G);
    const int quads = (row_groups + SEARCH_WAVES - 1) / SEARCH_WAVES;
    const int64_t max_units = (int64_t)quads * ((a.s.m_tiles + FIRST_TURN - 1) / FIRST_TURN);
    if (max_units < wgs) wgs = (int)(max_units > 0 ? max_units : 1);
    return launch_detail(TK_SEARCH, 100 + FIRST_G, search_first_kernel<CT, FIRST_G, RAWT>, dim3(wgs, batch), dim3(SEARCH_WAVES * 64), 0, s, a);
}

hipError_t launch_search_first(const FirstSearchArgs& a, int batch, int compute, hipStream_t s) {
    if (a.s.nq <= 0 || batch <= 0) return hipSuccess;
    const bool raw = a.raw_tgt.map[0] != nullptr;  // else the candidates are the prepared map s.tgt itself
    if (compute == FNN_F16) return raw ? launch_search_first_t<CT_F16, true>(a, batch, s) : launch_search_first_t<CT_F16, false>(a, batch, s);
    if (compute == FNN_BF16) return raw ? launch_search_first_t<CT_BF16, true>(a, batch, s) : launch_search_first_t<CT_BF16, false>(a, batch, s);
    return hipErrorInvalidValue;
}

hipError_t launch_resolve_raw(const FirstSearchArgs& a, int batch, int compute, int32_t* out_idx, float* out_score, hipStream_t s) {
    if (a.s.nq <= 0 || batch <= 0) return hipSuccess;
    int wgs = (a.s.nq + 3) / 4;
    const int cap = 2048 / batch > 64 ? 2048 / batch : 64;
    if (wgs > cap) wgs = cap;
    if (compute == FNN_F16) return launch(TK_RESOLVE, resolve_raw_kernel<CT_F16>, dim3(wgs, batch), dim3(256), 0, s, a, out_idx, out_score);
    if (compute == FNN_BF16) return launch(TK_RESOLVE, resolve_raw_kernel<CT_BF16>, dim3(wgs, batch), dim3(256), 0, s, a, out_idx, out_score);
    return hipErrorInvalidValue;
}

template <int CT, int DP>
static hipError_t launch_resolve_t(const SearchArgs& a, int batch, int32_t* out_idx, float* out_score, hipStream_t s) {
    int wgs = (a.nq + 3) / 4;
    const int cap = 2048 / batch > 64 ? 2048 / batch : 64;  // measured best: more waves only add dispatch time
    if (wgs > cap) wgs = cap;
    return launch(TK_RESOLVE, resolve_kernel<CT, DP>, dim3(wgs, batch), dim3(256), 0, s, a, out_idx, out_score);
}

hipError_t launch_resolve(const SearchArgs& a, int batch, int compute, int dp, int32_t* out_idx, float* out_score,
                          hipStream_t s) {
    if (a.nq <= 0 || batch <= 0) return hipSuccess;
    if (compute == FNN_F16) {
        if (dp == 16) return launch_resolve_t<CT_F16, 16>(a, batch, out_idx, out_score, s);
        if (dp == 24) return launch_resolve_t<CT_F16, 24>(a, batch, out_idx, out_score, s);
        if (dp == 32) return launch_resolve_t<CT_F16, 32>(a, batch, out_idx, out_score, s);
        if (dp == 48) return launch_resolve_t<CT_F16, 48>(a, batch, out_idx, out_score, s);
        if (dp == 64) return launch_resolve_t<CT_F16, 64>(a, batch, out_idx, out_score, s);
        if (dp == 80) return launch_resolve_t<CT_F16, 80>(a, batch, out_idx, out_score, s);
        if (dp == 96) return launch_resolve_t<CT_F16, 96>(a, batch, out_idx, out_score, s);
    } else if (compute == FNN_BF16) {
        if (dp == 16) return launch_resolve_t<CT_BF16, 16>(a, batch, out_idx, out_score, s);
        if (dp == 24) return launch_resolve_t<CT_BF16, 24>(a, batch, out_idx, out_score, s);
        if (dp == 32) return launch_resolve_t<CT_BF16, 32>(a, batch, out_idx, out_score, s);
    } else {
        if (dp == 8) return launch_resolve_t<CT_F32, 8>(a, batch, out_idx, out_score, s);
        if (dp == 16) return launch_resolve_t<CT_F32, 16>(a, batch, out_idx, out_score, s);
        if (dp == 24) return launch_resolve_t<CT_F32, 24>(a, batch, out_idx, out_score, s);
        if (dp == 32) return launch_resolve_t<CT_F32, 32>(a, batch, out_idx, out_score, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace fnn
