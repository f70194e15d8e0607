// All-pairs mutual nearest neighbours (paper section 3.2.5, "Problem Context"): every score
// S[i][j] = <D1[i], D2[j]> is formed exactly once on the matrix cores and folded, while it
// is still in a register, into BOTH running maxima -- the best candidate j of query i and
// the best query i of candidate j -- so the quadratic score matrix never exists in memory.
//
// Pass 1 (dense_kernel) works at about 1.3 vector operations per score by tracking only
// maxima plus a COARSE location:
//   * a wave keeps J candidate tiles (32 pixels of D2 each) resident and sweeps query
//     blocks (32 pixels of D1) past them, two blocks per step;
//   * best candidate of a query: a 3-input-max fold over the 16 result registers of each
//     product; the location kept is the wave's group of J tiles (J*32 consecutive candidates);
//   * best query of a candidate: one 3-input max per result register folds the two query
//     blocks of a step into a running maximum per (candidate, lane); once per super-block of
//     S query blocks the 32 lanes are reduced and the winning lane is noted.  D1 is stored
//     "segment major" (dense_perm.hpp) so that the S queries one lane sees inside a
//     super-block are S CONSECUTIVE pixels: the location kept is that run of S pixels.
//   Locations are ordered like the pixels they cover, so "largest score, then lowest
//   location" (a 64-bit max on packed keys) always keeps the run that holds the lowest
//   index among equal scores.
// Pass 2 buckets the pixels by their winning unit and recomputes, 32 pixels of one unit at a
// time, just that unit with the same matrix instruction -- bit-identical scores -- and names
// the lowest index that attains the maximum.  Then the reciprocity filter and an ordered
// compaction.
#include "dense_perm.hpp"
#include "fnn_device.hpp"
#include "fnn_kernels.hpp"
#include "trace.hpp"

namespace fnn {

__device__ __forceinline__ float max3f(float a, float b, float c) { return __builtin_fmaxf(__builtin_fmaxf(a, b), c); }

__device__ __forceinline__ float fold16f(float seed, const f32x16& x) {
    const float t0 = max3f(x[0], x[1], x[2]);
    const float t1 = max3f(x[3], x[4], x[5]);
    const float t2 = max3f(x[6], x[7], x[8]);
    const float t3 = max3f(x[9], x[10], x[11]);
    const float t4 = max3f(x[12], x[13], x[14]);
    const float t5 = max3f(t0, t1, t2);
    const float t6 = max3f(t3, t4, x[15]);
    return max3f(seed, t5, t6);
}

// One super-block (S query blocks) swept past the wave's J resident candidate tiles.  TAIL
// selects the variant that masks padding pixels (queries >= n, candidates >= m); it is only
// needed for the last super-block / last candidate group, so the hot variant carries no
// masking code at all.
template <int CT, int DP, bool TAIL>
__device__ __forceinline__ void dense_sweep(const DenseArgs& a, const typename Ops<CT, DP>::Frag (&cand)[DENSE_J],
                                            float (&cmax)[DENSE_J][16], const char* qbase, int sbg, int tbase,
                                            u64* lds_rows, int unit_row, int c, int h) {
    using O = Ops<CT, DP>;
    using Frag = typename O::Frag;
    constexpr int J = DENSE_J, S = DENSE_S;
    const float ninf = -__builtin_inff();
    Frag qa = O::load_tile(qbase, c, h);
    Frag qb = O::load_tile(qbase + 32 * O::ROW_BYTES, c, h);
    // Software pipeline: the matrix instructions of the NEXT product pair are issued before
    // the current pair's 32 result registers are folded, so the matrix cores stay busy while
    // the vector ALU works.
    // Two buffers used alternately (J is even, so every step starts on buffer 0 again and no
    // register copies are needed).
    static_assert(DENSE_J % 2 == 0, "the pipeline alternates two result buffers");
    f32x16 pa[2], pb[2];
    pa[0] = O::mma(cand[0], qa);
    pb[0] = O::mma(cand[0], qb);
    for (int t = 0; t < S; t += 2) {
        // prefetch the next two query blocks (the last step reloads its own)
        const int tn = min(t + 2, S - 2);
        const Frag na = O::load_tile(qbase + (int64_t)tn * 32 * O::ROW_BYTES, c, h);
        const Frag nb = O::load_tile(qbase + (int64_t)(tn + 1) * 32 * O::ROW_BYTES, c, h);
        float ra = ninf, rb = ninf;
#pragma unroll
        for (int jt = 0; jt < J; ++jt) {
            const int cur = jt & 1, nxt = cur ^ 1;
            // next pair: the following resident tile, or tile 0 against the next query blocks
            // (after the last step that product is computed once more and never folded)
            if (jt + 1 < J) {
                pa[nxt] = O::mma(cand[jt + 1], qa);
                pb[nxt] = O::mma(cand[jt + 1], qb);
            } else {
                pa[nxt] = O::mma(cand[0], na);
                pb[nxt] = O::mma(cand[0], nb);
            }
            if (TAIL) {
                const int ia = segment_pixel(sbg, t, c);  // pixel of this lane's query in block t
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const bool cand_ok = (tbase + jt) * 32 + tile_row(v, h) < a.m;
                    if (!cand_ok || ia >= a.n) pa[cur][v] = ninf;
                    if (!cand_ok || ia + 1 >= a.n) pb[cur][v] = ninf;
                }
            }
            ra = fold16f(ra, pa[cur]);
            rb = fold16f(rb, pb[cur]);
#pragma unroll
            for (int v = 0; v < 16; ++v) cmax[jt][v] = max3f(cmax[jt][v], pa[cur][v], pb[cur][v]);
        }
        // best candidate of the two queries over this wave's J tiles -> workgroup table:
        // lane half 0 files block t, half 1 files block t+1
        const float mine = cross_half_max(ra, rb);
        if (!TAIL || mine != ninf) atomicMax(&lds_rows[(t + h) * 32 + c], pack_key(mine, unit_row));
        qa = na;
        qb = nb;
    }
}

// For registers V..15: the lowest lane of each wave half whose x[v] equals tops[v], handed to
// the lane of that half that holds register v after transpose_max16 (rows 0 of the halves).
template <int V>
__device__ __forceinline__ void locate_first_lanes(const float (&x)[16], const float (&tops)[16], int& first_lane) {
    if constexpr (V < 16) {
        const u64 hit = __ballot(x[V] == tops[V]);
        // bit 31 is forced so that the count is defined (and in range) even for an empty mask
        const int lane_lo = __builtin_ctz((unsigned)hit | 0x80000000u);
        const int lane_hi = __builtin_ctz((unsigned)(hit >> 32) | 0x80000000u);
        first_lane = write_lane<holder_lane(V)>(first_lane, lane_lo);
        first_lane = write_lane<32 + holder_lane(V)>(first_lane, lane_hi);
        locate_first_lanes<V + 1>(x, tops, first_lane);
    }
}

// Best query of each resident candidate inside one super-block: a transposing reduction
// leaves the maximum of register v with the lanes that hold v; the 16 maxima of a half go
// round through the wave's LDS words so that every lane can test its own value against them;
// the lowest lane that attains each maximum is read off the comparison mask and handed to the
// holding lane, which files the key (one LDS operation per tile).
__device__ __forceinline__ void dense_flush_columns(const float (&cmax)[DENSE_J][16], float* lds_tops, u64* lds_col_keys,
                                                    int sbg, int lane, int h, int held) {
    const float ninf = -__builtin_inff();
#pragma unroll
    for (int jt = 0; jt < DENSE_J; ++jt) {
        const float top = transpose_max16(cmax[jt], lane);
        lds_tops[h * 16 + held] = top;  // the two rows of a half store the same value
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        float tops[16];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 t4 = reinterpret_cast<const float4*>(lds_tops + h * 16)[q];
            tops[4 * q + 0] = t4.x;
            tops[4 * q + 1] = t4.y;
            tops[4 * q + 2] = t4.z;
            tops[4 * q + 3] = t4.w;
        }
        __builtin_amdgcn_wave_barrier();
        int first_lane = 0;
        locate_first_lanes<0>(cmax[jt], tops, first_lane);
        if ((lane & 16) == 0 && top != ninf)
            atomicMax(&lds_col_keys[jt * 32 + tile_row(held, h)], pack_key(top, sbg * 32 + first_lane));
    }
}

// The 16-bit rows of the two-term representation (96 to 192 bytes) need more than half the
// register file for the resident tiles, the query ring and the result buffers: one wave per
// SIMD there.  Everything else runs two (measured: fp16 d = 24 2.4 ms against 3.6 ms with one
// wave, fp32 d = 24 14.0 against 15.6 ms, although both spill a little outside the hot loop).
template <int CT, int DP>
constexpr int dense_waves_per_simd() {
    return (CT != CT_F32 && Ops<CT, DP>::ROW_BYTES > 64) ? 1 : 2;
}
// The work of one workgroup of pass 1: its super-blocks of queries swept past its candidate groups.
template <int CT, int DP>
// lds_row_keys: [sb_per_wg * S * 32] keys indexed by the query's stored slot in the workgroup's
// range; lds_col_keys: J * 32 keys and lds_tops: 32 floats of the calling wave.
__device__ __forceinline__ void dense_workgroup(const DenseArgs& a, u64* lds_row_keys, u64* lds_col_keys, float* lds_tops) {
    using O = Ops<CT, DP>;
    using Frag = typename O::Frag;
    constexpr int J = DENSE_J, S = DENSE_S;
    const int lane = threadIdx.x & 63, c = lane & 31, h = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int held = held_register(lane);
    const int b = blockIdx.z;
    const float ninf = -__builtin_inff();

    const int sb0 = blockIdx.y * a.sb_per_wg;          // first super-block of this workgroup
    const int n_sb = min(a.sb_per_wg, a.n_sb - sb0);
    const int group0 = blockIdx.x * a.groups_per_wg;   // first candidate group (DENSE_WAVES*J tiles)

    for (int i = threadIdx.x; i < a.sb_per_wg * S * 32; i += blockDim.x) lds_row_keys[i] = 0;
    __syncthreads();

    const char* d1 = a.d1 + (int64_t)b * a.d1_bstride;
    const char* d2 = a.d2 + (int64_t)b * a.d2_bstride;
    u64* row_keys = a.row_keys + (int64_t)b * a.n;
    u64* col_keys = a.col_keys + (int64_t)b * a.m;

    for (int g = 0; g < a.groups_per_wg; ++g) {
        const int tbase = ((group0 + g) * DENSE_WAVES + wave) * J;  // this wave's first candidate tile
        if (tbase >= a.m_tiles) break;                              // uniform per wave; no barrier in this loop

        Frag cand[J];
#pragma unroll
        for (int jt = 0; jt < J; ++jt) {
            cand[jt] = O::load(d2 + ((int64_t)min(tbase + jt, a.m_tiles - 1) * 32 + c) * O::ROW_BYTES, h);
            lds_col_keys[jt * 32 + c] = 0;  // both lane halves store the same zero
        }
        const bool cand_tail = (tbase + J) * 32 > a.m;              // some resident candidate is past the map

        for (int sb = 0; sb < n_sb; ++sb) {
            const int sbg = sb0 + sb;
            const bool query_tail = (sbg + 1) * (32 * S) > a.n;     // some query of this super-block is padding
            float cmax[J][16];
#pragma unroll
            for (int jt = 0; jt < J; ++jt)
#pragma unroll
                for (int v = 0; v < 16; ++v) cmax[jt][v] = ninf;

            const char* qbase = d1 + (int64_t)sbg * S * 32 * O::ROW_BYTES;  // uniform: the lane offset is added by load_tile
            if (cand_tail || query_tail)
                dense_sweep<CT, DP, true>(a, cand, cmax, qbase, sbg, tbase, lds_row_keys + sb * S * 32, tbase / J, c, h);
            else
                dense_sweep<CT, DP, false>(a, cand, cmax, qbase, sbg, tbase, lds_row_keys + sb * S * 32, tbase / J, c, h);

            dense_flush_columns(cmax, lds_tops, lds_col_keys, sbg, lane, h, held);
        }

        // this wave's candidates are complete for the workgroup's query range
#pragma unroll
        for (int jt = 0; jt < J; ++jt) {
            const int j = (tbase + jt) * 32 + c;
            const u64 key = lds_col_keys[jt * 32 + c];
            if (h == 0 && j < a.m && key) atomicMax(&col_keys[j], key);
        }
    }

    __syncthreads();
    for (int slot = threadIdx.x; slot < n_sb * S * 32; slot += blockDim.x) {
        const u64 key = lds_row_keys[slot];
        const int i = segment_pixel(sb0 + slot / (S * 32), (slot / 32) % S, slot % 32);
        if (key && i < a.n) atomicMax(&row_keys[i], key);
    }
}

template <int CT, int DP>
__global__ __launch_bounds__(DENSE_WAVES * 64) __attribute__((amdgpu_waves_per_eu(dense_waves_per_simd<CT, DP>())))
void dense_kernel(DenseArgs a) {
    extern __shared__ u64 lds[];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    u64* col_keys = lds + (size_t)a.sb_per_wg * DENSE_S * 32;
    dense_workgroup<CT, DP>(a, lds, col_keys + wave * (DENSE_J * 32),
                            reinterpret_cast<float*>(col_keys + DENSE_WAVES * (DENSE_J * 32)) + wave * 32);
}

// ---- pass 1 with the query blocks staged through LDS (16-bit formats, 24 channels) ----------
// The four waves of a workgroup sweep the SAME query blocks past their own resident tiles, so
// in dense_kernel every block crosses the vector memory path four times per workgroup.  Here a
// workgroup fetches each block once: a turn is DENSE_TURN_BLOCKS query blocks (four steps);
// while the waves compute on one LDS slot, the next turn's blocks -- two per wave -- are on
// their way into the other slot through direct global->LDS loads, which occupy no registers.
// One workgroup barrier per turn, taken at the start of the turn's last step: by then every wave
// holds that step's blocks in registers, so the slot can be refilled at once for the turn after
// next, and the first blocks of the next turn can be read from the other slot in time for the
// software pipeline to run on across the turn boundary.  Arithmetic, keys and results are those
// of dense_kernel.
#ifndef FNN_DENSE_STAGED
#define FNN_DENSE_STAGED 1
#endif
constexpr bool DENSE_STAGED = FNN_DENSE_STAGED != 0;
constexpr int DENSE_TURN_STEPS = 4;
constexpr int DENSE_TURN_BLOCKS = 2 * DENSE_TURN_STEPS;
constexpr int DENSE_TURNS = DENSE_S / DENSE_TURN_BLOCKS;  // turns per super-block
static_assert(DENSE_S % DENSE_TURN_BLOCKS == 0 && DENSE_TURNS % 2 == 0, "a sweep is a whole, even number of turns");
static_assert(DENSE_TURN_BLOCKS == 2 * DENSE_WAVES, "every wave stages two blocks of a turn");
static_assert(DENSE_TURN_STEPS % 2 == 0, "the steps of a turn alternate two register sets");

// One slot of the stage.  The two slots are separate LDS variables, so that the compiler can tell
// a read of one slot from a load in flight into the other and need not wait for it.
struct DenseSlot {
    uint4 lo[DENSE_TURN_BLOCKS][64];  // channels 8h..8h+7 of lane (c, h)'s row
    uint2 hi[DENSE_TURN_BLOCKS][64];  // channels 16+4h..16+4h+3
};

#define FNN_LDS_PTR(p) ((void __attribute__((address_space(3)))*)(p))

// This wave's two blocks of the turn that starts at `turn` (uniform; 48-byte rows) into slot `st`.
// A direct load writes lane l's bytes at the LDS base + l * size: 16 bytes per lane give the
// `lo` words in lane order; the `hi` words (8 bytes per reading lane) take two 4-byte loads in
// which lane l fetches word l & 1 of reading lane l >> 1 (first half) or 32 + (l >> 1).
__device__ __forceinline__ void dense_stage_turn(DenseSlot& st, const char* turn, int wave) {
    // The lane number is read afresh and the byte offsets are recomputed from it (a few
    // operations per turn): held across the sweep they were spilled, and a reload behind the
    // loads issued here would wait for all of them.
    uint32_t l;
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(l));
    const uint32_t c = l & 31, h = l >> 5, pair = l >> 1, word = l & 1;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int blk = 2 * wave + i;
        const char* src = turn + (int64_t)blk * (32 * 48);
        __builtin_amdgcn_global_load_lds((const void*)(src + (c * 48u + 16u * h)), FNN_LDS_PTR(&st.lo[blk][0]), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((const void*)(src + (pair * 48u + 32u + 4u * word)), FNN_LDS_PTR(&st.hi[blk][0]), 4, 0, 0);
        __builtin_amdgcn_global_load_lds((const void*)(src + (pair * 48u + 40u + 4u * word)), FNN_LDS_PTR(&st.hi[blk][32]), 4, 0, 0);
    }
}

// Where the workgroup's query stream stands: turn k of the stream is turn k % DENSE_TURNS of
// super-block (k / DENSE_TURNS) % n_sb (the stream repeats for every candidate group).
struct DenseStream {
    const char* d1;   // first super-block of the workgroup
    int n_sb;
    int total;        // turns in the whole stream
    __device__ __forceinline__ const char* turn(int k) const {
        k = min(k, total - 1);  // past the end: re-read the last turn, never used
        const int sb = (k / DENSE_TURNS) % n_sb, t = k % DENSE_TURNS;
        return d1 + ((int64_t)sb * DENSE_S + (int64_t)t * DENSE_TURN_BLOCKS) * (32 * 48);
    }
};

// One super-block swept past the wave's resident tiles, blocks taken from the LDS stage.  k0 is
// the stream turn the sweep starts with (even: slot 0); on entry that turn is staged and
// visible, and turn k0 + 1 is on its way.  The same holds for k0 + DENSE_TURNS on return.
template <int CT>
__device__ __forceinline__ void dense_sweep_staged(const DenseArgs& a, const typename Ops<CT, 24>::Frag (&cand)[DENSE_J],
                                                   float (&cmax)[DENSE_J][16], DenseSlot& slot0, DenseSlot& slot1, const DenseStream& stream,
                                                   int k0, u64* lds_rows, int unit_row, int wave, int lane) {
    using O = Ops<CT, 24>;
    using Frag = typename O::Frag;
    constexpr int J = DENSE_J;
    const int c = lane & 31, h = lane >> 5;
    const float ninf = -__builtin_inff();
    // Lane l's fragment of a staged block: 16 bytes at l * 16 and 8 bytes at l * 8.  The lane offset
    // is produced afresh where it is needed (three operations per step): kept in a register across
    // the unrolled sweep it was spilled, and a reload behind the direct loads waits for all of them.
    auto lane_offset = [&]() {
        uint32_t o;
        asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0\n\tv_lshlrev_b32 %0, 4, %0" : "=v"(o));
        return o;
    };
    auto staged = [&](const DenseSlot& st, int blk, uint32_t o16) {
        Frag f;
        f.lo = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(&st.lo[blk][0]) + o16);
        f.hi = *reinterpret_cast<const uint2*>(reinterpret_cast<const char*>(&st.hi[blk][0]) + (o16 >> 1));
        return f;
    };
    // Best candidate of the step's two queries over this wave's J tiles -> workgroup table (lane half
    // 0 files block t, half 1 block t + 1).  The updates of a turn are filed together just before
    // the turn's barrier, where the loads in flight have to be waited for anyway: the compiler
    // orders every LDS atomic after them.
    float row_best[DENSE_TURN_STEPS];
    auto file_row_best = [&](int s, int t) { atomicMax(&lds_rows[(t + h) * 32 + c], pack_key(row_best[s], unit_row)); };
    Frag q[2][2];  // [register set][block of the step]
    {
        const uint32_t o16 = lane_offset();
        q[0][0] = staged(slot0, 0, o16);
        q[0][1] = staged(slot0, 1, o16);
    }
    f32x16 pa[2], pb[2];
    pa[0] = O::mma(cand[0], q[0][0]);
    pb[0] = O::mma(cand[0], q[0][1]);

    auto turn = [&](int tt, auto slot_tag) {
        constexpr int SLOT = decltype(slot_tag)::value;
        DenseSlot& mine = SLOT ? slot1 : slot0;
        DenseSlot& next = SLOT ? slot0 : slot1;
#pragma unroll
        for (int s = 0; s < DENSE_TURN_STEPS; ++s) {
            const int set = s & 1, other = set ^ 1;
            const int t = tt * DENSE_TURN_BLOCKS + 2 * s;  // first query block of the step
            const uint32_t o16 = lane_offset();
            if (s + 1 < DENSE_TURN_STEPS) {
                q[other][0] = staged(mine, 2 * s + 2, o16);
                q[other][1] = staged(mine, 2 * s + 3, o16);
            } else {
                // every wave holds this step's blocks: the next turn has landed (the barrier
                // waits for this wave's loads first), and this slot is free for the one after
                {   // the last step of the turn before (in the sweep's first turn: step 0 once more, which is
                    // harmless and keeps this stretch free of branches)
                    const float carried = tt > 0 ? row_best[DENSE_TURN_STEPS - 1] : row_best[0];
                    const int carried_t = tt > 0 ? t - DENSE_TURN_BLOCKS : 0;
                    atomicMax(&lds_rows[(carried_t + h) * 32 + c], pack_key(carried, unit_row));
                }
#pragma unroll
                for (int done = 0; done + 1 < DENSE_TURN_STEPS; ++done) file_row_best(done, tt * DENSE_TURN_BLOCKS + 2 * done);
                __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's share of the next turn is in LDS
                __syncthreads();
                dense_stage_turn(mine, stream.turn(k0 + tt + 2), wave);
                q[other][0] = staged(next, 0, o16);
                q[other][1] = staged(next, 1, o16);
            }
            float ra = ninf, rb = ninf;
#pragma unroll
            for (int jt = 0; jt < J; ++jt) {
                const int cur = jt & 1, nxt = cur ^ 1;
                if (jt + 1 < J) {
                    pa[nxt] = O::mma(cand[jt + 1], q[set][0]);
                    pb[nxt] = O::mma(cand[jt + 1], q[set][1]);
                } else {  // tile 0 against the next step's blocks (after the last step: computed, never folded)
                    pa[nxt] = O::mma(cand[0], q[other][0]);
                    pb[nxt] = O::mma(cand[0], q[other][1]);
                }
                ra = fold16f(ra, pa[cur]);
                rb = fold16f(rb, pb[cur]);
#pragma unroll
                for (int v = 0; v < 16; ++v) cmax[jt][v] = max3f(cmax[jt][v], pa[cur][v], pb[cur][v]);
            }
            row_best[s] = cross_half_max(ra, rb);
            __builtin_amdgcn_sched_barrier(0);  // steps are scheduled one by one, as in the rolled loop of dense_kernel
        }
    };
    for (int tt = 0; tt < DENSE_TURNS; tt += 2) {
        turn(tt, std::integral_constant<int, 0>{});
        turn(tt + 1, std::integral_constant<int, 1>{});
    }
    file_row_best(DENSE_TURN_STEPS - 1, DENSE_S - 2);
}

template <int CT>
__global__ __launch_bounds__(DENSE_WAVES * 64) __attribute__((amdgpu_waves_per_eu(2)))
void dense_staged_kernel(DenseArgs a) {
    using O = Ops<CT, 24>;
    using Frag = typename O::Frag;
    constexpr int J = DENSE_J, S = DENSE_S;
    // Every LDS object is a variable of its own (no dynamic LDS): the compiler then knows that the
    // key tables are not the stage, and does not wait for a load in flight when it updates them.
    __shared__ DenseSlot slot0, slot1;
    __shared__ u64 row_key_table[S * 32];               // one super-block per workgroup
    __shared__ u64 col_key_table[DENSE_WAVES][J * 32];
    __shared__ float top_table[DENSE_WAVES][32];
    u64* lds_row_keys = row_key_table;
    const int lane = threadIdx.x & 63, c = lane & 31, h = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    u64* lds_col_keys = col_key_table[wave];
    float* lds_tops = top_table[wave];
    const int held = held_register(lane);
    const int b = blockIdx.z;
    const float ninf = -__builtin_inff();

    const int sb0 = blockIdx.y;  // launched with one super-block per workgroup
    const int n_sb = 1;
    const int group0 = blockIdx.x * a.groups_per_wg;
    // groups of this workgroup that hold a candidate tile at all (uniform)
    const int groups_left = (a.m_tiles - group0 * DENSE_TILES_PER_GROUP + DENSE_TILES_PER_GROUP - 1) / DENSE_TILES_PER_GROUP;
    const int n_groups = min(a.groups_per_wg, groups_left);
    if (n_groups <= 0 || n_sb <= 0) return;
    // A workgroup that meets padding -- queries past n or candidates past m -- takes the
    // unstaged path, whose sweep can mask them: at most one row and one column of workgroups.
    if ((int64_t)(sb0 + n_sb) * (32 * S) > a.n || (int64_t)(group0 + n_groups) * (DENSE_TILES_PER_GROUP * 32) > a.m) {
        dense_workgroup<CT, 24>(a, lds_row_keys, lds_col_keys, lds_tops);
        return;
    }

    const char* d1 = a.d1 + (int64_t)b * a.d1_bstride;
    const char* d2 = a.d2 + (int64_t)b * a.d2_bstride;
    u64* row_keys = a.row_keys + (int64_t)b * a.n;
    u64* col_keys = a.col_keys + (int64_t)b * a.m;

    DenseStream stream;
    stream.d1 = d1 + (int64_t)sb0 * S * (32 * 48);
    stream.n_sb = n_sb;
    stream.total = n_groups * n_sb * DENSE_TURNS;

    dense_stage_turn(slot0, stream.turn(0), wave);
    for (int i = threadIdx.x; i < S * 32; i += blockDim.x) lds_row_keys[i] = 0;
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    __syncthreads();
    dense_stage_turn(slot1, stream.turn(1), wave);

    int k = 0;  // stream turn the next sweep starts with
    for (int g = 0; g < n_groups; ++g) {
        const int tbase = ((group0 + g) * DENSE_WAVES + wave) * J;  // this wave's first candidate tile (all inside the map)
        Frag cand[J];
#pragma unroll
        for (int jt = 0; jt < J; ++jt) {
            cand[jt] = O::load(d2 + ((int64_t)(tbase + jt) * 32 + c) * O::ROW_BYTES, h);
            lds_col_keys[jt * 32 + c] = 0;
        }

        for (int sb = 0; sb < n_sb; ++sb, k += DENSE_TURNS) {
            const int sbg = sb0 + sb;
            float cmax[J][16];
#pragma unroll
            for (int jt = 0; jt < J; ++jt)
#pragma unroll
                for (int v = 0; v < 16; ++v) cmax[jt][v] = ninf;

            dense_sweep_staged<CT>(a, cand, cmax, slot0, slot1, stream, k, lds_row_keys + sb * S * 32, tbase / J, wave, lane);

            dense_flush_columns(cmax, lds_tops, lds_col_keys, sbg, lane, h, held);
        }

#pragma unroll
        for (int jt = 0; jt < J; ++jt) {
            const int j = (tbase + jt) * 32 + c;
            const u64 key = lds_col_keys[jt * 32 + c];
            if (h == 0 && j < a.m && key) atomicMax(&col_keys[j], key);
        }
    }

    __syncthreads();
    for (int slot = threadIdx.x; slot < n_sb * S * 32; slot += blockDim.x) {
        const u64 key = lds_row_keys[slot];
        const int i = segment_pixel(sb0 + slot / (S * 32), (slot / 32) % S, slot % 32);
        if (key && i < a.n) atomicMax(&row_keys[i], key);
    }
}

// ---- pass 2: exact indices ---------------------------------------------------------------
// Every query knows the group of J tiles that holds its best candidate, every candidate the
// run of S queries that holds its best query.  Resolving them one by one would read a whole
// group (6 KB) or run (3 KB) per pixel and use one column of each matrix product.  Instead
// the pixels are first bucketed by their winning unit (count, scan, fill: a counting sort
// whose order inside a bucket does not matter); a wave then takes 32 pixels of ONE unit,
// reads the unit once and resolves all 32 with full 32x32 products -- the same matrix
// instruction on the same operands as pass 1, so every score has the bits pass 1 saw.
// Buckets start on chunk boundaries; the tail of a bucket's last chunk is masked off.
constexpr int BUCKET_THREADS = 1024;

__device__ __forceinline__ int row_unit_of(const DenseArgs& a, u64 key) {
    return max(0, min(key_index(key), a.row_units - 1));
}
__device__ __forceinline__ int col_unit_of(const DenseArgs& a, u64 key) {
    return max(0, min(key_index(key), a.col_units - 1));
}

// Bucket sizes.  LOCAL: the workgroup first counts its BUCKET_PER_THREAD * 1024 pixels of each
// image into a histogram in LDS and then adds only the non-empty bins to the global counters
// (device-wide atomics are slow; this cuts them several times).  Without LOCAL (more units
// than fit in LDS) every pixel updates the global counters directly.
constexpr int BUCKET_PER_THREAD = 4;

template <bool LOCAL>
__global__ __launch_bounds__(BUCKET_THREADS) void dense_bucket_count_kernel(DenseArgs a) {
    extern __shared__ int hist[];
    const int b = blockIdx.y;
    const int units = a.row_units + a.col_units;
    int32_t* counts = a.unit_counts + (int64_t)b * units;
    if (LOCAL) {
        for (int u = threadIdx.x; u < units; u += BUCKET_THREADS) hist[u] = 0;
        __syncthreads();
    }
    constexpr int PER = LOCAL ? BUCKET_PER_THREAD : 1;
    const int64_t first = (int64_t)blockIdx.x * PER * BUCKET_THREADS + threadIdx.x;
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const int64_t i = first + (int64_t)k * BUCKET_THREADS;
        if (i < a.n) {
            const u64 key = a.row_keys[(int64_t)b * a.n + i];
            if (key) atomicAdd(LOCAL ? &hist[row_unit_of(a, key)] : &counts[row_unit_of(a, key)], 1);
        }
        if (i < a.m) {
            const u64 key = a.col_keys[(int64_t)b * a.m + i];
            if (key) atomicAdd(LOCAL ? &hist[a.row_units + col_unit_of(a, key)] : &counts[a.row_units + col_unit_of(a, key)], 1);
        }
    }
    if (LOCAL) {
        __syncthreads();
        for (int u = threadIdx.x; u < units; u += BUCKET_THREADS) {
            const int c = hist[u];
            if (c) atomicAdd(&counts[u], c);
        }
    }
}

// blockIdx.x = side (0: queries by tile group, 1: candidates by run), blockIdx.y = pair.
// Exclusive scan of the bucket sizes rounded up to chunks of 32: every thread takes a run of
// consecutive units, so one pass over the counters and one block-wide scan suffice.  Writes
// each bucket's first list position (the fill cursor), the unit of every chunk and the chunk
// total.  List positions between a bucket's last pixel and the end of its last chunk stay
// unwritten; the resolve kernels know the fill level of a bucket from its cursor.
__global__ __launch_bounds__(BUCKET_THREADS) void dense_bucket_scan_kernel(DenseArgs a) {
    __shared__ int wave_sums[BUCKET_THREADS / 64];
    const int side = blockIdx.x, b = blockIdx.y;
    const int n_units = side ? a.col_units : a.row_units;
    const int unit0 = side ? a.row_units : 0;
    const int64_t list0 = side ? a.rows_cap : 0;
    const int32_t* counts = a.unit_counts + (int64_t)b * (a.row_units + a.col_units) + unit0;
    int32_t* cursor = a.unit_cursor + (int64_t)b * (a.row_units + a.col_units) + unit0;
    int32_t* chunk_unit = a.chunk_unit + ((int64_t)b * (a.rows_cap + a.cols_cap) + list0) / 32;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int per = (n_units + BUCKET_THREADS - 1) / BUCKET_THREADS;
    const int u0 = min((int)threadIdx.x * per, n_units), u1 = min(u0 + per, n_units);
    int mine = 0;  // chunks of this thread's units
    for (int u = u0; u < u1; ++u) mine += (counts[u] + 31) / 32;
    int x = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int y = __shfl_up(x, d);
        if (lane >= d) x += y;
    }
    if (lane == 63) wave_sums[wave] = x;
    __syncthreads();
    int offset = 0, total = 0;
    for (int w = 0; w < BUCKET_THREADS / 64; ++w) {
        if (w < wave) offset += wave_sums[w];
        total += wave_sums[w];
    }
    int first = offset + x - mine;  // first chunk of unit u0
    for (int u = u0; u < u1; ++u) {
        const int chunks = (counts[u] + 31) / 32;
        cursor[u] = first * 32;
        for (int k = 0; k < chunks; ++k) chunk_unit[first + k] = u;
        first += chunks;
    }
    if (threadIdx.x == 0) a.chunk_totals[b * 2 + side] = total;
}

// Every pixel takes the next free position of its bucket.  LOCAL: positions are first handed
// out inside the workgroup (LDS), then each non-empty bin reserves its share of the bucket
// with ONE global atomic.  A pixel without a key (no candidate at all) gets its final "none"
// result here.
template <bool LOCAL>
__global__ __launch_bounds__(BUCKET_THREADS) void dense_bucket_fill_kernel(DenseArgs a, int32_t* nn12, float* s12,
                                                                           int32_t* nn21, float* s21) {
    extern __shared__ int hist[];
    const int b = blockIdx.y;
    const int units = a.row_units + a.col_units;
    int32_t* cursor = a.unit_cursor + (int64_t)b * units;
    int32_t* list = a.lists + (int64_t)b * (a.rows_cap + a.cols_cap);
    if (LOCAL) {
        for (int u = threadIdx.x; u < units; u += BUCKET_THREADS) hist[u] = 0;
        __syncthreads();
    }
    constexpr int PER = LOCAL ? BUCKET_PER_THREAD : 1;
    const int64_t first = (int64_t)blockIdx.x * PER * BUCKET_THREADS + threadIdx.x;
    int unit_r[PER], rank_r[PER], unit_c[PER], rank_c[PER];  // unit < 0: nothing to file
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const int64_t i = first + (int64_t)k * BUCKET_THREADS;
        unit_r[k] = unit_c[k] = -1;
        rank_r[k] = rank_c[k] = 0;
        if (i < a.n) {
            const u64 key = a.row_keys[(int64_t)b * a.n + i];
            if (key) {
                unit_r[k] = row_unit_of(a, key);
                rank_r[k] = atomicAdd(LOCAL ? &hist[unit_r[k]] : &cursor[unit_r[k]], 1);
            } else {
                nn12[(int64_t)b * a.n + i] = -1;
                if (s12) s12[(int64_t)b * a.n + i] = -__builtin_inff();
            }
        }
        if (i < a.m) {
            const u64 key = a.col_keys[(int64_t)b * a.m + i];
            if (key) {
                unit_c[k] = a.row_units + col_unit_of(a, key);
                rank_c[k] = atomicAdd(LOCAL ? &hist[unit_c[k]] : &cursor[unit_c[k]], 1);
            } else {
                nn21[(int64_t)b * a.m + i] = -1;
                if (s21) s21[(int64_t)b * a.m + i] = -__builtin_inff();
            }
        }
    }
    if (LOCAL) {
        __syncthreads();
        for (int u = threadIdx.x; u < units; u += BUCKET_THREADS) {
            const int c = hist[u];
            if (c) hist[u] = atomicAdd(&cursor[u], c);  // first position of this workgroup's share
        }
        __syncthreads();
    }
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const int64_t i = first + (int64_t)k * BUCKET_THREADS;
        if (unit_r[k] >= 0) list[(LOCAL ? hist[unit_r[k]] : 0) + rank_r[k]] = (int32_t)i;
        if (unit_c[k] >= 0) list[a.rows_cap + (LOCAL ? hist[unit_c[k]] : 0) + rank_c[k]] = (int32_t)i;
    }
}

// Queries: a wave takes 32 queries whose best candidate lies in the same group of J tiles.
// Lane c holds query list[c]; result register v of lane (c, h) for tile jt is that query's
// score against candidate (tbase + jt)*32 + tile_row(v, h), so the lowest index at the
// maximum is found inside the lane (registers ascend with the candidate) and across its
// two halves.
template <int CT, int DP>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2)))
void dense_resolve_rows_kernel(DenseArgs a, int32_t* nn12, float* s12) {
    using O = Ops<CT, DP>;
    using Frag = typename O::Frag;
    constexpr int J = DENSE_J;
    const int lane = threadIdx.x & 63, c = lane & 31, h = lane >> 5;
    const int wave = blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n_waves = gridDim.x * 4;
    const int b = blockIdx.y;
    const char* d1 = a.d1 + (int64_t)b * a.d1_bstride;
    const char* d2 = a.d2 + (int64_t)b * a.d2_bstride;
    const int32_t* list = a.lists + (int64_t)b * (a.rows_cap + a.cols_cap);
    const int32_t* chunk_unit = a.chunk_unit + ((int64_t)b * (a.rows_cap + a.cols_cap)) / 32;
    const int32_t* cursor = a.unit_cursor + (int64_t)b * (a.row_units + a.col_units);  // after the fill: end of bucket
    const int total = min(a.chunk_totals[b * 2 + 0], (int)(a.rows_cap / 32));
    const float ninf = -__builtin_inff();
    for (int w = wave; w < total; w += n_waves) {
        const int unit = max(0, min(chunk_unit[w], a.row_units - 1));
        const int tbase = unit * J;
        const int i = w * 32 + c < cursor[unit] ? list[(int64_t)w * 32 + c] : -1;  // past the bucket's fill level
        const Frag q = O::load(d1 + segment_slot(max(0, min(i, a.n - 1))) * O::ROW_BYTES, h);
        f32x16 x[J];
        float top = ninf;
#pragma unroll
        for (int jt = 0; jt < J; ++jt) {
            const Frag cand = O::load_tile(d2 + (int64_t)min(tbase + jt, a.m_tiles - 1) * (32 * O::ROW_BYTES), c, h);
            x[jt] = O::mma(cand, q);
#pragma unroll
            for (int v = 0; v < 16; ++v)
                if (tbase + jt >= a.m_tiles || (tbase + jt) * 32 + tile_row(v, h) >= a.m) x[jt][v] = ninf;
            top = fold16f(top, x[jt]);
        }
        top = __builtin_fmaxf(top, __shfl_xor(top, 32));
        int row = J * 32;
#pragma unroll
        for (int jt = J - 1; jt >= 0; --jt)
#pragma unroll
            for (int v = 15; v >= 0; --v)
                if (x[jt][v] == top) row = jt * 32 + tile_row(v, h);
        row = min(row, __shfl_xor(row, 32));
        if (h == 0 && i >= 0 && i < a.n) {
            nn12[(int64_t)b * a.n + i] = row < J * 32 ? tbase * 32 + row : -1;
            if (s12) s12[(int64_t)b * a.n + i] = top;
        }
    }
}

// Candidates: a wave takes 32 candidates whose best query lies in the same run of S queries.
// Lane c supplies candidate list[c] as a row operand and, per part, query run0 + part*32 + c
// as a column operand: register v of lane (c, h) is the score of that query against
// candidate list[tile_row(v, h)].  Per candidate the maximum over the 32 lanes of a half
// and the lowest lane that attains it (part 0 before part 1) are taken as in pass 1.
template <int CT, int DP>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2)))
void dense_resolve_cols_kernel(DenseArgs a, int32_t* nn21, float* s21) {
    using O = Ops<CT, DP>;
    using Frag = typename O::Frag;
    constexpr int S = DENSE_S, PARTS = DENSE_S / 32;
    const int lane = threadIdx.x & 63, c = lane & 31, h = lane >> 5;
    const int wave = blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n_waves = gridDim.x * 4;
    const int b = blockIdx.y;
    const char* d1 = a.d1 + (int64_t)b * a.d1_bstride;
    const char* d2 = a.d2 + (int64_t)b * a.d2_bstride;
    const int32_t* list = a.lists + (int64_t)b * (a.rows_cap + a.cols_cap) + a.rows_cap;
    const int32_t* chunk_unit = a.chunk_unit + ((int64_t)b * (a.rows_cap + a.cols_cap) + a.rows_cap) / 32;
    const int32_t* cursor = a.unit_cursor + (int64_t)b * (a.row_units + a.col_units) + a.row_units;
    const int total = min(a.chunk_totals[b * 2 + 1], (int)(a.cols_cap / 32));
    const float ninf = -__builtin_inff();
    for (int w = wave; w < total; w += n_waves) {
        const int unit = max(0, min(chunk_unit[w], a.col_units - 1));
        const int64_t run0 = (int64_t)unit * S;  // first pixel of the run
        const int j = w * 32 + c < cursor[unit] ? list[(int64_t)w * 32 + c] : -1;  // past the bucket's fill level
        const Frag cand = O::load(d2 + (int64_t)max(0, min(j, a.m - 1)) * O::ROW_BYTES, h);
        f32x16 x[PARTS];
#pragma unroll
        for (int part = 0; part < PARTS; ++part) {
            const int64_t i = run0 + part * 32 + c;  // the run lies inside the padded map
            const Frag q = O::load(d1 + segment_slot(i) * O::ROW_BYTES, h);
            x[part] = O::mma(cand, q);
            if (i >= a.n) {
#pragma unroll
                for (int v = 0; v < 16; ++v) x[part][v] = ninf;
            }
        }
        float mine_top = ninf;
        int mine_first = 0;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            float y = x[0][v];
#pragma unroll
            for (int part = 1; part < PARTS; ++part) y = __builtin_fmaxf(y, x[part][v]);
            const float top = half_max(y);
            int first_lo = PARTS * 32, first_hi = PARTS * 32;
#pragma unroll
            for (int part = PARTS - 1; part >= 0; --part) {  // descending: ends on the lowest part
                const u64 hit = __ballot(x[part][v] == top);
                const unsigned lo = (unsigned)hit, hi = (unsigned)(hit >> 32);
                if (lo) first_lo = part * 32 + __builtin_ctz(lo);
                if (hi) first_hi = part * 32 + __builtin_ctz(hi);
            }
            if (tile_row(v, h) == c) {  // this lane files candidate list[c]
                mine_top = top;
                mine_first = h ? first_hi : first_lo;
            }
        }
        if (h == ((c >> 2) & 1) && j >= 0 && j < a.m) {
            nn21[(int64_t)b * a.m + j] = mine_first < PARTS * 32 ? (int32_t)(run0 + mine_first) : -1;
            if (s21) s21[(int64_t)b * a.m + j] = mine_top;
        }
    }
}

// ---- reciprocity filter and ordered compaction of the pairs ------------------------------
constexpr int FINAL_THREADS = 1024;

__global__ __launch_bounds__(FINAL_THREADS) void dense_count_kernel(DenseFinalArgs a, int blocks_per_pair) {
    __shared__ int wave_sums[17];
    const int b = blockIdx.y;
    const int i = blockIdx.x * FINAL_THREADS + threadIdx.x;
    bool mutual = false;
    if (i < a.n) {
        const int32_t j = a.nn12[(int64_t)b * a.n + i];
        if (j >= 0 && j < a.m) mutual = a.nn21[(int64_t)b * a.m + j] == i;
    }
    int total;
    block_scan_flag(mutual, wave_sums, total);
    if (threadIdx.x == 0) a.block_counts[(int64_t)b * blocks_per_pair + blockIdx.x] = total;
}

__global__ __launch_bounds__(FINAL_THREADS) void dense_scan_kernel(DenseFinalArgs a, int blocks_per_pair) {
    // exclusive scan of the per-block counts of one pair, in place; total -> n_pairs
    __shared__ int wave_sums[17];
    const int b = blockIdx.x;
    int32_t* counts = a.block_counts + (int64_t)b * blocks_per_pair;
    int running = 0;
    for (int start = 0; start < blocks_per_pair; start += FINAL_THREADS) {
        const int i = start + (int)threadIdx.x;
        const int v = i < blocks_per_pair ? counts[i] : 0;
        int x = v;
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int y = __shfl_up(x, d);
            if (lane >= d) x += y;
        }
        __syncthreads();
        if (lane == 63) wave_sums[wave] = x;
        __syncthreads();
        int offset = 0, sum = 0;
        for (int w = 0; w < FINAL_THREADS / 64; ++w) {
            if (w < wave) offset += wave_sums[w];
            sum += wave_sums[w];
        }
        if (i < blocks_per_pair) counts[i] = running + offset + x - v;
        running += sum;
    }
    if (threadIdx.x == 0) a.n_pairs[b] = running;
}

__global__ __launch_bounds__(FINAL_THREADS) void dense_scatter_kernel(DenseFinalArgs a, int blocks_per_pair) {
    __shared__ int wave_sums[17];
    const int b = blockIdx.y;
    const int i = blockIdx.x * FINAL_THREADS + threadIdx.x;
    const int cap = min(a.n, a.m);
    int32_t* pairs = a.pairs + (int64_t)b * cap * 2;
    bool mutual = false;
    int32_t j = -1;
    if (i < a.n) {
        j = a.nn12[(int64_t)b * a.n + i];
        if (j >= 0 && j < a.m) mutual = a.nn21[(int64_t)b * a.m + j] == i;
    }
    int total;
    const int pos = a.block_counts[(int64_t)b * blocks_per_pair + blockIdx.x] + block_scan_flag(mutual, wave_sums, total);
    if (mutual) {
        pairs[2 * pos + 0] = i;
        pairs[2 * pos + 1] = j;
    }
    // entries past the number of pairs are -1
    const int n_pairs = a.n_pairs[b];
    if (i >= n_pairs && i < cap) {
        pairs[2 * i + 0] = -1;
        pairs[2 * i + 1] = -1;
    }
}

template <int CT, int DP>
static hipError_t launch_dense_t(const DenseArgs& a, int batch, int32_t* nn12, float* s12, int32_t* nn21, float* s21,
                                 hipStream_t s) {
    const int groups = (a.m_tiles + DENSE_TILES_PER_GROUP - 1) / DENSE_TILES_PER_GROUP;
    dim3 grid((groups + a.groups_per_wg - 1) / a.groups_per_wg, (a.n_sb + a.sb_per_wg - 1) / a.sb_per_wg, batch);
    const size_t lds_bytes = ((size_t)a.sb_per_wg * DENSE_S * 32 + DENSE_WAVES * DENSE_J * 32) * sizeof(u64) +
                             DENSE_WAVES * 32 * sizeof(float);  // row keys, column keys, 32 maxima per wave
    hipError_t e;
    if constexpr (DENSE_STAGED && CT != CT_F32 && DP == 24) {
        if (a.sb_per_wg != 1) return hipErrorInvalidValue;  // the staged kernel's key table holds one super-block
        e = launch_detail(TK_DENSE, 1, dense_staged_kernel<CT>, grid, dim3(DENSE_WAVES * 64), 0, s, a);
    } else {
        e = launch(TK_DENSE, dense_kernel<CT, DP>, grid, dim3(DENSE_WAVES * 64), lds_bytes, s, a);
    }
    if (e != hipSuccess) return e;
    const int most = a.n > a.m ? a.n : a.m;
    const size_t hist_bytes = ((size_t)a.row_units + a.col_units) * sizeof(int);
    const bool local = hist_bytes <= 64 * 1024;  // the bucket histogram fits in LDS
    const int per_wg = BUCKET_THREADS * (local ? BUCKET_PER_THREAD : 1);
    const dim3 bucket_grid((most + per_wg - 1) / per_wg, batch);
    if (local)
        e = launch(TK_DENSE_RESOLVE, dense_bucket_count_kernel<true>, bucket_grid, dim3(BUCKET_THREADS), hist_bytes, s, a);
    else
        e = launch(TK_DENSE_RESOLVE, dense_bucket_count_kernel<false>, bucket_grid, dim3(BUCKET_THREADS), 0, s, a);
    if (e != hipSuccess) return e;
    e = launch(TK_DENSE_RESOLVE, dense_bucket_scan_kernel, dim3(2, batch), dim3(BUCKET_THREADS), 0, s, a);
    if (e != hipSuccess) return e;
    if (local)
        e = launch(TK_DENSE_RESOLVE, dense_bucket_fill_kernel<true>, bucket_grid, dim3(BUCKET_THREADS), hist_bytes, s, a,
                   nn12, s12, nn21, s21);
    else
        e = launch(TK_DENSE_RESOLVE, dense_bucket_fill_kernel<false>, bucket_grid, dim3(BUCKET_THREADS), 0, s, a, nn12,
                   s12, nn21, s21);
    if (e != hipSuccess) return e;
    const int cap = 4096 / batch > 64 ? 4096 / batch : 64;
    int wgs = (int)((a.rows_cap / 32 + 3) / 4);
    if (wgs > cap) wgs = cap;
    e = launch(TK_DENSE_RESOLVE, dense_resolve_rows_kernel<CT, DP>, dim3(wgs, batch), dim3(256), 0, s, a, nn12, s12);
    if (e != hipSuccess) return e;
    wgs = (int)((a.cols_cap / 32 + 3) / 4);
    if (wgs > cap) wgs = cap;
    return launch(TK_DENSE_RESOLVE, dense_resolve_cols_kernel<CT, DP>, dim3(wgs, batch), dim3(256), 0, s, a, nn21, s21);
}

hipError_t launch_dense(const DenseArgs& a, int batch, int compute, int dp, int32_t* nn12, float* s12, int32_t* nn21,
                        float* s21, hipStream_t s) {
    if (a.n <= 0 || a.m <= 0 || batch <= 0) return hipSuccess;
    if (compute == FNN_F16) {
        if (dp == 16) return launch_dense_t<CT_F16, 16>(a, batch, nn12, s12, nn21, s21, s);
        if (dp == 24) return launch_dense_t<CT_F16, 24>(a, batch, nn12, s12, nn21, s21, s);
        if (dp == 32) return launch_dense_t<CT_F16, 32>(a, batch, nn12, s12, nn21, s21, s);
        if (dp == 48) return launch_dense_t<CT_F16, 48>(a, batch, nn12, s12, nn21, s21, s);
        if (dp == 64) return launch_dense_t<CT_F16, 64>(a, batch, nn12, s12, nn21, s21, s);
        if (dp == 80) return launch_dense_t<CT_F16, 80>(a, batch, nn12, s12, nn21, s21, s);
        if (dp == 96) return launch_dense_t<CT_F16, 96>(a, batch, nn12, s12, nn21, s21, s);
    } else if (compute == FNN_BF16) {
        if (dp == 16) return launch_dense_t<CT_BF16, 16>(a, batch, nn12, s12, nn21, s21, s);
        if (dp == 24) return launch_dense_t<CT_BF16, 24>(a, batch, nn12, s12, nn21, s21, s);
        if (dp == 32) return launch_dense_t<CT_BF16, 32>(a, batch, nn12, s12, nn21, s21, s);
    } else {
        if (dp == 8) return launch_dense_t<CT_F32, 8>(a, batch, nn12, s12, nn21, s21, s);
        if (dp == 16) return launch_dense_t<CT_F32, 16>(a, batch, nn12, s12, nn21, s21, s);
        if (dp == 24) return launch_dense_t<CT_F32, 24>(a, batch, nn12, s12, nn21, s21, s);
        if (dp == 32) return launch_dense_t<CT_F32, 32>(a, batch, nn12, s12, nn21, s21, s);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_dense_final(const DenseFinalArgs& a, int batch, hipStream_t s) {
    const int most = a.n > a.m ? a.n : a.m;
    const int blocks = (most + FINAL_THREADS - 1) / FINAL_THREADS;
    if (blocks == 0 || batch <= 0) return hipSuccess;
    hipError_t e = launch(TK_DENSE_FINAL, dense_count_kernel, dim3(blocks, batch), dim3(FINAL_THREADS), 0, s, a, blocks);
    if (e != hipSuccess) return e;
    e = launch(TK_DENSE_FINAL, dense_scan_kernel, dim3(batch), dim3(FINAL_THREADS), 0, s, a, blocks);
    if (e != hipSuccess) return e;
    return launch(TK_DENSE_FINAL, dense_scatter_kernel, dim3(blocks, batch), dim3(FINAL_THREADS), 0, s, a, blocks);
}

}  // namespace fnn
