// One-directional nearest-neighbour search: the single loop of Algorithm 2 ("FastNN-Lite",
// section 3.4.3) with its distance block fused away.  Each wave keeps a few 32-query blocks
// resident in registers, streams candidate tiles past them, forms every 32x32 block of
// scores with matrix instructions (fp32 accumulation, Algorithm 3) and folds it at once into
// a per-query running best, so no score ever leaves the register file and memory traffic is
// one pass over the candidate map per resident query group.
//
// Work split (decided on the device from the live query count, so the host never needs to
// read it back): the queries form row groups of R*32, the candidate tiles are cut into
// chunks, one wave takes one (row group, chunk) unit and merges its result into the packed
// keys with a 64-bit atomic max (score first, lowest index on ties).
#include "fnn_device.hpp"
#include "fnn_kernels.hpp"
#include "trace.hpp"

namespace fnn {

constexpr int SEARCH_R = 4;           // 32-query blocks resident per wave
constexpr int SEARCH_MIN_TILES = 4;   // shortest chunk worth a wave
constexpr int SEARCH_WAVES = 4;       // waves per workgroup

template <int CT, int DP, int R>
__global__ __launch_bounds__(SEARCH_WAVES * 64) void search_kernel(SearchArgs a) {
    using O = Ops<CT, DP>;
    using Frag = typename O::Frag;
    const int lane = threadIdx.x & 63, c = lane & 31, h = lane >> 5;
    const int wave = blockIdx.x * SEARCH_WAVES + (threadIdx.x >> 6);
    const int n_waves = gridDim.x * SEARCH_WAVES;
    const int b = blockIdx.y;

    int n_act = a.nq;
    if (a.nq_active) n_act = min(max(a.nq_active[b], 0), a.nq);
    if (n_act <= 0 || a.m_tiles <= 0) return;

    const int row_groups = (n_act + 32 * R - 1) / (32 * R);
    int chunks = max(1, n_waves / row_groups);
    int tiles_per_chunk = max((a.m_tiles + chunks - 1) / chunks, SEARCH_MIN_TILES);
    chunks = (a.m_tiles + tiles_per_chunk - 1) / tiles_per_chunk;

    const char* src = a.src + (int64_t)b * a.src_bstride;
    const char* tgt = a.tgt + (int64_t)b * a.tgt_bstride;
    const int64_t qbase = (int64_t)b * a.nq;
    const float ninf = -__builtin_inff();

    const int64_t units = (int64_t)row_groups * chunks;
    for (int64_t unit = wave; unit < units; unit += n_waves) {
        const int chunk = (int)(unit / row_groups);
        const int rg = (int)(unit % row_groups);
        const int slot0 = rg * 32 * R;
        const int n_blk = min(R, (n_act - slot0 + 31) / 32);

        Frag q[R];
        float best[R];
        int best_j[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int slot = slot0 + r * 32 + c;
            int64_t row = 0;
            if (slot < n_act) {
                if (a.q_keys) row = (int64_t)(0xFFFFFFFFu - (uint32_t)(a.q_keys[qbase + slot] & 0xFFFFFFFFull));
                else if (a.q_idx) row = a.q_idx[qbase + slot];
                else row = slot;
            }
            row = min(max(row, (int64_t)0), (int64_t)a.src_rows - 1);  // never read outside the map
            q[r] = O::load(src + row * O::ROW_BYTES, h);
            best[r] = ninf;
            best_j[r] = 0x7FFFFFFF;
        }

        const int t0 = chunk * tiles_per_chunk;
        const int t1 = min(t0 + tiles_per_chunk, a.m_tiles);
        Frag cur = O::load(tgt + ((int64_t)t0 * 32 + c) * O::ROW_BYTES, h);
        for (int t = t0; t < t1; ++t) {
            Frag nxt = cur;
            if (t + 1 < t1) nxt = O::load(tgt + ((int64_t)(t + 1) * 32 + c) * O::ROW_BYTES, h);
            const int jbase = t * 32;
            const bool tail = jbase + 32 > a.m;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                if (r < n_blk) {
                    f32x16 acc = O::mma(cur, q[r]);
                    if (tail) {
#pragma unroll
                        for (int v = 0; v < 16; ++v)
                            if (jbase + tile_row(v, h) >= a.m) acc[v] = ninf;
                    }
                    // ascending v is ascending candidate index inside the lane; strict ">"
                    // keeps the lowest index among equal scores
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        if (acc[v] > best[r]) {
                            best[r] = acc[v];
                            best_j[r] = jbase + tile_row(v, h);
                        }
                    }
                }
            }
            cur = nxt;
        }

#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (r < n_blk) {
                const float ob = __shfl_xor(best[r], 32);
                const int oj = __shfl_xor(best_j[r], 32);
                if (ob > best[r] || (ob == best[r] && oj < best_j[r])) {
                    best[r] = ob;
                    best_j[r] = oj;
                }
                const int slot = slot0 + r * 32 + c;
                if (h == 0 && slot < n_act) atomicMax(&a.out_keys[qbase + slot], pack_key(best[r], best_j[r]));
            }
        }
    }
}

__global__ __launch_bounds__(256) void decode_kernel(DecodeArgs a) {
    const int b = blockIdx.y;
    int n_act = a.nq;
    if (a.nq_active) n_act = min(max(a.nq_active[b], 0), a.nq);
    for (int q = blockIdx.x * blockDim.x + threadIdx.x; q < n_act; q += gridDim.x * blockDim.x) {
        const u64 k = a.keys[(int64_t)b * a.nq + q];
        a.out_idx[(int64_t)b * a.nq + q] = key_index(k);
        if (a.out_score) a.out_score[(int64_t)b * a.nq + q] = key_score(k);
    }
}

template <int CT, int DP>
static hipError_t launch_search_t(const SearchArgs& a, int batch, hipStream_t s) {
    // enough waves to occupy every SIMD several times over, shared between the pairs
    int wgs = 2048 / batch;
    if (wgs < 128) wgs = 128;
    const int64_t max_units = (int64_t)((a.nq + 32 * SEARCH_R - 1) / (32 * SEARCH_R)) *
                              ((a.m_tiles + SEARCH_MIN_TILES - 1) / SEARCH_MIN_TILES);
    const int64_t need = (max_units + SEARCH_WAVES - 1) / SEARCH_WAVES;
    if (need < wgs) wgs = (int)(need > 0 ? need : 1);
    return launch(TK_SEARCH, search_kernel<CT, DP, SEARCH_R>, dim3(wgs, batch), dim3(SEARCH_WAVES * 64), 0, s, a);
}

hipError_t launch_search(const SearchArgs& a, int batch, int compute, int dp, hipStream_t s) {
    if (a.nq <= 0 || batch <= 0) return hipSuccess;
    if (compute == FNN_F16) {
        if (dp == 16) return launch_search_t<CT_F16, 16>(a, batch, s);
        if (dp == 32) return launch_search_t<CT_F16, 32>(a, batch, s);
    } else if (compute == FNN_BF16) {
        if (dp == 16) return launch_search_t<CT_BF16, 16>(a, batch, s);
        if (dp == 32) return launch_search_t<CT_BF16, 32>(a, batch, s);
    } else {
        if (dp == 8) return launch_search_t<CT_F32, 8>(a, batch, s);
        if (dp == 16) return launch_search_t<CT_F32, 16>(a, batch, s);
        if (dp == 24) return launch_search_t<CT_F32, 24>(a, batch, s);
        if (dp == 32) return launch_search_t<CT_F32, 32>(a, batch, s);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_decode(const DecodeArgs& a, int batch, hipStream_t s) {
    if (a.nq <= 0 || batch <= 0) return hipSuccess;
    int blocks = (a.nq + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    return launch(TK_DECODE, decode_kernel, dim3(blocks, batch), dim3(256), 0, s, a);
}

}  // namespace fnn
