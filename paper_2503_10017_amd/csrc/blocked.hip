// The paper's own two search schedules, kept as a measurable contrast to the fused search:
// Algorithm 1 ("Original FastNN": a double loop over blocks of A and blocks of B) and
// Algorithm 2 ("FastNN-Lite": a single loop over blocks of A against the whole of B), each
// as a host-driven sequence of two kernels per block -- dist_func writes the block of scores
// to memory, a second kernel selects from it -- the way a tensor framework runs them.  The
// results are identical to the fused search; only the schedule and the memory traffic differ
// (section 3.4.3, Figure 2: block accesses (P/BS)^2 versus P/BS).
#include <hip/hip_fp16.h>

#include "fnn_device.hpp"
#include "fnn_kernels.hpp"
#include "trace.hpp"

namespace fnn {

// dists[q][j] = score(query q0+q, candidate j0+j) for a block of queries and a range of
// candidate tiles; one wave per (32 queries, 32 candidates) product.  The queries take the
// row side of the matrix instruction here, so that a result register holds 32 consecutive
// candidates of one query and the stores are contiguous.
template <int CT, int DP>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2)))
void blocked_scores_kernel(BlockedArgs a, int q0, int nq_blk, int tile0, int n_tiles) {
    using O = Ops<CT, DP>;
    using Frag = typename O::Frag;
    const int lane = threadIdx.x & 63, c = lane & 31, h = lane >> 5;
    const int wave = blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int q_blocks = (nq_blk + 31) / 32;
    const int64_t units = (int64_t)q_blocks * n_tiles;
    for (int64_t unit = wave; unit < units; unit += (int64_t)gridDim.x * 4) {
        const int qb = (int)(unit / n_tiles), t = tile0 + (int)(unit % n_tiles);
        const int slot = q0 + qb * 32 + c;
        int64_t row = 0;
        if (slot < a.nq) row = a.q_idx ? a.q_idx[slot] : slot;
        row = min(max(row, (int64_t)0), (int64_t)a.src_rows - 1);
        const Frag qf = O::load(a.src + row * O::ROW_BYTES, h);
        const Frag cf = O::load(a.tgt + ((int64_t)t * 32 + c) * O::ROW_BYTES, h);
        const f32x16 acc = O::mma(qf, cf);  // register v of lane (c, h): query tile_row(v, h), candidate c
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int q_local = qb * 32 + tile_row(v, h);
            if (q_local < nq_blk) a.dists[(int64_t)q_local * a.ld + (int64_t)(t - tile0) * 32 + c] = acc[v];
        }
    }
}

// Negative control: the same score block with every product rounded to fp16 and the sum kept
// in fp16 (k ascending, separate multiply and add), one thread per (query, candidate).
template <int DP>
__global__ __launch_bounds__(256) void blocked_scores_half_kernel(BlockedArgs a, int q0, int nq_blk, int tile0, int n_tiles,
                                                                  int d) {
    const int64_t width = (int64_t)n_tiles * 32;
    const int64_t total = (int64_t)nq_blk * width;
    for (int64_t item = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; item < total; item += (int64_t)gridDim.x * blockDim.x) {
        const int q_local = (int)(item / width);
        const int64_t j_local = item % width;
        const int slot = q0 + q_local;
        int64_t row = a.q_idx ? a.q_idx[slot] : slot;
        row = min(max(row, (int64_t)0), (int64_t)a.src_rows - 1);
        const _Float16* qa = reinterpret_cast<const _Float16*>(a.src + row * (DP * 2));
        const _Float16* cb = reinterpret_cast<const _Float16*>(a.tgt + ((int64_t)tile0 * 32 + j_local) * (DP * 2));
        _Float16 acc = (_Float16)0.0f;
        for (int k = 0; k < d; ++k) {
#pragma clang fp contract(off)
            const _Float16 p = qa[k] * cb[k];  // rounded to binary16 here: no contraction in this scope
            acc = acc + p;
        }
        a.dists[(int64_t)q_local * a.ld + j_local] = (float)acc;
    }
}

// nearest_idx / min_dist update of Algorithm 1 (and the argmin of Algorithm 2): one wave per
// query scans its row of the score block in ascending candidate order and replaces the
// running best only on a strict improvement.
__global__ __launch_bounds__(256) void blocked_select_kernel(BlockedArgs a, int q0, int nq_blk, int j0, int width,
                                                              int first_block) {
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * 4 + (threadIdx.x >> 6);
    for (int q = wave; q < nq_blk; q += gridDim.x * 4) {
        const float* row = a.dists + (int64_t)q * a.ld;
        float best = -__builtin_inff();
        int best_j = 0x7FFFFFFF;
        for (int j = lane; j < width; j += 64) {
            const float s = (j0 + j < a.m) ? row[j] : -__builtin_inff();
            if (s > best) {  // ascending j within the lane: lowest index among equals
                best = s;
                best_j = j0 + j;
            }
        }
#pragma unroll
        for (int mask = 1; mask < 64; mask <<= 1) {
            const float ob = __shfl_xor(best, mask);
            const int oj = __shfl_xor(best_j, mask);
            if (ob > best || (ob == best && oj < best_j)) {
                best = ob;
                best_j = oj;
            }
        }
        if (lane == 0 && best_j != 0x7FFFFFFF) {
            const int slot = q0 + q;
            if (first_block || best > a.out_score[slot]) {  // later blocks hold higher indices: strict ">"
                a.out_score[slot] = best;
                a.out_idx[slot] = best_j;
            }
        }
    }
}

template <int CT, int DP>
static hipError_t run_blocked_t(const BlockedArgs& a, int d, int block_rows, int block_cols, hipStream_t s) {
    const int m_tiles = (a.m + 31) / 32;
    const int col_tiles = block_cols > 0 ? (block_cols + 31) / 32 : m_tiles;  // 0: the whole of B at once
    for (int q0 = 0; q0 < a.nq; q0 += block_rows) {                           // loop over blocks of A
        const int nq_blk = a.nq - q0 < block_rows ? a.nq - q0 : block_rows;
        for (int t0 = 0; t0 < m_tiles; t0 += col_tiles) {                     // loop over blocks of B (one trip for Alg. 2)
            const int n_tiles = m_tiles - t0 < col_tiles ? m_tiles - t0 : col_tiles;
            const int64_t units = (int64_t)((nq_blk + 31) / 32) * n_tiles;
            int wgs = (int)((units + 3) / 4 < 8192 ? (units + 3) / 4 : 8192);
            hipError_t e;
            if (CT == CT_F16 && a.half_accumulate)
                e = launch(TK_BLOCKED, blocked_scores_half_kernel<DP>, dim3(8192), dim3(256), 0, s, a, q0, nq_blk, t0, n_tiles, d);
            else
                e = launch(TK_BLOCKED, blocked_scores_kernel<CT, DP>, dim3(wgs), dim3(256), 0, s, a, q0, nq_blk, t0, n_tiles);
            if (e != hipSuccess) return e;
            wgs = (nq_blk + 3) / 4;
            e = launch(TK_BLOCKED, blocked_select_kernel, dim3(wgs), dim3(256), 0, s, a, q0, nq_blk, t0 * 32, n_tiles * 32,
                       t0 == 0 ? 1 : 0);
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

hipError_t run_blocked(const BlockedArgs& a, int compute, int d, int dp, int block_rows, int block_cols, hipStream_t s) {
    if (a.nq <= 0 || a.m <= 0) return hipSuccess;
    if (compute == FNN_F16) {
        if (dp == 16) return run_blocked_t<CT_F16, 16>(a, d, block_rows, block_cols, s);
        if (dp == 24) return run_blocked_t<CT_F16, 24>(a, d, block_rows, block_cols, s);
        if (dp == 32) return run_blocked_t<CT_F16, 32>(a, d, block_rows, block_cols, s);
    } else if (compute == FNN_BF16) {
        if (dp == 16) return run_blocked_t<CT_BF16, 16>(a, d, block_rows, block_cols, s);
        if (dp == 24) return run_blocked_t<CT_BF16, 24>(a, d, block_rows, block_cols, s);
        if (dp == 32) return run_blocked_t<CT_BF16, 32>(a, d, block_rows, block_cols, s);
    } else {
        if (dp == 8) return run_blocked_t<CT_F32, 8>(a, d, block_rows, block_cols, s);
        if (dp == 16) return run_blocked_t<CT_F32, 16>(a, d, block_rows, block_cols, s);
        if (dp == 24) return run_blocked_t<CT_F32, 24>(a, d, block_rows, block_cols, s);
        if (dp == 32) return run_blocked_t<CT_F32, 32>(a, d, block_rows, block_cols, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace fnn
