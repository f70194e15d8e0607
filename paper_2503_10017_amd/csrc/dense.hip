// All-pairs mutual nearest neighbours (paper section 3.2, "Problem Context"): every score
// S[i][j] = <D1[i], D2[j]> is formed exactly once on the matrix cores and folded, while it
// is still in a register, into BOTH running maxima -- the best candidate j of query i and
// the best query i of candidate j -- so the quadratic score matrix never exists in memory.
//
// A wave keeps J candidate tiles (32 pixels of D2 each) resident together with one running
// best per resident candidate and result lane, and sweeps the workgroup's query range past
// them.  Per query block the best candidate over the wave's tiles goes into a per-workgroup
// key table in LDS; after the sweep the per-candidate bests are reduced across lanes and
// merged into the global key table; the LDS table is merged into the global one at the end.
// All merges are 64-bit max operations on (score, inverted index) keys.
#include "fnn_device.hpp"
#include "fnn_kernels.hpp"
#include "trace.hpp"

namespace fnn {


template <int CT, int DP, int J>
__global__ __launch_bounds__(DENSE_WAVES * 64) void dense_kernel(DenseArgs a) {
    using O = Ops<CT, DP>;
    using Frag = typename O::Frag;
    extern __shared__ u64 lds_row_keys[];  // [q_per_wg]

    const int lane = threadIdx.x & 63, c = lane & 31, h = lane >> 5;
    const int wave = threadIdx.x >> 6;
    const int b = blockIdx.z;
    const float ninf = -__builtin_inff();

    const int q0 = blockIdx.y * a.q_per_wg;                       // first query of this workgroup
    const int q_blocks = min(a.q_per_wg / 32, a.n_blocks - q0 / 32);
    const int tiles_per_group = DENSE_WAVES * J;
    const int tile0 = blockIdx.x * a.groups_per_wg * tiles_per_group;

    for (int i = threadIdx.x; i < a.q_per_wg; i += blockDim.x) lds_row_keys[i] = 0;
    __syncthreads();

    const char* d1 = a.d1 + (int64_t)b * a.d1_bstride;
    const char* d2 = a.d2 + (int64_t)b * a.d2_bstride;
    u64* row_keys = a.row_keys + (int64_t)b * a.n;
    u64* col_keys = a.col_keys + (int64_t)b * a.m;

    for (int g = 0; g < a.groups_per_wg; ++g) {
        const int tbase = tile0 + g * tiles_per_group + wave * J;
        if (tbase >= a.m_tiles) break;  // uniform per wave; no barrier inside this loop

        Frag cand[J];
        float cbest[J][16];
        int cblk[J][16];
#pragma unroll
        for (int jt = 0; jt < J; ++jt) {
            const int t = min(tbase + jt, a.m_tiles - 1);
            cand[jt] = O::load(d2 + ((int64_t)t * 32 + c) * O::ROW_BYTES, h);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                cbest[jt][v] = ninf;
                cblk[jt][v] = 0;
            }
        }

        for (int ib = 0; ib < q_blocks; ++ib) {
            const int i = q0 + ib * 32 + c;  // this lane's query
            const Frag q = O::load(d1 + (int64_t)i * O::ROW_BYTES, h);
            const bool q_valid = i < a.n;
            float rbest = ninf;
            int rj = 0x7FFFFFFF;
#pragma unroll
            for (int jt = 0; jt < J; ++jt) {
                const int t = tbase + jt;
                if (t < a.m_tiles) {
                    f32x16 acc = O::mma(cand[jt], q);
                    const int jbase = t * 32;
                    if (!q_valid) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) acc[v] = ninf;
                    }
                    if (jbase + 32 > a.m) {
#pragma unroll
                        for (int v = 0; v < 16; ++v)
                            if (jbase + tile_row(v, h) >= a.m) acc[v] = ninf;
                    }
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        // best candidate of this query: ascending v, ascending jt = ascending j
                        if (acc[v] > rbest) {
                            rbest = acc[v];
                            rj = jbase + tile_row(v, h);
                        }
                        // best query of this candidate: ascending ib = ascending i in this lane
                        if (acc[v] > cbest[jt][v]) {
                            cbest[jt][v] = acc[v];
                            cblk[jt][v] = ib;
                        }
                    }
                }
            }
            const float ob = __shfl_xor(rbest, 32);
            const int oj = __shfl_xor(rj, 32);
            if (ob > rbest || (ob == rbest && oj < rj)) {
                rbest = ob;
                rj = oj;
            }
            if (h == 0 && q_valid && rj != 0x7FFFFFFF)
                atomicMax(&lds_row_keys[ib * 32 + c], pack_key(rbest, rj));
        }

        // per-candidate bests: reduce over the 32 lanes (queries) of each half, then merge
#pragma unroll
        for (int jt = 0; jt < J; ++jt) {
            const int t = tbase + jt;
            if (t < a.m_tiles) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    u64 key = 0;
                    if (cbest[jt][v] != ninf) key = pack_key(cbest[jt][v], q0 + cblk[jt][v] * 32 + c);
#pragma unroll
                    for (int mask = 1; mask < 32; mask <<= 1) {
                        const u64 other = shfl_xor_u64(key, mask);
                        key = other > key ? other : key;
                    }
                    const int j = t * 32 + tile_row(v, h);
                    if (c == 0 && j < a.m && key) atomicMax(&col_keys[j], key);
                }
            }
        }
    }

    __syncthreads();
    for (int i = threadIdx.x; i < a.q_per_wg; i += blockDim.x) {
        const u64 key = lds_row_keys[i];
        if (key && q0 + i < a.n) atomicMax(&row_keys[q0 + i], key);
    }
}

// ---- decode the key tables, apply the reciprocity filter, compact the pairs in order ----
constexpr int FINAL_THREADS = 1024;

__global__ __launch_bounds__(FINAL_THREADS) void dense_decode_kernel(DenseFinalArgs a, int blocks_per_pair) {
    __shared__ int wave_sums[17];
    const int b = blockIdx.y;
    const int i = blockIdx.x * FINAL_THREADS + threadIdx.x;
    const u64* row_keys = a.row_keys + (int64_t)b * a.n;
    const u64* col_keys = a.col_keys + (int64_t)b * a.m;
    bool mutual = false;
    if (i < a.n) {
        const u64 k = row_keys[i];
        const int32_t j = key_index(k);
        a.nn12[(int64_t)b * a.n + i] = j;
        if (a.s12) a.s12[(int64_t)b * a.n + i] = key_score(k);
        if (j >= 0 && j < a.m) mutual = key_index(col_keys[j]) == i;
    }
    if (i < a.m) {
        const u64 k = col_keys[i];
        a.nn21[(int64_t)b * a.m + i] = key_index(k);
        if (a.s21) a.s21[(int64_t)b * a.m + i] = key_score(k);
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
        // inclusive scan inside the wave, then across waves
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
static hipError_t launch_dense_t(const DenseArgs& a, int batch, hipStream_t s) {
    const int tiles_per_wg = a.groups_per_wg * DENSE_WAVES * DENSE_J;
    dim3 grid((a.m_tiles + tiles_per_wg - 1) / tiles_per_wg, (a.n_blocks * 32 + a.q_per_wg - 1) / a.q_per_wg, batch);
    return launch(TK_DENSE, dense_kernel<CT, DP, DENSE_J>, grid, dim3(DENSE_WAVES * 64),
                  (size_t)a.q_per_wg * sizeof(u64), s, a);
}

hipError_t launch_dense(const DenseArgs& a, int batch, int compute, int dp, hipStream_t s) {
    if (a.n <= 0 || a.m <= 0 || batch <= 0) return hipSuccess;
    if (compute == FNN_F16) {
        if (dp == 16) return launch_dense_t<CT_F16, 16>(a, batch, s);
        if (dp == 32) return launch_dense_t<CT_F16, 32>(a, batch, s);
    } else if (compute == FNN_BF16) {
        if (dp == 16) return launch_dense_t<CT_BF16, 16>(a, batch, s);
        if (dp == 32) return launch_dense_t<CT_BF16, 32>(a, batch, s);
    } else {
        if (dp == 8) return launch_dense_t<CT_F32, 8>(a, batch, s);
        if (dp == 16) return launch_dense_t<CT_F32, 16>(a, batch, s);
        if (dp == 24) return launch_dense_t<CT_F32, 24>(a, batch, s);
        if (dp == 32) return launch_dense_t<CT_F32, 32>(a, batch, s);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_dense_final(const DenseFinalArgs& a, int batch, hipStream_t s) {
    const int most = a.n > a.m ? a.n : a.m;
    const int blocks = (most + FINAL_THREADS - 1) / FINAL_THREADS;
    if (blocks == 0 || batch <= 0) return hipSuccess;
    hipError_t e = launch(TK_DENSE_FINAL, dense_decode_kernel, dim3(blocks, batch), dim3(FINAL_THREADS), 0, s, a, blocks);
    if (e != hipSuccess) return e;
    e = launch(TK_DENSE_FINAL, dense_scan_kernel, dim3(batch), dim3(FINAL_THREADS), 0, s, a, blocks);
    if (e != hipSuccess) return e;
    return launch(TK_DENSE_FINAL, dense_scatter_kernel, dim3(blocks, batch), dim3(FINAL_THREADS), 0, s, a, blocks);
}

}  // namespace fnn
