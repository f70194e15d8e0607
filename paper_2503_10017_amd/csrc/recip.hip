// Bookkeeping of the FastNN iteration (paper section 3.2, "FastNN Algorithm", steps 1-4):
// the reciprocity test U^{t+1} == U^t, the removal of converged seeds by a prefix-sum
// compaction of the ones still moving, and the final reduction of the matches to a sorted
// set.  Everything lives on the device: the host enqueues a fixed sequence of kernels and
// never reads a count back.
#include "fnn_device.hpp"
#include "fnn_kernels.hpp"
#include "trace.hpp"

namespace fnn {

constexpr int STEP_THREADS = 1024;

__global__ __launch_bounds__(256) void recip_init_kernel(RecipState st, const int32_t* seeds, int32_t n_seeds) {
    const int b = blockIdx.y;
    const int64_t base = (int64_t)b * n_seeds;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n_seeds; i += gridDim.x * blockDim.x) {
        st.cur_u[0][base + i] = seeds[base + i];
        st.seed_id[0][base + i] = i;
        st.keys_f[base + i] = 0;
        st.keys_b[base + i] = 0;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) st.n_active[b] = n_seeds;
}

struct StepArgs {
    const int32_t* cur_u;     // U^t per slot
    const int32_t* seed_id;
    int32_t* next_u;          // U^{t+1} of the survivors, compacted
    int32_t* next_seed_id;
    int32_t* n_active;
    u64* keys_f;              // V^t per slot (index field); cleared for the next search
    u64* keys_b;              // U^{t+1} per slot; cleared for the next search
    int32_t n_seeds;
    int32_t t;
    int32_t mode;
    int32_t* seed_i;
    int32_t* seed_j;
    int32_t* seed_iter;
};

// One workgroup per image pair walks the live slots in order, so survivors keep their
// relative order (the result does not depend on it, but runs are reproducible).
__global__ __launch_bounds__(STEP_THREADS) void recip_step_kernel(StepArgs a) {
    __shared__ int wave_sums[17];
    const int b = blockIdx.x;
    const int64_t base = (int64_t)b * a.n_seeds;
    const int n_act = min(max(a.n_active[b], 0), a.n_seeds);
    int kept = 0;
    for (int start = 0; start < n_act; start += STEP_THREADS) {
        const int slot = start + (int)threadIdx.x;
        bool survive = false;
        int32_t u_next = 0, sid = 0;
        if (slot < n_act) {
            const u64 kf = a.keys_f[base + slot];
            const u64 kb = a.keys_b[base + slot];
            const int32_t u = a.cur_u[base + slot];
            sid = a.seed_id[base + slot];
            const int32_t v = key_index(kf);
            u_next = key_index(kb);
            const bool converged = (a.mode != 2) && (u_next == u);
            if (converged) {
                a.seed_i[base + sid] = u;
                a.seed_j[base + sid] = v;
                a.seed_iter[base + sid] = a.t;
            } else if (a.mode != 0) {
                a.seed_i[base + sid] = u;
                a.seed_j[base + sid] = v;
                a.seed_iter[base + sid] = -1;
            } else {
                survive = true;
            }
            a.keys_f[base + slot] = 0;
            a.keys_b[base + slot] = 0;
        }
        int total;
        const int pos = kept + block_scan_flag(survive, wave_sums, total);
        if (survive) {
            a.next_u[base + pos] = u_next;
            a.next_seed_id[base + pos] = sid;
        }
        kept += total;
    }
    __syncthreads();
    if (threadIdx.x == 0) a.n_active[b] = (a.mode == 0) ? kept : 0;
}

struct DedupArgs {
    const int32_t* seed_i;
    const int32_t* seed_j;
    const int32_t* seed_iter;
    int32_t n_seeds;
    int32_t n_sort;     // power of two >= n_seeds
    u64* global_buf;    // [batch][n_sort] when the keys do not fit in LDS, else NULL
    int32_t* pairs;
    int32_t* n_pairs;
};

// Sort the keys (i << 32 | j) of the converged seeds with a bitonic network, then keep the
// first of every run: the match set M, ascending in (i, j).
__global__ __launch_bounds__(STEP_THREADS) void recip_dedup_kernel(DedupArgs a) {
    extern __shared__ u64 lds_buf[];
    __shared__ int wave_sums[17];
    const int b = blockIdx.x;
    const int64_t base = (int64_t)b * a.n_seeds;
    u64* buf = a.global_buf ? a.global_buf + (int64_t)b * a.n_sort : lds_buf;
    const u64 none = ~0ull;

    for (int i = threadIdx.x; i < a.n_sort; i += STEP_THREADS) {
        u64 k = none;
        if (i < a.n_seeds && a.seed_iter[base + i] >= 0)
            k = ((u64)(uint32_t)a.seed_i[base + i] << 32) | (u64)(uint32_t)a.seed_j[base + i];
        buf[i] = k;
    }
    __syncthreads();
    for (int k = 2; k <= a.n_sort; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = threadIdx.x; i < a.n_sort; i += STEP_THREADS) {
                const int partner = i ^ j;
                if (partner > i) {
                    const u64 x = buf[i], y = buf[partner];
                    const bool ascending = (i & k) == 0;
                    if ((x > y) == ascending) {
                        buf[i] = y;
                        buf[partner] = x;
                    }
                }
            }
            __syncthreads();
        }
    }
    int count = 0;
    for (int start = 0; start < a.n_sort; start += STEP_THREADS) {
        const int i = start + (int)threadIdx.x;
        u64 k = none;
        bool first = false;
        if (i < a.n_sort) {
            k = buf[i];
            first = (k != none) && (i == 0 || buf[i - 1] != k);
        }
        int total;
        const int pos = count + block_scan_flag(first, wave_sums, total);
        if (first) {
            a.pairs[(base + pos) * 2 + 0] = (int32_t)(k >> 32);
            a.pairs[(base + pos) * 2 + 1] = (int32_t)(k & 0xFFFFFFFFull);
        }
        count += total;
    }
    for (int i = count + threadIdx.x; i < a.n_seeds; i += STEP_THREADS) {
        a.pairs[(base + i) * 2 + 0] = -1;
        a.pairs[(base + i) * 2 + 1] = -1;
    }
    if (threadIdx.x == 0) a.n_pairs[b] = count;
}

hipError_t launch_recip_init(const RecipState& st, const int32_t* seeds, int32_t n_seeds, int batch, hipStream_t s) {
    int blocks = (n_seeds + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 256) blocks = 256;
    return launch(TK_RECIP_INIT, recip_init_kernel, dim3(blocks, batch), dim3(256), 0, s, st, seeds, n_seeds);
}

hipError_t launch_recip_step(const RecipState& st, int which, int32_t n_seeds, int batch, int t, int mode,
                             int32_t* seed_i, int32_t* seed_j, int32_t* seed_iter, hipStream_t s) {
    StepArgs a;
    a.cur_u = st.cur_u[which];
    a.seed_id = st.seed_id[which];
    a.next_u = st.cur_u[which ^ 1];
    a.next_seed_id = st.seed_id[which ^ 1];
    a.n_active = st.n_active;
    a.keys_f = st.keys_f;
    a.keys_b = st.keys_b;
    a.n_seeds = n_seeds;
    a.t = t;
    a.mode = mode;
    a.seed_i = seed_i;
    a.seed_j = seed_j;
    a.seed_iter = seed_iter;
    return launch(TK_RECIP_STEP, recip_step_kernel, dim3(batch), dim3(STEP_THREADS), 0, s, a);
}

hipError_t launch_recip_dedup(const RecipState& st, int32_t n_seeds, int batch,
                              const int32_t* seed_i, const int32_t* seed_j, const int32_t* seed_iter,
                              int32_t* pairs, int32_t* n_pairs, hipStream_t s) {
    DedupArgs a;
    a.seed_i = seed_i;
    a.seed_j = seed_j;
    a.seed_iter = seed_iter;
    a.n_seeds = n_seeds;
    a.n_sort = (int32_t)st.sort_len;
    a.pairs = pairs;
    a.n_pairs = n_pairs;
    const size_t lds_bytes = (size_t)st.sort_len * sizeof(u64);
    const bool in_lds = lds_bytes <= 48 * 1024;
    a.global_buf = in_lds ? nullptr : st.sort_buf;
    return launch(TK_RECIP_DEDUP, recip_dedup_kernel, dim3(batch), dim3(STEP_THREADS), in_lds ? lds_bytes : 0, s, a);
}

}  // namespace fnn
