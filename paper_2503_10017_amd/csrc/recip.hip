// Bookkeeping of the FastNN iteration (paper section 3.2.5, "FastNN Algorithm", steps 1-4):
// the reciprocity test U^{t+1} == U^t, the removal of converged seeds by a prefix-sum
// compaction of the ones still moving, and the final reduction of the matches to a sorted
// set (a distribution sort over the pixel range).  Everything lives on the device: the host enqueues a fixed sequence of kernels and
// never reads a count back.
#include "fnn_device.hpp"
#include "fnn_kernels.hpp"
#include "trace.hpp"

namespace fnn {

constexpr int STEP_THREADS = 1024;
constexpr size_t DEDUP_LDS_BYTES = 60 * 1024;  // dynamic LDS a launch may ask for without raising the kernel's limit (64 KB incl. static)

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
    int32_t n_words;      // ceil(n / 32): words of the per-pair pixel bitmap
    uint32_t* bitmap;     // [batch][n_words], zero on entry
    int32_t* word_rank;   // [batch][n_words] scratch
    int32_t* pairs;
    int32_t* n_pairs;
};

// Exclusive prefix sum of one int per thread over the block (same contract as
// block_scan_flag).
__device__ __forceinline__ int block_scan_int(int value, int* wave_sums, int& total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = (blockDim.x + 63) >> 6;
    int x = value;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int y = __shfl_up(x, d);
        if (lane >= d) x += y;
    }
    __syncthreads();
    if (lane == 63) wave_sums[wave] = x;
    __syncthreads();
    int offset = 0, sum = 0;
    for (int w = 0; w < nwaves; ++w) {
        const int s = wave_sums[w];
        if (w < wave) offset += s;
        sum += s;
    }
    total = sum;
    return offset + x - value;
}

// The match set M, sorted by (i, j) without duplicates.  A match's j is the nearest
// neighbour of its i, so two converged seeds with equal i carry equal j and sorting the
// pairs is sorting their i.  That is done as a distribution sort over the pixel range: mark
// the i of every converged seed in a bitmap, rank the set bits with a prefix sum of word
// popcounts, and let every converged seed write its pair at the rank of its i (seeds that
// share a match write the same value to the same place).
//
// LOCAL: bitmap and ranks live in the workgroup's LDS (passed as dynamic shared memory: n_words
// 32-bit words of bitmap, then n_words ranks of type RANK) instead of the workspace, which takes
// the global-memory round trips out of this latency-bound kernel; the launcher uses it whenever
// the two tables fit, with 16-bit ranks (at most 65535 seeds) for the larger images.
template <bool LOCAL, typename RANK>
__global__ __launch_bounds__(STEP_THREADS) void recip_dedup_kernel(DedupArgs a) {
    __shared__ int wave_sums[17];
    extern __shared__ uint32_t dedup_tables[];
    const int b = blockIdx.x;
    const int64_t base = (int64_t)b * a.n_seeds;
    uint32_t* bitmap = LOCAL ? dedup_tables : a.bitmap + (int64_t)b * a.n_words;
    RANK* word_rank = LOCAL ? reinterpret_cast<RANK*>(dedup_tables + a.n_words)
                            : reinterpret_cast<RANK*>(a.word_rank + (int64_t)b * a.n_words);
    if (LOCAL) {
        for (int w = threadIdx.x; w < a.n_words; w += STEP_THREADS) bitmap[w] = 0;
        __syncthreads();
    }

    for (int s = threadIdx.x; s < a.n_seeds; s += STEP_THREADS) {
        if (a.seed_iter[base + s] >= 0) {
            const uint32_t i = (uint32_t)a.seed_i[base + s];
            atomicOr(&bitmap[i >> 5], 1u << (i & 31));
        }
    }
    __syncthreads();

    // contiguous run of words per thread, so that ranks ascend with the thread index
    const int per_thread = (a.n_words + STEP_THREADS - 1) / STEP_THREADS;
    const int w0 = min((int)threadIdx.x * per_thread, a.n_words);
    const int w1 = min(w0 + per_thread, a.n_words);
    int mine = 0;
    for (int w = w0; w < w1; ++w)
        mine += __popc(__hip_atomic_load(&bitmap[w], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    int count;
    int rank = block_scan_int(mine, wave_sums, count);
    for (int w = w0; w < w1; ++w) {
        word_rank[w] = (RANK)rank;
        rank += __popc(__hip_atomic_load(&bitmap[w], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    }
    __syncthreads();

    for (int s = threadIdx.x; s < a.n_seeds; s += STEP_THREADS) {
        if (a.seed_iter[base + s] >= 0) {
            const uint32_t i = (uint32_t)a.seed_i[base + s];
            const uint32_t word = __hip_atomic_load(&bitmap[i >> 5], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const int pos = (int)__hip_atomic_load(&word_rank[i >> 5], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) +
                            __popc(word & ((1u << (i & 31)) - 1u));
            a.pairs[(base + pos) * 2 + 0] = (int32_t)i;
            a.pairs[(base + pos) * 2 + 1] = a.seed_j[base + s];
        }
    }
    for (int i = count + threadIdx.x; i < a.n_seeds; i += STEP_THREADS) {
        a.pairs[(base + i) * 2 + 0] = -1;
        a.pairs[(base + i) * 2 + 1] = -1;
    }
    if (threadIdx.x == 0) a.n_pairs[b] = count;
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

// Dynamic LDS the 16-bit-rank variant of the final sort may use on this device (0: none beyond
// the default): what the device grants one workgroup, less the kernel's static LDS and some
// slack, raised once through the kernel's attribute.
static size_t dedup_large_lds_limit() {
    static DeviceCache limit;
    const long long granted = limit.get([](int dev) -> long long {
        int per_block = 0;
        if (hipDeviceGetAttribute(&per_block, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess ||
            per_block <= 64 * 1024)
            return 0;
        const int grant = per_block - 1024;
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(recip_dedup_kernel<true, uint16_t>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, grant) == hipSuccess)
            return grant;
        (void)hipGetLastError();  // not granted: the workspace variant serves these sizes
        return 0;
    });
    return granted > 0 ? (size_t)granted : 0;
}

hipError_t launch_recip_dedup(const RecipState& st, int32_t n_seeds, int batch,
                              const int32_t* seed_i, const int32_t* seed_j, const int32_t* seed_iter,
                              int32_t* pairs, int32_t* n_pairs, hipStream_t s) {
    DedupArgs a;
    a.seed_i = seed_i;
    a.seed_j = seed_j;
    a.seed_iter = seed_iter;
    a.n_seeds = n_seeds;
    a.n_words = (int32_t)st.n_words;
    a.bitmap = st.bitmap;
    a.word_rank = st.word_rank;
    a.pairs = pairs;
    a.n_pairs = n_pairs;
    const size_t tables = (size_t)st.n_words * 2 * sizeof(uint32_t);
    if (tables <= DEDUP_LDS_BYTES)
        return launch(TK_RECIP_DEDUP, recip_dedup_kernel<true, int32_t>, dim3(batch), dim3(STEP_THREADS), tables, s, a);
    // larger images: 16-bit ranks, and a workgroup may be granted more than the default 64 KB
    const size_t narrow = (size_t)st.n_words * (sizeof(uint32_t) + sizeof(uint16_t));
    if (n_seeds <= 65535 && narrow <= dedup_large_lds_limit())
        return launch(TK_RECIP_DEDUP, recip_dedup_kernel<true, uint16_t>, dim3(batch), dim3(STEP_THREADS), narrow, s, a);
    return launch(TK_RECIP_DEDUP, recip_dedup_kernel<false, int32_t>, dim3(batch), dim3(STEP_THREADS), 0, s, a);
}

}  // namespace fnn
