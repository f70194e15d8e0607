// Measurement aid behind fnn_measure_ceiling (see include/fnn_measure.h): what this device sustains on
// the instruction mix of one 32x32 block of scores, with everything else taken away.  The
// loops below work on registers only (operands are made up from the lane number, results are
// reduced to one word per thread that is stored at the end), two waves per SIMD like the real
// kernels, R = 4 independent blocks in flight per wave like the search kernel.
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include "../../include/fnn_measure.h"
#include "fnn_device.hpp"

namespace fnn {

namespace {

constexpr int CEIL_THREADS = 256;  // 4 waves per workgroup, 2 workgroups per CU = 2 waves per SIMD
constexpr int CEIL_R = 4;

__device__ __forceinline__ float ceil_max3(float a, float b, float c) { return __builtin_fmaxf(__builtin_fmaxf(a, b), c); }
__device__ __forceinline__ float ceil_fold16(float seed, const f32x16& x) {
    const float t0 = ceil_max3(x[0], x[1], x[2]), t1 = ceil_max3(x[3], x[4], x[5]), t2 = ceil_max3(x[6], x[7], x[8]);
    const float t3 = ceil_max3(x[9], x[10], x[11]), t4 = ceil_max3(x[12], x[13], x[14]);
    return ceil_max3(seed, ceil_max3(t0, t1, t2), ceil_max3(t3, t4, x[15]));
}

__device__ __forceinline__ _Float16 ceil_operand(uint32_t i) {
    uint32_t x = i * 2654435761u;
    x ^= x >> 15;
    x *= 2246822519u;
    x ^= x >> 13;
    return (_Float16)((float)(x >> 8) * (1.0f / 16777216.0f) - 0.5f);
}

// MIX 0: one K=16 instruction per block.  1: K=16 + K=8 (a 24-channel block).  2: two K=16
// (a 32-channel block).  3: MIX 1 plus the eight 3-input maxima that fold a block into a running
// best (the search kernel's arithmetic).  4: MIX 1 plus sixteen 3-input maxima per block, a fold
// and a running element-wise maximum over pairs of blocks (the dense kernel's arithmetic).
// 5: the 32x32 block as four 16x16x32 instructions (24 channels padded to 32).
// BF16: the same loops on the bfloat16 instructions (MIX 1, 3, 4).
typedef float f32x4 __attribute__((ext_vector_type(4)));
template <int MIX, bool BF16>
__global__ __launch_bounds__(CEIL_THREADS) __attribute__((amdgpu_waves_per_eu(2)))
void ceiling_kernel(float* out, int trips) {
    const int lane = threadIdx.x & 63;
    // Operands: hashed values in [-0.5, 0.5) with full fp16 significands, made up from the lane
    // number and never read from memory.  (What the matrix cores sustain depends on the data: with
    // operands of one or two significant bits the same loops run about 20 % faster, presumably
    // because the part is power-limited under matrix load; descriptors are not like that.)
    f16x8 cand, cand2, q[CEIL_R];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        cand[e] = ceil_operand(lane * 8 + e);
        cand2[e] = ceil_operand(1000 + lane * 8 + e);
#pragma unroll
        for (int r = 0; r < CEIL_R; ++r) q[r][e] = ceil_operand(2000 + (r * 64 + lane) * 8 + e);
    }
    if constexpr (BF16) {
        // the same bit patterns read as bfloat16 would be tiny numbers with a 7-bit significand
        // pattern of their own; convert the values instead (bf16 keeps 8 significant bits)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            cand[e] = __builtin_bit_cast(_Float16, (__bf16)(float)cand[e]);
            cand2[e] = __builtin_bit_cast(_Float16, (__bf16)(float)cand2[e]);
#pragma unroll
            for (int r = 0; r < CEIL_R; ++r) q[r][e] = __builtin_bit_cast(_Float16, (__bf16)(float)q[r][e]);
        }
    }
    float best[CEIL_R];
    f32x16 cmax[CEIL_R / 2];
#pragma unroll
    for (int r = 0; r < CEIL_R; ++r) best[r] = -__builtin_inff();
#pragma unroll
    for (int p = 0; p < CEIL_R / 2; ++p)
#pragma unroll
        for (int v = 0; v < 16; ++v) cmax[p][v] = -__builtin_inff();

    // one block: the matrix instructions of MIX on operands (cand, cand2) x q
    auto block = [&](const f16x8& q_r) {
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if constexpr (MIX == 5) {
            // four 16x16 quadrants, K = 32 each; every one takes this block's query operand (in
            // either role) so that none can be shared between blocks or hoisted out of the loop
            const f32x4 z4 = {0.f, 0.f, 0.f, 0.f};
            const f32x4 a0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(cand, q_r, z4, 0, 0, 0);
            const f32x4 a1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(cand2, q_r, z4, 0, 0, 0);
            const f32x4 a2 = __builtin_amdgcn_mfma_f32_16x16x32_f16(q_r, cand, z4, 0, 0, 0);
            const f32x4 a3 = __builtin_amdgcn_mfma_f32_16x16x32_f16(q_r, cand2, z4, 0, 0, 0);
            f32x16 acc;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                acc[v] = a1[v];
                acc[4 + v] = a2[v];
                acc[8 + v] = a3[v];
                acc[12 + v] = a0[v];
            }
            return acc;
        } else if constexpr (BF16) {
            f32x16 acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, cand),
                                                                 __builtin_bit_cast(bf16x8, q_r), zero, 0, 0, 0);
            const f16x4 ch = {cand2[0], cand2[1], cand2[2], cand2[3]}, qh = {q_r[4], q_r[5], q_r[6], q_r[7]};
            acc = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(__builtin_bit_cast(i16x4, ch), __builtin_bit_cast(i16x4, qh),
                                                           acc, 0, 0, 0);
            return acc;
        } else {
            f32x16 acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(cand, q_r, zero, 0, 0, 0);
            if constexpr (MIX == 1 || MIX == 3 || MIX == 4) {
                const f16x4 ch = {cand2[0], cand2[1], cand2[2], cand2[3]}, qh = {q_r[4], q_r[5], q_r[6], q_r[7]};
                acc = __builtin_amdgcn_mfma_f32_32x32x8f16(ch, qh, acc, 0, 0, 0);
            } else if constexpr (MIX == 2) {
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(cand2, q_r, acc, 0, 0, 0);
            }
            return acc;
        }
    };

    if constexpr (MIX < 3 || MIX == 5) {
        for (int trip = 0; trip < trips; ++trip) {
            // the operands are "new" every trip as far as the compiler can tell, so no product is hoisted
            asm volatile("" : "+v"(cand), "+v"(cand2));
#pragma unroll
            for (int r = 0; r < CEIL_R; ++r) {
                const f32x16 acc = block(q[r]);
                if constexpr (MIX == 5) {  // one operation per instruction keeps all four alive
                    best[r] = ceil_max3(best[r], ceil_max3(acc[0], acc[4], acc[8]), acc[12]);
                } else {
                    best[r] = __builtin_fmaxf(best[r], acc[0]);  // one operation keeps the block alive
                }
            }
        }
    } else {
        // With vector work: the next pair of blocks is issued before the current pair is folded
        // (the fastest order found for these loops: 42 against 43 ns for MIX 3, 50 against 53-58 ns
        // for MIX 4 when all matrix instructions of a trip come first).
        static_assert(CEIL_R == 4, "two pairs of blocks per trip");
        f32x16 pa[2], pb[2];
        pa[0] = block(q[0]);
        pb[0] = block(q[1]);
        for (int trip = 0; trip < trips; ++trip) {
            asm volatile("" : "+v"(cand), "+v"(cand2));
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const int cur = p, nxt = p ^ 1;
                pa[nxt] = block(q[2 * nxt]);
                pb[nxt] = block(q[2 * nxt + 1]);
                best[2 * cur] = ceil_fold16(best[2 * cur], pa[cur]);
                best[2 * cur + 1] = ceil_fold16(best[2 * cur + 1], pb[cur]);
                if constexpr (MIX == 4) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) cmax[cur][v] = ceil_max3(cmax[cur][v], pa[cur][v], pb[cur][v]);
                }
            }
        }
        best[0] += pa[0][0] + pb[0][0];  // the pair issued last is never folded
    }
    float word = 0.f;
#pragma unroll
    for (int r = 0; r < CEIL_R; ++r) word += best[r];
    if constexpr (MIX == 4) {
#pragma unroll
        for (int p = 0; p < CEIL_R / 2; ++p) word += ceil_fold16(0.f, cmax[p]);
    }
    out[(size_t)blockIdx.x * CEIL_THREADS + threadIdx.x] = word;
}

template <int MIX, bool BF16 = false>
hipError_t run_ceiling(float* out, int grid, int trips, hipStream_t s, float* ms) {
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return hipErrorUnknown;
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return hipErrorUnknown;
    }
    hipLaunchKernelGGL((ceiling_kernel<MIX, BF16>), dim3(grid), dim3(CEIL_THREADS), 0, s, out, 16);  // warm-up
    hipError_t err = hipGetLastError();
    float best = 0.f;
    for (int rep = 0; rep < 3 && err == hipSuccess; ++rep) {
        hipExtLaunchKernelGGL((ceiling_kernel<MIX, BF16>), dim3(grid), dim3(CEIL_THREADS), 0, s, e0, e1, 0, out, trips);
        err = hipGetLastError();
        if (err == hipSuccess) err = hipEventSynchronize(e1);
        float t = 0.f;
        if (err == hipSuccess) err = hipEventElapsedTime(&t, e0, e1);
        if (rep == 0 || t < best) best = t;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    *ms = best;
    return err;
}

}  // namespace
}  // namespace fnn

#pragma GCC visibility push(default)
extern "C" {

int32_t fnn_measure_ceiling(int32_t mix, int32_t blocks_per_wave, void* scratch, size_t scratch_bytes,
                            float* ns_per_block, void* stream) {
    using namespace fnn;
    if (!scratch || !ns_per_block) return FNN_E_NULL;
    if (mix < 0 || mix > 8 || blocks_per_wave < CEIL_R || blocks_per_wave > (1 << 24)) return FNN_E_RANGE;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return FNN_E_HIP;
    const int grid = prop.multiProcessorCount * 2;  // two workgroups of four waves per CU: two waves per SIMD
    if (((uintptr_t)scratch % 4) != 0 || scratch_bytes < (size_t)grid * CEIL_THREADS * sizeof(float)) return FNN_E_WORKSPACE;
    const int trips = blocks_per_wave / CEIL_R;
    float ms = 0.f;
    hipError_t err = hipSuccess;
    hipStream_t s = (hipStream_t)stream;
    float* out = (float*)scratch;
    switch (mix) {
        case 0: err = run_ceiling<0>(out, grid, trips, s, &ms); break;
        case 1: err = run_ceiling<1>(out, grid, trips, s, &ms); break;
        case 2: err = run_ceiling<2>(out, grid, trips, s, &ms); break;
        case 3: err = run_ceiling<3>(out, grid, trips, s, &ms); break;
        case 4: err = run_ceiling<4>(out, grid, trips, s, &ms); break;
        case 5: err = run_ceiling<5>(out, grid, trips, s, &ms); break;
        case 6: err = run_ceiling<1, true>(out, grid, trips, s, &ms); break;
        case 7: err = run_ceiling<3, true>(out, grid, trips, s, &ms); break;
        default: err = run_ceiling<4, true>(out, grid, trips, s, &ms); break;
    }
    if (err != hipSuccess) return FNN_E_HIP;
    // a SIMD works on two waves' blocks at once
    *ns_per_block = ms * 1e6f / ((float)trips * CEIL_R * 2.0f);
    return FNN_OK;
}

}  // extern "C"
#pragma GCC visibility pop
