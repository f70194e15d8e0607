// Prepare step: copy the caller's descriptor maps into the workspace in the format the
// matrix instructions consume -- the compute format of Algorithm 3 ("HybridCast": inputs
// rounded to 16 bits, round-to-nearest-even) or plain fp32 -- with the channel count zero
// padded to the instruction's K and the pixel count zero padded to whole 32-pixel tiles.
#include "dense_perm.hpp"
#include "fnn_device.hpp"
#include "fnn_kernels.hpp"
#include "trace.hpp"

namespace fnn {

__device__ __forceinline__ float load_as_float(const void* base, int64_t idx, int dtype) {
    if (dtype == FNN_F32) return reinterpret_cast<const float*>(base)[idx];
    const uint16_t raw = reinterpret_cast<const uint16_t*>(base)[idx];
    if (dtype == FNN_F16) {
        return (float)__builtin_bit_cast(_Float16, raw);
    }
    return __uint_as_float((uint32_t)raw << 16);
}

// Euclidean norm of one source descriptor as FNN_FLAG_NORMALIZE defines it: squares and
// sums rounded separately (no fused multiply-add), channels in ascending order.
__device__ __forceinline__ float descriptor_norm(const void* src, int64_t first, int d, int dtype) {
    float sum = 0.0f;
    for (int k = 0; k < d; ++k) {
        const float x = load_as_float(src, first + k, dtype);
        sum = __fadd_rn(sum, __fmul_rn(x, x));
    }
    return __fsqrt_rn(sum);
}

// x as the compute format holds it (round to nearest even), back in fp32.
__device__ __forceinline__ float round_to_compute(float x, int compute) {
    if (compute == FNN_F16) return (float)(_Float16)x;
    if (compute == FNN_BF16) return __uint_as_float((uint32_t)float_to_bf16_rne(x) << 16);
    return x;
}

// -1/2 * |x|^2 of one descriptor AS PREPARED (normalised if asked, rounded to the compute
// format): fp32 sum, channels ascending, squares and sums rounded separately.
__device__ __forceinline__ float minus_half_norm2(const void* src, int64_t first, int d, int dtype, int compute,
                                                  float divide_by) {
    float sum = 0.0f;
    for (int k = 0; k < d; ++k) {
        float x = load_as_float(src, first + k, dtype);
        if (divide_by > 0.0f) x = __fdiv_rn(x, divide_by);
        x = round_to_compute(x, compute);
        sum = __fadd_rn(sum, __fmul_rn(x, x));
    }
    return -0.5f * sum;
}

// Side jobs spread over all threads of the launch (see PrepExtra).
__device__ __forceinline__ void prep_side_jobs(const PrepArgs& a) {
    const PrepExtra& x = a.extra;
    const int64_t tid = ((int64_t)blockIdx.y * gridDim.x + blockIdx.x) * blockDim.x + threadIdx.x;
    const int64_t n_threads = (int64_t)gridDim.x * gridDim.y * blockDim.x;
    if (x.zero_ptr)
        for (int64_t i = tid; i < x.zero_count; i += n_threads) x.zero_ptr[i] = 0;
    if (x.seeds) {
        const int64_t total = (int64_t)a.batch * x.n_seeds;
        for (int64_t i = tid; i < total; i += n_threads) {
            x.cur_u[i] = x.seeds[i];
            x.seed_id[i] = (int32_t)(i % x.n_seeds);
        }
        for (int64_t b = tid; b < a.batch; b += n_threads) x.n_active[b] = x.n_seeds;
    }
}

// One thread produces 8 consecutive channels of one output row.
__global__ __launch_bounds__(256) void prep_kernel(PrepArgs a) {
    prep_side_jobs(a);
    const int side_idx = blockIdx.y / a.batch;
    const int b = blockIdx.y % a.batch;
    const PrepSide& sd = a.side[side_idx];
    const int groups = a.dp / 8;
    const int64_t total = sd.n_pad * groups;
    const int esize = (a.compute == FNN_F32) ? 4 : 2;
    char* dst = reinterpret_cast<char*>(sd.dst) + (int64_t)b * sd.n_pad * a.dp * esize;
    const void* src = sd.src[b];
    for (int64_t item = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; item < total;
         item += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = item / groups;                               // stored row
        const int64_t pix = sd.segment_major ? slot_pixel(row) : row;   // pixel it holds
        const int g = (int)(item % groups);
        // channels that carry data: the descriptor, or three copies of it (FNN_FLAG_SPLIT)
        const int data_channels = a.split ? 3 * a.d : a.d;
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int k = g * 8 + e;
            const int ch = a.split ? k % a.d : k;
            v[e] = (pix < sd.n && k < data_channels) ? load_as_float(src, pix * sd.row_stride + ch, sd.dtype) : 0.0f;
        }
        float norm = 0.0f;
        if (a.normalize && pix < sd.n) {
            norm = descriptor_norm(src, pix * sd.row_stride, a.d, sd.dtype);
            if (norm > 0.0f) {
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = __fdiv_rn(v[e], norm);
            }
        }
        // Two-term fp16 representation: copy 0 holds hi, and of copies 1 and 2 image 1 holds
        // (hi, lo), image 2 (lo, hi), so that a row of one times a row of the other sums
        // hi*hi + hi*lo + lo*hi.
        if (a.split) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int k = g * 8 + e;
                if (k < data_channels) {
                    const int copy = k / a.d;
                    const float hi = (float)(_Float16)v[e];
                    const float lo = (float)(_Float16)__fsub_rn(v[e], hi);
                    v[e] = (copy == 0 || copy == (sd.second_image ? 2 : 1)) ? hi : lo;
                }
            }
        }
        // L2 score: channels d.. hold the unit partners and -|x|^2/2 (see FNN_FLAG_L2).  For a
        // 16-bit format the norm term is split into a rounded value and the rounded remainder.
        const int extra = a.compute == FNN_F32 ? 1 : 2;
        if (a.l2 && pix < sd.n && g * 8 + 8 > a.d && g * 8 < a.d + 2 * extra) {
            const float term = minus_half_norm2(src, pix * sd.row_stride, a.d, sd.dtype, a.compute, norm);
            const float hi = round_to_compute(term, a.compute);
            const float lo = round_to_compute(term - hi, a.compute);
            const int ones0 = a.d + (sd.second_image ? extra : 0);   // first unit channel
            const int term0 = a.d + (sd.second_image ? 0 : extra);   // first norm channel
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int k = g * 8 + e;
                if (k >= ones0 && k < ones0 + extra) v[e] = 1.0f;
                if (k == term0) v[e] = hi;
                if (extra == 2 && k == term0 + 1) v[e] = lo;
            }
        }
        if (a.compute == FNN_F32) {
            float4* out = reinterpret_cast<float4*>(dst + (row * a.dp + g * 8) * 4);
            out[0] = make_float4(v[0], v[1], v[2], v[3]);
            out[1] = make_float4(v[4], v[5], v[6], v[7]);
        } else {
            uint16_t hbits[8];
#pragma unroll
            for (int e = 0; e < 8; ++e)
                hbits[e] = (a.compute == FNN_F16) ? float_to_f16_rne(v[e]) : float_to_bf16_rne(v[e]);
            uint4 packed;
            packed.x = hbits[0] | ((uint32_t)hbits[1] << 16);
            packed.y = hbits[2] | ((uint32_t)hbits[3] << 16);
            packed.z = hbits[4] | ((uint32_t)hbits[5] << 16);
            packed.w = hbits[6] | ((uint32_t)hbits[7] << 16);
            *reinterpret_cast<uint4*>(dst + (row * a.dp + g * 8) * 2) = packed;
        }
    }
}

// Fast path for the options that need a whole row at once (FNN_FLAG_NORMALIZE, FNN_FLAG_L2) on
// fp32 sources with d a multiple of 8: one thread per row.  The row is read once with 16-byte
// loads; norm and squared length are formed in registers exactly as descriptor_norm and
// minus_half_norm2 define them (channels ascending, every product and sum rounded on its own).
// IN = d / 8, OUT = dp / 8.
template <int IN, int OUT, int COMPUTE>
__global__ __launch_bounds__(256) void prep_rows_f32_kernel(PrepArgs a) {
    prep_side_jobs(a);
    const int side_idx = blockIdx.y / a.batch;
    const int b = blockIdx.y % a.batch;
    const PrepSide& sd = a.side[side_idx];
    constexpr int ESIZE = (COMPUTE == FNN_F32) ? 4 : 2;
    constexpr int D = IN * 8, DP = OUT * 8;
    constexpr int EXTRA = (COMPUTE == FNN_F32) ? 1 : 2;  // channels per L2 term
    char* dst = reinterpret_cast<char*>(sd.dst) + (int64_t)b * sd.n_pad * DP * ESIZE;
    const float* src = reinterpret_cast<const float*>(sd.src[b]);
    for (uint32_t row = blockIdx.x * blockDim.x + threadIdx.x; row < (uint32_t)sd.n_pad; row += gridDim.x * blockDim.x) {
        const int64_t pix = sd.segment_major ? slot_pixel(row) : (int64_t)row;
        float v[DP];
#pragma unroll
        for (int e = 0; e < DP; ++e) v[e] = 0.0f;
        if (pix < sd.n) {
            const float4* p = reinterpret_cast<const float4*>(src + pix * sd.row_stride);
#pragma unroll
            for (int q = 0; q < IN * 2; ++q) {
                const float4 x = p[q];
                v[4 * q + 0] = x.x;
                v[4 * q + 1] = x.y;
                v[4 * q + 2] = x.z;
                v[4 * q + 3] = x.w;
            }
            if (a.normalize) {
                float sum = 0.0f;
#pragma unroll
                for (int e = 0; e < D; ++e) sum = __fadd_rn(sum, __fmul_rn(v[e], v[e]));
                const float norm = __fsqrt_rn(sum);
                if (norm > 0.0f) {
#pragma unroll
                    for (int e = 0; e < D; ++e) v[e] = __fdiv_rn(v[e], norm);
                }
            }
#pragma unroll
            for (int e = 0; e < D; ++e) v[e] = round_to_compute(v[e], COMPUTE);
            if (a.l2) {
                float sum = 0.0f;
#pragma unroll
                for (int e = 0; e < D; ++e) sum = __fadd_rn(sum, __fmul_rn(v[e], v[e]));
                const float term = -0.5f * sum;
                const float hi = round_to_compute(term, COMPUTE);
                const float lo = round_to_compute(term - hi, COMPUTE);
                const int ones0 = D + (sd.second_image ? EXTRA : 0);
                const int term0 = D + (sd.second_image ? 0 : EXTRA);
#pragma unroll
                for (int e = D; e < D + 2 * EXTRA; ++e) {
                    if (e >= ones0 && e < ones0 + EXTRA) v[e] = 1.0f;
                    if (e == term0) v[e] = hi;
                    if (EXTRA == 2 && e == term0 + 1) v[e] = lo;
                }
            }
        }
        if (COMPUTE == FNN_F32) {
            float4* out = reinterpret_cast<float4*>(dst + (int64_t)row * DP * 4);
#pragma unroll
            for (int q = 0; q < OUT * 2; ++q) out[q] = make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
        } else {
            uint4* out = reinterpret_cast<uint4*>(dst + (int64_t)row * DP * 2);
#pragma unroll
            for (int q = 0; q < OUT; ++q) {
                uint32_t w[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    // the values are already representable: the conversion is exact
                    const float lo = v[8 * q + 2 * e], hi = v[8 * q + 2 * e + 1];
                    const uint32_t l16 = (COMPUTE == FNN_F16) ? float_to_f16_rne(lo) : float_to_bf16_rne(lo);
                    const uint32_t h16 = (COMPUTE == FNN_F16) ? float_to_f16_rne(hi) : float_to_bf16_rne(hi);
                    w[e] = l16 | (h16 << 16);
                }
                out[q] = make_uint4(w[0], w[1], w[2], w[3]);
            }
        }
    }
}

// FNN_FLAG_SPLIT on fp32 sources with d = 8 * IN whole 16-byte vectors: one thread per row
// reads the descriptor once and writes its three copies (see prep_kernel for the layout).
template <int IN>
__global__ __launch_bounds__(256) void prep_split_rows_kernel(PrepArgs a) {
    prep_side_jobs(a);
    const int side_idx = blockIdx.y / a.batch;
    const int b = blockIdx.y % a.batch;
    const PrepSide& sd = a.side[side_idx];
    constexpr int D = IN * 8, DP = padded_d(3 * D, FNN_F16);
    char* dst = reinterpret_cast<char*>(sd.dst) + (int64_t)b * sd.n_pad * DP * 2;
    const float* src = reinterpret_cast<const float*>(sd.src[b]);
    const int lo_copy = sd.second_image ? 1 : 2;  // which of copies 1, 2 holds the lo terms
    for (uint32_t row = blockIdx.x * blockDim.x + threadIdx.x; row < (uint32_t)sd.n_pad; row += gridDim.x * blockDim.x) {
        const int64_t pix = sd.segment_major ? slot_pixel(row) : (int64_t)row;
        uint32_t hi[D], lo[D];
#pragma unroll
        for (int e = 0; e < D; ++e) hi[e] = lo[e] = 0;
        if (pix < sd.n) {
            float v[D];
            const float4* p = reinterpret_cast<const float4*>(src + pix * sd.row_stride);
#pragma unroll
            for (int q = 0; q < IN * 2; ++q) {
                const float4 x = p[q];
                v[4 * q + 0] = x.x;
                v[4 * q + 1] = x.y;
                v[4 * q + 2] = x.z;
                v[4 * q + 3] = x.w;
            }
            if (a.normalize) {
                float sum = 0.0f;
#pragma unroll
                for (int e = 0; e < D; ++e) sum = __fadd_rn(sum, __fmul_rn(v[e], v[e]));
                const float norm = __fsqrt_rn(sum);
                if (norm > 0.0f) {
#pragma unroll
                    for (int e = 0; e < D; ++e) v[e] = __fdiv_rn(v[e], norm);
                }
            }
#pragma unroll
            for (int e = 0; e < D; ++e) {
                const _Float16 h = (_Float16)v[e];
                hi[e] = __builtin_bit_cast(uint16_t, h);
                lo[e] = float_to_f16_rne(__fsub_rn(v[e], (float)h));
            }
        }
        uint4* out = reinterpret_cast<uint4*>(dst + (int64_t)row * DP * 2);
#pragma unroll
        for (int q = 0; q < DP / 8; ++q) {
            uint32_t w[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                uint32_t half[2];
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const int k = 8 * q + 2 * e + t;       // compile-time channel of the output row
                    const int copy = k / D, ch = k % D;
                    half[t] = (k >= 3 * D) ? 0u : ((copy == lo_copy) ? lo[ch] : hi[ch]);
                }
                w[e] = half[0] | (half[1] << 16);
            }
            out[q] = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
}

template <int IN, int OUT>
static hipError_t launch_prep_rows(const PrepArgs& a, dim3 grid, hipStream_t s) {
    if (a.compute == FNN_F32) return launch(TK_PREP, prep_rows_f32_kernel<IN, OUT, FNN_F32>, grid, dim3(256), 0, s, a);
    if (a.compute == FNN_F16) return launch(TK_PREP, prep_rows_f32_kernel<IN, OUT, FNN_F16>, grid, dim3(256), 0, s, a);
    return launch(TK_PREP, prep_rows_f32_kernel<IN, OUT, FNN_BF16>, grid, dim3(256), 0, s, a);
}

// Fast path: fp32 source whose rows are whole 16-byte vectors and need no channel padding
// (d == dp).  GROUPS = dp / 8 is a compile-time constant so that the row / group split of the
// item index costs a multiply, and every thread moves two 16-byte loads into one (16-bit
// formats) or two (fp32) 16-byte stores.
template <int GROUPS, int COMPUTE>
__global__ __launch_bounds__(256) void prep_f32_kernel(PrepArgs a) {
    prep_side_jobs(a);
    const int side_idx = blockIdx.y / a.batch;
    const int b = blockIdx.y % a.batch;
    const PrepSide& sd = a.side[side_idx];
    const uint32_t total = (uint32_t)sd.n_pad * GROUPS;
    constexpr int ESIZE = (COMPUTE == FNN_F32) ? 4 : 2;
    char* dst = reinterpret_cast<char*>(sd.dst) + (int64_t)b * sd.n_pad * (GROUPS * 8) * ESIZE;
    const float* src = reinterpret_cast<const float*>(sd.src[b]);
    for (uint32_t item = blockIdx.x * blockDim.x + threadIdx.x; item < total; item += gridDim.x * blockDim.x) {
        const uint32_t row = item / GROUPS;
        const uint32_t g = item - row * GROUPS;
        const int64_t pix = sd.segment_major ? slot_pixel(row) : (int64_t)row;
        float4 lo = make_float4(0.f, 0.f, 0.f, 0.f), hi = lo;
        if (pix < sd.n) {
            const float4* p = reinterpret_cast<const float4*>(src + pix * sd.row_stride + g * 8);
            lo = p[0];
            hi = p[1];
        }
        if (COMPUTE == FNN_F32) {
            float4* out = reinterpret_cast<float4*>(dst + ((int64_t)item * 8) * 4);
            out[0] = lo;
            out[1] = hi;
        } else {
            const float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
            uint16_t hbits[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) hbits[e] = (COMPUTE == FNN_F16) ? float_to_f16_rne(v[e]) : float_to_bf16_rne(v[e]);
            uint4 packed;
            packed.x = hbits[0] | ((uint32_t)hbits[1] << 16);
            packed.y = hbits[2] | ((uint32_t)hbits[3] << 16);
            packed.z = hbits[4] | ((uint32_t)hbits[5] << 16);
            packed.w = hbits[6] | ((uint32_t)hbits[7] << 16);
            *reinterpret_cast<uint4*>(dst + ((int64_t)item * 8) * 2) = packed;
        }
    }
}

template <int GROUPS>
static hipError_t launch_prep_fast(const PrepArgs& a, dim3 grid, hipStream_t s) {
    if (a.compute == FNN_F32) return launch(TK_PREP, prep_f32_kernel<GROUPS, FNN_F32>, grid, dim3(256), 0, s, a);
    if (a.compute == FNN_F16) return launch(TK_PREP, prep_f32_kernel<GROUPS, FNN_F16>, grid, dim3(256), 0, s, a);
    return launch(TK_PREP, prep_f32_kernel<GROUPS, FNN_BF16>, grid, dim3(256), 0, s, a);
}

__global__ __launch_bounds__(256) void fill_none_kernel(int32_t* idx, float* score, int64_t count) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (int64_t)gridDim.x * blockDim.x) {
        idx[i] = -1;
        if (score) score[i] = -__builtin_inff();
    }
}

hipError_t launch_fill_i32f32(int32_t* idx, float* score, int64_t count, hipStream_t s) {
    if (count <= 0) return hipSuccess;
    int64_t blocks = (count + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    return launch(TK_FILL, fill_none_kernel, dim3((unsigned)blocks), dim3(256), 0, s, idx, score, count);
}

// The side jobs alone.
__global__ __launch_bounds__(256) void init_kernel(PrepArgs a) { prep_side_jobs(a); }

hipError_t launch_prep(const PrepArgs& a, hipStream_t s) {
    int64_t most = 0;
    for (int i = 0; i < a.n_sides; ++i) {
        const int64_t items = a.side[i].n_pad * (a.dp / 8);
        if (items > most) most = items;
    }
    if (most == 0) {
        // no map to convert (empty, or all used in place): only the side jobs, if any
        int64_t work = a.extra.zero_ptr ? a.extra.zero_count : 0;
        if (a.extra.seeds && (int64_t)a.batch * a.extra.n_seeds > work) work = (int64_t)a.batch * a.extra.n_seeds;
        if (work <= 0) return hipSuccess;
        int64_t init_blocks = (work + 255) / 256;
        if (init_blocks > 1024) init_blocks = 1024;
        return launch(TK_PREP, init_kernel, dim3((unsigned)init_blocks, 1), dim3(256), 0, s, a);
    }
    int64_t blocks = (most + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    dim3 grid((unsigned)blocks, (unsigned)(a.n_sides * a.batch));
    bool vector_rows = most < (int64_t)1 << 31;  // fp32 sources whose rows are whole, aligned 16-byte vectors
    for (int i = 0; i < a.n_sides && vector_rows; ++i) {
        const PrepSide& sd = a.side[i];
        vector_rows = sd.dtype == FNN_F32 && sd.row_stride % 4 == 0;
        for (int b = 0; b < a.batch && vector_rows; ++b) vector_rows = ((uintptr_t)sd.src[b] % 16) == 0;
    }
    if (vector_rows && a.split && a.d % 8 == 0 && a.dp == padded_d(3 * a.d, FNN_F16)) {
        switch (a.d / 8) {
            case 1: return launch(TK_PREP, prep_split_rows_kernel<1>, grid, dim3(256), 0, s, a);
            case 2: return launch(TK_PREP, prep_split_rows_kernel<2>, grid, dim3(256), 0, s, a);
            case 3: return launch(TK_PREP, prep_split_rows_kernel<3>, grid, dim3(256), 0, s, a);
            case 4: return launch(TK_PREP, prep_split_rows_kernel<4>, grid, dim3(256), 0, s, a);
        }
    }
    if (vector_rows && !a.split && (a.normalize || a.l2) && a.d % 8 == 0) {
        const int in = a.d / 8, out = a.dp / 8;
        if (in == 1 && out == 1) return launch_prep_rows<1, 1>(a, grid, s);
        if (in == 1 && out == 2) return launch_prep_rows<1, 2>(a, grid, s);
        if (in == 2 && out == 2) return launch_prep_rows<2, 2>(a, grid, s);
        if (in == 2 && out == 3) return launch_prep_rows<2, 3>(a, grid, s);
        if (in == 3 && out == 3) return launch_prep_rows<3, 3>(a, grid, s);
        if (in == 3 && out == 4) return launch_prep_rows<3, 4>(a, grid, s);
        if (in == 4 && out == 4) return launch_prep_rows<4, 4>(a, grid, s);
    }
    const bool fast = vector_rows && a.d == a.dp && !a.l2 && !a.normalize && !a.split;
    if (fast) {
        switch (a.dp / 8) {
            case 1: return launch_prep_fast<1>(a, grid, s);
            case 2: return launch_prep_fast<2>(a, grid, s);
            case 3: return launch_prep_fast<3>(a, grid, s);
            case 4: return launch_prep_fast<4>(a, grid, s);
        }
    }
    return launch(TK_PREP, prep_kernel, grid, dim3(256), 0, s, a);
}

}  // namespace fnn
