// Device-side building blocks shared by the libfnn kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fnn {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned long long u64;

enum : int { CT_F32 = 0, CT_F16 = 1, CT_BF16 = 2 };

// ---------------------------------------------------------------------------------------
// Packed 64-bit candidate key: high word = score bits mapped so that unsigned order equals
// float order, low word = inverted index.  An unsigned max therefore picks the largest
// score and, among equal scores, the lowest index -- the strict "<" update of the paper's
// Algorithm 1 -- no matter in which order candidates arrive.  Key 0 means "no candidate".
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t order_bits(float s) {
    s = s + 0.0f;  // -0 -> +0 so that equal floats have equal keys
    const uint32_t b = __float_as_uint(s);
    // negative: flip every bit; non-negative: set the sign bit
    return b ^ ((uint32_t)((int32_t)b >> 31) | 0x80000000u);
}
__device__ __forceinline__ float unorder_bits(uint32_t o) {
    uint32_t b = (o & 0x80000000u) ? (o & 0x7FFFFFFFu) : ~o;
    return __uint_as_float(b);
}
__device__ __forceinline__ u64 pack_key(float s, int32_t idx) {
    return ((u64)order_bits(s) << 32) | (u64)(0xFFFFFFFFu - (uint32_t)idx);
}
__device__ __forceinline__ int32_t key_index(u64 k) {
    return k ? (int32_t)(0xFFFFFFFFu - (uint32_t)(k & 0xFFFFFFFFull)) : -1;
}
__device__ __forceinline__ float key_score(u64 k) {
    return k ? unorder_bits((uint32_t)(k >> 32)) : -__builtin_inff();
}

__device__ __forceinline__ u64 shfl_xor_u64(u64 v, int mask) {
    uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
    lo = __shfl_xor(lo, mask);
    hi = __shfl_xor(hi, mask);
    return ((u64)hi << 32) | lo;
}

// ---------------------------------------------------------------------------------------
// Matrix-core fragments.  A prepared map stores DP elements per pixel (zero padded).  In a
// 32-pixel tile lane (c = lane & 31, h = lane >> 5) owns pixel c and a fixed half of its
// channels (the contiguous half [h*DP/2, (h+1)*DP/2) in the generic layout), for the
// operand on either side of the product, so both sides agree on which channel sits in
// which slot of which matrix instruction.
// mma(a, b): a = 32 candidate pixels, b = 32 query pixels.  Result register v of lane (c, h)
// is the score of query c against candidate 8*(v/4) + 4*h + (v%4) of the tile.
// ---------------------------------------------------------------------------------------
template <int CT, int DP>
struct Ops {
    static constexpr int ESIZE = (CT == CT_F32) ? 4 : 2;
    static constexpr int ROW_BYTES = DP * ESIZE;
    static constexpr int LANE_BYTES = ROW_BYTES / 2;
    static constexpr int NV = LANE_BYTES / 16;
    static_assert(LANE_BYTES % 16 == 0, "lane slice must be whole 16-byte vectors");

    struct Frag {
        uint4 v[NV];
    };

    static __device__ __forceinline__ Frag load(const char* row, int h) {
        const uint4* p = reinterpret_cast<const uint4*>(row + h * LANE_BYTES);
        Frag f;
#pragma unroll
        for (int i = 0; i < NV; ++i) f.v[i] = p[i];
        return f;
    }

    static __device__ __forceinline__ f32x16 mma(const Frag& a, const Frag& b) {
        f32x16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            if constexpr (CT == CT_F16) {
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a.v[i]),
                                                             __builtin_bit_cast(f16x8, b.v[i]), acc, 0, 0, 0);
            } else if constexpr (CT == CT_BF16) {
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a.v[i]),
                                                              __builtin_bit_cast(bf16x8, b.v[i]), acc, 0, 0, 0);
            } else {
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.v[i].x), __uint_as_float(b.v[i].x), acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.v[i].y), __uint_as_float(b.v[i].y), acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.v[i].z), __uint_as_float(b.v[i].z), acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.v[i].w), __uint_as_float(b.v[i].w), acc, 0, 0, 0);
            }
        }
        return acc;
    }
};

// 24 channels in a 16-bit format: 48-byte rows, no padding.  Channels 0..15 go through one
// K=16 matrix instruction (lane half h supplies channels 8h..8h+7), channels 16..23 through
// one K=8 instruction (lane half h supplies channels 16+4h..16+4h+3).
template <int CT>
struct OpsHalf24 {
    static constexpr int ESIZE = 2;
    static constexpr int ROW_BYTES = 48;

    struct Frag {
        uint4 lo;
        uint2 hi;
    };

    static __device__ __forceinline__ Frag load(const char* row, int h) {
        Frag f;
        f.lo = *reinterpret_cast<const uint4*>(row + 16 * h);
        f.hi = *reinterpret_cast<const uint2*>(row + 32 + 8 * h);
        return f;
    }

    static __device__ __forceinline__ f32x16 mma(const Frag& a, const Frag& b) {
        f32x16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if constexpr (CT == CT_F16) {
            acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a.lo), __builtin_bit_cast(f16x8, b.lo),
                                                         acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x8f16(__builtin_bit_cast(f16x4, a.hi), __builtin_bit_cast(f16x4, b.hi),
                                                       acc, 0, 0, 0);
        } else {
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a.lo),
                                                          __builtin_bit_cast(bf16x8, b.lo), acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(__builtin_bit_cast(i16x4, a.hi),
                                                           __builtin_bit_cast(i16x4, b.hi), acc, 0, 0, 0);
        }
        return acc;
    }
};
template <>
struct Ops<CT_F16, 24> : OpsHalf24<CT_F16> {};
template <>
struct Ops<CT_BF16, 24> : OpsHalf24<CT_BF16> {};

// Cross-lane helpers (pure vector-ALU data movement, no LDS round trip).
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
    return __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(x), CTRL, 0xF, 0xF, true));
}
// Maximum over the 32 lanes of each wave half, delivered to every lane of that half.
__device__ __forceinline__ float half_max(float x) {
    x = __builtin_fmaxf(x, dpp_move<0xB1>(x));   // quad_perm [1,0,3,2]: lane ^ 1
    x = __builtin_fmaxf(x, dpp_move<0x4E>(x));   // quad_perm [2,3,0,1]: lane ^ 2
    x = __builtin_fmaxf(x, dpp_move<0x141>(x));  // row_half_mirror: joins the two quads of 8 lanes
    x = __builtin_fmaxf(x, dpp_move<0x140>(x));  // row_mirror: joins the two halves of a 16-lane row
    // the two rows of a half trade places
    const auto sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __builtin_fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
}
// For values a (kept by lanes 0..31) and b (kept by lanes 32..63): lane c gets
// max(a[c], a[c+32]), lane c+32 gets max(b[c], b[c+32]).
__device__ __forceinline__ float cross_half_max(float a, float b) {
    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    return __builtin_fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
}

// Candidate offset inside a tile of result register v for lane half h.
__device__ __forceinline__ constexpr int tile_row(int v, int h) { return 8 * (v >> 2) + 4 * h + (v & 3); }

// ---------------------------------------------------------------------------------------
// Exclusive prefix sum of one flag per thread over a block of up to 1024 threads (16
// waves).  `wave_sums` is 17 ints of shared memory.  Every thread of the block must call
// it; returns the number of set flags in threads before this one, `total` = all of them.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ int block_scan_flag(bool flag, int* wave_sums, int& total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = (blockDim.x + 63) >> 6;
    const u64 ballot = __ballot(flag);
    const int before = __popcll(ballot & ((1ull << lane) - 1ull));
    __syncthreads();  // protect wave_sums from the previous use
    if (lane == 0) wave_sums[wave] = __popcll(ballot);
    __syncthreads();
    int offset = 0, sum = 0;
    for (int w = 0; w < nwaves; ++w) {
        const int s = wave_sums[w];
        if (w < wave) offset += s;
        sum += s;
    }
    total = sum;
    return offset + before;
}

}  // namespace fnn
