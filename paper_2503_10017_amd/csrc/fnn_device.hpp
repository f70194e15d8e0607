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
// Rounding of an fp32 descriptor value to the 16-bit compute formats (round to nearest even;
// finite inputs), the cast of Algorithm 3 ("HybridCast").  Every place that rounds uses these.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ uint16_t float_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ uint16_t float_to_f16_rne(float f) {
    _Float16 hf = (_Float16)f;  // v_cvt_f16_f32 rounds to nearest even
    return __builtin_bit_cast(uint16_t, hf);
}
// two values rounded to compute format CT (CT_F16 or CT_BF16) in one 32-bit word, `lo` in the low half
template <int CT>
__device__ __forceinline__ uint32_t round_pair(float lo, float hi) {
    if constexpr (CT == CT_F16) return (uint32_t)float_to_f16_rne(lo) | ((uint32_t)float_to_f16_rne(hi) << 16);
    else return (uint32_t)float_to_bf16_rne(lo) | ((uint32_t)float_to_bf16_rne(hi) << 16);
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

    // The same for lane c of a 32-pixel tile whose address `tile` is the same in every lane:
    // written as uniform base + 32-bit lane offset so that the load takes its base from scalar
    // registers and a streaming loop spends no vector instruction on addresses.
    static __device__ __forceinline__ Frag load_tile(const char* tile, uint32_t c, int h) {
        const uint32_t off = c * (uint32_t)ROW_BYTES + (uint32_t)h * (uint32_t)LANE_BYTES;
        Frag f;
#pragma unroll
        for (int i = 0; i < NV; ++i) f.v[i] = *reinterpret_cast<const uint4*>(tile + (off + 16u * i));
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

    // uniform tile address + 32-bit lane offsets (see Ops::load_tile)
    static __device__ __forceinline__ Frag load_tile(const char* tile, uint32_t c, int h) {
        Frag f;
        f.lo = *reinterpret_cast<const uint4*>(tile + (c * 48u + 16u * (uint32_t)h));
        f.hi = *reinterpret_cast<const uint2*>(tile + (c * 48u + 32u + 8u * (uint32_t)h));
        return f;
    }

    // The 12 fp32 values of an unprepared row that lane half h's fragment is made of (channels
    // 8h..8h+7 and 16+4h..16+4h+3), and the fragment they round to: bit for bit what the
    // prepare pass would have stored.  `row` must be 16-byte aligned.
    struct Raw {
        float4 a, b, c;
    };
    static __device__ __forceinline__ Raw load_raw(const float* row, int h) {
        Raw r;
        r.a = *reinterpret_cast<const float4*>(row + 8 * h);
        r.b = *reinterpret_cast<const float4*>(row + 8 * h + 4);
        r.c = *reinterpret_cast<const float4*>(row + 16 + 4 * h);
        return r;
    }
    static __device__ __forceinline__ Raw zero_raw() {
        Raw r;
        r.a = r.b = r.c = make_float4(0.f, 0.f, 0.f, 0.f);
        return r;
    }
    static __device__ __forceinline__ Frag round_raw(const Raw& r) {
        Frag f;
        f.lo = make_uint4(round_pair<CT>(r.a.x, r.a.y), round_pair<CT>(r.a.z, r.a.w), round_pair<CT>(r.b.x, r.b.y),
                          round_pair<CT>(r.b.z, r.b.w));
        f.hi = make_uint2(round_pair<CT>(r.c.x, r.c.y), round_pair<CT>(r.c.z, r.c.w));
        return f;
    }
    // lane (c, h)'s fragment into row c of a prepared 32-pixel tile (the layout load_tile reads)
    static __device__ __forceinline__ void store_tile(char* tile, uint32_t c, int h, const Frag& f) {
        *reinterpret_cast<uint4*>(tile + (c * 48u + 16u * (uint32_t)h)) = f.lo;
        *reinterpret_cast<uint2*>(tile + (c * 48u + 32u + 8u * (uint32_t)h)) = f.hi;
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

// Transposing maximum over the 32 lanes of each wave half, for 16 registers at once.  A
// plain butterfly costs 5 steps per register; here every step halves the number of live
// registers instead: after the step that joins lanes l and l^1 a lane keeps only the
// registers of one parity, after the next step one register in four, and so on, so the 16
// registers cost 8+4+2+1 select-and-join steps plus one row exchange.  On return lane l
// holds max over its half of x[held_register(l)].  The later steps join mirrored lanes
// (l with l^7, l with l^15), so the selection bits are chosen such that both partners of a
// step hold the same register: e0 = b0^b2, e1 = b1^b2, e2 = b2^b3, e3 = b3 (b = lane bits).
__device__ __forceinline__ int held_register(int lane) {
    const int b0 = lane & 1, b1 = (lane >> 1) & 1, b2 = (lane >> 2) & 1, b3 = (lane >> 3) & 1;
    return (b0 ^ b2) | ((b1 ^ b2) << 1) | ((b2 ^ b3) << 2) | (b3 << 3);
}
// Lane (0..15) of a 16-lane row that ends up holding register v: the inverse of held_register.
__device__ __forceinline__ constexpr int holder_lane(int v) {
    const int b3 = (v >> 3) & 1, b2 = ((v >> 2) & 1) ^ b3, b1 = ((v >> 1) & 1) ^ b2, b0 = (v & 1) ^ b2;
    return b0 | (b1 << 1) | (b2 << 2) | (b3 << 3);
}
template <int CTRL>
__device__ __forceinline__ float dpp_max(float x) { return __builtin_fmaxf(x, dpp_move<CTRL>(x)); }
__device__ __forceinline__ float transpose_max16(const float (&x)[16], int lane) {
    const int held = held_register(lane);
    const bool e0 = held & 1, e1 = held & 2, e2 = held & 4, e3 = held & 8;
    // both sides of every selection are formed first: a cross-lane move must be executed by
    // all lanes, so it cannot sit inside the arms of a conditional
    float y8[8], y4[4], y2[2];
#pragma unroll
    for (int k = 0; k < 8; ++k) {  // joins l and l ^ 1
        const float even = dpp_max<0xB1>(x[2 * k]), odd = dpp_max<0xB1>(x[2 * k + 1]);
        y8[k] = e0 ? odd : even;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {  // l and l ^ 2
        const float even = dpp_max<0x4E>(y8[2 * k]), odd = dpp_max<0x4E>(y8[2 * k + 1]);
        y4[k] = e1 ? odd : even;
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {  // l and l ^ 7
        const float even = dpp_max<0x141>(y4[2 * k]), odd = dpp_max<0x141>(y4[2 * k + 1]);
        y2[k] = e2 ? odd : even;
    }
    const float even = dpp_max<0x140>(y2[0]), odd = dpp_max<0x140>(y2[1]);  // l and l ^ 15
    const float y1 = e3 ? odd : even;
    const auto sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(y1), __float_as_uint(y1), false, false);
    return __builtin_fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));                              // both rows
}

// Lane LANE of `old` replaced by a wave-uniform value (the other lanes keep theirs).
template <int LANE>
__device__ __forceinline__ int write_lane(int old, int uniform_value) {
    static_assert(LANE >= 0 && LANE < 64, "lane of a 64-wide wave");
    asm("v_writelane_b32 %0, %1, %2" : "+v"(old) : "s"(uniform_value), "n"(LANE));
    return old;
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
