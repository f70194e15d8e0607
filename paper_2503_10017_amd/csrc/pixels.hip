// The step after the matching path: the match set M, which the search kernels hold as flat
// pixel ids, written the way the problem statement writes a correspondence (section 3.1,
// "Problem Statement"): i = (w_i, h_i), j = (w_j, h_j), with an optional filter on the
// confidence maps that the regression heads emit next to the pointmaps (section 3.2.3).
#include "fnn_device.hpp"
#include "fnn_kernels.hpp"
#include "trace.hpp"

namespace fnn {

constexpr int PIXEL_THREADS = 1024;

// conf >= threshold as an ordered comparison that does not rely on how the compiler treats
// NaN (the library is built with the assumption that scores are finite): a NaN on either side
// is recognised from its bits and fails the test.
__device__ __forceinline__ bool confident(float conf, float threshold) {
    const uint32_t cb = __float_as_uint(conf) & 0x7FFFFFFFu, tb = __float_as_uint(threshold) & 0x7FFFFFFFu;
    if (cb > 0x7F800000u || tb > 0x7F800000u) return false;
    return conf >= threshold;
}

// One workgroup per image pair walks the pair list in chunks of 1024; a prefix sum over the
// "kept" flags gives every surviving match its slot, so the output keeps the input order.
__global__ __launch_bounds__(PIXEL_THREADS) void pairs_to_pixels_kernel(PixelArgs a) {
    __shared__ int wave_sums[17];
    const int b = blockIdx.x;
    const int32_t* pairs = a.pairs + (int64_t)b * a.max_pairs * 2;
    int32_t* out = a.out_xy + (int64_t)b * a.max_pairs * 4;
    const float* c1 = a.conf1 ? a.conf1 + (int64_t)b * a.n : nullptr;
    const float* c2 = a.conf2 ? a.conf2 + (int64_t)b * a.m : nullptr;
    int64_t count = a.n_pairs[b];
    count = count < 0 ? 0 : (count > a.max_pairs ? a.max_pairs : count);
    int64_t kept = 0;
    for (int64_t start = 0; start < count; start += PIXEL_THREADS) {
        const int64_t p = start + threadIdx.x;
        bool keep = false;
        int32_t i = 0, j = 0;
        if (p < count) {
            i = pairs[2 * p];
            j = pairs[2 * p + 1];
            keep = i >= 0 && i < a.n && j >= 0 && j < a.m;
            if (keep && c1) keep = confident(c1[i], a.min_conf1);  // a NaN confidence drops the match
            if (keep && c2) keep = confident(c2[j], a.min_conf2);
        }
        int total;
        const int before = block_scan_flag(keep, wave_sums, total);
        if (keep) {
            int32_t* row = out + (kept + before) * 4;
            row[0] = i % a.width1;
            row[1] = i / a.width1;
            row[2] = j % a.width2;
            row[3] = j / a.width2;
        }
        kept += total;
    }
    for (int64_t e = kept * 4 + threadIdx.x; e < a.max_pairs * 4; e += PIXEL_THREADS) out[e] = -1;
    if (threadIdx.x == 0) a.out_count[b] = (int32_t)kept;
}

hipError_t launch_pairs_to_pixels(const PixelArgs& a, int batch, hipStream_t s) {
    return launch(TK_PIXELS, pairs_to_pixels_kernel, dim3(batch), dim3(PIXEL_THREADS), 0, s, a);
}

}  // namespace fnn
