// "Segment major" storage of image 1 for the dense kernel.  Pixels are grouped into
// super-blocks of 32*S; inside a super-block, query block t (t < S) holds in its lane c the
// pixel  sb*32*S + c*S + t.  A lane that walks the S blocks of a super-block therefore sees
// S consecutive pixels, which makes "the lane that held the maximum" a contiguous pixel run.
#pragma once
#include <stdint.h>

namespace fnn {

constexpr int DENSE_S = 128;     // query blocks per super-block (a run is S consecutive pixels)

// pixel held by lane c of block t of super-block sb
__host__ __device__ inline int segment_pixel(int sb, int t, int c) { return sb * (32 * DENSE_S) + c * DENSE_S + t; }

// stored row (slot) of pixel i
__host__ __device__ inline int64_t segment_slot(int64_t i) {
    const int64_t sb = i / (32 * DENSE_S);
    const int w = (int)(i % (32 * DENSE_S));
    return (sb * DENSE_S + (w % DENSE_S)) * 32 + (w / DENSE_S);
}

// pixel stored in row `slot`
__host__ __device__ inline int64_t slot_pixel(int64_t slot) {
    const int64_t block = slot / 32;
    const int c = (int)(slot % 32);
    return (block / DENSE_S) * (32 * DENSE_S) + (int64_t)c * DENSE_S + (block % DENSE_S);
}

}  // namespace fnn
