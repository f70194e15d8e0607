// C entry points of libfnn (see include/fnn.h): argument checks, workspace carving and the
// fixed kernel sequences.  Nothing here synchronises with the device or allocates memory.
#include <hip/hip_runtime.h>
#include <string.h>

#include "dense_perm.hpp"
#include "fnn_kernels.hpp"

using namespace fnn;

namespace {

constexpr int64_t MAX_PIXELS = 2147483647LL - 64;
constexpr int64_t MAX_DENSE_PIXELS = 1LL << 30;  // keeps the padded bucket lists of the dense mode within int32
constexpr size_t WS_ALIGN = 256;

struct Carver {
    char* base;
    size_t used;
    void* take(size_t bytes) {
        void* p = base ? base + used : nullptr;
        used += (bytes + WS_ALIGN - 1) / WS_ALIGN * WS_ALIGN;
        return p;
    }
};

bool valid_dtype(int32_t t) { return t == FNN_F32 || t == FNN_F16 || t == FNN_BF16; }

struct MapsLayout {
    void* p1;
    void* p2;
    int64_t n_pad, m_pad;
    int64_t bstride1, bstride2;  // bytes per pair
    int dp;
};

MapsLayout carve_maps(Carver& cv, int batch, int64_t n, int64_t m, int d, int compute, int64_t n_align = 32) {
    MapsLayout L;
    L.dp = padded_d(d, compute);
    L.n_pad = round_up(n, n_align);
    L.m_pad = round_up(m, 32);
    const int es = elem_size(compute);
    L.bstride1 = L.n_pad * L.dp * es;
    L.bstride2 = L.m_pad * L.dp * es;
    L.p1 = cv.take((size_t)batch * L.bstride1);
    L.p2 = cv.take((size_t)batch * L.bstride2);
    return L;
}

struct NearestLayout {
    MapsLayout maps;
    u64* keys;
};
NearestLayout carve_nearest(Carver& cv, int batch, int64_t n, int64_t m, int d, int64_t nq, int compute) {
    NearestLayout L;
    L.maps = carve_maps(cv, batch, n, m, d, compute);
    L.keys = (u64*)cv.take((size_t)batch * nq * sizeof(u64));
    return L;
}

struct RecipLayout {
    MapsLayout maps;
    RecipState st;
    int64_t zero_words;  // 64-bit words from keys_f to the end of the bitmap
};
RecipLayout carve_recip(Carver& cv, int batch, int64_t n, int64_t m, int d, int64_t n_seeds, int compute) {
    RecipLayout L;
    L.maps = carve_maps(cv, batch, n, m, d, compute);
    const size_t per = (size_t)batch * n_seeds;
    // keys_f, keys_b and the bitmap are adjacent so that one range clears all three
    const size_t z0 = cv.used;
    L.st.keys_f = (u64*)cv.take(per * sizeof(u64));
    L.st.keys_b = (u64*)cv.take(per * sizeof(u64));
    L.st.n_words = (n + 31) / 32;
    L.st.bitmap = (uint32_t*)cv.take((size_t)batch * L.st.n_words * sizeof(uint32_t));
    L.zero_words = (int64_t)((cv.used - z0) / sizeof(u64));
    L.st.cur_u[0] = (int32_t*)cv.take(per * sizeof(int32_t));
    L.st.cur_u[1] = (int32_t*)cv.take(per * sizeof(int32_t));
    L.st.seed_id[0] = (int32_t*)cv.take(per * sizeof(int32_t));
    L.st.seed_id[1] = (int32_t*)cv.take(per * sizeof(int32_t));
    L.st.n_active = (int32_t*)cv.take((size_t)batch * sizeof(int32_t));
    L.st.word_rank = (int32_t*)cv.take((size_t)batch * L.st.n_words * sizeof(int32_t));
    return L;
}

struct DenseLayout {
    MapsLayout maps;
    u64* row_keys;
    u64* col_keys;
    int32_t* unit_counts;
    int64_t zero_words;  // 64-bit words from row_keys to the end of unit_counts
    int32_t row_units, col_units;
    int64_t rows_cap, cols_cap;
    int32_t* unit_cursor;
    int32_t* lists;
    int32_t* chunk_unit;
    int32_t* chunk_totals;
    int32_t* block_counts;
    int64_t blocks_per_pair;
};
DenseLayout carve_dense(Carver& cv, int batch, int64_t n, int64_t m, int d, int compute) {
    DenseLayout L;
    L.maps = carve_maps(cv, batch, n, m, d, compute, 32 * DENSE_S);
    // the two key tables and the bucket counters are adjacent so that one range clears them all
    const size_t z0 = cv.used;
    L.row_keys = (u64*)cv.take((size_t)batch * (n + m) * sizeof(u64));
    L.col_keys = L.row_keys ? L.row_keys + (size_t)batch * n : nullptr;
    L.row_units = (int32_t)((L.maps.m_pad / 32 + DENSE_J - 1) / DENSE_J);
    L.col_units = (int32_t)(L.maps.n_pad / DENSE_S);
    const size_t units = (size_t)batch * ((size_t)L.row_units + L.col_units);
    L.unit_counts = (int32_t*)cv.take(units * sizeof(int32_t));
    L.zero_words = (int64_t)((cv.used - z0) / sizeof(u64));
    L.unit_cursor = (int32_t*)cv.take(units * sizeof(int32_t));
    L.rows_cap = round_up(n, 32) + 32 * (int64_t)L.row_units;
    L.cols_cap = round_up(m, 32) + 32 * (int64_t)L.col_units;
    L.lists = (int32_t*)cv.take((size_t)batch * (L.rows_cap + L.cols_cap) * sizeof(int32_t));
    L.chunk_unit = (int32_t*)cv.take((size_t)batch * ((L.rows_cap + L.cols_cap) / 32) * sizeof(int32_t));
    L.chunk_totals = (int32_t*)cv.take((size_t)batch * 2 * sizeof(int32_t));
    const int64_t most = n > m ? n : m;
    L.blocks_per_pair = (most + 1023) / 1024;
    L.block_counts = (int32_t*)cv.take((size_t)batch * (L.blocks_per_pair + 1) * sizeof(int32_t));
    return L;
}

bool shape_ok(int32_t batch, int64_t n, int64_t m, int32_t d, int64_t nq) {
    return batch >= 1 && batch <= FNN_MAX_BATCH && n >= 0 && m >= 0 && n <= MAX_PIXELS && m <= MAX_PIXELS &&
           d >= 1 && d <= FNN_MAX_D && nq >= 0 && nq <= MAX_PIXELS;
}

// Checks a host array of `batch` maps that must share shape and format.
int32_t check_maps(int32_t batch, const fnn_map* maps) {
    if (!maps) return FNN_E_NULL;
    for (int b = 0; b < batch; ++b) {
        const fnn_map& mp = maps[b];
        if (!valid_dtype(mp.dtype)) return FNN_E_DTYPE;
        if (mp.n < 0 || mp.n > MAX_PIXELS || mp.d < 1 || mp.d > FNN_MAX_D || mp.row_stride < mp.d) return FNN_E_SHAPE;
        if (mp.n != maps[0].n || mp.d != maps[0].d || mp.dtype != maps[0].dtype || mp.row_stride != maps[0].row_stride)
            return FNN_E_SHAPE;
        if (mp.n > 0 && !mp.data) return FNN_E_NULL;
    }
    return FNN_OK;
}

int32_t check_opts(const fnn_opts* o) {
    if (!o) return FNN_E_NULL;
    if (!valid_dtype(o->compute)) return FNN_E_DTYPE;
    if (o->max_iter < 0) return FNN_E_RANGE;
    if (o->flags & ~(FNN_FLAG_NORMALIZE | FNN_FLAG_HALF_ACCUMULATE | FNN_FLAG_L2 | FNN_FLAG_SPLIT)) return FNN_E_RANGE;
    for (int i = 0; i < 5; ++i)
        if (o->reserved[i] != 0) return FNN_E_RANGE;
    return FNN_OK;
}

// Channels the prepared rows must hold for this call (descriptor + L2 norm channels), or
// -1 when they do not fit the widest row the kernels take.
int32_t row_channels(int32_t d, const fnn_opts* o) {
    const bool split = (o->flags & FNN_FLAG_SPLIT) != 0;
    const int32_t de = effective_d(d, o->compute, (o->flags & FNN_FLAG_L2) != 0, split);
    return de <= (split ? MAX_ROW_CHANNELS : FNN_MAX_D) ? de : -1;
}
// FNN_FLAG_SPLIT is defined for fp16 products and the dot-product score only.
bool split_unsupported(const fnn_opts* o) {
    return (o->flags & FNN_FLAG_SPLIT) && (o->compute != FNN_F16 || (o->flags & FNN_FLAG_L2));
}

int32_t check_workspace(const void* ws, size_t have, size_t need) {
    if (need == 0) return FNN_OK;
    if (!ws || ((uintptr_t)ws % WS_ALIGN) != 0 || have < need) return FNN_E_WORKSPACE;
    return FNN_OK;
}

void fill_prep_side(PrepSide& sd, int32_t batch, const fnn_map* maps, int64_t n_pad, void* dst, int second_image) {
    memset(&sd, 0, sizeof(sd));
    sd.second_image = second_image;
    for (int b = 0; b < batch; ++b) sd.src[b] = maps[b].data;
    sd.n = maps[0].n;
    sd.n_pad = n_pad;
    sd.row_stride = maps[0].row_stride;
    sd.dtype = maps[0].dtype;
    sd.dst = dst;
}

// A batch of caller maps that already has the layout the kernels read: stored in the compute
// format, dp channels per row, rows packed, whole 32-pixel tiles, 16-byte aligned, and the
// pairs equally spaced in memory (one stacked array).  Such maps are used where they are.
bool direct_layout(int32_t batch, const fnn_map* maps, const fnn_opts* opts, int dp, const char** base, int64_t* bstride) {
    const fnn_map& m0 = maps[0];
    if (opts->flags != 0) return false;
    for (int b = 0; b < batch; ++b)
        if (maps[b].dtype != opts->compute || maps[b].d != dp || maps[b].row_stride != dp || maps[b].n != m0.n) return false;
    if (m0.n <= 0 || m0.n % 32 != 0 || ((uintptr_t)m0.data % 16) != 0) return false;
    const int64_t bytes = m0.n * dp * elem_size(opts->compute);
    int64_t stride = 0;
    if (batch > 1) {
        stride = (const char*)maps[1].data - (const char*)m0.data;
        if (stride < bytes || stride % 16 != 0) return false;
        for (int b = 2; b < batch; ++b)
            if ((const char*)maps[b].data != (const char*)m0.data + (int64_t)b * stride) return false;
    }
    *base = (const char*)m0.data;
    *bstride = stride;
    return true;
}

// Caller maps that the fused first searches can read where they are (they round the fp32 rows
// themselves and write the prepared copy as a by-product): plain fp32 rows of 24 channels that
// start on 16-byte boundaries, a 16-bit compute format, no options, enough queries.
bool raw_rows(int32_t batch, const fnn_map* maps) {
    for (int i = 0; i < batch; ++i)
        if (maps[i].dtype != FNN_F32 || maps[i].d != 24 || maps[i].row_stride % 4 != 0 || maps[i].n <= 0 ||
            ((uintptr_t)maps[i].data % 16) != 0)
            return false;
    return true;
}
bool raw_options(const fnn_opts* opts) {
    return opts->flags == 0 && (opts->compute == FNN_F16 || opts->compute == FNN_BF16);
}
bool raw_first_search(int32_t batch, const fnn_map* a, const fnn_map* b, const fnn_opts* opts, int64_t n_queries) {
    return raw_options(opts) && first_search_applies(n_queries, a[0].n, batch) && first_search_applies(n_queries, b[0].n, batch) &&
           raw_rows(batch, a) && raw_rows(batch, b);
}
void fill_raw(RawMaps& r, int32_t batch, const fnn_map* maps) {
    memset(&r, 0, sizeof(r));
    for (int i = 0; i < batch; ++i) r.map[i] = (const float*)maps[i].data;
    r.row_stride = maps[0].row_stride;
}

// Prepares the maps that are not used in place (skip_a / skip_b) and runs the side jobs.
hipError_t prep_both(int32_t batch, const fnn_map* a, const fnn_map* b, const MapsLayout& L, int d, const fnn_opts* opts,
                     hipStream_t s, const PrepExtra& extra, bool first_segment_major = false, bool skip_a = false,
                     bool skip_b = false) {
    const int compute = opts->compute;
    PrepArgs pa;
    memset(&pa, 0, sizeof(pa));
    pa.extra = extra;
    int sides = 0;
    if (!skip_a) {
        fill_prep_side(pa.side[sides], batch, a, L.n_pad, L.p1, 0);
        pa.side[sides].segment_major = first_segment_major ? 1 : 0;
        ++sides;
    }
    if (!skip_b) {
        fill_prep_side(pa.side[sides], batch, b, L.m_pad, L.p2, 1);
        ++sides;
    }
    pa.n_sides = sides;
    pa.batch = batch;
    pa.d = d;
    pa.dp = L.dp;
    pa.compute = compute;
    pa.normalize = (opts->flags & FNN_FLAG_NORMALIZE) ? 1 : 0;
    pa.l2 = (opts->flags & FNN_FLAG_L2) ? 1 : 0;
    pa.split = (opts->flags & FNN_FLAG_SPLIT) ? 1 : 0;
    return launch_prep(pa, s);
}

#define FNN_TRY(expr)                        \
    do {                                     \
        if ((expr) != hipSuccess) return FNN_E_HIP; \
    } while (0)

}  // namespace

// ---- scratch of fnn_reciprocal_static ----------------------------------------------------------
// One array per device (every device that loads the library holds its own copy at its own
// address, for the life of the process).  In host code the array's name is only a handle: the
// memory is reached through the address that hipGetSymbolAddress returns for the current device,
// looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[FNN_STATIC_SCRATCH_BYTES];

static struct StaticScratch {
    std::mutex mu;
    void* ptr[DeviceCache::MAX_DEVICES] = {};
} g_static_scratch;

// Address of the current device's scratch array, or NULL (a HIP call failed).  Allocates nothing.
static void* static_scratch_for_current_device() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= DeviceCache::MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> lock(g_static_scratch.mu);
    if (!g_static_scratch.ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_static_scratch.ptr[dev] = p;
    }
    return g_static_scratch.ptr[dev];
}

#pragma GCC visibility push(default)
extern "C" {

const char* fnn_status_string(int32_t status) {
    switch (status) {
        case FNN_OK: return "ok";
        case FNN_E_NULL: return "a required pointer is NULL";
        case FNN_E_SHAPE: return "shape out of range or inconsistent";
        case FNN_E_DTYPE: return "unknown storage or compute format";
        case FNN_E_RANGE: return "option out of range";
        case FNN_E_WORKSPACE: return "workspace missing, misaligned or too small";
        case FNN_E_HIP: return "a HIP call or kernel launch failed";
        case FNN_E_UNSUPPORTED: return "request not supported by this build";
        default: return "unknown status";
    }
}

size_t fnn_workspace_bytes_opts(int32_t batch, int64_t n, int64_t m, int32_t d, int64_t n_queries,
                                const fnn_opts* opts) {
    if (!shape_ok(batch, n, m, d, n_queries) || check_opts(opts) != FNN_OK || split_unsupported(opts)) return 0;
    const int32_t de = row_channels(d, opts);
    if (de < 0) return 0;
    const int32_t compute = opts->compute;
    size_t most = 0;
    {
        Carver cv{nullptr, 0};
        carve_nearest(cv, batch, n, m, de, n_queries, compute);
        most = cv.used;
    }
    {
        Carver cv{nullptr, 0};
        carve_recip(cv, batch, n, m, de, n_queries, compute);
        if (cv.used > most) most = cv.used;
    }
    {
        Carver cv{nullptr, 0};
        carve_dense(cv, batch, n, m, de, compute);
        if (cv.used > most) most = cv.used;
    }
    return most + WS_ALIGN;
}

size_t fnn_workspace_bytes(int32_t batch, int64_t n, int64_t m, int32_t d, int64_t n_queries, int32_t compute) {
    fnn_opts o;
    memset(&o, 0, sizeof(o));
    o.compute = compute;
    return fnn_workspace_bytes_opts(batch, n, m, d, n_queries, &o);
}

int32_t fnn_nearest(int32_t batch, const fnn_map* src, const int32_t* q_idx, int64_t nq, const int32_t* nq_active,
                    const fnn_map* tgt, const fnn_opts* opts, int32_t* out_idx, float* out_score, void* workspace,
                    size_t workspace_bytes, void* stream) {
    if (batch < 1 || batch > FNN_MAX_BATCH) return FNN_E_SHAPE;
    int32_t st = check_maps(batch, src);
    if (st != FNN_OK) return st;
    st = check_maps(batch, tgt);
    if (st != FNN_OK) return st;
    st = check_opts(opts);
    if (st != FNN_OK) return st;
    if ((opts->flags & FNN_FLAG_HALF_ACCUMULATE) || split_unsupported(opts)) return FNN_E_UNSUPPORTED;
    const int64_t n = src[0].n, m = tgt[0].n;
    const int32_t d = src[0].d;
    if (tgt[0].d != d || nq < 0 || nq > MAX_PIXELS) return FNN_E_SHAPE;
    const int32_t de = row_channels(d, opts);
    if (de < 0) return FNN_E_SHAPE;
    if (!q_idx && nq > n) return FNN_E_SHAPE;
    if (nq > 0 && n == 0) return FNN_E_SHAPE;
    if (nq > 0 && !out_idx) return FNN_E_NULL;
    if (nq == 0) return FNN_OK;

    Carver cv{(char*)workspace, 0};
    NearestLayout L = carve_nearest(cv, batch, n, m, de, nq, opts->compute);
    st = check_workspace(workspace, workspace_bytes, cv.used);
    if (st != FNN_OK) return st;
    hipStream_t s = (hipStream_t)stream;

    PrepExtra extra;
    memset(&extra, 0, sizeof(extra));
    extra.zero_ptr = L.keys;  // the key table starts empty
    extra.zero_count = (int64_t)batch * nq;
    const char *p1 = (const char*)L.maps.p1, *p2 = (const char*)L.maps.p2;
    int64_t bs1 = L.maps.bstride1, bs2 = L.maps.bstride2;
    const bool direct1 = direct_layout(batch, src, opts, L.maps.dp, &p1, &bs1);
    const bool direct2 = direct_layout(batch, tgt, opts, L.maps.dp, &p2, &bs2);
    // With every query live and enough of them, the search runs in the kernel that stages the
    // candidate tiles through LDS; fp32 maps of the paper's shape are then read where they are (no
    // prepare pass: the search leaves the prepared candidates behind for the resolve pass).
    const bool staged_shape = !nq_active && first_search_applies(nq, m, batch);
    const bool fused = staged_shape && raw_options(opts) && raw_rows(batch, src) && raw_rows(batch, tgt);
    const bool staged = fused || (staged_shape && L.maps.dp == 24 && opts->compute != FNN_F32);
    FNN_TRY(prep_both(batch, src, tgt, L.maps, d, opts, s, extra, false, direct1 || fused, direct2 || fused));
    SearchArgs sa;
    memset(&sa, 0, sizeof(sa));
    sa.src = p1;
    sa.src_bstride = bs1;
    sa.src_rows = (int32_t)L.maps.n_pad;
    sa.q_idx = q_idx;
    sa.nq_active = nq_active;
    sa.nq = (int32_t)nq;
    sa.tgt = p2;
    sa.tgt_bstride = bs2;
    sa.m = (int32_t)m;
    sa.m_tiles = (int32_t)(L.maps.m_pad / 32);
    sa.out_keys = L.keys;
    if (staged) {
        FirstSearchArgs first;
        memset(&first, 0, sizeof(first));
        first.s = sa;
        if (fused) {
            first.s.src_rows = (int32_t)n;  // query rows are clamped to the caller's map, which has no padding rows
            fill_raw(first.raw_tgt, batch, tgt);
            fill_raw(first.raw_src, batch, src);
            first.raw_queries = 1;
        }
        FNN_TRY(launch_search_first(first, batch, opts->compute, s));
        if (fused) {
            FNN_TRY(launch_resolve_raw(first, batch, opts->compute, out_idx, out_score, s));
            return FNN_OK;
        }
    } else {
        FNN_TRY(launch_search(sa, batch, opts->compute, L.maps.dp, s));
    }
    FNN_TRY(launch_resolve(sa, batch, opts->compute, L.maps.dp, out_idx, out_score, s));
    return FNN_OK;
}

size_t fnn_blocked_workspace_bytes(int64_t n, int64_t m, int32_t d, int32_t block_rows, int32_t block_cols,
                                   int32_t compute) {
    if (!shape_ok(1, n, m, d, 0) || !valid_dtype(compute) || block_rows < 1 || block_cols < 0) return 0;
    Carver cv{nullptr, 0};
    carve_maps(cv, 1, n, m, d, compute);
    const int64_t ld = block_cols > 0 ? round_up(block_cols, 32) : round_up(m, 32);
    cv.take((size_t)block_rows * ld * sizeof(float));
    return cv.used + WS_ALIGN;
}

int32_t fnn_nearest_blocked(const fnn_map* src, const int32_t* q_idx, int64_t nq, const fnn_map* tgt,
                            const fnn_opts* opts, int32_t block_rows, int32_t block_cols, int32_t* out_idx,
                            float* out_score, void* workspace, size_t workspace_bytes, void* stream) {
    int32_t st = check_maps(1, src);
    if (st != FNN_OK) return st;
    st = check_maps(1, tgt);
    if (st != FNN_OK) return st;
    st = check_opts(opts);
    if (st != FNN_OK) return st;
    if ((opts->flags & FNN_FLAG_HALF_ACCUMULATE) && opts->compute != FNN_F16) return FNN_E_UNSUPPORTED;
    if (opts->flags & (FNN_FLAG_L2 | FNN_FLAG_SPLIT)) return FNN_E_UNSUPPORTED;
    const int64_t n = src[0].n, m = tgt[0].n;
    const int32_t d = src[0].d;
    if (tgt[0].d != d || nq < 0 || nq > MAX_PIXELS || block_rows < 1 || block_cols < 0) return FNN_E_SHAPE;
    if ((!q_idx && nq > n) || (nq > 0 && n == 0)) return FNN_E_SHAPE;
    if (nq > 0 && (!out_idx || !out_score)) return FNN_E_NULL;
    if (nq == 0) return FNN_OK;

    Carver cv{(char*)workspace, 0};
    MapsLayout L = carve_maps(cv, 1, n, m, d, opts->compute);
    const int64_t ld = block_cols > 0 ? round_up(block_cols, 32) : round_up(m, 32);
    float* dists = (float*)cv.take((size_t)block_rows * ld * sizeof(float));
    st = check_workspace(workspace, workspace_bytes, cv.used);
    if (st != FNN_OK) return st;
    hipStream_t s = (hipStream_t)stream;

    PrepExtra extra;
    memset(&extra, 0, sizeof(extra));
    FNN_TRY(prep_both(1, src, tgt, L, d, opts, s, extra));
    if (m == 0) {
        FNN_TRY(launch_fill_i32f32(out_idx, out_score, nq, s));
        return FNN_OK;
    }
    BlockedArgs ba;
    memset(&ba, 0, sizeof(ba));
    ba.src = (const char*)L.p1;
    ba.src_rows = (int32_t)L.n_pad;
    ba.q_idx = q_idx;
    ba.nq = (int32_t)nq;
    ba.tgt = (const char*)L.p2;
    ba.m = (int32_t)m;
    ba.dists = dists;
    ba.ld = ld;
    ba.out_idx = out_idx;
    ba.out_score = out_score;
    ba.half_accumulate = (opts->flags & FNN_FLAG_HALF_ACCUMULATE) ? 1 : 0;
    FNN_TRY(run_blocked(ba, opts->compute, d, L.dp, block_rows, (int)(block_cols > 0 ? ld : 0), s));
    return FNN_OK;
}

// The FastNN iteration.  use_static: the workspace is the library's own scratch array of the
// current device (looked up only after every argument check has passed).
static int32_t reciprocal_impl(int32_t batch, const fnn_map* d1, const fnn_map* d2, const int32_t* seeds, int64_t n_seeds,
                               const fnn_opts* opts, int32_t* seed_i, int32_t* seed_j, int32_t* seed_iter, int32_t* pairs,
                               int32_t* n_pairs, void* workspace, size_t workspace_bytes, bool use_static, void* stream) {
    if (batch < 1 || batch > FNN_MAX_BATCH) return FNN_E_SHAPE;
    int32_t st = check_maps(batch, d1);
    if (st != FNN_OK) return st;
    st = check_maps(batch, d2);
    if (st != FNN_OK) return st;
    st = check_opts(opts);
    if (st != FNN_OK) return st;
    if ((opts->flags & FNN_FLAG_HALF_ACCUMULATE) || split_unsupported(opts)) return FNN_E_UNSUPPORTED;
    const int64_t n = d1[0].n, m = d2[0].n;
    const int32_t d = d1[0].d;
    if (d2[0].d != d || n_seeds < 0 || n_seeds > MAX_PIXELS) return FNN_E_SHAPE;
    const int32_t de = row_channels(d, opts);
    if (de < 0) return FNN_E_SHAPE;
    if (n_seeds > 0 && (n == 0 || m == 0)) return FNN_E_SHAPE;
    if (!n_pairs) return FNN_E_NULL;
    if (n_seeds > 0 && (!seeds || !seed_i || !seed_j || !seed_iter || !pairs)) return FNN_E_NULL;

    if (use_static) {
        Carver need{nullptr, 0};
        carve_recip(need, batch, n, m, de, n_seeds, opts->compute);
        if (need.used > FNN_STATIC_SCRATCH_BYTES) return FNN_E_WORKSPACE;  // before the device is touched
        workspace = static_scratch_for_current_device();
        if (!workspace) return FNN_E_HIP;
        workspace_bytes = FNN_STATIC_SCRATCH_BYTES;
    }
    Carver cv{(char*)workspace, 0};
    RecipLayout L = carve_recip(cv, batch, n, m, de, n_seeds, opts->compute);
    st = check_workspace(workspace, workspace_bytes, cv.used);
    if (st != FNN_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    const int compute = opts->compute;
    const int32_t ns = (int32_t)n_seeds;

    if (ns == 0) {
        // nothing to match: only the counts are defined
        RecipState none = L.st;
        none.n_words = 0;
        FNN_TRY(launch_recip_dedup(none, 0, batch, seed_i, seed_j, seed_iter, pairs, n_pairs, s));
        return FNN_OK;
    }

    // the prepare launch also clears the key tables and the sort bitmap and sets U^0 = seeds
    PrepExtra extra;
    memset(&extra, 0, sizeof(extra));
    extra.zero_ptr = L.st.keys_f;
    extra.zero_count = L.zero_words;
    extra.seeds = seeds;
    extra.cur_u = L.st.cur_u[0];
    extra.seed_id = L.st.seed_id[0];
    extra.n_active = L.st.n_active;
    extra.n_seeds = ns;
    const char *p1 = (const char*)L.maps.p1, *p2 = (const char*)L.maps.p2;
    int64_t bs1 = L.maps.bstride1, bs2 = L.maps.bstride2;
    const bool direct1 = direct_layout(batch, d1, opts, L.maps.dp, &p1, &bs1);
    const bool direct2 = direct_layout(batch, d2, opts, L.maps.dp, &p2, &bs2);
    // fp32 maps of the paper's shape: no prepare pass; the first forward and the first backward
    // search read the caller's maps and leave the prepared copies behind for the later searches
    const bool fused = raw_first_search(batch, d1, d2, opts, n_seeds);
    // the same LDS-staged kernel serves the first two searches on prepared 24-channel maps
    const bool staged = fused || (L.maps.dp == 24 && opts->compute != FNN_F32 && first_search_applies(n_seeds, n, batch) &&
                                  first_search_applies(n_seeds, m, batch));
    FNN_TRY(prep_both(batch, d1, d2, L.maps, d, opts, s, extra, false, direct1 || fused, direct2 || fused));

    SearchArgs fwd;  // queries in image 1 -> candidates in image 2
    memset(&fwd, 0, sizeof(fwd));
    fwd.src = p1;
    fwd.src_bstride = bs1;
    fwd.src_rows = (int32_t)L.maps.n_pad;
    fwd.nq_active = L.st.n_active;
    fwd.nq = ns;
    fwd.tgt = p2;
    fwd.tgt_bstride = bs2;
    fwd.m = (int32_t)m;
    fwd.m_tiles = (int32_t)(L.maps.m_pad / 32);
    fwd.out_keys = L.st.keys_f;

    SearchArgs bwd;  // queries in image 2 (named by the index field of keys_f) -> image 1
    memset(&bwd, 0, sizeof(bwd));
    bwd.src = p2;
    bwd.src_bstride = bs2;
    bwd.src_rows = (int32_t)L.maps.m_pad;
    bwd.q_keys = L.st.keys_f;
    bwd.nq_active = L.st.n_active;
    bwd.nq = ns;
    bwd.tgt = p1;
    bwd.tgt_bstride = bs1;
    bwd.m = (int32_t)n;
    bwd.m_tiles = (int32_t)(L.maps.n_pad / 32);
    bwd.out_keys = L.st.keys_b;

    int which = 0;
    fwd.q_idx = L.st.cur_u[which];
    if (fused) {
        FirstSearchArgs first;  // V^0 = NN_2(U^0): queries and candidates still raw; writes the prepared image 2
        first.s = fwd;
        first.s.src_rows = (int32_t)n;  // query rows are clamped to the caller's map, which has no padding rows
        fill_raw(first.raw_tgt, batch, d2);
        fill_raw(first.raw_src, batch, d1);
        first.raw_queries = 1;
        FNN_TRY(launch_search_first(first, batch, compute, s));
        FNN_TRY(launch_resolve_raw(first, batch, compute, nullptr, nullptr, s));
    } else if (staged) {
        FirstSearchArgs first;
        memset(&first, 0, sizeof(first));
        first.s = fwd;
        FNN_TRY(launch_search_first(first, batch, compute, s));
        FNN_TRY(launch_resolve(fwd, batch, compute, L.maps.dp, nullptr, nullptr, s));
    } else {
        FNN_TRY(launch_search(fwd, batch, compute, L.maps.dp, s));  // V^0 = NN_2(U^0)
        FNN_TRY(launch_resolve(fwd, batch, compute, L.maps.dp, nullptr, nullptr, s));
    }
    if (opts->max_iter == 0) {
        FNN_TRY(launch_recip_step(L.st, which, ns, batch, 0, 2, seed_i, seed_j, seed_iter, s));
    }
    for (int t = 0; t < opts->max_iter; ++t) {
        const bool last = (t == opts->max_iter - 1);
        if (staged && t == 0) {
            FirstSearchArgs first;  // U^1 = NN_1(V^0): queries from the prepared image 2; if raw, writes the prepared image 1
            memset(&first, 0, sizeof(first));
            first.s = bwd;
            if (fused) fill_raw(first.raw_tgt, batch, d1);
            FNN_TRY(launch_search_first(first, batch, compute, s));
        } else {
            FNN_TRY(launch_search(bwd, batch, compute, L.maps.dp, s));  // U^{t+1} = NN_1(V^t)
        }
        FNN_TRY(launch_resolve(bwd, batch, compute, L.maps.dp, nullptr, nullptr, s));
        FNN_TRY(launch_recip_step(L.st, which, ns, batch, t, last ? 1 : 0, seed_i, seed_j, seed_iter, s));
        if (last) break;
        which ^= 1;
        fwd.q_idx = L.st.cur_u[which];
        FNN_TRY(launch_search(fwd, batch, compute, L.maps.dp, s));  // V^{t+1} = NN_2(U^{t+1})
        FNN_TRY(launch_resolve(fwd, batch, compute, L.maps.dp, nullptr, nullptr, s));
    }
    FNN_TRY(launch_recip_dedup(L.st, ns, batch, seed_i, seed_j, seed_iter, pairs, n_pairs, s));
    return FNN_OK;
}

int32_t fnn_reciprocal(int32_t batch, const fnn_map* d1, const fnn_map* d2, const int32_t* seeds, int64_t n_seeds,
                       const fnn_opts* opts, int32_t* seed_i, int32_t* seed_j, int32_t* seed_iter, int32_t* pairs,
                       int32_t* n_pairs, void* workspace, size_t workspace_bytes, void* stream) {
    return reciprocal_impl(batch, d1, d2, seeds, n_seeds, opts, seed_i, seed_j, seed_iter, pairs, n_pairs, workspace,
                           workspace_bytes, false, stream);
}

int32_t fnn_reciprocal_static(int32_t batch, const fnn_map* d1, const fnn_map* d2, const int32_t* seeds, int64_t n_seeds,
                              const fnn_opts* opts, int32_t* seed_i, int32_t* seed_j, int32_t* seed_iter, int32_t* pairs,
                              int32_t* n_pairs, void* stream) {
    return reciprocal_impl(batch, d1, d2, seeds, n_seeds, opts, seed_i, seed_j, seed_iter, pairs, n_pairs, nullptr, 0,
                           true, stream);
}

int32_t fnn_mutual_dense(int32_t batch, const fnn_map* d1, const fnn_map* d2, const fnn_opts* opts, int32_t* nn12,
                         float* s12, int32_t* nn21, float* s21, int32_t* pairs, int32_t* n_pairs, void* workspace,
                         size_t workspace_bytes, void* stream) {
    if (batch < 1 || batch > FNN_MAX_BATCH) return FNN_E_SHAPE;
    int32_t st = check_maps(batch, d1);
    if (st != FNN_OK) return st;
    st = check_maps(batch, d2);
    if (st != FNN_OK) return st;
    st = check_opts(opts);
    if (st != FNN_OK) return st;
    if ((opts->flags & FNN_FLAG_HALF_ACCUMULATE) || split_unsupported(opts)) return FNN_E_UNSUPPORTED;
    const int64_t n = d1[0].n, m = d2[0].n;
    const int32_t d = d1[0].d;
    if (d2[0].d != d) return FNN_E_SHAPE;
    if (n > MAX_DENSE_PIXELS || m > MAX_DENSE_PIXELS) return FNN_E_SHAPE;
    const int32_t de = row_channels(d, opts);
    if (de < 0) return FNN_E_SHAPE;
    if (!n_pairs) return FNN_E_NULL;
    if ((n > 0 && !nn12) || (m > 0 && !nn21)) return FNN_E_NULL;
    if (n > 0 && m > 0 && !pairs) return FNN_E_NULL;

    Carver cv{(char*)workspace, 0};
    DenseLayout L = carve_dense(cv, batch, n, m, de, opts->compute);
    st = check_workspace(workspace, workspace_bytes, cv.used);
    if (st != FNN_OK) return st;
    hipStream_t s = (hipStream_t)stream;

    PrepExtra extra;
    memset(&extra, 0, sizeof(extra));
    extra.zero_ptr = L.row_keys;  // both key tables and the bucket counters start empty
    extra.zero_count = L.zero_words;
    if (n > 0 && m > 0) FNN_TRY(prep_both(batch, d1, d2, L.maps, d, opts, s, extra, true));

    DenseArgs da;
    memset(&da, 0, sizeof(da));
    da.d1 = (const char*)L.maps.p1;
    da.d1_bstride = L.maps.bstride1;
    da.d2 = (const char*)L.maps.p2;
    da.d2_bstride = L.maps.bstride2;
    da.n = (int32_t)n;
    da.m = (int32_t)m;
    da.n_sb = (int32_t)(L.maps.n_pad / (32 * DENSE_S));
    da.m_tiles = (int32_t)(L.maps.m_pad / 32);
    da.row_keys = L.row_keys;
    da.col_keys = L.col_keys;
    da.row_units = L.row_units;
    da.col_units = L.col_units;
    da.rows_cap = L.rows_cap;
    da.cols_cap = L.cols_cap;
    da.unit_counts = L.unit_counts;
    da.unit_cursor = L.unit_cursor;
    da.lists = L.lists;
    da.chunk_unit = L.chunk_unit;
    da.chunk_totals = L.chunk_totals;
    // Workgroup tile: one query super-block (32 KB of LDS keys) x up to 8 candidate groups (of
    // DENSE_WAVES x DENSE_J tiles).  Larger tiles mean fewer merges into the global key
    // tables; small problems shrink the tile until the grid covers the chip a few times.
    const int64_t groups_total = (da.m_tiles + DENSE_TILES_PER_GROUP - 1) / DENSE_TILES_PER_GROUP;
    const int64_t sb_per_wg = 1;
    int64_t groups_per_wg = 8;
    auto wg_count = [&]() {
        return ((da.n_sb + sb_per_wg - 1) / sb_per_wg) * ((groups_total + groups_per_wg - 1) / groups_per_wg) * batch;
    };
    while (groups_per_wg > 1 && wg_count() < 1024) groups_per_wg >>= 1;
    da.sb_per_wg = (int32_t)sb_per_wg;
    da.groups_per_wg = (int32_t)groups_per_wg;
    if (n > 0 && m > 0) FNN_TRY(launch_dense(da, batch, opts->compute, L.maps.dp, nn12, s12, nn21, s21, s));
    else if (n > 0) FNN_TRY(launch_fill_i32f32(nn12, s12, (int64_t)batch * n, s));
    else if (m > 0) FNN_TRY(launch_fill_i32f32(nn21, s21, (int64_t)batch * m, s));

    DenseFinalArgs fa;
    fa.n = (int32_t)n;
    fa.m = (int32_t)m;
    fa.nn12 = nn12;
    fa.nn21 = nn21;
    fa.pairs = pairs;
    fa.n_pairs = n_pairs;
    fa.block_counts = L.block_counts;
    FNN_TRY(launch_dense_final(fa, batch, s));
    if (n == 0 && m == 0) {
        // no kernel ran: n_pairs still has to be defined
        FNN_TRY(launch_recip_dedup(RecipState{}, 0, batch, nullptr, nullptr, nullptr, pairs, n_pairs, s));
    }
    return FNN_OK;
}

int32_t fnn_pairs_to_pixels(int32_t batch, const int32_t* pairs, const int32_t* n_pairs, int64_t max_pairs, int64_t n,
                            int32_t width1, int64_t m, int32_t width2, const float* conf1, const float* conf2,
                            float min_conf1, float min_conf2, int32_t* out_xy, int32_t* out_count, void* stream) {
    if (batch < 1 || batch > FNN_MAX_BATCH || max_pairs < 0 || max_pairs > MAX_PIXELS || n < 0 || m < 0 ||
        n > MAX_PIXELS || m > MAX_PIXELS || width1 < 1 || width2 < 1)
        return FNN_E_SHAPE;
    if (!n_pairs || !out_count) return FNN_E_NULL;
    if (max_pairs > 0 && (!pairs || !out_xy)) return FNN_E_NULL;
    PixelArgs pa;
    memset(&pa, 0, sizeof(pa));
    pa.pairs = pairs;
    pa.n_pairs = n_pairs;
    pa.max_pairs = max_pairs;
    pa.n = n;
    pa.m = m;
    pa.width1 = width1;
    pa.width2 = width2;
    pa.conf1 = conf1;
    pa.conf2 = conf2;
    pa.min_conf1 = min_conf1;
    pa.min_conf2 = min_conf2;
    pa.out_xy = out_xy;
    pa.out_count = out_count;
    FNN_TRY(launch_pairs_to_pixels(pa, batch, (hipStream_t)stream));
    return FNN_OK;
}

}  // extern "C"
#pragma GCC visibility pop
