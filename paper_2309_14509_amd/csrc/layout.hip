// Layout transforms around the two all-to-alls of a sequence-parallel attention layer
// (paper Section 3.1): pure, bit-exact data movement, bound by HBM bandwidth.
//
// All four transforms (and both output layouts) are one regrouping
//     A[n][p][w]  <->  B[p][n][w]        n < rows,  p < groups,  w < run
// where a "run" is the contiguous block that moves as a unit (Hl*d elements for the
// rank-regrouping, d elements for the head-major layout).  A run is 256 B - 1.8 KB for the
// shapes of interest, so 16-byte lanes are coalesced on both the read and the write side
// without staging through LDS: a wavefront covers 1 KiB, i.e. whole runs or large pieces of one.
// A workgroup is one wavefront: it reads 1 KiB of consecutive A elements and writes them to one
// or a few runs of B.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "internal.h"

namespace uly {

// Exact n / d for n < 2^31 with one 32x32->64 multiply and a shift.
struct FastDiv {
    uint32_t mul, shift;
};

static FastDiv make_fastdiv(uint32_t d) {
    uint32_t L = 0;
    while ((1ull << L) < d) ++L;
    FastDiv f;
    f.shift = 31 + L;
    f.mul = (uint32_t)(((1ull << f.shift) / d) + 1);
    return f;
}

__device__ __forceinline__ uint32_t fastdiv(uint32_t n, FastDiv f) {
    return (uint32_t)(((uint64_t)n * f.mul) >> f.shift);
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// One wavefront per workgroup, one element per lane: measured on MI355X, HBM streams best with very
// many tiny workgroups in flight (6.1 TB/s here against 4.3 TB/s with 256 lanes x 8 elements and
// 5.8 TB/s with 512 lanes x 1), more than with several loads in flight per lane.
constexpr int kThreads = 64;
constexpr int kTileVecs = 1 << 16;   // index arithmetic is 32-bit inside a tile of whole rows of about this size

// Up to kMaxTensors tensors of one shape per launch (blockIdx.y selects the tensor).
struct TensorPtrs {
    const void* src[kMaxTensors];
    void* dst[kMaxTensors];
};

// TO_B = true : dst(B) <- src(A)      TO_B = false : dst(A) <- src(B)
// Workgroup blockIdx.x handles 64 consecutive vectors (slice `s`) of row tile `t` of A:
// blockIdx.x = t * slices + s.
template <typename Vec, bool TO_B>
__global__ __launch_bounds__(kThreads) void regroup_kernel(TensorPtrs ptrs, int64_t rows, uint32_t row_vecs,
                                                           uint32_t run_vecs, FastDiv div_row, FastDiv div_run,
                                                           uint32_t tile_rows, uint32_t slices, FastDiv div_slices) {
    const Vec* __restrict__ src = static_cast<const Vec*>(ptrs.src[blockIdx.y]);
    Vec* __restrict__ dst = static_cast<Vec*>(ptrs.dst[blockIdx.y]);
    const uint32_t tile = fastdiv(blockIdx.x, div_slices);
    const uint32_t slice = blockIdx.x - tile * slices;
    const int64_t n0 = (int64_t)tile * tile_rows;
    const int64_t rem = rows - n0;
    const uint32_t my_rows = rem < (int64_t)tile_rows ? (uint32_t)rem : tile_rows;
    const uint32_t f = slice * kThreads + threadIdx.x;          // vector index inside the tile
    if (f >= my_rows * row_vecs) return;
    const uint32_t r = fastdiv(f, div_row);
    const uint32_t w = f - r * row_vecs;
    const uint32_t p = fastdiv(w, div_run);
    const uint32_t ww = w - p * run_vecs;
    const int64_t a_idx = n0 * row_vecs + f;
    const int64_t b_idx = ((int64_t)p * rows + n0 + r) * run_vecs + ww;
    if (TO_B) __builtin_nontemporal_store(__builtin_nontemporal_load(src + a_idx), dst + b_idx);
    else __builtin_nontemporal_store(__builtin_nontemporal_load(src + b_idx), dst + a_idx);
}

template <typename Vec>
static int launch_regroup(const TensorPtrs& ptrs, int count, int64_t rows, int64_t groups, int64_t run_bytes,
                          bool to_b, hipStream_t stream) {
    const int64_t run_vecs = run_bytes / (int64_t)sizeof(Vec);
    const int64_t row_vecs = run_vecs * groups;
    if (row_vecs >= (1ll << 24)) return ULY_ERR_SHAPE;   // keeps every in-tile index far below 2^31
    const uint32_t tile_rows = (uint32_t)(row_vecs >= kTileVecs ? 1 : kTileVecs / row_vecs);
    const int64_t tiles = (rows + tile_rows - 1) / tile_rows;
    const int64_t slices = ((int64_t)tile_rows * row_vecs + kThreads - 1) / kThreads;
    const int64_t blocks = tiles * slices;
    if (blocks <= 0) return ULY_OK;
    if (blocks > 0x7FFFFFFFll) return ULY_ERR_SHAPE;
    const FastDiv div_row = make_fastdiv((uint32_t)row_vecs), div_run = make_fastdiv((uint32_t)run_vecs);
    const FastDiv div_slices = make_fastdiv((uint32_t)slices);
    const dim3 grid((uint32_t)blocks, (uint32_t)count);
    if (to_b)
        regroup_kernel<Vec, true><<<grid, dim3(kThreads), 0, stream>>>(
            ptrs, rows, (uint32_t)row_vecs, (uint32_t)run_vecs, div_row, div_run, tile_rows, (uint32_t)slices, div_slices);
    else
        regroup_kernel<Vec, false><<<grid, dim3(kThreads), 0, stream>>>(
            ptrs, rows, (uint32_t)row_vecs, (uint32_t)run_vecs, div_row, div_run, tile_rows, (uint32_t)slices, div_slices);
    return hipGetLastError() == hipSuccess ? ULY_OK : ULY_ERR_LAUNCH;
}

// ------------------------------------------------------------------------------------------
// Runs of a single 1-, 2- or 4-byte element: the regrouping is a plain 2-D transpose
// A[rows][groups] <-> B[groups][rows], and a lane of the direct kernel would move only that one
// element to a scattered address (measured: 0.9 / 1.9 TB/s at 2 / 4 bytes against 4.0 TB/s at 8 and
// 5.1 TB/s and more from 16 bytes on; staged, 2.3 / 4.3 TB/s at 2 / 4 bytes and no gain at 8).  Here a tile of tr rows x tg groups goes through LDS, so that the
// global reads follow the source order and the global writes the destination order: both sides
// touch contiguous memory.
// ------------------------------------------------------------------------------------------
constexpr int kStageThreads = 256;
constexpr int kStageElems = 4096;          // elements per tile
constexpr int kStageMaxGroups = 64;        // groups per tile

template <typename E, bool TO_B>
__global__ __launch_bounds__(kStageThreads) void regroup_staged_kernel(TensorPtrs ptrs, int64_t rows, uint32_t groups,
                                                                      uint32_t tg, uint32_t tr, FastDiv div_tg,
                                                                      FastDiv div_tr) {
    __shared__ E tile[kStageElems + kStageMaxGroups];          // [tg][tr + 1]: odd pitch spreads the banks
    const E* __restrict__ src = static_cast<const E*>(ptrs.src[blockIdx.z]);
    E* __restrict__ dst = static_cast<E*>(ptrs.dst[blockIdx.z]);
    const int64_t n0 = (int64_t)blockIdx.x * tr;
    const uint32_t p0 = blockIdx.y * tg;
    const uint32_t pitch = tr + 1;
    const uint32_t count = tg * tr;
    // element idx of the tile in A order is (row idx / tg, group idx % tg), in B order (group idx / tr, row idx % tr)
    for (uint32_t idx = threadIdx.x; idx < count; idx += kStageThreads) {
        uint32_t r, pp;
        if (TO_B) { r = fastdiv(idx, div_tg); pp = idx - r * tg; }
        else { pp = fastdiv(idx, div_tr); r = idx - pp * tr; }
        const int64_t n = n0 + r;
        const uint32_t p = p0 + pp;
        if (n < rows && p < groups) tile[pp * pitch + r] = TO_B ? src[n * groups + p] : src[(int64_t)p * rows + n];
    }
    __syncthreads();
    for (uint32_t idx = threadIdx.x; idx < count; idx += kStageThreads) {
        uint32_t r, pp;
        if (TO_B) { pp = fastdiv(idx, div_tr); r = idx - pp * tr; }
        else { r = fastdiv(idx, div_tg); pp = idx - r * tg; }
        const int64_t n = n0 + r;
        const uint32_t p = p0 + pp;
        if (n < rows && p < groups) {
            if (TO_B) dst[(int64_t)p * rows + n] = tile[pp * pitch + r];
            else dst[n * groups + p] = tile[pp * pitch + r];
        }
    }
}

template <typename E>
static int launch_staged(const TensorPtrs& ptrs, int count, int64_t rows, int64_t groups, bool to_b, hipStream_t stream) {
    if (groups >= (1ll << 31)) return ULY_ERR_SHAPE;
    const uint32_t tg = (uint32_t)(groups < kStageMaxGroups ? groups : kStageMaxGroups);
    const uint32_t tr = kStageElems / tg;
    const int64_t row_tiles = (rows + tr - 1) / tr, group_tiles = (groups + tg - 1) / tg;
    if (row_tiles > 0x7FFFFFFFll || group_tiles > 65535) return ULY_ERR_SHAPE;
    const dim3 grid((uint32_t)row_tiles, (uint32_t)group_tiles, (uint32_t)count);
    const FastDiv div_tg = make_fastdiv(tg), div_tr = make_fastdiv(tr);
    if (to_b)
        regroup_staged_kernel<E, true><<<grid, dim3(kStageThreads), 0, stream>>>(ptrs, rows, (uint32_t)groups, tg, tr,
                                                                                 div_tg, div_tr);
    else
        regroup_staged_kernel<E, false><<<grid, dim3(kStageThreads), 0, stream>>>(ptrs, rows, (uint32_t)groups, tg, tr,
                                                                                  div_tg, div_tr);
    return hipGetLastError() == hipSuccess ? ULY_OK : ULY_ERR_LAUNCH;
}

// A[rows][groups][run_bytes] <-> B[groups][rows][run_bytes] for `count` tensors of one shape in one
// launch; to_b selects the direction.
int regroup_multi(const void* const* src, void* const* dst, int count, int64_t rows, int64_t groups, int64_t run_bytes,
                  bool to_b, void* stream) {
    hipStream_t s = (hipStream_t)stream;
    if (rows == 0 || groups == 0 || run_bytes == 0 || count == 0) return ULY_OK;
    if (count < 0 || count > kMaxTensors) return ULY_ERR_SHAPE;
    TensorPtrs ptrs = {};
    for (int i = 0; i < count; ++i) { ptrs.src[i] = src[i]; ptrs.dst[i] = dst[i]; }
    if (groups > 1) {          // short runs: transpose through LDS (with one group the map is a plain copy)
        if (run_bytes == 4) return launch_staged<uint32_t>(ptrs, count, rows, groups, to_b, s);
        if (run_bytes == 2) return launch_staged<uint16_t>(ptrs, count, rows, groups, to_b, s);
        if (run_bytes == 1) return launch_staged<uint8_t>(ptrs, count, rows, groups, to_b, s);
    }
    if (run_bytes % 16 == 0) return launch_regroup<u32x4>(ptrs, count, rows, groups, run_bytes, to_b, s);
    if (run_bytes % 8 == 0) return launch_regroup<u32x2>(ptrs, count, rows, groups, run_bytes, to_b, s);
    if (run_bytes % 4 == 0) return launch_regroup<uint32_t>(ptrs, count, rows, groups, run_bytes, to_b, s);
    if (run_bytes % 2 == 0) return launch_regroup<uint16_t>(ptrs, count, rows, groups, run_bytes, to_b, s);
    return launch_regroup<uint8_t>(ptrs, count, rows, groups, run_bytes, to_b, s);
}

int regroup(const void* src, void* dst, int64_t rows, int64_t groups, int64_t run_bytes, bool to_b, void* stream) {
    return regroup_multi(&src, &dst, 1, rows, groups, run_bytes, to_b, stream);
}

}  // namespace uly
