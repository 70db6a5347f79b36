// Device-side building blocks shared by the attention kernels (gfx950 / CDNA4, wave64).
//
// MFMA operand conventions used throughout (v_mfma_f32_32x32x16_bf16, lane l, g = l / 32):
//   A (32 x 16): lane holds row  l % 32, contraction indices 8g .. 8g+7   (8 elements = one 16-byte load)
//   B (16 x 32): lane holds col  l % 32, contraction indices 8g .. 8g+7
//   C/D (32 x 32): register r of lane l is row 8*(r/4) + 4g + (r%4), column l % 32
// Every kernel keeps the "long" reduction axis of its softmax in the rows of C, so that a lane
// owns one column (one query, or one key) and row statistics need no cross-lane traffic beyond
// one exchange between lanes l and l^32.
#ifndef ULY_ATTN_COMMON_H
#define ULY_ATTN_COMMON_H

#include <hip/hip_runtime.h>
#include <stdint.h>

// Element type of Q, K, V, O and the gradients: bf16, or fp16 when the translation unit is compiled
// with ULY_BUILD_F16 (the build compiles every attention source once per type; everything in them
// lives in namespace uly::bf16 or uly::f16).  Both types use the same MFMA shape and layouts.
#if defined(ULY_BUILD_F16)
#define ULY_ELEM_NS f16
#else
#define ULY_ELEM_NS bf16
#endif

namespace uly {
namespace ULY_ELEM_NS {

#if defined(ULY_BUILD_F16)
typedef _Float16 e16;
#else
typedef __bf16 e16;
#endif
typedef e16 e16x8 __attribute__((ext_vector_type(8)));
typedef e16 e16x4 __attribute__((ext_vector_type(4)));
typedef e16 e16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

#define ULY_LDS(T, ptr) ((__attribute__((address_space(3))) T*)(ptr))

constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ f32x16 mfma32(e16x8 a, e16x8 b, f32x16 c) {
#if defined(ULY_BUILD_F16)
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
#else
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
#endif
}

// The same MFMA with its result in vector registers.  The compiler's own MFMAs of a kernel that uses more than
// 256 registers all accumulate in accumulation registers, from which every score would have to be copied before
// the vector unit can touch it; written out by hand, S (and dP) land where the softmax reads them, and the fixed
// operand comes from an accumulation register.  The compiler does not see these as MFMAs, so callers keep the
// distance the hardware needs themselves: at least eight other MFMAs (or mfma32_v_settle) between the last
// of these and the first vector instruction that reads the result; an accumulation chain on one register set
// needs nothing.
#if defined(ULY_BUILD_F16)
#define ULY_MFMA32_ASM "v_mfma_f32_32x32x16_f16"
#else
#define ULY_MFMA32_ASM "v_mfma_f32_32x32x16_bf16"
#endif
__device__ __forceinline__ void mfma32_v_first(f32x16& d, const e16x8& a, const e16x8& b) {
    asm volatile(ULY_MFMA32_ASM " %0, %1, %2, 0" : "=&v"(d) : "v"(a), "a"(b));
}
__device__ __forceinline__ void mfma32_v_acc(f32x16& d, const e16x8& a, const e16x8& b) {
    asm volatile(ULY_MFMA32_ASM " %0, %1, %2, %0" : "+v"(d) : "v"(a), "a"(b));
}
template <typename T> __device__ __forceinline__ void lds_tie1(T& r);
// Idles until MFMAs issued just before have written their results, and keeps those registers allocated until
// then.  Needed wherever such a result is read right away, and also where it is never read (the S computed for
// the block after the last one): to the compiler a register whose value is dead is free at once, and whatever it
// put there would be overwritten when the MFMA completes.
template <typename... T> __device__ __forceinline__ void mfma32_v_settle(T&... acc) {
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15");
    (lds_tie1(acc), ...);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Registers 8u..8u+7 of a C/D block, rounded to the element type: a B operand whose contraction index e
// is C-row 16u + 8*(e/4) + 4g + (e%4).
__device__ __forceinline__ e16x8 pack_b_operand(const f32x16& c, int u) {
    e16x8 r;
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = (e16)c[8 * u + e];
    return r;
}

// Exchange between lane l and lane l^32 (v_permlane32_swap): returns {own value, other half's value}
// in some order.  The instruction swaps the upper half of its first register with the lower half
// of its second, so the two operands must live in different registers: the copy is made opaque
// to the compiler to keep it from allocating both to one register.
__device__ __forceinline__ void xhalf_pair(float x, float& a, float& b) {
    int x0 = __float_as_int(x), x1 = x0;
    asm volatile("" : "+v"(x1));
    auto r = __builtin_amdgcn_permlane32_swap(x0, x1, false, false);
    const int r0 = r[0], r1 = r[1];      // (element-wise bit casts straight off the vector are mis-folded)
    a = __int_as_float(r0);
    b = __int_as_float(r1);
}
// Combine a per-lane value with the lane that holds the other half of the same column.
__device__ __forceinline__ float xhalf_max(float x) {
    float a, b;
    xhalf_pair(x, a, b);
    return fmaxf(a, b);
}
__device__ __forceinline__ float xhalf_sum(float x) {
    float a, b;
    xhalf_pair(x, a, b);
    return a + b;
}

// ------------------------------------------------------------------------------------------
// LDS tiles filled straight from global memory (global_load_lds_dwordx4: no VGPR staging).
//
// A tile is ROWS x D 16-bit elements, rows unpadded (D*2 bytes); the 16-byte chunk c of row r is stored at
// chunk position c ^ swz(r).  One wave-wide load writes 1 KiB of consecutive LDS (lane L -> byte
// 16*L), so the swizzle is applied by choosing which global chunk each lane fetches.  swz is
// chosen so that both access patterns are bank-conflict free:
//   row reads  (16 lanes = 16 consecutive rows, same logical chunk)       -> 16 distinct chunks
//   transposing reads (16 lanes = 4 consecutive rows x 2 chunks)            -> 8 distinct chunks
// It only depends on r mod 16, so tile-row offsets that are multiples of 16 are plain immediates.
// ------------------------------------------------------------------------------------------
template <int D> __device__ __forceinline__ int swz(int r);
template <> __device__ __forceinline__ int swz<128>(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }
template <> __device__ __forceinline__ int swz<64>(int r) {
    const int i = (r >> 1) & 7;
    return (i & 4) | ((i & 1) << 1) | ((i >> 1) & 1);
}
// Swizzle for tiles that are only read through transposing reads: it depends on r mod 4 (D = 128) or
// r mod 8 (D = 64) only, so rows 8 apart sit a constant distance apart and one address register
// serves both 4-row groups of a transposing operand.
template <int D> __device__ __forceinline__ int swz_tr(int r);
template <> __device__ __forceinline__ int swz_tr<128>(int r) { return (r & 3) << 2; }
template <> __device__ __forceinline__ int swz_tr<64>(int r) { return ((r >> 1) & 1) << 1; }

struct SwzBoth {
    template <int D> __device__ static __forceinline__ int f(int r) { return swz<D>(r); }
};
struct SwzTr {
    template <int D> __device__ static __forceinline__ int f(int r) { return swz_tr<D>(r); }
};

// element offset of (row r, logical chunk c) inside a swizzled tile
template <int D, typename S = SwzBoth> __device__ __forceinline__ int tile_off(int r, int c) {
    return r * D + ((c ^ S::template f<D>(r)) << 3);
}

template <int D, int ROWS, int WAVES, typename S = SwzBoth> struct DirectTile {
    static constexpr int kChunksPerRow = D / 8;
    static constexpr int kRowsPerSlab = 64 / kChunksPerRow;          // rows written by one wave-wide load
    static constexpr int kSlabs = ROWS / kRowsPerSlab;
    static constexpr int kPerWave = kSlabs / WAVES;
    static_assert(kSlabs % WAVES == 0, "tile must divide evenly over the waves");

    // Per-lane byte offset (from the first row of a tile) of the chunk this lane fetches in its first
    // load; the wave's further loads are WAVES*kRowsPerSlab rows (a multiple of 16, so the same
    // swizzle) further down, a uniform step.  Neither changes from tile to tile.
    struct LaneOffsets {
        uint32_t off0;
        int64_t step_bytes;
    };
    static_assert((WAVES * kRowsPerSlab) % 16 == 0, "loads of one wave must share their swizzle");
    __device__ static __forceinline__ LaneOffsets lane_offsets(int64_t row_stride, int wave, int lane) {
        LaneOffsets lo;
        const int lr = lane / kChunksPerRow, pc = lane % kChunksPerRow;
        const int r = wave * kRowsPerSlab + lr;                      // row inside the tile
        lo.off0 = (uint32_t)(r * row_stride * 2) + (uint32_t)(((pc ^ S::template f<D>(r)) << 4));
        lo.step_bytes = (int64_t)WAVES * kRowsPerSlab * row_stride * 2;
        return lo;
    }
    // Issue this wave's loads of a full tile whose first row is at `tile_base` (all rows valid).
    __device__ static __forceinline__ void issue(e16* tile, const e16* tile_base, const LaneOffsets& lo, int wave) {
#pragma unroll
        for (int i = 0; i < kPerWave; ++i) {
            const char* src = reinterpret_cast<const char*>(tile_base) + i * lo.step_bytes + lo.off0;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                             ULY_LDS(void, tile + (wave + i * WAVES) * kRowsPerSlab * D), 16, 0, 0);
        }
    }
    // Branch-free variant for loops that must stay one basic block.  `tail` holds this lane's offsets
    // for the one tile that runs past the end of the tensor (rows clamped to the last valid row; the
    // callers mask them out); `is_tail` is uniform.
    struct TailOffsets {
        uint32_t off[kPerWave];
    };
    __device__ static __forceinline__ TailOffsets tail_offsets(int64_t row_stride, int wave, int lane, int n_rows) {
        TailOffsets to;
        const int tail_r0 = (n_rows / ROWS) * ROWS;                  // first row of the ragged tile
        const int lr = lane / kChunksPerRow, pc = lane % kChunksPerRow;
#pragma unroll
        for (int i = 0; i < kPerWave; ++i) {
            const int r = (wave + i * WAVES) * kRowsPerSlab + lr;
            int gr = tail_r0 + r;
            gr = gr < n_rows ? gr : n_rows - 1;
            to.off[i] = (uint32_t)((gr - tail_r0) * row_stride * 2) + (uint32_t)(((pc ^ S::template f<D>(r)) << 4));
        }
        return to;
    }
    __device__ static __forceinline__ void issue_sel(e16* tile, const e16* tile_base, const LaneOffsets& lo,
                                                     const TailOffsets& to, bool is_tail, int wave) {
#pragma unroll
        for (int i = 0; i < kPerWave; ++i) {
            const uint32_t voff = is_tail ? to.off[i] : lo.off0;
            const int64_t soff = is_tail ? 0 : i * lo.step_bytes;
            const char* src = reinterpret_cast<const char*>(tile_base) + soff + voff;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                             ULY_LDS(void, tile + (wave + i * WAVES) * kRowsPerSlab * D), 16, 0, 0);
        }
    }
    // Same for a tile that may run past the end of the tensor: rows at or beyond n_rows are clamped
    // to the last valid row (callers mask them out).
    __device__ static __forceinline__ void issue_clamped(e16* tile, const e16* base, int64_t row_stride, int row0,
                                                         int n_rows, int wave, int lane) {
        // This path runs at most once per workgroup.  The lane id is made opaque here so that none of
        // its address arithmetic is hoisted out of the caller's loop (where it would pin ~30 VGPRs).
        asm volatile("" : "+v"(lane));
        const int lr = lane / kChunksPerRow, pc = lane % kChunksPerRow;
#pragma unroll
        for (int i = 0; i < kPerWave; ++i) {
            const int slab = wave + i * WAVES;
            const int r = slab * kRowsPerSlab + lr;
            int gr = row0 + r;
            gr = gr < n_rows ? gr : n_rows - 1;
            const e16* src = base + (int64_t)gr * row_stride + ((pc ^ S::template f<D>(r)) << 3);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                             ULY_LDS(void, tile + slab * kRowsPerSlab * D), 16, 0, 0);
        }
    }
};

// ------------------------------------------------------------------------------------------
// Hand-placed LDS reads.  The hot loops issue their operand reads a full phase before the MFMAs that
// consume them; the reads are inline asm (per-lane byte address + immediate) so that their position
// in the instruction stream is fixed and each address costs no VALU work.  The compiler does not
// count these in lgkmcnt, so every consumer is preceded by lds_wait<N>(regs...), which both waits
// and ties the registers to the wait (nothing that uses them can be scheduled above it).
// ------------------------------------------------------------------------------------------
template <int IMM> __device__ __forceinline__ e16x8 lds_b128(uint32_t addr) {
    e16x8 r;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(IMM));
    return r;
}
template <int IMM> __device__ __forceinline__ e16x4 lds_tr_b64(uint32_t addr) {
    e16x4 r;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(IMM));
    return r;
}
template <int N> __device__ __forceinline__ void lds_wait(e16x8& a, e16x8& b, e16x8& c, e16x8& d) {
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(N));
}
template <int N> __device__ __forceinline__ void lds_wait(e16x4& a, e16x4& b, e16x4& c, e16x4& d) {
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(N));
}
template <int N> __device__ __forceinline__ void lds_wait(e16x8& a, e16x8& b) {
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N));
}
template <int N> __device__ __forceinline__ void lds_wait(e16x4& a, e16x4& b) {
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N));
}
// Generic form: wait_lgkm<N>() followed by lds_tie(regs...) orders every later use of `regs` behind
// the wait (volatile asm statements keep their order; the empty asm redefines the registers).
template <int N> __device__ __forceinline__ void wait_lgkm() { asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N)); }
template <int N> __device__ __forceinline__ void wait_vm() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }
template <typename T> __device__ __forceinline__ void lds_tie1(T& r) { asm volatile("" : "+v"(r)); }
template <typename... T> __device__ __forceinline__ void lds_tie(T&... r) { (lds_tie1(r), ...); }
template <int IMM> __device__ __forceinline__ f32x4 lds_f32x4(uint32_t addr) {
    f32x4 r;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(IMM));
    return r;
}
// byte address of an LDS object as the hardware sees it
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return (uint32_t)(uintptr_t)ULY_LDS(const char, p);
}

// Workgroup barrier that implies no memory waits.  (__syncthreads() makes the compiler drain every
// outstanding load first, which would collapse a ring of tiles in flight to a single one; callers of
// this one wait for exactly the loads and LDS reads they depend on.)
__device__ __forceinline__ void barrier_no_drain() { asm volatile("s_barrier" ::: "memory"); }
// Wait until every direct-to-LDS load this wave has issued has landed.
__device__ __forceinline__ void wait_direct_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

}  // namespace ULY_ELEM_NS
}  // namespace uly
#endif
