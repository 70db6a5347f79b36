// Exact softmax attention (paper Equation 1 and its gradients) for head dimension 256.
//
// The kernels for d = 64 and 128 keep a whole head row of accumulators, operands and a software
// pipeline in the registers of one wave; at d = 256 that does not fit.  These kernels trade the
// pipeline for simplicity: one wave per SIMD (up to 512 registers), every head row handled as two
// 128-channel halves (so the LDS tiles, their swizzle and the direct-to-LDS loader are the d = 128
// ones), operand reads left to the compiler (ordinary LDS loads and the transposing-read builtin, no
// hand-placed waits), double-buffered 32-token tiles with one barrier per tile.  Same mathematics,
// same data layout, same MFMA operand conventions as attn_fwd.hip / attn_bwd.hip:
//   forward   lane = query:  S^T = K Q^T,  O^T += V^T P^T
//   dK, dV    lane = key:    S = Q K^T, dP = dO V^T,  dV^T += dO^T P,  dK^T += Q^T dS
//   dQ        lane = query:  S^T = K Q^T, dP^T = V dO^T,  dQ^T += K^T dS^T
#include "attn_common.h"
#include "internal.h"

namespace uly {
namespace ULY_ELEM_NS {

namespace d256 {

constexpr int kHalfD = 128;                  // channels per LDS tile
constexpr int kRows = 32;                    // tokens per streamed tile
constexpr int kHT = kRows * kHalfD;          // elements of one half tile (8 KiB)
constexpr int kBuf = 4 * kHT;                // one buffer: two halves of each of two tensors
constexpr int kThreads = 256;                // 4 waves, one per SIMD
constexpr int kOwn = 128;                    // tokens owned by a workgroup (32 per wave)
constexpr int NT = 16;                       // 16-channel contraction steps over d = 256
constexpr int NCB = 8;                       // 32-channel blocks of d = 256
using Loader = DirectTile<kHalfD, kRows, 4, SwzBoth>;
typedef short s16x4 __attribute__((ext_vector_type(4)));

// 16-byte chunk `chunk` of row `row` of a half tile: an A operand row (lane = row, 8 contraction values)
__device__ __forceinline__ e16x8 row_read(const e16* tile, int row, int chunk) {
    return *reinterpret_cast<const e16x8*>(tile + tile_off<kHalfD>(row, chunk));
}
// A operand "32 channels of block cb x rows 16u .. 16u+15", the rows in the order in which a C/D block
// holds them in registers (so that a B operand packed straight from C registers matches)
__device__ __forceinline__ e16x8 tr_read(const e16* tile, int u, int cb, int lane) {
    const int g = lane >> 5, i = lane & 15, h = (lane >> 4) & 1;
    const int row = 16 * u + 4 * g + (i >> 2), chunk = 4 * cb + 2 * h + ((i & 3) >> 1);
    const e16* p0 = tile + tile_off<kHalfD>(row, chunk) + 4 * (i & 1);
    const e16* p1 = tile + tile_off<kHalfD>(row + 8, chunk) + 4 * (i & 1);
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(ULY_LDS(s16x4, const_cast<e16*>(p0)));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(ULY_LDS(s16x4, const_cast<e16*>(p1)));
    return __builtin_shufflevector(__builtin_bit_cast(e16x4, lo), __builtin_bit_cast(e16x4, hi), 0, 1, 2, 3, 4, 5, 6, 7);
}

// Loads rows r0 .. r0+31 of two [tokens, 256] tensors (head bases a, b) as four half tiles of buffer `buf`:
// a channels 0-127, a channels 128-255, b channels 0-127, b channels 128-255.  Rows past n_rows re-read the
// last row (callers mask them).
__device__ __forceinline__ void load_tiles(e16* buf, const e16* a, const e16* b, int64_t row_stride, int r0,
                                           int n_rows, const Loader::LaneOffsets& lo, int wave, int lane) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        if (r0 + kRows <= n_rows) {
            Loader::issue(buf + h * kHT, a + (int64_t)r0 * row_stride + h * kHalfD, lo, wave);
            Loader::issue(buf + (2 + h) * kHT, b + (int64_t)r0 * row_stride + h * kHalfD, lo, wave);
        } else {
            Loader::issue_clamped(buf + h * kHT, a + h * kHalfD, row_stride, r0, n_rows, wave, lane);
            Loader::issue_clamped(buf + (2 + h) * kHT, b + h * kHalfD, row_stride, r0, n_rows, wave, lane);
        }
    }
}

__device__ __forceinline__ void zero(f32x16& x) {
#pragma unroll
    for (int r = 0; r < 16; ++r) x[r] = 0.f;
}

// ------------------------------------------------------------------------------------------
// Forward: a workgroup owns 128 queries of one head (lane = query), key tiles of 32.
// ------------------------------------------------------------------------------------------
template <bool CAUSAL>
__global__ __launch_bounds__(kThreads, 2) void attn_fwd256_kernel(
    const e16* __restrict__ Q, const e16* __restrict__ K, const e16* __restrict__ V, e16* __restrict__ O,
    float* __restrict__ LSE, int N, int Nk, int n_qtiles, int64_t row_stride, int64_t head_stride,
    int64_t kv_head_stride, float scale) {
    __shared__ __attribute__((aligned(1024))) e16 smem[2 * kBuf];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, ln = lane & 31;
    const int head = blockIdx.x / n_qtiles;
    const int qt = n_qtiles - 1 - (blockIdx.x - head * n_qtiles);      // causal: the longest tiles start first
    const int64_t hoff = (int64_t)head * head_stride;
    const e16* Kh = K + (int64_t)head * kv_head_stride;
    const e16* Vh = V + (int64_t)head * kv_head_stride;
    const int q0 = qt * kOwn, q_row = q0 + wave * 32 + ln, q_ld = q_row < N ? q_row : N - 1;
    e16x8 qreg[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
        qreg[t] = *reinterpret_cast<const e16x8*>(Q + hoff + (int64_t)q_ld * row_stride + 16 * t + 8 * g);
    int k_end = Nk;
    if (CAUSAL) { const int lim = q0 + kOwn; k_end = lim < Nk ? lim : Nk; }
    const int n_kb = (k_end + kRows - 1) / kRows;
    const int jmax = CAUSAL ? (q_row < Nk - 1 ? q_row : Nk - 1) : Nk - 1;      // last key this query sees
    const Loader::LaneOffsets lo = Loader::lane_offsets(row_stride, wave, lane);
    const float sl2 = scale * kLog2e;

    float m_used = -INFINITY, l_run = 0.f;
    f32x16 oacc[NCB];
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) zero(oacc[cb]);

    load_tiles(smem, Kh, Vh, row_stride, 0, Nk, lo, wave, lane);
#pragma unroll 1
    for (int kb = 0; kb < n_kb; ++kb) {
        wait_direct_loads();
        __syncthreads();          // tile kb has landed for every wave; every wave is done with the other buffer
        if (kb + 1 < n_kb) load_tiles(smem + ((kb + 1) & 1) * kBuf, Kh, Vh, row_stride, (kb + 1) * kRows, Nk, lo, wave, lane);
        const e16* buf = smem + (kb & 1) * kBuf;
        f32x16 s;
        zero(s);
#pragma unroll
        for (int t = 0; t < NT; ++t) s = mfma32(row_read(buf + (t >> 3) * kHT, ln, 2 * (t & 7) + g), qreg[t], s);
        // key kb*32 + c_r + 4g (c_r = 8*(r/4) + r%4) is visible iff it is <= jmax
        const int lim = jmax - kb * kRows - 4 * g;
#pragma unroll
        for (int r = 0; r < 16; ++r)
            if (8 * (r >> 2) + (r & 3) > lim) s[r] = -INFINITY;
        float m_blk = s[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) m_blk = fmaxf(m_blk, s[r]);
        m_blk = xhalf_max(m_blk);
        if (__builtin_amdgcn_ballot_w64(m_blk > m_used) != 0) {
            const float m_new = fmaxf(m_used, m_blk);
            const float m_fin = (m_new == -INFINITY) ? 0.f : m_new;     // a row with nothing visible yet
            const float alpha = fast_exp2((m_used - m_fin) * sl2);
            l_run *= alpha;
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[cb][r] *= alpha;
            m_used = m_new;
        }
        const float ms = (m_used == -INFINITY ? 0.f : m_used) * sl2;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            s[r] = fast_exp2(__builtin_fmaf(s[r], sl2, -ms));
            l_run += s[r];
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const e16x8 pb = pack_b_operand(s, u);
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb)
                oacc[cb] = mfma32(tr_read(buf + (2 + (cb >> 2)) * kHT, u, cb & 3, lane), pb, oacc[cb]);
        }
    }
    const float l_tot = xhalf_sum(l_run);
    const float inv = 1.f / l_tot;
    if (q_row < N) {
        e16* orow = O + hoff + (int64_t)q_row * row_stride;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                e16x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = (e16)(oacc[cb][4 * rq + e] * inv);
                *reinterpret_cast<e16x4*>(orow + 32 * cb + 8 * rq + 4 * g) = w;
            }
        if (g == 0) LSE[(int64_t)head * N + q_row] = m_used * scale + __logf(l_tot);
    }
}

// ------------------------------------------------------------------------------------------
// dK, dV: a workgroup owns 128 keys of one head (lane = key), query tiles of 32.
// ------------------------------------------------------------------------------------------
template <bool CAUSAL>
__global__ __launch_bounds__(kThreads, 1) void attn_bwd256_dkv_kernel(
    const e16* __restrict__ Q, const e16* __restrict__ K, const e16* __restrict__ V, const e16* __restrict__ dO,
    const float* __restrict__ LSE2, const float* __restrict__ DELTA, int64_t ws_stride, e16* __restrict__ dK,
    e16* __restrict__ dV, int N, int Nk, int n_ktiles, int64_t row_stride, int64_t head_stride,
    int64_t kv_head_stride, float scale) {
    __shared__ __attribute__((aligned(1024))) e16 smem[2 * kBuf];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, ln = lane & 31;
    const int head = blockIdx.x / n_ktiles;
    const int kt = blockIdx.x - head * n_ktiles;                      // causal: the first key tiles are the longest
    const e16* Qh = Q + (int64_t)head * head_stride;
    const e16* dOh = dO + (int64_t)head * head_stride;
    const int64_t kv_hoff = (int64_t)head * kv_head_stride;
    const float* lse_h = LSE2 + (int64_t)head * ws_stride;
    const float* del_h = DELTA + (int64_t)head * ws_stride;
    const int j0 = kt * kOwn, j_col = j0 + wave * 32 + ln, j_ld = j_col < Nk ? j_col : Nk - 1;
    e16x8 kreg[NT], vreg[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        kreg[t] = *reinterpret_cast<const e16x8*>(K + kv_hoff + (int64_t)j_ld * row_stride + 16 * t + 8 * g);
        vreg[t] = *reinterpret_cast<const e16x8*>(V + kv_hoff + (int64_t)j_ld * row_stride + 16 * t + 8 * g);
    }
    const int nblk = (N + kRows - 1) / kRows;
    const int b0 = CAUSAL ? j0 / kRows : 0;                          // first query block that sees a key of this tile
    const Loader::LaneOffsets lo = Loader::lane_offsets(row_stride, wave, lane);
    const float sl2 = scale * kLog2e;
    f32x16 dk_acc[NCB], dv_acc[NCB];
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) { zero(dk_acc[cb]); zero(dv_acc[cb]); }

    if (b0 < nblk) load_tiles(smem, Qh, dOh, row_stride, b0 * kRows, N, lo, wave, lane);
#pragma unroll 1
    for (int b = b0; b < nblk; ++b) {
        wait_direct_loads();
        __syncthreads();
        if (b + 1 < nblk) load_tiles(smem + ((b - b0 + 1) & 1) * kBuf, Qh, dOh, row_stride, (b + 1) * kRows, N, lo, wave, lane);
        const e16* buf = smem + ((b - b0) & 1) * kBuf;
        const int i0 = b * kRows;
        // statistics of rows i0 + 8q + 4g .. +3 (padded arrays: rows >= N hold lse2 = +inf, delta = 0)
        f32x4 lse4[4], del4[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            lse4[q] = *reinterpret_cast<const f32x4*>(lse_h + i0 + 8 * q + 4 * g);
            del4[q] = *reinterpret_cast<const f32x4*>(del_h + i0 + 8 * q + 4 * g);
        }
        f32x16 s, dp;
        zero(s);
        zero(dp);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            s = mfma32(row_read(buf + (t >> 3) * kHT, ln, 2 * (t & 7) + g), kreg[t], s);
            dp = mfma32(row_read(buf + (2 + (t >> 3)) * kHT, ln, 2 * (t & 7) + g), vreg[t], dp);
        }
        __builtin_amdgcn_sched_barrier(0);            // (phase boundaries keep the live ranges of the operand reads short)
        e16x8 pb[2], dsb[2];
        const int jrel = j_col - 4 * g - i0;          // causal: row offset c_r is masked iff c_r < jrel
        auto softmax_half = [&](int u) __attribute__((always_inline)) {      // P and dS of C rows 8u .. 8u+7
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int r = 8 * u + e;
                float x = __builtin_fmaf(s[r], sl2, -lse4[r >> 2][r & 3]);
                if (CAUSAL) x = (8 * (r >> 2) + (r & 3) < jrel) ? -INFINITY : x;
                const float p = fast_exp2(x);
                pb[u][e] = (e16)p;
                dsb[u][e] = (e16)(p * (dp[r] - del4[r >> 2][r & 3]));
            }
        };
        softmax_half(0);
        __builtin_amdgcn_sched_barrier(0);
        // the matrix products of the first half, with the vector work of the second half between them
        softmax_half(1);
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
            dv_acc[cb] = mfma32(tr_read(buf + (2 + (cb >> 2)) * kHT, 0, cb & 3, lane), pb[0], dv_acc[cb]);
            dk_acc[cb] = mfma32(tr_read(buf + (cb >> 2) * kHT, 0, cb & 3, lane), dsb[0], dk_acc[cb]);
        }
#pragma unroll
        for (int i = 0; i < 2 * NCB; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);    // the two transposing reads of an operand
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);    // MFMA
            __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);    // VALU
            __builtin_amdgcn_sched_group_barrier(0x400, 1, 0);    // transcendental
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
            dv_acc[cb] = mfma32(tr_read(buf + (2 + (cb >> 2)) * kHT, 1, cb & 3, lane), pb[1], dv_acc[cb]);
            dk_acc[cb] = mfma32(tr_read(buf + (cb >> 2) * kHT, 1, cb & 3, lane), dsb[1], dk_acc[cb]);
            if ((cb & 1) == 1) __builtin_amdgcn_sched_barrier(0);
        }
    }
    if (j_col < Nk) {
        e16* krow = dK + kv_hoff + (int64_t)j_col * row_stride;
        e16* vrow = dV + kv_hoff + (int64_t)j_col * row_stride;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                e16x4 wk, wv;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    wk[e] = (e16)(dk_acc[cb][4 * rq + e] * scale);
                    wv[e] = (e16)dv_acc[cb][4 * rq + e];
                }
                *reinterpret_cast<e16x4*>(krow + 32 * cb + 8 * rq + 4 * g) = wk;
                *reinterpret_cast<e16x4*>(vrow + 32 * cb + 8 * rq + 4 * g) = wv;
            }
    }
}

// ------------------------------------------------------------------------------------------
// dQ: a workgroup owns 128 queries of one head (lane = query), key tiles of 32.
// ------------------------------------------------------------------------------------------
template <bool CAUSAL>
__global__ __launch_bounds__(kThreads, 1) void attn_bwd256_dq_kernel(
    const e16* __restrict__ Q, const e16* __restrict__ K, const e16* __restrict__ V, const e16* __restrict__ dO,
    const float* __restrict__ LSE2, const float* __restrict__ DELTA, int64_t ws_stride, e16* __restrict__ dQ, int N,
    int Nk, int n_qtiles, int64_t row_stride, int64_t head_stride, int64_t kv_head_stride, float scale) {
    __shared__ __attribute__((aligned(1024))) e16 smem[2 * kBuf];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, ln = lane & 31;
    const int head = blockIdx.x / n_qtiles;
    const int qt = n_qtiles - 1 - (blockIdx.x - head * n_qtiles);
    const int64_t hoff = (int64_t)head * head_stride;
    const e16* Kh = K + (int64_t)head * kv_head_stride;
    const e16* Vh = V + (int64_t)head * kv_head_stride;
    const int q0 = qt * kOwn, q_row = q0 + wave * 32 + ln, q_ld = q_row < N ? q_row : N - 1;
    e16x8 qreg[NT], doreg[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        qreg[t] = *reinterpret_cast<const e16x8*>(Q + hoff + (int64_t)q_ld * row_stride + 16 * t + 8 * g);
        doreg[t] = *reinterpret_cast<const e16x8*>(dO + hoff + (int64_t)q_ld * row_stride + 16 * t + 8 * g);
    }
    const float lse2 = LSE2[(int64_t)head * ws_stride + q_row];      // padded: +inf for q_row >= N
    const float delta = DELTA[(int64_t)head * ws_stride + q_row];
    int k_end = Nk;
    if (CAUSAL) { const int lim = q0 + kOwn; k_end = lim < Nk ? lim : Nk; }
    const int n_kb = (k_end + kRows - 1) / kRows;
    const int klim = (CAUSAL ? (q_row < Nk - 1 ? q_row : Nk - 1) : Nk - 1) - 4 * g;
    const Loader::LaneOffsets lo = Loader::lane_offsets(row_stride, wave, lane);
    const float sl2 = scale * kLog2e;
    f32x16 acc[NCB];
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) zero(acc[cb]);

    load_tiles(smem, Kh, Vh, row_stride, 0, Nk, lo, wave, lane);
#pragma unroll 1
    for (int kb = 0; kb < n_kb; ++kb) {
        wait_direct_loads();
        __syncthreads();
        if (kb + 1 < n_kb) load_tiles(smem + ((kb + 1) & 1) * kBuf, Kh, Vh, row_stride, (kb + 1) * kRows, Nk, lo, wave, lane);
        const e16* buf = smem + (kb & 1) * kBuf;
        f32x16 s, dp;
        zero(s);
        zero(dp);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            s = mfma32(row_read(buf + (t >> 3) * kHT, ln, 2 * (t & 7) + g), qreg[t], s);
            dp = mfma32(row_read(buf + (2 + (t >> 3)) * kHT, ln, 2 * (t & 7) + g), doreg[t], dp);
        }
        __builtin_amdgcn_sched_barrier(0);
        e16x8 dsb[2];
        const int krel = klim - kb * kRows;           // key offset c_r is masked iff c_r > krel
        auto softmax_half = [&](int u) __attribute__((always_inline)) {      // dS^T of C rows 8u .. 8u+7
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int r = 8 * u + e;
                float x = __builtin_fmaf(s[r], sl2, -lse2);
                x = (8 * (r >> 2) + (r & 3) > krel) ? -INFINITY : x;
                const float p = fast_exp2(x);
                dsb[u][e] = (e16)(p * (dp[r] - delta));
            }
        };
        softmax_half(0);
        __builtin_amdgcn_sched_barrier(0);
        // the matrix products of the first half, with the vector work of the second half between them
        softmax_half(1);
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) acc[cb] = mfma32(tr_read(buf + (cb >> 2) * kHT, 0, cb & 3, lane), dsb[0], acc[cb]);
#pragma unroll
        for (int i = 0; i < NCB; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);    // the two transposing reads of an operand
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);    // MFMA
            __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);    // VALU
            __builtin_amdgcn_sched_group_barrier(0x400, 1, 0);    // transcendental
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) acc[cb] = mfma32(tr_read(buf + (cb >> 2) * kHT, 1, cb & 3, lane), dsb[1], acc[cb]);
    }
    if (q_row < N) {
        e16* orow = dQ + hoff + (int64_t)q_row * row_stride;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                e16x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = (e16)(acc[cb][4 * rq + e] * scale);
                *reinterpret_cast<e16x4*>(orow + 32 * cb + 8 * rq + 4 * g) = w;
            }
    }
}

}  // namespace d256

int attn256_fwd_launch(const void* q, const void* k, const void* v, void* o, float* lse, int64_t N, int64_t Nk, int Hl,
                       float scale, int causal, TensorStrides st, TensorStrides kv, void* stream) {
    const int64_t n_qtiles = (N + d256::kOwn - 1) / d256::kOwn;
    if (n_qtiles * Hl > 0x7FFFFFFFll) return ULY_ERR_SHAPE;
    const dim3 grid((uint32_t)(n_qtiles * Hl)), block(d256::kThreads);
    hipStream_t s = (hipStream_t)stream;
    if (causal)
        d256::attn_fwd256_kernel<true><<<grid, block, 0, s>>>((const e16*)q, (const e16*)k, (const e16*)v, (e16*)o, lse,
                                                               (int)N, (int)Nk, (int)n_qtiles, st.row, st.head, kv.head, scale);
    else
        d256::attn_fwd256_kernel<false><<<grid, block, 0, s>>>((const e16*)q, (const e16*)k, (const e16*)v, (e16*)o, lse,
                                                                (int)N, (int)Nk, (int)n_qtiles, st.row, st.head, kv.head, scale);
    return hipGetLastError() == hipSuccess ? ULY_OK : ULY_ERR_LAUNCH;
}

// The dK/dV (stage bit 1) and dQ (stage bit 2) kernels; the statistics in `delta`, `lse2` (padded rows of
// `stride` floats per head) come from the delta kernel the caller has run.
int attn256_bwd_launch(int stage_mask, const void* q, const void* k, const void* v, const void* dout, const float* delta,
                       const float* lse2, int64_t stride, void* dq, void* dk, void* dv, int64_t N, int64_t Nk, int Hl,
                       float scale, int causal, TensorStrides st, TensorStrides kv, void* stream) {
    const int64_t n_qtiles = (N + d256::kOwn - 1) / d256::kOwn, n_ktiles = (Nk + d256::kOwn - 1) / d256::kOwn;
    if (n_qtiles * Hl > 0x7FFFFFFFll || n_ktiles * Hl > 0x7FFFFFFFll) return ULY_ERR_SHAPE;
    const e16 *Q = (const e16*)q, *K = (const e16*)k, *V = (const e16*)v, *dO = (const e16*)dout;
    const dim3 gkv((uint32_t)(n_ktiles * Hl)), gq((uint32_t)(n_qtiles * Hl)), block(d256::kThreads);
    hipStream_t s = (hipStream_t)stream;
    if (stage_mask & 2) {
        if (causal)
            d256::attn_bwd256_dkv_kernel<true><<<gkv, block, 0, s>>>(Q, K, V, dO, lse2, delta, stride, (e16*)dk, (e16*)dv,
                                                                     (int)N, (int)Nk, (int)n_ktiles, st.row, st.head, kv.head, scale);
        else
            d256::attn_bwd256_dkv_kernel<false><<<gkv, block, 0, s>>>(Q, K, V, dO, lse2, delta, stride, (e16*)dk, (e16*)dv,
                                                                      (int)N, (int)Nk, (int)n_ktiles, st.row, st.head, kv.head, scale);
        if (hipGetLastError() != hipSuccess) return ULY_ERR_LAUNCH;
    }
    if (stage_mask & 4) {
        if (causal)
            d256::attn_bwd256_dq_kernel<true><<<gq, block, 0, s>>>(Q, K, V, dO, lse2, delta, stride, (e16*)dq, (int)N, (int)Nk,
                                                                   (int)n_qtiles, st.row, st.head, kv.head, scale);
        else
            d256::attn_bwd256_dq_kernel<false><<<gq, block, 0, s>>>(Q, K, V, dO, lse2, delta, stride, (e16*)dq, (int)N, (int)Nk,
                                                                    (int)n_qtiles, st.row, st.head, kv.head, scale);
        if (hipGetLastError() != hipSuccess) return ULY_ERR_LAUNCH;
    }
    return ULY_OK;
}

}  // namespace ULY_ELEM_NS
}  // namespace uly
