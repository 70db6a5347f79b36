// Backward pass of exact softmax attention (gradients of paper Equation 1; the probabilities are
// recomputed from Q, K and the saved log-sum-exp instead of being stored).
//
//   D_i   = sum_c dO_ic O_ic                                  (delta kernel)
//   P_ij  = exp(scale * Q_i.K_j - LSE_i)   dP_ij = dO_i.V_j   dS_ij = P_ij (dP_ij - D_i)
//   dQ_i  = scale * sum_j dS_ij K_j                            (dq kernel: one workgroup per query tile)
//   dK_j  = scale * sum_i dS_ij Q_i,  dV_j = sum_i P_ij dO_i   (dkv kernel: one workgroup per key tile)
//
// Two kernels instead of one with atomics: each output element is owned by exactly one lane, so
// the result is deterministic and needs no fp32 dQ buffer, at the price of recomputing S and dP.
#include "attn_common.h"
#include "internal.h"

namespace uly {

constexpr int kBwdThreads = 256;

// ------------------------------------------------------------------------------------------
// delta[h, i] = sum_c dO[i,h,c] * O[i,h,c]
// ------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void attn_bwd_delta_kernel(const bf16* __restrict__ O, const bf16* __restrict__ dO,
                                                             float* __restrict__ delta, int N, int Hl,
                                                             int64_t row_stride, int64_t head_stride) {
    constexpr int LPR = D / 8;                                   // lanes per (token, head) row
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t pair = gid / LPR;
    const int sub = (int)(gid % LPR);
    const bool live = pair < (int64_t)N * Hl;
    const int64_t row = live ? pair / Hl : 0;
    const int head = live ? (int)(pair % Hl) : 0;
    const int64_t off = row * row_stride + head * head_stride + sub * 8;
    const bf16x8 a = *reinterpret_cast<const bf16x8*>(O + off);
    const bf16x8 b = *reinterpret_cast<const bf16x8*>(dO + off);
    float acc = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc += (float)a[e] * (float)b[e];
#pragma unroll
    for (int m = LPR / 2; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 64);
    if (live && sub == 0) delta[(int64_t)head * N + row] = acc;
}

// ------------------------------------------------------------------------------------------
// dQ: same tiling as the forward pass (a lane owns one query, keys run down the C rows).
// ------------------------------------------------------------------------------------------
constexpr int kDqBQ = 128;
constexpr int kDqBK = 64;

template <int D, bool CAUSAL>
__global__ __launch_bounds__(kBwdThreads, 2) void attn_bwd_dq_kernel(
    const bf16* __restrict__ Q, const bf16* __restrict__ K, const bf16* __restrict__ V, const bf16* __restrict__ dO,
    const float* __restrict__ LSE, const float* __restrict__ DELTA, bf16* __restrict__ dQ, int N, int n_qtiles,
    int64_t row_stride, int64_t head_stride, float scale) {
    constexpr int RS = LdsStride<D>::row, TS = LdsStride<D>::tr;
    constexpr int NT = D / 16, NKB = kDqBK / 32, NCB = D / 32;
    using IO = TileIO<D, kDqBK, kBwdThreads>;

    __shared__ __attribute__((aligned(16))) bf16 k_row[kDqBK * RS];   // K for S^T      (row reads)
    __shared__ __attribute__((aligned(16))) bf16 k_tr[kDqBK * TS];    // K for dQ^T     (transposing reads)
    __shared__ __attribute__((aligned(16))) bf16 v_row[kDqBK * RS];   // V for dP^T     (row reads)

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, ln = lane & 31;
    const int head = blockIdx.x / n_qtiles;
    const int qt = n_qtiles - 1 - (blockIdx.x - head * n_qtiles);
    const int q0 = qt * kDqBQ;
    const int64_t hoff = (int64_t)head * head_stride;
    const bf16* Kh = K + hoff;
    const bf16* Vh = V + hoff;

    const int q_row = q0 + wave * 32 + ln;
    const int q_ld = q_row < N ? q_row : N - 1;
    bf16x8 qreg[NT], doreg[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        qreg[t] = *reinterpret_cast<const bf16x8*>(Q + hoff + (int64_t)q_ld * row_stride + 16 * t + 8 * g);
        doreg[t] = *reinterpret_cast<const bf16x8*>(dO + hoff + (int64_t)q_ld * row_stride + 16 * t + 8 * g);
    }
    const float sl2 = scale * kLog2e;
    const float lse2 = LSE[(int64_t)head * N + q_ld] * kLog2e;
    const float delta = DELTA[(int64_t)head * N + q_ld];

    f32x16 acc[NCB];
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[cb][r] = 0.f;

    int k_end = N;
    if (CAUSAL) { const int lim = q0 + kDqBQ; k_end = lim < N ? lim : N; }
    const int n_kt = (k_end + kDqBK - 1) / kDqBK;
    const int wave_qmin = q0 + wave * 32;

    u32x4 kreg[IO::kPerThread], vreg[IO::kPerThread];
    IO::load(kreg, Kh, row_stride, 0, N, tid);
    IO::load(vreg, Vh, row_stride, 0, N, tid);

    for (int kt = 0; kt < n_kt; ++kt) {
        const int k0 = kt * kDqBK;
        __syncthreads();
        IO::store(kreg, k_row, RS, tid);
        IO::store(kreg, k_tr, TS, tid);
        IO::store(vreg, v_row, RS, tid);
        __syncthreads();
        if (kt + 1 < n_kt) {
            IO::load(kreg, Kh, row_stride, k0 + kDqBK, N, tid);
            IO::load(vreg, Vh, row_stride, k0 + kDqBK, N, tid);
        }
        if (CAUSAL && k0 > wave_qmin + 31) continue;

        f32x16 s[NKB], dp[NKB];
#pragma unroll
        for (int b = 0; b < NKB; ++b) {
#pragma unroll
            for (int r = 0; r < 16; ++r) { s[b][r] = 0.f; dp[b][r] = 0.f; }
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                s[b] = mfma32(lds_read_row8(k_row + (32 * b + ln) * RS + 16 * t + 8 * g), qreg[t], s[b]);
                dp[b] = mfma32(lds_read_row8(v_row + (32 * b + ln) * RS + 16 * t + 8 * g), doreg[t], dp[b]);
            }
        }
        const bool need_mask = (CAUSAL && k0 + kDqBK - 1 > wave_qmin) || (k0 + kDqBK > N);
#pragma unroll
        for (int b = 0; b < NKB; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float p = fast_exp2(__builtin_fmaf(s[b][r], sl2, -lse2));
                if (need_mask) {
                    const int j = k0 + 32 * b + crow(r, g);
                    if ((CAUSAL && j > q_row) || j >= N) p = 0.f;
                }
                s[b][r] = p * (dp[b][r] - delta);                      // dS^T
            }
#pragma unroll
        for (int b = 0; b < NKB; ++b)
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const bf16x8 dsb = pack_b_operand(s[b], u);
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb)
                    acc[cb] = mfma32(lds_read_transposed_a(k_tr, TS, 32 * b + 16 * u, 32 * cb, lane), dsb, acc[cb]);
            }
    }

    if (q_row < N) {
        bf16* orow = dQ + hoff + (int64_t)q_row * row_stride;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                bf16x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = (bf16)(acc[cb][4 * rq + e] * scale);
                *reinterpret_cast<bf16x4*>(orow + 32 * cb + 8 * rq + 4 * g) = w;
            }
    }
}

// ------------------------------------------------------------------------------------------
// dK, dV: one workgroup owns 128 keys (a lane owns one key, queries run down the C rows).
// ------------------------------------------------------------------------------------------
constexpr int kDkvBK = 128;   // keys per workgroup
constexpr int kDkvBQ = 64;    // queries per LDS tile

template <int D, bool CAUSAL>
__global__ __launch_bounds__(kBwdThreads, 1) void attn_bwd_dkv_kernel(
    const bf16* __restrict__ Q, const bf16* __restrict__ K, const bf16* __restrict__ V, const bf16* __restrict__ dO,
    const float* __restrict__ LSE, const float* __restrict__ DELTA, bf16* __restrict__ dK, bf16* __restrict__ dV,
    int N, int n_ktiles, int64_t row_stride, int64_t head_stride, float scale) {
    constexpr int RS = LdsStride<D>::row, TS = LdsStride<D>::tr;
    constexpr int NT = D / 16, NRB = kDkvBQ / 32, NCB = D / 32;
    using IO = TileIO<D, kDkvBQ, kBwdThreads>;

    __shared__ __attribute__((aligned(16))) bf16 q_row_t[kDkvBQ * RS];
    __shared__ __attribute__((aligned(16))) bf16 q_tr[kDkvBQ * TS];
    __shared__ __attribute__((aligned(16))) bf16 do_row_t[kDkvBQ * RS];
    __shared__ __attribute__((aligned(16))) bf16 do_tr[kDkvBQ * TS];
    __shared__ __attribute__((aligned(16))) float lse_s[kDkvBQ];
    __shared__ __attribute__((aligned(16))) float delta_s[kDkvBQ];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, ln = lane & 31;
    const int head = blockIdx.x / n_ktiles;
    const int ktile = blockIdx.x - head * n_ktiles;          // key tile 0 is the heaviest: first
    const int j0 = ktile * kDkvBK;
    const int64_t hoff = (int64_t)head * head_stride;
    const bf16* Qh = Q + hoff;
    const bf16* dOh = dO + hoff;
    const float* lse_h = LSE + (int64_t)head * N;
    const float* delta_h = DELTA + (int64_t)head * N;

    const int j_col = j0 + wave * 32 + ln;                   // this lane's key
    const int j_ld = j_col < N ? j_col : N - 1;
    bf16x8 kreg[NT], vreg[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        kreg[t] = *reinterpret_cast<const bf16x8*>(K + hoff + (int64_t)j_ld * row_stride + 16 * t + 8 * g);
        vreg[t] = *reinterpret_cast<const bf16x8*>(V + hoff + (int64_t)j_ld * row_stride + 16 * t + 8 * g);
    }
    const float sl2 = scale * kLog2e;

    f32x16 dk_acc[NCB], dv_acc[NCB];
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) { dk_acc[cb][r] = 0.f; dv_acc[cb][r] = 0.f; }

    const int n_it = (N + kDkvBQ - 1) / kDkvBQ;
    const int it0 = CAUSAL ? j0 / kDkvBQ : 0;
    const int wave_jmin = j0 + wave * 32;

    u32x4 qpre[IO::kPerThread], dopre[IO::kPerThread];
    float lse_pre = 0.f, delta_pre = 0.f;
    auto prefetch = [&](int it) {
        const int i0 = it * kDkvBQ;
        IO::load(qpre, Qh, row_stride, i0, N, tid);
        IO::load(dopre, dOh, row_stride, i0, N, tid);
        if (tid < kDkvBQ) {
            int i = i0 + tid;
            i = i < N ? i : N - 1;
            lse_pre = lse_h[i] * kLog2e;
            delta_pre = delta_h[i];
        }
    };
    if (it0 < n_it) prefetch(it0);

    for (int it = it0; it < n_it; ++it) {
        const int i0 = it * kDkvBQ;
        __syncthreads();
        IO::store(qpre, q_row_t, RS, tid);
        IO::store(qpre, q_tr, TS, tid);
        IO::store(dopre, do_row_t, RS, tid);
        IO::store(dopre, do_tr, TS, tid);
        if (tid < kDkvBQ) { lse_s[tid] = lse_pre; delta_s[tid] = delta_pre; }
        __syncthreads();
        if (it + 1 < n_it) prefetch(it + 1);
        // every query of this tile precedes every key of this wave: nothing visible
        if (CAUSAL && i0 + kDkvBQ - 1 < wave_jmin) continue;

        f32x16 s[NRB], dp[NRB];
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) { s[rb][r] = 0.f; dp[rb][r] = 0.f; }
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                s[rb] = mfma32(lds_read_row8(q_row_t + (32 * rb + ln) * RS + 16 * t + 8 * g), kreg[t], s[rb]);
                dp[rb] = mfma32(lds_read_row8(do_row_t + (32 * rb + ln) * RS + 16 * t + 8 * g), vreg[t], dp[rb]);
            }
        }
        const bool need_mask = (CAUSAL && i0 < wave_jmin + 31) || (i0 + kDkvBQ > N);
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const f32x4 l4 = *reinterpret_cast<const f32x4*>(lse_s + 32 * rb + 8 * rq + 4 * g);
                const f32x4 d4 = *reinterpret_cast<const f32x4*>(delta_s + 32 * rb + 8 * rq + 4 * g);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int r = 4 * rq + e;
                    float p = fast_exp2(__builtin_fmaf(s[rb][r], sl2, -l4[e]));
                    if (need_mask) {
                        const int i = i0 + 32 * rb + 8 * rq + 4 * g + e;
                        if ((CAUSAL && j_col > i) || i >= N) p = 0.f;
                    }
                    s[rb][r] = p;
                    dp[rb][r] = p * (dp[rb][r] - d4[e]);
                }
            }
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const bf16x8 pb = pack_b_operand(s[rb], u);
                const bf16x8 dsb = pack_b_operand(dp[rb], u);
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb) {
                    dv_acc[cb] = mfma32(lds_read_transposed_a(do_tr, TS, 32 * rb + 16 * u, 32 * cb, lane), pb, dv_acc[cb]);
                    dk_acc[cb] = mfma32(lds_read_transposed_a(q_tr, TS, 32 * rb + 16 * u, 32 * cb, lane), dsb, dk_acc[cb]);
                }
            }
    }

    if (j_col < N) {
        bf16* krow = dK + hoff + (int64_t)j_col * row_stride;
        bf16* vrow = dV + hoff + (int64_t)j_col * row_stride;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                bf16x4 wk, wv;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    wk[e] = (bf16)(dk_acc[cb][4 * rq + e] * scale);
                    wv[e] = (bf16)dv_acc[cb][4 * rq + e];
                }
                *reinterpret_cast<bf16x4*>(krow + 32 * cb + 8 * rq + 4 * g) = wk;
                *reinterpret_cast<bf16x4*>(vrow + 32 * cb + 8 * rq + 4 * g) = wv;
            }
    }
}

template <int D>
static int launch_bwd(int stage_mask, const void* q, const void* k, const void* v, const void* o, const void* dout,
                      const float* lse, void* dq, void* dk, void* dv, float* delta, int64_t N, int Hl, float scale,
                      int causal, TensorStrides st, hipStream_t stream) {
    const int64_t pairs = N * Hl;
    const int64_t delta_blocks = (pairs * (D / 8) + 255) / 256;
    const int64_t n_qtiles = (N + kDqBQ - 1) / kDqBQ, n_ktiles = (N + kDkvBK - 1) / kDkvBK;
    if (delta_blocks > 0x7FFFFFFFll || n_qtiles * Hl > 0x7FFFFFFFll) return ULY_ERR_SHAPE;
    const bf16 *Q = (const bf16*)q, *K = (const bf16*)k, *V = (const bf16*)v, *dO = (const bf16*)dout;
    const dim3 gkv((uint32_t)(n_ktiles * Hl)), gq((uint32_t)(n_qtiles * Hl)), block(kBwdThreads);

    if (stage_mask & 1) {
        attn_bwd_delta_kernel<D><<<dim3((uint32_t)delta_blocks), dim3(256), 0, stream>>>((const bf16*)o, dO, delta,
                                                                                         (int)N, Hl, st.row, st.head);
        if (hipGetLastError() != hipSuccess) return ULY_ERR_LAUNCH;
    }
    if (stage_mask & 2) {
        if (causal)
            attn_bwd_dkv_kernel<D, true><<<gkv, block, 0, stream>>>(Q, K, V, dO, lse, delta, (bf16*)dk, (bf16*)dv,
                                                                    (int)N, (int)n_ktiles, st.row, st.head, scale);
        else
            attn_bwd_dkv_kernel<D, false><<<gkv, block, 0, stream>>>(Q, K, V, dO, lse, delta, (bf16*)dk, (bf16*)dv,
                                                                     (int)N, (int)n_ktiles, st.row, st.head, scale);
        if (hipGetLastError() != hipSuccess) return ULY_ERR_LAUNCH;
    }
    if (stage_mask & 4) {
        if (causal)
            attn_bwd_dq_kernel<D, true><<<gq, block, 0, stream>>>(Q, K, V, dO, lse, delta, (bf16*)dq, (int)N,
                                                                  (int)n_qtiles, st.row, st.head, scale);
        else
            attn_bwd_dq_kernel<D, false><<<gq, block, 0, stream>>>(Q, K, V, dO, lse, delta, (bf16*)dq, (int)N,
                                                                   (int)n_qtiles, st.row, st.head, scale);
        if (hipGetLastError() != hipSuccess) return ULY_ERR_LAUNCH;
    }
    return ULY_OK;
}

int attn_bwd_launch(int stage_mask, const void* q, const void* k, const void* v, const void* o, const void* dout,
                    const float* lse, void* dq, void* dk, void* dv, float* delta, int64_t N, int Hl, int d,
                    float scale, int causal, TensorStrides st, void* stream) {
    if (d == 128)
        return launch_bwd<128>(stage_mask, q, k, v, o, dout, lse, dq, dk, dv, delta, N, Hl, scale, causal, st,
                               (hipStream_t)stream);
    return launch_bwd<64>(stage_mask, q, k, v, o, dout, lse, dq, dk, dv, delta, N, Hl, scale, causal, st,
                          (hipStream_t)stream);
}

}  // namespace uly
