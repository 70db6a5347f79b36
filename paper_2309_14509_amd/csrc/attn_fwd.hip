// Forward pass of exact softmax attention (paper Equation 1, causal variant of Section 3.4)
// for the local heads of one GPU: tiled online softmax, bf16 MFMA, fp32 accumulation.
//
// Work decomposition: one workgroup (4 waves) owns 128 consecutive queries of one head; each wave
// owns 32 of them as the COLUMNS of its MFMA tiles:
//     S^T (keys x queries) = K_tile (LDS, row reads) * Q^T (registers)
//     O^T (d x queries)   += V_tile^T (LDS, transposing reads) * P^T (registers, straight from S^T)
// so a lane owns one query: the running max / sum are per-lane scalars and the only cross-lane
// step per tile is one exchange between lanes l and l^32.
//
// K/V tiles of 64 keys go from global memory straight into a double-buffered, swizzled LDS tile
// (no VGPR staging); one barrier per tile.  The rescale of the output accumulator is skipped for
// every tile in which no row of the wave sees a new maximum (most tiles of a long sequence); the
// reference maximum of a row is always its exact running maximum, so its largest weight is exactly 1.
#include "attn_common.h"
#include "internal.h"

namespace uly {

constexpr int kFwdThreads = 256;
constexpr int kFwdWaves = 4;
constexpr int kFwdBQ = 128;   // queries per workgroup
constexpr int kFwdBK = 64;    // keys per LDS tile

template <int D, bool CAUSAL>
__global__ __launch_bounds__(kFwdThreads, 2) void attn_fwd_kernel(const bf16* __restrict__ Q, const bf16* __restrict__ K,
                                                                   const bf16* __restrict__ V, bf16* __restrict__ O,
                                                                   float* __restrict__ LSE, int N, int n_qtiles,
                                                                   int64_t row_stride, int64_t head_stride,
                                                                   float scale) {
    constexpr int NT = D / 16;          // contraction steps over the head dim
    constexpr int NKB = kFwdBK / 32;    // 32-key blocks per tile
    constexpr int NCB = D / 32;         // 32-channel blocks of the output
    constexpr int TILE = kFwdBK * D;    // elements per LDS tile
    using Loader = DirectTile<D, kFwdBK, kFwdWaves>;

    // two buffers per tensor, as separate objects so that reads of one are known not to touch the other
    __shared__ __attribute__((aligned(1024))) bf16 k_lds0[TILE];
    __shared__ __attribute__((aligned(1024))) bf16 k_lds1[TILE];
    __shared__ __attribute__((aligned(1024))) bf16 v_lds0[TILE];
    __shared__ __attribute__((aligned(1024))) bf16 v_lds1[TILE];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, ln = lane & 31;
    // head-major order, heaviest (last) query tile of a head first
    const int head = blockIdx.x / n_qtiles;
    const int qt = n_qtiles - 1 - (blockIdx.x - head * n_qtiles);
    const int q0 = qt * kFwdBQ;
    const int64_t hoff = (int64_t)head * head_stride;
    const bf16* Qh = Q + hoff;
    const bf16* Kh = K + hoff;
    const bf16* Vh = V + hoff;

    int k_end = N;
    if (CAUSAL) { const int lim = q0 + kFwdBQ; k_end = lim < N ? lim : N; }
    const int n_kt = (k_end + kFwdBK - 1) / kFwdBK;

    const typename Loader::LaneOffsets ld_off = Loader::lane_offsets(row_stride, wave, lane);
    Loader::issue_clamped(k_lds0, Kh, row_stride, 0, N, wave, lane);
    Loader::issue_clamped(v_lds0, Vh, row_stride, 0, N, wave, lane);

    const int q_row = q0 + wave * 32 + ln;                     // this lane's query
    const int q_ld = q_row < N ? q_row : N - 1;
    bf16x8 qreg[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
        qreg[t] = *reinterpret_cast<const bf16x8*>(Qh + (int64_t)q_ld * row_stride + 16 * t + 8 * g);

    // per-lane LDS element offsets (tile-row offsets that are multiples of 16 are added as immediates)
    int k_off[NT];                      // row read of K: row ln, chunk 2t+g
#pragma unroll
    for (int t = 0; t < NT; ++t) k_off[t] = tile_off<D>(ln, 2 * t + g);
    int v_off[NCB][2];                  // transposing read of V: rows 4g+(i>>2) (+8), channels 32cb+16h+4(i&3)
    {
        const int i = lane & 15, h = (lane >> 4) & 1;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int hh = 0; hh < 2; ++hh)
                v_off[cb][hh] = tile_off<D>(4 * g + (i >> 2) + 8 * hh, 4 * cb + 2 * h + ((i & 3) >> 1)) + 4 * (i & 1);
    }

    const float sl2 = scale * kLog2e;
    float m_used = -INFINITY;    // reference maximum (raw logits) that the exponentials are taken against
    float ms = 0.f;              // m_used * sl2 (0 while m_used is -inf)
    float l_run = 0.f;           // this lane's share of the running sum
    f32x16 oacc[NCB];
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[cb][r] = 0.f;

    const int wave_qmin = q0 + wave * 32;

    wait_direct_loads();
    __syncthreads();

    auto do_tile = [&](const bf16* kt_lds, const bf16* vt_lds, bf16* kn_lds, bf16* vn_lds, int kt)
                       __attribute__((always_inline)) {
        const int k0 = kt * kFwdBK;
        if (kt + 1 < n_kt) {                 // next tile -> the other buffer (everyone left it at the last barrier)
            const int kn = k0 + kFwdBK;
            if (kn + kFwdBK <= N) {
                Loader::issue(kn_lds, Kh + (int64_t)kn * row_stride, ld_off, wave);
                Loader::issue(vn_lds, Vh + (int64_t)kn * row_stride, ld_off, wave);
            } else {
                Loader::issue_clamped(kn_lds, Kh, row_stride, kn, N, wave, lane);
                Loader::issue_clamped(vn_lds, Vh, row_stride, kn, N, wave, lane);
            }
        }
        // A wave whose queries all precede this tile has nothing to do (only in diagonal tiles).
        if (!(CAUSAL && k0 > wave_qmin + 31)) {
            // ---- S^T = K Q^T
            f32x16 s[NKB];
#pragma unroll
            for (int b = 0; b < NKB; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[b][r] = 0.f;
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int b = 0; b < NKB; ++b)
                    s[b] = mfma32(lds_read_row8(kt_lds + k_off[t] + 32 * b * D), qreg[t], s[b]);

            // ---- mask (diagonal tiles and the ragged last tile only)
            const bool need_mask = (CAUSAL && k0 + kFwdBK - 1 > wave_qmin) || (k0 + kFwdBK > N);
            if (need_mask) {
#pragma unroll
                for (int b = 0; b < NKB; ++b)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int j = k0 + 32 * b + crow(r, g);
                        if ((CAUSAL && j > q_row) || j >= N) s[b][r] = -INFINITY;
                    }
            }
            // ---- online softmax; the rescale runs only when some row of this wave has a new maximum
            float m_tile = s[0][0];
#pragma unroll
            for (int b = 0; b < NKB; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) m_tile = fmaxf(m_tile, s[b][r]);
            m_tile = xhalf_max(m_tile);
            const bool advance = m_tile > m_used;      // always true on the first tile (m_used = -inf)
            if (__builtin_amdgcn_ballot_w64(advance) != 0) {
                const float m_new = fmaxf(m_used, m_tile);
                const float m_fin = (m_new == -INFINITY) ? 0.f : m_new;          // padding rows only
                const float alpha = fast_exp2((m_used - m_fin) * sl2);
                l_run *= alpha;
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[cb][r] *= alpha;
                m_used = m_new;
                ms = m_fin * sl2;
            }
            float rs[4] = {0.f, 0.f, 0.f, 0.f};          // four chains instead of one 32-deep add chain
#pragma unroll
            for (int b = 0; b < NKB; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float p = fast_exp2(__builtin_fmaf(s[b][r], sl2, -ms));
                    s[b][r] = p;
                    rs[r & 3] += p;
                }
            l_run += (rs[0] + rs[1]) + (rs[2] + rs[3]);

            // ---- O^T += V^T P^T
            // Rows with few visible keys are where |O| is largest and where bf16 rounding of P would be
            // the dominant error, so the diagonal tiles carry P in two bf16 pieces (P = hi + lo).
            if (need_mask) {
#pragma unroll
                for (int b = 0; b < NKB; ++b)
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        const bf16x8 pb = pack_b_operand(s[b], u);
                        bf16x8 plo;
#pragma unroll
                        for (int e = 0; e < 8; ++e) plo[e] = (bf16)(s[b][8 * u + e] - (float)pb[e]);
#pragma unroll
                        for (int cb = 0; cb < NCB; ++cb) {
                            const bf16* vp = vt_lds + (32 * b + 16 * u) * D;
                            const bf16x4 lo = lds_read_tr4(vp + v_off[cb][0]), hi = lds_read_tr4(vp + v_off[cb][1]);
                            const bf16x8 va = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                            oacc[cb] = mfma32(va, pb, oacc[cb]);
                            oacc[cb] = mfma32(va, plo, oacc[cb]);
                        }
                    }
            } else {
#pragma unroll
                for (int b = 0; b < NKB; ++b)
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        const bf16x8 pb = pack_b_operand(s[b], u);
#pragma unroll
                        for (int cb = 0; cb < NCB; ++cb) {
                            const bf16* vp = vt_lds + (32 * b + 16 * u) * D;
                            const bf16x4 lo = lds_read_tr4(vp + v_off[cb][0]), hi = lds_read_tr4(vp + v_off[cb][1]);
                            oacc[cb] = mfma32(__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7), pb, oacc[cb]);
                        }
                    }
            }
        }
        wait_direct_loads();
        __syncthreads();
    };

    for (int kt = 0; kt < n_kt; kt += 2) {
        do_tile(k_lds0, v_lds0, k_lds1, v_lds1, kt);
        if (kt + 1 < n_kt) do_tile(k_lds1, v_lds1, k_lds0, v_lds0, kt + 1);
    }

    // ---- epilogue: normalise, store O (bf16) and LSE (natural log)
    const float l_tot = xhalf_sum(l_run);
    const float inv = 1.f / l_tot;
    if (q_row < N) {
        bf16* orow = O + hoff + (int64_t)q_row * row_stride;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                bf16x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = (bf16)(oacc[cb][4 * rq + e] * inv);
                *reinterpret_cast<bf16x4*>(orow + 32 * cb + 8 * rq + 4 * g) = w;
            }
        if (g == 0) LSE[(int64_t)head * N + q_row] = m_used * scale + __logf(l_tot);
    }
}

template <int D>
static int launch_fwd(const void* q, const void* k, const void* v, void* o, float* lse, int64_t N, int Hl,
                      float scale, int causal, TensorStrides st, hipStream_t stream) {
    const int64_t n_qtiles = (N + kFwdBQ - 1) / kFwdBQ;
    const int64_t blocks = n_qtiles * Hl;
    if (blocks > 0x7FFFFFFFll) return ULY_ERR_SHAPE;
    dim3 grid((uint32_t)blocks), block(kFwdThreads);
    if (causal)
        attn_fwd_kernel<D, true><<<grid, block, 0, stream>>>((const bf16*)q, (const bf16*)k, (const bf16*)v, (bf16*)o,
                                                             lse, (int)N, (int)n_qtiles, st.row, st.head, scale);
    else
        attn_fwd_kernel<D, false><<<grid, block, 0, stream>>>((const bf16*)q, (const bf16*)k, (const bf16*)v,
                                                              (bf16*)o, lse, (int)N, (int)n_qtiles, st.row, st.head,
                                                              scale);
    return hipGetLastError() == hipSuccess ? ULY_OK : ULY_ERR_LAUNCH;
}

int attn_fwd_launch(const void* q, const void* k, const void* v, void* o, float* lse, int64_t N, int Hl, int d,
                    float scale, int causal, TensorStrides st, void* stream) {
    if (d == 128) return launch_fwd<128>(q, k, v, o, lse, N, Hl, scale, causal, st, (hipStream_t)stream);
    return launch_fwd<64>(q, k, v, o, lse, N, Hl, scale, causal, st, (hipStream_t)stream);
}

}  // namespace uly
