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
#include <type_traits>

#include "attn_common.h"
#include "internal.h"

namespace uly {
namespace ULY_ELEM_NS {

// ------------------------------------------------------------------------------------------
// Row statistics for the backward kernels, in a padded [Hl, stride] layout (stride >= N rounded up to 128, + 64):
//   delta[h, i] = sum_c dO[i,h,c] * O[i,h,c]        lse2[h, i] = LSE[h, i] * log2(e)
// Rows N .. stride-1 get delta = 0 and lse2 = +inf, so that a padding row's probability
// exp2(s - lse2) is exactly 0 without any test in the consumers.
// ------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void attn_bwd_delta_kernel(const e16* __restrict__ O, const e16* __restrict__ dO,
                                                             const float* __restrict__ LSE, float* __restrict__ delta,
                                                             float* __restrict__ lse2, int N, int Hl, int64_t stride,
                                                             int64_t row_stride, int64_t head_stride) {
    constexpr int LPR = D / 8;                                   // lanes per (token, head) row
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t pair = gid / LPR;
    const int sub = (int)(gid % LPR);
    const bool in_grid = pair < stride * Hl;
    const int64_t row = in_grid ? pair / Hl : 0;
    const int head = in_grid ? (int)(pair % Hl) : 0;
    const bool live = in_grid && row < N;
    const int64_t ld_row = live ? row : 0;
    const int64_t off = ld_row * row_stride + head * head_stride + sub * 8;
    const e16x8 a = *reinterpret_cast<const e16x8*>(O + off);
    const e16x8 b = *reinterpret_cast<const e16x8*>(dO + off);
    float acc = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc += (float)a[e] * (float)b[e];
#pragma unroll
    for (int m = LPR / 2; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 64);
    if (in_grid && sub == 0) {
        delta[(int64_t)head * stride + row] = live ? acc : 0.f;
        lse2[(int64_t)head * stride + row] = live ? LSE[(int64_t)head * N + row] * kLog2e : INFINITY;
    }
}

// ------------------------------------------------------------------------------------------
// dQ: one workgroup (4 waves, one per SIMD) owns 128 queries; a lane owns one query (a column of
// S^T), keys run down the C rows.  K and V stream through LDS in 32-key tiles (ring of 4, filled
// straight from global memory two iterations ahead).  Same software pipeline as the dK/dV kernel:
//     matrix pipe:  S^T, dP^T of block b+1      vector pipe:  dS^T of block b      (region A)
//     matrix pipe:  dQ^T += K^T dS^T of block b                                    (region B)
// ------------------------------------------------------------------------------------------
constexpr int kDqThreads = 256;
constexpr int kDqWaves = 4;
constexpr int kDqBQ = 128;    // queries per workgroup
constexpr int kDqBK = 32;     // keys per LDS tile
constexpr int kDqRing = 4;

// SPARSE (causal only) in both backward kernels: the (query, key) pairs are further restricted to the
// blocks of a CSR pattern over 256 x 256 token blocks (see the forward kernel).  The dQ kernel walks the
// block columns listed for its block row (row_ptr, col_idx: ascending, diagonal last); the dK/dV kernel
// the block rows listed for its block column (col_ptr, row_idx: ascending, diagonal first).
constexpr int kSparseBlockBwd = 256;

template <int D, bool CAUSAL, bool SPARSE = false, bool PLAN = false>
__global__ __launch_bounds__(kDqThreads, 1) void attn_bwd_dq_kernel(
    const e16* __restrict__ Q, const e16* __restrict__ K, const e16* __restrict__ V, const e16* __restrict__ dO,
    const float* __restrict__ LSE2, const float* __restrict__ DELTA, int64_t ws_stride, e16* __restrict__ dQ, int N,
    int Nk, int n_qtiles, int64_t row_stride, int64_t head_stride, int64_t kv_head_stride, float scale,
    const int* __restrict__ row_ptr, const int* __restrict__ col_idx, const int4* __restrict__ plan,
    float* __restrict__ partial, int slots_per_head) {
    static_assert(!SPARSE || CAUSAL, "the sparse pattern refines the causal mask");
    static_assert(!PLAN || SPARSE || !CAUSAL, "dense causal query tiles are paired, not planned");
    constexpr int NT = D / 16, NCB = D / 32;
    constexpr int TILE = kDqBK * D;
    constexpr int TB = TILE * 2;
    constexpr int KB = 0, VB = kDqRing * TB;    // byte offsets of the K ring and the V ring
    constexpr int HALF = 16 * D * 2;
    using Loader = DirectTile<D, kDqBK, kDqWaves, SwzBoth>;
    constexpr int LPT = 2 * Loader::kPerWave;   // global loads per wave per tile

    __shared__ __attribute__((aligned(1024))) e16 smem[2 * kDqRing * TILE];

    const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5, ln = lane & 31;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // uniform: LDS tile addresses stay scalar
    // Work assignment (causal): a workgroup takes query tile n_qtiles-1-pr and then its mirror image
    // pr, so every workgroup does the same amount of work.  It walks the key blocks of the first tile
    // upwards from the start of the sequence and those of the second downwards from its diagonal: at
    // any moment all workgroups that started together read one of only two key blocks, which keeps
    // the K/V stream in the L2 caches instead of re-fetching it per workgroup.
    // PLAN (unmasked attention with few query tiles; block rows of a pattern): grid (heads, work items); an
    // item is a query tile and a range of its walk, the items of a cut tile write fp32 partial sums (see the
    // plan kernels).
    const int n_pairs = (CAUSAL && !SPARSE) ? (n_qtiles + 1) / 2 : n_qtiles;
    const int head = PLAN ? blockIdx.x : blockIdx.x / n_pairs;
    int pr = blockIdx.x - head * n_pairs;
    int p_off = 0, p_end = 0, slot = -1;
    if (PLAN) {
        const int4 hdr = plan[0];
        if ((int)blockIdx.y >= hdr.x) return;
        const int4 it = plan[1 + blockIdx.y];
        pr = it.x;
        p_off = it.y;
        p_end = it.z;
        slot = (int)blockIdx.y < hdr.y ? (int)blockIdx.y : -1;
    }
    const int64_t hoff = (int64_t)head * head_stride;
    // N queries, Nk keys (Nk = N for self-attention); K and V may have their own head stride
    const e16* Kh = K + (int64_t)head * kv_head_stride;
    const e16* Vh = V + (int64_t)head * kv_head_stride;

    // Key blocks are walked in whole groups of four; blocks nblk .. do not exist (all their keys are
    // masked) and re-read the data of the last real block.
    const int nblk = (Nk + kDqBK - 1) / kDqBK;

    const typename Loader::LaneOffsets ld = Loader::lane_offsets(row_stride, wave, lane);
    const typename Loader::TailOffsets ld_tail = Loader::tail_offsets(row_stride, wave, lane, Nk);
    auto load_tile = [&](int slot, int tb) __attribute__((always_inline)) {     // branch-free
        tb = tb < nblk ? tb : nblk - 1;          // blocks past the end re-read the last real one
        const int r0 = tb * kDqBK;
        const bool is_tail = r0 + kDqBK > Nk;
        Loader::issue_sel(smem + slot * TILE, Kh + (int64_t)r0 * row_stride, ld, ld_tail, is_tail, wave);
        Loader::issue_sel(smem + (kDqRing + slot) * TILE, Vh + (int64_t)r0 * row_stride, ld, ld_tail, is_tail, wave);
    };
    const float sl2 = scale * kLog2e;
    // For the stretch of a walk whose fetches are consecutive whole blocks (no clamp, no ragged tile): running
    // pointers, one step per tile, instead of an address computed from the block index.
    const e16* k_next = nullptr;
    const e16* v_next = nullptr;
    int64_t tile_step = 0;              // elements from one fetched block to the next (negative walking down)
    auto load_tile_next = [&](int slot) __attribute__((always_inline)) {
        Loader::issue(smem + slot * TILE, k_next, ld, wave);
        Loader::issue(smem + (kDqRing + slot) * TILE, v_next, ld, wave);
        k_next += tile_step;
        v_next += tile_step;
    };

    const uint32_t sbase = lds_addr(smem);
    uint32_t r_adr[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) r_adr[t] = sbase + 2 * tile_off<D>(ln, 2 * t + g);
    uint32_t t_adr[NCB][2];
    {
        const int i = lane & 15, h = (lane >> 4) & 1;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int hh = 0; hh < 2; ++hh)
                t_adr[cb][hh] = sbase + 2 * (tile_off<D>(4 * g + (i >> 2) + 8 * hh, 4 * cb + 2 * h + ((i & 3) >> 1)) +
                                             4 * (i & 1));
    }

    const int n_parts = (CAUSAL && !SPARSE && n_qtiles - 1 - pr != pr) ? 2 : 1;
#pragma unroll 1
    for (int part = 0; part < n_parts; ++part) {
    const int qt = (CAUSAL && !SPARSE && part == 0) ? n_qtiles - 1 - pr : pr;
    const int dir = part == 0 ? 1 : -1;                        // walking direction over the key blocks
    const int q0 = qt * kDqBQ;
    // blocks to process (a multiple of 4); the last four in sequence order carry the mask (diagonal
    // and/or end of the sequence), all others are entirely visible
    int cnt = CAUSAL ? (q0 + kDqBQ) / kDqBK : (nblk + 3) & ~3;
    // SPARSE: BPS key blocks for every listed block column but the last (the diagonal one), which
    // contributes the key blocks from its start up to this tile's own diagonal
    constexpr int BPS = kSparseBlockBwd / kDqBK;
    int sp0 = 0, n_off = 0, diag0 = 0;
    if (SPARSE) {
        const int brow = q0 / kSparseBlockBwd;
        sp0 = row_ptr[brow];
        n_off = BPS * (row_ptr[brow + 1] - sp0 - 1);
        diag0 = brow * BPS;
        cnt = n_off + (q0 + kDqBQ) / kDqBK - diag0;
    }
    // block at walk position p; positions past the end re-read the last one (their tiles are never used)
    auto blk = [&](int p) __attribute__((always_inline)) {
        if (PLAN) p += p_off;
        p = p < cnt ? p : cnt - 1;
        if (SPARSE) return p < n_off ? BPS * col_idx[sp0 + p / BPS] + p % BPS : diag0 + (p - n_off);
        return dir > 0 ? p : cnt - 1 - p;
    };
    // positions this workgroup processes; the last four run the masking variant, which masks nothing
    // unless they are the end of the sequence
    const int walk = PLAN ? p_end - p_off : cnt;
#pragma unroll
    for (int i = 0; i < kDqRing; ++i) load_tile(i, blk(i));

    // ---- this lane's query: Q and dO rows as B operands, its two row statistics
    const int q_row = q0 + wave * 32 + ln;
    const int q_ld = q_row < N ? q_row : N - 1;
    e16x8 qreg[NT], doreg[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        qreg[t] = *reinterpret_cast<const e16x8*>(Q + hoff + (int64_t)q_ld * row_stride + 16 * t + 8 * g);
        doreg[t] = *reinterpret_cast<const e16x8*>(dO + hoff + (int64_t)q_ld * row_stride + 16 * t + 8 * g);
    }
    const float lse2 = LSE2[(int64_t)head * ws_stride + q_row];     // padded: +inf for q_row >= N
    const float delta = DELTA[(int64_t)head * ws_stride + q_row];
    // key offset c_r (inside a block starting at k0) is masked iff c_r > klim - k0
    const int klim = (CAUSAL ? (q_row < Nk - 1 ? q_row : Nk - 1) : Nk - 1) - 4 * g;


    f32x16 acc[NCB];
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[cb][r] = 0.f;

    f32x16 s[2], dp[2];
    e16x8 krow[NT], vrow[NT];
    e16x4 kt_lo[2][NCB], kt_hi[2][NCB];

    auto read_krow = [&](auto slot_tag) __attribute__((always_inline)) {
        constexpr int SL = decltype(slot_tag)::value;
#pragma unroll
        for (int t = 0; t < NT; ++t) krow[t] = lds_b128<KB + SL * TB>(r_adr[t]);
    };
    auto read_vrow = [&](auto slot_tag) __attribute__((always_inline)) {
        constexpr int SL = decltype(slot_tag)::value;
#pragma unroll
        for (int t = 0; t < NT; ++t) vrow[t] = lds_b128<VB + SL * TB>(r_adr[t]);
    };
    auto read_transposed = [&](auto slot_tag) __attribute__((always_inline)) {
        constexpr int SL = decltype(slot_tag)::value;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
            kt_lo[0][cb] = lds_tr_b64<KB + SL * TB>(t_adr[cb][0]);
            kt_hi[0][cb] = lds_tr_b64<KB + SL * TB>(t_adr[cb][1]);
        }
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
            kt_lo[1][cb] = lds_tr_b64<KB + SL * TB + HALF>(t_adr[cb][0]);
            kt_hi[1][cb] = lds_tr_b64<KB + SL * TB + HALF>(t_adr[cb][1]);
        }
    };
    auto tie_krow = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < NT; ++t) lds_tie(krow[t]);
    };
    auto tie_vrow = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < NT; ++t) lds_tie(vrow[t]);
    };
    auto tie_transposed = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) lds_tie(kt_lo[u][cb], kt_hi[u][cb]);
    };
    auto zero = [&](f32x16& x) __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < 16; ++r) x[r] = 0.f;
    };

    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, 1>;
    using S2 = std::integral_constant<int, 2>;
    using S3 = std::integral_constant<int, 3>;

    // ---- prologue: the tiles of positions 0, 1 resident; S^T, dP^T of position 0; then the row operands
    // of position 1
    wait_vm<2 * LPT>();
    __syncthreads();
    read_krow(S0{});
    read_vrow(S0{});
    wait_lgkm<0>();
    tie_krow();
    tie_vrow();
    // The Q and dO operands live in accumulation registers, where the matrix unit reads them directly; S^T and
    // dP^T come out in vector registers, where the vector unit reads them directly (mfma32_v_*).
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        asm volatile("" : "+a"(qreg[t]));
        asm volatile("" : "+a"(doreg[t]));
    }
    mfma32_v_first(s[0], krow[0], qreg[0]);
    mfma32_v_first(dp[0], vrow[0], doreg[0]);
#pragma unroll
    for (int t = 1; t < NT; ++t) {
        mfma32_v_acc(s[0], krow[t], qreg[t]);
        mfma32_v_acc(dp[0], vrow[t], doreg[t]);
    }
    read_krow(S1{});
    read_vrow(S1{});
    mfma32_v_settle(s[0], dp[0]);
    __builtin_amdgcn_sched_barrier(0);

    // LDS reads in flight at entry, oldest first: K rows of b+1, V rows of b+1.
    // ("b+1", "b+2" below mean the blocks of the next walk positions)
    auto iteration = [&](auto masked_tag, auto slot_tag, auto slot2_tag, int p, int b_next, auto simple_tag)
                         __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        constexpr bool SIMPLE = decltype(simple_tag)::value;      // fetch through the running pointers
        constexpr int SL = decltype(slot_tag)::value;
        constexpr int PAR = SL & 1;
        const int krel = klim - blk(p) * kDqBK;        // (b_next: the tile fetched into this position's slot)
        e16x8 dsb[2];
        // dS^T of block b (vector pipe), a pair of key rows at a time, in three stages a step apart so that no
        // instruction waits for the one before it: exponent, exponential, product (packed at once)
        float xv[8], pv[8];
        auto softmax_stage = [&](int u, int step) __attribute__((always_inline)) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {             // pair j: rows 8u+2j, 8u+2j+1
                const int first = NT == 8 ? j + j / 2 : j / 2, r = 8 * u + 2 * j;
                if (step == first) {
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const int rr = r + e;
                        float x = __builtin_fmaf(s[PAR][rr], sl2, -lse2);
                        if (MASKED) x = (8 * (rr >> 2) + (rr & 3) > krel) ? -INFINITY : x;
                        xv[2 * j + e] = x;
                    }
                }
                if (step == first + 1) {
                    pv[2 * j] = fast_exp2(xv[2 * j]);
                    pv[2 * j + 1] = fast_exp2(xv[2 * j + 1]);
                }
                if (step == first + 2) {
                    e16x2 dk = {(e16)(pv[2 * j] * (dp[PAR][r] - delta)), (e16)(pv[2 * j + 1] * (dp[PAR][r + 1] - delta))};
                    asm volatile("" : "+v"(dk));      // packed here, not wherever the values are finally used
                    dsb[u][2 * j] = dk[0];
                    dsb[u][2 * j + 1] = dk[1];
                }
            }
        };
        // One MFMA of the next block's S^T (WHICH = 0) or dP^T (1), then this step's share of the vector work on
        // rows 8u .. 8u+7 of block b; the MFMAs are fixed in place and the vector work does not cross them.
        auto a_step = [&](auto which_tag, int t, int u) __attribute__((always_inline)) {
            constexpr int WHICH = decltype(which_tag)::value;
            if (WHICH == 0) {
                if (t == 0) mfma32_v_first(s[PAR ^ 1], krow[0], qreg[0]);
                else mfma32_v_acc(s[PAR ^ 1], krow[t], qreg[t]);
            } else {
                if (t == 0) mfma32_v_first(dp[PAR ^ 1], vrow[0], doreg[0]);
                else mfma32_v_acc(dp[PAR ^ 1], vrow[t], doreg[t]);
            }
            softmax_stage(u, t);
            __builtin_amdgcn_sched_barrier(0);
        };
        using W0 = std::integral_constant<int, 0>;
        using W1 = std::integral_constant<int, 1>;

        wait_lgkm<NT>();                              // K rows of b+1 (the V rows may still be in flight)
        tie_krow();
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < NT; ++t) a_step(W0{}, t, 0);
        wait_lgkm<0>();
        tie_vrow();
        read_transposed(slot_tag);                    // K^T of block b, for region B
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < NT; ++t) a_step(W1{}, t, 1);

        wait_lgkm<0>();
        tie_transposed();
        wait_vm<LPT>();                               // tile b+2 has landed; everyone is done with tile b
        barrier_no_drain();
        if (SIMPLE) load_tile_next(SL);
        else load_tile(SL, b_next);
        read_krow(slot2_tag);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb)
                acc[cb] = mfma32(__builtin_shufflevector(kt_lo[u][cb], kt_hi[u][cb], 0, 1, 2, 3, 4, 5, 6, 7), dsb[u],
                                 acc[cb]);
        __builtin_amdgcn_sched_barrier(0);
        read_vrow(slot2_tag);
    };

    using Plain = std::integral_constant<bool, false>;
    using Masked = std::integral_constant<bool, true>;
    using General = std::integral_constant<bool, false>;
    using Simple = std::integral_constant<bool, true>;
    // The compiler may move registers (copies at control-flow joins, spills) without knowing that a
    // hand-issued LDS read into them is still in flight, so outside the steady-state loop every
    // iteration is followed by settle(): all reads landed, their registers tied.
    auto settle = [&]() __attribute__((always_inline)) {
        wait_lgkm<0>();
        tie_krow();
        tie_vrow();
        __builtin_amdgcn_sched_barrier(0);
    };
    // The masked group is the last one in sequence order: walked last going up, first going down.
    int p = 0;
    settle();
    if (dir < 0) {
        iteration(Masked{}, S0{}, S2{}, 0, blk(kDqRing), General{}); settle();
        iteration(Masked{}, S1{}, S3{}, 1, blk(1 + kDqRing), General{}); settle();
        iteration(Masked{}, S2{}, S0{}, 2, blk(2 + kDqRing), General{}); settle();
        iteration(Masked{}, S3{}, S1{}, 3, blk(3 + kDqRing), General{}); settle();
        p = 4;
    }
    const int plain_end = dir > 0 ? walk - 4 : walk;
    if constexpr (!SPARSE && !PLAN) {
        // Groups of four iterations whose fetches (walk positions p+4 .. p+7) are neither clamped to the end of
        // the walk nor reach the last block of the sequence (which may be ragged) or the ones after it.  The
        // dK/dV-free region B of this kernel is short (8 MFMAs), and the scalar address arithmetic of the
        // general fetch does not fit behind it.
        const int hi = (dir > 0 ? (cnt < nblk - 1 ? cnt : nblk - 1) : cnt) - 7;     // groups starting below hi
        const bool whole = dir > 0 || cnt - 1 - (p + kDqRing) <= nblk - 2;          // walking down: the first fetch
        int simple_end = (whole && hi > p) ? p + ((hi - p + 3) / 4) * 4 : p;
        simple_end = simple_end < plain_end ? simple_end : plain_end;
        if (p < simple_end) {
            const int bi = blk(p + kDqRing);
            k_next = Kh + (int64_t)bi * kDqBK * row_stride;
            v_next = Vh + (int64_t)bi * kDqBK * row_stride;
            tile_step = (int64_t)dir * kDqBK * row_stride;
            for (; p < simple_end; p += 4) {
                iteration(Plain{}, S0{}, S2{}, p, 0, Simple{});
                iteration(Plain{}, S1{}, S3{}, p + 1, 0, Simple{});
                iteration(Plain{}, S2{}, S0{}, p + 2, 0, Simple{});
                iteration(Plain{}, S3{}, S1{}, p + 3, 0, Simple{});
            }
            settle();
        }
    }
    for (; p < plain_end; p += 4) {
        // the blocks fetched during these four iterations; with a pattern they lie in one sparse block (the walk
        // position is a multiple of 4 and a sparse block holds 8), so one look-up in the pattern serves all four
        int bn[4];
        if (SPARSE) {
            const int b = blk(p + kDqRing);
            const bool past = p + kDqRing + (PLAN ? p_off : 0) >= cnt;
#pragma unroll
            for (int i = 0; i < 4; ++i) bn[i] = past ? b : b + i;
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) bn[i] = blk(p + kDqRing + i);
        }
        iteration(Plain{}, S0{}, S2{}, p, bn[0], General{});
        iteration(Plain{}, S1{}, S3{}, p + 1, bn[1], General{});
        iteration(Plain{}, S2{}, S0{}, p + 2, bn[2], General{});
        iteration(Plain{}, S3{}, S1{}, p + 3, bn[3], General{});
    }
    settle();
    if (dir > 0) {
        iteration(Masked{}, S0{}, S2{}, p, blk(p + kDqRing), General{}); settle();
        iteration(Masked{}, S1{}, S3{}, p + 1, blk(p + 1 + kDqRing), General{}); settle();
        iteration(Masked{}, S2{}, S0{}, p + 2, blk(p + 2 + kDqRing), General{}); settle();
        iteration(Masked{}, S3{}, S1{}, p + 3, blk(p + 3 + kDqRing), General{}); settle();
    }
    // Nothing may still be writing LDS when this query tile ends, and the operand reads issued for a
    // block that does not exist must have landed before their (now dead) registers are reused; the same
    // goes for the S^T and dP^T of that block, which are still on their way through the matrix unit.
    wait_vm<0>();
    wait_lgkm<0>();
    mfma32_v_settle(s[0], s[1], dp[0], dp[1]);
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) lds_tie(acc[cb]);
    __builtin_amdgcn_sched_barrier(0);

    if (PLAN && slot >= 0) {
        // one of several items of this query tile: fp32 partial sums [slot][query][channel]
        float* prow = partial + ((int64_t)head * slots_per_head + slot) * (kDqBQ * D) + (wave * 32 + ln) * D;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                f32x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = acc[cb][4 * rq + e] * scale;
                *reinterpret_cast<f32x4*>(prow + 32 * cb + 8 * rq + 4 * g) = w;
            }
    } else if (q_row < N) {
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
    barrier_no_drain();          // every wave is done with the ring before the next query tile refills it
    }   // query tiles of this workgroup
}

// ------------------------------------------------------------------------------------------
// dK, dV: one workgroup (4 waves, one per SIMD, up to 512 registers each) owns 128 keys; a lane owns
// one key (a column of S), queries run down the C rows.  Q and dO stream through LDS in 32-query
// tiles (ring of 4, filled straight from global memory two iterations ahead, swizzled so that both
// the row reads for S = Q K^T, dP = dO V^T and the transposing reads for dV^T += dO^T P,
// dK^T += Q^T dS are conflict-free).  Software pipeline, per iteration b:
//     matrix pipe:  S, dP of block b+1          vector pipe:  P, dS of block b      (region A)
//     matrix pipe:  dV, dK of block b                                              (region B)
// The two streams of region A sit in one basic block and are interleaved instruction by
// instruction, so a single wave keeps the matrix pipe busy while it does its exponentials.
// ------------------------------------------------------------------------------------------
constexpr int kDkvThreads = 256;
constexpr int kDkvWaves = 4;
constexpr int kDkvBK = 128;   // keys per workgroup
constexpr int kDkvBQ = 32;    // queries per LDS tile
constexpr int kDkvRing = 4;   // LDS tiles per tensor

template <int D, bool CAUSAL, bool SPARSE = false, bool PLAN = SPARSE>
__global__ __launch_bounds__(kDkvThreads, 1) void attn_bwd_dkv_kernel(
    const e16* __restrict__ Q, const e16* __restrict__ K, const e16* __restrict__ V, const e16* __restrict__ dO,
    const float* __restrict__ LSE2, const float* __restrict__ DELTA, int64_t ws_stride, e16* __restrict__ dK,
    e16* __restrict__ dV, int N, int Nk, int n_ktiles, int64_t row_stride, int64_t head_stride,
    int64_t kv_head_stride, float scale, const int* __restrict__ col_ptr, const int* __restrict__ row_idx,
    const int4* __restrict__ plan, float* __restrict__ partial, int slots_per_head) {
    static_assert(!SPARSE || CAUSAL, "the sparse pattern refines the causal mask");
    static_assert(!SPARSE || PLAN, "block columns of a pattern are walked through the work plan");
    static_assert(!(PLAN && CAUSAL && !SPARSE), "dense causal key tiles are paired, not planned");
    constexpr int NT = D / 16, NCB = D / 32;
    constexpr int TILE = kDkvBQ * D;            // elements per tile
    constexpr int TB = TILE * 2;                // bytes per tile
    constexpr int QB = 0, DOB = kDkvRing * TB;  // byte offsets of the Q ring and the dO ring
    constexpr int HALF = 16 * D * 2;            // bytes per 16 rows
    constexpr int STAT = 512;                   // bytes per ring slot of row statistics: 64 lse2, 64 delta
    using Loader = DirectTile<D, kDkvBQ, kDkvWaves, SwzBoth>;
    constexpr int LPT = 2 * Loader::kPerWave + 2;   // global loads per wave per tile (Q, dO, lse2, delta)

    __shared__ __attribute__((aligned(1024))) e16 smem[2 * kDkvRing * TILE];
    __shared__ __attribute__((aligned(256))) float stat[kDkvRing * (STAT / 4)];

    const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5, ln = lane & 31;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // uniform: LDS tile addresses stay scalar
    // Work assignment (causal): a workgroup takes key tile `pr` and then its mirror image
    // n_ktiles-1-pr, so every workgroup does the same amount of work.  It walks the query blocks of
    // the first tile downwards from the end of the sequence and those of the second upwards from its
    // diagonal: at any moment all workgroups that started together read one of only two query
    // blocks, which keeps the Q/dO stream in the L2 caches instead of re-fetching it per workgroup.
    // PLAN: grid (heads, work items); an item of the plan is a key tile and a range of the walk
    // positions of its column (long columns are cut into several items, see the plan kernels).
    const int n_pairs = (CAUSAL && !SPARSE) ? (n_ktiles + 1) / 2 : n_ktiles;
    const int head = PLAN ? blockIdx.x : blockIdx.x / n_pairs;
    int pr = blockIdx.x - head * n_pairs;
    int p_off = 0, p_end = 0, slot = -1;
    if (PLAN) {
        const int4 hdr = plan[0];                 // {items, items that write partial sums, ..}
        if ((int)blockIdx.y >= hdr.x) return;     // the grid is an upper bound on the number of items
        const int4 it = plan[1 + blockIdx.y];     // {key tile, first walk position, end, -}
        pr = it.x;
        p_off = it.y;
        p_end = it.z;
        slot = (int)blockIdx.y < hdr.y ? (int)blockIdx.y : -1;
    }
    const int64_t hoff = (int64_t)head * head_stride;
    const e16* Qh = Q + hoff;
    const e16* dOh = dO + hoff;
    const int64_t kv_hoff = (int64_t)head * kv_head_stride;   // N queries, Nk keys (Nk = N for self-attention)
    const float* lse_h = LSE2 + (int64_t)head * ws_stride;
    const float* del_h = DELTA + (int64_t)head * ws_stride;

    // Query blocks are walked in whole groups of four: blocks nblk .. nblk4-1 do not exist, their rows
    // read the padded statistics (probability exactly 0) and the data of the last real block.
    const int nblk = (N + kDkvBQ - 1) / kDkvBQ;
    const int nblk4 = (nblk + 3) & ~3;

    // ---- global -> LDS tile loads (tile index clamped: past the end the last tile is simply re-read)
    const typename Loader::LaneOffsets ld = Loader::lane_offsets(row_stride, wave, lane);
    const typename Loader::TailOffsets ld_tail = Loader::tail_offsets(row_stride, wave, lane, N);
    // The loads of one tile, in pieces (PART 0: Q, 1: dO, 2: row statistics) so that the hot loop can
    // spread them between its MFMAs.  Branch-free.
    auto load_part = [&](auto part_tag, int slot, int tb) __attribute__((always_inline)) {
        constexpr int PART = decltype(part_tag)::value;
        const int rs = tb * kDkvBQ;                     // statistics: the block's own rows (padded past N)
        tb = tb < nblk ? tb : nblk - 1;
        const int r0 = tb * kDkvBQ;
        const bool is_tail = r0 + kDkvBQ > N;
        if (PART == 0) Loader::issue_sel(smem + slot * TILE, Qh + (int64_t)r0 * row_stride, ld, ld_tail, is_tail, wave);
        if (PART == 1)
            Loader::issue_sel(smem + (kDkvRing + slot) * TILE, dOh + (int64_t)r0 * row_stride, ld, ld_tail, is_tail, wave);
        if (PART == 2) {
            // row statistics: 64 floats each (the padded arrays make rows r0 .. r0+63 readable, also for blocks past the end); every
            // wave issues the same two loads so that all waves count the same number of loads per tile
            float* sdst = stat + slot * (STAT / 4);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(lse_h + rs + lane),
                                             ULY_LDS(void, sdst), 4, 0, 0);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(del_h + rs + lane),
                                             ULY_LDS(void, sdst + 64), 4, 0, 0);
        }
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    using P2 = std::integral_constant<int, 2>;
    auto load_tile = [&](int slot, int tb) __attribute__((always_inline)) {
        load_part(P0{}, slot, tb);
        load_part(P1{}, slot, tb);
        load_part(P2{}, slot, tb);
    };
    const float sl2 = scale * kLog2e;

    // ---- per-lane LDS byte addresses inside a tile (ring slot, tensor and 16-row offsets are immediates)
    const uint32_t sbase = lds_addr(smem);
    uint32_t r_adr[NT];                 // row read: row ln, chunk 2t+g
#pragma unroll
    for (int t = 0; t < NT; ++t) r_adr[t] = sbase + 2 * tile_off<D>(ln, 2 * t + g);
    uint32_t t_adr[NCB][2];             // transposing read: rows 4g+(i>>2) (+8), channels 32cb+16h+4(i&3)
    {
        const int i = lane & 15, h = (lane >> 4) & 1;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int hh = 0; hh < 2; ++hh)
                t_adr[cb][hh] = sbase + 2 * (tile_off<D>(4 * g + (i >> 2) + 8 * hh, 4 * cb + 2 * h + ((i & 3) >> 1)) +
                                             4 * (i & 1));
    }
    const uint32_t st_adr = lds_addr(stat) + 16 * g;    // rows 8q+4g .. +3 of a slot: immediate 32q (+256: delta)

    const int n_parts = (CAUSAL && !SPARSE && n_ktiles - 1 - pr != pr) ? 2 : 1;
#pragma unroll 1
    for (int part = 0; part < n_parts; ++part) {
    const int ktile = part == 0 ? pr : n_ktiles - 1 - pr;
    const int dir = (CAUSAL && !SPARSE && part == 0) ? -1 : 1;   // walking direction over the query blocks
    const int j0 = ktile * kDkvBK;
    const int b0 = CAUSAL ? j0 / kDkvBQ : 0;                  // first block that sees a key of this tile
    int cnt = nblk4 - b0;                                     // blocks to process (a multiple of 4)
    // SPARSE: the diagonal block row (listed first) contributes the query blocks from this tile's
    // diagonal to its end, every further listed block row BPS query blocks
    constexpr int BPS = kSparseBlockBwd / kDkvBQ;
    int sp0 = 0, n_diag = 0;
    if (SPARSE) {
        const int bcol = j0 / kSparseBlockBwd;
        sp0 = col_ptr[bcol];
        n_diag = (bcol + 1) * BPS - b0;
        cnt = n_diag + BPS * (col_ptr[bcol + 1] - sp0 - 1);
    }
    // block at walk position p; positions past the end re-read the last one (their tiles are never used)
    auto blk = [&](int p) __attribute__((always_inline)) {
        if (PLAN) p += p_off;
        p = p < cnt ? p : cnt - 1;
        if (SPARSE) return p < n_diag ? b0 + p : BPS * row_idx[sp0 + 1 + (p - n_diag) / BPS] + (p - n_diag) % BPS;
        return dir > 0 ? b0 + p : nblk4 - 1 - p;
    };
    const int walk = PLAN ? p_end - p_off : cnt;              // positions this workgroup processes
#pragma unroll
    for (int i = 0; i < kDkvRing; ++i) load_tile(i, blk(i));

    // ---- this lane's key: K and V rows as B operands
    const int j_col = j0 + wave * 32 + ln;
    const int j_ld = j_col < Nk ? j_col : Nk - 1;
    e16x8 kreg[NT], vreg[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        kreg[t] = *reinterpret_cast<const e16x8*>(K + kv_hoff + (int64_t)j_ld * row_stride + 16 * t + 8 * g);
        vreg[t] = *reinterpret_cast<const e16x8*>(V + kv_hoff + (int64_t)j_ld * row_stride + 16 * t + 8 * g);
    }
    const int jcol_g = j_col - 4 * g;            // causal test: row offset c_r is masked iff c_r < jcol_g - i0

    f32x16 dk_acc[NCB], dv_acc[NCB];
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) { dk_acc[cb][r] = 0.f; dv_acc[cb][r] = 0.f; }

    // pipeline registers
    f32x16 s[2], dp[2];                 // [parity]: scores / dP of the current and of the next block
    e16x8 rowq[NT], rowdo[NT];         // row operands of the block whose S, dP are computed next
    f32x4 lse4[4], del4[4];             // statistics of the block whose P, dS are computed next
    e16x4 qt_lo[2][NCB], qt_hi[2][NCB], dot_lo[2][NCB], dot_hi[2][NCB];   // transposed operands of the current block

    auto read_rowq = [&](auto slot_tag) __attribute__((always_inline)) {
        constexpr int SL = decltype(slot_tag)::value;
#pragma unroll
        for (int t = 0; t < NT; ++t) rowq[t] = lds_b128<QB + SL * TB>(r_adr[t]);
    };
    auto read_rowq_part = [&](auto slot_tag, int t0, int t1) __attribute__((always_inline)) {
        constexpr int SL = decltype(slot_tag)::value;
#pragma unroll
        for (int t = 0; t < NT; ++t)
            if (t >= t0 && t < t1) rowq[t] = lds_b128<QB + SL * TB>(r_adr[t]);
    };
    auto read_rowdo = [&](auto slot_tag) __attribute__((always_inline)) {
        constexpr int SL = decltype(slot_tag)::value;
#pragma unroll
        for (int t = 0; t < NT; ++t) rowdo[t] = lds_b128<DOB + SL * TB>(r_adr[t]);
    };
    auto read_stats = [&](auto slot_tag) __attribute__((always_inline)) {
        constexpr int SL = decltype(slot_tag)::value;
        lse4[0] = lds_f32x4<SL * STAT + 0>(st_adr);   lse4[1] = lds_f32x4<SL * STAT + 32>(st_adr);
        lse4[2] = lds_f32x4<SL * STAT + 64>(st_adr);  lse4[3] = lds_f32x4<SL * STAT + 96>(st_adr);
        del4[0] = lds_f32x4<SL * STAT + 256>(st_adr); del4[1] = lds_f32x4<SL * STAT + 288>(st_adr);
        del4[2] = lds_f32x4<SL * STAT + 320>(st_adr); del4[3] = lds_f32x4<SL * STAT + 352>(st_adr);
    };
    // transposed operands of rows 0-15 (U = 0) or 16-31 (U = 1) of a block; one channel block cb
    auto read_transposed = [&](auto slot_tag, auto u_tag, int cb) __attribute__((always_inline)) {
        constexpr int SL = decltype(slot_tag)::value;
        constexpr int U = decltype(u_tag)::value;
#pragma unroll
        for (int c = 0; c < NCB; ++c)
            if (c == cb) {
                dot_lo[U][c] = lds_tr_b64<DOB + SL * TB + U * HALF>(t_adr[c][0]);
                dot_hi[U][c] = lds_tr_b64<DOB + SL * TB + U * HALF>(t_adr[c][1]);
                qt_lo[U][c] = lds_tr_b64<QB + SL * TB + U * HALF>(t_adr[c][0]);
                qt_hi[U][c] = lds_tr_b64<QB + SL * TB + U * HALF>(t_adr[c][1]);
            }
    };
    auto tie_rowq = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < NT; ++t) lds_tie(rowq[t]);
        lds_tie(lse4[0], lse4[1], lse4[2], lse4[3], del4[0], del4[1], del4[2], del4[3]);
    };
    auto tie_rowdo = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < NT; ++t) lds_tie(rowdo[t]);
    };
    auto tie_transposed = [&](int u) __attribute__((always_inline)) {
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) lds_tie(dot_lo[u][cb], dot_hi[u][cb], qt_lo[u][cb], qt_hi[u][cb]);
    };
    using U0 = std::integral_constant<int, 0>;
    using U1 = std::integral_constant<int, 1>;
    auto zero = [&](f32x16& x) __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < 16; ++r) x[r] = 0.f;
    };

    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, 1>;
    using S2 = std::integral_constant<int, 2>;
    using S3 = std::integral_constant<int, 3>;

    // ---- prologue: the tiles of positions 0, 1 resident; S, dP of position 0; then (in this order) the
    // statistics of position 0 and the row operands of position 1
    wait_vm<2 * LPT>();
    __syncthreads();
    read_rowq(S0{});
    read_rowdo(S0{});
    wait_lgkm<0>();
    tie_rowq();
    tie_rowdo();
    // The K and V operands live in accumulation registers, where the matrix unit reads them directly; S and dP
    // come out in vector registers, where the vector unit reads them directly (mfma32_v_*).
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        asm volatile("" : "+a"(kreg[t]));
        asm volatile("" : "+a"(vreg[t]));
    }
    mfma32_v_first(s[0], rowq[0], kreg[0]);
    mfma32_v_first(dp[0], rowdo[0], vreg[0]);
#pragma unroll
    for (int t = 1; t < NT; ++t) {
        mfma32_v_acc(s[0], rowq[t], kreg[t]);
        mfma32_v_acc(dp[0], rowdo[t], vreg[t]);
    }
    read_stats(S0{});
    read_rowq(S1{});
    read_rowdo(S1{});
    mfma32_v_settle(s[0], dp[0]);
    __builtin_amdgcn_sched_barrier(0);

    // One iteration: walk position p (block b) lives in ring slot SL (its parity selects the s/dp set);
    // "b+1", "b+2" below mean the blocks of the next positions.
    // LDS reads in flight at entry, oldest first: statistics of b, Q rows of b+1, dO rows of b+1.
    auto iteration = [&](auto masked_tag, auto slot_tag, auto slot1_tag, auto slot2_tag, int p, int b_next)
                         __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        constexpr int SL = decltype(slot_tag)::value;
        constexpr int PAR = SL & 1;
        const int i0 = blk(p) * kDkvBQ;
        const int jrel = jcol_g - i0;                  // (b_next: the tile fetched into this position's slot)
        e16x8 pb[2], dsb[2];
        // P and dS of block b (vector pipe), a pair of query rows at a time, in three stages a step apart so that
        // no instruction waits for the one before it: exponent, exponential, product (both packed at once)
        float xv[8], pv[8];
        auto softmax_stage = [&](int u, int step) __attribute__((always_inline)) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {             // pair j: rows 8u+2j, 8u+2j+1
                const int first = NT == 8 ? j + j / 2 : j / 2, r = 8 * u + 2 * j;
                if (step == first) {
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const int rr = r + e;
                        float x = __builtin_fmaf(s[PAR][rr], sl2, -lse4[rr >> 2][rr & 3]);
                        if (MASKED && CAUSAL) x = (8 * (rr >> 2) + (rr & 3) < jrel) ? -INFINITY : x;
                        xv[2 * j + e] = x;
                    }
                }
                if (step == first + 1) {
                    pv[2 * j] = fast_exp2(xv[2 * j]);
                    pv[2 * j + 1] = fast_exp2(xv[2 * j + 1]);
                }
                if (step == first + 2) {
                    e16x2 pk = {(e16)pv[2 * j], (e16)pv[2 * j + 1]};
                    e16x2 dk = {(e16)(pv[2 * j] * (dp[PAR][r] - del4[r >> 2][r & 3])),
                                (e16)(pv[2 * j + 1] * (dp[PAR][r + 1] - del4[(r + 1) >> 2][(r + 1) & 3]))};
                    asm volatile("" : "+v"(pk), "+v"(dk));    // packed here, not wherever the values are finally used
                    pb[u][2 * j] = pk[0];
                    pb[u][2 * j + 1] = pk[1];
                    dsb[u][2 * j] = dk[0];
                    dsb[u][2 * j + 1] = dk[1];
                }
            }
        };
        // One MFMA of the next block's S (WHICH = 0) or dP (1), then this step's share of the vector work on rows
        // 8u .. 8u+7 of block b; the MFMAs are fixed in place and the vector work does not cross them.
        auto a_step = [&](auto which_tag, int t, int u) __attribute__((always_inline)) {
            constexpr int WHICH = decltype(which_tag)::value;
            if (WHICH == 0) {
                if (t == 0) mfma32_v_first(s[PAR ^ 1], rowq[0], kreg[0]);
                else mfma32_v_acc(s[PAR ^ 1], rowq[t], kreg[t]);
            } else {
                if (t == 0) mfma32_v_first(dp[PAR ^ 1], rowdo[0], vreg[0]);
                else mfma32_v_acc(dp[PAR ^ 1], rowdo[t], vreg[t]);
            }
            softmax_stage(u, t);
            __builtin_amdgcn_sched_barrier(0);
        };
        using W0 = std::integral_constant<int, 0>;
        using W1 = std::integral_constant<int, 1>;

        wait_lgkm<NT>();                              // all but the dO rows: statistics of b, Q rows of b+1
        tie_rowq();
        __builtin_amdgcn_sched_barrier(0);
        // ---- region A1: S of block b+1 (matrix pipe) || P, dS of rows 0-15 of block b (vector pipe)
#pragma unroll
        for (int t = 0; t < NT; ++t) a_step(W0{}, t, 0);
        wait_lgkm<0>();                               // dO rows of b+1
        tie_rowdo();
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) read_transposed(slot_tag, U0{}, cb);   // for region B1; lands during A2
        __builtin_amdgcn_sched_barrier(0);
        // ---- region A2: dP of block b+1 || P, dS of rows 16-31 of block b
#pragma unroll
        for (int t = 0; t < NT; ++t) a_step(W1{}, t, 1);
        wait_lgkm<0>();
        tie_transposed(0);
        __builtin_amdgcn_sched_barrier(0);

        // ---- region B: dV^T += dO^T P, dK^T += Q^T dS.  Every other instruction of the iteration is
        // placed behind one of these MFMAs so that it issues while the matrix pipe is busy.
        // B1 (rows 0-15): the transposed operands of rows 16-31 go into the registers the dO rows left
        // free, early enough to have landed when B1 ends.
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
            const e16x8 da = __builtin_shufflevector(dot_lo[0][cb], dot_hi[0][cb], 0, 1, 2, 3, 4, 5, 6, 7);
            const e16x8 qa = __builtin_shufflevector(qt_lo[0][cb], qt_hi[0][cb], 0, 1, 2, 3, 4, 5, 6, 7);
            dv_acc[cb] = mfma32(da, pb[0], dv_acc[cb]);
            __builtin_amdgcn_sched_barrier(0);
            if (2 * cb < NCB) read_transposed(slot_tag, U1{}, 2 * cb);
            __builtin_amdgcn_sched_barrier(0);
            dk_acc[cb] = mfma32(qa, dsb[0], dk_acc[cb]);
            __builtin_amdgcn_sched_barrier(0);
            if (2 * cb + 1 < NCB) read_transposed(slot_tag, U1{}, 2 * cb + 1);
            __builtin_amdgcn_sched_barrier(0);
        }
        // ---- everyone is done with tile b (its last reads have landed) and tile b+2 has landed (its
        // loads were issued two iterations ago)
        wait_lgkm<0>();
        tie_transposed(1);
        wait_vm<LPT>();
        barrier_no_drain();
        __builtin_amdgcn_sched_barrier(0);
        // B2 (rows 16-31): Q rows of block b+2 (into the registers of the transposed operands B1 used),
        // statistics of block b+1, and the loads of tile b+4 into the slot of tile b
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
            const e16x8 da = __builtin_shufflevector(dot_lo[1][cb], dot_hi[1][cb], 0, 1, 2, 3, 4, 5, 6, 7);
            const e16x8 qa = __builtin_shufflevector(qt_lo[1][cb], qt_hi[1][cb], 0, 1, 2, 3, 4, 5, 6, 7);
            dv_acc[cb] = mfma32(da, pb[1], dv_acc[cb]);
            __builtin_amdgcn_sched_barrier(0);
            if (NCB == 4) {
                if (cb == 0) read_rowq_part(slot2_tag, 0, 4);
                if (cb == 1) read_stats(slot1_tag);
                if (cb == 2) load_part(P1{}, SL, b_next);
            } else {
                if (cb == 0) read_rowq_part(slot2_tag, 0, NT);
                if (cb == 1) { load_part(P0{}, SL, b_next); load_part(P1{}, SL, b_next); }
            }
            __builtin_amdgcn_sched_barrier(0);
            dk_acc[cb] = mfma32(qa, dsb[1], dk_acc[cb]);
            __builtin_amdgcn_sched_barrier(0);
            if (NCB == 4) {
                if (cb == 0) read_rowq_part(slot2_tag, 4, 8);
                if (cb == 1) load_part(P0{}, SL, b_next);
                if (cb == 2) load_part(P2{}, SL, b_next);
            } else {
                if (cb == 0) read_stats(slot1_tag);
                if (cb == 1) load_part(P2{}, SL, b_next);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        read_rowdo(slot2_tag);                        // dO rows of block b+2, into the registers B2's operands used
    };

    // Only the four blocks on the diagonal (queries that precede some key of the workgroup) need the
    // mask; they come first when walking up and last when walking down.
    using Plain = std::integral_constant<bool, false>;
    using Masked = std::integral_constant<bool, true>;
    // The compiler may move registers (copies at control-flow joins, spills) without knowing that a
    // hand-issued LDS read into them is still in flight, so outside the steady-state loop every
    // iteration is followed by settle(): all reads landed, their registers tied.
    auto settle = [&]() __attribute__((always_inline)) {
        wait_lgkm<0>();
        tie_rowq();
        tie_rowdo();
        __builtin_amdgcn_sched_barrier(0);
    };
    int p = 0;
    settle();
    if (CAUSAL && dir > 0) {
        iteration(Masked{}, S0{}, S1{}, S2{}, 0, blk(kDkvRing)); settle();
        iteration(Masked{}, S1{}, S2{}, S3{}, 1, blk(1 + kDkvRing)); settle();
        iteration(Masked{}, S2{}, S3{}, S0{}, 2, blk(2 + kDkvRing)); settle();
        iteration(Masked{}, S3{}, S0{}, S1{}, 3, blk(3 + kDkvRing)); settle();
        p = 4;
    }
    const int plain_end = (CAUSAL && dir < 0) ? walk - 4 : walk;
    for (; p < plain_end; p += 4) {
        // the blocks fetched during these four iterations; with a pattern they lie in one sparse block (walk
        // positions are multiples of 4, a sparse block holds 8 and the diagonal part 4 or 8), so one look-up in
        // the pattern serves all four
        int bn[4];
        if (SPARSE) {
            const int b = blk(p + kDkvRing);
            const bool past = p + kDkvRing + (PLAN ? p_off : 0) >= cnt;
#pragma unroll
            for (int i = 0; i < 4; ++i) bn[i] = past ? b : b + i;
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) bn[i] = blk(p + kDkvRing + i);
        }
        iteration(Plain{}, S0{}, S1{}, S2{}, p, bn[0]);
        iteration(Plain{}, S1{}, S2{}, S3{}, p + 1, bn[1]);
        iteration(Plain{}, S2{}, S3{}, S0{}, p + 2, bn[2]);
        iteration(Plain{}, S3{}, S0{}, S1{}, p + 3, bn[3]);
    }
    settle();
    if (CAUSAL && dir < 0) {
        iteration(Masked{}, S0{}, S1{}, S2{}, p, blk(p + kDkvRing)); settle();
        iteration(Masked{}, S1{}, S2{}, S3{}, p + 1, blk(p + 1 + kDkvRing)); settle();
        iteration(Masked{}, S2{}, S3{}, S0{}, p + 2, blk(p + 2 + kDkvRing)); settle();
        iteration(Masked{}, S3{}, S0{}, S1{}, p + 3, blk(p + 3 + kDkvRing)); settle();
    }
    // Nothing may still be writing LDS when this key tile ends, and the operand reads issued for a
    // block that does not exist must have landed before their (now dead) registers are reused; the same
    // goes for the S and dP of that block, which are still on their way through the matrix unit.
    wait_vm<0>();
    wait_lgkm<0>();
    mfma32_v_settle(s[0], s[1], dp[0], dp[1]);
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) lds_tie(dk_acc[cb], dv_acc[cb]);
    __builtin_amdgcn_sched_barrier(0);

    if (PLAN && slot >= 0) {
        // one of several items of this key tile: fp32 partial sums [slot][dK, dV][key][channel]
        float* prow = partial + ((int64_t)head * slots_per_head + slot) * (2 * kDkvBK * D) + (wave * 32 + ln) * D;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                f32x4 wk, wv;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    wk[e] = dk_acc[cb][4 * rq + e] * scale;
                    wv[e] = dv_acc[cb][4 * rq + e];
                }
                *reinterpret_cast<f32x4*>(prow + 32 * cb + 8 * rq + 4 * g) = wk;
                *reinterpret_cast<f32x4*>(prow + kDkvBK * D + 32 * cb + 8 * rq + 4 * g) = wv;
            }
    } else if (j_col < Nk) {
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
    barrier_no_drain();          // every wave is done with the ring before the next key tile refills it
    }   // key tiles of this workgroup
}

// ------------------------------------------------------------------------------------------
// Work plan of the block-sparse dK/dV kernel.  A key tile's walk has cnt query blocks (a multiple
// of 4), anything from 4 to the whole sequence: one workgroup per key tile would leave the launch
// waiting for the few longest block columns.  Columns longer than L blocks are therefore cut into
// items of at most L blocks (a multiple of 4); the workgroups of a cut column write fp32 partial
// sums, which the reduce kernel adds in a fixed order.  L = max(kPlanMinLen, total work / kPlanTarget)
// so that no item exceeds a small part of one CU's share; that needs at most
// sum over cut columns of ceil(cnt / L) <= 2 * total / L <= 2 * kPlanTarget / Hl partial-sum slots per head.
// The workspace holds that many, but never more than two per key tile; a pattern that would need more
// gets L raised until its cut items fit.
//   plan[0] = {items, cut items, L, 0};  plan[1 + s] = {key tile, first position, end position, 0};
//   cut items come first (s = slot of their partial sums);  red[ktile] = {first slot, items} (items 1: not cut).
// One workgroup; every thread scans a contiguous range of key tiles.
// ------------------------------------------------------------------------------------------
constexpr int kPlanThreads = 1024;
constexpr int kPlanTarget = 4096;   // items the cut columns are aimed at, over all heads: 16 per CU, so that
                                    // a CU's share is many items (with 1024 a pattern whose work sits in long
                                    // columns left the launch a quarter longer than its average CU)
constexpr int kDenseCutTarget = 1024;   // the same for unmasked attention with a short side (uniform items)
constexpr int kPlanMinLen = 32;     // query blocks; below this the per-item overhead would show

// Slots for partial sums per head: what the target can ask for, but no more than two per key tile (the
// partial sums then take at most four times the fp32 size of dK and dV; short sequences gain nothing from
// finer cuts).  If a pattern would need more, the plan kernel raises L until it fits.
inline int plan_slots_per_head(int64_t n_ktiles, int64_t nblk4, int Hl) {
    (void)nblk4;
    const int64_t by_target = 2 * ((kPlanTarget + Hl - 1) / Hl);
    const int64_t by_size = 2 * n_ktiles + 1;
    return (int)(by_target < by_size ? by_target : by_size);
}
inline int64_t plan_items_bound(int64_t n_ktiles, int64_t nblk4, int Hl) {
    return n_ktiles + plan_slots_per_head(n_ktiles, nblk4, Hl) + 1;          // whole columns + cut items
}

__device__ __forceinline__ int block_scan_exclusive(int v, int* sh, int* total) {
    const int tid = threadIdx.x;
    sh[tid] = v;
    __syncthreads();
    for (int off = 1; off < kPlanThreads; off <<= 1) {
        const int add = tid >= off ? sh[tid - off] : 0;
        __syncthreads();
        sh[tid] += add;
        __syncthreads();
    }
    const int incl = sh[tid];
    *total = sh[kPlanThreads - 1];
    __syncthreads();
    return incl - v;
}

// mode 0: key tiles of dK/dV walk query blocks (ptr = col_ptr);  mode 1: query tiles of dQ walk key blocks
// (ptr = row_ptr);  mode 2: query tiles of the forward walk 64-key tiles (ptr = row_ptr);  mode 3: the same for
// dense causal attention (no pattern, ptr unused).  Whole tiles are listed longest first: ascending for
// columns, descending for rows (later rows see more).
__global__ __launch_bounds__(kPlanThreads) void sparse_plan_kernel(int mode, const int* __restrict__ ptr, int n_tiles,
                                                                   int N, int Hl, int slots_per_head, int target,
                                                                   int4* __restrict__ plan, int2* __restrict__ red) {
    __shared__ int sh[kPlanThreads];
    __shared__ unsigned long long sh_total;
    const int tid = threadIdx.x;
    const int chunk = (n_tiles + kPlanThreads - 1) / kPlanThreads;
    const int k0 = tid * chunk < n_tiles ? tid * chunk : n_tiles;
    const int k1 = k0 + chunk < n_tiles ? k0 + chunk : n_tiles;
    auto count = [&](int t) {
        if (mode >= 2) {                                   // forward: 256 queries, 4 tiles of 64 keys per sparse block
            const int q0 = t * 256, k_end = q0 + 256 < N ? q0 + 256 : N;
            if (mode == 3) return (k_end + 63) / 64;      // dense causal: every key tile up to the diagonal
            return 4 * (ptr[t + 1] - ptr[t] - 1) + (k_end - q0 + 63) / 64;
        }
        const int b = t / 2, listed = ptr[b + 1] - ptr[b] - 1;   // 128-token tiles: two per sparse block, 8 blocks of 32
        return 8 * listed + (mode == 0 ? 8 - 4 * (t & 1) : 4 + 4 * (t & 1));
    };
    if (tid == 0) sh_total = 0;
    __syncthreads();
    unsigned long long mine = 0;
    for (int t = k0; t < k1; ++t) mine += (unsigned long long)count(t);
    atomicAdd(&sh_total, mine);
    __syncthreads();
    const unsigned long long want = (sh_total * (unsigned long long)Hl + target - 1) / target;
    int L = want > 0x3FFFFFFFull ? 0x3FFFFFFF : (int)want;
    L = (L + 3) & ~3;
    const int min_len = mode >= 2 ? kPlanMinLen / 2 : kPlanMinLen;      // 1024 tokens either way
    L = L < min_len ? min_len : L;
    // items of a tile that walks cnt units: pieces of len units
    auto piece_len = [&](int cnt) {
        const int n = (cnt + L - 1) / L;
        return (((cnt + n - 1) / n) + 3) & ~3;
    };
    int n_cut = 0, n_whole = 0, cut_total = 0, whole_total = 0, cut_at = 0, whole_at = 0;
    for (int attempt = 0; attempt < 24; ++attempt) {
        n_cut = n_whole = 0;
        for (int t = k0; t < k1; ++t) {
            const int cnt = count(t);
            if (cnt > L) n_cut += (cnt + piece_len(cnt) - 1) / piece_len(cnt);
            else ++n_whole;
        }
        cut_at = block_scan_exclusive(n_cut, sh, &cut_total);
        whole_at = block_scan_exclusive(n_whole, sh, &whole_total);
        if (cut_total <= slots_per_head) break;
        // more cut items than slots: coarser cuts, by about the factor that is missing (in the end none)
        const long long scaled = ((long long)L * cut_total + slots_per_head - 1) / slots_per_head;
        const long long next = scaled > (long long)L + 4 ? scaled : (long long)L + 4;
        L = (attempt < 22 && next < 0x3FFFFFF0ll) ? (int)((next + 3) & ~3ll) : 0x3FFFFFFC;
    }
    if (tid == 0) plan[0] = make_int4(cut_total + whole_total, cut_total, L, 0);
    int cs = cut_at, wi = whole_at;
    for (int t = k0; t < k1; ++t) {
        const int cnt = count(t);
        if (cnt > L) {
            const int len = piece_len(cnt), n = (cnt + len - 1) / len;
            red[t] = make_int2(cs, n);
            for (int i = 0; i < n; ++i, ++cs)
                plan[1 + cs] = make_int4(t, i * len, (i + 1) * len < cnt ? (i + 1) * len : cnt, 0);
        } else {
            red[t] = make_int2(-1, 1);
            plan[1 + cut_total + (mode == 0 ? wi : whole_total - 1 - wi)] = make_int4(t, 0, cnt, 0);
            ++wi;
        }
    }
}

int sparse_plan_launch(int mode, const int* ptr, int64_t n_tiles, int64_t N, int Hl, int slots_per_head, int target,
                       void* plan, void* red, void* stream) {
    sparse_plan_kernel<<<dim3(1), dim3(kPlanThreads), 0, (hipStream_t)stream>>>(
        mode, ptr, (int)n_tiles, (int)N, Hl, slots_per_head, target, (int4*)plan, (int2*)red);
    return hipGetLastError() == hipSuccess ? ULY_OK : ULY_ERR_LAUNCH;
}

// The same kind of plan for unmasked attention when one side has few tiles: every tile (key tile of
// dK/dV, query tile of dQ) walks cnt blocks of the other side and is cut into `pieces` items of `len`
// blocks, so plan and reduce table are closed forms.
__global__ __launch_bounds__(256) void dense_plan_kernel(int n_tiles, int cnt, int pieces, int len,
                                                         int4* __restrict__ plan, int2* __restrict__ red) {
    const int s = blockIdx.x * 256 + threadIdx.x;
    const int items = n_tiles * pieces;
    if (s == 0) plan[0] = make_int4(items, pieces > 1 ? items : 0, len, 0);
    if (s >= items) return;
    const int t = s / pieces, i = s - t * pieces;
    plan[1 + s] = make_int4(t, i * len, (i + 1) * len < cnt ? (i + 1) * len : cnt, 0);
    if (i == 0) red[t] = pieces > 1 ? make_int2(s, pieces) : make_int2(-1, 1);
}

// How n_tiles tiles that walk cnt blocks each are cut: only when the tiles alone would leave most of
// the 256 CUs idle and the walk is long enough to share out.
struct DenseCut {
    int pieces, len;
};
inline DenseCut dense_cut(int64_t n_tiles, int64_t cnt, int Hl) {
    DenseCut c{1, (int)cnt};
    if (n_tiles * Hl >= 512 || cnt < 2 * kPlanMinLen) return c;
    int64_t want = (kDenseCutTarget + n_tiles * Hl - 1) / (n_tiles * Hl);    // pieces that give about kDenseCutTarget items
    const int64_t most = cnt / kPlanMinLen;
    want = want < most ? want : most;
    if (want < 2) return c;
    const int64_t len = (((cnt + want - 1) / want) + 3) & ~(int64_t)3;
    c.len = (int)len;
    c.pieces = (int)((cnt + len - 1) / len);
    return c;
}

// Adds the partial sums of the cut tiles (fixed order: deterministic) and writes the NTENS outputs
// (dK and dV of a key tile, or dQ of a query tile; 128 rows per tile either way).
// Grid (any, heads): the workgroups of a head share out (cut item, 1024-float chunk) tasks; the task of
// a tile's first item does the tile, the others are skipped.
constexpr int kReduceBlocks = 256;
template <int D, int NTENS>
__global__ __launch_bounds__(256) void partial_reduce_kernel(const int4* __restrict__ plan, const int2* __restrict__ red,
                                                             const float* __restrict__ partial, int slots_per_head,
                                                             e16* __restrict__ out0, e16* __restrict__ out1, int n_rows,
                                                             int64_t row_stride, int64_t head_stride) {
    constexpr int ROWS = 128;
    constexpr int PER = ROWS * D;                         // floats per tensor and slot
    constexpr int CH = NTENS * PER / 1024;                // chunks per slot
    const int head = blockIdx.y;
    const int n_cut = plan[0].y;
    for (int t = blockIdx.x; t < n_cut * CH; t += gridDim.x) {
        const int s = t / CH, e = (t % CH) * 1024 + threadIdx.x * 4;
        const int4 it = plan[1 + s];
        if (it.y != 0) continue;                          // not the first item of its tile
        const int tile = it.x, n = red[tile].y;
        const float* base = partial + ((int64_t)head * slots_per_head + s) * (NTENS * PER) + e;
        f32x4 acc = *reinterpret_cast<const f32x4*>(base);
#pragma unroll 4
        for (int i = 1; i < n; ++i) acc += *reinterpret_cast<const f32x4*>(base + (int64_t)i * (NTENS * PER));
        const int which = e / PER, row = (e % PER) / D, ch = e % D;
        const int j = tile * ROWS + row;
        if (j >= n_rows) continue;
        e16x4 w;
#pragma unroll
        for (int c = 0; c < 4; ++c) w[c] = (e16)acc[c];
        e16* dst = (which ? out1 : out0) + (int64_t)head * head_stride + (int64_t)j * row_stride + ch;
        *reinterpret_cast<e16x4*>(dst) = w;
    }
}

// padded row stride of the statistics arrays in the workspace
inline int64_t stats_stride(int64_t N) { return ((N + 255) / 256) * 256 + 64; }   // covers whole sparse blocks

// Workspace of the block-sparse backward, in floats from its start: the two statistics arrays, then work
// plan, per-tile reduce table and partial sums of the dK/dV kernel and the same three of the dQ kernel
// (each section 256-byte aligned).
constexpr int kRowPlanTarget = 2048;      // items the cut block rows are aimed at (dQ), over all heads
struct SparseWorkspace {
    int64_t plan_at, red_at, partial_at, q_plan_at, q_red_at, q_partial_at, total;
    int64_t items_bound, q_items_bound;
    int slots_per_head, q_slots_per_head;
};
inline int row_slots_per_head(int64_t n_tiles, int target, int Hl) {
    const int64_t by_target = 2 * ((target + Hl - 1) / Hl), by_size = 4 * n_tiles + 1;    // at most four slots per tile
    return (int)(by_target < by_size ? by_target : by_size);
}
inline SparseWorkspace sparse_workspace(int64_t N, int Hl, int d) {
    const int64_t n_ktiles = (N + kDkvBK - 1) / kDkvBK, n_qtiles = (N + kDqBQ - 1) / kDqBQ;
    const int64_t nblk4 = (((N + kDkvBQ - 1) / kDkvBQ) + 3) & ~(int64_t)3;
    auto up = [](int64_t x) { return (x + 63) & ~(int64_t)63; };
    SparseWorkspace w;
    w.items_bound = plan_items_bound(n_ktiles, nblk4, Hl);
    w.slots_per_head = plan_slots_per_head(n_ktiles, nblk4, Hl);
    w.q_slots_per_head = row_slots_per_head(n_qtiles, kRowPlanTarget, Hl);
    w.q_items_bound = n_qtiles + w.q_slots_per_head + 1;
    w.plan_at = up(2 * stats_stride(N) * Hl);
    w.red_at = up(w.plan_at + 4 * (1 + w.items_bound));
    w.partial_at = up(w.red_at + 2 * n_ktiles);
    w.q_plan_at = up(w.partial_at + (int64_t)w.slots_per_head * Hl * 2 * kDkvBK * d);
    w.q_red_at = up(w.q_plan_at + 4 * (1 + w.q_items_bound));
    w.q_partial_at = up(w.q_red_at + 2 * n_qtiles);
    w.total = w.q_partial_at + (int64_t)w.q_slots_per_head * Hl * kDqBQ * d;
    return w;
}

// Workspace of the backward of unmasked attention whose tiles may be cut (cross-attention entry
// points): the statistics, then plan, reduce table and partial sums for dK/dV and for dQ (a side that
// is not cut takes no space).
struct CutWorkspace {
    DenseCut kv, q;                       // how key tiles (dK/dV) and query tiles (dQ) are cut
    int64_t kv_items, q_items;
    int64_t kv_plan_at, kv_red_at, kv_partial_at, q_plan_at, q_red_at, q_partial_at, total;
};
inline CutWorkspace cut_workspace(int64_t N, int64_t Nk, int Hl, int d) {
    const int64_t n_qtiles = (N + kDqBQ - 1) / kDqBQ, n_ktiles = (Nk + kDkvBK - 1) / kDkvBK;
    const int64_t q_blocks4 = (((N + kDkvBQ - 1) / kDkvBQ) + 3) & ~(int64_t)3;     // walked by a key tile
    const int64_t k_blocks4 = (((Nk + kDqBK - 1) / kDqBK) + 3) & ~(int64_t)3;      // walked by a query tile
    auto up = [](int64_t x) { return (x + 63) & ~(int64_t)63; };
    CutWorkspace w;
    w.kv = dense_cut(n_ktiles, q_blocks4, Hl);
    w.q = dense_cut(n_qtiles, k_blocks4, Hl);
    w.kv_items = n_ktiles * w.kv.pieces;
    w.q_items = n_qtiles * w.q.pieces;
    int64_t at = up(2 * stats_stride(N) * Hl);
    w.kv_plan_at = at;
    if (w.kv.pieces > 1) at = up(at + 4 * (1 + w.kv_items));
    w.kv_red_at = at;
    if (w.kv.pieces > 1) at = up(at + 2 * n_ktiles);
    w.kv_partial_at = at;
    if (w.kv.pieces > 1) at = up(at + w.kv_items * Hl * 2 * kDkvBK * d);
    w.q_plan_at = at;
    if (w.q.pieces > 1) at = up(at + 4 * (1 + w.q_items));
    w.q_red_at = at;
    if (w.q.pieces > 1) at = up(at + 2 * n_qtiles);
    w.q_partial_at = at;
    if (w.q.pieces > 1) at = up(at + w.q_items * Hl * kDqBQ * d);
    w.total = at;
    return w;
}

template <int D>
static int launch_bwd(int stage_mask, const void* q, const void* k, const void* v, const void* o, const void* dout,
                      const float* lse, void* dq, void* dk, void* dv, float* ws, int64_t N, int64_t Nk, int Hl,
                      float scale, int causal, bool may_cut, TensorStrides st, TensorStrides kv, hipStream_t stream) {
    const int64_t stride = stats_stride(N);
    float* delta = ws;
    float* lse2 = ws + stride * Hl;
    const int64_t delta_blocks = (stride * Hl * (D / 8) + 255) / 256;
    const int64_t n_qtiles = (N + kDqBQ - 1) / kDqBQ, n_ktiles = (Nk + kDkvBK - 1) / kDkvBK;
    if (delta_blocks > 0x7FFFFFFFll || n_qtiles * Hl > 0x7FFFFFFFll) return ULY_ERR_SHAPE;
    // unmasked attention with few tiles on one side (the workspace then has room for partial sums)
    CutWorkspace cw = cut_workspace(N, Nk, Hl, D);
    if (causal || !may_cut) cw.kv.pieces = cw.q.pieces = 1;
    if (cw.kv_items > 65535 || cw.q_items > 65535 || Hl > 65535) cw.kv.pieces = cw.q.pieces = 1;     // grid y dimensions
    const e16 *Q = (const e16*)q, *K = (const e16*)k, *V = (const e16*)v, *dO = (const e16*)dout;
    // causal: a workgroup takes a pair of key tiles (query tiles)
    const int64_t n_kwg = causal ? (n_ktiles + 1) / 2 : n_ktiles, n_qwg = causal ? (n_qtiles + 1) / 2 : n_qtiles;
    const dim3 gkv((uint32_t)(n_kwg * Hl)), gq((uint32_t)(n_qwg * Hl));

    if (stage_mask & 1) {
        attn_bwd_delta_kernel<D><<<dim3((uint32_t)delta_blocks), dim3(256), 0, stream>>>(
            (const e16*)o, dO, lse, delta, lse2, (int)N, Hl, stride, st.row, st.head);
        if (hipGetLastError() != hipSuccess) return ULY_ERR_LAUNCH;
    }
    if (stage_mask & 2) {
        if (causal)
            attn_bwd_dkv_kernel<D, true><<<gkv, dim3(kDkvThreads), 0, stream>>>(
                Q, K, V, dO, lse2, delta, stride, (e16*)dk, (e16*)dv, (int)N, (int)Nk, (int)n_ktiles, st.row, st.head,
                kv.head, scale, nullptr, nullptr, nullptr, nullptr, 0);
        else if (cw.kv.pieces > 1) {
            int4* plan = reinterpret_cast<int4*>(ws + cw.kv_plan_at);
            int2* red = reinterpret_cast<int2*>(ws + cw.kv_red_at);
            float* partial = ws + cw.kv_partial_at;
            const int q_blocks4 = (int)((((N + kDkvBQ - 1) / kDkvBQ) + 3) & ~(int64_t)3);
            dense_plan_kernel<<<dim3((uint32_t)((cw.kv_items + 255) / 256)), dim3(256), 0, stream>>>(
                (int)n_ktiles, q_blocks4, cw.kv.pieces, cw.kv.len, plan, red);
            if (hipGetLastError() != hipSuccess) return ULY_ERR_LAUNCH;
            attn_bwd_dkv_kernel<D, false, false, true>
                <<<dim3((uint32_t)Hl, (uint32_t)cw.kv_items), dim3(kDkvThreads), 0, stream>>>(
                    Q, K, V, dO, lse2, delta, stride, (e16*)dk, (e16*)dv, (int)N, (int)Nk, (int)n_ktiles, st.row, st.head,
                    kv.head, scale, nullptr, nullptr, plan, partial, (int)cw.kv_items);
            if (hipGetLastError() != hipSuccess) return ULY_ERR_LAUNCH;
            partial_reduce_kernel<D, 2><<<dim3(kReduceBlocks, (uint32_t)Hl), dim3(256), 0, stream>>>(
                plan, red, partial, (int)cw.kv_items, (e16*)dk, (e16*)dv, (int)Nk, kv.row, kv.head);
        } else
            attn_bwd_dkv_kernel<D, false><<<gkv, dim3(kDkvThreads), 0, stream>>>(
                Q, K, V, dO, lse2, delta, stride, (e16*)dk, (e16*)dv, (int)N, (int)Nk, (int)n_ktiles, st.row, st.head,
                kv.head, scale, nullptr, nullptr, nullptr, nullptr, 0);
        if (hipGetLastError() != hipSuccess) return ULY_ERR_LAUNCH;
    }
    if (stage_mask & 4) {
        if (causal)
            attn_bwd_dq_kernel<D, true><<<gq, dim3(kDqThreads), 0, stream>>>(
                Q, K, V, dO, lse2, delta, stride, (e16*)dq, (int)N, (int)Nk, (int)n_qtiles, st.row, st.head, kv.head, scale,
                nullptr, nullptr, nullptr, nullptr, 0);
        else if (cw.q.pieces > 1) {
            int4* plan = reinterpret_cast<int4*>(ws + cw.q_plan_at);
            int2* red = reinterpret_cast<int2*>(ws + cw.q_red_at);
            float* partial = ws + cw.q_partial_at;
            const int k_blocks4 = (int)((((Nk + kDqBK - 1) / kDqBK) + 3) & ~(int64_t)3);
            dense_plan_kernel<<<dim3((uint32_t)((cw.q_items + 255) / 256)), dim3(256), 0, stream>>>(
                (int)n_qtiles, k_blocks4, cw.q.pieces, cw.q.len, plan, red);
            if (hipGetLastError() != hipSuccess) return ULY_ERR_LAUNCH;
            attn_bwd_dq_kernel<D, false, false, true>
                <<<dim3((uint32_t)Hl, (uint32_t)cw.q_items), dim3(kDqThreads), 0, stream>>>(
                    Q, K, V, dO, lse2, delta, stride, (e16*)dq, (int)N, (int)Nk, (int)n_qtiles, st.row, st.head, kv.head,
                    scale, nullptr, nullptr, plan, partial, (int)cw.q_items);
            if (hipGetLastError() != hipSuccess) return ULY_ERR_LAUNCH;
            partial_reduce_kernel<D, 1><<<dim3(kReduceBlocks, (uint32_t)Hl), dim3(256), 0, stream>>>(
                plan, red, partial, (int)cw.q_items, (e16*)dq, nullptr, (int)N, st.row, st.head);
        } else
            attn_bwd_dq_kernel<D, false><<<gq, dim3(kDqThreads), 0, stream>>>(
                Q, K, V, dO, lse2, delta, stride, (e16*)dq, (int)N, (int)Nk, (int)n_qtiles, st.row, st.head, kv.head, scale,
                nullptr, nullptr, nullptr, nullptr, 0);
        if (hipGetLastError() != hipSuccess) return ULY_ERR_LAUNCH;
    }
    return ULY_OK;
}

// Block-sparse causal backward (all three stages): one key tile / query tile per workgroup.
template <int D>
static int launch_bwd_sparse(const void* q, const void* k, const void* v, const void* o, const void* dout,
                             const float* lse, void* dq, void* dk, void* dv, float* ws, const int* row_ptr,
                             const int* col_idx, const int* col_ptr, const int* row_idx, int64_t N, int Hl, float scale,
                             TensorStrides st, hipStream_t stream) {
    const int64_t stride = stats_stride(N);
    float* delta = ws;
    float* lse2 = ws + stride * Hl;
    const int64_t delta_blocks = (stride * Hl * (D / 8) + 255) / 256;
    const int64_t n_qtiles = (N + kDqBQ - 1) / kDqBQ, n_ktiles = (N + kDkvBK - 1) / kDkvBK;
    if (delta_blocks > 0x7FFFFFFFll || n_qtiles * Hl > 0x7FFFFFFFll) return ULY_ERR_SHAPE;
    const e16 *Q = (const e16*)q, *K = (const e16*)k, *V = (const e16*)v, *dO = (const e16*)dout;
    attn_bwd_delta_kernel<D><<<dim3((uint32_t)delta_blocks), dim3(256), 0, stream>>>(
        (const e16*)o, dO, lse, delta, lse2, (int)N, Hl, stride, st.row, st.head);
    if (hipGetLastError() != hipSuccess) return ULY_ERR_LAUNCH;
    // work plan, then the items, then the sums of the cut columns
    const SparseWorkspace w = sparse_workspace(N, Hl, D);
    if (w.items_bound > 65535 || w.q_items_bound > 65535 || Hl > 65535) return ULY_ERR_SHAPE;      // grid y dimensions
    int4* plan = reinterpret_cast<int4*>(ws + w.plan_at);
    int2* red = reinterpret_cast<int2*>(ws + w.red_at);
    float* partial = ws + w.partial_at;
    if (sparse_plan_launch(0, col_ptr, n_ktiles, N, Hl, w.slots_per_head, kPlanTarget, plan, red, stream) != ULY_OK)
        return ULY_ERR_LAUNCH;
    attn_bwd_dkv_kernel<D, true, true><<<dim3((uint32_t)Hl, (uint32_t)w.items_bound), dim3(kDkvThreads), 0, stream>>>(
        Q, K, V, dO, lse2, delta, stride, (e16*)dk, (e16*)dv, (int)N, (int)N, (int)n_ktiles, st.row, st.head, st.head,
        scale, col_ptr, row_idx, plan, partial, w.slots_per_head);
    if (hipGetLastError() != hipSuccess) return ULY_ERR_LAUNCH;
    partial_reduce_kernel<D, 2><<<dim3(kReduceBlocks, (uint32_t)Hl), dim3(256), 0, stream>>>(
        plan, red, partial, w.slots_per_head, (e16*)dk, (e16*)dv, (int)N, st.row, st.head);
    if (hipGetLastError() != hipSuccess) return ULY_ERR_LAUNCH;
    // the same for the block rows of the dQ kernel
    int4* q_plan = reinterpret_cast<int4*>(ws + w.q_plan_at);
    int2* q_red = reinterpret_cast<int2*>(ws + w.q_red_at);
    float* q_partial = ws + w.q_partial_at;
    if (sparse_plan_launch(1, row_ptr, n_qtiles, N, Hl, w.q_slots_per_head, kRowPlanTarget, q_plan, q_red, stream) != ULY_OK)
        return ULY_ERR_LAUNCH;
    attn_bwd_dq_kernel<D, true, true, true>
        <<<dim3((uint32_t)Hl, (uint32_t)w.q_items_bound), dim3(kDqThreads), 0, stream>>>(
            Q, K, V, dO, lse2, delta, stride, (e16*)dq, (int)N, (int)N, (int)n_qtiles, st.row, st.head, st.head, scale,
            row_ptr, col_idx, q_plan, q_partial, w.q_slots_per_head);
    if (hipGetLastError() != hipSuccess) return ULY_ERR_LAUNCH;
    partial_reduce_kernel<D, 1><<<dim3(kReduceBlocks, (uint32_t)Hl), dim3(256), 0, stream>>>(
        q_plan, q_red, q_partial, w.q_slots_per_head, (e16*)dq, nullptr, (int)N, st.row, st.head);
    return hipGetLastError() == hipSuccess ? ULY_OK : ULY_ERR_LAUNCH;
}

int attn_bwd_sparse_launch(const void* q, const void* k, const void* v, const void* o, const void* dout,
                           const float* lse, void* dq, void* dk, void* dv, float* ws, const int* row_ptr,
                           const int* col_idx, const int* col_ptr, const int* row_idx, int64_t N, int Hl, int d,
                           float scale, TensorStrides st, void* stream) {
    if (d == 128)
        return launch_bwd_sparse<128>(q, k, v, o, dout, lse, dq, dk, dv, ws, row_ptr, col_idx, col_ptr, row_idx, N, Hl,
                                      scale, st, (hipStream_t)stream);
    return launch_bwd_sparse<64>(q, k, v, o, dout, lse, dq, dk, dv, ws, row_ptr, col_idx, col_ptr, row_idx, N, Hl, scale,
                                 st, (hipStream_t)stream);
}

int64_t attn_bwd_workspace_floats(int64_t N, int Hl) { return 2 * stats_stride(N) * Hl; }
int64_t attn_bwd_sparse_workspace_floats(int64_t N, int Hl, int d) { return sparse_workspace(N, Hl, d).total; }

int64_t attn_bwd_cut_workspace_floats(int64_t N, int64_t Nk, int Hl, int d) {
    if (d == 256) return attn_bwd_workspace_floats(N, Hl);      // the d = 256 kernels do not cut
    return cut_workspace(N, Nk, Hl, d).total;
}

int attn_bwd_launch(int stage_mask, const void* q, const void* k, const void* v, const void* o, const void* dout,
                    const float* lse, void* dq, void* dk, void* dv, float* ws, int64_t N, int64_t Nk, int Hl, int d,
                    float scale, int causal, int may_cut, TensorStrides st, TensorStrides kv, void* stream) {
    if (d == 256) {
        const int64_t stride = stats_stride(N);
        float* delta = ws;
        float* lse2 = ws + stride * Hl;
        if (stage_mask & 1) {
            const int64_t delta_blocks = (stride * Hl * (256 / 8) + 255) / 256;
            if (delta_blocks > 0x7FFFFFFFll) return ULY_ERR_SHAPE;
            attn_bwd_delta_kernel<256><<<dim3((uint32_t)delta_blocks), dim3(256), 0, (hipStream_t)stream>>>(
                (const e16*)o, (const e16*)dout, lse, delta, lse2, (int)N, Hl, stride, st.row, st.head);
            if (hipGetLastError() != hipSuccess) return ULY_ERR_LAUNCH;
        }
        return attn256_bwd_launch(stage_mask, q, k, v, dout, delta, lse2, stride, dq, dk, dv, N, Nk, Hl, scale, causal, st,
                                  kv, stream);
    }
    if (d == 128)
        return launch_bwd<128>(stage_mask, q, k, v, o, dout, lse, dq, dk, dv, ws, N, Nk, Hl, scale, causal, may_cut != 0,
                               st, kv, (hipStream_t)stream);
    return launch_bwd<64>(stage_mask, q, k, v, o, dout, lse, dq, dk, dv, ws, N, Nk, Hl, scale, causal, may_cut != 0, st,
                          kv, (hipStream_t)stream);
}

}  // namespace ULY_ELEM_NS
}  // namespace uly
