// Forward pass of exact softmax attention (paper Equation 1, causal variant of Section 3.4)
// for the local heads of one GPU: tiled online softmax, 16-bit (bf16 or fp16) MFMA, fp32 accumulation.
//
// Work decomposition: one workgroup (8 waves) owns 256 consecutive queries of one head; each wave
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
#include <type_traits>

#include "attn_common.h"
#include "internal.h"

namespace uly {
namespace ULY_ELEM_NS {

constexpr int kFwdThreads = 512;
constexpr int kFwdWaves = 8;
constexpr int kFwdBQ = 256;   // queries per workgroup
constexpr int kFwdBK = 64;    // keys per LDS tile
// Causal work assignment.  true: a workgroup takes a query tile and then its mirror image (equal work
// per workgroup, K/V stream shared in L2: 12x less traffic beyond L2 at N = 128K).  false: one tile
// per workgroup, heaviest first.  Measured on MI355X the forward kernel is 4% faster with false: two
// workgroups share a CU, and when all of them walk in step their softmax and MFMA phases collide.
constexpr bool kFwdPair = false;

// SPARSE (causal only): the keys a query tile sees are further restricted to the 256-key blocks listed for
// its block row in a CSR pattern (row_ptr, col_idx: ascending block columns, the diagonal one last); a
// query tile is exactly one block row.  Dense kernels ignore the two pointers.
constexpr int kSparseBlock = 256;
static_assert(kFwdBQ == kSparseBlock && kSparseBlock % kFwdBK == 0, "a query tile must be one sparse block row");

// CUT: grid (heads, work items); a workgroup takes a range of the key tiles of its query tile and, when the
// tile has several such items, writes instead of O and LSE what the combine kernel needs to merge them:
// the unnormalised fp32 accumulators and, per query, the maximum the exponentials were taken against and
// the sum of the exponentials.
//   unmasked attention with few query tiles: item = query tile x piece of `cut_len` tiles (closed form);
//   block-sparse, and dense causal with few query tiles: items come from a device-made plan (long rows are cut,
//   see sparse_plan_launch).
//   part_o [head][slot][256 queries][D] fp32,   part_ml [head][slot][256 queries][2] fp32 (max, sum)
template <int D, bool CAUSAL, bool SPARSE = false, bool CUT = false>
__global__ __launch_bounds__(kFwdThreads, 1) void attn_fwd_kernel(const e16* __restrict__ Q, const e16* __restrict__ K,
                                                                   const e16* __restrict__ V, e16* __restrict__ O,
                                                                   float* __restrict__ LSE, int N, int Nk, int n_qtiles,
                                                                   int64_t row_stride, int64_t head_stride, int64_t kv_head_stride,
                                                                   float scale, const int* __restrict__ row_ptr,
                                                                   const int* __restrict__ col_idx, int cut_pieces,
                                                                   int cut_len, float* __restrict__ part_o,
                                                                   float* __restrict__ part_ml,
                                                                   const int4* __restrict__ plan, int slots_per_head) {
    static_assert(!SPARSE || CAUSAL, "the sparse pattern refines the causal mask");
    constexpr int NT = D / 16;              // contraction steps over the head dim
    constexpr int NCB = D / 32;             // 32-channel blocks of the output
    constexpr int TILE = kFwdBK * D;        // elements per LDS tile
    constexpr int TB = TILE * 2;            // bytes per LDS tile
    constexpr int BLK = 32 * D * 2;         // bytes per 32-key block inside a tile
    constexpr int HALF = 16 * D * 2;        // bytes per 16 keys
    // byte offsets of the four tile buffers inside one LDS object: K0 K1 V0 V1
    constexpr int K0 = 0, K1 = TB, V0 = 2 * TB, V1 = 3 * TB;
    using KLoader = DirectTile<D, kFwdBK, kFwdWaves, SwzBoth>;     // K: row reads
    using VLoader = DirectTile<D, kFwdBK, kFwdWaves, SwzTr>;       // V: transposing reads only

    // The last NQL of the NT query operand chunks live in LDS instead of registers (the kernel is a few
    // registers short of keeping all of Q, the O accumulators and one block of operands resident).
    constexpr int NQL = (D == 128) ? 2 : 0;
    constexpr int NQR = NT - NQL;
    constexpr int QROW = NQL * 32 + 16;      // bytes per query row in LDS, padded: conflict-free row reads
    __shared__ __attribute__((aligned(1024))) e16 smem[4 * TILE];
    __shared__ __attribute__((aligned(16))) char q_lds[NQL ? kFwdBQ * QROW : 16];

    const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5, ln = lane & 31;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // uniform: keeps wave-derived addresses scalar
    // Work assignment (causal): a workgroup takes query tile n_qtiles-1-pr and then its mirror image
    // pr, so every workgroup does the same amount of work.  It walks the key tiles of the first
    // upwards from the start of the sequence and those of the second downwards from its diagonal: at
    // any moment all workgroups that started together read one of only two key tiles, which keeps
    // the K/V stream in the L2 caches instead of re-fetching it per workgroup.
    const int n_pairs = (CAUSAL && kFwdPair && !SPARSE) ? (n_qtiles + 1) / 2 : n_qtiles;
    const int head = CUT ? blockIdx.x : blockIdx.x / n_pairs;
    int pr = blockIdx.x - head * n_pairs;
    int t_off = 0, t_len = 0, slot = -1;          // CUT: first key tile (walk position) of this item, their number
    if (CUT && CAUSAL) {                          // block-sparse or dense causal: items of uneven length, from a plan
        const int4 hdr = plan[0];                 // {items, items that write partial results, ..}
        if ((int)blockIdx.y >= hdr.x) return;     // the grid is an upper bound on the number of items
        const int4 it = plan[1 + blockIdx.y];     // {query tile, first walk position, end, -}
        pr = it.x;
        t_off = it.y;
        t_len = it.z - it.y;
        slot = (int)blockIdx.y < hdr.y ? (int)blockIdx.y : -1;
    } else if (CUT) {
        pr = blockIdx.y / cut_pieces;
        t_off = (blockIdx.y - pr * cut_pieces) * cut_len;
        t_len = cut_len;
        slot = blockIdx.y;
    }
    const int64_t hoff = (int64_t)head * head_stride;
    const e16* Qh = Q + hoff;
    // N queries attend to Nk keys (Nk = N for self-attention); K and V may have their own head stride
    const e16* Kh = K + (int64_t)head * kv_head_stride;
    const e16* Vh = V + (int64_t)head * kv_head_stride;

    const typename KLoader::LaneOffsets k_ld = KLoader::lane_offsets(row_stride, wave, lane);
    const typename VLoader::LaneOffsets v_ld = VLoader::lane_offsets(row_stride, wave, lane);
    auto load_tile = [&](int kbuf, int vbuf, int kt) __attribute__((always_inline)) {     // buffer byte offsets
        const int r0 = kt * kFwdBK;
        if (r0 + kFwdBK <= Nk) {
            KLoader::issue(smem + kbuf / 2, Kh + (int64_t)r0 * row_stride, k_ld, wave);
            VLoader::issue(smem + vbuf / 2, Vh + (int64_t)r0 * row_stride, v_ld, wave);
        } else {
            KLoader::issue_clamped(smem + kbuf / 2, Kh, row_stride, r0, Nk, wave, lane);
            VLoader::issue_clamped(smem + vbuf / 2, Vh, row_stride, r0, Nk, wave, lane);
        }
    };
    // per-lane LDS byte addresses inside a tile (buffer, block and half-block offsets are immediates)
    const uint32_t sbase = lds_addr(smem);
    // row read of K: row ln, chunk 2t+g.  The swizzle is an XOR on the chunk index and 2t, g occupy
    // different bits of it, so the address of chunk 2t+g is that of chunk g with t XORed in: one
    // register instead of NT, at one VALU instruction per read.
    const uint32_t k_adr0 = sbase + 2 * tile_off<D>(ln, g);
    uint32_t v_adr[NCB];                // transposing read of V: rows 4g+(i>>2) (+8: immediate), channels 32cb+16h+4(i&3)
    {
        const int i = lane & 15, h = (lane >> 4) & 1;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
            v_adr[cb] = sbase + 2 * (tile_off<D, SwzTr>(4 * g + (i >> 2), 4 * cb + 2 * h + ((i & 3) >> 1)) + 4 * (i & 1));
    }
    constexpr int ROW8 = 8 * D * 2;     // bytes between the two 4-row groups of a transposing operand

    const float sl2 = scale * kLog2e;

    const int n_parts = (CAUSAL && kFwdPair && !SPARSE && n_qtiles - 1 - pr != pr) ? 2 : 1;
#pragma unroll 1
    for (int part = 0; part < n_parts; ++part) {
    const int qt = (!CUT && CAUSAL && part == 0) ? n_qtiles - 1 - pr : pr;
    const int dir = part == 0 ? 1 : -1;                        // walking direction over the key tiles
    const int q0 = qt * kFwdBQ;
    int k_end = Nk;
    if (CAUSAL) { const int lim = q0 + kFwdBQ; k_end = lim < Nk ? lim : Nk; }
    constexpr int TPB = kSparseBlock / kFwdBK;                 // key tiles per sparse block
    int n_kt = (k_end + kFwdBK - 1) / kFwdBK;
    int sp0 = 0;                                               // first entry of this block row in col_idx
    if (SPARSE) {
        sp0 = row_ptr[qt];
        // every listed block but the last (the diagonal one) is entirely visible: TPB tiles each
        n_kt = TPB * (row_ptr[qt + 1] - sp0 - 1) + (k_end - q0 + kFwdBK - 1) / kFwdBK;
    }
    if (CUT) n_kt = n_kt - t_off < t_len ? n_kt - t_off : t_len;
    auto tile_of = [&](int pos) __attribute__((always_inline)) {
        if (SPARSE) return TPB * col_idx[sp0 + (pos + t_off) / TPB] + (pos + t_off) % TPB;
        if (CUT) return t_off + pos;
        return dir > 0 ? pos : n_kt - 1 - pos;
    };
    load_tile(K0, V0, tile_of(0));
    if (n_kt > 1) load_tile(K1, V1, tile_of(1));

    // (an opaque copy of the thread id: the address arithmetic of this once-per-tile set-up must not be
    // hoisted out of the loop over query tiles, where it would stay live across the hot loop)
    int tid_p = tid;
    asm volatile("" : "+v"(tid_p));
    const int wave_p = wave, g_p = (tid_p >> 5) & 1, ln_p = tid_p & 31;
    const int q_row = q0 + wave_p * 32 + ln_p;                 // this lane's query
    const int q_ld = q_row < N ? q_row : N - 1;
    e16x8 qreg[NQR];
#pragma unroll
    for (int t = 0; t < NQR; ++t)
        qreg[t] = *reinterpret_cast<const e16x8*>(Qh + (int64_t)q_ld * row_stride + 16 * t + 8 * g_p);
    const uint32_t q_adr = lds_addr(q_lds) + (wave_p * 32 + ln_p) * QROW + g_p * 16;
#pragma unroll
    for (int t = NQR; t < NT; ++t)      // only this wave reads these rows back: no barrier needed
        *reinterpret_cast<e16x8*>(q_lds + (wave_p * 32 + ln_p) * QROW + (2 * (t - NQR) + g_p) * 16) =
            *reinterpret_cast<const e16x8*>(Qh + (int64_t)q_ld * row_stride + 16 * t + 8 * g_p);


    float m_used = -INFINITY;    // reference maximum (raw logits) that the exponentials are taken against
    float l_run = 0.f;           // this lane's share of the running sum
    f32x16 oacc[NCB];
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[cb][r] = 0.f;

    // K operands of one 32-key block.  The first half is read one phase ahead (during the PV MFMAs of
    // the previous block), the second half at the start of the block itself, behind the first half's
    // MFMAs: only half of them are live while the register pressure peaks.
    e16x8 ka[NT];
    auto read_k = [&](auto off_tag, auto half_tag) __attribute__((always_inline)) {
        constexpr int OFF = decltype(off_tag)::value;
        constexpr int H = decltype(half_tag)::value;
        uint32_t a0 = k_adr0;
        asm volatile("" : "+v"(a0));          // keeps the XORed addresses from being precomputed and kept live
#pragma unroll
        for (int t = H * (NT / 2); t < (H + 1) * (NT / 2); ++t) ka[t] = lds_b128<OFF>(a0 ^ (uint32_t)(t << 5));
    };
    auto wait_k = [&](auto half_tag) __attribute__((always_inline)) {
        constexpr int H = decltype(half_tag)::value;
        if constexpr (NT / 2 == 4) {
            lds_wait<0>(ka[4 * H], ka[4 * H + 1], ka[4 * H + 2], ka[4 * H + 3]);
        } else {
            lds_wait<0>(ka[2 * H], ka[2 * H + 1]);
        }
    };
    using First = std::integral_constant<int, 0>;
    using Second = std::integral_constant<int, 1>;

    // tile 0 was issued first: wait for it alone (the loads of tile 1 may still be in flight)
    if (n_kt > 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * KLoader::kPerWave) : "memory");
    else wait_direct_loads();
    __syncthreads();
    read_k(std::integral_constant<int, K0>{}, First{});
    wait_k(First{});                    // before the loops are entered: at a join the compiler may copy these registers

    // One 32-key block: S^T (K operands already on their way) -> read V of the first 16 keys -> softmax
    // -> read the next block's K -> PV of the first 16 keys -> read V of the last 16 keys -> PV of those.
    // In the last block of a tile the barrier, the loads of the tile two positions on and the K reads of the next tile sit
    // just before the last PV: by then every wave has finished reading this tile's buffers.
    auto do_block = [&](auto masked_tag, auto kb_tag, auto vb_tag, auto kn_tag, auto kfree_tag, auto vfree_tag, int kb0,
                        int pos)
                        __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        constexpr int VB = decltype(vb_tag)::value;        // this block's V rows
        constexpr int KFREE = decltype(kfree_tag)::value;  // >= 0: last block of a tile; buffers to refill
        constexpr int VFREE = decltype(vfree_tag)::value;
        constexpr bool LAST = KFREE >= 0;

        wait_k(First{});
        read_k(kb_tag, Second{});
        e16x8 ql[NQL ? NQL : 1];
        if constexpr (NQL == 2) {
            ql[0] = lds_b128<0>(q_adr);
            ql[1] = lds_b128<32>(q_adr);
        }
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int t = 0; t < NT / 2; ++t) s = mfma32(ka[t], qreg[t], s);
        wait_k(Second{});
        if constexpr (NQL == 2) lds_wait<0>(ql[0], ql[1]);
#pragma unroll
        for (int t = NT / 2; t < NT; ++t) s = mfma32(ka[t], t < NQR ? qreg[t < NQR ? t : 0] : ql[t >= NQR ? t - NQR : 0], s);
        __builtin_amdgcn_sched_barrier(0);      // the reads below reuse ka: keep them behind the MFMAs

        // V operands of the first 16 keys: they arrive during the softmax
        e16x4 vlo[NCB], vhi[NCB];
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
            vlo[cb] = lds_tr_b64<VB>(v_adr[cb]);
            vhi[cb] = lds_tr_b64<VB + ROW8>(v_adr[cb]);
        }

        if (MASKED) {
            // key kb0 + c_r + 4g (c_r = 8*(r/4) + r%4) is visible iff it is <= jmax: one limit per block
            const int jmax = CAUSAL ? (q_row < Nk - 1 ? q_row : Nk - 1) : Nk - 1;
            const int lim = jmax - kb0 - 4 * g;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (8 * (r >> 2) + (r & 3) > lim) s[r] = -INFINITY;
        }
        // online softmax; the rescale runs only when some row of this wave has a new maximum
        float m_blk = s[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) m_blk = fmaxf(m_blk, s[r]);
        m_blk = xhalf_max(m_blk);
        if (__builtin_amdgcn_ballot_w64(m_blk > m_used) != 0) {      // always taken on the first block
            const float m_new = fmaxf(m_used, m_blk);
            const float m_fin = (m_new == -INFINITY) ? 0.f : m_new;  // a row with nothing visible yet
            const float alpha = fast_exp2((m_used - m_fin) * sl2);
            l_run *= alpha;
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[cb][r] *= alpha;
            m_used = m_new;
        }
        const float ms = (m_used == -INFINITY ? 0.f : m_used) * sl2;
        float rs0 = 0.f, rs1 = 0.f;
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            s[r] = fast_exp2(__builtin_fmaf(s[r], sl2, -ms));
            s[r + 1] = fast_exp2(__builtin_fmaf(s[r + 1], sl2, -ms));
            rs0 += s[r];
            rs1 += s[r + 1];
        }
        l_run += rs0 + rs1;

        // O^T += V^T P^T, 16 keys at a time.  MASKED: rows with few visible keys are where |O| is largest
        // and where rounding P to 16 bits would be the dominant error, so diagonal blocks carry P in two
        // 16-bit pieces (hi + lo).
        auto pv_half = [&](int u) __attribute__((always_inline)) {
            const e16x8 pb = pack_b_operand(s, u);
            e16x8 plo;
            if (MASKED) {
#pragma unroll
                for (int e = 0; e < 8; ++e) plo[e] = (e16)(s[8 * u + e] - (float)pb[e]);
            }
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) {
                const e16x8 va = __builtin_shufflevector(vlo[cb], vhi[cb], 0, 1, 2, 3, 4, 5, 6, 7);
                oacc[cb] = mfma32(va, pb, oacc[cb]);
                if (MASKED) oacc[cb] = mfma32(va, plo, oacc[cb]);
            }
        };
        auto wait_v = [&]() __attribute__((always_inline)) {
#pragma unroll
            for (int cb = 0; cb < NCB; cb += 2) lds_wait<0>(vlo[cb], vhi[cb], vlo[cb + 1], vhi[cb + 1]);
        };
        auto read_v_second = [&]() __attribute__((always_inline)) {
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) {
                vlo[cb] = lds_tr_b64<VB + HALF>(v_adr[cb]);
                vhi[cb] = lds_tr_b64<VB + HALF + ROW8>(v_adr[cb]);
            }
        };
        wait_v();
        if (!LAST) read_k(kn_tag, First{});  // arrives while the PV MFMAs run; not live during the softmax
        pv_half(0);
        __builtin_amdgcn_sched_barrier(0);  // the second half reuses the V registers of the first
        read_v_second();
        wait_v();
        if (LAST) {
            // every wave is done reading this tile's buffers once it gets here
            wait_direct_loads();
            __syncthreads();
            if (pos + 2 < n_kt) load_tile(KFREE, VFREE, tile_of(pos + 2));
            if (pos + 1 < n_kt) read_k(kn_tag, First{});
        }
        pv_half(1);
        if (LAST) {
            // The K reads for the next tile were issued eight MFMAs ago.  They are waited for here, before
            // control flow joins again (end of the tile, loop edges), because at a join the compiler may copy
            // registers without knowing that a hand-issued read into them is still on its way.
            __builtin_amdgcn_sched_barrier(0);
            wait_k(First{});
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // Blocks entirely below the diagonal for every wave and inside the sequence need no mask.
    int n_full = Nk / kFwdBK;
    if (CAUSAL) { const int lim = q0 / kFwdBK; n_full = lim < n_full ? lim : n_full; }
    using Plain = std::integral_constant<bool, false>;
    using Masked = std::integral_constant<bool, true>;
    using None = std::integral_constant<int, -1>;
#define ULY_IC(x) std::integral_constant<int, (x)> {}
    auto tile_even = [&](auto mt, int pos) __attribute__((always_inline)) {      // tile in K0/V0, next in K1/V1
        const int kb0 = tile_of(pos) * kFwdBK;
        do_block(mt, ULY_IC(K0), ULY_IC(V0), ULY_IC(K0 + BLK), None{}, None{}, kb0, pos);
        do_block(mt, ULY_IC(K0 + BLK), ULY_IC(V0 + BLK), ULY_IC(K1), ULY_IC(K0), ULY_IC(V0), kb0 + 32, pos);
    };
    auto tile_odd = [&](auto mt, int pos) __attribute__((always_inline)) {
        const int kb0 = tile_of(pos) * kFwdBK;
        do_block(mt, ULY_IC(K1), ULY_IC(V1), ULY_IC(K1 + BLK), None{}, None{}, kb0, pos);
        do_block(mt, ULY_IC(K1 + BLK), ULY_IC(V1 + BLK), ULY_IC(K0), ULY_IC(K1), ULY_IC(V1), kb0 + 32, pos);
    };
#undef ULY_IC
    // Walk position `pos` holds key tile tile_of(pos) in buffer pos % 2.  Pairs of unmasked tiles run in
    // the branch-free loop; whatever precedes them (walking down: the diagonal comes first) and whatever
    // follows (walking up: the diagonal and the end of the sequence come last) goes one tile at a time.
    auto pair_ok = [&](int pos) __attribute__((always_inline)) {
        return (pos & 1) == 0 && pos + 1 < n_kt && tile_of(pos) < n_full && tile_of(pos + 1) < n_full;
    };
    int pos = 0;
#pragma unroll 1
    for (int phase = 0; phase < 2; ++phase) {
        for (; pos < n_kt && !pair_ok(pos); ++pos) {
            const bool plain = tile_of(pos) < n_full;
            if (pos & 1) { if (plain) tile_odd(Plain{}, pos); else tile_odd(Masked{}, pos); }
            else { if (plain) tile_even(Plain{}, pos); else tile_even(Masked{}, pos); }
        }
        if (phase == 0) {
            for (; pair_ok(pos); pos += 2) {
                tile_even(Plain{}, pos);
                tile_odd(Plain{}, pos + 1);
            }
            // The K reads issued for the next tile must have landed before control leaves the loop: the
            // compiler may spill or copy their registers there, unaware that they are still in flight.
            wait_k(First{});
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // ---- epilogue: normalise, store O (element type) and LSE (natural log)
    const float l_tot = xhalf_sum(l_run);
    const float inv = 1.f / l_tot;
    if (CUT && slot >= 0) {
        const int64_t at = (int64_t)head * slots_per_head + slot;
        const int row = wave * 32 + ln;
        float* prow = part_o + (at * kFwdBQ + row) * D;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                f32x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = oacc[cb][4 * rq + e];
                *reinterpret_cast<f32x4*>(prow + 32 * cb + 8 * rq + 4 * g) = w;
            }
        if (g == 0) {
            part_ml[(at * kFwdBQ + row) * 2] = m_used;
            part_ml[(at * kFwdBQ + row) * 2 + 1] = l_tot;
        }
    } else if (q_row < N) {
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
    __syncthreads();             // every wave is done with the tile buffers before the next query tile refills them
    }   // query tiles of this workgroup
}

// ------------------------------------------------------------------------------------------
// Forward for d = 128 with 64 queries per wave.  The kernel above takes one operand of every MFMA
// from LDS (1 KiB per wave and MFMA), which at the full matrix rate is the whole LDS bandwidth of a
// CU.  Here a lane owns two queries (two 32-query column blocks), so every K row operand and every
// V^T operand read from LDS feeds two MFMAs.  That takes 128 accumulator + 64 Q-operand registers,
// so it runs one wave per SIMD (4 waves = 256 queries per workgroup, one workgroup per CU) and
// overlaps its vector work with its matrix work inside the wave.  Iteration p:
//     region A   matrix: S^T of block p+1              vector: exponentials of block p (10 of its 16 score pairs)
//     region B   matrix: O^T += V^T P^T of block p-1   vector: the other exponentials, row maxima of block p+1
// The product with V lags one block behind the exponentials so that neither region waits for the
// vector unit.  K and V stream through rings of four 32-key LDS tiles.  The reference maximum of a
// row moves only when a score exceeds it by more than kQ64Lazy in the exponent (it need not be the true
// maximum: the result does not depend on it), which after the first blocks is practically never.
// ------------------------------------------------------------------------------------------
constexpr int kQ64Threads = 256;
constexpr int kQ64BK = 32;
constexpr int kQ64Ring = 4;
constexpr float kQ64Lazy = 8.f;

// CUT: grid (heads, work items); an item is a query tile and a range of its 64-key tiles, from a device-made
// plan (causal) or in equal pieces (no mask), as for attn_fwd_kernel; items of a cut tile write fp32 partial
// results (unnormalised O, reference maximum, sum) that attn_fwd_combine_kernel merges.
template <bool CAUSAL, bool CUT = false>
__global__ __launch_bounds__(kQ64Threads, 1) void attn_fwd_q64_kernel(
    const e16* __restrict__ Q, const e16* __restrict__ K, const e16* __restrict__ V, e16* __restrict__ O,
    float* __restrict__ LSE, int N, int Nk, int n_qtiles, int64_t row_stride, int64_t head_stride,
    int64_t kv_head_stride, float scale, int cut_pieces, int cut_len, float* __restrict__ part_o,
    float* __restrict__ part_ml, const int4* __restrict__ plan, int slots_per_head) {
    constexpr int D = 128, NT = D / 16, NCB = D / 32;
    constexpr int TILE = kQ64BK * D, TB = TILE * 2;
    constexpr int KB = 0, VB = kQ64Ring * TB;       // byte offsets of the K ring and the V ring
    constexpr int HALF = 16 * D * 2;
    using Loader = DirectTile<D, kQ64BK, 4, SwzBoth>;
    constexpr int LPT = 2 * Loader::kPerWave;       // global loads per wave and iteration (one K tile, one V tile)

    __shared__ __attribute__((aligned(1024))) e16 smem[2 * kQ64Ring * TILE];

    const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5, ln = lane & 31;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // uniform: LDS tile addresses stay scalar
    const int head = CUT ? blockIdx.x : blockIdx.x / n_qtiles;
    int qt = n_qtiles - 1 - (blockIdx.x - head * n_qtiles);            // causal: the longest tiles start first
    int t_off = 0, t_len = 0, slot = -1;          // CUT: first 64-key tile of this item, their number, partial-result slot
    if (CUT && CAUSAL) {
        const int4 hdr = plan[0];                 // {items, items that write partial results, ..}
        if ((int)blockIdx.y >= hdr.x) return;     // the grid is an upper bound on the number of items
        const int4 it = plan[1 + blockIdx.y];     // {query tile, first tile, end, -}
        qt = it.x;
        t_off = it.y;
        t_len = it.z - it.y;
        slot = (int)blockIdx.y < hdr.y ? (int)blockIdx.y : -1;
    } else if (CUT) {
        qt = blockIdx.y / cut_pieces;
        t_off = (blockIdx.y - qt * cut_pieces) * cut_len;
        t_len = cut_len;
        slot = blockIdx.y;
    }
    const int64_t hoff = (int64_t)head * head_stride;
    const e16* Kh = K + (int64_t)head * kv_head_stride;
    const e16* Vh = V + (int64_t)head * kv_head_stride;
    const int nblk = (Nk + kQ64BK - 1) / kQ64BK;

    const typename Loader::LaneOffsets ld = Loader::lane_offsets(row_stride, wave, lane);
    const typename Loader::TailOffsets ld_tail = Loader::tail_offsets(row_stride, wave, lane, Nk);
    // Fetches block tb; blocks past the end re-read the last real one (all their keys are masked); branch-free.
    // The steady-state iterations never reach the last block and fetch through running pointers instead.
    auto load_tile = [&](e16* tile, const e16* base, int tb) __attribute__((always_inline)) {
        tb = tb < nblk ? tb : nblk - 1;
        const int r0 = tb * kQ64BK;
        Loader::issue_sel(tile, base + (int64_t)r0 * row_stride, ld, ld_tail, r0 + kQ64BK > Nk, wave);
    };
    const int64_t tile_elems = (int64_t)kQ64BK * row_stride;
    const float sl2 = scale * kLog2e;
    const float lazy = kQ64Lazy / sl2;              // in units of raw scores

    const uint32_t sbase = lds_addr(smem);
    uint32_t r_adr[NT];                 // row read of K: row ln, chunk 2t+g
#pragma unroll
    for (int t = 0; t < NT; ++t) r_adr[t] = sbase + 2 * tile_off<D>(ln, 2 * t + g);
    uint32_t t_adr[NCB][2];             // transposing read of V: rows 4g+(i>>2) (+8), channels 32cb+16h+4(i&3)
    {
        const int i = lane & 15, h = (lane >> 4) & 1;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int hh = 0; hh < 2; ++hh)
                t_adr[cb][hh] = sbase + 2 * (tile_off<D>(4 * g + (i >> 2) + 8 * hh, 4 * cb + 2 * h + ((i & 3) >> 1)) +
                                             4 * (i & 1));
    }

    const int q0 = qt * kFwdBQ;
    // Key blocks b_lo .. b_hi-1, walked as cnt (a multiple of 4) local positions; causal: up to the end of this
    // tile's diagonal.  Blocks from b_hi on are masked entirely.
    int b_lo = 0, b_hi = CAUSAL ? (q0 + kFwdBQ) / kQ64BK : nblk;
    if (CUT) {
        int k_end = Nk;
        if (CAUSAL) { const int lim = q0 + kFwdBQ; k_end = lim < Nk ? lim : Nk; }
        const int n_kt = (k_end + kFwdBK - 1) / kFwdBK - t_off;          // 64-key tiles left from t_off on
        b_lo = 2 * t_off;
        b_hi = b_lo + 2 * (n_kt < t_len ? n_kt : t_len);
    }
    const int cnt = (b_hi - b_lo + 3) & ~3;
    // K tiles of blocks 0..3; V tiles of blocks 0, 1 and, in slot 3, block 0 once more: the first iteration
    // multiplies zeros with that slot, which therefore has to hold finite numbers
#pragma unroll
    for (int i = 0; i < kQ64Ring; ++i) load_tile(smem + i * TILE, Kh, b_lo + i);
    load_tile(smem + (kQ64Ring + 0) * TILE, Vh, b_lo);
    load_tile(smem + (kQ64Ring + 1) * TILE, Vh, b_lo + 1);
    load_tile(smem + (kQ64Ring + 3) * TILE, Vh, b_lo);
    // the tiles iteration 0 fetches: K of the fifth block, V of the third
    const e16* k_next = Kh + (b_lo + kQ64Ring) * tile_elems;
    const e16* v_next = Vh + (b_lo + 2) * tile_elems;

    // ---- this lane's two queries: Q rows as B operands
    int q_row[2], klim[2];
    e16x8 qreg[2][NT];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        q_row[qb] = q0 + wave * 64 + qb * 32 + ln;
        const int q_ld = q_row[qb] < N ? q_row[qb] : N - 1;
        // key offset c_r (inside a block starting at k0) is masked iff c_r > klim - k0
        int last = CAUSAL ? (q_row[qb] < Nk - 1 ? q_row[qb] : Nk - 1) : Nk - 1;        // last visible key
        if (CUT) last = last < b_hi * kQ64BK - 1 ? last : b_hi * kQ64BK - 1;
        klim[qb] = last - 4 * g;
#pragma unroll
        for (int t = 0; t < NT; ++t)
            qreg[qb][t] = *reinterpret_cast<const e16x8*>(Q + hoff + (int64_t)q_ld * row_stride + 16 * t + 8 * g);
    }

    float m_used[2] = {-INFINITY, -INFINITY}, ms[2], l_run[2] = {0.f, 0.f};
    float pend[2] = {1.f, 1.f};         // factor O still has to take after the next product with V
    bool pending = false;               // (wave-uniform)
    f32x16 oacc[2][NCB];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[qb][cb][r] = 0.f;

    f32x16 s[2][2];                     // [parity][query block]: scores of the current and of the next block
    e16x8 krow[NT];
    e16x4 vt_lo[2][NCB], vt_hi[2][NCB];
    e16x8 pb_prev[2][2];                // P^T of the previous block, packed as B operands
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int e = 0; e < 8; ++e) pb_prev[qb][u][e] = (e16)0.f;

    // K rows of a block: channels 0..63 (half 0) or 64..127 (half 1)
    auto read_krow = [&](auto slot_tag, auto half_tag) __attribute__((always_inline)) {
        constexpr int SL = decltype(slot_tag)::value;
        constexpr int T0 = decltype(half_tag)::value * (NT / 2);
#pragma unroll
        for (int t = T0; t < T0 + NT / 2; ++t) krow[t] = lds_b128<KB + SL * TB>(r_adr[t]);
    };
    auto read_transposed = [&](auto slot_tag, auto half_tag) __attribute__((always_inline)) {
        constexpr int SL = decltype(slot_tag)::value;
        constexpr int U = decltype(half_tag)::value;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
            vt_lo[U][cb] = lds_tr_b64<VB + SL * TB + U * HALF>(t_adr[cb][0]);
            vt_hi[U][cb] = lds_tr_b64<VB + SL * TB + U * HALF>(t_adr[cb][1]);
        }
    };
    auto tie_krow = [&](auto half_tag) __attribute__((always_inline)) {
        constexpr int T0 = decltype(half_tag)::value * (NT / 2);
#pragma unroll
        for (int t = T0; t < T0 + NT / 2; ++t) lds_tie(krow[t]);
    };
    auto tie_transposed = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) lds_tie(vt_lo[u][cb], vt_hi[u][cb]);
    };
    auto tie_half = [&](auto half_tag) __attribute__((always_inline)) {
        constexpr int U = decltype(half_tag)::value;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) lds_tie(vt_lo[U][cb], vt_hi[U][cb]);
    };
    // O^T += V^T P^T over 16 keys of the previous block, for both query blocks
    auto pv_half = [&](auto half_tag) __attribute__((always_inline)) {
        constexpr int U = decltype(half_tag)::value;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
            const e16x8 va = __builtin_shufflevector(vt_lo[U][cb], vt_hi[U][cb], 0, 1, 2, 3, 4, 5, 6, 7);
            oacc[0][cb] = mfma32(va, pb_prev[0][U], oacc[0][cb]);
            oacc[1][cb] = mfma32(va, pb_prev[1][U], oacc[1][cb]);
        }
    };
    auto zero = [&](f32x16& x) __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < 16; ++r) x[r] = 0.f;
    };
    // masks block kb in s[par], takes its row maxima and says whether a reference maximum must move
    auto block_max = [&](int par, bool masked, int kb, float (&m_blk)[2]) __attribute__((always_inline)) {
        bool moved = false;
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            if (masked) {
                const int krel = klim[qb] - kb * kQ64BK;
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (8 * (r >> 2) + (r & 3) > krel) s[par][qb][r] = -INFINITY;
            }
            float mb = s[par][qb][0];
#pragma unroll
            for (int r = 1; r < 16; ++r) mb = fmaxf(mb, s[par][qb][r]);
            m_blk[qb] = xhalf_max(mb);
            moved = moved || (m_blk[qb] > m_used[qb] + lazy);
        }
        return moved;
    };
    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, 1>;
    using S2 = std::integral_constant<int, 2>;
    using S3 = std::integral_constant<int, 3>;

    // ---- prologue: everything asked for so far resident; S^T of block 0 and its maxima; then the K rows of block 1
    wait_vm<0>();
    __syncthreads();
    // The Q operands live in accumulation registers, where the matrix unit reads them directly; together with O
    // and the scores they fill that half of the register file, everything else stays in the vector half.
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int t = 0; t < NT; ++t) asm volatile("" : "+a"(qreg[qb][t]));
    read_krow(S0{}, S0{});
    read_krow(S0{}, S1{});
    wait_lgkm<0>();
    tie_krow(S0{});
    tie_krow(S1{});
    mfma32_v_first(s[0][0], krow[0], qreg[0][0]);
    mfma32_v_first(s[0][1], krow[0], qreg[1][0]);
#pragma unroll
    for (int t = 1; t < NT; ++t) {
        mfma32_v_acc(s[0][0], krow[t], qreg[0][t]);
        mfma32_v_acc(s[0][1], krow[t], qreg[1][t]);
    }
    mfma32_v_settle(s[0][0], s[0][1]);            // the vector unit must not read the scores before they are written
    __builtin_amdgcn_sched_barrier(0);
    {
        float m_blk[2];
        block_max(0, true, b_lo, m_blk);
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            m_used[qb] = m_blk[qb];
            ms[qb] = (m_used[qb] == -INFINITY ? 0.f : m_used[qb]) * sl2;
        }
    }
    // (no other work between a hand-issued read and its wait here: outside the loop the compiler moves registers
    // around freely, also ones whose data is still on its way)
    __builtin_amdgcn_sched_barrier(0);
    read_krow(S1{}, S0{});
    wait_lgkm<0>();
    tie_krow(S0{});
    __builtin_amdgcn_sched_barrier(0);

    // One iteration.  At entry: s[SL & 1] holds the scores of block p, whose maxima are already in m_used; the K
    // rows of block p+1 (channels 0..63) are in registers; pb_prev is P^T of block p-1, whose V tile is in slot (SL+3) % 4; no LDS
    // read is in flight.  K tiles are fetched four blocks ahead, V tiles two (their slot is free a block later).
    auto iteration = [&](auto masked_tag, auto slot_tag, auto slot2_tag, auto slotv_tag, int p) __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked_tag)::value;      // block p+1 may need the mask
        constexpr int SL = decltype(slot_tag)::value;
        constexpr int SLV = decltype(slotv_tag)::value;
        constexpr int PAR = SL & 1;
        e16x8 pb[2][2];
        float rs[2] = {0.f, 0.f};
        // exponentials of the score pair j (0..15) of block p: query block j / 8, registers 2 (j % 8), +1
        auto exp_pair = [&](int j) __attribute__((always_inline)) {
            const int qb = j >> 3, r = 2 * (j & 7);
            const float p0 = fast_exp2(__builtin_fmaf(s[PAR][qb][r], sl2, -ms[qb]));
            const float p1 = fast_exp2(__builtin_fmaf(s[PAR][qb][r + 1], sl2, -ms[qb]));
            rs[qb] += p0;
            rs[qb] += p1;
            e16x2 pk = {(e16)p0, (e16)p1};
            asm volatile("" : "+v"(pk));              // packed here, not wherever the value is finally used
            pb[qb][r >> 3][r & 7] = pk[0];
            pb[qb][r >> 3][(r & 7) + 1] = pk[1];
        };
        // The first ten score pairs of block p go through three stages one MFMA apart (exponent, exponential, sum and
        // packing), so that no vector instruction waits for the one before it; pair j starts at step j + j / 2.
        constexpr int kStaged = 10;
        float xv[2 * kStaged], pv[2 * kStaged];
        auto exp_stage = [&](int step) __attribute__((always_inline)) {
#pragma unroll
            for (int j = 0; j < kStaged; ++j) {
                const int first = j + j / 2, qb = j >> 3, r = 2 * (j & 7);
                if (step == first) {
                    xv[2 * j] = __builtin_fmaf(s[PAR][qb][r], sl2, -ms[qb]);
                    xv[2 * j + 1] = __builtin_fmaf(s[PAR][qb][r + 1], sl2, -ms[qb]);
                }
                if (step == first + 1) {
                    pv[2 * j] = fast_exp2(xv[2 * j]);
                    pv[2 * j + 1] = fast_exp2(xv[2 * j + 1]);
                }
                if (step == first + 2) {
                    rs[qb] += pv[2 * j];
                    rs[qb] += pv[2 * j + 1];
                    e16x2 pk = {(e16)pv[2 * j], (e16)pv[2 * j + 1]};
                    asm volatile("" : "+v"(pk));      // packed here, not wherever the value is finally used
                    pb[qb][r >> 3][r & 7] = pk[0];
                    pb[qb][r >> 3][(r & 7) + 1] = pk[1];
                }
            }
        };
        // S^T of block p+1, K channels 16t..16t+15, for both query blocks, each MFMA followed by one step of the
        // vector work on block p (the MFMAs are fixed in place; the vector work may not cross them)
        auto s_step = [&](int t) __attribute__((always_inline)) {
            if (t == 0) mfma32_v_first(s[PAR ^ 1][0], krow[0], qreg[0][0]);
            else mfma32_v_acc(s[PAR ^ 1][0], krow[t], qreg[0][t]);
            exp_stage(2 * t);
            __builtin_amdgcn_sched_barrier(0);
            if (t == 0) mfma32_v_first(s[PAR ^ 1][1], krow[0], qreg[1][0]);
            else mfma32_v_acc(s[PAR ^ 1][1], krow[t], qreg[1][t]);
            exp_stage(2 * t + 1);
            __builtin_amdgcn_sched_barrier(0);
        };
        // ---- region A, first half
        read_krow(std::integral_constant<int, (SL + 1) % kQ64Ring>{}, S1{});     // K rows of block p+1, channels 64..127
        __builtin_amdgcn_sched_barrier(0);
        s_step(0);
        s_step(1);
        s_step(2);
        s_step(3);
        // ---- region A, second half
        wait_lgkm<0>();
        tie_krow(S1{});
        read_transposed(slotv_tag, S0{});             // V^T of block p-1, keys 0..15
        __builtin_amdgcn_sched_barrier(0);
        s_step(4);
        s_step(5);
        s_step(6);
        s_step(7);

        // ---- region B: tiles up to p+2 (K) and p+1 (V) have landed; everyone is done with the K tile of block p
        // and the V tile of block p-2, which are refilled with the K tile of block p+4 and the V tile of block p+2
        wait_vm<LPT>();
        barrier_no_drain();
        if (MASKED) {
            load_tile(smem + SL * TILE, Kh, b_lo + p + kQ64Ring);
            load_tile(smem + (kQ64Ring + (SLV + 3) % kQ64Ring) * TILE, Vh, b_lo + p + 2);
        } else {                                      // block p+4 is not the last one here: no clamp, no ragged tile
            Loader::issue(smem + SL * TILE, k_next, ld, wave);
            Loader::issue(smem + (kQ64Ring + (SLV + 3) % kQ64Ring) * TILE, v_next, ld, wave);
            k_next += tile_elems;
            v_next += tile_elems;
        }
        read_transposed(slotv_tag, S1{});             // V^T of block p-1, keys 16..31
        wait_lgkm<2 * NCB>();                         // the reads of region A
        tie_half(S0{});
        read_krow(slot2_tag, S0{});                   // K rows of block p+2 (channels 0..63), for the next iteration
        __builtin_amdgcn_sched_barrier(0);
        pv_half(S0{});
        exp_pair(10); exp_pair(11); exp_pair(12);
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);
            __builtin_amdgcn_sched_group_barrier(0x400, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        wait_lgkm<NT / 2>();                          // the V^T reads of this region (the K rows may still be in flight)
        tie_half(S1{});
        __builtin_amdgcn_sched_barrier(0);
        pv_half(S1{});
        exp_pair(13); exp_pair(14); exp_pair(15);
        float m_blk[2];
        const bool moved = block_max(PAR ^ 1, MASKED, b_lo + p + 1, m_blk);
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, MASKED ? 16 : 7, 0);
            __builtin_amdgcn_sched_group_barrier(0x400, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            l_run[qb] += rs[qb];
#pragma unroll
            for (int u = 0; u < 2; ++u) pb_prev[qb][u] = pb[qb][u];
        }
        // The compiler may move registers at control-flow joins (the rescale branch, the loop edges) without
        // knowing that a hand-issued LDS read into them is in flight: the reads land before any branch.
        wait_lgkm<0>();
        tie_krow(S0{});
        __builtin_amdgcn_sched_barrier(0);
        if (pending) {                                // O now holds blocks up to p-1, all under the maximum before last
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[qb][cb][r] *= pend[qb];
            pending = false;
        }
        if (__builtin_amdgcn_ballot_w64(moved) != 0) {
            // The row sums carry the old reference maximum and move now.  So do O and the P^T of block p, which is
            // already rounded and still to be multiplied with V: O moves once that product is in it (a second
            // rounding of P^T is avoided that way).
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                const float m_new = fmaxf(m_used[qb], m_blk[qb]);
                const float m_fin = (m_new == -INFINITY) ? 0.f : m_new;     // a row with nothing visible yet
                const float alpha = fast_exp2((m_used[qb] - m_fin) * sl2);
                l_run[qb] *= alpha;
                pend[qb] = alpha;
                m_used[qb] = m_new;
                ms[qb] = m_fin * sl2;
            }
            pending = true;
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    using Plain = std::integral_constant<bool, false>;
    using Masked = std::integral_constant<bool, true>;
    // An iteration at local position p needs no mask if block b_lo+p+1, whose maxima it takes, is entirely
    // visible (before this tile's diagonal, inside the sequence and the item), and may fetch through the running
    // pointers if the blocks it fetches (K: b_lo+p+4, V: b_lo+p+2) are not the last, possibly ragged, block of
    // the sequence or one after it.  The block after the last does not exist and is masked entirely.
    int fb = CAUSAL ? q0 / kQ64BK : Nk / kQ64BK;              // first block that needs the mask
    fb = fb < b_hi ? fb : b_hi;
    int plain_end = (fb - b_lo - 1 < nblk - 5 - b_lo ? fb - b_lo - 1 : nblk - 5 - b_lo) & ~3;
    plain_end = plain_end > 0 ? plain_end : 0;
    int p = 0;
    for (; p < plain_end; p += 4) {
        iteration(Plain{}, S0{}, S2{}, S3{}, p);
        iteration(Plain{}, S1{}, S3{}, S0{}, p + 1);
        iteration(Plain{}, S2{}, S0{}, S1{}, p + 2);
        iteration(Plain{}, S3{}, S1{}, S2{}, p + 3);
    }
    for (; p < cnt; p += 4) {
        iteration(Masked{}, S0{}, S2{}, S3{}, p);
        iteration(Masked{}, S1{}, S3{}, S0{}, p + 1);
        iteration(Masked{}, S2{}, S0{}, S1{}, p + 2);
        iteration(Masked{}, S3{}, S1{}, S2{}, p + 3);
    }
    // ---- the product with V of the last block (cnt is a multiple of 4: its V tile is in slot 3).  After it
    // nothing is writing LDS any more.  The scores of the block after the last one, which nobody reads, are still
    // on their way through the matrix unit: their registers stay untouched until they have arrived.
    mfma32_v_settle(s[0][0], s[0][1], s[1][0], s[1][1]);
    read_transposed(S3{}, S0{});
    read_transposed(S3{}, S1{});
    wait_vm<0>();
    wait_lgkm<0>();
    tie_transposed();
    __builtin_amdgcn_sched_barrier(0);
    pv_half(S0{});
    pv_half(S1{});
    __builtin_amdgcn_sched_barrier(0);
    if (pending) {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[qb][cb][r] *= pend[qb];
    }

#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const float l_tot = xhalf_sum(l_run[qb]);
        const float inv = 1.f / l_tot;
        if (CUT && slot >= 0) {
            // one of several items of this query tile: fp32 partial results [slot][query][channel], [slot][query][m, l]
            const int64_t at = (int64_t)head * slots_per_head + slot;
            const int row = wave * 64 + qb * 32 + ln;
            float* prow = part_o + (at * kFwdBQ + row) * D;
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                for (int rq = 0; rq < 4; ++rq) {
                    f32x4 w;
#pragma unroll
                    for (int e = 0; e < 4; ++e) w[e] = oacc[qb][cb][4 * rq + e];
                    *reinterpret_cast<f32x4*>(prow + 32 * cb + 8 * rq + 4 * g) = w;
                }
            if (g == 0) {
                part_ml[(at * kFwdBQ + row) * 2] = m_used[qb];
                part_ml[(at * kFwdBQ + row) * 2 + 1] = l_tot;
            }
        } else if (q_row[qb] < N) {
            e16* orow = O + hoff + (int64_t)q_row[qb] * row_stride;
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                for (int rq = 0; rq < 4; ++rq) {
                    e16x4 w;
#pragma unroll
                    for (int e = 0; e < 4; ++e) w[e] = (e16)(oacc[qb][cb][4 * rq + e] * inv);
                    *reinterpret_cast<e16x4*>(orow + 32 * cb + 8 * rq + 4 * g) = w;
                }
            if (g == 0) LSE[(int64_t)head * N + q_row[qb]] = m_used[qb] * scale + __logf(l_tot);
        }
    }
}

// Merges the pieces of the cut query tiles: with m = max_i m_i and w_i = exp(scale (m_i - m)),
//   l = sum_i w_i l_i,   O = sum_i w_i O_i / l,   LSE = scale m + log l        (pieces in a fixed order).
// Grid (query tiles x 32, heads): a workgroup merges 8 query rows, 32 lanes per row (D / 32 floats each).
// `red` (block-sparse: from the plan) gives a tile's first slot and its number of pieces; without it every tile has
// `pieces` consecutive slots.
template <int D>
__global__ __launch_bounds__(256) void attn_fwd_combine_kernel(const float* __restrict__ part_o,
                                                               const float* __restrict__ part_ml, int pieces,
                                                               const int2* __restrict__ red, int slots_per_head,
                                                               e16* __restrict__ O, float* __restrict__ LSE, int N,
                                                               int64_t row_stride, int64_t head_stride, float scale) {
    constexpr int PER = D / 32;                                       // floats per lane and row
    constexpr int GROUPS = kFwdBQ / 8;                                // row groups per query tile
    const int qt = blockIdx.x / GROUPS, head = blockIdx.y;
    int first = qt * pieces;
    if (red) {
        const int2 r = red[qt];
        if (r.y <= 1) return;                                         // not cut: its workgroup wrote O and LSE itself
        first = r.x;
        pieces = r.y;
    }
    const int64_t slot0 = (int64_t)head * slots_per_head + first;     // the pieces of a tile are consecutive slots
    const float sl2 = scale * kLog2e;
    {
        const int r = (blockIdx.x % GROUPS) * 8 + threadIdx.x / 32;
        const int q_row = qt * kFwdBQ + r;
        if (q_row >= N) return;
        const int c0 = (threadIdx.x % 32) * PER;
        float m = -INFINITY;
        for (int i = 0; i < pieces; ++i) m = fmaxf(m, part_ml[((slot0 + i) * kFwdBQ + r) * 2]);
        float l = 0.f, acc[PER];
#pragma unroll
        for (int c = 0; c < PER; ++c) acc[c] = 0.f;
        for (int i = 0; i < pieces; ++i) {
            const float* ml = part_ml + ((slot0 + i) * kFwdBQ + r) * 2;
            const float w = fast_exp2((ml[0] - m) * sl2);
            l += w * ml[1];
            const float* src = part_o + ((slot0 + i) * kFwdBQ + r) * D + c0;
#pragma unroll
            for (int c = 0; c < PER; ++c) acc[c] += w * src[c];
        }
        const float inv = 1.f / l;
        e16* dst = O + (int64_t)head * head_stride + (int64_t)q_row * row_stride + c0;
#pragma unroll
        for (int c = 0; c < PER; ++c) dst[c] = (e16)(acc[c] * inv);
        if (threadIdx.x % 32 == 0) LSE[(int64_t)head * N + q_row] = m * scale + __logf(l);
    }
}

// How the key tiles of unmasked attention with few query tiles are cut (the forward runs two
// workgroups per CU: 512 places).  Pieces of at least 16 tiles (1024 keys).
struct FwdCut {
    int pieces, len;
};
inline FwdCut fwd_cut(int64_t n_qtiles, int64_t n_kt, int Hl) {
    FwdCut c{1, (int)n_kt};
    if (n_qtiles * Hl >= 512 || n_kt < 32) return c;
    int64_t want = (1024 + n_qtiles * Hl - 1) / (n_qtiles * Hl);
    const int64_t most = n_kt / 16;
    want = want < most ? want : most;
    if (want < 2) return c;
    const int64_t len = (((n_kt + want - 1) / want) + 1) & ~(int64_t)1;
    c.len = (int)len;
    c.pieces = (int)((n_kt + len - 1) / len);
    return c;
}
inline int64_t fwd_cut_workspace_floats_of(int64_t N, int64_t Nk, int Hl, int d) {
    const int64_t n_qtiles = (N + kFwdBQ - 1) / kFwdBQ, n_kt = (Nk + kFwdBK - 1) / kFwdBK;
    const FwdCut c = fwd_cut(n_qtiles, n_kt, Hl);
    if (c.pieces < 2) return 0;
    return n_qtiles * c.pieces * Hl * (int64_t)kFwdBQ * (d + 2);
}

// Workspace of the plan-driven forward (block-sparse; dense causal with few query tiles), in floats: work plan,
// per-tile table, partial results of the cut rows (at most four slots per query tile and head, and no more than
// the target asks for).
constexpr int kFwdRowPlanTarget = 1024;
struct SparseFwdWorkspace {
    int64_t plan_at, red_at, part_o_at, part_ml_at, total, items_bound;
    int slots_per_head;
};
inline SparseFwdWorkspace sparse_fwd_workspace(int64_t N, int Hl, int d) {
    const int64_t n_qtiles = (N + kFwdBQ - 1) / kFwdBQ;
    auto up = [](int64_t x) { return (x + 63) & ~(int64_t)63; };
    SparseFwdWorkspace w;
    const int64_t by_target = 2 * ((kFwdRowPlanTarget + Hl - 1) / Hl), by_size = 4 * n_qtiles + 1;
    w.slots_per_head = (int)(by_target < by_size ? by_target : by_size);
    w.items_bound = n_qtiles + w.slots_per_head + 1;
    w.plan_at = 0;
    w.red_at = up(4 * (1 + w.items_bound));
    w.part_o_at = up(w.red_at + 2 * n_qtiles);
    w.part_ml_at = up(w.part_o_at + (int64_t)w.slots_per_head * Hl * kFwdBQ * d);
    w.total = w.part_ml_at + (int64_t)w.slots_per_head * Hl * kFwdBQ * 2;
    return w;
}
int64_t attn_fwd_sparse_workspace_floats(int64_t N, int Hl, int d) { return sparse_fwd_workspace(N, Hl, d).total; }

// Dense causal attention is planned only when its query tiles alone would leave places idle or unevenly used
// (two workgroups per CU: 512 places; beyond a thousand tiles, starting the longest first evens them out).
inline bool causal_fwd_is_planned(int64_t N, int Hl) { return ((N + kFwdBQ - 1) / kFwdBQ) * Hl < 1024; }
int64_t attn_fwd_causal_workspace_floats(int64_t N, int Hl, int d) {
    if (d == 256 || !causal_fwd_is_planned(N, Hl)) return 0;
    return sparse_fwd_workspace(N, Hl, d).total;
}

template <int D>
static int launch_fwd(const void* q, const void* k, const void* v, void* o, float* lse, float* ws, int64_t N,
                      int64_t Nk, int Hl, float scale, int causal, TensorStrides st, TensorStrides kv,
                      hipStream_t stream) {
    const int64_t n_qtiles = (N + kFwdBQ - 1) / kFwdBQ;
    // unmasked attention with few query tiles and a workspace for the pieces
    const FwdCut cut = (!causal && ws) ? fwd_cut(n_qtiles, (Nk + kFwdBK - 1) / kFwdBK, Hl) : FwdCut{1, 0};
    if (cut.pieces > 1 && n_qtiles * cut.pieces <= 65535 && Hl <= 65535) {
        const int64_t items = n_qtiles * cut.pieces;
        float* part_o = ws;
        float* part_ml = ws + items * Hl * (int64_t)kFwdBQ * D;
        if constexpr (D == 128)
            attn_fwd_q64_kernel<false, true><<<dim3((uint32_t)Hl, (uint32_t)items), dim3(kQ64Threads), 0, stream>>>(
                (const e16*)q, (const e16*)k, (const e16*)v, (e16*)o, lse, (int)N, (int)Nk, (int)n_qtiles, st.row, st.head,
                kv.head, scale, cut.pieces, cut.len, part_o, part_ml, nullptr, (int)items);
        else
            attn_fwd_kernel<D, false, false, true><<<dim3((uint32_t)Hl, (uint32_t)items), dim3(kFwdThreads), 0, stream>>>(
                (const e16*)q, (const e16*)k, (const e16*)v, (e16*)o, lse, (int)N, (int)Nk, (int)n_qtiles, st.row, st.head,
                kv.head, scale, nullptr, nullptr, cut.pieces, cut.len, part_o, part_ml, nullptr, (int)items);
        if (hipGetLastError() != hipSuccess) return ULY_ERR_LAUNCH;
        attn_fwd_combine_kernel<D><<<dim3((uint32_t)(n_qtiles * (kFwdBQ / 8)), (uint32_t)Hl), dim3(256), 0, stream>>>(
            part_o, part_ml, cut.pieces, nullptr, (int)items, (e16*)o, lse, (int)N, st.row, st.head, scale);
        return hipGetLastError() == hipSuccess ? ULY_OK : ULY_ERR_LAUNCH;
    }
    if (causal && ws && causal_fwd_is_planned(N, Hl)) {
        const SparseFwdWorkspace w = sparse_fwd_workspace(N, Hl, D);
        if (w.items_bound <= 65535 && Hl <= 65535) {
            int4* plan = reinterpret_cast<int4*>(ws + w.plan_at);
            int2* red = reinterpret_cast<int2*>(ws + w.red_at);
            float* part_o = ws + w.part_o_at;
            float* part_ml = ws + w.part_ml_at;
            if (sparse_plan_launch(3, nullptr, n_qtiles, N, Hl, w.slots_per_head, kFwdRowPlanTarget, plan, red, stream) != ULY_OK)
                return ULY_ERR_LAUNCH;
            if constexpr (D == 128)
                attn_fwd_q64_kernel<true, true>
                    <<<dim3((uint32_t)Hl, (uint32_t)w.items_bound), dim3(kQ64Threads), 0, stream>>>(
                        (const e16*)q, (const e16*)k, (const e16*)v, (e16*)o, lse, (int)N, (int)Nk, (int)n_qtiles, st.row,
                        st.head, kv.head, scale, 1, 0, part_o, part_ml, plan, w.slots_per_head);
            else
                attn_fwd_kernel<D, true, false, true>
                    <<<dim3((uint32_t)Hl, (uint32_t)w.items_bound), dim3(kFwdThreads), 0, stream>>>(
                        (const e16*)q, (const e16*)k, (const e16*)v, (e16*)o, lse, (int)N, (int)Nk, (int)n_qtiles, st.row,
                        st.head, kv.head, scale, nullptr, nullptr, 1, 0, part_o, part_ml, plan, w.slots_per_head);
            if (hipGetLastError() != hipSuccess) return ULY_ERR_LAUNCH;
            attn_fwd_combine_kernel<D><<<dim3((uint32_t)(n_qtiles * (kFwdBQ / 8)), (uint32_t)Hl), dim3(256), 0, stream>>>(
                part_o, part_ml, 0, red, w.slots_per_head, (e16*)o, lse, (int)N, st.row, st.head, scale);
            return hipGetLastError() == hipSuccess ? ULY_OK : ULY_ERR_LAUNCH;
        }
    }
    const int64_t blocks = ((causal && kFwdPair) ? (n_qtiles + 1) / 2 : n_qtiles) * Hl;    // causal: pairs of query tiles
    if (blocks > 0x7FFFFFFFll) return ULY_ERR_SHAPE;
    if constexpr (D == 128) {
        // one workgroup per query tile, 64 queries per wave
        const dim3 grid((uint32_t)(n_qtiles * Hl)), block(kQ64Threads);
        if (causal)
            attn_fwd_q64_kernel<true><<<grid, block, 0, stream>>>((const e16*)q, (const e16*)k, (const e16*)v, (e16*)o, lse,
                                                                  (int)N, (int)Nk, (int)n_qtiles, st.row, st.head, kv.head,
                                                                  scale, 1, 0, nullptr, nullptr, nullptr, 0);
        else
            attn_fwd_q64_kernel<false><<<grid, block, 0, stream>>>((const e16*)q, (const e16*)k, (const e16*)v, (e16*)o, lse,
                                                                   (int)N, (int)Nk, (int)n_qtiles, st.row, st.head, kv.head,
                                                                   scale, 1, 0, nullptr, nullptr, nullptr, 0);
    } else {
        dim3 grid((uint32_t)blocks), block(kFwdThreads);
        if (causal)
            attn_fwd_kernel<D, true><<<grid, block, 0, stream>>>((const e16*)q, (const e16*)k, (const e16*)v, (e16*)o,
                                                                 lse, (int)N, (int)Nk, (int)n_qtiles, st.row, st.head, kv.head,
                                                                 scale, nullptr, nullptr, 1, 0, nullptr, nullptr, nullptr, 0);
        else
            attn_fwd_kernel<D, false><<<grid, block, 0, stream>>>((const e16*)q, (const e16*)k, (const e16*)v,
                                                                  (e16*)o, lse, (int)N, (int)Nk, (int)n_qtiles, st.row, st.head,
                                                                  kv.head, scale, nullptr, nullptr, 1, 0, nullptr, nullptr, nullptr,
                                                                  0);
    }
    return hipGetLastError() == hipSuccess ? ULY_OK : ULY_ERR_LAUNCH;
}

template <int D>
static int launch_fwd_sparse(const void* q, const void* k, const void* v, void* o, float* lse, float* ws,
                             const int* row_ptr, const int* col_idx, int64_t N, int Hl, float scale, TensorStrides st,
                             hipStream_t stream) {
    const int64_t n_qtiles = (N + kFwdBQ - 1) / kFwdBQ;
    const SparseFwdWorkspace w = sparse_fwd_workspace(N, Hl, D);
    if (w.items_bound > 65535 || Hl > 65535 || n_qtiles * (kFwdBQ / 8) > 0x7FFFFFFFll) return ULY_ERR_SHAPE;
    int4* plan = reinterpret_cast<int4*>(ws + w.plan_at);
    int2* red = reinterpret_cast<int2*>(ws + w.red_at);
    float* part_o = ws + w.part_o_at;
    float* part_ml = ws + w.part_ml_at;
    if (sparse_plan_launch(2, row_ptr, n_qtiles, N, Hl, w.slots_per_head, kFwdRowPlanTarget, plan, red, stream) != ULY_OK)
        return ULY_ERR_LAUNCH;
    attn_fwd_kernel<D, true, true, true><<<dim3((uint32_t)Hl, (uint32_t)w.items_bound), dim3(kFwdThreads), 0, stream>>>(
        (const e16*)q, (const e16*)k, (const e16*)v, (e16*)o, lse, (int)N, (int)N, (int)n_qtiles, st.row, st.head, st.head,
        scale, row_ptr, col_idx, 1, 0, part_o, part_ml, plan, w.slots_per_head);
    if (hipGetLastError() != hipSuccess) return ULY_ERR_LAUNCH;
    attn_fwd_combine_kernel<D><<<dim3((uint32_t)(n_qtiles * (kFwdBQ / 8)), (uint32_t)Hl), dim3(256), 0, stream>>>(
        part_o, part_ml, 0, red, w.slots_per_head, (e16*)o, lse, (int)N, st.row, st.head, scale);
    return hipGetLastError() == hipSuccess ? ULY_OK : ULY_ERR_LAUNCH;
}

int attn_fwd_sparse_launch(const void* q, const void* k, const void* v, void* o, float* lse, float* ws,
                           const int* row_ptr, const int* col_idx, int64_t N, int Hl, int d, float scale,
                           TensorStrides st, void* stream) {
    if (d == 128)
        return launch_fwd_sparse<128>(q, k, v, o, lse, ws, row_ptr, col_idx, N, Hl, scale, st, (hipStream_t)stream);
    return launch_fwd_sparse<64>(q, k, v, o, lse, ws, row_ptr, col_idx, N, Hl, scale, st, (hipStream_t)stream);
}

int64_t attn_fwd_cut_workspace_floats(int64_t N, int64_t Nk, int Hl, int d) {
    if (d == 256) return 0;                   // the d = 256 kernels do not cut
    return fwd_cut_workspace_floats_of(N, Nk, Hl, d);
}

int attn_fwd_launch(const void* q, const void* k, const void* v, void* o, float* lse, float* ws, int64_t N, int64_t Nk,
                    int Hl, int d, float scale, int causal, TensorStrides st, TensorStrides kv, void* stream) {
    if (d == 256) return attn256_fwd_launch(q, k, v, o, lse, N, Nk, Hl, scale, causal, st, kv, stream);
    if (d == 128) return launch_fwd<128>(q, k, v, o, lse, ws, N, Nk, Hl, scale, causal, st, kv, (hipStream_t)stream);
    return launch_fwd<64>(q, k, v, o, lse, ws, N, Nk, Hl, scale, causal, st, kv, (hipStream_t)stream);
}

}  // namespace ULY_ELEM_NS

#if !defined(ULY_BUILD_F16)
using namespace bf16;

// ------------------------------------------------------------------------------------------
// Measurement aid: nothing but bf16 MFMAs (four independent accumulation chains per wave, one wave
// per SIMD, operands taken from a caller-filled buffer so that they toggle like real data).  What
// this sustains is the matrix rate the part actually allows under its power limit; the attention
// kernels are quoted against it next to the published peak.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256, 1) void mfma_probe_kernel(const e16* __restrict__ data, float* __restrict__ sink,
                                                            int iters) {
    __shared__ float pad[24 * 1024];                 // 96 KiB: one workgroup per CU
    if (iters < 0) pad[threadIdx.x] = 0.f;
    e16x8 a[8], b[8];
    const e16x8* src = reinterpret_cast<const e16x8*>(data);
#pragma unroll
    for (int t = 0; t < 8; ++t) { a[t] = src[threadIdx.x + 512 * t]; b[t] = src[threadIdx.x + 512 * t + 256]; }
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
#pragma unroll 1
    for (int it = 0; it < iters; ++it)
#pragma unroll
        for (int t = 0; t < 8; ++t) acc[t & 3] = mfma32(a[t], b[t], acc[t & 3]);
    float tot = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) tot += acc[i][r];
    if (tot == 12345.678f) sink[blockIdx.x * 256 + threadIdx.x] = tot + pad[0];   // keeps the loop alive; practically never true
}

// The same with one operand of every MFMA read from LDS (1 KiB per wave and MFMA, the operand traffic of the
// attention kernels, whose other operand sits in registers): 64 KiB of `data` are staged in LDS, the reads of
// the next eight MFMAs are issued before the current eight run.  What this sustains bounds any kernel that feeds
// its matrix pipe this way.
__global__ __launch_bounds__(256, 1) void mfma_lds_probe_kernel(const e16* __restrict__ data, float* __restrict__ sink,
                                                                int iters) {
    __shared__ __attribute__((aligned(1024))) e16 tile[8 * 32 * 128];      // eight 32 x 128 tiles: 64 KiB
    __shared__ float pad[8 * 1024];                                        // keeps it at one workgroup per CU
    if (iters < 0) pad[threadIdx.x] = 0.f;
    const int lane = threadIdx.x & 63, g = lane >> 5, ln = lane & 31;
    const e16x8* src = reinterpret_cast<const e16x8*>(data);
    for (int i = threadIdx.x; i < 8 * 32 * 128 / 8; i += 256) reinterpret_cast<e16x8*>(tile)[i] = src[i];
    e16x8 b[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) b[t] = src[threadIdx.x + 512 * t + 256];
    __syncthreads();
    const uint32_t base = lds_addr(tile);
    uint32_t adr[8];                                 // row ln, chunk 2t+g of a swizzled tile: conflict-free row reads
#pragma unroll
    for (int t = 0; t < 8; ++t) adr[t] = base + 2 * tile_off<128>(ln, 2 * t + g);
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    e16x8 a0[8], a1[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) a0[t] = lds_b128<0>(adr[t]);
#pragma unroll 1
    for (int it = 0; it < iters; it += 2) {
        const uint32_t off1 = (uint32_t)((it + 1) & 7) * 8192u, off0 = (uint32_t)((it + 2) & 7) * 8192u;
#pragma unroll
        for (int t = 0; t < 8; ++t) a1[t] = lds_b128<0>(adr[t] + off1);
        wait_lgkm<8>();
        lds_tie(a0[0], a0[1], a0[2], a0[3], a0[4], a0[5], a0[6], a0[7]);
#pragma unroll
        for (int t = 0; t < 8; ++t) acc[t & 3] = mfma32(a0[t], b[t], acc[t & 3]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < 8; ++t) a0[t] = lds_b128<0>(adr[t] + off0);
        wait_lgkm<8>();
        lds_tie(a1[0], a1[1], a1[2], a1[3], a1[4], a1[5], a1[6], a1[7]);
#pragma unroll
        for (int t = 0; t < 8; ++t) acc[t & 3] = mfma32(a1[t], b[t], acc[t & 3]);
        __builtin_amdgcn_sched_barrier(0);
    }
    wait_lgkm<0>();
    lds_tie(a0[0], a0[1], a0[2], a0[3], a0[4], a0[5], a0[6], a0[7]);
    float tot = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) tot += acc[i][r];
    if (tot == 12345.678f) sink[blockIdx.x * 256 + threadIdx.x] = tot + pad[0] + (float)a0[0][0];
}

// data: at least kProbeBytes of device memory filled by the caller; sink: at least blocks*256 floats;
// lds_fed: one operand of every MFMA comes from LDS (iters is rounded up to an even number)
int mfma_probe_launch(const void* data, float* sink, int blocks, int iters, int lds_fed, void* stream) {
    if (lds_fed)
        mfma_lds_probe_kernel<<<dim3((uint32_t)blocks), dim3(256), 0, (hipStream_t)stream>>>((const e16*)data, sink,
                                                                                             (iters + 1) & ~1);
    else
        mfma_probe_kernel<<<dim3((uint32_t)blocks), dim3(256), 0, (hipStream_t)stream>>>((const e16*)data, sink, iters);
    return hipGetLastError() == hipSuccess ? ULY_OK : ULY_ERR_LAUNCH;
}
#endif

}  // namespace uly
