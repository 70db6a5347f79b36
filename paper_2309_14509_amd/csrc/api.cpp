// C ABI of libulysses: argument validation (no HIP call is made before it passes) and dispatch.
#include <stdint.h>

#include "internal.h"

namespace {

inline bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }

struct Range {
    const void* p;
    uint64_t bytes;
};

inline bool overlap(const Range& a, const Range& b) {
    if (a.bytes == 0 || b.bytes == 0) return false;
    const uintptr_t a0 = (uintptr_t)a.p, b0 = (uintptr_t)b.p;
    return a0 < b0 + b.bytes && b0 < a0 + a.bytes;
}

// Every output against every input and every other output.
template <int NI, int NO>
bool any_alias(const Range (&in)[NI], const Range (&out)[NO]) {
    for (int o = 0; o < NO; ++o) {
        for (int i = 0; i < NI; ++i)
            if (overlap(out[o], in[i])) return true;
        for (int o2 = o + 1; o2 < NO; ++o2)
            if (overlap(out[o], out[o2])) return true;
    }
    return false;
}

// Common checks of the four layout transforms; on success *total_bytes is the tensor size.
int check_layout_args(const void* src, const void* dst, int64_t n_local, int H, int d, int P, int elem_bytes,
                      int layout, uint64_t* total_bytes) {
    if (n_local < 0 || H <= 0 || d <= 0 || P <= 0 || H % P != 0) return ULY_ERR_SHAPE;
    if (elem_bytes != 1 && elem_bytes != 2 && elem_bytes != 4) return ULY_ERR_UNSUPPORTED;
    if (layout != ULY_LAYOUT_SEQ_HEAD && layout != ULY_LAYOUT_HEAD_SEQ) return ULY_ERR_UNSUPPORTED;
    const uint64_t row_bytes = (uint64_t)H * (uint64_t)d * (uint64_t)elem_bytes;   // < 2^64: three ints
    if (row_bytes >= (1ull << 40)) return ULY_ERR_SHAPE;
    if ((uint64_t)n_local >= (1ull << 62) / row_bytes) return ULY_ERR_SHAPE;
    if ((uint64_t)n_local * (uint64_t)P >= (1ull << 40)) return ULY_ERR_SHAPE;      // N = P * n_local
    *total_bytes = (uint64_t)n_local * row_bytes;
    if (*total_bytes == 0) return ULY_OK;                                           // nothing to move
    if (!src || !dst) return ULY_ERR_NULL;
    if (misaligned(src) || misaligned(dst)) return ULY_ERR_ALIGN;
    const Range in[1] = {{src, *total_bytes}}, out[1] = {{dst, *total_bytes}};
    if (any_alias(in, out)) return ULY_ERR_ALIAS;
    return ULY_OK;
}

// Checks of the three-tensor transforms: each (src, dst) pair as above, and no output may overlap any
// input or another output.
int check_layout_args3(const void* const src[3], void* const dst[3], int64_t n_local, int H, int d, int P,
                       int elem_bytes, int layout, uint64_t* total_bytes) {
    if (!src || !dst) {
        // the pointer arrays themselves are required even for empty tensors
        return ULY_ERR_NULL;
    }
    for (int t = 0; t < 3; ++t) {
        const int rc = check_layout_args(src[t], dst[t], n_local, H, d, P, elem_bytes, layout, total_bytes);
        if (rc != ULY_OK) return rc;
    }
    if (*total_bytes == 0) return ULY_OK;
    const Range in[3] = {{src[0], *total_bytes}, {src[1], *total_bytes}, {src[2], *total_bytes}};
    const Range out[3] = {{dst[0], *total_bytes}, {dst[1], *total_bytes}, {dst[2], *total_bytes}};
    if (any_alias(in, out)) return ULY_ERR_ALIAS;
    return ULY_OK;
}

int check_attn_common(int64_t N, int Hl, int d, int layout, uint64_t* tensor_bytes) {
    if (N < 0 || Hl <= 0 || d <= 0) return ULY_ERR_SHAPE;
    if (d != 64 && d != 128 && d != 256) return ULY_ERR_UNSUPPORTED;
    layout &= ~ULY_ELEM_F16;                                           // the element type flag rides on the layout word
    if (layout != ULY_LAYOUT_SEQ_HEAD && layout != ULY_LAYOUT_HEAD_SEQ) return ULY_ERR_UNSUPPORTED;
    if (N >= (1ll << 31)) return ULY_ERR_SHAPE;                       // tile counters are 32-bit
    if ((uint64_t)N * (uint64_t)Hl >= (1ull << 40)) return ULY_ERR_SHAPE;
    if ((uint64_t)Hl * (uint64_t)d > (1ull << 22)) return ULY_ERR_SHAPE;    // in-tile byte offsets are 32-bit
    *tensor_bytes = (uint64_t)N * (uint64_t)Hl * (uint64_t)d * 2u;
    return ULY_OK;
}

}  // namespace

extern "C" {

int ulysses_pack(const void* x, void* send, int64_t n_local, int H, int d, int P, int elem_bytes, void* stream) {
    uint64_t bytes;
    const int rc = check_layout_args(x, send, n_local, H, d, P, elem_bytes, ULY_LAYOUT_SEQ_HEAD, &bytes);
    if (rc != ULY_OK) return rc;
    return uly::regroup(x, send, n_local, P, (int64_t)(H / P) * d * elem_bytes, /*to_b=*/true, stream);
}

int ulysses_pack_qkv(const void* const x[3], void* const send[3], int64_t n_local, int H, int d, int P,
                     int elem_bytes, void* stream) {
    uint64_t bytes = 0;
    const int rc = check_layout_args3(x, send, n_local, H, d, P, elem_bytes, ULY_LAYOUT_SEQ_HEAD, &bytes);
    if (rc != ULY_OK || bytes == 0) return rc;
    return uly::regroup_multi(x, send, 3, n_local, P, (int64_t)(H / P) * d * elem_bytes, /*to_b=*/true, stream);
}

int ulysses_unpack_qkv(const void* const recv[3], void* const y[3], int64_t n_local, int H, int d, int P,
                       int elem_bytes, int out_layout, void* stream) {
    uint64_t bytes = 0;
    const int rc = check_layout_args3(recv, y, n_local, H, d, P, elem_bytes, out_layout, &bytes);
    if (rc != ULY_OK || bytes == 0) return rc;
    const int64_t N = n_local * P;
    const int Hl = H / P;
    if (out_layout == ULY_LAYOUT_SEQ_HEAD || Hl == 1)
        return uly::regroup_multi(recv, y, 3, N, 1, (int64_t)Hl * d * elem_bytes, true, stream);
    return uly::regroup_multi(recv, y, 3, N, Hl, (int64_t)d * elem_bytes, /*to_b=*/true, stream);
}

int ulysses_unpack_rev(const void* recv, void* y, int64_t n_local, int H, int d, int P, int elem_bytes,
                       void* stream) {
    uint64_t bytes;
    const int rc = check_layout_args(recv, y, n_local, H, d, P, elem_bytes, ULY_LAYOUT_SEQ_HEAD, &bytes);
    if (rc != ULY_OK) return rc;
    return uly::regroup(recv, y, n_local, P, (int64_t)(H / P) * d * elem_bytes, /*to_b=*/false, stream);
}

int ulysses_unpack(const void* recv, void* y, int64_t n_local, int H, int d, int P, int elem_bytes,
                   int out_layout, void* stream) {
    uint64_t bytes;
    const int rc = check_layout_args(recv, y, n_local, H, d, P, elem_bytes, out_layout, &bytes);
    if (rc != ULY_OK) return rc;
    const int64_t N = n_local * P;
    const int Hl = H / P;
    if (out_layout == ULY_LAYOUT_SEQ_HEAD || Hl == 1)       // same linear order: one straight copy
        return uly::regroup(recv, y, N, 1, (int64_t)Hl * d * elem_bytes, true, stream);
    return uly::regroup(recv, y, N, Hl, (int64_t)d * elem_bytes, /*to_b=*/true, stream);   // [N,Hl,d] -> [Hl,N,d]
}

int ulysses_pack_rev(const void* o, void* send, int64_t n_local, int H, int d, int P, int elem_bytes,
                     int in_layout, void* stream) {
    uint64_t bytes;
    const int rc = check_layout_args(o, send, n_local, H, d, P, elem_bytes, in_layout, &bytes);
    if (rc != ULY_OK) return rc;
    const int64_t N = n_local * P;
    const int Hl = H / P;
    if (in_layout == ULY_LAYOUT_SEQ_HEAD || Hl == 1)
        return uly::regroup(o, send, N, 1, (int64_t)Hl * d * elem_bytes, true, stream);
    return uly::regroup(o, send, N, Hl, (int64_t)d * elem_bytes, /*to_b=*/false, stream);  // [Hl,N,d] -> [N,Hl,d]
}

int ulysses_pack_rev_qkv(const void* const g[3], void* const send[3], int64_t n_local, int H, int d, int P,
                         int elem_bytes, int in_layout, void* stream) {
    uint64_t bytes = 0;
    const int rc = check_layout_args3(g, send, n_local, H, d, P, elem_bytes, in_layout, &bytes);
    if (rc != ULY_OK || bytes == 0) return rc;
    const int64_t N = n_local * P;
    const int Hl = H / P;
    if (in_layout == ULY_LAYOUT_SEQ_HEAD || Hl == 1)
        return uly::regroup_multi(g, send, 3, N, 1, (int64_t)Hl * d * elem_bytes, true, stream);
    return uly::regroup_multi(g, send, 3, N, Hl, (int64_t)d * elem_bytes, /*to_b=*/false, stream);
}

int ulysses_unpack_rev_qkv(const void* const recv[3], void* const y[3], int64_t n_local, int H, int d, int P,
                           int elem_bytes, void* stream) {
    uint64_t bytes = 0;
    const int rc = check_layout_args3(recv, y, n_local, H, d, P, elem_bytes, ULY_LAYOUT_SEQ_HEAD, &bytes);
    if (rc != ULY_OK || bytes == 0) return rc;
    return uly::regroup_multi(recv, y, 3, n_local, P, (int64_t)(H / P) * d * elem_bytes, /*to_b=*/false, stream);
}

// Shared by self-attention (Nk == N) and cross-attention (causal == 0, Nk keys for N queries).
static int attn_fwd_checked(const void* q, const void* k, const void* v, void* o, float* lse, void* workspace,
                            size_t workspace_bytes, bool takes_workspace, int64_t N, int64_t Nk, int Hl, int d,
                            float scale, int causal, int layout, void* stream) {
    uint64_t tb, tbk;
    int rc = check_attn_common(N, Hl, d, layout, &tb);
    if (rc == ULY_OK) rc = check_attn_common(Nk, Hl, d, layout, &tbk);
    if (rc != ULY_OK) return rc;
    if (!(scale > 0.0f) || scale - scale != 0.0f) return ULY_ERR_UNSUPPORTED;     // scale must be finite and > 0
    if (N == 0) return ULY_OK;
    if (Nk == 0) return ULY_ERR_SHAPE;                                             // softmax over no keys
    if (!q || !k || !v || !o || !lse) return ULY_ERR_NULL;
    const size_t need = !takes_workspace ? 0
                        : causal         ? ulysses_attn_fwd_workspace_bytes(N, Hl, d, 1)
                                         : ulysses_xattn_fwd_workspace_bytes(N, Nk, Hl, d);
    if (need > 0 && (!workspace || workspace_bytes < need)) return ULY_ERR_WORKSPACE;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(lse)) return ULY_ERR_ALIGN;
    if (need > 0 && misaligned(workspace)) return ULY_ERR_ALIGN;
    const Range in[3] = {{q, tb}, {k, tbk}, {v, tbk}};
    const Range out[3] = {{o, tb}, {lse, (uint64_t)N * Hl * 4u}, {need > 0 ? workspace : nullptr, need}};
    if (any_alias(in, out)) return ULY_ERR_ALIAS;
    const int lay = layout & ~ULY_ELEM_F16;
    return (layout & ULY_ELEM_F16 ? uly::f16::attn_fwd_launch : uly::bf16::attn_fwd_launch)(
        q, k, v, o, lse, need > 0 ? (float*)workspace : nullptr, N, Nk, Hl, d, scale, causal != 0,
        uly::strides_for(lay, N, Hl, d), uly::strides_for(lay, Nk, Hl, d), stream);
}

int ulysses_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse, int64_t N, int Hl, int d,
                     float scale, int causal, int layout, void* stream) {
    return attn_fwd_checked(q, k, v, o, lse, nullptr, 0, false, N, N, Hl, d, scale, causal, layout, stream);
}

size_t ulysses_attn_fwd_workspace_bytes(int64_t N, int Hl, int d, int causal) {
    if (!causal) return ulysses_xattn_fwd_workspace_bytes(N, N, Hl, d);
    uint64_t tb;
    if (N <= 0 || check_attn_common(N, Hl, d, ULY_LAYOUT_SEQ_HEAD, &tb) != ULY_OK) return 0;
    return (size_t)uly::bf16::attn_fwd_causal_workspace_floats(N, Hl, d) * sizeof(float);
}

int ulysses_attn_fwd_ws(const void* q, const void* k, const void* v, void* o, float* lse, void* workspace,
                        size_t workspace_bytes, int64_t N, int Hl, int d, float scale, int causal, int layout,
                        void* stream) {
    return attn_fwd_checked(q, k, v, o, lse, workspace, workspace_bytes, true, N, N, Hl, d, scale, causal, layout, stream);
}

size_t ulysses_xattn_fwd_workspace_bytes(int64_t Nq, int64_t Nk, int Hl, int d) {
    uint64_t tb;
    if (Nq <= 0 || Nk <= 0 || check_attn_common(Nq, Hl, d, ULY_LAYOUT_SEQ_HEAD, &tb) != ULY_OK ||
        check_attn_common(Nk, Hl, d, ULY_LAYOUT_SEQ_HEAD, &tb) != ULY_OK)
        return 0;
    return (size_t)uly::bf16::attn_fwd_cut_workspace_floats(Nq, Nk, Hl, d) * sizeof(float);
}

int ulysses_xattn_fwd(const void* q, const void* k, const void* v, void* o, float* lse, void* workspace,
                      size_t workspace_bytes, int64_t Nq, int64_t Nk, int Hl, int d, float scale, int layout,
                      void* stream) {
    return attn_fwd_checked(q, k, v, o, lse, workspace, workspace_bytes, true, Nq, Nk, Hl, d, scale, 0, layout, stream);
}

size_t ulysses_attn_bwd_workspace_bytes(int64_t N, int Hl, int d) {
    (void)d;
    if (N <= 0 || Hl <= 0) return 0;
    return (size_t)uly::bf16::attn_bwd_workspace_floats(N, Hl) * sizeof(float);      // the same for both element types
}

size_t ulysses_xattn_bwd_workspace_bytes(int64_t Nq, int64_t Nk, int Hl, int d) {
    uint64_t tb;
    if (Nq <= 0 || Nk <= 0 || check_attn_common(Nq, Hl, d, ULY_LAYOUT_SEQ_HEAD, &tb) != ULY_OK ||
        check_attn_common(Nk, Hl, d, ULY_LAYOUT_SEQ_HEAD, &tb) != ULY_OK)
        return ulysses_attn_bwd_workspace_bytes(Nq, Hl, d);
    return (size_t)uly::bf16::attn_bwd_cut_workspace_floats(Nq, Nk, Hl, d) * sizeof(float);
}

static int attn_bwd_checked(int stage_mask, const void* q, const void* k, const void* v, const void* o,
                            const void* dout, const float* lse, void* dq, void* dk, void* dv, void* workspace,
                            size_t workspace_bytes, int64_t N, int64_t Nk, int Hl, int d, float scale, int causal,
                            int may_cut, int layout, void* stream) {
    uint64_t tb, tbk;
    int rc = check_attn_common(N, Hl, d, layout, &tb);
    if (rc == ULY_OK) rc = check_attn_common(Nk, Hl, d, layout, &tbk);
    if (rc != ULY_OK) return rc;
    if (!(scale > 0.0f) || scale - scale != 0.0f) return ULY_ERR_UNSUPPORTED;
    if (N == 0 && Nk == 0) return ULY_OK;
    if (N == 0 || Nk == 0) return ULY_ERR_SHAPE;          // gradients of an empty side are not defined here
    if (!q || !k || !v || !o || !dout || !lse || !dq || !dk || !dv) return ULY_ERR_NULL;
    const size_t need = may_cut ? ulysses_xattn_bwd_workspace_bytes(N, Nk, Hl, d) : ulysses_attn_bwd_workspace_bytes(N, Hl, d);
    if (need > 0 && (!workspace || workspace_bytes < need)) return ULY_ERR_WORKSPACE;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(dout) || misaligned(lse) ||
        misaligned(dq) || misaligned(dk) || misaligned(dv) || misaligned(workspace))
        return ULY_ERR_ALIGN;
    const uint64_t lb = (uint64_t)N * Hl * 4u;
    const Range in[6] = {{q, tb}, {k, tbk}, {v, tbk}, {o, tb}, {dout, tb}, {lse, lb}};
    const Range out[4] = {{dq, tb}, {dk, tbk}, {dv, tbk}, {workspace, need}};
    if (any_alias(in, out)) return ULY_ERR_ALIAS;
    const int lay = layout & ~ULY_ELEM_F16;
    return (layout & ULY_ELEM_F16 ? uly::f16::attn_bwd_launch : uly::bf16::attn_bwd_launch)(
        stage_mask, q, k, v, o, dout, lse, dq, dk, dv, (float*)workspace, N, Nk, Hl, d, scale, causal != 0, may_cut,
        uly::strides_for(lay, N, Hl, d), uly::strides_for(lay, Nk, Hl, d), stream);
}

int ulysses_attn_bwd(const void* q, const void* k, const void* v, const void* o, const void* dout, const float* lse,
                     void* dq, void* dk, void* dv, void* workspace, size_t workspace_bytes, int64_t N, int Hl,
                     int d, float scale, int causal, int layout, void* stream) {
    return attn_bwd_checked(7, q, k, v, o, dout, lse, dq, dk, dv, workspace, workspace_bytes, N, N, Hl, d, scale,
                            causal, /*may_cut=*/0, layout, stream);
}

int ulysses_attn_bwd_stage(int stage, const void* q, const void* k, const void* v, const void* o, const void* dout,
                           const float* lse, void* dq, void* dk, void* dv, void* workspace, size_t workspace_bytes,
                           int64_t N, int Hl, int d, float scale, int causal, int layout, void* stream) {
    if (stage != ULY_BWD_STAGE_DELTA && stage != ULY_BWD_STAGE_DKV && stage != ULY_BWD_STAGE_DQ)
        return ULY_ERR_UNSUPPORTED;
    return attn_bwd_checked(1 << stage, q, k, v, o, dout, lse, dq, dk, dv, workspace, workspace_bytes, N, N, Hl, d,
                            scale, causal, /*may_cut=*/0, layout, stream);
}

int ulysses_xattn_bwd(const void* q, const void* k, const void* v, const void* o, const void* dout, const float* lse,
                      void* dq, void* dk, void* dv, void* workspace, size_t workspace_bytes, int64_t Nq, int64_t Nk,
                      int Hl, int d, float scale, int layout, void* stream) {
    return attn_bwd_checked(7, q, k, v, o, dout, lse, dq, dk, dv, workspace, workspace_bytes, Nq, Nk, Hl, d, scale, 0,
                            /*may_cut=*/1, layout, stream);
}

size_t ulysses_sparse_attn_fwd_workspace_bytes(int64_t N, int Hl, int d) {
    uint64_t tb;
    if (check_attn_common(N, Hl, d, ULY_LAYOUT_SEQ_HEAD, &tb) != ULY_OK || d == 256 || N == 0 || N > ULY_SPARSE_MAX_N)
        return 0;
    return (size_t)uly::bf16::attn_fwd_sparse_workspace_floats(N, Hl, d) * sizeof(float);
}

int ulysses_sparse_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse, const int32_t* row_ptr,
                            const int32_t* col_idx, void* workspace, size_t workspace_bytes, int64_t N, int Hl, int d,
                            float scale, int layout, void* stream) {
    uint64_t tb;
    const int rc = check_attn_common(N, Hl, d, layout, &tb);
    if (rc != ULY_OK) return rc;
    if (d == 256) return ULY_ERR_UNSUPPORTED;                    // the sparse kernels exist for d = 64 and 128
    if (!(scale > 0.0f) || scale - scale != 0.0f) return ULY_ERR_UNSUPPORTED;
    if (N == 0) return ULY_OK;
    if (N > ULY_SPARSE_MAX_N) return ULY_ERR_SHAPE;              // the work items are a grid dimension
    if (!q || !k || !v || !o || !lse || !row_ptr || !col_idx) return ULY_ERR_NULL;
    const size_t need = ulysses_sparse_attn_fwd_workspace_bytes(N, Hl, d);
    if (!workspace || workspace_bytes < need) return ULY_ERR_WORKSPACE;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(lse) || misaligned(workspace))
        return ULY_ERR_ALIGN;
    if (((uintptr_t)row_ptr | (uintptr_t)col_idx) & 3u) return ULY_ERR_ALIGN;
    const Range in[3] = {{q, tb}, {k, tb}, {v, tb}};
    const Range out[3] = {{o, tb}, {lse, (uint64_t)N * Hl * 4u}, {workspace, need}};
    if (any_alias(in, out)) return ULY_ERR_ALIAS;
    return (layout & ULY_ELEM_F16 ? uly::f16::attn_fwd_sparse_launch : uly::bf16::attn_fwd_sparse_launch)(
        q, k, v, o, lse, (float*)workspace, row_ptr, col_idx, N, Hl, d, scale,
        uly::strides_for(layout & ~ULY_ELEM_F16, N, Hl, d), stream);
}

size_t ulysses_sparse_attn_bwd_workspace_bytes(int64_t N, int Hl, int d) {
    uint64_t tb;
    if (check_attn_common(N, Hl, d, ULY_LAYOUT_SEQ_HEAD, &tb) != ULY_OK || d == 256 || N == 0 || N > ULY_SPARSE_MAX_N)
        return 0;
    return (size_t)uly::bf16::attn_bwd_sparse_workspace_floats(N, Hl, d) * sizeof(float);
}

int ulysses_sparse_attn_bwd(const void* q, const void* k, const void* v, const void* o, const void* dout,
                            const float* lse, void* dq, void* dk, void* dv, const int32_t* row_ptr,
                            const int32_t* col_idx, const int32_t* col_ptr, const int32_t* row_idx, void* workspace,
                            size_t workspace_bytes, int64_t N, int Hl, int d, float scale, int layout, void* stream) {
    uint64_t tb;
    const int rc = check_attn_common(N, Hl, d, layout, &tb);
    if (rc != ULY_OK) return rc;
    if (!(scale > 0.0f) || scale - scale != 0.0f) return ULY_ERR_UNSUPPORTED;
    if (d == 256) return ULY_ERR_UNSUPPORTED;
    if (N == 0) return ULY_OK;
    if (N > ULY_SPARSE_MAX_N) return ULY_ERR_SHAPE;          // the work items of dK/dV are a grid dimension
    if (!q || !k || !v || !o || !dout || !lse || !dq || !dk || !dv || !row_ptr || !col_idx || !col_ptr || !row_idx)
        return ULY_ERR_NULL;
    const size_t need = ulysses_sparse_attn_bwd_workspace_bytes(N, Hl, d);
    if (need > 0 && (!workspace || workspace_bytes < need)) return ULY_ERR_WORKSPACE;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(dout) || misaligned(lse) ||
        misaligned(dq) || misaligned(dk) || misaligned(dv) || misaligned(workspace))
        return ULY_ERR_ALIGN;
    if (((uintptr_t)row_ptr | (uintptr_t)col_idx | (uintptr_t)col_ptr | (uintptr_t)row_idx) & 3u) return ULY_ERR_ALIGN;
    const uint64_t lb = (uint64_t)N * Hl * 4u;
    const Range in[6] = {{q, tb}, {k, tb}, {v, tb}, {o, tb}, {dout, tb}, {lse, lb}};
    const Range out[4] = {{dq, tb}, {dk, tb}, {dv, tb}, {workspace, need}};
    if (any_alias(in, out)) return ULY_ERR_ALIAS;
    return (layout & ULY_ELEM_F16 ? uly::f16::attn_bwd_sparse_launch : uly::bf16::attn_bwd_sparse_launch)(
        q, k, v, o, dout, lse, dq, dk, dv, (float*)workspace, row_ptr, col_idx, col_ptr, row_idx, N, Hl, d, scale,
        uly::strides_for(layout & ~ULY_ELEM_F16, N, Hl, d), stream);
}

static int probe_checked(const void* data, size_t data_bytes, float* sink, size_t sink_bytes, int blocks, int iters,
                         int lds_fed, void* stream) {
    if (blocks <= 0 || iters <= 0 || blocks > 65536 || iters > (1 << 30)) return ULY_ERR_SHAPE;
    if (!data || !sink) return ULY_ERR_NULL;
    if (misaligned(data) || misaligned(sink)) return ULY_ERR_ALIGN;
    if (data_bytes < uly::kProbeBytes || sink_bytes < (size_t)blocks * 256 * sizeof(float)) return ULY_ERR_WORKSPACE;
    return uly::mfma_probe_launch(data, sink, blocks, iters, lds_fed, stream);
}

int ulysses_probe_mfma(const void* data, size_t data_bytes, float* sink, size_t sink_bytes, int blocks, int iters,
                       void* stream) {
    return probe_checked(data, data_bytes, sink, sink_bytes, blocks, iters, 0, stream);
}

int ulysses_probe_mfma_lds(const void* data, size_t data_bytes, float* sink, size_t sink_bytes, int blocks, int iters,
                           void* stream) {
    return probe_checked(data, data_bytes, sink, sink_bytes, blocks, iters, 1, stream);
}

const char* ulysses_status_string(int status) {
    switch (status) {
        case ULY_OK: return "ok";
        case ULY_ERR_NULL: return "a required pointer is NULL";
        case ULY_ERR_SHAPE: return "invalid shape (non-positive dimension, H not a multiple of P, or size overflow)";
        case ULY_ERR_UNSUPPORTED: return "unsupported head dimension, element size or layout";
        case ULY_ERR_ALIGN: return "pointer is not 16-byte aligned";
        case ULY_ERR_ALIAS: return "output buffer overlaps an input or another output";
        case ULY_ERR_WORKSPACE: return "workspace is NULL or too small";
        case ULY_ERR_LAUNCH: return "HIP kernel launch failed";
        default: return "unknown status";
    }
}

int ulysses_abi_version(void) { return 1; }

}  // extern "C"
