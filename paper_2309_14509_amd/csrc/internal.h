// Internal declarations shared by the translation units of libulysses (not part of the ABI).
#ifndef ULY_INTERNAL_H
#define ULY_INTERNAL_H

#include <stddef.h>
#include <stdint.h>

#include "../../include/ulysses.h"

namespace uly {

// A[rows][groups][run_bytes] <-> B[groups][rows][run_bytes] (to_b: dst is B).  Device pointers.
int regroup(const void* src, void* dst, int64_t rows, int64_t groups, int64_t run_bytes, bool to_b, void* stream);
// The same for `count` (<= kMaxTensors) tensors of one shape in a single launch.
constexpr int kMaxTensors = 3;
int regroup_multi(const void* const* src, void* const* dst, int count, int64_t rows, int64_t groups, int64_t run_bytes,
                  bool to_b, void* stream);

// Element strides (in bf16 elements) of a [token, head, channel] tensor in either layout.
struct TensorStrides {
    int64_t row;    // between consecutive tokens of one head
    int64_t head;   // between consecutive heads of one token
};

inline TensorStrides strides_for(int layout, int64_t N, int Hl, int d) {
    TensorStrides s;
    if (layout == ULY_LAYOUT_HEAD_SEQ) { s.row = d; s.head = N * (int64_t)d; }
    else { s.row = (int64_t)Hl * d; s.head = d; }
    return s;
}

// N queries attend to Nk keys/values (Nk = N for self-attention; causal requires Nk = N).  `st` are the
// strides of the query-side tensors (q, o, dout, dq), `kv` those of k, v, dk, dv.
int attn_fwd_launch(const void* q, const void* k, const void* v, void* o, float* lse, int64_t N, int64_t Nk, int Hl,
                    int d, float scale, int causal, TensorStrides st, TensorStrides kv, void* stream);

// MFMA-only probe (measurement aid): `blocks` workgroups of 256 lanes, `iters` x 8 MFMAs per wave.
constexpr size_t kProbeBytes = 64 * 1024;        // operand bytes read from `data`
int mfma_probe_launch(const void* data, float* sink, int blocks, int iters, void* stream);

// Block-sparse causal forward: keys restricted to the 256-key blocks of a CSR pattern (device arrays).
int attn_fwd_sparse_launch(const void* q, const void* k, const void* v, void* o, float* lse, const int* row_ptr,
                           const int* col_idx, int64_t N, int Hl, int d, float scale, TensorStrides st, void* stream);

// floats of scratch the backward kernels need (padded row statistics: delta and lse*log2e); N = queries
int64_t attn_bwd_workspace_floats(int64_t N, int Hl);

// stage_mask: bit 0 delta, bit 1 dK/dV, bit 2 dQ (kernels run in that order)
int attn_bwd_launch(int stage_mask, const void* q, const void* k, const void* v, const void* o, const void* dout,
                    const float* lse, void* dq, void* dk, void* dv, float* delta, int64_t N, int64_t Nk, int Hl, int d,
                    float scale, int causal, TensorStrides st, TensorStrides kv, void* stream);

// floats of scratch of the block-sparse backward: the statistics, the dK/dV work plan and the fp32
// partial sums of block columns that are cut into several work items
int64_t attn_bwd_sparse_workspace_floats(int64_t N, int Hl, int d);

// Block-sparse causal backward; row_ptr/col_idx list the block columns of each block row, col_ptr/row_idx
// the block rows of each block column (device arrays).
int attn_bwd_sparse_launch(const void* q, const void* k, const void* v, const void* o, const void* dout,
                           const float* lse, void* dq, void* dk, void* dv, float* delta, const int* row_ptr,
                           const int* col_idx, const int* col_ptr, const int* row_idx, int64_t N, int Hl, int d,
                           float scale, TensorStrides st, void* stream);

}  // namespace uly
#endif
