// Launch functions of the attention kernels.  internal.h includes this file once per element type,
// inside namespace uly::bf16 and inside namespace uly::f16 (no include guard on purpose); the
// attention sources are compiled once per element type and define the functions of their namespace.
// Sizes and strides count 16-bit elements.

// N queries attend to Nk keys/values (Nk = N for self-attention; causal requires Nk = N).  `st` are the
// strides of the query-side tensors (q, o, dout, dq), `kv` those of k, v, dk, dv.
// `ws` (may be null: then nothing is cut): scratch that lets attention with few query tiles cut the keys of a
// tile into several work items, merged by a second kernel: attn_fwd_cut_workspace_floats floats without a mask,
// attn_fwd_causal_workspace_floats with the causal mask.
int64_t attn_fwd_cut_workspace_floats(int64_t N, int64_t Nk, int Hl, int d);
int64_t attn_fwd_causal_workspace_floats(int64_t N, int Hl, int d);
int attn_fwd_launch(const void* q, const void* k, const void* v, void* o, float* lse, float* ws, int64_t N, int64_t Nk,
                    int Hl, int d, float scale, int causal, TensorStrides st, TensorStrides kv, void* stream);

// Block-sparse causal forward: keys restricted to the 256-key blocks of a CSR pattern (device arrays).
// `ws`: attn_fwd_sparse_workspace_floats floats of scratch (work plan; partial results of block rows that are cut).
int64_t attn_fwd_sparse_workspace_floats(int64_t N, int Hl, int d);
int attn_fwd_sparse_launch(const void* q, const void* k, const void* v, void* o, float* lse, float* ws,
                           const int* row_ptr, const int* col_idx, int64_t N, int Hl, int d, float scale,
                           TensorStrides st, void* stream);

// floats of scratch the backward kernels need (padded row statistics: delta and lse*log2e); N = queries
int64_t attn_bwd_workspace_floats(int64_t N, int Hl);

// floats of scratch when unmasked attention may cut its tiles into several work items (may_cut below):
// the statistics plus work plans and fp32 partial sums; equals attn_bwd_workspace_floats when nothing is cut
int64_t attn_bwd_cut_workspace_floats(int64_t N, int64_t Nk, int Hl, int d);

// stage_mask: bit 0 delta, bit 1 dK/dV, bit 2 dQ (kernels run in that order).  may_cut: without a mask,
// when one side has too few tiles to fill the device, its tiles are cut into work items (the workspace
// must then have attn_bwd_cut_workspace_floats floats).
int attn_bwd_launch(int stage_mask, const void* q, const void* k, const void* v, const void* o, const void* dout,
                    const float* lse, void* dq, void* dk, void* dv, float* delta, int64_t N, int64_t Nk, int Hl, int d,
                    float scale, int causal, int may_cut, TensorStrides st, TensorStrides kv, void* stream);

// floats of scratch of the block-sparse backward: the statistics, the dK/dV work plan and the fp32
// partial sums of block columns that are cut into several work items
int64_t attn_bwd_sparse_workspace_floats(int64_t N, int Hl, int d);

// Block-sparse causal backward; row_ptr/col_idx list the block columns of each block row, col_ptr/row_idx
// the block rows of each block column (device arrays).
int attn_bwd_sparse_launch(const void* q, const void* k, const void* v, const void* o, const void* dout,
                           const float* lse, void* dq, void* dk, void* dv, float* delta, const int* row_ptr,
                           const int* col_idx, const int* col_ptr, const int* row_idx, int64_t N, int Hl, int d,
                           float scale, TensorStrides st, void* stream);

// Head dimension 256 (attn_d256.hip): simpler kernels, no work plans.  The backward launcher runs the dK/dV
// (bit 1) and dQ (bit 2) stages on statistics the caller has produced with the delta kernel.
int attn256_fwd_launch(const void* q, const void* k, const void* v, void* o, float* lse, int64_t N, int64_t Nk, int Hl,
                       float scale, int causal, TensorStrides st, TensorStrides kv, void* stream);
int attn256_bwd_launch(int stage_mask, const void* q, const void* k, const void* v, const void* dout, const float* delta,
                       const float* lse2, int64_t stride, void* dq, void* dk, void* dv, int64_t N, int64_t Nk, int Hl,
                       float scale, int causal, TensorStrides st, TensorStrides kv, void* stream);

// Work plan of a block-sparse kernel, made on the device from one of the pattern's pointer arrays (mode 0: key
// tiles of dK/dV from col_ptr, 1: query tiles of dQ from row_ptr, 2: query tiles of the forward from row_ptr):
// tiles whose walk is long are cut into items; plan = int4[1 + items], red = int2[tiles].
int sparse_plan_launch(int mode, const int* ptr, int64_t n_tiles, int64_t N, int Hl, int slots_per_head, int target,
                       void* plan, void* red, void* stream);
