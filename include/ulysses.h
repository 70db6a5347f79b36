/*
 * ulysses.h - C ABI of the single-GPU share of Ulysses sequence parallelism on MI355X (gfx950).
 *
 * One GPU's work inside a sequence-parallel attention layer (paper Section 3.1, Figure 2):
 *
 *   x [N/P, H, d]  --ulysses_pack-->  P send chunks  ==(all-to-all, NOT in this library)==>
 *   P received chunks  --ulysses_unpack-->  [N, H/P, d]  --ulysses_attn_fwd/bwd (Equation 1)-->
 *   o [N, H/P, d]  --ulysses_pack_rev-->  P send chunks  ==(all-to-all)==>  --ulysses_unpack_rev--> [N/P, H, d]
 *
 * Conventions shared by every entry point
 *  - All data pointers are DEVICE pointers (hipMalloc'd or equivalent), 16-byte aligned, owned by the
 *    caller.  The library allocates nothing, keeps no state between calls and never synchronises.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is enqueued
 *    asynchronously on it; outputs are valid once the stream reaches the end of the enqueued work.
 *  - Tensors are dense, row-major, last index fastest.  Sources and destinations must not overlap.
 *  - Every function returns a ULY_* status.  All argument validation happens before the first HIP
 *    call, so bad arguments are reported without touching the device.  Nothing is printed, thrown
 *    or aborted.  A size of zero tokens is valid, does nothing, and does not look at the pointers.
 *  - Head ownership is block-contiguous (rank p owns heads [p*H/P, (p+1)*H/P)) and sequence shards
 *    are contiguous in rank order (rank q holds tokens [q*N/P, (q+1)*N/P)).  The paper only requires
 *    non-overlapping head subsets and a partitioned sequence; these are the fixed choices that make
 *    the byte layout unique.  H must be a multiple of P.
 */
#ifndef ULYSSES_H
#define ULYSSES_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    ULY_OK = 0,
    ULY_ERR_NULL = 1,        /* a required pointer is NULL                                   */
    ULY_ERR_SHAPE = 2,       /* zero/negative dimension, H % P != 0, size overflow           */
    ULY_ERR_UNSUPPORTED = 3, /* head dim not in {64,128}, layout enum, element size, scale<=0 */
    ULY_ERR_ALIGN = 4,       /* a pointer is not 16-byte aligned                             */
    ULY_ERR_ALIAS = 5,       /* an output range overlaps an input (or another output) range  */
    ULY_ERR_WORKSPACE = 6,   /* workspace NULL or smaller than the *_workspace_bytes() value */
    ULY_ERR_LAUNCH = 7       /* the HIP runtime refused a launch                             */
};

enum {
    ULY_LAYOUT_SEQ_HEAD = 0, /* [N, Hl, d]  token-major (default)  */
    ULY_LAYOUT_HEAD_SEQ = 1  /* [Hl, N, d]  head-major             */
};

/* Element type of the attention entry points: OR this flag into their `layout` argument when
 * q, k, v, o, dout, dq, dk, dv hold IEEE fp16 instead of bf16 (lse and the workspace do not
 * change).  The layout transforms ignore element types (they take elem_bytes) and reject the flag. */
enum {
    ULY_ELEM_BF16 = 0,
    ULY_ELEM_F16 = 0x100
};

/* ---------------------------------------------------------------------------------------------
 * Layout transforms around the two all-to-alls (Section 3.1; message sizes in Section 3.2).
 * Pure data movement of `elem_bytes`-sized elements (1, 2 or 4); results are bit-exact.
 * n_local = N/P tokens held by this rank, H total heads, d head dimension, P ranks, Hl = H/P.
 * ------------------------------------------------------------------------------------------- */

/* Send side of the first all-to-all.
 *   x    [n_local, H, d]        in
 *   send [P, n_local, Hl, d]    out;  send[p, n, hl, :] = x[n, p*Hl + hl, :]
 * Chunk p is the contiguous message for destination rank p. */
int ulysses_pack(const void* x, void* send, int64_t n_local, int H, int d, int P,
                 int elem_bytes, void* stream);

/* Receive side of the first all-to-all.
 *   recv [P, n_local, Hl, d]    in;  chunk q arrived from source rank q
 *   y    [P*n_local, Hl, d]     out  (ULY_LAYOUT_SEQ_HEAD):  y[q*n_local + n, hl, :] = recv[q, n, hl, :]
 *        [Hl, P*n_local, d]     out  (ULY_LAYOUT_HEAD_SEQ):  y[hl, q*n_local + n, :] = recv[q, n, hl, :] */
int ulysses_unpack(const void* recv, void* y, int64_t n_local, int H, int d, int P,
                   int elem_bytes, int out_layout, void* stream);

/* Q, K and V in one launch: the paper sends the three tensors as one all-to-all message of 3Nh
 * elements (Section 3.2), so their layout transforms are issued together.  `x`, `send` (`recv`, `y`)
 * are HOST arrays of three device pointers; tensor t is transformed exactly as by ulysses_pack
 * (ulysses_unpack).  All three share one shape; no output may overlap any input or other output.
 * The arrays are read before the call returns. */
int ulysses_pack_qkv(const void* const x[3], void* const send[3], int64_t n_local, int H, int d, int P,
                     int elem_bytes, void* stream);
int ulysses_unpack_qkv(const void* const recv[3], void* const y[3], int64_t n_local, int H, int d, int P,
                       int elem_bytes, int out_layout, void* stream);

/* Send side of the second all-to-all (attention output back to sequence-parallel form).
 *   o    [P*n_local, Hl, d] or [Hl, P*n_local, d] (in_layout)   in
 *   send [P, n_local, Hl, d]    out;  send[q, n, hl, :] = o(token q*n_local + n, head hl) */
int ulysses_pack_rev(const void* o, void* send, int64_t n_local, int H, int d, int P,
                     int elem_bytes, int in_layout, void* stream);

/* Receive side of the second all-to-all.
 *   recv [P, n_local, Hl, d]    in;  chunk p arrived from the rank owning heads [p*Hl, (p+1)*Hl)
 *   y    [n_local, H, d]        out; y[n, p*Hl + hl, :] = recv[p, n, hl, :] */
int ulysses_unpack_rev(const void* recv, void* y, int64_t n_local, int H, int d, int P,
                       int elem_bytes, void* stream);

/* The reverse transforms for three tensors of one shape in one launch: the backward pass returns
 * dQ, dK and dV to sequence-parallel form the way the forward pass brought Q, K and V in (the
 * gradient of an all-to-all is the opposite all-to-all, Section 3.1).  HOST arrays of three device
 * pointers, as for ulysses_pack_qkv; tensor t is transformed exactly as by ulysses_pack_rev
 * (ulysses_unpack_rev). */
int ulysses_pack_rev_qkv(const void* const g[3], void* const send[3], int64_t n_local, int H, int d, int P,
                         int elem_bytes, int in_layout, void* stream);
int ulysses_unpack_rev_qkv(const void* const recv[3], void* const y[3], int64_t n_local, int H, int d, int P,
                           int elem_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Exact softmax attention per local head, Equation 1:  O = Softmax(Q K^T * scale) V,
 * softmax over keys.  causal != 0 restricts query i to keys j <= i (global token positions,
 * diagonal included).  q, k, v, o, dout, dq, dk, dv are bf16 in `layout` (fp16 with
 * layout | ULY_ELEM_F16; this holds for the cross- and sparse-attention entry points too);
 * arithmetic is 16-bit MFMA with fp32 accumulation and fp32 softmax; outputs are rounded to the
 * element type (nearest even).  The paper does not state a precision.
 * N tokens (0 <= N < 2^31), Hl local heads with Hl * d <= 2^22, d in {64, 128, 256} (ULY_ERR_SHAPE /
 * ULY_ERR_UNSUPPORTED otherwise; d = 256 runs simpler, slower kernels and is not available for the
 * block-sparse entry points).  `scale` is normally 1/sqrt(d) and must
 * be finite and > 0 (anything else is ULY_ERR_UNSUPPORTED).
 * ------------------------------------------------------------------------------------------- */

/* Forward.
 *   lse [Hl, N] fp32 out: natural-log sum-exp of the scaled, masked logits of every query row.
 *   It is the only state besides o that the backward pass needs. */
int ulysses_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                     int64_t N, int Hl, int d, float scale, int causal, int layout, void* stream);

/* Forward with a workspace (for callers that can give one): the same quantities as ulysses_attn_fwd
 * (the same bits when nothing is cut, otherwise equal up to the order of fp32 sums).  When the
 * sequence is short enough that one workgroup per 256 queries would leave much of the device idle (fewer
 * than 1024 such tiles over all heads), the keys of long rows are cut into several work items whose fp32
 * partial results a second kernel merges in a fixed order.  ulysses_attn_fwd_workspace_bytes is 0 when
 * nothing would be cut (workspace may then be NULL) and stays below 600 MiB otherwise; ULY_ERR_WORKSPACE
 * if the workspace is NULL or too small, ULY_ERR_ALIGN if it is not 16-byte aligned. */
size_t ulysses_attn_fwd_workspace_bytes(int64_t N, int Hl, int d, int causal);
int ulysses_attn_fwd_ws(const void* q, const void* k, const void* v, void* o, float* lse,
                        void* workspace, size_t workspace_bytes,
                        int64_t N, int Hl, int d, float scale, int causal, int layout, void* stream);

/* Bytes of device scratch the backward pass needs (two fp32 per query row and head, rows padded). */
size_t ulysses_attn_bwd_workspace_bytes(int64_t N, int Hl, int d);

/* Backward: gradients of sum(O * dout) with respect to q, k, v.  The probabilities are recomputed
 * from q, k and the saved lse; o is used only for the row terms D_i = dout_i . o_i.
 *   workspace: device scratch of at least ulysses_attn_bwd_workspace_bytes() bytes, 16-byte aligned;
 *   its contents on entry are ignored and on exit unspecified.
 * Results are deterministic (no atomics): the same inputs give the same bits. */
int ulysses_attn_bwd(const void* q, const void* k, const void* v, const void* o, const void* dout,
                     const float* lse, void* dq, void* dk, void* dv,
                     void* workspace, size_t workspace_bytes,
                     int64_t N, int Hl, int d, float scale, int causal, int layout, void* stream);

/* One stage of ulysses_attn_bwd, with the same arguments and the same checks.  Calling stages
 * ULY_BWD_STAGE_DELTA, ULY_BWD_STAGE_DKV, ULY_BWD_STAGE_DQ in that order on one stream is exactly
 * ulysses_attn_bwd; they exist so that a caller can time or overlap the kernels separately.
 *   DELTA: workspace <- row statistics dout_i . o_i and lse_i * log2(e)   (reads o, dout, lse)
 *   DKV  : dk, dv                            (reads q, k, v, dout, lse, workspace)
 *   DQ   : dq                                (reads q, k, v, dout, lse, workspace)
 * An unknown stage is ULY_ERR_UNSUPPORTED. */
enum { ULY_BWD_STAGE_DELTA = 0, ULY_BWD_STAGE_DKV = 1, ULY_BWD_STAGE_DQ = 2 };
int ulysses_attn_bwd_stage(int stage,
                           const void* q, const void* k, const void* v, const void* o, const void* dout,
                           const float* lse, void* dq, void* dk, void* dv,
                           void* workspace, size_t workspace_bytes,
                           int64_t N, int Hl, int d, float scale, int causal, int layout, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Cross-attention (Section 3.4 lists it beside self- and causal attention): Equation 1 with Nq
 * queries attending to Nk keys/values of the same local heads, no mask.
 *   q, o, dout, dq: Nq tokens;  k, v, dk, dv: Nk tokens;  all bf16 in `layout` (each tensor with its
 *   own token count: [Nq, Hl, d] / [Nk, Hl, d], or head-major);  lse [Hl, Nq] fp32.
 * Same arithmetic, precision and checks as the self-attention entry points.
 * Nq == 0 does nothing; Nk == 0 with Nq > 0 is ULY_ERR_SHAPE (a softmax over no keys).
 * Workspaces (caller-owned device memory, 16-byte aligned; ULY_ERR_WORKSPACE if too small): when
 * one side has too few tokens to occupy the device with one workgroup per tile, the other side of
 * each tile is cut into several work items whose fp32 partial results a second kernel merges in a
 * fixed order (deterministic).  ulysses_xattn_fwd_workspace_bytes is 0 for shapes that are not cut
 * (workspace may then be NULL); ulysses_xattn_bwd_workspace_bytes always covers the row statistics.
 * Both stay below about 600 MiB whatever the sizes.
 * ------------------------------------------------------------------------------------------- */
size_t ulysses_xattn_fwd_workspace_bytes(int64_t Nq, int64_t Nk, int Hl, int d);
int ulysses_xattn_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                      void* workspace, size_t workspace_bytes,
                      int64_t Nq, int64_t Nk, int Hl, int d, float scale, int layout, void* stream);
size_t ulysses_xattn_bwd_workspace_bytes(int64_t Nq, int64_t Nk, int Hl, int d);
int ulysses_xattn_bwd(const void* q, const void* k, const void* v, const void* o, const void* dout,
                      const float* lse, void* dq, void* dk, void* dv,
                      void* workspace, size_t workspace_bytes,
                      int64_t Nq, int64_t Nk, int Hl, int d, float scale, int layout, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Block-sparse causal attention.  The paper names blocked sparse attention among the supported
 * forms (Section 3.4) and evaluates it (Section 4.3) without fixing a pattern; here the caller gives
 * one: key j is visible to query i iff j <= i AND block (i / 256, j / 256) belongs to the pattern.
 * Equation 1 is evaluated over the visible keys; all local heads share the pattern.
 *
 * The pattern is a set of blocks of ULY_SPARSE_BLOCK x ULY_SPARSE_BLOCK tokens, nb = ceil(N / 256)
 * block rows and columns, given in compressed form as DEVICE arrays of int32:
 *   row_ptr [nb + 1], col_idx [nnz]: block row r sees block columns col_idx[row_ptr[r] .. row_ptr[r+1]),
 *       strictly ascending, every one <= r, and the last one == r (each diagonal block is required:
 *       a query always sees itself);
 *   col_ptr [nb + 1], row_idx [nnz]: the same set by columns (backward only): block column c is seen
 *       by block rows row_idx[col_ptr[c] .. col_ptr[c+1]), strictly ascending, the first one == c.
 * The arrays live in device memory, so the library cannot check their contents: a pattern that
 * breaks these rules is undefined behaviour (the Python binding builds and checks them on the host).
 * Other arguments, precision and status codes are those of ulysses_attn_fwd / _bwd with causal = 1;
 * the pattern arrays must be non-NULL and 4-byte aligned.
 * Workspaces (caller-owned device memory, 16-byte aligned, required for N > 0; the *_workspace_bytes
 * functions return 0 for a shape the library rejects).  Both hold a work plan that the library derives
 * from the pattern on the device: one workgroup per tile would leave the launch waiting for a few long
 * block rows or columns (global tokens, summary blocks), so tiles whose walk is long are cut into
 * several work items whose fp32 partial results a second kernel merges in a fixed order (results are
 * deterministic).  Forward: the plan and the partial results of cut block rows (at most four slots of
 * 256 queries x (d + 2) floats per query tile and head, and at most 2048 in all).  Backward: the row
 * statistics of the dense backward, plans, and partial sums of cut block columns (dK/dV: at most 8192
 * slots of 128 keys x d x 2 tensors, 1 GiB at d = 128, never more than two per 128 keys and head) and
 * of cut block rows (dQ: at most 4096 slots of 128 queries x d, never more than four per 128 queries
 * and head).  A pattern that would need more slots gets coarser cuts.
 * Sequences beyond ULY_SPARSE_MAX_N tokens are ULY_ERR_SHAPE (work items are a grid dimension).
 * ------------------------------------------------------------------------------------------- */
#define ULY_SPARSE_BLOCK 256
#define ULY_SPARSE_MAX_N 8000000
size_t ulysses_sparse_attn_fwd_workspace_bytes(int64_t N, int Hl, int d);
int ulysses_sparse_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                            const int32_t* row_ptr, const int32_t* col_idx,
                            void* workspace, size_t workspace_bytes,
                            int64_t N, int Hl, int d, float scale, int layout, void* stream);
size_t ulysses_sparse_attn_bwd_workspace_bytes(int64_t N, int Hl, int d);
int ulysses_sparse_attn_bwd(const void* q, const void* k, const void* v, const void* o, const void* dout,
                            const float* lse, void* dq, void* dk, void* dv,
                            const int32_t* row_ptr, const int32_t* col_idx,
                            const int32_t* col_ptr, const int32_t* row_idx,
                            void* workspace, size_t workspace_bytes,
                            int64_t N, int Hl, int d, float scale, int layout, void* stream);

/* Measurement aid for benchmarks (no paper counterpart): launches `blocks` workgroups (one per CU is
 * the intended use: blocks = number of CUs) of 4 waves that issue iters x 8 bf16 32x32x16 MFMAs each
 * and nothing else; 2 * 32*32*16 FLOP per MFMA.  Timed by the caller, it gives the matrix rate the
 * device sustains under its power limit on the data in `data`.
 *   data: device buffer of at least 65536 bytes, read as bf16 operands (fill it like real data);
 *   sink: device buffer of at least blocks * 256 floats (written only in a practically impossible case).
 * ULY_ERR_WORKSPACE if a buffer is too small. */
int ulysses_probe_mfma(const void* data, size_t data_bytes, float* sink, size_t sink_bytes,
                       int blocks, int iters, void* stream);
/* The same loop with one operand of every MFMA read from LDS (1 KiB per wave and MFMA, the way the
 * attention kernels feed their matrix pipe; the other operand stays in registers): the rate a kernel with
 * that operand traffic can reach at most.  iters is rounded up to an even number. */
int ulysses_probe_mfma_lds(const void* data, size_t data_bytes, float* sink, size_t sink_bytes,
                           int blocks, int iters, void* stream);

/* Static, NUL-terminated description of a status code (never NULL). */
const char* ulysses_status_string(int status);

/* Library ABI version (bumped when a signature changes). */
int ulysses_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ULYSSES_H */
