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

// Element strides (in 16-bit elements) of a [token, head, channel] tensor in either layout.
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

// MFMA-only probe (measurement aid): `blocks` workgroups of 256 lanes, `iters` x 8 MFMAs per wave; lds_fed: one
// operand of every MFMA is read from LDS instead of sitting in registers.
constexpr size_t kProbeBytes = 64 * 1024;        // operand bytes read from `data`
int mfma_probe_launch(const void* data, float* sink, int blocks, int iters, int lds_fed, void* stream);

// The attention kernels exist once per element type of Q, K, V, O and the gradients (accumulation
// and the softmax are fp32 either way).
namespace bf16 {
#include "attn_launch.h"
}
namespace f16 {
#include "attn_launch.h"
}

}  // namespace uly
#endif
