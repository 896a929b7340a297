// Internal declarations shared by the translation units of libtofu (not part of the C ABI).
#ifndef TOFU_INTERNAL_H_
#define TOFU_INTERNAL_H_

#include <stddef.h>
#include <stdint.h>

#include "tofu.h"

namespace tofu {

// Record a thread-local error message and return `code` (printf-style).
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

// Number of iteration dimensions of an operator kind (3 / 5 / 3 / 5), or 0 for an unknown kind.
int iter_ndim(int32_t kind);

// Index range of every iteration dimension left to one worker after applying the plan.
// Order of the dimensions follows the TOFU_*_DIM_* enumerators.
struct IterRanges {
  int64_t lo[5];
  int64_t hi[5];
};
int apply_splits(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits, IterRanges* r,
                 int32_t* is_partial);

// Checks of the operator description itself (positive sizes, output extents >= 1).
int check_op(const tofu_op_desc_t* op);
int64_t conv_out_extent(int64_t size, int64_t ksize, int64_t stride, int64_t pad);

// Element strides of a tensor: the given ones, or dense row-major over the extent when all are zero.
void effective_strides(const tofu_tensor_t* t, int64_t* stride);

// True when `outer` contains `inner` in every dimension (an empty inner box is contained in anything).
bool contains(const tofu_region_t* outer, const tofu_region_t* inner);
int64_t volume(const tofu_region_t* r);

// Validate a tensor argument: non-null, ndim as expected, lo <= hi, and extent contains `need`.
int check_tensor(const char* name, const tofu_tensor_t* t, int32_t ndim, const tofu_region_t* need);

// Proof that the boxes of `srcs` tile the box `want` exactly once they are clipped to it:
// pairwise disjoint (else TOFU_ERR_OVERLAP) and of the same total volume (else TOFU_ERR_UNCOVERED).
// inter[j] receives the clipped box of srcs[j] (possibly empty); sources that hold part of the
// box must have a data pointer.  `name` labels the array in error messages.
int check_tiling(const char* name, const tofu_region_t* want, const tofu_tensor_t* srcs, int32_t nsrc, tofu_region_t* inter);

// Pointer to the element at global coordinate `coord` (which must lie inside the extent).
const float* element_ptr(const tofu_tensor_t* t, const int64_t* stride, const int64_t* coord);

// Lowest and one-past-highest byte address touched when the box `box` of tensor `t` (which must
// lie inside t's extent) is read or written through the element strides `stride`.
void box_byte_span(const tofu_tensor_t* t, const int64_t* stride, const tofu_region_t* box, const char** lo, const char** hi);

// ---- launch plans (shared by tofu_workspace_bytes and the entry points) ----
// Number of K slices the matmul kernel cuts its own reduction into for an m x n x k shard.
int matmul_split_k(int64_t m, int64_t n, int64_t k);
// Workspace the weight-gradient kernel needs for a shard of co x ci output channels and nb images of ho x wo outputs.
size_t wgrad_workspace_bytes(int64_t co, int64_t ci, int64_t nb, int64_t ho, int64_t wo);

// Workspace the convolution kernels need for a shard of P positions in BH x BW output boxes with
// co output and ci input channels (the segment slots of its balanced last wave, possibly 0).
size_t conv_workspace_bytes(int64_t P, int64_t BH, int64_t BW, int64_t co, int64_t ci, int KH = 3, int KW = 3);

// Columns per chunk the conv1d shard cuts an output row of `bw` columns into (a divisor of bw):
// the convolution kernel then sees bw / chunk rows of `chunk` columns whose windows overlap.
int64_t conv1d_chunk(int64_t bw);

// Enqueue dst[i] = sum_j parts[j][i] (fixed order j = 0..k-1); used by the public reduce and
// by the kernels that split their own reduction.  Pointers are device pointers.
int launch_reduce(float* dst, const float* const* parts, int k, int64_t count, void* stream);
// The same with a reduction mode: 0 sum left to right, 1 sum pairwise, 2 / 3 product likewise, 4 max, 5 min.
int launch_reduce_mode(float* dst, const float* const* parts, int k, int64_t count, int mode, void* stream);

}  // namespace tofu

#endif  // TOFU_INTERNAL_H_
