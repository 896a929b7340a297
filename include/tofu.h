/*
 * tofu.h -- C ABI of the shard hot path of Tofu's partition-n-reduce method
 * (arXiv 1807.08887) for one AMD MI355X (gfx950).
 *
 * One worker's share of a partitioned operator is: derive the worker's
 * coordinate ranges (Sec. 4.2, Case-1 / Case-2; Sec. 5.2 recursion), assemble
 * the input region it needs from the blocks that hold it (Sec. 6, fused remote
 * fetch), run the *same* operator on those smaller inputs (Sec. 3.1), and --
 * when a reduction dimension was split -- sum the k partial outputs
 * (Sec. 3.1 way 2; Sec. 6 output reduction).
 *
 * Conventions shared by every entry point
 *   - Element type is IEEE fp32 everywhere on the device.
 *   - A region is a half-open box [lo,hi) per dimension in the GLOBAL
 *     coordinates of the unpartitioned tensor.  The paper writes inclusive
 *     ranges [a,b]; that is [a,b+1) here.
 *   - A tofu_tensor_t describes a caller-owned DEVICE buffer holding the box
 *     `extent` of a global tensor.  stride[d] is the element stride of
 *     dimension d inside that buffer; stride[] all zero means dense row-major
 *     over the extent.  The library never allocates, frees or synchronises:
 *     every call only validates on the host and enqueues kernels on
 *     `hip_stream` (a hipStream_t passed as void*; NULL = the null stream).
 *   - Return value: TOFU_OK (0) or a negative tofu_status_t.  All argument
 *     checks happen on the host before anything is launched; after a failure
 *     tofu_last_error() returns a thread-local description.
 *   - Layouts: matmul A[M,K], B[K,N], C[M,N] row-major.  conv2d x[N,C_in,H,W],
 *     w[C_out,C_in,KH,KW] (output channel outermost), y[N,C_out,H_out,W_out].
 *     The convolution is a cross-correlation (index x+dx, no filter flip) as in
 *     the paper's conv1d loop nest (Fig. 1), with zero padding `pad`.  conv1d
 *     itself keeps the figure's shapes: data[B,C_in,W], filters[C_in,C_out,KW],
 *     out[B,C_out,W-KW+1], no padding.
 */
#ifndef TOFU_H_
#define TOFU_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TOFU_MAX_DIMS 6

typedef enum {
  TOFU_OK = 0,
  TOFU_ERR_INVALID_ARG = -1,        /* null pointer, bad ndim, k<1, shard outside [0,k), k>extent, bad dim */
  TOFU_ERR_REGION_MISMATCH = -2,    /* a tensor's extent does not contain the box the shard needs        */
  TOFU_ERR_UNCOVERED = -3,          /* fetch sources leave part of dst->extent without data              */
  TOFU_ERR_OVERLAP = -4,            /* two fetch sources both claim a coordinate of dst->extent          */
  TOFU_ERR_WORKSPACE_TOO_SMALL = -5,
  TOFU_ERR_UNSUPPORTED = -6,        /* operator parameters outside what the kernels implement            */
  TOFU_ERR_HIP = -7                 /* a HIP runtime call failed; see tofu_last_error()                  */
} tofu_status_t;

/* Tensor region (Sec. 4.2: a partition strategy is given by the input regions
 * each worker needs).  Half-open, global coordinates. */
typedef struct {
  int32_t ndim;
  int64_t lo[TOFU_MAX_DIMS];
  int64_t hi[TOFU_MAX_DIMS];
} tofu_region_t;

/* A device buffer that holds box `extent` of some global tensor. */
typedef struct {
  void* data;                       /* DEVICE pointer, fp32, caller-owned                     */
  tofu_region_t extent;             /* which global box the buffer holds                      */
  int64_t stride[TOFU_MAX_DIMS];    /* element strides; all 0 = dense row-major over extent   */
} tofu_tensor_t;

/* One basic partition step p_i (Appendix A.1): split ONE iteration dimension
 * of the operator k ways and keep part `shard`.  A plan is a sequence of
 * steps; each later step cuts the range left by the earlier ones (Sec. 5.2),
 * so <(d,2,a),(d,2,b)> is the quarter 2a+b of d when 4 divides the extent. */
typedef struct {
  int32_t dim;                      /* one of the TOFU_*_DIM_* names below, per operator kind */
  int32_t k;                        /* number of parts, >= 1                                  */
  int32_t shard;                    /* which part, 0 <= shard < k                             */
} tofu_split_t;

typedef enum {
  TOFU_OP_MATMUL = 0,               /* C[m,n]      = sum_k A[m,k] B[k,n]                                     */
  TOFU_OP_CONV2D = 1,               /* y[n,co,h,w] = sum_{ci,kh,kw} x[n,ci,h*s+kh-p,w*s+kw-p] w[co,ci,kh,kw] */
  TOFU_OP_CONV2D_WGRAD = 2,         /* dw[co,ci,kh,kw] = sum_{n,h,w} dy[n,co,h,w] x[n,ci,h*s+kh-p,w*s+kw-p]  */
  TOFU_OP_CONV2D_DGRAD = 3,         /* dx[n,ci,ih,iw]  = sum_{co,kh,kw} dy[n,co,h,w] w[co,ci,kh,kw] over the
                                       (h,w) with h*s+kh-p = ih, w*s+kw-p = iw                               */
  TOFU_OP_LSTM_CELL = 4,            /* element-wise over (b,h): c' = sig(f) c + sig(i) tanh(g), h' = sig(o) tanh(c')
                                       with (i,f,g,o) = gates[b,h,0..3]; shapes: batch = M, hidden units = N  */
  TOFU_OP_CONV1D = 5                /* the paper's running example (Fig. 1 and 3):
                                       out[b,co,x] = sum_{ci,dx} data[b,ci,x+dx] filters[ci,co,dx]; data is
                                       [batch, c_in, W], filters [c_in, c_out, KW], out [batch, c_out, W-KW+1];
                                       no padding, no stride (H, KH, stride, pad are not read)               */
} tofu_op_kind_t;

/* Iteration dimensions a split may name.  Output dimensions give Case-1
 * (concatenate, Sec. 4.2); reduction dimensions give Case-2 (the shard's
 * output is a full-size partial that tofu_partition_reduce must sum). */
enum { TOFU_MM_DIM_M = 0, TOFU_MM_DIM_N = 1, TOFU_MM_DIM_K = 2 /* reduction */ };
enum { TOFU_CONV_DIM_N = 0, TOFU_CONV_DIM_CO = 1, TOFU_CONV_DIM_H = 2, TOFU_CONV_DIM_W = 3,
       TOFU_CONV_DIM_CI = 4 /* reduction */ };
enum { TOFU_WGRAD_DIM_CO = 0, TOFU_WGRAD_DIM_CI = 1, TOFU_WGRAD_DIM_N = 2 /* reduction */ };
enum { TOFU_LSTM_DIM_B = 0, TOFU_LSTM_DIM_H = 1 };   /* element-wise: no reduction dimension */
/* data gradient: H and W are the rows / columns of dx, i.e. of the forward INPUT */
enum { TOFU_DGRAD_DIM_N = 0, TOFU_DGRAD_DIM_CI = 1, TOFU_DGRAD_DIM_H = 2, TOFU_DGRAD_DIM_W = 3,
       TOFU_DGRAD_DIM_CO = 4 /* reduction */ };

/* conv1d: an X split reads a window-widened range of data (never padding: the data tensor is
 * longer than the output by KW - 1) */
enum { TOFU_CONV1D_DIM_B = 0, TOFU_CONV1D_DIM_CO = 1, TOFU_CONV1D_DIM_X = 2, TOFU_CONV1D_DIM_CI = 3 /* reduction */ };

/* Operator description with the shapes of the UNPARTITIONED operator. */
typedef struct {
  int32_t kind;                     /* tofu_op_kind_t */
  int64_t M, N, K;                  /* matmul */
  int64_t batch, c_in, c_out, H, W; /* conv: input is [batch,c_in,H,W] */
  int64_t KH, KW, stride, pad;      /* conv: dilation 1, groups 1; output H_out = (H+2*pad-KH)/stride+1 */
} tofu_op_desc_t;

/* ---- host-only integer helpers (exact, no device work) ------------------ */

/* Part `shard` of a k-way even split of [0,extent) (Sec. 4.2 halves, Sec. 5.2
 * k_i-way steps): [floor(shard*extent/k), floor((shard+1)*extent/k)).  Parts
 * are disjoint, ordered, cover the extent and differ in size by at most one.
 * Errors: extent<0, k<1, shard outside [0,k), k>extent -> INVALID_ARG. */
int tofu_shard_range(int64_t extent, int32_t k, int32_t shard, int64_t* lo, int64_t* hi);

/* Regions of one shard (Sec. 4.2).  Applies `splits` in order to the
 * operator's iteration space and returns
 *   out_box      the box of the output tensor this shard writes (the whole
 *                output when only reduction dimensions were split),
 *   in_boxes[0]  the box of the first input it reads  (A | x | x  | dy | gates  | data),
 *   in_boxes[1]  the box of the second input it reads (B | w | dy | w  | c_prev | filters),
 *                in the order matmul | conv2d | wgrad | dgrad | lstm cell | conv1d,
 *   pad_lo/hi[2] conv only: rows/columns (index 0 = H, 1 = W) of the needed
 *                window that fall outside the global input on the low/high
 *                side and are therefore zeros; in_boxes[0] is already clipped,
 *   is_partial   1 when a reduction dimension was split (Case-2), else 0.
 * For conv spatial splits the input box is the output range widened by the
 * filter window ("halo", Sec. 4.2); for the data gradient it is the range of
 * dy positions whose windows reach the shard's dx rows / columns, and pad_lo/hi
 * count the window positions of that range that lie outside dy.
 * Any of the out pointers may be NULL. */
int tofu_op_regions(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                    tofu_region_t* out_box, tofu_region_t* in_boxes,
                    int64_t* pad_lo, int64_t* pad_hi, int32_t* is_partial);

/* Bytes of device workspace the shard call for (op, splits) may use; the
 * caller passes a 16-byte aligned DEVICE buffer at least this large (0 means
 * none is needed; a smaller buffer -> WORKSPACE_TOO_SMALL).  The kernels cut
 * their own reductions to fill the GPU -- K slices of a tall-skinny matmul,
 * (tile, channel step) or (tile, image) segments of the convolutions -- and the
 * workspace holds those partial tiles until a second kernel sums them in a
 * fixed order; the data gradient also keeps its reversed filters there and the
 * conv1d its re-ordered filters.  The
 * content is scratch: nothing is carried from one call to the next, and calls
 * that run concurrently need separate workspaces.  An invalid operator or plan
 * also returns 0; that case is told apart by tofu_last_error(), which is set
 * then and only then (a valid call that needs no workspace leaves the text of
 * this thread empty). */
size_t tofu_workspace_bytes(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits);

/* Thread-local text for the last non-zero status returned on this thread. */
const char* tofu_last_error(void);

/* ---- device entry points ------------------------------------------------ */

/* Fused region fetch (Sec. 6, MultiFetch): assemble dst->extent from `nsrc`
 * source blocks in ONE launch.  `srcs` is a HOST array of descriptors whose
 * data pointers are device pointers; each source contributes the
 * intersection of its extent with dst->extent.  The sources must tile
 * dst->extent exactly: a hole -> UNCOVERED, a doubly-claimed coordinate ->
 * OVERLAP (both detected on the host from the boxes alone).  All tensors
 * must have the same ndim (1..TOFU_MAX_DIMS).  An empty dst->extent is a
 * no-op.  nsrc is limited to 16.  dst must not alias any source. */
int tofu_region_fetch(const tofu_tensor_t* dst, const tofu_tensor_t* srcs, int32_t nsrc,
                      void* hip_stream);

/* Shard of a matrix multiplication (Sec. 3.1: the same operator on smaller
 * inputs).  A, B, C are addressed by GLOBAL coordinate through their extents,
 * so the caller may pass the full tensors, owned blocks or freshly fetched
 * regions; each extent must contain the box tofu_op_regions derives, else
 * REGION_MISMATCH.  Writes C over the shard's output box only.  When K was
 * split the values written are the partial sums over the shard's K range. */
int tofu_shard_matmul(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                      const tofu_tensor_t* A, const tofu_tensor_t* B, const tofu_tensor_t* C,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* Shard of a 2-D convolution forward pass (Fig. 1 generalised to two spatial
 * dimensions; Sec. 4.2 Case-1 for N/CO/H/W splits incl. halo, Case-2 for CI).
 * Implemented for KH = KW = 3, stride 1, pad 0 or 1 -> otherwise UNSUPPORTED.
 * Input rows/columns outside the GLOBAL tensor are zeros; rows inside the
 * global tensor but outside x->extent are REGION_MISMATCH, never zeros. */
int tofu_shard_conv2d(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                      const tofu_tensor_t* x, const tofu_tensor_t* w, const tofu_tensor_t* y,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* The same convolution shard with the fetch fused into it (Sec. 6: the
 * consumer reads its input region straight from the blocks that hold it, so
 * no assembled copy of the region exists).  `x_srcs` is a HOST array of
 * 1 <= nsrc <= 16 descriptors of DEVICE blocks of the global input tensor.
 * Clipped to the input box tofu_op_regions derives, the blocks must tile that
 * box exactly (a hole -> UNCOVERED, a coordinate held twice -> OVERLAP), and
 * every block that holds part of the box must span all of the box's channels
 * (blocks cut along N, H or W -- the halo case); otherwise UNSUPPORTED and the
 * caller assembles the region with tofu_region_fetch.  Results are bit-identical
 * to tofu_shard_conv2d on the assembled region.  Other rules as above. */
int tofu_shard_conv2d_fused(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                            const tofu_tensor_t* x_srcs, int32_t nsrc, const tofu_tensor_t* w,
                            const tofu_tensor_t* y, void* workspace, size_t workspace_bytes,
                            void* hip_stream);

/* Shard of the convolution's weight gradient.  The batch index is a
 * reduction index of this operator, so a batch split is Case-2 (Sec. 4.2)
 * and dw receives a full-size partial.  Same parameter limits as above. */
int tofu_shard_conv2d_wgrad(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                            const tofu_tensor_t* x, const tofu_tensor_t* dy, const tofu_tensor_t* dw,
                            void* workspace, size_t workspace_bytes, void* hip_stream);

/* Shard of the convolution's data gradient (the backward operator that shares
 * the forward operator's partition group, Sec. 5.1).  The output channel is a
 * reduction index of this operator, so a CO split is Case-2 (Sec. 4.2) and dx
 * receives a full-size partial; N / CI / H / W splits are Case-1, H and W
 * splits reading a halo-widened box of dy.  Implemented for KH = KW = 3,
 * stride 1, pad 1 -> otherwise UNSUPPORTED.  The workspace (see
 * tofu_workspace_bytes; 16-byte aligned) receives the shard's filters with
 * taps reversed and channels exchanged.  dy rows inside the global tensor but
 * outside dy->extent are REGION_MISMATCH, never zeros. */
int tofu_shard_conv2d_dgrad(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                            const tofu_tensor_t* dy, const tofu_tensor_t* w, const tofu_tensor_t* dx,
                            void* workspace, size_t workspace_bytes, void* hip_stream);

/* Shard of the paper's running example, the 1-D convolution of Fig. 1 / Fig. 3:
 *   out[b,co,x] = sum_{ci,dx} data[b,ci,x+dx] * filters[ci,co,dx]
 * op->kind = TOFU_OP_CONV1D with batch, c_in, c_out, W (length of data) and KW (window); splits
 * name TOFU_CONV1D_DIM_B / _CO / _X (Case-1; an X split reads its output range widened by the
 * window, Sec. 4.2) or _CI (Case-2: out receives a full-size partial).
 *   data    [batch, c_in, W]        filters [c_in, c_out, KW]  (the index order of Fig. 1)
 *   out     [batch, c_out, W-KW+1]
 * all addressed by global coordinate through their extents and strides.  Implemented for
 * KW = 3 -> otherwise UNSUPPORTED.  Filters whose memory order is [c_out][c_in][KW] (strides
 * (3, 3*n, 1) with n a multiple of 4, 16-byte aligned) are read in place; any other layout is
 * first re-ordered into the workspace.  The shard's X range is cut into equal chunks of at most
 * 272 columns; a range whose length has no suitable divisor (say a large prime) is UNSUPPORTED.
 * tofu_workspace_bytes covers the re-ordered filters and the kernel's segment slots.  The
 * _accumulate form adds to what the output box holds, like the other accumulate calls. */
int tofu_shard_conv1d(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                      const tofu_tensor_t* data, const tofu_tensor_t* filters, const tofu_tensor_t* out,
                      void* workspace, size_t workspace_bytes, void* hip_stream);
int tofu_shard_conv1d_accumulate(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                                 const tofu_tensor_t* data, const tofu_tensor_t* filters, const tofu_tensor_t* out,
                                 void* workspace, size_t workspace_bytes, void* hip_stream);

/* LSTM cell update that consumes the gate GEMM's output (the element-wise
 * stage of the layer; Sec. 5.1: consecutive element-wise operators are merged
 * and share their producer's partition).  op->kind = TOFU_OP_LSTM_CELL with
 * op->M = batch and op->N = hidden units; splits name TOFU_LSTM_DIM_B / _H.
 *   gates   [batch, hidden, 4]  pre-activations of the input, forget, cell and
 *           output gate of each hidden unit (the gate GEMM's N index is
 *           4 * h + gate, so an N shard that is a multiple of 4 holds whole units),
 *   c_prev  [batch, hidden]     cell state before the step,
 *   c_new, h_new [batch, hidden] written over the shard's box only;
 *           c_new may be c_prev itself (the same address and strides: each element
 *           is read before the same thread writes it); any other overlap in memory
 *           between an output box and an input or the other output -> INVALID_ARG.
 * All four are addressed by global coordinate through their extents, like the
 * other shard calls; the innermost stride of gates must be 1.  No workspace. */
int tofu_shard_lstm_cell(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                         const tofu_tensor_t* gates, const tofu_tensor_t* c_prev,
                         const tofu_tensor_t* c_new, const tofu_tensor_t* h_new, void* hip_stream);

/* Partition-n-reduce output step (Sec. 3.1 way 2; Sec. 6): dst[i] =
 * partials[0][i] + partials[1][i] + ... + partials[k-1][i], summed in that
 * order in fp32, for i in [0,count).  `partials` is a HOST array of k DEVICE
 * pointers (1 <= k <= 16), each to `count` dense fp32 values.  dst may be
 * partials[0] (in-place aggregation, Sec. 7.2); no other aliasing.  count = 0
 * is a no-op. */
int tofu_partition_reduce(void* dst, const void* const* partials, int32_t k, int64_t count,
                          void* hip_stream);

/* Reducers of the operator description language (Sec. 4.1) and the two orders
 * in which k partials can be combined.  TOFU_ORDER_LINEAR folds j = 0..k-1 left
 * to right; TOFU_ORDER_TREE folds pairwise, fold(l,r) = fold(l,m) (+) fold(m,r)
 * with m = l + ceil((r-l)/2), the shape of the recursion's binary tree of
 * workers (Sec. 5.2).  Max and Min are exact in any order; a NaN input is
 * ignored while another input holds a number (fmax / fmin convention). */
typedef enum { TOFU_REDUCE_SUM = 0, TOFU_REDUCE_MAX = 1, TOFU_REDUCE_MIN = 2, TOFU_REDUCE_PROD = 3 } tofu_reducer_t;
typedef enum { TOFU_ORDER_LINEAR = 0, TOFU_ORDER_TREE = 1 } tofu_reduce_order_t;

/* tofu_partition_reduce with a chosen reducer and order; (SUM, LINEAR) is
 * bit-identical to tofu_partition_reduce.  Same argument rules and errors; an
 * unknown reducer or order -> INVALID_ARG. */
int tofu_partition_reduce_ex(void* dst, const void* const* partials, int32_t k, int64_t count,
                             int32_t reducer, int32_t order, void* hip_stream);

/* One worker's share of the spread-out reduction (Sec. 6: the reduction work is
 * divided over all workers instead of one aggregating everything): combine only
 * the elements [lo, hi) = [floor(share*count/shares), floor((share+1)*count/shares))
 * of the k partials and write dst[lo..hi); everything outside that range is left
 * untouched.  dst and every partial point at element 0 of the full-length
 * arrays.  The values written are bit-identical to those tofu_partition_reduce_ex
 * writes at the same indices, so running all `shares` shares reproduces it.
 * 1 <= shares, 0 <= share < shares, else INVALID_ARG; an empty share is a no-op.
 * Other rules as for tofu_partition_reduce_ex. */
int tofu_partition_reduce_scatter(void* dst, const void* const* partials, int32_t k, int64_t count,
                                  int32_t shares, int32_t share, int32_t reducer, int32_t order,
                                  void* hip_stream);

/* Reduction fused into the producer (Sec. 7.2: gradients of a large model are
 * aggregated in place rather than kept as separate partials): the same shard
 * calls, but the shard's result is ADDED to what the output box already holds,
 * out = out + result, one fp32 addition per element after the shard's own sum is
 * complete.  Running the k shards of a Case-2 split one after another on one
 * stream, the first through the plain call and the others through these, leaves
 * exactly what k separate partials followed by tofu_partition_reduce (left to
 * right) would: ((P0 + P1) + P2) + ..., bit for bit, without the k partial
 * buffers or the reduce pass.  Arguments, workspace, limits and errors are those
 * of the plain calls; calls that add to one output box must be ordered (same
 * stream), concurrent ones race. */
int tofu_shard_matmul_accumulate(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                                 const tofu_tensor_t* A, const tofu_tensor_t* B, const tofu_tensor_t* C,
                                 void* workspace, size_t workspace_bytes, void* hip_stream);
int tofu_shard_conv2d_accumulate(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                                 const tofu_tensor_t* x, const tofu_tensor_t* w, const tofu_tensor_t* y,
                                 void* workspace, size_t workspace_bytes, void* hip_stream);
int tofu_shard_conv2d_wgrad_accumulate(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                                       const tofu_tensor_t* x, const tofu_tensor_t* dy, const tofu_tensor_t* dw,
                                       void* workspace, size_t workspace_bytes, void* hip_stream);
int tofu_shard_conv2d_dgrad_accumulate(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                                       const tofu_tensor_t* dy, const tofu_tensor_t* w, const tofu_tensor_t* dx,
                                       void* workspace, size_t workspace_bytes, void* hip_stream);

/* tofu_shard_matmul for callers that cannot allocate device memory or bring a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * checks, kernels and results (bit for bit) as tofu_shard_matmul, but the K slices of a
 * tall-skinny shard go to an array of TOFU_STATIC_SCRATCH_BYTES bytes that is part of the
 * library's device image; each GPU the library runs on holds its copy until the process ends.
 * The call allocates and frees nothing and synchronises nothing.  A shard whose K slices need
 * more (tofu_workspace_bytes tells) -> WORKSPACE_TOO_SMALL, nothing launched.  The array's device
 * address is looked up on the first call on each device (make that call outside stream capture);
 * `hip_stream` must belong to the current device.  Every call on a GPU shares that GPU's array:
 * nothing in it has to be cleared (every slice element read was written by the same call), but
 * calls that overlap in time on one GPU race -- order them on one stream. */
#define TOFU_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
int tofu_shard_matmul_noalloc(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                              const tofu_tensor_t* A, const tofu_tensor_t* B, const tofu_tensor_t* C,
                              void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* TOFU_H_ */
