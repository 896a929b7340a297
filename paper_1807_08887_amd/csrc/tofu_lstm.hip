// LSTM cell update that follows the gate GEMM (arXiv 1807.08887 Sec. 5.1: element-wise operators
// are merged with their neighbours and share their producer's partition, so a worker applies it
// to exactly the hidden units whose gate columns its GEMM shard produced).
//   (i, f, g, o) = gates[b, h, 0..3];  c' = sigmoid(f) c + sigmoid(i) tanh(g);  h' = sigmoid(o) tanh(c')
// Pure streaming: 28 bytes per (b, h) element (16 read for the gates, 4 for c, 4 + 4 written), no
// reuse, so the kernel is bound by HBM bandwidth.  One lane per hidden unit: its four gates are
// one 16-byte load, and neighbouring lanes read and write neighbouring words of c, c' and h'.
#include <hip/hip_runtime.h>

#include "tofu_internal.h"
#include "tofu_mfma.h"

namespace tofu {

struct LstmArgs {
  const float* gates;   // element (b_lo, h_lo, 0)
  const float* c_prev;  // element (b_lo, h_lo)
  float* c_new;
  float* h_new;
  int64_t g_rs, g_hs;   // gates: batch stride, hidden-unit stride (gate stride is 1)
  int64_t cp_rs, cp_hs, cn_rs, cn_hs, hn_rs, hn_hs;
  int rows, cols;       // shard box: batch rows x hidden units
  int vec;              // 1: every hidden unit's four gates are one aligned 16-byte vector
};

__device__ __forceinline__ float sigmoidf(float x) { return 1.0f / (1.0f + expf(-x)); }

__global__ void __launch_bounds__(256) lstm_cell_kernel(const LstmArgs p) {
  const int64_t total = (int64_t)p.rows * p.cols;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
    const int b = (int)(e / p.cols), h = (int)(e - (int64_t)b * p.cols);
    const float* g = p.gates + b * p.g_rs + h * p.g_hs;
    v4f32 q;
    if (p.vec) {
      q = __builtin_nontemporal_load(reinterpret_cast<const v4f32*>(g));
    } else {
      q[0] = g[0]; q[1] = g[1]; q[2] = g[2]; q[3] = g[3];
    }
    const float c = p.c_prev[b * p.cp_rs + h * p.cp_hs];
    const float cn = sigmoidf(q[1]) * c + sigmoidf(q[0]) * tanhf(q[2]);
    p.c_new[b * p.cn_rs + h * p.cn_hs] = cn;
    p.h_new[b * p.hn_rs + h * p.hn_hs] = sigmoidf(q[3]) * tanhf(cn);
  }
}

}  // namespace tofu

extern "C" int tofu_shard_lstm_cell(const tofu_op_desc_t* op, const tofu_split_t* splits, int32_t nsplits,
                                    const tofu_tensor_t* gates, const tofu_tensor_t* c_prev, const tofu_tensor_t* c_new,
                                    const tofu_tensor_t* h_new, void* hip_stream) {
  using namespace tofu;
  if (!op || op->kind != TOFU_OP_LSTM_CELL) return fail(TOFU_ERR_INVALID_ARG, "operator description is not an lstm cell");
  tofu_region_t out_box, in_boxes[2];
  int32_t partial = 0;
  int rc = tofu_op_regions(op, splits, nsplits, &out_box, in_boxes, nullptr, nullptr, &partial);
  if (rc) return rc;
  if ((rc = check_tensor("gates", gates, 3, &in_boxes[0]))) return rc;
  if ((rc = check_tensor("c_prev", c_prev, 2, &in_boxes[1]))) return rc;
  if ((rc = check_tensor("c_new", c_new, 2, &out_box))) return rc;
  if ((rc = check_tensor("h_new", h_new, 2, &out_box))) return rc;
  const int64_t rows = out_box.hi[0] - out_box.lo[0], cols = out_box.hi[1] - out_box.lo[1];
  if (rows == 0 || cols == 0) return TOFU_OK;
  if (rows >= (1 << 30) || cols >= (1 << 30)) return fail(TOFU_ERR_UNSUPPORTED, "lstm cell shard extent exceeds 2^30");
  int64_t gs[3], ps[2], ns[2], hs[2];
  effective_strides(gates, gs);
  effective_strides(c_prev, ps);
  effective_strides(c_new, ns);
  effective_strides(h_new, hs);
  if (gs[2] != 1) return fail(TOFU_ERR_UNSUPPORTED, "lstm cell: the four gates of a hidden unit must be adjacent (innermost stride 1)");
  LstmArgs p;
  p.gates = element_ptr(gates, gs, in_boxes[0].lo);
  p.c_prev = element_ptr(c_prev, ps, in_boxes[1].lo);
  p.c_new = const_cast<float*>(element_ptr(c_new, ns, out_box.lo));
  p.h_new = const_cast<float*>(element_ptr(h_new, hs, out_box.lo));
  // Aliasing, by the bytes the shard's boxes span: the outputs overlap no input and not each other, except that
  // c_new may be c_prev itself (same address and strides: every element is read before the same lane writes it).
  {
    const char *g0, *g1, *p0, *p1, *n0, *n1, *h0, *h1;
    box_byte_span(gates, gs, &in_boxes[0], &g0, &g1);
    box_byte_span(c_prev, ps, &in_boxes[1], &p0, &p1);
    box_byte_span(c_new, ns, &out_box, &n0, &n1);
    box_byte_span(h_new, hs, &out_box, &h0, &h1);
    auto overlap = [](const char* a0, const char* a1, const char* b0, const char* b1) { return a0 < b1 && b0 < a1; };
    if (overlap(h0, h1, n0, n1) || overlap(h0, h1, p0, p1) || overlap(h0, h1, g0, g1))
      return fail(TOFU_ERR_INVALID_ARG, "h_new must not overlap c_new, c_prev or gates in memory");
    if (overlap(n0, n1, g0, g1)) return fail(TOFU_ERR_INVALID_ARG, "c_new must not overlap gates in memory");
    const bool in_place = static_cast<const void*>(p.c_new) == static_cast<const void*>(p.c_prev) && ns[0] == ps[0] && ns[1] == ps[1];
    if (overlap(n0, n1, p0, p1) && !in_place)
      return fail(TOFU_ERR_INVALID_ARG, "c_new overlaps c_prev without being the same view (same address and strides)");
  }
  p.g_rs = gs[0]; p.g_hs = gs[1];
  p.cp_rs = ps[0]; p.cp_hs = ps[1]; p.cn_rs = ns[0]; p.cn_hs = ns[1]; p.hn_rs = hs[0]; p.hn_hs = hs[1];
  p.rows = (int)rows; p.cols = (int)cols;
  p.vec = gs[1] % 4 == 0 && gs[0] % 4 == 0 && (reinterpret_cast<uintptr_t>(p.gates) & 15) == 0;
  const int64_t total = rows * cols;
  const int blocks = (int)((total + 255) / 256 < 16384 ? (total + 255) / 256 : 16384);
  hipLaunchKernelGGL(lstm_cell_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream), p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(TOFU_ERR_HIP, "lstm cell launch failed: %s", hipGetErrorString(e));
  return TOFU_OK;
}
