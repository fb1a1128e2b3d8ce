// Host-side launch interface of the gfx950 kernels.  Every function enqueues work on `stream`
// and returns the HIP status of the launch; none allocates memory.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace lms {

// Geometry of one convolution, normalised to three spatial axes (2-D: depth extent 1).
struct ConvGeom {
  int64_t n = 1;        // batch
  int in_sp[3] = {1, 1, 1};   // input (x / dx) spatial extents D, H, W
  int out_sp[3] = {1, 1, 1};  // output (y / dy) spatial extents
  int filt[3] = {1, 1, 1};
  int stride[3] = {1, 1, 1};
  int pad[3] = {0, 0, 0};
  int c = 1, k = 1;     // input / output channels
  int64_t in_rows() const { return n * in_sp[0] * in_sp[1] * in_sp[2]; }
  int64_t out_rows() const { return n * out_sp[0] * out_sp[1] * out_sp[2]; }
  int taps() const { return filt[0] * filt[1] * filt[2]; }
};

// Epilogue of the implicit-GEMM kernels: v = acc*scale[col] + shift[col] + add[row][col];
// relu: v = max(v, 0); mask: v = mask[row][col] > 0 ? v : 0; stored as bf16.
struct Epilogue {
  const float* scale = nullptr;
  const float* shift = nullptr;
  const void* add = nullptr;
  const void* mask = nullptr;
  int relu = 0;
};

// Workspace needs in bytes (pure functions of the geometry: plans must not depend on addresses).
uint64_t conv_fwd_ws(const ConvGeom& g);                 // packed (transposed) filter
uint64_t conv_dgrad_ws(const ConvGeom& g, bool scaled);  // filter times scale, if scaled
uint64_t conv_wgrad_ws(const ConvGeom& g, bool with_colsum = false);   // split partial sums (and those of the column sums)
uint64_t tconv_fwd_ws(const ConvGeom& g);
uint64_t tconv_wgrad_ws(const ConvGeom& g);
// two-stage deterministic reductions: cols > 0: one result per column; cols == 0: scalar result
// (rows = number of per-row partial values the first stage keeps: 0 for MSE and narrow softmax,
// the row count for softmax over more than 64 classes)
uint64_t reduce_ws(int64_t rows, int cols);

// y[N, out_sp, K] = epilogue(conv(x[N, in_sp, C], w[taps, C, K]))
hipError_t conv_fwd(const ConvGeom& g, const void* x, const void* w, const Epilogue& ep, void* y, void* ws, hipStream_t s);
// dx[N, in_sp, C] = epilogue(conv^T(dy[N, out_sp, K], w * scale_k))   (ep.scale is the forward scale)
hipError_t conv_dgrad(const ConvGeom& g, const void* dy, const void* w, const Epilogue& ep, void* dx, void* ws, hipStream_t s);
// dw[taps, C, K] (fp32) = sum over rows of x (x) dy
// colsum_out (or null): k floats, the sums of dy over all positions per channel, from the same pass over dy where the
// kernel allows (ws: conv_wgrad_ws(g, true) bytes then)
hipError_t conv_wgrad(const ConvGeom& g, const void* x, const void* dy, float* dw, void* ws, hipStream_t s, float* colsum_out = nullptr);
// Transposed convolution, window = stride = 2 (geometry: in_sp = small side, out_sp = 2*in_sp, filt 2).
hipError_t tconv_fwd(const ConvGeom& g, const void* x, const void* w, void* y, void* ws, hipStream_t s);
hipError_t tconv_dgrad(const ConvGeom& g, const void* dy, const void* w, const Epilogue& ep, void* dx, hipStream_t s);
hipError_t tconv_wgrad(const ConvGeom& g, const void* x, const void* dy, float* dw, void* ws, hipStream_t s);

// Pooling.  Geometry as for a convolution with c == k.
hipError_t maxpool_fwd(const ConvGeom& g, const void* x, void* y, hipStream_t s);
hipError_t maxpool_bwd(const ConvGeom& g, const void* dy, const void* x, int mask_relu, void* dx, hipStream_t s);
hipError_t gap_fwd(int64_t n, int64_t positions, int c, const void* x, void* y, hipStream_t s);
hipError_t gap_bwd(int64_t n, int64_t positions, int c, const void* dy, const void* mask, void* dx, hipStream_t s);

// Channel concatenation / slicing on [rows, C] views.
hipError_t copy_channels(int64_t rows, const void* src, int src_c, int src_begin, void* dst, int dst_c, int dst_begin,
                         int count, const void* mask, hipStream_t s);

// Losses.  ws: reduce_ws(., 0) bytes as described there.  loss: device fp32 scalar.
hipError_t mse_loss(int64_t numel, const void* y, const void* t, float* loss, void* ws, hipStream_t s);
hipError_t mse_grad(int64_t numel, const void* y, const void* t, const void* mask, void* dy, hipStream_t s);
hipError_t softmax_ce_loss(int64_t rows, int classes, const void* z, const int32_t* labels, float* loss, void* ws, hipStream_t s);
hipError_t softmax_ce_grad(int64_t rows, int classes, const void* z, const int32_t* labels, const void* mask, void* dz, hipStream_t s);

// out = (g0 + .. + g{n-1}) * [mask > 0]
hipError_t grad_sum(int64_t numel, int n, const void* const* g, const void* mask, void* out, hipStream_t s);
// out[c] (fp32) = sum over rows of dy[row][c]; ws: reduce_ws(rows, c) bytes
hipError_t colsum(int64_t rows, int c, const void* dy, float* out, void* ws, hipStream_t s);
// out[c] = part[0][c] + part[1][c] + ... (fp32, `parts` rows, fixed order)
hipError_t col_reduce(const float* part, int64_t parts, int c, float* out, hipStream_t s);
// dw[j][k] = raw[j][k] * scale[k]
hipError_t scale_cols(int64_t j, int k, const float* raw, const float* scale, float* out, hipStream_t s);
// out[k] = sum_j w[j][k] * raw[j][k]
hipError_t dot_cols(int64_t j, int k, const float* raw, const void* w, float* out, hipStream_t s);
// copies `bytes` between device memory and device-mapped pinned host memory (either direction) with a
// grid of at most `nblocks` work-groups; both pointers 16-byte aligned
hipError_t swap_copy(void* dst, const void* src, uint64_t bytes, int nblocks, hipStream_t s);
// Lossless swap encoding of tensors of 16-bit elements (numel a multiple of 8): slots of 2048 elements, each a count
// of non-zero elements, a bitmap, a mode header and the non-zero elements (raw, or 12-bit codes relative to the
// slot's largest exponent); the host buffer needs swap_encoded_bytes(numel) bytes.
// swap_encoded_moved_bytes reads the trailer of an encoded host buffer (after the copy has finished): the bytes
// the encoder wrote into slots = the bytes a decoder reads.
uint64_t swap_encoded_bytes(uint64_t numel);
// trailer: also write the moved-bytes trailer (a second small kernel that reads the counts back over the link); a
// caller that skips it gets the same number from swap_encoded_counted_bytes once the encode has finished.
hipError_t swap_encode(void* dst_host, const void* src, uint64_t numel, int nblocks, hipStream_t s, bool trailer = true);
uint64_t swap_encoded_counted_bytes(const void* host, uint64_t numel);
hipError_t swap_decode(void* dst, const void* src_host, uint64_t numel, int nblocks, hipStream_t s);
// The same on the slots [slot_begin, slot_end) of the tensor (slot = swap_slot_elements() elements, swap_slot_stride()
// bytes of the host buffer).  stage (device memory, (slot_end - slot_begin) * swap_slot_stride() bytes, or null) / w
// (a multiple of 16): the first w bytes of each slot are written to / read from stage + (slot - slot_begin) * stride
// instead of the host buffer, so that a copy engine can carry them over the link (a pitched copy of w-byte rows); the
// kernels reach the host directly only for what lies beyond w.
hipError_t swap_encode_range(void* dst_host, const void* src, uint64_t numel, int64_t slot_begin, int64_t slot_end, void* stage, int w,
                             int nblocks, hipStream_t s);
hipError_t swap_decode_range(void* dst, const void* src_host, uint64_t numel, int64_t slot_begin, int64_t slot_end, const void* stage, int w,
                             int nblocks, hipStream_t s);
uint64_t swap_staging_bytes();     // arena bytes the executor's staged swaps take (exec.cpp)
uint64_t swap_slot_stride();
uint64_t swap_slot_elements();
// Host side, after the encode has finished: the encoded bytes (as swap_encoded_counted_bytes); link_bytes: what a
// staged transfer of width w_used moved over the link (0: the slots' own bytes); w_next: the smallest multiple of 64
// bytes that holds 95 % of the slots whole.
uint64_t swap_slot_statistics(const void* host, uint64_t numel, int w_used, int* w_next, uint64_t* link_bytes);
uint64_t swap_encoded_moved_bytes(const void* host, uint64_t numel);
// out = p - lr * g (g fp32; p and out bf16 or fp32; out may alias p)
hipError_t sgd_update(int64_t numel, bool f32, const void* p, const float* g, float lr, void* out, hipStream_t s);
// Up to SGD_BATCH updates out = p - lr * g in one launch (the same arithmetic per element as sgd_update): the
// per-parameter updates of a deep network are hundreds of launches of a few microseconds each.
constexpr int SGD_BATCH = 64;
struct SgdBatch {
  const void* p[SGD_BATCH];
  const float* g[SGD_BATCH];
  void* out[SGD_BATCH];
  long long n[SGD_BATCH];
  float lr[SGD_BATCH];
  int first[SGD_BATCH + 1];         // first work-group of each tensor; first[count] = work-groups of the launch
  unsigned long long f32_mask;      // bit t: tensor t is fp32 (else bf16)
  int count;
};
int sgd_batch_blocks(int64_t numel);
hipError_t sgd_update_batch(const SgdBatch& b, hipStream_t s);
// fill `bytes` (multiple of 2) with a 16-bit pattern
hipError_t fill16(void* p, uint64_t bytes, uint16_t pattern, hipStream_t s);

// fp32 check mode (check_f32.hip): the same operations on fp32 tensors, plain kernels.  check_conv covers forward and
// data gradient of convolution and transposed convolution (ep.scale multiplies the forward output channels in both).
hipError_t check_conv(const ConvGeom& g, int data_gradient, int tconv, const void* a, const void* w, const Epilogue& ep, void* out,
                      hipStream_t s);
hipError_t check_wgrad(const ConvGeom& g, int tconv, const void* x, const void* dy, float* dw, hipStream_t s);
hipError_t check_maxpool_fwd(const ConvGeom& g, const void* x, void* y, hipStream_t s);
hipError_t check_maxpool_bwd(const ConvGeom& g, const void* dy, const void* x, int mask_relu, void* dx, hipStream_t s);
hipError_t check_gap_fwd(int64_t n, int64_t positions, int c, const void* x, void* y, hipStream_t s);
hipError_t check_gap_bwd(int64_t n, int64_t positions, int c, const void* dy, const void* mask, void* dx, hipStream_t s);
hipError_t check_copy_channels(int64_t rows, const void* src, int src_c, int src_begin, void* dst, int dst_c, int dst_begin, int count,
                               const void* mask, hipStream_t s);
hipError_t check_mse_loss(int64_t numel, const void* y, const void* t, float* loss, hipStream_t s);
hipError_t check_mse_grad(int64_t numel, const void* y, const void* t, const void* mask, void* dy, hipStream_t s);
hipError_t check_ce_loss(int64_t rows, int classes, const void* z, const int32_t* labels, float* loss, hipStream_t s);
hipError_t check_ce_grad(int64_t rows, int classes, const void* z, const int32_t* labels, const void* mask, void* dz, hipStream_t s);
hipError_t check_grad_sum(int64_t numel, int n, const void* const* g, const void* mask, void* out, hipStream_t s);
hipError_t check_col_reduce(int64_t rows, int cols, const float* a, const void* w, float* out, hipStream_t s);

// Matrix-pipe probe (probe.hip): iters x 16 products and 16-byte LDS reads per wave, 2048 waves; floating-point operations of a launch.
hipError_t launch_mfma_probe(unsigned iters, int random_operands, hipStream_t s);
uint64_t mfma_probe_flops(unsigned iters);

}  // namespace lms
