// fp32 check mode: every operation of the training step on fp32 tensors, written as plain one-thread-per-output
// kernels with fp32 (reductions: fp64) accumulation.  This path exists to compare the graph, the automatic
// differentiation, the memory plan and the swapping of the library with the fp64 oracle at 1e-4, without the
// rounding of bf16 storage in between; it is not tuned.  Layouts are those of the bf16 path: activations
// channels-last, filters [taps][C][K], weight gradients fp32 in the filter layout.
#include <hip/hip_runtime.h>

#include <cmath>

#include "kernels.hpp"

namespace lms {

namespace {

constexpr int CT = 256;
inline unsigned cgrid(long long n) { return (unsigned)((n + CT - 1) / CT); }

struct CkGeom {
  long long rows_out;            // output rows of this launch
  int nout, red;                 // output channels, reduction channels
  int asp[3], osp[3];            // spatial extents of the gathered operand / of the output
  int filt[3], stride[3], pad[3];
  int transposed;                // 0: src = o*stride + tap - pad; 1: src = (o + pad - tap) / stride if divisible
  int w_rows_are_out;            // 0: w[tap][r][n] (forward); 1: w[tap][n][r] (data gradient)
};

__device__ __forceinline__ int ck_src(int o, int t, int stride, int pad, int extent, int transposed) {
  if (!transposed) {
    const int i = o * stride + t - pad;
    return (i >= 0 && i < extent) ? i : -1;
  }
  const int i = o + pad - t;
  if (i < 0) return -1;
  const int q = i / stride;
  return (q * stride == i && q < extent) ? q : -1;
}

// out[m][n] = epi(sum_{tap, r} a[src(m, tap)][r] * w(tap, r, n) * rscale[r])
__global__ __launch_bounds__(CT) void ck_conv_kernel(CkGeom g, const float* a, const float* w, const float* rscale, const float* scale,
                                                     const float* shift, const float* add, const float* mask, int relu, float* out) {
  const long long idx = (long long)blockIdx.x * CT + threadIdx.x;
  if (idx >= g.rows_out * g.nout) return;
  const int n = (int)(idx % g.nout);
  long long t = idx / g.nout;
  const int ow = (int)(t % g.osp[2]); t /= g.osp[2];
  const int oh = (int)(t % g.osp[1]); t /= g.osp[1];
  const int od = (int)(t % g.osp[0]); t /= g.osp[0];
  float acc = 0.f;
  int tap = 0;
  for (int kd = 0; kd < g.filt[0]; ++kd)
    for (int kh = 0; kh < g.filt[1]; ++kh)
      for (int kw = 0; kw < g.filt[2]; ++kw, ++tap) {
        const int id = ck_src(od, kd, g.stride[0], g.pad[0], g.asp[0], g.transposed);
        const int ih = ck_src(oh, kh, g.stride[1], g.pad[1], g.asp[1], g.transposed);
        const int iw = ck_src(ow, kw, g.stride[2], g.pad[2], g.asp[2], g.transposed);
        if (id < 0 || ih < 0 || iw < 0) continue;
        const float* ar = a + (((t * g.asp[0] + id) * g.asp[1] + ih) * g.asp[2] + iw) * g.red;
        for (int r = 0; r < g.red; ++r) {
          const float wv = g.w_rows_are_out ? w[((long long)tap * g.nout + n) * g.red + r] : w[((long long)tap * g.red + r) * g.nout + n];
          acc = fmaf(ar[r], rscale ? wv * rscale[r] : wv, acc);
        }
      }
  float v = acc;
  if (scale) v = fmaf(v, scale[n], shift ? shift[n] : 0.f);
  else if (shift) v += shift[n];
  if (add) v += add[idx];
  if (relu) v = fmaxf(v, 0.f);
  if (mask && !(mask[idx] > 0.f)) v = 0.f;
  out[idx] = v;
}

// dw[tap][c][k] = sum over rows m of the strided side: x[src(m, tap)][c] * dy[m][k]          (convolution)
// dw[tap][c][k] = sum over rows p of the small grid:   x[p][c] * dy[2p + tap][k]             (transposed convolution)
struct CkWgrad {
  long long rows;                // rows that are summed over
  int c, k;
  int xsp[3], ysp[3];            // spatial extents of x and of dy
  int filt[3], stride[3], pad[3];
  int tconv;
};
__global__ __launch_bounds__(CT) void ck_wgrad_kernel(CkWgrad g, const float* x, const float* dy, float* dw) {
  const long long idx = (long long)blockIdx.x * CT + threadIdx.x;
  const int taps = g.filt[0] * g.filt[1] * g.filt[2];
  if (idx >= (long long)taps * g.c * g.k) return;
  const int k = (int)(idx % g.k);
  const int c = (int)((idx / g.k) % g.c);
  int tap = (int)(idx / g.k / g.c);
  const int kw = tap % g.filt[2]; tap /= g.filt[2];
  const int kh = tap % g.filt[1]; tap /= g.filt[1];
  const int kd = tap;
  const int* lsp = g.tconv ? g.xsp : g.ysp;          // the grid the loop runs over
  double s = 0.0;
  for (long long m = 0; m < g.rows; ++m) {
    long long t = m;
    const int pw = (int)(t % lsp[2]); t /= lsp[2];
    const int ph = (int)(t % lsp[1]); t /= lsp[1];
    const int pd = (int)(t % lsp[0]); t /= lsp[0];
    if (g.tconv) {
      const long long yrow = ((t * g.ysp[0] + 2 * pd + kd) * g.ysp[1] + 2 * ph + kh) * g.ysp[2] + 2 * pw + kw;
      s += (double)x[m * g.c + c] * (double)dy[yrow * g.k + k];
    } else {
      const int id = pd * g.stride[0] + kd - g.pad[0], ih = ph * g.stride[1] + kh - g.pad[1], iw = pw * g.stride[2] + kw - g.pad[2];
      if (id < 0 || id >= g.xsp[0] || ih < 0 || ih >= g.xsp[1] || iw < 0 || iw >= g.xsp[2]) continue;
      const long long xrow = ((t * g.xsp[0] + id) * g.xsp[1] + ih) * g.xsp[2] + iw;
      s += (double)x[xrow * g.c + c] * (double)dy[m * g.k + k];
    }
  }
  dw[idx] = (float)s;
}

struct CkPool { int isp[3], osp[3], win[3], stride[3], pad[3], c; };
__global__ __launch_bounds__(CT) void ck_maxpool_fwd_kernel(CkPool p, const float* x, float* y, long long total) {
  const long long idx = (long long)blockIdx.x * CT + threadIdx.x;
  if (idx >= total) return;
  const int ch = (int)(idx % p.c);
  long long t = idx / p.c;
  const int ow = (int)(t % p.osp[2]); t /= p.osp[2];
  const int oh = (int)(t % p.osp[1]); t /= p.osp[1];
  const int od = (int)(t % p.osp[0]); t /= p.osp[0];
  float best = -INFINITY;
  for (int kd = 0; kd < p.win[0]; ++kd)
    for (int kh = 0; kh < p.win[1]; ++kh)
      for (int kw = 0; kw < p.win[2]; ++kw) {
        const int id = od * p.stride[0] + kd - p.pad[0], ih = oh * p.stride[1] + kh - p.pad[1], iw = ow * p.stride[2] + kw - p.pad[2];
        if (id < 0 || id >= p.isp[0] || ih < 0 || ih >= p.isp[1] || iw < 0 || iw >= p.isp[2]) continue;
        const float v = x[(((t * p.isp[0] + id) * p.isp[1] + ih) * p.isp[2] + iw) * p.c + ch];
        if (v > best) best = v;
      }
  y[idx] = best;
}
// scatter-free form: one thread per window finds its first maximum (row-major window order); windows may overlap, so
// the gradient of an input element is gathered by one thread per input element over the windows that contain it
__global__ __launch_bounds__(CT) void ck_maxpool_bwd_kernel(CkPool p, const float* dy, const float* x, int mask_relu, float* dx, long long total) {
  const long long idx = (long long)blockIdx.x * CT + threadIdx.x;
  if (idx >= total) return;
  const int ch = (int)(idx % p.c);
  long long t = idx / p.c;
  int i3[3];
  i3[2] = (int)(t % p.isp[2]); t /= p.isp[2];
  i3[1] = (int)(t % p.isp[1]); t /= p.isp[1];
  i3[0] = (int)(t % p.isp[0]); t /= p.isp[0];
  const float mine = x[idx];
  float g = 0.f;
  for (int od = 0; od < p.osp[0]; ++od) {
    if (i3[0] < od * p.stride[0] - p.pad[0] || i3[0] >= od * p.stride[0] - p.pad[0] + p.win[0]) continue;
    for (int oh = 0; oh < p.osp[1]; ++oh) {
      if (i3[1] < oh * p.stride[1] - p.pad[1] || i3[1] >= oh * p.stride[1] - p.pad[1] + p.win[1]) continue;
      for (int ow = 0; ow < p.osp[2]; ++ow) {
        if (i3[2] < ow * p.stride[2] - p.pad[2] || i3[2] >= ow * p.stride[2] - p.pad[2] + p.win[2]) continue;
        // first maximum of this window in row-major order
        float best = -INFINITY;
        int bd = -1, bh = -1, bw = -1;
        for (int kd = 0; kd < p.win[0]; ++kd)
          for (int kh = 0; kh < p.win[1]; ++kh)
            for (int kw = 0; kw < p.win[2]; ++kw) {
              const int id = od * p.stride[0] + kd - p.pad[0], ih = oh * p.stride[1] + kh - p.pad[1], iw = ow * p.stride[2] + kw - p.pad[2];
              if (id < 0 || id >= p.isp[0] || ih < 0 || ih >= p.isp[1] || iw < 0 || iw >= p.isp[2]) continue;
              const float v = x[(((t * p.isp[0] + id) * p.isp[1] + ih) * p.isp[2] + iw) * p.c + ch];
              if (v > best) { best = v; bd = id; bh = ih; bw = iw; }
            }
        if (bd == i3[0] && bh == i3[1] && bw == i3[2]) g += dy[(((t * p.osp[0] + od) * p.osp[1] + oh) * p.osp[2] + ow) * p.c + ch];
      }
    }
  }
  if (mask_relu && !(mine > 0.f)) g = 0.f;
  dx[idx] = g;
}

__global__ __launch_bounds__(CT) void ck_gap_fwd_kernel(const float* x, float* y, long long n, long long positions, int c) {
  const long long idx = (long long)blockIdx.x * CT + threadIdx.x;
  if (idx >= n * c) return;
  const int ch = (int)(idx % c);
  const long long b = idx / c;
  double s = 0.0;
  for (long long q = 0; q < positions; ++q) s += x[(b * positions + q) * c + ch];
  y[idx] = (float)(s / (double)positions);
}
__global__ __launch_bounds__(CT) void ck_gap_bwd_kernel(const float* dy, const float* mask, float* dx, long long total, long long positions, int c) {
  const long long idx = (long long)blockIdx.x * CT + threadIdx.x;
  if (idx >= total) return;
  const int ch = (int)(idx % c);
  const long long b = idx / c / positions;
  float g = dy[b * c + ch] / (float)positions;
  if (mask && !(mask[idx] > 0.f)) g = 0.f;
  dx[idx] = g;
}
__global__ __launch_bounds__(CT) void ck_copy_channels_kernel(const float* src, int src_c, int src_begin, float* dst, int dst_c, int dst_begin,
                                                              int count, const float* mask, long long total) {
  const long long idx = (long long)blockIdx.x * CT + threadIdx.x;
  if (idx >= total) return;
  const int ch = (int)(idx % count);
  const long long r = idx / count;
  float v = src[r * src_c + src_begin + ch];
  const long long o = r * dst_c + dst_begin + ch;
  if (mask && !(mask[o] > 0.f)) v = 0.f;
  dst[o] = v;
}

// one block, fixed order: block-strided fp64 partial sums, then a tree
__device__ __forceinline__ double ck_block_sum(double v, double* sh) {
  sh[threadIdx.x] = v;
  __syncthreads();
  for (int d = CT / 2; d > 0; d >>= 1) {
    if ((int)threadIdx.x < d) sh[threadIdx.x] += sh[threadIdx.x + d];
    __syncthreads();
  }
  return sh[0];
}
__global__ __launch_bounds__(CT) void ck_mse_kernel(const float* y, const float* t, long long n, float* loss) {
  __shared__ double sh[CT];
  double s = 0.0;
  for (long long i = threadIdx.x; i < n; i += CT) {
    const double d = (double)y[i] - (double)t[i];
    s += d * d;
  }
  const double tot = ck_block_sum(s, sh);
  if (threadIdx.x == 0) loss[0] = (float)(tot / (double)n);
}
__global__ __launch_bounds__(CT) void ck_mse_grad_kernel(const float* y, const float* t, const float* mask, long long n, float* dy) {
  const long long i = (long long)blockIdx.x * CT + threadIdx.x;
  if (i >= n) return;
  float g = 2.0f / (float)n * (y[i] - t[i]);
  if (mask && !(mask[i] > 0.f)) g = 0.f;
  dy[i] = g;
}
__global__ __launch_bounds__(CT) void ck_ce_kernel(const float* z, const int32_t* lab, long long rows, int classes, float* loss) {
  __shared__ double sh[CT];
  double s = 0.0;
  for (long long r = threadIdx.x; r < rows; r += CT) {
    const float* zr = z + r * classes;
    float mx = zr[0];
    for (int c = 1; c < classes; ++c) mx = fmaxf(mx, zr[c]);
    double se = 0.0;
    for (int c = 0; c < classes; ++c) se += exp((double)zr[c] - (double)mx);
    s += (double)mx + log(se) - (double)zr[lab[r]];
  }
  const double tot = ck_block_sum(s, sh);
  if (threadIdx.x == 0) loss[0] = (float)(tot / (double)rows);
}
__global__ __launch_bounds__(CT) void ck_ce_grad_kernel(const float* z, const int32_t* lab, long long rows, int classes, const float* mask, float* dz) {
  const long long r = (long long)blockIdx.x * CT + threadIdx.x;
  if (r >= rows) return;
  const float* zr = z + r * classes;
  float mx = zr[0];
  for (int c = 1; c < classes; ++c) mx = fmaxf(mx, zr[c]);
  double se = 0.0;
  for (int c = 0; c < classes; ++c) se += exp((double)zr[c] - (double)mx);
  for (int c = 0; c < classes; ++c) {
    float g = (float)((exp((double)zr[c] - (double)mx) / se - (c == lab[r] ? 1.0 : 0.0)) / (double)rows);
    if (mask && !(mask[r * classes + c] > 0.f)) g = 0.f;
    dz[r * classes + c] = g;
  }
}
struct CkPtrs { const float* g[4]; };
__global__ __launch_bounds__(CT) void ck_grad_sum_kernel(CkPtrs in, int n_in, const float* mask, long long n, float* out) {
  const long long i = (long long)blockIdx.x * CT + threadIdx.x;
  if (i >= n) return;
  float s = in.g[0][i];
  for (int j = 1; j < n_in; ++j) s += in.g[j][i];
  if (mask && !(mask[i] > 0.f)) s = 0.f;
  out[i] = s;
}
// out[col] = sum_r a[r][col] (w == nullptr) or sum_r a[r][col] * w[r][col]
__global__ __launch_bounds__(CT) void ck_col_reduce_kernel(const float* a, const float* w, long long rows, int cols, float* out) {
  const int col = blockIdx.x * CT + threadIdx.x;
  if (col >= cols) return;
  double s = 0.0;
  for (long long r = 0; r < rows; ++r) s += w ? (double)a[r * cols + col] * (double)w[r * cols + col] : (double)a[r * cols + col];
  out[col] = (float)s;
}

CkGeom conv_geom(const ConvGeom& g, bool data_gradient, bool tconv) {
  CkGeom c{};
  // forward conv: gather from x (in grid) to y (out grid), src = o*stride + tap - pad
  // data gradient of conv: gather from dy (out grid) to dx (in grid), transposed
  // forward tconv: gather from x (small, "in") to y (large, "out"), transposed with stride 2, pad 0
  // data gradient of tconv: gather from dy (large) to dx (small), plain with stride 2, pad 0
  const bool to_in = data_gradient;
  c.rows_out = to_in ? g.in_rows() : g.out_rows();
  c.nout = to_in ? g.c : g.k;
  c.red = to_in ? g.k : g.c;
  for (int i = 0; i < 3; ++i) {
    c.asp[i] = to_in ? g.out_sp[i] : g.in_sp[i];
    c.osp[i] = to_in ? g.in_sp[i] : g.out_sp[i];
    c.filt[i] = g.filt[i]; c.stride[i] = g.stride[i]; c.pad[i] = g.pad[i];
  }
  c.transposed = (data_gradient != tconv) ? 1 : 0;
  c.w_rows_are_out = data_gradient ? 1 : 0;
  return c;
}

}  // namespace

hipError_t check_conv(const ConvGeom& g, int data_gradient, int tconv, const void* a, const void* w, const Epilogue& ep, void* out,
                      hipStream_t s) {
  const CkGeom c = conv_geom(g, data_gradient != 0, tconv != 0);
  // the forward scale multiplies output channels; in the data gradient those are the reduction channels
  const float* rscale = data_gradient ? ep.scale : nullptr;
  const float* scale = data_gradient ? nullptr : ep.scale;
  hipLaunchKernelGGL(ck_conv_kernel, dim3(cgrid(c.rows_out * c.nout)), dim3(CT), 0, s, c, (const float*)a, (const float*)w, rscale, scale,
                     data_gradient ? nullptr : ep.shift, (const float*)ep.add, (const float*)ep.mask, ep.relu, (float*)out);
  return hipGetLastError();
}
hipError_t check_wgrad(const ConvGeom& g, int tconv, const void* x, const void* dy, float* dw, hipStream_t s) {
  CkWgrad w{};
  w.rows = tconv ? g.in_rows() : g.out_rows();
  w.c = g.c; w.k = g.k; w.tconv = tconv;
  for (int i = 0; i < 3; ++i) { w.xsp[i] = g.in_sp[i]; w.ysp[i] = g.out_sp[i]; w.filt[i] = g.filt[i]; w.stride[i] = g.stride[i]; w.pad[i] = g.pad[i]; }
  hipLaunchKernelGGL(ck_wgrad_kernel, dim3(cgrid((long long)g.taps() * g.c * g.k)), dim3(CT), 0, s, w, (const float*)x, (const float*)dy, dw);
  return hipGetLastError();
}
static CkPool ck_pool(const ConvGeom& g) {
  CkPool p{};
  p.c = g.c;
  for (int i = 0; i < 3; ++i) { p.isp[i] = g.in_sp[i]; p.osp[i] = g.out_sp[i]; p.win[i] = g.filt[i]; p.stride[i] = g.stride[i]; p.pad[i] = g.pad[i]; }
  return p;
}
hipError_t check_maxpool_fwd(const ConvGeom& g, const void* x, void* y, hipStream_t s) {
  const long long total = g.out_rows() * g.c;
  hipLaunchKernelGGL(ck_maxpool_fwd_kernel, dim3(cgrid(total)), dim3(CT), 0, s, ck_pool(g), (const float*)x, (float*)y, total);
  return hipGetLastError();
}
hipError_t check_maxpool_bwd(const ConvGeom& g, const void* dy, const void* x, int mask_relu, void* dx, hipStream_t s) {
  const long long total = g.in_rows() * g.c;
  hipLaunchKernelGGL(ck_maxpool_bwd_kernel, dim3(cgrid(total)), dim3(CT), 0, s, ck_pool(g), (const float*)dy, (const float*)x, mask_relu, (float*)dx, total);
  return hipGetLastError();
}
hipError_t check_gap_fwd(int64_t n, int64_t positions, int c, const void* x, void* y, hipStream_t s) {
  hipLaunchKernelGGL(ck_gap_fwd_kernel, dim3(cgrid(n * c)), dim3(CT), 0, s, (const float*)x, (float*)y, (long long)n, (long long)positions, c);
  return hipGetLastError();
}
hipError_t check_gap_bwd(int64_t n, int64_t positions, int c, const void* dy, const void* mask, void* dx, hipStream_t s) {
  const long long total = n * positions * c;
  hipLaunchKernelGGL(ck_gap_bwd_kernel, dim3(cgrid(total)), dim3(CT), 0, s, (const float*)dy, (const float*)mask, (float*)dx, total, (long long)positions, c);
  return hipGetLastError();
}
hipError_t check_copy_channels(int64_t rows, const void* src, int src_c, int src_begin, void* dst, int dst_c, int dst_begin, int count,
                               const void* mask, hipStream_t s) {
  const long long total = rows * count;
  hipLaunchKernelGGL(ck_copy_channels_kernel, dim3(cgrid(total)), dim3(CT), 0, s, (const float*)src, src_c, src_begin, (float*)dst, dst_c, dst_begin,
                     count, (const float*)mask, total);
  return hipGetLastError();
}
hipError_t check_mse_loss(int64_t numel, const void* y, const void* t, float* loss, hipStream_t s) {
  hipLaunchKernelGGL(ck_mse_kernel, dim3(1), dim3(CT), 0, s, (const float*)y, (const float*)t, (long long)numel, loss);
  return hipGetLastError();
}
hipError_t check_mse_grad(int64_t numel, const void* y, const void* t, const void* mask, void* dy, hipStream_t s) {
  hipLaunchKernelGGL(ck_mse_grad_kernel, dim3(cgrid(numel)), dim3(CT), 0, s, (const float*)y, (const float*)t, (const float*)mask, (long long)numel, (float*)dy);
  return hipGetLastError();
}
hipError_t check_ce_loss(int64_t rows, int classes, const void* z, const int32_t* labels, float* loss, hipStream_t s) {
  hipLaunchKernelGGL(ck_ce_kernel, dim3(1), dim3(CT), 0, s, (const float*)z, labels, (long long)rows, classes, loss);
  return hipGetLastError();
}
hipError_t check_ce_grad(int64_t rows, int classes, const void* z, const int32_t* labels, const void* mask, void* dz, hipStream_t s) {
  hipLaunchKernelGGL(ck_ce_grad_kernel, dim3(cgrid(rows)), dim3(CT), 0, s, (const float*)z, labels, (long long)rows, classes, (const float*)mask, (float*)dz);
  return hipGetLastError();
}
hipError_t check_grad_sum(int64_t numel, int n, const void* const* g, const void* mask, void* out, hipStream_t s) {
  if (n < 1 || n > 4) return hipErrorInvalidValue;
  CkPtrs in{};
  for (int i = 0; i < n; ++i) in.g[i] = (const float*)g[i];
  hipLaunchKernelGGL(ck_grad_sum_kernel, dim3(cgrid(numel)), dim3(CT), 0, s, in, n, (const float*)mask, (long long)numel, (float*)out);
  return hipGetLastError();
}
hipError_t check_col_reduce(int64_t rows, int cols, const float* a, const void* w, float* out, hipStream_t s) {
  hipLaunchKernelGGL(ck_col_reduce_kernel, dim3(cgrid(cols)), dim3(CT), 0, s, a, (const float*)w, (long long)rows, cols, out);
  return hipGetLastError();
}

}  // namespace lms
