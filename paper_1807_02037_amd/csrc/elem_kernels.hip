// HBM-bound helper kernels of the training step: losses, pooling, gradient sums, channel copies,
// per-channel reductions.  All reductions are two-stage with fixed partition sizes and fixed
// summation order, so results are bit-identical from run to run.
#include <hip/hip_runtime.h>

#include "kernels.hpp"

namespace lms {

namespace {

__device__ __forceinline__ float bf2f(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ uint16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

inline unsigned cdiv(long long a, long long b) { return (unsigned)((a + b - 1) / b); }
constexpr int TB = 256;
constexpr int MAX_PARTS = 1024;

inline int parts_for(long long n) {
  long long p = (n + TB * 8 - 1) / (TB * 8);
  return (int)(p < 1 ? 1 : (p > MAX_PARTS ? MAX_PARTS : p));
}

// Eight bf16 values of a 16-byte vector as floats.
__device__ __forceinline__ void unpack8(const uint4& q, float (&f)[8]) {
  const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
  for (int e = 0; e < 8; ++e) f[e] = __uint_as_float((e & 1) ? (w[e >> 1] & 0xffff0000u) : (w[e >> 1] << 16));
}

// Sum of v over the block in a fixed tree order; result valid in thread 0.
__device__ __forceinline__ float block_sum(float v, float* sh) {
  sh[threadIdx.x] = v;
  __syncthreads();
  for (int s = TB / 2; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) sh[threadIdx.x] += sh[threadIdx.x + s];
    __syncthreads();
  }
  return sh[0];
}

__global__ __launch_bounds__(TB) void mse_partial_kernel(const uint16_t* y, const uint16_t* t, long long n, float* part) {
  __shared__ float sh[TB];
  const long long per = (n + gridDim.x - 1) / gridDim.x;
  const long long lo = (long long)blockIdx.x * per;
  const long long hi = lo + per < n ? lo + per : n;
  float s = 0.f;
  for (long long i = lo + threadIdx.x; i < hi; i += TB) {
    const float d = bf2f(y[i]) - bf2f(t[i]);
    s += d * d;
  }
  const float tot = block_sum(s, sh);
  if (threadIdx.x == 0) part[blockIdx.x] = tot;
}

__global__ __launch_bounds__(TB) void finish_mean_kernel(const float* part, int nparts, float denom, float* out) {
  __shared__ float sh[TB];
  float s = 0.f;
  for (int i = threadIdx.x; i < nparts; i += TB) s += part[i];
  const float tot = block_sum(s, sh);
  if (threadIdx.x == 0) out[0] = tot / denom;
}

__global__ __launch_bounds__(TB) void mse_grad_kernel(const uint16_t* y, const uint16_t* t, const uint16_t* mask, long long n,
                                                      float coef, uint16_t* dy) {
  const long long i = (long long)blockIdx.x * TB + threadIdx.x;
  if (i >= n) return;
  float g = coef * (bf2f(y[i]) - bf2f(t[i]));
  if (mask && !(bf2f(mask[i]) > 0.f)) g = 0.f;
  dy[i] = f2bf(g);
}

// Softmax cross-entropy, one thread per row (few classes) ...
__global__ __launch_bounds__(TB) void ce_rows_kernel(const uint16_t* z, const int32_t* lab, long long rows, int classes,
                                                     float* part, const uint16_t* mask, uint16_t* dz, float inv_rows) {
  __shared__ float sh[TB];
  const long long per = (rows + gridDim.x - 1) / gridDim.x;
  const long long lo = (long long)blockIdx.x * per;
  const long long hi = lo + per < rows ? lo + per : rows;
  float s = 0.f;
  for (long long r = lo + threadIdx.x; r < hi; r += TB) {
    const uint16_t* zr = z + r * classes;
    float mx = bf2f(zr[0]);
    for (int c = 1; c < classes; ++c) mx = fmaxf(mx, bf2f(zr[c]));
    float se = 0.f;
    for (int c = 0; c < classes; ++c) se += __expf(bf2f(zr[c]) - mx);
    const int l = lab[r];
    if (part) s += mx + __logf(se) - bf2f(zr[l]);
    if (dz) {
      for (int c = 0; c < classes; ++c) {
        float g = (__expf(bf2f(zr[c]) - mx) / se - (c == l ? 1.f : 0.f)) * inv_rows;
        if (mask && !(bf2f(mask[r * classes + c]) > 0.f)) g = 0.f;
        dz[r * classes + c] = f2bf(g);
      }
    }
  }
  if (part) {
    const float tot = block_sum(s, sh);
    if (threadIdx.x == 0) part[blockIdx.x] = tot;
  }
}

// ... and one work-group per row (many classes): part[row] = loss of the row.
__global__ __launch_bounds__(TB) void ce_wide_kernel(const uint16_t* z, const int32_t* lab, int classes, float* part,
                                                     const uint16_t* mask, uint16_t* dz, float inv_rows) {
  __shared__ float sh[TB];
  __shared__ float bc;
  const long long r = blockIdx.x;
  const uint16_t* zr = z + r * classes;
  float mx = -INFINITY;
  for (int c = threadIdx.x; c < classes; c += TB) mx = fmaxf(mx, bf2f(zr[c]));
  sh[threadIdx.x] = mx;
  __syncthreads();
  for (int s = TB / 2; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) sh[threadIdx.x] = fmaxf(sh[threadIdx.x], sh[threadIdx.x + s]);
    __syncthreads();
  }
  if (threadIdx.x == 0) bc = sh[0];
  __syncthreads();
  mx = bc;
  __syncthreads();
  float se = 0.f;
  for (int c = threadIdx.x; c < classes; c += TB) se += __expf(bf2f(zr[c]) - mx);
  const float tot = block_sum(se, sh);
  if (threadIdx.x == 0) bc = tot;
  __syncthreads();
  se = bc;
  const int l = lab[r];
  if (part && threadIdx.x == 0) part[r] = mx + __logf(se) - bf2f(zr[l]);
  if (dz) {
    for (int c = threadIdx.x; c < classes; c += TB) {
      float g = (__expf(bf2f(zr[c]) - mx) / se - (c == l ? 1.f : 0.f)) * inv_rows;
      if (mask && !(bf2f(mask[r * classes + c]) > 0.f)) g = 0.f;
      dz[r * classes + c] = f2bf(g);
    }
  }
}

struct Ptrs4 { const uint16_t* g[4]; };
__global__ __launch_bounds__(TB) void grad_sum_kernel(Ptrs4 in, int n_in, const uint16_t* mask, long long n, uint16_t* out) {
  const long long i = (long long)blockIdx.x * TB + threadIdx.x;
  if (i >= n) return;
  float s = bf2f(in.g[0][i]);
  for (int j = 1; j < n_in; ++j) s += bf2f(in.g[j][i]);
  if (mask && !(bf2f(mask[i]) > 0.f)) s = 0.f;
  out[i] = f2bf(s);
}

// Column sums: stage 1 sums a slice of rows per work-group, stage 2 adds the slices in order.
// Column reductions over a [rows][cols] fp32 matrix with few columns per block and many row lanes:
// a block owns 32 columns, its 32 row lanes stride over the rows, the lanes' sums are added in a fixed order.
//   w == nullptr: out[col] = sum_r a[r][col];  else out[col] = sum_r a[r][col] * bf16 w[r][col].
__global__ __launch_bounds__(1024) void col_reduce_kernel(const float* a, const uint16_t* w, long long rows, int cols, float* out) {
  __shared__ float sh[32][33];
  const int cl = threadIdx.x & 31, rl = threadIdx.x >> 5;
  const int col = blockIdx.x * 32 + cl;
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  if (col < cols) {
    long long r = rl;
    if (w) {
      for (; r + 96 < rows; r += 128) {
        s0 += a[r * cols + col] * bf2f(w[r * cols + col]);
        s1 += a[(r + 32) * cols + col] * bf2f(w[(r + 32) * cols + col]);
        s2 += a[(r + 64) * cols + col] * bf2f(w[(r + 64) * cols + col]);
        s3 += a[(r + 96) * cols + col] * bf2f(w[(r + 96) * cols + col]);
      }
      for (; r < rows; r += 32) s0 += a[r * cols + col] * bf2f(w[r * cols + col]);
    } else {
      for (; r + 96 < rows; r += 128) {
        s0 += a[r * cols + col];
        s1 += a[(r + 32) * cols + col];
        s2 += a[(r + 64) * cols + col];
        s3 += a[(r + 96) * cols + col];
      }
      for (; r < rows; r += 32) s0 += a[r * cols + col];
    }
  }
  sh[rl][cl] = (s0 + s1) + (s2 + s3);
  __syncthreads();
  if (rl == 0 && col < cols) {
    float t = 0.f;
#pragma unroll
    for (int j = 0; j < 32; ++j) t += sh[j][cl];
    out[col] = t;
  }
}

// Partial column sums of a bf16 [rows][c] tensor, 8 channels per load.  Needs c % 8 == 0 and TB % (c / 8) == 0,
// so a thread keeps the same 8 channels for all its rows.  part[block][c].
__global__ __launch_bounds__(TB) void colsum_partial_vec_kernel(const uint4* dy, long long rows, int c, float* part) {
  __shared__ float sh[TB][9];
  const int cv = c >> 3;
  const int nrl = TB / cv, rl = threadIdx.x / cv, v = threadIdx.x % cv;
  const long long per = (rows + gridDim.x - 1) / gridDim.x;
  const long long lo = (long long)blockIdx.x * per;
  const long long hi = lo + per < rows ? lo + per : rows;
  float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (long long r = lo + rl; r < hi; r += nrl) {
    float f[8];
    unpack8(dy[r * cv + v], f);
#pragma unroll
    for (int e = 0; e < 8; ++e) s[e] += f[e];
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) sh[threadIdx.x][e] = s[e];
  __syncthreads();
  if (rl == 0) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float t = 0.f;
      for (int j = 0; j < nrl; ++j) t += sh[j * cv + v][e];
      part[(long long)blockIdx.x * c + v * 8 + e] = t;
    }
  }
}

__global__ __launch_bounds__(TB) void colsum_partial_kernel(const uint16_t* dy, long long rows, int c, float* part) {
  __shared__ float sh[TB];
  const long long per = (rows + gridDim.x - 1) / gridDim.x;
  const long long lo = (long long)blockIdx.x * per;
  const long long hi = lo + per < rows ? lo + per : rows;
  int ct = 1;
  while (ct < c && ct < TB) ct <<= 1;          // channels handled side by side
  const int rl = threadIdx.x / ct, nrl = TB / ct, ch0 = threadIdx.x % ct;
  for (int cb = 0; cb < c; cb += ct) {
    const int ch = cb + ch0;
    float s = 0.f;
    if (ch < c)
      for (long long r = lo + rl; r < hi; r += nrl) s += bf2f(dy[r * c + ch]);
    sh[threadIdx.x] = s;
    __syncthreads();
    if (rl == 0 && ch < c) {
      float tot = 0.f;
      for (int j = 0; j < nrl; ++j) tot += sh[j * ct + ch0];
      part[(long long)blockIdx.x * c + ch] = tot;
    }
    __syncthreads();
  }
}

__global__ void scale_cols_kernel(const float* raw, const float* scale, float* out, long long total, int k) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < total) out[i] = raw[i] * scale[i % k];
}
__global__ void fill16_kernel(uint16_t* p, long long n, uint16_t v) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

struct PoolP {
  long long n;
  int isp[3], osp[3], win[3], stride[3], pad[3], c;
};

__global__ __launch_bounds__(TB) void maxpool_fwd_kernel(PoolP p, const uint16_t* x, uint16_t* y, long long total) {
  const long long idx = (long long)blockIdx.x * TB + threadIdx.x;
  if (idx >= total) return;
  const int ch = (int)(idx % p.c);
  long long t = idx / p.c;
  const int ow = (int)(t % p.osp[2]); t /= p.osp[2];
  const int oh = (int)(t % p.osp[1]); t /= p.osp[1];
  const int od = (int)(t % p.osp[0]); t /= p.osp[0];
  float best = -INFINITY;
  for (int kd = 0; kd < p.win[0]; ++kd) {
    const int id = od * p.stride[0] + kd - p.pad[0];
    if (id < 0 || id >= p.isp[0]) continue;
    for (int kh = 0; kh < p.win[1]; ++kh) {
      const int ih = oh * p.stride[1] + kh - p.pad[1];
      if (ih < 0 || ih >= p.isp[1]) continue;
      for (int kw = 0; kw < p.win[2]; ++kw) {
        const int iw = ow * p.stride[2] + kw - p.pad[2];
        if (iw < 0 || iw >= p.isp[2]) continue;
        const float v = bf2f(x[(((t * p.isp[0] + id) * p.isp[1] + ih) * p.isp[2] + iw) * p.c + ch]);
        if (v > best) best = v;
      }
    }
  }
  y[idx] = f2bf(best);
}

// ---- 2-D max pooling with a 3x3 window, stride 2, padding 1 (the pooling after the first convolution of ResNet),
// channel count a multiple of 8.  Forward: one thread per output position and 8-channel vector.
__global__ __launch_bounds__(TB) void maxpool3s2_fwd_kernel(PoolP p, const uint4* x, uint4* y, long long total) {
  const long long idx = (long long)blockIdx.x * TB + threadIdx.x;     // (output position, channel vector)
  if (idx >= total) return;
  const int c8 = p.c >> 3;
  const int cv = (int)(idx % c8);
  long long t = idx / c8;
  const int ow = (int)(t % p.osp[2]); t /= p.osp[2];
  const int oh = (int)(t % p.osp[1]); t /= p.osp[1];
  float best[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) best[e] = -INFINITY;
#pragma unroll
  for (int kh = 0; kh < 3; ++kh) {
    const int ih = 2 * oh - 1 + kh;
#pragma unroll
    for (int kw = 0; kw < 3; ++kw) {
      const int iw = 2 * ow - 1 + kw;
      if ((unsigned)ih < (unsigned)p.isp[1] && (unsigned)iw < (unsigned)p.isp[2]) {
        float v[8];
        unpack8(x[((t * p.isp[1] + ih) * p.isp[2] + iw) * c8 + cv], v);
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (v[e] > best[e]) best[e] = v[e];
      }
    }
  }
  uint32_t w[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) w[e] = (uint32_t)f2bf(best[2 * e]) | ((uint32_t)f2bf(best[2 * e + 1]) << 16);
  y[idx] = make_uint4(w[0], w[1], w[2], w[3]);
}

// Backward: a work-group owns 16 x 16 input positions and 64 channels.  It first finds, for each of the 9 x 9
// windows that touch them, the first maximum in row-major window order (a 4-bit code per channel, kept in LDS
// together with the window's dy), then every input position collects dy from the windows (at most 4, in row-major
// order of the windows) whose code names it.  The maxima are found once per window instead of once per input
// element and window.
constexpr int P3_IN = 16, P3_WIN = P3_IN / 2 + 1;
__global__ __launch_bounds__(TB) void maxpool3s2_bwd_kernel(PoolP p, const uint4* dy, const uint4* x, int mask_relu, uint4* dx,
                                                            int tiles_h, int tiles_w) {
  __shared__ __attribute__((aligned(16))) uint2 scode[P3_WIN * P3_WIN][8];      // 8 channel vectors x 8 one-byte codes
  __shared__ __attribute__((aligned(16))) uint4 sdy[P3_WIN * P3_WIN][8];
  int b = blockIdx.x;
  const int tb = b % tiles_w; b /= tiles_w;
  const int ta = b % tiles_h; b /= tiles_h;
  const long long n = b;
  const int c8 = p.c >> 3;
  const int cv0 = blockIdx.y * 8;
  const int a = ta * (P3_IN / 2), bb = tb * (P3_IN / 2);                        // first window row / column
  for (int item = threadIdx.x; item < P3_WIN * P3_WIN * 8; item += TB) {
    const int w = item >> 3, cvl = item & 7, cv = cv0 + cvl;
    const int oh = a + w / P3_WIN, ow = bb + w % P3_WIN;
    uint32_t code[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) code[e] = 15u;
    uint4 d = make_uint4(0, 0, 0, 0);
    if (oh < p.osp[1] && ow < p.osp[2] && cv < c8) {
      float best[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) best[e] = -INFINITY;
#pragma unroll
      for (int kh = 0; kh < 3; ++kh) {
        const int ih = 2 * oh - 1 + kh;
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
          const int iw = 2 * ow - 1 + kw;
          if ((unsigned)ih < (unsigned)p.isp[1] && (unsigned)iw < (unsigned)p.isp[2]) {
            float v[8];
            unpack8(x[((n * p.isp[1] + ih) * p.isp[2] + iw) * c8 + cv], v);
#pragma unroll
            for (int e = 0; e < 8; ++e)
              if (v[e] > best[e]) { best[e] = v[e]; code[e] = (uint32_t)(kh * 3 + kw); }
          }
        }
      }
      d = dy[((n * p.osp[1] + oh) * p.osp[2] + ow) * c8 + cv];
    }
    scode[w][cvl] = make_uint2(code[0] | (code[1] << 8) | (code[2] << 16) | (code[3] << 24),
                               code[4] | (code[5] << 8) | (code[6] << 16) | (code[7] << 24));
    sdy[w][cvl] = d;
  }
  __syncthreads();
  for (int item = threadIdx.x; item < P3_IN * P3_IN * 8; item += TB) {
    const int pos = item >> 3, cvl = item & 7, cv = cv0 + cvl;
    const int ih = 2 * a + pos / P3_IN, iw = 2 * bb + pos % P3_IN;
    if (ih >= p.isp[1] || iw >= p.isp[2] || cv >= c8) continue;
    float g[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) g[e] = 0.f;
    const int oh_hi = (ih + 1) >> 1, ow_hi = (iw + 1) >> 1;
    const int oh_lo = oh_hi - (ih & 1), ow_lo = ow_hi - (iw & 1);
    for (int oh = oh_lo; oh <= oh_hi; ++oh)
      for (int ow = ow_lo; ow <= ow_hi; ++ow) {
        if (oh >= p.osp[1] || ow >= p.osp[2]) continue;
        const int w = (oh - a) * P3_WIN + (ow - bb);
        const uint32_t me = (uint32_t)((ih - (2 * oh - 1)) * 3 + (iw - (2 * ow - 1)));
        const uint2 cd = scode[w][cvl];
        float d[8];
        unpack8(sdy[w][cvl], d);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const uint32_t ce = ((e < 4 ? cd.x : cd.y) >> ((e & 3) * 8)) & 255u;
          if (ce == me) g[e] += d[e];
        }
      }
    const long long o = ((n * p.isp[1] + ih) * p.isp[2] + iw) * c8 + cv;
    float mine[8];
    if (mask_relu) unpack8(x[o], mine);
    uint32_t wd[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float v0 = (mask_relu && !(mine[2 * e] > 0.f)) ? 0.f : g[2 * e];
      const float v1 = (mask_relu && !(mine[2 * e + 1] > 0.f)) ? 0.f : g[2 * e + 1];
      wd[e] = (uint32_t)f2bf(v0) | ((uint32_t)f2bf(v1) << 16);
    }
    dx[o] = make_uint4(wd[0], wd[1], wd[2], wd[3]);
  }
}

// Gradient of max pooling, gather form: an input element receives dy of every window whose first
// maximum (row-major window order) it is.  Windows are visited in row-major order of their position.
__global__ __launch_bounds__(TB) void maxpool_bwd_kernel(PoolP p, const uint16_t* dy, const uint16_t* x, int mask_relu,
                                                         uint16_t* dx, long long total) {
  const long long idx = (long long)blockIdx.x * TB + threadIdx.x;
  if (idx >= total) return;
  const int ch = (int)(idx % p.c);
  long long t = idx / p.c;
  int i3[3];
  i3[2] = (int)(t % p.isp[2]); t /= p.isp[2];
  i3[1] = (int)(t % p.isp[1]); t /= p.isp[1];
  i3[0] = (int)(t % p.isp[0]); t /= p.isp[0];
  const float mine = bf2f(x[idx]);
  float g = 0.f;
  if (!(mask_relu && !(mine > 0.f))) {
    int lo[3], hi[3];
    for (int a = 0; a < 3; ++a) {
      const int num = i3[a] + p.pad[a] - p.win[a] + 1;
      lo[a] = num <= 0 ? 0 : (num + p.stride[a] - 1) / p.stride[a];
      hi[a] = (i3[a] + p.pad[a]) / p.stride[a];
      if (hi[a] > p.osp[a] - 1) hi[a] = p.osp[a] - 1;
    }
    for (int od = lo[0]; od <= hi[0]; ++od)
      for (int oh = lo[1]; oh <= hi[1]; ++oh)
        for (int ow = lo[2]; ow <= hi[2]; ++ow) {
          // is this element the first maximum of window (od, oh, ow)?
          bool winner = true;
          for (int kd = 0; kd < p.win[0] && winner; ++kd) {
            const int id = od * p.stride[0] + kd - p.pad[0];
            if (id < 0 || id >= p.isp[0]) continue;
            for (int kh = 0; kh < p.win[1] && winner; ++kh) {
              const int ih = oh * p.stride[1] + kh - p.pad[1];
              if (ih < 0 || ih >= p.isp[1]) continue;
              for (int kw = 0; kw < p.win[2]; ++kw) {
                const int iw = ow * p.stride[2] + kw - p.pad[2];
                if (iw < 0 || iw >= p.isp[2]) continue;
                const float v = bf2f(x[(((t * p.isp[0] + id) * p.isp[1] + ih) * p.isp[2] + iw) * p.c + ch]);
                const bool before = (id < i3[0]) || (id == i3[0] && (ih < i3[1] || (ih == i3[1] && iw < i3[2])));
                if (v > mine || (before && v == mine)) { winner = false; break; }
              }
            }
          }
          if (winner) g += bf2f(dy[(((t * p.osp[0] + od) * p.osp[1] + oh) * p.osp[2] + ow) * p.c + ch]);
        }
  }
  dx[idx] = f2bf(g);
}

// The same gather with 8 channels per thread (channel count a multiple of 8).
__global__ __launch_bounds__(TB) void maxpool_bwd_vec_kernel(PoolP p, const uint4* dy, const uint4* x, int mask_relu, uint4* dx,
                                                             long long total) {
  const long long idx = (long long)blockIdx.x * TB + threadIdx.x;     // (input position, channel vector)
  if (idx >= total) return;
  const int c8 = p.c >> 3;
  const int cv = (int)(idx % c8);
  long long t = idx / c8;
  int i3[3];
  i3[2] = (int)(t % p.isp[2]); t /= p.isp[2];
  i3[1] = (int)(t % p.isp[1]); t /= p.isp[1];
  i3[0] = (int)(t % p.isp[0]); t /= p.isp[0];
  float mine[8], g[8];
  unpack8(x[idx], mine);
#pragma unroll
  for (int e = 0; e < 8; ++e) g[e] = 0.f;
  int lo[3], hi[3];
  for (int a = 0; a < 3; ++a) {
    const int num = i3[a] + p.pad[a] - p.win[a] + 1;
    lo[a] = num <= 0 ? 0 : (num + p.stride[a] - 1) / p.stride[a];
    hi[a] = (i3[a] + p.pad[a]) / p.stride[a];
    if (hi[a] > p.osp[a] - 1) hi[a] = p.osp[a] - 1;
  }
  for (int od = lo[0]; od <= hi[0]; ++od)
    for (int oh = lo[1]; oh <= hi[1]; ++oh)
      for (int ow = lo[2]; ow <= hi[2]; ++ow) {
        bool winner[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) winner[e] = true;
        for (int kd = 0; kd < p.win[0]; ++kd) {
          const int id = od * p.stride[0] + kd - p.pad[0];
          if (id < 0 || id >= p.isp[0]) continue;
          for (int kh = 0; kh < p.win[1]; ++kh) {
            const int ih = oh * p.stride[1] + kh - p.pad[1];
            if (ih < 0 || ih >= p.isp[1]) continue;
            for (int kw = 0; kw < p.win[2]; ++kw) {
              const int iw = ow * p.stride[2] + kw - p.pad[2];
              if (iw < 0 || iw >= p.isp[2]) continue;
              float v[8];
              unpack8(x[(((t * p.isp[0] + id) * p.isp[1] + ih) * p.isp[2] + iw) * c8 + cv], v);
              const bool before = (id < i3[0]) || (id == i3[0] && (ih < i3[1] || (ih == i3[1] && iw < i3[2])));
#pragma unroll
              for (int e = 0; e < 8; ++e)
                if (v[e] > mine[e] || (before && v[e] == mine[e])) winner[e] = false;
            }
          }
        }
        float d[8];
        unpack8(dy[(((t * p.osp[0] + od) * p.osp[1] + oh) * p.osp[2] + ow) * c8 + cv], d);
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (winner[e]) g[e] += d[e];
      }
  uint32_t w[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float a = (mask_relu && !(mine[2 * e] > 0.f)) ? 0.f : g[2 * e];
    const float b = (mask_relu && !(mine[2 * e + 1] > 0.f)) ? 0.f : g[2 * e + 1];
    w[e] = (uint32_t)f2bf(a) | ((uint32_t)f2bf(b) << 16);
  }
  dx[idx] = make_uint4(w[0], w[1], w[2], w[3]);
}

// Non-overlapping pooling (window = stride = 2, no padding), 8 channels per thread.  One thread owns one
// window: forward writes its maximum, backward routes dy to the first maximum (row-major window order).
template <int BWD>
__global__ __launch_bounds__(TB) void maxpool2_kernel(PoolP p, const uint4* x, const uint4* dy, int mask_relu, uint4* out, long long total) {
  const long long idx = (long long)blockIdx.x * TB + threadIdx.x;     // (output position, channel vector)
  if (idx >= total) return;
  const int c8 = p.c / 8;
  const int cv = (int)(idx % c8);
  long long t = idx / c8;
  const int ow = (int)(t % p.osp[2]); t /= p.osp[2];
  const int oh = (int)(t % p.osp[1]); t /= p.osp[1];
  const int od = (int)(t % p.osp[0]); t /= p.osp[0];
  const int nd = p.win[0], nh = p.win[1], nw = p.win[2];               // 1 or 2 each
  float best[8];
  int arg[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { best[e] = -INFINITY; arg[e] = 0; }
  int k = 0;
  for (int kd = 0; kd < nd; ++kd)
    for (int kh = 0; kh < nh; ++kh)
      for (int kw = 0; kw < nw; ++kw, ++k) {
        const long long src = ((((t * p.isp[0] + od * nd + kd) * p.isp[1] + oh * nh + kh) * p.isp[2] + ow * nw + kw)) * c8 + cv;
        float f[8];
        unpack8(x[src], f);
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (f[e] > best[e]) { best[e] = f[e]; arg[e] = k; }
      }
  if (!BWD) {
    // the maximum is one of the inputs: copy its bits
    uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
    for (int e = 0; e < 8; ++e) w[e >> 1] |= (__float_as_uint(best[e]) >> 16) << ((e & 1) * 16);
    out[idx] = make_uint4(w[0], w[1], w[2], w[3]);
    return;
  }
  const uint4 g = dy[idx];
  const uint32_t gw[4] = {g.x, g.y, g.z, g.w};
  k = 0;
  for (int kd = 0; kd < nd; ++kd)
    for (int kh = 0; kh < nh; ++kh)
      for (int kw = 0; kw < nw; ++kw, ++k) {
        const long long dst = ((((t * p.isp[0] + od * nd + kd) * p.isp[1] + oh * nh + kh) * p.isp[2] + ow * nw + kw)) * c8 + cv;
        uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const bool win = arg[e] == k && !(mask_relu && !(best[e] > 0.f));
          const uint32_t ge = (gw[e >> 1] >> ((e & 1) * 16)) & 0xffffu;
          if (win) w[e >> 1] |= ge << ((e & 1) * 16);
        }
        out[dst] = make_uint4(w[0], w[1], w[2], w[3]);
      }
}

struct Ptrs4v { const uint4* g[4]; };
__global__ __launch_bounds__(TB) void grad_sum_vec_kernel(Ptrs4v in, int n_in, const uint4* mask, long long n8, uint4* out) {
  const long long i = (long long)blockIdx.x * TB + threadIdx.x;
  if (i >= n8) return;
  float s[8], f[8];
  unpack8(in.g[0][i], s);
  for (int j = 1; j < n_in; ++j) {
    unpack8(in.g[j][i], f);
#pragma unroll
    for (int e = 0; e < 8; ++e) s[e] += f[e];
  }
  if (mask) {
    unpack8(mask[i], f);
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (!(f[e] > 0.f)) s[e] = 0.f;
  }
  uint32_t w[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) w[e] = (uint32_t)f2bf(s[2 * e]) | ((uint32_t)f2bf(s[2 * e + 1]) << 16);
  out[i] = make_uint4(w[0], w[1], w[2], w[3]);
}

// Vector forms of the squared-error kernels (8 elements per load); same partial layout as the scalar ones.
__global__ __launch_bounds__(TB) void mse_partial_vec_kernel(const uint4* y, const uint4* t, long long n8, float* part) {
  __shared__ float sh[TB];
  float s = 0.f;
  for (long long i = (long long)blockIdx.x * TB + threadIdx.x; i < n8; i += (long long)gridDim.x * TB) {
    float a[8], b[8];
    unpack8(y[i], a);
    unpack8(t[i], b);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float d = a[e] - b[e];
      s += d * d;
    }
  }
  const float tot = block_sum(s, sh);
  if (threadIdx.x == 0) part[blockIdx.x] = tot;
}

__global__ __launch_bounds__(TB) void mse_grad_vec_kernel(const uint4* y, const uint4* t, const uint4* mask, long long n8, float coef,
                                                          uint4* dy) {
  const long long i = (long long)blockIdx.x * TB + threadIdx.x;
  if (i >= n8) return;
  float a[8], b[8];
  unpack8(y[i], a);
  unpack8(t[i], b);
#pragma unroll
  for (int e = 0; e < 8; ++e) a[e] = coef * (a[e] - b[e]);
  if (mask) {
    unpack8(mask[i], b);
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (!(b[e] > 0.f)) a[e] = 0.f;
  }
  uint32_t w[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) w[e] = (uint32_t)f2bf(a[2 * e]) | ((uint32_t)f2bf(a[2 * e + 1]) << 16);
  dy[i] = make_uint4(w[0], w[1], w[2], w[3]);
}

__global__ __launch_bounds__(TB) void gap_fwd_kernel(const uint16_t* x, uint16_t* y, long long n, long long positions, int c) {
  const long long idx = (long long)blockIdx.x * TB + threadIdx.x;
  if (idx >= n * c) return;
  const int ch = (int)(idx % c);
  const long long b = idx / c;
  float s = 0.f;
  for (long long q = 0; q < positions; ++q) s += bf2f(x[(b * positions + q) * c + ch]);
  y[idx] = f2bf(s / (float)positions);
}
__global__ __launch_bounds__(TB) void gap_bwd_kernel(const uint16_t* dy, const uint16_t* mask, uint16_t* dx, long long total,
                                                     long long positions, int c) {
  const long long idx = (long long)blockIdx.x * TB + threadIdx.x;
  if (idx >= total) return;
  const int ch = (int)(idx % c);
  const long long b = idx / c / positions;
  float g = bf2f(dy[b * c + ch]) / (float)positions;
  if (mask && !(bf2f(mask[idx]) > 0.f)) g = 0.f;
  dx[idx] = f2bf(g);
}

__global__ __launch_bounds__(TB) void copy_channels_kernel(const uint16_t* src, int src_c, int src_begin, uint16_t* dst, int dst_c,
                                                           int dst_begin, int count, const uint16_t* mask, long long total) {
  const long long idx = (long long)blockIdx.x * TB + threadIdx.x;
  if (idx >= total) return;
  const int ch = (int)(idx % count);
  const long long r = idx / count;
  uint16_t v = src[r * src_c + src_begin + ch];
  const long long o = r * dst_c + dst_begin + ch;
  if (mask && !(bf2f(mask[o]) > 0.f)) v = 0;
  dst[o] = v;
}
__global__ __launch_bounds__(TB) void copy_channels_vec_kernel(const uint4* src, int src_c8, int src_begin8, uint4* dst, int dst_c8,
                                                               int dst_begin8, int count8, long long total) {
  const long long idx = (long long)blockIdx.x * TB + threadIdx.x;
  if (idx >= total) return;
  const int ch = (int)(idx % count8);
  const long long r = idx / count8;
  dst[r * dst_c8 + dst_begin8 + ch] = src[r * src_c8 + src_begin8 + ch];
}

// Swap copy between HBM and pinned host memory (mapped into the device address space): a small
// persistent grid so that the copy, which is bound by the host link, leaves the other CUs to the
// compute stream.  Four independent 16-byte accesses per thread per round keep enough requests in flight.
__global__ __launch_bounds__(TB) void swap_copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, long long n16) {
  const long long stride = (long long)gridDim.x * TB;
  long long i = (long long)blockIdx.x * TB + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    dst[i] = a; dst[i + stride] = b; dst[i + 2 * stride] = c; dst[i + 3 * stride] = d;
  }
  for (; i < n16; i += stride) dst[i] = src[i];
}
__global__ void swap_copy_tail_kernel(unsigned char* dst, const unsigned char* src, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}

// Lossless swap encoding (the encoding / decoding pair that Section 4.2.1 allows in place of the two
// identities).  Slots of 2048 16-bit elements (bfloat16 bit patterns).  A slot holds a 256-byte bitmap (bit i%8 of
// byte i/8: element i is not 0x0000), a 16-byte header (byte 0: mode, byte 1: largest exponent field of the
// non-zero elements) and the non-zero elements in order: raw (mode 0: 16 bits each) or packed (mode bit 0) as codes
// of 7 mantissa bits, 4 or 5 (mode bit 1: wide) bits of emax - exponent and a sign bit only if some value has one
// (mode bit 2: signed), 11 to 13 bits, as a little-endian bit stream.  A slot is packed iff all exponent fields lie
// within 31 of the largest, wide iff not within 15.  A packed slot without signs is stored split instead (mode bit
// 3, the wide bit clear) iff that takes fewer bytes: with d = emax - exponent, one byte (d & 1) << 7 | mantissa per
// element, padding to a multiple of 4, then the quotients d >> 1 in unary (so many zero bits and a one bit per
// element) as a little-endian bit stream: a Rice code of the differences, which crowd near zero.  Header bytes 2-3:
// the slot's value bytes.  Slot s starts at s * 4368 bytes, so work-groups handle slots
// independently and a copy moves only bitmap, header and values.  After the slots: one u32 per slot (count of
// non-zero elements in bits 0-11, bits 15 / 14 / 13 / 12: packed / wide / signed / split, value bytes in bits 16-31;
// padded to 16 bytes), then a 16-byte trailer with the slot bytes a copy moves.  One work-group of 256
// threads per slot round, 8 elements per thread; a work-group owns a contiguous run of slots and writes their
// counts in one go.
constexpr int ENC_EL = 2048, ENC_MAP = 256, ENC_HDR = 16, ENC_VAL = ENC_MAP + ENC_HDR, ENC_STRIDE = ENC_VAL + 2 * ENC_EL, ENC_TRAILER = 16;
constexpr int ENC_RUN = 1024;     // slots per work-group at most (counts kept in LDS)
constexpr int ENC_SPAN = 15, ENC_SPAN_WIDE = 31;      // exponent spans that 4 and 5 bits of difference cover
constexpr int ENC_PACKED = 1, ENC_WIDE = 2, ENC_SIGNED = 4, ENC_SPLIT = 8;

__host__ __device__ inline long long enc_counts_offset(long long nslots) { return nslots * ENC_STRIDE; }
__host__ __device__ inline long long enc_trailer_offset(long long nslots) { return nslots * ENC_STRIDE + (4 * nslots + 15) / 16 * 16; }
__host__ __device__ inline int enc_code_bits(int mode) { return 7 + ((mode & ENC_WIDE) ? 5 : 4) + ((mode & ENC_SIGNED) ? 1 : 0); }
__host__ __device__ inline int enc_value_bytes(int cnt, int mode) { return (mode & ENC_PACKED) ? (enc_code_bits(mode) * cnt + 7) / 8 : 2 * cnt; }

// exclusive prefix of cnt over the 256 threads of the block and the block total (wsum: 4 ints of LDS)
__device__ __forceinline__ int block_prefix(int cnt, int* wsum, int& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = cnt;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int t = __shfl_up(inc, d, 64);
    if (lane >= d) inc += t;
  }
  if (lane == 63) wsum[wave] = inc;
  __syncthreads();
  int base = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j)
    if (j < wave) base += wsum[j];
  total = wsum[0] + wsum[1] + wsum[2] + wsum[3];
  return base + inc - cnt;
}

// 32 values (LDS, 64-byte aligned; the first `valid` count) -> 32 codes of B bits = B words of the bit stream.
template <int B>
__device__ __forceinline__ void enc_pack32(const uint16_t* v, int valid, uint32_t emax, bool sgn, uint32_t* out) {
  unsigned long long acc = 0;
  int nb = 0, o = 0;
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    const uint4 q = *reinterpret_cast<const uint4*>(v + 8 * g);
    const uint32_t qw[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint32_t x = (qw[i >> 1] >> (16 * (i & 1))) & 0xffffu;
      uint32_t code = (emax - ((x >> 7) & 0xffu)) << 7 | (x & 0x7fu);
      if (sgn) code |= (x >> 15) << (B - 1);
      if (8 * g + i >= valid) code = 0;
      acc |= (unsigned long long)code << nb;
      nb += B;
      if (nb >= 32) {
        out[o++] = (uint32_t)acc;
        acc >>= 32;
        nb -= 32;
      }
    }
  }
}

// The slots [slot_begin, slot_end) of a tensor.  stage / wstage: the first wstage bytes (a multiple of 16) of each of these slots
// go to device memory at stage + (slot - slot_begin) * ENC_STRIDE instead of the host buffer (a copy engine carries
// them over afterwards); bytes beyond wstage, and everything if stage is null, are written to the host buffer directly.
__global__ __launch_bounds__(TB) void swap_encode_kernel(unsigned char* __restrict__ dst, const uint4* __restrict__ src, long long n8,
                                                         long long nslots, long long slot_begin, long long slot_end, long long per,
                                                         unsigned char* __restrict__ stage, int wstage) {
  __shared__ __attribute__((aligned(16))) uint16_t vals[ENC_EL];
  __shared__ __attribute__((aligned(16))) uint32_t pk[ENC_EL * 13 / 32];      // packed values of a slot
  __shared__ __attribute__((aligned(16))) unsigned char bitmap[ENC_MAP];
  __shared__ uint32_t counts[ENC_RUN];
  __shared__ int wsum[4], wsum2[4], wmx[4], wmn[4], wsg[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const long long lo0 = slot_begin + (long long)blockIdx.x * per;
  const long long hi0 = lo0 + per < slot_end ? lo0 + per : slot_end;
  // the slot counts of a run of ENC_RUN slots are kept in LDS and written together
  // the elements of a slot are requested one slot ahead: they arrive while this one is packed and stored
  uint4 q_next = make_uint4(0, 0, 0, 0);
  if (lo0 < hi0 && lo0 * TB + tid < n8) q_next = src[lo0 * TB + tid];
  for (long long lo = lo0; lo < hi0; lo += ENC_RUN) {
  const long long hi = lo + ENC_RUN < hi0 ? lo + ENC_RUN : hi0;
  for (long long slot = lo; slot < hi; ++slot) {
    const uint4 q = q_next;
    q_next = make_uint4(0, 0, 0, 0);
    if (slot + 1 < hi0 && (slot + 1) * TB + tid < n8) q_next = src[(slot + 1) * TB + tid];
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
    uint32_t m = 0;
    int emx = 0, emn = 255, sg = 0;       // exponent fields and sign bits of this thread's non-zero elements
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t v = (w[e >> 1] >> (16 * (e & 1))) & 0xffffu;
      if (v) {
        m |= 1u << e;
        const int ex = (int)((v >> 7) & 0xffu);
        emx = ex > emx ? ex : emx;
        emn = ex < emn ? ex : emn;
        sg |= (int)(v >> 15);
      }
    }
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int a = __shfl_xor(emx, d, 64), b = __shfl_xor(emn, d, 64);
      emx = a > emx ? a : emx;
      emn = b < emn ? b : emn;
      sg |= __shfl_xor(sg, d, 64);
    }
    if (lane == 0) { wmx[wave] = emx; wmn[wave] = emn; wsg[wave] = sg; }
    bitmap[tid] = (unsigned char)m;
    int total;
    const int off0 = block_prefix(__popc(m), wsum, total);   // its barrier also publishes wmx / wmn
    int off = off0;
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (m & (1u << e)) vals[off++] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
    int emax = wmx[0], emin = wmn[0];
#pragma unroll
    for (int j = 1; j < 4; ++j) {
      emax = wmx[j] > emax ? wmx[j] : emax;
      emin = wmn[j] < emin ? wmn[j] : emin;
    }
    const bool sgn = (wsg[0] | wsg[1] | wsg[2] | wsg[3]) != 0;
    int mode = 0;
    if (total > 0 && emax - emin <= ENC_SPAN_WIDE)
      mode = ENC_PACKED | (emax - emin > ENC_SPAN ? ENC_WIDE : 0) | (sgn ? ENC_SIGNED : 0);
    // the split form: this thread's share of the unary stream, one bit per element and per step of 2 in emax - exponent
    const bool may_split = (mode & ENC_PACKED) && !sgn;
    int ubits = 0;
    if (may_split) {
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (m & (1u << e)) ubits += ((emax - (int)((w[e >> 1] >> (16 * (e & 1) + 7)) & 0xffu)) >> 1) + 1;
    }
    int utotal;
    const int uoff = block_prefix(ubits, wsum2, utotal);
    const int first = (total + 3) & ~3;                       // where the unary stream starts
    const bool split = may_split && first + ((utotal + 7) >> 3) < enc_value_bytes(total, mode);
    if (split) mode = ENC_PACKED | ENC_SPLIT;
    const int nbytes = split ? first + ((utotal + 7) >> 3) : enc_value_bytes(total, mode);
    if (tid == 0)
      counts[slot - lo] = (uint32_t)total | (mode & ENC_PACKED ? 0x8000u : 0u) | (mode & ENC_WIDE ? 0x4000u : 0u) |
                          (mode & ENC_SIGNED ? 0x2000u : 0u) | (mode & ENC_SPLIT ? 0x1000u : 0u) | (uint32_t)nbytes << 16;
    if (split)
      for (int i = tid; i < (utotal + 31) >> 5; i += TB) pk[(first >> 2) + i] = 0;
    __syncthreads();
    unsigned char* out = dst + slot * ENC_STRIDE;
    unsigned char* sout = stage + (slot - slot_begin) * ENC_STRIDE;
    // byte o of the slot: staged below w, host beyond
    auto at = [&](int o) -> uint4* { return reinterpret_cast<uint4*>((o < wstage ? sout : out) + o); };
    if (tid < ENC_MAP / 16) *at(tid * 16) = *reinterpret_cast<const uint4*>(bitmap + tid * 16);
    if (tid == ENC_MAP / 16) *at(ENC_MAP) = make_uint4((mode ? ((uint32_t)mode | (uint32_t)emax << 8) : 0u) | (uint32_t)nbytes << 16, 0, 0, 0);
    const unsigned char* packed = reinterpret_cast<const unsigned char*>(vals);
    if (split) {
      unsigned char* pb = reinterpret_cast<unsigned char*>(pk);
      int j = off0, ub = uoff;
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (m & (1u << e)) {
          const uint32_t v = (w[e >> 1] >> (16 * (e & 1))) & 0xffffu;
          const uint32_t d = (uint32_t)emax - ((v >> 7) & 0xffu);
          pb[j++] = (unsigned char)((d & 1u) << 7 | (v & 0x7fu));
          ub += (int)(d >> 1);
          atomicOr(&pk[(first >> 2) + (ub >> 5)], 1u << (ub & 31));
          ++ub;
        }
      __syncthreads();
      packed = pb;
    } else if (mode) {
      // thread t packs the values [32t, 32t + 32): 32 codes of B bits are B words of the bit stream
      const int bits = enc_code_bits(mode);
      if (32 * tid < total) {
        const uint16_t* v = vals + 32 * tid;
        uint32_t* o = pk + bits * tid;
        const int valid = total - 32 * tid;
        if (bits == 11) enc_pack32<11>(v, valid, (uint32_t)emax, false, o);
        else if (bits == 13) enc_pack32<13>(v, valid, (uint32_t)emax, true, o);
        else enc_pack32<12>(v, valid, (uint32_t)emax, sgn, o);
      }
      __syncthreads();
      packed = reinterpret_cast<const unsigned char*>(pk);
    }
    const int nv = (nbytes + 15) >> 4;
    for (int i = tid; i < nv; i += TB)
      *at(ENC_VAL + i * 16) = *reinterpret_cast<const uint4*>(packed + i * 16);
    __syncthreads();      // LDS is reused by the next slot
  }
  uint32_t* cdst = reinterpret_cast<uint32_t*>(dst + enc_counts_offset(nslots)) + lo;
  for (long long i = tid; i < hi - lo; i += TB) cdst[i] = counts[i];
  __syncthreads();      // counts is reused by the next run
  }
}

// Trailer of an encoded buffer: slot bytes moved = sum over slots of bitmap + header + value bytes rounded up to 16
// bytes, from the count region (read back over the host link with wide loads).
__global__ __launch_bounds__(TB) void swap_trailer_kernel(unsigned char* buf, long long nslots) {
  __shared__ unsigned long long sh[TB];
  const uint4* c = reinterpret_cast<const uint4*>(buf + enc_counts_offset(nslots));
  const long long nv = (nslots + 3) / 4;
  unsigned long long s = 0;
  for (long long i = threadIdx.x; i < nv; i += TB) {
    const uint4 q = c[i];
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (i * 4 + e < nslots) s += ENC_VAL + (unsigned long long)(((w[e] >> 16) + 15) / 16 * 16);
  }
  sh[threadIdx.x] = s;
  __syncthreads();
  for (int d = TB / 2; d > 0; d >>= 1) {
    if ((int)threadIdx.x < d) sh[threadIdx.x] += sh[threadIdx.x + d];
    __syncthreads();
  }
  if (threadIdx.x == 0)
    *reinterpret_cast<uint4*>(buf + enc_trailer_offset(nslots)) = make_uint4((uint32_t)sh[0], (uint32_t)(sh[0] >> 32), 0, 0);
}

// The slots [slot_begin, slot_end); stage / wstage as in the encoder: the first wstage bytes of each slot are read from device
// memory (brought there by a copy engine), the rest from the host buffer.
__global__ __launch_bounds__(TB) void swap_decode_kernel(uint4* __restrict__ dst, const unsigned char* __restrict__ src, long long n8,
                                                         long long slot_begin, long long slot_end,
                                                         const unsigned char* __restrict__ stage, int wstage) {
  __shared__ __attribute__((aligned(16))) uint32_t vals[ENC_EL / 2 + 4];      // value bytes of a slot (+ one vector: the code fetch reads two words)
  __shared__ __attribute__((aligned(16))) unsigned char bitmap[ENC_VAL];      // bitmap and header
  __shared__ uint16_t upos[ENC_EL];       // split slots: position of each element's one bit in the unary stream
  __shared__ int wsum[4], wsum2[4];
  const int tid = threadIdx.x;
  constexpr int HV = ENC_VAL / 16;        // vectors of bitmap + header
  // Bitmap and header of the next slot are requested while the values of this one are on their way.  (Requesting the
  // next slot's values as well, one more round trip ahead, raises the stand-alone rate from 49 to 53 GB/s and makes
  // the swapped ResNet-50 step 2 % longer: the deeper queue on the link slows the convolutions beside the decoder.)
  auto at = [&](long long slot, int o) -> const uint4* {
    return reinterpret_cast<const uint4*>((o < wstage ? stage + (slot - slot_begin) * ENC_STRIDE : src + slot * ENC_STRIDE) + o);
  };
  uint4 next_map = make_uint4(0, 0, 0, 0);
  if (tid < HV && slot_begin + (long long)blockIdx.x < slot_end) next_map = *at(slot_begin + blockIdx.x, tid * 16);
  for (long long slot = slot_begin + blockIdx.x; slot < slot_end; slot += gridDim.x) {
    if (tid < HV) *reinterpret_cast<uint4*>(bitmap + tid * 16) = next_map;
    __syncthreads();
    const uint32_t m = bitmap[tid];
    const int mode = bitmap[ENC_MAP];
    const uint32_t emax = bitmap[ENC_MAP + 1];
    int nbytes = (int)bitmap[ENC_MAP + 2] | (int)bitmap[ENC_MAP + 3] << 8;
    nbytes = nbytes < 2 * ENC_EL ? nbytes : 2 * ENC_EL;     // a damaged header must not lead outside the slot
    const int bits = enc_code_bits(mode);
    const uint32_t dmask = (mode & ENC_WIDE) ? 31u : 15u;
    // the value bytes: at most one 16-byte vector per thread
    if (tid < ((nbytes + 15) >> 4))
      *reinterpret_cast<uint4*>(reinterpret_cast<unsigned char*>(vals) + tid * 16) = *at(slot, ENC_VAL + tid * 16);
    const long long nxt = slot + gridDim.x;
    if (tid < HV && nxt < slot_end) next_map = *at(nxt, tid * 16);
    int total;
    int off = block_prefix(__popc(m), wsum, total);
    if (mode & ENC_SPLIT) {
      // The unary stream: every thread takes a contiguous run of its words, counts their one bits, and after a prefix
      // sum over the threads knows which elements they belong to: element r's one bit sits at stream position upos[r].
      const int first = (total + 3) & ~3;
      const int ubytes = nbytes - first;                   // bytes of the stream; what follows in its last word is unspecified
      const int uwords = (ubytes + 3) >> 2;
      const int wpt = (uwords + TB - 1) / TB;
      const uint32_t* uw = vals + (first >> 2);
      auto word_at = [&](int i) -> uint32_t {
        const int valid = ubytes - 4 * i;
        return valid >= 4 ? uw[i] : uw[i] & ((1u << (8 * valid)) - 1u);
      };
      int ones = 0;
      for (int i = tid * wpt; i < (tid + 1) * wpt && i < uwords; ++i) ones += __popc(word_at(i));
      int all;
      int r = block_prefix(ones, wsum2, all);
      for (int i = tid * wpt; i < (tid + 1) * wpt && i < uwords; ++i) {
        uint32_t x = word_at(i);
        while (x) {
          const int b = __ffs(x) - 1;
          x &= x - 1;
          if (r < ENC_EL) upos[r] = (uint16_t)(32 * i + b);
          ++r;
        }
      }
      __syncthreads();
    }
    uint32_t w[4] = {0, 0, 0, 0};
    const uint16_t* v16 = reinterpret_cast<const uint16_t*>(vals);
    const unsigned char* v8 = reinterpret_cast<const unsigned char*>(vals);
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (m & (1u << e)) {
        uint32_t v;
        if (mode & ENC_SPLIT) {
          const int q = (int)upos[off] - (off ? (int)upos[off - 1] + 1 : 0);
          const uint32_t byte = v8[off];
          v = (emax - (2u * (uint32_t)q + (byte >> 7))) << 7 | (byte & 0x7fu);
        } else if (mode & ENC_PACKED) {
          const int bit = bits * off;
          const uint32_t code = __builtin_amdgcn_alignbit(vals[(bit >> 5) + 1], vals[bit >> 5], bit & 31) & ((1u << bits) - 1u);
          v = (emax - ((code >> 7) & dmask)) << 7 | (code & 0x7fu);
          if (mode & ENC_SIGNED) v |= (code >> (bits - 1)) << 15;
        } else {
          v = v16[off];
        }
        ++off;
        w[e >> 1] |= (v & 0xffffu) << (16 * (e & 1));
      }
    const long long vi = slot * TB + tid;
    if (vi < n8) dst[vi] = make_uint4(w[0], w[1], w[2], w[3]);
    __syncthreads();      // LDS is reused by the next slot
  }
}

// Update of Section 3.3: out = p - lr * g, in the parameter's storage type (bf16: round to nearest even).  out may be p.
__global__ __launch_bounds__(TB) void sgd_bf16_kernel(const uint16_t* p, const float* g, float lr, long long n, uint16_t* out) {
  const long long i = (long long)blockIdx.x * TB + threadIdx.x;
  if (i < n) out[i] = f2bf(__builtin_fmaf(-lr, g[i], bf2f(p[i])));
}
__global__ __launch_bounds__(TB) void sgd_f32_kernel(const float* p, const float* g, float lr, long long n, float* out) {
  const long long i = (long long)blockIdx.x * TB + threadIdx.x;
  if (i < n) out[i] = __builtin_fmaf(-lr, g[i], p[i]);
}

__global__ __launch_bounds__(TB) void sgd_multi_kernel(SgdBatch b) {
  // the tensor this work-group belongs to: the last one whose first work-group is not after it (uniform: scalar code)
  int lo = 0, hi = b.count;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (b.first[mid] <= (int)blockIdx.x) lo = mid; else hi = mid;
  }
  const long long i = (long long)((int)blockIdx.x - b.first[lo]) * TB + threadIdx.x;
  if (i >= b.n[lo]) return;
  const float g = b.g[lo][i], lr = b.lr[lo];
  if ((b.f32_mask >> lo) & 1ull) {
    static_cast<float*>(b.out[lo])[i] = __builtin_fmaf(-lr, g, static_cast<const float*>(b.p[lo])[i]);
  } else {
    static_cast<uint16_t*>(b.out[lo])[i] = f2bf(__builtin_fmaf(-lr, g, bf2f(static_cast<const uint16_t*>(b.p[lo])[i])));
  }
}

PoolP pool_params(const ConvGeom& g) {
  PoolP p;
  p.n = g.n;
  p.c = g.c;
  for (int i = 0; i < 3; ++i) {
    p.isp[i] = g.in_sp[i]; p.osp[i] = g.out_sp[i]; p.win[i] = g.filt[i]; p.stride[i] = g.stride[i]; p.pad[i] = g.pad[i];
  }
  return p;
}

}  // namespace

uint64_t reduce_ws(int64_t rows, int cols) {
  // MAX_PARTS slices of `cols` values; a scalar reduction may instead keep one value per row
  if (cols > 0) return (uint64_t)MAX_PARTS * cols * 4;
  return (uint64_t)(rows > MAX_PARTS ? rows : MAX_PARTS) * 4;
}

hipError_t mse_loss(int64_t numel, const void* y, const void* t, float* loss, void* ws, hipStream_t s) {
  const int parts = parts_for(numel);
  if ((numel & 7) == 0 && (((uintptr_t)y | (uintptr_t)t) & 15) == 0)
    hipLaunchKernelGGL(mse_partial_vec_kernel, dim3(parts), dim3(TB), 0, s, (const uint4*)y, (const uint4*)t, (long long)(numel / 8), (float*)ws);
  else
  hipLaunchKernelGGL(mse_partial_kernel, dim3(parts), dim3(TB), 0, s, (const uint16_t*)y, (const uint16_t*)t, (long long)numel, (float*)ws);
  hipLaunchKernelGGL(finish_mean_kernel, dim3(1), dim3(TB), 0, s, (const float*)ws, parts, (float)numel, loss);
  return hipGetLastError();
}
hipError_t mse_grad(int64_t numel, const void* y, const void* t, const void* mask, void* dy, hipStream_t s) {
  if ((numel & 7) == 0 && (((uintptr_t)y | (uintptr_t)t | (uintptr_t)mask | (uintptr_t)dy) & 15) == 0) {
    hipLaunchKernelGGL(mse_grad_vec_kernel, dim3(cdiv(numel / 8, TB)), dim3(TB), 0, s, (const uint4*)y, (const uint4*)t,
                       (const uint4*)mask, (long long)(numel / 8), 2.0f / (float)numel, (uint4*)dy);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(mse_grad_kernel, dim3(cdiv(numel, TB)), dim3(TB), 0, s, (const uint16_t*)y, (const uint16_t*)t,
                     (const uint16_t*)mask, (long long)numel, 2.0f / (float)numel, (uint16_t*)dy);
  return hipGetLastError();
}
hipError_t softmax_ce_loss(int64_t rows, int classes, const void* z, const int32_t* labels, float* loss, void* ws, hipStream_t s) {
  int parts;
  if (classes <= 64) {
    parts = parts_for(rows);
    hipLaunchKernelGGL(ce_rows_kernel, dim3(parts), dim3(TB), 0, s, (const uint16_t*)z, labels, (long long)rows, classes, (float*)ws,
                       (const uint16_t*)nullptr, (uint16_t*)nullptr, 0.f);
  } else {
    parts = (int)rows;
    hipLaunchKernelGGL(ce_wide_kernel, dim3((unsigned)rows), dim3(TB), 0, s, (const uint16_t*)z, labels, classes, (float*)ws,
                       (const uint16_t*)nullptr, (uint16_t*)nullptr, 0.f);
  }
  hipLaunchKernelGGL(finish_mean_kernel, dim3(1), dim3(TB), 0, s, (const float*)ws, parts, (float)rows, loss);
  return hipGetLastError();
}
hipError_t softmax_ce_grad(int64_t rows, int classes, const void* z, const int32_t* labels, const void* mask, void* dz, hipStream_t s) {
  const float inv = 1.0f / (float)rows;
  if (classes <= 64)
    hipLaunchKernelGGL(ce_rows_kernel, dim3(cdiv(rows, TB)), dim3(TB), 0, s, (const uint16_t*)z, labels, (long long)rows, classes,
                       (float*)nullptr, (const uint16_t*)mask, (uint16_t*)dz, inv);
  else
    hipLaunchKernelGGL(ce_wide_kernel, dim3((unsigned)rows), dim3(TB), 0, s, (const uint16_t*)z, labels, classes, (float*)nullptr,
                       (const uint16_t*)mask, (uint16_t*)dz, inv);
  return hipGetLastError();
}
hipError_t grad_sum(int64_t numel, int n, const void* const* g, const void* mask, void* out, hipStream_t s) {
  if (n < 1 || n > 4) return hipErrorInvalidValue;
  bool aligned = (numel & 7) == 0 && ((uintptr_t)out & 15) == 0 && (!mask || ((uintptr_t)mask & 15) == 0);
  for (int i = 0; i < n; ++i) aligned = aligned && ((uintptr_t)g[i] & 15) == 0;
  if (aligned) {
    Ptrs4v in{};
    for (int i = 0; i < n; ++i) in.g[i] = (const uint4*)g[i];
    hipLaunchKernelGGL(grad_sum_vec_kernel, dim3(cdiv(numel / 8, TB)), dim3(TB), 0, s, in, n, (const uint4*)mask, (long long)(numel / 8), (uint4*)out);
    return hipGetLastError();
  }
  Ptrs4 in{};
  for (int i = 0; i < n; ++i) in.g[i] = (const uint16_t*)g[i];
  hipLaunchKernelGGL(grad_sum_kernel, dim3(cdiv(numel, TB)), dim3(TB), 0, s, in, n, (const uint16_t*)mask, (long long)numel, (uint16_t*)out);
  return hipGetLastError();
}
hipError_t colsum(int64_t rows, int c, const void* dy, float* out, void* ws, hipStream_t s) {
  long long p = (rows + 63) / 64;
  const int parts = (int)(p < 1 ? 1 : (p > MAX_PARTS ? MAX_PARTS : p));
  if ((c & 7) == 0 && c <= 8 * TB && TB % (c >> 3) == 0 && ((uintptr_t)dy & 15) == 0)
    hipLaunchKernelGGL(colsum_partial_vec_kernel, dim3(parts), dim3(TB), 0, s, (const uint4*)dy, (long long)rows, c, (float*)ws);
  else
    hipLaunchKernelGGL(colsum_partial_kernel, dim3(parts), dim3(TB), 0, s, (const uint16_t*)dy, (long long)rows, c, (float*)ws);
  hipLaunchKernelGGL(col_reduce_kernel, dim3(cdiv(c, 32)), dim3(1024), 0, s, (const float*)ws, (const uint16_t*)nullptr, (long long)parts, c, out);
  return hipGetLastError();
}
hipError_t col_reduce(const float* part, int64_t parts, int c, float* out, hipStream_t s) {
  hipLaunchKernelGGL(col_reduce_kernel, dim3(cdiv(c, 32)), dim3(1024), 0, s, part, (const uint16_t*)nullptr, (long long)parts, c, out);
  return hipGetLastError();
}
hipError_t scale_cols(int64_t j, int k, const float* raw, const float* scale, float* out, hipStream_t s) {
  const long long total = (long long)j * k;
  hipLaunchKernelGGL(scale_cols_kernel, dim3(cdiv(total, TB)), dim3(TB), 0, s, raw, scale, out, total, k);
  return hipGetLastError();
}
hipError_t dot_cols(int64_t j, int k, const float* raw, const void* w, float* out, hipStream_t s) {
  hipLaunchKernelGGL(col_reduce_kernel, dim3(cdiv(k, 32)), dim3(1024), 0, s, raw, (const uint16_t*)w, (long long)j, k, out);
  return hipGetLastError();
}
hipError_t fill16(void* p, uint64_t bytes, uint16_t pattern, hipStream_t s) {
  const long long n = (long long)(bytes / 2);
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(fill16_kernel, dim3(cdiv(n, TB)), dim3(TB), 0, s, (uint16_t*)p, n, pattern);
  return hipGetLastError();
}
hipError_t swap_copy(void* dst, const void* src, uint64_t bytes, int nblocks, hipStream_t s) {
  const long long n16 = (long long)(bytes / 16);
  if (n16) {
    long long want = (n16 + TB - 1) / TB;
    if (want > nblocks) want = nblocks;
    hipLaunchKernelGGL(swap_copy_kernel, dim3((unsigned)want), dim3(TB), 0, s, (uint4*)dst, (const uint4*)src, n16);
  }
  const int tail = (int)(bytes - (uint64_t)n16 * 16);
  if (tail) hipLaunchKernelGGL(swap_copy_tail_kernel, dim3(1), dim3(16), 0, s, (unsigned char*)dst + n16 * 16, (const unsigned char*)src + n16 * 16, tail);
  return hipGetLastError();
}
uint64_t swap_encoded_bytes(uint64_t numel) {
  return (uint64_t)enc_trailer_offset((long long)((numel + ENC_EL - 1) / ENC_EL)) + ENC_TRAILER;
}
hipError_t swap_encode_range(void* dst_host, const void* src, uint64_t numel, int64_t slot_begin, int64_t slot_end, void* stage, int w,
                             int nblocks, hipStream_t s) {
  if (numel % 8) return hipErrorInvalidValue;
  const long long nslots = (long long)((numel + ENC_EL - 1) / ENC_EL);
  if (slot_begin < 0 || slot_end > nslots || slot_begin > slot_end || (w & 15) || w < 0 || w > ENC_STRIDE) return hipErrorInvalidValue;
  const long long count = slot_end - slot_begin;
  if (count == 0) return hipSuccess;
  long long grid = count < nblocks ? count : nblocks;
  const long long per = (count + grid - 1) / grid;
  grid = (count + per - 1) / per;
  hipLaunchKernelGGL(swap_encode_kernel, dim3((unsigned)grid), dim3(TB), 0, s, (unsigned char*)dst_host, (const uint4*)src,
                     (long long)(numel / 8), nslots, (long long)slot_begin, (long long)slot_end, per, (unsigned char*)stage, stage ? w : 0);
  return hipGetLastError();
}
hipError_t swap_encode(void* dst_host, const void* src, uint64_t numel, int nblocks, hipStream_t s, bool trailer) {
  const long long nslots = (long long)((numel + ENC_EL - 1) / ENC_EL);
  const hipError_t e = swap_encode_range(dst_host, src, numel, 0, nslots, nullptr, 0, nblocks, s);
  if (e != hipSuccess) return e;
  if (trailer && nslots) hipLaunchKernelGGL(swap_trailer_kernel, dim3(1), dim3(TB), 0, s, (unsigned char*)dst_host, nslots);
  return hipGetLastError();
}
hipError_t swap_decode_range(void* dst, const void* src_host, uint64_t numel, int64_t slot_begin, int64_t slot_end, const void* stage, int w,
                             int nblocks, hipStream_t s) {
  if (numel % 8) return hipErrorInvalidValue;
  const long long nslots = (long long)((numel + ENC_EL - 1) / ENC_EL);
  if (slot_begin < 0 || slot_end > nslots || slot_begin > slot_end || (w & 15) || w < 0 || w > ENC_STRIDE) return hipErrorInvalidValue;
  const long long count = slot_end - slot_begin;
  if (count == 0) return hipSuccess;
  const long long grid = count < nblocks ? count : nblocks;
  hipLaunchKernelGGL(swap_decode_kernel, dim3((unsigned)grid), dim3(TB), 0, s, (uint4*)dst, (const unsigned char*)src_host,
                     (long long)(numel / 8), (long long)slot_begin, (long long)slot_end, (const unsigned char*)stage, stage ? w : 0);
  return hipGetLastError();
}
hipError_t swap_decode(void* dst, const void* src_host, uint64_t numel, int nblocks, hipStream_t s) {
  const long long nslots = (long long)((numel + ENC_EL - 1) / ENC_EL);
  return swap_decode_range(dst, src_host, numel, 0, nslots, nullptr, 0, nblocks, s);
}
uint64_t swap_slot_stride() { return ENC_STRIDE; }
uint64_t swap_slot_elements() { return ENC_EL; }
// From the count region of a finished encode: bytes of all slots (as swap_encoded_counted_bytes); the bytes a staged
// transfer of width w_used moved over the link (every slot its first w_used bytes, longer slots their tails as well;
// w_used 0: the slots' own bytes); and the width for the next transfer of a tensor like this one: the smallest multiple
// of 64 bytes that holds 95 % of the slots whole.
uint64_t swap_slot_statistics(const void* host, uint64_t numel, int w_used, int* w_next, uint64_t* link_bytes) {
  const long long nslots = (long long)((numel + ENC_EL - 1) / ENC_EL);
  const uint32_t* c = reinterpret_cast<const uint32_t*>(static_cast<const unsigned char*>(host) + enc_counts_offset(nslots));
  constexpr int BINS = ENC_STRIDE / 16 + 1;
  long long hist[BINS] = {0};
  uint64_t total = 0;
  for (long long i = 0; i < nslots; ++i) {
    int vb = (int)(c[i] >> 16);
    if (vb > 2 * ENC_EL) vb = 2 * ENC_EL;
    const int bytes = ENC_VAL + (vb + 15) / 16 * 16;
    total += (uint64_t)bytes;
    ++hist[bytes / 16];
  }
  long long seen = 0;
  int w = ENC_STRIDE;
  for (int b = 0; b < BINS; ++b) {
    seen += hist[b];
    if (seen * 100 >= nslots * 95) { w = b * 16; break; }
  }
  w = (w + 63) / 64 * 64;
  if (w > ENC_STRIDE) w = ENC_STRIDE;
  uint64_t link = 0;
  for (int b = 0; b < BINS; ++b) link += (uint64_t)hist[b] * (uint64_t)(b * 16 > w_used ? b * 16 : w_used);
  if (w_next) *w_next = w;
  if (link_bytes) *link_bytes = link;
  return total;
}
// The trailer's value recomputed on the host from the count region of a finished encode.
uint64_t swap_encoded_counted_bytes(const void* host, uint64_t numel) {
  const long long nslots = (long long)((numel + ENC_EL - 1) / ENC_EL);
  const uint32_t* c = reinterpret_cast<const uint32_t*>(static_cast<const unsigned char*>(host) + enc_counts_offset(nslots));
  uint64_t total = 0;
  for (long long i = 0; i < nslots; ++i) total += ENC_VAL + (uint64_t)(((c[i] >> 16) + 15) / 16 * 16);
  return total;
}
uint64_t swap_encoded_moved_bytes(const void* host, uint64_t numel) {
  const long long nslots = (long long)((numel + ENC_EL - 1) / ENC_EL);
  return *reinterpret_cast<const uint64_t*>(static_cast<const unsigned char*>(host) + enc_trailer_offset(nslots));
}
hipError_t sgd_update(int64_t numel, bool f32, const void* p, const float* g, float lr, void* out, hipStream_t s) {
  if (numel == 0) return hipSuccess;
  if (f32) hipLaunchKernelGGL(sgd_f32_kernel, dim3(cdiv(numel, TB)), dim3(TB), 0, s, (const float*)p, g, lr, (long long)numel, (float*)out);
  else hipLaunchKernelGGL(sgd_bf16_kernel, dim3(cdiv(numel, TB)), dim3(TB), 0, s, (const uint16_t*)p, g, lr, (long long)numel, (uint16_t*)out);
  return hipGetLastError();
}
int sgd_batch_blocks(int64_t numel) { return (int)cdiv(numel, TB); }
hipError_t sgd_update_batch(const SgdBatch& b, hipStream_t s) {
  if (b.count <= 0 || b.first[b.count] <= 0) return hipSuccess;
  hipLaunchKernelGGL(sgd_multi_kernel, dim3(b.first[b.count]), dim3(TB), 0, s, b);
  return hipGetLastError();
}
static bool pool2_fast(const ConvGeom& g) {
  if ((g.c & 7) != 0) return false;
  for (int i = 0; i < 3; ++i) {
    if (g.pad[i] != 0 || g.filt[i] != g.stride[i] || (g.filt[i] != 1 && g.filt[i] != 2)) return false;
    if (g.in_sp[i] != g.out_sp[i] * g.filt[i]) return false;      // every input element lies in exactly one window
  }
  return true;
}
static bool pool3s2_fast(const ConvGeom& g) {
  if ((g.c & 7) != 0 || g.in_sp[0] != 1 || g.filt[0] != 1) return false;
  for (int i = 1; i < 3; ++i)
    if (g.filt[i] != 3 || g.stride[i] != 2 || g.pad[i] != 1) return false;
  return g.in_rows() * (g.c / 8) < 0x7fffffffLL * 64;
}
hipError_t maxpool_fwd(const ConvGeom& g, const void* x, void* y, hipStream_t s) {
  if (pool3s2_fast(g) && (((uintptr_t)x | (uintptr_t)y) & 15) == 0) {
    const long long total = g.out_rows() * (g.c / 8);
    hipLaunchKernelGGL(maxpool3s2_fwd_kernel, dim3(cdiv(total, TB)), dim3(TB), 0, s, pool_params(g), (const uint4*)x, (uint4*)y, total);
    return hipGetLastError();
  }
  if (pool2_fast(g)) {
    const long long total = g.out_rows() * (g.c / 8);
    hipLaunchKernelGGL(maxpool2_kernel<0>, dim3(cdiv(total, TB)), dim3(TB), 0, s, pool_params(g), (const uint4*)x, (const uint4*)nullptr, 0, (uint4*)y, total);
    return hipGetLastError();
  }
  const long long total = g.out_rows() * g.c;
  hipLaunchKernelGGL(maxpool_fwd_kernel, dim3(cdiv(total, TB)), dim3(TB), 0, s, pool_params(g), (const uint16_t*)x, (uint16_t*)y, total);
  return hipGetLastError();
}
hipError_t maxpool_bwd(const ConvGeom& g, const void* dy, const void* x, int mask_relu, void* dx, hipStream_t s) {
  if (pool3s2_fast(g) && (((uintptr_t)dy | (uintptr_t)x | (uintptr_t)dx) & 15) == 0) {
    const int th = (g.in_sp[1] + P3_IN - 1) / P3_IN, tw = (g.in_sp[2] + P3_IN - 1) / P3_IN;
    const long long blocks = (long long)g.n * th * tw;
    const int cgroups = (g.c / 8 + 7) / 8;
    if (blocks < 0x7fffffffLL && cgroups < 65536) {
      hipLaunchKernelGGL(maxpool3s2_bwd_kernel, dim3((unsigned)blocks, (unsigned)cgroups), dim3(TB), 0, s, pool_params(g), (const uint4*)dy,
                         (const uint4*)x, mask_relu, (uint4*)dx, th, tw);
      return hipGetLastError();
    }
  }
  if (pool2_fast(g)) {
    const long long total = g.out_rows() * (g.c / 8);
    hipLaunchKernelGGL(maxpool2_kernel<1>, dim3(cdiv(total, TB)), dim3(TB), 0, s, pool_params(g), (const uint4*)x, (const uint4*)dy, mask_relu, (uint4*)dx, total);
    return hipGetLastError();
  }
  if ((g.c & 7) == 0 && (((uintptr_t)dy | (uintptr_t)x | (uintptr_t)dx) & 15) == 0) {
    const long long total8 = g.in_rows() * (g.c / 8);
    hipLaunchKernelGGL(maxpool_bwd_vec_kernel, dim3(cdiv(total8, TB)), dim3(TB), 0, s, pool_params(g), (const uint4*)dy, (const uint4*)x,
                       mask_relu, (uint4*)dx, total8);
    return hipGetLastError();
  }
  const long long total = g.in_rows() * g.c;
  hipLaunchKernelGGL(maxpool_bwd_kernel, dim3(cdiv(total, TB)), dim3(TB), 0, s, pool_params(g), (const uint16_t*)dy, (const uint16_t*)x,
                     mask_relu, (uint16_t*)dx, total);
  return hipGetLastError();
}
hipError_t gap_fwd(int64_t n, int64_t positions, int c, const void* x, void* y, hipStream_t s) {
  hipLaunchKernelGGL(gap_fwd_kernel, dim3(cdiv(n * c, TB)), dim3(TB), 0, s, (const uint16_t*)x, (uint16_t*)y, (long long)n, (long long)positions, c);
  return hipGetLastError();
}
hipError_t gap_bwd(int64_t n, int64_t positions, int c, const void* dy, const void* mask, void* dx, hipStream_t s) {
  const long long total = n * positions * c;
  hipLaunchKernelGGL(gap_bwd_kernel, dim3(cdiv(total, TB)), dim3(TB), 0, s, (const uint16_t*)dy, (const uint16_t*)mask, (uint16_t*)dx, total,
                     (long long)positions, c);
  return hipGetLastError();
}
hipError_t copy_channels(int64_t rows, const void* src, int src_c, int src_begin, void* dst, int dst_c, int dst_begin, int count,
                         const void* mask, hipStream_t s) {
  if (!mask && ((src_c | src_begin | dst_c | dst_begin | count) & 7) == 0) {
    const long long total = rows * (count / 8);
    hipLaunchKernelGGL(copy_channels_vec_kernel, dim3(cdiv(total, TB)), dim3(TB), 0, s, (const uint4*)src, src_c / 8, src_begin / 8,
                       (uint4*)dst, dst_c / 8, dst_begin / 8, count / 8, total);
  } else {
    const long long total = rows * count;
    hipLaunchKernelGGL(copy_channels_kernel, dim3(cdiv(total, TB)), dim3(TB), 0, s, (const uint16_t*)src, src_c, src_begin, (uint16_t*)dst,
                       dst_c, dst_begin, count, (const uint16_t*)mask, total);
  }
  return hipGetLastError();
}

}  // namespace lms
