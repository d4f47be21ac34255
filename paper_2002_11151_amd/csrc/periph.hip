// Digital peripheral operations of a crossbar-based network (Sec. IV-B: ReLU, batch normalisation and
// pooling are computed in the digital domain and are not touched by the crossbar non-idealities), plus
// the loss and the plain SGD step of the digital parameters, so that a whole training step runs on the
// GPU.  Activations are NHWC float tensors; sums that decide statistics are accumulated in double
// precision in a fixed order (deterministic).  All of it is HBM-bound elementwise or reduction work.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "xbar.h"

namespace {

inline bool aligned16(const void* p) { return p != nullptr && (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
inline unsigned blocks_for(size_t n) { return (unsigned)((n + 255) / 256); }
constexpr int kStatRows = 512;    // rows per block of the per-channel reductions

__global__ __launch_bounds__(256) void relu_fwd_kernel(const float* x, float* y, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) y[i] = x[i] > 0.0f ? x[i] : 0.0f;
}

__global__ __launch_bounds__(256) void relu_bwd_kernel(const float* y, const float* dy, float* dx, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) dx[i] = y[i] > 0.0f ? dy[i] : 0.0f;
}

// Logistic function; the exponential is taken in double precision so that the float result is the
// correctly rounded one in all but rare cases.
__global__ __launch_bounds__(256) void sigmoid_fwd_kernel(const float* x, float* y, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) y[i] = (float)(1.0 / (1.0 + ::exp(-(double)x[i])));
}

__global__ __launch_bounds__(256) void sigmoid_bwd_kernel(const float* y, const float* dy, float* dx, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) {
    const double s = (double)y[i];
    dx[i] = (float)((double)dy[i] * s * (1.0 - s));
  }
}

__global__ __launch_bounds__(256) void add_kernel(const float* a, const float* b, float* y, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) y[i] = a[i] + b[i];
}

__global__ __launch_bounds__(256) void sgd_kernel(float* p, const float* g, size_t n, float lr) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] -= lr * g[i];
}

// Per-channel sums over a block of rows: part[chunk][channel][2] = (sum x, sum x^2), or with BWD
// (sum dy, sum dy xhat).  CT = channels per strip (a power of two, at most 64); the 256 threads are
// 256 / CT row groups x CT channels, so narrow layers still use every lane.
template <bool BWD, int CT>
__global__ __launch_bounds__(256) void bn_partial_kernel(const float* x, const float* dy, const float* mean,
                                                         const float* invstd, double* part, size_t rows, int C) {
  constexpr int G = 256 / CT;
  __shared__ double red[2][G][CT];
  const int cl = threadIdx.x % CT, grp = threadIdx.x / CT;
  const int c = blockIdx.y * CT + cl;
  const size_t r0 = (size_t)blockIdx.x * kStatRows;
  const size_t r1 = r0 + kStatRows < rows ? r0 + kStatRows : rows;
  double s0 = 0.0, s1 = 0.0;
  if (c < C) {
    const double mu = BWD ? (double)mean[c] : 0.0, is = BWD ? (double)invstd[c] : 0.0;
#pragma unroll 4
    for (size_t r = r0 + grp; r < r1; r += G) {
      const double v = (double)x[r * C + c];
      if (BWD) {
        const double g = (double)dy[r * C + c];
        s0 += g;                       // sum dy
        s1 += g * ((v - mu) * is);     // sum dy xhat
      } else {
        s0 += v;
        s1 += v * v;
      }
    }
  }
  red[0][grp][cl] = s0;
  red[1][grp][cl] = s1;
  __syncthreads();
  if (grp == 0 && c < C) {
    double t0 = 0.0, t1 = 0.0;
    for (int g = 0; g < G; ++g) {      // fixed order
      t0 += red[0][g][cl];
      t1 += red[1][g][cl];
    }
    double* out = part + ((size_t)blockIdx.x * C + c) * 2;
    out[0] = t0;
    out[1] = t1;
  }
}

// One wave per channel adds the chunk sums: lane l takes chunks l, l + 64, ..., then a fixed
// butterfly over the lanes.
__device__ __forceinline__ void bn_chunk_sums(const double* part, int chunks, int C, int c, double& s0, double& s1) {
  const int lane = threadIdx.x & 63;
  s0 = s1 = 0.0;
  for (int k = lane; k < chunks; k += 64) {
    s0 += part[((size_t)k * C + c) * 2];
    s1 += part[((size_t)k * C + c) * 2 + 1];
  }
#pragma unroll
  for (int d = 32; d; d >>= 1) {
    s0 += __shfl_xor(s0, d, 64);
    s1 += __shfl_xor(s1, d, 64);
  }
}

__global__ __launch_bounds__(256) void bn_finalize_fwd_kernel(const double* part, int chunks, int C, size_t rows,
                                                              float eps, float* mean, float* invstd) {
  const int c = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (c >= C) return;                                 // whole waves leave together
  double s0, s1;
  bn_chunk_sums(part, chunks, C, c, s0, s1);
  if ((threadIdx.x & 63) != 0) return;
  const double mu = s0 / (double)rows;
  double var = s1 / (double)rows - mu * mu;        // biased variance of the batch
  if (var < 0.0) var = 0.0;
  mean[c] = (float)mu;
  invstd[c] = (float)(1.0 / ::sqrt(var + (double)eps));
}

__global__ __launch_bounds__(256) void bn_finalize_bwd_kernel(const double* part, int chunks, int C, float* dgamma,
                                                              float* dbeta) {
  const int c = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (c >= C) return;
  double s0, s1;
  bn_chunk_sums(part, chunks, C, c, s0, s1);
  if ((threadIdx.x & 63) != 0) return;
  dbeta[c] = (float)s0;
  dgamma[c] = (float)s1;
}

__global__ __launch_bounds__(256) void bn_apply_fwd_kernel(const float* x, const float* gamma, const float* beta,
                                                           const float* mean, const float* invstd, float* y, size_t n,
                                                           int C) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const int c = (int)(i % C);
  y[i] = (float)((double)gamma[c] * (((double)x[i] - (double)mean[c]) * (double)invstd[c]) + (double)beta[c]);
}

__global__ __launch_bounds__(256) void bn_apply_bwd_kernel(const float* x, const float* dy, const float* gamma,
                                                           const float* mean, const float* invstd, const float* dgamma,
                                                           const float* dbeta, float* dx, size_t n, int C, double inv_rows) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const int c = (int)(i % C);
  const double xhat = ((double)x[i] - (double)mean[c]) * (double)invstd[c];
  dx[i] = (float)((double)gamma[c] * (double)invstd[c] *
                  ((double)dy[i] - (double)dbeta[c] * inv_rows - xhat * (double)dgamma[c] * inv_rows));
}

__global__ __launch_bounds__(256) void avgpool_fwd_kernel(const float* x, float* y, int batch, int positions, int C) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)batch * C) return;
  const int c = (int)(i % C);
  const size_t b = i / C;
  double s = 0.0;
  for (int p = 0; p < positions; ++p) s += (double)x[(b * positions + p) * C + c];
  y[i] = (float)(s / (double)positions);
}

__global__ __launch_bounds__(256) void avgpool_bwd_kernel(const float* dy, float* dx, int batch, int positions, int C) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)batch * positions * C) return;
  const int c = (int)(i % C);
  const size_t b = i / ((size_t)positions * C);
  dx[i] = dy[b * C + c] / (float)positions;
}

struct PoolGeom {
  int B, H, W, C, k, stride, pad, OH, OW;
};

__global__ __launch_bounds__(256) void maxpool_fwd_kernel(const float* x, float* y, int32_t* arg, PoolGeom g) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)g.B * g.OH * g.OW * g.C) return;
  const int c = (int)(i % g.C);
  size_t u = i / g.C;
  const int ow = (int)(u % g.OW);
  u /= g.OW;
  const int oh = (int)(u % g.OH), b = (int)(u / g.OH);
  float best = -INFINITY;
  int32_t best_at = -1;
  for (int kh = 0; kh < g.k; ++kh) {
    const int ih = oh * g.stride - g.pad + kh;
    if (ih < 0 || ih >= g.H) continue;
    for (int kw = 0; kw < g.k; ++kw) {
      const int iw = ow * g.stride - g.pad + kw;
      if (iw < 0 || iw >= g.W) continue;
      const int32_t at = ih * g.W + iw;                      // position inside the image; first maximum wins
      const float v = x[(((size_t)b * g.H + ih) * g.W + iw) * g.C + c];
      if (v > best) { best = v; best_at = at; }
    }
  }
  y[i] = best;
  arg[i] = best_at;
}

// Gather form of the backward pass: an input pixel adds the errors of the windows that chose it.
__global__ __launch_bounds__(256) void maxpool_bwd_kernel(const float* dy, const int32_t* arg, float* dx, PoolGeom g) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)g.B * g.H * g.W * g.C) return;
  const int c = (int)(i % g.C);
  size_t u = i / g.C;
  const int iw = (int)(u % g.W);
  u /= g.W;
  const int ih = (int)(u % g.H), b = (int)(u / g.H);
  const int32_t me = ih * g.W + iw;
  float s = 0.0f;
  for (int kh = 0; kh < g.k; ++kh) {
    const int oy = ih + g.pad - kh;
    if (oy < 0 || oy % g.stride) continue;
    const int oh = oy / g.stride;
    if (oh >= g.OH) continue;
    for (int kw = 0; kw < g.k; ++kw) {
      const int ox = iw + g.pad - kw;
      if (ox < 0 || ox % g.stride) continue;
      const int ow = ox / g.stride;
      if (ow >= g.OW) continue;
      const size_t o = (((size_t)b * g.OH + oh) * g.OW + ow) * g.C + c;
      if (arg[o] == me) s += dy[o];
    }
  }
  dx[i] = s;
}

// One wave per sample: loss = log(sum exp(z - max)) - (z_label - max), dlogits = scale (softmax - onehot).
__global__ __launch_bounds__(64) void softmax_xent_kernel(const float* logits, const int32_t* labels, float* loss,
                                                          float* dlogits, int classes, float scale) {
  const int b = blockIdx.x, lane = threadIdx.x;
  const float* z = logits + (size_t)b * classes;
  float mx = -INFINITY;
  for (int j = lane; j < classes; j += 64) mx = fmaxf(mx, z[j]);
  for (int d = 32; d; d >>= 1) mx = fmaxf(mx, __shfl_xor(mx, d, 64));
  double s = 0.0;
  for (int j = lane; j < classes; j += 64) s += ::exp((double)z[j] - (double)mx);
  for (int d = 32; d; d >>= 1) s += __shfl_xor(s, d, 64);
  const int label = labels[b];
  const bool known = label >= 0 && label < classes;          // an unknown label gives a NaN loss, no target
  if (lane == 0) loss[b] = known ? (float)(::log(s) - ((double)z[label] - (double)mx)) : NAN;
  for (int j = lane; j < classes; j += 64) {
    const double pj = ::exp((double)z[j] - (double)mx) / s;
    dlogits[(size_t)b * classes + j] = (float)((double)scale * (pj - (j == label ? 1.0 : 0.0)));
  }
}

// Parameter-free residual shortcut across a stage boundary: spatial subsampling by `stride` and zero
// padding of the new channels, half before and half behind the old ones.
struct ShortcutGeom {
  int B, H, W, C, stride, OH, OW, OC, lo;
};

__global__ __launch_bounds__(256) void shortcut_fwd_kernel(const float* x, float* y, ShortcutGeom g) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)g.B * g.OH * g.OW * g.OC) return;
  const int oc = (int)(i % g.OC);
  size_t u = i / g.OC;
  const int ow = (int)(u % g.OW);
  u /= g.OW;
  const int oh = (int)(u % g.OH), b = (int)(u / g.OH);
  const int c = oc - g.lo;
  y[i] = (c >= 0 && c < g.C) ? x[(((size_t)b * g.H + oh * g.stride) * g.W + ow * g.stride) * g.C + c] : 0.0f;
}

__global__ __launch_bounds__(256) void shortcut_bwd_kernel(const float* dy, float* dx, ShortcutGeom g) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)g.B * g.H * g.W * g.C) return;
  const int c = (int)(i % g.C);
  size_t u = i / g.C;
  const int iw = (int)(u % g.W);
  u /= g.W;
  const int ih = (int)(u % g.H), b = (int)(u / g.H);
  const bool kept = ih % g.stride == 0 && iw % g.stride == 0 && ih / g.stride < g.OH && iw / g.stride < g.OW;
  dx[i] = kept ? dy[(((size_t)b * g.OH + ih / g.stride) * g.OW + iw / g.stride) * g.OC + c + g.lo] : 0.0f;
}

// max |x|: per-block maxima, then one block over them.  |x| is compared as an unsigned integer (the
// order of non-negative floats); a NaN input gives a NaN-patterned result.
__global__ __launch_bounds__(256) void absmax_kernel(const float* x, size_t n, uint32_t* part) {
  __shared__ uint32_t red[4];
  uint32_t m = 0;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    const uint32_t v = __float_as_uint(x[i]) & 0x7FFFFFFFu;
    m = v > m ? v : m;
  }
  for (int d = 32; d; d >>= 1) {
    const uint32_t o = (uint32_t)__shfl_xor((int)m, d, 64);
    m = o > m ? o : m;
  }
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) m = red[w] > m ? red[w] : m;
    part[blockIdx.x] = m;
  }
}

template <bool BWD>
void launch_bn_partial(const float* x, const float* dy, const float* mean, const float* invstd, double* part, size_t rows,
                       int channels, int chunks, hipStream_t st) {
  if (channels <= 16)
    hipLaunchKernelGGL((bn_partial_kernel<BWD, 16>), dim3((unsigned)chunks, (unsigned)((channels + 15) / 16)), dim3(256), 0,
                       st, x, dy, mean, invstd, part, rows, channels);
  else if (channels <= 32)
    hipLaunchKernelGGL((bn_partial_kernel<BWD, 32>), dim3((unsigned)chunks, 1u), dim3(256), 0, st, x, dy, mean, invstd, part,
                       rows, channels);
  else
    hipLaunchKernelGGL((bn_partial_kernel<BWD, 64>), dim3((unsigned)chunks, (unsigned)((channels + 63) / 64)), dim3(256), 0,
                       st, x, dy, mean, invstd, part, rows, channels);
}

inline int launched() { return hipGetLastError() == hipSuccess ? XBAR_OK : XBAR_EHIP; }

}  // namespace

extern "C" {

int xbar_relu_fwd(const float* x, float* y, size_t n, void* hip_stream) {
  if (n == 0) return XBAR_ESHAPE;
  if (!aligned16(x) || !aligned16(y)) return XBAR_EALIGN;
  hipLaunchKernelGGL(relu_fwd_kernel, dim3(blocks_for(n)), dim3(256), 0, reinterpret_cast<hipStream_t>(hip_stream), x, y, n);
  return launched();
}

int xbar_relu_bwd(const float* y, const float* dy, float* dx, size_t n, void* hip_stream) {
  if (n == 0) return XBAR_ESHAPE;
  if (!aligned16(y) || !aligned16(dy) || !aligned16(dx)) return XBAR_EALIGN;
  hipLaunchKernelGGL(relu_bwd_kernel, dim3(blocks_for(n)), dim3(256), 0, reinterpret_cast<hipStream_t>(hip_stream), y, dy,
                     dx, n);
  return launched();
}

int xbar_sigmoid_fwd(const float* x, float* y, size_t n, void* hip_stream) {
  if (n == 0) return XBAR_ESHAPE;
  if (!aligned16(x) || !aligned16(y)) return XBAR_EALIGN;
  hipLaunchKernelGGL(sigmoid_fwd_kernel, dim3(blocks_for(n)), dim3(256), 0, reinterpret_cast<hipStream_t>(hip_stream), x, y, n);
  return launched();
}

int xbar_sigmoid_bwd(const float* y, const float* dy, float* dx, size_t n, void* hip_stream) {
  if (n == 0) return XBAR_ESHAPE;
  if (!aligned16(y) || !aligned16(dy) || !aligned16(dx)) return XBAR_EALIGN;
  hipLaunchKernelGGL(sigmoid_bwd_kernel, dim3(blocks_for(n)), dim3(256), 0, reinterpret_cast<hipStream_t>(hip_stream), y, dy,
                     dx, n);
  return launched();
}

int xbar_add(const float* a, const float* b, float* y, size_t n, void* hip_stream) {
  if (n == 0) return XBAR_ESHAPE;
  if (!aligned16(a) || !aligned16(b) || !aligned16(y)) return XBAR_EALIGN;
  hipLaunchKernelGGL(add_kernel, dim3(blocks_for(n)), dim3(256), 0, reinterpret_cast<hipStream_t>(hip_stream), a, b, y, n);
  return launched();
}

int xbar_sgd(float* p, const float* g, size_t n, float lr, void* hip_stream) {
  if (n == 0) return XBAR_ESHAPE;
  if (!aligned16(p) || !aligned16(g)) return XBAR_EALIGN;
  if (!std::isfinite(lr)) return XBAR_EINVAL;
  hipLaunchKernelGGL(sgd_kernel, dim3(blocks_for(n)), dim3(256), 0, reinterpret_cast<hipStream_t>(hip_stream), p, g, n, lr);
  return launched();
}

size_t xbar_bn_workspace_bytes(size_t rows, int channels) {
  if (rows == 0 || channels <= 0) return 0;
  const size_t chunks = (rows + kStatRows - 1) / kStatRows;
  return align256(chunks * (size_t)channels * 2 * sizeof(double));
}

int xbar_bn_fwd(const float* x, const float* gamma, const float* beta, float* y, float* mean, float* invstd, size_t rows,
                int channels, float eps, void* ws, size_t ws_bytes, void* hip_stream) {
  if (rows == 0 || channels <= 0 || rows > ((size_t)1 << 31)) return XBAR_ESHAPE;
  if (!aligned16(x) || !aligned16(gamma) || !aligned16(beta) || !aligned16(y) || !aligned16(mean) || !aligned16(invstd) ||
      !aligned16(ws))
    return XBAR_EALIGN;
  if (!(eps >= 0.0f) || !std::isfinite(eps)) return XBAR_EINVAL;
  if (ws_bytes < xbar_bn_workspace_bytes(rows, channels)) return XBAR_EWORKSPACE;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  const int chunks = (int)((rows + kStatRows - 1) / kStatRows);
  double* part = reinterpret_cast<double*>(ws);
  launch_bn_partial<false>(x, nullptr, nullptr, nullptr, part, rows, channels, chunks, st);
  if (launched()) return XBAR_EHIP;
  hipLaunchKernelGGL(bn_finalize_fwd_kernel, dim3((unsigned)((channels + 3) / 4)), dim3(256), 0, st, part, chunks, channels,
                     rows, eps, mean, invstd);
  if (launched()) return XBAR_EHIP;
  const size_t n = rows * (size_t)channels;
  hipLaunchKernelGGL(bn_apply_fwd_kernel, dim3(blocks_for(n)), dim3(256), 0, st, x, gamma, beta, mean, invstd, y, n, channels);
  return launched();
}

int xbar_bn_bwd(const float* x, const float* dy, const float* gamma, const float* mean, const float* invstd, float* dx,
                float* dgamma, float* dbeta, size_t rows, int channels, void* ws, size_t ws_bytes, void* hip_stream) {
  if (rows == 0 || channels <= 0 || rows > ((size_t)1 << 31)) return XBAR_ESHAPE;
  if (!aligned16(x) || !aligned16(dy) || !aligned16(gamma) || !aligned16(mean) || !aligned16(invstd) || !aligned16(dx) ||
      !aligned16(dgamma) || !aligned16(dbeta) || !aligned16(ws))
    return XBAR_EALIGN;
  if (ws_bytes < xbar_bn_workspace_bytes(rows, channels)) return XBAR_EWORKSPACE;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  const int chunks = (int)((rows + kStatRows - 1) / kStatRows);
  double* part = reinterpret_cast<double*>(ws);
  launch_bn_partial<true>(x, dy, mean, invstd, part, rows, channels, chunks, st);
  if (launched()) return XBAR_EHIP;
  hipLaunchKernelGGL(bn_finalize_bwd_kernel, dim3((unsigned)((channels + 3) / 4)), dim3(256), 0, st, part, chunks, channels,
                     dgamma, dbeta);
  if (launched()) return XBAR_EHIP;
  const size_t n = rows * (size_t)channels;
  hipLaunchKernelGGL(bn_apply_bwd_kernel, dim3(blocks_for(n)), dim3(256), 0, st, x, dy, gamma, mean, invstd, dgamma, dbeta,
                     dx, n, channels, 1.0 / (double)rows);
  return launched();
}

int xbar_avgpool_fwd(const float* x, float* y, int batch, int positions, int channels, void* hip_stream) {
  if (batch <= 0 || positions <= 0 || channels <= 0) return XBAR_ESHAPE;
  if (!aligned16(x) || !aligned16(y)) return XBAR_EALIGN;
  hipLaunchKernelGGL(avgpool_fwd_kernel, dim3(blocks_for((size_t)batch * channels)), dim3(256), 0,
                     reinterpret_cast<hipStream_t>(hip_stream), x, y, batch, positions, channels);
  return launched();
}

int xbar_avgpool_bwd(const float* dy, float* dx, int batch, int positions, int channels, void* hip_stream) {
  if (batch <= 0 || positions <= 0 || channels <= 0) return XBAR_ESHAPE;
  if (!aligned16(dy) || !aligned16(dx)) return XBAR_EALIGN;
  hipLaunchKernelGGL(avgpool_bwd_kernel, dim3(blocks_for((size_t)batch * positions * channels)), dim3(256), 0,
                     reinterpret_cast<hipStream_t>(hip_stream), dy, dx, batch, positions, channels);
  return launched();
}

static int pool_geom(const xbar_conv_geom* q, PoolGeom* g) {
  if (!q) return XBAR_EINVAL;
  if (q->batch <= 0 || q->in_h <= 0 || q->in_w <= 0 || q->in_c <= 0 || q->k_h <= 0 || q->k_h != q->k_w || q->stride <= 0 ||
      q->pad < 0 || 2 * q->pad > q->k_h || q->in_h + 2 * q->pad < q->k_h || q->in_w + 2 * q->pad < q->k_w)
    return XBAR_ESHAPE;
  if (q->out_h != (q->in_h + 2 * q->pad - q->k_h) / q->stride + 1 ||
      q->out_w != (q->in_w + 2 * q->pad - q->k_w) / q->stride + 1)
    return XBAR_ESHAPE;
  if ((long long)q->in_h * q->in_w >= (1ll << 31)) return XBAR_ESHAPE;
  g->B = q->batch; g->H = q->in_h; g->W = q->in_w; g->C = q->in_c; g->k = q->k_h; g->stride = q->stride; g->pad = q->pad;
  g->OH = q->out_h; g->OW = q->out_w;
  return XBAR_OK;
}

int xbar_maxpool_fwd(const float* x, float* y, int32_t* argmax, const xbar_conv_geom* geom, void* hip_stream) {
  PoolGeom g;
  const int rc = pool_geom(geom, &g);
  if (rc) return rc;
  if (!aligned16(x) || !aligned16(y) || !aligned16(argmax)) return XBAR_EALIGN;
  hipLaunchKernelGGL(maxpool_fwd_kernel, dim3(blocks_for((size_t)g.B * g.OH * g.OW * g.C)), dim3(256), 0,
                     reinterpret_cast<hipStream_t>(hip_stream), x, y, argmax, g);
  return launched();
}

int xbar_maxpool_bwd(const float* dy, const int32_t* argmax, float* dx, const xbar_conv_geom* geom, void* hip_stream) {
  PoolGeom g;
  const int rc = pool_geom(geom, &g);
  if (rc) return rc;
  if (!aligned16(dy) || !aligned16(dx) || !aligned16(argmax)) return XBAR_EALIGN;
  hipLaunchKernelGGL(maxpool_bwd_kernel, dim3(blocks_for((size_t)g.B * g.H * g.W * g.C)), dim3(256), 0,
                     reinterpret_cast<hipStream_t>(hip_stream), dy, argmax, dx, g);
  return launched();
}

static int shortcut_geom(int batch, int h, int w, int channels, int stride, int out_channels, ShortcutGeom* g) {
  if (batch <= 0 || h <= 0 || w <= 0 || channels <= 0 || stride <= 0 || out_channels < channels) return XBAR_ESHAPE;
  g->B = batch; g->H = h; g->W = w; g->C = channels; g->stride = stride;
  g->OH = (h + stride - 1) / stride; g->OW = (w + stride - 1) / stride; g->OC = out_channels;
  g->lo = (out_channels - channels) / 2;
  return XBAR_OK;
}

int xbar_shortcut_fwd(const float* x, float* y, int batch, int h, int w, int channels, int stride, int out_channels,
                      void* hip_stream) {
  ShortcutGeom g;
  const int rc = shortcut_geom(batch, h, w, channels, stride, out_channels, &g);
  if (rc) return rc;
  if (!aligned16(x) || !aligned16(y)) return XBAR_EALIGN;
  hipLaunchKernelGGL(shortcut_fwd_kernel, dim3(blocks_for((size_t)g.B * g.OH * g.OW * g.OC)), dim3(256), 0,
                     reinterpret_cast<hipStream_t>(hip_stream), x, y, g);
  return launched();
}

int xbar_shortcut_bwd(const float* dy, float* dx, int batch, int h, int w, int channels, int stride, int out_channels,
                      void* hip_stream) {
  ShortcutGeom g;
  const int rc = shortcut_geom(batch, h, w, channels, stride, out_channels, &g);
  if (rc) return rc;
  if (!aligned16(dy) || !aligned16(dx)) return XBAR_EALIGN;
  hipLaunchKernelGGL(shortcut_bwd_kernel, dim3(blocks_for((size_t)g.B * g.H * g.W * g.C)), dim3(256), 0,
                     reinterpret_cast<hipStream_t>(hip_stream), dy, dx, g);
  return launched();
}

int xbar_absmax(const float* x, size_t n, float* result, void* ws, size_t ws_bytes, void* hip_stream) {
  if (n == 0) return XBAR_ESHAPE;
  if (!aligned16(x) || !aligned16(result) || !aligned16(ws)) return XBAR_EALIGN;
  if (ws_bytes < 1024 * sizeof(uint32_t)) return XBAR_EWORKSPACE;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  const unsigned blocks = (unsigned)((n + 255) / 256 < 1024 ? (n + 255) / 256 : 1024);
  uint32_t* part = reinterpret_cast<uint32_t*>(ws);
  hipLaunchKernelGGL(absmax_kernel, dim3(blocks), dim3(256), 0, st, x, n, part);
  if (launched()) return XBAR_EHIP;
  // the partial maxima are bit patterns of non-negative floats: the same kernel reduces them once more
  hipLaunchKernelGGL(absmax_kernel, dim3(1), dim3(256), 0, st, reinterpret_cast<const float*>(part), (size_t)blocks,
                     reinterpret_cast<uint32_t*>(result));
  return launched();
}

int xbar_softmax_xent(const float* logits, const int32_t* labels, float* loss, float* dlogits, int batch, int classes,
                      float scale, void* hip_stream) {
  if (batch <= 0 || classes <= 0) return XBAR_ESHAPE;
  if (!aligned16(logits) || !aligned16(labels) || !aligned16(loss) || !aligned16(dlogits)) return XBAR_EALIGN;
  if (!std::isfinite(scale)) return XBAR_EINVAL;
  hipLaunchKernelGGL(softmax_xent_kernel, dim3((unsigned)batch), dim3(64), 0, reinterpret_cast<hipStream_t>(hip_stream),
                     logits, labels, loss, dlogits, classes, scale);
  return launched();
}

}  // extern "C"
