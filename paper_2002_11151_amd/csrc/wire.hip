// All-paths analytical wire model (Sec. IV-D: more paths than the shortest one): kernels and their launch.
#include "xbar_common.h"

using namespace xbar_detail;

namespace {

// ---------------------------------------------------------------------------------------------
// wire model with all first-order paths (Sec. IV-D: more paths than the shortest one)
//   a_ij = sum_j' G_ij' (r_source + (min(j,j') + 1) r_row)      drops on the row wire
//   b_ij = sum_i' G_i'j ((R - max(i,i')) r_col + r_sense)       rises on the column wire
//   G_ni = G / (1 + a + b),   plane = (G_ni+ - G_ni-) / dG
// Both sums split into a prefix and a suffix part, so one scan along the row and two walks along
// the column replace the O(R + C) sum per device.  Scratch: A[S_w][2][K][N] (double) and the quantised
// weights q[K][N]; the row kernel writes a into A, the column kernel adds b and leaves the plane
// value in the slot of array 0 (with one converter per array: each array's value in its own slot).
// ---------------------------------------------------------------------------------------------
struct WireArgs {
  const float* W;
  double* A;         // [S_w][2][K][N]
  int32_t* q;        // [K][N] signed quantised weights
  int K, N, R, C, S_w, slice_bits, weight_bits, tiles_c;
  uint32_t flags;
  double g_min, dg, var_sigma, r_row, r_col, r_source, r_sense;
  float w_max;
  uint64_t seed, step;
  const unsigned long long* step_add;   // optional device counter added to step
};

__global__ __launch_bounds__(256) void wire_quantize_kernel(WireArgs a) {
  const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= (size_t)a.K * a.N) return;
  const double qw = (double)((1u << a.weight_bits) - 1);
  a.q[t] = (int32_t)::rint(clampd((double)a.W[t] / (double)a.w_max, -1.0, 1.0) * qw);
}

// Conductances of the device pair (slice s) of weight (k, n) before the wire model.
__device__ __forceinline__ void wire_device_pair(const WireArgs& a, NormalStream& rng, int q, int k, int n, int s,
                                                 double g[2]) {
  const int digit = (int)(((uint32_t)::abs(q) >> (a.slice_bits * s)) & ((1u << a.slice_bits) - 1));
  g[0] = a.g_min + (q > 0 ? digit * a.dg : 0.0);
  g[1] = a.g_min + (q < 0 ? digit * a.dg : 0.0);
  if (a.flags & XBAR_NI_VARIATION) {
    const uint64_t dev = (((uint64_t)k * (uint64_t)a.N + (uint64_t)n) * (uint64_t)a.S_w + (uint64_t)s) * 2;
    g[0] *= 1.0 + a.var_sigma * rng.get(dev);
    g[1] *= 1.0 + a.var_sigma * rng.get(dev + 1);
  }
}

// grid (tiles x 4 quarters of the tile rows, S_w); a wave scans one tile row at a time (both arrays),
// lane l holds the ceil(C / 64) consecutive columns that start at l ceil(C / 64).
__global__ __launch_bounds__(256) void wire_rows_kernel(WireArgs a) {
  const int tile = blockIdx.x >> 2, quarter = blockIdx.x & 3;
  const int tr = tile / a.tiles_c, tc = tile % a.tiles_c;
  const int s = blockIdx.y;
  const int k0 = tr * a.R, n0 = tc * a.C;
  const int rows = min(a.R, a.K - k0), cols = min(a.C, a.N - n0);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int cpl = (a.C + 63) >> 6;
  const int i_end = min(rows, (quarter + 1) * (a.R / 4));
  const size_t pol_stride = (size_t)a.K * a.N;
  NormalStream rng(a.seed, kStreamVariation, effective_step(a.step, a.step_add));
  for (int i = quarter * (a.R / 4) + wave; i < i_end; i += 4) {
    double l0[4][2], l1[4][2];                       // inclusive prefixes inside the lane
    double run0[2] = {0.0, 0.0}, run1[2] = {0.0, 0.0};
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (u >= cpl) break;
      const int j = lane * cpl + u;
      double g[2] = {0.0, 0.0};
      if (j < cols) wire_device_pair(a, rng, a.q[(size_t)(k0 + i) * a.N + n0 + j], k0 + i, n0 + j, s, g);
#pragma unroll
      for (int pol = 0; pol < 2; ++pol) {
        run0[pol] += g[pol];                         // sum_{j' <= j} G
        run1[pol] += (double)(j + 1) * g[pol];       // sum_{j' <= j} (j' + 1) G
        l0[u][pol] = run0[pol];
        l1[u][pol] = run1[pol];
      }
    }
    double before0[2], before1[2], total[2];         // sums over the lanes to the left, and the row total
#pragma unroll
    for (int pol = 0; pol < 2; ++pol) {
      const double inc0 = wave_inclusive_scan(run0[pol], lane);
      const double inc1 = wave_inclusive_scan(run1[pol], lane);
      before0[pol] = inc0 - run0[pol];
      before1[pol] = inc1 - run1[pol];
      total[pol] = __shfl(inc0, 63, 64);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (u >= cpl) break;
      const int j = lane * cpl + u;
      if (j < cols) {
        const size_t at = ((size_t)(2 * s) * a.K + k0 + i) * a.N + n0 + j;
#pragma unroll
        for (int pol = 0; pol < 2; ++pol) {
          const double p0 = before0[pol] + l0[u][pol], p1 = before1[pol] + l1[u][pol];
          a.A[at + pol * pol_stride] = a.r_source * total[pol] + a.r_row * (p1 + (double)(j + 1) * (total[pol] - p0));
        }
      }
    }
  }
}

// grid (tiles x strips of 64 columns, S_w); thread = (quarter of the tile rows, column).  First walk:
// per-quarter totals; after the exchange a second walk knows, at every row, the sums over all devices
// above and below and finishes the plane value.
__global__ __launch_bounds__(256) void wire_cols_kernel(WireArgs a) {
  __shared__ double tot[2][2][4][64];              // [sum of G | sum of (R - i) G][array][quarter][column]
  const int strips = (a.C + 63) / 64;
  const int tile = blockIdx.x / strips, strip = blockIdx.x % strips;
  const int tr = tile / a.tiles_c, tc = tile % a.tiles_c;
  const int s = blockIdx.y;
  const int k0 = tr * a.R, n0 = tc * a.C;
  const int rows = min(a.R, a.K - k0), cols = min(a.C, a.N - n0);
  const int seg = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int j = strip * 64 + lane;
  const bool active = j < cols;
  const int i_begin = seg * (a.R / 4), i_end = min(rows, i_begin + a.R / 4);
  NormalStream rng(a.seed, kStreamVariation, effective_step(a.step, a.step_add));
  double t0[2] = {0.0, 0.0}, t1[2] = {0.0, 0.0};
  if (active)
    for (int i = i_begin; i < i_end; ++i) {
      double g[2];
      wire_device_pair(a, rng, a.q[(size_t)(k0 + i) * a.N + n0 + j], k0 + i, n0 + j, s, g);
#pragma unroll
      for (int pol = 0; pol < 2; ++pol) {
        t0[pol] += g[pol];
        t1[pol] += (double)(a.R - i) * g[pol];
      }
    }
#pragma unroll
  for (int pol = 0; pol < 2; ++pol) {
    tot[0][pol][seg][lane] = t0[pol];
    tot[1][pol][seg][lane] = t1[pol];
  }
  __syncthreads();
  if (!active) return;
  double above[2], below[2], total[2];
#pragma unroll
  for (int pol = 0; pol < 2; ++pol) {
    above[pol] = 0.0;                                // sum_{i' <= i} G, starts at the quarters above
    below[pol] = t1[pol];                            // sum_{i' > i} (R - i') G, starts with this and later quarters
    total[pol] = 0.0;
    for (int g4 = 0; g4 < 4; ++g4) {
      const double x0 = tot[0][pol][g4][lane];
      total[pol] += x0;
      if (g4 < seg) above[pol] += x0;
      if (g4 > seg) below[pol] += tot[1][pol][g4][lane];
    }
  }
  const size_t pol_stride = (size_t)a.K * a.N;
  for (int ib = i_begin; ib < i_end; ib += 4) {      // quarter lengths are multiples of 4
    int q[4];
    double wa[4][2];
#pragma unroll
    for (int u = 0; u < 4; ++u) {                    // loads first: they do not wait for the stores below
      const int i = min(ib + u, i_end - 1);
      const size_t at = ((size_t)(2 * s) * a.K + k0 + i) * a.N + n0 + j;
      q[u] = a.q[(size_t)(k0 + i) * a.N + n0 + j];
      wa[u][0] = a.A[at];
      wa[u][1] = a.A[at + pol_stride];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = ib + u;
      if (i < i_end) {
        double g[2], e[2];
        wire_device_pair(a, rng, q[u], k0 + i, n0 + j, s, g);
#pragma unroll
        for (int pol = 0; pol < 2; ++pol) {
          above[pol] += g[pol];
          below[pol] -= (double)(a.R - i) * g[pol];
          const double b = a.r_col * ((double)(a.R - i) * above[pol] + below[pol]) + a.r_sense * total[pol];
          e[pol] = g[pol] / (1.0 + wa[u][pol] + b);
        }
        const size_t at = ((size_t)(2 * s) * a.K + k0 + i) * a.N + n0 + j;
        if (a.flags & XBAR_ADC_PER_ARRAY) {            // each array is read on its own
          a.A[at] = e[0] / a.dg;
          a.A[at + pol_stride] = e[1] / a.dg;
        } else {
          a.A[at] = (e[0] - e[1]) / a.dg;
        }
      }
    }
  }
}

}  // namespace

namespace xbar_detail {

int launch_wire_model(const xbar_config* cfg, const float* W, int K, int N, float w_max, uint64_t step, double* wire_u,
                      hipStream_t st) {
  const Derived d = derive(cfg);
  WireArgs w;
  w.W = W; w.A = wire_u;
  w.q = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(wire_u) + align256((size_t)16 * d.S_w * K * N));
  w.K = K; w.N = N; w.R = cfg->xbar_rows; w.C = cfg->xbar_cols; w.S_w = d.S_w;
  w.slice_bits = cfg->slice_bits; w.weight_bits = cfg->weight_bits;
  w.tiles_c = cdiv(N, cfg->xbar_cols);
  w.flags = cfg->flags;
  w.g_min = 1.0 / (double)cfg->r_max;
  w.dg = (1.0 / (double)cfg->r_min - w.g_min) / (double)((1 << cfg->slice_bits) - 1);
  w.var_sigma = (double)cfg->var_sigma;
  w.r_row = (double)cfg->r_row; w.r_col = (double)cfg->r_col;
  w.r_source = (double)cfg->r_source; w.r_sense = (double)cfg->r_sense;
  w.w_max = w_max; w.seed = cfg->seed; w.step = step; w.step_add = current_step_source();
  const unsigned tiles = (unsigned)(cdiv(K, cfg->xbar_rows) * w.tiles_c);
  hipLaunchKernelGGL(wire_quantize_kernel, dim3((unsigned)(((size_t)K * N + 255) / 256)), dim3(256), 0, st, w);
  if (hipGetLastError() != hipSuccess) return XBAR_EHIP;
  hipLaunchKernelGGL(wire_rows_kernel, dim3(tiles * 4u, (unsigned)d.S_w), dim3(256), 0, st, w);
  if (hipGetLastError() != hipSuccess) return XBAR_EHIP;
  hipLaunchKernelGGL(wire_cols_kernel, dim3(tiles * (unsigned)((cfg->xbar_cols + 63) / 64), (unsigned)d.S_w), dim3(256),
                     0, st, w);
  if (hipGetLastError() != hipSuccess) return XBAR_EHIP;
  return XBAR_OK;
}

}  // namespace xbar_detail
