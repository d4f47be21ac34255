// Circuit-level crossbar model (Sec. IV-A) producing the stored distortion profile of Sec. IV-D:
// kernels and xbar_fcm_profile.
#include "xbar_common.h"

using namespace xbar_detail;

namespace {

// ---------------------------------------------------------------------------------------------
// circuit-level crossbar model (Sec. IV-A: solve Ohm's and Kirchhoff's laws per crossbar instance;
// Sec. IV-D: the distortion profile D = (G_ideal - G_nonideal) / G_ideal that is stored and reused)
//
// Per crossbar, slice and array, with x_ij the device currents for the row voltages v:
//   x_ij / G_ij + sum_j' x_ij' wr(j,j') + sum_i' x_i'j wc(i,i') = v_i          (D + L) x = P v
//   wr(j,j') = r_source + (min(j,j') + 1) r_row,   wc(i,i') = (R - max(i,i')) r_col + r_sense
// L is the resistance matrix of the wires: symmetric, positive semidefinite, and applied in O(R C)
// by row and column prefix sums.  With x = s y, s = sqrt(G), the system (I + S L S) y = s v is
// symmetric positive definite with all eigenvalues >= 1 and a small condition number; conjugate
// gradients solve it for one unit row voltage at a time, and row i of the non-ideal conductance
// matrix is the column sums of x.  Devices that do not exist have s = 0 and drop out.
// ---------------------------------------------------------------------------------------------
struct FcmArgs {
  const float* W;
  float* profile;        // [S_w][2][K][N]
  double* scratch;       // per resident block: s, y, r, p, q of R C doubles each
  int K, N, R, C, S_w, slice_bits, weight_bits, tiles_c;
  int groups, rhs_per_group, n_items, max_iter;
  uint32_t flags;
  double g_min, dg, var_sigma, r_row, r_col, r_source, r_sense, tol2;
  float w_max;
  uint64_t seed, step;
  const unsigned long long* step_add;   // optional device counter added to step
};

// Sum over the 256 threads of the block, returned to all of them; fixed order.
__device__ __forceinline__ double block_sum(double v, double* red) {
#pragma unroll
  for (int d = 32; d; d >>= 1) v += __shfl_xor(v, d, 64);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

__global__ __launch_bounds__(256) void fcm_kernel(FcmArgs a) {
  __shared__ double red[4];
  __shared__ double tot[2][4][64];                  // column pass: quarter totals per column of a strip
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int R = a.R, C = a.C;
  const int cpl = (C + 63) >> 6, strips = (C + 63) >> 6;
  const size_t rc = (size_t)R * C;
  double* sg = a.scratch + (size_t)blockIdx.x * 5 * rc;
  double* y = sg + rc;
  double* r = y + rc;
  double* p = r + rc;
  double* q = p + rc;
  NormalStream rng(a.seed, kStreamVariation, effective_step(a.step, a.step_add));

  for (int item = blockIdx.x; item < a.n_items; item += gridDim.x) {
    const int group = item % a.groups;
    const int t1 = item / a.groups;
    const int pol = t1 & 1;
    const int s = (t1 >> 1) % a.S_w;
    const int tile = (t1 >> 1) / a.S_w;
    const int k0 = (tile / a.tiles_c) * R, n0 = (tile % a.tiles_c) * C;
    const int rows = min(R, a.K - k0), cols = min(C, a.N - n0);
    const int i_begin = wave * (R / 4), i_end = min(rows, i_begin + R / 4);   // this wave's quarter (column pass)

    __syncthreads();                                 // the previous item is done with the scratch
    for (int i = wave; i < rows; i += 4)
      for (int j = lane; j < cols; j += 64) {
        const double qw = (double)((1u << a.weight_bits) - 1);
        const double wq = ::rint(clampd((double)a.W[(size_t)(k0 + i) * a.N + n0 + j] / (double)a.w_max, -1.0, 1.0) * qw);
        const int digit = (int)(((uint32_t)::fabs(wq) >> (a.slice_bits * s)) & ((1u << a.slice_bits) - 1));
        const bool mine = pol == 0 ? wq > 0.0 : wq < 0.0;
        double g = a.g_min + (mine ? digit * a.dg : 0.0);
        if (a.flags & XBAR_NI_VARIATION) {
          const uint64_t dev =
              (((uint64_t)(k0 + i) * (uint64_t)a.N + (uint64_t)(n0 + j)) * (uint64_t)a.S_w + (uint64_t)s) * 2 + pol;
          g *= 1.0 + a.var_sigma * rng.get(dev);
        }
        sg[(size_t)i * C + j] = ::sqrt(::fmax(g, 0.0));
      }
    __syncthreads();

    const int rhs_end = min(rows, (group + 1) * a.rhs_per_group);
    for (int rhs = group * a.rhs_per_group; rhs < rhs_end; ++rhs) {
      // y = 0, r = b = s on the driven row, p = 0 (the first direction is r)
      double part = 0.0;
      for (int i = wave; i < rows; i += 4)
        for (int j = lane; j < cols; j += 64) {
          const size_t at = (size_t)i * C + j;
          const double b = i == rhs ? sg[at] : 0.0;
          y[at] = 0.0;
          r[at] = b;
          p[at] = 0.0;
          part += b * b;
        }
      double rr = block_sum(part, red);              // also orders the stores above before the reads below
      const double stop = a.tol2 * rr;
      double beta = 0.0;
      for (int it = 0; it < a.max_iter && rr > stop; ++it) {
        // rows: p <- r + beta p;  q <- p + s Lr(s p)
        for (int i = wave; i < rows; i += 4) {
          const size_t base = (size_t)i * C;
          double pv[4], sv[4], l0[4], l1[4];
          double run0 = 0.0, run1 = 0.0;
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            if (u >= cpl) break;
            const int j = lane * cpl + u;
            pv[u] = sv[u] = 0.0;
            if (j < cols) {
              pv[u] = r[base + j] + beta * p[base + j];
              sv[u] = sg[base + j];
              p[base + j] = pv[u];
            }
            const double cur = sv[u] * pv[u];
            run0 += cur;
            run1 += (double)(j + 1) * cur;
            l0[u] = run0;
            l1[u] = run1;
          }
          const double inc0 = wave_inclusive_scan(run0, lane), inc1 = wave_inclusive_scan(run1, lane);
          const double total = __shfl(inc0, 63, 64);
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            if (u >= cpl) break;
            const int j = lane * cpl + u;
            if (j < cols) {
              const double p0 = inc0 - run0 + l0[u], p1 = inc1 - run1 + l1[u];
              const double lr = a.r_source * total + a.r_row * (p1 + (double)(j + 1) * (total - p0));
              q[base + j] = pv[u] + sv[u] * lr;
            }
          }
        }
        __syncthreads();
        // columns: q <- q + s Lc(s p);  p.q
        double pq = 0.0;
        for (int strip = 0; strip < strips; ++strip) {
          const int j = strip * 64 + lane;
          const bool active = j < cols;
          double t0 = 0.0, t1s = 0.0;
          if (active)
            for (int i = i_begin; i < i_end; ++i) {
              const size_t at = (size_t)i * C + j;
              const double cur = sg[at] * p[at];
              t0 += cur;
              t1s += (double)(R - i) * cur;
            }
          tot[0][wave][lane] = t0;
          tot[1][wave][lane] = t1s;
          __syncthreads();
          if (active) {
            double above = 0.0, below = t1s, total = 0.0;
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
              const double x0 = tot[0][g4][lane];
              total += x0;
              if (g4 < wave) above += x0;
              if (g4 > wave) below += tot[1][g4][lane];
            }
            for (int ib = i_begin; ib < i_end; ib += 4) {
              double sv[4], pv[4], qv[4];
#pragma unroll
              for (int u = 0; u < 4; ++u) {            // loads first: they do not wait for the stores below
                const size_t at = (size_t)min(ib + u, i_end - 1) * C + j;
                sv[u] = sg[at];
                pv[u] = p[at];
                qv[u] = q[at];
              }
#pragma unroll
              for (int u = 0; u < 4; ++u) {
                const int i = ib + u;
                if (i < i_end) {
                  const double cur = sv[u] * pv[u];
                  above += cur;
                  below -= (double)(R - i) * cur;
                  const double lc = a.r_col * ((double)(R - i) * above + below) + a.r_sense * total;
                  const double qn = qv[u] + sv[u] * lc;
                  q[(size_t)i * C + j] = qn;
                  pq += pv[u] * qn;
                }
              }
            }
          }
          __syncthreads();                             // tot is reused by the next strip
        }
        pq = block_sum(pq, red);
        const double alpha = rr / pq;
        // y <- y + alpha p;  r <- r - alpha q
        part = 0.0;
        for (int i = wave; i < rows; i += 4)
          for (int j = lane; j < cols; j += 64) {
            const size_t at = (size_t)i * C + j;
            y[at] += alpha * p[at];
            const double rn = r[at] - alpha * q[at];
            r[at] = rn;
            part += rn * rn;
          }
        const double rr_new = block_sum(part, red);
        beta = rr_new / rr;
        rr = rr_new;
      }
      // row rhs of the non-ideal conductance matrix: column sums of x = s y
      for (int strip = 0; strip < strips; ++strip) {
        const int j = strip * 64 + lane;
        double e = 0.0;
        if (j < cols)
          for (int i = i_begin; i < i_end; ++i) e += sg[(size_t)i * C + j] * y[(size_t)i * C + j];
        tot[0][wave][lane] = e;
        __syncthreads();
        if (wave == 0 && j < cols) {
          const double e_all = (tot[0][0][lane] + tot[0][1][lane]) + (tot[0][2][lane] + tot[0][3][lane]);
          const double sv = sg[(size_t)rhs * C + j];
          const double g = sv * sv;
          a.profile[((size_t)(2 * s + pol) * a.K + k0 + rhs) * a.N + n0 + j] = g > 0.0 ? (float)((g - e_all) / g) : 0.0f;
        }
        __syncthreads();
      }
    }
  }
}

// Same solve for 64 x 64 and 128 x 128 crossbars with the whole state on chip.  NT threads form a
// (NT / 16) x 16 grid; thread (ty, tx) owns the SR x SC devices at rows SR ty.., columns SC tx..;
// residual and search direction live in its registers, sqrt(G) in LDS.  Prefix sums along a row run
// over the 16 consecutive lanes that share ty (DPP row shifts), along a column over the 4 lane groups
// of a wave (shuffles) and over the waves (LDS).  A p is computed twice per iteration (for p.Ap, then
// for the residual update) instead of being stored: registers and LDS together hold three vectors of
// crossbar size plus sqrt(G), not four.
template <int CTRL>
__device__ __forceinline__ double dpp_row_f64(double x) {   // lanes whose source lies outside the row of 16 get 0
  union { double d; int i[2]; } v, o;
  v.d = x;
  o.i[0] = __builtin_amdgcn_update_dpp(0, v.i[0], CTRL, 0xF, 0xF, false);
  o.i[1] = __builtin_amdgcn_update_dpp(0, v.i[1], CTRL, 0xF, 0xF, false);
  return o.d;
}

__device__ __forceinline__ double row16_inclusive_scan(double x) {
  x += dpp_row_f64<0x111>(x);                        // row_shr:1
  x += dpp_row_f64<0x112>(x);                        // row_shr:2
  x += dpp_row_f64<0x114>(x);                        // row_shr:4
  x += dpp_row_f64<0x118>(x);                        // row_shr:8
  return x;
}

template <int NW>
__device__ __forceinline__ double block_sum_n(double v, double* red) {
#pragma unroll
  for (int d = 32; d; d >>= 1) v += __shfl_xor(v, d, 64);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  double t = 0.0;
#pragma unroll
  for (int w = 0; w < NW; ++w) t += red[w];
  return t;
}

template <int SR, int SC, int NT>
__global__ __launch_bounds__(NT) void fcm_onchip_kernel(FcmArgs a) {
  extern __shared__ double fcm_lds[];
  constexpr int NW = NT / 64;                        // waves; 4 thread rows (ty) per wave
  constexpr int R = (NT / 16) * SR, C = 16 * SC;     // == a.R, a.C
  double* s_lds = fcm_lds;                           // [SR * SC][NT]: element (ar, bc) of thread tid
  double* xch = fcm_lds + SR * SC * NT;              // [2][NW][16 tx][SC]
  double* red = xch + 2 * NW * 16 * SC;              // [NW]
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int tx = tid & 15, ty = tid >> 4;
  const int i0 = ty * SR, j0 = tx * SC;
  NormalStream rng(a.seed, kStreamVariation, effective_step(a.step, a.step_add));

  for (int item = blockIdx.x; item < a.n_items; item += gridDim.x) {
    const int group = item % a.groups;
    const int t1 = item / a.groups;
    const int pol = t1 & 1;
    const int s = (t1 >> 1) % a.S_w;
    const int tile = (t1 >> 1) / a.S_w;
    const int k0 = (tile / a.tiles_c) * R, n0 = (tile % a.tiles_c) * C;
    const int rows = min(R, a.K - k0), cols = min(C, a.N - n0);

    __syncthreads();
    for (int ar = 0; ar < SR; ++ar)
      for (int bc = 0; bc < SC; ++bc) {
        const int i = i0 + ar, j = j0 + bc;
        double g = 0.0;
        if (i < rows && j < cols) {
          const double qw = (double)((1u << a.weight_bits) - 1);
          const double wq =
              ::rint(clampd((double)a.W[(size_t)(k0 + i) * a.N + n0 + j] / (double)a.w_max, -1.0, 1.0) * qw);
          const int digit = (int)(((uint32_t)::fabs(wq) >> (a.slice_bits * s)) & ((1u << a.slice_bits) - 1));
          const bool mine = pol == 0 ? wq > 0.0 : wq < 0.0;
          g = a.g_min + (mine ? digit * a.dg : 0.0);
          if (a.flags & XBAR_NI_VARIATION) {
            const uint64_t dev =
                (((uint64_t)(k0 + i) * (uint64_t)a.N + (uint64_t)(n0 + j)) * (uint64_t)a.S_w + (uint64_t)s) * 2 + pol;
            g *= 1.0 + a.var_sigma * rng.get(dev);
          }
        }
        s_lds[(ar * SC + bc) * NT + tid] = ::sqrt(::fmax(g, 0.0));
      }
    // every thread reads back only what it wrote itself: no barrier needed for s_lds

    const int rhs_end = min(rows, (group + 1) * a.rhs_per_group);
    for (int rhs = group * a.rhs_per_group; rhs < rhs_end; ++rhs) {
      double r[SR][SC], p[SR][SC], e_acc[SC];
      double part = 0.0;
#pragma unroll
      for (int ar = 0; ar < SR; ++ar)
#pragma unroll
        for (int bc = 0; bc < SC; ++bc) {
          r[ar][bc] = (i0 + ar == rhs) ? s_lds[(ar * SC + bc) * NT + tid] : 0.0;
          p[ar][bc] = 0.0;
          part += r[ar][bc] * r[ar][bc];
        }
#pragma unroll
      for (int bc = 0; bc < SC; ++bc) e_acc[bc] = 0.0;
      double rr = block_sum_n<NW>(part, red);
      const double stop = a.tol2 * rr;
      double beta = 0.0;
      for (int it = 0; it < a.max_iter && rr > stop; ++it) {
        // p <- r + beta p, and the sums of u = s p over this thread's part of every row and column
        double row0[SR], row1[SR], rtot[SR], col0[SC], col1[SC], ctot[SC];
#pragma unroll
        for (int x = 0; x < SR; ++x) row0[x] = row1[x] = 0.0;
#pragma unroll
        for (int x = 0; x < SC; ++x) col0[x] = col1[x] = 0.0;
#pragma unroll
        for (int ar = 0; ar < SR; ++ar)
#pragma unroll
          for (int bc = 0; bc < SC; ++bc) {
            p[ar][bc] = r[ar][bc] + beta * p[ar][bc];
            const double u = s_lds[(ar * SC + bc) * NT + tid] * p[ar][bc];
            row0[ar] += u;
            row1[ar] += (double)(j0 + bc + 1) * u;
            col0[bc] += u;
            col1[bc] += (double)(R - (i0 + ar)) * u;
          }
        // rows: sums over the threads to the left (same ty = one DPP row of 16 lanes), and the row totals
#pragma unroll
        for (int ar = 0; ar < SR; ++ar) {
          const double inc0 = row16_inclusive_scan(row0[ar]), inc1 = row16_inclusive_scan(row1[ar]);
          rtot[ar] = dpp_row_f64<0x15F>(inc0);         // row_newbcast:15
          row0[ar] = inc0 - row0[ar];                  // sum_{j' < j0} u
          row1[ar] = inc1 - row1[ar];                  // sum_{j' < j0} (j' + 1) u
        }
        // columns: sums over the lane groups above inside the wave, then over the waves
#pragma unroll
        for (int bc = 0; bc < SC; ++bc) {
          double inc0 = col0[bc], inc1 = col1[bc];
          double y0 = __shfl_up(inc0, 16, 64), y1 = __shfl_up(inc1, 16, 64);
          if (lane >= 16) { inc0 += y0; inc1 += y1; }
          y0 = __shfl_up(inc0, 32, 64); y1 = __shfl_up(inc1, 32, 64);
          if (lane >= 32) { inc0 += y0; inc1 += y1; }
          if (lane >= 48) {                            // last group of the wave holds the wave's sums
            xch[(0 * NW + wave) * 16 * SC + tx * SC + bc] = inc0;
            xch[(1 * NW + wave) * 16 * SC + tx * SC + bc] = inc1;
          }
          col0[bc] = inc0 - col0[bc];                  // groups above, inside the wave
          col1[bc] = inc1 - col1[bc];
        }
        __syncthreads();
#pragma unroll
        for (int bc = 0; bc < SC; ++bc) {
          double all0 = 0.0, all1 = 0.0, before0 = 0.0, before1 = 0.0;
#pragma unroll
          for (int w = 0; w < NW; ++w) {
            const double w0 = xch[(0 * NW + w) * 16 * SC + tx * SC + bc], w1 = xch[(1 * NW + w) * 16 * SC + tx * SC + bc];
            all0 += w0;
            all1 += w1;
            if (w < wave) { before0 += w0; before1 += w1; }
          }
          ctot[bc] = all0;
          col0[bc] += before0;                         // sum_{i' < i0} u
          col1[bc] = all1 - (before1 + col1[bc]);      // sum_{i' >= i0} (R - i') u
        }
        // A p = p + s (Lr + Lc)(u): first for p.Ap, walking down the rows (the column sums end one
        // block further down) ...
        double pq = 0.0;
#pragma unroll
        for (int ar = 0; ar < SR; ++ar) {
          double run0 = row0[ar], run1 = row1[ar];
#pragma unroll
          for (int bc = 0; bc < SC; ++bc) {
            const double sv = s_lds[(ar * SC + bc) * NT + tid];
            const double u = sv * p[ar][bc];
            const double jj = (double)(j0 + bc + 1), ii = (double)(R - (i0 + ar));
            run0 += u;
            run1 += jj * u;
            col0[bc] += u;
            col1[bc] -= ii * u;
            const double lr = a.r_source * rtot[ar] + a.r_row * (run1 + jj * (rtot[ar] - run0));
            const double lc = a.r_col * (ii * col0[bc] + col1[bc]) + a.r_sense * ctot[bc];
            pq += p[ar][bc] * (p[ar][bc] + sv * (lr + lc));
          }
        }
        pq = block_sum_n<NW>(pq, red);
        const double alpha = rr / pq;
        // ... then again for r <- r - alpha A p, walking back up and undoing the column sums
        part = 0.0;
#pragma unroll
        for (int ar = SR - 1; ar >= 0; --ar) {
          double run0 = row0[ar], run1 = row1[ar];
#pragma unroll
          for (int bc = 0; bc < SC; ++bc) {
            const double sv = s_lds[(ar * SC + bc) * NT + tid];
            const double u = sv * p[ar][bc];
            const double jj = (double)(j0 + bc + 1), ii = (double)(R - (i0 + ar));
            run0 += u;
            run1 += jj * u;
            const double lr = a.r_source * rtot[ar] + a.r_row * (run1 + jj * (rtot[ar] - run0));
            const double lc = a.r_col * (ii * col0[bc] + col1[bc]) + a.r_sense * ctot[bc];
            col0[bc] -= u;
            col1[bc] += ii * u;
            const double rn = r[ar][bc] - alpha * (p[ar][bc] + sv * (lr + lc));
            r[ar][bc] = rn;
            part += rn * rn;
          }
        }
#pragma unroll
        for (int bc = 0; bc < SC; ++bc) e_acc[bc] += alpha * ctot[bc];   // column sums of x = s y, y = sum alpha p
        const double rr_new = block_sum_n<NW>(part, red);
        beta = rr_new / rr;
        rr = rr_new;
      }
      if (rhs >= i0 && rhs < i0 + SR) {
#pragma unroll
        for (int bc = 0; bc < SC; ++bc) {
          const int j = j0 + bc;
          if (j < cols) {
            const double sv = s_lds[((rhs - i0) * SC + bc) * NT + tid];
            const double g = sv * sv;
            a.profile[((size_t)(2 * s + pol) * a.K + k0 + rhs) * a.N + n0 + j] =
                g > 0.0 ? (float)((g - e_acc[bc]) / g) : 0.0f;
          }
        }
      }
    }
  }
}

struct FcmPlan {
  int n_items, groups, rhs_per_group, blocks;
  int onchip;            // 0: state in the workspace; 64 / 128: square crossbars of that size, state on chip
  size_t lds_bytes, ws_bytes;
};

FcmPlan plan_fcm(const xbar_config* c, const Derived& d, int K, int N) {
  FcmPlan p;
  const int per_drive_sets = cdiv(K, c->xbar_rows) * cdiv(N, c->xbar_cols) * d.S_w * 2;   // (tile, slice, array)
  // split the driven rows of a crossbar over several blocks when there are few crossbars
  p.groups = std::min(c->xbar_rows / 4, std::max(1, cdiv(2048, per_drive_sets)));
  p.rhs_per_group = cdiv(c->xbar_rows, p.groups);
  p.groups = cdiv(c->xbar_rows, p.rhs_per_group);
  p.n_items = per_drive_sets * p.groups;
  p.onchip = (c->xbar_rows == c->xbar_cols && (c->xbar_rows == 64 || c->xbar_rows == 128)) ? c->xbar_rows : 0;
  {  // s, the column exchange area [2][waves][16][SC] and the reduction slots
    const int nt = 256, sc = p.onchip / 16;
    p.lds_bytes = ((size_t)p.onchip * p.onchip + 2 * (nt / 64) * 16 * sc + nt / 64) * sizeof(double);
  }
  // the workspace is sized for the general kernel in every case (it is the fallback)
  const size_t slot = (size_t)5 * c->xbar_rows * c->xbar_cols * sizeof(double);
  p.blocks = std::min(p.n_items, slot > (size_t)1 << 20 ? 1024 : 2048);
  p.ws_bytes = align256((size_t)p.blocks * slot);
  return p;
}

}  // namespace

namespace xbar_detail {
size_t fcm_workspace_bytes(const xbar_config* cfg, int K, int N) { return plan_fcm(cfg, derive(cfg), K, N).ws_bytes; }
}  // namespace xbar_detail

extern "C" {

int xbar_fcm_profile(const xbar_config* cfg, const float* W, int K, int N, float w_max, uint64_t step, float* profile,
                     void* ws, size_t ws_bytes, void* hip_stream) {
  int rc = xbar_config_validate(cfg);
  if (rc) return rc;
  if ((rc = check_shape(1, K, N))) return rc;
  if (!aligned16(W) || !aligned16(profile) || !aligned16(ws)) return XBAR_EALIGN;
  if (!finite_pos(w_max)) return XBAR_EINVAL;
  const Derived d = derive(cfg);
  const FcmPlan p = plan_fcm(cfg, d, K, N);
  if (ws_bytes < p.ws_bytes) return XBAR_EWORKSPACE;
  FcmArgs a;
  a.W = W; a.profile = profile; a.scratch = reinterpret_cast<double*>(ws);
  a.K = K; a.N = N; a.R = cfg->xbar_rows; a.C = cfg->xbar_cols; a.S_w = d.S_w;
  a.slice_bits = cfg->slice_bits; a.weight_bits = cfg->weight_bits; a.tiles_c = cdiv(N, cfg->xbar_cols);
  a.groups = p.groups; a.rhs_per_group = p.rhs_per_group; a.n_items = p.n_items;
  a.max_iter = 500;
  a.flags = cfg->flags;
  a.g_min = 1.0 / (double)cfg->r_max;
  a.dg = (1.0 / (double)cfg->r_min - a.g_min) / (double)((1 << cfg->slice_bits) - 1);
  a.var_sigma = (double)cfg->var_sigma;
  a.r_row = (double)cfg->r_row; a.r_col = (double)cfg->r_col;
  a.r_source = (double)cfg->r_source; a.r_sense = (double)cfg->r_sense;
  a.tol2 = 1e-22;                                   // relative residual 1e-11
  a.w_max = w_max; a.seed = cfg->seed; a.step = step; a.step_add = current_step_source();
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  if (p.onchip) {
    const void* fn = p.onchip == 128 ? reinterpret_cast<const void*>(&fcm_onchip_kernel<8, 8, 256>)
                                     : reinterpret_cast<const void*>(&fcm_onchip_kernel<4, 4, 256>);
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.lds_bytes) == hipSuccess) {
      if (p.onchip == 128)
        hipLaunchKernelGGL((fcm_onchip_kernel<8, 8, 256>), dim3((unsigned)p.blocks), dim3(256), p.lds_bytes, st, a);
      else
        hipLaunchKernelGGL((fcm_onchip_kernel<4, 4, 256>), dim3((unsigned)p.blocks), dim3(256), p.lds_bytes, st, a);
      return hipGetLastError() == hipSuccess ? XBAR_OK : XBAR_EHIP;
    }
    (void)hipGetLastError();                         // no such LDS size on this device: general kernel
  }
  hipLaunchKernelGGL(fcm_kernel, dim3((unsigned)p.blocks), dim3(256), 0, st, a);
  if (hipGetLastError() != hipSuccess) return XBAR_EHIP;
  return XBAR_OK;
}

}  // extern "C"
