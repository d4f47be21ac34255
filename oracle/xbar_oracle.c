/*
 * TEST INFRASTRUCTURE -- scalar CPU oracle of the non-ideal crossbar training operations.
 *
 * This file is the plain, slow, obviously-correct statement of what the GPU library must compute.
 * It is only ever used by the tests, by the smoke check and by the "cpu_baseline" leg of the
 * benchmark.  It shares no code, header, table or constant with the HIP path (the parameter struct
 * below is re-typed by hand), every floating-point step is IEEE double, every integer step is
 * int64, all loops are scalar and run in index order.
 *
 * What is modelled (TxSim, arXiv 2002.11151):
 *   Sec. IV    -- a layer is DAC model -> crossbar array model -> ADC model, in the forward and in
 *                 the backward pass; inputs are scaled before the DAC and outputs after the ADC.
 *   Sec. IV-A  -- non-ideal conductance matrix generator: weights are mapped to one or more
 *                 limited-precision devices (bit slices), partitioned into crossbar instances,
 *                 split into a positive and a negative array whose currents are subtracted,
 *                 process variation is applied per device, then the wire-parasitic model
 *                 converts ideal into non-ideal conductances and the instances are stitched.
 *   Sec. IV-B  -- three-stage model: digital inputs -> voltages, voltages x non-ideal
 *                 conductances -> column currents, currents -> ADC codes.
 *   Sec. IV-C  -- update model: gradient -> scale -> ideal conductance change -> state dependent
 *                 write non-linearity (factor v) -> Gaussian write noise (factor gamma) ->
 *                 times learning rate, subtracted from the stored conductance.
 *   Sec. IV-D  -- approximate analytical model (shortest path per device, series resistance of
 *                 source, row wire, column wire and sense; optionally all first-order paths, i.e.
 *                 the wire drops caused by every device that shares the row or the column) and
 *                 the stored distortion profile D = (G_ideal - G_nonideal) / G_ideal of
 *                 interpolated FCM.
 *   Sec. V     -- default parameters (Rmin 100 kOhm, Rmax 1 MOhm, 1 Ohm / 4.6 Ohm wire per cell,
 *                 2-bit devices, bit-streamed inputs).
 *
 * Readings taken where the paper is silent are listed next to the code that takes them.
 * PARITY UNPINNED (no printed value or formula survives in the paper text): the shape of the
 * update non-linearity (Eq. 1 is an image), the DAC transfer table, the units of gamma.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* flag bits (same numeric values as the library's, typed again here on purpose) */
#define XO_VARIATION    1u
#define XO_WIRE_AAM     2u
#define XO_WIRE_PROFILE 4u
#define XO_UPD_NL       8u
#define XO_UPD_NOISE    16u
#define XO_DAC_LUT      32u
#define XO_INPUT_SIGNED 64u
#define XO_WIRE_AAM2    128u
#define XO_ADC_CURVE    256u
#define XO_ADC_PER_ARRAY 512u
#define XO_INPUT_OFFSET 1024u
#define XO_PULSE_CODED 2048u
#define XO_PULSE_MAGNITUDE 4096u

#define XO_STREAM_VARIATION 1u
#define XO_STREAM_WRITE     2u
#define XO_STREAM_PULSE_ROWS  3u
#define XO_STREAM_PULSE_COLS  4u
#define XO_STREAM_PULSE_NOISE 5u
#define XO_STREAM_WRITE_PAIR  6u

typedef struct xo_config {
  uint32_t struct_size, abi_version;
  int32_t xbar_rows, xbar_cols;
  int32_t weight_bits, slice_bits;
  int32_t input_bits, stream_bits;
  int32_t adc_bits;
  uint32_t flags;
  float r_min, r_max;
  float v_max;
  float r_row, r_col;
  float r_source, r_sense;
  float var_sigma;
  float upd_nl_v, upd_noise_gamma;
  float adc_fs_fwd, adc_fs_bwd;
  float dac_lut[16];
  float adc_curve[17];
  uint64_t seed;
} xo_config;

/* ------------------------------------------------------------------------------------------- */
/* Counter-based random numbers: Philox-4x32 with 10 rounds (Salmon et al., SC'11), written from */
/* the published round function; then Box-Muller.  The paper names the distribution only.      */
/* ------------------------------------------------------------------------------------------- */
void xo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Standard normal number i of (seed, stream, step).  Four consecutive i share one Philox block:
 * words (0,1) give numbers 0 and 1 (cosine and sine branch), words (2,3) give numbers 2 and 3. */
double xo_normal(uint64_t seed, uint32_t stream, uint64_t step, uint64_t i) {
  uint64_t blk = i >> 2;
  uint32_t ctr[4] = {(uint32_t)blk, (uint32_t)(blk >> 32), (uint32_t)step, (uint32_t)(step >> 32)};
  uint32_t key[2] = {(uint32_t)seed ^ (0x9E3779B9u * stream),
                     (uint32_t)(seed >> 32) ^ (0xBB67AE85u * stream)};
  uint32_t w[4];
  xo_philox4x32_10(ctr, key, w);
  int pair = (int)((i & 3u) >> 1);
  double u1 = ((double)w[2 * pair] + 0.5) * (1.0 / 4294967296.0);
  double u2 = ((double)w[2 * pair + 1] + 0.5) * (1.0 / 4294967296.0);
  double r = sqrt(-2.0 * log(u1));
  double th = 6.283185307179586476925286766559 * u2;
  return (i & 1u) ? r * sin(th) : r * cos(th);
}

/* ------------------------------------------------------------------------------------------- */
static double clampd(double x, double lo, double hi) { return x < lo ? lo : (x > hi ? hi : x); }

/* Sec. IV-A, first generator step: a weight becomes a signed integer of weight_bits magnitude
 * bits (the sign selects the positive or the negative array).  Rounding: half to even.        */
int64_t xo_quantize_weight(float w, float w_max, int weight_bits) {
  double qw = (double)((1ll << weight_bits) - 1);
  return (int64_t)rint(clampd((double)w / (double)w_max, -1.0, 1.0) * qw);
}

/* Digits of a magnitude, least significant slice first: one digit per limited-precision device. */
void xo_digits(uint64_t mag, int digit_bits, int n_digits, int32_t* d) {
  for (int s = 0; s < n_digits; ++s)
    d[s] = (int32_t)((mag >> (digit_bits * s)) & ((1ull << digit_bits) - 1));
}

/* Sec. IV: inputs are scaled, then quantised to input_bits magnitude bits (half to even).
 * Unsigned inputs clamp to [0,1], signed ones to [-1,1].                                        */
int64_t xo_quantize_input(float x, float x_scale, int input_bits, int is_signed) {
  double qa = (double)((1ll << input_bits) - 1);
  return (int64_t)rint(clampd((double)x / (double)x_scale, is_signed ? -1.0 : 0.0, 1.0) * qa);
}

/* Offset-binary code of a signed input (variant of the two-phase scheme for signed inputs on
 * drivers that only supply 0 .. v_max, Sec. V): the range [-scale, scale] is mapped onto the
 * driver's range, u = rne((x / scale + 1) / 2 * (2^bits - 1)), so that one phase streams the
 * input and the constant half-range is taken out digitally afterwards.  The coded value is
 * (2 u - (2^bits - 1)) / (2^bits - 1) * scale.  Zero is not a code: the range has an odd number
 * of steps, its middle lies half a step from the two nearest codes and rounds to the even one. */
int64_t xo_quantize_input_offset(float x, float x_scale, int input_bits) {
  double qa = (double)((1ll << input_bits) - 1);
  return (int64_t)rint(clampd(((double)x / (double)x_scale + 1.0) * 0.5, 0.0, 1.0) * qa);
}

/* Sums of the quantised weights over the rows (colsum[n], used by the forward pass) and over the
 * columns (rowsum[k], backward pass): what the digital correction of the offset-binary scheme
 * multiplies the half-range with.  The digital side knows the programmed (ideal) weights.      */
int xo_weight_sums(const xo_config* cfg, const float* W, int K, int N, float w_max, int64_t* colsum, int64_t* rowsum) {
  if (!cfg || !W || !colsum || !rowsum || K <= 0 || N <= 0) return -1;
  for (int n = 0; n < N; ++n) colsum[n] = 0;
  for (int k = 0; k < K; ++k) {
    rowsum[k] = 0;
    for (int n = 0; n < N; ++n) {
      int64_t q = xo_quantize_weight(W[(size_t)k * N + n], w_max, cfg->weight_bits);
      colsum[n] += q;
      rowsum[k] += q;
    }
  }
  return 0;
}

/* ADC of Sec. IV-B with the identity transfer curve: a signed mid-tread quantiser that saturates.
 * The gain is the single-precision quotient Q / full_scale (the precision the converter
 * decision is defined in); the product with the current and the rounding are done exactly.    */
int64_t xo_adc(double current, float full_scale, int adc_bits) {
  int64_t q = (1ll << (adc_bits - 1)) - 1;
  float gain = (float)q / full_scale;
  double c = rint(current * (double)gain);
  if (c > (double)q) c = (double)q;
  if (c < -(double)q) c = -(double)q;
  return (int64_t)c;
}

/* Unsigned converter of one array (variant of Sec. IV-A's pair of arrays: instead of subtracting
 * the two column currents in front of one signed converter, each array has a converter of its
 * own and the codes are subtracted digitally): all 2^bits - 1 codes on the positive side.        */
int64_t xo_adc_unsigned(double current, float full_scale, int adc_bits) {
  int64_t q = (1ll << adc_bits) - 1;
  float gain = (float)q / full_scale;
  double c = rint(current * (double)gain);
  if (c > (double)q) c = (double)q;
  if (c < 0.0) c = 0.0;
  return (int64_t)c;
}

/* Non-linear converter (Sec. IV-B: the ADC model is the user's; Sec. V: the paper's is calibrated with
 * SPICE): a monotone transfer curve f on the normalised current x = I / full_scale in [-1, 1], given
 * by its values at the 17 equidistant points x = -1 + i / 8 and linear in between;
 * code = clamp(rne(Q f(x)), -Q, Q).  The identity curve is the linear converter above.            */
int64_t xo_adc_curve(const float* curve, double current, float full_scale, int adc_bits) {
  int64_t q = (1ll << (adc_bits - 1)) - 1;
  float gain = (float)q / full_scale;
  double x = current * (double)gain / (double)q;
  if (x > 1.0) x = 1.0;
  if (x < -1.0) x = -1.0;
  double t = (x + 1.0) * 8.0;
  int i = (int)floor(t);
  if (i > 15) i = 15;
  double f = (double)curve[i] + (t - (double)i) * ((double)curve[i + 1] - (double)curve[i]);
  double c = rint((double)q * f);
  if (c > (double)q) c = (double)q;
  if (c < -(double)q) c = -(double)q;
  return (int64_t)c;
}

/* ------------------------------------------------------------------------------------------- */
/* Non-ideal conductance matrix generator (Sec. IV-A, IV-D).                                    */
/* Output: U[s][ki][ni] = (G+ - G-) / dG, the stitched signed plane of slice s in units of one  */
/* device level, for the weights W[ki][ni] that sit at absolute positions (k_idx[ki], n_idx[ni]) */
/* of a K_full x N_full layer (NULL index arrays mean the identity).                            */
/* profile: D[s][pol][k][n] over the full layer (pol 0 = positive array), or NULL.              */
/* ------------------------------------------------------------------------------------------- */
/* Device conductance before the wire model: digit -> level of the array that carries the sign of
 * the weight (the other array rests at the lowest conductance), then process variation.          */
static void device_pair(const xo_config* cfg, int sign, int digit, uint64_t k, uint64_t n, int s, int S,
                        int N_full, uint64_t step, double g_min, double dg, double g[2]) {
  g[0] = g_min + (sign > 0 ? digit * dg : 0.0);
  g[1] = g_min + (sign < 0 ? digit * dg : 0.0);
  if (cfg->flags & XO_VARIATION)       /* independent multiplicative Gaussian per device */
    for (int pol = 0; pol < 2; ++pol) {
      uint64_t dev = ((k * (uint64_t)N_full + n) * (uint64_t)S + (uint64_t)s) * 2 + (uint64_t)pol;
      g[pol] *= 1.0 + (double)cfg->var_sigma * xo_normal(cfg->seed, XO_STREAM_VARIATION, step, dev);
    }
}

/* Conductances of every device before the wire model (after variation): G[S][2][K][N], array index
 * 0 = positive.  Input of the circuit-level crossbar model (Sec. IV-A: non-ideal conductance matrix
 * generator), whose linear solve lives in oracle/nodal.py.                                          */
int xo_device_conductances(const xo_config* cfg, const float* W, int K, int N, float w_max, uint64_t step,
                           double* G) {
  const int S = cfg->weight_bits / cfg->slice_bits;
  const int levels = (1 << cfg->slice_bits) - 1;
  const double g_min = 1.0 / (double)cfg->r_max;
  const double dg = (1.0 / (double)cfg->r_min - g_min) / (double)levels;
  int32_t d[64];
  if (S > 64) return -1;
  for (int k = 0; k < K; ++k)
    for (int n = 0; n < N; ++n) {
      const int64_t q = xo_quantize_weight(W[(size_t)k * N + n], w_max, cfg->weight_bits);
      xo_digits((uint64_t)(q < 0 ? -q : q), cfg->slice_bits, S, d);
      for (int s = 0; s < S; ++s) {
        double g[2];
        device_pair(cfg, (q > 0) - (q < 0), d[s], (uint64_t)k, (uint64_t)n, s, S, N, step, g_min, dg, g);
        G[(((size_t)s * 2 + 0) * K + k) * N + n] = g[0];
        G[(((size_t)s * 2 + 1) * K + k) * N + n] = g[1];
      }
    }
  return 0;
}

int xo_planes(const xo_config* cfg, const float* W, int Ks, int Ns, const int32_t* k_idx,
              const int32_t* n_idx, int K_full, int N_full, float w_max, uint64_t step,
              const float* profile, double* U) {
  const int R = cfg->xbar_rows, C = cfg->xbar_cols;
  const int S = cfg->weight_bits / cfg->slice_bits;
  const int levels = (1 << cfg->slice_bits) - 1;
  const double g_min = 1.0 / (double)cfg->r_max;
  const double g_max = 1.0 / (double)cfg->r_min;
  const double dg = (g_max - g_min) / (double)levels;
  const uint32_t array_ni = cfg->flags & (XO_VARIATION | XO_WIRE_AAM | XO_WIRE_PROFILE | XO_WIRE_AAM2);
  /* one converter per array: the two arrays are kept apart, U[pol][s][k][n] = G_ni(pol) / dG       */
  const int per_array = (cfg->flags & XO_ADC_PER_ARRAY) != 0;
  const size_t pol_stride = (size_t)S * Ks * Ns;
  int32_t d[64];
  if (S > 64) return -1;
  if (cfg->flags & XO_WIRE_AAM2) {
    /* All first-order paths (Sec. IV-D: the analytical model extended beyond the shortest path): the voltage at a device
     * drops by the current of EVERY device on its row through the row-wire segments they share
     * with it, and rises on the column side by the current of every device on its column through
     * the shared column segments:
     *   a_ij = sum_j' G_ij' (r_source + (min(j,j') + 1) r_row)
     *   b_ij = sum_i' G_i'j ((R - max(i,i')) r_col + r_sense)
     *   G_ni = G / (1 + a + b)          (the j' = j and i' = i terms alone give the single-path model)
     * Needs whole tiles, so no sub-matrix addressing here.                                          */
    if (k_idx || n_idx || Ks != K_full || Ns != N_full) return -3;
    double* G = (double*)malloc(sizeof(double) * 2 * (size_t)R * C);
    if (!G) return -2;
    for (int s = 0; s < S; ++s)
      for (int k0 = 0; k0 < Ks; k0 += R)
        for (int n0 = 0; n0 < Ns; n0 += C) {
          const int rows = k0 + R < Ks ? R : Ks - k0, cols = n0 + C < Ns ? C : Ns - n0;
          for (int i = 0; i < rows; ++i)
            for (int j = 0; j < cols; ++j) {
              const int64_t q = xo_quantize_weight(W[(size_t)(k0 + i) * Ns + n0 + j], w_max, cfg->weight_bits);
              xo_digits((uint64_t)(q < 0 ? -q : q), cfg->slice_bits, S, d);
              double g[2];
              device_pair(cfg, (q > 0) - (q < 0), d[s], (uint64_t)(k0 + i), (uint64_t)(n0 + j), s, S, N_full, step,
                          g_min, dg, g);
              G[((size_t)0 * R + i) * C + j] = g[0];
              G[((size_t)1 * R + i) * C + j] = g[1];
            }
          for (int i = 0; i < rows; ++i)
            for (int j = 0; j < cols; ++j) {
              double e[2];
              for (int pol = 0; pol < 2; ++pol) {
                const double* Gp = G + (size_t)pol * R * C;
                double a = 0.0, b = 0.0;
                for (int jj = 0; jj < cols; ++jj)
                  a += Gp[(size_t)i * C + jj] *
                       ((double)cfg->r_source + (double)((j < jj ? j : jj) + 1) * (double)cfg->r_row);
                for (int ii = 0; ii < rows; ++ii)
                  b += Gp[(size_t)ii * C + j] *
                       ((double)(R - (i > ii ? i : ii)) * (double)cfg->r_col + (double)cfg->r_sense);
                e[pol] = Gp[(size_t)i * C + j] / (1.0 + a + b);
              }
              if (per_array) {
                U[((size_t)s * Ks + k0 + i) * Ns + n0 + j] = e[0] / dg;
                U[pol_stride + ((size_t)s * Ks + k0 + i) * Ns + n0 + j] = e[1] / dg;
              } else {
                U[((size_t)s * Ks + k0 + i) * Ns + n0 + j] = (e[0] - e[1]) / dg;
              }
            }
        }
    free(G);
    return 0;
  }
  for (int ki = 0; ki < Ks; ++ki) {
    for (int ni = 0; ni < Ns; ++ni) {
      const int64_t k = k_idx ? k_idx[ki] : ki;
      const int64_t n = n_idx ? n_idx[ni] : ni;
      const int64_t q = xo_quantize_weight(W[(size_t)ki * Ns + ni], w_max, cfg->weight_bits);
      const int sign = (q > 0) - (q < 0);
      xo_digits((uint64_t)(q < 0 ? -q : q), cfg->slice_bits, S, d);
      for (int s = 0; s < S; ++s) {
        double* out = &U[((size_t)s * Ks + ki) * Ns + ni];
        if (!array_ni && !per_array) {   /* ideal arrays: the pair difference is the digit itself */
          *out = (double)(sign * d[s]);
          continue;
        }
        double g[2];
        device_pair(cfg, sign, d[s], (uint64_t)k, (uint64_t)n, s, S, N_full, step, g_min, dg, g);
        for (int pol = 0; pol < 2; ++pol) {
          if (cfg->flags & XO_WIRE_AAM) {    /* single shortest path through device (i, j)     */
            int i = (int)(k % R), j = (int)(n % C);
            double rho = (double)cfg->r_source + (double)(j + 1) * (double)cfg->r_row +
                         (double)(R - i) * (double)cfg->r_col + (double)cfg->r_sense;
            g[pol] = g[pol] / (1.0 + rho * g[pol]);
          } else if (cfg->flags & XO_WIRE_PROFILE) {   /* stored distortion, Sec. IV-D          */
            double dist = (double)profile[(((size_t)s * 2 + pol) * K_full + k) * N_full + n];
            g[pol] = g[pol] * (1.0 - dist);
          }
        }
        if (per_array) {
          out[0] = g[0] / dg;
          out[pol_stride] = g[1] / dg;
        } else {
          *out = (g[0] - g[1]) / dg;
        }
      }
    }
  }
  return 0;
}

/* DAC of Sec. IV-B: digit of one streaming cycle -> row voltage in units of one input level. */
static double dac(const xo_config* cfg, int digit) {
  if (cfg->flags & XO_DAC_LUT) return (double)cfg->dac_lut[digit] * (double)((1 << cfg->stream_bits) - 1);
  return (double)digit;
}

/* ------------------------------------------------------------------------------------------- */
/* One VMM pass through the tiles (Sec. IV, IV-B).                                              */
/*   transposed == 0 (forward):  in[M][L_in = K], out[M][L_out = Ns]; U[s][K][Ns];             */
/*                               the contraction runs over the rows of one row tile,            */
/*                               results of the row tiles are added digitally.                  */
/*   transposed == 1 (backward): in[M][L_in = N], out[M][L_out = Ks]; U[s][Ks][N];             */
/*                               the same devices are driven from the columns, currents are     */
/*                               read on the rows, contraction over the columns of one column   */
/*                               tile, results of the column tiles are added digitally.         */
/* Every (tile, slice, cycle, phase) current gets its own ADC conversion, then shift-and-add.   */
/* codes (optional): [phase][cycle][slice][tile][m][out] as int32; acc (optional): the integer  */
/* shift-and-add result per output before the final scaling.                                    */
/* ------------------------------------------------------------------------------------------- */
static int vmm(const xo_config* cfg, const double* U, int Ks, int Ns, int transposed, const float* in,
               float* out, int M, float in_scale, float w_max, int is_signed, float adc_fs,
               int32_t* codes, int64_t* acc_out, const int64_t* wsum) {
  const int S = cfg->weight_bits / cfg->slice_bits;
  const int B = cfg->input_bits / cfg->stream_bits;
  /* signed inputs: two phases (positive parts, negative parts), or one phase of offset-binary codes */
  const int offset = is_signed && (cfg->flags & XO_INPUT_OFFSET) != 0;
  const int P = (is_signed && !offset) ? 2 : 1;
  if (offset && !wsum) return -3;
  const int L_in = transposed ? Ns : Ks;
  const int L_out = transposed ? Ks : Ns;
  const int tile = transposed ? cfg->xbar_cols : cfg->xbar_rows;
  const int T = (L_in + tile - 1) / tile;
  const int per_array = (cfg->flags & XO_ADC_PER_ARRAY) != 0;
  const int NP = per_array ? 2 : 1;
  const int64_t q_adc = per_array ? (1ll << cfg->adc_bits) - 1 : (1ll << (cfg->adc_bits - 1)) - 1;
  const double lsb = (double)adc_fs / (double)q_adc;
  const double qa = (double)((1ll << cfg->input_bits) - 1);
  const double qw = (double)((1ll << cfg->weight_bits) - 1);
  const double scale = lsb * (double)in_scale * (double)w_max / (qa * qw);
  int64_t* a = (int64_t*)malloc(sizeof(int64_t) * (size_t)L_in);
  if (!a) return -2;
  for (int m = 0; m < M; ++m) {
    for (int l = 0; l < L_in; ++l)
      a[l] = offset ? xo_quantize_input_offset(in[(size_t)m * L_in + l], in_scale, cfg->input_bits)
                    : xo_quantize_input(in[(size_t)m * L_in + l], in_scale, cfg->input_bits, is_signed);
    for (int o = 0; o < L_out; ++o) {
      int64_t acc = 0;
      for (int p = 0; p < P; ++p)
        for (int b = 0; b < B; ++b)
          for (int s = 0; s < S; ++s)
            for (int pol = 0; pol < NP; ++pol)
              for (int t = 0; t < T; ++t) {
                int l0 = t * tile, l1 = l0 + tile < L_in ? l0 + tile : L_in;
                const double* Up = U + (size_t)pol * S * Ks * Ns;
                double current = 0.0;
                for (int l = l0; l < l1; ++l) {
                  int64_t mag = p == 0 ? (a[l] > 0 ? a[l] : 0) : (a[l] < 0 ? -a[l] : 0);
                  int digit = (int)((mag >> (cfg->stream_bits * b)) & ((1 << cfg->stream_bits) - 1));
                  double u = transposed ? Up[((size_t)s * Ks + o) * Ns + l] : Up[((size_t)s * Ks + l) * Ns + o];
                  current += dac(cfg, digit) * u;
                }
                int64_t code;
                if (per_array) code = xo_adc_unsigned(current, adc_fs, cfg->adc_bits);
                else if (cfg->flags & XO_ADC_CURVE) code = xo_adc_curve(cfg->adc_curve, current, adc_fs, cfg->adc_bits);
                else code = xo_adc(current, adc_fs, cfg->adc_bits);
                if (codes)      /* [phase][cycle][slice][array][tile][m][out] */
                  codes[((((((size_t)p * B + b) * S + s) * NP + pol) * T + t) * M + m) * L_out + o] = (int32_t)code;
                int64_t weight = 1ll << (cfg->slice_bits * s + cfg->stream_bits * b);
                acc += (p == 0 ? 1 : -1) * (pol == 0 ? 1 : -1) * weight * code;
              }
      if (acc_out) acc_out[(size_t)m * L_out + o] = acc;
      if (offset) {
        /* sum_l xhat_l what_l with xhat = (2 u - Qa) / Qa * in_scale, what = q / Qw * w_max and
         * sum_l u_l q_l read from the converters as acc * lsb: twice the converted sum minus the
         * half-range times the weight sum, which the digital side knows                            */
        const double half_range = (double)in_scale * (double)w_max / qw;
        out[(size_t)m * L_out + o] = (float)((double)acc * (2.0 * scale) - (double)wsum[o] * half_range);
      } else {
        out[(size_t)m * L_out + o] = (float)((double)acc * scale);
      }
    }
  }
  free(a);
  return 0;
}

/* wsum: with XO_INPUT_OFFSET the weight sums of xo_weight_sums (colsum for the forward, rowsum for
 * the backward pass), else unused.                                                               */
int xo_fwd_planes(const xo_config* cfg, const double* U, const float* X, float* Y, int M, int K, int Ns,
                  float w_max, float x_scale, int32_t* codes, int64_t* acc, const int64_t* wsum) {
  return vmm(cfg, U, K, Ns, 0, X, Y, M, x_scale, w_max, (cfg->flags & XO_INPUT_SIGNED) != 0,
             cfg->adc_fs_fwd, codes, acc, wsum);
}

int xo_bwd_planes(const xo_config* cfg, const double* U, const float* dY, float* dX, int M, int Ks, int N,
                  float w_max, float g_scale, int32_t* codes, int64_t* acc, const int64_t* wsum) {
  return vmm(cfg, U, Ks, N, 1, dY, dX, M, g_scale, w_max, 1, cfg->adc_fs_bwd, codes, acc, wsum);
}

/* Plane values of a whole layer: one per (slice, weight), two with one converter per array. */
static size_t layer_plane_count(const xo_config* cfg, int K, int N) {
  return (size_t)((cfg->flags & XO_ADC_PER_ARRAY) ? 2 : 1) * (size_t)(cfg->weight_bits / cfg->slice_bits) * K * N;
}

/* Forward VMM of a whole layer: Y[M][N] from W[K][N] and X[M][K]. */
int xo_fwd(const xo_config* cfg, const float* W, const float* X, float* Y, int M, int K, int N, float w_max,
           float x_scale, uint64_t step, const float* profile, int32_t* codes, int64_t* acc) {
  double* U = (double*)malloc(sizeof(double) * layer_plane_count(cfg, K, N));
  int64_t* sums = (int64_t*)malloc(sizeof(int64_t) * ((size_t)K + N));
  int rc = (U && sums) ? 0 : -2;
  if (!rc) rc = xo_planes(cfg, W, K, N, NULL, NULL, K, N, w_max, step, profile, U);
  if (!rc) rc = xo_weight_sums(cfg, W, K, N, w_max, sums, sums + N);
  if (!rc) rc = xo_fwd_planes(cfg, U, X, Y, M, K, N, w_max, x_scale, codes, acc, sums);
  free(U);
  free(sums);
  return rc;
}

/* Backward VMM of a whole layer: dX[M][K] from W[K][N] and dY[M][N], same device draw as the
 * forward pass of the same step.                                                               */
int xo_bwd(const xo_config* cfg, const float* W, const float* dY, float* dX, int M, int K, int N, float w_max,
           float g_scale, uint64_t step, const float* profile, int32_t* codes, int64_t* acc) {
  double* U = (double*)malloc(sizeof(double) * layer_plane_count(cfg, K, N));
  int64_t* sums = (int64_t*)malloc(sizeof(int64_t) * ((size_t)K + N));
  int rc = (U && sums) ? 0 : -2;
  if (!rc) rc = xo_planes(cfg, W, K, N, NULL, NULL, K, N, w_max, step, profile, U);
  if (!rc) rc = xo_weight_sums(cfg, W, K, N, w_max, sums, sums + N);
  if (!rc) rc = xo_bwd_planes(cfg, U, dY, dX, M, K, N, w_max, g_scale, codes, acc, sums + N);
  free(U);
  free(sums);
  return rc;
}

/* ------------------------------------------------------------------------------------------- */
/* Update model (Sec. IV-C).  W[Ks][Ns] in place; X[M][Ks], dY[M][Ns] hold the columns of the   */
/* activations / errors that belong to the weights at absolute (k_idx, n_idx) of a layer with   */
/* N_full columns (NULL = identity).  grad (optional) receives sum_m X dY.                     */
/*                                                                                               */
/* Readings: the differential pair is one effective device with normalised state                 */
/* g = W / w_max in [-1, 1], x = (g + 1) / 2; all conductance changes are in units of            */
/* (Gmax - Gmin).  delta = grad_scale * grad is the ideal change.  The written change is         */
/* delta * exp(-v x) when the conductance goes up and delta * exp(-v (1 - x)) when it goes down  */
/* (direction = sign of -lr * delta): saturating, asymmetric, equal to the ideal change at v = 0.*/
/* Write noise: Gaussian, sigma = gamma * sqrt(|delta|) in the same units, added before the      */
/* learning rate.  The state is clamped to the device range afterwards.                          */
/* ------------------------------------------------------------------------------------------- */
int xo_update(const xo_config* cfg, float* W, const float* X, const float* dY, int M, int Ks, int Ns,
              const int32_t* k_idx, const int32_t* n_idx, int N_full, float w_max, float grad_scale, float lr,
              uint64_t step, double* grad_out) {
  for (int ki = 0; ki < Ks; ++ki)
    for (int ni = 0; ni < Ns; ++ni) {
      double grad = 0.0;
      for (int m = 0; m < M; ++m) grad += (double)X[(size_t)m * Ks + ki] * (double)dY[(size_t)m * Ns + ni];
      if (grad_out) grad_out[(size_t)ki * Ns + ni] = grad;
      const uint64_t k = k_idx ? (uint64_t)k_idx[ki] : (uint64_t)ki;
      const uint64_t n = n_idx ? (uint64_t)n_idx[ni] : (uint64_t)ni;
      const double g = (double)W[(size_t)ki * Ns + ni] / (double)w_max;
      const double delta = (double)grad_scale * grad;
      double written = delta;
      if (cfg->flags & XO_UPD_NL) {
        double x = clampd(0.5 * (g + 1.0), 0.0, 1.0);
        double change = -(double)lr * delta;
        if (change > 0.0) written = delta * exp(-(double)cfg->upd_nl_v * x);
        else if (change < 0.0) written = delta * exp(-(double)cfg->upd_nl_v * (1.0 - x));
      }
      if (cfg->flags & XO_UPD_NOISE) {
        double sigma = (double)cfg->upd_noise_gamma * sqrt(fabs(delta));
        written += sigma * xo_normal(cfg->seed, XO_STREAM_WRITE, step, k * (uint64_t)N_full + n);
      }
      const double g_new = clampd(g - (double)lr * written, -1.0, 1.0);
      W[(size_t)ki * Ns + ni] = (float)((double)w_max * g_new);
    }
  return 0;
}

/* ------------------------------------------------------------------------------------------- */
/* Update with per-polarity device state.  The aggregate model above treats the positive and the  */
/* negative device of a weight as ONE effective device (Sec. IV-C speaks of "the" conductance G of  */
/* a weight).  This variant keeps both conductances of the pair (Sec. IV-A: positive and negative   */
/* conductances in two arrays whose currents are subtracted) as states of their own, gp and gn in   */
/* [0, 1] (units of Gmax - Gmin above Gmin), with W = w_max (gp - gn).                               */
/* Reading (the paper gives no rule for how a write is shared by the pair): the ideal change is     */
/* split evenly and applied in opposite directions, gp <- gp - lr w_p, gn <- gn + lr w_n, where each */
/* device sees half the ideal change delta / 2, scaled by the write non-linearity at ITS OWN state   */
/* and direction (exp(-v g) when it rises, exp(-v (1 - g)) when it falls) and with a noise draw of   */
/* its own, sigma = gamma sqrt(|delta| / 2) (the two variances add up to the effective device's      */
/* gamma^2 |delta|); each device is clamped to [0, 1] on its own.  Normal number 2 (k N + n) + pol   */
/* of stream 6.  With v = gamma = 0 and no device at a rail the pair's difference moves exactly as   */
/* the effective device does.  xo_pair_init places a weight symmetrically about mid-range:           */
/* gp = (1 + g) / 2, gn = (1 - g) / 2, g = clamp(W / w_max, -1, 1).                                  */
/* ------------------------------------------------------------------------------------------- */
void xo_pair_init(const float* W, float* Gp, float* Gn, size_t count, float w_max) {
  for (size_t i = 0; i < count; ++i) {
    const double g = clampd((double)W[i] / (double)w_max, -1.0, 1.0);
    Gp[i] = (float)(0.5 * (1.0 + g));
    Gn[i] = (float)(0.5 * (1.0 - g));
  }
}

int xo_update_pair(const xo_config* cfg, float* Gp, float* Gn, float* W, const float* X, const float* dY, int M, int K,
                   int N, float w_max, float grad_scale, float lr, uint64_t step) {
  for (int k = 0; k < K; ++k)
    for (int n = 0; n < N; ++n) {
      double grad = 0.0;
      for (int m = 0; m < M; ++m) grad += (double)X[(size_t)m * K + k] * (double)dY[(size_t)m * N + n];
      const size_t at = (size_t)k * N + n;
      const double delta = (double)grad_scale * grad;
      double state[2] = {(double)Gp[at], (double)Gn[at]};
      for (int pol = 0; pol < 2; ++pol) {
        const double half = 0.5 * delta;
        /* the weight falls when lr delta > 0: then the positive device falls and the negative one rises */
        const double change = (pol == 0 ? -1.0 : 1.0) * (double)lr * half;
        double written = half;
        if (cfg->flags & XO_UPD_NL) {
          const double x = clampd(state[pol], 0.0, 1.0);
          if (change > 0.0) written = half * exp(-(double)cfg->upd_nl_v * x);
          else if (change < 0.0) written = half * exp(-(double)cfg->upd_nl_v * (1.0 - x));
        }
        if (cfg->flags & XO_UPD_NOISE)
          written += (double)cfg->upd_noise_gamma * sqrt(fabs(half)) *
                     xo_normal(cfg->seed, XO_STREAM_WRITE_PAIR, step, 2 * (uint64_t)at + (uint64_t)pol);
        state[pol] = clampd(state[pol] + (pol == 0 ? -1.0 : 1.0) * (double)lr * written, 0.0, 1.0);
      }
      Gp[at] = (float)state[0];
      Gn[at] = (float)state[1];
      W[at] = (float)((double)w_max * ((double)Gp[at] - (double)Gn[at]));
    }
  return 0;
}

/* ------------------------------------------------------------------------------------------- */
/* Pulse-level update (Sec. IV-C names the parallel update schemes whose result the aggregate    */
/* model above describes; this is the stochastic bit-stream scheme of its reference [ibm_RPU]):  */
/* every sample m applies its inputs to the rows and its errors to the columns as random pulse  */
/* trains of `bl` slots; a device is pulsed once in every slot in which its row and its column  */
/* both fire.  A value fires with probability p = min(1, |value| / range) per slot, so the       */
/* expected number of pulses is bl p_x p_d, proportional to the product: the outer-product       */
/* update, one sample at a time, without ever forming the gradient.                              */
/*                                                                                               */
/* Readings: slot j of element `index` fires when uniform 32-bit word j of the element's Philox   */
/* blocks (block index*8 + j/4, word j%4, streams 3 / 4 for rows / columns) is below             */
/* rne(p 2^32).  A pulse moves the state g = W / w_max by dw_min against the sign of x d         */
/* (descent); with XO_UPD_NL the move is scaled by exp(-v x) going up and exp(-v (1 - x)) going   */
/* down, x = (g + 1) / 2, evaluated at the state the pulse finds.  With XO_UPD_NOISE every pulse   */
/* carries the noise the aggregate model gives it: there the standard deviation gamma sqrt(dG)   */
/* belongs to the ideal change BEFORE the learning rate (Sec. IV-C), and the mean written change  */
/* of this scheme equals the aggregate update at the learning rate                                */
/* lr = bl dw_min w_max / (x_range d_range); one pulse is the ideal change dw_min / lr, its noise  */
/* after the learning rate lr gamma sqrt(dw_min / lr) = gamma sqrt(lr dw_min), times a normal     */
/* number (number m*32 + j of stream 5 keyed with step*2^31 + device index).  The state is        */
/* clamped to [-1, 1] after every pulse.  Samples in order, devices independent.                  */
/*                                                                                               */
/* XO_PULSE_CODED: the deterministic alternative the same passage names (values coded in the      */
/* timing of the pulses instead of random streams).  Reading: the bl slots form Tx frames of Td    */
/* sub-slots, Tx = floor(sqrt(bl)), Td = floor(bl / Tx) (slots beyond Tx Td stay unused); a row     */
/* holds its line for the first nx = rne(p_x Tx) frames (pulse duration codes |x|), a column fires  */
/* in the first nd = rne(p_d Td) sub-slots of every frame (pulse count per frame codes |d|): the     */
/* device sees exactly nx nd coincidences, the product of the two coded values.  Everything else    */
/* (pulse size, device model, order) as above, with Tx Td in place of bl in the learning rate.       */
/*                                                                                                   */
/* XO_PULSE_MAGNITUDE: values coded in the magnitude of ONE pulse per sample (the other coding the   */
/* passage names).  Reading: a row carries a pulse of height lx = rne(p_x bl) out of bl levels, a     */
/* column one of height ld = rne(p_d bl); the device answers the product of the two heights: one      */
/* write of lx ld quanta of dw_min (a full-scale pair writes bl^2 dw_min, so bl^2 takes the place of  */
/* bl in the learning rate), against the sign of x d.  It is ONE write: the non-linearity is          */
/* evaluated once, at the state the write finds, and scales all of it; the noise is one draw with     */
/* the standard deviation the aggregate model gives a change of that size, gamma sqrt(lr lx ld        */
/* dw_min) (normal number m * 32 of the device's stream); one clamp.  The reported pulse count of a    */
/* device is its signed number of quanta.                                                              */
/* ------------------------------------------------------------------------------------------- */
void xo_pulse_frames(int bl, int* tx, int* td) {
  int t = 1;
  while ((t + 1) * (t + 1) <= bl) ++t;
  *tx = t;
  *td = bl / t;
}

/* Slot j = frame * Td + sub-slot.  is_col = 0: frames 0 .. nx-1 entirely; 1: sub-slots 0 .. nd-1 of every frame. */
uint32_t xo_pulse_code(double p, int bl, int is_col) {
  int tx, td;
  xo_pulse_frames(bl, &tx, &td);
  const int level = (int)rint(clampd(p, 0.0, 1.0) * (double)(is_col ? td : tx));
  uint32_t bits = 0;
  for (int frame = 0; frame < tx; ++frame)
    for (int sub = 0; sub < td; ++sub)
      if (is_col ? sub < level : frame < level) bits |= 1u << (frame * td + sub);
  return bits;
}

uint32_t xo_pulse_train(uint64_t seed, uint32_t stream, uint64_t step, uint64_t index, double p, int bl) {
  const uint32_t key[2] = {(uint32_t)seed ^ (0x9E3779B9u * stream), (uint32_t)(seed >> 32) ^ (0xBB67AE85u * stream)};
  const uint64_t threshold = (uint64_t)rint(clampd(p, 0.0, 1.0) * 4294967296.0);
  uint32_t bits = 0;
  for (int j = 0; j < bl; j += 4) {
    const uint64_t blk = index * 8 + (uint64_t)(j >> 2);
    const uint32_t ctr[4] = {(uint32_t)blk, (uint32_t)(blk >> 32), (uint32_t)step, (uint32_t)(step >> 32)};
    uint32_t w[4];
    xo_philox4x32_10(ctr, key, w);
    for (int e = 0; e < 4 && j + e < bl; ++e)
      if ((uint64_t)w[e] < threshold) bits |= 1u << (j + e);
  }
  return bits;
}

/* Sampled form: W[K][N], X[M][K], dY[M][N] are the devices at absolute rows k_idx[] and columns n_idx[]  */
/* of a layer with K_full x N_full devices (NULL: the layer itself); devices are independent, so the    */
/* sampled ones end exactly where they end in the whole layer.                                          */
int xo_update_pulsed_at(const xo_config* cfg, float* W, const float* X, const float* dY, int M, int K, int N,
                        const int32_t* k_idx, const int32_t* n_idx, int K_full, int N_full,
                        float w_max, float x_range, float d_range, int bl, float dw_min, uint64_t step,
                        int64_t* pulses_out) {
  if (bl < 1 || bl > 31 || M <= 0 || K <= 0 || N <= 0 || K_full < K || N_full < N) return -1;
  double* g = (double*)malloc(sizeof(double) * (size_t)K * N);
  uint32_t* a = (uint32_t*)malloc(sizeof(uint32_t) * ((size_t)K + N));
  if (!g || !a) { free(g); free(a); return -2; }
  uint32_t* b = a + K;
  for (size_t i = 0; i < (size_t)K * N; ++i) g[i] = (double)W[i] / (double)w_max;
  if (pulses_out) memset(pulses_out, 0, sizeof(int64_t) * (size_t)K * N);
  const int coded = (cfg->flags & XO_PULSE_CODED) != 0;
  const int magnitude = (cfg->flags & XO_PULSE_MAGNITUDE) != 0;
  if (coded && magnitude) { free(g); free(a); return -1; }
  int slots = bl;
  if (coded) {
    int tx, td;
    xo_pulse_frames(bl, &tx, &td);
    slots = tx * td;
  }
  if (magnitude) slots = bl * bl;
  const double lr_eq = (double)slots * (double)dw_min * (double)w_max / ((double)x_range * (double)d_range);
  const double sigma = (double)cfg->upd_noise_gamma * sqrt(lr_eq * (double)dw_min);
  for (int m = 0; m < M; ++m) {
    /* bit 31 of a train carries the sign of its value */
    for (int k = 0; k < K; ++k) {
      const double x = (double)X[(size_t)m * K + k];
      const uint64_t kf = k_idx ? (uint64_t)k_idx[k] : (uint64_t)k;
      if (magnitude) a[k] = (uint32_t)rint(clampd(fabs(x) / (double)x_range, 0.0, 1.0) * (double)bl) | (x < 0.0 ? 0x80000000u : 0u);
      else
      a[k] = (coded ? xo_pulse_code(fabs(x) / (double)x_range, bl, 0)
                    : xo_pulse_train(cfg->seed, XO_STREAM_PULSE_ROWS, step, (uint64_t)m * K_full + kf, fabs(x) / (double)x_range, bl)) |
             (x < 0.0 ? 0x80000000u : 0u);
    }
    for (int n = 0; n < N; ++n) {
      const double d = (double)dY[(size_t)m * N + n];
      const uint64_t nf = n_idx ? (uint64_t)n_idx[n] : (uint64_t)n;
      if (magnitude) b[n] = (uint32_t)rint(clampd(fabs(d) / (double)d_range, 0.0, 1.0) * (double)bl) | (d < 0.0 ? 0x80000000u : 0u);
      else
      b[n] = (coded ? xo_pulse_code(fabs(d) / (double)d_range, bl, 1)
                    : xo_pulse_train(cfg->seed, XO_STREAM_PULSE_COLS, step, (uint64_t)m * N_full + nf, fabs(d) / (double)d_range, bl)) |
             (d < 0.0 ? 0x80000000u : 0u);
    }
    for (int k = 0; k < K; ++k)
      for (int n = 0; n < N; ++n) {
        const double dir = ((a[k] ^ b[n]) & 0x80000000u) ? 1.0 : -1.0;   /* against the sign of x d */
        const uint64_t dev = (k_idx ? (uint64_t)k_idx[k] : (uint64_t)k) * (uint64_t)N_full + (n_idx ? (uint64_t)n_idx[n] : (uint64_t)n);
        double* gs = &g[(size_t)k * N + n];
        if (magnitude) {                                                  /* one write of lx ld quanta */
          const int quanta = (int)(a[k] & 0x7FFFFFFFu) * (int)(b[n] & 0x7FFFFFFFu);
          if (!quanta) continue;
          double move = (double)dw_min * (double)quanta;
          if (cfg->flags & XO_UPD_NL) {
            const double x = clampd(0.5 * (*gs + 1.0), 0.0, 1.0);
            move *= dir > 0.0 ? exp(-(double)cfg->upd_nl_v * x) : exp(-(double)cfg->upd_nl_v * (1.0 - x));
          }
          double next = *gs + dir * move;
          if (cfg->flags & XO_UPD_NOISE)
            next += sigma * sqrt((double)quanta) * xo_normal(cfg->seed, XO_STREAM_PULSE_NOISE, (step << 31) | dev, (uint64_t)m * 32);
          *gs = clampd(next, -1.0, 1.0);
          if (pulses_out) pulses_out[(size_t)k * N + n] += (dir > 0.0 ? 1 : -1) * quanta;
          continue;
        }
        const uint32_t both = a[k] & b[n] & 0x7FFFFFFFu;
        if (!both) continue;
        int count = 0;
        for (uint32_t v = both; v; v &= v - 1) ++count;
        for (int j = 0; j < count; ++j) {
          double move = (double)dw_min;
          if (cfg->flags & XO_UPD_NL) {
            const double x = clampd(0.5 * (*gs + 1.0), 0.0, 1.0);
            move *= dir > 0.0 ? exp(-(double)cfg->upd_nl_v * x) : exp(-(double)cfg->upd_nl_v * (1.0 - x));
          }
          double next = *gs + dir * move;
          if (cfg->flags & XO_UPD_NOISE)
            next += sigma * xo_normal(cfg->seed, XO_STREAM_PULSE_NOISE, (step << 31) | dev, (uint64_t)m * 32 + j);
          *gs = clampd(next, -1.0, 1.0);
        }
        if (pulses_out) pulses_out[(size_t)k * N + n] += (dir > 0.0 ? 1 : -1) * count;
      }
  }
  for (size_t i = 0; i < (size_t)K * N; ++i) W[i] = (float)((double)w_max * g[i]);
  free(g);
  free(a);
  return 0;
}

int xo_update_pulsed(const xo_config* cfg, float* W, const float* X, const float* dY, int M, int K, int N,
                     float w_max, float x_range, float d_range, int bl, float dw_min, uint64_t step,
                     int64_t* pulses_out) {
  return xo_update_pulsed_at(cfg, W, X, dY, M, K, N, NULL, NULL, K, N, w_max, x_range, d_range, bl, dw_min, step, pulses_out);
}

unsigned xo_config_size(void) { return (unsigned)sizeof(xo_config); }
