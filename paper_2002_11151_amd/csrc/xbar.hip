// xbar: emulation of non-ideal resistive-crossbar training operations on MI355X (gfx950).
// HIP kernels and the C-ABI entry points declared in include/xbar.h.
//
// Method: TxSim (arXiv 2002.11151) Sec. IV (DAC -> array -> ADC per layer, forward and backward),
// Sec. IV-A (non-ideal conductance matrix generator), Sec. IV-C (update model), Sec. IV-D
// (approximate analytical wire model / stored distortion profile).
//
// Kernel plan
//   tile_planes     weights -> quantise -> bit slices -> device conductances -> variation -> wire model
//                   -> stitched signed planes U, written as fp16 MFMA B-operand fragments
//                   (one term when U is an exact digit, hi + lo terms when U is a real number)
//   quantize_input  activations / errors -> integer magnitudes, written as MFMA A-operand fragments
//                   that keep the raw 8-bit magnitude in each 16-bit lane
//   vmm             per (tile, slice, cycle, phase): MFMA contraction (fp16 operands, fp32
//                   accumulate) + ADC + shift-and-add fused in registers
//   vmm_finish      sum of the integer partial results over tile chunks -> scaled fp32 output
//   grad_gemm       X^T dY with fp32 MFMA, split over the batch
//   update_write    batch-partial sum -> non-linear, noisy conductance write, in place
//
// Operand trick of vmm: a 16-bit lane that holds the integer field `digit << shift` (shift < 10) is,
// read as fp16, the subnormal number digit * 2^(shift-24).  The matrix cores of gfx950 take fp16
// subnormals exactly, so one AND with a digit mask turns the raw magnitudes into the A operand of
// any streaming cycle; the power of two is folded into the ADC gain.
//
// Cycles of 1 or 2 bits (the paper's streaming scheme) run on the block-scaled 6-bit / 4-bit matrix
// instruction instead (v_mfma_scale_f32_32x32x64_f8f6f4: 64 rows per instruction in the time fp16 takes
// for 16): a digit d is the E2M1 code d (value d / 2), a plane value is a sum of E2M3 numbers times
// powers of two that the instruction applies as block scales (xbar_common.h), accumulated in fp32 with
// the leading term first.
#include "xbar_common.h"

using namespace xbar_detail;

namespace {

// ---------------------------------------------------------------------------------------------
// generator: weights -> operand planes (Sec. IV-A, IV-D)
// ---------------------------------------------------------------------------------------------
struct TileArgs {
  const float* W;
  const float* profile;
  const double* wire_u;  // all-paths wire model: plane values [S_w][2][K][N], array index 0 (else unused)
  uint16_t* planes;  // start of this copy
  int K, N, R, C, S_w, slice_bits, weight_bits, terms;
  int tile, ks, T, OP;
  int pol_out;       // -1: difference of the pair (array 0 minus array 1); 0 / 1: that array alone
  uint32_t flags;
  double g_min, dg, var_sigma, r_row, r_col, r_source, r_sense, hi_scale, hi_inv_scale;
  float w_max;
  uint64_t seed, step;
  const unsigned long long* step_add;   // optional device counter added to step
  long long n_threads;
  int term_exp[kMaxTermsF6];            // kFmtF6: power of two of every term
};

// Plane value of slice s of weight (k, n), in units of one device level: the signed difference of the
// device pair, or the conductance of one of the two devices.
__device__ __forceinline__ double plane_value(const TileArgs& a, NormalStream& rng, int sign, int digit, int s, int k,
                                              int n) {
  if (a.flags & XBAR_NI_WIRE_AAM2) return a.wire_u[((size_t)(2 * s + (a.pol_out > 0 ? 1 : 0)) * a.K + k) * a.N + n];
  if (a.pol_out < 0 && !(a.flags & (XBAR_NI_VARIATION | XBAR_NI_WIRE_AAM | XBAR_NI_WIRE_PROFILE)))
    return (double)(sign * digit);
  double g[2];
  g[0] = a.g_min + (sign > 0 ? digit * a.dg : 0.0);
  g[1] = a.g_min + (sign < 0 ? digit * a.dg : 0.0);
#pragma unroll
  for (int pol = 0; pol < 2; ++pol) {
    if (a.flags & XBAR_NI_VARIATION) {
      const uint64_t dev = (((uint64_t)k * (uint64_t)a.N + (uint64_t)n) * (uint64_t)a.S_w + (uint64_t)s) * 2 + pol;
      g[pol] *= 1.0 + a.var_sigma * rng.get(dev);
    }
    if (a.flags & XBAR_NI_WIRE_AAM) {
      const int i = k % a.R, j = n % a.C;
      const double rho = a.r_source + (double)(j + 1) * a.r_row + (double)(a.R - i) * a.r_col + a.r_sense;
      g[pol] = g[pol] / (1.0 + rho * g[pol]);
    } else if (a.flags & XBAR_NI_WIRE_PROFILE) {
      const double dist = (double)a.profile[(((size_t)s * 2 + pol) * a.K + k) * a.N + n];
      g[pol] = g[pol] * (1.0 - dist);
    }
  }
  return (a.pol_out < 0 ? g[0] - g[1] : g[a.pol_out]) / a.dg;
}

// One thread produces the 8 consecutive contraction-index entries of one output column that make up
// one 16-byte operand chunk of one slice (blockIdx.y), for every term.
//   TRANSPOSED = false: contraction index k (rows), output index n;  = true: contraction n, output k.
template <bool TRANSPOSED>
__global__ __launch_bounds__(256) void tile_planes_kernel(TileArgs a) {
  const long long tid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (tid >= a.n_threads) return;
  // thread -> (chunk of 8 along the contraction, output index); output index fastest within 32
  const int out_len_pad = a.OP * 32;
  const int o = (int)(tid % out_len_pad);
  const int cg = (int)(tid / out_len_pad);        // global 8-chunk along the contraction
  const int c0 = cg * 8;
  const int t = c0 / a.tile;
  const int within = c0 - t * a.tile;
  const int j = within / 16, half = (within % 16) / 8;
  const int lane = (o % 32) + 32 * half;
  const int op = o / 32;
  const int Lc = TRANSPOSED ? a.N : a.K;          // contraction length
  const int Lo = TRANSPOSED ? a.K : a.N;

  NormalStream rng(a.seed, kStreamVariation, effective_step(a.step, a.step_add));
  const double qw = (double)((1u << a.weight_bits) - 1);
  const uint32_t dmask = (1u << a.slice_bits) - 1;

  int sign[8];
  uint32_t mag[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int c = c0 + e;
    sign[e] = 0;
    mag[e] = 0;
    if (c < Lc && o < Lo) {
      const int k = TRANSPOSED ? o : c, n = TRANSPOSED ? c : o;
      const double q = ::rint(clampd((double)a.W[(size_t)k * a.N + n] / (double)a.w_max, -1.0, 1.0) * qw);
      sign[e] = (q > 0.0) - (q < 0.0);
      mag[e] = (uint32_t)::fabs(q);
    }
  }
  const size_t blk0 = ((size_t)t * a.OP + op) * a.S_w;
  const int s = blockIdx.y;                         // one slice per grid row: short serial chains
  union { u32x4 v; _Float16 h[8]; } hi, lo;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int c = c0 + e;
    double u = 0.0;
    if (c < Lc && o < Lo) {
      const int k = TRANSPOSED ? o : c, n = TRANSPOSED ? c : o;
      u = plane_value(a, rng, sign[e], (int)((mag[e] >> (a.slice_bits * s)) & dmask), s, k, n);
    }
    // leading term on the grid 2^-hi_frac (coarser where fp16 cannot hold it), residual in fp16
    const _Float16 h = a.terms == 2 ? (_Float16)(::rint(u * a.hi_scale) * a.hi_inv_scale) : (_Float16)u;
    hi.h[e] = h;
    lo.h[e] = (_Float16)(u - (double)h);
  }
  const size_t chunk = ((blk0 + s) * a.terms * a.ks + j) * 64 + lane;   // in 16-byte units
  reinterpret_cast<u32x4*>(a.planes)[chunk] = hi.v;
  if (a.terms == 2) reinterpret_cast<u32x4*>(a.planes)[chunk + (size_t)a.ks * 64] = lo.v;
}

// E2M3 number (1 sign, 2 exponent, 3 mantissa bits, bias 1: multiples of 1/8 up to 2, of 1/4 up to 4, of
// 1/2 up to 7.5) nearest to x; returns its 6-bit code and the number itself.
__device__ __forceinline__ uint32_t e2m3_nearest(double x, double& value) {
  const double a = ::fabs(x);
  uint32_t code;
  double v;
  if (a < 2.0) {
    const double k = ::rint(a * 8.0);                 // 0 .. 16; codes continue linearly into the next binade
    code = (uint32_t)k;
    v = k * 0.125;
  } else if (a < 4.0) {
    const double k = ::rint(a * 4.0);                 // 8 .. 16
    code = 8u + (uint32_t)k;
    v = k * 0.25;
  } else {
    const double k = ::fmin(::rint(a * 2.0), 15.0);   // 8 .. 15: 7.5 is the largest number
    code = 16u + (uint32_t)k;
    v = k * 0.5;
  }
  if (x < 0.0 && code) {
    code |= 32u;
    v = -v;
  }
  value = v;
  return code;
}

// Planes in the 6-bit format: one thread produces the 8 contraction entries (48 bits per term) that one
// byte pair group of the input stage covers, for one output column and one slice (blockIdx.y).
// Thread -> (output index fastest, then the 8-entry slot of the tile, then the tile); slots of k-steps
// that the tile does not reach are skipped, slots beyond its rows inside a k-step are written as zeros.
template <bool TRANSPOSED>
__global__ __launch_bounds__(256) void tile_planes_f6_kernel(TileArgs a) {
  const long long tid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (tid >= a.n_threads) return;
  const int out_len_pad = a.OP * 32;
  const int o = (int)(tid % out_len_pad);
  const int cg = (int)(tid / out_len_pad);
  const int slots = a.ks * 8;                       // 8-entry slots per tile (whole k-steps of 64)
  const int t = cg / slots, slot = cg - t * slots;
  const int within = slot * 8;
  const int Lc = TRANSPOSED ? a.N : a.K;
  const int Lo = TRANSPOSED ? a.K : a.N;
  const int rows = min(a.tile, Lc - t * a.tile);
  const int J = within >> 6;
  if (J * 64 >= rows) return;                       // the contraction never reads this k-step
  const int w = (within & 63) >> 4, half = (within & 15) >> 3;
  const int lane = (o & 31) + 32 * half;
  const int op = o >> 5;
  const int c0 = t * a.tile + within;
  const int s = blockIdx.y;

  NormalStream rng(a.seed, kStreamVariation, effective_step(a.step, a.step_add));
  const double qw = (double)((1u << a.weight_bits) - 1);
  const uint32_t dmask = (1u << a.slice_bits) - 1;
  unsigned long long bits[kMaxTermsF6];
#pragma unroll
  for (int j = 0; j < kMaxTermsF6; ++j) bits[j] = 0ull;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int c = c0 + e;
    if (within + e >= rows || o >= Lo) continue;
    const int k = TRANSPOSED ? o : c, n = TRANSPOSED ? c : o;
    const double q = ::rint(clampd((double)a.W[(size_t)k * a.N + n] / (double)a.w_max, -1.0, 1.0) * qw);
    const int sign = (q > 0.0) - (q < 0.0);
    const uint32_t mag = (uint32_t)::fabs(q);
    double left = plane_value(a, rng, sign, (int)((mag >> (a.slice_bits * s)) & dmask), s, k, n);
    const int nibble = 2 * (e & 3) + (e >> 2);       // where the input stage's byte e lands in the digit word
#pragma unroll
    for (int j = 0; j < kMaxTermsF6; ++j) {
      if (j >= a.terms) break;
      double v;
      const uint32_t code = e2m3_nearest(::ldexp(left, -a.term_exp[j]), v);
      left -= ::ldexp(v, a.term_exp[j]);
      bits[j] |= (unsigned long long)code << (6 * nibble);
    }
  }
  // 24-byte record of the lane: bytes 0..15 in the fragment's first KiB, 16..23 in its last half KiB
  const size_t frag0 = (((size_t)t * a.OP + op) * a.S_w + s) * a.terms * a.ks + J;
  uint8_t* base = reinterpret_cast<uint8_t*>(a.planes);
#pragma unroll
  for (int j = 0; j < kMaxTermsF6; ++j) {
    if (j >= a.terms) break;
    uint8_t* frag = base + (frag0 + (size_t)j * a.ks) * 1536;
#pragma unroll
    for (int h = 0; h < 3; ++h) {
      const int off = 6 * w + 2 * h;
      uint8_t* dst = off < 16 ? frag + lane * 16 + off : frag + 1024 + lane * 8 + (off - 16);
      *reinterpret_cast<uint16_t*>(dst) = (uint16_t)(bits[j] >> (16 * h));
    }
  }
}


// ---------------------------------------------------------------------------------------------
// sums of the quantised weights over rows and columns: what the digital correction of offset-binary
// inputs multiplies the half-range with (the digital side knows the programmed weights)
// ---------------------------------------------------------------------------------------------
struct SumArgs {
  const float* W;
  long long* colsum;   // [N] sum over k
  long long* rowsum;   // [K] sum over n
  int K, N, weight_bits;
  float w_max;
};

__global__ __launch_bounds__(256) void clear_sums_kernel(SumArgs a) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < a.N) a.colsum[i] = 0;
  if (i < a.K) a.rowsum[i] = 0;
}

// Block = 64 rows x 64 columns; wave w takes rows w, w + 4, ..: lane = column.  Integer atomics: the
// result does not depend on the order.
__global__ __launch_bounds__(256) void weight_sums_kernel(SumArgs a) {
  const int nb = (a.N + 63) / 64;
  const int k0 = (blockIdx.x / nb) * 64, n = (blockIdx.x % nb) * 64 + (threadIdx.x & 63);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const double qw = (double)((1u << a.weight_bits) - 1);
  long long col = 0;
  for (int k = k0 + wave; k < min(k0 + 64, a.K); k += 4) {
    long long q = 0;
    if (n < a.N) q = (long long)::rint(clampd((double)a.W[(size_t)k * a.N + n] / (double)a.w_max, -1.0, 1.0) * qw);
    col += q;
    long long r = q;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) r += __shfl_xor(r, d, 64);
    if (lane == 0) atomicAdd(reinterpret_cast<unsigned long long*>(&a.rowsum[k]), (unsigned long long)r);
  }
  if (n < a.N) atomicAdd(reinterpret_cast<unsigned long long*>(&a.colsum[n]), (unsigned long long)col);
}

// ---------------------------------------------------------------------------------------------
// input quantiser (Sec. IV: inputs are scaled and sent to the DAC)
// ---------------------------------------------------------------------------------------------
struct QuantArgs {
  const float* X;
  uint8_t* A;        // [phase][MP][T][ks][64 lanes][8 bytes]
  int M, L, MP, T, ks, tile, P, input_bits;
  int offset;        // signed inputs as offset-binary codes in one phase (P == 1)
  float scale;
  long long n_threads;
  ConvGeom conv;     // used by the CONV instantiation only
};

template <bool CONV>
__global__ __launch_bounds__(256) void quantize_input_kernel(QuantArgs a) {
  const long long tid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (tid >= a.n_threads) return;
  // one wave = 32 rows x one pair of k-steps (32 consecutive inputs of a row = one 128-byte line)
  const int lane = (int)(tid & 63);
  const long long wv = tid >> 6;                    // (mp, t, jp)
  const int npair = (a.ks + 1) >> 1;
  const int jp = (int)(wv % npair);
  const int t = (int)((wv / npair) % a.T);
  const int mp = (int)(wv / ((long long)npair * a.T));
  const int m = mp * 32 + (lane & 31);
  const double qa = (double)((1u << a.input_bits) - 1);
  const double lo = a.P == 2 ? -1.0 : 0.0;
  const double scale = (double)a.scale;
  u32x2* out = reinterpret_cast<u32x2*>(a.A);
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int j = 2 * jp + h;
    if (j >= a.ks) break;
    const int l0 = t * a.tile + j * 16 + (lane >> 5) * 8;
    const int lend = min(a.L, (t + 1) * a.tile);
    float x[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = 0.0f;
    if (CONV) {
      if (m < a.M) {
        const ConvRow cr = conv_row(a.conv, m);
        int c = l0 % a.conv.C, kk = l0 / a.conv.C;
        int kw = kk % a.conv.KW, kh = kk / a.conv.KW;
        if ((a.conv.C & 7) == 0 && l0 + 8 <= lend) {   // the 8 inputs are 8 channels of one pixel
          const int ih = cr.ih0 + kh, iw = cr.iw0 + kw;
          if (ih >= 0 && ih < a.conv.H && iw >= 0 && iw < a.conv.W) {
            const float* px = a.X + (cr.off + ((long long)kh * a.conv.W + kw) * a.conv.C + c);
            const float4 v0 = *reinterpret_cast<const float4*>(px);
            const float4 v1 = *reinterpret_cast<const float4*>(px + 4);
            x[0] = v0.x; x[1] = v0.y; x[2] = v0.z; x[3] = v0.w;
            x[4] = v1.x; x[5] = v1.y; x[6] = v1.z; x[7] = v1.w;
          }
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            if (l0 + e < lend) x[e] = conv_fetch(a.X, a.conv, cr, kh, kw, c);
            if (++c == a.conv.C) {
              c = 0;
              if (++kw == a.conv.KW) { kw = 0; ++kh; }
            }
          }
        }
      }
    } else if (m < a.M) {
      const float* row = a.X + (size_t)m * a.L;
      if ((a.L & 3) == 0 && l0 + 8 <= lend) {
        const float4 v0 = *reinterpret_cast<const float4*>(row + l0);
        const float4 v1 = *reinterpret_cast<const float4*>(row + l0 + 4);
        x[0] = v0.x; x[1] = v0.y; x[2] = v0.z; x[3] = v0.w;
        x[4] = v1.x; x[5] = v1.y; x[6] = v1.z; x[7] = v1.w;
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (l0 + e < lend) x[e] = row[l0 + e];
      }
    }
    union { u32x2 v; uint8_t b[8]; } pos, neg;
    if (a.offset) {
      // u = rne((x / scale + 1) / 2 * Qa): every input that exists is driven, a value of zero (also a
      // position outside the image) at mid-range; rows beyond the layer are not driven at all
      const int n_driven = m < a.M ? min(max(lend - l0, 0), 8) : 0;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int u = (int)::rint(clampd(((double)x[e] / scale + 1.0) * 0.5, 0.0, 1.0) * qa);
        pos.b[e] = (uint8_t)(e < n_driven ? u : 0);
      }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int q = (int)::rint(clampd((double)x[e] / scale, lo, 1.0) * qa);
        pos.b[e] = (uint8_t)(q > 0 ? q : 0);
        neg.b[e] = (uint8_t)(q < 0 ? -q : 0);
      }
    }
    const size_t blk = ((size_t)mp * a.T + t) * a.ks + j;
    out[blk * 64 + lane] = pos.v;
    if (a.P == 2) out[((size_t)a.MP * a.T * a.ks + blk) * 64 + lane] = neg.v;
  }
}

// ---------------------------------------------------------------------------------------------
// crossbar-tile contraction + ADC + shift-and-add (Sec. IV-B), forward and backward
// ---------------------------------------------------------------------------------------------
struct VmmArgs {
  const u32x2* A;      // quantised input fragments, 8 magnitudes (bytes) per lane
  const u32x4* B;      // plane fragments of this direction
  void* part;          // [nchunk][M][Lout] int32 (narrow) or int64 (wide, split)
  int16_t* codes;      // optional [P][S_in][S_w][npol][T][M][Lout]
  unsigned long long* hist;   // optional: kStatBins counters of |code| instead of the codes themselves
  int dac_levels;             // 0: equidistant DAC levels; else 2^stream_bits entries of dac_lut are used
  float dac_lut[16];          //    (general kernel variants only)
  int adc_curve_on;           // non-linear converter (general kernel variants only)
  float adc_curve[17];
  float q_adc, inv_q_adc;
  int M, Lin, Lout, MP, OP, MB, T, P, VT;
  int npol;                   // converters per column (1: differential, 2: one per array); VT = P * npol * T
  size_t pol_stride;          // 16-byte units between the planes of the two arrays
  int S_w, S_in, slice_bits, stream_bits, ks, tile;
  int ks16;                   // k-steps of 16 rows per tile in the staged input (= ks with fp16 planes)
  int sg;                     // kFmtF6: slices per staged group
  int scale_lo, scale_hi;     // kFmtF6: block-scale bytes (127 + exponent) of terms 0..3 and of term 4
  int vt_per_chunk, nchunk, lds_kb;
  int split_sg;               // slices per 32-bit group of the split wide path
  int direct;                 // single chunk and nothing to correct: the kernel scales and stores the result itself
  int total_wg, per_xcd;
  float gain;          // float(Q) / adc_fs
  float clamp_lo, clamp_hi;   // kMagic -+ Q
  uint32_t bias_per_vt;       // kMagicBits * sum of all shift weights, mod 2^32
  float* out;                 // final output, written directly when there is a single chunk
  double scale;               // lsb * in_scale * w_max / (Qa * Qw)
};

constexpr int kStatBins = 4096;
__shared__ uint32_t stat_hist[kStatBins];   // per-block histogram of the statistics pass (code-tap variants only)

// Asynchronous 16-byte-per-lane copy global -> LDS: `lds_wave_base` is the same for the whole wave.
__device__ __forceinline__ void copy16_global_to_lds(const u32x4* g, u32x4* lds_wave_base) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                   (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 0);
}

// A operand of one streaming cycle from the raw magnitudes: mask the digit, then spread the bytes
// into 16-bit lanes (2 AND + 4 byte permutes per 16-byte fragment).
__device__ __forceinline__ half8 digit_fragment(const u32x2 raw, uint32_t mask8) {
  const uint32_t m0 = raw.x & mask8, m1 = raw.y & mask8;
  u32x4 v;
  v.x = __builtin_amdgcn_perm(0u, m0, 0x0C010C00u);
  v.y = __builtin_amdgcn_perm(0u, m0, 0x0C030C02u);
  v.z = __builtin_amdgcn_perm(0u, m1, 0x0C010C00u);
  v.w = __builtin_amdgcn_perm(0u, m1, 0x0C030C02u);
  return __builtin_bit_cast(half8, v);
}

// DAC level table: operand that is 1.0 where the digit of this cycle equals `level`, else 0 (the
// currents of the levels are weighted with their table voltages afterwards).  Byte-parallel equality
// test, then the bytes become the high bytes of fp16 lanes (0x3C00 = 1.0).
__device__ __forceinline__ half8 level_fragment(const u32x2 raw, int in_shift, uint32_t digit_mask8, int level) {
  const uint32_t want = (uint32_t)level * 0x01010101u;
  uint32_t m[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const uint32_t x = (((h ? raw.y : raw.x) >> in_shift) & digit_mask8) ^ want;      // zero byte <=> digit == level
    const uint32_t nonzero = (((x & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | x) & 0x80808080u;
    m[h] = ((nonzero ^ 0x80808080u) >> 7) * 0x3Cu;                                    // 0x3C per matching byte
  }
  u32x4 v;
  v.x = __builtin_amdgcn_perm(0u, m[0], 0x010C000Cu);
  v.y = __builtin_amdgcn_perm(0u, m[0], 0x030C020Cu);
  v.z = __builtin_amdgcn_perm(0u, m[1], 0x010C000Cu);
  v.w = __builtin_amdgcn_perm(0u, m[1], 0x030C020Cu);
  return __builtin_bit_cast(half8, v);
}

// The plane fragment is the A operand and the sparse input digits are the B operand of the matrix
// instruction (the tile comes out transposed: lanes index the batch row, registers the output
// column): with the sparse operand on the B port the chip sustains a ~15 % higher matrix rate under
// its power limit than the other way round.
// Contraction of one (slice, cycle) in two passes over the k-steps: first the leading term, which sits
// on a fixed binary grid so that its products add without any rounding, then the residual term onto
// that exact sum.  Measured against the oracle this order leaves 1e-6 differing ADC codes, evenly one
// LSB high and low; residual first leaves 4e-6 .. 1.4e-5, all one LSB low (the matrix instruction
// rounds its sum downwards and did so at every leading-term step), and alternating the terms per
// k-step 1e-4.  Fragments are fetched two ahead.
template <int PM, int NK, int TERMS>
__device__ __forceinline__ void vmm_contract(const half8 (&ab)[PM][NK], const u32x4* bptr, float16v (&acc)[PM]) {
  constexpr int NF = TERMS * NK;
  u32x4 f0 = bptr[0], f1 = NF > 1 ? bptr[64] : f0;
#pragma unroll
  for (int i = 0; i < NF; ++i) {
    const u32x4 cur = f0;
    f0 = f1;
    if (i + 2 < NF) f1 = bptr[(i + 2) * 64];
    const half8 bf = __builtin_bit_cast(half8, cur);
#pragma unroll
    for (int pm = 0; pm < PM; ++pm) {
      if (i == 0) {
        const float16v zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        acc[pm] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf, ab[pm][0], zero, 0, 0, 0);
      } else {
        acc[pm] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf, ab[pm][i % NK], acc[pm], 0, 0, 0);
      }
    }
  }
}

// ADC + shift-and-add of one (slice, cycle): code = clamp(rne(I * gain)), y += code << sh.
// Three VALU operations per conversion: fma with 1.5 * 2^23 (rounds to nearest even in the mantissa),
// med3 (saturation), shift-add of the raw float bits (the accumulated constant is removed later).
template <int PM>
__device__ __forceinline__ void vmm_adc_narrow(const float16v (&acc)[PM], float gain_b, float clamp_lo, float clamp_hi,
                                               int sh, uint32_t (&y)[PM][16]) {
  const float vmagic = kMagic;
#pragma unroll
  for (int pm = 0; pm < PM; ++pm)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float f = __builtin_fmaf(acc[pm][r], gain_b, vmagic);
      f = __builtin_amdgcn_fmed3f(f, clamp_lo, clamp_hi);
      y[pm][r] = (__builtin_bit_cast(uint32_t, f) << sh) + y[pm][r];
    }
}

// Contraction of one (slice, cycle) with the ADC / shift-and-add of the PREVIOUS (slice, cycle)
// woven in between the matrix instructions: after the MFMAs of each fragment a fixed share of the
// previous result is converted.  On gfx950 up to ~5 VALU operations issued between two MFMAs of the
// same wave run in the shadow of the matrix pipe, whereas VALU work that sits in a block of its own
// does not overlap reliably; scheduling barriers keep the compiler from regrouping the pattern.
template <int PM, int NK, int TERMS, bool DO_ADC>
__device__ __forceinline__ void vmm_contract_adc(const half8 (&ab)[PM][NK], const u32x4* bptr, float16v (&acc)[PM],
                                                 const float16v (&old)[PM], float gain_old, float clamp_lo,
                                                 float clamp_hi, int sh_old, uint32_t (&y)[PM][16]) {
  constexpr int NF = TERMS * NK;
  constexpr int NV = 16 * PM;                       // conversions of the previous result
  const float vmagic = kMagic;
  constexpr int PF = NF < 2 ? NF : 2;               // fragments in flight from LDS
  u32x4 fr[PF];
#pragma unroll
  for (int i = 0; i < PF; ++i) fr[i] = bptr[i * 64];
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int i = 0; i < NF; ++i) {
    const u32x4 cur = fr[i % PF];
    if (i + PF < NF) fr[i % PF] = bptr[(i + PF) * 64];
    const half8 bf = __builtin_bit_cast(half8, cur);
#pragma unroll
    for (int pm = 0; pm < PM; ++pm) {
      if (i == 0) {
        const float16v zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        acc[pm] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf, ab[pm][0], zero, 0, 0, 0);
      } else {
        acc[pm] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf, ab[pm][i % NK], acc[pm], 0, 0, 0);
      }
      // the share of the previous result that rides in the shadow of this matrix instruction
      if (DO_ADC) {
        constexpr int NQ = NF * PM;
        const int q = i * PM + pm;
#pragma unroll
        for (int v = (q * NV) / NQ; v < ((q + 1) * NV) / NQ; ++v) {
          const int vp = v / 16, r = v % 16;
          float f = __builtin_fmaf(old[vp][r], gain_old, vmagic);
          f = __builtin_amdgcn_fmed3f(f, clamp_lo, clamp_hi);
          y[vp][r] = (__builtin_bit_cast(uint32_t, f) << sh_old) + y[vp][r];
        }
      }
      if (kBarrierPerMfma) __builtin_amdgcn_sched_barrier(0);
    }
    if (!kBarrierPerMfma) __builtin_amdgcn_sched_barrier(0);
  }
}

// Sign with which the converter's code enters the sum (negative-phase inputs subtract, and so does the
// array of the negative weights when it is read on its own) and the saturation bounds: a differential
// converter saturates at -+ Q, one on a single array at 0 and Q (mirrored where the code is negated).
template <bool PER_ARRAY>
__device__ __forceinline__ void adc_sign_and_range(const VmmArgs& a, int p, int pol, float& gain, float& lo, float& hi) {
  if constexpr (!PER_ARRAY) {
    gain = p ? -a.gain : a.gain;
    lo = a.clamp_lo;
    hi = a.clamp_hi;
  } else {
    const bool neg = (p ^ pol) != 0;
    gain = neg ? -a.gain : a.gain;
    lo = neg ? a.clamp_lo : kMagic;
    hi = neg ? kMagic : a.clamp_hi;
  }
}

// Software-pipelined slice group (fast path: 32-bit accumulators, no code tap, even slice count).
template <int PM, int KSMAX, int NK, int TERMS, bool PER_ARRAY>
__device__ __forceinline__ void vmm_tile_group_pipelined(const VmmArgs& a, const u32x4* lds,
                                                         const u32x2 (&raw)[PM][KSMAX], int ns, int shift_slice0, int p,
                                                         int pol, int lane, uint32_t (&y)[PM][16]) {
  constexpr int NF = TERMS * NK;
  const uint32_t digit_mask8 = ((1u << a.stream_bits) - 1u) * 0x01010101u;
  float gain_p, clamp_lo, clamp_hi;
  adc_sign_and_range<PER_ARRAY>(a, p, pol, gain_p, clamp_lo, clamp_hi);
  const u32x4* bbase = lds + lane;
  half8 ab[PM][NK];
  float16v acc0[PM], acc1[PM];
  int sh_prev = 0;
  float gain_prev = 0.f;
  for (int b = 0; b < a.S_in; ++b) {
    const int in_shift = a.stream_bits * b;
    const uint32_t mask8 = digit_mask8 << in_shift;
    // operand lanes hold digit * 2^(in_shift - 24); undo that power of two in the ADC gain
    const float gain_b = ldexpf(gain_p, 24 - in_shift);
#pragma unroll
    for (int pm = 0; pm < PM; ++pm)
#pragma unroll
      for (int j = 0; j < NK; ++j) ab[pm][j] = digit_fragment(raw[pm][j], mask8);
    for (int sl = 0; sl < ns; sl += 2) {
      const int sh0 = a.slice_bits * (shift_slice0 + sl) + in_shift;
      const int sh1 = sh0 + a.slice_bits;
      // even slice -> acc0, while the ADC of the previous odd slice (acc1) runs
      if (b == 0 && sl == 0)
        vmm_contract_adc<PM, NK, TERMS, false>(ab, bbase + (size_t)sl * NF * 64, acc0, acc1, gain_prev, clamp_lo,
                                               clamp_hi, sh_prev, y);
      else
        vmm_contract_adc<PM, NK, TERMS, true>(ab, bbase + (size_t)sl * NF * 64, acc0, acc1, gain_prev, clamp_lo,
                                              clamp_hi, sh_prev, y);
      // odd slice -> acc1, while the ADC of the even slice (acc0) runs
      vmm_contract_adc<PM, NK, TERMS, true>(ab, bbase + (size_t)(sl + 1) * NF * 64, acc1, acc0, gain_b, clamp_lo,
                                            clamp_hi, sh0, y);
      sh_prev = sh1;
      gain_prev = gain_b;
    }
  }
  vmm_adc_narrow<PM>(acc1, gain_prev, clamp_lo, clamp_hi, sh_prev, y);   // drain
}

// ADC + shift-and-add of one (slice, cycle) for the general kernel variants: 32- or 64-bit sums, optional
// transfer curve, code tap or statistics.  Same code decision as the three-operation form.
template <int PM, bool WIDE, bool CODES, bool PER_ARRAY>
__device__ __forceinline__ void vmm_adc_general(const VmmArgs& a, const float16v (&acc)[PM], float gain_used, float clamp_lo,
                                                float clamp_hi, int sh, int p, int pol, int b, int s, int t, int lane,
                                                int mp0, int op, uint32_t (&y)[PM][16], long long (&y64)[PM][16]) {
  const float vmagic = kMagic;
  const int neg = PER_ARRAY ? p ^ pol : p;
#pragma unroll
  for (int pm = 0; pm < PM; ++pm) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      uint32_t bits;
      if (CODES && a.adc_curve_on) {
        // transfer curve on the true (phase-signed) current: x in [-1, 1], 16 linear pieces
        const float u = acc[pm][r] * (p ? -gain_used : gain_used);          // ideal code units
        const float v = fminf(fmaxf(u * a.inv_q_adc * 8.0f, -8.0f), 8.0f);    // x in units of one piece
        const float start = fminf(floorf(v), 7.0f);                           // v - start is exact
        const int piece = (int)start + 8;
        const float lo = a.adc_curve[piece], hi = a.adc_curve[piece + 1];
        const float fx = __builtin_fmaf(v - start, hi - lo, lo);
        const float c = fminf(fmaxf(rintf(a.q_adc * fx), -a.q_adc), a.q_adc);
        bits = kMagicBits + (uint32_t)(p ? -(int)c : (int)c);               // as the linear path leaves it
      } else {
        float f = __builtin_fmaf(acc[pm][r], gain_used, vmagic);
        f = __builtin_amdgcn_fmed3f(f, clamp_lo, clamp_hi);
        bits = __builtin_bit_cast(uint32_t, f);
      }
      if (WIDE) {
        y64[pm][r] += (long long)((int)(bits - kMagicBits)) << sh;
      } else {
        y[pm][r] = (bits << sh) + y[pm][r];
      }
      if (CODES) {
        const int m = (mp0 + pm) * 32 + (lane & 31);
        const int o = op * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (m < a.M && o < a.Lout) {
          int code = (int)(bits - kMagicBits);
          if (a.hist) {
            atomicAdd(&stat_hist[min(::abs(code), kStatBins - 1)], 1u);
          } else if (a.codes) {
            if (neg) code = -code;                   // what the converter itself read
            const size_t converter = ((((size_t)p * a.S_in + b) * a.S_w + s) * (PER_ARRAY ? 2 : 1) + pol) * a.T + t;
            a.codes[(converter * a.M + m) * a.Lout + o] = (int16_t)code;
          }
        }
      }
    }
  }
}

// General slice group (64-bit accumulators and / or ADC code tap, any slice count): same arithmetic,
// no software pipelining.
template <int PM, int KSMAX, int NK, int TERMS, bool WIDE, bool CODES, bool PER_ARRAY>
__device__ __forceinline__ void vmm_tile_group(const VmmArgs& a, const u32x4* lds, const u32x2 (&raw)[PM][KSMAX],
                                               int ns, int sg0, int p, int pol, int t, int lane, int mp0, int op,
                                               uint32_t (&y)[PM][16], long long (&y64)[PM][16]) {
  constexpr int NF = TERMS * NK;
  const uint32_t digit_mask8 = ((1u << a.stream_bits) - 1u) * 0x01010101u;
  float gain_p, clamp_lo, clamp_hi;
  adc_sign_and_range<PER_ARRAY>(a, p, pol, gain_p, clamp_lo, clamp_hi);
  for (int b = 0; b < a.S_in; ++b) {
    const int in_shift = a.stream_bits * b;
    const uint32_t mask8 = digit_mask8 << in_shift;
    const float gain_b = ldexpf(gain_p, 24 - in_shift);
    half8 ab[PM][NK];
#pragma unroll
    for (int pm = 0; pm < PM; ++pm)
#pragma unroll
      for (int j = 0; j < NK; ++j) ab[pm][j] = digit_fragment(raw[pm][j], mask8);
    const float gain_lut = gain_p;                     // level operands are 1.0: no power of two to undo
    for (int sl = 0; sl < ns; ++sl) {
      const int s = sg0 + sl;
      const int sh = a.slice_bits * s + in_shift;
      float16v acc[PM];
      if (CODES && a.dac_levels) {
        // I = sum over levels of V_level x (current of the rows that sit at that level)
#pragma unroll
        for (int pm = 0; pm < PM; ++pm)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[pm][r] = 0.0f;
        for (int level = (a.dac_lut[0] != 0.0f ? 0 : 1); level < a.dac_levels; ++level) {
#pragma unroll
          for (int pm = 0; pm < PM; ++pm)
#pragma unroll
            for (int j = 0; j < NK; ++j) ab[pm][j] = level_fragment(raw[pm][j], in_shift, digit_mask8, level);
          float16v part[PM];
          vmm_contract<PM, NK, TERMS>(ab, lds + lane + (size_t)sl * NF * 64, part);
          const float volt = a.dac_lut[level];
#pragma unroll
          for (int pm = 0; pm < PM; ++pm)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[pm][r] = __builtin_fmaf(volt, part[pm][r], acc[pm][r]);
        }
      } else {
        vmm_contract<PM, NK, TERMS>(ab, lds + lane + (size_t)sl * NF * 64, acc);
      }
      const float gain_used = (CODES && a.dac_levels) ? gain_lut : gain_b;
      vmm_adc_general<PM, WIDE, CODES, PER_ARRAY>(a, acc, gain_used, clamp_lo, clamp_hi, sh, p, pol, b, s, t, lane, mp0, op,
                                                  y, y64);
    }
  }
}

// One virtual tile (phase, contraction tile): load the raw magnitudes, then loop over slice groups:
// stage the plane fragments of the group in LDS (compact: only the NK used k-steps), compute.
// WIDE: 0 = 32-bit sums, 1 = 64-bit sums in registers (general path), 2 = one slice group per call
// (the one that starts at slice `only_sg0`) summed in 32 bits with shifts relative to the group; the
// caller widens and adds up the groups.
template <int PM, int KSMAX, int NK, int TERMS, int WIDE, bool CODES, bool PER_ARRAY>
__device__ __forceinline__ void vmm_tile(const VmmArgs& a, u32x4* lds, int p, int pol, int t, int lane, int mp0, int op,
                                         uint32_t (&y)[PM][16], long long (&y64)[PM][16], int only_sg0) {

  u32x2 raw[PM][KSMAX];
#pragma unroll
  for (int pm = 0; pm < PM; ++pm)
#pragma unroll
    for (int j = 0; j < NK; ++j) {
      u32x2 v = {0, 0};
      if (mp0 + pm < a.MP) v = a.A[((((size_t)p * a.MP + mp0 + pm) * a.T + t) * a.ks16 + j) * 64 + lane];
      raw[pm][j] = v;
    }
  constexpr int NF = TERMS * NK;
  const int sg = WIDE == 2 ? a.split_sg : min(a.S_w, a.lds_kb / NF);   // slices per staged group
  const int sg_first = WIDE == 2 ? only_sg0 : 0, sg_end = WIDE == 2 ? only_sg0 + sg : a.S_w;
  for (int sg0 = sg_first; sg0 < sg_end; sg0 += sg) {
    const int ns = min(sg, a.S_w - sg0);
    const u32x4* src = a.B + (((size_t)t * a.OP + op) * a.S_w + sg0) * TERMS * a.ks * 64;
    if constexpr (PER_ARRAY) src += (size_t)pol * a.pol_stride;
    __syncthreads();                                   // everyone is done with the previous group
    // global [slice][term][ks][64] -> LDS [slice][term * NK + j][64]; one 1 KiB fragment per wave pass
    // Each wave copies whole 1 KiB fragments straight from global memory into LDS (no registers in
    // between, all copies of a wave in flight at once): lane l of the wave supplies the address of
    // its 16 bytes, the hardware writes them at fragment base + 16 l.
    const int nwv = blockDim.x >> 6, nfr = ns * NF;
    for (int f = threadIdx.x >> 6; f < nfr; f += nwv) {
      const int sl = f / NF, r = f - sl * NF;
      const int term = r / NK, j = r - term * NK;
      // LDS order within a slice = global order: leading term (0), then residual term (1)
      const int gterm = term;
      copy16_global_to_lds(src + ((sl * TERMS + gterm) * a.ks + j) * 64 + lane, lds + f * 64);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if constexpr (WIDE == 2) {
      vmm_tile_group_pipelined<PM, KSMAX, NK, TERMS, PER_ARRAY>(a, lds, raw, ns, 0, p, pol, lane, y);
    } else {
      if (!WIDE && !CODES && (ns & 1) == 0)
        vmm_tile_group_pipelined<PM, KSMAX, NK, TERMS, PER_ARRAY>(a, lds, raw, ns, sg0, p, pol, lane, y);
      else
        vmm_tile_group<PM, KSMAX, NK, TERMS, WIDE == 1, CODES, PER_ARRAY>(a, lds, raw, ns, sg0, p, pol, t, lane, mp0, op, y, y64);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// the same contraction on the 6-bit / 4-bit block-scaled matrix instruction (cycles of 1 or 2 bits)
// ---------------------------------------------------------------------------------------------
typedef int int4v __attribute__((ext_vector_type(4)));
typedef int int8v __attribute__((ext_vector_type(8)));
typedef int int16v __attribute__((ext_vector_type(16)));

// LDS bytes of one (slice, term): its fragments of 1.5 KiB, rounded up to the whole KiB that the staging copies move
__host__ __device__ constexpr int f6_term_stride(int nk64) { return ((nk64 * 1536 + 1023) / 1024) * 1024; }

// Digits of one streaming cycle as E2M1 codes (digit d is code d, value d / 2): the bytes of two input
// words become the low and the high 4-bit fields of one operand word (2 rotates, 1 AND, 1 AND-OR per
// 8 inputs).  `low_mask` has the digit mask in every byte.
template <int NK64>
__device__ __forceinline__ void digit_codes_f4(const u32x2 (&raw)[4 * NK64], int in_shift, uint32_t low_mask, int4v (&dg)[NK64]) {
  const uint32_t rot_lo = (uint32_t)in_shift & 31u, rot_hi = (uint32_t)(in_shift - 4) & 31u;
#pragma unroll
  for (int J = 0; J < NK64; ++J)
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const u32x2 r = raw[4 * J + w];
      const uint32_t lo = __builtin_amdgcn_alignbit(r.x, r.x, rot_lo) & low_mask;
      dg[J][w] = (int)((__builtin_amdgcn_alignbit(r.y, r.y, rot_hi) & (low_mask << 4)) | lo);
    }
}

// acc = c + 2^(scale of the term) * (E2M3 plane fragment) x (E2M1 digits); the scale byte of term 0..3 is
// byte 0..3 of scale_lo, that of term 4 byte 0 of scale_hi; the digits carry no scale (127 = 2^0).
__device__ __forceinline__ float16v mfma_f6_term(int term, const int8v& pa, const int8v& pb, const float16v& c, int scale_lo,
                                                 int scale_hi) {
  switch (term) {
    case 0: return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(pa, pb, c, 2, 4, 0, scale_lo, 0, 127);
    case 1: return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(pa, pb, c, 2, 4, 1, scale_lo, 0, 127);
    case 2: return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(pa, pb, c, 2, 4, 2, scale_lo, 0, 127);
    case 3: return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(pa, pb, c, 2, 4, 3, scale_lo, 0, 127);
    default: return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(pa, pb, c, 2, 4, 0, scale_hi, 0, 127);
  }
}

// Contraction of one (slice, cycle), terms in order (the leading term's sum is exact, the smaller terms
// land on it), with the ADC / shift-and-add of the PREVIOUS (slice, cycle) woven in between the matrix
// instructions.  xb / yb: this lane's address in the first KiB / last half KiB of the slice's first fragment.
template <int PM, int NK64, int NT, bool DO_ADC>
__device__ __forceinline__ void vmm6_contract_adc(const int4v (&dg)[PM][NK64], const char* xb, const char* yb,
                                                  float16v (&acc)[PM], const float16v (&old)[PM], float gain_old,
                                                  float clamp_lo, float clamp_hi, int sh_old, uint32_t (&y)[PM][16],
                                                  int scale_lo, int scale_hi) {
  constexpr int NF = NT * NK64;
  constexpr int STRIDE = f6_term_stride(NK64);
  constexpr int NV = 16 * PM;
  const float vmagic = kMagic;
  constexpr int PF = NF < 2 ? NF : 2;
  u32x4 fx[PF];
  u32x2 fy[PF];
#pragma unroll
  for (int i = 0; i < PF; ++i) {
    const int off = (i / NK64) * STRIDE + (i % NK64) * 1536;
    fx[i] = *reinterpret_cast<const u32x4*>(xb + off);
    fy[i] = *reinterpret_cast<const u32x2*>(yb + off);
  }
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int i = 0; i < NF; ++i) {
    const u32x4 cx = fx[i % PF];
    const u32x2 cy = fy[i % PF];
    if (i + PF < NF) {
      const int off = ((i + PF) / NK64) * STRIDE + ((i + PF) % NK64) * 1536;
      fx[i % PF] = *reinterpret_cast<const u32x4*>(xb + off);
      fy[i % PF] = *reinterpret_cast<const u32x2*>(yb + off);
    }
    const int8v pa = {(int)cx.x, (int)cx.y, (int)cx.z, (int)cx.w, (int)cy.x, (int)cy.y, 0, 0};
    const int term = i / NK64, J = i % NK64;
#pragma unroll
    for (int pm = 0; pm < PM; ++pm) {
      const int8v pb = {dg[pm][J][0], dg[pm][J][1], dg[pm][J][2], dg[pm][J][3], 0, 0, 0, 0};
      if (i == 0) {
        const float16v zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        acc[pm] = mfma_f6_term(0, pa, pb, zero, scale_lo, scale_hi);
      } else {
        acc[pm] = mfma_f6_term(term, pa, pb, acc[pm], scale_lo, scale_hi);
      }
      if (DO_ADC) {
        constexpr int NQ = NF * PM;
        const int q = i * PM + pm;
#pragma unroll
        for (int v = (q * NV) / NQ; v < ((q + 1) * NV) / NQ; ++v) {
          const int vp = v / 16, r = v % 16;
          float f = __builtin_fmaf(old[vp][r], gain_old, vmagic);
          f = __builtin_amdgcn_fmed3f(f, clamp_lo, clamp_hi);
          y[vp][r] = (__builtin_bit_cast(uint32_t, f) << sh_old) + y[vp][r];
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }
}

// Software-pipelined slice group (32-bit accumulators, no code tap, even slice count).
template <int PM, int NK64, int NT, bool PER_ARRAY>
__device__ __forceinline__ void vmm6_tile_group_pipelined(const VmmArgs& a, const char* lds, const u32x2 (&raw)[PM][4 * NK64],
                                                          int ns, int shift_slice0, int p, int pol, int lane,
                                                          uint32_t (&y)[PM][16]) {
  constexpr int SLICE = NT * f6_term_stride(NK64);
  const uint32_t low_mask = ((1u << a.stream_bits) - 1u) * 0x01010101u;
  float gain_p, clamp_lo, clamp_hi;
  adc_sign_and_range<PER_ARRAY>(a, p, pol, gain_p, clamp_lo, clamp_hi);
  const float gain = 2.0f * gain_p;                   // a digit enters as d / 2
  const char* xb = lds + lane * 16;
  const char* yb = lds + 1024 + lane * 8;
  int4v dg[PM][NK64];
  float16v acc0[PM], acc1[PM];
  int sh_prev = 0;
  for (int b = 0; b < a.S_in; ++b) {
    const int in_shift = a.stream_bits * b;
#pragma unroll
    for (int pm = 0; pm < PM; ++pm) digit_codes_f4<NK64>(raw[pm], in_shift, low_mask, dg[pm]);
    for (int sl = 0; sl < ns; sl += 2) {
      const int sh0 = a.slice_bits * (shift_slice0 + sl) + in_shift;
      const int sh1 = sh0 + a.slice_bits;
      if (b == 0 && sl == 0)
        vmm6_contract_adc<PM, NK64, NT, false>(dg, xb + sl * SLICE, yb + sl * SLICE, acc0, acc1, gain, clamp_lo, clamp_hi,
                                               sh_prev, y, a.scale_lo, a.scale_hi);
      else
        vmm6_contract_adc<PM, NK64, NT, true>(dg, xb + sl * SLICE, yb + sl * SLICE, acc0, acc1, gain, clamp_lo, clamp_hi,
                                              sh_prev, y, a.scale_lo, a.scale_hi);
      vmm6_contract_adc<PM, NK64, NT, true>(dg, xb + (sl + 1) * SLICE, yb + (sl + 1) * SLICE, acc1, acc0, gain, clamp_lo,
                                            clamp_hi, sh0, y, a.scale_lo, a.scale_hi);
      sh_prev = sh1;
    }
  }
  vmm_adc_narrow<PM>(acc1, gain, clamp_lo, clamp_hi, sh_prev, y);   // drain
}

// General slice group (64-bit sums, code tap, transfer curve, statistics, odd slice counts).
template <int PM, int NK64, int NT, bool WIDE, bool CODES, bool PER_ARRAY>
__device__ __forceinline__ void vmm6_tile_group(const VmmArgs& a, const char* lds, const u32x2 (&raw)[PM][4 * NK64], int ns,
                                                int sg0, int p, int pol, int t, int lane, int mp0, int op,
                                                uint32_t (&y)[PM][16], long long (&y64)[PM][16]) {
  constexpr int SLICE = NT * f6_term_stride(NK64);
  const uint32_t low_mask = ((1u << a.stream_bits) - 1u) * 0x01010101u;
  float gain_p, clamp_lo, clamp_hi;
  adc_sign_and_range<PER_ARRAY>(a, p, pol, gain_p, clamp_lo, clamp_hi);
  const float gain = 2.0f * gain_p;
  const char* xb = lds + lane * 16;
  const char* yb = lds + 1024 + lane * 8;
  for (int b = 0; b < a.S_in; ++b) {
    const int in_shift = a.stream_bits * b;
    int4v dg[PM][NK64];
#pragma unroll
    for (int pm = 0; pm < PM; ++pm) digit_codes_f4<NK64>(raw[pm], in_shift, low_mask, dg[pm]);
    for (int sl = 0; sl < ns; ++sl) {
      const int s = sg0 + sl;
      const int sh = a.slice_bits * s + in_shift;
      float16v acc[PM], none[PM];
      uint32_t unused[PM][16];
      vmm6_contract_adc<PM, NK64, NT, false>(dg, xb + sl * SLICE, yb + sl * SLICE, acc, none, 0.f, 0.f, 0.f, 0, unused,
                                             a.scale_lo, a.scale_hi);
      vmm_adc_general<PM, WIDE, CODES, PER_ARRAY>(a, acc, gain, clamp_lo, clamp_hi, sh, p, pol, b, s, t, lane, mp0, op, y, y64);
    }
  }
}

// One virtual tile on the 6-bit path: NK64 k-steps of 64 rows (nk16 staged input steps of 16).
template <int PM, int NK64, int NT, int WIDE, bool CODES, bool PER_ARRAY>
__device__ __forceinline__ void vmm6_tile(const VmmArgs& a, u32x4* lds, int p, int pol, int t, int nk16, int lane, int mp0,
                                          int op, uint32_t (&y)[PM][16], long long (&y64)[PM][16], int only_sg0) {
  u32x2 raw[PM][4 * NK64];
#pragma unroll
  for (int pm = 0; pm < PM; ++pm)
#pragma unroll
    for (int j = 0; j < 4 * NK64; ++j) {
      u32x2 v = {0, 0};
      if (mp0 + pm < a.MP && j < nk16) v = a.A[((((size_t)p * a.MP + mp0 + pm) * a.T + t) * a.ks16 + j) * 64 + lane];
      raw[pm][j] = v;
    }
  constexpr int STRIDE = f6_term_stride(NK64);
  constexpr int UNITS = STRIDE / 1024;               // KiB copies per (slice, term)
  const int sg = WIDE == 2 ? a.split_sg : a.sg;
  const int sg_first = WIDE == 2 ? only_sg0 : 0, sg_end = WIDE == 2 ? only_sg0 + sg : a.S_w;
  for (int sg0 = sg_first; sg0 < sg_end; sg0 += sg) {
    const int ns = min(sg, a.S_w - sg0);
    // global [slice][term][k-steps of the whole tile][1.5 KiB] -> LDS [slice][term][STRIDE]: only the NK64 used steps
    const u32x4* src = a.B + (((size_t)t * a.OP + op) * a.S_w + sg0) * NT * a.ks * 96;
    if constexpr (PER_ARRAY) src += (size_t)pol * a.pol_stride;
    __syncthreads();                                   // everyone is done with the previous group
    const int nwv = blockDim.x >> 6, ncopy = ns * NT * UNITS;
    for (int c = threadIdx.x >> 6; c < ncopy; c += nwv) {
      const int st = c / UNITS, u = c - st * UNITS;    // (slice, term) pair, KiB within it
      copy16_global_to_lds(src + (size_t)st * a.ks * 96 + u * 64 + lane, lds + (st * UNITS + u) * 64);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    const char* stage = reinterpret_cast<const char*>(lds);
    if constexpr (WIDE == 2) {
      vmm6_tile_group_pipelined<PM, NK64, NT, PER_ARRAY>(a, stage, raw, ns, 0, p, pol, lane, y);
    } else {
      if (!WIDE && !CODES && (ns & 1) == 0)
        vmm6_tile_group_pipelined<PM, NK64, NT, PER_ARRAY>(a, stage, raw, ns, sg0, p, pol, lane, y);
      else
        vmm6_tile_group<PM, NK64, NT, WIDE == 1, CODES, PER_ARRAY>(a, stage, raw, ns, sg0, p, pol, t, lane, mp0, op, y, y64);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// block-level driver shared by both operand formats: virtual tiles of the chunk, partial results
// ---------------------------------------------------------------------------------------------
// Tile functors: run one virtual tile (phase p, array pol, contraction tile t with `rows` rows).
template <int PM, int KSMAX, int TERMS, int WIDE, bool CODES, bool PER_ARRAY>
struct TileF16 {
  __device__ __forceinline__ void operator()(const VmmArgs& a, u32x4* lds, int p, int pol, int t, int rows, int lane, int mp0,
                                             int op, uint32_t (&y)[PM][16], long long (&y64)[PM][16], int only_sg0) const {
    const int nk = (rows + 15) >> 4;
#define XBAR_NK_CASE(n) \
  case n:               \
    if constexpr (n <= KSMAX)                                                                                       \
      vmm_tile<PM, KSMAX, n, TERMS, WIDE, CODES, PER_ARRAY>(a, lds, p, pol, t, lane, mp0, op, y, y64, only_sg0); \
    break;
    switch (nk) {
      XBAR_NK_CASE(1) XBAR_NK_CASE(2) XBAR_NK_CASE(3) XBAR_NK_CASE(4) XBAR_NK_CASE(5) XBAR_NK_CASE(6)
      XBAR_NK_CASE(7) XBAR_NK_CASE(8) XBAR_NK_CASE(9) XBAR_NK_CASE(10) XBAR_NK_CASE(11) XBAR_NK_CASE(12)
      XBAR_NK_CASE(13) XBAR_NK_CASE(14) XBAR_NK_CASE(15) XBAR_NK_CASE(16)
      default: break;
    }
#undef XBAR_NK_CASE
  }
};

template <int PM, int NT, int WIDE, bool CODES, bool PER_ARRAY>
struct TileF6 {
  __device__ __forceinline__ void operator()(const VmmArgs& a, u32x4* lds, int p, int pol, int t, int rows, int lane, int mp0,
                                             int op, uint32_t (&y)[PM][16], long long (&y64)[PM][16], int only_sg0) const {
    const int nk16 = (rows + 15) >> 4;
    switch ((rows + 63) >> 6) {
      case 1: vmm6_tile<PM, 1, NT, WIDE, CODES, PER_ARRAY>(a, lds, p, pol, t, nk16, lane, mp0, op, y, y64, only_sg0); break;
      case 2: vmm6_tile<PM, 2, NT, WIDE, CODES, PER_ARRAY>(a, lds, p, pol, t, nk16, lane, mp0, op, y, y64, only_sg0); break;
      case 3: vmm6_tile<PM, 3, NT, WIDE, CODES, PER_ARRAY>(a, lds, p, pol, t, nk16, lane, mp0, op, y, y64, only_sg0); break;
      case 4: vmm6_tile<PM, 4, NT, WIDE, CODES, PER_ARRAY>(a, lds, p, pol, t, nk16, lane, mp0, op, y, y64, only_sg0); break;
      default: break;
    }
  }
};

template <int PM, int WIDE, bool CODES, bool PER_ARRAY, class TileFn>
__device__ __forceinline__ void vmm_block(const VmmArgs& a, u32x4* lds, const TileFn& run_tile) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  // consecutive block ids go to different XCDs; give each XCD a contiguous range of logical work so
  // that blocks sharing the same planes share one L2
  const int logical = (blockIdx.x & 7) * a.per_xcd + (blockIdx.x >> 3);
  if (logical >= a.total_wg) return;
  // chunk is the fastest index: every XCD then gets the same mix of (slightly unequal) chunks
  const int chunk = logical % a.nchunk;
  const int grp = logical / a.nchunk;
  const int mb = grp % a.MB;
  const int op = grp / a.MB;
  const int mp0 = (mb * nw + wave) * PM;
  if constexpr (CODES) {
    if (a.hist) {
      for (int i = threadIdx.x; i < kStatBins; i += blockDim.x) stat_hist[i] = 0;
      __syncthreads();
    }
  }

  uint32_t y[PM][16];
  long long y64[PM][16];
#pragma unroll
  for (int pm = 0; pm < PM; ++pm)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      y[pm][r] = 0;
      y64[pm][r] = 0;
    }

  // virtual tiles spread evenly over the chunks: the first VT % nchunk chunks get one more
  const int vt_base = a.VT / a.nchunk, vt_rem = a.VT - vt_base * a.nchunk;
  const int vt0 = chunk * vt_base + min(chunk, vt_rem);
  const int vt1 = vt0 + vt_base + (chunk < vt_rem ? 1 : 0);
#define XBAR_ALL_VIRTUAL_TILES                                                                              \
  for (int vt = vt0; vt < vt1; ++vt) {                                                                      \
    /* vt = (phase, array, tile), tile fastest */                                                           \
    const int pa = vt / a.T, t = vt - pa * a.T;                                                             \
    const int p = PER_ARRAY ? pa >> 1 : pa, pol = PER_ARRAY ? pa & 1 : 0;                                   \
    const int rows = min(a.tile, a.Lin - t * a.tile);                                                       \
    run_tile(a, lds, p, pol, t, rows, lane, mp0, op, y, y64, only_sg0);                                     \
  }
  if constexpr (WIDE == 2) {
    // Sums that overflow 32 bits, fast path: one pass over the chunk's virtual tiles per slice group,
    // each summed in 32 bits with shifts relative to the group's first slice, then widened, shifted
    // into place and added to the chunk's 64-bit partial result (every element has one owner lane).
    const uint32_t bias = a.bias_per_vt * (uint32_t)(vt1 - vt0);
    long long* part = reinterpret_cast<long long*>(a.part) + (size_t)chunk * a.M * a.Lout;
    for (int only_sg0 = 0; only_sg0 < a.S_w; only_sg0 += a.split_sg) {
      XBAR_ALL_VIRTUAL_TILES
      const int up = a.slice_bits * only_sg0;
      // the element addresses are the same for every group: keep the compiler from computing all of
      // them ahead of the loop, where they would sit in registers throughout the contraction
      int lane_now = lane, mp_now = mp0;
      asm volatile("" : "+v"(lane_now), "+v"(mp_now));
#pragma unroll
      for (int pm = 0; pm < PM; ++pm)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = (mp_now + pm) * 32 + (lane_now & 31);
          const int o = op * 32 + 8 * (r >> 2) + 4 * (lane_now >> 5) + (r & 3);
          if (m < a.M && o < a.Lout && mp_now + pm < a.MP) {
            long long v = (long long)(int32_t)(y[pm][r] - bias) << up;
            if (only_sg0) v += part[(size_t)m * a.Lout + o];
            part[(size_t)m * a.Lout + o] = v;
          }
          y[pm][r] = 0;
        }
    }
    return;
  } else {
    const int only_sg0 = 0;
    XBAR_ALL_VIRTUAL_TILES
  }
#undef XBAR_ALL_VIRTUAL_TILES
  if constexpr (CODES) {
    if (a.hist) {                                  // statistics pass: the counters are the only result
      __syncthreads();
      for (int i = threadIdx.x; i < kStatBins; i += blockDim.x)
        if (stat_hist[i]) atomicAdd(&a.hist[i], (unsigned long long)stat_hist[i]);
      return;
    }
  }
  // partial result of this chunk
  const uint32_t bias = a.bias_per_vt * (uint32_t)(vt1 - vt0);
#pragma unroll
  for (int pm = 0; pm < PM; ++pm)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = (mp0 + pm) * 32 + (lane & 31);
      const int o = op * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      if (m < a.M && o < a.Lout && mp0 + pm < a.MP) {
        const size_t idx = ((size_t)chunk * a.M + m) * a.Lout + o;
        if (a.direct) {        // nothing to add up across chunks: scale and store the result itself
          const long long sum = WIDE ? y64[pm][r] : (long long)(int32_t)(y[pm][r] - bias);
          a.out[idx] = (float)((double)sum * a.scale);
        } else if (WIDE) {
          reinterpret_cast<long long*>(a.part)[idx] = y64[pm][r];
        } else {
          reinterpret_cast<int32_t*>(a.part)[idx] = (int32_t)(y[pm][r] - bias);
        }
      }
    }
}

template <int PM, int KSMAX, int TERMS, int WIDE, bool CODES, bool PER_ARRAY>
__global__ __launch_bounds__(256, 2) void vmm_kernel(VmmArgs a) {
  extern __shared__ u32x4 lds[];
  vmm_block<PM, WIDE, CODES, PER_ARRAY>(a, lds, TileF16<PM, KSMAX, TERMS, WIDE, CODES, PER_ARRAY>());
}

template <int NT, int WIDE, bool CODES, bool PER_ARRAY>
__global__ __launch_bounds__(256, 2) void vmm6_kernel(VmmArgs a) {
  extern __shared__ u32x4 lds[];
  vmm_block<2, WIDE, CODES, PER_ARRAY>(a, lds, TileF6<2, NT, WIDE, CODES, PER_ARRAY>());
}

struct FinishArgs {
  const void* part;
  float* out;
  long long n;   // M * Lout
  int nchunk, wide, Lout;
  double scale;
  const long long* wsum;   // offset-binary inputs: weight sum per output, else null
  double half_range;       //   and the half-range it is multiplied with
};

__global__ __launch_bounds__(256) void vmm_finish_kernel(FinishArgs a) {
#pragma clang fp contract(off)   // product, product, difference: each rounded on its own
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= a.n) return;
  long long sum = 0;
  for (int c = 0; c < a.nchunk; ++c)
    sum += a.wide ? reinterpret_cast<const long long*>(a.part)[(size_t)c * a.n + i]
                  : (long long)reinterpret_cast<const int32_t*>(a.part)[(size_t)c * a.n + i];
  double y = (double)sum * a.scale;
  if (a.wsum) y = y - (double)a.wsum[i % a.Lout] * a.half_range;
  a.out[i] = (float)y;
}

// ---------------------------------------------------------------------------------------------
// update model (Sec. IV-C)
// ---------------------------------------------------------------------------------------------
struct GradArgs {
  const float* X;   // [M][K], or the NHWC image with CONV
  const float* D;   // [M][N]
  float* part;      // [mchunks][K][N]
  int M, K, N, KB, NB, m_per_chunk;
  ConvGeom conv;
};

constexpr int kGradMS = 32;   // batch rows per LDS stage = two k-steps of the bf16 matrix instruction
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// fp32 value as a leading bf16 and a bf16 residual (together 16 significant bits).
__device__ __forceinline__ void split_bf16(float x, __bf16& hi, __bf16& lo) {
  hi = (__bf16)x;
  lo = (__bf16)(x - (float)hi);
}

// 128 x 128 tile of X^T dY per block, 4 waves as 2 x 2, each wave 64 x 64 = 2 x 2 MFMA tiles of
// v_mfma_f32_32x32x16_bf16.  Both operands are split into two bf16 terms while they are staged into
// LDS and hi.hi + hi.lo + lo.hi is accumulated in fp32: three bf16 matrix instructions of 16 rows do
// the work of eight fp32 ones of 2 rows at a relative error near 2^-16 per product, far inside the
// tolerance of the update.  When the layer has at most 64 rows (SPLIT_K) or columns (SPLIT_N) the
// waves that would work on padding take a share of the batch rows instead and write a partial sum of
// their own.  CONV: X is an NHWC image and the patch rows are gathered on the fly.
template <bool SPLIT_K, bool SPLIT_N, bool CONV>
__global__ __launch_bounds__(256) void grad_gemm_kernel(GradArgs a) {
  // [term][group of 8 batch rows][column] -> 8 bf16 along the batch
  __shared__ bf16x8 xs[2][kGradMS / 8][128];
  __shared__ bf16x8 ds[2][kGradMS / 8][128];
  __shared__ ConvRow crow[2][kGradMS];               // patches of the rows of the stage being fetched
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wk = wave >> 1, wn = wave & 1;
  const int kb = blockIdx.x % a.KB, nb = blockIdx.x / a.KB;
  const int k0 = kb * 128, n0 = nb * 128;
  const int m_begin = blockIdx.y * a.m_per_chunk;
  const int m_end = min(a.M, m_begin + a.m_per_chunk);
  constexpr int PARTS = (SPLIT_K ? 2 : 1) * (SPLIT_N ? 2 : 1);     // batch shares
  const int share = (SPLIT_K ? wk : 0) * (SPLIT_N ? 2 : 1) + (SPLIT_N ? wn : 0);
  const int koff = SPLIT_K ? 0 : wk * 64, noff = SPLIT_N ? 0 : wn * 64;
  float16v acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  // staging: this thread fetches column (tid & 127) of 16 of the 32 rows of a stage: row groups
  // (tid >> 7) and (tid >> 7) + 2
  const int col = tid & 127, g_first = tid >> 7;
  float px[16], pd[16];
  int ckh = 0, ckw = 0, cc = 0;
  if (CONV) {                                        // the kernel position of this thread's column is fixed
    const int k = min(k0 + col, a.K - 1);
    cc = k % a.conv.C;
    ckw = (k / a.conv.C) % a.conv.KW;
    ckh = (k / a.conv.C) / a.conv.KW;
  }
  auto stage_rows = [&](int m0, int buf) {            // CONV: the first threads decompose the stage's rows
    if (CONV && tid < kGradMS) crow[buf][tid] = conv_row(a.conv, min(m0 + tid, a.M - 1));
  };
  auto prefetch = [&](int m0, int buf) {
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int row = (g_first + 2 * q) * 8 + e;
        const int m = m0 + row;
        float x = 0.0f, d = 0.0f;
        if (m < m_end) {
          if (k0 + col < a.K)
            x = CONV ? conv_fetch(a.X, a.conv, crow[buf][row], ckh, ckw, cc) : a.X[(size_t)m * a.K + k0 + col];
          if (n0 + col < a.N) d = a.D[(size_t)m * a.N + n0 + col];
        }
        px[q * 8 + e] = x;
        pd[q * 8 + e] = d;
      }
  };
  int stage = 0;
  stage_rows(m_begin, 0);
  if (CONV) __syncthreads();
  prefetch(m_begin, 0);
  for (int m0 = m_begin; m0 < m_end; m0 += kGradMS, stage ^= 1) {
    if (m0 + kGradMS < m_end) stage_rows(m0 + kGradMS, stage ^ 1);
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      bf16x8 xh, xl, dh, dl;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        __bf16 h, l;
        split_bf16(px[q * 8 + e], h, l);
        xh[e] = h; xl[e] = l;
        split_bf16(pd[q * 8 + e], h, l);
        dh[e] = h; dl[e] = l;
      }
      xs[0][g_first + 2 * q][col] = xh;
      xs[1][g_first + 2 * q][col] = xl;
      ds[0][g_first + 2 * q][col] = dh;
      ds[1][g_first + 2 * q][col] = dl;
    }
    __syncthreads();
    if (m0 + kGradMS < m_end) prefetch(m0 + kGradMS, stage ^ 1);
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      // batch shares: two shares alternate over the k-steps of a stage, four also over the stages
      if (PARTS == 2 && ks != share) continue;
      if (PARTS == 4 && (ks != (share & 1) || (stage != (share >> 1)))) continue;
      const int g8 = 2 * ks + (lane >> 5);
      bf16x8 ah[2], al[2], bh[2], bl[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        ah[i] = xs[0][g8][koff + 32 * i + (lane & 31)];
        al[i] = xs[1][g8][koff + 32 * i + (lane & 31)];
        bh[i] = ds[0][g8][noff + 32 * i + (lane & 31)];
        bl[i] = ds[1][g8][noff + 32 * i + (lane & 31)];
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[i], bh[j], acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], bl[j], acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], bh[j], acc[i][j], 0, 0, 0);
        }
    }
  }
  float* out = a.part + ((size_t)blockIdx.y * PARTS + share) * a.K * a.N;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int k = k0 + koff + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        const int n = n0 + noff + j * 32 + (lane & 31);
        if (k < a.K && n < a.N) out[(size_t)k * a.N + n] = acc[i][j][r];
      }
}

// Backward pass of a convolution layer: the crossbars give the error of every patch element
// (dXcol[M][K]); an input pixel collects, digitally, the errors of every patch it belongs to.
struct Col2imArgs {
  const float* col;  // [M][K]
  float* dX;         // NHWC
  ConvGeom conv;
  int B, K;
  long long n;
};

__global__ __launch_bounds__(256) void col2im_kernel(Col2imArgs a) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= a.n) return;
  const ConvGeom& g = a.conv;
  const int c = (int)(t % g.C);
  long long u = t / g.C;
  const int iw = (int)(u % g.W);
  u /= g.W;
  const int ih = (int)(u % g.H), b = (int)(u / g.H);
  float sum = 0.0f;
  for (int kh = 0; kh < g.KH; ++kh) {
    const int oy = ih + g.pad - kh;
    if (oy < 0 || oy % g.stride) continue;
    const int oh = oy / g.stride;
    if (oh >= g.OH) continue;
    for (int kw = 0; kw < g.KW; ++kw) {
      const int ox = iw + g.pad - kw;
      if (ox < 0 || ox % g.stride) continue;
      const int ow = ox / g.stride;
      if (ow >= g.OW) continue;
      const long long m = ((long long)b * g.OH + oh) * g.OW + ow;
      sum += a.col[m * a.K + (kh * g.KW + kw) * g.C + c];
    }
  }
  a.dX[t] = sum;
}

struct WriteArgs {
  float* W;
  const float* part;
  long long n;      // K * N
  int mchunks;
  uint32_t flags;
  double w_max, grad_scale, lr, v, gamma;
  uint64_t seed, step;
  const unsigned long long* step_add;   // optional device counter added to step
};

// 32 consecutive weights per block; the 8 thread groups of a block add up interleaved subsets of the
// batch partials (fixed order, so the result does not depend on scheduling), group 0 then writes.
__global__ __launch_bounds__(256) void update_write_kernel(WriteArgs a) {
  __shared__ double red[8][32];
  const int e = threadIdx.x & 31, grp = threadIdx.x >> 5;
  const long long i = (long long)blockIdx.x * 32 + e;
  double partial = 0.0;
  if (i < a.n)
    for (int c = grp; c < a.mchunks; c += 8) partial += (double)a.part[(size_t)c * a.n + i];
  red[grp][e] = partial;
  __syncthreads();
  if (grp != 0 || i >= a.n) return;
  double grad = 0.0;
#pragma unroll
  for (int g = 0; g < 8; ++g) grad += red[g][e];
  const double g = (double)a.W[i] / a.w_max;
  const double delta = a.grad_scale * grad;
  double written = delta;
  if (a.flags & XBAR_NI_UPD_NL) {
    const double x = clampd(0.5 * (g + 1.0), 0.0, 1.0);
    const double change = -a.lr * delta;
    if (change > 0.0) written = delta * ::exp(-a.v * x);
    else if (change < 0.0) written = delta * ::exp(-a.v * (1.0 - x));
  }
  if (a.flags & XBAR_NI_UPD_NOISE) {
    NormalStream rng(a.seed, kStreamWrite, effective_step(a.step, a.step_add));
    written += a.gamma * ::sqrt(::fabs(delta)) * rng.get((uint64_t)i);
  }
  const double g_new = clampd(g - a.lr * written, -1.0, 1.0);
  a.W[i] = (float)(a.w_max * g_new);
}



// ---------------------------------------------------------------------------------------------
// instrumentation: sustained matrix-instruction rate
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void mfma_probe_kernel(float* out, int iters, int mode) {
  uint32_t x = threadIdx.x * 2654435761u + 12345u;
  union { half8 h; uint32_t u[4]; } ua, ub;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x ^= x << 13; x ^= x >> 17; x ^= x << 5;
    // two fp16 values in [-4, 4) per word; sign, exponent and mantissa bits all toggle
    ua.u[i] = mode == 1 ? (x & 0x00010001u) : ((x & 0x83ff83ffu) | 0x3c003c00u);
    x ^= x << 13; x ^= x >> 17; x ^= x << 5;
    ub.u[i] = (x & 0x83ff83ffu) | 0x3c003c00u;
  }
  float16v c0, c1;
#pragma unroll
  for (int r = 0; r < 16; ++r) c0[r] = c1[r] = 0.0f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(ub.h, ua.h, c0, 0, 0, 0);   // dense on A, sparse on B
      c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(ub.h, ua.h, c1, 0, 0, 0);
    }
  }
  float s = 0.0f;
#pragma unroll
  for (int r = 0; r < 16; ++r) s += c0[r] + c1[r];
  out[blockIdx.x * 256 + threadIdx.x] = s;
}

// Same loop with the 8-bit integer instruction (32 x 32 x 32 per instruction, twice the products).
__global__ __launch_bounds__(256) void mfma_probe_i8_kernel(int* out, int iters, int mode) {
  uint32_t x = threadIdx.x * 2654435761u + 12345u;
  int4v a, b;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x ^= x << 13; x ^= x >> 17; x ^= x << 5;
    a[i] = (int)(mode == 3 ? (x & 0x01010101u) : x);       // single-bit digits as in the emulation, or any bytes
    x ^= x << 13; x ^= x >> 17; x ^= x << 5;
    b[i] = (int)x;
  }
  int16v c0, c1;
#pragma unroll
  for (int r = 0; r < 16; ++r) c0[r] = c1[r] = 0;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      c0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(b, a, c0, 0, 0, 0);
      c1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(b, a, c1, 0, 0, 0);
    }
  }
  int s = 0;
#pragma unroll
  for (int r = 0; r < 16; ++r) s += c0[r] + c1[r];
  out[blockIdx.x * 256 + threadIdx.x] = s;
}

// ---------------------------------------------------------------------------------------------
// host dispatch
// ---------------------------------------------------------------------------------------------
thread_local hipEvent_t g_trace_before = nullptr, g_trace_after = nullptr;
thread_local const unsigned long long* g_step_source = nullptr;

__global__ void step_advance_kernel(unsigned long long* counter) { *counter += 1ull; }

struct VmmPlan {
  PlaneGeom g;
  int ks16;            // k-steps of 16 rows per tile in the staged input
  int sg;              // kFmtF6: slices per staged group
  int Lin, Lout, MP, P, VT, vt_per_chunk, nchunk, pm, nw, MB, lds_kb;
  int wide;            // 0: sums fit 32 bits; 1: 64-bit sums; 2: 32-bit sums per slice group, widened per group
  int split_sg;        // slices per group of mode 2
  uint32_t bias_split; // kMagicBits * sum of the shift weights of one such group, mod 2^32
  int offset;          // signed inputs in one phase of offset-binary codes
  uint32_t bias_per_vt;
  size_t a_bytes, part_bytes, ws_bytes, lds_bytes;
};

VmmPlan plan_vmm(const xbar_config* c, const Derived& d, int M, int K, int N, bool transposed) {
  VmmPlan p;
  p.g = plane_geom(c, d, K, N, transposed);
  p.Lin = transposed ? N : K;
  p.Lout = transposed ? K : N;
  p.MP = cdiv(M, 32);
  const bool is_signed = transposed || (c->flags & XBAR_INPUT_SIGNED);
  p.offset = (is_signed && (c->flags & XBAR_INPUT_OFFSET)) ? 1 : 0;
  p.P = (is_signed && !p.offset) ? 2 : 1;
  p.VT = p.P * d.npol * p.g.T;
  // sum of the shift-and-add weights of one virtual tile
  unsigned long long wsum = 0;
  for (int s = 0; s < d.S_w; ++s)
    for (int b = 0; b < d.S_in; ++b) wsum += 1ull << (c->slice_bits * s + c->stream_bits * b);
  p.bias_per_vt = (uint32_t)((unsigned long long)kMagicBits * wsum);
  const unsigned long long per_vt = wsum * (unsigned long long)d.q_adc;
  const unsigned long long fit = per_vt ? ((1ull << 31) - 1) / per_vt : (1ull << 31);
  p.wide = fit < 1 ? 1 : 0;
  p.ks16 = p.g.tile / 16;
  // KiB of operand per slice and output patch in the LDS stage
  const int slice_kb = d.fmt == kFmtF6 ? d.terms * f6_term_stride(p.g.ks) / 1024 : d.terms * p.g.ks;
  p.sg = d.S_w;
  if (d.fmt == kFmtF6) {
    // as many slices per stage as fit 64 KiB; an even number when not all fit (the pipelined path pairs them)
    const int fit_sg = std::max(1, 64 / slice_kb);
    if (fit_sg < d.S_w) p.sg = fit_sg >= 2 ? (fit_sg & ~1) : 1;
    p.lds_kb = p.sg * slice_kb;
  } else {
    p.lds_kb = std::max(slice_kb, std::min(d.S_w * slice_kb, 64));   // staged slice group, at most 64 KiB
  }
  p.lds_bytes = (size_t)p.lds_kb * 1024;
  // 64-bit sums: the software-pipelined path still serves if the slices split into equal, even
  // groups that fit the LDS stage and whose own sum fits 32 bits
  p.split_sg = 0;
  p.bias_split = 0;
  unsigned long long fit_split = 0;
  if (p.wide) {
    for (int sg = std::min(d.S_w, p.lds_kb / slice_kb) & ~1; sg >= 2; sg -= 2) {
      if (d.S_w % sg) continue;
      unsigned long long wg = 0;
      for (int s = 0; s < sg; ++s)
        for (int b = 0; b < d.S_in; ++b) wg += 1ull << (c->slice_bits * s + c->stream_bits * b);
      const unsigned long long f = ((1ull << 31) - 1) / (wg * (unsigned long long)d.q_adc);
      if (f < 1) continue;
      p.wide = 2;
      p.split_sg = sg;
      p.bias_split = (uint32_t)((unsigned long long)kMagicBits * wg);
      fit_split = f;
      break;
    }
  }
  p.pm = (d.fmt == kFmtF6 || p.g.ks <= 8) ? 2 : 1;
  p.nw = std::min(4, std::max(1, cdiv(p.MP, p.pm)));
  p.MB = cdiv(p.MP, p.pm * p.nw);
  const int groups = p.g.OP * p.MB;
  int want_chunks = std::max(1, cdiv(4096, groups));      // 8 rounds of 2 blocks on 256 CUs: the last, partly
                                                          // filled round costs less (measured: 0.8 % per step over 2048)
  int per = std::max(1, cdiv(p.VT, want_chunks));
  if (!p.wide) per = (int)std::min<unsigned long long>((unsigned long long)per, fit);
  if (p.wide == 2) per = (int)std::min<unsigned long long>((unsigned long long)per, fit_split);
  p.nchunk = cdiv(p.VT, per);
  p.vt_per_chunk = cdiv(p.VT, p.nchunk);                  // same number of chunks, evenly filled
  p.a_bytes = align256((size_t)p.P * p.MP * p.g.T * p.ks16 * 512);
  p.part_bytes = align256((size_t)p.nchunk * M * p.Lout * (p.wide ? 8 : 4));
  p.ws_bytes = p.a_bytes + p.part_bytes;
  return p;
}

struct UpdPlan {
  int KB, NB, mchunks, m_per_chunk, parts;   // parts: partial sums per batch chunk (padding waves reused)
  size_t ws_bytes;
};

UpdPlan plan_update(int M, int K, int N) {
  UpdPlan p;
  p.KB = cdiv(K, 128);
  p.NB = cdiv(N, 128);
  const int tiles = p.KB * p.NB;
  int want = std::max(1, cdiv(1024, tiles));
  int per = std::max(kGradMS, cdiv(cdiv(M, want), kGradMS) * kGradMS);
  p.m_per_chunk = per;
  p.mchunks = cdiv(M, per);
  p.parts = (K <= 64 ? 2 : 1) * (N <= 64 ? 2 : 1);
  p.ws_bytes = align256((size_t)p.mchunks * p.parts * K * N * sizeof(float));
  return p;
}

template <int PM, int KSMAX, int TERMS, bool PER_ARRAY>
hipError_t launch_vmm_variant(const VmmArgs& a, const VmmPlan& p, bool codes, hipStream_t st) {
  const dim3 grid((unsigned)(a.per_xcd * 8)), block((unsigned)(p.nw * 64));
  void (*k)(VmmArgs);
  if (p.wide == 2 && !codes) k = vmm_kernel<PM, KSMAX, TERMS, 2, false, PER_ARRAY>;
  else if (p.wide) k = codes ? vmm_kernel<PM, KSMAX, TERMS, 1, true, PER_ARRAY> : vmm_kernel<PM, KSMAX, TERMS, 1, false, PER_ARRAY>;
  else k = codes ? vmm_kernel<PM, KSMAX, TERMS, 0, true, PER_ARRAY> : vmm_kernel<PM, KSMAX, TERMS, 0, false, PER_ARRAY>;
  if (p.lds_bytes > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)p.lds_bytes);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(k, grid, block, p.lds_bytes, st, a);
  return hipGetLastError();
}

template <int NT, bool PER_ARRAY>
hipError_t launch_vmm6_variant(const VmmArgs& a, const VmmPlan& p, bool codes, hipStream_t st) {
  const dim3 grid((unsigned)(a.per_xcd * 8)), block((unsigned)(p.nw * 64));
  void (*k)(VmmArgs);
  if (p.wide == 2 && !codes) k = vmm6_kernel<NT, 2, false, PER_ARRAY>;
  else if (p.wide) k = codes ? vmm6_kernel<NT, 1, true, PER_ARRAY> : vmm6_kernel<NT, 1, false, PER_ARRAY>;
  else k = codes ? vmm6_kernel<NT, 0, true, PER_ARRAY> : vmm6_kernel<NT, 0, false, PER_ARRAY>;
  if (p.lds_bytes > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)p.lds_bytes);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(k, grid, block, p.lds_bytes, st, a);
  return hipGetLastError();
}

hipError_t launch_vmm6(const VmmArgs& a, const VmmPlan& p, int terms, bool codes, hipStream_t st) {
  if (a.npol == 2) return launch_vmm6_variant<5, true>(a, p, codes, st);   // single arrays: always the full schedule
  switch (terms) {
    case 1: return launch_vmm6_variant<1, false>(a, p, codes, st);
    case 4: return launch_vmm6_variant<4, false>(a, p, codes, st);
    case 5: return launch_vmm6_variant<5, false>(a, p, codes, st);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_vmm(const VmmArgs& a, const VmmPlan& p, int terms, bool codes, hipStream_t st) {
  const int ks = p.g.ks;
  if (a.npol == 2)                                    // planes of single arrays always come in two terms
    return ks <= 8 ? launch_vmm_variant<2, 8, 2, true>(a, p, codes, st) : launch_vmm_variant<1, 16, 2, true>(a, p, codes, st);
  if (ks <= 8) return terms == 2 ? launch_vmm_variant<2, 8, 2, false>(a, p, codes, st) : launch_vmm_variant<2, 8, 1, false>(a, p, codes, st);
  return terms == 2 ? launch_vmm_variant<1, 16, 2, false>(a, p, codes, st) : launch_vmm_variant<1, 16, 1, false>(a, p, codes, st);
}

int run_vmm(const xbar_config* cfg, const void* planes, const float* in, float* out, int M, int K, int N,
            float w_max, float in_scale, void* ws, size_t ws_bytes, int16_t* codes, void* stream, bool transposed,
            const ConvGeom* conv = nullptr, unsigned long long* hist = nullptr) {
  int rc = xbar_config_validate(cfg);
  if (rc) return rc;
  if ((rc = check_shape(M, K, N))) return rc;
  if (!aligned16(planes) || !aligned16(in) || (!hist && !aligned16(out)) || !aligned16(ws)) return XBAR_EALIGN;
  if (codes && (reinterpret_cast<uintptr_t>(codes) & 1u)) return XBAR_EALIGN;
  if (!finite_pos(w_max) || !finite_pos(in_scale)) return XBAR_EINVAL;
  // DAC level table: with 1-bit cycles (the paper's streaming scheme) and a zero level at 0 V the
  // table is one factor on every current, which goes into the ADC gain.
  // Other tables run through the general kernel variants, one contraction per level.
  float dac_gain = 1.0f;
  bool level_table = false;
  if (cfg->flags & XBAR_DAC_LUT) {
    if (cfg->stream_bits == 1 && cfg->dac_lut[0] == 0.0f) dac_gain = cfg->dac_lut[1];
    else if (cfg->stream_bits <= 4) level_table = true;
    else return XBAR_ENOTSUP;                        // the table has 16 entries
  }
  const Derived d = derive(cfg);
  const VmmPlan p = plan_vmm(cfg, d, M, K, N, transposed);
  // the statistics pass writes no partial sums: the staged input is all it needs
  if (ws_bytes < (hist ? p.a_bytes : p.ws_bytes)) return XBAR_EWORKSPACE;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const float adc_fs = transposed ? cfg->adc_fs_bwd : cfg->adc_fs_fwd;

  QuantArgs qa;
  qa.X = in;
  qa.A = reinterpret_cast<uint8_t*>(ws);
  qa.M = M; qa.L = p.Lin; qa.MP = p.MP; qa.T = p.g.T; qa.ks = p.ks16; qa.tile = p.g.tile; qa.P = p.P;
  qa.input_bits = cfg->input_bits;
  qa.offset = p.offset;
  qa.scale = in_scale;
  qa.n_threads = (long long)p.MP * p.g.T * ((p.ks16 + 1) / 2) * 64;
  if (conv) {
    qa.conv = *conv;
    hipLaunchKernelGGL(quantize_input_kernel<true>, dim3((unsigned)((qa.n_threads + 255) / 256)), dim3(256), 0, st, qa);
  } else {
    hipLaunchKernelGGL(quantize_input_kernel<false>, dim3((unsigned)((qa.n_threads + 255) / 256)), dim3(256), 0, st, qa);
  }
  if (hipGetLastError() != hipSuccess) return XBAR_EHIP;

  const PlaneGeom gf = plane_geom(cfg, d, K, N, false);
  VmmArgs a;
  a.A = reinterpret_cast<const u32x2*>(ws);
  a.B = reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(planes) + (transposed ? align256(gf.bytes) : 0));
  a.part = reinterpret_cast<char*>(ws) + p.a_bytes;
  a.codes = codes;
  a.hist = hist;
  a.adc_curve_on = (cfg->flags & XBAR_ADC_CURVE) ? 1 : 0;
  for (int i = 0; i < 17; ++i) a.adc_curve[i] = cfg->adc_curve[i];
  a.q_adc = (float)d.q_adc;
  a.inv_q_adc = 1.0f / (float)d.q_adc;
  a.dac_levels = level_table ? 1 << cfg->stream_bits : 0;
  // table entries are voltages over v_max; one input level is v_max / (2^stream_bits - 1)
  for (int i = 0; i < 16; ++i) a.dac_lut[i] = (float)((double)cfg->dac_lut[i] * (double)((1 << cfg->stream_bits) - 1));
  a.M = M; a.Lin = p.Lin; a.Lout = p.Lout; a.MP = p.MP; a.OP = p.g.OP; a.MB = p.MB; a.T = p.g.T; a.P = p.P;
  a.npol = d.npol; a.pol_stride = p.g.pol_bytes / 16;
  a.VT = p.VT; a.S_w = d.S_w; a.S_in = d.S_in; a.slice_bits = cfg->slice_bits; a.stream_bits = cfg->stream_bits;
  a.ks = p.g.ks; a.tile = p.g.tile; a.vt_per_chunk = p.vt_per_chunk; a.nchunk = p.nchunk; a.lds_kb = p.lds_kb;
  a.ks16 = p.ks16; a.sg = p.sg;
  a.scale_lo = a.scale_hi = 0;
  for (int j = 0; j < kMaxTermsF6; ++j) {
    const int byte = 127 + d.term_exp[j];
    if (j < 4) a.scale_lo |= byte << (8 * j);
    else a.scale_hi |= byte;
  }
  const bool general = codes != nullptr || hist != nullptr || level_table || a.adc_curve_on;
  const bool split = p.wide == 2 && !general;          // adds its groups up in the partial-sum buffer
  a.split_sg = p.split_sg;
  a.direct = (p.nchunk == 1 && !p.offset && !split) ? 1 : 0;
  a.total_wg = p.nchunk * p.g.OP * p.MB;
  a.per_xcd = cdiv(a.total_wg, 8);
  a.gain = (float)d.q_adc / adc_fs * dac_gain;
  a.clamp_lo = kMagic - (float)d.q_adc;
  a.clamp_hi = kMagic + (float)d.q_adc;
  a.bias_per_vt = split ? p.bias_split : p.bias_per_vt;
  a.out = out;
  {
    const double lsb = (double)adc_fs / (double)d.q_adc;
    const double qa_max = (double)((1u << cfg->input_bits) - 1), qw_max = (double)((1u << cfg->weight_bits) - 1);
    a.scale = lsb * (double)in_scale * (double)w_max / (qa_max * qw_max);
    if (p.offset) a.scale = 2.0 * a.scale;           // coded value = (2 u - Qa) / Qa
  }
  hipEvent_t ev0 = g_trace_before, ev1 = g_trace_after;
  g_trace_before = g_trace_after = nullptr;
  if (ev0 && hipEventRecord(ev0, st) != hipSuccess) return XBAR_EHIP;
  if ((d.fmt == kFmtF6 ? launch_vmm6(a, p, d.terms, general, st) : launch_vmm(a, p, d.terms, general, st)) != hipSuccess)
    return XBAR_EHIP;
  if (ev1 && hipEventRecord(ev1, st) != hipSuccess) return XBAR_EHIP;
  if (hist) return XBAR_OK;

  if (!a.direct) {
    FinishArgs f;
    f.part = a.part;
    f.out = out;
    f.n = (long long)M * p.Lout;
    f.nchunk = p.nchunk;
    f.wide = p.wide != 0;
    f.Lout = p.Lout;
    f.scale = a.scale;
    f.wsum = nullptr;
    f.half_range = 0.0;
    if (p.offset) {    // minus the half-range times the sum of the programmed weights of this output
      const long long* sums = reinterpret_cast<const long long*>(reinterpret_cast<const char*>(planes) +
                                                                  weight_sums_offset(cfg, d, K, N));
      f.wsum = transposed ? sums + N : sums;
      f.half_range = (double)in_scale * (double)w_max / (double)((1u << cfg->weight_bits) - 1);
    }
    hipLaunchKernelGGL(vmm_finish_kernel, dim3((unsigned)((f.n + 255) / 256)), dim3(256), 0, st, f);
    if (hipGetLastError() != hipSuccess) return XBAR_EHIP;
  }
  return XBAR_OK;
}


int run_update(const xbar_config* cfg, float* W, const float* X, const float* dY, int M, int K, int N, float w_max,
               float grad_scale, float lr, uint64_t step, void* ws, size_t ws_bytes, void* hip_stream, const ConvGeom* conv) {
  int rc = xbar_config_validate(cfg);
  if (rc) return rc;
  if ((rc = check_shape(M, K, N))) return rc;
  if (!aligned16(W) || !aligned16(X) || !aligned16(dY) || !aligned16(ws)) return XBAR_EALIGN;
  if (!finite_pos(w_max) || !std::isfinite(grad_scale) || !std::isfinite(lr)) return XBAR_EINVAL;
  const UpdPlan p = plan_update(M, K, N);
  if (ws_bytes < p.ws_bytes) return XBAR_EWORKSPACE;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  GradArgs g;
  g.X = X; g.D = dY; g.part = reinterpret_cast<float*>(ws);
  g.M = M; g.K = K; g.N = N; g.KB = p.KB; g.NB = p.NB; g.m_per_chunk = p.m_per_chunk;
  {
    const dim3 grid((unsigned)(p.KB * p.NB), (unsigned)p.mchunks), block(256);
    if (conv) {
      g.conv = *conv;
      if (K <= 64 && N <= 64) hipLaunchKernelGGL((grad_gemm_kernel<true, true, true>), grid, block, 0, st, g);
      else if (K <= 64) hipLaunchKernelGGL((grad_gemm_kernel<true, false, true>), grid, block, 0, st, g);
      else if (N <= 64) hipLaunchKernelGGL((grad_gemm_kernel<false, true, true>), grid, block, 0, st, g);
      else hipLaunchKernelGGL((grad_gemm_kernel<false, false, true>), grid, block, 0, st, g);
    } else {
      if (K <= 64 && N <= 64) hipLaunchKernelGGL((grad_gemm_kernel<true, true, false>), grid, block, 0, st, g);
      else if (K <= 64) hipLaunchKernelGGL((grad_gemm_kernel<true, false, false>), grid, block, 0, st, g);
      else if (N <= 64) hipLaunchKernelGGL((grad_gemm_kernel<false, true, false>), grid, block, 0, st, g);
      else hipLaunchKernelGGL((grad_gemm_kernel<false, false, false>), grid, block, 0, st, g);
    }
  }
  if (hipGetLastError() != hipSuccess) return XBAR_EHIP;
  WriteArgs w;
  w.W = W; w.part = g.part; w.n = (long long)K * N; w.mchunks = p.mchunks * p.parts; w.flags = cfg->flags;
  w.w_max = (double)w_max; w.grad_scale = (double)grad_scale; w.lr = (double)lr;
  w.v = (double)cfg->upd_nl_v; w.gamma = (double)cfg->upd_noise_gamma;
  w.seed = cfg->seed; w.step = step; w.step_add = current_step_source();
  hipLaunchKernelGGL(update_write_kernel, dim3((unsigned)((w.n + 31) / 32)), dim3(256), 0, st, w);
  if (hipGetLastError() != hipSuccess) return XBAR_EHIP;
  return XBAR_OK;
}

}  // namespace

namespace xbar_detail {
// Checks a convolution geometry and derives the layer's matrix shape: M = batch x output positions,
// K = kernel height x kernel width x input channels.
int conv_dims(const xbar_conv_geom* q, ConvGeom* g, int* M, int* K) {
  if (!q) return XBAR_EINVAL;
  if (q->batch <= 0 || q->in_h <= 0 || q->in_w <= 0 || q->in_c <= 0 || q->k_h <= 0 || q->k_w <= 0 || q->stride <= 0 ||
      q->pad < 0 || q->out_h <= 0 || q->out_w <= 0)
    return XBAR_ESHAPE;
  if (q->in_h + 2 * q->pad < q->k_h || q->in_w + 2 * q->pad < q->k_w) return XBAR_ESHAPE;
  if (q->out_h != (q->in_h + 2 * q->pad - q->k_h) / q->stride + 1 ||
      q->out_w != (q->in_w + 2 * q->pad - q->k_w) / q->stride + 1)
    return XBAR_ESHAPE;
  const long long m = (long long)q->batch * q->out_h * q->out_w, k = (long long)q->k_h * q->k_w * q->in_c;
  const long long pixels = (long long)q->batch * q->in_h * q->in_w * q->in_c;
  if (m >= (1ll << 31) || k >= (1ll << 31) || pixels >= (1ll << 38)) return XBAR_ESHAPE;
  g->H = q->in_h; g->W = q->in_w; g->C = q->in_c; g->KH = q->k_h; g->KW = q->k_w;
  g->stride = q->stride; g->pad = q->pad; g->OH = q->out_h; g->OW = q->out_w;
  *M = (int)m;
  *K = (int)k;
  return XBAR_OK;
}

const unsigned long long* current_step_source() { return g_step_source; }
}  // namespace xbar_detail

// ---------------------------------------------------------------------------------------------
// C ABI
// ---------------------------------------------------------------------------------------------
extern "C" {

uint32_t xbar_abi_version(void) { return XBAR_ABI_VERSION; }

int xbar_probe_mfma_rate(int mode, int iters, void* out, size_t out_bytes, void* hip_stream) {
  if (mode < 0 || mode > 3 || iters <= 0 || iters > (1 << 24)) return XBAR_EINVAL;
  if (!aligned16(out)) return XBAR_EALIGN;
  if (out_bytes < (size_t)512 * 256 * sizeof(float)) return XBAR_EWORKSPACE;
  if (mode >= 2) {
    hipLaunchKernelGGL(mfma_probe_i8_kernel, dim3(512), dim3(256), 0, reinterpret_cast<hipStream_t>(hip_stream),
                       reinterpret_cast<int*>(out), iters, mode);
    return hipGetLastError() == hipSuccess ? XBAR_OK : XBAR_EHIP;
  }
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(512), dim3(256), 0, reinterpret_cast<hipStream_t>(hip_stream),
                     reinterpret_cast<float*>(out), iters, mode);
  return hipGetLastError() == hipSuccess ? XBAR_OK : XBAR_EHIP;
}

void xbar_set_step_source(const unsigned long long* device_step) { g_step_source = device_step; }

int xbar_step_advance(unsigned long long* device_step, void* hip_stream) {
  if (!device_step || (reinterpret_cast<uintptr_t>(device_step) & 7u)) return XBAR_EALIGN;
  hipLaunchKernelGGL(step_advance_kernel, dim3(1), dim3(1), 0, reinterpret_cast<hipStream_t>(hip_stream), device_step);
  return hipGetLastError() == hipSuccess ? XBAR_OK : XBAR_EHIP;
}

void xbar_trace_next_vmm(void* before, void* after) {
  g_trace_before = reinterpret_cast<hipEvent_t>(before);
  g_trace_after = reinterpret_cast<hipEvent_t>(after);
}

const char* xbar_strerror(int code) {
  switch (code) {
    case XBAR_OK: return "ok";
    case XBAR_EINVAL: return "invalid parameter struct or scalar argument";
    case XBAR_ESHAPE: return "M, K, N must be positive, K*N below 2^31 and M*K, M*N below 2^38 elements";
    case XBAR_EALIGN: return "null or misaligned pointer (16 bytes required)";
    case XBAR_EWORKSPACE: return "workspace or plane buffer too small";
    case XBAR_EHIP: return "HIP kernel launch failed";
    case XBAR_ENOTSUP: return "not supported by the GPU kernels";
    default: return "unknown xbar status";
  }
}

int xbar_config_validate(const xbar_config* c) {
  if (!c) return XBAR_EINVAL;
  if (c->struct_size != sizeof(xbar_config) || c->abi_version != XBAR_ABI_VERSION) return XBAR_EINVAL;
  if (c->xbar_rows < 16 || c->xbar_rows > 256 || c->xbar_rows % 16) return XBAR_EINVAL;
  if (c->xbar_cols < 16 || c->xbar_cols > 256 || c->xbar_cols % 16) return XBAR_EINVAL;
  if (c->slice_bits < 1 || c->slice_bits > 4) return XBAR_EINVAL;
  if (c->weight_bits < 1 || c->weight_bits > 16 || c->weight_bits % c->slice_bits) return XBAR_EINVAL;
  if (c->input_bits < 1 || c->input_bits > 8) return XBAR_EINVAL;
  if (c->stream_bits < 1 || c->stream_bits > c->input_bits || c->input_bits % c->stream_bits) return XBAR_EINVAL;
  if (c->adc_bits < 2 || c->adc_bits > 16) return XBAR_EINVAL;
  if (c->flags & ~0xFFFu) return XBAR_EINVAL;
  if (c->flags & XBAR_ADC_PER_ARRAY) {
    if (c->flags & XBAR_ADC_CURVE) return XBAR_EINVAL;     // the curve is that of a signed converter
    if (c->adc_bits > 15) return XBAR_EINVAL;              // unsigned codes are reported as int16
  }
  if (c->flags & XBAR_ADC_CURVE)
    for (int i = 0; i < 17; ++i) {
      if (!std::isfinite(c->adc_curve[i]) || c->adc_curve[i] < -1.0f || c->adc_curve[i] > 1.0f) return XBAR_EINVAL;
      if (i && c->adc_curve[i] < c->adc_curve[i - 1]) return XBAR_EINVAL;     // a converter is monotone
    }
  {  // at most one wire model
    const uint32_t w = c->flags & (XBAR_NI_WIRE_AAM | XBAR_NI_WIRE_PROFILE | XBAR_NI_WIRE_AAM2);
    if (w & (w - 1)) return XBAR_EINVAL;
  }
  if (!finite_pos(c->r_min) || !finite_pos(c->r_max) || !(c->r_max > c->r_min)) return XBAR_EINVAL;
  if (!finite_pos(c->v_max)) return XBAR_EINVAL;
  if (!finite_nonneg(c->r_row) || !finite_nonneg(c->r_col) || !finite_nonneg(c->r_source) ||
      !finite_nonneg(c->r_sense))
    return XBAR_EINVAL;
  if (!finite_nonneg(c->var_sigma) || !finite_nonneg(c->upd_nl_v) || !finite_nonneg(c->upd_noise_gamma))
    return XBAR_EINVAL;
  if (!finite_pos(c->adc_fs_fwd) || !finite_pos(c->adc_fs_bwd)) return XBAR_EINVAL;
  if (c->flags & XBAR_DAC_LUT)
    for (int i = 0; i < (1 << c->stream_bits) && i < 16; ++i)
      if (!std::isfinite(c->dac_lut[i])) return XBAR_EINVAL;
  return XBAR_OK;
}

size_t xbar_planes_bytes(const xbar_config* cfg, int K, int N) {
  if (xbar_config_validate(cfg) || check_shape(1, K, N)) return 0;
  const Derived d = derive(cfg);
  return weight_sums_offset(cfg, d, K, N) + weight_sums_bytes(cfg, K, N);
}

size_t xbar_workspace_bytes(const xbar_config* cfg, int op, int M, int K, int N) {
  if (xbar_config_validate(cfg) || check_shape(M, K, N)) return 0;
  const Derived d = derive(cfg);
  if (op == XBAR_OP_FWD) return plan_vmm(cfg, d, M, K, N, false).ws_bytes;
  if (op == XBAR_OP_BWD) return plan_vmm(cfg, d, M, K, N, true).ws_bytes;
  if (op == XBAR_OP_UPDATE) return plan_update(M, K, N).ws_bytes;
  if (op == XBAR_OP_FCM) return fcm_workspace_bytes(cfg, K, N);
  if (op == XBAR_OP_UPDATE_PULSED) return pulsed_workspace_bytes(M, K, N);
  return 0;
}

int xbar_tile(const xbar_config* cfg, const float* W, int K, int N, float w_max, uint64_t step, const float* profile,
              void* planes, size_t planes_bytes, void* hip_stream) {
  int rc = xbar_config_validate(cfg);
  if (rc) return rc;
  if ((rc = check_shape(1, K, N))) return rc;
  if (!aligned16(W) || !aligned16(planes)) return XBAR_EALIGN;
  if ((cfg->flags & XBAR_NI_WIRE_PROFILE) && !aligned16(profile)) return XBAR_EALIGN;
  if (!finite_pos(w_max)) return XBAR_EINVAL;
  if (planes_bytes < xbar_planes_bytes(cfg, K, N)) return XBAR_EWORKSPACE;
  const Derived d = derive(cfg);
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  double* wire_u = nullptr;
  if (cfg->flags & XBAR_NI_WIRE_AAM2) {
    wire_u = reinterpret_cast<double*>(reinterpret_cast<char*>(planes) + align256(plane_geom(cfg, d, K, N, false).bytes) +
                                       align256(plane_geom(cfg, d, K, N, true).bytes));
    if ((rc = launch_wire_model(cfg, W, K, N, w_max, step, wire_u, st))) return rc;
  }
  if (cfg->flags & XBAR_INPUT_OFFSET) {
    SumArgs sa;
    sa.W = W;
    sa.colsum = reinterpret_cast<long long*>(reinterpret_cast<char*>(planes) + weight_sums_offset(cfg, d, K, N));
    sa.rowsum = sa.colsum + N;
    sa.K = K; sa.N = N; sa.weight_bits = cfg->weight_bits; sa.w_max = w_max;
    hipLaunchKernelGGL(clear_sums_kernel, dim3((unsigned)cdiv(std::max(K, N), 256)), dim3(256), 0, st, sa);
    if (hipGetLastError() != hipSuccess) return XBAR_EHIP;
    hipLaunchKernelGGL(weight_sums_kernel, dim3((unsigned)(cdiv(K, 64) * cdiv(N, 64))), dim3(256), 0, st, sa);
    if (hipGetLastError() != hipSuccess) return XBAR_EHIP;
  }
  size_t offset = 0;
  for (int dir = 0; dir < 2; ++dir)
  for (int pol = 0; pol < d.npol; ++pol) {
    const PlaneGeom g = plane_geom(cfg, d, K, N, dir == 1);
    TileArgs a;
    a.W = W;
    a.profile = profile;
    a.wire_u = wire_u;
    a.pol_out = d.npol == 2 ? pol : -1;
    a.planes = reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(planes) + offset + (size_t)pol * g.pol_bytes);
    a.K = K; a.N = N; a.R = cfg->xbar_rows; a.C = cfg->xbar_cols; a.S_w = d.S_w;
    a.slice_bits = cfg->slice_bits; a.weight_bits = cfg->weight_bits; a.terms = d.terms;
    a.tile = g.tile; a.ks = g.ks; a.T = g.T; a.OP = g.OP;
    a.flags = cfg->flags;
    a.g_min = 1.0 / (double)cfg->r_max;
    a.dg = (1.0 / (double)cfg->r_min - a.g_min) / (double)((1 << cfg->slice_bits) - 1);
    a.var_sigma = (double)cfg->var_sigma;
    a.r_row = (double)cfg->r_row;
    a.r_col = (double)cfg->r_col;
    a.r_source = (double)cfg->r_source;
    a.r_sense = (double)cfg->r_sense;
    {  // |U| < 2^slice_bits: fp16 holds multiples of 2^-(11 - slice_bits) below that bound exactly; one
       // array alone adds the off-state conductance (below the full range for on/off ratios from 2): one bit less
      const int hi_frac = (d.npol == 2 ? 10 : 11) - cfg->slice_bits;
      a.hi_scale = std::ldexp(1.0, hi_frac);
      a.hi_inv_scale = std::ldexp(1.0, -hi_frac);
    }
    a.w_max = w_max;
    a.seed = cfg->seed;
    a.step = step;
    a.step_add = current_step_source();
    for (int j = 0; j < kMaxTermsF6; ++j) a.term_exp[j] = d.term_exp[j];
    // every k-step that the contraction reads is written whole, padding included
    const int Lc = dir == 1 ? N : K;
    if (d.fmt == kFmtF6) {
      a.n_threads = (long long)g.T * g.ks * 8 * g.OP * 32;
      const unsigned blocks = (unsigned)((a.n_threads + 255) / 256);
      if (dir == 0) hipLaunchKernelGGL(tile_planes_f6_kernel<false>, dim3(blocks, (unsigned)d.S_w), dim3(256), 0, st, a);
      else hipLaunchKernelGGL(tile_planes_f6_kernel<true>, dim3(blocks, (unsigned)d.S_w), dim3(256), 0, st, a);
      if (hipGetLastError() != hipSuccess) return XBAR_EHIP;
      if (pol == d.npol - 1) offset += align256(g.bytes);
      continue;
    }
    const long long chunks = (long long)cdiv(Lc, 16) * 2;
    a.n_threads = chunks * g.OP * 32;
    const unsigned blocks = (unsigned)((a.n_threads + 255) / 256);
    if (dir == 0) hipLaunchKernelGGL(tile_planes_kernel<false>, dim3(blocks, (unsigned)d.S_w), dim3(256), 0, st, a);
    else hipLaunchKernelGGL(tile_planes_kernel<true>, dim3(blocks, (unsigned)d.S_w), dim3(256), 0, st, a);
    if (hipGetLastError() != hipSuccess) return XBAR_EHIP;
    if (pol == d.npol - 1) offset += align256(g.bytes);
  }
  return XBAR_OK;
}

int xbar_fwd(const xbar_config* cfg, const void* planes, const float* X, float* Y, int M, int K, int N, float w_max,
             float x_scale, void* ws, size_t ws_bytes, int16_t* codes, void* hip_stream) {
  return run_vmm(cfg, planes, X, Y, M, K, N, w_max, x_scale, ws, ws_bytes, codes, hip_stream, false);
}

int xbar_bwd(const xbar_config* cfg, const void* planes, const float* dY, float* dX, int M, int K, int N, float w_max,
             float g_scale, void* ws, size_t ws_bytes, int16_t* codes, void* hip_stream) {
  return run_vmm(cfg, planes, dY, dX, M, K, N, w_max, g_scale, ws, ws_bytes, codes, hip_stream, true);
}

int xbar_update(const xbar_config* cfg, float* W, const float* X, const float* dY, int M, int K, int N, float w_max,
                float grad_scale, float lr, uint64_t step, void* ws, size_t ws_bytes, void* hip_stream) {
  return run_update(cfg, W, X, dY, M, K, N, w_max, grad_scale, lr, step, ws, ws_bytes, hip_stream, nullptr);
}

size_t xbar_conv_workspace_bytes(const xbar_config* cfg, int op, const xbar_conv_geom* geom, int N) {
  ConvGeom g;
  int M, K;
  if (xbar_config_validate(cfg) || conv_dims(geom, &g, &M, &K) || check_shape(M, K, N)) return 0;
  const Derived d = derive(cfg);
  if (op == XBAR_OP_FWD) return plan_vmm(cfg, d, M, K, N, false).ws_bytes;
  if (op == XBAR_OP_BWD) return plan_vmm(cfg, d, M, K, N, true).ws_bytes + align256((size_t)M * K * sizeof(float));
  if (op == XBAR_OP_UPDATE) return plan_update(M, K, N).ws_bytes;
  if (op == XBAR_OP_UPDATE_PULSED) return pulsed_workspace_bytes(M, K, N);
  return 0;
}

int xbar_conv_fwd(const xbar_config* cfg, const void* planes, const float* X, float* Y, const xbar_conv_geom* geom,
                  int N, float w_max, float x_scale, void* ws, size_t ws_bytes, int16_t* codes, void* hip_stream) {
  ConvGeom g;
  int M, K;
  const int rc = conv_dims(geom, &g, &M, &K);
  if (rc) return rc;
  return run_vmm(cfg, planes, X, Y, M, K, N, w_max, x_scale, ws, ws_bytes, codes, hip_stream, false,
                 conv_is_dense(geom) ? nullptr : &g);
}

int xbar_conv_bwd(const xbar_config* cfg, const void* planes, const float* dY, float* dX, const xbar_conv_geom* geom,
                  int N, float w_max, float g_scale, void* ws, size_t ws_bytes, void* hip_stream) {
  ConvGeom g;
  int M, K;
  int rc = conv_dims(geom, &g, &M, &K);
  if (rc) return rc;
  if ((rc = xbar_config_validate(cfg))) return rc;
  if ((rc = check_shape(M, K, N))) return rc;
  if (!aligned16(dX) || !aligned16(ws)) return XBAR_EALIGN;
  const size_t need = xbar_conv_workspace_bytes(cfg, XBAR_OP_BWD, geom, N);
  if (ws_bytes < need) return XBAR_EWORKSPACE;
  if (conv_is_dense(geom))       // every pixel is its own patch: the crossbar output is the result
    return run_vmm(cfg, planes, dY, dX, M, K, N, w_max, g_scale, ws, ws_bytes, nullptr, hip_stream, true);
  const size_t col_bytes = align256((size_t)M * K * sizeof(float));
  float* col = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + (need - col_bytes));
  if ((rc = run_vmm(cfg, planes, dY, col, M, K, N, w_max, g_scale, ws, need - col_bytes, nullptr, hip_stream, true))) return rc;
  Col2imArgs c;
  c.col = col; c.dX = dX; c.conv = g; c.B = geom->batch; c.K = K;
  c.n = (long long)geom->batch * g.H * g.W * g.C;
  hipLaunchKernelGGL(col2im_kernel, dim3((unsigned)((c.n + 255) / 256)), dim3(256), 0,
                     reinterpret_cast<hipStream_t>(hip_stream), c);
  return hipGetLastError() == hipSuccess ? XBAR_OK : XBAR_EHIP;
}

int xbar_conv_update(const xbar_config* cfg, float* W, const float* X, const float* dY, const xbar_conv_geom* geom, int N,
                     float w_max, float grad_scale, float lr, uint64_t step, void* ws, size_t ws_bytes, void* hip_stream) {
  ConvGeom g;
  int M, K;
  const int rc = conv_dims(geom, &g, &M, &K);
  if (rc) return rc;
  return run_update(cfg, W, X, dY, M, K, N, w_max, grad_scale, lr, step, ws, ws_bytes, hip_stream,
                    conv_is_dense(geom) ? nullptr : &g);
}

namespace {
int run_histogram(const xbar_config* cfg, const void* planes, const float* in, int M, int K, int N, float in_scale, int op,
                  float bin_width, unsigned long long* hist, void* ws, size_t ws_bytes, void* hip_stream, const ConvGeom* conv);
}

int xbar_adc_histogram(const xbar_config* cfg, const void* planes, const float* in, int M, int K, int N, float in_scale,
                       int op, float bin_width, unsigned long long* hist, void* ws, size_t ws_bytes, void* hip_stream) {
  return run_histogram(cfg, planes, in, M, K, N, in_scale, op, bin_width, hist, ws, ws_bytes, hip_stream, nullptr);
}

int xbar_conv_adc_histogram(const xbar_config* cfg, const void* planes, const float* in, const xbar_conv_geom* geom, int N,
                            float in_scale, int op, float bin_width, unsigned long long* hist, void* ws, size_t ws_bytes,
                            void* hip_stream) {
  ConvGeom g;
  int M, K;
  const int rc = conv_dims(geom, &g, &M, &K);
  if (rc) return rc;
  // forward: the patches are gathered from the image; backward: the errors are a plain [M][N] matrix
  const bool gather = op == XBAR_OP_FWD && !conv_is_dense(geom);
  return run_histogram(cfg, planes, in, M, K, N, in_scale, op, bin_width, hist, ws, ws_bytes, hip_stream, gather ? &g : nullptr);
}

namespace {
int run_histogram(const xbar_config* cfg, const void* planes, const float* in, int M, int K, int N, float in_scale, int op,
                  float bin_width, unsigned long long* hist, void* ws, size_t ws_bytes, void* hip_stream, const ConvGeom* conv) {
  int rc = xbar_config_validate(cfg);
  if (rc) return rc;
  if (op != XBAR_OP_FWD && op != XBAR_OP_BWD) return XBAR_EINVAL;
  if (!finite_pos(bin_width)) return XBAR_EINVAL;
  if (!aligned16(hist)) return XBAR_EALIGN;
  // a converter with one code per bin: code = rne(I / bin_width), clamped to the last bin
  xbar_config c = *cfg;
  c.flags &= ~XBAR_ADC_CURVE;                        // the statistics are of the currents themselves
  c.adc_bits = (c.flags & XBAR_ADC_PER_ARRAY) ? 12 : 13;   // 4095 codes on the side(s) the converter has
  c.adc_fs_fwd = c.adc_fs_bwd = (float)(kStatBins - 1) * bin_width;
  if (!finite_pos(c.adc_fs_fwd)) return XBAR_EINVAL;
  return run_vmm(&c, planes, in, nullptr, M, K, N, 1.0f, in_scale, ws, ws_bytes, nullptr, hip_stream, op == XBAR_OP_BWD,
                 conv, hist);
}
}  // namespace

}  // extern "C"
