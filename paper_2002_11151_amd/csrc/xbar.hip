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
#include "vmm_device.h"

using namespace xbar_detail;

namespace {

// ---------------------------------------------------------------------------------------------
// generator: weights -> operand planes (Sec. IV-A, IV-D)
// ---------------------------------------------------------------------------------------------
struct TileArgs {
  const float* W;
  const float* profile;
  const uint32_t* codes; // term codes of every plane value (single-path wire model alone), this copy's orientation
  const double* wire_u;  // all-paths wire model: plane values [S_w][2][K][N], array index 0 (else unused)
  uint16_t* planes;  // start of this copy
  int K, N, R, C, S_w, slice_bits, weight_bits, terms;
  int tile, ks, T, OP;
  int spt;           // table-driven generator: slices per thread
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
// pol_out: -1: difference of the pair (array 0 minus array 1); 0 / 1: that array alone.
__device__ __forceinline__ double plane_value(const TileArgs& a, NormalStream& rng, int sign, int digit, int s, int k,
                                              int n, int pol_out) {
  if (a.flags & XBAR_NI_WIRE_AAM2) return a.wire_u[((size_t)(2 * s + (pol_out > 0 ? 1 : 0)) * a.K + k) * a.N + n];
  if (pol_out < 0 && !(a.flags & (XBAR_NI_VARIATION | XBAR_NI_WIRE_AAM | XBAR_NI_WIRE_PROFILE)))
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
  return (pol_out < 0 ? g[0] - g[1] : g[pol_out]) / a.dg;
}

__device__ __forceinline__ double plane_value(const TileArgs& a, NormalStream& rng, int sign, int digit, int s, int k,
                                              int n) {
  return plane_value(a, rng, sign, digit, s, k, n, a.pol_out);
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


// General 6-bit generator, first pass: one thread per device pair (k, n) and slice (blockIdx.y) computes the plane
// value -- quantisation, variation draw, wire model: the arithmetic of tile_planes_f6_kernel -- once, splits it
// into the terms of the schedule and stores the codes as one word per array: words[array][slice][k][n].
__global__ __launch_bounds__(256) void device_words_kernel(TileArgs a, uint32_t* words, int npol) {
  const long long tid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (tid >= (long long)a.K * a.N) return;
  const int n = (int)(tid % a.N), k = (int)(tid / a.N);
  const int s = blockIdx.y;
  NormalStream rng(a.seed, kStreamVariation, effective_step(a.step, a.step_add));
  const double qw = (double)((1u << a.weight_bits) - 1);
  const uint32_t dmask = (1u << a.slice_bits) - 1;
  const double q = ::rint(clampd((double)a.W[(size_t)k * a.N + n] / (double)a.w_max, -1.0, 1.0) * qw);
  const int sign = (q > 0.0) - (q < 0.0);
  const int digit = (int)(((uint32_t)::fabs(q) >> (a.slice_bits * s)) & dmask);
  for (int pol = 0; pol < npol; ++pol) {
    double left = plane_value(a, rng, sign, digit, s, k, n, npol == 2 ? pol : -1);
    uint32_t word = 0;
#pragma unroll
    for (int j = 0; j < kMaxTermsF6; ++j) {
      if (j >= a.terms) break;
      double v;
      const uint32_t code = e2m3_nearest(::ldexp(left, -a.term_exp[j]), v);
      left -= ::ldexp(v, a.term_exp[j]);
      word |= code << (6 * j);
    }
    words[(((size_t)pol * a.S_w + s) * a.K + k) * a.N + n] = word;
  }
}

// Second pass: one plane copy from the words of its array (a.codes: [slice][k][n]), integer work only.  One wave
// per fragment group (tile, output patch of 32, k-step of 64, slice): it reads the 64 x 32 words of its patch with
// whole-line loads (along n, the fastest index of the words, whichever index this copy contracts over), turns them
// through LDS, and every lane packs the 32 codes of its record for each term and writes it with one 16-byte and one
// 8-byte store.  a.n_threads: 64 x the number of fragment groups.
template <bool TRANSPOSED>
__global__ __launch_bounds__(256) void tile_planes_f6_words_kernel(TileArgs a) {
  __shared__ uint32_t turn[4][64][33];              // [wave][contraction entry][output], one word of padding per row
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const long long grp = (long long)blockIdx.x * 4 + wave;
  if (grp * 64 >= a.n_threads) return;              // whole waves leave: no block-wide barrier below
  const int J = (int)(grp % a.ks);
  const int op = (int)((grp / a.ks) % a.OP);
  const int t = (int)(grp / ((long long)a.ks * a.OP));
  const int s = blockIdx.y;
  const int Lc = TRANSPOSED ? a.N : a.K;
  const int Lo = TRANSPOSED ? a.K : a.N;
  const int rows = min(a.tile, Lc - t * a.tile);
  if (J * 64 >= rows) return;                       // the contraction never reads this k-step
  const int c_first = t * a.tile + J * 64;          // first contraction index of the group
  const int c_count = min(64, rows - J * 64);       // entries beyond it are padding (zero codes)
  const int o_first = op * 32;
  const uint32_t* words = a.codes + (size_t)s * a.K * a.N;
  uint32_t (&mine)[64][33] = turn[wave];
  if (TRANSPOSED) {                                 // words[k = output][n = contraction]: a row of 64 entries per output
    for (int ol = 0; ol < 32; ++ol) {
      const int o = o_first + ol;
      mine[lane][ol] = (o < Lo && lane < c_count) ? words[(size_t)o * a.N + c_first + lane] : 0u;
    }
  } else {                                          // words[k = contraction][n = output]: two rows of 32 outputs at a time
    for (int cl = lane >> 5; cl < 64; cl += 2) {
      const int o = o_first + (lane & 31);
      mine[cl][lane & 31] = (o < Lo && cl < c_count) ? words[(size_t)(c_first + cl) * a.N + o] : 0u;
    }
  }
  __builtin_amdgcn_wave_barrier();                  // one wave: its LDS writes are ordered before its LDS reads
  const int ol = lane & 31, half = lane >> 5;
  uint32_t rec[kMaxTermsF6][6];
#pragma unroll
  for (int j = 0; j < kMaxTermsF6; ++j)
#pragma unroll
    for (int x = 0; x < 6; ++x) rec[j][x] = 0u;
#pragma unroll
  for (int w = 0; w < 4; ++w)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t word = mine[w * 16 + half * 8 + e][ol];
      const int code_at = 8 * w + 2 * (e & 3) + (e >> 2);   // place of this entry among the lane's 32 codes
      const int bit = 6 * code_at, x = bit >> 5, sh = bit & 31;
#pragma unroll
      for (int j = 0; j < kMaxTermsF6; ++j) {
        if (j >= a.terms) break;
        const uint32_t code = (word >> (6 * j)) & 63u;
        rec[j][x] |= code << sh;
        if (sh > 26) rec[j][x + 1] |= code >> (32 - sh);
      }
    }
  const size_t frag0 = (((size_t)t * a.OP + op) * a.S_w + s) * a.terms * a.ks + J;
  uint8_t* base = reinterpret_cast<uint8_t*>(a.planes);
#pragma unroll
  for (int j = 0; j < kMaxTermsF6; ++j) {
    if (j >= a.terms) break;
    uint8_t* frag = base + (frag0 + (size_t)j * a.ks) * 1536;
    *reinterpret_cast<u32x4*>(frag + lane * 16) = u32x4{rec[j][0], rec[j][1], rec[j][2], rec[j][3]};
    *reinterpret_cast<u32x2*>(frag + 1024 + lane * 8) = u32x2{rec[j][4], rec[j][5]};
  }
}

// Term codes of the plane value of every (sign, digit, row, column): one thread per (digit, row, column)
// computes the value with the arithmetic of plane_value, splits it into the terms of the schedule and
// writes both signs in both orientations.
__global__ __launch_bounds__(256) void code_table_kernel(TileArgs a, uint32_t* table) {
  const int nd = (1 << a.slice_bits) - 1;
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= nd * a.R * a.C) return;
  const int j = idx % a.C, i = (idx / a.C) % a.R, digit = idx / (a.C * a.R) + 1;
  NormalStream rng(a.seed, kStreamVariation, 0);    // not drawn from: the table exists without variation only
  const size_t words = (size_t)2 * nd * a.R * a.C;
#pragma unroll
  for (int neg = 0; neg < 2; ++neg) {
    double left = plane_value(a, rng, neg ? -1 : 1, digit, 0, i, j);
    uint32_t word = 0;
    for (int t = 0; t < a.terms; ++t) {
      double v;
      const uint32_t code = e2m3_nearest(::ldexp(left, -a.term_exp[t]), v);
      left -= ::ldexp(v, a.term_exp[t]);
      word |= code << (6 * t);
    }
    const size_t plane = (size_t)(neg * nd + digit - 1) * a.R * a.C;
    table[plane + (size_t)i * a.C + j] = word;
    table[words + plane + (size_t)j * a.R + i] = word;
  }
}

// Planes in the 6-bit format from the table of term codes: the thread mapping and the records of
// tile_planes_f6_kernel; a plane value is one table word, looked up by (sign, digit, place in the array).
template <bool TRANSPOSED>
__global__ __launch_bounds__(256) void tile_planes_f6_table_kernel(TileArgs a) {
  const long long tid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (tid >= a.n_threads) return;
  const int out_len_pad = a.OP * 32;
  const int o = (int)(tid % out_len_pad);
  const int cg = (int)(tid / out_len_pad);
  const int slots = a.ks * 8;
  const int t = cg / slots, slot = cg - t * slots;
  const int within = slot * 8;
  const int Lc = TRANSPOSED ? a.N : a.K;
  const int Lo = TRANSPOSED ? a.K : a.N;
  const int rows = min(a.tile, Lc - t * a.tile);
  const int J = within >> 6;
  if (J * 64 >= rows) return;
  const int w = (within & 63) >> 4, half = (within & 15) >> 3;
  const int lane = (o & 31) + 32 * half;
  const int op = o >> 5;
  const int c0 = t * a.tile + within;
  const double qw = (double)((1u << a.weight_bits) - 1);
  const uint32_t dmask = (1u << a.slice_bits) - 1;
  const int nd = (int)dmask;
  // table of this orientation: [sign][digit - 1][contraction place][output place]
  const int out_len = TRANSPOSED ? a.R : a.C;       // places along the output index
  const uint32_t* codes = a.codes + (size_t)within * out_len + o % out_len;
  const size_t plane_words = (size_t)a.R * a.C;
  uint32_t mag[8];                                  // 0 for padding
  int first[8];                                     // table plane of digit 1 with the sign of the weight
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    mag[e] = 0;
    first[e] = 0;
    if (within + e >= rows || o >= Lo) continue;
    const int c = c0 + e;
    const int k = TRANSPOSED ? o : c, n = TRANSPOSED ? c : o;
    const double q = ::rint(clampd((double)a.W[(size_t)k * a.N + n] / (double)a.w_max, -1.0, 1.0) * qw);
    mag[e] = (uint32_t)::fabs(q);
    first[e] = q < 0.0 ? nd : 0;
  }
  uint8_t* base = reinterpret_cast<uint8_t*>(a.planes);
  const int s_end = min(a.S_w, ((int)blockIdx.y + 1) * a.spt);
  for (int s = (int)blockIdx.y * a.spt; s < s_end; ++s) {
    unsigned long long bits[kMaxTermsF6];
#pragma unroll
    for (int j = 0; j < kMaxTermsF6; ++j) bits[j] = 0ull;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int digit = (int)((mag[e] >> (a.slice_bits * s)) & dmask);
      if (!digit) continue;                          // both devices of the pair in the same state: exactly zero
      const uint32_t word = codes[(size_t)(first[e] + digit - 1) * plane_words + (size_t)e * out_len];
      const int nibble = 2 * (e & 3) + (e >> 2);     // where the input stage's byte e lands in the digit word
#pragma unroll
      for (int j = 0; j < kMaxTermsF6; ++j) {
        if (j >= a.terms) break;
        bits[j] |= (unsigned long long)((word >> (6 * j)) & 63u) << (6 * nibble);
      }
    }
    const size_t frag0 = (((size_t)t * a.OP + op) * a.S_w + s) * a.terms * a.ks + J;
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
  uint8_t* A;        // [phase][MP][T][ks][64 lanes][8 bytes]: magnitudes (fp16 path) or their nibbles (6-bit path)
  int M, L, MP, T, ks, tile, P, input_bits;
  int offset;        // signed inputs as offset-binary codes in one phase (P == 1)
  int nibbles;       // 6-bit path: a lane's 8 bytes nibble by nibble (word 0: low nibbles, word 1: high nibbles)
  float scale;
  long long n_threads;
  ConvGeom conv;     // used by the CONV instantiation only
};

// The 8 magnitudes of a lane (bytes of v.x, then of v.y) as the contraction kernel of the 6-bit path reads them:
// 4-bit field 2 j of word 0 holds the low nibble of byte j of v.x, field 2 j + 1 that of byte j of v.y; word 1
// the high nibbles in the same places.  A streaming cycle's digits are then one shift and one AND away.
__device__ __forceinline__ u32x2 nibble_words(u32x2 v) {
  u32x2 z;
  z.x = (v.x & 0x0f0f0f0fu) | ((v.y & 0x0f0f0f0fu) << 4);
  z.y = ((v.x >> 4) & 0x0f0f0f0fu) | (v.y & 0xf0f0f0f0u);
  return z;
}

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
    // The code is decided in double precision (as the oracle decides it).  The same expression in single
    // precision is within 255 x 3 x 2^-24 < 5e-5 of the exact value (one correctly rounded division, one
    // addition with offset coding, one product), so it rounds to the same code unless it lies within 1e-4 of
    // half a step: those few inputs (2e-4 of them) are decided again in double precision.
    int code[8];
    bool sure = true;
    const float qa_f = (float)qa, lo_f = (float)lo;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float r = x[e] / a.scale;
      const float y = (a.offset ? fminf(fmaxf((r + 1.0f) * 0.5f, 0.0f), 1.0f) : fminf(fmaxf(r, lo_f), 1.0f)) * qa_f;
      const float k = ::rintf(y);
      sure = sure && ::fabsf(y - k) <= 0.4999f;      // a NaN is not sure
      code[e] = (int)k;
    }
    if (!sure) {
#pragma unroll
      for (int e = 0; e < 8; ++e)
        code[e] = a.offset ? (int)::rint(clampd(((double)x[e] / scale + 1.0) * 0.5, 0.0, 1.0) * qa)
                           : (int)::rint(clampd((double)x[e] / scale, lo, 1.0) * qa);
    }
    if (a.offset) {
      // u = rne((x / scale + 1) / 2 * Qa): every input that exists is driven, a value of zero (also a
      // position outside the image) at mid-range; rows beyond the layer are not driven at all
      const int n_driven = m < a.M ? min(max(lend - l0, 0), 8) : 0;
#pragma unroll
      for (int e = 0; e < 8; ++e) pos.b[e] = (uint8_t)(e < n_driven ? code[e] : 0);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        pos.b[e] = (uint8_t)(code[e] > 0 ? code[e] : 0);
        neg.b[e] = (uint8_t)(code[e] < 0 ? -code[e] : 0);
      }
    }
    if (a.nibbles) {
      pos.v = nibble_words(pos.v);
      if (a.P == 2) neg.v = nibble_words(neg.v);
    }
    const size_t blk = ((size_t)mp * a.T + t) * a.ks + j;
    out[blk * 64 + lane] = pos.v;
    if (a.P == 2) out[((size_t)a.MP * a.T * a.ks + blk) * 64 + lane] = neg.v;
  }
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

// V consecutive outputs per thread (V = 4 where the row length allows it: 16-byte loads).
template <int V>
__global__ __launch_bounds__(256) void vmm_finish_kernel(FinishArgs a) {
#pragma clang fp contract(off)   // product, product, difference: each rounded on its own
  const long long i = ((long long)blockIdx.x * blockDim.x + threadIdx.x) * V;
  if (i >= a.n) return;
  long long sum[V];
#pragma unroll
  for (int v = 0; v < V; ++v) sum[v] = 0;
  for (int c = 0; c < a.nchunk; ++c) {
    if (a.wide) {
      const long long* src = reinterpret_cast<const long long*>(a.part) + (size_t)c * a.n + i;
      if constexpr (V == 4) {
        const longlong2 w0 = *reinterpret_cast<const longlong2*>(src), w1 = *reinterpret_cast<const longlong2*>(src + 2);
        sum[0] += w0.x; sum[1] += w0.y; sum[2] += w1.x; sum[3] += w1.y;
      } else {
        sum[0] += src[0];
      }
    } else {
      const int32_t* src = reinterpret_cast<const int32_t*>(a.part) + (size_t)c * a.n + i;
      if constexpr (V == 4) {
        const int4 w = *reinterpret_cast<const int4*>(src);
        sum[0] += w.x; sum[1] += w.y; sum[2] += w.z; sum[3] += w.w;
      } else {
        sum[0] += src[0];
      }
    }
  }
  float y[V];
#pragma unroll
  for (int v = 0; v < V; ++v) {
    double r = (double)sum[v] * a.scale;
    if (a.wsum) r = r - (double)a.wsum[(i + v) % a.Lout] * a.half_range;
    y[v] = (float)r;
  }
  if constexpr (V == 4) *reinterpret_cast<float4*>(a.out + i) = make_float4(y[0], y[1], y[2], y[3]);
  else a.out[i] = y[0];
}

// ---------------------------------------------------------------------------------------------
// update model (Sec. IV-C)
// ---------------------------------------------------------------------------------------------
struct GradArgs {
  const float* X;   // [M][K], or the NHWC image with CONV
  const float* D;   // [M][N]
  float* part;      // [mchunks][K][N]
  int M, K, N, KB, NB, m_per_chunk;
  int total_wg, per_xcd;   // blocks of the launch; logical blocks per XCD (the grid is 8 x per_xcd)
  ConvGeom conv;
};

constexpr int kGradMS = 32;   // batch rows per LDS stage = two k-steps of the bf16 matrix instruction
constexpr int kGradKS = kGradMS / 16;
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
  // consecutive block ids go to different XCDs; give each XCD a contiguous range of logical blocks, tiles
  // fastest, so that the tiles of one batch chunk (which read the same rows of X and dY) share one L2
  const int logical = (blockIdx.x & 7) * a.per_xcd + (blockIdx.x >> 3);
  if (logical >= a.total_wg) return;
  const int tile_id = logical % (a.KB * a.NB), chunk_id = logical / (a.KB * a.NB);
  const int kb = tile_id % a.KB, nb = tile_id / a.KB;
  const int k0 = kb * 128, n0 = nb * 128;
  const int m_begin = chunk_id * a.m_per_chunk;
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

  // staging: this thread fetches column (tid & 127) of half the rows of a stage: the groups of 8 rows
  // (tid >> 7), (tid >> 7) + 2, ...
  const int col = tid & 127, g_first = __builtin_amdgcn_readfirstlane(tid >> 7);   // the same for a whole wave
  float px[8 * kGradKS], pd[8 * kGradKS];
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
  // Loads without branches (a load behind a per-element bounds test costs two jumps and an execution-mask
  // round trip each): indices are clamped into the tensors here, and what lies outside is replaced by zero
  // where the values are used, one stage later, so that no load is waited for before the matrix instructions.
  const bool k_ok = k0 + col < a.K, n_ok = n0 + col < a.N;
  const int kc = min(k0 + col, a.K - 1), nc = min(n0 + col, a.N - 1);
  const long long conv_col = CONV ? ((long long)ckh * a.conv.W + ckw) * a.conv.C + cc : 0;
  uint32_t inside = 0;       // CONV: bit (q * 8 + e) set when that element of the fetched stage lies inside the image
  auto prefetch = [&](int m0, int buf) {
    // one 64-bit product per stage and operand; the row offsets are the same for every lane (scalar arithmetic)
    const float* xrow = a.X + (size_t)m0 * a.K + kc;
    const float* drow = a.D + (size_t)m0 * a.N + nc;
    const int last = a.M - 1 - m0;
    uint32_t in = 0;
#pragma unroll
    for (int q = 0; q < kGradKS; ++q)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int row = (g_first + 2 * q) * 8 + e;
        const int rc = min(row, last);
        if (CONV) {
          const ConvRow r = crow[buf][row];
          const int ih = r.ih0 + ckh, iw = r.iw0 + ckw;
          const bool ok = (ih >= 0) & (ih < a.conv.H) & (iw >= 0) & (iw < a.conv.W);
          px[q * 8 + e] = a.X[ok ? r.off + conv_col : 0];
          in |= (ok ? 1u : 0u) << (q * 8 + e);
        } else {
          px[q * 8 + e] = xrow[(size_t)rc * a.K];
        }
        pd[q * 8 + e] = drow[(size_t)rc * a.N];
      }
    inside = in;
  };
  int stage = 0;
  stage_rows(m_begin, 0);
  if (CONV) __syncthreads();
  prefetch(m_begin, 0);
  for (int m0 = m_begin; m0 < m_end; m0 += kGradMS, stage ^= 1) {
    if (m0 + kGradMS < m_end) stage_rows(m0 + kGradMS, stage ^ 1);
    __syncthreads();
#pragma unroll
    for (int q = 0; q < kGradKS; ++q) {
      bf16x8 xh, xl, dh, dl;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int row = (g_first + 2 * q) * 8 + e;
        const bool row_ok = m0 + row < m_end;
        const bool x_ok = row_ok & k_ok & (!CONV || ((inside >> (q * 8 + e)) & 1u) != 0);
        __bf16 h, l;
        split_bf16(x_ok ? px[q * 8 + e] : 0.0f, h, l);
        xh[e] = h; xl[e] = l;
        split_bf16((row_ok & n_ok) ? pd[q * 8 + e] : 0.0f, h, l);
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
    for (int ks = 0; ks < kGradKS; ++ks) {
      // batch shares: two shares alternate over the k-steps of a stage, four take one k-step in four
      if (PARTS == 2 && (ks & 1) != share) continue;
      if (PARTS == 4 && (ks & 3) != share) continue;
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
  float* out = a.part + ((size_t)chunk_id * PARTS + share) * a.K * a.N;
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
// The adding-up pass of a backward convolution: every input pixel gathers the patch errors that its
// places in the patches received, straight from the partial sums: the value of a patch entry is the one
// vmm_finish_kernel would store, and the entries of a pixel are added in single precision in the order
// (kernel row, kernel column).  The [M][K] matrix of patch errors is never written.
struct FinishCol2imArgs {
  FinishArgs f;      // f.out unused; f.n = M * K
  float* dX;         // NHWC
  ConvGeom conv;
  int K;
  long long n_img;
};

// V consecutive channels of a pixel per thread (V = 4 where the channel count allows it: 16-byte loads keep
// four times the bytes in flight, which is what bounds this pass).
template <int V>
__global__ __launch_bounds__(256) void vmm_finish_col2im_kernel(FinishCol2imArgs a) {
#pragma clang fp contract(off)   // product, product, difference: each rounded on its own
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t * V >= a.n_img) return;
  const ConvGeom& g = a.conv;
  const int c = (int)((t * V) % g.C);
  long long u = (t * V) / g.C;
  const int iw = (int)(u % g.W);
  u /= g.W;
  const int ih = (int)(u % g.H), b = (int)(u / g.H);
  float sum[V];
#pragma unroll
  for (int v = 0; v < V; ++v) sum[v] = 0.0f;
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
      const int k = (kh * g.KW + kw) * g.C + c;
      const long long i = m * a.K + k;
      long long acc[V];
#pragma unroll
      for (int v = 0; v < V; ++v) acc[v] = 0;
      for (int ch = 0; ch < a.f.nchunk; ++ch) {
        if (a.f.wide) {
          const long long* src = reinterpret_cast<const long long*>(a.f.part) + (size_t)ch * a.f.n + i;
#pragma unroll
          for (int v = 0; v < V; v += 2) {
            if constexpr (V >= 2) {
              const longlong2 w = *reinterpret_cast<const longlong2*>(src + v);
              acc[v] += w.x;
              acc[v + 1] += w.y;
            } else {
              acc[v] += src[v];
            }
          }
        } else {
          const int32_t* src = reinterpret_cast<const int32_t*>(a.f.part) + (size_t)ch * a.f.n + i;
          if constexpr (V == 4) {
            const int4 w = *reinterpret_cast<const int4*>(src);
            acc[0] += w.x; acc[1] += w.y; acc[2] += w.z; acc[3] += w.w;
          } else {
            acc[0] += src[0];
          }
        }
      }
#pragma unroll
      for (int v = 0; v < V; ++v) {
        double y = (double)acc[v] * a.f.scale;
        if (a.f.wsum) y = y - (double)a.f.wsum[k + v] * a.f.half_range;
        sum[v] += (float)y;
      }
    }
  }
  if constexpr (V == 4) {
    *reinterpret_cast<float4*>(a.dX + t * 4) = make_float4(sum[0], sum[1], sum[2], sum[3]);
  } else {
    a.dX[t] = sum[0];
  }
}

struct WriteArgs {
  float* W;
  float* Gp;        // per-polarity device state (update_pair_write_kernel): positive device, in [0, 1]
  float* Gn;        //   negative device
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



// The same write with the two devices of a weight as states of their own (a variant of Sec. IV-C's one
// conductance per weight; Sec. IV-A keeps positive and negative conductances in two arrays): half the ideal
// change to each, in opposite directions, each with the non-linearity at its own state and direction, a noise
// draw of its own (sigma = gamma sqrt(|delta| / 2), numbers 2 i and 2 i + 1 of the pair stream) and its own
// clamp to [0, 1]; W = w_max (gp - gn).
__global__ __launch_bounds__(256) void update_pair_write_kernel(WriteArgs a) {
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
  const double half = 0.5 * (a.grad_scale * grad);
  double state[2] = {(double)a.Gp[i], (double)a.Gn[i]};
  NormalStream rng(a.seed, kStreamWritePair, effective_step(a.step, a.step_add));
#pragma unroll
  for (int pol = 0; pol < 2; ++pol) {
    const double dir = pol == 0 ? -1.0 : 1.0;        // the positive device falls when the weight falls
    const double change = dir * a.lr * half;
    double written = half;
    if (a.flags & XBAR_NI_UPD_NL) {
      const double x = clampd(state[pol], 0.0, 1.0);
      if (change > 0.0) written = half * ::exp(-a.v * x);
      else if (change < 0.0) written = half * ::exp(-a.v * (1.0 - x));
    }
    if (a.flags & XBAR_NI_UPD_NOISE) written += a.gamma * ::sqrt(::fabs(half)) * rng.get(2 * (uint64_t)i + (uint64_t)pol);
    state[pol] = clampd(state[pol] + dir * a.lr * written, 0.0, 1.0);
  }
  const float gp = (float)state[0], gn = (float)state[1];
  a.Gp[i] = gp;
  a.Gn[i] = gn;
  a.W[i] = (float)(a.w_max * ((double)gp - (double)gn));
}

struct PairInitArgs {
  const float* W;
  float* Gp;
  float* Gn;
  long long n;
  double w_max;
};

// A weight placed symmetrically about mid-range: gp = (1 + g) / 2, gn = (1 - g) / 2, g = clamp(W / w_max).
__global__ __launch_bounds__(256) void pair_init_kernel(PairInitArgs a) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= a.n) return;
  const double g = clampd((double)a.W[i] / a.w_max, -1.0, 1.0);
  a.Gp[i] = (float)(0.5 * (1.0 + g));
  a.Gn[i] = (float)(0.5 * (1.0 - g));
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

// The block-scaled 6-bit x 4-bit instruction alone: pseudo-random E2M3 codes, single-bit E2M1 digits.
__global__ __launch_bounds__(256) void mfma_probe_f6_kernel(float* out, int iters) {
  uint32_t x = threadIdx.x * 2654435761u + 12345u;
  int8v a = {0, 0, 0, 0, 0, 0, 0, 0}, b = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int i = 0; i < 6; ++i) {
    x ^= x << 13; x ^= x >> 17; x ^= x << 5;
    a[i] = (int)x;
    x ^= x << 13; x ^= x >> 17; x ^= x << 5;
    if (i < 4) b[i] = (int)(x & 0x11111111u);
  }
  float16v c0, c1;
#pragma unroll
  for (int r = 0; r < 16; ++r) c0[r] = c1[r] = 0.0f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      c0 = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c0, 2, 4, 0, 127 - 8, 0, 127);
      c1 = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c1, 2, 4, 0, 127 - 8, 0, 127);
    }
  }
  float s = 0.0f;
#pragma unroll
  for (int r = 0; r < 16; ++r) s += c0[r] + c1[r];
  out[blockIdx.x * 256 + threadIdx.x] = s;
}

// The contraction kernel's own inner loop (vmm6_contract_adc: 4 terms, 128 rows, two row patches) on
// synthetic operands: plane fragments of 4 slices in LDS, digits rebuilt every 4 passes as in the kernel.
template <bool DO_ADC>
__global__ __launch_bounds__(256, 2) void contraction_loop_probe_kernel(float* out, int iters) {
  extern __shared__ u32x4 lds[];
  constexpr int SLICE = 4 * f6_term_stride(2);       // 12 KiB
  uint32_t x = (threadIdx.x + 977u * blockIdx.x) * 2654435761u + 777u;
  for (int i = threadIdx.x; i < 4 * SLICE / 16; i += 256) {
    u32x4 v;
    x ^= x << 13; x ^= x >> 17; x ^= x << 5; v.x = x;
    x ^= x << 13; x ^= x >> 17; x ^= x << 5; v.y = x;
    x ^= x << 13; x ^= x >> 17; x ^= x << 5; v.z = x;
    x ^= x << 13; x ^= x >> 17; x ^= x << 5; v.w = x;
    lds[i] = v;
  }
  __syncthreads();
  const int lane = threadIdx.x & 63;
  u32x2 raw[2][8];
#pragma unroll
  for (int pm = 0; pm < 2; ++pm)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      x ^= x << 13; x ^= x >> 17; x ^= x << 5; raw[pm][j].x = x;
      x ^= x << 13; x ^= x >> 17; x ^= x << 5; raw[pm][j].y = x;
    }
  const char* xb = reinterpret_cast<const char*>(lds) + lane * 16;
  const char* yb = reinterpret_cast<const char*>(lds) + 1024 + lane * 8;
  // terms 2^0, 2^-6, 2^-11, 2^-16 as for the single-path wire model at the paper's parameters
  const int scale_lo = 127 | (121 << 8) | (116 << 16) | (111 << 24), scale_hi = 127;
  int4v dg[2][2];
  float16v acc0[2], acc1[2];
  uint32_t y[2][16];
#pragma unroll
  for (int pm = 0; pm < 2; ++pm)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      acc0[pm][r] = acc1[pm][r] = 0.0f;
      y[pm][r] = 0;
    }
  for (int it = 0; it < iters; ++it) {
    const int sl = (it & 1) * 2;
    if ((it & 1) == 0) {
#pragma unroll
      for (int pm = 0; pm < 2; ++pm) digit_codes_f4<2, false>(raw[pm], (it >> 1) & 3, 0x11111111u, dg[pm]);
    }
    vmm6_contract_adc<2, 2, 4, DO_ADC>(dg, xb + sl * SLICE, yb + sl * SLICE, acc0, acc1, 3.96875f, kMagic - 127.0f,
                                       kMagic + 127.0f, it & 15, y, scale_lo, scale_hi);
    vmm6_contract_adc<2, 2, 4, DO_ADC>(dg, xb + (sl + 1) * SLICE, yb + (sl + 1) * SLICE, acc1, acc0, 3.96875f,
                                       kMagic - 127.0f, kMagic + 127.0f, (it + 2) & 15, y, scale_lo, scale_hi);
    if (!DO_ADC)     // nothing consumes the sums in this variant: keep the compiler from dropping the instructions
      asm volatile("" ::"v"(acc0[0]), "v"(acc0[1]), "v"(acc1[0]), "v"(acc1[1]));
  }
  float s = 0.0f;
  uint32_t t = 0;
#pragma unroll
  for (int pm = 0; pm < 2; ++pm)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      s += acc0[pm][r] + acc1[pm][r];
      t += y[pm][r];
    }
  out[blockIdx.x * 256 + threadIdx.x] = s + (float)t;
}

// ---------------------------------------------------------------------------------------------
// host dispatch
// ---------------------------------------------------------------------------------------------
thread_local hipEvent_t g_trace_before = nullptr, g_trace_after = nullptr;
thread_local const unsigned long long* g_step_source = nullptr;

__global__ void step_advance_kernel(unsigned long long* counter) { *counter += 1ull; }

// Scratch of xbar_fwd_static: one array per GPU that the library runs on, held until the process ends.
// The name is a host-side stand-in; host code uses the device address that hipGetSymbolAddress returns.
static __device__ __align__(256) unsigned char scratch[XBAR_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of this GPU's copy of the scratch array (looked up once per device, with that device current).
int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return XBAR_EHIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return XBAR_EHIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return XBAR_OK;
}

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
    // all slices in one stage when they fit 72 KiB (two blocks of a compute unit share its 160 KiB); else as
    // many as fit 64 KiB, an even number (the pipelined path pairs them)
    const int fit_sg = d.S_w * slice_kb <= 72 ? d.S_w : std::max(1, 64 / slice_kb);
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
  // 32-bit sums hold `fit` virtual tiles: a chunk with more adds them to a 64-bit partial sum of its own in
  // between (no extra chunks, so no extra partial results for the adding-up pass to read)
  p.flush_every = (!p.wide && (unsigned long long)per > fit) ? (int)fit : 0;
  if (p.wide == 2) per = (int)std::min<unsigned long long>((unsigned long long)per, fit_split);
  p.nchunk = cdiv(p.VT, per);
  p.vt_per_chunk = cdiv(p.VT, p.nchunk);                  // same number of chunks, evenly filled
  p.a_bytes = align256((size_t)p.P * p.MP * p.g.T * p.ks16 * 512);
  p.part_bytes = align256((size_t)p.nchunk * M * p.Lout * ((p.wide || p.flush_every) ? 8 : 4));
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
  // two resident blocks per compute unit: more batch chunks only add partial sums (measured: 512 blocks beat 256, 1024, 2048)
  int want = std::max(1, cdiv(512, tiles));
  int per = std::max(kGradMS, cdiv(cdiv(M, want), kGradMS) * kGradMS);
  p.m_per_chunk = per;
  p.mchunks = cdiv(M, per);
  p.parts = (K <= 64 ? 2 : 1) * (N <= 64 ? 2 : 1);
  p.ws_bytes = align256((size_t)p.mchunks * p.parts * K * N * sizeof(float));
  return p;
}

hipError_t launch_vmm6(const VmmArgs& a, const VmmPlan& p, int terms, bool codes, hipStream_t st) {
  return terms == 5 ? launch_vmm_f6_b(a, p, terms, codes, st) : launch_vmm_f6_a(a, p, terms, codes, st);
}

hipError_t launch_vmm(const VmmArgs& a, const VmmPlan& p, int terms, bool codes, hipStream_t st) {
  return p.g.ks <= 8 ? launch_vmm_f16_a(a, p, terms, codes, st) : launch_vmm_f16_b(a, p, terms, codes, st);
}

int run_vmm(const xbar_config* cfg, const void* planes, const float* in, float* out, int M, int K, int N,
            float w_max, float in_scale, void* ws, size_t ws_bytes, int16_t* codes, void* stream, bool transposed,
            const ConvGeom* conv = nullptr, unsigned long long* hist = nullptr, const ConvGeom* scatter = nullptr) {
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
  qa.nibbles = d.fmt == kFmtF6 ? 1 : 0;
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
  a.flush_every = hist ? 0 : p.flush_every;            // the statistics pass keeps no sums
  a.direct = (p.nchunk == 1 && !p.offset && !split && !scatter) ? 1 : 0;   // a scatter gathers from the partial sums
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
    f.wide = p.wide != 0 || p.flush_every != 0;
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
    if (scatter) {     // backward convolution: out is the NHWC image of input errors
      FinishCol2imArgs fc;
      fc.f = f;
      fc.dX = out;
      fc.conv = *scatter;
      fc.K = p.Lout;
      fc.n_img = (long long)(M / (scatter->OH * scatter->OW)) * scatter->H * scatter->W * scatter->C;
      // 16-byte accesses: channels in fours (then K = kernel positions x channels is a multiple of 4 too)
      if (scatter->C % 4 == 0)
        hipLaunchKernelGGL(vmm_finish_col2im_kernel<4>, dim3((unsigned)((fc.n_img / 4 + 255) / 256)), dim3(256), 0, st, fc);
      else
        hipLaunchKernelGGL(vmm_finish_col2im_kernel<1>, dim3((unsigned)((fc.n_img + 255) / 256)), dim3(256), 0, st, fc);
    } else {
      if (f.n % 4 == 0)
        hipLaunchKernelGGL(vmm_finish_kernel<4>, dim3((unsigned)((f.n / 4 + 255) / 256)), dim3(256), 0, st, f);
      else
        hipLaunchKernelGGL(vmm_finish_kernel<1>, dim3((unsigned)((f.n + 255) / 256)), dim3(256), 0, st, f);
    }
    if (hipGetLastError() != hipSuccess) return XBAR_EHIP;
  }
  return XBAR_OK;
}


int run_update(const xbar_config* cfg, float* W, const float* X, const float* dY, int M, int K, int N, float w_max,
               float grad_scale, float lr, uint64_t step, void* ws, size_t ws_bytes, void* hip_stream, const ConvGeom* conv,
               float* Gp = nullptr, float* Gn = nullptr) {
  int rc = xbar_config_validate(cfg);
  if (rc) return rc;
  if ((rc = check_shape(M, K, N))) return rc;
  if (!aligned16(W) || !aligned16(X) || !aligned16(dY) || !aligned16(ws)) return XBAR_EALIGN;
  if ((Gp || Gn) && (!aligned16(Gp) || !aligned16(Gn))) return XBAR_EALIGN;
  if (!finite_pos(w_max) || !std::isfinite(grad_scale) || !std::isfinite(lr)) return XBAR_EINVAL;
  const UpdPlan p = plan_update(M, K, N);
  if (ws_bytes < p.ws_bytes) return XBAR_EWORKSPACE;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  GradArgs g;
  g.X = X; g.D = dY; g.part = reinterpret_cast<float*>(ws);
  g.M = M; g.K = K; g.N = N; g.KB = p.KB; g.NB = p.NB; g.m_per_chunk = p.m_per_chunk;
  {
    g.total_wg = p.KB * p.NB * p.mchunks;
    g.per_xcd = cdiv(g.total_wg, 8);
    const dim3 grid((unsigned)(g.per_xcd * 8)), block(256);
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
  w.W = W; w.Gp = Gp; w.Gn = Gn; w.part = g.part; w.n = (long long)K * N; w.mchunks = p.mchunks * p.parts; w.flags = cfg->flags;
  w.w_max = (double)w_max; w.grad_scale = (double)grad_scale; w.lr = (double)lr;
  w.v = (double)cfg->upd_nl_v; w.gamma = (double)cfg->upd_noise_gamma;
  w.seed = cfg->seed; w.step = step; w.step_add = current_step_source();
  if (Gp) hipLaunchKernelGGL(update_pair_write_kernel, dim3((unsigned)((w.n + 31) / 32)), dim3(256), 0, st, w);
  else hipLaunchKernelGGL(update_write_kernel, dim3((unsigned)((w.n + 31) / 32)), dim3(256), 0, st, w);
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
  if (mode < 0 || mode > 6 || iters <= 0 || iters > (1 << 24)) return XBAR_EINVAL;
  if (!aligned16(out)) return XBAR_EALIGN;
  if (out_bytes < (size_t)512 * 256 * sizeof(float)) return XBAR_EWORKSPACE;
  if (mode == 4) {
    hipLaunchKernelGGL(mfma_probe_f6_kernel, dim3(512), dim3(256), 0, reinterpret_cast<hipStream_t>(hip_stream),
                       reinterpret_cast<float*>(out), iters);
    return hipGetLastError() == hipSuccess ? XBAR_OK : XBAR_EHIP;
  }
  if (mode >= 5) {
    const size_t lds_bytes = 4 * 4 * f6_term_stride(2);
    if (mode == 5)
      hipLaunchKernelGGL(contraction_loop_probe_kernel<false>, dim3(512), dim3(256), lds_bytes,
                         reinterpret_cast<hipStream_t>(hip_stream), reinterpret_cast<float*>(out), iters);
    else
      hipLaunchKernelGGL(contraction_loop_probe_kernel<true>, dim3(512), dim3(256), lds_bytes,
                         reinterpret_cast<hipStream_t>(hip_stream), reinterpret_cast<float*>(out), iters);
    return hipGetLastError() == hipSuccess ? XBAR_OK : XBAR_EHIP;
  }
  if (mode >= 2) {
    hipLaunchKernelGGL(mfma_probe_i8_kernel, dim3(512), dim3(256), 0, reinterpret_cast<hipStream_t>(hip_stream),
                       reinterpret_cast<int*>(out), iters, mode);
    return hipGetLastError() == hipSuccess ? XBAR_OK : XBAR_EHIP;
  }
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(512), dim3(256), 0, reinterpret_cast<hipStream_t>(hip_stream),
                     reinterpret_cast<float*>(out), iters, mode);
  return hipGetLastError() == hipSuccess ? XBAR_OK : XBAR_EHIP;
}

float xbar_adc_range_from_histogram(const unsigned long long* hist, int bins, float bin_width, double quantile) {
  if (!hist || bins <= 0 || !finite_pos(bin_width) || !(quantile > 0.0) || quantile > 1.0) return 0.0f;
  double total = 0.0;
  for (int b = 0; b < bins; ++b) total += (double)hist[b];
  double cum = 0.0;
  int b = 0;
  for (; b < bins - 1; ++b) {
    cum += (double)hist[b];
    if (cum >= quantile * total) break;
  }
  const double current = std::max(((double)b + 0.5) * (double)bin_width, (double)bin_width);
  return (float)std::exp2(std::ceil(std::log2(current)));
}

int xbar_plane_format(const xbar_config* cfg, int* terms) {
  const int rc = xbar_config_validate(cfg);
  if (rc) return rc;
  const Derived d = derive(cfg);
  if (terms) *terms = d.terms;
  return d.fmt;
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
    case XBAR_ESCRATCH: return "shape needs more scratch memory than the library's static array holds (XBAR_STATIC_SCRATCH_BYTES)";
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
  if (c->flags & ~0x1FFFu) return XBAR_EINVAL;
  if ((c->flags & XBAR_PULSE_CODED) && (c->flags & XBAR_PULSE_MAGNITUDE)) return XBAR_EINVAL;   // one pulse coding
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
  return device_words_offset(cfg, d, K, N) + device_words_bytes(d, K, N);
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
      a.codes = nullptr;
      if (uses_code_table(d)) {
        uint32_t* table = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(planes) + code_table_offset(cfg, d, K, N));
        if (dir == 0) {
          const int entries = ((1 << cfg->slice_bits) - 1) * cfg->xbar_rows * cfg->xbar_cols;
          hipLaunchKernelGGL(code_table_kernel, dim3((unsigned)cdiv(entries, 256)), dim3(256), 0, st, a, table);
          if (hipGetLastError() != hipSuccess) return XBAR_EHIP;
        }
        a.codes = table + (dir == 1 ? code_table_words(cfg) : 0);
        // a thread quantises its weights once for all the slices it covers: as many slices per thread as
        // still leave about four waves for every SIMD of the chip
        a.spt = (int)std::min<long long>(d.S_w, std::max<long long>(1, a.n_threads * d.S_w / 262144));
        const dim3 grid(blocks, (unsigned)cdiv(d.S_w, a.spt));
        if (dir == 0) hipLaunchKernelGGL(tile_planes_f6_table_kernel<false>, grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL(tile_planes_f6_table_kernel<true>, grid, dim3(256), 0, st, a);
      } else if (uses_device_words(d)) {
        uint32_t* words = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(planes) + device_words_offset(cfg, d, K, N));
        if (dir == 0 && pol == 0) {                  // every device once, for both copies and both arrays
          const unsigned wblocks = (unsigned)(((long long)K * N + 255) / 256);
          hipLaunchKernelGGL(device_words_kernel, dim3(wblocks, (unsigned)d.S_w), dim3(256), 0, st, a, words, d.npol);
          if (hipGetLastError() != hipSuccess) return XBAR_EHIP;
        }
        a.codes = words + (size_t)pol * d.S_w * K * N;
        a.n_threads = (long long)g.T * g.OP * g.ks * 64;   // one wave per fragment group
        const dim3 pgrid((unsigned)((a.n_threads + 255) / 256), (unsigned)d.S_w);
        if (dir == 0) hipLaunchKernelGGL(tile_planes_f6_words_kernel<false>, pgrid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL(tile_planes_f6_words_kernel<true>, pgrid, dim3(256), 0, st, a);
      } else if (dir == 0) hipLaunchKernelGGL(tile_planes_f6_kernel<false>, dim3(blocks, (unsigned)d.S_w), dim3(256), 0, st, a);
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

int xbar_fwd_static(const xbar_config* cfg, const void* planes, const float* X, float* Y, int M, int K, int N, float w_max,
                    float x_scale, void* hip_stream) {
  int rc = xbar_config_validate(cfg);
  if (rc) return rc;
  if ((rc = check_shape(M, K, N))) return rc;
  const size_t need = plan_vmm(cfg, derive(cfg), M, K, N, false).ws_bytes;
  if (need > (size_t)XBAR_STATIC_SCRATCH_BYTES) return XBAR_ESCRATCH;
  void* ws = nullptr;
  if ((rc = static_scratch(&ws))) return rc;
  return run_vmm(cfg, planes, X, Y, M, K, N, w_max, x_scale, ws, (size_t)XBAR_STATIC_SCRATCH_BYTES, nullptr, hip_stream, false);
}

int xbar_bwd(const xbar_config* cfg, const void* planes, const float* dY, float* dX, int M, int K, int N, float w_max,
             float g_scale, void* ws, size_t ws_bytes, int16_t* codes, void* hip_stream) {
  return run_vmm(cfg, planes, dY, dX, M, K, N, w_max, g_scale, ws, ws_bytes, codes, hip_stream, true);
}

int xbar_update(const xbar_config* cfg, float* W, const float* X, const float* dY, int M, int K, int N, float w_max,
                float grad_scale, float lr, uint64_t step, void* ws, size_t ws_bytes, void* hip_stream) {
  return run_update(cfg, W, X, dY, M, K, N, w_max, grad_scale, lr, step, ws, ws_bytes, hip_stream, nullptr);
}

int xbar_pair_init(const float* W, float* Gp, float* Gn, int K, int N, float w_max, void* hip_stream) {
  const int rc = check_shape(1, K, N);
  if (rc) return rc;
  if (!aligned16(W) || !aligned16(Gp) || !aligned16(Gn)) return XBAR_EALIGN;
  if (!finite_pos(w_max)) return XBAR_EINVAL;
  PairInitArgs a;
  a.W = W; a.Gp = Gp; a.Gn = Gn; a.n = (long long)K * N; a.w_max = (double)w_max;
  hipLaunchKernelGGL(pair_init_kernel, dim3((unsigned)((a.n + 255) / 256)), dim3(256), 0, reinterpret_cast<hipStream_t>(hip_stream), a);
  return hipGetLastError() == hipSuccess ? XBAR_OK : XBAR_EHIP;
}

int xbar_update_pair(const xbar_config* cfg, float* Gp, float* Gn, float* W, const float* X, const float* dY, int M, int K,
                     int N, float w_max, float grad_scale, float lr, uint64_t step, void* ws, size_t ws_bytes, void* hip_stream) {
  if (!Gp || !Gn) return XBAR_EALIGN;
  return run_update(cfg, W, X, dY, M, K, N, w_max, grad_scale, lr, step, ws, ws_bytes, hip_stream, nullptr, Gp, Gn);
}

int xbar_conv_update_pair(const xbar_config* cfg, float* Gp, float* Gn, float* W, const float* X, const float* dY,
                          const xbar_conv_geom* geom, int N, float w_max, float grad_scale, float lr, uint64_t step, void* ws,
                          size_t ws_bytes, void* hip_stream) {
  if (!Gp || !Gn) return XBAR_EALIGN;
  ConvGeom g;
  int M, K;
  const int rc = conv_dims(geom, &g, &M, &K);
  if (rc) return rc;
  return run_update(cfg, W, X, dY, M, K, N, w_max, grad_scale, lr, step, ws, ws_bytes, hip_stream,
                    conv_is_dense(geom) ? nullptr : &g, Gp, Gn);
}

size_t xbar_conv_workspace_bytes(const xbar_config* cfg, int op, const xbar_conv_geom* geom, int N) {
  ConvGeom g;
  int M, K;
  if (xbar_config_validate(cfg) || conv_dims(geom, &g, &M, &K) || check_shape(M, K, N)) return 0;
  const Derived d = derive(cfg);
  if (op == XBAR_OP_FWD) return plan_vmm(cfg, d, M, K, N, false).ws_bytes;
  if (op == XBAR_OP_BWD) return plan_vmm(cfg, d, M, K, N, true).ws_bytes;
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
  // the adding-up pass gathers every input pixel's patch errors from the partial sums
  return run_vmm(cfg, planes, dY, dX, M, K, N, w_max, g_scale, ws, ws_bytes, nullptr, hip_stream, true, nullptr, nullptr, &g);
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
