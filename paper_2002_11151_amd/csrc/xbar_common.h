// Shared by the translation units of libxbar.so: constants, the geometry of the plane buffer, the
// counter-based random numbers and small device helpers.  Internal: the boundary is include/xbar.h.
#ifndef XBAR_COMMON_H_
#define XBAR_COMMON_H_

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <mutex>

#include "xbar.h"

namespace xbar_detail {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr uint32_t kMagicBits = 0x4B400000u;  // bits of 1.5 * 2^23: adding it rounds to an integer (RNE)
constexpr float kMagic = 12582912.0f;
constexpr int kStreamVariation = 1, kStreamWrite = 2;
constexpr int kStreamPulseRows = 3, kStreamPulseCols = 4, kStreamPulseNoise = 5, kStreamWritePair = 6;
constexpr bool kBarrierPerMfma = false;   // scheduling fence after every MFMA (true) or every fragment (false)

// ---------------------------------------------------------------------------------------------
// host-side geometry shared by the entry points
// ---------------------------------------------------------------------------------------------
// Operand format of the plane buffer and of the contraction kernel.
//   kFmtF16: fp16 fragments for v_mfma_f32_32x32x16_f16, one term (exact digits) or two (leading term on
//            a fixed grid + fp16 residual); input digits as fp16 subnormals.  Serves every configuration.
//   kFmtF6:  6-bit floating-point (E2M3) fragments for v_mfma_scale_f32_32x32x64_f8f6f4 with the input
//            digits as 4-bit floating-point (E2M1) codes: a plane value is a sum of up to 5 terms, each
//            an E2M3 number times a power of two that the instruction applies as a block scale, all
//            accumulated in one fp32 sum, leading term first.  64 rows per instruction at the time of
//            16 in fp16.  For cycles of 1 or 2 bits (digit d is the E2M1 code d, value d / 2) without
//            a general DAC level table.
constexpr int kFmtF16 = 0, kFmtF6 = 1;
constexpr int kMaxTermsF6 = 5;

struct Derived {
  int S_w, S_in, terms, q_adc;
  int npol;            // converters per crossbar column: 1 (pair read differentially) or 2 (one per array)
  uint32_t array_ni;
  int fmt;             // kFmtF16 or kFmtF6
  int term_exp[kMaxTermsF6];   // kFmtF6: term j of a plane value is (E2M3 number) x 2^term_exp[j]
};

// kFmtF6 term schedule.  Term 0 is the E2M3 number nearest to U / 2^x0 (|U| up to 7.5 x 2^x0: more than
// twice the top device level).  What it leaves is at most a quarter of 2^x0, or `bound` when the plane
// values are known to stay that close to whole levels (single-path wire model alone).  Every later term
// holds the E2M3 number nearest to what is left, in units of the smallest power of two whose largest
// E2M3 number (7.5) still covers it; a number in binade b of the format (b = 0 below 2, 1 below 4, else
// 2) then leaves at most 2^(b - 4) units.  Terms are added until what is left is at most `max_error`
// device levels (and there are `min_terms` of them), 5 at most; ideal arrays need term 0 alone.
// Returns the number of terms.
static inline int f6_schedule(int slice_bits, bool ideal, double bound, double max_error, int min_terms, int* term_exp) {
  const int x0 = slice_bits - 2;
  term_exp[0] = x0;
  for (int j = 1; j < kMaxTermsF6; ++j) term_exp[j] = x0;
  if (ideal) return 1;
  double left = std::ldexp(1.0, x0 - 2);
  if (bound > 0.0 && bound < left) left = bound;
  int n = 1;
  while (n < kMaxTermsF6) {
    int e = (int)std::ceil(std::log2(left / 7.5));
    if (std::ldexp(7.5, e) < left) ++e;
    term_exp[n++] = e;
    const double units = left / std::ldexp(1.0, e);
    left = std::ldexp(1.0, e - 4 + (units <= 2.0 ? 0 : units <= 4.0 ? 1 : 2));
    if (left <= max_error && n >= min_terms) break;
  }
  return n;
}

// Budget of the planes' own representation error, as the share of converter codes that it may move
// across a rounding boundary: half of the tolerance of 1e-4 on the codes, and no more than keeps the
// layer outputs within a relative L2 distance of 1e-3 of exact arithmetic on the planes.  A code that
// changes by one in (slice s, cycle b) moves an output by 2^(slice_bits s + stream_bits b) code weights,
// so a share f of changed codes gives a relative L2 distance of about
//   sqrt(1.42 f P / rows) / (8 gain rx rw)
// (P = 2 input phases, rows per tile, gain in codes per device level, rx and rw the rms of inputs and
// weights over their scales; the 8 is 2^21 / (255 x 65535) for the sizes that matter): with rx rw = 0.05
// that is f <= 5.6e-8 gain^2 rows.
constexpr double kPlaneFlipShare = 5e-5;
constexpr double kPlaneFlipShareL2 = 5.6e-8;

static inline Derived derive(const xbar_config* c) {
  Derived d;
  d.S_w = c->weight_bits / c->slice_bits;
  d.S_in = c->input_bits / c->stream_bits;
  d.array_ni = c->flags & (XBAR_NI_VARIATION | XBAR_NI_WIRE_AAM | XBAR_NI_WIRE_PROFILE | XBAR_NI_WIRE_AAM2);
  d.npol = (c->flags & XBAR_ADC_PER_ARRAY) ? 2 : 1;
  // one array alone carries the off-state conductance of every device: never whole device levels
  d.terms = (d.array_ni || d.npol == 2) ? 2 : 1;
  // signed converter on the difference of the pair, or unsigned converter on one array's current
  d.q_adc = d.npol == 2 ? (1 << c->adc_bits) - 1 : (1 << (c->adc_bits - 1)) - 1;
  const bool level_table = (c->flags & XBAR_DAC_LUT) && !(c->stream_bits == 1 && c->dac_lut[0] == 0.0f);
  d.fmt = (c->stream_bits <= 2 && !level_table) ? kFmtF6 : kFmtF16;
  for (int j = 0; j < kMaxTermsF6; ++j) d.term_exp[j] = 0;
  if (d.fmt == kFmtF6) {
    // single-path wire model alone: |U - digit| <= rho_max (Gmax^2 + Gmin^2) / (one device level)
    double bound = 0.0;
    if (d.npol == 1 && d.array_ni == XBAR_NI_WIRE_AAM) {
      const double g_min = 1.0 / (double)c->r_max, g_max = 1.0 / (double)c->r_min;
      const double dg = (g_max - g_min) / (double)((1 << c->slice_bits) - 1);
      const double rho = (double)c->r_source + (double)c->xbar_cols * (double)c->r_row +
                         (double)c->xbar_rows * (double)c->r_col + (double)c->r_sense;
      bound = rho * (g_max * g_max + g_min * g_min) / dg;
    }
    // A representation error e of a plane value, uniform within +-left, moves a column current of `rows`
    // devices, about half of them driven, by about 0.46 left xmax sqrt(rows / 2) device levels (mean
    // magnitude of the sum); times the converter gain that is the share of codes that change, since a
    // code changes when a rounding boundary lies within the shift.
    double gain = (double)d.q_adc / (double)std::min(c->adc_fs_fwd, c->adc_fs_bwd);
    if ((c->flags & XBAR_DAC_LUT) && !level_table) gain *= std::fabs((double)c->dac_lut[1]);
    const double packed = (c->flags & XBAR_ADC_CURVE) ? 4.0 : 1.0;   // a converter curve may pack its thresholds closer
    const double rows = (double)std::max(c->xbar_rows, c->xbar_cols);
    const double per_level = packed * gain * (double)((1 << c->stream_bits) - 1) * 0.46 * std::sqrt(rows / 2.0);
    const double share = std::min(kPlaneFlipShare, kPlaneFlipShareL2 * gain * gain * (double)std::min(c->xbar_rows, c->xbar_cols));
    // kernels exist for 1, 4 and 5 terms; one array alone: for 5 terms only
    d.terms = f6_schedule(c->slice_bits, d.terms == 1, bound, share / per_level, d.npol == 2 ? 5 : 4, d.term_exp);
  }
  return d;
}

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
static inline int cdiv(int a, int b) { return (a + b - 1) / b; }

// Plane buffer: forward copy then backward copy.  One copy is
// [array][tile][output patch of 32][slice][term][k-step][fragment]; there is one "array" (the difference
// of the pair) unless every array has a converter of its own.  kFmtF16: k-steps of 16 rows, a fragment is
// 64 lanes x 8 halves (1 KiB).  kFmtF6: k-steps of 64 rows, a fragment is 64 lanes x 16 bytes followed by
// 64 lanes x 8 bytes (1.5 KiB): the 24 bytes of a lane hold its 32 six-bit codes, code e at bit 6 e.
// Lane l = (output column l % 32, half l / 32); code e of that lane is contraction row
//   64 J + 16 (e / 8) + 8 (l / 32) + (e % 8) / 2 + 4 (e % 2)
// of k-step J, which is where the input stage's bytes land when they are packed into 4-bit digits.
struct PlaneGeom {
  int tile, ks, T, OP;          // contraction tile length, k-steps per tile, tiles, output patches
  int frag_bytes;               // bytes of one fragment
  size_t pol_bytes, bytes;      // one array, all arrays
};

constexpr size_t kPlanePad = 1024;   // behind each copy: staging copies whole KiB and may read past the last fragment

// Scratch of the all-paths wire model, kept behind the two plane copies.
static inline size_t wire_scratch_bytes(const xbar_config* c, const Derived& d, int K, int N) {
  return (c->flags & XBAR_NI_WIRE_AAM2) ? align256((size_t)16 * d.S_w * K * N) + align256((size_t)4 * K * N) : 0;
}

// Weight sums for the digital correction of offset-binary inputs, kept behind the wire scratch:
// colsum[N] then rowsum[K], 64-bit.
static inline size_t weight_sums_bytes(const xbar_config* c, int K, int N) {
  return (c->flags & XBAR_INPUT_OFFSET) ? align256((size_t)8 * ((size_t)K + N)) : 0;
}

// Term codes of every plane value that can occur, kept behind the weight sums.  With the single-path wire
// model alone (kFmtF6, one converter per column) a plane value depends only on the digit, the sign of the
// weight and the place of the device pair in its array, so xbar_tile computes each once and the plane
// generators look them up: [orientation][sign][digit - 1][row][column] words of 32 bits, term j's 6-bit
// code at bit 6 j; orientation 1 is the same table with rows and columns exchanged.
static inline bool uses_code_table(const Derived& d) {
  return d.fmt == kFmtF6 && d.npol == 1 && d.array_ni == XBAR_NI_WIRE_AAM;
}
static inline size_t code_table_words(const xbar_config* c) {
  return (size_t)2 * ((1u << c->slice_bits) - 1) * c->xbar_rows * c->xbar_cols;   // one orientation
}
static inline size_t code_table_bytes(const xbar_config* c, const Derived& d) {
  return uses_code_table(d) ? align256(2 * code_table_words(c) * sizeof(uint32_t)) : 0;
}

// General 6-bit generator (variation, stored profile, all-paths model, one array alone): every device is computed
// once -- its term codes as one 32-bit word (term j at bit 6 j), [array][slice][k][n], kept behind the table -- and
// both plane copies are packed from those words.
static inline bool uses_device_words(const Derived& d) { return d.fmt == kFmtF6 && !uses_code_table(d) && d.terms > 1; }
static inline size_t device_words_bytes(const Derived& d, int K, int N) {
  return uses_device_words(d) ? align256((size_t)4 * d.npol * d.S_w * K * N) : 0;
}

static inline PlaneGeom plane_geom(const xbar_config* c, const Derived& d, int K, int N, bool transposed) {
  PlaneGeom g;
  g.tile = transposed ? c->xbar_cols : c->xbar_rows;
  g.ks = d.fmt == kFmtF6 ? cdiv(g.tile, 64) : g.tile / 16;
  g.frag_bytes = d.fmt == kFmtF6 ? 1536 : 1024;
  g.T = cdiv(transposed ? N : K, g.tile);
  g.OP = cdiv(transposed ? K : N, 32);
  g.pol_bytes = (size_t)g.T * g.OP * d.S_w * d.terms * g.ks * g.frag_bytes;
  g.bytes = g.pol_bytes * d.npol + (d.fmt == kFmtF6 ? kPlanePad : 0);
  return g;
}

static inline size_t weight_sums_offset(const xbar_config* c, const Derived& d, int K, int N) {
  return align256(plane_geom(c, d, K, N, false).bytes) + align256(plane_geom(c, d, K, N, true).bytes) +
         wire_scratch_bytes(c, d, K, N);
}

static inline size_t code_table_offset(const xbar_config* c, const Derived& d, int K, int N) {
  return weight_sums_offset(c, d, K, N) + weight_sums_bytes(c, K, N);
}

static inline size_t device_words_offset(const xbar_config* c, const Derived& d, int K, int N) {
  return code_table_offset(c, d, K, N) + code_table_bytes(c, d);
}

// ---------------------------------------------------------------------------------------------
// device helpers
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                              uint32_t k1, uint32_t out[4]) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t h0 = __umulhi(0xD2511F53u, c0), l0 = 0xD2511F53u * c0;
    const uint32_t h1 = __umulhi(0xCD9E8D57u, c2), l1 = 0xCD9E8D57u * c2;
    const uint32_t n0 = h1 ^ c1 ^ k0, n2 = h0 ^ c3 ^ k1;
    c0 = n0; c1 = l1; c2 = n2; c3 = l0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Standard normal number i of (seed, stream, step): four consecutive i share one Philox block,
// words (0,1) -> numbers 0,1 (cosine, sine branch of Box-Muller), words (2,3) -> numbers 2,3.
struct NormalStream {
  uint32_t k0, k1, s0, s1;
  uint64_t cached_blk;
  uint32_t w[4];
  __device__ NormalStream(uint64_t seed, uint32_t stream, uint64_t step) {
    k0 = (uint32_t)seed ^ (0x9E3779B9u * stream);
    k1 = (uint32_t)(seed >> 32) ^ (0xBB67AE85u * stream);
    s0 = (uint32_t)step;
    s1 = (uint32_t)(step >> 32);
    cached_blk = ~0ull;
  }
  __device__ double get(uint64_t i) {
    const uint64_t blk = i >> 2;
    if (blk != cached_blk) {
      philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), s0, s1, k0, k1, w);
      cached_blk = blk;
    }
    const bool second = (i & 2u) != 0;
    const double u1 = ((double)(second ? w[2] : w[0]) + 0.5) * (1.0 / 4294967296.0);
    const double u2 = ((double)(second ? w[3] : w[1]) + 0.5) * (1.0 / 4294967296.0);
    const double r = ::sqrt(-2.0 * ::log(u1));
    // angle 2 pi u2: the half-turn form reduces the argument exactly and costs a fraction of sin / cos
    double sn, cs;
    ::sincospi(2.0 * u2, &sn, &cs);
    return (i & 1u) ? r * sn : r * cs;
  }
};

// Step of the random-number streams: the step argument of the call plus, when the caller has named one,
// a counter in device memory -- a captured graph of a training step then draws new devices and new write
// noise on every replay although its kernel arguments are frozen.
__device__ __forceinline__ uint64_t effective_step(uint64_t step, const unsigned long long* step_add) {
  return step + (step_add ? (uint64_t)*step_add : 0ull);
}

__device__ __forceinline__ double clampd(double x, double lo, double hi) { return x < lo ? lo : (x > hi ? hi : x); }

__device__ __forceinline__ double wave_inclusive_scan(double x, int lane) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const double y = __shfl_up(x, d, 64);
    if (lane >= d) x += y;
  }
  return x;
}

// ---------------------------------------------------------------------------------------------
// convolution geometry
// ---------------------------------------------------------------------------------------------
// Convolution as a crossbar layer (Sec. IV: the kernels of a layer are unrolled into the columns of
// the weight matrix, every output position applies one input patch to the rows): input X in NHWC,
// row m = (b, oh, ow) of the layer's input matrix is the patch of that output position and its
// contraction index is l = (kh KW + kw) C + c.  Positions outside the image read 0 V.
struct ConvGeom {
  int H, W, C, KH, KW, stride, pad, OH, OW;
};

struct ConvRow {       // patch of one output position: element (kh, kw, c) is X[off + (kh W + kw) C + c]
  long long off;
  int ih0, iw0;
};

__device__ __forceinline__ ConvRow conv_row(const ConvGeom& g, int m) {
  const int ow = m % g.OW, t = m / g.OW;
  const int oh = t % g.OH, b = t / g.OH;
  ConvRow r;
  r.ih0 = oh * g.stride - g.pad;
  r.iw0 = ow * g.stride - g.pad;
  r.off = (((long long)b * g.H + r.ih0) * g.W + r.iw0) * g.C;
  return r;
}

__device__ __forceinline__ float conv_fetch(const float* X, const ConvGeom& g, const ConvRow& r, int kh, int kw, int c) {
  const int ih = r.ih0 + kh, iw = r.iw0 + kw;
  if (ih < 0 || ih >= g.H || iw < 0 || iw >= g.W) return 0.0f;
  return X[r.off + ((long long)kh * g.W + kw) * g.C + c];
}

// ---------------------------------------------------------------------------------------------
// host-side argument checks
// ---------------------------------------------------------------------------------------------
static inline bool aligned16(const void* p) { return p && (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static inline bool finite_pos(float x) { return std::isfinite(x) && x > 0.0f; }
static inline bool finite_nonneg(float x) { return std::isfinite(x) && x >= 0.0f; }

static inline int check_shape(int M, int K, int N) {
  if (M <= 0 || K <= 0 || N <= 0) return XBAR_ESHAPE;
  // weights are indexed with 32 bits, activations with 64 (bounded to keep grids and buffers sane)
  if ((long long)K * N >= (1ll << 31)) return XBAR_ESHAPE;
  if ((long long)M * K >= (1ll << 38) || (long long)M * N >= (1ll << 38)) return XBAR_ESHAPE;
  return XBAR_OK;
}

// ---------------------------------------------------------------------------------------------
// entry points of one translation unit that another one calls (not exported)
// ---------------------------------------------------------------------------------------------
#define XBAR_INTERNAL __attribute__((visibility("hidden")))
// wire.hip: all-paths wire model of W into the scratch wire_u[S_w][2][K][N] (+ quantised weights behind it)
XBAR_INTERNAL int launch_wire_model(const xbar_config* cfg, const float* W, int K, int N, float w_max, uint64_t step,
                                    double* wire_u, hipStream_t st);
// fcm.hip, pulse.hip: workspace sizes of xbar_fcm_profile and xbar_update_pulsed
XBAR_INTERNAL size_t fcm_workspace_bytes(const xbar_config* cfg, int K, int N);
XBAR_INTERNAL size_t pulsed_workspace_bytes(int M, int K, int N);
// xbar.hip: the device counter named with xbar_set_step_source (this thread), or null
XBAR_INTERNAL const unsigned long long* current_step_source();
// xbar.hip: checks a convolution geometry and derives the layer's matrix shape (M = batch x output
// positions, K = kernel height x kernel width x input channels)
XBAR_INTERNAL int conv_dims(const xbar_conv_geom* q, ConvGeom* g, int* M, int* K);
// A 1 x 1 convolution with stride 1 and no padding IS its patch matrix: X[batch H W][C].
static inline bool conv_is_dense(const xbar_conv_geom* q) { return q->k_h == 1 && q->k_w == 1 && q->stride == 1 && q->pad == 0; }

}  // namespace xbar_detail

#endif  // XBAR_COMMON_H_
