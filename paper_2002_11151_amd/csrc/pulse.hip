// Pulse-level weight update with stochastic pulse trains (Sec. IV-C): kernels and xbar_update_pulsed.
#include "xbar_common.h"

using namespace xbar_detail;

namespace {

// Deterministic pulse coding: the bl slots form tx frames of td sub-slots, tx = floor(sqrt(bl)), td = floor(bl / tx).
void coded_frames(int bl, int* tx, int* td) {
  int t = 1;
  while ((t + 1) * (t + 1) <= bl) ++t;
  *tx = t;
  *td = bl / t;
}


// ---------------------------------------------------------------------------------------------
// pulse-level update (Sec. IV-C names the parallel update schemes; this is the one with stochastic
// pulse trains, whose coincidences multiply): every sample drives rows and columns with random
// trains of `bl` slots, a value fires with probability min(1, |value| / range) per slot, and a device
// is pulsed once per slot in which its row and its column both fire, against the sign of x d.
//   train: slot j of element i fires when uniform word j (Philox block 8 i + j / 4, word j % 4,
//          stream 3 for rows, 4 for columns) is below rne(p 2^32); bit 31 carries the value's sign
//   pulse: g += dir dw_min [exp(-v x) up | exp(-v (1 - x)) down, x = (g + 1) / 2]
//               + gamma sqrt(lr dw_min) normal(m 32 + j of stream 5 keyed (step << 31) | device),
//               lr = bl dw_min w_max / (x_range d_range): the aggregate model's noise for one pulse,
//          clamped to [-1, 1]; samples in order, pulses of a sample in order
// ---------------------------------------------------------------------------------------------
struct PulseArgs {
  float* W;
  const float* X;        // [M][K]
  const float* D;        // [M][N]
  uint32_t* rows;        // [mc][K] trains of the current chunk of samples
  uint32_t* cols;        // [mc][N]
  double* state;         // [K][N] g between chunks
  long long* pulses;     // optional [K][N] signed pulse counts
  int M, K, N, bl, m0, mc, first, last;
  uint32_t flags;
  double w_max, x_range, d_range, dw_min, v, sigma;
  uint64_t seed, step;
  const unsigned long long* step_add;   // optional device counter added to step
  ConvGeom conv;                        // convolution layer: X is the NHWC image and row m of the layer's
                                        //   input matrix is gathered from it (CONV variant of the train kernel)
  int coded, tx, td;                    // 1: deterministic time coding, tx frames of td sub-slots; 2: magnitude coding
  unsigned long long* marks;            // two-phase walk: [n_words][K N] one bit per sample and device
  unsigned long long* summary;          //   [ceil(n_words / 64)][K N] one bit per word that is not empty
  int n_words;                          //   64-sample words of the current chunk
};

__device__ __forceinline__ uint32_t pulse_train(uint32_t k0, uint32_t k1, uint64_t step, uint64_t index, double p, int bl) {
  const uint64_t threshold = (uint64_t)::rint(clampd(p, 0.0, 1.0) * 4294967296.0);
  uint32_t bits = 0;
  for (int j = 0; j < bl; j += 4) {
    const uint64_t blk = index * 8 + (uint64_t)(j >> 2);
    uint32_t w[4];
    philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), (uint32_t)step, (uint32_t)(step >> 32), k0, k1, w);
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (j + e < bl && (uint64_t)w[e] < threshold) bits |= 1u << (j + e);
  }
  return bits;
}

// Deterministic code of a value: slot = frame * td + sub-slot; a row takes the first rne(p tx) frames
// whole, a column the first rne(p td) sub-slots of every frame.
__device__ __forceinline__ uint32_t pulse_code(double p, int tx, int td, bool is_col) {
  const int level = (int)::rint(clampd(p, 0.0, 1.0) * (double)(is_col ? td : tx));
  if (!is_col) return level * td >= 32 ? 0xFFFFFFFFu : (1u << (level * td)) - 1u;      // level * td <= 31 slots
  const uint32_t frame = (1u << level) - 1u;                                          // level <= td <= 31
  uint32_t bits = 0;
  for (int f = 0; f < tx; ++f) bits |= frame << (f * td);
  return bits;
}

// Magnitude coding: ONE pulse per sample whose height is the level rne(p bl) of bl; bit 30 marks a pulse that
// is there at all, so that "row and column share a set bit" still means "this device is written".
__device__ __forceinline__ uint32_t pulse_height(double p, int bl) {
  const uint32_t level = (uint32_t)::rint(clampd(p, 0.0, 1.0) * (double)bl);
  return level ? (level | 0x40000000u) : 0u;
}

// One thread per element of the chunk's inputs, then of its errors.
template <bool CONV>
__global__ __launch_bounds__(256) void pulse_trains_kernel(PulseArgs a) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long n_rows = (long long)a.mc * a.K, n_cols = (long long)a.mc * a.N;
  if (t < n_rows) {
    const uint64_t index = (uint64_t)a.m0 * a.K + (uint64_t)t;               // m K + k
    double x;
    if constexpr (CONV) {        // element (m, k) of the patch matrix: k = (kh KW + kw) C + c
      const int m = a.m0 + (int)(t / a.K), k = (int)(t % a.K);
      const int c = k % a.conv.C, kk = k / a.conv.C;
      x = (double)conv_fetch(a.X, a.conv, conv_row(a.conv, m), kk / a.conv.KW, kk % a.conv.KW, c);
    } else {
      x = (double)a.X[index];
    }
    const uint32_t k0 = (uint32_t)a.seed ^ (0x9E3779B9u * kStreamPulseRows);
    const uint32_t k1 = (uint32_t)(a.seed >> 32) ^ (0xBB67AE85u * kStreamPulseRows);
    const uint32_t train = a.coded == 2 ? pulse_height(::fabs(x) / a.x_range, a.bl)
                           : a.coded  ? pulse_code(::fabs(x) / a.x_range, a.tx, a.td, false)
                                      : pulse_train(k0, k1, effective_step(a.step, a.step_add), index, ::fabs(x) / a.x_range, a.bl);
    a.rows[t] = train | (x < 0.0 ? 0x80000000u : 0u);
  } else if (t < n_rows + n_cols) {
    const long long u = t - n_rows;
    const uint64_t index = (uint64_t)a.m0 * a.N + (uint64_t)u;
    const double d = (double)a.D[index];
    const uint32_t k0 = (uint32_t)a.seed ^ (0x9E3779B9u * kStreamPulseCols);
    const uint32_t k1 = (uint32_t)(a.seed >> 32) ^ (0xBB67AE85u * kStreamPulseCols);
    const uint32_t train = a.coded == 2 ? pulse_height(::fabs(d) / a.d_range, a.bl)
                           : a.coded  ? pulse_code(::fabs(d) / a.d_range, a.tx, a.td, true)
                                      : pulse_train(k0, k1, effective_step(a.step, a.step_add), index, ::fabs(d) / a.d_range, a.bl);
    a.cols[u] = train | (d < 0.0 ? 0x80000000u : 0u);
  }
}

// One pulse of device `dev` (ordinal `ord` within sample m), upwards when `up`.  The device model is
// chosen at compile time, and the step of the noise stream is read before the walk: nothing that is the
// same for all lanes is tested (and no pointer that may be null is followed) inside the per-lane walk.
// `units`: quanta of dw_min that this one write carries (1 for a pulse of a train; the product of the two pulse
// heights with magnitude coding, where the non-linearity and the noise belong to the write as a whole).
template <bool NL, bool NOISE, bool MAG = false>
__device__ __forceinline__ double one_pulse(const PulseArgs& a, double g, bool up, int m, int ord, uint64_t dev,
                                            uint64_t step, int units = 1) {
#pragma clang fp contract(off)   // every product and sum rounds on its own
  double move = MAG ? a.dw_min * (double)units : a.dw_min;
  if constexpr (NL) {
    const double x = clampd(0.5 * (g + 1.0), 0.0, 1.0);
    move *= up ? ::exp(-a.v * x) : ::exp(-a.v * (1.0 - x));
  }
  double next = g + (up ? 1.0 : -1.0) * move;
  if constexpr (NOISE) {
    NormalStream rng(a.seed, kStreamPulseNoise, (step << 31) | dev);
    if constexpr (MAG) next += a.sigma * ::sqrt((double)units) * rng.get((uint64_t)m * 32 + (uint64_t)ord);
    else next += a.sigma * rng.get((uint64_t)m * 32 + (uint64_t)ord);
  }
  return clampd(next, -1.0, 1.0);
}

// Block = (16 P) x (16 P) devices, thread = P x P of them with their states in registers; the trains
// of a stage of samples go through LDS, transposed ([row or column][sample]) so that a lane reads
// the trains of consecutive samples of its row and of its column with 16-byte loads.
// A device's pulses are sequential, but devices do not wait for each other sample by sample: all
// lanes first mark, in step, the samples of the stage in which their row and column share a slot (one
// bit per sample and device), then every lane works through its own marked samples one pulse per turn,
// so a wave runs for as long as its busiest device has pulses in the stage, not for the sum over the
// samples of the busiest device of each.
// MARKED: the marks come from pulse_mark_kernel (layers with few devices: that pass fills the chip, this
// one cannot) instead of being worked out here, stage by stage.
template <int P, bool NL, bool NOISE, bool MARKED = false, bool MAG = false>
__global__ __launch_bounds__(256) void pulse_apply_kernel(PulseArgs a) {
  constexpr int TE = 16 * P;              // tile edge
  constexpr int ST = 4096 / TE;           // samples per stage (a multiple of 16)
  constexpr int LD = ST + 4;              // words per row or column: 16-byte aligned, spread over the banks
  __shared__ __align__(16) uint32_t rt[TE * LD];
  __shared__ __align__(16) uint32_t ct[TE * LD];
  const int nb = (a.N + TE - 1) / TE;
  const int kt = (blockIdx.x / nb) * TE, nt = (blockIdx.x % nb) * TE;
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  const int k0 = kt + P * ty, n0 = nt + P * tx;
  const uint64_t step = effective_step(a.step, a.step_add);
  double g[P][P];
  int cnt[P][P];
#pragma unroll
  for (int i = 0; i < P; ++i)
#pragma unroll
    for (int j = 0; j < P; ++j) {
      const int k = k0 + i, n = n0 + j;
      cnt[i][j] = 0;
      g[i][j] = 0.0;
      if (k < a.K && n < a.N)
        g[i][j] = a.first ? (double)a.W[(size_t)k * a.N + n] / a.w_max : a.state[(size_t)k * a.N + n];
    }
  for (int s0 = 0; s0 < a.mc; s0 += ST) {
    const int ns = min(ST, a.mc - s0);
    const int ns16 = (ns + 15) & ~15;      // whole groups of 16 (ST is a multiple): samples past the end hold no train
    // the stage's trains: all loads of a thread are issued before the first one is needed
    constexpr int PER = ST * TE / 256;     // 16 elements of either matrix per thread
    uint32_t rv[PER], cv[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int e = threadIdx.x + 256 * u, sm = e / TE, c = e % TE;
      const bool live = sm < ns;
      rv[u] = (live && kt + c < a.K) ? a.rows[(size_t)(s0 + sm) * a.K + kt + c] : 0u;
      cv[u] = (live && nt + c < a.N) ? a.cols[(size_t)(s0 + sm) * a.N + nt + c] : 0u;
    }
    __syncthreads();                       // everyone is done with the previous stage
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int e = threadIdx.x + 256 * u, sm = e / TE, c = e % TE;
      rt[c * LD + sm] = rv[u];
      ct[c * LD + sm] = cv[u];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < P; ++i)
#pragma unroll
      for (int j = 0; j < P; ++j) {
        const uint64_t dev = (uint64_t)(k0 + i) * a.N + (uint64_t)(n0 + j);
        const uint32_t* rp = &rt[(P * ty + i) * LD];
        const uint32_t* cp = &ct[(P * tx + j) * LD];
        double gs = g[i][j];
        int moved = 0;
        // all lanes together: which samples of the stage have a slot in which row and column both fire
        constexpr int NW = ST / 64;
        uint64_t live[NW];
#pragma unroll
        for (int w = 0; w < NW; ++w) {
          live[w] = 0;
          if constexpr (MARKED) {
            const int word = s0 / 64 + w;
            if (word < a.n_words && k0 + i < a.K && n0 + j < a.N)
              live[w] = a.marks[(size_t)word * ((size_t)a.K * a.N) + dev];
            continue;
          }
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int at = 64 * w + 4 * v;
            if (at < ns16) {
              const u32x4 r = *reinterpret_cast<const u32x4*>(rp + at);
              const u32x4 c = *reinterpret_cast<const u32x4*>(cp + at);
              const uint32_t four = (min(r.x & c.x & 0x7FFFFFFFu, 1u)) | (min(r.y & c.y & 0x7FFFFFFFu, 1u) << 1) |
                                    (min(r.z & c.z & 0x7FFFFFFFu, 1u) << 2) | (min(r.w & c.w & 0x7FFFFFFFu, 1u) << 3);
              live[w] |= (uint64_t)four << (4 * v);
            }
          }
        }
        // every lane for itself, one pulse per turn: its marked samples in order, the pulses of a
        // sample in order
        uint32_t q = 0;
        bool up = false;
        int m = 0, ord = 0, units = 1;
        for (;;) {
          if (q == 0) {
            int w = -1;
            uint64_t word = 0;
#pragma unroll
            for (int t = NW - 1; t >= 0; --t)
              if (live[t]) {
                w = t;
                word = live[t];
              }
            if (w < 0) break;                          // the stage is done for this device
            const int e = __builtin_ctzll(word);
#pragma unroll
            for (int t = 0; t < NW; ++t)
              if (t == w) live[t] = word & (word - 1);
            const int at = 64 * w + e;
            const uint32_t rw = rp[at], cw = cp[at];
            q = rw & cw & 0x7FFFFFFFu;
            if constexpr (MAG) {                        // one write of (row height) x (column height) quanta
              units = (int)(rw & 31u) * (int)(cw & 31u);
              q = 1u;
            }
            up = ((rw ^ cw) >> 31) != 0;               // against the sign of x d
            m = a.m0 + s0 + at;
            ord = 0;
          }
          q &= q - 1;
          gs = one_pulse<NL, NOISE, MAG>(a, gs, up, m, ord, dev, step, units);
          ++ord;
          moved += up ? units : -units;
        }
        g[i][j] = gs;
        cnt[i][j] += moved;
      }
  }
#pragma unroll
  for (int i = 0; i < P; ++i)
#pragma unroll
    for (int j = 0; j < P; ++j) {
      const int k = k0 + i, n = n0 + j;
      if (k < a.K && n < a.N) {
        const size_t at = (size_t)k * a.N + n;
        if (a.last) a.W[at] = (float)(a.w_max * g[i][j]);
        else a.state[at] = g[i][j];
        if (a.pulses) a.pulses[at] = (a.first ? 0 : a.pulses[at]) + cnt[i][j];
      }
    }
}

// Two-phase walk for layers with few devices and many samples (convolution layers: a 144 x 16 layer has
// 9 blocks of devices and 131072 samples).  Phase 1, one block per (16 x 16 devices, stage of 256
// samples at a time, 4096 per block), fills the chip: it marks the samples in which a device's row and
// column share a slot, one bit per sample and device, plus one summary bit per 64-sample word that is
// not empty.  Phase 2, one thread per device, walks only the marked samples, in order (summary ->
// word -> sample), fetching their two trains from memory: the sequential part shrinks to the pulses.
__global__ __launch_bounds__(256) void pulse_mark_kernel(PulseArgs a) {
  constexpr int TE = 16, ST = 256, LD = ST + 4, PER = ST * TE / 256, NW = ST / 64, SEG = 64 * 64;
  __shared__ __align__(16) uint32_t rt[TE * LD];
  __shared__ __align__(16) uint32_t ct[TE * LD];
  const int nb = (a.N + TE - 1) / TE, tiles = ((a.K + TE - 1) / TE) * nb;
  const int tile = blockIdx.x % tiles, seg = blockIdx.x / tiles;     // segment = 64 words = 4096 samples
  const int kt = (tile / nb) * TE, nt = (tile % nb) * TE;
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  const int k = kt + ty, n = nt + tx;
  const bool valid = k < a.K && n < a.N;
  const uint32_t* rp = &rt[ty * LD];
  const uint32_t* cp = &ct[tx * LD];
  const size_t kn = (size_t)a.K * a.N, dev = (size_t)k * a.N + n;
  unsigned long long summary = 0;                  // bit = word of the segment that has a marked sample
  for (int s0 = seg * SEG; s0 < min(a.mc, (seg + 1) * SEG); s0 += ST) {
    const int ns = min(ST, a.mc - s0);
    __syncthreads();                               // everyone is done with the previous stage
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int e = threadIdx.x + 256 * u, sm = e / TE, c = e % TE;
      const bool live = sm < ns;
      rt[c * LD + sm] = (live && kt + c < a.K) ? a.rows[(size_t)(s0 + sm) * a.K + kt + c] : 0u;
      ct[c * LD + sm] = (live && nt + c < a.N) ? a.cols[(size_t)(s0 + sm) * a.N + nt + c] : 0u;
    }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const int word = s0 / 64 + w;
      unsigned long long bits = 0;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int at = 64 * w + 4 * v;
        const u32x4 r = *reinterpret_cast<const u32x4*>(rp + at);
        const u32x4 c = *reinterpret_cast<const u32x4*>(cp + at);
        const uint32_t four = (min(r.x & c.x & 0x7FFFFFFFu, 1u)) | (min(r.y & c.y & 0x7FFFFFFFu, 1u) << 1) |
                              (min(r.z & c.z & 0x7FFFFFFFu, 1u) << 2) | (min(r.w & c.w & 0x7FFFFFFFu, 1u) << 3);
        bits |= (unsigned long long)four << (4 * v);
      }
      if (valid && word < a.n_words) {
        a.marks[(size_t)word * kn + dev] = bits;
        if (bits) summary |= 1ull << (word - 64 * seg);
      }
    }
  }
  if (valid) a.summary[(size_t)seg * kn + dev] = summary;
}

template <bool NL, bool NOISE>
__global__ __launch_bounds__(256) void pulse_walk_kernel(PulseArgs a) {
  const size_t kn = (size_t)a.K * a.N;
  const size_t dev = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (dev >= kn) return;
  const int k = (int)(dev / a.N), n = (int)(dev % a.N);
  const uint64_t step = effective_step(a.step, a.step_add);
  const int n_seg = (a.n_words + 63) / 64;
  double gs = a.first ? (double)a.W[dev] / a.w_max : a.state[dev];
  int moved = 0, next_seg = 0, word_base = 0, seg_base = 0, m = 0, ord = 0;
  unsigned long long word = 0, summary = 0;
  uint32_t q = 0;
  bool up = false;
  // every lane for itself, one pulse per turn (as in pulse_apply_kernel)
  for (;;) {
    if (q == 0) {
      if (word == 0) {                               // next word with a marked sample, by way of the summaries
        while (summary == 0 && next_seg < n_seg) {
          summary = a.summary[(size_t)next_seg * kn + dev];
          seg_base = 64 * next_seg;
          ++next_seg;
        }
        if (summary == 0) break;                     // no marked sample left
        const int wi = seg_base + __builtin_ctzll(summary);
        summary &= summary - 1;
        word = a.marks[(size_t)wi * kn + dev];       // not empty: its summary bit is set
        word_base = 64 * wi;
      }
      const int at = word_base + __builtin_ctzll(word);
      word &= word - 1;
      const uint32_t rw = a.rows[(size_t)at * a.K + k], cw = a.cols[(size_t)at * a.N + n];
      q = rw & cw & 0x7FFFFFFFu;                     // not empty: the sample is marked
      up = ((rw ^ cw) >> 31) != 0;
      m = a.m0 + at;
      ord = 0;
    }
    q &= q - 1;
    gs = one_pulse<NL, NOISE>(a, gs, up, m, ord, (uint64_t)dev, step);
    ++ord;
    moved += up ? 1 : -1;
  }
  if (a.last) a.W[dev] = (float)(a.w_max * gs);
  else a.state[dev] = gs;
  if (a.pulses) a.pulses[dev] = (a.first ? 0 : a.pulses[dev]) + moved;
}

constexpr int kTwoPhaseBlocks = 4096;

struct PulsePlan {
  int mc;                       // samples per chunk (the trains of one chunk are resident at a time)
  size_t rows_bytes, cols_bytes, ws_bytes;
  int two_phase;                // mark, then walk the marked samples (few devices, many samples)
  size_t marks_bytes;
};

PulsePlan plan_pulsed(int M, int K, int N) {
  PulsePlan p;
  const long long per_sample = 4ll * ((long long)K + N);
  long long mc = std::max(64ll, ((64ll << 20) / per_sample) / 64 * 64);
  // mark-then-walk where one device per thread does not already come in thousands of blocks and there are
  // enough samples for the marking pass to pay; its marks (one bit per sample and device) stay within 256 MiB
  const long long kn = (long long)K * N;
  const long long mark_samples = ((8ll << 28) / kn) / 4096 * 4096;
  p.two_phase = (long long)cdiv(K, 16) * cdiv(N, 16) < kTwoPhaseBlocks && M >= 2048 && mark_samples >= 4096;
  if (p.two_phase) mc = std::min(mc, mark_samples);
  p.mc = (int)std::min<long long>(mc, M);
  p.rows_bytes = align256((size_t)4 * p.mc * K);
  p.cols_bytes = align256((size_t)4 * p.mc * N);
  p.ws_bytes = p.rows_bytes + p.cols_bytes + align256((size_t)8 * K * N);
  p.marks_bytes = 0;
  if (p.two_phase) {
    p.marks_bytes = align256((size_t)cdiv(p.mc, 64) * 8 * (size_t)K * N) + align256((size_t)cdiv(p.mc, 4096) * 8 * (size_t)K * N);
    p.ws_bytes += p.marks_bytes;
  }
  return p;
}

}  // namespace

namespace xbar_detail {
size_t pulsed_workspace_bytes(int M, int K, int N) { return plan_pulsed(M, K, N).ws_bytes; }
}  // namespace xbar_detail

namespace {
int run_update_pulsed(const xbar_config* cfg, float* W, const float* X, const float* dY, int M, int K, int N, float w_max,
                      float x_range, float d_range, int bl, float dw_min, uint64_t step, long long* pulses, void* ws,
                      size_t ws_bytes, void* hip_stream, const ConvGeom* conv) {
  int rc = xbar_config_validate(cfg);
  if (rc) return rc;
  if ((rc = check_shape(M, K, N))) return rc;
  if (!aligned16(W) || !aligned16(X) || !aligned16(dY) || !aligned16(ws)) return XBAR_EALIGN;
  if (pulses && (reinterpret_cast<uintptr_t>(pulses) & 7u)) return XBAR_EALIGN;
  if (!finite_pos(w_max) || !finite_pos(x_range) || !finite_pos(d_range) || !finite_pos(dw_min)) return XBAR_EINVAL;
  if (bl < 1 || bl > 31 || step >= (1ull << 33)) return XBAR_EINVAL;
  const PulsePlan p = plan_pulsed(M, K, N);
  if (ws_bytes < p.ws_bytes) return XBAR_EWORKSPACE;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  PulseArgs a;
  a.W = W; a.X = X; a.D = dY;
  a.rows = reinterpret_cast<uint32_t*>(ws);
  a.cols = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(ws) + p.rows_bytes);
  a.state = reinterpret_cast<double*>(reinterpret_cast<char*>(ws) + p.rows_bytes + p.cols_bytes);
  a.pulses = pulses;
  a.marks = reinterpret_cast<unsigned long long*>(reinterpret_cast<char*>(ws) + p.rows_bytes + p.cols_bytes +
                                                  align256((size_t)8 * K * N));
  a.summary = reinterpret_cast<unsigned long long*>(reinterpret_cast<char*>(a.marks) +
                                                    align256((size_t)cdiv(p.mc, 64) * 8 * (size_t)K * N));
  a.M = M; a.K = K; a.N = N; a.bl = bl;
  a.flags = cfg->flags;
  a.w_max = (double)w_max; a.x_range = (double)x_range; a.d_range = (double)d_range; a.dw_min = (double)dw_min;
  a.v = (double)cfg->upd_nl_v;
  // the aggregate model's noise for one pulse: its standard deviation gamma sqrt(dG) belongs to the ideal change
  // before the learning rate, and this scheme's mean equals the aggregate update at lr = bl dw_min w_max / (x_range d_range)
  a.coded = (cfg->flags & XBAR_PULSE_CODED) ? 1 : (cfg->flags & XBAR_PULSE_MAGNITUDE) ? 2 : 0;
  coded_frames(bl, &a.tx, &a.td);
  const int slots = a.coded == 1 ? a.tx * a.td : a.coded == 2 ? bl * bl : bl;
  const double lr_eq = (double)slots * (double)dw_min * (double)w_max / ((double)x_range * (double)d_range);
  a.sigma = (double)cfg->upd_noise_gamma * std::sqrt(lr_eq * (double)dw_min);
  a.seed = cfg->seed; a.step = step; a.step_add = current_step_source();
  a.conv = conv ? *conv : ConvGeom{};
  // 4 x 4 devices per thread when that still fills the chip, else one device per thread
  const bool patch4 = (long long)cdiv(K, 64) * cdiv(N, 64) >= 512;
  const int edge = patch4 ? 64 : 16;
  const unsigned tiles = (unsigned)(cdiv(K, edge) * cdiv(N, edge));
  for (int m0 = 0; m0 < M; m0 += p.mc) {
    a.m0 = m0;
    a.mc = std::min(p.mc, M - m0);
    a.first = m0 == 0;
    a.last = m0 + a.mc >= M;
    const long long elems = (long long)a.mc * ((long long)K + N);
    if (conv) hipLaunchKernelGGL(pulse_trains_kernel<true>, dim3((unsigned)((elems + 255) / 256)), dim3(256), 0, st, a);
    else hipLaunchKernelGGL(pulse_trains_kernel<false>, dim3((unsigned)((elems + 255) / 256)), dim3(256), 0, st, a);
    if (hipGetLastError() != hipSuccess) return XBAR_EHIP;
    const bool nl = (cfg->flags & XBAR_NI_UPD_NL) != 0, noise = (cfg->flags & XBAR_NI_UPD_NOISE) != 0;
    if (a.coded == 2) {
      // magnitude coding: a device is written in every sample in which both of its lines carry a pulse, so
      // there is little for a marking pass to skip; always the staged kernel
      void (*k)(PulseArgs);
      if (patch4)
        k = nl ? (noise ? pulse_apply_kernel<4, true, true, false, true> : pulse_apply_kernel<4, true, false, false, true>)
               : (noise ? pulse_apply_kernel<4, false, true, false, true> : pulse_apply_kernel<4, false, false, false, true>);
      else
        k = nl ? (noise ? pulse_apply_kernel<1, true, true, false, true> : pulse_apply_kernel<1, true, false, false, true>)
               : (noise ? pulse_apply_kernel<1, false, true, false, true> : pulse_apply_kernel<1, false, false, false, true>);
      hipLaunchKernelGGL(k, dim3(tiles), dim3(256), 0, st, a);
      if (hipGetLastError() != hipSuccess) return XBAR_EHIP;
      continue;
    }
    if (p.two_phase) {
      a.n_words = cdiv(a.mc, 64);
      const unsigned tiles16 = (unsigned)(cdiv(K, 16) * cdiv(N, 16));
      hipLaunchKernelGGL(pulse_mark_kernel, dim3(tiles16 * (unsigned)cdiv(a.mc, 4096)), dim3(256), 0, st, a);
      if (hipGetLastError() != hipSuccess) return XBAR_EHIP;
      if (noise) {
        // lanes decoupled over the whole chunk: with a normal number per pulse every turn counts
        void (*walk)(PulseArgs) = nl ? pulse_walk_kernel<true, true> : pulse_walk_kernel<false, true>;
        hipLaunchKernelGGL(walk, dim3((unsigned)cdiv(K * N, 64)), dim3(64), 0, st, a);     // one wave per block: spread over the chip
      } else {
        // cheap pulses: the trains of a stage in LDS beat the walk's loads from memory (measured 6.7 against
        // 9.6 ms on a 144 x 16 layer with 131072 samples; with noise 21 against 15 ms)
        void (*staged)(PulseArgs) = nl ? pulse_apply_kernel<1, true, false, true> : pulse_apply_kernel<1, false, false, true>;
        hipLaunchKernelGGL(staged, dim3(tiles16), dim3(256), 0, st, a);
      }
      if (hipGetLastError() != hipSuccess) return XBAR_EHIP;
      continue;
    }
    void (*k)(PulseArgs);
    if (patch4)
      k = nl ? (noise ? pulse_apply_kernel<4, true, true> : pulse_apply_kernel<4, true, false>)
             : (noise ? pulse_apply_kernel<4, false, true> : pulse_apply_kernel<4, false, false>);
    else
      k = nl ? (noise ? pulse_apply_kernel<1, true, true> : pulse_apply_kernel<1, true, false>)
             : (noise ? pulse_apply_kernel<1, false, true> : pulse_apply_kernel<1, false, false>);
    hipLaunchKernelGGL(k, dim3(tiles), dim3(256), 0, st, a);
    if (hipGetLastError() != hipSuccess) return XBAR_EHIP;
  }
  return XBAR_OK;
}
}  // namespace

extern "C" {

int xbar_update_pulsed(const xbar_config* cfg, float* W, const float* X, const float* dY, int M, int K, int N, float w_max,
                       float x_range, float d_range, int bl, float dw_min, uint64_t step, long long* pulses, void* ws,
                       size_t ws_bytes, void* hip_stream) {
  return run_update_pulsed(cfg, W, X, dY, M, K, N, w_max, x_range, d_range, bl, dw_min, step, pulses, ws, ws_bytes,
                           hip_stream, nullptr);
}

int xbar_conv_update_pulsed(const xbar_config* cfg, float* W, const float* X, const float* dY, const xbar_conv_geom* geom,
                            int N, float w_max, float x_range, float d_range, int bl, float dw_min, uint64_t step,
                            long long* pulses, void* ws, size_t ws_bytes, void* hip_stream) {
  ConvGeom g;
  int M, K;
  const int rc = conv_dims(geom, &g, &M, &K);
  if (rc) return rc;
  return run_update_pulsed(cfg, W, X, dY, M, K, N, w_max, x_range, d_range, bl, dw_min, step, pulses, ws, ws_bytes,
                           hip_stream, conv_is_dense(geom) ? nullptr : &g);
}

int xbar_pulse_slots(const xbar_config* cfg, int bl) {
  const int rc = xbar_config_validate(cfg);
  if (rc) return rc;
  if (bl < 1 || bl > 31) return XBAR_EINVAL;
  if (cfg->flags & XBAR_PULSE_MAGNITUDE) return bl * bl;
  if (!(cfg->flags & XBAR_PULSE_CODED)) return bl;
  int tx, td;
  coded_frames(bl, &tx, &td);
  return tx * td;
}

}  // extern "C"
