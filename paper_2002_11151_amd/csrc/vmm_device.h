// Contraction kernels of libxbar.so (crossbar-tile contraction + ADC + shift-and-add, Sec. IV-B) as
// templates, so that their instantiations can be compiled in several translation units side by side:
// vmm_f16_a.hip / vmm_f16_b.hip (fp16 planes), vmm_f6_a.hip / vmm_f6_b.hip (6-bit planes), and the
// instrumentation kernels of xbar.hip.  Internal: the boundary is include/xbar.h.
#ifndef XBAR_VMM_DEVICE_H_
#define XBAR_VMM_DEVICE_H_

#include "xbar_common.h"
#include <type_traits>

namespace xbar_detail {

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
  int flush_every;            // 32-bit sums: added to the block's own 64-bit partial sum every so many virtual tiles (0: never)
  int direct;                 // single chunk and nothing to correct: the kernel scales and stores the result itself
  int total_wg, per_xcd;
  float gain;          // float(Q) / adc_fs
  float clamp_lo, clamp_hi;   // kMagic -+ Q
  uint32_t bias_per_vt;       // kMagicBits * sum of all shift weights, mod 2^32
  float* out;                 // final output, written directly when there is a single chunk
  double scale;               // lsb * in_scale * w_max / (Qa * Qw)
};

constexpr int kStatBins = 4096;
static __shared__ uint32_t stat_hist[kStatBins];   // per-block histogram of the statistics pass (code-tap variants only)

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
// LOW_FIRST (one converter per array): the smaller terms first, the leading term last.  A single array's
// current is a sum of positive products that only grows, so the leading sum is large when the residual
// products land on it and every one of those steps rounds at its magnitude; the other way round the residual
// sum is small (precise), and the exact leading products round only where the sum crosses into a new binade:
// about one unit in the last place of the result in all, instead of one per residual step.
template <int TERMS, int NK, bool LOW_FIRST>
__device__ __forceinline__ constexpr int fragment_of_step(int i) {
  return LOW_FIRST ? (TERMS - 1 - i / NK) * NK + i % NK : i;
}

template <int PM, int NK, int TERMS, bool LOW_FIRST = false>
__device__ __forceinline__ void vmm_contract(const half8 (&ab)[PM][NK], const u32x4* bptr, float16v (&acc)[PM]) {
  constexpr int NF = TERMS * NK;
  u32x4 f0 = bptr[fragment_of_step<TERMS, NK, LOW_FIRST>(0) * 64],
        f1 = NF > 1 ? bptr[fragment_of_step<TERMS, NK, LOW_FIRST>(1) * 64] : f0;
#pragma unroll
  for (int i = 0; i < NF; ++i) {
    const u32x4 cur = f0;
    f0 = f1;
    if (i + 2 < NF) f1 = bptr[fragment_of_step<TERMS, NK, LOW_FIRST>(i + 2) * 64];
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
template <int PM, int NK, int TERMS, bool DO_ADC, bool LOW_FIRST = false>
__device__ __forceinline__ void vmm_contract_adc(const half8 (&ab)[PM][NK], const u32x4* bptr, float16v (&acc)[PM],
                                                 const float16v (&old)[PM], float gain_old, float clamp_lo,
                                                 float clamp_hi, int sh_old, uint32_t (&y)[PM][16]) {
  constexpr int NF = TERMS * NK;
  constexpr int NV = 16 * PM;                       // conversions of the previous result
  const float vmagic = kMagic;
  constexpr int PF = NF < 2 ? NF : 2;               // fragments in flight from LDS
  u32x4 fr[PF];
#pragma unroll
  for (int i = 0; i < PF; ++i) fr[i] = bptr[fragment_of_step<TERMS, NK, LOW_FIRST>(i) * 64];
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int i = 0; i < NF; ++i) {
    const u32x4 cur = fr[i % PF];
    if (i + PF < NF) fr[i % PF] = bptr[fragment_of_step<TERMS, NK, LOW_FIRST>(i + PF) * 64];
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
        vmm_contract_adc<PM, NK, TERMS, false, PER_ARRAY>(ab, bbase + (size_t)sl * NF * 64, acc0, acc1, gain_prev, clamp_lo,
                                               clamp_hi, sh_prev, y);
      else
        vmm_contract_adc<PM, NK, TERMS, true, PER_ARRAY>(ab, bbase + (size_t)sl * NF * 64, acc0, acc1, gain_prev, clamp_lo,
                                              clamp_hi, sh_prev, y);
      // odd slice -> acc1, while the ADC of the even slice (acc0) runs
      vmm_contract_adc<PM, NK, TERMS, true, PER_ARRAY>(ab, bbase + (size_t)(sl + 1) * NF * 64, acc1, acc0, gain_b, clamp_lo,
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
          vmm_contract<PM, NK, TERMS, PER_ARRAY>(ab, lds + lane + (size_t)sl * NF * 64, part);
          const float volt = a.dac_lut[level];
#pragma unroll
          for (int pm = 0; pm < PM; ++pm)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[pm][r] = __builtin_fmaf(volt, part[pm][r], acc[pm][r]);
        }
      } else {
        vmm_contract<PM, NK, TERMS, PER_ARRAY>(ab, lds + lane + (size_t)sl * NF * 64, acc);
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
    for (int f = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); f < nfr; f += nwv) {   // wave index: scalar
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

// Digits of one streaming cycle as E2M1 codes (digit d is code d, value d / 2).  The input stage stores the 8-bit
// magnitudes of a lane's 8 inputs nibble by nibble: 4-bit field f of word 0 holds the low four bits of input
// f / 2 of the first (f even) or the second (f odd) group of four, word 1 the high four bits; a cycle's digits are
// then one shift and one AND per 8 inputs.  HIGH: the cycle's bits lie in the high nibbles (word 1);
// `shift`: their place within the nibble; `nibble_mask`: the digit mask in every 4-bit field.
template <int NK64, bool HIGH>
__device__ __forceinline__ void digit_codes_f4(const u32x2 (&raw)[4 * NK64], int shift, uint32_t nibble_mask, int4v (&dg)[NK64]) {
#pragma unroll
  for (int J = 0; J < NK64; ++J)
#pragma unroll
    for (int w = 0; w < 4; ++w) dg[J][w] = (int)(((HIGH ? raw[4 * J + w].y : raw[4 * J + w].x) >> shift) & nibble_mask);
}

// The same for a cycle whose place is known at run time only (general path).
template <int NK64>
__device__ __forceinline__ void digit_codes_f4_any(const u32x2 (&raw)[4 * NK64], int in_shift, uint32_t nibble_mask, int4v (&dg)[NK64]) {
  if (in_shift >= 4) digit_codes_f4<NK64, true>(raw, in_shift - 4, nibble_mask, dg);
  else digit_codes_f4<NK64, false>(raw, in_shift, nibble_mask, dg);
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
template <int PM, int NK64, int NT, bool DO_ADC, bool LOW_FIRST = false>
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
    const int f = fragment_of_step<NT, NK64, LOW_FIRST>(i);
    const int off = (f / NK64) * STRIDE + (f % NK64) * 1536;
    fx[i] = *reinterpret_cast<const u32x4*>(xb + off);
    fy[i] = *reinterpret_cast<const u32x2*>(yb + off);
    // keeps the 8-byte reads of the first two fragments apart: merged into one instruction they land in
    // registers of their own and have to be copied behind the 16-byte parts
    __builtin_amdgcn_sched_barrier(0);
  }
#pragma unroll
  for (int i = 0; i < NF; ++i) {
    const u32x4 cx = fx[i % PF];
    const u32x2 cy = fy[i % PF];
    if (i + PF < NF) {
      const int f = fragment_of_step<NT, NK64, LOW_FIRST>(i + PF);
      const int off = (f / NK64) * STRIDE + (f % NK64) * 1536;
      fx[i % PF] = *reinterpret_cast<const u32x4*>(xb + off);
      fy[i % PF] = *reinterpret_cast<const u32x2*>(yb + off);
    }
    const int8v pa = {(int)cx.x, (int)cx.y, (int)cx.z, (int)cx.w, (int)cy.x, (int)cy.y, 0, 0};
    const int term = fragment_of_step<NT, NK64, LOW_FIRST>(i) / NK64, J = i % NK64;
#pragma unroll
    for (int pm = 0; pm < PM; ++pm) {
      const int8v pb = {dg[pm][J][0], dg[pm][J][1], dg[pm][J][2], dg[pm][J][3], 0, 0, 0, 0};
      if (i == 0) {
        const float16v zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        acc[pm] = mfma_f6_term(term, pa, pb, zero, scale_lo, scale_hi);
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
  const uint32_t nibble_mask = ((1u << a.stream_bits) - 1u) * 0x11111111u;
  float gain_p, clamp_lo, clamp_hi;
  adc_sign_and_range<PER_ARRAY>(a, p, pol, gain_p, clamp_lo, clamp_hi);
  const float gain = 2.0f * gain_p;                   // a digit enters as d / 2
  const char* xb = lds + lane * 16;
  const char* yb = lds + 1024 + lane * 8;
  int4v dg[PM][NK64];
  float16v acc0[PM], acc1[PM];
  int sh_prev = 0;
  // one streaming cycle: digits, then every slice pair; `high`: the cycle's bits are in the high nibbles
  auto cycle = [&](int b, auto high) {
    const int in_shift = a.stream_bits * b;
#pragma unroll
    for (int pm = 0; pm < PM; ++pm) digit_codes_f4<NK64, decltype(high)::value>(raw[pm], in_shift & 3, nibble_mask, dg[pm]);
    for (int sl = 0; sl < ns; sl += 2) {
      const int sh0 = a.slice_bits * (shift_slice0 + sl) + in_shift;
      const int sh1 = sh0 + a.slice_bits;
      if (b == 0 && sl == 0)
        vmm6_contract_adc<PM, NK64, NT, false, PER_ARRAY>(dg, xb + sl * SLICE, yb + sl * SLICE, acc0, acc1, gain, clamp_lo, clamp_hi,
                                               sh_prev, y, a.scale_lo, a.scale_hi);
      else
        vmm6_contract_adc<PM, NK64, NT, true, PER_ARRAY>(dg, xb + sl * SLICE, yb + sl * SLICE, acc0, acc1, gain, clamp_lo, clamp_hi,
                                              sh_prev, y, a.scale_lo, a.scale_hi);
      vmm6_contract_adc<PM, NK64, NT, true, PER_ARRAY>(dg, xb + (sl + 1) * SLICE, yb + (sl + 1) * SLICE, acc1, acc0, gain, clamp_lo,
                                            clamp_hi, sh0, y, a.scale_lo, a.scale_hi);
      sh_prev = sh1;
    }
  };
  const int b_low = min(a.S_in, 4 / a.stream_bits);   // cycles whose bits lie in the low nibbles
  for (int b = 0; b < b_low; ++b) cycle(b, std::false_type{});
  for (int b = b_low; b < a.S_in; ++b) cycle(b, std::true_type{});
  vmm_adc_narrow<PM>(acc1, gain, clamp_lo, clamp_hi, sh_prev, y);   // drain
}

// General slice group (64-bit sums, code tap, transfer curve, statistics, odd slice counts).
template <int PM, int NK64, int NT, bool WIDE, bool CODES, bool PER_ARRAY>
__device__ __forceinline__ void vmm6_tile_group(const VmmArgs& a, const char* lds, const u32x2 (&raw)[PM][4 * NK64], int ns,
                                                int sg0, int p, int pol, int t, int lane, int mp0, int op,
                                                uint32_t (&y)[PM][16], long long (&y64)[PM][16]) {
  constexpr int SLICE = NT * f6_term_stride(NK64);
  const uint32_t nibble_mask = ((1u << a.stream_bits) - 1u) * 0x11111111u;
  float gain_p, clamp_lo, clamp_hi;
  adc_sign_and_range<PER_ARRAY>(a, p, pol, gain_p, clamp_lo, clamp_hi);
  const float gain = 2.0f * gain_p;
  const char* xb = lds + lane * 16;
  const char* yb = lds + 1024 + lane * 8;
  for (int b = 0; b < a.S_in; ++b) {
    const int in_shift = a.stream_bits * b;
    int4v dg[PM][NK64];
#pragma unroll
    for (int pm = 0; pm < PM; ++pm) digit_codes_f4_any<NK64>(raw[pm], in_shift, nibble_mask, dg[pm]);
    for (int sl = 0; sl < ns; ++sl) {
      const int s = sg0 + sl;
      const int sh = a.slice_bits * s + in_shift;
      float16v acc[PM], none[PM];
      uint32_t unused[PM][16];
      vmm6_contract_adc<PM, NK64, NT, false, PER_ARRAY>(dg, xb + sl * SLICE, yb + sl * SLICE, acc, none, 0.f, 0.f, 0.f, 0, unused,
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
    for (int c = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); c < ncopy; c += nwv) {   // wave index: scalar
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
  // the wave index is the same for all lanes: as a scalar, everything derived from it (row patches, addresses) is scalar too
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), nw = blockDim.x >> 6;
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
  }
#undef XBAR_ALL_VIRTUAL_TILES
  // 32-bit sums hold only a few virtual tiles (3 with 16-bit weights, 8-bit inputs and an 8-bit converter).
  // Rather than cutting the contraction into that many more chunks, each with a partial result of its own
  // in memory, a block with more virtual tiles than that adds its sums to a 64-bit partial result every
  // `flush_every` tiles: every element has one owner lane, which reads back only what it wrote itself.
  int since = 0;
  const bool flushing = WIDE == 0 && a.flush_every > 0 && vt1 - vt0 > a.flush_every;
  for (int vt = vt0; vt < vt1; ++vt) {
    /* vt = (phase, array, tile), tile fastest */
    const int pa = vt / a.T, t = vt - pa * a.T;
    const int p = PER_ARRAY ? pa >> 1 : pa, pol = PER_ARRAY ? pa & 1 : 0;
    const int rows = min(a.tile, a.Lin - t * a.tile);
    run_tile(a, lds, p, pol, t, rows, lane, mp0, op, y, y64, 0);
    ++since;
    if constexpr (WIDE == 0) {
      if (flushing && since == a.flush_every && vt + 1 < vt1) {
        const bool first = vt + 1 - vt0 == a.flush_every;
        const uint32_t bias = a.bias_per_vt * (uint32_t)since;
        long long* part = reinterpret_cast<long long*>(a.part) + (size_t)chunk * a.M * a.Lout;
        int lane_now = lane, mp_now = mp0;              // as above: no element addresses kept across the contraction
        asm volatile("" : "+v"(lane_now), "+v"(mp_now));
#pragma unroll
        for (int pm = 0; pm < PM; ++pm)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int m = (mp_now + pm) * 32 + (lane_now & 31);
            const int o = op * 32 + 8 * (r >> 2) + 4 * (lane_now >> 5) + (r & 3);
            if (m < a.M && o < a.Lout && mp_now + pm < a.MP) {
              long long v = (long long)(int32_t)(y[pm][r] - bias);
              if (!first) v += part[(size_t)m * a.Lout + o];
              part[(size_t)m * a.Lout + o] = v;
            }
            y[pm][r] = 0;
          }
        since = 0;
      }
    }
  }
  if constexpr (CODES) {
    if (a.hist) {                                  // statistics pass: the counters are the only result
      __syncthreads();
      for (int i = threadIdx.x; i < kStatBins; i += blockDim.x)
        if (stat_hist[i]) atomicAdd(&a.hist[i], (unsigned long long)stat_hist[i]);
      return;
    }
  }
  // partial result of this chunk
  const uint32_t bias = a.bias_per_vt * (uint32_t)since;
#pragma unroll
  for (int pm = 0; pm < PM; ++pm)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = (mp0 + pm) * 32 + (lane & 31);
      const int o = op * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      if (m < a.M && o < a.Lout && mp0 + pm < a.MP) {
        const size_t idx = ((size_t)chunk * a.M + m) * a.Lout + o;
        long long sum = WIDE ? y64[pm][r] : (long long)(int32_t)(y[pm][r] - bias);
        if (flushing) sum += reinterpret_cast<const long long*>(a.part)[idx];
        if (a.direct) {        // nothing to add up across chunks: scale and store the result itself
          a.out[idx] = (float)((double)sum * a.scale);
        } else if (WIDE || a.flush_every > 0) {
          reinterpret_cast<long long*>(a.part)[idx] = sum;
        } else {
          reinterpret_cast<int32_t*>(a.part)[idx] = (int32_t)sum;
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

// ---------------------------------------------------------------------------------------------
// host side: launch plan and launch of one kernel variant
// ---------------------------------------------------------------------------------------------
struct VmmPlan {
  PlaneGeom g;
  int ks16;            // k-steps of 16 rows per tile in the staged input
  int sg;              // kFmtF6: slices per staged group
  int Lin, Lout, MP, P, VT, vt_per_chunk, nchunk, pm, nw, MB, lds_kb;
  int wide;            // 0: sums fit 32 bits; 1: 64-bit sums; 2: 32-bit sums per slice group, widened per group
  int flush_every;     // wide == 0: virtual tiles a 32-bit sum holds, when a chunk has more than that (else 0)
  int split_sg;        // slices per group of mode 2
  uint32_t bias_split; // kMagicBits * sum of the shift weights of one such group, mod 2^32
  int offset;          // signed inputs in one phase of offset-binary codes
  uint32_t bias_per_vt;
  size_t a_bytes, part_bytes, ws_bytes, lds_bytes;
};

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

// Launchers, one per translation unit of kernel instantiations.
XBAR_INTERNAL hipError_t launch_vmm_f16_a(const VmmArgs& a, const VmmPlan& p, int terms, bool codes, hipStream_t st);   // tiles of up to 128 rows
XBAR_INTERNAL hipError_t launch_vmm_f16_b(const VmmArgs& a, const VmmPlan& p, int terms, bool codes, hipStream_t st);   // tiles of up to 256 rows
XBAR_INTERNAL hipError_t launch_vmm_f6_a(const VmmArgs& a, const VmmPlan& p, int terms, bool codes, hipStream_t st);    // 1 or 4 terms
XBAR_INTERNAL hipError_t launch_vmm_f6_b(const VmmArgs& a, const VmmPlan& p, int terms, bool codes, hipStream_t st);    // 5 terms

}  // namespace xbar_detail

#endif  // XBAR_VMM_DEVICE_H_
