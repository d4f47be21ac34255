/*
 * xbar -- functional emulation of non-ideal resistive-crossbar training operations on one MI355X.
 *
 * C ABI of the GPU library.  Plain pointers and sizes only; every tensor pointer is a DEVICE pointer
 * to row-major contiguous memory that the caller owns (allocate it with any HIP allocator, e.g. a
 * torch tensor) and that must be 16-byte aligned.  The library never allocates or frees device
 * memory and never synchronises: every call only enqueues kernels on the HIP stream that is passed
 * in (NULL = the default stream) and returns.  Scratch memory comes from the caller (`ws`); its
 * contents are undefined after a call and two calls that share one workspace must be ordered on one
 * stream.  Return value: XBAR_OK or a negative XBAR_E* code; no exception crosses this boundary and
 * the library keeps no state between calls (two per-thread settings aside: the one-shot instrumentation
 * hook at the end and the optional step counter of xbar_set_step_source).
 *
 * A layer is the GEMM  Y[M x N] = X[M x K] . W[K x N]:  K = fan-in = crossbar rows, N = fan-out =
 * crossbar columns, M = batch (times output positions after im2col).  The weight matrix is cut into
 * crossbar instances of xbar_rows x xbar_cols devices; every weight is stored as
 * S_w = weight_bits / slice_bits devices of slice_bits each (least significant slice first) in a
 * positive or a negative array; inputs are streamed in S_in = input_bits / stream_bits cycles of
 * stream_bits each; signed inputs are applied in two phases (positive part, negative part), or in one
 * phase of offset-binary codes with XBAR_INPUT_OFFSET.
 * Model after TxSim (arXiv 2002.11151): Sec. IV (layer = DAC -> array -> ADC, forward and
 * backward), Sec. IV-A (non-ideal conductance matrix generator), Sec. IV-B (three-stage model),
 * Sec. IV-C (update model), Sec. IV-D (approximate analytical wire model, stored distortion
 * profile), Sec. V (parameter values).
 */
#ifndef XBAR_H_
#define XBAR_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define XBAR_ABI_VERSION 2u

/* flags */
#define XBAR_NI_VARIATION    1u   /* per-device multiplicative Gaussian process variation (Sec. IV-A)   */
#define XBAR_NI_WIRE_AAM     2u   /* wire parasitics, approximate analytical model (Sec. IV-D)          */
#define XBAR_NI_WIRE_PROFILE 4u   /* wire parasitics from a stored distortion profile (Sec. IV-D)       */
#define XBAR_NI_UPD_NL       8u   /* state-dependent write non-linearity (Sec. IV-C)                    */
#define XBAR_NI_UPD_NOISE    16u  /* Gaussian write noise (Sec. IV-C)                                   */
#define XBAR_DAC_LUT         32u  /* DAC levels from dac_lut instead of equidistant (Sec. IV-B).  1-bit
                                     cycles with dac_lut[0] == 0 cost nothing (one factor on the gain);
                                     other tables up to 4 bits per cycle take one contraction per level
                                     in the unpipelined kernel variant; 8-bit cycles: ENOTSUP            */
#define XBAR_INPUT_SIGNED    64u  /* forward inputs are signed (two phases); backward always is         */
#define XBAR_ADC_CURVE       256u /* non-linear converter: monotone transfer curve adc_curve (Sec. IV-B, V);
                                     runs in the unpipelined kernel variant                              */
#define XBAR_NI_WIRE_AAM2    128u /* wire parasitics, analytical model with every first-order path: the
                                     drops that all devices of a row / column cause on the wire segments
                                     they share (Sec. IV-D: more paths than the shortest one); at most one
                                     of the three wire flags                                             */
#define XBAR_ADC_PER_ARRAY   512u /* one unsigned converter per array instead of one signed converter on
                                     the difference of the array pair (a variant of the pair of Sec. IV-A):
                                     code = clamp(rne(I_array * gain), 0, Q), Q = 2^adc_bits - 1, gain =
                                     float(Q) / adc_fs; the codes of the negative array are subtracted
                                     digitally.  Twice the conversions and contraction work; adc_bits <= 15;
                                     not with XBAR_ADC_CURVE                                             */
#define XBAR_INPUT_OFFSET    1024u /* signed inputs (forward with XBAR_INPUT_SIGNED, backward always) are
                                     streamed in ONE phase as offset-binary codes instead of two phases
                                     of magnitudes (variant for drivers that supply 0 .. v_max only, Sec. V):
                                     u = rne((x / scale + 1) / 2 * (2^input_bits - 1)), coded value
                                     (2 u - Qa) / Qa * scale (steps twice as coarse; zero lies half a step
                                     beside a code); the half-range is removed digitally:
                                     out = float(double(sum) * 2 lsb scale w_max / (Qa Qw)
                                                 - double(wsum) * scale w_max / Qw),
                                     wsum = sum of the quantised weights of that output (xbar_tile keeps
                                     them in the plane buffer).  Every input is driven, also a zero and a
                                     convolution's padding (mid-range): size adc_fs for that.  Half the
                                     conversions and contraction work of the two-phase scheme          */
#define XBAR_PULSE_CODED     2048u /* pulse-level updates use deterministic, time-coded pulses (Sec. IV-C names
                                     them beside the stochastic streams) instead of random trains: the bl
                                     slots form Tx frames of Td sub-slots, Tx = floor(sqrt(bl)), Td =
                                     floor(bl / Tx); a row holds its line for the first rne(p_x Tx) frames, a
                                     column fires in the first rne(p_d Td) sub-slots of every frame, so a
                                     device sees exactly rne(p_x Tx) rne(p_d Td) coincidences; Tx Td takes the
                                     place of bl in the learning rate.  seed and step then only key the
                                     write noise                                                        */

#define XBAR_PULSE_MAGNITUDE 4096u /* pulse-level updates use ONE pulse per sample and line whose height codes the value
                                     (the other coding Sec. IV-C names): a row carries a pulse of height
                                     lx = rne(p_x bl) out of bl levels, a column one of height ld = rne(p_d bl), and the
                                     device answers the product of the two heights with one write of lx ld quanta of
                                     dw_min; bl^2 takes the place of bl in the learning rate.  The non-linearity is
                                     evaluated once per write, at the state it finds; the noise is one draw of standard
                                     deviation gamma sqrt(lr lx ld dw_min) (normal number m 32 of the device's stream).
                                     The reported pulse count is the signed number of quanta.  Not with
                                     XBAR_PULSE_CODED                                                     */

/* status codes */
#define XBAR_OK          0
#define XBAR_EINVAL     -1   /* bad parameter struct (sizes, bit widths, NaN/negative physical values) */
#define XBAR_ESHAPE     -2   /* M, K or N not positive, K*N >= 2^31, or M*K / M*N >= 2^38             */
#define XBAR_EALIGN     -3   /* a pointer is NULL or not 16-byte aligned                              */
#define XBAR_EWORKSPACE -4   /* workspace / plane buffer smaller than the size query says             */
#define XBAR_EHIP       -5   /* a HIP call failed (kernel launch)                                     */
#define XBAR_ENOTSUP    -6   /* valid in the model, not implemented by the GPU kernels                */
#define XBAR_ESCRATCH   -7   /* xbar_fwd_static: the shape needs more than XBAR_STATIC_SCRATCH_BYTES   */

/* operations, for xbar_workspace_bytes */
#define XBAR_OP_FWD    0
#define XBAR_OP_BWD    1
#define XBAR_OP_UPDATE 2
#define XBAR_OP_FCM    3   /* pass M = 1 */
#define XBAR_OP_UPDATE_PULSED 4

/* Parameter struct: plain data, caller-owned, read during the call only (Sec. IV lists the three
 * input groups; Sec. V and VI-B give the values used in the paper, quoted below as "paper:"). */
typedef struct xbar_config {
  uint32_t struct_size;   /* sizeof(xbar_config) */
  uint32_t abi_version;   /* XBAR_ABI_VERSION */
  int32_t xbar_rows;      /* R: 64, 128 or 256 (multiple of 16 in 16..256)       paper: 64            */
  int32_t xbar_cols;      /* C: same range                                       paper: 64            */
  int32_t weight_bits;    /* magnitude bits of a weight, 1..16; the sign selects the array            */
  int32_t slice_bits;     /* bits per device, divides weight_bits, 1..4          paper: 2             */
  int32_t input_bits;     /* magnitude bits of an input, 1..8                                         */
  int32_t stream_bits;    /* bits per DAC cycle, divides input_bits              paper: 1             */
  int32_t adc_bits;       /* 2..16, signed mid-tread converter with Q = 2^(adc_bits-1) - 1 codes/side */
  uint32_t flags;         /* XBAR_NI_* | XBAR_DAC_LUT | XBAR_ADC_CURVE | XBAR_INPUT_SIGNED |          */
                          /*   XBAR_ADC_PER_ARRAY | XBAR_INPUT_OFFSET | XBAR_PULSE_CODED | XBAR_PULSE_MAGNITUDE */
  float r_min, r_max;     /* device resistance range in Ohm                      paper: 1e5, 1e6      */
  float v_max;            /* input voltage range in V (results do not depend on it) paper: 1          */
  float r_row, r_col;     /* wire resistance per cell in Ohm                     paper: 1, 4.6        */
  float r_source, r_sense;/* driver / sense resistance in Ohm (paper names them, gives no value)      */
  float var_sigma;        /* relative standard deviation of the device variation                      */
  float upd_nl_v;         /* write non-linearity factor v                        paper: 0.01          */
  float upd_noise_gamma;  /* write noise factor gamma                            paper: 5             */
  float adc_fs_fwd;       /* ADC full scale of the forward pass, in units of (one input level) x      */
  float adc_fs_bwd;       /*   (one device level); same for the backward pass.  Code = clamp(         */
                          /*   rne(I * gain), -Q, Q) with gain = float(Q) / adc_fs in single          */
                          /*   precision; LSB = adc_fs / Q.                                           */
  float dac_lut[16];      /* voltage of DAC level i divided by v_max, used with XBAR_DAC_LUT          */
  float adc_curve[17];    /* with XBAR_ADC_CURVE: values in [-1, 1], non-decreasing, of the converter's  */
                          /*   transfer curve f at x = -1 + i/8 (x = current / adc_fs, clamped; linear   */
                          /*   between the points); code = clamp(rne(Q f(x)), -Q, Q).  f(x) = x is the   */
                          /*   linear converter.  Evaluated in single precision on the GPU.              */
  uint64_t seed;          /* key of the counter-based random numbers (Philox-4x32-10 + Box-Muller)    */
} xbar_config;

/* Host-only checks of the parameter struct (no GPU needed). */
int xbar_config_validate(const xbar_config* cfg);
const char* xbar_strerror(int code);
uint32_t xbar_abi_version(void);

/*
 * Non-ideal conductance matrix generator (Sec. IV-A, Sec. IV-D): weights -> bit-sliced conductance
 * planes per crossbar tile, stitched as U = (G+ - G-) / (one device level), in the operand layout of
 * the contraction kernels (one copy for the forward, one for the backward direction); with
 * XBAR_ADC_PER_ARRAY the planes G+ / level and G- / level are kept apart (twice the bytes).
 *   W        [K][N] float, read only (the preserved ideal copy of Sec. IV-A)
 *   w_max    weights are clamped to [-w_max, w_max] and quantised to weight_bits magnitude bits,
 *            q = rne(clamp(W / w_max) * (2^weight_bits - 1)), evaluated in double precision
 *   step     keys the variation draw: the same (seed, step) gives the same devices
 *   profile  [S_w][2][K][N] float distortion D (index 1: 0 = positive array), G <- G (1 - D);
 *            required with XBAR_NI_WIRE_PROFILE, ignored otherwise
 *   planes   output, xbar_planes_bytes(cfg, K, N) bytes, opaque
 * With XBAR_NI_WIRE_AAM2 the plane buffer also holds (16 S_w + 4) K N bytes of scratch, and wherever 6-bit planes
 * carry an array non-ideality other than the single-path wire model alone (variation, profile, all-paths model,
 * XBAR_ADC_PER_ARRAY) 4 S_w K N bytes per array: every device is computed once there and both copies are packed
 * from it (the size query includes both); tile (i, j) indices count from the tile's first row / column, devices beyond K / N
 * carry no current.
 * Device (slice s, array pol) of weight (k, n) uses normal number ((k N + n) S_w + s) 2 + pol of
 * the variation stream.  Rows / columns beyond K / N hold no device.
 */
size_t xbar_planes_bytes(const xbar_config* cfg, int K, int N);
int xbar_tile(const xbar_config* cfg, const float* W, int K, int N, float w_max, uint64_t step,
              const float* profile, void* planes, size_t planes_bytes, void* hip_stream);

/*
 * Step counter in device memory, for callers that replay a captured HIP graph of a training step: kernel
 * arguments are frozen in a graph, so the `step` that keys the device variation (Sec. IV-A) and the write
 * noise (Sec. IV-C) would repeat.  After xbar_set_step_source(p) every later call of this host thread that
 * takes a `step` (xbar_tile, xbar_update, xbar_conv_update, xbar_update_pulsed, xbar_conv_update_pulsed, xbar_fcm_profile) uses
 * step + *p, read by the kernels when they run; NULL switches it off.  p: 8-byte aligned device address that
 * stays valid while such kernels may run.  xbar_step_advance enqueues *p += 1 on the stream (one thread, no
 * memset: it can be part of the graph).
 */
void xbar_set_step_source(const unsigned long long* device_step);
int xbar_step_advance(unsigned long long* device_step, void* hip_stream);

/* Bytes of scratch memory that xbar_fwd / xbar_bwd / xbar_update need for this shape. */
size_t xbar_workspace_bytes(const xbar_config* cfg, int op, int M, int K, int N);

/*
 * Forward VMM (Sec. IV, IV-B): Y[M][N] from X[M][K] through the planes of xbar_tile.
 *   a = rne(clamp(X / x_scale, lo, 1) * (2^input_bits - 1)) in double precision, lo = -1 with
 *   XBAR_INPUT_SIGNED else 0; every (row tile, slice, cycle, phase) column current is converted by
 *   its own ADC, the codes are shifted and added over slices, cycles, phases and row tiles in
 *   integers, and Y = float(double(sum) * lsb * x_scale * w_max / ((2^input_bits-1)(2^weight_bits-1))).
 *   codes: NULL, or int16 [phase][cycle][slice][row tile][M][N] receiving every ADC code (testing);
 *   with XBAR_ADC_PER_ARRAY [phase][cycle][slice][array][row tile][M][N], array 0 = positive weights,
 *   and the sum takes the codes of array 1 negatively.
 */
int xbar_fwd(const xbar_config* cfg, const void* planes, const float* X, float* Y, int M, int K, int N,
             float w_max, float x_scale, void* ws, size_t ws_bytes, int16_t* codes, void* hip_stream);

/*
 * xbar_fwd for callers that cannot allocate or hand over scratch memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the same kernels and results as xbar_fwd without
 * the code tap, with the workspace in an array of XBAR_STATIC_SCRATCH_BYTES that the library holds on every
 * GPU it runs on until the process ends.  The call allocates and frees nothing; its first call on a device
 * looks the array's address up (with that device current).  Shapes whose xbar_workspace_bytes(cfg,
 * XBAR_OP_FWD, M, K, N) exceeds the array return XBAR_ESCRATCH and enqueue nothing.  All calls on one GPU
 * share the array: two calls must not overlap (order them on one stream, or synchronise between streams);
 * nothing in it has to start at zero (every byte that is read is written first by the same call).
 */
#define XBAR_STATIC_SCRATCH_BYTES (32u << 20)
int xbar_fwd_static(const xbar_config* cfg, const void* planes, const float* X, float* Y, int M, int K, int N,
                    float w_max, float x_scale, void* hip_stream);

/*
 * Backward VMM (Sec. IV: same procedure as forward): dX[M][K] from dY[M][N]; the same devices are
 * driven from the columns and read on the rows, one ADC conversion per (column tile, slice, cycle,
 * phase), accumulated over column tiles.  dY / g_scale is quantised like a signed forward input.
 *   codes: NULL, or int16 [phase][cycle][slice][column tile][M][K] ([..][slice][array][column tile][..]
 *   with XBAR_ADC_PER_ARRAY).
 */
int xbar_bwd(const xbar_config* cfg, const void* planes, const float* dY, float* dX, int M, int K, int N,
             float w_max, float g_scale, void* ws, size_t ws_bytes, int16_t* codes, void* hip_stream);

/*
 * Weight update (Sec. IV-C): W[K][N] in place from X[M][K] and dY[M][N].
 *   grad = sum_m X[m][k] dY[m][n];  delta = grad_scale * grad (ideal change, in units of Gmax-Gmin,
 *   state g = W / w_max in [-1, 1]);  write non-linearity: delta * exp(-v x) when the conductance
 *   rises, delta * exp(-v (1 - x)) when it falls, x = (g + 1) / 2;  write noise:
 *   + gamma sqrt(|delta|) * normal number (k N + n) of the write stream of `step`;
 *   g <- clamp(g - lr * written, -1, 1);  W <- w_max g.
 */
int xbar_update(const xbar_config* cfg, float* W, const float* X, const float* dY, int M, int K, int N,
                float w_max, float grad_scale, float lr, uint64_t step, void* ws, size_t ws_bytes,
                void* hip_stream);

/*
 * Weight update with per-polarity device state (variant of xbar_update; Sec. IV-A keeps the positive and the
 * negative conductances of the weights in two arrays, Sec. IV-C writes one conductance per weight): the two
 * devices of a weight are states of their own, Gp[K][N] and Gn[K][N] in [0, 1] (units of Gmax - Gmin above
 * Gmin), W = w_max (Gp - Gn).  The ideal change delta (as in xbar_update) is split evenly and applied in
 * opposite directions: gp <- clamp(gp - lr w_p, 0, 1), gn <- clamp(gn + lr w_n, 0, 1), where each device sees
 * delta / 2, scaled by the write non-linearity at ITS OWN state and direction (exp(-v g) rising,
 * exp(-v (1 - g)) falling) plus gamma sqrt(|delta| / 2) times normal number 2 (k N + n) + pol (pol 0 =
 * positive device) of stream 6 of `step`.  Gp, Gn in place; W receives w_max (Gp - Gn) for xbar_tile.
 * With v = gamma = 0 and no device at a rail the weights move exactly as under xbar_update.
 * xbar_pair_init places a weight symmetrically about mid-range: gp = (1 + g) / 2, gn = (1 - g) / 2,
 * g = clamp(W / w_max, -1, 1).  Workspace: xbar_workspace_bytes(cfg, XBAR_OP_UPDATE, ...) (convolution:
 * xbar_conv_workspace_bytes).
 */
int xbar_pair_init(const float* W, float* Gp, float* Gn, int K, int N, float w_max, void* hip_stream);
int xbar_update_pair(const xbar_config* cfg, float* Gp, float* Gn, float* W, const float* X, const float* dY, int M,
                     int K, int N, float w_max, float grad_scale, float lr, uint64_t step, void* ws, size_t ws_bytes,
                     void* hip_stream);

/*
 * Pulse-level weight update (Sec. IV-C names the parallel update schemes whose result xbar_update
 * models in one aggregate write; this is the scheme with stochastic pulse trains): W[K][N] in place,
 * one sample at a time and one pulse at a time, the gradient is never formed.
 *   Sample m drives row k with a random train of `bl` slots (1..31) that fires with probability
 *   min(1, |X[m][k]| / x_range) per slot, column n likewise from dY[m][n] / d_range; device (k, n) is
 *   pulsed once per slot in which both fire, against the sign of X dY (descent).  Expected pulses:
 *   bl p_x p_d, so the mean written change is the outer-product update with learning rate
 *   bl dw_min w_max / (x_range d_range).
 *   Train: slot j of element i (i = m K + k for rows, m N + n for columns) fires when uniform word j
 *   of the element (Philox-4x32-10 block 8 i + j / 4, word j % 4, counter words 2, 3 = step, key =
 *   seed mixed with stream 3 for rows, 4 for columns, as for the normal numbers) is below rne(p 2^32).
 *   Pulse: state g = W / w_max moves by dw_min; with XBAR_NI_UPD_NL the move is scaled by exp(-v x)
 *   upwards and exp(-v (1 - x)) downwards, x = (g + 1) / 2 at the state the pulse finds; with
 *   XBAR_NI_UPD_NOISE every pulse adds upd_noise_gamma sqrt(lr dw_min), lr the learning rate above (the noise
 *   xbar_update gives the same change: there the standard deviation belongs to the change before the
 *   learning rate), times normal number m 32 + j (j = ordinal of the pulse within the sample) of stream 5
 *   of step (step << 31) | (k N + n); g is clamped to [-1, 1] after every pulse.  Double precision throughout, W <- float(w_max g) at the end.
 *   step < 2^33.  pulses: NULL, or int64 [K][N] receiving the signed number of pulses per device.
 *   ws: xbar_workspace_bytes(cfg, XBAR_OP_UPDATE_PULSED, M, K, N).
 */
int xbar_update_pulsed(const xbar_config* cfg, float* W, const float* X, const float* dY, int M, int K, int N,
                       float w_max, float x_range, float d_range, int bl, float dw_min, uint64_t step,
                       long long* pulses, void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Convolution layers (Sec. IV: a layer's kernels are the columns of its weight matrix, one output
 * position applies one input patch to the rows).  Activations are NHWC float tensors; the weight
 * matrix W[K][N] has K = k_h k_w in_c rows ordered (kh, kw, c) with c fastest and N = output
 * channels; M = batch x out_h x out_w.  The patches are gathered on the fly by the input stage (no
 * im2col matrix is materialised in the forward pass or the update); positions outside the image read 0.
 *   xbar_conv_fwd     Y[batch][out_h][out_w][N]  from X[batch][in_h][in_w][in_c]; codes as xbar_fwd
 *   xbar_conv_bwd     dX (shape of X) from dY (shape of Y): xbar_bwd gives the error of every patch
 *                     element into the workspace, every input pixel then adds up, in fp32, the errors
 *                     of the patches it belongs to (a digital accumulation)
 *   xbar_conv_update  W in place from X and dY, as xbar_update on the patch matrix
 *   xbar_conv_update_pulsed  W in place, as xbar_update_pulsed on the patch matrix: every output position is
 *                     one sample (its patch drives the rows, its error the columns), element index
 *                     i = m K + k of the row trains counts in the patch matrix
 * out_h must equal (in_h + 2 pad - k_h) / stride + 1 (likewise out_w), else XBAR_ESHAPE.
 * xbar_conv_workspace_bytes: op = XBAR_OP_FWD / XBAR_OP_BWD / XBAR_OP_UPDATE / XBAR_OP_UPDATE_PULSED.
 */
typedef struct xbar_conv_geom {
  int32_t batch, in_h, in_w, in_c;
  int32_t k_h, k_w, stride, pad;
  int32_t out_h, out_w;
} xbar_conv_geom;

size_t xbar_conv_workspace_bytes(const xbar_config* cfg, int op, const xbar_conv_geom* geom, int N);
int xbar_conv_fwd(const xbar_config* cfg, const void* planes, const float* X, float* Y, const xbar_conv_geom* geom,
                  int N, float w_max, float x_scale, void* ws, size_t ws_bytes, int16_t* codes, void* hip_stream);
int xbar_conv_bwd(const xbar_config* cfg, const void* planes, const float* dY, float* dX, const xbar_conv_geom* geom,
                  int N, float w_max, float g_scale, void* ws, size_t ws_bytes, void* hip_stream);
int xbar_conv_update(const xbar_config* cfg, float* W, const float* X, const float* dY, const xbar_conv_geom* geom,
                     int N, float w_max, float grad_scale, float lr, uint64_t step, void* ws, size_t ws_bytes,
                     void* hip_stream);
int xbar_conv_update_pair(const xbar_config* cfg, float* Gp, float* Gn, float* W, const float* X, const float* dY,
                          const xbar_conv_geom* geom, int N, float w_max, float grad_scale, float lr, uint64_t step,
                          void* ws, size_t ws_bytes, void* hip_stream);   /* as xbar_update_pair on the patch matrix */
int xbar_conv_update_pulsed(const xbar_config* cfg, float* W, const float* X, const float* dY,
                            const xbar_conv_geom* geom, int N, float w_max, float x_range, float d_range, int bl,
                            float dw_min, uint64_t step, long long* pulses, void* ws, size_t ws_bytes,
                            void* hip_stream);

/*
 * Digital peripheral operations (Sec. IV-B: ReLU, batch normalisation and pooling are computed in the
 * digital domain, untouched by the crossbar non-idealities), the loss and the plain SGD step of the
 * digital parameters, so that a whole training step can stay on the GPU.  Float NHWC tensors, n =
 * number of elements; `rows` = batch x positions, channels fastest.  Statistics are accumulated in
 * double precision in a fixed order.
 *   relu_bwd      takes the forward OUTPUT y (dx = dy where y > 0)
 *   sigmoid       y = 1 / (1 + exp(-x)); sigmoid_bwd takes the forward OUTPUT y (dx = dy y (1 - y))
 *   bn_fwd        training mode: per-channel batch mean and biased variance; writes y, mean and
 *                 invstd = 1 / sqrt(var + eps) (kept for bn_bwd)
 *   bn_bwd        dx, dgamma = sum dy xhat, dbeta = sum dy; ws: xbar_bn_workspace_bytes(rows, channels)
 *   avgpool       global average over the `positions` of every (sample, channel)
 *   maxpool       square window k_h = k_w with stride and padding from the geometry struct (in_c =
 *                 channels, 2 pad <= k); argmax[out element] = position ih * in_w + iw of the first
 *                 maximum, kept for maxpool_bwd
 *   softmax_xent  loss[b] = -log softmax(logits[b])[labels[b]]; dlogits = scale (softmax - onehot);
 *                 a label outside [0, classes) gives a NaN loss and no target
 *   sgd           p <- p - lr g
 *   shortcut      parameter-free residual shortcut across a stage boundary: y[b][oh][ow][:] = x[b][oh stride]
 *                 [ow stride][:] with (out_channels - channels) zero channels added, half in front
 *   absmax        result[0] (device) = max |x[i]|; ws: 4096 bytes.  For choosing the input ranges
 *                 (x_scale, g_scale, w_max) of a layer from data (Sec. IV-B: ranges are data dependent).
 */
int xbar_relu_fwd(const float* x, float* y, size_t n, void* hip_stream);
int xbar_relu_bwd(const float* y, const float* dy, float* dx, size_t n, void* hip_stream);
int xbar_sigmoid_fwd(const float* x, float* y, size_t n, void* hip_stream);
int xbar_sigmoid_bwd(const float* y, const float* dy, float* dx, size_t n, void* hip_stream);
int xbar_add(const float* a, const float* b, float* y, size_t n, void* hip_stream);
int xbar_sgd(float* p, const float* g, size_t n, float lr, void* hip_stream);
size_t xbar_bn_workspace_bytes(size_t rows, int channels);
int xbar_bn_fwd(const float* x, const float* gamma, const float* beta, float* y, float* mean, float* invstd, size_t rows,
                int channels, float eps, void* ws, size_t ws_bytes, void* hip_stream);
int xbar_bn_bwd(const float* x, const float* dy, const float* gamma, const float* mean, const float* invstd, float* dx,
                float* dgamma, float* dbeta, size_t rows, int channels, void* ws, size_t ws_bytes, void* hip_stream);
int xbar_avgpool_fwd(const float* x, float* y, int batch, int positions, int channels, void* hip_stream);
int xbar_avgpool_bwd(const float* dy, float* dx, int batch, int positions, int channels, void* hip_stream);
int xbar_maxpool_fwd(const float* x, float* y, int32_t* argmax, const xbar_conv_geom* geom, void* hip_stream);
int xbar_maxpool_bwd(const float* dy, const int32_t* argmax, float* dx, const xbar_conv_geom* geom, void* hip_stream);
int xbar_softmax_xent(const float* logits, const int32_t* labels, float* loss, float* dlogits, int batch, int classes,
                      float scale, void* hip_stream);
int xbar_shortcut_fwd(const float* x, float* y, int batch, int h, int w, int channels, int stride, int out_channels,
                      void* hip_stream);
int xbar_shortcut_bwd(const float* dy, float* dx, int batch, int h, int w, int channels, int stride, int out_channels,
                      void* hip_stream);
int xbar_absmax(const float* x, size_t n, float* result, void* ws, size_t ws_bytes, void* hip_stream);

/*
 * ADC range statistics (Sec. IV-B: the maximum current through the ADCs is data dependent and comes
 * from output distribution statistics).  Runs the input stage and the contraction of xbar_fwd
 * (op = XBAR_OP_FWD: in = X[M][K]) or xbar_bwd (XBAR_OP_BWD: in = dY[M][N]) and, instead of
 * converting, counts every column current that an ADC would see: hist[b] += number of conversions
 * with rne(|I| / bin_width) == b, the last of the 4096 bins takes everything beyond.  I and bin_width
 * are in the unit of adc_fs (one input level x one device level); adc_bits / adc_fs of cfg are not used.
 * With XBAR_ADC_PER_ARRAY the currents counted are those of the single arrays.
 *   hist  4096 uint64 device counters, added to (clear them before the first call)
 *   ws    the workspace of the same xbar_fwd / xbar_bwd call
 * The caller picks adc_fs from the histogram (a high quantile, rounded up as it sees fit).
 */
#define XBAR_ADC_HIST_BINS 4096
int xbar_adc_histogram(const xbar_config* cfg, const void* planes, const float* in, int M, int K, int N,
                       float in_scale, int op, float bin_width, unsigned long long* hist, void* ws, size_t ws_bytes,
                       void* hip_stream);
/* The same for a convolution layer: op = XBAR_OP_FWD takes the NHWC image X (patches gathered as in
 * xbar_conv_fwd), op = XBAR_OP_BWD the errors dY[batch][out_h][out_w][N]; ws as for xbar_conv_fwd / the
 * crossbar part of xbar_conv_bwd (xbar_conv_workspace_bytes of the same op is enough). */
int xbar_conv_adc_histogram(const xbar_config* cfg, const void* planes, const float* in, const xbar_conv_geom* geom,
                            int N, float in_scale, int op, float bin_width, unsigned long long* hist, void* ws,
                            size_t ws_bytes, void* hip_stream);

/*
 * Circuit-level crossbar model (Sec. IV-A: Ohm's and Kirchhoff's laws solved for every crossbar
 * instance; Sec. IV-D: its result kept as the distortion profile D = (G_ideal - G_nonideal) / G_ideal
 * and reused for the following iterations).  For every crossbar tile, slice and array the exact
 * linear map from row voltages to sensed column currents is computed (wire geometry as in the
 * analytical model: driver at the column-0 end of every row wire through r_source, sense at the far
 * end of every column wire through r_sense, r_row / r_col per cell; devices beyond K / N absent);
 * entry (i, j) of that map is the non-ideal conductance of device (i, j).
 *   W, w_max, step  as for xbar_tile (the variation draw of `step` is included when its flag is set;
 *                   the wire flags of cfg are ignored)
 *   profile         output [S_w][2][K][N] float, the input format of XBAR_NI_WIRE_PROFILE
 *   ws              xbar_workspace_bytes(cfg, XBAR_OP_FCM, 1, K, N) bytes
 * Iterative solve (conjugate gradients on the device currents, relative residual 1e-11, at most 500
 * iterations per driven row); cost grows with R times the number of devices.
 */
int xbar_fcm_profile(const xbar_config* cfg, const float* W, int K, int N, float w_max, uint64_t step,
                     float* profile, void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Instrumentation for the benchmark (no part of the method): one-shot, per host thread.  The next
 * xbar_fwd or xbar_bwd call of this thread records the HIP event `before` on its stream right before
 * the contraction kernel (the dominant kernel; the input quantiser runs before it, the output
 * scaling after it) and `after` right behind it.  Both are hipEvent_t handles owned by the caller.
 */
void xbar_trace_next_vmm(void* before, void* after);

/*
 * Instrumentation for the benchmark (no part of the method): enqueues a kernel that does nothing but
 * dependent-chain fp16 matrix instructions (the instruction the contraction uses, v_mfma_f32_32x32x16_f16)
 * on register-resident operands, 2 waves per SIMD on every CU, so that the caller can time the matrix
 * rate the chip sustains (it is power limited well below the nominal peak once operands toggle).
 *   mode 0: both operands pseudo-random fp16;  mode 1: B operand = sparse single-bit patterns as in
 *   the emulation, A pseudo-random.   iters: loop count; the kernel issues 16 * iters MFMAs per wave
 *   on 2048 waves, i.e. 2 * 16 * iters * 2048 * 16384 flops.   out: 2 MiB of device scratch.
 *   modes 2, 3: the same two operand patterns with the 8-bit integer instruction
 *   (v_mfma_i32_32x32x32_i8, twice the operations per instruction), for comparison.
 *   mode 4: the block-scaled 6-bit x 4-bit instruction (v_mfma_scale_f32_32x32x64_f8f6f4, four times the
 *   operations per instruction) on pseudo-random 6-bit codes and single-bit digits.
 *   modes 5, 6: the inner loop of the contraction kernel itself on synthetic operands (its code, not a
 *   copy): 4 terms, 128-row tiles, two row patches per wave, plane fragments read from LDS; mode 5 without
 *   and mode 6 with the ADC / shift-and-add operations woven between the matrix instructions.  Each
 *   iteration is two (slice, cycle) passes = 32 matrix instructions per wave; time(6) / time(5) - 1 is the
 *   time the fused epilogue adds.  The kernel uses 48 KiB of LDS.
 */
int xbar_probe_mfma_rate(int mode, int iters, void* out, size_t out_bytes, void* hip_stream);

/*
 * ADC range from measured statistics (Sec. IV-B: the converter's maximum current comes from output
 * distribution statistics): the smallest power of two that is at least the `quantile` (in (0, 1]) of the
 * |column current| distribution counted by xbar_adc_histogram, hist[b] = conversions with
 * rne(|I| / bin_width) == b; the current of bin b is taken as (b + 0.5) bin_width, at least bin_width.
 * Host-only: `hist` is a HOST copy of the `bins` counters.  Returns 0 for invalid arguments.
 */
float xbar_adc_range_from_histogram(const unsigned long long* hist, int bins, float bin_width, double quantile);

/*
 * Slots of a pulse train of `bl` slots that carry pulses (what takes the place of bl in the learning rate
 * of xbar_update_pulsed): bl for stochastic trains, Tx Td with XBAR_PULSE_CODED.  Host-only.  Negative status
 * for an invalid configuration or bl outside 1..31.
 */
int xbar_pulse_slots(const xbar_config* cfg, int bl);

/*
 * Operand format that the contraction uses for this configuration (information for the benchmark's
 * accounting): returns 0 = fp16 planes (v_mfma_f32_32x32x16_f16) or 1 = 6-bit planes with 4-bit digits
 * (v_mfma_scale_f32_32x32x64_f8f6f4; cycles of 1 or 2 bits without a general DAC level table), or a
 * negative status for an invalid configuration; *terms (may be NULL) receives the number of operand terms
 * a plane value is split into, i.e. matrix instructions issued per useful one.
 */
int xbar_plane_format(const xbar_config* cfg, int* terms);

#ifdef __cplusplus
}
#endif
#endif /* XBAR_H_ */
