/*
 * mixdq.h — C ABI of the MI355X (gfx950) quantized-linear library.
 *
 * The library implements the deployment hot path that the MixDQ paper (arxiv 2405.17873)
 * configures: mixed-precision quantized linear layers of a text-to-image UNet.
 *
 * Conventions (all entry points)
 *   - Return value: MQ_OK (0) or a negative MQ_ERR_* code.  Nothing is printed, nothing aborts.
 *   - Every pointer is a DEVICE pointer unless its name ends in _host.  The caller owns every buffer;
 *     the library allocates no device memory.  Scratch memory is a caller-provided workspace whose
 *     size comes from the matching *_workspace_bytes() query (256-byte aligned, contents on entry
 *     irrelevant, contents on return unspecified).  A workspace is in use from the call until the
 *     work the call enqueued has finished: calls on ONE stream may share a workspace, calls that
 *     may run at the same time on different streams need a workspace each.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue work on
 *     that stream and return without synchronising.  Arguments are validated on the host before any
 *     launch; a call that returns an error has launched nothing.
 *   - Weights are W[N,K] (output channel x input channel, K contiguous), activations X[M,K] with row
 *     stride ldx (elements), outputs Y[M,N] with row stride ldy (elements).
 *   - Quantisation parameters follow the paper's problem statement (Sec. 4.1 "Quantization Scheme"):
 *     one bit-width per layer, scale (float32) and zero point (int32) per output channel for weights,
 *     one scale and zero point per tensor for activations (device pointers to one element each).
 *   - 16-bit floats are IEEE binary16 (MQ_F16) or bfloat16 (MQ_BF16), passed as raw 2-byte elements.
 */
#ifndef MIXDQ_H
#define MIXDQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MQ_OK 0
#define MQ_ERR_BAD_ARG (-1)             /* null required pointer, contradictory options, misaligned pointer */
#define MQ_ERR_BAD_SHAPE (-2)           /* non-positive size, stride smaller than the row, K not a multiple of the pack group */
#define MQ_ERR_UNSUPPORTED_BITS (-3)    /* bits outside {2,3,4,8} (or outside {4,8} where stated) */
#define MQ_ERR_WORKSPACE_TOO_SMALL (-4)
#define MQ_ERR_HIP (-5)                 /* a HIP runtime call failed; see mq_last_hip_error() */
#define MQ_ERR_UNSUPPORTED_LAYOUT (-6)  /* the GEMM entry points take MQ_LAYOUT_KERNEL only */
#define MQ_ERR_OVERFLOW_RISK (-7)       /* K so large that an int32 accumulator could overflow (255*255*K >= 2^31) */
#define MQ_ERR_INFEASIBLE (-8)          /* bit-width allocation: no assignment fits the budget */
#define MQ_ERR_TOO_LARGE (-9)           /* bit-width allocation: the exact search outgrew its state limit */

#define MQ_LAYOUT_CANONICAL 0 /* interchange format: each row a little-endian bit stream, code k at bits [k*b, k*b+b) */
#define MQ_LAYOUT_KERNEL 1    /* opaque tile-major format consumed by the GEMMs; needs K % 64 == 0 */

#define MQ_F16 0
#define MQ_BF16 1

/* Library version and the last HIP error code seen by a failing call (0 if none). */
int mq_version(void);
int mq_last_hip_error(void);

/* Tuning and test hook: force the GEMM workgroup tile (0: 128x256, 1: 128x128, 2: 64x64, 3 and 4: as 1 and 2 with the
 * reduction split over two wave groups inside the workgroup, 5: 64x128, 6: 96x256; -1: automatic choice
 * from the problem shape; a mode that does not have the tile takes its nearest one).  Process-wide, not thread safe;
 * results do not depend on the tile beyond the order of the fp32 sums. */
void mq_tune_force_tile(int tile);

/* Tuning and test hook: split of a GEMM's reduction over several workgroups per output tile (0: automatic, for
 * problems with few tiles and a long reduction; 1: never; n > 1: n parts wherever the reduction has that many
 * pipeline stages).  The partial sums pass through the caller's workspace (mq_split_workspace_bytes).  In the
 * automatic mode a call whose workspace is absent or too small splits into fewer parts or not at all; with a forced
 * part count such a call returns MQ_ERR_WORKSPACE_TOO_SMALL.  A split result is deterministic (the parts are added
 * in a fixed order) but may differ from the unsplit one in the last bit of a 16-bit output.
 * Process-wide, not thread safe. */
void mq_tune_force_splits(int parts);

/* Workspace that lets the weight-only and 8-bit-activation linears split the reduction of an [M,K] x [N,K] problem
 * over several workgroups per output tile (an upper bound over the tile choices; 0 for shapes that are never split:
 * more than 64 tiles of 128 x 128, or K < 1024).  It depends on the current mq_tune_force_splits setting. */
size_t mq_split_workspace_bytes(int M, int N, int K);

/* Tuning and test hook: height, in row blocks, of the bands in which a GEMM's workgroups walk the output tiles
 * (0: automatic; 1: row block by row block; n: n row blocks side by side, column by column).  It decides which
 * operand tiles the workgroups that run at the same time share in a cache, never a result.  Process-wide, not thread
 * safe. */
void mq_tune_force_band(int rows);

/* Per-kernel timing for benchmarks.  While enabled, every kernel launch of the library is bracketed by two HIP
 * events recorded on the stream it is launched on.  mq_prof_read waits for the pending events of one slot and
 * returns, accumulated since the last reset: the kernel's name (host buffer), number of launches, elapsed
 * milliseconds, algorithmic operations (2*M*N*K per GEMM launch) and algorithmic bytes (activations read once,
 * packed weights, per-channel vectors, output written once).  Host bookkeeping only; costs two event records per
 * launch.  Slots 0..mq_prof_num_slots()-1; slots that never ran report zero launches. */
int mq_prof_enable(int on);
int mq_prof_num_slots(void);
int mq_prof_read(int slot, char* name_host, int name_cap, long long* launches_host, double* ms_host,
                 double* ops_host, double* bytes_host);
int mq_prof_reset(void);
/* An event pair costs a few microseconds of stream time and breaks back-to-back dispatch, so a benchmark that also
 * reports whole-run throughput restricts the bracketing: only launches of `slot` (-1: every kernel), and of those
 * only every `stride`-th.  Totals then cover the bracketed launches only. */
int mq_prof_filter(int slot, int stride);
/* Microseconds an event pair adds to the kernel it brackets, measured (once, synchronising on `stream`) with a
 * one-workgroup kernel that spins for 20 us of the constant 100 MHz clock.  Subtract it from a bracketed average
 * to compare with a profiler's kernel durations. */
double mq_prof_bracket_overhead_us(void* stream);
/* A plain device-to-device copy kernel (kernel name mq::prof_copy_kernel) of `bytes` bytes (multiple of 16, 16-byte
 * aligned pointers): the known-size reference that hardware HBM traffic counters are scaled by. */
int mq_prof_copy(void* dst, const void* src, size_t bytes, void* stream);

/* Microbenchmarks of the chip, for reporting results against what this machine can reach (the published peaks assume
 * the highest clock).  Runs one kernel of fixed work five times between events on `stream`, synchronises, and writes
 * the best elapsed time in milliseconds to *ms_host.  buf: device memory, 16-byte aligned, at least 4 KiB (kind 5: the
 * region that is streamed; make it larger than the last-level cache).  Work per launch:
 *   0  int8 MFMA only: 512 workgroups x 4 waves x 4096 x 4 MFMAs of 32x32x32 (65536 operations each)
 *   1  fp16 MFMA only: the same count of 32x32x16 MFMAs (32768 operations each)
 *   2  vector ALU only: 512 x 4 waves x 4096 x 32 instructions (the cycles of kind 0's MFMAs)
 *   3  the MFMAs of 0 and the ALU instructions of 2 interleaved in ONE wave (1 MFMA, 8 ALU instructions, ...)
 *   4  the MFMA waves of 0 and the ALU waves of 2 side by side, one of each on every SIMD
 *   5  read-only stream over buf: buf_bytes - 4096 bytes read
 *   6  LDS reads (ds_read_b128, the GEMMs' swizzled row pattern): 1024 workgroups x 4 waves x 4000 x 8 KiB
 *   7  L2 -> LDS copies (the LDS-writing buffer loads of the GEMMs' operand pipeline) out of the first 2 MiB of buf
 *      (buf_bytes >= 2 MiB), which stay in every XCD's L2: 768 workgroups x 4 waves x 2048 x 8 KiB
 *   8  as 3 with 4 ALU instructions behind every MFMA instead of 8
 * Kinds 2 to 4 and 8 show how far matrix and vector instructions overlap on one SIMD: how many vector instructions
 * fit under a 32-cycle MFMA before they cost time of their own. */
int mq_prof_microbench(int kind, void* buf, size_t buf_bytes, double* ms_host, void* stream);

/* Phase timing inside the GEMM kernels: while clk != NULL every GEMM launch with at most `workgroups` workgroups
 * writes four shader-clock samples per workgroup (start, main loop entered, epilogue entered, end) to
 * clk[4*workgroup .. 4*workgroup+3] (device memory, caller owned).  Clocks of different XCDs are not comparable;
 * differences inside one workgroup are.  Pass NULL to switch it off. */
void mq_prof_phase_buffer(long long* clk, long workgroups);

/* ------------------------------------------------------------------------------------------------
 * Offline preparation
 * ---------------------------------------------------------------------------------------------- */

/* Uniform min-max quantisation of a weight matrix, one (scale, zero point) per output channel
 * (paper Sec. 4.1 "Quantization Scheme"; bit-widths per layer, Sec. 3.3).
 *   w        [N,K] 16-bit floats (dtype MQ_F16 or MQ_BF16), K contiguous.
 *   bits     2, 3, 4 or 8.
 *   symmetric == 0: asymmetric; the range is widened to contain 0; scale = (hi-lo)/(2^bits-1),
 *                   zp = clamp(rne(-lo/scale)), code = clamp(rne(x/scale) + zp, 0, 2^bits-1); all fp32,
 *                   x/scale taken as one multiply by the fp32 reciprocal; an all-zero row gets scale 1.
 *   symmetric != 0: scale = absmax/(2^(bits-1)-1), code = clamp(rne(x/scale), -Q, Q) stored as two's
 *                   complement int8, zp = 0.
 *   codes    [N,K] uint8 out (one code per byte), scale [N] float out, zp [N] int32 out.
 * Errors: MQ_ERR_BAD_ARG (null pointer, bad dtype), MQ_ERR_BAD_SHAPE, MQ_ERR_UNSUPPORTED_BITS, MQ_ERR_HIP. */
int mq_quantize_weights(const void* w, int N, int K, int bits, int symmetric, int dtype, uint8_t* codes,
                        float* scale, int32_t* zp, void* stream);

/* Size in bytes of the packed form of an N x K code matrix.  Canonical: N*K*bits/8 (needs K*bits % 8 == 0).
 * Kernel layout: ceil(N/32)*32 rows are stored (padding rows hold code 0), K % 64 == 0 is required.
 * bits = 16 stands for unquantised 16-bit weights (paper Sec. 4.2 and App. C item 1: about 1 % of the layers,
 * the most sensitive ones, stay at FP16): they take the same tile order, 2 bytes per weight.
 * Returns 0 for an unsupported combination. */
size_t mq_packed_bytes(int N, int K, int bits, int layout);

/* Bit-pack one-code-per-byte weights (storage accounting of the paper's Tab. 1 "Storage Opt.").
 *   codes   [N,K] uint8; only the low `bits` bits of each code are used.
 *   packed  mq_packed_bytes(...) bytes out.
 *   colsum  nullable [N] int32 out: sum over k of the code, read as two's complement int8 when
 *           codes_signed != 0 (8-bit symmetric weights), else as unsigned.  The integer GEMMs need it.
 *   bits = 16: `codes` points to [N,K] 16-bit values (fp16 or bf16 bit patterns; the packer only moves them),
 *           canonical is the matrix itself, colsum must be null.
 * Errors: as above plus MQ_ERR_BAD_SHAPE when K is not a multiple of the layout's group. */
int mq_pack_weights(const uint8_t* codes, int N, int K, int bits, int layout, int codes_signed, void* packed,
                    int32_t* colsum, void* stream);

/* Inverse of mq_pack_weights for either layout (a test aid; also converts between layouts).  bits = 16: `codes`
 * receives [N,K] 16-bit values. */
int mq_unpack_weights(const void* packed, int N, int K, int bits, int layout, uint8_t* codes, void* stream);

/* ------------------------------------------------------------------------------------------------
 * Hot path
 * ---------------------------------------------------------------------------------------------- */

/* Layers that share their input (the q, k, v projections of a block; K and V of the text context) can run as one
 * call: in MQ_LAYOUT_KERNEL a weight matrix is stored in tiles of 32 output channels, so the packed form of the
 * row-stacked matrix [N1 + N2 + ..., K] is the concatenation of the parts' packed buffers (every Ni % 32 == 0, same
 * K and bits), and scale / zero point / colsum concatenate likewise.  One launch instead of three fills the chip
 * better, and the activations are quantised once. */

/* Weight-only linear, W{2,3,4,8}A16 (paper App. C item 2: low-bit weights, 16-bit floating-point compute):
 *     Y[m,n] = round16( sum_k X[m,k] * scale[n] * (code[n,k] - zp[n]) + bias[n] ),  fp32 accumulation.
 *   x      [M,K] row stride ldx, 16-byte aligned, ldx % 8 == 0.     y [M,N] row stride ldy, 16-byte aligned, ldy % 8 == 0.
 *   packed MQ_LAYOUT_KERNEL, unsigned codes.   bias nullable [N] (same 16-bit dtype as x and y).
 *   K % 64 == 0, N % 8 == 0, M*ldx*2 < 2^31 bytes, (N+31)*K < 2^31 elements and, at bits = 16, < 2^30.
 *   ws, ws_bytes  optional workspace (ws may be NULL) of mq_split_workspace_bytes(M, N, K) bytes: with it, a problem of
 *   few output tiles and a long reduction (a handful of rows against K >= 1024) is spread over more workgroups.
 *   bits = 16: the layer is kept at 16 bits; packed holds the weights themselves (same dtype as x) in
 *   MQ_LAYOUT_KERNEL, w_scale and w_zp are ignored (may be null):  Y = round16( sum_k X[m,k] * W[n,k] + bias[n] ).
 *   residual nullable [M,N] of the same 16-bit dtype, row stride ldr (ldr % 4 == 0, 8-byte aligned): added in fp32
 *   before the rounding, Y = round16( ... + bias[n] + residual[m,n] ).  It may be y itself.  It serves a block's skip
 *   connection, and the split of a layer over a channel-concatenated input [trunk | shortcut] into two layers with
 *   their own quantisation parameters (paper Sec. 4.1, "Quantization Scheme"): the second call adds the first one's
 *   output.  The same operand, with the same meaning, exists on the entry points below that take `residual`. */
int mq_qlinear_w_only(const void* x, int M, int K, int ldx, const void* packed, int N, int bits, int layout,
                      const float* w_scale, const int32_t* w_zp, const void* bias, void* y, int ldy, int dtype,
                      const void* residual, int ldr, void* ws, size_t ws_bytes, void* stream);

/* Workspace for the 8-bit-activation entry points below (M rows of K activations): the int8 copy of the activations,
 * their row sums, the min/max partials and the activation parameters.  A workspace larger than this is welcome: what
 * lies beyond serves the split of the reduction (add mq_split_workspace_bytes(M, N, K)). */
size_t mq_qlinear_a8_workspace_bytes(int M, int K);

/* W8A8 linear (paper Sec. 4.3 / App. C item 4: integer GEMM behind an FP16->INT8 conversion):
 *     qx  = clamp(rne(x/s_x) + z_x, 0, 255)               per-tensor, unsigned 8 bit
 *     ACC = sum_k (qx[m,k] - z_x) * (qw[n,k] - z_w[n])    int32
 *     Y   = fp16( ACC * s_x * s_w[n] + bias[n] )
 *   x        [M,K] fp16, row stride ldx (ldx % 8 == 0, 16-byte aligned).
 *   packed   8-bit weights, MQ_LAYOUT_KERNEL; w_signed != 0: two's complement codes (symmetric scheme),
 *            else unsigned codes with zero points w_zp.
 *   w_colsum [N] from mq_pack_weights.
 *   act_scale/act_zp  both NULL: dynamic — min/max of X is reduced on the device; otherwise static
 *            (calibrated, Sec. 4.1) parameters are read from these device scalars.
 *   acc_debug         nullable [M,N] int32 out: ACC, for bit-exact checks.
 *   residual, ldr     nullable fp16 [M,N], as for mq_qlinear_w_only: Y = fp16( ACC * s_x * s_w[n] + bias[n] + residual ).
 *   act_scale_out/act_zp_out  nullable device scalars out: the parameters that were used.
 *   K % 64 == 0 and K <= 33024; N % 8 == 0.
 * Errors: MQ_ERR_BAD_ARG when exactly one of act_scale/act_zp is NULL; MQ_ERR_OVERFLOW_RISK;
 *         MQ_ERR_WORKSPACE_TOO_SMALL; and the common ones. */
int mq_qlinear_w8a8(const void* x, int M, int K, int ldx, const void* packed, int N, int layout, int w_signed,
                    const float* w_scale, const int32_t* w_zp, const int32_t* w_colsum, const float* act_scale,
                    const int32_t* act_zp, const void* bias, void* y, int ldy, int32_t* acc_debug,
                    const void* residual, int ldr, float* act_scale_out, int32_t* act_zp_out, void* ws,
                    size_t ws_bytes, void* stream);

/* W4A8 linear: as above with asymmetric unsigned 4-bit weight codes (the INT4 operator the paper leaves as
 * future work, App. C item 4); the codes are widened to int8 in registers ahead of the int8 MFMA. */
int mq_qlinear_w4a8(const void* x, int M, int K, int ldx, const void* packed, int N, int layout,
                    const float* w_scale, const int32_t* w_zp, const int32_t* w_colsum, const float* act_scale,
                    const int32_t* act_zp, const void* bias, void* y, int ldy, int32_t* acc_debug,
                    const void* residual, int ldr, float* act_scale_out, int32_t* act_zp_out, void* ws,
                    size_t ws_bytes, void* stream);

/* W2A8 linear: as above with asymmetric unsigned 2-bit weight codes.  The paper's W4A8 configurations are mixed:
 * their weight bit-widths come from {2,4,8} (Sec. 3.3) under 8-bit activations, so 2-bit layers meet the integer
 * GEMM too; the codes are widened to int8 in registers like the 4-bit ones. */
int mq_qlinear_w2a8(const void* x, int M, int K, int ldx, const void* packed, int N, int layout,
                    const float* w_scale, const int32_t* w_zp, const int32_t* w_colsum, const float* act_scale,
                    const int32_t* act_zp, const void* bias, void* y, int ldy, int32_t* acc_debug,
                    const void* residual, int ldr, float* act_scale_out, int32_t* act_zp_out, void* ws,
                    size_t ws_bytes, void* stream);

/* For callers that cannot allocate device memory or hand over a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid allocation): mq_qlinear_w8a8 / _w4a8 / _w2a8 (by w_bits = 8, 4, 2; w_signed
 * only with 8) with the workspace in a device array that is part of the library, mq_builtin_workspace_bytes() =
 * 48 MiB per GPU the library runs on, held until the process ends.  The call allocates nothing and frees nothing.
 * All other arguments, results and errors are those of the entry points above, bit for bit.
 *   Limit: mq_qlinear_a8_workspace_bytes(M, K) <= mq_builtin_workspace_bytes(), else MQ_ERR_WORKSPACE_TOO_SMALL
 *   (M * K up to about 50 M activations: every linear of the configured workloads fits); what the activation
 *   workspace leaves of the array serves the split of the reduction.
 *   Every call on a GPU uses that GPU's one array, which keeps the previous call's contents (nothing in it has to
 *   start at zero: every byte that is read is written first, the split counters by a clearing kernel).  Calls that
 *   may overlap on one GPU - different streams, or a captured graph replayed while another call runs - race on it:
 *   keep them on one stream. */
size_t mq_builtin_workspace_bytes(void);
int mq_qlinear_a8_builtin_ws(const void* x, int M, int K, int ldx, const void* packed, int N, int w_bits, int layout,
                             int w_signed, const float* w_scale, const int32_t* w_zp, const int32_t* w_colsum,
                             const float* act_scale, const int32_t* act_zp, const void* bias, void* y, int ldy,
                             int32_t* acc_debug, const void* residual, int ldr, float* act_scale_out,
                             int32_t* act_zp_out, void* stream);

/* ------------------------------------------------------------------------------------------------
 * Feed-forward pair with the activation kept in 8 bits between its two linears (an extension: paper Sec. 4.3
 * names the separate FP16->INT8 conversion layers as the overhead of the W8A8 path; this removes the one between
 * the gated projection and the output linear of a transformer block's feed-forward, and the 8C-wide fp16
 * tensor between them never reaches memory).
 *
 * The int8 activation layout ("A8 layout") that links the two calls: row stride mq_a8_row_bytes(K) = K rounded
 * up to 128 (or more, a multiple of 128), byte value a' = code - 128 (two's complement), inside every group of 8
 * consecutive k the bytes are stored in the order 0,4,1,5,2,6,3,7, and the bytes from K to the stride are zero.
 * ---------------------------------------------------------------------------------------------- */
size_t mq_a8_row_bytes(int K);

/* Gated projection (GEGLU) with 8-bit input and output.  The weight matrix has 2H rows: rows [0,H) produce the
 * value, rows [H,2H) the gate.
 *     lin[m,n]  = fma( (float)ACC[m,n], s_x * s_w[n], bias[n] )            ACC as in mq_qlinear_w8a8
 *     h[m,j]    = lin[m,j] * gelu( lin[m,H+j] )                            j in [0,H)
 *     code[m,j] = clamp( rne(h / s_o) + z_o, 0, 255 )                      h / s_o as a multiply by the fp32 1/s_o
 * gelu(g) = 0.5 g (1 + erf(g / sqrt 2)).  ACC is exact; everything after it is evaluated in fp32 (erf as
 * 1 - exp(-x P(x)) with a fitted degree-6 polynomial P and the hardware's 2^t, |error| < 3e-7), so a code equals the one the same formulas
 * give in exact arithmetic except where h / s_o lies within that fp32 error (about 1e-5 of a code step for typical
 * values) of a rounding boundary, where it may be the neighbouring code.
 *   x [M,K] fp16 (as in mq_qlinear_w8a8, dynamic or static activation parameters), packed: w_bits = 2, 4 or 8,
 *   MQ_LAYOUT_KERNEL, 2H rows; w_scale, w_zp, w_colsum, bias [2H].  H % 32 == 0.
 *   out_scale, out_zp: device pointers to the static parameters (s_o, z_o) of the gated product.
 *   a8_out  [M, mq_a8_row_bytes(H)] int8 out, A8 layout, 16-byte aligned.
 *   h16_out nullable [M,H] fp16 out (row stride ldh, ldh % 8 == 0): the gated product itself.
 *   ws: mq_qlinear_a8_workspace_bytes(M, K). */
int mq_qlinear_a8_geglu(const void* x, int M, int K, int ldx, const void* packed, int H, int w_bits, int layout,
                        int w_signed, const float* w_scale, const int32_t* w_zp, const int32_t* w_colsum,
                        const float* act_scale, const int32_t* act_zp, const void* bias, const float* out_scale,
                        const int32_t* out_zp, int8_t* a8_out, void* h16_out, int ldh, float* act_scale_out,
                        int32_t* act_zp_out, void* ws, size_t ws_bytes, void* stream);

/* The same gated projection with DYNAMIC parameters of its 8-bit output: the range of the gated product is only
 * known once all of it exists, so the product is written as fp16 (h16, required, [M,H], row stride ldh) while every
 * workgroup of the projection leaves the minimum and maximum of what it wrote; a second kernel turns h16 into
 * codes exactly as the dynamic activation quantisation of mq_qlinear_w8a8 would (min/max over the fp16 values, the
 * same fp32 formulas), without reading h16 a first time for its range.  The 8C-wide projection output still never
 * reaches memory.  out_scale_out / out_zp_out: device pointers (required) that receive the parameters; they and
 * a8_out are what mq_qlinear_a8_codes takes.  ws: mq_qlinear_a8_geglu_dynamic_workspace_bytes(M, K, H). */
size_t mq_qlinear_a8_geglu_dynamic_workspace_bytes(int M, int K, int H);
int mq_qlinear_a8_geglu_dynamic(const void* x, int M, int K, int ldx, const void* packed, int H, int w_bits,
                                int layout, int w_signed, const float* w_scale, const int32_t* w_zp,
                                const int32_t* w_colsum, const float* act_scale, const int32_t* act_zp,
                                const void* bias, void* h16, int ldh, int8_t* a8_out, float* out_scale_out,
                                int32_t* out_zp_out, float* act_scale_out, int32_t* act_zp_out, void* ws,
                                size_t ws_bytes, void* stream);

/* The gated projection on the weight-only path, W{2,3,4,8}A16, fp16 in and out:
 *     h[m,j] = fp16( lin[m,j] * gelu(lin[m,H+j]) ),  lin = X . dequant(W)^T + bias over the 2H weight rows
 * (fp32 accumulation, the same fp32 gelu as above).  h [M,H] row stride ldh (ldh % 8 == 0).  H % 32 == 0. */
int mq_qlinear_w_only_geglu(const void* x, int M, int K, int ldx, const void* packed, int H, int bits, int layout,
                            const float* w_scale, const int32_t* w_zp, const void* bias, void* h, int ldh,
                            void* stream);

/* The weight-only gated projection with 8-bit output, W{2,3,4,8}A16: for a feed-forward whose projection keeps
 * 16-bit activations while its output linear takes 8-bit ones.  lin and h as above, code[m,j] = clamp(rne(h / s_o) +
 * z_o, 0, 255) from the fp32 product (the accumulation is the fp16 MFMA's, so a code may be the neighbour of the one
 * exact arithmetic gives where h / s_o lies within that arithmetic's error of a rounding boundary).
 * out_scale, out_zp: device pointers to the static parameters; a8_out [M, mq_a8_row_bytes(H)] in the A8 layout;
 * h16_out nullable [M,H] fp16 (row stride ldh). */
int mq_qlinear_w_only_geglu_a8(const void* x, int M, int K, int ldx, const void* packed, int H, int bits, int layout,
                               const float* w_scale, const int32_t* w_zp, const void* bias, const float* out_scale,
                               const int32_t* out_zp, int8_t* a8_out, void* h16_out, int ldh, void* stream);

/* W8A8 / W4A8 / W2A8 linear on activations that arrive as codes in the A8 layout (row stride lda bytes) together with
 * their parameters (device pointers act_scale, act_zp): ACC and Y as in mq_qlinear_w8a8.  The row sums of the
 * codes, which the zero-point correction needs, are taken inside the GEMM; no workspace.  residual: nullable fp16
 * [M,N], row stride ldr, added before the rounding (the block's skip connection after a feed-forward). */
int mq_qlinear_a8_codes(const int8_t* a8, int M, int K, int lda, const float* act_scale, const int32_t* act_zp,
                        const void* packed, int N, int w_bits, int layout, int w_signed, const float* w_scale,
                        const int32_t* w_zp, const int32_t* w_colsum, const void* bias, void* y, int ldy,
                        int32_t* acc_debug, const void* residual, int ldr, void* stream);

/* ------------------------------------------------------------------------------------------------
 * 3x3 convolution, stride 1, zero padding 1 (paper Sec. 4.1 "Quantization Scheme": the convolution layers are
 * quantised like the linear ones, weights per output channel over the whole 3x3xCin filter, activations per tensor).
 * Channels-last tensors: x [B,H,W,Cin], y [B,H,W,N] (contiguous).  The weight matrix handed to mq_quantize_weights /
 * mq_pack_weights is [N, 9*Cin] with k = (r*3 + s)*Cin + c (filter row r, filter column s, input channel c), in
 * MQ_LAYOUT_KERNEL.  No im2col copy is made: the GEMM's activation loads address the taps themselves, and taps
 * outside the image read as zero.  Cin % 64 == 0, N % 8 == 0, B*H*W*Cin*2 < 2^31.
 * stride: 1, or 2 for the UNet's downsampling convolutions: the output is then [B,Ho,Wo,N] with Ho = (H-1)/2 + 1,
 * Wo = (W-1)/2 + 1, output pixel (i,j) centred on input pixel (2i,2j); y, residual and acc_debug have that shape.
 * A 1x1 convolution needs no entry point of its own: on channels-last tensors it is the linear layer over the
 * [B*H*W, Cin] matrix.
 * residual: nullable [B,H,W,N] fp16, contiguous, added before the rounding (may be y itself): the skip connection of
 * a residual block, or the output of the convolution over the other part of a split channel-concatenated input.
 * ---------------------------------------------------------------------------------------------- */

/* Weight-only convolution, W{2,3,4,8}A16:
 *     y = fp16( sum_{r,s,c} x[b,i+r-1,j+s-1,c] * scale[n]*(code - zp[n]) + bias[n] + residual[b,i,j,n] ). */
int mq_conv3x3_w_only(const void* x, int B, int H, int W, int Cin, int stride, const void* packed, int N, int bits,
                      int layout, const float* w_scale, const int32_t* w_zp, const void* bias, void* y,
                      const void* residual, void* stream);

/* Sums of the weight codes per filter tap, [9][N] int32 (tap = r*3 + s): needed by mq_conv3x3_a8 for the output
 * pixels whose filter reaches outside the image.  codes [N, 9*Cin] as handed to mq_pack_weights. */
int mq_conv_tap_sums(const uint8_t* codes, int N, int Cin, int bits, int codes_signed, int32_t* tapsum, void* stream);

size_t mq_conv3x3_a8_workspace_bytes(int B, int H, int W, int Cin);

/* W8A8 / W4A8 / W2A8 convolution: activations quantised per tensor (dynamic min/max over x, or the given static
 * parameters) as in mq_qlinear_w8a8; a padded position holds the value 0, whose code is the zero point:
 *     ACC[m,n] = sum over in-image (r,s), c of (qx - z_x)(qw - z_w[n]),
 *     y = fp16(ACC * s_x * s_w[n] + bias[n] + residual[m,n]).
 * The activation parameters are those of the whole input tensor, whatever the stride.
 * acc_debug nullable [B*Ho*Wo, N] int32. */
int mq_conv3x3_a8(const void* x, int B, int H, int W, int Cin, int stride, const void* packed, int N, int w_bits,
                  int layout, int w_signed, const float* w_scale, const int32_t* w_zp, const int32_t* w_colsum,
                  const int32_t* w_tapsum, const float* act_scale, const int32_t* act_zp, const void* bias, void* y,
                  int32_t* acc_debug, const void* residual, float* act_scale_out, int32_t* act_zp_out, void* ws,
                  size_t ws_bytes, void* stream);

size_t mq_bos_aware_kv_proj_workspace_bytes(int B, int T, int K);

/* BOS-aware cross-attention K/V projection (paper Sec. 3.1).  ctx is the text embedding [B,T,K] fp16,
 * contiguous; token 0 of every prompt is the outlier BOS row.
 *   - tokens 1..T-1: 8-bit-activation linear as above (w_bits 8, 4 or 2); dynamic activation parameters are the
 *     min/max over those tokens only.
 *   - token 0: exactly one of
 *         w_f16   [N,K] unquantised fp16 weights -> Y[b,0,:] = fp16(ctx[b,0,:] . w_f16^T + bias), fp32 accumulate
 *         bos_out [N]   pre-computed fp16 output, copied to Y[b,0,:] for every prompt.
 *   - naive_all_rows != 0: comparator that quantises all B*T rows, BOS included (w_f16/bos_out ignored).
 *   y [B,T,N] fp16 contiguous. */
int mq_bos_aware_kv_proj(const void* ctx, int B, int T, int K, const void* packed, int N, int w_bits, int layout,
                         int w_signed, const float* w_scale, const int32_t* w_zp, const int32_t* w_colsum,
                         const void* w_f16, const void* bos_out, const float* act_scale, const int32_t* act_zp,
                         const void* bias, void* y, int naive_all_rows, float* act_scale_out, int32_t* act_zp_out,
                         void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------------
 * Bit-width allocation (host only: every pointer in this section is a HOST pointer, no GPU is touched, nothing is
 * enqueued).  It produces the per-layer `bits` that the entry points above take.
 * ---------------------------------------------------------------------------------------------- */

/* The integer programme of paper Sec. 3.3, Eq. 2, solved exactly: choose one candidate per layer,
 *     maximise  sum_i sens[i][c_i]   subject to  sum_i cost[i][c_i] <= budget.
 *   sens_host [n_layers][n_choices] sensitivity scores (higher is better, any finite values),
 *   cost_host [n_layers][n_choices] non-negative resource costs (for an average-bit-width budget: elements * bits).
 *   choice_host [n_layers] out: index of the chosen candidate per layer.  objective_host, cost_used_host: nullable
 *   scalars out: the objective (scores added in layer order, double precision) and the cost of the choice.
 * Where several assignments reach the maximum, one of them is returned.
 * Errors: MQ_ERR_INFEASIBLE when even the cheapest assignment exceeds the budget; MQ_ERR_TOO_LARGE. */
int mq_alloc_solve(int n_layers, int n_choices, const double* sens_host, const int64_t* cost_host, int64_t budget,
                   int32_t* choice_host, double* objective_host, int64_t* cost_used_host);

/* SplitBudget of paper App. A, Alg. 1.  The ratio k is read as the ratio of the two groups' average bit-widths:
 *     avg_quality = budget_all / (k * params_content + params_quality),  budget_content = floor(k * avg_quality * params_content),
 *     budget_quality = budget_all - budget_content. */
int mq_alloc_split_budget(int64_t budget_all, int64_t params_content, int64_t params_quality, double k,
                          int64_t* budget_content_host, int64_t* budget_quality_host);

/* The two loops of paper App. A, Alg. 1 up to (not including) image generation and scoring, which need the model:
 * n_budgets budgets spaced linearly in [B_all - dB, B_all] (B_all = floor(avg_bits_target * P), dB =
 * floor(delta_avg_bits * P), P = all elements of both groups) times n_ratios ratios spaced linearly in [k_lo, k_hi];
 * for each pair the budget is split, Eq. 2 is solved per group with cost = elements * bits, and the two
 * configurations are returned for the caller to score.  Candidate e = budget index * n_ratios + ratio index.
 *   sens_*_host [n][n_choices], params_*_host [n] element counts, bits_host [n_choices].
 *   budgets_host [E][3] out: budget, content budget, quality budget.  k_host [E] out.  feasible_host [E] out: 1 when
 *   both groups fit.  objectives_host [E][2] out (content, quality).  choice_content_host [E][n_content],
 *   choice_quality_host [E][n_quality] out: candidate indices, -1 where infeasible.  E = n_budgets * n_ratios. */
int mq_alloc_search(int n_content, const double* sens_content_host, const int64_t* params_content_host, int n_quality,
                    const double* sens_quality_host, const int64_t* params_quality_host, int n_choices,
                    const int32_t* bits_host, double avg_bits_target, double delta_avg_bits, int n_budgets, double k_lo,
                    double k_hi, int n_ratios, int64_t* budgets_host, double* k_host, int32_t* feasible_host,
                    double* objectives_host, int32_t* choice_content_host, int32_t* choice_quality_host);

#ifdef __cplusplus
}
#endif
#endif /* MIXDQ_H */
