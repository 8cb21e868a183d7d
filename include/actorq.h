/*
 * actorq.h -- C ABI of the MI355X (gfx950) ActorQ hot path: 8-bit actor policy inference.
 *
 * Paper: "QuaRL / ActorQ: Quantization for Fast and Environmentally Sustainable
 * Reinforcement Learning" (arXiv 1910.01055).  Sec. 3.1 puts a quantizer block between
 * the fp32 learner and the actors; Sec. 3.2 defines the quantizer (uniform affine
 * post-training quantization, per channel for convolutions, weights and activations at
 * the same precision); the actors then run the policy in 8 bits.  The three calls named
 * aq_quantize_params, aq_policy_forward_int8 and aq_policy_forward_fp32 are those two
 * blocks plus the full-precision actor the paper compares against.
 *
 * Conventions
 *  - Every pointer named d_* is a DEVICE pointer owned by the caller (for instance a torch
 *    tensor's data_ptr()), contiguous, at least 16-byte aligned.  The library never frees
 *    or keeps such a pointer beyond the stream work it enqueues.  h_* are host pointers.
 *  - The handle aq_policy and everything inside it are owned by the library.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Unless a call
 *    says it synchronizes, it only enqueues work on `stream` and returns.
 *  - Argument errors are returned at once as aq_status; nothing throws or aborts.  Errors
 *    that only the device can see (non-finite weights, a requantization multiplier outside
 *    the representable shift range) set a flag read by aq_policy_status().
 *  - A handle may be used from one thread at a time; distinct handles are independent.
 *  - There is no CPU fallback: without a GPU every compute call returns AQ_EHIP.
 *
 * Layouts
 *  - FC weights: fp32 [N][K] row-major (N = output features).
 *  - Conv weights: fp32 [Cout][kh][kw][Cin]; activations NHWC; VALID padding; a conv
 *    layer's output [oh][ow][Cout] is flattened in (h, w, c) order before an FC layer.
 *  - Observations: fp32 [B][K0] (AQ_IN_F32) or uint8 [B][H][W][C] (AQ_IN_U8, consumed as
 *    raw codes with scale 1 and zero-point 0).
 *  - Actions: fp32 [B][A] for AQ_HEAD_TANH / AQ_HEAD_LINEAR, int32 [B] for AQ_HEAD_ARGMAX
 *    (lowest index wins ties).
 */
#ifndef ACTORQ_H
#define ACTORQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct aq_policy aq_policy;

typedef enum {
    AQ_OK = 0,
    AQ_EINVAL = 1,     /* bad argument (NULL, negative size, unknown enum) */
    AQ_ESHAPE = 2,     /* layer shapes do not chain, or a shape the kernels do not support */
    AQ_ENONFINITE = 3, /* NaN/Inf among the weights (reported by aq_policy_status) */
    AQ_ENOTQUANT = 4,  /* aq_policy_forward_int8 before aq_quantize_params */
    AQ_EHIP = 5,       /* a HIP runtime call or kernel launch failed */
    AQ_ENOMEM = 6,
    AQ_ERANGE = 7,     /* a requantization multiplier needs a shift outside [1, 62] */
    AQ_ETOOBIG = 8     /* the call would need more scratch memory than it may use without allocating: a batch
                          beyond the static buffer of aq_policy_forward_int8_static, or an internal buffer that
                          would have to grow while `stream` is being captured into a graph */
} aq_status;

typedef enum { AQ_FC = 0, AQ_CONV2D = 1 } aq_kind;
typedef enum { AQ_ACT_NONE = 0, AQ_ACT_RELU = 1, AQ_ACT_LN_TANH = 2 } aq_act;
typedef enum { AQ_HEAD_TANH = 0, AQ_HEAD_ARGMAX = 1, AQ_HEAD_LINEAR = 2 } aq_head;
/* Sec. 3.2: per-tensor asymmetric unsigned codes (scale + zero-point from min(W,0), max(W,0)),
 * or the per-(output-)channel form with a symmetric range, codes in [-127, 127]. */
typedef enum { AQ_W_TENSOR_ASYM_U8 = 0, AQ_W_CHANNEL_SYM_S8 = 1 } aq_wscheme;
typedef enum { AQ_IN_F32 = 0, AQ_IN_U8 = 1 } aq_intype;

/* One layer.  FC: in_c = K, out_c = N, in_h = in_w = kh = kw = stride = 1.
 * `act` is applied to the layer's output; it is ignored on the last layer (the head follows). */
typedef struct {
    int32_t kind;
    int32_t in_h, in_w, in_c;
    int32_t out_c;
    int32_t kh, kw, stride;
    int32_t act;
} aq_layer;

typedef struct {
    int32_t n_layers;       /* 1 .. AQ_MAX_LAYERS */
    const aq_layer* layers; /* host array, copied by aq_policy_create */
    int32_t head;           /* aq_head */
    int32_t wscheme;        /* aq_wscheme */
    int32_t in_type;        /* aq_intype */
    int32_t qdenom;         /* denominator of delta in Sec. 3.2: 255 (= 2^8 - 1, default) or 256 (= 2^8, literal) */
    float ln_eps;           /* LayerNorm epsilon (biased variance, eps inside the square root) */
    int32_t wbits;          /* weight precision n of Sec. 3.2's Q_n: 2..8, 0 = 8.  Below 8 the weight codes use
                               [0, 2^n - 1] (per tensor) or [-(2^(n-1) - 1), 2^(n-1) - 1] (per channel) and still
                               travel in 8-bit containers on the int8 matrix cores; delta's denominator is 2^n - 1,
                               or 2^n when qdenom = 256.  Activations stay at 8 bits. */
} aq_net;

#define AQ_MAX_LAYERS 8

/* Range of one activation tensor (extended to contain 0 by the quantizer, as min(.,0)/max(.,0)
 * do for weights).  A policy with L layers has L ranges: the network input, then the output of
 * every hidden layer after its activation. */
typedef struct {
    float lo, hi;
} aq_range;

/* Optional intermediate outputs of aq_policy_forward_int8, for checking against a reference.
 * Each member is a host array of n_layers device pointers (or NULL), each entry NULL or a
 * caller-owned device buffer:
 *   acc[l]  int32 [rows_l][N_l]  zero-point-corrected accumulator incl. bias, rows_l = B * oh * ow
 *   act[l]  uint8 [rows_l][N_l]  unsigned activation codes leaving hidden layer l
 *   ln_t[l] fp32  [rows_l][N_l]  LayerNorm+tanh value before it is re-quantized (AQ_ACT_LN_TANH layers)
 * a0: uint8 [B][K0] quantized observation; y: fp32 [B][A] dequantized last-layer output before the head. */
typedef struct {
    int32_t* const* acc;
    uint8_t* const* act;
    float* const* ln_t;
    uint8_t* a0;
    float* y;
} aq_taps;

/* Creates a policy handle for `net` on the current HIP device.  Validates that the layers chain
 * (AQ_ESHAPE otherwise) and that every layer is within the size limits of the int32 accumulation:
 * K = kh * kw * in_c <= 65536, out_c <= 2^20, in_h and in_w <= 16384 (AQ_ESHAPE beyond them).
 * Allocates the per-layer device buffers (packed 8-bit weights, per-channel constants). */
aq_status aq_policy_create(const aq_net* net, aq_policy** out);
aq_status aq_policy_destroy(aq_policy* p);

/* Pre-allocates the internal activation buffers for batches up to max_batch, so that later
 * forwards with batch <= max_batch allocate nothing.  Forwards grow the buffers themselves when needed
 * (such a call waits for the device, frees and allocates; while `stream` is being captured into a graph
 * it returns AQ_ETOOBIG instead, so reserve before capturing). */
aq_status aq_policy_reserve(aq_policy* p, int64_t max_batch);

/* Chooses the 8-bit forward's launch plan: 0 = automatic (whole-network fused kernel when the
 * network is an MLP that fits it, else one launch per layer, with the leading convolutions of a
 * frame policy in a single launch where their shapes allow it), 1 = fused only (AQ_ESHAPE from the
 * forward if it does not fit), 2 = one launch per layer (convolutions as in 0), 3 = one launch per
 * layer for every layer, 4 = plan 2 with sub-byte weight streaming where the policy allows it (see
 * aq_policy_subbyte_layers; choosing it the first time allocates the nibble copies of the weights,
 * AQ_ENOMEM if that fails, and the first forward pass after every quantize or import rewrites them with
 * one small launch per layer).  All plans compute identical integers.  Other values: AQ_EINVAL. */
aq_status aq_policy_set_path(aq_policy* p, int32_t path);

/* *n_layers = how many leading convolution layers the 8-bit forward of this handle runs as a single
 * launch under the current launch plan (0: none; it takes 8-bit frames, per-channel symmetric weights,
 * kh * kw * in_c and kw * in_c multiples of 32, stride * in_c and in_w * in_c multiples of 16), given a
 * 16-byte aligned observation buffer.  No GPU work. */
aq_status aq_policy_conv_stack_layers(const aq_policy* p, int32_t* n_layers);
/* The same for the half-precision forward (its rules: 8-bit frames, kw * in_c a multiple of 16,
 * stride * in_c and in_w * in_c multiples of 8, out_c a multiple of 4, two to four convolutions). */
aq_status aq_policy_fp16_conv_stack_layers(const aq_policy* p, int32_t* n_layers);

/* Which compiled variant of the whole-network kernels a forward of `batch` >= 1 rows launches under the
 * current launch plan: *rows = batch rows per workgroup (16, 32, 64 or 128), *tiles = 32-feature tiles per
 * wavefront and pass (1 or 2); both 0 when the forward runs one launch per layer instead (a network the
 * kernels do not take, or launch plan 2 / 3).  *kind is the kernel: 0 = the general kernel; 1 = the
 * software-pipelined kernel for wide layers (64 rows, two tiles; per-channel weights, fp32 observations, hidden
 * widths multiples of 64 without LayerNorm, every K a multiple of 128, at most 64 outputs); 2 = the kernel for
 * small networks (16, 32 or 64 rows by batch size; either weight scheme, fp32 or 8-bit observations, at most four
 * fully connected layers, first-layer inputs and hidden widths up to 256, at most 64 outputs); 3 = the same kernel
 * in the form it takes while every workgroup has a CU to itself (batch <= 4096, 16 rows: a layer's operands are
 * requested behind the epilogue two layers earlier).  Kinds 1 to 3 need a
 * 16-byte aligned observation buffer; an unaligned one takes the general kernel with the rows and tiles its own
 * plan gives (not reported here).  With the weight scheme and whether intermediate outputs are requested this
 * names the variant, so that a test can show that every one it times is also checked.  No GPU work. */
aq_status aq_policy_fused_plan(const aq_policy* p, int64_t batch, int32_t* rows, int32_t* tiles, int32_t* kind);

/* How many layers of a forward pass at this batch size read their weights sub-byte.  A policy whose weight
 * precision is n <= 4 bits (aq_net.wbits; the precision sweep of the paper's appendix on quantization-aware
 * training) with per-channel symmetric weights keeps, once launch plan 4 is chosen (aq_policy_set_path), its fully
 * connected layers' codes a second time as nibbles (two codes per byte); under that plan the few-row layer kernel -- one launch per layer
 * at batch sizes below 8192, the paper's own regime of actors that run one observation at a time -- streams
 * those, half the weight bytes, and expands them in registers; the integer results are those of the 8-bit
 * containers, bit for bit.  It is a plan to choose, not the default: at the sizes measured the layer's time is
 * requests and latency, not bytes, and the expansion costs more than the bytes save.  Every other plan, and under
 * plan 4 the convolutions and batches from 8192 on, read the 8-bit containers: the answer is then 0.
 * batch >= 1; NULL arguments: AQ_EINVAL. */
aq_status aq_policy_subbyte_layers(const aq_policy* p, int64_t batch, int32_t* n_layers);

/* Synchronizes `stream` and returns the sticky device-side error of the last
 * aq_quantize_params or aq_policy_import_blob (AQ_OK, AQ_ENONFINITE, AQ_ERANGE, or AQ_EINVAL for a
 * blob whose header does not match). */
aq_status aq_policy_status(aq_policy* p, void* stream);

/* The quantized policy as one contiguous blob, for the learner-to-actor broadcast of Sec. 3.1 (the
 * step whose cost Sec. 5.3 breaks out; the paper notes that loading the quantized parameters into the
 * actor's model re-packs the weights).  The blob holds the 8-bit weights already in the forward
 * kernels' operand order, every per-channel constant and the activation quantization parameters,
 * behind a 64-byte header (magic, format version, a hash of the network description, payload size):
 * importing it is two device-to-device copies and no arithmetic.  A blob is valid only for a handle
 * created from the same aq_net on the same library version.
 *   aq_policy_blob_size: *bytes = size of the blob for this handle's network (no GPU work).
 *   aq_policy_export_blob: writes the blob to d_blob (caller-owned device memory, 16-byte aligned,
 *     at least `bytes` long; AQ_EINVAL if shorter than the blob, AQ_ENOTQUANT before any
 *     aq_quantize_params / import).  Enqueues on `stream`.
 *   aq_policy_import_blob: installs a blob (same size rules).  Enqueues on `stream`; a header that does
 *     not match this handle's network sets a device-side flag that aq_policy_status() reports as
 *     AQ_EINVAL (the payload is then unspecified, as after non-finite weights).  The handle counts as
 *     quantized afterwards. */
aq_status aq_policy_blob_size(const aq_policy* p, uint64_t* bytes);
aq_status aq_policy_export_blob(const aq_policy* p, void* d_blob, uint64_t bytes, void* stream);
aq_status aq_policy_import_blob(aq_policy* p, const void* d_blob, uint64_t bytes, void* stream);

/* The same hand-off with the weight codes stored sub-byte: a policy whose weight precision is n < 8 bits
 * (aq_net.wbits) travels as n-bit fields, 8 codes per n bytes, and is expanded to the 8-bit operand layout
 * on import (constants and activation parameters as in the plain blob).  With n = 8 the packed blob is the
 * plain one byte for byte, apart from its magic number.  Size, export, import and their errors as above;
 * a packed blob only loads into a handle of the same network description and the same wbits. */
aq_status aq_policy_packed_blob_size(const aq_policy* p, uint64_t* bytes);
aq_status aq_policy_export_packed_blob(const aq_policy* p, void* d_blob, uint64_t bytes, void* stream);
aq_status aq_policy_import_packed_blob(aq_policy* p, const void* d_blob, uint64_t bytes, void* stream);

/* Exploration on the actor (Sec. 4.1: a Gaussian noise layer on the policy output whose sigma
 * depends on the actor; for the discrete-control policies, epsilon-greedy), applied in place to the
 * actions of a preceding forward on the same stream.
 *   tanh / linear heads: actions[b][n] += d_sigma[b] * z, z ~ N(0, 1); d_sigma: device fp32 [batch]
 *     (the paper draws each actor's sigma from U(0, 0.2)); no clipping.
 *   argmax head: with probability epsilon actions[b] becomes a uniform action index (d_sigma unused).
 * Random numbers come from the counter-based generator Philox4x32-10 (Salmon et al., SC'11) with
 * key = seed and counter = (row, block, step): the same (seed, step, row) always gives the same
 * draw, different steps give independent draws, no generator state is kept.  z comes from
 * Box-Muller on 24-bit uniforms: block = n / 4, words (0, 1) -> features 4 block + (0, 1) as
 * (cos, sin), words (2, 3) -> features 4 block + (2, 3); epsilon-greedy uses block 0xFFFFFFFF,
 * word 0 for the test u < epsilon (u = (word >> 8) / 2^24) and word 1 for the index
 * floor(word * A / 2^32).  batch must be below 2^32.  AQ_EINVAL for a NULL d_sigma with a
 * continuous head or an epsilon outside [0, 1]. */
typedef struct {
    uint64_t seed;
    uint64_t step;
    const float* d_sigma;
    float epsilon;
} aq_explore;
aq_status aq_policy_explore(const aq_policy* p, void* d_actions, int64_t batch, const aq_explore* ex, void* stream);

/* One actor step: aq_policy_forward_int8 followed by aq_policy_explore with the same arguments (ex may
 * be NULL: no exploration).  The Gaussian noise is added inside the forward kernel where that kernel
 * writes the actions itself (fused plan, tanh / linear head, at most 64 actions); otherwise the
 * exploration runs as a second launch on the same stream.  Same results either way. */
aq_status aq_policy_step_int8(aq_policy* p, const void* d_obs, int64_t batch, void* d_actions,
                              const aq_explore* ex, const aq_taps* taps_or_null, void* stream);

/* Sec. 3.2 applied to one tensor, for the learner-to-actor broadcast: quantizes fp32
 * d_w[rows][cols] to 8-bit codes in canonical row-major order.
 *   AQ_W_TENSOR_ASYM_U8: one (scale, zero-point) for the whole tensor -> d_scale[1], d_zp[1], uint8 codes.
 *   AQ_W_CHANNEL_SYM_S8: one scale per row -> d_scale[rows], d_zp[rows] = 0, int8 codes.
 * d_workspace: at least 16 KiB of device memory the call may overwrite (partial ranges of the
 * workgroups).  Word 2 of it (int32) is a sticky flag: the call sets it to 1 when it meets a
 * non-finite input and never clears it, so zero it once before the first call.
 * qdenom selects the precision n = 2..8 and the reading of delta's denominator: 2^n - 1 (255 for 8 bits, the
 * default reading) or 2^n (256: the literal formula); codes lie in [0, 2^n - 1] resp. [-(2^(n-1) - 1),
 * 2^(n-1) - 1] and are stored one per byte.  Any other value: AQ_EINVAL.
 * cols must be a multiple of 4 and d_w 16-byte aligned. */
aq_status aq_quantize_tensor(const float* d_w, int64_t rows, int64_t cols, int32_t wscheme, int32_t qdenom,
                             void* d_codes, float* d_scale, int32_t* d_zp, void* d_workspace, void* stream);

/* Measurement aid for aq_quantize_tensor: moves the same bytes (n fp32 values read, n bytes written: the
 * top byte of each value) with no arithmetic and no reduction, so that a benchmark can report what plain
 * streaming reaches at the size it quantizes -- the ceiling of the quantize pass at that size.  n a multiple
 * of 4, d_in 16-byte aligned (AQ_ESHAPE otherwise).  Enqueues on `stream`. */
aq_status aq_stream_reference(const float* d_in, int64_t n, void* d_out, void* stream);

/* Measurement aid for aq_policy_forward_int8 on wide layers at large batch: the inner loop of the whole-network
 * kernel that serves them and nothing else -- per workgroup (8 wavefronts, one workgroup per CU) 64 activation
 * rows of K = 1024 held in LDS, per wavefront and k-step four 32x32x32 int8 MFMAs on 2 x 1 KiB of weight operands
 * read from device memory in operand order (stream_weights != 0) or kept in registers (stream_weights = 0: the first
 * four k-steps' operands again and again), no
 * epilogue and no barrier -- so that a benchmark can report the int8 rate the matrix cores sustain in that loop
 * shape on given operands: the ceiling of the kernel's passes.  (The rate depends on the operand values: the
 * clock under matrix load drops with the bits that toggle.)
 * d_weights: 1 MiB of device memory, 16 feature tiles x 64 k-steps x 1 KiB (lane l of a tile's k-step holds 16
 * bytes: feature l mod 32, k = 16 * (l / 32) .. + 15), walked round and round; wavefront w uses tiles 2w, 2w + 1.
 * d_acts: 64 x 1024 int8, row-major, walked 32 k-steps round and round.  Both 16-byte aligned (AQ_ESHAPE).
 * ksteps: k-steps per wavefront, a positive multiple of 4; workgroups: 1 .. 65536 (AQ_EINVAL otherwise).
 * d_acc: 32768 int32 the call overwrites with workgroup 0's accumulators, index
 * (((w * 2 + feature tile) * 2 + row tile) * 16 + r) * 64 + lane, where register r of lane l is feature
 * 8 * (r / 4) + 4 * (l / 32) + r % 4 and row l mod 32 of the 32 x 32 tile.  Work per call: workgroups * ksteps *
 * 32 MFMAs of 65536 op.  NULL pointers: AQ_EINVAL.  Enqueues on `stream`. */
aq_status aq_mfma_loop_reference(const void* d_weights, const void* d_acts, int32_t ksteps, int32_t stream_weights,
                                 int32_t workgroups, int32_t* d_acc, void* stream);

/* The quantizer block (Sec. 3.1 / 3.2): turns the learner's fp32 parameters into the 8-bit
 * policy held by `p`: weight codes in the kernels' packed layout, per-channel scales, the
 * activation (scale, zero-point) of every range, integer biases, requantization multipliers
 * and shifts.  h_d_w[l], h_d_b[l]: device pointers to layer l's weights and bias (bias may be
 * NULL = zeros).  h_d_gamma[l], h_d_beta[l]: LayerNorm gain/offset for AQ_ACT_LN_TANH layers
 * (NULL entries = 1 and 0; the arrays themselves may be NULL).  h_ranges: n_layers activation
 * ranges (entry 0 is ignored for AQ_IN_U8).  h_d_w = NULL (then h_d_b, h_d_gamma, h_d_beta must be NULL as
 * well) quantizes the parameters kept by aq_policy_set_params_fp32 (AQ_ENOTQUANT if there are none).
 * Asynchronous; LayerNorm parameters are copied. */
aq_status aq_quantize_params(aq_policy* p, const float* const* h_d_w, const float* const* h_d_b,
                             const float* const* h_d_gamma, const float* const* h_d_beta,
                             const aq_range* h_ranges, void* stream);

/* Copies layer l's quantized parameters, in canonical order, into caller buffers (any may be NULL):
 * d_codes: uint8/int8 weight codes in the fp32 weights' layout; d_w_scale[N] fp32; d_w_zp[N] int32;
 * d_bias_q[N] int32; d_mult[N] int32 and d_rshift[N] int32 (0 where the layer is not requantized);
 * d_m[N] fp32 = input scale * weight scale. */
aq_status aq_policy_export_layer(const aq_policy* p, int32_t layer, void* d_codes, float* d_w_scale,
                                 int32_t* d_w_zp, int32_t* d_bias_q, int32_t* d_mult, int32_t* d_rshift,
                                 float* d_m, void* stream);
/* Copies the n_layers activation (scale, zero-point) pairs. */
aq_status aq_policy_export_act_qparams(const aq_policy* p, float* d_scale, int32_t* d_zp, void* stream);

/* Actor inference on the 8-bit policy (Sec. 3.1): d_obs -> observation quantize -> for every
 * layer int8 x int8 -> int32 accumulation, then requantize (+ReLU) / LayerNorm+tanh+requantize, or
 * on the last layer dequantize and apply the head -> d_actions.  batch >= 0 (0 is a no-op).
 * taps may be NULL.  Asynchronous once the internal buffers cover `batch`. */
aq_status aq_policy_forward_int8(aq_policy* p, const void* d_obs, int64_t batch, void* d_actions,
                                 const aq_taps* taps, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid it): aq_policy_forward_int8 without intermediate outputs, guaranteed to call no
 * hipMalloc / hipFree or any other allocating routine and never to wait for the device.  The scratch of the
 * one-launch-per-layer plan (two 8-bit activation maps, the fp32 rows in front of a LayerNorm row kernel,
 * the logits of an argmax head) lives in a buffer of AQ_STATIC_SCRATCH_BYTES that is part of the library's
 * device image: every GPU the library runs on holds it until the process ends.  A batch that needs more
 * than that -- 2 * (batch * widest hidden map + 64 bytes) + 4 * batch * (LayerNorm width + argmax logits),
 * each piece rounded up to 256 bytes; e.g. batch <= 650 for an 84 x 84 x 4 frame policy whose first
 * convolution yields 20 x 20 x 32 -- is refused with AQ_ETOOBIG and nothing is launched.  Networks that run
 * as the single whole-network kernel (see aq_policy_fused_plan) keep everything on chip, use none of the
 * buffer and take any batch.  Same arguments, results and other errors as aq_policy_forward_int8.
 * All calls on one GPU share that GPU's buffer, whatever the handle or stream: calls that overlap in time on
 * one GPU race; serialize them (one stream, or events).  Nothing in the buffer has to start at zero and the
 * call reads no byte of it that it has not written itself. */
#define AQ_STATIC_SCRATCH_BYTES (16u << 20)
aq_status aq_policy_forward_int8_static(aq_policy* p, const void* d_obs, int64_t batch, void* d_actions,
                                        void* stream);

/* ---- The full-precision actor (the paper's fp32 baseline, q = 32) and the min/max calibration of the
 * activation ranges (Sec. 3.1: the learner owns the fp32 policy, the quantizer block hands the actors an
 * 8-bit one; Sec. 3.2: activations are quantized like weights, which needs their ranges).
 *
 * aq_policy_set_params_fp32: copies the learner's fp32 parameters (same arrays and layouts as
 *   aq_quantize_params; NULL biases, gains, offsets = 0, 1, 0) into buffers of the handle, device to device on
 *   `stream`.  The first call allocates them (hipMalloc; AQ_ETOOBIG while `stream` is being captured).
 *   Afterwards the calls below need no parameter arrays, and aq_quantize_params accepts h_d_w = NULL (with
 *   h_d_b, h_d_gamma, h_d_beta NULL too) to quantize this copy.
 *   Why the copy is a call of its own and not part of aq_quantize_params: calibration has to run before the
 *   quantizer (the ranges are its input), and a model pull that only wants the 8-bit policy would otherwise
 *   pay a second 4 bytes per parameter of HBM writes on every pull.
 * aq_policy_forward_fp32: the fp32 actor on the kept parameters, d_obs -> d_actions (fp32 [batch][A], or
 *   int32 [batch] for AQ_HEAD_ARGMAX).  AQ_ENOTQUANT before aq_policy_set_params_fp32.  Asynchronous once the
 *   internal buffers cover `batch` (see aq_policy_reserve).
 * aq_calibrate_fp32: runs the fp32 actor on a calibration batch (batch >= 1) and writes to the HOST array
 *   h_ranges_out[n_layers] the (min, max) of the network input and of every hidden layer's output after its
 *   activation -- the ranges aq_quantize_params takes.  Waits for `stream` (AQ_EINVAL while it is being
 *   captured).  AQ_ENOTQUANT before aq_policy_set_params_fp32.
 * aq_policy_forward_fp32_params: the same actor on parameter arrays passed with the call (nothing kept),
 *   with the calibration as an optional device-side output and no wait: d_ranges_out (may be NULL) receives
 *   2 * n_layers floats, (min, max) per activation tensor as above. */
aq_status aq_policy_set_params_fp32(aq_policy* p, const float* const* h_d_w, const float* const* h_d_b,
                                    const float* const* h_d_gamma, const float* const* h_d_beta, void* stream);
aq_status aq_policy_forward_fp32(aq_policy* p, const void* d_obs, int64_t batch, void* d_actions, void* stream);
aq_status aq_calibrate_fp32(aq_policy* p, const void* d_obs, int64_t batch, aq_range* h_ranges_out, void* stream);
aq_status aq_policy_forward_fp32_params(aq_policy* p, const float* const* h_d_w, const float* const* h_d_b,
                                        const float* const* h_d_gamma, const float* const* h_d_beta,
                                        const void* d_obs, int64_t batch, void* d_actions, float* d_ranges_out,
                                        void* stream);

/* ---- Half-precision actor (Sec. 3.2: trained policies are also quantized "to fp16"; the run-time
 * breakdown of Sec. 5 runs actors at q = 16 next to q = 8 and q = 32).  Every tensor of this policy is an
 * IEEE binary16 value: parameters, the observation and the output of every operator (affine layer,
 * LayerNorm, tanh, action head), each rounded once to nearest-even from a result accumulated in fp32 on
 * the fp16 matrix cores.
 *
 * aq_convert_params_fp16: rounds the learner's fp32 parameters (same arrays and layouts as
 * aq_quantize_params; biases, gains, offsets may be NULL as there) to binary16 and stores the weights in
 * matrix-core operand order inside the policy.  The first call allocates that storage (hipMalloc);
 * later calls overwrite it asynchronously on `stream`.  A parameter that is not finite after rounding
 * (|v| >= 65520) is reported as AQ_ENONFINITE by aq_policy_status.
 *
 * aq_policy_forward_fp16: d_obs (fp32 or uint8 as declared by the policy) -> d_actions (fp32 [batch][A]
 * holding binary16 values, or int32 [batch] for AQ_HEAD_ARGMAX; ties go to the lowest index).
 * taps_out (may be NULL): n_layers device pointers (each may be NULL) that receive layer l's binary16
 * output after its activation, [batch * oh * ow][out_c].  AQ_ENOTQUANT before the first
 * aq_convert_params_fp16.  Grows internal activation buffers on demand like aq_policy_forward_int8.
 * A frame policy's leading convolutions run as one launch where their shapes allow it (see
 * aq_policy_fp16_conv_stack_layers; launch plan 3 and a tap on any but the last of them select one launch
 * per layer); both forms compute identical values. */
aq_status aq_convert_params_fp16(aq_policy* p, const float* const* h_d_w, const float* const* h_d_b,
                                 const float* const* h_d_gamma, const float* const* h_d_beta, void* stream);
aq_status aq_policy_forward_fp16(aq_policy* p, const void* d_obs, int64_t batch, void* d_actions,
                                 void* const* taps_out, void* stream);

const char* aq_status_string(aq_status s);

#ifdef __cplusplus
}
#endif
#endif /* ACTORQ_H */
