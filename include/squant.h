/* SQuant weight-quantization solver for AMD MI355X (gfx950) -- C ABI.
 *
 * Implements the progressive CASE-flipping solver of "SQuant: On-the-Fly Data-Free
 * Quantization via Diagonal Hessian Approximation" (ICLR 2022), Section 3.3-3.4:
 * Algorithm 1 (progressive SQuant), Algorithm 2 (SQuantFlip) and Algorithm 3
 * (perturbation update, Appendix B.3), preceded by the per-output-channel
 * quantization range of Section 4 (symmetric absmax scale) and the
 * scale/clip/round formula of Section 2.2.
 *
 * A weight tensor is W[cout][cin][kh][kw], contiguous, row-major, binary32
 * (Section 2.1: M = cout output channels, N = cin "kernels" per output channel,
 * K = kh*kw elements per kernel; a fully connected layer is kh = kw = 1; for a
 * grouped / depthwise convolution cin is the per-group input channel count).
 *
 * For every output channel m:
 *   scales[m] = max|W[m]| / qmax,  qmax = 2^(bits-1) - 1   (1.0f if the channel is all zero)
 *   x = W / scales[m] (one IEEE division), clamped to [-qmax, qmax]
 *   SQuant-E : code = round-half-even(x), perturbation p = code - x      (Eq. 5)
 *   SQuant-K : per kernel, flip the k = round(|sum p|) same-sign elements with
 *              the largest |p| one step against the sum                 (Eq. 6, Alg. 2)
 *   update   : per kernel, keep one flip candidate                      (Alg. 3)
 *   SQuant-C : per channel, flip the candidate of the k_c = round(|sum p|)
 *              same-sign kernels with the largest candidate |p|         (Eq. 7, Alg. 2)
 * Perturbations are held in Q23 fixed point (steps of 2^-23) and summed as integers, an exact half
 * in round(|sum|) takes the fewer flips, and ties in a top-k go to the lowest
 * index, so the result does not depend on launch geometry and is reproducible
 * bit for bit.
 *
 * Conventions for every entry point
 *   - pointers named d_* are DEVICE pointers (HIP), h_* are HOST pointers;
 *   - the caller owns every buffer; the library allocates no device memory and keeps
 *     no state between calls;
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream); calls
 *     enqueue work and return; outputs are valid once the stream has been synchronised;
 *     the calls only launch kernels (no allocation, no memset, no host synchronisation),
 *     so they may be captured into a HIP graph;
 *   - codes must not alias the weights; inputs must be finite (NaN/Inf: memory
 *     safe, result unspecified);
 *   - arguments are checked on the host before anything is launched and an
 *     integer status is returned (never an exception or abort).
 */
#ifndef SQUANT_H_
#define SQUANT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Which stages run (Section 4.3 ablation names E, E&K, E&K&C, E&C). */
typedef enum {
  SQUANT_MODE_E = 0,   /* rounding only */
  SQUANT_MODE_EK = 1,  /* + kernel-wise flip */
  SQUANT_MODE_EKC = 2, /* + output-channel-wise flip (the full method) */
  SQUANT_MODE_EC = 3   /* channel-wise flip on the rounded weights, no kernel-wise flip */
} squant_mode_t;

typedef enum {
  SQUANT_OK = 0,
  SQUANT_ERR_NULL = 1,      /* a required pointer is NULL */
  SQUANT_ERR_SHAPE = 2,     /* a dimension is <= 0, or the sizes overflow */
  SQUANT_ERR_BITS = 3,      /* bits outside [2, 8] */
  SQUANT_ERR_MODE = 4,      /* unknown mode */
  SQUANT_ERR_WORKSPACE = 5, /* a workspace size without a workspace pointer */
  SQUANT_ERR_DEVICE = 6,    /* a HIP call failed */
  SQUANT_ERR_UNSUPPORTED = 7, /* not returned by this version: every channel within the shape limits is taken */
  SQUANT_ERR_FORMAT = 8     /* unknown weight or output type, or a buffer misaligned for its element type */
} squant_status_t;

/* What the solver writes for each weight (squant_quantize_ex).  Section 2.2 defines the
 * quantised weight as an integer code times the scale and Algorithm 1 returns that
 * product; a deployment stores the codes, and at 4 bits and below two of them fit a byte.
 *   INT8  one int8 code per weight, the tensor's own layout.
 *   INT4  bits <= 4 only.  Output channel m occupies bytes [m*R, (m+1)*R) with
 *         R = (cin*kh*kw + 1) / 2; byte j of a row holds element 2j in its low nibble and
 *         element 2j+1 in its high nibble, each the code's 4-bit two's complement; the
 *         unused high nibble of an odd row's last byte is 0.
 *   F32   the dequantised weight (float)code * scales[m] (one binary32 multiply), the
 *         tensor's own layout.
 *   BF16  that binary32 product rounded to bfloat16 (round to nearest, ties to even),
 *         2 bytes per weight, the tensor's own layout. */
typedef enum {
  SQUANT_OUT_INT8 = 0,
  SQUANT_OUT_INT4 = 1,
  SQUANT_OUT_F32 = 2,
  SQUANT_OUT_BF16 = 3
} squant_output_t;

/* Element type of the weights handed in.  The solver's arithmetic is binary32 whatever the
 * type: binary16 and bfloat16 weights are widened exactly first. */
typedef enum {
  SQUANT_W_F32 = 0,
  SQUANT_W_F16 = 1,  /* IEEE binary16 */
  SQUANT_W_BF16 = 2  /* bfloat16: the upper 16 bits of a binary32 */
} squant_wtype_t;

/* One weight tensor of a batched call. */
typedef struct {
  const void* w;             /* in : device, cout*cin*kh*kw weights (binary32 unless the call says otherwise) */
  void* codes;               /* out: device; int8 codes in [-qmax, qmax], same count and layout as w,
                                unless the call names another squant_output_t */
  float* scales;             /* out: device, cout binary32 */
  int32_t cout, cin, kh, kw;
} squant_tensor_t;

/* Quantize one tensor (Algorithm 1 over all output channels).
 * d_w [cout*cin*kh*kw] in, d_codes [same count] out, d_scales [cout] out. */
int squant_quantize(const float* d_w, int32_t cout, int32_t cin, int32_t kh, int32_t kw,
                    int32_t bits, squant_mode_t mode, int8_t* d_codes, float* d_scales,
                    void* stream);

/* Device bytes squant_quantize_batched asks for as workspace: 0.  The kernels carry the
 * tensor descriptors in their kernel arguments (up to 256 per launch) and need no memory
 * beyond the inputs and outputs; the size calls and the workspace arguments stay in the
 * signatures so that callers written against them keep working. */
size_t squant_batched_workspace_bytes(int32_t n_tensors);

/* Quantize a set of tensors (the layers of a network are independent, Section 4.2)
 * with a few launches for the whole set instead of one per tensor.
 * h_tensors: HOST array of n_tensors descriptors holding DEVICE pointers; it may be
 * freed or reused as soon as the call returns.  d_workspace / workspace_bytes: may be
 * NULL / 0 (squant_batched_workspace_bytes is 0); a buffer that is passed is neither read
 * nor written; a size without a pointer is SQUANT_ERR_WORKSPACE.  n_tensors = 0 is a no-op. */
int squant_quantize_batched(const squant_tensor_t* h_tensors, int32_t n_tensors, int32_t bits,
                            squant_mode_t mode, void* d_workspace, size_t workspace_bytes,
                            void* stream);

/* Bytes of the output buffer of one tensor in the given format (0 on invalid arguments). */
size_t squant_output_bytes(int32_t cout, int32_t cin, int32_t kh, int32_t kw, squant_output_t output);

/* squant_quantize / squant_quantize_batched with the weight type and the output format
 * chosen by the caller (Algorithm 1; Section 2.2 for the dequantised form).  d_w holds
 * cout*cin*kh*kw elements of `wtype`, aligned to their size; d_out is a buffer of
 * squant_output_bytes() bytes, aligned to 4 bytes for F32 and to 2 for BF16 output; in the batched call the
 * `w` and `codes` members of each descriptor play these two roles and every tensor shares
 * wtype and output.  SQUANT_OUT_INT4 needs bits <= 4 (SQUANT_ERR_BITS otherwise).  With
 * SQUANT_W_F32 and SQUANT_OUT_INT8 the calls are the plain ones above. */
int squant_quantize_ex(const void* d_w, squant_wtype_t wtype, int32_t cout, int32_t cin,
                       int32_t kh, int32_t kw, int32_t bits, squant_mode_t mode,
                       squant_output_t output, void* d_out, float* d_scales, void* stream);
int squant_quantize_batched_ex(const squant_tensor_t* h_tensors, int32_t n_tensors,
                               squant_wtype_t wtype, int32_t bits, squant_mode_t mode,
                               squant_output_t output, void* d_workspace, size_t workspace_bytes,
                               void* stream);

/* Activation ranges without data (Section 4, experimental set-up: a wide, batch-norm based
 * range per activation tensor, clipped per tensor).  The output of a batch-norm layer is
 * taken as N(beta_c, gamma_c^2) per channel c, so channel c spans
 * [beta_c - n_sigma*|gamma_c|, beta_c + n_sigma*|gamma_c|] (each bound: one binary32 multiply,
 * one add / subtract); the tensor's range is [min_c, max_c] of these, with the lower end (and
 * the upper, should it be negative) raised to 0 when a ReLU follows.  The uniform quantizer
 * on that range with 2^bits levels: scale = (hi - lo) / (2^bits - 1) (1.0f for an empty range),
 * zero_point = round-half-even(-lo / scale) clamped to [0, 2^bits - 1]. */
typedef struct {
  const float* gamma;  /* in : device, `channels` binary32 batch-norm weights */
  const float* beta;   /* in : device, `channels` binary32 batch-norm biases */
  int32_t channels;
  int32_t relu;        /* non-zero: a ReLU follows the batch norm */
} squant_bn_t;

typedef struct {
  float lo, hi, scale;
  int32_t zero_point;
} squant_act_range_t;

/* Device bytes squant_activation_ranges asks for as workspace: 0 (the layer descriptors
 * travel in the kernel arguments, 256 per launch). */
size_t squant_activation_workspace_bytes(int32_t n_layers);

/* h_layers: HOST array of n_layers descriptors holding DEVICE pointers (reusable as soon as
 * the call returns); d_ranges: device, n_layers results; d_workspace as for
 * squant_quantize_batched (may be NULL / 0).
 * bits in [2, 16], n_sigma finite and >= 0 (SQUANT_ERR_BITS / SQUANT_ERR_SHAPE otherwise). */
int squant_activation_ranges(const squant_bn_t* h_layers, int32_t n_layers, float n_sigma,
                             int32_t bits, squant_act_range_t* d_ranges, void* d_workspace,
                             size_t workspace_bytes, void* stream);

/* One layer of a network: its weight tensor and, where a batch norm follows it, that
 * layer's parameters (bn.gamma == NULL: no activation range for this layer). */
typedef struct {
  squant_tensor_t weight;
  squant_bn_t bn;
} squant_layer_t;

/* Device bytes squant_quantize_network asks for as workspace: 0. */
size_t squant_network_workspace_bytes(int32_t n_layers);

/* The data-free pipeline of Section 4 for a whole network in one call: every weight tensor
 * through the SQuant solver (binary32 weights, int8 codes, as squant_quantize_batched) and
 * every batch-norm output through squant_activation_ranges, on the same stream.  d_ranges
 * holds n_layers entries; entry i is written only when layer i has batch-norm parameters. */
int squant_quantize_network(const squant_layer_t* h_layers, int32_t n_layers, int32_t weight_bits,
                            squant_mode_t mode, int32_t act_bits, float n_sigma,
                            squant_act_range_t* d_ranges, void* d_workspace,
                            size_t workspace_bytes, void* stream);

/* Largest cin*kh*kw one output channel may have: 2^30, the bound of the shape check (0 for an
 * invalid kernel size).  Channels that fit none of the kernels which keep a channel on chip
 * (3x3 beyond cin 4096, other kernel sizes beyond about 32 K elements, 1x1 / FC rows beyond
 * about 160 K elements or off 16-byte alignment beyond 13 K) go through a streaming kernel
 * that walks the weights several times: correct for any shape, a fraction of the speed. */
int64_t squant_max_channel_elems(int32_t kh, int32_t kw);

const char* squant_status_string(int status);
int squant_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SQUANT_H_ */
