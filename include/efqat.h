/*
 * efqat.h -- C ABI of the EfQAT backward hot path for AMD MI355X (gfx950).
 *
 * EfQAT (arXiv 2411.11038) speeds up quantization-aware training by computing the
 * weight gradient of a quantized linear / convolution layer only for the k most
 * important output channels, while the input gradient stays complete (Alg. 1,
 * Fig. 1).  This library is that layer-level path:
 *
 *   efqat_fakequant_fwd    Eq. 1-4   codes, straight-through clip masks, scales
 *   efqat_channel_select   Eq. 6 + Top-K (Sec. 3.2), k = floor(r*C_out) (Sec. 3.4)
 *   efqat_linear_bwd       Eq. 5 restricted as in Alg. 1, plus S_x / Z_x / S_w gradients
 *   efqat_conv_bwd         the same two contractions with Eq. 8's shapes
 *
 * Conventions common to every call
 *   - Every tensor pointer is a DEVICE pointer owned by the caller; the library
 *     allocates nothing and keeps no state between calls (the benchmark timing hooks
 *     at the end of this file excepted).  Scratch memory comes in through
 *     (ws, ws_bytes); the matching *_workspace_bytes() query gives the size needed (a
 *     host-only computation).  ws must be 256-byte aligned.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     enqueue kernels on it and return without synchronising.  Two calls that share
 *     a workspace must be ordered on one stream.
 *   - Return value: 0 on success, a negative EFQAT_ERR_* otherwise.  Arguments are
 *     checked on the host before anything is launched, so a failing call has touched
 *     no device memory (EFQAT_ERR_HIP, a failed launch, excepted).
 *   - Layouts are dense row-major with the last index fastest.  Linear weights are
 *     W[C_out][C_in] (Y = X W^T, the convention the paper follows); conv activations
 *     are NHWC, conv weights OHWI, conv output gradients [N][H_out][W_out][C_out].
 *   - Clip masks are bit arrays: one row of ceil(cols/32) 32-bit words per tensor row;
 *     bit (j % 32) of word (j / 32) is 1 when element j was NOT clipped, i.e. its
 *     un-clamped integer code lies inside the closed code range (the gradient passes
 *     straight through), 0 when it was clipped.  Unused high bits of the last word are 0.
 *   - Rounding is to nearest, ties to even.  The integer code is decided on the
 *     correctly rounded single-precision quotient x / scale.
 */
#ifndef EFQAT_H_
#define EFQAT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EFQAT_VERSION 200

/* element types of activation / gradient tensors */
#define EFQAT_F32 0
#define EFQAT_BF16 1

/* quantizer kinds for efqat_fakequant_fwd */
#define EFQAT_QUANT_ACT_PER_TENSOR_ASYM 0 /* Eq. 1 / Eq. 2 */
#define EFQAT_QUANT_W_PER_ROW_SYM 1       /* Eq. 3 / Eq. 4 */

/* layout of the output gradient handed to the backward calls */
#define EFQAT_DY_TOKEN_MAJOR 0   /* [T][C_out]  (conv: [N][Ho][Wo][C_out]) */
#define EFQAT_DY_CHANNEL_MAJOR 1 /* [C_out][T]  (conv: [C_out][N][Ho][Wo]): the rows of the
                                    output-gradient matrix that Alg. 1 extracts are contiguous */

#define EFQAT_OK 0
#define EFQAT_ERR_NULL_PTR (-1)
#define EFQAT_ERR_BAD_SHAPE (-2)
#define EFQAT_ERR_BAD_BITS (-3)
#define EFQAT_ERR_BAD_K (-4)
#define EFQAT_ERR_BAD_LAYOUT (-5)
#define EFQAT_ERR_WORKSPACE (-6)
#define EFQAT_ERR_HIP (-7)
#define EFQAT_ERR_BAD_DTYPE (-8)
#define EFQAT_ERR_ALIGNMENT (-9)

int efqat_version(void);
/* Static string for an error code (never NULL). */
const char* efqat_strerror(int code);

/* Sec. 3.4: number of updated rows floor(r * C_out) for r = num/den, in integer
 * arithmetic.  Returns -1 for c_out < 0, num < 0, den <= 0 or num > den. */
int64_t efqat_k_from_ratio(int64_t c_out, int64_t num, int64_t den);

/* ------------------------------------------------------------------ fake-quant forward
 * Eq. 1 (mode ACT_PER_TENSOR_ASYM) or Eq. 3 with its bounds un-swapped, i.e.
 * clamp(round(w/S_w), -(2^(b-1)-1), 2^(b-1)-1) (mode W_PER_ROW_SYM), over a [rows][cols]
 * tensor.  For a conv weight pass rows = C_out, cols = KH*KW*C_in.
 *
 *   x           in   [rows][cols], dtype F32 or BF16
 *   bits        2..8
 *   init_minmax 1: first compute the quantizer parameters from the data -- Eq. 2 with
 *                  [alpha, beta] = [min x, max x] (one S_x, Z_x), or Eq. 4 per row -- and
 *                  write them to scale / zero_point; 0: read them as given.
 *                  A zero range (max == min, all-zero row) yields scale 1.
 *   scale       in/out  float[1] (act) or float[rows] (weights)
 *   zero_point  in/out  float[1] (act; may be non-integer after training: the forward
 *                  uses round(Z_x)); ignored (may be NULL) for weights, Z_w = 0
 *   codes       out  uint8 [rows][cols] (act) or int8 [rows][cols] (weights; b-bit values
 *                  are stored one per byte)
 *   clip_bits   out  uint32 [rows][ceil(cols/32)]
 *   xq          out, nullable  bf16 [rows][cols] de-quantised values S*(code - Z)
 */
size_t efqat_fakequant_fwd_workspace_bytes(int64_t rows, int64_t cols, int mode);
int efqat_fakequant_fwd(const void* x, int dtype, int64_t rows, int64_t cols, int mode, int bits,
                        int init_minmax, float* scale, float* zero_point, void* codes,
                        uint32_t* clip_bits, void* xq, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------ channel select
 * Eq. 6 with one block per output channel, I[c] = mean_j |w[c][j]| over `block` master
 * weights (C_in, or KH*KW*C_in for a conv), accumulated in double precision; then the
 * Top-K of Sec. 3.2: the k channels with the largest I, equal scores going to the lower
 * index, written in ascending index order.
 *
 *   w       in   float [c_out][block]
 *   k       0..c_out  (0 is valid: nothing is written to idx)
 *   scores  out, nullable  double[c_out]
 *   idx     out  int32[k]  (may be NULL when k == 0)
 */
size_t efqat_channel_select_workspace_bytes(int64_t c_out);
int efqat_channel_select(const float* w, int64_t c_out, int64_t block, int64_t k, double* scores,
                         int32_t* idx, void* ws, size_t ws_bytes, void* stream);

/* efqat_channel_select for callers that cannot allocate device memory or hand over a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the per-channel
 * scores are kept in a device array that is part of the library image (512 KiB on every GPU the
 * library runs on, for the life of the process) and are not returned.  Same w, k, idx and result as
 * efqat_channel_select; c_out above EFQAT_STATIC_SELECT_MAX_CHANNELS is EFQAT_ERR_WORKSPACE.  The call
 * allocates and frees nothing.  All calls on one GPU share that array: calls that overlap on one GPU
 * (different streams) race; order them.  The array's address is looked up on the first call on each
 * GPU, so make that first call outside a graph capture. */
#define EFQAT_STATIC_SELECT_MAX_CHANNELS 65536
int efqat_channel_select_static(const float* w, int64_t c_out, int64_t block, int64_t k, int32_t* idx,
                                void* stream);

/* Weight side of one training step in a single call: efqat_fakequant_fwd(mode W_PER_ROW_SYM, fp32
 * weights) followed by efqat_channel_select on the same weights, with identical results (Eq. 3 / Eq. 4
 * codes, clip masks and scales; Eq. 6 scores; Top-K).  With init_minmax != 0 and rows of at most 16384
 * weights (a multiple of 32, 16-byte aligned) the master weights are read once: the kernel that holds a
 * row in registers for its scale and codes also sums its magnitudes.
 *   w        in   float [c_out][block]
 *   scale    in/out float[c_out];  codes out int8 [c_out][block];  clip_bits out uint32 [c_out][ceil(block/32)]
 *   k        0..c_out;  scores out, nullable double[c_out];  idx out int32[k] ascending */
size_t efqat_weight_quant_select_workspace_bytes(int64_t c_out);
int efqat_weight_quant_select(const float* w, int64_t c_out, int64_t block, int bits, int init_minmax,
                              float* scale, int8_t* codes, uint32_t* clip_bits, int64_t k, double* scores,
                              int32_t* idx, void* ws, size_t ws_bytes, void* stream);

/* EfQAT-CWPN (Table 2): one Top-K over the channels of several layers together.
 *   scores      in   double[total] = the per-layer score arrays of efqat_channel_select,
 *                    concatenated in layer order (device)
 *   layer_off   in   int64[n_layers+1] (device), ascending prefix offsets into scores,
 *                    layer_off[0] = 0, layer_off[n_layers] = total
 *   k_total     0..total
 *   idx         out  int32[k_total]: selected channels, layer by layer, ascending channel
 *                    index within each layer (index local to its layer)
 *   k_per_layer out  int32[n_layers] (device): how many channels of each layer were selected
 * Ties go to the earlier layer, then the lower channel.  EfQAT-LWPN is the same call on one
 * score per layer (n_layers = total). */
size_t efqat_network_select_workspace_bytes(int64_t total);
int efqat_network_select(const double* scores, const int64_t* layer_off, int64_t n_layers,
                         int64_t total, int64_t k_total, int32_t* idx, int32_t* k_per_layer,
                         void* ws, size_t ws_bytes, void* stream);

/* EfQAT-LWPN (Table 2): the blocks are whole layers; the importance of a layer is the mean
 * |w| over all of its weights (Eq. 6 with one block per layer), which equals the mean of its
 * per-channel scores because every channel of a layer has the same number of weights.  The
 * k_layers most important layers are unfrozen entirely (their channel count is reported),
 * the others frozen entirely (count 0); ties go to the earlier layer.
 *   scores       in   double[layer_off[n_layers]] per-channel scores, layer after layer (device)
 *   layer_off    in   int64[n_layers+1] ascending prefix offsets (device)
 *   k_layers     0..n_layers
 *   layer_scores out, nullable  double[n_layers]
 *   layer_idx    out  int32[k_layers] ascending (may be NULL when k_layers == 0)
 *   k_per_layer  out  int32[n_layers]: C_out of the layer if it is unfrozen, else 0 */
size_t efqat_layer_select_workspace_bytes(int64_t n_layers);
int efqat_layer_select(const double* scores, const int64_t* layer_off, int64_t n_layers,
                       int64_t k_layers, double* layer_scores, int32_t* layer_idx,
                       int32_t* k_per_layer, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------ bias gradient
 * db[c] = sum_t dY[t][c] for every output channel: biases (and normalisation parameters) are
 * never frozen (Sec. 3.4; the optimizer step of Alg. 1 always updates them).  For a
 * convolution pass T = N*Ho*Wo.
 *   dy   in   [T][c_out] (token major) or [c_out][T] (channel major), fp32 or bf16
 *   db   out  float[c_out], fully overwritten
 * fp32 partial sums over chunks of tokens, summed in double precision in a fixed order
 * (bit-reproducible). */
size_t efqat_bias_grad_workspace_bytes(int64_t T, int64_t c_out, int dy_layout);
int efqat_bias_grad(const void* dy, int dy_dtype, int dy_layout, int64_t T, int64_t c_out,
                    float* db, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------ choice of the dX kernel
 * Argument dx_kernel of the *_ex entry points below, for tests and measurements; the plain entry
 * points use AUTO.  It chooses the kernel of the dX product (Eq. 5 left) where more than one applies
 * (bf16 token-major dY, C_out % 8 == 0, C_in % 16 == 0): AUTO picks by problem size, BF16 always
 * stages a bf16 copy of W_q^T, INT8 always reads the weight operand from the int8 codes.  BF16_PINNED
 * (any linear layer, and convolutions whose dX product runs on a staged im2col matrix) stages the bf16
 * copy and always uses the 192 x 192 kernel with the hand-pinned instruction order, which AUTO and
 * BF16 take only where the planner picks that tile.  All choices give the same results up to the
 * order of the fp32 sums.  The workspace size depends on it: *_workspace_bytes_ex takes it too. */
#define EFQAT_DX_KERNEL_AUTO 0
#define EFQAT_DX_KERNEL_BF16 1
#define EFQAT_DX_KERNEL_INT8 2
#define EFQAT_DX_KERNEL_BF16_PINNED 3

/* ------------------------------------------------------------------ linear backward
 * Backward step of Alg. 1 for one layer Y = X_q W_q^T, X_q = S_x (x_codes - Z_x),
 * W_q[c][:] = S_w[c] w_codes[c][:]:
 *
 *   dX      = (dY W_q) with clipped activations zeroed            (Eq. 5 left; all channels)
 *   dW[id]  = (dY[:, id]^T X_q) with clipped weights zeroed       (Eq. 5 right, rows id only)
 *   dS_w[id], dS_x, dZ_x: gradients of the quantizer parameters through Eq. 1 / Eq. 3 with
 *   d round(u)/du = 1:  in range  d X_q/d S_x = round(x/S_x) - x/S_x, d X_q/d Z_x = 0;
 *   clipped  d X_q/d S_x = code - Z_x, d X_q/d Z_x = -S_x; weights alike with Z_w = 0.
 *   S_w gradients exist only for the updated rows (Sec. 3.2, quantization granularity).
 *
 * The products run on bf16 matrix cores with fp32 accumulation: dY and W_q are rounded
 * to bf16 (x_codes - Z_x is exact in bf16).
 *
 *   dy        in  [T][c_out] or [c_out][T] per dy_layout, dtype dy_dtype
 *   x_codes   in  uint8 [T][c_in];   x_clip  in  uint32 [T][ceil(c_in/32)]
 *   x         in  [T][c_in] original activations (dtype x_dtype), for dS_x
 *   s_x, z_x  in  float[1] each, device
 *   w_codes   in  int8 [c_out][c_in]; w_clip in uint32 [c_out][ceil(c_in/32)]
 *   w         in  float [c_out][c_in] master weights, for dS_w;  s_w in float[c_out]
 *   idx       in  int32[k], strictly ascending, each in [0, c_out) (not checked on the
 *                 device: out-of-range entries are the caller's error); NULL iff k == 0
 *   dx        out [T][c_in], dtype dx_dtype
 *   dw        out float: scatter == 0 -> [k][c_in], row m is channel idx[m];
 *                        scatter == 1 -> [c_out][c_in], only rows idx are written
 *   ds_w      out float: [k] (scatter == 0) or [c_out] with only entries idx written
 *   ds_x,dz_x out float[1] each
 *   dw / ds_w may be NULL when k == 0 (dX, dS_x, dZ_x are still produced).
 * Alignment: dy 16 bytes; x_codes and w_codes 16 bytes when c_in is a multiple of 16 (their
 * tiles are then copied 16 bytes at a time); everything else to its element size.  A
 * misaligned pointer is reported as EFQAT_ERR_ALIGNMENT, never read.
 * The workspace size depends on k in both directions (k == c_out needs no compacted copy of
 * dY): query it for the k that is passed.
 */
size_t efqat_linear_bwd_workspace_bytes(int64_t T, int64_t c_in, int64_t c_out, int64_t k,
                                        int dy_dtype, int dy_layout);
int efqat_linear_bwd(const void* dy, int dy_dtype, int dy_layout, int64_t T, int64_t c_in,
                     int64_t c_out, const uint8_t* x_codes, const uint32_t* x_clip, const void* x,
                     int x_dtype, const float* s_x, const float* z_x, const int8_t* w_codes,
                     const uint32_t* w_clip, const float* w, const float* s_w, const int32_t* idx,
                     int64_t k, void* dx, int dx_dtype, float* dw, int scatter, float* ds_w,
                     float* ds_x, float* dz_x, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------ weight operand made beforehand
 * Where the dX product (Eq. 5 left) of efqat_linear_bwd multiplies by a bf16 copy of W_q^T, that copy
 * depends on the weight codes and scales only, not on dY or the activations.  A caller that quantizes
 * its weights away from the critical path (another stream, an earlier point of the step) can have it
 * made there and hand it to efqat_linear_bwd_ex (argument w_operand), which then skips that pass;
 * results are bit-identical to efqat_linear_bwd.
 *
 *   efqat_linear_bwd_weight_operand_bytes  size of the operand buffer for a layer, or 0 when the
 *       dX product of that layer reads the int8 codes themselves (no copy exists; the buffer is
 *       then ignored).
 *   efqat_linear_bwd_weight_operand        fills it from w_codes int8 [c_out][c_in] and s_w
 *       float [c_out]: operand = bf16 [c_in][round_up(c_out, 8)] with
 *       operand[i][c] = bf16(s_w[c] * w_codes[c][i]), zero padding, then 256 zero bytes.
 *       operand: device, 256-byte aligned, owned by the caller, read-only afterwards.
 * The operand must come from the same w_codes, s_w, sizes, dy_dtype and dy_layout as the backward
 * call, and the work that fills it must be ordered before that call's stream reaches it (the
 * caller's events).  A buffer that is too small is EFQAT_ERR_WORKSPACE. */
size_t efqat_linear_bwd_weight_operand_bytes(int64_t T, int64_t c_in, int64_t c_out, int dy_dtype,
                                             int dy_layout);
int efqat_linear_bwd_weight_operand(const int8_t* w_codes, const float* s_w, int64_t T, int64_t c_in,
                                    int64_t c_out, int dy_dtype, int dy_layout, void* operand,
                                    size_t operand_bytes, void* stream);

/* ------------------------------------------------------------------ backward + optimizer step
 * Optimizer step of Alg. 1 on the unfrozen channels, applied in the same pass over the k updated rows
 * that finishes the weight gradient, so that it need not travel through memory.  Frozen rows, their
 * scales and every piece of optimizer state that belongs to them are not touched.
 *
 * Weight rows idx keep the optimizer of the full-precision run (Sec. 4 "Setup"): SGD with momentum
 * and weight decay,
 *   g   = dW[c][:] + weight_decay * w[c][:]
 *   buf = momentum * mom_w[c][:] + g  (stored back)  when momentum != 0, else buf = g
 *   w[c][:] -= lr_w * buf
 * Their scales s_w[idx] are quantization parameters, which are always trained with Adam (Sec. 4
 * "Setup"); with g = dS_w[c], per channel c in idx,
 *   adam_t[c] += 1;  m = beta1 m + (1 - beta1) g;  v = beta2 v + (1 - beta2) g^2   (stored back)
 *   s_w[c] -= lr_s * (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps)
 * (Adam as published, with bias correction and no weight decay).  The paper gives no betas or eps
 * and does not say what the Adam state of a frozen channel does: here every channel has its own
 * moments and step count, which advance only when that channel is updated.
 *
 * w and s_w are read (old values: dX, the clip masks and dS_w refer to them) and then updated in
 * place; dw and ds_w become optional (NULL: not written). */
typedef struct efqat_opt_step {
  float lr_w;          /* learning rate of the weights */
  float momentum;      /* 0: plain SGD, mom_w is ignored and may be NULL */
  float weight_decay;  /* weights only */
  float* mom_w;        /* device, float [c_out][c_in] (conv: [c_out][KH][KW][c_in]) */
  float lr_s;          /* Adam on the weight scales: learning rate, */
  float beta1, beta2;  /*   decay rates in [0, 1), */
  float eps;           /*   eps >= 0 */
  float* adam_m;       /* device, float [c_out]: first moments  (zero before the first step) */
  float* adam_v;       /* device, float [c_out]: second moments (zero before the first step) */
  int32_t* adam_t;     /* device, int32 [c_out]: steps taken per channel (zero before the first) */
} efqat_opt_step;

/* efqat_linear_bwd with four optional extras (all NULL / 0: exactly efqat_linear_bwd):
 *   w_operand    the dX weight operand made beforehand (see above); needs dx_kernel == AUTO
 *   step         fused optimizer step (see above); w and s_w are then updated in place
 *   dx_kernel    EFQAT_DX_KERNEL_*
 *   side_stream  a second HIP stream of the caller (default priority) on the same device.  The two
 *                products of Eq. 5 do not depend on each other: with a second stream the compaction
 *                of the selected dY columns and the dW product are enqueued there, behind
 *                everything `stream` held when the call was made, and run beside the dX product, so
 *                that the partly filled last round of workgroups of either product is filled by the
 *                other.  The call joins the branch back into `stream` before the pass that finishes
 *                dW, dS_w, dS_x and dZ_x: as without it, every output is ready in `stream` order,
 *                and results are bit-identical.  The fork and join use two HIP events that the
 *                library creates at the first such call of a host thread on a device and keeps
 *                (no other state; nothing is created on later calls).  Ignored when k == 0, when it
 *                equals `stream`, and on the layouts whose dW product runs on staged copies.
 * Workspace: efqat_linear_bwd_workspace_bytes_ex with the same dx_kernel. */
size_t efqat_linear_bwd_workspace_bytes_ex(int64_t T, int64_t c_in, int64_t c_out, int64_t k,
                                           int dy_dtype, int dy_layout, int dx_kernel);
int efqat_linear_bwd_ex(const void* dy, int dy_dtype, int dy_layout, int64_t T, int64_t c_in,
                        int64_t c_out, const uint8_t* x_codes, const uint32_t* x_clip, const void* x,
                        int x_dtype, const float* s_x, const float* z_x, const int8_t* w_codes,
                        const uint32_t* w_clip, float* w, float* s_w, const int32_t* idx, int64_t k,
                        void* dx, int dx_dtype, float* dw, int scatter, float* ds_w, float* ds_x,
                        float* dz_x, const void* w_operand, const efqat_opt_step* step, int dx_kernel,
                        void* ws, size_t ws_bytes, void* stream, void* side_stream);

/* ------------------------------------------------------------------ conv backward
 * Same as efqat_linear_bwd for Y[n][ho][wo][co] = sum_{kh,kw,ci}
 * X_q[n][ho*stride+kh-pad][wo*stride+kw-pad][ci] * W_q[co][kh][kw][ci] (zero outside the
 * image), the contraction sizes of Eq. 8.  x_codes/x/dx are [N][H][W][c_in]; x_clip has one
 * bit row per pixel ([N*H*W][ceil(c_in/32)]); w_codes/w/dw are [..][KH][KW][c_in] with
 * w_clip rows of ceil(KH*KW*c_in/32) words; dy is [N][Ho][Wo][c_out] (token major) or
 * [c_out][N][Ho][Wo] (channel major), Ho = (H + 2 pad - KH)/stride + 1.
 */
size_t efqat_conv_bwd_workspace_bytes(int64_t N, int64_t H, int64_t W, int64_t c_in, int64_t c_out,
                                      int64_t KH, int64_t KW, int64_t stride, int64_t pad,
                                      int64_t k, int dy_dtype, int dy_layout);
int efqat_conv_bwd(const void* dy, int dy_dtype, int dy_layout, int64_t N, int64_t H, int64_t W,
                   int64_t c_in, int64_t c_out, int64_t KH, int64_t KW, int64_t stride,
                   int64_t pad, const uint8_t* x_codes, const uint32_t* x_clip, const void* x,
                   int x_dtype, const float* s_x, const float* z_x, const int8_t* w_codes,
                   const uint32_t* w_clip, const float* w, const float* s_w, const int32_t* idx,
                   int64_t k, void* dx, int dx_dtype, float* dw, int scatter, float* ds_w,
                   float* ds_x, float* dz_x, void* ws, size_t ws_bytes, void* stream);

/* efqat_conv_bwd with the optional fused optimizer step, dX kernel choice and second stream of
 * efqat_linear_bwd_ex. */
size_t efqat_conv_bwd_workspace_bytes_ex(int64_t N, int64_t H, int64_t W, int64_t c_in, int64_t c_out,
                                         int64_t KH, int64_t KW, int64_t stride, int64_t pad,
                                         int64_t k, int dy_dtype, int dy_layout, int dx_kernel);
int efqat_conv_bwd_ex(const void* dy, int dy_dtype, int dy_layout, int64_t N, int64_t H, int64_t W,
                      int64_t c_in, int64_t c_out, int64_t KH, int64_t KW, int64_t stride, int64_t pad,
                      const uint8_t* x_codes, const uint32_t* x_clip, const void* x, int x_dtype,
                      const float* s_x, const float* z_x, const int8_t* w_codes, const uint32_t* w_clip,
                      float* w, float* s_w, const int32_t* idx, int64_t k, void* dx, int dx_dtype,
                      float* dw, int scatter, float* ds_w, float* ds_x, float* dz_x,
                      const efqat_opt_step* step, int dx_kernel, void* ws, size_t ws_bytes, void* stream,
                      void* side_stream);

/* ------------------------------------------------------------------ low-precision forward
 * The forward product of Sec. 3.1, Y = X_q W_q^T, computed from the 8-bit codes on the int8 matrix
 * cores with exact int32 accumulation:
 *   y[t][c] = S_x * S_w[c] * sum_i (x_codes[t][i] - round(Z_x)) * w_codes[c][i]
 * (the paper leaves this pass out of its timings; it is here because it consumes exactly what
 * efqat_fakequant_fwd emits).
 *   x_codes  in  uint8 [T][c_in];  w_codes  in  int8 [c_out][c_in];  s_x, z_x float[1];  s_w float[c_out]
 *   y        out [T][c_out], dtype y_dtype (F32 or BF16)
 *   c_in <= 131072.  Codes must be 16-byte aligned unless c_in is not a multiple of 16 (then they
 *   are copied into zero-padded rows in the workspace). */
size_t efqat_linear_fwd_workspace_bytes(int64_t T, int64_t c_in, int64_t c_out);
int efqat_linear_fwd(const uint8_t* x_codes, const float* s_x, const float* z_x, const int8_t* w_codes,
                     const float* s_w, int64_t T, int64_t c_in, int64_t c_out, void* y, int y_dtype,
                     void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------ kernel timing (benchmarks)
 * To report each kernel class against its roofline a benchmark can have the library bracket its
 * launches with HIP events on the stream they go to.  This is the only process-wide state of the
 * library; it is off by default and not thread-safe.
 *   efqat_profile_enable(on)  on != 0 starts a new measurement (counters reset), 0 stops it.
 *                             At most 4096 brackets per class are recorded.
 *   efqat_profile_read(which, total_ms, launches)  waits for the recorded events of one class
 *                             (host pointers out: summed time in ms, number of brackets). */
#define EFQAT_PROF_DX 0          /* input-gradient product with its fused epilogue */
#define EFQAT_PROF_DW 1          /* weight-gradient product */
#define EFQAT_PROF_FWD 2         /* low-precision forward product */
#define EFQAT_PROF_PREP 3        /* operand preparation: compaction of the selected dY columns, staged copies */
#define EFQAT_PROF_FINISH 4      /* second pass of the weight gradient (split-K sum, masks, dS_w, dS_x, dZ_x) */
#define EFQAT_PROF_QUANT_ACT 5   /* efqat_fakequant_fwd, activations (all its kernels) */
#define EFQAT_PROF_QUANT_W 6     /* efqat_fakequant_fwd, weights */
#define EFQAT_PROF_IMPORTANCE 7  /* Eq. 6 scores */
#define EFQAT_PROF_TOPK 8        /* Top-K */
#define EFQAT_PROF_BIAS 9        /* efqat_bias_grad (both kernels) */
#define EFQAT_PROF_CLASSES 10
int efqat_profile_enable(int on);
int efqat_profile_read(int which, double* total_ms, int64_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* EFQAT_H_ */
