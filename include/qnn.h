/*
 * qnn.h -- C ABI of the MI355X (gfx950) quantized-inference library.
 *
 * The library implements the integer inference scheme of "Quantizing deep
 * convolutional networks for efficient inference: A whitepaper" (arXiv
 * 1806.08342): uint8 activations with one affine quantizer (Delta, z) per
 * tensor, int8 (or 4-bit) weights with one symmetric quantizer per output
 * channel, int32 accumulation with the zero-point correction of eq. 5-6 and an
 * int32 bias, and a fixed-point rescale back to uint8 with the ReLU / ReLU6
 * clamp fused in.
 *
 * General rules for every entry point
 *   - Pointers marked DEVICE are HIP device pointers owned by the caller
 *     (for example the storage of a torch tensor).  Pointers marked HOST are
 *     ordinary host pointers.  The library never allocates, frees or keeps
 *     any of them, and never allocates device memory of its own.
 *   - Scratch memory comes from the caller: the dense entry points take
 *     `workspace` (DEVICE, 16-byte aligned, may be NULL) and `workspace_bytes`.
 *     qnn_qgemm_workspace_bytes / qnn_qconv2d_workspace_bytes say how much a
 *     shape can use (0 for most): the int32 partial sums of products whose K
 *     is divided over several workgroups because they have too few output
 *     tiles for the chip, and the activation row sums of the asymmetric-weight
 *     entry points.  With a smaller or NULL workspace the symmetric entry
 *     points take a route that needs none (same result, possibly slower); the
 *     asymmetric ones return QNN_EINVAL.  The workspace is written and read by
 *     the kernels of that one call only; its contents need no initialisation
 *     and mean nothing afterwards.  Calls that may run concurrently (different
 *     streams, graph branches) need workspaces that do not overlap.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Device entry points only enqueue work on that stream and return; they
 *     never synchronise.  Output buffers must not overlap input buffers.
 *   - Return value: QNN_OK, or an error code; on error nothing is enqueued.
 *     QNN_EINVAL      a null pointer, a non-positive size, a parameter outside
 *                     the documented range.  An EMPTY input is not an error: n == 0
 *                     elements, M == 0 rows of a product, or N == 0 images of a
 *                     convolution return QNN_OK without enqueuing anything and
 *                     without looking at the pointers (all other sizes must be
 *                     positive);
 *     QNN_EUNSUPPORTED a documented feature this build does not implement;
 *     QNN_ELAUNCH     the HIP runtime refused the launch (qnn_last_error()
 *                     gives the HIP error text).
 *     The contents of device arrays (mult, shift, bias) are trusted and not read
 *     on the host; `shift` entries must lie in [-31, 31], which the host helper
 *     qnn_quantize_multiplier guarantees (the kernels treat a value outside as the
 *     nearest end of that range).
 *
 * The fixed-point rescale (not defined by the paper; this is the library's
 * definition, referred to as RESCALE(a; mult, shift) below), on an int32 a:
 *   1. if shift < 0:  a <- saturate_int32(a * 2^(-shift))
 *   2. h = nearest integer to a*mult / 2^31, ties toward +infinity, computed
 *      exactly in 64 bits; the single overflowing case a = mult = INT32_MIN
 *      gives INT32_MAX                    (saturating rounding doubling high multiply)
 *   3. r = nearest integer to h / 2^max(shift,0), ties away from zero
 *   so that r ~= a * mult * 2^(-31-shift).  Outputs are
 *   y = clamp(act_min, act_max, z_out + r) stored as uint8, 0 <= act_min <= act_max <= 255,
 *   0 <= z_out <= 255.  ReLU is act_min = z_out; ReLU6 additionally lowers act_max
 *   (qnn_act_range).
 */
#ifndef QNN_H
#define QNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { QNN_OK = 0, QNN_EINVAL = 1, QNN_EUNSUPPORTED = 2, QNN_ELAUNCH = 3 } qnn_status;

/* storage order of the GEMM weight operand B (a K x N matrix) */
#define QNN_B_COLUMNS_CONTIGUOUS 0 /* element (k,n) at B[n*ldb + k]: one output column = one contiguous kernel */
#define QNN_B_ROWS_CONTIGUOUS 1    /* element (k,n) at B[k*ldb + n] */

/* Text of the last HIP error seen by a call that returned QNN_ELAUNCH on this thread
 * (HOST string owned by the library, valid until the next failing call). */
const char *qnn_last_error(void);

/* Library version, "major.minor". */
const char *qnn_version(void);

/* ---------------------------------------------------------------- device entry points */

/* Uniform affine quantizer, Sec. 2.1 eq. 1-2:
 *   q[i] = clamp(qmin, qmax, round(x[i] / scale) + zero_point)
 * x / scale is one IEEE binary32 division, round() rounds ties away from zero, NaN
 * quantizes like 0.0.  Requires scale > 0 finite and 0 <= qmin <= zero_point <= qmax <= 255.
 * x: DEVICE fp32[n] (read), q: DEVICE uint8[n] (written).  n == 0 is a no-op. */
qnn_status qnn_quantize(const float *x, uint8_t *q, size_t n, float scale, int32_t zero_point, int32_t qmin,
                        int32_t qmax, void *stream);

/* De-quantizer, Sec. 2.1 eq. 3:  x[i] = (q[i] - zero_point) * scale  (one binary32 multiply).
 * q: DEVICE uint8[n] (read), x: DEVICE fp32[n] (written).  0 <= zero_point <= 255. */
qnn_status qnn_dequantize(const uint8_t *q, float *x, size_t n, float scale, int32_t zero_point, void *stream);

/* Stand-alone rescale of an int32 accumulator tensor to uint8 (the epilogue of the
 * convolution kernels as a kernel of its own):
 *   y[r][c] = clamp(act_min, act_max, z_out + RESCALE(acc[r][c]; mult[p], shift[p])),
 *   p = c when per_channel != 0 (Sec. 2.6: one quantizer per output channel), else 0.
 * acc: DEVICE int32[rows*channels] row-major (read); y: DEVICE uint8[rows*channels] (written);
 * mult, shift: DEVICE int32[channels] (or [1]). */
qnn_status qnn_requantize(const int32_t *acc, uint8_t *y, size_t rows, size_t channels, const int32_t *mult,
                          const int32_t *shift, int per_channel, int32_t z_out, int32_t act_min, int32_t act_max,
                          void *stream);

/* Quantized matrix product / fully connected layer, Sec. 2.1 eq. 4-6 with z_w = 0:
 *   C[m][n] = clamp(act_min, act_max, z_out + RESCALE(bias[n] + sum_k (A[m][k] - z_a) * B[k][n]; mult[n], shift[n]))
 * The sum is evaluated as sum_k A*B - z_a * sum_k B[k][n] (eq. 5-6; the weight column
 * sums are formed inside the kernel), in int32; |sum| must stay below 2^31, which K <= 65536
 * guarantees (larger K is rejected with QNN_EINVAL).
 * A: DEVICE uint8, M x K row-major, row pitch lda >= K (bytes = elements).
 * B: DEVICE weights, K x N, layout b_layout; weight_bits 8 -> int8 elements; weight_bits 4 ->
 *    two's-complement nibbles, element 2j of a column in the low nibble of byte j and element
 *    2j+1 in the high nibble (requires QNN_B_COLUMNS_CONTIGUOUS, K and ldb even; ldb counts
 *    elements, so a column occupies ldb/2 bytes).
 *    QNN_B_COLUMNS_CONTIGUOUS is the fast layout; QNN_B_ROWS_CONTIGUOUS is accepted for int8
 *    and runs a slower gather path (use qnn_pack_b once, weights being constant at inference).
 * bias: DEVICE int32[N] or NULL (scale s_a * Delta_n, zero-point 0); mult, shift: DEVICE int32[N].
 * C: DEVICE uint8, M x N row-major, row pitch ldc >= N (written).
 * workspace: DEVICE scratch of workspace_bytes bytes or NULL (see the general rules). */
qnn_status qnn_qgemm(const uint8_t *A, int64_t lda, int32_t z_a, const void *B, int64_t ldb, int b_layout,
                     int weight_bits, int64_t M, int64_t N, int64_t K, const int32_t *bias, const int32_t *mult,
                     const int32_t *shift, int32_t z_out, int32_t act_min, int32_t act_max, uint8_t *C, int64_t ldc,
                     void *workspace, size_t workspace_bytes, void *stream);

/* qnn_qgemm for callers that cannot allocate device memory and have no workspace to pass: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and same
 * result as qnn_qgemm; the scratch memory (partial sums of products whose K is divided over several
 * workgroups) is a static 16 MiB device array inside the library, which every GPU the library runs on
 * holds until the process ends.  The call allocates nothing.  A product whose plan asks for more than
 * 16 MiB of scratch (qnn_qgemm_workspace_bytes) is rejected with QNN_EUNSUPPORTED and a message in
 * qnn_last_error().  The array is shared by all calls on one GPU and keeps the last call's contents
 * (every call writes what it reads, nothing needs clearing): calls that overlap on one GPU -- other
 * streams, concurrent graph branches -- race on it; order them, or use qnn_qgemm with separate
 * workspaces.  The device address of the array is looked up at the first call on each device (make
 * that call outside stream capture). */
qnn_status qnn_qgemm_noalloc(const uint8_t *A, int64_t lda, int32_t z_a, const void *B, int64_t ldb, int b_layout,
                             int weight_bits, int64_t M, int64_t N, int64_t K, const int32_t *bias, const int32_t *mult,
                             const int32_t *shift, int32_t z_out, int32_t act_min, int32_t act_max, uint8_t *C, int64_t ldc,
                             void *stream);

/* Scratch bytes that qnn_qgemm / qnn_qgemm_add (asym == 0) or qnn_qgemm_asym (asym != 0) can use for an
 * M x N x K product with weight_bits-bit weights, and the same for the convolution entry points
 * (Sec. 2.1 eq. 4-6: the partial sums are pieces of the same integer sum, so the result does not
 * depend on whether they are used).  Host-only; 0 when the shape needs none. */
size_t qnn_qgemm_workspace_bytes(int64_t M, int64_t N, int64_t K, int weight_bits, int asym);
size_t qnn_qconv2d_workspace_bytes(int N, int H, int W, int Cin, int Cout, int kh, int kw, int weight_bits, int stride_h,
                                   int stride_w, int pad_h, int pad_w, int asym);

/* Tuning switch `name` ("QNN_FORCE_TILE", "QNN_FORCE_SPLIT", "QNN_NO_SHORTK", "QNN_BRES", "QNN_STEM_BLOCK",
 * "QNN_XCD_ROWS", "QNN_DW_RH", "QNN_DW_MAD", "QNN_GEMM_PRIO", "QNN_PERSIST", "QNN_DW_VARIANT") set to the
 * HOST string `value`, or back to its default with value == NULL.  The switches start from the
 * environment variables of the same names, read once when the library is first used; they select among
 * kernels that give identical results (the parity tests use them to reach every variant on small shapes).
 * Not synchronised: change them only while no other thread is inside a library call. */
qnn_status qnn_tuning_set(const char *name, const char *value);

/* Name of the kernel configuration (a tile "<BM>x<BN>", with "/k<n>" when K is divided over n
 * workgroups per tile, or "shortk" / "skinny16") that qnn_qgemm and the convolution entry points
 * select for an aligned int8 M x N x K product (M = output pixels, N = output channels, K = kh*kw*Cin);
 * for logging and profiling.  HOST string owned by the library; "" for non-positive sizes. */
const char *qnn_qgemm_plan(int64_t M, int64_t N, int64_t K);

/* Transpose a K x N int8 matrix with contiguous rows (src[k*ld_src + n]) into the
 * columns-contiguous layout (dst[n*ld_dst + k]) that qnn_qgemm runs fastest on.
 * src, dst: DEVICE int8; ld_src >= N, ld_dst >= K. */
qnn_status qnn_pack_b(const int8_t *src, int64_t ld_src, int64_t K, int64_t N, int8_t *dst, int64_t ld_dst,
                      void *stream);

/* Quantized 2-D convolution (cross-correlation), Sec. 2.1 eq. 4-6 with z_w = 0:
 *   y[n][ho][wo][co] = clamp(act_min, act_max, z_out + RESCALE(bias[co] +
 *        sum_{a,b,ci} (x[n][ho*stride_h - pad_h + a][wo*stride_w - pad_w + b][ci] - z_x) * w[co][a][b][ci];
 *        mult[co], shift[co]))
 * Taps outside the image contribute 0, i.e. the border is padded with the code z_x of real
 * zero (Sec. 2.1: zero padding causes no quantization error).
 * x: DEVICE uint8 NHWC [N][H][W][Cin] contiguous (read).
 * w: DEVICE weights [Cout][kh][kw][Cin] contiguous; weight_bits 8 -> int8; 4 -> nibble pairs along
 *    Cin as in qnn_qgemm (Cin even).
 * Ho = (H + 2 pad_h - kh)/stride_h + 1, Wo likewise; y: DEVICE uint8 NHWC [N][Ho][Wo][Cout] (written).
 * kh*kw*Cin <= 65536.  bias may be NULL; bias, mult, shift: DEVICE int32[Cout]. */
qnn_status qnn_qconv2d(const uint8_t *x, int N, int H, int W, int Cin, int32_t z_x, const void *w, int Cout, int kh,
                       int kw, int weight_bits, int stride_h, int stride_w, int pad_h, int pad_w, const int32_t *bias,
                       const int32_t *mult, const int32_t *shift, int32_t z_out, int32_t act_min, int32_t act_max,
                       uint8_t *y, void *workspace, size_t workspace_bytes, void *stream);

/* Depthwise convolution (one kh x kw kernel per channel; the separable layers of the
 * MobileNet family the paper evaluates), same arithmetic as qnn_qconv2d per channel:
 *   y[n][ho][wo][c] = clamp(..., z_out + RESCALE(bias[c] + sum_{a,b} (x[n][hi][wi][c] - z_x) * w[a][b][c]; mult[c], shift[c]))
 * x: DEVICE uint8 NHWC [N][H][W][C]; w: DEVICE int8 [kh][kw][C]; y: DEVICE uint8 NHWC [N][Ho][Wo][C].
 * kh, kw <= 7.  bias may be NULL; bias, mult, shift: DEVICE int32[C]. */
qnn_status qnn_qdwconv2d(const uint8_t *x, int N, int H, int W, int C, int32_t z_x, const int8_t *w, int kh, int kw,
                         int stride_h, int stride_w, int pad_h, int pad_w, const int32_t *bias, const int32_t *mult,
                         const int32_t *shift, int32_t z_out, int32_t act_min, int32_t act_max, uint8_t *y,
                         void *stream);

/* Element-wise addition of two uint8 tensors that carry different quantizers (Sec. 3.2.1:
 * both operands are rescaled to a common scale before the add; a following ReLU is the clamp):
 *   ta = (a[i] - z_a) * 2^left_shift,  tb = (b[i] - z_b) * 2^left_shift
 *   u  = RESCALE(ta; mult_a, shift_a) + RESCALE(tb; mult_b, shift_b)
 *   y[i] = clamp(act_min, act_max, z_out + RESCALE(u; mult_o, shift_o))
 * Parameters come from qnn_qadd_params.  0 <= left_shift <= 22.
 * a, b: DEVICE uint8[n] (read); y: DEVICE uint8[n] (written). */
qnn_status qnn_qadd(const uint8_t *a, int32_t z_a, int32_t mult_a, int32_t shift_a, const uint8_t *b, int32_t z_b,
                    int32_t mult_b, int32_t shift_b, int32_t left_shift, int32_t mult_o, int32_t shift_o,
                    int32_t z_out, int32_t act_min, int32_t act_max, uint8_t *y, size_t n, void *stream);

/* Re-quantization of uint8 codes from one quantizer to another (Sec. 3.2.1: the inputs of a
 * concatenation have to be rescaled to the output's quantizer before they are laid side by side):
 *   y[m][c] = clamp(act_min, act_max, z_out + RESCALE(x[m][c] - z_in; mult, shift)),
 * mult, shift from qnn_quantize_multiplier(s_in / s_out).  rows x cols elements with row pitches
 * ldx, ldy >= cols, so y can be a channel slice of the concatenated NHWC tensor (ldy = its channel count).
 * x: DEVICE uint8 (read); y: DEVICE uint8 (written); the two must not overlap. */
qnn_status qnn_rescale_u8(const uint8_t *x, int64_t ldx, int32_t z_in, int32_t mult, int32_t shift, int32_t z_out,
                          int32_t act_min, int32_t act_max, uint8_t *y, int64_t ldy, int64_t rows, int64_t cols,
                          void *stream);

/* The add of Sec. 3.2.1 fused behind the layer that produces one of its operands (the last 1x1
 * convolution of a residual block; fusing operators is what Sec. 3.2.1 and the accelerator
 * recommendations of Sec. 7 advise): the layer's uint8 result never goes to memory.  Bit for bit the same as
 *   qnn_qgemm / qnn_qconv2d (with z_out = z_mid, act_min = mid_min, act_max = mid_max) into a
 *   temporary t, followed by
 *   qnn_qadd(t, z_mid, mult_m, shift_m, residual, z_r, mult_r, shift_r, left_shift, mult_o, shift_o,
 *            z_out, act_min, act_max).
 * (z_mid, mid_min, mid_max): the quantizer and clamp of the layer's own uint8 result (the first
 * operand of the add).  add: HOST pointer, read during the call.
 * residual: DEVICE uint8, same shape as the output ([M][N] with row pitch ldr >= N for qgemm, dense
 * NHWC [N][Ho][Wo][Cout] for qconv2d), must not overlap the output.  Layers whose kernel cannot apply
 * the add in its epilogue run it as a second pass over the output; the result is the same. */
typedef struct qnn_add_params {
    int32_t mult_m, shift_m;        /* the layer's result enters the add with these */
    int32_t z_r, mult_r, shift_r;   /* the residual operand */
    int32_t left_shift, mult_o, shift_o;
    int32_t z_out, act_min, act_max; /* quantizer / fused activation of the sum */
} qnn_add_params;

qnn_status qnn_qgemm_add(const uint8_t *A, int64_t lda, int32_t z_a, const void *B, int64_t ldb, int b_layout,
                         int weight_bits, int64_t M, int64_t N, int64_t K, const int32_t *bias, const int32_t *mult,
                         const int32_t *shift, int32_t z_mid, int32_t mid_min, int32_t mid_max, const uint8_t *residual,
                         int64_t ldr, const qnn_add_params *add, uint8_t *C, int64_t ldc, void *workspace,
                         size_t workspace_bytes, void *stream);

qnn_status qnn_qconv2d_add(const uint8_t *x, int N, int H, int W, int Cin, int32_t z_x, const void *w, int Cout, int kh,
                           int kw, int weight_bits, int stride_h, int stride_w, int pad_h, int pad_w,
                           const int32_t *bias, const int32_t *mult, const int32_t *shift, int32_t z_mid,
                           int32_t mid_min, int32_t mid_max, const uint8_t *residual, const qnn_add_params *add,
                           uint8_t *y, void *workspace, size_t workspace_bytes, void *stream);

/* The same layers with asymmetric per-channel weights: column / output channel n carries its own
 * zero-point z_w[n] (Sec. 2.1 affine quantizer at the per-channel granularity of Sec. 2.6; the scheme the
 * post-training experiments of Sec. 3.1 find most accurate).  The sum becomes
 *   sum_k (A[m][k] - z_a) * (B[k][n] - z_w[n])
 * = sum_k A*B - z_a * sum_k B[k][n] - z_w[n] * sum_k A[m][k] + K * z_a * z_w[n]        (eq. 5-6)
 * The activation sums of the third term are shared by all channels: one extra pass over A forms
 * them per output row (for a convolution: over the taps inside the image; padding holds the code
 * z_x and adds nothing), into the caller's workspace (required here: QNN_EINVAL when it is NULL,
 * misaligned or smaller than the workspace query says).
 * z_w: DEVICE int32[N] (resp. [Cout]), each in [-128, 127] for 8-bit and [-8, 7] for 4-bit weights.
 * K (resp. kh*kw*Cin) <= 32768, which keeps |sum| below 2^31.  Everything else as in qnn_qgemm /
 * qnn_qconv2d. */
qnn_status qnn_qgemm_asym(const uint8_t *A, int64_t lda, int32_t z_a, const void *B, int64_t ldb, int b_layout,
                          int weight_bits, const int32_t *z_w, int64_t M, int64_t N, int64_t K, const int32_t *bias,
                          const int32_t *mult, const int32_t *shift, int32_t z_out, int32_t act_min, int32_t act_max,
                          uint8_t *C, int64_t ldc, void *workspace, size_t workspace_bytes, void *stream);

qnn_status qnn_qconv2d_asym(const uint8_t *x, int N, int H, int W, int Cin, int32_t z_x, const void *w, int Cout, int kh,
                            int kw, int weight_bits, const int32_t *z_w, int stride_h, int stride_w, int pad_h, int pad_w,
                            const int32_t *bias, const int32_t *mult, const int32_t *shift, int32_t z_out,
                            int32_t act_min, int32_t act_max, uint8_t *y, void *workspace, size_t workspace_bytes,
                            void *stream);

/* Quantizer parameters from the data, on the device (Sec. 2.5: activation ranges are the minimum and
 * maximum of the tensor, or their moving average across batches; Sec. 2.1 turns a range into scale
 * and zero-point).  No value travels to the host.
 * state: DEVICE, 24 bytes, owned by the caller; xmin / xmax persist between calls (the moving
 *        average), key_min / key_max are work space of the reduction.
 * qnn_minmax: batch range over the FINITE elements of x (NaN and +-inf are skipped; no finite element:
 *   range [0, 0]); momentum == 0: state range = batch range; 0 < momentum < 1:
 *   state.x = momentum * state.x + (1 - momentum) * batch (products and sum each rounded once in
 *   binary64, result rounded to binary32; the caller initialises xmin / xmax before the first such call);
 *   then (scale, zero_point) = qnn_choose_qparams(xmin, xmax, bits), evaluated on the device.
 * qnn_quantize_with: qnn_quantize with scale / zero_point read from state, codes 0..255.
 * qnn_quantize_dynamic: qnn_minmax(momentum 0, 8 bits) followed by qnn_quantize_with.
 * x: DEVICE fp32[n] (read); q: DEVICE uint8[n] (written).  n == 0 is allowed. */
typedef struct qnn_dyn_qparams {
    float scale;
    int32_t zero_point;
    float xmin, xmax;
    uint32_t key_min, key_max;
} qnn_dyn_qparams;

qnn_status qnn_minmax(const float *x, size_t n, float momentum, int bits, qnn_dyn_qparams *state, void *stream);
qnn_status qnn_quantize_with(const float *x, uint8_t *q, size_t n, const qnn_dyn_qparams *state, void *stream);
qnn_status qnn_quantize_dynamic(const float *x, uint8_t *q, size_t n, qnn_dyn_qparams *state, void *stream);

/* Simulated quantization for quantization-aware training (Sec. 2.4).
 * Forward (eq. 12-13): y[i] = dequantize(quantize(x[i])) with the given quantizer and code range
 *   [qmin, qmax] within 0..65535 (0..15 for 4-bit, 0..65535 for 16-bit activations, Sec. 3.3); same
 *   arithmetic as qnn_quantize / qnn_dequantize (qnn_quantize_u16 / qnn_dequantize_u16 beyond a byte), so y
 *   is bit-identical to calling the two.
 * Backward (straight-through estimator, eq. 14-15): grad_x[i] = grad_y[i] if x_min <= x[i] <= x_max, else
 *   0, with x_min = (qmin - zero_point) * scale and x_max = (qmax - zero_point) * scale in binary32
 *   (NaN inputs get no gradient).
 * x, grad_y: DEVICE fp32[n] (read); y, grad_x: DEVICE fp32[n] (written). */
qnn_status qnn_simquant(const float *x, float *y, size_t n, float scale, int32_t zero_point, int32_t qmin, int32_t qmax,
                        void *stream);
qnn_status qnn_simquant_backward(const float *x, const float *grad_y, float *grad_x, size_t n, float scale,
                                 int32_t zero_point, int32_t qmin, int32_t qmax, void *stream);

/* Quantizer and de-quantizer of Sec. 2.1 (eq. 1-3) for codes of up to 16 bits, stored as uint16: the
 * arithmetic of qnn_quantize / qnn_dequantize with [qmin, qmax] within 0..65535 (Sec. 3.3 evaluates
 * 16-bit activations).  x: DEVICE fp32[n]; q: DEVICE uint16[n] (2-byte aligned; 4 elements per lane when x
 * is 16-byte and q 8-byte aligned).  n == 0 is allowed.  QNN_EINVAL as for the byte versions. */
qnn_status qnn_quantize_u16(const float *x, uint16_t *q, size_t n, float scale, int32_t zero_point, int32_t qmin,
                            int32_t qmax, void *stream);
qnn_status qnn_dequantize_u16(const uint16_t *q, float *x, size_t n, float scale, int32_t zero_point, void *stream);

/* Depthwise convolution with a zero-point per channel of the weights (as qnn_qconv2d_asym; one lane per
 * output evaluates sum (x - z_x)(w - z_w[c]) over the taps inside the image directly).  z_w: DEVICE int32[C]. */
qnn_status qnn_qdwconv2d_asym(const uint8_t *x, int N, int H, int W, int C, int32_t z_x, const int8_t *w, int kh, int kw,
                              const int32_t *z_w, int stride_h, int stride_w, int pad_h, int pad_w, const int32_t *bias,
                              const int32_t *mult, const int32_t *shift, int32_t z_out, int32_t act_min, int32_t act_max,
                              uint8_t *y, void *stream);

/* Calibration of the machine for the benchmark (not part of the inference path).
 * qnn_calibrate_mfma: `workgroups` workgroups of 8 waves each issue iters x 4 independent
 *   v_mfma_i32_32x32x32_i8 from registers only (random_operands != 0: a different pseudo-random
 *   byte pattern in every operand register; 0: all bytes equal); *ops (HOST) receives the number of
 *   integer operations the launch performs (2 per multiply-accumulate).  sink: DEVICE int32
 *   [workgroups * 512] (written).
 * qnn_calibrate_copy: dst[0..bytes) = src[0..bytes), 16 bytes per lane and access; bytes % 16 == 0,
 *   both DEVICE pointers 16-byte aligned.
 * qnn_calibrate_rescale: `workgroups` workgroups of 256 lanes each rescale iters x 16 accumulators held in
 *   registers with the instruction sequence of the fused epilogues (RESCALE + clamp + byte packing in its
 *   cheapest exact form); *outputs (HOST) receives the number of accumulators rescaled.  sink: DEVICE int32
 *   [workgroups * 256] (written). */
qnn_status qnn_calibrate_mfma(int workgroups, int iters, int random_operands, int32_t *sink, double *ops, void *stream);
qnn_status qnn_calibrate_copy(const void *src, void *dst, size_t bytes, void *stream);
qnn_status qnn_calibrate_rescale(int workgroups, int iters, int32_t *sink, double *outputs, void *stream);

/* ------------------------------------------------------------------ host-only helpers */

/* Quantizer parameters from a real range, Sec. 2.1: the range is first widened to contain 0,
 * scale = (xmax - xmin) / (2^bits - 1) rounded to binary32, zero_point = round(-xmin / scale)
 * clamped to [0, 2^bits - 1].  A degenerate range gives scale 1, zero_point 0.
 * scale, zero_point: HOST outputs.  2 <= bits <= 16. */
qnn_status qnn_choose_qparams(double xmin, double xmax, int bits, float *scale, int32_t *zero_point);

/* (mult, shift) with real_mult ~= mult * 2^(-31 - shift), mult in [2^30, 2^31); real_mult = 0 or
 * below 2^-32 gives (0, 0); real_mult >= 2^31 is QNN_EINVAL.  HOST outputs. */
qnn_status qnn_quantize_multiplier(double real_mult, int32_t *mult, int32_t *shift);

/* Clamp range of a fused activation in the quantized output domain (Sec. 3.2.1):
 * kind 0 none -> [0,255]; 1 ReLU -> [z_out,255]; 2 ReLU6 -> [z_out, min(255, z_out + round(6/s_out))]. */
qnn_status qnn_act_range(int kind, float s_out, int32_t z_out, int32_t *act_min, int32_t *act_max);

/* The seven integer parameters of qnn_qadd from the three real scales (left_shift = 20). */
qnn_status qnn_qadd_params(double s_a, double s_b, double s_out, int32_t *left_shift, int32_t *mult_a,
                           int32_t *shift_a, int32_t *mult_b, int32_t *shift_b, int32_t *mult_o, int32_t *shift_o);

/* Symmetric per-channel weight quantizer, Sec. 2.2 eq. 7-11 and Sec. 2.6: for each of `channels`
 * kernels of `per_channel` fp32 values, delta[c] = max|w_c| / (2^(bits-1) - 1) (1 if the kernel is
 * all zero) and wq = clamp(round(w / delta[c])), ties away from zero, clamp range
 * [-(2^(bits-1) - 1), 2^(bits-1) - 1] if restricted else [-2^(bits-1), 2^(bits-1) - 1].  bits is 8 or 4.
 * w: HOST fp32[channels*per_channel]; wq: HOST int8 (one value per byte); delta: HOST fp32[channels]. */
qnn_status qnn_quantize_weights(const float *w, size_t channels, size_t per_channel, int bits, int restricted,
                                int8_t *wq, float *delta);

/* Pack n (even) int8 values in [-8,7] two per byte, element 2j in the low nibble.  HOST pointers. */
qnn_status qnn_pack_int4(const int8_t *v, size_t n, uint8_t *packed);

#ifdef __cplusplus
}
#endif
#endif /* QNN_H */
