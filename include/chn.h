/*
 * chn.h -- C ABI of libchn: the array kernels that a define-by-run training step issues to a
 * NumPy-like GPU array layer, written for AMD MI355X (gfx950).
 *
 * The paper (Section "GPU Support by CuPy") describes a GPU ndarray that is a drop-in for
 * numpy.ndarray -- standard dtypes, transpose, reshape, broadcasting -- on which two kinds of kernels
 * run, element-wise maps and reductions (Section "Custom CUDA Kernels"), plus dense products backed
 * by a BLAS.  A training step (Section "On Demand Graph Construction") calls these operation by
 * operation: forward, then each recorded operation's backward once in reverse order, then the
 * optimiser.  This header is that operation set as plain C calls.
 *
 * Conventions that hold for every call
 *   - chn_array describes caller-owned DEVICE memory: shape plus BYTE strides (NumPy convention).
 *     Descriptors live on the host, are read during the call and never retained.
 *   - Strides must be non-negative multiples of the item size.  Stride 0 is allowed on inputs (a
 *     broadcast view) and refused on outputs.
 *   - The library allocates and frees nothing.  Calls that need scratch take a caller-owned device
 *     workspace `ws` of at least chn_*_workspace_bytes(...) bytes, 256-byte aligned.
 *   - Every call validates on the host, enqueues its kernels on `stream` (a hipStream_t; NULL = the
 *     default stream) and returns without synchronising.  Device faults surface at the caller's next
 *     synchronisation.
 *   - Return value: CHN_OK or a negative chn_status; chn_last_error() gives a thread-local detail
 *     string for the most recent failure.  A failing call enqueues nothing.
 *   - Arrays with zero elements are valid: the call returns CHN_OK and does nothing, except that a
 *     reduction over an empty axis writes the fold's identity.
 *   - An output may alias an input only when both descriptors are identical (in-place update);
 *     partially overlapping views are the caller's responsibility.
 *   - Index values are never used as offsets unchecked: a label outside [0, C) is treated like
 *     `ignore_label` (no loss, no gradient, not counted), a token id outside [0, V) gathers a row of
 *     zeros and receives no gradient.  Nothing is reported: the device cannot fail a call.
 */
#ifndef CHN_H_
#define CHN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CHN_MAX_NDIM 8

typedef enum { CHN_F32 = 0, CHN_BF16 = 1, CHN_I32 = 2, CHN_I64 = 3 } chn_dtype;

typedef struct {
  void *data;                    /* device pointer, caller-owned                         */
  int32_t ndim;                  /* 0 .. CHN_MAX_NDIM                                    */
  int64_t shape[CHN_MAX_NDIM];
  int64_t strides[CHN_MAX_NDIM]; /* bytes                                                */
  int32_t dtype;                 /* a chn_dtype                                          */
} chn_array;

typedef int32_t chn_status;
enum {
  CHN_OK = 0,
  CHN_ERR_NULL = -1,      /* a required pointer is NULL                                  */
  CHN_ERR_NDIM = -2,      /* ndim out of range or not what the call needs                */
  CHN_ERR_DTYPE = -3,     /* unsupported or inconsistent dtype combination               */
  CHN_ERR_SHAPE = -4,     /* not broadcastable / inner dimensions differ / wrong output  */
  CHN_ERR_STRIDE = -5,    /* negative, misaligned, zero on an output, or unsupported     */
  CHN_ERR_OP = -6,        /* unknown operation / epilogue code or wrong operand count    */
  CHN_ERR_AXIS = -7,      /* axis out of range                                           */
  CHN_ERR_WORKSPACE = -8, /* workspace missing, misaligned or too small                  */
  CHN_ERR_LAUNCH = -9,    /* the HIP runtime refused a launch                            */
  CHN_ERR_COMPILE = -10   /* a user-defined kernel's snippet does not compile            */
};

typedef void *chn_stream; /* hipStream_t */

/* ---- element-wise map with NumPy broadcasting -------------------------------------------------
 * Section "Custom CUDA Kernels": an element-wise kernel applies one operation to every element;
 * the figure "Example of a user-defined kernel" (my_mad, w = x*y + z) is CHN_OP_MAD.  Operands are
 * right-aligned and size-1 dimensions repeat (Section "GPU Support by CuPy": broadcasting); every
 * input must broadcast to the shape of `out`.  All inputs share one dtype (F32 or BF16); `out` is F32 or
 * BF16; arithmetic is fp32; a BF16 store rounds to nearest even.  Any byte strides are accepted
 * (transposed and sliced views included).  `scalars` is a host array read during the call. */
typedef enum {
  CHN_OP_COPY = 0,  /* out = x                      (1 input; also the dtype cast)               */
  CHN_OP_ADD,       /* x + y                                                                     */
  CHN_OP_SUB,       /* x - y                                                                     */
  CHN_OP_MUL,       /* x * y                                                                     */
  CHN_OP_MAD,       /* x * y + z                    (3 inputs)                                   */
  CHN_OP_MAD_RELU,  /* max(0, x * y + z)            (3 inputs)                                   */
  CHN_OP_RELU,      /* max(0, x)                                                                 */
  CHN_OP_RELU_BWD,  /* gy * [y > 0]                 (inputs gy, y: the forward OUTPUT)           */
  CHN_OP_GELU,      /* 0.5 x (1 + erf(x / sqrt 2))                                               */
  CHN_OP_GELU_BWD,  /* gy * (Phi(z) + z phi(z))     (inputs gy, z: the forward input)            */
  CHN_OP_SCALE,     /* s0 * x                       (1 scalar)                                   */
  CHN_OP_AXPY,      /* x + s0 * y                   (1 scalar)                                   */
  CHN_OP_ADD_RELU,  /* max(0, x + y)                (bias + activation)                          */
  CHN_OP_ADD_GELU,  /* gelu(x + y)                                                               */
  CHN_OP_FILL,      /* s0                           (0 inputs, 1 scalar)                         */
  CHN_OP_SIGMOID,   /* 1 / (1 + exp(-x))                                                         */
  CHN_OP_TANH,      /* tanh(x)                                                                   */
  CHN_OP_SQRT,      /* sqrt(x)                                                                   */
  CHN_OP_EXP,       /* exp(x)                                                                    */
  CHN_OP_GELU_BWD2, /* g * phi(z) (2 - z^2)         (inputs g, z: gelu''(z) = phi(z)(2 - z^2), what a
                       differentiable backward of GELU needs -- Section "Double Backpropagation")  */
  CHN_OP_COUNT_
} chn_op;

chn_status chn_elementwise_broadcast(int op, int n_in, const chn_array *const *in,
                                     const chn_array *out, const float *scalars, int n_scalars,
                                     chn_stream stream);

/* ---- reduction over one axis or several ---------------------------------------------------------
 * Section "Custom CUDA Kernels": a reduction kernel folds elements by a binary operator (sum folds
 * by +).  `axis` may be negative (NumPy style), CHN_AXES(mask) for several axes at once (bit d set =
 * dimension d is folded) or CHN_AXIS_ALL (both defined with the user-defined kernels below).  `out`
 * has the input's shape without the folded axes (keepdims = 0) or with them set to 1 (keepdims != 0).
 * Input F32 or BF16, any byte strides; accumulation is fp32 in a fixed order (bit-reproducible run
 * to run); `out` F32 or BF16.  An empty axis writes 0 (sum) or -inf (max).
 * Several axes are folded one after the other, last first, over fp32 intermediates in the workspace
 * (neighbouring axes of a contiguous array count as one; so does a sum over everything):
 * chn_reduce_axis_workspace_bytes takes the same axis code. */
typedef enum { CHN_REDUCE_SUM = 0, CHN_REDUCE_MAX = 1 } chn_reduce_op;

size_t chn_reduce_axis_workspace_bytes(const chn_array *in, int axis);
/* Index of the largest element along `axis` (the classification example of Section "API Design"
 * reports accuracy: the arg-max of the logits against the labels).  `out`: I32 or I64, contiguous,
 * shaped like chn_reduce_axis's.  Among equal maxima the smallest index wins; a NaN is never
 * selected (a slice of nothing but NaN yields 0).  An empty axis is CHN_ERR_SHAPE.  No workspace. */
chn_status chn_argmax_axis(const chn_array *in, int axis, int keepdims, const chn_array *out,
                           chn_stream stream);
chn_status chn_reduce_axis(int op, const chn_array *in, int axis, int keepdims,
                           const chn_array *out, void *ws, size_t ws_bytes, chn_stream stream);
/* chn_reduce_axis for callers that cannot allocate device memory or bring a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and
 * results (bit for bit) as chn_reduce_axis, but the partial sums of a reduction that is cut into
 * slices live in an array built into the library -- CHN_REDUCE_STATIC_SCRATCH_BYTES of device memory
 * that every GPU the library runs on holds until the process ends -- and the call allocates and frees
 * nothing (the array's device address is looked up once per device, on the first call there).
 * A reduction whose chn_reduce_axis_workspace_bytes exceeds that size is refused with
 * CHN_ERR_WORKSPACE and nothing is launched (the 8192 x 8192 column sums need 2 MiB).  All calls on
 * one GPU share the one array: calls that may overlap there (different streams, different threads)
 * race and must be ordered by the caller; calls on one stream are ordered by the stream.  Nothing in
 * the array has to start at zero: every partial sum that is read has been written by the same call. */
#define CHN_REDUCE_STATIC_SCRATCH_BYTES (8u << 20)
chn_status chn_reduce_axis_static(int op, const chn_array *in, int axis, int keepdims,
                                  const chn_array *out, chn_stream stream);

/* ---- dense product ------------------------------------------------------------------------------
 * C = epilogue(alpha * A B + beta * C).  A (M,K), B (K,N), C (M,N) are 2-d views; a transposed
 * operand is expressed by its strides, so the fully connected layer of the model-definition figure,
 * y = x @ W.T + b with W (n_out, n_in), is A = x, B = the (n_in, n_out) view of W with strides
 * swapped, epilogue CHN_EPI_BIAS.  A and B must each have one unit-stride dimension; C (and
 * `preact_out`, `aux`) must be row-major (unit stride along N).
 * dtypes: A,B F32 -> C F32 (fp32 matrix cores); A,B BF16 -> C BF16 or F32 (fp32 accumulation).
 * Epilogue, applied to v = alpha*acc + beta*C in fp32 before the single final rounding:
 *   BIAS       v + bias[n]                         bias (N,) F32
 *   BIAS_RELU  max(0, v + bias[n])
 *   BIAS_GELU  gelu(v + bias[n]); when preact_out != NULL it receives v + bias[n] (same dtype and
 *              shape as C) for the backward pass
 *   RELU_BWD   v * [aux > 0]                       aux (M,N): the retained forward output
 *   GELU_BWD   v * gelu'(aux)                      aux (M,N): the retained pre-activation
 *              With these two, preact_out != NULL asks for a second result: an F32 array of shape
 *              (M/128, N) whose row r receives the column sums of rows 128r .. 128r+127 of C, taken
 *              over the values as stored (after rounding to C's dtype), in a fixed order.  C is the
 *              gradient with respect to a layer's pre-activation, so the column sum of these few
 *              rows is that layer's bias gradient and no second pass over C is needed.  Requires M
 *              and N to be multiples of 256, beta == 0, 16-byte aligned rows of C, aux and the sums,
 *              and operands whose rows allow 8-byte pieces (CHN_ERR_SHAPE / OP / STRIDE otherwise);
 *              the product then runs on 256x256 tiles, uncut.
 *   BF16_COPY  v, and preact_out (M,N) BF16 receives v rounded to bfloat16 as well (C must be F32):
 *              with alpha = -lr, beta = 1 and C the fp32 master weights, the weight-gradient product
 *              of a layer becomes the SGD update W <- W - lr * dW of Section "Background and
 *              Motivation"'s training loop together with the refresh of the bf16 working copy, and
 *              the gradient never travels through memory
 * Unused optional arguments are NULL.  beta != 0 reads C before writing it.
 * Operands are read in aligned pieces of up to 16 bytes.  Where the unit stride of A runs along M (of
 * B: along N) and the rows are 8- or 16-byte aligned, the last piece of a row may reach past the row's
 * last element, by less than the piece and never out of the piece's own aligned 16 bytes: what it
 * brings (row padding, or the start of the next row) is multiplied into rows or columns that are not
 * part of C and is never stored.  A short unit-stride extent that is not a multiple of 8 bytes (a
 * gradient with 10 classes, say) is therefore best given rows padded to 16 bytes.
 * gelu / gelu' in the epilogue use a five-term rational erf (absolute error below 1.5e-7 in Phi) when C
 * is F32; when C is BF16 they are odd polynomials of the clamped argument (absolute error below 7e-5 in
 * Phi and 1.6e-4 in gelu': under the rounding of the bfloat16 result except in the negative tail, where
 * it is an absolute 2e-4 |x| on values smaller than 0.1).
 * Workspace: optional.  chn_gemm_workspace_bytes returns what a product with few output tiles and a
 * long K would use to be cut along K (fp32 partial sums per cut, added in a fixed order by a second
 * kernel: bit-reproducible); `ws` is device memory, 256-byte aligned, owned by the caller and free
 * again when the call's work on `stream` is done.  With ws == NULL, too small or misaligned the
 * product runs uncut -- same result up to summation order, possibly slower.
 * Errors (nothing is launched): CHN_ERR_NULL / NDIM / DTYPE / SHAPE / STRIDE for malformed or
 * mismatched views (a bias or aux that the epilogue needs and that is NULL: CHN_ERR_NULL), CHN_ERR_OP
 * for an unknown epilogue or a preact_out given to the NONE / BIAS / BIAS_RELU epilogues
 * (BF16_COPY requires it), CHN_ERR_LAUNCH
 * if the launch itself is refused.  M == 0 or N == 0 is a no-op; K == 0 applies the
 * epilogue to beta * C. */
typedef enum {
  CHN_EPI_NONE = 0,
  CHN_EPI_BIAS,
  CHN_EPI_BIAS_RELU,
  CHN_EPI_BIAS_GELU,
  CHN_EPI_RELU_BWD,
  CHN_EPI_GELU_BWD,
  CHN_EPI_BF16_COPY,
  CHN_EPI_COUNT_
} chn_epilogue;

size_t chn_gemm_workspace_bytes(const chn_array *A, const chn_array *B, const chn_array *C);
chn_status chn_gemm(const chn_array *A, const chn_array *B, const chn_array *C, float alpha,
                    float beta, int epilogue, const chn_array *bias, const chn_array *aux,
                    const chn_array *preact_out, void *ws, size_t ws_bytes, chn_stream stream);

/* ---- LSTM cell ------------------------------------------------------------------------------------
 * The paper names LSTMs as a motivating model class (Section "Introduction") and an RNN language
 * model as an application; it prints no equations, so the cell is the textbook one without
 * peepholes.  z (B,4H) holds the gate pre-activations x W + h U, gate blocks of width H along the
 * last axis in the order i, f, g, o; `bias` (4H,) or NULL is added to z.
 *   i,f,o = sigmoid(z_i,z_f,z_o)  g = tanh(z_g)  c = f*c_prev + i*g  h = o*tanh(c)
 * c_prev, c, h are (B,H); `gates` (B,4H) or NULL receives the activated i,f,g,o for the backward.
 * F32, rows may be pitched (stride[0] free), unit stride along the last axis.  Mixed precision: the
 * arrays that feed matrix products -- h here, dh and dz in the backward -- may be BF16 (stores round to
 * nearest even); z, gates and the cell state are always F32. */
chn_status chn_lstm_fwd(const chn_array *z, const chn_array *bias, const chn_array *c_prev,
                        const chn_array *c, const chn_array *h, const chn_array *gates,
                        chn_stream stream);

/* Backward from retained OUTPUTS only (Section "Function-wise Local Memory Usage Reduction": an
 * operation such as tanh can compute its gradient from its output): inputs are the activated
 * `gates`, c_prev, c, the incoming dh and dc_next (NULL = zero); outputs dz (B,4H), dc_prev (B,H).
 *   do = dh*tanh(c)  dc = dc_next + dh*o*(1-tanh(c)^2)  di = dc*g  dg = dc*i  df = dc*c_prev
 *   dc_prev = dc*f   dz_i = di*i(1-i)  dz_f = df*f(1-f)  dz_g = dg*(1-g^2)  dz_o = do*o(1-o) */
chn_status chn_lstm_bwd(const chn_array *gates, const chn_array *c_prev, const chn_array *c,
                        const chn_array *dh, const chn_array *dc_next, const chn_array *dz,
                        const chn_array *dc_prev, chn_stream stream);

/* One time step of the recurrent layer in one launch: the recurrent product and the cell fused.
 * Forward:  z = zx + h_prev U (+ bias), then the cell above.  zx (B,4H) F32 holds the input part
 * x W of this step; h_prev (B,H) and Ut (4H,H) -- the TRANSPOSE of the recurrent matrix U (H,4H),
 * so that both operands are unit-stride along the contraction -- share one dtype, F32 or BF16; h
 * is written in that dtype; c_prev, c, gates F32.  z itself is not stored.
 * Backward: dh <- dh + dz_next U^T (dz_next (B,4H) and U (H,4H) in dh's dtype; dz_next NULL for the
 * last step: dh is used as it is), stored back into `dh` (the total gradient of h_t, rounded to
 * BF16 in mixed precision -- the rounded value is what the cell sees), then the cell's backward
 * above: dz (B,4H) in dh's dtype, dc_prev F32.
 * Requirements beyond the unfused calls: H a multiple of 32 (pad with inert units), rows of
 * h_prev, Ut, dz_next and U on 16-byte boundaries; otherwise CHN_ERR_SHAPE / CHN_ERR_STRIDE and
 * the caller uses chn_gemm + chn_lstm_fwd / chn_lstm_bwd.  Sums run in fp32 on the matrix cores
 * in an order that differs from chn_gemm's; results agree within the product tolerance. */
chn_status chn_lstm_step_fwd(const chn_array *zx, const chn_array *h_prev, const chn_array *Ut,
                             const chn_array *bias, const chn_array *c_prev, const chn_array *c,
                             const chn_array *h, const chn_array *gates, chn_stream stream);
chn_status chn_lstm_step_bwd(const chn_array *dz_next, const chn_array *U, const chn_array *dh,
                             const chn_array *gates, const chn_array *c_prev, const chn_array *c,
                             const chn_array *dc_next, const chn_array *dz,
                             const chn_array *dc_prev, chn_stream stream);

/* The forward pass of the recurrent layer over a whole sequence in ONE launch (Sec. 2.2's loop over time,
 * Sec. 3.2's NStepLSTM): for t = 0 .. n_steps-1,
 *   block t+1 of Hs, Cs = cell(zx block t + block t of Hs . Ut^T + bias, block t of Cs),  block t of gates.
 * zx (n_steps*B, 4H) F32; Ut (4H, H) F32 or BF16; bias (4H) F32 or NULL; Hs ((n_steps+1)*B, H) of Ut's type
 * and Cs ((n_steps+1)*B, H) F32 with block 0 holding the initial state (read) and blocks 1.. written;
 * gates (n_steps*B, 4H) F32 or NULL.  All device, row-major with unit inner stride, rows of Hs and Ut on
 * 16-byte boundaries.  Same formulas as n_steps calls of chn_lstm_step_fwd (fp32 sums on the matrix cores,
 * the contraction cut in four; the gate activations on the hardware's exponential and reciprocal, relative
 * error a few 1e-7; agrees with them within the product tolerance).
 *
 * The grid stays on the device for the whole sequence - (H/8) x ceil(B/64) workgroups, each holding its rows
 * of Ut in LDS - and exchanges h between steps through device memory, so every workgroup must be resident at
 * once: H % 8 == 0 (BF16: % 16), a row of h of at most 3072 bytes (H <= 768 F32, 1536 BF16) and no more
 * workgroups than the device has compute units; otherwise CHN_ERR_SHAPE and the caller uses the per-step
 * calls.  ws: chn_lstm_seq_workspace_bytes(B) bytes, 256-byte aligned, the library's until the work on
 * `stream` is done.  A workgroup waits for the others a bounded number of polls (chn_lstm_seq_spin_limit;
 * the default is worth seconds).  If a wait runs out - another kernel holds compute units the grid needs -
 * every workgroup leaves, the outputs are incomplete, and the first 4 bytes of ws read 1 instead of 0 once
 * the stream is synchronised: the caller checks that word and repeats the work with the per-step calls.
 * Launch it on one stream at a time per device. */
size_t chn_lstm_seq_workspace_bytes(int64_t batch);
/* CHN_OK if chn_lstm_seq_fwd takes a batch of `batch` rows and `hidden` units of `dtype` (CHN_F32 / CHN_BF16)
 * on the current device, else the status it would return (chn_last_error says why): ask before planning. */
chn_status chn_lstm_seq_supported(int64_t batch, int64_t hidden, int dtype);
chn_status chn_lstm_seq_fwd(const chn_array *zx, const chn_array *Ut, const chn_array *bias, const chn_array *Hs,
                            const chn_array *Cs, const chn_array *gates, int64_t n_steps, void *ws, size_t ws_bytes,
                            chn_stream stream);
/* Back-propagation through time over the whole sequence in ONE launch (Sec. 2.2: the backward walk over the
 * graph the loop over time built), last step first: for t = n_steps-1 .. 0,
 *   block t of dHs <- block t of dHs + (block t+1 of dZ) . U^T        (nothing added for the last step)
 *   block t of dZ, dc <- cell backward(block t of gates, blocks t and t+1 of Cs, block t of dHs, dc)
 * starting from dc = dc_last (or 0 if NULL); dc0 receives the gradient of the initial cell state.
 * U (H, 4H) F32 or BF16; dHs (n_steps*B, H) and dZ (n_steps*B, 4H) of U's type (dHs in: the gradient reaching
 * each h_t from above; out: the total); gates (n_steps*B, 4H), Cs ((n_steps+1)*B, H), dc_last, dc0 (B, H) F32.
 * All device, row-major, unit inner stride; rows of U on 16-byte, of dZ on 8-byte boundaries.  Same arithmetic
 * as the chain of chn_lstm_step_bwd calls: in mixed precision the cell sees the bf16-rounded total dh and the
 * product reads the bf16-rounded dz; the fp32 sums run in another order (64 gate columns per workgroup on the
 * matrix cores, then the H/16 partial sums in workgroup order).
 *
 * Resident grid of (H/16) x ceil(B/32) workgroups, each with its columns of U in registers: H % 16 == 0,
 * H <= 768 (F32) / 1536 (BF16), no more workgroups than compute units; otherwise CHN_ERR_SHAPE
 * (chn_lstm_seq_bwd_supported asks beforehand).  ws: chn_lstm_seq_bwd_workspace_bytes(B, H) bytes (the partial
 * sums the workgroups exchange: 2 * ceil(B/32) * (H/16)^2 * 2 KiB), 256-byte aligned.  Waits, the status word
 * in the first 4 bytes of ws and chn_lstm_seq_spin_limit as for chn_lstm_seq_fwd. */
chn_status chn_lstm_seq_bwd_supported(int64_t batch, int64_t hidden, int dtype);
size_t chn_lstm_seq_bwd_workspace_bytes(int64_t batch, int64_t hidden);
chn_status chn_lstm_seq_bwd(const chn_array *U, const chn_array *dHs, const chn_array *gates, const chn_array *Cs,
                            const chn_array *dc_last, const chn_array *dZ, const chn_array *dc0, int64_t n_steps,
                            void *ws, size_t ws_bytes, chn_stream stream);
/* Number of polls after which a waiting workgroup of chn_lstm_seq_fwd / _bwd gives up (process-wide, >= 0; the
 * default is 2^20).  With 0 the first wait gives up without looking: tests use it to see the status word
 * raised and the kernel end after its first step. */
void chn_lstm_seq_spin_limit(int64_t polls);

/* ---- softmax cross-entropy ------------------------------------------------------------------------
 * The classifier loss of the paper's MNIST example (Section "API Design"); textbook definition.
 * logits (N,C) F32 or BF16, row-major; labels (N,) I32 or I64.  Rows whose label equals
 * `ignore_label` contribute no loss and no gradient and are not counted in N_valid.
 *   lse_n = max_c z + log sum_c exp(z - max)   loss_n = lse_n - z[n, label_n]
 *   loss_mean = (1/N_valid) sum_n loss_n       (0 when N_valid = 0)
 * loss_mean: 0-d (or 1-element) F32.  loss_rows, lse: (N,) F32 or NULL.
 * Workspace: chn_softmax_ce_workspace_bytes(N). */
size_t chn_softmax_ce_workspace_bytes(int64_t n_rows);
chn_status chn_softmax_ce_fwd(const chn_array *logits, const chn_array *labels,
                              int64_t ignore_label, const chn_array *loss_mean,
                              const chn_array *loss_rows, const chn_array *lse, void *ws,
                              size_t ws_bytes, chn_stream stream);

/* dlogits[n,c] = (upstream / N_valid) * (softmax(z)[n,c] - [c == label_n]); ignored rows get 0.
 * `lse` (N,) F32 from the forward, or NULL to recompute it.  dlogits (N,C) F32 or BF16 and may be
 * the logits array itself (in place). */
chn_status chn_softmax_ce_bwd(const chn_array *logits, const chn_array *labels,
                              int64_t ignore_label, const chn_array *lse, float upstream,
                              const chn_array *dlogits, void *ws, size_t ws_bytes,
                              chn_stream stream);

/* The derivative of chn_softmax_ce_bwd, for gradients of gradients (Section "Double Backpropagation":
 * a backward pass that is itself differentiated).  With G = chn_softmax_ce_bwd(logits, labels, upstream)
 * and gg (N,C) the gradient that reaches G:
 *   dlogits[n,c] = (upstream / N_valid) p[n,c] (gg[n,c] - sum_k p[n,k] gg[n,k])   (0 on ignored rows)
 *   dupstream    = (1 / N_valid) sum over valid n, all c of gg[n,c] (p[n,c] - [c == label_n])
 * p = softmax(logits); dupstream: a single F32 value or NULL.  F32 only; `lse` as above; workspace:
 * chn_softmax_ce_workspace_bytes(N). */
chn_status chn_softmax_ce_bwd2(const chn_array *logits, const chn_array *labels, int64_t ignore_label,
                               const chn_array *lse, float upstream, const chn_array *gg,
                               const chn_array *dlogits, const chn_array *dupstream, void *ws,
                               size_t ws_bytes, chn_stream stream);

/* Both of the above in one call, for a training step, where the gradient follows the loss at once:
 * loss_mean, lse (or NULL) and dlogits as defined there, the logits read from memory once.  dlogits
 * may be the logits array itself (same dtype and row pitch).  A problem of at most 64 classes and
 * 8192 rows runs as a single launch of a single workgroup and needs no workspace; otherwise the
 * workspace is that of chn_softmax_ce_fwd.  Errors as for the two separate calls. */
chn_status chn_softmax_ce_fwd_bwd(const chn_array *logits, const chn_array *labels,
                                  int64_t ignore_label, const chn_array *loss_mean,
                                  const chn_array *lse, float upstream, const chn_array *dlogits,
                                  void *ws, size_t ws_bytes, chn_stream stream);

/* ---- optimiser --------------------------------------------------------------------------------------
 * Stochastic gradient descent (Section "Background and Motivation" names it as the optimiser of the
 * run phase): param <- param - lr * grad, no momentum, decay or clipping.  param, grad: F32,
 * contiguous, same shape.  `lowp_copy` (BF16, same shape, contiguous) or NULL receives the updated
 * value rounded to nearest even: the working copy of a mixed-precision master weight. */
chn_status chn_sgd_update(const chn_array *param, const chn_array *grad, float lr,
                          const chn_array *lowp_copy, chn_stream stream);

/* The same update for `n` tensors (a whole model's parameter set) in as few launches as the kernel
 * argument space allows (40 tensors per launch).  lowp_copies may be NULL, and so may its entries. */
chn_status chn_sgd_update_multi(int n, const chn_array *const *params,
                                const chn_array *const *grads, float lr,
                                const chn_array *const *lowp_copies, chn_stream stream);

/* Adam (the paper names it as an optimiser choice in the code figure of Section "Distributed Parallel
 * Training"; the update is Algorithm 1 of Kingma & Ba, "Adam: A Method for Stochastic Optimization"):
 *   m <- beta1 m + (1 - beta1) g        v <- beta2 v + (1 - beta2) g^2
 *   param <- param - lr * (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps)
 * for `n` tensors at once.  params, grads, ms, vs: F32, contiguous, same shape per tensor; m and v
 * are the caller's state, zero before the first call; `step` counts calls from 1.  The
 * hyper-parameters are doubles: 1 - beta and the bias corrections are formed on the host in double
 * precision and rounded to fp32 once.  lowp_copies as for chn_sgd_update_multi.
 * Errors: CHN_ERR_OP for step < 1 or a beta outside [0, 1); otherwise as for chn_sgd_update_multi. */
chn_status chn_adam_update_multi(int n, const chn_array *const *params,
                                 const chn_array *const *grads, const chn_array *const *ms,
                                 const chn_array *const *vs, double lr, double beta1, double beta2,
                                 double eps, int64_t step, const chn_array *const *lowp_copies,
                                 chn_stream stream);

/* ---- embedding ----------------------------------------------------------------------------------------
 * Array indexing of the ndarray layer (Section "GPU Support by CuPy") as the language model uses it:
 * out[n,:] = table[ids[n],:] (bit copies), and its gradient
 * dtable[v,:] = (accumulate ? dtable[v,:] : 0) + sum over n with ids[n] == v of dout[n,:],
 * summed in increasing n (bit-reproducible).  table/dtable (V,D) F32 or BF16 (fwd) / F32 (bwd),
 * ids (N,) I32 or I64, out/dout (N,D); row-major with unit inner stride. */
chn_status chn_embed_fwd(const chn_array *table, const chn_array *ids, const chn_array *out,
                         chn_stream stream);
chn_status chn_embed_bwd(const chn_array *ids, const chn_array *dout, const chn_array *dtable,
                         int accumulate, chn_stream stream);

/* ---- user-defined kernels ----------------------------------------------------------------------------
 * Section "Custom CUDA Kernels" and the figure "Example of a user-defined kernel": a kernel is
 * declared by a list of input parameters, a list of output parameters ("<type> <name>", comma
 * separated), C++ snippets over those names and a kernel name; the library wraps the snippets into
 * a complete kernel, compiles it at run time (hipRTC, for the architecture of the current device),
 * and caches the code object in memory and on disk so that later runs do not compile again.
 * Types: float32, bfloat16, int32, int64, or any other identifier, which is a TYPE PARAMETER (the
 * paper's generic types): it is bound by the dtype of the arrays passed for it, all parameters that
 * share it must receive one dtype, and one kernel object serves every binding.  Inside a snippet a
 * parameter has its COMPUTE type -- float for float32 and bfloat16 arrays (a bfloat16 store rounds
 * to nearest even), int, long long -- and a type parameter names that compute type.
 *
 * Objects: chn_*_kernel_create parses and checks the declaration (nothing is compiled yet) and
 * returns a host object owned by the caller until chn_user_kernel_destroy.  These objects are the
 * one place where the library allocates: host memory for the object, and device code memory when a
 * specialisation is loaded; a launch of an already loaded specialisation allocates nothing.  A
 * kernel object may be used from several threads (calls on one object are serialised).
 *
 * Arguments of a call: `in[i]` is the array for input parameter i, or NULL when that parameter is
 * a SCALAR, whose value is then the next entry of `scalars` (host doubles, converted to the
 * parameter's compute type; a type parameter used only by scalars is an error).  Inputs broadcast
 * NumPy-style; any non-negative byte strides.
 *
 * Element-wise kernel: `operation` is a statement list that assigns every output name, e.g.
 * "w = x * y + z"; it runs once per element of the outputs (all outputs share one shape, every
 * input broadcasts to it).  Also visible: `i`, the C-order flat index of the element (long long).
 *
 * Reduction kernel: the value map_expr (over the input names) of every element is folded by
 * reduce_expr, an expression over `a` and `b`, starting from `identity`; post_map_expr is a
 * statement list that assigns every output from the folded value `a` (scalar parameters are
 * visible too).  The fold runs in the compute type of the first output, over one axis (negative
 * counts from the end), over several (CHN_AXES(mask), dimensions of the broadcast input shape) or
 * over all of them (CHN_AXIS_ALL); outputs have the common input shape
 * without the reduced dimensions (keepdims: with them set to 1).  reduce_expr must be associative
 * and commutative; the order of the fold is fixed for given shapes (bit-reproducible).  An empty
 * reduced range yields post_map(identity).  Workspace as for chn_reduce_axis.
 *
 * chn_*_kernel_prepare compiles (or fetches) the specialisation a call with these descriptors
 * would use without loading or launching it -- it needs no GPU once an architecture is configured.
 * chn_user_kernel_config: `cache_dir` (default $CHN_KERNEL_CACHE_DIR, else ~/.cache/libchn/kernels)
 * and `arch` (default: the current device's, e.g. "gfx950"); NULL keeps a setting, "" restores the
 * default.  Cache files are
 * named by a digest of the generated source, the architecture, the compiler version and the library
 * version, and written atomically; an unwritable cache is not an error.  Without a configured
 * directory and without $HOME there is no disk cache; directories are created with mode 0700 and a
 * cached file is used only when it belongs to the calling user and is writable by nobody else.
 * Errors: CHN_ERR_OP (malformed declaration, wrong argument count), CHN_ERR_DTYPE (array dtype
 * against the declaration, inconsistent binding of a type parameter), CHN_ERR_SHAPE, CHN_ERR_AXIS,
 * CHN_ERR_WORKSPACE, CHN_ERR_COMPILE (chn_last_error holds the compiler's first error),
 * CHN_ERR_LAUNCH.  A failing call enqueues nothing. */
typedef struct chn_user_kernel chn_user_kernel;
#define CHN_AXIS_ALL (-1000)
#define CHN_AXES(mask) (0x40000000 + (mask)) /* several axes at once: bit d set = dimension d is reduced */

chn_status chn_user_kernel_config(const char *cache_dir, const char *arch);
/* process-wide counters: compiler runs, code objects found on disk, found in memory */
void chn_user_kernel_stats(long long *compiles, long long *disk_hits, long long *memory_hits);
void chn_user_kernel_destroy(chn_user_kernel *k);

chn_status chn_elementwise_kernel_create(const char *in_params, const char *out_params,
                                         const char *operation, const char *name,
                                         const char *preamble /* or NULL: code placed before the kernel */,
                                         chn_user_kernel **out);
chn_status chn_elementwise_kernel_prepare(chn_user_kernel *k, int n_in, const chn_array *const *in,
                                          int n_out, const chn_array *const *out);
chn_status chn_elementwise_kernel_launch(chn_user_kernel *k, int n_in, const chn_array *const *in,
                                         int n_out, const chn_array *const *out,
                                         const double *scalars, chn_stream stream);

chn_status chn_reduction_kernel_create(const char *in_params, const char *out_params,
                                       const char *map_expr, const char *reduce_expr,
                                       const char *post_map_expr, const char *identity,
                                       const char *name, const char *preamble,
                                       chn_user_kernel **out);
size_t chn_reduction_kernel_workspace_bytes(chn_user_kernel *k, int n_in, const chn_array *const *in,
                                            int n_out, const chn_array *const *out, int axis,
                                            int keepdims);
chn_status chn_reduction_kernel_prepare(chn_user_kernel *k, int n_in, const chn_array *const *in,
                                        int n_out, const chn_array *const *out, int axis,
                                        int keepdims);
chn_status chn_reduction_kernel_launch(chn_user_kernel *k, int n_in, const chn_array *const *in,
                                       int n_out, const chn_array *const *out, const double *scalars,
                                       int axis, int keepdims, void *ws, size_t ws_bytes,
                                       chn_stream stream);
/* The generated source of the specialisation a call would use (axis/keepdims: reductions only).
 * Copies at most buf_bytes - 1 characters plus a terminator; *needed (if not NULL) receives the
 * full size including the terminator. */
chn_status chn_user_kernel_source(chn_user_kernel *k, int n_in, const chn_array *const *in, int n_out,
                                  const chn_array *const *out, int axis, int keepdims, char *buf,
                                  size_t buf_bytes, size_t *needed);

/* ---- diagnostics ---------------------------------------------------------------------------------------- */
const char *chn_status_string(chn_status status);
const char *chn_last_error(void); /* thread-local, valid until the next failing call on the thread */
int chn_version(void);

/* Host-only query used by tests: which kernel family a call would take, without launching.
 * Returns a small integer code (>= 0) or a negative chn_status.  Element-wise families:
 * 0 flat contiguous/row-broadcast, 1 pitched rows, 2 tile-transposed, 3 general strided. */
int chn_elementwise_plan(int op, int n_in, const chn_array *const *in, const chn_array *out);
/* The same for chn_gemm: bits 0-1 macro tile (0: 64x64, 1: 128x128, 2: 256x256, 3: 256x128 - bfloat16
 * products with both operands unit-stride along K whose N is too small for 256 blocks of the square tile),
 * bit 2 set when a kernel that copies operand tiles straight from global memory into LDS is taken, bit 3 when that
 * is the kernel that works on the tile with eight waves (bfloat16 products), bits 4 and up the number of
 * K splits (1 = none;
 * have_workspace = 0 plans as chn_gemm does without workspace). */
int chn_gemm_plan(const chn_array *A, const chn_array *B, const chn_array *C, int have_workspace);
/* Test hook: replace the planner's choice for every later chn_gemm / chn_gemm_plan of the process.
 * tile: 0 .. 3 as above, or -1 for the planner's own; splits: a number of K splits >= 1 (used when a
 * workspace allows it), or -1; direct_copy: 0 keeps products off the direct-copy kernels, -1 or 1 lets
 * the planner take them where they fit, 2 / 3 additionally fix the four-wave / eight-wave kernel.  A forced value that the operands do not allow (the large tiles
 * need 8-byte pieces) is ignored.  Results do not depend on the plan beyond summation order; the tests
 * use this to run short products on the large tiles.  (-1, -1, -1) restores normal planning. */
void chn_gemm_plan_override(int tile, int splits, int direct_copy);

#ifdef __cplusplus
}
#endif
#endif /* CHN_H_ */
