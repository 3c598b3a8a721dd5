/*
 * ffint8 — C-ABI of the FF-INT8 layer-local training step for AMD MI355X (gfx950).
 *
 * The operations follow "FF-INT8: Efficient Forward-Forward DNN Training on Edge
 * Devices with INT8 Precision" (arXiv 2506.22771): Section IV-B (single-layer
 * dataflow), Eq. (1)/(2) (losses), Section IV-C with Eq. (3)/(4) and Algorithm 1
 * (look-ahead, one forward pass that updates every layer), Section V-A
 * (theta = 2.0, lambda schedule).
 *
 * Conventions common to every entry point
 *  - Every data pointer is a DEVICE pointer unless marked [host].  Descriptors
 *    (ff_layer_desc, ff_net_desc, ff_net_state and the pointer arrays inside
 *    ff_net_state) are [host] memory.
 *  - The caller owns every buffer.  The library allocates and frees no device
 *    memory and keeps no pointer after a call returns.  (Host-side HIP objects
 *    it does create, once and for the life of the process: two streams and
 *    three events per device on the first ff_train_step that runs update
 *    chains on several streams, see FF_LAUNCH_LANES; events of the optional
 *    timing instrumentation at the end of this file, off unless
 *    ff_timing_enable is called.)
 *  - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *    the default stream).  Calls return without synchronising; scalars that are
 *    produced on the device (scales, losses) stay on the device.
 *  - Arguments, shapes and the launch limits of the kernels (FF_ERR_UNSUPPORTED
 *    for sizes beyond them: a tensor of 2^32 elements or more, more than
 *    8 388 480 rows in a quantised matrix, more than 65535 output features or
 *    channels) are validated on the host before anything is launched; on such
 *    an error nothing has been enqueued and no output has been touched.
 *    FF_ERR_HIP reports a failure of the HIP runtime itself (a launch that the
 *    runtime rejects); kernels enqueued before it have run.  The library never
 *    throws, aborts or prints.
 *  - int8 matrices are row-major with a row pitch of ff_pitch(cols) bytes:
 *    cols rounded up to 16, and to 128 for rows longer than 512 bytes (those
 *    then start on cache lines, which the contraction's 128-byte copies want;
 *    784 -> 896, 2000 -> 2048).  The pad bytes of every int8 tensor the library
 *    WRITES are zero, and every int8 tensor it READS must have zero pad bytes
 *    up to cols rounded up to 16 (nothing reads a row beyond that).
 *    int32 matrices are row-major with a row pitch of ff_pitch32(cols)
 *    elements (cols rounded up to 4).  fp32 tensors are contiguous.
 *  - Base addresses: int8 / int32 / workspace buffers 16-byte aligned
 *    (FF_ERR_ALIGN otherwise); fp32 buffers 4-byte aligned.
 *  - Determinism: equal inputs and equal (seed, stream_tag / step) give
 *    bit-identical outputs on every run; all cross-workgroup accumulations are
 *    integer sums or maxima.
 *  - In the default reading there is no input-gradient output: the method
 *    never forms g^A (Section IV-B).  Only the FF_LOOKAHEAD_CHAIN variant, which
 *    takes Eq. (4) as an exact derivative, has one (ff_layer_input_grad).
 */
#ifndef FFINT8_H
#define FFINT8_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t ff_status;
enum {
    FF_OK = 0,
    FF_ERR_INVALID_ARG = -1,    /* null pointer, negative size, bad enum value        */
    FF_ERR_SHAPE = -2,          /* inconsistent or unsupported shape                  */
    FF_ERR_ALIGN = -3,          /* a buffer is not aligned as required                */
    FF_ERR_WORKSPACE = -4,      /* workspace too small                                */
    FF_ERR_OVERFLOW_BOUND = -5, /* an int32 accumulator could overflow for this shape */
    FF_ERR_UNSUPPORTED = -6,    /* valid request this build does not implement        */
    FF_ERR_HIP = -7             /* a HIP runtime call failed                          */
};
enum { FF_ROUND_NEAREST_EVEN = 0, FF_ROUND_STOCHASTIC = 1 };
enum { FF_PASS_POS = +1, FF_PASS_NEG = -1 };
enum { FF_DENSE = 0, FF_CONV2D = 1, FF_DWCONV2D = 2 };

/* Stochastic-rounding stream kinds used by ff_train_step (see ff_stream_tag). */
enum { FF_KIND_ACT = 0, FF_KIND_GRAD = 1, FF_KIND_CHAIN = 2 };

/* Smallest workspace accepted by the single-operation entry points. */
#define FF_WS_MIN_BYTES 1024u

/* One FF layer.  kind FF_DENSE uses batch / in_features / out_features; kind FF_CONV2D
 * uses batch, H, W, C_in, C_out, ksize (1 or 3), stride (1 or 2), pad (= ksize/2),
 * input NHWC, weights [C_out][ksize][ksize][C_in].
 * kind FF_DWCONV2D is a depthwise convolution (one ksize x ksize filter per channel): C_out == C_in, ksize 3,
 * stride 1 or 2, pad 1; weights [C][ksize][ksize], i.e. a [N = C, K = ksize^2] matrix; a_q NHWC as for
 * FF_CONV2D; w_q int8 [C, ff_pitch(ksize^2)].
 * batch = samples in ONE pass (positive or negative).
 * relu: 1 = activities are ReLU(s*acc) (the default reading), 0 = identity.
 * l2norm_out: 1 = the input handed to the next layer is y / ||y||_2 per sample. */
typedef struct {
    int32_t kind, batch, in_features, out_features;
    int32_t H, W, C_in, C_out, ksize, stride, pad;
    int32_t relu, l2norm_out;
    /* Basic residual blocks in ff_train_step (all zero = a plain chain; see "Residual blocks" below). */
    int32_t input_back; /* the layer input is the output of layer i-1-input_back (0 or 1) */
    int32_t role;       /* FF_ROLE_LAYER or FF_ROLE_PROJECTION */
    int32_t skip;       /* FF_SKIP_NONE, FF_SKIP_IDENTITY or FF_SKIP_PROJECTION */
} ff_layer_desc;

/* Residual blocks (the paper's Section IV-C names ResNet-style blocks and gives no mechanics; this is the
 * reading built here).  A basic block is conv1, conv2 and, when the shape changes, a 1x1 projection of the
 * block input, listed as [projection,] conv1, conv2:
 *   projection  role = FF_ROLE_PROJECTION: contraction only; no activity, goodness, loss or output of its own
 *               (its rows of `loss` and `goodness` are 0).  relu and l2norm_out must be 0.
 *   conv1       an ordinary layer; input_back = 1 when a projection precedes it (both read the block input).
 *   conv2       skip = FF_SKIP_IDENTITY:   y = act(s*acc + s_x * x_q), x_q = int8 input of layer i-1, or
 *               skip = FF_SKIP_PROJECTION: y = act(s*acc + s_p * acc of layer i-2).
 *               y is the block output: the goodness, the loss and the local gradient 2*c*y of this layer are
 *               taken on it, it is the input of the layers that follow, and the projection is updated with
 *               the same int8 local gradient.  Goodness: with amax = max|y| over the pass,
 *               G = fp32(sum floor((y/amax)^2 * 2^40) * 2^-40 * amax^2) (an integer sum: order-free).
 *               C_out % 4 == 0, l2norm_out == 0. */
enum { FF_ROLE_LAYER = 0, FF_ROLE_PROJECTION = 1 };
enum { FF_SKIP_NONE = 0, FF_SKIP_IDENTITY = 1, FF_SKIP_PROJECTION = 2 };

/* A stack of layers trained together by ff_train_step. [host]
 * Consecutive layers must fit: dense K = previous N; convolution H, W, C_in = previous H_out, W_out, C_out; a dense
 * layer after a convolution reads its NHWC output flattened (in_features = H_out * W_out * C_out, C_out % 4 == 0).
 * A convolution after a dense layer is FF_ERR_UNSUPPORTED. */
typedef struct {
    int32_t n_layers;
    int32_t batch;               /* samples per pass (>= 1); must equal every layer's batch */
    const ff_layer_desc* layers; /* [host] n_layers entries */
    const int32_t* train_layer;  /* [host] n_layers flags, or NULL = every layer is trained.  A layer whose flag
                                    is 0 takes part in the forward pass and in the look-ahead sums of the layers
                                    before it, but its weights are left as they are (the greedy layer-by-layer
                                    schedule of Section III trains layer i with layers < i frozen). */
    int32_t lookahead;           /* FF_LOOKAHEAD_COEFF (0, the default reading) or FF_LOOKAHEAD_CHAIN, see below */
    const float* theta_layer;    /* [host] n_layers goodness thresholds, or NULL = the `theta` argument of
                                    ff_train_step for every layer (Section V-A uses one value, 2.0).  With freshly
                                    initialised weights the goodness of different layers differs by orders of
                                    magnitude; a threshold per layer keeps Eq. (1) and Eq. (2) away from saturation
                                    in all of them. */
    int32_t launch_mode;         /* FF_LAUNCH_AUTO (0), _KERNELS, _FUSED or _LANES, see below */
} ff_net_desc;

/* How ff_train_step issues its work.
 * FF_LAUNCH_KERNELS: one kernel per operation (quantise, contraction, goodness/loss, ...), about nine launches per
 *   layer.
 * FF_LAUNCH_FUSED: the whole step as ONE persistent kernel (after the fill that clears the workspace head) whose
 *   workgroups meet at device-wide barriers where the method has device-wide dependencies (a per-tensor absmax, a
 *   per-sample goodness).  For the launch-bound regime of small networks and batches, the one nearest the paper's
 *   own batch of 32 (Section V-A).  Plain dense stacks (no convolutions, residual wiring or FF_LOOKAHEAD_CHAIN) of at
 *   most 8 layers and 1024 samples per pass; FF_ERR_UNSUPPORTED otherwise.  Same results, bit for bit.
 * FF_LAUNCH_LANES: one kernel per operation, but the update chains of different layers (local gradient -> weight
 *   gradient -> update -> requantise; independent of each other, the learning being layer-local) go to up to three
 *   streams at once: the caller's and two that the library creates once per device (default priority) and keeps.  The
 *   chains are forked off the caller's stream after the look-ahead kernel and joined back before the call returns, so
 *   the step remains one piece of work in stream order, also under graph capture (a capture started before the
 *   library's streams exist runs on the caller's stream alone).  Every lane has its own copy of the chain scratch in
 *   the workspace.  For stacks of many small layers, whose single launches leave compute units idle.  Not with
 *   FF_LOOKAHEAD_CHAIN (FF_ERR_UNSUPPORTED).  Same results, bit for bit.  The library's streams and their fork / join
 *   events are shared by all calls on a device: steps that use lanes must not be issued from several host threads at
 *   the same time (steps issued one after the other, on any streams, are fine).
 * FF_LAUNCH_AUTO: FF_LAUNCH_FUSED when the stack qualifies and one pass through it is at most 2^27 multiply-adds
 *   (784 -> 500 -> 500 at 64 samples is 41 M); else lanes when the layers are small -- three below 2^33 multiply-adds
 *   per layer and pass on average, two below 2^36 -- else FF_LAUNCH_KERNELS.
 * ff_workspace_bytes depends on the mode (the fused step keeps every layer's int8 local gradient; lanes multiply the
 * chain scratch). */
enum { FF_LAUNCH_AUTO = 0, FF_LAUNCH_KERNELS = 1, FF_LAUNCH_FUSED = 2, FF_LAUNCH_LANES = 3 };

/* How the later layers' losses enter a layer's update (Eq. (3), Eq. (4)).
 * FF_LOOKAHEAD_COEFF: through their per-sample loss derivatives only (ff_lookahead); no gradient crosses a layer
 *   boundary, as Section IV-C describes the cost of the method.
 * FF_LOOKAHEAD_CHAIN: Eq. (4) taken literally as a derivative through the later layers, in int8 (a variant; the
 *   paper gives no int8 form of it).  Dense layers with l2norm_out = 0 only, else FF_ERR_UNSUPPORTED.  Per pass,
 *   from the last layer down, with c_i = dL_i/dG_i, y_i the activities and E_k = 0:
 *     h_i = (2 c_i y_i + E_i) * act'          quantised (stochastic, stream kind FF_KIND_CHAIN) -> h_q, s_h
 *     E_{i-1} = s_h s_W (h_q W_q)             ff_layer_input_grad, pre-step weights
 *     g_i = (2 c_i y_i + lambda E_i) * act'   quantised (stream kind FF_KIND_GRAD), then the weight gradient and
 *                                             the update as in the default reading.
 *   lambda = 0 gives the default step bit for bit; the last layer's update is the same for every lambda. */
enum { FF_LOOKAHEAD_COEFF = 0, FF_LOOKAHEAD_CHAIN = 1 };

/* Trainable state. [host] arrays of n_layers DEVICE pointers.
 * w_master[i]: fp32 [N_i, K_i] contiguous (conv: [C_out][k][k][C_in]).
 * w_q[i]:      int8 [N_i, ff_pitch(K_i)], s_w[i]: one fp32.  Both must hold the nearest-even
 *              quantisation of w_master[i] on entry to ff_train_step (ff_quantize produces it)
 *              and hold that of the updated weights on return. */
typedef struct {
    float* const* w_master;
    int8_t* const* w_q;
    float* const* s_w;
} ff_net_state;

/* Row pitch in bytes of an int8 matrix with `cols` columns; row pitch in elements of an int32 one. */
int64_t ff_pitch(int64_t cols);
int64_t ff_pitch32(int64_t cols);

/* Stream tag ff_train_step uses for (step, layer, pass index 0=pos/1=neg, kind). */
uint64_t ff_stream_tag(uint64_t step, uint32_t layer, uint32_t pass_idx, uint32_t kind);

const char* ff_status_string(ff_status s);
const char* ff_version(void);

/* ---------------------------------------------------------------------------------------------
 * ff_quantize — per-tensor symmetric uniform int8 quantiser (Section IV; Section IV-B: stochastic
 * rounding for the layer input A; nearest-even is used for weights).
 *   x      [rows, cols] fp32 contiguous (in)
 *   q      [rows, ff_pitch(cols)] int8 (out, may be NULL)
 *   q_t    [cols, ff_pitch(rows)] int8, the transposed copy the weight-gradient contraction reads
 *          (out, may be NULL; at least one of q, q_t must be given)
 *   scale  one fp32 (out): absmax/127, or 1 when absmax < 2^-100 (all codes are then 0)
 * codes = clamp(round(x * (127/absmax)), -127, 127).  Stochastic rounding draws one uniform per
 * element from a counter-based generator keyed by (seed, stream_tag, row*cols+col).
 * rows*cols == 0 is accepted (scale = 1).  ws: >= FF_WS_MIN_BYTES of scratch.
 * ------------------------------------------------------------------------------------------- */
ff_status ff_quantize(const float* x, int64_t rows, int64_t cols, int32_t round_mode, uint64_t seed,
                      uint64_t stream_tag, int8_t* q, int8_t* q_t, float* scale, void* ws,
                      size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * ff_layer_forward — the int8 x int8 -> int32 contraction of one layer for one pass
 * (Section IV-B: int8 operands, int32 accumulators), with the per-sample reductions the
 * goodness needs fused into its epilogue (Algorithm 1: G = ||y||^2).
 *   a_q      int8 [M, ff_pitch(K)] (dense: M = batch, K = in_features)               (in)
 *   w_q      int8 [N, ff_pitch(K)]                                                   (in)
 *   acc      int32 [M, ff_pitch32(N)]: acc[m][n] = sum_k a_q[m][k] * w_q[n][k]       (out)
 *   gsum_int uint64 [batch]: sum over the sample of (v*v >> r), v = act(acc) as an integer,
 *            r = ff_goodness_shift(layer)                                            (out)
 *   vmax     int32 [batch]: max over the sample of |v|                               (out)
 * Returns FF_ERR_OVERFLOW_BOUND if K * 127^2 could exceed int32.
 * ------------------------------------------------------------------------------------------- */
ff_status ff_layer_forward(const ff_layer_desc* layer, const int8_t* a_q, const int8_t* w_q,
                           int32_t* acc, uint64_t* gsum_int, int32_t* vmax, void* ws,
                           size_t ws_bytes, void* stream);

/* Convolution layers (kind FF_CONV2D) in the single-operation entry points
 *   - M = batch * H_out * W_out rows (one per output pixel, NHWC order), K = ksize^2 * C_in with the reduction
 *     index ordered (kh, kw, ci), N = C_out.  a_q is the NHWC int8 input [batch, H, W, ff_pitch(C_in)]
 *     (what ff_quantize writes for rows = batch*H*W, cols = C_in); w_q is [C_out, ff_pitch(K)].
 *   - ff_layer_forward runs an implicit GEMM when C_in % 16 == 0 (a 1x1 stride-1 convolution reads a_q as the
 *     dense operand it is, for any C_in); otherwise it first writes the patch matrix into ws.  ff_layer_backward_local takes the SAME NHWC a_q in its a_q_t argument and materialises the
 *     transposed patches of one weight-gradient chunk at a time in ws.  Both need
 *     ws_bytes >= ff_layer_workspace_bytes(layer).
 *   - A weight-gradient reduction over more than 133144 rows (M * 127^2 would not fit int32) is split into
 *     ff_layer_dw_chunks(layer) equal blocks of samples, block size = the largest power of two whose rows still
 *     fit; dw_acc then holds that many [N, ff_pitch32(K)] accumulators back to back, and ff_layer_update
 *     combines them in order (positive chunks, then negative chunks).  At most 2 chunks per pass. */
int32_t ff_layer_dw_chunks(const ff_layer_desc* layer);        /* [host only]; -1 for an invalid descriptor */
size_t ff_layer_workspace_bytes(const ff_layer_desc* layer);   /* [host only]; 0 for an invalid descriptor  */

/* Right shift applied to each squared integer activity before it is summed into gsum_int:
 * the smallest r >= 0 with (127^2 K)^2 * T / 2^r < 2^64, T = activities per sample.  [host only] */
int32_t ff_goodness_shift(const ff_layer_desc* layer);

/* ---------------------------------------------------------------------------------------------
 * ff_goodness_loss — goodness, FF loss and its derivative for one layer and one pass.
 *   goodness[b]  = fp32( gsum_int[b] * 2^r * s_y^2 ),  s_y = s_a * s_w   (Section III, Algorithm 1)
 *   positive pass (Eq. (1)): L = log(1 + exp(-(G - theta))), coeff = dL/dG = -sigmoid(-(G - theta))
 *   negative pass (Eq. (2)): L = log(1 + exp(+(G - theta))), coeff = dL/dG = +sigmoid(+(G - theta))
 *   loss_mean    = mean of L over the batch (one fp32)
 *   next_amax    = absmax of the tensor this layer hands to the next one, act(s_y*acc) or its
 *                  L2-normalised form (one fp32; may be NULL)
 * s_a, s_w: device scalars (in).  vmax: as produced by ff_layer_forward (in).
 * ------------------------------------------------------------------------------------------- */
ff_status ff_goodness_loss(const ff_layer_desc* layer, const uint64_t* gsum_int, const int32_t* vmax,
                           const float* s_a, const float* s_w, int32_t pass_sign, float theta,
                           float* goodness, float* coeff, float* loss_mean, float* next_amax,
                           void* stream);

/* ---------------------------------------------------------------------------------------------
 * ff_layer_handoff — the next layer's int8 input straight from this layer's accumulators
 * (Algorithm 1: the forward pass continues through all layers): a = act(s_y * acc), divided by
 * sqrt(goodness[b]) when layer->l2norm_out, quantised with `round_mode` against `amax`
 * (the value ff_goodness_loss wrote to next_amax).
 *   q   [M, ff_pitch(N)] (may be NULL), q_t [N, ff_pitch(M)] (may be NULL), scale: one fp32.
 * For a conv layer the rows are output pixels (NHWC), M = batch * H_out * W_out.
 * batch == 0 is accepted: nothing is read, scale = 1.
 * ------------------------------------------------------------------------------------------- */
ff_status ff_layer_handoff(const ff_layer_desc* layer, const int32_t* acc, const float* s_a,
                           const float* s_w, const float* goodness, const float* amax,
                           int32_t round_mode, uint64_t seed, uint64_t stream_tag, int8_t* q,
                           int8_t* q_t, float* scale, void* stream);

/* ---------------------------------------------------------------------------------------------
 * ff_lookahead — look-ahead combination of the per-sample loss derivatives (Eq. (3), Eq. (4)):
 *   coeff_total[i][b] = coeff[i][b] + lambda * sum_{j > i} coeff[j][b]
 * evaluated as S_k = 0, S_i = S_{i+1} + coeff[i+1], coeff_total[i] = fma(lambda, S_i, coeff[i]).
 * coeff, coeff_total: fp32 [n_layers, batch].  lambda = 0 returns coeff bit for bit.
 * ------------------------------------------------------------------------------------------- */
ff_status ff_lookahead(const float* coeff, int32_t n_layers, int64_t batch, float lambda,
                       float* coeff_total, void* stream);

/* ---------------------------------------------------------------------------------------------
 * ff_layer_backward_local — int8 local gradient and int8 weight-gradient contraction of one layer
 * for one pass (Section IV-B: g^Y is quantised to int8; only g^W is formed).
 *   g[m][n]      = (2 * coeff_total[b(m)]) * act(s_y * acc[m][n])
 *   gy_q_t       int8 [N, ff_pitch(M)]: quantised g, transposed, scale s_g               (out)
 *   dw_acc       int32 [N, ff_pitch32(K)]: dw_acc[n][k] = sum_m gy_q[m][n] * a_q[m][k]   (out)
 *   a_q_t        int8 [K, ff_pitch(M)]: the transposed copy ff_quantize / ff_layer_handoff wrote (in)
 *   dw_acc holds ff_layer_dw_chunks(layer) accumulators (1 unless M > 133144).
 * Convolutions: a_q_t is the NHWC int8 layer input itself.  Depthwise layers (FF_DWCONV2D): gy_q_t receives the
 * gradient ROW-MAJOR, int8 [M, ff_pitch(C)], and dw_acc is int32 [C, ff_pitch32(9)] with
 * dw_acc[c][kh*3+kw] = sum over output pixels of gy_q[m][c] * a_q[pixel(m) + tap][c].
 * ws: >= ff_layer_workspace_bytes(layer).  batch == 0 is accepted: s_g = 1 and dw_acc is all zero.
 * ------------------------------------------------------------------------------------------- */
ff_status ff_layer_backward_local(const ff_layer_desc* layer, const int32_t* acc, const int32_t* vmax,
                                  const float* s_a, const float* s_w, const float* coeff_total,
                                  int32_t round_mode, uint64_t seed, uint64_t stream_tag,
                                  const int8_t* a_q_t, int8_t* gy_q_t, float* s_g, int32_t* dw_acc,
                                  void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * ff_layer_backward_local_noalloc — ff_layer_backward_local for callers that cannot allocate device
 * memory or pass a workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, outputs and errors, without ws / ws_bytes: the scratch (absmax slot, patch
 * matrix of a convolution, partial sums of a split reduction) is a fixed array of
 * FF_NOALLOC_SCRATCH_BYTES inside the library's device image, one copy per GPU, held until the process
 * ends.  The call allocates and frees nothing and creates no HIP objects.
 *   - A layer that needs more scratch than that (ff_layer_workspace_bytes(layer) >
 *     FF_NOALLOC_SCRATCH_BYTES) is refused with FF_ERR_WORKSPACE before anything is launched.
 *   - Every call on a GPU uses that GPU's one array, which keeps the previous call's contents; nothing
 *     in it needs to start at zero.  Calls that overlap on one GPU (different streams, different
 *     threads) race on it: serialise them.
 * ff_noalloc_scratch_bytes() returns FF_NOALLOC_SCRATCH_BYTES. [host only]
 * ------------------------------------------------------------------------------------------- */
#define FF_NOALLOC_SCRATCH_BYTES (16u << 20)
size_t ff_noalloc_scratch_bytes(void);
ff_status ff_layer_backward_local_noalloc(const ff_layer_desc* layer, const int32_t* acc,
                                          const int32_t* vmax, const float* s_a, const float* s_w,
                                          const float* coeff_total, int32_t round_mode, uint64_t seed,
                                          uint64_t stream_tag, const int8_t* a_q_t, int8_t* gy_q_t,
                                          float* s_g, int32_t* dw_acc, void* stream);

/* ---------------------------------------------------------------------------------------------
 * ff_chain_gradients, ff_layer_input_grad — the two operations FF_LOOKAHEAD_CHAIN adds (Eq. (4) as an exact
 * derivative; dense layers).
 * ff_chain_gradients, one layer and pass:  y = act(s_a s_w acc);  E = (s_h s_w_up) e_acc, or 0 if e_acc == NULL
 *   h[m][n] = (2 coeff[m] y + E) * mask          fp32 [M, N] contiguous (out, may be NULL with h_amax)
 *   g[m][n] = fma(lambda, E, 2 coeff[m] y) * mask fp32 [M, N] contiguous (out)
 *   mask = acc > 0 under ReLU, 1 otherwise;  h_amax, g_amax: absmax of the two tensors (one fp32 each, out).
 *   acc int32 [M, ff_pitch32(N)], e_acc int32 [M, ff_pitch32(N)], coeff fp32 [M]; s_a, s_w, s_h, s_w_up device
 *   scalars (s_h, s_w_up unused without e_acc).  h and g are then quantised with ff_quantize.
 * ff_layer_input_grad:  e_acc[m][k] = sum_n h_q[m][n] * w_q_t[k][n]   (int32 [M, ff_pitch32(K)])
 *   h_q int8 [M, ff_pitch(N)]; w_q_t int8 [K, ff_pitch(N)] is the TRANSPOSED int8 weight matrix (ff_quantize's q_t
 *   output for the [N, K] master weights).  FF_ERR_OVERFLOW_BOUND if N * 127^2 could exceed int32.
 * ------------------------------------------------------------------------------------------- */
ff_status ff_chain_gradients(const ff_layer_desc* layer, const int32_t* acc, const float* s_a, const float* s_w,
                             const float* coeff, const int32_t* e_acc, const float* s_h, const float* s_w_up,
                             float lambda, float* h, float* g, float* h_amax, float* g_amax, void* stream);
ff_status ff_layer_input_grad(const ff_layer_desc* layer, const int8_t* h_q, const int8_t* w_q_t, int32_t* e_acc,
                              void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * ff_layer_update — SGD step on the fp32 master weights from both passes' integer accumulators
 * and requantisation (Algorithm 1, the update line of the inner loop):
 *   g = fp32(dw_pos) * (s_g_pos * s_a_pos);  g = fma(fp32(dw_neg), s_g_neg * s_a_neg, g)
 *   w = fma(-(lr / total_samples), g, w)
 *   w_q, s_w = nearest-even quantisation of the new w.
 * w_master fp32 [N, K] (in/out); dw_* int32 [N, ff_pitch32(K)]; w_q int8 [N, ff_pitch(K)].
 * ------------------------------------------------------------------------------------------- */
ff_status ff_layer_update(const ff_layer_desc* layer, float* w_master, const int32_t* dw_acc_pos,
                          const float* s_g_pos, const float* s_a_pos, const int32_t* dw_acc_neg,
                          const float* s_g_neg, const float* s_a_neg, float lr, int32_t total_samples,
                          int8_t* w_q, float* s_w, void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * ff_train_step — one iteration of Algorithm 1 over the positive and the negative set:
 * one int8 forward pass through all layers per set, goodness of every layer, then for every layer
 * the look-ahead loss derivative, the int8 local gradient, the int8 weight gradient and one
 * combined update.  Every layer's update uses activations computed with the pre-step weights.
 *   x_pos, x_neg  fp32 [batch, in_features] (dense first layer) or NHWC (conv)        (in)
 *   loss          fp32 [n_layers, 2]: mean loss per layer, [.,0] positive, [.,1] negative (out)
 *   goodness      fp32 [n_layers, 2, batch]                                           (out)
 *   ws            >= ff_workspace_bytes(net) bytes
 * Stochastic rounding streams: ff_stream_tag(step, layer, pass, kind) under `seed`.
 * net->lookahead selects how the later layers' losses enter (see FF_LOOKAHEAD_COEFF / FF_LOOKAHEAD_CHAIN above).
 * ------------------------------------------------------------------------------------------- */
ff_status ff_train_step(const ff_net_desc* net, const ff_net_state* state, const float* x_pos,
                        const float* x_neg, float theta, float lambda, float lr, uint64_t seed,
                        uint64_t step, float* loss, float* goodness, void* ws, size_t ws_bytes,
                        void* stream);

/* ---------------------------------------------------------------------------------------------
 * ff_train_step_at — ff_train_step with the step number in DEVICE memory: the kernels read
 * *step_dev when they run, not when the call is made, so a HIP graph captured from one call can
 * be replayed for every later iteration of Algorithm 1 (a launch-bound small network spends most
 * of an eagerly launched step on launch latency).  advance != 0: the last kernel of the call adds
 * one to *step_dev.  Same results, bit for bit, as ff_train_step(step = *step_dev).
 *   step_dev  one uint64 (in/out, 8-byte aligned); must stay allocated while a graph holding the
 *             call is alive.
 * The call neither allocates nor synchronises and enqueues kernels only, so it may be made on a
 * stream under capture (kernel timing, if enabled, is skipped for captured launches).  All other
 * arguments, outputs and errors as ff_train_step.
 * ------------------------------------------------------------------------------------------- */
ff_status ff_train_step_at(const ff_net_desc* net, const ff_net_state* state, const float* x_pos,
                           const float* x_neg, float theta, float lambda, float lr, uint64_t seed,
                           uint64_t* step_dev, int32_t advance, float* loss, float* goodness,
                           void* ws, size_t ws_bytes, void* stream);

/* Bytes of workspace ff_train_step needs for `net`; 0 if the descriptor is invalid. [host only] */
size_t ff_workspace_bytes(const ff_net_desc* net);

/* ---------------------------------------------------------------------------------------------
 * Instrumentation (not part of the method).  ff_timing_enable(class_mask): bit c of the mask
 * selects kernel class c (-1 = every class, 0 = off).  Every launch of a selected class is
 * bracketed by a pair of HIP events recorded on the launch stream; ff_timing_read waits for the
 * recorded events and returns the summed device time and the launch count of one kernel class.
 * An event record keeps the next launch from overlapping the previous kernel's tail, so timing
 * every class costs several per cent of a step; timing only the contractions costs under one.
 * Events are host-side objects created on first use (at most FF_TIMING_MAX_RECORDS pairs; launches
 * beyond that are not recorded; launches on a stream under capture are never recorded).
 * Not thread-safe; meant for benchmarks.
 * ------------------------------------------------------------------------------------------- */
enum {
    FF_K_GEMM_FWD = 0,   /* forward contraction (+ fused goodness reductions) */
    FF_K_GEMM_DW = 1,    /* weight-gradient contraction                       */
    FF_K_QUANT_ACT = 2,  /* activation quantise (fp32 input or hand-off)      */
    FF_K_QUANT_GRAD = 3, /* local-gradient quantise                           */
    FF_K_QUANT_W = 4,    /* weight requantise                                 */
    FF_K_UPDATE = 5,     /* weight update                                     */
    FF_K_ABSMAX = 6,     /* absmax of the fp32 input                          */
    FF_K_SMALL = 7,      /* fills, goodness/loss, look-ahead                  */
    FF_K_IM2COL = 8,     /* patch matrices of convolution layers              */
    FF_K_RESIDUAL = 9,   /* block output and its goodness (residual layers)   */
    FF_K_DWCONV = 10,    /* depthwise convolution: forward and weight gradient */
    FF_K_CHAIN = 11,     /* FF_LOOKAHEAD_CHAIN: gradient combination, its quantisation, input-gradient contraction */
    FF_K_FUSED = 12,     /* the single-launch step of a small dense stack (FF_LAUNCH_FUSED)  */
    FF_K_COUNT = 13
};
#define FF_TIMING_MAX_RECORDS 16384
ff_status ff_timing_enable(int32_t class_mask);
/* Clock probe of the contraction launches: while `counters` (16 uint64 in DEVICE memory, zeroed by the caller,
 * 8-byte aligned) is set, every workgroup of the forward and weight-gradient contraction kernels adds
 *   [0] the shader-clock cycles it was alive, [1] the ticks of the constant 100 MHz clock over the same interval
 *       ([0] / [1] * 100 MHz = the clock the launches actually ran at under the power manager),
 *   per tile, as seen by the workgroup's first thread, for weight-gradient launches in [2..6] and for forward
 *   launches in [8..12]: shader clocks from the start of the tile to its first fragments (operand round trip),
 *   of the main loop, of the epilogue, of the wait for the other wavefronts' epilogues, and the tile count.
 * NULL switches it off (the default).  The buffer must stay allocated while set. */
ff_status ff_timing_clock_probe(uint64_t* counters);
/* Phase stamps of the single-launch step (FF_LAUNCH_FUSED): while `stamps` (FF_FUSED_STAMPS uint64 in DEVICE memory,
 * 8-byte aligned) is set, the first workgroup of every such launch stores the constant 100 MHz clock at its start
 * ([0]), after each device-wide barrier ([1], [2], ...: 2 * n_layers + 3 barriers) and at its end: differences of
 * consecutive entries are the durations of the phases (absmax of the input; per layer: quantise, forward contraction;
 * last goodness + look-ahead + gradient quantise; weight gradient + update; requantise).  NULL switches it off. */
#define FF_FUSED_STAMPS 32
ff_status ff_timing_fused_stamps(uint64_t* stamps);
/* Ceiling probe (measurement aid, not part of the train step): one launch of a kernel that issues nothing but the
 * int8 MFMA instruction of the contraction kernel on register-resident operands -- one workgroup of 8 wavefronts per
 * compute unit, `iterations` x 8 instructions per wavefront -- on operand words of the given kind: 0 zeros, 1 every
 * code equal to 1, 2 pseudo-random words.  Timed by the caller (events on `stream`), it gives the rate the matrix pipes
 * sustain under the power manager for that kind of data, with no operand movement at all.
 *   sink      DEVICE, at least 256 * 512 * 4 bytes (512 KiB): receives one word per thread (keeps the work live)
 *   counters  DEVICE, 2 uint64 zeroed by the caller, or NULL: [0] += shader-clock cycles, [1] += 100 MHz ticks, per
 *             workgroup (their ratio * 100 MHz = the clock the launch ran at)
 *   ops       HOST out: int8 operations (2 per multiply-add) of the launch
 * Errors: FF_ERR_INVALID_ARG, FF_ERR_ALIGN, FF_ERR_WORKSPACE (sink too small), FF_ERR_HIP. */
ff_status ff_probe_mfma_ceiling(int32_t operand_kind, int32_t iterations, int32_t* sink, size_t sink_bytes,
                                uint64_t* counters, double* ops, void* stream);
ff_status ff_timing_reset(void);
ff_status ff_timing_read(int32_t kernel_class, double* total_ms, int64_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* FFINT8_H */
