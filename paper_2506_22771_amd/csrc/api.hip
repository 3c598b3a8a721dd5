// C-ABI entry points of libffint8: argument validation on the host, then kernel launches on the
// caller's stream.  Nothing here allocates device memory or synchronises.
#include <string.h>

#include <mutex>

#include "ff_internal.hpp"

namespace ffi {

constexpr int64_t INT32_SAFE_LEN = 2147483647ll / (127 * 127);  // longest reduction that cannot overflow int32
constexpr int MAX_LAYERS = 32;
constexpr int MAX_LANES = 3;   // streams that run the update chains of different layers side by side
constexpr int MAX_CHUNKS = 2;  // weight-gradient accumulators per pass (k_update combines at most 4 terms)

// Shapes of one layer as the kernels see them.
struct Dims {
    int kind;
    int64_t B, M, K, N, rps;   // M rows per pass (dense: B; conv: B*Ho*Wo), rps rows per sample
    int64_t in_rows, in_cols;  // 2-D view of the layer input: dense [B, K]; conv [B*H*W, C_in]
    bool implicit;             // conv whose forward runs as an implicit GEMM (C_in % 16 == 0)
    bool pointwise;            // 1x1 stride-1 convolution: its transposed patch matrix is the transposed input itself
    ConvGeom g;                // conv only
    int n_chunks;              // weight-gradient accumulators per pass
    int64_t chunk_b;           // samples per accumulator
    int src;                   // ff_train_step: index of the layer whose output is this layer's input (-1: the net input)
    int role, skip;            // residual-block wiring (ff_layer_desc)
};

// Sizes the quantise kernels accept: fewer than 2^32 elements (32-bit element index in the random stream) and at
// most 65535 row blocks of 128 rows (grid.y).
static bool quant_shape_ok(int64_t rows, int64_t cols)
{
    return rows >= 0 && cols >= 0 && (cols == 0 || rows < (int64_t(1) << 32) / cols) && (rows + 127) / 128 <= 65535;
}

static ff_status layer_dims(const ff_layer_desc* L, Dims* d)
{
    if (!L) return FF_ERR_INVALID_ARG;
    if (L->batch < 0) return FF_ERR_INVALID_ARG;
    memset(d, 0, sizeof(*d));
    d->kind = L->kind;
    d->B = L->batch;
    if (L->kind == FF_DENSE) {
        if (L->in_features <= 0 || L->out_features <= 0) return FF_ERR_SHAPE;
        d->M = L->batch;
        d->K = L->in_features;
        d->N = L->out_features;
        d->rps = 1;
        d->in_rows = L->batch;
        d->in_cols = L->in_features;
    } else if (L->kind == FF_CONV2D || L->kind == FF_DWCONV2D) {
        if (L->H <= 0 || L->W <= 0 || L->C_in <= 0 || L->C_out <= 0) return FF_ERR_SHAPE;
        if (L->kind == FF_DWCONV2D && (L->C_in != L->C_out || L->ksize != 3)) return FF_ERR_SHAPE;
        if ((L->ksize != 1 && L->ksize != 3) || (L->stride != 1 && L->stride != 2) || L->pad != L->ksize / 2)
            return FF_ERR_SHAPE;
        ConvGeom& g = d->g;
        g.H = L->H;
        g.W = L->W;
        g.Cin = L->C_in;
        g.cpitch = (int32_t)pitch8(L->C_in);
        g.ks = L->ksize;
        g.stride = L->stride;
        g.pad = L->pad;
        g.Ho = (L->H + 2 * L->pad - L->ksize) / L->stride + 1;
        g.Wo = (L->W + 2 * L->pad - L->ksize) / L->stride + 1;
        d->rps = (int64_t)g.Ho * g.Wo;
        d->M = d->B * d->rps;
        d->K = L->kind == FF_DWCONV2D ? (int64_t)L->ksize * L->ksize : (int64_t)L->ksize * L->ksize * L->C_in;
        d->N = L->C_out;
        d->in_rows = d->B * L->H * L->W;
        d->in_cols = L->C_in;
        d->implicit = L->kind == FF_CONV2D && (L->C_in & 15) == 0;
        d->pointwise = L->kind == FF_CONV2D && L->ksize == 1 && L->stride == 1;
        if (d->in_rows * g.cpitch >= (int64_t(1) << 31) || d->M >= (int64_t(1) << 31)) return FF_ERR_UNSUPPORTED;
    } else {
        return FF_ERR_INVALID_ARG;
    }
    // Launch limits of the kernels behind this layer, checked here so that an unsupported size is reported before
    // anything has been enqueued: the quantisers index elements with 32 bits and put 128 rows per workgroup on
    // grid.y; the update puts one weight row (or four) on grid.y; the depthwise kernels one sample.
    if (!quant_shape_ok(d->in_rows, d->in_cols) || !quant_shape_ok(d->M, d->N) || !quant_shape_ok(d->N, d->K) ||
        d->N > 65535 || (L->kind == FF_DWCONV2D && d->B > 65535))
        return FF_ERR_UNSUPPORTED;
    // Weight-gradient reduction: one accumulator if M * 127^2 fits int32, otherwise equal blocks of `per`
    // samples, per = the largest power of two with per * rps <= 133144.
    if (d->M <= INT32_SAFE_LEN) {
        d->n_chunks = 1;
        d->chunk_b = d->B;
    } else {
        int64_t per = 1;
        if (d->rps > INT32_SAFE_LEN) return FF_ERR_OVERFLOW_BOUND;
        while (per * 2 * d->rps <= INT32_SAFE_LEN) per *= 2;
        d->chunk_b = per;
        d->n_chunks = (int)((d->B + per - 1) / per);
        if ((per * d->rps) & 15) return FF_ERR_UNSUPPORTED;  // chunk starts must fall on 16-byte boundaries
    }
    return FF_OK;
}

static bool aligned16(const void* p) { return (((uintptr_t)p) & 15) == 0; }
static bool aligned4(const void* p) { return (((uintptr_t)p) & 3) == 0; }
#define HIPCHK(e) do { if ((e) != hipSuccess) return FF_ERR_HIP; } while (0)
// launch bracketed by timing events of kernel class `cls` on the stream `s` of the enclosing function
#define HIPCHK_T(cls, e) do { hipError_t _err; { Timed _t((cls), s); _err = (e); } if (_err != hipSuccess) return FF_ERR_HIP; } while (0)

static int32_t goodness_shift(int64_t K, int64_t terms)
{
    const unsigned __int128 a = (unsigned __int128)16129u * (unsigned __int128)K;
    const unsigned __int128 bound = a * a * (unsigned __int128)terms;
    int r = 0;
    while ((bound >> r) >> 64) ++r;
    return r;
}

// Scratch one layer needs per pass beyond FF_WS_MIN_BYTES.
// `col`: the row-major patch matrix of an explicit-im2col forward or the transposed patch matrix of one
// weight-gradient chunk (conv only).  `part`: partial accumulators of a split weight-gradient reduction.
// have_aqt: the caller keeps a transposed copy of a pointwise layer's input, which serves as its patch matrix.
static size_t layer_col_bytes(const Dims& d, bool have_aqt = false)
{
    if (d.kind != FF_CONV2D) return 0;   // dense and depthwise layers need no patch matrix
    const size_t fwd = d.implicit || d.pointwise ? 0 : (size_t)(d.M * pitch8(d.K));
    const size_t bwd = have_aqt && d.pointwise ? 0 : (size_t)(d.K * pitch8(d.chunk_b * d.rps));
    return align_up(fwd > bwd ? fwd : bwd, 256);
}
static size_t layer_part_bytes(const Dims& d, int nb)
{
    if (d.kind == FF_DWCONV2D) return 0;
    const GemmPlan p = gemm_plan(d.N, d.K, min(d.M, d.chunk_b * d.rps), nb, true);
    if (p.splits <= 1) return 0;
    return align_up((size_t)p.splits * (size_t)(d.N * pitch32(d.K)) * sizeof(int32_t), 256);
}
static size_t layer_scratch_bytes(const Dims& d) { return layer_col_bytes(d) + layer_part_bytes(d, 1); }

// ---- workspace of ff_train_step ------------------------------------------------------------------
struct WsLayout {
    int k;
    int64_t B;
    Dims d[MAX_LAYERS];
    // byte offsets
    size_t off_slots;      // uint32: out_amax[k+1][2] (slot 0: the net input, slot j+1: output of layer j),
                           // g_amax[k][2], w_amax[k]
    size_t off_gsum;       // uint64 [k][2][B]
    size_t off_vmax;       // int32  [k][2][B]
    size_t off_gl;         // scratch of the goodness / loss kernel (see GoodnessArgs::loss_part)
    size_t zero_bytes;     // the region [0, zero_bytes) is cleared at the start of a step
    size_t off_scales;     // fp32: s_a[k][2], s_g[k][2]
    // Scratch of one layer's update chain (local gradient -> weight gradient -> update -> requantise), `lanes` copies
    // `lane_stride` bytes apart: off_wbmax, off_gy, off_dw, off_col and off_part below are those of lane 0.  The chains
    // of different layers are independent of each other (layer-local learning), so a step may run them on several
    // streams at once, each with a scratch of its own.
    int lanes;
    size_t lane_stride;
    size_t off_wbmax;      // uint32 [UPDATE_MAX_BLOCKS]
    size_t off_c, off_ct;  // fp32 [k][2][B]
    size_t off_gy, st_gy;  // int8 scratch [2][st_gy]: transposed quantised local gradient
    size_t off_dw, st_dw, dw_bytes;  // int32 scratch [2][MAX_CHUNKS][dw_bytes]; st_dw = pass stride (bytes)
    size_t off_col, st_col;          // int8 scratch [2][st_col]: patch matrices of conv layers
    size_t off_part, st_part;        // int32 scratch [2][st_part] (bytes): partial sums of split weight gradients
    size_t off_aq[MAX_LAYERS], st_aq[MAX_LAYERS];    // quantised layer input [2][st]: dense layers share one scratch
    size_t off_aqt[MAX_LAYERS], st_aqt[MAX_LAYERS];  // dense and 1x1 stride-1 conv: transposed quantised input [2][st], retained
    size_t off_acc[MAX_LAYERS], st_acc[MAX_LAYERS];  // int32 accumulators [2][st] (bytes), retained
    size_t off_y[MAX_LAYERS], st_y[MAX_LAYERS];      // residual layers: fp32 block output [2][st] (bytes), retained
    // exact-derivative look-ahead only (all sizes 0 otherwise)
    int chain;
    size_t off_hf, off_gf, st_f;   // fp32 scratch [2][st_f] each: the two gradients of a layer before quantisation
    size_t off_hq, st_hq;          // int8 scratch [2][st_hq]: the gradient handed down, row-major
    size_t off_e, st_e;            // int32 scratch [2][st_e] (bytes): input-gradient accumulators
    size_t off_wqt;                // int8 scratch: transposed int8 weights of one layer
    // single-launch step of a small dense stack (all sizes 0 when the stack does not qualify)
    int fused_ok;                  // the stack qualifies for the single-launch kernel
    int fused_auto;                // ... and is small enough that FF_LAUNCH_AUTO picks it
    int fused_wgs;                 // workgroups of that launch
    size_t off_fgy[MAX_LAYERS], st_fgy[MAX_LAYERS];   // per layer: transposed int8 local gradient [2][st]
    size_t total;
};

static ff_status make_layout(const ff_net_desc* net, WsLayout* w)
{
    if (!net || !net->layers) return FF_ERR_INVALID_ARG;
    if (net->n_layers < 1 || net->n_layers > MAX_LAYERS) return FF_ERR_SHAPE;
    if (net->batch < 1) return FF_ERR_SHAPE;
    w->k = net->n_layers;
    w->B = net->batch;
    for (int i = 0; i < w->k; ++i) {
        const ff_status st = layer_dims(&net->layers[i], &w->d[i]);
        if (st != FF_OK) return st;
        const Dims& d = w->d[i];
        if (net->layers[i].batch != net->batch) return FF_ERR_SHAPE;
        if (d.K > INT32_SAFE_LEN) return FF_ERR_OVERFLOW_BOUND;
        if (d.n_chunks > MAX_CHUNKS) return FF_ERR_UNSUPPORTED;
        const ff_layer_desc& L = net->layers[i];
        Dims& dd = w->d[i];
        dd.role = L.role;
        dd.skip = L.skip;
        if (L.input_back < 0 || L.input_back > 1) return FF_ERR_UNSUPPORTED;
        if (L.role != FF_ROLE_LAYER && L.role != FF_ROLE_PROJECTION) return FF_ERR_INVALID_ARG;
        if (L.skip != FF_SKIP_NONE && L.skip != FF_SKIP_IDENTITY && L.skip != FF_SKIP_PROJECTION) return FF_ERR_INVALID_ARG;
        dd.src = i - 1 - L.input_back;
        if (dd.src < -1) return FF_ERR_SHAPE;
        if (dd.src >= 0) {
            const Dims& p = w->d[dd.src];
            if (p.role == FF_ROLE_PROJECTION) return FF_ERR_SHAPE;   // a projection has no output of its own
            if (p.kind == FF_DENSE && d.kind != FF_DENSE) return FF_ERR_UNSUPPORTED;   // no dense -> conv transition
            if (p.kind != FF_DENSE && d.kind == FF_DENSE) {
                // flatten: the NHWC output [B, H_out, W_out, C] read as [B, H_out * W_out * C]; its int32 rows must be
                // contiguous (C % 4 == 0)
                if ((p.N & 3) != 0) return FF_ERR_UNSUPPORTED;
                if (d.K != p.rps * p.N) return FF_ERR_SHAPE;
            } else if (d.kind == FF_DENSE && d.K != p.N) {
                return FF_ERR_SHAPE;
            }
            if (d.kind != FF_DENSE && (d.g.Cin != p.N || d.g.H != p.g.Ho || d.g.W != p.g.Wo)) return FF_ERR_SHAPE;
        }
        if (L.role == FF_ROLE_PROJECTION) {
            // [projection, conv1 (reads the same input), conv2 (adds the projection)]
            if (d.kind != FF_CONV2D || L.relu || L.l2norm_out || L.skip != FF_SKIP_NONE) return FF_ERR_INVALID_ARG;   // (a depthwise projection is not a case)
            if (i + 2 >= w->k || net->layers[i + 1].input_back != 1 || net->layers[i + 1].role != FF_ROLE_LAYER ||
                net->layers[i + 2].skip != FF_SKIP_PROJECTION)
                return FF_ERR_SHAPE;
        }
        if (L.skip != FF_SKIP_NONE) {
            if (d.kind != FF_CONV2D || L.role != FF_ROLE_LAYER || L.l2norm_out || (d.N & 3) || L.input_back != 0)
                return FF_ERR_UNSUPPORTED;
            if (d.B > 65535 || d.rps * (d.N >> 2) > (int64_t(1) << 28))   // launch limits of the block-output kernels
                return FF_ERR_UNSUPPORTED;
            if (L.skip == FF_SKIP_IDENTITY) {
                if (i < 1) return FF_ERR_SHAPE;
                const Dims& c1 = w->d[i - 1];   // the block input is the input of conv1
                if (c1.role != FF_ROLE_LAYER || c1.kind != FF_CONV2D || c1.g.Cin != d.N || c1.g.H != d.g.Ho ||
                    c1.g.W != d.g.Wo)
                    return FF_ERR_SHAPE;
            } else {
                if (i < 2) return FF_ERR_SHAPE;
                const Dims& pr = w->d[i - 2];
                if (pr.role != FF_ROLE_PROJECTION || pr.N != d.N || pr.g.Ho != d.g.Ho || pr.g.Wo != d.g.Wo)
                    return FF_ERR_SHAPE;
            }
        }
    }
    const size_t A = 256;
    size_t off = 0;
    const size_t k = (size_t)w->k, B = (size_t)w->B;
    w->off_slots = off;
    // + h_amax[k][2], wt_amax[k] (exact-derivative look-ahead)
    off = align_up(off + sizeof(uint32_t) * (k * 8 + 2), A);
    w->off_gsum = off;
    off = align_up(off + sizeof(uint64_t) * k * 2 * B, A);
    w->off_vmax = off;
    off = align_up(off + sizeof(int32_t) * k * 2 * B, A);
    w->off_gl = off;   // goodness / loss kernel with several workgroups: uint64 partial sums [2][GL_MAX_WG], uint32 counters [2]
    off = align_up(off + sizeof(uint64_t) * 2 * GL_MAX_WG + sizeof(uint32_t) * 2, A);
    w->zero_bytes = off;
    w->off_scales = off;
    off = align_up(off + sizeof(float) * (k * 4 + 4), A);   // + s_h[2], the scale of the transposed weight copy
    w->off_c = off;
    off = align_up(off + sizeof(float) * k * 2 * B, A);
    w->off_ct = off;
    off = align_up(off + sizeof(float) * k * 2 * B, A);
    size_t aq_dense = 0, gy = 0, dw = 0, col = 0, part = 0;
    for (int i = 0; i < w->k; ++i) {
        const Dims& d = w->d[i];
        if (d.kind == FF_DENSE) aq_dense = max(aq_dense, (size_t)(d.in_rows * pitch8(d.in_cols)));
        gy = max(gy, d.kind == FF_DWCONV2D ? (size_t)(d.M * pitch8(d.N)) : (size_t)(d.N * pitch8(d.M)));
        dw = max(dw, (size_t)(d.N * pitch32(d.K)) * sizeof(int32_t));
        col = max(col, layer_col_bytes(d, true));
        part = max(part, layer_part_bytes(d, 2));
    }
    aq_dense = align_up(aq_dense, A);
    const size_t off_aq_dense = off;
    off += 2 * aq_dense;
    if (net->launch_mode != FF_LAUNCH_AUTO && net->launch_mode != FF_LAUNCH_KERNELS && net->launch_mode != FF_LAUNCH_FUSED &&
        net->launch_mode != FF_LAUNCH_LANES)
        return FF_ERR_INVALID_ARG;
    // Single-launch step: plain dense stacks of at most FU_MAX_LAYERS layers and FU_MAX_B samples per pass.  It keeps
    // the local gradient of EVERY layer (the per-operation path reuses one scratch for all layers), hence the extra
    // buffers; weight gradients are applied straight from the accumulator registers.
    w->fused_ok = net->lookahead != FF_LOOKAHEAD_CHAIN && w->k <= FU_MAX_LAYERS && w->B <= FU_MAX_B;
    double macs = 0.0;
    int64_t fwd_tiles = 0, dw_tiles = 0;
    for (int i = 0; i < w->k && w->fused_ok; ++i) {
        const Dims& d = w->d[i];
        const ff_layer_desc& L = net->layers[i];
        if (d.kind != FF_DENSE || L.role != FF_ROLE_LAYER || L.skip != FF_SKIP_NONE || L.input_back != 0 || d.n_chunks != 1)
            w->fused_ok = 0;
        // (the kernel indexes with 32 bits)
        if (d.N * pitch8(d.K) > (int64_t(1) << 30) || d.K * pitch8(d.B) > (int64_t(1) << 30) || d.N * pitch8(d.B) > (int64_t(1) << 30))
            w->fused_ok = 0;
        macs += (double)d.B * (double)d.K * (double)d.N;
        fwd_tiles = max(fwd_tiles, 2 * ((d.B + 31) / 32) * ((d.N + 31) / 32));
        dw_tiles += ((d.N + 31) / 32) * ((d.K + 31) / 32);
    }
    w->fused_auto = w->fused_ok && macs <= (double)(int64_t(1) << 27);   // 41 M for 784 -> 500 -> 500 at 64 samples
    // workgroups: one per forward tile (both passes), and enough wavefronts (8 per workgroup) to take the weight-gradient
    // tiles of all layers in one round; an even number
    w->fused_wgs = (int)min((int64_t)256, max(max((int64_t)32, fwd_tiles), (dw_tiles + FU_THREADS / 64 - 1) / (FU_THREADS / 64)));
    w->fused_wgs = (w->fused_wgs + 1) & ~1;
    // Update chains on several streams: asked for (FF_LAUNCH_LANES), or chosen (FF_LAUNCH_AUTO) when the layers are small
    // enough that single launches leave compute units idle -- mean multiply-adds per layer and pass below 2^33 (three
    // lanes) or 2^36 (two).  Large dense layers fill the chip on their own and share one power budget: one lane.
    {
        double mean = 0.0;
        for (int i = 0; i < w->k; ++i) mean += (double)w->d[i].M * (double)w->d[i].K * (double)w->d[i].N;
        mean /= (double)w->k;
        int lanes = 1;
        if (net->lookahead == FF_LOOKAHEAD_COEFF && w->k >= 2) {
            if (net->launch_mode == FF_LAUNCH_LANES) lanes = MAX_LANES;
            else if (net->launch_mode == FF_LAUNCH_AUTO && !w->fused_auto)
                lanes = mean < 8589934592.0 ? MAX_LANES : (mean < 68719476736.0 ? 2 : 1);
        } else if (net->launch_mode == FF_LAUNCH_LANES) {
            return FF_ERR_UNSUPPORTED;
        }
        w->lanes = min(lanes, w->k);
    }
    const size_t lane0 = off;
    w->off_wbmax = off;   // per-workgroup maxima of a small weight update (UpdateArgs::block_max)
    off = align_up(off + sizeof(uint32_t) * UPDATE_MAX_BLOCKS, A);
    w->st_gy = align_up(gy, A);
    w->off_gy = off;
    off += 2 * w->st_gy;
    w->dw_bytes = align_up(dw, A);
    w->st_dw = MAX_CHUNKS * w->dw_bytes;
    w->off_dw = off;
    off += 2 * w->st_dw;
    w->st_col = col;
    w->off_col = off;
    off += 2 * w->st_col;
    w->st_part = part;
    w->off_part = off;
    off += 2 * w->st_part;
    w->lane_stride = align_up(off - lane0, A);
    off = lane0 + (size_t)w->lanes * w->lane_stride;
    for (int i = 0; i < w->k; ++i) {
        const Dims& d = w->d[i];
        if (d.kind == FF_DENSE) {
            w->off_aq[i] = off_aq_dense;
            w->st_aq[i] = aq_dense;
            w->st_aqt[i] = align_up((size_t)(d.K * pitch8(d.M)), A);
            w->off_aqt[i] = off;
            off += 2 * w->st_aqt[i];
        } else {
            w->st_aq[i] = align_up((size_t)(d.in_rows * pitch8(d.in_cols)), A);
            w->off_aq[i] = off;
            off += 2 * w->st_aq[i];
            w->st_aqt[i] = d.pointwise ? align_up((size_t)(d.K * pitch8(d.M)), A) : 0;
            w->off_aqt[i] = d.pointwise ? off : 0;
            off += 2 * w->st_aqt[i];
        }
        w->st_acc[i] = align_up((size_t)(d.M * pitch32(d.N)) * sizeof(int32_t), A);
        w->off_acc[i] = off;
        off += 2 * w->st_acc[i];
        w->st_y[i] = d.skip != FF_SKIP_NONE ? align_up((size_t)(d.M * d.N) * sizeof(float), A) : 0;
        w->off_y[i] = off;
        off += 2 * w->st_y[i];
    }
    w->chain = net->lookahead == FF_LOOKAHEAD_CHAIN;
    w->st_f = w->st_hq = w->st_e = 0;
    w->off_hf = w->off_gf = w->off_hq = w->off_e = w->off_wqt = off;
    if (net->lookahead != FF_LOOKAHEAD_COEFF && net->lookahead != FF_LOOKAHEAD_CHAIN) return FF_ERR_INVALID_ARG;
    if (w->chain) {
        size_t f = 0, hq = 0, e = 0, wqt = 0;
        for (int i = 0; i < w->k; ++i) {
            const Dims& d = w->d[i];
            const ff_layer_desc& L = net->layers[i];
            if (d.kind != FF_DENSE || L.l2norm_out || L.role != FF_ROLE_LAYER || L.skip != FF_SKIP_NONE || L.input_back)
                return FF_ERR_UNSUPPORTED;
            if (d.N > INT32_SAFE_LEN) return FF_ERR_OVERFLOW_BOUND;   // reduction length of the input gradient
            f = max(f, (size_t)(d.M * d.N) * sizeof(float));
            if (i > 0) {
                hq = max(hq, (size_t)(d.M * pitch8(d.N)));
                e = max(e, (size_t)(d.M * pitch32(d.K)) * sizeof(int32_t));
                wqt = max(wqt, (size_t)(d.K * pitch8(d.N)));
            }
        }
        w->st_f = align_up(f, A);
        w->off_hf = off;
        off += 2 * w->st_f;
        w->off_gf = off;
        off += 2 * w->st_f;
        w->st_hq = align_up(hq, A);
        w->off_hq = off;
        off += 2 * w->st_hq;
        w->st_e = align_up(e, A);
        w->off_e = off;
        off += 2 * w->st_e;
        w->off_wqt = off;
        off += align_up(wqt, A);
    }
    for (int i = 0; i < w->k; ++i) w->off_fgy[i] = w->st_fgy[i] = 0;
    if (net->launch_mode == FF_LAUNCH_FUSED && !w->fused_ok) return FF_ERR_UNSUPPORTED;
    if (w->fused_ok && net->launch_mode != FF_LAUNCH_KERNELS && (w->fused_auto || net->launch_mode == FF_LAUNCH_FUSED)) {
        for (int i = 0; i < w->k; ++i) {
            const Dims& d = w->d[i];
            w->st_fgy[i] = align_up((size_t)(d.N * pitch8(d.M)), A);
            w->off_fgy[i] = off;
            off += 2 * w->st_fgy[i];
        }
    } else {
        w->fused_auto = 0;
        if (net->launch_mode != FF_LAUNCH_FUSED) w->fused_ok = 0;
    }
    w->total = off;
    return FF_OK;
}

// ---- instrumentation: HIP events around each launch, recorded on the launch stream -----------------
struct TimingState {
    uint32_t mask = 0;   // bit c set: launches of kernel class c are timed
    int n = 0;
    hipEvent_t* ev = nullptr;  // 2 per record
    int8_t* cls = nullptr;
    int created = 0;
};
static TimingState g_timing;
static unsigned long long* g_clock_probe = nullptr;   // device counters of ff_timing_clock_probe (null: off)
static unsigned long long* g_fused_stamps = nullptr;  // device buffer of ff_timing_fused_stamps (null: off)

struct Timed {
    hipStream_t s;
    int idx = -1;
    Timed(int kernel_class, hipStream_t stream) : s(stream)
    {
        TimingState& t = g_timing;
        if (!((t.mask >> kernel_class) & 1u) || t.n >= FF_TIMING_MAX_RECORDS) return;
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;   // no event records into a graph under capture
        if (hipStreamIsCapturing(s, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) return;
        if (!t.ev) {
            t.ev = new hipEvent_t[2 * FF_TIMING_MAX_RECORDS];
            t.cls = new int8_t[FF_TIMING_MAX_RECORDS];
        }
        while (t.created <= t.n) {
            if (hipEventCreate(&t.ev[2 * t.created]) != hipSuccess) return;
            if (hipEventCreate(&t.ev[2 * t.created + 1]) != hipSuccess) return;
            ++t.created;
        }
        idx = t.n++;
        t.cls[idx] = (int8_t)kernel_class;
        (void)hipEventRecord(t.ev[2 * idx], s);
    }
    ~Timed()
    {
        if (idx >= 0) (void)hipEventRecord(g_timing.ev[2 * idx + 1], s);
    }
};

// ---- the two contractions of a layer, for nb passes at once ------------------------------------------
// Forward: acc[z] = A_q[z] x W_q^T (+ per-sample sums).  `aq` is the quantised layer input (dense: [M, pitch(K)];
// conv: NHWC), `col` scratch for an explicit patch matrix (3x3 or strided conv with C_in % 16 != 0).
static ff_status run_forward(const Dims& d, int relu, const int8_t* aq, int64_t st_aq, const int8_t* w_q, int32_t* acc,
                             int64_t st_acc, unsigned long long* gsum, int32_t* vmax, int64_t st_g, int8_t* col,
                             int64_t st_col, int nb, hipStream_t s)
{
    if (d.kind == FF_DWCONV2D) {
        DwArgs p;
        memset(&p, 0, sizeof(p));
        p.a = aq;
        p.st_a = st_aq;
        p.w_q = w_q;
        p.g = d.g;
        p.B = (int32_t)d.B;
        p.acc = acc;
        p.ldacc = pitch32(d.N);
        p.st_acc = st_acc;
        p.gsum = gsum;
        p.vmax = vmax;
        p.st_g = st_g;
        p.relu = relu;
        p.rshift = goodness_shift(d.K, d.rps * d.N);
        p.nb = nb;
        HIPCHK_T(FF_K_DWCONV, launch_dwconv_forward(p, s));
        return FF_OK;
    }
    GemmArgs g;
    memset(&g, 0, sizeof(g));
    g.Q = w_q;
    g.st_q = 0;
    g.C = acc;
    g.st_c = st_acc;
    g.I = (int32_t)d.M;
    g.J = (int32_t)d.N;
    g.R = (int32_t)d.K;
    g.ldq = pitch8(d.K);
    g.ldc = pitch32(d.N);
    g.gsum = gsum;
    g.vmax = vmax;
    g.st_g = st_g;
    g.rows_per_sample = (int32_t)d.rps;
    g.relu = relu;
    g.rshift = goodness_shift(d.K, d.rps * d.N);
    g.nb = nb;
    g.splits = 1;
    if (d.kind == FF_DENSE || d.pointwise) {
        // (a 1x1 stride-1 convolution: the NHWC input [B*H*W, pitch(C_in)] is its own patch matrix)
        g.P = aq;
        g.st_p = st_aq;
        g.ldp = pitch8(d.K);
    } else if (d.implicit) {
        g.P = aq;
        g.st_p = st_aq;
        g.ldp = 16;  // unused by the implicit loader
        g.conv = 1;
        g.H = d.g.H; g.W = d.g.W; g.Cin = d.g.Cin; g.cpitch = d.g.cpitch; g.ks = d.g.ks;
        g.stride = d.g.stride; g.pad = d.g.pad; g.Ho = d.g.Ho; g.Wo = d.g.Wo;
        g.p_bytes = d.in_rows * d.g.cpitch;
    } else {
        Im2colArgs ic;
        memset(&ic, 0, sizeof(ic));
        ic.a = aq;
        ic.st_a = st_aq;
        ic.out = col;
        ic.st_out = st_col;
        ic.g = d.g;
        ic.K = (int32_t)d.K;
        ic.b0 = 0;
        ic.b1 = (int32_t)d.B;
        ic.ld_out = pitch8(d.K);
        ic.nb = nb;
        HIPCHK_T(FF_K_IM2COL, launch_im2col(ic, false, s));
        g.P = col;
        g.st_p = st_col;
        g.ldp = pitch8(d.K);
    }
    g.clk = g_clock_probe;
    HIPCHK_T(FF_K_GEMM_FWD, launch_gemm_nt_i8(g, s));
    return FF_OK;
}

// Convolutions whose weight gradient reads column-shifted planes of the input instead of the full transposed
// patch matrix (see GemmArgs::conv == 2).
static bool wgrad_uses_planes(const Dims& d, int64_t nbatch, int nb)
{
    if (d.kind != FF_CONV2D || d.g.ks != 3 || (d.g.Wo & 15) != 0) return false;
    const int64_t bytes = (int64_t)d.g.ks * d.g.Cin * pitch8(nbatch * d.g.H * d.g.Wo);
    return bytes < (int64_t(1) << 31) && im2col_planes_ok(d.g, nbatch * nb);
}

// Weight gradient: dw[z][c] = gy_q_t[z][:, chunk c] x (patches of chunk c)^T for every chunk c.
// `aqt` is the transposed quantised input (dense; also a 1x1 stride-1 convolution when aqt_transposed is set) or the
// NHWC quantised input (conv; patches are materialised chunk by chunk into `colT`).  dw accumulators of one pass are dw_elems apart.
static ff_status run_wgrad(const Dims& d, const int8_t* gy_t, int64_t st_gy, const int8_t* aqt, int64_t st_aqt,
                           int8_t* colT, int64_t st_colT, int32_t* part, int64_t st_part, int32_t* dw, int64_t st_dw,
                           int64_t dw_elems, int nb, hipStream_t s, bool aqt_transposed = false)
{
    // depthwise accumulators are added to with atomics and must start at zero: one fill over all passes and chunks when
    // that span is small (it usually is: C x 12 words per accumulator), else one per accumulator
    const int64_t dw_span = (int64_t)(nb - 1) * st_dw + (int64_t)(d.n_chunks - 1) * dw_elems + d.N * pitch32(d.K);
    const bool dw_one_fill = d.kind == FF_DWCONV2D && dw_span <= (int64_t(1) << 20);
    if (dw_one_fill) HIPCHK_T(FF_K_SMALL, launch_fill_u32((uint32_t*)dw, dw_span, 0u, s));
    for (int c = 0; c < d.n_chunks; ++c) {
        const int64_t b0 = c * d.chunk_b, b1 = min(d.B, b0 + d.chunk_b);
        const int64_t m0 = b0 * d.rps, mc = (b1 - b0) * d.rps;
        if (d.kind == FF_DWCONV2D) {
            // gy_t holds the ROW-MAJOR int8 gradient [M, pitch(C)] for this layer kind
            for (int z = 0; z < nb && !dw_one_fill; ++z)
                HIPCHK_T(FF_K_SMALL, launch_fill_u32((uint32_t*)(dw + z * st_dw + c * dw_elems), d.N * pitch32(d.K), 0u, s));
            DwArgs p;
            memset(&p, 0, sizeof(p));
            p.a = aqt;
            p.st_a = st_aqt;
            p.g = d.g;
            p.B = (int32_t)d.B;
            p.gy = gy_t;
            p.ldg = pitch8(d.N);
            p.st_gy = st_gy;
            p.dw = dw + c * dw_elems;
            p.st_dw = st_dw;
            p.b0 = (int32_t)b0;
            p.b1 = (int32_t)b1;
            p.nb = nb;
            HIPCHK_T(FF_K_DWCONV, launch_dwconv_wgrad(p, s));
            continue;
        }
        GemmArgs g;
        memset(&g, 0, sizeof(g));
        g.P = gy_t + m0;
        g.st_p = st_gy;
        g.ldp = pitch8(d.M);
        g.C = dw + c * dw_elems;
        g.st_c = st_dw;
        g.I = (int32_t)d.N;
        g.J = (int32_t)d.K;
        g.R = (int32_t)mc;
        g.ldc = pitch32(d.K);
        g.rows_per_sample = 1;
        g.nb = nb;
        if (d.kind == FF_DENSE || aqt_transposed) {   // a 1x1 stride-1 convolution is a dense layer over its pixels
            g.Q = aqt + m0;
            g.st_q = st_aqt;
            g.ldq = pitch8(d.M);
        } else {
            Im2colArgs ic;
            memset(&ic, 0, sizeof(ic));
            ic.a = aqt;
            ic.st_a = st_aqt;
            ic.out = colT;
            ic.st_out = st_colT;
            ic.g = d.g;
            ic.b0 = (int32_t)b0;
            ic.b1 = (int32_t)b1;
            ic.nb = nb;
            g.Q = colT;
            g.st_q = st_colT;
            if (wgrad_uses_planes(d, b1 - b0, nb)) {
                // 3x3 convolution on rows of whole 16-pixel chunks: only the three column-shifted planes of the input
                // are written (a third of the patch matrix); the contraction applies the row offsets itself
                const int64_t ld3 = pitch8((b1 - b0) * d.g.H * d.g.Wo);
                ic.K = (int32_t)(d.g.ks * d.g.Cin);
                ic.ld_out = ld3;
                ic.wtaps_only = 1;
                HIPCHK_T(FF_K_IM2COL, launch_im2col(ic, true, s));
                g.ldq = ld3;
                g.conv = 2;
                g.H = d.g.H; g.W = d.g.W; g.Cin = d.g.Cin; g.cpitch = d.g.cpitch; g.ks = d.g.ks;
                g.stride = d.g.stride; g.pad = d.g.pad; g.Ho = d.g.Ho; g.Wo = d.g.Wo;
                g.p_bytes = (int64_t)ic.K * ld3;
            } else {
                ic.K = (int32_t)d.K;
                ic.ld_out = pitch8(mc);
                HIPCHK_T(FF_K_IM2COL, launch_im2col(ic, true, s));
                g.ldq = pitch8(mc);
            }
        }
        g.splits = gemm_plan(g.I, g.J, g.R, nb, true).splits;
        g.clk = g_clock_probe;
        if (g.splits > 1) {
            int32_t* out = g.C;
            g.C = part;
            g.st_c = st_part;
            g.st_split = d.N * pitch32(d.K);
            HIPCHK_T(FF_K_GEMM_DW, launch_gemm_nt_i8(g, s));
            HIPCHK_T(FF_K_GEMM_DW, launch_reduce_splits(part, g.splits, g.st_split, st_part, out, st_dw, g.st_split, nb, s));
        } else {
            HIPCHK_T(FF_K_GEMM_DW, launch_gemm_nt_i8(g, s));
        }
    }
    return FF_OK;
}

}  // namespace ffi

using namespace ffi;

extern "C" {

int64_t ff_pitch(int64_t cols) { return pitch8(cols); }
int64_t ff_pitch32(int64_t cols) { return pitch32(cols); }

uint64_t ff_stream_tag(uint64_t step, uint32_t layer, uint32_t pass_idx, uint32_t kind)
{
    return stream_tag_of(step, layer, pass_idx, kind);
}

const char* ff_status_string(ff_status s)
{
    switch (s) {
        case FF_OK: return "ok";
        case FF_ERR_INVALID_ARG: return "invalid argument";
        case FF_ERR_SHAPE: return "inconsistent or unsupported shape";
        case FF_ERR_ALIGN: return "buffer not aligned as required";
        case FF_ERR_WORKSPACE: return "workspace too small";
        case FF_ERR_OVERFLOW_BOUND: return "an int32 accumulator could overflow for this shape";
        case FF_ERR_UNSUPPORTED: return "not implemented in this build";
        case FF_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

const char* ff_version(void) { return "ffint8 0.4 (gfx950)"; }

int32_t ff_goodness_shift(const ff_layer_desc* layer)
{
    Dims d;
    if (layer_dims(layer, &d) != FF_OK) return -1;
    return goodness_shift(d.K, d.rps * d.N);
}

int32_t ff_layer_dw_chunks(const ff_layer_desc* layer)
{
    Dims d;
    if (layer_dims(layer, &d) != FF_OK) return -1;
    return d.n_chunks;
}

size_t ff_layer_workspace_bytes(const ff_layer_desc* layer)
{
    Dims d;
    if (layer_dims(layer, &d) != FF_OK) return 0;
    return FF_WS_MIN_BYTES + layer_scratch_bytes(d);
}

ff_status ff_quantize(const float* x, int64_t rows, int64_t cols, int32_t round_mode, uint64_t seed,
                      uint64_t stream_tag, int8_t* q, int8_t* q_t, float* scale, void* ws, size_t ws_bytes,
                      void* stream)
{
    if (rows < 0 || cols < 0 || !scale || (!q && !q_t) || !ws) return FF_ERR_INVALID_ARG;
    if (round_mode != FF_ROUND_NEAREST_EVEN && round_mode != FF_ROUND_STOCHASTIC) return FF_ERR_INVALID_ARG;
    if (!quant_shape_ok(rows, cols)) return FF_ERR_UNSUPPORTED;
    if (ws_bytes < FF_WS_MIN_BYTES) return FF_ERR_WORKSPACE;
    if (!aligned16(ws) || (q && !aligned16(q)) || (q_t && !aligned16(q_t)) || !aligned4(scale)) return FF_ERR_ALIGN;
    hipStream_t s = (hipStream_t)stream;
    if (rows == 0 || cols == 0) {
        const float one = 1.0f;
        uint32_t bits;
        memcpy(&bits, &one, 4);
        HIPCHK_T(FF_K_SMALL, launch_fill_u32((uint32_t*)scale, 1, bits, s));
        return FF_OK;
    }
    if (!x) return FF_ERR_INVALID_ARG;
    if (!aligned4(x)) return FF_ERR_ALIGN;
    uint32_t* slot = (uint32_t*)ws;
    HIPCHK_T(FF_K_SMALL, launch_fill_u32(slot, 1, 0u, s));
    HIPCHK_T(FF_K_ABSMAX, launch_absmax(x, 0, 1, rows * cols, slot, s));
    QuantArgs a;
    memset(&a, 0, sizeof(a));
    a.x = x;
    a.amax_bits = slot;
    a.round_mode = round_mode;
    a.key = make_sr_key(seed, stream_tag);
    a.rows = rows;
    a.cols = cols;
    a.q = q;
    a.ldq = pitch8(cols);
    a.q_t = q_t;
    a.ldqt = pitch8(rows);
    a.scale = scale;
    a.nb = 1;
    a.rows_per_sample = 1;
    HIPCHK_T(FF_K_QUANT_ACT, launch_quantize(QSRC_F32, a, s));
    return FF_OK;
}

ff_status ff_layer_forward(const ff_layer_desc* layer, const int8_t* a_q, const int8_t* w_q, int32_t* acc,
                           uint64_t* gsum_int, int32_t* vmax, void* ws, size_t ws_bytes, void* stream)
{
    Dims d;
    const ff_status st = layer_dims(layer, &d);
    if (st != FF_OK) return st;
    if (!a_q || !w_q || !acc || !gsum_int || !vmax) return FF_ERR_INVALID_ARG;
    if (!aligned16(a_q) || !aligned16(w_q) || !aligned16(acc) || (((uintptr_t)gsum_int) & 7) || !aligned4(vmax))
        return FF_ERR_ALIGN;
    if (d.K > INT32_SAFE_LEN) return FF_ERR_OVERFLOW_BOUND;
    const bool need_col = d.kind == FF_CONV2D && !d.implicit;
    if (need_col) {
        if (!ws) return FF_ERR_INVALID_ARG;
        if (!aligned16(ws)) return FF_ERR_ALIGN;
        if (ws_bytes < FF_WS_MIN_BYTES + layer_scratch_bytes(d)) return FF_ERR_WORKSPACE;
    }
    hipStream_t s = (hipStream_t)stream;
    if (d.B == 0) return FF_OK;
    HIPCHK_T(FF_K_SMALL, launch_fill_u32((uint32_t*)gsum_int, 2 * d.B, 0u, s));
    HIPCHK_T(FF_K_SMALL, launch_fill_u32((uint32_t*)vmax, d.B, 0u, s));
    int8_t* col = need_col ? (int8_t*)ws + FF_WS_MIN_BYTES : nullptr;
    return run_forward(d, layer->relu ? 1 : 0, a_q, 0, w_q, acc, 0, (unsigned long long*)gsum_int, vmax, 0, col, 0, 1, s);
}

ff_status ff_goodness_loss(const ff_layer_desc* layer, const uint64_t* gsum_int, const int32_t* vmax,
                           const float* s_a, const float* s_w, int32_t pass_sign, float theta, float* goodness,
                           float* coeff, float* loss_mean, float* next_amax, void* stream)
{
    Dims d;
    const ff_status st = layer_dims(layer, &d);
    if (st != FF_OK) return st;
    if (!gsum_int || !vmax || !s_a || !s_w || !goodness || !coeff || !loss_mean) return FF_ERR_INVALID_ARG;
    if (pass_sign != FF_PASS_POS && pass_sign != FF_PASS_NEG) return FF_ERR_INVALID_ARG;
    if ((((uintptr_t)gsum_int) & 7) || !aligned4(vmax) || !aligned4(goodness) || !aligned4(coeff)) return FF_ERR_ALIGN;
    hipStream_t s = (hipStream_t)stream;
    GoodnessArgs a;
    memset(&a, 0, sizeof(a));
    a.gsum = (const unsigned long long*)gsum_int;
    a.vmax = vmax;
    a.s_a = s_a;
    a.s_w = s_w;
    a.rshift = goodness_shift(d.K, d.rps * d.N);
    a.l2norm = layer->l2norm_out ? 1 : 0;
    a.pass_sign = pass_sign;
    a.theta = theta;
    a.B = d.B;
    a.goodness = goodness;
    a.coeff = coeff;
    a.loss_mean = loss_mean;
    a.next_amax_bits = (uint32_t*)next_amax;
    a.nb = 1;
    HIPCHK_T(FF_K_SMALL, launch_goodness_loss(a, s));
    return FF_OK;
}

ff_status ff_layer_handoff(const ff_layer_desc* layer, const int32_t* acc, const float* s_a, const float* s_w,
                           const float* goodness, const float* amax, int32_t round_mode, uint64_t seed,
                           uint64_t stream_tag, int8_t* q, int8_t* q_t, float* scale, void* stream)
{
    Dims d;
    const ff_status st = layer_dims(layer, &d);
    if (st != FF_OK) return st;
    if (!acc || !s_a || !s_w || !amax || !scale || (!q && !q_t)) return FF_ERR_INVALID_ARG;
    if (layer->l2norm_out && !goodness) return FF_ERR_INVALID_ARG;
    if (round_mode != FF_ROUND_NEAREST_EVEN && round_mode != FF_ROUND_STOCHASTIC) return FF_ERR_INVALID_ARG;
    if (!aligned16(acc) || (q && !aligned16(q)) || (q_t && !aligned16(q_t))) return FF_ERR_ALIGN;
    hipStream_t s = (hipStream_t)stream;
    if (d.M == 0) {   // empty batch: no codes; the scale of an empty tensor is 1, as in ff_quantize
        HIPCHK_T(FF_K_SMALL, launch_fill_u32((uint32_t*)scale, 1, 0x3F800000u, s));
        return FF_OK;
    }
    QuantArgs a;
    memset(&a, 0, sizeof(a));
    a.acc = acc;
    a.ldacc = pitch32(d.N);
    a.s_a = s_a;
    a.s_w = s_w;
    a.per_sample = goodness;
    a.rows_per_sample = (int32_t)d.rps;
    a.relu = layer->relu ? 1 : 0;
    a.l2norm = layer->l2norm_out ? 1 : 0;
    a.amax_bits = (const uint32_t*)amax;
    a.round_mode = round_mode;
    a.key = make_sr_key(seed, stream_tag);
    a.rows = d.M;
    a.cols = d.N;
    a.q = q;
    a.ldq = pitch8(d.N);
    a.q_t = q_t;
    a.ldqt = pitch8(d.M);
    a.scale = scale;
    a.nb = 1;
    HIPCHK_T(FF_K_QUANT_ACT, launch_quantize(QSRC_HANDOFF, a, s));
    return FF_OK;
}

ff_status ff_lookahead(const float* coeff, int32_t n_layers, int64_t batch, float lambda, float* coeff_total,
                       void* stream)
{
    if (!coeff || !coeff_total || batch < 0) return FF_ERR_INVALID_ARG;
    if (n_layers < 1 || n_layers > MAX_LAYERS) return FF_ERR_SHAPE;
    if (batch == 0) return FF_OK;
    hipStream_t s = (hipStream_t)stream;
    LookaheadArgs a;
    memset(&a, 0, sizeof(a));
    a.coeff = coeff;
    a.coeff_total = coeff_total;
    a.k = n_layers;
    a.np = 1;
    a.B = batch;
    a.st_layer = batch;
    a.st_pass = 0;
    a.lambda = lambda;
    HIPCHK_T(FF_K_SMALL, launch_lookahead(a, s));
    return FF_OK;
}

ff_status ff_layer_backward_local(const ff_layer_desc* layer, const int32_t* acc, const int32_t* vmax,
                                  const float* s_a, const float* s_w, const float* coeff_total, int32_t round_mode,
                                  uint64_t seed, uint64_t stream_tag, const int8_t* a_q_t, int8_t* gy_q_t,
                                  float* s_g, int32_t* dw_acc, void* ws, size_t ws_bytes, void* stream)
{
    Dims d;
    const ff_status st = layer_dims(layer, &d);
    if (st != FF_OK) return st;
    if (!acc || !vmax || !s_a || !s_w || !coeff_total || !a_q_t || !gy_q_t || !s_g || !dw_acc || !ws)
        return FF_ERR_INVALID_ARG;
    if (round_mode != FF_ROUND_NEAREST_EVEN && round_mode != FF_ROUND_STOCHASTIC) return FF_ERR_INVALID_ARG;
    if (ws_bytes < FF_WS_MIN_BYTES + layer_scratch_bytes(d)) return FF_ERR_WORKSPACE;
    if (!aligned16(acc) || !aligned16(a_q_t) || !aligned16(gy_q_t) || !aligned16(dw_acc) || !aligned16(ws))
        return FF_ERR_ALIGN;
    hipStream_t s = (hipStream_t)stream;
    if (d.B == 0) {   // empty batch: scale 1 (as for any empty tensor) and an all-zero weight gradient
        HIPCHK_T(FF_K_SMALL, launch_fill_u32((uint32_t*)s_g, 1, 0x3F800000u, s));
        HIPCHK_T(FF_K_SMALL, launch_fill_u32((uint32_t*)dw_acc, d.N * pitch32(d.K), 0u, s));
        return FF_OK;
    }
    uint32_t* slot = (uint32_t*)ws;
    HIPCHK_T(FF_K_SMALL, launch_grad_amax(coeff_total, vmax, s_a, s_w, d.B, slot, s));
    QuantArgs a;
    memset(&a, 0, sizeof(a));
    a.acc = acc;
    a.ldacc = pitch32(d.N);
    a.s_a = s_a;
    a.s_w = s_w;
    a.per_sample = coeff_total;
    a.rows_per_sample = (int32_t)d.rps;
    a.relu = layer->relu ? 1 : 0;
    a.amax_bits = slot;
    a.round_mode = round_mode;
    a.key = make_sr_key(seed, stream_tag);
    a.rows = d.M;
    a.cols = d.N;
    if (d.kind == FF_DWCONV2D) {   // the depthwise weight gradient reads the gradient row-major
        a.q = gy_q_t;
        a.ldq = pitch8(d.N);
    } else {
        a.q_t = gy_q_t;
        a.ldqt = pitch8(d.M);
    }
    a.scale = s_g;
    a.nb = 1;
    HIPCHK_T(FF_K_QUANT_GRAD, launch_quantize(QSRC_GRAD, a, s));
    const int64_t dw_elems = d.N * pitch32(d.K);
    int8_t* colT = (int8_t*)ws + FF_WS_MIN_BYTES;
    return run_wgrad(d, gy_q_t, 0, a_q_t, 0, colT, 0, (int32_t*)(colT + layer_col_bytes(d)), 0, dw_acc, 0, dw_elems, 1, s);
}

// ---- the entry point that allocates nothing: its scratch is a fixed array in the library's own device image ----
// Each GPU holds its own copy of the array at its own address; in host code the array's name is only a handle for
// hipGetSymbolAddress, never a device address.  The address is looked up once per device (with that device current)
// and kept; launches and kernels only ever see that pointer.
static __device__ __align__(256) unsigned char scratch[FF_NOALLOC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
static void* g_scratch_ptr[MAX_DEVICES];
static std::mutex g_scratch_mutex;

static ff_status scratch_of_current_device(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return FF_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return FF_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return FF_OK;
}

size_t ff_noalloc_scratch_bytes(void) { return FF_NOALLOC_SCRATCH_BYTES; }

ff_status ff_layer_backward_local_noalloc(const ff_layer_desc* layer, const int32_t* acc, const int32_t* vmax,
                                          const float* s_a, const float* s_w, const float* coeff_total,
                                          int32_t round_mode, uint64_t seed, uint64_t stream_tag, const int8_t* a_q_t,
                                          int8_t* gy_q_t, float* s_g, int32_t* dw_acc, void* stream)
{
    Dims d;
    const ff_status st = layer_dims(layer, &d);
    if (st != FF_OK) return st;
    // the layer's patch matrix and split partial sums must fit the fixed array
    if (FF_WS_MIN_BYTES + layer_scratch_bytes(d) > FF_NOALLOC_SCRATCH_BYTES) return FF_ERR_WORKSPACE;
    void* ws = nullptr;
    const ff_status ss = scratch_of_current_device(&ws);
    if (ss != FF_OK) return ss;
    // Nothing in the array has to start at zero: the absmax slot is stored (not accumulated into), the patch matrix
    // is written whole (pad bytes included) before the contraction reads it, and every split stores its own partial
    // sums before they are added up.
    return ff_layer_backward_local(layer, acc, vmax, s_a, s_w, coeff_total, round_mode, seed, stream_tag, a_q_t,
                                   gy_q_t, s_g, dw_acc, ws, FF_NOALLOC_SCRATCH_BYTES, stream);
}

ff_status ff_chain_gradients(const ff_layer_desc* layer, const int32_t* acc, const float* s_a, const float* s_w,
                             const float* coeff, const int32_t* e_acc, const float* s_h, const float* s_w_up,
                             float lambda, float* h, float* g, float* h_amax, float* g_amax, void* stream)
{
    Dims d;
    const ff_status st = layer_dims(layer, &d);
    if (st != FF_OK) return st;
    if (d.kind != FF_DENSE) return FF_ERR_UNSUPPORTED;
    if (!acc || !s_a || !s_w || !coeff || !g || !g_amax) return FF_ERR_INVALID_ARG;
    if (e_acc && (!s_h || !s_w_up)) return FF_ERR_INVALID_ARG;
    if ((h == nullptr) != (h_amax == nullptr)) return FF_ERR_INVALID_ARG;
    if (!aligned16(acc) || (e_acc && !aligned16(e_acc)) || !aligned4(g) || (h && !aligned4(h)) || !aligned4(g_amax) ||
        (h_amax && !aligned4(h_amax)))
        return FF_ERR_ALIGN;
    hipStream_t s = (hipStream_t)stream;
    HIPCHK_T(FF_K_SMALL, launch_fill_u32((uint32_t*)g_amax, 1, 0u, s));
    if (h_amax) HIPCHK_T(FF_K_SMALL, launch_fill_u32((uint32_t*)h_amax, 1, 0u, s));
    ChainArgs ca;
    memset(&ca, 0, sizeof(ca));
    ca.acc = acc;
    ca.ldacc = pitch32(d.N);
    ca.s_a = s_a;
    ca.s_w = s_w;
    ca.coeff = coeff;
    ca.e_acc = e_acc;
    ca.lde = pitch32(d.N);
    ca.s_h = s_h;
    ca.s_w_up = s_w_up;
    ca.lambda = lambda;
    ca.relu = layer->relu ? 1 : 0;
    ca.M = d.M;
    ca.N = d.N;
    ca.h = h;
    ca.g = g;
    ca.h_amax_bits = (uint32_t*)h_amax;   // the bit pattern of a non-negative fp32 is the value itself
    ca.g_amax_bits = (uint32_t*)g_amax;
    ca.nb = 1;
    HIPCHK_T(FF_K_CHAIN, launch_chain_combine(ca, s));
    return FF_OK;
}

ff_status ff_layer_input_grad(const ff_layer_desc* layer, const int8_t* h_q, const int8_t* w_q_t, int32_t* e_acc,
                              void* ws, size_t ws_bytes, void* stream)
{
    Dims d;
    const ff_status st = layer_dims(layer, &d);
    if (st != FF_OK) return st;
    if (d.kind != FF_DENSE) return FF_ERR_UNSUPPORTED;
    if (!h_q || !w_q_t || !e_acc || !ws) return FF_ERR_INVALID_ARG;
    if (ws_bytes < FF_WS_MIN_BYTES) return FF_ERR_WORKSPACE;
    if (!aligned16(h_q) || !aligned16(w_q_t) || !aligned16(e_acc)) return FF_ERR_ALIGN;
    if (d.N > INT32_SAFE_LEN) return FF_ERR_OVERFLOW_BOUND;
    hipStream_t s = (hipStream_t)stream;
    GemmArgs ga;
    memset(&ga, 0, sizeof(ga));
    ga.P = h_q;
    ga.Q = w_q_t;
    ga.C = e_acc;
    ga.I = (int32_t)d.M;
    ga.J = (int32_t)d.K;
    ga.R = (int32_t)d.N;
    ga.ldp = pitch8(d.N);
    ga.ldq = pitch8(d.N);
    ga.ldc = pitch32(d.K);
    ga.nb = 1;
    ga.splits = 1;
    HIPCHK_T(FF_K_CHAIN, launch_gemm_nt_i8(ga, s));
    return FF_OK;
}

ff_status ff_layer_update(const ff_layer_desc* layer, float* w_master, const int32_t* dw_acc_pos,
                          const float* s_g_pos, const float* s_a_pos, const int32_t* dw_acc_neg,
                          const float* s_g_neg, const float* s_a_neg, float lr, int32_t total_samples,
                          int8_t* w_q, float* s_w, void* ws, size_t ws_bytes, void* stream)
{
    Dims d;
    const ff_status st = layer_dims(layer, &d);
    if (st != FF_OK) return st;
    if (!w_master || !dw_acc_pos || !s_g_pos || !s_a_pos || !dw_acc_neg || !s_g_neg || !s_a_neg || !w_q || !s_w || !ws)
        return FF_ERR_INVALID_ARG;
    if (total_samples < 1) return FF_ERR_INVALID_ARG;
    if (ws_bytes < FF_WS_MIN_BYTES) return FF_ERR_WORKSPACE;
    if (!aligned4(w_master) || !aligned16(dw_acc_pos) || !aligned16(dw_acc_neg) || !aligned16(w_q) || !aligned16(ws))
        return FF_ERR_ALIGN;
    if (d.n_chunks > MAX_CHUNKS) return FF_ERR_UNSUPPORTED;
    hipStream_t s = (hipStream_t)stream;
    uint32_t* slot = (uint32_t*)ws;
    HIPCHK_T(FF_K_SMALL, launch_fill_u32(slot, 1, 0u, s));
    const int64_t dw_elems = d.N * pitch32(d.K);
    UpdateArgs u;
    memset(&u, 0, sizeof(u));
    u.w = w_master;
    u.N = d.N;
    u.K = d.K;
    u.lddw = pitch32(d.K);
    u.n_terms = 2 * d.n_chunks;
    for (int c = 0; c < d.n_chunks; ++c) {
        u.dw[c] = dw_acc_pos + c * dw_elems;
        u.s_g[c] = s_g_pos;
        u.s_a[c] = s_a_pos;
        u.dw[d.n_chunks + c] = dw_acc_neg + c * dw_elems;
        u.s_g[d.n_chunks + c] = s_g_neg;
        u.s_a[d.n_chunks + c] = s_a_neg;
    }
    u.lr = lr;
    u.total_samples = total_samples;
    u.w_amax_bits = slot;
    HIPCHK_T(FF_K_UPDATE, launch_update(u, s));
    QuantArgs a;
    memset(&a, 0, sizeof(a));
    a.x = w_master;
    a.amax_bits = slot;
    a.round_mode = FF_ROUND_NEAREST_EVEN;
    a.rows = d.N;
    a.cols = d.K;
    a.q = w_q;
    a.ldq = pitch8(d.K);
    a.scale = s_w;
    a.nb = 1;
    a.rows_per_sample = 1;
    HIPCHK_T(FF_K_QUANT_W, launch_quantize(QSRC_F32, a, s));
    return FF_OK;
}

size_t ff_workspace_bytes(const ff_net_desc* net)
{
    WsLayout w;
    if (make_layout(net, &w) != FF_OK) return 0;
    return w.total;
}

}  // extern "C"

// One iteration of Algorithm 1.  step_dev == null: the step number is `step`; otherwise it is read from device
// memory by the kernels (and advanced by one at the end when `advance` is set).
// Streams and events of the update-chain lanes: lane 0 is the caller's stream, lanes 1 .. MAX_LANES - 1 are streams
// the library creates once per device (default priority, non-blocking) and keeps until the process ends.  A step forks
// them off the caller's stream with an event after the look-ahead kernel and joins them back before it returns, so for
// the caller the step is still one piece of work in stream order (also under graph capture, where fork and join
// become graph edges).
struct LanePool {
    hipStream_t st[MAX_LANES - 1];
    hipEvent_t fork, join[MAX_LANES - 1];
    bool ready;
};
static LanePool g_lanes[MAX_DEVICES];
static std::mutex g_lanes_mutex;

static LanePool* lanes_of_current_device(bool may_create)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> lock(g_lanes_mutex);
    LanePool& p = g_lanes[dev];
    if (p.ready) return &p;
    if (!may_create) return nullptr;
    bool ok = hipEventCreateWithFlags(&p.fork, hipEventDisableTiming) == hipSuccess;
    for (int i = 0; i < MAX_LANES - 1 && ok; ++i)
        ok = hipStreamCreateWithFlags(&p.st[i], hipStreamNonBlocking) == hipSuccess &&
             hipEventCreateWithFlags(&p.join[i], hipEventDisableTiming) == hipSuccess;
    if (!ok) return nullptr;   // (whatever was created stays allocated; the step then runs on one stream)
    p.ready = true;
    return &p;
}

static ff_status train_step_impl(const ff_net_desc* net, const ff_net_state* state, const float* x_pos,
                                 const float* x_neg, float theta, float lambda, float lr, uint64_t seed, uint64_t step,
                                 uint64_t* step_dev, int32_t advance, float* loss, float* goodness, void* ws,
                                 size_t ws_bytes, void* stream)
{
    WsLayout w;
    const ff_status st = make_layout(net, &w);
    if (st != FF_OK) return st;
    if (!state || !state->w_master || !state->w_q || !state->s_w || !x_pos || !x_neg || !loss || !goodness || !ws)
        return FF_ERR_INVALID_ARG;
    for (int i = 0; i < w.k; ++i) {
        if (!state->w_master[i] || !state->w_q[i] || !state->s_w[i]) return FF_ERR_INVALID_ARG;
        if (!aligned4(state->w_master[i]) || !aligned16(state->w_q[i])) return FF_ERR_ALIGN;
    }
    if (ws_bytes < w.total) return FF_ERR_WORKSPACE;
    if (!aligned16(ws) || !aligned4(x_pos) || !aligned4(x_neg) || !aligned4(loss) || !aligned4(goodness))
        return FF_ERR_ALIGN;
    hipStream_t s = (hipStream_t)stream;
    char* base = (char*)ws;
    const int k = w.k;
    const int64_t B = w.B;
    uint32_t* out_amax = (uint32_t*)(base + w.off_slots);  // [k+1][2]: slot 0 the net input, slot j+1 the output of layer j
    uint32_t* g_amax = out_amax + 2 * (k + 1);             // [k][2]
    uint32_t* w_amax = g_amax + 2 * k;                     // [k]
    unsigned long long* gsum = (unsigned long long*)(base + w.off_gsum);
    int32_t* vmax = (int32_t*)(base + w.off_vmax);
    float* s_a = (float*)(base + w.off_scales);  // [k][2]
    float* s_g = s_a + 2 * k;                    // [k][2]
    float* c = (float*)(base + w.off_c);
    float* ct = (float*)(base + w.off_ct);

    const int64_t n_in = w.d[0].in_rows * w.d[0].in_cols;
    const int64_t st_x = ((intptr_t)x_neg - (intptr_t)x_pos) / (intptr_t)sizeof(float);
    if (w.fused_ok && (w.fused_auto || net->launch_mode == FF_LAUNCH_FUSED)) {
        // the whole step in one persistent launch (small dense stacks; see fused.hip): it clears what it adds to itself
        FusedArgs fa;
        memset(&fa, 0, sizeof(fa));
        fa.k = k;
        fa.B = (int32_t)B;
        fa.lambda = lambda;
        fa.lr = lr;
        fa.seed = seed;
        fa.step = step;
        fa.step_dev = step_dev;
        fa.advance = advance;
        fa.x = x_pos;
        fa.st_x = st_x;
        fa.wg_amax = (uint32_t*)(base + w.off_wbmax);   // (UPDATE_MAX_BLOCKS words: more than the 256 workgroups at most)
        fa.w_amax = w_amax;
        fa.gsum = gsum;
        fa.vmax = vmax;
        fa.s_a = s_a;
        fa.s_g = s_g;
        fa.c = c;
        fa.ct = ct;
        fa.goodness = goodness;
        fa.loss = loss;
        for (int i = 0; i < k; ++i) {
            const Dims& d = w.d[i];
            FusedLayer& fl = fa.L[i];
            fl.K = (int32_t)d.K;
            fl.N = (int32_t)d.N;
            fl.relu = net->layers[i].relu ? 1 : 0;
            fl.l2norm = net->layers[i].l2norm_out ? 1 : 0;
            fl.train = (!net->train_layer || net->train_layer[i]) ? 1 : 0;
            fl.rshift = goodness_shift(d.K, d.rps * d.N);
            fl.theta = net->theta_layer ? net->theta_layer[i] : theta;
            fl.w = state->w_master[i];
            fl.wq = state->w_q[i];
            fl.sw = state->s_w[i];
            fl.aq = (int8_t*)(base + w.off_aq[i]);
            fl.st_aq = (int64_t)w.st_aq[i];
            fl.aqt = (int8_t*)(base + w.off_aqt[i]);
            fl.st_aqt = (int64_t)w.st_aqt[i];
            fl.acc = (int32_t*)(base + w.off_acc[i]);
            fl.st_acc = (int64_t)(w.st_acc[i] / sizeof(int32_t));
            fl.gy = (int8_t*)(base + w.off_fgy[i]);
            fl.st_gy = (int64_t)w.st_fgy[i];
        }
        fa.stamps = g_fused_stamps;
        HIPCHK_T(FF_K_FUSED, launch_fused_dense_step(fa, w.fused_wgs, s));
        return FF_OK;
    }
    HIPCHK_T(FF_K_SMALL, launch_fill_u32((uint32_t*)base, (int64_t)(w.zero_bytes / 4), 0u, s));
    HIPCHK_T(FF_K_ABSMAX, launch_absmax(x_pos, st_x, 2, n_in, out_amax, s));

    // ---- streams: the caller's, plus the library's own where the step runs independent work side by side
    hipStream_t lane_stream[MAX_LANES];
    for (int l = 0; l < MAX_LANES; ++l) lane_stream[l] = s;
    int n_lanes = 1;
    LanePool* pool = nullptr;
    if (w.lanes > 1 && !w.chain) {
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        const bool capturing = hipStreamIsCapturing(s, &cap) == hipSuccess && cap != hipStreamCaptureStatusNone;
        pool = lanes_of_current_device(!capturing);   // nothing is created while a graph is being captured
        if (pool) {
            n_lanes = w.lanes;
            for (int l = 1; l < n_lanes; ++l) lane_stream[l] = pool->st[l - 1];
        }
    }
    const hipStream_t s_main = s;

    // ---- forward pass through all layers, both data sets together (Algorithm 1) -----------------
    bool proj_pending = false;   // a projection's forward pass is running on the second stream
    for (int i = 0; i < k; ++i) {
        const Dims& d = w.d[i];
        const ff_layer_desc& L = net->layers[i];
        const bool dense = d.kind == FF_DENSE;
        // The 1x1 projection of a residual block and the block's first convolution read the same input and do not
        // depend on each other: with a second stream at hand the projection (quantiser + contraction; no patch
        // scratch: it reads the input tensor directly) runs there, and the block's second convolution waits for it.
        const bool side = n_lanes > 1 && d.role == FF_ROLE_PROJECTION && (d.implicit || d.pointwise) && !proj_pending;
        hipStream_t s = s_main;
        if (side) {
            if (hipEventRecord(pool->fork, s_main) != hipSuccess || hipStreamWaitEvent(lane_stream[1], pool->fork, 0) != hipSuccess)
                return FF_ERR_HIP;
            s = lane_stream[1];
        }
        QuantArgs a;
        memset(&a, 0, sizeof(a));
        int src;
        if (d.src < 0) {
            src = QSRC_F32;
            a.x = x_pos;
            a.st_x = st_x;
            a.rows_per_sample = 1;
        } else if (w.d[d.src].skip != FF_SKIP_NONE) {
            // the source is a residual layer: its block output is held as fp32
            src = QSRC_F32;
            a.x = (const float*)(base + w.off_y[d.src]);
            a.st_x = (int64_t)(w.st_y[d.src] / sizeof(float));
            a.rows_per_sample = 1;
        } else {
            const int j = d.src;
            const Dims& dp = w.d[j];
            const ff_layer_desc& Lp = net->layers[j];
            src = QSRC_HANDOFF;
            a.acc = (const int32_t*)(base + w.off_acc[j]);
            a.st_acc = (int64_t)(w.st_acc[j] / sizeof(int32_t));
            a.ldacc = pitch32(dp.N);
            a.s_a = s_a + 2 * j;
            a.st_s_a = 1;
            a.s_w = state->s_w[j];
            a.st_s_w = 0;
            a.per_sample = goodness + (int64_t)j * 2 * B;
            a.st_per_sample = B;
            a.rows_per_sample = (int32_t)dp.rps;
            if (dp.kind != FF_DENSE && dense) {   // flatten: one row of H_out * W_out * C contiguous accumulators per sample
                a.ldacc = d.K;
                a.rows_per_sample = 1;
            }
            a.relu = Lp.relu ? 1 : 0;
            a.l2norm = Lp.l2norm_out ? 1 : 0;
        }
        a.amax_bits = out_amax + 2 * (d.src + 1);
        a.st_amax = 1;
        a.round_mode = FF_ROUND_STOCHASTIC;
        a.key = make_sr_key(seed, ff_stream_tag(step, (uint32_t)i, 0, FF_KIND_ACT));
        a.key2 = make_sr_key(seed, ff_stream_tag(step, (uint32_t)i, 1, FF_KIND_ACT));
        a.step_dev = step_dev;
        a.seed = seed;
        a.tag_layer = (uint32_t)i;
        a.tag_kind = FF_KIND_ACT;
        a.rows = d.in_rows;
        a.cols = d.in_cols;
        a.q = (int8_t*)(base + w.off_aq[i]);
        a.st_q = (int64_t)w.st_aq[i];
        a.ldq = pitch8(d.in_cols);
        if (dense || d.pointwise) {
            a.q_t = (int8_t*)(base + w.off_aqt[i]);
            a.st_qt = (int64_t)w.st_aqt[i];
            a.ldqt = pitch8(d.M);
            a.qt_streaming = 1;   // read again only by this layer's weight gradient, after every forward pass
        }
        a.scale = s_a + 2 * i;
        a.st_scale = 1;
        a.nb = 2;
        const bool plain = d.role == FF_ROLE_LAYER && d.skip == FF_SKIP_NONE;   // goodness straight from the accumulators
        ff_status fs = [&]() -> ff_status {
            if (d.role == FF_ROLE_PROJECTION) {
                // no activity of its own: zero coefficients (nothing enters the look-ahead sums), zero loss / goodness rows
                // (on the projection's own stream: nothing reads them before the look-ahead kernel)
                HIPCHK_T(FF_K_SMALL, launch_fill_u32((uint32_t*)(c + (int64_t)i * 2 * B), 2 * B, 0u, s));
                HIPCHK_T(FF_K_SMALL, launch_fill_u32((uint32_t*)(goodness + (int64_t)i * 2 * B), 2 * B, 0u, s));
                HIPCHK_T(FF_K_SMALL, launch_fill_u32((uint32_t*)(loss + 2 * i), 2, 0u, s));
            }
            HIPCHK_T(FF_K_QUANT_ACT, launch_quantize(src, a, s));
            return run_forward(d, L.relu ? 1 : 0, (const int8_t*)(base + w.off_aq[i]), (int64_t)w.st_aq[i], state->w_q[i],
                               (int32_t*)(base + w.off_acc[i]), (int64_t)(w.st_acc[i] / sizeof(int32_t)),
                               plain ? gsum + (int64_t)i * 2 * B : nullptr, vmax + (int64_t)i * 2 * B, B,
                               (int8_t*)(base + w.off_col), (int64_t)w.st_col, 2, s);
        }();
        if (side) {   // (whatever happened on the second stream, it is joined back)
            if (hipEventRecord(pool->join[0], s) != hipSuccess) fs = fs != FF_OK ? fs : FF_ERR_HIP;
            proj_pending = true;
            if (fs != FF_OK) (void)hipStreamWaitEvent(s_main, pool->join[0], 0);
        }
        if (fs != FF_OK) return fs;
        if (d.role == FF_ROLE_PROJECTION) continue;
        if (!plain) {
            ResidualArgs ra;
            memset(&ra, 0, sizeof(ra));
            ra.acc = (const int32_t*)(base + w.off_acc[i]);
            ra.ldacc = pitch32(d.N);
            ra.st_acc = (int64_t)(w.st_acc[i] / sizeof(int32_t));
            ra.s_a = s_a + 2 * i;
            ra.st_s_a = 1;
            ra.s_w = state->s_w[i];
            ra.skip = d.skip;
            if (d.skip == FF_SKIP_IDENTITY) {
                ra.xq = (const int8_t*)(base + w.off_aq[i - 1]);
                ra.ldx = pitch8(w.d[i - 1].in_cols);
                ra.st_xq = (int64_t)w.st_aq[i - 1];
                ra.s_x = s_a + 2 * (i - 1);
                ra.st_s_x = 1;
            } else {
                ra.accp = (const int32_t*)(base + w.off_acc[i - 2]);
                ra.ldaccp = pitch32(w.d[i - 2].N);
                ra.st_accp = (int64_t)(w.st_acc[i - 2] / sizeof(int32_t));
                ra.s_ap = s_a + 2 * (i - 2);
                ra.st_s_ap = 1;
                ra.s_wp = state->s_w[i - 2];
            }
            ra.relu = L.relu ? 1 : 0;
            ra.M = d.M;
            ra.N = d.N;
            ra.rows_per_sample = (int32_t)d.rps;
            ra.y = (float*)(base + w.off_y[i]);
            ra.st_y = (int64_t)(w.st_y[i] / sizeof(float));
            ra.ymax_bits = (uint32_t*)(vmax + (int64_t)i * 2 * B);
            ra.st_b = B;
            ra.nb = 2;
            if (d.skip == FF_SKIP_PROJECTION && proj_pending) {   // the projection's accumulators are read from here on
                if (hipStreamWaitEvent(s_main, pool->join[0], 0) != hipSuccess) return FF_ERR_HIP;
                proj_pending = false;
            }
            HIPCHK_T(FF_K_RESIDUAL, launch_residual_act(ra, s));
            GoodnessFxArgs fa;
            memset(&fa, 0, sizeof(fa));
            fa.y = ra.y;
            fa.st_y = ra.st_y;
            fa.M = d.M;
            fa.N = d.N;
            fa.rows_per_sample = (int32_t)d.rps;
            fa.ymax_bits = ra.ymax_bits;
            fa.amax_bits = out_amax + 2 * (i + 1);
            fa.st_amax = 1;
            fa.gsum = gsum + (int64_t)i * 2 * B;
            fa.st_b = B;
            fa.nb = 2;
            HIPCHK_T(FF_K_RESIDUAL, launch_goodness_fx(fa, s));
        }

        GoodnessArgs ga;
        memset(&ga, 0, sizeof(ga));
        ga.gsum = gsum + (int64_t)i * 2 * B;
        ga.vmax = vmax + (int64_t)i * 2 * B;
        ga.s_a = s_a + 2 * i;
        ga.s_w = state->s_w[i];
        ga.rshift = goodness_shift(d.K, d.rps * d.N);
        ga.l2norm = L.l2norm_out ? 1 : 0;
        ga.pass_sign = FF_PASS_POS;
        ga.theta = net->theta_layer ? net->theta_layer[i] : theta;
        ga.B = B;
        ga.goodness = goodness + (int64_t)i * 2 * B;
        ga.coeff = c + (int64_t)i * 2 * B;
        ga.loss_mean = loss + 2 * i;
        // the absmax of this layer's output, i.e. of the input of whichever layers read it
        ga.next_amax_bits = plain ? out_amax + 2 * (i + 1) : nullptr;
        ga.fx_amax_bits = plain ? nullptr : out_amax + 2 * (i + 1);
        ga.nb = 2;
        ga.st_b = B;
        ga.st_scalar = 1;
        ga.loss_part = (unsigned long long*)(base + w.off_gl);
        ga.wg_counter = (uint32_t*)(base + w.off_gl + sizeof(uint64_t) * 2 * GL_MAX_WG);
        HIPCHK_T(FF_K_SMALL, launch_goodness_loss(ga, s));
    }

    if (proj_pending && hipStreamWaitEvent(s_main, pool->join[0], 0) != hipSuccess) return FF_ERR_HIP;

    // ---- look-ahead coefficients of every layer (Eq. (3)/(4)) and the absmax of every local gradient
    if (!w.chain) {
        LookaheadArgs la;
        memset(&la, 0, sizeof(la));
        la.coeff = c;
        la.coeff_total = ct;
        la.k = k;
        la.np = 2;
        la.B = B;
        la.st_layer = 2 * B;
        la.st_pass = B;
        la.lambda = lambda;
        la.vmax = vmax;
        la.s_a = s_a;
        la.s_w = state->s_w;
        la.g_amax_bits = g_amax;
        for (int i = 0; i < k; ++i)
            if (w.d[i].skip != FF_SKIP_NONE) la.fx_mask |= 1u << i;
        HIPCHK_T(FF_K_SMALL, launch_lookahead(la, s));
    }

    // ---- per layer: int8 local gradient, int8 weight gradient, update (Algorithm 1, inner loop) ----
    // weights of layer `t` from the transposed int8 gradient in the scratch (quantised for layer `gl`): weight-gradient
    // contraction per pass and chunk, combined update, requantisation
    // ---- lanes: which copy of the chain scratch and which stream a layer's update chain uses
    int lane_of[MAX_LAYERS];
    {
        // longest chain first onto the lane with the least work so far (cost ~ multiply-adds of the layer)
        double load[MAX_LANES];
        for (int l = 0; l < MAX_LANES; ++l) load[l] = 0.0;
        bool placed[MAX_LAYERS];
        for (int i = 0; i < k; ++i) { placed[i] = false; lane_of[i] = 0; }
        for (int n = 0; n < k && n_lanes > 1; ++n) {
            int best = -1;
            double bc = -1.0;
            for (int i = 0; i < k; ++i) {
                const double c = (double)w.d[i].M * (double)w.d[i].K * (double)w.d[i].N;
                if (!placed[i] && c > bc) { bc = c; best = i; }
            }
            int l = 0;
            for (int j = 1; j < n_lanes; ++j)
                if (load[j] < load[l]) l = j;
            placed[best] = true;
            lane_of[best] = l;
            load[l] += bc;
        }
        // a projection is updated by the chain of the block's second convolution
        for (int i = 0; i < k; ++i)
            if (w.d[i].skip == FF_SKIP_PROJECTION && i >= 2) lane_of[i - 2] = lane_of[i];
    }
    // joins the lanes back into the caller's stream: explicitly at the end of the chains, and on every early way out
    struct Join {
        LanePool* pool;
        hipStream_t* st;
        int n;
        ff_status finish()
        {
            bool ok = true;
            for (int l = 1; l < n; ++l) {
                ok = hipEventRecord(pool->join[l - 1], st[l]) == hipSuccess && ok;
                ok = hipStreamWaitEvent(st[0], pool->join[l - 1], 0) == hipSuccess && ok;
            }
            n = 1;
            return ok ? FF_OK : FF_ERR_HIP;
        }
        ~Join() { (void)finish(); }
    };

    auto wgrad_update = [&](int t, int gl) -> ff_status {
        const Dims& d = w.d[t];
        const int lane = lane_of[gl];
        hipStream_t s = lane_stream[lane];                        // (shadows the caller's stream inside the chain)
        char* base = (char*)ws + (size_t)lane * w.lane_stride;   // lane-scoped scratch: gy, dw, col, part, wbmax
        char* const base0 = (char*)ws;                            // what lives outside the lanes
        const bool dense = d.kind == FF_DENSE || d.pointwise;   // layers that keep a transposed copy of their input
        const int64_t dw_elems = (int64_t)(w.dw_bytes / sizeof(int32_t));
        const ff_status ws_ = run_wgrad(d, (const int8_t*)(base + w.off_gy), (int64_t)w.st_gy,
                                        dense ? (const int8_t*)(base0 + w.off_aqt[t]) : (const int8_t*)(base0 + w.off_aq[t]),
                                        dense ? (int64_t)w.st_aqt[t] : (int64_t)w.st_aq[t], (int8_t*)(base + w.off_col),
                                        (int64_t)w.st_col, (int32_t*)(base + w.off_part),
                                        (int64_t)(w.st_part / sizeof(int32_t)), (int32_t*)(base + w.off_dw),
                                        (int64_t)(w.st_dw / sizeof(int32_t)), dw_elems, 2, s, d.pointwise);
        if (ws_ != FF_OK) return ws_;

        UpdateArgs u;
        memset(&u, 0, sizeof(u));
        u.w = state->w_master[t];
        u.N = d.N;
        u.K = d.K;
        u.lddw = pitch32(d.K);
        u.n_terms = 2 * d.n_chunks;
        for (int p = 0; p < 2; ++p)
            for (int cc = 0; cc < d.n_chunks; ++cc) {
                const int tt = p * d.n_chunks + cc;
                u.dw[tt] = (const int32_t*)(base + w.off_dw + p * w.st_dw + cc * w.dw_bytes);
                u.s_g[tt] = s_g + 2 * gl + p;
                u.s_a[tt] = s_a + 2 * t + p;
            }
        u.lr = lr;
        u.total_samples = (int32_t)(2 * B);
        u.w_amax_bits = w_amax + t;
        // small tensors: one maximum per workgroup, reduced by the quantiser below, instead of atomics on one word
        const int64_t nblk = update_blocks(d.N, d.K);
        uint32_t* wbmax = (uint32_t*)(base + w.off_wbmax);
        const bool per_block = nblk <= UPDATE_MAX_BLOCKS;
        if (per_block) u.block_max = wbmax;
        HIPCHK_T(FF_K_UPDATE, launch_update(u, s));

        QuantArgs qa;
        memset(&qa, 0, sizeof(qa));
        qa.x = state->w_master[t];
        qa.amax_bits = per_block ? wbmax : w_amax + t;
        qa.amax_n = per_block ? (int32_t)nblk : 0;
        qa.round_mode = FF_ROUND_NEAREST_EVEN;
        qa.rows = d.N;
        qa.cols = d.K;
        qa.q = state->w_q[t];
        qa.ldq = pitch8(d.K);
        qa.scale = state->s_w[t];
        qa.nb = 1;
        qa.rows_per_sample = 1;
        HIPCHK_T(FF_K_QUANT_W, launch_quantize(QSRC_F32, qa, s));
        return FF_OK;
    };
    auto trained = [&](int t) { return !net->train_layer || net->train_layer[t]; };

    if (w.chain) {
        // ---- Eq. (4) as an exact derivative: from the last layer down, the int8 gradient h_i is handed through the
        // pre-step weights of layer i to the layer below (dense layers only, checked by make_layout)
        uint32_t* h_amax = w_amax + k;        // [k][2]
        uint32_t* wt_amax = h_amax + 2 * k;   // [k]
        float* s_h = s_g + 2 * k;             // [2]
        float* s_wt = s_h + 2;                // scale of the transposed weight copy (equals s_w of the layer)
        float* hf = (float*)(base + w.off_hf);
        float* gf = (float*)(base + w.off_gf);
        const int64_t st_f = (int64_t)(w.st_f / sizeof(float));
        int8_t* hq = (int8_t*)(base + w.off_hq);
        int32_t* eacc = (int32_t*)(base + w.off_e);
        int8_t* wqt = (int8_t*)(base + w.off_wqt);
        for (int i = k - 1; i >= 0; --i) {
            const Dims& d = w.d[i];
            const ff_layer_desc& L = net->layers[i];
            ChainArgs ca;
            memset(&ca, 0, sizeof(ca));
            ca.acc = (const int32_t*)(base + w.off_acc[i]);
            ca.ldacc = pitch32(d.N);
            ca.st_acc = (int64_t)(w.st_acc[i] / sizeof(int32_t));
            ca.s_a = s_a + 2 * i;
            ca.st_s_a = 1;
            ca.s_w = state->s_w[i];
            ca.coeff = c + (int64_t)i * 2 * B;
            ca.st_coeff = B;
            if (i < k - 1) {
                ca.e_acc = eacc;
                ca.lde = pitch32(d.N);
                ca.st_e = (int64_t)(w.st_e / sizeof(int32_t));
                ca.s_h = s_h;
                ca.st_s_h = 1;
                ca.s_w_up = s_wt;   // pre-step weight scale of layer i + 1 (state->s_w[i + 1] already holds the updated one)
            }
            ca.lambda = lambda;
            ca.relu = L.relu ? 1 : 0;
            ca.M = d.M;
            ca.N = d.N;
            ca.h = i > 0 ? hf : nullptr;
            ca.g = gf;
            ca.st_out = st_f;
            ca.h_amax_bits = h_amax + 2 * i;
            ca.g_amax_bits = g_amax + 2 * i;
            ca.st_amax = 1;
            ca.nb = 2;
            // The last layer has nothing ahead of it: h = g = 2 c y, which the quantiser forms straight from the
            // accumulators (absmax by monotonicity, as in the default step); no fp32 tensors are written.
            const bool top = i == k - 1;
            int qsrc = QSRC_F32;
            QuantArgs a;
            memset(&a, 0, sizeof(a));
            if (top) {
                for (int p = 0; p < 2; ++p)
                    HIPCHK_T(FF_K_SMALL, launch_grad_amax(c + ((int64_t)i * 2 + p) * B, vmax + ((int64_t)i * 2 + p) * B,
                                                          s_a + 2 * i + p, state->s_w[i], B, g_amax + 2 * i + p, s));
                qsrc = QSRC_GRAD;
                a.acc = ca.acc;
                a.st_acc = ca.st_acc;
                a.ldacc = ca.ldacc;
                a.s_a = ca.s_a;
                a.st_s_a = 1;
                a.s_w = ca.s_w;
                a.per_sample = ca.coeff;
                a.st_per_sample = B;
                a.relu = ca.relu;
            } else {
                HIPCHK_T(FF_K_CHAIN, launch_chain_combine(ca, s));
                a.x = gf;
                a.st_x = st_f;
            }
            a.rows_per_sample = 1;
            a.amax_bits = g_amax + 2 * i;
            a.st_amax = 1;
            a.round_mode = FF_ROUND_STOCHASTIC;
            a.key = make_sr_key(seed, ff_stream_tag(step, (uint32_t)i, 0, FF_KIND_GRAD));
            a.key2 = make_sr_key(seed, ff_stream_tag(step, (uint32_t)i, 1, FF_KIND_GRAD));
            a.step_dev = step_dev;
            a.seed = seed;
            a.tag_layer = (uint32_t)i;
            a.tag_kind = FF_KIND_GRAD;
            a.rows = d.M;
            a.cols = d.N;
            a.q_t = (int8_t*)(base + w.off_gy);
            a.st_qt = (int64_t)w.st_gy;
            a.ldqt = pitch8(d.M);
            a.scale = s_g + 2 * i;
            a.st_scale = 1;
            a.nb = 2;
            if (trained(i)) HIPCHK_T(FF_K_QUANT_GRAD, launch_quantize(qsrc, a, s));

            if (i > 0) {
                QuantArgs hqa = a;
                if (!top) {
                    hqa.x = hf;
                    hqa.amax_bits = h_amax + 2 * i;
                }
                hqa.key = make_sr_key(seed, ff_stream_tag(step, (uint32_t)i, 0, FF_KIND_CHAIN));
                hqa.key2 = make_sr_key(seed, ff_stream_tag(step, (uint32_t)i, 1, FF_KIND_CHAIN));
                hqa.tag_kind = FF_KIND_CHAIN;
                hqa.q_t = nullptr;
                hqa.st_qt = 0;
                hqa.ldqt = 0;
                hqa.q = hq;
                hqa.st_q = (int64_t)w.st_hq;
                hqa.ldq = pitch8(d.N);
                hqa.scale = s_h;
                HIPCHK_T(FF_K_CHAIN, launch_quantize(qsrc, hqa, s));

                // transposed int8 copy of the pre-step weights: the same codes as w_q, [K, pitch(N)]
                const int64_t nw = d.N * d.K;
                HIPCHK_T(FF_K_CHAIN, launch_absmax(state->w_master[i], 0, 1, nw, wt_amax + i, s));
                QuantArgs wa;
                memset(&wa, 0, sizeof(wa));
                wa.x = state->w_master[i];
                wa.amax_bits = wt_amax + i;
                wa.round_mode = FF_ROUND_NEAREST_EVEN;
                wa.rows = d.N;
                wa.cols = d.K;
                wa.q_t = wqt;
                wa.ldqt = pitch8(d.N);
                wa.scale = s_wt;
                wa.nb = 1;
                wa.rows_per_sample = 1;
                HIPCHK_T(FF_K_CHAIN, launch_quantize(QSRC_F32, wa, s));

                GemmArgs ga;
                memset(&ga, 0, sizeof(ga));
                ga.P = hq;
                ga.Q = wqt;
                ga.C = eacc;
                ga.I = (int32_t)d.M;
                ga.J = (int32_t)d.K;
                ga.R = (int32_t)d.N;
                ga.ldp = pitch8(d.N);
                ga.ldq = pitch8(d.N);
                ga.ldc = pitch32(d.K);
                ga.nb = 2;
                ga.st_p = (int64_t)w.st_hq;
                ga.st_q = 0;
                ga.st_c = (int64_t)(w.st_e / sizeof(int32_t));
                ga.splits = 1;
                HIPCHK_T(FF_K_CHAIN, launch_gemm_nt_i8(ga, s));
            }
            if (trained(i)) {
                const ff_status us = wgrad_update(i, i);
                if (us != FF_OK) return us;
            }
        }
        if (step_dev && advance) HIPCHK_T(FF_K_SMALL, launch_advance_u64(step_dev, s));
        return FF_OK;
    }

    {
    Join join{pool, lane_stream, n_lanes};
    if (n_lanes > 1) {   // fork: the lanes start where the caller's stream stands now (all forward passes, the look-ahead)
        if (hipEventRecord(pool->fork, s) != hipSuccess) return FF_ERR_HIP;
        for (int l = 1; l < n_lanes; ++l)
            if (hipStreamWaitEvent(lane_stream[l], pool->fork, 0) != hipSuccess) return FF_ERR_HIP;
    }
    for (int i = 0; i < k; ++i) {
        const Dims& d = w.d[i];
        if (d.role == FF_ROLE_PROJECTION) continue;   // updated with the gradient of the block output, layer i + 2
        const bool with_proj = d.skip == FF_SKIP_PROJECTION && trained(i - 2);
        if (!trained(i) && !with_proj) continue;      // frozen layer: forward only
        const ff_layer_desc& L = net->layers[i];
        hipStream_t ls = lane_stream[lane_of[i]];
        char* const lbase = base + (size_t)lane_of[i] * w.lane_stride;   // this chain's copy of the scratch
        QuantArgs a;
        memset(&a, 0, sizeof(a));
        int src = QSRC_GRAD;
        if (d.skip != FF_SKIP_NONE) {
            src = QSRC_F32_GRAD;
            a.x = (const float*)(base + w.off_y[i]);
            a.st_x = (int64_t)(w.st_y[i] / sizeof(float));
        } else {
            a.acc = (const int32_t*)(base + w.off_acc[i]);
            a.st_acc = (int64_t)(w.st_acc[i] / sizeof(int32_t));
            a.ldacc = pitch32(d.N);
            a.s_a = s_a + 2 * i;
            a.st_s_a = 1;
            a.s_w = state->s_w[i];
        }
        a.per_sample = ct + (int64_t)i * 2 * B;
        a.st_per_sample = B;
        a.rows_per_sample = (int32_t)d.rps;
        a.relu = L.relu ? 1 : 0;
        a.amax_bits = g_amax + 2 * i;
        a.st_amax = 1;
        a.round_mode = FF_ROUND_STOCHASTIC;
        a.key = make_sr_key(seed, ff_stream_tag(step, (uint32_t)i, 0, FF_KIND_GRAD));
        a.key2 = make_sr_key(seed, ff_stream_tag(step, (uint32_t)i, 1, FF_KIND_GRAD));
        a.step_dev = step_dev;
        a.seed = seed;
        a.tag_layer = (uint32_t)i;
        a.tag_kind = FF_KIND_GRAD;
        a.rows = d.M;
        a.cols = d.N;
        if (d.kind == FF_DWCONV2D) {   // the depthwise weight gradient reads the gradient row-major
            a.q = (int8_t*)(lbase + w.off_gy);
            a.st_q = (int64_t)w.st_gy;
            a.ldq = pitch8(d.N);
        } else {
            a.q_t = (int8_t*)(lbase + w.off_gy);
            a.st_qt = (int64_t)w.st_gy;
            a.ldqt = pitch8(d.M);
        }
        a.scale = s_g + 2 * i;
        a.st_scale = 1;
        a.nb = 2;
        HIPCHK_T(FF_K_QUANT_GRAD, launch_quantize(src, a, ls));

        if (trained(i)) {
            const ff_status us = wgrad_update(i, i);
            if (us != FF_OK) return us;
        }
        if (with_proj) {
            const ff_status us = wgrad_update(i - 2, i);
            if (us != FF_OK) return us;
        }
    }
    const ff_status js = join.finish();
    if (js != FF_OK) return js;
    }
    if (step_dev && advance) HIPCHK_T(FF_K_SMALL, launch_advance_u64(step_dev, s));
    return FF_OK;
}

extern "C" {

ff_status ff_train_step(const ff_net_desc* net, const ff_net_state* state, const float* x_pos, const float* x_neg,
                        float theta, float lambda, float lr, uint64_t seed, uint64_t step, float* loss,
                        float* goodness, void* ws, size_t ws_bytes, void* stream)
{
    return train_step_impl(net, state, x_pos, x_neg, theta, lambda, lr, seed, step, nullptr, 0, loss, goodness, ws,
                           ws_bytes, stream);
}

ff_status ff_train_step_at(const ff_net_desc* net, const ff_net_state* state, const float* x_pos, const float* x_neg,
                           float theta, float lambda, float lr, uint64_t seed, uint64_t* step_dev, int32_t advance,
                           float* loss, float* goodness, void* ws, size_t ws_bytes, void* stream)
{
    if (!step_dev || ((uintptr_t)step_dev & 7)) return step_dev ? FF_ERR_ALIGN : FF_ERR_INVALID_ARG;
    return train_step_impl(net, state, x_pos, x_neg, theta, lambda, lr, seed, 0, step_dev, advance, loss, goodness, ws,
                           ws_bytes, stream);
}

ff_status ff_timing_enable(int32_t class_mask)
{
    g_timing.mask = (uint32_t)class_mask & ((1u << FF_K_COUNT) - 1u);
    return FF_OK;
}

ff_status ff_timing_clock_probe(uint64_t* counters)
{
    if (counters && ((uintptr_t)counters & 7)) return FF_ERR_ALIGN;
    g_clock_probe = (unsigned long long*)counters;
    return FF_OK;
}

ff_status ff_probe_mfma_ceiling(int32_t operand_kind, int32_t iterations, int32_t* sink, size_t sink_bytes,
                                uint64_t* counters, double* ops, void* stream)
{
    if (operand_kind < 0 || operand_kind > 2 || iterations < 1 || !sink || !ops) return FF_ERR_INVALID_ARG;
    if (!aligned4(sink) || (counters && ((uintptr_t)counters & 7))) return FF_ERR_ALIGN;
    const int g = num_cus();
    if (sink_bytes < (size_t)g * 512 * sizeof(int32_t)) return FF_ERR_WORKSPACE;
    int wgs = 0;
    if (launch_mfma_ceiling(sink, iterations, operand_kind, (unsigned long long*)counters, &wgs, (hipStream_t)stream) != hipSuccess)
        return FF_ERR_HIP;
    *ops = (double)wgs * 8.0 * (double)iterations * 8.0 * 65536.0;   // workgroups x wavefronts x iterations x MFMAs x ops
    return FF_OK;
}

ff_status ff_timing_fused_stamps(uint64_t* stamps)
{
    if (stamps && ((uintptr_t)stamps & 7)) return FF_ERR_ALIGN;
    g_fused_stamps = (unsigned long long*)stamps;
    return FF_OK;
}

ff_status ff_timing_reset(void)
{
    g_timing.n = 0;
    return FF_OK;
}

ff_status ff_timing_read(int32_t kernel_class, double* total_ms, int64_t* launches)
{
    if (!total_ms || !launches || kernel_class < 0 || kernel_class >= FF_K_COUNT) return FF_ERR_INVALID_ARG;
    double tot = 0.0;
    int64_t cnt = 0;
    for (int i = 0; i < g_timing.n; ++i) {
        if (g_timing.cls[i] != kernel_class) continue;
        if (hipEventSynchronize(g_timing.ev[2 * i + 1]) != hipSuccess) return FF_ERR_HIP;
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, g_timing.ev[2 * i], g_timing.ev[2 * i + 1]) != hipSuccess) return FF_ERR_HIP;
        tot += (double)ms;
        ++cnt;
    }
    *total_ms = tot;
    *launches = cnt;
    return FF_OK;
}

}  // extern "C"
