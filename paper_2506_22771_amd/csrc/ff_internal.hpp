// Internal declarations shared by the HIP translation units of libffint8 (gfx950 only).
// Host-side launchers are declared here; each is defined next to its kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/ffint8.h"

namespace ffi {

// ---- layout helpers -------------------------------------------------------------------------
// Row pitch of an int8 matrix in bytes: a multiple of 16 (the copy granule); rows longer than 512 bytes start on 128-byte
// lines, so that the 128-byte chunks the contraction copies per reduction step never straddle two cache lines (reduction
// lengths such as 784 or 2000 would otherwise cost every copy two line requests).  Kernels read a row only up to its
// length rounded up to 16; the bytes after that are padding that nothing reads.
__host__ __device__ static inline int64_t pitch8(int64_t cols)
{
    return cols <= 512 ? (cols + 15) & ~int64_t(15) : (cols + 127) & ~int64_t(127);
}
__host__ __device__ static inline int64_t pitch32(int64_t cols) { return (cols + 3) & ~int64_t(3); }
static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- stochastic-rounding key (Section IV-B cites stochastic rounding; the generator is ours) --
struct SrKey {
    uint32_t k0;  // low word of the 64-bit key
    uint32_t k1;  // (high word | 1), multiplies the high half of the element index
};
// key = finaliser of splitmix64 over (seed, stream tag); the same code runs on the host and, when the step
// number lives in device memory, at the head of the quantise kernels
__host__ __device__ inline SrKey make_sr_key(uint64_t seed, uint64_t tag)
{
    uint64_t z = seed + 0x9E3779B97F4A7C15ull * (tag + 1ull);
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    SrKey k;
    k.k0 = (uint32_t)z;
    k.k1 = (uint32_t)(z >> 32) | 1u;
    return k;
}
// stream tag of (step, layer, pass, kind): step << 20 | layer << 4 | pass << 2 | kind
__host__ __device__ inline uint64_t stream_tag_of(uint64_t step, uint32_t layer, uint32_t pass_idx, uint32_t kind)
{
    return (step << 20) | ((uint64_t)layer << 4) | ((uint64_t)pass_idx << 2) | (uint64_t)kind;
}

// ---- quantise kernels (elementwise.hip) -----------------------------------------------------
// QSRC_F32_GRAD: fp32 activities times the per-sample factor 2*coeff_total (local gradient of a residual layer)
enum QSource { QSRC_F32 = 0, QSRC_HANDOFF = 1, QSRC_GRAD = 2, QSRC_F32_GRAD = 3 };

// One quantisation problem; `nb` problems (1 or 2) are launched together with the strides below.
struct QuantArgs {
    // source
    const float* x;          // QSRC_F32: [rows, cols] contiguous
    const int32_t* acc;      // QSRC_HANDOFF / QSRC_GRAD: [rows, ldacc]
    int64_t ldacc;
    const float* s_a;        // device scalars (HANDOFF / GRAD)
    const float* s_w;
    const float* per_sample; // HANDOFF with l2norm: goodness[B]; GRAD, F32_GRAD: coeff_total[B]
    int32_t rows_per_sample;
    int32_t relu, l2norm;
    // quantiser
    const uint32_t* amax_bits;  // device: bit pattern of the non-negative fp32 absmax
    int32_t amax_n;             // > 1: amax_bits is an array of that many candidates, the absmax is their maximum
    int32_t round_mode;
    SrKey key;
    // destination
    int64_t rows, cols;
    int8_t* q;    // [rows, ldq] or null
    int64_t ldq;
    int8_t* q_t;  // [cols, ldqt] or null
    int64_t ldqt;
    int32_t qt_streaming;  // q_t is not read again soon: store it with a streaming hint
    float* scale;  // device scalar out
    // batching (second problem = first + strides, in elements of the respective type)
    int32_t nb;
    int64_t st_x, st_acc, st_per_sample, st_q, st_qt;
    int32_t st_s_a, st_s_w, st_amax, st_scale;
    SrKey key2;  // key of the second problem
    // step number in device memory (null: the keys above are used).  The kernel then derives its key from
    // (seed, stream tag of (*step_dev, tag_layer, problem index, tag_kind)).
    const uint64_t* step_dev;
    uint64_t seed;
    uint32_t tag_layer, tag_kind;
};
hipError_t launch_quantize(int src, const QuantArgs& a, hipStream_t s);

// absmax of |x| over n floats of tensor z (x + z*st_x, z < nb) into slot[z] (bit pattern, atomic max;
// slots must be zeroed first).
hipError_t launch_absmax(const float* x, int64_t st_x, int nb, int64_t n, uint32_t* slot, hipStream_t s);
hipError_t launch_fill_u32(uint32_t* p, int64_t n, uint32_t v, hipStream_t s);
hipError_t launch_advance_u64(uint64_t* counter, hipStream_t s);   // *counter += 1, in stream order

// ---- per-sample kernels ----------------------------------------------------------------------
struct GoodnessArgs {
    const unsigned long long* gsum;
    const int32_t* vmax;
    const float* s_a;
    const float* s_w;
    int32_t rshift, l2norm;
    int32_t pass_sign;  // sign of the first problem; the second problem (nb == 2) uses the opposite
    float theta;
    int64_t B;
    float* goodness;
    float* coeff;
    float* loss_mean;
    uint32_t* next_amax_bits;  // may be null
    // non-null: gsum holds the fixed-point sums of a residual layer, G = fp32(gsum * 2^-40 * amax^2) with amax
    // from this slot (stride st_scalar); s_a, s_w and vmax are then unused
    const uint32_t* fx_amax_bits;
    int32_t nb;
    int64_t st_b;  // stride between problems for the [B] arrays
    int32_t st_scalar;  // stride for s_a / loss_mean / next_amax (s_w is shared)
    // Optional (large batches): several workgroups per pass.  loss_part: [nb][GL_MAX_WG] partial loss sums, wg_counter:
    // [nb]; the counters and the next_amax slots must be zero on entry, and the kernel leaves the counters zero.  The
    // workgroup that finishes last adds the partial sums in index order, so the mean does not depend on timing.
    unsigned long long* loss_part;
    uint32_t* wg_counter;
};
constexpr int GL_MAX_WG = 32;
hipError_t launch_goodness_loss(const GoodnessArgs& a, hipStream_t s);

// coeff / coeff_total: [k][np][B] with strides; also (optionally) the absmax of each layer's local gradient.
struct LookaheadArgs {
    const float* coeff;
    float* coeff_total;
    int32_t k, np;
    int64_t B;
    int64_t st_layer, st_pass;
    float lambda;
    // optional gradient absmax (null vmax => skipped)
    const int32_t* vmax;       // same [k][np][B] strides
    const float* s_a;          // [k][np]
    const float* const* s_w;   // device array of k pointers to the layers' weight scales (may be null if vmax null)
    uint32_t* g_amax_bits;     // [k][np], zeroed
    uint32_t fx_mask;          // bit i: layer i's vmax entries are the fp32 bit patterns of max|y| (residual layer)
};
hipError_t launch_lookahead(const LookaheadArgs& a, hipStream_t s);

// ---- residual layers: block output y = act(s*acc + skip) as fp32, and its order-free goodness sums ------------
struct ResidualArgs {
    const int32_t* acc;  // [M, ldacc]
    int64_t ldacc, st_acc;
    const float* s_a;    // [z * st_s_a]
    const float* s_w;
    int32_t st_s_a;
    int32_t skip;        // FF_SKIP_IDENTITY / FF_SKIP_PROJECTION
    const int8_t* xq;    // identity: int8 [M, ldx] with scale s_x[z * st_s_x]
    int64_t ldx, st_xq;
    const float* s_x;
    int32_t st_s_x;
    const int32_t* accp; // projection: int32 [M, ldaccp] with scale s_ap[z * st_s_ap] * s_wp[0]
    int64_t ldaccp, st_accp;
    const float* s_ap;
    int32_t st_s_ap;
    const float* s_wp;
    int32_t relu;
    int64_t M, N;        // N % 4 == 0
    int32_t rows_per_sample;
    float* y;            // [M, N] contiguous
    int64_t st_y;
    uint32_t* ymax_bits; // [B] per pass (stride st_b), zeroed: bit pattern of max|y| per sample
    int64_t st_b;
    int32_t nb;
};
hipError_t launch_residual_act(const ResidualArgs& a, hipStream_t s);

struct GoodnessFxArgs {
    const float* y;      // [M, N] contiguous
    int64_t st_y;
    int64_t M, N;
    int32_t rows_per_sample;
    const uint32_t* ymax_bits; // [B] per pass (stride st_b): bit patterns of max|y| per sample
    uint32_t* amax_bits;       // slot per pass (stride st_amax), written: max|y| over the pass
    int32_t st_amax;
    unsigned long long* gsum;  // [B] per pass (stride st_b), zeroed
    int64_t st_b;
    int32_t nb;
};
hipError_t launch_goodness_fx(const GoodnessFxArgs& a, hipStream_t s);

// ---- exact-derivative look-ahead (Eq. (4) taken literally; dense ReLU stacks) -----------------------------------
// Per element of one layer and pass: y = act(fp32(acc) * (s_a*s_w)), t = (2 c[b]) * y, E = fp32(e_acc) * (s_h*s_w_up)
// (0 without e_acc: the last layer), mask = acc > 0 under ReLU:
//   h = (t + E) * mask          -- handed down to the layer below (null h: not needed, first layer)
//   g = fma(lambda, E, t) * mask -- this layer's own local gradient
// and the absmax of both tensors (bit patterns, atomic max into zeroed slots).
struct ChainArgs {
    const int32_t* acc;  // [M, ldacc]
    int64_t ldacc, st_acc;
    const float* s_a;    // [z * st_s_a]
    int32_t st_s_a;
    const float* s_w;
    const float* coeff;  // [B] per pass (stride st_coeff): dL/dG of THIS layer
    int64_t st_coeff;
    const int32_t* e_acc;  // [M, lde] or null
    int64_t lde, st_e;
    const float* s_h;      // [z * st_s_h]: scale of the int8 gradient handed down by the layer above
    int32_t st_s_h;
    const float* s_w_up;   // weight scale of the layer above
    float lambda;
    int32_t relu;
    int64_t M, N;
    float* h;  // [M, N] contiguous per pass (stride st_out), may be null
    float* g;  // [M, N] contiguous per pass
    int64_t st_out;
    uint32_t* h_amax_bits;  // [z * st_amax], zeroed; may be null with h
    uint32_t* g_amax_bits;
    int32_t st_amax;
    int32_t nb;
};
hipError_t launch_chain_combine(const ChainArgs& a, hipStream_t s);

// absmax of the local gradient for one layer / pass: max_b |2 c[b]| * (float(vmax[b]) * s_y) -> slot bits.
hipError_t launch_grad_amax(const float* coeff_total, const int32_t* vmax, const float* s_a,
                            const float* s_w, int64_t B, uint32_t* slot, hipStream_t s);

struct UpdateArgs {
    float* w;  // [N, K] contiguous
    int64_t N, K, lddw;
    int32_t n_terms;  // <= 4
    const int32_t* dw[4];
    const float* s_g[4];
    const float* s_a[4];
    float lr;
    int32_t total_samples;
    uint32_t* w_amax_bits;  // zeroed slot
    // Optional, for tensors of at most UPDATE_MAX_BLOCKS workgroups (update_blocks() below): every workgroup stores its
    // maximum here instead of meeting the others at w_amax_bits (hundreds of simultaneous atomics on one word cost
    // more than the rest of a small update); the quantiser that follows takes the maximum of the array
    // (QuantArgs::amax_n).
    uint32_t* block_max;
};
constexpr int UPDATE_MAX_BLOCKS = 1024;
int64_t update_blocks(int64_t N, int64_t K);   // workgroups launch_update starts for an [N, K] tensor
hipError_t launch_update(const UpdateArgs& a, hipStream_t s);

// ---- int8 contraction (gemm_i8.hip):  C[i][j] = sum_r P[i][r] * Q[j][r] -----------------------
struct GemmArgs {
    const int8_t* P;  // [I, ldp]
    const int8_t* Q;  // [J, ldq]
    int32_t* C;       // [I, ldc]
    int32_t I, J, R;  // R = reduction length in bytes (pad bytes beyond it are zero)
    int64_t ldp, ldq, ldc;
    // fused per-sample reductions (forward only; null gsum => plain contraction)
    unsigned long long* gsum;
    int32_t* vmax;
    int32_t rows_per_sample, relu, rshift;
    // batching over blockIdx.z
    int32_t nb;
    int64_t st_p, st_q, st_c, st_g;
    // split reduction (blockIdx.y): split s stores its partial sums at C + s*st_split; launch_reduce_splits
    // adds them up (integer sums: exact and order-free).  1 = no split.  Not combined with the fused reductions.
    int32_t splits;
    int64_t st_split;
    // implicit-GEMM convolution (conv != 0): P is an NHWC int8 tensor [B, H, W, cpitch] and row i of the
    // contraction is output pixel (b, ho, wo); reduction index r = (kh*ks + kw)*Cin + ci.  Cin % 16 == 0.
    // conv == 2: Q is a set of planes S[kw][ci][(b, h, wo)] (row pitch ldq bytes) written by launch_im2col with
    // wtaps_only; row j of the contraction is (kh, kw, ci), the reduction runs over output pixels.  W_out % 16 == 0.
    int32_t conv, H, W, Cin, cpitch, ks, stride, pad, Ho, Wo;
    int64_t p_bytes;  // bytes of one implicit operand tensor (conv only; must be < 2^31)
    // log2 of C_in (conv == 1), of H_out * W_out and of W_out (conv == 2) when those are powers of two, else -1: the
    // loaders then index with shifts instead of integer divisions.  Filled in by launch_gemm_nt_i8.
    int32_t cin_shift, hw_shift, wo_shift;
    // instrumentation (null normally): every workgroup adds the shader-clock cycles and the 100 MHz constant-clock
    // ticks it was alive to clk[0] and clk[1] (their ratio is the mean shader clock during the launch) and the
    // shader clocks of each tile by phase to clk[2..6] / clk[8..12]
    unsigned long long* clk;   // 16 counters, see ff_timing_clock_probe
};
hipError_t launch_gemm_nt_i8(const GemmArgs& a, hipStream_t s);
int num_cus();   // compute units of the current device (256 when the query fails)
// register-resident MFMA loop (see ff_probe_mfma_ceiling): one workgroup of 512 threads per compute unit
hipError_t launch_mfma_ceiling(int32_t* sink, int iters, int kind, unsigned long long* clk, int* workgroups, hipStream_t s);
struct GemmPlan {
    int bm, bn, splits;
};
GemmPlan gemm_plan(int64_t I, int64_t J, int64_t R, int nb, bool allow_split);
// out[z][e] = sum over s < splits of part[z][s][e], e < n (n a multiple of 4); strides in elements
hipError_t launch_reduce_splits(const int32_t* part, int splits, int64_t st_split, int64_t st_part_z, int32_t* out,
                                int64_t st_out_z, int64_t n, int nb, hipStream_t s);

// ---- single-launch step of a small dense stack (fused.hip) ---------------------------------------------------------
constexpr int FU_MAX_LAYERS = 8;
constexpr int FU_THREADS = 512;
constexpr int FU_MAX_B = 2 * FU_THREADS;   // samples per pass
struct FusedLayer {
    int32_t K, N, relu, l2norm, train, rshift;
    float theta;
    float* w;      // fp32 master weights [N, K]
    int8_t* wq;    // [N, pitch8(K)]
    float* sw;
    // workspace of the step, two passes each (strides in elements of the respective type)
    int8_t* aq;    int64_t st_aq;    // quantised layer input [B, pitch8(K)]
    int8_t* aqt;   int64_t st_aqt;   // its transposed copy [K, pitch8(B)]
    int32_t* acc;  int64_t st_acc;   // accumulators [B, pitch32(N)]
    int8_t* gy;    int64_t st_gy;    // transposed int8 local gradient [N, pitch8(B)]
};
struct FusedArgs {
    int32_t k, B;
    float lambda, lr;
    uint64_t seed, step;
    uint64_t* step_dev;   // null: `step` is used
    int32_t advance;
    const float* x;       // positive set; the negative set is st_x elements further on
    int64_t st_x;
    uint32_t* wg_amax;    // [workgroups]: per-workgroup absmax of the net input
    uint32_t* w_amax;     // [k]
    unsigned long long* gsum;   // [k][2][B]
    int32_t* vmax;        // [k][2][B]
    float* s_a;           // [k][2]
    float* s_g;           // [k][2]
    float* c;             // [k][2][B]
    float* ct;            // [k][2][B]
    float* goodness;      // [k][2][B]
    float* loss;          // [k][2]
    unsigned* bar;        // device-wide barrier counters (filled in by the launcher)
    unsigned long long* stamps;   // instrumentation, see ff_timing_fused_stamps (null normally)
    FusedLayer L[FU_MAX_LAYERS];
};
hipError_t launch_fused_dense_step(const FusedArgs& a, int workgroups, hipStream_t s);

// ---- explicit im2col (conv.hip) ----------------------------------------------------------------------
struct ConvGeom {
    int32_t H, W, Cin, cpitch, ks, stride, pad, Ho, Wo;
};
struct Im2colArgs {
    const int8_t* a;  // NHWC int8 [B, H, W, cpitch]
    int8_t* out;      // transposed: [K, ld_out] over samples [b0, b1); row-major: [(b1-b0)*Ho*Wo, ld_out]
    ConvGeom g;
    int32_t K, b0, b1;
    int64_t ld_out;
    int32_t nb;
    int64_t st_a, st_out;
    // transposed only: write the horizontal taps alone, as planes S[kw][ci][(b, h, wo)] over INPUT rows h:
    // S = A[b][h][wo * stride + kw - pad][ci], zero outside the image (K = ks * C_in rows of ld_out bytes)
    int32_t wtaps_only;
};
hipError_t launch_im2col(const Im2colArgs& p, bool transposed, hipStream_t s);
// ---- depthwise convolution (conv.hip): one ks x ks filter per channel, HBM-bound -----------------------------
struct DwArgs {
    const int8_t* a;    // NHWC int8 [B, H, W, cpitch]
    int64_t st_a;
    const int8_t* w_q;  // [C, 16]: nine taps (kh, kw) per channel, zero pad bytes
    ConvGeom g;         // Cin = C
    int32_t B;
    // forward
    int32_t* acc;       // [B*Ho*Wo, ldacc]
    int64_t ldacc, st_acc;
    unsigned long long* gsum;  // [B] per pass (stride st_g), zeroed; may be null
    int32_t* vmax;
    int64_t st_g;
    int32_t relu, rshift;
    // weight gradient over the samples [b0, b1)
    const int8_t* gy;   // row-major int8 local gradient [B*Ho*Wo, ldg]
    int64_t ldg, st_gy;
    int32_t* dw;        // [C, 12] int32, zeroed
    int64_t st_dw;
    int32_t b0, b1;
    int32_t nb;
};
hipError_t launch_dwconv_forward(const DwArgs& p, hipStream_t s);
hipError_t launch_dwconv_wgrad(const DwArgs& p, hipStream_t s);

// true when launch_im2col can write the planes for this geometry (LDS slab fits, grid limits)
bool im2col_planes_ok(const ConvGeom& g, int64_t nbatch_times_nb);

}  // namespace ffi
