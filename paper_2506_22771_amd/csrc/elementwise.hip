// HBM-bound kernels of the FF-INT8 layer step for gfx950: absmax, the int8 quantiser in its three
// source flavours (fp32 tensor, hand-off from accumulators, local gradient from accumulators),
// goodness / loss, look-ahead, and the weight update.
//
// Numerics follow the paper's Section IV (symmetric uniform quantiser), Section IV-B (stochastic
// rounding of the layer input, int8 local gradient), Eq. (1)/(2) (losses) and Eq. (3)/(4)
// (look-ahead).  Every fp32 operation that decides an int8 code is a single correctly rounded IEEE
// operation in a fixed order; this file must be compiled with -ffp-contract=off.
#include "ff_internal.hpp"
#include "device_math.hpp"

namespace ffi {

// Block-wide maximum of non-negative values' bit patterns, then one atomic per block.
template <int THREADS>
__device__ __forceinline__ void block_atomic_max_bits(uint32_t bits, uint32_t* slot)
{
    __shared__ uint32_t red[THREADS / 64];
    const uint32_t w = wave_max_u32(bits);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = w;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t m = red[0];
#pragma unroll
        for (int i = 1; i < THREADS / 64; ++i) m = max(m, red[i]);
        // thousands of workgroups target one word: skip the atomic when the slot already holds a larger value
        // (the slot only grows, so a stale read can only cause a harmless extra atomic)
        if (m != 0 && m > __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(slot, m);
    }
}

// ------------------------------------------------------------------------------------------------
// fill
// ------------------------------------------------------------------------------------------------
__global__ void k_fill_u32(uint32_t* p, int64_t n, uint32_t v)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = v;
}

hipError_t launch_fill_u32(uint32_t* p, int64_t n, uint32_t v, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(k_fill_u32, dim3((unsigned)blocks), dim3(256), 0, s, p, n, v);
    return hipGetLastError();
}

__global__ void k_advance_u64(uint64_t* counter)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) counter[0] += 1;
}

hipError_t launch_advance_u64(uint64_t* counter, hipStream_t s)
{
    hipLaunchKernelGGL(k_advance_u64, dim3(1), dim3(64), 0, s, counter);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// absmax of fp32 tensors -> bit pattern in slot[z] (HBM-bound: 4 bytes read per element).
// blockIdx.y selects the tensor (x + z*stride); four independent 16-byte loads per thread per trip.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t absbits4(const float4 v)
{
    const uint32_t a = max(__float_as_uint(v.x) & 0x7FFFFFFFu, __float_as_uint(v.y) & 0x7FFFFFFFu);
    const uint32_t b = max(__float_as_uint(v.z) & 0x7FFFFFFFu, __float_as_uint(v.w) & 0x7FFFFFFFu);
    return max(a, b);
}

typedef float f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 ldf4(const float4* p)   // streaming hint: the tensor is larger than the caches
{
    const f32x4 v = __builtin_nontemporal_load((const f32x4*)p);
    return make_float4(v.x, v.y, v.z, v.w);
}

__global__ __launch_bounds__(256) void k_absmax_f32(const float* __restrict__ x0, int64_t st_x, int64_t n,
                                                    uint32_t* __restrict__ slot)
{
    const float* __restrict__ x = x0 + (int64_t)blockIdx.y * st_x;
    // scalar head until 16-byte alignment, float4 body, scalar tail
    const uintptr_t addr = (uintptr_t)x;
    int64_t head = (int64_t)(((16 - (addr & 15)) & 15) >> 2);
    if (head > n) head = n;
    const int64_t nvec = (n - head) >> 2;
    const float4* __restrict__ xv = (const float4*)(x + head);
    const int64_t gtid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    uint32_t m = 0;
    // a workgroup walks contiguous 16 KB spans (measured: 6.2 TB/s against 5.5 TB/s for grid-strided loads)
    constexpr int64_t SPAN = 4 * 256;
    for (int64_t b = (int64_t)blockIdx.x * SPAN; b < nvec; b += (int64_t)gridDim.x * SPAN) {
        const int64_t i = b + threadIdx.x;
        const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
        const float4 v0 = i < nvec ? ldf4(xv + i) : z, v1 = i + 256 < nvec ? ldf4(xv + i + 256) : z;
        const float4 v2 = i + 512 < nvec ? ldf4(xv + i + 512) : z, v3 = i + 768 < nvec ? ldf4(xv + i + 768) : z;
        m = max(m, max(max(absbits4(v0), absbits4(v1)), max(absbits4(v2), absbits4(v3))));
    }
    if (gtid < head) m = max(m, __float_as_uint(x[gtid]) & 0x7FFFFFFFu);
    const int64_t tail0 = head + (nvec << 2);
    if (tail0 + gtid < n) m = max(m, __float_as_uint(x[tail0 + gtid]) & 0x7FFFFFFFu);
    block_atomic_max_bits<256>(m, slot + blockIdx.y);
}

hipError_t launch_absmax(const float* x, int64_t st_x, int nb, int64_t n, uint32_t* slot, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    int64_t blocks = (n + 256 * 16 - 1) / (256 * 16);
    if (blocks > 4096) blocks = 4096;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(k_absmax_f32, dim3((unsigned)blocks, (unsigned)nb), dim3(256), 0, s, x, st_x, n, slot);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// quantiser
// ------------------------------------------------------------------------------------------------
// 16-byte load of data that is not read again soon (source tensors of the quantisers): a streaming hint keeps it
// from displacing what the next kernels will read
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ld_stream16(const void* p)
{
    const u32x4 v = __builtin_nontemporal_load((const u32x4*)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}

constexpr int QT_THREADS = 256;
// Tile of one workgroup: CB column blocks of four columns, 2 x (256 / CB) row blocks of four rows: 128 x 64 elements
// for CB = 16, 256 x 32 for CB = 8 (matrices of at most 32 columns: no idle column lanes, and with a row pitch of
// 32 columns or fewer the tile is one contiguous span of memory).
template <int CB> struct QTile {
    static constexpr int COLS = 4 * CB;
    static constexpr int RH = 4 * (QT_THREADS / CB);   // rows of one half tile (u = 0 / 1)
    static constexpr int ROWS = 2 * RH;
    static constexpr int LDW = ROWS / 4 + 1;           // words per column in the transposed LDS tile (+1: bank spread)
    static constexpr int CHUNKS = ROWS / 16;           // 16-byte pieces of one transposed column
};

// Each thread owns two 4x4 element blocks (rows 4*rb+j, cols 4*cb+c).  Codes are packed four columns
// to a word for q, byte-transposed in registers for q_t and regrouped through LDS so that q_t is
// written in 16-byte pieces.  All eight 16-byte loads of a thread are issued before any arithmetic.
// VEC: 16-byte loads are legal (always for the int32 sources; for fp32 when cols % 4 == 0 and the base
// is 16-byte aligned).  Tensors have fewer than 2^32 elements (checked by the entry points), so the low
// word of the element index is the whole index.
template <int SRC, bool STOCH, bool VEC, int CB = 16>
__global__ __launch_bounds__(QT_THREADS) void k_quantize(QuantArgs a)
{
    constexpr int QT_ROWS = QTile<CB>::ROWS, QT_COLS = QTile<CB>::COLS, QT_LDW = QTile<CB>::LDW, QT_RH = QTile<CB>::RH;
    const int z = blockIdx.z;
    const float* __restrict__ x = a.x ? a.x + z * a.st_x : nullptr;
    const int32_t* __restrict__ acc = a.acc ? a.acc + z * a.st_acc : nullptr;
    const float* __restrict__ per_sample = a.per_sample ? a.per_sample + z * a.st_per_sample : nullptr;
    int8_t* __restrict__ q = a.q ? a.q + z * a.st_q : nullptr;
    int8_t* __restrict__ q_t = a.q_t ? a.q_t + z * a.st_qt : nullptr;
    SrKey key = z ? a.key2 : a.key;
    if (a.step_dev) key = make_sr_key(a.seed, stream_tag_of(a.step_dev[0], a.tag_layer, (uint32_t)z, a.tag_kind));

    // a vanishing range (absmax < 2^-100, all-zero tensor included) quantises to zero codes with scale 1
    uint32_t amax_word = a.amax_bits[z * a.st_amax];
    if (a.amax_n > 1) {   // (uniform) the producer left one candidate per workgroup
        __shared__ uint32_t amx[QT_THREADS / 64];
        uint32_t mm = 0;
        for (int i = threadIdx.x; i < a.amax_n; i += QT_THREADS) mm = max(mm, a.amax_bits[z * a.st_amax + i]);
        mm = wave_max_u32(mm);
        if ((threadIdx.x & 63) == 0) amx[threadIdx.x >> 6] = mm;
        __syncthreads();
        amax_word = max(max(amx[0], amx[1]), max(amx[2], amx[3]));
    }
    const float amax = __uint_as_float(amax_word);
    const bool live = amax >= 0x1p-100f;
    const float inv = live ? 127.0f / amax : 0.0f;
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0)
        a.scale[z * a.st_scale] = live ? amax / 127.0f : 1.0f;

    constexpr bool F32SRC = SRC == QSRC_F32 || SRC == QSRC_F32_GRAD;   // the source is an fp32 tensor
    float s_y = 1.0f;
    if (!F32SRC) s_y = a.s_a[z * a.st_s_a] * a.s_w[z * a.st_s_w];

    const int64_t r0 = (int64_t)blockIdx.y * QT_ROWS;
    const int64_t c0 = (int64_t)blockIdx.x * QT_COLS;
    const int t = threadIdx.x;
    const int cb = t & (CB - 1);
    const int64_t col = c0 + 4 * cb;
    const bool col_in = col < a.cols;

    __shared__ uint32_t tileT[QT_COLS * QT_LDW];

    // ---- loads: 2 blocks x 4 rows x 16 bytes, raw bits.  Row (u, j) of this thread is rowb + QT_RH*u + j:
    // all per-row offsets are (compile-time constant) x (uniform pitch), i.e. scalar-unit work.
    const int64_t rowb = r0 + 4 * (t / CB);
    const float* __restrict__ px0 = F32SRC ? x + rowb * a.cols + col : nullptr;
    const int32_t* __restrict__ pa0 = !F32SRC ? acc + rowb * a.ldacc + col : nullptr;
    int8_t* __restrict__ pq0 = q ? q + rowb * a.ldq + col : nullptr;
    uint32_t raw[2][4][4];
    float rowf[2][4];   // per-row factor (GRAD: 2*coeff; HANDOFF+l2norm: sqrt(goodness))
    const bool ragged = (a.cols & 3) != 0;   // the int32 sources' pad columns hold junk: mask them at load
#pragma unroll
    for (int u = 0; u < 2; ++u) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int dr = QT_RH * u + j;
            const int64_t row = rowb + dr;
            const bool in = row < a.rows && col_in;
            uint32_t w0 = 0, w1 = 0, w2 = 0, w3 = 0;
            if (F32SRC) {
                const float* px = px0 + (int64_t)dr * a.cols;
                if (VEC) {
                    if (in) {
                        const uint4 f = ld_stream16(px);
                        w0 = f.x; w1 = f.y; w2 = f.z; w3 = f.w;
                    }
                } else if (in) {
                    w0 = __float_as_uint(px[0]);
                    if (col + 1 < a.cols) w1 = __float_as_uint(px[1]);
                    if (col + 2 < a.cols) w2 = __float_as_uint(px[2]);
                    if (col + 3 < a.cols) w3 = __float_as_uint(px[3]);
                }
            } else if (in) {
                const uint4 f = ld_stream16(pa0 + (int64_t)dr * a.ldacc);  // pitch is a multiple of 4
                w0 = f.x; w1 = f.y; w2 = f.z; w3 = f.w;
                if (ragged) {
                    if (col + 1 >= a.cols) w1 = 0;
                    if (col + 2 >= a.cols) w2 = 0;
                    if (col + 3 >= a.cols) w3 = 0;
                }
            }
            raw[u][j][0] = w0; raw[u][j][1] = w1; raw[u][j][2] = w2; raw[u][j][3] = w3;
            float rf = 1.0f;
            if (SRC == QSRC_GRAD || SRC == QSRC_F32_GRAD || (SRC == QSRC_HANDOFF && a.l2norm)) {
                rf = 0.0f;
                if (in) {
                    const int64_t smp = a.rows_per_sample == 1 ? row : row / a.rows_per_sample;
                    rf = SRC == QSRC_HANDOFF ? sqrtf(per_sample[smp]) : 2.0f * per_sample[smp];
                }
            }
            rowf[u][j] = rf;
        }
    }

    // ---- quantise
    const uint64_t idx0 = (uint64_t)rowb * (uint64_t)a.cols + (uint64_t)col;   // element index of (row rowb, col)
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int rb = (t / CB) + (QT_THREADS / CB) * u;
        uint32_t rowpack[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int dr = QT_RH * u + j;
            const int64_t row = rowb + dr;
            const uint32_t base_lo = (uint32_t)idx0 + (uint32_t)dr * (uint32_t)a.cols;
            uint32_t pack = 0;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                float v = F32SRC ? __uint_as_float(raw[u][j][c]) : (float)(int)raw[u][j][c];
                if (SRC == QSRC_F32_GRAD) v = rowf[u][j] * v;
                if (!F32SRC) {
                    v = v * s_y;
                    if (a.relu) v = fmaxf(v, 0.0f);
                    if (SRC == QSRC_GRAD) v = rowf[u][j] * v;
                    else if (a.l2norm) v = rowf[u][j] > 0.0f ? v / rowf[u][j] : 0.0f;
                }
                // elements outside the tensor were loaded as zero and a dead range has inv == 0: in both
                // cases t == 0, so the code is 0 in either rounding mode without any masking
                const int code = quant_code<STOCH>(v, inv, (base_lo + (uint32_t)c) ^ key.k0);
                pack |= ((uint32_t)code & 0xFFu) << (8 * c);
            }
            rowpack[j] = pack;
            if (q && row < a.rows && col < a.ldq) *(uint32_t*)(pq0 + (int64_t)dr * a.ldq) = pack;
        }
        if (q_t) {
            // 4x4 byte transpose: colpack[c] = byte c of rowpack[0..3]
            const uint32_t t0 = __builtin_amdgcn_perm(rowpack[1], rowpack[0], 0x05010400u);
            const uint32_t t1 = __builtin_amdgcn_perm(rowpack[1], rowpack[0], 0x07030602u);
            const uint32_t t2 = __builtin_amdgcn_perm(rowpack[3], rowpack[2], 0x05010400u);
            const uint32_t t3 = __builtin_amdgcn_perm(rowpack[3], rowpack[2], 0x07030602u);
            tileT[(4 * cb + 0) * QT_LDW + rb] = __builtin_amdgcn_perm(t2, t0, 0x05040100u);
            tileT[(4 * cb + 1) * QT_LDW + rb] = __builtin_amdgcn_perm(t2, t0, 0x07060302u);
            tileT[(4 * cb + 2) * QT_LDW + rb] = __builtin_amdgcn_perm(t3, t1, 0x05040100u);
            tileT[(4 * cb + 3) * QT_LDW + rb] = __builtin_amdgcn_perm(t3, t1, 0x07060302u);
        }
    }
    if (q_t) {
        __syncthreads();
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int e = t + QT_THREADS * u;
            const int cl = e / QTile<CB>::CHUNKS, ch = e % QTile<CB>::CHUNKS;
            const int64_t oc = c0 + cl;
            const int64_t orow = r0 + 16 * ch;
            if (oc < a.cols && orow < a.ldqt) {
                int4 o;
                o.x = (int)tileT[cl * QT_LDW + 4 * ch + 0];
                o.y = (int)tileT[cl * QT_LDW + 4 * ch + 1];
                o.z = (int)tileT[cl * QT_LDW + 4 * ch + 2];
                o.w = (int)tileT[cl * QT_LDW + 4 * ch + 3];
                // the transposed copy of a layer input is read by the weight-gradient contraction much later
                // (streaming store); that of a local gradient right away
                if (a.qt_streaming) __builtin_nontemporal_store((u32x4){(uint32_t)o.x, (uint32_t)o.y, (uint32_t)o.z, (uint32_t)o.w}, (u32x4*)(q_t + oc * a.ldqt + orow));
                else *(int4*)(q_t + oc * a.ldqt + orow) = o;
            }
        }
    }
}

template <int SRC, bool STOCH>
static void launch_quantize_t(const QuantArgs& a, hipStream_t s)
{
    const dim3 block(QT_THREADS);
    bool vec = true;
    if (SRC == QSRC_F32 || SRC == QSRC_F32_GRAD) {
        vec = (a.cols & 3) == 0 && (((uintptr_t)a.x) & 15) == 0 && ((a.st_x & 3) == 0 || a.nb == 1);
    }
    if (a.cols <= QTile<8>::COLS && vec) {
        const dim3 grid(1, (unsigned)((a.rows + QTile<8>::ROWS - 1) / QTile<8>::ROWS), (unsigned)a.nb);
        hipLaunchKernelGGL((k_quantize<SRC, STOCH, true, 8>), grid, block, 0, s, a);
        return;
    }
    // (column tiles up to the row pitch of q, so that its pad bytes are written too: zeros)
    const int64_t span = a.q && a.ldq > a.cols ? a.ldq : a.cols;
    const dim3 grid((unsigned)((span + QTile<16>::COLS - 1) / QTile<16>::COLS),
                    (unsigned)((a.rows + QTile<16>::ROWS - 1) / QTile<16>::ROWS), (unsigned)a.nb);
    if (vec) hipLaunchKernelGGL((k_quantize<SRC, STOCH, true>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((k_quantize<SRC, STOCH, SRC != QSRC_F32 && SRC != QSRC_F32_GRAD>), grid, block, 0, s, a);
}

hipError_t launch_quantize(int src, const QuantArgs& a, hipStream_t s)
{
    if (a.rows <= 0 || a.cols <= 0) return hipSuccess;
    const bool st = a.round_mode == FF_ROUND_STOCHASTIC;
    switch (src) {
        case QSRC_F32:
            if (st) launch_quantize_t<QSRC_F32, true>(a, s);
            else launch_quantize_t<QSRC_F32, false>(a, s);
            break;
        case QSRC_HANDOFF:
            if (st) launch_quantize_t<QSRC_HANDOFF, true>(a, s);
            else launch_quantize_t<QSRC_HANDOFF, false>(a, s);
            break;
        case QSRC_F32_GRAD:
            if (st) launch_quantize_t<QSRC_F32_GRAD, true>(a, s);
            else launch_quantize_t<QSRC_F32_GRAD, false>(a, s);
            break;
        default:
            if (st) launch_quantize_t<QSRC_GRAD, true>(a, s);
            else launch_quantize_t<QSRC_GRAD, false>(a, s);
            break;
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// goodness, loss, dL/dG, absmax of the hand-off tensor: one workgroup per pass, fixed reduction order
// ------------------------------------------------------------------------------------------------
constexpr int GL_THREADS = 1024;

__global__ __launch_bounds__(GL_THREADS) void k_goodness_loss(GoodnessArgs a)
{
    const int z = blockIdx.x;
    const unsigned long long* gsum = a.gsum + z * a.st_b;
    const int32_t* vmax = a.vmax + z * a.st_b;
    float* goodness = a.goodness + z * a.st_b;
    float* coeff = a.coeff + z * a.st_b;
    const int sign = z ? -a.pass_sign : a.pass_sign;
    const bool fx = a.fx_amax_bits != nullptr;
    const float s_y = fx ? 1.0f : a.s_a[z * a.st_scalar] * a.s_w[0];
    const float fx_amax = fx ? __uint_as_float(a.fx_amax_bits[z * a.st_scalar]) : 0.0f;
    const double s_yd = fx ? (double)fx_amax : (double)s_y;
    const double pow2r = fx ? 0x1p-40 : (double)(1ull << a.rshift);

    double lsum = 0.0;
    uint32_t amax_bits = 0;
    const int wg = blockIdx.y, nwg = gridDim.y;
    for (int64_t b = (int64_t)wg * GL_THREADS + threadIdx.x; b < a.B; b += (int64_t)nwg * GL_THREADS) {
        double g = (double)gsum[b];
        g = g * pow2r;
        g = g * s_yd;
        g = g * s_yd;
        const float G = (fx && fx_amax < 0x1p-100f) ? 0.0f : (float)g;
        goodness[b] = G;
        const float x = G - a.theta;
        const float e = exp_nonpos(-fabsf(x));
        const float den = 1.0f + e;
        const float sig_big = 1.0f / den;
        const float sig_small = e / den;
        float c, xs;
        if (sign > 0) {
            c = -(x >= 0.0f ? sig_small : sig_big);
            xs = -x;
        } else {
            c = (x >= 0.0f ? sig_big : sig_small);
            xs = x;
        }
        coeff[b] = c;
        // the reported loss (softplus) is not fed back into anything: fp32 terms, summed in fp64
        lsum += (double)(fmaxf(xs, 0.0f) + log1pf(expf(-fabsf(xs))));
        if (a.next_amax_bits) {
            float ymax = (float)vmax[b] * s_y;
            if (a.l2norm) {
                const float nrm = sqrtf(G);
                ymax = nrm > 0.0f ? ymax / nrm : 0.0f;
            }
            amax_bits = max(amax_bits, __float_as_uint(ymax));
        }
    }
    __shared__ double red[GL_THREADS];
    __shared__ uint32_t redm[GL_THREADS];
    red[threadIdx.x] = lsum;
    redm[threadIdx.x] = amax_bits;
    __syncthreads();
    for (int s = GL_THREADS / 2; s > 0; s >>= 1) {
        if (threadIdx.x < s) {
            red[threadIdx.x] += red[threadIdx.x + s];
            redm[threadIdx.x] = max(redm[threadIdx.x], redm[threadIdx.x + s]);
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        if (nwg == 1) {
            a.loss_mean[z * a.st_scalar] = a.B > 0 ? (float)(red[0] / (double)a.B) : 0.0f;
            if (a.next_amax_bits) a.next_amax_bits[z * a.st_scalar] = redm[0];
        } else {
            if (a.next_amax_bits && redm[0]) atomicMax(a.next_amax_bits + z * a.st_scalar, redm[0]);
            unsigned long long* part = a.loss_part + z * GL_MAX_WG;
            __hip_atomic_store(part + wg, (unsigned long long)__double_as_longlong(red[0]), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
            __threadfence();
            if (atomicAdd(a.wg_counter + z, 1u) == (unsigned)(nwg - 1)) {
                // last workgroup of this pass: every partial sum has been published; add them in index order
                __threadfence();
                double t = 0.0;
                for (int i = 0; i < nwg; ++i)
                    t += __longlong_as_double((long long)__hip_atomic_load(part + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
                a.loss_mean[z * a.st_scalar] = (float)(t / (double)a.B);
                __hip_atomic_store(a.wg_counter + z, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

hipError_t launch_goodness_loss(const GoodnessArgs& a, hipStream_t s)
{
    // one workgroup of 1024 threads per pass, or (large batches, scratch given) one per 1024 samples
    int nwg = 1;
    if (a.loss_part && a.wg_counter && a.B >= 2 * GL_THREADS) nwg = (int)min((int64_t)GL_MAX_WG, (a.B + GL_THREADS - 1) / GL_THREADS);
    hipLaunchKernelGGL(k_goodness_loss, dim3((unsigned)a.nb, (unsigned)nwg), dim3(GL_THREADS), 0, s, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// residual layers: block output y = act(fp32(acc) * s_y + skip), one rounding per operation, stored as
// fp32; max|y| per sample and over the pass (bit patterns, atomic max).  A thread owns four columns.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v)
{
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const unsigned lo = (unsigned)__shfl_xor((int)(unsigned)v, d), hi = (unsigned)__shfl_xor((int)(unsigned)(v >> 32), d);
        v += ((unsigned long long)hi << 32) | lo;
    }
    return v;
}

// Work split of the two residual kernels: blockIdx.y = sample, blockIdx.x = a contiguous share of the sample's
// terms (RES_VPT four-element vectors per thread), blockIdx.z = pass.  A workgroup therefore reduces for ONE
// sample and issues one atomic.
constexpr int RES_VPT = 4;

template <typename T, typename F>
__device__ __forceinline__ T block_reduce_256(T v, F op, T* red)
{
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return op(op(red[0], red[1]), op(red[2], red[3]));
}

__global__ __launch_bounds__(256) void k_residual_act(ResidualArgs a)
{
    const int z = blockIdx.z;
    const int64_t smp = blockIdx.y;
    const int N = (int)a.N;
    const int tv = a.rows_per_sample * (N >> 2);   // vectors per sample
    const float s_y = a.s_a[z * a.st_s_a] * a.s_w[0];
    const float s_u = a.skip == FF_SKIP_IDENTITY ? a.s_x[z * a.st_s_x] : a.s_ap[z * a.st_s_ap] * a.s_wp[0];
    const int64_t row0 = smp * a.rows_per_sample;
    uint32_t m = 0;
#pragma unroll
    for (int it = 0; it < RES_VPT; ++it) {
        const int v = ((int)blockIdx.x * RES_VPT + it) * 256 + (int)threadIdx.x;
        if (v >= tv) break;
        const int e = v * 4;
        const int r = e / N, col = e - r * N;
        const int64_t row = row0 + r;
        // the accumulators of a residual layer are not read again (everything downstream uses y): streaming hint
        const uint4 cw = ld_stream16(a.acc + z * a.st_acc + row * a.ldacc + col);
        const int4 c = make_int4((int)cw.x, (int)cw.y, (int)cw.z, (int)cw.w);
        float u[4];
        if (a.skip == FF_SKIP_IDENTITY) {
            const uint32_t xw = *(const uint32_t*)(a.xq + z * a.st_xq + row * a.ldx + col);
#pragma unroll
            for (int q = 0; q < 4; ++q) u[q] = (float)(int)(int8_t)(xw >> (8 * q)) * s_u;
        } else {
            const int4 cp = *(const int4*)(a.accp + z * a.st_accp + row * a.ldaccp + col);
            u[0] = (float)cp.x * s_u; u[1] = (float)cp.y * s_u; u[2] = (float)cp.z * s_u; u[3] = (float)cp.w * s_u;
        }
        const int cc[4] = {c.x, c.y, c.z, c.w};
        float yv[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float t = (float)cc[q] * s_y;
            float w = t + u[q];
            if (a.relu) w = fmaxf(w, 0.0f);
            yv[q] = w;
            m = max(m, __float_as_uint(fabsf(w)));
        }
        *(float4*)(a.y + z * a.st_y + row * N + col) = make_float4(yv[0], yv[1], yv[2], yv[3]);
    }
    __shared__ uint32_t red[4];
    const uint32_t bm = block_reduce_256(wave_max_u32(m), [](uint32_t x, uint32_t y) { return max(x, y); }, red);
    if (threadIdx.x == 0 && bm) atomicMax(a.ymax_bits + z * a.st_b + smp, bm);
}

hipError_t launch_residual_act(const ResidualArgs& a, hipStream_t s)
{
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    const int64_t tv = (int64_t)a.rows_per_sample * (a.N >> 2);
    const int64_t B = a.M / a.rows_per_sample;
    const unsigned bx = (unsigned)((tv + 256 * RES_VPT - 1) / (256 * RES_VPT));
    if (B > 65535 || tv > (int64_t(1) << 28)) return hipErrorInvalidValue;   // grid y limit; 32-bit in-sample offsets
    hipLaunchKernelGGL(k_residual_act, dim3(bx, (unsigned)B, (unsigned)a.nb), dim3(256), 0, s, a);
    return hipGetLastError();
}

// Fixed-point goodness sums of an fp32 activity tensor: per element floor(r * r * 2^40), r = y * (1 / amax) in
// fp32, the product in fp64 (exact); unsigned 64-bit integer sums per sample (order-free).  amax is the maximum
// of the per-sample maxima, recomputed by every workgroup; workgroup (0, 0) of a pass also stores it to the slot
// the quantisers of the next layers read.
__global__ __launch_bounds__(256) void k_goodness_fx(GoodnessFxArgs a)
{
    const int z = blockIdx.z;
    const int64_t smp = blockIdx.y;
    const int64_t B = gridDim.y;
    __shared__ uint32_t redm[4];
    __shared__ unsigned long long reds[4];
    uint32_t mb = 0;
    for (int64_t b = threadIdx.x; b < B; b += 256) mb = max(mb, a.ymax_bits[z * a.st_b + b]);
    mb = block_reduce_256(wave_max_u32(mb), [](uint32_t x, uint32_t y) { return max(x, y); }, redm);
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) a.amax_bits[z * a.st_amax] = mb;
    const float amax = __uint_as_float(mb);
    const float inv = amax >= 0x1p-100f ? 1.0f / amax : 0.0f;
    const int64_t tv = (int64_t)a.rows_per_sample * (a.N >> 2);
    const float* ys = a.y + z * a.st_y + smp * tv * 4;
    unsigned long long q = 0;
#pragma unroll
    for (int it = 0; it < RES_VPT; ++it) {
        const int64_t v = ((int64_t)blockIdx.x * RES_VPT + it) * 256 + threadIdx.x;
        if (v >= tv) break;
        const float4 w = *(const float4*)(ys + v * 4);
        const float ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float r = ww[e] * inv;
            q += (unsigned long long)((double)r * (double)r * 0x1p40);
        }
    }
    const unsigned long long t =
        block_reduce_256(wave_sum_u64(q), [](unsigned long long x, unsigned long long y) { return x + y; }, reds);
    if (threadIdx.x == 0 && t) atomicAdd(a.gsum + z * a.st_b + smp, t);
}

hipError_t launch_goodness_fx(const GoodnessFxArgs& a, hipStream_t s)
{
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    const int64_t tv = (int64_t)a.rows_per_sample * (a.N >> 2);
    const int64_t B = a.M / a.rows_per_sample;
    const unsigned bx = (unsigned)((tv + 256 * RES_VPT - 1) / (256 * RES_VPT));
    if (B > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_goodness_fx, dim3(bx, (unsigned)B, (unsigned)a.nb), dim3(256), 0, s, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// look-ahead (Eq. (3)/(4)): per sample, walk the layers from the last to the first
// ------------------------------------------------------------------------------------------------
struct LookaheadKArgs {
    LookaheadArgs a;
    const float* s_w[32];
};

__global__ __launch_bounds__(256) void k_lookahead(LookaheadKArgs ka)
{
    const LookaheadArgs& a = ka.a;
    const int p = blockIdx.y;
    const int64_t b = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const bool live = b < a.B;
    float S = 0.0f;
    for (int i = a.k - 1; i >= 0; --i) {
        const int64_t off = i * a.st_layer + p * a.st_pass + (live ? b : 0);
        const float c = live ? a.coeff[off] : 0.0f;
        const float ct = __builtin_fmaf(a.lambda, S, c);
        S = S + c;
        if (live) a.coeff_total[off] = ct;
        if (a.vmax) {
            uint32_t bits = 0;
            if (live) {
                float ymax;
                if ((a.fx_mask >> i) & 1u) {
                    ymax = __uint_as_float((uint32_t)a.vmax[off]);
                } else {
                    const float s_y = a.s_a[i * a.np + p] * ka.s_w[i][0];
                    ymax = (float)a.vmax[off] * s_y;
                }
                bits = __float_as_uint(fabsf(2.0f * ct) * ymax);
            }
            bits = wave_max_u32(bits);
            if ((threadIdx.x & 63) == 0 && bits) atomicMax(a.g_amax_bits + i * a.np + p, bits);
        }
    }
}

hipError_t launch_lookahead_impl(const LookaheadArgs& a, const float* const* s_w_host, hipStream_t s)
{
    LookaheadKArgs ka;
    ka.a = a;
    for (int i = 0; i < 32; ++i) ka.s_w[i] = (s_w_host && i < a.k) ? s_w_host[i] : nullptr;
    hipLaunchKernelGGL(k_lookahead, dim3((unsigned)((a.B + 255) / 256), (unsigned)a.np), dim3(256), 0, s, ka);
    return hipGetLastError();
}

hipError_t launch_lookahead(const LookaheadArgs& a, hipStream_t s)
{
    // a.s_w is a HOST array of device pointers here; they travel in the kernel argument block
    return launch_lookahead_impl(a, a.s_w, s);
}

__global__ __launch_bounds__(1024) void k_grad_amax(const float* __restrict__ ct, const int32_t* __restrict__ vmax,
                                                    const float* __restrict__ s_a, const float* __restrict__ s_w,
                                                    int64_t B, uint32_t* __restrict__ slot)
{
    const float s_y = s_a[0] * s_w[0];
    uint32_t bits = 0;
    for (int64_t b = threadIdx.x; b < B; b += 1024) {
        const float ymax = (float)vmax[b] * s_y;
        bits = max(bits, __float_as_uint(fabsf(2.0f * ct[b]) * ymax));
    }
    __shared__ uint32_t red[16];
    bits = wave_max_u32(bits);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = bits;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t m = 0;
        for (int i = 0; i < 16; ++i) m = max(m, red[i]);
        *slot = m;
    }
}

hipError_t launch_grad_amax(const float* ct, const int32_t* vmax, const float* s_a, const float* s_w, int64_t B,
                            uint32_t* slot, hipStream_t s)
{
    hipLaunchKernelGGL(k_grad_amax, dim3(1), dim3(1024), 0, s, ct, vmax, s_a, s_w, B, slot);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Exact-derivative look-ahead: the two gradients of a dense layer (see ChainArgs).  A thread owns four
// consecutive columns of one row; HBM-bound (two int32 tensors read, two fp32 tensors written).
// ------------------------------------------------------------------------------------------------
template <bool VEC>
__global__ __launch_bounds__(256) void k_chain_combine(ChainArgs a)
{
    const int z = blockIdx.y;
    const int64_t ngroups = (a.N + 3) >> 2;
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    uint32_t mh = 0, mg = 0;
    if (e < a.M * ngroups) {
        const int64_t m = e / ngroups;
        const int64_t j0 = (e - m * ngroups) << 2;
        const float s_y = a.s_a[z * a.st_s_a] * a.s_w[0];
        const float s_e = a.e_acc ? a.s_h[z * a.st_s_h] * a.s_w_up[0] : 0.0f;
        const float d = 2.0f * a.coeff[z * a.st_coeff + m];
        const uint4 av = ld_stream16(a.acc + z * a.st_acc + m * a.ldacc + j0);
        uint4 ev = make_uint4(0u, 0u, 0u, 0u);
        if (a.e_acc) ev = ld_stream16(a.e_acc + z * a.st_e + m * a.lde + j0);
        const int ai[4] = {(int)av.x, (int)av.y, (int)av.z, (int)av.w};
        const int ei[4] = {(int)ev.x, (int)ev.y, (int)ev.z, (int)ev.w};
        float hv[4], gv[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            float y = (float)ai[c] * s_y;
            if (a.relu && y < 0.0f) y = 0.0f;
            const float t = d * y;
            const float E = a.e_acc ? (float)ei[c] * s_e : 0.0f;
            const bool live = (!a.relu || ai[c] > 0) && j0 + c < a.N;
            hv[c] = live ? t + E : 0.0f;
            gv[c] = live ? __builtin_fmaf(a.lambda, E, t) : 0.0f;
            mh = max(mh, __float_as_uint(hv[c]) & 0x7FFFFFFFu);
            mg = max(mg, __float_as_uint(gv[c]) & 0x7FFFFFFFu);
        }
        float* gp = a.g + z * a.st_out + m * a.N + j0;
        float* hp = a.h ? a.h + z * a.st_out + m * a.N + j0 : nullptr;
        if (VEC) {
            *(float4*)gp = make_float4(gv[0], gv[1], gv[2], gv[3]);
            if (hp) *(float4*)hp = make_float4(hv[0], hv[1], hv[2], hv[3]);
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (j0 + c < a.N) {
                    gp[c] = gv[c];
                    if (hp) hp[c] = hv[c];
                }
        }
    }
    block_atomic_max_bits<256>(mg, a.g_amax_bits + z * a.st_amax);
    if (a.h) {
        __syncthreads();   // the reduction buffer of the first call is read by thread 0 until here
        block_atomic_max_bits<256>(mh, a.h_amax_bits + z * a.st_amax);
    }
}

hipError_t launch_chain_combine(const ChainArgs& a, hipStream_t s)
{
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    const int64_t total = a.M * ((a.N + 3) >> 2);
    const int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks, (unsigned)a.nb);
    const bool vec = (a.N & 3) == 0 && ((((uintptr_t)a.g) & 15) == 0) && (!a.h || (((uintptr_t)a.h) & 15) == 0) &&
                     (a.st_out & 3) == 0;
    if (vec) hipLaunchKernelGGL(k_chain_combine<true>, grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL(k_chain_combine<false>, grid, dim3(256), 0, s, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// weight update (HBM-bound: 4 B x (1 + n_terms) read + 4 B written per weight) with fused absmax.
// One workgroup per (row, 4096-column segment); a thread owns four groups of four columns, 256 groups
// apart, and issues all of its loads before the arithmetic.
// ------------------------------------------------------------------------------------------------
constexpr int UP_SEG = 4096;

template <bool VEC>
__global__ __launch_bounds__(256) void k_update(UpdateArgs a)
{
    float sc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) sc[j] = j < a.n_terms ? a.s_g[j][0] * a.s_a[j][0] : 0.0f;
    const float lr_eff = a.lr / (float)a.total_samples;
    const int64_t kbase = (int64_t)blockIdx.x * UP_SEG + 4 * threadIdx.x;
    uint32_t m = 0;
    for (int64_t n = blockIdx.y; n < a.N; n += gridDim.y) {
        float* __restrict__ wrow = a.w + n * a.K;
        float w[4][4];
        int4 d[4][4];
        int cnt[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int64_t k = kbase + g * 1024;
            cnt[g] = (int)max((int64_t)0, min((int64_t)4, a.K - k));
            if (VEC) {
                float4 f = make_float4(0.f, 0.f, 0.f, 0.f);
                if (cnt[g]) f = *(const float4*)(wrow + k);
                w[g][0] = f.x; w[g][1] = f.y; w[g][2] = f.z; w[g][3] = f.w;
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) w[g][c] = c < cnt[g] ? wrow[k + c] : 0.0f;
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                d[g][j] = make_int4(0, 0, 0, 0);
                if (j < a.n_terms && cnt[g]) {   // last use of the accumulators: streaming hint
                    const uint4 v = ld_stream16(a.dw[j] + n * a.lddw + k);
                    d[g][j] = make_int4((int)v.x, (int)v.y, (int)v.z, (int)v.w);
                }
            }
        }
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int64_t k = kbase + g * 1024;
            float gr[4];
            gr[0] = (float)d[g][0].x * sc[0]; gr[1] = (float)d[g][0].y * sc[0];
            gr[2] = (float)d[g][0].z * sc[0]; gr[3] = (float)d[g][0].w * sc[0];
#pragma unroll
            for (int j = 1; j < 4; ++j) {
                if (j < a.n_terms) {
                    gr[0] = __builtin_fmaf((float)d[g][j].x, sc[j], gr[0]);
                    gr[1] = __builtin_fmaf((float)d[g][j].y, sc[j], gr[1]);
                    gr[2] = __builtin_fmaf((float)d[g][j].z, sc[j], gr[2]);
                    gr[3] = __builtin_fmaf((float)d[g][j].w, sc[j], gr[3]);
                }
            }
#pragma unroll
            for (int c = 0; c < 4; ++c) w[g][c] = __builtin_fmaf(-lr_eff, gr[c], w[g][c]);
            if (VEC) {
                if (cnt[g]) {
                    *(float4*)(wrow + k) = make_float4(w[g][0], w[g][1], w[g][2], w[g][3]);
#pragma unroll
                    for (int c = 0; c < 4; ++c) m = max(m, __float_as_uint(w[g][c]) & 0x7FFFFFFFu);
                }
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (c < cnt[g]) {
                        wrow[k + c] = w[g][c];
                        m = max(m, __float_as_uint(w[g][c]) & 0x7FFFFFFFu);
                    }
            }
        }
    }
    if (a.block_max) {
        m = wave_max_u32(m);
        __shared__ uint32_t bm[4];
        if ((threadIdx.x & 63) == 0) bm[threadIdx.x >> 6] = m;
        __syncthreads();
        if (threadIdx.x == 0) a.block_max[blockIdx.y * gridDim.x + blockIdx.x] = max(max(bm[0], bm[1]), max(bm[2], bm[3]));
    } else {
        block_atomic_max_bits<256>(m, a.w_amax_bits);
    }
}

static dim3 update_grid(int64_t N, int64_t K)
{
    // Mid-sized tensors (thousands of short rows): a workgroup takes four rows in turn, so that fewer workgroups meet
    // at the absmax word (cfg2: 21 -> 17 us per launch).  Few rows: one each, the chain of dependent loads stays short.
    const int64_t rows_y = N >= 1024 && N * K <= (int64_t(8) << 20) ? (N + 3) / 4 : N;
    return dim3((unsigned)((K + UP_SEG - 1) / UP_SEG), (unsigned)rows_y);
}

int64_t update_blocks(int64_t N, int64_t K)
{
    if (N <= 0 || K <= 0) return 0;
    const dim3 g = update_grid(N, K);
    return (int64_t)g.x * g.y;
}

hipError_t launch_update(const UpdateArgs& a, hipStream_t s)
{
    if (a.N <= 0 || a.K <= 0) return hipSuccess;
    const dim3 grid = update_grid(a.N, a.K);
    if (a.block_max && (int64_t)grid.x * grid.y > UPDATE_MAX_BLOCKS) return hipErrorInvalidValue;
    const bool vec = (a.K & 3) == 0 && ((((uintptr_t)a.w) & 15) == 0);
    if (vec) hipLaunchKernelGGL(k_update<true>, grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL(k_update<false>, grid, dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace ffi
