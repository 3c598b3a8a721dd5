// Explicit im2col helpers for the convolution layers of the FF-INT8 step (gfx950).
//
// The forward convolution runs as an implicit GEMM inside k_gemm_nt_i8 whenever C_in is a multiple of
// 16.  Two cases need a materialised matrix:
//  * the weight-gradient contraction (Section IV-B: only g^W is formed) reduces over output pixels, and
//    the MFMA wants 16 consecutive reduction bytes per operand row, so the input patches are written
//    transposed, colT[(kh,kw,ci)][m], m = (b, ho, wo) over a range of samples;
//  * a first layer with a handful of channels (C_in = 3) has reduction rows of 27 bytes that no
//    16-byte copy can address, so its patches are written row-major, col[m][(kh,kw,ci)].
// Both are byte gathers from the quantised NHWC activations (pure data movement; taps outside the image
// give 0).
#include "ff_internal.hpp"

namespace ffi {

__device__ __forceinline__ int gather_byte(const int8_t* __restrict__ a, const ConvGeom& g, int b, int ho, int wo,
                                           int kh, int kw, int ci)
{
    const int hi = ho * g.stride - g.pad + kh, wi = wo * g.stride - g.pad + kw;
    if ((unsigned)hi >= (unsigned)g.H || (unsigned)wi >= (unsigned)g.W) return 0;
    return (int)(uint8_t)a[(((int64_t)b * g.H + hi) * g.W + wi) * g.cpitch + ci];
}

// colT[j][m - m0] for j < K, m in [b0*Ho*Wo, b1*Ho*Wo); one thread per 16-byte chunk of a colT row.
// Bytes beyond the range (row pad) are written as zero.
__global__ __launch_bounds__(256) void k_im2col_t(Im2colArgs p)
{
    const int z = blockIdx.z;
    const int8_t* __restrict__ a = p.a + z * p.st_a;
    int8_t* __restrict__ out = p.out + z * p.st_out;
    const ConvGeom& g = p.g;
    const int64_t chunks_per_row = p.ld_out >> 4;
    const int64_t total = (int64_t)p.K * chunks_per_row;
    const int hw = g.Ho * g.Wo;
    const int64_t mcount = (int64_t)(p.b1 - p.b0) * hw;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
        const int j = (int)(e / chunks_per_row);
        const int64_t ml = (e - (int64_t)j * chunks_per_row) << 4;
        const int tap = j / g.Cin, ci = j - tap * g.Cin;
        const int kh = tap / g.ks, kw = tap - kh * g.ks;
        uint32_t w[4] = {0u, 0u, 0u, 0u};
        int b = p.b0 + (int)(ml / hw);
        int rem = (int)(ml - (int64_t)(b - p.b0) * hw);
        int ho = rem / g.Wo, wo = rem - ho * g.Wo;
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            if (ml + t < mcount) w[t >> 2] |= (uint32_t)gather_byte(a, g, b, ho, wo, kh, kw, ci) << (8 * (t & 3));
            if (++wo == g.Wo) {
                wo = 0;
                if (++ho == g.Ho) { ho = 0; ++b; }
            }
        }
        *(uint4*)(out + (int64_t)j * p.ld_out + ml) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// col[m][j] for every output pixel m of all samples, j < K, row pitch ld_out; one thread per 16-byte chunk.
__global__ __launch_bounds__(256) void k_im2col(Im2colArgs p)
{
    const int z = blockIdx.z;
    const int8_t* __restrict__ a = p.a + z * p.st_a;
    int8_t* __restrict__ out = p.out + z * p.st_out;
    const ConvGeom& g = p.g;
    const int64_t chunks_per_row = p.ld_out >> 4;
    const int hw = g.Ho * g.Wo;
    const int64_t M = (int64_t)(p.b1 - p.b0) * hw;
    const int64_t total = M * chunks_per_row;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
        const int64_t m = e / chunks_per_row;
        const int j0 = (int)(e - m * chunks_per_row) << 4;
        const int b = p.b0 + (int)(m / hw);
        const int rem = (int)(m - (int64_t)(b - p.b0) * hw);
        const int ho = rem / g.Wo, wo = rem - ho * g.Wo;
        uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            const int j = j0 + t;
            if (j < p.K) {
                const int tap = j / g.Cin, ci = j - tap * g.Cin;
                const int kh = tap / g.ks, kw = tap - kh * g.ks;
                w[t >> 2] |= (uint32_t)gather_byte(a, g, b, ho, wo, kh, kw, ci) << (8 * (t & 3));
            }
        }
        *(uint4*)(out + m * p.ld_out + j0) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// Transposed patches through an LDS slab.
// One workgroup: one sample, RH output rows, FT_CT channels.  The input rows those outputs touch are staged
// channel-major in LDS ([channel][row][padded column], zero borders), so that the global gathers become one
// pass of 16-byte loads, and every colT row receives RH * W_out contiguous bytes per workgroup in 16-byte
// stores (lanes run over the chunks of one colT row first).
// FAST (MODE 1: stride 1, W_out % 16 == 0): the 16 reduction bytes of an output chunk -- 16 consecutive output pixels
// of one row, one tap, one channel -- are 16 consecutive LDS bytes at the tap's column offset: five aligned
// words and a byte alignment.  Maps 8 or 4 pixels wide at stride 1 do the same per output row (MODE 2 / 3); otherwise
// (stride 2, other widths) each byte is gathered from LDS (MODE 0).
// Requires H_out * W_out % 16 == 0 (chunks do not straddle samples) and RH * W_out % 16 == 0.
constexpr int FT_CT = 32;

// MODE 2 / 3: a chunk is two (four) output rows of eight (four) consecutive LDS bytes each.
template <int MODE>
__global__ __launch_bounds__(256) void k_im2col_t_slab(Im2colArgs p, int RH)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t slab[];
    const ConvGeom& g = p.g;
    const int nbatch = p.b1 - p.b0;
    const int z = blockIdx.z / nbatch, bl = blockIdx.z - z * nbatch, b = p.b0 + bl;
    const int8_t* __restrict__ a = p.a + z * p.st_a;
    int8_t* __restrict__ out = p.out + z * p.st_out;
    // vertical geometry: the full patch rows, or (planes of horizontal taps only) the input rows themselves
    const int vks = p.wtaps_only ? 1 : g.ks, vstride = p.wtaps_only ? 1 : g.stride, vpad = p.wtaps_only ? 0 : g.pad;
    const int HoE = p.wtaps_only ? g.H : g.Ho;
    const int ho0 = blockIdx.x * RH, c0 = blockIdx.y * FT_CT;
    const int NR = (RH - 1) * vstride + vks;         // input rows of the slab
    const int WP = (g.W + 2 * g.pad + 3 + 4) & ~3;   // padded row length, a spare word for the 5-word read
    const int t = threadIdx.x;
    // ---- stage: every slab position (row, padded column, 16-channel group) is written once, zero outside the image
    const int ngroups = FT_CT / 16;
    const int npos = NR * WP * ngroups;
    for (int e = t; e < npos; e += 256) {
        const int cg = e % ngroups, pos = e / ngroups;
        const int wp = pos % WP, hl = pos / WP;
        const int hi = ho0 * vstride - vpad + hl, wi = wp - g.pad;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if ((unsigned)hi < (unsigned)g.H && (unsigned)wi < (unsigned)g.W && c0 + 16 * cg < g.cpitch)
            v = *(const uint4*)(a + (((int64_t)b * g.H + hi) * g.W + wi) * g.cpitch + c0 + 16 * cg);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int c = 0; c < 16; ++c)
            slab[((cg * 16 + c) * NR + hl) * WP + wp] = (uint8_t)(w[c >> 2] >> (8 * (c & 3)));
    }
    __syncthreads();
    // ---- emit
    const int nchunk = (RH * g.Wo) >> 4;    // 16-byte chunks of one colT row in this workgroup
    const int ntap = vks * g.ks;
    const int nct = min(FT_CT, g.Cin - c0);
    const int total = ntap * nct * nchunk;
    const int64_t mbase = (int64_t)bl * HoE * g.Wo + (int64_t)ho0 * g.Wo;
    for (int e = t; e < total; e += 256) {
        const int ch = e % nchunk, r = e / nchunk;
        const int ci = r % nct, tap = r / nct;
        const int kh = tap / g.ks, kw = tap - kh * g.ks;
        uint4 o;
        if (MODE == 2 || MODE == 3) {
            constexpr int PPC = MODE == 2 ? 2 : 4;     // output rows per chunk
            uint32_t ow[4];
#pragma unroll
            for (int r = 0; r < PPC; ++r) {
                const int off = (ci * NR + ch * PPC + r + kh) * WP + kw;
                const uint32_t* wp = (const uint32_t*)(slab + (off & ~3));
                const uint32_t sh = (uint32_t)(off & 3);
                if (MODE == 2) {
                    const uint32_t w0 = wp[0], w1 = wp[1], w2 = wp[2];
                    ow[2 * r] = __builtin_amdgcn_alignbyte(w1, w0, sh);
                    ow[2 * r + 1] = __builtin_amdgcn_alignbyte(w2, w1, sh);
                } else {
                    ow[r] = __builtin_amdgcn_alignbyte(wp[1], wp[0], sh);
                }
            }
            o = make_uint4(ow[0], ow[1], ow[2], ow[3]);
        } else if (MODE == 1) {
            const int cpr = g.Wo >> 4;              // chunks per output row
            const int hl = ch / cpr, w16 = ch - hl * cpr;
            const int off = (ci * NR + hl + kh) * WP + w16 * 16 + kw;
            const uint32_t* wp = (const uint32_t*)(slab + (off & ~3));
            const uint32_t w0 = wp[0], w1 = wp[1], w2 = wp[2], w3 = wp[3], w4 = wp[4];
            const uint32_t sh = (uint32_t)(off & 3);
            o.x = __builtin_amdgcn_alignbyte(w1, w0, sh);
            o.y = __builtin_amdgcn_alignbyte(w2, w1, sh);
            o.z = __builtin_amdgcn_alignbyte(w3, w2, sh);
            o.w = __builtin_amdgcn_alignbyte(w4, w3, sh);
        } else {
            uint32_t w[4] = {0u, 0u, 0u, 0u};
            int ml = ch * 16;
            int hl = ml / g.Wo, wo = ml - hl * g.Wo;
            const uint8_t* base = slab + (ci * NR + kh) * WP + kw;
#pragma unroll
            for (int tt = 0; tt < 16; ++tt) {
                w[tt >> 2] |= (uint32_t)base[hl * vstride * WP + wo * g.stride] << (8 * (tt & 3));
                if (++wo == g.Wo) { wo = 0; ++hl; }
            }
            o = make_uint4(w[0], w[1], w[2], w[3]);
        }
        *(uint4*)(out + (int64_t)(tap * g.Cin + c0 + ci) * p.ld_out + mbase + ch * 16) = o;
    }
}

// Rows per workgroup of the slab kernel: about 256 contiguous bytes per output row, a divisor of the row count,
// RH * W_out % 16 == 0.  Returns 0 when the slab path cannot serve the geometry.
static int slab_rows(const ConvGeom& g, bool wtaps_only, int64_t grid_z, size_t* lds_bytes)
{
    const int HoE = wtaps_only ? g.H : g.Ho;
    if (((HoE * g.Wo) & 15) != 0 || grid_z > 65535) return 0;
    int RH = 256 / g.Wo;
    if (RH < 1) RH = 1;
    if (RH > HoE) RH = HoE;
    while (RH > 1 && (HoE % RH || ((RH * g.Wo) & 15))) --RH;
    if (HoE % RH || ((RH * g.Wo) & 15)) RH = HoE;
    const int vks = wtaps_only ? 1 : g.ks, vstride = wtaps_only ? 1 : g.stride;
    const int NR = (RH - 1) * vstride + vks, WP = (g.W + 2 * g.pad + 3 + 4) & ~3;
    *lds_bytes = (size_t)FT_CT * NR * WP + 16;
    return *lds_bytes <= 64 * 1024 ? RH : 0;
}

bool im2col_planes_ok(const ConvGeom& g, int64_t nbatch_times_nb)
{
    size_t lds;
    return (g.Wo & 15) == 0 && slab_rows(g, true, nbatch_times_nb, &lds) > 0;
}

hipError_t launch_im2col(const Im2colArgs& p, bool transposed, hipStream_t s)
{
    const int64_t rows = transposed ? p.K : (int64_t)(p.b1 - p.b0) * p.g.Ho * p.g.Wo;
    const int64_t total = rows * (p.ld_out >> 4);
    if (total <= 0) return hipSuccess;
    const ConvGeom& g = p.g;
    if (transposed) {
        size_t lds = 0;
        const int RH = slab_rows(g, p.wtaps_only != 0, (int64_t)p.nb * (p.b1 - p.b0), &lds);
        if (RH > 0) {
            const int HoE = p.wtaps_only ? g.H : g.Ho;
            const dim3 grid((unsigned)(HoE / RH), (unsigned)((g.Cin + FT_CT - 1) / FT_CT), (unsigned)(p.nb * (p.b1 - p.b0)));
            if (g.stride == 1 && (g.Wo & 15) == 0) hipLaunchKernelGGL(k_im2col_t_slab<1>, grid, dim3(256), lds, s, p, RH);
            else if (g.stride == 1 && g.Wo == 8) hipLaunchKernelGGL(k_im2col_t_slab<2>, grid, dim3(256), lds, s, p, RH);
            else if (g.stride == 1 && g.Wo == 4) hipLaunchKernelGGL(k_im2col_t_slab<3>, grid, dim3(256), lds, s, p, RH);
            else hipLaunchKernelGGL(k_im2col_t_slab<0>, grid, dim3(256), lds, s, p, RH);
            return hipGetLastError();
        }
        if (p.wtaps_only) return hipErrorInvalidValue;   // the generic kernel below writes full patches only
    }
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65535) blocks = 65535;
    const dim3 grid((unsigned)blocks, 1, (unsigned)p.nb);
    if (transposed) hipLaunchKernelGGL(k_im2col_t, grid, dim3(256), 0, s, p);
    else hipLaunchKernelGGL(k_im2col, grid, dim3(256), 0, s, p);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------------------
// Depthwise convolution.  Forward: a thread owns four channels of one output pixel (nine 4-byte taps, 16-byte
// store of the accumulators); blockIdx.y = sample, so the per-sample goodness sums / maxima are reduced in the
// workgroup and leave as one atomic each.  HBM-bound on the int32 output (4 bytes written per input byte).
// ------------------------------------------------------------------------------------------------------------
constexpr int DW_PIX = 8;   // output pixels per thread

__device__ __forceinline__ unsigned long long dw_wave_sum_u64(unsigned long long v)
{
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const unsigned lo = (unsigned)__shfl_xor((int)(unsigned)v, d), hi = (unsigned)__shfl_xor((int)(unsigned)(v >> 32), d);
        v += ((unsigned long long)hi << 32) | lo;
    }
    return v;
}

// 4x4 byte transpose: word j of x holds bytes (channels) 0..3 of item j; word e of o holds byte e of items 0..3.
__device__ __forceinline__ void dw_transpose4x4(const uint32_t x[4], uint32_t o[4])
{
    const uint32_t t0 = __builtin_amdgcn_perm(x[1], x[0], 0x05010400u);
    const uint32_t t1 = __builtin_amdgcn_perm(x[1], x[0], 0x07030602u);
    const uint32_t t2 = __builtin_amdgcn_perm(x[3], x[2], 0x05010400u);
    const uint32_t t3 = __builtin_amdgcn_perm(x[3], x[2], 0x07030602u);
    o[0] = __builtin_amdgcn_perm(t2, t0, 0x05040100u);
    o[1] = __builtin_amdgcn_perm(t2, t0, 0x07060302u);
    o[2] = __builtin_amdgcn_perm(t3, t1, 0x05040100u);
    o[3] = __builtin_amdgcn_perm(t3, t1, 0x07060302u);
}

// blockIdx.x = share of the sample's output pixels, blockIdx.y = sample, blockIdx.z = pass * channel groups + group.
// A thread keeps the 36 weights of its four channels in registers and walks over DW_PIX pixels, 256 / quads apart.
__global__ __launch_bounds__(256) void k_dwconv_forward(DwArgs p, int cgroups)
{
    const ConvGeom& g = p.g;
    const int z = blockIdx.z / cgroups, cg0 = (blockIdx.z - z * cgroups) * 64;
    const int b = blockIdx.y;
    const int C = g.Cin;
    const int nq = min(16, (C - cg0 + 3) >> 2);          // channel quads of this workgroup
    const int lanes = 256 / nq;                          // pixel lanes
    const int q = threadIdx.x % nq, pl = threadIdx.x / nq;
    const int c0 = cg0 + 4 * q;
    const int hw = g.Ho * g.Wo;
    const int8_t* __restrict__ a = p.a + z * p.st_a;
    unsigned long long sq = 0;
    int vm = 0;
    if (pl < lanes) {
        // the nine taps of a channel are nine consecutive bytes of its weight row: three packed words per channel
        uint32_t w[4][3];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            uint4 wr = make_uint4(0u, 0u, 0u, 0u);
            if (c0 + e < C) wr = *(const uint4*)(p.w_q + (int64_t)(c0 + e) * 16);
            w[e][0] = wr.x; w[e][1] = wr.y; w[e][2] = wr.z;
        }
        if (g.stride == 1 && (g.Wo & 3) == 0) {
            // Stride 1, rows of whole 4-pixel groups: four consecutive output pixels at a time.  The six input columns
            // they touch are loaded once per kernel row and transposed to (channel word x pixel bytes); the word of
            // output j is a byte alignment of two such words, and a kernel row is one packed dot product with the
            // three taps of that row (fourth byte zero): half the loads and address arithmetic of the loop below.
            uint32_t wk[4][3];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                wk[e][0] = w[e][0] & 0x00FFFFFFu;
                wk[e][1] = __builtin_amdgcn_alignbyte(w[e][1], w[e][0], 3u) & 0x00FFFFFFu;
                wk[e][2] = __builtin_amdgcn_alignbyte(w[e][2], w[e][1], 2u) & 0x00FFFFFFu;
            }
            const int ngrp = hw >> 2;
            const int grp0 = (int)blockIdx.x * lanes * (DW_PIX / 4) + pl;
            for (int it = 0; it < DW_PIX / 4; ++it) {
                const int grp = grp0 + it * lanes;
                if (grp >= ngrp) break;
                const int pix = 4 * grp;
                const int ho = pix / g.Wo, wo = pix - ho * g.Wo;
                int acc[4][4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[j][e] = 0;
#pragma unroll
                for (int kh = 0; kh < 3; ++kh) {
                    const int hi = ho + kh - g.pad;
                    if ((unsigned)hi >= (unsigned)g.H) continue;
                    const int8_t* arow = a + (((int64_t)b * g.H + hi) * g.W) * g.cpitch + c0;
                    uint32_t X[8];
#pragma unroll
                    for (int j = 0; j < 6; ++j) {
                        const int wi = wo - g.pad + j;
                        X[j] = (unsigned)wi < (unsigned)g.W ? *(const uint32_t*)(arow + (int64_t)wi * g.cpitch) : 0u;
                    }
                    X[6] = 0u;
                    X[7] = 0u;
                    uint32_t TA[4], TB[4];
                    dw_transpose4x4(X, TA);
                    dw_transpose4x4(X + 4, TB);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        acc[0][e] = __builtin_amdgcn_sdot4((int)TA[e], (int)wk[e][kh], acc[0][e], false);
                        acc[1][e] = __builtin_amdgcn_sdot4((int)__builtin_amdgcn_alignbyte(TB[e], TA[e], 1u), (int)wk[e][kh], acc[1][e], false);
                        acc[2][e] = __builtin_amdgcn_sdot4((int)__builtin_amdgcn_alignbyte(TB[e], TA[e], 2u), (int)wk[e][kh], acc[2][e], false);
                        acc[3][e] = __builtin_amdgcn_sdot4((int)__builtin_amdgcn_alignbyte(TB[e], TA[e], 3u), (int)wk[e][kh], acc[3][e], false);
                    }
                }
                typedef int i32x4 __attribute__((ext_vector_type(4)));
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    __builtin_nontemporal_store((i32x4){acc[j][0], acc[j][1], acc[j][2], acc[j][3]},
                                                (i32x4*)(p.acc + z * p.st_acc + ((int64_t)b * hw + pix + j) * p.ldacc + c0));
                    if (p.gsum && p.relu && p.rshift == 0) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const unsigned y = (unsigned)max(acc[j][e], 0);
                            sq += (unsigned long long)y * y;
                            vm = max(vm, (int)y);
                        }
                    } else if (p.gsum) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            int y = acc[j][e];
                            if (p.relu) y = max(y, 0);
                            const long long yl = (long long)y;
                            sq += ((unsigned long long)(yl * yl)) >> p.rshift;
                            vm = max(vm, y < 0 ? -y : y);
                        }
                    }
                }
            }
        } else {
        const int pix0 = (int)blockIdx.x * lanes * DW_PIX + pl;
#pragma unroll 2
        for (int it = 0; it < DW_PIX; ++it) {
            const int pix = pix0 + it * lanes;
            if (pix >= hw) break;
            const int ho = pix / g.Wo, wo = pix - ho * g.Wo;
            uint32_t x[9];   // tap words: byte e = channel c0 + e
#pragma unroll
            for (int kh = 0; kh < 3; ++kh)
#pragma unroll
                for (int kw = 0; kw < 3; ++kw) {
                    const int hi = ho * g.stride + kh - g.pad, wi = wo * g.stride + kw - g.pad;
                    x[kh * 3 + kw] = ((unsigned)hi < (unsigned)g.H && (unsigned)wi < (unsigned)g.W)
                                         ? *(const uint32_t*)(a + (((int64_t)b * g.H + hi) * g.W + wi) * g.cpitch + c0)
                                         : 0u;
                }
            // two 4x4 byte transposes turn (tap words x channel bytes) into (channel words x tap bytes), which is
            // the operand order of the packed int8 dot product
            int acc[4];
            {
                uint32_t lo[4], hi4[4];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const uint32_t* xs = x + 4 * h;
                    const uint32_t t0 = __builtin_amdgcn_perm(xs[1], xs[0], 0x05010400u);
                    const uint32_t t1 = __builtin_amdgcn_perm(xs[1], xs[0], 0x07030602u);
                    const uint32_t t2 = __builtin_amdgcn_perm(xs[3], xs[2], 0x05010400u);
                    const uint32_t t3 = __builtin_amdgcn_perm(xs[3], xs[2], 0x07030602u);
                    uint32_t* o = h ? hi4 : lo;
                    o[0] = __builtin_amdgcn_perm(t2, t0, 0x05040100u);
                    o[1] = __builtin_amdgcn_perm(t2, t0, 0x07060302u);
                    o[2] = __builtin_amdgcn_perm(t3, t1, 0x05040100u);
                    o[3] = __builtin_amdgcn_perm(t3, t1, 0x07060302u);
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    int sacc = (int)(int8_t)(x[8] >> (8 * e)) * (int)(int8_t)(w[e][2] & 0xFFu);
                    sacc = __builtin_amdgcn_sdot4((int)lo[e], (int)w[e][0], sacc, false);
                    sacc = __builtin_amdgcn_sdot4((int)hi4[e], (int)w[e][1], sacc, false);
                    acc[e] = sacc;
                }
            }
            {   // like the contraction's forward output: not read again soon, non-temporal store
                typedef int i32x4 __attribute__((ext_vector_type(4)));
                __builtin_nontemporal_store((i32x4){acc[0], acc[1], acc[2], acc[3]},
                                            (i32x4*)(p.acc + z * p.st_acc + ((int64_t)b * hw + pix) * p.ldacc + c0));
            }
            if (p.gsum) {
                // channels beyond C read zero inputs and zero weights: their y is 0
                if (p.relu && p.rshift == 0) {        // the usual case: one 32x32+64-bit multiply-add per activity
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const unsigned y = (unsigned)max(acc[e], 0);
                        sq += (unsigned long long)y * y;
                        vm = max(vm, (int)y);
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        int y = acc[e];
                        if (p.relu) y = max(y, 0);
                        const long long yl = (long long)y;
                        sq += ((unsigned long long)(yl * yl)) >> p.rshift;
                        vm = max(vm, y < 0 ? -y : y);
                    }
                }
            }
        }
        }
    }
    if (p.gsum) {
        __shared__ unsigned long long rs[4];
        __shared__ int rm[4];
        sq = dw_wave_sum_u64(sq);
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) vm = max(vm, __shfl_xor(vm, d));
        if ((threadIdx.x & 63) == 0) { rs[threadIdx.x >> 6] = sq; rm[threadIdx.x >> 6] = vm; }
        __syncthreads();
        if (threadIdx.x == 0) {
            const unsigned long long t = rs[0] + rs[1] + rs[2] + rs[3];
            const int m = max(max(rm[0], rm[1]), max(rm[2], rm[3]));
            if (t) atomicAdd(p.gsum + z * p.st_g + b, t);
            if (m) atomicMax(p.vmax + z * p.st_g + b, m);
        }
    }
}

hipError_t launch_dwconv_forward(const DwArgs& p, hipStream_t s)
{
    const ConvGeom& g = p.g;
    if (p.B <= 0) return hipSuccess;
    const int cgroups = (g.Cin + 63) / 64;
    if (g.ks != 3 || p.B > 65535 || (int64_t)cgroups * p.nb > 65535) return hipErrorInvalidValue;
    // pixels per workgroup depend on the group's quad count; size the grid for full groups (16 quads, 16 lanes),
    // narrower groups have more lanes and finish their share early
    const int64_t hw = (int64_t)g.Ho * g.Wo;
    const unsigned bx = (unsigned)((hw + 16 * DW_PIX - 1) / (16 * DW_PIX));
    hipLaunchKernelGGL(k_dwconv_forward, dim3(bx, (unsigned)p.B, (unsigned)(cgroups * p.nb)), dim3(256), 0, s, p, cgroups);
    return hipGetLastError();
}

// Weight gradient of a depthwise convolution: dw[c][tap] = sum over output pixels of gy[m][c] * a[pixel(m) + tap][c].
// A workgroup owns DW_ROWS output pixels (of the samples [b0, b1)) and a group of up to 64 channels; a thread owns four
// channels and every (256 / quads)-th row, keeps 36 int32 partial sums, adds them to LDS accumulators with LDS atomics,
// and the workgroup adds those to dw with integer atomics (exact and order-free; dw must be zero on entry).
constexpr int DW_ROWS = 512;

__global__ __launch_bounds__(256) void k_dwconv_wgrad(DwArgs p)
{
    const ConvGeom& g = p.g;
    const int z = blockIdx.z;
    const int C = g.Cin;
    const int cg0 = blockIdx.y * 64;
    const int nq = min(16, (C - cg0 + 3) >> 2);          // channel quads of this workgroup
    const int lanes = 256 / nq;                          // row lanes
    const int q = threadIdx.x % nq, rl = threadIdx.x / nq;
    const int c0 = cg0 + 4 * q;
    const int hw = g.Ho * g.Wo;
    const int64_t m0 = (int64_t)p.b0 * hw, m1 = (int64_t)p.b1 * hw;
    const int8_t* __restrict__ a = p.a + z * p.st_a;
    const int8_t* __restrict__ gy = p.gy + z * p.st_gy;
    __shared__ int lacc[64 * 9];
    for (int e = threadIdx.x; e < 64 * 9; e += 256) lacc[e] = 0;
    __syncthreads();
    int part[4][9];
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int t = 0; t < 9; ++t) part[e][t] = 0;
    if (rl < lanes && g.stride == 1 && (g.Wo & 3) == 0) {
        // Stride 1, rows of whole 4-pixel groups: four consecutive output pixels at a time.  The gradient words and
        // the six input columns they touch are transposed to (channel word x pixel bytes), a horizontal tap is then
        // a byte alignment of two such words, and every (channel, tap) takes one packed dot product over the four
        // pixels: 116 ALU operations per group against 288 for the pixel-by-pixel loop below.
        const int64_t r0 = m0 + (int64_t)blockIdx.x * DW_ROWS;
        const int64_t r1 = min(m1, r0 + DW_ROWS);
        for (int64_t m = r0 + 4 * rl; m < r1; m += 4 * lanes) {
            const int b = (int)(m / hw), pix = (int)(m - (int64_t)b * hw);
            const int ho = pix / g.Wo, wo = pix - ho * g.Wo;
            uint32_t gq[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) gq[j] = *(const uint32_t*)(gy + (m + j) * p.ldg + c0);
            if ((gq[0] | gq[1] | gq[2] | gq[3]) == 0u) continue;   // a rectified gradient is zero wherever the activity is
            uint32_t G[4];
            dw_transpose4x4(gq, G);
#pragma unroll
            for (int kh = 0; kh < 3; ++kh) {
                const int hi = ho + kh - g.pad;
                if ((unsigned)hi >= (unsigned)g.H) continue;
                const int8_t* arow = a + (((int64_t)b * g.H + hi) * g.W) * g.cpitch + c0;
                uint32_t X[8];
#pragma unroll
                for (int j = 0; j < 6; ++j) {
                    const int wi = wo - g.pad + j;
                    X[j] = (unsigned)wi < (unsigned)g.W ? *(const uint32_t*)(arow + (int64_t)wi * g.cpitch) : 0u;
                }
                X[6] = 0u;
                X[7] = 0u;
                uint32_t TA[4], TB[4];
                dw_transpose4x4(X, TA);
                dw_transpose4x4(X + 4, TB);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    part[e][kh * 3 + 0] = __builtin_amdgcn_sdot4((int)G[e], (int)TA[e], part[e][kh * 3 + 0], false);
                    part[e][kh * 3 + 1] = __builtin_amdgcn_sdot4((int)G[e], (int)__builtin_amdgcn_alignbyte(TB[e], TA[e], 1u),
                                                                 part[e][kh * 3 + 1], false);
                    part[e][kh * 3 + 2] = __builtin_amdgcn_sdot4((int)G[e], (int)__builtin_amdgcn_alignbyte(TB[e], TA[e], 2u),
                                                                 part[e][kh * 3 + 2], false);
                }
            }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int t = 0; t < 9; ++t)
                if (part[e][t]) atomicAdd(&lacc[(4 * q + e) * 9 + t], part[e][t]);
    } else if (rl < lanes) {
        const int64_t r0 = m0 + (int64_t)blockIdx.x * DW_ROWS;
        const int64_t r1 = min(m1, r0 + DW_ROWS);
        for (int64_t m = r0 + rl; m < r1; m += lanes) {
            const int b = (int)(m / hw), pix = (int)(m - (int64_t)b * hw);
            const int ho = pix / g.Wo, wo = pix - ho * g.Wo;
            const uint32_t gw = *(const uint32_t*)(gy + m * p.ldg + c0);
            if (gw == 0u) continue;   // a rectified gradient is zero wherever the activity is
            int gv[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) gv[e] = (int)(int8_t)(gw >> (8 * e));
#pragma unroll
            for (int kh = 0; kh < 3; ++kh)
#pragma unroll
                for (int kw = 0; kw < 3; ++kw) {
                    const int hi = ho * g.stride + kh - g.pad, wi = wo * g.stride + kw - g.pad;
                    if ((unsigned)hi < (unsigned)g.H && (unsigned)wi < (unsigned)g.W) {
                        const uint32_t x = *(const uint32_t*)(a + (((int64_t)b * g.H + hi) * g.W + wi) * g.cpitch + c0);
#pragma unroll
                        for (int e = 0; e < 4; ++e) part[e][kh * 3 + kw] += gv[e] * (int)(int8_t)(x >> (8 * e));
                    }
                }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int t = 0; t < 9; ++t)
                if (part[e][t]) atomicAdd(&lacc[(4 * q + e) * 9 + t], part[e][t]);
    }
    __syncthreads();
    for (int e = threadIdx.x; e < 64 * 9; e += 256) {
        const int c = cg0 + e / 9, t = e - (e / 9) * 9;
        if (c < C && lacc[e]) atomicAdd(p.dw + z * p.st_dw + (int64_t)c * 12 + t, lacc[e]);
    }
}

hipError_t launch_dwconv_wgrad(const DwArgs& p, hipStream_t s)
{
    const ConvGeom& g = p.g;
    const int64_t rows = (int64_t)(p.b1 - p.b0) * g.Ho * g.Wo;
    if (rows <= 0) return hipSuccess;
    if (g.ks != 3) return hipErrorInvalidValue;
    const int64_t bx = (rows + DW_ROWS - 1) / DW_ROWS;
    if (bx > 0x7FFFFFFF || (g.Cin + 63) / 64 > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_dwconv_wgrad, dim3((unsigned)bx, (unsigned)((g.Cin + 63) / 64), (unsigned)p.nb), dim3(256), 0, s, p);
    return hipGetLastError();
}

}  // namespace ffi
