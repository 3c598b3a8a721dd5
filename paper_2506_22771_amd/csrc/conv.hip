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

hipError_t launch_im2col(const Im2colArgs& p, bool transposed, hipStream_t s)
{
    const int64_t rows = transposed ? p.K : (int64_t)(p.b1 - p.b0) * p.g.Ho * p.g.Wo;
    const int64_t total = rows * (p.ld_out >> 4);
    if (total <= 0) return hipSuccess;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65535) blocks = 65535;
    const dim3 grid((unsigned)blocks, 1, (unsigned)p.nb);
    if (transposed) hipLaunchKernelGGL(k_im2col_t, grid, dim3(256), 0, s, p);
    else hipLaunchKernelGGL(k_im2col, grid, dim3(256), 0, s, p);
    return hipGetLastError();
}

}  // namespace ffi
