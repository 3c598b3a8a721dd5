// int8 x int8 -> int32 contraction for gfx950 with v_mfma_i32_32x32x32_i8:
//     C[i][j] = sum_r P[i][r] * Q[j][r]          (both operands reduction-contiguous, "NT")
// It serves the forward pass (P = quantised activations [M,K], Q = quantised weights [N,K]; the
// paper's Section IV-B: int8 inputs, int32 accumulation) and the weight-gradient contraction
// (P = transposed quantised local gradient [N,M], Q = transposed quantised activations [K,M]).
//
// Forward launches fuse the per-sample reductions the goodness needs (Algorithm 1: G = ||y||^2)
// into the epilogue: sum of squared integer activities (uint64) and their maximum, accumulated
// with integer atomics, hence independent of workgroup order.
//
// Tiling: a workgroup of WM x WN wavefronts computes a BM x BN tile; operand tiles of 64 reduction
// bytes are staged in LDS (two stages, global loads for step k+1 in flight while step k is
// multiplied); 16-byte chunks are XOR-swizzled so that both the 16-byte LDS writes and the MFMA
// fragment reads are bank-conflict free.  The Q tile feeds the MFMA "A" operand and the P tile the
// "B" operand, so that every lane ends up with one row i of C and four consecutive columns j per
// accumulator quad: 16-byte stores, and the per-row reductions stay inside a lane.
#include "ff_internal.hpp"

namespace ffi {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BK = 64;  // reduction bytes per stage

__device__ __forceinline__ int swz(int row, int kc) { return row * BK + ((kc ^ ((row >> 2) & 3)) << 4); }

template <int BM, int BN, int WM, int WN, bool EPI>
__global__ __launch_bounds__(WM* WN * 64) void k_gemm_nt_i8(GemmArgs a)
{
    constexpr int T = WM * WN * 64;
    constexpr int WTM = BM / WM, WTN = BN / WN;  // wave tile
    constexpr int TI = WTM / 32, TJ = WTN / 32;  // MFMA tiles per wave
    constexpr int CH_P = BM * 4 / T, CH_Q = BN * 4 / T;
    static_assert(BM * 4 % T == 0 && BN * 4 % T == 0, "tile/threads mismatch");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of 32");

    __shared__ __attribute__((aligned(16))) int8_t lds[2][(BM + BN) * BK];

    const int z = blockIdx.z;
    const int8_t* __restrict__ P = a.P + z * a.st_p;
    const int8_t* __restrict__ Q = a.Q + z * a.st_q;
    int32_t* __restrict__ C = a.C + z * a.st_c;

    // tile coordinates: blockIdx.x walks i-tiles fastest inside a group of j-tiles
    const int tiles_i = (a.I + BM - 1) / BM;
    const int bi = blockIdx.x % tiles_i, bj = blockIdx.x / tiles_i;
    const int i0 = bi * BM, j0 = bj * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int Rpad = (a.R + 15) & ~15;
    const int nk = (Rpad + BK - 1) / BK;

    v4i regP[CH_P], regQ[CH_Q];
    auto gload = [&](int k0) {
#pragma unroll
        for (int s = 0; s < CH_P; ++s) {
            const int c = tid + s * T, row = c >> 2, kc = c & 3;
            const int gi = i0 + row, kb = k0 + kc * 16;
            v4i v = {0, 0, 0, 0};
            if (gi < a.I && kb < Rpad) v = *(const v4i*)(P + (int64_t)gi * a.ldp + kb);
            regP[s] = v;
        }
#pragma unroll
        for (int s = 0; s < CH_Q; ++s) {
            const int c = tid + s * T, row = c >> 2, kc = c & 3;
            const int gj = j0 + row, kb = k0 + kc * 16;
            v4i v = {0, 0, 0, 0};
            if (gj < a.J && kb < Rpad) v = *(const v4i*)(Q + (int64_t)gj * a.ldq + kb);
            regQ[s] = v;
        }
    };
    auto lstore = [&](int buf) {
#pragma unroll
        for (int s = 0; s < CH_P; ++s) {
            const int c = tid + s * T, row = c >> 2, kc = c & 3;
            *(v4i*)(&lds[buf][swz(row, kc)]) = regP[s];
        }
#pragma unroll
        for (int s = 0; s < CH_Q; ++s) {
            const int c = tid + s * T, row = c >> 2, kc = c & 3;
            *(v4i*)(&lds[buf][BM * BK + swz(row, kc)]) = regQ[s];
        }
    };

    v16i acc[TI][TJ];
#pragma unroll
    for (int ti = 0; ti < TI; ++ti)
#pragma unroll
        for (int tj = 0; tj < TJ; ++tj)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[ti][tj][v] = 0;

    const int lr = lane & 31, lh = lane >> 5;
    gload(0);
    lstore(0);
    __syncthreads();
    int buf = 0;
    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) gload((kt + 1) * BK);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            v4i fp[TI], fq[TJ];
#pragma unroll
            for (int ti = 0; ti < TI; ++ti)
                fp[ti] = *(const v4i*)(&lds[buf][swz(wm * WTM + ti * 32 + lr, ks * 2 + lh)]);
#pragma unroll
            for (int tj = 0; tj < TJ; ++tj)
                fq[tj] = *(const v4i*)(&lds[buf][BM * BK + swz(wn * WTN + tj * 32 + lr, ks * 2 + lh)]);
#pragma unroll
            for (int ti = 0; ti < TI; ++ti)
#pragma unroll
                for (int tj = 0; tj < TJ; ++tj)
                    acc[ti][tj] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fq[tj], fp[ti], acc[ti][tj], 0, 0, 0);
        }
        if (kt + 1 < nk) lstore(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }

    // Epilogue.  Lane (lr, lh) of tile (ti, tj) holds C[i][j] for i = i0 + wm*WTM + ti*32 + lr and
    // j = j0 + wn*WTN + tj*32 + 8*g + 4*lh + e, accumulator register v = 4*g + e.
#pragma unroll
    for (int ti = 0; ti < TI; ++ti) {
        const int i = i0 + wm * WTM + ti * 32 + lr;
        unsigned long long sq = 0;
        int vm = 0;
#pragma unroll
        for (int tj = 0; tj < TJ; ++tj) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int j = j0 + wn * WTN + tj * 32 + 8 * g + 4 * lh;
                const int c0 = acc[ti][tj][4 * g + 0], c1 = acc[ti][tj][4 * g + 1];
                const int c2 = acc[ti][tj][4 * g + 2], c3 = acc[ti][tj][4 * g + 3];
                if (i < a.I) {
                    int32_t* dst = C + (int64_t)i * a.ldc + j;
                    if (j + 3 < a.J) {
                        *(v4i*)dst = (v4i){c0, c1, c2, c3};
                    } else {
                        if (j + 0 < a.J) dst[0] = c0;
                        if (j + 1 < a.J) dst[1] = c1;
                        if (j + 2 < a.J) dst[2] = c2;
                    }
                }
                if (EPI) {
                    // columns j >= J and rows i >= I hold exact zeros (their operand rows were zero-filled)
                    const int cc[4] = {c0, c1, c2, c3};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        int v = cc[e];
                        if (a.relu) v = max(v, 0);
                        const long long vl = (long long)v;
                        sq += ((unsigned long long)(vl * vl)) >> a.rshift;
                        vm = max(vm, v < 0 ? -v : v);
                    }
                }
            }
        }
        if (EPI) {
            // the two half-waves hold the two column halves of the same row
            const unsigned lo = (unsigned)sq, hi = (unsigned)(sq >> 32);
            const unsigned lo2 = (unsigned)__shfl_xor((int)lo, 32), hi2 = (unsigned)__shfl_xor((int)hi, 32);
            sq += ((unsigned long long)hi2 << 32) | lo2;
            vm = max(vm, __shfl_xor(vm, 32));
            if (lh == 0 && i < a.I) {
                const int smp = i / a.rows_per_sample;
                atomicAdd(a.gsum + z * a.st_g + smp, sq);
                atomicMax(a.vmax + z * a.st_g + smp, vm);
            }
        }
    }
}

template <int BM, int BN, int WM, int WN>
static hipError_t launch_cfg(const GemmArgs& a, hipStream_t s)
{
    const int tiles_i = (a.I + BM - 1) / BM, tiles_j = (a.J + BN - 1) / BN;
    const dim3 grid((unsigned)(tiles_i * tiles_j), 1, (unsigned)a.nb), block(WM * WN * 64);
    if (a.gsum) hipLaunchKernelGGL((k_gemm_nt_i8<BM, BN, WM, WN, true>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((k_gemm_nt_i8<BM, BN, WM, WN, false>), grid, block, 0, s, a);
    return hipGetLastError();
}

hipError_t launch_gemm_nt_i8(const GemmArgs& a, hipStream_t s)
{
    if (a.I <= 0 || a.J <= 0) return hipSuccess;
    // pick the largest tile that still yields at least ~2 workgroups per compute unit
    const int64_t want = 512;
    auto tiles = [&](int bm, int bn) { return (int64_t)((a.I + bm - 1) / bm) * ((a.J + bn - 1) / bn) * a.nb; };
    if (tiles(256, 256) >= want) return launch_cfg<256, 256, 2, 4>(a, s);
    if (tiles(128, 128) >= want) return launch_cfg<128, 128, 2, 2>(a, s);
    return launch_cfg<64, 64, 2, 2>(a, s);
}

}  // namespace ffi
