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
// Structure (measured choices, see the design notes):
//  * A workgroup of WM x WN wavefronts computes a BM x BN tile in steps of BK = 128 reduction bytes,
//    i.e. whole 128-byte lines of both operands per row (half lines halve the useful L2 bandwidth).
//  * Operand tiles go from global memory straight into LDS with buffer_load_dwordx4 ... lds (no VGPR
//    staging; rows and reduction tails beyond the matrix read as zero through the buffer's range
//    check).  Two LDS stages; the copy of step k+1 is in flight while step k is multiplied.  The copies
//    are issued from inline assembly and tracked by hand with vmcnt: through the compiler's builtin
//    every LDS read would wait for all outstanding copies, and __syncthreads() would drain them too.
//  * 16-byte chunks are XOR-swizzled inside each 128-byte row so that the MFMA fragment reads
//    (32 rows x 16 bytes per half-wave, ds_read_b128) hit all 64 banks; bank-conflict counter = 0.
//  * MFMA fragments are double-buffered in registers: the reads for sub-step s+1 are issued before
//    the MFMAs of sub-step s.
//  * The Q tile feeds the MFMA "A" operand and the P tile the "B" operand, so that every lane ends up
//    with one row i of C and four consecutive columns j per accumulator quad: 16-byte stores, and the
//    per-row reductions stay inside a lane (one cross-half-wave shuffle at the end).
//  * Large dense problems run as a persistent launch: one workgroup per compute unit walks over its
//    share of the 256 x 256 tiles; the copies of a tile's first two reduction steps go out together, and
//    those of the NEXT tile's first step are issued at the start of the epilogue, into the LDS stage
//    that the accumulator staging does not use, so that their round trip runs under the stores.
//  * Within a reduction step half of the wavefronts issue the next copies before the step's last
//    multiplies and half after them: every SIMD keeps multiplying while the copy instructions queue up.
#include "ff_internal.hpp"

namespace ffi {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BK = 128;  // reduction bytes per LDS stage

#ifndef FF_PRO2
#define FF_PRO2 1
#endif
#ifndef FF_PERSIST
#define FF_PERSIST 1
#endif
#ifndef FF_NEXT_TILE_PREFETCH
#define FF_NEXT_TILE_PREFETCH 1
#endif
#ifndef FF_SPLIT_ISSUE
#define FF_SPLIT_ISSUE 1
#endif
#ifndef FF_DEEP
// 1: tiles smaller than 256 x 256 use three or four LDS stages (two or three copies in flight).  Measured: the contraction
// launches get 4-5 % shorter on their own, but the steps of the small and convolution configurations get 2-3 % longer
// (a workgroup that holds most of the LDS keeps the next kernel's workgroups off the compute unit while the launch drains).
#define FF_DEEP 0
#endif
#ifndef FF_SPLIT_TARGET_BIG
#define FF_SPLIT_TARGET_BIG 256
#endif
#ifndef FF_STAGED_EPI
#define FF_STAGED_EPI 1   // 1: interior tiles leave through LDS as whole rows (see the epilogue)
#endif

template <int N> __device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// 16 bytes per lane from a buffer (byte offset voffset + soffset) straight into LDS at lds_base + lane*16.
// The compiler is not told about the LDS write, so it adds no waits of its own: completion is tracked by
// hand with vmcnt.  Out-of-range offsets read as zero (buffer range check).
__device__ __forceinline__ void lds_dma16(__amdgpu_buffer_rsrc_t rsrc, int voffset, int soffset, unsigned lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds" ::"s"(lds_base), "v"(voffset), "s"(rsrc), "s"(soffset) : "memory", "m0");
}
constexpr int OOB = 0x7FFFFFF0;  // a byte offset beyond any buffer
__device__ __forceinline__ unsigned long long shfl_xor_u64(unsigned long long v, int d)
{
    const unsigned lo = (unsigned)__shfl_xor((int)(unsigned)v, d), hi = (unsigned)__shfl_xor((int)(unsigned)(v >> 32), d);
    return ((unsigned long long)hi << 32) | lo;
}
// Lanes of one wavefront exchange data through LDS in the epilogues: the hardware executes a wave's LDS
// instructions in order, but the compiler reasons per thread and, without a fence, may keep a value it loaded
// earlier instead of re-reading a location another lane has written since.
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
__device__ __forceinline__ int swz(int row, int kc) { return row * BK + ((kc ^ ((row >> 1) & 7)) << 4); }

// MODE 0: store C; 1: store C and accumulate the per-sample goodness sums / maxima; 2: split reduction, this
// workgroup stores the partial sums of its share of the reduction steps at C + blockIdx.y * st_split.
// CONV 0: both operands are matrices.  1: P is an NHWC tensor, row i of the contraction is an output pixel and
// the reduction runs over (tap, channel) (forward pass of a convolution as an implicit GEMM).  2: Q is a set of
// column-shifted channel-major planes S[kw][ci][(b, h, wo)] of the layer input, row j of the contraction is
// (tap, channel) and the reduction runs over output pixels (weight gradient of a convolution as an implicit
// GEMM: the vertical tap offset is an address offset of whole 16-byte chunks, rows outside the image read as
// zero through the range check).
template <int BM, int BN, int WM, int WN, int MODE, int CONV>
__global__ __launch_bounds__(WM* WN * 64) void k_gemm_nt_i8(GemmArgs a)
{
    constexpr bool EPI = MODE == 1;
    constexpr int T = WM * WN * 64;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int TI = WTM / 32, TJ = WTN / 32;
    constexpr int CH_P = BM * 8 / T, CH_Q = BN * 8 / T;
    constexpr int STAGE_BYTES = (BM + BN) * BK;
    static_assert(BM * 8 % T == 0 && BN * 8 % T == 0, "tile/threads mismatch");
    // epilogue staging: one slice of EROWS rows of a wave's tile, rows padded by 16 bytes to spread the banks.  The
    // 256-row tiles stage in the SECOND operand stage (and a little beyond it; 16 rows at a time for the 256 x 256 tile,
    // so that it fits), which leaves the first stage free for the first copies of the workgroup's next tile (persistent
    // launches); the others 32 rows from 0.
    constexpr bool PREFETCH = FF_NEXT_TILE_PREFETCH && BM == 256 && CONV != 2 && MODE != 2;
    constexpr int EROWS = PREFETCH && BN == 256 ? 16 : 32;
    constexpr int EROW = WTN * 4 + 16;
    constexpr int ESLICE = EROWS * EROW;
    constexpr int EOFF = PREFETCH ? STAGE_BYTES : 0;
    // LDS stages: two for the big tile (128 KB); the smaller tiles, whose launches are short chains of reduction steps
    // that each wait for a round trip to memory, keep up to three copies in flight
    constexpr int NS = (FF_DEEP && !(BM == 256 && BN == 256)) ? (4 * STAGE_BYTES <= 160 * 1024 ? 4 : 3) : 2;
    constexpr int CH = CH_P + CH_Q;   // copy instructions of one thread per reduction step
    static_assert((NS - 1) * CH < 64, "vmcnt range");
    constexpr int LDS_BYTES = NS * STAGE_BYTES > EOFF + WM * WN * ESLICE ? NS * STAGE_BYTES : EOFF + WM * WN * ESLICE;
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
    __shared__ __attribute__((aligned(16))) int8_t lds[LDS_BYTES];

    // clock probe: the counters are wavefront-uniform (scalar registers); only the final atomics are per thread
    unsigned long long clk0 = 0, rt0 = 0;
    if (a.clk) {
        clk0 = clock64();
        rt0 = wall_clock64();
    }
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int Rpad = (a.R + 15) & ~15;
    const int nk_all = (Rpad + BK - 1) / BK;
    // this workgroup's share of the reduction steps
    const int nk_per = (nk_all + a.splits - 1) / a.splits;
    const int kt0 = MODE == 2 ? (int)blockIdx.y * nk_per : 0;
    const int nk = MODE == 2 ? min(nk_all, kt0 + nk_per) : nk_all;   // the plan leaves no split empty
    const int tiles_i = (a.I + BM - 1) / BM;
    const int tiles_z = tiles_i * ((a.J + BN - 1) / BN);
    const int ntiles = tiles_z * a.nb;
    // Tiles of all nb problems are numbered t = z * tiles_z + bj * tiles_i + bi.  A launch has either one workgroup
    // per tile, or (persistent: large dense problems) one workgroup per compute unit that takes every gridDim.x-th
    // tile in turn -- no workgroup start-up and drain between a compute unit's tiles.
    bool prefetched = false;   // the copies of this tile's first reduction step were issued during the previous tile's epilogue
    for (int t = blockIdx.x; t < ntiles; t += gridDim.x) {
    unsigned long long pht = 0, ph1 = 0, ph2 = 0;   // phase marks of the clock probe
    if (a.clk) pht = clock64();
    const int z = t / tiles_z, tz = t - z * tiles_z;
    const int bi = tz % tiles_i, bj = tz / tiles_i;
    const int8_t* __restrict__ P = a.P + z * a.st_p;
    const int8_t* __restrict__ Q = a.Q + z * a.st_q;
    int32_t* __restrict__ C = a.C + z * a.st_c;
    const int i0 = bi * BM, j0 = bj * BN;
    if (MODE == 2) C += (int64_t)blockIdx.y * a.st_split;

    const int rows_p = min(BM, a.I - i0), rows_q = min(BN, a.J - j0);
    __amdgpu_buffer_rsrc_t rp = CONV == 1 ? __builtin_amdgcn_make_buffer_rsrc((void*)P, 0, (int)a.p_bytes, 0x00020000)
                                          : __builtin_amdgcn_make_buffer_rsrc((void*)(P + (int64_t)i0 * a.ldp), 0, (int)(rows_p * a.ldp), 0x00020000);
    __amdgpu_buffer_rsrc_t rq = CONV == 2 ? __builtin_amdgcn_make_buffer_rsrc((void*)Q, 0, (int)a.p_bytes, 0x00020000)
                                          : __builtin_amdgcn_make_buffer_rsrc((void*)(Q + (int64_t)j0 * a.ldq), 0, (int)(rows_q * a.ldq), 0x00020000);
    // Every chunk of one thread has the same k column: chunk index c = s*T + tid, T a multiple of 8,
    // LDS slot (row = c >> 3, c & 7) holds reduction chunk (c & 7) ^ ((row >> 1) & 7) of that row.
    const int kcol = (((tid & 7) ^ ((tid >> 4) & 7))) * 16;
    int offP[CH_P], offQ[CH_Q];
    int hi0[CONV == 1 ? CH_P : 1], wi0[CONV == 1 ? CH_P : 1];   // conv: input pixel of tap (0,0) for the chunk's output pixel
    int khq[CONV == 2 ? CH_Q : 1];                              // planes: vertical tap offset (kh - pad) of the chunk's row
#pragma unroll
    for (int s = 0; s < CH_P; ++s) {
        const int row = (s * T + tid) >> 3;
        if (CONV == 1) {
            const int m = i0 + row;
            const int b = m / (a.Ho * a.Wo), rem = m - b * (a.Ho * a.Wo);
            const int ho = rem / a.Wo, wo = rem - ho * a.Wo;
            hi0[s] = m < a.I ? ho * a.stride - a.pad : -(1 << 20);   // rows beyond the matrix never pass the bounds test
            wi0[s] = wo * a.stride - a.pad;
            offP[s] = ((b * a.H + hi0[s]) * a.W + wi0[s]) * a.cpitch;
        } else {
            offP[s] = row * (int)a.ldp + kcol;
        }
    }
#pragma unroll
    for (int s = 0; s < CH_Q; ++s) {
        const int row = (s * T + tid) >> 3;
        if (CONV == 2) {
            const int j = j0 + row;   // (tap, channel) = (kh, kw, ci)
            const int tap = j / a.Cin, ci = j - tap * a.Cin;
            const int kh = tap / a.ks, kw = tap - kh * a.ks;
            khq[s] = j < a.J ? kh - a.pad : -(1 << 20);   // rows beyond the matrix never pass the bounds test
            offQ[s] = (kw * a.Cin + ci) * (int)a.ldq;
        } else {
            offQ[s] = row * (int)a.ldq + kcol;
        }
    }
    auto issue = [&](int kt, int buf) {
        const int k0 = __builtin_amdgcn_readfirstlane(kt * BK);   // wave-uniform: it travels in a scalar register
        const bool ok = k0 + kcol < Rpad;   // only the last step can have chunks beyond the reduction length
        int8_t* base = lds + buf * STAGE_BYTES;
        if (CONV == 1) {
            const int k = k0 + kcol;
            // (power-of-two channel counts and 3x3 kernels, the usual case, without integer divisions)
            const int tap = a.cin_shift >= 0 ? k >> a.cin_shift : k / a.Cin;
            const int ci0 = k - tap * a.Cin;
            const int kh = a.ks == 3 ? (tap * 11) >> 5 : tap / a.ks;
            const int kw = tap - kh * a.ks;
            const int dk = (kh * a.W + kw) * a.cpitch + ci0;
#pragma unroll
            for (int s = 0; s < CH_P; ++s) {
                const bool in = ok && (unsigned)(hi0[s] + kh) < (unsigned)a.H && (unsigned)(wi0[s] + kw) < (unsigned)a.W;
                lds_dma16(rp, in ? offP[s] + dk : OOB, 0, (unsigned)(uintptr_t)(base + (s * T + wave * 64) * 16));
            }
        } else {
#pragma unroll
            for (int s = 0; s < CH_P; ++s)
                lds_dma16(rp, ok ? offP[s] : OOB - k0, k0, (unsigned)(uintptr_t)(base + (s * T + wave * 64) * 16));
        }
        if (CONV == 2) {
            // the chunk's 16 reduction positions are 16 consecutive output pixels of one output row (W_out % 16 == 0)
            const int m = k0 + kcol;
            const int hw = a.Ho * a.Wo;
            // (power-of-two maps, the usual case, without integer divisions)
            const int b = a.hw_shift >= 0 ? m >> a.hw_shift : m / hw;
            const int rem = m - b * hw;
            const int ho = a.wo_shift >= 0 ? rem >> a.wo_shift : rem / a.Wo;
            const int wo = rem - ho * a.Wo;
            const int hb = ho * a.stride;
            const int base_in = b * a.H * a.Wo + wo;
#pragma unroll
            for (int s = 0; s < CH_Q; ++s) {
                const int hi = hb + khq[s];
                const bool in = ok && (unsigned)hi < (unsigned)a.H;
                lds_dma16(rq, in ? offQ[s] + base_in + hi * a.Wo : OOB, 0,
                          (unsigned)(uintptr_t)(base + BM * BK + (s * T + wave * 64) * 16));
            }
        } else {
#pragma unroll
            for (int s = 0; s < CH_Q; ++s)
                lds_dma16(rq, ok ? offQ[s] : OOB - k0, k0, (unsigned)(uintptr_t)(base + BM * BK + (s * T + wave * 64) * 16));
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
    v4i fp[2][TI], fq[2][TJ];
    auto ldfrag = [&](int set, const int8_t* sb, int ks) {
#pragma unroll
        for (int ti = 0; ti < TI; ++ti) fp[set][ti] = *(const v4i*)(sb + swz(wm * WTM + ti * 32 + lr, ks * 2 + lh));
#pragma unroll
        for (int tj = 0; tj < TJ; ++tj) fq[set][tj] = *(const v4i*)(sb + BM * BK + swz(wn * WTN + tj * 32 + lr, ks * 2 + lh));
    };
    auto mma = [&](int set) {
#pragma unroll
        for (int ti = 0; ti < TI; ++ti)
#pragma unroll
            for (int tj = 0; tj < TJ; ++tj)
                acc[ti][tj] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fq[set][tj], fp[set][ti], acc[ti][tj], 0, 0, 0);
    };

    // Pipeline: stage kt is multiplied while the copy of stage kt+1 is in flight.  The last fragment reads of
    // stage kt are issued before the barrier of step kt, so its buffer is free right after that barrier and
    // the copy of stage kt+2 is issued there: one copy is in flight at every moment, each with a whole step
    // of time to land.
#if FF_PRO2
    if (PREFETCH && prefetched) {
        // Step 0 is in LDS already: every wavefront waited for its own copies of it before the stores of the previous
        // epilogue, and the barrier at the end of that tile made them visible to all.  Only step 1 goes out now; the
        // main loop waits for it (and, copies and stores completing in issue order, for the previous tile's stores).
        if (kt0 + 1 < nk) issue(kt0 + 1, 1);
        ldfrag(0, lds, 0);
    } else {
    // all stages are free at the start of a tile: the copies of the first NS steps go out together, so that only
    // one round trip to memory is exposed (copies complete in issue order)
    issue(kt0, 0);
#pragma unroll
    for (int i = 1; i < NS; ++i)
        if (kt0 + i < nk) issue(kt0 + i, i);
    if (kt0 + NS - 1 < nk) wait_vmcnt<(NS - 1) * CH>();
    else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    ldfrag(0, lds, 0);
    }
#else
    issue(kt0, 0);
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    ldfrag(0, lds, 0);
    if (kt0 + 1 < nk) issue(kt0 + 1, 1);
#endif
    if (a.clk) ph1 = clock64();
    int cur = 0;   // stage of step kt: (kt - kt0) % NS
    for (int kt = kt0; kt < nk; ++kt) {
        const int nxt = cur + 1 == NS ? 0 : cur + 1;
        const int8_t* sb = lds + cur * STAGE_BYTES;
        const int8_t* sn = lds + nxt * STAGE_BYTES;
        ldfrag(1, sb, 1);
        mma(0);
        ldfrag(0, sb, 2);
        mma(1);
        ldfrag(1, sb, 3);
        mma(0);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        // the copies of step kt + 1 must have landed; those of the NS - 2 steps after it may stay in flight (near the
        // end of the reduction fewer are outstanding: wait for all)
        if (NS > 2 && kt + NS - 1 < nk) wait_vmcnt<(NS - 2) * CH>();
        else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
#if FF_SPLIT_ISSUE
        // The copy instructions of a step keep the address unit busy for about a thousand clocks (64 KB at 64 bytes
        // per clock).  Half of the wavefronts -- one of the two on every SIMD -- issue theirs before the last
        // multiplies of the step, the other half after them, so that every SIMD has multiplies to run while the
        // copies queue up.
        const bool early = wave < WM * WN / 2;
        if (early && kt + NS < nk) issue(kt + NS, cur);
        if (kt + 1 < nk) ldfrag(0, sn, 0);
        mma(1);
        if (!early && kt + NS < nk) issue(kt + NS, cur);
#else
        if (kt + NS < nk) issue(kt + NS, cur);
        if (kt + 1 < nk) ldfrag(0, sn, 0);
        mma(1);
#endif
        cur = nxt;
    }

    // Epilogue.  A lane holds, per accumulator quad, four consecutive columns of ONE row, so a direct store
    // instruction writes 32-byte pieces of 32 different rows.  Interior tiles therefore go through LDS (free
    // after the main loop; each wave uses a private slice, no barrier needed): 16-byte writes row by row,
    // then reads that give every store instruction whole contiguous row segments of WTN*4 bytes.
    // Edge tiles take the same route when J is a multiple of 4 (a lane's 16 bytes then never straddle the last
    // column): rows and column groups beyond the matrix are simply not stored.
    if (a.clk) ph2 = clock64();
    // Persistent launches of the big dense tile: the copies of the NEXT tile's first reduction step go out now, into
    // the first operand stage (nobody reads the stages any more; the staging below keeps to the second one), so that
    // their round trip to memory runs under this tile's epilogue instead of in front of the next tile's main loop.
    bool wait_copies = false;
    prefetched = false;
    if (PREFETCH && t + (int)gridDim.x < ntiles) {
        const int tn = t + (int)gridDim.x;
        const int zn = tn / tiles_z, tzn = tn - zn * tiles_z;
        const int i0n = (tzn % tiles_i) * BM, j0n = (tzn / tiles_i) * BN;
        if (CONV == 1) {
            // the pixel offsets of the current tile are not needed any more: those of the next one take their place
            rp = __builtin_amdgcn_make_buffer_rsrc((void*)(a.P + zn * a.st_p), 0, (int)a.p_bytes, 0x00020000);
#pragma unroll
            for (int s = 0; s < CH_P; ++s) {
                const int m = i0n + ((s * T + tid) >> 3);
                const int b = m / (a.Ho * a.Wo), rem = m - b * (a.Ho * a.Wo);
                const int ho = rem / a.Wo, wo = rem - ho * a.Wo;
                hi0[s] = m < a.I ? ho * a.stride - a.pad : -(1 << 20);
                wi0[s] = wo * a.stride - a.pad;
                offP[s] = ((b * a.H + hi0[s]) * a.W + wi0[s]) * a.cpitch;
            }
        } else {
            rp = __builtin_amdgcn_make_buffer_rsrc((void*)(a.P + zn * a.st_p + (int64_t)i0n * a.ldp), 0, (int)(min(BM, a.I - i0n) * a.ldp), 0x00020000);
        }
        rq = __builtin_amdgcn_make_buffer_rsrc((void*)(a.Q + zn * a.st_q + (int64_t)j0n * a.ldq), 0, (int)(min(BN, a.J - j0n) * a.ldq), 0x00020000);
        issue(0, 0);
        prefetched = true;
        wait_copies = true;
    }
    const bool interior = i0 + BM <= a.I && j0 + BN <= a.J;
    const bool staged = FF_STAGED_EPI && (interior || (a.J & 3) == 0);
    const bool fast_sq = a.relu && a.rshift == 0;
    int8_t* const ebase = lds + EOFF + wave * ESLICE;
    if (wait_copies && !staged) {   // (copies and stores complete in issue order: wait before the first store)
        wait_vmcnt<0>();
        wait_copies = false;
    }
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
                if (!staged && i < a.I) {
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
                    const int cc[4] = {c0, c1, c2, c3};
                    if (fast_sq) {
                        // ReLU and no pre-shift (every dense layer): one 32x32+64-bit multiply-add per element
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const unsigned v = (unsigned)max(cc[e], 0);
                            sq += (unsigned long long)v * v;
                            vm = max(vm, (int)v);
                        }
                    } else {
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
        }
        if (staged) {
            // EROWS rows of the 32 at a time: the lanes that hold those rows write their quads, then every store
            // instruction takes whole contiguous row segments
#pragma unroll
            for (int h = 0; h < 32 / EROWS; ++h) {
                if (EROWS == 32 || (lr / EROWS) == h) {
#pragma unroll
                    for (int tj = 0; tj < TJ; ++tj)
#pragma unroll
                        for (int g = 0; g < 4; ++g)
                            *(v4i*)(ebase + (lr % EROWS) * EROW + (tj * 32 + 8 * g + 4 * lh) * 4) =
                                (v4i){acc[ti][tj][4 * g + 0], acc[ti][tj][4 * g + 1], acc[ti][tj][4 * g + 2], acc[ti][tj][4 * g + 3]};
                }
                wave_lds_fence();
                if (wait_copies) {   // once per tile, before its first store (copies and stores complete in issue order)
                    wait_vmcnt<0>();
                    wait_copies = false;
                }
                constexpr int LPR = WTN / 4;          // lanes (16 bytes each) per staged row
                constexpr int RPI = 64 / LPR;         // rows per store instruction
                const int rl = lane / LPR, cc = lane - rl * LPR;
                const int row0 = i0 + wm * WTM + ti * 32 + h * EROWS;
                int32_t* const ctile = C + (int64_t)row0 * a.ldc + j0 + wn * WTN + cc * 4;
#pragma unroll
                for (int r = 0; r < EROWS / RPI; ++r) {
                    const int row = r * RPI + rl;
                    const v4i v = *(const v4i*)(ebase + row * EROW + cc * 16);
                    if (!interior && (row0 + row >= a.I || j0 + wn * WTN + cc * 4 >= a.J)) continue;
                    // forward accumulators are not read again until other kernels have streamed more than the caches
                    // hold: a non-temporal store keeps them from displacing what is needed next.  Weight gradients are
                    // read by the update right away: ordinary stores.
                    if (MODE == 1) __builtin_nontemporal_store(v, (v4i*)(ctile + (int64_t)row * a.ldc));
                    else *(v4i*)(ctile + (int64_t)row * a.ldc) = v;
                }
                wave_lds_fence();
            }
        }
        if (EPI) {
            // the two half-waves hold the two column halves of the same row
            sq += shfl_xor_u64(sq, 32);
            vm = max(vm, __shfl_xor(vm, 32));
            if ((a.rows_per_sample & 31) == 0) {
                // all 32 rows of this MFMA tile belong to one sample (convolution): one atomic per wave.
                // Rows beyond the matrix hold exact zeros and add nothing.
#pragma unroll
                for (int d = 1; d < 32; d <<= 1) {
                    sq += shfl_xor_u64(sq, d);
                    vm = max(vm, __shfl_xor(vm, d));
                }
                const int i_first = i0 + wm * WTM + ti * 32;
                if (lane == 0 && i_first < a.I) {
                    const int smp = i_first / a.rows_per_sample;
                    atomicAdd(a.gsum + z * a.st_g + smp, sq);
                    atomicMax(a.vmax + z * a.st_g + smp, vm);
                }
            } else if (lh == 0 && i < a.I) {
                const int smp = i / a.rows_per_sample;
                atomicAdd(a.gsum + z * a.st_g + smp, sq);
                atomicMax(a.vmax + z * a.st_g + smp, vm);
            }
        }
    }
    // the staging slices of the epilogue lie in the operand stages: every wave must be done with them before the
    // copies of the next tile land there
    unsigned long long ph3 = 0;
    if (a.clk) ph3 = clock64();
    if (t + (int)gridDim.x < ntiles) __builtin_amdgcn_s_barrier();
    if (a.clk) {
        // shader clocks of this tile by phase: slots 2.. for plain / split launches, 8.. for forward launches
        const unsigned long long ph4 = clock64();
        if (threadIdx.x == 0) {
        unsigned long long* pc = a.clk + (MODE == 1 ? 8 : 2);
        atomicAdd(pc + 0, ph1 - pht);   // tile start to the first fragments (operand round trip)
        atomicAdd(pc + 1, ph2 - ph1);   // main loop
        atomicAdd(pc + 2, ph3 - ph2);   // epilogue of wave 0
        atomicAdd(pc + 3, ph4 - ph3);   // waiting for the other waves' epilogues
        atomicAdd(pc + 4, 1ull);        // tiles
        }
    }
    }   // tile loop
    if (a.clk && threadIdx.x == 0) {
        atomicAdd(a.clk + 0, (unsigned long long)clock64() - clk0);
        atomicAdd(a.clk + 1, (unsigned long long)wall_clock64() - rt0);
    }
}


int num_cus()
{
    static int n = 0;   // (one GPU model per process: the count of the first device queried is kept)
    if (n == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) n = v;
        else n = 256;
    }
    return n;
}

template <int BM, int BN, int WM, int WN>
static hipError_t launch_cfg(const GemmArgs& a, hipStream_t s)
{
    const int tiles_i = (a.I + BM - 1) / BM, tiles_j = (a.J + BN - 1) / BN;
    const int64_t ntiles = (int64_t)tiles_i * tiles_j * a.nb;
    if (ntiles > 0x7FFFFFFF) return hipErrorInvalidValue;
    const int mode = a.splits > 1 ? 2 : (a.gsum ? 1 : 0);
    // persistent launch (256-row tiles of dense and implicit-convolution operands): as many workgroups as fit the chip at
    // once -- one per compute unit, two where a workgroup takes at most half of the LDS -- when each has at least two
    // whole tiles
    int64_t gx = ntiles;
    if (FF_PERSIST && FF_NEXT_TILE_PREFETCH && BM == 256 && a.conv != 2 && mode != 2) {
        const int stage = (BM + BN) * BK, eslice = (BN == 256 ? 16 : 32) * (BN / WN * 4 + 16);
        const int lds = 2 * stage > stage + WM * WN * eslice ? 2 * stage : stage + WM * WN * eslice;   // as in the kernel
        const int64_t resident = (int64_t)num_cus() * (lds <= 80 * 1024 ? 2 : 1);
        if (ntiles >= 2 * resident && ntiles % resident == 0) gx = resident;
    }
    const dim3 grid((unsigned)gx, (unsigned)a.splits, 1), block(WM * WN * 64);
    if (a.conv == 1) {
        if (mode == 1) hipLaunchKernelGGL((k_gemm_nt_i8<BM, BN, WM, WN, 1, 1>), grid, block, 0, s, a);
        else if (mode == 0) hipLaunchKernelGGL((k_gemm_nt_i8<BM, BN, WM, WN, 0, 1>), grid, block, 0, s, a);
        else return hipErrorInvalidValue;
    } else if (a.conv == 2) {
        if (mode == 2) hipLaunchKernelGGL((k_gemm_nt_i8<BM, BN, WM, WN, 2, 2>), grid, block, 0, s, a);
        else if (mode == 0) hipLaunchKernelGGL((k_gemm_nt_i8<BM, BN, WM, WN, 0, 2>), grid, block, 0, s, a);
        else return hipErrorInvalidValue;
    } else {
        if (mode == 1) hipLaunchKernelGGL((k_gemm_nt_i8<BM, BN, WM, WN, 1, 0>), grid, block, 0, s, a);
        else if (mode == 0) hipLaunchKernelGGL((k_gemm_nt_i8<BM, BN, WM, WN, 0, 0>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((k_gemm_nt_i8<BM, BN, WM, WN, 2, 0>), grid, block, 0, s, a);
    }
    return hipGetLastError();
}

// Tile shape and number of reduction splits for one launch.
//  * The tile is as wide as the output allows (a 256-wide tile on a 64-column output would waste three
//    quarters of the MFMA work) and tall only if that still leaves about two workgroups per compute unit.
//  * allow_split (weight gradients): when the output alone has too few tiles -- a convolution's weight
//    gradient has few output elements and a very long reduction -- a split reduction fills the chip.
GemmPlan gemm_plan(int64_t I, int64_t J, int64_t R, int nb, bool allow_split)
{
    GemmPlan p;
    p.splits = 1;
    // edge of the tile along one dimension: weigh the padding it leaves against the lower efficiency of narrow
    // tiles (relative MFMA rates measured on this kernel: 256 -> 1, 128 -> 0.85, 64 -> 0.65)
    auto edge = [](int64_t n) {
        const int e[3] = {256, 128, 64};
        const double eff[3] = {1.0, 0.85, 0.65};
        int best = 64;
        double score = -1.0;
        for (int i = 0; i < 3; ++i) {
            const double sc = eff[i] * (double)n / (double)((n + e[i] - 1) / e[i] * e[i]);
            if (sc > score + 1e-9) { score = sc; best = e[i]; }
        }
        return best;
    };
    p.bn = edge(J);
    auto tiles = [&](int bm, int bn) { return ((I + bm - 1) / bm) * ((J + bn - 1) / bn) * nb; };
    const int64_t nk = (R + BK - 1) / BK;
    if (allow_split && tiles(edge(I), p.bn) < 384 && nk >= 32) {
        // Weight gradient of a convolution: few output elements, a very long reduction.  Keep the tile as large as
        // the output allows (operand traffic falls with the tile edge) and create the missing parallelism by
        // splitting the reduction: about two workgroups per compute unit, never more (a third partial round
        // would idle most of the chip), at least 16 reduction steps per split.
        p.bm = edge(I);
        // (a 256 x 256 tile takes 128 KB of LDS, one workgroup per compute unit: one round of 256 workgroups, each with
        // twice the reduction steps, writes and re-reads half the partial sums of two rounds of 512)
        int64_t sp = (p.bm == 256 && p.bn == 256 ? FF_SPLIT_TARGET_BIG : 512) / tiles(p.bm, p.bn);
        // ... (8 where one partial result is small, at most 256 KB: writing and adding up the partials then costs little)
        const int64_t min_steps = I * J * 4 <= (256 << 10) ? 8 : 16;
        if (sp > nk / min_steps) sp = nk / min_steps;
        if (sp < 1) sp = 1;
        const int64_t per = (nk + sp - 1) / sp;
        p.splits = (int)((nk + per - 1) / per);   // no split without reduction steps
        return p;
    }
    // tall tiles only if that still leaves about two workgroups per compute unit
    p.bm = (I > 128 && tiles(256, p.bn) >= 512) ? 256 : ((I > 64 && tiles(128, p.bn) >= 512) ? 128 : 64);
    // even the shortest tile leaves under two workgroups per compute unit: narrower tiles (measured on 2048 x 2000 x 2000:
    // 64 x 128 tiles 13 % faster than 64 x 256)
    if (p.bm == 64 && p.bn == 256 && tiles(64, 256) < 512) p.bn = 128;
    return p;
}

__global__ __launch_bounds__(256) void k_reduce_splits(const int32_t* __restrict__ part, int splits, int64_t st_split,
                                                       int64_t st_part_z, int32_t* __restrict__ out, int64_t st_out_z,
                                                       int64_t n4)
{
    const int4* __restrict__ p = (const int4*)(part + blockIdx.y * st_part_z);
    int4* __restrict__ o = (int4*)(out + blockIdx.y * st_out_z);
    const int64_t s4 = st_split >> 2;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < n4; e += (int64_t)gridDim.x * 256) {
        int4 acc = p[e];
        for (int s = 1; s < splits; ++s) {
            const int4 v = p[e + s * s4];
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
        o[e] = acc;
    }
}

// Many splits of a small output (convolutions with few channels): a thread of the kernel above would walk the splits
// one dependent load after the other.  Here 16 lanes share the splits of each 16-byte group and meet in LDS.
__global__ __launch_bounds__(256) void k_reduce_splits_wide(const int32_t* __restrict__ part, int splits, int64_t st_split,
                                                            int64_t st_part_z, int32_t* __restrict__ out, int64_t st_out_z,
                                                            int64_t n4)
{
    const int4* __restrict__ p = (const int4*)(part + blockIdx.y * st_part_z);
    int4* __restrict__ o = (int4*)(out + blockIdx.y * st_out_z);
    const int64_t s4 = st_split >> 2;
    const int el = threadIdx.x & 15, sl = threadIdx.x >> 4;
    const int64_t e = (int64_t)blockIdx.x * 16 + el;
    int4 acc = make_int4(0, 0, 0, 0);
    if (e < n4)
        for (int sp = sl; sp < splits; sp += 16) {
            const int4 v = p[e + sp * s4];
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
    __shared__ int4 red[16][16];
    red[sl][el] = acc;
    __syncthreads();
    if (sl == 0 && e < n4) {
#pragma unroll
        for (int r = 1; r < 16; ++r) {
            const int4 v = red[r][el];
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
        o[e] = acc;
    }
}

hipError_t launch_reduce_splits(const int32_t* part, int splits, int64_t st_split, int64_t st_part_z, int32_t* out,
                                int64_t st_out_z, int64_t n, int nb, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    const int64_t n4 = n >> 2;
    if (splits >= 32 && n4 <= (int64_t(1) << 20)) {
        hipLaunchKernelGGL(k_reduce_splits_wide, dim3((unsigned)((n4 + 15) / 16), (unsigned)nb), dim3(256), 0, s, part,
                           splits, st_split, st_part_z, out, st_out_z, n4);
        return hipGetLastError();
    }
    int64_t blocks = (n4 + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(k_reduce_splits, dim3((unsigned)blocks, (unsigned)nb), dim3(256), 0, s, part, splits, st_split,
                       st_part_z, out, st_out_z, n4);
    return hipGetLastError();
}

hipError_t launch_gemm_nt_i8(const GemmArgs& a_in, hipStream_t s)
{
    GemmArgs a = a_in;   // (the loaders' shift counts are filled in below)
    if (a.I <= 0 || a.J <= 0) return hipSuccess;
    // byte offsets of the operand copies are 32-bit (tile-relative for dense operands, tensor-relative for conv)
    if (a.ldp >= (int64_t(1) << 22) || a.ldq >= (int64_t(1) << 22)) return hipErrorInvalidValue;
    if (a.conv == 1 && (a.p_bytes >= (int64_t(1) << 31) || (a.Cin & 15) != 0)) return hipErrorInvalidValue;
    // planes: chunks of 16 output pixels must lie in one output row; the reduction covers whole samples
    if (a.conv == 2 && (a.p_bytes >= (int64_t(1) << 31) || (a.Wo & 15) != 0 || a.R % (a.Ho * a.Wo) != 0 || a.gsum))
        return hipErrorInvalidValue;
    if (a.conv < 0 || a.conv > 2) return hipErrorInvalidValue;
    if (a.splits < 1 || (a.splits > 1 && (a.gsum || a.conv == 1))) return hipErrorInvalidValue;
    auto shift_of = [](int v) {   // log2 of a power of two, else -1
        if (v <= 0 || (v & (v - 1)) != 0) return -1;
        int sh = 0;
        while ((1 << sh) < v) ++sh;
        return sh;
    };
    a.cin_shift = a.conv == 1 ? shift_of(a.Cin) : -1;
    a.hw_shift = a.conv == 2 ? shift_of(a.Ho * a.Wo) : -1;
    a.wo_shift = a.conv == 2 ? shift_of(a.Wo) : -1;
    GemmPlan p = gemm_plan(a.I, a.J, a.R, a.nb, a.splits > 1);
    const int bm = p.bm, bn = p.bn;
    if (bn == 256) {
        if (bm == 256) return launch_cfg<256, 256, 4, 2>(a, s);
        if (bm == 128) return launch_cfg<128, 256, 2, 2>(a, s);
        return launch_cfg<64, 256, 1, 4>(a, s);
    }
    if (bn == 128) {
        if (bm == 256) return launch_cfg<256, 128, 4, 2>(a, s);
        if (bm == 128) return launch_cfg<128, 128, 2, 2>(a, s);
        return launch_cfg<64, 128, 2, 2>(a, s);
    }
    if (bm == 256) return launch_cfg<256, 64, 4, 1>(a, s);
    if (bm == 128) return launch_cfg<128, 64, 4, 1>(a, s);
    return launch_cfg<64, 64, 2, 2>(a, s);
}

// ------------------------------------------------------------------------------------------------------------
// Ceiling probe: nothing but v_mfma_i32_32x32x32_i8 on register-resident operands, two wavefronts per SIMD, eight
// independent accumulators per wavefront (the contraction kernel's own shape of MFMA work, without any operand
// movement).  What it sustains on a given kind of operand values is the most the matrix pipes deliver under the
// power manager: the datasheet rate on zeros, clearly less once every multiplier input toggles.
// ------------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(512) void k_mfma_ceiling(int32_t* __restrict__ sink, int iters, int kind,
                                                      unsigned long long* __restrict__ clk)
{
    unsigned long long c0 = 0, r0 = 0;
    if (clk) {
        c0 = clock64();
        r0 = wall_clock64();
    }
    v16i acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0;
    // operand words: 0 -> zeros, 1 -> every code 1, 2 -> one pseudo-random word per lane and register
    v4i fa[4], fb[2];
#pragma unroll
    for (int i = 0; i < 6; ++i)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            uint32_t h = (threadIdx.x * 24u + (uint32_t)(i * 4 + v) + 1u) * 0x9E3779B1u;
            h ^= h >> 15;
            h *= 0x85EBCA6Bu;
            h ^= h >> 13;
            const int word = kind == 0 ? 0 : (kind == 1 ? 0x01010101 : (int)h);
            if (i < 4) fa[i][v] = word;
            else fb[i - 4][v] = word;
        }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i & 3], fb[i >> 2], acc[i], 0, 0, 0);
    }
    int sum = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) sum += acc[i][v];
    sink[blockIdx.x * 512 + threadIdx.x] = sum;   // keeps the accumulators live
    if (clk && threadIdx.x == 0) {
        atomicAdd(clk + 0, (unsigned long long)clock64() - c0);
        atomicAdd(clk + 1, (unsigned long long)wall_clock64() - r0);
    }
}

hipError_t launch_mfma_ceiling(int32_t* sink, int iters, int kind, unsigned long long* clk, int* workgroups, hipStream_t s)
{
    const int g = num_cus();
    if (workgroups) *workgroups = g;
    hipLaunchKernelGGL(k_mfma_ceiling, dim3((unsigned)g), dim3(512), 0, s, sink, iters, kind, clk);
    return hipGetLastError();
}

}  // namespace ffi
