// One iteration of Algorithm 1 for a SMALL dense stack as a single persistent kernel (gfx950).
//
// The regime nearest the paper's own batch of 32 (Section V-A) is bound by launch latency, not by arithmetic:
// a step of 784 -> 500 -> 500 at 64 + 64 samples is 18 dependent kernels of 2-10 us each.  Here the whole step --
// quantise (Section IV-B), int8 forward contraction with the goodness sums (Algorithm 1), losses and their
// derivatives (Eq. (1), Eq. (2)), look-ahead (Eq. (3), Eq. (4)), int8 local gradient, int8 weight gradient, update and
// requantisation -- runs in ONE launch of a few dozen workgroups that meet at a device-wide barrier wherever the
// method has a true device-wide dependency (a per-tensor absmax, a per-sample goodness).  The arithmetic is the one
// the per-operation kernels use (device_math.hpp; same operation order), so both paths give the same bits.
//
// Work inside a phase is spread by grid-stride loops over all threads of the launch; contractions give every
// wavefront 32 x 32 output tiles (v_mfma_i32_32x32x32_i8, fragments straight from global memory: the operands of such
// a step fit the L2 many times over), with the reduction split over the wavefronts of a workgroup when there are no
// more tiles than workgroups.  All sizes are small by construction (the launcher checks them), so element indices
// are 32-bit.
//
// Barrier: one counter; every workgroup adds one and spins until the count reaches (barrier number) x (workgroups).
// All workgroups must be resident at once, which holds because the grid is at most one workgroup per compute unit.
// Agent-scope release / acquire fences on the two sides make the phases' global writes visible across the XCDs' L2
// caches.  The counter lives in a small static array of the library's device image (zero when the library is loaded);
// the workgroup that leaves the kernel last sets it back to zero, so the launch needs no clearing kernel in front of
// it and can be replayed from a HIP graph.  Launches that overlap on one GPU would share the counter: serialise them.
#include <mutex>

#include "device_math.hpp"
#include "ff_internal.hpp"

namespace ffi {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int FU_WAVES = FU_THREADS / 64;

// [0] barrier counter, [1] set when a barrier wait ran into its bound, [2] count of workgroups that have left
static __device__ __align__(256) unsigned g_fu_sync[64];

__device__ __forceinline__ unsigned long long shfl_xor_u64f(unsigned long long v, int d)
{
    const unsigned lo = (unsigned)__shfl_xor((int)(unsigned)v, d), hi = (unsigned)__shfl_xor((int)(unsigned)(v >> 32), d);
    return ((unsigned long long)hi << 32) | lo;
}

struct FuCtx {
    unsigned* bar;
    unsigned long long* stamps;   // instrumentation (null normally): workgroup 0 records the 100 MHz clock after every barrier
    unsigned epoch, G;
    int gtid, gsz;   // global thread index / thread count
};

__device__ __forceinline__ void grid_barrier(FuCtx& c)
{
    __syncthreads();   // every wavefront's stores of the phase have reached the L2
    c.epoch += 1;
    if (threadIdx.x == 0) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");   // write the phase's data back past this XCD's L2
        __hip_atomic_fetch_add(c.bar, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned target = c.epoch * c.G;
        // Every workgroup reaches every barrier, so the wait ends as soon as the slowest one arrives.  The spin is
        // bounded all the same (about a second): should a workgroup ever fail to arrive, the others leave with wrong
        // results and bar[1] set instead of holding the GPU.
        unsigned spins = 0;
        while (__hip_atomic_load(c.bar, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            __builtin_amdgcn_s_sleep(1);
            if (++spins > (1u << 20)) {
                __hip_atomic_store(c.bar + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        if (c.stamps && blockIdx.x == 0) c.stamps[c.epoch] = wall_clock64();
    }
    __syncthreads();
}

__device__ __forceinline__ float ld_f32(const float* p)   // a scalar another workgroup wrote in an earlier phase
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t ld_u32(const uint32_t* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---- quantiser over 4 x 4 element blocks -------------------------------------------------------------------------
// KIND 0: fp32 tensor; 1: hand-off from accumulators (optionally divided by sqrt(goodness)); 2: local gradient
struct FuQuant {
    const float* x;        // KIND 0: [rows, cols]
    const int32_t* acc;    // KIND 1, 2: [rows, ldacc]
    int ldacc;
    float s_y;             // KIND 1, 2
    int relu, l2norm;
    const float* rowf_lds; // KIND 1 with l2norm: goodness per row (LDS)
    const float* ct;       // KIND 2: coeff_total per row (global)
    float amax;
    uint32_t k0;           // low word of the random stream's key
    int rows, cols;
    int8_t* q;  int ldq;   // null or [rows, ldq]
    int8_t* q_t; int ldqt; // null or [cols, ldqt]
    float* scale;
};

// one 4 x 4 block: rows 4 rb .., columns 4 cb ..
template <int KIND, bool STOCH>
__device__ __forceinline__ void fu_quantize_block(const FuQuant& a, float inv, int rb, int cb)
{
    const bool vec = KIND != 0 || ((a.cols & 3) == 0 && (((uintptr_t)a.x) & 15) == 0);
    const int col0 = 4 * cb;
    uint32_t rowpack[4];
    // all loads of the block first
    float v[4][4];
    float rf[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = 4 * rb + j;
        rf[j] = 1.0f;
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) v[j][cc] = 0.0f;
        if (row < a.rows && col0 < a.cols) {
            if (KIND == 0) {
                const float* px = a.x + row * a.cols + col0;
                if (vec) {
                    const v4f f = *(const v4f*)px;
                    v[j][0] = f.x; v[j][1] = f.y; v[j][2] = f.z; v[j][3] = f.w;
                } else {
#pragma unroll
                    for (int cc = 0; cc < 4; ++cc) if (col0 + cc < a.cols) v[j][cc] = px[cc];
                }
            } else {
                const v4i f = *(const v4i*)(a.acc + row * a.ldacc + col0);   // the pitch is a multiple of 4
#pragma unroll
                for (int cc = 0; cc < 4; ++cc) v[j][cc] = (float)f[cc];
                if (KIND == 2) rf[j] = 2.0f * a.ct[row];
                else if (a.l2norm) rf[j] = sqrtf(a.rowf_lds[row]);
            }
        }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = 4 * rb + j;
        uint32_t pack = 0;
        if (row < a.rows && col0 < a.cols) {
            const uint32_t idx = (uint32_t)row * (uint32_t)a.cols + (uint32_t)col0;
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) {
                float t = v[j][cc];
                if (KIND != 0) {
                    t = t * a.s_y;
                    if (a.relu) t = fmaxf(t, 0.0f);
                    if (KIND == 2) t = rf[j] * t;
                    else if (a.l2norm) t = rf[j] > 0.0f ? t / rf[j] : 0.0f;
                }
                if (col0 + cc < a.cols) {   // (the accumulators' pad columns hold junk)
                    const int code = quant_code<STOCH>(t, inv, (idx + (uint32_t)cc) ^ a.k0);
                    pack |= ((uint32_t)code & 0xFFu) << (8 * cc);
                }
            }
        }
        rowpack[j] = pack;
        if (a.q && row < a.rows && col0 < a.ldq) *(uint32_t*)(a.q + row * a.ldq + col0) = pack;
    }
    if (a.q_t && 4 * rb < a.ldqt) {
        const uint32_t t0 = __builtin_amdgcn_perm(rowpack[1], rowpack[0], 0x05010400u);
        const uint32_t t1 = __builtin_amdgcn_perm(rowpack[1], rowpack[0], 0x07030602u);
        const uint32_t t2 = __builtin_amdgcn_perm(rowpack[3], rowpack[2], 0x05010400u);
        const uint32_t t3 = __builtin_amdgcn_perm(rowpack[3], rowpack[2], 0x07030602u);
        const uint32_t colpack[4] = {__builtin_amdgcn_perm(t2, t0, 0x05040100u), __builtin_amdgcn_perm(t2, t0, 0x07060302u),
                                     __builtin_amdgcn_perm(t3, t1, 0x05040100u), __builtin_amdgcn_perm(t3, t1, 0x07060302u)};
#pragma unroll
        for (int cc = 0; cc < 4; ++cc)
            if (col0 + cc < a.cols) *(uint32_t*)(a.q_t + (col0 + cc) * a.ldqt + 4 * rb) = colpack[cc];
    }
}

__device__ __forceinline__ int fu_quant_blocks(const FuQuant& a, int& ncb)
{
    const int rext = a.q_t ? max(a.ldqt, a.rows) : a.rows;
    const int cext = a.q ? max(a.ldq, a.cols) : a.cols;
    ncb = (cext + 3) >> 2;
    return ((rext + 3) >> 2) * ncb;
}

// tid0 / nthreads: this thread's index and the thread count among the threads that share the tensor
template <int KIND, bool STOCH>
__device__ __forceinline__ void fu_quantize(const FuQuant& a, int tid0, int nthreads)
{
    const bool live = a.amax >= 0x1p-100f;
    const float inv = live ? 127.0f / a.amax : 0.0f;
    if (tid0 == 0) *a.scale = live ? a.amax / 127.0f : 1.0f;
    int ncb;
    const int nb = fu_quant_blocks(a, ncb);
    for (int e = tid0; e < nb; e += nthreads) {
        const int rb = e / ncb, cb = e - rb * ncb;
        fu_quantize_block<KIND, STOCH>(a, inv, rb, cb);
    }
}

// ---- int8 contraction C[i][j] = sum_r P[i][r] * Q[j][r] over 32 x 32 tiles --------------------------------------------
struct FuGemm {
    const int8_t* P; const int8_t* Q; int32_t* C;
    int I, J, R;
    int ldp, ldq, ldc;
    unsigned long long* gsum;   // per row of C (null: plain contraction)
    int32_t* vmax;
    int relu, rshift;
};

// part / nparts: this wavefront's share of the reduction steps of the tile (ti, tj)
__device__ __forceinline__ v16i fu_tile(const FuGemm& g, int ti, int tj, int part, int nparts, int lane)
{
    const int lr = lane & 31, lh = lane >> 5;
    const int Rpad = (g.R + 15) & ~15;
    const int nks = (Rpad + 31) >> 5;
    const int per = (nks + nparts - 1) / nparts;
    const int ks0 = part * per, ks1 = min(nks, ks0 + per);
    const int i = ti * 32 + lr, j = tj * 32 + lr;
    const int8_t* pp = g.P + i * g.ldp + 16 * lh;
    const int8_t* pq = g.Q + j * g.ldq + 16 * lh;
    const bool pin = i < g.I, qin = j < g.J;
    v16i acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0;
    const v4i zero = {0, 0, 0, 0};
    for (int ks = ks0; ks < ks1; ks += 4) {
        v4i fp[4], fq[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int k0 = (ks + u) * 32;
            const bool kin = ks + u < ks1 && k0 + 16 * lh < Rpad;
            fp[u] = (kin && pin) ? *(const v4i*)(pp + k0) : zero;
            fq[u] = (kin && qin) ? *(const v4i*)(pq + k0) : zero;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(fq[u], fp[u], acc, 0, 0, 0);
    }
    return acc;
}

// a lane holds row i = 32 ti + (lane & 31), columns 32 tj + 8 g + 4 (lane >> 5) + e at acc[4 g + e]
__device__ __forceinline__ void fu_tile_store(const FuGemm& g, int ti, int tj, const v16i& acc, int lane)
{
    const int lr = lane & 31, lh = lane >> 5;
    const int i = ti * 32 + lr;
    unsigned long long sq = 0;
    int vm = 0;
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) {
        const int j = tj * 32 + 8 * gq + 4 * lh;
        if (i < g.I && j < g.J) {
            if ((g.J & 3) == 0) {   // 16-byte store (the pitch is a multiple of 4)
                *(v4i*)(g.C + i * g.ldc + j) = (v4i){acc[4 * gq], acc[4 * gq + 1], acc[4 * gq + 2], acc[4 * gq + 3]};
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) if (j + e < g.J) g.C[i * g.ldc + j + e] = acc[4 * gq + e];
            }
        }
        if (g.gsum) {   // columns beyond J hold exact zeros and add nothing
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                int v = acc[4 * gq + e];
                if (g.relu) v = max(v, 0);
                const long long vl = (long long)v;
                sq += ((unsigned long long)(vl * vl)) >> g.rshift;
                vm = max(vm, v < 0 ? -v : v);
            }
        }
    }
    if (g.gsum) {
        sq += shfl_xor_u64f(sq, 32);
        vm = max(vm, __shfl_xor(vm, 32));
        if (lh == 0 && i < g.I) {
            atomicAdd(g.gsum + i, sq);
            atomicMax(g.vmax + i, vm);
        }
    }
}

// All problems of one phase; `get(p)` builds problem p, tiles are numbered problem by problem.
template <typename F>
__device__ __forceinline__ void fu_gemm_phase(F get, int np, const FuCtx& c, int* red /* LDS: (FU_WAVES - 1) x 16 x 64 ints */)
{
    int total = 0;
    for (int p = 0; p < np; ++p) {
        const FuGemm g = get(p);
        total += ((g.I + 31) >> 5) * ((g.J + 31) >> 5);
    }
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    auto locate = [&](int t, int& ti, int& tj) -> FuGemm {
        int p = 0;
        FuGemm g = get(0);
        int n = ((g.I + 31) >> 5) * ((g.J + 31) >> 5);
        while (t >= n && p + 1 < np) {
            t -= n;
            g = get(++p);
            n = ((g.I + 31) >> 5) * ((g.J + 31) >> 5);
        }
        const int tn = (g.J + 31) >> 5;
        ti = t / tn;
        tj = t - ti * tn;
        return g;
    };
    if (total <= (int)c.G) {
        // no more tiles than workgroups: a workgroup takes a tile, each of its wavefronts a share of the reduction
        for (int t = blockIdx.x; t < total; t += (int)c.G) {
            int ti, tj;
            const FuGemm g = locate(t, ti, tj);
            v16i acc = fu_tile(g, ti, tj, wave, FU_WAVES, lane);
            if (wave > 0) {
#pragma unroll
                for (int v = 0; v < 16; ++v) red[((wave - 1) * 16 + v) * 64 + lane] = acc[v];
            }
            __syncthreads();
            if (wave == 0) {
#pragma unroll
                for (int w = 0; w < FU_WAVES - 1; ++w)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[v] += red[(w * 16 + v) * 64 + lane];
                fu_tile_store(g, ti, tj, acc, lane);
            }
            __syncthreads();
        }
    } else {
        // a wavefront takes two tiles per trip, so that the fragment loads of both are in flight together
        const int nwaves = (int)c.G * FU_WAVES;
        for (int t = (int)blockIdx.x * FU_WAVES + wave; t < total; t += 2 * nwaves) {
            int ti0, tj0, ti1 = 0, tj1 = 0;
            const FuGemm g0 = locate(t, ti0, tj0);
            const bool two = t + nwaves < total;
            FuGemm g1 = g0;
            if (two) g1 = locate(t + nwaves, ti1, tj1);
            const v16i acc0 = fu_tile(g0, ti0, tj0, 0, 1, lane);
            if (two) {
                const v16i acc1 = fu_tile(g1, ti1, tj1, 0, 1, lane);
                fu_tile_store(g0, ti0, tj0, acc0, lane);
                fu_tile_store(g1, ti1, tj1, acc1, lane);
            } else {
                fu_tile_store(g0, ti0, tj0, acc0, lane);
            }
        }
    }
}

// goodness, dL/dG and the loss term of one sample (Algorithm 1; Eq. (1), Eq. (2)); returns the goodness
__device__ __forceinline__ float fu_goodness(unsigned long long gs, double pow2r, double s_yd, float theta, int sign, float& cf, float& lterm)
{
    double g = (double)gs;
    g = g * pow2r;
    g = g * s_yd;
    g = g * s_yd;
    const float Gv = (float)g;
    const float x = Gv - theta;
    const float e = exp_nonpos(-fabsf(x));
    const float den = 1.0f + e;
    const float sig_big = 1.0f / den, sig_small = e / den;
    float xs;
    if (sign > 0) { cf = -(x >= 0.0f ? sig_small : sig_big); xs = -x; }
    else { cf = (x >= 0.0f ? sig_big : sig_small); xs = x; }
    lterm = fmaxf(xs, 0.0f) + log1pf(expf(-fabsf(xs)));
    return Gv;
}

__device__ __forceinline__ double block_sum_f64(double v, double* s_sum)
{
    for (int d = 32; d > 0; d >>= 1) v += __shfl_xor(v, d);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) s_sum[threadIdx.x >> 6] = v;
    __syncthreads();
    double t = 0.0;
#pragma unroll
    for (int w = 0; w < FU_WAVES; ++w) t += s_sum[w];
    return t;
}
__device__ __forceinline__ uint32_t block_max_u32(uint32_t v, uint32_t* s_max)
{
    v = wave_max_u32(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) s_max[threadIdx.x >> 6] = v;
    __syncthreads();
    uint32_t m = 0;
#pragma unroll
    for (int w = 0; w < FU_WAVES; ++w) m = max(m, s_max[w]);
    return m;
}

// ------------------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(FU_THREADS) void k_fused_dense_step(FusedArgs a)
{
    __shared__ float sG[2 * FU_MAX_B];              // goodness of the current layer, both passes
    __shared__ int red[(FU_WAVES - 1) * 16 * 64];   // split-reduction exchange of the contractions
    __shared__ float sCt[FU_MAX_LAYERS * 2 * FU_MAX_B];   // look-ahead coefficients of every layer, both passes
    __shared__ float s_gamax[FU_MAX_LAYERS * 2];           // absmax of every layer's local gradient, both passes
    __shared__ uint32_t s_bits[FU_MAX_LAYERS * 2 * FU_WAVES];   // per-wavefront maxima awaiting the exchange
    __shared__ uint32_t s_max[FU_WAVES];
    __shared__ double s_sum[FU_WAVES];

    FuCtx c;
    c.bar = a.bar;
    c.stamps = a.stamps;
    c.epoch = 0;
    c.G = gridDim.x;
    c.gtid = (int)blockIdx.x * FU_THREADS + (int)threadIdx.x;
    c.gsz = (int)gridDim.x * FU_THREADS;
    const int k = a.k, B = a.B;
    const int tid = threadIdx.x, lane = tid & 63;
    const uint64_t step = a.step_dev ? a.step_dev[0] : a.step;
    // the two passes of a tensor-wise phase are worked on side by side: the lower half of the launch's workgroups takes
    // the positive set, the upper half the negative one (the grid has an even number of workgroups)
    const int half = c.gsz >> 1, hp = c.gtid >= half ? 1 : 0, htid = c.gtid - hp * half;
    if (c.stamps && c.gtid == 0) c.stamps[0] = wall_clock64();

    // ---- absmax of the net input, both data sets
    {
        const float* x = a.x + hp * a.st_x;
        const int n = B * a.L[0].K;
        uint32_t m = 0;
        if ((n & 3) == 0 && (((uintptr_t)x) & 15) == 0) {
            for (int e = htid; e < (n >> 2); e += half) {
                const v4f f = ((const v4f*)x)[e];
                m = max(max(m, __float_as_uint(f.x) & 0x7FFFFFFFu), max(__float_as_uint(f.y) & 0x7FFFFFFFu,
                        max(__float_as_uint(f.z) & 0x7FFFFFFFu, __float_as_uint(f.w) & 0x7FFFFFFFu)));
            }
        } else {
            for (int e = htid; e < n; e += half) m = max(m, __float_as_uint(x[e]) & 0x7FFFFFFFu);
        }
        m = block_max_u32(m, s_max);   // (a workgroup lies in one half)
        if (tid == 0) a.wg_amax[blockIdx.x] = m;
        // the sums the contractions will add to, and the absmax words of the new weights, start at zero
        for (int e = c.gtid; e < 2 * k * B; e += c.gsz) {
            a.gsum[e] = 0ull;
            a.vmax[e] = 0;
        }
        if (c.gtid < k) a.w_amax[c.gtid] = 0u;
    }
    grid_barrier(c);

    for (int i = 0; i < k; ++i) {
        const FusedLayer& L = a.L[i];
        // ---- quantise the layer input (stochastic rounding; Section IV-B): from the net input, or straight from the
        // previous layer's accumulators.  For the latter every workgroup first forms that layer's goodness values and
        // the absmax of its output itself (at most a thousand samples: cheaper than another device-wide barrier); the
        // workgroup with the index of the pass also stores goodness, loss and dL/dG.
        float amax_in[2];
        if (i == 0) {
            // maximum of the workgroups' partial maxima: the lower half of the grid took the positive set
            uint32_t m0 = 0, m1 = 0;
            for (int j = tid; j < (int)c.G; j += FU_THREADS) {
                const uint32_t v = a.wg_amax[j];
                if (j < (int)(c.G >> 1)) m0 = max(m0, v);
                else m1 = max(m1, v);
            }
            m0 = wave_max_u32(m0);
            m1 = wave_max_u32(m1);
            if (lane == 0) {
                s_bits[tid >> 6] = m0;
                s_bits[FU_WAVES + (tid >> 6)] = m1;
            }
            __syncthreads();
            for (int p = 0; p < 2; ++p) {
                uint32_t m = 0;
#pragma unroll
                for (int w = 0; w < FU_WAVES; ++w) m = max(m, s_bits[p * FU_WAVES + w]);
                amax_in[p] = __uint_as_float(m);
            }
        } else {
            const FusedLayer& Lp = a.L[i - 1];
            const int wv = tid >> 6;
            double lsum = 0.0;   // of the pass this workgroup writes for (workgroups 0 and 1)
            for (int p = 0; p < 2; ++p) {
                const float s_y = ld_f32(a.s_a + 2 * (i - 1) + p) * ld_f32(Lp.sw);
                const double s_yd = (double)s_y, pow2r = (double)(1ull << Lp.rshift);
                const bool writer = (int)blockIdx.x == p;
                uint32_t mb = 0;
                for (int b = tid; b < B; b += FU_THREADS) {
                    const int o = ((i - 1) * 2 + p) * B + b;
                    float cf, lterm;
                    const float Gv = fu_goodness(a.gsum[o], pow2r, s_yd, Lp.theta, p == 0 ? 1 : -1, cf, lterm);
                    sG[p * FU_MAX_B + b] = Gv;
                    float ymax = (float)a.vmax[o] * s_y;
                    if (Lp.l2norm) {
                        const float nrm = sqrtf(Gv);
                        ymax = nrm > 0.0f ? ymax / nrm : 0.0f;
                    }
                    mb = max(mb, __float_as_uint(ymax));
                    if (writer) {
                        a.goodness[o] = Gv;
                        a.c[o] = cf;
                        lsum += (double)lterm;
                    }
                }
                mb = wave_max_u32(mb);
                if (lane == 0) s_bits[p * FU_WAVES + wv] = mb;
            }
            for (int d = 32; d > 0; d >>= 1) lsum += __shfl_xor(lsum, d);
            if (lane == 0) s_sum[wv] = lsum;
            __syncthreads();
            for (int p = 0; p < 2; ++p) {
                uint32_t m = 0;
#pragma unroll
                for (int w = 0; w < FU_WAVES; ++w) m = max(m, s_bits[p * FU_WAVES + w]);
                amax_in[p] = __uint_as_float(m);
            }
            if ((int)blockIdx.x < 2 && tid == 0) {
                double t = 0.0;
#pragma unroll
                for (int w = 0; w < FU_WAVES; ++w) t += s_sum[w];
                a.loss[2 * (i - 1) + (int)blockIdx.x] = (float)(t / (double)B);
            }
            __syncthreads();   // sG is complete
        }
        {
            const int p = hp;
            FuQuant q;
            q.x = a.x + p * a.st_x;
            q.acc = i == 0 ? nullptr : a.L[i - 1].acc + p * a.L[i - 1].st_acc;
            q.ldacc = i == 0 ? 0 : (int)pitch32(a.L[i - 1].N);
            q.s_y = i == 0 ? 1.0f : ld_f32(a.s_a + 2 * (i - 1) + p) * ld_f32(a.L[i - 1].sw);
            q.relu = i == 0 ? 0 : a.L[i - 1].relu;
            q.l2norm = i == 0 ? 0 : a.L[i - 1].l2norm;
            q.rowf_lds = sG + p * FU_MAX_B;
            q.ct = nullptr;
            q.amax = amax_in[p];
            q.k0 = make_sr_key(a.seed, stream_tag_of(step, (uint32_t)i, (uint32_t)p, FF_KIND_ACT)).k0;
            q.rows = B;
            q.cols = L.K;
            q.q = L.aq + p * L.st_aq;
            q.ldq = (int)pitch8(L.K);
            q.q_t = L.aqt + p * L.st_aqt;
            q.ldqt = (int)pitch8(B);
            q.scale = a.s_a + 2 * i + p;
            if (i == 0) fu_quantize<0, true>(q, htid, half);
            else fu_quantize<1, true>(q, htid, half);
        }
        grid_barrier(c);

        // ---- forward contraction with the per-sample goodness sums and maxima (Algorithm 1)
        fu_gemm_phase([&](int p) {
            FuGemm g;
            g.P = L.aq + p * L.st_aq;
            g.Q = L.wq;
            g.C = L.acc + p * L.st_acc;
            g.I = B;
            g.J = L.N;
            g.R = L.K;
            g.ldp = (int)pitch8(L.K);
            g.ldq = (int)pitch8(L.K);
            g.ldc = (int)pitch32(L.N);
            g.gsum = a.gsum + (i * 2 + p) * B;
            g.vmax = a.vmax + (i * 2 + p) * B;
            g.relu = L.relu;
            g.rshift = L.rshift;
            return g;
        }, 2, c, red);
        grid_barrier(c);
    }

    // ---- last layer: goodness, loss, dL/dG; the look-ahead coefficients of every layer (Eq. (3), Eq. (4)); the absmax of
    // every local gradient.  All of it is per sample and there are at most a thousand samples, so every workgroup
    // forms these values itself, in LDS, instead of meeting the others at one more barrier; the workgroup with the
    // index of the pass stores the last layer's goodness, loss and dL/dG.  Then: the int8 local gradient of every
    // trained layer (Section IV-B), transposed for the weight-gradient contraction.
    {
        const int il = k - 1, wv = tid >> 6;
        const FusedLayer& Ll = a.L[il];
        double lsum = 0.0;
        for (int p = 0; p < 2; ++p) {
            const float s_yl = ld_f32(a.s_a + 2 * il + p) * ld_f32(Ll.sw);
            const double s_yd = (double)s_yl, pow2r = (double)(1ull << Ll.rshift);
            const bool writer = (int)blockIdx.x == p;
            for (int b = tid; b < B; b += FU_THREADS) {
                const int o = (il * 2 + p) * B + b;
                float cf, lterm;
                const float Gv = fu_goodness(a.gsum[o], pow2r, s_yd, Ll.theta, p == 0 ? 1 : -1, cf, lterm);
                sG[p * FU_MAX_B + b] = cf;   // (sG now holds dL/dG of the last layer; a thread reads back its own entries only)
                if (writer) {
                    a.goodness[o] = Gv;
                    a.c[o] = cf;
                    lsum += (double)lterm;
                }
            }
        }
        for (int d = 32; d > 0; d >>= 1) lsum += __shfl_xor(lsum, d);
        if (lane == 0) s_sum[wv] = lsum;
        // look-ahead: no exchange inside the loops, so that the loads of all layers are in flight together
        for (int p = 0; p < 2; ++p) {
            float S[FU_MAX_B / FU_THREADS];
#pragma unroll
            for (int u = 0; u < FU_MAX_B / FU_THREADS; ++u) S[u] = 0.0f;
            for (int li = k - 1; li >= 0; --li) {
                const float s_y = ld_f32(a.s_a + 2 * li + p) * ld_f32(a.L[li].sw);
                uint32_t bits = 0;
#pragma unroll
                for (int u = 0; u < FU_MAX_B / FU_THREADS; ++u) {
                    const int b = tid + u * FU_THREADS;
                    if (b < B) {
                        const int o = (li * 2 + p) * B + b;
                        const float cf = li == k - 1 ? sG[p * FU_MAX_B + b] : a.c[o];
                        const float ctv = __builtin_fmaf(a.lambda, S[u], cf);
                        S[u] = S[u] + cf;
                        sCt[(li * 2 + p) * FU_MAX_B + b] = ctv;
                        const float ymax = (float)a.vmax[o] * s_y;
                        bits = max(bits, __float_as_uint(fabsf(2.0f * ctv) * ymax));
                    }
                }
                bits = wave_max_u32(bits);
                if (lane == 0) s_bits[(li * 2 + p) * FU_WAVES + wv] = bits;
            }
        }
        __syncthreads();
        if (tid < 2 * k) {
            uint32_t m = 0;
#pragma unroll
            for (int w = 0; w < FU_WAVES; ++w) m = max(m, s_bits[tid * FU_WAVES + w]);
            s_gamax[tid] = __uint_as_float(m);
        }
        if ((int)blockIdx.x < 2 && tid == 0) {
            double t = 0.0;
#pragma unroll
            for (int w = 0; w < FU_WAVES; ++w) t += s_sum[w];
            a.loss[2 * il + (int)blockIdx.x] = (float)(t / (double)B);
        }
        __syncthreads();   // sCt and s_gamax are complete
    }
    {
        // one index space over the 4 x 4 blocks of all trained layers, so that a thread's blocks of different layers are
        // in flight together
        const int p = hp;
        auto grad_quant = [&](int i) {
            const FusedLayer& L = a.L[i];
            FuQuant q;
            q.x = nullptr;
            q.acc = L.acc + p * L.st_acc;
            q.ldacc = (int)pitch32(L.N);
            q.s_y = ld_f32(a.s_a + 2 * i + p) * ld_f32(L.sw);
            q.relu = L.relu;
            q.l2norm = 0;
            q.rowf_lds = nullptr;
            q.ct = sCt + (i * 2 + p) * FU_MAX_B;
            q.amax = s_gamax[i * 2 + p];
            q.k0 = make_sr_key(a.seed, stream_tag_of(step, (uint32_t)i, (uint32_t)p, FF_KIND_GRAD)).k0;
            q.rows = B;
            q.cols = L.N;
            q.q = nullptr;
            q.ldq = 0;
            q.q_t = L.gy + p * L.st_gy;
            q.ldqt = (int)pitch8(B);
            q.scale = a.s_g + 2 * i + p;
            return q;
        };
        int total = 0;
        for (int i = 0; i < k; ++i) {
            if (!a.L[i].train) continue;
            const FuQuant q = grad_quant(i);
            int ncb;
            if (htid == 0) *q.scale = q.amax >= 0x1p-100f ? q.amax / 127.0f : 1.0f;
            total += fu_quant_blocks(q, ncb);
        }
        for (int e0 = htid; e0 < total; e0 += half) {
            int e = e0, li = 0, ncb = 1;
            for (int i = 0; i < k; ++i) {
                if (!a.L[i].train) continue;
                const FuQuant q = grad_quant(i);
                const int nb = fu_quant_blocks(q, ncb);
                li = i;
                if (e < nb) break;
                e -= nb;
            }
            const FuQuant q = grad_quant(li);
            const float inv = q.amax >= 0x1p-100f ? 127.0f / q.amax : 0.0f;
            const int rb = e / ncb, cb = e - rb * ncb;
            fu_quantize_block<2, true>(q, inv, rb, cb);
        }
    }
    grid_barrier(c);

    // ---- int8 weight gradients of every trained layer and the update of the fp32 master weights (Algorithm 1) in one
    // go: a wavefront contracts the SAME 32 x 32 tile of dW for the positive and the negative pass and applies both to
    // its tile of the weights straight from the accumulators (dW[n][k] = sum_m gy[m][n] a[m][k] is never written out);
    // the absmax of the new weights goes to one atomic per workgroup and layer.
    {
        const float lr_eff = a.lr / (float)(2 * B);
        int total = 0;
        for (int i = 0; i < k; ++i)
            if (a.L[i].train) total += ((a.L[i].N + 31) >> 5) * ((a.L[i].K + 31) >> 5);
        const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        const int nwaves = (int)c.G * FU_WAVES;
        uint32_t m_l[FU_MAX_LAYERS];
#pragma unroll
        for (int i = 0; i < FU_MAX_LAYERS; ++i) m_l[i] = 0;
        for (int t0 = (int)blockIdx.x * FU_WAVES + wave; t0 < total; t0 += nwaves) {
            int li = 0, t = t0;
            for (int i = 0; i < k; ++i) {
                if (!a.L[i].train) continue;
                const int n = ((a.L[i].N + 31) >> 5) * ((a.L[i].K + 31) >> 5);
                li = i;
                if (t < n) break;
                t -= n;
            }
            const FusedLayer& L = a.L[li];
            const int tn = (L.K + 31) >> 5, ti = t / tn, tj = t - ti * tn;
            FuGemm g;
            g.I = L.N;
            g.J = L.K;
            g.R = B;
            g.ldp = (int)pitch8(B);
            g.ldq = (int)pitch8(B);
            g.ldc = 0;
            g.C = nullptr;
            g.gsum = nullptr;
            g.vmax = nullptr;
            g.relu = 0;
            g.rshift = 0;
            const int lr = lane & 31, lh = lane >> 5;
            const int n = ti * 32 + lr;
            const bool vec = (L.K & 3) == 0 && (((uintptr_t)L.w) & 15) == 0;
            // the tile of the weights first: its loads are in flight with the fragments'
            float wv[4][4];
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int kk = tj * 32 + 8 * gq + 4 * lh;
#pragma unroll
                for (int e = 0; e < 4; ++e) wv[gq][e] = 0.0f;
                if (n < L.N && kk < L.K) {
                    const float* pw = L.w + n * L.K + kk;
                    if (vec) {
                        const v4f f = *(const v4f*)pw;
                        wv[gq][0] = f.x; wv[gq][1] = f.y; wv[gq][2] = f.z; wv[gq][3] = f.w;
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) if (kk + e < L.K) wv[gq][e] = pw[e];
                    }
                }
            }
            // both passes' contractions side by side: two reduction steps of each per trip, all eight loads first
            v16i d0, d1;
#pragma unroll
            for (int v = 0; v < 16; ++v) { d0[v] = 0; d1[v] = 0; }
            {
                const int Rpad = (B + 15) & ~15, nks = (Rpad + 31) >> 5;
                const int jq = tj * 32 + lr;
                const bool pin = n < L.N, qin = jq < L.K;
                const int8_t* pp = L.gy + n * g.ldp + 16 * lh;
                const int8_t* pq = L.aqt + jq * g.ldq + 16 * lh;
                const v4i zero = {0, 0, 0, 0};
                for (int ks = 0; ks < nks; ks += 2) {
                    v4i fp0[2], fq0[2], fp1[2], fq1[2];
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        const int k0 = (ks + u) * 32;
                        const bool kin = ks + u < nks && k0 + 16 * lh < Rpad;
                        fp0[u] = (kin && pin) ? *(const v4i*)(pp + k0) : zero;
                        fq0[u] = (kin && qin) ? *(const v4i*)(pq + k0) : zero;
                        fp1[u] = (kin && pin) ? *(const v4i*)(pp + L.st_gy + k0) : zero;
                        fq1[u] = (kin && qin) ? *(const v4i*)(pq + L.st_aqt + k0) : zero;
                    }
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        d0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(fq0[u], fp0[u], d0, 0, 0, 0);
                        d1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(fq1[u], fp1[u], d1, 0, 0, 0);
                    }
                }
            }
            const float sc0 = ld_f32(a.s_g + 2 * li) * ld_f32(a.s_a + 2 * li);
            const float sc1 = ld_f32(a.s_g + 2 * li + 1) * ld_f32(a.s_a + 2 * li + 1);
            uint32_t m = 0;
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int kk = tj * 32 + 8 * gq + 4 * lh;
                if (n < L.N && kk < L.K) {
                    float* pw = L.w + n * L.K + kk;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float gr = (float)d0[4 * gq + e] * sc0;
                        gr = __builtin_fmaf((float)d1[4 * gq + e], sc1, gr);
                        wv[gq][e] = __builtin_fmaf(-lr_eff, gr, wv[gq][e]);
                        if (kk + e < L.K) m = max(m, __float_as_uint(wv[gq][e]) & 0x7FFFFFFFu);
                    }
                    if (vec) {
                        *(v4f*)pw = (v4f){wv[gq][0], wv[gq][1], wv[gq][2], wv[gq][3]};
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) if (kk + e < L.K) pw[e] = wv[gq][e];
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < FU_MAX_LAYERS; ++i) if (i == li) m_l[i] = max(m_l[i], m);
        }
#pragma unroll
        for (int i = 0; i < FU_MAX_LAYERS; ++i) {
            if (i < k && a.L[i].train) {   // (uniform)
                const uint32_t m = block_max_u32(m_l[i], s_max);
                if (tid == 0 && m) atomicMax(a.w_amax + i, m);
            }
        }
    }
    grid_barrier(c);

    // ---- requantise the weights (nearest even)
    for (int i = 0; i < k; ++i) {
        const FusedLayer& L = a.L[i];
        if (!L.train) continue;
        FuQuant q;
        q.x = L.w;
        q.acc = nullptr;
        q.ldacc = 0;
        q.s_y = 1.0f;
        q.relu = 0;
        q.l2norm = 0;
        q.rowf_lds = nullptr;
        q.ct = nullptr;
        q.amax = __uint_as_float(ld_u32(a.w_amax + i));
        q.k0 = 0u;
        q.rows = L.N;
        q.cols = L.K;
        q.q = L.wq;
        q.ldq = (int)pitch8(L.K);
        q.q_t = nullptr;
        q.ldqt = 0;
        q.scale = L.sw;
        fu_quantize<0, false>(q, c.gtid, c.gsz);
    }
    if (c.stamps) {
        __syncthreads();
        if (c.gtid == 0) c.stamps[c.epoch + 1] = wall_clock64();
    }
    if (a.step_dev && a.advance && c.gtid == 0) a.step_dev[0] = step + 1;   // every workgroup read the step at its start
    // the last workgroup to leave puts the counters back to zero for the next launch (nobody waits at a barrier any more)
    if (tid == 0) {
        const unsigned old = __hip_atomic_fetch_add(c.bar + 2, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (old == c.G - 1) {
            __hip_atomic_store(c.bar + 0, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(c.bar + 2, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// Device address of this GPU's copy of the counters: looked up once per device, with that device current.  In host code
// the array's name is only a handle for hipGetSymbolAddress.
static hipError_t fused_sync_ptr(unsigned** out)
{
    constexpr int MAX_DEV = 64;
    static unsigned* ptr[MAX_DEV];
    static std::mutex mtx;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEV) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mtx);
    if (!ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_fu_sync));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        ptr[dev] = (unsigned*)p;
    }
    *out = ptr[dev];
    return hipSuccess;
}

hipError_t launch_fused_dense_step(const FusedArgs& a_in, int workgroups, hipStream_t s)
{
    if (workgroups < 2 || workgroups > 256 || (workgroups & 1) || a_in.k < 1 || a_in.k > FU_MAX_LAYERS || a_in.B < 1 ||
        a_in.B > FU_MAX_B)
        return hipErrorInvalidValue;
    FusedArgs a = a_in;
    const hipError_t e = fused_sync_ptr(&a.bar);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_fused_dense_step, dim3((unsigned)workgroups), dim3(FU_THREADS), 0, s, a);
    return hipGetLastError();
}

}  // namespace ffi
