// libhot: HIP kernels and C ABI of the per-GPU Gaussian sample layer of
// sampling-parallel Bayes-by-Backprop (arxiv 2604.04736, Algorithm 2; Algorithm 1 is
// the one-GPU case).  Written for gfx950 (MI355X) only.
//
// The kernels are streaming work (about 0.2 flop per byte when eps is read from memory),
// so the design follows the HBM roofline, not the matrix cores:
//   * a thread owns 16-byte column chunks; a wave's load instruction covers 1 KiB of
//     one row, contiguous, so every HBM burst is fully used;
//   * mu and sigma are loaded once per column and stay in registers across the sample
//     loop; the rows of several samples are requested together (UNROLL) and a thread
//     owns several chunks (CHUNKS) so that each wave keeps many 16-byte loads in flight;
//   * the KL term leaves one fp64 partial per workgroup; a one-workgroup kernel launched
//     right behind adds them in a fixed order (deterministic, no floating-point atomics,
//     and no fence inside the streaming kernel: a device-scope release there has to
//     write back the die's whole L2, which cost a factor of four with large grids; grids of
//     at most 64 workgroups, where a second launch costs more than that, finish the sum
//     themselves through an arrival counter);
//   * there is no reuse between threads, hence no LDS staging: LDS only carries the
//     four per-wave partial sums of the KL reduction;
//   * when the arrays exceed the 256 MiB memory-side cache EVERY access of a full tile carries the
//     non-temporal hint, mu, sigma and the gradient outputs included: a single stream of ordinary
//     accesses makes the kernel allocate in that cache and pay for evicting whatever dirty lines
//     the kernel before it left there (measured at 200 M weights: the forward kernel took 0.85 ms
//     after an all-hinted kernel, 0.88 ms after the backward kernel and 0.92 ms after an ordinary
//     element-wise kernel; with all accesses hinted 0.83 ms after any of them).
// With GEN the kernels draw eps in registers from a counter-based generator instead of
// reading it (4 bytes per item less in each direction, at the price of integer and
// transcendental arithmetic): forward and backward regenerate identical values.
#include <hip/hip_runtime.h>

#include <new>

#include "hot.h"
#include "vec.h"
#include "draw.h"
#include "adam.h"

namespace {

constexpr int kBlock = 256;             // threads per workgroup = 4 wavefronts of 64
constexpr int kWaves = kBlock / 64;
constexpr int kMaxGrid = 65536;         // upper bound on workgroups (size of the partials buffer)
constexpr int kFinishBlock = 1024;      // threads of the one workgroup that adds the KL partials
constexpr int kTicketGrid = 64;         // up to this many workgroups the forward kernel finishes the KL sum itself

typedef u4 u4u __attribute__((aligned(4)));

// eps[s, col .. col+3]: read from memory, or drawn (col is a multiple of 4).
template <bool ALIGNED, bool NT, bool GEN>
__device__ __forceinline__ f4 eps4(const float *eps, long ld, int s, long col, const Rng &rng)
{
    if constexpr (GEN) return eps_quad(col >> 2, s, rng);
    else return load4<ALIGNED, NT>(eps + (size_t)s * (size_t)ld + col);
}

// eps[s, i] of a single weight (the ragged tail): read at its offset, or drawn with its quad.
template <bool GEN>
__device__ __forceinline__ float eps1(const float *eps, size_t at, long i, int s, const Rng &rng)
{
    if constexpr (GEN) {
        const f4 e = eps_quad(i >> 2, s, rng);
        const int j = (int)(i & 3);
        return j == 0 ? e[0] : (j == 1 ? e[1] : (j == 2 ? e[2] : e[3]));
    } else {
        return eps[at];
    }
}

// One addend of the prior-matching line of Algorithm 2 (without the factor 1/2):
// sigma^2 + mu^2 - 1 - ln sigma^2, with ln sigma^2 taken as 2 ln sigma.  sigma is split exactly
// into mantissa and exponent, ln sigma = (exponent + log2 mantissa) ln 2: only log2 of a number in
// [1/2, 1) goes through the fp32 hardware logarithm (absolute error below 6e-8), the rest is fp64.
// sigma = 0 gives +inf, sigma < 0 gives NaN.
__device__ __forceinline__ double kl_addend(float m, float sd)
{
    const double md = (double)m, sdd = (double)sd;
    const float mant = __builtin_amdgcn_frexp_mantf(sd);
    const int ex = __builtin_amdgcn_frexp_expf(sd);
    const double ln_sd = ((double)ex + (double)__builtin_amdgcn_logf(mant)) * 0.69314718055994530942;
    return fma(sdd, sdd, fma(md, md, -1.0)) - 2.0 * ln_sd;
}

// grad_mu and grad_sigma of one weight, in fp64, from its fp64 sample sums (Algorithm 2, gradient
// and averaging lines; d KL / d mu = mu, d KL / d sigma = sigma - 1/sigma).
__device__ __forceinline__ void finish_grad(double sum_g, double sum_ge, float m, float sd,
                                            double g, double k, double &gm, double &gs)
{
    // k = 0 (a partial call that leaves the KL part to another one) must not turn sigma = 0 into NaN
    const double kl_m = k != 0.0 ? k * (double)m : 0.0;
    const double kl_s = k != 0.0 ? k * ((double)sd - (double)(1.0f / sd)) : 0.0;
    gm = fma(g, sum_g, kl_m);
    gs = fma(g, sum_ge, kl_s);
}

// What the backward kernel does with the finished gradients of a column chunk.
//
// StoreGrad: writes them (or adds them to what the outputs hold) as fp32: Algorithm 2, where the
// all-reduce over GPUs comes next.
struct StoreGrad {
    float *gmu, *gsig;
    int accumulate;
    static constexpr bool kReduces = false;   // no per-workgroup sum behind the tile loop
    template <bool ALIGNED, bool NT>
    __device__ __forceinline__ void quad(long col, f4, f4, const double (&gm)[4], const double (&gs)[4], double &) const
    {
        f4 om = {0.0f, 0.0f, 0.0f, 0.0f}, os = {0.0f, 0.0f, 0.0f, 0.0f};
        if (accumulate) {
            om = load4<ALIGNED, NT>(gmu + col);
            os = load4<ALIGNED, NT>(gsig + col);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            om[j] = (float)(gm[j] + (double)om[j]);
            os[j] = (float)(gs[j] + (double)os[j]);
        }
        store4<ALIGNED, NT>(gmu + col, om);
        store4<ALIGNED, NT>(gsig + col, os);
    }
    __device__ __forceinline__ void one(long i, float, float, double gm, double gs, double &) const
    {
        gmu[i] = (float)(gm + (double)(accumulate ? gmu[i] : 0.0f));
        gsig[i] = (float)(gs + (double)(accumulate ? gsig[i] : 0.0f));
    }
};

// AdamUpdate: Algorithm 1 (one GPU, nothing to all-reduce): the gradients, rounded to fp32 exactly
// as StoreGrad would store them, go straight into the optimizer's update of mu, sigma and their
// moments, and are never written.
struct AdamUpdate {
    float *mu, *sigma, *m_mu, *v_mu, *m_sig, *v_sig;
    AdamConst c;
    static constexpr bool kReduces = false;
    // updates m, sd (and the moments in memory) in place and stores them
    template <bool ALIGNED>
    __device__ __forceinline__ void update4(long col, f4 &m, f4 &sd, const double (&gm)[4], const double (&gs)[4]) const
    {
        f4 a0 = load4<ALIGNED, true>(m_mu + col), b0 = load4<ALIGNED, true>(v_mu + col);
        f4 a1 = load4<ALIGNED, true>(m_sig + col), b1 = load4<ALIGNED, true>(v_sig + col);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float t = m[j], a = a0[j], b = b0[j];
            adam_one(t, a, b, (float)gm[j], c);
            m[j] = t; a0[j] = a; b0[j] = b;
            t = sd[j]; a = a1[j]; b = b1[j];
            adam_one_sigma(t, a, b, (float)gs[j], c);
            sd[j] = t; a1[j] = a; b1[j] = b;
        }
        store4<ALIGNED, true>(mu + col, m);
        store4<ALIGNED, true>(sigma + col, sd);
        store4<ALIGNED, true>(m_mu + col, a0);
        store4<ALIGNED, true>(v_mu + col, b0);
        store4<ALIGNED, true>(m_sig + col, a1);
        store4<ALIGNED, true>(v_sig + col, b1);
    }
    __device__ __forceinline__ void update1(long i, float &m, float &sd, double gm, double gs) const
    {
        float a = m_mu[i], b = v_mu[i];
        adam_one(m, a, b, (float)gm, c);
        mu[i] = m; m_mu[i] = a; v_mu[i] = b;
        a = m_sig[i]; b = v_sig[i];
        adam_one_sigma(sd, a, b, (float)gs, c);
        sigma[i] = sd; m_sig[i] = a; v_sig[i] = b;
    }
    template <bool ALIGNED, bool NT>
    __device__ __forceinline__ void quad(long col, f4 m, f4 sd, const double (&gm)[4], const double (&gs)[4], double &) const
    {
        update4<ALIGNED>(col, m, sd, gm, gs);
    }
    __device__ __forceinline__ void one(long i, float m, float sd, double gm, double gs, double &) const
    {
        update1(i, m, sd, gm, gs);
    }
};

// AdamUpdateSample: Algorithm 1's whole step behind the network's backward pass.  After AdamUpdate's
// update the next step's reparameterisation and prior-matching lines run on the updated mu, sigma
// while they are still in registers: w[s, :] = mu + sigma * eps_s with eps drawn for the NEXT step, and
// the KL addends of the updated parameters go into the workgroup's partial sum (as in the forward kernel).
struct AdamUpdateSample {
    AdamUpdate adam;
    float *w;
    long ld;
    int s_loc;
    Rng next;          // the draw of the next step
    double *partials;  // one KL partial per workgroup, or nullptr when no KL is wanted
    static constexpr bool kReduces = true;
    template <bool ALIGNED, bool NT>
    __device__ __forceinline__ void quad(long col, f4 m, f4 sd, const double (&gm)[4], const double (&gs)[4], double &kl) const
    {
        adam.template update4<ALIGNED>(col, m, sd, gm, gs);
        for (int s = 0; s < s_loc; ++s) {
            const f4 e = eps_quad(col >> 2, s, next);
            f4 r;
#pragma unroll
            for (int j = 0; j < 4; ++j) r[j] = __builtin_fmaf(sd[j], e[j], m[j]);
            store4<ALIGNED, NT>(w + (size_t)s * (size_t)ld + col, r);
        }
        if (partials) {
#pragma unroll
            for (int j = 0; j < 4; ++j) kl += kl_addend(m[j], sd[j]);
        }
    }
    __device__ __forceinline__ void one(long i, float m, float sd, double gm, double gs, double &kl) const
    {
        adam.update1(i, m, sd, gm, gs);
        for (int s = 0; s < s_loc; ++s)
            w[(size_t)s * (size_t)ld + (size_t)i] = __builtin_fmaf(sd, eps1<true>(nullptr, 0, i, s, next), m);
        if (partials) kl += kl_addend(m, sd);
    }
};

// What the forward kernel does to the (mu, sigma) of a chunk before it samples from them.
//
// NoPrologue: nothing (Algorithm 2's reparameterisation line on the parameters as they are).
struct NoPrologue {
    template <bool ALIGNED>
    __device__ __forceinline__ void quad(long, f4 &, f4 &) const {}
    __device__ __forceinline__ void one(long, float &, float &) const {}
};

// AdamPrologue: the update line of the previous step first ("Update mu and sigma using optimizer"),
// on the all-reduced gradients, with hot_adam_step's arithmetic; the updated parameters are stored
// and, still in registers, sampled from, so they are not read a second time.
struct AdamPrologue {
    float *mu, *sigma;
    const float *gmu, *gsig;
    float *m_mu, *v_mu, *m_sig, *v_sig;
    AdamConst c;
    template <bool ALIGNED>
    __device__ __forceinline__ void quad(long col, f4 &m, f4 &sd) const
    {
        const f4 g0 = load4<ALIGNED, true>(gmu + col), g1 = load4<ALIGNED, true>(gsig + col);
        f4 a0 = load4<ALIGNED, true>(m_mu + col), b0 = load4<ALIGNED, true>(v_mu + col);
        f4 a1 = load4<ALIGNED, true>(m_sig + col), b1 = load4<ALIGNED, true>(v_sig + col);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float t = m[j], a = a0[j], b = b0[j];
            adam_one(t, a, b, g0[j], c);
            m[j] = t; a0[j] = a; b0[j] = b;
            t = sd[j]; a = a1[j]; b = b1[j];
            adam_one_sigma(t, a, b, g1[j], c);
            sd[j] = t; a1[j] = a; b1[j] = b;
        }
        store4<ALIGNED, true>(mu + col, m);
        store4<ALIGNED, true>(sigma + col, sd);
        store4<ALIGNED, true>(m_mu + col, a0);
        store4<ALIGNED, true>(v_mu + col, b0);
        store4<ALIGNED, true>(m_sig + col, a1);
        store4<ALIGNED, true>(v_sig + col, b1);
    }
    __device__ __forceinline__ void one(long i, float &m, float &sd) const
    {
        float a = m_mu[i], b = v_mu[i];
        adam_one(m, a, b, gmu[i], c);
        mu[i] = m; m_mu[i] = a; v_mu[i] = b;
        a = m_sig[i]; b = v_sig[i];
        adam_one_sigma(sd, a, b, gsig[i], c);
        sigma[i] = sd; m_sig[i] = a; v_sig[i] = b;
    }
};

// Sum over the workgroup, complete in thread 0.  Fixed tree, hence deterministic.
__device__ __forceinline__ double block_sum(double v, double *lds)
{
    v = wave_sum(v);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __syncthreads();
    if (lane == 0) lds[wave] = v;
    __syncthreads();
    double total = 0.0;
    if (threadIdx.x == 0) {
#pragma unroll
        for (int i = 0; i < kWaves; ++i) total += lds[i];
    }
    return total;
}

// What a forward workgroup does with its threads' KL sums: one fp64 partial per workgroup, left for the
// finish kernel (ticket == nullptr), or, on small grids, added up by the workgroup that arrives last.
__device__ __forceinline__ void kl_leave(double kl, double *partials, unsigned *ticket, double *kl_out)
{
    __shared__ double lds[kWaves];
    const double mine = block_sum(kl, lds);
    if (ticket == nullptr) {
        if (threadIdx.x == 0) partials[blockIdx.x] = mine;
    } else {
        // Small grids (at most kTicketGrid workgroups, where a launch costs more than the kernel):
        // the workgroup that arrives last adds the partials, so no second kernel is needed.  Each
        // workgroup pays one device-scope release and the tickets are drawn one after the other
        // (about 56 ns each), which is why large grids use the finish kernel instead.  Nothing waits
        // on anything: whoever draws the last ticket does the sum, in lane order, hence deterministically.
        __shared__ int last;
        if (threadIdx.x == 0) {
            __hip_atomic_store(&partials[blockIdx.x], mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const unsigned drawn = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
            last = drawn == gridDim.x - 1 ? 1 : 0;
        }
        __syncthreads();
        if (last && threadIdx.x < 64) {
            double v = 0.0;
            if (threadIdx.x < gridDim.x)
                v = __hip_atomic_load(&partials[threadIdx.x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            v = wave_sum(v);
            if (threadIdx.x == 0) {
                *kl_out = 0.5 * v;
                __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch
            }
        }
    }
}

// ---------------------------------------------------------------------------------
// Forward: reparameterisation line  w[s,i] = mu[i] + sigma[i] * eps[s,i]  for every local
// sample, fused with the prior-matching line (mu and sigma are in registers anyway).
// ---------------------------------------------------------------------------------

// Rows s .. s+U-1 of one thread's chunks: all eps values first, then multiply-add and store.
template <int CHUNKS, int U, bool ALIGNED, bool NT, bool GEN>
__device__ __forceinline__ void forward_rows(int s, long col0, long ld, const f4 (&m)[CHUNKS],
                                             const f4 (&sd)[CHUNKS], const float *__restrict__ eps,
                                             float *__restrict__ w, const Rng &rng)
{
    constexpr long kStep = (long)kBlock * 4;
    f4 e[U][CHUNKS];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int c = 0; c < CHUNKS; ++c) e[u][c] = eps4<ALIGNED, NT, GEN>(eps, ld, s + u, col0 + c * kStep, rng);
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int c = 0; c < CHUNKS; ++c) {
            f4 r;
#pragma unroll
            for (int j = 0; j < 4; ++j) r[j] = __builtin_fmaf(sd[c][j], e[u][c][j], m[c][j]);
            store4<ALIGNED, NT>(w + (size_t)(s + u) * (size_t)ld + col0 + c * kStep, r);
        }
}

template <int CHUNKS, int UNROLL, bool ALIGNED, bool NT, bool KL, bool GEN, class PRO>
__global__ void __launch_bounds__(kBlock)
hot_forward_kernel(long n, long ld, int s_loc,
                   const float *mu, const float *sigma,
                   const float *__restrict__ eps, float *__restrict__ w,
                   double *partials, unsigned *ticket, double *__restrict__ kl_out, PRO pro, Rng rng)
{
    constexpr long kTile = (long)kBlock * 4 * CHUNKS;   // columns per tile
    constexpr long kStep = (long)kBlock * 4;            // columns between a thread's chunks
    const long n_tiles = (n + kTile - 1) / kTile;
    double kl = 0.0;

    for (long tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const long col0 = tile * kTile + (long)threadIdx.x * 4;
        if ((tile + 1) * kTile <= n) {
            f4 m[CHUNKS], sd[CHUNKS];
#pragma unroll
            for (int c = 0; c < CHUNKS; ++c) {
                m[c] = load4<ALIGNED, NT>(mu + col0 + c * kStep);
                sd[c] = load4<ALIGNED, NT>(sigma + col0 + c * kStep);
                pro.template quad<ALIGNED>(col0 + c * kStep, m[c], sd[c]);
            }
            int s = 0;
            for (; s + UNROLL <= s_loc; s += UNROLL)
                forward_rows<CHUNKS, UNROLL, ALIGNED, NT, GEN>(s, col0, ld, m, sd, eps, w, rng);
            for (; s < s_loc; ++s) forward_rows<CHUNKS, 1, ALIGNED, NT, GEN>(s, col0, ld, m, sd, eps, w, rng);
            if constexpr (KL) {
#pragma unroll
                for (int c = 0; c < CHUNKS; ++c)
#pragma unroll
                    for (int j = 0; j < 4; ++j) kl += kl_addend(m[c][j], sd[c][j]);
            }
        } else {
            // ragged last tile: whole chunks as vectors, the final 1..3 columns one by one
            for (int c = 0; c < CHUNKS; ++c) {
                const long col = col0 + c * kStep;
                if (col + 4 <= n) {
                    f4 m = load4<ALIGNED, false>(mu + col);
                    f4 sd = load4<ALIGNED, false>(sigma + col);
                    pro.template quad<ALIGNED>(col, m, sd);
                    for (int s = 0; s < s_loc; ++s) {
                        const f4 e = eps4<ALIGNED, false, GEN>(eps, ld, s, col, rng);
                        f4 r;
#pragma unroll
                        for (int j = 0; j < 4; ++j) r[j] = __builtin_fmaf(sd[j], e[j], m[j]);
                        store4<ALIGNED, false>(w + (size_t)s * (size_t)ld + col, r);
                    }
                    if constexpr (KL) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) kl += kl_addend(m[j], sd[j]);
                    }
                } else {
                    for (long i = col; i < n; ++i) {
                        float m = mu[i], sd = sigma[i];
                        pro.one(i, m, sd);
                        for (int s = 0; s < s_loc; ++s) {
                            const size_t at = (size_t)s * (size_t)ld + (size_t)i;
                            w[at] = __builtin_fmaf(sd, eps1<GEN>(eps, at, i, s, rng), m);
                        }
                        if constexpr (KL) kl += kl_addend(m, sd);
                    }
                }
            }
        }
    }

    if constexpr (KL) kl_leave(kl, partials, ticket, kl_out);
}

// ---------------------------------------------------------------------------------
// Forward for rows of w that do not start on 64-byte boundaries (a pitch that is not a multiple of 16
// floats, or such a base address).  The memory system takes a wave's 1 KiB store at full speed only when
// it covers whole 64-byte words; otherwise both ends of every such store are half words, which costs the
// streaming forward kernel 8-19 % and a store-dominated one up to 40 %.  Here the column window of a
// workgroup is therefore moved, row by row, by that row's misalignment a (0..15 floats): thread t stores
// the four columns c0 + 4t - a .. c0 + 4t - a + 3, whose address is 16-byte aligned and, over a wave,
// 64-byte aligned and contiguous.  mu and sigma of the shifted columns come out of LDS, where the
// workgroup stages its tile plus the 16 columns to its left once; eps is read at whatever alignment its
// array has (loads do not mind).  The KL sum is taken over the unshifted tile, thread by thread as in the
// kernel above, so its value does not depend on which kernel ran.  Four chunks per thread, fixed.  Measured
// (16 samples, 6 M and 20 M weights, pitch 16 bytes off the grid): 148 and 511-530 us against 153-161 and
// 556-593 us for the kernel above on the same arrays and 142 and 511 us with an aligned pitch.  The
// drawing variant gains nothing from it (it waits for its arithmetic, not for its stores) and has none.
// ---------------------------------------------------------------------------------
template <bool NT, bool KL>
__global__ void __launch_bounds__(kBlock)
hot_forward_shifted_kernel(long n, long ld, int s_loc, const float *mu, const float *sigma,
                           const float *__restrict__ eps, float *__restrict__ w,
                           double *partials, unsigned *ticket, double *__restrict__ kl_out)
{
    constexpr int CH = 4;
    constexpr int kHalo = 16;                         // columns staged to the left of the tile
    constexpr int kStep = kBlock * 4;                 // columns between a thread's chunks
    constexpr int kTile = kStep * CH;
    // staged column c0 - kHalo + i lives in [i mod 4][i div 4]: a wave's 64 threads, each reading element k of
    // its four shifted columns, then read 64 consecutive words of one of the four arrays (no bank conflicts
    // at any shift, and no shuffling in registers)
    constexpr int kQuads = (kHalo + kTile) / 4;
    __shared__ float lds_mu[4][kQuads], lds_sg[4][kQuads];
    const long n_windows = (n + (kHalo - 1) + kTile - 1) / kTile;    // the windows reach back by up to 15 columns
    const unsigned long w_base = (unsigned long)(reinterpret_cast<uintptr_t>(w) >> 2);
    const int t4 = (int)threadIdx.x * 4;
    double kl = 0.0;

    for (long tile = blockIdx.x; tile < n_windows; tile += gridDim.x) {
        const long c0 = tile * kTile;
        __syncthreads();          // the previous tile's readers are done with the staging buffers
        f4 m[CH], sd[CH];
        if (c0 + kTile <= n) {      // a whole tile (uniform over the workgroup): all eight loads in flight together
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                m[c] = load4<false, NT>(mu + c0 + c * kStep + t4);
                sd[c] = load4<false, NT>(sigma + c0 + c * kStep + t4);
            }
            if constexpr (KL) {
#pragma unroll
                for (int c = 0; c < CH; ++c)
#pragma unroll
                    for (int j = 0; j < 4; ++j) kl += kl_addend(m[c][j], sd[c][j]);
            }
        } else {
            for (int c = 0; c < CH; ++c) {
                const long col = c0 + c * kStep + t4;
                m[c] = f4{0.0f, 0.0f, 0.0f, 0.0f};
                sd[c] = f4{1.0f, 1.0f, 1.0f, 1.0f};
                for (int j = 0; j < 4; ++j)
                    if (col + j < n) {
                        m[c][j] = mu[col + j];
                        sd[c][j] = sigma[col + j];
                        if constexpr (KL) kl += kl_addend(m[c][j], sd[c][j]);
                    }
            }
        }
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int q = (kHalo + c * kStep + t4) >> 2;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                lds_mu[j][q] = m[c][j];
                lds_sg[j][q] = sd[c][j];
            }
        }
        if (threadIdx.x < kHalo) {
            const long col = c0 - kHalo + (long)threadIdx.x;
            const bool ok = col >= 0 && col < n;
            lds_mu[threadIdx.x & 3][threadIdx.x >> 2] = ok ? mu[col] : 0.0f;
            lds_sg[threadIdx.x & 3][threadIdx.x >> 2] = ok ? sigma[col] : 1.0f;
        }
        __syncthreads();

        for (int s = 0; s < s_loc; ++s) {
            const int a = (int)((w_base + (unsigned long)s * (unsigned long)ld) & 15ul);   // this row's misalignment in floats
            float *w_row = w + (size_t)s * (size_t)ld;
            const float *e_row = eps + (size_t)s * (size_t)ld;
            f4 e[CH];
            if (c0 - a >= 0 && c0 + kTile - a <= n) {
                // the whole shifted window lies inside the row (uniform over the workgroup): no guards, the
                // four eps loads in flight together
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    const long cs = c0 + c * kStep + t4 - a;
                    e[c] = load4<false, NT>(e_row + cs);
                }
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    const long cs = c0 + c * kStep + t4 - a;
                    const int at = kHalo + c * kStep + t4 - a;
                    f4 r;
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        r[j] = __builtin_fmaf(lds_sg[(at + j) & 3][(at + j) >> 2], e[c][j], lds_mu[(at + j) & 3][(at + j) >> 2]);
                    store4<true, NT>(w_row + cs, r);
                }
                continue;
            }
            bool full[CH];
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                const long cs = c0 + c * kStep + t4 - a;
                full[c] = cs >= 0 && cs + 4 <= n;
                if (full[c]) {
                    e[c] = load4<false, NT>(e_row + cs);
                }
            }
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                const long cs = c0 + c * kStep + t4 - a;
                const int at = kHalo + c * kStep + t4 - a;          // 1 .. kHalo + kTile - 4
                if (full[c]) {
                    f4 r;
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        r[j] = __builtin_fmaf(lds_sg[(at + j) & 3][(at + j) >> 2], e[c][j], lds_mu[(at + j) & 3][(at + j) >> 2]);
                    store4<true, NT>(w_row + cs, r);
                } else {
                    // the two ends of a row: the columns of this quad that exist, one by one
                    for (int j = 0; j < 4; ++j) {
                        const long col = cs + j;
                        if (col >= 0 && col < n) {
                            w_row[col] = __builtin_fmaf(lds_sg[(at + j) & 3][(at + j) >> 2], e_row[col], lds_mu[(at + j) & 3][(at + j) >> 2]);
                        }
                    }
                }
            }
        }
    }
    if constexpr (KL) kl_leave(kl, partials, ticket, kl_out);
}

// Adds the per-workgroup KL partials in a fixed order and applies the factor 1/2 of the
// prior-matching line.  One workgroup; runs right after the forward kernel on its stream.
__global__ void __launch_bounds__(kFinishBlock)
hot_kl_finish_kernel(const double *__restrict__ partials, int count, double *__restrict__ kl_out)
{
    __shared__ double lds[kFinishBlock / 64];
    // Thread t owns the pairs t, t + 1024, t + 2048, ...; eight 16-byte loads are in flight per round
    // and the values are added in index order.  The buffer holds an even number of slots.
    typedef double d2 __attribute__((ext_vector_type(2)));
    const d2 *pairs = reinterpret_cast<const d2 *>(partials);
    const int n_pairs = (count + 1) / 2;
    double acc = 0.0;
    for (int j0 = threadIdx.x; j0 < n_pairs; j0 += kFinishBlock * 8) {
        d2 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int j = j0 + u * kFinishBlock;
            v[u] = j < n_pairs ? pairs[j] : d2{0.0, 0.0};
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int j = j0 + u * kFinishBlock;
            acc += v[u][0];
            if (2 * j + 1 < count) acc += v[u][1];
        }
    }
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double total = 0.0;
#pragma unroll
        for (int i = 0; i < kFinishBlock / 64; ++i) total += lds[i];
        *kl_out = 0.5 * total;
    }
}

// ---------------------------------------------------------------------------------
// Backward: column sums over the local samples of grad_w and grad_w * eps, then the
// KL gradient and the scaling (Algorithm 2, loss / gradient / averaging lines).
// ---------------------------------------------------------------------------------
template <int CHUNKS, int U, bool ALIGNED, bool NT, bool GEN>
__device__ __forceinline__ void backward_rows(int s, long col0, long ld, double (&sum_g)[CHUNKS][4],
                                              double (&sum_ge)[CHUNKS][4], const float *__restrict__ eps,
                                              const float *__restrict__ gw, const Rng &rng)
{
    constexpr long kStep = (long)kBlock * 4;
    f4 gv[U][CHUNKS], ev[U][CHUNKS];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int c = 0; c < CHUNKS; ++c) {
            gv[u][c] = load4<ALIGNED, NT>(gw + (size_t)(s + u) * (size_t)ld + col0 + c * kStep);
            ev[u][c] = eps4<ALIGNED, NT, GEN>(eps, ld, s + u, col0 + c * kStep, rng);
        }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int c = 0; c < CHUNKS; ++c)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const double gd = (double)gv[u][c][j];
                sum_g[c][j] += gd;
                sum_ge[c][j] = fma(gd, (double)ev[u][c][j], sum_ge[c][j]);
            }
}

template <int CHUNKS, int UNROLL, bool ALIGNED, bool NT, bool GEN, class EPI>
__global__ void __launch_bounds__(kBlock)
hot_backward_kernel(long n, long ld, int s_loc, double g, double k,
                    const float *mu, const float *sigma,
                    const float *__restrict__ eps, const float *__restrict__ gw, EPI epi, Rng rng)
{
    constexpr long kTile = (long)kBlock * 4 * CHUNKS;
    constexpr long kStep = (long)kBlock * 4;
    const long n_tiles = (n + kTile - 1) / kTile;
    double acc = 0.0;   // what a reducing epilogue sums per thread (the KL addends of AdamUpdateSample)

    for (long tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const long col0 = tile * kTile + (long)threadIdx.x * 4;
        if ((tile + 1) * kTile <= n) {
            f4 m[CHUNKS], sd[CHUNKS];
#pragma unroll
            for (int c = 0; c < CHUNKS; ++c) {
                m[c] = load4<ALIGNED, NT>(mu + col0 + c * kStep);
                sd[c] = load4<ALIGNED, NT>(sigma + col0 + c * kStep);
            }
            double sum_g[CHUNKS][4], sum_ge[CHUNKS][4];
#pragma unroll
            for (int c = 0; c < CHUNKS; ++c)
#pragma unroll
                for (int j = 0; j < 4; ++j) sum_g[c][j] = sum_ge[c][j] = 0.0;
            int s = 0;
            for (; s + UNROLL <= s_loc; s += UNROLL)
                backward_rows<CHUNKS, UNROLL, ALIGNED, NT, GEN>(s, col0, ld, sum_g, sum_ge, eps, gw, rng);
            for (; s < s_loc; ++s)
                backward_rows<CHUNKS, 1, ALIGNED, NT, GEN>(s, col0, ld, sum_g, sum_ge, eps, gw, rng);
#pragma unroll
            for (int c = 0; c < CHUNKS; ++c) {
                double gm[4], gs[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) finish_grad(sum_g[c][j], sum_ge[c][j], m[c][j], sd[c][j], g, k, gm[j], gs[j]);
                epi.template quad<ALIGNED, NT>(col0 + c * kStep, m[c], sd[c], gm, gs, acc);
            }
        } else {
            for (int c = 0; c < CHUNKS; ++c) {
                const long col = col0 + c * kStep;
                if (col + 4 <= n) {
                    const f4 m = load4<ALIGNED, false>(mu + col);
                    const f4 sd = load4<ALIGNED, false>(sigma + col);
                    double sum_g[4] = {0.0, 0.0, 0.0, 0.0}, sum_ge[4] = {0.0, 0.0, 0.0, 0.0};
                    for (int s = 0; s < s_loc; ++s) {
                        const f4 gv = load4<ALIGNED, false>(gw + (size_t)s * (size_t)ld + col);
                        const f4 ev = eps4<ALIGNED, false, GEN>(eps, ld, s, col, rng);
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const double gd = (double)gv[j];
                            sum_g[j] += gd;
                            sum_ge[j] = fma(gd, (double)ev[j], sum_ge[j]);
                        }
                    }
                    double gm[4], gs[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) finish_grad(sum_g[j], sum_ge[j], m[j], sd[j], g, k, gm[j], gs[j]);
                    epi.template quad<ALIGNED, false>(col, m, sd, gm, gs, acc);
                } else {
                    for (long i = col; i < n; ++i) {
                        double sum_g = 0.0, sum_ge = 0.0;
                        for (int s = 0; s < s_loc; ++s) {
                            const size_t at = (size_t)s * (size_t)ld + (size_t)i;
                            const double gd = (double)gw[at];
                            sum_g += gd;
                            sum_ge = fma(gd, (double)eps1<GEN>(eps, at, i, s, rng), sum_ge);
                        }
                        const float m = mu[i], sd = sigma[i];
                        double gm, gs;
                        finish_grad(sum_g, sum_ge, m, sd, g, k, gm, gs);
                        epi.one(i, m, sd, gm, gs, acc);
                    }
                }
            }
        }
    }
    if constexpr (EPI::kReduces) {
        if (epi.partials) {      // uniform over the grid
            __shared__ double lds[kWaves];
            const double mine = block_sum(acc, lds);
            if (threadIdx.x == 0) epi.partials[blockIdx.x] = mine;
        }
    }
}

// ---------------------------------------------------------------------------------
// The draw on its own: eps[s, i] as floats (BITS = false) or the raw generator words
// (BITS = true).  One thread per quad, all local samples.
// ---------------------------------------------------------------------------------
template <bool BITS, bool ALIGNED>
__global__ void __launch_bounds__(kBlock)
hot_sample_kernel(long n, long ld, int s_loc, void *__restrict__ out, Rng rng)
{
    const long n_quads = (n + 3) / 4;
    for (long quad = (long)blockIdx.x * kBlock + threadIdx.x; quad < n_quads; quad += (long)gridDim.x * kBlock) {
        const long col = quad * 4;
        for (int s = 0; s < s_loc; ++s) {
            const u4 x = eps_words(quad, s, rng);
            const size_t at = (size_t)s * (size_t)ld + (size_t)col;
            if constexpr (BITS) {
                unsigned *o = static_cast<unsigned *>(out) + at;
                if (col + 4 <= n) {
                    if constexpr (ALIGNED) *reinterpret_cast<u4 *>(o) = x;
                    else *reinterpret_cast<u4u *>(o) = x;
                } else {
                    for (long i = col; i < n; ++i) o[i - col] = x[(int)(i - col)];
                }
            } else {
                const f4 e = eps_from_words(x);
                float *o = static_cast<float *>(out) + at;
                if (col + 4 <= n) store4<ALIGNED, false>(o, e);
                else
                    for (long i = col; i < n; ++i) o[i - col] = e[(int)(i - col)];
            }
        }
    }
}

// ---------------------------------------------------------------------------------
// Measurement aid: a plain copy with the same 16-byte accesses, four per thread.  Its known
// traffic calibrates the HBM byte counters and gives the copy ceiling of the machine.
// ---------------------------------------------------------------------------------
template <bool NT>
__global__ void __launch_bounds__(kBlock)
hot_probe_copy_kernel(const f4 *__restrict__ src, f4 *__restrict__ dst, long n_vec)
{
    constexpr int kPer = 4;
    const long base = (long)blockIdx.x * (kBlock * kPer) + threadIdx.x;
    f4 v[kPer];
#pragma unroll
    for (int c = 0; c < kPer; ++c) {
        const long at = base + (long)c * kBlock;
        if (at < n_vec) v[c] = NT ? __builtin_nontemporal_load(src + at) : src[at];
    }
#pragma unroll
    for (int c = 0; c < kPer; ++c) {
        const long at = base + (long)c * kBlock;
        if (at < n_vec) {
            if (NT) __builtin_nontemporal_store(v[c], dst + at);
            else dst[at] = v[c];
        }
    }
}

// Second measurement aid: READS read streams and WRITES write streams of equal length, one
// 16 KiB tile of each per workgroup, no arithmetic beyond adding the inputs.  It gives the
// machine's ceiling for a given mix of read and write traffic (mixed traffic runs well below
// the read-only rate on this memory system), which is what the kernels above can be held to.
struct ProbeStreams {
    const f4 *src[6];
    f4 *dst[2];
};

template <int READS, int WRITES>
__global__ void __launch_bounds__(kBlock)
hot_probe_streams_kernel(ProbeStreams p, long n_vec)
{
    constexpr int kPer = 4;
    const long base = (long)blockIdx.x * (kBlock * kPer) + threadIdx.x;
    f4 v[READS][kPer];
#pragma unroll
    for (int r = 0; r < READS; ++r)
#pragma unroll
        for (int c = 0; c < kPer; ++c) {
            const long at = base + (long)c * kBlock;
            v[r][c] = at < n_vec ? __builtin_nontemporal_load(p.src[r] + at) : f4{0.0f, 0.0f, 0.0f, 0.0f};
        }
    f4 acc[kPer];
#pragma unroll
    for (int c = 0; c < kPer; ++c) {
        acc[c] = v[0][c];
#pragma unroll
        for (int r = 1; r < READS; ++r) acc[c] += v[r][c];
    }
    if constexpr (WRITES == 0) {
        // read-only: the store never happens for ordinary data but keeps the loads alive
        float s = 0.0f;
#pragma unroll
        for (int c = 0; c < kPer; ++c) s += acc[c][0] + acc[c][1] + acc[c][2] + acc[c][3];
        if (s == -1.2345678e-30f && base == 0) p.dst[0][0] = acc[0];
    } else {
#pragma unroll
        for (int w = 0; w < WRITES; ++w)
#pragma unroll
            for (int c = 0; c < kPer; ++c) {
                const long at = base + (long)c * kBlock;
                if (at < n_vec) __builtin_nontemporal_store(acc[c], p.dst[w] + at);
            }
    }
}

template <int READS>
void probe_streams_go(int writes, dim3 grid, hipStream_t s, const ProbeStreams &p, long n_vec)
{
    if (writes == 0) hot_probe_streams_kernel<READS, 0><<<grid, dim3(kBlock), 0, s>>>(p, n_vec);
    else if (writes == 1) hot_probe_streams_kernel<READS, 1><<<grid, dim3(kBlock), 0, s>>>(p, n_vec);
    else hot_probe_streams_kernel<READS, 2><<<grid, dim3(kBlock), 0, s>>>(p, n_vec);
}

// ---------------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------------

struct FwdArgs {
    long n, ld;
    int s_loc;
    const float *mu, *sigma, *eps;
    float *w;
    double *partials;
    unsigned *ticket;
    double *kl_out;
    bool want_kl;
    const AdamPrologue *adam;   // not NULL: update (mu, sigma) first
    Rng rng;
    dim3 grid;
    hipStream_t stream;
};

// Template dispatch over (chunks, unroll, aligned, non-temporal, [KL]); GEN is fixed by the caller.
// The updating variant always carries the KL reduction (its partials are simply not finished when
// the caller wants no KL).
template <bool GEN, int CH, int U, bool AL, bool NT>
void fwd_go(const FwdArgs &a)
{
    if (a.adam)
        hot_forward_kernel<CH, U, AL, NT, true, GEN, AdamPrologue><<<a.grid, dim3(kBlock), 0, a.stream>>>(
            a.n, a.ld, a.s_loc, a.mu, a.sigma, a.eps, a.w, a.partials, a.ticket, a.kl_out, *a.adam, a.rng);
    else if (a.want_kl)
        hot_forward_kernel<CH, U, AL, NT, true, GEN, NoPrologue><<<a.grid, dim3(kBlock), 0, a.stream>>>(
            a.n, a.ld, a.s_loc, a.mu, a.sigma, a.eps, a.w, a.partials, a.ticket, a.kl_out, NoPrologue{}, a.rng);
    else
        hot_forward_kernel<CH, U, AL, NT, false, GEN, NoPrologue><<<a.grid, dim3(kBlock), 0, a.stream>>>(
            a.n, a.ld, a.s_loc, a.mu, a.sigma, a.eps, a.w, a.partials, a.ticket, a.kl_out, NoPrologue{}, a.rng);
}
template <bool GEN, int CH, int U>
void fwd_flags(bool al, bool nt, const FwdArgs &a)
{
    if (al) {
        if (nt) fwd_go<GEN, CH, U, true, true>(a);
        else fwd_go<GEN, CH, U, true, false>(a);
    } else {
        if (nt) fwd_go<GEN, CH, U, false, true>(a);
        else fwd_go<GEN, CH, U, false, false>(a);
    }
}
template <bool GEN, int CH>
void fwd_unroll(int u, bool al, bool nt, const FwdArgs &a)
{
    if (u >= 4) fwd_flags<GEN, CH, 4>(al, nt, a);
    else if (u >= 2) fwd_flags<GEN, CH, 2>(al, nt, a);
    else fwd_flags<GEN, CH, 1>(al, nt, a);
}
template <bool GEN>
void fwd_dispatch(int ch, int u, bool al, bool nt, const FwdArgs &a)
{
    if (ch >= 4) fwd_unroll<GEN, 4>(u, al, nt, a);
    else if (ch >= 2) fwd_unroll<GEN, 2>(u, al, nt, a);
    else fwd_unroll<GEN, 1>(u, al, nt, a);
}

template <class EPI>
struct BwdArgs {
    long n, ld;
    int s_loc;
    double g, k;
    const float *mu, *sigma, *eps, *gw;
    EPI epi;
    Rng rng;
    dim3 grid;
    hipStream_t stream;
};

template <bool GEN, int CH, int U, bool AL, bool NT, class EPI>
void bwd_go(const BwdArgs<EPI> &a)
{
    hot_backward_kernel<CH, U, AL, NT, GEN, EPI><<<a.grid, dim3(kBlock), 0, a.stream>>>(
        a.n, a.ld, a.s_loc, a.g, a.k, a.mu, a.sigma, a.eps, a.gw, a.epi, a.rng);
}
template <bool GEN, int CH, int U, class EPI>
void bwd_flags(bool al, bool nt, const BwdArgs<EPI> &a)
{
    if (al) {
        if (nt) bwd_go<GEN, CH, U, true, true>(a);
        else bwd_go<GEN, CH, U, true, false>(a);
    } else {
        if (nt) bwd_go<GEN, CH, U, false, true>(a);
        else bwd_go<GEN, CH, U, false, false>(a);
    }
}
template <bool GEN, int CH, class EPI>
void bwd_unroll(int u, bool al, bool nt, const BwdArgs<EPI> &a)
{
    if (u >= 4) bwd_flags<GEN, CH, 4>(al, nt, a);
    else if (u >= 2) bwd_flags<GEN, CH, 2>(al, nt, a);
    else bwd_flags<GEN, CH, 1>(al, nt, a);
}
template <bool GEN, class EPI>
void bwd_dispatch(int ch, int u, bool al, bool nt, const BwdArgs<EPI> &a)
{
    if (ch >= 4) bwd_unroll<GEN, 4>(u, al, nt, a);
    else if (ch >= 2) bwd_unroll<GEN, 2>(u, al, nt, a);
    else bwd_unroll<GEN, 1>(u, al, nt, a);
}

// Makes desc.device current for the lifetime of the object.
struct DeviceGuard {
    int prev = -1;
    bool switched = false;
    hipError_t err = hipSuccess;
    explicit DeviceGuard(int device)
    {
        err = hipGetDevice(&prev);
        if (err == hipSuccess && prev != device) {
            err = hipSetDevice(device);
            switched = (err == hipSuccess);
        }
    }
    ~DeviceGuard()
    {
        if (switched) (void)hipSetDevice(prev);
    }
};

}  // namespace

namespace hot_detail {
static thread_local int g_last_hip = 0;
int note_hip(hipError_t e)
{
    if (e == hipSuccess) return HOT_OK;
    g_last_hip = (int)e;
    return HOT_EHIP;
}
}  // namespace hot_detail

struct hot_plan {
    hot_desc d;
    double g, k;
    double *partials;   // kMaxGrid fp64 KL partial sums, one per forward workgroup, then the arrival counter
    hot_launch cfg[4];  // indexed by HOT_KERNEL_*
    int last_hip;
};

namespace {

int fail_hip(hot_plan *p, hipError_t e)
{
    if (p) p->last_hip = (int)e;
    return HOT_EHIP;
}

int pick_unroll(int want, int s_loc)
{
    int u = want >= 4 ? 4 : (want >= 2 ? 2 : 1);
    while (u > 1 && u > s_loc) u >>= 1;
    return u;
}

bool valid_kernel(int kernel) { return kernel >= HOT_KERNEL_FORWARD && kernel <= HOT_KERNEL_BACKWARD_RNG; }

bool valid_launch(const hot_launch &c)
{
    auto one_of = [](int v) { return v == 0 || v == 1 || v == 2 || v == 4; };
    return c.grid_blocks >= 0 && c.grid_blocks <= kMaxGrid && one_of(c.chunks) && one_of(c.unroll) &&
           (c.nontemporal == 0 || c.nontemporal == 1);
}

// Number of workgroups: one per column tile, capped by the configured bound.
unsigned grid_for(long n, const hot_launch &c)
{
    const long tile = (long)kBlock * 4 * c.chunks;
    const long tiles = (n + tile - 1) / tile;
    return (unsigned)(tiles < c.grid_blocks ? tiles : c.grid_blocks);
}

// kl_only: the prior-matching term alone.  The forward kernel runs over zero samples, so it touches
// neither eps nor w (both may be NULL) and only its KL part is left.
int forward_impl(hot_plan *plan, int kernel, const Rng *rng, const float *mu, const float *sigma,
                 const float *eps, float *w, double *kl_out, void *stream, bool kl_only = false,
                 const AdamPrologue *adam = nullptr, bool adam_aligned = true)
{
    const bool gen = rng != nullptr || kl_only;      // kl_only: no eps array to look at
    if (!mu || !sigma || (!kl_only && !w) || (!gen && !eps) || (kl_only && !kl_out)) return HOT_EINVAL;
    if (!aligned4(mu) || !aligned4(sigma) || (!kl_only && !aligned4(w)) || (!gen && !aligned4(eps))) return HOT_EINVAL;
    if (kl_out && (reinterpret_cast<uintptr_t>(kl_out) & 7u)) return HOT_EINVAL;
    const hot_desc &d = plan->d;
    const hot_launch &c = plan->cfg[kernel];
    const bool al = aligned16(mu) && aligned16(sigma) && (kl_only || aligned16(w)) && (gen || aligned16(eps)) &&
                    (kl_only || d.ld % 4 == 0) && adam_aligned;

    FwdArgs a;
    a.n = d.n_weights;
    a.ld = d.ld;
    a.s_loc = kl_only ? 0 : d.s_local;
    a.mu = mu;
    a.sigma = sigma;
    a.eps = eps;
    a.w = w;
    a.partials = plan->partials;
    a.want_kl = kl_out != nullptr;
    a.kl_out = kl_out;
    a.adam = adam;
    a.rng = rng ? *rng : Rng{0, 0, 0, 0};
    a.grid = dim3(grid_for(d.n_weights, c));
    a.stream = static_cast<hipStream_t>(stream);

    // Rows of w off the 64-byte grid, streamed with non-temporal stores, eps from its array: the kernel that
    // moves its column window row by row (fixed shape: four chunks).
    const bool rows_on_grid = (reinterpret_cast<uintptr_t>(w) & 63u) == 0 && (d.s_local == 1 || d.ld % 16 == 0);
    const bool shifted = !kl_only && !adam && !gen && c.nontemporal != 0 && !rows_on_grid;
    if (shifted) {
        const long windows = (d.n_weights + 15 + 4095) / 4096;
        a.grid = dim3((unsigned)(windows < c.grid_blocks ? windows : c.grid_blocks));
    }
    const bool self_finish = a.want_kl && a.grid.x <= (unsigned)kTicketGrid;
    a.ticket = self_finish ? reinterpret_cast<unsigned *>(plan->partials + kMaxGrid) : nullptr;

    DeviceGuard guard(d.device);
    if (guard.err != hipSuccess) return fail_hip(plan, guard.err);
    if (shifted) {
        const dim3 block(kBlock);
        if (a.want_kl) hot_forward_shifted_kernel<true, true><<<a.grid, block, 0, a.stream>>>(a.n, a.ld, a.s_loc, a.mu, a.sigma, a.eps, a.w, a.partials, a.ticket, a.kl_out);
        else hot_forward_shifted_kernel<true, false><<<a.grid, block, 0, a.stream>>>(a.n, a.ld, a.s_loc, a.mu, a.sigma, a.eps, a.w, a.partials, a.ticket, a.kl_out);
    } else if (gen) fwd_dispatch<true>(c.chunks, c.unroll, al, c.nontemporal != 0, a);
    else fwd_dispatch<false>(c.chunks, c.unroll, al, c.nontemporal != 0, a);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && kl_out && !self_finish) {
        hot_kl_finish_kernel<<<dim3(1), dim3(kFinishBlock), 0, a.stream>>>(plan->partials, (int)a.grid.x, kl_out);
        e = hipGetLastError();
    }
    return e == hipSuccess ? HOT_OK : fail_hip(plan, e);
}

// Launches the backward kernel with the given epilogue.  rows samples starting at local sample
// first_row (eps and grad_w point at the first of them); rows = 0 means all of the plan's samples.
// aligned_out: whether every array the epilogue touches is 16-byte aligned.
template <class EPI>
int backward_launch(hot_plan *plan, int kernel, const Rng *rng, const float *mu, const float *sigma,
                    const float *eps, const float *grad_w, const EPI &epi, bool aligned_out, void *stream,
                    int first_row, int rows, bool add_kl)
{
    const bool gen = rng != nullptr;
    const hot_desc &d = plan->d;
    const hot_launch &c = plan->cfg[kernel];
    const bool al = aligned16(mu) && aligned16(sigma) && aligned16(grad_w) && aligned_out &&
                    (gen || aligned16(eps)) && (d.ld % 4 == 0);

    BwdArgs<EPI> a;
    a.n = d.n_weights;
    a.ld = d.ld;
    a.s_loc = rows > 0 ? rows : d.s_local;
    a.g = plan->g;
    a.k = add_kl ? plan->k : 0.0;
    a.mu = mu;
    a.sigma = sigma;
    a.eps = eps;
    a.gw = grad_w;
    a.epi = epi;
    a.rng = gen ? *rng : Rng{0, 0, 0, 0};
    a.rng.first_sample += (unsigned)first_row;
    a.grid = dim3(grid_for(d.n_weights, c));
    a.stream = static_cast<hipStream_t>(stream);

    DeviceGuard guard(d.device);
    if (guard.err != hipSuccess) return fail_hip(plan, guard.err);
    if (gen) bwd_dispatch<true>(c.chunks, pick_unroll(c.unroll, a.s_loc), al, c.nontemporal != 0, a);
    else bwd_dispatch<false>(c.chunks, pick_unroll(c.unroll, a.s_loc), al, c.nontemporal != 0, a);
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? HOT_OK : fail_hip(plan, e);
}

int backward_impl(hot_plan *plan, int kernel, const Rng *rng, const float *mu, const float *sigma,
                  const float *eps, const float *grad_w, float *grad_mu, float *grad_sigma, void *stream,
                  int first_row = 0, int rows = 0, bool accumulate = false, bool add_kl = true)
{
    const bool gen = rng != nullptr;
    if (!mu || !sigma || !grad_w || !grad_mu || !grad_sigma || (!gen && !eps)) return HOT_EINVAL;
    if (!aligned4(mu) || !aligned4(sigma) || !aligned4(grad_w) || !aligned4(grad_mu) || !aligned4(grad_sigma) ||
        (!gen && !aligned4(eps)))
        return HOT_EINVAL;
    const StoreGrad epi{grad_mu, grad_sigma, accumulate ? 1 : 0};
    return backward_launch(plan, kernel, rng, mu, sigma, eps, grad_w, epi, aligned16(grad_mu) && aligned16(grad_sigma),
                           stream, first_row, rows, add_kl);
}

int sample_impl(hot_plan *plan, const hot_rng *rng, void *out, bool bits, void *stream)
{
    Rng r;
    if (!plan || !out || !aligned4(out) || !make_rng(rng, plan->d.s_local, r)) return HOT_EINVAL;
    const hot_desc &d = plan->d;
    const bool al = aligned16(out) && (d.ld % 4 == 0);
    const long quads = (d.n_weights + 3) / 4;
    long blocks = (quads + kBlock - 1) / kBlock;
    if (blocks > kMaxGrid) blocks = kMaxGrid;
    const dim3 grid((unsigned)blocks), block(kBlock);
    hipStream_t s = static_cast<hipStream_t>(stream);

    DeviceGuard guard(d.device);
    if (guard.err != hipSuccess) return fail_hip(plan, guard.err);
    if (bits) {
        if (al) hot_sample_kernel<true, true><<<grid, block, 0, s>>>(d.n_weights, d.ld, d.s_local, out, r);
        else hot_sample_kernel<true, false><<<grid, block, 0, s>>>(d.n_weights, d.ld, d.s_local, out, r);
    } else {
        if (al) hot_sample_kernel<false, true><<<grid, block, 0, s>>>(d.n_weights, d.ld, d.s_local, out, r);
        else hot_sample_kernel<false, false><<<grid, block, 0, s>>>(d.n_weights, d.ld, d.s_local, out, r);
    }
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? HOT_OK : fail_hip(plan, e);
}

}  // namespace

extern "C" {

int hot_version(void) { return HOT_VERSION; }

const char *hot_strerror(int code)
{
    switch (code) {
    case HOT_OK: return "success";
    case HOT_EINVAL: return "invalid argument";
    case HOT_ENOMEM: return "out of memory";
    case HOT_EHIP: return "HIP runtime error (see hot_last_hip_error)";
    default: return "unknown error code";
    }
}

int64_t hot_recommended_ld(int64_t n_weights)
{
    if (n_weights < 1) return HOT_EINVAL;
    return (n_weights + 63) / 64 * 64;
}

int hot_create(hot_plan **out, const hot_desc *desc)
{
    if (!out || !desc) return HOT_EINVAL;
    const hot_desc &d = *desc;
    if (d.n_weights < 1 || d.ld < d.n_weights || d.s_local < 1 || d.s_total < d.s_local) return HOT_EINVAL;
    if (!(d.dataset_size > 0.0) || !(d.dataset_size < 1.0 / 0.0)) return HOT_EINVAL;
    if (d.flags != HOT_REDUCE_SUM && d.flags != HOT_REDUCE_MEAN && d.flags != HOT_REDUCE_NONE) return HOT_EINVAL;
    // element offsets (s_local - 1) * ld + n_weights must fit in 63 bits
    if (d.ld > (INT64_MAX / 4) / d.s_local) return HOT_EINVAL;
    int n_dev = 0;
    if (hipError_t e = hipGetDeviceCount(&n_dev); e != hipSuccess) return hot_detail::note_hip(e);
    if (d.device < 0 || d.device >= n_dev) return HOT_EINVAL;

    hot_plan *p = new (std::nothrow) hot_plan();
    if (!p) return HOT_ENOMEM;
    p->d = d;
    if (d.flags == HOT_REDUCE_NONE) {
        p->g = 1.0;
        p->k = 1.0 / d.dataset_size;
    } else if (d.flags == HOT_REDUCE_MEAN) {
        p->g = 1.0 / (double)d.s_local;
        p->k = 1.0 / d.dataset_size;
    } else {
        p->g = 1.0 / (double)d.s_total;
        p->k = (double)d.s_local / ((double)d.s_total * d.dataset_size);
    }
    p->partials = nullptr;
    p->last_hip = 0;

    DeviceGuard guard(d.device);
    hipError_t e = guard.err;
    // one slot past the partials holds the arrival counter of the self-finishing small-grid forward kernel
    if (e == hipSuccess) e = hipMalloc((void **)&p->partials, sizeof(double) * (kMaxGrid + 1));
    if (e == hipSuccess) e = hipMemset(p->partials + kMaxGrid, 0, sizeof(double));
    if (e == hipSuccess) e = hipStreamSynchronize(nullptr);   // the counter is zero before any stream uses the plan
    if (e != hipSuccess) {
        const bool oom = (e == hipErrorOutOfMemory);
        if (p->partials) (void)hipFree(p->partials);
        (void)hipGetLastError();
        delete p;
        return oom ? HOT_ENOMEM : hot_detail::note_hip(e);
    }
    // Defaults from launch-shape sweeps on MI355X, each kernel timed with the other one running in
    // between (timing a kernel back to back with itself lets part of its input stay in the 256 MiB
    // memory-side cache and favours shapes that lose in a real step): four chunks per thread for
    // the array kernels, single rows in flight forward, as many rows as there are (up to four)
    // backward.  Non-temporal hints pay only when the streamed arrays are larger than that cache.
    const bool streams_exceed_cache = (double)d.s_local * (double)d.ld * 4.0 >= 256.0 * 1048576.0;
    hot_launch &f = p->cfg[HOT_KERNEL_FORWARD], &b = p->cfg[HOT_KERNEL_BACKWARD];
    f.grid_blocks = b.grid_blocks = kMaxGrid;
    f.chunks = b.chunks = 4;
    f.unroll = 1;
    b.unroll = pick_unroll(4, d.s_local);
    f.nontemporal = b.nontemporal = streams_exceed_cache ? 1 : 0;
    // With fewer than four samples the four-chunk backward kernels are fat (over 200 registers per lane,
    // two workgroups per compute unit) and short: below 16 M weights their last, partly filled round of
    // workgroups costs 5-10 %, which one chunk per thread avoids.
    const bool few_tiles = d.n_weights < (16L << 20);
    if (d.s_local < 4 && few_tiles) b.chunks = 1;
    // The drawing variants have no eps loads to keep in flight.  Forward: as above up to seven samples;
    // from eight on one chunk per thread (38 registers, eight waves per SIMD) hides the generator's
    // latencies better than four independent chains in five waves (10-20 % at 8 M to 25 M weights).
    // Backward: two chunks and single rows from four samples on.
    hot_launch &fr = p->cfg[HOT_KERNEL_FORWARD_RNG], &br = p->cfg[HOT_KERNEL_BACKWARD_RNG];
    fr = f;
    if (d.s_local >= 8) fr.chunks = 1;
    br = b;
    br.chunks = d.s_local >= 4 ? 2 : (few_tiles ? 1 : 4);
    br.unroll = pick_unroll(d.s_local >= 4 ? 1 : 2, d.s_local);
    *out = p;
    return HOT_OK;
}

int hot_destroy(hot_plan *plan)
{
    if (!plan) return HOT_OK;
    int rc = HOT_OK;
    {
        DeviceGuard guard(plan->d.device);
        if (plan->partials && hipFree(plan->partials) != hipSuccess) rc = HOT_EHIP;
    }
    delete plan;
    return rc;
}

int hot_set_launch(hot_plan *plan, int kernel, const hot_launch *cfg)
{
    if (!plan || !cfg || !valid_kernel(kernel)) return HOT_EINVAL;
    if (!valid_launch(*cfg)) return HOT_EINVAL;
    hot_launch &c = plan->cfg[kernel];
    if (cfg->grid_blocks) c.grid_blocks = cfg->grid_blocks;
    if (cfg->chunks) c.chunks = cfg->chunks;
    if (cfg->unroll) c.unroll = pick_unroll(cfg->unroll, plan->d.s_local);
    c.nontemporal = cfg->nontemporal;
    return HOT_OK;
}

int hot_get_launch(const hot_plan *plan, int kernel, hot_launch *cfg)
{
    if (!plan || !cfg || !valid_kernel(kernel)) return HOT_EINVAL;
    *cfg = plan->cfg[kernel];
    return HOT_OK;
}

int hot_last_hip_error(const hot_plan *plan) { return plan ? plan->last_hip : hot_detail::g_last_hip; }

int hot_forward(hot_plan *plan, const float *mu, const float *sigma, const float *eps, float *w,
                double *kl_out, void *stream)
{
    if (!plan) return HOT_EINVAL;
    return forward_impl(plan, HOT_KERNEL_FORWARD, nullptr, mu, sigma, eps, w, kl_out, stream);
}

int hot_kl(hot_plan *plan, const float *mu, const float *sigma, double *kl_out, void *stream)
{
    if (!plan) return HOT_EINVAL;
    return forward_impl(plan, HOT_KERNEL_FORWARD, nullptr, mu, sigma, nullptr, nullptr, kl_out, stream, true);
}

int hot_adam_forward(hot_plan *plan, const hot_rng *rng, const hot_adam *params, float *mu, float *sigma,
                     const float *grad_mu, const float *grad_sigma, float *m_mu, float *v_mu, float *m_sigma,
                     float *v_sigma, const float *eps, float *w, double *kl_out, void *stream)
{
    if (!plan || (rng != nullptr) == (eps != nullptr)) return HOT_EINVAL;      // exactly one source of eps
    if (!grad_mu || !grad_sigma || !m_mu || !v_mu || !m_sigma || !v_sigma) return HOT_EINVAL;
    const void *ptrs[6] = {grad_mu, grad_sigma, m_mu, v_mu, m_sigma, v_sigma};
    bool al = true;
    for (const void *q : ptrs) {
        if (!aligned4(q)) return HOT_EINVAL;
        al = al && aligned16(q);
    }
    AdamPrologue pro;
    if (!make_adam_const(params, pro.c)) return HOT_EINVAL;
    pro.mu = mu;
    pro.sigma = sigma;
    pro.gmu = grad_mu;
    pro.gsig = grad_sigma;
    pro.m_mu = m_mu;
    pro.v_mu = v_mu;
    pro.m_sig = m_sigma;
    pro.v_sig = v_sigma;
    Rng r;
    if (rng && !make_rng(rng, plan->d.s_local, r)) return HOT_EINVAL;
    return forward_impl(plan, rng ? HOT_KERNEL_FORWARD_RNG : HOT_KERNEL_FORWARD, rng ? &r : nullptr, mu, sigma, eps, w, kl_out,
                        stream, false, &pro, al);
}

int hot_backward(hot_plan *plan, const float *mu, const float *sigma, const float *eps,
                 const float *grad_w, float *grad_mu, float *grad_sigma, void *stream)
{
    if (!plan) return HOT_EINVAL;
    return backward_impl(plan, HOT_KERNEL_BACKWARD, nullptr, mu, sigma, eps, grad_w, grad_mu, grad_sigma, stream);
}

int hot_forward_rng(hot_plan *plan, const hot_rng *rng, const float *mu, const float *sigma, float *w,
                    double *kl_out, void *stream)
{
    Rng r;
    if (!plan || !make_rng(rng, plan->d.s_local, r)) return HOT_EINVAL;
    return forward_impl(plan, HOT_KERNEL_FORWARD_RNG, &r, mu, sigma, nullptr, w, kl_out, stream);
}

int hot_backward_rng(hot_plan *plan, const hot_rng *rng, const float *mu, const float *sigma,
                     const float *grad_w, float *grad_mu, float *grad_sigma, void *stream)
{
    Rng r;
    if (!plan || !make_rng(rng, plan->d.s_local, r)) return HOT_EINVAL;
    return backward_impl(plan, HOT_KERNEL_BACKWARD_RNG, &r, mu, sigma, nullptr, grad_w, grad_mu, grad_sigma, stream);
}

int hot_backward_rows(hot_plan *plan, const hot_rng *rng, const float *mu, const float *sigma, const float *eps,
                      const float *grad_w, int32_t first_row, int32_t rows, int32_t accumulate, int32_t add_kl,
                      float *grad_mu, float *grad_sigma, void *stream)
{
    if (!plan || first_row < 0 || rows < 1 || (long)first_row + rows > plan->d.s_local) return HOT_EINVAL;
    if ((rng != nullptr) == (eps != nullptr)) return HOT_EINVAL;      // exactly one source of eps
    if (rng) {
        Rng r;
        if (!make_rng(rng, plan->d.s_local, r)) return HOT_EINVAL;
        return backward_impl(plan, HOT_KERNEL_BACKWARD_RNG, &r, mu, sigma, nullptr, grad_w, grad_mu, grad_sigma, stream,
                             first_row, rows, accumulate != 0, add_kl != 0);
    }
    return backward_impl(plan, HOT_KERNEL_BACKWARD, nullptr, mu, sigma, eps, grad_w, grad_mu, grad_sigma, stream,
                         first_row, rows, accumulate != 0, add_kl != 0);
}

int hot_backward_adam(hot_plan *plan, const hot_rng *rng, const hot_adam *params, float *mu, float *sigma,
                      const float *eps, const float *grad_w, float *m_mu, float *v_mu, float *m_sigma, float *v_sigma,
                      void *stream)
{
    if (!plan || plan->d.s_local != plan->d.s_total) return HOT_EINVAL;   // one GPU holds all samples
    if ((rng != nullptr) == (eps != nullptr)) return HOT_EINVAL;          // exactly one source of eps
    if (!mu || !sigma || !grad_w || !m_mu || !v_mu || !m_sigma || !v_sigma) return HOT_EINVAL;
    const void *ptrs[8] = {mu, sigma, grad_w, m_mu, v_mu, m_sigma, v_sigma, eps};
    bool al = true;
    for (int i = 0; i < (eps ? 8 : 7); ++i) {
        if (!aligned4(ptrs[i])) return HOT_EINVAL;
        if (i >= 3 && i < 7) al = al && aligned16(ptrs[i]);
    }
    AdamUpdate epi;
    if (!make_adam_const(params, epi.c)) return HOT_EINVAL;
    epi.mu = mu;
    epi.sigma = sigma;
    epi.m_mu = m_mu;
    epi.v_mu = v_mu;
    epi.m_sig = m_sigma;
    epi.v_sig = v_sigma;
    Rng r;
    if (rng && !make_rng(rng, plan->d.s_local, r)) return HOT_EINVAL;
    return backward_launch(plan, rng ? HOT_KERNEL_BACKWARD_RNG : HOT_KERNEL_BACKWARD, rng ? &r : nullptr, mu, sigma, eps,
                           grad_w, epi, al, stream, 0, 0, true);
}

int hot_backward_adam_forward(hot_plan *plan, const hot_rng *rng, const hot_rng *rng_next, const hot_adam *params,
                              float *mu, float *sigma, const float *grad_w, float *m_mu, float *v_mu, float *m_sigma,
                              float *v_sigma, float *w, double *kl_out, void *stream)
{
    if (!plan || plan->d.s_local != plan->d.s_total) return HOT_EINVAL;   // one GPU holds all samples
    if (!mu || !sigma || !grad_w || !m_mu || !v_mu || !m_sigma || !v_sigma || !w || w == grad_w) return HOT_EINVAL;
    if (kl_out && (reinterpret_cast<uintptr_t>(kl_out) & 7u)) return HOT_EINVAL;
    const void *ptrs[8] = {mu, sigma, grad_w, m_mu, v_mu, m_sigma, v_sigma, w};
    bool al = true;
    for (int i = 0; i < 8; ++i) {
        if (!aligned4(ptrs[i])) return HOT_EINVAL;
        if (i >= 3) al = al && aligned16(ptrs[i]);
    }
    AdamUpdateSample epi;
    if (!make_adam_const(params, epi.adam.c)) return HOT_EINVAL;
    Rng r, rn;
    if (!make_rng(rng, plan->d.s_local, r) || !make_rng(rng_next, plan->d.s_local, rn)) return HOT_EINVAL;
    epi.adam.mu = mu;
    epi.adam.sigma = sigma;
    epi.adam.m_mu = m_mu;
    epi.adam.v_mu = v_mu;
    epi.adam.m_sig = m_sigma;
    epi.adam.v_sig = v_sigma;
    epi.w = w;
    epi.ld = plan->d.ld;
    epi.s_loc = plan->d.s_local;
    epi.next = rn;
    epi.partials = kl_out ? plan->partials : nullptr;
    const int rc = backward_launch(plan, HOT_KERNEL_BACKWARD_RNG, &r, mu, sigma, nullptr, grad_w, epi, al, stream, 0, 0, true);
    if (rc != HOT_OK || !kl_out) return rc;
    DeviceGuard guard(plan->d.device);
    if (guard.err != hipSuccess) return fail_hip(plan, guard.err);
    const unsigned blocks = grid_for(plan->d.n_weights, plan->cfg[HOT_KERNEL_BACKWARD_RNG]);
    hot_kl_finish_kernel<<<dim3(1), dim3(kFinishBlock), 0, static_cast<hipStream_t>(stream)>>>(plan->partials, (int)blocks, kl_out);
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? HOT_OK : fail_hip(plan, e);
}

int hot_sample_eps(hot_plan *plan, const hot_rng *rng, float *eps, void *stream)
{
    return sample_impl(plan, rng, eps, false, stream);
}

int hot_sample_bits(hot_plan *plan, const hot_rng *rng, uint32_t *bits, void *stream)
{
    return sample_impl(plan, rng, bits, true, stream);
}

int hot_probe_copy(void *dst, const void *src, int64_t bytes, int nontemporal, void *stream)
{
    if (!dst || !src || bytes < 16 || (bytes & 15) || !aligned16(dst) || !aligned16(src)) return HOT_EINVAL;
    if (nontemporal != 0 && nontemporal != 1) return HOT_EINVAL;
    const long n_vec = bytes / 16;
    const long blocks = (n_vec + kBlock * 4 - 1) / (kBlock * 4);
    if (blocks > 0x7fffffffL) return HOT_EINVAL;
    const dim3 grid((unsigned)blocks), block(kBlock);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const f4 *in = static_cast<const f4 *>(src);
    f4 *out = static_cast<f4 *>(dst);
    if (nontemporal) hot_probe_copy_kernel<true><<<grid, block, 0, s>>>(in, out, n_vec);
    else hot_probe_copy_kernel<false><<<grid, block, 0, s>>>(in, out, n_vec);
    return hot_detail::note_hip(hipGetLastError());
}

int hot_probe_streams(void *arena, int64_t stream_bytes, int reads, int writes, void *stream)
{
    if (!arena || !aligned16(arena) || stream_bytes < 16 || (stream_bytes & 15)) return HOT_EINVAL;
    if (reads < 1 || reads > 6 || writes < 0 || writes > 2) return HOT_EINVAL;
    const long n_vec = stream_bytes / 16;
    const long blocks = (n_vec + kBlock * 4 - 1) / (kBlock * 4);
    if (blocks > 0x7fffffffL) return HOT_EINVAL;
    ProbeStreams p;
    char *base = static_cast<char *>(arena);
    for (int r = 0; r < 6; ++r) p.src[r] = reinterpret_cast<const f4 *>(base + (size_t)(r < reads ? r : 0) * (size_t)stream_bytes);
    // with no write stream the (never taken) store targets the first read stream
    for (int w = 0; w < 2; ++w) p.dst[w] = reinterpret_cast<f4 *>(base + (size_t)(w < writes ? reads + w : 0) * (size_t)stream_bytes);
    const dim3 grid((unsigned)blocks);
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (reads) {
    case 1: probe_streams_go<1>(writes, grid, s, p, n_vec); break;
    case 2: probe_streams_go<2>(writes, grid, s, p, n_vec); break;
    case 3: probe_streams_go<3>(writes, grid, s, p, n_vec); break;
    case 4: probe_streams_go<4>(writes, grid, s, p, n_vec); break;
    case 5: probe_streams_go<5>(writes, grid, s, p, n_vec); break;
    default: probe_streams_go<6>(writes, grid, s, p, n_vec); break;
    }
    return hot_detail::note_hip(hipGetLastError());
}

}  // extern "C"
