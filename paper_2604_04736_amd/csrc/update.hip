// libhot: the two steps next to the Gaussian sample layer in the paper's algorithms
// (arxiv 2604.04736), both streaming kernels bound by HBM:
//   hot_adam_step              the optimizer-update line that closes the inner loop of
//                              Algorithm 1 / 2 (Adam, the paper's example): one pass over eight input and six
//                              output arrays (56 bytes per weight), Adam as published by Kingma & Ba;
//   hot_forward_dropout_rng,   Monte Carlo dropout in weight space (section "Monte Carlo Dropout":
//   hot_backward_dropout_rng   each weight carries a random 0/1 keep factor), the mask being a
//                              threshold on the same counter-based generator words the Gaussian
//                              draw uses, so it is never stored and the backward pass regenerates it.
#include <hip/hip_runtime.h>

#include <cmath>

#include "hot.h"
#include "vec.h"
#include "draw.h"
#include "adam.h"

namespace {

constexpr int kBlock = 256;

// Four 16-byte chunks per thread and non-temporal accesses measured best on MI355X (5.6 TB/s
// against 5.3 TB/s with one chunk and cached accesses).
constexpr int kAdamChunks = 4;

// A workgroup takes tiles of kBlock * kAdamChunks quads; every array is read and written through a range-checked
// window over the tile's whole quads (vec.h: a load beyond it returns zeros, a store beyond it is dropped), so no
// thread branches around its accesses.  Behind branches (one per chunk, as this kernel had them) the compiler cannot
// count the memory operations in flight across the joins and waits for all of them, loads and the previous chunk's
// stores alike, before each chunk's stores.  Here the 32 loads of a tile are issued first and its 24 stores follow
// the arithmetic without a wait between them.  The last one to three weights of a vector whose length is no
// multiple of four are updated one by one by a single thread.
__global__ void __launch_bounds__(kBlock)
hot_adam_kernel(long n, AdamConst c, float *__restrict__ mu, float *__restrict__ sigma,
                const float *__restrict__ gmu, const float *__restrict__ gsig, float *__restrict__ m_mu,
                float *__restrict__ v_mu, float *__restrict__ m_sig, float *__restrict__ v_sig)
{
    constexpr int CH = kAdamChunks;
    constexpr bool NT = true;
    constexpr long kTile = (long)kBlock * 4 * CH;      // weights per tile
    const long whole = n & ~3L;                         // weights in whole quads
    const long n_tiles = (whole + kTile - 1) / kTile;
    for (long tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const long begin = tile * kTile;
        const unsigned bytes = (unsigned)(((begin + kTile < whole ? begin + kTile : whole) - begin) * 4);
        const window_t w_p0 = window(mu + begin, bytes), w_p1 = window(sigma + begin, bytes);
        const window_t w_g0 = window(gmu + begin, bytes), w_g1 = window(gsig + begin, bytes);
        const window_t w_m0 = window(m_mu + begin, bytes), w_v0 = window(v_mu + begin, bytes);
        const window_t w_m1 = window(m_sig + begin, bytes), w_v1 = window(v_sig + begin, bytes);
        f4 p0[CH], p1[CH], g0[CH], g1[CH], m0[CH], v0[CH], m1[CH], v1[CH];
#pragma unroll
        for (int q = 0; q < CH; ++q) {
            const unsigned off = threadIdx.x * 16u + (unsigned)q * (kBlock * 16u);
            p0[q] = window_load4<NT>(w_p0, off); p1[q] = window_load4<NT>(w_p1, off);
            g0[q] = window_load4<NT>(w_g0, off); g1[q] = window_load4<NT>(w_g1, off);
            m0[q] = window_load4<NT>(w_m0, off); v0[q] = window_load4<NT>(w_v0, off);
            m1[q] = window_load4<NT>(w_m1, off); v1[q] = window_load4<NT>(w_v1, off);
        }
#pragma unroll
        for (int q = 0; q < CH; ++q) {
            const unsigned off = threadIdx.x * 16u + (unsigned)q * (kBlock * 16u);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float t = p0[q][j], a = m0[q][j], b = v0[q][j];
                adam_one(t, a, b, g0[q][j], c);
                p0[q][j] = t; m0[q][j] = a; v0[q][j] = b;
                t = p1[q][j]; a = m1[q][j]; b = v1[q][j];
                adam_one_sigma(t, a, b, g1[q][j], c);
                p1[q][j] = t; m1[q][j] = a; v1[q][j] = b;
            }
            window_store4<NT>(w_p0, off, p0[q]);
            window_store4<NT>(w_p1, off, p1[q]);
            window_store4<NT>(w_m0, off, m0[q]);
            window_store4<NT>(w_v0, off, v0[q]);
            window_store4<NT>(w_m1, off, m1[q]);
            window_store4<NT>(w_v1, off, v1[q]);
        }
    }
    if (whole < n && blockIdx.x == 0 && threadIdx.x == 0) {
        for (long i = whole; i < n; ++i) {
            float t = mu[i], a = m_mu[i], b = v_mu[i];
            adam_one(t, a, b, gmu[i], c);
            mu[i] = t; m_mu[i] = a; v_mu[i] = b;
            t = sigma[i]; a = m_sig[i]; b = v_sig[i];
            adam_one_sigma(t, a, b, gsig[i], c);
            sigma[i] = t; m_sig[i] = a; v_sig[i] = b;
        }
    }
}

// b[s, 4q .. 4q+3] = (generator word < floor(keep * 2^32)), as multipliers 1/keep or 0.  The threshold lies in
// [0, 2^32] and arrives as last_kept = threshold - 1 for a 32-bit compare (keep = 1 keeps every word); a
// threshold of 0 (keep below 2^-32) arrives as last_kept = 0 with inv_keep = 0, so nothing is kept.
__device__ __forceinline__ f4 mask_quad(long quad, int s, const Rng &rng, unsigned last_kept, float inv_keep)
{
    const u4 x = eps_words(quad, s, rng);
    f4 b;
#pragma unroll
    for (int j = 0; j < 4; ++j) b[j] = x[j] <= last_kept ? inv_keep : 0.0f;
    return b;
}

// Which generator quad masks the weights 4 chunk .. 4 chunk + 3: their own (one Bernoulli variable per
// weight), or, with period = K > 0, that of the input units (4 chunk) mod K .. of a [*, K] weight
// matrix (one variable per unit and sample, shared by the unit's weights to all outputs).
__device__ __forceinline__ long mask_quad_index(long chunk, long period, long unit_quad0)
{
    return period > 0 ? unit_quad0 + (((chunk * 4) % period) >> 2) : chunk;
}

__device__ __forceinline__ float pick(f4 v, int j) { return j == 0 ? v[0] : (j == 1 ? v[1] : (j == 2 ? v[2] : v[3])); }

template <bool ALIGNED, bool NT>
__global__ void __launch_bounds__(kBlock)
hot_dropout_forward_kernel(long n, long ld, int s_loc, const float *__restrict__ mu, float *__restrict__ w,
                           Rng rng, unsigned last_kept, float inv_keep, long period, long unit_quad0)
{
    const long n_chunks = (n + 3) / 4;
    for (long chunk = (long)blockIdx.x * kBlock + threadIdx.x; chunk < n_chunks; chunk += (long)gridDim.x * kBlock) {
        const long col = chunk * 4;
        const long mq = mask_quad_index(chunk, period, unit_quad0);
        if (col + 4 <= n) {
            const f4 m = load4<ALIGNED, NT>(mu + col);
            for (int s = 0; s < s_loc; ++s) {
                const f4 b = mask_quad(mq, s, rng, last_kept, inv_keep);
                store4<ALIGNED, NT>(w + (size_t)s * (size_t)ld + col, m * b);
            }
        } else {
            for (int s = 0; s < s_loc; ++s) {
                const f4 b = mask_quad(mq, s, rng, last_kept, inv_keep);
                for (long i = col; i < n; ++i) w[(size_t)s * (size_t)ld + (size_t)i] = mu[i] * pick(b, (int)(i - col));
            }
        }
    }
}

template <bool ALIGNED, bool NT>
__global__ void __launch_bounds__(kBlock)
hot_dropout_backward_kernel(long n, long ld, int s_loc, double g, const float *__restrict__ gw,
                            float *__restrict__ gmu, Rng rng, unsigned last_kept, float inv_keep, long period,
                            long unit_quad0)
{
    const long n_chunks = (n + 3) / 4;
    for (long chunk = (long)blockIdx.x * kBlock + threadIdx.x; chunk < n_chunks; chunk += (long)gridDim.x * kBlock) {
        const long col = chunk * 4;
        const long mq = mask_quad_index(chunk, period, unit_quad0);
        if (col + 4 <= n) {
            double acc[4] = {0.0, 0.0, 0.0, 0.0};
            int s = 0;
            for (; s + 2 <= s_loc; s += 2) {
                const f4 v0 = load4<ALIGNED, NT>(gw + (size_t)s * (size_t)ld + col);
                const f4 v1 = load4<ALIGNED, NT>(gw + (size_t)(s + 1) * (size_t)ld + col);
                const f4 b0 = mask_quad(mq, s, rng, last_kept, inv_keep);
                const f4 b1 = mask_quad(mq, s + 1, rng, last_kept, inv_keep);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc[j] = fma((double)v0[j], (double)b0[j], acc[j]);
                    acc[j] = fma((double)v1[j], (double)b1[j], acc[j]);
                }
            }
            for (; s < s_loc; ++s) {
                const f4 v0 = load4<ALIGNED, NT>(gw + (size_t)s * (size_t)ld + col);
                const f4 b0 = mask_quad(mq, s, rng, last_kept, inv_keep);
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[j] = fma((double)v0[j], (double)b0[j], acc[j]);
            }
            f4 o;
#pragma unroll
            for (int j = 0; j < 4; ++j) o[j] = (float)(g * acc[j]);
            store4<ALIGNED, NT>(gmu + col, o);
        } else {
            double acc[3] = {0.0, 0.0, 0.0};
            for (int s = 0; s < s_loc; ++s) {
                const f4 b = mask_quad(mq, s, rng, last_kept, inv_keep);
#pragma unroll
                for (int j = 0; j < 3; ++j)
                    if (col + j < n) acc[j] = fma((double)gw[(size_t)s * (size_t)ld + (size_t)(col + j)], (double)pick(b, j), acc[j]);
            }
#pragma unroll
            for (int j = 0; j < 3; ++j)
                if (col + j < n) gmu[col + j] = (float)(g * acc[j]);
        }
    }
}

unsigned blocks_for(long chunks)
{
    long b = (chunks + kBlock - 1) / kBlock;
    if (b > (1L << 22)) b = 1L << 22;
    if (b < 1) b = 1;
    return (unsigned)b;
}

// The kernels' form of the keep threshold floor(keep * 2^32) in [0, 2^32] (see mask_quad).
struct DropMask {
    unsigned last_kept;
    float inv_keep;
};

DropMask drop_mask(double keep)
{
    double t = std::floor(keep * 4294967296.0);
    if (t > 4294967296.0) t = 4294967296.0;
    if (t < 1.0) return DropMask{0u, 0.0f};
    return DropMask{(unsigned)(t - 1.0), (float)(1.0 / keep)};
}

}  // namespace

extern "C" {

int hot_adam_step(const hot_adam *p, int64_t n, float *mu, float *sigma, const float *grad_mu,
                  const float *grad_sigma, float *m_mu, float *v_mu, float *m_sigma, float *v_sigma, void *stream)
{
    if (n < 1 || !mu || !sigma || !grad_mu || !grad_sigma || !m_mu || !v_mu || !m_sigma || !v_sigma) return HOT_EINVAL;
    AdamConst c;
    if (!make_adam_const(p, c)) return HOT_EINVAL;
    const void *ptrs[8] = {mu, sigma, grad_mu, grad_sigma, m_mu, v_mu, m_sigma, v_sigma};
    for (const void *q : ptrs)
        if (!aligned4(q)) return HOT_EINVAL;
    const dim3 grid(blocks_for(((n + 3) / 4 + kAdamChunks - 1) / kAdamChunks)), block(kBlock);
    hipStream_t s = static_cast<hipStream_t>(stream);
    hot_adam_kernel<<<grid, block, 0, s>>>(n, c, mu, sigma, grad_mu, grad_sigma, m_mu, v_mu, m_sigma, v_sigma);
    return hot_detail::note_hip(hipGetLastError());
}

static int dropout_forward_impl(const hot_desc *d, const hot_rng *rng, double keep, long period, long unit_offset,
                                const float *mu, float *w, void *stream)
{
    if (!d || !mu || !w || !aligned4(mu) || !aligned4(w)) return HOT_EINVAL;
    if (period < 0 || (period & 3) || unit_offset < 0 || (unit_offset & 3)) return HOT_EINVAL;
    if (d->n_weights < 1 || d->ld < d->n_weights || d->s_local < 1 || d->s_total < d->s_local) return HOT_EINVAL;
    if (d->ld > (INT64_MAX / 4) / d->s_local) return HOT_EINVAL;      // element offsets must fit in 63 bits
    if (!(keep > 0.0 && keep <= 1.0)) return HOT_EINVAL;
    Rng r;
    if (!make_rng(rng, d->s_local, r)) return HOT_EINVAL;
    const bool al = aligned16(mu) && aligned16(w) && (d->ld % 4 == 0);
    const bool nt = (double)d->s_local * (double)d->ld * 4.0 >= 256.0 * 1048576.0;
    const dim3 grid(blocks_for((d->n_weights + 3) / 4)), block(kBlock);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const DropMask dm = drop_mask(keep);
    const unsigned thr = dm.last_kept;
    const float inv = dm.inv_keep;
    if (al && nt) hot_dropout_forward_kernel<true, true><<<grid, block, 0, s>>>(d->n_weights, d->ld, d->s_local, mu, w, r, thr, inv, period, unit_offset >> 2);
    else if (al) hot_dropout_forward_kernel<true, false><<<grid, block, 0, s>>>(d->n_weights, d->ld, d->s_local, mu, w, r, thr, inv, period, unit_offset >> 2);
    else hot_dropout_forward_kernel<false, false><<<grid, block, 0, s>>>(d->n_weights, d->ld, d->s_local, mu, w, r, thr, inv, period, unit_offset >> 2);
    return hot_detail::note_hip(hipGetLastError());
}

static int dropout_backward_impl(const hot_desc *d, const hot_rng *rng, double keep, long period, long unit_offset,
                                 const float *grad_w, float *grad_mu, void *stream)
{
    if (!d || !grad_w || !grad_mu || !aligned4(grad_w) || !aligned4(grad_mu)) return HOT_EINVAL;
    if (period < 0 || (period & 3) || unit_offset < 0 || (unit_offset & 3)) return HOT_EINVAL;
    if (d->n_weights < 1 || d->ld < d->n_weights || d->s_local < 1 || d->s_total < d->s_local) return HOT_EINVAL;
    if (d->ld > (INT64_MAX / 4) / d->s_local) return HOT_EINVAL;      // element offsets must fit in 63 bits
    if (d->flags != HOT_REDUCE_SUM && d->flags != HOT_REDUCE_MEAN && d->flags != HOT_REDUCE_NONE) return HOT_EINVAL;
    if (!(keep > 0.0 && keep <= 1.0)) return HOT_EINVAL;
    Rng r;
    if (!make_rng(rng, d->s_local, r)) return HOT_EINVAL;
    const bool al = aligned16(grad_w) && aligned16(grad_mu) && (d->ld % 4 == 0);
    const bool nt = (double)d->s_local * (double)d->ld * 4.0 >= 256.0 * 1048576.0;
    const double g = d->flags == HOT_REDUCE_NONE ? 1.0
                     : (d->flags == HOT_REDUCE_MEAN ? 1.0 / (double)d->s_local : 1.0 / (double)d->s_total);
    const dim3 grid(blocks_for((d->n_weights + 3) / 4)), block(kBlock);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const DropMask dm = drop_mask(keep);
    const unsigned thr = dm.last_kept;
    const float inv = dm.inv_keep;
    if (al && nt) hot_dropout_backward_kernel<true, true><<<grid, block, 0, s>>>(d->n_weights, d->ld, d->s_local, g, grad_w, grad_mu, r, thr, inv, period, unit_offset >> 2);
    else if (al) hot_dropout_backward_kernel<true, false><<<grid, block, 0, s>>>(d->n_weights, d->ld, d->s_local, g, grad_w, grad_mu, r, thr, inv, period, unit_offset >> 2);
    else hot_dropout_backward_kernel<false, false><<<grid, block, 0, s>>>(d->n_weights, d->ld, d->s_local, g, grad_w, grad_mu, r, thr, inv, period, unit_offset >> 2);
    return hot_detail::note_hip(hipGetLastError());
}

int hot_forward_dropout_rng(const hot_desc *d, const hot_rng *rng, double keep, const float *mu, float *w, void *stream)
{
    return dropout_forward_impl(d, rng, keep, 0, 0, mu, w, stream);
}

int hot_backward_dropout_rng(const hot_desc *d, const hot_rng *rng, double keep, const float *grad_w, float *grad_mu,
                             void *stream)
{
    return dropout_backward_impl(d, rng, keep, 0, 0, grad_w, grad_mu, stream);
}

int hot_forward_dropout_units_rng(const hot_desc *d, const hot_rng *rng, double keep, int64_t in_features,
                                  int64_t unit_offset, const float *mu, float *w, void *stream)
{
    if (in_features < 4) return HOT_EINVAL;
    return dropout_forward_impl(d, rng, keep, in_features, unit_offset, mu, w, stream);
}

int hot_backward_dropout_units_rng(const hot_desc *d, const hot_rng *rng, double keep, int64_t in_features,
                                   int64_t unit_offset, const float *grad_w, float *grad_mu, void *stream)
{
    if (in_features < 4) return HOT_EINVAL;
    return dropout_backward_impl(d, rng, keep, in_features, unit_offset, grad_w, grad_mu, stream);
}

}  // extern "C"
