// libhot, backward half of the sample layer (arxiv 2604.04736, Algorithm 2: loss, gradient and averaging
// lines; Algorithm 1: with the optimizer step and the next sampling in its epilogue): hot_backward,
// hot_backward_rng, hot_backward_rows, hot_backward_adam, hot_backward_adam_forward.  The design notes
// common to both halves are at the top of hot.hip.  gfx950 only.
#include "sample_layer.h"

namespace {

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
    // Every epilogue works in two steps: load() for all of a thread's chunks, then quad() chunk by chunk.  A load
    // that follows a store in program order can only be waited for together with that store, so what an epilogue
    // reads is fetched before its first chunk is written.
    // Here: what the outputs hold, if the gradients are to be added to it.  The loads go through a range-checked
    // window (vec.h) that is empty unless accumulate is set: no branch, hence no join at which the compiler would
    // have to wait for every outstanding access, the previous chunk's stores included.
    struct State {
        f4 om, os;
    };
    // tile: the tile's first column, bytes: its size, off: byte offset of this quad in the tile, col = tile + off / 4
    template <bool ALIGNED, bool NT>
    __device__ __forceinline__ void load(long tile, unsigned bytes, unsigned off, long, bool, State &st) const
    {
        const unsigned held = accumulate ? bytes : 0u;
        st.om = window_load4<NT>(window(gmu + tile, held), off);
        st.os = window_load4<NT>(window(gsig + tile, held), off);
    }
    // The same right before a chunk's stores, behind a branch: nothing is issued when there is nothing to add.
    template <bool ALIGNED, bool NT>
    __device__ __forceinline__ void load_late(long col, State &st) const
    {
        st.om = st.os = f4{0.0f, 0.0f, 0.0f, 0.0f};
        if (accumulate) {
            st.om = load4<ALIGNED, NT>(gmu + col);
            st.os = load4<ALIGNED, NT>(gsig + col);
        }
    }
    template <bool ALIGNED, bool NT>
    __device__ __forceinline__ void quad(long col, f4, f4, const double (&gm)[4], const double (&gs)[4], double &, State &st) const
    {
        f4 om, os;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            om[j] = (float)(gm[j] + (double)st.om[j]);
            os[j] = (float)(gs[j] + (double)st.os[j]);
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
    // The moments are read chunk by chunk inside the update, not ahead of it: holding those of all four chunks
    // costs the kernels with this epilogue a wave per SIMD (the one that also writes the next samples: 2.43 ->
    // 2.60 ms at 209 M weights x 2 samples; backward + Adam at 6.3 M x 16: 0.186 -> 0.195 ms).
    struct State {};
    template <bool ALIGNED, bool NT>
    __device__ __forceinline__ void load(long, unsigned, unsigned, long, bool, State &) const {}
    template <bool ALIGNED, bool NT>
    __device__ __forceinline__ void load_late(long, State &) const {}
    // updates m, sd and the moments in place and stores them
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
    __device__ __forceinline__ void quad(long col, f4 m, f4 sd, const double (&gm)[4], const double (&gs)[4], double &, State &) const
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
    using State = AdamUpdate::State;
    template <bool ALIGNED, bool NT>
    __device__ __forceinline__ void load(long, unsigned, unsigned, long, bool, State &) const {}
    template <bool ALIGNED, bool NT>
    __device__ __forceinline__ void load_late(long, State &) const {}
    template <bool ALIGNED, bool NT>
    __device__ __forceinline__ void quad(long col, f4 m, f4 sd, const double (&gm)[4], const double (&gs)[4], double &kl, State &) const
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

// ---------------------------------------------------------------------------------
// Backward: column sums over the local samples of grad_w and grad_w * eps, then the
// KL gradient and the scaling (Algorithm 2, loss / gradient / averaging lines).
// ---------------------------------------------------------------------------------
// Rows s .. s+U-1 of one thread's chunks: all loads first, then the sums.  FULL: the tile has all its CHUNKS * 1024
// columns and is read through plain pointers; otherwise through range-checked windows of `bytes` bytes from column
// `begin` on (no branches: see window() in vec.h; what lies beyond the tile reads as zero and adds nothing).
template <int CHUNKS, int U, bool ALIGNED, bool NT, bool GEN, bool FULL>
__device__ __forceinline__ void backward_rows(int s, long begin, unsigned bytes, long ld, double (&sum_g)[CHUNKS][4],
                                              double (&sum_ge)[CHUNKS][4], const float *__restrict__ eps,
                                              const float *__restrict__ gw, const Rng &rng)
{
    constexpr long kStep = (long)kBlock * 4;
    const long col0 = begin + (long)threadIdx.x * 4;
    const unsigned off0 = threadIdx.x * 16u;
    f4 gv[U][CHUNKS], ev[U][CHUNKS];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        [[maybe_unused]] window_t in;
        if constexpr (!FULL) in = window(gw + (size_t)(s + u) * (size_t)ld + begin, bytes);
#pragma unroll
        for (int c = 0; c < CHUNKS; ++c) {
            if constexpr (FULL) {
                gv[u][c] = load4<ALIGNED, NT>(gw + (size_t)(s + u) * (size_t)ld + col0 + c * kStep);
                ev[u][c] = eps4<ALIGNED, NT, GEN>(eps, ld, s + u, col0 + c * kStep, rng);
            } else {
                gv[u][c] = window_load4<NT>(in, off0 + c * (unsigned)(kStep * 4));
                ev[u][c] = eps4_window<NT, GEN>(eps, ld, s + u, begin, bytes, off0 + c * (unsigned)(kStep * 4), rng);
            }
        }
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

// One column tile [begin, end) of the backward kernel for one thread: mu and sigma of its chunks, the sample sums,
// the finished gradients handed to the epilogue.
template <int CHUNKS, int UNROLL, bool ALIGNED, bool NT, bool GEN, bool FULL, class EPI>
__device__ __forceinline__ void backward_tile(long begin, long end, long ld, int s_loc, double g, double k,
                                              const float *mu, const float *sigma, const float *__restrict__ eps,
                                              const float *__restrict__ gw, const EPI &epi, const Rng &rng, double &acc)
{
    constexpr long kStep = (long)kBlock * 4;
    const long col0 = begin + (long)threadIdx.x * 4;
    const unsigned bytes = (unsigned)(((end & ~3L) - begin) * 4);     // the tile's whole quads
    f4 m[CHUNKS], sd[CHUNKS];
    bool ok[CHUNKS];
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
        ok[c] = FULL || col0 + c * kStep + 4 <= end;
        if constexpr (FULL) {
            m[c] = load4<ALIGNED, NT>(mu + col0 + c * kStep);
            sd[c] = load4<ALIGNED, NT>(sigma + col0 + c * kStep);
        } else {
            m[c] = window_load4<NT>(window(mu + begin, bytes), threadIdx.x * 16u + c * (unsigned)(kStep * 4));
            sd[c] = window_load4<NT>(window(sigma + begin, bytes), threadIdx.x * 16u + c * (unsigned)(kStep * 4));
        }
    }
    double sum_g[CHUNKS][4], sum_ge[CHUNKS][4];
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c)
#pragma unroll
        for (int j = 0; j < 4; ++j) sum_g[c][j] = sum_ge[c][j] = 0.0;
    int s = 0;
    for (; s + UNROLL <= s_loc; s += UNROLL)
        backward_rows<CHUNKS, UNROLL, ALIGNED, NT, GEN, FULL>(s, begin, bytes, ld, sum_g, sum_ge, eps, gw, rng);
    for (; s < s_loc; ++s)
        backward_rows<CHUNKS, 1, ALIGNED, NT, GEN, FULL>(s, begin, bytes, ld, sum_g, sum_ge, eps, gw, rng);
    // What the epilogue reads is fetched for all chunks ahead of the first chunk's stores where that measured
    // faster (four rows in flight: 6.3 M x 16 0.143 -> 0.141 ms, 7.7 M x 13 0.155 -> 0.152; eps drawn: 0.803 ->
    // 0.796 ms at 209 M x 2), chunk by chunk behind a branch where it did not (two rows in flight, eps from its
    // array: 1.090 ms against 1.100 at 209 M x 2, where even loads from an empty window take their time).
    constexpr bool kAhead = GEN || UNROLL >= 4;
    constexpr unsigned kTileBytes = FULL ? (unsigned)(CHUNKS * kStep * 4) : 0u;
    typename EPI::State st[CHUNKS];
    if constexpr (kAhead) {
#pragma unroll
        for (int c = 0; c < CHUNKS; ++c)
            epi.template load<ALIGNED, NT>(begin, FULL ? kTileBytes : bytes, threadIdx.x * 16u + c * (unsigned)(kStep * 4),
                                           col0 + c * kStep, ok[c], st[c]);
    }
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c)
        if (ok[c]) {
            if constexpr (!kAhead) epi.template load_late<ALIGNED, NT>(col0 + c * kStep, st[c]);
            double gm[4], gs[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) finish_grad(sum_g[c][j], sum_ge[c][j], m[c][j], sd[c][j], g, k, gm[j], gs[j]);
            epi.template quad<ALIGNED, NT>(col0 + c * kStep, m[c], sd[c], gm, gs, acc, st[c]);
        }
}

template <int CHUNKS, int UNROLL, bool ALIGNED, bool NT, bool GEN, class EPI>
__global__ void __launch_bounds__(kBlock)
hot_backward_kernel(long n, long ld, int s_loc, long width, double g, double k,
                    const float *mu, const float *sigma,
                    const float *__restrict__ eps, const float *__restrict__ gw, EPI epi, Rng rng)
{
    // Column tiles as in the forward kernel: tile t is [t * width, min(n, (t + 1) * width)), width <= CHUNKS * 1024.
    constexpr long kStep = (long)kBlock * 4;
    const long n_tiles = (n + width - 1) / width;
    double acc = 0.0;   // what a reducing epilogue sums per thread (the KL addends of AdamUpdateSample)

    for (long tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const long begin = tile * width;
        const long end = begin + width < n ? begin + width : n;
        if (end - begin == CHUNKS * kStep) {
            // (four rows in flight, eps from its array: the full tile through windows too, where a row's base address
            // sits in scalar registers and all rows share the four chunk offsets, instead of 32 per-thread 64-bit
            // addresses per step: measured, 6.3 M x 16 0.143 ms against 0.153 through plain pointers)
            backward_tile<CHUNKS, UNROLL, ALIGNED, NT, GEN, (GEN || UNROLL < 4)>(begin, end, ld, s_loc, g, k, mu, sigma, eps, gw, epi, rng, acc);
        } else {
            // A narrower tile (the last one) goes through range-checked windows.  With eps from its array, chunk by chunk
            // in a loop that is kept a loop on purpose: unrolled, the windowed body takes as many registers as the full
            // one, and the compiler then staggers the full tile's loads instead of issuing them all ahead of the sums
            // (209 M weights x 2 samples: 1.124 ms against 1.103).  With eps drawn, all chunks at once: there the same
            // unrolled body leaves the full tile's code two waves per SIMD instead of three, and faster (0.805 ms
            // against 0.824).
            if constexpr (GEN) {
                backward_tile<CHUNKS, UNROLL, ALIGNED, NT, GEN, false>(begin, end, ld, s_loc, g, k, mu, sigma, eps, gw, epi, rng, acc);
            } else {
#pragma unroll 1
                for (long from = begin; from < end; from += kStep)
                    backward_tile<1, UNROLL, ALIGNED, NT, GEN, false>(from, from + kStep < end ? from + kStep : end, ld, s_loc,
                                                                      g, k, mu, sigma, eps, gw, epi, rng, acc);
            }
            // the final 1..3 columns of the vector (n not a multiple of 4), one by one, by the thread whose quad they start
            if (end == n && (n & 3)) {
                const long first = n & ~3L;
                if ((long)threadIdx.x * 4 == (first - begin) % kStep) {
                    for (long i = first; i < n; ++i) {
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

template <class EPI>
struct BwdArgs {
    long n, ld, width;
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
        a.n, a.ld, a.s_loc, a.width, a.g, a.k, a.mu, a.sigma, a.eps, a.gw, a.epi, a.rng);
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
    const Tiling tiling = tiling_for(d.n_weights, c);
    a.width = tiling.width;
    a.grid = dim3(tiling.grid);
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

}  // namespace

extern "C" {

int hot_backward(hot_plan *plan, const float *mu, const float *sigma, const float *eps,
                 const float *grad_w, float *grad_mu, float *grad_sigma, void *stream)
{
    if (!plan) return HOT_EINVAL;
    return backward_impl(plan, HOT_KERNEL_BACKWARD, nullptr, mu, sigma, eps, grad_w, grad_mu, grad_sigma, stream);
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
    const unsigned blocks = tiling_for(plan->d.n_weights, plan->cfg[HOT_KERNEL_BACKWARD_RNG]).grid;
    hot_kl_finish_kernel<<<dim3(1), dim3(kFinishBlock), 0, static_cast<hipStream_t>(stream)>>>(plan->partials, (int)blocks, kl_out);
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? HOT_OK : fail_hip(plan, e);
}

}  // extern "C"
