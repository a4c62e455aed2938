// libhot, forward half of the sample layer (arxiv 2604.04736, Algorithm 2: reparameterisation and
// prior-matching lines): hot_forward, hot_forward_rng, hot_kl, hot_adam_forward.  The design notes
// common to both halves are at the top of hot.hip.  gfx950 only.
#include <atomic>

#include "sample_layer.h"

// Scratch of hot_forward_static (the entry point that allocates nothing): the per-workgroup KL partial sums
// that a plan otherwise keeps in memory of its own.  One copy per GPU, loaded with the library's code object and
// held until the process ends (512 KiB).  In host code the name is only a handle for hipGetSymbolAddress; the
// device address it returns (one per device) is what kernels and runtime calls are given.
static __device__ __align__(256) double scratch[65536];

namespace {

// What the forward kernel does to the (mu, sigma) of a chunk before it samples from them.
//
// NoPrologue: nothing (Algorithm 2's reparameterisation line on the parameters as they are).
struct NoPrologue {
    struct State {};
    template <bool ALIGNED>
    __device__ __forceinline__ void load(long, State &) const {}
    template <bool ALIGNED>
    __device__ __forceinline__ void apply(long, f4 &, f4 &, State &) const {}
    __device__ __forceinline__ void one(long, float &, float &) const {}
};

// AdamPrologue: the optimizer-update line of the previous step first (Algorithm 1 / 2, end of the inner loop),
// on the all-reduced gradients, with hot_adam_step's arithmetic; the updated parameters are stored
// and, still in registers, sampled from, so they are not read a second time.
struct AdamPrologue {
    float *mu, *sigma;
    const float *gmu, *gsig;
    float *m_mu, *v_mu, *m_sig, *v_sig;
    AdamConst c;
    // In two steps, so that the kernel can issue the loads of all of a thread's chunks before the first store (the
    // arrays are updated in place, and a load that follows a store to the same array in program order stays behind it).
    struct State {
        f4 g0, g1, a0, b0, a1, b1;
    };
    template <bool ALIGNED>
    __device__ __forceinline__ void load(long col, State &st) const
    {
        st.g0 = load4<ALIGNED, true>(gmu + col); st.g1 = load4<ALIGNED, true>(gsig + col);
        st.a0 = load4<ALIGNED, true>(m_mu + col); st.b0 = load4<ALIGNED, true>(v_mu + col);
        st.a1 = load4<ALIGNED, true>(m_sig + col); st.b1 = load4<ALIGNED, true>(v_sig + col);
    }
    template <bool ALIGNED>
    __device__ __forceinline__ void apply(long col, f4 &m, f4 &sd, State &st) const
    {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float t = m[j], a = st.a0[j], b = st.b0[j];
            adam_one(t, a, b, st.g0[j], c);
            m[j] = t; st.a0[j] = a; st.b0[j] = b;
            t = sd[j]; a = st.a1[j]; b = st.b1[j];
            adam_one_sigma(t, a, b, st.g1[j], c);
            sd[j] = t; st.a1[j] = a; st.b1[j] = b;
        }
        store4<ALIGNED, true>(mu + col, m);
        store4<ALIGNED, true>(sigma + col, sd);
        store4<ALIGNED, true>(m_mu + col, st.a0);
        store4<ALIGNED, true>(v_mu + col, st.b0);
        store4<ALIGNED, true>(m_sig + col, st.a1);
        store4<ALIGNED, true>(v_sig + col, st.b1);
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

// Rows s .. s+U-1 of one thread's chunks: all eps values first, then multiply-add and store.  FULL: the tile has
// all its CHUNKS * 1024 columns and is accessed through plain pointers; otherwise through range-checked windows of
// `bytes` bytes from column `begin` on (no branches: see window() in vec.h).
template <int CHUNKS, int U, bool ALIGNED, bool NT, bool GEN, bool FULL>
__device__ __forceinline__ void forward_rows(int s, long begin, unsigned bytes, long ld, const f4 (&m)[CHUNKS],
                                             const f4 (&sd)[CHUNKS], const float *__restrict__ eps,
                                             float *__restrict__ w, const Rng &rng)
{
    constexpr long kStep = (long)kBlock * 4;
    const long col0 = begin + (long)threadIdx.x * 4;
    const unsigned off0 = threadIdx.x * 16u;
    f4 e[U][CHUNKS];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int c = 0; c < CHUNKS; ++c) {
            if constexpr (FULL) e[u][c] = eps4<ALIGNED, NT, GEN>(eps, ld, s + u, col0 + c * kStep, rng);
            else e[u][c] = eps4_window<NT, GEN>(eps, ld, s + u, begin, bytes, off0 + c * (unsigned)(kStep * 4), rng);
        }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        [[maybe_unused]] window_t out;
        if constexpr (!FULL) out = window(w + (size_t)(s + u) * (size_t)ld + begin, bytes);
#pragma unroll
        for (int c = 0; c < CHUNKS; ++c) {
            f4 r;
#pragma unroll
            for (int j = 0; j < 4; ++j) r[j] = __builtin_fmaf(sd[c][j], e[u][c][j], m[c][j]);
            if constexpr (FULL) store4<ALIGNED, NT>(w + (size_t)(s + u) * (size_t)ld + col0 + c * kStep, r);
            else window_store4<NT>(out, off0 + c * (unsigned)(kStep * 4), r);
        }
    }
}

// One column tile [begin, end) of the forward kernel for one thread: mu and sigma of its chunks (through the
// prologue), all rows, and the KL addends.
template <int CHUNKS, int UNROLL, bool ALIGNED, bool NT, bool KL, bool GEN, bool FULL, class PRO>
__device__ __forceinline__ void forward_tile(long begin, long end, long ld, int s_loc, const float *mu, const float *sigma,
                                             const float *__restrict__ eps, float *__restrict__ w, const PRO &pro,
                                             const Rng &rng, double &kl)
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
    typename PRO::State st[CHUNKS];
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c)
        if (ok[c]) pro.template load<ALIGNED>(col0 + c * kStep, st[c]);
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c)
        if (ok[c]) pro.template apply<ALIGNED>(col0 + c * kStep, m[c], sd[c], st[c]);
    int s = 0;
    for (; s + UNROLL <= s_loc; s += UNROLL)
        forward_rows<CHUNKS, UNROLL, ALIGNED, NT, GEN, FULL>(s, begin, bytes, ld, m, sd, eps, w, rng);
    for (; s < s_loc; ++s) forward_rows<CHUNKS, 1, ALIGNED, NT, GEN, FULL>(s, begin, bytes, ld, m, sd, eps, w, rng);
    if constexpr (KL) {
#pragma unroll
        for (int c = 0; c < CHUNKS; ++c)
            if (ok[c]) {
#pragma unroll
                for (int j = 0; j < 4; ++j) kl += kl_addend(m[c][j], sd[c][j]);
            }
    }
}

template <int CHUNKS, int UNROLL, bool ALIGNED, bool NT, bool KL, bool GEN, class PRO>
__global__ void __launch_bounds__(kBlock)
hot_forward_kernel(long n, long ld, int s_loc, long width,
                   const float *mu, const float *sigma,
                   const float *__restrict__ eps, float *__restrict__ w,
                   double *partials, unsigned *ticket, double *__restrict__ kl_out, PRO pro, Rng rng)
{
    // Column tile t is [t * width, min(n, (t + 1) * width)): width <= CHUNKS * 1024 columns, a multiple of 64
    // (tiling_for() picks it).  A thread's chunks sit 1024 columns apart from the tile's first column on.
    constexpr long kStep = (long)kBlock * 4;            // columns between a thread's chunks
    const long n_tiles = (n + width - 1) / width;
    double kl = 0.0;

    for (long tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const long begin = tile * width;
        const long end = begin + width < n ? begin + width : n;
        if (end - begin == CHUNKS * kStep) {
            forward_tile<CHUNKS, UNROLL, ALIGNED, NT, KL, GEN, true>(begin, end, ld, s_loc, mu, sigma, eps, w, pro, rng, kl);
        } else {
            // a narrower tile: the same, every chunk guarded
            forward_tile<CHUNKS, UNROLL, ALIGNED, NT, KL, GEN, false>(begin, end, ld, s_loc, mu, sigma, eps, w, pro, rng, kl);
            // the final 1..3 columns of the vector (n not a multiple of 4), one by one, by the thread whose quad they start
            if (end == n && (n & 3)) {
                const long first = n & ~3L;
                const long off = first - begin;
                if ((long)threadIdx.x * 4 == off % kStep) {
                    for (long i = first; i < n; ++i) {
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

struct FwdArgs {
    long n, ld, width;
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
            a.n, a.ld, a.s_loc, a.width, a.mu, a.sigma, a.eps, a.w, a.partials, a.ticket, a.kl_out, *a.adam, a.rng);
    else if (a.want_kl)
        hot_forward_kernel<CH, U, AL, NT, true, GEN, NoPrologue><<<a.grid, dim3(kBlock), 0, a.stream>>>(
            a.n, a.ld, a.s_loc, a.width, a.mu, a.sigma, a.eps, a.w, a.partials, a.ticket, a.kl_out, NoPrologue{}, a.rng);
    else
        hot_forward_kernel<CH, U, AL, NT, false, GEN, NoPrologue><<<a.grid, dim3(kBlock), 0, a.stream>>>(
            a.n, a.ld, a.s_loc, a.width, a.mu, a.sigma, a.eps, a.w, a.partials, a.ticket, a.kl_out, NoPrologue{}, a.rng);
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

// kl_only: the prior-matching term alone.  The forward kernel runs over zero samples, so it touches
// neither eps nor w (both may be NULL) and only its KL part is left.
// The pointer rules of the forward calls: present where needed, 4-byte aligned, kl_out 8-byte aligned.
bool forward_pointers_ok(bool gen, bool kl_only, const float *mu, const float *sigma, const float *eps, const float *w,
                         const double *kl_out)
{
    if (!mu || !sigma || (!kl_only && !w) || (!gen && !eps) || (kl_only && !kl_out)) return false;
    if (!aligned4(mu) || !aligned4(sigma) || (!kl_only && !aligned4(w)) || (!gen && !aligned4(eps))) return false;
    return !(kl_out && (reinterpret_cast<uintptr_t>(kl_out) & 7u));
}

// finish_kernel_always: never let the forward kernel add the partials itself (that path needs an arrival
// counter that is zero before the launch; the finish kernel needs no state at all).
int forward_impl(hot_plan *plan, int kernel, const Rng *rng, const float *mu, const float *sigma,
                 const float *eps, float *w, double *kl_out, void *stream, bool kl_only = false,
                 const AdamPrologue *adam = nullptr, bool adam_aligned = true, bool finish_kernel_always = false)
{
    const bool gen = rng != nullptr || kl_only;      // kl_only: no eps array to look at
    if (!forward_pointers_ok(gen, kl_only, mu, sigma, eps, w, kl_out)) return HOT_EINVAL;
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
    const Tiling tiling = tiling_for(d.n_weights, c);
    a.width = tiling.width;
    a.grid = dim3(tiling.grid);
    a.stream = static_cast<hipStream_t>(stream);

    // Rows of w off the 64-byte grid, streamed with non-temporal stores, eps from its array, four chunks per
    // thread: the kernel that moves its column window row by row (its shape is fixed at four chunks; with
    // fewer, i.e. few column tiles, the general kernel runs).
    const bool rows_on_grid = (reinterpret_cast<uintptr_t>(w) & 63u) == 0 && (d.s_local == 1 || d.ld % 16 == 0);
    const bool shifted = !kl_only && !adam && !gen && c.nontemporal != 0 && c.chunks == 4 && !rows_on_grid;
    if (shifted) {      // (its windows reach back by up to 15 columns, so there may be one more of them than tiles)
        const long windows = (d.n_weights + 15 + 4095) / 4096;
        a.grid = dim3((unsigned)(windows < c.grid_blocks ? windows : c.grid_blocks));
    }
    const bool self_finish = a.want_kl && a.grid.x <= (unsigned)kTicketGrid && !finish_kernel_always;
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

static_assert(sizeof(scratch) == sizeof(double) * kMaxGrid, "one KL partial per workgroup of the largest grid");

// Device address of `scratch` on each device, looked up on the first call there.
constexpr int kMaxDevices = 64;
std::atomic<double *> g_scratch_ptr[kMaxDevices];

}  // namespace

extern "C" {

int hot_forward_static(const hot_desc *desc, const float *mu, const float *sigma, const float *eps, float *w,
                       double *kl_out, void *stream)
{
    if (!desc || !valid_desc(*desc)) return HOT_EINVAL;
    if (desc->device < 0 || desc->device >= kMaxDevices) return HOT_EINVAL;
    if (desc->n_weights > HOT_STATIC_MAX_WEIGHTS) return HOT_ERANGE;
    if (!forward_pointers_ok(false, false, mu, sigma, eps, w, kl_out)) return HOT_EINVAL;      // before any HIP call
    double *ptr = g_scratch_ptr[desc->device].load(std::memory_order_acquire);
    if (!ptr) {
        // first call on this device: with it current, ask the runtime where its copy of the array lives
        // (threads that race here look up the same address)
        int n_dev = 0;
        if (hipError_t e = hipGetDeviceCount(&n_dev); e != hipSuccess) return hot_detail::note_hip(e);
        if (desc->device >= n_dev) return HOT_EINVAL;
        DeviceGuard guard(desc->device);
        if (guard.err != hipSuccess) return hot_detail::note_hip(guard.err);
        void *at = nullptr;
        if (hipError_t e = hipGetSymbolAddress(&at, HIP_SYMBOL(scratch)); e != hipSuccess) return hot_detail::note_hip(e);
        if (!at) return hot_detail::note_hip(hipErrorInvalidSymbol);
        ptr = static_cast<double *>(at);
        g_scratch_ptr[desc->device].store(ptr, std::memory_order_release);
    }
    // a plan on the stack: the description, the default launch geometry, and the static array for its partials
    hot_plan tmp;
    tmp.d = *desc;
    set_scaling(tmp);
    default_launches(tmp);
    tmp.partials = ptr;
    tmp.last_hip = 0;
    const int rc = forward_impl(&tmp, HOT_KERNEL_FORWARD, nullptr, mu, sigma, eps, w, kl_out, stream, false, nullptr, true, true);
    if (rc == HOT_EHIP) (void)hot_detail::note_hip(static_cast<hipError_t>(tmp.last_hip));
    return rc;
}

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

int hot_forward_rng(hot_plan *plan, const hot_rng *rng, const float *mu, const float *sigma, float *w,
                    double *kl_out, void *stream)
{
    Rng r;
    if (!plan || !make_rng(rng, plan->d.s_local, r)) return HOT_EINVAL;
    return forward_impl(plan, HOT_KERNEL_FORWARD_RNG, &r, mu, sigma, nullptr, w, kl_out, stream);
}

}  // extern "C"
