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
//     four per-wave partial sums of the KL reduction (the one exception is the forward kernel
//     for rows off the 64-byte grid, which stages mu and sigma so that a column can be stored
//     by another thread than the one that loaded it);
//   * when the arrays exceed the 256 MiB memory-side cache EVERY access of a full tile carries the
//     non-temporal hint, mu, sigma and the gradient outputs included: a single stream of ordinary
//     accesses makes the kernel allocate in that cache and pay for evicting whatever dirty lines
//     the kernel before it left there (measured at 200 M weights: the forward kernel took 0.85 ms
//     after an all-hinted kernel, 0.88 ms after the backward kernel and 0.92 ms after an ordinary
//     element-wise kernel; with all accesses hinted 0.83 ms after any of them).
// With GEN the kernels draw eps in registers from a counter-based generator instead of
// reading it (4 bytes per item less in each direction, at the price of integer and
// transcendental arithmetic): forward and backward regenerate identical values.
// The forward kernels are in forward.hip, the backward kernels in backward.hip; this file holds the plan,
// the draw on its own and the measurement aids.
#include <new>

#include "sample_layer.h"

namespace {

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

// The same for the stream counts of workloads with many samples (C3: 18 read + 16 write streams forward, 34 + 2
// backward), which no thread can hold in registers at once: like the kernels, a thread walks the read streams
// four at a time, adding them up, and then writes the sum to every write stream, one after the other.
// AL = false: the streams only keep dword alignment (a pitch that is no multiple of 16 bytes, as the rows of a sample
// matrix with an odd leading dimension): the same 16-byte accesses from dword addresses.
template <bool AL>
__global__ void __launch_bounds__(kBlock)
hot_probe_many_streams_kernel(const float *__restrict__ arena, long stream_floats, int reads, int writes, long n_vec)
{
    constexpr int kPer = 4;
    const long base = (long)blockIdx.x * (kBlock * kPer) + threadIdx.x;
    f4 acc[kPer];
#pragma unroll
    for (int c = 0; c < kPer; ++c) acc[c] = f4{0.0f, 0.0f, 0.0f, 0.0f};
    float *out = const_cast<float *>(arena) + (size_t)reads * (size_t)stream_floats;
    if (base + (long)(kPer - 1) * kBlock < n_vec) {       // a whole tile (uniform over the workgroup)
        int r = 0;
        for (; r + 4 <= reads; r += 4) {
            f4 v[4][kPer];
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int c = 0; c < kPer; ++c)
                    v[u][c] = load4<AL, true>(arena + (size_t)(r + u) * (size_t)stream_floats + 4 * (base + (long)c * kBlock));
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int c = 0; c < kPer; ++c) acc[c] += v[u][c];
        }
        for (; r < reads; ++r) {
            f4 v[kPer];
#pragma unroll
            for (int c = 0; c < kPer; ++c)
                v[c] = load4<AL, true>(arena + (size_t)r * (size_t)stream_floats + 4 * (base + (long)c * kBlock));
#pragma unroll
            for (int c = 0; c < kPer; ++c) acc[c] += v[c];
        }
        for (int w = 0; w < writes; ++w)
#pragma unroll
            for (int c = 0; c < kPer; ++c)
                store4<AL, true>(out + (size_t)w * (size_t)stream_floats + 4 * (base + (long)c * kBlock), acc[c]);
    } else {
        for (int c = 0; c < kPer; ++c) {
            const long at = base + (long)c * kBlock;
            if (at >= n_vec) continue;
            f4 sum = f4{0.0f, 0.0f, 0.0f, 0.0f};
            for (int r = 0; r < reads; ++r) sum += load4<AL, false>(arena + (size_t)r * (size_t)stream_floats + 4 * at);
            for (int w = 0; w < writes; ++w) store4<AL, false>(out + (size_t)w * (size_t)stream_floats + 4 * at, sum);
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

namespace {

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
    case HOT_ERANGE: return "problem larger than the fixed capacity of this no-allocation entry point";
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
    if (!valid_desc(d)) return HOT_EINVAL;
    int n_dev = 0;
    if (hipError_t e = hipGetDeviceCount(&n_dev); e != hipSuccess) return hot_detail::note_hip(e);
    if (d.device < 0 || d.device >= n_dev) return HOT_EINVAL;

    hot_plan *p = new (std::nothrow) hot_plan();
    if (!p) return HOT_ENOMEM;
    p->d = d;
    set_scaling(*p);
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
    default_launches(*p);
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
    if (!arena || !aligned16(arena) || stream_bytes < 16 || (stream_bytes & 3)) return HOT_EINVAL;
    if (reads < 1 || reads > 64 || writes < 0 || writes > 64) return HOT_EINVAL;
    const long n_vec = stream_bytes / 16;       // (a last partial quad of every stream is left alone)
    const long blocks = (n_vec + kBlock * 4 - 1) / (kBlock * 4);
    if (blocks > 0x7fffffffL) return HOT_EINVAL;
    const bool skewed = (stream_bytes & 15) != 0;
    if (reads > 6 || writes > 2 || skewed) {      // more streams than a thread holds at once, or streams off the 16-byte grid: the looping kernel
        if (writes == 0) return HOT_EINVAL;
        const dim3 grid((unsigned)blocks), block(kBlock);
        hipStream_t s = static_cast<hipStream_t>(stream);
        if (skewed) hot_probe_many_streams_kernel<false><<<grid, block, 0, s>>>(static_cast<const float *>(arena), stream_bytes / 4, reads, writes, n_vec);
        else hot_probe_many_streams_kernel<true><<<grid, block, 0, s>>>(static_cast<const float *>(arena), stream_bytes / 4, reads, writes, n_vec);
        return hot_detail::note_hip(hipGetLastError());
    }
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
