// Pieces shared by the translation units of the sample layer (hot.hip, forward.hip, backward.hip):
// constants, the eps accessors, the KL addend, the workgroup sum, the KL finish kernel, the plan and the
// host helpers around it.  gfx950 only.
#ifndef HOT_SAMPLE_LAYER_H
#define HOT_SAMPLE_LAYER_H

#include <hip/hip_runtime.h>

#include "hot.h"
#include "vec.h"
#include "draw.h"
#include "adam.h"

// What hot_create returns: the description, the scaling constants g and k derived from it, the plan's own
// device scratch and the launch geometry of the four kernels.
struct hot_plan {
    hot_desc d;
    double g, k;
    double *partials;   // kMaxGrid fp64 KL partial sums, one per forward workgroup, then the arrival counter
    hot_launch cfg[4];  // indexed by HOT_KERNEL_*
    int last_hip;
};

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

// The same inside a column tile that begins at column `begin` and holds `bytes` bytes of whole quads: read through
// a range-checked window (zeros beyond it), or drawn.  off = byte offset of the quad from the tile's first column.
template <bool NT, bool GEN>
__device__ __forceinline__ f4 eps4_window(const float *eps, long ld, int s, long begin, unsigned bytes, unsigned off, const Rng &rng)
{
    if constexpr (GEN) return eps_quad((begin + (off >> 2)) >> 2, s, rng);
    else return window_load4<NT>(window(eps + (size_t)s * (size_t)ld + begin, bytes), off);
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

// Adds the per-workgroup KL partials in a fixed order and applies the factor 1/2 of the
// prior-matching line.  One workgroup; runs right after the forward kernel on its stream.
__global__ void __launch_bounds__(kFinishBlock) __attribute__((unused))
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

inline int fail_hip(hot_plan *p, hipError_t e)
{
    if (p) p->last_hip = (int)e;
    return HOT_EHIP;
}

inline int pick_unroll(int want, int s_loc)
{
    int u = want >= 4 ? 4 : (want >= 2 ? 2 : 1);
    while (u > 1 && u > s_loc) u >>= 1;
    return u;
}

inline bool valid_kernel(int kernel) { return kernel >= HOT_KERNEL_FORWARD && kernel <= HOT_KERNEL_BACKWARD_RNG; }

inline bool valid_launch(const hot_launch &c)
{
    auto one_of = [](int v) { return v == 0 || v == 1 || v == 2 || v == 4; };
    return c.grid_blocks >= 0 && c.grid_blocks <= kMaxGrid && one_of(c.chunks) && one_of(c.unroll) &&
           (c.nontemporal == 0 || c.nontemporal == 1);
}

// What every entry point requires of a description (device aside).
inline bool valid_desc(const hot_desc &d)
{
    if (d.n_weights < 1 || d.ld < d.n_weights || d.s_local < 1 || d.s_total < d.s_local) return false;
    if (!(d.dataset_size > 0.0) || !(d.dataset_size < 1.0 / 0.0)) return false;
    if (d.flags != HOT_REDUCE_SUM && d.flags != HOT_REDUCE_MEAN && d.flags != HOT_REDUCE_NONE) return false;
    // element offsets (s_local - 1) * ld + n_weights must fit in 63 bits
    return d.ld <= (INT64_MAX / 4) / d.s_local;
}

// g and k of the gradient and averaging lines of Algorithm 2 for the plan's reduce convention.
inline void set_scaling(hot_plan &p)
{
    const hot_desc &d = p.d;
    if (d.flags == HOT_REDUCE_NONE) {
        p.g = 1.0;
        p.k = 1.0 / d.dataset_size;
    } else if (d.flags == HOT_REDUCE_MEAN) {
        p.g = 1.0 / (double)d.s_local;
        p.k = 1.0 / d.dataset_size;
    } else {
        p.g = 1.0 / (double)d.s_total;
        p.k = (double)d.s_local / ((double)d.s_total * d.dataset_size);
    }
}

// Largest number of 16-byte chunks per thread (4, 2, 1) whose column tiles number at least 512 and fill their
// rounds of 256 (one per compute unit) to 90 %; one chunk if none does.
inline int balanced_chunks(long n)
{
    for (int c = 4; c > 1; c >>= 1) {
        const long tile = (long)kBlock * 4 * c;
        const long tiles = (n + tile - 1) / tile;
        const long rounds = (tiles + 255) / 256;
        if (tiles >= 512 && tiles * 10 >= rounds * 256 * 9) return c;
    }
    return 1;
}

// The default launch geometry of the four kernels for the plan's description.
inline void default_launches(hot_plan &p)
{
    // Defaults from launch-shape sweeps on MI355X, each kernel timed with the other one running in
    // between (timing a kernel back to back with itself lets part of its input stay in the 256 MiB
    // memory-side cache and favours shapes that lose in a real step): four chunks per thread for
    // the array kernels, single rows in flight forward, as many rows as there are (up to four)
    // backward.
    // Non-temporal hints at every size: in training the network runs between the two calls and leaves the
    // memory-side cache full of its own, partly dirty, lines; a kernel that allocates there (plain accesses)
    // then pays for their write-back and finds none of its own data.  Measured with an unrelated 512 MiB
    // element-wise kernel before each call, hinted accesses are 10-45 % faster from 256 K weights up to the
    // largest sizes (2.7 M weights x 4 samples: forward 39 -> 26 us, backward 48 -> 27 us); with the two calls
    // back to back and nothing else on the GPU, plain accesses are 0-15 % faster while all arrays fit in the
    // cache together and up to 30 % slower once they do not.
    const hot_desc &d = p.d;
    hot_launch &f = p.cfg[HOT_KERNEL_FORWARD], &b = p.cfg[HOT_KERNEL_BACKWARD];
    f.grid_blocks = b.grid_blocks = kMaxGrid;
    // Chunks per thread: four, unless that leaves fewer than two workgroups per compute unit or a last round of
    // workgroups that is mostly empty (2.7 M weights are 658 tiles of 4096: 2.6 rounds of 256); then two, then one
    // (2.7 M weights x 4 samples with other work between the calls: backward 28.4 us with four chunks, 26.5 with one).
    f.chunks = b.chunks = balanced_chunks(d.n_weights);
    f.unroll = 1;
    b.unroll = pick_unroll(4, d.s_local);
    f.nontemporal = b.nontemporal = 1;
    // With fewer than four samples the four-chunk backward kernels are fat (over 200 registers per lane,
    // two workgroups per compute unit) and short: below 16 M weights their last, partly filled round of
    // workgroups costs 5-10 %, which one chunk per thread avoids.
    const bool few_tiles = d.n_weights < (16L << 20);
    if (d.s_local < 4 && few_tiles) b.chunks = 1;
    // The drawing variants have no eps loads to keep in flight.  Forward: as above up to seven samples;
    // from eight on one chunk per thread (38 registers, eight waves per SIMD) hides the generator's
    // latencies better than four independent chains in five waves (10-20 % at 8 M to 25 M weights).
    // Backward: single rows in flight at every size (two rows of draws in flight cost registers and with them waves:
    // 209 M weights x 2 samples 1.07 ms against 0.81, 64 M x 3 0.38 against 0.30, 20 M x 8 0.178 against 0.169); four
    // chunks per thread from 16 M weights on, below that two from four samples on (6.3 M x 16, 7.7 M x 13), else one.
    hot_launch &fr = p.cfg[HOT_KERNEL_FORWARD_RNG], &br = p.cfg[HOT_KERNEL_BACKWARD_RNG];
    fr = f;
    if (d.s_local >= 8) fr.chunks = 1;
    br = b;
    br.chunks = few_tiles ? (d.s_local >= 4 ? 2 : 1) : 4;
    if (br.chunks > f.chunks) br.chunks = f.chunks;      // (f.chunks: what the number of tiles allows)
    br.unroll = 1;
}

// How the N columns are cut into tiles, one workgroup each (capped by the configured bound, beyond which workgroups
// stride over the tiles): tiles of chunks * 1024 columns, the last one narrower.  The kernels take any width that is
// a multiple of 64 columns (narrower tiles go through range-checked windows, see vec.h).  Cutting the width down so
// that every compute unit holds the same number of equally wide tiles was built and measured (13 samples, 6.3 M to
// 13 M weights, other work between the calls): no gain over full tiles within +-3 %; what does vary by 5 % from one
// N to the next is not the partly filled last round of workgroups.
struct Tiling {
    long width;       // columns per tile
    unsigned grid;    // workgroups
};

inline Tiling tiling_for(long n, const hot_launch &c)
{
    const long width = (long)kBlock * 4 * c.chunks;
    const long tiles = (n + width - 1) / width;
    return Tiling{width, (unsigned)(tiles < c.grid_blocks ? tiles : c.grid_blocks)};
}

}  // namespace

#endif  // HOT_SAMPLE_LAYER_H
