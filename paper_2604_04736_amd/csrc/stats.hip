// libhot: predictive statistics over the Monte-Carlo samples (arxiv 2604.04736: the S
// predictions of a step are aggregated into a mean, the model's output, and a standard
// deviation, its uncertainty; with the samples spread over GPUs the exact variant the paper
// mentions after Algorithm 2 needs two numbers per output from every GPU).
//
//   hot_stats_local   this GPU's rows yhat[S_loc, ld] -> per output (mean, M2 = sum of squared
//                     deviations from that mean), fp64: the two numbers to communicate;
//   hot_stats_merge   the partials of all GPUs -> mean and standard deviation over all samples;
//   hot_stats_whole   both steps in one pass when one GPU holds all samples.
//
// Both are streaming column reductions, bound by HBM (4 + 16/S_loc bytes per prediction for
// the local pass), laid out like the backward kernel: a thread owns four consecutive
// outputs, rows are read with 16-byte loads, sums are carried in fp64.
#include <hip/hip_runtime.h>

#include "hot.h"
#include "vec.h"

namespace {

constexpr int kBlock = 256;
constexpr int kRowsInFlight = 4;
constexpr int kMaxParts = 64;

// (mean, M2) of one column from the shifted sums  sd = sum (y - y0),  sq = sum (y - y0)^2  over
// its n rows, y0 the first row: mean = y0 + sd/n, M2 = sq - sd^2/n.  Shifting by a sample keeps
// the subtraction well conditioned (sq <= n * M2), and every difference y - y0 is exact in fp64.
__device__ __forceinline__ void finish_column(double y0, double sd, double sq, double n, double &mean, double &m2)
{
    const double md = sd / n;
    mean = y0 + md;
    const double v = fma(-sd, md, sq);
    m2 = v > 0.0 ? v : 0.0;
}

// FINAL = false: the two fp64 partials (mean, M2) per output.  FINAL = true (all samples are on this
// GPU, nothing to merge): mean and standard deviation sqrt(M2 / divisor) as fp32, in the same pass.
template <bool FINAL>
__device__ __forceinline__ void put_column(long i, double mean, double m2, double divisor, void *out_a, void *out_b)
{
    if constexpr (FINAL) {
        static_cast<float *>(out_a)[i] = (float)mean;
        static_cast<float *>(out_b)[i] = (float)sqrt(m2 / divisor);
    } else {
        static_cast<double *>(out_a)[i] = mean;
        static_cast<double *>(out_b)[i] = m2;
    }
}

// Four finished columns at once: 16-byte stores (the fp32 final results; the fp64 partials as two
// 16-byte halves each).
template <bool FINAL>
__device__ __forceinline__ void put_quad(long col, const double (&mean)[4], const double (&m2)[4], double divisor,
                                         void *out_a, void *out_b)
{
    if constexpr (FINAL) {
        f4 a, b;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            a[j] = (float)mean[j];
            b[j] = (float)sqrt(m2[j] / divisor);
        }
        store4<false, false>(static_cast<float *>(out_a) + col, a);
        store4<false, false>(static_cast<float *>(out_b) + col, b);
    } else {
        typedef double d2 __attribute__((ext_vector_type(2)));
        typedef d2 d2u __attribute__((aligned(8)));
        d2u *pa = reinterpret_cast<d2u *>(static_cast<double *>(out_a) + col);
        d2u *pb = reinterpret_cast<d2u *>(static_cast<double *>(out_b) + col);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            pa[h] = d2{mean[2 * h], mean[2 * h + 1]};
            pb[h] = d2{m2[2 * h], m2[2 * h + 1]};
        }
    }
}

// NT (arrays larger than the memory-side cache): the rows are read with the non-temporal hint.  Which
// of the remaining accesses carry it was measured on MI355X at 16 x 2^24 predictions, the kernel
// alternating with a copy kernel: the outputs are best stored plainly in both variants (hinted stores
// cost 5-10 %), the first row is best hinted in the partial-sums variant (0.224 against 0.245 ms) and
// plain in the one-pass variant (0.199 against 0.212 ms); both then run at 6.0-6.1 TB/s.
template <bool ALIGNED, bool FINAL, bool NT>
__global__ void __launch_bounds__(kBlock)
hot_stats_local_kernel(long m, long ld, int s_loc, double divisor, const float *__restrict__ y, void *__restrict__ mean,
                       void *__restrict__ m2)
{
    const long n_chunks = (m + 3) / 4;
    const double n = (double)s_loc;
    for (long chunk = (long)blockIdx.x * kBlock + threadIdx.x; chunk < n_chunks; chunk += (long)gridDim.x * kBlock) {
        const long col = chunk * 4;
        if (col + 4 <= m) {
            const f4 first = load4<ALIGNED, NT && !FINAL>(y + col);
            double sd[4] = {0.0, 0.0, 0.0, 0.0}, sq[4] = {0.0, 0.0, 0.0, 0.0};
            int s = 1;
            for (; s + kRowsInFlight <= s_loc; s += kRowsInFlight) {
                f4 v[kRowsInFlight];
#pragma unroll
                for (int u = 0; u < kRowsInFlight; ++u) v[u] = load4<ALIGNED, NT>(y + (size_t)(s + u) * (size_t)ld + col);
#pragma unroll
                for (int u = 0; u < kRowsInFlight; ++u)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const double d = (double)v[u][j] - (double)first[j];
                        sd[j] += d;
                        sq[j] = fma(d, d, sq[j]);
                    }
            }
            for (; s < s_loc; ++s) {
                const f4 v = load4<ALIGNED, NT>(y + (size_t)s * (size_t)ld + col);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const double d = (double)v[j] - (double)first[j];
                    sd[j] += d;
                    sq[j] = fma(d, d, sq[j]);
                }
            }
            double a[4], b[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) finish_column((double)first[j], sd[j], sq[j], n, a[j], b[j]);
            put_quad<FINAL>(col, a, b, divisor, mean, m2);
        } else {
            for (long i = col; i < m; ++i) {
                const double y0 = (double)y[i];
                double sd = 0.0, sq = 0.0;
                for (int s = 1; s < s_loc; ++s) {
                    const double d = (double)y[(size_t)s * (size_t)ld + (size_t)i] - y0;
                    sd += d;
                    sq = fma(d, d, sq);
                }
                double a, b;
                finish_column(y0, sd, sq, n, a, b);
                put_column<FINAL>(i, a, b, divisor, mean, m2);
            }
        }
    }
}

struct Counts {
    int parts;
    double n[kMaxParts];   // samples behind each partial
    double total, divisor; // sum of n, and total - ddof
};

// Pooled statistics of `parts` groups (Chan, Golub, LeVeque 1979, applied to all groups at
// once): mean = sum n_p mean_p / n;  M2 = sum [ M2_p + n_p (mean_p - mean)^2 ].  One thread per
// output; the partials are read twice (they are small and stay in cache).
__global__ void __launch_bounds__(kBlock)
hot_stats_merge_kernel(long m, long ld, Counts c, const double *__restrict__ means, const double *__restrict__ m2s,
                       float *__restrict__ mean_out, float *__restrict__ std_out)
{
    for (long i = (long)blockIdx.x * kBlock + threadIdx.x; i < m; i += (long)gridDim.x * kBlock) {
        // shift by the first group's mean so that the weighted sum does not cancel
        const double m0 = means[i];
        double wsum = 0.0;
        for (int p = 1; p < c.parts; ++p) wsum = fma(c.n[p], means[(size_t)p * (size_t)ld + (size_t)i] - m0, wsum);
        const double shift = wsum / c.total;      // pooled mean - m0
        double ss = 0.0;
        for (int p = 0; p < c.parts; ++p) {
            const double d = (means[(size_t)p * (size_t)ld + (size_t)i] - m0) - shift;
            ss += fma(c.n[p] * d, d, m2s[(size_t)p * (size_t)ld + (size_t)i]);
        }
        mean_out[i] = (float)(m0 + shift);
        std_out[i] = (float)sqrt(ss / c.divisor);
    }
}

// Whether the prediction array is larger than the 256 MiB memory-side cache (then it is streamed with
// non-temporal hints; a smaller one is left to the caches, where the network has just written it).
bool exceeds_cache(int rows, long ld) { return (double)rows * (double)ld * 4.0 >= 256.0 * 1048576.0; }

unsigned blocks_for(long work_items)
{
    long b = (work_items + kBlock - 1) / kBlock;
    if (b > 65536) b = 65536;
    if (b < 1) b = 1;
    return (unsigned)b;
}

}  // namespace

extern "C" {

int hot_stats_local(const float *yhat, int64_t m, int64_t ld, int32_t s_local, double *mean, double *m2, void *stream)
{
    if (!yhat || !mean || !m2 || m < 1 || ld < m || s_local < 1) return HOT_EINVAL;
    if (!aligned4(yhat) || (reinterpret_cast<uintptr_t>(mean) & 7u) || (reinterpret_cast<uintptr_t>(m2) & 7u))
        return HOT_EINVAL;
    if (ld > (INT64_MAX / 4) / s_local) return HOT_EINVAL;
    const bool al = aligned16(yhat) && (ld % 4 == 0);
    const bool nt = exceeds_cache(s_local, ld);
    const dim3 grid(blocks_for((m + 3) / 4)), block(kBlock);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (al && nt) hot_stats_local_kernel<true, false, true><<<grid, block, 0, s>>>(m, ld, s_local, 1.0, yhat, mean, m2);
    else if (al) hot_stats_local_kernel<true, false, false><<<grid, block, 0, s>>>(m, ld, s_local, 1.0, yhat, mean, m2);
    else if (nt) hot_stats_local_kernel<false, false, true><<<grid, block, 0, s>>>(m, ld, s_local, 1.0, yhat, mean, m2);
    else hot_stats_local_kernel<false, false, false><<<grid, block, 0, s>>>(m, ld, s_local, 1.0, yhat, mean, m2);
    return hot_detail::note_hip(hipGetLastError());
}

int hot_stats_whole(const float *yhat, int64_t m, int64_t ld, int32_t s, int32_t ddof, float *mean_out, float *std_out,
                    void *stream)
{
    if (!yhat || !mean_out || !std_out || m < 1 || ld < m || s < 1 || (ddof != 0 && ddof != 1)) return HOT_EINVAL;
    if (!aligned4(yhat) || !aligned4(mean_out) || !aligned4(std_out)) return HOT_EINVAL;
    if (ld > (INT64_MAX / 4) / s) return HOT_EINVAL;
    const bool al = aligned16(yhat) && (ld % 4 == 0);
    const double divisor = (double)s - (double)ddof;     // 0 for one sample with ddof = 1: std is then NaN, as defined
    const dim3 grid(blocks_for((m + 3) / 4)), block(kBlock);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool nt = exceeds_cache(s, ld);
    if (al && nt) hot_stats_local_kernel<true, true, true><<<grid, block, 0, st>>>(m, ld, s, divisor, yhat, mean_out, std_out);
    else if (al) hot_stats_local_kernel<true, true, false><<<grid, block, 0, st>>>(m, ld, s, divisor, yhat, mean_out, std_out);
    else if (nt) hot_stats_local_kernel<false, true, true><<<grid, block, 0, st>>>(m, ld, s, divisor, yhat, mean_out, std_out);
    else hot_stats_local_kernel<false, true, false><<<grid, block, 0, st>>>(m, ld, s, divisor, yhat, mean_out, std_out);
    return hot_detail::note_hip(hipGetLastError());
}

int hot_stats_merge(const double *means, const double *m2s, const int32_t *counts, int32_t parts, int64_t m,
                    int64_t ld, int32_t ddof, float *mean_out, float *std_out, void *stream)
{
    if (!means || !m2s || !counts || !mean_out || !std_out) return HOT_EINVAL;
    if (parts < 1 || parts > kMaxParts || m < 1 || ld < m || (ddof != 0 && ddof != 1)) return HOT_EINVAL;
    if ((reinterpret_cast<uintptr_t>(means) & 7u) || (reinterpret_cast<uintptr_t>(m2s) & 7u) || !aligned4(mean_out) ||
        !aligned4(std_out))
        return HOT_EINVAL;
    Counts c;
    c.parts = parts;
    c.total = 0.0;
    for (int p = 0; p < kMaxParts; ++p) c.n[p] = 0.0;
    for (int p = 0; p < parts; ++p) {
        if (counts[p] < 1) return HOT_EINVAL;
        c.n[p] = (double)counts[p];
        c.total += c.n[p];
    }
    c.divisor = c.total - (double)ddof;      // 0 for one sample with ddof = 1: std is then NaN or inf, as defined
    const dim3 grid(blocks_for(m)), block(kBlock);
    hot_stats_merge_kernel<<<grid, block, 0, static_cast<hipStream_t>(stream)>>>(m, ld, c, means, m2s, mean_out, std_out);
    return hot_detail::note_hip(hipGetLastError());
}

}  // extern "C"
