// libhot: one sampled Bayesian linear layer with the weight draw fused into the contraction
// (arxiv 2604.04736, Algorithm 1 / 2: reparameterisation line followed by ForwardPass, for the
// case that the layer is a Linear):
//     y_s = x (mu_W + sigma_W (.) eps_s)^T + (mu_b + sigma_b (.) eps_s^b)        for every local sample s
// The sampled weights never exist in memory: a wave draws the eps of a 16-output x 32-input tile
// in registers (Philox + Box-Muller on the vector ALU), forms w = fma(sigma, eps, mu) and feeds
// it straight to the matrix cores as the B operand of v_mfma_f32_16x16x4_f32, while the minibatch
// x is the A operand.  mu_W and sigma_W are read once per block of rows and sample chunk; eps for
// weight (o, k) is the draw of flat parameter index weight_offset + o*K + k, i.e. exactly the value
// hot_forward_rng would put into w for the same hot_rng.
//
// Lane roles inside a wave (MFMA 16x16x4: lane l supplies A[m = l%16][kk = l/16] and
// B[kk = l/16][n = l%16], and receives D[4*(l/16) + r][l%16] in register r): lane (j, n) owns the
// eight consecutive inputs k = kb + 8j .. kb + 8j + 7 of output column n (two draws of four), and,
// as an A lane, the same eight inputs of row m = n of x.  MFMA number i of a 32-input block then
// takes element i of every lane's eight: the contraction index is merely enumerated in a different
// order, and every 128-byte line of mu_W, sigma_W and x is consumed by one iteration.
#include <hip/hip_runtime.h>

#include "hot.h"
#include "vec.h"
#include "draw.h"

namespace {

constexpr int kMaxWaves = 16;  // waves of a workgroup; they split the input dimension among themselves
constexpr int kColsPerWave = 16;
constexpr int kRowsPerTile = 16;
constexpr int kInputsPerIter = 32;

// More row tiles need more registers per lane: such workgroups are limited to fewer waves.
constexpr int max_waves(int rb) { return rb >= 4 ? 4 : (rb >= 2 ? 8 : kMaxWaves); }

// Four samples' accumulators are live together only where the register file holds them without spills.
constexpr bool four_samples_fit(int rb, bool per_sample_x) { return rb == 2 || (rb == 1 && !per_sample_x); }

struct LinearArgs {
    long rows, in_features, out_features, ldx;
    long x_sample_stride;   // floats between the inputs of consecutive samples (XS kernels only)
    int s_loc;
    long weight_quad0;   // (weight_offset) / 4
    long bias_quad0;     // (bias_offset) / 4
    const float *x, *mu_w, *sigma_w, *mu_b, *sigma_b;
    float *y;
    Rng rng;
};

// A workgroup owns 16 output columns and 16*RB rows; its waves take the 32-input blocks round-robin
// and their partial tiles are added through LDS in wave order (deterministic).  XS: every sample has
// its own input (a layer inside the network); its rows are then loaded per sample, right before
// that sample's draw, whose arithmetic covers their latency.
template <int RB, int ST, bool XS>
__global__ void __launch_bounds__(64 * max_waves(RB), RB >= 4 ? 2 : 1)
hot_linear_forward_kernel(LinearArgs a)
{
    extern __shared__ float partial[];   // [waves - 1][ST * RB * 4][64]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, waves = blockDim.x >> 6;
    const int n = lane & 15, j = lane >> 4;
    const long K = a.in_features, O = a.out_features, R = a.rows;
    const long o = (long)blockIdx.x * kColsPerWave + n;
    const long r0 = (long)blockIdx.y * (kRowsPerTile * RB);
    const bool o_ok = o < O;
    const float *mu_row = a.mu_w + (o_ok ? o : 0) * K;
    const float *sg_row = a.sigma_w + (o_ok ? o : 0) * K;
    const long quad_row = a.weight_quad0 + ((o_ok ? o : 0) * K >> 2);

    for (int s0 = 0; s0 < a.s_loc; s0 += ST) {
        f4 acc[ST][RB];
#pragma unroll
        for (int st = 0; st < ST; ++st)
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) acc[st][rb] = f4{0.0f, 0.0f, 0.0f, 0.0f};

        for (long kb = (long)wave * kInputsPerIter; kb < K; kb += (long)waves * kInputsPerIter) {
            const long k = kb + 8 * j;
            f4 m4[2], sd4[2], xa[RB][2];
            bool ok[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                ok[h] = o_ok && (k + 4 * h < K);
                m4[h] = ok[h] ? load4<true, false>(mu_row + k + 4 * h) : f4{0.0f, 0.0f, 0.0f, 0.0f};
                sd4[h] = ok[h] ? load4<true, false>(sg_row + k + 4 * h) : f4{0.0f, 0.0f, 0.0f, 0.0f};
                if constexpr (!XS) {
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb) {
                        const long row = r0 + kRowsPerTile * rb + n;
                        xa[rb][h] = (row < R && k + 4 * h < K) ? load4<true, false>(a.x + row * a.ldx + k + 4 * h)
                                                                : f4{0.0f, 0.0f, 0.0f, 0.0f};
                    }
                }
            }
#pragma unroll
            for (int st = 0; st < ST; ++st) {
                if (s0 + st < a.s_loc) {          // uniform over the wave
                    if constexpr (XS) {
                        const float *xs = a.x + (size_t)(s0 + st) * (size_t)a.x_sample_stride;
#pragma unroll
                        for (int h = 0; h < 2; ++h)
#pragma unroll
                            for (int rb = 0; rb < RB; ++rb) {
                                const long row = r0 + kRowsPerTile * rb + n;
                                xa[rb][h] = (row < R && k + 4 * h < K) ? load4<true, false>(xs + row * a.ldx + k + 4 * h)
                                                                        : f4{0.0f, 0.0f, 0.0f, 0.0f};
                            }
                    }
                    f4 w4[2];
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        w4[h] = f4{0.0f, 0.0f, 0.0f, 0.0f};
                        if (ok[h]) {
                            const f4 e = eps_quad(quad_row + ((k + 4 * h) >> 2), s0 + st, a.rng);
#pragma unroll
                            for (int c = 0; c < 4; ++c) w4[h][c] = __builtin_fmaf(sd4[h][c], e[c], m4[h][c]);
                        }
                    }
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int c = 0; c < 4; ++c)
#pragma unroll
                            for (int rb = 0; rb < RB; ++rb)
                                acc[st][rb] = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[rb][h][c], w4[h][c], acc[st][rb], 0, 0, 0);
                }
            }
        }

        if (waves > 1) {
            __syncthreads();            // the previous chunk's readers are done with the buffer
            if (wave > 0) {
#pragma unroll
                for (int st = 0; st < ST; ++st)
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            partial[((wave - 1) * (ST * RB * 4) + (st * RB + rb) * 4 + r) * 64 + lane] = acc[st][rb][r];
            }
            __syncthreads();
            if (wave == 0) {
                for (int v = 1; v < waves; ++v)
#pragma unroll
                    for (int st = 0; st < ST; ++st)
#pragma unroll
                        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                            for (int r = 0; r < 4; ++r)
                                acc[st][rb][r] += partial[((v - 1) * (ST * RB * 4) + (st * RB + rb) * 4 + r) * 64 + lane];
            }
        }
        if (wave != 0) continue;        // wave 0 holds the complete tile and writes it

#pragma unroll
        for (int st = 0; st < ST; ++st) {
            if (s0 + st < a.s_loc) {
                float bias = 0.0f;
                if (a.mu_b && o_ok) {
                    const f4 e = eps_quad(a.bias_quad0 + (o >> 2), s0 + st, a.rng);
                    const int c = (int)(o & 3);
                    const float ev = c == 0 ? e[0] : (c == 1 ? e[1] : (c == 2 ? e[2] : e[3]));
                    bias = __builtin_fmaf(a.sigma_b[o], ev, a.mu_b[o]);
                }
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const long row = r0 + kRowsPerTile * rb + 4 * j + r;
                        if (row < R && o_ok) a.y[((size_t)(s0 + st) * (size_t)R + (size_t)row) * (size_t)O + (size_t)o] = acc[st][rb][r] + bias;
                    }
            }
        }
    }
}

template <int RB, bool XS>
void linear_go_st(int st, dim3 grid, int waves, hipStream_t s, const LinearArgs &a)
{
    const dim3 block(64 * waves);
    const size_t lds = waves > 1 ? (size_t)(waves - 1) * (size_t)(st * RB * 4) * 64 * sizeof(float) : 0;
    if constexpr (four_samples_fit(RB, XS)) {
        if (st == 4) { hot_linear_forward_kernel<RB, 4, XS><<<grid, block, lds, s>>>(a); return; }
    }
    if (st >= 2) hot_linear_forward_kernel<RB, 2, XS><<<grid, block, lds, s>>>(a);
    else hot_linear_forward_kernel<RB, 1, XS><<<grid, block, lds, s>>>(a);
}

template <int RB>
void linear_go(int st, dim3 grid, int waves, hipStream_t s, const LinearArgs &a)
{
    if (a.x_sample_stride != 0) linear_go_st<RB, true>(st, grid, waves, s, a);
    else linear_go_st<RB, false>(st, grid, waves, s, a);
}

}  // namespace

extern "C" {

int hot_linear_forward_rng(const hot_linear_desc *d, const hot_rng *rng, const float *x, const float *mu_w,
                           const float *sigma_w, const float *mu_b, const float *sigma_b, float *y, void *stream)
{
    if (!d || !x || !mu_w || !sigma_w || !y) return HOT_EINVAL;
    if ((mu_b == nullptr) != (sigma_b == nullptr)) return HOT_EINVAL;
    if (d->rows < 1 || d->in_features < 4 || (d->in_features & 3) || d->out_features < 1 || d->s_local < 1) return HOT_EINVAL;
    if (d->ldx < d->in_features || (d->ldx & 3) || d->weight_offset < 0 || (d->weight_offset & 3)) return HOT_EINVAL;
    if (d->reserved != 0 || d->x_sample_stride < 0 || (d->x_sample_stride & 3)) return HOT_EINVAL;
    if (d->x_sample_stride != 0 && (d->rows > INT64_MAX / d->ldx || d->x_sample_stride < d->rows * d->ldx ||
                                    d->x_sample_stride > INT64_MAX / 4 / d->s_local))
        return HOT_EINVAL;
    if (mu_b && (d->bias_offset < 0 || (d->bias_offset & 3))) return HOT_EINVAL;
    if (!aligned16(x) || !aligned16(mu_w) || !aligned16(sigma_w) || !aligned4(y)) return HOT_EINVAL;
    if (mu_b && (!aligned4(mu_b) || !aligned4(sigma_b))) return HOT_EINVAL;
    if (d->out_features > (INT64_MAX / 8) / d->in_features) return HOT_EINVAL;
    Rng r;
    if (!make_rng(rng, d->s_local, r)) return HOT_EINVAL;

    LinearArgs a;
    a.rows = d->rows;
    a.in_features = d->in_features;
    a.out_features = d->out_features;
    a.ldx = d->ldx;
    a.x_sample_stride = d->x_sample_stride;
    a.s_loc = d->s_local;
    a.weight_quad0 = d->weight_offset >> 2;
    a.bias_quad0 = mu_b ? d->bias_offset >> 2 : 0;
    a.x = x;
    a.mu_w = mu_w;
    a.sigma_w = sigma_w;
    a.mu_b = mu_b;
    a.sigma_b = sigma_b;
    a.y = y;
    a.rng = r;

    // rows per workgroup: 16, 32 or 64 (one, two or four MFMA row tiles share every drawn weight)
    const int rb = d->rows > 32 ? 4 : (d->rows > 16 ? 2 : 1);
    // samples whose accumulators are live together (they share the loads of mu_W, sigma_W and x)
    const int st = d->s_local >= 4 && four_samples_fit(rb, d->x_sample_stride != 0) ? 4 : (d->s_local >= 2 ? 2 : 1);
    const long gx = (d->out_features + kColsPerWave - 1) / kColsPerWave;
    const long gy = (d->rows + kRowsPerTile * rb - 1) / (kRowsPerTile * rb);
    if (gx > 0x7fffffffL || gy > 65535) return HOT_EINVAL;
    // waves per workgroup: enough to give every SIMD of the chip several waves, bounded by the
    // number of 32-input blocks and by 64 KiB of LDS for the partial tiles
    const long k_blocks = (d->in_features + kInputsPerIter - 1) / kInputsPerIter;
    int waves = 1;
    while (waves < max_waves(rb) && gx * gy * waves < 8192 && 2L * waves <= k_blocks &&
           (size_t)(2 * waves - 1) * (size_t)(st * rb * 4) * 64 * sizeof(float) <= 65536)
        waves *= 2;
    const dim3 grid((unsigned)gx, (unsigned)gy);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (rb == 4) linear_go<4>(st, grid, waves, s, a);
    else if (rb == 2) linear_go<2>(st, grid, waves, s, a);
    else linear_go<1>(st, grid, waves, s, a);
    return hot_detail::note_hip(hipGetLastError());
}

}  // extern "C"
