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
//
// Kernels of this file, by regime:
//   forward   hot_linear_forward_kernel        up to a few hundred rows: every wave draws what it multiplies
//             hot_linear_forward_rows_kernel   from 256 rows: four waves x 64 rows share every draw through LDS
//             hot_linear_slab_kernel           from 256 rows on layers that fill the chip: 256 to 1024 rows x 32 to 128 outputs per
//                                              workgroup, x loaded straight into LDS, the drawn weights shared through it,
//                                              v_mfma_f32_32x32x2_f32; also the input gradients of such layers
//   backward  hot_linear_wgrad_kernel          weight and bias gradients (per-sample G never stored); variants for
//                                              few tiles (waves split the rows), many rows (operands prefetched,
//                                              two output groups per wave), tiles dealt out by XCD
//             hot_linear_wgrad_tile_kernel     the same for large layers: 128 inputs x 128 outputs per workgroup, rows of
//                                              x and dy loaded straight into LDS
//             hot_linear_xgrad_kernel          input gradients up to a few hundred rows
//             hot_linear_xgrad_rows_kernel     input gradients from 256 rows: shared draws, as in the forward kernel
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

// The matrix pipeline writes the registers of an accumulator over several passes after the instruction has
// issued, and only wait states keep a following read from seeing the old value.  The compiler inserts them,
// but left them out where a branch lay between the last matrix instruction and the first read of its result:
// in one kernel variant the register written last came back stale (one row's product missing from one
// column of the weight gradients; found by comparing launch shapes on random layer sizes).  Every run of
// matrix instructions whose results are read next therefore ends here: 32 wait states that the scheduler
// may not move, more than any of these instructions needs.
__device__ __forceinline__ void mfma_results_settle()
{
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

// So that no read of a result can be written without those wait states: the accumulator registers of the
// matrix instructions are private to MfmaAcc, which hands them out only against an MfmaSettled, and constructing
// one of those issues the wait states.  Construct it behind the last mac() of a run; one serves all accumulators.
struct MfmaSettled {
    __device__ __forceinline__ MfmaSettled() { mfma_results_settle(); }
    MfmaSettled(const MfmaSettled &) = delete;
    MfmaSettled &operator=(const MfmaSettled &) = delete;
};

typedef float f16v __attribute__((ext_vector_type(16)));
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));

template <class V, int N>
class MfmaAcc {
    V v_;

public:
    __device__ __forceinline__ MfmaAcc()
    {
#pragma unroll
        for (int i = 0; i < N; ++i) v_[i] = 0.0f;
    }
    // v += a (x) b over the instruction's contraction block
    __device__ __forceinline__ void mac(float a, float b)
    {
        if constexpr (N == 4) v_ = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, v_, 0, 0, 0);
        else v_ = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, v_, 0, 0, 0);
    }
    // the same over sixteen contraction indices of bf16 operands (32 x 32 blocks only)
    __device__ __forceinline__ void mac(bf8 a, bf8 b) { v_ = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, v_, 0, 0, 0); }
    __device__ __forceinline__ V read(const MfmaSettled &) const { return v_; }
};
typedef MfmaAcc<f4, 4> Acc16x16;        // v_mfma_f32_16x16x4_f32: four result registers per lane
typedef MfmaAcc<f16v, 16> Acc32x32;     // v_mfma_f32_32x32x2_f32: sixteen

__device__ __forceinline__ float pick4_of(f4 v, int c) { return c == 0 ? v[0] : (c == 1 ? v[1] : (c == 2 ? v[2] : v[3])); }

struct LinearArgs {
    long rows, in_features, out_features, ldx;
    long x_sample_stride;   // floats between the inputs of consecutive samples (0: one input for all)
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
        Acc16x16 mm[ST][RB];

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
                                mm[st][rb].mac(xa[rb][h][c], w4[h][c]);
                }
            }
        }
        const MfmaSettled settled;
        f4 acc[ST][RB];
#pragma unroll
        for (int st = 0; st < ST; ++st)
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) acc[st][rb] = mm[st][rb].read(settled);

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

// ---------------------------------------------------------------------------------
// The same layer for many rows (hundreds and more: a transformer layer's tokens).  In the kernel above
// every wave draws the weights of its own 16 x 32 tile and uses them for at most 64 rows, so from a few
// hundred rows on the vector ALUs spend more time drawing than the matrix cores multiplying (the two do
// not overlap on this chip).  Here the four waves of a workgroup take 64 rows each (256 rows per
// workgroup) and SHARE every draw through LDS: per iteration of 64 inputs each of the 256 threads draws
// one quad of the 16-output x 64-input weight tile and stores it in LDS; after one barrier every wave
// reads its B operands from there (16-byte reads; the 272-byte row pitch spreads the 16 output rows over
// the banks) and multiplies its own 64 rows: 64 matrix instructions per drawn quad instead of 16.  The
// LDS tile is double-buffered, so one barrier per iteration suffices: a buffer is overwritten two
// iterations later, behind the barrier of the iteration in between, which a wave passes only after it
// has finished reading.  eps, lane roles inside a wave and the order of the contraction index are those
// of the kernel above (MFMA number i of a 32-input block takes element i of every lane's eight inputs).
// ---------------------------------------------------------------------------------
constexpr int kRowsKernelWaves = 4;
constexpr int kRowsKernelRows = 64 * kRowsKernelWaves;   // rows per workgroup
constexpr int kRowsKernelInputs = 64;                    // inputs per iteration: one drawn quad per thread
constexpr int kRowsKernelPitch = kRowsKernelInputs + 4;  // floats per output row of the LDS tile

template <int ST, int NO, bool XS>
__global__ void __launch_bounds__(64 * kRowsKernelWaves)
hot_linear_forward_rows_kernel(LinearArgs a)
{
    // NO column tiles of 16 outputs per workgroup.  More tiles reuse every loaded row of x more often but
    // cost accumulators: with two samples in flight one tile is fastest (86-90 TFLOP/s on 4096^3 and
    // 8192^2 x 1024; two and four tiles leave one wave per SIMD and reach 75-90), a single sample affords two
    // tiles (81 against 64 TFLOP/s).
    __shared__ __attribute__((aligned(16))) float tile[2][ST][NO * 16 * kRowsKernelPitch];
    // x is loaded with consecutive lanes on consecutive addresses (lane (n, j): inputs kb + 4 n .. + 3
    // of a row 4 q + j) and brought into the operand layout (lane (n, j): row n) through a wave's own 32 rows
    // of LDS, half a tile at a time: loading in the operand layout, where every lane of a 16-byte load sits
    // in another row, made the loads of x cost a third of the kernel's time (89 -> 105 TFLOP/s on 4096^3 with
    // the lane pattern alone).
    __shared__ __attribute__((aligned(16))) float turn[kRowsKernelWaves][32 * kRowsKernelPitch];
    static_assert(!XS || ST == 1, "one input per sample: one sample per pass");
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, j = lane >> 4;
    const long K = a.in_features, O = a.out_features, R = a.rows;
    const long o0 = (long)blockIdx.x * (kColsPerWave * NO);
    const long r0 = (long)blockIdx.y * kRowsKernelRows + (long)wave * 64;
    // as a drawing thread: quad dq of the 16 quads of outputs o0 + dn, o0 + dn + 16, ... in every iteration
    const int dn = (int)threadIdx.x >> 4, dq = (int)threadIdx.x & 15;

    for (int s0 = 0; s0 < a.s_loc; s0 += ST) {
        Acc16x16 mm[ST][4][NO];

        int buf = 0;
        for (long kb = 0; kb < K; kb += kRowsKernelInputs, buf ^= 1) {
            // this wave's rows of x (shared input): row 16 rb + n, inputs kb + 32 blk + 8 j + 4 h .. + 3
            f4 xa[4][2][2];
            f4 xg[4][4];          // as loaded: row 16 rb + 4 q + j, inputs kb + 4 n .. + 3
            {
                const float *xs = XS ? a.x + (size_t)s0 * (size_t)a.x_sample_stride : a.x;     // XS: the pass's one sample
#pragma unroll
                for (int rb = 0; rb < 4; ++rb)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const long row = r0 + kRowsPerTile * rb + 4 * q + j, k = kb + 4 * n;
                        xg[rb][q] = (row < R && k < K) ? load4<true, false>(xs + row * a.ldx + k) : f4{0.0f, 0.0f, 0.0f, 0.0f};
                    }
            }
            // draw this thread's quads for every sample of the chunk and put them into the tile
            const long kd = kb + 4 * dq;
#pragma unroll
            for (int no = 0; no < NO; ++no) {
                const long o_draw = o0 + 16 * no + dn;
                const bool draw_ok = o_draw < O && kd < K;
                const f4 m4 = draw_ok ? load4<true, false>(a.mu_w + o_draw * K + kd) : f4{0.0f, 0.0f, 0.0f, 0.0f};
                const f4 sd4 = draw_ok ? load4<true, false>(a.sigma_w + o_draw * K + kd) : f4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int st = 0; st < ST; ++st) {
                    f4 w4 = {0.0f, 0.0f, 0.0f, 0.0f};
                    if (draw_ok && s0 + st < a.s_loc) {
                        const f4 e = eps_quad(a.weight_quad0 + ((o_draw * K + kd) >> 2), s0 + st, a.rng);
#pragma unroll
                        for (int c = 0; c < 4; ++c) w4[c] = __builtin_fmaf(sd4[c], e[c], m4[c]);
                    }
                    *reinterpret_cast<f4 *>(&tile[buf][st][(16 * no + dn) * kRowsKernelPitch + 4 * dq]) = w4;
                }
            }
            {
                // Two halves of 32 rows through the wave's own LDS rows.  Only this wave touches them and the LDS
                // executes a wave's instructions in order, so no barrier is needed, only the program order.  It
                // happens ahead of the workgroup's barrier: a wave that drew faster turns its x while it would wait.
                float *mine = turn[wave];
#pragma unroll
                for (int half = 0; half < 2; ++half) {
#pragma unroll
                    for (int r2 = 0; r2 < 2; ++r2)
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            *reinterpret_cast<f4 *>(&mine[(16 * r2 + 4 * q + j) * kRowsKernelPitch + 4 * n]) = xg[2 * half + r2][q];
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
                    for (int r2 = 0; r2 < 2; ++r2)
#pragma unroll
                        for (int blk = 0; blk < 2; ++blk)
#pragma unroll
                            for (int h = 0; h < 2; ++h)
                                xa[2 * half + r2][blk][h] =
                                    *reinterpret_cast<const f4 *>(&mine[(16 * r2 + n) * kRowsKernelPitch + 32 * blk + 8 * j + 4 * h]);
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                }
            }
            __syncthreads();
#pragma unroll
            for (int st = 0; st < ST; ++st) {
                if (s0 + st < a.s_loc) {          // uniform over the workgroup
#pragma unroll
                    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
                        for (int h = 0; h < 2; ++h)
#pragma unroll
                            for (int no = 0; no < NO; ++no) {
                                const f4 wq = *reinterpret_cast<const f4 *>(&tile[buf][st][(16 * no + n) * kRowsKernelPitch + 32 * blk + 8 * j + 4 * h]);
#pragma unroll
                                for (int c = 0; c < 4; ++c)
#pragma unroll
                                    for (int rb = 0; rb < 4; ++rb)
                                        mm[st][rb][no].mac(xa[rb][blk][h][c], wq[c]);
                            }
                }
            }
        }
        const MfmaSettled settled;
        f4 acc[ST][4][NO];
#pragma unroll
        for (int st = 0; st < ST; ++st)
#pragma unroll
            for (int rb = 0; rb < 4; ++rb)
#pragma unroll
                for (int no = 0; no < NO; ++no) acc[st][rb][no] = mm[st][rb][no].read(settled);
        __syncthreads();        // the chunk's last reads are done before the next chunk's first draw lands in buffer 0

#pragma unroll
        for (int st = 0; st < ST; ++st) {
            if (s0 + st < a.s_loc) {
#pragma unroll
                for (int no = 0; no < NO; ++no) {
                    const long o = o0 + 16 * no + n;
                    const bool o_ok = o < O;
                    float bias = 0.0f;
                    if (a.mu_b && o_ok) {
                        const f4 e = eps_quad(a.bias_quad0 + (o >> 2), s0 + st, a.rng);
                        const int c = (int)(o & 3);
                        const float ev = c == 0 ? e[0] : (c == 1 ? e[1] : (c == 2 ? e[2] : e[3]));
                        bias = __builtin_fmaf(a.sigma_b[o], ev, a.mu_b[o]);
                    }
#pragma unroll
                    for (int rb = 0; rb < 4; ++rb)
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const long row = r0 + kRowsPerTile * rb + 4 * j + r;
                            if (row < R && o_ok) a.y[((size_t)(s0 + st) * (size_t)R + (size_t)row) * (size_t)O + (size_t)o] = acc[st][rb][no][r] + bias;
                        }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------
// The same layer for hundreds to thousands of rows.  On this chip the fp32 matrix instructions and the vector ALU do not
// run side by side (the fp32 matrix rate equals the packed fp32 vector rate: the same multipliers serve both; measured
// with the two kinds of work in different waves of one SIMD, the times add), so every cycle spent drawing is lost to
// the contraction, and the share of the draw is 81 / (rows per workgroup): a third at 256 rows, a seventh at 512.  Here
// a workgroup of eight waves owns 512 rows (64 per wave) x 32 to 128 outputs (one of sixteen: 1024 rows x 64 outputs; one
// of four: 256 rows x 32 or 64); per step of 16 contraction indices a thread draws at most ONE quad of the weight tile
// (two samples per pass: the second half of the drawing threads takes the second sample).
// x never passes through registers: each wave sends for the 16 inputs of its own 64 rows with buffer loads that write
// straight into LDS (lane l of an instruction leaves its 16 bytes at the instruction's LDS address + 16 l, zeros for an
// offset outside the window), into a region that only this wave reads, so x needs no barrier at all.  Rows are 64 bytes
// there without padding; so that the operand reads (lane = row, 16 bytes at a fixed input) still spread over all banks,
// the quad q of row r sits at position q ^ swizzle(r) of its row, which the loading lanes arrange by choosing which
// quad of memory they fetch.  The drawn weight tile is shared by the waves and laid out the same way.
// One barrier per step, in its middle.  A step on tile i (buffers i % 2):
//     read the operands of the second half (inputs 8 .. 15) of tile i;  matrix instructions of the first half, whose
//     operands are in registers already;  wait for everything sent for a step ago, barrier (every wave has now read
//     tile i, and tile i + 1 is complete);  draw tile i + 2 into the weight buffer just freed, send for mu, sigma of
//     tile i + 3 (registers) and for x of tile i + 2 (the x region just freed);  matrix instructions of the second half,
//     with the reads of the first-half operands of tile i + 1 issued ahead of their last quarter.
// Behind the barrier nothing waits for LDS or memory: loads have a whole step of matrix instructions to arrive, and
// the first matrix instruction behind it has its operands.  (The kernel this replaces kept both tiles in padded
// LDS arrays filled through registers and met at a barrier at the end of every step, behind which every wave first
// had to read its operands: 105-115 TFLOP/s where this one reaches 130.)
// The matrix instruction is v_mfma_f32_32x32x2_f32: lanes 0-31 hold inputs k .. k + 3 of their row or output, lanes
// 32-63 inputs k + 4 .. k + 7; instruction i takes element i of both operands, so the contraction index is enumerated
// in another order, identically on both sides.  All global accesses go through range-checked windows (see vec.h).
// ---------------------------------------------------------------------------------
constexpr int kSlabRows = 512;               // rows per workgroup of eight waves (sixteen: twice as many, four: half)
constexpr int kSlabK = 16;                   // contraction indices per step
constexpr unsigned kOutside = 0xFFFFFFF0u;   // a byte offset beyond any window

// (LDS pointers keep their address space through the call: as generic pointers they would become flat accesses)
typedef __attribute__((address_space(3))) float lds_float;
typedef __attribute__((address_space(3))) f4 lds_f4;
typedef __attribute__((address_space(3))) void lds_void;

typedef __attribute__((address_space(3))) char lds_char;
typedef __attribute__((address_space(3))) unsigned short lds_ushort;
typedef unsigned u2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) u2 lds_u2;
typedef __attribute__((address_space(3))) bf8 lds_bf8;

// The kernel's products on the bf16 matrix instruction (v_mfma_f32_32x32x16_bf16: sixteen contraction indices in half
// the cycles that v_mfma_f32_32x32x2_f32 takes for two) at the accuracy of fp32: a float is the exact sum of three
// pieces of at most eight significant bits each, x = x1 + x2 + x3 up to 2^-25 |x| (each piece is the remainder rounded
// to bf16, both remainders are exact), each piece is a bf16 number, and a product of two pieces is exact in the fp32
// accumulator.  x w = x1 w1 + (x1 w2 + x2 w1) + (x1 w3 + x2 w2 + x3 w1) + terms below 2^-24 |x w|: six products, summed
// from the smallest on.  The matrix pipe does 6 x 32 = 192 cycles of work per 32 x 32 x 16 block instead of 512.
constexpr bool kSlabBf16 = true;
constexpr bool kTileBf16 = true;      // the same in the weight-gradient tile kernel

typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
typedef float f2 __attribute__((ext_vector_type(2)));

// the pieces of two floats, each piece pair packed in one register (v_cvt_pk_bf16_f32 rounds to nearest even)
__device__ __forceinline__ void split2_bf16(float x0, float x1, unsigned &p1, unsigned &p2, unsigned &p3)
{
    p1 = __builtin_bit_cast(unsigned, __builtin_convertvector(f2{x0, x1}, bf2));
    const float r0 = x0 - __builtin_bit_cast(float, p1 << 16), r1 = x1 - __builtin_bit_cast(float, p1 & 0xFFFF0000u);
    p2 = __builtin_bit_cast(unsigned, __builtin_convertvector(f2{r0, r1}, bf2));
    const float s0 = r0 - __builtin_bit_cast(float, p2 << 16), s1 = r1 - __builtin_bit_cast(float, p2 & 0xFFFF0000u);
    p3 = __builtin_bit_cast(unsigned, __builtin_convertvector(f2{s0, s1}, bf2));
}

// the pieces of eight floats (a then b), packed as the matrix instruction takes them
__device__ __forceinline__ void split8_bf16(const f4 &a, const f4 &b, bf8 &p1, bf8 &p2, bf8 &p3)
{
    u4 q1, q2, q3;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float x0 = j < 2 ? a[2 * j] : b[2 * j - 4], x1 = j < 2 ? a[2 * j + 1] : b[2 * j - 3];
        unsigned t1, t2, t3;
        split2_bf16(x0, x1, t1, t2, t3);
        q1[j] = t1;
        q2[j] = t2;
        q3[j] = t3;
    }
    p1 = __builtin_bit_cast(bf8, q1);
    p2 = __builtin_bit_cast(bf8, q2);
    p3 = __builtin_bit_cast(bf8, q3);
}

// What the kernel works on: out_s[row][n] = sum_c in_s[row][c] W_s(n, c) + bias_s[n] with W_s drawn.  Forward (TR = false):
// in = x, c runs over the layer's inputs, n over its outputs, weight (n, c) has flat index n * C + c (the generator's
// quads run along c).  Input gradients (TR = true): in = dy, c runs over the layer's outputs, n over its inputs, weight
// (n, c) has flat index c * N + n (the quads run along n: a drawn quad goes into four rows of the tile), no bias.
struct SlabArgs {
    long rows, contract, outs;   // R, C, N
    long ld_in;                  // pitch of the rows of `in`
    long in_sample_stride;       // floats between the inputs of consecutive samples (0: one input for all)
    int s_begin, s_end;          // the local samples of this launch: workgroups with blockIdx.z = p take those of pass p
    long weight_quad0, bias_quad0;
    const float *in, *mu_w, *sigma_w, *mu_b, *sigma_b;
    float *out;                  // [S_loc, R, N] packed
    Rng rng;
};

__device__ __forceinline__ void everything_arrived_then_barrier()
{
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// position of a row's quads in LDS: quad q of row r (r counted within a block of 16) is stored as quad q ^ slab_swizzle(r);
// any 8 and any 16 consecutive rows then put a given q into different banks
__device__ __forceinline__ int slab_swizzle(int r) { return ((r >> 1) & 3) ^ ((r >> 3) & 1); }

// WAVES: 4, 8 or 16 waves of 64 rows each (16: half the draw per row again; their registers then allow 64 outputs and one
// sample; 4: for layers that 512 rows per workgroup fill badly: twice the draw per row, but up to four such workgroups
// share a compute unit, one's matrix instructions covering what the others wait for); CBW: blocks of 32 outputs per
// workgroup (every wave multiplies its 64 rows by all of them); ST samples per pass (they share the input tile); OWN:
// every sample has an input of its own (then ST = 1).
// RBW: blocks of 32 rows per wave; one only with four waves (128 rows per workgroup, for 65 to 128 rows: half the matrix
// work per draw again).
template <int WAVES, int CBW, int ST, bool OWN, bool TR, int RBW = 2, bool BF = (kSlabBf16 && RBW == 2)>
__global__ void __launch_bounds__(64 * WAVES, CBW * ST <= 2 ? (BF && WAVES != 16 ? 3 : 4) : 2)
hot_linear_slab_kernel(SlabArgs a)
{
    static_assert(ST == 1 || ST == 2, "one or two samples per pass");
    static_assert(!OWN || ST == 1, "one input per sample: one sample per pass");
    static_assert(WAVES == 8 || ((WAVES == 16 || WAVES == 4) && CBW * ST <= 2), "sixteen waves have 128 registers each, and so have four: four such workgroups share a compute unit");
    static_assert(RBW == 2 || (RBW == 1 && WAVES == 4), "32 rows per wave only in workgroups of four waves");
    constexpr int WROWS = 32 * RBW, OUTS = 32 * CBW, KS = kSlabK;
    constexpr int XW = WROWS * KS;           // floats of a wave's region of x
    constexpr int WT = OUTS * KS;            // floats of one sample's weight tile
    constexpr int NX = WROWS / 16;           // load instructions per wave and step
    constexpr int QUADS = ST * OUTS * 4;     // quads drawn per step
    static_assert(QUADS <= 64 * WAVES && QUADS % 64 == 0, "whole waves draw");
    __shared__ __attribute__((aligned(16))) float xs0[WAVES * XW], xs1[WAVES * XW];
    // (BF: three planes of bf16 pieces instead of one of floats)
    __shared__ __attribute__((aligned(16))) float ws0[ST * WT * (BF ? 3 : 2) / 2], ws1[ST * WT * (BF ? 3 : 2) / 2];
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int C = (int)a.contract, N = (int)a.outs, R = (int)a.rows;
    const int n0 = (int)blockIdx.x * OUTS, r0 = (int)blockIdx.y * (WROWS * WAVES);

    // reading operands: lane (l32, half) holds, for half-step k8, inputs 8 k8 + 4 half .. + 3 of row / output l32 of a block of 32
    int op_off[2];
#pragma unroll
    for (int k8 = 0; k8 < 2; ++k8) op_off[k8] = (l32 >> 4) * 256 + (4 * (l32 & 15) + ((2 * k8 + half) ^ slab_swizzle(l32 & 15))) * 4;

    // loading x: instruction j of a step brings rows 16 j .. 16 j + 15 of this wave's 64, lane l the quad that belongs at position l
    const int lq = (lane & 3) ^ slab_swizzle(lane >> 2);
    const int x_cols = C - 4 * lq;           // this lane's quad exists in the step that starts at cb0 while cb0 < x_cols
    unsigned x_first[NX];
    bool x_ok[NX];
#pragma unroll
    for (int j = 0; j < NX; ++j) {
        const long row = (long)r0 + wave * WROWS + 16 * j + (lane >> 2);
        x_ok[j] = row < R;
        x_first[j] = (unsigned)((row * a.ld_in + 4 * lq) * 4);
    }
    // drawing: sample d_st of the pass, quad d_idx of the step's tile: outputs n0 + d_n (.. + 3 if TR), contraction
    // indices cb0 + d_c (.. + 3 if not TR)
    const bool draws = t < QUADS;
    const int d_st = t / (OUTS * 4), d_idx = t % (OUTS * 4);
    const int d_n = TR ? 4 * (d_idx % (OUTS / 4)) : d_idx >> 2;
    const int d_c = TR ? d_idx / (OUTS / 4) : 4 * (d_idx & 3);
    const bool d_ok = draws && n0 + d_n < N;
    const int d_cols = C - d_c;
    const long d_flat = TR ? (long)d_c * N + n0 + d_n : (long)(n0 + d_n) * C + d_c;
    const unsigned w_step = TR ? (unsigned)(KS * N * 4) : (unsigned)(KS * 4);      // bytes from one step's quad to the next
    int d_put[TR ? 4 : 1];                   // where the drawn weights go in the tile (floats; BF: bytes within a plane)
    if constexpr (BF) {
        // A plane holds, per sample and output, 32 bytes: two chunks of eight bf16, chunk h with the contraction indices
        // 4 h .. 4 h + 3 and 8 + 4 h .. 8 + 4 h + 3 (what lanes 32 h .. 32 h + 31 feed to one matrix instruction), stored
        // as chunk h ^ bit 3 of the output (so that 16 consecutive outputs spread over all banks).
        const int h = (d_c >> 2) & 1, part = d_c >> 3;
#pragma unroll
        for (int e = 0; e < (TR ? 4 : 1); ++e)
            d_put[e] = (d_st * OUTS + d_n + e) * 32 + ((h ^ (((d_n + e) >> 3) & 1)) << 4) + part * 8 + (TR ? (d_c & 3) * 2 : 0);
    } else if constexpr (!TR) d_put[0] = d_st * WT + (4 * d_n + ((d_c >> 2) ^ slab_swizzle(d_n & 15))) * 4;
    else {
#pragma unroll
        for (int e = 0; e < 4; ++e) d_put[e] = d_st * WT + (4 * (d_n + e) + ((d_c >> 2) ^ slab_swizzle((d_n + e) & 15))) * 4 + (d_c & 3);
    }
    const window_t mu_win = window(a.mu_w, (unsigned)((long)C * N * 4)), sg_win = window(a.sigma_w, (unsigned)((long)C * N * 4));
    const unsigned in_bytes = (unsigned)((((long)R - 1) * a.ld_in + C) * 4);
    lds_float *const X0 = (lds_float *)xs0, *const X1 = (lds_float *)xs1, *const W0 = (lds_float *)ws0, *const W1 = (lds_float *)ws1;

    const int s0 = a.s_begin + (int)blockIdx.z * ST, s_hi = a.s_end;      // this workgroup's pass: samples s0 .. s0 + ST - 1 below s_hi
    {
        const window_t in_win = window(OWN ? a.in + (size_t)s0 * (size_t)a.in_sample_stride : a.in, in_bytes);
        Acc32x32 mm[ST][RBW][CBW];

        unsigned x_off[NX], w_off = (unsigned)(d_flat * 4);
#pragma unroll
        for (int j = 0; j < NX; ++j) x_off[j] = x_first[j];
        long d_quad = a.weight_quad0 + (d_flat >> 2);
        const bool d_live = d_ok && s0 + d_st < s_hi;

        // sends for mu and sigma of this thread's quad of the step that starts at cb0 (every call advances one step)
        f4 m4, sd4;
        auto ask_w = [&](int cb0) {
            const int off = (int)((d_ok && cb0 < d_cols) ? w_off : kOutside);
            m4 = window_load4<false>(mu_win, off);
            sd4 = window_load4<false>(sg_win, off);
            w_off += w_step;
        };
        // draws that quad and puts it into the tile (every call advances one step; zeros beyond the layer's edges)
        auto put_w = [&](int cb0, lds_float *wsb) {
            if (draws) {
                f4 w4 = {0.0f, 0.0f, 0.0f, 0.0f};
                if (d_live && cb0 < d_cols) {
                    const f4 e = eps_quad(d_quad, s0 + d_st, a.rng);
#pragma unroll
                    for (int c = 0; c < 4; ++c) w4[c] = __builtin_fmaf(sd4[c], e[c], m4[c]);
                }
                if constexpr (BF) {
                    // three bf16 pieces of every weight (see split2_bf16): a quad along the contraction is 8 bytes per plane
                    unsigned pc[3][2];
                    split2_bf16(w4[0], w4[1], pc[0][0], pc[1][0], pc[2][0]);
                    split2_bf16(w4[2], w4[3], pc[0][1], pc[1][1], pc[2][1]);
#pragma unroll
                    for (int pl = 0; pl < 3; ++pl) {
                        lds_char *plane = (lds_char *)wsb + pl * (ST * OUTS * 32);
                        if constexpr (!TR) *(lds_u2 *)(plane + d_put[0]) = u2{pc[pl][0], pc[pl][1]};
                        else {
#pragma unroll
                            for (int e = 0; e < 4; ++e) *(lds_ushort *)(plane + d_put[e]) = (unsigned short)(pc[pl][e >> 1] >> (16 * (e & 1)));
                        }
                    }
                } else if constexpr (!TR) *(lds_f4 *)(wsb + d_put[0]) = w4;
                else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) wsb[d_put[e]] = w4[e];
                }
                d_quad += TR ? (long)(KS / 4) * N : KS / 4;
            }
        };
        // sends for this wave's rows of the step that starts at cb0, straight into its region of xsb (every call advances one step)
        auto ask_x = [&](int cb0, lds_float *xsb) {
            const bool col_ok = cb0 < x_cols;
#pragma unroll
            for (int j = 0; j < NX; ++j) {
                __builtin_amdgcn_raw_ptr_buffer_load_lds(in_win, (lds_void *)(xsb + wave * XW + j * 256), 16,
                                                         (int)((x_ok[j] && col_ok) ? x_off[j] : kOutside), 0, 0, 0);
                x_off[j] += KS * 4;
            }
        };
        f4 xa[2][RBW], wb[2][ST][CBW];      // operand registers of the two half-steps
        auto read_ops = [&](int k8, const lds_float *xsb, const lds_float *wsb) {
            const volatile lds_f4 *xp = (const volatile lds_f4 *)(xsb + wave * XW + op_off[k8]);
            const volatile lds_f4 *wp = (const volatile lds_f4 *)(wsb + op_off[k8]);
#pragma unroll
            for (int rb = 0; rb < RBW; ++rb) xa[k8][rb] = xp[rb * 128];
            if constexpr (!BF) {
#pragma unroll
                for (int st = 0; st < ST; ++st)
#pragma unroll
                    for (int cb = 0; cb < CBW; ++cb) wb[k8][st][cb] = wp[(st * WT + cb * 512) / 4];
            }
        };
        auto multiply = [&](int k8, int i0, int i1) {
#pragma unroll
            for (int i = i0; i < i1; ++i)
#pragma unroll
                for (int st = 0; st < ST; ++st)
#pragma unroll
                    for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
                        for (int cb = 0; cb < CBW; ++cb) mm[st][rb][cb].mac(xa[k8][rb][i], wb[k8][st][cb][i]);
        };
        // BF: one step on the bf16 matrix instruction.  The operands of the step are read (x as floats, the weights
        // as their three planes), x is cut into its pieces, and six products per block of 32 x 32 leave out only the
        // terms below 2^-24 of the full product; then the barrier, behind which the buffers just read are refilled.
        auto step_bf = [&](int cb0, lds_float *xsb, lds_float *wsb) {
            read_ops(0, xsb, wsb);
            read_ops(1, xsb, wsb);
#pragma unroll
            for (int rb = 0; rb < RBW; ++rb) {
                bf8 a1, a2, a3;
                split8_bf16(xa[0][rb], xa[1][rb], a1, a2, a3);
#pragma unroll
                for (int st = 0; st < ST; ++st)
#pragma unroll
                    for (int cb = 0; cb < CBW; ++cb) {
                        const volatile lds_bf8 *wp = (const volatile lds_bf8 *)((const lds_char *)wsb + ((st * OUTS + cb * 32 + l32) * 32 + ((half ^ ((l32 >> 3) & 1)) << 4)));
                        const bf8 b1 = wp[0], b2 = wp[ST * OUTS * 2], b3 = wp[2 * ST * OUTS * 2];
                        mm[st][rb][cb].mac(a3, b1);
                        mm[st][rb][cb].mac(a2, b2);
                        mm[st][rb][cb].mac(a1, b3);
                        mm[st][rb][cb].mac(a2, b1);
                        mm[st][rb][cb].mac(a1, b2);
                        mm[st][rb][cb].mac(a1, b1);
                    }
            }
            everything_arrived_then_barrier();
            put_w(cb0 + 2 * KS, wsb);
            ask_w(cb0 + 3 * KS);
            ask_x(cb0 + 2 * KS, xsb);
        };
        auto step = [&](int cb0, lds_float *xsb, lds_float *wsb, const lds_float *xsn, const lds_float *wsn) {
            read_ops(1, xsb, wsb);
            multiply(0, 0, 4);
            everything_arrived_then_barrier();
            put_w(cb0 + 2 * KS, wsb);
            ask_w(cb0 + 3 * KS);
            ask_x(cb0 + 2 * KS, xsb);
            multiply(1, 0, 3);
            read_ops(0, xsn, wsn);
            multiply(1, 3, 4);
        };

        ask_x(0, X0);
        ask_x(KS, X1);
        ask_w(0);
        put_w(0, W0);
        ask_w(KS);
        put_w(KS, W1);
        ask_w(2 * KS);
        everything_arrived_then_barrier();
        if constexpr (BF) {
            for (int cb0 = 0; cb0 < C; cb0 += 2 * KS) {
                step_bf(cb0, X0, W0);
                step_bf(cb0 + KS, X1, W1);
            }
        } else {
            read_ops(0, X0, W0);
            for (int cb0 = 0; cb0 < C; cb0 += 2 * KS) {      // (an odd number of steps is followed by one on zeros)
                step(cb0, X0, W0, X1, W1);
                step(cb0 + KS, X1, W1, X0, W0);
            }
        }
        const MfmaSettled settled;

        // result register i of a 32 x 32 block: row 8 (i / 4) + 4 (lane / 32) + i % 4, column lane % 32
        int r0w = r0 + wave * WROWS + 4 * half, n0l = n0 + l32;
        asm volatile("" : "+v"(r0w), "+v"(n0l));       // (so that the offsets below are formed here, not ahead of the loop)
#pragma unroll
        for (int st = 0; st < ST; ++st) {
            if (s0 + st < s_hi) {
                const window_t out_win = window(a.out + (size_t)(s0 + st) * (size_t)R * (size_t)N, (unsigned)((long)R * N * 4));
#pragma unroll
                for (int cb = 0; cb < CBW; ++cb) {
                    const int n = n0l + 32 * cb;
                    const bool n_ok = n < N;
                    float bias = 0.0f;
                    if (!TR && a.mu_b && n_ok) {
                        const f4 e = eps_quad(a.bias_quad0 + (n >> 2), s0 + st, a.rng);
                        bias = __builtin_fmaf(a.sigma_b[n], pick4_of(e, n & 3), a.mu_b[n]);
                    }
#pragma unroll
                    for (int rb = 0; rb < RBW; ++rb) {
                        const f16v acc = mm[st][rb][cb].read(settled);
#pragma unroll
                        for (int i = 0; i < 16; ++i) {
                            const int row = r0w + 32 * rb + 8 * (i >> 2) + (i & 3);
                            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, acc[i] + bias), out_win,
                                                                  (n_ok && row < R) ? (int)(((unsigned)row * (unsigned)N + (unsigned)n) * 4u) : (int)kOutside, 0, 0);
                        }
                    }
                }
            }
        }
    }
}

// Whether the kernel above can address this problem (its windows take 32-bit byte offsets, its indices are 32-bit).
inline bool slab_kernel_fits(long rows, long contract, long outs, long ld_in)
{
    const unsigned long long lim = 0xFFFFFFF0ull;
    return (unsigned long long)((rows + 2 * kSlabRows) * ld_in + contract) * 4 < lim && (unsigned long long)(contract + 4 * kSlabK) * outs * 4 < lim &&
           (unsigned long long)(rows + 2 * kSlabRows) * (outs + 128) * 4 < lim && (rows + kSlabRows - 1) / kSlabRows <= 65535;
}

constexpr int kComputeUnits = 256;
constexpr int kSlabMinRows = 512;             // below, the kernels whose workgroups hold 256 rows
// Least share of the chip's time that the tiles of a launch must fill, measured against the kernels for fewer rows on 130
// layer shapes.  Forward with a shared x: wins from 0.6 on (1.1-2x; between 0.45 and 0.6 anything from 0.73x to 1.2x).
// Forward with one x per sample, where the other kernel is weaker: from 0.45 on (1.4-1.5x between 0.45 and 0.6).  Input
// gradients, whose other kernel packs several 256-row workgroups into a compute unit: from 0.72 on (1.0-1.3x), and from
// 0.6 on where the tiles of 32 inputs are the best shape (1.0-1.2x there; the wider shapes 0.95-0.97x).
constexpr double kSlabMinFillForward = 0.6, kSlabMinFillForwardOwnX = 0.45, kSlabMinFillInputGrad = 0.72, kSlabMinFillInputGradNarrow = 0.6;

// A launch shape of the kernel above and what it costs.  One workgroup per compute unit runs at a time (two of the narrow
// ones, at half speed each), so a launch takes its number of rounds times the time of a workgroup, which per step is, per
// block of 32 outputs and sample, about 2050 cycles of matrix instructions for 512 rows plus 325 of drawing, and
// 600 for the barrier and what else does not overlap; the wider tile also loads x half as often.  The constants are
// fitted to timings of 130 layer shapes; the model only has to rank the shapes of one layer.
struct SlabShape {
    int waves;      // 4, 8 or 16; 0: none
    int cbw;        // blocks of 32 outputs per workgroup
    double cost;
    int rbw = 2;    // blocks of 32 rows per wave (one: four waves of 32 rows, for 65 to 128 rows)
    double fill = 1.0;      // four-wave shapes: the share of its compute units' workgroup slots that the launch fills
};

// Four waves: 256 rows x 32 or 64 output-samples.  Up to four such workgroups share a compute unit and run at the rate of
// its matrix pipes together (measured per step and workgroup: 2700 cycles for 64 output-samples, 1600 for 32, whose x is
// re-read twice as often), one alone at that plus 600.  Against the kernels for few rows they win from a fill of 0.52 of the
// compute units' last workgroup on (measured on 160 layer shapes of 256 to 7260 rows: 1.1-2.2x from there, 0.3-0.9x below).
constexpr double kSlab4MinFill = 0.52;
constexpr long kSlab4MinRows = 129;
// From 65 to 128 rows the four waves take 32 rows each: half the matrix work per draw again, measured per step and
// workgroup 1850 cycles for 64 output-samples and 1170 for 32, 300 more for one alone on its compute unit.  Against the
// kernels for few rows, which draw every weight once per 64 rows: 96 and 128 rows x 8192^2 1.13-1.27x, x 2160 x 8640 with
// one x per sample 1.2-1.28x; a narrow workgroup alone on its compute unit (one wave per SIMD) loses (96 x 4096^2: 0.87x),
// so the shapes of 32 output-samples need two workgroups per compute unit.
constexpr long kSlab4HalfMinRows = 65;
constexpr double kSlab4HalfMinFill = 0.52;

inline SlabShape slab_shape4(long rows, long outs, long passes, int st)
{
    SlabShape best = {0, 0, 0.0};
    if (passes < 1 || passes > 65535 || rows < kSlab4HalfMinRows) return best;
    const bool half = rows <= 128;
    const long tile_rows = half ? 128 : 256;
    for (int cbw = st == 2 ? 1 : 2; cbw >= 1; cbw /= 2) {
        const long col_tiles = (outs + 32 * cbw - 1) / (32 * cbw), wgs = col_tiles * ((rows + tile_rows - 1) / tile_rows) * passes;
        const long per_cu = (wgs + kComputeUnits - 1) / kComputeUnits;
        const double exact = (double)outs / (32 * cbw) * (double)rows / (double)tile_rows * (double)passes;
        if (exact < (half ? kSlab4HalfMinFill : kSlab4MinFill) * (double)(per_cu * kComputeUnits)) continue;
        if (half && cbw * st == 1 && wgs < 2 * kComputeUnits) continue;
        const double wide = half ? 1850.0 : 2700.0, narrow = half ? 1170.0 : 1600.0;
        const double cost = (double)per_cu * (cbw * st == 2 ? wide : narrow) + (per_cu == 1 ? (half ? 300.0 : 600.0) : 0.0);
        if (best.waves == 0 || cost < best.cost) best = SlabShape{4, cbw, cost, half ? 1 : 2, exact / (double)(per_cu * kComputeUnits)};
    }
    return best;
}

// the cheapest of the eight-wave shapes with `st` samples per pass and tiles of 32 * narrow .. 32 * wide outputs
inline SlabShape slab_shape8(long rows, long outs, long passes, int st, int narrow, int wide)
{
    SlabShape best = {0, 0, 0.0};
    if (passes < 1 || passes > 65535) return best;
    const long row_blocks = (rows + kSlabRows - 1) / kSlabRows;
    for (int cbw = wide; cbw >= narrow; cbw /= 2) {
        const long wgs = ((outs + 32 * cbw - 1) / (32 * cbw)) * row_blocks * passes;
        // (two narrow workgroups share a compute unit and cover part of each other's waits: about 5 % by measurement)
        const double cost = (double)((wgs + kComputeUnits - 1) / kComputeUnits) * (2375.0 * cbw * st + 600.0) * (cbw * st <= 2 ? 0.95 : 1.0);
        if (best.waves == 0 || cost < best.cost) best = SlabShape{8, cbw, cost};
    }
    return best;
}

// sixteen waves: 1024 rows x 64 outputs, one sample per pass
inline SlabShape slab_shape16(long rows, long outs, long passes)
{
    if (passes < 1 || passes > 65535 || rows <= kSlabRows) return SlabShape{0, 0, 0.0};
    const long wgs = ((outs + 63) / 64) * ((rows + 2 * kSlabRows - 1) / (2 * kSlabRows)) * passes;
    // (measured on layers that both shapes fill: 0.966 of the time of 512 rows x 64 outputs x 2 samples)
    return SlabShape{16, 2, (double)((wgs + kComputeUnits - 1) / kComputeUnits) * 9750.0};
}

// what the samples of a launch would cost on a chip they fill evenly
inline double slab_full(long rows, long outs, long samples)
{
    return (double)rows / kSlabRows * (double)outs / 32.0 * (double)samples * 2375.0 / kComputeUnits;
}

// Launches it for the samples s_begin .. s_end - 1, ST per pass, one pass per layer of the grid along z.
template <int WAVES, int CBW, int ST, bool OWN, bool TR, int RBW = 2>
void slab_go(hipStream_t s, SlabArgs a, int s_begin, int s_end)
{
    a.s_begin = s_begin;
    a.s_end = s_end;
    const dim3 grid((unsigned)((a.outs + 32 * CBW - 1) / (32 * CBW)), (unsigned)((a.rows + 32 * RBW * WAVES - 1) / (32 * RBW * WAVES)),
                    (unsigned)((s_end - s_begin + ST - 1) / ST));
    hot_linear_slab_kernel<WAVES, CBW, ST, OWN, TR, RBW><<<grid, dim3(64 * WAVES), 0, s>>>(a);
}

// one sample per pass, in the shape chosen
template <bool OWN, bool TR>
void slab_go_singles(const SlabShape &shape, hipStream_t s, const SlabArgs &a, int s_begin, int s_end)
{
    if (shape.waves == 16) slab_go<16, 2, 1, OWN, TR>(s, a, s_begin, s_end);
    else if (shape.waves == 4 && shape.rbw == 1 && shape.cbw == 2) slab_go<4, 2, 1, OWN, TR, 1>(s, a, s_begin, s_end);
    else if (shape.waves == 4 && shape.rbw == 1) slab_go<4, 1, 1, OWN, TR, 1>(s, a, s_begin, s_end);
    else if (shape.waves == 4 && shape.cbw == 2) slab_go<4, 2, 1, OWN, TR>(s, a, s_begin, s_end);
    else if (shape.waves == 4) slab_go<4, 1, 1, OWN, TR>(s, a, s_begin, s_end);
    else if (shape.cbw == 4) slab_go<8, 4, 1, OWN, TR>(s, a, s_begin, s_end);
    else if (shape.cbw == 2) slab_go<8, 2, 1, OWN, TR>(s, a, s_begin, s_end);
    else slab_go<8, 1, 1, OWN, TR>(s, a, s_begin, s_end);
}

// the cheaper of the shapes with one sample per pass, or none where the chip would stand too empty
// (min_fill_narrow: the bar where that shape has tiles of 32 outputs)
inline SlabShape slab_shape_singles(long rows, long outs, long samples, double min_fill, double min_fill_narrow)
{
    SlabShape best = {0, 0, 0.0};
    if (rows >= kSlabMinRows) {
        best = slab_shape8(rows, outs, samples, 1, 1, 4);
        const SlabShape tall = slab_shape16(rows, outs, samples);
        if (tall.waves && (!best.waves || tall.cost < best.cost)) best = tall;
        const double bar = best.waves == 8 && best.cbw == 1 ? min_fill_narrow : min_fill;
        if (best.waves && slab_full(rows, outs, samples) < bar * best.cost) best.waves = 0;
    }
    const SlabShape small = slab_shape4(rows, outs, samples, 1);
    if (small.waves && (!best.waves || small.cost < best.cost)) best = small;
    return best;
}

// How the forward call runs a layer on the kernel above: pairs of samples that share x (samples 0 .. 2 * pairs - 1) in
// `two` and the samples behind them one at a time in `one`; neither where the layer is left to the kernels for fewer rows.
struct SlabForwardPlan {
    int pair_samples;     // samples that go two to a pass
    SlabShape two, one;   // (waves == 0: not used)
};

inline SlabForwardPlan slab_forward_plan(const hot_linear_desc *d)
{
    SlabForwardPlan p = {0, SlabShape{0, 0, 0.0}, SlabShape{0, 0, 0.0}};
    if (d->rows < kSlab4HalfMinRows || !slab_kernel_fits(d->rows, d->in_features, d->out_features, d->ldx)) return p;
    const int S = d->s_local;
    if (d->x_sample_stride != 0 || S == 1) {
        const double bar = d->x_sample_stride != 0 ? kSlabMinFillForwardOwnX : kSlabMinFillForward;
        p.one = slab_shape_singles(d->rows, d->out_features, S, bar, bar);
        return p;
    }
    // two samples to a pass and an odd last one on its own (512-row or 256-row workgroups), or every sample on its own in the
    // tall shape: whichever is cheapest among those that fill the chip well enough
    const int pairs = S / 2, odd = S & 1;
    const SlabShape none = {0, 0, 0.0}, free = {8, 0, 0.0};
    double best = 0.0;
    if (d->rows >= kSlabMinRows) {
        const SlabShape two = slab_shape8(d->rows, d->out_features, pairs, 2, 1, 2);
        const SlabShape last = odd ? slab_shape8(d->rows, d->out_features, 1, 1, 1, 4) : free;
        const SlabShape tall = slab_shape16(d->rows, d->out_features, S);
        const double full = slab_full(d->rows, d->out_features, S);
        if (tall.waves && (!two.waves || !last.waves || tall.cost < two.cost + last.cost)) {
            if (full >= kSlabMinFillForward * tall.cost) {
                p.one = tall;
                best = tall.cost;
            }
        } else if (two.waves && last.waves && full >= kSlabMinFillForward * (two.cost + last.cost)) {
            p.pair_samples = 2 * pairs;
            p.two = two;
            p.one = odd ? last : none;
            best = two.cost + last.cost;
        }
    }
    const SlabShape two4 = slab_shape4(d->rows, d->out_features, pairs, 2);
    const SlabShape last4 = odd ? slab_shape4(d->rows, d->out_features, 1, 1) : free;
    if (two4.waves && last4.waves && (best == 0.0 || two4.cost + last4.cost < best)) {
        p.pair_samples = 2 * pairs;
        p.two = two4;
        p.one = odd ? last4 : none;
    }
    return p;
}

// ... and the input gradients (dy is the input, read in 16-byte quads: rows of dy must allow that)
inline SlabShape slab_input_grad_shape(const hot_linear_desc *d, bool dy_aligned)
{
    if (d->rows < kSlab4HalfMinRows || (d->out_features & 3) != 0 || !dy_aligned ||
        !slab_kernel_fits(d->rows, d->out_features, d->in_features, d->out_features))
        return SlabShape{0, 0, 0.0};
    return slab_shape_singles(d->rows, d->in_features, d->s_local, kSlabMinFillInputGrad, kSlabMinFillInputGradNarrow);
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


// ---------------------------------------------------------------------------------
// Backward.  Weight gradients: a wave owns 16 outputs x 64 inputs and contracts over the rows with
// the TRANSPOSED product P_s[k][o] = sum_r x_s[r][k] dy_s[r][o] (x as the A operand, dy as B).  A lane
// loads four consecutive inputs of a row of x at once and hands element i to matrix instruction i, so
// that register c of the four accumulators holds four consecutive inputs k of one output o: exactly one
// quad of the generator, drawn once per sample, and one 16-byte access to mu, sigma and the two
// gradient arrays.  Input gradients: dx_s^T[k][r] = sum_o W_s[o][k] dy_s[r][o] with
// the drawn weights as the A operand; MFMA number i of a step takes element i of every lane's
// quad (as in the forward kernel), so result register rr of the four accumulators again holds
// four consecutive inputs and dx is written with 16-byte stores.
// ---------------------------------------------------------------------------------
struct LinearGradArgs {
    long rows, in_features, out_features, ldx, x_sample_stride;
    int s_loc;
    long weight_quad0, bias_quad0;
    double g, k;            // scaling of the data part and of the KL part of the gradients
    const float *x, *dy, *mu_w, *sigma_w, *mu_b, *sigma_b;
    float *gmu_w, *gsig_w, *gmu_b, *gsig_b, *dx;
    float *ws;              // PARTS kernels: partial sums [part][gm, gs][O*K + O]
    long rows_per_part;     // PARTS kernels: rows of one part, a multiple of 16
    int x_parts;            // input gradients for many rows: parts the outputs are cut into (1: dx written directly)
    long outs_per_part;     // outputs of one such part, a multiple of 16; partial dx blocks go to ws[part][S][R][K]
    Rng rng;
};

__device__ __forceinline__ float pick4(f4 v, int c) { return c == 0 ? v[0] : (c == 1 ? v[1] : (c == 2 ? v[2] : v[3])); }

// The four lanes (j = 0..3, same n) of a 16-lane column each hold four quads q[0..3], lane j's quad t
// belonging to position 16 j + 4 t of a 64-wide block.  Afterwards lane j's quad t belongs to position
// 16 t + 4 j: a store of quad t then covers 64 contiguous bytes per 16-lane column instead of four separate
// 16-byte pieces (the memory system wants whole 64-byte words).  A 4 x 4 transpose over j in four rounds of
// lane shuffles; every lane of the wave must call it.
__device__ __forceinline__ void transpose_quads_over_j(f4 (&q)[4], int j, int n)
{
    f4 out[4];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const int give = (j - d) & 3, from = (((j + d) & 3) << 4) | n, slot = (j + d) & 3;
        f4 v = q[0];
#pragma unroll
        for (int t = 1; t < 4; ++t)
            if (give == t) v = q[t];
        f4 r;
#pragma unroll
        for (int c = 0; c < 4; ++c) r[c] = __shfl(v[c], from);
#pragma unroll
        for (int t = 0; t < 4; ++t)
            if (slot == t) out[t] = r;
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) q[t] = out[t];
}

// grad_mu, grad_sigma of one parameter from its sums over the samples (gradient and averaging lines
// of Algorithm 2; d KL / d mu = mu, d KL / d sigma = sigma - 1/sigma).  In single precision: six operations per
// parameter.  An fp64 form (the flat sample layer's, which is bound by memory) cost these kernels, bound by vector
// arithmetic at few rows, about 1000 cycles per 16 x 64 tile, 40 % of a draw (8192^2 at 16 rows: weight gradients
// 0.289 -> 0.271 ms; at 1024 rows 127.6 -> 130 TFLOP/s); each term is rounded once more, 1e-7 of its magnitude.
__device__ __forceinline__ void finish_pair(float sum_g, float sum_ge, float m, float sd, float g, float k,
                                            float &gm, float &gs)
{
    const float kl_m = k != 0.0f ? k * m : 0.0f;
    const float kl_s = k != 0.0f ? k * (sd - __builtin_amdgcn_rcpf(sd)) : 0.0f;
    gm = __builtin_fmaf(g, sum_g, kl_m);
    gs = __builtin_fmaf(g, sum_ge, kl_s);
}

constexpr int kWgradWaves = 4;       // waves per workgroup when every wave has a tile of its own
constexpr int kWgradMaxSplit = 8;    // most waves that share one tile (60 KiB of LDS for their partial sums)
constexpr int kWgradRowsPerIter = 16;
constexpr int kWgradDeepRows = 128;  // from this many rows on operands are prefetched one row block ahead
constexpr int kWgradWideRows = 512;  // from this many rows on a wave may own several output groups
constexpr int kWgradMaxParts = 16;    // most row parts of a run with a workspace
constexpr int kWgradPartials = 34;   // per lane: 16 + 16 weight-gradient sums and the two bias sums

// SPLIT = false: the four waves of a workgroup own one tile each.  SPLIT = true (layers with few
// tiles and many rows): the waves of a workgroup share one tile, take the 16-row blocks round-robin,
// apply each sample's eps to their own partial product (the gradient is linear in it) and add their
// sums through LDS in wave order at the end.  DEEP (many rows): operands of the next row block are
// fetched while the current one multiplies; it costs a wave per SIMD, which the few-row shapes need more.
// OB: 16-output groups per tile.  At many rows the kernel is bound by the 16-byte loads of x (with them
// taken out it runs at 100-119 TFLOP/s instead of 60-80, with the loads of dy taken out nothing changes);
// two output groups per wave use every loaded quad of x twice.
//
// Workgroups go to the eight XCDs round-robin and each XCD has an L2 of its own, so the tiles are dealt
// out by XCD: the list of tiles, ordered so that the larger of the two operands changes slowest (output
// groups outermost when O >= K: dy is the larger one; input groups outermost otherwise), is cut into eight
// contiguous ranges, one per XCD.  The larger operand then enters one L2 only (two at a range boundary) and
// the smaller one each L2 once, where the plain order had every XCD stream both (40 % L2 misses at 7260
// rows).  Only locality depends on the round-robin placement, not the result.
constexpr int kXcds = 8;

constexpr int wgrad_max_split(int ob) { return kWgradMaxSplit / ob; }   // at most 60 KiB of LDS

template <bool SPLIT, bool DEEP, int OB, bool PARTS = false>
__global__ void __launch_bounds__(64 * (SPLIT ? wgrad_max_split(OB) : kWgradWaves), 1)
hot_linear_wgrad_kernel(LinearGradArgs a)
{
    extern __shared__ float partial[];   // SPLIT: [waves - 1][OB][kWgradPartials][64]
    const int lane = threadIdx.x & 63, waves = blockDim.x >> 6;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // uniform: tile and trip counts stay scalar
    const int n = lane & 15, j = lane >> 4;
    const long K = a.in_features, O = a.out_features, R = a.rows;
    const long k_groups = (K + 63) / 64;
    const long o_tiles = ((O + 15) / 16 + OB - 1) / OB, tiles = k_groups * o_tiles, per_xcd = (tiles + kXcds - 1) / kXcds;
    const long xcd = blockIdx.x % kXcds, nth = blockIdx.x / kXcds;      // nth workgroup of its XCD
    const long local = SPLIT ? nth : nth * kWgradWaves + wave;
    const long tile = xcd * per_xcd + local;
    // no such tile: a whole workgroup (SPLIT) or a whole wave of a kernel without barriers leaves
    if (local >= per_xcd || tile >= tiles) return;
    const bool outputs_outermost = O >= K;
    const long o0 = (outputs_outermost ? tile / k_groups : tile % o_tiles) * (16 * OB);
    const long k0 = (outputs_outermost ? tile % k_groups : tile / o_tiles) * 64;
    long o[OB];
    bool o_ok[OB];
#pragma unroll
    for (int b = 0; b < OB; ++b) {
        o[b] = o0 + 16 * b + n;
        o_ok[b] = o[b] < O;
    }
    const bool bias_tile = a.mu_b != nullptr && k0 == 0;     // uniform over the wave: this tile also owns its outputs' biases
    // PARTS: workgroup (x, y) owns the rows of part y only and leaves its sums in the workspace
    const long r_lo = PARTS ? (long)blockIdx.y * a.rows_per_part : 0;
    const long r_hi = PARTS ? (r_lo + a.rows_per_part < R ? r_lo + a.rows_per_part : R) : R;
    const long row_first = r_lo + (SPLIT ? (long)wave * kWgradRowsPerIter : 0);
    const long row_step = SPLIT ? (long)waves * kWgradRowsPerIter : kWgradRowsPerIter;

    // gm[b][t], gs[b][t]: the sums for the generator quad of inputs k0 + 16 j + 4 t .. + 3 of output o[b]
    f4 gm[OB][4], gs[OB][4];
    float gb_m[OB], gb_s[OB];
#pragma unroll
    for (int b = 0; b < OB; ++b) {
#pragma unroll
        for (int t = 0; t < 4; ++t) gm[b][t] = gs[b][t] = f4{0.0f, 0.0f, 0.0f, 0.0f};
        gb_m[b] = gb_s[b] = 0.0f;
    }
    const long k_lane = k0 + 4 * n;          // as an A lane: the four inputs k_lane .. k_lane + 3 of a row, one 16-byte load
    const bool k_lane_ok = k_lane < K;

    for (int s = 0; s < a.s_loc; ++s) {
        const float *xs = a.x + (size_t)s * (size_t)a.x_sample_stride;
        const float *dys = a.dy + (size_t)s * (size_t)R * (size_t)O;
        // matrix instruction i of a row block takes element i of every lane's four inputs, so P[.][i] collects
        // the inputs k0 + 4 m + i (m = 0..15) and register c of P[.][i] is input k0 + 16 j + 4 c + i: the four
        // P[.][.][c] are the four consecutive inputs of one generator quad
        Acc16x16 mm[OB][4], mm_b[OB];
        // Whole blocks of 16 rows first, with nothing in the loop but the loads, the offset increments and the
        // matrix instructions: lanes outside the layer (o >= O, inputs >= K) read a valid address instead, which
        // only reaches rows and columns of P that are never stored.  The last, partial block is predicated per
        // row: rows beyond the last one must contribute zeros, they are summed over.
        constexpr int Q = kWgradRowsPerIter / 4;
        long pd[OB][Q], px[Q];      // offsets, not pointers: the loads stay global loads
#pragma unroll
        for (int q = 0; q < Q; ++q) {
#pragma unroll
            for (int b = 0; b < OB; ++b) pd[b][q] = (row_first + 4 * q + j) * O + (o_ok[b] ? o[b] : O - 1);
            px[q] = (row_first + 4 * q + j) * a.ldx + (k_lane_ok ? k_lane : 0);
        }
        const long d_step = row_step * O, x_step = row_step * a.ldx;
        const long full = r_hi - row_first >= kWgradRowsPerIter ? (r_hi - kWgradRowsPerIter - row_first) / row_step + 1 : 0;
        auto multiply = [&](const float (&bv)[OB][Q], const f4 (&av)[Q]) {
#pragma unroll
            for (int q = 0; q < Q; ++q)
#pragma unroll
                for (int b = 0; b < OB; ++b)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        mm[b][i].mac(av[q][i], bv[b][q]);
            if (bias_tile) {             // column sums of dy: the same contraction against ones
#pragma unroll
                for (int q = 0; q < Q; ++q)
#pragma unroll
                    for (int b = 0; b < OB; ++b) mm_b[b].mac(1.0f, bv[b][q]);
            }
        };
        if constexpr (DEEP) {
            // Two register sets of operands.  Every fetch is unconditional (behind a branch around loads the
            // compiler waits for all of them at the join): past the last whole block the offsets stop moving
            // and that block is simply read again.
            float bA[OB][Q], bB[OB][Q];
            f4 aA[Q], aB[Q];
            long fetched = 0;
            auto fetch = [&](float (&bv)[OB][Q], f4 (&av)[Q]) {
                ++fetched;
                const long dd = fetched < full ? d_step : 0, dx = fetched < full ? x_step : 0;
#pragma unroll
                for (int q = 0; q < Q; ++q) {
#pragma unroll
                    for (int b = 0; b < OB; ++b) {
                        bv[b][q] = dys[pd[b][q]];
                        pd[b][q] += dd;
                    }
                    av[q] = load4<true, false>(xs + px[q]);
                    px[q] += dx;
                }
            };
            if (full > 0) {
                fetch(bA, aA);
                for (long it = 0; it < full; it += 2) {
                    fetch(bB, aB);
                    __builtin_amdgcn_sched_barrier(0);
                    multiply(bA, aA);
                    __builtin_amdgcn_sched_barrier(0);
                    fetch(bA, aA);
                    __builtin_amdgcn_sched_barrier(0);
                    if (it + 1 < full) multiply(bB, aB);
                    __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int q = 0; q < Q; ++q) {        // on to the partial block
#pragma unroll
                    for (int b = 0; b < OB; ++b) pd[b][q] += d_step;
                    px[q] += x_step;
                }
            }
        } else {
            for (long it = 0; it < full; ++it) {
                float bv[OB][Q];
                f4 av[Q];
#pragma unroll
                for (int q = 0; q < Q; ++q) {
#pragma unroll
                    for (int b = 0; b < OB; ++b) {
                        bv[b][q] = dys[pd[b][q]];
                        pd[b][q] += d_step;
                    }
                    av[q] = load4<true, false>(xs + px[q]);
                    px[q] += x_step;
                }
                __builtin_amdgcn_sched_barrier(0);      // all loads first, one wait
                multiply(bv, av);
            }
        }
        const long rb = row_first + full * row_step;
        if (rb < r_hi) {
            float bv[OB][Q];
            f4 av[Q];
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                const bool r_ok = rb + 4 * q + j < r_hi;
#pragma unroll
                for (int b = 0; b < OB; ++b) bv[b][q] = r_ok ? dys[pd[b][q]] : 0.0f;
                av[q] = r_ok ? load4<true, false>(xs + px[q]) : f4{0.0f, 0.0f, 0.0f, 0.0f};
            }
            multiply(bv, av);
        }
        const MfmaSettled settled;
        f4 P[OB][4], Pb[OB];
#pragma unroll
        for (int b = 0; b < OB; ++b) {
#pragma unroll
            for (int i = 0; i < 4; ++i) P[b][i] = mm[b][i].read(settled);
            Pb[b] = mm_b[b].read(settled);
        }
        if (row_first < r_hi) {          // a wave without rows has nothing to add (uniform over the wave)
#pragma unroll
            for (int b = 0; b < OB; ++b) {
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const long col = k0 + 16 * j + 4 * t;
                    if (o_ok[b] && col < K) {
                        const f4 e = eps_quad(a.weight_quad0 + ((o[b] * K + col) >> 2), s, a.rng);
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            gm[b][t][c] += P[b][c][t];
                            gs[b][t][c] = __builtin_fmaf(P[b][c][t], e[c], gs[b][t][c]);
                        }
                    }
                }
                if (bias_tile && o_ok[b]) {      // every register of Pb holds sum_r dy_s[r][o]
                    const f4 e = eps_quad(a.bias_quad0 + (o[b] >> 2), s, a.rng);
                    gb_m[b] += Pb[b][0];
                    gb_s[b] = __builtin_fmaf(Pb[b][0], pick4(e, (int)(o[b] & 3)), gb_s[b]);
                }
            }
        }
    }

    if constexpr (SPLIT) {
        if (wave > 0) {
#pragma unroll
            for (int b = 0; b < OB; ++b) {
                float *mine = partial + (size_t)((wave - 1) * OB + b) * kWgradPartials * 64 + lane;
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        mine[(t * 4 + c) * 64] = gm[b][t][c];
                        mine[(16 + t * 4 + c) * 64] = gs[b][t][c];
                    }
                mine[32 * 64] = gb_m[b];
                mine[33 * 64] = gb_s[b];
            }
        }
        __syncthreads();
        if (wave != 0) return;
        for (int v = 1; v < waves; ++v)
#pragma unroll
            for (int b = 0; b < OB; ++b) {
                const float *theirs = partial + (size_t)((v - 1) * OB + b) * kWgradPartials * 64 + lane;
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        gm[b][t][c] += theirs[(t * 4 + c) * 64];
                        gs[b][t][c] += theirs[(16 + t * 4 + c) * 64];
                    }
                gb_m[b] += theirs[32 * 64];
                gb_s[b] += theirs[33 * 64];
            }
    }

    // A lane holds the 16 consecutive inputs k0 + 16 j .. + 15 of its output: the four lanes of an output
    // exchange quads so that store t covers the 64 contiguous bytes k0 + 16 t .. + 15 of every row.
#pragma unroll
    for (int b = 0; b < OB; ++b) {
        transpose_quads_over_j(gm[b], j, n);
        transpose_quads_over_j(gs[b], j, n);
        if constexpr (PARTS) {          // the raw sums of this part; hot_linear_wgrad_finish_kernel adds the parts up
            const long per = O * K + ((O + 3) & ~3L);       // a multiple of 4 floats: quads stay 16-byte aligned
            float *mine = a.ws + (size_t)blockIdx.y * 2 * (size_t)per;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const long col = k0 + 16 * t + 4 * j;
                if (o_ok[b] && col < K) {
                    store4<true, false>(mine + o[b] * K + col, gm[b][t]);
                    store4<true, false>(mine + per + o[b] * K + col, gs[b][t]);
                }
            }
            if (bias_tile && j == 0 && o_ok[b]) {
                mine[O * K + o[b]] = gb_m[b];
                mine[per + O * K + o[b]] = gb_s[b];
            }
            continue;
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const long col = k0 + 16 * t + 4 * j;
            if (o_ok[b] && col < K) {
                const long at = o[b] * K + col;
                const f4 m4 = load4<true, false>(a.mu_w + at), sd4 = load4<true, false>(a.sigma_w + at);
                f4 om, os;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    float u, v;
                    finish_pair(gm[b][t][c], gs[b][t][c], m4[c], sd4[c], (float)a.g, (float)a.k, u, v);
                    om[c] = u;
                    os[c] = v;
                }
                store4<true, false>(a.gmu_w + at, om);
                store4<true, false>(a.gsig_w + at, os);
            }
        }
        if (bias_tile && j == 0 && o_ok[b]) {
            float u, v;
            finish_pair(gb_m[b], gb_s[b], a.mu_b[o[b]], a.sigma_b[o[b]], (float)a.g, (float)a.k, u, v);
            a.gmu_b[o[b]] = u;
            a.gsig_b[o[b]] = v;
        }
    }
}

// Adds the parts of a PARTS run in their order and finishes the gradients: thread q owns quad q of the
// O*K weights (K is a multiple of 4, so a quad never leaves its row), the first O threads also one bias.
__global__ void __launch_bounds__(256)
hot_linear_wgrad_finish_kernel(LinearGradArgs a, int parts)
{
    const long K = a.in_features, O = a.out_features, per = O * K + ((O + 3) & ~3L);
    const long q = (long)blockIdx.x * 256 + threadIdx.x;
    if (q < O * K / 4) {
        f4 gm = {0.0f, 0.0f, 0.0f, 0.0f}, gs = gm;
        for (int p = 0; p < parts; ++p) {
            const float *theirs = a.ws + (size_t)p * 2 * (size_t)per;
            const f4 u = load4<true, false>(theirs + 4 * q), v = load4<true, false>(theirs + per + 4 * q);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                gm[c] += u[c];
                gs[c] += v[c];
            }
        }
        const f4 m4 = load4<true, false>(a.mu_w + 4 * q), sd4 = load4<true, false>(a.sigma_w + 4 * q);
        f4 om, os;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            float u, v;
            finish_pair(gm[c], gs[c], m4[c], sd4[c], (float)a.g, (float)a.k, u, v);
            om[c] = u;
            os[c] = v;
        }
        store4<true, false>(a.gmu_w + 4 * q, om);
        store4<true, false>(a.gsig_w + 4 * q, os);
    }
    if (a.mu_b != nullptr && q < O) {
        float gm = 0.0f, gs = 0.0f;
        for (int p = 0; p < parts; ++p) {
            const float *theirs = a.ws + (size_t)p * 2 * (size_t)per;
            gm += theirs[O * K + q];
            gs += theirs[per + O * K + q];
        }
        float u, v;
        finish_pair(gm, gs, a.mu_b[q], a.sigma_b[q], (float)a.g, (float)a.k, u, v);
        a.gmu_b[q] = u;
        a.gsig_b[q] = v;
    }
}

// The PARTS run: every tile once per part (grid y), then the finish kernel.
template <int OB>
void wgrad_go_parts(long tiles, int waves, int parts, hipStream_t s, const LinearGradArgs &a)
{
    const long per_xcd = (tiles + kXcds - 1) / kXcds;
    const size_t lds = (size_t)(waves - 1) * OB * kWgradPartials * 64 * sizeof(float);
    hot_linear_wgrad_kernel<true, true, OB, true><<<dim3((unsigned)(kXcds * per_xcd), (unsigned)parts), dim3(64 * waves), lds, s>>>(a);
    const long quads = a.out_features * a.in_features / 4;
    const long threads = quads > a.out_features ? quads : a.out_features;
    hot_linear_wgrad_finish_kernel<<<dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s>>>(a, parts);
}

template <bool SPLIT, bool DEEP, int OB>
void wgrad_go(long tiles, int waves, hipStream_t s, const LinearGradArgs &a)
{
    const long per_xcd = (tiles + kXcds - 1) / kXcds;      // the kernel deals the tiles out by XCD
    const long wgs = SPLIT ? per_xcd : (per_xcd + kWgradWaves - 1) / kWgradWaves;
    const size_t lds = SPLIT ? (size_t)(waves - 1) * OB * kWgradPartials * 64 * sizeof(float) : 0;
    hot_linear_wgrad_kernel<SPLIT, DEEP, OB><<<dim3((unsigned)(kXcds * wgs)), dim3(64 * waves), lds, s>>>(a);
}

// ---------------------------------------------------------------------------------
// Weight gradients of large layers.  The kernel above gives a wave a tile of 16-32 outputs x 64 inputs, about 10
// flops per byte it loads: at thousands of rows the second-level caches cannot feed that (the matrix pipes were 42 %
// busy).  Here a workgroup of four waves owns 128 inputs x 128 outputs and takes 16 rows of x and of dy at a time
// through LDS (32 flops per byte loaded).  The rows go from memory straight into LDS (buffer loads with the LDS
// bit, 16 bytes per lane, consecutive lanes on consecutive addresses): no registers and no vector-ALU instruction
// carry them.  A wave multiplies its 64 inputs x 64 outputs as 2 x 2 blocks of v_mfma_f32_32x32x2_f32 with x as
// the A operand and dy as the B operand, so result registers 4 q .. 4 q + 3 of a lane are the inputs
// 8 q + 4 (lane / 32) .. + 3 of output lane % 32: one generator quad, as above.  Four pairs of buffers take turns: the
// rows of a step are sent for three steps ahead, and the one barrier of a step lies in its middle, with the operands
// of the matrix instructions behind it already in registers (see the row loop); two workgroups share a compute unit,
// so what one still waits for is covered by the other's matrix instructions.  Rows beyond the last
// and columns beyond the layer are masked by offsets outside the range-checked windows and arrive as zeros; a wave
// skips the 32 x 32 blocks that lie outside the layer altogether.  The finished sums leave through LDS so that
// every store instruction covers 128 contiguous bytes per row of the gradient arrays.
// Vector-ALU instructions are kept out of the row loop as far as possible, since each takes its cycles from the
// matrix instructions: the lanes' offsets advance by a uniform step, rows are masked by one comparison per load,
// and the LDS reads carry their offsets as immediates (volatile: merged into two-address reads they needed a
// computed base register each).  Measured on the way, at 4096^3 with two samples: 16-row steps staged through
// registers 123 TFLOP/s; 32-row steps straight into two pairs of LDS buffers, one barrier at the end of a step, one
// set of accumulators for all samples with the eps-weighted sum built by summation by parts (two draws per sample)
// 134; this form 136-139 (the kernel above: 114, the library's GEMM alone: 146) and at 1024 x 8192^2, where the
// draws weigh more, 119 -> 127; tiles of 64 inputs x 256 outputs, 2-8 % slower; row parts through a workspace for
// layers of fewer tiles, behind the kernel above (7260 x 540 x 2160, five or six parts: 0.46-0.49 against 0.42 ms;
// 16640 x 192 x 768: 0.21 against 0.17 ms).
// ---------------------------------------------------------------------------------
constexpr int kTileSide = 128;        // inputs and outputs per workgroup
constexpr int kTileRows = 16;         // rows per step
constexpr int kTurnPitch = 36;        // floats per row of a wave's 32 x 32 block on its way out (16-byte aligned rows)


// WHOLE: every 32 x 32 block of the workgroup's tile reaches into the layer (no block is skipped, no column masked).
// XB, DB: the four buffers of 16 rows x 128 columns of x and of dy.
template <bool WHOLE>
__device__ __forceinline__ void wgrad_tile_body(const LinearGradArgs &a, lds_float *const (&XB)[4], lds_float *const (&DB)[4], long o0, long k0)
{
    constexpr int WK = 2, TK = kTileSide, TO = kTileSide;         // 2 x 2 waves of 64 inputs x 64 outputs
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int wk = wave % WK, wo = wave / WK;
    const long K = a.in_features, O = a.out_features, R = a.rows;

    // which of this wave's 2 x 2 blocks of 32 x 32 reach into the layer (uniform over the wave): the others are skipped
    bool ok[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) ok[i][j] = WHOLE || (k0 + 64 * wk + 32 * i < K && o0 + 64 * wo + 32 * j < O);
    const bool bias_wave = a.mu_b != nullptr && k0 == 0 && wk == 0 && ok[0][0];      // these waves also sum dy over the rows

    // As a loading wave: the tiles go from memory straight into LDS (buffer loads with the LDS bit: lane l of
    // an instruction leaves its 16 bytes at the instruction's LDS address + 16 l, zeros for an offset outside the
    // window), 64 consecutive quads of a tile per instruction, instruction 4 m + wave of the tile for this wave.
    // A quad outside the layer's columns gets a row number that is never below the rows left.
    constexpr int XI = kTileRows * TK / 4 / 256, DI = kTileRows * TO / 4 / 256;       // instructions per wave and tile
    int x_row[XI], d_row[DI];
    unsigned x_first[XI], d_first[DI];
#pragma unroll
    for (int m = 0; m < XI; ++m) {
        const int idx = (4 * m + wave) * 64 + lane;
        const long col = k0 + 4 * (idx % (TK / 4));
        x_row[m] = (WHOLE || col < K) ? idx / (TK / 4) : 1 << 30;
        x_first[m] = (unsigned)((idx / (TK / 4) * a.ldx + col) * 4);
    }
#pragma unroll
    for (int m = 0; m < DI; ++m) {
        const int idx = (4 * m + wave) * 64 + lane;
        const long col = o0 + 4 * (idx % (TO / 4));
        d_row[m] = (WHOLE || col < O) ? idx / (TO / 4) : 1 << 30;
        d_first[m] = (unsigned)((idx / (TO / 4) * O + col) * 4);
    }
    const unsigned x_step = (unsigned)(kTileRows * a.ldx * 4), d_step = (unsigned)(kTileRows * O * 4);
    const int rows = (int)R;

    // The products of one sample over all rows, into the accumulators mm (and the column sums of dy into sb).
    // A step is 16 rows; four buffers, loads three steps ahead.  Step i (buffers i % 4): read the operands of its last 8
    // rows; matrix instructions of its first 8 rows, whose operands are in registers already; wait for the loads
    // of step i + 1 (sent for two steps ago; those of step i + 2 may still be on their way), barrier; send for step
    // i + 3 (its buffers held step i - 1, read for the last time before this barrier); matrix instructions of the last 8
    // rows, with the reads of the first operands of step i + 1 ahead of their last quarter.  Nothing behind the barrier waits for LDS or memory.  The steps are taken four at a time so that
    // every access names its buffer; up to three steps behind the last row run on zeros.
    auto all_rows = [&](int s, Acc32x32 (&mm)[2][2], float (&sb)[2]) {
        const window_t x_win = window(a.x + (size_t)s * (size_t)a.x_sample_stride, (unsigned)(((R - 1) * a.ldx + K) * 4));
        const window_t d_win = window(a.dy + (size_t)s * (size_t)R * (size_t)O, (unsigned)(R * O * 4));
        unsigned x_off[XI], d_off[DI];
#pragma unroll
        for (int m = 0; m < XI; ++m) x_off[m] = x_first[m];
#pragma unroll
        for (int m = 0; m < DI; ++m) d_off[m] = d_first[m];

        // requests the next 16 rows of both operands, of which rows_left exist, into one pair of buffers
        auto request = [&](lds_float *xt, lds_float *dt, int rows_left) {
#pragma unroll
            for (int m = 0; m < XI; ++m) {
                __builtin_amdgcn_raw_ptr_buffer_load_lds(x_win, (lds_void *)(xt + (4 * m + wave) * 256), 16,
                                                         (int)(x_row[m] < rows_left ? x_off[m] : kOutside), 0, 0, 0);
                x_off[m] += x_step;
            }
#pragma unroll
            for (int m = 0; m < DI; ++m) {
                __builtin_amdgcn_raw_ptr_buffer_load_lds(d_win, (lds_void *)(dt + (4 * m + wave) * 256), 16,
                                                         (int)(d_row[m] < rows_left ? d_off[m] : kOutside), 0, 0, 0);
                d_off[m] += d_step;
            }
        };
        constexpr int P = kTileRows / 2, H = P / 2;       // pairs of rows per step and per half-step
        float av[P][2], bv[P][2];
        auto read_half = [&](int h, const lds_float *xt, const lds_float *dt) {
            const volatile lds_float *xb = xt + half * TK + 64 * wk + l32;
            const volatile lds_float *db = dt + half * TO + 64 * wo + l32;
#pragma unroll
            for (int p = h * H; p < (h + 1) * H; ++p)
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    av[p][i] = xb[2 * p * TK + 32 * i];
                    bv[p][i] = db[2 * p * TO + 32 * i];
                }
        };
        auto multiply = [&](int p0, int p1) {
            if (bias_wave) {
#pragma unroll
                for (int p = p0; p < p1; ++p) {
                    sb[0] += bv[p][0];
                    sb[1] += bv[p][1];
                }
            }
            if constexpr (WHOLE) {
#pragma unroll
                for (int p = p0; p < p1; ++p)
#pragma unroll
                    for (int i = 0; i < 2; ++i)
#pragma unroll
                        for (int j = 0; j < 2; ++j) mm[i][j].mac(av[p][i], bv[p][j]);
            } else {
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        if (ok[i][j]) {
#pragma unroll
                            for (int p = p0; p < p1; ++p) mm[i][j].mac(av[p][i], bv[p][j]);
                        }
            }
        };

        request(XB[0], DB[0], rows);
        request(XB[1], DB[1], rows - kTileRows);
        request(XB[2], DB[2], rows - 2 * kTileRows);
        everything_arrived_then_barrier();
        if constexpr (kTileBf16) {
            // On the bf16 matrix instruction (see split2_bf16): the 16 rows of a step are its contraction block.  Lanes
            // 0-31 hold the even rows of a column, lanes 32-63 the odd ones, on both sides alike.  A step reads its
            // operands, cuts them into pieces, multiplies, and meets the others at the barrier, behind which the
            // buffers of the step before are refilled.
            for (int left = rows; left > 0;) {
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    read_half(0, XB[b], DB[b]);
                    read_half(1, XB[b], DB[b]);
                    if (bias_wave) {
#pragma unroll
                        for (int p = 0; p < P; ++p) {
                            sb[0] += bv[p][0];
                            sb[1] += bv[p][1];
                        }
                    }
                    bf8 a1[2], a2[2], a3[2];
#pragma unroll
                    for (int i = 0; i < 2; ++i)
                        split8_bf16(f4{av[0][i], av[1][i], av[2][i], av[3][i]}, f4{av[4][i], av[5][i], av[6][i], av[7][i]}, a1[i], a2[i], a3[i]);
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        bf8 b1, b2, b3;
                        split8_bf16(f4{bv[0][j], bv[1][j], bv[2][j], bv[3][j]}, f4{bv[4][j], bv[5][j], bv[6][j], bv[7][j]}, b1, b2, b3);
#pragma unroll
                        for (int i = 0; i < 2; ++i)
                            if (WHOLE || ok[i][j]) {
                                mm[i][j].mac(a3[i], b1);
                                mm[i][j].mac(a2[i], b2);
                                mm[i][j].mac(a1[i], b3);
                                mm[i][j].mac(a2[i], b1);
                                mm[i][j].mac(a1[i], b2);
                                mm[i][j].mac(a1[i], b1);
                            }
                    }
                    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(XI + DI) : "memory");
                    request(XB[(b + 3) % 4], DB[(b + 3) % 4], left - 3 * kTileRows);
                    left -= kTileRows;
                }
            }
            everything_arrived_then_barrier();       // every wave is done with the buffers
            return;
        }
        read_half(0, XB[0], DB[0]);
        for (int left = rows; left > 0;) {
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                read_half(1, XB[b], DB[b]);
                multiply(0, H);
                // all but the loads sent for last (XI + DI of them, for step i + 2) have arrived, and this wave's reads
                asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(XI + DI) : "memory");
                request(XB[(b + 3) % 4], DB[(b + 3) % 4], left - 3 * kTileRows);
                multiply(H, P - 1);
                read_half(0, XB[(b + 1) % 4], DB[(b + 1) % 4]);
                multiply(P - 1, P);
                left -= kTileRows;
            }
        }
        everything_arrived_then_barrier();       // every wave is done with the buffers
    };

    // Two samples at a time, each with accumulators of its own: P_s = sum_r x_s[r] (x) dy_s[r], whose sum and whose sum
    // weighted with eps_s leave together (one draw per sample and weight).  Further pairs of samples add to what the
    // pairs before left in the gradient arrays (the same thread holds the same weights every time); the last pair
    // applies the scale and the KL part.
    float gb_m[2] = {0.0f, 0.0f}, gb_s[2] = {0.0f, 0.0f};
    lds_float *const mine = XB[wave];        // a buffer per wave for turning its blocks on their way out
    for (int s0 = 0; s0 < a.s_loc; s0 += 2) {
        const bool two = s0 + 1 < a.s_loc, first = s0 == 0, last = s0 + 2 >= a.s_loc;
        Acc32x32 m0[2][2], m1[2][2];
        float sb0[2] = {0.0f, 0.0f}, sb1[2] = {0.0f, 0.0f};
        all_rows(s0, m0, sb0);
        if (two) all_rows(s0 + 1, m1, sb1);
        const MfmaSettled settled;

        long o0e = o0 + 64 * wo, k0e = k0 + 64 * wk;
        asm volatile("" : "+v"(o0e), "+v"(k0e));       // (so that the addresses below are formed here, not ahead of the row loops)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                if (!ok[i][j]) continue;
                const f16v p0 = m0[i][j].read(settled), p1 = m1[i][j].read(settled);      // (p1 is zero without a second sample)
                const long o = o0e + 32 * j + l32;
                f4 u[4], v[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const long k = k0e + 32 * i + 8 * q + 4 * half;
                    f4 sum = {0.0f, 0.0f, 0.0f, 0.0f}, wsum = {0.0f, 0.0f, 0.0f, 0.0f};
                    if (WHOLE || (o < O && k < K)) {
                        const long quad = a.weight_quad0 + ((o * K + k) >> 2);
                        const f4 e0 = eps_quad(quad, s0, a.rng);
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            sum[c] = p0[4 * q + c];
                            wsum[c] = p0[4 * q + c] * e0[c];
                        }
                        if (two) {
                            const f4 e1 = eps_quad(quad, s0 + 1, a.rng);
#pragma unroll
                            for (int c = 0; c < 4; ++c) {
                                sum[c] += p1[4 * q + c];
                                wsum[c] = __builtin_fmaf(p1[4 * q + c], e1[c], wsum[c]);
                            }
                        }
                    }
                    u[q] = sum;
                    v[q] = wsum;
                }
                // Only this wave touches its buffer and the LDS executes a wave's instructions in order: program order suffices.
                f4 ut[4], vt[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) *reinterpret_cast<lds_f4 *>(mine + l32 * kTurnPitch + 8 * q + 4 * half) = u[q];
#pragma unroll
                for (int it = 0; it < 4; ++it) ut[it] = *reinterpret_cast<const lds_f4 *>(mine + (8 * it + (lane >> 3)) * kTurnPitch + 4 * (lane & 7));
#pragma unroll
                for (int q = 0; q < 4; ++q) *reinterpret_cast<lds_f4 *>(mine + l32 * kTurnPitch + 8 * q + 4 * half) = v[q];
#pragma unroll
                for (int it = 0; it < 4; ++it) vt[it] = *reinterpret_cast<const lds_f4 *>(mine + (8 * it + (lane >> 3)) * kTurnPitch + 4 * (lane & 7));
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    const int row = 8 * it + (lane >> 3), quad = lane & 7;
                    const long oo = o0e + 32 * j + row, k = k0e + 32 * i + 4 * quad;
                    if (WHOLE || (oo < O && k < K)) {
                        const long at = oo * K + k;
                        f4 om = ut[it], os = vt[it];
                        if (!first) {
                            om += load4<true, false>(a.gmu_w + at);
                            os += load4<true, false>(a.gsig_w + at);
                        }
                        if (last) {
                            const f4 m4 = load4<true, false>(a.mu_w + at), sd4 = load4<true, false>(a.sigma_w + at);
#pragma unroll
                            for (int c = 0; c < 4; ++c) {
                                float pm, ps;
                                finish_pair(om[c], os[c], m4[c], sd4[c], (float)a.g, (float)a.k, pm, ps);
                                om[c] = pm;
                                os[c] = ps;
                            }
                        }
                        store4<true, false>(a.gmu_w + at, om);
                        store4<true, false>(a.gsig_w + at, os);
                    }
                }
            }
        if (bias_wave) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const long o = o0 + 64 * wo + 32 * j + l32;
                if (o < O) {
                    const float t0 = sb0[j] + __shfl_xor(sb0[j], 32);     // even and odd rows of the steps
                    gb_m[j] += t0;
                    gb_s[j] = __builtin_fmaf(t0, pick4(eps_quad(a.bias_quad0 + (o >> 2), s0, a.rng), (int)(o & 3)), gb_s[j]);
                    if (two) {
                        const float t1 = sb1[j] + __shfl_xor(sb1[j], 32);
                        gb_m[j] += t1;
                        gb_s[j] = __builtin_fmaf(t1, pick4(eps_quad(a.bias_quad0 + (o >> 2), s0 + 1, a.rng), (int)(o & 3)), gb_s[j]);
                    }
                }
            }
        }
        everything_arrived_then_barrier();       // (the buffers go back to the rows of the next pair)
    }
    if (bias_wave && half == 0) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const long o = o0 + 64 * wo + 32 * j + l32;
            if (o < O) {
                float p, r;
                finish_pair(gb_m[j], gb_s[j], a.mu_b[o], a.sigma_b[o], (float)a.g, (float)a.k, p, r);
                a.gmu_b[o] = p;
                a.gsig_b[o] = r;
            }
        }
    }
}

__global__ void __launch_bounds__(256, 2)
hot_linear_wgrad_tile_kernel(LinearGradArgs a)
{
    constexpr int TK = kTileSide, TO = kTileSide;
    // four pairs of operand buffers, [16][128] of x and of dy each; at the end every wave turns its blocks in one of them
    __shared__ __attribute__((aligned(16))) float x0[kTileRows * TK], x1[kTileRows * TK], x2[kTileRows * TK], x3[kTileRows * TK];
    __shared__ __attribute__((aligned(16))) float d0[kTileRows * TO], d1[kTileRows * TO], d2[kTileRows * TO], d3[kTileRows * TO];
    static_assert(kTileRows * TK >= 32 * kTurnPitch, "a wave's block fits in any of the buffers");
    lds_float *XB[4], *DB[4];           // (filled by assignments: as a constant table of LDS addresses it would not link)
    XB[0] = (lds_float *)x0, XB[1] = (lds_float *)x1, XB[2] = (lds_float *)x2, XB[3] = (lds_float *)x3;
    DB[0] = (lds_float *)d0, DB[1] = (lds_float *)d1, DB[2] = (lds_float *)d2, DB[3] = (lds_float *)d3;
    const long K = a.in_features, O = a.out_features;
    const long k_tiles = (K + TK - 1) / TK, o_tiles = (O + TO - 1) / TO;
    const long tiles = k_tiles * o_tiles, per_xcd = (tiles + kXcds - 1) / kXcds;
    const long xcd = blockIdx.x % kXcds, nth = blockIdx.x / kXcds;      // the tiles are dealt out by XCD as above
    const long tile = xcd * per_xcd + nth;
    if (nth >= per_xcd || tile >= tiles) return;          // the whole workgroup
    // The tile list runs through bands of eight rows of tiles, column by column inside a band, so that the 64 tiles an
    // XCD works on at a time are about 8 x 8 and share 16 columns of x and dy in its L2 (listed row by row they were
    // 2 x 32 and shared 34).
    const long band = tile / (8 * k_tiles), bands = o_tiles / 8;
    const long height = band < bands ? 8 : o_tiles - 8 * bands, within = tile - (band < bands ? band : bands) * 8 * k_tiles;
    const long o0 = (8 * (band < bands ? band : bands) + within % height) * TO;
    const long k0 = (within / height) * TK;
    // (uniform over the workgroup, so all its waves meet at the same barriers)
    if (k0 + TK <= K && o0 + TO <= O) wgrad_tile_body<true>(a, XB, DB, o0, k0);
    else wgrad_tile_body<false>(a, XB, DB, o0, k0);
}

// Whether the kernel above can address this problem (its windows take 32-bit byte offsets).
inline bool wgrad_tile_fits(const hot_linear_desc *d)
{
    const unsigned long long lim = 0xFFFFFFF0ull;
    if (d->out_features & 3) return false;        // rows of dy are read in 16-byte quads
    return (unsigned long long)((d->rows + kTileRows) * d->ldx + d->in_features) * 4 < lim &&
           (unsigned long long)(d->rows + kTileRows) * d->out_features * 4 < lim;
}

inline long wgrad_tile_count(const hot_linear_desc *d)
{
    return ((d->in_features + kTileSide - 1) / kTileSide) * ((d->out_features + kTileSide - 1) / kTileSide);
}

void wgrad_tile_go(hipStream_t s, const LinearGradArgs &a, long tiles)
{
    const long per_xcd = (tiles + kXcds - 1) / kXcds;
    hot_linear_wgrad_tile_kernel<<<dim3((unsigned)(kXcds * per_xcd)), dim3(256), 0, s>>>(a);
}

// A wave's finished 64-input x 16*RB-row tile of one sample's dx goes to memory.  Register rr of accumulator
// i is input k0 + 16 j + 4 rr + i of row r0 + 16 rb + n; the lanes of a row exchange quads so that each store
// covers 64 contiguous bytes of the row.  Every lane of the wave must call it.
template <int RB>
__device__ __forceinline__ void store_dx_tile(const f4 (&acc)[RB][4], float *dx, int s, long r0, long k0, int j, int n,
                                              const LinearGradArgs &a)
{
    const long K = a.in_features, R = a.rows;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const long row = r0 + kRowsPerTile * rb + n;
        f4 q[4];
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) q[rr] = f4{acc[rb][0][rr], acc[rb][1][rr], acc[rb][2][rr], acc[rb][3][rr]};
        transpose_quads_over_j(q, j, n);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const long col = k0 + 16 * t + 4 * j;
            if (row < R && col < K)
                store4<true, false>(dx + ((size_t)s * (size_t)R + (size_t)row) * (size_t)K + (size_t)col, q[t]);
        }
    }
}

// A workgroup owns 64 inputs x 16*RB rows of one sample's dx; its waves take the outputs in blocks
// of sixteen, round-robin, and their partial tiles are added through LDS in wave order.
constexpr int kXgradOutputsPerStep = 16;
template <int RB>
__global__ void __launch_bounds__(64 * max_waves(RB), RB >= 4 ? 2 : 1)
hot_linear_xgrad_kernel(LinearGradArgs a)
{
    extern __shared__ float partial[];   // [waves - 1][RB * 16][64]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, waves = blockDim.x >> 6;
    const int n = lane & 15, j = lane >> 4;
    const long K = a.in_features, O = a.out_features, R = a.rows;
    const long k0 = (long)blockIdx.x * 64, r0 = (long)blockIdx.y * (kRowsPerTile * RB);
    const int s = blockIdx.z;
    const float *dys = a.dy + (size_t)s * (size_t)R * (size_t)O;
    const long kq = k0 + 4 * n;          // this lane's quad of inputs (as an A lane)
    const bool k_ok = kq < K;

    Acc16x16 mm[RB][4];

    // dy is read as quads of four consecutive outputs (lane (n, j): outputs ob + 4 j .. + 3 of row n; dword
    // alignment suffices), and matrix instruction (c, i) takes element c of them against element i of the
    // weight quad of output ob + 4 j + c: one 16-byte load per row block where single values took four loads.
    // Rows beyond R read row R - 1: they only reach accumulator columns that are never stored.
    long at[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const long row = r0 + kRowsPerTile * rb + n;
        at[rb] = (row < R ? row : R - 1) * O + 4 * j;
    }
    for (long ob = (long)wave * kXgradOutputsPerStep; ob < O; ob += (long)waves * kXgradOutputsPerStep) {
        f4 m4[4], sd4[4], dyq[RB];
        bool ok[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const long o = ob + 4 * j + c;
            ok[c] = k_ok && o < O;
            m4[c] = ok[c] ? load4<true, false>(a.mu_w + o * K + kq) : f4{0.0f, 0.0f, 0.0f, 0.0f};
            sd4[c] = ok[c] ? load4<true, false>(a.sigma_w + o * K + kq) : f4{0.0f, 0.0f, 0.0f, 0.0f};
        }
        if (ob + kXgradOutputsPerStep <= O) {        // uniform over the wave
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) dyq[rb] = load4<false, false>(dys + at[rb] + ob);
        } else {                                     // last, partial step: outputs beyond O contribute zeros
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int c = 0; c < 4; ++c) dyq[rb][c] = ob + 4 * j + c < O ? dys[at[rb] + ob + c] : 0.0f;
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            f4 w4 = {0.0f, 0.0f, 0.0f, 0.0f};
            if (ok[c]) {
                const long o = ob + 4 * j + c;
                const f4 e = eps_quad(a.weight_quad0 + ((o * K + kq) >> 2), s, a.rng);
#pragma unroll
                for (int i = 0; i < 4; ++i) w4[i] = __builtin_fmaf(sd4[c][i], e[i], m4[c][i]);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
                    mm[rb][i].mac(w4[i], dyq[rb][c]);
        }
    }
    const MfmaSettled settled;
    f4 acc[RB][4];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[rb][i] = mm[rb][i].read(settled);

    if (waves > 1) {
        if (wave > 0) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr)
                        partial[((wave - 1) * (RB * 16) + (rb * 4 + i) * 4 + rr) * 64 + lane] = acc[rb][i][rr];
        }
        __syncthreads();
        if (wave == 0) {
            for (int v = 1; v < waves; ++v)
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int rr = 0; rr < 4; ++rr)
                            acc[rb][i][rr] += partial[((v - 1) * (RB * 16) + (rb * 4 + i) * 4 + rr) * 64 + lane];
        }
    }
    if (wave != 0) return;

    store_dx_tile<RB>(acc, a.dx, s, r0, k0, j, n, a);
}

// ---------------------------------------------------------------------------------
// Input gradients for many rows: as in the forward kernel for many rows, the four waves of a workgroup
// take up to 64 rows each and share every draw through LDS.  A workgroup owns 64 inputs x 256 rows of one
// sample's dx and walks over the outputs 16 at a time: each of its 256 threads draws one quad of the
// 16-output x 64-input weight tile (wave c, lane (m, j): output ob + 4 j + c, inputs k0 + 4 m .. + 3) into
// LDS, and after one barrier every wave reads the four quads of its lane position and multiplies its own
// 64 rows: 64 matrix instructions per drawn quad instead of 16.  A lane reads dy as quads of four
// consecutive outputs (one 16-byte load per row block and iteration; dy needs dword alignment only) and
// matrix instruction (c, i) takes element c of the dy quads against element i of weight quad c: the
// contraction index is only enumerated in another order.  Tile double-buffered, one barrier per iteration,
// as in the forward kernel; accumulators and epilogue are those of the kernel above.
// ---------------------------------------------------------------------------------
constexpr int kXgradRowsKernelOutputs = 16;    // outputs per iteration: one drawn quad per thread
constexpr int kXgradMaxParts = 16;             // most parts the outputs are cut into with a workspace

// RB: 16-row blocks per wave (a workgroup owns 64 RB rows); fewer of them where 256-row workgroups would be too few.
template <int RB>
__global__ void __launch_bounds__(256)
hot_linear_xgrad_rows_kernel(LinearGradArgs a)
{
    __shared__ __attribute__((aligned(16))) float tile[2][4 * 64 * 4];     // [buffer][c][j][m] quads
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15, j = lane >> 4;
    const long K = a.in_features, O = a.out_features, R = a.rows;
    // with a workspace the outputs may be cut into parts for different workgroups (grid x = input groups x parts):
    // this one contracts over the outputs o_lo .. o_hi - 1 only and leaves its block in the workspace
    const long k_groups = (K + 63) / 64;
    const long part = (long)blockIdx.x / k_groups, k0 = ((long)blockIdx.x % k_groups) * 64;
    const long o_lo = a.x_parts > 1 ? part * a.outs_per_part : 0;
    const long o_hi = a.x_parts > 1 && o_lo + a.outs_per_part < O ? o_lo + a.outs_per_part : O;
    const long r0 = ((long)blockIdx.y * 4 + wave) * (kRowsPerTile * RB);
    const int s = blockIdx.z;
    const float *dys = a.dy + (size_t)s * (size_t)R * (size_t)O;
    const long kq = k0 + 4 * n;          // this lane's quad of inputs (as a drawing thread and as an A lane)
    const bool k_ok = kq < K;

    Acc16x16 mm[RB][4];
    // rows beyond R read row R - 1 instead: they only reach columns of the accumulators that are never stored
    long at[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const long row = r0 + kRowsPerTile * rb + n;
        at[rb] = (row < R ? row : R - 1) * O + 4 * j;
    }

    int buf = 0;
    for (long ob = o_lo; ob < o_hi; ob += kXgradRowsKernelOutputs, buf ^= 1) {
        const long o_draw = ob + 4 * j + wave;
        const bool draw_ok = k_ok && o_draw < o_hi;
        f4 w4 = {0.0f, 0.0f, 0.0f, 0.0f};
        f4 dyq[RB];
        if (ob + kXgradRowsKernelOutputs <= o_hi) {      // uniform
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) dyq[rb] = load4<false, false>(dys + at[rb] + ob);
        } else {                                         // last, partial step: outputs beyond O contribute zeros
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int c = 0; c < 4; ++c) dyq[rb][c] = ob + 4 * j + c < o_hi ? dys[at[rb] + ob + c] : 0.0f;
        }
        if (draw_ok) {
            const f4 m4 = load4<true, false>(a.mu_w + o_draw * K + kq), sd4 = load4<true, false>(a.sigma_w + o_draw * K + kq);
            const f4 e = eps_quad(a.weight_quad0 + ((o_draw * K + kq) >> 2), s, a.rng);
#pragma unroll
            for (int c = 0; c < 4; ++c) w4[c] = __builtin_fmaf(sd4[c], e[c], m4[c]);
        }
        *reinterpret_cast<f4 *>(&tile[buf][((wave * 4 + j) * 16 + n) * 4]) = w4;
        __syncthreads();
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const f4 wq = *reinterpret_cast<const f4 *>(&tile[buf][((c * 4 + j) * 16 + n) * 4]);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
                    mm[rb][i].mac(wq[i], dyq[rb][c]);
        }
    }
    const MfmaSettled settled;
    f4 acc[RB][4];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[rb][i] = mm[rb][i].read(settled);

    float *dst = a.x_parts > 1 ? a.ws + (size_t)part * (size_t)a.s_loc * (size_t)R * (size_t)K : a.dx;
    store_dx_tile<RB>(acc, dst, s, r0, k0, j, n, a);
}

// dx = the sum of the parts' blocks in the workspace, in part order; one quad per thread.
__global__ void __launch_bounds__(256)
hot_linear_dx_sum_kernel(float *__restrict__ dx, const float *__restrict__ ws, long quads, int parts)
{
    const long q = (long)blockIdx.x * 256 + threadIdx.x;
    if (q >= quads) return;
    f4 sum = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int p = 0; p < parts; ++p) {
        const f4 v = load4<true, false>(ws + (size_t)p * (size_t)quads * 4 + (size_t)q * 4);
#pragma unroll
        for (int c = 0; c < 4; ++c) sum[c] += v[c];
    }
    store4<true, false>(dx + (size_t)q * 4, sum);
}

// ---------------------------------------------------------------------------------
// Few rows (at most 32) with the input gradients wanted: both gradients in ONE pass over the weights.  The kernels
// above each draw every eps of the layer, and at few rows the draw is most of their time (four generator quads
// per lane and 16 x 64 tile: about 2600 vector cycles, against 512 matrix cycles per 16 rows and product); here a
// wave draws the quads of its tile once per sample and uses them for both products.  No drawn value has to move
// between lanes for that: with dy as the A operand and element i of a lane's quad of x as the B operand, result
// register rr of accumulator i is G[ob + 4 j + rr][k0 + 4 n + i], so lane (n, j) receives the weight gradients of
// exactly the four quads (outputs ob + 4 j + c, inputs k0 + 4 n .. + 3) that the input-gradient kernel has it draw.
//
// A workgroup of four waves owns 64 inputs (its strip of x waits in LDS) and one part of the outputs; its waves
// take that part's 16-output tiles round-robin, and the accumulators of every sample's dx stay in registers over
// the whole loop (16 RB per sample and lane: that bounds rows x samples).  Per tile and sample: dy of the tile
// (once per operand layout), the draw, G = dy^T x, sum_s G and sum_s G eps in registers, w = mu + sigma eps in
// the registers of eps, dx += dy w; the loads of a sample (and of the tile's mu, sigma) are issued before its draw.  After the last
// sample the tile's gradients are finished and stored, 256 contiguous bytes per output row.  At the end the
// waves' dx tiles are added through LDS in wave order and go to the workspace as this part's block (straight to
// dx if the layer has one part); hot_linear_dx_sum_kernel adds the blocks in part order.  No atomics.
// ---------------------------------------------------------------------------------
constexpr int kOnePassWaves = 4;
constexpr int kOnePassMaxRows = 32;
constexpr int kOnePassAccumulators = 8;     // most (16-row blocks) x (samples) whose dx accumulators a lane holds

template <int RB, int SMAX>
__global__ void __launch_bounds__(64 * kOnePassWaves, RB * SMAX <= 4 ? 2 : 1)
hot_linear_backward_one_pass_kernel(LinearGradArgs a)
{
    extern __shared__ __attribute__((aligned(16))) float strip[];   // [copies of x][16 RB rows][64 inputs]; at the end [waves - 1][16 RB][64]
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15, j = lane >> 4;
    const long K = a.in_features, O = a.out_features, R = a.rows;
    const long k0 = (long)blockIdx.x * 64;
    const long part = blockIdx.y;
    const long o_lo = part * a.outs_per_part;
    const long o_hi = o_lo + a.outs_per_part < O ? o_lo + a.outs_per_part : O;
    const long kq = k0 + 4 * n;             // this lane's quad of inputs
    const bool k_ok = kq < K;
    const bool bias_strip = a.mu_b != nullptr && blockIdx.x == 0;    // this strip's workgroups also own the biases of their outputs
    constexpr int kStripQuads = 16 * RB * 16;
    const float gf = (float)a.g, kf = (float)a.k;

    // rows beyond R and inputs beyond K enter as zeros: they are summed over
    const int copies = a.x_sample_stride != 0 ? a.s_loc : 1;
    for (int at = threadIdx.x; at < copies * kStripQuads; at += 64 * kOnePassWaves) {
        const int copy = at / kStripQuads, rest = at % kStripQuads, row = rest >> 4, q = rest & 15;
        f4 v = {0.0f, 0.0f, 0.0f, 0.0f};
        if (row < R && k0 + 4 * q < K)
            v = load4<true, false>(a.x + (size_t)copy * (size_t)a.x_sample_stride + (size_t)row * (size_t)a.ldx + (size_t)(k0 + 4 * q));
        *reinterpret_cast<f4 *>(strip + (size_t)at * 4) = v;
    }
    __syncthreads();

    // dx: register rr of mx[s][rb][i] is input k0 + 16 j + 4 rr + i of row 16 rb + n of sample s
    Acc16x16 mx[SMAX][RB][4];

    // Lanes outside the layer (outputs >= O, inputs >= K) read a valid address instead; what they read is never used.
    auto fetch_parameters = [&](long ob, f4 (&m)[4], f4 (&sd)[4]) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const long o = ob + 4 * j + c;
            const long at = (o < O ? o : O - 1) * K + (k_ok ? kq : 0);
            m[c] = load4<true, false>(a.mu_w + at);
            sd[c] = load4<true, false>(a.sigma_w + at);
        }
    };

    // dy of a tile and sample, once per operand layout: as the A operand of G (lane (n, j): output ob + n, rows 4 q + j; rows
    // beyond R are zeros) and as the B operand of dx (row 16 rb + n, outputs ob + 4 j .. + 3; rows beyond R read row R - 1,
    // which only reaches columns of the accumulators that are never stored; outputs beyond O must be zeros)
    auto fetch_dy = [&](long ob, int s, float (&dya)[4 * RB], f4 (&dyq)[RB]) {
        const float *dys = a.dy + (size_t)s * (size_t)R * (size_t)O;
        const long o_a = ob + n < O ? ob + n : O - 1;
#pragma unroll
        for (int q = 0; q < 4 * RB; ++q) {      // (rows beyond R: row R - 1 for now; zeroed where the values are used, behind the draw)
            const long row = 4 * q + j;
            dya[q] = dys[(row < R ? row : R - 1) * O + o_a];
        }
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const long row = 16 * rb + n;
            const float *at = dys + (row < R ? row : R - 1) * O + ob + 4 * j;
            if (ob + 16 <= O) dyq[rb] = load4<false, false>(at);       // uniform over the wave
            else {
#pragma unroll
                for (int c = 0; c < 4; ++c) dyq[rb][c] = ob + 4 * j + c < O ? at[c] : 0.0f;
            }
        }
    };

    // The loads of a tile's first sample and of its mu, sigma are issued at the end of the tile before, ahead of that
    // tile's stores: loads and stores complete in order, and a wait for a load issued behind the stores would also wait
    // until the gradients have reached memory.  A wave without tiles fetches a valid tile and uses nothing.
    const long ob_first = o_lo + 16 * wave;
    f4 m4[4], sd4[4];
    float dya0[4 * RB];
    f4 dyq0[RB];
    fetch_parameters(ob_first < o_hi ? ob_first : o_lo, m4, sd4);
    fetch_dy(ob_first < o_hi ? ob_first : o_lo, 0, dya0, dyq0);
    for (long ob = ob_first; ob < o_hi; ob += 16 * kOnePassWaves) {
        bool ok[4];
        long quad[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const long o = ob + 4 * j + c;
            ok[c] = k_ok && o < O;
            quad[c] = a.weight_quad0 + (((o < O ? o : O - 1) * K + (k_ok ? kq : 0)) >> 2);
        }
        f4 gm[4], gs[4], gbm = {0.0f, 0.0f, 0.0f, 0.0f}, gbs = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int c = 0; c < 4; ++c) gm[c] = gs[c] = f4{0.0f, 0.0f, 0.0f, 0.0f};

#pragma unroll
        for (int s = 0; s < SMAX; ++s) {
            if (s < a.s_loc) {                  // uniform over the grid
                float dya[4 * RB];
                f4 dyq[RB];
                if (s == 0) {
#pragma unroll
                    for (int q = 0; q < 4 * RB; ++q) dya[q] = dya0[q];
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb) dyq[rb] = dyq0[rb];
                } else {
                    fetch_dy(ob, s, dya, dyq);
                }
                // every load of this sample, the rows of x from LDS among them, is on its way before its draw, whose
                // arithmetic covers their latency
                const float *xs = strip + (a.x_sample_stride != 0 ? s : 0) * (kStripQuads * 4);
                constexpr bool kEarlyX = RB * SMAX <= 2;        // (registers for it only in the lightest shape)
                f4 xq[4 * RB];
                if constexpr (kEarlyX) {
#pragma unroll
                    for (int q = 0; q < 4 * RB; ++q) xq[q] = *reinterpret_cast<const f4 *>(xs + (4 * q + j) * 64 + 4 * n);
                }
                __builtin_amdgcn_sched_barrier(0);
                f4 e[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) e[c] = eps_quad(quad[c], s, a.rng);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int q = 0; q < 4 * RB; ++q)
                    if (4 * q + j >= R) dya[q] = 0.0f;

                Acc16x16 mg[4], mb;
#pragma unroll
                for (int q = 0; q < 4 * RB; ++q) {
                    if constexpr (!kEarlyX) xq[q] = *reinterpret_cast<const f4 *>(xs + (4 * q + j) * 64 + 4 * n);
#pragma unroll
                    for (int i = 0; i < 4; ++i) mg[i].mac(dya[q], xq[q][i]);
                }
                if (bias_strip) {               // column sums of dy: the same contraction against ones
#pragma unroll
                    for (int q = 0; q < 4 * RB; ++q) mb.mac(dya[q], 1.0f);
                }
                f4 P[4], Pb;
                {
                    const MfmaSettled settled;
#pragma unroll
                    for (int i = 0; i < 4; ++i) P[i] = mg[i].read(settled);
                    Pb = mb.read(settled);
                }
#pragma unroll
                for (int c = 0; c < 4; ++c)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        gm[c][i] += P[i][c];
                        gs[c][i] = __builtin_fmaf(P[i][c], e[c][i], gs[c][i]);
                    }
                if (bias_strip) {               // register rr of Pb: sum_r dy_s[r][ob + 4 j + rr], the four outputs of one generator quad
                    const f4 eb = eps_quad(a.bias_quad0 + ((ob + 4 * j) >> 2), s, a.rng);
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) {
                        gbm[rr] += Pb[rr];
                        gbs[rr] = __builtin_fmaf(Pb[rr], eb[rr], gbs[rr]);
                    }
                }
#pragma unroll
                for (int c = 0; c < 4; ++c)
#pragma unroll
                    for (int i = 0; i < 4; ++i) e[c][i] = ok[c] ? __builtin_fmaf(sd4[c][i], e[c][i], m4[c][i]) : 0.0f;
#pragma unroll
                for (int c = 0; c < 4; ++c)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int rb = 0; rb < RB; ++rb) mx[s][rb][i].mac(e[c][i], dyq[rb][c]);
            }
        }

        // the tile's gradients; then the next tile's loads into the registers they leave; then the stores
        f4 om[4], os[4];
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float u, v;
                finish_pair(gm[c][i], gs[c][i], m4[c][i], sd4[c][i], gf, kf, u, v);
                om[c][i] = u;
                os[c][i] = v;
            }
        f4 ob_m = {0.0f, 0.0f, 0.0f, 0.0f}, ob_s = {0.0f, 0.0f, 0.0f, 0.0f};
        if (bias_strip) {
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const long o = ob + 4 * j + rr < O ? ob + 4 * j + rr : O - 1;
                float u, v;
                finish_pair(gbm[rr], gbs[rr], a.mu_b[o], a.sigma_b[o], gf, kf, u, v);
                ob_m[rr] = u;
                ob_s[rr] = v;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        {
            const long ob_next = ob + 16 * kOnePassWaves < o_hi ? ob + 16 * kOnePassWaves : ob;
            fetch_parameters(ob_next, m4, sd4);
            fetch_dy(ob_next, 0, dya0, dyq0);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (ok[c]) {
                const long at = (ob + 4 * j + c) * K + kq;
                store4<true, false>(a.gmu_w + at, om[c]);
                store4<true, false>(a.gsig_w + at, os[c]);
            }
        }
        if (bias_strip && n == 0) {
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const long o = ob + 4 * j + rr;
                if (o < O) {
                    a.gmu_b[o] = ob_m[rr];
                    a.gsig_b[o] = ob_s[rr];
                }
            }
        }
    }

    __syncthreads();        // every wave is done with the strip of x: its LDS now carries the waves' partial tiles
    float *dst = a.x_parts > 1 ? a.ws + (size_t)part * (size_t)a.s_loc * (size_t)R * (size_t)K : a.dx;
#pragma unroll
    for (int s = 0; s < SMAX; ++s) {
        if (s < a.s_loc) {
            f4 acc[RB][4];
            {
                const MfmaSettled settled;
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                    for (int i = 0; i < 4; ++i) acc[rb][i] = mx[s][rb][i].read(settled);
            }
            if (wave > 0) {
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int rr = 0; rr < 4; ++rr)
                            strip[((wave - 1) * (RB * 16) + (rb * 4 + i) * 4 + rr) * 64 + lane] = acc[rb][i][rr];
            }
            __syncthreads();
            if (wave == 0) {
                for (int v = 1; v < kOnePassWaves; ++v)
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                        for (int i = 0; i < 4; ++i)
#pragma unroll
                            for (int rr = 0; rr < 4; ++rr)
                                acc[rb][i][rr] += strip[((v - 1) * (RB * 16) + (rb * 4 + i) * 4 + rr) * 64 + lane];
                store_dx_tile<RB>(acc, dst, s, 0, k0, j, n, a);
            }
            __syncthreads();    // the next sample's tiles overwrite these
        }
    }
}

// ---------------------------------------------------------------------------------
// The same one pass for more rows (33 to 128): the four waves of a workgroup split the ROWS (16 RBW each) and share
// every draw.  Per 16-output x 64-input tile and sample, wave c draws quad c of every lane position (output
// ob + 4 j + c, inputs k0 + 4 n .. + 3), forms w = mu + sigma eps and leaves it in LDS; behind a barrier every wave reads
// the four quads of its lane position, which are exactly its A operands of dx += dy w for its own rows, and multiplies
// G = dy^T x over its own rows; the partial G of the waves meet in LDS, and behind a second barrier wave c adds
// those of quad c in wave order and applies the eps that it drew itself.  A wave so holds the dx accumulators of its
// own rows only (16 RBW per sample) and one quad's gradient sums: few registers, several workgroups per compute
// unit, which take turns at the barriers.  No reduction of dx at the end: every wave stores its own rows.
// ---------------------------------------------------------------------------------
constexpr int kSplitRowsWaves = 4;

template <int RBW, int SMAX>
__global__ void __launch_bounds__(64 * kSplitRowsWaves, 2)
hot_linear_backward_split_rows_kernel(LinearGradArgs a)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    // [4][64] quads of drawn weights; [4 waves][5][64] quads of partial G (the fifth: column sums of dy); then the strip of x
    float *const wt = lds, *const gp = lds + 4 * 64 * 4, *const strip = gp + kSplitRowsWaves * 5 * 64 * 4;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15, j = lane >> 4;
    const long K = a.in_features, O = a.out_features, R = a.rows;
    const long k0 = (long)blockIdx.x * 64;
    const long part = blockIdx.y;
    const long o_lo = part * a.outs_per_part;
    const long o_hi = o_lo + a.outs_per_part < O ? o_lo + a.outs_per_part : O;
    const long kq = k0 + 4 * n;
    const bool k_ok = kq < K;
    const bool bias_strip = a.mu_b != nullptr && blockIdx.x == 0;
    const float gf = (float)a.g, kf = (float)a.k;
    constexpr int kRows = 16 * RBW * kSplitRowsWaves;       // rows of the workgroup
    constexpr int kStripQuads = kRows * 16;
    const int r0 = 16 * RBW * wave;                         // this wave's rows

    const int copies = a.x_sample_stride != 0 ? a.s_loc : 1;
    for (int at = threadIdx.x; at < copies * kStripQuads; at += 64 * kSplitRowsWaves) {
        const int copy = at / kStripQuads, rest = at % kStripQuads, row = rest >> 4, q = rest & 15;
        f4 v = {0.0f, 0.0f, 0.0f, 0.0f};
        if (row < R && k0 + 4 * q < K)
            v = load4<true, false>(a.x + (size_t)copy * (size_t)a.x_sample_stride + (size_t)row * (size_t)a.ldx + (size_t)(k0 + 4 * q));
        *reinterpret_cast<f4 *>(strip + (size_t)at * 4) = v;
    }
    __syncthreads();

    // dx of this wave's rows: register rr of mx[s][rb][i] is input k0 + 16 j + 4 rr + i of row r0 + 16 rb + n
    Acc16x16 mx[SMAX][RBW][4];

    for (long ob = o_lo; ob < o_hi; ob += 16) {         // every wave walks every tile of the part
        // this wave's quad of the tile
        const long o_own = ob + 4 * j + wave;
        const bool ok = k_ok && o_own < O;
        const long at_own = (o_own < O ? o_own : O - 1) * K + (k_ok ? kq : 0);
        const f4 m4 = load4<true, false>(a.mu_w + at_own), sd4 = load4<true, false>(a.sigma_w + at_own);
        const long quad = a.weight_quad0 + (at_own >> 2);
        f4 gm = {0.0f, 0.0f, 0.0f, 0.0f}, gs = {0.0f, 0.0f, 0.0f, 0.0f};
        float gbm = 0.0f, gbs = 0.0f;

#pragma unroll
        for (int s = 0; s < SMAX; ++s) {
            if (s < a.s_loc) {                  // uniform over the grid
                const float *dys = a.dy + (size_t)s * (size_t)R * (size_t)O;
                // dy of the tile and this wave's rows, once per operand layout (as in the kernel above), and the rows of x
                float dya[4 * RBW];
                f4 dyq[RBW], xq[4 * RBW];
                const long o_a = ob + n < O ? ob + n : O - 1;
#pragma unroll
                for (int q = 0; q < 4 * RBW; ++q) {
                    const long row = r0 + 4 * q + j;
                    dya[q] = dys[(row < R ? row : R - 1) * O + o_a];
                }
#pragma unroll
                for (int rb = 0; rb < RBW; ++rb) {
                    const long row = r0 + 16 * rb + n;
                    const float *at = dys + (row < R ? row : R - 1) * O + ob + 4 * j;
                    if (ob + 16 <= O) dyq[rb] = load4<false, false>(at);       // uniform over the wave
                    else {
#pragma unroll
                        for (int c = 0; c < 4; ++c) dyq[rb][c] = ob + 4 * j + c < O ? at[c] : 0.0f;
                    }
                }
                const float *xs = strip + (a.x_sample_stride != 0 ? s : 0) * (kStripQuads * 4);
#pragma unroll
                for (int q = 0; q < 4 * RBW; ++q) xq[q] = *reinterpret_cast<const f4 *>(xs + (r0 + 4 * q + j) * 64 + 4 * n);
                __builtin_amdgcn_sched_barrier(0);      // all of it on its way before the draw

                const f4 e = eps_quad(quad, s, a.rng);
                f4 w;
#pragma unroll
                for (int i = 0; i < 4; ++i) w[i] = ok ? __builtin_fmaf(sd4[i], e[i], m4[i]) : 0.0f;
                *reinterpret_cast<f4 *>(wt + (wave * 64 + lane) * 4) = w;
                __syncthreads();        // the tile's four quads per lane position are there (and the sums below have been read)

                f4 wq[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) wq[c] = *reinterpret_cast<const f4 *>(wt + (c * 64 + lane) * 4);
#pragma unroll
                for (int q = 0; q < 4 * RBW; ++q)
                    if (r0 + 4 * q + j >= R) dya[q] = 0.0f;      // rows beyond R are summed over: zeros
                Acc16x16 mg[4], mb;
#pragma unroll
                for (int q = 0; q < 4 * RBW; ++q)
#pragma unroll
                    for (int i = 0; i < 4; ++i) mg[i].mac(dya[q], xq[q][i]);
                if (bias_strip) {
#pragma unroll
                    for (int q = 0; q < 4 * RBW; ++q) mb.mac(dya[q], 1.0f);
                }
#pragma unroll
                for (int c = 0; c < 4; ++c)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int rb = 0; rb < RBW; ++rb) mx[s][rb][i].mac(wq[c][i], dyq[rb][c]);
                {
                    const MfmaSettled settled;
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) {
                        const f4 p = {mg[0].read(settled)[rr], mg[1].read(settled)[rr], mg[2].read(settled)[rr], mg[3].read(settled)[rr]};
                        *reinterpret_cast<f4 *>(gp + ((wave * 5 + rr) * 64 + lane) * 4) = p;
                    }
                    if (bias_strip) *reinterpret_cast<f4 *>(gp + ((wave * 5 + 4) * 64 + lane) * 4) = mb.read(settled);
                }
                __syncthreads();        // the waves' partial sums are there (and every wave has read the drawn quads)

                f4 sum = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int v = 0; v < kSplitRowsWaves; ++v) {
                    const f4 p = *reinterpret_cast<const f4 *>(gp + ((v * 5 + wave) * 64 + lane) * 4);
#pragma unroll
                    for (int i = 0; i < 4; ++i) sum[i] += p[i];
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    gm[i] += sum[i];
                    gs[i] = __builtin_fmaf(sum[i], e[i], gs[i]);
                }
                if (bias_strip) {       // element rr of the fifth quad: sum over the wave's rows of dy_s[r][ob + 4 j + rr]; this wave's output: rr = wave
                    float col = 0.0f;
#pragma unroll
                    for (int v = 0; v < kSplitRowsWaves; ++v)
                        col += pick4(*reinterpret_cast<const f4 *>(gp + ((v * 5 + 4) * 64 + lane) * 4), wave);
                    const f4 eb = eps_quad(a.bias_quad0 + ((ob + 4 * j) >> 2), s, a.rng);
                    gbm += col;
                    gbs = __builtin_fmaf(col, pick4(eb, wave), gbs);
                }
            }
        }

        if (ok) {
            f4 om, os;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float u, v;
                finish_pair(gm[i], gs[i], m4[i], sd4[i], gf, kf, u, v);
                om[i] = u;
                os[i] = v;
            }
            store4<true, false>(a.gmu_w + o_own * K + kq, om);
            store4<true, false>(a.gsig_w + o_own * K + kq, os);
        }
        if (bias_strip && n == 0 && o_own < O) {
            float u, v;
            finish_pair(gbm, gbs, a.mu_b[o_own], a.sigma_b[o_own], gf, kf, u, v);
            a.gmu_b[o_own] = u;
            a.gsig_b[o_own] = v;
        }
    }

    float *dst = a.x_parts > 1 ? a.ws + (size_t)part * (size_t)a.s_loc * (size_t)R * (size_t)K : a.dx;
#pragma unroll
    for (int s = 0; s < SMAX; ++s) {
        if (s < a.s_loc) {
            f4 acc[RBW][4];
            {
                const MfmaSettled settled;
#pragma unroll
                for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
                    for (int i = 0; i < 4; ++i) acc[rb][i] = mx[s][rb][i].read(settled);
            }
            store_dx_tile<RBW>(acc, dst, s, r0, k0, j, n, a);
        }
    }
}

// Launch shape of the two kernels above; rb == 0: the layer goes to the two separate kernels.
struct OnePassPlan {
    int rb, smax;       // split: 16-row blocks per wave; else per workgroup.  smax: samples a lane holds accumulators for
    bool split;         // the waves split the rows and share the draws
    long parts, outs_per_part;
};

// Where the waves split the rows: 33 to 128 rows, one or two samples, half a million weights (measured against the two
// separate kernels at 2 samples: 64 rows 1.5-1.7x at 516 x 2100 to 2160 x 8640, 1.17x at 8192 x 8192; 128 rows 1.45x at
// 540 x 2160, 1.04x at 8192 x 8192; slower on smaller layers, whose few tiles leave the barriers exposed (100 x 260 x 1000:
// 0.93x), with four samples (0.83x at 64 x 2048 x 2048: two waves per SIMD) and at 256 rows x 1 sample (0.88x)).  Up to
// 64 rows it also beats a wave drawing whole tiles for all rows (8192 x 8192: 0.66 against 0.72 ms).
constexpr int kSplitRowsFrom = kOnePassMaxRows + 1, kSplitRowsMaxRows = 128;
constexpr long kSplitRowsMinWeights = 512 * 1024;

// ws_bytes as in wgrad_shape
OnePassPlan one_pass_plan(const hot_linear_desc *d, bool input_gradients, int64_t ws_bytes)
{
    OnePassPlan p{0, 0, false, 1, 0};
    if (!input_gradients || d->rows > kSplitRowsMaxRows) return p;
    int rb, smax;
    bool split = false;
    long budget;        // workgroups that fill the chip once
    if (d->rows >= kSplitRowsFrom) {
        if (d->s_local > 2 || d->in_features * d->out_features < kSplitRowsMinWeights) return p;
        split = true;
        rb = d->rows > 64 ? 2 : 1;
        smax = 2;
        budget = 768;       // (three workgroups share a compute unit)
    } else {
        rb = d->rows > 16 ? 2 : 1;
        smax = d->s_local <= 2 ? 2 : (d->s_local <= 4 ? 4 : 8);
        if (d->s_local > 8 || rb * smax > kOnePassAccumulators) return p;
        budget = rb * smax <= 4 ? 512 : 256;    // (the lighter shapes fit two workgroups on a compute unit)
    }
    const long strips = (d->in_features + 63) / 64, tiles = (d->out_features + 15) / 16;
    // Workgroups for every compute unit from the strips of inputs alone where the strips are that many; fewer strips cut
    // the outputs into parts (a part keeps a tile per wave, four tiles where the waves share them), whose blocks of dx go
    // through the workspace.
    long parts = budget / strips;
    if (parts > tiles / 4) parts = tiles / 4;
    if (parts > 65535) parts = 65535;
    if (parts < 1) parts = 1;
    const int64_t block_bytes = (int64_t)d->s_local * d->rows * d->in_features * (int64_t)sizeof(float);
    if (parts > 1 && ws_bytes >= 0 && parts * block_bytes > ws_bytes) parts = ws_bytes / block_bytes;
    if (parts <= 1) {
        // no workspace (or one too small for two blocks): only where the strips alone nearly fill the chip
        if (strips < 200) return p;
        parts = 1;
    }
    p.outs_per_part = (tiles + parts - 1) / parts * 16;
    p.parts = (d->out_features + p.outs_per_part - 1) / p.outs_per_part;       // every part begins below O
    p.rb = rb;
    p.smax = smax;
    p.split = split;
    return p;
}

template <int RB, int SMAX>
void one_pass_go(const OnePassPlan &p, hipStream_t s, const LinearGradArgs &a)
{
    const size_t strip_bytes = (size_t)SMAX * 16 * RB * 64 * sizeof(float);
    const size_t tiles_bytes = (size_t)(kOnePassWaves - 1) * 16 * RB * 64 * sizeof(float);
    const dim3 grid((unsigned)((a.in_features + 63) / 64), (unsigned)p.parts);
    hot_linear_backward_one_pass_kernel<RB, SMAX><<<grid, dim3(64 * kOnePassWaves), strip_bytes > tiles_bytes ? strip_bytes : tiles_bytes, s>>>(a);
}

template <int RBW, int SMAX>
void split_rows_go(const OnePassPlan &p, hipStream_t s, const LinearGradArgs &a)
{
    const int copies = a.x_sample_stride != 0 ? a.s_loc : 1;
    const size_t lds = ((size_t)(4 + kSplitRowsWaves * 5) * 64 * 4 + (size_t)copies * 16 * RBW * kSplitRowsWaves * 64) * sizeof(float);
    const dim3 grid((unsigned)((a.in_features + 63) / 64), (unsigned)p.parts);
    hot_linear_backward_split_rows_kernel<RBW, SMAX><<<grid, dim3(64 * kSplitRowsWaves), lds, s>>>(a);
}

template <int RB>
void xgrad_go(dim3 grid, int waves, hipStream_t s, const LinearGradArgs &a)
{
    const size_t lds = waves > 1 ? (size_t)(waves - 1) * (size_t)(RB * 16) * 64 * sizeof(float) : 0;
    hot_linear_xgrad_kernel<RB><<<grid, dim3(64 * waves), lds, s>>>(a);
}

// Input gradients for many rows on too few workgroups of 256 rows (few 64-input groups, around a thousand
// rows): with a workspace the contraction over the outputs is cut into parts (1024 x 540 x 2160: 72
// workgroups, 0.15 ms with 64-row workgroups instead).  Returns the number of parts, 1 for none.
// ws_bytes as in wgrad_shape.
inline long xgrad_outs_per_part(const hot_linear_desc *d, int parts)
{
    return ((d->out_features + parts - 1) / parts + kXgradRowsKernelOutputs - 1) / kXgradRowsKernelOutputs * kXgradRowsKernelOutputs;
}

int xgrad_parts(const hot_linear_desc *d, int64_t ws_bytes)
{
    if (ws_bytes == 0 || d->rows < kSlab4MinRows) return 1;
    const long k_groups = (d->in_features + 63) / 64, gy = (d->rows + 255) / 256;
    const long wgs = k_groups * gy * d->s_local;
    if (wgs >= 256 || gy > 65535) return 1;
    const int64_t block_bytes = (int64_t)d->s_local * d->rows * d->in_features * (int64_t)sizeof(float);
    int parts = 1;
    // up to two workgroups per compute unit; a part keeps at least 64 outputs (four steps)
    while (parts < kXgradMaxParts && wgs * parts < 512 && d->out_features >= 64L * (2 * parts) &&
           (ws_bytes < 0 || (int64_t)(2 * parts) * block_bytes <= ws_bytes))
        parts *= 2;
    // (the parts must all exist: the last one begins below O)
    while (parts > 1 && xgrad_outs_per_part(d, parts) * (parts - 1) >= d->out_features) parts /= 2;
    return parts;
}

// Launch shape of the weight-gradient kernel.
struct WgradShape {
    long tiles, rows_per_part;
    int ob, split, parts;
    bool deep;
    bool tile;      // the kernel with tiles of 128 x 128 instead (no parts; the other fields do not apply)
};

inline int64_t wgrad_part_bytes(const hot_linear_desc *d)
{
    return 2 * (d->out_features * d->in_features + ((d->out_features + 3) & ~(int64_t)3)) * (int64_t)sizeof(float);
}

// ws_bytes: what the caller's workspace holds (0: none; a negative value: as much as wanted, for the size query)
// wide_through_parts: count on eight row parts when deciding for two output groups per tile
WgradShape wgrad_shape_with(const hot_linear_desc *d, int64_t ws_bytes, bool wide_through_parts)
{
    WgradShape w;
    w.tile = false;
    const long k_groups = (d->in_features + 63) / 64;
    const long o_groups = (d->out_features + kColsPerWave - 1) / kColsPerWave;
    w.deep = d->rows >= kWgradDeepRows;
    // two output groups per tile where that still leaves a wave for every SIMD twice over after the row split
    // (four per tile were measured too: 90 against 95 TFLOP/s at 4096^2 x 1024, their registers spill)
    const long wide_waves = k_groups * ((o_groups + 1) / 2) * wgrad_max_split(2) * (wide_through_parts ? 8 : 1);
    w.ob = (d->rows >= kWgradWideRows && d->out_features >= 32 && wide_waves >= 2048) ? 2 : 1;
    w.tiles = k_groups * ((o_groups + w.ob - 1) / w.ob);
    // few tiles and many rows: let several waves share a tile (each then draws the tile's eps itself)
    // (up to a wave on every SIMD twice over; beyond that only while a wave keeps a thousand rows: finer pieces
    // even out the last round of waves, but every piece draws eps and adds through LDS again)
    w.split = 1;
    while (w.split < wgrad_max_split(w.ob) && d->rows >= 2L * w.split * kWgradRowsPerIter &&
           (w.tiles * w.split < 2048 || (w.tiles * w.split < 6144 && d->rows >= 1024L * w.split)))
        w.split *= 2;
    // Still too few waves for the chip (the tiles are few and a workgroup cannot hold more waves), or a number
    // of waves that fills the last round of the chip's 2048 wave slots (two per SIMD) badly: with a workspace
    // the rows are cut into parts for different workgroups, whose sums a second kernel adds in part order.
    // Measured: 1152 waves -> 4 or 8 parts (0.25 -> 0.19 ms), 2448 -> 2 parts (0.47 -> 0.42 ms; 4 parts lose),
    // 2048 -> none (2 parts: 0.19 -> 0.21 ms).  A wave keeps at least 128 rows.
    w.parts = 1;
    w.rows_per_part = 0;
    const long waves = w.tiles * w.split, last_round = waves % 2048;
    const bool fills_its_rounds = waves >= 2048 && (last_round == 0 || last_round > 1536);
    if (w.deep && ws_bytes != 0 && w.split == wgrad_max_split(w.ob) && !fills_its_rounds) {
        int parts = 1;
        while (parts < kWgradMaxParts && waves * parts < 4096 && d->rows >= 256L * w.split * (2 * parts) &&
               (ws_bytes < 0 || (int64_t)(2 * parts) * wgrad_part_bytes(d) <= ws_bytes))
            parts *= 2;
        if (parts > 1) {
            w.parts = parts;
            w.rows_per_part = ((d->rows + parts - 1) / parts + kWgradRowsPerIter - 1) / kWgradRowsPerIter * kWgradRowsPerIter;
        }
    }
    return w;
}

WgradShape wgrad_shape(const hot_linear_desc *d, int64_t ws_bytes)
{
    // Large layers at hundreds of rows and more: the kernel with tiles of 128 x 128.  Two workgroups share a compute
    // unit, so 512 tiles make a round, and a last round that is nearly empty costs as much as a full one; since the
    // kernel multiplies bf16 pieces it wins all the same (measured against the kernel above at 160 to 7260 rows: 1156
    // tiles 1.2-1.6x, 520 to 576 tiles 1.05-1.5x), and from 140 tiles and 256 rows on too (144 to 306 tiles 1.0-1.4x;
    // 128 tiles 0.8-0.95x, 85 tiles 0.5-0.8x: those stay with the kernel above, whose smaller tiles and row split fill
    // the chip better, as do few-tile layers whose rows a workspace spreads over the chip).
    const long tile_count = wgrad_tile_count(d);
    const bool fills = tile_count >= 512 || (tile_count >= 140 && d->rows >= 256 && !(ws_bytes != 0 && d->rows >= 8192));
    if (wgrad_tile_fits(d) && d->rows >= kSlab4MinRows && fills) {
        WgradShape w = wgrad_shape_with(d, 0, false);
        w.parts = 1;
        w.rows_per_part = 0;
        w.tile = true;
        return w;
    }
    if (ws_bytes != 0 && d->rows >= 8192) {     // with parts, smaller layers afford the wide tiles too (16640 x 192 x 768: 51 -> 57 TFLOP/s)
        const WgradShape w = wgrad_shape_with(d, ws_bytes, true);
        if (w.parts > 1) return w;              // (else the workspace was too small for that)
    }
    return wgrad_shape_with(d, ws_bytes, false);
}

}  // namespace

extern "C" {

int hot_linear_launch_shape(const hot_linear_desc *d, int which)
{
    if (!d || d->rows < 1 || d->in_features < 4 || (d->in_features & 3) || d->out_features < 1 || d->s_local < 1) return HOT_EINVAL;
    if (d->ldx < d->in_features || (d->ldx & 3) || d->x_sample_stride < 0 || which < 0 || which > 2) return HOT_EINVAL;
    if (d->out_features > (INT64_MAX / 8) / d->in_features || d->rows > (INT64_MAX / 8) / d->ldx) return HOT_EINVAL;
    if (which == 2) {
        const OnePassPlan p = one_pass_plan(d, true, -1);
        return p.rb ? (p.split ? 100 : 0) + 10 * p.rb + p.smax : 0;
    }
    auto code = [](const SlabShape &h, int st) { return h.waves ? 100 * (h.rbw == 1 ? 2 : h.waves) + 10 * h.cbw + st : 0; };
    if (which == 1) return code(slab_input_grad_shape(d, true), 1);
    const SlabForwardPlan p = slab_forward_plan(d);
    return p.two.waves ? code(p.two, 2) + 1000 * (p.one.waves ? p.one.cbw : 0) : code(p.one, 1);
}

int64_t hot_linear_backward_workspace_bytes(const hot_linear_desc *d)
{
    if (!d || d->rows < 1 || d->in_features < 4 || (d->in_features & 3) || d->out_features < 1 || d->s_local < 1) return HOT_EINVAL;
    if (d->out_features > (INT64_MAX / 64) / d->in_features) return HOT_EINVAL;
    if (d->rows > (INT64_MAX / 64) / d->in_features || d->rows * d->in_features > (INT64_MAX / 64) / d->s_local) return HOT_EINVAL;
    const WgradShape w = wgrad_shape(d, -1);
    const int64_t for_weights = w.parts > 1 ? (int64_t)w.parts * wgrad_part_bytes(d) : 0;
    const int x_parts = xgrad_parts(d, -1);
    const int64_t for_inputs = x_parts > 1 ? (int64_t)x_parts * d->s_local * d->rows * d->in_features * (int64_t)sizeof(float) : 0;
    int64_t most = for_weights > for_inputs ? for_weights : for_inputs;     // the two kernels use it one after the other
    // (whether input gradients will be asked for the query does not know: enough for either way)
    if (const OnePassPlan plan = one_pass_plan(d, true, -1); plan.rb && plan.parts > 1) {
        const int64_t for_one_pass = plan.parts * (int64_t)d->s_local * d->rows * d->in_features * (int64_t)sizeof(float);
        if (for_one_pass > most) most = for_one_pass;
    }
    return most;
}

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

    hipStream_t s = static_cast<hipStream_t>(stream);
    // Many rows (from 256) and at least 128 workgroups of 256 rows: the kernel whose waves share every draw
    // through LDS (measured against the kernel above: 1.05-1.4x from there on, slower below).  Two samples per
    // pass and one column tile when several samples share x; a single sample, and samples with inputs of
    // their own (one per pass), afford two column tiles.
    // Hundreds to thousands of rows on a layer that fills the chip with tiles of 512 rows: the kernel that stages x and the
    // drawn weights through LDS.  Samples that share x go two to a pass (they share every loaded row), an odd last one,
    // a single one and samples with inputs of their own one to a pass with tiles twice as wide.
    if (const SlabForwardPlan plan = slab_forward_plan(d); plan.two.waves || plan.one.waves) {
        SlabArgs b;
        b.rows = d->rows;
        b.contract = d->in_features;
        b.outs = d->out_features;
        b.ld_in = d->ldx;
        b.in_sample_stride = d->x_sample_stride;
        b.s_begin = b.s_end = 0;
        b.weight_quad0 = a.weight_quad0;
        b.bias_quad0 = a.bias_quad0;
        b.in = x;
        b.mu_w = mu_w;
        b.sigma_w = sigma_w;
        b.mu_b = mu_b;
        b.sigma_b = sigma_b;
        b.out = y;
        b.rng = r;
        if (plan.two.waves == 4 && plan.two.rbw == 1) slab_go<4, 1, 2, false, false, 1>(s, b, 0, plan.pair_samples);
        else if (plan.two.waves == 4) slab_go<4, 1, 2, false, false>(s, b, 0, plan.pair_samples);
        else if (plan.two.waves) {
            if (plan.two.cbw == 2) slab_go<8, 2, 2, false, false>(s, b, 0, plan.pair_samples);
            else slab_go<8, 1, 2, false, false>(s, b, 0, plan.pair_samples);
        }
        if (plan.one.waves) {
            if (d->x_sample_stride != 0) slab_go_singles<true, false>(plan.one, s, b, plan.pair_samples, d->s_local);
            else slab_go_singles<false, false>(plan.one, s, b, plan.pair_samples, d->s_local);
        }
        return hot_detail::note_hip(hipGetLastError());
    }
    {
        const bool xs = d->x_sample_stride != 0;
        const int no = (d->s_local == 1 || xs) ? 2 : 1;      // one sample per pass: its x loads serve two column tiles
        const long gx = (d->out_features + kColsPerWave * no - 1) / (kColsPerWave * no);
        const long gy = (d->rows + kRowsKernelRows - 1) / kRowsKernelRows;
        if (d->rows >= 256 && gx * gy >= 128 && gx <= 0x7fffffffL && gy <= 65535) {
            const dim3 grid((unsigned)gx, (unsigned)gy), block(64 * kRowsKernelWaves);
            if (xs) hot_linear_forward_rows_kernel<1, 2, true><<<grid, block, 0, s>>>(a);
            else if (no == 2) hot_linear_forward_rows_kernel<1, 2, false><<<grid, block, 0, s>>>(a);
            else hot_linear_forward_rows_kernel<2, 1, false><<<grid, block, 0, s>>>(a);
            return hot_detail::note_hip(hipGetLastError());
        }
    }
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
    if (rb == 4) linear_go<4>(st, grid, waves, s, a);
    else if (rb == 2) linear_go<2>(st, grid, waves, s, a);
    else linear_go<1>(st, grid, waves, s, a);
    return hot_detail::note_hip(hipGetLastError());
}

int hot_linear_backward_rng_ws(const hot_linear_desc *d, int32_t s_total, double dataset_size, uint32_t flags,
                               const hot_rng *rng, const float *x, const float *dy, const float *mu_w,
                               const float *sigma_w, const float *mu_b, const float *sigma_b, float *grad_mu_w,
                               float *grad_sigma_w, float *grad_mu_b, float *grad_sigma_b, float *dx, void *workspace,
                               int64_t workspace_bytes, void *stream)
{
    if (!d || !x || !dy || !mu_w || !sigma_w || !grad_mu_w || !grad_sigma_w) return HOT_EINVAL;
    if (workspace && (workspace_bytes < 0 || !aligned16(workspace))) return HOT_EINVAL;
    if ((mu_b == nullptr) != (sigma_b == nullptr) || (mu_b == nullptr) != (grad_mu_b == nullptr) ||
        (mu_b == nullptr) != (grad_sigma_b == nullptr))
        return HOT_EINVAL;
    if (d->rows < 1 || d->in_features < 4 || (d->in_features & 3) || d->out_features < 1 || d->s_local < 1) return HOT_EINVAL;
    if (d->ldx < d->in_features || (d->ldx & 3) || d->weight_offset < 0 || (d->weight_offset & 3)) return HOT_EINVAL;
    if (d->reserved != 0 || d->x_sample_stride < 0 || (d->x_sample_stride & 3)) return HOT_EINVAL;
    if (d->x_sample_stride != 0 && (d->rows > INT64_MAX / d->ldx || d->x_sample_stride < d->rows * d->ldx ||
                                    d->x_sample_stride > INT64_MAX / 4 / d->s_local))
        return HOT_EINVAL;
    if (mu_b && (d->bias_offset < 0 || (d->bias_offset & 3))) return HOT_EINVAL;
    if (s_total < d->s_local || !(dataset_size > 0.0) || !(dataset_size < 1.0 / 0.0)) return HOT_EINVAL;
    if (flags != HOT_REDUCE_SUM && flags != HOT_REDUCE_MEAN && flags != HOT_REDUCE_NONE) return HOT_EINVAL;
    if (!aligned16(x) || !aligned16(mu_w) || !aligned16(sigma_w) || !aligned16(grad_mu_w) || !aligned16(grad_sigma_w) ||
        !aligned4(dy) || (dx && !aligned16(dx)))
        return HOT_EINVAL;
    if (mu_b && (!aligned4(mu_b) || !aligned4(sigma_b) || !aligned4(grad_mu_b) || !aligned4(grad_sigma_b))) return HOT_EINVAL;
    if (d->out_features > (INT64_MAX / 8) / d->in_features) return HOT_EINVAL;
    // element offsets into dy and dx must fit: S_loc * R * max(O, K)
    const int64_t widest = d->out_features > d->in_features ? d->out_features : d->in_features;
    if (d->rows > (INT64_MAX / 8) / widest || d->rows * widest > (INT64_MAX / 8) / d->s_local) return HOT_EINVAL;
    // the grid of the input-gradient kernel is (64-input groups, row blocks, samples): checked here so that
    // a refused call has launched nothing
    if (dx && (d->s_local > 65535 || (d->rows + kRowsPerTile - 1) / kRowsPerTile > 65535)) return HOT_EINVAL;
    Rng r;
    if (!make_rng(rng, d->s_local, r)) return HOT_EINVAL;

    LinearGradArgs a;
    a.rows = d->rows;
    a.in_features = d->in_features;
    a.out_features = d->out_features;
    a.ldx = d->ldx;
    a.x_sample_stride = d->x_sample_stride;
    a.s_loc = d->s_local;
    a.weight_quad0 = d->weight_offset >> 2;
    a.bias_quad0 = mu_b ? d->bias_offset >> 2 : 0;
    if (flags == HOT_REDUCE_NONE) {
        a.g = 1.0;
        a.k = 1.0 / dataset_size;
    } else if (flags == HOT_REDUCE_MEAN) {
        a.g = 1.0 / (double)d->s_local;
        a.k = 1.0 / dataset_size;
    } else {
        a.g = 1.0 / (double)s_total;
        a.k = (double)d->s_local / ((double)s_total * dataset_size);
    }
    a.x = x;
    a.dy = dy;
    a.mu_w = mu_w;
    a.sigma_w = sigma_w;
    a.mu_b = mu_b;
    a.sigma_b = sigma_b;
    a.gmu_w = grad_mu_w;
    a.gsig_w = grad_sigma_w;
    a.gmu_b = grad_mu_b;
    a.gsig_b = grad_sigma_b;
    a.dx = dx;
    a.ws = nullptr;
    a.rows_per_part = 0;
    a.x_parts = 1;
    a.outs_per_part = 0;
    a.rng = r;
    hipStream_t s = static_cast<hipStream_t>(stream);

    const long k_groups = (d->in_features + 63) / 64;
    const long o_groups = (d->out_features + kColsPerWave - 1) / kColsPerWave;
    if (k_groups * o_groups > 0x7fffff00L) return HOT_EINVAL;      // the grid may exceed the number of tiles by a few workgroups
    // Few rows and input gradients wanted: both gradients in one pass over the weights, every eps drawn once.
    if (const OnePassPlan plan = one_pass_plan(d, dx != nullptr, workspace ? workspace_bytes : 0); plan.rb) {
        a.ws = static_cast<float *>(workspace);
        a.x_parts = (int)plan.parts;
        a.outs_per_part = plan.outs_per_part;
        if (plan.split) {
            if (plan.rb == 2) split_rows_go<2, 2>(plan, s, a);
            else split_rows_go<1, 2>(plan, s, a);
        } else if (plan.rb == 2 && plan.smax == 2) one_pass_go<2, 2>(plan, s, a);
        else if (plan.rb == 2) one_pass_go<2, 4>(plan, s, a);
        else if (plan.smax == 2) one_pass_go<1, 2>(plan, s, a);
        else if (plan.smax == 4) one_pass_go<1, 4>(plan, s, a);
        else one_pass_go<1, 8>(plan, s, a);
        if (plan.parts > 1) {
            const long quads = (long)d->s_local * d->rows * d->in_features / 4;
            hot_linear_dx_sum_kernel<<<dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, s>>>(dx, a.ws, quads, (int)plan.parts);
        }
        return hot_detail::note_hip(hipGetLastError());
    }
    const WgradShape shape = wgrad_shape(d, workspace ? workspace_bytes : 0);
    if (shape.tile) {
        wgrad_tile_go(s, a, wgrad_tile_count(d));
    } else {
        const long tiles = shape.tiles;
        const int split = shape.split, ob = shape.ob;
        const bool deep = shape.deep;
        if (shape.parts > 1) {
            a.ws = static_cast<float *>(workspace);
            a.rows_per_part = shape.rows_per_part;
            if (ob == 2) wgrad_go_parts<2>(tiles, split, shape.parts, s, a);
            else wgrad_go_parts<1>(tiles, split, shape.parts, s, a);
        } else if (split > 1) {
            if (ob == 2) wgrad_go<true, true, 2>(tiles, split, s, a);
            else if (deep) wgrad_go<true, true, 1>(tiles, split, s, a);
            else wgrad_go<true, false, 1>(tiles, split, s, a);
        } else {
            if (ob == 2) wgrad_go<false, true, 2>(tiles, kWgradWaves, s, a);
            else if (deep) wgrad_go<false, true, 1>(tiles, kWgradWaves, s, a);
            else wgrad_go<false, false, 1>(tiles, kWgradWaves, s, a);
        }
    }
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return hot_detail::note_hip(e);
    if (!dx) return HOT_OK;

    // Row tiles per workgroup: more of them share each drawn weight, fewer of them give more
    // workgroups and more waves per workgroup.  Take the most sharing that still puts a wave on
    // every SIMD of the chip (1024), else whatever yields the most waves.
    const long o_blocks = (d->out_features + kXgradOutputsPerStep - 1) / kXgradOutputsPerStep;
    auto waves_for = [&](int rb_, long gy_) {
        int w = 1;
        while (w < max_waves(rb_) && k_groups * gy_ * d->s_local * w < 8192 && 2L * w <= o_blocks &&
               (size_t)(2 * w - 1) * (size_t)(rb_ * 16) * 64 * sizeof(float) <= 65536)
            w *= 2;
        return w;
    };
    // Hundreds to thousands of rows on a layer whose dx fills the chip with tiles of 512 rows: the kernel of the forward pass
    // with dy as its input and the weight tile drawn transposed (rows of dy are read in 16-byte quads).
    // (a workspace that lets the kernel below cut the outputs into parts beats a four-wave launch that leaves a quarter of
    // its slots empty: 256 x 2160 x 8640, 136 workgroups of 256 rows x 32 inputs: the whole call 0.71 -> 0.53 ms)
    const int parts_at_hand = xgrad_parts(d, workspace ? workspace_bytes : 0);
    if (const SlabShape one = slab_input_grad_shape(d, aligned16(dy)); one.waves && !(parts_at_hand > 1 && one.waves == 4 && one.fill < 0.75)) {
        SlabArgs b;
        b.rows = d->rows;
        b.contract = d->out_features;
        b.outs = d->in_features;
        b.ld_in = d->out_features;
        b.in_sample_stride = d->rows * d->out_features;
        b.s_begin = b.s_end = 0;
        b.weight_quad0 = a.weight_quad0;
        b.bias_quad0 = 0;
        b.in = dy;
        b.mu_w = mu_w;
        b.sigma_w = sigma_w;
        b.mu_b = b.sigma_b = nullptr;
        b.out = dx;
        b.rng = r;
        slab_go_singles<true, true>(one, s, b, 0, d->s_local);
        return hot_detail::note_hip(hipGetLastError());
    }
    // many rows: the workgroup-shared draw, with as many rows per workgroup (256, 128, 64) as still give every
    // compute unit a workgroup
    if (const int x_parts = parts_at_hand; x_parts > 1) {
        // too few 256-row workgroups: the outputs are cut into parts, summed from the workspace afterwards
        a.ws = static_cast<float *>(workspace);
        a.x_parts = x_parts;
        a.outs_per_part = xgrad_outs_per_part(d, x_parts);
        const long gy_c = (d->rows + 255) / 256;
        hot_linear_xgrad_rows_kernel<4><<<dim3((unsigned)(k_groups * x_parts), (unsigned)gy_c, (unsigned)d->s_local), dim3(256), 0, s>>>(a);
        const long quads = (long)d->s_local * d->rows * d->in_features / 4;
        hot_linear_dx_sum_kernel<<<dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, s>>>(dx, a.ws, quads, x_parts);
        return hot_detail::note_hip(hipGetLastError());
    }
    if (d->rows >= 256) {
        // Rows per workgroup: 64 x cand.  All workgroups of these shapes are resident at once and those that share a
        // compute unit share its SIMDs, so the kernel takes (most workgroups on one compute unit) x (one workgroup's
        // work): per step 512 x cand matrix cycles per wave plus about 900 for the draw and the rest.  The count that
        // minimises the product wins: 7260 rows x 540 inputs x 2 samples are 522 workgroups of 256 rows (three on ten
        // compute units, two on the others: a third of the chip's time idle) but 684 of 192 rows (0.48 -> 0.40 ms).
        int best = 0;
        long best_cost = 0, best_gy = 0;
        for (int cand = 4; cand >= 1; --cand) {
            const long gy_c = (d->rows + 64 * cand - 1) / (64 * cand);
            const long wgs = k_groups * gy_c * d->s_local;
            if (gy_c > 65535 || wgs < 256) continue;     // (none fits: the kernel below, 15 % faster than 64-row workgroups there)
            const long cost = ((wgs + 255) / 256) * (512L * cand + 900);
            if (best == 0 || cost < best_cost) {
                best = cand;
                best_cost = cost;
                best_gy = gy_c;
            }
        }
        if (best) {
            const dim3 grid((unsigned)k_groups, (unsigned)best_gy, (unsigned)d->s_local);
            if (best == 4) hot_linear_xgrad_rows_kernel<4><<<grid, dim3(256), 0, s>>>(a);
            else if (best == 3) hot_linear_xgrad_rows_kernel<3><<<grid, dim3(256), 0, s>>>(a);
            else if (best == 2) hot_linear_xgrad_rows_kernel<2><<<grid, dim3(256), 0, s>>>(a);
            else hot_linear_xgrad_rows_kernel<1><<<grid, dim3(256), 0, s>>>(a);
            return hot_detail::note_hip(hipGetLastError());
        }
    }
    int rb = 1, waves = 1;
    long gy = 0, best = -1;
    for (int cand = d->rows > 32 ? 4 : (d->rows > 16 ? 2 : 1); cand >= 1; cand >>= 1) {
        const long gy_c = (d->rows + kRowsPerTile * cand - 1) / (kRowsPerTile * cand);
        const int w_c = waves_for(cand, gy_c);
        const long total = k_groups * gy_c * d->s_local * w_c;
        if (total > best) {
            best = total;
            rb = cand;
            waves = w_c;
            gy = gy_c;
        }
        if (total >= 1024) break;
    }
    const dim3 grid((unsigned)k_groups, (unsigned)gy, (unsigned)d->s_local);
    if (rb == 4) xgrad_go<4>(grid, waves, s, a);
    else if (rb == 2) xgrad_go<2>(grid, waves, s, a);
    else xgrad_go<1>(grid, waves, s, a);
    return hot_detail::note_hip(hipGetLastError());
}

int hot_linear_backward_rng(const hot_linear_desc *d, int32_t s_total, double dataset_size, uint32_t flags,
                            const hot_rng *rng, const float *x, const float *dy, const float *mu_w,
                            const float *sigma_w, const float *mu_b, const float *sigma_b, float *grad_mu_w,
                            float *grad_sigma_w, float *grad_mu_b, float *grad_sigma_b, float *dx, void *stream)
{
    return hot_linear_backward_rng_ws(d, s_total, dataset_size, flags, rng, x, dy, mu_w, sigma_w, mu_b, sigma_b, grad_mu_w,
                                      grad_sigma_w, grad_mu_b, grad_sigma_b, dx, nullptr, 0, stream);
}

}  // extern "C"
