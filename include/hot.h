/*
 * libhot -- the per-GPU mean-field Gaussian sample layer of sampling-parallel
 * Bayes-by-Backprop training, for AMD MI355X (gfx950).
 *
 * What it computes is the part of Algorithm 2 of arxiv 2604.04736 ("Sampling
 * Parallelism for Fast and Efficient Bayesian Learning") that one GPU runs on its
 * share of the Monte-Carlo samples and that does not depend on the network:
 * the reparameterisation line, the prior-matching (KL) line, and the chain rule
 * from per-sample weight gradients to the gradients of mu and sigma with the
 * scaling of the loss and averaging lines.  Algorithm 1 is the case of one GPU.
 *
 * Notation: N weights with mean mu[i] and standard deviation sigma[i] (sigma > 0 is
 * a precondition; IEEE propagation otherwise); S samples per step over all GPUs;
 * S_loc of them on this GPU; |D| the dataset size.  2-D arrays are row-major
 * [S_loc, ld] with row pitch ld >= N floats; columns N..ld-1 are never read or
 * written.  All data pointers are DEVICE pointers owned by the caller, must stay
 * valid until the stream has executed the call, and outputs must not alias
 * anything else.  Pointers need only 4-byte alignment; when every pointer is
 * 16-byte aligned and ld is a multiple of 4 the aligned fast path is taken.
 *
 * Every run call is asynchronous on the given stream (a hipStream_t passed as
 * void*; NULL is the default stream) and does no host synchronisation.  A plan may
 * be used by one stream at a time.  The same inputs with the same plan and launch
 * configuration give bitwise identical outputs (no floating-point atomics).
 *
 * All functions return HOT_OK or a negative error code; nothing aborts, throws or
 * prints.
 */
#ifndef HOT_H
#define HOT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HOT_VERSION 302 /* major*10000 + minor*100 + patch */

enum {
    HOT_OK = 0,
    HOT_EINVAL = -1, /* bad argument (null pointer, size out of range, misaligned to 4 bytes) */
    HOT_ENOMEM = -2, /* host or device allocation failed */
    HOT_EHIP = -3,   /* a HIP call failed; hot_last_hip_error() gives its code */
    HOT_ERANGE = -4  /* the problem is larger than the fixed capacity of an entry point that allocates nothing */
};

/* hot_desc.flags */
#define HOT_REDUCE_SUM 0u  /* g = 1/S,     k = S_loc/(S*|D|): add the outputs of all GPUs      */
#define HOT_REDUCE_MEAN 1u /* g = 1/S_loc, k = 1/|D|:         average the outputs of all GPUs  */
#define HOT_REDUCE_NONE 2u /* g = 1,       k = 1/|D|: grad_w already carries the caller's scaling (it is
                              dJ/dw of an objective J; the outputs are then dJ/dmu, dJ/dsigma of J + KL/|D|) */

typedef struct hot_plan hot_plan;

/* Problem statement of Algorithm 2 ("Require" line and loop bounds). */
typedef struct hot_desc {
    int64_t n_weights;   /* N >= 1 */
    int64_t ld;          /* row pitch of eps, w, grad_w in floats, >= N */
    int32_t s_local;     /* S_loc >= 1: samples on this GPU */
    int32_t s_total;     /* S >= S_loc: samples over all GPUs */
    double dataset_size; /* |D| > 0 */
    int32_t device;      /* HIP device ordinal that owns the buffers and the stream */
    uint32_t flags;      /* HOT_REDUCE_SUM, HOT_REDUCE_MEAN or HOT_REDUCE_NONE */
} hot_desc;

/* Launch geometry of one kernel; a zero field means "library default". */
typedef struct hot_launch {
    int32_t grid_blocks; /* upper bound on workgroups (each strides over column tiles), <= 65536 */
    int32_t chunks;      /* 16-byte column chunks per thread and tile: 1, 2 or 4 (default: 4 where that leaves at least
                            512 column tiles that fill their rounds of 256 workgroups to 90 %, else 2, else 1) */
    int32_t unroll;      /* sample rows whose loads are issued together: 1, 2 or 4 */
    int32_t nontemporal; /* 1: every array is accessed with non-temporal hints (the default: the arrays are touched once
                            per step and should not displace, or pay for displacing, what the network left in the
                            memory-side cache); 0: plain accesses (faster only when nothing else runs between the
                            calls and all arrays fit in that cache together) */
} hot_launch;

#define HOT_KERNEL_FORWARD 0
#define HOT_KERNEL_BACKWARD 1
#define HOT_KERNEL_FORWARD_RNG 2
#define HOT_KERNEL_BACKWARD_RNG 3

/*
 * Which draw of eps ~ N(0, I) the *_rng / hot_sample_* calls use (Algorithm 2, sampling
 * line: every GPU draws samples that no other GPU draws).  The paper names no generator;
 * this library fixes Philox-4x32 with 10 rounds (Salmon et al., SC'11) and Box-Muller:
 *   key     = (seed mod 2^32, seed div 2^32)
 *   counter = (q mod 2^32, q div 2^32, first_sample + s, step),  q = i div 4
 *   the four output words x0..x3 belong to weights 4q..4q+3; for the pairs (x0,x1), (x2,x3):
 *   u = ((xa >> 8) + 1) / 2^24,  f = (xb >> 8) / 2^24,  r = sqrt(-2 ln u),
 *   eps = r cos(2 pi f) for the even weight of the pair, r sin(2 pi f) for the odd one.
 * eps[s, i] is therefore a pure function of (seed, step, first_sample + s, i): GPUs that
 * use one seed and disjoint sample ranges draw disjoint streams, and the backward call
 * regenerates exactly (bit for bit) what the forward call used.
 */
typedef struct hot_rng {
    uint64_t seed;
    uint32_t step;         /* training-step counter */
    uint32_t first_sample; /* global index of local sample 0; first_sample + S_loc <= 2^32 */
} hot_rng;

/*
 * Validates the description, fixes g and k, and allocates the plan's own device
 * scratch (per-workgroup KL partial sums in fp64, 512 KiB) on desc->device.  *out is
 * written only on success.
 */
int hot_create(hot_plan **out, const hot_desc *desc);

/*
 * Algorithm 2, reparameterisation and prior-matching lines:
 *   w[s,i]  = fma(sigma[i], eps[s,i], mu[i])           for s < S_loc, i < N   (fp32, one rounding)
 *   *kl_out = 1/2 sum_i (sigma_i^2 + mu_i^2 - 1 - 2 ln sigma_i)               (fp64 accumulation)
 * mu, sigma: [N]; eps: [S_loc, ld] in; w: [S_loc, ld] out; kl_out: one device
 * double, or NULL to skip the KL term.
 */
int hot_forward(hot_plan *plan, const float *mu, const float *sigma, const float *eps,
                float *w, double *kl_out, void *stream);

/*
 * The prior-matching term of Algorithm 2 on its own: kl_out = 1/2 sum_i (sigma_i^2 + mu_i^2 - 1 -
 * ln sigma_i^2), for callers that never materialise w (the fused linear layer) but report the loss.
 * Same kernel, launch geometry and summation order as hot_forward's KL part (the value is bitwise
 * the one hot_forward returns); reads 8 bytes per weight.  kl_out: DEVICE, one double, required.
 */
int hot_kl(hot_plan *plan, const float *mu, const float *sigma, double *kl_out, void *stream);

/*
 * hot_forward for callers that cannot allocate device memory or create a plan: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, launch geometry and results
 * as hot_forward on a plan made from `desc` (w bit for bit; kl_out is always summed by the one-workgroup finish
 * kernel, so for at most 64 workgroups it may differ from hot_forward's in the last bits), but the
 * per-workgroup KL partial sums live in a static device array of the library (512 KiB on every GPU the
 * library runs on, held until the process ends) instead of a plan's own memory, and the call itself
 * allocates nothing, on the host or on the device, and frees nothing.
 * Capacity: desc->n_weights <= HOT_STATIC_MAX_WEIGHTS (one partial per 4096-weight tile); beyond it the
 * call returns HOT_ERANGE and launches nothing.  desc as for hot_create (desc->device < 64); pointer, layout,
 * stream and error rules as for hot_forward; a failed HIP call is reported by hot_last_hip_error(NULL).
 * The first call on a device looks up the array's address there (hipGetSymbolAddress, with that device
 * current): make that call outside any stream capture.  Nothing in the array needs to be zero before a call
 * (every partial is written before it is read).  All calls on one GPU share the array: calls that overlap
 * there (different streams or host threads) race on it; calls on one stream are ordered and safe.
 */
#define HOT_STATIC_MAX_WEIGHTS 268435456 /* 2^28 */
int hot_forward_static(const hot_desc *desc, const float *mu, const float *sigma, const float *eps, float *w,
                       double *kl_out, void *stream);

/*
 * Algorithm 2, loss / gradient / averaging lines, local share of this GPU.  With
 * grad_w[s,i] = dL_data,s/dw[s,i] from back-propagation through the network:
 *   grad_mu[i]    = g * sum_s grad_w[s,i]            + k * mu[i]
 *   grad_sigma[i] = g * sum_s grad_w[s,i] * eps[s,i] + k * (sigma[i] - 1/sigma[i])
 * (chain rule through w = mu + sigma*eps and the derivative of the KL line; g and k
 * as selected by hot_desc.flags).  Sums over s are accumulated in fp64 and rounded to
 * fp32 once.  grad_w, eps: [S_loc, ld] in; grad_mu, grad_sigma: [N] out, overwritten.
 */
int hot_backward(hot_plan *plan, const float *mu, const float *sigma, const float *eps,
                 const float *grad_w, float *grad_mu, float *grad_sigma, void *stream);

/*
 * The same two steps with eps drawn inside the kernels instead of read from memory
 * (4 bytes per item less in each direction; no eps array exists).  Arguments as above,
 * without eps; `rng` selects the draw.  hot_backward_rng must be given the hot_rng of
 * the hot_forward_rng call whose w produced grad_w.
 */
int hot_forward_rng(hot_plan *plan, const hot_rng *rng, const float *mu, const float *sigma,
                    float *w, double *kl_out, void *stream);
int hot_backward_rng(hot_plan *plan, const hot_rng *rng, const float *mu, const float *sigma,
                     const float *grad_w, float *grad_mu, float *grad_sigma, void *stream);

/*
 * The backward step over a SUBSET of the local samples, for callers that obtain the per-sample
 * weight gradients one (or a few) at a time and do not want to hold grad_w for all S_loc
 * samples: processes local samples first_row .. first_row + rows - 1.  grad_w (and eps, if
 * given) point at [rows, ld] arrays holding just those samples.  Exactly one of rng / eps is
 * non-NULL: with rng the eps of those samples is regenerated (sample index first_sample +
 * first_row + r), with eps it is read.  accumulate != 0 adds into grad_mu / grad_sigma instead
 * of overwriting them; add_kl != 0 adds the KL part k * mu, k * (sigma - 1/sigma) (k covers all
 * S_loc samples, so set it on exactly one of the calls of a step).  The calls of one step
 * together equal one hot_backward / hot_backward_rng up to fp32 rounding of the running sums.
 */
int hot_backward_rows(hot_plan *plan, const hot_rng *rng, const float *mu, const float *sigma, const float *eps,
                      const float *grad_w, int32_t first_row, int32_t rows, int32_t accumulate, int32_t add_kl,
                      float *grad_mu, float *grad_sigma, void *stream);

/*
 * The draw on its own: eps[S_loc, ld] as fp32 (exactly the values the *_rng calls use), or
 * the raw generator words bits[S_loc, ld] (word i mod 4 of quad i div 4), for callers and
 * tests that want the array.
 */
int hot_sample_eps(hot_plan *plan, const hot_rng *rng, float *eps, void *stream);
int hot_sample_bits(hot_plan *plan, const hot_rng *rng, uint32_t *bits, void *stream);

/* Frees the plan's scratch.  NULL is a no-op.  The stream must have finished with the plan. */
int hot_destroy(hot_plan *plan);

/* Overrides / reads back the launch geometry of one kernel of this plan. */
int hot_set_launch(hot_plan *plan, int kernel, const hot_launch *cfg);
int hot_get_launch(const hot_plan *plan, int kernel, hot_launch *cfg);

/*
 * hipError_t of the last failed HIP call made through this plan (0 if none).  With plan = NULL:
 * of the last failed HIP call this thread made through an entry point that takes no plan
 * (hot_create, hot_stats_*, hot_linear_*, hot_adam_step, hot_*_dropout_rng, hot_probe_*).
 */
int hot_last_hip_error(const hot_plan *plan);

/*
 * One sampled Bayesian linear layer, the weight draw fused into the contraction (Algorithm
 * 1 / 2: reparameterisation line + ForwardPass for a Linear layer):
 *   y[s, r, o] = sum_k x_s[r, k] * fma(sigma_W[o, k], eps_s[o, k], mu_W[o, k])
 *                + fma(sigma_b[o], eps_s^b[o], mu_b[o])
 * x_s is the minibatch itself, shared by all samples (x_sample_stride = 0: the first layer), or
 * the previous layer's output under the same weight sample (x_sample_stride = floats from x_s
 * to x_{s+1}: every later layer).
 * eps of weight (o, k) is the draw (see hot_rng) of flat parameter index weight_offset + o*K + k,
 * eps of bias o that of bias_offset + o: the layer sees exactly the w that hot_forward_rng
 * would write for a parameter vector holding this layer at those offsets, without w ever
 * existing in memory.  x: [rows, ldx] or [s_local, rows, ldx]; mu_W, sigma_W: [out_features, in_features] packed
 * row-major; mu_b, sigma_b: [out_features] or both NULL; y: [s_local, rows, out_features]
 * packed, out.  All DEVICE pointers; x, mu_W, sigma_W 16-byte aligned; in_features, ldx,
 * weight_offset, bias_offset multiples of 4.  The contraction runs on the matrix cores at fp32
 * accuracy: on the fp32 instructions (v_mfma_f32_16x16x4_f32, v_mfma_f32_32x32x2_f32), or, in the tiles of 256 rows
 * and more, on v_mfma_f32_32x32x16_bf16 with every product formed from three bf16 pieces of both factors (six
 * partial products; what they leave out is below 3 * 2^-24 of a product; measured errors up to 7e-7 of the sum of
 * addend magnitudes, against 3e-7 on the fp32 instruction; a factor below about 1e-33 in magnitude has pieces
 * below bf16's normal range, which the instruction may flush, and an infinite factor gives NaN, not infinity).
 * Runs on the current device, asynchronous on `stream`.
 * Up to a few hundred rows a wave draws the weights it multiplies (re-drawing eps per block of 64
 * rows is then cheaper than writing and re-reading w); from 256 rows on, given at least 128 workgroups
 * of 256 rows x 16 outputs, the four waves of a workgroup share every draw through LDS; where tiles of 256, 512
 * or 1024 rows x 32 to 128 outputs fill the chip (hot_linear_launch_shape tells; the 256-row tiles from 129 rows
 * on, tiles of 128 rows from 65 to 128), four, eight or sixteen waves share it and x goes from memory straight into LDS (150-190 TFLOP/s
 * of fp32 work on layers that fill the chip).  The draw and the matrix instructions do not overlap on this chip; against writing w once
 * with hot_forward_rng and calling a library GEMM the call is 1.8-2.9x faster up to tens of rows, level at
 * 64 rows, 1.8-2.0x at the 7260 and 16640 rows of a Swin and a ViT layer, and 1.4x on the largest squares;
 * between about 80 and 500 rows large layers stay behind that route (0.75-1.0x at 8192 x 8192, 0.7-0.95x at
 * 2160 x 8640): one draw serves too few rows there and the two do not overlap.
 */
typedef struct hot_linear_desc {
    int64_t rows;          /* R >= 1: rows of x (batch x tokens) */
    int64_t in_features;   /* K >= 4, multiple of 4 */
    int64_t out_features;  /* O >= 1 */
    int64_t ldx;           /* pitch of x in floats, >= K, multiple of 4 */
    int64_t weight_offset; /* flat parameter index of W[0, 0], multiple of 4 */
    int64_t bias_offset;   /* flat parameter index of b[0], multiple of 4 (ignored without bias) */
    int32_t s_local;       /* S_loc >= 1 */
    int32_t reserved;      /* must be 0 */
    int64_t x_sample_stride; /* 0: one x for all samples; else >= rows * ldx, multiple of 4 */
} hot_linear_desc;

int hot_linear_forward_rng(const hot_linear_desc *desc, const hot_rng *rng, const float *x, const float *mu_w,
                           const float *sigma_w, const float *mu_b, const float *sigma_b, float *y, void *stream);

/*
 * Back-propagation through the same layer (Algorithm 1 / 2: the gradient and averaging lines for a
 * Linear layer), again without the sampled weights, and without the per-sample weight gradients,
 * ever existing in memory.  dy[s_local, rows, out_features] (packed, DEVICE) holds dL_s/dy_s.  With
 * G_s[o,k] = sum_r dy_s[r,o] x_s[r,k] and Gb_s[o] = sum_r dy_s[r,o]:
 *   grad_mu_w[o,k]    = g sum_s G_s[o,k]              + k_kl mu_w[o,k]
 *   grad_sigma_w[o,k] = g sum_s G_s[o,k] eps_s[o,k]   + k_kl (sigma_w[o,k] - 1/sigma_w[o,k])
 *   grad_mu_b, grad_sigma_b likewise from Gb_s and the bias draws
 *   dx[s,r,k]         = sum_o dy_s[r,o] fma(sigma_w[o,k], eps_s[o,k], mu_w[o,k])
 * i.e. what hot_backward_rng returns for grad_w = G on the flat parameter vector that holds the
 * layer at desc's offsets (g and k_kl from s_total, dataset_size and flags exactly as hot_create
 * derives them from hot_desc; eps regenerated from rng as in the forward call).  Both contractions
 * run on the matrix cores in fp32.  grad_mu_w, grad_sigma_w: [out_features, in_features] packed,
 * 16-byte aligned, overwritten; grad_mu_b, grad_sigma_b: [out_features], both NULL exactly when
 * mu_b is; dx: [s_local, rows, in_features] packed, 16-byte aligned, one block per sample also
 * when x is shared (the caller adds them up), or NULL to skip it (a first layer); with dx, rows <=
 * 1 048 560 and s_local <= 65 535 (grid limits; HOT_EINVAL beyond, before anything runs).  Other arguments
 * and rules as for hot_linear_forward_rng.  Every weight is drawn once per sample (and per wave that
 * shares its tile) for the weight gradients, and for dx once per block of 64 rows, or, from 256 rows
 * on, once per workgroup of 64 to 256 rows (its waves share the draws through LDS), or, where tiles of 512
 * or 1024 rows fill the chip, once per such tile (the forward pass's kernel for many rows with dy as its
 * input; it needs out_features to be a multiple of 4 and dy 16-byte aligned).  Large layers
 * (from 129 rows on, at least 512 tiles of 128 inputs x 128 outputs, or from 256 rows on at least 140) take their
 * weight gradients from a kernel that stages x and dy through LDS and multiplies bf16 pieces of both, as the
 * forward call's large tiles do (up to 180 TFLOP/s of fp32 work); it needs out_features to
 * be a multiple of 4 and rows * max(ldx, out_features) * 4 below 4 GiB, else the first kernel runs; with more
 * than two samples it adds up pairs of samples in grad_mu_w and grad_sigma_w themselves.  All of these kernels
 * scale the sums and add the KL part in fp32 (g * sum + k * mu, g * sum + k * (sigma - 1/sigma) with the hardware's
 * reciprocal: 1e-7 of each term), where hot_backward does it in fp64.  Against
 * library GEMMs for dx and G followed by hot_backward_rng the call is 1.1-3x faster up to tens of rows (with a
 * workspace, see below; 0.8-3x without) and at 1.08-1.25x for thousands of rows; between about 100 and 450 rows it
 * mostly stays behind on large layers (0.65-1.0x).
 */
int hot_linear_backward_rng(const hot_linear_desc *desc, int32_t s_total, double dataset_size, uint32_t flags,
                            const hot_rng *rng, const float *x, const float *dy, const float *mu_w,
                            const float *sigma_w, const float *mu_b, const float *sigma_b, float *grad_mu_w,
                            float *grad_sigma_w, float *grad_mu_b, float *grad_sigma_b, float *dx, void *stream);

/*
 * Which launch shape the calls above choose for a layer (host arithmetic only; for tests and for tuning, same
 * passages of the paper).  which = 0: hot_linear_forward_rng; which = 1: the input-gradient part of
 * hot_linear_backward_rng (dy taken to be 16-byte aligned).  Returns 0 where the layer goes to the kernels for up
 * to a few hundred rows per workgroup; else, for the kernel with 256, 512 or 1024 rows per workgroup (64 per wave),
 * 100 * waves + 10 * (outputs per workgroup / 32) + samples per pass of its (first) launch, e.g. 822: eight waves
 * (512 rows), 64 outputs, two samples per pass; 1621: sixteen waves (1024 rows), 64 outputs, one sample per pass;
 * 412: four waves (256 rows), 32 outputs, two samples per pass; 2xx: four waves of 32 rows each (128 rows), e.g. 212;
 * plus 1000 * (outputs per workgroup / 32) of a second launch that takes an odd last sample on its own.
 * which = 2: hot_linear_backward_rng_ws with dx wanted and all the workspace it asks for: 10 * (16-row blocks) +
 * (samples a lane holds accumulators for) of the kernel that takes both gradients in one pass, e.g. 12, 24, 18,
 * plus 100 where the waves split the rows (blocks per wave: 112, 122); 0 where the two separate kernels run.
 * HOT_EINVAL for a malformed desc or another `which`.
 */
int hot_linear_launch_shape(const hot_linear_desc *desc, int which);

/*
 * The same call with device scratch of the caller's (same passage of the paper; only the launch shape
 * differs).  A layer with few weights and many rows (a ViT layer: 192 x 768 weights, 16 640 rows) has too
 * few 16-output x 64-input tiles to give every compute unit weight-gradient work, and the waves of one
 * workgroup are all that can add up the rows of a tile without memory.  With a workspace the rows are cut
 * into up to 16 parts for different workgroups; each part leaves its sums there and a second kernel adds
 * them in part order and finishes the gradients: deterministic, no atomics.  The input gradients use the
 * same memory afterwards where 256-row workgroups are too few for the chip (few inputs, around a thousand
 * rows): the outputs they contract over are cut into parts, whose dx blocks a second kernel adds.
 * Up to 128 rows with dx wanted the workspace buys more: weight and input gradients then come from ONE pass
 * over the weights, every eps drawn once instead of once per kernel, and the draw is most of the time at so
 * few rows.  Up to 32 rows (where a lane's registers hold the dx accumulators of all samples: 32 rows: 4 samples,
 * 16 rows: 8) every wave draws the tiles it multiplies (16 rows: 1.4x at 8192 x 8192, 2.1x at 2160 x 8640
 * against the call without a workspace); from 33 to 128 rows, for one or two samples on layers of half a million
 * weights and more, the four waves of a workgroup split the rows and share the draws through LDS (64 rows: 1.6x
 * at 2160 x 8640, 1.17x at 8192 x 8192).  A workgroup owns 64 inputs and keeps their dx in registers over all
 * outputs; layers with fewer than 256 such strips cut the outputs into parts, whose dx blocks go through the
 * workspace as above (s_local * rows * in_features * 4 bytes per part).
 * hot_linear_backward_workspace_bytes(desc) returns the number of bytes with which the call splits as far
 * as it wants to (0: this shape would not use a workspace; HOT_EINVAL for a malformed desc).  workspace:
 * DEVICE, 16-byte aligned, owned by the caller, contents undefined afterwards, or NULL (then the call is
 * hot_linear_backward_rng); with fewer bytes than asked for the call splits less, or not at all.  Calls
 * that share a workspace must not overlap.  Results agree with hot_linear_backward_rng to the rounding of
 * a different order of summation (over the rows; for dx over the outputs).
 */
int64_t hot_linear_backward_workspace_bytes(const hot_linear_desc *desc);
int hot_linear_backward_rng_ws(const hot_linear_desc *desc, int32_t s_total, double dataset_size, uint32_t flags,
                               const hot_rng *rng, const float *x, const float *dy, const float *mu_w,
                               const float *sigma_w, const float *mu_b, const float *sigma_b, float *grad_mu_w,
                               float *grad_sigma_w, float *grad_mu_b, float *grad_sigma_b, float *dx, void *workspace,
                               int64_t workspace_bytes, void *stream);

/*
 * The optimizer-update line that closes the inner loop of Algorithm 1 / 2 (the paper names Adam as
 * its example), run on the all-reduced gradients.  The paper gives no hyper-parameters:
 * they are inputs.  Adam as published (Kingma and Ba, ICLR 2015), for mu and for sigma with
 * their own moments, in place, fp32:
 *   g = grad_scale * grad;  m = beta1 m + (1-beta1) g;  v = beta2 v + (1-beta2) g^2
 *   theta -= lr * (m / (1-beta1^t)) / (sqrt(v / (1-beta2^t)) + eps);  then, if sigma_min > 0,
 *   sigma = max(sigma, sigma_min)   (the paper needs sigma > 0 but does not say how it is kept).
 * All arrays [n] fp32 DEVICE, 4-byte aligned (16-byte aligned for the fast path); the six
 * state arrays are read and overwritten.  One pass: 56 bytes per weight.  Current device.
 */
typedef struct hot_adam {
    double lr, beta1, beta2, eps;
    double grad_scale; /* e.g. 1/P after a sum all-reduce of mean-convention gradients; 1 otherwise */
    double sigma_min;  /* <= 0: no clamp */
    int64_t step;      /* t >= 1 */
} hot_adam;

int hot_adam_step(const hot_adam *params, int64_t n, float *mu, float *sigma, const float *grad_mu,
                  const float *grad_sigma, float *m_mu, float *v_mu, float *m_sigma, float *v_sigma,
                  void *stream);

/*
 * Algorithm 1 (one GPU holds all S samples, so nothing is all-reduced between the gradient line
 * and the update line): hot_backward followed by hot_adam_step in ONE pass.  The gradients
 * grad_mu, grad_sigma of hot_backward are formed in registers, rounded to fp32 exactly as
 * hot_backward would store them, and consumed by the Adam update of hot_adam_step; they are
 * never written.  The result is bit-identical to the two calls, at 16 bytes per weight less
 * traffic than they need together (8 written, 8 read back).
 * Requires a plan with s_local == s_total (else HOT_EINVAL: with several GPUs the all-reduce
 * has to come between the two steps).  Exactly one of rng / eps is non-NULL (eps regenerated
 * from rng, or read from eps[S, ld]).  mu, sigma [N] and the four moment arrays [N] are read
 * and overwritten; grad_w [S, ld] is read.  Layout, alignment, stream and error rules as for
 * hot_backward; the launch geometry is that of HOT_KERNEL_BACKWARD (HOT_KERNEL_BACKWARD_RNG
 * with rng).
 */
int hot_backward_adam(hot_plan *plan, const hot_rng *rng, const hot_adam *params, float *mu, float *sigma,
                      const float *eps, const float *grad_w, float *m_mu, float *v_mu, float *m_sigma,
                      float *v_sigma, void *stream);

/*
 * Algorithm 1's whole step behind the network's backward pass in ONE pass: hot_backward_rng, hot_adam_step
 * and the hot_forward_rng of the NEXT step.  The gradients are formed in registers and consumed by the Adam
 * update as in hot_backward_adam; the updated mu, sigma are stored and, still in registers, sampled from
 * with the next step's draw: w[s,i] = fma(sigma[i], eps_next[s,i], mu[i]), and *kl_out (DEVICE, one double,
 * or NULL) receives the KL term of the UPDATED parameters.  Results are bit-identical to
 * hot_backward_adam(rng) followed by hot_forward_rng(rng_next) (kl_out: equal up to the order in which the
 * fp64 per-workgroup partial sums are added, and identical when both kernels run with the same chunks and
 * grid bound on more than 64 workgroups), at 8 bytes per weight and one launch less.  Requires s_local == s_total.  rng: the draw that produced grad_w; rng_next: the draw of the
 * next step (normally the same seed with step + 1).  mu, sigma, the four moment arrays [N]: read and
 * overwritten; grad_w [S, ld]: read; w [S, ld]: written, must not be grad_w.  Layout, alignment, stream and
 * error rules as for hot_backward; launch geometry: HOT_KERNEL_BACKWARD_RNG.
 */
int hot_backward_adam_forward(hot_plan *plan, const hot_rng *rng, const hot_rng *rng_next, const hot_adam *params,
                              float *mu, float *sigma, const float *grad_w, float *m_mu, float *v_mu, float *m_sigma,
                              float *v_sigma, float *w, double *kl_out, void *stream);

/*
 * The update line of step t and the reparameterisation and prior-matching lines of step t + 1 in
 * ONE pass (Algorithm 2 once the all-reduced gradients are there; also Algorithm 1):
 * hot_adam_step followed by hot_forward / hot_forward_rng.  The updated mu, sigma are stored and,
 * still in registers, sampled from, so they are not read back: 8 bytes per weight and one launch
 * less than the two calls, bit-identical results (mu, sigma, moments, w, kl_out).  Exactly one of
 * rng / eps is non-NULL (rng: the draw of the NEW step).  grad_mu, grad_sigma [N]: read; the six
 * state arrays: read and overwritten; w [S_loc, ld], kl_out: as in hot_forward (kl_out is the KL of
 * the UPDATED parameters; may be NULL).  Launch geometry: HOT_KERNEL_FORWARD(_RNG).
 */
int hot_adam_forward(hot_plan *plan, const hot_rng *rng, const hot_adam *params, float *mu, float *sigma,
                     const float *grad_mu, const float *grad_sigma, float *m_mu, float *v_mu, float *m_sigma,
                     float *v_sigma, const float *eps, float *w, double *kl_out, void *stream);

/*
 * Monte Carlo dropout in weight space (section "Monte Carlo Dropout": in the variational reading of
 * dropout each weight carries a random 0/1 keep factor; each of the S stochastic passes uses its
 * own mask).  For sample s and weight i the mask bit is (generator word of (s, i) <
 * floor(keep * 2^32)), compared as 64-bit integers so that keep = 1 keeps every weight, the word being
 * the one hot_sample_bits returns for the same hot_rng:
 *   forward   w[s,i]     = mu[i] * bit / keep                  (1/keep keeps E[w] = mu)
 *   backward  grad_mu[i] = g * sum_s grad_w[s,i] * bit / keep   (g = 1/S; 1/S_loc with HOT_REDUCE_MEAN; 1 with HOT_REDUCE_NONE)
 * The mask is never stored; the backward call regenerates it.  desc gives N, ld, S_loc, S and
 * the reduce convention (dataset_size and device are not used); 0 < keep <= 1.  Layouts and
 * alignment rules as for hot_forward / hot_backward.  Current device.
 */
int hot_forward_dropout_rng(const hot_desc *desc, const hot_rng *rng, double keep, const float *mu, float *w,
                            void *stream);
int hot_backward_dropout_rng(const hot_desc *desc, const hot_rng *rng, double keep, const float *grad_w,
                             float *grad_mu, void *stream);

/*
 * The same layer with one Bernoulli variable per NEURON and sample instead of one per weight
 * (the same section also describes dropout unit-wise, zeroing whole neurons): mu is the [out, in_features]
 * row-major weight matrix of a layer (desc->n_weights = out * in_features), and dropping input
 * unit k of sample s zeroes column k, i.e. all weights i with i mod in_features == k.  The mask
 * bit of unit k is (generator word of flat index unit_offset + k < floor(keep * 2^32)), so
 * layers of one network use disjoint unit_offset ranges.  in_features >= 4 and unit_offset are
 * multiples of 4.  Everything else as above.
 */
int hot_forward_dropout_units_rng(const hot_desc *desc, const hot_rng *rng, double keep, int64_t in_features,
                                  int64_t unit_offset, const float *mu, float *w, void *stream);
int hot_backward_dropout_units_rng(const hot_desc *desc, const hot_rng *rng, double keep, int64_t in_features,
                                   int64_t unit_offset, const float *grad_w, float *grad_mu, void *stream);

/*
 * Predictive statistics over the samples (the paper's training description and its Monte
 * Carlo dropout section: the mean of the S predictions is the model's output, their standard
 * deviation its uncertainty; and the remark after Algorithm 2 that mean and standard
 * deviation CAN be aggregated exactly across GPUs by communicating two numbers per output).
 * Both calls run on the current device and are asynchronous on `stream`.
 *
 * hot_stats_local: yhat[S_loc, ld] (fp32, DEVICE, row s = the M outputs predicted with weight
 * sample s, M = batch x output dimension flattened, ld >= M) -> mean[M] and m2[M] (fp64,
 * DEVICE): the mean of this GPU's rows and the sum of their squared deviations from it.
 * These are the two numbers per output a GPU contributes (its count S_loc is known).
 */
int hot_stats_local(const float *yhat, int64_t m, int64_t ld, int32_t s_local, double *mean, double *m2,
                    void *stream);

/*
 * hot_stats_merge: the partials of `parts` (1..64) GPUs, means[parts, ld] and m2s[parts, ld]
 * (fp64, DEVICE, e.g. after an all-gather), with counts[parts] (HOST array, samples behind
 * each partial, each >= 1) -> mean_out[M], std_out[M] (fp32, DEVICE) over all samples:
 *   n = sum_p n_p;  mean = sum_p n_p mean_p / n;
 *   std = sqrt( sum_p [ m2_p + n_p (mean_p - mean)^2 ] / (n - ddof) ),  ddof = 0 or 1
 * (the paper does not say which standard deviation it means).  parts = 1 finishes a single
 * GPU's statistics.
 */
int hot_stats_merge(const double *means, const double *m2s, const int32_t *counts, int32_t parts, int64_t m,
                    int64_t ld, int32_t ddof, float *mean_out, float *std_out, void *stream);

/*
 * hot_stats_local and hot_stats_merge in one pass for a GPU that holds all S samples (nothing to
 * merge): yhat[S, ld] -> mean_out[M], std_out[M] (fp32, DEVICE), std = sqrt(M2 / (S - ddof)) with
 * the same shifted fp64 sums.  Arguments and rules as for the two calls.
 */
int hot_stats_whole(const float *yhat, int64_t m, int64_t ld, int32_t s, int32_t ddof, float *mean_out,
                    float *std_out, void *stream);

/*
 * Measurement aid, not a step of the paper's path: copies `bytes` (a multiple of 16;
 * both DEVICE pointers 16-byte aligned, ranges disjoint) on the current device with
 * the same 16-byte accesses the kernels use.  Its traffic is known exactly (bytes
 * read, bytes written), which calibrates HBM byte counters and gives the machine's
 * copy ceiling.  nontemporal: 0 or 1 (hints on both loads and stores).
 */
int hot_probe_copy(void *dst, const void *src, int64_t bytes, int nontemporal, void *stream);

/*
 * Measurement aid: `reads` (1..64) read streams and `writes` (0..64) write streams of
 * stream_bytes each (a multiple of 4; with a multiple of 16 every stream keeps the arena's
 * 16-byte alignment, otherwise the streams are as skewed against the 16- and 64-byte grids as
 * the rows of a sample matrix with that pitch, their last 1 to 3 floats are left alone and
 * writes must be >= 1), laid out back to back in `arena` (a DEVICE buffer
 * of (reads + writes) * stream_bytes bytes, 16-byte aligned; read streams first).  Every
 * write stream receives the element-wise sum of the read streams.  With the stream counts
 * of one of the kernels above it measures the machine's ceiling for that kernel's mix of
 * read and write traffic.  Up to 6 read and 2 write streams a thread loads all of them before it
 * stores; beyond that (then writes >= 1) it walks the read streams four at a time and the write
 * streams one at a time, as the kernels walk their sample rows.
 */
int hot_probe_streams(void *arena, int64_t stream_bytes, int reads, int writes, void *stream);

/* Static, never NULL. */
const char *hot_strerror(int code);

/*
 * Smallest pitch >= n_weights that keeps every row 256-byte aligned (multiple of 64 floats).  Any pitch is
 * legal.  What MI355X rewards is rows of w that start on 64-byte boundaries, 16-byte aligned or not:
 * hot_forward re-aligns its stores row by row and loses at most 5 % on other pitches; hot_forward_rng and
 * the dropout forward calls do not and lose 4 % (two samples) to 19 % (sixteen samples), up to 40 % for
 * hot_forward_rng with a launch override of four chunks; the backward calls only read rows and lose 1-5 %.
 */
int64_t hot_recommended_ld(int64_t n_weights);

int hot_version(void);

#ifdef __cplusplus
}
#endif

#endif /* HOT_H */
