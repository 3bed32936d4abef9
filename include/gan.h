/*
 * C ABI of the grouped per-label DC-CGAN training library for gfx950.
 *
 * The paper (Section 2) factorises the data distribution over the K labels
 * (Eq. 5) and trains K independent conditional GANs, pair k seeing only the
 * samples of label k.  This library holds all K (generator, discriminator)
 * pairs on one GPU and advances all of them by one iteration per call:
 * route the minibatch by label, run G and D forward, the discriminator cost
 * (Eq. 3) and its backward pass, Adam on theta_D, the generator cost (Eq. 4)
 * through the updated D, its backward pass, Adam on theta_G.
 *
 * Conventions
 *  - Every function returns a gan_status and never throws or aborts: a shape the kernels do not support is
 *    refused with GAN_E_SHAPE before anything is launched (gan_last_error has the reason).
 *  - "DEVICE" pointers are HIP device pointers owned by the caller (for
 *    example a torch tensor's data_ptr()); "HOST" pointers are ordinary host
 *    memory.  The context owns parameters, Adam moments, BatchNorm running
 *    statistics and all workspace; the caller owns every argument buffer.
 *  - gan_train_step and gan_generate enqueue work on the stream given to
 *    gan_create and return without waiting; the caller may reuse the input
 *    buffers for stream-ordered work as soon as the call returns.  The
 *    gan_get_* / gan_set_* functions synchronise that stream.
 *  - Argument errors detectable on the host (null pointer, n < 0,
 *    n > max_total_batch) fail immediately with no side effects.  A label id
 *    outside [0, n_labels) is only visible on the device: that sample is
 *    dropped from every model, a sticky flag is raised, and the next
 *    gan_get_losses returns GAN_E_LABEL (and clears the flag).
 *  - Image tensors are [n, C, H, W] fp32 with values in [-1, 1] (the generator
 *    ends in tanh); noise is [n, z_dim] fp32; row i of each array describes
 *    sample i, in any label order.
 *
 * Network family (one shape for all K pairs; widths per configuration):
 *   G: [z ; onehot_cond_g(y)] -> linear -> [g_ch[0], g_h0, g_h0] -> BN -> ReLU
 *      -> { convT k4 s2 p1 -> BN -> ReLU } x (n_g - 1) -> convT k4 s2 p1 (+bias) -> tanh
 *   D: [x ; cond_d one-hot label maps] -> conv k4 s2 p1 (+bias) -> LeakyReLU
 *      -> { conv k4 s2 p1 -> BN -> LeakyReLU } x (n_d - 1) -> flatten -> linear (+bias) -> logit
 * (layer types as in the paper's Tables 1-4: linear input stage, BatchNorm with momentum 0.1,
 *  LeakyReLU slope 0.2, tanh output; D returns a logit and the sigmoid lives in the cost.)
 *
 * Flat parameter order seen by gan_get_params / gan_set_params (fp32 master values):
 *   G: fc.w [g_ch[0]*g_h0*g_h0, z_dim+cond_g] (rows in (c,h,w) order), bn0.gamma, bn0.beta,
 *      then per transposed conv i: w [Cin, Cout, 4, 4], and (gamma, beta) [Cout] or, for the last, bias [img_c].
 *   D: c1.w [d_ch[0], img_c+cond_d, 4, 4], c1.b, then per conv j: w [Cout, Cin, 4, 4], gamma, beta,
 *      then fc.w [d_ch[last]*h*h] (in (c,h,w) order), fc.b.
 */
#ifndef GAN_H
#define GAN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gan_ctx gan_ctx;

typedef enum {
  GAN_OK = 0,
  GAN_E_ARG = -1,     /* null pointer, negative size, bad index                       */
  GAN_E_SHAPE = -2,   /* configuration the kernels do not support (see gan_create)    */
  GAN_E_OOM = -3,     /* device allocation failed                                     */
  GAN_E_HIP = -4,     /* a HIP call or kernel launch failed; see gan_last_error       */
  GAN_E_LABEL = -5,   /* an out-of-range label id was seen since the last query       */
  GAN_E_STATE = -6    /* call not valid in the current state (e.g. no step taken yet) */
} gan_status;

typedef enum { GAN_FP32 = 0, GAN_BF16_FP32MASTER = 1 } gan_precision;

#define GAN_MAX_LAYERS 8

typedef struct {
  uint32_t struct_size;     /* sizeof(gan_config), for versioning                                     */
  int32_t  precision;       /* gan_precision: storage/contraction type of activations and weights     */
  int32_t  n_models;        /* K of Eq. 5: number of independent (G, D) pairs                         */
  int32_t  n_labels;        /* label ids lie in [0, n_labels); model(label) = label, or 0 if K == 1   */
  int32_t  cond_g;          /* one-hot width concatenated to z (0: unconditional generator)           */
  int32_t  cond_d;          /* number of one-hot label maps appended to D's input (0: none)           */
  int32_t  z_dim;           /* d_Z                                                                    */
  int32_t  img_c, img_hw;   /* image channels (1..4) and side                                         */
  int32_t  g_h0;            /* side of G's first feature map; img_hw = g_h0 * 2^n_g                   */
  int32_t  n_g;             /* number of transposed convolutions in G                                 */
  int32_t  g_ch[GAN_MAX_LAYERS]; /* input channels of each transposed conv (multiples of 64)          */
  int32_t  n_d;             /* number of strided convolutions in D                                    */
  int32_t  d_ch[GAN_MAX_LAYERS]; /* output channels of each conv (multiples of 64)                    */
  int32_t  max_total_batch; /* largest n any call will pass; sizes the workspace                      */
  float    lr, beta1, beta2, adam_eps;        /* Adam (the paper: lr 2e-4)                            */
  float    bn_eps, bn_momentum, leaky_slope;  /* the paper's tables: momentum 0.1, slope 0.2          */
  float    d_loss_scale, g_loss_scale;        /* the factors 1/2 in Eq. 3 and Eq. 4                   */
  float    init_std;        /* built-in initialiser: weights ~ N(0, init_std^2), gamma 1, the rest 0  */
  uint64_t seed;            /* seed of the built-in initialiser and of the dropout masks              */
  int32_t  family;          /* gan_family: which networks (see below)                                 */
  float    bn_eps_first;    /* GAN_FAMILY_PAPER: epsilon of G's first BatchNorm (Table 1: 1e-5)       */
  float    dropout_p;       /* GAN_FAMILY_PAPER: dropout probability in D (Table 2: 0.25), in [0, 1)  */
} gan_config;

/* GAN_FAMILY_STRIDED (0): the k4 s2 p1 convolution / transposed-convolution networks described above.
   GAN_FAMILY_PAPER (1): the networks exactly as the paper's Tables 1 and 2 print them (Section 4), unconditional
   (cond_g = cond_d = 0; the label only selects the model):
     G: z -> linear (+bias) -> ReLU -> [g_ch[0], g_h0, g_h0] -> BN(bn_eps_first)
        -> { Upsample x2 -> Conv k3 s1 p1 (g_ch[i-1] -> g_ch[i]) -> BN(bn_eps) -> LeakyReLU } for i = 1 .. n_g-1
        -> Conv k3 s1 p1 (g_ch[n_g-1] -> img_c, +bias) -> tanh                       img_hw = g_h0 * 2^(n_g-1)
     D: { Conv k3 s2 p1 (+bias) -> LeakyReLU -> Dropout(dropout_p) [-> BN(bn_eps), not after the first] } x n_d
        -> flatten -> linear (+bias) -> logit
   g_ch must be multiples of 64; d_ch may be any width up to 1024 (held padded to multiples of 64, the padding stays
   exactly zero).  Dropout is active in all three discriminator passes of an iteration (real, fake, fake through the
   updated D: pass ids 0, 1, 2), kept values scaled by 1 / (1 - p); the mask is the one gan_op_dropout documents, with
   layer = 1 .. n_d, step = the number of iterations the model has run (counting this one) and seed = cfg.seed.
   Flat parameter order:
     G: fc.w [g_ch[0]*g_h0*g_h0, z_dim] (rows in (c,h,w) order), fc.b, bn0.gamma, bn0.beta, then per block i:
        conv.w [g_ch[i], g_ch[i-1], 3, 3], gamma, beta; then conv.w [img_c, g_ch[n_g-1], 3, 3], conv.b.
     D: per conv j: w [d_ch[j], Cin, 3, 3], b [d_ch[j]], and for j > 0 gamma, beta; then fc.w [d_ch[last]*h*h] in
        (c,h,w) order, fc.b.
   BatchNorm running statistics (gan_get_bn_running): the BN layers in network order, real channels only. */
typedef enum { GAN_FAMILY_STRIDED = 0, GAN_FAMILY_PAPER = 1 } gan_family;

/* Allocate a context on the current device.  hip_stream is a hipStream_t (0 = the null stream).
   Fails with GAN_E_SHAPE when a channel count is not a multiple of 64, img_c > 4, the sides do not
   match (img_hw = g_h0 * 2^n_g, img_hw divisible by 2^n_d), n_models is neither 1 nor n_labels, a layer has more
   than 1024 channels, or max_total_batch makes one segment of an activation tensor 2 GiB or larger (the
   kernels address a segment with 32-bit byte offsets). */
gan_status gan_create(const gan_config* cfg, void* hip_stream, gan_ctx** out);
gan_status gan_destroy(gan_ctx* ctx);

/* One training iteration for every model that receives at least one sample (Section 2: Eq. 3, Eq. 4, Adam).
   label_ids: DEVICE int32 [n]; noise: DEVICE fp32 [n, z_dim]; real_batch: DEVICE fp32 [n, img_c, img_hw, img_hw].
   A model with no sample in this call is left untouched (parameters, moments, step count, statistics).
   Reproducibility: every sum runs in an order fixed by the configuration (model count, layer shapes,
   max_total_batch) and by the model's own samples, so a model's result is bit-identical from run to run, does not
   depend on the other models' samples in the call, and does not depend on the order of the flat batch beyond the
   relative order of that model's own samples. */
gan_status gan_train_step(gan_ctx* ctx, const int32_t* label_ids, const float* noise,
                          const float* real_batch, int32_t n);

/* x = G_k(z) for each sample, k = model(label) (the sampling half of Eq. 5's mixture).
   out_images: DEVICE fp32 [n, img_c, img_hw, img_hw], rows in the caller's order.
   use_running_stats = 0: BatchNorm uses the statistics of the generated batch, per model (as during training);
   1: the running statistics. */
gan_status gan_generate(gan_ctx* ctx, const int32_t* label_ids, const float* noise, int32_t n,
                        float* out_images, int32_t use_running_stats);

/* Costs of the last step: d_loss[k] = J_D of Eq. 3, g_loss[k] = -J_G of Eq. 4 (the quantity G minimises),
   counts[k] = samples model k received (0 => both losses are reported as 0).  HOST arrays [n_models];
   any of them may be NULL. */
gan_status gan_get_losses(gan_ctx* ctx, float* d_loss, float* g_loss, int32_t* counts);

/* ---- parity / checkpoint surface ---------------------------------------------------------------- */
/* which: 0 = generator, 1 = discriminator.  All buffers HOST, fp32, in the flat order documented above. */
gan_status gan_param_count(const gan_ctx* ctx, int32_t which, int64_t* per_model);
gan_status gan_get_params(gan_ctx* ctx, int32_t which, int32_t model, float* dst, int64_t n);
gan_status gan_set_params(gan_ctx* ctx, int32_t which, int32_t model, const float* src, int64_t n);
/* Adam first / second moments (may be NULL) and step count of one model. */
gan_status gan_get_opt_state(gan_ctx* ctx, int32_t which, int32_t model, float* m, float* v, int64_t* t);
/* Restore what gan_get_opt_state returned (resuming from a checkpoint): moments in the parameter order (either may be
   NULL: left as it is) and the step count t >= 0 that the next update increments. */
gan_status gan_set_opt_state(gan_ctx* ctx, int32_t which, int32_t model, const float* m, const float* v, int64_t t);
/* Gradients used by the last update of this model (same order as the parameters). */
gan_status gan_get_grads(gan_ctx* ctx, int32_t which, int32_t model, float* dst, int64_t n);
/* BatchNorm running statistics, concatenated over the network's BN layers. */
gan_status gan_bn_count(const gan_ctx* ctx, int32_t which, int64_t* per_model);
gan_status gan_get_bn_running(gan_ctx* ctx, int32_t which, int32_t model, float* mean, float* var, int64_t n);
gan_status gan_set_bn_running(gan_ctx* ctx, int32_t which, int32_t model, const float* mean, const float* var, int64_t n);
/* Routing of the last training step (gan_generate and gan_sample route into buffers of their own and change neither
   this nor the counts gan_get_losses reports): perm[j] = caller index of the j-th sample in model-major order (stable within a
   model), offs[k]..offs[k+1] = model k's rows.  HOST int32 [n of that step] and [n_models + 1]. */
gan_status gan_get_routing(gan_ctx* ctx, int32_t* perm, int32_t* offs);
/* Text of the last error on this context (never NULL). */
const char* gan_last_error(const gan_ctx* ctx);

/* Second stream (enable = 1; off by default): the weight-gradient GEMMs and the Adam updates of the convolution weights
   of a training step run on a stream of the library's own (default priority) beside the backward chain on the
   caller's stream, ordered by events; everything is joined back into the caller's stream before gan_train_step
   returns, and the results are the same bit for bit.  Fills the chip where the chain's launches leave it idle
   (1.7 % shorter steps on the largest workload); launches that share the chip run longer individually, which shows
   in per-launch timings.  Synchronises the stream. */
gan_status gan_use_second_stream(gan_ctx* ctx, int32_t enable);

/* Replayable steps (enable = 1; off by default): a gan_train_step call whose three device pointers and n equal those
   of one of the last eight distinct calls is captured into a HIP graph once and replayed from then on (same kernels,
   same order, same results bit for bit; the eight most recently used argument sets are kept).  For callers whose host
   thread, not the device, limits the step rate: a replay is one host call instead of a hundred and more launches; on
   an idle host it is no faster than the launches.  enable = 0: plain launches again (also the case while per-launch
   timing is on).  The caller's buffers are read when the step runs, as always. */
gan_status gan_use_graphs(gan_ctx* ctx, int32_t enable);
/* Number of training steps of this context that ran as graph replays so far (HOST int64). */
gan_status gan_graph_replays(const gan_ctx* ctx, int64_t* n);

/* ---- profiling ------------------------------------------------------------------------------------ */
/* Time kernel launches of the next steps with HIP events on the stream each launch goes to: enable = 1 every launch, one
   family per kernel instantiation; 2 every launch, one family per layer shape; 3 only the MFMA kernels (GEMM and
   weight-gradient instantiations); 0 stop.  Costs two events per timed launch, each of which drains the stream;
   off by default. */
gan_status gan_profile_enable(gan_ctx* ctx, int32_t enable);
/* Accumulated since enabling: for each of up to `cap` kernel families, its name (pointer to a static string),
   launch count, total milliseconds, and the algorithmic flops and bytes those launches stood for.
   One more family, "(mfma busy)", holds the time during which at least one GEMM or weight-gradient launch ran (the
   library runs some of them side by side on two streams, so their durations add up to more than that) with their
   summed work.  HOST arrays; *n_out receives the number of families.  Synchronises the stream. */
gan_status gan_profile_read(gan_ctx* ctx, int32_t cap, const char** names, int64_t* launches, double* ms,
                            double* flops, double* bytes, int32_t* n_out);

/* ---- next to the training step ----------------------------------------------------------------------- */
/* n samples of the mixture of Eq. 5: label_i is drawn from the class prior p_y, then x_i = G_{label_i}(noise_i).
   prior: HOST double [n_labels], non-negative, not all zero (it is normalised by its sum).  u: DEVICE fp32 [n],
   the caller's uniforms in [0, 1): label_i is the first k whose cumulative probability (running sums of
   prior[k] / sum in double, in index order) exceeds u_i.  noise, out_images, use_running_stats: as gan_generate
   (the paper combines the trained generators, so the running statistics, 1, are the usual choice).
   out_labels: DEVICE int32 [n].  Returns GAN_E_ARG for a bad prior.  Copies the cumulative prior to the device
   synchronously, then enqueues on the context's stream. */
gan_status gan_sample(gan_ctx* ctx, const double* prior, const float* u, const float* noise, int32_t n,
                      float* out_images, int32_t* out_labels, int32_t use_running_stats);

/* One-way analysis of variance of the image intensities by class: the F-statistic per channel that Section 4 quotes
   for each dataset as the justification for partitioning by label.  Observation (i, c) = mean of channel c over the
   pixels of image i; groups = label ids in [0, n_labels) (others are ignored).
   label_ids: DEVICE int32 [n]; images: DEVICE fp32 [n, img_c, img_hw, img_hw]; n <= max_total_batch;
   F: HOST double [img_c].  All arithmetic in double, in a fixed order.  Synchronises the stream.
   Returns GAN_E_STATE (and F = 0) when fewer than two labels occur or there are not more images than labels. */
gan_status gan_anova_f(gan_ctx* ctx, const int32_t* label_ids, const float* images, int32_t n, double* F);

/* ---- for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses
   that forbid hipMalloc) ------------------------------------------------------------------------------------------
   gan_anova_f_static computes what gan_anova_f computes, without a context and without any device allocation: its
   intermediate results (per-image channel means, per-label sums, counts and squared deviations) live in a static
   device array of about 2.1 MiB that every device the library runs on holds until the process ends (its address is
   looked up once per device, at the first call with that device current).  The caller passes the shape that a context
   would carry.  label_ids: DEVICE int32 [n]; images: DEVICE fp32 [n, img_c, img_hw, img_hw]; F: HOST double [img_c];
   hip_stream: a hipStream_t (0 = the null stream), synchronised before returning.
   Limits: n <= GAN_ANOVA_STATIC_MAX_IMAGES, n_labels <= GAN_ANOVA_STATIC_MAX_LABELS, img_c <= 4; anything larger
   returns GAN_E_SHAPE.  Other errors as gan_anova_f (GAN_E_STATE and F = 0 when fewer than two labels occur or there
   are not more images than labels).  gan_static_last_error() gives the text of the last error of this entry point.
   All calls on one device share that device's array: calls that overlap on one device (different streams or threads)
   race; calls in sequence need no clearing, every element read is written first by the same call. */
#define GAN_ANOVA_STATIC_MAX_IMAGES 65536
#define GAN_ANOVA_STATIC_MAX_LABELS 1024
gan_status gan_anova_f_static(const int32_t* label_ids, const float* images, int32_t n, int32_t n_labels, int32_t img_c,
                              int32_t img_hw, void* hip_stream, double* F);
const char* gan_static_last_error(void);

/* ---- what the chip delivers to the simplest kernels (Section 5 of the paper reports GPU usage only; these give the
   achievable ceilings the step's kernels are reported against, next to the published peaks) -------------- */
/* TFLOP/s of a register-only MFMA loop in the arithmetic of `precision` (bf16 inputs, or fp32), every CU busy.
   Allocates and frees a small buffer; synchronises the stream.  *tflops is a HOST double. */
gan_status gan_probe_mfma(int32_t precision, void* hip_stream, double* tflops);
/* GB/s (bytes read + bytes written per second) of a plain device-to-device copy of `bytes` (a multiple of 16, at
   least 1 MiB); allocates and frees two buffers of that size; synchronises the stream.  *gbps is a HOST double. */
gan_status gan_probe_copy(int64_t bytes, void* hip_stream, double* gbps);

/* ---- single operations, for per-kernel parity tests ---------------------------------------------- */
/* All pointers DEVICE.  Activations are NHWC in the context's storage type (fp32, or bf16 as uint16),
   rows model-major; offs is DEVICE int32 [n_groups + 1] of sample offsets.  Weights are in the library's
   internal layout [tap = ky*4+kx][c_big][c_small] ("up" form) or [tap][c_small][c_big] ("down" form), one
   block per model, in the storage type; gradients of weights are fp32 in the "up" form.
   "big" is the tensor with the larger spatial side (2*hs), "small" the one with side hs:
     down : small[n,y,x,cs]  = sum_{ky,kx,cb} big[n,2y-1+ky,2x-1+kx,cb] * w[ky,kx,cb,cs]      (conv forward, convT dgrad)
     up   : big[n,Y,X,cb]    = sum_{ky,kx,cs : Y=2y-1+ky, X=2x-1+kx} small[n,y,x,cs] * w[ky,kx,cb,cs]  (convT forward, conv dgrad)
     wgrad: dw[ky,kx,cb,cs]  = sum_{n,y,x} big[n,2y-1+ky,2x-1+kx,cb] * small[n,y,x,cs]
   n_groups models, group g uses weight block g.  n_samples = offs[n_groups] must be given by the caller. */
/* Which of the forward-type GEMM's tile shapes gan_op_conv_down / gan_op_conv_up use from now on: rows = 64, 128 or
   256 rows per tile (with 256 the width follows the output channels: 64, 128 or 256 columns), 0 = chosen from the
   problem size as inside a training step.  Lets a test run one case through every instantiation. */
gan_status gan_op_tile_rows(gan_ctx* ctx, int32_t rows);
gan_status gan_op_conv_down(gan_ctx* ctx, const void* big, const void* w_down, void* small_out, const int32_t* offs,
                            int32_t n_groups, int32_t n_samples, int32_t cb, int32_t cs, int32_t hs);
gan_status gan_op_conv_up(gan_ctx* ctx, const void* small_in, const void* w_up, void* big_out, const int32_t* offs,
                          int32_t n_groups, int32_t n_samples, int32_t cb, int32_t cs, int32_t hs);
gan_status gan_op_conv_wgrad(gan_ctx* ctx, const void* big, const void* small_in, float* dw, const int32_t* offs,
                             int32_t n_groups, int32_t n_samples, int32_t cb, int32_t cs, int32_t hs);

/* Single operations of the networks exactly as printed in Tables 1 and 2 (Section 4), synchronous like the ones above.
   (The training step for those networks is gan_train_step with family = GAN_FAMILY_PAPER.)

   gan_op_dropout: in place on a DEVICE tensor [n_samples][h][w][ch] of the context's storage type whose samples are
     grouped by model (offs: DEVICE int32 [n_groups + 1]): element <- element * keep / (1 - p) (Table 2: Dropout(0.25)).
     keep comes from Philox-4x32-10 (Salmon et al., SC'11): counter = (q low, q high, layer + 256 * pass_id, step) with
     q = index / 4, key = (seed low, seed high ^ group), index = ((n * ch + c) * h + y) * w + x with n counted inside
     the group; keep iff (output word number index % 4 >> 8) >= ceil(p * 2^24): four consecutive elements share one
     evaluation of the generator.  The backward pass is the same call on the gradient.
     layer in [0, 255]; p in [0, 1).
   gan_op_w3_to_w4: the weights that turn "Upsample(2) then Conv k3 s1 p1" (Table 1) into the k4 s2 p1 transposed
     convolution of gan_op_conv_up: per axis, tap t of the 4-tap filter is the sum of the 3-tap filter's taps in
     S(t), S = {2}, {1, 2}, {0, 1}, {0}.  w3: DEVICE fp32 [n_groups][3*3][cb][cs]; w4: DEVICE storage type
     [n_groups][4*4][cb][cs]; w4t: the same with cb and cs exchanged (the layout gan_op_conv_down reads).
   gan_op_dw4_to_dw3: the adjoint map for the weight gradient, DEVICE fp32 [n_groups][16][cb][cs] -> [n_groups][9][cb][cs]. */
gan_status gan_op_dropout(gan_ctx* ctx, void* x, const int32_t* offs, int32_t n_groups, int32_t n_samples, int32_t ch,
                          int32_t h, int32_t w, float p, uint64_t seed, int32_t step, int32_t layer, int32_t pass_id);
gan_status gan_op_w3_to_w4(gan_ctx* ctx, const float* w3, void* w4, void* w4t, int32_t n_groups, int32_t cb, int32_t cs);
gan_status gan_op_dw4_to_dw3(gan_ctx* ctx, const float* dw4, float* dw3, int32_t n_groups, int32_t cb, int32_t cs);

#ifdef __cplusplus
}
#endif
#endif
