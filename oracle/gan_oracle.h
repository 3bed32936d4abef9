/*
 * CPU oracle for the label-partitioned DC-CGAN training step.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT A PRODUCT PATH.  It is a plain, slow,
 * direct-loop implementation of what one training iteration computes, written
 * from the paper's problem statement (Section 2: spaces Z, Y, X, the functions
 * G and D, Eq. 3 for the discriminator cost, Eq. 4 for the generator cost,
 * the per-step "two minibatches + Adam" iteration, and Eq. 5, the per-label
 * factorisation that makes the K models independent).  It shares no source,
 * header, table or helper with the GPU library; only tests, the smoke check
 * and the benchmark's CPU-baseline leg may load it.
 *
 * Arithmetic type: `oreal` is double unless ORACLE_REAL is defined at build
 * time.  Tensors are NCHW, parameters are in the layouts the paper's software
 * (a stock autodiff framework) uses: conv weight [Cout][Cin][k][k], transposed
 * conv weight [Cin][Cout][k][k], linear weight [out][in].
 *
 * Parity pins: every function below is pinned by the CPU tests (brute force
 * on tiny shapes, the conv / transposed-conv adjoint identity, central finite
 * differences, BatchNorm moment invariants, closed forms of the logistic loss
 * and of Adam's first steps, an independent library's CPU ops as a black
 * box).  No function here is "parity unpinned".
 */
#ifndef GAN_ORACLE_H
#define GAN_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#ifndef ORACLE_REAL
#define ORACLE_REAL double
#endif
typedef ORACLE_REAL oreal;

#define ORACLE_MAX_LAYERS 8

/* One (G, D) pair per label (Eq. 5).  All K = n_models pairs have this shape.
 *
 * Generator:     [z ; onehot(y)] (z_dim + cond_g) -> linear -> reshape
 *                [g_ch[0], g_h0, g_h0] -> BN -> ReLU ->
 *                { convT k4 s2 p1 : g_ch[i-1] -> g_ch[i] -> BN -> ReLU } for i = 1..n_g-1
 *                -> convT k4 s2 p1 : g_ch[n_g-1] -> img_c (+bias) -> tanh
 * Discriminator: [x ; cond_d one-hot label maps] -> conv k4 s2 p1 -> d_ch[0] (+bias) -> LeakyReLU
 *                { conv k4 s2 p1 -> d_ch[j] -> BN -> LeakyReLU } for j = 1..n_d-1
 *                -> flatten (c,h,w) -> linear -> 1 logit (+bias)
 */
typedef struct {
  uint32_t struct_size;
  int32_t  n_models;      /* K in Eq. 5                                              */
  int32_t  n_labels;      /* label ids are in [0, n_labels)                          */
  int32_t  cond_g;        /* one-hot width concatenated to z (0 = none)              */
  int32_t  cond_d;        /* number of one-hot label maps appended to D's input      */
  int32_t  z_dim;         /* d_Z, 100 in the paper's tables                          */
  int32_t  img_c, img_hw; /* image channels, image side                              */
  int32_t  g_h0;          /* side of G's first feature map                           */
  int32_t  n_g;           /* number of transposed convolutions in G                  */
  int32_t  g_ch[ORACLE_MAX_LAYERS]; /* g_ch[0..n_g-1] input channels of each convT   */
  int32_t  n_d;           /* number of strided convolutions in D                     */
  int32_t  d_ch[ORACLE_MAX_LAYERS]; /* d_ch[0..n_d-1] output channels of each conv   */
  double   lr, beta1, beta2, adam_eps;
  double   bn_eps, bn_momentum, leaky_slope;
  double   d_loss_scale, g_loss_scale;   /* the factors 1/2 of Eq. 3 and Eq. 4      */
} oracle_config;

typedef struct oracle_ctx oracle_ctx;

/* ---- whole-step interface (host pointers everywhere) ------------------- */
int  oracle_create(const oracle_config* cfg, oracle_ctx** out);
void oracle_destroy(oracle_ctx* ctx);
int64_t oracle_param_count(const oracle_ctx* ctx, int which /*0 = G, 1 = D*/);
int  oracle_get_params(const oracle_ctx* ctx, int which, int model, oreal* dst);
int  oracle_set_params(oracle_ctx* ctx, int which, int model, const oreal* src);
int  oracle_get_opt_state(const oracle_ctx* ctx, int which, int model, oreal* m, oreal* v, int64_t* t);
/* restore a saved state (m, v may be NULL: left as they are); t is the number of updates taken so far */
int  oracle_set_opt_state(oracle_ctx* ctx, int which, int model, const oreal* m, const oreal* v, int64_t t);
int  oracle_set_bn_running(oracle_ctx* ctx, int which, int model, const oreal* mean, const oreal* var);
int  oracle_get_grads(const oracle_ctx* ctx, int which, int model, oreal* dst); /* of the last step */
/* BN running statistics, concatenated over the BN layers of the network: mean then var */
int64_t oracle_bn_count(const oracle_ctx* ctx, int which);
int  oracle_get_bn_running(const oracle_ctx* ctx, int which, int model, oreal* mean, oreal* var);
/* only_model < 0: step every model that received samples; otherwise only that one
   (the others are left untouched) -- used to check a subset of a large run. */
int  oracle_train_step(oracle_ctx* ctx, const int32_t* label_ids, const oreal* noise,
                       const oreal* real_batch, int32_t n, int32_t only_model);
int  oracle_generate(oracle_ctx* ctx, const int32_t* label_ids, const oreal* noise, int32_t n,
                     oreal* out_images, int32_t use_running_stats, int32_t only_model);
int  oracle_get_losses(const oracle_ctx* ctx, oreal* d_loss, oreal* g_loss, int32_t* counts);
int  oracle_get_routing(const oracle_ctx* ctx, int32_t* perm, int32_t* offs);
/* Losses only (no update): J_D of Eq. 3 and -J_G of Eq. 4 for one model on given samples, with
   train-mode BN, at the current parameters.  For finite-difference tests. */
int  oracle_eval_losses(oracle_ctx* ctx, int model, const int32_t* label_ids, const oreal* noise,
                        const oreal* real_batch, int32_t n, oreal* jd, oreal* jg);
/* Analytic gradients of the two costs at the current parameters, no update:
   gD = dJ_D/dtheta_D, gG = d(-J_G)/dtheta_G with theta_D held fixed. */
int  oracle_eval_grads(oracle_ctx* ctx, int model, const int32_t* label_ids, const oreal* noise,
                       const oreal* real_batch, int32_t n, oreal* gD, oreal* gG);
int  oracle_threads(void);

/* ---- bf16-storage emulation (a diagnostic reference, not the definition of the method) ---------------------
   With the switch on, the step rounds -- to the 16-bit format with a single's sign, exponent and top 7 mantissa bits,
   round to nearest even, via single precision -- exactly the tensors a 16-bit-storage implementation keeps in that
   format, and nothing else:
     * the network inputs (z with its one-hot part, the real images) and the generated images;
     * the weights read by the linear layer of G and by every (transposed) convolution -- per element, except the
       one-hot label planes of D's first convolution, whose taps enter as one rounded sum per output position (the
       sum of the taps inside the image) next to the rounded bias; D's final linear layer reads unrounded weights;
     * every layer output as stored: the pre-normalisation tensor (BatchNorm statistics are taken before that
       rounding, the normalisation reads the rounded tensor) and the activated tensor;
     * every stored activation gradient: after the tanh derivative, after D's linear layer, after each BatchNorm
       backward, after each data-gradient contraction (for the tensor feeding D's first convolution: after its
       LeakyReLU derivative).
   Sums, BatchNorm statistics, costs, parameter gradients, Adam and the master parameters are left in oreal.
   Off (the default) the code path is the plain algorithm, bit for bit.  Pinned by: the rounding function against
   the format's definition (ties, specials), switch-off identity, representability of the stored outputs, and the
   distance to the plain result staying within the format's error. */
int   oracle_set_bf16_emulation(oracle_ctx* ctx, int on);
oreal oracle_round_bf16(oreal x);

/* ---- single operations (for pins and for per-kernel parity tests) ------ */
void oracle_conv2d(const oreal* X, const oreal* W, const oreal* bias, oreal* Y,
                   int N, int Cin, int H, int Wd, int Cout, int k, int s, int p);
void oracle_conv2d_bwd(const oreal* X, const oreal* W, const oreal* dY,
                       oreal* dX, oreal* dW, oreal* db,
                       int N, int Cin, int H, int Wd, int Cout, int k, int s, int p);
void oracle_conv_transpose2d(const oreal* X, const oreal* W, const oreal* bias, oreal* Y,
                             int N, int Cin, int H, int Wd, int Cout, int k, int s, int p);
void oracle_conv_transpose2d_bwd(const oreal* X, const oreal* W, const oreal* dY,
                                 oreal* dX, oreal* dW, oreal* db,
                                 int N, int Cin, int H, int Wd, int Cout, int k, int s, int p);
void oracle_linear(const oreal* X, const oreal* W, const oreal* bias, oreal* Y, int N, int in, int out);
void oracle_linear_bwd(const oreal* X, const oreal* W, const oreal* dY,
                       oreal* dX, oreal* dW, oreal* db, int N, int in, int out);
void oracle_bn_train(const oreal* X, const oreal* gamma, const oreal* beta, oreal eps,
                     oreal* Y, oreal* mean, oreal* var, int N, int C, int HW);
void oracle_bn_eval(const oreal* X, const oreal* gamma, const oreal* beta, oreal eps,
                    const oreal* mean, const oreal* var, oreal* Y, int N, int C, int HW);
void oracle_bn_bwd(const oreal* X, const oreal* gamma, const oreal* mean, const oreal* var, oreal eps,
                   const oreal* dY, oreal* dX, oreal* dgamma, oreal* dbeta, int N, int C, int HW);
void oracle_bn_running_update(oreal* rmean, oreal* rvar, const oreal* mean, const oreal* var,
                              oreal momentum, int C, int64_t count);
void oracle_leaky_relu(const oreal* X, oreal* Y, int64_t n, oreal slope);       /* slope 0 = ReLU */
void oracle_leaky_relu_bwd(const oreal* X, const oreal* dY, oreal* dX, int64_t n, oreal slope);
void oracle_tanh(const oreal* X, oreal* Y, int64_t n);
void oracle_tanh_bwd(const oreal* Y, const oreal* dY, oreal* dX, int64_t n);
/* loss = scale * mean_i softplus(sign * s_i) ; ds_i = scale * sign * sigmoid(sign * s_i) / n.
   sign = -1 : -log D(.) term (target "real") ; sign = +1 : -log(1 - D(.)) term (target "fake"). */
oreal oracle_logistic_loss(const oreal* s, int n, int sign, oreal scale, oreal* ds);
void oracle_adam(oreal* theta, oreal* m, oreal* v, const oreal* g, int64_t n, int64_t t,
                 oreal lr, oreal beta1, oreal beta2, oreal eps);
void oracle_route(const int32_t* label_ids, int n, int n_models, int n_labels,
                  int32_t* perm, int32_t* offs, int32_t* n_bad);

/* ---- the mixture over the per-label generators (Eq. 5) ------------------------------------------------- */
/* Class draws from the prior p_y: label_i = the first k whose cumulative probability exceeds u_i, where the
   cumulative probabilities are the running sums (in double, in index order) of prior[k] / sum(prior) and u_i in
   [0, 1) is supplied by the caller.  Always in double, whatever oreal is: the decision is an integer.
   Returns -1 if the prior has a negative entry or sums to zero. */
int oracle_draw_labels(const double* prior, int n_labels, const float* u, int n, int32_t* labels);
/* Samples of the mixture: labels drawn as above, then image i = G_{label_i}(noise_i) (running statistics when
   use_running_stats != 0, statistics of the generated batch per model otherwise).  Same return codes as
   oracle_generate. */
int oracle_sample(oracle_ctx* ctx, const double* prior, const float* u, const oreal* noise, int32_t n,
                  oreal* out_images, int32_t* out_labels, int32_t use_running_stats);

/* ---- one-way analysis of variance of the image intensities by class (Section 4: the F-statistic quoted per
   channel for every dataset).  Observation (i, c) = the mean of channel c over the pixels of image i; groups =
   labels; F_c = [sum_k n_k (m_kc - m_c)^2 / (K' - 1)] / [sum_k sum_{i in k} (x_ic - m_kc)^2 / (n' - K')] over the
   K' labels that occur and the n' images with a valid label.  images: [n, C, H, W] floats.  Always in double.
   Returns -1 when fewer than two labels occur or n' <= K'. ------------------------------------------------- */
int oracle_anova_f(const int32_t* label_ids, const float* images, int n, int n_labels, int C, int HW, double* F);

#ifdef __cplusplus
}
#endif
#endif
