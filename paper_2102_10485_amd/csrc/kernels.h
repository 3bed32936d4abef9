// Host launchers of the bandwidth-bound kernels (routing, staging, BatchNorm + activation, the skinny first /
// last layers, losses, Adam).  T is the storage type of activations: float or bf16_t.
#pragma once

#include "common.h"

namespace gan {

constexpr int ROUTE_CHUNKS = 256;   // sequential chunks of the flat batch, one thread each
constexpr int MAX_GEOMS = 32;

// One "geometry" = how rows of a layer split into tiles: rows per sample and rows per tile.
struct GeomTable {
  int n;
  int rps[MAX_GEOMS];
  int tile_rows[MAX_GEOMS];
};

struct RouteBuffers {
  int* cnt;           // [ROUTE_CHUNKS][L] scratch
  int* counts;        // [L]
  int* offs;          // [L+1]
  int* perm;          // [n]
  int* sample_model;  // [n] model of the j-th routed sample
  int* sample_slot;   // [n] label-map slot of the j-th routed sample
  int* tpre;          // [MAX_GEOMS][L+1]
  int* tmodel;        // [MAX_GEOMS][tmodel_stride]: model of every tile of every geometry (built with tpre)
  int tmodel_stride;
  int* flags;         // [0]: out-of-range label seen
  int* order;         // [L] models by decreasing sample count (ties by index), for kernels whose work per model
                      //     follows the count (may be NULL)
};

void launch_route(const int* label_ids, int n, int L, int n_labels, const GeomTable& geoms, const RouteBuffers& rb,
                  hipStream_t st);

template <typename T>
void launch_stage(const int* label_ids, const float* noise, const float* real, int n, int L, int zdim, int cond_g, int kp,
                  int img_c, int img_hw, const RouteBuffers& rb, T* zin, T* xd, hipStream_t st);
template <typename T>
void launch_unstage(const T* fake, float* out, int n, int L, int img_c, int img_hw, const RouteBuffers& rb, hipStream_t st);

// Batch statistics and the normalise+activate passes.  Groups = (segment, model); rows of group (s, l) are the
// rps rows of each of samples s*seg_samples + offs[l] .. offs[l+1].
struct NormArgs {
  const void* x;            // pre-normalisation tensor [rows][C]
  void* y;                  // apply: activated output ; bwd apply: dx
  const void* dy;           // bwd: gradient w.r.t. the activated output
  float* mean;              // [nseg_total*L][C] (indexed by absolute segment)
  float* var;
  float* rstd;
  float* sums;              // bwd: [seg*L + l][C][2] = (sum g, sum g*xhat)
  const float* gamma;       // model 0; per-model stride pstride
  const float* beta;
  float* dgamma;            // bwd param grads (may be NULL)
  float* dbeta;
  long long pstride;
  float* run_mean;          // model 0, stride rstride (may be NULL)
  float* run_var;
  long long rstride;
  const int* offs;
  const int* counts;
  const int* sample_model;
  int L, C, rps;
  int seg_first, nseg, seg_samples;
  int n;                    // samples per segment passed by the caller (upper bound of offs[L])
  int act;                  // ACT_RELU / ACT_LRELU
  float slope, eps, momentum;
  int fold_running;         // statistics from the GEMM's partials, one segment: that kernel also updates the running statistics
  int fold_grads;           // backward reduction, one segment: its last stage also writes dgamma / dbeta
};
// statistics from the per-tile column sums a GEMM left behind (stat_partial of ConvArgs)
// (wsplit: sub-tiles per tile, conv_stat_split of the GEMM's tile)
void launch_bn_stats_from_partial(const NormArgs& a, const float* partial, const int* tpre, int ub_tiles, int nphase,
                                  int groups, int tile_rows, int gemm_rps, int wsplit, hipStream_t st);
void launch_bn_running(const NormArgs& a, hipStream_t st);
void launch_bn_from_running(const NormArgs& a, hipStream_t st);   // mean/rstd <- running statistics
template <typename T> void launch_bn_apply(const NormArgs& a, hipStream_t st);
constexpr int BN_RED_ROWS = 256;    // rows per block of the backward reduction (tile prefix geometry (rps, BN_RED_ROWS))
template <typename T>
void launch_bn_bwd_reduce(const NormArgs& a, const int* tpre, const int* tmodel, int ub_tiles, float* partial, hipStream_t st);
void launch_bn_param_grad(const NormArgs& a, hipStream_t st);
template <typename T> void launch_bn_bwd_apply(const NormArgs& a, hipStream_t st);

// The layers touching the image (1..4 channels) run as row-by-row GEMMs over an explicit patch matrix.
struct Im2colArgs {
  const void* img;          // NHWC image-side tensor (storage type), side 2*Hs, indexed by absolute sample; or NULL
  const float* real;        // caller's NCHW fp32 batch, gathered through perm (used when img == NULL)
  const int* perm;
  void* out;                // [rows][Kc] (storage type), rows indexed by absolute sample
  const int* offs;
  const int* sample_slot;
  int L, n, CB, Hs, Kc;
  int nslot;                // 0: tap columns only ; > 0: + 9*nslot class indicators + one constant column
  int seg, seg_samples;     // absolute segment of both the source tensor and the output rows
};
template <typename T> void launch_im2col(const Im2colArgs& a, hipStream_t st);

struct PackArgs {
  const float* w;           // model 0 master weights [16][CBT][Cs]; per-model stride pstride
  const float* bias;        // [Cs] (may be NULL)
  float* dw;                // unpack: gradient block of model 0, same layout as w
  float* dbias;             // unpack: may be NULL
  long long pstride;
  void* wp;                 // pack: [L][Cs][Kc] storage type
  const float* dwp;         // unpack: [nsplit][L][Kc][Cs] fp32 partial blocks
  int L, CB, CBT, Cs, Kc, nslot, nsplit;
};
template <typename T> void launch_pack_w(const PackArgs& a, hipStream_t st);
void launch_unpack_dw(const PackArgs& a, hipStream_t st);

// Transposed convolution onto the image side (G's last layer; data gradient of D's first layer).
struct UpImgArgs {
  const void* feat;         // [samples][Hs][Hs][Cs] storage type, indexed by absolute sample
  const void* w;            // model 0 storage-type weights [16][CBT][Cs]; w_stride elements between models
  long long w_stride;
  void* out;                // [samples][2Hs][2Hs][CB] storage type, indexed by absolute sample
  const void* aux;          // mode 2: the saved tanh output, same indexing as out
  const float* bias;        // mode 1: [CB] of model 0, bias_stride between models
  long long bias_stride;
  const int* offs;
  const int* sample_model;
  int L, n, seg, seg_samples;
  int CB, CBT, Cs, Hs;
  int mode;                 // 0: plain ; 1: + bias, tanh ; 2: times (1 - aux^2)
};
template <typename T> void launch_up_img(const UpImgArgs& a, hipStream_t st);

int img_bias_chunks(int L);          // pixel chunks per model of the image-side bias gradient
struct ImgBiasArgs {
  const void* img;          // [pixels][CB] of segment 0
  float* partial;           // [L][img_bias_chunks(L)][4]
  float* dbias;             // model 0, stride pstride
  long long pstride;
  const int* offs;
  int L, CB, HW;
};
template <typename T> void launch_img_bias_grad(const ImgBiasArgs& a, hipStream_t st);

// D's final linear layer (one logit), the two costs, and their gradients.
struct HeadArgs {
  const void* feat;         // [rows][K] last feature map, flattened (h,w,c)
  void* dfeat;              // gradient w.r.t. it
  const float* w;           // model 0 [K] then bias; per-model stride pstride
  const float* b;
  float* dw;
  float* db;
  long long pstride;
  float* logits;            // [nseg_total * seg_samples]
  float* dlogits;
  float* loss;              // [L]
  const int* offs;
  const int* sample_model;
  int L, K, seg_first, nseg, seg_samples, n;
  int mode;                 // loss: 0 = discriminator cost on (real, fake) ; 1 = generator cost on fake
  float scale;
  // head_bwd_w: rsplit > 1 shares every model's rows among rsplit blocks per K chunk; their partial sums go to
  // part[rsplit][L][K + 4] (the bias term at index K) and are added in order by a second kernel
  float* part;
  int rsplit;
};
template <typename T> void launch_head_fwd(const HeadArgs& a, hipStream_t st);
void launch_loss(const HeadArgs& a, hipStream_t st);
template <typename T> void launch_head_bwd_data(const HeadArgs& a, hipStream_t st);
template <typename T> void launch_head_bwd_w(const HeadArgs& a, hipStream_t st);

constexpr int ADAM_MAX_REGIONS = 8;
struct AdamArgs {
  float* theta; float* m; float* v; const float* g;
  void* shadow;             // storage-type copy of theta (NULL when the storage type is fp32)
  void* shadow_t;           // storage-type copy with every region below transposed: [tap][cs][cb]
  long long P;              // elements per model
  int L;
  const int* counts;
  int* t;                   // [L] step counts
  float* bc;                // [L][2] scratch: 1-beta1^t, 1-beta2^t
  float lr, beta1, beta2, eps;
  // Convolution weights [16][Cb][Cs] (Cb, Cs multiples of 64) that need the transposed copy: updated tile by tile.
  // Everything else is the list of gaps between them, updated as flat ranges.
  int nregions;
  long long reg_w[ADAM_MAX_REGIONS];
  int reg_cb[ADAM_MAX_REGIONS], reg_cs[ADAM_MAX_REGIONS];
  int reg_tile0[ADAM_MAX_REGIONS + 1];    // prefix of 64 x 64 tiles (filled by the launcher)
  int ngaps;
  long long gap_lo[ADAM_MAX_REGIONS + 1], gap_hi[ADAM_MAX_REGIONS + 1];
  int gap_blk0[ADAM_MAX_REGIONS + 2];     // prefix of 1024-element blocks (filled by the launcher)
  int tile_first, tile_count;             // the 64 x 64 tiles (per model) of a launch over some of the regions
};
// T: storage type of the shadows.  launch_adam does the whole update; the parts below do it piecewise (plan first).
template <typename T> void launch_adam(AdamArgs a, hipStream_t st);
bool adam_plan(AdamArgs& a);
void launch_adam_prepare(const AdamArgs& a, hipStream_t st);
void launch_adam_gaps(const AdamArgs& a, hipStream_t st);
template <typename T> void launch_adam_region(AdamArgs a, int region, hipStream_t st);
template <typename T> void launch_cast_shadow(const float* theta, T* shadow, long long total, hipStream_t st);
// dst[tap][cs][cb] <- src[tap][cb][cs] for every model (src: T or float master)
template <typename T, typename S>
void launch_transpose_w(const S* src, T* dst, long long pstride, int L, int Cb, int Cs, hipStream_t st);

// dW[l * dw_stride + i] = part[(0 * L + l) * size + i] + part[(1 * L + l) * size + i] + ... (nsplit terms, in this
// order), i < size (a multiple of 4), l < L
void launch_sum_splits(const float* part, float* dW, long long dw_stride, long long size, int L, int nsplit, hipStream_t st);

void launch_tile_prefix(const int* offs, int L, int rps, int tile_rows, int* tpre, hipStream_t st);
// tmodel[t] = model of tile t for t < tpre[L] (cap entries available)
void launch_tile_models(const int* tpre, int L, int* tmodel, int cap, hipStream_t st);

// Class draws: labels[i] = first k with cdf[k] > (double)u[i]; if none (rounding), `last` .
void launch_draw_labels(const float* u, const double* cdf, int n_labels, int last, int n, int* labels, hipStream_t st);

// One-way analysis of variance of the per-image channel means by label; all arithmetic in double, fixed order.
//   x[i][c]    = mean over the pixels of channel c of image i (images: NCHW fp32)
//   gsum[k][c] = sum of x over the images of label k, gcnt[k] = their number
//   ssw[k][c]  = sum over the images of label k of (x - gsum/gcnt)^2
void launch_anova(const int* label_ids, const float* images, int n, int n_labels, int C, int HW, double* x, double* gsum,
                  int* gcnt, double* ssw, hipStream_t st);

// ---- pieces of the networks as printed in the paper's Tables 1 and 2 (paper_layers.hip) ----
// In-place dropout of an NHWC tensor whose samples are grouped by model (offs[g] .. offs[g+1]): the keep-mask comes
// from Philox-4x32-10 with counter (element index low, high, layer + 256 * pass, step), key (seed low, seed high ^ g),
// element index ((n C + c) H + y) W + x, n counted inside the group; kept values are scaled by 1 / (1 - p).
template <typename T>
void launch_dropout(T* x, const int* offs, int n_groups, int n, int C, int H, int W, float p, unsigned long long seed, int step,
                    int layer, int pass_id, hipStream_t st);
// w4[g][ty*4+tx][cb][cs] = sum of w3[g][ky*3+kx][cb][cs] over ky in S(ty), kx in S(tx), S = {2}, {1,2}, {0,1}, {0}
// (Upsample x2 + Conv k3 s1 p1 == ConvTranspose k4 s2 p1 with these taps); w4t is the same with cb and cs exchanged.
// group g reads w3 + g * w3_stride and writes w4 + g * w4_stride, w4t + g * w4_stride (strides in elements; 0: packed)
template <typename T>
void launch_w3_to_w4(const float* w3, T* w4, T* w4t, int n_groups, int cb, int cs, hipStream_t st, long long w3_stride = 0,
                     long long w4_stride = 0);
void launch_dw4_to_dw3(const float* dw4, float* dw3, int n_groups, int cb, int cs, hipStream_t st, long long dw4_stride = 0,
                       long long dw3_stride = 0);   // the adjoint map

// ---- the training step of the networks as printed in Tables 1 and 2 (paper_step.hip) ----
// One pass over a stored NHWC tensor whose samples are grouped by model: rows of sample j (model-major) are HW pixels
// of Cpad channels, of which the first C are real (the rest is channel padding and is left alone).
struct PointArgs {
  void* x;                  // forward: the layer output, in place ; backward: the gradient, in place ; sums: the tensor
  const void* saved;        // backward: the forward result at the same positions
  const float* bias;        // forward: [C] of model 0, pstride between models (may be NULL)
  long long pstride;
  const int* offs;
  const int* sample_model;
  const int* steps;         // dropout: per-model count of iterations taken (NULL when thr == 0)
  int step_add;             // the iteration number is steps[l] + step_add
  int L, n, C, Cpad, HW;
  int seg_first, nseg, seg_samples;
  int pass_of_seg[2];       // dropout: pass id of each processed segment
  int layer;
  unsigned thr;             // ceil(p 2^24); 0: no dropout
  float scale;              // 1 / (1 - p)
  float slope;              // activation: x > 0 ? x : slope x   (1: none)
  unsigned seed_lo, seed_hi;
};
template <typename T> void launch_point_fwd(const PointArgs& a, hipStream_t st);     // x <- dropout(act(x + bias))
template <typename T> void launch_point_bwd(const PointArgs& a, hipStream_t st);     // g <- g * keep * scale * act'(saved)
// out[l * out_stride + c] = sum over the segments and rows of model l of x[.., c]
template <typename T> void launch_col_sum(const PointArgs& a, float* out, long long out_stride, hipStream_t st);
// batch statistics (mean, biased variance, 1/sqrt(var + eps)) of a stored tensor with Cpad channels per row
template <typename T> void launch_bn_stats_direct(const NormArgs& a, int Cpad, hipStream_t st);
// zero the gradient entries of the fourth tap row and column of a k3 filter held as [16][Cb][Cs]
void launch_clear_fourth_taps(float* dw, long long pstride, int L, int Cb, int Cs, hipStream_t st);

// Conv k3 s1 p1 between Cin feature channels (64 or 128) and CO image channels (1..4), side H, NHWC, rows model-major.
struct Conv3Args {
  const void* in;           // features [samples][H][H][Cin] (segment 0)
  void* out;                // forward: tanh(conv + bias) into segment out_seg of the image buffer
  const void* dout;         // backward: gradient w.r.t. the pre-tanh output, segment out_seg of the image-gradient buffer
  void* din;                // backward: gradient w.r.t. the features
  const float* w;           // [9][CO][Cin] of model 0, w_stride between models
  long long w_stride;
  const float* bias;        // [CO] of model 0
  long long bias_stride;
  const int* offs;
  const int* sample_model;
  int L, n, H, Cin, CO;
  int out_seg, seg_samples;
};
template <typename T> void launch_conv3_fwd(const Conv3Args& a, hipStream_t st);
template <typename T> void launch_conv3_dgrad(const Conv3Args& a, hipStream_t st);
// part: [conv3_wgrad_splits(L)][L][9*CO*Cin] scratch ; dw: [9][CO][Cin] of model 0, dw_stride between models
int conv3_wgrad_splits(int L);
template <typename T> void launch_conv3_wgrad(const Conv3Args& a, float* part, float* dw, long long dw_stride, hipStream_t st);

}  // namespace gan
