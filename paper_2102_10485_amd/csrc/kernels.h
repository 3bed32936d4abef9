// Host launchers of the bandwidth-bound kernels (routing, staging, BatchNorm + activation, the skinny first /
// last layers, losses, Adam).  T is the storage type of activations: float or bf16_t.
#pragma once

#include "common.h"

namespace gan {

constexpr int ROUTE_CHUNKS = 256;   // sequential chunks of the flat batch, one thread each
constexpr int MAX_GEOMS = 16;

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
  int* flags;         // [0]: out-of-range label seen
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
};
template <typename T> void launch_bn_stats(const NormArgs& a, hipStream_t st);
void launch_bn_running(const NormArgs& a, hipStream_t st);
void launch_bn_from_running(const NormArgs& a, hipStream_t st);   // mean/rstd <- running statistics
template <typename T> void launch_bn_apply(const NormArgs& a, hipStream_t st);
template <typename T> void launch_bn_bwd_reduce(const NormArgs& a, hipStream_t st);
void launch_bn_param_grad(const NormArgs& a, hipStream_t st);
template <typename T> void launch_bn_bwd_apply(const NormArgs& a, hipStream_t st);

// The layers touching the image (1..4 channels): D's first conv and G's last transposed conv.
struct SkinnyArgs {
  const void* img;          // image-side tensor [rows_big][CB] (storage type), side 2*Hs
  const void* feat;         // feature-side tensor [rows_small][Cs], side Hs
  void* out;
  const float* w;           // model 0 master weights [16][CBT][Cs]; per-model stride pstride
  const float* bias;        // may be NULL
  long long pstride;
  const float* table;       // label-map table [L][nslot][9][Cs] (may be NULL)
  const int* sample_slot;
  int nslot;
  const void* aux;          // up+tanh_bwd: the tanh output at the same position
  const int* offs;
  const int* tpre;
  int L, CB, CBT, Cs, Hs;
  int seg_first, nseg, seg_samples, ub_tiles;
  int lrelu;                // down: apply LeakyReLU(slope)
  int tanh_out;             // up: 1 = add bias and apply tanh ; 2 = multiply by (1 - aux^2)
  float slope;
  float* partial;           // wgrad: [nseg][ub_tiles][256/Cs][16*CB][Cs]
  float* dw;                // wgrad: model 0 gradient [16][CBT][Cs], stride pstride
  float* dbias;             // G last layer: [CB] per model (may be NULL)
};
constexpr int SKINNY_DOWN_ROWS = 32;
constexpr int SKINNY_UP_ROWS = 32;
constexpr int SKINNY_WGRAD_ROWS = 2048;
template <typename T> void launch_skinny_down(const SkinnyArgs& a, hipStream_t st);
template <typename T> void launch_skinny_up(const SkinnyArgs& a, hipStream_t st);
template <typename T> void launch_skinny_wgrad(const SkinnyArgs& a, hipStream_t st);
template <typename T> void launch_img_bias_grad(const SkinnyArgs& a, hipStream_t st);

// Label maps of D's first conv: a constant one-hot plane contributes a per-position bias (border classes 3 x 3).
struct LabelMapArgs {
  const float* w;           // model 0 [16][CBT][Cs]
  float* dw;
  float* dbias;             // [Cs] per model
  long long pstride;
  float* table;             // [L][nslot][9][Cs]
  float* rsum;              // [L][nslot][9][Cs]
  const void* dfeat;        // dx of the first conv's output [rows][Cs]
  const int* offs;
  const int* sample_slot;
  int L, nslot, CB, CBT, Cs, Hs, nseg, seg_samples;
};
void launch_labelmap_table(const LabelMapArgs& a, hipStream_t st);
template <typename T> void launch_labelmap_reduce(const LabelMapArgs& a, hipStream_t st);
void launch_labelmap_grads(const LabelMapArgs& a, hipStream_t st);

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
};
template <typename T> void launch_head_fwd(const HeadArgs& a, hipStream_t st);
void launch_loss(const HeadArgs& a, hipStream_t st);
template <typename T> void launch_head_bwd_data(const HeadArgs& a, hipStream_t st);
template <typename T> void launch_head_bwd_w(const HeadArgs& a, hipStream_t st);

struct AdamArgs {
  float* theta; float* m; float* v; const float* g;
  void* shadow;             // storage-type copy of theta (NULL when the storage type is fp32)
  long long P;              // elements per model
  int L;
  const int* counts;
  int* t;                   // [L] step counts
  float* bc;                // [L][2] scratch: 1-beta1^t, 1-beta2^t
  float lr, beta1, beta2, eps;
};
void launch_adam(const AdamArgs& a, hipStream_t st);
template <typename T> void launch_cast_shadow(const float* theta, T* shadow, long long total, hipStream_t st);
// dst[tap][cs][cb] <- src[tap][cb][cs] for every model (src: T or float master)
template <typename T, typename S>
void launch_transpose_w(const S* src, T* dst, long long pstride, int L, int Cb, int Cs, hipStream_t st);

void launch_tile_prefix(const int* offs, int L, int rps, int tile_rows, int* tpre, hipStream_t st);

}  // namespace gan
