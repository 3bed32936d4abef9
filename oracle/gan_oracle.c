/*
 * CPU oracle (test infrastructure only) -- see gan_oracle.h.
 *
 * Every operation is the textbook definition written as direct loops; the
 * training step takes the steps of the paper's iteration in its order
 * (Section 2: sample a minibatch of x and one of z, update theta_D on Eq. 3,
 * update theta_G on Eq. 4, with Adam), once per label-model (Eq. 5).
 */
#include "gan_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define KSZ 4   /* kernel size, stride and padding of every (transposed) convolution in the nets */
#define STR 2
#define PAD 1

/* ======================================================================= */
/* single operations                                                       */
/* ======================================================================= */

/* Cross-correlation: Y[n,co,oy,ox] = b[co] + sum_{ci,ky,kx} X[n,ci,oy*s-p+ky,ox*s-p+kx] W[co,ci,ky,kx],
   reads outside X count as zero. */
void oracle_conv2d(const oreal* X, const oreal* W, const oreal* bias, oreal* Y,
                   int N, int Cin, int H, int Wd, int Cout, int k, int s, int p) {
  const int Ho = (H + 2 * p - k) / s + 1, Wo = (Wd + 2 * p - k) / s + 1;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int co = 0; co < Cout; ++co) {
      oreal* y = Y + ((int64_t)n * Cout + co) * Ho * Wo;
      for (int i = 0; i < Ho * Wo; ++i) y[i] = bias ? bias[co] : (oreal)0;
      for (int ci = 0; ci < Cin; ++ci) {
        const oreal* x = X + ((int64_t)n * Cin + ci) * H * Wd;
        for (int ky = 0; ky < k; ++ky)
          for (int kx = 0; kx < k; ++kx) {
            const oreal w = W[(((int64_t)co * Cin + ci) * k + ky) * k + kx];
            for (int oy = 0; oy < Ho; ++oy) {
              const int iy = oy * s - p + ky;
              if (iy < 0 || iy >= H) continue;
              for (int ox = 0; ox < Wo; ++ox) {
                const int ix = ox * s - p + kx;
                if (ix < 0 || ix >= Wd) continue;
                y[oy * Wo + ox] += w * x[iy * Wd + ix];
              }
            }
          }
      }
    }
}

/* Gradients of conv2d by differentiating its defining sum term by term. */
void oracle_conv2d_bwd(const oreal* X, const oreal* W, const oreal* dY,
                       oreal* dX, oreal* dW, oreal* db,
                       int N, int Cin, int H, int Wd, int Cout, int k, int s, int p) {
  const int Ho = (H + 2 * p - k) / s + 1, Wo = (Wd + 2 * p - k) / s + 1;
  if (dW) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int co = 0; co < Cout; ++co)
      for (int ci = 0; ci < Cin; ++ci)
        for (int ky = 0; ky < k; ++ky)
          for (int kx = 0; kx < k; ++kx) {
            oreal acc = 0;
            for (int n = 0; n < N; ++n) {
              const oreal* x = X + ((int64_t)n * Cin + ci) * H * Wd;
              const oreal* dy = dY + ((int64_t)n * Cout + co) * Ho * Wo;
              for (int oy = 0; oy < Ho; ++oy) {
                const int iy = oy * s - p + ky;
                if (iy < 0 || iy >= H) continue;
                for (int ox = 0; ox < Wo; ++ox) {
                  const int ix = ox * s - p + kx;
                  if (ix < 0 || ix >= Wd) continue;
                  acc += x[iy * Wd + ix] * dy[oy * Wo + ox];
                }
              }
            }
            dW[(((int64_t)co * Cin + ci) * k + ky) * k + kx] = acc;
          }
  }
  if (db) {
    for (int co = 0; co < Cout; ++co) {
      oreal acc = 0;
      for (int n = 0; n < N; ++n) {
        const oreal* dy = dY + ((int64_t)n * Cout + co) * Ho * Wo;
        for (int i = 0; i < Ho * Wo; ++i) acc += dy[i];
      }
      db[co] = acc;
    }
  }
  if (dX) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
      for (int ci = 0; ci < Cin; ++ci) {
        oreal* dx = dX + ((int64_t)n * Cin + ci) * H * Wd;
        for (int i = 0; i < H * Wd; ++i) dx[i] = 0;
        for (int co = 0; co < Cout; ++co) {
          const oreal* dy = dY + ((int64_t)n * Cout + co) * Ho * Wo;
          for (int ky = 0; ky < k; ++ky)
            for (int kx = 0; kx < k; ++kx) {
              const oreal w = W[(((int64_t)co * Cin + ci) * k + ky) * k + kx];
              for (int oy = 0; oy < Ho; ++oy) {
                const int iy = oy * s - p + ky;
                if (iy < 0 || iy >= H) continue;
                for (int ox = 0; ox < Wo; ++ox) {
                  const int ix = ox * s - p + kx;
                  if (ix < 0 || ix >= Wd) continue;
                  dx[iy * Wd + ix] += w * dy[oy * Wo + ox];
                }
              }
            }
        }
      }
  }
}

/* Transposed convolution: the adjoint of conv2d with the same weight tensor read as [Cin][Cout][k][k].
   Y[n,co,oy,ox] = b[co] + sum over (ci,ky,kx,iy,ix) with oy = iy*s-p+ky, ox = ix*s-p+kx of X[n,ci,iy,ix] W[ci,co,ky,kx].
   Output side (H-1)*s - 2p + k. */
void oracle_conv_transpose2d(const oreal* X, const oreal* W, const oreal* bias, oreal* Y,
                             int N, int Cin, int H, int Wd, int Cout, int k, int s, int p) {
  const int Ho = (H - 1) * s - 2 * p + k, Wo = (Wd - 1) * s - 2 * p + k;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int co = 0; co < Cout; ++co) {
      oreal* y = Y + ((int64_t)n * Cout + co) * Ho * Wo;
      for (int i = 0; i < Ho * Wo; ++i) y[i] = bias ? bias[co] : (oreal)0;
      for (int ci = 0; ci < Cin; ++ci) {
        const oreal* x = X + ((int64_t)n * Cin + ci) * H * Wd;
        for (int ky = 0; ky < k; ++ky)
          for (int kx = 0; kx < k; ++kx) {
            const oreal w = W[(((int64_t)ci * Cout + co) * k + ky) * k + kx];
            for (int iy = 0; iy < H; ++iy) {
              const int oy = iy * s - p + ky;
              if (oy < 0 || oy >= Ho) continue;
              for (int ix = 0; ix < Wd; ++ix) {
                const int ox = ix * s - p + kx;
                if (ox < 0 || ox >= Wo) continue;
                y[oy * Wo + ox] += w * x[iy * Wd + ix];
              }
            }
          }
      }
    }
}

void oracle_conv_transpose2d_bwd(const oreal* X, const oreal* W, const oreal* dY,
                                 oreal* dX, oreal* dW, oreal* db,
                                 int N, int Cin, int H, int Wd, int Cout, int k, int s, int p) {
  const int Ho = (H - 1) * s - 2 * p + k, Wo = (Wd - 1) * s - 2 * p + k;
  if (dW) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int ci = 0; ci < Cin; ++ci)
      for (int co = 0; co < Cout; ++co)
        for (int ky = 0; ky < k; ++ky)
          for (int kx = 0; kx < k; ++kx) {
            oreal acc = 0;
            for (int n = 0; n < N; ++n) {
              const oreal* x = X + ((int64_t)n * Cin + ci) * H * Wd;
              const oreal* dy = dY + ((int64_t)n * Cout + co) * Ho * Wo;
              for (int iy = 0; iy < H; ++iy) {
                const int oy = iy * s - p + ky;
                if (oy < 0 || oy >= Ho) continue;
                for (int ix = 0; ix < Wd; ++ix) {
                  const int ox = ix * s - p + kx;
                  if (ox < 0 || ox >= Wo) continue;
                  acc += x[iy * Wd + ix] * dy[oy * Wo + ox];
                }
              }
            }
            dW[(((int64_t)ci * Cout + co) * k + ky) * k + kx] = acc;
          }
  }
  if (db) {
    for (int co = 0; co < Cout; ++co) {
      oreal acc = 0;
      for (int n = 0; n < N; ++n) {
        const oreal* dy = dY + ((int64_t)n * Cout + co) * Ho * Wo;
        for (int i = 0; i < Ho * Wo; ++i) acc += dy[i];
      }
      db[co] = acc;
    }
  }
  if (dX) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
      for (int ci = 0; ci < Cin; ++ci) {
        oreal* dx = dX + ((int64_t)n * Cin + ci) * H * Wd;
        for (int i = 0; i < H * Wd; ++i) dx[i] = 0;
        for (int co = 0; co < Cout; ++co) {
          const oreal* dy = dY + ((int64_t)n * Cout + co) * Ho * Wo;
          for (int ky = 0; ky < k; ++ky)
            for (int kx = 0; kx < k; ++kx) {
              const oreal w = W[(((int64_t)ci * Cout + co) * k + ky) * k + kx];
              for (int iy = 0; iy < H; ++iy) {
                const int oy = iy * s - p + ky;
                if (oy < 0 || oy >= Ho) continue;
                for (int ix = 0; ix < Wd; ++ix) {
                  const int ox = ix * s - p + kx;
                  if (ox < 0 || ox >= Wo) continue;
                  dx[iy * Wd + ix] += w * dy[oy * Wo + ox];
                }
              }
            }
        }
      }
  }
}

void oracle_linear(const oreal* X, const oreal* W, const oreal* bias, oreal* Y, int N, int in, int out) {
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int o = 0; o < out; ++o) {
      oreal acc = bias ? bias[o] : (oreal)0;
      for (int i = 0; i < in; ++i) acc += X[(int64_t)n * in + i] * W[(int64_t)o * in + i];
      Y[(int64_t)n * out + o] = acc;
    }
}

void oracle_linear_bwd(const oreal* X, const oreal* W, const oreal* dY,
                       oreal* dX, oreal* dW, oreal* db, int N, int in, int out) {
  if (dW) {
#pragma omp parallel for schedule(static)
    for (int o = 0; o < out; ++o)
      for (int i = 0; i < in; ++i) {
        oreal acc = 0;
        for (int n = 0; n < N; ++n) acc += dY[(int64_t)n * out + o] * X[(int64_t)n * in + i];
        dW[(int64_t)o * in + i] = acc;
      }
  }
  if (db) {
    for (int o = 0; o < out; ++o) {
      oreal acc = 0;
      for (int n = 0; n < N; ++n) acc += dY[(int64_t)n * out + o];
      db[o] = acc;
    }
  }
  if (dX) {
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
      for (int i = 0; i < in; ++i) {
        oreal acc = 0;
        for (int o = 0; o < out; ++o) acc += dY[(int64_t)n * out + o] * W[(int64_t)o * in + i];
        dX[(int64_t)n * in + i] = acc;
      }
  }
}

/* Training-mode batch normalisation over (n, y, x) per channel: biased variance normalises. */
void oracle_bn_train(const oreal* X, const oreal* gamma, const oreal* beta, oreal eps,
                     oreal* Y, oreal* mean, oreal* var, int N, int C, int HW) {
#pragma omp parallel for schedule(static)
  for (int c = 0; c < C; ++c) {
    const oreal cnt = (oreal)N * HW;
    oreal mu = 0;
    for (int n = 0; n < N; ++n)
      for (int i = 0; i < HW; ++i) mu += X[((int64_t)n * C + c) * HW + i];
    mu /= cnt;
    oreal v = 0;
    for (int n = 0; n < N; ++n)
      for (int i = 0; i < HW; ++i) {
        const oreal d = X[((int64_t)n * C + c) * HW + i] - mu;
        v += d * d;
      }
    v /= cnt;
    mean[c] = mu;
    var[c] = v;
    const oreal rstd = (oreal)1 / sqrt(v + eps);
    for (int n = 0; n < N; ++n)
      for (int i = 0; i < HW; ++i) {
        const int64_t j = ((int64_t)n * C + c) * HW + i;
        Y[j] = gamma[c] * ((X[j] - mu) * rstd) + beta[c];
      }
  }
}

void oracle_bn_eval(const oreal* X, const oreal* gamma, const oreal* beta, oreal eps,
                    const oreal* mean, const oreal* var, oreal* Y, int N, int C, int HW) {
  for (int c = 0; c < C; ++c) {
    const oreal rstd = (oreal)1 / sqrt(var[c] + eps);
    for (int n = 0; n < N; ++n)
      for (int i = 0; i < HW; ++i) {
        const int64_t j = ((int64_t)n * C + c) * HW + i;
        Y[j] = gamma[c] * ((X[j] - mean[c]) * rstd) + beta[c];
      }
  }
}

/* With xhat = (x - mu) * rstd and S = N*HW:
   dbeta = sum dy ; dgamma = sum dy*xhat ; dx = gamma*rstd*(dy - dbeta/S - xhat*dgamma/S). */
void oracle_bn_bwd(const oreal* X, const oreal* gamma, const oreal* mean, const oreal* var, oreal eps,
                   const oreal* dY, oreal* dX, oreal* dgamma, oreal* dbeta, int N, int C, int HW) {
#pragma omp parallel for schedule(static)
  for (int c = 0; c < C; ++c) {
    const oreal cnt = (oreal)N * HW;
    const oreal rstd = (oreal)1 / sqrt(var[c] + eps);
    oreal sb = 0, sg = 0;
    for (int n = 0; n < N; ++n)
      for (int i = 0; i < HW; ++i) {
        const int64_t j = ((int64_t)n * C + c) * HW + i;
        sb += dY[j];
        sg += dY[j] * ((X[j] - mean[c]) * rstd);
      }
    if (dbeta) dbeta[c] = sb;
    if (dgamma) dgamma[c] = sg;
    for (int n = 0; n < N; ++n)
      for (int i = 0; i < HW; ++i) {
        const int64_t j = ((int64_t)n * C + c) * HW + i;
        const oreal xh = (X[j] - mean[c]) * rstd;
        dX[j] = gamma[c] * rstd * (dY[j] - sb / cnt - xh * sg / cnt);
      }
  }
}

/* running <- (1-mom)*running + mom*batch ; the variance stored is the unbiased one.
   With a single element (count == 1) the unbiased variance is undefined: the variance is left alone. */
void oracle_bn_running_update(oreal* rmean, oreal* rvar, const oreal* mean, const oreal* var,
                              oreal momentum, int C, int64_t count) {
  for (int c = 0; c < C; ++c) {
    rmean[c] = ((oreal)1 - momentum) * rmean[c] + momentum * mean[c];
    if (count > 1)
      rvar[c] = ((oreal)1 - momentum) * rvar[c] + momentum * var[c] * ((oreal)count / (oreal)(count - 1));
  }
}

void oracle_leaky_relu(const oreal* X, oreal* Y, int64_t n, oreal slope) {
  for (int64_t i = 0; i < n; ++i) Y[i] = X[i] > 0 ? X[i] : slope * X[i];
}
void oracle_leaky_relu_bwd(const oreal* X, const oreal* dY, oreal* dX, int64_t n, oreal slope) {
  for (int64_t i = 0; i < n; ++i) dX[i] = X[i] > 0 ? dY[i] : slope * dY[i];
}
void oracle_tanh(const oreal* X, oreal* Y, int64_t n) {
  for (int64_t i = 0; i < n; ++i) Y[i] = tanh(X[i]);
}
void oracle_tanh_bwd(const oreal* Y, const oreal* dY, oreal* dX, int64_t n) {
  for (int64_t i = 0; i < n; ++i) dX[i] = dY[i] * ((oreal)1 - Y[i] * Y[i]);
}

static oreal softplus_(oreal u) { return (u > 0 ? u : (oreal)0) + log1p(exp(-fabs(u))); }
static oreal sigmoid_(oreal u) {
  if (u >= 0) return (oreal)1 / ((oreal)1 + exp(-u));
  const oreal e = exp(u);
  return e / ((oreal)1 + e);
}

/* With D = sigmoid(s): -log D = softplus(-s), -log(1-D) = softplus(s)  (Eq. 3, Eq. 4). */
oreal oracle_logistic_loss(const oreal* s, int n, int sign, oreal scale, oreal* ds) {
  oreal acc = 0;
  for (int i = 0; i < n; ++i) {
    const oreal u = (oreal)sign * s[i];
    acc += softplus_(u);
    if (ds) ds[i] = scale * (oreal)sign * sigmoid_(u) / (oreal)n;
  }
  return scale * acc / (oreal)n;
}

/* Adam with bias correction, epsilon added outside the square root, no weight decay. */
void oracle_adam(oreal* theta, oreal* m, oreal* v, const oreal* g, int64_t n, int64_t t,
                 oreal lr, oreal beta1, oreal beta2, oreal eps) {
  const oreal c1 = (oreal)1 - pow(beta1, (oreal)t), c2 = (oreal)1 - pow(beta2, (oreal)t);
  for (int64_t i = 0; i < n; ++i) {
    m[i] = beta1 * m[i] + ((oreal)1 - beta1) * g[i];
    v[i] = beta2 * v[i] + ((oreal)1 - beta2) * g[i] * g[i];
    const oreal mh = m[i] / c1, vh = v[i] / c2;
    theta[i] -= lr * mh / (sqrt(vh) + eps);
  }
}

/* Stable partition of sample indices by model.  model(i) = label if there is one model per label,
   0 if there is a single model.  Out-of-range labels are dropped and counted. */
void oracle_route(const int32_t* label_ids, int n, int n_models, int n_labels,
                  int32_t* perm, int32_t* offs, int32_t* n_bad) {
  int pos = 0, bad = 0;
  for (int l = 0; l < n_models; ++l) {
    offs[l] = pos;
    for (int i = 0; i < n; ++i) {
      const int y = label_ids[i];
      if (y < 0 || y >= n_labels) continue;
      const int mdl = (n_models == 1) ? 0 : y;
      if (mdl == l) perm[pos++] = i;
    }
  }
  offs[n_models] = pos;
  for (int i = 0; i < n; ++i)
    if (label_ids[i] < 0 || label_ids[i] >= n_labels) ++bad;
  for (int i = pos; i < n; ++i) perm[i] = -1;
  if (n_bad) *n_bad = bad;
}

int oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ======================================================================= */
/* the networks                                                            */
/* ======================================================================= */

typedef struct {
  int64_t w, bias, gamma, beta;   /* offsets into the flat parameter vector, -1 if absent */
  int64_t rs;                     /* offset into the running-statistics vector, -1 if no BN */
  int64_t nw; int nbias, nbn;     /* number of weights, of biases, of BN channels */
  int cin, cout, hin, hout;       /* hin/hout: input / output side (1 for the linear layers' flat side) */
} layer_t;

typedef struct {
  int64_t nparams, nbn;
  int nlayers;
  layer_t L[ORACLE_MAX_LAYERS + 2];
} net_t;

struct oracle_ctx {
  oracle_config cfg;
  net_t G, D;
  oreal *thG, *mG, *vG, *gG;     /* [n_models][G.nparams] */
  oreal *thD, *mD, *vD, *gD;
  oreal *rmG, *rvG, *rmD, *rvD;  /* running mean / var [n_models][nbn] */
  int64_t *tG, *tD;              /* Adam step counts per model */
  oreal *jd, *jg;                /* last losses per model */
  int32_t *counts, *perm, *offs;
  int32_t last_n, n_bad;
  int emul;                      /* bf16-storage emulation (see oracle_set_bf16_emulation); 0 = the plain algorithm */
};

/* ---- bf16-storage emulation -------------------------------------------------------------------------------
   A 16-bit storage format with the sign, the 8 exponent bits and the top 7 mantissa bits of an IEEE single
   ("bfloat16"); conversion from a single rounds to nearest, ties to even.  A value held in a wider type is first
   rounded to single (that is what an fp32 accumulator holds), then to the 16-bit format. */
oreal oracle_round_bf16(oreal x) {
  union { float f; uint32_t u; } c;
  c.f = (float)x;
  if ((c.u & 0x7fffffffu) > 0x7f800000u) return x;          /* NaN stays NaN */
  c.u += 0x7fffu + ((c.u >> 16) & 1u);
  c.u &= 0xffff0000u;
  return (oreal)c.f;
}
static void qv(const oracle_ctx* c, oreal* x, int64_t n) {
  if (!c->emul) return;
  for (int64_t i = 0; i < n; ++i) x[i] = oracle_round_bf16(x[i]);
}
/* The weights as a 16-bit-storage implementation multiplies them: a copy of theta with the weights of layers
   [0, nl) rounded (biases and BatchNorm parameters stay as they are).  NULL when emulation is off. */
static oreal* shadow_weights(const oracle_ctx* c, const net_t* net, const oreal* th, int nl) {
  if (!c->emul) return NULL;
  oreal* q = (oreal*)malloc(sizeof(oreal) * (size_t)net->nparams);
  memcpy(q, th, sizeof(oreal) * (size_t)net->nparams);
  for (int i = 0; i < nl; ++i) qv(c, q + net->L[i].w, net->L[i].nw);
  return q;
}
int oracle_set_bf16_emulation(oracle_ctx* c, int on) {
  if (!c) return -1;
  c->emul = on ? 1 : 0;
  return 0;
}

static void build_nets(oracle_ctx* c) {
  const oracle_config* f = &c->cfg;
  net_t* G = &c->G;
  int64_t o = 0, r = 0;
  int li = 0;
  /* G layer 0: linear (no bias: BN follows) + BN over g_ch[0] channels */
  layer_t* l = &G->L[li++];
  l->cin = f->z_dim + f->cond_g; l->cout = f->g_ch[0] * f->g_h0 * f->g_h0; l->hin = 1; l->hout = f->g_h0;
  l->nw = (int64_t)l->cin * l->cout; l->nbias = 0; l->nbn = f->g_ch[0];
  l->w = o; o += l->nw; l->bias = -1;
  l->gamma = o; o += f->g_ch[0]; l->beta = o; o += f->g_ch[0]; l->rs = r; r += f->g_ch[0];
  int h = f->g_h0;
  for (int i = 1; i <= f->n_g; ++i) {
    l = &G->L[li++];
    l->cin = f->g_ch[i - 1]; l->cout = (i < f->n_g) ? f->g_ch[i] : f->img_c; l->hin = h; l->hout = 2 * h; h *= 2;
    l->nw = (int64_t)l->cin * l->cout * KSZ * KSZ; l->w = o; o += l->nw;
    if (i < f->n_g) { l->nbias = 0; l->nbn = l->cout; l->bias = -1; l->gamma = o; o += l->cout; l->beta = o; o += l->cout; l->rs = r; r += l->cout; }
    else { l->nbias = l->cout; l->nbn = 0; l->bias = o; o += l->cout; l->gamma = l->beta = -1; l->rs = -1; }
  }
  G->nlayers = li; G->nparams = o; G->nbn = r;

  net_t* D = &c->D;
  o = 0; r = 0; li = 0; h = f->img_hw;
  for (int j = 0; j < f->n_d; ++j) {
    l = &D->L[li++];
    l->cin = (j == 0) ? f->img_c + f->cond_d : f->d_ch[j - 1]; l->cout = f->d_ch[j]; l->hin = h; l->hout = h / 2; h /= 2;
    l->nw = (int64_t)l->cin * l->cout * KSZ * KSZ; l->w = o; o += l->nw;
    if (j == 0) { l->nbias = l->cout; l->nbn = 0; l->bias = o; o += l->cout; l->gamma = l->beta = -1; l->rs = -1; }
    else { l->nbias = 0; l->nbn = l->cout; l->bias = -1; l->gamma = o; o += l->cout; l->beta = o; o += l->cout; l->rs = r; r += l->cout; }
  }
  l = &D->L[li++];
  l->cin = f->d_ch[f->n_d - 1] * h * h; l->cout = 1; l->hin = h; l->hout = 1;
  l->nw = l->cin; l->nbias = 1; l->nbn = 0;
  l->w = o; o += l->cin; l->bias = o; o += 1; l->gamma = l->beta = -1; l->rs = -1;
  D->nlayers = li; D->nparams = o; D->nbn = r;
}

/* small deterministic generator for the built-in initialiser only (tests overwrite the parameters) */
static uint64_t splitmix(uint64_t* s) {
  uint64_t z = (*s += 0x9E3779B97F4A7C15ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
static double gauss(uint64_t* s) {
  const double u1 = ((splitmix(s) >> 11) + 1.0) / 9007199254740993.0;
  const double u2 = (splitmix(s) >> 11) / 9007199254740992.0;
  return sqrt(-2.0 * log(u1)) * cos(6.283185307179586 * u2);
}

static void init_net(const net_t* net, oreal* th, uint64_t* seed) {
  for (int i = 0; i < net->nlayers; ++i) {
    const layer_t* l = &net->L[i];
    for (int64_t j = 0; j < l->nw; ++j) th[l->w + j] = (oreal)(0.02 * gauss(seed));
    for (int j = 0; j < l->nbias; ++j) th[l->bias + j] = 0;
    for (int j = 0; j < l->nbn; ++j) { th[l->gamma + j] = 1; th[l->beta + j] = 0; }
  }
}

int oracle_create(const oracle_config* cfg, oracle_ctx** out) {
  if (!cfg || !out || cfg->struct_size != sizeof(oracle_config)) return -1;
  if (cfg->n_models < 1 || cfg->n_g < 1 || cfg->n_d < 1 || cfg->n_g > ORACLE_MAX_LAYERS || cfg->n_d > ORACLE_MAX_LAYERS) return -1;
  if (cfg->n_models != 1 && cfg->n_models != cfg->n_labels) return -1;
  if (cfg->g_h0 << cfg->n_g != cfg->img_hw) return -2;
  if ((cfg->img_hw >> cfg->n_d) << cfg->n_d != cfg->img_hw) return -2;
  oracle_ctx* c = (oracle_ctx*)calloc(1, sizeof(oracle_ctx));
  c->cfg = *cfg;
  build_nets(c);
  const int K = cfg->n_models;
#define ALLOC(p, n) p = (oreal*)calloc((size_t)(n), sizeof(oreal))
  ALLOC(c->thG, K * c->G.nparams); ALLOC(c->mG, K * c->G.nparams); ALLOC(c->vG, K * c->G.nparams); ALLOC(c->gG, K * c->G.nparams);
  ALLOC(c->thD, K * c->D.nparams); ALLOC(c->mD, K * c->D.nparams); ALLOC(c->vD, K * c->D.nparams); ALLOC(c->gD, K * c->D.nparams);
  ALLOC(c->rmG, K * c->G.nbn); ALLOC(c->rvG, K * c->G.nbn); ALLOC(c->rmD, K * c->D.nbn); ALLOC(c->rvD, K * c->D.nbn);
  ALLOC(c->jd, K); ALLOC(c->jg, K);
#undef ALLOC
  c->tG = (int64_t*)calloc(K, sizeof(int64_t)); c->tD = (int64_t*)calloc(K, sizeof(int64_t));
  c->counts = (int32_t*)calloc(K, sizeof(int32_t)); c->offs = (int32_t*)calloc(K + 1, sizeof(int32_t));
  c->perm = NULL; c->last_n = 0;
  uint64_t seed = 0x210210485ull;
  for (int k = 0; k < K; ++k) {
    init_net(&c->G, c->thG + k * c->G.nparams, &seed);
    init_net(&c->D, c->thD + k * c->D.nparams, &seed);
    for (int64_t j = 0; j < c->G.nbn; ++j) c->rvG[k * c->G.nbn + j] = 1;
    for (int64_t j = 0; j < c->D.nbn; ++j) c->rvD[k * c->D.nbn + j] = 1;
  }
  *out = c;
  return 0;
}

void oracle_destroy(oracle_ctx* c) {
  if (!c) return;
  free(c->thG); free(c->mG); free(c->vG); free(c->gG); free(c->thD); free(c->mD); free(c->vD); free(c->gD);
  free(c->rmG); free(c->rvG); free(c->rmD); free(c->rvD); free(c->jd); free(c->jg);
  free(c->tG); free(c->tD); free(c->counts); free(c->offs); free(c->perm);
  free(c);
}

int64_t oracle_param_count(const oracle_ctx* c, int which) { return which == 0 ? c->G.nparams : c->D.nparams; }
int64_t oracle_bn_count(const oracle_ctx* c, int which) { return which == 0 ? c->G.nbn : c->D.nbn; }

int oracle_get_params(const oracle_ctx* c, int which, int model, oreal* dst) {
  if (model < 0 || model >= c->cfg.n_models) return -1;
  const int64_t P = oracle_param_count(c, which);
  memcpy(dst, (which == 0 ? c->thG : c->thD) + model * P, P * sizeof(oreal));
  return 0;
}
int oracle_set_params(oracle_ctx* c, int which, int model, const oreal* src) {
  if (model < 0 || model >= c->cfg.n_models) return -1;
  const int64_t P = oracle_param_count(c, which);
  memcpy((which == 0 ? c->thG : c->thD) + model * P, src, P * sizeof(oreal));
  return 0;
}
int oracle_get_opt_state(const oracle_ctx* c, int which, int model, oreal* m, oreal* v, int64_t* t) {
  if (model < 0 || model >= c->cfg.n_models) return -1;
  const int64_t P = oracle_param_count(c, which);
  if (m) memcpy(m, (which == 0 ? c->mG : c->mD) + model * P, P * sizeof(oreal));
  if (v) memcpy(v, (which == 0 ? c->vG : c->vD) + model * P, P * sizeof(oreal));
  if (t) *t = (which == 0 ? c->tG : c->tD)[model];
  return 0;
}
int oracle_set_opt_state(oracle_ctx* c, int which, int model, const oreal* m, const oreal* v, int64_t t) {
  if (model < 0 || model >= c->cfg.n_models || t < 0) return -1;
  const int64_t P = oracle_param_count(c, which);
  if (m) memcpy((which == 0 ? c->mG : c->mD) + model * P, m, P * sizeof(oreal));
  if (v) memcpy((which == 0 ? c->vG : c->vD) + model * P, v, P * sizeof(oreal));
  (which == 0 ? c->tG : c->tD)[model] = t;
  return 0;
}
int oracle_set_bn_running(oracle_ctx* c, int which, int model, const oreal* mean, const oreal* var) {
  if (model < 0 || model >= c->cfg.n_models) return -1;
  const int64_t B = oracle_bn_count(c, which);
  memcpy((which == 0 ? c->rmG : c->rmD) + model * B, mean, B * sizeof(oreal));
  memcpy((which == 0 ? c->rvG : c->rvD) + model * B, var, B * sizeof(oreal));
  return 0;
}
int oracle_get_grads(const oracle_ctx* c, int which, int model, oreal* dst) {
  if (model < 0 || model >= c->cfg.n_models) return -1;
  const int64_t P = oracle_param_count(c, which);
  memcpy(dst, (which == 0 ? c->gG : c->gD) + model * P, P * sizeof(oreal));
  return 0;
}
int oracle_get_bn_running(const oracle_ctx* c, int which, int model, oreal* mean, oreal* var) {
  if (model < 0 || model >= c->cfg.n_models) return -1;
  const int64_t B = oracle_bn_count(c, which);
  memcpy(mean, (which == 0 ? c->rmG : c->rmD) + model * B, B * sizeof(oreal));
  memcpy(var, (which == 0 ? c->rvG : c->rvD) + model * B, B * sizeof(oreal));
  return 0;
}

/* ---- forward / backward of one model on b samples ---------------------- */

typedef struct {
  int b;
  oreal* in;                       /* network input (G: [b, z+cond]; D: [b, C+cond, H, H]) */
  oreal* pre[ORACLE_MAX_LAYERS + 2];   /* layer output before BN / activation */
  oreal* act[ORACLE_MAX_LAYERS + 2];   /* after BN + activation (what the next layer reads) */
  oreal* mean[ORACLE_MAX_LAYERS + 2];
  oreal* var[ORACLE_MAX_LAYERS + 2];
} cache_t;

static int64_t layer_out_elems(const net_t* net, int i, int b) {
  const layer_t* l = &net->L[i];
  if (i == 0 && net->L[0].hin == 1 && net->L[0].hout > 1) return (int64_t)b * l->cout; /* G linear */
  if (l->hout == 1) return (int64_t)b * l->cout;                                        /* D linear */
  return (int64_t)b * l->cout * l->hout * l->hout;
}

static void cache_alloc(cache_t* c, const net_t* net, int b, int64_t in_elems) {
  memset(c, 0, sizeof(*c));
  c->b = b;
  c->in = (oreal*)malloc(sizeof(oreal) * (size_t)(in_elems > 0 ? in_elems : 1));
  for (int i = 0; i < net->nlayers; ++i) {
    const int64_t e = layer_out_elems(net, i, b);
    c->pre[i] = (oreal*)malloc(sizeof(oreal) * (size_t)e);
    c->act[i] = (oreal*)malloc(sizeof(oreal) * (size_t)e);
    c->mean[i] = (oreal*)calloc(4096, sizeof(oreal));
    c->var[i] = (oreal*)calloc(4096, sizeof(oreal));
  }
}
static void cache_free(cache_t* c, const net_t* net) {
  free(c->in);
  for (int i = 0; i < net->nlayers; ++i) { free(c->pre[i]); free(c->act[i]); free(c->mean[i]); free(c->var[i]); }
}

/* BN in training mode, or with given running statistics when run_mean != NULL and use_running. */
static void bn_layer(const oracle_ctx* c, const layer_t* l, const oreal* th, const oreal* x, oreal* y,
                     oreal* mean, oreal* var, int b, int C, int HW,
                     oreal* rm, oreal* rv, int update_running, int use_running) {
  if (use_running) {
    qv(c, (oreal*)x, (int64_t)b * C * HW);            /* emulation: the stored tensor is what gets normalised */
    oracle_bn_eval(x, th + l->gamma, th + l->beta, (oreal)c->cfg.bn_eps, rm + l->rs, rv + l->rs, y, b, C, HW);
    return;
  }
  oracle_bn_train(x, th + l->gamma, th + l->beta, (oreal)c->cfg.bn_eps, y, mean, var, b, C, HW);
  if (c->emul) {
    /* the statistics above come from the accumulators; what is stored, and normalised, is the rounded tensor */
    qv(c, (oreal*)x, (int64_t)b * C * HW);
    oracle_bn_eval(x, th + l->gamma, th + l->beta, (oreal)c->cfg.bn_eps, mean, var, y, b, C, HW);
  }
  if (update_running)
    oracle_bn_running_update(rm + l->rs, rv + l->rs, mean, var, (oreal)c->cfg.bn_momentum, C, (int64_t)b * HW);
}

/* G: [z ; onehot] -> linear -> BN -> ReLU -> {convT -> BN -> ReLU}* -> convT(+bias) -> tanh
   Emulation (c->emul): the input, the weights the contractions read, and every tensor a layer hands to the next
   are rounded to the 16-bit format; sums, statistics, biases and BatchNorm parameters are not. */
static void g_forward(const oracle_ctx* c, const oreal* th, cache_t* k, oreal* rm, oreal* rv,
                      int update_running, int use_running) {
  const net_t* G = &c->G;
  const int b = k->b;
  const layer_t* l = &G->L[0];
  const int C0 = c->cfg.g_ch[0], hw0 = c->cfg.g_h0 * c->cfg.g_h0;
  oreal* thq = shadow_weights(c, G, th, G->nlayers);
  const oreal* tw = thq ? thq : th;                                          /* where the contractions read weights */
  qv(c, k->in, (int64_t)b * l->cin);
  oracle_linear(k->in, tw + l->w, NULL, k->pre[0], b, l->cin, l->cout);      /* [b, C0*h0*h0] == [b,C0,h0,h0] */
  bn_layer(c, l, th, k->pre[0], k->act[0], k->mean[0], k->var[0], b, C0, hw0, rm, rv, update_running, use_running);
  oracle_leaky_relu(k->act[0], k->act[0], (int64_t)b * C0 * hw0, (oreal)0);
  qv(c, k->act[0], (int64_t)b * C0 * hw0);
  for (int i = 1; i < G->nlayers; ++i) {
    l = &G->L[i];
    const int64_t e = (int64_t)b * l->cout * l->hout * l->hout;
    oracle_conv_transpose2d(k->act[i - 1], tw + l->w, l->bias >= 0 ? th + l->bias : NULL, k->pre[i],
                            b, l->cin, l->hin, l->hin, l->cout, KSZ, STR, PAD);
    if (l->gamma >= 0) {
      bn_layer(c, l, th, k->pre[i], k->act[i], k->mean[i], k->var[i], b, l->cout, l->hout * l->hout, rm, rv,
               update_running, use_running);
      oracle_leaky_relu(k->act[i], k->act[i], e, (oreal)0);
    } else {
      oracle_tanh(k->pre[i], k->act[i], e);
    }
    qv(c, k->act[i], e);
  }
  free(thq);
}

/* Given dfake = d cost / d G(z), fill g (all of G's parameter gradients).
   Emulation: every activation gradient that is stored between two operations is rounded (after the tanh derivative,
   after each data gradient, after each BatchNorm backward); parameter gradients are not. */
static void g_backward(const oracle_ctx* c, const oreal* th, const cache_t* k, const oreal* dfake, oreal* g) {
  const net_t* G = &c->G;
  const int b = k->b;
  const int last = G->nlayers - 1;
  int64_t e = layer_out_elems(G, last, b);
  oreal* thq = shadow_weights(c, G, th, G->nlayers);
  const oreal* tw = thq ? thq : th;
  oreal* dcur = (oreal*)malloc(sizeof(oreal) * (size_t)e);
  oracle_tanh_bwd(k->act[last], dfake, dcur, e);                 /* gradient w.r.t. the last layer's pre-activation */
  qv(c, dcur, e);
  for (int i = last; i >= 1; --i) {
    const layer_t* l = &G->L[i];
    const int64_t ein = layer_out_elems(G, i - 1, b);
    oreal* dprev = (oreal*)malloc(sizeof(oreal) * (size_t)ein);
    oracle_conv_transpose2d_bwd(k->act[i - 1], tw + l->w, dcur, dprev, g + l->w, l->bias >= 0 ? g + l->bias : NULL,
                                b, l->cin, l->hin, l->hin, l->cout, KSZ, STR, PAD);
    free(dcur);
    qv(c, dprev, ein);
    /* dprev is w.r.t. act[i-1] = ReLU(BN(pre[i-1])) */
    const layer_t* lp = &G->L[i - 1];
    const int Cp = (i - 1 == 0) ? c->cfg.g_ch[0] : lp->cout;
    const int HWp = lp->hout * lp->hout;
    oreal* dbn = (oreal*)malloc(sizeof(oreal) * (size_t)ein);
    /* ReLU'(u) with u = BN output; act = ReLU(u) > 0 exactly when u > 0 */
    oracle_leaky_relu_bwd(k->act[i - 1], dprev, dbn, ein, (oreal)0);
    oracle_bn_bwd(k->pre[i - 1], th + lp->gamma, k->mean[i - 1], k->var[i - 1], (oreal)c->cfg.bn_eps, dbn, dprev,
                  g + lp->gamma, g + lp->beta, b, Cp, HWp);
    free(dbn);
    qv(c, dprev, ein);
    dcur = dprev;
  }
  const layer_t* l0 = &G->L[0];
  oracle_linear_bwd(k->in, tw + l0->w, dcur, NULL, g + l0->w, NULL, b, l0->cin, l0->cout);
  free(dcur);
  free(thq);
}

/* Emulation of the first convolution's label planes.  A one-hot label plane is constant over the image, so its part
   of the output at (oy, ox) is the sum of that channel's taps that fall inside the image; a 16-bit-storage
   implementation holds that sum (one per border class of the position) and the bias as stored values.  Adds
   round(sum of valid taps of the sample's label channel) + round(bias) to Y, whose convolution ran over the image
   channels only. */
static void add_label_planes_emul(const oracle_ctx* c, const layer_t* l, const oreal* th, const cache_t* k, oreal* Y) {
  const int C = c->cfg.img_c, cd = c->cfg.cond_d, H = l->hin, Ho = l->hout;
  const int HW = H * H;
  for (int r = 0; r < k->b; ++r) {
    int y = -1;                                        /* the label plane that is one for this sample */
    for (int j = 0; j < cd; ++j)
      if (k->in[((int64_t)r * (C + cd) + C + j) * HW] != (oreal)0) y = j;
    for (int co = 0; co < l->cout; ++co)
      for (int oy = 0; oy < Ho; ++oy)
        for (int ox = 0; ox < Ho; ++ox) {
          oreal sum = 0;
          if (y >= 0)
            for (int ky = 0; ky < KSZ; ++ky)
              for (int kx = 0; kx < KSZ; ++kx) {
                const int iy = oy * STR - PAD + ky, ix = ox * STR - PAD + kx;
                if (iy < 0 || iy >= H || ix < 0 || ix >= H) continue;
                sum += th[l->w + (((int64_t)co * l->cin + C + y) * KSZ + ky) * KSZ + kx];
              }
          Y[(((int64_t)r * l->cout + co) * Ho + oy) * Ho + ox] += oracle_round_bf16(sum) + oracle_round_bf16(th[l->bias + co]);
        }
  }
}

/* D: conv(+bias) -> LReLU -> {conv -> BN -> LReLU}* -> flatten -> linear(+bias); logits in act[last].
   Emulation: as in g_forward; the final linear layer reads the unrounded weights (it is not a 16-bit contraction). */
static void d_forward(const oracle_ctx* c, const oreal* th, cache_t* k, oreal* rm, oreal* rv, int update_running) {
  const net_t* D = &c->D;
  const int b = k->b;
  const oreal slope = (oreal)c->cfg.leaky_slope;
  const oreal* cur = k->in;
  oreal* thq = shadow_weights(c, D, th, D->nlayers - 1);
  const oreal* tw = thq ? thq : th;
  if (c->emul) {
    const layer_t* l0 = &D->L[0];
    qv(c, k->in, (int64_t)b * l0->cin * l0->hin * l0->hin);
    /* the label planes are handled by add_label_planes_emul: take their taps out of the convolution */
    for (int co = 0; co < l0->cout; ++co)
      for (int ci = c->cfg.img_c; ci < l0->cin; ++ci)
        for (int t = 0; t < KSZ * KSZ; ++t) thq[l0->w + ((int64_t)co * l0->cin + ci) * KSZ * KSZ + t] = 0;
  }
  for (int j = 0; j < D->nlayers - 1; ++j) {
    const layer_t* l = &D->L[j];
    const int64_t e = (int64_t)b * l->cout * l->hout * l->hout;
    if (c->emul && j == 0) {
      oracle_conv2d(cur, tw + l->w, NULL, k->pre[j], b, l->cin, l->hin, l->hin, l->cout, KSZ, STR, PAD);
      add_label_planes_emul(c, l, th, k, k->pre[j]);
    } else {
      oracle_conv2d(cur, tw + l->w, l->bias >= 0 ? th + l->bias : NULL, k->pre[j], b, l->cin, l->hin, l->hin, l->cout,
                    KSZ, STR, PAD);
    }
    if (l->gamma >= 0) {
      bn_layer(c, l, th, k->pre[j], k->act[j], k->mean[j], k->var[j], b, l->cout, l->hout * l->hout, rm, rv,
               update_running, 0);
      /* keep the BN output in pre-activation form for the backward pass of the LeakyReLU */
      oreal* u = (oreal*)malloc(sizeof(oreal) * (size_t)e);
      memcpy(u, k->act[j], sizeof(oreal) * (size_t)e);
      oracle_leaky_relu(u, k->act[j], e, slope);
      free(u);
    } else {
      oracle_leaky_relu(k->pre[j], k->act[j], e, slope);
    }
    qv(c, k->act[j], e);
    cur = k->act[j];
  }
  const int last = D->nlayers - 1;
  const layer_t* l = &D->L[last];
  oracle_linear(cur, th + l->w, th + l->bias, k->pre[last], b, l->cin, 1);
  memcpy(k->act[last], k->pre[last], sizeof(oreal) * (size_t)b);
  free(thq);
}

/* Accumulates (+=) parameter gradients into g; if dinput != NULL also returns d/d(network input).
   Emulation: a stored activation gradient is rounded once, after the last operation applied to it before it is
   stored: the gradient handed to a BatchNorm layer right after the data-gradient contraction, the gradient handed to
   the first convolution after its LeakyReLU derivative, the gradient of the network input not at all (the caller
   multiplies it by the tanh derivative first). */
static void d_backward(const oracle_ctx* c, const oreal* th, const cache_t* k, const oreal* ds, oreal* g,
                       oreal* dinput) {
  const net_t* D = &c->D;
  const int b = k->b;
  const oreal slope = (oreal)c->cfg.leaky_slope;
  const int last = D->nlayers - 1;
  oreal* thq = shadow_weights(c, D, th, D->nlayers - 1);
  const oreal* tw = thq ? thq : th;
  oreal* gl = (oreal*)calloc((size_t)D->nparams, sizeof(oreal));   /* this pass's gradients */
  const layer_t* l = &D->L[last];
  oreal* dcur = (oreal*)malloc(sizeof(oreal) * (size_t)((int64_t)b * l->cin));
  oracle_linear_bwd(k->act[last - 1], th + l->w, ds, dcur, gl + l->w, gl + l->bias, b, l->cin, 1);
  qv(c, dcur, (int64_t)b * l->cin);
  for (int j = last - 1; j >= 0; --j) {
    l = &D->L[j];
    const int64_t e = (int64_t)b * l->cout * l->hout * l->hout;
    oreal* dpre = (oreal*)malloc(sizeof(oreal) * (size_t)e);
    if (l->gamma >= 0) {
      /* LeakyReLU'(u): act > 0 exactly when u > 0 (slope > 0) */
      oreal* du = (oreal*)malloc(sizeof(oreal) * (size_t)e);
      oracle_leaky_relu_bwd(k->act[j], dcur, du, e, slope);
      oracle_bn_bwd(k->pre[j], th + l->gamma, k->mean[j], k->var[j], (oreal)c->cfg.bn_eps, du, dpre,
                    gl + l->gamma, gl + l->beta, b, l->cout, l->hout * l->hout);
      free(du);
    } else {
      oracle_leaky_relu_bwd(k->pre[j], dcur, dpre, e, slope);
    }
    qv(c, dpre, e);
    free(dcur);
    const oreal* xin = (j == 0) ? k->in : k->act[j - 1];
    const int64_t ein = (int64_t)b * l->cin * l->hin * l->hin;
    oreal* dprev = NULL;
    if (j > 0 || dinput) dprev = (j == 0) ? dinput : (oreal*)malloc(sizeof(oreal) * (size_t)ein);
    oracle_conv2d_bwd(xin, tw + l->w, dpre, dprev, gl + l->w, l->bias >= 0 ? gl + l->bias : NULL,
                      b, l->cin, l->hin, l->hin, l->cout, KSZ, STR, PAD);
    free(dpre);
    if (j >= 1 && D->L[j - 1].gamma >= 0) qv(c, dprev, ein);       /* consumed by a BatchNorm backward as stored */
    dcur = (j == 0) ? NULL : dprev;
  }
  for (int64_t i = 0; i < D->nparams; ++i) g[i] += gl[i];
  free(gl);
  free(thq);
}

/* Build the inputs of one model from the flat batch: rows idx[0..b). */
static void fill_g_input(const oracle_ctx* c, cache_t* k, const int32_t* idx, const int32_t* label_ids,
                         const oreal* noise) {
  const int zd = c->cfg.z_dim, cg = c->cfg.cond_g, w = zd + cg;
  for (int r = 0; r < k->b; ++r) {
    const int i = idx[r];
    for (int j = 0; j < zd; ++j) k->in[(int64_t)r * w + j] = noise[(int64_t)i * zd + j];
    for (int j = 0; j < cg; ++j) k->in[(int64_t)r * w + zd + j] = (j == label_ids[i]) ? (oreal)1 : (oreal)0;
  }
}
/* images: [b, img_c, H, H] already gathered for this model; labels of the same rows */
static void fill_d_input(const oracle_ctx* c, cache_t* k, const oreal* images, const int32_t* idx,
                         const int32_t* label_ids) {
  const int C = c->cfg.img_c, cd = c->cfg.cond_d, HW = c->cfg.img_hw * c->cfg.img_hw;
  for (int r = 0; r < k->b; ++r) {
    oreal* dst = k->in + (int64_t)r * (C + cd) * HW;
    memcpy(dst, images + (int64_t)r * C * HW, sizeof(oreal) * (size_t)C * HW);
    for (int j = 0; j < cd; ++j) {
      const oreal v = (j == label_ids[idx[r]]) ? (oreal)1 : (oreal)0;
      for (int p = 0; p < HW; ++p) dst[(int64_t)(C + j) * HW + p] = v;
    }
  }
}

typedef struct { oreal jd, jg; } losses_t;

/* One iteration for one model.  mode 0: full step (updates).  mode 1: losses only at the current parameters.
   mode 2: gradients only at the current parameters (gD_out, gG_out), no update. */
static losses_t model_iteration(oracle_ctx* c, int mdl, const int32_t* idx, int b, const int32_t* label_ids,
                                const oreal* noise, const oreal* real_batch, int mode, oreal* gD_out, oreal* gG_out) {
  const oracle_config* f = &c->cfg;
  const int C = f->img_c, HW = f->img_hw * f->img_hw;
  const int64_t PG = c->G.nparams, PD = c->D.nparams;
  oreal *thG = c->thG + mdl * PG, *thD = c->thD + mdl * PD;
  oreal *rmG = c->rmG + mdl * c->G.nbn, *rvG = c->rvG + mdl * c->G.nbn;
  oreal *rmD = c->rmD + mdl * c->D.nbn, *rvD = c->rvD + mdl * c->D.nbn;
  const int upd = (mode == 0);
  losses_t out;

  /* the minibatch of x for this label, and the minibatch of z */
  oreal* xr = (oreal*)malloc(sizeof(oreal) * (size_t)b * C * HW);
  for (int r = 0; r < b; ++r)
    memcpy(xr + (int64_t)r * C * HW, real_batch + (int64_t)idx[r] * C * HW, sizeof(oreal) * (size_t)C * HW);

  cache_t kg; cache_alloc(&kg, &c->G, b, (int64_t)b * (f->z_dim + f->cond_g));
  fill_g_input(c, &kg, idx, label_ids, noise);
  g_forward(c, thG, &kg, rmG, rvG, upd, 0);
  const oreal* fake = kg.act[c->G.nlayers - 1];

  /* discriminator cost, Eq. 3, on (real, fake as a constant) */
  cache_t kr, kf;
  const int64_t din = (int64_t)b * (C + f->cond_d) * HW;
  cache_alloc(&kr, &c->D, b, din); cache_alloc(&kf, &c->D, b, din);
  fill_d_input(c, &kr, xr, idx, label_ids);
  fill_d_input(c, &kf, fake, idx, label_ids);
  d_forward(c, thD, &kr, rmD, rvD, upd);
  d_forward(c, thD, &kf, rmD, rvD, upd);
  const int dl = c->D.nlayers - 1;
  oreal* dsr = (oreal*)malloc(sizeof(oreal) * (size_t)b);
  oreal* dsf = (oreal*)malloc(sizeof(oreal) * (size_t)b);
  out.jd = oracle_logistic_loss(kr.act[dl], b, -1, (oreal)f->d_loss_scale, dsr)
         + oracle_logistic_loss(kf.act[dl], b, +1, (oreal)f->d_loss_scale, dsf);
  if (mode != 1) {
    oreal* gD = (mode == 0) ? c->gD + mdl * PD : gD_out;
    memset(gD, 0, sizeof(oreal) * (size_t)PD);
    d_backward(c, thD, &kr, dsr, gD, NULL);
    d_backward(c, thD, &kf, dsf, gD, NULL);
    if (mode == 0) {
      c->tD[mdl] += 1;
      oracle_adam(thD, c->mD + mdl * PD, c->vD + mdl * PD, gD, PD, c->tD[mdl],
                  (oreal)f->lr, (oreal)f->beta1, (oreal)f->beta2, (oreal)f->adam_eps);
    }
  }
  cache_free(&kr, &c->D);

  /* generator cost, Eq. 4 (maximised => minimise its negative), through the (updated) discriminator,
     same fake batch, same z */
  d_forward(c, thD, &kf, rmD, rvD, upd);
  out.jg = oracle_logistic_loss(kf.act[dl], b, -1, (oreal)f->g_loss_scale, dsf);
  if (mode != 1) {
    oreal* scratch = (oreal*)calloc((size_t)PD, sizeof(oreal));   /* theta_D is not controlled by G: discarded */
    oreal* dxin = (oreal*)malloc(sizeof(oreal) * (size_t)din);
    d_backward(c, thD, &kf, dsf, scratch, dxin);
    free(scratch);
    oreal* dfake = (oreal*)malloc(sizeof(oreal) * (size_t)b * C * HW);
    for (int r = 0; r < b; ++r)
      memcpy(dfake + (int64_t)r * C * HW, dxin + (int64_t)r * (C + f->cond_d) * HW, sizeof(oreal) * (size_t)C * HW);
    free(dxin);
    oreal* gG = (mode == 0) ? c->gG + mdl * PG : gG_out;
    memset(gG, 0, sizeof(oreal) * (size_t)PG);
    g_backward(c, thG, &kg, dfake, gG);
    free(dfake);
    if (mode == 0) {
      c->tG[mdl] += 1;
      oracle_adam(thG, c->mG + mdl * PG, c->vG + mdl * PG, gG, PG, c->tG[mdl],
                  (oreal)f->lr, (oreal)f->beta1, (oreal)f->beta2, (oreal)f->adam_eps);
    }
  }
  cache_free(&kf, &c->D);
  cache_free(&kg, &c->G);
  free(dsr); free(dsf); free(xr);
  return out;
}

int oracle_train_step(oracle_ctx* c, const int32_t* label_ids, const oreal* noise,
                      const oreal* real_batch, int32_t n, int32_t only_model) {
  if (!c || n < 0 || (n > 0 && (!label_ids || !noise || !real_batch))) return -1;
  const int K = c->cfg.n_models;
  free(c->perm);
  c->perm = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
  oracle_route(label_ids, n, K, c->cfg.n_labels, c->perm, c->offs, &c->n_bad);
  c->last_n = n;
  for (int l = 0; l < K; ++l) {
    const int b = c->offs[l + 1] - c->offs[l];
    c->counts[l] = b;
    if (only_model >= 0 && l != only_model) continue;
    if (b == 0) { c->jd[l] = 0; c->jg[l] = 0; continue; }   /* a model with no samples is left untouched */
    const losses_t r = model_iteration(c, l, c->perm + c->offs[l], b, label_ids, noise, real_batch, 0, NULL, NULL);
    c->jd[l] = r.jd; c->jg[l] = r.jg;
  }
  return c->n_bad ? -5 : 0;
}

int oracle_eval_losses(oracle_ctx* c, int model, const int32_t* label_ids, const oreal* noise,
                       const oreal* real_batch, int32_t n, oreal* jd, oreal* jg) {
  int32_t* idx = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
  for (int i = 0; i < n; ++i) idx[i] = i;
  const losses_t r = model_iteration(c, model, idx, n, label_ids, noise, real_batch, 1, NULL, NULL);
  free(idx);
  *jd = r.jd; *jg = r.jg;
  return 0;
}

int oracle_eval_grads(oracle_ctx* c, int model, const int32_t* label_ids, const oreal* noise,
                      const oreal* real_batch, int32_t n, oreal* gD, oreal* gG) {
  int32_t* idx = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
  for (int i = 0; i < n; ++i) idx[i] = i;
  model_iteration(c, model, idx, n, label_ids, noise, real_batch, 2, gD, gG);
  free(idx);
  return 0;
}

int oracle_generate(oracle_ctx* c, const int32_t* label_ids, const oreal* noise, int32_t n,
                    oreal* out_images, int32_t use_running_stats, int32_t only_model) {
  if (!c || n < 0) return -1;
  const int K = c->cfg.n_models;
  const int C = c->cfg.img_c, HW = c->cfg.img_hw * c->cfg.img_hw;
  int32_t* perm = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
  int32_t* offs = (int32_t*)malloc(sizeof(int32_t) * (size_t)(K + 1));
  int32_t bad = 0;
  oracle_route(label_ids, n, K, c->cfg.n_labels, perm, offs, &bad);
  for (int l = 0; l < K; ++l) {
    const int b = offs[l + 1] - offs[l];
    if (b == 0 || (only_model >= 0 && l != only_model)) continue;
    cache_t kg; cache_alloc(&kg, &c->G, b, (int64_t)b * (c->cfg.z_dim + c->cfg.cond_g));
    fill_g_input(c, &kg, perm + offs[l], label_ids, noise);
    g_forward(c, c->thG + l * c->G.nparams, &kg, c->rmG + l * c->G.nbn, c->rvG + l * c->G.nbn, 0, use_running_stats);
    const oreal* fake = kg.act[c->G.nlayers - 1];
    for (int r = 0; r < b; ++r)
      memcpy(out_images + (int64_t)perm[offs[l] + r] * C * HW, fake + (int64_t)r * C * HW, sizeof(oreal) * (size_t)C * HW);
    cache_free(&kg, &c->G);
  }
  free(perm); free(offs);
  return bad ? -5 : 0;
}

/* Eq. 5: the model distribution is the prior-weighted mixture of the per-label generators. */
int oracle_draw_labels(const double* prior, int n_labels, const float* u, int n, int32_t* labels) {
  double total = 0.0;
  for (int k = 0; k < n_labels; ++k) {
    if (!(prior[k] >= 0.0)) return -1;
    total += prior[k];
  }
  if (!(total > 0.0)) return -1;
  for (int i = 0; i < n; ++i) {
    const double ui = (double)u[i];
    double cum = 0.0;
    int pick = -1;
    for (int k = 0; k < n_labels; ++k) {
      cum += prior[k] / total;
      if (pick < 0 && prior[k] > 0.0 && ui < cum) pick = k;
    }
    if (pick < 0)                       /* rounding left the last cumulative value below u: the last possible class */
      for (int k = n_labels - 1; k >= 0; --k)
        if (prior[k] > 0.0) { pick = k; break; }
    labels[i] = pick;
  }
  return 0;
}

int oracle_sample(oracle_ctx* c, const double* prior, const float* u, const oreal* noise, int32_t n,
                  oreal* out_images, int32_t* out_labels, int32_t use_running_stats) {
  if (!c || n < 0) return -1;
  if (oracle_draw_labels(prior, c->cfg.n_labels, u, n, out_labels) != 0) return -1;
  return oracle_generate(c, out_labels, noise, n, out_images, use_running_stats, -1);
}

int oracle_anova_f(const int32_t* label_ids, const float* images, int n, int n_labels, int C, int HW, double* F) {
  int rc = 0;
  double* x = (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
  double* gsum = (double*)malloc(sizeof(double) * (size_t)n_labels);
  int* gcnt = (int*)malloc(sizeof(int) * (size_t)n_labels);
  for (int c = 0; c < C; ++c) {
    for (int i = 0; i < n; ++i) {                  /* observation: mean intensity of channel c of image i */
      const float* p = images + ((int64_t)i * C + c) * HW;
      double s = 0.0;
      for (int q = 0; q < HW; ++q) s += (double)p[q];
      x[i] = s / (double)HW;
    }
    for (int k = 0; k < n_labels; ++k) { gsum[k] = 0.0; gcnt[k] = 0; }
    double all = 0.0;
    int nn = 0;
    for (int i = 0; i < n; ++i) {
      const int y = label_ids[i];
      if (y < 0 || y >= n_labels) continue;
      gsum[y] += x[i]; gcnt[y] += 1; all += x[i]; nn += 1;
    }
    int kk = 0;
    for (int k = 0; k < n_labels; ++k) kk += gcnt[k] > 0;
    if (kk < 2 || nn <= kk) { rc = -1; F[c] = 0.0; continue; }
    const double grand = all / (double)nn;
    double ssb = 0.0, ssw = 0.0;
    for (int k = 0; k < n_labels; ++k)
      if (gcnt[k] > 0) {
        const double mk = gsum[k] / (double)gcnt[k];
        ssb += (double)gcnt[k] * (mk - grand) * (mk - grand);
      }
    for (int i = 0; i < n; ++i) {
      const int y = label_ids[i];
      if (y < 0 || y >= n_labels) continue;
      const double mk = gsum[y] / (double)gcnt[y];
      ssw += (x[i] - mk) * (x[i] - mk);
    }
    F[c] = (ssb / (double)(kk - 1)) / (ssw / (double)(nn - kk));
  }
  free(x); free(gsum); free(gcnt);
  return rc;
}

int oracle_get_losses(const oracle_ctx* c, oreal* d_loss, oreal* g_loss, int32_t* counts) {
  for (int l = 0; l < c->cfg.n_models; ++l) {
    if (d_loss) d_loss[l] = c->jd[l];
    if (g_loss) g_loss[l] = c->jg[l];
    if (counts) counts[l] = c->counts[l];
  }
  return 0;
}

int oracle_get_routing(const oracle_ctx* c, int32_t* perm, int32_t* offs) {
  if (perm && c->perm) memcpy(perm, c->perm, sizeof(int32_t) * (size_t)c->last_n);
  if (offs) memcpy(offs, c->offs, sizeof(int32_t) * (size_t)(c->cfg.n_models + 1));
  return 0;
}
