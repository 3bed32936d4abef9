// Kernels of the training step for the networks exactly as the paper's Tables 1 and 2 print them (Section 4), next to
// what the k4 s2 p1 engine already provides:
//   D block: Conv k3 s2 p1 (+bias) -> LeakyReLU -> Dropout(0.25) [-> BatchNorm(eps 0.8)]  -- the convolution runs on
//            the engine as a k4 s2 p1 one whose fourth tap row and column are zero, channel counts padded to 64;
//            bias, activation and dropout are one pass over its output, BatchNorm takes its statistics from the
//            stored tensor (they cannot come from the GEMM: the activation and the dropout sit in between);
//   G input: Linear (+bias) -> ReLU -> BatchNorm(eps 1e-5)                                 -- same pass, no dropout;
//   G last : Conv k3 s1 p1 (+bias) -> tanh onto the image, and its two gradients (direct kernels: 1-4 output channels).
// All sums run in a fixed order (thread-strided partial sums, then ordered merges), so a model's result does not depend
// on what else is in the launch.
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace gan {

__device__ inline unsigned philox_word0(unsigned c0, unsigned c1, unsigned c2, unsigned c3, unsigned k0, unsigned k1) {
  // Philox-4x32-10 (Salmon et al., SC'11), first output word; same definition as in paper_layers.hip
  constexpr unsigned M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    if (r > 0) { k0 += W0; k1 += W1; }
    const unsigned hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
    const unsigned hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
    const unsigned n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
  }
  return c0;
}

// keep-mask of element (n inside its model, c, pixel) of a [n][C][H][W]-indexed tensor: see gan_op_dropout in gan.h
__device__ inline bool dropout_keep(const PointArgs& a, int l, int n_local, int c, int pix, int pass_id, unsigned step) {
  const unsigned long long lin = ((unsigned long long)n_local * a.C + c) * a.HW + pix;
  const unsigned w0 = philox_word0((unsigned)lin, (unsigned)(lin >> 32), (unsigned)(a.layer + 256 * pass_id), step, a.seed_lo,
                                   a.seed_hi ^ (unsigned)l);
  return (w0 >> 8) >= a.thr;
}

// forward: x <- dropout(act(x + bias))      (mode 0)
// backward: g <- g * keep * scale * act'(saved)   (mode 1; saved = the forward result: positive exactly where the
//           pre-activation was, zero where dropped -- and there the gradient is zero anyway)
template <typename T, int MODE>
__global__ __launch_bounds__(256) void point_kernel(PointArgs a) {
  const int j = blockIdx.x, sidx = blockIdx.y;
  if (j >= a.offs[a.L]) return;
  const int l = a.sample_model[j];
  const int seg = a.seg_first + sidx;
  const int n_local = j - a.offs[l];
  const unsigned step = a.steps ? (unsigned)(a.steps[l] + a.step_add) : 0u;
  const int pass_id = a.pass_of_seg[sidx];
  const long long base = ((long long)seg * a.seg_samples + j) * a.HW * a.Cpad;
  T* x = static_cast<T*>(a.x) + base;
  const T* saved = MODE == 1 ? static_cast<const T*>(a.saved) + base : nullptr;
  const float* bias = (MODE == 0 && a.bias) ? a.bias + (long long)l * a.pstride : nullptr;
  const int total = a.HW * a.C;
  for (int t = threadIdx.x; t < total; t += 256) {
    const int pix = t / a.C, c = t - pix * a.C;
    const long long o = (long long)pix * a.Cpad + c;
    float v = to_float(x[o]);
    if (MODE == 0) {
      if (bias) v += bias[c];
      v = v > 0.f ? v : v * a.slope;
    } else {
      if (!(to_float(saved[o]) > 0.f)) v *= a.slope;
    }
    if (a.thr > 0) v = dropout_keep(a, l, n_local, c, pix, pass_id, step) ? v * a.scale : 0.f;
    x[o] = from_float<T>(v);
  }
}
template <typename T> void launch_point_fwd(const PointArgs& a, hipStream_t st) {
  if (a.n == 0 || a.nseg == 0) return;
  hipLaunchKernelGGL((point_kernel<T, 0>), dim3((unsigned)a.n, (unsigned)a.nseg), dim3(256), 0, st, a);
}
template <typename T> void launch_point_bwd(const PointArgs& a, hipStream_t st) {
  if (a.n == 0 || a.nseg == 0) return;
  if (!a.saved) return launch_fail("activation backward: no saved forward tensor");
  hipLaunchKernelGGL((point_kernel<T, 1>), dim3((unsigned)a.n, (unsigned)a.nseg), dim3(256), 0, st, a);
}
template void launch_point_fwd<float>(const PointArgs&, hipStream_t);
template void launch_point_fwd<bf16_t>(const PointArgs&, hipStream_t);
template void launch_point_bwd<float>(const PointArgs&, hipStream_t);
template void launch_point_bwd<bf16_t>(const PointArgs&, hipStream_t);

// Rows of (segment, model): samples offs[l] .. offs[l+1] of segment seg, HW rows each, Cpad channels per row.
// Block = 16 channels x 16 row lanes; every lane adds its rows in order, then the lanes are added in order.
constexpr int PS_LANES = 16;
__device__ inline float lanes_sum(float v, float (*sh)[16], int cx, int rl) {
  sh[rl][cx] = v;
  __syncthreads();
  float s = 0.f;
  if (rl == 0)
    for (int k = 0; k < PS_LANES; ++k) s += sh[k][cx];
  __syncthreads();
  return s;       // valid in lane 0
}

// dbias[l][c] (+)= sum over the segments and rows of g (mode: the segments are added in order inside the block)
template <typename T>
__global__ __launch_bounds__(256) void col_sum_kernel(PointArgs a, float* __restrict__ out, long long out_stride) {
  __shared__ float sh[PS_LANES][16];
  const int cx = threadIdx.x & 15, rl = threadIdx.x >> 4;
  const int cblocks = (a.C + 15) / 16;
  const int c = (blockIdx.x % cblocks) * 16 + cx;
  const int l = blockIdx.x / cblocks;
  const int cnt = a.offs[l + 1] - a.offs[l];
  if (cnt == 0) return;
  const long long rows = (long long)cnt * a.HW;
  float tot = 0.f;
  for (int s = 0; s < a.nseg; ++s) {
    const T* g = static_cast<const T*>(a.x) + ((long long)(a.seg_first + s) * a.seg_samples + a.offs[l]) * a.HW * a.Cpad;
    float acc = 0.f;
    if (c < a.C)
      for (long long r = rl; r < rows; r += PS_LANES) acc += to_float(g[r * a.Cpad + c]);
    tot += lanes_sum(acc, sh, cx, rl);
  }
  if (rl == 0 && c < a.C) out[(long long)l * out_stride + c] = tot;
}
template <typename T> void launch_col_sum(const PointArgs& a, float* out, long long out_stride, hipStream_t st) {
  if (a.nseg == 0) return;
  hipLaunchKernelGGL((col_sum_kernel<T>), dim3((unsigned)(a.L * ((a.C + 15) / 16))), dim3(256), 0, st, a, out, out_stride);
}
template void launch_col_sum<float>(const PointArgs&, float*, long long, hipStream_t);
template void launch_col_sum<bf16_t>(const PointArgs&, float*, long long, hipStream_t);

// Batch statistics of a stored tensor per (segment, model, channel): mean, biased variance (from the deviations, second
// pass), 1 / sqrt(var + eps); written where the BatchNorm passes expect them ([(segment) * L + model][C]).
template <typename T>
__global__ __launch_bounds__(256) void bn_stats_direct_kernel(NormArgs a, int Cpad) {
  __shared__ float sh[PS_LANES][16];
  __shared__ float mean_sh[16];
  const int cx = threadIdx.x & 15, rl = threadIdx.x >> 4;
  const int cblocks = (a.C + 15) / 16;
  const int c = (blockIdx.x % cblocks) * 16 + cx;
  const int l = (blockIdx.x / cblocks) % a.L;
  const int sidx = blockIdx.x / (cblocks * a.L);
  const int cnt = a.offs[l + 1] - a.offs[l];
  if (cnt == 0) return;
  const long long rows = (long long)cnt * a.rps;
  const T* x = static_cast<const T*>(a.x) + ((long long)(a.seg_first + sidx) * a.seg_samples + a.offs[l]) * a.rps * Cpad;
  float acc = 0.f;
  if (c < a.C)
    for (long long r = rl; r < rows; r += PS_LANES) acc += to_float(x[r * Cpad + c]);
  const float s1 = lanes_sum(acc, sh, cx, rl);
  if (rl == 0) mean_sh[cx] = s1 / (float)rows;
  __syncthreads();
  const float mean = mean_sh[cx];
  acc = 0.f;
  if (c < a.C)
    for (long long r = rl; r < rows; r += PS_LANES) { const float d = to_float(x[r * Cpad + c]) - mean; acc += d * d; }
  const float s2 = lanes_sum(acc, sh, cx, rl);
  if (rl == 0 && c < a.C) {
    const float var = s2 / (float)rows;
    const long long o = (long long)((a.seg_first + sidx) * a.L + l) * a.C + c;
    a.mean[o] = mean;
    a.var[o] = var;
    a.rstd[o] = 1.0f / sqrtf(var + a.eps);
  }
}
template <typename T> void launch_bn_stats_direct(const NormArgs& a, int Cpad, hipStream_t st) {
  const long long tot = (long long)a.nseg * a.L * ((a.C + 15) / 16);
  if (tot == 0) return;
  hipLaunchKernelGGL((bn_stats_direct_kernel<T>), dim3((unsigned)tot), dim3(256), 0, st, a, Cpad);
}
template void launch_bn_stats_direct<float>(const NormArgs&, int, hipStream_t);
template void launch_bn_stats_direct<bf16_t>(const NormArgs&, int, hipStream_t);

// A k3 convolution held in the engine's k4 layout [16][Cb][Cs]: the fourth tap row and column are not parameters.
// Their gradient entries (the engine computes all 16) are cleared before Adam, so they stay exactly zero.
__global__ void clear_fourth_taps_kernel(float* __restrict__ dw, long long pstride, int L, int per_tap) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;      // (l, 7 taps, per_tap)
  if (idx >= (long long)L * 7 * per_tap) return;
  const int e = (int)(idx % per_tap);
  const int k = (int)((idx / per_tap) % 7);
  const int l = (int)(idx / ((long long)per_tap * 7));
  const int tap = k < 4 ? 12 + k : 3 + 4 * (k - 4);       // ky = 3 (taps 12..15), then kx = 3 for ky = 0, 1, 2
  dw[(long long)l * pstride + (long long)tap * per_tap + e] = 0.f;
}
void launch_clear_fourth_taps(float* dw, long long pstride, int L, int Cb, int Cs, hipStream_t st) {
  const long long tot = (long long)L * 7 * Cb * Cs;
  if (tot == 0) return;
  hipLaunchKernelGGL(clear_fourth_taps_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st, dw, pstride, L, Cb * Cs);
}

// ---- G's last layer: Conv k3 s1 p1 from Cin feature channels onto the 1-4 image channels --------------------------
// weights [9][CO][Cin] of model l at w + l * w_stride (fp32 master); feature / image tensors NHWC, rows model-major.
constexpr int C3_MAXCO = 4;
constexpr int C3_MAX_SPLITS = 32;

// G's last convolution of the tables: k3 s1 p1 from Cin (64 or 128) feature channels to CO <= 4 image channels, + bias,
// tanh.  Too few output channels for the MFMA engine; three direct kernels whose global accesses are whole channel
// rows (128 bytes and more per pixel) and whose reuse goes through LDS:
//   forward : block = (sample, tile of R full image rows).  The (R+2) x (H+2) halo tile of the input sits in LDS in the
//             storage type, pixels (Cin * sizeof(T) + 4) bytes apart (an odd number of words: the threads of a wave,
//             one output pixel each, read different banks); the weights sit there as [tap][ci][4] floats, read by all
//             threads at once.
//   dgrad   : block = (sample, tile of R rows); the halo tile of dout (4 floats per pixel) in LDS; thread = (input
//             channel, pixel lane), its 9 x CO weights in registers, whole channel rows written.
//   wgrad   : block = (row split, model), loops over the split's samples: dout with halo in LDS, thread = (input
//             channel, pixel lane) with 9 x CO accumulators, one 128-byte row of the input per wave and pixel; the
//             pixel lanes, then the splits, are added in a fixed order.
template <typename T> __device__ inline int c3_pixel_stride(int Cin) { return Cin * (int)sizeof(T) + 4; }

template <typename T>
__global__ __launch_bounds__(256) void conv3_fwd_kernel(Conv3Args a, int R) {
  extern __shared__ __attribute__((aligned(16))) unsigned char c3_lds[];
  const int j = blockIdx.y;
  if (j >= a.offs[a.L]) return;
  const int l = a.sample_model[j];
  const int H = a.H, Cin = a.Cin, CO = a.CO;
  const int y0 = blockIdx.x * R;
  float4* wsh = reinterpret_cast<float4*>(c3_lds);                         // [9][Cin] x (co 0..3)
  unsigned char* tile = c3_lds + (size_t)9 * Cin * sizeof(float4);          // [(R+2)][(H+2)] pixels
  const int PS = c3_pixel_stride<T>(Cin);
  const float* w = a.w + (long long)l * a.w_stride;
  for (int t = threadIdx.x; t < 9 * Cin; t += blockDim.x) {
    const int tap = t / Cin, ci = t - tap * Cin;
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    for (int co = 0; co < CO; ++co) v[co] = w[((long long)tap * CO + co) * Cin + ci];
    wsh[t] = make_float4(v[0], v[1], v[2], v[3]);
  }
  // halo tile: 4-byte words of the rows y0-1 .. y0+R, columns -1 .. H (zeros outside the image)
  const T* in = static_cast<const T*>(a.in) + (long long)j * H * H * Cin;
  const int wpp = Cin * (int)sizeof(T) / 4;                                // words per pixel
  const int words = (R + 2) * (H + 2) * wpp;
  for (int t = threadIdx.x; t < words; t += blockDim.x) {
    const int pix = t / wpp, wd = t - pix * wpp;
    const int r = pix / (H + 2), xx = pix - r * (H + 2);
    const int y = y0 - 1 + r, x = xx - 1;
    unsigned val = 0;
    if ((unsigned)y < (unsigned)H && (unsigned)x < (unsigned)H)
      val = reinterpret_cast<const unsigned*>(in + ((long long)y * H + x) * Cin)[wd];
    *reinterpret_cast<unsigned*>(tile + (size_t)pix * PS + wd * 4) = val;
  }
  __syncthreads();
  const int p = threadIdx.x;
  const int ry = p / H, x = p - ry * H;
  const int y = y0 + ry;
  if (ry >= R || y >= H) return;
  float acc[4];
#pragma unroll
  for (int co = 0; co < 4; ++co) acc[co] = co < CO ? a.bias[(long long)l * a.bias_stride + co] : 0.f;
#pragma unroll
  for (int ky = 0; ky < 3; ++ky)
#pragma unroll
    for (int kx = 0; kx < 3; ++kx) {
      const unsigned char* px = tile + (size_t)((ry + ky) * (H + 2) + (x + kx)) * PS;
      const float4* wt = wsh + (ky * 3 + kx) * Cin;
      if (sizeof(T) == 2) {
        for (int c2 = 0; c2 < Cin / 2; ++c2) {
          const unsigned pr = *reinterpret_cast<const unsigned*>(px + c2 * 4);
          const float v0 = __uint_as_float(pr << 16), v1 = __uint_as_float(pr & 0xffff0000u);
          const float4 w0 = wt[2 * c2], w1 = wt[2 * c2 + 1];
          acc[0] += v0 * w0.x; acc[1] += v0 * w0.y; acc[2] += v0 * w0.z; acc[3] += v0 * w0.w;
          acc[0] += v1 * w1.x; acc[1] += v1 * w1.y; acc[2] += v1 * w1.z; acc[3] += v1 * w1.w;
        }
      } else {
        for (int ci = 0; ci < Cin; ++ci) {
          const float v = *reinterpret_cast<const float*>(px + ci * 4);
          const float4 w0 = wt[ci];
          acc[0] += v * w0.x; acc[1] += v * w0.y; acc[2] += v * w0.z; acc[3] += v * w0.w;
        }
      }
    }
  T* out = static_cast<T*>(a.out) + ((long long)a.out_seg * a.seg_samples + j) * H * H * CO + ((long long)y * H + x) * CO;
#pragma unroll
  for (int co = 0; co < 4; ++co)
    if (co < CO) out[co] = from_float<T>(tanhf(acc[co]));
}

// din[n][y][x][ci] = sum_{ky,kx,co} dout[n][y-ky+1][x-kx+1][co] * w[ky][kx][co][ci]
template <typename T>
__global__ __launch_bounds__(256) void conv3_dgrad_kernel(Conv3Args a, int R) {
  extern __shared__ __attribute__((aligned(16))) unsigned char c3_lds[];
  const int j = blockIdx.y;
  if (j >= a.offs[a.L]) return;
  const int l = a.sample_model[j];
  const int H = a.H, Cin = a.Cin, CO = a.CO;
  const int y0 = blockIdx.x * R;
  float4* dsh = reinterpret_cast<float4*>(c3_lds);                         // [(R+2)][(H+2)] x (co 0..3)
  const T* dout = static_cast<const T*>(a.dout) + ((long long)a.out_seg * a.seg_samples + j) * H * H * CO;
  for (int t = threadIdx.x; t < (R + 2) * (H + 2); t += blockDim.x) {
    const int r = t / (H + 2), xx = t - r * (H + 2);
    const int y = y0 - 1 + r, x = xx - 1;
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    if ((unsigned)y < (unsigned)H && (unsigned)x < (unsigned)H)
      for (int co = 0; co < CO; ++co) v[co] = to_float(dout[((long long)y * H + x) * CO + co]);
    dsh[t] = make_float4(v[0], v[1], v[2], v[3]);
  }
  const int ci = threadIdx.x % Cin, pl = threadIdx.x / Cin, lanes = blockDim.x / Cin;
  const float* w = a.w + (long long)l * a.w_stride;
  float wr[9][4];
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int co = 0; co < 4; ++co) wr[t][co] = co < CO ? w[((long long)t * CO + co) * Cin + ci] : 0.f;
  __syncthreads();
  T* din = static_cast<T*>(a.din) + (long long)j * H * H * Cin;
  const int rows = min(R, H - y0);
  for (int p = pl; p < rows * H; p += lanes) {
    const int ry = p / H, x = p - ry * H;
    float acc = 0.f;
#pragma unroll
    for (int ky = 0; ky < 3; ++ky)
#pragma unroll
      for (int kx = 0; kx < 3; ++kx) {
        // output pixel (y - ky + 1, x - kx + 1) sits at halo position (ry - ky + 2, x - kx + 2)
        const float4 d = dsh[(ry - ky + 2) * (H + 2) + (x - kx + 2)];
        acc += d.x * wr[ky * 3 + kx][0] + d.y * wr[ky * 3 + kx][1] + d.z * wr[ky * 3 + kx][2] + d.w * wr[ky * 3 + kx][3];
      }
    din[((long long)(y0 + ry) * H + x) * Cin + ci] = from_float<T>(acc);
  }
}

// dw[ky][kx][co][ci] = sum_{n,y,x} dout[n][y][x][co] * in[n][y+ky-1][x+kx-1][ci]
template <typename T>
__global__ __launch_bounds__(256) void conv3_wgrad_kernel(Conv3Args a, float* __restrict__ part, int splits) {
  extern __shared__ __attribute__((aligned(16))) unsigned char c3_lds[];
  const int l = blockIdx.y, split = blockIdx.x;
  const int s0 = a.offs[l], cnt = a.offs[l + 1] - s0;
  if (cnt == 0) return;
  const int H = a.H, Cin = a.Cin, CO = a.CO;
  constexpr int R = 8;                                                   // input rows per tile
  float4* dsh = reinterpret_cast<float4*>(c3_lds);                         // [(R+2)][(H+2)] x (co 0..3), zeros outside the image
  float* red = reinterpret_cast<float*>(c3_lds + (size_t)(R + 2) * (H + 2) * sizeof(float4));   // [lanes][9*CO][Cin]
  const int ci = threadIdx.x % Cin, pl = threadIdx.x / Cin, lanes = blockDim.x / Cin;
  const int per = (cnt + splits - 1) / splits;
  const int n_lo = split * per, n_hi = min(cnt, n_lo + per);
  float acc[9][4];
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int co = 0; co < 4; ++co) acc[t][co] = 0.f;
  for (int n = n_lo; n < n_hi; ++n) {
    const T* in = static_cast<const T*>(a.in) + (long long)(s0 + n) * H * H * Cin;
    const T* dout = static_cast<const T*>(a.dout) + ((long long)a.out_seg * a.seg_samples + s0 + n) * H * H * CO;
    for (int y0 = 0; y0 < H; y0 += R) {                                   // input rows y0 .. y0+R-1 need dout rows y0-1 .. y0+R
      __syncthreads();                                                    // the previous tile has been read
      for (int t = threadIdx.x; t < (R + 2) * (H + 2); t += blockDim.x) {
        const int r = t / (H + 2), xx = t - r * (H + 2);
        const int y = y0 - 1 + r, x = xx - 1;
        float v[4] = {0.f, 0.f, 0.f, 0.f};
        if ((unsigned)y < (unsigned)H && (unsigned)x < (unsigned)H)
          for (int co = 0; co < CO; ++co) v[co] = to_float(dout[((long long)y * H + x) * CO + co]);
        dsh[t] = make_float4(v[0], v[1], v[2], v[3]);
      }
      __syncthreads();
      const int rows = min(R, H - y0);
      for (int p = pl; p < rows * H; p += lanes) {                         // pixel of the INPUT inside the tile
        const int ry = p / H, ix = p - ry * H;
        const float v = to_float(in[((long long)(y0 + ry) * H + ix) * Cin + ci]);
#pragma unroll
        for (int ky = 0; ky < 3; ++ky)
#pragma unroll
          for (int kx = 0; kx < 3; ++kx) {
            // output pixel (iy - ky + 1, ix - kx + 1) at halo position (ry - ky + 2, ix - kx + 2)
            const float4 d = dsh[(ry - ky + 2) * (H + 2) + (ix - kx + 2)];
            acc[ky * 3 + kx][0] += v * d.x; acc[ky * 3 + kx][1] += v * d.y;
            acc[ky * 3 + kx][2] += v * d.z; acc[ky * 3 + kx][3] += v * d.w;
          }
      }
    }
  }
  // pixel lanes added in order through LDS
  for (int t = 0; t < 9; ++t)
    for (int co = 0; co < CO; ++co) red[((size_t)pl * 9 * CO + t * CO + co) * Cin + ci] = acc[t][co];
  __syncthreads();
  for (int e = threadIdx.x; e < 9 * CO * Cin; e += blockDim.x) {
    float s = 0.f;
    for (int k = 0; k < lanes; ++k) s += red[(size_t)k * 9 * CO * Cin + e];
    part[((long long)split * a.L + l) * 9 * CO * Cin + e] = s;
  }
}
__global__ void conv3_wgrad_final_kernel(Conv3Args a, const float* __restrict__ part, float* __restrict__ dw, long long dw_stride,
                                         int splits) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const int per = 9 * a.CO * a.Cin;
  if (idx >= (long long)a.L * per) return;
  const int l = (int)(idx / per), e = (int)(idx - (long long)l * per);
  if (a.offs[l + 1] == a.offs[l]) return;
  float s = 0.f;
  for (int k = 0; k < splits; ++k) s += part[((long long)k * a.L + l) * per + e];
  dw[(long long)l * dw_stride + e] = s;
}
// row splits per model of the weight gradient: enough blocks to fill the chip, a function of the model count only
int conv3_wgrad_splits(int L) { return min(max((1024 + L - 1) / L, 1), C3_MAX_SPLITS); }

static bool conv3_ok(const Conv3Args& a) {
  return a.CO >= 1 && a.CO <= C3_MAXCO && (a.Cin == 64 || a.Cin == 128) && a.H >= 1 && a.H <= 64 && a.w && a.offs && a.sample_model;
}
// rows of the image per forward block: at most 256 pixels, and a halo tile that fits `budget` bytes of LDS (0: none does)
static int conv3_tile_rows(int H, int pixel_bytes, long long budget) {
  int R = H < 256 / H ? H : 256 / H;
  if (R < 1) R = 1;
  while (R > 1 && (long long)(R + 2) * (H + 2) * pixel_bytes > budget) --R;
  return (long long)(R + 2) * (H + 2) * pixel_bytes <= budget ? R : 0;
}
template <typename T> void launch_conv3_fwd(const Conv3Args& a, hipStream_t st) {
  if (a.n == 0) return;
  if (!conv3_ok(a) || !a.in || !a.out || !a.bias) return launch_fail("image-side k3 convolution: unsupported shape or null operand");
  const int ps = a.Cin * (int)sizeof(T) + 4;
  const int R = conv3_tile_rows(a.H, ps, 60 * 1024 - 9 * a.Cin * 16);     // 60 KiB of LDS per block with the weights
  if (R == 0) return launch_fail("image-side k3 convolution: one image row with its halo does not fit the LDS budget");
  const size_t lds = (size_t)9 * a.Cin * 16 + (size_t)(R + 2) * (a.H + 2) * ps;
  const int threads = (R * a.H + 63) / 64 * 64;
  hipLaunchKernelGGL((conv3_fwd_kernel<T>), dim3((a.H + R - 1) / R, a.n), dim3(threads), lds, st, a, R);
}
template <typename T> void launch_conv3_dgrad(const Conv3Args& a, hipStream_t st) {
  if (a.n == 0) return;
  if (!conv3_ok(a) || !a.dout || !a.din) return launch_fail("image-side k3 convolution: unsupported shape or null operand");
  const int R = a.H < 8 ? a.H : 8;
  hipLaunchKernelGGL((conv3_dgrad_kernel<T>), dim3((a.H + R - 1) / R, a.n), dim3(256), (size_t)(R + 2) * (a.H + 2) * 16, st, a, R);
}
template <typename T> void launch_conv3_wgrad(const Conv3Args& a, float* part, float* dw, long long dw_stride, hipStream_t st) {
  if (a.n == 0) return;
  if (!conv3_ok(a) || !a.dout || !a.in || !part || !dw) return launch_fail("image-side k3 convolution: unsupported shape or null operand");
  const int splits = conv3_wgrad_splits(a.L);
  const size_t lds = (size_t)(8 + 2) * (a.H + 2) * 16 + (size_t)(256 / a.Cin) * 9 * a.CO * a.Cin * sizeof(float);
  hipLaunchKernelGGL((conv3_wgrad_kernel<T>), dim3(splits, a.L), dim3(256), lds, st, a, part, splits);
  const long long tot = (long long)a.L * 9 * a.CO * a.Cin;
  hipLaunchKernelGGL(conv3_wgrad_final_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st, a, part, dw, dw_stride, splits);
}
template void launch_conv3_fwd<float>(const Conv3Args&, hipStream_t);
template void launch_conv3_fwd<bf16_t>(const Conv3Args&, hipStream_t);
template void launch_conv3_dgrad<float>(const Conv3Args&, hipStream_t);
template void launch_conv3_dgrad<bf16_t>(const Conv3Args&, hipStream_t);
template void launch_conv3_wgrad<float>(const Conv3Args&, float*, float*, long long, hipStream_t);
template void launch_conv3_wgrad<bf16_t>(const Conv3Args&, float*, float*, long long, hipStream_t);

}  // namespace gan
