// Kernels of the training step for the networks exactly as the paper's Tables 1 and 2 print them (Section 4), next to
// what the k4 s2 p1 engine already provides:
//   D block: Conv k3 s2 p1 (+bias) -> LeakyReLU -> Dropout(0.25) [-> BatchNorm(eps 0.8)]  -- the convolution runs on
//            the engine as a k4 s2 p1 one whose fourth tap row and column are zero, channel counts padded to 64;
//            bias, activation and dropout are one pass over its output, BatchNorm takes its statistics from the
//            stored tensor (they cannot come from the GEMM: the activation and the dropout sit in between);
//   G input: Linear (+bias) -> ReLU -> BatchNorm(eps 1e-5)                                 -- same pass, no dropout;
//   G last : Conv k3 s1 p1 (+bias) -> tanh onto the image, and its two gradients: conv3_mfma.hip.
// All sums run in a fixed order (thread-strided partial sums, then ordered merges), so a model's result does not depend
// on what else is in the launch.
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace gan {

__device__ inline void philox4(unsigned c0, unsigned c1, unsigned c2, unsigned c3, unsigned k0, unsigned k1, unsigned (&out)[4]) {
  // Philox-4x32-10 (Salmon et al., SC'11), all four output words; same definition as in paper_layers.hip
  constexpr unsigned M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    if (r > 0) { k0 += W0; k1 += W1; }
    const unsigned long long p0 = (unsigned long long)M0 * c0, p1 = (unsigned long long)M1 * c2;     // one wide multiply each
    const unsigned hi0 = (unsigned)(p0 >> 32), lo0 = (unsigned)p0, hi1 = (unsigned)(p1 >> 32), lo1 = (unsigned)p1;
    const unsigned n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// the four output words that hold the keep-decisions of elements lin .. lin + 3 (lin a multiple of 4) of a
// [n][C][H][W]-indexed tensor, or the one of element lin (any lin): see gan_op_dropout in gan.h
__device__ inline void dropout_words(const PointArgs& a, int l, unsigned long long lin, int pass_id, unsigned step, unsigned (&w)[4]) {
  philox4((unsigned)(lin >> 2), (unsigned)(lin >> 34), (unsigned)(a.layer + 256 * pass_id), step, a.seed_lo, a.seed_hi ^ (unsigned)l, w);
}

// forward: x <- dropout(act(x + bias))      (mode 0)
// backward: g <- g * keep * scale * act'(saved)   (mode 1; saved = the forward result: positive exactly where the
//           pre-activation was, zero where dropped -- and there the gradient is zero anyway)
template <typename T, int MODE>
__device__ inline float point_value(const PointArgs& a, float v, const T* saved, const float* bias, int o, int c) {
  if (MODE == 0) {
    if (bias) v += bias[c];
    v = v > 0.f ? v : v * a.slope;
  } else {
    if (!(to_float(saved[o]) > 0.f)) v *= a.slope;
  }
  return v;
}
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
  // (pixel, channel) carried along instead of divided out: the kernel is bound by its vector instructions
  const int dp = 256 / a.C, dc = 256 - dp * a.C;
  int pix = (int)threadIdx.x / a.C, c = (int)threadIdx.x - pix * a.C;
  if (a.thr > 0 && (a.HW & 3) == 0) {
    // a thread takes four consecutive pixels of one channel: consecutive element indices, one generator evaluation
    const int total = (a.HW >> 2) * a.C;
    for (int t = threadIdx.x; t < total; t += 256, pix += dp, c += dc) {
      if (c >= a.C) { c -= a.C; ++pix; }              // pix counts groups of four pixels here
      unsigned w[4];
      dropout_words(a, l, ((unsigned long long)n_local * a.C + c) * a.HW + pix * 4, pass_id, step, w);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int o = (pix * 4 + k) * a.Cpad + c;
        const float v = point_value<T, MODE>(a, to_float(x[o]), saved, bias, o, c);
        x[o] = from_float<T>((w[k] >> 8) >= a.thr ? v * a.scale : 0.f);
      }
    }
    return;
  }
  const int total = a.HW * a.C;
  for (int t = threadIdx.x; t < total; t += 256, pix += dp, c += dc) {
    if (c >= a.C) { c -= a.C; ++pix; }
    const int o = pix * a.Cpad + c;
    float v = point_value<T, MODE>(a, to_float(x[o]), saved, bias, o, c);
    if (a.thr > 0) {
      const unsigned long long lin = ((unsigned long long)n_local * a.C + c) * a.HW + pix;
      unsigned w[4];
      dropout_words(a, l, lin, pass_id, step, w);
      const unsigned sel = (unsigned)lin & 3u;
      const unsigned wd = sel == 0 ? w[0] : (sel == 1 ? w[1] : (sel == 2 ? w[2] : w[3]));
      v = (wd >> 8) >= a.thr ? v * a.scale : 0.f;
    }
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
// Block = CB_ channels of one (segment,) model: CB_ / EPV channel lanes of 16 bytes x 256 / lanes row lanes; every row
// lane adds its rows (rl, rl + RL, ...) in order, then the lanes are added in order -- whole 16-byte loads of 64 or
// 128 contiguous bytes per row instead of one element per thread.
constexpr int PS_CH = 32;                     // channels per block
template <typename T> struct PsVec { static constexpr int N = 16 / (int)sizeof(T); };
template <typename T> __device__ inline void ps_load(const T* p, float (&v)[PsVec<T>::N]) {
  const uint4 t = *reinterpret_cast<const uint4*>(p);
  if constexpr (sizeof(T) == 2) {
    v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xffff0000u);
    v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xffff0000u);
    v[4] = __uint_as_float(t.z << 16); v[5] = __uint_as_float(t.z & 0xffff0000u);
    v[6] = __uint_as_float(t.w << 16); v[7] = __uint_as_float(t.w & 0xffff0000u);
  } else {
    v[0] = __uint_as_float(t.x); v[1] = __uint_as_float(t.y); v[2] = __uint_as_float(t.z); v[3] = __uint_as_float(t.w);
  }
}
// sum over the row lanes, in lane order, of every lane's EPV values; result for channel cx (< PS_CH) in the threads
// with threadIdx.x < PS_CH
template <int EPV>
__device__ inline float ps_lanes_sum(const float (&v)[EPV], float* sh, int cl, int rl, int RL) {
  __syncthreads();                                   // the buffer's previous use is over
#pragma unroll
  for (int e = 0; e < EPV; ++e) sh[rl * PS_CH + cl * EPV + e] = v[e];
  __syncthreads();
  float s = 0.f;
  if ((int)threadIdx.x < PS_CH)
    for (int k = 0; k < RL; ++k) s += sh[k * PS_CH + threadIdx.x];
  return s;
}

// dbias[l][c] = sum over the segments and rows of g (the segments are added in order inside the block)
template <typename T>
__global__ __launch_bounds__(256) void col_sum_kernel(PointArgs a, float* __restrict__ out, long long out_stride) {
  constexpr int EPV = PsVec<T>::N, CG = PS_CH / EPV, RL = 256 / CG;
  __shared__ float sh[RL * PS_CH];
  const int cl = threadIdx.x % CG, rl = threadIdx.x / CG;
  const int cblocks = (a.Cpad + PS_CH - 1) / PS_CH;
  const int c0 = (blockIdx.x % cblocks) * PS_CH;
  const int l = blockIdx.x / cblocks;
  const int cnt = a.offs[l + 1] - a.offs[l];
  if (cnt == 0) return;
  const long long rows = (long long)cnt * a.HW;
  const bool live = c0 + cl * EPV < a.Cpad;          // Cpad is a multiple of 8: a 16-byte group is inside or outside
  float tot = 0.f;
  for (int s = 0; s < a.nseg; ++s) {
    const T* g = static_cast<const T*>(a.x) + ((long long)(a.seg_first + s) * a.seg_samples + a.offs[l]) * a.HW * a.Cpad + c0 + cl * EPV;
    float acc[EPV];
#pragma unroll
    for (int e = 0; e < EPV; ++e) acc[e] = 0.f;
    if (live)
      for (long long r = rl; r < rows; r += RL) {
        float v[EPV];
        ps_load<T>(g + r * a.Cpad, v);
#pragma unroll
        for (int e = 0; e < EPV; ++e) acc[e] += v[e];
      }
    tot += ps_lanes_sum<EPV>(acc, sh, cl, rl, RL);
  }
  const int c = c0 + (int)threadIdx.x;
  if ((int)threadIdx.x < PS_CH && c < a.C) out[(long long)l * out_stride + c] = tot;
}
template <typename T> void launch_col_sum(const PointArgs& a, float* out, long long out_stride, hipStream_t st) {
  if (a.nseg == 0) return;
  if (a.Cpad % 8 != 0) return launch_fail("column sums: the channel count of a row must be a multiple of 8");
  hipLaunchKernelGGL((col_sum_kernel<T>), dim3((unsigned)(a.L * ((a.Cpad + PS_CH - 1) / PS_CH))), dim3(256), 0, st, a, out, out_stride);
}
template void launch_col_sum<float>(const PointArgs&, float*, long long, hipStream_t);
template void launch_col_sum<bf16_t>(const PointArgs&, float*, long long, hipStream_t);

// Batch statistics of a stored tensor per (segment, model, channel): mean, biased variance (from the deviations, second
// pass), 1 / sqrt(var + eps); written where the BatchNorm passes expect them ([(segment) * L + model][C]).
template <typename T>
__global__ __launch_bounds__(256) void bn_stats_direct_kernel(NormArgs a, int Cpad) {
  constexpr int EPV = PsVec<T>::N, CG = PS_CH / EPV, RL = 256 / CG;
  __shared__ float sh[RL * PS_CH];
  __shared__ float mean_sh[PS_CH];
  const int cl = threadIdx.x % CG, rl = threadIdx.x / CG;
  const int cblocks = (Cpad + PS_CH - 1) / PS_CH;
  const int c0 = (blockIdx.x % cblocks) * PS_CH;
  const int l = (blockIdx.x / cblocks) % a.L;
  const int sidx = blockIdx.x / (cblocks * a.L);
  const int cnt = a.offs[l + 1] - a.offs[l];
  if (cnt == 0) return;
  const long long rows = (long long)cnt * a.rps;
  const bool live = c0 + cl * EPV < Cpad;
  const T* x = static_cast<const T*>(a.x) + ((long long)(a.seg_first + sidx) * a.seg_samples + a.offs[l]) * a.rps * Cpad + c0 + cl * EPV;
  float acc[EPV];
#pragma unroll
  for (int e = 0; e < EPV; ++e) acc[e] = 0.f;
  if (live)
    for (long long r = rl; r < rows; r += RL) {
      float v[EPV];
      ps_load<T>(x + r * Cpad, v);
#pragma unroll
      for (int e = 0; e < EPV; ++e) acc[e] += v[e];
    }
  const float s1 = ps_lanes_sum<EPV>(acc, sh, cl, rl, RL);
  if ((int)threadIdx.x < PS_CH) mean_sh[threadIdx.x] = s1 / (float)rows;
  __syncthreads();
  float mean[EPV];
#pragma unroll
  for (int e = 0; e < EPV; ++e) { mean[e] = mean_sh[cl * EPV + e]; acc[e] = 0.f; }
  if (live)
    for (long long r = rl; r < rows; r += RL) {
      float v[EPV];
      ps_load<T>(x + r * Cpad, v);
#pragma unroll
      for (int e = 0; e < EPV; ++e) { const float d = v[e] - mean[e]; acc[e] += d * d; }
    }
  const float s2 = ps_lanes_sum<EPV>(acc, sh, cl, rl, RL);
  const int c = c0 + (int)threadIdx.x;
  if ((int)threadIdx.x < PS_CH && c < a.C) {
    const float var = s2 / (float)rows;
    const long long o = (long long)((a.seg_first + sidx) * a.L + l) * a.C + c;
    a.mean[o] = mean_sh[threadIdx.x];
    a.var[o] = var;
    a.rstd[o] = 1.0f / sqrtf(var + a.eps);
  }
}
template <typename T> void launch_bn_stats_direct(const NormArgs& a, int Cpad, hipStream_t st) {
  const long long tot = (long long)a.nseg * a.L * ((Cpad + PS_CH - 1) / PS_CH);
  if (tot == 0) return;
  if (Cpad % 8 != 0) return launch_fail("batch statistics: the channel count of a row must be a multiple of 8");
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

}  // namespace gan
