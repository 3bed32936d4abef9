// Pieces of the networks exactly as the paper's Tables 1 and 2 print them that the k4 s2 p1 engine does not have:
// the dropout mask (a counter-based generator, so that any other implementation can reproduce it bit for bit) and the
// two small linear maps that let "Upsample x2, then Conv k3 s1 p1" run as a k4 s2 p1 transposed convolution.
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace gan {

// Philox-4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, "Parallel random numbers: as easy as 1, 2, 3", SC'11), from
// its definition: a round maps (c0, c1, c2, c3) to (hi(M1 c2) ^ c1 ^ k0, lo(M1 c2), hi(M0 c0) ^ c3 ^ k1, lo(M0 c0));
// the key is advanced by the two Weyl constants between rounds.  All four output words.
__device__ inline void philox4x32_10(unsigned c0, unsigned c1, unsigned c2, unsigned c3, unsigned k0, unsigned k1, unsigned (&out)[4]) {
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

// x[j][y][x][c] (rows grouped by model: group g holds samples offs[g] .. offs[g+1]) <- x * keep / (1 - p), where
// keep(element) = (word[index % 4] >> 8) >= thr with thr = ceil(p 2^24), counter = (index / 4 low, high, layer + 256
// pass, step), key = (seed low, seed high ^ group), index = ((n C + c) H + y) W + x, n = j - offs[g].
template <typename T>
__global__ __launch_bounds__(256) void dropout_kernel(T* __restrict__ x, const int* __restrict__ offs, int n_groups, long long total,
                                                      int C, int H, int W, unsigned thr, float scale, unsigned seed_lo,
                                                      unsigned seed_hi, unsigned c2, unsigned step) {
  const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
  if (e >= total) return;
  const int c = (int)(e % C);
  const long long pix = e / C;
  const int xw = (int)(pix % W);
  const int y = (int)((pix / W) % H);
  const int j = (int)(pix / ((long long)W * H));
  int lo = 0, hi = n_groups;                       // group of sample j: offs[lo] <= j < offs[lo + 1]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (offs[mid] <= j) lo = mid; else hi = mid;
  }
  if (j >= offs[n_groups]) return;                 // rows past the routed samples are left alone
  const unsigned long long lin = (((unsigned long long)(j - offs[lo]) * C + c) * H + y) * W + xw;
  unsigned w[4];
  philox4x32_10((unsigned)(lin >> 2), (unsigned)(lin >> 34), c2, step, seed_lo, seed_hi ^ (unsigned)lo, w);
  const unsigned sel = (unsigned)lin & 3u;
  const unsigned wd = sel == 0 ? w[0] : (sel == 1 ? w[1] : (sel == 2 ? w[2] : w[3]));
  x[e] = (wd >> 8) >= thr ? from_float<T>(to_float(x[e]) * scale) : from_float<T>(0.f);
}
template <typename T>
void launch_dropout(T* x, const int* offs, int n_groups, int n, int C, int H, int W, float p, unsigned long long seed, int step,
                    int layer, int pass_id, hipStream_t st) {
  const long long total = (long long)n * H * W * C;
  if (total == 0) return;
  if (!(p >= 0.f && p < 1.f) || n_groups < 1) return launch_fail("dropout: probability outside [0, 1), or no group");
  const double t = ceil((double)p * 16777216.0);
  hipLaunchKernelGGL((dropout_kernel<T>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, x, offs, n_groups, total, C, H, W,
                     (unsigned)t, 1.0f / (1.0f - p), (unsigned)(seed & 0xffffffffull), (unsigned)(seed >> 32),
                     (unsigned)(layer + 256 * pass_id), (unsigned)step);
}
template void launch_dropout<float>(float*, const int*, int, int, int, int, int, float, unsigned long long, int, int, int, hipStream_t);
template void launch_dropout<bf16_t>(bf16_t*, const int*, int, int, int, int, int, float, unsigned long long, int, int, int, hipStream_t);

// Upsample x2 + Conv k3 s1 p1 as ConvTranspose k4 s2 p1: per axis, tap t4 of the transposed convolution is the sum of
// the 3-tap filter's taps in S(t4), S(0) = {2}, S(1) = {1, 2}, S(2) = {0, 1}, S(3) = {0}.
__device__ inline void taps_of(int t4, int& first, int& count) {
  first = t4 == 0 ? 2 : (t4 == 1 ? 1 : 0);
  count = (t4 == 1 || t4 == 2) ? 2 : 1;
}
// w3: fp32 [G][9][cb][cs] ; w4: T [G][16][cb][cs] ; w4t: T [G][16][cs][cb] (written by the tiled transpose afterwards)
// grid (chunks of cb * cs, 16 taps, G): no index divisions beyond one 32-bit one
template <typename T>
__global__ __launch_bounds__(256) void w3_to_w4_kernel(const float* __restrict__ w3, T* __restrict__ w4, int cb, int cs, long long w3_stride,
                                                       long long w4_stride) {
  const int inner = blockIdx.x * 256 + threadIdx.x;                       // b * cs + s
  if (inner >= cb * cs) return;
  const int t = blockIdx.y;
  const long long g = blockIdx.z;
  int y0, ny, x0, nx;
  taps_of(t >> 2, y0, ny);
  taps_of(t & 3, x0, nx);
  float v = 0.f;
  for (int ky = y0; ky < y0 + ny; ++ky)
    for (int kx = x0; kx < x0 + nx; ++kx) v += w3[g * w3_stride + (long long)(ky * 3 + kx) * cb * cs + inner];
  w4[g * w4_stride + (long long)t * cb * cs + inner] = from_float<T>(v);
}
// w4t[g][t][s][b] = w4[g][t][b][s] for channel counts the tiled transpose does not take (element by element)
template <typename T>
__global__ __launch_bounds__(256) void transpose_plain_kernel(const T* __restrict__ w4, T* __restrict__ w4t, int cb, int cs, long long stride) {
  const int inner = blockIdx.x * 256 + threadIdx.x;
  if (inner >= cb * cs) return;
  const int b = inner / cs, s = inner - b * cs;
  const long long base = (long long)blockIdx.z * stride + (long long)blockIdx.y * cb * cs;
  w4t[base + (long long)s * cb + b] = w4[base + inner];
}
template <typename T>
void launch_w3_to_w4(const float* w3, T* w4, T* w4t, int n_groups, int cb, int cs, hipStream_t st, long long w3_stride,
                     long long w4_stride) {
  if (n_groups == 0 || cb == 0 || cs == 0) return;
  if (n_groups > 65535 || (long long)cb * cs >= (1LL << 31)) return launch_fail("summed-tap weights: more than 65535 groups, or a filter plane of 2^31 elements");
  const long long s4 = w4_stride ? w4_stride : (long long)16 * cb * cs;
  hipLaunchKernelGGL((w3_to_w4_kernel<T>), dim3((unsigned)((cb * cs + 255) / 256), 16, (unsigned)n_groups), dim3(256), 0, st, w3, w4, cb, cs,
                     w3_stride ? w3_stride : (long long)9 * cb * cs, s4);
  if (w4t) {
    if (cb % 32 == 0) launch_transpose_w<T, T>(w4, w4t, s4, n_groups, cb, cs, st);      // 32 x 32 tiles through LDS
    else hipLaunchKernelGGL((transpose_plain_kernel<T>), dim3((unsigned)((cb * cs + 255) / 256), 16, (unsigned)n_groups), dim3(256), 0, st, w4, w4t, cb, cs, s4);
  }
}
template void launch_w3_to_w4<float>(const float*, float*, float*, int, int, int, hipStream_t, long long, long long);
template void launch_w3_to_w4<bf16_t>(const float*, bf16_t*, bf16_t*, int, int, int, hipStream_t, long long, long long);

// the adjoint map: dw3[ky][kx] = sum of dw4[t4y][t4x] over the t4 whose sets contain ky / kx.  fp32 [G][16][cb][cs] -> [G][9][cb][cs]
__global__ __launch_bounds__(256) void dw4_to_dw3_kernel(const float* __restrict__ dw4, float* __restrict__ dw3, long long total,
                                                         int cb, int cs, long long dw4_stride, long long dw3_stride) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;      // (g, tap9, cb, cs)
  if (idx >= total) return;
  const long long inner = idx % ((long long)cb * cs);
  const int t = (int)((idx / ((long long)cb * cs)) % 9);
  const long long g = idx / ((long long)cb * cs * 9);
  const int ky = t / 3, kx = t - 3 * ky;
  // 3-tap index k belongs to S(3 - k) and S(2 - k)
  float v = 0.f;
  for (int ay = 2 - ky; ay <= 3 - ky; ++ay)
    for (int ax = 2 - kx; ax <= 3 - kx; ++ax) v += dw4[g * dw4_stride + ((long long)(ay * 4 + ax) * cb) * cs + inner];
  dw3[g * dw3_stride + (long long)t * cb * cs + inner] = v;
}
void launch_dw4_to_dw3(const float* dw4, float* dw3, int n_groups, int cb, int cs, hipStream_t st, long long dw4_stride,
                       long long dw3_stride) {
  const long long total = (long long)n_groups * 9 * cb * cs;
  if (total == 0) return;
  hipLaunchKernelGGL(dw4_to_dw3_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, dw4, dw3, total, cb, cs,
                     dw4_stride ? dw4_stride : (long long)16 * cb * cs, dw3_stride ? dw3_stride : (long long)9 * cb * cs);
}

}  // namespace gan
