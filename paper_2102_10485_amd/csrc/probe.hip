// Two measurements of what this chip delivers to the simplest possible kernels, for reporting the step's kernels
// against achievable rather than published peaks: a register-only MFMA loop and a plain device-to-device copy.
#include <hip/hip_runtime.h>

#include "../../include/gan.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// 8 independent accumulators per wave keep the MFMA pipe full; operands never change.
template <bool BF16>
__global__ __launch_bounds__(256) void mfma_loop_kernel(float* out, int iters) {
  floatx16 acc[8];
  for (int i = 0; i < 8; ++i)
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  const uint4 a = make_uint4(threadIdx.x, 1, 2, 3), b = make_uint4(5, 6, 7, threadIdx.x);
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (BF16) {
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc[i], 0, 0, 0);
      } else {
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc[i], 0, 0, 0);
      }
    }
  }
  float s = 0.f;
  for (int i = 0; i < 8; ++i)
    for (int e = 0; e < 16; ++e) s += acc[i][e];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// four 16-byte streaming loads in flight per thread, then four streaming stores
__global__ __launch_bounds__(256) void copy_kernel(const float4* __restrict__ src, float4* __restrict__ dst, long long n) {
  typedef float f4 __attribute__((ext_vector_type(4)));
  const f4* s = reinterpret_cast<const f4*>(src);
  f4* d = reinterpret_cast<f4*>(dst);
  const long long stride = (long long)gridDim.x * blockDim.x;
  long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  for (; i + 3 * stride < n; i += 4 * stride) {
    const f4 a = __builtin_nontemporal_load(s + i), b = __builtin_nontemporal_load(s + i + stride);
    const f4 c = __builtin_nontemporal_load(s + i + 2 * stride), e = __builtin_nontemporal_load(s + i + 3 * stride);
    __builtin_nontemporal_store(a, d + i);
    __builtin_nontemporal_store(b, d + i + stride);
    __builtin_nontemporal_store(c, d + i + 2 * stride);
    __builtin_nontemporal_store(e, d + i + 3 * stride);
  }
  for (; i < n; i += stride) d[i] = s[i];
}

template <typename F>
bool time_ms(hipStream_t st, int reps, F launch, float* ms) {
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return false;
  launch();                                                  // warm-up
  bool ok = hipEventRecord(e0, st) == hipSuccess;
  for (int i = 0; i < reps; ++i) launch();
  ok = ok && hipEventRecord(e1, st) == hipSuccess && hipEventSynchronize(e1) == hipSuccess &&
       hipEventElapsedTime(ms, e0, e1) == hipSuccess;
  *ms /= (float)reps;
  hipEventDestroy(e0);
  hipEventDestroy(e1);
  return ok && hipGetLastError() == hipSuccess;
}

}  // namespace

extern "C" gan_status gan_probe_mfma(int32_t precision, void* hip_stream, double* tflops) {
  if (!tflops || (precision != GAN_FP32 && precision != GAN_BF16_FP32MASTER)) return GAN_E_ARG;
  hipStream_t st = (hipStream_t)hip_stream;
  const int blocks = 256 * 8, iters = 2000;
  float* out = nullptr;
  if (hipMalloc(&out, (size_t)blocks * 256 * sizeof(float)) != hipSuccess) return GAN_E_OOM;
  float ms = 0.f;
  const bool bf16 = precision == GAN_BF16_FP32MASTER;
  const bool ok = time_ms(st, 3, [&] {
    if (bf16) hipLaunchKernelGGL(mfma_loop_kernel<true>, dim3(blocks), dim3(256), 0, st, out, iters);
    else hipLaunchKernelGGL(mfma_loop_kernel<false>, dim3(blocks), dim3(256), 0, st, out, iters);
  }, &ms);
  (void)hipFree(out);
  if (!ok) return GAN_E_HIP;
  const double flop_per_mfma = 2.0 * 32 * 32 * (bf16 ? 16 : 2);
  *tflops = (double)blocks * 4 /* waves */ * 8 * iters * flop_per_mfma / (ms * 1e9);
  return GAN_OK;
}

extern "C" gan_status gan_probe_copy(int64_t bytes, void* hip_stream, double* gbps) {
  if (!gbps || bytes < (1 << 20) || bytes % 16) return GAN_E_ARG;
  hipStream_t st = (hipStream_t)hip_stream;
  float4 *src = nullptr, *dst = nullptr;
  if (hipMalloc(&src, (size_t)bytes) != hipSuccess) return GAN_E_OOM;
  if (hipMalloc(&dst, (size_t)bytes) != hipSuccess) { (void)hipFree(src); return GAN_E_OOM; }
  (void)hipMemsetAsync(src, 0, (size_t)bytes, st);
  float ms = 0.f;
  const long long n = bytes / 16;
  const bool ok = time_ms(st, 5, [&] { hipLaunchKernelGGL(copy_kernel, dim3(256 * 16), dim3(256), 0, st, src, dst, n); }, &ms);
  (void)hipFree(src);
  (void)hipFree(dst);
  if (!ok) return GAN_E_HIP;
  *gbps = 2.0 * (double)bytes / (ms * 1e6);                  // bytes read + bytes written
  return GAN_OK;
}
