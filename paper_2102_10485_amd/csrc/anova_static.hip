// gan_anova_f_static: the per-channel analysis of variance for callers that cannot allocate device memory.  The
// intermediate results of its three kernels (per-image channel means, per-label sums, counts and squared deviations)
// live in one file-scope device array instead of buffers obtained from hipMalloc; every device the library runs
// on holds its own copy of that array until the process ends.
#include "../../include/gan.h"

#include <mutex>

#include "anova_host.h"
#include "kernels.h"

using namespace gan;

namespace {

constexpr int MAX_N = GAN_ANOVA_STATIC_MAX_IMAGES;
constexpr int MAX_K = GAN_ANOVA_STATIC_MAX_LABELS;
constexpr int MAX_C = 4;
constexpr size_t OFF_X = 0;                                                     // double [MAX_N][MAX_C]
constexpr size_t OFF_GSUM = OFF_X + (size_t)MAX_N * MAX_C * sizeof(double);      // double [MAX_K][MAX_C]
constexpr size_t OFF_SSW = OFF_GSUM + (size_t)MAX_K * MAX_C * sizeof(double);    // double [MAX_K][MAX_C]
constexpr size_t OFF_GCNT = OFF_SSW + (size_t)MAX_K * MAX_C * sizeof(double);    // int    [MAX_K]
constexpr size_t SCRATCH_BYTES = OFF_GCNT + (size_t)MAX_K * sizeof(int);

// In host code this name is only a handle for hipGetSymbolAddress, never an address to hand to a kernel.
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_lock;
unsigned char* g_scratch_ptr[MAX_DEVICES];     // device address of `scratch` on each device, filled at first use
const char* g_static_error = "";

gan_status static_fail(gan_status s, const char* msg) {
  g_static_error = msg;
  return s;
}

// Device address of this device's copy of the array (looked up once per device, with that device current).
gan_status scratch_of_current_device(unsigned char** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return static_fail(GAN_E_HIP, "no current HIP device");
  std::lock_guard<std::mutex> g(g_lock);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return static_fail(GAN_E_HIP, "hipGetSymbolAddress failed for the static scratch array");
    }
    g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
  }
  *out = g_scratch_ptr[dev];
  return GAN_OK;
}

}  // namespace

extern "C" {

const char* gan_static_last_error(void) { return g_static_error; }

gan_status gan_anova_f_static(const int32_t* label_ids, const float* images, int32_t n, int32_t n_labels, int32_t img_c,
                              int32_t img_hw, void* hip_stream, double* F) {
  if (!F || img_c < 1 || img_c > MAX_C) return static_fail(GAN_E_ARG, "F is null or img_c outside [1, 4]");
  for (int ch = 0; ch < img_c; ++ch) F[ch] = 0.0;
  if (n < 0 || n_labels < 1 || img_hw < 1) return static_fail(GAN_E_ARG, "negative n, or n_labels / img_hw below 1");
  if (n > MAX_N) return static_fail(GAN_E_SHAPE, "n exceeds GAN_ANOVA_STATIC_MAX_IMAGES (the static scratch array holds no more)");
  if (n_labels > MAX_K) return static_fail(GAN_E_SHAPE, "n_labels exceeds GAN_ANOVA_STATIC_MAX_LABELS (the static scratch array holds no more)");
  if (n == 0) return static_fail(GAN_E_STATE, "no images");
  if (!label_ids || !images) return static_fail(GAN_E_ARG, "null pointer");
  unsigned char* base = nullptr;
  const gan_status s = scratch_of_current_device(&base);
  if (s != GAN_OK) return s;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  double* x = reinterpret_cast<double*>(base + OFF_X);
  double* gsum = reinterpret_cast<double*>(base + OFF_GSUM);
  double* ssw = reinterpret_cast<double*>(base + OFF_SSW);
  int* gcnt = reinterpret_cast<int*>(base + OFF_GCNT);
  // the three kernels write every element they later read (x[0, n*C), gsum / ssw [0, K*C), gcnt [0, K)), so nothing
  // left by an earlier call has to be cleared
  launch_anova(label_ids, images, n, n_labels, img_c, img_hw * img_hw, x, gsum, gcnt, ssw, st);
  static thread_local double h_gsum[MAX_K * MAX_C], h_ssw[MAX_K * MAX_C];
  static thread_local int h_gcnt[MAX_K];
  const size_t kc = (size_t)n_labels * img_c;
  if (hipGetLastError() != hipSuccess || hipStreamSynchronize(st) != hipSuccess ||
      hipMemcpy(h_gsum, gsum, kc * sizeof(double), hipMemcpyDeviceToHost) != hipSuccess ||
      hipMemcpy(h_ssw, ssw, kc * sizeof(double), hipMemcpyDeviceToHost) != hipSuccess ||
      hipMemcpy(h_gcnt, gcnt, (size_t)n_labels * sizeof(int), hipMemcpyDeviceToHost) != hipSuccess)
    return static_fail(GAN_E_HIP, "analysis of variance failed on the device");
  if (!anova_f_from_sums(h_gsum, h_ssw, h_gcnt, n_labels, img_c, F))
    return static_fail(GAN_E_STATE, "fewer than two labels present, or not more images than labels");
  return GAN_OK;
}

}  // extern "C"
