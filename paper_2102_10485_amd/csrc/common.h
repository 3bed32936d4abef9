// Shared declarations of the gfx950 kernels and their host launchers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gan {

// bf16 storage: upper half of an fp32, round-to-nearest-even on conversion.
struct bf16_t {
  unsigned short v;
};

__host__ __device__ inline float to_float(float x) { return x; }
__host__ __device__ inline float to_float(bf16_t x) {
  union { unsigned u; float f; } c;
  c.u = (unsigned)x.v << 16;
  return c.f;
}
__host__ __device__ inline unsigned short f32_to_bf16_bits(float f) {
  union { unsigned u; float f; } c;
  c.f = f;
  unsigned u = c.u;
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;   // NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (unsigned short)(u >> 16);
}
template <typename T> __host__ __device__ inline T from_float(float f);
template <> __host__ __device__ inline float from_float<float>(float f) { return f; }
// On the device the conversion is the hardware's (v_cvt_pk_bf16_f32, round to nearest even like the function above);
// the software rounding costs six vector instructions per element, which made several kernels instruction-bound.
#if defined(__HIP_DEVICE_COMPILE__)
typedef float gan_f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 gan_bf16x2 __attribute__((ext_vector_type(2)));
__host__ __device__ inline unsigned pack2_bf16(float lo, float hi) {
  const gan_f32x2 v = {lo, hi};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(v, gan_bf16x2));
}
template <> __host__ __device__ inline bf16_t from_float<bf16_t>(float f) {
  bf16_t r;
  r.v = __builtin_bit_cast(unsigned short, (__bf16)f);
  return r;
}
#else
__host__ __device__ inline unsigned pack2_bf16(float lo, float hi) { return (unsigned)f32_to_bf16_bits(lo) | ((unsigned)f32_to_bf16_bits(hi) << 16); }
template <> __host__ __device__ inline bf16_t from_float<bf16_t>(float f) {
  bf16_t r;
  r.v = f32_to_bf16_bits(f);
  return r;
}
#endif

// A host launcher that finds its assumptions violated records the reason and launches nothing; the library call in
// progress then returns an error status with this text (nothing in the library ends the process).
void launch_fail(const char* msg);
const char* take_launch_error();   // the first reason recorded on this thread since the last call, or nullptr

enum ConvMode { MODE_DOWN = 0, MODE_UP = 1, MODE_DENSE = 2 };
enum Epilogue { EPI_NONE = 0, EPI_ACT_BWD = 1, EPI_LRELU = 2 };
enum Act { ACT_RELU = 0, ACT_LRELU = 1 };

// Arguments of the grouped implicit-GEMM forward-type kernel (down / up / dense).
struct ConvArgs {
  const void* A;         // gathered activations (storage type)
  const void* W;         // weights of model 0, K-contiguous: [tap][N][C] (storage type)
  void* Out;             // output activations (storage type)
  const void* Aux;       // EPI_ACT_BWD: saved forward output at the output position (storage type)
  float* stat_partial;   // if set: per sub-tile (the row block of one wave row of the tile; conv_stat_split of them per tile) the
                         // column sums of the output and of its squared deviations from the sub-tile's column mean,
                         // [(((phase * nseg + segment) * ub_tiles + tile) * split + block) * N + col][2], for the BatchNorm that follows
  int w_nstride;         // rows per tap in the weight block (>= N)
  const int* offs;       // [L+1] sample offsets of the models inside one segment
  const int* tpre;       // [L+1] prefix of M-tiles per model for this geometry
  const int* tmodel;     // model of every M-tile of this geometry (NULL: found by bisection in tpre)
  long long w_stride;    // elements between two models' weight blocks
  int L;                 // models
  int seg_first, nseg;   // segments to process: rows of segment s start at sample s*seg_samples
  int seg_samples;
  int C, N;              // channels per tap of A, output channels
  int Hin;               // side of the gathered tensor
  int Hr;                // side of the row space (rows per sample = Hr*Hr)
  int ub_tiles;          // launched upper bound of M-tiles per (segment, phase)
  int tile_rows;         // rows per M-tile the prefix array was built for (conv_tile_rows)
  int hr_shift;          // log2(Hr) or -1 (filled by the launcher)
  float slope;           // EPI_ACT_BWD: derivative on the non-positive side
};

// Arguments of the grouped weight-gradient kernel: dW[tap][cb][cs] = sum_rows big(tap)[cb] * small[cs].
struct WgradArgs {
  const void* Big;       // tensor gathered through the taps, side 2*Hs, channels Cb (ntaps == 1: read row by row)
  const void* Small;     // tensor indexed directly by row, side Hs, channels Cs
  float* dW;             // fp32 output of model 0: [ntaps][Cb][Cs]
  const int* offs;       // [L+1]
  const int* order;      // [L] models by decreasing row count, or NULL: which model a group of blocks takes (the
                         //     big models start first and the XCDs get equal shares; no effect on the results)
  long long dw_stride;   // elements between two models' blocks
  int L, nseg, seg_samples;
  int Cb, Cs, Hs;
  int ntaps;             // 16 (conv) or 1 (dense)
  int ksplit;            // >= 1: the rows of each segment are shared by this many blocks, each writing its own
  long long split_stride;//        partial block dW + split * split_stride (the caller adds them in order)
  int hs_shift;          // log2(Hs) or -1 (filled by the launcher)
};

template <typename T> void launch_conv(int mode, int epi, const ConvArgs& a, hipStream_t st);
template <typename T> void launch_wgrad(const WgradArgs& a, hipStream_t st);
// names of the kernel instantiations the two launchers pick (per-kernel timing)
const char* conv_variant_name(int mode, int epi, const ConvArgs& a);
const char* wgrad_variant_name(const WgradArgs& a);
// output tiles per model of the weight-gradient launch for this layer shape
int wgrad_tiles_per_model(int ntaps, int Cb, int Cs);

// rows per M-tile the forward-type kernel will use for n_out output channels and about rows_per_model rows
int conv_tile_rows(int n_out, long long rows_per_model_hint, int n_models);
// row blocks per tile with their own BatchNorm partial sums, for the tile the forward-type kernel uses for n_out channels
int conv_stat_split(int n_out, int tile_rows);

}  // namespace gan
