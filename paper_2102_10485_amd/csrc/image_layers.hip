// The two layers that touch the image (1..4 channels): D's first convolution and G's last transposed
// convolution.  With so few image channels their implicit-GEMM K (16 taps x channels) is tiny, so the image
// side is expanded once into an explicit patch matrix ("im2col") of 64-column rows and the layers run on the
// same MFMA engine as everything else, as plain row-by-row GEMMs:
//   forward of D's first conv      : feat = patches x Wp^T
//   its weight gradient            : dWp  = patches^T x dfeat
//   data gradient of G's last convT: dfeat = patches(d image) x Wp^T ; its weight gradient likewise.
//
// A one-hot label map is a constant plane: its contribution to D's first convolution is a per-position bias
// that only differs at the border (3 x 3 position classes), and its weight gradient is the sum of dfeat over the
// positions where the tap falls inside the image.  Both are exact.  The patch matrix therefore carries, after the
// 16*CB tap columns, one indicator column per (label slot, position class) and one constant column: the packed
// weight holds the summed label-map taps and the bias there, so the forward GEMM adds them and the weight-
// gradient GEMM returns the class sums and the bias gradient with no extra pass over the feature tensor.
#include <stdlib.h>

#include <algorithm>

#include "kernels.h"

namespace gan {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <typename T> __device__ inline float ldf(const T* p) { return to_float(*p); }

// Position class along one axis: 0 = first output row/col (tap 0 outside), 1 = interior, 2 = last (tap 3 outside).
__device__ inline bool tap_valid(int cls, int k) { return !((cls == 0 && k == 0) || (cls == 2 && k == 3)); }
__device__ inline int pos_class(int y, int x, int Hs) {
  return (y == 0 ? 0 : (y == Hs - 1 ? 2 : 1)) * 3 + (x == 0 ? 0 : (x == Hs - 1 ? 2 : 1));
}

__device__ inline void store8(float* p, const float (&v)[8]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
__device__ inline void store8(bf16_t* p, const float (&v)[8]) {
  uint4 t;
  t.x = pack2_bf16(v[0], v[1]);
  t.y = pack2_bf16(v[2], v[3]);
  t.z = pack2_bf16(v[4], v[5]);
  t.w = pack2_bf16(v[6], v[7]);
  *reinterpret_cast<uint4*>(p) = t;
}

// One thread per 8 columns of one patch row.
template <typename T>
__global__ __launch_bounds__(256) void im2col_kernel(Im2colArgs a) {
  const int g8 = a.Kc >> 3;
  const int rps = a.Hs * a.Hs, Hb = 2 * a.Hs;
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long long)a.n * rps * g8) return;
  const long long row = idx / g8;
  const int m0 = (int)(idx - row * g8) * 8;
  const int j = (int)(row / rps), pix = (int)(row - (long long)j * rps);
  if (j >= a.offs[a.L]) return;
  const int y = pix / a.Hs, x = pix - y * a.Hs;
  const int ntap = 16 * a.CB;
  const T* img = nullptr;
  const float* real = nullptr;
  if (a.img) img = static_cast<const T*>(a.img) + ((long long)a.seg * a.seg_samples + j) * Hb * Hb * a.CB;
  else real = a.real + (long long)a.perm[j] * a.CB * Hb * Hb;
  float v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int m = m0 + e;
    float val = 0.f;
    if (m < ntap) {
      const int tap = m / a.CB, cb = m - tap * a.CB;
      const int iy = 2 * y - 1 + (tap >> 2), ix = 2 * x - 1 + (tap & 3);
      if ((unsigned)iy < (unsigned)Hb && (unsigned)ix < (unsigned)Hb)
        val = img ? ldf(img + ((long long)iy * Hb + ix) * a.CB + cb) : real[((long long)cb * Hb + iy) * Hb + ix];
    } else if (a.nslot > 0) {
      const int q = m - ntap;
      if (q < 9 * a.nslot) val = (q / 9 == a.sample_slot[j] && q % 9 == pos_class(y, x, a.Hs)) ? 1.f : 0.f;
      else if (q == 9 * a.nslot) val = 1.f;
    }
    v[e] = val;
  }
  store8(static_cast<T*>(a.out) + (((long long)a.seg * a.seg_samples + j) * rps + pix) * a.Kc + m0, v);
}
// Same result, one block per sample: the sample's image goes through LDS once (NHWC, storage type, with a one-pixel
// border of zeros so that no tap needs a bounds test), and every thread keeps the decoding of its 8 columns -- for a
// tap column the offset of its element from the patch's first one -- while it walks down the sample's patch rows.
template <typename T>
__global__ __launch_bounds__(256) void im2col_sample_kernel(Im2colArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  T* tile = reinterpret_cast<T*>(lds_raw);                       // [Hb + 2][Hb + 2][CB]
  const int j = blockIdx.x;
  if (j >= a.offs[a.L]) return;
  const int g8 = a.Kc >> 3;
  const int nt = blockDim.x;                                      // a multiple of g8 (the launcher's choice), at most 256
  const int rps = a.Hs * a.Hs, Hb = 2 * a.Hs, CB = a.CB;
  const int npix = Hb * Hb, Hp = Hb + 2;
  // the border: rows 0 and Hp - 1, columns 0 and Hp - 1
  for (int t = threadIdx.x; t < 4 * Hp * CB; t += nt) {
    const int side = t / (Hp * CB), r = t - side * (Hp * CB);
    const int q = r / CB, cb = r - q * CB;
    const int py = side == 0 ? 0 : (side == 1 ? Hp - 1 : q), px = side < 2 ? q : (side == 2 ? 0 : Hp - 1);
    tile[(py * Hp + px) * CB + cb] = from_float<T>(0.f);
  }
  if (a.img) {
    const T* img = static_cast<const T*>(a.img) + ((long long)a.seg * a.seg_samples + j) * npix * CB;
    for (int t = threadIdx.x; t < npix * CB; t += nt) {
      const int pxl = t / CB, cb = t - pxl * CB;
      const int py = pxl / Hb, px = pxl - py * Hb;
      tile[((py + 1) * Hp + px + 1) * CB + cb] = img[t];
    }
  } else {
    const float* real = a.real + (long long)a.perm[j] * CB * npix;     // NCHW fp32; npix is a multiple of 4
    const int nq = npix >> 2;
    if ((reinterpret_cast<uintptr_t>(a.real) & 15) != 0) {             // caller's buffer not 16-byte aligned: scalar loads
      for (int t = threadIdx.x; t < npix * CB; t += nt) {
        const int cb = t / npix, pxl = t - cb * npix;
        const int py = pxl / Hb, px = pxl - py * Hb;
        tile[((py + 1) * Hp + px + 1) * CB + cb] = from_float<T>(real[t]);
      }
    } else
    for (int t = threadIdx.x; t < CB * nq; t += nt) {
      const int cb = t / nq, pxl = 4 * (t - cb * nq);
      const float4 v = reinterpret_cast<const float4*>(real)[t];
      const float vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int k = 0; k < 4; ++k) {                                    // (four pixels of a row, unless Hb % 4 == 2)
        const int py = (pxl + k) / Hb, px = pxl + k - py * Hb;
        tile[((py + 1) * Hp + px + 1) * CB + cb] = from_float<T>(vv[k]);
      }
    }
  }
  const int ntap = 16 * CB;                        // a multiple of 8: a group of 8 columns is all taps or none
  const int slot = a.nslot > 0 ? a.sample_slot[j] : 0;
  T* out = static_cast<T*>(a.out) + ((long long)a.seg * a.seg_samples + j) * rps * a.Kc;
  // The columns after the taps (label-map indicators, the constant one, padding) depend on the pixel only through its
  // position class: their 9 possible rows are written once, behind the image tile.
  const int gtap = ntap >> 3, gsp = g8 - gtap;     // groups of tap columns, of the others
  T* special = tile + Hp * Hp * CB + ((16 - ((Hp * Hp * CB * (int)sizeof(T)) & 15)) & 15) / (int)sizeof(T);   // 16-byte aligned; [9][gsp * 8]
  for (int t = threadIdx.x; t < 9 * gsp * 8; t += nt) {
    const int cls = t / (gsp * 8), q = t - cls * (gsp * 8);          // q: column - ntap
    float val = 0.f;
    if (a.nslot > 0) {
      if (q < 9 * a.nslot) val = (q / 9 == slot && q % 9 == cls) ? 1.f : 0.f;
      else if (q == 9 * a.nslot) val = 1.f;
    }
    special[t] = from_float<T>(val);
  }
  __syncthreads();
  // A thread keeps its group of 8 columns (the block's thread count is a multiple of the groups per row) and walks
  // down the patch rows in steps of threads / g8; the row's (y, x) is carried along instead of divided out, and the values
  // travel as stored (no conversion): the kernel is bound by its vector instructions otherwise.
  const int g = (int)threadIdx.x % g8, pstep = nt / g8;
  int off[8];                                      // tap columns: element offset from the patch's corner
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int m = g * 8 + e;
    const int tap = m / CB, cb = m - tap * CB;
    off[e] = m < ntap ? ((tap >> 2) * Hp + (tap & 3)) * CB + cb : 0;
  }
  const bool taps = g < gtap;
  constexpr int VB = 8 * (int)sizeof(T);           // bytes of a group
  int pix = (int)threadIdx.x / g8;
  int y = pix / a.Hs, x = pix - y * a.Hs;
  for (; pix < rps; pix += pstep) {
    uint4 pk[VB / 16];
    if (taps) {
      const T* corner = tile + (2 * y * Hp + 2 * x) * CB;      // padded position of input pixel (2y - 1, 2x - 1)
      T v[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = corner[off[e]];
      if constexpr (sizeof(T) == 2) {
        pk[0].x = (unsigned)v[0].v | ((unsigned)v[1].v << 16);
        pk[0].y = (unsigned)v[2].v | ((unsigned)v[3].v << 16);
        pk[0].z = (unsigned)v[4].v | ((unsigned)v[5].v << 16);
        pk[0].w = (unsigned)v[6].v | ((unsigned)v[7].v << 16);
      } else {
        const unsigned* u = reinterpret_cast<const unsigned*>(v);
        pk[0] = make_uint4(u[0], u[1], u[2], u[3]);
        pk[VB / 16 - 1] = make_uint4(u[4], u[5], u[6], u[7]);
      }
    } else {
      const uint4* src = reinterpret_cast<const uint4*>(special + (pos_class(y, x, a.Hs) * gsp + (g - gtap)) * 8);
#pragma unroll
      for (int k = 0; k < VB / 16; ++k) pk[k] = src[k];
    }
    uint4* dst = reinterpret_cast<uint4*>(out + (long long)pix * a.Kc + g * 8);
#pragma unroll
    for (int k = 0; k < VB / 16; ++k) dst[k] = pk[k];
    x += pstep;
    while (x >= a.Hs) { x -= a.Hs; ++y; }
  }
}
template <typename T> void launch_im2col(const Im2colArgs& a, hipStream_t st) {
  const long long tot = (long long)a.n * a.Hs * a.Hs * (a.Kc / 8);
  if (tot == 0) return;
  // the zero-bordered image tile, then (16-byte aligned) the 9 possible rows of the columns behind the taps
  const size_t lds = (size_t)(2 * a.Hs + 2) * (2 * a.Hs + 2) * a.CB * sizeof(T) + 16 + (size_t)9 * (a.Kc - 16 * a.CB) * sizeof(T);
  const int g8 = a.Kc / 8;
  if (lds <= 64 * 1024 && g8 >= 1 && g8 <= 256 && a.Kc >= 16 * a.CB) {
    if (lds > 48 * 1024)   // above the default dynamic limit: ask for it (idempotent, cheap)
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&im2col_sample_kernel<T>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipLaunchKernelGGL((im2col_sample_kernel<T>), dim3((unsigned)a.n), dim3((unsigned)(256 / g8 * g8)), lds, st, a);
    return;
  }
  hipLaunchKernelGGL((im2col_kernel<T>), dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st, a);
}
template void launch_im2col<float>(const Im2colArgs&, hipStream_t);
template void launch_im2col<bf16_t>(const Im2colArgs&, hipStream_t);

// Wp[l][cs][m]: the taps, then the summed label-map taps per (slot, class), then the bias.
template <typename T>
__global__ void pack_w_kernel(PackArgs a) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long long)a.L * a.Cs * a.Kc) return;
  const int m = (int)(idx % a.Kc);
  const int cs = (int)((idx / a.Kc) % a.Cs);
  const int l = (int)(idx / ((long long)a.Kc * a.Cs));
  const float* w = a.w + (long long)l * a.pstride;
  const int ntap = 16 * a.CB;
  float val = 0.f;
  if (m < ntap) {
    const int tap = m / a.CB, cb = m - tap * a.CB;
    val = w[((long long)tap * a.CBT + cb) * a.Cs + cs];
  } else if (a.nslot > 0) {
    const int q = m - ntap;
    if (q < 9 * a.nslot) {
      const int slot = q / 9, cls = q - slot * 9;
      if (a.CBT > a.CB) {
        const int label = (a.L == 1) ? slot : l;
        for (int tap = 0; tap < 16; ++tap)
          if (tap_valid(cls / 3, tap >> 2) && tap_valid(cls % 3, tap & 3))
            val += w[((long long)tap * a.CBT + a.CB + label) * a.Cs + cs];
      }
    } else if (q == 9 * a.nslot && a.bias) {
      val = a.bias[(long long)l * a.pstride + cs];
    }
  }
  static_cast<T*>(a.wp)[idx] = from_float<T>(val);
}
template <typename T> void launch_pack_w(const PackArgs& a, hipStream_t st) {
  const long long tot = (long long)a.L * a.Cs * a.Kc;
  hipLaunchKernelGGL((pack_w_kernel<T>), dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st, a);
}
template void launch_pack_w<float>(const PackArgs&, hipStream_t);
template void launch_pack_w<bf16_t>(const PackArgs&, hipStream_t);

// dWp[l][m][cs] (fp32) -> the gradient block: taps, label-map channels (class sums over the positions where the
// tap is inside), bias.
// element (l, m, cs) of the packed gradient: the split partial blocks added in order
__device__ inline float dwp_at(const PackArgs& a, int l, int m, int cs) {
  float s = 0.f;
  for (int k = 0; k < a.nsplit; ++k) s += a.dwp[(((long long)k * a.L + l) * a.Kc + m) * a.Cs + cs];
  return s;
}

__global__ void unpack_dw_kernel(PackArgs a) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const int Cs = a.Cs;
  const long long n_tap = (long long)a.L * 16 * a.CB * Cs;
  const long long n_lab = (a.nslot > 0 && a.CBT > a.CB) ? (long long)a.L * a.nslot * 16 * Cs : 0;
  const long long n_bias = (a.nslot > 0 && a.dbias) ? (long long)a.L * Cs : 0;
  const int ntap = 16 * a.CB;
  if (idx < n_tap) {
    const int cs = (int)(idx % Cs);
    const int m = (int)((idx / Cs) % ntap);
    const int l = (int)(idx / ((long long)Cs * ntap));
    const int tap = m / a.CB, cb = m - tap * a.CB;
    a.dw[(long long)l * a.pstride + ((long long)tap * a.CBT + cb) * Cs + cs] = dwp_at(a, l, m, cs);
    return;
  }
  long long j = idx - n_tap;
  if (j < n_lab) {
    const int cs = (int)(j % Cs);
    const int tap = (int)((j / Cs) % 16);
    const int slot = (int)((j / ((long long)Cs * 16)) % a.nslot);
    const int l = (int)(j / ((long long)Cs * 16 * a.nslot));
    const int label = (a.L == 1) ? slot : l;
    float s = 0.f;
    for (int cls = 0; cls < 9; ++cls)
      if (tap_valid(cls / 3, tap >> 2) && tap_valid(cls % 3, tap & 3))
        s += dwp_at(a, l, ntap + slot * 9 + cls, cs);
    a.dw[(long long)l * a.pstride + ((long long)tap * a.CBT + a.CB + label) * Cs + cs] = s;
    return;
  }
  j -= n_lab;
  if (j < n_bias) {
    const int l = (int)(j / Cs), cs = (int)(j - (long long)l * Cs);
    a.dbias[(long long)l * a.pstride + cs] = dwp_at(a, l, ntap + 9 * a.nslot, cs);
  }
}
// part[0][i] <- part[0][i] + part[1][i] + ... (nsplit blocks of size4 float4 each), in a fixed order: lane group q of
// a block adds the blocks q, q + 4, ... in turn, then (q0 + q1) + (q2 + q3).  One thread per element would walk the
// splits one load after the other: with one model and 128 splits that chain alone took 0.13 ms.
__global__ __launch_bounds__(256) void reduce_splits_kernel(float* __restrict__ part, long long size4, int nsplit) {
  __shared__ float4 red[4][64];
  const int c = threadIdx.x & 63, q = threadIdx.x >> 6;
  const long long i = (long long)blockIdx.x * 64 + c;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  if (i < size4) {
    const float4* p = reinterpret_cast<const float4*>(part) + i;
#pragma unroll 4
    for (int k = q; k < nsplit; k += 4) {
      const float4 t = p[(long long)k * size4];
      acc.x += t.x; acc.y += t.y; acc.z += t.z; acc.w += t.w;
    }
  }
  red[q][c] = acc;
  __syncthreads();
  if (q == 0 && i < size4) {
    const float4 a0 = red[0][c], a1 = red[1][c], a2 = red[2][c], a3 = red[3][c];
    reinterpret_cast<float4*>(part)[i] = make_float4((a0.x + a1.x) + (a2.x + a3.x), (a0.y + a1.y) + (a2.y + a3.y),
                                                      (a0.z + a1.z) + (a2.z + a3.z), (a0.w + a1.w) + (a2.w + a3.w));
  }
}
void launch_unpack_dw(const PackArgs& a0, hipStream_t st) {
  PackArgs a = a0;
  const long long block = (long long)a.L * a.Kc * a.Cs;       // floats per split
  if (a.nsplit > 4 && block % 4 == 0) {
    // many row splits: add them up with a kernel that has enough threads, in place into the first block
    hipLaunchKernelGGL(reduce_splits_kernel, dim3((unsigned)((block / 4 + 63) / 64)), dim3(256), 0, st, const_cast<float*>(a.dwp), block / 4,
                       a.nsplit);
    a.nsplit = 1;
  }
  const long long tot = (long long)a.L * a.Cs * (16 * a.CB + (a.nslot > 0 ? a.nslot * 16 + 1 : 0));
  hipLaunchKernelGGL(unpack_dw_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st, a);
}

// dbias[cb] = sum over the model's image-side pixels (G's last layer): block (chunk of pixels, model) partial
// sums, then one small pass adds the chunks in order.
template <typename T>
__global__ __launch_bounds__(256) void img_bias_partial_kernel(ImgBiasArgs a) {
  __shared__ float red[256];
  const int l = blockIdx.y;
  const int cnt = a.offs[l + 1] - a.offs[l];
  const long long pix = (long long)cnt * a.HW;
  const long long per = (pix + gridDim.x - 1) / gridDim.x;
  const long long p0 = per * blockIdx.x, p1 = min(pix, p0 + per);
  const T* img = static_cast<const T*>(a.img) + (long long)a.offs[l] * a.HW * a.CB;
  for (int cb = 0; cb < a.CB; ++cb) {
    float s = 0.f;
    for (long long i = p0 + threadIdx.x; i < p1; i += 256) s += ldf(img + i * a.CB + cb);
    red[threadIdx.x] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
      if (threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
      __syncthreads();
    }
    if (threadIdx.x == 0) a.partial[((long long)l * gridDim.x + blockIdx.x) * 4 + cb] = red[0];
    __syncthreads();
  }
}
// one block per model: thread t adds the chunks t, t + 256, ... in turn, then a fixed tree over the threads
__global__ __launch_bounds__(256) void img_bias_final_kernel(ImgBiasArgs a, int chunks) {
  __shared__ float red[256];
  const int l = blockIdx.x;
  if (a.offs[l + 1] == a.offs[l]) return;
  for (int cb = 0; cb < a.CB; ++cb) {
    float s = 0.f;
    for (int k = threadIdx.x; k < chunks; k += 256) s += a.partial[((long long)l * chunks + k) * 4 + cb];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
      if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
      __syncthreads();
    }
    if (threadIdx.x == 0) a.dbias[(long long)l * a.pstride + cb] = red[0];
    __syncthreads();
  }
}
// chunks of a model's pixels: enough blocks to fill the chip with few models; a function of the model count only
int img_bias_chunks(int L) { return std::min(std::max(2048 / (L > 0 ? L : 1), 32), 256); }
template <typename T> void launch_img_bias_grad(const ImgBiasArgs& a, hipStream_t st) {
  const int chunks = img_bias_chunks(a.L);
  hipLaunchKernelGGL((img_bias_partial_kernel<T>), dim3(chunks, a.L), dim3(256), 0, st, a);
  hipLaunchKernelGGL(img_bias_final_kernel, dim3(a.L), dim3(256), 0, st, a, chunks);
}
template void launch_img_bias_grad<float>(const ImgBiasArgs&, hipStream_t);
template void launch_img_bias_grad<bf16_t>(const ImgBiasArgs&, hipStream_t);

// ---------------------------------------------------------------------------------------------------------
// Transposed convolution onto the image (or the data gradient of D's first convolution, which is the same
// operation): img[n, 2y+py, 2x+px][cb] = sum over the 4 taps of that phase and cs of feat[n, y+dy, x+dx][cs] * w[tap][cb][cs].
// One block = an 8 x 8 patch of feature pixels of one sample with its 1-pixel halo held in LDS, so every feature
// row is read from memory once for all 4 phases x 4 taps; the (phase, image channel) pairs -- at most 16 -- are the N
// side of a 32 x 32 MFMA tile, and the block's four waves share the reduction over the 3 x 3 neighbourhood.
// Epilogue: bias + tanh, or times (1 - y^2).
// ---------------------------------------------------------------------------------------------------------
__device__ inline void up_mma(floatx16& acc, const uint4& a, const uint4& b, bf16_t) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
}
__device__ inline void up_mma(floatx16& acc, const uint4& a, const uint4& b, float) {
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
}

constexpr int UP_TS = 8;                    // patch side (feature pixels)
constexpr int UP_HALO = UP_TS + 2;

template <typename T, int CS>
__global__ __launch_bounds__(256) void up_img_kernel(UpImgArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  constexpr int Cs = CS;
  const int CB = a.CB, Hs = a.Hs, Hb = 2 * a.Hs;
  constexpr int rowB = Cs * (int)sizeof(T) + 16;              // bytes per halo row / weight row in LDS
  unsigned char* Fl = lds;                                    // [UP_HALO*UP_HALO][rowB]
  unsigned char* Wl = lds + UP_HALO * UP_HALO * rowB;         // [16 taps][CB][rowB]
  const int j = blockIdx.y;                                   // routed sample inside the segment
  if (j >= a.offs[a.L]) return;
  const int l = a.sample_model[j];
  const long long sample = (long long)a.seg * a.seg_samples + j;
  const int tiles = (Hs + UP_TS - 1) / UP_TS;
  const int y0 = (blockIdx.x / tiles) * UP_TS, x0 = (blockIdx.x % tiles) * UP_TS;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  constexpr int cpr = Cs * (int)sizeof(T) / 16;               // 16-byte chunks per row
  const T* feat = static_cast<const T*>(a.feat) + sample * (long long)Hs * Hs * Cs;
  // all of the block's global loads are issued before the first of them is stored to LDS
  constexpr int NF = (UP_HALO * UP_HALO * cpr + 255) / 256;
  uint4 fv[NF];
#pragma unroll
  for (int k = 0; k < NF; ++k) {
    const int i = tid + 256 * k;
    const int hr = i / cpr, ch = i - hr * cpr;
    const int y = y0 - 1 + hr / UP_HALO, x = x0 - 1 + hr % UP_HALO;
    fv[k] = make_uint4(0, 0, 0, 0);
    if (i < UP_HALO * UP_HALO * cpr && (unsigned)y < (unsigned)Hs && (unsigned)x < (unsigned)Hs)
      fv[k] = *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(feat + ((long long)y * Hs + x) * Cs) + ch * 16);
  }
  const T* w = static_cast<const T*>(a.w) + (long long)l * a.w_stride;
  constexpr int NW = (16 * 4 * cpr + 255) / 256;                // CB <= 4
  uint4 wv[NW];
#pragma unroll
  for (int k = 0; k < NW; ++k) {
    const int i = tid + 256 * k;
    const int wr = i / cpr, ch = i - wr * cpr;                  // wr = tap * CB + cb
    const int tap = (int)(((unsigned)wr * (65536u / (unsigned)CB + 1u)) >> 16), cb = wr - tap * CB;   // wr / CB, wr < 64
    wv[k] = make_uint4(0, 0, 0, 0);
    if (i < 16 * CB * cpr)
      wv[k] = *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(w + ((long long)tap * a.CBT + cb) * Cs) + ch * 16);
  }
#pragma unroll
  for (int k = 0; k < NF; ++k) {
    const int i = tid + 256 * k;
    const int hr = i / cpr, ch = i - hr * cpr;
    if (i < UP_HALO * UP_HALO * cpr) *reinterpret_cast<uint4*>(Fl + hr * rowB + ch * 16) = fv[k];
  }
#pragma unroll
  for (int k = 0; k < NW; ++k) {
    const int i = tid + 256 * k;
    const int wr = i / cpr, ch = i - wr * cpr;
    if (i < 16 * CB * cpr) *reinterpret_cast<uint4*>(Wl + wr * rowB + ch * 16) = wv[k];
  }
  __syncthreads();

  // One product for all four output phases: columns = (phase, image channel) -- 4 * CB of the MFMA tile's 32 --, rows =
  // the patch's 64 pixels, K = (neighbour pixel, feature channel) over the 3 x 3 neighbourhood; a neighbour at offset
  // (dy, dx) meets output phase (py, px) through filter tap ky = 1, 2 (dy = 0), 3 (dy = -1, py = 0) or 0 (dy = +1,
  // py = 1), likewise kx, and not at all otherwise (those lanes multiply zeros).  The four waves share the feature
  // channels: wave w takes K-steps [w, w + 1) * ksteps / 4 of every neighbour, so everything but a lane's weight row
  // is a compile-time offset.
  const int r = lane & 31, h = lane >> 5;
  const int NC = 4 * CB;
  const unsigned mCB = 65536u / (unsigned)CB + 1u;            // i / CB == (i * mCB) >> 16 for the small i below
  const int ph = (int)(((unsigned)r * mCB) >> 16), cbn = r - ph * CB;
  const int py = ph >> 1, px = ph & 1;
  floatx16 acc[2];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
  constexpr int ksteps = Cs * (int)sizeof(T) / 32;            // 32 bytes of K per MFMA step (16 per lane half)
  constexpr int kpw = ksteps / 4;
  static_assert(ksteps % 4 == 0, "K-steps per wave");
  const int kbase = __builtin_amdgcn_readfirstlane(wave) * (kpw * 32) + h * 16;
  const unsigned char* frow0[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int q = t * 32 + r;                                 // pixel of the patch: (q / 8, q % 8)
    frow0[t] = Fl + ((q / UP_TS + 1) * UP_HALO + (q % UP_TS + 1)) * rowB + kbase;
  }
  const unsigned char* wcol = Wl + cbn * rowB + kbase;        // + tap * CB rows
#pragma unroll
  for (int nb = 0; nb < 9; ++nb) {
    const int dy = nb / 3 - 1, dx = nb % 3 - 1;               // compile-time after unrolling
    const int ky = dy == 0 ? (py == 0 ? 1 : 2) : (dy < 0 ? (py == 0 ? 3 : -1) : (py == 1 ? 0 : -1));
    const int kx = dx == 0 ? (px == 0 ? 1 : 2) : (dx < 0 ? (px == 0 ? 3 : -1) : (px == 1 ? 0 : -1));
    const bool has = r < NC && ky >= 0 && kx >= 0;
    const unsigned char* brow = wcol + (has ? (ky * 4 + kx) * CB * rowB : 0);
#pragma unroll
    for (int k = 0; k < kpw; ++k) {
      uint4 b = *reinterpret_cast<const uint4*>(brow + k * 32);
      if (!has) b = make_uint4(0, 0, 0, 0);
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const uint4 av = *reinterpret_cast<const uint4*>(frow0[t] + (dy * UP_HALO + dx) * rowB + k * 32);
        up_mma(acc[t], av, b, T());
      }
    }
  }
  // epilogue: each wave leaves its partial sums of the real columns in LDS (the halo tile and the weights are no longer
  // read); all 256 threads then add the four, share the (1 - y^2) / tanh work and write whole output rows.
  __syncthreads();
  float* ep = reinterpret_cast<float*>(lds);                  // [4 waves][64 pixels][NC]
  if (r < NC) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int q = t * 32 + (e >> 2) * 8 + h * 4 + (e & 3);
        ep[(wave * 64 + q) * NC + r] = acc[t][e];
      }
  }
  __syncthreads();
  T* out = static_cast<T*>(a.out);
  const T* aux = static_cast<const T*>(a.aux);
  const int rowlen = 2 * UP_TS * CB;                          // contiguous output elements per patch row
  const unsigned mRow = 65536u / (unsigned)rowlen + 1u;       // exact for i < 1024, rowlen <= 64
  for (int i = tid; i < 2 * UP_TS * rowlen; i += 256) {
    const int Yl = (int)(((unsigned)i * mRow) >> 16), rem = i - Yl * rowlen;
    const int Xl = (int)(((unsigned)rem * mCB) >> 16), cb = rem - Xl * CB;
    const int Y = 2 * y0 + Yl, X = 2 * x0 + Xl;
    if (Y >= Hb || X >= Hb) continue;
    const long long o = ((sample * Hb + Y) * Hb + X) * CB + cb;
    const int q = (Yl >> 1) * UP_TS + (Xl >> 1), col = ((Yl & 1) * 2 + (Xl & 1)) * CB + cb;
    float v = (ep[q * NC + col] + ep[(64 + q) * NC + col]) + (ep[(128 + q) * NC + col] + ep[(192 + q) * NC + col]);
    if (a.mode == 1) v = tanhf(v + a.bias[(long long)l * a.bias_stride + cb]);
    else if (a.mode == 2) { const float yv = to_float(aux[o]); v *= (1.f - yv * yv); }
    out[o] = from_float<T>(v);
  }
}
template <typename T> void launch_up_img(const UpImgArgs& a, hipStream_t st) {
  if (a.n == 0) return;
  if (!a.feat || !a.w || !a.out || a.CB < 1 || a.CB > 4 || (a.Cs != 64 && a.Cs != 128) || (a.mode == 1 && !a.bias) || (a.mode == 2 && !a.aux))
    return launch_fail("image-side transposed convolution: null operand, more than 4 image channels, or feature channels other than 64 / 128");
  const int tiles = (a.Hs + UP_TS - 1) / UP_TS;
  const int rowB = a.Cs * (int)sizeof(T) + 16;
  const size_t lds = (size_t)(UP_HALO * UP_HALO + 16 * a.CB) * rowB;
  if (lds > 160 * 1024) return launch_fail("image-side transposed convolution: tile does not fit the LDS");
  if (a.Cs == 64) {
    hipLaunchKernelGGL((up_img_kernel<T, 64>), dim3(tiles * tiles, a.n), dim3(256), lds, st, a);
  } else if (a.Cs == 128) {
    if (lds > 48 * 1024)   // above the default dynamic limit: ask for it (idempotent, cheap)
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&up_img_kernel<T, 128>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)lds);
    hipLaunchKernelGGL((up_img_kernel<T, 128>), dim3(tiles * tiles, a.n), dim3(256), lds, st, a);
  }
}
template void launch_up_img<float>(const UpImgArgs&, hipStream_t);
template void launch_up_img<bf16_t>(const UpImgArgs&, hipStream_t);

}  // namespace gan
