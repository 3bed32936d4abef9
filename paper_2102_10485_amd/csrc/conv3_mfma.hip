// G's last layer of the networks as the paper's Table 1 prints them: Conv k3 s1 p1 from Cin (64 or 128) feature
// channels onto the 1-4 image channels, + bias, tanh -- and its two gradients.  With so few output channels the layer
// does not fit the grouped GEMM engine's tiles, but it is still a contraction, and direct loops over it were bound by
// their vector instructions (4.9 ms of a 15.7 ms step).  Three small MFMA kernels on 8 x 8 pixel patches:
//   forward : R[halo pixel][(tap, co)] = sum_ci F[halo pixel][ci] w[tap][co][ci] for the patch with its one-pixel halo
//             (rows = the 100 halo pixels, 32 per wave; columns = the 9 CO pairs; K = the feature channels), then every
//             output pixel adds the nine entries its neighbours hold for it.
//   dgrad   : din[p][ci] = sum_{tap, co} P[p][(tap, co)] * w[tap][co][ci] with P[p][(ky, kx, co)] =
//             dout[p - (ky - 1, kx - 1)][co]: rows = pixels, K = 9 CO (padded to whole MFMA steps), columns = Cin.
//   wgrad   : dw[(tap, co)][ci] = sum_p P[p][(tap, co)] * in[p][ci]: K = pixels, the slow index of both operands in
//             memory.  bf16: the feature tile goes to LDS as it is and the transposing LDS read delivers it pixel-fastest,
//             P is read element by element out of the dout halo tile.  fp32 (no 32-bit transposing read): both operands
//             are written to LDS pixel-fastest.  A block walks the patches of its share of a model's samples, each wave
//             taking a quarter of every patch's pixels, and the waves' sums are added in order at the end.
// Storage type T on the MFMA inputs (bf16: v_mfma_f32_32x32x16_bf16, fp32: v_mfma_f32_32x32x2_f32), fp32 sums; the
// fp32 master weights are rounded to T on their way into LDS, as every other layer's weights are in their storage copy.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "kernels.h"

namespace gan {

typedef float c3_f16 __attribute__((ext_vector_type(16)));
typedef __bf16 c3_bf8 __attribute__((ext_vector_type(8)));

// one MFMA step over 32 bytes of K per row (16 per lane half): 16 bf16 or 8 floats
__device__ inline void c3_mma(c3_f16& acc, const uint4& a, const uint4& b, bf16_t) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(c3_bf8, a), __builtin_bit_cast(c3_bf8, b), acc, 0, 0, 0);
}
__device__ inline void c3_mma(c3_f16& acc, const uint4& a, const uint4& b, float) {
  // four k-pairs; lane half h supplies k = 4h + j to MFMA j, for A and B alike
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
}
// row of an accumulator element: MFMA 32 x 32 output, element e of lane (r = lane % 32, h = lane / 32) is row
// (e / 4) * 8 + h * 4 + e % 4 of column r
__device__ inline int c3_acc_row(int e, int h) { return (e >> 2) * 8 + h * 4 + (e & 3); }

constexpr int C3_TS = 8;                 // patch side
constexpr int C3_HALO = C3_TS + 2;
constexpr int C3_MAXCO = 4;
constexpr int C3_MAX_SPLITS = 32;

// ---- forward -----------------------------------------------------------------------------------------------------
// One block per sample: the model's weights go into LDS once, then the sample's patches one after the other, the next
// patch's halo tile on its way (in registers) while the current one is multiplied.  Per patch one product
// R[halo pixel][(tap, co)] = sum_ci F[halo pixel][ci] w[tap][co][ci] over all feature channels -- each wave takes 32
// of the 100 halo pixels, so no sums cross waves -- left in LDS transposed; an output pixel then adds its nine
// neighbours' entries, one per tap.  (Multiplying per output pixel instead, with K = (neighbour, channel), needs 4.5
// times the MFMAs for the same result and was bound by them and by the partial sums' way through LDS.)
constexpr int C3_RTS = 128 * 4 + 16;     // bytes per row of the transposed product: 128 halo-pixel slots of fp32
template <typename T, int CIN>
__global__ __launch_bounds__(256) void conv3_fwd_kernel(Conv3Args a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  constexpr int SZ = (int)sizeof(T);
  constexpr int rowB = CIN * SZ + 16;                          // bytes per pixel / weight row in LDS
  constexpr int cpr = CIN * SZ / 16;                           // 16-byte chunks per row
  const int H = a.H, CO = a.CO;
  const int nct = 9 * CO > 32 ? 2 : 1;                         // column tiles of (tap, co)
  unsigned char* Fl = lds;                                     // [C3_HALO * C3_HALO][rowB]
  unsigned char* Wl = lds + C3_HALO * C3_HALO * rowB;          // [32 nct][rowB], rows from 9 CO on are zero
  unsigned char* RT = Wl + 32 * nct * rowB;                    // [32 nct][C3_RTS]
  // (the fourth wave's row tile runs over the end of Fl into Wl: finite values, whose products nobody reads)
  const int j = blockIdx.x;
  if (j >= a.offs[a.L]) return;
  const int l = a.sample_model[j];
  const int tiles = (H + C3_TS - 1) / C3_TS;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const T* in = static_cast<const T*>(a.in) + (long long)j * H * H * CIN;
  T* out = static_cast<T*>(a.out) + ((long long)a.out_seg * a.seg_samples + j) * H * H * CO;
  constexpr int NF = (C3_HALO * C3_HALO * cpr + 255) / 256;
  uint4 fv[NF];
  auto fetch = [&](int tile) {
    const int y0 = (tile / tiles) * C3_TS, x0 = (tile % tiles) * C3_TS;
#pragma unroll
    for (int k = 0; k < NF; ++k) {
      const int i = tid + 256 * k;
      const int hr = i / cpr, ch = i - hr * cpr;
      const int y = y0 - 1 + hr / C3_HALO, x = x0 - 1 + hr % C3_HALO;
      fv[k] = make_uint4(0, 0, 0, 0);
      if (i < C3_HALO * C3_HALO * cpr && (unsigned)y < (unsigned)H && (unsigned)x < (unsigned)H)
        fv[k] = *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(in + ((long long)y * H + x) * CIN) + ch * 16);
    }
  };
  fetch(0);
  for (int i = tid; i < 32 * nct * rowB / 16; i += 256) reinterpret_cast<uint4*>(Wl)[i] = make_uint4(0, 0, 0, 0);
  __syncthreads();
  const float* w = a.w + (long long)l * a.w_stride;            // [9][CO][CIN] fp32
  for (int i = tid; i < 9 * CO * CIN; i += 256) {
    const int row = i / CIN, ci = i - row * CIN;
    *reinterpret_cast<T*>(Wl + row * rowB + ci * SZ) = from_float<T>(w[i]);
  }
  const int r = lane & 31, h = lane >> 5;
  constexpr int ksteps = CIN * SZ / 32;
  const unsigned char* arow = Fl + (wave * 32 + r) * rowB + h * 16;
  const unsigned char* bcol = Wl + r * rowB + h * 16;
  const unsigned mCO = 65536u / (unsigned)CO + 1u;             // i / CO for i < 256
  // the output element of this thread (one per thread: 64 CO <= 256) and where its nine terms lie in RT
  const int oq = (int)(((unsigned)tid * mCO) >> 16), oco = tid - oq * CO;
  const unsigned char* rsrc = RT + oco * C3_RTS + ((oq / C3_TS) * C3_HALO + oq % C3_TS) * 4;
  const float bias_o = tid < 64 * CO ? a.bias[(long long)l * a.bias_stride + oco] : 0.f;
  for (int tile = 0; tile < tiles * tiles; ++tile) {
    const int y0 = (tile / tiles) * C3_TS, x0 = (tile % tiles) * C3_TS;
    __syncthreads();                                           // the previous patch: multiplied and written out
#pragma unroll
    for (int k = 0; k < NF; ++k) {
      const int i = tid + 256 * k;
      const int hr = i / cpr, ch = i - hr * cpr;
      if (i < C3_HALO * C3_HALO * cpr) *reinterpret_cast<uint4*>(Fl + hr * rowB + ch * 16) = fv[k];
    }
    if (tile + 1 < tiles * tiles) fetch(tile + 1);
    __syncthreads();
    c3_f16 acc[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
#pragma unroll
    for (int ks = 0; ks < ksteps; ++ks) {
      const uint4 av = *reinterpret_cast<const uint4*>(arow + ks * 32);
#pragma unroll
      for (int t = 0; t < 2; ++t)
        if (t < nct) {
          const uint4 bv = *reinterpret_cast<const uint4*>(bcol + t * 32 * rowB + ks * 32);
          c3_mma(acc[t], av, bv, T());
        }
    }
    // element e of lane (r, h): halo pixel wave * 32 + (e / 4) * 8 + h * 4 + e % 4 of column r: four pixels per store
#pragma unroll
    for (int t = 0; t < 2; ++t)
      if (t < nct) {
#pragma unroll
        for (int g = 0; g < 4; ++g)
          *reinterpret_cast<float4*>(RT + (t * 32 + r) * C3_RTS + (wave * 32 + g * 8 + h * 4) * 4) =
              make_float4(acc[t][4 * g], acc[t][4 * g + 1], acc[t][4 * g + 2], acc[t][4 * g + 3]);
      }
    __syncthreads();
    if (tid < 64 * CO) {
      const int y = y0 + oq / C3_TS, x = x0 + oq % C3_TS;
      if (y < H && x < H) {
        // tap (ky, kx) reads pixel p + (ky - 1, kx - 1): halo position (qy + ky, qx + kx); taps added in order
        float v = 0.f;
#pragma unroll
        for (int tap = 0; tap < 9; ++tap)
          v += *reinterpret_cast<const float*>(rsrc + tap * CO * C3_RTS + ((tap / 3) * C3_HALO + tap % 3) * 4);
        out[((long long)y * H + x) * CO + oco] = from_float<T>(tanhf(v + bias_o));
      }
    }
  }
}

// ---- the gradient patch matrix shared by dgrad and wgrad ------------------------------------------------------------
// D: the 10 x 10 halo tile of dout around the patch, C3_MAXCO values of T per pixel (zeros outside the image)
template <typename T>
__device__ inline void c3_load_dout(const Conv3Args& a, const T* dout, int y0, int x0, T* D) {
  for (int t = threadIdx.x; t < C3_HALO * C3_HALO * C3_MAXCO; t += 256) {
    const int px = t >> 2, co = t & 3;
    const int y = y0 - 1 + px / C3_HALO, x = x0 - 1 + px % C3_HALO;
    T v = from_float<T>(0.f);
    if (co < a.CO && (unsigned)y < (unsigned)a.H && (unsigned)x < (unsigned)a.H) v = dout[((long long)y * a.H + x) * a.CO + co];
    D[t] = v;
  }
}
// P[(ky, kx, co)][pixel q of the patch] = dout at pixel q - (ky - 1, kx - 1) = halo position (qy - ky + 2, qx - kx + 2)
template <typename T>
__device__ inline T c3_patch_value(const T* D, int q, int tap, int co) {
  const int ky = tap / 3, kx = tap - ky * 3;
  return D[(((q >> 3) - ky + 2) * C3_HALO + ((q & 7) - kx + 2)) * C3_MAXCO + co];
}

// ---- data gradient ---------------------------------------------------------------------------------------------------
// One block per sample, the weights (transposed, rounded to T) in LDS once, the next patch's dout halo on its way while
// the current patch is multiplied.
template <typename T, int CIN>
__global__ __launch_bounds__(256) void conv3_dgrad_kernel(Conv3Args a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  constexpr int SZ = (int)sizeof(T);
  constexpr int KB = (9 * C3_MAXCO * SZ + 31) / 32 * 32;       // bytes of K per row, whole MFMA steps (for the widest CO)
  constexpr int prow = KB + 16;
  constexpr int orow = CIN * SZ + 16;
  T* D = reinterpret_cast<T*>(lds);                                            // [100][4]
  unsigned char* PA = lds + ((C3_HALO * C3_HALO * C3_MAXCO * SZ + 15) & ~15);  // [64 pixels][prow]
  unsigned char* WT = PA + 64 * prow;                                          // [CIN][prow]: w transposed, (tap, co) fastest
  unsigned char* OUT = WT + CIN * prow;                                        // [64 pixels][orow]
  const int j = blockIdx.x;
  if (j >= a.offs[a.L]) return;
  const int l = a.sample_model[j];
  const int H = a.H, CO = a.CO;
  const int tiles = (H + C3_TS - 1) / C3_TS;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const T* dout = static_cast<const T*>(a.dout) + ((long long)a.out_seg * a.seg_samples + j) * H * H * CO;
  T* din = static_cast<T*>(a.din) + (long long)j * H * H * CIN;
  constexpr int ND = (C3_HALO * C3_HALO * C3_MAXCO + 255) / 256;
  T dreg[ND];
  auto fetch = [&](int tile) {
    const int y0 = (tile / tiles) * C3_TS, x0 = (tile % tiles) * C3_TS;
#pragma unroll
    for (int k = 0; k < ND; ++k) {
      const int t = tid + 256 * k;
      const int px = t >> 2, co = t & 3;
      const int y = y0 - 1 + px / C3_HALO, x = x0 - 1 + px % C3_HALO;
      dreg[k] = from_float<T>(0.f);
      if (t < C3_HALO * C3_HALO * C3_MAXCO && co < CO && (unsigned)y < (unsigned)H && (unsigned)x < (unsigned)H)
        dreg[k] = dout[((long long)y * H + x) * CO + co];
    }
  };
  fetch(0);
  // zero the operand rows (K beyond 9 CO must multiply as zero), then the weights
  for (int t = tid; t < (64 + CIN) * prow / 16; t += 256) reinterpret_cast<uint4*>(PA)[t] = make_uint4(0, 0, 0, 0);
  __syncthreads();
  const float* w = a.w + (long long)l * a.w_stride;            // [9][CO][CIN]
  for (int i = tid; i < 9 * CO * CIN; i += 256) {
    const int k = i / CIN, ci = i - k * CIN;
    *reinterpret_cast<T*>(WT + ci * prow + k * SZ) = from_float<T>(w[i]);
  }
  // (row tile, column tile) pairs: 2 x CIN / 32, dealt to the four waves
  constexpr int NT = CIN / 32, PAIRS = 2 * NT / 4;
  static_assert(2 * NT % 4 == 0, "tile pairs per wave");
  const int r = lane & 31, h = lane >> 5;
  const int mt = wave & 1;
  const int ksteps = (9 * CO * SZ + 31) / 32;
  constexpr int cpr = CIN * SZ / 16;
  for (int tile = 0; tile < tiles * tiles; ++tile) {
    const int y0 = (tile / tiles) * C3_TS, x0 = (tile % tiles) * C3_TS;
    __syncthreads();                                           // the previous patch: multiplied and written out
#pragma unroll
    for (int k = 0; k < ND; ++k) {
      const int t = tid + 256 * k;
      if (t < C3_HALO * C3_HALO * C3_MAXCO) D[t] = dreg[k];
    }
    if (tile + 1 < tiles * tiles) fetch(tile + 1);
    __syncthreads();
    for (int i = tid; i < 64 * 9; i += 256) {
      const int tap = i >> 6, q = i & 63;
      for (int co = 0; co < CO; ++co) *reinterpret_cast<T*>(PA + q * prow + (tap * CO + co) * SZ) = c3_patch_value<T>(D, q, tap, co);
    }
    __syncthreads();
    c3_f16 acc[PAIRS];
#pragma unroll
    for (int i = 0; i < PAIRS; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    for (int ks = 0; ks < ksteps; ++ks) {
      const uint4 av = *reinterpret_cast<const uint4*>(PA + (mt * 32 + r) * prow + h * 16 + ks * 32);
#pragma unroll
      for (int i = 0; i < PAIRS; ++i) {
        const int nt = (wave >> 1) + 2 * i;
        const uint4 bv = *reinterpret_cast<const uint4*>(WT + (nt * 32 + r) * prow + h * 16 + ks * 32);
        c3_mma(acc[i], av, bv, T());
      }
    }
#pragma unroll
    for (int i = 0; i < PAIRS; ++i) {
      const int nt = (wave >> 1) + 2 * i;
#pragma unroll
      for (int e = 0; e < 16; ++e)
        *reinterpret_cast<T*>(OUT + (mt * 32 + c3_acc_row(e, h)) * orow + (nt * 32 + r) * SZ) = from_float<T>(acc[i][e]);
    }
    __syncthreads();
    for (int i = tid; i < 64 * cpr; i += 256) {
      const int q = i / cpr, ch = i - q * cpr;
      const int y = y0 + q / C3_TS, x = x0 + q % C3_TS;
      if (y >= H || x >= H) continue;
      *reinterpret_cast<uint4*>(reinterpret_cast<unsigned char*>(din + ((long long)y * H + x) * CIN) + ch * 16) =
          *reinterpret_cast<const uint4*>(OUT + q * orow + ch * 16);
    }
  }
}

// ---- weight gradient -------------------------------------------------------------------------------------------------
template <typename T, int CIN>
__global__ __launch_bounds__(256) void conv3_wgrad_kernel(Conv3Args a, float* __restrict__ part, int splits) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  constexpr int SZ = (int)sizeof(T);
  constexpr int krow = 64 * SZ + 16;                           // bytes per operand row: the patch's 64 pixels
  constexpr int MT = (9 * C3_MAXCO + 31) / 32;                 // row tiles of (tap, co): 2 (36 rows at CO = 4)
  constexpr int NT = CIN / 32;
  T* D = reinterpret_cast<T*>(lds);                                            // [100][4]
  unsigned char* PT = lds + ((C3_HALO * C3_HALO * C3_MAXCO * SZ + 15) & ~15);  // [MT * 32 rows (tap, co)][krow]
  unsigned char* IT = PT + MT * 32 * krow;                                     // [CIN][krow]: the feature tile, pixel fastest
  float* red = reinterpret_cast<float*>(PT);                                   // [MT * 32][CIN] sums over the waves, over the operands at the end
  const int l = blockIdx.y, split = blockIdx.x;
  const int s0 = a.offs[l], cnt = a.offs[l + 1] - s0;
  if (cnt == 0) return;
  const int H = a.H, CO = a.CO;
  const int tiles = (H + C3_TS - 1) / C3_TS;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r = lane & 31, h = lane >> 5;
  const int per = (cnt + splits - 1) / splits;
  const int n_lo = split * per, n_hi = min(cnt, n_lo + per);
  const int mtiles = 9 * CO > 32 ? 2 : 1;
  c3_f16 acc[MT][NT];
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int n = 0; n < NT; ++n)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[m][n][e] = 0.f;
  for (int t = tid; t < MT * 32 * krow / 16; t += 256) reinterpret_cast<uint4*>(PT)[t] = make_uint4(0, 0, 0, 0);   // rows beyond 9 CO stay zero
  constexpr int cpr = CIN * SZ / 16, EPV = 16 / SZ;
  constexpr int ksteps = 64 * SZ / 32, kpw = ksteps / 4;       // each wave takes a quarter of the patch's pixels
  static_assert(ksteps % 4 == 0, "pixels per wave");
  // The global loads of patch i + 1 (dout halo and feature tile, into registers) are issued before patch i is
  // multiplied: with three barriers and little arithmetic per patch the loop is otherwise a chain of load latencies.
  constexpr int ND = (C3_HALO * C3_HALO * C3_MAXCO + 255) / 256, NI = 64 * cpr / 256;
  static_assert(64 * cpr % 256 == 0, "feature tile chunks per thread");
  T dreg[ND];
  uint4 ireg[NI];
  const int per_sample = tiles * tiles, npatch = (n_hi - n_lo) * per_sample;
  auto fetch = [&](int idx) {
    const int n = n_lo + idx / per_sample, tile = idx % per_sample;
    const int y0 = (tile / tiles) * C3_TS, x0 = (tile % tiles) * C3_TS;
    const T* in = static_cast<const T*>(a.in) + (long long)(s0 + n) * H * H * CIN;
    const T* dout = static_cast<const T*>(a.dout) + ((long long)a.out_seg * a.seg_samples + s0 + n) * H * H * CO;
#pragma unroll
    for (int k = 0; k < ND; ++k) {
      const int t = tid + 256 * k;
      const int px = t >> 2, co = t & 3;
      const int y = y0 - 1 + px / C3_HALO, x = x0 - 1 + px % C3_HALO;
      dreg[k] = from_float<T>(0.f);
      if (t < C3_HALO * C3_HALO * C3_MAXCO && co < CO && (unsigned)y < (unsigned)H && (unsigned)x < (unsigned)H)
        dreg[k] = dout[((long long)y * H + x) * CO + co];
    }
    // a wave takes one 16-byte channel group of all 64 pixels: its lanes then write 64 consecutive elements of a
    // row of IT (rows a multiple of 16 bytes apart would all fall into one bank if a lane's neighbours held the
    // other channel groups of the same pixel); the tile's lines come out of the L1 for the other groups
#pragma unroll
    for (int k = 0; k < NI; ++k) {
      const int i = tid + 256 * k;
      const int ch = i >> 6, q = i & 63;
      const int y = y0 + q / C3_TS, x = x0 + q % C3_TS;
      ireg[k] = make_uint4(0, 0, 0, 0);
      if (y < H && x < H) ireg[k] = *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(in + ((long long)y * H + x) * CIN) + ch * 16);
    }
  };
  if (npatch > 0) fetch(0);
  for (int idx = 0; idx < npatch; ++idx) {
    __syncthreads();                                           // the previous patch has been multiplied
#pragma unroll
    for (int k = 0; k < ND; ++k) {
      const int t = tid + 256 * k;
      if (t < C3_HALO * C3_HALO * C3_MAXCO) D[t] = dreg[k];
    }
#pragma unroll
    for (int k = 0; k < NI; ++k) {
      const int i = tid + 256 * k;
      const int ch = i >> 6, q = i & 63;
      const T* e = reinterpret_cast<const T*>(&ireg[k]);
#pragma unroll
      for (int kk = 0; kk < EPV; ++kk) *reinterpret_cast<T*>(IT + (ch * EPV + kk) * krow + q * SZ) = e[kk];
    }
    if (idx + 1 < npatch) fetch(idx + 1);
    __syncthreads();
    for (int i = tid; i < 64 * 9; i += 256) {
      const int tap = i >> 6, q = i & 63;
      for (int co = 0; co < CO; ++co) *reinterpret_cast<T*>(PT + (tap * CO + co) * krow + q * SZ) = c3_patch_value<T>(D, q, tap, co);
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kpw; ++k) {
      const int koff = (wave * kpw + k) * 32 + h * 16;
      uint4 bv[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) bv[nt] = *reinterpret_cast<const uint4*>(IT + (nt * 32 + r) * krow + koff);
#pragma unroll
      for (int m = 0; m < MT; ++m) {
        if (m < mtiles) {
          const uint4 av = *reinterpret_cast<const uint4*>(PT + (m * 32 + r) * krow + koff);
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) c3_mma(acc[m][nt], av, bv[nt], T());
        }
      }
    }
  }
  // the four waves' sums, added in wave order
  for (int wv = 0; wv < 4; ++wv) {
    __syncthreads();
    if (wave == wv) {
#pragma unroll
      for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            float* dst = red + (m * 32 + c3_acc_row(e, h)) * CIN + nt * 32 + r;
            *dst = wv == 0 ? acc[m][nt][e] : *dst + acc[m][nt][e];
          }
    }
  }
  __syncthreads();
  for (int e = tid; e < 9 * CO * CIN; e += 256) part[((long long)split * a.L + l) * 9 * CO * CIN + e] = red[e];
}
// bf16 storage: the same sums without the transposed copies.  The feature tile stays in LDS as it lies in memory
// ([pixel][channel], 16-byte writes) and ds_read_b64_tr_b16 transposes it on the way to the MFMA operand: within a
// block of 16 lanes, lane i receives element i % 4 of the 8-byte groups addressed by lanes i / 4 + {0, 4, 8, 12}, so
// pointing lane s at pixel s / 4, channel group s % 4 hands lane i four consecutive pixels of channel i.  The other
// operand, P[(tap, co)][pixel] = dout[pixel - (ky - 1, kx - 1)][co], is read straight out of the dout halo tile: eight
// consecutive pixels of a patch row are eight 2-byte reads at fixed offsets from a per-lane base that never changes.
// Two barriers per patch instead of three, no scattered LDS writes.
typedef short c3_short4 __attribute__((ext_vector_type(4)));
__device__ inline uint2 c3_read_tr16(const unsigned char* p) {
  const c3_short4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) c3_short4*)(p));
  return __builtin_bit_cast(uint2, v);
}
template <int CIN>
__global__ __launch_bounds__(256) void conv3_wgrad_tr_kernel(Conv3Args a, float* __restrict__ part, int splits) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  typedef bf16_t T;
  constexpr int SZ = 2;
  constexpr int rowB = CIN * SZ + 16;                          // bytes per pixel row of the feature tile
  constexpr int MT = (9 * C3_MAXCO + 31) / 32;                 // row tiles of (tap, co)
  constexpr int NT = CIN / 32;
  constexpr int DBYTES = (C3_HALO * C3_HALO * C3_MAXCO * SZ + 15) & ~15;
  T* D = reinterpret_cast<T*>(lds);                            // [100][4]
  unsigned char* Fq = lds + DBYTES;                            // [64 pixels][rowB]
  float* red = reinterpret_cast<float*>(lds);                  // [MT * 32][CIN] sums over the waves, over the operands at the end
  const int l = blockIdx.y, split = blockIdx.x;
  const int s0 = a.offs[l], cnt = a.offs[l + 1] - s0;
  if (cnt == 0) return;
  const int H = a.H, CO = a.CO;
  const int tiles = (H + C3_TS - 1) / C3_TS;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r = lane & 31, h = lane >> 5;
  const int per = (cnt + splits - 1) / splits;
  const int n_lo = split * per, n_hi = min(cnt, n_lo + per);
  const int mtiles = 9 * CO > 32 ? 2 : 1;
  c3_f16 acc[MT][NT];
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int n = 0; n < NT; ++n)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[m][n][e] = 0.f;
  // a wave takes the patch rows 2 wave and 2 wave + 1 (one K-step of 16 pixels), lane half h the row 2 wave + h
  const unsigned short* dsrc[MT];
  bool rowok[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    const int rr = m * 32 + r;
    rowok[m] = rr < 9 * CO;
    const int tap = rowok[m] ? rr / CO : 0, co = rowok[m] ? rr - tap * CO : 0;
    const int ky = tap / 3, kx = tap - ky * 3;
    dsrc[m] = reinterpret_cast<const unsigned short*>(D) + (((2 * wave + h) - ky + 2) * C3_HALO + (2 - kx)) * C3_MAXCO + co;
  }
  const int s16 = lane & 15, hb = (lane >> 4) & 1;
  const unsigned char* fsrc = Fq + (wave * 16 + 8 * h + (s16 >> 2)) * rowB + (2 * hb + ((s16 & 3) >> 1)) * 16 + 8 * (s16 & 1);
  constexpr int cpr = CIN * SZ / 16;
  constexpr int ND = (C3_HALO * C3_HALO * C3_MAXCO + 255) / 256, NI = 64 * cpr / 256;
  static_assert(64 * cpr % 256 == 0, "feature tile chunks per thread");
  T dreg[ND];
  uint4 ireg[NI];
  const int per_sample = tiles * tiles, npatch = (n_hi - n_lo) * per_sample;
  auto fetch = [&](int idx) {
    const int n = n_lo + idx / per_sample, tile = idx % per_sample;
    const int y0 = (tile / tiles) * C3_TS, x0 = (tile % tiles) * C3_TS;
    const T* in = static_cast<const T*>(a.in) + (long long)(s0 + n) * H * H * CIN;
    const T* dout = static_cast<const T*>(a.dout) + ((long long)a.out_seg * a.seg_samples + s0 + n) * H * H * CO;
#pragma unroll
    for (int k = 0; k < ND; ++k) {
      const int t = tid + 256 * k;
      const int px = t >> 2, co = t & 3;
      const int y = y0 - 1 + px / C3_HALO, x = x0 - 1 + px % C3_HALO;
      dreg[k] = from_float<T>(0.f);
      if (t < C3_HALO * C3_HALO * C3_MAXCO && co < CO && (unsigned)y < (unsigned)H && (unsigned)x < (unsigned)H)
        dreg[k] = dout[((long long)y * H + x) * CO + co];
    }
#pragma unroll
    for (int k = 0; k < NI; ++k) {
      const int i = tid + 256 * k;
      const int q = i / cpr, ch = i - q * cpr;
      const int y = y0 + q / C3_TS, x = x0 + q % C3_TS;
      ireg[k] = make_uint4(0, 0, 0, 0);
      if (y < H && x < H) ireg[k] = *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(in + ((long long)y * H + x) * CIN) + ch * 16);
    }
  };
  if (npatch > 0) fetch(0);
  for (int idx = 0; idx < npatch; ++idx) {
    __syncthreads();                                           // the previous patch has been multiplied
#pragma unroll
    for (int k = 0; k < ND; ++k) {
      const int t = tid + 256 * k;
      if (t < C3_HALO * C3_HALO * C3_MAXCO) D[t] = dreg[k];
    }
#pragma unroll
    for (int k = 0; k < NI; ++k) {
      const int i = tid + 256 * k;
      const int q = i / cpr, ch = i - q * cpr;
      *reinterpret_cast<uint4*>(Fq + q * rowB + ch * 16) = ireg[k];
    }
    if (idx + 1 < npatch) fetch(idx + 1);
    __syncthreads();
    uint4 bv[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const uint2 lo = c3_read_tr16(fsrc + nt * 64), hi = c3_read_tr16(fsrc + nt * 64 + 4 * rowB);
      bv[nt] = make_uint4(lo.x, lo.y, hi.x, hi.y);
    }
#pragma unroll
    for (int m = 0; m < MT; ++m) {
      if (m < mtiles) {
        unsigned v[8];
#pragma unroll
        for (int qx = 0; qx < 8; ++qx) v[qx] = rowok[m] ? (unsigned)dsrc[m][qx * C3_MAXCO] : 0u;
        const uint4 av = make_uint4(v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16));
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) c3_mma(acc[m][nt], av, bv[nt], T());
      }
    }
  }
  // the four waves' sums, added in wave order
  for (int wv = 0; wv < 4; ++wv) {
    __syncthreads();
    if (wave == wv) {
#pragma unroll
      for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            float* dst = red + (m * 32 + c3_acc_row(e, h)) * CIN + nt * 32 + r;
            *dst = wv == 0 ? acc[m][nt][e] : *dst + acc[m][nt][e];
          }
    }
  }
  __syncthreads();
  for (int e = tid; e < 9 * CO * CIN; e += 256) part[((long long)split * a.L + l) * 9 * CO * CIN + e] = red[e];
}
__global__ void conv3_wgrad_final_kernel(Conv3Args a, const float* __restrict__ part, float* __restrict__ dw, long long dw_stride,
                                         int splits) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const int per = 9 * a.CO * a.Cin;
  if (idx >= (long long)a.L * per) return;
  const int l = (int)(idx / per), e = (int)(idx - (long long)l * per);
  if (a.offs[l + 1] == a.offs[l]) return;
  float s = 0.f;
#pragma unroll 8
  for (int k = 0; k < splits; ++k) s += part[((long long)k * a.L + l) * per + e];
  dw[(long long)l * dw_stride + e] = s;
}
// row splits per model of the weight gradient: enough blocks to fill the chip, a function of the model count only
int conv3_wgrad_splits(int L) { return min(max((2048 + L - 1) / L, 1), C3_MAX_SPLITS); }

static bool conv3_ok(const Conv3Args& a) {
  return a.CO >= 1 && a.CO <= C3_MAXCO && (a.Cin == 64 || a.Cin == 128) && a.H >= 1 && a.H <= 64 && a.w && a.offs && a.sample_model;
}
template <typename K> static void c3_allow_lds(K kernel, size_t lds) {
  if (lds > 48 * 1024)   // above the default dynamic limit: ask for it (idempotent, cheap)
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
}
template <typename T> void launch_conv3_fwd(const Conv3Args& a, hipStream_t st) {
  if (a.n == 0) return;
  if (!conv3_ok(a) || !a.in || !a.out || !a.bias) return launch_fail("image-side k3 convolution: unsupported shape or null operand");
  const int nct = 9 * a.CO > 32 ? 2 : 1;
  const size_t lds = (size_t)(C3_HALO * C3_HALO + 32 * nct) * (a.Cin * sizeof(T) + 16) + (size_t)32 * nct * C3_RTS;
  const dim3 grid(a.n);
  if (a.Cin == 64) { c3_allow_lds(&conv3_fwd_kernel<T, 64>, lds); hipLaunchKernelGGL((conv3_fwd_kernel<T, 64>), grid, dim3(256), lds, st, a); }
  else { c3_allow_lds(&conv3_fwd_kernel<T, 128>, lds); hipLaunchKernelGGL((conv3_fwd_kernel<T, 128>), grid, dim3(256), lds, st, a); }
}
template <typename T> void launch_conv3_dgrad(const Conv3Args& a, hipStream_t st) {
  if (a.n == 0) return;
  if (!conv3_ok(a) || !a.dout || !a.din) return launch_fail("image-side k3 convolution: unsupported shape or null operand");
  const int SZ = (int)sizeof(T);
  const size_t prow = (size_t)(9 * C3_MAXCO * SZ + 31) / 32 * 32 + 16;
  const size_t lds = (size_t)((C3_HALO * C3_HALO * C3_MAXCO * SZ + 15) & ~15) + (64 + a.Cin) * prow + (size_t)64 * (a.Cin * SZ + 16);
  const dim3 grid(a.n);
  if (a.Cin == 64) { c3_allow_lds(&conv3_dgrad_kernel<T, 64>, lds); hipLaunchKernelGGL((conv3_dgrad_kernel<T, 64>), grid, dim3(256), lds, st, a); }
  else { c3_allow_lds(&conv3_dgrad_kernel<T, 128>, lds); hipLaunchKernelGGL((conv3_dgrad_kernel<T, 128>), grid, dim3(256), lds, st, a); }
}
template <typename T> void launch_conv3_wgrad(const Conv3Args& a, float* part, float* dw, long long dw_stride, hipStream_t st) {
  if (a.n == 0) return;
  if (!conv3_ok(a) || !a.dout || !a.in || !part || !dw) return launch_fail("image-side k3 convolution: unsupported shape or null operand");
  const int splits = conv3_wgrad_splits(a.L);
  const int SZ = (int)sizeof(T);
  const size_t krow = (size_t)64 * SZ + 16;
  const int MT = (9 * C3_MAXCO + 31) / 32;
  const size_t lds = (size_t)((C3_HALO * C3_HALO * C3_MAXCO * SZ + 15) & ~15) + std::max((MT * 32 + a.Cin) * krow, (size_t)MT * 32 * a.Cin * 4);
  const dim3 grid(splits, a.L);
  if constexpr (sizeof(T) == 2) {
    const size_t lds_tr = std::max((size_t)((C3_HALO * C3_HALO * C3_MAXCO * SZ + 15) & ~15) + (size_t)64 * (a.Cin * SZ + 16), (size_t)MT * 32 * a.Cin * 4);
    if (a.Cin == 64) { c3_allow_lds(&conv3_wgrad_tr_kernel<64>, lds_tr); hipLaunchKernelGGL((conv3_wgrad_tr_kernel<64>), grid, dim3(256), lds_tr, st, a, part, splits); }
    else { c3_allow_lds(&conv3_wgrad_tr_kernel<128>, lds_tr); hipLaunchKernelGGL((conv3_wgrad_tr_kernel<128>), grid, dim3(256), lds_tr, st, a, part, splits); }
  } else {
    if (a.Cin == 64) { c3_allow_lds(&conv3_wgrad_kernel<T, 64>, lds); hipLaunchKernelGGL((conv3_wgrad_kernel<T, 64>), grid, dim3(256), lds, st, a, part, splits); }
    else { c3_allow_lds(&conv3_wgrad_kernel<T, 128>, lds); hipLaunchKernelGGL((conv3_wgrad_kernel<T, 128>), grid, dim3(256), lds, st, a, part, splits); }
  }
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
