// Grouped implicit-GEMM engine on MFMA for the k4 s2 p1 (transposed) convolutions and the linear layers of all
// per-label models at once.  One launch covers every model (Eq. 5 of the paper makes them independent, so the
// "batch of small GEMMs" is a single grid): an M-tile never crosses a model boundary, and each tile reads its
// own model's weights.
//
// Forward-type kernel (conv_gemm_kernel): C[row][n] = sum_{tap, c} A(row, tap)[c] * W[tap][n][c]
//   down : rows are output pixels of the small tensor, 16 taps gathered from the big tensor at (2y-1+ky, 2x-1+kx)
//   up   : rows are the pixels of one output phase (Y%2, X%2) of the big tensor, 4 taps gathered from the small one
//   dense: one tap, rows are samples (linear layer)
// Weight-gradient kernel (wgrad_kernel): dW[tap][cb][cs] = sum_rows Big(row, tap)[cb] * Small(row)[cs]; the
//   reduction index is the slow memory index of both operands, so tiles are transposed in registers on their
//   way into LDS.
//
// Both stage 128-byte K-rows in LDS (row stride 144 bytes) and feed v_mfma_f32_32x32x16_bf16 (bf16 storage) or
// v_mfma_f32_32x32x2_f32 (fp32 storage) from 16-byte LDS reads; accumulation is fp32 in both cases.
#include <stdlib.h>

#include "common.h"

namespace gan {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int BM = 128;          // tile rows
constexpr int BN = 128;          // tile columns
constexpr int BKB = 128;         // bytes of K per LDS row
constexpr int LDS_STRIDE = BKB + 16;
constexpr int NTHREADS = 256;    // 4 waves as 2 x 2, each 64 x 64 of the tile

int conv_tile_m() { return BM; }

__device__ inline void mma16B(floatx16& acc, const uint4& a, const uint4& b, bf16_t) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
}
__device__ inline void mma16B(floatx16& acc, const uint4& a, const uint4& b, float) {
  // four k-pairs; lane half h supplies k = 4h + j to MFMA j, for A and B alike
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
}

// One K-chunk held in LDS: every wave multiplies its (TM*32) x (TN*32) sub-tile.
template <typename T, int TM, int TN>
__device__ inline void tile_mma(floatx16 (&acc)[TM][TN], const unsigned char* As, const unsigned char* Bs, int wm, int wn,
                                int lane) {
  const int r = lane & 31, h = lane >> 5;
#pragma unroll
  for (int vs = 0; vs < BKB / 32; ++vs) {
    uint4 a[TM], b[TN];
#pragma unroll
    for (int t = 0; t < TM; ++t)
      a[t] = *reinterpret_cast<const uint4*>(As + (wm * TM * 32 + t * 32 + r) * LDS_STRIDE + (vs * 2 + h) * 16);
#pragma unroll
    for (int t = 0; t < TN; ++t)
      b[t] = *reinterpret_cast<const uint4*>(Bs + (wn * TN * 32 + t * 32 + r) * LDS_STRIDE + (vs * 2 + h) * 16);
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
      for (int tn = 0; tn < TN; ++tn) mma16B(acc[tm][tn], a[tm], b[tn], T());
  }
}

__device__ inline void store_out(float* p, float v) { *p = v; }
__device__ inline void store_out(bf16_t* p, float v) { *p = from_float<bf16_t>(v); }

// BN_ = 128: waves 2 x 2, each 64 x 64.  BN_ = 32 (image-side outputs, N <= 32): waves 4 x 1, each 32 x 32.
template <typename T, int MODE, int EPI, int BN_>
__global__ __launch_bounds__(NTHREADS) void conv_gemm_kernel(ConvArgs p) {
  constexpr int WN = BN_ == 128 ? 2 : 1, WM = 4 / WN;
  constexpr int TM = BM / (WM * 32), TN = BN_ / (WN * 32);
  __shared__ __attribute__((aligned(16))) unsigned char As[BM * LDS_STRIDE];
  __shared__ __attribute__((aligned(16))) unsigned char Bs[BN_ * LDS_STRIDE];
  constexpr int BK = BKB / (int)sizeof(T);
  constexpr int EPV = 16 / (int)sizeof(T);
  constexpr int BN = BN_;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;

  // ---- which tile: consecutive virtual ids stay on one XCD (block ids are dealt round-robin to the 8 XCDs)
  const int NT = (p.N + BN - 1) / BN;
  const int Ttot = p.tpre[p.L];
  const int total = Ttot * NT;
  const int per_xcd = (total + 7) >> 3;
  const int slot = blockIdx.x >> 3;
  if (slot >= per_xcd) return;
  const int v = (blockIdx.x & 7) * per_xcd + slot;
  if (v >= total) return;
  const int mt = v / NT, nt = v - mt * NT;
  int lo = 0, hi = p.L;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (p.tpre[mid] <= mt) lo = mid; else hi = mid;
  }
  const int l = lo;
  const int seg = p.seg_first + blockIdx.y;
  const int s0 = p.offs[l], s1 = p.offs[l + 1];
  const int Hr = p.Hr, Hin = p.Hin, C = p.C, N = p.N;
  const int rps = Hr * Hr;
  const int Mrows = (s1 - s0) * rps;
  const int m0 = (mt - p.tpre[l]) * BM;
  const long long sample_base = (long long)seg * p.seg_samples + s0;
  const int py = (MODE == MODE_UP) ? (int)(blockIdx.z >> 1) : 0;
  const int px = (MODE == MODE_UP) ? (int)(blockIdx.z & 1) : 0;

  const T* __restrict__ A = static_cast<const T*>(p.A);
  const T* __restrict__ W = static_cast<const T*>(p.W) + (long long)l * p.w_stride;

  // ---- per-thread load assignment: 16-byte chunk (tid % 8) of rows tid/8 + 32 i
  const int chunk = tid & 7;
  const int row0 = tid >> 3;
  long long abase[4];
  int aby[4], abx[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = m0 + row0 + 32 * i;
    if (r < Mrows) {
      if (MODE == MODE_DENSE) {               // rows are read directly: one "tap" at (0, 0) of a 1 x 1 map
        abase[i] = (sample_base * rps + r) * (long long)C;
        aby[i] = 0;
        abx[i] = 0;
      } else {
        const int n = r / rps, rem = r - n * rps;
        const int y = rem / Hr, x = rem - y * Hr;
        abase[i] = (sample_base + n) * (long long)(Hin * Hin) * C;
        aby[i] = (MODE == MODE_DOWN) ? 2 * y - 1 : y;
        abx[i] = (MODE == MODE_DOWN) ? 2 * x - 1 : x;
      }
    } else {
      abase[i] = 0;
      aby[i] = -100000;   // never in range
      abx[i] = -100000;
    }
  }

  const int ntaps = (MODE == MODE_DOWN) ? 16 : (MODE == MODE_UP ? 4 : 1);
  const int nk = ntaps * C / BK;

  const int wns = p.w_nstride;   // rows per tap in the weight block (N, or more when only some rows are used)
  uint4 ra[4], rb[BN / 32];
  auto load_chunk = [&](int kc) {
    const int kk = kc * BK;
    const int tap = kk / C;
    const int c0 = kk - tap * C + chunk * EPV;
    int dy, dx, wtap;
    if (MODE == MODE_DOWN) {
      dy = tap >> 2; dx = tap & 3; wtap = tap;
    } else if (MODE == MODE_UP) {
      const int a = tap >> 1, b = tap & 1;
      dy = py == 0 ? (a == 0 ? 0 : -1) : (a == 0 ? 1 : 0);
      dx = px == 0 ? (b == 0 ? 0 : -1) : (b == 0 ? 1 : 0);
      const int ky = py == 0 ? (a == 0 ? 1 : 3) : (a == 0 ? 0 : 2);
      const int kx = px == 0 ? (b == 0 ? 1 : 3) : (b == 0 ? 0 : 2);
      wtap = ky * 4 + kx;
    } else {
      dy = 0; dx = 0; wtap = 0;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int iy = aby[i] + dy, ix = abx[i] + dx;
      const bool ok = (unsigned)iy < (unsigned)Hin && (unsigned)ix < (unsigned)Hin;
      ra[i] = ok ? *reinterpret_cast<const uint4*>(A + abase[i] + (long long)(iy * Hin + ix) * C + c0)
                 : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < BN / 32; ++i) {
      const int col = nt * BN + row0 + 32 * i;
      rb[i] = (col < N) ? *reinterpret_cast<const uint4*>(W + ((long long)wtap * wns + col) * C + c0)
                        : make_uint4(0, 0, 0, 0);
    }
  };
  auto store_chunk = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      *reinterpret_cast<uint4*>(As + (row0 + 32 * i) * LDS_STRIDE + chunk * 16) = ra[i];
#pragma unroll
    for (int i = 0; i < BN / 32; ++i)
      *reinterpret_cast<uint4*>(Bs + (row0 + 32 * i) * LDS_STRIDE + chunk * 16) = rb[i];
  };

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  load_chunk(0);
  store_chunk();
  __syncthreads();
  for (int kc = 0; kc < nk; ++kc) {
    if (kc + 1 < nk) load_chunk(kc + 1);          // global loads in flight while the MFMAs run
    tile_mma<T, TM, TN>(acc, As, Bs, wm, wn, lane);
    __syncthreads();
    if (kc + 1 < nk) {
      store_chunk();
      __syncthreads();
    }
  }

  // ---- epilogue: output row index of every tile row, through LDS (As is free now)
  long long* orow = reinterpret_cast<long long*>(As);
  if (tid < BM) {
    const int r = m0 + tid;
    long long o = -1;
    if (r < Mrows) {
      if (MODE == MODE_UP) {
        const int n = r / rps, rem = r - n * rps;
        const int y = rem / Hr, x = rem - y * Hr;
        const int Hb = 2 * Hr;
        o = ((sample_base + n) * Hb + (2 * y + py)) * Hb + (2 * x + px);
      } else {
        o = sample_base * rps + r;
      }
    }
    orow[tid] = o;
  }
  __syncthreads();
  T* __restrict__ Out = static_cast<T*>(p.Out);
  const T* __restrict__ Aux = static_cast<const T*>(p.Aux);
#pragma unroll
  for (int tm = 0; tm < TM; ++tm)
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
      const int col = nt * BN + wn * TN * 32 + tn * 32 + (lane & 31);
      if (col >= N) continue;
      float bias = 0.f;
      if (EPI == EPI_BIAS_TANH) bias = p.bias[(long long)l * p.bias_stride + col];
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int rr = wm * TM * 32 + tm * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
        const long long o = orow[rr];
        if (o < 0) continue;
        float val = acc[tm][tn][e];
        if (EPI == EPI_ACT_BWD) {                 // times the activation's derivative, from the saved output
          const float f = to_float(Aux[o * N + col]);
          val = f > 0.f ? val : val * p.slope;
        } else if (EPI == EPI_LRELU) {
          val = val > 0.f ? val : val * p.slope;
        } else if (EPI == EPI_BIAS_TANH) {
          val = tanhf(val + bias);
        } else if (EPI == EPI_TANH_BWD) {         // times 1 - y^2, y the saved tanh output
          const float y = to_float(Aux[o * N + col]);
          val *= (1.f - y * y);
        }
        store_out(Out + o * N + col, val);
      }
    }
}

template <typename T, int MODE, int EPI, int BN_>
static void launch_one(const ConvArgs& a, hipStream_t st) {
  const int NT = (a.N + BN_ - 1) / BN_;
  const long long blocks = ((long long)a.ub_tiles * NT + 7) / 8 * 8;
  if (blocks == 0 || a.nseg == 0) return;
  dim3 grid((unsigned)blocks, (unsigned)a.nseg, MODE == MODE_UP ? 4 : 1);
  hipLaunchKernelGGL((conv_gemm_kernel<T, MODE, EPI, BN_>), grid, dim3(NTHREADS), 0, st, a);
}

// The (mode, epilogue, tile) combinations the networks use.
template <typename T>
void launch_conv(int mode, int epi, const ConvArgs& a, hipStream_t st) {
  // the kernel's assumptions, checked before anything is launched
  if (!a.A || !a.W || !a.Out || !a.offs || !a.tpre || a.N < 1 || a.w_nstride < a.N || a.C % (BKB / (int)sizeof(T)) != 0 ||
      ((epi == EPI_ACT_BWD || epi == EPI_TANH_BWD) && !a.Aux) || (epi == EPI_BIAS_TANH && !a.bias))
    abort();
  const bool narrow = a.N <= 32;
  if (mode == MODE_DOWN && epi == EPI_NONE && !narrow) return launch_one<T, MODE_DOWN, EPI_NONE, 128>(a, st);
  if (mode == MODE_UP && epi == EPI_NONE && !narrow) return launch_one<T, MODE_UP, EPI_NONE, 128>(a, st);
  if (mode == MODE_UP && epi == EPI_ACT_BWD && !narrow) return launch_one<T, MODE_UP, EPI_ACT_BWD, 128>(a, st);
  if (mode == MODE_UP && epi == EPI_NONE && narrow) return launch_one<T, MODE_UP, EPI_NONE, 32>(a, st);
  if (mode == MODE_UP && epi == EPI_BIAS_TANH && narrow) return launch_one<T, MODE_UP, EPI_BIAS_TANH, 32>(a, st);
  if (mode == MODE_UP && epi == EPI_TANH_BWD && narrow) return launch_one<T, MODE_UP, EPI_TANH_BWD, 32>(a, st);
  if (mode == MODE_DENSE && epi == EPI_NONE && !narrow) return launch_one<T, MODE_DENSE, EPI_NONE, 128>(a, st);
  if (mode == MODE_DENSE && epi == EPI_LRELU && !narrow) return launch_one<T, MODE_DENSE, EPI_LRELU, 128>(a, st);
  abort();   // a combination no caller uses
}
template void launch_conv<float>(int, int, const ConvArgs&, hipStream_t);
template void launch_conv<bf16_t>(int, int, const ConvArgs&, hipStream_t);

// ---------------------------------------------------------------------------------------------------------
// weight gradient
// ---------------------------------------------------------------------------------------------------------

// 8 x 8 transpose of 16-bit values held as 8 rows of uint4 (in place).
__device__ inline void transpose8x8_b16(uint4 (&r)[8]) {
  unsigned in[8][4];
#pragma unroll
  for (int i = 0; i < 8; ++i) { in[i][0] = r[i].x; in[i][1] = r[i].y; in[i][2] = r[i].z; in[i][3] = r[i].w; }
  unsigned out[8][4];
#pragma unroll
  for (int j = 0; j < 8; ++j)        // output row j = input column j
#pragma unroll
    for (int q = 0; q < 4; ++q) {    // output dword q holds input rows 2q, 2q+1
      const unsigned a = in[2 * q][j >> 1], b = in[2 * q + 1][j >> 1];
      out[j][q] = (j & 1) ? ((a >> 16) | (b & 0xffff0000u)) : ((a & 0xffffu) | (b << 16));
    }
#pragma unroll
  for (int i = 0; i < 8; ++i) r[i] = make_uint4(out[i][0], out[i][1], out[i][2], out[i][3]);
}

template <typename T>
__global__ __launch_bounds__(NTHREADS) void wgrad_kernel(WgradArgs p) {
  __shared__ __attribute__((aligned(16))) unsigned char As[BM * LDS_STRIDE];
  __shared__ __attribute__((aligned(16))) unsigned char Bs[BN * LDS_STRIDE];
  constexpr int BKR = BKB / (int)sizeof(T);     // rows (reduction index) per chunk: 64 (bf16) or 32 (fp32)
  constexpr bool IS16 = sizeof(T) == 2;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  // ---- tile: all tiles of a model run on one XCD, models are dealt round-robin to XCDs
  const int Cb = p.Cb, Cs = p.Cs, Hs = p.Hs;
  const int Mtot = p.ntaps * Cb;
  const int MT = (Mtot + BM - 1) / BM, NT = (Cs + BN - 1) / BN;
  const int ntiles = MT * NT;
  const int bid = blockIdx.x;
  const int l = (bid / (8 * ntiles)) * 8 + (bid & 7);
  if (l >= p.L) return;
  const int tile = (bid >> 3) % ntiles;
  const int mt = tile / NT, nt = tile - mt * NT;
  const int s0 = p.offs[l], s1 = p.offs[l + 1];
  const int rps = Hs * Hs;
  const int R = (s1 - s0) * rps;
  const int Hb = (p.ntaps == 1) ? 1 : 2 * Hs;
  const T* __restrict__ Big = static_cast<const T*>(p.Big);
  const T* __restrict__ Small = static_cast<const T*>(p.Small);

  // ---- loader roles: waves 0-1 fill A^T (gathered big tensor), waves 2-3 fill B^T (small tensor)
  const bool roleA = wave < 2;
  const int t = tid & 127;
  // bf16: 16 channel groups of 8 x 8 row groups of 8 ; fp32: 32 channel groups of 4 x 4 row lanes, 8 rows each strided by 4
  const int cg = IS16 ? (t & 15) : (t & 31);
  const int rg = IS16 ? (t >> 4) : (t >> 5);
  constexpr int EPV = 16 / (int)sizeof(T);
  int ch, ky = 1, kx = 1;
  bool chan_ok = true;
  if (roleA) {
    const int m = mt * BM + cg * EPV;
    chan_ok = m < Mtot;
    const int tap = m / Cb;
    ch = m - tap * Cb;
    if (p.ntaps != 1) { ky = tap >> 2; kx = tap & 3; }
  } else {
    ch = nt * BN + cg * EPV;
    chan_ok = ch < Cs;
  }

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  uint4 reg[8];
  for (int seg = 0; seg < p.nseg; ++seg) {
    const long long sample_base = (long long)seg * p.seg_samples + s0;
    for (int k0 = 0; k0 < R; k0 += BKR) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int r = k0 + (IS16 ? rg * 8 + j : rg + 4 * j);
        uint4 val = make_uint4(0, 0, 0, 0);
        if (r < R && chan_ok) {
          if (roleA && p.ntaps == 1) {           // rows of the big tensor are read directly
            val = *reinterpret_cast<const uint4*>(Big + (sample_base * rps + r) * (long long)Cb + ch);
          } else if (roleA) {
            const int n = r / rps, rem = r - n * rps;
            const int y = rem / Hs, x = rem - y * Hs;
            const int iy = 2 * y - 1 + ky, ix = 2 * x - 1 + kx;
            if ((unsigned)iy < (unsigned)Hb && (unsigned)ix < (unsigned)Hb)
              val = *reinterpret_cast<const uint4*>(Big + (((sample_base + n) * Hb + iy) * Hb + ix) * (long long)Cb + ch);
          } else {
            val = *reinterpret_cast<const uint4*>(Small + (sample_base * rps + r) * (long long)Cs + ch);
          }
        }
        reg[j] = val;
      }
      __syncthreads();                      // previous chunk's MFMAs are done with the LDS tiles
      unsigned char* dst = roleA ? As : Bs;
      if (IS16) {
        transpose8x8_b16(reg);
#pragma unroll
        for (int j = 0; j < 8; ++j)
          *reinterpret_cast<uint4*>(dst + (cg * 8 + j) * LDS_STRIDE + rg * 16) = reg[j];
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int kr = rg + 4 * j;
          unsigned* d0 = reinterpret_cast<unsigned*>(dst + (cg * 4) * LDS_STRIDE + kr * 4);
          d0[0] = reg[j].x;
          d0[LDS_STRIDE / 4] = reg[j].y;
          d0[2 * LDS_STRIDE / 4] = reg[j].z;
          d0[3 * LDS_STRIDE / 4] = reg[j].w;
        }
      }
      __syncthreads();
      tile_mma<T, 2, 2>(acc, As, Bs, wm, wn, lane);
    }
  }

  float* __restrict__ dW = p.dW + (long long)l * p.dw_stride;
#pragma unroll
  for (int tm = 0; tm < 2; ++tm)
#pragma unroll
    for (int tn = 0; tn < 2; ++tn) {
      const int col = nt * BN + wn * 64 + tn * 32 + (lane & 31);
      if (col >= Cs) continue;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = mt * BM + wm * 64 + tm * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
        if (m < Mtot) dW[(long long)m * Cs + col] = acc[tm][tn][e];
      }
    }
}

template <typename T>
void launch_wgrad(const WgradArgs& a, hipStream_t st) {
  if (!a.Big || !a.Small || !a.dW || !a.offs || a.Cb % 8 || a.Cs % 8 || (a.ntaps != 1 && a.ntaps != 16)) abort();
  const int MT = (a.ntaps * a.Cb + BM - 1) / BM, NT = (a.Cs + BN - 1) / BN;
  const long long blocks = (long long)((a.L + 7) / 8) * 8 * MT * NT;
  if (blocks == 0) return;
  hipLaunchKernelGGL((wgrad_kernel<T>), dim3((unsigned)blocks), dim3(NTHREADS), 0, st, a);
}
template void launch_wgrad<float>(const WgradArgs&, hipStream_t);
template void launch_wgrad<bf16_t>(const WgradArgs&, hipStream_t);

}  // namespace gan
