// Grouped implicit-GEMM engine on MFMA for the k4 s2 p1 (transposed) convolutions and the linear layers of all
// per-label models at once.  One launch covers every model (Eq. 5 of the paper makes them independent, so the
// "batch of small GEMMs" is a single grid): an M-tile never crosses a model boundary, and each tile reads its
// own model's weights.
//
// Forward-type kernel (conv_gemm_kernel): C[row][n] = sum_{tap, c} A(row, tap)[c] * W[tap][n][c]
//   down : rows are output pixels of the small tensor, 16 taps gathered from the big tensor at (2y-1+ky, 2x-1+kx)
//   up   : rows are the pixels of one output phase (Y%2, X%2) of the big tensor, 4 taps gathered from the small one
//   dense: one tap, rows are read directly (linear layer, patch-matrix layers)
// Weight-gradient kernel (wgrad_kernel): dW[tap][cb][cs] = sum_rows Big(row, tap)[cb] * Small(row)[cs]; the
//   reduction index is the slow memory index of both operands, so tiles are transposed in registers on their
//   way into LDS.
//
// Both stage 128-byte K-rows in LDS (two buffers) and feed v_mfma_f32_32x32x16_bf16 (bf16 storage) or
// v_mfma_f32_32x32x2_f32 (fp32 storage) from 16-byte LDS reads; accumulation is fp32 in both cases.
// Forward-type kernel: K-chunks of KB bytes per row travel global -> LDS directly (buffer_load_dwordx4 ... lds, no
// registers in between) into a ring of NST buffers while the MFMAs of the current chunk run.  The 256 x 256 tile uses
// KB = 128 with two buffers (one block per CU); the 256 x 128 and 128 x 128 tiles use KB = 64 with three, which leaves
// room for two blocks per CU so that one block's epilogue and barriers hide behind the other's MFMAs; the 256 x 64
// tile fits two blocks per CU with KB = 128 and two buffers.  The 16-byte chunk c of row
// R sits at position c ^ ((R / (256/KB)) % (KB/16)), which keeps both the 1 KiB-per-wave copies and the MFMA operand
// reads conflict-free.  Weight-gradient kernels: bf16 copies tiles in memory layout and transposes while reading LDS;
// fp32 goes global -> registers (transposes) -> LDS, row stride 144 bytes.
// One barrier per chunk in both.
#include <stdio.h>
#include <stdlib.h>

#include "common.h"
#include <type_traits>

namespace gan {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int BKB = 128;         // bytes of K per LDS row
constexpr int LDS_STRIDE = BKB + 16;

// Block tile BM x BN computed by WM x WN waves, each (TM*32) x (TN*32); forward kernel: KB bytes of K per LDS row,
// NST buffers.
template <int BM_, int BN_, int WM_, int WN_, int KB_ = 128, int NST_ = 2>
struct Tile {
  static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, KB = KB_, NST = NST_;
  static constexpr int NT = 64 * WM_ * WN_;
  static constexpr int TM = BM_ / (32 * WM_), TN = BN_ / (32 * WN_);
  static constexpr int CPR = KB_ / 16;               // 16-byte chunks per LDS row
  static constexpr int RPP = NT / CPR;               // tile rows filled per loader pass
  static constexpr int PA = BM_ / RPP, PB = BN_ / RPP;
};
typedef Tile<256, 256, 2, 4, 128, 2> TileBig;    // 512 threads, wave tile 128 x 64, 128 KiB of LDS
typedef Tile<256, 128, 4, 2, 64, 3> TileMid;     // 512 threads, wave tile 64 x 64, 72 KiB of LDS
typedef Tile<128, 128, 2, 2, 64, 3> TileSmall;   // 256 threads, wave tile 64 x 64 (few rows per model), 48 KiB of LDS
typedef Tile<256, 64, 4, 1, 128, 2> TileNarrow;  // 256 threads, wave tile 64 x 64, for layers with 64 output channels:
                                                 // 128-byte chunks, two buffers of 40 KiB, so two blocks still share a CU
typedef Tile<64, 64, 2, 2, 64, 3> TileTiny;      // 256 threads, wave tile 32 x 32, 24 KiB of LDS: workloads so small that
                                                 // the larger tiles would leave most of the chip without a block

int conv_tile_rows(int n_out, long long rows_per_model_hint, int n_models) {
  // fewer than 128 tiles of 256 rows x 128 columns in a launch of one segment: the chip has 256 units to fill
  if (rows_per_model_hint > 0 && n_models > 0) {
    const long long tiles = n_models * ((rows_per_model_hint + 255) / 256) * ((n_out + 127) / 128);
    if (tiles < 128) return TileTiny::BM;
  }
  if (rows_per_model_hint > 0 && rows_per_model_hint <= 128) return TileSmall::BM;
  return TileBig::BM;
}

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

// One K-chunk of the fp32 weight-gradient kernel held in LDS: every wave multiplies its (TM*32) x (TN*32) sub-tile.
// Rows 144 bytes apart, chunk c of tile row R at position (c + R/16) mod 8 (that kernel writes its tiles transposed,
// eight rows apart per lane; the rotation spreads those writes over the banks).
template <typename T, int TM, int TN>
__device__ inline void tile_mma(floatx16 (&acc)[TM][TN], const unsigned char* As, const unsigned char* Bs, int wm, int wn,
                                int lane) {
  const int r = lane & 31, h = lane >> 5;
  const int rot = r >> 4;        // tile rows start at multiples of 32, so R/16 = const + r/16
#pragma unroll
  for (int vs = 0; vs < BKB / 32; ++vs) {
    uint4 a[TM], b[TN];
#pragma unroll
    for (int t = 0; t < TM; ++t)
      a[t] = *reinterpret_cast<const uint4*>(As + (wm * TM * 32 + t * 32 + r) * LDS_STRIDE +
                                             ((vs * 2 + h + 2 * (wm * TM + t) + rot) & 7) * 16);
#pragma unroll
    for (int t = 0; t < TN; ++t)
      b[t] = *reinterpret_cast<const uint4*>(Bs + (wn * TN * 32 + t * 32 + r) * LDS_STRIDE +
                                             ((vs * 2 + h + 2 * (wn * TN + t) + rot) & 7) * 16);
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
      for (int tn = 0; tn < TN; ++tn) mma16B(acc[tm][tn], a[tm], b[tn], T());
  }
}

// One K-chunk of the forward-type kernel: rows KB bytes apart, the 16-byte chunk c of tile row R at position
// c ^ ((R / (256/KB)) % (KB/16)).  Sixteen lanes reading one chunk index of sixteen consecutive rows then touch
// sixteen different 16-byte slots of the 256-byte bank period, and so do the rows one wave-wide copy fills.
template <int KB>
__device__ inline int fwd_swz(int row) { return (row / (256 / KB)) % (KB / 16); }
// The operand reads of the forward-type kernel are issued by hand so that the reads of K-step vs+1 are in flight
// while the MFMAs of K-step vs run (two register sets).  The compiler does not count these reads, so the waits are
// explicit; each wait names the registers it makes valid, which orders the MFMAs behind it.
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
template <int OFF>
__device__ inline void lds_read16(u32x4& d, unsigned addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(d) : "v"(addr), "n"(OFF) : "memory");
}
template <int N, int TM, int TN>
__device__ inline void lds_wait(u32x4 (&a)[TM], u32x4 (&b)[TN]) {
  static_assert(TM <= 4 && TN <= 4, "operand list below");
  // at most N reads still in flight; all of a[] and b[] were issued before those
  if constexpr (TM == 4 && TN == 2)
    asm volatile("s_waitcnt lgkmcnt(%6)" : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(b[0]), "+v"(b[1]) : "n"(N) : "memory");
  else if constexpr (TM == 2 && TN == 2)
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a[0]), "+v"(a[1]), "+v"(b[0]), "+v"(b[1]) : "n"(N) : "memory");
  else if constexpr (TM == 1 && TN == 1)
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a[0]), "+v"(b[0]) : "n"(N) : "memory");
  else
    static_assert(TM == 4 && TN == 2, "add the operand list for this wave tile");
}
template <int I, int N, typename F>
__device__ inline void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}
template <typename T, int TM, int TN, int KB>
__device__ inline void tile_mma_fwd(floatx16 (&acc)[TM][TN], const unsigned char* As, const unsigned char* Bs, int wm, int wn,
                                    int lane) {
  const int r = lane & 31, h = lane >> 5;
  const int sw = fwd_swz<KB>(r);   // tile rows start at multiples of 32, a multiple of the swizzle period
  constexpr int NV = KB / 32;
  // LDS byte address of this lane's 16 bytes of K-step 0 in its first A / B row; K-step vs sits at the same
  // address with bit 5 .. flipped by vs (chunk index (2 vs + h) ^ sw = (2 vs) ^ (h ^ sw): no carries)
  const unsigned a0 = (unsigned)(uintptr_t)As + (wm * TM * 32 + r) * KB + ((h ^ sw) << 4);
  const unsigned b0 = (unsigned)(uintptr_t)Bs + (wn * TN * 32 + r) * KB + ((h ^ sw) << 4);
  u32x4 a[2][TM], b[2][TN];
  auto fetch = [&](auto vs, auto set) {
    const unsigned aa = a0 ^ (vs.value << 5), bb = b0 ^ (vs.value << 5);
    static_for<0, TM>([&](auto t) { lds_read16<t.value * 32 * KB>(a[set.value][t.value], aa); });
    static_for<0, TN>([&](auto t) { lds_read16<t.value * 32 * KB>(b[set.value][t.value], bb); });
  };
  fetch(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
  static_for<0, NV>([&](auto vs) {
    constexpr int cur = vs.value & 1;
    if constexpr (vs.value + 1 < NV) {
      fetch(std::integral_constant<int, vs.value + 1>{}, std::integral_constant<int, cur ^ 1>{});
      lds_wait<TM + TN>(a[cur], b[cur]);
    } else {
      lds_wait<0>(a[cur], b[cur]);
    }
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
      for (int tn = 0; tn < TN; ++tn)
        mma16B(acc[tm][tn], __builtin_bit_cast(uint4, a[cur][tm]), __builtin_bit_cast(uint4, b[cur][tn]), T());
    __builtin_amdgcn_sched_barrier(0);       // keep these MFMAs in front of the next K-step's wait
  });
}

// 16 bytes per lane from a buffer straight into LDS: the wave's 64 lanes fill the 1 KiB starting at lds_base
// (wave-uniform) in lane order; a lane whose byte offset lies outside the buffer (NO_ROW below) delivers zeros,
// which is how padding taps, rows past a model's end and columns past N are filled.  Completion is counted by
// vmcnt like any vector load.
typedef int int4v __attribute__((ext_vector_type(4)));
constexpr unsigned NO_ROW = 0xffffffffu;
__device__ inline int4v make_rsrc(const void* base, unsigned long long bytes) {
  const unsigned long long p = (unsigned long long)base;
  int4v r;
  r.x = __builtin_amdgcn_readfirstlane((int)(unsigned)p);
  r.y = __builtin_amdgcn_readfirstlane((int)((unsigned)(p >> 32) & 0xffffu));                 // stride 0: raw buffer
  r.z = __builtin_amdgcn_readfirstlane((int)(unsigned)(bytes > 0xfffffff0ull ? 0xfffffff0ull : bytes));
  r.w = 0x00020000;
  return r;
}
__device__ inline void load16_to_lds(const int4v& rsrc, unsigned byte_off, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tbuffer_load_dwordx4 %0, %1, 0 offen lds"
               : : "v"(byte_off), "s"(rsrc), "s"(lds_base) : "memory", "m0");
}
__device__ inline void wait_vm0() { asm volatile("s_waitcnt vmcnt(0)" : : : "memory"); }
// wait until at most `chunks` (wave-uniform; 2 or more counts as 2) groups of LPT loads are still in flight
template <int LPT>
__device__ inline void wait_vm_chunks(int chunks) {
  static_assert(2 * LPT <= 63, "vmcnt range");
  if (chunks >= 2) asm volatile("s_waitcnt vmcnt(%0)" : : "n"(2 * LPT) : "memory");
  else if (chunks == 1) asm volatile("s_waitcnt vmcnt(%0)" : : "n"(LPT) : "memory");
  else asm volatile("s_waitcnt vmcnt(0)" : : : "memory");
}

__device__ inline void store_out(float* p, float v) { *p = v; }
__device__ inline void store_out(bf16_t* p, float v) { *p = from_float<bf16_t>(v); }

// row of a model -> (sample, y, x); shift form when the side is a power of two
__device__ inline void decode_row(int r, int H, int rps, int sh, int& n, int& y, int& x) {
  if (sh >= 0) {
    n = r >> (2 * sh);
    const int rem = r & (rps - 1);
    y = rem >> sh;
    x = rem & (H - 1);
  } else {
    n = r / rps;
    const int rem = r - n * rps;
    y = rem / H;
    x = rem - y * H;
  }
}
// Row order of the forward-type kernel inside a model: pixel row y slowest, then the sample, then x.  A tile of
// consecutive rows then covers few pixel rows (one, when samples * H is a multiple of the tile height), and the taps
// that fall above or below the map for all of them are skipped as whole K-chunks.  row_block = samples * H.
__device__ inline void decode_row_yfirst(int r, int H, int row_block, int sh, int& n, int& y, int& x) {
  y = r / row_block;
  const int rem = r - y * row_block;
  if (sh >= 0) {
    n = rem >> sh;
    x = rem & (H - 1);
  } else {
    n = rem / H;
    x = rem - n * H;
  }
}
static int log2_or_neg(int v) {
  for (int s = 0; s < 30; ++s)
    if ((1 << s) == v) return s;
  return -1;
}

template <typename T, int MODE, int EPI, typename TL>
__global__ __launch_bounds__(TL::NT) void conv_gemm_kernel(ConvArgs p) {
  constexpr int BM = TL::BM, BN = TL::BN, TM = TL::TM, TN = TL::TN, PA = TL::PA, PB = TL::PB, RPP = TL::RPP;
  constexpr int KB = TL::KB, NST = TL::NST;
  constexpr int SMEM_RING = NST * (BM + BN) * KB;
  constexpr int SMEM_EPI = BM * 8 + (TL::NT / 64) * 32 * (TN * 32 * 4 + 16);   // see the epilogue
  constexpr int SMEM = SMEM_RING > SMEM_EPI ? SMEM_RING : SMEM_EPI;
  __shared__ __attribute__((aligned(1024))) unsigned char smem[SMEM];
  unsigned char* const As = smem;                      // buffer s at As + s * BM * KB
  unsigned char* const Bs = smem + NST * BM * KB;      // buffer s at Bs + s * BN * KB
  constexpr int BK = KB / (int)sizeof(T);              // elements of K per chunk
  constexpr int LINES = 128 / KB;                      // chunks per 128-byte line
  constexpr int LINES_ = LINES;
  constexpr int EPV = 16 / (int)sizeof(T);
  constexpr int LPT = PA + PB;                         // loads per thread per chunk
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / TL::WN, wn = wave % TL::WN;

  // ---- which tile: consecutive virtual ids stay on one XCD (block ids are dealt round-robin to the 8 XCDs).
  // Virtual id = ((M-tile * segments + segment) * phases + phase) * N-tiles + N-tile: blocks that run together on
  // an XCD read the same activations (other phase / N-tile) or the same model's weights (other M-tile, segment)
  // out of that XCD's L2.
  constexpr int NPH = (MODE == MODE_UP) ? 4 : 1;
  const int NT = (p.N + BN - 1) / BN;
  const int Ttot = p.tpre[p.L];
  const int total = Ttot * NT * p.nseg * NPH;
  const int per_xcd = (total + 7) >> 3;
  const int slot = blockIdx.x >> 3;
  if (slot >= per_xcd) return;
  const int v = (blockIdx.x & 7) * per_xcd + slot;
  if (v >= total) return;
  const int nt = v % NT;
  const int v1 = v / NT;
  const int phase = v1 % NPH;
  const int v2 = v1 / NPH;
  const int sidx = v2 % p.nseg;
  const int mt = v2 / p.nseg;
  int lo = 0;
  if (p.tmodel) {
    lo = p.tmodel[mt];
  } else {
    int hi = p.L;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (p.tpre[mid] <= mt) lo = mid; else hi = mid;
    }
  }
  const int l = lo;
  const int seg = p.seg_first + sidx;
  const int s0 = p.offs[l], s1 = p.offs[l + 1];
  const int Hr = p.Hr, Hin = p.Hin, C = p.C, N = p.N;
  const int rps = Hr * Hr;
  const int Mrows = (s1 - s0) * rps;
  const int m0 = (mt - p.tpre[l]) * BM;
  const long long sample_base = (long long)seg * p.seg_samples + s0;
  const int py = phase >> 1, px = phase & 1;

  constexpr int SZ = (int)sizeof(T);
  const int cpl = C * SZ / 128;   // 128-byte channel lines per tap
  // Pixel rows this tile covers (rows are ordered y, sample, x) and the taps that are inside the map for at least
  // one of them: a tap row that is outside for the whole tile contributes zeros only and its K-chunks are skipped.
  const int row_block = (s1 - s0) * Hr;
  int cnt_lo = 4, cnt_hi = 4;     // down: valid taps of the classes with ky even / odd ; up: cnt_lo = valid taps
  bool first_gone = false;        // the skipped taps are the first ones of their group (otherwise the last ones)
  if (MODE != MODE_DENSE) {
    const int y_lo = m0 / row_block, y_hi = (min(m0 + BM, Mrows) - 1) / row_block;
    const bool top_only = y_hi == 0, bottom_only = y_lo == Hr - 1;          // only the first / last pixel row
    if (MODE == MODE_DOWN) {
      if (top_only) cnt_lo = 2;                      // ky = 0 reads row -1
      if (bottom_only) cnt_hi = 2;                   // ky = 3 reads row Hin
      first_gone = top_only;
    } else {
      // phase py = 0 gathers rows y and y - 1, py = 1 rows y + 1 and y (tap index a = 0, 1 in this order)
      if (py == 0 && top_only) cnt_lo = 2;           // a = 1 (row y - 1) is gone: the last ones
      if (py == 1 && bottom_only) { cnt_lo = 2; first_gone = true; }   // a = 0 (row y + 1) is gone
    }
  }
  const int chunks_per_tap = cpl * LINES_;
  const int nk = (MODE == MODE_DOWN) ? 2 * (cnt_lo + cnt_hi) * chunks_per_tap
                                     : (MODE == MODE_UP ? cnt_lo * chunks_per_tap : C / BK);
  const int wns = p.w_nstride;   // rows per tap in the weight block (N, or more when only some rows are used)
  // this model's slice of the gathered tensor (one segment) and its weight block, as bounds-checked buffers
  const int nsamp = s1 - s0;
  const long long a_elems = (MODE == MODE_DENSE) ? (long long)nsamp * rps * C : (long long)nsamp * Hin * Hin * C;
  const T* a_base = static_cast<const T*>(p.A) + ((MODE == MODE_DENSE) ? sample_base * rps * C : sample_base * (long long)(Hin * Hin) * C);
  const int4v a_rsrc = make_rsrc(a_base, (unsigned long long)a_elems * SZ);
  const int4v w_rsrc = make_rsrc(static_cast<const T*>(p.W) + (long long)l * p.w_stride,
                                 (unsigned long long)(MODE == MODE_DENSE ? 1 : 16) * wns * C * SZ);

  // ---- per-thread load assignment: rows tid/CPR + RPP i, LDS position tid % CPR of the row, which holds the row's
  // 16-byte chunk (tid % CPR) ^ swizzle(row) (RPP is a multiple of the swizzle period, so the same chunk in every
  // pass).  Per row: byte offset of its pixel at tap offset (0, 0) and the set of taps that stay inside the map.
  constexpr int CPR = TL::CPR;
  const int row0 = tid / CPR;
  const int chunk = (tid % CPR) ^ fwd_swz<KB>(row0);
  unsigned apix[PA], amask[PA], bcol[PB];
#pragma unroll
  for (int i = 0; i < PA; ++i) {
    const int r = m0 + row0 + RPP * i;
    apix[i] = 0;
    amask[i] = 0;
    if (r < Mrows) {
      if (MODE == MODE_DENSE) {
        apix[i] = (unsigned)((r * C + chunk * EPV) * SZ);
        amask[i] = 1;
      } else {
        int n, y, x;
        decode_row_yfirst(r, Hr, row_block, p.hr_shift, n, y, x);
        const int by = (MODE == MODE_DOWN) ? 2 * y - 1 : y, bx = (MODE == MODE_DOWN) ? 2 * x - 1 : x;
        apix[i] = (unsigned)((((n * Hin + by) * Hin + bx) * C + chunk * EPV) * SZ);     // may wrap below zero: masked
        if (MODE == MODE_DOWN) {             // tap (ky, kx) is inside iff row by + ky and column bx + kx are: separable
          unsigned xm = 0;
#pragma unroll
          for (int k = 0; k < 4; ++k) xm |= ((unsigned)(bx + k) < (unsigned)Hin ? 1u : 0u) << k;
#pragma unroll
          for (int k = 0; k < 4; ++k)
            if ((unsigned)(by + k) < (unsigned)Hin) amask[i] |= xm << (4 * k);
        } else {
          for (int t = 0; t < 4; ++t) {
            const int dy = py == 0 ? ((t >> 1) == 0 ? 0 : -1) : ((t >> 1) == 0 ? 1 : 0);
            const int dx = px == 0 ? ((t & 1) == 0 ? 0 : -1) : ((t & 1) == 0 ? 1 : 0);
            const int iy = by + dy, ix = bx + dx;
            if ((unsigned)iy < (unsigned)Hin && (unsigned)ix < (unsigned)Hin) amask[i] |= 1u << t;
          }
        }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < PB; ++i) {
    const int col = nt * BN + row0 + RPP * i;
    bcol[i] = col < N ? (unsigned)((col * C + chunk * EPV) * SZ) : NO_ROW;
  }

  const unsigned lds0 = (unsigned)(uintptr_t)smem;     // LDS byte address of the buffers
  // K-chunk kc -> which tap it gathers and the wave-uniform byte offsets it adds to a row's base offsets.
  // K order, fastest first: the chunks of one 128-byte line; the taps whose gathers land on the same input pixels
  // shifted by one (down: the 4 taps of a (ky%2, kx%2) class, up: the phase's 4 taps), which find their rows in
  // L2; the channel line; (down) the class.
  auto chunk_offsets = [&](int kc, int& tap, unsigned& a_delta, unsigned& w_delta) {
    int cc;
    if (MODE == MODE_DOWN) {
      // classes 0, 1 hold the taps with ky in {0, 2}, classes 2, 3 those with ky in {1, 3}; a class keeps cnt taps
      const int per_lo = cnt_lo * chunks_per_tap;                 // chunks of one class with ky even
      int cls, rest;
      if (kc < 2 * per_lo) { cls = kc >= per_lo ? 1 : 0; rest = kc - cls * per_lo; }
      else { const int k2 = kc - 2 * per_lo, per_hi = cnt_hi * chunks_per_tap; cls = k2 >= per_hi ? 3 : 2; rest = k2 - (cls - 2) * per_hi; }
      const int cnt = cls < 2 ? cnt_lo : cnt_hi;
      const int part = rest % LINES, jr = rest / LINES;
      const int j = cnt == 4 ? (jr & 3) : (jr & 1);
      const int line = cnt == 4 ? (jr >> 2) : (jr >> 1);
      // the two taps left in a class of two are its kx pair at the one valid ky: ky = 2 (top tile, even class) or
      // ky = 1 (bottom tile, odd class)
      const int j4 = cnt == 4 ? j : j + ((cls < 2) ? 2 : 0);
      cc = line * LINES + part;
      tap = (((cls >> 1) + 2 * (j4 >> 1)) << 2) + (cls & 1) + 2 * (j4 & 1);
    } else if (MODE == MODE_UP) {
      const int part = kc % LINES, jr = kc / LINES;
      const int j = cnt_lo == 4 ? (jr & 3) : (jr & 1);
      const int line = cnt_lo == 4 ? (jr >> 2) : (jr >> 1);
      cc = line * LINES + part;
      tap = cnt_lo == 4 ? j : j + (first_gone ? 2 : 0);
    } else {
      cc = kc;
      tap = 0;
    }
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
    a_delta = (unsigned)(((dy * Hin + dx) * C + cc * BK) * SZ);    // wave-uniform
    w_delta = (unsigned)((wtap * wns * C + cc * BK) * SZ);
  };
  auto load_chunk = [&](int kc, int stage) {
    int tap;
    unsigned a_delta, w_delta;
    chunk_offsets(kc, tap, a_delta, w_delta);
    const unsigned a_dst = lds0 + (stage * BM + wave * (1024 / KB)) * KB;        // + pass * RPP rows
    const unsigned b_dst = lds0 + (NST * BM + stage * BN + wave * (1024 / KB)) * KB;
#pragma unroll
    for (int i = 0; i < PA; ++i)
      load16_to_lds(a_rsrc, ((amask[i] >> tap) & 1u) ? apix[i] + a_delta : NO_ROW, a_dst + i * RPP * KB);
#pragma unroll
    for (int i = 0; i < PB; ++i)
      load16_to_lds(w_rsrc, bcol[i] != NO_ROW ? bcol[i] + w_delta : NO_ROW, b_dst + i * RPP * KB);
  };
  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // Ring of NST buffers: chunk c lives in buffer c % NST.  While chunk c is multiplied, chunks c+1 .. c+NST-1 are on
  // their way; the barrier that ends iteration c tells every wave that chunk c+1 has landed everywhere and that
  // buffer c % NST may be refilled (with chunk c+NST, by the next iteration).
  for (int c = 0; c < NST - 1 && c < nk; ++c) load_chunk(c, c);
  wait_vm_chunks<LPT>(min(nk, NST - 1) - 1);
  __syncthreads();
  for (int kc = 0; kc < nk; ++kc) {
    if (kc + NST - 1 < nk) load_chunk(kc + NST - 1, (kc + NST - 1) % NST);
    tile_mma_fwd<T, TM, TN, KB>(acc, As + (kc % NST) * BM * KB, Bs + (kc % NST) * BN * KB, wm, wn, lane);
    wait_vm_chunks<LPT>(min(nk - 1, kc + NST - 1) - (kc + 1));     // chunks after kc+1 may stay in flight
    __syncthreads();
  }

  // ---- epilogue: output row index of every tile row, through LDS (the buffers are free now)
  long long* orow = reinterpret_cast<long long*>(smem);
  for (int t = tid; t < BM; t += TL::NT) {
    const int r = m0 + t;
    long long o = -1;
    if (r < Mrows) {
      if (MODE == MODE_DENSE) {
        o = sample_base * rps + r;
      } else {
        int n, y, x;
        decode_row_yfirst(r, Hr, row_block, p.hr_shift, n, y, x);
        const int Hb = 2 * Hr;
        if (MODE == MODE_UP) o = ((sample_base + n) * Hb + (2 * y + py)) * Hb + (2 * x + px);
        else o = ((sample_base + n) * Hr + y) * Hr + x;
      }
    }
    orow[t] = o;
  }
  __syncthreads();
  T* __restrict__ Out = static_cast<T*>(p.Out);
  const T* __restrict__ Aux = static_cast<const T*>(p.Aux);
  {
    // Each wave passes its 32 x (TN*32) blocks (fp32) through a private LDS patch so that every lane stores 16
    // contiguous bytes of an output row (full N is a multiple of 64 for these tiles).  The patch belongs to one
    // wave, whose LDS operations execute in order: no block-wide barrier is needed around it.
    constexpr int WCOLS = TN * 32;
    constexpr int PSTRIDE = WCOLS * 4 + 16;                             // bytes per patch row
    constexpr int CPR = WCOLS / EPV;                                    // 16-byte output chunks per patch row
    unsigned char* patch = smem + BM * 8 + wave * (32 * PSTRIDE);       // after the row table
    static_assert(SMEM >= BM * 8 + (TL::NT / 64) * 32 * PSTRIDE && SMEM_EPI == BM * 8 + (TL::NT / 64) * 32 * PSTRIDE, "patch area");
    const int colw = nt * BN + wn * WCOLS;                              // first column of this wave
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
#pragma unroll
      for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int pr = (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
          float val = acc[tm][tn][e];
          if (EPI == EPI_LRELU) val = val > 0.f ? val : val * p.slope;
          *reinterpret_cast<float*>(patch + pr * PSTRIDE + (tn * 32 + (lane & 31)) * 4) = val;
        }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int i = 0; i < 32 * CPR / 64; ++i) {
        const int cid = lane + 64 * i;
        const int pr = cid / CPR, pc = cid - pr * CPR;
        const long long o = orow[wm * TM * 32 + tm * 32 + pr];
        const int col = colw + pc * EPV;
        if (o >= 0 && col < N) {
          float vf[EPV];
#pragma unroll
          for (int k = 0; k < EPV; k += 4) {
            const float4 t4 = *reinterpret_cast<const float4*>(patch + pr * PSTRIDE + (pc * EPV + k) * 4);
            vf[k] = t4.x; vf[k + 1] = t4.y; vf[k + 2] = t4.z; vf[k + 3] = t4.w;
          }
          if (EPI == EPI_ACT_BWD) {               // times the activation's derivative, from the saved output
            const uint4 araw = *reinterpret_cast<const uint4*>(Aux + o * N + col);
            const T* aa = reinterpret_cast<const T*>(&araw);
#pragma unroll
            for (int k = 0; k < EPV; ++k)
              if (!(to_float(aa[k]) > 0.f)) vf[k] *= p.slope;
          }
          uint4 vraw;
          if constexpr (sizeof(T) == 2) {
            vraw = make_uint4(pack2_bf16(vf[0], vf[1]), pack2_bf16(vf[2], vf[3]), pack2_bf16(vf[4], vf[5]), pack2_bf16(vf[6], vf[7]));
          } else {
            vraw = make_uint4(__float_as_uint(vf[0]), __float_as_uint(vf[1]), __float_as_uint(vf[2]), __float_as_uint(vf[3]));
          }
          {
            typedef unsigned u4 __attribute__((ext_vector_type(4)));
            u4 q; q.x = vraw.x; q.y = vraw.y; q.z = vraw.z; q.w = vraw.w;
            __builtin_nontemporal_store(q, reinterpret_cast<u4*>(Out + o * N + col));      // read next by another kernel, never by this one
          }
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
  }
  if (p.stat_partial) {
    // For the BatchNorm that follows.  Every wave's (TM*32)-row block of the tile is a sub-tile of its own: per column
    // the sum of its fp32 results and the sum of their squared deviations from the sub-tile's column mean, which the
    // statistics kernel merges across sub-tiles with the pairwise-update formula (no E[x^2] - mean^2 over a whole
    // channel).  One pass over the accumulators with the sub-tile's first row as the shift K:
    //   sum = K n + sum(x - K),   M2 = sum((x - K)^2) - (sum(x - K))^2 / n
    // (a sample of the column is as good a shift as its mean up to a few units of the last place), no block-wide
    // barrier and nothing shared between the waves, so a wave is done when its own stores and sums are.
    constexpr int SUB = TM * 32;
    const int nvalid = min(max(Mrows - m0 - wm * SUB, 0), SUB);          // valid rows of this wave's sub-tile: a prefix
    const long long tix = (((long long)phase * p.nseg + sidx) * p.ub_tiles + mt) * TL::WM + wm;
    if (nvalid > 0) {
#pragma unroll
      for (int tn = 0; tn < TN; ++tn) {
        const float K = __shfl(acc[0][tn][0], lane & 31, 64);           // row 0 of the sub-tile, this lane's column
        float s1 = 0.f, s2 = 0.f;
        if (nvalid == SUB) {
#pragma unroll
          for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
              const float d = acc[tm][tn][e] - K;
              s1 += d;
              s2 += d * d;
            }
        } else {
#pragma unroll
          for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
              const int rr = tm * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
              const float d = acc[tm][tn][e] - K;
              if (rr < nvalid) { s1 += d; s2 += d * d; }
            }
        }
        s1 += __shfl_xor(s1, 32, 64);
        s2 += __shfl_xor(s2, 32, 64);
        const int col = nt * BN + wn * TN * 32 + tn * 32 + (lane & 31);
        if (lane < 32 && col < N) {
          const float nf = (float)nvalid;
          p.stat_partial[(tix * N + col) * 2] = K * nf + s1;
          p.stat_partial[(tix * N + col) * 2 + 1] = fmaxf(s2 - s1 * s1 / nf, 0.f);
        }
      }
    }
  }
}

template <typename T, int MODE, int EPI, typename TL>
static void launch_one(ConvArgs a, hipStream_t st) {
  if (a.tile_rows != TL::BM) return launch_fail("GEMM: the tile prefix array was built for another tile height");
  a.hr_shift = log2_or_neg(a.Hr);
  const int NT = (a.N + TL::BN - 1) / TL::BN;
  const long long blocks = ((long long)a.ub_tiles * NT * a.nseg * (MODE == MODE_UP ? 4 : 1) + 7) / 8 * 8;
  if (blocks == 0 || a.nseg == 0) return;
  dim3 grid((unsigned)blocks, 1, 1);
  hipLaunchKernelGGL((conv_gemm_kernel<T, MODE, EPI, TL>), grid, dim3(TL::NT), 0, st, a);
}

template <typename T, int MODE, int EPI>
static void launch_wide(const ConvArgs& a, hipStream_t st) {
  if (a.tile_rows == TileTiny::BM) return launch_one<T, MODE, EPI, TileTiny>(a, st);
  if (a.tile_rows == TileSmall::BM) return launch_one<T, MODE, EPI, TileSmall>(a, st);
  if (a.N <= TileNarrow::BN) return launch_one<T, MODE, EPI, TileNarrow>(a, st);
  if (a.N % 256 == 0) return launch_one<T, MODE, EPI, TileBig>(a, st);
  return launch_one<T, MODE, EPI, TileMid>(a, st);
}

// Row blocks per tile that leave their own BatchNorm partial sums (the WM of the tile launch_wide picks).
int conv_stat_split(int n_out, int tile_rows) {
  if (tile_rows == TileTiny::BM) return TileTiny::WM;
  if (tile_rows == TileSmall::BM) return TileSmall::WM;
  if (n_out <= TileNarrow::BN) return TileNarrow::WM;
  if (n_out % 256 == 0) return TileBig::WM;
  return TileMid::WM;
}

// The (mode, epilogue, tile) combinations the networks use.
template <typename T>
void launch_conv(int mode, int epi, const ConvArgs& a, hipStream_t st) {
  // the kernel's assumptions, checked before anything is launched
  if (!a.A || !a.W || !a.Out || !a.offs || !a.tpre || a.N < 1 || a.w_nstride < a.N || a.C % (128 / (int)sizeof(T)) != 0 ||
      (epi == EPI_ACT_BWD && !a.Aux))
    return launch_fail("GEMM: null operand, or channel counts that are not whole 128-byte lines");
  if (a.N < 64) return launch_fail("GEMM: fewer than 64 output channels (image-side outputs have their own kernel)");
  {
    // the loaders address one model's slice of A and one weight block with 32-bit byte offsets
    const long long side = mode == MODE_DENSE ? a.Hr : a.Hin;
    if ((long long)a.seg_samples * side * side * a.C * (long long)sizeof(T) >= (1LL << 31) ||
        16LL * a.w_nstride * a.C * (long long)sizeof(T) >= (1LL << 31))
      return launch_fail("GEMM: one segment of the gathered tensor, or one weight block, is 2 GiB or larger");
  }
  if (mode == MODE_DOWN && epi == EPI_NONE) return launch_wide<T, MODE_DOWN, EPI_NONE>(a, st);
  if (mode == MODE_UP && epi == EPI_NONE) return launch_wide<T, MODE_UP, EPI_NONE>(a, st);
  if (mode == MODE_UP && epi == EPI_ACT_BWD) return launch_wide<T, MODE_UP, EPI_ACT_BWD>(a, st);
  if (mode == MODE_DENSE && epi == EPI_NONE) return launch_wide<T, MODE_DENSE, EPI_NONE>(a, st);
  if (mode == MODE_DENSE && epi == EPI_LRELU) return launch_wide<T, MODE_DENSE, EPI_LRELU>(a, st);
  launch_fail("GEMM: (mode, epilogue) combination without an instantiation");
}
// Name of the kernel instantiation launch_conv picks (for per-kernel timing): mode, epilogue, tile.
const char* conv_variant_name(int mode, int epi, const ConvArgs& a) {
  static const char* modes[3] = {"down", "up", "dense"};
  static const char* epis[3] = {"", "+actbwd", "+lrelu"};
  static char names[3][3][5][48];
  const int tile = a.tile_rows == TileTiny::BM ? 4 : (a.tile_rows == TileSmall::BM ? 2 : (a.N <= TileNarrow::BN ? 3 : (a.N % 256 == 0 ? 0 : 1)));
  static const char* tiles[5] = {"256x256", "256x128", "128x128", "256x64", "64x64"};
  char* n = names[mode][epi][tile];
  if (!n[0]) snprintf(n, 48, "gemm_%s%s<%s>", modes[mode], epis[epi], tiles[tile]);
  return n;
}
const char* wgrad_variant_name(const WgradArgs& a) {
  if (a.ntaps * a.Cb <= 64) return "wgrad<64x128>";
  return a.Cs % 256 == 0 ? "wgrad<256x256>" : "wgrad<256x128>";
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

// Which model the i-th group of blocks works on.  Groups are dealt round-robin to the 8 XCDs in rows of eight; with
// the models sorted by decreasing size the rows alternate direction, so that every XCD gets the same share of the
// rows and starts with its largest models.
__device__ inline int wgrad_model(const WgradArgs& p, int i) {
  if (!p.order) return i;
  const int row = i >> 3;
  if ((row & 1) && row * 8 + 8 <= p.L) i = row * 8 + 7 - (i & 7);
  return p.order[i];
}

// A loader task = 8 rows of the reduction index x one 16-byte channel group of one operand.
//   bf16: 8 consecutive rows x 8 channels, transposed in registers, written as 8 x 16 bytes
//   fp32: 8 rows strided by 4 x 4 channels, written as 32 scalars
template <typename T, typename TL>
__global__ __launch_bounds__(TL::NT) void wgrad_kernel(WgradArgs p) {
  constexpr int BM = TL::BM, BN = TL::BN, TM = TL::TM, TN = TL::TN;
  __shared__ __attribute__((aligned(16))) unsigned char As[2][BM * LDS_STRIDE];
  __shared__ __attribute__((aligned(16))) unsigned char Bs[2][BN * LDS_STRIDE];
  constexpr int BKR = BKB / (int)sizeof(T);     // rows (reduction index) per chunk: 64 (bf16) or 32 (fp32)
  constexpr bool IS16 = sizeof(T) == 2;
  constexpr int EPV = 16 / (int)sizeof(T);
  constexpr int NTASK = (BM + BN + TL::NT - 1) / TL::NT;   // loader tasks per thread
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / TL::WN, wn = wave % TL::WN;

  // ---- tile: all tiles of one (model, row split) run on one XCD -- they read the same rows -- and the
  // (model, split) pairs are dealt round-robin to the XCDs
  const int Cb = p.Cb, Cs = p.Cs, Hs = p.Hs;
  const int Mtot = p.ntaps * Cb;
  const int MT = (Mtot + BM - 1) / BM, NT = (Cs + BN - 1) / BN;
  const int bid = blockIdx.x;
  const int unit = (bid / (8 * MT * NT)) * 8 + (bid & 7);
  if (unit >= p.L * p.ksplit) return;
  const int l = wgrad_model(p, unit / p.ksplit), split = unit % p.ksplit;
  const int tile = (bid >> 3) % (MT * NT);
  const int mt = tile / NT, nt = tile - mt * NT;
  const int s0 = p.offs[l], s1 = p.offs[l + 1];
  const int rps = Hs * Hs;
  const int R = (s1 - s0) * rps;
  const int Hb = 2 * Hs;
  const T* __restrict__ Big = static_cast<const T*>(p.Big);
  const T* __restrict__ Small = static_cast<const T*>(p.Small);
  // this block's share of each segment's rows
  const int rows_split = ((R + p.ksplit - 1) / p.ksplit + BKR - 1) / BKR * BKR;
  const int r_lo = split * rows_split, r_hi = min(R, r_lo + rows_split);

  // ---- loader tasks
  int t_ch[NTASK], t_ky[NTASK], t_kx[NTASK], t_cg[NTASK], t_rg[NTASK];
  bool t_isA[NTASK], t_ok[NTASK];
#pragma unroll
  for (int k = 0; k < NTASK; ++k) {
    const int t = tid + k * TL::NT;
    t_isA[k] = t < BM;
    const int u = t_isA[k] ? t : t - BM;                  // task index inside its operand
    const int groups = (t_isA[k] ? BM : BN) / EPV;        // channel groups
    t_cg[k] = u % groups;
    t_rg[k] = u / groups;
    t_ky[k] = 1; t_kx[k] = 1;
    if (t_isA[k]) {
      const int m = mt * BM + t_cg[k] * EPV;
      t_ok[k] = m < Mtot;
      const int tap = m / Cb;
      t_ch[k] = m - tap * Cb;
      if (p.ntaps != 1) { t_ky[k] = tap >> 2; t_kx[k] = tap & 3; }
    } else {
      t_ch[k] = nt * BN + t_cg[k] * EPV;
      t_ok[k] = t < BM + BN && t_ch[k] < Cs;
    }
  }

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  uint4 reg[NTASK][8];
  auto load_chunk = [&](long long sample_base, int k0) {
#pragma unroll
    for (int k = 0; k < NTASK; ++k)
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int r = k0 + (IS16 ? t_rg[k] * 8 + j : t_rg[k] + 4 * j);
        uint4 val = make_uint4(0, 0, 0, 0);
        if (r < r_hi && t_ok[k]) {
          if (!t_isA[k]) {
            val = *reinterpret_cast<const uint4*>(Small + (sample_base * rps + r) * (long long)Cs + t_ch[k]);
          } else if (p.ntaps == 1) {             // rows of the big tensor are read directly
            val = *reinterpret_cast<const uint4*>(Big + (sample_base * rps + r) * (long long)Cb + t_ch[k]);
          } else {
            int n, y, x;
            decode_row(r, Hs, rps, p.hs_shift, n, y, x);
            const int iy = 2 * y - 1 + t_ky[k], ix = 2 * x - 1 + t_kx[k];
            if ((unsigned)iy < (unsigned)Hb && (unsigned)ix < (unsigned)Hb)
              val = *reinterpret_cast<const uint4*>(Big + (((sample_base + n) * Hb + iy) * Hb + ix) * (long long)Cb + t_ch[k]);
          }
        }
        reg[k][j] = val;
      }
  };
  auto store_chunk = [&](int buf) {
#pragma unroll
    for (int k = 0; k < NTASK; ++k) {
      if (tid + k * TL::NT >= BM + BN) continue;
      unsigned char* dst = t_isA[k] ? As[buf] : Bs[buf];
      if (IS16) {
        transpose8x8_b16(reg[k]);
#pragma unroll
        for (int j = 0; j < 8; ++j)   // row t_cg*8 + j, chunk t_rg rotated by row/16 = t_cg/2
          *reinterpret_cast<uint4*>(dst + (t_cg[k] * 8 + j) * LDS_STRIDE + ((t_rg[k] + (t_cg[k] >> 1)) & 7) * 16) = reg[k][j];
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int kr = t_rg[k] + 4 * j;                       // rows t_cg*4 .. +3 share row/16 = t_cg/4
          unsigned* d0 = reinterpret_cast<unsigned*>(dst + (t_cg[k] * 4) * LDS_STRIDE +
                                                     (((kr >> 2) + (t_cg[k] >> 2)) & 7) * 16 + (kr & 3) * 4);
          d0[0] = reg[k][j].x;
          d0[LDS_STRIDE / 4] = reg[k][j].y;
          d0[2 * LDS_STRIDE / 4] = reg[k][j].z;
          d0[3 * LDS_STRIDE / 4] = reg[k][j].w;
        }
      }
    }
  };

  // chunks of all segments as one sequence
  const int per_seg = r_hi > r_lo ? (r_hi - r_lo + BKR - 1) / BKR : 0;
  const int nchunks = per_seg * p.nseg;
  auto chunk_pos = [&](int c, long long& sample_base, int& k0) {
    const int seg = c / per_seg;
    sample_base = (long long)seg * p.seg_samples + s0;
    k0 = r_lo + (c - seg * per_seg) * BKR;
  };
  if (nchunks > 0) {
    long long sb; int k0;
    chunk_pos(0, sb, k0);
    load_chunk(sb, k0);
    store_chunk(0);
    __syncthreads();
    for (int c = 0; c < nchunks; ++c) {
      const bool more = c + 1 < nchunks;
      if (more) { chunk_pos(c + 1, sb, k0); load_chunk(sb, k0); }
      tile_mma<T, TM, TN>(acc, As[c & 1], Bs[c & 1], wm, wn, lane);
      if (more) store_chunk((c + 1) & 1);
      __syncthreads();
    }
  }

  float* __restrict__ dW = p.dW + (long long)split * p.split_stride + (long long)l * p.dw_stride;
#pragma unroll
  for (int tm = 0; tm < TM; ++tm)
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
      const int col = nt * BN + wn * TN * 32 + tn * 32 + (lane & 31);
      if (col >= Cs) continue;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = mt * BM + wm * TM * 32 + tm * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
        if (m < Mtot) dW[(long long)m * Cs + col] = acc[tm][tn][e];
      }
    }
}

// ---- bf16 weight gradient: tiles stay in their memory layout ---------------------------------------------
// Both operands are stored [row][channel] in HBM while the MFMA wants, per lane, eight consecutive rows (the
// reduction index) of one channel.  The bf16 kernel copies K-chunks of 64 rows x BM (BN) channels global -> LDS
// as they are and lets ds_read_b64_tr_b16 do the transposition on the way to the registers: within each block of
// 16 lanes, lane i receives element i%4 of the 8-byte groups addressed by lanes i/4, 4 + i/4, 8 + i/4, 12 + i/4.
// Pointing lane s of a block at row (s/4), channel group (s%4) therefore hands lane i rows 0..3 of channel i.
// LDS rows are BM*2 (BN*2) bytes; the 16-byte chunk c of row R sits at position c ^ swz(R) so that the four rows
// a 32-lane half reads fall into different 64-byte bank groups.
constexpr int WG_KR = 64;      // rows (reduction index) per chunk
template <int ROWB>
__device__ inline int wg_swz(int row) {   // in 16-byte chunks
  return ROWB >= 256 ? 4 * (row & 3) : 4 * ((row >> 1) & 1);
}
typedef short short4v __attribute__((ext_vector_type(4)));
__device__ inline uint2 lds_read_tr16(const unsigned char* p) {
  const short4v v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v*)(p));
  return __builtin_bit_cast(uint2, v);
}

template <typename TL>
__global__ __launch_bounds__(TL::NT) void wgrad_tr_kernel(WgradArgs p) {
  typedef bf16_t T;
  constexpr int BM = TL::BM, BN = TL::BN, TM = TL::TM, TN = TL::TN, NT_ = TL::NT;
  constexpr int RBA = BM * 2, RBB = BN * 2;                 // bytes per LDS row
  constexpr int CPA = BM / 8, CPB = BN / 8;                 // 16-byte chunks per row
  constexpr int PA = WG_KR * CPA / NT_, PB = WG_KR * CPB / NT_;
  constexpr int RPA = NT_ / CPA, RPB = NT_ / CPB;           // rows per loader pass (multiples of 4)
  static_assert(WG_KR * CPA % NT_ == 0 && WG_KR * CPB % NT_ == 0 && RPA % 4 == 0 && RPB % 4 == 0, "loader shape");
  constexpr int STAGE_A = WG_KR * RBA, STAGE_B = WG_KR * RBB;
  __shared__ __attribute__((aligned(1024))) unsigned char smem[2 * (STAGE_A + STAGE_B)];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / TL::WN, wn = wave % TL::WN;

  // ---- tile: all tiles of one (model, row split) run on one XCD -- they read the same rows -- and the
  // (model, split) pairs are dealt round-robin to the XCDs
  const int Cb = p.Cb, Cs = p.Cs, Hs = p.Hs;
  const int Mtot = p.ntaps * Cb;
  const int MT = (Mtot + BM - 1) / BM, NTL = (Cs + BN - 1) / BN;
  const int bid = blockIdx.x;
  const int unit = (bid / (8 * MT * NTL)) * 8 + (bid & 7);
  if (unit >= p.L * p.ksplit) return;
  const int l = wgrad_model(p, unit / p.ksplit), split = unit % p.ksplit;
  const int tile = (bid >> 3) % (MT * NTL);
  const int mt = tile / NTL, nt = tile - mt * NTL;
  const int s0 = p.offs[l], s1 = p.offs[l + 1];
  const int rps = Hs * Hs;
  const int R = (s1 - s0) * rps;
  const int Hb = 2 * Hs;
  const int rows_split = ((R + p.ksplit - 1) / p.ksplit + WG_KR - 1) / WG_KR * WG_KR;
  const int r_lo = split * rows_split, r_hi = min(R, r_lo + rows_split);

  // ---- loader: slot = pass * NT + tid is the 16-byte LDS slot; it holds chunk (slot % CP) ^ swz(row) of row slot / CP
  const int rowA0 = tid / CPA, rowB0 = tid / CPB;
  const int chA = (tid % CPA) ^ wg_swz<RBA>(rowA0), chB = (tid % CPB) ^ wg_swz<RBB>(rowB0);
  const int mA = mt * BM + chA * 8;                          // first of this thread's 8 channels along M
  const bool okA = mA < Mtot;
  const int tapA = okA ? mA / Cb : 0;
  const int cA = mA - tapA * Cb;
  const int kyA = p.ntaps == 1 ? 1 : (tapA >> 2), kxA = p.ntaps == 1 ? 1 : (tapA & 3);
  const int cB = nt * BN + chB * 8;
  const bool okB = cB < Cs;
  const unsigned lds0 = (unsigned)(uintptr_t)smem;
  const long long big_per_sample = p.ntaps == 1 ? (long long)rps * Cb : (long long)Hb * Hb * Cb;

  // Chunks start at multiples of 64 rows.  With a power-of-two side of at most 64 a chunk is a whole number of
  // samples or of pixel rows, so a thread's rows keep their x, their y offset inside the chunk and their sample
  // offset: everything that depends on the row is computed once, and a chunk only adds a wave-uniform offset
  // (sample n0, pixel row y0 of the chunk's first row) and re-tests the vertical border.
  const bool fast = p.ntaps == 1 || (p.hs_shift >= 0 && Hs <= 64);
  // Reduction order "pixel row first" (y, sample, x) for the models whose samples * H rows per pixel row are whole
  // chunks: a chunk then lies inside one pixel row y0, the vertical border test is the same for the whole chunk, and
  // the chunks of the one pixel row whose tap row ky falls outside the map (y0 = 0 for ky = 0, y0 = H - 1 for
  // ky = 3) hold zeros only and are skipped.  The tile's taps share one ky (4 * Cb >= BM).  The choice depends on the
  // model's own sample count only.
  const int rb = (s1 - s0) * Hs;                    // rows per pixel row
  const bool yfirst = p.ntaps == 16 && fast && rb % WG_KR == 0 && 4 * Cb >= BM && Cb % 8 == 0 && (BM % Cb == 0 || Cb % BM == 0);
  const int ky_tile = (mt * BM / Cb) >> 2;
  unsigned fa_off[PA], fb_off[PB];
  int fa_iy[PA];                   // 2 * (y inside the chunk) - 1 + ky ; a large value marks a lane that never loads
#pragma unroll
  for (int i = 0; i < PA; ++i) {
    const int c = rowA0 + i * RPA;
    fa_off[i] = 0;
    fa_iy[i] = 1 << 20;
    if (okA) {
      if (p.ntaps == 1) {
        fa_off[i] = (unsigned)((c * Cb + cA) * 2);
        fa_iy[i] = 0;
      } else if (yfirst) {
        // row c of a chunk: sample n0 + c / H, x = c % H, pixel row y0 (chunk-uniform)
        const int sh = p.hs_shift;
        const int ni = c >> sh, xi = c & (Hs - 1);
        const int ix = 2 * xi - 1 + kxA;
        if ((unsigned)ix < (unsigned)Hb) {
          fa_iy[i] = kyA - 1;
          fa_off[i] = (unsigned)((((ni * Hb + fa_iy[i]) * Hb + ix) * Cb + cA) * 2);    // may wrap below zero: masked
        }
      } else if (fast) {
        const int sh = p.hs_shift;
        const int ni = c >> (2 * sh), rem = c & (rps - 1);
        const int yi = rem >> sh, xi = rem & (Hs - 1);
        const int ix = 2 * xi - 1 + kxA;
        if ((unsigned)ix < (unsigned)Hb) {
          fa_iy[i] = 2 * yi - 1 + kyA;
          fa_off[i] = (unsigned)((((ni * Hb + fa_iy[i]) * Hb + ix) * Cb + cA) * 2);    // may wrap below zero: masked
        }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < PB; ++i) {
    const int c = rowB0 + i * RPB;
    if (yfirst) fb_off[i] = (unsigned)((((c >> p.hs_shift) * rps + (c & (Hs - 1))) * Cs + cB) * 2);
    else fb_off[i] = (unsigned)((c * Cs + cB) * 2);
  }

  auto load_chunk = [&](int seg, int k0, int stage) {
    const long long sb = (long long)seg * p.seg_samples + s0;
    const int4v a_rsrc = make_rsrc(static_cast<const T*>(p.Big) + sb * big_per_sample, (unsigned long long)(s1 - s0) * big_per_sample * 2);
    const int4v b_rsrc = make_rsrc(static_cast<const T*>(p.Small) + sb * rps * Cs, (unsigned long long)R * Cs * 2);
    const unsigned a_dst = lds0 + stage * STAGE_A + wave * 1024;
    const unsigned b_dst = lds0 + 2 * STAGE_A + stage * STAGE_B + wave * 1024;
    const int left = r_hi - k0;                 // rows of this chunk that exist
    unsigned b_delta = (unsigned)(k0 * Cs * 2);
    if (fast) {
      unsigned a_delta;
      int y2 = 0;
      if (p.ntaps == 1) {
        a_delta = (unsigned)(k0 * Cb * 2);
      } else if (yfirst) {
        const int y0 = k0 / rb, n0 = (k0 - y0 * rb) >> p.hs_shift;
        a_delta = (unsigned)(((n0 * Hb + 2 * y0) * Hb) * Cb * 2);
        y2 = 2 * y0;
        b_delta = (unsigned)(((n0 * Hs + y0) * Hs) * Cs * 2);
      } else {
        const int n0 = k0 >> (2 * p.hs_shift), y0 = (k0 & (rps - 1)) >> p.hs_shift;
        a_delta = (unsigned)(((n0 * Hb + 2 * y0) * Hb) * Cb * 2);
        y2 = 2 * y0;
      }
#pragma unroll
      for (int i = 0; i < PA; ++i) {
        const bool ok = rowA0 + i * RPA < left && (unsigned)(fa_iy[i] + y2) < (unsigned)Hb;
        load16_to_lds(a_rsrc, ok ? fa_off[i] + a_delta : NO_ROW, a_dst + i * NT_ * 16);
      }
    } else {
#pragma unroll
      for (int i = 0; i < PA; ++i) {
        const int r = k0 + rowA0 + i * RPA;
        unsigned off = NO_ROW;
        if (r < r_hi && okA) {
          int n, y, x;
          decode_row(r, Hs, rps, p.hs_shift, n, y, x);
          const int iy = 2 * y - 1 + kyA, ix = 2 * x - 1 + kxA;
          if ((unsigned)iy < (unsigned)Hb && (unsigned)ix < (unsigned)Hb) off = (unsigned)((((n * Hb + iy) * Hb + ix) * Cb + cA) * 2);
        }
        load16_to_lds(a_rsrc, off, a_dst + i * NT_ * 16);
      }
    }
#pragma unroll
    for (int i = 0; i < PB; ++i)
      load16_to_lds(b_rsrc, (rowB0 + i * RPB < left && okB) ? fb_off[i] + b_delta : NO_ROW, b_dst + i * NT_ * 16);
  };

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // ---- fragment addressing: lane = 32 * kgrp + 16 * hb + s ; it points at row 8*kgrp + 4*half + s/4 of the k-step,
  // channels 16*hb + 4*(s%4) .. +3 of the 32-channel fragment
  const int s16 = lane & 15, hb = (lane >> 4) & 1, kgrp = lane >> 5;
  const int frow = 8 * kgrp + (s16 >> 2);                    // + 16 * kstep + 4 * half
  const int fch = 2 * hb + ((s16 & 3) >> 1);                 // 16-byte chunk inside the 32-channel fragment (0..3)
  const int fbyte = 8 * (s16 & 1);
  const int swzA = wg_swz<RBA>(frow), swzB = wg_swz<RBB>(frow);   // frow % 4 (and (frow/2) % 2) do not change with kstep or half
  auto mma_chunk = [&](int stage) {
    const unsigned char* As = smem + stage * STAGE_A;
    const unsigned char* Bs = smem + 2 * STAGE_A + stage * STAGE_B;
#pragma unroll
    for (int ks = 0; ks < WG_KR / 16; ++ks) {
      uint4 a[TM], b[TN];
#pragma unroll
      for (int t = 0; t < TM; ++t) {
        const int ch = ((wm * TM + t) * 4 + fch) ^ swzA;
        const unsigned char* q0 = As + (ks * 16 + frow) * RBA + ch * 16 + fbyte;
        const uint2 lo = lds_read_tr16(q0), hi = lds_read_tr16(q0 + 4 * RBA);
        a[t] = make_uint4(lo.x, lo.y, hi.x, hi.y);
      }
#pragma unroll
      for (int t = 0; t < TN; ++t) {
        const int ch = ((wn * TN + t) * 4 + fch) ^ swzB;
        const unsigned char* q0 = Bs + (ks * 16 + frow) * RBB + ch * 16 + fbyte;
        const uint2 lo = lds_read_tr16(q0), hi = lds_read_tr16(q0 + 4 * RBB);
        b[t] = make_uint4(lo.x, lo.y, hi.x, hi.y);
      }
#pragma unroll
      for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) mma16B(acc[tm][tn], a[tm], b[tn], T());
    }
  };

  // chunks of all segments as one sequence; in pixel-row-first order the chunks [bad0, bad0 + nbad) of every segment
  // (the pixel row whose tap row is outside the map) are left out
  const int per_seg_all = r_hi > r_lo ? (r_hi - r_lo + WG_KR - 1) / WG_KR : 0;
  int bad0 = 0, nbad = 0;
  if (yfirst && per_seg_all > 0 && (ky_tile == 0 || ky_tile == 3)) {
    const int yb = ky_tile == 0 ? 0 : Hs - 1;
    const int lo = max(yb * rb, r_lo), hi = min((yb + 1) * rb, r_hi);      // rows of that pixel row inside this block's share
    if (hi > lo) { bad0 = (lo - r_lo) / WG_KR; nbad = (hi - lo) / WG_KR; } // both multiples of the chunk height
  }
  const int per_seg = per_seg_all - nbad;
  const int nchunks = per_seg * p.nseg;
  auto chunk_row = [&](int cin) { return r_lo + (cin < bad0 ? cin : cin + nbad) * WG_KR; };
  if (nchunks > 0) {
    load_chunk(0, chunk_row(0), 0);
    wait_vm0();
    __syncthreads();
    int seg = 0, cin = 0;
    for (int c = 0; c < nchunks; ++c) {
      if (c + 1 < nchunks) {
        if (++cin == per_seg) { cin = 0; ++seg; }
        load_chunk(seg, chunk_row(cin), (c + 1) & 1);
      }
      mma_chunk(c & 1);
      wait_vm0();
      __syncthreads();
    }
  }

  // Epilogue: each wave passes its 32 x (TN*32) blocks through a private LDS patch (the K buffers are free after the
  // loop's last barrier) so that every lane stores 16 contiguous bytes of a row of dW.
  float* __restrict__ dW = p.dW + (long long)split * p.split_stride + (long long)l * p.dw_stride;
  constexpr int WCOLS = TN * 32;
  constexpr int PSTRIDE = WCOLS * 4 + 16;
  constexpr int CPRW = WCOLS / 4;                                       // 16-byte chunks per patch row
  static_assert((TL::NT / 64) * 32 * PSTRIDE <= 2 * (STAGE_A + STAGE_B), "patch area");
  unsigned char* patch = smem + wave * (32 * PSTRIDE);
  const int colw = nt * BN + wn * WCOLS;
#pragma unroll
  for (int tm = 0; tm < TM; ++tm) {
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int pr = (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
        *reinterpret_cast<float*>(patch + pr * PSTRIDE + (tn * 32 + (lane & 31)) * 4) = acc[tm][tn][e];
      }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int i = 0; i < 32 * CPRW / 64; ++i) {
      const int cid = lane + 64 * i;
      const int pr = cid / CPRW, pc = cid - pr * CPRW;
      const int m = mt * BM + wm * TM * 32 + tm * 32 + pr;
      const int col = colw + pc * 4;
      if (m < Mtot && col < Cs) {       // Cs is a multiple of 8: a 16-byte chunk is inside or outside
        typedef float f4 __attribute__((ext_vector_type(4)));
        const float4 t = *reinterpret_cast<const float4*>(patch + pr * PSTRIDE + pc * 16);
        f4 q; q.x = t.x; q.y = t.y; q.z = t.z; q.w = t.w;
        __builtin_nontemporal_store(q, reinterpret_cast<f4*>(dW + (long long)m * Cs + col));   // read next by the update kernel
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
}

typedef Tile<64, 128, 1, 4> TileWgImg;    // patch-matrix layers: 64 packed columns x 128 feature channels

template <typename T, typename TL>
static void launch_wgrad_one(WgradArgs a, hipStream_t st) {
  a.hs_shift = log2_or_neg(a.Hs);
  const int MT = (a.ntaps * a.Cb + TL::BM - 1) / TL::BM, NT = (a.Cs + TL::BN - 1) / TL::BN;
  const long long blocks = ((long long)a.L * a.ksplit + 7) / 8 * 8 * MT * NT;
  if (blocks == 0) return;
  if (sizeof(T) == 2) {
    // 32-bit byte offsets inside one model's slice of either operand
    const long long side = a.ntaps == 1 ? a.Hs : 2 * a.Hs;
    if ((long long)a.seg_samples * side * side * a.Cb * 2 >= (1LL << 31) || (long long)a.seg_samples * a.Hs * a.Hs * a.Cs * 2 >= (1LL << 31))
      return launch_fail("weight gradient: one segment of an operand is 2 GiB or larger");
    hipLaunchKernelGGL((wgrad_tr_kernel<TL>), dim3((unsigned)blocks), dim3(TL::NT), 0, st, a);
  } else {
    hipLaunchKernelGGL((wgrad_kernel<T, TL>), dim3((unsigned)blocks), dim3(TL::NT), 0, st, a);
  }
}

template <typename T>
void launch_wgrad(const WgradArgs& a, hipStream_t st) {
  if (!a.Big || !a.Small || !a.dW || !a.offs || a.Cb % 8 || a.Cs % 8 || (a.ntaps != 1 && a.ntaps != 16) || a.ksplit < 1 ||
      (a.ksplit > 1 && a.split_stride <= 0))
    return launch_fail("weight gradient: null operand, channel counts that are not multiples of 8, or a bad row split");
  if (a.ntaps * a.Cb <= 64) return launch_wgrad_one<T, TileWgImg>(a, st);
  if (a.Cs % 256 == 0) return launch_wgrad_one<T, TileBig>(a, st);
  return launch_wgrad_one<T, TileMid>(a, st);
}
int wgrad_tiles_per_model(int ntaps, int Cb, int Cs) {
  const int M = ntaps * Cb;
  if (M <= 64) return (M + TileWgImg::BM - 1) / TileWgImg::BM * ((Cs + TileWgImg::BN - 1) / TileWgImg::BN);
  if (Cs % 256 == 0) return (M + TileBig::BM - 1) / TileBig::BM * (Cs / TileBig::BN);
  return (M + TileMid::BM - 1) / TileMid::BM * ((Cs + TileMid::BN - 1) / TileMid::BN);
}
template void launch_wgrad<float>(const WgradArgs&, hipStream_t);
template void launch_wgrad<bf16_t>(const WgradArgs&, hipStream_t);

}  // namespace gan
