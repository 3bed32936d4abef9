// The two layers that touch the image (1..4 channels): D's first convolution and G's last transposed
// convolution, their data and weight gradients, and the one-hot label maps of D's input.  With so few image
// channels these are far below an MFMA tile and are bound by the feature-side tensor's memory traffic, so they
// are plain FMA kernels that read / write the feature tensor exactly once.
//
// A one-hot label map is a constant plane, so its contribution to D's first convolution is a per-position bias
// that only differs at the border (3 x 3 position classes), and its weight gradient is a sum of dY over the
// positions where the tap falls inside the image; both are exact, not approximations.
#include "kernels.h"

namespace gan {

struct TileLoc { int l, m0, rows, seg; long long sample_base; };

// tile id -> (model, first row in the model); false if the block has no work
__device__ inline bool locate_tile(const int* tpre, const int* offs, int L, int tile, int tile_rows, int rps, int seg,
                                   int seg_samples, TileLoc& o) {
  if (tile >= tpre[L]) return false;
  int lo = 0, hi = L;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (tpre[mid] <= tile) lo = mid; else hi = mid;
  }
  o.l = lo;
  o.m0 = (tile - tpre[lo]) * tile_rows;
  o.rows = (offs[lo + 1] - offs[lo]) * rps;
  o.seg = seg;
  o.sample_base = (long long)seg * seg_samples + offs[lo];
  return true;
}

template <typename T> __device__ inline float ldf(const T* p) { return to_float(*p); }

// ---- down: feat[row][cs] = sum_{tap, cb} img[pixel(row, tap)][cb] * w[tap][cb][cs] (+bias +label table) (LeakyReLU)
template <typename T>
__global__ __launch_bounds__(256) void skinny_down_kernel(SkinnyArgs a) {
  extern __shared__ float wl[];                      // [16][CB][Cs]
  TileLoc t;
  if (!locate_tile(a.tpre, a.offs, a.L, blockIdx.x, SKINNY_DOWN_ROWS, a.Hs * a.Hs, a.seg_first + blockIdx.y,
                   a.seg_samples, t)) return;
  const int CB = a.CB, Cs = a.Cs, Hs = a.Hs, Hb = 2 * a.Hs;
  const float* w = a.w + (long long)t.l * a.pstride;
  for (int i = threadIdx.x; i < 16 * CB * Cs; i += 256) {
    const int cs = i % Cs, tc = i / Cs, cb = tc % CB, tap = tc / CB;
    wl[i] = w[((long long)tap * a.CBT + cb) * Cs + cs];
  }
  __syncthreads();
  const int p = threadIdx.x >> 3, q = threadIdx.x & 7;
  const int cpt = Cs >> 3;                           // channels per thread: 8 or 16
  const int r = t.m0 + p;
  if (r >= t.rows) return;
  const int rps = Hs * Hs;
  const int n = r / rps, rem = r - n * rps, y = rem / Hs, x = rem - y * Hs;
  const long long sample = t.sample_base + n;
  float acc[16];
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  const int cs0 = q * cpt;
  if (a.bias) {
#pragma unroll
    for (int e = 0; e < 16; ++e)
      if (e < cpt) acc[e] = a.bias[(long long)t.l * a.pstride + cs0 + e];
  }
  if (a.table) {
    const int slot = a.sample_slot[t.sample_base - (long long)t.seg * a.seg_samples + n];
    const int cls = (y == 0 ? 0 : (y == Hs - 1 ? 2 : 1)) * 3 + (x == 0 ? 0 : (x == Hs - 1 ? 2 : 1));
    const float* tb = a.table + (((long long)t.l * a.nslot + slot) * 9 + cls) * Cs + cs0;
#pragma unroll
    for (int e = 0; e < 16; ++e)
      if (e < cpt) acc[e] += tb[e];
  }
  const T* img = static_cast<const T*>(a.img) + sample * Hb * Hb * CB;
  for (int ky = 0; ky < 4; ++ky) {
    const int iy = 2 * y - 1 + ky;
    if ((unsigned)iy >= (unsigned)Hb) continue;
    for (int kx = 0; kx < 4; ++kx) {
      const int ix = 2 * x - 1 + kx;
      if ((unsigned)ix >= (unsigned)Hb) continue;
      for (int cb = 0; cb < CB; ++cb) {
        const float v = ldf(img + ((long long)iy * Hb + ix) * CB + cb);
        const float* wr = wl + ((ky * 4 + kx) * CB + cb) * Cs + cs0;
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (e < cpt) acc[e] += v * wr[e];
      }
    }
  }
  T* out = static_cast<T*>(a.out) + (t.sample_base * rps + r) * Cs + cs0;
#pragma unroll
  for (int e = 0; e < 16; ++e)
    if (e < cpt) {
      float v = acc[e];
      if (a.lrelu) v = v > 0.f ? v : v * a.slope;
      out[e] = from_float<T>(v);
    }
}
template <typename T> void launch_skinny_down(const SkinnyArgs& a, hipStream_t st) {
  if (a.ub_tiles == 0 || a.nseg == 0) return;
  const size_t lds = (size_t)16 * a.CB * a.Cs * sizeof(float);
  hipLaunchKernelGGL((skinny_down_kernel<T>), dim3(a.ub_tiles, a.nseg), dim3(256), lds, st, a);
}
template void launch_skinny_down<float>(const SkinnyArgs&, hipStream_t);
template void launch_skinny_down<bf16_t>(const SkinnyArgs&, hipStream_t);

// ---- up: img[n, 2y+py, 2x+px][cb] = sum over (ky, kx) of matching parity, cs of feat[n, y+dy, x+dx][cs] * w[tap][cb][cs]
//      8 lanes share one small pixel (each a slice of cs) and produce its 2 x 2 output pixels.
template <typename T>
__global__ __launch_bounds__(256) void skinny_up_kernel(SkinnyArgs a) {
  extern __shared__ float wl[];                      // [16][CB][Cs]
  TileLoc t;
  if (!locate_tile(a.tpre, a.offs, a.L, blockIdx.x, SKINNY_UP_ROWS, a.Hs * a.Hs, a.seg_first + blockIdx.y,
                   a.seg_samples, t)) return;
  const int CB = a.CB, Cs = a.Cs, Hs = a.Hs, Hb = 2 * a.Hs;
  const float* w = a.w + (long long)t.l * a.pstride;
  for (int i = threadIdx.x; i < 16 * CB * Cs; i += 256) {
    const int cs = i % Cs, tc = i / Cs, cb = tc % CB, tap = tc / CB;
    wl[i] = w[((long long)tap * a.CBT + cb) * Cs + cs];
  }
  __syncthreads();
  const int p = threadIdx.x >> 3, q = threadIdx.x & 7;
  const int cpt = Cs >> 3;
  const int r = t.m0 + p;
  const bool live = r < t.rows;                      // all 8 lanes of a pixel agree; shuffles below stay inside them
  const int rps = Hs * Hs;
  const int rr = live ? r : 0;
  const int n = rr / rps, rem = rr - n * rps, y = rem / Hs, x = rem - y * Hs;
  const long long sample = t.sample_base + n;
  const int cs0 = q * cpt;
  float acc[4][4];                                   // [phase][cb]
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
  const T* feat = static_cast<const T*>(a.feat) + sample * rps * Cs;
  if (live) {
#pragma unroll
    for (int dy = -1; dy <= 1; ++dy) {
      const int iy = y + dy;
      if ((unsigned)iy >= (unsigned)Hs) continue;
#pragma unroll
      for (int dx = -1; dx <= 1; ++dx) {
        const int ix = x + dx;
        if ((unsigned)ix >= (unsigned)Hs) continue;
        float f[16];
        const T* fp = feat + ((long long)iy * Hs + ix) * Cs + cs0;
#pragma unroll
        for (int e = 0; e < 16; ++e) f[e] = (e < cpt) ? ldf(fp + e) : 0.f;
        // (py, ky) pairs that read offset dy: 2y+py = 2(y+dy) - 1 + ky
#pragma unroll
        for (int py = 0; py < 2; ++py) {
          const int ky = py + 1 - 2 * dy;
          if (ky < 0 || ky > 3) continue;
#pragma unroll
          for (int px = 0; px < 2; ++px) {
            const int kx = px + 1 - 2 * dx;
            if (kx < 0 || kx > 3) continue;
#pragma unroll
            for (int cb = 0; cb < 4; ++cb) {
              if (cb >= CB) continue;
              const float* wr = wl + ((ky * 4 + kx) * CB + cb) * Cs + cs0;
              float s = 0.f;
#pragma unroll
              for (int e = 0; e < 16; ++e)
                if (e < cpt) s += f[e] * wr[e];
              acc[py * 2 + px][cb] += s;
            }
          }
        }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float v = acc[i][j];
      v += __shfl_xor(v, 1, 64);
      v += __shfl_xor(v, 2, 64);
      v += __shfl_xor(v, 4, 64);
      acc[i][j] = v;
    }
  if (!live || q >= 4) return;
  // lane q < 4 writes output phase q
  const int py = q >> 1, px = q & 1;
  const long long o = ((sample * Hb + (2 * y + py)) * Hb + (2 * x + px)) * CB;
  T* out = static_cast<T*>(a.out);
#pragma unroll
  for (int cb = 0; cb < 4; ++cb) {
    if (cb >= CB) continue;
    float v = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (i == q) v = acc[i][cb];
    if (a.tanh_out == 1) {
      v = tanhf(v + a.bias[(long long)t.l * a.pstride + cb]);
    } else if (a.tanh_out == 2) {
      const float yv = ldf(static_cast<const T*>(a.aux) + o + cb);
      v *= (1.f - yv * yv);
    }
    out[o + cb] = from_float<T>(v);
  }
}
template <typename T> void launch_skinny_up(const SkinnyArgs& a, hipStream_t st) {
  if (a.ub_tiles == 0 || a.nseg == 0) return;
  const size_t lds = (size_t)16 * a.CB * a.Cs * sizeof(float);
  hipLaunchKernelGGL((skinny_up_kernel<T>), dim3(a.ub_tiles, a.nseg), dim3(256), lds, st, a);
}
template void launch_skinny_up<float>(const SkinnyArgs&, hipStream_t);
template void launch_skinny_up<bf16_t>(const SkinnyArgs&, hipStream_t);

// ---- wgrad: dw[tap][cb][cs] = sum_rows img[pixel(row, tap)][cb] * feat[row][cs]
//      stage 1: per (segment, tile of rows, row lane) partial sums; stage 2: add them in a fixed order.
template <typename T>
__global__ __launch_bounds__(256) void skinny_wgrad_partial_kernel(SkinnyArgs a) {
  __shared__ float imgl[32][64];                     // [row in sub-chunk][tap*CB + cb]
  TileLoc t;
  if (!locate_tile(a.tpre, a.offs, a.L, blockIdx.x, SKINNY_WGRAD_ROWS, a.Hs * a.Hs, blockIdx.y, a.seg_samples, t)) return;
  const int CB = a.CB, Cs = a.Cs, Hs = a.Hs, Hb = 2 * a.Hs, rps = Hs * Hs;
  const int nq = 256 / Cs;
  const int cs = threadIdx.x % Cs, rq = threadIdx.x / Cs;
  const int NT = 16 * CB;
  float acc[64];
#pragma unroll
  for (int i = 0; i < 64; ++i) acc[i] = 0.f;
  const T* img = static_cast<const T*>(a.img);
  const T* feat = static_cast<const T*>(a.feat) + t.sample_base * rps * Cs;
  const int rend = min(t.rows, t.m0 + SKINNY_WGRAD_ROWS);
  for (int r0 = t.m0; r0 < rend; r0 += 32) {
    __syncthreads();
    for (int i = threadIdx.x; i < 32 * NT; i += 256) {
      const int rr = i / NT, tc = i - rr * NT, tap = tc / CB, cb = tc - tap * CB;
      const int r = r0 + rr;
      float v = 0.f;
      if (r < rend) {
        const int n = r / rps, rem = r - n * rps, y = rem / Hs, x = rem - y * Hs;
        const int iy = 2 * y - 1 + (tap >> 2), ix = 2 * x - 1 + (tap & 3);
        if ((unsigned)iy < (unsigned)Hb && (unsigned)ix < (unsigned)Hb)
          v = ldf(img + (((t.sample_base + n) * Hb + iy) * Hb + ix) * CB + cb);
      }
      imgl[rr][tc] = v;
    }
    __syncthreads();
    for (int rr = rq; rr < 32; rr += nq) {
      const int r = r0 + rr;
      if (r >= rend) break;
      const float s = ldf(feat + (long long)r * Cs + cs);
#pragma unroll
      for (int i = 0; i < 64; ++i)
        if (i < NT) acc[i] += imgl[rr][i] * s;
    }
  }
  float* part = a.partial + (((long long)blockIdx.y * a.ub_tiles + blockIdx.x) * nq + rq) * NT * Cs;
#pragma unroll
  for (int i = 0; i < 64; ++i)
    if (i < NT) part[(long long)i * Cs + cs] = acc[i];
}

__global__ void skinny_wgrad_final_kernel(SkinnyArgs a) {
  const int NT = 16 * a.CB, Cs = a.Cs, nq = 256 / a.Cs;
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long long)a.L * NT * Cs) return;
  const int l = (int)(idx / (NT * Cs));
  const int rem = (int)(idx - (long long)l * NT * Cs);
  const int tc = rem / Cs, cs = rem - tc * Cs;
  if (a.offs[l + 1] == a.offs[l]) return;
  float s = 0.f;
  for (int seg = 0; seg < a.nseg; ++seg)
    for (int tile = a.tpre[l]; tile < a.tpre[l + 1]; ++tile)
      for (int q = 0; q < nq; ++q)
        s += a.partial[((((long long)seg * a.ub_tiles + tile) * nq + q) * NT + tc) * Cs + cs];
  const int tap = tc / a.CB, cb = tc - tap * a.CB;
  a.dw[(long long)l * a.pstride + ((long long)tap * a.CBT + cb) * Cs + cs] = s;
}
template <typename T> void launch_skinny_wgrad(const SkinnyArgs& a, hipStream_t st) {
  if (a.ub_tiles > 0 && a.nseg > 0)
    hipLaunchKernelGGL((skinny_wgrad_partial_kernel<T>), dim3(a.ub_tiles, a.nseg), dim3(256), 0, st, a);
  const long long tot = (long long)a.L * 16 * a.CB * a.Cs;
  hipLaunchKernelGGL(skinny_wgrad_final_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st, a);
}
template void launch_skinny_wgrad<float>(const SkinnyArgs&, hipStream_t);
template void launch_skinny_wgrad<bf16_t>(const SkinnyArgs&, hipStream_t);

// ---- dbias[cb] = sum over the model's image-side pixels (G's last layer); one block per model
template <typename T>
__global__ __launch_bounds__(256) void img_bias_grad_kernel(SkinnyArgs a) {
  __shared__ float red[256];
  const int l = blockIdx.x;
  const int cnt = a.offs[l + 1] - a.offs[l];
  if (cnt == 0) return;
  const int Hb = 2 * a.Hs;
  const long long pix = (long long)cnt * Hb * Hb;
  const T* img = static_cast<const T*>(a.img) + (long long)a.offs[l] * Hb * Hb * a.CB;
  for (int cb = 0; cb < a.CB; ++cb) {
    float s = 0.f;
    for (long long i = threadIdx.x; i < pix; i += 256) s += ldf(img + i * a.CB + cb);
    red[threadIdx.x] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
      if (threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
      __syncthreads();
    }
    if (threadIdx.x == 0) a.dbias[(long long)l * a.pstride + cb] = red[0];
    __syncthreads();
  }
}
template <typename T> void launch_img_bias_grad(const SkinnyArgs& a, hipStream_t st) {
  hipLaunchKernelGGL((img_bias_grad_kernel<T>), dim3(a.L), dim3(256), 0, st, a);
}
template void launch_img_bias_grad<float>(const SkinnyArgs&, hipStream_t);
template void launch_img_bias_grad<bf16_t>(const SkinnyArgs&, hipStream_t);

// ---- label maps -------------------------------------------------------------------------------------------
// Position class along one axis: 0 = first output row/col (tap 0 outside), 1 = interior, 2 = last (tap 3 outside).
__device__ inline bool tap_valid(int cls, int k) { return !((cls == 0 && k == 0) || (cls == 2 && k == 3)); }

__global__ void labelmap_table_kernel(LabelMapArgs a) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long tot = (long long)a.L * a.nslot * 9 * a.Cs;
  if (idx >= tot) return;
  const int cs = (int)(idx % a.Cs);
  const int cls = (int)((idx / a.Cs) % 9);
  const int slot = (int)((idx / ((long long)a.Cs * 9)) % a.nslot);
  const int l = (int)(idx / ((long long)a.Cs * 9 * a.nslot));
  const int label = (a.L == 1) ? slot : l;
  const float* w = a.w + (long long)l * a.pstride;
  float s = 0.f;
  for (int ky = 0; ky < 4; ++ky)
    for (int kx = 0; kx < 4; ++kx)
      if (tap_valid(cls / 3, ky) && tap_valid(cls % 3, kx))
        s += w[((long long)(ky * 4 + kx) * a.CBT + a.CB + label) * a.Cs + cs];
  a.table[idx] = s;
}
void launch_labelmap_table(const LabelMapArgs& a, hipStream_t st) {
  const long long tot = (long long)a.L * a.nslot * 9 * a.Cs;
  hipLaunchKernelGGL(labelmap_table_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st, a);
}

// rsum[l][slot][class][cs] = sum of dfeat over the model's rows with that slot and position class; block (slot, model)
template <typename T>
__global__ __launch_bounds__(256) void labelmap_reduce_kernel(LabelMapArgs a) {
  __shared__ float red[4][9][128];
  const int l = blockIdx.y, slot = blockIdx.x;
  const int Cs = a.Cs, Hs = a.Hs, rps = Hs * Hs;
  const int nq = 256 / Cs;
  const int cs = threadIdx.x % Cs, rq = threadIdx.x / Cs;
  const int s0 = a.offs[l], cnt = a.offs[l + 1] - s0;
  float acc[9];
#pragma unroll
  for (int i = 0; i < 9; ++i) acc[i] = 0.f;
  for (int seg = 0; seg < a.nseg; ++seg) {
    const T* df = static_cast<const T*>(a.dfeat) + ((long long)seg * a.seg_samples + s0) * rps * Cs;
    for (int n = 0; n < cnt; ++n) {
      if (a.sample_slot[s0 + n] != slot) continue;
      for (int pix = rq; pix < rps; pix += nq) {
        const int y = pix / Hs, x = pix - y * Hs;
        const int cls = (y == 0 ? 0 : (y == Hs - 1 ? 2 : 1)) * 3 + (x == 0 ? 0 : (x == Hs - 1 ? 2 : 1));
        const float v = ldf(df + ((long long)n * rps + pix) * Cs + cs);
#pragma unroll
        for (int i = 0; i < 9; ++i)
          if (i == cls) acc[i] += v;
      }
    }
  }
#pragma unroll
  for (int i = 0; i < 9; ++i) red[rq][i][cs] = acc[i];
  __syncthreads();
  for (int i = threadIdx.x; i < 9 * Cs; i += 256) {
    const int c = i % Cs, cls = i / Cs;
    float s = 0.f;
    for (int q = 0; q < nq; ++q) s += red[q][cls][c];
    a.rsum[(((long long)l * a.nslot + slot) * 9 + cls) * Cs + c] = s;
  }
}
template <typename T> void launch_labelmap_reduce(const LabelMapArgs& a, hipStream_t st) {
  hipLaunchKernelGGL((labelmap_reduce_kernel<T>), dim3(a.nslot, a.L), dim3(256), 0, st, a);
}
template void launch_labelmap_reduce<float>(const LabelMapArgs&, hipStream_t);
template void launch_labelmap_reduce<bf16_t>(const LabelMapArgs&, hipStream_t);

// dw of the label-map channels and the bias gradient from the class sums
__global__ void labelmap_grads_kernel(LabelMapArgs a) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const int Cs = a.Cs;
  const long long nw = (a.CBT > a.CB) ? (long long)a.L * a.nslot * 16 * Cs : 0;
  if (idx < nw) {
    const int cs = (int)(idx % Cs);
    const int tap = (int)((idx / Cs) % 16);
    const int slot = (int)((idx / ((long long)Cs * 16)) % a.nslot);
    const int l = (int)(idx / ((long long)Cs * 16 * a.nslot));
    if (a.offs[l + 1] == a.offs[l]) return;
    const int label = (a.L == 1) ? slot : l;
    const float* rs = a.rsum + ((long long)l * a.nslot + slot) * 9 * Cs;
    float s = 0.f;
    for (int cls = 0; cls < 9; ++cls)
      if (tap_valid(cls / 3, tap >> 2) && tap_valid(cls % 3, tap & 3)) s += rs[cls * Cs + cs];
    a.dw[(long long)l * a.pstride + ((long long)tap * a.CBT + a.CB + label) * Cs + cs] = s;
    return;
  }
  const long long j = idx - nw;
  if (j >= (long long)a.L * Cs) return;
  const int l = (int)(j / Cs), cs = (int)(j - (long long)l * Cs);
  if (a.offs[l + 1] == a.offs[l]) return;
  float s = 0.f;
  for (int slot = 0; slot < a.nslot; ++slot)
    for (int cls = 0; cls < 9; ++cls) s += a.rsum[(((long long)l * a.nslot + slot) * 9 + cls) * Cs + cs];
  a.dbias[(long long)l * a.pstride + cs] = s;
}
void launch_labelmap_grads(const LabelMapArgs& a, hipStream_t st) {
  const long long nw = (a.CBT > a.CB) ? (long long)a.L * a.nslot * 16 * a.Cs : 0;
  const long long tot = nw + (long long)a.L * a.Cs;
  hipLaunchKernelGGL(labelmap_grads_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st, a);
}

}  // namespace gan
