// Bandwidth-bound kernels of the training step: label routing, staging, BatchNorm statistics / apply / backward
// fused with the activation, D's linear head and the two logistic costs (Eq. 3, Eq. 4), Adam, layout copies.
// Every reduction has a fixed order that does not depend on the number of models, so results are deterministic
// and a model's numbers do not change with what else is in the launch.
#include "kernels.h"

namespace gan {

// ---------------------------------------------------------------------------------------------------------
// routing: stable partition of the flat batch by model
// ---------------------------------------------------------------------------------------------------------

__device__ inline int model_of_label(int y, int L) { return L == 1 ? 0 : y; }

// One block of ROUTE_CHUNKS threads does the whole partition: thread t owns the t-th run of consecutive samples.
//   1. per-(chunk, model) counts;  2. per model, the exclusive scan over the chunks (a chunk's samples of a model follow
//   those of the chunks before it: stable) and the model's total;  3. model offsets, the tile prefix of every geometry
//   and the models' order by size, each a short serial loop on its own thread(s);  4. the scatter.
// The count table lives in LDS when it fits (256 x L ints), the totals and offsets when L <= ROUTE_LDS_MODELS, the
// labels (fetched once, coalesced) when there is room left; otherwise they are the global arrays, which one block may
// use the same way (barriers order its own global accesses).  Every serial loop reads sixteen (labels: eight) values
// ahead of using them: the loops are chains of memory latencies otherwise, because a load may not pass the store in
// front of it.
constexpr int ROUTE_LDS_MODELS = 4096;
constexpr int ROUTE_LDS_CNT_BYTES = 112 * 1024;
constexpr int ROUTE_LDS_BYTES = 152 * 1024;
// (the three placements are template parameters so that every access is known to be an LDS or a global one: through
// pointers that may be either, each LDS access took several times as long)
template <bool small, bool cnt_in_lds, bool lab_in_lds>
__global__ __launch_bounds__(ROUTE_CHUNKS) void route_kernel(const int* __restrict__ label_ids, int n, int L, int n_labels,
                                                              GeomTable geoms, RouteBuffers rb) {
  extern __shared__ int route_lds[];
  static_assert(small || !cnt_in_lds, "the count table is in LDS only together with the totals");
  const int t = threadIdx.x;
  int* cl = small ? route_lds : rb.counts;                     // [L]
  int* ol = small ? route_lds + L : rb.offs;                   // [L + 1]
  int* cnt = cnt_in_lds ? route_lds + (2 * L + 1) : rb.cnt;    // [ROUTE_CHUNKS][L]
  int* labl = route_lds + (small ? 2 * L + 1 : 0) + (cnt_in_lds ? ROUTE_CHUNKS * L : 0);   // [n]
  const int* lab = lab_in_lds ? labl : label_ids;
  if (lab_in_lds)
    for (int i = t; i < n; i += 8 * ROUTE_CHUNKS) {
      int ys[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) ys[k] = i + k * ROUTE_CHUNKS < n ? label_ids[i + k * ROUTE_CHUNKS] : 0;
#pragma unroll
      for (int k = 0; k < 8; ++k)
        if (i + k * ROUTE_CHUNKS < n) labl[i + k * ROUTE_CHUNKS] = ys[k];
    }
  for (int i = t; i < ROUTE_CHUNKS * L; i += ROUTE_CHUNKS) cnt[i] = 0;
  __syncthreads();
  int* row = cnt + (long long)t * L;
  const int chunk = (n + ROUTE_CHUNKS - 1) / ROUTE_CHUNKS;
  const int i0 = min(n, t * chunk), i1 = min(n, i0 + chunk);
  bool bad = false;
  for (int i = i0; i < i1; i += 8) {
    int ys[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) ys[k] = i + k < i1 ? lab[i + k] : -1;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      if (i + k >= i1) continue;
      if (ys[k] < 0 || ys[k] >= n_labels) { bad = true; continue; }
      row[model_of_label(ys[k], L)] += 1;
    }
  }
  if (bad) rb.flags[0] = 1;
  __syncthreads();
  for (int l = t; l < L; l += ROUTE_CHUNKS) {
    int run = 0;
    for (int c0 = 0; c0 < ROUTE_CHUNKS; c0 += 16) {
      int v[16];
#pragma unroll
      for (int k = 0; k < 16; ++k) v[k] = cnt[(long long)(c0 + k) * L + l];
#pragma unroll
      for (int k = 0; k < 16; ++k) {
        cnt[(long long)(c0 + k) * L + l] = run;
        run += v[k];
      }
    }
    cl[l] = run;
    rb.counts[l] = run;
  }
  __syncthreads();
  if (t <= geoms.n && t < 64) {
    // t == 0: the model offsets; t - 1 = g: the tile prefix of geometry g
    const int g = t - 1;
    const int rps = t == 0 ? 1 : geoms.rps[g], tr = t == 0 ? 1 : geoms.tile_rows[g];
    int* dst = t == 0 ? rb.offs : rb.tpre + (long long)g * (L + 1);
    // tile heights are powers of two: a shift, not a division per model (two loops, so that the division is not
    // computed and thrown away)
    const int sh = (tr & (tr - 1)) == 0 ? __ffs(tr) - 1 : -1;
    int run = 0;
    auto prefix = [&](auto tiles_of) {
      for (int l0 = 0; l0 < L; l0 += 16) {
        int v[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) v[k] = l0 + k < L ? cl[l0 + k] : 0;
#pragma unroll
        for (int k = 0; k < 16; ++k) {
          if (l0 + k >= L) continue;
          dst[l0 + k] = run;
          if (t == 0) ol[l0 + k] = run;
          run += tiles_of(v[k]);
        }
      }
    };
    if (t == 0) prefix([](int c) { return c; });
    else if (sh >= 0) prefix([=](int c) { return (c * rps + tr - 1) >> sh; });
    else prefix([=](int c) { return (c * rps + tr - 1) / tr; });
    dst[L] = run;
    if (t == 0) ol[L] = run;
  } else if (t >= 64 && rb.order) {
    // order[rank of l] = l, rank = number of models with more samples, or as many and a smaller index
    for (int l = t - 64; l < L; l += ROUTE_CHUNKS - 64) {
      const int c = cl[l];
      int rank = 0;
      for (int j = 0; j < L; ++j) {
        const int cj = cl[j];
        rank += (cj > c || (cj == c && j < l)) ? 1 : 0;
      }
      rb.order[rank] = l;
    }
  }
  __syncthreads();
  for (int i = i0; i < i1; i += 8) {
    int ys[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) ys[k] = i + k < i1 ? lab[i + k] : -1;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      if (i + k >= i1 || ys[k] < 0 || ys[k] >= n_labels) continue;
      const int mdl = model_of_label(ys[k], L);
      const int pos = ol[mdl] + row[mdl];
      row[mdl] += 1;
      rb.perm[pos] = i + k;
      rb.sample_model[pos] = mdl;
      rb.sample_slot[pos] = (L == 1) ? ys[k] : 0;
    }
  }
}

// model of every tile of every geometry: grid (tile blocks, geometries)
__global__ void tile_model_kernel(const int* __restrict__ tpre_all, int L, int* __restrict__ tmodel_all, int stride) {
  const int* tpre = tpre_all + (long long)blockIdx.y * (L + 1);
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= tpre[L] || t >= stride) return;
  int lo = 0, hi = L;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (tpre[mid] <= t) lo = mid; else hi = mid;
  }
  tmodel_all[(long long)blockIdx.y * stride + t] = lo;
}
__global__ __launch_bounds__(256) void sum_splits_kernel(const float* __restrict__ part, float* __restrict__ dW, long long dw_stride,
                                                          long long size4, int L, int nsplit) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= size4 * L) return;
  const int l = (int)(idx / size4);
  const long long i = idx - (long long)l * size4;
  const float4* p = reinterpret_cast<const float4*>(part) + (long long)l * size4 + i;
  float4 s = p[0];
#pragma unroll 8
  for (int k = 1; k < nsplit; ++k) {
    const float4 t = p[(long long)k * L * size4];
    s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
  }
  *reinterpret_cast<float4*>(dW + (long long)l * dw_stride + 4 * i) = s;
}
void launch_sum_splits(const float* part, float* dW, long long dw_stride, long long size, int L, int nsplit, hipStream_t st) {
  if (size % 4 != 0 || dw_stride % 4 != 0 || ((uintptr_t)dW & 15) != 0 || ((uintptr_t)part & 15) != 0)
    return launch_fail("sum of row splits: sizes and pointers must be multiples of 16 bytes");
  const long long tot = size / 4 * L;
  if (tot == 0) return;
  hipLaunchKernelGGL(sum_splits_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st, part, dW, dw_stride, size / 4, L, nsplit);
}

void launch_tile_models(const int* tpre, int L, int* tmodel, int cap, hipStream_t st) {
  if (cap <= 0) return;
  hipLaunchKernelGGL(tile_model_kernel, dim3((cap + 255) / 256, 1), dim3(256), 0, st, tpre, L, tmodel, cap);
}

void launch_route(const int* label_ids, int n, int L, int n_labels, const GeomTable& geoms, const RouteBuffers& rb,
                  hipStream_t st) {
  if (geoms.n > 62) return launch_fail("routing: more tile geometries than the kernel has threads for");
  const int small = L <= ROUTE_LDS_MODELS ? 1 : 0;
  const int cnt_in_lds = small && (size_t)ROUTE_CHUNKS * L * 4 <= (size_t)ROUTE_LDS_CNT_BYTES ? 1 : 0;
  size_t lds = (small ? (size_t)(2 * L + 1) * 4 : 0) + (cnt_in_lds ? (size_t)ROUTE_CHUNKS * L * 4 : 0);
  const int lab_in_lds = lds + (size_t)n * 4 <= (size_t)ROUTE_LDS_BYTES ? 1 : 0;
  if (lab_in_lds) lds += (size_t)n * 4;
  auto go = [&](auto kernel) {
    if (lds > 48 * 1024)   // above the default dynamic limit: ask for it (idempotent, cheap)
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipLaunchKernelGGL(kernel, dim3(1), dim3(ROUTE_CHUNKS), lds, st, label_ids, n, L, n_labels, geoms, rb);
  };
  if (cnt_in_lds) { if (lab_in_lds) go(&route_kernel<true, true, true>); else go(&route_kernel<true, true, false>); }
  else if (small) { if (lab_in_lds) go(&route_kernel<true, false, true>); else go(&route_kernel<true, false, false>); }
  else { if (lab_in_lds) go(&route_kernel<false, false, true>); else go(&route_kernel<false, false, false>); }
  if (rb.tmodel && geoms.n > 0)
    hipLaunchKernelGGL(tile_model_kernel, dim3((rb.tmodel_stride + 255) / 256, geoms.n), dim3(256), 0, st, rb.tpre, L, rb.tmodel,
                       rb.tmodel_stride);
}

__global__ void tile_prefix_kernel(const int* offs, int L, int rps, int tile_rows, int* tpre) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    int run = 0;
    for (int l = 0; l < L; ++l) {
      tpre[l] = run;
      run += ((offs[l + 1] - offs[l]) * rps + tile_rows - 1) / tile_rows;
    }
    tpre[L] = run;
  }
}
void launch_tile_prefix(const int* offs, int L, int rps, int tile_rows, int* tpre, hipStream_t st) {
  hipLaunchKernelGGL(tile_prefix_kernel, dim3(1), dim3(64), 0, st, offs, L, rps, tile_rows, tpre);
}

// ---------------------------------------------------------------------------------------------------------
// staging: gather through perm, NCHW fp32 -> NHWC storage type; z | one-hot | zero padding
// ---------------------------------------------------------------------------------------------------------

template <typename T>
__global__ void stage_images_kernel(const float* __restrict__ real, const int* __restrict__ perm, const int* offs, int L,
                                    int n, int C, int HW, T* __restrict__ xd) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;   // (j, pixel)
  if (idx >= (long long)n * HW) return;
  const int j = (int)(idx / HW), pix = (int)(idx - (long long)j * HW);
  if (j >= offs[L]) return;
  const int src = perm[j];
  for (int c = 0; c < C; ++c) xd[idx * C + c] = from_float<T>(real[((long long)src * C + c) * HW + pix]);
}

template <typename T>
__global__ void stage_noise_kernel(const float* __restrict__ noise, const int* __restrict__ label_ids,
                                   const int* __restrict__ perm, const int* offs, int L, int n, int zdim, int cond_g,
                                   int kp, T* __restrict__ zin) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;   // (j, k)
  if (idx >= (long long)n * kp) return;
  const int j = (int)(idx / kp), k = (int)(idx - (long long)j * kp);
  if (j >= offs[L]) return;
  const int src = perm[j];
  float v = 0.f;
  if (k < zdim) v = noise[(long long)src * zdim + k];
  else if (k < zdim + cond_g) v = (k - zdim == label_ids[src]) ? 1.f : 0.f;
  zin[idx] = from_float<T>(v);
}

template <typename T>
void launch_stage(const int* label_ids, const float* noise, const float* real, int n, int L, int zdim, int cond_g, int kp,
                  int img_c, int img_hw, const RouteBuffers& rb, T* zin, T* xd, hipStream_t st) {
  if (n == 0) return;
  const int HW = img_hw * img_hw;
  if (real) {
    const long long tot = (long long)n * HW;
    hipLaunchKernelGGL((stage_images_kernel<T>), dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st, real, rb.perm,
                       rb.offs, L, n, img_c, HW, xd);
  }
  const long long tot = (long long)n * kp;
  hipLaunchKernelGGL((stage_noise_kernel<T>), dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st, noise, label_ids,
                     rb.perm, rb.offs, L, n, zdim, cond_g, kp, zin);
}
template void launch_stage<float>(const int*, const float*, const float*, int, int, int, int, int, int, int,
                                  const RouteBuffers&, float*, float*, hipStream_t);
template void launch_stage<bf16_t>(const int*, const float*, const float*, int, int, int, int, int, int, int,
                                   const RouteBuffers&, bf16_t*, bf16_t*, hipStream_t);

template <typename T>
__global__ void unstage_kernel(const T* __restrict__ fake, const int* __restrict__ perm, const int* offs, int L, int n, int C,
                               int HW, float* __restrict__ out) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long long)n * HW) return;
  const int j = (int)(idx / HW), pix = (int)(idx - (long long)j * HW);
  if (j >= offs[L]) return;
  const int dst = perm[j];
  for (int c = 0; c < C; ++c) out[((long long)dst * C + c) * HW + pix] = to_float(fake[idx * C + c]);
}
template <typename T>
void launch_unstage(const T* fake, float* out, int n, int L, int img_c, int img_hw, const RouteBuffers& rb, hipStream_t st) {
  if (n == 0) return;
  const int HW = img_hw * img_hw;
  const long long tot = (long long)n * HW;
  hipLaunchKernelGGL((unstage_kernel<T>), dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st, fake, rb.perm, rb.offs,
                     L, n, img_c, HW, out);
}
template void launch_unstage<float>(const float*, float*, int, int, int, int, const RouteBuffers&, hipStream_t);
template void launch_unstage<bf16_t>(const bf16_t*, float*, int, int, int, int, const RouteBuffers&, hipStream_t);

// ---------------------------------------------------------------------------------------------------------
// BatchNorm
// ---------------------------------------------------------------------------------------------------------

// Loads 4 consecutive channels as floats.
__device__ inline void load4(const float* p, float (&v)[4]) {
  const float4 t = *reinterpret_cast<const float4*>(p);
  v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
}
__device__ inline void load4(const bf16_t* p, float (&v)[4]) {
  const uint2 t = *reinterpret_cast<const uint2*>(p);
  v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xffff0000u);
  v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xffff0000u);
}
__device__ inline void store4(float* p, const float (&v)[4]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
}
__device__ inline void store4(bf16_t* p, const float (&v)[4]) {
  uint2 t;
  t.x = pack2_bf16(v[0], v[1]);
  t.y = pack2_bf16(v[2], v[3]);
  *reinterpret_cast<uint2*>(p) = t;
}

// 16 bytes of consecutive channels as floats: 4 (fp32) or 8 (bf16).
template <typename T> struct Vec16 { static constexpr int N = 16 / (int)sizeof(T); };
__device__ inline void loadv(const float* p, float (&v)[4]) { load4(p, v); }
__device__ inline void loadv(const bf16_t* p, float (&v)[8]) {
  typedef unsigned u4 __attribute__((ext_vector_type(4)));
  const u4 t = __builtin_nontemporal_load(reinterpret_cast<const u4*>(p));
  v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xffff0000u);
  v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xffff0000u);
  v[4] = __uint_as_float(t.z << 16); v[5] = __uint_as_float(t.z & 0xffff0000u);
  v[6] = __uint_as_float(t.w << 16); v[7] = __uint_as_float(t.w & 0xffff0000u);
}
__device__ inline void storev(float* p, const float (&v)[4]) { store4(p, v); }
__device__ inline void storev(bf16_t* p, const float (&v)[8]) {
  uint4 t;
  t.x = pack2_bf16(v[0], v[1]);
  t.y = pack2_bf16(v[2], v[3]);
  t.z = pack2_bf16(v[4], v[5]);
  t.w = pack2_bf16(v[6], v[7]);
  typedef unsigned u4 __attribute__((ext_vector_type(4)));
  u4 q; q.x = t.x; q.y = t.y; q.z = t.z; q.w = t.w;
  __builtin_nontemporal_store(q, reinterpret_cast<u4*>(p));
}

// mean / var / rstd from what the producing GEMM left per sub-tile and column: (sum, sum of squared deviations from
// the sub-tile's mean); a tile of tile_rows rows is wsplit sub-tiles of tile_rows / wsplit rows, the last ones of a
// model's last tile possibly empty.  Sub-tiles (and output phases, and column runs) of one (segment, model) are merged
// in a fixed order with the pairwise update  mean += d n_t/(n+n_t),  M2 += M2_t + d^2 n n_t/(n+n_t),  d = mean_t - mean.
// The GEMM's N columns are `groups` runs of the C channels (the linear layer feeding G's first BatchNorm has one
// run per pixel of the first feature map; the convolutions have one).
// A block = 16 channels x RED_SLICES slices of the (phase, sub-tile) sequence of one (segment, model): every thread
// merges its contiguous slice in order, then the slices are merged in order.  The slicing depends on the model's own
// tile count only.
constexpr int RED_SLICES = 16;      // slices of the backward reduction's second stage
// Threads of a block = SL slices x CX channels.  16 x 16 as a rule; 64 x 4 when a model has so many tiles (one pair
// over the whole batch) that sixteen chains of dependent merges would be the whole kernel.  The choice follows from
// the configuration (tile bound per model), never from a batch.
template <int SL, int CX>
__global__ __launch_bounds__(256) void bn_stats_from_partial_kernel(NormArgs a, const float* __restrict__ partial,
                                                                    const int* __restrict__ tpre, int ub_tiles, int nphase,
                                                                    int groups, int tile_rows, int gemm_rps, int wsplit) {
  static_assert(SL * CX == 256, "block shape");
  __shared__ float sh[SL][CX][3];
  const int cx = threadIdx.x % CX, sl = threadIdx.x / CX;
  const int cblocks = (a.C + CX - 1) / CX;
  const int c = (blockIdx.x % cblocks) * CX + cx;
  const int l = (blockIdx.x / cblocks) % a.L;
  const int sidx = blockIdx.x / (cblocks * a.L);
  const int cnt = a.offs[l + 1] - a.offs[l];
  if (cnt == 0) return;                                // block-uniform
  const int rows = cnt * gemm_rps;                     // rows of this model in the GEMM's row space (per phase)
  const int t0 = tpre[l], nsub = (tpre[l + 1] - t0) * wsplit, sub_rows = tile_rows / wsplit;
  // the sequence a slice is cut from: (phase, sub-tile, column run), the column runs fastest
  const int seq = nphase * nsub * groups, per = (seq + SL - 1) / SL;
  float n = 0.f, mean = 0.f, m2 = 0.f;
  const float inv_sub = 1.f / (float)sub_rows;
  if (c < a.C)
#pragma unroll 4
    for (int qg = sl * per; qg < min(seq, (sl + 1) * per); ++qg) {  // (unrolled: the loads of four entries are in flight together)
      const int q = qg / groups, g = qg - q * groups;
      const int ph = q / nsub, t = q - ph * nsub;
      const int left = rows - t * sub_rows;
      if (left <= 0) continue;                         // an empty sub-tile at the end of the model's last tile: never written
      const float nt = (float)min(sub_rows, left);
      const long long o = ((((long long)ph * a.nseg + sidx) * ub_tiles * wsplit + (long long)t0 * wsplit + t) * ((long long)a.C * groups) + g * a.C + c) * 2;
      // one division per merge: a full sub-tile's mean through the reciprocal of its height, the second weight from the first
      const float d = (left >= sub_rows ? partial[o] * inv_sub : partial[o] / nt) - mean;
      const float nn = n + nt;
      const float w = nt / nn;
      mean += d * w;
      m2 += partial[o + 1] + d * d * (n * w);
      n = nn;
    }
  sh[sl][cx][0] = n; sh[sl][cx][1] = mean; sh[sl][cx][2] = m2;
  __syncthreads();
  if (sl != 0 || c >= a.C) return;
  for (int k = 1; k < SL; ++k) {
    const float nt = sh[k][cx][0];
    if (nt == 0.f) continue;                           // an empty slice
    const float d = sh[k][cx][1] - mean;
    const float nn = n + nt;
    const float w = nt / nn;
    mean += d * w;
    m2 += sh[k][cx][2] + d * d * (n * w);
    n = nn;
  }
  const float var = m2 / n;
  const long long o = (long long)((a.seg_first + sidx) * a.L + l) * a.C + c;
  a.mean[o] = mean;
  a.var[o] = var;
  a.rstd[o] = 1.0f / sqrtf(var + a.eps);
  if (a.fold_running) {     // one segment: what bn_running_kernel would do next, without the launch
    const long long S = (long long)cnt * a.rps;
    const long long ro = (long long)l * a.rstride + c;
    a.run_mean[ro] = (1.f - a.momentum) * a.run_mean[ro] + a.momentum * mean;
    if (S > 1) a.run_var[ro] = (1.f - a.momentum) * a.run_var[ro] + a.momentum * var * ((float)S / (float)(S - 1));
  }
}
void launch_bn_stats_from_partial(const NormArgs& a, const float* partial, const int* tpre, int ub_tiles, int nphase,
                                  int groups, int tile_rows, int gemm_rps, int wsplit, hipStream_t st) {
  if ((long long)a.nseg * a.L * a.C == 0) return;
  if (!tpre || !partial) return launch_fail("BatchNorm statistics: no tile prefix array or no partial sums");
  if (wsplit < 1 || tile_rows % wsplit) return launch_fail("BatchNorm statistics: the tile height is not a whole number of sub-tiles");
  const bool many = (long long)ub_tiles * wsplit * nphase * groups > 1024LL * a.L;       // entries per model, by the launch's upper bound
  if (many) {
    const long long tot = (long long)a.nseg * a.L * ((a.C + 3) / 4);
    hipLaunchKernelGGL((bn_stats_from_partial_kernel<64, 4>), dim3((unsigned)tot), dim3(256), 0, st, a, partial, tpre, ub_tiles, nphase,
                       groups, tile_rows, gemm_rps, wsplit);
  } else {
    const long long tot = (long long)a.nseg * a.L * ((a.C + 15) / 16);
    hipLaunchKernelGGL((bn_stats_from_partial_kernel<16, 16>), dim3((unsigned)tot), dim3(256), 0, st, a, partial, tpre, ub_tiles, nphase,
                       groups, tile_rows, gemm_rps, wsplit);
  }
}

// running <- (1 - momentum) running + momentum * batch, once per segment in order; unbiased variance stored.
__global__ void bn_running_kernel(NormArgs a) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= a.L * a.C) return;
  const int l = idx / a.C, c = idx - l * a.C;
  const int cnt = a.offs[l + 1] - a.offs[l];
  if (cnt == 0) return;
  const long long S = (long long)cnt * a.rps;
  float rm = a.run_mean[(long long)l * a.rstride + c], rv = a.run_var[(long long)l * a.rstride + c];
  for (int s = 0; s < a.nseg; ++s) {
    const long long o = (long long)((a.seg_first + s) * a.L + l) * a.C + c;
    rm = (1.f - a.momentum) * rm + a.momentum * a.mean[o];
    if (S > 1) rv = (1.f - a.momentum) * rv + a.momentum * a.var[o] * ((float)S / (float)(S - 1));
  }
  a.run_mean[(long long)l * a.rstride + c] = rm;
  a.run_var[(long long)l * a.rstride + c] = rv;
}
void launch_bn_running(const NormArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(bn_running_kernel, dim3((a.L * a.C + 255) / 256), dim3(256), 0, st, a);
}

__global__ void bn_from_running_kernel(NormArgs a) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= a.L * a.C) return;
  const int l = idx / a.C, c = idx - l * a.C;
  const long long o = (long long)(a.seg_first * a.L + l) * a.C + c;
  const float rv = a.run_var[(long long)l * a.rstride + c];
  a.mean[o] = a.run_mean[(long long)l * a.rstride + c];
  a.var[o] = rv;
  a.rstd[o] = 1.0f / sqrtf(rv + a.eps);
}
void launch_bn_from_running(const NormArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(bn_from_running_kernel, dim3((a.L * a.C + 255) / 256), dim3(256), 0, st, a);
}

// y = act(gamma * (x - mean) * rstd + beta).  One block per (sample, segment): a thread keeps the parameters of its
// 16 bytes of channels in registers and walks down the sample's rows.
template <typename T>
__global__ __launch_bounds__(256) void bn_apply_kernel(NormArgs a) {
  constexpr int EPV = Vec16<T>::N;
  const int j = blockIdx.x, sidx = blockIdx.y;
  if (j >= a.offs[a.L]) return;
  const int l = a.sample_model[j];
  const int seg = a.seg_first + sidx;
  const int cg = a.C / EPV;                           // channel groups per row
  const long long base = ((long long)seg * a.seg_samples + j) * a.rps * a.C;
  const T* x = static_cast<const T*>(a.x) + base;
  T* y = static_cast<T*>(a.y) + base;
  const long long so = (long long)(seg * a.L + l) * a.C;
  // a thread's channel group is fixed when the block's thread count is a multiple of cg (the usual case); otherwise
  // it changes from pass to pass and the parameters are reloaded
  const int total = a.rps * cg;
  int cur = -1;
  float sc[EPV], mu[EPV], be[EPV];
  for (int t = threadIdx.x; t < total; t += 256) {
    const int r = t / cg, g = t - r * cg;
    if (g != cur) {
      cur = g;
#pragma unroll
      for (int k = 0; k < EPV; ++k) {
        const int c = g * EPV + k;
        sc[k] = a.gamma[(long long)l * a.pstride + c] * a.rstd[so + c];
        mu[k] = a.mean[so + c];
        be[k] = a.beta[(long long)l * a.pstride + c];
      }
    }
    float v[EPV];
    loadv(x + (long long)r * a.C + g * EPV, v);
#pragma unroll
    for (int k = 0; k < EPV; ++k) {
      const float u = (v[k] - mu[k]) * sc[k] + be[k];
      v[k] = u > 0.f ? u : u * a.slope;
    }
    storev(y + (long long)r * a.C + g * EPV, v);
  }
}
template <typename T> void launch_bn_apply(const NormArgs& a, hipStream_t st) {
  if (a.n == 0 || a.nseg == 0) return;
  hipLaunchKernelGGL((bn_apply_kernel<T>), dim3((unsigned)a.n, (unsigned)a.nseg), dim3(256), 0, st, a);
}
template void launch_bn_apply<float>(const NormArgs&, hipStream_t);
template void launch_bn_apply<bf16_t>(const NormArgs&, hipStream_t);

// sums[g][c] = (sum g, sum g * xhat) with g = dy * act'(u), u = gamma * xhat + beta.
// Stage 1: block (tile of BN_RED_ROWS rows of one model, segment), all channels -> partial[segment][tile][C][2].
// Stage 2: the tiles of a (segment, model) added in order.
template <typename T>
__global__ __launch_bounds__(256) void bn_bwd_reduce_kernel(NormArgs a, const int* __restrict__ tpre, const int* __restrict__ tmodel,
                                                            int ub_tiles, float* __restrict__ partial) {
  constexpr int EPV = Vec16<T>::N;
  extern __shared__ float red[];                    // [2][RL][C]
  const int tile = blockIdx.x;
  if (tile >= tpre[a.L]) return;
  int lo = 0;
  if (tmodel) {
    lo = tmodel[tile];
  } else {
    int hi = a.L;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (tpre[mid] <= tile) lo = mid; else hi = mid;
    }
  }
  const int l = lo, sidx = blockIdx.y;
  const int seg = a.seg_first + sidx;
  const int cnt = a.offs[l + 1] - a.offs[l];
  const int g = seg * a.L + l;
  const int cg = a.C / EPV;                         // channel lanes (<= 256, a divisor of 256 or not)
  const int RL = 256 / cg;                          // row lanes
  const int cl = threadIdx.x % cg, rl = threadIdx.x / cg;
  const long long rows = (long long)cnt * a.rps;
  const long long r0 = (long long)(tile - tpre[l]) * BN_RED_ROWS;
  const long long r1 = min(rows, r0 + BN_RED_ROWS);
  const long long base = ((long long)seg * a.seg_samples + a.offs[l]) * a.rps * a.C + cl * EPV;
  const T* x = static_cast<const T*>(a.x) + base;
  const T* dy = static_cast<const T*>(a.dy) + base;
  float mu[EPV], rs[EPV], ga[EPV], be[EPV], sg[EPV], sgx[EPV];
#pragma unroll
  for (int e = 0; e < EPV; ++e) {
    const int c = cl * EPV + e;
    mu[e] = a.mean[(long long)g * a.C + c];
    rs[e] = a.rstd[(long long)g * a.C + c];
    ga[e] = a.gamma[(long long)l * a.pstride + c];
    be[e] = a.beta[(long long)l * a.pstride + c];
    sg[e] = 0.f;
    sgx[e] = 0.f;
  }
  if (rl < RL) {
    // four rows per trip: eight 16-byte loads in flight per thread (the sums stay in row order)
    long long r = r0 + rl;
    for (; r + 3 * RL < r1; r += 4 * RL) {
      float v[4][EPV], d[4][EPV];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        loadv(x + (r + k * RL) * a.C, v[k]);
        loadv(dy + (r + k * RL) * a.C, d[k]);
      }
#pragma unroll
      for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
          const float xh = (v[k][e] - mu[e]) * rs[e];
          const float u = ga[e] * xh + be[e];
          const float gg = u > 0.f ? d[k][e] : d[k][e] * a.slope;
          sg[e] += gg;
          sgx[e] += gg * xh;
        }
    }
    for (; r < r1; r += RL) {
      float v[EPV], d[EPV];
      loadv(x + r * a.C, v);
      loadv(dy + r * a.C, d);
#pragma unroll
      for (int e = 0; e < EPV; ++e) {
        const float xh = (v[e] - mu[e]) * rs[e];
        const float u = ga[e] * xh + be[e];
        const float gg = u > 0.f ? d[e] : d[e] * a.slope;
        sg[e] += gg;
        sgx[e] += gg * xh;
      }
    }
#pragma unroll
    for (int e = 0; e < EPV; ++e) {
      red[(0 * RL + rl) * a.C + cl * EPV + e] = sg[e];
      red[(1 * RL + rl) * a.C + cl * EPV + e] = sgx[e];
    }
  }
  __syncthreads();
  for (int t = threadIdx.x; t < 2 * a.C; t += 256) {
    const int w = t / a.C, c = t - w * a.C;
    float acc = 0.f;
    for (int i = 0; i < RL; ++i) acc += red[(w * RL + i) * a.C + c];
    partial[(((long long)sidx * ub_tiles + tile) * a.C + c) * 2 + w] = acc;
  }
}
__global__ __launch_bounds__(256) void bn_bwd_reduce_final_kernel(NormArgs a, const int* __restrict__ tpre, int ub_tiles,
                                                                  const float* __restrict__ partial) {
  __shared__ float sh[RED_SLICES][16][2];
  const int cx = threadIdx.x & 15, sl = threadIdx.x >> 4;
  const int cblocks = (a.C + 15) / 16;
  const int c = (blockIdx.x % cblocks) * 16 + cx;
  const int l = (blockIdx.x / cblocks) % a.L;
  const int sidx = blockIdx.x / (cblocks * a.L);
  if (a.offs[l + 1] == a.offs[l]) return;              // block-uniform
  const int t0 = tpre[l], ntiles = tpre[l + 1] - t0;
  const int per = (ntiles + RED_SLICES - 1) / RED_SLICES;
  float s0 = 0.f, s1 = 0.f;
  if (c < a.C)
#pragma unroll 8
    for (int t = t0 + sl * per; t < t0 + min(ntiles, (sl + 1) * per); ++t) {     // (eight tiles' loads in flight, added in order)
      const long long o = (((long long)sidx * ub_tiles + t) * a.C + c) * 2;
      s0 += partial[o];
      s1 += partial[o + 1];
    }
  sh[sl][cx][0] = s0; sh[sl][cx][1] = s1;
  __syncthreads();
  if (sl != 0 || c >= a.C) return;
  for (int k = 1; k < RED_SLICES; ++k) { s0 += sh[k][cx][0]; s1 += sh[k][cx][1]; }
  const long long o = ((long long)((a.seg_first + sidx) * a.L + l) * a.C + c) * 2;
  a.sums[o] = s0;
  a.sums[o + 1] = s1;
  if (a.fold_grads) {       // one segment: what bn_param_grad_kernel would do next, without the launch
    a.dbeta[(long long)l * a.pstride + c] = 0.f + s0;
    a.dgamma[(long long)l * a.pstride + c] = 0.f + s1;
  }
}
template <typename T>
void launch_bn_bwd_reduce(const NormArgs& a, const int* tpre, const int* tmodel, int ub_tiles, float* partial, hipStream_t st) {
  if (a.nseg == 0 || ub_tiles == 0) return;
  if (!tpre) return launch_fail("BatchNorm backward: no tile prefix array");
  const int cg = a.C / Vec16<T>::N;
  if (cg < 1 || cg > 256) return launch_fail("BatchNorm backward: one thread per 16 bytes of a row needs at most 256 of them");
  const size_t lds = (size_t)2 * (256 / cg) * a.C * sizeof(float);
  hipLaunchKernelGGL((bn_bwd_reduce_kernel<T>), dim3(ub_tiles, a.nseg), dim3(256), lds, st, a, tpre, tmodel, ub_tiles, partial);
  const long long tot = (long long)a.nseg * a.L * ((a.C + 15) / 16);
  hipLaunchKernelGGL(bn_bwd_reduce_final_kernel, dim3((unsigned)tot), dim3(256), 0, st, a, tpre, ub_tiles, partial);
}
template void launch_bn_bwd_reduce<float>(const NormArgs&, const int*, const int*, int, float*, hipStream_t);
template void launch_bn_bwd_reduce<bf16_t>(const NormArgs&, const int*, const int*, int, float*, hipStream_t);

// dgamma, dbeta: the segments' sums added in order.
__global__ void bn_param_grad_kernel(NormArgs a) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= a.L * a.C) return;
  const int l = idx / a.C, c = idx - l * a.C;
  if (a.offs[l + 1] == a.offs[l]) return;
  float db = 0.f, dg = 0.f;
  for (int s = 0; s < a.nseg; ++s) {
    const long long o = ((long long)((a.seg_first + s) * a.L + l) * a.C + c) * 2;
    db += a.sums[o];
    dg += a.sums[o + 1];
  }
  a.dbeta[(long long)l * a.pstride + c] = db;
  a.dgamma[(long long)l * a.pstride + c] = dg;
}
void launch_bn_param_grad(const NormArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(bn_param_grad_kernel, dim3((a.L * a.C + 255) / 256), dim3(256), 0, st, a);
}

// dx = gamma * rstd * (g - sum_g / S - xhat * sum_gx / S).  Same block shape as the forward pass.
template <typename T>
__global__ __launch_bounds__(256) void bn_bwd_apply_kernel(NormArgs a) {
  constexpr int EPV = Vec16<T>::N;
  const int j = blockIdx.x, sidx = blockIdx.y;
  if (j >= a.offs[a.L]) return;
  const int l = a.sample_model[j];
  const int seg = a.seg_first + sidx;
  const int cg = a.C / EPV;
  const float invS = 1.0f / ((float)(a.offs[l + 1] - a.offs[l]) * (float)a.rps);
  const long long base = ((long long)seg * a.seg_samples + j) * a.rps * a.C;
  const T* x = static_cast<const T*>(a.x) + base;
  const T* dy = static_cast<const T*>(a.dy) + base;
  T* dx = static_cast<T*>(a.y) + base;
  const long long so = (long long)(seg * a.L + l) * a.C;
  const int total = a.rps * cg;
  int cur = -1;
  float rs[EPV], ga[EPV], mu[EPV], be[EPV], s1[EPV], s2[EPV];
  for (int t = threadIdx.x; t < total; t += 256) {
    const int r = t / cg, g = t - r * cg;
    if (g != cur) {
      cur = g;
#pragma unroll
      for (int k = 0; k < EPV; ++k) {
        const int c = g * EPV + k;
        rs[k] = a.rstd[so + c];
        ga[k] = a.gamma[(long long)l * a.pstride + c];
        mu[k] = a.mean[so + c];
        be[k] = a.beta[(long long)l * a.pstride + c];
        s1[k] = a.sums[(so + c) * 2] * invS;
        s2[k] = a.sums[(so + c) * 2 + 1] * invS;
      }
    }
    float v[EPV], d[EPV];
    loadv(x + (long long)r * a.C + g * EPV, v);
    loadv(dy + (long long)r * a.C + g * EPV, d);
#pragma unroll
    for (int k = 0; k < EPV; ++k) {
      const float xh = (v[k] - mu[k]) * rs[k];
      const float u = ga[k] * xh + be[k];
      const float gg = u > 0.f ? d[k] : d[k] * a.slope;
      v[k] = ga[k] * rs[k] * (gg - s1[k] - xh * s2[k]);
    }
    storev(dx + (long long)r * a.C + g * EPV, v);
  }
}
template <typename T> void launch_bn_bwd_apply(const NormArgs& a, hipStream_t st) {
  if (a.n == 0 || a.nseg == 0) return;
  hipLaunchKernelGGL((bn_bwd_apply_kernel<T>), dim3((unsigned)a.n, (unsigned)a.nseg), dim3(256), 0, st, a);
}
template void launch_bn_bwd_apply<float>(const NormArgs&, hipStream_t);
template void launch_bn_bwd_apply<bf16_t>(const NormArgs&, hipStream_t);

// ---------------------------------------------------------------------------------------------------------
// D's linear head, the costs, and their gradients
// ---------------------------------------------------------------------------------------------------------

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// one wave per row: logit = <feat[row], w[model]> + b[model]
template <typename T>
__global__ __launch_bounds__(256) void head_fwd_kernel(HeadArgs a) {
  const int lane = threadIdx.x & 63;
  const long long wrow = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (wrow >= (long long)a.n * a.nseg) return;
  const int sidx = (int)(wrow / a.n), j = (int)(wrow - (long long)sidx * a.n);
  if (j >= a.offs[a.L]) return;
  const int l = a.sample_model[j];
  const long long r = (long long)(a.seg_first + sidx) * a.seg_samples + j;
  const T* f = static_cast<const T*>(a.feat) + r * a.K;
  const float* w = a.w + (long long)l * a.pstride;
  float acc = 0.f;
#pragma unroll 8
  for (int k = lane * 4; k < a.K; k += 256) {     // (eight steps' loads in flight, added in order)
    float v[4];
    load4(f + k, v);
    const float4 ww = *reinterpret_cast<const float4*>(w + k);
    acc += v[0] * ww.x + v[1] * ww.y + v[2] * ww.z + v[3] * ww.w;
  }
  acc = wave_sum(acc);
  if (lane == 0) a.logits[r] = acc + a.b[(long long)l * a.pstride];
}
template <typename T> void launch_head_fwd(const HeadArgs& a, hipStream_t st) {
  const long long rows = (long long)a.n * a.nseg;
  if (rows == 0) return;
  hipLaunchKernelGGL((head_fwd_kernel<T>), dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, a);
}
template void launch_head_fwd<float>(const HeadArgs&, hipStream_t);
template void launch_head_fwd<bf16_t>(const HeadArgs&, hipStream_t);

__device__ inline float softplus_f(float u) { return fmaxf(u, 0.f) + log1pf(expf(-fabsf(u))); }
__device__ inline float sigmoid_f(float u) {
  if (u >= 0.f) return 1.f / (1.f + expf(-u));
  const float e = expf(u);
  return e / (1.f + e);
}

// One block per model.  mode 0 (Eq. 3): J_D = scale*mean softplus(-s_real) + scale*mean softplus(s_fake),
// segments (0, 1).  mode 1 (Eq. 4, negated): scale*mean softplus(-s_fake') on segment seg_first.
__global__ __launch_bounds__(256) void loss_kernel(HeadArgs a) {
  __shared__ float red[256];
  const int l = blockIdx.x;
  const int s0 = a.offs[l], cnt = a.offs[l + 1] - s0;
  if (cnt == 0) { if (threadIdx.x == 0) a.loss[l] = 0.f; return; }
  const float inv = 1.f / (float)cnt;
  float acc = 0.f;
  for (int s = 0; s < a.nseg; ++s) {
    const int seg = a.seg_first + s;
    const float sign = (a.mode == 0 && seg == 1) ? 1.f : -1.f;
    for (int i = threadIdx.x; i < cnt; i += 256) {
      const long long r = (long long)seg * a.seg_samples + s0 + i;
      const float u = sign * a.logits[r];
      acc += softplus_f(u);
      a.dlogits[r] = a.scale * sign * sigmoid_f(u) * inv;
    }
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) a.loss[l] = a.scale * red[0] * inv;
}
void launch_loss(const HeadArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(loss_kernel, dim3(a.L), dim3(256), 0, st, a);
}

// dfeat[row][k] = dlogit[row] * w[model][k]; a thread takes 8 consecutive k of one row (K is a multiple of 8: the
// feature maps have whole 64-channel lines), blockIdx.y the segment; 32-bit index arithmetic (the launcher checks).
template <typename T>
__global__ __launch_bounds__(256) void head_bwd_data_kernel(HeadArgs a) {
  const unsigned k8 = (unsigned)a.K >> 3;
  const unsigned idx = blockIdx.x * 256u + threadIdx.x;
  const unsigned j = idx / k8;
  if (j >= (unsigned)a.n || (int)j >= a.offs[a.L]) return;
  const int k = (int)(idx - j * k8) * 8;
  const int l = a.sample_model[j];
  const long long r = (long long)(a.seg_first + (int)blockIdx.y) * a.seg_samples + j;
  const float d = a.dlogits[r];
  const float* w = a.w + (long long)l * a.pstride + k;
  const float4 w0 = *reinterpret_cast<const float4*>(w), w1 = *reinterpret_cast<const float4*>(w + 4);
  const float v[8] = {d * w0.x, d * w0.y, d * w0.z, d * w0.w, d * w1.x, d * w1.y, d * w1.z, d * w1.w};
  T* dst = static_cast<T*>(a.dfeat) + r * a.K + k;
  if constexpr (sizeof(T) == 2) {
    storev(dst, v);
  } else {
    *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4*>(dst + 4) = make_float4(v[4], v[5], v[6], v[7]);
  }
}
template <typename T> void launch_head_bwd_data(const HeadArgs& a, hipStream_t st) {
  const long long tot = (long long)a.n * (a.K / 8);
  if (tot == 0 || a.nseg == 0) return;
  if (a.K % 8 != 0 || tot + 256 >= (1LL << 32)) return launch_fail("head data gradient: K must be a multiple of 8 and n * K / 8 below 2^32");
  hipLaunchKernelGGL((head_bwd_data_kernel<T>), dim3((unsigned)((tot + 255) / 256), (unsigned)a.nseg), dim3(256), 0, st, a);
}
template void launch_head_bwd_data<float>(const HeadArgs&, hipStream_t);
template void launch_head_bwd_data<bf16_t>(const HeadArgs&, hipStream_t);

// dw[model][k] = sum_rows dlogit[row] * feat[row][k] ; db = sum_rows dlogit.  Block (k chunk of 1024, model).
template <typename T>
__global__ __launch_bounds__(256) void head_bwd_w_kernel(HeadArgs a) {
  const int l = blockIdx.y;
  const int s0 = a.offs[l], cnt = a.offs[l + 1] - s0;
  if (cnt == 0) return;
  const int k = blockIdx.x * 1024 + threadIdx.x * 4;
  const int rsplit = a.rsplit > 1 ? a.rsplit : 1, sp = blockIdx.z;
  const int per = (cnt + rsplit - 1) / rsplit;
  const int i0 = sp * per, i1 = min(cnt, i0 + per);
  float acc[4] = {0, 0, 0, 0}, accb = 0.f;
  for (int s = 0; s < a.nseg; ++s) {
    const long long r0 = (long long)(a.seg_first + s) * a.seg_samples + s0;
#pragma unroll 8
    for (int i = i0; i < i1; ++i) {               // (eight rows' loads in flight, added in order)
      const float d = a.dlogits[r0 + i];
      accb += d;
      if (k < a.K) {
        float v[4];
        load4(static_cast<const T*>(a.feat) + (r0 + i) * a.K + k, v);
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] += d * v[e];
      }
    }
  }
  if (rsplit > 1) {
    float* part = a.part + ((long long)sp * a.L + l) * (a.K + 4);
    if (k < a.K) *reinterpret_cast<float4*>(part + k) = make_float4(acc[0], acc[1], acc[2], acc[3]);
    if (blockIdx.x == 0 && threadIdx.x == 0) part[a.K] = accb;
    return;
  }
  if (k < a.K) *reinterpret_cast<float4*>(a.dw + (long long)l * a.pstride + k) = make_float4(acc[0], acc[1], acc[2], acc[3]);
  if (blockIdx.x == 0 && threadIdx.x == 0) a.db[(long long)l * a.pstride] = accb;
}
// the row splits' partial sums, added in order (index K: the bias term)
__global__ void head_bwd_w_final_kernel(HeadArgs a) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long long)a.L * (a.K + 1)) return;
  const int l = (int)(idx / (a.K + 1)), k = (int)(idx - (long long)l * (a.K + 1));
  if (a.offs[l + 1] == a.offs[l]) return;
  float s = 0.f;
#pragma unroll 8
  for (int sp = 0; sp < a.rsplit; ++sp) s += a.part[((long long)sp * a.L + l) * (a.K + 4) + k];     // loads in flight together, sum in order
  if (k < a.K) a.dw[(long long)l * a.pstride + k] = s;
  else a.db[(long long)l * a.pstride] = s;
}
template <typename T> void launch_head_bwd_w(const HeadArgs& a, hipStream_t st) {
  if (a.K % 4 != 0 || (a.rsplit > 1 && !a.part)) return launch_fail("linear head: feature count not a multiple of 4, or no buffer for the row splits");
  const int rsplit = a.rsplit > 1 ? a.rsplit : 1;
  hipLaunchKernelGGL((head_bwd_w_kernel<T>), dim3((a.K + 1023) / 1024, a.L, rsplit), dim3(256), 0, st, a);
  if (rsplit > 1) {
    const long long tot = (long long)a.L * (a.K + 1);
    hipLaunchKernelGGL(head_bwd_w_final_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, st, a);
  }
}
template void launch_head_bwd_w<float>(const HeadArgs&, hipStream_t);
template void launch_head_bwd_w<bf16_t>(const HeadArgs&, hipStream_t);

// ---------------------------------------------------------------------------------------------------------
// Adam (bias-corrected, epsilon outside the root), all models and tensors of one network in one sweep
// ---------------------------------------------------------------------------------------------------------

__global__ void adam_prepare_kernel(AdamArgs a) {
  const int l = blockIdx.x * blockDim.x + threadIdx.x;
  if (l >= a.L) return;
  if (a.counts[l] == 0) return;
  const int t = a.t[l] + 1;
  a.t[l] = t;
  a.bc[2 * l] = (float)(1.0 - pow((double)a.beta1, (double)t));
  a.bc[2 * l + 1] = (float)(1.0 - pow((double)a.beta2, (double)t));
}

// streaming accesses of the optimiser state: every element is touched once per step
__device__ inline float4 ld_stream(const float* p) {
  typedef float f4 __attribute__((ext_vector_type(4)));
  const f4 v = __builtin_nontemporal_load(reinterpret_cast<const f4*>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ inline void st_stream(float* p, const float4& v) {
  typedef float f4 __attribute__((ext_vector_type(4)));
  f4 t; t.x = v.x; t.y = v.y; t.z = v.z; t.w = v.w;
  __builtin_nontemporal_store(t, reinterpret_cast<f4*>(p));
}
__device__ inline void adam_update4(const AdamArgs& a, float bc1, float bc2, const float4& g, float4& th, float4& m, float4& v,
                                    float (&tt)[4]) {
  const float gg[4] = {g.x, g.y, g.z, g.w};
  float mm[4] = {m.x, m.y, m.z, m.w}, vv[4] = {v.x, v.y, v.z, v.w};
  tt[0] = th.x; tt[1] = th.y; tt[2] = th.z; tt[3] = th.w;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    mm[e] = a.beta1 * mm[e] + (1.f - a.beta1) * gg[e];
    vv[e] = a.beta2 * vv[e] + (1.f - a.beta2) * gg[e] * gg[e];
    const float mh = mm[e] / bc1, vh = vv[e] / bc2;
    tt[e] -= a.lr * mh / (sqrtf(vh) + a.eps);
  }
  th = make_float4(tt[0], tt[1], tt[2], tt[3]);
  m = make_float4(mm[0], mm[1], mm[2], mm[3]);
  v = make_float4(vv[0], vv[1], vv[2], vv[3]);
}

// the ranges between the tiled regions
__global__ __launch_bounds__(256) void adam_kernel(AdamArgs a) {
  const int l = blockIdx.y;
  if (a.counts[l] == 0) return;
  int r = 0;
  while (r + 1 < a.ngaps && (int)blockIdx.x >= a.gap_blk0[r + 1]) ++r;
  const long long i = a.gap_lo[r] + ((long long)(blockIdx.x - a.gap_blk0[r]) * 256 + threadIdx.x) * 4;
  if (i >= a.gap_hi[r]) return;
  const long long o = (long long)l * a.P + i;
  const float4 g = ld_stream(a.g + o);
  float4 th = ld_stream(a.theta + o);
  float4 m = ld_stream(a.m + o);
  float4 v = ld_stream(a.v + o);
  float tt[4];
  adam_update4(a, a.bc[2 * l], a.bc[2 * l + 1], g, th, m, v, tt);
  st_stream(a.theta + o, th);
  st_stream(a.m + o, m);
  st_stream(a.v + o, v);
  if (a.shadow) store4(static_cast<bf16_t*>(a.shadow) + o, tt);
}

// One 64 (cb) x 64 (cs) tile of one tap of a convolution weight: the update, the storage-type copy, and - through
// LDS - the transposed storage-type copy, so that the new weights are read from HBM once.
template <typename T>
__global__ __launch_bounds__(256) void adam_tile_kernel(AdamArgs a) {
  constexpr int EPV = 16 / (int)sizeof(T);
  constexpr int TSTRIDE = 64 * (int)sizeof(T) + 16;            // bytes per transposed row (64 cb)
  __shared__ __attribute__((aligned(16))) unsigned char tile[64 * TSTRIDE];
  // a block takes the (tile, model) pairs blockIdx.x, blockIdx.x + gridDim.x, ... of this launch (the launcher's
  // grid covers them all)
  const long long items = (long long)a.tile_count * a.L;
  for (long long item = blockIdx.x; item < items; item += gridDim.x) {
    const int l = (int)(item / a.tile_count);
    if (a.counts[l] == 0) continue;
    const int bx = (int)(item - (long long)l * a.tile_count) + a.tile_first;
    int r = 0;
    while (r + 1 < a.nregions && bx >= a.reg_tile0[r + 1]) ++r;
    const int Cb = a.reg_cb[r], Cs = a.reg_cs[r];
    const int tcs_n = Cs >> 6, tcb_n = Cb >> 6;
    int q = bx - a.reg_tile0[r];
    const int tcs = q % tcs_n; q /= tcs_n;
    const int tcb = q % tcb_n;
    const int tap = q / tcb_n;
    const long long base = (long long)l * a.P + a.reg_w[r];
    const float bc1 = a.bc[2 * l], bc2 = a.bc[2 * l + 1];
    const int c4 = (threadIdx.x & 15) * 4, r0 = threadIdx.x >> 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = r0 + 16 * i;                                // cb inside the tile
      const long long o = base + ((long long)tap * Cb + tcb * 64 + row) * Cs + tcs * 64 + c4;
      const float4 g = ld_stream(a.g + o);
      float4 th = ld_stream(a.theta + o);
      float4 m = ld_stream(a.m + o);
      float4 v = ld_stream(a.v + o);
      float tt[4];
      adam_update4(a, bc1, bc2, g, th, m, v, tt);
      st_stream(a.theta + o, th);
      st_stream(a.m + o, m);
      st_stream(a.v + o, v);
      if (a.shadow) store4(static_cast<bf16_t*>(a.shadow) + o, tt);
#pragma unroll
      for (int e = 0; e < 4; ++e) *reinterpret_cast<T*>(tile + (c4 + e) * TSTRIDE + row * (int)sizeof(T)) = from_float<T>(tt[e]);
    }
    __syncthreads();
    T* dst = static_cast<T*>(a.shadow_t) + base;
    constexpr int CPR = 64 / EPV;                                 // 16-byte chunks per transposed row
#pragma unroll
    for (int i = 0; i < 64 * CPR / 256; ++i) {
      const int cid = threadIdx.x + 256 * i;
      const int cs = cid / CPR, ch = cid - cs * CPR;
      const uint4 val = *reinterpret_cast<const uint4*>(tile + cs * TSTRIDE + ch * 16);
      *reinterpret_cast<uint4*>(dst + ((long long)tap * Cs + tcs * 64 + cs) * Cb + tcb * 64 + ch * EPV) = val;
    }
    __syncthreads();                                              // the tile is rewritten by the next pair
  }
}

// Fills the launch geometry: the tiled regions (sorted by offset: the caller's job) and the gaps between them, which
// cover the rest of [0, P).  False (and a launch error) when the regions do not fit the kernels.
bool adam_plan(AdamArgs& a) {
  if (a.nregions < 0 || a.nregions > ADAM_MAX_REGIONS || a.P % 8) {
    launch_fail("Adam: too many weight regions, or a parameter block that is not a multiple of 8");
    return false;
  }
  long long pos = 0;
  a.ngaps = 0;
  a.reg_tile0[0] = 0;
  a.gap_blk0[0] = 0;
  a.tile_first = 0;
  for (int r = 0; r <= a.nregions; ++r) {
    const long long lo = r < a.nregions ? a.reg_w[r] : a.P;
    if (lo < pos || lo % 4) { launch_fail("Adam: weight regions must be sorted and 16-byte aligned"); return false; }
    if (lo > pos) {
      a.gap_lo[a.ngaps] = pos; a.gap_hi[a.ngaps] = lo;
      a.gap_blk0[a.ngaps + 1] = a.gap_blk0[a.ngaps] + (int)((lo - pos + 1023) / 1024);
      ++a.ngaps;
    }
    if (r < a.nregions) {
      if (a.reg_cb[r] % 64 || a.reg_cs[r] % 64 || !a.shadow_t) {
        launch_fail("Adam: tiled regions need channel counts that are multiples of 64");
        return false;
      }
      a.reg_tile0[r + 1] = a.reg_tile0[r] + 16 * (a.reg_cb[r] / 64) * (a.reg_cs[r] / 64);
      pos = lo + 16LL * a.reg_cb[r] * a.reg_cs[r];
    }
  }
  return true;
}
// The three parts of one update of a planned AdamArgs, in any order after the first: the step counts and bias
// corrections; the gaps; one tiled region (or all of them, region < 0).  Each element is updated by exactly one part.
void launch_adam_prepare(const AdamArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(adam_prepare_kernel, dim3((a.L + 255) / 256), dim3(256), 0, st, a);
}
void launch_adam_gaps(const AdamArgs& a, hipStream_t st) {
  if (a.ngaps > 0) hipLaunchKernelGGL(adam_kernel, dim3((unsigned)a.gap_blk0[a.ngaps], a.L), dim3(256), 0, st, a);
}
template <typename T>
void launch_adam_region(AdamArgs a, int region, hipStream_t st) {
  if (a.nregions == 0 || region >= a.nregions) return;
  const int first = region < 0 ? 0 : a.reg_tile0[region];
  const int last = region < 0 ? a.reg_tile0[a.nregions] : a.reg_tile0[region + 1];
  a.tile_first = first;
  a.tile_count = last - first;
  const long long blocks = (long long)a.tile_count * a.L;
  if (blocks > 0x7fffffffLL) return launch_fail("Adam: more than 2^31 weight tiles in one launch");
  if (blocks > 0) hipLaunchKernelGGL((adam_tile_kernel<T>), dim3((unsigned)blocks), dim3(256), 0, st, a);
}
template void launch_adam_region<float>(AdamArgs, int, hipStream_t);
template void launch_adam_region<bf16_t>(AdamArgs, int, hipStream_t);

template <typename T>
void launch_adam(AdamArgs a, hipStream_t st) {
  if (!adam_plan(a)) return;
  launch_adam_prepare(a, st);
  launch_adam_gaps(a, st);
  launch_adam_region<T>(a, -1, st);
}
template void launch_adam<float>(AdamArgs, hipStream_t);
template void launch_adam<bf16_t>(AdamArgs, hipStream_t);

template <typename T>
__global__ void cast_shadow_kernel(const float* __restrict__ theta, T* __restrict__ shadow, long long total) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < total) shadow[i] = from_float<T>(theta[i]);
}
template <typename T> void launch_cast_shadow(const float* theta, T* shadow, long long total, hipStream_t st) {
  if (total == 0) return;
  hipLaunchKernelGGL((cast_shadow_kernel<T>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, theta, shadow, total);
}
template void launch_cast_shadow<bf16_t>(const float*, bf16_t*, long long, hipStream_t);
template void launch_cast_shadow<float>(const float*, float*, long long, hipStream_t);

// dst[tap][cs][cb] <- src[tap][cb][cs]; block = 32 x 32 tile, grid (tiles, 16 taps, L)
template <typename T, typename S>
__global__ void transpose_w_kernel(const S* __restrict__ src, T* __restrict__ dst, long long pstride, int Cb, int Cs) {
  __shared__ float tile[32][33];
  const int tb = Cb / 32;
  const int tcs = blockIdx.x / tb, tcb = blockIdx.x - tcs * tb;
  const long long base = (long long)blockIdx.z * pstride + (long long)blockIdx.y * Cb * Cs;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 256 threads: 8 rows per pass
  for (int r = ty; r < 32; r += 8) {
    const int cb = tcb * 32 + r, cs = tcs * 32 + tx;
    tile[r][tx] = (cs < Cs) ? to_float(src[base + (long long)cb * Cs + cs]) : 0.f;
  }
  __syncthreads();
  for (int r = ty; r < 32; r += 8) {
    const int cs = tcs * 32 + r, cb = tcb * 32 + tx;
    if (cs < Cs) dst[base + (long long)cs * Cb + cb] = from_float<T>(tile[tx][r]);
  }
}
template <typename T, typename S>
void launch_transpose_w(const S* src, T* dst, long long pstride, int L, int Cb, int Cs, hipStream_t st) {
  dim3 grid((Cb / 32) * ((Cs + 31) / 32), 16, L);
  hipLaunchKernelGGL((transpose_w_kernel<T, S>), grid, dim3(256), 0, st, src, dst, pstride, Cb, Cs);
}
template void launch_transpose_w<float, float>(const float*, float*, long long, int, int, int, hipStream_t);
template void launch_transpose_w<bf16_t, bf16_t>(const bf16_t*, bf16_t*, long long, int, int, int, hipStream_t);

// ---------------------------------------------------------------------------------------------------------
// Mixture sampling (Eq. 5): class draws from the prior.  The cumulative probabilities come from the host in
// double; the comparison is done in double so that the integer result does not depend on who computes it.
// ---------------------------------------------------------------------------------------------------------
__global__ void draw_labels_kernel(const float* __restrict__ u, const double* __restrict__ cdf, int K, int last, int n,
                                   int* __restrict__ labels) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const double ui = (double)u[i];
  int lo = 0, hi = K;                 // first k in [0, K) with cdf[k] > ui (cdf is non-decreasing), K if none
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (cdf[mid] > ui) hi = mid; else lo = mid + 1;
  }
  labels[i] = lo < K ? lo : last;
}
void launch_draw_labels(const float* u, const double* cdf, int n_labels, int last, int n, int* labels, hipStream_t st) {
  if (n == 0) return;
  hipLaunchKernelGGL(draw_labels_kernel, dim3((n + 255) / 256), dim3(256), 0, st, u, cdf, n_labels, last, n, labels);
}

// ---------------------------------------------------------------------------------------------------------
// One-way ANOVA of the image intensities by class (Section 4).  Three small kernels, double arithmetic, every sum in
// a fixed order: thread-strided partial sums, then a tree over the 256 threads.
// ---------------------------------------------------------------------------------------------------------
__device__ inline double block_sum_256(double v, double* sh) {
  sh[threadIdx.x] = v;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) sh[threadIdx.x] += sh[threadIdx.x + s];
    __syncthreads();
  }
  const double r = sh[0];
  __syncthreads();
  return r;
}
__global__ __launch_bounds__(256) void anova_image_mean_kernel(const float* __restrict__ images, int C, int HW, double* __restrict__ x) {
  __shared__ double sh[256];
  const long long ic = blockIdx.x;                                     // image * C + channel
  const float* p = images + ic * HW;
  double s = 0.0;
  for (int q = threadIdx.x; q < HW; q += 256) s += (double)p[q];
  s = block_sum_256(s, sh);
  if (threadIdx.x == 0) x[ic] = s / (double)HW;
}
__global__ __launch_bounds__(256) void anova_group_kernel(const int* __restrict__ label_ids, const double* __restrict__ x, int n, int C,
                                                          const double* __restrict__ gsum_in, const int* __restrict__ gcnt_in,
                                                          double* __restrict__ out, int* __restrict__ gcnt_out) {
  __shared__ double sh[256];
  const int k = blockIdx.x, c = blockIdx.y;
  // pass 1 (gsum_in == NULL): sum of x and count ; pass 2: sum of squared deviations from the group mean
  double mean = 0.0;
  if (gsum_in) {
    const int cnt = gcnt_in[k];
    mean = cnt > 0 ? gsum_in[(long long)k * C + c] / (double)cnt : 0.0;
  }
  double s = 0.0, cntd = 0.0;
  for (int i = threadIdx.x; i < n; i += 256) {
    if (label_ids[i] != k) continue;
    const double v = x[(long long)i * C + c];
    if (gsum_in) { s += (v - mean) * (v - mean); } else { s += v; cntd += 1.0; }
  }
  s = block_sum_256(s, sh);
  if (!gsum_in) cntd = block_sum_256(cntd, sh);
  if (threadIdx.x == 0) {
    out[(long long)k * C + c] = s;
    if (!gsum_in && c == 0) gcnt_out[k] = (int)cntd;
  }
}
void launch_anova(const int* label_ids, const float* images, int n, int n_labels, int C, int HW, double* x, double* gsum,
                  int* gcnt, double* ssw, hipStream_t st) {
  if (n == 0) return;
  hipLaunchKernelGGL(anova_image_mean_kernel, dim3((unsigned)((long long)n * C)), dim3(256), 0, st, images, C, HW, x);
  hipLaunchKernelGGL(anova_group_kernel, dim3(n_labels, C), dim3(256), 0, st, label_ids, x, n, C, (const double*)nullptr,
                     (const int*)nullptr, gsum, gcnt);
  hipLaunchKernelGGL(anova_group_kernel, dim3(n_labels, C), dim3(256), 0, st, label_ids, x, n, C, (const double*)gsum,
                     (const int*)gcnt, ssw, (int*)nullptr);
}

}  // namespace gan
