// Host side of the library: context, arenas, parameter layout, and the launch sequence of one training step
// (Section 2 of the paper: cost of Eq. 3 and Adam on theta_D, then cost of Eq. 4 through the updated D and Adam on
// theta_G, for all label models of Eq. 5 at once).
#include "../../include/gan.h"

#include <math.h>
#include <stdio.h>
#include <string.h>
#include <algorithm>

#include <set>
#include <string>
#include <vector>

#include "anova_host.h"
#include "kernels.h"

using namespace gan;

namespace gan {
static thread_local const char* g_launch_error = nullptr;
void launch_fail(const char* msg) { if (!g_launch_error) g_launch_error = msg; }
const char* take_launch_error() { const char* e = g_launch_error; g_launch_error = nullptr; return e; }
}  // namespace gan

namespace {

inline long long round_up(long long x, long long m) { return (x + m - 1) / m * m; }

// the weight gradient of a patch-matrix layer has a tiny output and a long reduction: its rows are split over this
// many blocks per model, and the partial blocks are added in a fixed order when they are unpacked
// Row splits of the image-side weight gradients (one or a few output tiles per model): 8 when there are many
// models, more when the models alone would leave most of the chip idle.  A function of the model count only.
static int img_ksplit_for(int L) { return std::min(std::max(800 / L, 8), 128); }
constexpr int WG_MAX_KSPLIT = 16;

// A (transposed) convolution between a "big" tensor (Cb channels, side 2*Hs) and a "small" one (Cs, side Hs).
// Internal weight layout [tap][Cb (or CBT)][Cs].
struct ConvLayer {
  int Cb = 0, CBT = 0, Cs = 0, Hs = 0;
  long long w = -1, bias = -1, gamma = -1, beta = -1;   // offsets into the per-model parameter block
  long long rs = -1;                                    // offset into the running-statistics block
  int bnC = 0;                                          // channels normalised after this layer (0: none)
  int nbias = 0;
  // networks as printed in the paper's tables: real (unpadded) channel counts, and for G's blocks the place of the
  // summed-tap k4 weights in the storage-type arenas
  int cs_real = 0, cb_real = 0;
  long long w4 = -1;
};

struct Net {
  std::vector<ConvLayer> conv;     // G: transposed convs 1..n_g ; D: convs 1..n_d
  // linear layer: G's input stage (J outputs, Kp padded inputs, followed by BN over C0) / D's head (K inputs)
  long long fc_w = -1, fc_b = -1, fc_gamma = -1, fc_beta = -1, fc_rs = -1;
  int J = 0, Kz = 0, Kp = 0, C0 = 0, h0 = 0, K = 0;
  long long P = 0;                 // internal parameters per model (multiple of 64: keeps 16-byte alignment)
  long long Pext = 0;              // parameters per model in the documented order
  long long nbn = 0;
  std::vector<long long> ext2int;  // documented index -> internal index
  std::vector<long long> bn_ext2int;   // documented running-statistics index -> internal (empty: identical)
  std::vector<int> ext_kind;       // per documented element: 0 weight, 1 gamma, 2 zero-initialised (built-in initialiser)
  // networks as printed in the paper's tables (G): k4 weights with summed taps, [tap][cb][cs] and [tap][cs][cb]
  long long fc_bias = -1, P4 = 0;
  void *w4u = nullptr, *w4d = nullptr;
  float *theta = nullptr, *m = nullptr, *v = nullptr, *g = nullptr;
  void *shadow_u = nullptr, *shadow_d = nullptr;   // storage-type copies: [tap][cb][cs] and [tap][cs][cb]
  float *run_mean = nullptr, *run_var = nullptr;
  int* t = nullptr;
  float* bc = nullptr;
};

struct ProfEntry { const char* name; hipEvent_t e0, e1; double flops, bytes; };

}  // namespace

struct gan_ctx {
  gan_config cfg;
  hipStream_t st = nullptr;
  bool bf16 = false;
  int L = 0, NB = 0;
  Net G, D;
  GeomTable geoms;
  RouteBuffers rb;                 // the set the launch helpers use (the training step's, except inside gan_generate)
  RouteBuffers rb_gen;             // gan_generate / gan_sample route into this one
  // workspace (storage type unless noted)
  void *zin = nullptr, *xd = nullptr, *dimg = nullptr, *bufA = nullptr, *bufB = nullptr;
  std::vector<void*> gpre, gact, dpre, dact;
  std::vector<float*> g_mean, g_var, g_rstd, g_sums, d_mean, d_var, d_rstd, d_sums;
  float *logits = nullptr, *dlogits = nullptr, *loss_d = nullptr, *loss_g = nullptr;
  // image-side layers: patch matrices, packed weights, packed weight gradients
  void *colD = nullptr, *colG = nullptr, *wpD = nullptr, *wpG = nullptr;
  float *dwp = nullptr, *bias_partial = nullptr, *stat_partial = nullptr;
  int img_ksplit = 8;
  float* head_part = nullptr;      // row-split partial sums of the linear head's weight gradient (few models only)
  int head_rsplit = 1;
  float* wg_part = nullptr;        // row-split partial weight gradients (few models only)
  bool paper = false;              // the networks as printed in the paper's tables
  float *dw4 = nullptr, *c3_part = nullptr;   // paper G: k4 weight gradient of one block; row-split partials of the last conv
  int KcD = 0, KcG = 0;
  int nslot = 1;
  int last_n = -1;
  bool shadows_dirty = true;
  std::string err;
  std::vector<void*> allocs;
  // mixture sampling and ANOVA: buffers allocated at first use
  double* cdf = nullptr;            // [n_labels]
  double *an_x = nullptr, *an_gsum = nullptr, *an_ssw = nullptr;   // [NB*img_c], [n_labels*img_c] x 2
  int* an_gcnt = nullptr;           // [n_labels]
  // profiling
  bool prof = false, prof_detail = false, prof_gemm_only = false;
  std::set<std::string> prof_names;
  std::vector<ProfEntry> prof_entries;
  std::vector<hipEvent_t> event_pool;
  // A second stream (default priority) for the weight gradients and the Adam updates of the convolution weights, which
  // nothing later in the backward chain waits for: they can run beside it and fill the chip where the chain's kernels
  // leave it idle (tile-count tails, bandwidth-bound passes).  Ordering between the two streams is by events.  Off
  // unless the caller asks (gan_use_second_stream): it shortens the largest workload's step by 1.7 %, and every
  // kernel that shares the chip with another one runs longer, which blurs per-kernel timings.
  hipStream_t side = nullptr;
  bool side_on = false;
  std::vector<hipEvent_t> order_events;
  size_t order_next = 0;
  // Replayable steps.  A training step's launches depend on the call's arguments only through the three device
  // pointers and n (everything else the kernels read lives in device tables the step itself rebuilds), so a call that
  // repeats the arguments of a recent call can be captured once into a HIP graph (on `cap`, an internal stream: the
  // caller's may be the legacy default stream, which cannot be captured) and replayed on the caller's stream from
  // then on: one host call instead of a hundred and more.  Off unless the caller asks (gan_use_graphs): on this
  // part the steps are bound by the chain of dependent kernels on the device, not by the host's launch calls, and a
  // replay measured 0-4 % slower than the plain launches in every configuration.
  struct StepGraph { const void *lab, *noise, *real; int n; hipGraphExec_t exec; unsigned long long used; };
  hipStream_t cap = nullptr;
  std::vector<StepGraph> graphs;
  bool graphs_on = false;
  struct StepArgs { const void *lab, *noise, *real; int n; };
  std::vector<StepArgs> seen;      // the last eight distinct argument sets that ran as plain launches
  unsigned long long calls = 0, replays = 0;
  int op_tile_rows = 0;            // single-operation entry points: tile height forced by the caller (0: chosen as in a step)
};

namespace {

size_t esize(const gan_ctx* c) { return c->bf16 ? 2 : 4; }

gan_status fail(gan_ctx* c, gan_status s, const std::string& msg) {
  if (c) c->err = msg;
  return s;
}

// After a call has enqueued its launches: a refused launch (shape the kernels do not support) or a HIP launch error.
gan_status launch_status(gan_ctx* c) {
  const char* refused = take_launch_error();
  const hipError_t e = hipGetLastError();
  if (refused) return fail(c, GAN_E_SHAPE, refused);
  if (e != hipSuccess) return fail(c, GAN_E_HIP, std::string("launch failed: ") + hipGetErrorString(e));
  return GAN_OK;
}

bool dev_alloc(gan_ctx* c, void** p, size_t bytes) {
  if (bytes == 0) bytes = 16;
  if (hipMalloc(p, bytes) != hipSuccess) { (void)hipGetLastError(); return false; }
  c->allocs.push_back(*p);
  return true;
}

int geom_id(gan_ctx* c, int rps, int tile_rows) {
  for (int i = 0; i < c->geoms.n; ++i)
    if (c->geoms.rps[i] == rps && c->geoms.tile_rows[i] == tile_rows) return i;
  if (c->geoms.n >= MAX_GEOMS) return -1;
  c->geoms.rps[c->geoms.n] = rps;
  c->geoms.tile_rows[c->geoms.n] = tile_rows;
  return c->geoms.n++;
}
const int* tmodel_of(gan_ctx* c, int rps, int tile_rows) {
  for (int i = 0; i < c->geoms.n; ++i)
    if (c->geoms.rps[i] == rps && c->geoms.tile_rows[i] == tile_rows) return c->rb.tmodel + (long long)i * c->rb.tmodel_stride;
  return nullptr;
}
const int* tpre_of(gan_ctx* c, int rps, int tile_rows) {
  int g = -1;
  for (int i = 0; i < c->geoms.n; ++i)
    if (c->geoms.rps[i] == rps && c->geoms.tile_rows[i] == tile_rows) g = i;
  if (g < 0) {   // every geometry a launch uses is registered at create; anything else would read an unbuilt prefix
    launch_fail("a launch asked for a tile geometry that was not registered when the context was created");
    return nullptr;   // the launchers refuse a null prefix array
  }
  return c->rb.tpre + (long long)g * (c->L + 1);
}
// tile height for a layer: from the average rows per model at the sizing batch (fixed at create, so the prefix
// arrays built at every routing match)
int layer_tile_rows(const gan_ctx* c, int n_out, int rps) {
  return conv_tile_rows(n_out, (long long)c->NB * rps / c->L, c->L);
}
int ub_tiles(const gan_ctx* c, int n, int rps, int tile_rows) {
  return (int)(((long long)n * rps) / tile_rows) + (n < c->L ? n : c->L);
}

// ---- profiling: two events around a launch ------------------------------------------------------------
struct Scope {
  gan_ctx* c; int idx = -1; hipStream_t st;
  // st: the stream the launch goes to (default: the caller's)
  Scope(gan_ctx* c_, const char* name, double flops, double bytes, const char* detail = nullptr, hipStream_t st_ = nullptr)
      : c(c_), st(st_ ? st_ : c_->st) {
    if (!c->prof) return;
    if (c->prof_gemm_only && strncmp(name, "gemm_", 5) != 0 && strncmp(name, "wgrad", 5) != 0) return;
    if (c->prof_detail && detail) name = c->prof_names.insert(std::string(name) + detail).first->c_str();
    ProfEntry e; e.name = name; e.flops = flops; e.bytes = bytes;
    for (hipEvent_t* ev : {&e.e0, &e.e1}) {          // events are reused across profiling sessions
      if (c->event_pool.empty()) hipEventCreateWithFlags(ev, hipEventDisableSystemFence);   // device-side timing only: no system-scope fence
      else { *ev = c->event_pool.back(); c->event_pool.pop_back(); }
    }
    hipEventRecord(e.e0, st);
    c->prof_entries.push_back(e);
    idx = (int)c->prof_entries.size() - 1;
  }
  ~Scope() { if (idx >= 0) hipEventRecord(c->prof_entries[idx].e1, st); }
};

// The stream for work that may run beside the caller's stream (per-launch timing records its events on whichever
// stream a launch goes to, so the timed steps run exactly like the untimed ones).
hipStream_t side_stream(gan_ctx* c) { return (c->side && c->side_on) ? c->side : c->st; }
// whatever is enqueued on `later` from now on starts after everything enqueued on `earlier` so far
void order_after(gan_ctx* c, hipStream_t later, hipStream_t earlier) {
  if (later == earlier) return;
  if (c->order_next == c->order_events.size()) {
    hipEvent_t e;
    if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) return launch_fail("could not create an ordering event");
    c->order_events.push_back(e);
  }
  hipEvent_t e = c->order_events[c->order_next++];
  hipEventRecord(e, earlier);
  hipStreamWaitEvent(later, e, 0);
}

template <typename T> void adam_region_call(gan_ctx* c, const AdamArgs& a, int region, hipStream_t st);

double valid_tap_fraction(int Hs) {   // k4 s2 p1: per axis 2 of the 4*Hs (row, tap) pairs fall outside
  const double f = (4.0 * Hs - 2.0) / (4.0 * Hs);
  return f * f;
}

// ---- parameter layout ----------------------------------------------------------------------------------
void build_layout(gan_ctx* c) {
  const gan_config& f = c->cfg;
  {
    Net& G = c->G;
    long long o = 0, ext = 0, r = 0;
    G.Kz = f.z_dim + f.cond_g;
    G.Kp = (int)round_up(G.Kz, 64);
    G.C0 = f.g_ch[0]; G.h0 = f.g_h0; G.J = G.C0 * G.h0 * G.h0;
    G.fc_w = o; o += (long long)G.J * G.Kp;
    G.fc_gamma = o; o += G.C0; G.fc_beta = o; o += G.C0; G.fc_rs = r; r += G.C0;
    o = round_up(o, 8);
    // documented order: fc.w [(c,h,w)][Kz]
    G.ext2int.reserve(1 << 20);
    for (int ch = 0; ch < G.C0; ++ch)
      for (int y = 0; y < G.h0; ++y)
        for (int x = 0; x < G.h0; ++x)
          for (int i = 0; i < G.Kz; ++i)
            G.ext2int.push_back(G.fc_w + ((long long)((y * G.h0 + x) * G.C0 + ch)) * G.Kp + i);
    for (int ch = 0; ch < G.C0; ++ch) G.ext2int.push_back(G.fc_gamma + ch);
    for (int ch = 0; ch < G.C0; ++ch) G.ext2int.push_back(G.fc_beta + ch);
    int h = f.g_h0;
    for (int i = 1; i <= f.n_g; ++i) {
      ConvLayer l;
      l.Cs = f.g_ch[i - 1]; l.Cb = (i < f.n_g) ? f.g_ch[i] : f.img_c; l.CBT = l.Cb; l.Hs = h;
      l.w = o; o += (long long)16 * l.CBT * l.Cs;
      for (int cs = 0; cs < l.Cs; ++cs)
        for (int cb = 0; cb < l.Cb; ++cb)
          for (int tap = 0; tap < 16; ++tap) G.ext2int.push_back(l.w + ((long long)tap * l.CBT + cb) * l.Cs + cs);
      if (i < f.n_g) {
        l.gamma = o; o += l.Cb; l.beta = o; o += l.Cb; l.rs = r; r += l.Cb; l.bnC = l.Cb;
        for (int ch = 0; ch < l.Cb; ++ch) G.ext2int.push_back(l.gamma + ch);
        for (int ch = 0; ch < l.Cb; ++ch) G.ext2int.push_back(l.beta + ch);
      } else {
        l.bias = o; l.nbias = l.Cb; o += l.Cb;
        for (int ch = 0; ch < l.Cb; ++ch) G.ext2int.push_back(l.bias + ch);
      }
      o = round_up(o, 8);
      G.conv.push_back(l);
      h *= 2;
    }
    G.P = round_up(o, 64); G.Pext = (long long)G.ext2int.size(); G.nbn = r; (void)ext;
  }
  {
    Net& D = c->D;
    long long o = 0, r = 0;
    int h = f.img_hw;
    for (int j = 0; j < f.n_d; ++j) {
      ConvLayer l;
      l.Cb = (j == 0) ? f.img_c : f.d_ch[j - 1];
      l.CBT = (j == 0) ? f.img_c + f.cond_d : l.Cb;
      l.Cs = f.d_ch[j]; l.Hs = h / 2;
      l.w = o; o += (long long)16 * l.CBT * l.Cs;
      for (int cs = 0; cs < l.Cs; ++cs)
        for (int cb = 0; cb < l.CBT; ++cb)
          for (int tap = 0; tap < 16; ++tap) D.ext2int.push_back(l.w + ((long long)tap * l.CBT + cb) * l.Cs + cs);
      if (j == 0) {
        l.bias = o; l.nbias = l.Cs; o += l.Cs;
        for (int ch = 0; ch < l.Cs; ++ch) D.ext2int.push_back(l.bias + ch);
      } else {
        l.gamma = o; o += l.Cs; l.beta = o; o += l.Cs; l.rs = r; r += l.Cs; l.bnC = l.Cs;
        for (int ch = 0; ch < l.Cs; ++ch) D.ext2int.push_back(l.gamma + ch);
        for (int ch = 0; ch < l.Cs; ++ch) D.ext2int.push_back(l.beta + ch);
      }
      o = round_up(o, 8);
      D.conv.push_back(l);
      h /= 2;
    }
    const int Cl = f.d_ch[f.n_d - 1];
    D.K = Cl * h * h; D.h0 = h; D.C0 = Cl;
    D.fc_w = o; o += D.K;
    for (int ch = 0; ch < Cl; ++ch)
      for (int y = 0; y < h; ++y)
        for (int x = 0; x < h; ++x) D.ext2int.push_back(D.fc_w + (long long)(y * h + x) * Cl + ch);
    D.fc_b = o; o += 1;
    D.ext2int.push_back(D.fc_b);
    D.P = round_up(o, 64); D.Pext = (long long)D.ext2int.size(); D.nbn = r;
  }
}

// The networks as printed in the paper's Tables 1 and 2.  D's k3 s2 p1 convolutions sit in the engine's k4 layout
// (fourth tap row / column and channel padding are not parameters and stay zero); G's Upsample + k3 blocks keep their
// 3 x 3 weights as parameters and run on k4 weights with summed taps rebuilt after every update.
void build_layout_paper(gan_ctx* c) {
  const gan_config& f = c->cfg;
  auto pad64 = [](int v) { return (int)round_up(v, 64); };
  {
    Net& G = c->G;
    long long o = 0, r = 0, o4 = 0;
    G.Kz = f.z_dim; G.Kp = (int)round_up(G.Kz, 64);
    G.C0 = f.g_ch[0]; G.h0 = f.g_h0; G.J = G.C0 * G.h0 * G.h0;
    G.fc_w = o; o += (long long)G.J * G.Kp;
    G.fc_bias = o; o += G.J;
    G.fc_gamma = o; o += G.C0; G.fc_beta = o; o += G.C0; G.fc_rs = r; r += G.C0;
    o = round_up(o, 8);
    auto ext = [&](long long internal, int kind) { G.ext2int.push_back(internal); G.ext_kind.push_back(kind); };
    for (int ch = 0; ch < G.C0; ++ch)
      for (int y = 0; y < G.h0; ++y)
        for (int x = 0; x < G.h0; ++x)
          for (int i = 0; i < G.Kz; ++i) ext(G.fc_w + ((long long)((y * G.h0 + x) * G.C0 + ch)) * G.Kp + i, 0);
    for (int ch = 0; ch < G.C0; ++ch)
      for (int y = 0; y < G.h0; ++y)
        for (int x = 0; x < G.h0; ++x) ext(G.fc_bias + (long long)(y * G.h0 + x) * G.C0 + ch, 2);
    for (int ch = 0; ch < G.C0; ++ch) ext(G.fc_gamma + ch, 1);
    for (int ch = 0; ch < G.C0; ++ch) ext(G.fc_beta + ch, 2);
    int h = f.g_h0;
    for (int i = 1; i < f.n_g; ++i) {                       // Upsample x2 + Conv k3: 3 x 3 master weights [9][cb][cs]
      ConvLayer l;
      l.Cs = f.g_ch[i - 1]; l.Cb = f.g_ch[i]; l.CBT = l.Cb; l.Hs = h; l.cs_real = l.Cs; l.cb_real = l.Cb;
      l.w = o; o += (long long)9 * l.Cb * l.Cs;
      l.w4 = o4; o4 += (long long)16 * l.Cb * l.Cs;
      for (int co = 0; co < l.Cb; ++co)
        for (int ci = 0; ci < l.Cs; ++ci)
          for (int tap = 0; tap < 9; ++tap) ext(l.w + ((long long)tap * l.Cb + co) * l.Cs + ci, 0);
      l.gamma = o; o += l.Cb; l.beta = o; o += l.Cb; l.rs = r; r += l.Cb; l.bnC = l.Cb;
      for (int ch = 0; ch < l.Cb; ++ch) ext(l.gamma + ch, 1);
      for (int ch = 0; ch < l.Cb; ++ch) ext(l.beta + ch, 2);
      o = round_up(o, 8);
      G.conv.push_back(l);
      h *= 2;
    }
    {                                                       // last: Conv k3 s1 p1 onto the image, [9][img_c][cs]
      ConvLayer l;
      l.Cs = f.g_ch[f.n_g - 1]; l.Cb = f.img_c; l.CBT = l.Cb; l.Hs = h; l.cs_real = l.Cs; l.cb_real = l.Cb;
      l.w = o; o += (long long)9 * l.Cb * l.Cs;
      for (int co = 0; co < l.Cb; ++co)
        for (int ci = 0; ci < l.Cs; ++ci)
          for (int tap = 0; tap < 9; ++tap) ext(l.w + ((long long)tap * l.Cb + co) * l.Cs + ci, 0);
      l.bias = o; l.nbias = l.Cb; o += l.Cb;
      for (int ch = 0; ch < l.Cb; ++ch) ext(l.bias + ch, 2);
      o = round_up(o, 8);
      G.conv.push_back(l);
    }
    G.P = round_up(o, 64); G.Pext = (long long)G.ext2int.size(); G.nbn = r; G.P4 = round_up(o4, 64);
  }
  {
    Net& D = c->D;
    long long o = 0, r = 0;
    auto ext = [&](long long internal, int kind) { D.ext2int.push_back(internal); D.ext_kind.push_back(kind); };
    int h = f.img_hw;
    for (int j = 0; j < f.n_d; ++j) {
      ConvLayer l;
      l.cb_real = (j == 0) ? f.img_c : f.d_ch[j - 1];
      l.cs_real = f.d_ch[j];
      l.Cb = (j == 0) ? f.img_c : pad64(l.cb_real); l.CBT = l.Cb; l.Cs = pad64(l.cs_real); l.Hs = h / 2;
      l.w = o; o += (long long)16 * l.CBT * l.Cs;
      for (int co = 0; co < l.cs_real; ++co)
        for (int ci = 0; ci < l.cb_real; ++ci)
          for (int ky = 0; ky < 3; ++ky)
            for (int kx = 0; kx < 3; ++kx) ext(l.w + ((long long)(ky * 4 + kx) * l.CBT + ci) * l.Cs + co, 0);
      l.bias = o; l.nbias = l.Cs; o += l.Cs;
      for (int ch = 0; ch < l.cs_real; ++ch) ext(l.bias + ch, 2);
      if (j > 0) {
        l.gamma = o; o += l.Cs; l.beta = o; o += l.Cs; l.rs = r; l.bnC = l.Cs;
        for (int ch = 0; ch < l.cs_real; ++ch) ext(l.gamma + ch, 1);
        for (int ch = 0; ch < l.cs_real; ++ch) ext(l.beta + ch, 2);
        for (int ch = 0; ch < l.cs_real; ++ch) D.bn_ext2int.push_back(r + ch);
        r += l.Cs;
      }
      o = round_up(o, 8);
      D.conv.push_back(l);
      h /= 2;
    }
    const ConvLayer& last = D.conv.back();
    D.K = last.Cs * h * h; D.h0 = h; D.C0 = last.Cs;
    D.fc_w = o; o += D.K;
    for (int ch = 0; ch < last.cs_real; ++ch)
      for (int y = 0; y < h; ++y)
        for (int x = 0; x < h; ++x) ext(D.fc_w + (long long)(y * h + x) * last.Cs + ch, 0);
    D.fc_b = o; o += 1;
    ext(D.fc_b, 2);
    D.P = round_up(o, 64); D.Pext = (long long)D.ext2int.size(); D.nbn = r;
  }
}

bool alloc_net(gan_ctx* c, Net& n) {
  const size_t tot = (size_t)c->L * n.P;
  bool ok = dev_alloc(c, (void**)&n.theta, tot * 4) && dev_alloc(c, (void**)&n.m, tot * 4) &&
            dev_alloc(c, (void**)&n.v, tot * 4) && dev_alloc(c, (void**)&n.g, tot * 4) &&
            dev_alloc(c, &n.shadow_d, tot * esize(c)) &&
            dev_alloc(c, (void**)&n.run_mean, (size_t)c->L * n.nbn * 4) &&
            dev_alloc(c, (void**)&n.run_var, (size_t)c->L * n.nbn * 4) &&
            dev_alloc(c, (void**)&n.t, (size_t)c->L * 4) && dev_alloc(c, (void**)&n.bc, (size_t)c->L * 8);
  if (!ok) return false;
  if (c->bf16) { if (!dev_alloc(c, &n.shadow_u, tot * 2)) return false; }
  else n.shadow_u = n.theta;
  hipMemsetAsync(n.theta, 0, tot * 4, c->st);
  hipMemsetAsync(n.m, 0, tot * 4, c->st);
  hipMemsetAsync(n.v, 0, tot * 4, c->st);
  hipMemsetAsync(n.g, 0, tot * 4, c->st);
  hipMemsetAsync(n.shadow_d, 0, tot * esize(c), c->st);
  hipMemsetAsync(n.run_mean, 0, (size_t)c->L * n.nbn * 4, c->st);
  hipMemsetAsync(n.t, 0, (size_t)c->L * 4, c->st);
  hipMemsetAsync(n.bc, 0, (size_t)c->L * 8, c->st);
  return true;
}

// ---- built-in initialiser (host side, documented order; tests overwrite it through gan_set_params) ------
__global__ void init_normal_kernel(float* p, long long count, float std, unsigned long long seed, int inner, int inner_valid) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= count) return;
  if ((int)(i % inner) >= inner_valid) { p[i] = 0.f; return; }
  unsigned long long z = seed + 0x9E3779B97F4A7C15ull * (unsigned long long)(i + 1);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  z ^= z >> 31;
  const float u1 = ((float)(unsigned)(z >> 40) + 1.0f) * (1.0f / 16777217.0f);
  const float u2 = (float)(unsigned)((z >> 8) & 0xffffffu) * (1.0f / 16777216.0f);
  p[i] = std * sqrtf(-2.0f * logf(u1)) * cosf(6.2831853f * u2);
}
__global__ void fill_kernel(float* p, long long count, float v) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) p[i] = v;
}
void init_normal(gan_ctx* c, float* p, long long count, int inner, int inner_valid, unsigned long long salt) {
  hipLaunchKernelGGL(init_normal_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, c->st, p, count,
                     c->cfg.init_std, c->cfg.seed * 0x100000001B3ull + salt, inner, inner_valid);
}
void fill(gan_ctx* c, float* p, long long count, float v) {
  if (count == 0) return;
  hipLaunchKernelGGL(fill_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, c->st, p, count, v);
}

void builtin_init(gan_ctx* c) {
  unsigned long long salt = 1;
  for (int l = 0; l < c->L; ++l) {
    Net& G = c->G;
    float* th = G.theta + (long long)l * G.P;
    init_normal(c, th + G.fc_w, (long long)G.J * G.Kp, G.Kp, G.Kz, salt++);
    fill(c, th + G.fc_gamma, G.C0, 1.f);
    for (auto& cl : G.conv) {
      init_normal(c, th + cl.w, (long long)16 * cl.CBT * cl.Cs, 1, 1, salt++);
      if (cl.bnC) fill(c, th + cl.gamma, cl.bnC, 1.f);
    }
    Net& D = c->D;
    th = D.theta + (long long)l * D.P;
    for (auto& cl : D.conv) {
      init_normal(c, th + cl.w, (long long)16 * cl.CBT * cl.Cs, 1, 1, salt++);
      if (cl.bnC) fill(c, th + cl.gamma, cl.bnC, 1.f);
    }
    init_normal(c, th + D.fc_w, D.K, 1, 1, salt++);
  }
  fill(c, c->G.run_var, (long long)c->L * c->G.nbn, 1.f);
  fill(c, c->D.run_var, (long long)c->L * c->D.nbn, 1.f);
}

// Built-in initialiser of the networks as printed in the tables: drawn on the host in the documented order and placed
// through the index map, so that padding and the unused fourth taps stay zero.
static float host_normal(unsigned long long& st) {
  auto next = [&]() {
    unsigned long long z = (st += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
  };
  const double u1 = ((double)(next() >> 11) + 1.0) / 9007199254740993.0, u2 = (double)(next() >> 11) / 9007199254740992.0;
  return (float)(sqrt(-2.0 * log(u1)) * cos(6.283185307179586 * u2));
}
bool builtin_init_paper(gan_ctx* c) {
  unsigned long long st = c->cfg.seed * 0x100000001B3ull + 17;
  for (Net* n : {&c->G, &c->D}) {
    std::vector<float> tmp((size_t)n->P);
    for (int l = 0; l < c->L; ++l) {
      std::fill(tmp.begin(), tmp.end(), 0.f);
      for (long long i = 0; i < n->Pext; ++i) {
        const int kind = n->ext_kind[(size_t)i];
        tmp[(size_t)n->ext2int[(size_t)i]] = kind == 0 ? c->cfg.init_std * host_normal(st) : (kind == 1 ? 1.f : 0.f);
      }
      if (hipMemcpy(n->theta + (long long)l * n->P, tmp.data(), (size_t)n->P * 4, hipMemcpyHostToDevice) != hipSuccess) return false;
    }
  }
  fill(c, c->G.run_var, (long long)c->L * c->G.nbn, 1.f);
  fill(c, c->D.run_var, (long long)c->L * c->D.nbn, 1.f);
  return true;
}

// ---- storage-type copies of the weights ------------------------------------------------------------------
PackArgs pack_args(gan_ctx* c, Net& net, const ConvLayer& cl, int Kc, int nslot, void* wp);

template <typename T>
void refresh_transposes(gan_ctx* c, Net& n, bool isG) {
  // the image-side layer multiplies a patch matrix: [cs][Kc] with the label-map sums and the bias folded in
  if (isG) launch_pack_w<T>(pack_args(c, n, n.conv.back(), c->KcG, 0, c->wpG), c->st);
  else launch_pack_w<T>(pack_args(c, n, n.conv.front(), c->KcD, c->nslot, c->wpD), c->st);
  // layers run by the GEMM engine in "down" form need [tap][cs][cb]
  for (size_t i = 0; i < n.conv.size(); ++i) {
    const ConvLayer& cl = n.conv[i];
    const bool gemm = isG ? (i + 1 < n.conv.size()) : (i > 0);
    if (!gemm) continue;
    Scope s(c, "transpose_w", 0, (double)c->L * 16 * cl.Cb * cl.Cs * 2 * sizeof(T));
    if (c->bf16)
      launch_transpose_w<bf16_t, bf16_t>((const bf16_t*)n.shadow_u + cl.w, (bf16_t*)n.shadow_d + cl.w, n.P, c->L, cl.Cb, cl.Cs, c->st);
    else
      launch_transpose_w<float, float>((const float*)n.theta + cl.w, (float*)n.shadow_d + cl.w, n.P, c->L, cl.Cb, cl.Cs, c->st);
  }
}
// k4 weights with summed taps of G's Upsample + Conv k3 blocks, from the 3 x 3 master weights
template <typename T>
void paper_rebuild_w4(gan_ctx* c) {
  Net& G = c->G;
  for (size_t i = 0; i + 1 < G.conv.size(); ++i) {
    const ConvLayer& cl = G.conv[i];
    launch_w3_to_w4<T>(G.theta + cl.w, (T*)G.w4u + cl.w4, (T*)G.w4d + cl.w4, c->L, cl.Cb, cl.Cs, c->st, G.P, G.P4);
  }
}
void refresh_shadows(gan_ctx* c) {
  for (Net* n : {&c->G, &c->D}) {
    if (c->bf16) launch_cast_shadow<bf16_t>(n->theta, (bf16_t*)n->shadow_u, (long long)c->L * n->P, c->st);
    if (c->paper && n == &c->G) {
      if (c->bf16) paper_rebuild_w4<bf16_t>(c); else paper_rebuild_w4<float>(c);
      continue;
    }
    if (c->bf16) refresh_transposes<bf16_t>(c, *n, n == &c->G); else refresh_transposes<float>(c, *n, n == &c->G);
  }
  c->shadows_dirty = false;
}

// ---- launch helpers ---------------------------------------------------------------------------------------
template <typename T>
void conv_call(gan_ctx* c, const char* name, int mode, int epi, const void* A, const void* W, long long wstride, void* Out,
               const void* Aux, int C, int N, int Hin, int Hr, int seg_first, int nseg, int n, int w_nstride = 0,
               double flops_alg = -1.0, bool stats = false) {
  ConvArgs a = {};
  a.A = A; a.W = W; a.Out = Out; a.Aux = Aux; a.w_nstride = w_nstride ? w_nstride : N;
  const int tr = layer_tile_rows(c, N, Hr * Hr);
  a.offs = c->rb.offs; a.tpre = tpre_of(c, Hr * Hr, tr); a.tmodel = tmodel_of(c, Hr * Hr, tr); a.tile_rows = tr;
  a.w_stride = wstride; a.L = c->L; a.seg_first = seg_first; a.nseg = nseg; a.seg_samples = n;
  a.C = C; a.N = N; a.Hin = Hin; a.Hr = Hr; a.ub_tiles = ub_tiles(c, n, Hr * Hr, tr);
  a.slope = c->cfg.leaky_slope;
  a.stat_partial = stats ? c->stat_partial : nullptr;
  const int ntaps = mode == MODE_DOWN ? 16 : (mode == MODE_UP ? 4 : 1);
  const int phases = mode == MODE_UP ? 4 : 1;
  const double rows = (double)n * nseg * Hr * Hr * phases;
  const double frac = mode == MODE_DENSE ? 1.0 : valid_tap_fraction(Hr);
  const double flops = flops_alg >= 0 ? flops_alg : 2.0 * rows * N * C * ntaps * frac;
  const double in_elems = mode == MODE_DENSE ? rows * C : (double)n * nseg * Hin * Hin * C;
  const double bytes = sizeof(T) * (in_elems + rows * N + (double)c->L * (mode == MODE_DENSE ? 1 : 16) * C * N);
  char detail[64];
  snprintf(detail, sizeof(detail), "[C%d N%d H%d seg%d]", C, N, Hr, nseg);
  (void)name;
  Scope s(c, conv_variant_name(mode, epi, a), flops, bytes, detail);
  launch_conv<T>(mode, epi, a, c->st);
}

// Row splits of a weight-gradient launch whose output tiles alone would not fill the chip (few models): every
// model's rows are shared by this many blocks per tile, whose partial results are added in a fixed order.  A function
// of the configuration only -- the number of models and the layer's shape -- never of the batch.
int wgrad_ksplit(const gan_ctx* c, int Cb, int Cs, int ntaps) {
  const long long blocks = (long long)c->L * wgrad_tiles_per_model(ntaps, Cb, Cs);
  return (int)std::min<long long>(std::max<long long>(512 / blocks, 1), WG_MAX_KSPLIT);
}

// ksplit == 0: split as wgrad_ksplit says, through c->wg_part, and leave the sum in dW; ksplit >= 1: the caller's
// own split (partials left at dW + split * L * stride).
template <typename T>
void wgrad_call(gan_ctx* c, const char* name, const void* Big, const void* Small, float* dW, long long stride, int Cb, int Cs,
                int Hs, int ntaps, int nseg, int n, double flops_alg = -1.0, int ksplit = 0, hipStream_t st = nullptr) {
  if (!st) st = c->st;
  WgradArgs a = {};
  a.Big = Big; a.Small = Small; a.dW = dW; a.offs = c->rb.offs; a.order = c->rb.order; a.dw_stride = stride;
  a.L = c->L; a.nseg = nseg; a.seg_samples = n; a.Cb = Cb; a.Cs = Cs; a.Hs = Hs; a.ntaps = ntaps; a.ksplit = ksplit;
  a.split_stride = (long long)c->L * stride;
  const long long layer = (long long)ntaps * Cb * Cs;
  const int auto_split = ksplit == 0 ? wgrad_ksplit(c, Cb, Cs, ntaps) : 0;
  if (ksplit == 0) {
    a.ksplit = auto_split;
    if (auto_split > 1) {
      a.dW = c->wg_part; a.dw_stride = layer; a.split_stride = (long long)c->L * layer;
    }
  }
  const double rows = (double)n * nseg * Hs * Hs;
  const double frac = ntaps == 1 ? 1.0 : valid_tap_fraction(Hs);
  const double big_elems = ntaps == 1 ? rows * Cb : (double)n * nseg * 4 * Hs * Hs * Cb;
  const double bytes = sizeof(T) * (big_elems + rows * Cs) + 4.0 * c->L * ntaps * Cb * Cs;
  char detail[64];
  snprintf(detail, sizeof(detail), "[Cb%d Cs%d H%d seg%d]", Cb, Cs, Hs, nseg);
  (void)name;
  {
    Scope s(c, wgrad_variant_name(a), flops_alg >= 0 ? flops_alg : 2.0 * rows * Cb * Cs * ntaps * frac, bytes, detail, st);
    launch_wgrad<T>(a, st);
  }
  if (auto_split > 1) launch_sum_splits(c->wg_part, dW, stride, layer, c->L, auto_split, st);
}

template <typename T>
NormArgs norm_args(gan_ctx* c, Net& net, int C, int rps, long long gamma, long long beta, long long rs, float* mean, float* var,
                   float* rstd, float* sums, int seg_first, int nseg, int n, float slope) {
  NormArgs a;
  memset(&a, 0, sizeof(a));
  a.mean = mean; a.var = var; a.rstd = rstd; a.sums = sums;
  a.gamma = net.theta + gamma; a.beta = net.theta + beta; a.dgamma = net.g + gamma; a.dbeta = net.g + beta;
  a.pstride = net.P;
  a.run_mean = net.run_mean + rs; a.run_var = net.run_var + rs; a.rstride = net.nbn;
  a.offs = c->rb.offs; a.counts = c->rb.counts; a.sample_model = c->rb.sample_model;
  a.L = c->L; a.C = C; a.rps = rps; a.seg_first = seg_first; a.nseg = nseg; a.seg_samples = n; a.n = n;
  a.slope = slope; a.eps = c->cfg.bn_eps; a.momentum = c->cfg.bn_momentum;
  return a;
}

// BatchNorm (batch statistics, or the running ones) + activation: x -> y
// gemm_rps / gemm_phases describe the GEMM that produced x and left per-tile column sums in c->stat_partial
template <typename T>
void bn_forward(gan_ctx* c, NormArgs a, const void* x, void* y, bool use_running, bool update_running, int gemm_rps,
                int gemm_phases, int col_groups = 1) {
  a.x = x; a.y = y;
  const double elems = (double)a.n * a.nseg * a.rps * a.C;
  if (use_running) {
    launch_bn_from_running(a, c->st);
  } else {
    const int tr = layer_tile_rows(c, a.C * col_groups, gemm_rps);     // the tile height of the GEMM that left the partials (N = C * col_groups)
    a.fold_running = update_running && a.nseg == 1 && a.run_mean && a.run_var;
    launch_bn_stats_from_partial(a, c->stat_partial, tpre_of(c, gemm_rps, tr), ub_tiles(c, a.n, gemm_rps, tr), gemm_phases, col_groups, tr,
                                 gemm_rps, conv_stat_split(a.C * col_groups, tr), c->st);
    if (update_running && !a.fold_running) launch_bn_running(a, c->st);
  }
  Scope s(c, "bn_apply", 0, 2 * elems * sizeof(T));
  launch_bn_apply<T>(a, c->st);
}

// dy (w.r.t. the activated output) -> dx (w.r.t. the pre-normalisation tensor), plus dgamma / dbeta
template <typename T>
void bn_backward(gan_ctx* c, NormArgs a, const void* x, const void* dy, void* dx, bool param_grads) {
  a.x = x; a.dy = dy; a.y = dx;
  a.fold_grads = param_grads && a.nseg == 1;
  const double elems = (double)a.n * a.nseg * a.rps * a.C;
  {
    Scope s(c, "bn_bwd_reduce", 0, 2 * elems * sizeof(T));
    launch_bn_bwd_reduce<T>(a, tpre_of(c, a.rps, BN_RED_ROWS), tmodel_of(c, a.rps, BN_RED_ROWS), ub_tiles(c, a.n, a.rps, BN_RED_ROWS),
                            c->stat_partial, c->st);
  }
  if (param_grads && !a.fold_grads) launch_bn_param_grad(a, c->st);
  Scope s(c, "bn_bwd_apply", 0, 3 * elems * sizeof(T));
  launch_bn_bwd_apply<T>(a, c->st);
}

double img_flops(const ConvLayer& cl, int n, int nseg) {
  return 2.0 * n * nseg * cl.Hs * cl.Hs * 16 * cl.Cb * cl.Cs * valid_tap_fraction(cl.Hs);
}

// Patch matrix of an image-side tensor (or of the caller's real batch when img == NULL).
template <typename T>
void im2col_call(gan_ctx* c, const ConvLayer& cl, const void* img, const float* real, void* out, int Kc, int nslot, int seg, int n) {
  Im2colArgs a;
  memset(&a, 0, sizeof(a));
  a.img = img; a.real = real; a.perm = c->rb.perm; a.out = out; a.offs = c->rb.offs; a.sample_slot = c->rb.sample_slot;
  a.L = c->L; a.n = n; a.CB = cl.Cb; a.Hs = cl.Hs; a.Kc = Kc; a.nslot = nslot; a.seg = seg; a.seg_samples = n;
  const double rows = (double)n * cl.Hs * cl.Hs;
  Scope s(c, "im2col", 0, rows * (4.0 * cl.Cb * (real ? 4 : sizeof(T)) + (double)Kc * sizeof(T)));
  launch_im2col<T>(a, c->st);
}

// transposed conv onto the image side: feat (absolute segment seg) -> out (same segment indexing)
template <typename T>
void up_img_call(gan_ctx* c, Net& net, const ConvLayer& cl, const void* feat, void* out, const void* aux, int mode, int seg, int n) {
  UpImgArgs a;
  memset(&a, 0, sizeof(a));
  a.feat = feat; a.w = (const T*)net.shadow_u + cl.w; a.w_stride = net.P; a.out = out; a.aux = aux;
  a.bias = mode == 1 ? net.theta + cl.bias : nullptr; a.bias_stride = net.P;
  a.offs = c->rb.offs; a.sample_model = c->rb.sample_model; a.L = c->L; a.n = n; a.seg = seg; a.seg_samples = n;
  a.CB = cl.Cb; a.CBT = cl.CBT; a.Cs = cl.Cs; a.Hs = cl.Hs; a.mode = mode;
  Scope s(c, "up_img", img_flops(cl, n, 1), sizeof(T) * (double)n * cl.Hs * cl.Hs * (cl.Cs + 4.0 * cl.Cb * (mode == 2 ? 2 : 1)));
  launch_up_img<T>(a, c->st);
}

PackArgs pack_args(gan_ctx* c, Net& net, const ConvLayer& cl, int Kc, int nslot, void* wp) {
  PackArgs a;
  memset(&a, 0, sizeof(a));
  a.w = net.theta + cl.w; a.bias = (nslot > 0 && cl.bias >= 0) ? net.theta + cl.bias : nullptr;
  a.dw = net.g + cl.w; a.dbias = (nslot > 0 && cl.bias >= 0) ? net.g + cl.bias : nullptr;
  a.pstride = net.P; a.wp = wp; a.dwp = c->dwp;
  a.L = c->L; a.CB = cl.Cb; a.CBT = cl.CBT; a.Cs = cl.Cs; a.Kc = Kc; a.nslot = nslot; a.nsplit = c->img_ksplit;
  return a;
}

// ---- the networks -------------------------------------------------------------------------------------------
template <typename T>
void g_forward(gan_ctx* c, int n, bool use_running, bool update_running) {
  Net& G = c->G;
  const float relu = 0.f;
  conv_call<T>(c, "gemm_dense", MODE_DENSE, EPI_NONE, c->zin, (const T*)G.shadow_u + G.fc_w, G.P, c->gpre[0], nullptr, G.Kp, G.J,
               1, 1, 0, 1, n, 0, -1.0, !use_running);
  bn_forward<T>(c, norm_args<T>(c, G, G.C0, G.h0 * G.h0, G.fc_gamma, G.fc_beta, G.fc_rs, c->g_mean[0], c->g_var[0], c->g_rstd[0],
                                c->g_sums[0], 0, 1, n, relu),
                c->gpre[0], c->gact[0], use_running, update_running, 1, 1, G.h0 * G.h0);
  const int nl = (int)G.conv.size();
  for (int i = 0; i + 1 < nl; ++i) {
    const ConvLayer& cl = G.conv[i];
    conv_call<T>(c, "gemm_up", MODE_UP, EPI_NONE, c->gact[i], (const T*)G.shadow_u + cl.w, G.P, c->gpre[i + 1], nullptr, cl.Cs, cl.Cb,
                 cl.Hs, cl.Hs, 0, 1, n, 0, -1.0, !use_running);
    bn_forward<T>(c, norm_args<T>(c, G, cl.Cb, 4 * cl.Hs * cl.Hs, cl.gamma, cl.beta, cl.rs, c->g_mean[i + 1], c->g_var[i + 1],
                                  c->g_rstd[i + 1], c->g_sums[i + 1], 0, 1, n, relu),
                  c->gpre[i + 1], c->gact[i + 1], use_running, update_running, cl.Hs * cl.Hs, 4);
  }
  // last transposed conv (+bias, tanh) straight into the fake half of D's image buffer
  const ConvLayer& cl = G.conv[nl - 1];
  // G's samples sit in segment 0, the fake images in segment 1 of D's image buffer: offset the output pointer
  T* fake = (T*)c->xd + (long long)n * 4 * cl.Hs * cl.Hs * cl.Cb;
  up_img_call<T>(c, G, cl, c->gact[nl - 1], fake, nullptr, 1, 0, n);
}

template <typename T>
void d_forward(gan_ctx* c, int n, int seg_first, int nseg, bool update_running) {
  Net& D = c->D;
  const float slope = c->cfg.leaky_slope;
  // first conv (+label maps, bias, LeakyReLU) as a row-by-row GEMM over the patch matrix
  const ConvLayer& c1 = D.conv[0];
  conv_call<T>(c, "gemm_dense_img", MODE_DENSE, EPI_LRELU, c->colD, c->wpD, (long long)c1.Cs * c->KcD, c->dact[0], nullptr, c->KcD,
               c1.Cs, 1, c1.Hs, seg_first, nseg, n, 0, img_flops(c1, n, nseg));
  const int nl = (int)D.conv.size();
  for (int j = 1; j < nl; ++j) {
    const ConvLayer& cl = D.conv[j];
    conv_call<T>(c, "gemm_down", MODE_DOWN, EPI_NONE, c->dact[j - 1], (const T*)D.shadow_d + cl.w, D.P, c->dpre[j], nullptr, cl.Cb,
                 cl.Cs, 2 * cl.Hs, cl.Hs, seg_first, nseg, n, 0, -1.0, true);
    bn_forward<T>(c, norm_args<T>(c, D, cl.Cs, cl.Hs * cl.Hs, cl.gamma, cl.beta, cl.rs, c->d_mean[j], c->d_var[j], c->d_rstd[j],
                                  c->d_sums[j], seg_first, nseg, n, slope),
                  c->dpre[j], c->dact[j], false, update_running, cl.Hs * cl.Hs, 1);
  }
  HeadArgs h;
  memset(&h, 0, sizeof(h));
  h.feat = c->dact[nl - 1]; h.w = D.theta + D.fc_w; h.b = D.theta + D.fc_b; h.pstride = D.P; h.logits = c->logits;
  h.offs = c->rb.offs; h.sample_model = c->rb.sample_model; h.L = c->L; h.K = D.K;
  h.seg_first = seg_first; h.nseg = nseg; h.seg_samples = n; h.n = n;
  Scope s(c, "head_fwd", 0, sizeof(T) * (double)n * nseg * D.K);
  launch_head_fwd<T>(h, c->st);
}

// mode 0: discriminator cost on (real, fake); mode 1: generator cost on the fake segment
void loss_call(gan_ctx* c, int n, int mode) {
  HeadArgs h;
  memset(&h, 0, sizeof(h));
  h.logits = c->logits; h.dlogits = c->dlogits; h.loss = mode == 0 ? c->loss_d : c->loss_g;
  h.offs = c->rb.offs; h.L = c->L; h.seg_first = mode == 0 ? 0 : 1; h.nseg = mode == 0 ? 2 : 1; h.seg_samples = n; h.n = n;
  h.mode = mode; h.scale = mode == 0 ? c->cfg.d_loss_scale : c->cfg.g_loss_scale;
  launch_loss(h, c->st);
}

// Backward through D.  param_grads: fill D's gradient block (both segments summed).  to_image: continue down to
// d cost / d fake, multiplied by the tanh derivative, into dimg.
// adam (with param_grads): D's planned update, whose step counts are already advanced; the update of a convolution's
// weights is enqueued beside the chain as soon as its gradient is complete and its data gradient has read the old ones.
template <typename T>
void d_backward(gan_ctx* c, int n, int seg_first, int nseg, bool param_grads, bool to_image, const AdamArgs* adam = nullptr) {
  Net& D = c->D;
  hipStream_t side = side_stream(c);
  const float slope = c->cfg.leaky_slope;
  const int nl = (int)D.conv.size();
  HeadArgs h;
  memset(&h, 0, sizeof(h));
  h.feat = c->dact[nl - 1]; h.dfeat = c->bufA; h.w = D.theta + D.fc_w; h.b = D.theta + D.fc_b;
  h.dw = D.g + D.fc_w; h.db = D.g + D.fc_b; h.pstride = D.P; h.dlogits = c->dlogits;
  h.part = c->head_part; h.rsplit = c->head_rsplit;
  h.offs = c->rb.offs; h.sample_model = c->rb.sample_model; h.L = c->L; h.K = D.K;
  h.seg_first = seg_first; h.nseg = nseg; h.seg_samples = n; h.n = n;
  { Scope s(c, "head_bwd_data", 0, sizeof(T) * (double)n * nseg * D.K); launch_head_bwd_data<T>(h, c->st); }
  if (param_grads) { Scope s(c, "head_bwd_w", 0, sizeof(T) * (double)n * nseg * D.K); launch_head_bwd_w<T>(h, c->st); }
  int pending = -1;                // region of D's planned update whose turn comes next
  for (int j = nl - 1; j >= 1; --j) {
    const ConvLayer& cl = D.conv[j];
    // in place: the pre-normalisation tensor is not needed again in this step, its gradient takes its place
    void* dx = c->dpre[j];
    bn_backward<T>(c, norm_args<T>(c, D, cl.Cs, cl.Hs * cl.Hs, cl.gamma, cl.beta, cl.rs, c->d_mean[j], c->d_var[j], c->d_rstd[j],
                                   c->d_sums[j], seg_first, nseg, n, slope),
                   c->dpre[j], c->bufA, dx, param_grads);
    if (param_grads) {
      // Beside the chain, in this order: the update of the layer above (its data gradient, which read the old weights,
      // is done; being bandwidth-bound it pairs with the data-gradient GEMM below), then this layer's weight gradient.
      order_after(c, side, c->st);
      if (adam && pending >= 0) adam_region_call<T>(c, *adam, pending, side);
      wgrad_call<T>(c, "gemm_wgrad", c->dact[j - 1], dx, D.g + cl.w, D.P, cl.Cb, cl.Cs, cl.Hs, 16, nseg, n, -1.0, 0, side);
      pending = j - 1;
    }
    // data gradient; for the first conv's output the LeakyReLU derivative is applied in the epilogue
    conv_call<T>(c, "gemm_up", MODE_UP, j == 1 ? EPI_ACT_BWD : EPI_NONE, dx, (const T*)D.shadow_u + cl.w, D.P, c->bufA,
                 j == 1 ? c->dact[0] : nullptr, cl.Cs, cl.Cb, cl.Hs, cl.Hs, seg_first, nseg, n);
  }
  if (param_grads && adam && pending >= 0) {
    order_after(c, side, c->st);
    adam_region_call<T>(c, *adam, pending, side);
  }
  const ConvLayer& c1 = D.conv[0];
  if (param_grads) {
    // taps, label-map class sums and the bias gradient in one GEMM over the patch matrix
    wgrad_call<T>(c, "gemm_wgrad_img", c->colD, c->bufA, c->dwp, (long long)c->KcD * c1.Cs, c->KcD, c1.Cs, c1.Hs, 1, nseg, n,
                  img_flops(c1, n, nseg), c->img_ksplit);
    launch_unpack_dw(pack_args(c, D, c1, c->KcD, c->nslot, c->wpD), c->st);
  }
  if (to_image)   // d cost / d fake, times the tanh derivative (fake segment only)
    up_img_call<T>(c, D, c1, c->bufA, c->dimg, c->xd, 2, 1, n);
}

// Backward through G from dimg (fake segment) = d cost / d (pre-tanh output).
template <typename T>
void g_backward(gan_ctx* c, int n, const AdamArgs* adam = nullptr) {
  Net& G = c->G;
  hipStream_t side = side_stream(c);
  const int nl = (int)G.conv.size();
  const ConvLayer& last = G.conv[nl - 1];
  const T* dlast = (const T*)c->dimg + (long long)n * 4 * last.Hs * last.Hs * last.Cb;
  {
    im2col_call<T>(c, last, dlast, nullptr, c->colG, c->KcG, 0, 0, n);
    wgrad_call<T>(c, "gemm_wgrad_img", c->colG, c->gact[nl - 1], c->dwp, (long long)c->KcG * last.Cs, c->KcG, last.Cs, last.Hs, 1, 1, n,
                  img_flops(last, n, 1), c->img_ksplit);
    launch_unpack_dw(pack_args(c, G, last, c->KcG, 0, c->wpG), c->st);
    ImgBiasArgs b;
    b.img = dlast; b.partial = c->bias_partial; b.dbias = G.g + last.bias; b.pstride = G.P; b.offs = c->rb.offs;
    b.L = c->L; b.CB = last.Cb; b.HW = 4 * last.Hs * last.Hs;
    launch_img_bias_grad<T>(b, c->st);
    conv_call<T>(c, "gemm_dense_img", MODE_DENSE, EPI_NONE, c->colG, c->wpG, (long long)last.Cs * c->KcG, c->bufA, nullptr, c->KcG,
                 last.Cs, 1, last.Hs, 0, 1, n, 0, img_flops(last, n, 1));
  }
  int pending = -1;
  for (int i = nl - 2; i >= 0; --i) {
    const ConvLayer& cl = G.conv[i];
    void* dx = c->gpre[i + 1];     // in place, as in D
    bn_backward<T>(c, norm_args<T>(c, G, cl.Cb, 4 * cl.Hs * cl.Hs, cl.gamma, cl.beta, cl.rs, c->g_mean[i + 1], c->g_var[i + 1],
                                   c->g_rstd[i + 1], c->g_sums[i + 1], 0, 1, n, 0.f),
                   c->gpre[i + 1], c->bufA, dx, true);
    order_after(c, side, c->st);
    if (adam && pending >= 0) adam_region_call<T>(c, *adam, pending, side);      // as in D
    wgrad_call<T>(c, "gemm_wgrad", dx, c->gact[i], G.g + cl.w, G.P, cl.Cb, cl.Cs, cl.Hs, 16, 1, n, -1.0, 0, side);
    pending = i;
    conv_call<T>(c, "gemm_down", MODE_DOWN, EPI_NONE, dx, (const T*)G.shadow_d + cl.w, G.P, c->bufA, nullptr, cl.Cb, cl.Cs,
                 2 * cl.Hs, cl.Hs, 0, 1, n);
  }
  bn_backward<T>(c, norm_args<T>(c, G, G.C0, G.h0 * G.h0, G.fc_gamma, G.fc_beta, G.fc_rs, c->g_mean[0], c->g_var[0], c->g_rstd[0],
                                 c->g_sums[0], 0, 1, n, 0.f),
                 c->gpre[0], c->bufA, c->gpre[0], true);
  // (row-split partial sums share one scratch area with the weight gradients above: same stream)
  order_after(c, side, c->st);
  if (adam && pending >= 0) adam_region_call<T>(c, *adam, pending, side);
  wgrad_call<T>(c, "gemm_wgrad_dense", c->gpre[0], c->zin, G.g + G.fc_w, G.P, G.J, G.Kp, 1, 1, 1, n, -1.0, 0, side);
  order_after(c, c->st, side);
}

// ---- the networks as printed in the paper's Tables 1 and 2 ---------------------------------------------------
PointArgs point_args(gan_ctx* c, void* x, int C, int Cpad, int HW, int seg_first, int nseg, int n) {
  PointArgs a;
  memset(&a, 0, sizeof(a));
  a.x = x; a.offs = c->rb.offs; a.sample_model = c->rb.sample_model; a.L = c->L; a.n = n; a.C = C; a.Cpad = Cpad; a.HW = HW;
  a.seg_first = seg_first; a.nseg = nseg; a.seg_samples = n; a.slope = 1.f; a.scale = 1.f;
  a.seed_lo = (unsigned)(c->cfg.seed & 0xffffffffull); a.seed_hi = (unsigned)(c->cfg.seed >> 32);
  return a;
}
// dropout of D's block `layer` (1-based) in the passes pass0 (first processed segment) and pass0 + 1
void with_dropout(gan_ctx* c, PointArgs& a, int layer, int pass0, int step_add) {
  const float p = c->cfg.dropout_p;
  if (!(p > 0.f)) return;
  a.thr = (unsigned)ceil((double)p * 16777216.0);
  a.scale = 1.0f / (1.0f - p);
  a.layer = layer; a.pass_of_seg[0] = pass0; a.pass_of_seg[1] = pass0 + 1;
  a.steps = c->D.t; a.step_add = step_add;
}

// BatchNorm whose statistics are taken from the stored tensor; no activation after it
template <typename T>
void bn_forward_direct(gan_ctx* c, NormArgs a, const void* x, void* y, float eps, bool use_running, bool update_running) {
  a.x = x; a.y = y; a.eps = eps; a.slope = 1.f;
  if (use_running) {
    launch_bn_from_running(a, c->st);
  } else {
    launch_bn_stats_direct<T>(a, a.C, c->st);
    if (update_running) launch_bn_running(a, c->st);
  }
  Scope s(c, "bn_apply", 0, 2.0 * a.n * a.nseg * a.rps * a.C * sizeof(T));
  launch_bn_apply<T>(a, c->st);
}

template <typename T>
void paper_g_forward(gan_ctx* c, int n, bool use_running, bool update_running) {
  Net& G = c->G;
  const gan_config& f = c->cfg;
  conv_call<T>(c, "gemm_dense", MODE_DENSE, EPI_NONE, c->zin, (const T*)G.shadow_u + G.fc_w, G.P, c->gpre[0], nullptr, G.Kp, G.J,
               1, 1, 0, 1, n);
  {
    PointArgs a = point_args(c, c->gpre[0], G.J, G.J, 1, 0, 1, n);          // + bias, ReLU
    a.bias = G.theta + G.fc_bias; a.pstride = G.P; a.slope = 0.f;
    Scope s(c, "bias_act_dropout", 0, 2.0 * n * G.J * sizeof(T));
    launch_point_fwd<T>(a, c->st);
  }
  bn_forward_direct<T>(c, norm_args<T>(c, G, G.C0, G.h0 * G.h0, G.fc_gamma, G.fc_beta, G.fc_rs, c->g_mean[0], c->g_var[0], c->g_rstd[0],
                                       c->g_sums[0], 0, 1, n, 1.f),
                       c->gpre[0], c->gact[0], f.bn_eps_first, use_running, update_running);
  const int nl = (int)G.conv.size();
  for (int i = 0; i + 1 < nl; ++i) {                   // Upsample x2 + Conv k3 as a k4 s2 p1 transposed convolution
    const ConvLayer& cl = G.conv[i];
    conv_call<T>(c, "gemm_up", MODE_UP, EPI_NONE, c->gact[i], (const T*)G.w4u + cl.w4, G.P4, c->gpre[i + 1], nullptr, cl.Cs, cl.Cb,
                 cl.Hs, cl.Hs, 0, 1, n, 0, -1.0, !use_running);
    NormArgs a = norm_args<T>(c, G, cl.Cb, 4 * cl.Hs * cl.Hs, cl.gamma, cl.beta, cl.rs, c->g_mean[i + 1], c->g_var[i + 1],
                              c->g_rstd[i + 1], c->g_sums[i + 1], 0, 1, n, f.leaky_slope);
    bn_forward<T>(c, a, c->gpre[i + 1], c->gact[i + 1], use_running, update_running, cl.Hs * cl.Hs, 4);
  }
  const ConvLayer& cl = G.conv[nl - 1];                // Conv k3 s1 p1 (+bias) -> tanh, into the fake half of D's image buffer
  Conv3Args a;
  memset(&a, 0, sizeof(a));
  a.in = c->gact[nl - 1]; a.out = c->xd; a.w = G.theta + cl.w; a.w_stride = G.P; a.bias = G.theta + cl.bias; a.bias_stride = G.P;
  a.offs = c->rb.offs; a.sample_model = c->rb.sample_model; a.L = c->L; a.n = n; a.H = cl.Hs; a.Cin = cl.Cs; a.CO = cl.Cb;
  a.out_seg = 1; a.seg_samples = n;
  Scope s(c, "conv3_img", 2.0 * n * cl.Hs * cl.Hs * 9 * cl.Cs * cl.Cb, sizeof(T) * (double)n * cl.Hs * cl.Hs * (cl.Cs + cl.Cb));
  launch_conv3_fwd<T>(a, c->st);
}

// pass0: dropout pass id of the first processed segment (real 0, fake 1, fake through the updated D 2);
// step_add: 1 before D's update of this iteration, 0 after it (the iteration number is D's step count + step_add)
template <typename T>
void paper_d_forward(gan_ctx* c, int n, int seg_first, int nseg, bool update_running, int pass0, int step_add) {
  Net& D = c->D;
  const gan_config& f = c->cfg;
  const ConvLayer& c1 = D.conv[0];
  conv_call<T>(c, "gemm_dense_img", MODE_DENSE, EPI_LRELU, c->colD, c->wpD, (long long)c1.Cs * c->KcD, c->dact[0], nullptr, c->KcD,
               c1.Cs, 1, c1.Hs, seg_first, nseg, n, 0, img_flops(c1, n, nseg));
  if (f.dropout_p > 0.f) {
    PointArgs a = point_args(c, c->dact[0], c1.cs_real, c1.Cs, c1.Hs * c1.Hs, seg_first, nseg, n);
    with_dropout(c, a, 1, pass0, step_add);
    Scope s(c, "bias_act_dropout", 0, 2.0 * n * nseg * c1.Hs * c1.Hs * c1.cs_real * sizeof(T));
    launch_point_fwd<T>(a, c->st);
  }
  const int nl = (int)D.conv.size();
  for (int j = 1; j < nl; ++j) {
    const ConvLayer& cl = D.conv[j];
    conv_call<T>(c, "gemm_down", MODE_DOWN, EPI_NONE, c->dact[j - 1], (const T*)D.shadow_d + cl.w, D.P, c->dpre[j], nullptr, cl.Cb,
                 cl.Cs, 2 * cl.Hs, cl.Hs, seg_first, nseg, n);
    PointArgs a = point_args(c, c->dpre[j], cl.cs_real, cl.Cs, cl.Hs * cl.Hs, seg_first, nseg, n);
    a.bias = D.theta + cl.bias; a.pstride = D.P; a.slope = f.leaky_slope;
    with_dropout(c, a, j + 1, pass0, step_add);
    { Scope s(c, "bias_act_dropout", 0, 2.0 * n * nseg * cl.Hs * cl.Hs * cl.cs_real * sizeof(T)); launch_point_fwd<T>(a, c->st); }
    bn_forward_direct<T>(c, norm_args<T>(c, D, cl.Cs, cl.Hs * cl.Hs, cl.gamma, cl.beta, cl.rs, c->d_mean[j], c->d_var[j], c->d_rstd[j],
                                         c->d_sums[j], seg_first, nseg, n, 1.f),
                         c->dpre[j], c->dact[j], f.bn_eps, false, update_running);
  }
  HeadArgs h;
  memset(&h, 0, sizeof(h));
  h.feat = c->dact[nl - 1]; h.w = D.theta + D.fc_w; h.b = D.theta + D.fc_b; h.pstride = D.P; h.logits = c->logits;
  h.offs = c->rb.offs; h.sample_model = c->rb.sample_model; h.L = c->L; h.K = D.K;
  h.seg_first = seg_first; h.nseg = nseg; h.seg_samples = n; h.n = n;
  Scope s(c, "head_fwd", 0, sizeof(T) * (double)n * nseg * D.K);
  launch_head_fwd<T>(h, c->st);
}

template <typename T>
void paper_d_backward(gan_ctx* c, int n, int seg_first, int nseg, bool param_grads, bool to_image, int pass0, int step_add) {
  Net& D = c->D;
  const gan_config& f = c->cfg;
  const int nl = (int)D.conv.size();
  HeadArgs h;
  memset(&h, 0, sizeof(h));
  h.feat = c->dact[nl - 1]; h.dfeat = c->bufA; h.w = D.theta + D.fc_w; h.b = D.theta + D.fc_b;
  h.dw = D.g + D.fc_w; h.db = D.g + D.fc_b; h.pstride = D.P; h.dlogits = c->dlogits;
  h.part = c->head_part; h.rsplit = c->head_rsplit;
  h.offs = c->rb.offs; h.sample_model = c->rb.sample_model; h.L = c->L; h.K = D.K;
  h.seg_first = seg_first; h.nseg = nseg; h.seg_samples = n; h.n = n;
  { Scope s(c, "head_bwd_data", 0, sizeof(T) * (double)n * nseg * D.K); launch_head_bwd_data<T>(h, c->st); }
  if (param_grads) { Scope s(c, "head_bwd_w", 0, sizeof(T) * (double)n * nseg * D.K); launch_head_bwd_w<T>(h, c->st); }
  for (int j = nl - 1; j >= 1; --j) {
    const ConvLayer& cl = D.conv[j];
    NormArgs na = norm_args<T>(c, D, cl.Cs, cl.Hs * cl.Hs, cl.gamma, cl.beta, cl.rs, c->d_mean[j], c->d_var[j], c->d_rstd[j],
                               c->d_sums[j], seg_first, nseg, n, 1.f);
    na.eps = f.bn_eps;
    bn_backward<T>(c, na, c->dpre[j], c->bufA, c->bufB, param_grads);         // -> gradient w.r.t. the dropped activations
    PointArgs a = point_args(c, c->bufB, cl.cs_real, cl.Cs, cl.Hs * cl.Hs, seg_first, nseg, n);
    a.saved = c->dpre[j]; a.slope = f.leaky_slope;
    with_dropout(c, a, j + 1, pass0, step_add);
    { Scope s(c, "act_dropout_bwd", 0, 3.0 * n * nseg * cl.Hs * cl.Hs * cl.cs_real * sizeof(T)); launch_point_bwd<T>(a, c->st); }
    if (param_grads) {
      launch_col_sum<T>(a, D.g + cl.bias, D.P, c->st);
      wgrad_call<T>(c, "gemm_wgrad", c->dact[j - 1], c->bufB, D.g + cl.w, D.P, cl.Cb, cl.Cs, cl.Hs, 16, nseg, n);
    }
    conv_call<T>(c, "gemm_up", MODE_UP, j == 1 ? EPI_ACT_BWD : EPI_NONE, c->bufB, (const T*)D.shadow_u + cl.w, D.P, c->bufA,
                 j == 1 ? c->dact[0] : nullptr, cl.Cs, cl.Cb, cl.Hs, cl.Hs, seg_first, nseg, n);
  }
  const ConvLayer& c1 = D.conv[0];
  if (f.dropout_p > 0.f) {      // the first block's dropout (its LeakyReLU derivative came with the data gradient above)
    PointArgs a = point_args(c, c->bufA, c1.cs_real, c1.Cs, c1.Hs * c1.Hs, seg_first, nseg, n);
    a.saved = c->dact[0];
    with_dropout(c, a, 1, pass0, step_add);
    Scope s(c, "act_dropout_bwd", 0, 2.0 * n * nseg * c1.Hs * c1.Hs * c1.cs_real * sizeof(T));
    launch_point_bwd<T>(a, c->st);
  }
  if (param_grads) {
    wgrad_call<T>(c, "gemm_wgrad_img", c->colD, c->bufA, c->dwp, (long long)c->KcD * c1.Cs, c->KcD, c1.Cs, c1.Hs, 1, nseg, n,
                  img_flops(c1, n, nseg), c->img_ksplit);
    launch_unpack_dw(pack_args(c, D, c1, c->KcD, c->nslot, c->wpD), c->st);
    for (const ConvLayer& cl : D.conv) launch_clear_fourth_taps(D.g + cl.w, D.P, c->L, cl.CBT, cl.Cs, c->st);
  }
  if (to_image) up_img_call<T>(c, D, c1, c->bufA, c->dimg, c->xd, 2, 1, n);
}

template <typename T>
void paper_g_backward(gan_ctx* c, int n) {
  Net& G = c->G;
  const gan_config& f = c->cfg;
  const int nl = (int)G.conv.size();
  const ConvLayer& last = G.conv[nl - 1];
  const T* dlast = (const T*)c->dimg + (long long)n * last.Hs * last.Hs * last.Cb;
  {
    Conv3Args a;
    memset(&a, 0, sizeof(a));
    a.in = c->gact[nl - 1]; a.dout = c->dimg; a.din = c->bufA; a.w = G.theta + last.w; a.w_stride = G.P;
    a.offs = c->rb.offs; a.sample_model = c->rb.sample_model; a.L = c->L; a.n = n; a.H = last.Hs; a.Cin = last.Cs; a.CO = last.Cb;
    a.out_seg = 1; a.seg_samples = n;
    { Scope s(c, "conv3_img_wgrad", 2.0 * n * last.Hs * last.Hs * 9 * last.Cs * last.Cb, sizeof(T) * (double)n * last.Hs * last.Hs * (last.Cs + last.Cb));
      launch_conv3_wgrad<T>(a, c->c3_part, G.g + last.w, G.P, c->st); }
    ImgBiasArgs b;
    b.img = dlast; b.partial = c->bias_partial; b.dbias = G.g + last.bias; b.pstride = G.P; b.offs = c->rb.offs;
    b.L = c->L; b.CB = last.Cb; b.HW = last.Hs * last.Hs;
    launch_img_bias_grad<T>(b, c->st);
    Scope s(c, "conv3_img_dgrad", 2.0 * n * last.Hs * last.Hs * 9 * last.Cs * last.Cb, sizeof(T) * (double)n * last.Hs * last.Hs * (last.Cs + last.Cb));
    launch_conv3_dgrad<T>(a, c->st);
  }
  for (int i = nl - 2; i >= 0; --i) {
    const ConvLayer& cl = G.conv[i];
    NormArgs na = norm_args<T>(c, G, cl.Cb, 4 * cl.Hs * cl.Hs, cl.gamma, cl.beta, cl.rs, c->g_mean[i + 1], c->g_var[i + 1],
                               c->g_rstd[i + 1], c->g_sums[i + 1], 0, 1, n, f.leaky_slope);
    bn_backward<T>(c, na, c->gpre[i + 1], c->bufA, c->bufB, true);
    const long long per = (long long)16 * cl.Cb * cl.Cs;
    wgrad_call<T>(c, "gemm_wgrad", c->bufB, c->gact[i], c->dw4, per, cl.Cb, cl.Cs, cl.Hs, 16, 1, n);
    launch_dw4_to_dw3(c->dw4, G.g + cl.w, c->L, cl.Cb, cl.Cs, c->st, per, G.P);
    conv_call<T>(c, "gemm_down", MODE_DOWN, EPI_NONE, c->bufB, (const T*)G.w4d + cl.w4, G.P4, c->bufA, nullptr, cl.Cb, cl.Cs,
                 2 * cl.Hs, cl.Hs, 0, 1, n);
  }
  NormArgs na = norm_args<T>(c, G, G.C0, G.h0 * G.h0, G.fc_gamma, G.fc_beta, G.fc_rs, c->g_mean[0], c->g_var[0], c->g_rstd[0],
                             c->g_sums[0], 0, 1, n, 1.f);
  na.eps = f.bn_eps_first;
  bn_backward<T>(c, na, c->gpre[0], c->bufA, c->bufB, true);
  PointArgs a = point_args(c, c->bufB, G.J, G.J, 1, 0, 1, n);                 // ReLU derivative from the stored output
  a.saved = c->gpre[0]; a.slope = 0.f;
  { Scope s(c, "act_dropout_bwd", 0, 3.0 * n * G.J * sizeof(T)); launch_point_bwd<T>(a, c->st); }
  launch_col_sum<T>(a, G.g + G.fc_bias, G.P, c->st);
  wgrad_call<T>(c, "gemm_wgrad_dense", c->bufB, c->zin, G.g + G.fc_w, G.P, G.J, G.Kp, 1, 1, 1, n);
}

template <typename T>
void paper_adam_g(gan_ctx* c) {
  Net& G = c->G;
  AdamArgs a = {};
  a.theta = G.theta; a.m = G.m; a.v = G.v; a.g = G.g; a.shadow = c->bf16 ? G.shadow_u : nullptr; a.shadow_t = nullptr;
  a.P = G.P; a.L = c->L; a.counts = c->rb.counts; a.t = G.t; a.bc = G.bc;
  a.lr = c->cfg.lr; a.beta1 = c->cfg.beta1; a.beta2 = c->cfg.beta2; a.eps = c->cfg.adam_eps;
  {
    Scope s(c, "adam", 0, (double)c->L * G.P * (28.0 + (c->bf16 ? 2.0 : 0.0)));
    launch_adam<T>(a, c->st);
  }
  paper_rebuild_w4<T>(c);
}

// The planned update of one network: every convolution weight the GEMM engine also reads in "down" form is a tiled
// region (the update writes that transposed copy too), in layer order; the rest of the block is the gaps.
template <typename T>
AdamArgs adam_args(gan_ctx* c, Net& net, bool isG) {
  AdamArgs a = {};
  a.theta = net.theta; a.m = net.m; a.v = net.v; a.g = net.g; a.shadow = c->bf16 ? net.shadow_u : nullptr;
  a.P = net.P; a.L = c->L; a.counts = c->rb.counts; a.t = net.t; a.bc = net.bc;
  a.lr = c->cfg.lr; a.beta1 = c->cfg.beta1; a.beta2 = c->cfg.beta2; a.eps = c->cfg.adam_eps;
  a.shadow_t = net.shadow_d;
  for (size_t i = 0; i < net.conv.size(); ++i) {
    const bool gemm = isG ? (i + 1 < net.conv.size()) : (i > 0);
    if (!gemm) continue;
    a.reg_w[a.nregions] = net.conv[i].w; a.reg_cb[a.nregions] = net.conv[i].Cb; a.reg_cs[a.nregions] = net.conv[i].Cs;
    ++a.nregions;
  }
  adam_plan(a);
  return a;
}
// bytes one update moves per element: g, theta, m, v in; theta, m, v out; the storage-type copy
inline double adam_bytes_per_element(const gan_ctx* c) { return 28.0 + (c->bf16 ? 2.0 : 0.0); }
template <typename T>
void adam_region_call(gan_ctx* c, const AdamArgs& a, int region, hipStream_t st) {
  double elems = 0;
  for (int r = 0; r < a.nregions; ++r)
    if (region < 0 || r == region) elems += 16.0 * a.reg_cb[r] * a.reg_cs[r];
  Scope s(c, "adam", 0, (double)c->L * elems * (adam_bytes_per_element(c) + sizeof(T)), nullptr, st);
  launch_adam_region<T>(a, region, st);
}
// what is left of a planned update once the regions are done (or enqueued beside): the gaps, and the packed weights of
// the image-side layer, rebuilt from the new master weights
template <typename T>
void adam_rest_call(gan_ctx* c, Net& net, bool isG, const AdamArgs& a) {
  {
    double elems = 0;
    for (int r = 0; r < a.ngaps; ++r) elems += (double)(a.gap_hi[r] - a.gap_lo[r]);
    Scope s(c, "adam", 0, (double)c->L * elems * adam_bytes_per_element(c));
    launch_adam_gaps(a, c->st);
  }
  if (isG) launch_pack_w<T>(pack_args(c, net, net.conv.back(), c->KcG, 0, c->wpG), c->st);
  else launch_pack_w<T>(pack_args(c, net, net.conv.front(), c->KcD, c->nslot, c->wpD), c->st);
}
// the whole update on the caller's stream
template <typename T>
void adam_call(gan_ctx* c, Net& net, bool isG) {
  const AdamArgs a = adam_args<T>(c, net, isG);
  launch_adam_prepare(a, c->st);
  adam_region_call<T>(c, a, -1, c->st);
  adam_rest_call<T>(c, net, isG, a);
}

template <typename T>
void route_and_stage(gan_ctx* c, const int32_t* label_ids, const float* noise, const float* real, int n) {
  launch_route(label_ids, n, c->L, c->cfg.n_labels, c->geoms, c->rb, c->st);
  {
    Scope s(c, "stage", 0, (double)n * c->cfg.z_dim * (4.0 + sizeof(T)));
    launch_stage<T>(label_ids, noise, nullptr, n, c->L, c->cfg.z_dim, c->cfg.cond_g, c->G.Kp, c->cfg.img_c, c->cfg.img_hw, c->rb,
                    (T*)c->zin, (T*)c->xd, c->st);
  }
  if (real) im2col_call<T>(c, c->D.conv[0], nullptr, real, c->colD, c->KcD, c->nslot, 0, n);   // the real half of D's input
}

template <typename T>
void paper_train_step(gan_ctx* c, const int32_t* label_ids, const float* noise, const float* real, int n) {
  if (c->shadows_dirty) refresh_shadows(c);
  route_and_stage<T>(c, label_ids, noise, real, n);
  paper_g_forward<T>(c, n, false, true);                               // fake = G(z)
  im2col_call<T>(c, c->D.conv[0], c->xd, nullptr, c->colD, c->KcD, c->nslot, 1, n);
  paper_d_forward<T>(c, n, 0, 2, true, 0, 1);                          // D(real), D(fake): dropout passes 0 and 1
  loss_call(c, n, 0);                                                  // Eq. 3
  paper_d_backward<T>(c, n, 0, 2, true, false, 0, 1);
  adam_call<T>(c, c->D, false);
  paper_d_forward<T>(c, n, 1, 1, true, 2, 0);                          // updated D on the same fake batch: pass 2
  loss_call(c, n, 1);                                                  // Eq. 4 (negated: minimised)
  paper_d_backward<T>(c, n, 1, 1, false, true, 2, 0);
  paper_g_backward<T>(c, n);
  paper_adam_g<T>(c);
}

template <typename T>
void train_step(gan_ctx* c, const int32_t* label_ids, const float* noise, const float* real, int n) {
  if (c->paper) return paper_train_step<T>(c, label_ids, noise, real, n);
  if (c->shadows_dirty) refresh_shadows(c);
  route_and_stage<T>(c, label_ids, noise, real, n);
  g_forward<T>(c, n, false, true);                 // fake = G(z)
  im2col_call<T>(c, c->D.conv[0], c->xd, nullptr, c->colD, c->KcD, c->nslot, 1, n);   // the fake half of D's input
  d_forward<T>(c, n, 0, 2, true);                  // D(real), D(fake): separate batch statistics per segment
  loss_call(c, n, 0);                              // Eq. 3
  c->order_next = 0;
  {
    const AdamArgs aD = adam_args<T>(c, c->D, false);
    launch_adam_prepare(aD, c->st);
    d_backward<T>(c, n, 0, 2, true, false, &aD);   // weight gradients and the convolutions' updates beside the chain
    adam_rest_call<T>(c, c->D, false, aD);
    order_after(c, c->st, side_stream(c));
  }
  d_forward<T>(c, n, 1, 1, true);                  // updated D on the same fake batch
  loss_call(c, n, 1);                              // Eq. 4 (negated: minimised)
  d_backward<T>(c, n, 1, 1, false, true);          // only data gradients: theta_D is not G's to move
  {
    const AdamArgs aG = adam_args<T>(c, c->G, true);
    launch_adam_prepare(aG, c->st);
    g_backward<T>(c, n, &aG);
    adam_rest_call<T>(c, c->G, true, aG);
    order_after(c, c->st, side_stream(c));
  }
}

bool check_config_paper(const gan_config* f, std::string& why) {
  if (f->n_g < 2 || f->n_g > GAN_MAX_LAYERS || f->n_d < 2 || f->n_d > GAN_MAX_LAYERS) { why = "n_g, n_d must be in [2, 8]"; return false; }
  if (f->img_c < 1 || f->img_c > 4) { why = "img_c must be in [1, 4]"; return false; }
  if (f->cond_g != 0 || f->cond_d != 0) { why = "the networks of the tables are unconditional: cond_g = cond_d = 0"; return false; }
  if ((f->g_h0 << (f->n_g - 1)) != f->img_hw) { why = "img_hw must equal g_h0 * 2^(n_g - 1)"; return false; }
  if (((f->img_hw >> f->n_d) << f->n_d) != f->img_hw || (f->img_hw >> f->n_d) < 1) { why = "img_hw must be divisible by 2^n_d"; return false; }
  for (int i = 0; i < f->n_g; ++i) if (f->g_ch[i] <= 0 || f->g_ch[i] % 64 || f->g_ch[i] > 1024) { why = "g_ch must be multiples of 64, at most 1024"; return false; }
  for (int i = 0; i < f->n_d; ++i) if (f->d_ch[i] <= 0 || f->d_ch[i] > 1024) { why = "d_ch must be in [1, 1024]"; return false; }
  if (f->g_ch[f->n_g - 1] != 64 && f->g_ch[f->n_g - 1] != 128) { why = "the last generator block must have 64 or 128 channels"; return false; }
  if (f->d_ch[0] > 128) { why = "the first discriminator block supports at most 128 channels"; return false; }
  if ((f->g_ch[0] * f->g_h0 * f->g_h0) % 128) { why = "g_ch[0]*g_h0^2 must be a multiple of 128"; return false; }
  if (f->z_dim < 1 || f->max_total_batch < 1) { why = "bad z_dim / max_total_batch"; return false; }
  if (!(f->dropout_p >= 0.f && f->dropout_p < 1.f) || !(f->bn_eps_first > 0.f) || !(f->bn_eps > 0.f)) { why = "bad dropout_p / epsilon"; return false; }
  return true;
}

bool check_config(const gan_config* f, std::string& why) {
  if (f->n_models < 1 || f->n_labels < 1) { why = "n_models and n_labels must be positive"; return false; }
  if (f->n_models != 1 && f->n_models != f->n_labels) { why = "n_models must be 1 or n_labels"; return false; }
  if (f->precision != GAN_FP32 && f->precision != GAN_BF16_FP32MASTER) { why = "unknown precision"; return false; }
  if (f->family == GAN_FAMILY_PAPER) return check_config_paper(f, why);
  if (f->family != GAN_FAMILY_STRIDED) { why = "unknown network family"; return false; }
  if (f->n_g < 2 || f->n_g > GAN_MAX_LAYERS || f->n_d < 2 || f->n_d > GAN_MAX_LAYERS) { why = "n_g, n_d must be in [2, 8]"; return false; }
  if (f->img_c < 1 || f->img_c > 4) { why = "img_c must be in [1, 4]"; return false; }
  if ((f->g_h0 << f->n_g) != f->img_hw) { why = "img_hw must equal g_h0 * 2^n_g"; return false; }
  if (((f->img_hw >> f->n_d) << f->n_d) != f->img_hw || (f->img_hw >> f->n_d) < 1) { why = "img_hw must be divisible by 2^n_d"; return false; }
  for (int i = 0; i < f->n_g; ++i) if (f->g_ch[i] <= 0 || f->g_ch[i] % 64) { why = "g_ch must be multiples of 64"; return false; }
  for (int i = 0; i < f->n_d; ++i) if (f->d_ch[i] <= 0 || f->d_ch[i] % 64) { why = "d_ch must be multiples of 64"; return false; }
  for (int i = 0; i < f->n_g; ++i) if (f->g_ch[i] > 1024) { why = "at most 1024 channels per layer"; return false; }
  for (int i = 0; i < f->n_d; ++i) if (f->d_ch[i] > 1024) { why = "at most 1024 channels per layer"; return false; }
  if (f->g_ch[f->n_g - 1] > 128 || f->d_ch[0] > 128) { why = "the layers next to the image support 64 or 128 feature channels"; return false; }
  if ((f->g_ch[0] * f->g_h0 * f->g_h0) % 128) { why = "g_ch[0]*g_h0^2 must be a multiple of 128"; return false; }
  if (f->z_dim < 1 || f->cond_g < 0 || f->cond_d < 0 || f->max_total_batch < 1) { why = "bad z_dim / cond / max_total_batch"; return false; }
  if (f->cond_g > f->n_labels || (f->cond_d != 0 && f->cond_d < f->n_labels)) { why = "cond_d must cover every label"; return false; }
  if (f->precision != GAN_FP32 && f->precision != GAN_BF16_FP32MASTER) { why = "unknown precision"; return false; }
  return true;
}

}  // namespace

// ---------------------------------------------------------------------------------------------------------
extern "C" {

gan_status gan_create(const gan_config* cfg, void* hip_stream, gan_ctx** out) {
  if (!cfg || !out || cfg->struct_size != sizeof(gan_config)) return GAN_E_ARG;
  std::string why;
  if (!check_config(cfg, why)) return GAN_E_SHAPE;
  gan_ctx* c = new gan_ctx();
  c->cfg = *cfg;
  c->st = (hipStream_t)hip_stream;
  c->bf16 = cfg->precision == GAN_BF16_FP32MASTER;
  c->L = cfg->n_models; c->NB = cfg->max_total_batch;
  c->nslot = (cfg->cond_d > 0 && c->L == 1) ? cfg->cond_d : 1;
  c->geoms.n = 0;
  c->paper = cfg->family == GAN_FAMILY_PAPER;
  if (c->paper) build_layout_paper(c); else build_layout(c);
  const int L = c->L, NB = c->NB;
  const size_t es = esize(c);
  bool ok = alloc_net(c, c->G) && alloc_net(c, c->D);
  // geometries used by any launch: (rows per sample, tile height) of every GEMM's row space
  {
    auto reg = [&](int rps, int tile_rows) { if (geom_id(c, rps, tile_rows) < 0) ok = false; };
    const ConvLayer& gl = c->G.conv.back();
    const ConvLayer& d1 = c->D.conv.front();
    reg(1, layer_tile_rows(c, c->G.J, 1));                                      // G's linear layer
    for (size_t i = 0; i + 1 < c->G.conv.size(); ++i) {
      const ConvLayer& cl = c->G.conv[i];
      reg(cl.Hs * cl.Hs, layer_tile_rows(c, cl.Cb, cl.Hs * cl.Hs));             // forward (up)
      reg(cl.Hs * cl.Hs, layer_tile_rows(c, cl.Cs, cl.Hs * cl.Hs));             // data gradient (down)
    }
    reg(gl.Hs * gl.Hs, layer_tile_rows(c, gl.Cs, gl.Hs * gl.Hs));               // its data gradient (patch GEMM)
    for (size_t j = 1; j < c->D.conv.size(); ++j) {
      const ConvLayer& cl = c->D.conv[j];
      reg(cl.Hs * cl.Hs, layer_tile_rows(c, cl.Cs, cl.Hs * cl.Hs));             // forward (down)
      reg(cl.Hs * cl.Hs, layer_tile_rows(c, cl.Cb, cl.Hs * cl.Hs));             // data gradient (up)
    }
    reg(d1.Hs * d1.Hs, layer_tile_rows(c, d1.Cs, d1.Hs * d1.Hs));               // first conv (patch GEMM)
    // row space of every BatchNorm, in blocks of BN_RED_ROWS rows (backward reduction)
    reg(c->G.h0 * c->G.h0, BN_RED_ROWS);
    for (size_t i = 0; i + 1 < c->G.conv.size(); ++i) reg(4 * c->G.conv[i].Hs * c->G.conv[i].Hs, BN_RED_ROWS);
    for (size_t j = 1; j < c->D.conv.size(); ++j) reg(c->D.conv[j].Hs * c->D.conv[j].Hs, BN_RED_ROWS);
  }
  // two sets of routing buffers: the training step's (what gan_get_losses / gan_get_routing report) and one for
  // gan_generate / gan_sample, so that generating between a step and its queries changes nothing they return
  RouteBuffers& rb = c->rb;
  for (RouteBuffers* r : {&c->rb, &c->rb_gen}) {
    ok = ok && dev_alloc(c, (void**)&r->cnt, (size_t)ROUTE_CHUNKS * L * 4) && dev_alloc(c, (void**)&r->counts, (size_t)L * 4) &&
         dev_alloc(c, (void**)&r->offs, (size_t)(L + 1) * 4) && dev_alloc(c, (void**)&r->perm, (size_t)NB * 4) &&
         dev_alloc(c, (void**)&r->sample_model, (size_t)NB * 4) && dev_alloc(c, (void**)&r->sample_slot, (size_t)NB * 4) &&
         dev_alloc(c, (void**)&r->tpre, (size_t)MAX_GEOMS * (L + 1) * 4) && dev_alloc(c, (void**)&r->order, (size_t)L * 4);
    int mx = 1;
    for (int g = 0; g < c->geoms.n; ++g) mx = std::max(mx, ub_tiles(c, NB, c->geoms.rps[g], c->geoms.tile_rows[g]));
    r->tmodel_stride = mx;
    ok = ok && dev_alloc(c, (void**)&r->tmodel, (size_t)c->geoms.n * mx * 4);
  }
  ok = ok && dev_alloc(c, (void**)&rb.flags, 16);
  c->rb_gen.flags = rb.flags;                  // one sticky out-of-range flag for both
  const long long img_elems = (long long)cfg->img_hw * cfg->img_hw * cfg->img_c;
  long long max_act = img_elems;
  ok = ok && dev_alloc(c, &c->zin, (size_t)NB * c->G.Kp * es) && dev_alloc(c, &c->xd, (size_t)2 * NB * img_elems * es) &&
       dev_alloc(c, &c->dimg, (size_t)2 * NB * img_elems * es);
  // G activations (one segment)
  {
    const int nl = (int)c->G.conv.size();
    c->gpre.resize(nl); c->gact.resize(nl); c->g_mean.resize(nl); c->g_var.resize(nl); c->g_rstd.resize(nl); c->g_sums.resize(nl);
    for (int i = 0; i < nl && ok; ++i) {
      const long long e = i == 0 ? c->G.J : (long long)4 * c->G.conv[i - 1].Hs * c->G.conv[i - 1].Hs * c->G.conv[i - 1].Cb;
      const int C = i == 0 ? c->G.C0 : c->G.conv[i - 1].Cb;
      max_act = e > max_act ? e : max_act;
      ok = dev_alloc(c, &c->gpre[i], (size_t)NB * e * es) && dev_alloc(c, &c->gact[i], (size_t)NB * e * es) &&
           dev_alloc(c, (void**)&c->g_mean[i], (size_t)2 * L * C * 4) && dev_alloc(c, (void**)&c->g_var[i], (size_t)2 * L * C * 4) &&
           dev_alloc(c, (void**)&c->g_rstd[i], (size_t)2 * L * C * 4) && dev_alloc(c, (void**)&c->g_sums[i], (size_t)4 * L * C * 4);
    }
  }
  // D activations (two segments: real, fake)
  {
    const int nl = (int)c->D.conv.size();
    c->dpre.assign(nl, nullptr); c->dact.assign(nl, nullptr);
    c->d_mean.assign(nl, nullptr); c->d_var.assign(nl, nullptr); c->d_rstd.assign(nl, nullptr); c->d_sums.assign(nl, nullptr);
    for (int j = 0; j < nl && ok; ++j) {
      const ConvLayer& cl = c->D.conv[j];
      const long long e = (long long)cl.Hs * cl.Hs * cl.Cs;
      max_act = e > max_act ? e : max_act;
      ok = dev_alloc(c, &c->dact[j], (size_t)2 * NB * e * es);
      if (j > 0)
        ok = ok && dev_alloc(c, &c->dpre[j], (size_t)2 * NB * e * es) && dev_alloc(c, (void**)&c->d_mean[j], (size_t)2 * L * cl.Cs * 4) &&
             dev_alloc(c, (void**)&c->d_var[j], (size_t)2 * L * cl.Cs * 4) && dev_alloc(c, (void**)&c->d_rstd[j], (size_t)2 * L * cl.Cs * 4) &&
             dev_alloc(c, (void**)&c->d_sums[j], (size_t)4 * L * cl.Cs * 4);
    }
  }
  {
    // column sums left by the GEMM in front of every BatchNorm: phases x segments x tiles x sub-tiles (at most 4) x columns x 2
    size_t mx = (size_t)4 * ub_tiles(c, NB, 1, layer_tile_rows(c, c->G.J, 1)) * c->G.J;
    for (size_t i = 0; i + 1 < c->G.conv.size(); ++i) {
      const ConvLayer& cl = c->G.conv[i];
      const size_t v = (size_t)4 * 4 * ub_tiles(c, NB, cl.Hs * cl.Hs, layer_tile_rows(c, cl.Cb, cl.Hs * cl.Hs)) * cl.Cb;
      mx = v > mx ? v : mx;
    }
    for (size_t j = 1; j < c->D.conv.size(); ++j) {
      const ConvLayer& cl = c->D.conv[j];
      const size_t v = (size_t)4 * 2 * ub_tiles(c, NB, cl.Hs * cl.Hs, layer_tile_rows(c, cl.Cs, cl.Hs * cl.Hs)) * cl.Cs;
      mx = v > mx ? v : mx;
    }
    // and the BatchNorm backward reduction: segments x row blocks x channels x 2
    {
      size_t v = (size_t)ub_tiles(c, NB, c->G.h0 * c->G.h0, BN_RED_ROWS) * c->G.C0;
      mx = v > mx ? v : mx;
      for (size_t i = 0; i + 1 < c->G.conv.size(); ++i) {
        const ConvLayer& cl = c->G.conv[i];
        v = (size_t)ub_tiles(c, NB, 4 * cl.Hs * cl.Hs, BN_RED_ROWS) * cl.Cb;
        mx = v > mx ? v : mx;
      }
      for (size_t j = 1; j < c->D.conv.size(); ++j) {
        const ConvLayer& cl = c->D.conv[j];
        v = (size_t)2 * ub_tiles(c, NB, cl.Hs * cl.Hs, BN_RED_ROWS) * cl.Cs;
        mx = v > mx ? v : mx;
      }
    }
    ok = ok && dev_alloc(c, (void**)&c->stat_partial, mx * 2 * 4);
  }
  ok = ok && dev_alloc(c, &c->bufA, (size_t)2 * NB * max_act * es) && dev_alloc(c, &c->bufB, (size_t)2 * NB * max_act * es) &&
       dev_alloc(c, (void**)&c->logits, (size_t)2 * NB * 4) && dev_alloc(c, (void**)&c->dlogits, (size_t)2 * NB * 4) &&
       dev_alloc(c, (void**)&c->loss_d, (size_t)L * 4) && dev_alloc(c, (void**)&c->loss_g, (size_t)L * 4);
  {
    const ConvLayer& c1 = c->D.conv[0];
    const ConvLayer& gl = c->G.conv.back();
    c->img_ksplit = img_ksplit_for(L);
    c->KcD = (int)round_up(16 * c1.Cb + 9 * c->nslot + 1, 64);
    c->KcG = (int)round_up(16 * gl.Cb, 64);
    const size_t d1 = (size_t)c->KcD * c1.Cs, g1 = (size_t)c->KcG * gl.Cs;
    ok = ok && dev_alloc(c, &c->colD, (size_t)2 * NB * c1.Hs * c1.Hs * c->KcD * es) &&
         dev_alloc(c, &c->colG, c->paper ? 16 : (size_t)NB * gl.Hs * gl.Hs * c->KcG * es) && dev_alloc(c, &c->wpD, (size_t)L * d1 * es) &&
         dev_alloc(c, &c->wpG, (size_t)L * g1 * es) && dev_alloc(c, (void**)&c->dwp, (size_t)c->img_ksplit * L * (d1 > g1 ? d1 : g1) * 4) &&
         dev_alloc(c, (void**)&c->bias_partial, (size_t)L * img_bias_chunks(L) * 4 * 4);
  }
  {
    // partial blocks of the weight gradients that are split over rows (few models only)
    size_t need = 0;
    auto want = [&](int Cb, int Cs, int ntaps) {
      const int ks = wgrad_ksplit(c, Cb, Cs, ntaps);
      if (ks > 1) need = std::max(need, (size_t)ks * L * ntaps * Cb * Cs * 4);
    };
    for (size_t j = 1; j < c->D.conv.size(); ++j) want(c->D.conv[j].Cb, c->D.conv[j].Cs, 16);
    for (size_t i = 0; i + 1 < c->G.conv.size(); ++i) want(c->G.conv[i].Cb, c->G.conv[i].Cs, 16);
    want(c->G.J, c->G.Kp, 1);
    c->wg_part = nullptr;
    if (need) ok = ok && dev_alloc(c, (void**)&c->wg_part, need);
    if (c->paper) {
      // G's summed-tap k4 weights (both layouts), the k4 weight gradient of one block, the last conv's row-split partials
      size_t per = 0;
      for (size_t i = 0; i + 1 < c->G.conv.size(); ++i) per = std::max(per, (size_t)16 * c->G.conv[i].Cb * c->G.conv[i].Cs);
      const ConvLayer& last = c->G.conv.back();
      ok = ok && dev_alloc(c, &c->G.w4u, (size_t)L * c->G.P4 * es) && dev_alloc(c, &c->G.w4d, (size_t)L * c->G.P4 * es) &&
           dev_alloc(c, (void**)&c->dw4, (size_t)L * per * 4) &&
           dev_alloc(c, (void**)&c->c3_part, (size_t)conv3_wgrad_splits(L) * L * 9 * last.Cb * last.Cs * 4);
    }
    // the linear head's weight gradient: blocks of 1024 columns per model, rows split when that leaves the chip idle
    c->head_rsplit = (int)std::min<long long>(std::max<long long>(512 / ((long long)L * ((c->D.K + 1023) / 1024)), 1), 64);
    if (c->head_rsplit > 1) ok = ok && dev_alloc(c, (void**)&c->head_part, (size_t)c->head_rsplit * L * (c->D.K + 4) * 4);
  }
  {
    // the GEMM loaders address one segment of any activation tensor or patch matrix with 32-bit byte offsets
    const ConvLayer& c1 = c->D.conv[0];
    const ConvLayer& gl = c->G.conv.back();
    const long long lim = 1LL << 31;
    const long long big = std::max({(long long)NB * max_act * (long long)es, (long long)NB * c1.Hs * c1.Hs * c->KcD * (long long)es,
                                    c->paper ? 0LL : (long long)NB * gl.Hs * gl.Hs * c->KcG * (long long)es});
    if (big >= lim) {
      for (void* p : c->allocs) (void)hipFree(p);
      delete c;
      return GAN_E_SHAPE;
    }
  }
  if (!ok) {
    for (void* p : c->allocs) (void)hipFree(p);
    delete c;
    return GAN_E_OOM;
  }
  hipMemsetAsync(rb.flags, 0, 16, c->st);
  hipMemsetAsync(rb.counts, 0, (size_t)L * 4, c->st);
  hipMemsetAsync(rb.offs, 0, (size_t)(L + 1) * 4, c->st);
  hipMemsetAsync(c->loss_d, 0, (size_t)L * 4, c->st);
  hipMemsetAsync(c->loss_g, 0, (size_t)L * 4, c->st);
  bool init_ok = true;
  if (c->paper) { hipStreamSynchronize(c->st); init_ok = builtin_init_paper(c); }
  else builtin_init(c);
  if (!init_ok || hipStreamSynchronize(c->st) != hipSuccess || hipGetLastError() != hipSuccess) {
    for (void* p : c->allocs) (void)hipFree(p);
    delete c;
    return GAN_E_HIP;
  }
  if (hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking) != hipSuccess) {
    (void)hipGetLastError();
    c->side = nullptr;                         // everything then runs on the caller's stream
  }
  if (hipStreamCreateWithFlags(&c->cap, hipStreamNonBlocking) != hipSuccess) {
    (void)hipGetLastError();
    c->cap = nullptr;                          // no replayable steps
  }
  c->shadows_dirty = true;
  *out = c;
  return GAN_OK;
}

gan_status gan_destroy(gan_ctx* c) {
  if (!c) return GAN_E_ARG;
  (void)hipStreamSynchronize(c->st);
  if (c->side) { (void)hipStreamSynchronize(c->side); (void)hipStreamDestroy(c->side); }
  for (auto& g : c->graphs) (void)hipGraphExecDestroy(g.exec);
  if (c->cap) (void)hipStreamDestroy(c->cap);
  for (auto& e : c->order_events) hipEventDestroy(e);
  for (auto& e : c->prof_entries) { hipEventDestroy(e.e0); hipEventDestroy(e.e1); }
  for (auto& e : c->event_pool) hipEventDestroy(e);
  for (void* p : c->allocs) (void)hipFree(p);
  delete c;
  return GAN_OK;
}

const char* gan_last_error(const gan_ctx* c) { return c ? c->err.c_str() : "null context"; }

gan_status gan_train_step(gan_ctx* c, const int32_t* label_ids, const float* noise, const float* real_batch, int32_t n) {
  if (!c) return GAN_E_ARG;
  if (n < 0 || n > c->NB) return fail(c, GAN_E_ARG, "n out of range [0, max_total_batch]");
  if (n > 0 && (!label_ids || !noise || !real_batch)) return fail(c, GAN_E_ARG, "null input pointer");
  c->last_n = n;
  if (n == 0) {
    hipMemsetAsync(c->rb.counts, 0, (size_t)c->L * 4, c->st);
    hipMemsetAsync(c->rb.offs, 0, (size_t)(c->L + 1) * 4, c->st);
    hipMemsetAsync(c->loss_d, 0, (size_t)c->L * 4, c->st);
    hipMemsetAsync(c->loss_g, 0, (size_t)c->L * 4, c->st);
    return GAN_OK;
  }
  (void)take_launch_error();
  ++c->calls;
  if (c->graphs_on && c->cap && !c->prof) {
    if (c->shadows_dirty) refresh_shadows(c);          // host-side condition: outside anything that is replayed
    gan_ctx::StepGraph* hit = nullptr;
    for (auto& g : c->graphs)
      if (g.lab == label_ids && g.noise == noise && g.real == real_batch && g.n == n) hit = &g;
    bool repeat = false;
    for (auto& a : c->seen) repeat = repeat || (a.lab == label_ids && a.noise == noise && a.real == real_batch && a.n == n);
    if (!hit && !repeat) {
      if (c->seen.size() >= 8) c->seen.erase(c->seen.begin());
      c->seen.push_back({label_ids, noise, real_batch, n});
    }
    if (!hit && repeat) {
      // capture this step's launches (both streams: the second one joins through the ordering events) without running them
      hipStream_t user = c->st;
      hipGraph_t graph = nullptr;
      hipGraphExec_t exec = nullptr;
      bool ok = hipStreamBeginCapture(c->cap, hipStreamCaptureModeRelaxed) == hipSuccess;
      if (ok) {
        c->st = c->cap;
        if (c->bf16) train_step<bf16_t>(c, label_ids, noise, real_batch, n);
        else train_step<float>(c, label_ids, noise, real_batch, n);
        c->st = user;
        ok = hipStreamEndCapture(c->cap, &graph) == hipSuccess && graph != nullptr;
      }
      const char* refused = take_launch_error();
      if (refused) {
        if (graph) (void)hipGraphDestroy(graph);
        (void)hipGetLastError();
        return fail(c, GAN_E_SHAPE, refused);
      }
      ok = ok && hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0) == hipSuccess;
      if (graph) (void)hipGraphDestroy(graph);
      if (ok) {
        if (c->graphs.size() >= 8) {                    // keep the eight most recently used
          size_t oldest = 0;
          for (size_t i = 1; i < c->graphs.size(); ++i)
            if (c->graphs[i].used < c->graphs[oldest].used) oldest = i;
          (void)hipGraphExecDestroy(c->graphs[oldest].exec);
          c->graphs.erase(c->graphs.begin() + oldest);
        }
        c->graphs.push_back({label_ids, noise, real_batch, n, exec, c->calls});
        hit = &c->graphs.back();
      } else {
        (void)hipGetLastError();
        c->graphs_on = false;                           // capture is not available here: plain launches from now on
      }
    }
    if (hit) {
      hit->used = c->calls;
      ++c->replays;
      if (hipGraphLaunch(hit->exec, c->st) != hipSuccess) return fail(c, GAN_E_HIP, "graph launch failed");
      return launch_status(c);
    }
  }
  if (c->bf16) train_step<bf16_t>(c, label_ids, noise, real_batch, n);
  else train_step<float>(c, label_ids, noise, real_batch, n);
  return launch_status(c);
}

gan_status gan_use_second_stream(gan_ctx* c, int32_t enable) {
  if (!c) return GAN_E_ARG;
  if (hipStreamSynchronize(c->st) != hipSuccess) return fail(c, GAN_E_HIP, "stream synchronisation failed");
  c->side_on = enable != 0 && c->side != nullptr;
  for (auto& g : c->graphs) (void)hipGraphExecDestroy(g.exec);      // captured with the other setting
  c->graphs.clear();
  c->seen.clear();
  return GAN_OK;
}

gan_status gan_graph_replays(const gan_ctx* c, int64_t* n) {
  if (!c || !n) return GAN_E_ARG;
  *n = (int64_t)c->replays;
  return GAN_OK;
}

gan_status gan_use_graphs(gan_ctx* c, int32_t enable) {
  if (!c) return GAN_E_ARG;
  c->graphs_on = enable != 0 && c->cap != nullptr;
  c->seen.clear();
  return GAN_OK;
}

gan_status gan_generate(gan_ctx* c, const int32_t* label_ids, const float* noise, int32_t n, float* out_images,
                        int32_t use_running_stats) {
  if (!c) return GAN_E_ARG;
  if (n < 0 || n > c->NB) return fail(c, GAN_E_ARG, "n out of range [0, max_total_batch]");
  if (n == 0) return GAN_OK;
  if (!label_ids || !noise || !out_images) return fail(c, GAN_E_ARG, "null pointer");
  if (c->shadows_dirty) refresh_shadows(c);
  (void)take_launch_error();
  const gan_config& f = c->cfg;
  const RouteBuffers train_rb = c->rb;         // the launch helpers read c->rb: point them at the generate set
  c->rb = c->rb_gen;
  if (c->bf16) {
    route_and_stage<bf16_t>(c, label_ids, noise, nullptr, n);
    if (c->paper) paper_g_forward<bf16_t>(c, n, use_running_stats != 0, false); else
    g_forward<bf16_t>(c, n, use_running_stats != 0, false);
    launch_unstage<bf16_t>((const bf16_t*)c->xd + (long long)n * f.img_hw * f.img_hw * f.img_c, out_images, n, c->L, f.img_c,
                           f.img_hw, c->rb, c->st);
  } else {
    route_and_stage<float>(c, label_ids, noise, nullptr, n);
    if (c->paper) paper_g_forward<float>(c, n, use_running_stats != 0, false); else
    g_forward<float>(c, n, use_running_stats != 0, false);
    launch_unstage<float>((const float*)c->xd + (long long)n * f.img_hw * f.img_hw * f.img_c, out_images, n, c->L, f.img_c,
                          f.img_hw, c->rb, c->st);
  }
  c->rb = train_rb;
  return launch_status(c);
}

gan_status gan_sample(gan_ctx* c, const double* prior, const float* u, const float* noise, int32_t n, float* out_images,
                      int32_t* out_labels, int32_t use_running_stats) {
  if (!c) return GAN_E_ARG;
  if (n < 0 || n > c->NB) return fail(c, GAN_E_ARG, "n out of range [0, max_total_batch]");
  if (!prior) return fail(c, GAN_E_ARG, "null prior");
  const int K = c->cfg.n_labels;
  double total = 0.0;
  int last = -1;
  for (int k = 0; k < K; ++k) {
    if (!(prior[k] >= 0.0)) return fail(c, GAN_E_ARG, "negative (or NaN) prior entry");
    total += prior[k];
    if (prior[k] > 0.0) last = k;
  }
  if (!(total > 0.0)) return fail(c, GAN_E_ARG, "the prior sums to zero");
  if (n == 0) return GAN_OK;
  if (!u || !noise || !out_images || !out_labels) return fail(c, GAN_E_ARG, "null pointer");
  std::vector<double> cdf((size_t)K);
  double cum = 0.0;
  for (int k = 0; k < K; ++k) { cum += prior[k] / total; cdf[(size_t)k] = cum; }
  if (!c->cdf && !dev_alloc(c, (void**)&c->cdf, (size_t)K * sizeof(double))) return fail(c, GAN_E_OOM, "cumulative prior");
  if (hipStreamSynchronize(c->st) != hipSuccess ||      // an earlier call may still read the buffer
      hipMemcpy(c->cdf, cdf.data(), (size_t)K * sizeof(double), hipMemcpyHostToDevice) != hipSuccess)
    return fail(c, GAN_E_HIP, "copy of the cumulative prior failed");
  launch_draw_labels(u, c->cdf, K, last, n, out_labels, c->st);
  return gan_generate(c, out_labels, noise, n, out_images, use_running_stats);
}

gan_status gan_anova_f(gan_ctx* c, const int32_t* label_ids, const float* images, int32_t n, double* F) {
  if (!c || !F) return GAN_E_ARG;
  if (n < 0 || n > c->NB) return fail(c, GAN_E_ARG, "n out of range [0, max_total_batch]");
  const gan_config& f = c->cfg;
  const int K = f.n_labels, C = f.img_c, HW = f.img_hw * f.img_hw;
  for (int ch = 0; ch < C; ++ch) F[ch] = 0.0;
  if (n == 0) return fail(c, GAN_E_STATE, "no images");
  if (!label_ids || !images) return fail(c, GAN_E_ARG, "null pointer");
  if (!c->an_x) {
    if (!dev_alloc(c, (void**)&c->an_x, (size_t)c->NB * C * sizeof(double)) ||
        !dev_alloc(c, (void**)&c->an_gsum, (size_t)K * C * sizeof(double)) ||
        !dev_alloc(c, (void**)&c->an_ssw, (size_t)K * C * sizeof(double)) || !dev_alloc(c, (void**)&c->an_gcnt, (size_t)K * sizeof(int)))
      return fail(c, GAN_E_OOM, "analysis-of-variance buffers");
  }
  launch_anova(label_ids, images, n, K, C, HW, c->an_x, c->an_gsum, c->an_gcnt, c->an_ssw, c->st);
  std::vector<double> gsum((size_t)K * C), ssw((size_t)K * C);
  std::vector<int> gcnt((size_t)K);
  if (hipStreamSynchronize(c->st) != hipSuccess ||
      hipMemcpy(gsum.data(), c->an_gsum, gsum.size() * sizeof(double), hipMemcpyDeviceToHost) != hipSuccess ||
      hipMemcpy(ssw.data(), c->an_ssw, ssw.size() * sizeof(double), hipMemcpyDeviceToHost) != hipSuccess ||
      hipMemcpy(gcnt.data(), c->an_gcnt, gcnt.size() * sizeof(int), hipMemcpyDeviceToHost) != hipSuccess)
    return fail(c, GAN_E_HIP, "analysis of variance failed on the device");
  if (!anova_f_from_sums(gsum.data(), ssw.data(), gcnt.data(), K, C, F))
    return fail(c, GAN_E_STATE, "fewer than two labels present, or not more images than labels");
  return GAN_OK;
}

static gan_status sync(gan_ctx* c) {
  const hipError_t e = hipStreamSynchronize(c->st);
  if (e != hipSuccess) return fail(c, GAN_E_HIP, std::string("stream failed: ") + hipGetErrorString(e));
  return GAN_OK;
}

gan_status gan_get_losses(gan_ctx* c, float* d_loss, float* g_loss, int32_t* counts) {
  if (!c) return GAN_E_ARG;
  gan_status s = sync(c);
  if (s != GAN_OK) return s;
  if (d_loss) hipMemcpy(d_loss, c->loss_d, (size_t)c->L * 4, hipMemcpyDeviceToHost);
  if (g_loss) hipMemcpy(g_loss, c->loss_g, (size_t)c->L * 4, hipMemcpyDeviceToHost);
  if (counts) hipMemcpy(counts, c->rb.counts, (size_t)c->L * 4, hipMemcpyDeviceToHost);
  int flag = 0;
  hipMemcpy(&flag, c->rb.flags, 4, hipMemcpyDeviceToHost);
  if (flag) {
    hipMemset(c->rb.flags, 0, 4);
    return fail(c, GAN_E_LABEL, "a label id outside [0, n_labels) was dropped");
  }
  return GAN_OK;
}

gan_status gan_param_count(const gan_ctx* c, int32_t which, int64_t* per_model) {
  if (!c || !per_model || which < 0 || which > 1) return GAN_E_ARG;
  *per_model = which == 0 ? c->G.Pext : c->D.Pext;
  return GAN_OK;
}
gan_status gan_bn_count(const gan_ctx* c, int32_t which, int64_t* per_model) {
  if (!c || !per_model || which < 0 || which > 1) return GAN_E_ARG;
  const Net& net = which == 0 ? c->G : c->D;
  *per_model = net.bn_ext2int.empty() ? net.nbn : (long long)net.bn_ext2int.size();
  return GAN_OK;
}

static gan_status read_block(gan_ctx* c, int which, int model, const float* dev_base, float* dst, int64_t n) {
  if (!c || !dst || which < 0 || which > 1 || model < 0 || model >= c->L) return GAN_E_ARG;
  Net& net = which == 0 ? c->G : c->D;
  if (n != net.Pext) return fail(c, GAN_E_ARG, "wrong element count");
  gan_status s = sync(c);
  if (s != GAN_OK) return s;
  std::vector<float> tmp((size_t)net.P);
  if (hipMemcpy(tmp.data(), dev_base + (long long)model * net.P, (size_t)net.P * 4, hipMemcpyDeviceToHost) != hipSuccess)
    return fail(c, GAN_E_HIP, "copy failed");
  for (long long i = 0; i < net.Pext; ++i) dst[i] = tmp[(size_t)net.ext2int[(size_t)i]];
  return GAN_OK;
}

gan_status gan_get_params(gan_ctx* c, int32_t which, int32_t model, float* dst, int64_t n) {
  if (!c || which < 0 || which > 1) return GAN_E_ARG;
  return read_block(c, which, model, (which == 0 ? c->G : c->D).theta, dst, n);
}
gan_status gan_get_grads(gan_ctx* c, int32_t which, int32_t model, float* dst, int64_t n) {
  if (!c || which < 0 || which > 1) return GAN_E_ARG;
  return read_block(c, which, model, (which == 0 ? c->G : c->D).g, dst, n);
}
gan_status gan_get_opt_state(gan_ctx* c, int32_t which, int32_t model, float* m, float* v, int64_t* t) {
  if (!c || which < 0 || which > 1 || model < 0 || model >= c->L) return GAN_E_ARG;
  Net& net = which == 0 ? c->G : c->D;
  gan_status s = GAN_OK;
  if (m) s = read_block(c, which, model, net.m, m, net.Pext);
  if (s == GAN_OK && v) s = read_block(c, which, model, net.v, v, net.Pext);
  if (s == GAN_OK && t) {
    s = sync(c);
    int tt = 0;
    hipMemcpy(&tt, net.t + model, 4, hipMemcpyDeviceToHost);
    *t = tt;
  }
  return s;
}

gan_status gan_set_params(gan_ctx* c, int32_t which, int32_t model, const float* src, int64_t n) {
  if (!c || !src || which < 0 || which > 1 || model < 0 || model >= c->L) return GAN_E_ARG;
  Net& net = which == 0 ? c->G : c->D;
  if (n != net.Pext) return fail(c, GAN_E_ARG, "wrong element count");
  gan_status s = sync(c);
  if (s != GAN_OK) return s;
  std::vector<float> tmp((size_t)net.P, 0.f);
  for (long long i = 0; i < net.Pext; ++i) tmp[(size_t)net.ext2int[(size_t)i]] = src[i];
  if (hipMemcpy(net.theta + (long long)model * net.P, tmp.data(), (size_t)net.P * 4, hipMemcpyHostToDevice) != hipSuccess)
    return fail(c, GAN_E_HIP, "copy failed");
  c->shadows_dirty = true;
  return GAN_OK;
}

static gan_status write_block(gan_ctx* c, Net& net, int model, float* dev_base, const float* src) {
  std::vector<float> tmp((size_t)net.P, 0.f);
  for (long long i = 0; i < net.Pext; ++i) tmp[(size_t)net.ext2int[(size_t)i]] = src[i];
  if (hipMemcpy(dev_base + (long long)model * net.P, tmp.data(), (size_t)net.P * 4, hipMemcpyHostToDevice) != hipSuccess)
    return fail(c, GAN_E_HIP, "copy failed");
  return GAN_OK;
}

gan_status gan_set_opt_state(gan_ctx* c, int32_t which, int32_t model, const float* m, const float* v, int64_t t) {
  if (!c || which < 0 || which > 1 || model < 0 || model >= c->L || t < 0 || t > 0x7fffffff) return GAN_E_ARG;
  Net& net = which == 0 ? c->G : c->D;
  gan_status s = sync(c);
  if (s == GAN_OK && m) s = write_block(c, net, model, net.m, m);
  if (s == GAN_OK && v) s = write_block(c, net, model, net.v, v);
  if (s == GAN_OK) {
    const int tt = (int)t;
    if (hipMemcpy(net.t + model, &tt, 4, hipMemcpyHostToDevice) != hipSuccess) return fail(c, GAN_E_HIP, "copy failed");
  }
  return s;
}

static long long bn_ext_count(const Net& net) { return net.bn_ext2int.empty() ? net.nbn : (long long)net.bn_ext2int.size(); }

gan_status gan_set_bn_running(gan_ctx* c, int32_t which, int32_t model, const float* mean, const float* var, int64_t n) {
  if (!c || !mean || !var || which < 0 || which > 1 || model < 0 || model >= c->L) return GAN_E_ARG;
  Net& net = which == 0 ? c->G : c->D;
  if (n != bn_ext_count(net)) return fail(c, GAN_E_ARG, "wrong element count");
  gan_status s = sync(c);
  if (s != GAN_OK) return s;
  std::vector<float> m((size_t)net.nbn, 0.f), v((size_t)net.nbn, 1.f);
  for (long long i = 0; i < n; ++i) {
    const long long k = net.bn_ext2int.empty() ? i : net.bn_ext2int[(size_t)i];
    m[(size_t)k] = mean[i]; v[(size_t)k] = var[i];
  }
  if (hipMemcpy(net.run_mean + (long long)model * net.nbn, m.data(), (size_t)net.nbn * 4, hipMemcpyHostToDevice) != hipSuccess ||
      hipMemcpy(net.run_var + (long long)model * net.nbn, v.data(), (size_t)net.nbn * 4, hipMemcpyHostToDevice) != hipSuccess)
    return fail(c, GAN_E_HIP, "copy failed");
  return GAN_OK;
}

gan_status gan_get_bn_running(gan_ctx* c, int32_t which, int32_t model, float* mean, float* var, int64_t n) {
  if (!c || !mean || !var || which < 0 || which > 1 || model < 0 || model >= c->L) return GAN_E_ARG;
  Net& net = which == 0 ? c->G : c->D;
  if (n != bn_ext_count(net)) return fail(c, GAN_E_ARG, "wrong element count");
  gan_status s = sync(c);
  if (s != GAN_OK) return s;
  std::vector<float> m((size_t)net.nbn), v((size_t)net.nbn);
  if (hipMemcpy(m.data(), net.run_mean + (long long)model * net.nbn, (size_t)net.nbn * 4, hipMemcpyDeviceToHost) != hipSuccess ||
      hipMemcpy(v.data(), net.run_var + (long long)model * net.nbn, (size_t)net.nbn * 4, hipMemcpyDeviceToHost) != hipSuccess)
    return fail(c, GAN_E_HIP, "copy failed");
  for (long long i = 0; i < n; ++i) {
    const long long k = net.bn_ext2int.empty() ? i : net.bn_ext2int[(size_t)i];
    mean[i] = m[(size_t)k]; var[i] = v[(size_t)k];
  }
  return GAN_OK;
}

gan_status gan_get_routing(gan_ctx* c, int32_t* perm, int32_t* offs) {
  if (!c) return GAN_E_ARG;
  if (c->last_n < 0) return fail(c, GAN_E_STATE, "no step has been taken");
  gan_status s = sync(c);
  if (s != GAN_OK) return s;
  if (offs) hipMemcpy(offs, c->rb.offs, (size_t)(c->L + 1) * 4, hipMemcpyDeviceToHost);
  if (perm && c->last_n > 0) {
    int nv = 0;
    hipMemcpy(&nv, c->rb.offs + c->L, 4, hipMemcpyDeviceToHost);
    for (int i = 0; i < c->last_n; ++i) perm[i] = -1;
    hipMemcpy(perm, c->rb.perm, (size_t)nv * 4, hipMemcpyDeviceToHost);
  }
  return GAN_OK;
}

gan_status gan_profile_enable(gan_ctx* c, int32_t enable) {
  if (!c) return GAN_E_ARG;
  gan_status s = sync(c);
  if (s != GAN_OK) return s;
  for (auto& e : c->prof_entries) { c->event_pool.push_back(e.e0); c->event_pool.push_back(e.e1); }
  c->prof_entries.clear();
  c->prof = enable != 0;
  c->prof_detail = enable == 2;     // 2: one family per layer shape
  c->prof_gemm_only = enable == 3;  // 3: only the MFMA kernels (fewest events in the stream)
  return GAN_OK;
}

gan_status gan_profile_read(gan_ctx* c, int32_t cap, const char** names, int64_t* launches, double* ms, double* flops,
                            double* bytes, int32_t* n_out) {
  if (!c || !names || !launches || !ms || !flops || !bytes || !n_out || cap < 1) return GAN_E_ARG;
  gan_status s = sync(c);
  if (s != GAN_OK) return s;
  int nf = 0;
  for (auto& e : c->prof_entries) {
    int k = -1;
    for (int i = 0; i < nf; ++i) if (strcmp(names[i], e.name) == 0) { k = i; break; }
    if (k < 0) {
      if (nf >= cap) continue;
      k = nf++;
      names[k] = e.name; launches[k] = 0; ms[k] = 0; flops[k] = 0; bytes[k] = 0;
    }
    float t = 0.f;
    hipEventElapsedTime(&t, e.e0, e.e1);
    launches[k] += 1; ms[k] += t; flops[k] += e.flops; bytes[k] += e.bytes;
  }
  // The MFMA launches of the two streams overlap: the time during which at least one of them ran (union of their
  // intervals on the clock of the first timed launch), with their summed work, as one more family.
  if (nf < cap && !c->prof_entries.empty()) {
    std::vector<std::pair<float, float>> iv;
    double fl = 0, by = 0;
    const hipEvent_t origin = c->prof_entries.front().e0;
    for (auto& e : c->prof_entries) {
      if (strncmp(e.name, "gemm_", 5) != 0 && strncmp(e.name, "wgrad", 5) != 0) continue;
      float t0 = 0.f, t1 = 0.f;
      if (hipEventElapsedTime(&t0, origin, e.e0) != hipSuccess || hipEventElapsedTime(&t1, origin, e.e1) != hipSuccess) continue;
      iv.push_back({t0, t1});
      fl += e.flops; by += e.bytes;
    }
    (void)hipGetLastError();
    if (!iv.empty()) {
      std::sort(iv.begin(), iv.end());
      double busy = 0;
      float lo = iv[0].first, hi = iv[0].second;
      for (auto& x : iv) {
        if (x.first <= hi) hi = std::max(hi, x.second);
        else { busy += hi - lo; lo = x.first; hi = x.second; }
      }
      busy += hi - lo;
      names[nf] = "(mfma busy)"; launches[nf] = (int64_t)iv.size(); ms[nf] = busy; flops[nf] = fl; bytes[nf] = by;
      ++nf;
    }
  }
  *n_out = nf;
  return GAN_OK;
}

// ---- single operations ------------------------------------------------------------------------------------
// enqueue, wait, and report: a refused launch, a launch error, or a failure while running
static gan_status finish_op(gan_ctx* c) {
  const gan_status launched = launch_status(c);
  const gan_status s = sync(c);
  return launched != GAN_OK ? launched : s;
}

static gan_status op_common(gan_ctx* c, const int32_t* offs, int n_groups, int rps, int tile_rows, int** tpre_out) {
  int* tp = nullptr;
  if (hipMalloc((void**)&tp, (size_t)(n_groups + 1) * 4) != hipSuccess) return fail(c, GAN_E_OOM, "tile prefix alloc");
  launch_tile_prefix(offs, n_groups, rps, tile_rows, tp, c->st);
  *tpre_out = tp;
  return GAN_OK;
}

// what the GEMM kernels address with 32-bit byte offsets: one segment of an operand
static bool fits_32bit(long long samples, long long side, long long channels, size_t es) {
  return samples * side * side * channels * (long long)es < (1LL << 31);
}

static gan_status op_conv(gan_ctx* c, int mode, const void* A, const void* W, void* Out, const int32_t* offs, int n_groups,
                          int n_samples, int C, int N, int Hin, int Hr, long long wstride) {
  if (!c || !A || !W || !Out || !offs || n_groups < 1 || n_samples < 0 || Hr < 1) return GAN_E_ARG;
  if (C < 64 || N < 64 || C % 64 || N % 64) return fail(c, GAN_E_SHAPE, "channel counts must be multiples of 64");
  if (!fits_32bit(n_samples, Hin, C, esize(c)) || !fits_32bit(n_samples, 2 * Hr, N, esize(c)) ||
      16LL * C * N * (long long)esize(c) >= (1LL << 31))
    return fail(c, GAN_E_SHAPE, "an operand of 2 GiB or more (the kernels use 32-bit byte offsets)");
  (void)take_launch_error();
  int* tp = nullptr;
  const int tr = c->op_tile_rows ? c->op_tile_rows : conv_tile_rows(N, (long long)n_samples * Hr * Hr / n_groups, n_groups);
  gan_status s = op_common(c, offs, n_groups, Hr * Hr, tr, &tp);
  if (s != GAN_OK) return s;
  ConvArgs a = {};
  a.A = A; a.W = W; a.Out = Out; a.Aux = nullptr; a.w_nstride = N; a.offs = offs; a.tpre = tp; a.w_stride = wstride; a.L = n_groups;
  a.seg_first = 0; a.nseg = 1; a.seg_samples = n_samples; a.C = C; a.N = N; a.Hin = Hin; a.Hr = Hr;
  a.ub_tiles = (int)(((long long)n_samples * Hr * Hr) / tr) + n_groups; a.slope = 0.f; a.tile_rows = tr;
  if (c->bf16) launch_conv<bf16_t>(mode, EPI_NONE, a, c->st); else launch_conv<float>(mode, EPI_NONE, a, c->st);
  s = finish_op(c);
  (void)hipFree(tp);
  return s;
}

gan_status gan_op_tile_rows(gan_ctx* c, int32_t rows) {
  if (!c) return GAN_E_ARG;
  if (rows != 0 && rows != 64 && rows != 128 && rows != 256) return fail(c, GAN_E_ARG, "tile heights are 64, 128 and 256 (0: automatic)");
  c->op_tile_rows = rows;
  return GAN_OK;
}

gan_status gan_op_conv_down(gan_ctx* c, const void* big, const void* w_down, void* small_out, const int32_t* offs,
                            int32_t n_groups, int32_t n_samples, int32_t cb, int32_t cs, int32_t hs) {
  return op_conv(c, MODE_DOWN, big, w_down, small_out, offs, n_groups, n_samples, cb, cs, 2 * hs, hs, (long long)16 * cb * cs);
}
gan_status gan_op_conv_up(gan_ctx* c, const void* small_in, const void* w_up, void* big_out, const int32_t* offs,
                          int32_t n_groups, int32_t n_samples, int32_t cb, int32_t cs, int32_t hs) {
  return op_conv(c, MODE_UP, small_in, w_up, big_out, offs, n_groups, n_samples, cs, cb, hs, hs, (long long)16 * cb * cs);
}
gan_status gan_op_conv_wgrad(gan_ctx* c, const void* big, const void* small_in, float* dw, const int32_t* offs,
                             int32_t n_groups, int32_t n_samples, int32_t cb, int32_t cs, int32_t hs) {
  if (!c || !big || !small_in || !dw || !offs || n_groups < 1 || n_samples < 0 || hs < 1) return GAN_E_ARG;
  if (cb < 8 || cs < 8 || (16 * cb) % 128 || cb % 8 || cs % 8) return fail(c, GAN_E_SHAPE, "unsupported channel counts");
  if (!fits_32bit(n_samples, 2 * hs, cb, esize(c)) || !fits_32bit(n_samples, hs, cs, esize(c)))
    return fail(c, GAN_E_SHAPE, "an operand of 2 GiB or more (the kernels use 32-bit byte offsets)");
  (void)take_launch_error();
  WgradArgs a = {};
  a.Big = big; a.Small = small_in; a.dW = dw; a.offs = offs; a.dw_stride = (long long)16 * cb * cs;
  a.L = n_groups; a.nseg = 1; a.seg_samples = n_samples; a.Cb = cb; a.Cs = cs; a.Hs = hs; a.ntaps = 16; a.ksplit = 1;
  if (c->bf16) launch_wgrad<bf16_t>(a, c->st); else launch_wgrad<float>(a, c->st);
  return finish_op(c);
}

gan_status gan_op_dropout(gan_ctx* c, void* x, const int32_t* offs, int32_t n_groups, int32_t n_samples, int32_t ch, int32_t h,
                          int32_t w, float p, uint64_t seed, int32_t step, int32_t layer, int32_t pass_id) {
  if (!c || !x || !offs || n_groups < 1 || n_samples < 0 || ch < 1 || h < 1 || w < 1 || step < 0 || layer < 0 || layer > 255 ||
      pass_id < 0)
    return GAN_E_ARG;
  if (!(p >= 0.f && p < 1.f)) return fail(c, GAN_E_ARG, "dropout probability outside [0, 1)");
  (void)take_launch_error();
  if (c->bf16) launch_dropout<bf16_t>(static_cast<bf16_t*>(x), offs, n_groups, n_samples, ch, h, w, p, seed, step, layer, pass_id, c->st);
  else launch_dropout<float>(static_cast<float*>(x), offs, n_groups, n_samples, ch, h, w, p, seed, step, layer, pass_id, c->st);
  return finish_op(c);
}
gan_status gan_op_w3_to_w4(gan_ctx* c, const float* w3, void* w4, void* w4t, int32_t n_groups, int32_t cb, int32_t cs) {
  if (!c || !w3 || !w4 || !w4t || n_groups < 1 || cb < 1 || cs < 1) return GAN_E_ARG;
  (void)take_launch_error();
  if (c->bf16) launch_w3_to_w4<bf16_t>(w3, static_cast<bf16_t*>(w4), static_cast<bf16_t*>(w4t), n_groups, cb, cs, c->st);
  else launch_w3_to_w4<float>(w3, static_cast<float*>(w4), static_cast<float*>(w4t), n_groups, cb, cs, c->st);
  return finish_op(c);
}
gan_status gan_op_dw4_to_dw3(gan_ctx* c, const float* dw4, float* dw3, int32_t n_groups, int32_t cb, int32_t cs) {
  if (!c || !dw4 || !dw3 || n_groups < 1 || cb < 1 || cs < 1) return GAN_E_ARG;
  (void)take_launch_error();
  launch_dw4_to_dw3(dw4, dw3, n_groups, cb, cs, c->st);
  return finish_op(c);
}

}  // extern "C"
