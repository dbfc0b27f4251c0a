// Host runtime of libpbkd.so: descriptor validation, workspace layout, the launch sequences of the
// teacher forward and of the student step, the block scheduler and the C ABI (include/pbkd.h).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <functional>
#include <memory>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

#include "../../include/pbkd.h"
#include "pbkd_internal.h"

namespace pbkd {
hipError_t init_conv_attributes();
}
using namespace pbkd;

namespace {

thread_local std::string g_err;

inline bool misaligned16(const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15) != 0; }

pbkd_status fail(pbkd_status st, const char *fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return st;
}

#define HIPCHK(expr)                                                                      \
  do {                                                                                    \
    hipError_t e_ = (expr);                                                               \
    if (e_ != hipSuccess) return fail(PBKD_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

// Optional per-launch timing: a pool of event pairs recorded around the launches whose kind is in the mask.
enum KernelKind {
  KK_CONV3X3 = 0, KK_CONV1X1, KK_PW_DGRAD, KK_PW_WGRAD, KK_DW_FWD, KK_DW_BWD, KK_CONV_WGRAD, KK_BN_FINALIZE,
  KK_HEAD_OUT, KK_HEAD_LOSS, KK_HEAD_BWD, KK_BN_BWD, KK_SGD, KK_REDUCE, KK_CONV_FIRST, KK_DWPW_FWD, KK_COUNT
};
const char *const kKindNames[KK_COUNT] = {
  "conv3x3_mfma", "conv1x1_mfma", "pw_dgrad_mfma", "pw_wgrad_mfma", "dw3x3_fwd", "dw3x3_bwd", "conv3x3_wgrad", "bn_finalize",
  "head_out", "head_loss", "head_bwd", "bn_bwd_apply", "sgd_momentum", "reduce_partials", "conv3x3_first", "dwpw_fwd"};

struct Prof {
  unsigned mask = 0;
  std::vector<hipEvent_t> ev;   // 2 per record
  std::vector<int> kind;
  size_t used = 0, cap = 0;
};

#define LAUNCH(pf, kk, st, expr)                                                            \
  do {                                                                                      \
    Prof *pf_ = (pf);                                                                       \
    const bool rec_ = pf_ && (pf_->mask >> (kk) & 1u) && pf_->used < pf_->cap;              \
    if (rec_) HIPCHK(hipEventRecord(pf_->ev[2 * pf_->used], (st)));                         \
    HIPCHK(expr);                                                                           \
    if (rec_) {                                                                             \
      HIPCHK(hipEventRecord(pf_->ev[2 * pf_->used + 1], (st)));                             \
      pf_->kind[pf_->used++] = (kk);                                                        \
    }                                                                                       \
  } while (0)

// The same for a launcher that can carry the two events itself (`expr` uses e0_ and e1_, null when not recording):
// the events then hold the dispatch's own time stamps and no event record sits between the kernels.
#define LAUNCH_CARRYING_EVENTS(pf, kk, expr)                                                \
  do {                                                                                      \
    Prof *pf_ = (pf);                                                                       \
    const bool rec_ = pf_ && (pf_->mask >> (kk) & 1u) && pf_->used < pf_->cap;              \
    hipEvent_t e0_ = rec_ ? pf_->ev[2 * pf_->used] : nullptr;                               \
    hipEvent_t e1_ = rec_ ? pf_->ev[2 * pf_->used + 1] : nullptr;                           \
    HIPCHK(expr);                                                                           \
    if (rec_) pf_->kind[pf_->used++] = (kk);                                                \
  } while (0)

struct LayerRT {
  int kind = 0, cin = 0, cout = 0, stride = 1, trainable = 0;
  int hin = 0, win = 0, hout = 0, wout = 0;
  // parameters: w0 = W (full / shortcut) or D (depthwise); w1 = P (pointwise) or null
  float *w0 = nullptr, *w1 = nullptr, *gamma = nullptr, *beta = nullptr;
  float *g_w0 = nullptr, *g_w1 = nullptr, *g_gamma = nullptr, *g_beta = nullptr;
  float *v_w0 = nullptr, *v_w1 = nullptr, *v_gamma = nullptr, *v_beta = nullptr;
  float *wpk = nullptr;             // weights of the MFMA conv producing z, packed (conv_pack_index)
  float *wpk_b = nullptr;           // pointwise weights packed for the data gradient (M = cin, K = cout)
  float *u = nullptr, *z = nullptr; // depthwise output, pre-BN conv output
  float *mean = nullptr, *rstd = nullptr, *scale = nullptr, *shift = nullptr;
  float *rmean = nullptr, *rvar = nullptr;   // running statistics (inference-mode BatchNorm)
  float *stat = nullptr;            // [cout][stat_parts] StatPart: per-tile statistics partials of z
  float *conv_part = nullptr;       // partial outputs of a 3x3 convolution whose K is split over workgroups
  float *wg_part = nullptr;         // partial sums of the conv weight gradient (pointwise: [splits][cout][cin]; full: [tiles][cout][cin][9])
  float *dw_part = nullptr;         // depthwise backward partials [tiles][cin][11]
  int stat_parts() const { return first_conv ? cfg.n_wgs : (taps == 9 ? cg.n_ptiles : pg.n_ptiles); }
  size_t n_w0 = 0, n_w1 = 0;
  int taps = 9;                     // of the MFMA conv producing z (9 full, 1 pointwise / shortcut)
  ConvGeom cg;                      // geometry of that conv when it is a 3x3
  PwGeom pg, pdg;                   // ... when it is a 1x1 (pointwise / shortcut): forward, data gradient
  DwGeom dwf, dwb;                  // depthwise forward / backward tiles
  WgradGeom wg;                     // pointwise weight gradient, or the full conv's when taps_wgrad
  CwGeom cw;                        // full-conv weight gradient (general kernel)
  bool first_conv = false;          // layer 0 with at most three input channels: its own forward kernel
  ConvFirstGeom cfg{};
  bool taps_wgrad = false;          // full conv with few input channels: its weight gradient runs on the matrix cores
  bool wgrad_bn_fused = false;      // ... and takes its BatchNorm's backward pass along (dz of this layer is never formed)
  bool fused_fwd = false;           // depthwise + pointwise forward in one kernel; pg then only describes the packing
  DwPwGeom dpg{};
};

// tuning aid: environment variable `name` set to the integer v
static bool env_is(const char *name, int v) {
  const char *e = std::getenv(name);
  return e && std::atoi(e) == v;
}

// Depthwise-separable layers whose forward pass may run as one kernel (stride 1, a shape the kernel's tiles divide).
// Measured on MI355X the fused kernel moves a quarter fewer bytes but is no faster than the two kernels it replaces
// (ImageNet-sized 64-channel layer: 406 us against 186 + 202 us; 16x16x128 layers: 24 us against 10 + 18.5 us, and it
// needs the producer's statistics finished by a kernel of their own), so it is OFF unless PBKD_DWPW=1 asks for it
// wherever the shape allows (read when a block is created).
bool choose_fused_fwd(int N, int cin, int cout, int h, int w, int stride, DwPwGeom &g) {
  if (!dwpw_ok(N, cin, cout, h, w, stride)) return false;
  g = dwpw_geom(N, cin, cout, h, w);
  if (!g.ok) return false;
  if (const char *env = std::getenv("PBKD_DWPW")) return std::atoi(env) != 0;
  return false;
}

struct Net {
  int n = 0, c = 0, h = 0, w = 0;
  int shortcut = 0, shortcut_stride = 1, pool = 0;
  float eps = 1e-5f;
  float bn_decay = 0.99f;
  bool track_running = false;       // set while a student step runs: finished statistics also move the running pair
  bool use_running = false;         // set while an inference-mode forward runs: no batch statistics at all
  std::vector<LayerRT> L;
  LayerRT sc;                       // projection shortcut (kind = -1)
  int last_c = 0, last_h = 0, last_w = 0;   // last layer's output (before the pool)
  int out_h = 0, out_w = 0;                 // block output
};

pbkd_status build_net(const pbkd_arch_desc *a, bool student, Net &net) {
  if (!a) return fail(PBKD_EINVAL, "null architecture descriptor");
  if (a->n_layers < 1 || !a->layers) return fail(PBKD_EINVAL, "a block needs at least one layer");
  if (a->n < 1 || a->c < 1 || a->h < 1 || a->w < 1) return fail(PBKD_ESHAPE, "block input shape must be positive");
  if (a->pool != 0 && a->pool != 2) return fail(PBKD_EINVAL, "pool must be 0 or 2");
  if (a->shortcut < 0 || a->shortcut > 2) return fail(PBKD_EINVAL, "shortcut must be 0, 1 (projection) or 2 (identity)");
  if (a->shortcut == 1 && a->shortcut_stride != 1 && a->shortcut_stride != 2)
    return fail(PBKD_EINVAL, "shortcut stride must be 1 or 2");
  if (!(a->bn_eps > 0.f)) return fail(PBKD_EINVAL, "bn_eps must be positive");
  if ((long long)a->n * a->c * a->h * a->w > 0x7fffffffLL) return fail(PBKD_EUNSUPPORTED, "input tensor exceeds 2^31 elements");
  net.n = a->n; net.c = a->c; net.h = a->h; net.w = a->w;
  net.shortcut = a->shortcut; net.shortcut_stride = a->shortcut_stride; net.pool = a->pool; net.eps = a->bn_eps;
  net.L.clear();
  int c = a->c, h = a->h, w = a->w;
  for (int l = 0; l < a->n_layers; ++l) {
    const pbkd_layer_desc &d = a->layers[l];
    if (d.kind != PBKD_CONV3X3 && d.kind != PBKD_DWSEP3X3) return fail(PBKD_EINVAL, "layer %d: unknown kind %d", l, d.kind);
    if (d.cin != c) return fail(PBKD_ESHAPE, "layer %d: cin %d does not match the incoming %d channels", l, d.cin, c);
    if (d.cout < 1 || d.cout > 65535) return fail(PBKD_ESHAPE, "layer %d: cout %d out of range", l, d.cout);
    if (d.stride != 1 && d.stride != 2) return fail(PBKD_EINVAL, "layer %d: stride must be 1 or 2", l);
    if (student && l > 0 && d.kind == PBKD_CONV3X3)
      return fail(PBKD_EUNSUPPORTED, "student layer %d: a full 3x3 convolution is supported only as layer 0 (no data gradient)", l);
    if (student && l > 0 && !d.trainable)
      return fail(PBKD_EUNSUPPORTED, "student layer %d: a frozen layer is supported only as layer 0", l);
    LayerRT r;
    r.kind = d.kind; r.cin = d.cin; r.cout = d.cout; r.stride = d.stride; r.trainable = student ? (d.trainable != 0) : 0;
    r.hin = h; r.win = w; r.hout = out_dim(h, d.stride); r.wout = out_dim(w, d.stride);
    if ((long long)a->n * r.cout * r.hout * r.wout > 0x7fffffffLL) return fail(PBKD_EUNSUPPORTED, "layer %d output exceeds 2^31 elements", l);
    if (d.kind == PBKD_CONV3X3) {
      // the 3x3 kernel's loaders address their input with 32-bit byte offsets
      if ((unsigned long long)a->n * d.cin * h * w * sizeof(float) >= (1ull << 32))
        return fail(PBKD_EUNSUPPORTED, "layer %d: a 3x3 convolution input of 4 GiB or more is not supported", l);
      r.n_w0 = (size_t)d.cout * d.cin * 9; r.n_w1 = 0; r.taps = 9;
      // a frozen teacher's products run on the bf16 matrix cores from operands split three ways (its weights are split
      // once, at upload); PBKD_CONV_SPLIT=0 keeps the fp32 MFMA kernel
      r.cg = conv_geom(9, a->n, d.cin, d.cout, r.hout, r.wout, d.stride, !student && !env_is("PBKD_CONV_SPLIT", 0));
      if (r.cg.split && (!conv_split_fits_width(r.cg, h, w, d.stride) ||
                         (unsigned long long)r.cg.ksplit * a->n * d.cout * r.hout * r.wout * sizeof(float) >= (1ull << 32)))
        r.cg = conv_geom(9, a->n, d.cin, d.cout, r.hout, r.wout, d.stride, false);   // aligned 16-byte fetches, 32-bit store offsets
      r.cw = cw_geom(a->n, d.cin, r.hout, r.wout, d.stride);
      r.first_conv = (l == 0) && conv_first_ok(d.cin, d.stride) &&
                     (unsigned long long)a->n * d.cout * r.hout * r.wout * sizeof(float) < (1ull << 32);   // its stores use 32-bit offsets
      if (r.first_conv) r.cfg = conv_first_geom(a->n, d.cin, d.cout, h, w);
      r.taps_wgrad = wgrad_taps_ok(d.cin, w, d.stride) && wgrad_taps_small(a->n, d.cout, d.cin, r.hout * r.wout);
      if (r.taps_wgrad) r.wg = wgrad_taps_geom(a->n, d.cout, d.cin, r.hout * r.wout);
      // behind a depthwise-separable layer the gradient arrives as g = dL/d(BatchNorm output): the weight-gradient
      // kernel then folds the BatchNorm backward in instead of reading a dz that a kernel of its own would have to write
      r.wgrad_bn_fused = r.taps_wgrad && l == 0 && a->n_layers >= 2 && a->layers[1].kind == PBKD_DWSEP3X3 &&
                         wgrad_taps_bn_ok(d.cin, w, d.stride) && !env_is("PBKD_WGRAD_BN_FUSED", 0);
      if (r.wgrad_bn_fused) r.wg = wgrad_taps_bn_geom(a->n, d.cout, d.cin, r.hout * r.wout);
    } else {
      r.n_w0 = (size_t)d.cin * 9; r.n_w1 = (size_t)d.cout * d.cin; r.taps = 1;
      r.pg = pw_geom(a->n, d.cin, d.cout, r.hout, r.wout, 1);
      r.fused_fwd = choose_fused_fwd(a->n, d.cin, d.cout, h, w, d.stride, r.dpg);
      if (r.fused_fwd) {             // the fused kernel reads the weights packed for its own channel tile
        r.pg = PwGeom{};
        r.pg.variant = -1;
        r.pg.bm = r.dpg.bm; r.pg.mtiles = r.dpg.mtiles; r.pg.nchunks = r.dpg.nchunks;
        r.pg.a_floats = 32 * r.dpg.bm; r.pg.n_ptiles = r.dpg.n_ptiles;
      }
      r.dwf = dw_geom(a->n, r.hout, r.wout, d.stride, false, h, w, l == 0, d.cin);
      r.dwb = dw_geom(a->n, r.hout, r.wout, d.stride, true, h, w, l == 0, d.cin);
      r.wg = wgrad_geom(a->n, d.cout, d.cin, r.hout * r.wout);
      r.pdg = pw_geom(a->n, d.cout, d.cin, r.hout, r.wout, 1);
    }
    net.L.push_back(r);
    c = d.cout; h = r.hout; w = r.wout;
  }
  net.last_c = c; net.last_h = h; net.last_w = w;
  if (a->shortcut == 2 && (c != a->c || h != a->h || w != a->w))
    return fail(PBKD_ESHAPE, "an identity skip needs the block's output [%d,%d,%d] to have the input's shape [%d,%d,%d]", c, h, w, a->c, a->h, a->w);
  if (a->shortcut == 1) {
    LayerRT &r = net.sc;
    r = LayerRT();
    r.kind = -1; r.cin = a->c; r.cout = c; r.stride = a->shortcut_stride; r.trainable = 0;
    r.hin = a->h; r.win = a->w; r.hout = out_dim(a->h, r.stride); r.wout = out_dim(a->w, r.stride);
    if (r.hout != h || r.wout != w)
      return fail(PBKD_ESHAPE, "shortcut output %dx%d does not match the main branch %dx%d", r.hout, r.wout, h, w);
    r.n_w0 = (size_t)c * a->c; r.taps = 1;
    r.pg = pw_geom(a->n, a->c, c, r.hout, r.wout, r.stride);
  }
  net.out_h = a->pool == 2 ? h / 2 : h;
  net.out_w = a->pool == 2 ? w / 2 : w;
  if (net.out_h < 1 || net.out_w < 1) return fail(PBKD_ESHAPE, "max-pool leaves an empty output");
  return PBKD_OK;
}

pbkd_status validate_pair(const pbkd_arch_desc *t, const pbkd_arch_desc *s, Net &tn, Net &sn) {
  pbkd_status st = build_net(t, false, tn);
  if (st != PBKD_OK) return st;
  st = build_net(s, true, sn);
  if (st != PBKD_OK) return st;
  if (tn.n != sn.n || tn.c != sn.c || tn.h != sn.h || tn.w != sn.w)
    return fail(PBKD_ESHAPE, "teacher and student block inputs differ");
  if (tn.last_c != sn.last_c || tn.out_h != sn.out_h || tn.out_w != sn.out_w)
    return fail(PBKD_ESHAPE, "teacher output [%d,%d,%d] and student output [%d,%d,%d] differ", tn.last_c, tn.out_h, tn.out_w,
                sn.last_c, sn.out_h, sn.out_w);
  return PBKD_OK;
}

unsigned long long net_flops(const Net &net, bool step) {
  unsigned long long total = 0;
  for (size_t l = 0; l < net.L.size(); ++l) {
    const LayerRT &r = net.L[l];
    const unsigned long long pix = (unsigned long long)net.n * r.hout * r.wout;
    if (r.kind == PBKD_CONV3X3) {
      const unsigned long long f = 2ull * 9 * r.cin * r.cout * pix;
      total += f;
      if (step && r.trainable) total += f + (l > 0 ? f : 0);
    } else {
      const unsigned long long fd = 2ull * 9 * r.cin * pix, fp = 2ull * r.cin * r.cout * pix;
      total += fd + fp;
      if (step && r.trainable) total += fd + fp + fp + (l > 0 ? fd : 0);
    }
  }
  if (net.shortcut == 1) total += 2ull * net.sc.cin * net.sc.cout * net.n * net.sc.hout * net.sc.wout;
  return total;
}

struct Bump {
  uintptr_t base;          // 0 when only the size is wanted: the addresses are then never formed as pointers into memory
  size_t off = 0;
  explicit Bump(char *b) : base(reinterpret_cast<uintptr_t>(b)) {}
  float *take(size_t floats) {
    const size_t o = off;
    off += (floats * sizeof(float) + 255) & ~(size_t)255;
    return reinterpret_cast<float *>(base + o);
  }
};

// One captured step: the argument tuple it was captured for and the executable graph.
struct StepGraph {
  int kind = 0;                       // 0: pbkd_distill_step, 1: pbkd_student_step, 2: pbkd_teacher_forward
  const void *x = nullptr, *t = nullptr;
  float lr = 0.f;
  hipStream_t s0 = nullptr, s1 = nullptr, aux = nullptr;
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;
};
constexpr size_t kMaxStepGraphs = 8;   // per block; the oldest is dropped beyond
// One captured all-block step: every argument of the call, flattened, and the executable graph.
struct ScheduleGraph {
  std::vector<unsigned long long> key;
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;
};
std::atomic<unsigned long long> g_next_uid{1};

}  // namespace

struct pbkd_block {
  Net t, s;
  std::vector<pbkd_layer_desc> t_layers, s_layers;
  float momentum = 0.9f;
  int loss_reduction = 0;
  char *ws = nullptr;
  size_t ws_bytes = 0;
  // student arenas: [trainable tensors ...][frozen tensors ...]; grads and momentum share the layout
  float *s_params = nullptr, *s_grads = nullptr, *s_mom = nullptr;
  size_t n_trainable = 0, n_student = 0;
  float *s_pk = nullptr;            // all packed copies of student conv weights, contiguous
  size_t n_pk = 0;
  int *map_f = nullptr, *map_b = nullptr;   // arena index -> index into s_pk (or -1)
  // student scratch
  float *gz = nullptr, *du = nullptr, *head_partial = nullptr, *loss_dev = nullptr;
  // the update kernel's work list: one job per trainable tensor (or adjacent pair), and the job of each workgroup
  GradJob *jobs_dev = nullptr;
  int *job_of_block_dev = nullptr;
  std::vector<GradJob> jobs;
  std::vector<int> job_of_block;
  int head_nblk = 1;
  hipStream_t last_stream = nullptr;
  bool has_loss = false;
  hipEvent_t ev_teacher = nullptr, ev_student = nullptr, ev_target_free = nullptr, ev_fork = nullptr;
  hipEvent_t ev_step_done[2] = {nullptr, nullptr};   // the ends of the last two eager two-stream steps, in turn
  unsigned step_count = 0;
  // The block's last two student steps issued by pbkd_distill_step_all: which input and target buffers they read, and
  // the event that ends them.  A caller that alternates between two sets of target buffers lets the next step's
  // teacher chain run a whole step ahead: a teacher launch waits only for the steps that read the buffer it overwrites.
  struct ReaderRec {
    const void *x = nullptr, *t = nullptr;
    hipEvent_t ev = nullptr;
    bool used = false;
  };
  ReaderRec readers[2];
  int reader_next = 0;
  // graph mode (pbkd_block_set_graph_mode): a step's launches are captured once per argument tuple and replayed
  bool graph_mode = false;
  std::vector<StepGraph> graphs;
  std::vector<ScheduleGraph> schedule_graphs;   // of pbkd_distill_step_all calls whose first block this is
  unsigned long long uid = 0;                   // distinguishes this handle from an earlier one at the same address
  // optional second stream for the weight-gradient branch of the backward pass (pbkd_block_set_aux_stream)
  hipStream_t aux = nullptr;
  std::vector<hipEvent_t> ev_dz, ev_wg;   // per student layer: dz ready (main -> aux), weight gradient done (aux -> main)
  double *mse_scratch = nullptr;           // 256 partials + result of pbkd_feature_mse
  float *gz2 = nullptr;                    // layers alternate between gz and gz2 for their dz
  float *gbuf(int l) const { return (l & 1) ? gz2 : gz; }
  Prof prof;
};

namespace {

void drop_graphs(pbkd_block &b) {
  for (StepGraph &g : b.graphs) {
    if (g.exec) (void)hipGraphExecDestroy(g.exec);
    if (g.graph) (void)hipGraphDestroy(g.graph);
  }
  b.graphs.clear();
  for (ScheduleGraph &g : b.schedule_graphs) {
    if (g.exec) (void)hipGraphExecDestroy(g.exec);
    if (g.graph) (void)hipGraphDestroy(g.graph);
  }
  b.schedule_graphs.clear();
}

size_t layer_slots(const LayerRT &r) { return r.kind == PBKD_DWSEP3X3 ? 4 : 3; }
size_t pack_floats_fwd(const LayerRT &r) {
  if (r.taps != 9) return pw_pack_floats(r.pg);
  return r.cg.split ? conv_split_pack_floats(r.cg) : conv_pack_floats(r.cg);
}

// Assigns every device pointer of the block inside [base, base+total) and returns total.  With
// base == nullptr the pointers are meaningless and only the size is of interest.
size_t layout(pbkd_block &b, char *base) {
  Bump bump(base);
  const int N = b.t.n;
  auto act = [&](LayerRT &r) {
    if (r.kind == PBKD_DWSEP3X3) r.u = bump.take((size_t)N * r.cin * r.hout * r.wout);
    r.z = bump.take((size_t)N * r.cout * r.hout * r.wout);
    r.mean = bump.take(r.cout); r.rstd = bump.take(r.cout); r.scale = bump.take(r.cout); r.shift = bump.take(r.cout);
    r.rmean = bump.take(r.cout); r.rvar = bump.take(r.cout);
    r.stat = bump.take((size_t)r.stat_parts() * r.cout * kStatFloats);
    if (r.taps == 9 && !r.first_conv && r.cg.ksplit > 1) r.conv_part = bump.take((size_t)r.cg.ksplit * N * r.cout * r.hout * r.wout);
  };
  // ---- teacher
  auto tparams = [&](LayerRT &r) {
    r.w0 = bump.take(r.n_w0);
    if (r.n_w1) r.w1 = bump.take(r.n_w1);
    r.gamma = bump.take(r.cout); r.beta = bump.take(r.cout);
    r.wpk = bump.take(pack_floats_fwd(r));
  };
  for (auto &r : b.t.L) { tparams(r); act(r); }
  if (b.t.shortcut == 1) { tparams(b.t.sc); act(b.t.sc); }
  // ---- student: arena order = trainable layers first, frozen ones after
  size_t total = 0, trainable = 0;
  auto count = [&](const LayerRT &r) { return r.n_w0 + r.n_w1 + 2 * (size_t)r.cout; };
  for (auto &r : b.s.L) { total += count(r); if (r.trainable) trainable += count(r); }
  if (b.s.shortcut == 1) total += count(b.s.sc);
  b.n_student = total; b.n_trainable = trainable;
  b.s_params = bump.take(total); b.s_grads = bump.take(total); b.s_mom = bump.take(total);
  b.map_f = reinterpret_cast<int *>(bump.take(total)); b.map_b = reinterpret_cast<int *>(bump.take(total));
  size_t npk = 0;
  auto pk_count = [&](const LayerRT &r) { return pack_floats_fwd(r) + (r.kind == PBKD_DWSEP3X3 ? pw_pack_floats(r.pdg) : 0); };
  for (auto &r : b.s.L) npk += pk_count(r);
  if (b.s.shortcut == 1) npk += pk_count(b.s.sc);
  b.n_pk = npk;
  b.s_pk = bump.take(npk);
  {
    size_t o = 0;
    auto assign = [&](LayerRT &r) {
      r.wpk = b.s_pk + o; o += pack_floats_fwd(r);
      if (r.kind == PBKD_DWSEP3X3) { r.wpk_b = b.s_pk + o; o += pw_pack_floats(r.pdg); }
    };
    for (auto &r : b.s.L) assign(r);
    if (b.s.shortcut == 1) assign(b.s.sc);
  }
  size_t off_t = 0, off_f = trainable;
  auto sparams = [&](LayerRT &r) {
    size_t &o = r.trainable ? off_t : off_f;
    auto put = [&](float *&p, float *&g, float *&v, size_t n) { p = b.s_params + o; g = b.s_grads + o; v = b.s_mom + o; o += n; };
    put(r.w0, r.g_w0, r.v_w0, r.n_w0);
    if (r.n_w1) put(r.w1, r.g_w1, r.v_w1, r.n_w1);
    put(r.gamma, r.g_gamma, r.v_gamma, r.cout);
    put(r.beta, r.g_beta, r.v_beta, r.cout);
  };
  for (auto &r : b.s.L) { sparams(r); act(r); }
  if (b.s.shortcut == 1) { sparams(b.s.sc); act(b.s.sc); }
  size_t zmax = 0, umax = 0;
  // The partial sums of every trainable layer stay until the update kernel at the end of the step adds them up,
  // so each layer has its own.  One gradient job per tensor; gamma and beta are adjacent in the arena and share one.
  b.jobs.clear();
  b.job_of_block.clear();
  auto add_job = [&](const float *partial, const float *first, size_t count, int nparts, int kind, int C) {
    GradJob j{};
    j.partial = partial; j.arena_off = (unsigned)(first - b.s_params); j.count = (int)count; j.nparts = nparts; j.kind = kind; j.C = C;
    j.flat = (kind == 2 || nparts <= kGradJobFlatMaxParts) ? 1 : 0;
    j.first_block = (int)b.job_of_block.size();
    b.job_of_block.insert(b.job_of_block.end(), grad_job_blocks(j), (int)b.jobs.size());
    b.jobs.push_back(j);
  };
  for (auto &r : b.s.L) {
    zmax = std::max(zmax, (size_t)N * r.cout * r.hout * r.wout);
    // gz also receives the gradient w.r.t. this layer's input (previous layer's output)
    zmax = std::max(zmax, (size_t)N * r.cin * r.hin * r.win);
    if (r.kind == PBKD_DWSEP3X3) umax = std::max(umax, (size_t)N * r.cin * r.hout * r.wout);
    if (!r.trainable) continue;
    if (r.kind == PBKD_DWSEP3X3) {
      r.wg_part = bump.take((size_t)r.wg.splits * r.cout * r.cin);
      r.dw_part = bump.take((size_t)r.dwb.n_tiles * r.cin * 11);
      add_job(r.dw_part, r.w0, r.n_w0, r.dwb.n_tiles, 1, r.cin);
      add_job(r.wg_part, r.w1, r.n_w1, r.wg.splits, 0, 0);
    } else {
      const int parts = r.taps_wgrad ? r.wg.slabs : r.cw.n_tiles;
      r.wg_part = bump.take((size_t)parts * r.cout * r.cin * 9);
      add_job(r.wg_part, r.w0, r.n_w0, parts, 0, 0);
    }
    add_job(nullptr, r.gamma, 2 * (size_t)r.cout, 0, 2, 0);
  }
  b.gz = bump.take(zmax); b.gz2 = bump.take(zmax); b.du = bump.take(umax ? umax : 1);
  b.jobs_dev = reinterpret_cast<GradJob *>(bump.take((b.jobs.size() * sizeof(GradJob) + 3) / 4 + 1));
  b.job_of_block_dev = reinterpret_cast<int *>(bump.take(b.job_of_block.size() + 1));
  b.head_nblk = head_blocks(N, b.s.last_h, b.s.last_w, b.s.pool);
  b.head_partial = bump.take((size_t)b.head_nblk * b.s.last_c * 3);
  b.loss_dev = bump.take(1);
  b.mse_scratch = reinterpret_cast<double *>(bump.take(2 * 257));
  return bump.off;
}

void copy_desc(const pbkd_arch_desc *a, std::vector<pbkd_layer_desc> &dst) { dst.assign(a->layers, a->layers + a->n_layers); }

// Packs canonical conv weights on the host into the layout the MFMA kernel stages (zero padded).
// fwd: A[m=o][k=c][tap] = w[(o*K + c)*taps + tap]; transposed (pointwise data gradient): A[m=c][k=o] = P[o][c].
std::vector<float> pack_host(const float *w, const ConvGeom &g, int taps, int M, int K, bool transposed) {
  std::vector<float> out(conv_pack_floats(g), 0.f);
  for (int m = 0; m < M; ++m)
    for (int k = 0; k < K; ++k)
      for (int tap = 0; tap < taps; ++tap) {
        const float v = transposed ? w[(size_t)k * M + m] : w[((size_t)m * K + k) * taps + tap];
        out[conv_pack_index(g, m, k, tap)] = v;
      }
  return out;
}

// bf16 nearest v (ties to even), as the upper half of an fp32 bit pattern
static uint16_t bf16_rn(float v) {
  uint32_t u;
  std::memcpy(&u, &v, sizeof u);
  if ((u & 0x7f800000u) == 0x7f800000u) return (uint16_t)(u >> 16);   // infinities and NaNs keep their upper half
  return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}
static float bf16_value(uint16_t h) {
  const uint32_t u = (uint32_t)h << 16;
  float v;
  std::memcpy(&v, &u, sizeof v);
  return v;
}
// The bf16-split kernel's weight image: w = w0 + w1 + w2 exactly (w0 = bf16 nearest w, w1 = bf16 nearest w - w0,
// w2 = the rest, which has at most eight significant bits left).
std::vector<uint16_t> pack_host_split(const float *w, const ConvGeom &g, int M, int K) {
  std::vector<uint16_t> out(conv_split_pack_floats(g) * 2, 0);
  for (int m = 0; m < M; ++m)
    for (int k = 0; k < K; ++k)
      for (int tap = 0; tap < 9; ++tap) {
        float v = w[((size_t)m * K + k) * 9 + tap];
        uint16_t piece[3];
        for (int pc = 0; pc < 3; ++pc) {
          piece[pc] = bf16_rn(v);
          v -= bf16_value(piece[pc]);
        }
        for (int c = 0; c < 3; ++c) {
          if (tap < 8) {
            out[conv_split_pack_index(g, m, k, c, tap / 2, tap % 2)] = piece[c];
          } else {          // the ninth tap: pieces paired with each other
            for (int h = 0; h < 2; ++h) out[conv_split_pack_index(g, m, k, c, 4, h)] = piece[kSplitLastW[c][h]];
          }
        }
      }
  return out;
}

// Uploads the packed copies of one layer's conv weights (host pointer to the canonical tensor).
pbkd_status upload_packed_pointwise(LayerRT &r, const float *p_host, bool with_dgrad, hipStream_t s);
pbkd_status upload_packed(LayerRT &r, const float *w_host, hipStream_t s) {
  if (r.kind == PBKD_DWSEP3X3) return PBKD_OK;   // depthwise weights are read directly; the pointwise ones come separately
  if (r.taps == 1) return upload_packed_pointwise(r, w_host, false, s);   // projection shortcut
  if (r.cg.split) {
    std::vector<uint16_t> pk = pack_host_split(w_host, r.cg, r.cout, r.cin);
    HIPCHK(hipMemcpyAsync(r.wpk, pk.data(), pk.size() * sizeof(uint16_t), hipMemcpyHostToDevice, s));
    HIPCHK(hipStreamSynchronize(s));
    return PBKD_OK;
  }
  std::vector<float> pk = pack_host(w_host, r.cg, r.taps, r.cout, r.cin, false);
  HIPCHK(hipMemcpyAsync(r.wpk, pk.data(), pk.size() * sizeof(float), hipMemcpyHostToDevice, s));
  HIPCHK(hipStreamSynchronize(s));   // pk is a temporary
  return PBKD_OK;
}
std::vector<float> pack_host_pw(const float *w, const PwGeom &g, int M, int K, bool transposed) {
  std::vector<float> out(pw_pack_floats(g), 0.f);
  for (int m = 0; m < M; ++m)
    for (int k = 0; k < K; ++k) out[pw_pack_index(g, m, k)] = transposed ? w[(size_t)k * M + m] : w[(size_t)m * K + k];
  return out;
}

pbkd_status upload_packed_pointwise(LayerRT &r, const float *p_host, bool with_dgrad, hipStream_t s) {
  std::vector<float> pk = pack_host_pw(p_host, r.pg, r.cout, r.cin, false);
  HIPCHK(hipMemcpyAsync(r.wpk, pk.data(), pk.size() * sizeof(float), hipMemcpyHostToDevice, s));
  HIPCHK(hipStreamSynchronize(s));
  if (with_dgrad) {
    std::vector<float> pb = pack_host_pw(p_host, r.pdg, r.cin, r.cout, true);
    HIPCHK(hipMemcpyAsync(r.wpk_b, pb.data(), pb.size() * sizeof(float), hipMemcpyHostToDevice, s));
    HIPCHK(hipStreamSynchronize(s));
  }
  return PBKD_OK;
}

std::once_flag g_init_once;
hipError_t g_init_err = hipSuccess;

// ---------------------------------------------------------------------------------- launch sequences

// Forward of one network up to the last layer's pre-BN output and its BatchNorm statistics (and the
// shortcut branch's).  BatchNorm+ReLU of layer l is applied by whoever reads z_l next.
BnPending bn_pending(const Net &net, const LayerRT &r) {
  BnPending b{};
  if (net.use_running) return b;   // nothing is ever pending in inference mode
  if (net.track_running) { b.rmean = r.rmean; b.rvar = r.rvar; b.decay = net.bn_decay; }
  b.partial = r.stat; b.n_parts = r.stat_parts(); b.count = (double)net.n * r.hout * r.wout; b.eps = net.eps;
  b.gamma = r.gamma; b.beta = r.beta; b.mean = r.mean; b.rstd = r.rstd; b.scale = r.scale; b.shift = r.shift;
  return b;
}

// Finishing the statistics inside the consumer costs every one of its workgroups a pass over the channel's
// partials; beyond this many partial reads per channel a separate kernel is cheaper.
constexpr long long kDeferMaxReads = 16384;
bool defer_ok(const LayerRT &r, int consumer_blocks_per_channel) {
  return (long long)r.stat_parts() * consumer_blocks_per_channel <= kDeferMaxReads;
}

bool head_defers(const Net &net) {
  const int nb = head_blocks(net.n, net.last_h, net.last_w, net.pool);
  return defer_ok(net.L.back(), nb) && (net.shortcut != 1 || defer_ok(net.sc, nb));
}

pbkd_status forward_net(Net &net, const float *x, hipStream_t st, Prof *pf) {
  const int N = net.n;
  const float *in = x, *in_scale = nullptr, *in_shift = nullptr;
  BnPending pend{};       // statistics of `in` that no kernel has finished yet
  const bool running = net.use_running;
  if (running) {          // every layer's scale and shift follow from its running pair before anything runs
    auto fixed = [&](LayerRT &r) -> pbkd_status {
      LAUNCH(pf, KK_BN_FINALIZE, st, launch_bn_running(r.gamma, r.beta, r.rmean, r.rvar, net.eps, r.mean, r.rstd, r.scale, r.shift, r.cout, st));
      return PBKD_OK;
    };
    for (auto &r : net.L) { pbkd_status e = fixed(r); if (e != PBKD_OK) return e; }
    if (net.shortcut == 1) { pbkd_status e = fixed(net.sc); if (e != PBKD_OK) return e; }
  }
  auto pointwise = [&](LayerRT &r, const float *src, int hin, int win, int stride) -> pbkd_status {
    PwArgs pa{};
    pa.in = src; pa.wpk = r.wpk; pa.out = r.z; pa.stat_partial = running ? nullptr : r.stat;
    pa.N = N; pa.Cin = r.cin; pa.Cout = r.cout; pa.HWin = hin * win; pa.Win = win; pa.Ho = r.hout; pa.Wo = r.wout;
    pa.stride = stride; pa.nchunks = r.pg.nchunks; pa.g = r.pg;
    LAUNCH(pf, KK_CONV1X1, st, launch_pw(pa, st));
    return PBKD_OK;
  };
  for (size_t l = 0; l < net.L.size(); ++l) {
    LayerRT &r = net.L[l];
    if (r.kind == PBKD_CONV3X3) {
      if (pend.partial) {   // the convolution's loader reads finished scale/shift arrays
        LAUNCH(pf, KK_BN_FINALIZE, st, launch_bn_finalize(pend, net.L[l - 1].cout, st));
        pend = BnPending{};
      }
      ConvArgs ca{};
      ca.in = in; ca.in_scale = in_scale; ca.in_shift = in_shift; ca.wpk = r.wpk;
      ca.Cin = r.cin; ca.H = r.hin; ca.W = r.win; ca.stride = r.stride;
      ca.out = r.z; ca.stat_partial = running ? nullptr : r.stat;
      ca.N = N; ca.Cout = r.cout; ca.Ho = r.hout; ca.Wo = r.wout; ca.g = r.cg; ca.split_out = r.conv_part;
      if (r.first_conv) {
        ca.w_canon = r.w0;
        LAUNCH_CARRYING_EVENTS(pf, KK_CONV_FIRST, launch_conv_first(ca, r.cfg, st, e0_, e1_));
      } else {
        LAUNCH_CARRYING_EVENTS(pf, KK_CONV3X3, launch_conv(9, ca, st, e0_, e1_));
        if (r.cg.ksplit > 1) LAUNCH(pf, KK_CONV3X3, st, launch_conv_ksplit_finish(ca, st));
      }
    } else if (r.fused_fwd) {
      // a workgroup of the fused kernel spans all input channels: it reads finished scale/shift arrays
      if (pend.partial) {
        LAUNCH(pf, KK_BN_FINALIZE, st, launch_bn_finalize(pend, net.L[l - 1].cout, st));
        pend = BnPending{};
      }
      DwPwArgs fa{};
      fa.in = in; fa.D = r.w0; fa.wpk = r.wpk; fa.in_scale = in_scale; fa.in_shift = in_shift;
      fa.u_out = r.u; fa.z_out = r.z; fa.stat_partial = running ? nullptr : r.stat;
      fa.N = N; fa.Cin = r.cin; fa.Cout = r.cout; fa.H = r.hin; fa.W = r.win; fa.g = r.dpg;
      LAUNCH(pf, KK_DWPW_FWD, st, launch_dwpw_fwd(fa, st));
    } else {
      // (the 2x2 kernel's workgroups span channels, so none of them can finish a channel's statistics)
      if (pend.partial && (r.dwf.fast == 2 || !defer_ok(net.L[l - 1], r.dwf.n_tiles))) {
        LAUNCH(pf, KK_BN_FINALIZE, st, launch_bn_finalize(pend, net.L[l - 1].cout, st));
        pend = BnPending{};
      }
      DwFwdArgs da{};
      da.in = in; da.D = r.w0; da.out = r.u; da.in_scale = in_scale; da.in_shift = in_shift; da.pend = pend;
      da.N = N; da.C = r.cin; da.H = r.hin; da.W = r.win; da.Ho = r.hout; da.Wo = r.wout; da.stride = r.stride; da.g = r.dwf;
      LAUNCH(pf, KK_DW_FWD, st, launch_dw_fwd(da, st));   // finishes the pending statistics of its input, if any
      pend = BnPending{};
      pbkd_status e = pointwise(r, r.u, r.hout, r.wout, 1);
      if (e != PBKD_OK) return e;
    }
    in = r.z; in_scale = r.scale; in_shift = r.shift;
    pend = bn_pending(net, r);
  }
  if (net.shortcut == 1) {
    pbkd_status e = pointwise(net.sc, x, net.sc.hin, net.sc.win, net.sc.stride);
    if (e != PBKD_OK) return e;
  }
  // the statistics of the last layer (and of the shortcut) stay pending: the head kernel that follows
  // finishes them (head_args with first = true), unless that would cost more than a kernel of its own
  if (!running && !head_defers(net)) {
    LayerRT &r = net.L.back();
    LAUNCH(pf, KK_BN_FINALIZE, st, launch_bn_finalize(bn_pending(net, r), r.cout, st));
    if (net.shortcut == 1) LAUNCH(pf, KK_BN_FINALIZE, st, launch_bn_finalize(bn_pending(net, net.sc), net.sc.cout, st));
  }
  return PBKD_OK;
}

// first: this is the first head launch after forward_net, the one that finishes the BatchNorm statistics.
// x: the block input (what an identity skip adds).
HeadArgs head_args(pbkd_block &b, Net &net, bool first, const float *x) {
  HeadArgs h{};
  LayerRT &r = net.L.back();
  h.z = r.z; h.scale = r.scale; h.shift = r.shift; h.mean = r.mean; h.rstd = r.rstd;
  if (net.shortcut == 1) { h.zs = net.sc.z; h.scale_s = net.sc.scale; h.shift_s = net.sc.shift; }
  if (net.shortcut == 2) { h.zs = x; h.identity_skip = 1; }
  if (first && !net.use_running && head_defers(net)) {
    h.pend = bn_pending(net, r);
    if (net.shortcut == 1) h.pend_s = bn_pending(net, net.sc);
  }
  h.N = net.n; h.C = net.last_c; h.H = net.last_h; h.W = net.last_w; h.pool = net.pool;
  h.n_blk = head_blocks(net.n, net.last_h, net.last_w, net.pool);
  (void)b;
  return h;
}

// Backward through the student block.  Layer l's dz lives in gbuf(l) (the two buffers alternate).  The
// weight gradients (and their partial-sum reductions) depend only on dz and stored activations, nothing
// downstream depends on them before the update: with an auxiliary stream they run beside the data-gradient
// chain.  The data gradient of layer l is written into gbuf(l-1) = gbuf(l+1), so it first waits for the
// weight gradient of layer l+1, which reads that buffer.
pbkd_status student_backward(pbkd_block &b, const float *x, hipStream_t st) {
  Net &net = b.s;
  Prof *pf = &b.prof;
  const int N = net.n;
  const int nl = (int)net.L.size();
  hipStream_t ws = b.aux ? b.aux : st;
  int lowest = nl;
  for (int l = nl - 1; l >= 0; --l) {
    LayerRT &r = net.L[l];
    if (!r.trainable) break;   // only layer 0 can be frozen; nothing below it needs a gradient
    lowest = l;
    float *dz = b.gbuf(l);
    if (b.aux) {
      HIPCHK(hipEventRecord(b.ev_dz[l], st));
      HIPCHK(hipStreamWaitEvent(ws, b.ev_dz[l], 0));
    }
    if (r.kind == PBKD_DWSEP3X3) {
      WgradArgs wa{};
      wa.dz = dz; wa.u = r.u; wa.partial = r.wg_part; wa.N = N; wa.Co = r.cout; wa.Ci = r.cin; wa.HW = r.hout * r.wout; wa.g = r.wg;
      LAUNCH(pf, KK_PW_WGRAD, ws, launch_pw_wgrad(wa, ws));   // its partials are summed by the update kernel
      if (b.aux) HIPCHK(hipEventRecord(b.ev_wg[l], ws));
      PwArgs pa{};   // du[n,c,p] = sum_o P[o,c] dz[n,o,p]: a 1x1 conv with P read as [K=cout][M=cin]
      pa.in = dz; pa.wpk = r.wpk_b; pa.out = b.du; pa.stat_partial = nullptr;
      pa.N = N; pa.Cin = r.cout; pa.Cout = r.cin; pa.HWin = r.hout * r.wout; pa.Win = r.wout; pa.Ho = r.hout; pa.Wo = r.wout;
      pa.stride = 1; pa.nchunks = r.pdg.nchunks; pa.g = r.pdg;
      LAUNCH(pf, KK_PW_DGRAD, st, launch_pw(pa, st));
      float *gprev = b.gbuf(l - 1);   // unused for l == 0
      DwBwdArgs da{};
      da.du = b.du; da.D = r.w0; da.gout = gprev; da.partial = r.dw_part;
      da.N = N; da.C = r.cin; da.H = r.hin; da.W = r.win; da.Ho = r.hout; da.Wo = r.wout; da.stride = r.stride; da.g = r.dwb;
      float *dg_prev = nullptr, *db_prev = nullptr;
      if (l == 0) {
        da.first_layer = 1; da.in = x;
      } else {
        LayerRT &q = net.L[l - 1];
        da.first_layer = 0; da.in = q.z; da.in_scale = q.scale; da.in_shift = q.shift; da.in_mean = q.mean; da.in_rstd = q.rstd;
        dg_prev = q.g_gamma; db_prev = q.g_beta;
        if (b.aux && l + 1 < nl) HIPCHK(hipStreamWaitEvent(st, b.ev_wg[l + 1], 0));
      }
      LAUNCH(pf, KK_DW_BWD, st, launch_dw_bwd(da, st));
      // of its partials, the depthwise weight gradient waits for the update kernel; the previous layer's dgamma and
      // dbeta are needed now: the BatchNorm-backward kernel sums them itself when they are few
      if (l > 0 && net.L[l - 1].trainable) {
        LayerRT &q = net.L[l - 1];
        const bool fold = r.dwb.n_tiles <= kBnBwdFoldMaxTiles && !q.wgrad_bn_fused;
        if (!fold) LAUNCH(pf, KK_REDUCE, st, launch_dw_bwd_finalize(r.dw_part, r.dwb.n_tiles, r.cin, nullptr, dg_prev, db_prev, st));
        if (!q.wgrad_bn_fused)   // (else the layer's weight-gradient kernel takes g, z and the two sums as they are)
          LAUNCH(pf, KK_BN_BWD, st, launch_bn_bwd_apply(gprev, q.z, q.scale, q.mean, q.rstd, q.g_gamma, q.g_beta,
                                                        fold ? r.dw_part : nullptr, r.dwb.n_tiles, N, q.cout, q.hout * q.wout, st));
      }
    } else {
      if (r.taps_wgrad) {   // dW[o][c][tap] as a product over pixels with the shifted input channels as columns
        WgradArgs wa{};
        wa.dz = dz; wa.u = x; wa.partial = r.wg_part; wa.N = N; wa.Co = r.cout; wa.Ci = 9 * r.cin; wa.HW = r.hout * r.wout;
        wa.W = r.wout; wa.g = r.wg;
        if (r.wgrad_bn_fused) {
          wa.z = r.z; wa.scale = r.scale; wa.mean = r.mean; wa.rstd = r.rstd; wa.dgamma = r.g_gamma; wa.dbeta = r.g_beta;
        }
        LAUNCH(pf, KK_CONV_WGRAD, ws, launch_pw_wgrad(wa, ws));
      } else {
        CwArgs ca{};
        ca.dz = dz; ca.x = x; ca.partial = r.wg_part;
        ca.N = N; ca.Cin = r.cin; ca.Cout = r.cout; ca.H = r.hin; ca.W = r.win; ca.Ho = r.hout; ca.Wo = r.wout; ca.stride = r.stride;
        ca.g = r.cw;
        LAUNCH(pf, KK_CONV_WGRAD, ws, launch_conv_wgrad(ca, ws));
      }
      if (b.aux) HIPCHK(hipEventRecord(b.ev_wg[l], ws));
    }
  }
  if (b.aux)   // the update (and the next forward pass, which overwrites the stored activations) needs them all
    for (int l = nl - 1; l >= lowest; --l) HIPCHK(hipStreamWaitEvent(st, b.ev_wg[l], 0));
  return PBKD_OK;
}

pbkd_status tensor_ptr(pbkd_block *b, int which, int layer, int slot, float **p, size_t *n) {
  const bool teacher = (which == PBKD_TEACHER_PARAM || which == PBKD_TEACHER_ACT || which == PBKD_TEACHER_BN_RUNNING);
  Net &net = teacher ? b->t : b->s;
  LayerRT *r = nullptr;
  if (layer >= 0 && layer < (int)net.L.size())
    r = &net.L[layer];
  else if (layer == (int)net.L.size() && net.shortcut == 1)
    r = &net.sc;
  else
    return fail(PBKD_EINVAL, "layer index %d out of range", layer);
  const size_t act_u = (size_t)net.n * r->cin * r->hout * r->wout, act_z = (size_t)net.n * r->cout * r->hout * r->wout;
  if (which == PBKD_STUDENT_ACT || which == PBKD_TEACHER_ACT) {
    switch (slot) {
      case 0: if (r->kind != PBKD_DWSEP3X3) return fail(PBKD_EINVAL, "layer %d has no depthwise output", layer);
              *p = r->u; *n = act_u; return PBKD_OK;
      case 1: *p = r->z; *n = act_z; return PBKD_OK;
      case 2: *p = r->mean; *n = r->cout; return PBKD_OK;
      case 3: *p = r->rstd; *n = r->cout; return PBKD_OK;
      case 4: *p = r->scale; *n = r->cout; return PBKD_OK;
      case 5: *p = r->shift; *n = r->cout; return PBKD_OK;
      default: return fail(PBKD_EINVAL, "activation slot %d out of range", slot);
    }
  }
  if (which == PBKD_STUDENT_BN_RUNNING || which == PBKD_TEACHER_BN_RUNNING) {
    if (slot != 0 && slot != 1) return fail(PBKD_EINVAL, "running-statistics slot %d out of range", slot);
    *p = slot == 0 ? r->rmean : r->rvar; *n = r->cout;
    return PBKD_OK;
  }
  if (slot < 0 || slot >= (int)layer_slots(*r)) return fail(PBKD_EINVAL, "slot %d out of range for layer %d", slot, layer);
  float *pw0, *pw1, *pg, *pb;
  if (which == PBKD_STUDENT_GRAD) { pw0 = r->g_w0; pw1 = r->g_w1; pg = r->g_gamma; pb = r->g_beta; }
  else if (which == PBKD_STUDENT_MOMENTUM) { pw0 = r->v_w0; pw1 = r->v_w1; pg = r->v_gamma; pb = r->v_beta; }
  else if (which == PBKD_STUDENT_PARAM || which == PBKD_TEACHER_PARAM) { pw0 = r->w0; pw1 = r->w1; pg = r->gamma; pb = r->beta; }
  else return fail(PBKD_EINVAL, "unknown tensor kind %d", which);
  if (r->kind == PBKD_DWSEP3X3) {
    if (slot == 0) { *p = pw0; *n = r->n_w0; } else if (slot == 1) { *p = pw1; *n = r->n_w1; }
    else if (slot == 2) { *p = pg; *n = r->cout; } else { *p = pb; *n = r->cout; }
  } else {
    if (slot == 0) { *p = pw0; *n = r->n_w0; } else if (slot == 1) { *p = pg; *n = r->cout; } else { *p = pb; *n = r->cout; }
  }
  return PBKD_OK;
}

}  // namespace

// =================================================================================== C ABI

extern "C" {

const char *pbkd_last_error(void) { return g_err.c_str(); }

pbkd_status pbkd_arch_validate(const pbkd_arch_desc *teacher, const pbkd_arch_desc *student) {
  Net t, s;
  return validate_pair(teacher, student, t, s);
}

size_t pbkd_block_workspace_bytes(const pbkd_arch_desc *teacher, const pbkd_arch_desc *student) {
  pbkd_block b;
  if (validate_pair(teacher, student, b.t, b.s) != PBKD_OK) return 0;
  return layout(b, nullptr);
}

unsigned long long pbkd_arch_flops(const pbkd_arch_desc *arch, int training_step) {
  Net n;
  if (build_net(arch, training_step != 0, n) != PBKD_OK) return 0;
  return net_flops(n, training_step != 0);
}

unsigned long long pbkd_block_flops(const pbkd_block_t *blk, int which) {
  if (!blk) return 0;
  switch (which) {
    case 0: return net_flops(blk->t, false);
    case 1: return net_flops(blk->s, false);
    case 2: return net_flops(blk->s, true);
    case 3: return net_flops(blk->t, false) + net_flops(blk->s, true);
    default: return 0;
  }
}

pbkd_status pbkd_block_create(const pbkd_arch_desc *teacher, const float *const *tp, const pbkd_arch_desc *student,
                              const float *const *sp, const pbkd_train_desc *train, void *device_workspace,
                              size_t workspace_bytes, void *hip_stream, pbkd_block_t **out) {
  if (!out) return fail(PBKD_EINVAL, "null output handle");
  *out = nullptr;
  if (!tp || !sp || !train || !device_workspace) return fail(PBKD_EINVAL, "null argument");
  if (train->loss_reduction != 0 && train->loss_reduction != 1) return fail(PBKD_EINVAL, "loss_reduction must be 0 or 1");
  if (!(train->momentum >= 0.f && train->momentum < 1.f)) return fail(PBKD_EINVAL, "momentum must be in [0,1)");
  if (!(train->bn_decay >= 0.f && train->bn_decay < 1.f)) return fail(PBKD_EINVAL, "bn_decay must be in [0,1)");
  std::unique_ptr<pbkd_block> b(new pbkd_block());
  b->uid = g_next_uid.fetch_add(1);
  pbkd_status st = validate_pair(teacher, student, b->t, b->s);
  if (st != PBKD_OK) return st;
  if (reinterpret_cast<uintptr_t>(device_workspace) & 255) return fail(PBKD_ENOMEM, "workspace must be 256-byte aligned");
  const size_t need = layout(*b, static_cast<char *>(device_workspace));
  if (workspace_bytes < need) return fail(PBKD_ENOMEM, "workspace of %zu bytes is smaller than the %zu needed", workspace_bytes, need);
  copy_desc(teacher, b->t_layers);
  copy_desc(student, b->s_layers);
  b->momentum = train->momentum;
  b->loss_reduction = train->loss_reduction;
  b->t.bn_decay = b->s.bn_decay = train->bn_decay;
  b->ws = static_cast<char *>(device_workspace);
  b->ws_bytes = need;

  std::call_once(g_init_once, [] {
    g_init_err = init_conv_attributes();
    if (g_init_err == hipSuccess) g_init_err = init_pw_attributes();
    if (g_init_err == hipSuccess) g_init_err = init_pw_wgrad_attributes();
    if (g_init_err == hipSuccess) g_init_err = init_dwpw_attributes();
  });
  if (g_init_err != hipSuccess) return fail(PBKD_EHIP, "kernel attribute setup: %s", hipGetErrorString(g_init_err));

  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  auto upload = [&](Net &net, const float *const *src) -> pbkd_status {
    int k = 0;
    auto one = [&](LayerRT &r) -> pbkd_status {
      float *dst[4] = {r.w0, r.n_w1 ? r.w1 : r.gamma, r.n_w1 ? r.gamma : r.beta, r.beta};
      size_t cnt[4] = {r.n_w0, r.n_w1 ? r.n_w1 : (size_t)r.cout, (size_t)r.cout, (size_t)r.cout};
      const int ns = r.n_w1 ? 4 : 3;
      for (int i = 0; i < ns; ++i) {
        if (!src[k]) return fail(PBKD_EINVAL, "null parameter pointer at position %d", k);
        HIPCHK(hipMemcpyAsync(dst[i], src[k], cnt[i] * sizeof(float), hipMemcpyHostToDevice, s));
        ++k;
      }
      return PBKD_OK;
    };
    for (auto &r : net.L) { pbkd_status e = one(r); if (e != PBKD_OK) return e; }
    if (net.shortcut == 1) { pbkd_status e = one(net.sc); if (e != PBKD_OK) return e; }
    return PBKD_OK;
  };
  st = upload(b->t, tp);
  if (st != PBKD_OK) return st;
  st = upload(b->s, sp);
  if (st != PBKD_OK) return st;
  if (b->n_pk > 0x7fffffffull) return fail(PBKD_EUNSUPPORTED, "packed student weights exceed 2^31 floats");
  {
    // packed copies of every conv weight, and the arena -> packed index maps the optimizer uses
    auto pack_net = [&](Net &net, const float *const *src, bool student) -> pbkd_status {
      int k = 0;
      auto one = [&](LayerRT &r) -> pbkd_status {
        pbkd_status e;
        if (r.kind == PBKD_DWSEP3X3) { e = upload_packed_pointwise(r, src[k + 1], student, s); k += 4; }
        else { e = upload_packed(r, src[k], s); k += 3; }
        return e;
      };
      for (auto &r : net.L) { pbkd_status e = one(r); if (e != PBKD_OK) return e; }
      if (net.shortcut == 1) { pbkd_status e = one(net.sc); if (e != PBKD_OK) return e; }
      return PBKD_OK;
    };
    st = pack_net(b->t, tp, false);
    if (st != PBKD_OK) return st;
    st = pack_net(b->s, sp, true);
    if (st != PBKD_OK) return st;
    std::vector<int> mf(b->n_student, -1), mb(b->n_student, -1);
    auto maps = [&](LayerRT &r) {
      if (r.kind == PBKD_DWSEP3X3) {
        const size_t base = r.w1 - b->s_params, off_f = r.wpk - b->s_pk, off_b = r.wpk_b - b->s_pk;
        for (int o = 0; o < r.cout; ++o)
          for (int c = 0; c < r.cin; ++c) {
            mf[base + (size_t)o * r.cin + c] = (int)(off_f + pw_pack_index(r.pg, o, c));
            mb[base + (size_t)o * r.cin + c] = (int)(off_b + pw_pack_index(r.pdg, c, o));
          }
      } else {
        const size_t base = r.w0 - b->s_params, off_f = r.wpk - b->s_pk;
        for (int o = 0; o < r.cout; ++o)
          for (int c = 0; c < r.cin; ++c)
            for (int tap = 0; tap < r.taps; ++tap)
              mf[base + ((size_t)o * r.cin + c) * r.taps + tap] =
                  (int)(off_f + (r.taps == 9 ? conv_pack_index(r.cg, o, c, tap) : pw_pack_index(r.pg, o, c)));
      }
    };
    for (auto &r : b->s.L) maps(r);
    if (b->s.shortcut == 1) maps(b->s.sc);
    HIPCHK(hipMemcpyAsync(b->map_f, mf.data(), mf.size() * sizeof(int), hipMemcpyHostToDevice, s));
    HIPCHK(hipMemcpyAsync(b->map_b, mb.data(), mb.size() * sizeof(int), hipMemcpyHostToDevice, s));
    HIPCHK(hipStreamSynchronize(s));
  }
  {
    // running statistics start at mean 0, variance 1
    int cmax = 1;
    auto widest = [&](const Net &net) {
      for (const auto &r : net.L) cmax = std::max(cmax, r.cout);
      if (net.shortcut == 1) cmax = std::max(cmax, net.sc.cout);
    };
    widest(b->t); widest(b->s);
    const std::vector<float> ones((size_t)cmax, 1.f);
    auto start = [&](Net &net) -> pbkd_status {
      auto one = [&](LayerRT &r) -> pbkd_status {
        HIPCHK(hipMemsetAsync(r.rmean, 0, r.cout * sizeof(float), s));
        HIPCHK(hipMemcpyAsync(r.rvar, ones.data(), r.cout * sizeof(float), hipMemcpyHostToDevice, s));
        return PBKD_OK;
      };
      for (auto &r : net.L) { pbkd_status e = one(r); if (e != PBKD_OK) return e; }
      if (net.shortcut == 1) { pbkd_status e = one(net.sc); if (e != PBKD_OK) return e; }
      return PBKD_OK;
    };
    st = start(b->t);
    if (st != PBKD_OK) return st;
    st = start(b->s);
    if (st != PBKD_OK) return st;
    HIPCHK(hipStreamSynchronize(s));   // `ones` is a temporary
  }
  if (!b->jobs.empty()) {
    HIPCHK(hipMemcpyAsync(b->jobs_dev, b->jobs.data(), b->jobs.size() * sizeof(GradJob), hipMemcpyHostToDevice, s));
    HIPCHK(hipMemcpyAsync(b->job_of_block_dev, b->job_of_block.data(), b->job_of_block.size() * sizeof(int), hipMemcpyHostToDevice, s));
    HIPCHK(hipStreamSynchronize(s));
  }
  HIPCHK(hipMemsetAsync(b->s_mom, 0, b->n_student * sizeof(float), s));
  HIPCHK(hipMemsetAsync(b->s_grads, 0, b->n_student * sizeof(float), s));
  HIPCHK(hipMemsetAsync(b->loss_dev, 0, sizeof(float), s));
  HIPCHK(hipStreamSynchronize(s));
  HIPCHK(hipEventCreateWithFlags(&b->ev_teacher, hipEventDisableTiming));
  HIPCHK(hipEventCreateWithFlags(&b->ev_student, hipEventDisableTiming));
  for (auto &r : b->readers) HIPCHK(hipEventCreateWithFlags(&r.ev, hipEventDisableTiming));
  HIPCHK(hipEventCreateWithFlags(&b->ev_target_free, hipEventDisableTiming));
  HIPCHK(hipEventCreateWithFlags(&b->ev_fork, hipEventDisableTiming));
  for (auto &e : b->ev_step_done) HIPCHK(hipEventCreateWithFlags(&e, hipEventDisableTiming));
  b->ev_dz.assign(b->s.L.size(), nullptr);
  b->ev_wg.assign(b->s.L.size(), nullptr);
  for (size_t l = 0; l < b->s.L.size(); ++l) {
    HIPCHK(hipEventCreateWithFlags(&b->ev_dz[l], hipEventDisableTiming));
    HIPCHK(hipEventCreateWithFlags(&b->ev_wg[l], hipEventDisableTiming));
  }
  *out = b.release();
  return PBKD_OK;
}

pbkd_status pbkd_block_destroy(pbkd_block_t *blk) {
  if (!blk) return PBKD_OK;
  if (blk->ev_teacher) (void)hipEventDestroy(blk->ev_teacher);
  if (blk->ev_student) (void)hipEventDestroy(blk->ev_student);
  for (auto &r : blk->readers)
    if (r.ev) (void)hipEventDestroy(r.ev);
  if (blk->ev_target_free) (void)hipEventDestroy(blk->ev_target_free);
  if (blk->ev_fork) (void)hipEventDestroy(blk->ev_fork);
  for (hipEvent_t e : blk->ev_step_done) if (e) (void)hipEventDestroy(e);
  drop_graphs(*blk);
  for (hipEvent_t e : blk->ev_dz) if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : blk->ev_wg) if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : blk->prof.ev) (void)hipEventDestroy(e);
  delete blk;
  return PBKD_OK;
}

// Teacher forward on st; target_dev is only written by the last kernel, which waits for `target_free`
// (the previous reader of target_dev on another stream) when one is given.
namespace {
// Sets one of a network's mode flags for the length of a scope.
struct FlagScope {
  bool &f;
  FlagScope(bool &flag, bool on) : f(flag) { f = on; }
  ~FlagScope() { f = false; }
};

// Forward of one network (teacher or student) into out_dev.  running: BatchNorm with the running statistics.
pbkd_status net_forward_impl(pbkd_block_t *blk, Net &net, const float *x_dev, float *out_dev, hipStream_t st,
                             hipEvent_t out_free, bool running) {
  FlagScope mode(net.use_running, running);
  pbkd_status e = forward_net(net, x_dev, st, &blk->prof);
  if (e != PBKD_OK) return e;
  if (out_free) HIPCHK(hipStreamWaitEvent(st, out_free, 0));
  HeadArgs h = head_args(*blk, net, true, x_dev);
  h.out = out_dev;
  LAUNCH(&blk->prof, KK_HEAD_OUT, st, launch_head(0, h, st));
  return PBKD_OK;
}
}  // namespace

static pbkd_status teacher_forward_impl(pbkd_block_t *blk, const float *x_dev, float *target_dev, hipStream_t st,
                                        hipEvent_t target_free) {
  return net_forward_impl(blk, blk->t, x_dev, target_dev, st, target_free, false);
}

// ---- graph mode.  `issue` enqueues a step's launches on `origin` (and on the streams it forks to and joins again);
// in graph mode they are captured once per argument tuple and the executable graph is launched on `origin` instead.
// Capture is per thread and relaxed, so other threads (and their allocations) are not disturbed.  A step that would
// time its kernels, or that runs on the NULL stream (which cannot be captured), is issued as it is.
static pbkd_status run_step(pbkd_block &b, const StepGraph &key, hipStream_t origin, const std::function<pbkd_status()> &issue) {
  if (!b.graph_mode || origin == nullptr || b.prof.mask != 0) return issue();
  for (StepGraph &g : b.graphs)
    if (g.kind == key.kind && g.x == key.x && g.t == key.t && g.lr == key.lr && g.s0 == key.s0 && g.s1 == key.s1 && g.aux == key.aux) {
      HIPCHK(hipGraphLaunch(g.exec, origin));
      return PBKD_OK;
    }
  StepGraph g = key;
  HIPCHK(hipStreamBeginCapture(origin, hipStreamCaptureModeRelaxed));
  const pbkd_status e = issue();
  const hipError_t he = hipStreamEndCapture(origin, &g.graph);
  if (e != PBKD_OK) {
    if (he == hipSuccess && g.graph) (void)hipGraphDestroy(g.graph);
    return e;
  }
  if (he != hipSuccess) return fail(PBKD_EHIP, "hipStreamEndCapture: %s", hipGetErrorString(he));
  const hipError_t hi = hipGraphInstantiate(&g.exec, g.graph, nullptr, nullptr, 0);
  if (hi != hipSuccess) {
    (void)hipGraphDestroy(g.graph);
    return fail(PBKD_EHIP, "hipGraphInstantiate: %s", hipGetErrorString(hi));
  }
  if (b.graphs.size() >= kMaxStepGraphs) {
    (void)hipGraphExecDestroy(b.graphs.front().exec);
    (void)hipGraphDestroy(b.graphs.front().graph);
    b.graphs.erase(b.graphs.begin());
  }
  b.graphs.push_back(g);
  HIPCHK(hipGraphLaunch(g.exec, origin));
  return PBKD_OK;
}

pbkd_status pbkd_teacher_forward(pbkd_block_t *blk, const float *x_dev, float *target_dev, void *hip_stream) {
  if (!blk || !x_dev || !target_dev) return fail(PBKD_EINVAL, "null argument");
  if (misaligned16(x_dev) || misaligned16(target_dev)) return fail(PBKD_EINVAL, "device tensors must be 16-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  StepGraph key;
  key.kind = 2; key.x = x_dev; key.t = target_dev; key.s0 = st; key.s1 = st;
  return run_step(*blk, key, st, [&]() { return teacher_forward_impl(blk, x_dev, target_dev, st, nullptr); });
}

pbkd_status pbkd_student_forward(pbkd_block_t *blk, const float *x_dev, float *out_dev, void *hip_stream) {
  if (!blk || !x_dev || !out_dev) return fail(PBKD_EINVAL, "null argument");
  if (misaligned16(x_dev) || misaligned16(out_dev)) return fail(PBKD_EINVAL, "device tensors must be 16-byte aligned");
  return net_forward_impl(blk, blk->s, x_dev, out_dev, static_cast<hipStream_t>(hip_stream), nullptr, false);
}

// Student step on st.  The forward pass does not need the target: `target_ready` (if given) is waited for
// only before the loss kernel, and `target_free` (if given) is recorded after the last kernel reading it.
static pbkd_status student_step_impl(pbkd_block &b, const float *x_dev, const float *target_dev, float lr, hipStream_t st,
                                     hipEvent_t target_ready, hipEvent_t target_free) {
  Prof *pf = &b.prof;
  FlagScope track(b.s.track_running, true);   // this pass's batch statistics also move the running ones
  pbkd_status e = forward_net(b.s, x_dev, st, pf);
  if (e != PBKD_OK) return e;
  if (target_ready) HIPCHK(hipStreamWaitEvent(st, target_ready, 0));
  LayerRT &last = b.s.L.back();
  const double cnt = b.loss_reduction == 0 ? (double)b.s.n * b.s.last_c * b.s.out_h * b.s.out_w : (double)b.s.n;
  HeadArgs h = head_args(b, b.s, true, x_dev);
  h.t = target_dev;
  h.gscale = (float)(2.0 / cnt);
  h.partial = b.head_partial;
  h.n_blk = b.head_nblk;
  LAUNCH(pf, KK_HEAD_LOSS, st, launch_head(1, h, st));
  // the backward head kernel sums the loss kernel's partials itself when that is cheap; else (or with a
  // frozen last layer, which has no backward kernel) a small kernel does
  const bool fuse = last.trainable && (long long)b.head_nblk * b.head_nblk <= kDeferMaxReads;
  if (!fuse)
    LAUNCH(pf, KK_REDUCE, st, launch_head_finalize(b.head_partial, b.head_nblk, b.s.last_c, (float)(1.0 / cnt), last.g_gamma, last.g_beta, b.loss_dev, st));
  if (last.trainable) {
    h.pend = BnPending{}; h.pend_s = BnPending{};
    h.dz = b.gbuf((int)b.s.L.size() - 1); h.dgamma = last.g_gamma; h.dbeta = last.g_beta;
    if (fuse) {
      h.dgamma_out = last.g_gamma; h.dbeta_out = last.g_beta; h.loss_out = b.loss_dev; h.loss_scale = (float)(1.0 / cnt);
    } else {
      h.partial = nullptr;
    }
    LAUNCH(pf, KK_HEAD_BWD, st, launch_head(2, h, st));
  }
  if (target_free) HIPCHK(hipEventRecord(target_free, st));
  if (last.trainable) {
    e = student_backward(b, x_dev, st);
    if (e != PBKD_OK) return e;
    LAUNCH(pf, KK_SGD, st, launch_reduce_update(b.jobs_dev, b.job_of_block_dev, (int)b.job_of_block.size(), b.s_params, b.s_mom, b.s_grads,
                                                lr, b.momentum, b.map_f, b.map_b, b.s_pk, st));
  }
  b.last_stream = st;
  b.has_loss = true;
  return PBKD_OK;
}

// Teacher forward and student step of one block: on one stream in sequence, or on two with the student's forward
// pass beside the teacher.  cross_call: the eager two-stream form also lets the NEXT call's teacher start while this
// call's student is in its backward pass (an event outside any one call, so not for a captured step).
static pbkd_status issue_distill(pbkd_block &b, const float *x_dev, float *target_dev, float lr, hipStream_t ss, hipStream_t ts,
                                 bool cross_call) {
  pbkd_status e;
  if (ss == ts) {
    e = teacher_forward_impl(&b, x_dev, target_dev, ts, nullptr);
    if (e != PBKD_OK) return e;
    return student_step_impl(b, x_dev, target_dev, lr, ss, nullptr, nullptr);
  }
  if (!cross_call) {                 // fork from the student's stream, join at the loss kernel
    HIPCHK(hipEventRecord(b.ev_fork, ss));
    HIPCHK(hipStreamWaitEvent(ts, b.ev_fork, 0));
  }
  // Calls are issued ahead of the GPU, so this call's teacher starts as early as its dependencies allow: while the
  // student is still in the previous step's backward pass.  PBKD_TEACHER_LAG=1 holds it back until the student step
  // before the previous one has ended, so that it runs beside the previous step's forward pass instead (measured on
  // MI355X: 2-4 % faster on the CIFAR-sized blocks, 2 % slower on the ImageNet-sized one; off unless asked for).
  const bool lag = cross_call && env_is("PBKD_TEACHER_LAG", 1);
  hipEvent_t done = b.ev_step_done[b.step_count & 1];
  if (lag) HIPCHK(hipStreamWaitEvent(ts, done, 0));       // (recorded two calls ago; never recorded: no wait)
  // only the kernel that writes target_dev waits for the previous call's last reader of it
  e = teacher_forward_impl(&b, x_dev, target_dev, ts, cross_call ? b.ev_target_free : nullptr);
  if (e != PBKD_OK) return e;
  HIPCHK(hipEventRecord(b.ev_teacher, ts));
  e = student_step_impl(b, x_dev, target_dev, lr, ss, b.ev_teacher, cross_call ? b.ev_target_free : nullptr);
  if (e != PBKD_OK) return e;
  if (cross_call) {
    HIPCHK(hipEventRecord(done, ss));
    ++b.step_count;
  }
  return PBKD_OK;
}

static pbkd_status distill_step_any(pbkd_block &b, const float *x_dev, float *target_dev, float lr, hipStream_t ss, hipStream_t ts) {
  const bool graph = b.graph_mode && ss != nullptr && b.prof.mask == 0;
  StepGraph key;
  key.kind = 0; key.x = x_dev; key.t = target_dev; key.lr = lr; key.s0 = ss; key.s1 = ts; key.aux = b.aux;
  const pbkd_status e = run_step(b, key, ss, [&]() { return issue_distill(b, x_dev, target_dev, lr, ss, ts, !graph); });
  if (e != PBKD_OK) return e;
  b.last_stream = ss;
  b.has_loss = true;
  return PBKD_OK;
}

pbkd_status pbkd_student_step(pbkd_block_t *blk, const float *x_dev, const float *target_dev, float lr, float *loss_host,
                              void *hip_stream) {
  if (!blk || !x_dev || !target_dev) return fail(PBKD_EINVAL, "null argument");
  if (misaligned16(x_dev) || misaligned16(target_dev)) return fail(PBKD_EINVAL, "device tensors must be 16-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  pbkd_block &b = *blk;
  StepGraph key;
  key.kind = 1; key.x = x_dev; key.t = target_dev; key.lr = lr; key.s0 = st; key.s1 = st; key.aux = b.aux;
  pbkd_status e = run_step(b, key, st, [&]() { return student_step_impl(b, x_dev, target_dev, lr, st, nullptr, nullptr); });
  if (e != PBKD_OK) return e;
  b.last_stream = st;
  b.has_loss = true;
  if (loss_host) {
    HIPCHK(hipMemcpyAsync(loss_host, b.loss_dev, sizeof(float), hipMemcpyDeviceToHost, st));
    HIPCHK(hipStreamSynchronize(st));
  }
  return PBKD_OK;
}

pbkd_status pbkd_distill_step(pbkd_block_t *blk, const float *x_dev, float *target_dev, float lr, float *loss_host,
                              void *student_stream, void *teacher_stream) {
  if (!blk || !x_dev || !target_dev) return fail(PBKD_EINVAL, "null argument");
  if (misaligned16(x_dev) || misaligned16(target_dev)) return fail(PBKD_EINVAL, "device tensors must be 16-byte aligned");
  hipStream_t ss = static_cast<hipStream_t>(student_stream), ts = static_cast<hipStream_t>(teacher_stream);
  pbkd_block &b = *blk;
  pbkd_status e = distill_step_any(b, x_dev, target_dev, lr, ss, ts);
  if (e != PBKD_OK) return e;
  if (loss_host) {
    HIPCHK(hipMemcpyAsync(loss_host, b.loss_dev, sizeof(float), hipMemcpyDeviceToHost, ss));
    HIPCHK(hipStreamSynchronize(ss));
  }
  return PBKD_OK;
}

pbkd_status pbkd_block_set_graph_mode(pbkd_block_t *blk, int on) {
  if (!blk) return fail(PBKD_EINVAL, "null argument");
  blk->graph_mode = on != 0;
  if (!blk->graph_mode) drop_graphs(*blk);
  return PBKD_OK;
}

pbkd_status pbkd_block_set_aux_stream(pbkd_block_t *blk, void *aux_stream) {
  if (!blk) return fail(PBKD_EINVAL, "null argument");
  blk->aux = static_cast<hipStream_t>(aux_stream);
  drop_graphs(*blk);               // captured steps hold the old branch
  return PBKD_OK;
}

pbkd_status pbkd_block_last_loss(pbkd_block_t *blk, float *loss_host) {
  if (!blk || !loss_host) return fail(PBKD_EINVAL, "null argument");
  if (!blk->has_loss) return fail(PBKD_ESTATE, "no student step has run on this block yet");
  HIPCHK(hipMemcpyAsync(loss_host, blk->loss_dev, sizeof(float), hipMemcpyDeviceToHost, blk->last_stream));
  HIPCHK(hipStreamSynchronize(blk->last_stream));
  return PBKD_OK;
}

pbkd_status pbkd_schedule_blocks(int n_blocks, const unsigned long long *weights, pbkd_block_t *const *blocks, int n_streams,
                                 int policy, int *stream_of_block, int *order, unsigned long long *stream_load) {
  if (n_blocks < 0 || n_streams < 1) return fail(PBKD_EINVAL, "need n_blocks >= 0 and n_streams >= 1");
  if (n_blocks > 0 && (!stream_of_block || !order)) return fail(PBKD_EINVAL, "null output array");
  if (!weights && n_blocks > 0 && !blocks) return fail(PBKD_EINVAL, "either weights or block handles are required");
  if (policy != 0 && policy != 1) return fail(PBKD_EINVAL, "policy must be 0 (worst-fit-decreasing) or 1 (round robin)");
  std::vector<unsigned long long> w(n_blocks), load(n_streams, 0ull);
  std::vector<int> count(n_streams, 0);
  for (int i = 0; i < n_blocks; ++i) {
    if (weights) w[i] = weights[i];
    else {
      if (!blocks[i]) return fail(PBKD_EINVAL, "null block handle %d", i);
      w[i] = pbkd_block_flops(blocks[i], 3);
    }
  }
  if (policy == 1) {
    for (int i = 0; i < n_blocks; ++i) {
      const int s = i % n_streams;
      stream_of_block[i] = s; order[i] = count[s]++; load[s] += w[i];
    }
  } else {
    std::vector<int> idx(n_blocks);
    for (int i = 0; i < n_blocks; ++i) idx[i] = i;
    std::stable_sort(idx.begin(), idx.end(), [&](int a, int c) { return w[a] > w[c]; });
    for (int i : idx) {
      int best = 0;
      for (int s = 1; s < n_streams; ++s)
        if (load[s] < load[best]) best = s;
      stream_of_block[i] = best; order[i] = count[best]++; load[best] += w[i];
    }
  }
  if (stream_load)
    for (int s = 0; s < n_streams; ++s) stream_load[s] = load[s];
  return PBKD_OK;
}

// Notes that the block's student step just issued on `st` read x and t (see pbkd_block::readers).
static pbkd_status note_reader(pbkd_block &b, const void *x, const void *t, hipStream_t st) {
  pbkd_block::ReaderRec &rec = b.readers[b.reader_next];
  b.reader_next ^= 1;
  rec.x = x; rec.t = t; rec.used = true;
  HIPCHK(hipEventRecord(rec.ev, st));
  return PBKD_OK;
}

pbkd_status pbkd_distill_step_all(int n_blocks, pbkd_block_t *const *blocks, const float *const *x_dev, float *const *target_dev,
                                  float lr, int n_streams, void *const *streams, const int *stream_of_block, const int *order,
                                  int chain, void *teacher_stream) {
  if (n_blocks < 1 || !blocks || !x_dev || !target_dev || n_streams < 1 || !streams || !stream_of_block || !order)
    return fail(PBKD_EINVAL, "bad argument");
  for (int i = 0; i < n_blocks; ++i) {
    if (!blocks[i] || !x_dev[i] || !target_dev[i]) return fail(PBKD_EINVAL, "null entry %d", i);
    if (stream_of_block[i] < 0 || stream_of_block[i] >= n_streams) return fail(PBKD_EINVAL, "stream index of block %d out of range", i);
    if (chain && i > 0 && x_dev[i] != target_dev[i - 1]) return fail(PBKD_EINVAL, "chain: x_dev[%d] must be target_dev[%d]", i, i - 1);
  }
  // issue order of the student steps: by position within the stream, then by stream
  std::vector<int> issue(n_blocks);
  for (int i = 0; i < n_blocks; ++i) issue[i] = i;
  std::stable_sort(issue.begin(), issue.end(), [&](int a, int c) {
    return order[a] != order[c] ? order[a] < order[c] : stream_of_block[a] < stream_of_block[c];
  });
  hipStream_t ts = static_cast<hipStream_t>(teacher_stream);
  auto stream_of = [&](int i) { return static_cast<hipStream_t>(streams[stream_of_block[i]]); };

  // ---- graph mode (every block has it on): the whole step is one fork/join graph launched on `origin`
  hipStream_t origin = chain ? ts : stream_of(issue[0]);
  bool graph = origin != nullptr;
  for (int i = 0; i < n_blocks && graph; ++i) graph = blocks[i]->graph_mode && blocks[i]->prof.mask == 0 && !blocks[i]->aux;
  if (graph) {
    std::vector<unsigned long long> key;
    auto put = [&](const void *q) { key.push_back((unsigned long long)reinterpret_cast<uintptr_t>(q)); };
    key.push_back((unsigned long long)n_blocks);
    key.push_back((unsigned long long)(chain != 0));
    unsigned lrbits;
    std::memcpy(&lrbits, &lr, sizeof lrbits);
    key.push_back(lrbits);
    put(ts);
    for (int i = 0; i < n_blocks; ++i) {
      key.push_back(blocks[i]->uid); put(x_dev[i]); put(target_dev[i]); put(stream_of(i)); key.push_back((unsigned long long)order[i]);
      if (misaligned16(x_dev[i]) || misaligned16(target_dev[i])) return fail(PBKD_EINVAL, "device tensors must be 16-byte aligned");
    }
    pbkd_block &owner = *blocks[0];
    ScheduleGraph *hit = nullptr;
    for (ScheduleGraph &g : owner.schedule_graphs)
      if (g.key == key) { hit = &g; break; }
    if (!hit) {
      auto issue_all = [&]() -> pbkd_status {
        std::vector<hipStream_t> used;       // streams forked from origin, each with the event that ends its work
        std::vector<hipEvent_t> tail;
        auto fork_to = [&](hipStream_t st, hipEvent_t after) -> pbkd_status {
          if (st == origin) return PBKD_OK;
          HIPCHK(hipStreamWaitEvent(st, after, 0));
          return PBKD_OK;
        };
        auto note = [&](hipStream_t st, hipEvent_t ev) {
          for (size_t k = 0; k < used.size(); ++k)
            if (used[k] == st) { tail[k] = ev; return; }
          used.push_back(st); tail.push_back(ev);
        };
        if (chain) {
          for (int i = 0; i < n_blocks; ++i) {
            pbkd_status e = teacher_forward_impl(blocks[i], x_dev[i], target_dev[i], ts, nullptr);
            if (e != PBKD_OK) return e;
            HIPCHK(hipEventRecord(blocks[i]->ev_teacher, ts));
          }
          for (int i : issue) {
            hipStream_t st = stream_of(i);
            pbkd_status e = fork_to(st, blocks[i]->ev_teacher);
            if (e != PBKD_OK) return e;
            e = student_step_impl(*blocks[i], x_dev[i], target_dev[i], lr, st, nullptr, nullptr);
            if (e != PBKD_OK) return e;
            HIPCHK(hipEventRecord(blocks[i]->ev_student, st));
            note(st, blocks[i]->ev_student);
          }
        } else {
          HIPCHK(hipEventRecord(owner.ev_fork, origin));
          for (int i : issue) {
            hipStream_t st = stream_of(i);
            bool seen = st == origin;
            for (hipStream_t u : used) seen = seen || u == st;
            if (!seen) HIPCHK(hipStreamWaitEvent(st, owner.ev_fork, 0));
            pbkd_status e = teacher_forward_impl(blocks[i], x_dev[i], target_dev[i], st, nullptr);
            if (e != PBKD_OK) return e;
            e = student_step_impl(*blocks[i], x_dev[i], target_dev[i], lr, st, nullptr, nullptr);
            if (e != PBKD_OK) return e;
            HIPCHK(hipEventRecord(blocks[i]->ev_student, st));
            note(st, blocks[i]->ev_student);
          }
        }
        for (size_t k = 0; k < used.size(); ++k)
          if (used[k] != origin) HIPCHK(hipStreamWaitEvent(origin, tail[k], 0));
        return PBKD_OK;
      };
      ScheduleGraph g;
      g.key = key;
      HIPCHK(hipStreamBeginCapture(origin, hipStreamCaptureModeRelaxed));
      const pbkd_status e = issue_all();
      const hipError_t he = hipStreamEndCapture(origin, &g.graph);
      if (e != PBKD_OK) {
        if (he == hipSuccess && g.graph) (void)hipGraphDestroy(g.graph);
        return e;
      }
      if (he != hipSuccess) return fail(PBKD_EHIP, "hipStreamEndCapture: %s", hipGetErrorString(he));
      const hipError_t hi = hipGraphInstantiate(&g.exec, g.graph, nullptr, nullptr, 0);
      if (hi != hipSuccess) {
        (void)hipGraphDestroy(g.graph);
        return fail(PBKD_EHIP, "hipGraphInstantiate: %s", hipGetErrorString(hi));
      }
      if (owner.schedule_graphs.size() >= kMaxStepGraphs) {
        (void)hipGraphExecDestroy(owner.schedule_graphs.front().exec);
        (void)hipGraphDestroy(owner.schedule_graphs.front().graph);
        owner.schedule_graphs.erase(owner.schedule_graphs.begin());
      }
      owner.schedule_graphs.push_back(std::move(g));
      hit = &owner.schedule_graphs.back();
    }
    HIPCHK(hipGraphLaunch(hit->exec, origin));
    for (int i = 0; i < n_blocks; ++i) {
      blocks[i]->last_stream = origin; blocks[i]->has_loss = true;
      HIPCHK(hipEventRecord(blocks[i]->ev_student, origin));      // (outside the graph: what a later eager call waits for)
      const pbkd_status e = note_reader(*blocks[i], x_dev[i], target_dev[i], origin);
      if (e != PBKD_OK) return e;
    }
    return PBKD_OK;
  }

  if (chain) {
    for (int i = 0; i < n_blocks; ++i) {
      // target_dev[i] was read by block i's student (as target) and block i+1's (as input) in earlier calls: the
      // launch that overwrites it waits for those of their last two steps that used this very buffer
      for (int j = i; j <= i + 1 && j < n_blocks; ++j)
        for (const pbkd_block::ReaderRec &r : blocks[j]->readers)
          if (r.used && (r.t == target_dev[i] || r.x == target_dev[i])) HIPCHK(hipStreamWaitEvent(ts, r.ev, 0));
      pbkd_status e = pbkd_teacher_forward(blocks[i], x_dev[i], target_dev[i], ts);
      if (e != PBKD_OK) return e;
      HIPCHK(hipEventRecord(blocks[i]->ev_teacher, ts));
    }
    for (int i : issue) {
      hipStream_t st = stream_of(i);
      pbkd_block::ReaderRec &rec = blocks[i]->readers[blocks[i]->reader_next];
      blocks[i]->reader_next ^= 1;
      // the block's earlier steps are over before this one starts (no-ops on the stream they ran on; with a new stream
      // assignment they are what keeps two steps of one block apart, now that the teacher chain no longer waits for them)
      if (rec.used) HIPCHK(hipStreamWaitEvent(st, rec.ev, 0));
      HIPCHK(hipStreamWaitEvent(st, blocks[i]->ev_student, 0));
      HIPCHK(hipStreamWaitEvent(st, blocks[i]->ev_teacher, 0));
      pbkd_status e = pbkd_student_step(blocks[i], x_dev[i], target_dev[i], lr, nullptr, st);
      if (e != PBKD_OK) return e;
      HIPCHK(hipEventRecord(blocks[i]->ev_student, st));
      rec.x = x_dev[i]; rec.t = target_dev[i]; rec.used = true;
      HIPCHK(hipEventRecord(rec.ev, st));
    }
  } else {
    for (int i : issue) {
      hipStream_t st = stream_of(i);
      // the block's previous step may have run on another stream (a new assignment): wait for it (nothing to wait
      // for on the same stream)
      HIPCHK(hipStreamWaitEvent(st, blocks[i]->ev_student, 0));
      pbkd_status e = pbkd_teacher_forward(blocks[i], x_dev[i], target_dev[i], st);
      if (e != PBKD_OK) return e;
      e = pbkd_student_step(blocks[i], x_dev[i], target_dev[i], lr, nullptr, st);
      if (e != PBKD_OK) return e;
      HIPCHK(hipEventRecord(blocks[i]->ev_student, st));
      e = note_reader(*blocks[i], x_dev[i], target_dev[i], st);
      if (e != PBKD_OK) return e;
    }
  }
  return PBKD_OK;
}

pbkd_status pbkd_network_forward(int n_blocks, pbkd_block_t *const *blocks, const int *use_student, int bn_mode,
                                 const float *x_dev, float *const *outs_dev, void *hip_stream) {
  if (n_blocks < 1 || !blocks || !use_student || !x_dev || !outs_dev) return fail(PBKD_EINVAL, "bad argument");
  if (bn_mode != 0 && bn_mode != 1) return fail(PBKD_EINVAL, "bn_mode must be 0 (batch statistics) or 1 (running statistics)");
  if (misaligned16(x_dev)) return fail(PBKD_EINVAL, "device tensors must be 16-byte aligned");
  for (int k = 0; k < n_blocks; ++k) {
    if (!blocks[k] || !outs_dev[k]) return fail(PBKD_EINVAL, "null entry %d", k);
    if (k > 0) {
      const Net &prev = blocks[k - 1]->t, &cur = blocks[k]->t;
      if (cur.n != prev.n || cur.c != prev.last_c || cur.h != prev.out_h || cur.w != prev.out_w)
        return fail(PBKD_ESHAPE, "block %d does not take block %d's output as its input", k, k - 1);
    }
  }
  const float *in = x_dev;
  for (int k = 0; k < n_blocks; ++k) {
    if (misaligned16(outs_dev[k])) return fail(PBKD_EINVAL, "device tensors must be 16-byte aligned");
    const pbkd_status e = net_forward_impl(blocks[k], use_student[k] ? blocks[k]->s : blocks[k]->t, in, outs_dev[k],
                                           static_cast<hipStream_t>(hip_stream), nullptr, bn_mode == 1);
    if (e != PBKD_OK) return e;
    in = outs_dev[k];
  }
  return PBKD_OK;
}

pbkd_status pbkd_feature_mse(pbkd_block_t *blk, const float *a_dev, const float *b_dev, size_t n, double *mse_host,
                             void *hip_stream) {
  if (!blk || !a_dev || !b_dev || !mse_host || n == 0) return fail(PBKD_EINVAL, "bad argument");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  HIPCHK(launch_feature_mse(a_dev, b_dev, n, blk->mse_scratch, st));
  HIPCHK(hipMemcpyAsync(mse_host, blk->mse_scratch + 256, sizeof(double), hipMemcpyDeviceToHost, st));
  HIPCHK(hipStreamSynchronize(st));
  return PBKD_OK;
}

pbkd_status pbkd_feature_mse_noalloc(const float *a_dev, const float *b_dev, size_t n, double *mse_host, void *hip_stream) {
  if (!a_dev || !b_dev || !mse_host || n == 0) return fail(PBKD_EINVAL, "bad argument");
  if (n > PBKD_FEATURE_MSE_NOALLOC_MAX_N)
    return fail(PBKD_EINVAL, "pbkd_feature_mse_noalloc: %zu elements exceed the maximum of %llu", n,
                (unsigned long long)PBKD_FEATURE_MSE_NOALLOC_MAX_N);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  double *scratch_dev = nullptr;   // this GPU's copy of the library's static array
  HIPCHK(feature_mse_static_scratch(&scratch_dev));
  HIPCHK(launch_feature_mse(a_dev, b_dev, n, scratch_dev, st));
  HIPCHK(hipMemcpyAsync(mse_host, scratch_dev + 256, sizeof(double), hipMemcpyDeviceToHost, st));
  HIPCHK(hipStreamSynchronize(st));
  return PBKD_OK;
}

pbkd_status pbkd_select_blocks(int n_blocks, pbkd_block_t *const *blocks, int bn_mode, const float *x_dev,
                               float *const *teacher_outs_dev, float *const *scratch_outs_dev, double threshold,
                               int *use_student, double *block_err, double *final_err, void *hip_stream) {
  if (n_blocks < 1 || !blocks || !x_dev || !teacher_outs_dev || !scratch_outs_dev || !use_student)
    return fail(PBKD_EINVAL, "bad argument");
  if (!(threshold == threshold)) return fail(PBKD_EINVAL, "threshold is not a number");
  for (int k = 0; k < n_blocks; ++k)
    if (!blocks[k] || !teacher_outs_dev[k] || !scratch_outs_dev[k] || teacher_outs_dev[k] == scratch_outs_dev[k])
      return fail(PBKD_EINVAL, "bad entry %d", k);
  std::vector<int> mask((size_t)n_blocks, 0);
  // the teacher network once: its block outputs are every candidate's input and the reference features
  pbkd_status e = pbkd_network_forward(n_blocks, blocks, mask.data(), bn_mode, x_dev, teacher_outs_dev, hip_stream);
  if (e != PBKD_OK) return e;
  const Net &last = blocks[n_blocks - 1]->t;
  const size_t n_feat = (size_t)last.n * last.last_c * last.out_h * last.out_w;
  const float *ref = teacher_outs_dev[n_blocks - 1];
  for (int k = 0; k < n_blocks; ++k) {
    // the network with only block k replaced equals the teacher up to block k-1
    std::fill(mask.begin(), mask.end(), 0);
    mask[k] = 1;
    const float *in = k == 0 ? x_dev : teacher_outs_dev[k - 1];
    e = pbkd_network_forward(n_blocks - k, blocks + k, mask.data() + k, bn_mode, in, scratch_outs_dev + k, hip_stream);
    if (e != PBKD_OK) return e;
    double err = 0.0;
    e = pbkd_feature_mse(blocks[0], scratch_outs_dev[n_blocks - 1], ref, n_feat, &err, hip_stream);
    if (e != PBKD_OK) return e;
    if (block_err) block_err[k] = err;
    use_student[k] = err < threshold ? 1 : 0;
  }
  if (final_err) {
    e = pbkd_network_forward(n_blocks, blocks, use_student, bn_mode, x_dev, scratch_outs_dev, hip_stream);
    if (e != PBKD_OK) return e;
    e = pbkd_feature_mse(blocks[0], scratch_outs_dev[n_blocks - 1], ref, n_feat, final_err, hip_stream);
    if (e != PBKD_OK) return e;
  }
  return PBKD_OK;
}

pbkd_status pbkd_run_tasks_work_stealing(int n_tasks, pbkd_block_t *const *blocks, const float *const *x_dev,
                                         float *const *target_dev, float lr, const int *steps, int n_streams,
                                         void *const *streams, const int *queue_of_task, int *ran_on, int *n_steals) {
  if (n_tasks < 1 || !blocks || !x_dev || !target_dev || !steps || n_streams < 1 || !streams || !queue_of_task)
    return fail(PBKD_EINVAL, "bad argument");
  for (int i = 0; i < n_tasks; ++i) {
    if (!blocks[i] || !x_dev[i] || !target_dev[i] || steps[i] < 0) return fail(PBKD_EINVAL, "bad task %d", i);
    if (queue_of_task[i] < 0 || queue_of_task[i] >= n_streams) return fail(PBKD_EINVAL, "queue index of task %d out of range", i);
    if (misaligned16(x_dev[i]) || misaligned16(target_dev[i])) return fail(PBKD_EINVAL, "device tensors must be 16-byte aligned");
  }
  std::vector<std::deque<int>> queue(n_streams);
  for (int i = 0; i < n_tasks; ++i) queue[queue_of_task[i]].push_back(i);
  std::vector<hipEvent_t> done(n_tasks, nullptr);
  std::vector<std::deque<int>> inflight(n_streams);   // tasks issued to a stream and not yet seen finished
  pbkd_status rc = PBKD_OK;
  int remaining = n_tasks, steals = 0;
  auto issue = [&](int t, int w) -> pbkd_status {
    hipStream_t st = static_cast<hipStream_t>(streams[w]);
    pbkd_status e = PBKD_OK;
    for (int k = 0; k < steps[t] && e == PBKD_OK; ++k) {
      e = pbkd_teacher_forward(blocks[t], x_dev[t], target_dev[t], st);
      if (e == PBKD_OK) e = pbkd_student_step(blocks[t], x_dev[t], target_dev[t], lr, nullptr, st);
    }
    if (e != PBKD_OK) return e;
    HIPCHK(hipEventCreateWithFlags(&done[t], hipEventDisableTiming));
    HIPCHK(hipEventRecord(done[t], st));
    inflight[w].push_back(t);
    if (ran_on) ran_on[t] = w;
    return PBKD_OK;
  };
  while (remaining > 0 && rc == PBKD_OK) {
    bool progressed = false;
    for (int w = 0; w < n_streams && rc == PBKD_OK; ++w) {
      while (!inflight[w].empty()) {
        const hipError_t q = hipEventQuery(done[inflight[w].front()]);
        if (q == hipSuccess) {
          inflight[w].pop_front();
        } else {
          (void)hipGetLastError();   // "not ready" is not an error
          break;
        }
      }
      int t = -1;
      if (!queue[w].empty()) {
        if (inflight[w].size() < 2) {          // one task running, one queued behind it keeps the stream fed
          t = queue[w].front();
          queue[w].pop_front();
        }
      } else if (inflight[w].empty()) {        // out of work: steal from the tail of the longest queue
        int victim = -1;
        for (int v = 0; v < n_streams; ++v)
          if (!queue[v].empty() && (victim < 0 || queue[v].size() > queue[victim].size())) victim = v;
        if (victim >= 0) {
          t = queue[victim].back();
          queue[victim].pop_back();
          ++steals;
        }
      }
      if (t >= 0) {
        rc = issue(t, w);
        --remaining;
        progressed = true;
      }
    }
    if (!progressed) std::this_thread::yield();
  }
  for (int i = 0; i < n_tasks; ++i)
    if (done[i]) {
      if (hipEventSynchronize(done[i]) != hipSuccess && rc == PBKD_OK) rc = fail(PBKD_EHIP, "hipEventSynchronize failed");
      (void)hipEventDestroy(done[i]);
    }
  if (n_steals) *n_steals = steals;
  return rc;
}

int pbkd_kernel_kinds(void) { return KK_COUNT; }

const char *pbkd_kernel_kind_name(int kind) { return (kind >= 0 && kind < KK_COUNT) ? kKindNames[kind] : ""; }

pbkd_status pbkd_block_profile_enable(pbkd_block_t *blk, unsigned kind_mask, int capacity) {
  if (!blk || capacity < 0) return fail(PBKD_EINVAL, "bad argument");
  Prof &p = blk->prof;
  HIPCHK(hipDeviceSynchronize());
  p.mask = capacity ? kind_mask : 0u;
  p.used = 0;
  while (p.ev.size() < 2 * (size_t)capacity) {
    hipEvent_t e;
    HIPCHK(hipEventCreate(&e));
    p.ev.push_back(e);
  }
  p.cap = (size_t)capacity;
  p.kind.assign(p.cap, 0);
  return PBKD_OK;
}

pbkd_status pbkd_block_profile_read(pbkd_block_t *blk, int n_kinds, double *ms_sum, int *launches) {
  if (!blk || !ms_sum || !launches || n_kinds < KK_COUNT) return fail(PBKD_EINVAL, "bad argument (need arrays of pbkd_kernel_kinds() entries)");
  Prof &p = blk->prof;
  for (int k = 0; k < n_kinds; ++k) { ms_sum[k] = 0.0; launches[k] = 0; }
  for (size_t i = 0; i < p.used; ++i) {
    HIPCHK(hipEventSynchronize(p.ev[2 * i + 1]));
    float ms = 0.f;
    HIPCHK(hipEventElapsedTime(&ms, p.ev[2 * i], p.ev[2 * i + 1]));
    ms_sum[p.kind[i]] += (double)ms;
    launches[p.kind[i]] += 1;
  }
  p.used = 0;
  return PBKD_OK;
}

pbkd_status pbkd_block_get_tensor(pbkd_block_t *blk, int which, int layer, int slot, float *host_out, size_t n) {
  if (!blk || !host_out) return fail(PBKD_EINVAL, "null argument");
  float *p = nullptr;
  size_t cnt = 0;
  pbkd_status e = tensor_ptr(blk, which, layer, slot, &p, &cnt);
  if (e != PBKD_OK) return e;
  if (cnt != n) return fail(PBKD_ESHAPE, "tensor has %zu floats, caller passed %zu", cnt, n);
  HIPCHK(hipDeviceSynchronize());
  HIPCHK(hipMemcpy(host_out, p, n * sizeof(float), hipMemcpyDeviceToHost));
  return PBKD_OK;
}

pbkd_status pbkd_block_set_tensor(pbkd_block_t *blk, int which, int layer, int slot, const float *host_in, size_t n) {
  if (!blk || !host_in) return fail(PBKD_EINVAL, "null argument");
  if (which == PBKD_STUDENT_ACT || which == PBKD_TEACHER_ACT || which == PBKD_STUDENT_GRAD)
    return fail(PBKD_EINVAL, "activations and gradients are read-only");
  float *p = nullptr;
  size_t cnt = 0;
  pbkd_status e = tensor_ptr(blk, which, layer, slot, &p, &cnt);
  if (e != PBKD_OK) return e;
  if (cnt != n) return fail(PBKD_ESHAPE, "tensor has %zu floats, caller passed %zu", cnt, n);
  HIPCHK(hipDeviceSynchronize());
  HIPCHK(hipMemcpy(p, host_in, n * sizeof(float), hipMemcpyHostToDevice));
  if (which == PBKD_TEACHER_PARAM || which == PBKD_STUDENT_PARAM) {
    // keep the packed copies of conv weights in step with the canonical tensor
    const bool student = which == PBKD_STUDENT_PARAM;
    Net &net = student ? blk->s : blk->t;
    LayerRT &r = (layer < (int)net.L.size()) ? net.L[layer] : net.sc;
    if (r.kind == PBKD_DWSEP3X3 && slot == 1) {
      e = upload_packed_pointwise(r, host_in, student, nullptr);
      if (e != PBKD_OK) return e;
    } else if (r.kind != PBKD_DWSEP3X3 && slot == 0) {
      e = upload_packed(r, host_in, nullptr);
      if (e != PBKD_OK) return e;
    }
    HIPCHK(hipDeviceSynchronize());
  }
  return PBKD_OK;
}

}  // extern "C"
