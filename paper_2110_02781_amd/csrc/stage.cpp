// Model description, stage object and the C ABI entry points for
// forward / loss / backward / update / weight stashing / profiling.
//
// A stage executes its units as a fixed sequence of kernel launches on the
// caller's stream.  Every convolution writes its raw output z once; the
// following BatchNorm is reduced to a per-channel scale/shift that the NEXT
// kernel applies on load together with the activation ("view"), so activated
// tensors are never written except at block outputs (where the residual is
// added) and at the stage boundary.  Backward mirrors this: per convolution a
// reduction for d(gamma), d(beta), one elementwise pass that forms dz, then
// weight- and data-gradient kernels.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/ftp.h"
#include "kernels.h"

using namespace ftp;

// ------------------------------------------------------------------ errors
static thread_local char g_err[512] = "";
void ftp_set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}
extern "C" const char* ftp_last_error(void) { return g_err; }

#define HIP_TRY(expr)                                                              \
  do {                                                                             \
    hipError_t e_ = (expr);                                                        \
    if (e_ != hipSuccess) {                                                        \
      ftp_set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
      return FTP_ERR_HIP;                                                          \
    }                                                                              \
  } while (0)

static const float kBnEps = 1e-5f, kBnMomentum = 0.1f;

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline int conv_out(int n, int k, int s, int p) { return (n + 2 * p - k) / s + 1; }

// ------------------------------------------------------------------- model
enum SubType { SUB_DIRECT = 0, SUB_PW = 1, SUB_DW = 2 };

struct Sub {           // convolution + BatchNorm + activation
  int type;
  ConvGeom g;          // N filled in per stage
  int act;
  size_t w_off, w_n;   // offsets relative to the unit's parameter vector
  size_t gamma_off, beta_off;
  size_t bn_off;       // channel offset relative to the unit's BatchNorm channels
};

struct UnitInfo {
  ftp_unit_desc d;
  int inH, inW, inC, outH, outW, outC;
  std::vector<Sub> subs;
  bool residual;
  size_t n_param, n_bn;
};

struct ftp_model {
  std::vector<UnitInfo> units;
  int dtype;
  int inH, inW, inC;
};

static int build_unit(const ftp_unit_desc& d, int H, int W, int C, int idx, UnitInfo* u) {
  u->d = d;
  u->inH = H; u->inW = W; u->inC = C;
  u->residual = false;
  u->n_param = 0; u->n_bn = 0;
  auto add_sub = [&](int type, int Hin, int Win, int Cin, int Cout, int kh, int kw, int s, int ph, int pw, int act) {
    Sub sb;
    sb.type = type;
    sb.g = ConvGeom{0, Hin, Win, Cin, conv_out(Hin, kh, s, ph), conv_out(Win, kw, s, pw), Cout, kh, kw, s, ph, pw};
    sb.act = act;
    sb.w_off = u->n_param;
    sb.w_n = (size_t)Cout * kh * kw * (type == SUB_DW ? 1 : Cin);
    sb.gamma_off = sb.w_off + sb.w_n;
    sb.beta_off = sb.gamma_off + Cout;
    sb.bn_off = u->n_bn;
    u->n_param = sb.beta_off + Cout;
    u->n_bn += Cout;
    u->subs.push_back(sb);
    return sb;
  };
  switch (d.kind) {
    case FTP_UNIT_CONV: {
      if (d.cin != C || d.cout < 8 || d.cout % 8 || d.kh < 1 || d.kw < 1 || d.stride < 1 || d.pad_h < 0 || d.pad_w < 0 ||
          d.act < 0 || d.act > 2) {
        ftp_set_error("unit %d (CONV): cin=%d must equal incoming channels %d, cout=%d a multiple of 8", idx, d.cin, C, d.cout);
        return FTP_ERR_SHAPE;
      }
      if (H + 2 * d.pad_h < d.kh || W + 2 * d.pad_w < d.kw) { ftp_set_error("unit %d: kernel larger than padded input", idx); return FTP_ERR_SHAPE; }
      bool pw = d.kh == 1 && d.kw == 1 && d.stride == 1 && d.pad_h == 0 && d.pad_w == 0 && C % 8 == 0;
      Sub sb = add_sub(pw ? SUB_PW : SUB_DIRECT, H, W, C, d.cout, d.kh, d.kw, d.stride, d.pad_h, d.pad_w, d.act);
      if (!pw && !conv_direct_supported(sb.g)) {
        ftp_set_error("unit %d: dense %dx%d conv with cin*cout=%d > 8192 is not supported", idx, d.kh, d.kw, C * d.cout);
        return FTP_ERR_UNSUPPORTED;
      }
      u->outH = sb.g.Hout; u->outW = sb.g.Wout; u->outC = d.cout;
      break;
    }
    case FTP_UNIT_INVRES: {
      if (d.cin != C || C % 8 || d.cout < 8 || d.cout % 8 || d.expand < 1 || (d.stride != 1 && d.stride != 2)) {
        ftp_set_error("unit %d (INVRES): cin=%d must equal incoming channels %d; channels multiples of 8; stride 1 or 2", idx, d.cin, C);
        return FTP_ERR_SHAPE;
      }
      int ce = C * d.expand;
      // the depthwise kernels address inside one image with 32-bit offsets formed from 24-bit factors
      if ((size_t)H * W >= ((size_t)1 << 24) || (size_t)H * W * ce >= ((size_t)1 << 31) || ce >= (1 << 24)) {
        ftp_set_error("unit %d (INVRES): a %dx%dx%d expanded feature map is beyond the depthwise kernels' in-image offsets "
                      "(H*W < 2^24 and H*W*C < 2^31)", idx, H, W, ce);
        return FTP_ERR_UNSUPPORTED;
      }
      if (d.expand != 1) add_sub(SUB_PW, H, W, C, ce, 1, 1, 1, 0, 0, FTP_ACT_RELU6);
      Sub dw = add_sub(SUB_DW, H, W, ce, ce, 3, 3, d.stride, 1, 1, FTP_ACT_RELU6);
      add_sub(SUB_PW, dw.g.Hout, dw.g.Wout, ce, d.cout, 1, 1, 1, 0, 0, FTP_ACT_NONE);
      u->outH = dw.g.Hout; u->outW = dw.g.Wout; u->outC = d.cout;
      u->residual = d.stride == 1 && d.cin == d.cout;
      break;
    }
    case FTP_UNIT_GAP:
      if (C % 8) { ftp_set_error("unit %d (GAP): channels must be a multiple of 8", idx); return FTP_ERR_SHAPE; }
      u->outH = 1; u->outW = 1; u->outC = C;
      break;
    case FTP_UNIT_FC:
      if (H != 1 || W != 1 || d.cin != C || d.cout < 1 || C % 8) {
        ftp_set_error("unit %d (FC): needs a [batch,1,1,%d] input with cin %% 8 == 0 (got %dx%dx%d)", idx, d.cin, H, W, C);
        return FTP_ERR_SHAPE;
      }
      u->n_param = (size_t)d.cout * C + d.cout;
      u->outH = 1; u->outW = 1; u->outC = d.cout;
      break;
    case FTP_UNIT_LOSS:
      if (H != 1 || W != 1 || d.cin != C) { ftp_set_error("unit %d (LOSS): needs [batch,1,1,classes] logits", idx); return FTP_ERR_SHAPE; }
      u->outH = 1; u->outW = 1; u->outC = C;
      break;
    default:
      ftp_set_error("unit %d: unknown kind %d", idx, d.kind);
      return FTP_ERR_ARG;
  }
  if (u->outH < 1 || u->outW < 1) { ftp_set_error("unit %d: empty output", idx); return FTP_ERR_SHAPE; }
  return FTP_OK;
}

extern "C" int ftp_model_create(const ftp_unit_desc* units, int L, int in_h, int in_w, int in_c, ftp_dtype act_dtype,
                                ftp_model** out) {
  if (!units || !out || L < 1 || in_h < 1 || in_w < 1 || in_c < 1 || (act_dtype != FTP_F32 && act_dtype != FTP_BF16)) {
    ftp_set_error("model_create: bad argument");
    return FTP_ERR_ARG;
  }
  ftp_model* m = new (std::nothrow) ftp_model();
  if (!m) { ftp_set_error("model_create: out of host memory"); return FTP_ERR_NOMEM; }
  m->dtype = (int)act_dtype;
  m->inH = in_h; m->inW = in_w; m->inC = in_c;
  int H = in_h, W = in_w, C = in_c;
  for (int i = 0; i < L; ++i) {
    UnitInfo u;
    int rc = build_unit(units[i], H, W, C, i, &u);
    if (rc != FTP_OK) { delete m; return rc; }
    if (units[i].kind == FTP_UNIT_LOSS && i + 1 != L) { ftp_set_error("unit %d: LOSS must be the last unit", i); delete m; return FTP_ERR_SHAPE; }
    if (units[i].kind == FTP_UNIT_LOSS && i > 0 && units[i - 1].kind == FTP_UNIT_CONV) {
      ftp_set_error("unit %d: LOSS may not directly follow a CONV unit", i); delete m; return FTP_ERR_SHAPE;
    }
    H = u.outH; W = u.outW; C = u.outC;
    m->units.push_back(u);
  }
  *out = m;
  return FTP_OK;
}

extern "C" void ftp_model_destroy(ftp_model* m) { delete m; }
extern "C" int ftp_model_num_units(const ftp_model* m) { return m ? (int)m->units.size() : FTP_ERR_ARG; }

extern "C" int ftp_model_unit_in_shape(const ftp_model* m, int u, int* h, int* w, int* c) {
  if (!m || u < 0 || u > (int)m->units.size() || !h || !w || !c) { ftp_set_error("unit_in_shape: bad argument"); return FTP_ERR_ARG; }
  if (u == (int)m->units.size()) { const UnitInfo& x = m->units.back(); *h = x.outH; *w = x.outW; *c = x.outC; }
  else { const UnitInfo& x = m->units[u]; *h = x.inH; *w = x.inW; *c = x.inC; }
  return FTP_OK;
}
extern "C" int ftp_model_unit_param_count(const ftp_model* m, int u, size_t* n) {
  if (!m || u < 0 || u >= (int)m->units.size() || !n) { ftp_set_error("unit_param_count: bad argument"); return FTP_ERR_ARG; }
  *n = m->units[u].n_param;
  return FTP_OK;
}
extern "C" int ftp_model_unit_bn_channels(const ftp_model* m, int u, size_t* n) {
  if (!m || u < 0 || u >= (int)m->units.size() || !n) { ftp_set_error("unit_bn_channels: bad argument"); return FTP_ERR_ARG; }
  *n = m->units[u].n_bn;
  return FTP_OK;
}

// -------------------------------------------------------------------- stage
struct UnitPlan {
  const UnitInfo* info;
  size_t p_off;                    // float offset of the unit's parameters in the flat buffers
  size_t bn_off;                   // channel offset in the running-stat arrays
  std::vector<size_t> z_off;       // per sub: byte offset of z in the slot stash
  std::vector<size_t> st_off;      // per sub: float offset of mean|invstd|scale|shift in the slot stats
  size_t out_off;                  // byte offset of the materialised unit output (if any)
  bool out_virtual;                // CONV unit whose output stays a view
  size_t in_mat_off;               // residual block fed by a view: materialised copy of its input
  bool need_in_mat;
};

struct Slot {
  char* stash = nullptr;     // intermediates; with recomputation all slots point at the stage's one shared stash
  char* xin_keep = nullptr;  // recomputation: the slot's own copy of its stage input
  float* stats = nullptr;
  float* snap_w = nullptr;   // fp32 parameter snapshot
  int timer_idx = -1;        // ring entry of the batch in this slot when execution timing is on
  void* snap_lp = nullptr;   // bfloat16 working-copy snapshot
  void* dlogits = nullptr;
  bool busy = false, has_snap = false, has_loss = false;
};

struct ProfEvents {          // optional per-unit timing (profile_layers)
  std::vector<hipEvent_t> f0, f1, b0, b1;
};

// Optional per-batch execution time of the stage (the online profiling that feeds the capacity estimate):
// a ring of event quadruples, one per forwarded batch, harvested by ftp_stage_timing_read.
struct ExecTimer {
  enum { kRing = 256 };
  hipEvent_t ev[kRing][4];       // forward begin/end, backward begin/end
  bool bwd_done[kRing];
  int used = 0;                  // entries handed out since the last read
  bool created = false;
};

struct ftp_stage {
  const ftp_model* model;
  int a, b, batch, dt, device;
  size_t es;
  std::vector<UnitPlan> plan;
  size_t n_param = 0, n_bn = 0;
  float *params = nullptr, *grads = nullptr, *mom = nullptr, *run_mean = nullptr, *run_var = nullptr;
  void* w_lp = nullptr;
  size_t stash_bytes = 0, stats_floats = 0, xin_bytes = 0, max_act_bytes = 0;
  std::vector<Slot> slots;
  char *gbuf[5] = {nullptr, nullptr, nullptr, nullptr, nullptr};   // boundary A/B, dz (even), dA, dz (odd)
  // Weight gradients depend on nothing downstream, so in backward they run on a second stream next to the
  // data-gradient chain: fork after dz is formed, join before that dz buffer is overwritten / at the end.
  hipStream_t side = nullptr;
  // fork / join of the side stream: one pair per dz buffer, and a third for the partial sums of the one-pass expand backward
  hipEvent_t ev_fork[3] = {nullptr, nullptr, nullptr}, ev_join[3] = {nullptr, nullptr, nullptr};
  bool join_pending[3] = {false, false, false};
  // Weight gradients of an inverted-residual unit whose tensors are small (kernels of 10 - 40 us): an event record
  // between two kernels of a stream costs about 3 us and a wait for a recent event of the other stream about 2 (both
  // measured), per layer as much as a finalize kernel.  Such a unit forks ONCE, behind its last layer: its layers write
  // their dz into a set of three buffers of their own (two sets, alternating from unit to unit), the weight gradients
  // are noted and all enqueued on the side stream at the end of the unit.
  struct PendingWgrad { int type; const void* dz; HView in; ConvGeom g; size_t M; float* gw; };
  PendingWgrad pend[3];
  int n_pend = 0;
  char* dzring[6] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
  size_t dzring_bytes = 0;
  hipEvent_t ev_bfork[2] = {nullptr, nullptr}, ev_bjoin[2] = {nullptr, nullptr};
  bool bjoin_pending[2] = {false, false};
  int bset = 0;
  bool bset_open = false;      // a layer of the current unit has written into the set
  unsigned n_sub_bwd = 0;
  float *bn_part = nullptr, *coef = nullptr, *ws = nullptr, *row_loss = nullptr;
  // A second partial-sum workspace for the weight gradient of the stage's very first layer when the stage forks
  // its weight gradients: that layer has no data gradient, so nothing follows it on the caller's stream and it
  // runs there, next to whatever the side stream still has queued, instead of behind it.
  float* ws_tail = nullptr;
  size_t ws_tail_floats = 0;
  // partial sums of the one-pass backward of the expand layers: it runs on the caller's stream while the side stream
  // may be using ws, so it has a workspace of its own
  float* ws_fused = nullptr;
  size_t ws_fused_floats = 0;
  int n_direct = 0;           // sublayers that use the patch-matrix buffer
  void* im2col = nullptr;     // patch matrix for the weight gradient of small dense convolutions
  // The conv output whose input patches the buffer holds right now (nullptr: none).  A forward that goes through the
  // patch matrix leaves it behind; if nothing has used the buffer since, the weight gradient of the same layer and
  // slot takes it as it is instead of writing the same matrix again.
  const void* im2col_of = nullptr;
  // The gradient tensor whose BatchNorm-backward partial sums bn_part holds already (left there by the depthwise data
  // gradient that produced it), and how many partials; nullptr: none.
  const void* bwd_sums_of = nullptr;
  int bwd_sums_P = 0;
  size_t im2col_elems = 0;
  size_t ws_floats = 0;
  int max_c = 0;
  bool has_loss = false;
  int classes = 0;
  ProfEvents* prof = nullptr;
  ExecTimer* timer = nullptr;   // non-null while execution timing is enabled
  // Recomputation: slots keep only their stage input; the intermediates of the batch whose forward ran last
  // live in one shared stash, and a backward of any other slot first runs the forward again.
  bool recompute = false;
  char* shared_stash = nullptr;
  int stash_owner = -1;         // slot whose intermediates the shared stash holds
  float bn_mom = kBnMomentum;   // 0 while a forward is being recomputed: running statistics stay put
  size_t dev_bytes = 0;         // device memory the stage allocated
};

static inline void dfree(void* p) { if (p) (void)hipFree(p); }

static void stage_free(ftp_stage* s) {
  if (!s) return;
  dfree(s->params); dfree(s->grads); dfree(s->mom); dfree(s->run_mean); dfree(s->run_var); dfree(s->w_lp);
  for (auto& sl : s->slots) { if (!s->recompute) dfree(sl.stash); dfree(sl.xin_keep); dfree(sl.stats); dfree(sl.snap_w); dfree(sl.snap_lp); dfree(sl.dlogits); }
  dfree(s->shared_stash);
  for (int i = 0; i < 5; ++i) dfree(s->gbuf[i]);
  if (s->side) (void)hipStreamDestroy(s->side);
  for (int i = 0; i < 3; ++i) {
    if (s->ev_fork[i]) (void)hipEventDestroy(s->ev_fork[i]);
    if (s->ev_join[i]) (void)hipEventDestroy(s->ev_join[i]);
  }
  for (int i = 0; i < 2; ++i) {
    if (s->ev_bfork[i]) (void)hipEventDestroy(s->ev_bfork[i]);
    if (s->ev_bjoin[i]) (void)hipEventDestroy(s->ev_bjoin[i]);
  }
  for (int i = 0; i < 6; ++i) dfree(s->dzring[i]);
  dfree(s->bn_part); dfree(s->coef); dfree(s->ws); dfree(s->ws_tail); dfree(s->ws_fused); dfree(s->row_loss); dfree(s->im2col);
  if (s->timer) {
    if (s->timer->created)
      for (auto& q : s->timer->ev)
        for (auto& e : q) (void)hipEventDestroy(e);
    delete s->timer;
  }
  delete s;
}

extern "C" void ftp_stage_destroy(ftp_stage* s) { stage_free(s); }

static thread_local size_t g_alloc_total = 0;

template <typename P>
static int dev_alloc(P** p, size_t bytes) {
  void* q = nullptr;
  hipError_t e = hipMalloc(&q, align_up(bytes ? bytes : 1, 256));
  if (e != hipSuccess) { ftp_set_error("hipMalloc(%zu bytes) failed: %s", bytes, hipGetErrorString(e)); return FTP_ERR_NOMEM; }
  *p = (P*)q;
  g_alloc_total += align_up(bytes ? bytes : 1, 256);
  return FTP_OK;
}

extern "C" int ftp_stage_create_ex(const ftp_model* m, int a, int b, int batch, int n_slots, unsigned flags, ftp_stage** out) {
  if (!m || !out) { ftp_set_error("stage_create: NULL argument"); return FTP_ERR_ARG; }
  if (flags & ~(unsigned)FTP_STAGE_RECOMPUTE) { ftp_set_error("stage_create: unknown flags 0x%x", flags); return FTP_ERR_ARG; }
  int L = (int)m->units.size();
  if (a < 0 || a >= b || b > L) { ftp_set_error("stage_create: bad unit range [%d,%d) for %d units", a, b, L); return FTP_ERR_ARG; }
  if (batch < 1 || n_slots < 1 || n_slots > 64) { ftp_set_error("stage_create: batch >= 1 and 1 <= n_slots <= 64 required"); return FTP_ERR_ARG; }
  ftp_stage* s = new (std::nothrow) ftp_stage();
  if (!s) { ftp_set_error("stage_create: out of host memory"); return FTP_ERR_NOMEM; }
  s->model = m; s->a = a; s->b = b; s->batch = batch; s->dt = m->dtype;
  s->recompute = (flags & FTP_STAGE_RECOMPUTE) != 0;
  g_alloc_total = 0;
  s->es = m->dtype == FTP_F32 ? 4 : 2;
  if (hipGetDevice(&s->device) != hipSuccess) { ftp_set_error("stage_create: no HIP device"); delete s; return FTP_ERR_HIP; }

  size_t stash = 0, stats = 0, max_act = 0, ws_floats = 1024;
  int max_c = 8;
  auto act_bytes = [&](int H, int W, int C) { return align_up((size_t)batch * H * W * C * s->es, 256); };
  const UnitInfo& first = m->units[a];
  s->xin_bytes = act_bytes(first.inH, first.inW, first.inC);
  stash += s->xin_bytes;
  max_act = s->xin_bytes;
  for (int i = a; i < b; ++i) {
    const UnitInfo& u = m->units[i];
    UnitPlan p;
    p.info = &u;
    p.p_off = s->n_param; s->n_param += align_up(u.n_param, 8);
    p.bn_off = s->n_bn; s->n_bn += u.n_bn;
    for (const Sub& sb : u.subs) {
      size_t zb = act_bytes(sb.g.Hout, sb.g.Wout, sb.g.Cout);
      p.z_off.push_back(stash); stash += zb;
      p.st_off.push_back(stats); stats += (size_t)4 * sb.g.Cout;
      if (zb > max_act) max_act = zb;
      size_t ib = act_bytes(sb.g.Hin, sb.g.Win, sb.g.Cin);
      if (ib > max_act) max_act = ib;
      if (sb.g.Cout > max_c) max_c = sb.g.Cout;
      ConvGeom g = sb.g; g.N = batch;
      size_t M = (size_t)batch * g.Hout * g.Wout;
      size_t need = sb.type == SUB_DIRECT ? conv_direct_wgrad_ws(g) : sb.type == SUB_DW ? dw_wgrad_ws(g) : pw_wgrad_ws(M, g.Cin, g.Cout);
      if (need > ws_floats) ws_floats = need;
      if (i == a && &sb == &u.subs[0]) s->ws_tail_floats = need;
      if (sb.type == SUB_PW && m->dtype == FTP_BF16 && pw_bwd_fused_ws(M, g.Cin, g.Cout) > s->ws_fused_floats)
        s->ws_fused_floats = pw_bwd_fused_ws(M, g.Cin, g.Cout);
      if (sb.type == SUB_DIRECT) ++s->n_direct;
      if (sb.type == SUB_DIRECT && conv_direct_gemm_ok(g) && conv_direct_gemm_wpad_elems(g) > ws_floats)
        ws_floats = conv_direct_gemm_wpad_elems(g);      // padded weight copy of the GEMM forward (at most 4 bytes each)
      if (sb.type == SUB_DIRECT && conv_direct_im2col_elems(g) > s->im2col_elems) s->im2col_elems = conv_direct_im2col_elems(g);
      if (sb.type == SUB_DIRECT && conv_direct_dgrad_gemm_ok(g)) {
        if (conv_direct_dgrad_gemm_im2col_elems(g) > s->im2col_elems) s->im2col_elems = conv_direct_dgrad_gemm_im2col_elems(g);
        if (conv_direct_dgrad_gemm_w_elems(g) > ws_floats) ws_floats = conv_direct_dgrad_gemm_w_elems(g);
      }
    }
    p.out_virtual = (u.d.kind == FTP_UNIT_CONV);
    p.out_off = 0;
    if (!p.out_virtual && u.d.kind != FTP_UNIT_LOSS) {
      size_t ob = act_bytes(u.outH, u.outW, u.outC);
      p.out_off = stash; stash += ob;
      if (ob > max_act) max_act = ob;
    }
    p.need_in_mat = u.residual && i > a && m->units[i - 1].d.kind == FTP_UNIT_CONV;
    p.in_mat_off = 0;
    if (p.need_in_mat) { p.in_mat_off = stash; stash += act_bytes(u.inH, u.inW, u.inC); }
    if (u.d.kind == FTP_UNIT_FC) {
      size_t need = pw_wgrad_ws((size_t)batch, u.inC, u.outC);
      if (need > ws_floats) ws_floats = need;
    }
    if (u.d.kind == FTP_UNIT_LOSS) { s->has_loss = true; s->classes = u.inC; }
    s->plan.push_back(p);
  }
  s->stash_bytes = stash; s->stats_floats = stats; s->max_act_bytes = max_act; s->ws_floats = ws_floats; s->max_c = max_c;

  int rc = FTP_OK;
  size_t np = s->n_param ? s->n_param : 8;
  size_t nb = s->n_bn ? s->n_bn : 8;
  if ((rc = dev_alloc(&s->params, np * 4)) || (rc = dev_alloc(&s->grads, np * 4)) || (rc = dev_alloc(&s->mom, np * 4)) ||
      (rc = dev_alloc(&s->run_mean, nb * 4)) || (rc = dev_alloc(&s->run_var, nb * 4))) { stage_free(s); return rc; }
  if (s->dt == FTP_BF16 && (rc = dev_alloc(&s->w_lp, np * 2))) { stage_free(s); return rc; }
  s->slots.resize(n_slots);
  if (s->recompute && (rc = dev_alloc(&s->shared_stash, stash))) { stage_free(s); return rc; }
  for (auto& sl : s->slots) {
    if (s->recompute) {
      sl.stash = s->shared_stash;
      if ((rc = dev_alloc(&sl.xin_keep, s->xin_bytes))) { stage_free(s); return rc; }
    } else if ((rc = dev_alloc(&sl.stash, stash))) { stage_free(s); return rc; }
    if ((rc = dev_alloc(&sl.stats, (stats ? stats : 8) * 4)) ||
        (rc = dev_alloc(&sl.snap_w, np * 4))) { stage_free(s); return rc; }
    if (s->dt == FTP_BF16 && (rc = dev_alloc(&sl.snap_lp, np * 2))) { stage_free(s); return rc; }
    if (s->has_loss && (rc = dev_alloc(&sl.dlogits, (size_t)batch * s->classes * s->es))) { stage_free(s); return rc; }
  }
  for (int i = 0; i < 5; ++i)
    if ((rc = dev_alloc(&s->gbuf[i], max_act))) { stage_free(s); return rc; }
  {
    hipError_t e = hipStreamCreateWithFlags(&s->side, hipStreamNonBlocking);     // default priority
    for (int i = 0; i < 3 && e == hipSuccess; ++i) {
      e = hipEventCreateWithFlags(&s->ev_fork[i], hipEventDisableTiming);
      if (e == hipSuccess) e = hipEventCreateWithFlags(&s->ev_join[i], hipEventDisableTiming);
    }
    for (int i = 0; i < 2 && e == hipSuccess; ++i) {
      e = hipEventCreateWithFlags(&s->ev_bfork[i], hipEventDisableTiming);
      if (e == hipSuccess) e = hipEventCreateWithFlags(&s->ev_bjoin[i], hipEventDisableTiming);
    }
    if (e != hipSuccess) { ftp_set_error("stage_create: stream/event creation failed: %s", hipGetErrorString(e)); stage_free(s); return FTP_ERR_HIP; }
  }
  if (s->max_act_bytes >= ((size_t)32 << 20)) {        // a stage that forks (stage_forks)
    s->dzring_bytes = max_act < ((size_t)64 << 20) ? max_act : ((size_t)64 << 20);
    for (int i = 0; i < 6; ++i)
      if ((rc = dev_alloc(&s->dzring[i], s->dzring_bytes))) { stage_free(s); return rc; }
  }
  if ((rc = dev_alloc(&s->bn_part, (size_t)kBnPartials * 2 * max_c * 4)) || (rc = dev_alloc(&s->coef, (size_t)3 * max_c * 4)) ||
      (rc = dev_alloc(&s->ws, ws_floats * 4)) || (rc = dev_alloc(&s->row_loss, (size_t)batch * 4))) { stage_free(s); return rc; }
  if (s->im2col_elems && (rc = dev_alloc(&s->im2col, s->im2col_elems * s->es))) { stage_free(s); return rc; }
  if (s->ws_fused_floats && (rc = dev_alloc(&s->ws_fused, s->ws_fused_floats * 4))) { stage_free(s); return rc; }
  if (s->max_act_bytes >= ((size_t)32 << 20) && s->ws_tail_floats && s->n_direct <= 1 &&
      (rc = dev_alloc(&s->ws_tail, s->ws_tail_floats * 4))) { stage_free(s); return rc; }

  // initial state: zero weights / momentum / gradients, running mean 0, running variance 1
  std::vector<float> ones(nb, 1.0f);
  hipError_t e = hipMemset(s->params, 0, np * 4);
  if (e == hipSuccess) e = hipMemset(s->grads, 0, np * 4);
  if (e == hipSuccess) e = hipMemset(s->mom, 0, np * 4);
  if (e == hipSuccess) e = hipMemset(s->run_mean, 0, nb * 4);
  if (e == hipSuccess) e = hipMemcpy(s->run_var, ones.data(), nb * 4, hipMemcpyHostToDevice);
  if (e == hipSuccess && s->w_lp) e = hipMemset(s->w_lp, 0, np * 2);
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) { ftp_set_error("stage_create: initialisation failed: %s", hipGetErrorString(e)); stage_free(s); return FTP_ERR_HIP; }
  s->dev_bytes = g_alloc_total;
  *out = s;
  return FTP_OK;
}

extern "C" int ftp_stage_create(const ftp_model* m, int a, int b, int batch, int n_slots, ftp_stage** out) {
  return ftp_stage_create_ex(m, a, b, batch, n_slots, 0u, out);
}

extern "C" int ftp_stage_device_bytes(const ftp_stage* s, size_t* bytes) {
  if (!s || !bytes) { ftp_set_error("stage_device_bytes: NULL argument"); return FTP_ERR_ARG; }
  *bytes = s->dev_bytes;
  return FTP_OK;
}

// ---- parameter import / export ------------------------------------------------
static int unit_check(const ftp_stage* s, int unit, size_t n, size_t expect, const void* p, const char* who) {
  if (!s || !p) { ftp_set_error("%s: NULL argument", who); return FTP_ERR_ARG; }
  if (unit < s->a || unit >= s->b) { ftp_set_error("%s: unit %d outside the stage [%d,%d)", who, unit, s->a, s->b); return FTP_ERR_ARG; }
  if (n != expect) { ftp_set_error("%s: unit %d has %zu values, caller passed %zu", who, unit, expect, n); return FTP_ERR_SHAPE; }
  return FTP_OK;
}

extern "C" int ftp_stage_import_weights(ftp_stage* s, int unit, const float* host_w, size_t n) {
  int rc = unit_check(s, unit, n, s ? (unit >= s->a && unit < s->b ? s->plan[unit - s->a].info->n_param : 0) : 0, host_w, "import_weights");
  if (rc) return rc;
  if (n == 0) return FTP_OK;
  const UnitPlan& p = s->plan[unit - s->a];
  HIP_TRY(hipMemcpy(s->params + p.p_off, host_w, n * 4, hipMemcpyHostToDevice));
  if (s->w_lp) {
    f32_to_storage(FTP_BF16, nullptr, s->params + p.p_off, (char*)s->w_lp + p.p_off * 2, n);
    HIP_TRY(hipGetLastError());
  if (const char* why = launch_plan_failure_take()) { ftp_set_error("%s", why); return FTP_ERR_UNSUPPORTED; }
    HIP_TRY(hipDeviceSynchronize());
  }
  return FTP_OK;
}

static int export_from(const ftp_stage* s, const float* base, int unit, float* host, size_t n, const char* who) {
  int rc = unit_check(s, unit, n, s ? (unit >= s->a && unit < s->b ? s->plan[unit - s->a].info->n_param : 0) : 0, host, who);
  if (rc) return rc;
  if (n == 0) return FTP_OK;
  HIP_TRY(hipDeviceSynchronize());
  HIP_TRY(hipMemcpy(host, base + s->plan[unit - s->a].p_off, n * 4, hipMemcpyDeviceToHost));
  return FTP_OK;
}
extern "C" int ftp_stage_export_weights(const ftp_stage* s, int unit, float* h, size_t n) { return export_from(s, s ? s->params : nullptr, unit, h, n, "export_weights"); }
extern "C" int ftp_stage_export_grads(const ftp_stage* s, int unit, float* h, size_t n) { return export_from(s, s ? s->grads : nullptr, unit, h, n, "export_grads"); }
extern "C" int ftp_stage_export_momentum(const ftp_stage* s, int unit, float* h, size_t n) { return export_from(s, s ? s->mom : nullptr, unit, h, n, "export_momentum"); }

extern "C" int ftp_stage_export_bn_stats(const ftp_stage* s, int unit, float* host, size_t n) {
  int rc = unit_check(s, unit, n, s ? (unit >= s->a && unit < s->b ? 2 * s->plan[unit - s->a].info->n_bn : 0) : 0, host, "export_bn_stats");
  if (rc) return rc;
  if (n == 0) return FTP_OK;
  const UnitPlan& p = s->plan[unit - s->a];
  HIP_TRY(hipDeviceSynchronize());
  // per BatchNorm: running_mean then running_var
  size_t o = 0;
  for (const Sub& sb : p.info->subs) {
    size_t C = sb.g.Cout;
    HIP_TRY(hipMemcpy(host + o, s->run_mean + p.bn_off + sb.bn_off, C * 4, hipMemcpyDeviceToHost));
    HIP_TRY(hipMemcpy(host + o + C, s->run_var + p.bn_off + sb.bn_off, C * 4, hipMemcpyDeviceToHost));
    o += 2 * C;
  }
  return FTP_OK;
}

static int inspect_check_owner(const ftp_stage* s, int slot, const char* who) {
  if (s->recompute && s->stash_owner != slot) {
    ftp_set_error("%s: with recomputation only the slot forwarded (or recomputed) last has intermediates, not slot %d", who, slot);
    return FTP_ERR_SLOT;
  }
  return FTP_OK;
}
static int inspect_check(const ftp_stage* s, int slot, int unit, int conv, const void* host, const char* who) {
  if (!s || !host) { ftp_set_error("%s: NULL argument", who); return FTP_ERR_ARG; }
  if (slot < 0 || slot >= (int)s->slots.size()) { ftp_set_error("%s: slot %d out of range", who, slot); return FTP_ERR_ARG; }
  if (unit < s->a || unit >= s->b) { ftp_set_error("%s: unit %d outside the stage [%d,%d)", who, unit, s->a, s->b); return FTP_ERR_ARG; }
  if (conv < 0 || conv >= (int)s->plan[unit - s->a].info->subs.size()) { ftp_set_error("%s: unit %d has no convolution %d", who, unit, conv); return FTP_ERR_ARG; }
  if (!s->slots[slot].busy) { ftp_set_error("%s: slot %d holds no forwarded batch", who, slot); return FTP_ERR_SLOT; }
  return FTP_OK;
}

extern "C" int ftp_stage_export_conv_output(const ftp_stage* s, int slot, int unit, int conv, float* host_z, size_t n) {
  int rc = inspect_check(s, slot, unit, conv, host_z, "export_conv_output");
  if (!rc) rc = inspect_check_owner(s, slot, "export_conv_output");
  if (rc) return rc;
  const UnitPlan& p = s->plan[unit - s->a];
  const Sub& sb = p.info->subs[conv];
  size_t expect = (size_t)s->batch * sb.g.Hout * sb.g.Wout * sb.g.Cout;
  if (n != expect) { ftp_set_error("export_conv_output: tensor has %zu values, caller passed %zu", expect, n); return FTP_ERR_SHAPE; }
  HIP_TRY(hipDeviceSynchronize());
  const char* src = s->slots[slot].stash + p.z_off[conv];
  if (s->dt == FTP_F32) {
    HIP_TRY(hipMemcpy(host_z, src, n * 4, hipMemcpyDeviceToHost));
  } else {
    std::vector<uint16_t> tmp(n);
    HIP_TRY(hipMemcpy(tmp.data(), src, n * 2, hipMemcpyDeviceToHost));
    for (size_t i = 0; i < n; ++i) { uint32_t u = (uint32_t)tmp[i] << 16; memcpy(&host_z[i], &u, 4); }
  }
  return FTP_OK;
}

extern "C" int ftp_stage_export_bn_batch_stats(const ftp_stage* s, int slot, int unit, int conv, float* host_s, size_t n) {
  int rc = inspect_check(s, slot, unit, conv, host_s, "export_bn_batch_stats");
  if (rc) return rc;
  const UnitPlan& p = s->plan[unit - s->a];
  size_t expect = (size_t)4 * p.info->subs[conv].g.Cout;
  if (n != expect) { ftp_set_error("export_bn_batch_stats: %zu values, caller passed %zu", expect, n); return FTP_ERR_SHAPE; }
  HIP_TRY(hipDeviceSynchronize());
  HIP_TRY(hipMemcpy(host_s, s->slots[slot].stats + p.st_off[conv], n * 4, hipMemcpyDeviceToHost));
  return FTP_OK;
}

// ---- helpers for the compute calls ------------------------------------------------
struct WeightSet { const float* w32; const char* lp; };

static inline const void* conv_w(const ftp_stage* s, const WeightSet& ws, size_t off) {
  return s->dt == FTP_F32 ? (const void*)(ws.w32 + off) : (const void*)(ws.lp + off * 2);
}

static int check_call(ftp_stage* s, int slot, const char* who) {
  if (!s) { ftp_set_error("%s: NULL stage", who); return FTP_ERR_ARG; }
  if (slot < 0 || slot >= (int)s->slots.size()) { ftp_set_error("%s: slot %d out of range (n_slots=%zu)", who, slot, s->slots.size()); return FTP_ERR_ARG; }
  return FTP_OK;
}

static HView plain(const void* p) { return HView{p, nullptr, nullptr, 0}; }

// Input view of every unit and of every convolution inside it, from the slot's buffers.
struct Views {
  std::vector<HView> unit_in;                 // per unit
  std::vector<std::vector<HView>> sub_out;    // per unit, per sub
};

static void build_views(const ftp_stage* s, const Slot& sl, Views* v) {
  HView cur = plain(sl.stash);                // stashed stage input at offset 0
  size_t n = s->plan.size();
  v->unit_in.resize(n);
  v->sub_out.resize(n);
  for (size_t i = 0; i < n; ++i) {
    const UnitPlan& p = s->plan[i];
    if (p.need_in_mat) cur = plain(sl.stash + p.in_mat_off);
    v->unit_in[i] = cur;
    for (size_t k = 0; k < p.info->subs.size(); ++k) {
      const Sub& sb = p.info->subs[k];
      float* st = sl.stats + p.st_off[k];
      v->sub_out[i].push_back(HView{sl.stash + p.z_off[k], st + 2 * sb.g.Cout, st + 3 * sb.g.Cout, sb.act});
    }
    if (p.out_virtual) cur = v->sub_out[i].back();
    else if (p.info->d.kind != FTP_UNIT_LOSS) cur = plain(sl.stash + p.out_off);
  }
}

// pend (in/out): on entry the unfinished BatchNorm of `in` (partial == nullptr: none); on exit, when
// defer is set and the statistics of this layer were left as partial sums, their description
static void sub_forward(ftp_stage* s, Slot& sl, const UnitPlan& p, size_t k, HView in, const WeightSet& W, hipStream_t st,
                        BnPending* pend = nullptr, bool defer = false) {
  const Sub& sb = p.info->subs[k];
  ConvGeom g = sb.g; g.N = s->batch;
  void* z = sl.stash + p.z_off[k];
  const void* w = conv_w(s, W, p.p_off + sb.w_off);
  size_t M = (size_t)s->batch * g.Hout * g.Wout;
  int P = 0;
  float* stt = sl.stats + p.st_off[k];
  int C = g.Cout;
  if (s->im2col_of == z) s->im2col_of = nullptr;     // this layer's input is a new one: patches kept from before are stale
  const float* gamma = W.w32 + p.p_off + sb.gamma_off;
  const float* beta = W.w32 + p.p_off + sb.beta_off;
  float* rm = s->run_mean + p.bn_off + sb.bn_off;
  float* rv = s->run_var + p.bn_off + sb.bn_off;
  if (sb.type == SUB_DW && dw_fwd_bn_small_ok(g)) {
    BnPending none{};
    dw_fwd_bn_small(s->dt, st, in, pend ? *pend : none, w, g, gamma, beta, stt, stt + C, stt + 2 * C, stt + 3 * C, rm, rv, kBnEps,
                    s->bn_mom, z);
    if (pend) pend->partial = nullptr;
    return;
  }
  if (sb.type == SUB_PW) {
    pw_fwd(s->dt, st, in, w, nullptr, M, g.Cin, g.Cout, z, s->bn_part, &P);   // statistics in the epilogue
    if (defer && pend) {
      *pend = BnPending{s->bn_part, P, M, gamma, beta, stt, stt + C, stt + 2 * C, stt + 3 * C, rm, rv};
      return;
    }
  } else if (sb.type == SUB_DIRECT && conv_direct_gemm_ok(g) && s->im2col &&
             conv_direct_gemm_wpad_elems(g) * s->es <= s->ws_floats * sizeof(float)) {
    // the float workspace is free during a forward: the padded weight copy lives there
    conv_direct_fwd_gemm(s->dt, st, in, w, g, s->im2col, s->ws, z, s->bn_part, &P);
    s->im2col_of = z;
  } else {
    if (sb.type == SUB_DW && dw_fwd_stats_ok(s->dt, g)) {
      dw_fwd(s->dt, st, in, w, g, z, s->bn_part, &P);           // few tiles: their sums are the partials
    } else {
      if (sb.type == SUB_DW) dw_fwd(s->dt, st, in, w, g, z);
      else conv_direct_fwd(s->dt, st, in, w, g, z);
      bn_stats(s->dt, st, z, M, g.Cout, s->bn_part, &P);
    }
  }
  bn_finalize(st, s->bn_part, P, M, C, gamma, beta, stt, stt + C, stt + 2 * C, stt + 3 * C, rm, rv, kBnEps, s->bn_mom);
}

// every unit of the stage over the input at offset 0 of the slot's stash, with the weights W
static int forward_units(ftp_stage* s, Slot& sl, const Views& v, const WeightSet& W, hipStream_t st) {
  for (size_t i = 0; i < s->plan.size(); ++i) {
    const UnitPlan& p = s->plan[i];
    const UnitInfo& u = *p.info;
    if (s->prof) HIP_TRY(hipEventRecord(s->prof->f0[i], st));
    if (p.need_in_mat) {
      // the previous CONV unit's output, materialised so the residual can read it
      HView prev = v.sub_out[i - 1].back();
      bn_apply(s->dt, st, prev, (size_t)s->batch * u.inH * u.inW, u.inC, nullptr, sl.stash + p.in_mat_off);
    }
    HView in = v.unit_in[i];
    switch (u.d.kind) {
      case FTP_UNIT_CONV:
        sub_forward(s, sl, p, 0, in, W, st);
        break;
      case FTP_UNIT_INVRES: {
        HView h = in;
        BnPending pend{};
        for (size_t k = 0; k < u.subs.size(); ++k) {
          // an expand layer in front of a short depthwise layer leaves its statistics to that layer's kernel
          bool defer = false;
          if (k + 1 < u.subs.size() && u.subs[k].type == SUB_PW && u.subs[k + 1].type == SUB_DW) {
            ConvGeom gn = u.subs[k + 1].g; gn.N = s->batch;
            defer = dw_fwd_bn_small_ok(gn) && (size_t)s->batch * u.subs[k].g.Hout * u.subs[k].g.Wout <= 16 * 128;
          }
          // ... and the project layer leaves them to the kernel that writes the block output
          const size_t Mo = (size_t)s->batch * u.outH * u.outW;
          if (k + 1 == u.subs.size() && u.subs[k].type == SUB_PW) defer = bn_finalize_apply_small_ok(Mo, u.outC) != 0;
          sub_forward(s, sl, p, k, h, W, st, &pend, defer);
          h = v.sub_out[i][k];
        }
        if (pend.partial) {
          bn_finalize_apply_small(s->dt, st, pend, h.z, (size_t)s->batch * u.outH * u.outW, u.outC, h.act, kBnEps, s->bn_mom,
                                  u.residual ? in.z : nullptr, sl.stash + p.out_off);
          pend.partial = nullptr;
        } else {
          bn_apply(s->dt, st, h, (size_t)s->batch * u.outH * u.outW, u.outC, u.residual ? in.z : nullptr, sl.stash + p.out_off);
        }
        break;
      }
      case FTP_UNIT_GAP:
        gap_fwd(s->dt, st, in, s->batch, u.inH * u.inW, u.inC, sl.stash + p.out_off);
        break;
      case FTP_UNIT_FC:
        pw_fwd(s->dt, st, in, conv_w(s, W, p.p_off), W.w32 + p.p_off + (size_t)u.outC * u.inC, (size_t)s->batch, u.inC,
               u.outC, sl.stash + p.out_off, nullptr, nullptr);
        break;
      default:
        break;  // LOSS: evaluated by ftp_stage_loss
    }
    if (s->prof) HIP_TRY(hipEventRecord(s->prof->f1[i], st));
  }
  return FTP_OK;
}

extern "C" int ftp_stage_forward(ftp_stage* s, int slot, const void* x_dev, void* y_dev, void* stream) {
  int rc = check_call(s, slot, "stage_forward");
  if (rc) return rc;
  if (!x_dev) { ftp_set_error("stage_forward: x_dev is NULL"); return FTP_ERR_ARG; }
  Slot& sl = s->slots[slot];
  if (sl.busy) { ftp_set_error("stage_forward: slot %d is busy (its backward has not run)", slot); return FTP_ERR_SLOT; }
  hipStream_t st = (hipStream_t)stream;
  const UnitInfo& first = *s->plan[0].info;
  size_t xin = (size_t)s->batch * first.inH * first.inW * first.inC * s->es;
  sl.timer_idx = -1;
  if (s->timer && s->timer->used < ExecTimer::kRing) {
    sl.timer_idx = s->timer->used++;
    s->timer->bwd_done[sl.timer_idx] = false;
    HIP_TRY(hipEventRecord(s->timer->ev[sl.timer_idx][0], st));
  }
  HIP_TRY(hipMemcpyAsync(sl.stash, x_dev, xin, hipMemcpyDeviceToDevice, st));
  if (s->recompute) {
    HIP_TRY(hipMemcpyAsync(sl.xin_keep, x_dev, xin, hipMemcpyDeviceToDevice, st));
    s->stash_owner = slot;
  }
  Views v;
  build_views(s, sl, &v);
  WeightSet W{s->params, (const char*)s->w_lp};
  if ((rc = forward_units(s, sl, v, W, st))) return rc;
  if (y_dev) {
    size_t li = s->plan.size() - 1;
    const UnitPlan& p = s->plan[li];
    const UnitInfo& u = *p.info;
    size_t M = (size_t)s->batch * u.outH * u.outW;
    if (p.out_virtual) {
      bn_apply(s->dt, st, v.sub_out[li].back(), M, u.outC, nullptr, y_dev);
    } else {
      const void* src = u.d.kind == FTP_UNIT_LOSS ? v.unit_in[li].z : (const void*)(sl.stash + p.out_off);
      HIP_TRY(hipMemcpyAsync(y_dev, src, M * u.outC * s->es, hipMemcpyDeviceToDevice, st));
    }
  }
  if (s->timer && sl.timer_idx >= 0) HIP_TRY(hipEventRecord(s->timer->ev[sl.timer_idx][1], st));
  HIP_TRY(hipGetLastError());
  if (const char* why = launch_plan_failure_take()) { ftp_set_error("%s", why); return FTP_ERR_UNSUPPORTED; }
  sl.busy = true; sl.has_snap = false; sl.has_loss = false;
  return FTP_OK;
}

extern "C" int ftp_stage_loss(ftp_stage* s, int slot, const int32_t* labels_dev, float* loss_dev, void* stream) {
  int rc = check_call(s, slot, "stage_loss");
  if (rc) return rc;
  if (!s->has_loss) { ftp_set_error("stage_loss: the stage does not end with the LOSS unit"); return FTP_ERR_ARG; }
  if (!labels_dev || !loss_dev) { ftp_set_error("stage_loss: NULL argument"); return FTP_ERR_ARG; }
  Slot& sl = s->slots[slot];
  if (!sl.busy) { ftp_set_error("stage_loss: slot %d holds no forwarded batch", slot); return FTP_ERR_SLOT; }
  if (s->recompute && s->stash_owner != slot) {
    ftp_set_error("stage_loss: with recomputation the loss of slot %d has to follow its forward directly (the logits are gone)", slot);
    return FTP_ERR_SLOT;
  }
  hipStream_t st = (hipStream_t)stream;
  Views v;
  build_views(s, sl, &v);
  size_t li = s->plan.size() - 1;
  if (s->prof) HIP_TRY(hipEventRecord(s->prof->f0[li], st));
  softmax_ce(s->dt, st, v.unit_in[li].z, labels_dev, s->batch, s->classes, s->row_loss, sl.dlogits, loss_dev);
  if (s->prof) HIP_TRY(hipEventRecord(s->prof->f1[li], st));
  HIP_TRY(hipGetLastError());
  if (const char* why = launch_plan_failure_take()) { ftp_set_error("%s", why); return FTP_ERR_UNSUPPORTED; }
  sl.has_loss = true;
  return FTP_OK;
}

extern "C" int ftp_stage_snapshot_weights(ftp_stage* s, int slot, void* stream) {
  int rc = check_call(s, slot, "stage_snapshot_weights");
  if (rc) return rc;
  Slot& sl = s->slots[slot];
  if (!sl.busy) { ftp_set_error("stage_snapshot_weights: slot %d holds no forwarded batch", slot); return FTP_ERR_SLOT; }
  hipStream_t st = (hipStream_t)stream;
  if (s->n_param) {
    HIP_TRY(hipMemcpyAsync(sl.snap_w, s->params, s->n_param * 4, hipMemcpyDeviceToDevice, st));
    if (s->w_lp) HIP_TRY(hipMemcpyAsync(sl.snap_lp, s->w_lp, s->n_param * 2, hipMemcpyDeviceToDevice, st));
  }
  sl.has_snap = true;
  return FTP_OK;
}

extern "C" int ftp_stage_copy_units(ftp_stage* dst, const ftp_stage* src, int unit_lo, int unit_hi, void* stream) {
  if (!dst || !src) { ftp_set_error("stage_copy_units: NULL stage"); return FTP_ERR_ARG; }
  if (dst->model != src->model || dst->dt != src->dt) {
    ftp_set_error("stage_copy_units: the two stages must come from the same model and storage type");
    return FTP_ERR_ARG;
  }
  if (unit_lo < 0 || unit_hi < unit_lo || unit_lo < dst->a || unit_hi > dst->b || unit_lo < src->a || unit_hi > src->b) {
    ftp_set_error("stage_copy_units: units [%d,%d) must lie inside both stages (dst [%d,%d), src [%d,%d))", unit_lo, unit_hi,
                  dst->a, dst->b, src->a, src->b);
    return FTP_ERR_ARG;
  }
  hipStream_t st = (hipStream_t)stream;
  for (int u = unit_lo; u < unit_hi; ++u) {
    const UnitPlan& pd = dst->plan[u - dst->a];
    const UnitPlan& ps = src->plan[u - src->a];
    const size_t n = pd.info->n_param, nb = pd.info->n_bn;
    if (n) {
      HIP_TRY(hipMemcpyAsync(dst->params + pd.p_off, src->params + ps.p_off, n * 4, hipMemcpyDeviceToDevice, st));
      HIP_TRY(hipMemcpyAsync(dst->mom + pd.p_off, src->mom + ps.p_off, n * 4, hipMemcpyDeviceToDevice, st));
      if (dst->w_lp) f32_to_storage(FTP_BF16, st, dst->params + pd.p_off, (char*)dst->w_lp + pd.p_off * 2, n);
    }
    if (nb) {
      HIP_TRY(hipMemcpyAsync(dst->run_mean + pd.bn_off, src->run_mean + ps.bn_off, nb * 4, hipMemcpyDeviceToDevice, st));
      HIP_TRY(hipMemcpyAsync(dst->run_var + pd.bn_off, src->run_var + ps.bn_off, nb * 4, hipMemcpyDeviceToDevice, st));
    }
  }
  HIP_TRY(hipGetLastError());
  if (const char* why = launch_plan_failure_take()) { ftp_set_error("%s", why); return FTP_ERR_UNSUPPORTED; }
  return FTP_OK;
}

extern "C" int ftp_stage_aggregate_weights(ftp_stage* s, const int* slots, int n, void* stream) {
  if (!s || !slots) { ftp_set_error("stage_aggregate_weights: NULL argument"); return FTP_ERR_ARG; }
  if (n < 1 || n > 8) { ftp_set_error("stage_aggregate_weights: 1 <= n <= 8 required, got %d", n); return FTP_ERR_ARG; }
  AggSources src{};
  for (int j = 0; j < n; ++j) {
    const int slot = slots[j];
    if (slot < 0 || slot >= (int)s->slots.size()) {
      ftp_set_error("stage_aggregate_weights: slot %d out of range (n_slots=%zu)", slot, s->slots.size());
      return FTP_ERR_ARG;
    }
    for (int q = 0; q < j; ++q)
      if (slots[q] == slot) { ftp_set_error("stage_aggregate_weights: slot %d listed twice", slot); return FTP_ERR_ARG; }
    if (!s->slots[slot].has_snap) {
      ftp_set_error("stage_aggregate_weights: slot %d holds no weight snapshot", slot);
      return FTP_ERR_SLOT;
    }
    src.p[j] = s->slots[slot].snap_w;
  }
  if (s->n_param) aggregate_weights((hipStream_t)stream, s->params, s->w_lp, src, n, s->n_param);
  HIP_TRY(hipGetLastError());
  if (const char* why = launch_plan_failure_take()) { ftp_set_error("%s", why); return FTP_ERR_UNSUPPORTED; }
  return FTP_OK;
}

// Backward of one convolution+BN+act: dA is the gradient of the activated output.
// Forms dz in one of two alternating buffers; accumulates weight / gamma / beta gradients; when dIn is
// non-NULL writes the gradient of the (activated) input there (+ res for pointwise).  The weight
// gradient runs on the stage's side stream unless per-unit profiling is on.
// mode: the whole layer, or from a dz that the caller formed (passed as dA)
enum { BWD_FULL = 0, BWD_FROM_DZ = 1 };
// stage_forks: the stage is large enough to run weight gradients on its second stream (decides which kernels a
// layer uses); stage_overlaps: it does so now (not while per-unit profiling needs everything on one stream)
static bool stage_forks(const ftp_stage* s) { return s->max_act_bytes >= ((size_t)32 << 20); }
static bool stage_overlaps(const ftp_stage* s) { return s->prof == nullptr && stage_forks(s); }

static int join_side(ftp_stage* s, hipStream_t st);
static int flush_unit_fork(ftp_stage* s, hipStream_t st);

static int sub_backward(ftp_stage* s, Slot& sl, const UnitPlan& p, size_t k, const void* dA, HView in, HView out,
                        void* dIn, const void* res, const WeightSet& W, hipStream_t st, int mode = BWD_FULL,
                        bool unit_fork = false) {
  const Sub& sb = p.info->subs[k];
  ConvGeom g = sb.g; g.N = s->batch;
  int C = g.Cout;
  size_t M = (size_t)s->batch * g.Hout * g.Wout;
  float* stt = sl.stats + p.st_off[k];
  // The fork/join costs four event calls per layer on the host and a cross-stream dependency on the device:
  // it pays only when the kernels are long.  Measured: a 32x32-input stage (largest activation 12 MB) is
  // 10 % faster on one stream, a 224x224 one 15 % slower.
  const bool overlap = mode == BWD_FULL && stage_overlaps(s) && M * (size_t)C >= ((size_t)1 << 20);
  int b = 0, rc_join = 0;
  void* dz = const_cast<void*>(dA);
  // one fork for the whole unit (see PendingWgrad): this layer's dz goes into the unit's buffer set
  const bool batched = unit_fork && overlap && k < 3 && sb.type != SUB_DIRECT && dIn != nullptr && s->dzring[0] != nullptr &&
                       M * (size_t)C * s->es <= s->dzring_bytes;
  // An expand layer in bfloat16: behind the BatchNorm reductions the rest of its backward (dz, data gradient,
  // weight gradient) is one pass on this stream; dz never reaches memory.
  if (mode == BWD_FULL && sb.type == SUB_PW && dIn && s->ws_fused && !bn_bwd_small_ok(M, C) &&
      pw_bwd_fused_ok(s->dt, M, g.Cin, g.Cout, in) && pw_bwd_fused_ws(M, g.Cin, g.Cout) <= s->ws_fused_floats) {
    int P = 0;
    if (s->bwd_sums_of == dA) P = s->bwd_sums_P;
    else bn_bwd_reduce(s->dt, st, dA, out.z, M, C, out.scale, out.shift, sb.act, s->bn_part, &P);
    s->bwd_sums_of = nullptr;
    bn_bwd_finalize(st, s->bn_part, P, M, C, W.w32 + p.p_off + sb.gamma_off, stt, stt + C, s->grads + p.p_off + sb.gamma_off,
                    s->grads + p.p_off + sb.beta_off, s->coef);
    // the sum of the kernel's partial weight gradients is off the data-gradient chain: it goes to the side stream,
    // and the next user of the partial buffer waits for it
    const bool aside = stage_overlaps(s);
    if (s->join_pending[2]) {
      HIP_TRY(hipStreamWaitEvent(st, s->ev_join[2], 0));
      s->join_pending[2] = false;
    }
    pw_bwd_fused(st, dA, out, s->coef, conv_w(s, W, p.p_off + sb.w_off), in.z, res, M, g.Cin, g.Cout, s->ws_fused,
                 s->grads + p.p_off + sb.w_off, dIn, aside ? s->side : st, aside ? s->ev_fork[2] : nullptr);
    if (aside) {
      HIP_TRY(hipEventRecord(s->ev_join[2], s->side));
      s->join_pending[2] = true;
    }
    return FTP_OK;
  }
  if (mode != BWD_FROM_DZ) {
    if (batched) dz = s->dzring[s->bset * 3 + (int)k];
    else {
      b = (int)(s->n_sub_bwd++ & 1u);
      dz = s->gbuf[b ? 4 : 2];
    }
    const bool small = bn_bwd_small_ok(M, C) != 0;
    if (!small) {
      int P = 0;
      if (s->bwd_sums_of == dA) P = s->bwd_sums_P;          // the producer of dA has left the sums
      else bn_bwd_reduce(s->dt, st, dA, out.z, M, C, out.scale, out.shift, sb.act, s->bn_part, &P);
      bn_bwd_finalize(st, s->bn_part, P, M, C, W.w32 + p.p_off + sb.gamma_off, stt, stt + C, s->grads + p.p_off + sb.gamma_off,
                      s->grads + p.p_off + sb.beta_off, s->coef);
    }
    if (batched) {
      if (!s->bset_open) {                // the unit's first write into this set: the weight gradients that last read it must be done
        if (s->bjoin_pending[s->bset]) {
          HIP_TRY(hipStreamWaitEvent(st, s->ev_bjoin[s->bset], 0));
          s->bjoin_pending[s->bset] = false;
        }
        s->bset_open = true;
      }
    } else if (s->join_pending[b]) {      // the weight gradient that last read this dz buffer must be done
      HIP_TRY(hipStreamWaitEvent(st, s->ev_join[b], 0));
      s->join_pending[b] = false;
    }
    if (small)
      bn_bwd_small(s->dt, st, dA, out.z, M, C, out.scale, out.shift, sb.act, W.w32 + p.p_off + sb.gamma_off, stt, stt + C,
                   s->grads + p.p_off + sb.gamma_off, s->grads + p.p_off + sb.beta_off, dz);
    else
      bn_bwd_apply(s->dt, st, dA, out.z, M, C, out.scale, out.shift, sb.act, s->coef, dz);
  }
  hipStream_t ws = st;
  // The depthwise data gradient and weight gradient want the same units (LDS tiles, vector ALU): side by side each
  // takes nearly twice as long.  The data gradient goes first, alone; the weight gradient then shares the GPU with
  // the memory-bound BatchNorm backward of the layer in front.
  const bool dgrad_first = overlap && sb.type == SUB_DW && dIn != nullptr;
  s->bwd_sums_of = nullptr;
  // a depthwise layer behind a BatchNorm + activation of the same unit (the expand layer's): its data gradient is that
  // BatchNorm's dA and can leave the backward sums on the way
  const bool with_sums = sb.type == SUB_DW && dIn != nullptr && mode == BWD_FULL && k > 0 && in.scale != nullptr &&
                         !bn_bwd_small_ok((size_t)s->batch * g.Hin * g.Win, g.Cout) && dw_dgrad_sums_ok(s->dt, g);
  auto run_dw_dgrad = [&]() {
    if (with_sums) {
      dw_dgrad(s->dt, st, dz, conv_w(s, W, p.p_off + sb.w_off), g, dIn, in, s->bn_part, &s->bwd_sums_P);
      s->bwd_sums_of = dIn;
    } else {
      dw_dgrad(s->dt, st, dz, conv_w(s, W, p.p_off + sb.w_off), g, dIn);
    }
  };
  if (dgrad_first) run_dw_dgrad();
  if (batched && mode == BWD_FULL) {
    // noted for the unit's fork; the data gradient goes on as it would behind a forked weight gradient
    if (s->n_pend >= 3) { ftp_set_error("stage_backward: more weight gradients noted for a unit than it has layers"); return FTP_ERR_UNSUPPORTED; }
    s->pend[s->n_pend++] = ftp_stage::PendingWgrad{sb.type, dz, in, g, M, s->grads + p.p_off + sb.w_off};
    if (sb.type == SUB_PW) pw_dgrad(s->dt, st, dz, conv_w(s, W, p.p_off + sb.w_off), res, M, g.Cin, g.Cout, dIn);
    else if (!dgrad_first) run_dw_dgrad();
    return FTP_OK;
  }
  // the first layer of the stage, last in this pass and without a data gradient: its weight gradient is all that is
  // left for this stream, so it runs here with a workspace of its own while the side stream works off its queue
  const bool tail_here = overlap && dIn == nullptr && s->ws_tail != nullptr && &p == &s->plan[0] && k == 0;
  float* wsp = tail_here ? s->ws_tail : s->ws;
  if (overlap && !tail_here) {
    HIP_TRY(hipEventRecord(s->ev_fork[b], st));
    HIP_TRY(hipStreamWaitEvent(s->side, s->ev_fork[b], 0));
    ws = s->side;
  }
  const void* w = conv_w(s, W, p.p_off + sb.w_off);
  float* gw = s->grads + p.p_off + sb.w_off;
  // a layer too short to fork still takes the partial-sum workspace: in a stage that forks its longer layers the
  // side stream may be in the middle of using it, so that work is waited for first
  if (!overlap && stage_overlaps(s) && (rc_join = join_side(s, st))) return rc_join;
  if (sb.type == SUB_PW && !overlap && dIn) {
    pw_bwd(s->dt, st, dz, w, res, in, M, g.Cin, g.Cout, s->ws, gw, dIn);
    return FTP_OK;
  }
  if (sb.type == SUB_DIRECT) {
    conv_direct_wgrad(s->dt, ws, dz, in, g, s->im2col, wsp, gw, s->im2col_of == out.z);
    s->im2col_of = nullptr;      // one weight gradient per forward: nobody else can want these patches
  }
  else if (sb.type == SUB_PW) pw_wgrad(s->dt, ws, dz, in, M, g.Cin, g.Cout, wsp, gw);
  else dw_wgrad(s->dt, ws, dz, in, g, wsp, gw);
  if (overlap && !tail_here) {
    HIP_TRY(hipEventRecord(s->ev_join[b], s->side));
    s->join_pending[b] = true;
  }
  if (dIn) {
    if (sb.type == SUB_DIRECT) {
      // the scratch buffers are shared with the weight gradients: fine on one stream, but a stage that runs them on
      // the side stream keeps the direct kernel
      if (conv_direct_dgrad_gemm_ok(g) && !stage_forks(s) && s->im2col) {
        conv_direct_dgrad_gemm(s->dt, st, dz, w, g, s->im2col, s->ws, dIn);
        s->im2col_of = nullptr;
      }
      else conv_direct_dgrad(s->dt, st, dz, w, g, dIn);
    }
    else if (sb.type == SUB_PW) pw_dgrad(s->dt, st, dz, w, res, M, g.Cin, g.Cout, dIn);
    else if (!dgrad_first) run_dw_dgrad();
  }
  return FTP_OK;
}

// the weight gradients a unit has noted: one fork behind everything the unit has enqueued, all of them on the side
// stream, one join event for the unit's buffer set
static int flush_unit_fork(ftp_stage* s, hipStream_t st) {
  if (s->n_pend == 0) { s->bset_open = false; return FTP_OK; }
  HIP_TRY(hipEventRecord(s->ev_bfork[s->bset], st));
  HIP_TRY(hipStreamWaitEvent(s->side, s->ev_bfork[s->bset], 0));
  for (int i = 0; i < s->n_pend; ++i) {
    const ftp_stage::PendingWgrad& w = s->pend[i];
    if (w.type == SUB_PW) pw_wgrad(s->dt, s->side, w.dz, w.in, w.M, w.g.Cin, w.g.Cout, s->ws, w.gw);
    else dw_wgrad(s->dt, s->side, w.dz, w.in, w.g, s->ws, w.gw);
  }
  HIP_TRY(hipEventRecord(s->ev_bjoin[s->bset], s->side));
  s->bjoin_pending[s->bset] = true;
  s->n_pend = 0;
  s->bset ^= 1;
  s->bset_open = false;
  return FTP_OK;
}

// all side-stream work of this backward is ordered before whatever the caller enqueues next
static int join_side(ftp_stage* s, hipStream_t st) {
  for (int b = 0; b < 3; ++b)
    if (s->join_pending[b]) {
      HIP_TRY(hipStreamWaitEvent(st, s->ev_join[b], 0));
      s->join_pending[b] = false;
    }
  for (int b = 0; b < 2; ++b)
    if (s->bjoin_pending[b]) {
      HIP_TRY(hipStreamWaitEvent(st, s->ev_bjoin[b], 0));
      s->bjoin_pending[b] = false;
    }
  return FTP_OK;
}

extern "C" int ftp_stage_backward(ftp_stage* s, int slot, const void* dy_dev, void* dx_dev, void* stream) {
  int rc = check_call(s, slot, "stage_backward");
  if (rc) return rc;
  Slot& sl = s->slots[slot];
  if (!sl.busy) { ftp_set_error("stage_backward: slot %d holds no forwarded batch", slot); return FTP_ERR_SLOT; }
  if (!dy_dev && !(s->has_loss && sl.has_loss)) {
    ftp_set_error("stage_backward: dy_dev is NULL and ftp_stage_loss has not seeded slot %d", slot);
    return FTP_ERR_ARG;
  }
  hipStream_t st = (hipStream_t)stream;
  if (s->timer && sl.timer_idx >= 0) HIP_TRY(hipEventRecord(s->timer->ev[sl.timer_idx][2], st));
  Views v;
  build_views(s, sl, &v);
  WeightSet W{sl.has_snap ? sl.snap_w : s->params, (const char*)(sl.has_snap ? sl.snap_lp : s->w_lp)};
  if (s->recompute && s->stash_owner != slot) {
    // the intermediates of this batch are gone: forward again from the kept input with the weights of its
    // forward; not a training forward, so the running statistics stay as they are
    const UnitInfo& first = *s->plan[0].info;
    HIP_TRY(hipMemcpyAsync(sl.stash, sl.xin_keep, (size_t)s->batch * first.inH * first.inW * first.inC * s->es,
                           hipMemcpyDeviceToDevice, st));
    s->bn_mom = 0.f;
    rc = forward_units(s, sl, v, W, st);
    s->bn_mom = kBnMomentum;
    if (rc) return rc;
    s->stash_owner = slot;
  }
  s->n_pend = 0; s->bset_open = false;              // nothing is left noted by a call that ended in an error
  const void* d = dy_dev ? dy_dev : sl.dlogits;     // gradient of the current unit's output (read only)
  int flip = 0;
  for (int i = (int)s->plan.size() - 1; i >= 0; --i) {
    const UnitPlan& p = s->plan[i];
    const UnitInfo& u = *p.info;
    if (s->prof) HIP_TRY(hipEventRecord(s->prof->b0[i], st));
    // where the gradient of this unit's input goes: the boundary buffer that does not hold d
    void* next = i > 0 ? (void*)s->gbuf[flip] : dx_dev;
    bool produced = true;
    HView in = v.unit_in[i];
    switch (u.d.kind) {
      case FTP_UNIT_LOSS:
        produced = false;   // the logits gradient passes through unchanged
        if (i == 0 && dx_dev) HIP_TRY(hipMemcpyAsync(dx_dev, d, (size_t)s->batch * u.inC * s->es, hipMemcpyDeviceToDevice, st));
        break;
      case FTP_UNIT_FC: {
        size_t woff = p.p_off;
        pw_wgrad(s->dt, st, d, in, (size_t)s->batch, u.inC, u.outC, s->ws, s->grads + woff);
        bias_grad(s->dt, st, d, s->batch, u.outC, s->grads + woff + (size_t)u.outC * u.inC);
        if (next) pw_dgrad(s->dt, st, d, conv_w(s, W, woff), nullptr, (size_t)s->batch, u.inC, u.outC, next);
        break;
      }
      case FTP_UNIT_GAP:
        if (next) gap_bwd(s->dt, st, d, s->batch, u.inH * u.inW, u.inC, next);
        break;
      case FTP_UNIT_CONV:
        if ((rc = sub_backward(s, sl, p, 0, d, in, v.sub_out[i][0], next, nullptr, W, st))) return rc;
        break;
      case FTP_UNIT_INVRES: {
        size_t ns = u.subs.size();
        void* tmp = s->gbuf[3];
        // project: gradient of the activated depthwise output
        // one fork for the unit when every layer's dz fits the small buffer sets
        bool uf = ns == 3 && s->dzring[0] != nullptr;
        for (const Sub& sb : u.subs)
          if ((size_t)s->batch * sb.g.Hout * sb.g.Wout * sb.g.Cout * s->es > s->dzring_bytes) uf = false;
        if ((rc = sub_backward(s, sl, p, ns - 1, d, v.sub_out[i][ns - 2], v.sub_out[i][ns - 1], tmp, nullptr, W, st, BWD_FULL, uf))) return rc;
        ConvGeom gd = ns == 3 ? u.subs[1].g : ConvGeom{};
        gd.N = s->batch;
        if (ns == 3 && !stage_forks(s) && dw_bwd_small_ok(gd)) {
          // short tensors: depthwise dgrad + wgrad and the expand layer's BatchNorm backward in one launch
          const Sub& s0 = u.subs[0];
          const Sub& s1 = u.subs[1];
          // the depthwise layer's own BatchNorm backward happens inside too: its dz never reaches memory
          void* dz1 = s->gbuf[(s->n_sub_bwd++ & 1u) ? 4 : 2];
          float* st0 = sl.stats + p.st_off[0];
          float* st1 = sl.stats + p.st_off[1];
          BnBwdIn bo{tmp, v.sub_out[i][1], W.w32 + p.p_off + s1.gamma_off, st1, st1 + s1.g.Cout,
                     s->grads + p.p_off + s1.gamma_off, s->grads + p.p_off + s1.beta_off};
          dw_bwd_small(s->dt, st, nullptr, bo, conv_w(s, W, p.p_off + s1.w_off), v.sub_out[i][0], gd, W.w32 + p.p_off + s0.gamma_off, st0,
                       st0 + s0.g.Cout, s->grads + p.p_off + s1.w_off, s->grads + p.p_off + s0.gamma_off,
                       s->grads + p.p_off + s0.beta_off, dz1);
          if ((rc = sub_backward(s, sl, p, 0, dz1, in, v.sub_out[i][0], next, u.residual ? d : nullptr, W, st, BWD_FROM_DZ))) return rc;
        } else if (ns == 3) {
          if ((rc = sub_backward(s, sl, p, 1, tmp, v.sub_out[i][0], v.sub_out[i][1], tmp, nullptr, W, st, BWD_FULL, uf))) return rc;
          if ((rc = sub_backward(s, sl, p, 0, tmp, in, v.sub_out[i][0], next, u.residual ? d : nullptr, W, st, BWD_FULL, uf))) return rc;
          if ((rc = flush_unit_fork(s, st))) return rc;
        } else {
          if (next && u.residual) {
            if ((rc = sub_backward(s, sl, p, 0, tmp, in, v.sub_out[i][0], tmp, nullptr, W, st))) return rc;
            bn_apply(s->dt, st, plain(tmp), (size_t)s->batch * u.inH * u.inW, u.inC, d, next);
          } else {
            if ((rc = sub_backward(s, sl, p, 0, tmp, in, v.sub_out[i][0], next, nullptr, W, st))) return rc;
          }
        }
        break;
      }
      default:
        break;
    }
    if (s->prof) HIP_TRY(hipEventRecord(s->prof->b1[i], st));
    if (produced && next) { d = next; if (i > 0) flip ^= 1; }
  }
  if ((rc = join_side(s, st))) return rc;
  if (s->timer && sl.timer_idx >= 0) {
    HIP_TRY(hipEventRecord(s->timer->ev[sl.timer_idx][3], st));
    s->timer->bwd_done[sl.timer_idx] = true;
    sl.timer_idx = -1;
  }
  HIP_TRY(hipGetLastError());
  if (const char* why = launch_plan_failure_take()) { ftp_set_error("%s", why); return FTP_ERR_UNSUPPORTED; }
  sl.busy = false; sl.has_snap = false; sl.has_loss = false;
  return FTP_OK;
}

extern "C" int ftp_stage_timing(ftp_stage* s, int enable) {
  if (!s) { ftp_set_error("stage_timing: NULL stage"); return FTP_ERR_ARG; }
  for (auto& sl : s->slots)
    if (sl.busy) { ftp_set_error("stage_timing: switch it while no batch is in flight"); return FTP_ERR_SLOT; }
  if (!enable) {
    if (s->timer) {
      if (s->timer->created)
        for (auto& q : s->timer->ev)
          for (auto& e : q) (void)hipEventDestroy(e);
      delete s->timer;
      s->timer = nullptr;
    }
    return FTP_OK;
  }
  if (!s->timer) {
    s->timer = new ExecTimer();
    for (auto& q : s->timer->ev)
      for (auto& e : q) HIP_TRY(hipEventCreate(&e));
    s->timer->created = true;
  }
  s->timer->used = 0;
  return FTP_OK;
}

extern "C" int ftp_stage_timing_read(ftp_stage* s, double* mean_ns, int* n_batches) {
  if (!s || !mean_ns || !n_batches) { ftp_set_error("stage_timing_read: NULL argument"); return FTP_ERR_ARG; }
  if (!s->timer) { ftp_set_error("stage_timing_read: execution timing is not enabled"); return FTP_ERR_ARG; }
  double sum = 0.0;
  int n = 0;
  for (int i = 0; i < s->timer->used; ++i) {
    if (!s->timer->bwd_done[i]) continue;              // forwarded, not yet backwarded: not a whole batch
    float f = 0.f, b = 0.f;
    HIP_TRY(hipEventSynchronize(s->timer->ev[i][3]));
    HIP_TRY(hipEventElapsedTime(&f, s->timer->ev[i][0], s->timer->ev[i][1]));
    HIP_TRY(hipEventElapsedTime(&b, s->timer->ev[i][2], s->timer->ev[i][3]));
    sum += ((double)f + (double)b) * 1e6;
    ++n;
  }
  for (auto& sl : s->slots) sl.timer_idx = -1;         // batches in flight are dropped from the measurement
  s->timer->used = 0;
  *n_batches = n;
  *mean_ns = n ? sum / n : 0.0;
  return FTP_OK;
}

extern "C" int ftp_stage_update(ftp_stage* s, const ftp_sgd* opt, void* stream) {
  if (!s || !opt) { ftp_set_error("stage_update: NULL argument"); return FTP_ERR_ARG; }
  if (!(std::isfinite(opt->lr) && std::isfinite(opt->momentum) && std::isfinite(opt->weight_decay))) {
    ftp_set_error("stage_update: non-finite hyper-parameter");
    return FTP_ERR_VALUE;
  }
  if (s->n_param) sgd_update((hipStream_t)stream, s->params, s->grads, s->mom, s->w_lp, s->n_param, opt->lr, opt->momentum, opt->weight_decay);
  HIP_TRY(hipGetLastError());
  if (const char* why = launch_plan_failure_take()) { ftp_set_error("%s", why); return FTP_ERR_UNSUPPORTED; }
  return FTP_OK;
}

// ------------------------------------------------------------ loss without a stage, without allocation
// Per-row losses of ftp_softmax_ce_static: partial results between its two kernels.  One copy per GPU, held until the
// process ends; in host code the name is only a handle for hipGetSymbolAddress, the kernels get the address.
enum { kStaticLossMaxBatch = FTP_STATIC_LOSS_MAX_BATCH, kStaticMaxDevices = 64 };
static __device__ __align__(256) float scratch[kStaticLossMaxBatch];
static float* g_scratch_ptr[kStaticMaxDevices];     // per device: the address of that GPU's copy
static std::mutex g_scratch_mu;

static int static_scratch(float** out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kStaticMaxDevices) { ftp_set_error("softmax_ce_static: device ordinal %d not supported", dev); return FTP_ERR_UNSUPPORTED; }
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    float* p = nullptr;
    HIP_TRY(hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)));    // with `dev` current: this GPU's copy
    if (!p) { ftp_set_error("softmax_ce_static: no device address for the scratch array"); return FTP_ERR_HIP; }
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return FTP_OK;
}

extern "C" int ftp_softmax_ce_static(const void* logits_dev, const int32_t* labels_dev, int batch, int classes, ftp_dtype dtype,
                                     void* dlogits_dev, float* loss_dev, void* stream) {
  if (!logits_dev || !labels_dev || !dlogits_dev || !loss_dev) { ftp_set_error("softmax_ce_static: NULL argument"); return FTP_ERR_ARG; }
  if (dtype != FTP_F32 && dtype != FTP_BF16) { ftp_set_error("softmax_ce_static: unknown dtype %d", (int)dtype); return FTP_ERR_ARG; }
  if (batch < 1 || classes < 1) { ftp_set_error("softmax_ce_static: batch and classes must be positive"); return FTP_ERR_ARG; }
  if (batch > kStaticLossMaxBatch) {
    ftp_set_error("softmax_ce_static: batch %d is beyond the %d rows the static scratch array holds", batch, (int)kStaticLossMaxBatch);
    return FTP_ERR_ARG;
  }
  float* rows = nullptr;
  int rc = static_scratch(&rows);
  if (rc) return rc;
  // every row < batch is written before it is read and nothing beyond is read: nothing has to start at zero
  softmax_ce((int)dtype, (hipStream_t)stream, logits_dev, labels_dev, batch, classes, rows, dlogits_dev, loss_dev);
  HIP_TRY(hipGetLastError());
  if (const char* why = launch_plan_failure_take()) { ftp_set_error("%s", why); return FTP_ERR_UNSUPPORTED; }
  return FTP_OK;
}

// ------------------------------------------------------------ profile_layers
__global__ void synth_fill_k(float* p, size_t n, uint32_t salt, float amp) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    uint32_t h = (uint32_t)i * 2654435761u + salt;
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13; h *= 3266489917u; h ^= h >> 16;
    p[i] = ((float)(h >> 8) * (1.0f / 8388608.0f) - 1.0f) * amp;
  }
}

extern "C" int ftp_profile_layers(const ftp_model* m, int batch, int reps, double* t_ns, int64_t* out_bytes, void* stream) {
  if (!m || !t_ns || !out_bytes || batch < 1 || reps < 1) { ftp_set_error("profile_layers: bad argument"); return FTP_ERR_ARG; }
  int L = (int)m->units.size();
  ftp_stage* s = nullptr;
  int rc = ftp_stage_create(m, 0, L, batch, 1, &s);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)stream;
  ProfEvents ev;
  float *x32 = nullptr, *loss = nullptr;
  void *x = nullptr, *dy = nullptr;
  int32_t* labels = nullptr;
  const UnitInfo& last = m->units[L - 1];
  size_t n_in = (size_t)batch * m->inH * m->inW * m->inC;
  size_t n_out = (size_t)batch * last.outH * last.outW * last.outC;
  size_t es = s->es;
  auto cleanup = [&]() {
    for (auto* vec : {&ev.f0, &ev.f1, &ev.b0, &ev.b1})
      for (hipEvent_t e : *vec) (void)hipEventDestroy(e);
    dfree(x32); dfree(x); dfree(dy); dfree(labels); dfree(loss);
    s->prof = nullptr;
    stage_free(s);
  };
#define PROF_TRY(expr)                                                                   \
  do {                                                                                   \
    hipError_t e_ = (expr);                                                              \
    if (e_ != hipSuccess) {                                                              \
      ftp_set_error("profile_layers: %s failed: %s", #expr, hipGetErrorString(e_));     \
      cleanup();                                                                         \
      return FTP_ERR_HIP;                                                                \
    }                                                                                    \
  } while (0)
  size_t nmax = n_in > n_out ? n_in : n_out;
  PROF_TRY(hipMalloc((void**)&x32, align_up(nmax * 4, 256)));
  PROF_TRY(hipMalloc(&x, align_up(n_in * es, 256)));
  PROF_TRY(hipMalloc(&dy, align_up(n_out * es, 256)));
  PROF_TRY(hipMalloc((void**)&labels, align_up((size_t)batch * 4, 256)));
  PROF_TRY(hipMalloc((void**)&loss, 256));
  // synthetic weights (uniform, variance 2/fan_in-like scale is irrelevant for timing), input and output gradient
  hipLaunchKernelGGL(synth_fill_k, dim3(1024), dim3(256), 0, st, s->params, s->n_param, 17u, 0.1f);
  if (s->w_lp) f32_to_storage(FTP_BF16, st, s->params, s->w_lp, s->n_param);
  hipLaunchKernelGGL(synth_fill_k, dim3(1024), dim3(256), 0, st, x32, n_in, 29u, 1.7f);
  f32_to_storage(s->dt, st, x32, x, n_in);
  hipLaunchKernelGGL(synth_fill_k, dim3(1024), dim3(256), 0, st, x32, n_out, 31u, 0.01f);
  f32_to_storage(s->dt, st, x32, dy, n_out);
  fill_zero(st, labels, align_up((size_t)batch * 4, 256));
  // gamma = 1 so that activations keep a sane scale
  for (const UnitPlan& p : s->plan)
    for (const Sub& sb : p.info->subs) {
      std::vector<float> ones(sb.g.Cout, 1.0f);
      PROF_TRY(hipMemcpyAsync(s->params + p.p_off + sb.gamma_off, ones.data(), ones.size() * 4, hipMemcpyHostToDevice, st));
      PROF_TRY(hipStreamSynchronize(st));
    }
  for (auto* vec : {&ev.f0, &ev.f1, &ev.b0, &ev.b1}) {
    vec->resize(L);
    for (int i = 0; i < L; ++i) PROF_TRY(hipEventCreate(&(*vec)[i]));
  }
  std::vector<double> acc(L, 0.0);
  bool has_loss = s->has_loss;
  for (int r = 0; r < reps + 2; ++r) {
    s->prof = &ev;
    rc = ftp_stage_forward(s, 0, x, nullptr, st);
    if (!rc && has_loss) rc = ftp_stage_loss(s, 0, labels, loss, st);
    if (!rc) rc = ftp_stage_backward(s, 0, has_loss ? nullptr : dy, nullptr, st);
    s->prof = nullptr;
    if (rc) { cleanup(); return rc; }
    PROF_TRY(hipStreamSynchronize(st));
    if (r < 2) continue;   // discarded warm-up runs
    for (int i = 0; i < L; ++i) {
      float f = 0.f, b = 0.f;
      PROF_TRY(hipEventElapsedTime(&f, ev.f0[i], ev.f1[i]));
      PROF_TRY(hipEventElapsedTime(&b, ev.b0[i], ev.b1[i]));
      acc[i] += ((double)f + (double)b) * 1e6;
    }
  }
  // The per-unit events need every unit to begin and end on the caller's stream, so a stage that normally runs its
  // weight gradients on a second stream was just timed without that overlap.  The per-unit times keep their
  // proportions and are scaled so that they add up to what a batch costs under the plan training really runs
  // (forward + loss + backward, timed like ftp_stage_timing does): the capacity equation divides a worker's
  // measured batch time by this sum, and the same device then comes out at capacity 1.
  double sum_units = 0.0, whole = 0.0;
  for (int i = 0; i < L; ++i) sum_units += acc[i] / reps;
  for (int r = 0; r < reps + 1; ++r) {
    PROF_TRY(hipEventRecord(ev.f0[0], st));
    rc = ftp_stage_forward(s, 0, x, nullptr, st);
    if (!rc && has_loss) rc = ftp_stage_loss(s, 0, labels, loss, st);
    if (!rc) rc = ftp_stage_backward(s, 0, has_loss ? nullptr : dy, nullptr, st);
    if (rc) { cleanup(); return rc; }
    PROF_TRY(hipEventRecord(ev.f1[0], st));
    PROF_TRY(hipStreamSynchronize(st));
    float ms = 0.f;
    PROF_TRY(hipEventElapsedTime(&ms, ev.f0[0], ev.f1[0]));
    if (r > 0) whole += (double)ms * 1e6;   // first run discarded: the other plan's kernels load their code
  }
  whole /= reps;
  const double k_plan = sum_units > 0.0 && whole > 0.0 ? whole / sum_units : 1.0;
  for (int i = 0; i < L; ++i) {
    double t = std::floor(acc[i] / reps * k_plan + 0.5);
    t_ns[i] = t < 1.0 ? 1.0 : t;
    const UnitInfo& u = m->units[i];
    out_bytes[i] = (int64_t)((size_t)batch * u.outH * u.outW * u.outC * es);
  }
  cleanup();
#undef PROF_TRY
  return FTP_OK;
}
