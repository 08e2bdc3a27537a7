// Host runtime of the PB tick engine: descriptor validation, arena planning,
// step-table compilation, the C ABI declared in include/pb.h.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <string>
#include <vector>

#include "../../include/pb.h"
#include "pb_device.h"

using namespace pb;

namespace {

thread_local std::string g_err;

// contexts built by pb_init_static share one static device array per GPU: one at a time
constexpr int MAX_STATIC_DEVS = 64;
bool g_static_busy[MAX_STATIC_DEVS] = {};
int g_static_dev = -1;   // device of the pb_init_static call in progress

int fail(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}

#define HIP_TRY(expr)                                                                    \
  do {                                                                                   \
    hipError_t e_ = (expr);                                                              \
    if (e_ != hipSuccess)                                                                \
      return fail(PB_E_HIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
  } while (0)

// ---------------------------------------------------------------- stage model
struct Stage {
  bool pre_gn = false, pre_relu = false, gap = false, post_gn = false, pool = false, add = false,
       proj = false, ce = false, is_conv = false, has_bias = false;
  int G = 0;                       // GroupNorm groups
  int Cin = 0, Hin = 0, Win = 0;   // stage input
  int C = 0, H = 0, W = 0;         // main op input (after optional GAP / flatten)
  int K = 0, OH = 0, OW = 0;       // main op output
  int k = 1, stride = 1, pad = 0;
  int pk = 0, ps = 0, pp = 0, PH = 0, PW = 0;
  int Cout = 0, Hout = 0, Wout = 0;   // stage output
  int skip_from = -1, sstride = 1, sC = 0, sH = 0, sW = 0;
  int tap_dist = 0;                // >0: a later stage (this + tap_dist) adds this stage's input
  int D = 0;        // natural delay 2(S-1-s): ticks between the stage's forward and backward pass of a sample
  int De = 0;       // delay the caller asks for (>= D): the forward pass uses weights that many updates old
  // parameter offsets in the padded flat arena (floats), -1 = absent
  int64_t off = 0, padded = 0, n_params = 0, n_head = 0;
  int64_t o_w = -1, o_b = -1, o_wp = -1, o_gamma = -1, o_beta = -1;
  int64_t n_w = 0, n_b = 0, n_wp = 0, n_gn = 0;
  int fan_w = 0, fan_wp = 0;
  int in_elems() const { return Cin * Hin * Win; }
  int out_elems() const { return Cout * Hout * Wout; }
  int z_elems() const { return K * OH * OW; }
  int gnC() const { return pre_gn ? Cin : K; }
};

int parse_net(const pb_net_desc* net, std::vector<Stage>& out) {
  if (!net || net->n_stages <= 0 || !net->stages) return fail(PB_E_INVALID, "empty network");
  if (net->in_c <= 0 || net->in_h <= 0 || net->in_w <= 0 || net->n_classes <= 0)
    return fail(PB_E_INVALID, "bad input dimensions");
  if (net->mitigation < 0 || net->mitigation > 3) return fail(PB_E_INVALID, "mitigation must be 0..3");
  if (net->bwd_weights != 0 && net->bwd_weights != 1) return fail(PB_E_INVALID, "bwd_weights=%d", net->bwd_weights);
  if (net->act_dtype != 0 && net->act_dtype != 1) return fail(PB_E_INVALID, "act_dtype=%d", net->act_dtype);
  if (net->act_dtype == 1 && net->kernel_set != 0) return fail(PB_E_UNSUPPORTED, "bf16 activations need kernel_set 0");
  if (net->kernel_set < 0 || net->kernel_set > 1) return fail(PB_E_INVALID, "kernel_set must be 0 or 1");
  if (net->lwp_form != 0 && net->lwp_form != 1) return fail(PB_E_INVALID, "lwp_form must be 0 or 1");
  if (!(net->sc_scale >= 0.f) || !(net->lwp_scale >= 0.f)) return fail(PB_E_INVALID, "sc_scale and lwp_scale must be >= 0");
  if (net->update_size < 0 || net->update_size > 65536) return fail(PB_E_INVALID, "update_size must be 0 (= 1) .. 65536");
  if (net->tuning && net->tuning->gemm_lds_kb != 0 && net->tuning->gemm_lds_kb != 62 && net->tuning->gemm_lds_kb != 76)
    return fail(PB_E_INVALID, "tuning.gemm_lds_kb must be 0, 62 or 76");
  const int S = net->n_stages;
  out.assign(S, Stage());
  int C = net->in_c, H = net->in_h, W = net->in_w;
  for (int s = 0; s < S; ++s) {
    Stage& st = out[s];
    const pb_stage& ps = net->stages[s];
    if (ps.n_ops <= 0 || !ps.ops) return fail(PB_E_INVALID, "stage %d has no ops", s);
    st.Cin = C; st.Hin = H; st.Win = W;
    st.D = 2 * (S - 1 - s);
    st.De = st.D;
    int i = 0;
    const int n = ps.n_ops;
    auto kind = [&](int j) { return j < n ? ps.ops[j].kind : -1; };
    if (kind(i) == PB_OP_GROUPNORM) {
      const pb_op& o = ps.ops[i];
      if (o.cin != C || o.groups <= 0 || C % o.groups) return fail(PB_E_INVALID, "stage %d: GroupNorm channels/groups mismatch", s);
      st.pre_gn = true; st.G = o.groups; ++i;
    }
    if (kind(i) == PB_OP_RELU) { st.pre_relu = true; ++i; }
    if (kind(i) == PB_OP_GLOBAL_AVGPOOL) {
      if (!st.pre_gn) return fail(PB_E_UNSUPPORTED, "stage %d: global average pool needs a GroupNorm before it", s);
      st.gap = true; ++i;
    }
    if (kind(i) != PB_OP_CONV2D && kind(i) != PB_OP_LINEAR)
      return fail(PB_E_INVALID, "stage %d: expected the weight layer at op %d", s, i);
    {
      const pb_op& o = ps.ops[i];
      st.is_conv = (o.kind == PB_OP_CONV2D);
      st.has_bias = o.has_bias != 0;
      if (st.is_conv) {
        if (st.gap) return fail(PB_E_UNSUPPORTED, "stage %d: conv after global average pool", s);
        if (o.cin != C || o.cout <= 0 || o.k <= 0 || o.stride <= 0 || o.pad < 0 || o.pad >= o.k)
          return fail(PB_E_INVALID, "stage %d: bad conv parameters", s);
        st.C = C; st.H = H; st.W = W; st.K = o.cout; st.k = o.k; st.stride = o.stride; st.pad = o.pad;
        st.OH = (H + 2 * o.pad - o.k) / o.stride + 1;
        st.OW = (W + 2 * o.pad - o.k) / o.stride + 1;
        if (st.OH <= 0 || st.OW <= 0) return fail(PB_E_INVALID, "stage %d: conv output is empty", s);
      } else {
        const int flat = st.gap ? C : C * H * W;
        if (o.cin != flat || o.cout <= 0) return fail(PB_E_INVALID, "stage %d: linear cin %d != input size %d", s, o.cin, flat);
        if (st.pre_gn && !st.gap && H * W > 1)
          return fail(PB_E_UNSUPPORTED, "stage %d: GroupNorm before a flattening linear layer", s);
        st.C = flat; st.H = 1; st.W = 1; st.K = o.cout; st.k = 1; st.stride = 1; st.pad = 0;
        st.OH = st.OW = 1;
      }
      st.fan_w = st.C * st.k * st.k;
      ++i;
    }
    st.Cout = st.K; st.Hout = st.OH; st.Wout = st.OW;
    if (kind(i) == PB_OP_GROUPNORM) {
      if (st.pre_gn) return fail(PB_E_UNSUPPORTED, "stage %d: two GroupNorms in one stage", s);
      const pb_op& o = ps.ops[i];
      if (o.cin != st.K || o.groups <= 0 || st.K % o.groups) return fail(PB_E_INVALID, "stage %d: GroupNorm channels/groups mismatch", s);
      if (kind(i + 1) != PB_OP_RELU) return fail(PB_E_UNSUPPORTED, "stage %d: GroupNorm after the layer must be followed by ReLU", s);
      st.post_gn = true; st.G = o.groups; i += 2;
      if (kind(i) == PB_OP_MAXPOOL) {
        const pb_op& p = ps.ops[i];
        if (p.k <= 0 || p.stride <= 0 || p.pad < 0 || 2 * p.pad > p.k) return fail(PB_E_INVALID, "stage %d: bad max-pool", s);
        st.pool = true; st.pk = p.k; st.ps = p.stride; st.pp = p.pad;
        st.PH = (st.OH + 2 * p.pad - p.k) / p.stride + 1;
        st.PW = (st.OW + 2 * p.pad - p.k) / p.stride + 1;
        if (st.PH <= 0 || st.PW <= 0) return fail(PB_E_INVALID, "stage %d: pool output is empty", s);
        st.Hout = st.PH; st.Wout = st.PW;
        ++i;
      }
    }
    if (kind(i) == PB_OP_ADD_SKIP) {
      const pb_op& o = ps.ops[i];
      if (st.post_gn) return fail(PB_E_UNSUPPORTED, "stage %d: skip add after a post-layer GroupNorm", s);
      const int a = o.skip_from_stage;
      if (a < 0 || a >= s) return fail(PB_E_INVALID, "stage %d: skip_from_stage %d out of range", s, a);
      if (out[a].tap_dist) return fail(PB_E_UNSUPPORTED, "stage %d tapped twice", a);
      if (s - a > out[a].D) return fail(PB_E_INVALID, "stage %d: skip source too far", s);
      st.add = true; st.skip_from = a; st.proj = o.has_proj != 0;
      st.sC = out[a].Cin; st.sH = out[a].Hin; st.sW = out[a].Win;
      st.sstride = st.proj ? std::max(1, (int)o.stride) : 1;
      if (st.proj) {
        if (o.cin != st.sC || o.cout != st.K) return fail(PB_E_INVALID, "stage %d: projection channels mismatch", s);
        if ((st.sH - 1) / st.sstride + 1 != st.OH || (st.sW - 1) / st.sstride + 1 != st.OW)
          return fail(PB_E_INVALID, "stage %d: projection output size mismatch", s);
        st.fan_wp = st.sC;
      } else if (st.sC != st.K || st.sH != st.OH || st.sW != st.OW) {
        return fail(PB_E_INVALID, "stage %d: identity skip shape mismatch", s);
      }
      out[a].tap_dist = s - a;
      ++i;
    }
    if (kind(i) == PB_OP_SOFTMAX_CE) {
      if (s != S - 1) return fail(PB_E_INVALID, "stage %d: loss only in the last stage", s);
      if (st.post_gn || st.add) return fail(PB_E_UNSUPPORTED, "loss stage with post-norm or skip");
      if (st.K != net->n_classes || st.OH * st.OW != 1) return fail(PB_E_INVALID, "logits size %d != n_classes %d", st.K * st.OH * st.OW, net->n_classes);
      st.ce = true; ++i;
    }
    if (i != n) return fail(PB_E_UNSUPPORTED, "stage %d: op %d (kind %d) does not fit the stage pattern", s, i, kind(i));
    if (s == S - 1 && !st.ce) return fail(PB_E_INVALID, "last stage must end with the loss");
    if (s == 0 && st.pre_gn) return fail(PB_E_UNSUPPORTED, "GroupNorm directly on the network input");
    C = st.Cout; H = st.Hout; W = st.Wout;
  }
  // parameter layout, canonical order inside a stage, stages padded to UPD_CHUNK
  int64_t off = 0;
  for (Stage& st : out) {
    st.off = off;
    int64_t o = 0;
    st.n_w = (int64_t)st.K * st.C * st.k * st.k; st.o_w = o; o += st.n_w;
    if (st.has_bias) { st.n_b = st.K; st.o_b = o; o += st.n_b; }
    if (st.proj) { st.n_wp = (int64_t)st.K * st.sC; st.o_wp = o; o += st.n_wp; }
    st.n_head = o;                                   // weight, bias, projection: contiguous, canonical order
    if (st.pre_gn || st.post_gn) {
      // GroupNorm scale and shift start on a 16-byte boundary: the vectorised update of the
      // tensors before them must not touch them when another step updates them (F_UPD_GN)
      o = (o + 3) / 4 * 4;
      st.n_gn = st.gnC(); st.o_gamma = o; o += st.n_gn; st.o_beta = o; o += st.n_gn;
    }
    st.n_params = st.n_head + 2 * st.n_gn;
    st.padded = (o + UPD_CHUNK - 1) / UPD_CHUNK * UPD_CHUNK;
    off += st.padded;
  }
  return PB_OK;
}

// delays[s] = the pipeline's own 2(S-1-s): depth-2 ring of predicted weights (one being read, one being
// written).  Larger: the forward pass reads a version that many updates older, kept in a deeper ring.
// Any delay smaller than the pipeline's own: a pipeline that never stalls cannot produce it (stage s+1
// would need stage s's output of the same tick), so the whole network switches to the sample-indexed
// form (Eqs. wi, sgdpb, wf): one tick pushes one sample through all stages in dependency order, forward
// pass of stage s with the weights delays[s] updates old, backward pass with the current ones, then the
// update.  That is a verification mode (a few launches per stage and tick), not a performance path.
int check_delays(std::vector<Stage>& st, const int32_t* delays, bool* sequential) {
  *sequential = false;
  if (!delays) return PB_OK;
  for (size_t s = 0; s < st.size(); ++s) {
    if (delays[s] < 0) return fail(PB_E_INVALID, "delay of stage %zu is negative", s);
    if (delays[s] < st[s].D) *sequential = true;
    if (delays[s] > 4096 + st[s].D) return fail(PB_E_UNSUPPORTED, "delay %d of stage %zu: too many weight versions", delays[s], s);
  }
  for (size_t s = 0; s < st.size(); ++s) {
    st[s].De = delays[s];
    if (*sequential) st[s].D = 0;      // nothing is in flight between a sample's forward and backward pass
  }
  return PB_OK;
}

// ------------------------------------------------------------------ arena
struct Plan {
  int64_t total = 0;   // floats
  int64_t alloc(int64_t n) {
    int64_t o = total;
    total += (n + 63) / 64 * 64;
    return o;
  }
};

struct StageBufs {
  int64_t aring = -1;   // normalised + rectified stage input (pre-norm conv stages)
  int64_t xring = -1, prest = -1, pooled = -1, zring = -1, postst = -1, gradbox = -1, skg = -1,
          da = -1, dz = -1, part = -1, logits = -1, dlogits = -1,
          projy = -1,   // output of the skip projection of the tick's forward sample (computed one phase ahead of the sum)
          dxparts = -1, // FWD_PARTS partial gradients with respect to the stage's output, left by the backward-data GEMM of
                        // the next stage (a thin layer) split over its reduction; summed by the stage's GroupNorm channel sums
          zparts = -1,  // FWD_PARTS partial outputs of a thin layer's forward GEMM split over its reduction (summed by its statistics step)
          w2 = -1,      // second copy of the stage's master parameters (stages whose update computes the weight gradient itself)
          gparts = -1;  // GRAD_PARTS copies of the stage's gradient block, the first one complete, the others partial
                        // weight gradients of a backward-weights GEMM whose reduction is split over workgroups
  int st_stride = 0;
};

struct Layout {
  int64_t P = 0;                      // padded parameter count
  int64_t w = 0, v = 0, g = 0;
  int64_t gacc = -1;                  // update size above one: gradients added up since each stage's latest update
  std::vector<int64_t> what;          // per stage: ring [De - D + 2][padded] of predicted-weight versions
  std::vector<StageBufs> sb;
  int64_t staging = 0, labels = 0, loss = 0, globals = 0, zero = 0, sync = 0;
  int64_t total = 0;
};

// A convolution over a large map with few weights has a weight gradient that is a long
// reduction with few output tiles: such a stage gets room for partial gradients.
constexpr int MAX_SYNC_PHASES = 8;   // phases that may share one launch (completion counters per stage and phase)
constexpr int GRAD_PARTS = 16;
// A layer on a map of at most 16 pixels with a long reduction is a matrix-vector product: its
// forward GEMM has as many tiles as it has blocks of 16 output channels, each streaming its rows of
// the weight matrix.  Followed by a GroupNorm (whose statistics step reads the whole output anyway),
// its reduction is split over workgroups that write partial outputs.
constexpr int FWD_PARTS = 8;
constexpr int THIN_MAX_PIXELS = 64;
bool fwd_split_candidate(const Stage& a) {
  return a.is_conv && a.post_gn && !a.add && (int64_t)a.OH * a.OW <= THIN_MAX_PIXELS && (int64_t)a.C * a.k * a.k >= 2048;
}
bool split_candidate(const Stage& a) { return a.is_conv && (int64_t)a.OH * a.OW >= 256 && a.padded <= 65536; }

// The same for the backward-data GEMM of a thin layer: it writes the gradient with respect to the
// previous stage's output.  Where that stage ends in a GroupNorm whose channel sums run in the
// one-wavefront-per-channel form over at most 64 gradient values per channel, they add the parts up.
bool bwd_split_consumer(const std::vector<Stage>& st, int s) {
  if (s + 1 >= (int)st.size()) return false;
  const Stage& a = st[s];
  const Stage& n = st[s + 1];
  if (!a.post_gn || !n.is_conv || n.pre_gn || n.pre_relu || n.tap_dist || n.add) return false;
  if ((int64_t)n.H * n.W > THIN_MAX_PIXELS || (int64_t)n.K * n.k * n.k < 2048) return false;
  // consumer: the channel sums behind a max-pool in their one-wavefront-per-channel form, or the fused
  // GroupNorm backward (one workgroup per group, gradient in registers)
  const int64_t per_channel = a.out_elems() / std::max(1, a.K);
  // (behind a max-pool: the wave form for maps of up to 64 pixels, else the form that stages the channel's map and its
  // pooled gradient in LDS)
  if (a.pool) return (per_channel <= 64 && a.OH * a.OW <= 64) || (int64_t)a.OH * a.OW + per_channel <= LDS_FLOATS;
  return a.G > 0 && (int64_t)(a.K / a.G) * a.OH * a.OW <= 4096 && (a.OH * a.OW) % 4 == 0;
}

// A 3x3 layer of stride 1 and padding 1 on a 2x2 or 4x4 map with many channels is a matrix-vector product:
// its forward and backward-data passes run as dot-product steps (K_DOT_FWD, K_DOT_BWD_X) in networks tiled
// for throughput.
bool dot_layer(const Stage& a) {
  return a.is_conv && a.k == 3 && a.stride == 1 && a.pad == 1 && a.H == a.W && (a.H == 2 || a.H == 4) && a.OH == a.H && a.OW == a.W &&
         !a.gap && !a.has_bias && !a.add && !a.pre_gn && !a.pre_relu && a.C % 64 == 0 && a.K % 8 == 0 && (int64_t)a.C * a.K >= 32768;
}

int st_stride_of(const Stage& s) { return (2 * s.G + 2 * s.gnC() + 63) / 64 * 64; }

// A 3x3 layer on a 2x2 or 4x4 map (the 512-channel layers of VGG-11): its weight gradient is an outer product of two
// tiny maps per weight, which the update step can compute while it streams the parameters (F_WGRAD).
bool fusew_shape(const Stage& a) {
  return a.is_conv && a.k == 3 && a.stride == 1 && a.pad == 1 && a.H == a.W && (a.H == 2 || a.H == 4) && a.OH == a.H && a.OW == a.W &&
         !a.gap && !a.has_bias && a.C * 9 >= 1171 && a.C * a.H * a.W <= 8192 && a.n_w % 4 == 0 && a.n_w >= 65536;
}

int what_depth(const Stage& a, bool stash) { return stash ? a.De + 2 : a.De - a.D + 2; }

void plan_arena(const std::vector<Stage>& st, bool stash, int loss_cap, Layout& L, Plan& pl, bool use_aring, int update_size) {
  const int S = (int)st.size();
  L.P = 0;
  for (const Stage& s : st) L.P += s.padded;
  // The forward (predicted) weights are kept as a ring of versions per stage: the update of tick t
  // writes slot (t+1) mod R, the forward pass of tick t reads slot (t - extra) mod R, extra = De - D,
  // R = extra + 2.  With the pipeline's own delays that is two copies alternating by tick parity, which
  // is what lets an update run beside forward work of its own tick.  Master weights and velocity are
  // updated in place: their only readers in a tick (the stage's backward steps) come before the
  // stage's update.  Without weight prediction the forward copy simply equals the master weights.
  L.w = pl.alloc(L.P); L.v = pl.alloc(L.P); L.g = pl.alloc(L.P);
  if (update_size > 1) L.gacc = pl.alloc(L.P);
  // Exception: a stage whose update computes the weight gradient itself needs nothing but the layer's two maps, which
  // are complete a phase before the stage's backward-data step has read the weights.  With a second copy of the
  // stage's master parameters (the update of tick t reads copy t mod 2 and writes the other) it runs beside that step.
  L.sb.assign(S, StageBufs());
  if (!stash && update_size == 1 && use_aring)
    for (int s = 0; s < S; ++s)
      if (fusew_shape(st[s])) L.sb[s].w2 = pl.alloc(st[s].padded);
  L.what.assign(S, 0);
  // Weight stashing (the backward pass uses the forward's predicted weights, Eq. sgdpb_weight_stash):
  // the version the forward pass of a sample read has to survive until its backward pass, De + 2 slots.
  for (int s = 0; s < S; ++s) L.what[s] = pl.alloc((int64_t)what_depth(st[s], stash) * st[s].padded);
  for (int s = 0; s < S; ++s) {
    const Stage& a = st[s];
    StageBufs& b = L.sb[s];
    b.xring = pl.alloc((int64_t)(a.D + 2) * a.in_elems());
    if (a.pre_gn || a.post_gn) b.st_stride = st_stride_of(a);
    if (a.pre_gn) b.prest = pl.alloc((int64_t)(a.D + 1) * b.st_stride);
    if (a.pre_gn && !a.gap && use_aring) b.aring = pl.alloc((int64_t)(a.D + 1) * a.in_elems());
    if (a.gap) b.pooled = pl.alloc((int64_t)(a.D + 1) * a.C);
    if (a.post_gn) {
      b.zring = pl.alloc((int64_t)(a.D + 1) * a.z_elems());
      b.postst = pl.alloc((int64_t)(a.D + 1) * b.st_stride);
      b.dz = pl.alloc(a.z_elems());
    }
    if (a.pre_gn || a.post_gn) b.part = pl.alloc(3 * a.gnC());
    if (a.pre_gn) b.da = pl.alloc(a.gap ? a.C : a.in_elems());
    if (s < S - 1) b.gradbox = pl.alloc(2 * (int64_t)a.out_elems());
    if (a.tap_dist) b.skg = pl.alloc((int64_t)(a.tap_dist + 1) * a.in_elems());
    if (a.proj) b.projy = pl.alloc(a.out_elems());
    if (split_candidate(a)) b.gparts = pl.alloc((int64_t)GRAD_PARTS * a.padded);
    if (fwd_split_candidate(a)) b.zparts = pl.alloc((int64_t)FWD_PARTS * a.z_elems());
    if (bwd_split_consumer(st, s)) b.dxparts = pl.alloc((int64_t)FWD_PARTS * a.out_elems());
    if (a.ce) { b.logits = pl.alloc(a.K); b.dlogits = pl.alloc(a.K); }
  }
  L.staging = pl.alloc(st[0].in_elems());
  L.labels = pl.alloc(S);
  L.loss = pl.alloc(loss_cap);
  L.globals = pl.alloc(64);
  L.zero = pl.alloc(64);
  L.sync = pl.alloc(SYNC_CNT + MAX_SYNC_PHASES * S);
}

// ---------------------------------------------------------------- context
struct Phase {
  std::vector<int> step_idx;       // indices into steps, in launch order
  int first = 0, count = 0, tiles = 0;
  bool fused = false;              // holds several phases: its workgroups wait for each other through completion counters
};

}  // namespace

struct pb_ctx {
  std::vector<Stage> st;
  int S = 0;
  int mitigation = 3;
  float lr = 0, m = 0;
  int loss_cap = 0;
  int64_t n_params = 0;
  Layout L;
  float* arena = nullptr;
  bool own_arena = false;
  int static_dev = -1;       // >= 0: the context lives in the library's static arena of that device
  hipStream_t stream = nullptr;
  int64_t ticks = 0;
  int launch_mode = 0;
  int kernel_set = 0;
  bool nt_stores = false;   // launch the kernel instantiation with non-temporal output stores
  bool sequential = false;   // sample-indexed form: one sample through all stages per tick (delays below the pipeline's own)
  bool lwp_w = false;  // LWP in its weight-difference form
  double sc_scale = 1.0, lwp_scale = 1.0;   // over-compensation factors on the stage delay
  bool stash = false;  // weight stashing: the backward pass reads the predicted weights its forward pass used
  bool bf16 = false;   // bf16 activation mode: tensors that cross a stage boundary are rounded to bf16
  int N = 1;           // update size: samples per update
  pb_tuning tune = {0, 0, 0.f, 0, 0, 0, 0, 0, 0};
  std::vector<char> pp_active;   // per stage: the update alternates between two copies of the master parameters
  int fuse_from = -1;          // >= 0: the phases from this one on share one launch, dependencies through completion
                               // counters (0: one launch per tick)
  uint32_t fused_ticks = 0;    // ticks launched in that form so far
  int32_t* sync_dev = nullptr; // error word, wait bound, counters
  std::vector<StepDesc> steps;         // sorted by phase
  std::vector<int64_t> rec_first;      // per step: index of its first per-workgroup record
  Plan* plan = nullptr;                // arena allocator while the step table is compiled
  std::vector<std::pair<int64_t, std::vector<int32_t>>> tables;   // (arena offset, contents) of the GEMM offset tables
  std::vector<Phase> phases;
  // device views
  StepDesc* recs_dev = nullptr;        // one descriptor copy per workgroup, in launch order
  Globals* globals_dev = nullptr;
  int32_t* zero_dev = nullptr;
  int32_t* labels_dev = nullptr;
  // resident-pool bookkeeping
  const float* pool = nullptr;
  const int32_t* pool_labels = nullptr;
  int n_pool = 0;
  int idx_base = 0;
  // host-fed ticks: the sample goes through a ring of pinned host buffers, so that the copy to the
  // device is asynchronous and the caller's buffer is free again when pb_tick returns
  static constexpr int N_PINNED = 8;
  float* pinned[N_PINNED] = {};
  hipEvent_t pinned_done[N_PINNED] = {};
  bool pinned_used[N_PINNED] = {};
  int pinned_next = 0;
  // profiling
  bool profiling = false;
  int max_events = 0;
  struct Ev { hipEvent_t a, b; int cls; };
  std::vector<Ev> evs;
  std::vector<Ev> ev_pool;
  float* f(int64_t off) const { return arena + off; }
};

namespace {

// the settings of the descriptor that shape the plan
void take_settings(pb_ctx* c, const pb_net_desc* net) {
  c->kernel_set = net->kernel_set;
  c->bf16 = net->act_dtype == 1;
  c->stash = net->bwd_weights == 1;
  c->N = net->update_size > 1 ? net->update_size : 1;
  if (net->tuning) c->tune = *net->tuning;
}

TRef ring(const pb_ctx* c, int64_t off, int depth, int stride, int lag) {
  TRef r;
  r.base = c->f(off); r.depth = depth; r.stride = stride; r.lag = lag; r.pad_ = 0;
  return r;
}

StepDesc blank(int kind, int stage, int first_tick) {
  StepDesc d;
  memset(&d, 0, sizeof d);
  d.kind = kind; d.stage = stage; d.first_tick = first_tick;
  d.x.depth = d.st.depth = d.y.depth = d.dy.depth = d.dx.depth = d.skip.depth = d.skg.depth = 1;
  return d;
}

int cdiv(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

// Streaming forms of the elementwise steps (networks tiled for throughput):
// floats per workgroup, and whether a ring can be read with 16-byte accesses.
constexpr int STREAM_GRAIN = 4 * 4 * BLK;
// (out of line, on integers: see arena_aligned16)
__attribute__((noinline)) bool ref_vec4(const pb_ctx* c, const TRef& r) {
  return (uintptr_t)r.base != 0 && ((uintptr_t)r.base - (uintptr_t)c->f(0)) % 16 == 0 && (r.depth == 1 || r.stride % 4 == 0);
}

int bwd_w_tiles(int K, int C, int k, int P, bool bias) {
  const int64_t nW = (int64_t)K * C * k * k;
  const int per = P > 16 ? BLK / 64 : BLK;
  return cdiv(nW, per) + (bias ? cdiv(K, per) : 0);
}

void sc_coeffs(double m, double D, double* a, double* b) {
  *a = (D == 0.0) ? 1.0 : pow(m, D);
  *b = (m == 1.0) ? D : (1.0 - *a) / (1.0 - m);
}

// ---------------------------------------------------------- GEMM tiling
int pow2_floor(int x) { int p = 1; while (p * 2 <= x) p *= 2; return p; }

// Tiling of one implicit-GEMM operand set.  mode 1 forward, 2 backward data,
// 3 backward weights.
int g_tile_target_bwd = 8; // ... of a backward step (a stage has two of them in the same phase)
int g_tile_target = 8;     // latency policy: workgroups a step is split into at least, when its shape allows
int g_gemm_lds = 15872;        // floats of LDS a GEMM tile is planned with (the kernel's array holds LDS_FLOATS)
double g_tile_budget_us = 0;   // throughput policy (> 0): longest tile a step should have, microseconds (estimate)
double g_budget_scale[4] = {1.0, 1.0, 1.0, 1.0};   // ... times this factor for the steps of a pass (index: GEMM mode), see compile_steps

// Given the wave arrangement (wm, wn, wk, ni), choose the chunking of the
// reduction that fits the LDS budget.  `fine`: search the channel count of a
// chunk in steps of 4 (else by halving).  Returns false if nothing fits.
// Rows of a map of row length `rowlen` that NT consecutive pixels starting at a
// multiple of NT can touch.
static int tile_rows(int NT, int rowlen, int nrows) {
  int r = (NT + rowlen - 2) / rowlen + 1;
  if (rowlen % NT == 0) r = 1;
  else if (NT % rowlen == 0) r = NT / rowlen;
  return std::min(nrows, r);
}

bool fit_gemm(GemmCfg& g, int C, int H, int W, int K, int OH, int OW, int k, int s, int pad, bool allow_vec, bool fine,
              int rows_cap = 0) {
  const int mode = g.gm, kk = k * k;
  g.MT = 16 * g.wm; g.NT = 16 * g.ni * g.wn;
  if (g.nsub < 1 || g.wk != 1) g.nsub = 1;   // the split of the reduction reuses the A block's LDS
  if (mode == 3) g.win = 0;
  g.nsub = std::min(g.nsub, cdiv(g.N, g.NT));
  g.tiles_n = cdiv(cdiv(g.N, g.NT), g.nsub);
  g.tiles = cdiv(g.M, g.MT) * g.tiles_n;
  // 16-byte row copies: source rows a multiple of 4 floats wide, no transform
  // while staging, and (backward data) unit stride so that no zeros interleave
  const int hl = (mode == 2) ? k - 1 - pad : pad;
  g.vec = 0;
  if (allow_vec && hl <= 4) {
    if (mode == 2) g.vec = (s == 1 && OW % 4 == 0) ? 1 : 0;
    else g.vec = (W % 4 == 0) ? 1 : 0;
  }
  if (mode == 2 && s > 1) g.vec = (s == 2 && hl <= 1 && OW % 2 == 0) ? 3 : 2;   // 3: pairs of gradient values per 16-byte vector
  g.xoff = g.vec == 1 ? 4 - hl : 0;
  // LDS per chunk: offset table, A block, patch
  auto a_size = [&](int QC) -> int64_t {
    const int QCpad = (QC + 15) / 16 * 16;
    if (mode == 2) return (int64_t)((QCpad + kk - 1) / kk + 1) * g.MT * kk;
    return (int64_t)g.MT * (QCpad + 4);
  };
  auto fits = [&](int QC, int CC, int PR, int Wp) {
    const int QCpad = (QC + 15) / 16 * 16;
    const int64_t need = QCpad + a_size(QC) + ((int64_t)CC * PR * Wp + 3) / 4 * 4 + 16;
    return need <= g_gemm_lds;
  };
  if (mode == 1 || mode == 2) {
    const int rowlen = mode == 1 ? OW : W, nrows = mode == 1 ? OH : H;
    const int rows_max = tile_rows(g.NT, rowlen, nrows);
    g.PR = mode == 1 ? (rows_max - 1) * s + k : rows_max + k - 1;
    g.Wp = mode == 1 ? W + 2 * pad : W + k - 1;
    if (g.vec == 1) g.Wp = (mode == 1 ? W : OW) + 8;
    if (g.vec == 3) g.Wp = (g.Wp + 3) / 4 * 4;
    if (g.win) {   // flattened 1x1 layer: one row, only the tile's own columns
      if (g.vec != 1 || H != 1 || OH != 1 || k != 1 || s != 1 || pad != 0) return false;
      g.win = g.NT; g.Wp = g.NT + 8;
    }
    const int nch = mode == 1 ? C : K;
    int CC = nch;
    if (fine) {
      while (CC > 1 && !fits(CC * kk, CC, g.PR, g.Wp)) CC = CC > 4 ? (CC - 1) / 4 * 4 : CC - 1;
      if (CC >= 1 && fits(CC * kk, CC, g.PR, g.Wp) && CC < nch) {
        // even out the chunks
        const int n = cdiv(nch, CC);
        int even = cdiv(nch, n);
        if (even > 4) even = (even + 3) / 4 * 4;
        if (even <= CC) CC = even;
      }
    } else {
      while (CC > 1 && !fits(CC * kk, CC, g.PR, g.Wp)) CC = (CC + 1) / 2;
      if (CC > 4) CC = CC / 4 * 4;   // keeps the chunks of a row 16-byte aligned
    }
    if (CC < 1 || !fits(CC * kk, CC, g.PR, g.Wp)) return false;
    g.CC = CC; g.QC = CC * kk; g.n_chunks = cdiv(nch, CC); g.rows_c = 0;
  } else {
    g.CC = std::min(C, (g.NT + kk - 2) / kk + 1);
    g.Wp = g.vec ? W + 8 : W + 2 * pad;
    auto pr = [&](int r) { return (r - 1) * s + k; };
    // one chunk holding every output row, else the largest row count whose
    // pixel count is a multiple of 4 (chunks in the middle must not be padded)
    // (rows_cap > 0: at most that many rows per chunk, for a reduction split over workgroups)
    int rows = 0;
    const int cap = rows_cap > 0 ? std::min(OH, rows_cap) : OH;
    if (cap == OH && fits(OH * OW, g.CC, pr(OH), g.Wp)) {
      rows = OH;
    } else {
      int step = 1;
      while ((step * OW) % 4) ++step;
      for (int r = step; r < OH && r <= std::max(cap, step); r += step) {
        if (!fits(r * OW, g.CC, pr(r), g.Wp)) break;
        rows = r;
      }
    }
    if (!rows) return false;
    g.rows_c = rows; g.QC = rows * OW; g.PR = pr(rows); g.n_chunks = cdiv(OH, rows);
  }
  g.QCpad = (g.QC + 15) / 16 * 16;
  g.parts = 1; g.cpp = g.n_chunks; g.tpp = g.tiles;
  // 16-byte fetches of the A block: every segment starts on a 16-byte boundary and
  // has a length that is a multiple of 4 (the caller withdraws this if the operand's
  // address does not allow it).  Forward / backward weights: segments are rows of the
  // reduction range; backward data: the MT x k x k weights of one output channel.
  if (mode == 2) g.avec = (C % 4 == 0) ? 1 : 0;
  else g.avec = (g.Q % 4 == 0 && (g.n_chunks == 1 || g.QC % 4 == 0)) ? 1 : 0;
  {
    const int q4 = (mode == 2) ? (g.QC + 3) / 4 * 4 : g.QCpad;
    const int64_t nseg = (mode == 2) ? (q4 + kk - 1) / kk : g.MT, seg = (mode == 2) ? g.MT * kk : q4;
    g.a_req = (int)cdiv(nseg * (g.avec ? (seg + 3) / 4 : seg), BLK);
  }
  g.LDA = (mode == 2) ? g.MT * kk : g.QCpad + 4;   // QCpad + 4 = 4 * odd: the 16 rows of a wave fall into different banks
  g.o_offq = 0;
  g.o_A = g.QCpad;
  g.o_patch = (int)(g.o_A + a_size(g.QC));
  if (g.o_patch % 4 || g.o_patch + (g.CC * g.PR * g.Wp + 3) / 4 * 4 > g_gemm_lds) return false;
  return true;
}

// Estimated duration of one tile, microseconds: a fixed part (descriptor, offset
// tables, epilogue), per chunk a fixed part, the staging of the A block and the
// patch (instruction-bound: counted in 16-byte requests per thread, of which the
// first 6 + 6 are prefetched while the previous chunk is contracted) and the
// MFMA loop, whose cost per MFMA falls with the number of column subtiles a
// wave keeps (one A fetch and one offset fetch per k-step whatever their number).
double est_tile_us(const GemmCfg& g, int k) {
  if (g.mm) {
    // dense form: per chunk of 32 reduction entries 8 mi ni MFMAs per wave, two workgroups sharing the matrix pipes,
    // and never less than the round trip of the next chunk's requests
    const double t_mfma = 2.0 * 8.0 * g.mi * g.ni * 32.0 / 2400.0;
    return 5.0 + g.n_chunks * std::max(2.2, t_mfma);
  }
  const int kk = k * k;
  const double a_fl = g.gm == 2 ? (double)((g.QCpad + kk - 1) / kk + 1) * g.MT * kk : (double)g.MT * g.QCpad;
  const double p_fl = (double)g.CC * g.PR * g.Wp;
  const double a_sl = a_fl / (g.avec ? 4 : 1) / BLK, p_sl = p_fl / ((g.vec == 1 || g.vec == 3) ? 4 : 1) / BLK;
  const double stage_a = 0.1 * std::min(a_sl, 6.0) + 0.3 * std::max(0.0, a_sl - 6.0);
  const double stage_p = g.vec == 1 ? 0.1 * std::min(p_sl, 6.0) + 0.3 * std::max(0.0, p_sl - 6.0) : 0.3 * p_sl;
  const double mf = (double)cdiv(cdiv(std::min(g.QC, g.Q), 4), g.wk) * g.ni;
  const double t_mfma = mf * (32.0 + 70.0 / g.ni) / 2400.0;
  const double t_chunk = 3.0 + stage_a + stage_p + t_mfma;   // fixed part: two barriers, the request code, fill and drain of the MFMA pipeline
  double t = 4.0 + g.n_chunks * t_chunk + (g.wk > 1 ? 0.5 : 0.0);
  // further column tiles of a backward-weights workgroup: no descriptor, no tables,
  // the patch already requested; the A block again only if the reduction is chunked
  if (g.nsub > 1) t += (g.nsub - 1) * (g.n_chunks * (2.5 + (g.n_chunks > 1 ? stage_a : 0.0) + stage_p + t_mfma) + 1.0);
  return t;
}

// Whether p lies a multiple of 16 bytes into the arena.  (Out of line and on integers: while a plan is only being
// sized the arena's base is null, and comparisons on pointers derived from it are not reliable after optimisation.)
__attribute__((noinline)) bool arena_aligned16(const pb_ctx* c, const float* p) {
  return ((uintptr_t)p - (uintptr_t)c->f(0)) % 16 == 0;
}

// Dense matrix-product form of a layer (pb_mm.h) in a network tiled for throughput: M x N result, reduction Q.
//   forward           M = cout, N = output pixels,  Q = cin k k   (a multiple of 32)
//   backward data     M = cin,  N = input pixels,   Q = cout k k  (a multiple of 32); k > 1: stride 1 only
//   backward weights  M = cout, N = cin k k (a multiple of 64), Q = output pixels, its chunks dealt out to up to
//                     max_parts groups of workgroups
// M is a multiple of 64.  A 1x1 layer of stride 1 whose map has a multiple of 4 pixels is a plain product of matrices
// as they lie in memory; every other shape gathers its pixel-indexed operand element by element (a 1x1 layer of
// stride 2, H = 2 OH, W = 2 OW, runs its backward data over the output pixels and scatters).
bool make_mm(const pb_ctx* c, int mode, int C, int H, int W, int K, int OH, int OW, int k, int stride, int pad, int max_parts,
             GemmCfg* out) {
  if (g_tile_budget_us <= 0 || c->kernel_set != 0 || c->tune.dense_1x1 < 0) return false;
  if (k < 1 || k > 7 || pad < 0 || pad >= k || (stride != 1 && stride != 2)) return false;
  if (k == 1 && stride == 2 && !(H == 2 * OH && W == 2 * OW)) return false;
  // k x k layers: their pixel-indexed operand would be gathered tap by tap, nine requests for what the patch-based tiles
  // fetch once and reuse from LDS -- measured 1.3 (ResNet-50) to 2.8 (VGG-11) times the tick of the patch-based tiles.
  // Planned only on request (pb_tuning.dense_1x1 = 2: forward and backward weights), which keeps the geometry tested.
  if (k > 1 && (mode == 2 || c->tune.dense_1x1 != 2)) return false;
  if (k == 1 && stride == 1 && (H != OH || W != OW || pad != 0)) return false;
  const int kk = k * k, P = OH * OW, HW = H * W;
  const int M = mode == 2 ? C : K;
  const int N = mode == 1 ? P : mode == 2 ? (k == 1 ? P : HW) : C * kk;
  const int Q = mode == 1 ? C * kk : mode == 2 ? K * kk : P;
  if (M % 64 || M < 64 || (int64_t)K * C * kk >= ((int64_t)1 << 30) || (int64_t)std::max(C, K) * std::max(HW, P) >= ((int64_t)1 << 30)) return false;
  if (mode == 3 ? (N % 64 || N < 64 || Q < 4) : (N < 16 || Q % MM_QC || Q < MM_QC)) return false;
  if (std::max(N, Q) >= (1 << 20)) return false;   // (index divisions in the kernel are exact below 2^21)
  GemmCfg g;
  memset(&g, 0, sizeof g);
  g.gm = mode; g.mm = 1; g.M = M; g.N = N; g.Q = Q;
  g.ps = stride; g.ck = k; g.cpad = pad;
  if (k == 1 && stride == 1) { g.pw = P; g.sw = HW; g.sh = 1; g.shw = HW; }          // the map as one row
  else if (mode == 2 && k > 1) { g.pw = W; g.sw = OW; g.sh = OH; g.shw = P; }          // pixel space: the input map; source: dY
  else { g.pw = OW; g.sw = W; g.sh = H; g.shw = HW; }                                  // pixel space: the output map; source: the input
  g.gather = k > 1 ? 1 : mode == 2 ? (P % 4 != 0) : (stride == 2 || P % 4 != 0);
  g.mi = M % 128 == 0 ? 4 : 2;
  g.ni = mode == 3 ? (N % 128 == 0 ? 4 : 2) : (N > 64 ? 4 : 2);
  if (mode != 3 && g.mi == 2 && g.ni == 2) return false;   // (no 64 x 64 tiles for these two passes)
  g.wm = 2; g.wn = 2; g.wk = 1; g.nsub = 1;
  g.MT = 32 * g.mi; g.NT = 32 * g.ni;
  if (2 * mm_chunk_floats(mode, g.MT, g.NT) > LDS_FLOATS) return false;
  g.tiles_n = cdiv(N, g.NT);
  g.tpp = (M / g.MT) * g.tiles_n;
  g.QC = g.QCpad = MM_QC; g.n_chunks = cdiv(Q, MM_QC);
  g.parts = 1; g.cpp = g.n_chunks;
  if (mode == 3) {
    GemmCfg one = g;
    for (int want = 2; want <= max_parts && want <= g.n_chunks && est_tile_us(one, 1) > 30.0; want *= 2) {
      g.cpp = cdiv(g.n_chunks, want);
      g.parts = cdiv(g.n_chunks, g.cpp);
      one.n_chunks = g.cpp;
    }
  }
  g.tiles = g.parts * g.tpp;
  *out = g;
  return true;
}

// Choose the wave arrangement and the chunking of one operand set.  `like` !=
// nullptr forces the wave arrangement of an existing configuration (projection
// accumulated into the same tile).  Returns false if no chunking fits the LDS
// budget.
//   Latency policy (small networks): at least g_tile_target tiles per step, rows
//   first.  Throughput policy (g_tile_budget_us > 0): of all arrangements whose
//   estimated tile duration stays within the budget, the one with the least total
//   work (tiles x duration); if none does, the one with the shortest tile.
bool make_gemm(int mode, int C, int H, int W, int K, int OH, int OW, int k, int s, int pad,
               const GemmCfg* like, GemmCfg* out, bool allow_vec = false, int max_sub = 16, bool flat = false,
               int max_parts = 1) {
  const int target = (mode == 1) ? g_tile_target : g_tile_target_bwd;
  GemmCfg g;
  memset(&g, 0, sizeof g);
  g.gm = mode;
  g.win = flat ? 1 : 0;
  const int kk = k * k, P = OH * OW, HWi = H * W;
  if (mode == 1) { g.M = K; g.N = P; g.Q = C * kk; }
  else if (mode == 2) { g.M = C; g.N = HWi; g.Q = K * kk; }
  else { g.M = K; g.N = C * kk; g.Q = P; }
  const int mt = cdiv(g.M, 16), n16 = cdiv(g.N, 16);
  if (!like && g_tile_budget_us <= 0 && mode == 3 && max_parts > 1 && g.Q >= 256) {
    // Latency policy, weight gradient over a large map: split the reduction (the output
    // rows) over 4 or 8 groups of workgroups, each small enough that one burst of requests
    // (about 8 per thread) brings in its rows of dZ and of the input; every group covers
    // all columns with as few tiles as the wave arrangement allows.
    GemmCfg t = g;
    t.wm = mt >= 4 ? 4 : mt >= 2 ? 2 : 1;
    const int rest = 4 / t.wm;
    t.wn = std::min(rest, pow2_floor(n16)); t.wk = rest / t.wn;
    t.ni = std::min(4, cdiv(n16, t.wn));
    if (t.ni == 3) t.ni = 4;
    const int NT = 16 * t.ni * t.wn, CC = std::min(C, (NT + kk - 2) / kk + 1), Wp = W + 8;
    int rows = OH;
    while (rows > 1 && cdiv(OH, rows) < std::min(max_parts, 8) &&
           (int64_t)16 * t.wm * rows * OW + (int64_t)CC * ((rows - 1) * s + k) * Wp > 8192) rows = (rows + 1) / 2;
    if (cdiv(OH, rows) >= 4 && fit_gemm(t, C, H, W, K, OH, OW, k, s, pad, allow_vec, false, rows) && t.n_chunks >= 4) {
      t.cpp = cdiv(t.n_chunks, std::min(max_parts, t.n_chunks));
      t.parts = cdiv(t.n_chunks, t.cpp);
      t.tpp = t.tiles;
      t.tiles = t.parts * t.tpp;
      *out = t;
      return true;
    }
  }
  if (like) {
    g.wm = like->wm; g.wn = like->wn; g.wk = like->wk; g.ni = like->ni;
  } else if (g_tile_budget_us > 0) {
    bool have = false;
    double best_work = 0, best_tile = 0;
    bool best_within = false;
    GemmCfg bestg;
    for (int wm = 1; wm <= 4; wm *= 2)
      for (int wn = 1; wm * wn <= 4; wn *= 2) {
        const int wk = 4 / (wm * wn);
        if (wm > 1 && 16 * (wm / 2) >= 16 * mt) continue;            // waves without rows
        if (wk > 1 && g.Q < 64 * wk) continue;
        for (int ni = 1; ni <= 4; ni *= 2)
        for (int nsub = 1; nsub <= (wk == 1 ? max_sub : 1); nsub *= 2) {
          if (wn * ni > 1 && (wn * ni) / 2 >= n16) continue;         // subtiles without columns
          if (nsub > 1 && 16 * ni * wn * (nsub / 2) >= g.N) continue; // column tiles beyond the last column
          GemmCfg c = g;
          c.wm = wm; c.wn = wn; c.wk = wk; c.ni = ni; c.nsub = nsub;
          if (!fit_gemm(c, C, H, W, K, OH, OW, k, s, pad, allow_vec, true)) continue;
          // backward weights of a stage with room for partial gradients: the chunks of the
          // reduction are dealt out to as many groups of workgroups (up to max_parts) as it
          // takes to bring one workgroup's share under 30 us
          GemmCfg e = c;
          double tt = est_tile_us(c, k);
          for (int want = 2; nsub == 1 && want <= max_parts && want <= c.n_chunks && tt > (mode == 3 ? 30.0 : 12.0); want *= 2) {
            e = c;
            e.cpp = cdiv(c.n_chunks, want);
            e.parts = cdiv(c.n_chunks, e.cpp);
            e.tiles = e.parts * e.tpp;
            GemmCfg one = e;
            one.n_chunks = e.cpp;   // what one workgroup contracts
            tt = est_tile_us(one, k);
          }
          const double work = tt * e.tiles;
          const bool within = tt <= g_tile_budget_us * g_budget_scale[mode];
          bool better;
          if (!have) better = true;
          else if (within != best_within) better = within;
          else if (within) better = work < best_work || (work == best_work && tt < best_tile);
          else better = tt < best_tile;
          if (better) { have = true; bestg = e; best_work = work; best_tile = tt; best_within = within; }
        }
      }
    if (!have) return false;
    *out = bestg;
    return true;
  } else {
    g.wm = mt >= 4 ? 4 : mt >= 2 ? 2 : 1;
    const int rest = 4 / g.wm;
    if (mode == 3 && g.Q >= 256) { g.wk = rest; g.wn = 1; }
    else { g.wn = std::min(rest, pow2_floor(n16)); g.wk = rest / g.wn; }
    g.ni = std::min(4, cdiv(n16, g.wn));
    auto tiles = [&]() { return cdiv(g.M, 16 * g.wm) * cdiv(g.N, 16 * g.ni * g.wn); };
    if (g.ni == 3) g.ni = 4;   // the kernels are instantiated for 1, 2 and 4 subtiles
    while (tiles() < target && g.ni > 1) g.ni /= 2;
    while (tiles() < target && g.wm > 1 && g.Q >= 64 * g.wk * 2) { g.wm /= 2; g.wk *= 2; }
    while (tiles() < target && g.wn > 1 && g.Q >= 64 * g.wk * 2) { g.wn /= 2; g.wk *= 2; }
    // the same tile with two column subtiles per wave and the reduction split once more: the A values and patch offsets
    // a wave fetches per k-step then feed two MFMAs (ResNet-20 23.4 -> 23.2 us per tick)
    if (g.wn >= 2 && g.ni == 1 && g.Q >= 64 * g.wk * 2) { g.wn /= 2; g.ni = 2; g.wk *= 2; }
  }
  if (!fit_gemm(g, C, H, W, K, OH, OW, k, s, pad, allow_vec, like && g_tile_budget_us > 0)) return false;
  *out = g;
  return true;
}

// Offset tables of one GEMM operand set (see pb_gemm.h): tq maps the
// chunk-relative reduction index, tn the column index, to offsets into the
// LDS patch.  They depend on the step only, not on the tile.
void gemm_tables(pb_ctx* c, const GemmCfg& g, int C, int H, int W, int K, int OH, int OW, int k, int s,
                 const int32_t** tq, const int32_t** tn) {
  const int kk = k * k, PRW = g.PR * g.Wp;
  std::vector<int32_t> q(g.QCpad, 0), n(g.N, 0);
  for (int i = 0; i < g.QC; ++i) {
    if (g.gm == 3) { const int r = i / OW, ow = i % OW; q[i] = r * s * g.Wp + ow * s; }
    else {
      const int cc = i / kk, tap = i % kk, kh = tap / k, kw = tap % k;
      q[i] = (g.gm == 1) ? cc * PRW + kh * g.Wp + kw : cc * PRW + (k - 1 - kh) * g.Wp + (k - 1 - kw);
    }
  }
  for (int i = 0; i < g.N; ++i) {
    if (g.gm == 1) { const int oh = i / OW, ow = i % OW; n[i] = oh * s * g.Wp + ow * s; }
    else if (g.gm == 2) { const int ih = i / W, iw = i % W; n[i] = ih * g.Wp + iw; }
    else { const int ci = i / kk, tap = i % kk, kh = tap / k, kw = tap % k; n[i] = ci * PRW + kh * g.Wp + kw; }
  }
  const int64_t oq = c->plan->alloc((int64_t)q.size()), on = c->plan->alloc((int64_t)n.size());
  c->tables.push_back({oq, std::move(q)});
  c->tables.push_back({on, std::move(n)});
  *tq = (const int32_t*)c->f(oq);
  *tn = (const int32_t*)c->f(on);
  (void)C; (void)H; (void)K; (void)OH;
}

// A dense layer on one sample (1x1 maps on both sides) whose operands allow 16-byte accesses: its three passes
// run as matrix-vector steps (K_FC_*) in networks tiled for throughput.
// (Kept out of line: inlined into the planner, hipcc 7.2 -O3 evaluated it to false at the weight-gradient call site
// with every one of its terms true; out of line it is right at all three.)
__attribute__((noinline)) bool fc_layer(const pb_ctx* c, const StepDesc& d, const float* w) {
  return c->kernel_set == 0 && g_tile_budget_us > 0 && d.H == 1 && d.W == 1 && d.OH == 1 && d.OW == 1 && d.k == 1 && d.stride == 1 &&
         d.pad == 0 && d.C % 4 == 0 && d.C >= 256 && d.K >= 1 && d.K <= 8192 && (int64_t)d.K * d.C < ((int64_t)1 << 30) &&
         w && ((uintptr_t)w - (uintptr_t)c->f(0)) % 16 == 0 && ((d.pmask & PF_W) == 0 || d.pstride % 4 == 0);
}

// Whether the A operand of a GEMM step (of its projection operand set if
// `second`) starts on a 16-byte boundary in every ring slot.
bool a_aligned(const pb_ctx* c, const StepDesc& d, bool second) {
  const float* p = second ? d.wp : (d.g.gm == 3 ? d.dy.base : d.w);
  if (!p || (p - c->f(0)) % 4) return false;
  return second || d.g.gm != 3 || d.dy.stride % 4 == 0;
}

// Limits of the fused last stage (one workgroup; see step_head): sizes of its
// register and LDS arrays.
constexpr int HEAD_MAX_IN = 8192, HEAD_MAX_CV = 512, HEAD_MAX_K = 16;
bool head_fits(int C, int HW, int K, bool gap, int G) {
  const int64_t n_in = (int64_t)C * HW, cv = gap ? C : n_in;
  if (cv > HEAD_MAX_CV || K > HEAD_MAX_K || C > 2 * BLK || G > BLK || G < 1 || C % G) return false;
  const int64_t tail = 2 * HEAD_MAX_CV + 2 * HEAD_MAX_K + 9 * (int64_t)C + 2 * G;
  // pooled form on maps of a multiple of 4 pixels (step_head_gap4): the input stays in registers
  // (up to 16 vectors per thread), LDS holds two partial sums per 4 elements
  if (gap && HW % 4 == 0) return n_in <= 2 * HEAD_MAX_IN && 2 * (n_in / 4) + tail <= LDS_FLOATS;
  return n_in <= HEAD_MAX_IN && (n_in + 3) / 4 * 4 + tail <= LDS_FLOATS;
}

// Coefficients of the stage's update (Eqs. gscv, gscw, scd, lwp_v_form) by mitigation mode.
void set_update_coeffs(const pb_ctx* c, const Stage& a, StepDesc* d) {
  double ca = 1.0, cb = 0.0;
  const double Du = c->N > 1 ? (double)a.De / c->N : (double)a.De;   // the stage's delay counted in updates
  if (c->mitigation == 1 || c->mitigation == 3) sc_coeffs((double)c->m, c->sc_scale * Du, &ca, &cb);
  const double T = (c->mitigation >= 2) ? c->lwp_scale * Du : 0.0;
  d->fa = (float)ca; d->fb = (float)cb; d->flrT = (float)((double)c->lr * T); d->flr = c->lr; d->fm = c->m;
  if (c->lwp_w) { d->flags |= F_LWP_W; d->flrT = (float)T; }   // w_hat = w' + T (w' - w)
}

// Whether the GroupNorm backward of a C x HW map in G groups can run as one
// workgroup per group (see step_gn_bwd): group in registers, slots inside a channel.
constexpr int GNB_MAX_N = 4096;
bool gn_bwd_fits(int C, int HW, int G) {
  if (G < 1 || C % G || HW % 4) return false;
  const int cpg = C / G;
  const int64_t n = (int64_t)cpg * HW;
  return n <= GNB_MAX_N && cpg <= BLK && n / 2 + 5 * cpg + 2 <= LDS_FLOATS;
}

// Streaming form of a K_GNB_APPLY step (see step_gnb_apply_stream): workgroups
// aligned to groups, STREAM_GRAIN floats each.
void stream_apply(const pb_ctx* c, StepDesc& e) {
  const int HW = e.H * e.W;
  if (g_tile_budget_us <= 0 || !(e.flags & F_DU_BUF) || HW % 4 || !ref_vec4(c, e.x) || !ref_vec4(c, e.dy) ||
      !ref_vec4(c, e.dx) || ((e.flags & F_ADD_SKG) && !ref_vec4(c, e.skg)))
    return;
  const int64_t gsz = (int64_t)(e.C / e.G) * HW;
  e.grain = STREAM_GRAIN;
  e.n = cdiv(gsz, e.grain);
  e.ntiles = e.G * e.n;
}

// Networks tiled for latency: the GroupNorm statistics of a layer of four small groups
// in one workgroup, a wavefront per group.
void gn_stats_wave(StepDesc& d) {
  const int64_t n = d.G > 0 ? (int64_t)(d.C / d.G) * d.H * d.W : 0;
  if (g_tile_budget_us > 0 || d.G < 1 || d.G > BLK / 64 || d.C / d.G > 64 || (d.H * d.W) % 4 || n > 4096) return;
  d.grain = 1;
  d.ntiles = 1;
}

// One wavefront per channel for a K_GNB_REDUCE step over a small map.
void wave_reduce(StepDesc& d) {
  // (a gradient routed back through a max-pool costs a window search per element: small maps only)
  if (g_tile_budget_us <= 0 || !(d.flags & (F_DU_BUF | F_DU_POOL)) || d.H * d.W > ((d.flags & F_DU_POOL) ? 64 : 1024)) return;
  d.grain = 1;
  d.ntiles = cdiv(d.C, GNB_WAVE_CH * (BLK / 64));
}

// Compile the network into the step table.  Every step carries the phase it
// may run in: steps of one stage's forward (or backward) chain depend on each
// other and get consecutive phases; different stages and the two passes of
// one stage are independent inside a tick (they work on different samples and
// read the start-of-tick weights), except for the last stage whose backward
// pass consumes the loss gradient of the same tick.
void compile_steps_once(pb_ctx* c, std::vector<std::pair<int, StepDesc>>& out);

// The step table of a tick.  Networks tiled for throughput are planned twice when the first plan leaves the chip
// partly empty: the tile budget makes tiles as large as it allows (least total work), which is right for a phase with
// more GEMM workgroups than the chip's 512 places and wrong for one with fewer -- there the phase lasts as long as its
// longest tile while places stay free.  The GEMM steps of such a pass are planned again with other budgets and the
// plan with the earliest estimated end of the phase is kept (wide network, forward pass: 205 tiles of 57 us -> 410 of
// 42 us, launch 71 -> 64 us).
void compile_steps(pb_ctx* c, std::vector<std::pair<int, StepDesc>>& out) {
  for (double& f : g_budget_scale) f = 1.0;
  compile_steps_once(c, out);
  if (g_tile_budget_us <= 0 || c->tune.tile_budget_us != 0.f || c->kernel_set != 0) return;
  std::vector<int> all, fwd, bwd;
  for (auto& p : out) {
    const StepDesc& d = p.second;
    if ((int)all.size() <= p.first) { all.resize(p.first + 1, 0); fwd.resize(p.first + 1, 0); bwd.resize(p.first + 1, 0); }
    const bool f = (d.kind == K_GEMM && d.g.gm == 1) || d.kind == K_DOT_FWD, b = (d.kind == K_GEMM && d.g.gm != 1) || d.kind == K_DOT_BWD_X;
    if (f || b) all[p.first] += d.ntiles;
    if (f) fwd[p.first] += d.ntiles;
    if (b) bwd[p.first] += d.ntiles;
  }
  if (all.empty()) return;
  const int pf = (int)(std::max_element(fwd.begin(), fwd.end()) - fwd.begin());
  const int pb = (int)(std::max_element(bwd.begin(), bwd.end()) - bwd.begin());
  // Candidates: a pass that fills fewer than 300 places (smaller budgets), a pass with somewhat more tiles than places
  // (up to 700; measured on a pass with 875 the estimate's choice was 2 % slower), which runs them in two rounds,
  // the second one short of tiles (larger budgets).  Each candidate plan is priced by the estimated end of the
  // pass's phase: its GEMM tiles dealt out, longest first, to 512 places.
  const bool cand_f = fwd[pf] > 0 && (all[pf] < 300 || (all[pf] > 512 && all[pf] < 700));
  const bool cand_b = bwd[pb] > 0 && pb != pf && (all[pb] < 300 || (all[pb] > 512 && all[pb] < 700));
  if (!cand_f && !cand_b) return;
  auto phase_end_us = [&](const std::vector<std::pair<int, StepDesc>>& v, int ph) {
    std::vector<double> dur;
    for (auto& p : v) {
      const StepDesc& d = p.second;
      if (p.first != ph) continue;
      double us = 0;
      if (d.kind == K_GEMM) {
        GemmCfg one = d.g;
        one.n_chunks = d.g.cpp;
        us = est_tile_us(one, d.k) + (d.gp.gm ? est_tile_us(d.gp, 1) : 0.0);
      } else if (d.kind == K_DOT_FWD || d.kind == K_DOT_BWD_X) {
        us = 12.0;
      } else {
        continue;
      }
      for (int i = 0; i < d.ntiles; ++i) dur.push_back(us);
    }
    std::sort(dur.begin(), dur.end(), std::greater<double>());
    std::vector<double> place(512, 0.0);   // (a heap would do; a phase has a few thousand tiles at most)
    std::make_heap(place.begin(), place.end(), std::greater<double>());
    double end = 0;
    for (double u : dur) {
      std::pop_heap(place.begin(), place.end(), std::greater<double>());
      place.back() += u;
      end = std::max(end, place.back());
      std::push_heap(place.begin(), place.end(), std::greater<double>());
    }
    return end;
  };
  double best_f = 1.0, best_b = 1.0, end_f = phase_end_us(out, pf), end_b = phase_end_us(out, pb);
  for (double f : {0.4, 0.5, 0.65, 0.8, 1.25, 1.5, 1.75, 2.0}) {
    std::vector<std::pair<int, StepDesc>> trial;
    for (double& q : g_budget_scale) q = 1.0;
    if (cand_f) g_budget_scale[1] = f;
    if (cand_b) g_budget_scale[2] = g_budget_scale[3] = f;
    c->tables.clear();
    compile_steps_once(c, trial);
    if (cand_f) { const double e = phase_end_us(trial, pf); if (e < 0.97 * end_f) { end_f = e; best_f = f; } }
    if (cand_b) { const double e = phase_end_us(trial, pb); if (e < 0.97 * end_b) { end_b = e; best_b = f; } }
  }
  g_budget_scale[1] = best_f;
  g_budget_scale[2] = g_budget_scale[3] = best_b;
  out.clear();
  c->tables.clear();
  compile_steps_once(c, out);
  for (double& f : g_budget_scale) f = 1.0;
}

void compile_steps_once(pb_ctx* c, std::vector<std::pair<int, StepDesc>>& out) {
  const int S = c->S;
  // all stages run concurrently: aim at a few workgroups per compute unit over
  // the whole phase rather than per step
  g_tile_target = std::max(4, std::min(32, 960 / (3 * S)));
  if (c->tune.tile_target > 0) g_tile_target = c->tune.tile_target;
  // the backward phase holds two GEMM steps per stage: fewer tiles each, so that the phase's workgroups
  // fit the 512 a chip holds at a time (ResNet-20: 16 / 9 measured 33.4 k ticks/s, 16 / 12 30.0 k, 16 / 8 27.0 k)
  g_tile_target_bwd = std::max(4, std::min(32, 540 / (3 * S)));
  if (c->tune.tile_target_bwd > 0) g_tile_target_bwd = c->tune.tile_target_bwd;
  // Networks whose tick is long compared with a launch are tiled for throughput:
  // the budget for the longest tile is the duration of a GEMM phase if the tick's
  // 6 flops per multiply-accumulate ran at a third of the fp32 MFMA peak, spread
  // over the two GEMM phases of a tick.
  {
    // (1x1 layers run as dense matrix products at about twice the rate of the patch-based tiles: counted half)
    double macs = 0;
    const bool dense = c->kernel_set == 0 && c->tune.dense_1x1 >= 0;
    for (const Stage& a : c->st) {
      macs += (double)a.K * a.OH * a.OW * a.C * a.k * a.k * (dense && a.k == 1 && a.K % 64 == 0 && a.C % 64 == 0 ? 0.5 : 1.0);
      if (a.proj) macs += (double)a.K * a.OH * a.OW * a.sC * (dense && a.K % 64 == 0 && a.sC % 64 == 0 ? 0.5 : 1.0);
    }
    const double tick_us = 6.0 * macs / 50e6;
    g_tile_budget_us = tick_us >= 10.0 ? std::max(16.0, 0.65 * tick_us) : 0.0;
    if (c->tune.tile_budget_us > 0.f) g_tile_budget_us = c->tune.tile_budget_us;
    else if (c->tune.tile_budget_us < 0.f) g_tile_budget_us = 0.0;
    // A compute unit has 160 KB of LDS and holds two workgroups: a tile may use up to 76 KB.  Planning with all of it
    // pays where the reductions are long (fewer chunks, each with its fixed costs: ResNet-50 +2.3 %, the wide ResNet
    // +0.7 % measured); for shorter ticks the planner's estimate favours arrangements that measure slower (VGG-11
    // -7.8 %), so those plan with 62 KB.
    g_gemm_lds = (c->tune.gemm_lds_kb == 76 || (c->tune.gemm_lds_kb == 0 && tick_us >= 60.0)) ? LDS_FLOATS : 15872;
  }
  const Layout& L = c->L;
  std::vector<int> bwd0(S, 0);   // per stage: phase its backward chain starts in
  // stages whose weight gradient is computed inside the update step (see F_WGRAD): the phase the
  // gradient's operands are complete in, and the operands
  struct FusedW { int phase = -1; TRef x, dy; int64_t pp = 0; };
  std::vector<FusedW> fusedw(S);
  c->pp_active.assign(S, 0);
  for (int s = 0; s < S; ++s) {
    const Stage& a = c->st[s];
    const StageBufs& b = L.sb[s];
    const int D = a.D;
    // slot 0 of the stage's ring of predicted weights; steps that read or write it carry a mask of the
    // pointer fields that k_phase has to move to the slot of the tick
    const float* wf = c->f(L.what[s]);                      // forward (predicted) parameters
    const float* wb = c->f(L.w + a.off);                    // backward (current) parameters
    const int wdepth = what_depth(a, c->stash);
    auto fwd_params = [&](StepDesc& d, int mask) {
      d.pmask = mask; d.pdepth = wdepth; d.plag = a.De - a.D; d.pstride = (int)a.padded;
    };
    auto writes_what = [&](StepDesc& d) {
      d.pmask = PF_WHAT; d.pdepth = wdepth; d.plag = -1; d.pstride = (int)a.padded;
    };
    // weights of a backward step: the current master weights, or with weight stashing the version the
    // sample's forward pass read, De updates ago, from the same ring
    const float* wbk = c->stash ? wf : wb;
    // (a stage with two copies of its master parameters: copy t mod 2)
    const int64_t pp_stride = (b.w2 >= 0 && !c->stash && c->N == 1 && c->kernel_set == 0 && g_tile_budget_us > 0 && !c->sequential)
                                  ? b.w2 - (L.w + a.off) : 0;
    auto bwd_params = [&](StepDesc& d, int mask) {
      if (!c->stash && pp_stride > 0) { d.pmask = mask; d.pdepth = 2; d.plag = 0; d.pstride = (int)pp_stride; }
      if (!c->stash) return;
      d.pmask = mask; d.pdepth = wdepth; d.plag = a.De; d.pstride = (int)a.padded;
    };
    float* gr = c->f(b.gparts >= 0 ? b.gparts : L.g + a.off);
    const bool seq = c->sequential;
    const int t_f = seq ? 0 : s, t_b = seq ? 0 : 2 * (S - 1) - s;
    const int ML = seq ? 0 : -1;                       // lag of the mailbox slot a producer writes (next tick's, or this tick's)
    auto SL = [&](int A) { return seq ? 0 : s - A; };   // lag of the skip tensor tapped at stage A
    auto TL = [&](int dist) { return seq ? 0 : dist; }; // lag of a skip gradient
    const int NS = seq ? 1 : S;                        // depth of the label ring / samples in flight before the loss
    const TRef x_f = ring(c, b.xring, D + 2, a.in_elems(), 0);
    const TRef x_b = ring(c, b.xring, D + 2, a.in_elems(), D);
    TRef y_out;   // where the stage output goes
    if (s < S - 1) y_out = ring(c, L.sb[s + 1].xring, c->st[s + 1].D + 2, a.out_elems(), ML);
    else y_out = ring(c, b.logits, 1, a.K, 0);
    int ph = 0;
    if (s == 0) {
      // the sample arrives in phase 0; the first stage's forward chain follows it
      StepDesc d = blank(K_INGEST, 0, 0);
      d.n = a.in_elems(); d.n_stages = NS;
      d.dx = x_f;
      d.labels = c->labels_dev;
      d.ntiles = cdiv(d.n, 4 * BLK);
      if (c->bf16) d.flags |= F_BF16_OUT;
      out.push_back({0, d});
      ph = 1;
    }
    // a small last stage runs as one workgroup: forward, loss and backward
    const bool fused_head = a.ce && c->kernel_set == 0 && !a.post_gn && !a.add && !a.is_conv && (a.gap ? a.pre_gn : !a.pre_gn) &&
                            head_fits(a.Cin, a.Hin * a.Win, a.K, a.gap, a.pre_gn ? a.G : 1) && s > 0;
    if (fused_head) {
      StepDesc d = blank(K_HEAD, s, t_f);
      d.C = a.Cin; d.H = a.Hin; d.W = a.Win; d.K = a.K; d.G = a.pre_gn ? a.G : 1;
      d.n_stages = NS; d.loss_cap = c->loss_cap;
      if (a.pre_gn) d.flags |= F_PRE_AFFINE;
      if (a.pre_relu) d.flags |= F_PRE_RELU;
      if (a.gap) d.flags |= F_DU_GAP;
      if (a.has_bias) { d.flags |= F_BIAS; d.b = wf + a.o_b; d.gb = gr + a.o_b; }
      d.x = x_f;
      d.w = wf + a.o_w; d.wp = wbk + a.o_w; d.gw = gr + a.o_w;
      if (a.pre_gn) {
        d.gamma = wf + a.o_gamma; d.beta = wf + a.o_beta;
        d.skip.base = const_cast<float*>(wbk + a.o_gamma);
        d.ggamma = gr + a.o_gamma; d.gbeta = gr + a.o_beta;
      }
      // d.wp, d.skip.base: the backward pass's weights (the last stage's own delay is 0, so with
      // stashing they are the very slot the forward pass reads)
      fwd_params(d, PF_W | (a.has_bias ? PF_B : 0) | (a.pre_gn ? PF_GAMMA | PF_BETA : 0) |
                        (c->stash ? PF_WP | (a.pre_gn ? PF_SKIPBASE : 0) : 0));
      d.dx = ring(c, L.sb[s - 1].gradbox, 2, a.in_elems(), ML);
      d.loss_log = c->f(L.loss);
      d.labels = c->labels_dev;
      d.ntiles = 1;
      if (c->bf16) d.flags |= F_BF16_OUT;
      out.push_back({0, d});
      continue;
    }
    // ------------------------------------------------------------ forward
    int fwd_parts = 1;   // > 1: the layer's forward GEMM leaves partial outputs (see fwd_split_candidate)
    if (a.pre_gn) {
      StepDesc d = blank(K_GN_STATS, s, t_f);
      d.C = a.Cin; d.H = a.Hin; d.W = a.Win; d.G = a.G;
      d.x = x_f; d.st = ring(c, b.prest, D + 1, b.st_stride, 0);
      d.gamma = wf + a.o_gamma; d.beta = wf + a.o_beta;
      fwd_params(d, PF_GAMMA | PF_BETA);
      if (b.aring >= 0) {
        d.y = ring(c, b.aring, D + 1, a.in_elems(), 0);
        if (a.pre_relu) d.flags |= F_PRE_RELU;
      }
      d.ntiles = a.G;
      gn_stats_wave(d);
      out.push_back({ph++, d});
    }
    if (a.gap) {
      StepDesc d = blank(K_GAP_FWD, s, t_f);
      d.C = a.Cin; d.H = a.Hin; d.W = a.Win; d.G = a.G;
      d.flags = F_PRE_AFFINE | (a.pre_relu ? F_PRE_RELU : 0);
      d.x = x_f; d.st = ring(c, b.prest, D + 1, b.st_stride, 0);
      d.y = ring(c, b.pooled, D + 1, a.C, 0);
      d.ntiles = a.Cin;
      out.push_back({ph++, d});
    }
    {
      StepDesc d = blank(K_CONV_FWD, s, t_f);
      d.C = a.C; d.H = a.H; d.W = a.W; d.K = a.K; d.OH = a.OH; d.OW = a.OW;
      d.k = a.k; d.stride = a.stride; d.pad = a.pad; d.G = a.G;
      if (a.gap) {
        d.x = ring(c, b.pooled, D + 1, a.C, 0);
      } else {
        d.x = x_f;
        if (b.aring >= 0) {
          d.x = ring(c, b.aring, D + 1, a.in_elems(), 0);     // already normalised and rectified
        } else {
          if (a.pre_gn) { d.flags |= F_PRE_AFFINE; d.st = ring(c, b.prest, D + 1, b.st_stride, 0); }
          if (a.pre_relu) d.flags |= F_PRE_RELU;
        }
      }
      d.w = wf + a.o_w;
      if (a.has_bias) { d.flags |= F_BIAS; d.b = wf + a.o_b; }
      if (a.post_gn) {
        d.y = ring(c, b.zring, D + 1, a.z_elems(), 0);
      } else {
        d.y = y_out;
        if (a.add) {
          const int A = a.skip_from;
          d.flags |= F_SKIP;
          d.skip = ring(c, L.sb[A].xring, c->st[A].D + 2, c->st[A].in_elems(), SL(A));
          d.sC = a.sC; d.sH = a.sH; d.sW = a.sW; d.sstride = a.sstride;
          if (a.proj) { d.flags |= F_PROJ; d.wp = wf + a.o_wp; }
          // The 1x1 projection of the skip tensor needs nothing the stage computes in this tick: when
          // the layer's GEMM is not the first step of the forward chain (pre-norm stages: the
          // statistics come first), the projection runs as a GEMM step of its own one phase earlier,
          // into a buffer that the layer's GEMM then adds like an identity skip.  Accumulated into the
          // same tile instead, it is a second operand set contracted after the first: 5 us more on the
          // two ResNet-20 stages that have one, which then set the length of the forward phase.
          if (a.proj && c->kernel_set == 0 && ph > 0 && b.projy >= 0) {
            StepDesc e = blank(K_CONV_FWD, s, t_f);
            e.C = a.sC; e.H = a.sH; e.W = a.sW; e.K = a.K; e.OH = a.OH; e.OW = a.OW;
            e.k = 1; e.stride = a.sstride; e.pad = 0; e.G = a.G;
            e.x = d.skip;
            e.w = wf + a.o_wp;
            fwd_params(e, PF_W);
            e.y = ring(c, b.projy, 1, a.out_elems(), 0);
            e.ntiles = cdiv((int64_t)a.K * a.OH * a.OW, BLK);
            GemmCfg ge, gd;
            const bool dense = arena_aligned16(c, e.w) && ref_vec4(c, e.x) &&
                               make_mm(c, 1, e.C, e.H, e.W, e.K, e.OH, e.OW, 1, e.stride, 0, 1, &gd);
            if (dense || make_gemm(1, e.C, e.H, e.W, e.K, e.OH, e.OW, 1, e.stride, 0, nullptr, &ge, true)) {
              if (dense) ge = gd;
              e.kind = K_GEMM; e.g = ge; e.ntiles = ge.tiles;
              if (!dense) gemm_tables(c, ge, e.C, e.H, e.W, e.K, e.OH, e.OW, 1, e.stride, &e.tq, &e.tn);
              out.push_back({ph - 1, e});
              d.flags &= ~F_PROJ;
              d.wp = nullptr;
              d.skip = e.y;
            }
          }
        }
      }
      fwd_params(d, PF_W | (a.has_bias ? PF_B : 0) | ((d.flags & F_PROJ) ? PF_WP : 0));
      d.ntiles = cdiv((int64_t)a.K * a.OH * a.OW, BLK);
      if (c->bf16 && !a.ce) d.flags |= F_BF16_OUT;   // the logits of the loss stage stay unrounded
      const bool dot_fwd = c->kernel_set == 0 && g_tile_budget_us > 0 && !c->bf16 && dot_layer(a) && !a.ce && ref_vec4(c, d.x);
      if (dot_fwd) {
        d.kind = K_DOT_FWD;
        d.n = a.H == 4 ? 4 : 8;            // output channels per workgroup
        d.ntiles = a.K / d.n;
      } else
      if (fc_layer(c, d, d.w) && !(d.flags & (F_PRE_AFFINE | F_PRE_RELU | F_SKIP | F_PROJ)) && ref_vec4(c, d.x)) {
        d.kind = K_FC_FWD;
        d.ntiles = cdiv(d.K, BLK / 64);
      } else
      if (c->kernel_set == 0) {
        GemmCfg g, gp;
        memset(&gp, 0, sizeof gp);
        const bool plain_src = !(d.flags & (F_PRE_AFFINE | F_PRE_RELU));
        // a 1x1 layer of stride 1 is a plain matrix product over the pixels: seen as a map of one row,
        // a column tile needs its own columns only, not whole rows of the map
        const bool flat = g_tile_budget_us > 0 && plain_src && !(d.flags & F_PROJ) && d.k == 1 && d.stride == 1 && d.pad == 0 &&
                          (d.H * d.W) % 4 == 0 && d.H > 1;
        if (flat) { d.W *= d.H; d.H = 1; d.OW *= d.OH; d.OH = 1; }
        const bool zsplit = a.post_gn && b.zparts >= 0 && !c->bf16 && g_tile_budget_us > 0 && !(d.flags & (F_SKIP | F_PROJ)) &&
                            (a.K / a.G) * a.OH * a.OW % 4 == 0 && (int64_t)(a.K / a.G) * a.OH * a.OW <= 32768 && a.K / a.G <= BLK;
        bool ok = make_gemm(1, d.C, d.H, d.W, d.K, d.OH, d.OW, d.k, d.stride, d.pad, nullptr, &g, plain_src, (d.flags & F_PROJ) ? 1 : 16, flat,
                            zsplit ? FWD_PARTS : 1);
        if (ok && (d.flags & F_PROJ)) ok = make_gemm(1, d.sC, d.sH, d.sW, d.K, d.OH, d.OW, 1, d.sstride, 0, &g, &gp, true);
        GemmCfg gd;
        if (ok && plain_src && !(d.flags & F_PROJ) && arena_aligned16(c, d.w) &&
            ref_vec4(c, d.x) && make_mm(c, 1, a.C, a.H, a.W, a.K, a.OH, a.OW, a.k, a.stride, a.pad, 1, &gd)) {
          d.kind = K_GEMM; d.g = gd; d.gp = gp; d.ntiles = gd.tiles;
        } else
        if (ok) {
          d.kind = K_GEMM; d.g = g; d.gp = gp; d.ntiles = g.tiles;
          if (g.parts > 1) { d.gw = c->f(b.zparts); d.gparts = g.parts; d.gpstride = (int)a.z_elems(); fwd_parts = g.parts; }
          gemm_tables(c, g, d.C, d.H, d.W, d.K, d.OH, d.OW, d.k, d.stride, &d.tq, &d.tn);
          if (d.flags & F_PROJ) gemm_tables(c, gp, d.sC, d.sH, d.sW, d.K, d.OH, d.OW, 1, d.sstride, &d.tq2, &d.tn2);
        }
      }
      out.push_back({ph++, d});
    }
    if (a.post_gn) {
      StepDesc d = blank(K_GN_STATS, s, t_f);
      d.C = a.K; d.H = a.OH; d.W = a.OW; d.G = a.G;
      d.x = ring(c, b.zring, D + 1, a.z_elems(), 0);
      d.st = ring(c, b.postst, D + 1, b.st_stride, 0);
      d.gamma = wf + a.o_gamma; d.beta = wf + a.o_beta;
      fwd_params(d, PF_GAMMA | PF_BETA);
      d.ntiles = a.G;
      if (fwd_parts > 1) { d.gw = c->f(b.zparts); d.gparts = fwd_parts; d.gpstride = (int)a.z_elems(); }
      else gn_stats_wave(d);
      out.push_back({ph++, d});
      StepDesc e = blank(K_POST_FWD, s, t_f);
      e.C = a.K; e.H = a.OH; e.W = a.OW; e.G = a.G;
      e.x = d.x; e.st = d.st; e.y = y_out;
      if (a.pool) { e.flags |= F_POOL; e.pk = a.pk; e.ps = a.ps; e.pp = a.pp; e.PH = a.PH; e.PW = a.PW; }
      e.ntiles = cdiv(a.out_elems(), BLK);
      if (c->bf16) e.flags |= F_BF16_OUT;
      out.push_back({ph++, e});
    }
    if (a.ce) {
      StepDesc d = blank(K_CE, s, t_f);
      d.n = a.K; d.n_stages = NS; d.loss_cap = c->loss_cap;
      d.x = ring(c, b.logits, 1, a.K, 0);
      d.dx = ring(c, b.dlogits, 1, a.K, 0);
      d.loss_log = c->f(L.loss);
      d.labels = c->labels_dev;
      d.ntiles = 1;
      out.push_back({ph++, d});
    }
    // ----------------------------------------------------------- backward
    int pb = (s == S - 1) ? ph : 0;
    bwd0[s] = pb;
    const TRef dy_src = (s == S - 1) ? ring(c, b.dlogits, 1, a.K, 0)
                                     : ring(c, b.gradbox, 2, a.out_elems(), 0);
    TRef dz_src = dy_src;
    if (a.post_gn) {
      StepDesc d = blank(K_GNB_REDUCE, s, t_b);
      d.C = a.K; d.H = a.OH; d.W = a.OW; d.G = a.G;
      d.flags = F_GN_RELU | (a.pool ? F_DU_POOL : F_DU_BUF);
      if (a.pool) { d.pk = a.pk; d.ps = a.ps; d.pp = a.pp; d.PH = a.PH; d.PW = a.PW; }
      d.x = ring(c, b.zring, D + 1, a.z_elems(), D);
      d.st = ring(c, b.postst, D + 1, b.st_stride, D);
      d.dy = dy_src;
      d.gamma = wbk + a.o_gamma;
      bwd_params(d, PF_GAMMA);
      d.ggamma = gr + a.o_gamma; d.gbeta = gr + a.o_beta;
      d.part = c->f(b.part);
      if (c->kernel_set == 0 && !a.pool && gn_bwd_fits(d.C, d.H * d.W, d.G)) {
        d.kind = K_GN_BWD;
        d.dx = ring(c, b.dz, 1, a.z_elems(), 0);
        d.ntiles = a.G;
        out.push_back({pb, d});
        // keep the backward GEMMs of every post-norm stage in the same phase as those of the stages
        // that need the two-step GroupNorm backward: a phase lasts as long as its longest tile, so
        // heavy steps spread over more phases cost more, not less
        pb += 2;
        dz_src = d.dx;
      } else {
        d.ntiles = a.K;
        StepDesc e = d;
        wave_reduce(d);
        out.push_back({pb++, d});
        e.kind = K_GNB_APPLY;
        e.dx = ring(c, b.dz, 1, a.z_elems(), 0);
        e.ntiles = cdiv(a.z_elems(), BLK);
        stream_apply(c, e);
        out.push_back({pb++, e});
        dz_src = e.dx;
      }
    }
    {   // weight gradient of the main layer
      StepDesc d = blank(K_CONV_BWD_W, s, t_b);
      d.C = a.C; d.H = a.H; d.W = a.W; d.K = a.K; d.OH = a.OH; d.OW = a.OW;
      d.k = a.k; d.stride = a.stride; d.pad = a.pad; d.G = a.G;
      if (a.gap) {
        d.x = ring(c, b.pooled, D + 1, a.C, D);
      } else {
        d.x = x_b;
        if (b.aring >= 0) {
          d.x = ring(c, b.aring, D + 1, a.in_elems(), D);
        } else {
          if (a.pre_gn) { d.flags |= F_PRE_AFFINE; d.st = ring(c, b.prest, D + 1, b.st_stride, D); }
          if (a.pre_relu) d.flags |= F_PRE_RELU;
        }
      }
      d.dy = dz_src;
      d.gw = gr + a.o_w;
      if (a.has_bias) { d.flags |= F_BIAS; d.gb = gr + a.o_b; }
      d.ntiles = bwd_w_tiles(a.K, a.C, a.k, a.OH * a.OW, a.has_bias);
      GemmCfg g;
      // A 3x3 layer on a 2x2 or 4x4 map (the 512-channel layers of VGG-11): its weight gradient is an outer
      // product of two tiny maps per weight; the update step computes it while it streams the parameters.
      const bool fuse_w = c->kernel_set == 0 && g_tile_budget_us > 0 && c->N == 1 && fusew_shape(a) &&
                          !(d.flags & (F_PRE_AFFINE | F_PRE_RELU)) && b.gparts < 0 && ref_vec4(c, d.x) && ref_vec4(c, d.dy);
      const bool fc_w = fc_layer(c, d, d.gw) && !(d.flags & (F_PRE_AFFINE | F_PRE_RELU)) && ref_vec4(c, d.x);
      if (fuse_w) {
        fusedw[s].phase = pb; fusedw[s].x = d.x; fusedw[s].dy = d.dy; fusedw[s].pp = pp_stride > 0 ? pp_stride : 0;
      } else if (fc_w) {
        if (a.has_bias) {
          StepDesc e = blank(K_BIAS_GRAD, s, t_b);
          e.K = a.K; e.OH = a.OH; e.OW = a.OW; e.dy = dz_src; e.gb = gr + a.o_b;
          e.ntiles = cdiv(a.K, BLK / 64);
          out.push_back({pb, e});
        }
        d.kind = K_FC_BWD_W; d.flags &= ~F_BIAS;
        d.ntiles = cdiv((int64_t)d.K * d.C, 4096);
      } else
      if (c->kernel_set == 0 && make_gemm(3, d.C, d.H, d.W, d.K, d.OH, d.OW, d.k, d.stride, d.pad, nullptr, &g,
                                          !(d.flags & (F_PRE_AFFINE | F_PRE_RELU)), 16, false, b.gparts >= 0 ? GRAD_PARTS : 1)) {
        if (a.has_bias) {
          StepDesc e = blank(K_BIAS_GRAD, s, t_b);
          e.K = a.K; e.OH = a.OH; e.OW = a.OW; e.dy = dz_src; e.gb = gr + a.o_b;
          e.ntiles = cdiv(a.K, BLK / 64);
          out.push_back({pb, e});
        }
        GemmCfg gd;
        const bool dense = !(d.flags & (F_PRE_AFFINE | F_PRE_RELU)) && ref_vec4(c, d.x) && ref_vec4(c, d.dy) &&
                           make_mm(c, 3, a.C, a.H, a.W, a.K, a.OH, a.OW, a.k, a.stride, a.pad, b.gparts >= 0 ? GRAD_PARTS : 1, &gd);
        if (dense) g = gd;
        d.kind = K_GEMM; d.g = g; d.ntiles = g.tiles; d.flags &= ~F_BIAS;
        d.gparts = g.parts; d.gpstride = (int)a.padded;
        if (!dense) gemm_tables(c, g, d.C, d.H, d.W, d.K, d.OH, d.OW, d.k, d.stride, &d.tq, &d.tn);
      }
      if (!fuse_w) out.push_back({pb, d});
    }
    if (s > 0) {   // data gradient of the main layer
      StepDesc d = blank(K_CONV_BWD_X, s, t_b);
      d.C = a.C; d.H = a.H; d.W = a.W; d.K = a.K; d.OH = a.OH; d.OW = a.OW;
      d.k = a.k; d.stride = a.stride; d.pad = a.pad;
      d.dy = dz_src;
      d.w = wbk + a.o_w;
      bwd_params(d, PF_W);
      if (a.pre_gn) {
        d.dx = ring(c, b.da, 1, a.gap ? a.C : a.in_elems(), 0);
      } else {
        d.dx = ring(c, L.sb[s - 1].gradbox, 2, a.in_elems(), ML);
        if (a.pre_relu) { d.flags |= F_MASK_X; d.x = x_b; }
        if (a.tap_dist) { d.flags |= F_ADD_SKG; d.skg = ring(c, b.skg, a.tap_dist + 1, a.in_elems(), TL(a.tap_dist)); }
        if (c->bf16) d.flags |= F_BF16_OUT;          // this gradient leaves the stage
      }
      d.ntiles = cdiv((int64_t)a.C * a.H * a.W, BLK);
      GemmCfg g;
      const bool flat = c->kernel_set == 0 && g_tile_budget_us > 0 && d.k == 1 && d.stride == 1 && d.pad == 0 &&
                        (d.H * d.W) % 4 == 0 && d.H > 1;
      if (flat) { d.W *= d.H; d.H = 1; d.OW *= d.OH; d.OH = 1; }
      const bool dxsplit = !a.pre_gn && s > 0 && L.sb[s - 1].dxparts >= 0 && !c->bf16 && g_tile_budget_us > 0 &&
                           !(d.flags & (F_MASK_X | F_ADD_SKG | F_BF16_OUT)) && !flat;
      const bool dot_bwd = c->kernel_set == 0 && g_tile_budget_us > 0 && !c->bf16 && dot_layer(a) && !(d.flags & (F_MASK_X | F_ADD_SKG | F_BF16_OUT)) &&
                           ref_vec4(c, d.dy) && ref_vec4(c, d.dx);
      if (fc_layer(c, d, d.w) && !(d.flags & (F_MASK_X | F_ADD_SKG)) && ref_vec4(c, d.dx)) {
        d.kind = K_FC_BWD_X;
        d.ntiles = cdiv(d.C, 64);
      } else
      if (dot_bwd) {
        // 64 input channels per workgroup; the output channels in as many parts as the gradient's consumer can
        // add up, so that the layer's weights are spread over C/64 x parts workgroups
        d.kind = K_DOT_BWD_X;
        const int parts = dxsplit ? FWD_PARTS : 1;
        d.n = cdiv(a.K, parts);
        d.ntiles = (a.C / 64) * parts;
        if (parts > 1) { d.gw = c->f(L.sb[s - 1].dxparts); d.gparts = parts; d.gpstride = (int)a.in_elems(); }
      } else
      if (c->kernel_set == 0 && make_gemm(2, d.C, d.H, d.W, d.K, d.OH, d.OW, d.k, d.stride, d.pad, nullptr, &g, true, 16, flat,
                                          dxsplit ? FWD_PARTS : 1)) {
        GemmCfg gd;
        const bool dense = arena_aligned16(c, d.w) && ref_vec4(c, d.dy) &&
                           make_mm(c, 2, a.C, a.H, a.W, a.K, a.OH, a.OW, a.k, a.stride, a.pad, 1, &gd);
        if (dense) g = gd;
        d.kind = K_GEMM; d.g = g; d.ntiles = g.tiles;
        if (g.parts > 1) { d.gw = c->f(L.sb[s - 1].dxparts); d.gparts = g.parts; d.gpstride = (int)a.in_elems(); }
        if (!dense) gemm_tables(c, g, d.C, d.H, d.W, d.K, d.OH, d.OW, d.k, d.stride, &d.tq, &d.tn);
      }
      out.push_back({pb, d});
    }
    if (a.add) {   // skip path: projection weight gradient and the gradient sent to the tap stage
      const int A = a.skip_from;
      const Stage& ta = c->st[A];
      const TRef skg_w = ring(c, L.sb[A].skg, ta.tap_dist + 1, ta.in_elems(), 0);
      if (a.proj) {
        StepDesc d = blank(K_CONV_BWD_W, s, t_b);
        d.C = a.sC; d.H = a.sH; d.W = a.sW; d.K = a.K; d.OH = a.OH; d.OW = a.OW;
        d.k = 1; d.stride = a.sstride; d.pad = 0;
        d.x = ring(c, L.sb[A].xring, ta.D + 2, ta.in_elems(), D + SL(A));
        d.dy = dy_src;
        d.gw = gr + a.o_wp;
        d.ntiles = bwd_w_tiles(a.K, a.sC, 1, a.OH * a.OW, false);
        GemmCfg g;
        if (c->kernel_set == 0 && make_gemm(3, d.C, d.H, d.W, d.K, d.OH, d.OW, 1, d.stride, 0, nullptr, &g, true, 16, false,
                                            b.gparts >= 0 ? GRAD_PARTS : 1)) {
          GemmCfg gd;
          const bool dense = ref_vec4(c, d.x) && ref_vec4(c, d.dy) &&
                             make_mm(c, 3, d.C, d.H, d.W, d.K, d.OH, d.OW, 1, d.stride, 0, b.gparts >= 0 ? GRAD_PARTS : 1, &gd);
          if (dense) g = gd;
          d.kind = K_GEMM; d.g = g; d.ntiles = g.tiles;
          d.gparts = g.parts; d.gpstride = (int)a.padded;
          if (!dense) gemm_tables(c, g, d.C, d.H, d.W, d.K, d.OH, d.OW, 1, d.stride, &d.tq, &d.tn);
        }
        out.push_back({pb, d});
        StepDesc e = blank(K_CONV_BWD_X, s, t_b);
        e.C = a.sC; e.H = a.sH; e.W = a.sW; e.K = a.K; e.OH = a.OH; e.OW = a.OW;
        e.k = 1; e.stride = a.sstride; e.pad = 0;
        e.dy = dy_src;
        e.w = wbk + a.o_wp;
        bwd_params(e, PF_W);
        e.dx = skg_w;
        if (c->bf16) e.flags |= F_BF16_OUT;
        e.ntiles = cdiv(ta.in_elems(), BLK);
        GemmCfg g2;
        if (c->kernel_set == 0 && make_gemm(2, e.C, e.H, e.W, e.K, e.OH, e.OW, 1, e.stride, 0, nullptr, &g2, true)) {
          GemmCfg gd;
          const bool dense = arena_aligned16(c, e.w) && ref_vec4(c, e.dy) && ref_vec4(c, e.dx) && ta.in_elems() % 2 == 0 &&
                             make_mm(c, 2, e.C, e.H, e.W, e.K, e.OH, e.OW, 1, e.stride, 0, 1, &gd);
          if (dense) g2 = gd;
          e.kind = K_GEMM; e.g = g2; e.ntiles = g2.tiles;
          if (!dense) gemm_tables(c, g2, e.C, e.H, e.W, e.K, e.OH, e.OW, 1, e.stride, &e.tq, &e.tn);
        }
        out.push_back({pb, e});
      } else {
        StepDesc d = blank(K_COPY, s, t_b);
        d.n = ta.in_elems();
        d.dy = dy_src; d.dx = skg_w;
        d.ntiles = cdiv(d.n, BLK);
        if (d.n % 4 == 0 && ref_vec4(c, d.dy) && ref_vec4(c, d.dx)) {
          d.grain = g_tile_budget_us > 0 ? STREAM_GRAIN : 2 * STREAM_GRAIN;   // fewer workgroups for a network tiled for latency
          d.ntiles = cdiv(d.n, d.grain);
        }
        out.push_back({pb, d});
      }
    }
    ++pb;
    if (a.pre_gn) {
      StepDesc d = blank(K_GNB_REDUCE, s, t_b);
      d.C = a.Cin; d.H = a.Hin; d.W = a.Win; d.G = a.G;
      d.flags = (a.pre_relu ? F_GN_RELU : 0) | (a.gap ? F_DU_GAP : F_DU_BUF);
      d.x = x_b;
      d.st = ring(c, b.prest, D + 1, b.st_stride, D);
      d.dy = ring(c, b.da, 1, a.gap ? a.C : a.in_elems(), 0);
      d.gamma = wbk + a.o_gamma;
      bwd_params(d, PF_GAMMA);
      d.ggamma = gr + a.o_gamma; d.gbeta = gr + a.o_beta;
      d.part = c->f(b.part);
      if (c->kernel_set == 0 && gn_bwd_fits(d.C, d.H * d.W, d.G)) {
        d.kind = K_GN_BWD;
        if (c->bf16) d.flags |= F_BF16_OUT;
        if (s > 0) {
          d.dx = ring(c, L.sb[s - 1].gradbox, 2, a.in_elems(), ML);
          if (a.tap_dist) { d.flags |= F_ADD_SKG; d.skg = ring(c, b.skg, a.tap_dist + 1, a.in_elems(), TL(a.tap_dist)); }
        }
        // this step ends the stage's backward chain and is the only producer of the scale / shift
        // gradients: it updates those two tensors itself, so that the rest of the stage can be
        // updated one phase earlier and no phase is left that holds nothing but updates
        // (not with weight stashing: the step would need two slots of the ring, the stashed scale it
        // reads and the new version it writes)
        // (nor with an update size above one: the gradients are then added up across ticks by the update step)
        if (!c->stash && c->N == 1) {
          d.flags |= F_UPD_GN | F_ALWAYS;
          set_update_coeffs(c, a, &d);
          d.v = c->f(L.v + a.off + a.o_gamma);
          d.w = wb + a.o_gamma;                       // master scale and shift, updated in place
          d.b = d.v;
          d.what = c->f(L.what[s] + a.o_gamma);
          writes_what(d);
        }
        d.ntiles = a.G;
        out.push_back({pb++, d});
      } else {
        d.ntiles = a.Cin;
        const StepDesc d_plain = d;
        wave_reduce(d);
        out.push_back({pb++, d});
        if (s > 0) {
          StepDesc e = d_plain;
          e.kind = K_GNB_APPLY;
          if (c->bf16) e.flags |= F_BF16_OUT;
          e.dx = ring(c, L.sb[s - 1].gradbox, 2, a.in_elems(), ML);
          if (a.tap_dist) { e.flags |= F_ADD_SKG; e.skg = ring(c, b.skg, a.tap_dist + 1, a.in_elems(), TL(a.tap_dist)); }
          e.ntiles = cdiv(a.in_elems(), BLK);
          stream_apply(c, e);
          out.push_back({pb++, e});
        }
      }
    }
  }
  // Sample-indexed form: the chains run one after the other -- forward of stage 0, 1, ..., then backward
  // of the last stage down to stage 0 -- instead of side by side.
  if (c->sequential) {
    auto is_bwd = [](const StepDesc& d) {
      return d.kind == K_GNB_REDUCE || d.kind == K_GNB_APPLY || d.kind == K_GN_BWD || d.kind == K_CONV_BWD_X ||
             d.kind == K_CONV_BWD_W || d.kind == K_BIAS_GRAD || d.kind == K_COPY || d.kind == K_DOT_BWD_X || d.kind == K_FC_BWD_X || d.kind == K_FC_BWD_W || (d.kind == K_GEMM && d.g.gm != 1);
    };
    std::vector<int> lenF(S, 0), lenB(S, 0), baseF(S, 0), baseB(S, 0);
    for (auto& pr : out) {
      const int st_ = pr.second.stage;
      if (is_bwd(pr.second)) lenB[st_] = std::max(lenB[st_], pr.first - bwd0[st_] + 1);
      else lenF[st_] = std::max(lenF[st_], pr.first + 1);
    }
    for (int s = 1; s < S; ++s) baseF[s] = baseF[s - 1] + lenF[s - 1];
    baseB[S - 1] = baseF[S - 1] + lenF[S - 1];
    for (int s = S - 2; s >= 0; --s) baseB[s] = baseB[s + 1] + lenB[s + 1];
    for (auto& pr : out) {
      const int st_ = pr.second.stage;
      pr.first = is_bwd(pr.second) ? baseB[st_] + (pr.first - bwd0[st_]) : baseF[st_] + pr.first;
    }
  }
  // 16-byte loads of the A operand need a 16-byte aligned operand (the arena is)
  for (auto& pr : out) {
    StepDesc& d = pr.second;
    if (d.kind != K_GEMM) continue;
    if (d.g.avec && !a_aligned(c, d, false)) { d.g.avec = 0; d.g.a_req *= 4; }
    if (d.gp.gm && d.gp.avec && !a_aligned(c, d, true)) { d.gp.avec = 0; d.gp.a_req *= 4; }
  }
  // ---- a backward-data GEMM that leaves partial gradients: its consumer, the channel sums of the
  // previous stage's GroupNorm (same gradient buffer), adds them up
  for (auto& pr : out) {
    const StepDesc& p = pr.second;
    const bool split_gemm = p.kind == K_GEMM && p.g.gm == 2 && p.g.parts > 1, split_dot = p.kind == K_DOT_BWD_X && p.gparts > 1;
    if (!split_gemm && !split_dot) continue;
    for (auto& qr : out) {
      StepDesc& q = qr.second;
      if ((q.kind == K_GNB_REDUCE || q.kind == K_GN_BWD) && q.stage == p.stage - 1 && q.dy.base == p.dx.base) {
        q.gw = p.gw; q.gparts = p.gparts; q.gpstride = p.gpstride;
      }
    }
  }
  // ---- fused update: one step per stage, in the phase after the last one that writes a gradient
  // of the stage (its readers use the other copy of the parameters, so they need not be waited for).
  // It runs from the first tick on: before the stage's first backward pass its gradient and
  // velocity are zero and the update only carries the parameters over to the other copy.
  for (int s = 0; s < S; ++s) {
    const Stage& a = c->st[s];
    int last_grad_phase = 0;
    bool gn_fused = false;
    int gparts = 1;   // partial weight gradients the stage's backward-weights steps leave
    for (auto& pr : out) {
      const StepDesc& e = pr.second;
      if (e.stage != s) continue;
      if (e.kind == K_GN_BWD && (e.flags & F_UPD_GN)) { gn_fused = true; continue; }
      const bool writes_grad = (e.kind == K_GEMM && e.g.gm == 3) || e.kind == K_CONV_BWD_W || e.kind == K_BIAS_GRAD ||
                               e.kind == K_GNB_REDUCE || e.kind == K_GN_BWD || e.kind == K_HEAD;
      if (writes_grad) last_grad_phase = std::max(last_grad_phase, pr.first);
      if (e.kind == K_GEMM && e.g.gm == 3) gparts = std::max(gparts, e.g.parts);
    }
    StepDesc d = blank(K_UPDATE, s, 0);
    if (fusedw[s].phase >= 0) {
      // (its operands are complete at the start of that phase; the stage's backward-data step, which reads the
      // weights, runs in it: the update follows a phase later unless it writes the other copy of the parameters)
      last_grad_phase = std::max(last_grad_phase, fusedw[s].pp > 0 ? fusedw[s].phase - 1 : fusedw[s].phase);
      d.ppstride = (int)fusedw[s].pp;
      d.flags |= F_WGRAD;
      d.x = fusedw[s].x; d.dy = fusedw[s].dy;
      d.C = a.C; d.H = a.H; d.W = a.W; d.K = a.K; d.OH = a.OH; d.OW = a.OW; d.k = 3; d.stride = 1; d.pad = 1;
    }
    set_update_coeffs(c, a, &d);
    d.w = c->f(L.w + a.off); d.v = c->f(L.v + a.off);
    d.gw = c->f(L.sb[s].gparts >= 0 ? L.sb[s].gparts : L.g + a.off);
    d.gparts = gparts; d.gpstride = (int)a.padded;
    d.wp = d.w; d.b = d.v;                             // master weights and velocity in place
    d.what = c->f(L.what[s]);
    d.pmask = PF_WHAT; d.pdepth = what_depth(a, c->stash); d.plag = -1; d.pstride = (int)a.padded;
    if (c->N > 1) {
      d.upd_n = c->N;
      d.upd_t0 = c->sequential ? 0 : 2 * (S - 1) - s;
      d.gacc = c->f(L.gacc + a.off);
      d.what0 = c->f(L.what[s]);
    }
    d.n = (int)(gn_fused ? a.o_gamma : a.padded);      // o_gamma is a multiple of 4
    d.ntiles = (int)cdiv(d.n, UPD_TILE);
    if (d.n > 0) out.push_back({last_grad_phase + 1, d});
    c->pp_active[s] = d.ppstride > 0;
  }
  // Networks tiled for latency run the kernel instantiation whose bulk outputs leave the L2
  // while the phase still runs instead of at its end (see PB_ST).  The update joins in only
  // where it retires long before its phase does, i.e. beside GEMM steps with a long
  // reduction; as the last thing a phase waits for it is quicker with plain stores (the
  // 4-stage MLP).
  c->nt_stores = g_tile_budget_us <= 0 && c->kernel_set == 0;
  if (c->tune.nt_stores) c->nt_stores = c->tune.nt_stores > 0;   // (tests: both instantiations, same arithmetic)
  // (forward and backward-data GEMMs split over their reduction, several column tiles per workgroup and
  // flattened 1x1 layers exist only in the other instantiation)
  for (auto& pr : out)
    if (pr.second.kind == K_GEMM && ((pr.second.g.gm != 3 && pr.second.g.parts > 1) || pr.second.g.nsub > 1 || pr.second.g.win > 0 || pr.second.g.mm ||
                                    pr.second.gp.nsub > 1 || pr.second.gp.win > 0)) c->nt_stores = false;
  for (auto& pr : out)
    if ((pr.second.kind == K_UPDATE && (pr.second.flags & F_WGRAD)) || pr.second.kind == K_DOT_FWD || pr.second.kind == K_DOT_BWD_X ||
        pr.second.kind == K_FC_FWD || pr.second.kind == K_FC_BWD_X || pr.second.kind == K_FC_BWD_W)
      c->nt_stores = false;
  if (c->nt_stores) {
    std::vector<char> long_gemm;
    for (auto& pr : out) {
      if ((int)long_gemm.size() <= pr.first) long_gemm.resize(pr.first + 1, 0);
      if (pr.second.kind == K_GEMM && pr.second.g.Q >= 256) long_gemm[pr.first] = 1;
    }
    for (auto& pr : out)
      if (pr.second.kind == K_UPDATE && long_gemm[pr.first]) pr.second.flags |= F_NT;
  }
}

// Launch order: by phase; inside a phase the steps are independent of each
// other, and as its longest workgroups bound the phase they go first in the grid.
void order_steps(std::vector<std::pair<int, StepDesc>>& tagged, bool one_launch = false) {   // one_launch: every phase in one launch
  auto step_cost = [](const StepDesc& d) -> int64_t {
    if (d.kind == K_HEAD) return (int64_t)1 << 40;
    if (g_tile_budget_us > 0) {
      // networks tiled for throughput: estimated duration of one workgroup, nanoseconds
      double us = 3.0;
      if (d.kind == K_GEMM) {
        GemmCfg one = d.g;
        one.n_chunks = d.g.cpp;   // what one workgroup contracts (a split reduction: its share of the chunks)
        us = est_tile_us(one, d.k);
        if (d.gp.gm) us += est_tile_us(d.gp, 1);
      } else if (d.kind == K_GN_STATS || d.kind == K_GN_BWD) {
        // (a group beyond the registers of a workgroup, 32768 elements, takes three passes over memory)
        const double n = (double)d.C / std::max(1, d.G) * d.H * d.W;
        us = 4.0 + n / BLK * (d.kind == K_GN_STATS && n > 32768 ? 1.0 : 0.05);
      } else if (d.kind == K_GNB_REDUCE) {
        // (routing the gradient back through a max-pool costs a window search per element: about 2 us per
        // 256 of them when the channel fits LDS, 7 us from global memory)
        const bool in_lds = (int64_t)d.H * d.W + (int64_t)d.PH * d.PW <= LDS_FLOATS;
        us = 4.0 + (d.grain == 1 ? 1.0 : (double)d.H * d.W / BLK * ((d.flags & F_DU_POOL) ? (in_lds ? 2.0 : 7.0) : 0.05));
      } else if (d.kind == K_DOT_FWD || d.kind == K_DOT_BWD_X) {
        us = 8.0;
      } else if (d.kind == K_UPDATE) {
        us = 15.0;
      } else if (d.kind == K_POST_FWD || d.kind == K_GNB_APPLY) {
        us = (d.flags & (F_POOL | F_DU_POOL)) ? 8.0 : 5.0;
      }
      return (int64_t)(us * 1000.0);
    }
    if (d.kind == K_GEMM) {
      const GemmCfg& g = d.g;
      return ((int64_t)1 << 20) + (int64_t)g.Q * g.ni / g.wk + ((int64_t)g.MT * g.Q + (int64_t)g.n_chunks * g.CC * g.PR * g.Wp) / 64;
    }
    if (d.kind == K_GN_STATS) return (int64_t)d.C / std::max(1, d.G) * d.H * d.W / 64 + 1000;
    if (d.kind == K_GNB_REDUCE) return (int64_t)d.H * d.W / 64 + 500;
    if (d.kind == K_GN_BWD) return (int64_t)d.C / std::max(1, d.G) * d.H * d.W / 32 + 1000;
    return 0;
  };
  // Networks tiled for latency: a phase may have somewhat more workgroups than the chip
  // holds at once (512: two per compute unit).  Workgroups are handed to the 32 shader
  // engines round robin and in order, so workgroup 512 + j waits for a slot in the engine
  // that took workgroups j, j + 32, ... (seen in per-workgroup start and end times).  The
  // shortest steps (copies, the sample, statistics) therefore go to the front, shortest
  // first, where they free a slot early in the engines the surplus workgroups will be
  // sent to; the surplus itself is the cheapest GEMM tiles, the longer of them first.
  auto rank = [](const StepDesc& d) {
    if (g_tile_budget_us > 0) return d.kind == K_HEAD ? 0 : 1;
    if (d.kind == K_HEAD) return 1;
    return (d.kind == K_GEMM || d.kind == K_GN_BWD) ? 2 : 0;
  };
  // One launch per tick: the workgroups of a later phase take their places while the first phase still runs
  // and wait there for their stage's earlier steps.  Those whose wait ends first go first: forward GEMMs (they
  // wait for a statistics step), then the GroupNorm backward (a backward-data GEMM), then updates and the rest.
  auto late_rank = [](const StepDesc& d) { return d.kind == K_GEMM ? 0 : d.kind == K_GN_BWD ? 1 : 2; };
  // Networks tiled for throughput, a phase whose GEMM tiles would keep the chip's 512 slots busy for less than
  // 100 us: the update steps go last.  Beside the tiles they stream parameters at a fraction of the bandwidth and
  // lengthen every tile's memory round trips; after them they have the chip to themselves (measured: wide 178 ->
  // 170 us per tick, VGG-11 96 -> 93).  In a long phase (ResNet-50's GEMM launches) they stay in the order of
  // cost, where they fill slots that would otherwise wait for bandwidth nobody uses (1 094 us against 1 112).
  std::vector<char> upd_last;
  if (g_tile_budget_us > 0) {
    std::vector<double> gemm_us;
    for (auto& p : tagged) {
      if ((int)gemm_us.size() <= p.first) gemm_us.resize(p.first + 1, 0.0);
      const int k = p.second.kind;
      if (k == K_GEMM || k == K_DOT_FWD || k == K_DOT_BWD_X) gemm_us[p.first] += step_cost(p.second) * 1e-3 * p.second.ntiles / 512.0;
    }
    for (double u : gemm_us) upd_last.push_back(u > 0.0 && u < 100.0);   // (a phase without tiles: in the order of cost)
  }
  std::stable_sort(tagged.begin(), tagged.end(),
                   [&](const std::pair<int, StepDesc>& x, const std::pair<int, StepDesc>& y) {
                     if (x.first != y.first) return x.first < y.first;
                     if (!one_launch && !upd_last.empty() && upd_last[x.first]) {
                       const bool ux = x.second.kind == K_UPDATE, uy = y.second.kind == K_UPDATE;
                       if (ux != uy) return uy;
                     }
                     if (one_launch && x.first > 0) {
                       const int lx = late_rank(x.second), ly = late_rank(y.second);
                       if (lx != ly) return lx < ly;
                       return step_cost(x.second) > step_cost(y.second);
                     }
                     const int rx = rank(x.second), ry = rank(y.second);
                     if (rx != ry) return rx < ry;
                     if (rx == 0 && g_tile_budget_us <= 0) return step_cost(x.second) < step_cost(y.second);
                     return step_cost(x.second) > step_cost(y.second);
                   });
}

// Host-side audit of the step table: every tensor reference a kernel will
// dereference must hold at least the elements that kernel's indexing reaches
// and must lie inside the arena.  Runs at pb_init and pb_arena_bytes, i.e.
// before anything is launched.
int validate_steps(const pb_ctx* c, const std::vector<std::pair<int, StepDesc>>& steps, int64_t arena_floats) {
  const float* lo = c->f(0);
  const float* hi = c->f(arena_floats);
  auto ref_ok = [&](const TRef& r, int64_t need) {
    if (r.depth < 1 || r.stride < need) return false;
    return r.base >= lo && r.base + (int64_t)r.depth * r.stride <= hi;
  };
  auto ptr_ok = [&](const float* p, int64_t need) { return p >= lo && p + need <= hi; };
  int idx = 0;
  for (const auto& pr : steps) {
    const StepDesc& d = pr.second;
    if (d.pmask) {
      // the ring of predicted-weight versions: every slot of every masked pointer inside the arena
      const float* ps[7] = {d.w, d.b, d.wp, d.gamma, d.beta, d.what, d.skip.base};
      bool pok = d.pdepth >= 2 && d.pstride > 0 && d.plag >= -1 && d.plag <= d.pdepth - 2 && (d.pmask & ~127) == 0;
      for (int f = 0; f < 7; ++f)
        if ((d.pmask >> f) & 1) pok = pok && ps[f] && ptr_ok(ps[f] + (int64_t)(d.pdepth - 1) * d.pstride, 1);
      if (!pok) return fail(PB_E_INVALID, "internal: step %d (kind %d, stage %d) has a bad weight-version ring", idx, d.kind, d.stage);
    }
    if (c->bf16 && (d.kind == K_CONV_FWD || d.kind == K_CONV_BWD_X))
      return fail(PB_E_UNSUPPORTED, "bf16 activations: stage %d has a layer the GEMM tiling cannot place", d.stage);
    const int64_t in = (int64_t)d.C * d.H * d.W, outn = (int64_t)d.K * d.OH * d.OW;
    const int64_t stn = 2 * d.G + 2 * d.C;
    bool ok = d.ntiles > 0;
    switch (d.kind) {
      case K_GN_STATS:
        if (d.grain == 1)   // one wavefront per group, one workgroup
          ok = ok && d.G > 0 && d.G <= BLK / 64 && d.C % d.G == 0 && d.ntiles == 1 && d.C / d.G <= 64 && (d.H * d.W) % 4 == 0 &&
               d.C / d.G * d.H * d.W <= 4096;
        else
          ok = ok && d.ntiles == d.G;
        if (d.gparts > 1)   // sums the partial outputs of a split forward GEMM: register form only
          ok = ok && d.gparts <= FWD_PARTS && d.grain != 1 && d.G > 0 && (int64_t)(d.C / d.G) * d.H * d.W <= 32768 && ((d.C / d.G) * d.H * d.W) % 4 == 0 && d.C / d.G <= BLK &&
               d.gpstride >= in && d.gpstride % 4 == 0 && ptr_ok(d.gw, (int64_t)(d.gparts - 1) * d.gpstride + in);
        ok = ok && d.G > 0 && d.C % d.G == 0 && ref_ok(d.x, in) && ref_ok(d.st, stn) &&
             ptr_ok(d.gamma, d.C) && ptr_ok(d.beta, d.C) && (!d.y.base || ref_ok(d.y, in));
        break;
      case K_GAP_FWD:
        ok = ok && d.ntiles == d.C && ref_ok(d.x, in) && ref_ok(d.y, d.C) &&
             (!(d.flags & F_PRE_AFFINE) || ref_ok(d.st, stn));
        break;
      case K_CONV_FWD:
        ok = ok && (int64_t)d.ntiles * BLK >= outn && ref_ok(d.x, in) && ref_ok(d.y, outn) &&
             ptr_ok(d.w, outn / (d.OH * d.OW) * d.C * d.k * d.k) &&
             (!(d.flags & F_PRE_AFFINE) || ref_ok(d.st, stn)) && (!(d.flags & F_BIAS) || ptr_ok(d.b, d.K));
        if (d.flags & F_SKIP) {
          if (d.flags & F_PROJ)
            ok = ok && ref_ok(d.skip, (int64_t)d.sC * d.sH * d.sW) && ptr_ok(d.wp, (int64_t)d.K * d.sC) &&
                 (d.OH - 1) * d.sstride < d.sH && (d.OW - 1) * d.sstride < d.sW;
          else
            ok = ok && ref_ok(d.skip, outn);
        }
        break;
      case K_POST_FWD:
        ok = ok && ref_ok(d.x, in) && ref_ok(d.st, stn) &&
             ref_ok(d.y, (d.flags & F_POOL) ? (int64_t)d.C * d.PH * d.PW : in);
        break;
      case K_CE:
        ok = ok && d.n > 0 && ref_ok(d.x, d.n) && ref_ok(d.dx, d.n) && ptr_ok(d.loss_log, d.loss_cap) &&
             ptr_ok((const float*)d.labels, d.n_stages);
        break;
      case K_GNB_REDUCE:
      case K_GNB_APPLY: {
        const int64_t dyn = (d.flags & F_DU_BUF) ? in : (d.flags & F_DU_GAP) ? d.C : (int64_t)d.C * d.PH * d.PW;
        ok = ok && d.G > 0 && d.C % d.G == 0 && ref_ok(d.x, in) && ref_ok(d.st, stn) && ref_ok(d.dy, dyn) &&
             ptr_ok(d.part, 3 * d.C) && ptr_ok(d.gamma, d.C);
        if (d.kind == K_GNB_REDUCE) {
          ok = ok && ptr_ok(d.ggamma, d.C) && ptr_ok(d.gbeta, d.C);
          if (d.grain == 1) ok = ok && (d.flags & (F_DU_BUF | F_DU_POOL)) && d.ntiles == cdiv(d.C, GNB_WAVE_CH * (BLK / 64));
          else ok = ok && d.grain == 0 && d.ntiles == d.C;
          if (d.gparts > 1) {   // sums partial gradients: wave form with at most 64 values per channel, or the form that
                                // stages a channel's pooled gradient in LDS
            ok = ok && d.gparts <= FWD_PARTS && d.gpstride >= dyn && ptr_ok(d.gw, (int64_t)(d.gparts - 1) * d.gpstride + dyn);
            if (d.grain == 1) ok = ok && dyn / d.C <= 64;
            else ok = ok && (d.flags & F_DU_POOL) && (int64_t)d.H * d.W + (int64_t)d.PH * d.PW <= LDS_FLOATS;
          }
        } else {
          ok = ok && ref_ok(d.dx, in) && (!(d.flags & F_ADD_SKG) || ref_ok(d.skg, in));
          if (d.grain > 0)
            ok = ok && d.grain % (4 * BLK) == 0 && (d.flags & F_DU_BUF) && (d.H * d.W) % 4 == 0 && d.n > 0 &&
                 (int64_t)d.n * d.grain >= (int64_t)(d.C / d.G) * d.H * d.W && d.ntiles == d.G * d.n && ref_vec4(c, d.x) &&
                 ref_vec4(c, d.dy) && ref_vec4(c, d.dx) && (!(d.flags & F_ADD_SKG) || ref_vec4(c, d.skg));
          else ok = ok && (int64_t)d.ntiles * BLK >= in;
        }
        break;
      }
      case K_GN_BWD: {
        const int64_t dyn = (d.flags & F_DU_BUF) ? in : d.C;
        ok = ok && gn_bwd_fits(d.C, d.H * d.W, d.G) && d.ntiles == d.G && !(d.flags & F_DU_POOL) &&
             ((d.flags & F_DU_BUF) || (d.flags & F_DU_GAP)) && ref_ok(d.x, in) && ref_ok(d.st, stn) && ref_ok(d.dy, dyn) &&
             ptr_ok(d.gamma, d.C) && ptr_ok(d.ggamma, d.C) && ptr_ok(d.gbeta, d.C) && (!d.dx.base || ref_ok(d.dx, in)) &&
             (!(d.flags & F_ADD_SKG) || (d.dx.base && ref_ok(d.skg, in)));
        if (d.gparts > 1)   // sums partial gradients (see bwd_split_consumer)
          ok = ok && d.gparts <= FWD_PARTS && (d.flags & F_DU_BUF) && d.gpstride >= in && d.gpstride % 4 == 0 && ptr_ok(d.gw, (int64_t)(d.gparts - 1) * d.gpstride + in);
        if (d.flags & F_UPD_GN)
          ok = ok && ptr_ok(d.v, 2 * d.C) && ptr_ok(d.w, 2 * d.C) && ptr_ok(d.b, 2 * d.C) && ptr_ok(d.gamma, 2 * d.C) &&
               d.what && ptr_ok(d.what, 2 * d.C);
        break;
      }
      case K_CONV_BWD_X:
        ok = ok && (int64_t)d.ntiles * BLK >= in && ref_ok(d.dy, outn) && ref_ok(d.dx, in) &&
             ptr_ok(d.w, (int64_t)d.K * d.C * d.k * d.k) && (!(d.flags & F_MASK_X) || ref_ok(d.x, in)) &&
             (!(d.flags & F_ADD_SKG) || ref_ok(d.skg, in));
        break;
      case K_CONV_BWD_W:
        ok = ok && d.ntiles == bwd_w_tiles(d.K, d.C, d.k, d.OH * d.OW, d.flags & F_BIAS) && ref_ok(d.x, in) &&
             ref_ok(d.dy, outn) && ptr_ok(d.gw, (int64_t)d.K * d.C * d.k * d.k) &&
             (!(d.flags & F_BIAS) || ptr_ok(d.gb, d.K)) && (!(d.flags & F_PRE_AFFINE) || ref_ok(d.st, stn));
        break;
      case K_COPY:
        ok = ok && ref_ok(d.dy, d.n) && ref_ok(d.dx, d.n);
        if (d.grain > 0)
          ok = ok && d.grain % (4 * BLK) == 0 && d.n % 4 == 0 && (int64_t)d.ntiles * d.grain >= d.n && ref_vec4(c, d.dy) && ref_vec4(c, d.dx);
        else ok = ok && (int64_t)d.ntiles * BLK >= d.n;
        break;
      case K_INGEST:
        ok = ok && (int64_t)d.ntiles * 4 * BLK >= d.n && ref_ok(d.dx, d.n) && ptr_ok((const float*)d.labels, d.n_stages);
        break;
      case K_UPDATE:
        ok = ok && d.n > 0 && d.n % 4 == 0 && d.ntiles == cdiv(d.n, UPD_TILE) && ptr_ok(d.w, d.n) && ptr_ok(d.v, d.n) &&
             ptr_ok(d.gw, d.n) && ptr_ok(d.wp, d.n) && ptr_ok(d.b, d.n) && (!d.what || ptr_ok(d.what, d.n)) &&
             d.what != nullptr;
        if (d.gparts > 1)
          ok = ok && d.gpstride >= d.n && d.gpstride % 4 == 0 && ptr_ok(d.gw, (int64_t)(d.gparts - 1) * d.gpstride + d.n);
        if (d.ppstride)
          ok = ok && d.ppstride > 0 && d.ppstride % 4 == 0 && d.ppstride >= d.n && (d.flags & F_WGRAD) && d.w == d.wp &&
               ptr_ok(d.w + d.ppstride, d.n);
        if (d.flags & F_WGRAD)
          ok = ok && !c->nt_stores && d.k == 3 && d.stride == 1 && d.pad == 1 && d.H == d.W && (d.H == 2 || d.H == 4) && d.OH == d.H &&
               d.OW == d.W && d.C * 9 >= 1171 && (int64_t)d.C * d.H * d.W + 8 * 16 + UPD_TILE / 2 <= LDS_FLOATS &&
               ((int64_t)d.K * d.C * 9) % 4 == 0 && (int64_t)d.K * d.C * 9 <= d.n && d.gparts <= 1 && d.upd_n <= 1 &&
               ref_ok(d.x, (int64_t)d.C * d.H * d.W) && ref_ok(d.dy, (int64_t)d.K * d.H * d.W) && ref_vec4(c, d.x) && ref_vec4(c, d.dy);
        if (d.upd_n > 1)
          ok = ok && d.upd_t0 >= 0 && ptr_ok(d.gacc, d.n) && d.pmask == PF_WHAT && d.plag == -1 &&
               ptr_ok(d.what0 + (int64_t)(d.pdepth - 1) * d.pstride, d.n) && d.what0 == d.what;
        else
          ok = ok && d.upd_n <= 1;
        break;
      case K_HEAD: {
        const int64_t cv = (d.flags & F_DU_GAP) ? d.C : in;
        ok = ok && d.ntiles == 1 && d.K > 0 && d.G > 0 && head_fits(d.C, d.H * d.W, d.K, (d.flags & F_DU_GAP) != 0, d.G) && ref_ok(d.x, in) &&
             ptr_ok(d.w, d.K * cv) && ptr_ok(d.wp, d.K * cv) && ptr_ok(d.gw, d.K * cv) && ptr_ok(d.loss_log, d.loss_cap) &&
             ptr_ok((const float*)d.labels, d.n_stages) && (!(d.flags & F_BIAS) || (ptr_ok(d.b, d.K) && ptr_ok(d.gb, d.K))) &&
             (!d.dx.base || ref_ok(d.dx, in)) && d.G > 0 && d.C % d.G == 0;
        if (d.flags & F_PRE_AFFINE)
          ok = ok && ptr_ok(d.gamma, d.C) && ptr_ok(d.beta, d.C) && ptr_ok(d.skip.base, d.C) && ptr_ok(d.ggamma, d.C) &&
               ptr_ok(d.gbeta, d.C) && (d.flags & F_DU_GAP);
        else
          ok = ok && !(d.flags & F_DU_GAP);
        break;
      }
      case K_BIAS_GRAD:
        ok = ok && d.ntiles * (BLK / 64) >= d.K && ref_ok(d.dy, outn) && ptr_ok(d.gb, d.K);
        break;
      case K_FC_FWD:
        ok = ok && !c->nt_stores && fc_layer(c, d, d.w) && !(d.flags & ~(F_ALWAYS | F_BIAS | F_BF16_OUT)) && d.ntiles == cdiv(d.K, BLK / 64) &&
             ref_ok(d.x, d.C) && ref_vec4(c, d.x) && ref_ok(d.y, d.K) && ptr_ok(d.w, (int64_t)d.K * d.C) && (!(d.flags & F_BIAS) || ptr_ok(d.b, d.K));
        break;
      case K_FC_BWD_X:
        ok = ok && !c->nt_stores && fc_layer(c, d, d.w) && !(d.flags & ~(F_ALWAYS | F_BF16_OUT)) && d.ntiles == cdiv(d.C, 64) &&
             (d.K + 3) / 4 * 4 + 16 * 64 <= LDS_FLOATS && ref_ok(d.dy, d.K) && ref_ok(d.dx, d.C) && ptr_ok(d.w, (int64_t)d.K * d.C);
        break;
      case K_FC_BWD_W:
        ok = ok && !c->nt_stores && fc_layer(c, d, d.gw) && !(d.flags & ~F_ALWAYS) && d.ntiles == cdiv((int64_t)d.K * d.C, 4096) &&
             ref_ok(d.x, d.C) && ref_vec4(c, d.x) && ref_ok(d.dy, d.K) && ptr_ok(d.gw, (int64_t)d.K * d.C);
        break;
      case K_DOT_FWD: {
        const int R = d.H == 4 ? 4 : 8;
        ok = ok && !c->nt_stores && d.k == 3 && d.stride == 1 && d.pad == 1 && d.H == d.W && (d.H == 2 || d.H == 4) && d.OH == d.H && d.OW == d.W &&
             d.n == R && d.K % R == 0 && d.ntiles == d.K / R && !(d.flags & ~F_ALWAYS) && ref_ok(d.x, in) && ref_vec4(c, d.x) &&
             ref_ok(d.y, outn) && ptr_ok(d.w, (int64_t)d.K * d.C * 9);
        break;
      }
      case K_DOT_BWD_X: {
        const int parts = d.gparts > 1 ? d.gparts : 1;
        ok = ok && !c->nt_stores && d.k == 3 && d.stride == 1 && d.pad == 1 && d.H == d.W && (d.H == 2 || d.H == 4) && d.OH == d.H && d.OW == d.W &&
             d.C % 64 == 0 && d.n >= 1 && (int64_t)d.n * parts >= d.K && (int64_t)d.n * (parts - 1) < d.K && d.ntiles == (d.C / 64) * parts &&
             !(d.flags & ~F_ALWAYS) && (int64_t)d.n * d.H * d.W + 4 * 64 * d.H * d.W <= LDS_FLOATS && ref_ok(d.dy, outn) && ref_vec4(c, d.dy) &&
             ref_ok(d.dx, in) && ref_vec4(c, d.dx) && ptr_ok(d.w, (int64_t)d.K * d.C * 9);
        if (parts > 1) {
          ok = ok && parts <= FWD_PARTS && d.gpstride >= in && d.gpstride % 4 == 0 && ptr_ok(d.gw, (int64_t)(parts - 1) * d.gpstride + in);
          bool consumed = false;
          for (auto& qr : steps)
            consumed = consumed || (((qr.second.kind == K_GNB_REDUCE && (qr.second.grain == 1 || (qr.second.flags & F_DU_POOL))) ||
                                     (qr.second.kind == K_GN_BWD && !(qr.second.flags & F_DU_GAP))) &&
                                    qr.second.gparts == d.gparts && qr.second.gw == d.gw && qr.second.dy.base == d.dx.base);
          ok = ok && consumed;
        }
        break;
      }
      case K_GEMM: {
        auto cfg_ok = [&](const GemmCfg& g, int C, int H, int W, int k, int s, int pad) {
          const int kk = k * k;
          bool o = g.wm * g.wn * g.wk == 4 && (g.ni == 1 || g.ni == 2 || g.ni == 4) && g.MT == 16 * g.wm && g.NT == 16 * g.ni * g.wn &&
                   g.nsub >= 1 && (g.nsub == 1 || (g.wk == 1 && !(d.flags & F_PROJ && g.gm == 1))) && g.tiles_n == cdiv(cdiv(g.N, g.NT), g.nsub) &&
                   g.parts >= 1 && g.cpp >= 1 && g.tpp == cdiv(g.M, g.MT) * g.tiles_n && g.tiles == g.parts * g.tpp &&
                   (int64_t)g.parts * g.cpp >= g.n_chunks && (int64_t)(g.parts - 1) * g.cpp < g.n_chunks &&
                   (g.parts == 1 || g.nsub == 1) && g.QCpad % 16 == 0 &&
                   g.QCpad >= g.QC && g.o_offq >= 0 && g.o_A >= g.o_offq + g.QCpad && g.o_A % 4 == 0 && g.o_patch % 4 == 0 &&
                   (int64_t)g.o_patch + ((int64_t)g.CC * g.PR * g.Wp + 3) / 4 * 4 <= LDS_FLOATS && LDS_FLOATS >= 4096 &&
                   (int64_t)g.n_chunks * g.QC >= g.Q;
          // the A block: MT rows of LDA floats, or (backward data) one MT*k*k segment per channel of the
          // chunk plus the zero segments the last k-step can reach
          if (g.gm == 2)
            o = o && g.LDA == g.MT * kk && (int64_t)g.o_A + (int64_t)((g.QCpad + kk - 1) / kk + 1) * g.MT * kk <= g.o_patch &&
                (!g.avec || C % 4 == 0);
          else
            o = o && g.LDA >= g.QCpad + 4 && g.LDA % 4 == 0 && (int64_t)g.o_A + (int64_t)g.MT * g.LDA <= g.o_patch &&
                (!g.avec || (g.Q % 4 == 0 && (g.n_chunks == 1 || g.QC % 4 == 0)));
          const int hl_ = (g.gm == 2) ? k - 1 - pad : pad;
          if (g.vec == 2) {
            o = o && g.gm == 2 && s > 1 && g.xoff == 0;
          } else if (g.vec == 3) {
            o = o && g.gm == 2 && s == 2 && hl_ >= 0 && hl_ <= 1 && d.OW % 2 == 0 && g.Wp % 4 == 0 && g.xoff == 0 &&
                (g.o_patch % 4) == 0 && g.win == 0;
          } else if (g.vec) {
            const int wsrc = (g.gm == 2) ? d.OW : W;
            if (g.win) o = o && g.win == g.NT && g.Wp == g.NT + 8 && H == 1 && d.OH == 1 && k == 1 && s == 1 && pad == 0 && g.gm != 3;
            else o = o && g.Wp == wsrc + 8;
            o = o && wsrc % 4 == 0 && g.xoff == 4 - hl_ && hl_ <= 4 && (g.gm != 2 || s == 1) &&
                (g.o_patch % 4) == 0 && !(d.flags & (F_PRE_AFFINE | F_PRE_RELU) && g.gm != 2);
          } else {
            o = o && g.xoff == 0 && g.win == 0;
          }
          if (g.gm == 1) {
            const int rows_max = tile_rows(g.NT, d.OW, d.OH);
            o = o && g.M == d.K && g.N == d.OH * d.OW && g.Q == C * kk && g.QC == g.CC * kk &&
                g.PR >= (rows_max - 1) * s + k && (g.win || (g.Wp >= W + 2 * pad && g.Wp >= (d.OW - 1) * s + k + g.xoff));
          } else if (g.gm == 2) {
            const int rows_max = tile_rows(g.NT, W, H);
            o = o && g.M == C && g.N == H * W && g.Q == d.K * kk && g.QC == g.CC * kk && g.PR >= rows_max + k - 1 &&
                (g.win || g.Wp >= W + k - 1 + g.xoff) && pad <= k - 1;
          } else if (g.gm == 3) {
            o = o && g.M == d.K && g.N == C * kk && g.Q == d.OH * d.OW && g.QC == g.rows_c * d.OW &&
                g.CC >= std::min(C, (g.NT + kk - 2) / kk + 1) && g.PR >= (g.rows_c - 1) * s + k && g.Wp >= W + 2 * pad &&
                g.Wp >= (d.OW - 1) * s + k + g.xoff && (g.n_chunks == 1 || g.QC % 4 == 0);
          } else {
            o = false;
          }
          return o;
        };
        // dense matrix-product form of a 1x1 layer: tile and operand shapes the kernel assumes without checking
        auto mm_ok = [&](const GemmCfg& g) {
          // the configuration is exactly what the planner makes of the step's own geometry (make_mm holds the shape
          // rules the kernel relies on); beyond that, the operands' alignment and the flags the dense form knows
          GemmCfg want;
          if (c->nt_stores || (d.flags & (F_PROJ | F_PRE_AFFINE | F_PRE_RELU)) || g.gm < 1 || g.gm > 3 ||
              !make_mm(c, g.gm, d.C, d.H, d.W, d.K, d.OH, d.OW, d.k, d.stride, d.pad, g.parts > 1 ? GRAD_PARTS : 1, &want) ||
              memcmp(&want, &g, sizeof g) != 0)
            return false;
          bool o = g.gm == 3 || (arena_aligned16(c, d.w) && (d.pmask == 0 || d.pstride % 4 == 0));
          if (g.gm == 1) o = o && ref_vec4(c, d.x);
          else if (g.gm == 2)
            o = o && ref_vec4(c, d.dy) &&
                (g.ps == 1 || (!(d.flags & (F_MASK_X | F_ADD_SKG)) && ref_vec4(c, d.dx) && (d.H * d.W) % 2 == 0 && d.W % 2 == 0));
          else o = o && ref_vec4(c, d.x) && ref_vec4(c, d.dy);
          return o;
        };
        if (d.g.mm) {
          ok = ok && d.ntiles == d.g.tiles && mm_ok(d.g) && d.gp.gm == 0;
        } else {
        ok = ok && (!d.g.avec || a_aligned(c, d, false)) && (!(d.flags & F_PROJ) || !d.gp.avec || a_aligned(c, d, true));
        ok = ok && d.ntiles == d.g.tiles && cfg_ok(d.g, d.C, d.H, d.W, d.k, d.stride, d.pad) &&
             ptr_ok((const float*)d.tq, d.g.QCpad) && ptr_ok((const float*)d.tn, d.g.N) &&
             (!(d.flags & F_PROJ) || d.g.gm != 1 || (ptr_ok((const float*)d.tq2, d.gp.QCpad) && ptr_ok((const float*)d.tn2, d.gp.N)));
        }
        const int64_t wn_ = (int64_t)d.K * d.C * d.k * d.k;
        if (d.g.gm == 1) {
          // a forward pass split over its reduction writes partial outputs gpstride floats apart
          if (d.g.parts > 1)
            ok = ok && d.gparts == d.g.parts && d.gpstride >= outn && d.gpstride % 4 == 0 && !(d.flags & (F_SKIP | F_PROJ | F_BF16_OUT)) &&
                 ptr_ok(d.gw, (int64_t)(d.g.parts - 1) * d.gpstride + outn);
          ok = ok && ref_ok(d.x, in) && ref_ok(d.y, outn) && ptr_ok(d.w, wn_) &&
               (!(d.flags & F_PRE_AFFINE) || ref_ok(d.st, stn)) && (!(d.flags & F_BIAS) || ptr_ok(d.b, d.K));
          if (d.flags & F_SKIP) {
            if (d.flags & F_PROJ)
              ok = ok && d.gp.gm == 1 && d.gp.wm == d.g.wm && d.gp.wn == d.g.wn && d.gp.wk == d.g.wk && d.gp.ni == d.g.ni &&
                   cfg_ok(d.gp, d.sC, d.sH, d.sW, 1, d.sstride, 0) && ref_ok(d.skip, (int64_t)d.sC * d.sH * d.sW) &&
                   ptr_ok(d.wp, (int64_t)d.K * d.sC) && (d.OH - 1) * d.sstride < d.sH && (d.OW - 1) * d.sstride < d.sW;
            else
              ok = ok && ref_ok(d.skip, outn);
          }
        } else if (d.g.gm == 2) {
          if (d.g.parts > 1) {   // partial gradients, summed by the previous stage's channel sums
            ok = ok && d.gparts == d.g.parts && d.gpstride >= in && !(d.flags & (F_MASK_X | F_ADD_SKG | F_BF16_OUT)) &&
                 ptr_ok(d.gw, (int64_t)(d.g.parts - 1) * d.gpstride + in);
            bool consumed = false;
            for (auto& qr : steps)
              consumed = consumed || (((qr.second.kind == K_GNB_REDUCE && (qr.second.grain == 1 || (qr.second.flags & F_DU_POOL))) ||
                                       (qr.second.kind == K_GN_BWD && !(qr.second.flags & F_DU_GAP))) &&
                                      qr.second.gparts == d.gparts && qr.second.gw == d.gw && qr.second.dy.base == d.dx.base);
            ok = ok && consumed;
          }
          ok = ok && ref_ok(d.dy, outn) && ref_ok(d.dx, in) && ptr_ok(d.w, wn_) &&
               (!(d.flags & F_MASK_X) || ref_ok(d.x, in)) && (!(d.flags & F_ADD_SKG) || ref_ok(d.skg, in));
        } else {
          ok = ok && ref_ok(d.x, in) && ref_ok(d.dy, outn) && ptr_ok(d.gw, wn_) &&
               (!(d.flags & F_PRE_AFFINE) || ref_ok(d.st, stn)) && !(d.flags & F_BIAS);
          // a split reduction writes partial gradients gpstride floats apart
          if (d.g.parts > 1)
            ok = ok && d.gparts == d.g.parts && d.gpstride >= wn_ && d.gpstride % 4 == 0 &&
                 ptr_ok(d.gw, (int64_t)(d.g.parts - 1) * d.gpstride + wn_);
        }
        break;
      }
      default:
        ok = false;
    }
    if (!ok) return fail(PB_E_INVALID, "internal: step %d (kind %d, stage %d) fails the bounds audit", idx, d.kind, d.stage);
    ++idx;
  }
  return PB_OK;
}

// ------------------------------------------------- initial weights (host)
inline uint64_t mix64(uint64_t z) {
  z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ULL;
  z ^= z >> 27; z *= 0x94D049BB133111EBULL;
  z ^= z >> 31;
  return z;
}

// Element e of parameter tensor `tensor`: outputs 2e and 2e+1 of a splitmix64
// stream started at seed ^ (GOLD*(tensor+1)); Box-Muller (cosine branch) in
// double; scaled by std and rounded once to float.
void fill_normal(float* dst, int64_t n, uint64_t seed, int tensor, double std_) {
  const uint64_t GOLD = 0x9E3779B97F4A7C15ULL;
  const uint64_t key = seed ^ (GOLD * (uint64_t)(tensor + 1));
  const double two_pi = 6.283185307179586476925286766559;
  for (int64_t e = 0; e < n; ++e) {
    const uint64_t r1 = mix64(key + GOLD * (2 * (uint64_t)e + 1));
    const uint64_t r2 = mix64(key + GOLD * (2 * (uint64_t)e + 2));
    const double u1 = ((double)(r1 >> 11) + 1.0) * 0x1.0p-53;
    const double u2 = (double)(r2 >> 11) * 0x1.0p-53;
    dst[e] = (float)(sqrt(-2.0 * log(u1)) * cos(two_pi * u2) * std_);
  }
}

void init_weights_host(const std::vector<Stage>& st, uint64_t seed, std::vector<float>& w) {
  int tensor = 0;
  for (const Stage& a : st) {
    float* p = w.data() + a.off;
    fill_normal(p + a.o_w, a.n_w, seed, tensor++, sqrt(2.0 / a.fan_w));
    if (a.has_bias) tensor++;                       // zeros
    if (a.proj) fill_normal(p + a.o_wp, a.n_wp, seed, tensor++, sqrt(2.0 / a.fan_wp));
    if (a.n_gn) {
      for (int64_t i = 0; i < a.n_gn; ++i) p[a.o_gamma + i] = 1.0f;
      tensor += 2;
    }
  }
}

// After the stream has been synchronised: did a dependency wait of a one-launch tick expire?
int check_device_error(pb_ctx* c) {
  if (c->fuse_from < 0) return PB_OK;
  int32_t err = 0;
  if (hipMemcpy(&err, c->sync_dev + SYNC_ERR, sizeof err, hipMemcpyDeviceToHost) != hipSuccess)
    return fail(PB_E_HIP, "device to host copy failed");
  if (err) return fail(PB_E_HIP, "a workgroup's wait for the steps it depends on expired (phases sharing a launch): results are invalid");
  return PB_OK;
}

int64_t copy_params_out(pb_ctx* c, int64_t arena_off, float* dst, int64_t cap) {
  if (!dst) return c->n_params;
  if (hipStreamSynchronize(c->stream) != hipSuccess) return fail(PB_E_HIP, "stream synchronize failed");
  if (int rc = check_device_error(c)) return rc;
  std::vector<float> tmp(c->L.P);
  if (hipMemcpy(tmp.data(), c->f(arena_off), sizeof(float) * c->L.P, hipMemcpyDeviceToHost) != hipSuccess)
    return fail(PB_E_HIP, "device to host copy failed");
  // stages with two copies of their master parameters: after an odd number of ticks the current ones are the second
  if (arena_off == c->L.w && (c->ticks & 1))
    for (size_t s = 0; s < c->st.size(); ++s)
      if (c->pp_active[s] &&
          hipMemcpy(tmp.data() + c->st[s].off, c->f(c->L.sb[s].w2), sizeof(float) * c->st[s].padded, hipMemcpyDeviceToHost) != hipSuccess)
        return fail(PB_E_HIP, "device to host copy failed");
  int64_t n = 0;
  auto put = [&](const float* src, int64_t cnt) {
    const int64_t take = std::min<int64_t>(cnt, cap - n);
    if (take > 0) { memcpy(dst + n, src, sizeof(float) * take); n += take; }
  };
  for (const Stage& a : c->st) {
    put(tmp.data() + a.off, a.n_head);
    if (a.n_gn) put(tmp.data() + a.off + a.o_gamma, 2 * a.n_gn);
  }
  return n;
}

struct ScopedEv {
  pb_ctx* c; int idx = -1;
  ScopedEv(pb_ctx* c_, int cls) : c(c_) {
    if (!c->profiling || (int)c->evs.size() >= c->max_events) return;
    pb_ctx::Ev e;
    if (!c->ev_pool.empty()) { e = c->ev_pool.back(); c->ev_pool.pop_back(); }
    else { if (hipEventCreate(&e.a) != hipSuccess || hipEventCreate(&e.b) != hipSuccess) return; }
    e.cls = cls;
    (void)hipEventRecord(e.a, c->stream);
    c->evs.push_back(e);
    idx = (int)c->evs.size() - 1;
  }
  ~ScopedEv() { if (idx >= 0) (void)hipEventRecord(c->evs[idx].b, c->stream); }
};

int run_one_tick(pb_ctx* c, const float* staging, int label) {
  // the kernels index every ring with a 32-bit tick counter
  if (c->ticks >= (int64_t)0x7fffff00) return fail(PB_E_UNSUPPORTED, "tick counter exhausted (2^31 ticks): start a new context");
  const int k = (int)c->ticks;   // t_base stays 0 on this path
  if (c->launch_mode == 0) {
    bool counted = false;
    for (const Phase& p : c->phases) {
      ScopedEv ev(c, 0);
      if (p.fused && !counted) { ++c->fused_ticks; counted = true; }
      launch_phase(c->recs_dev + c->rec_first[p.first], p.tiles, c->globals_dev, k, staging, label, c->nt_stores, c->stream,
                   p.fused ? c->sync_dev : nullptr, p.fused ? c->fused_ticks : 0u);
    }
  } else {
    // one launch per step (same records, same arithmetic); event classes: 1 = update steps, 2 = ingest
    for (const Phase& p : c->phases)
      for (int i = 0; i < p.count; ++i) {
        const StepDesc& sd = c->steps[p.first + i];
        ScopedEv ev(c, sd.kind == K_INGEST ? 2 : sd.kind == K_UPDATE ? 1 : 0);
        launch_phase(c->recs_dev + c->rec_first[p.first + i], sd.ntiles, c->globals_dev, k, staging, label,
                     c->nt_stores, c->stream);
      }
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(PB_E_HIP, "kernel launch failed: %s", hipGetErrorString(e));
  c->ticks++;
  return PB_OK;
}

}  // namespace

// =============================================================== the C ABI
extern "C" {

const char* pb_last_error(void) { return g_err.c_str(); }

size_t pb_arena_bytes(const pb_net_desc* net, const int32_t* delays) {
  std::vector<Stage> st;
  bool sequential = false;
  if (parse_net(net, st) != PB_OK || check_delays(st, delays, &sequential) != PB_OK) return 0;
  pb_ctx tmp;
  tmp.st = st; tmp.S = (int)st.size();
  take_settings(&tmp, net);
  tmp.sequential = sequential;
  const int cap = net->loss_capacity > 0 ? net->loss_capacity : (1 << 20);
  Plan pl;
  Layout L;
  plan_arena(st, net->bwd_weights == 1, cap, L, pl, net->kernel_set == 0, tmp.N);
  // step table, prefix, chunk map and segment table live in the arena too
  tmp.L = L; tmp.loss_cap = cap; tmp.arena = nullptr;
  tmp.labels_dev = (int32_t*)tmp.f(L.labels);
  std::vector<std::pair<int, StepDesc>> steps;
  tmp.plan = &pl;
  compile_steps(&tmp, steps);
  if (validate_steps(&tmp, steps, pl.total) != PB_OK) return 0;
  int64_t total_tiles = 0;
  for (auto& pr : steps) total_tiles += pr.second.ntiles;
  pl.alloc(total_tiles * (int64_t)sizeof(StepDesc) / 4 + 64);
  return (size_t)pl.total * sizeof(float) + 256;
}

int64_t pb_plan_summary(const pb_net_desc* net, char* buf, int64_t cap) {
  std::vector<Stage> st;
  if (parse_net(net, st) != PB_OK) return PB_E_INVALID;
  pb_ctx tmp;
  tmp.st = st; tmp.S = (int)st.size();
  take_settings(&tmp, net);
  const int lcap = net->loss_capacity > 0 ? net->loss_capacity : (1 << 20);
  Plan pl;
  plan_arena(st, net->bwd_weights == 1, lcap, tmp.L, pl, net->kernel_set == 0, tmp.N);
  tmp.loss_cap = lcap;
  std::vector<std::pair<int, StepDesc>> steps;
  tmp.plan = &pl;
  compile_steps(&tmp, steps);
  order_steps(steps);
  static const char* names[] = {"gn_stats", "gap_fwd", "conv_fwd", "post_fwd", "ce", "gnb_reduce", "gnb_apply",
                                "conv_bwd_x", "conv_bwd_w", "copy", "gemm", "bias_grad", "ingest", "update", "head", "gn_bwd", "dot_fwd", "dot_bwd_x", "fc_fwd", "fc_bwd_x", "fc_bwd_w"};
  std::string o;
  char line[400];
  for (auto& pr : steps) {
    const StepDesc& d = pr.second;
    snprintf(line, sizeof line, "stage %2d phase %d %-10s tiles %6d first_tick %3d C%dx%dx%d K%dx%dx%d k%d s%d", d.stage,
             pr.first, names[d.kind], d.ntiles, d.first_tick, d.C, d.H, d.W, d.K, d.OH, d.OW, d.k, d.stride);
    o += line;
    if (d.kind == K_GEMM) {
      const GemmCfg& g = d.g;
      if (g.mm)
        snprintf(line, sizeof line, " | gm%d M%d N%d Q%d dense mi%d ni%d tile %dx%d chunks %d/%d QC%d lds %d", g.gm, g.M, g.N, g.Q, g.mi, g.ni,
                 g.MT, g.NT, g.n_chunks, g.parts, g.QC, 2 * mm_chunk_floats(g.gm, g.MT, g.NT));
      else
      snprintf(line, sizeof line, " | gm%d M%d N%d Q%d waves %dx%dx%d ni%d tile %dx%d x%d chunks %d/%d QC%d CC%d PR%d Wp%d lds %d",
               g.gm, g.M, g.N, g.Q, g.wm, g.wn, g.wk, g.ni, g.MT, g.NT, g.nsub, g.n_chunks, g.parts, g.QC, g.CC, g.PR, g.Wp,
               g.o_patch + g.CC * g.PR * g.Wp);
      o += line;
    }
    {
      // algorithmic bytes of the streaming steps (each operand read or written once, 4 bytes per element)
      const int64_t in = (int64_t)d.C * d.H * d.W;
      int64_t el = -1;
      if (d.kind == K_GN_STATS) el = (d.gparts > 1 ? (int64_t)d.gparts * in + in : in) + (d.y.base ? in : 0);
      else if (d.kind == K_GN_BWD) el = in + ((d.flags & F_DU_GAP) ? d.C : in) + (d.dx.base ? in : 0) + ((d.flags & F_ADD_SKG) ? in : 0);
      else if (d.kind == K_GNB_REDUCE) el = in + ((d.flags & F_DU_BUF) ? in : (d.flags & F_DU_GAP) ? d.C : (int64_t)d.C * d.PH * d.PW);
      else if (d.kind == K_GNB_APPLY) el = 3 * in + ((d.flags & F_ADD_SKG) ? in : 0);
      else if (d.kind == K_POST_FWD) el = in + ((d.flags & F_POOL) ? (int64_t)d.C * d.PH * d.PW : in);
      else if (d.kind == K_COPY) el = 2 * (int64_t)d.n;
      else if (d.kind == K_UPDATE) el = 6 * (int64_t)d.n + (int64_t)(d.gparts - 1) * d.n - ((d.flags & F_WGRAD) ? (int64_t)d.K * d.C * 9 : 0);
      if (el >= 0) {
        snprintf(line, sizeof line, " | bytes %lld", (long long)(4 * el));
        o += line;
      }
    }
    o += "\n";
  }
  if (buf && cap > 0) {
    const int64_t n = std::min<int64_t>(cap - 1, (int64_t)o.size());
    memcpy(buf, o.data(), n);
    buf[n] = 0;
  }
  return (int64_t)o.size() + 1;
}

}  // extern "C"

namespace {

// pb_init and pb_init_static.  static_arena: the context lives in the library's own
// device array (handed in as base / base_bytes) and nothing is allocated or freed on the device.
int init_common(pb_ctx** out, const pb_net_desc* net, const int32_t* delays, float lr, float momentum,
                uint64_t seed, void* base, size_t base_bytes, bool static_arena) {
  if (!out) return fail(PB_E_INVALID, "out is NULL");
  *out = nullptr;
  std::vector<Stage> st;
  int rc = parse_net(net, st);
  if (rc != PB_OK) return rc;
  bool sequential = false;
  rc = check_delays(st, delays, &sequential);
  if (rc != PB_OK) return rc;
  if (!(momentum >= 0.f && momentum <= 1.f)) return fail(PB_E_INVALID, "momentum must be in [0,1]");
  if (!(lr >= 0.f)) return fail(PB_E_INVALID, "learning rate must be >= 0");
  const size_t need = pb_arena_bytes(net, delays);
  if (!need) return PB_E_INVALID;

  pb_ctx* c = new pb_ctx();
  c->st = st; c->S = (int)st.size();
  c->mitigation = net->mitigation; c->lr = lr; c->m = momentum;
  take_settings(c, net);
  c->lwp_w = net->lwp_form == 1;
  c->sequential = sequential;
  c->sc_scale = net->sc_scale > 0.f ? net->sc_scale : 1.0;
  c->lwp_scale = net->lwp_scale > 0.f ? net->lwp_scale : 1.0;
  c->loss_cap = net->loss_capacity > 0 ? net->loss_capacity : (1 << 20);
  c->stream = (hipStream_t)net->stream;
  for (const Stage& a : st) c->n_params += a.n_params;
  if (static_arena) {
    if (need > base_bytes) {
      delete c;
      return fail(PB_E_NOMEM, "this network needs %zu bytes of device memory, the library's static arena holds %zu: use pb_init",
                  need, base_bytes);
    }
    c->static_dev = g_static_dev;
  } else if (base) {
    if (base_bytes < need) { delete c; return fail(PB_E_NOMEM, "arena has %zu bytes, %zu needed", base_bytes, need); }
    if ((uintptr_t)base % 256) { delete c; return fail(PB_E_INVALID, "arena must be 256-byte aligned"); }
  } else {
    if (hipMalloc(&base, need) != hipSuccess) { delete c; return fail(PB_E_NOMEM, "hipMalloc of %zu bytes failed", need); }
    c->own_arena = true;
  }
  c->arena = (float*)base;
#define INIT_TRY(expr)                                                                  \
  do {                                                                                  \
    hipError_t e_ = (expr);                                                             \
    if (e_ != hipSuccess) {                                                             \
      fail(PB_E_HIP, "%s failed: %s", #expr, hipGetErrorString(e_));                    \
      pb_destroy(c);                                                                    \
      return PB_E_HIP;                                                                  \
    }                                                                                   \
  } while (0)
  if (static_arena) {
    // the array keeps the previous context's contents: everything must start at zero (a fill kernel,
    // so that the call stays free of runtime memory operations that may allocate)
    launch_fill_zero(base, (need + 15) / 16 * 16, c->stream);
    INIT_TRY(hipGetLastError());
  } else {
    INIT_TRY(hipMemsetAsync(base, 0, need, c->stream));
  }

  Plan pl;
  plan_arena(st, net->bwd_weights == 1, c->loss_cap, c->L, pl, net->kernel_set == 0, c->N);
  c->labels_dev = (int32_t*)c->f(c->L.labels);
  c->globals_dev = (Globals*)c->f(c->L.globals);
  c->zero_dev = (int32_t*)c->f(c->L.zero);
  c->sync_dev = (int32_t*)c->f(c->L.sync);

  std::vector<std::pair<int, StepDesc>> tagged;
  c->plan = &pl;
  compile_steps(c, tagged);
  if (validate_steps(c, tagged, pl.total) != PB_OK) { pb_destroy(c); return PB_E_INVALID; }
  int n_ph_all = 0;
  for (auto& p : tagged) n_ph_all = std::max(n_ph_all, p.first + 1);
  // Phases sharing a launch: pipelined form only (in the sample-indexed form steps of different stages depend on
  // each other inside a tick).
  //  * One launch per tick.  By policy only where the tick's workgroups number no more than the compute units:
  //    then all of them are resident at once, no waiting workgroup can hold a producer's place, and the launch
  //    boundary saved outweighs what the per-workgroup release and acquire cost (measured: a tick of 165
  //    workgroups gains 7 %, one of 944 workgroups takes twice as long).
  //  * The last phases in one launch.  A deep network's last phases hold the dependency chains of one or two
  //    stages only (the loss stage runs forward and backward in the same tick, the first stage's weight
  //    gradient is split and summed): a few hundred workgroups each, a launch each.  On request (tail_merge n)
  //    the phases from n on share a launch; only the workgroups of stages with a dependency inside it signal
  //    and wait.  Not chosen by policy: measured on the 50-stage network (phases 2-6 in one launch, about 3000
  //    of 9000 workgroups signalling or waiting) the tick takes 1215 us instead of 1125 -- a workgroup's release
  //    and acquire write back and invalidate its XCD's L2, which costs the other workgroups more than the four
  //    launch boundaries did -- and VGG-11 and the wide network lose as well (tail_merge -2 selects the
  //    candidate rule: the longest run of last phases with steps of at most two stages).
  std::vector<int64_t> wg_of(n_ph_all, 0);
  for (auto& p : tagged) wg_of[p.first] += p.second.ntiles;
  int n_cu = 0, cur_dev = 0;
  INIT_TRY(hipGetDevice(&cur_dev));
  INIT_TRY(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, cur_dev));
  const bool can_fuse = !c->sequential && n_ph_all >= 2 && n_ph_all <= MAX_SYNC_PHASES;
  if (c->tune.one_launch > 0 && !can_fuse) {
    pb_destroy(c);
    return fail(PB_E_UNSUPPORTED, "one launch per tick needs the pipelined form and 2..%d phases (this network has %d)", MAX_SYNC_PHASES, n_ph_all);
  }
  c->fuse_from = -1;
  if (c->tune.one_launch > 0) {
    c->fuse_from = 0;
  } else if (c->tune.one_launch == 0) {
    int64_t n_wg = 0;
    for (int64_t n : wg_of) n_wg += n;
    if (can_fuse && n_wg <= n_cu) c->fuse_from = 0;
  }
  if (c->fuse_from < 0 && c->tune.tail_merge > 0) {
    if (c->sequential || c->tune.tail_merge > n_ph_all - 2 || n_ph_all - c->tune.tail_merge > MAX_SYNC_PHASES) {
      pb_destroy(c);
      return fail(PB_E_UNSUPPORTED, "tail_merge %d: needs the pipelined form, at least two phases from there on and at most %d (this network has %d phases)",
                  c->tune.tail_merge, MAX_SYNC_PHASES, n_ph_all);
    }
    c->fuse_from = c->tune.tail_merge;
  } else if (c->fuse_from < 0 && c->tune.tail_merge == -2 && !c->sequential) {
    // the longest run of last phases that have at most 8 workgroups per compute unit each and, together, steps
    // of at most two stages; it joins the phase before it
    int first_light = n_ph_all;
    for (int ph = n_ph_all - 1; ph >= 2; --ph) {
      std::vector<int> stages;
      for (auto& p : tagged)
        if (p.first >= ph && std::find(stages.begin(), stages.end(), p.second.stage) == stages.end()) stages.push_back(p.second.stage);
      if (wg_of[ph] > 8 * (int64_t)n_cu || stages.size() > 2) break;
      first_light = ph;
    }
    if (first_light < n_ph_all && n_ph_all - (first_light - 1) <= MAX_SYNC_PHASES) c->fuse_from = first_light - 1;
  }
  order_steps(tagged, c->fuse_from == 0);
  for (auto& p : tagged) { p.second.sig_idx = -1; p.second.nwait = 0; }
  if (c->fuse_from >= 0) {
    // completion counter (stage, phase): workgroups of that stage in that phase.  A step waits for the nearest
    // earlier phase of the launch that holds work of its stage (whose workgroups waited for the one before in
    // their turn); a step signals if a later phase holds work of its stage.
    const int f0 = c->fuse_from, nf = n_ph_all - f0;
    std::vector<int> cnt((size_t)c->S * MAX_SYNC_PHASES, 0);
    for (auto& p : tagged)
      if (p.first >= f0) cnt[(size_t)p.second.stage * MAX_SYNC_PHASES + (p.first - f0)] += p.second.ntiles;
    for (auto& p : tagged) {
      if (p.first < f0) continue;
      StepDesc& d = p.second;
      const int me = p.first - f0;
      for (int q = me - 1; q >= 0; --q) {
        const int n = cnt[(size_t)d.stage * MAX_SYNC_PHASES + q];
        if (n > 0) { d.wait_idx[0] = d.stage * MAX_SYNC_PHASES + q; d.wait_n[0] = n; d.nwait = 1; break; }
      }
      for (int q = me + 1; q < nf; ++q)
        if (cnt[(size_t)d.stage * MAX_SYNC_PHASES + q] > 0) { d.sig_idx = d.stage * MAX_SYNC_PHASES + me; break; }
    }
  }
  const int n_steps = (int)tagged.size();
  c->steps.resize(n_steps);
  int n_ph = 0;
  for (auto& p : tagged) n_ph = std::max(n_ph, p.first + 1);
  c->phases.assign(n_ph, Phase());
  c->rec_first.assign(n_steps, 0);
  std::vector<StepDesc> recs;
  for (int i = 0, cur = -1, acc = 0; i < n_steps; ++i) {
    const int ph = tagged[i].first;
    if (ph != cur) { cur = ph; acc = 0; c->phases[ph].first = i; }
    c->steps[i] = tagged[i].second;
    c->rec_first[i] = (int64_t)recs.size();
    for (int tl = 0; tl < tagged[i].second.ntiles; ++tl) {
      recs.push_back(tagged[i].second);
      recs.back().tile = tl;
    }
    acc += tagged[i].second.ntiles;
    c->phases[ph].count++;
    c->phases[ph].tiles = acc;
  }
  if (c->fuse_from >= 0) {
    // (launch mode 1 still walks the steps one by one, in this same order: phase by phase)
    Phase& m = c->phases[c->fuse_from];
    m.fused = true;
    m.count = n_steps - m.first;
    m.tiles = (int)(recs.size() - (size_t)c->rec_first[m.first]);
    c->phases.resize(c->fuse_from + 1);
  }
  const int64_t o_recs = pl.alloc((int64_t)recs.size() * sizeof(StepDesc) / 4 + 64);
  if ((size_t)pl.total * sizeof(float) > need) { pb_destroy(c); return fail(PB_E_NOMEM, "internal: arena plan mismatch"); }
  c->recs_dev = (StepDesc*)c->f(o_recs);

  std::vector<float> w(c->L.P, 0.f);
  init_weights_host(st, seed, w);
  Globals g0;
  memset(&g0, 0, sizeof g0);
  g0.n_pool = 1;
  INIT_TRY(hipMemcpyAsync(c->f(c->L.w), w.data(), sizeof(float) * c->L.P, hipMemcpyHostToDevice, c->stream));
  for (int s = 0; s < c->S; ++s)     // slot 0 of every stage's ring of predicted weights: v = 0, so w_hat = w
    INIT_TRY(hipMemcpyAsync(c->f(c->L.what[s]), w.data() + st[s].off, sizeof(float) * st[s].padded, hipMemcpyHostToDevice, c->stream));
  INIT_TRY(hipMemcpyAsync(c->recs_dev, recs.data(), sizeof(StepDesc) * recs.size(), hipMemcpyHostToDevice, c->stream));
  INIT_TRY(hipMemcpyAsync(c->globals_dev, &g0, sizeof g0, hipMemcpyHostToDevice, c->stream));
  {
    const int32_t head[2] = {0, c->tune.spin_limit > 0 ? c->tune.spin_limit : (1 << 16)};   // error word, wait bound
    INIT_TRY(hipMemcpyAsync(c->sync_dev, head, sizeof head, hipMemcpyHostToDevice, c->stream));
  }
  for (auto& tb : c->tables)
    INIT_TRY(hipMemcpyAsync(c->f(tb.first), tb.second.data(), sizeof(int32_t) * tb.second.size(), hipMemcpyHostToDevice, c->stream));
  INIT_TRY(hipStreamSynchronize(c->stream));
  if (!static_arena) {
    const size_t bytes = sizeof(float) * st[0].in_elems();
    for (int i = 0; i < pb_ctx::N_PINNED; ++i) {
      INIT_TRY(hipHostMalloc((void**)&c->pinned[i], bytes, hipHostMallocDefault));
      INIT_TRY(hipEventCreateWithFlags(&c->pinned_done[i], hipEventDisableTiming));
    }
  }
#undef INIT_TRY
  *out = c;
  return PB_OK;
}

}  // namespace

extern "C" {

int pb_init(pb_ctx** out, const pb_net_desc* net, const int32_t* delays, float lr, float momentum,
            uint64_t seed) {
  if (!net) return fail(PB_E_INVALID, "empty network");
  return init_common(out, net, delays, lr, momentum, seed, net->device_arena, net->arena_bytes, false);
}

size_t pb_static_arena_bytes(void) { return STATIC_ARENA_BYTES; }

int pb_init_static(pb_ctx** out, const pb_net_desc* net, const int32_t* delays, float lr, float momentum,
                   uint64_t seed) {
  if (!net) return fail(PB_E_INVALID, "empty network");
  if (net->device_arena) return fail(PB_E_INVALID, "pb_init_static takes no device_arena: it uses the library's own");
  void* base = nullptr;
  int dev = -1;
  const hipError_t e = static_arena(&base, &dev);
  if (e != hipSuccess) return fail(PB_E_HIP, "static arena: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= MAX_STATIC_DEVS) return fail(PB_E_UNSUPPORTED, "device ordinal %d", dev);
  if (g_static_busy[dev])
    return fail(PB_E_UNSUPPORTED, "the static arena of device %d is held by another context: destroy it first", dev);
  g_static_dev = dev;
  const int rc = init_common(out, net, delays, lr, momentum, seed, base, STATIC_ARENA_BYTES, true);
  if (rc == PB_OK) g_static_busy[dev] = true;
  return rc;
}

int pb_tick(pb_ctx* c, const float* sample, int32_t label) {
  if (!c || !sample) return fail(PB_E_INVALID, "NULL argument");
  if (label < 0 || label >= c->st.back().K) return fail(PB_E_INVALID, "label %d out of range", label);
  float* staging = c->f(c->L.staging);
  const size_t bytes = sizeof(float) * c->st[0].in_elems();
  if (c->pinned[0]) {
    const int i = c->pinned_next;
    c->pinned_next = (i + 1) % pb_ctx::N_PINNED;
    if (c->pinned_used[i]) HIP_TRY(hipEventSynchronize(c->pinned_done[i]));   // its copy of N_PINNED ticks ago has landed
    memcpy(c->pinned[i], sample, bytes);
    HIP_TRY(hipMemcpyAsync(staging, c->pinned[i], bytes, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(hipEventRecord(c->pinned_done[i], c->stream));
    c->pinned_used[i] = true;
  } else {
    // (a context that must not allocate has no pinned buffers: the runtime stages the pageable copy itself)
    HIP_TRY(hipMemcpyAsync(staging, sample, bytes, hipMemcpyHostToDevice, c->stream));
  }
  return run_one_tick(c, staging, label);
}

int pb_run_resident(pb_ctx* c, const float* samples_dev, const int32_t* labels_dev, int32_t n_pool,
                    int64_t first_index, int64_t n_ticks) {
  if (!c || !samples_dev || !labels_dev || n_pool <= 0 || first_index < 0 || n_ticks < 0)
    return fail(PB_E_INVALID, "bad argument");
  // tick t consumes item (idx_base + t) mod n_pool
  const int64_t t0 = c->ticks;
  int64_t ib = (first_index - t0) % n_pool;
  if (ib < 0) ib += n_pool;
  if (c->pool != samples_dev || c->pool_labels != labels_dev || c->n_pool != n_pool || c->idx_base != (int)ib) {
    Globals g;
    memset(&g, 0, sizeof g);
    g.t_base = 0; g.idx_base = (int)ib; g.n_pool = n_pool; g.pool = samples_dev; g.pool_labels = labels_dev;
    launch_set_globals(c->globals_dev, g, c->stream);
    c->pool = samples_dev; c->pool_labels = labels_dev; c->n_pool = n_pool; c->idx_base = (int)ib;
  }
  for (int64_t j = 0; j < n_ticks; ++j) {
    int rc = run_one_tick(c, nullptr, 0);
    if (rc != PB_OK) return rc;
  }
  return PB_OK;
}

int64_t pb_read_weights(pb_ctx* c, float* dst, int64_t cap) {
  if (!c) return fail(PB_E_INVALID, "NULL context");
  return copy_params_out(c, c->L.w, dst, cap);
}

int64_t pb_read_velocity(pb_ctx* c, float* dst, int64_t cap) {
  if (!c) return fail(PB_E_INVALID, "NULL context");
  return copy_params_out(c, c->L.v, dst, cap);
}

int64_t pb_loss_history(pb_ctx* c, float* dst, int64_t cap) {
  if (!c) return fail(PB_E_INVALID, "NULL context");
  // pipelined: the sample fed by tick i reaches the loss at tick i + S - 1; sample-indexed form: at tick i
  const int64_t count = c->sequential ? c->ticks : std::max<int64_t>(0, c->ticks - c->S + 1);
  const int64_t avail = std::min<int64_t>(count, c->loss_cap);
  if (!dst) return avail;
  const int64_t n = std::min(avail, cap);
  if (n <= 0) return 0;
  HIP_TRY(hipStreamSynchronize(c->stream));
  if (int rc = check_device_error(c)) return rc;
  std::vector<float> ring_(c->loss_cap);
  HIP_TRY(hipMemcpy(ring_.data(), c->f(c->L.loss), sizeof(float) * c->loss_cap, hipMemcpyDeviceToHost));
  for (int64_t i = 0; i < n; ++i) dst[i] = ring_[(count - n + i) % c->loss_cap];
  return n;
}

int64_t pb_num_params(const pb_ctx* c) { return c ? c->n_params : 0; }
int64_t pb_num_ticks(const pb_ctx* c) { return c ? c->ticks : 0; }

int pb_set_launch_mode(pb_ctx* c, int32_t mode) {
  if (!c || mode < 0 || mode > 1) return fail(PB_E_INVALID, "bad launch mode");
  c->launch_mode = mode;
  return PB_OK;
}

int pb_profile_begin(pb_ctx* c, int32_t max_events) {
  if (!c || max_events <= 0) return fail(PB_E_INVALID, "bad argument");
  for (auto& e : c->evs) c->ev_pool.push_back(e);
  c->evs.clear();
  c->profiling = true;
  c->max_events = max_events;
  return PB_OK;
}

int pb_profile_end(pb_ctx* c, int32_t which, int64_t* n_launches, double* total_ms) {
  if (!c || !n_launches || !total_ms) return fail(PB_E_INVALID, "NULL argument");
  c->profiling = false;
  HIP_TRY(hipStreamSynchronize(c->stream));
  int64_t n = 0;
  double ms = 0;
  for (auto& e : c->evs) {
    if (e.cls != which) continue;
    float x = 0;
    HIP_TRY(hipEventElapsedTime(&x, e.a, e.b));
    ms += x; ++n;
  }
  *n_launches = n; *total_ms = ms;
  return PB_OK;
}

int pb_update_standalone(float* w, float* v, const float* g, float* what, int64_t n, float lr, float m,
                         float a, float b, float lrT, void* stream) {
  if (!w || !v || !g || n <= 0 || n % UPD_CHUNK) return fail(PB_E_INVALID, "n must be a positive multiple of %d", UPD_CHUNK);
  if (n / UPD_CHUNK > 0x7fffffff) return fail(PB_E_INVALID, "n too large");
  // the kernel moves 16 bytes per access
  if (((uintptr_t)w | (uintptr_t)v | (uintptr_t)g | (uintptr_t)what) % 16) return fail(PB_E_INVALID, "arrays must be 16-byte aligned");
  launch_update_flat(w, v, g, what, n, lr, m, a, b, lrT, (hipStream_t)stream);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(PB_E_HIP, "kernel launch failed: %s", hipGetErrorString(e));
  return PB_OK;
}

int pb_scale_hyperparameters(float lr_ref, float momentum_ref, int32_t n_ref, int32_t n, float* lr_out,
                             float* momentum_out) {
  if (!lr_out || !momentum_out) return fail(PB_E_INVALID, "NULL output pointer");
  if (n < 1 || n_ref < 1) return fail(PB_E_INVALID, "update sizes must be >= 1");
  if (!(momentum_ref >= 0.f && momentum_ref <= 1.f) || !(lr_ref >= 0.f))
    return fail(PB_E_INVALID, "reference momentum must be in [0,1] and reference learning rate >= 0");
  const double ratio = (double)n / (double)n_ref, mr = (double)momentum_ref;
  const double m = pow(mr, ratio);
  // m_ref = 1: (1-m)/(1-m_ref) -> n/n_ref
  const double lr = (mr == 1.0) ? (double)lr_ref * ratio * ratio : (1.0 - m) / (1.0 - mr) * ratio * (double)lr_ref;
  *lr_out = (float)lr;
  *momentum_out = (float)m;
  return PB_OK;
}

int pb_sync(pb_ctx* c) {
  if (!c) return fail(PB_E_INVALID, "NULL context");
  HIP_TRY(hipStreamSynchronize(c->stream));
  return check_device_error(c);
}

void pb_destroy(pb_ctx* c) {
  if (!c) return;
  (void)hipStreamSynchronize(c->stream);
  for (auto& e : c->evs) { (void)hipEventDestroy(e.a); (void)hipEventDestroy(e.b); }
  for (auto& e : c->ev_pool) { (void)hipEventDestroy(e.a); (void)hipEventDestroy(e.b); }
  for (int i = 0; i < pb_ctx::N_PINNED; ++i) {
    if (c->pinned[i]) (void)hipHostFree(c->pinned[i]);
    if (c->pinned_done[i]) (void)hipEventDestroy(c->pinned_done[i]);
  }
  if (c->own_arena && c->arena) (void)hipFree(c->arena);
  if (c->static_dev >= 0 && c->static_dev < MAX_STATIC_DEVS) g_static_busy[c->static_dev] = false;
  delete c;
}

}  // extern "C"

#ifdef PB_TIMING
// Development build only: workgroups per launch of a tick, in launch order.
extern "C" int pb_debug_phase_grids(pb_ctx* c, int32_t* out, int cap) {
  if (!c || !out) return -1;
  int n = 0;
  for (const Phase& p : c->phases) {
    if (n < cap) out[n] = p.tiles;
    ++n;
  }
  return n;
}
#endif
