// C ABI of the library: configuration, workspace plan, the sub-batch schedule of the paper's
// Algorithm 1 on two HIP streams, and thin single-operator wrappers.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <string>
#include <vector>

#include "common.h"

namespace oases {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
}
int hip_fail(hipError_t e, const char* what) {
  set_error("HIP error %d (%s) in %s", (int)e, hipGetErrorString(e), what);
  return OASES_EHIP;
}

// ---------------------------------------------------------------------------------------------
// schedule: operators in host issue order
// ---------------------------------------------------------------------------------------------
enum OpKind {
  // forward
  F_LN1, F_QKV, F_ATTN, F_PROJ, F_R1, F_FC1, F_FC2, F_R2,
  // backward
  B_BDR2, B_FC2_DGRAD, B_FC1_DGRAD, B_R3, B_FC2_WGRAD, B_FC1_WGRAD, B_B1_SUM, B_PROJ_DGRAD, B_PROJ_WGRAD, B_ATTN,
  B_QKV_DGRAD, B_R4, B_QKV_WGRAD, B_BQKV_SUM,
  // recompute mode: Recompute() of the saved sequences inside the backward pass
  R_LN2, R_FC1, R_LN1, R_QKV, R_ATTN,
  // stream join at the end of a pass
  JOIN,
  // rotary embedding of the LLaMA-style layer: table once per forward pass, rotation of Q and K behind QKV (forward,
  // recomputation), rotation back of dQ and dK behind the attention backward
  F_ROPE_TABLE, F_ROPE, R_ROPE, B_ROPE,
  // PROJ.wgrad and QKV.wgrad as one launch, where the shapes make that the faster way
  B_PQ_WGRAD,
  // second stage of every column reduction of the backward pass (bias and LayerNorm-parameter gradients), one launch
  B_COLSUMS
};
static const char* kOpName[] = {
    "LN1", "QKV", "ATTN", "PROJ", "R1+BDR1+LN2", "FC1+GELU", "FC2", "R2+BDR2",
    "BDR2.b", "FC2.dgrad+dGELU", "FC1.dgrad", "R3+LN2.b+BDR1.b", "FC2.wgrad", "FC1.wgrad", "b1.sum", "PROJ.dgrad",
    "PROJ.wgrad", "ATTN.b", "QKV.dgrad", "R4+LN1.b", "QKV.wgrad", "bqkv.sum",
    "LN2.r", "FC1+GELU.r", "LN1.r", "QKV.r", "ATTN.r", "join", "ROPE.table", "ROPE", "ROPE.r", "ROPE.b", "PROJ+QKV.wgrad", "colsums"};
// names of the same operator slots in the LLaMA-style layer (RMSNorm, SwiGLU)
static const char* op_name(int kind, bool llama, bool bert) {
  if (bert) {  // post-LN: the normalisation sits behind the residual sum, the layer input enters the GEMM as it is
    switch (kind) {
      case F_LN1: return "CAST";
      case R_LN1: return "CAST.r";
      case R_LN2: return "CAST2.r";
      case F_R1: return "R1+BDR1+LN1";
      case F_R2: return "R2+BDR2+LN2";
      case B_BDR2: return "LN2.b+BDR2.b";
      case B_R3: return "R3+LN1.b+BDR1.b";
      case B_R4: return "R4+LN2.b+BDR2.b";
      default: break;
    }
  }
  if (llama) {
    switch (kind) {
      case F_FC1: return "FC1+SWIGLU";
      case R_FC1: return "FC1+SWIGLU.r";
      case B_FC2_DGRAD: return "FC2.dgrad+dSWIGLU";
      case F_R1: return "R1+DR1+RMS2";
      case F_R2: return "R2+DR2";
      case B_BDR2: return "DR2.b";
      case B_R3: return "R3+RMS2.b+DR1.b";
      case B_R4: return "R4+RMS1.b";
      case F_LN1: return "RMS1";
      case R_LN1: return "RMS1.r";
      case R_LN2: return "RMS2.r";
      default: break;
    }
  }
  return kOpName[kind];
}

struct Op {
  int kind, layer, sub;
  int stream;  // 0 compute, 1 comm
  int wait;    // event to wait for before the op (-1 none)
  int record;  // event recorded after the op (-1 none)
};

// workspace tensors of a layer, in the order plan_workspace lays them out (index into oases_handle::tensors)
enum TensorId { T_u, T_mu1, T_rstd1, T_qkv, T_attn, T_lse, T_z1, T_x1, T_mu2, T_rstd2, T_v2, T_pre, T_f, T_z2, T_y, T_dz2, T_dg, T_dv2, T_dx1, T_dz1, T_da, T_delta, T_dqkv, T_du, T_dy, T_rope, T_s1, T_s2, T_ds2, T_COUNT };

struct Tensor {
  const char* name;
  size_t offset, bytes;
  bool shared;  // recompute mode: a forward activation that is rebuilt in backward, one copy for all layers
};

}  // namespace oases

using namespace oases;

struct oases_handle {
  oases_layer_cfg cfg;
  int h, nh, d, s, b, t, r, n, L, M, Ms, hp, fp, heads_l;
  int fw;        // columns of the FC1 output that is stored for backward: fp (GeLU), 2*fp (SwiGLU: gate and up)
  bool llama;    // OASES_ARCH_LLAMA: RMSNorm, rotary embedding, SwiGLU, no biases
  bool bert;     // OASES_ARCH_BERT: post-LayerNorm
  float eps, theta;
  std::vector<Op> fwd, bwd;
  int n_events;
  std::vector<hipEvent_t> events;  // created on first use
  std::vector<hipEvent_t> prof[2];  // OASES_FLAG_PROFILE: start/stop event per operator of each pass
  bool prof_ran[2] = {false, false};
  std::vector<Tensor> tensors;     // per-layer tensors, offsets relative to the layer base
  size_t layer_bytes, shared_off, scratch_comm_off, scratch_compute_off, gemm_ws_off, gemm_ws_bytes, total_bytes;
  // arena of partial rows of the backward pass's column reductions, per layer: five slots (see ColsumSlot)
  size_t colsum_off, colsum_layer_bytes, colsum_slot_off[5];
  int colsum_groups_sub, colsum_groups_all;  // row groups of a reduction over a sub-batch's rows / over all M rows
};

namespace oases {

static size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

static bool plan_workspace(oases_handle* H) {
  const size_t M = H->M, h = H->h, hp = H->hp, fp = H->fp, fw = H->fw, st = (size_t)H->b * H->heads_l * H->s;
  const size_t rope = H->llama ? (size_t)H->s * (H->d / 2) * 8 : 0;  // (cos, sin) table; layer 0's copy is the one in use
  struct { const char* n; size_t bytes; } list[] = {
      {"u", M * h * 2},      {"mu1", M * 4},        {"rstd1", M * 4},      {"qkv", M * 3 * hp * 2}, {"attn", M * hp * 2},
      {"lse", st * 4},       {"z1", M * h * 4},     {"x1", M * h * 4},     {"mu2", M * 4},          {"rstd2", M * 4},
      {"v2", M * h * 2},     {"pre", M * fw * 2},   {"f", M * fp * 2},     {"z2", M * h * 4},       {"y", M * h * 4},
      {"dz2", M * h * 2},    {"dg", M * fw * 2},    {"dv2", M * h * 4},    {"dx1", M * h * 4},      {"dz1", M * h * 2},
      {"da", M * hp * 2},    {"delta", st * 4},     {"dqkv", M * 3 * hp * 2}, {"du", M * h * 4},    {"dy", M * h * 4},
      {"rope", rope},
      // post-LN: the sums in front of the two LayerNorms (their backward needs them) and the gradient of the second one
      {"s1", H->bert ? M * h * 4 : 0}, {"s2", H->bert ? M * h * 4 : 0}, {"ds2", H->bert ? M * h * 4 : 0}};
  // Recompute mode (the paper's fine-grained recomputation, Sec. IV-B): only the input of each computation
  // sequence is kept per layer -- x (= y of the layer below) for [LN1,QKV,ATTN,PROJ] and x1 for [LN2,FC1,FC2] -- the
  // activations in between are rebuilt inside backward and live in one region shared by all layers.
  const bool recompute = H->cfg.flags & OASES_FLAG_RECOMPUTE;
  static const char* kAct[] = {"u", "qkv", "attn", "lse", "v2", "pre", "f", "z1", "z2"};
  size_t off = 0, soff = 0;
  for (auto& e : list) {
    bool act = false;
    for (const char* a : kAct) act = act || !strcmp(a, e.n);
    if (recompute && act) {
      H->tensors.push_back(Tensor{e.n, soff, e.bytes, true});
      soff += align_up(e.bytes);
    } else {
      H->tensors.push_back(Tensor{e.n, off, e.bytes, false});
      off += align_up(e.bytes);
    }
  }
  H->layer_bytes = off;
  static const char* kIdNames[T_COUNT] = {"u", "mu1", "rstd1", "qkv", "attn", "lse", "z1", "x1", "mu2", "rstd2", "v2", "pre", "f", "z2", "y", "dz2", "dg", "dv2", "dx1", "dz1", "da", "delta", "dqkv", "du", "dy", "rope", "s1", "s2", "ds2"};
  for (int i = 0; i < T_COUNT; i++)
    if ((int)H->tensors.size() != T_COUNT || strcmp(H->tensors[i].name, kIdNames[i])) return false;  // TensorId out of step with the list above
  size_t tot = off * H->L;
  H->shared_off = tot;
  tot += soff;
  H->scratch_comm_off = tot;
  tot += align_up((size_t)3 * kColPartials * h * 4);
  H->scratch_compute_off = tot;
  size_t wide = 3 * hp > fw ? 3 * hp : fw;
  tot += align_up((size_t)kColPartials * wide * 4);
  // Partial rows of the column reductions of a backward pass, kept until its single second-stage launch.  Slots of a
  // layer: three reduction-point kernels with up to three output arrays each, laid out [array][sub-batch][group][h], and
  // the two bias sums over all rows [group][columns].
  {
    H->colsum_groups_sub = colsum_groups(H->Ms);
    H->colsum_groups_all = colsum_groups(H->M);
    const size_t tri = align_up((size_t)3 * H->n * H->colsum_groups_sub * h * 4);
    size_t o = 0;
    for (int k = 0; k < 3; k++) { H->colsum_slot_off[k] = o; o += tri; }
    H->colsum_slot_off[3] = o; o += align_up((size_t)H->colsum_groups_all * fw * 4);
    H->colsum_slot_off[4] = o; o += align_up((size_t)H->colsum_groups_all * 3 * hp * 4);
    H->colsum_layer_bytes = o;
    H->colsum_off = tot;
    tot += o * H->L;
  }
  // split-K partial planes: up to 8 fp32 copies of the widest GEMM output of the layer
  const size_t Ms = H->Ms;
  size_t mn = Ms * h;
  for (size_t v : {Ms * 3 * hp, Ms * fw, fw * h, h * 3 * hp, hp * h}) mn = v > mn ? v : mn;
  H->gemm_ws_off = tot;
  H->gemm_ws_bytes = 8 * mn * 4 < kSplitKWorkspaceBytes ? 8 * mn * 4 : kSplitKWorkspaceBytes;
  tot += align_up(H->gemm_ws_bytes);
  H->total_bytes = tot;
  return true;
}

static size_t tensor_off(const oases_handle* H, const char* name, int layer) {
  for (auto& t : H->tensors)
    if (!strcmp(t.name, name)) return t.shared ? H->shared_off + t.offset : (size_t)layer * H->layer_bytes + t.offset;
  return (size_t)-1;
}

// Events: ev(layer, point, sub, kind): point 0..3 = R1..R4, kind 0 = "partial ready" (compute -> comm),
// kind 1 = "reduced and consumed" (comm -> compute).
static int ev_id(const oases_handle* H, int layer, int point, int sub, int kind) {
  return ((layer * 4 + point) * H->n + sub) * 2 + kind;
}

// Alg. 1 "At Forward": walk the operator sequence; at every communication operator start it for the
// current sub-batch and switch to the next sub-batch, rewinding to the start of the computation
// sequence; advance past the communication operator once every sub-batch has been through.
static void build_forward(oases_handle* H) {
  auto& ops = H->fwd;
  const int n = H->n;
  if (H->llama) ops.push_back(Op{F_ROPE_TABLE, 0, -1, 0, -1, -1});
  for (int l = 0; l < H->L; l++) {
    for (int j = 0; j < n; j++) {
      int w = l > 0 ? ev_id(H, l - 1, 1, j, 1) : -1;  // input of this layer comes out of R2 of the layer below
      if (l == 0) { ops.push_back(Op{F_LN1, l, j, 0, -1, -1}); }
      ops.push_back(Op{F_QKV, l, j, 0, w, -1});
      if (H->llama) ops.push_back(Op{F_ROPE, l, j, 0, -1, -1});
      ops.push_back(Op{F_ATTN, l, j, 0, -1, -1});
      ops.push_back(Op{F_PROJ, l, j, 0, -1, ev_id(H, l, 0, j, 0)});
      ops.push_back(Op{F_R1, l, j, 1, ev_id(H, l, 0, j, 0), ev_id(H, l, 0, j, 1)});
    }
    for (int j = 0; j < n; j++) {
      ops.push_back(Op{F_FC1, l, j, 0, ev_id(H, l, 0, j, 1), -1});
      ops.push_back(Op{F_FC2, l, j, 0, -1, ev_id(H, l, 1, j, 0)});
      ops.push_back(Op{F_R2, l, j, 1, ev_id(H, l, 1, j, 0), ev_id(H, l, 1, j, 1)});
    }
  }
  for (int j = 0; j < n; j++) ops.push_back(Op{JOIN, H->L - 1, j, 0, ev_id(H, H->L - 1, 1, j, 1), -1});
}

// Alg. 1 "At Backward" with stored activations: saved sequences are popped last-first (so the last
// sub-batch goes first); the backward operators of a sequence run until its communication operator,
// which is started asynchronously; the operators behind it (here: fused into the reduction-point kernel
// on the communication stream) fill in.  No reduction depends on a weight gradient, and a weight gradient sums
// over token rows, so the weight-gradient GEMMs of all sub-batches of a block are merged into one contraction
// over all M rows and issued behind the last sub-batch's reduction start, under which they run.
static void build_backward(oases_handle* H) {
  auto& ops = H->bwd;
  const int n = H->n, L = H->L;
  const bool recompute = H->cfg.flags & OASES_FLAG_RECOMPUTE;
  const bool chunks = H->n > H->b;  // sub-batches are parts of a sequence: attention of a chunk reads earlier chunks' K/V
  for (int j = n - 1; j >= 0; j--) ops.push_back(Op{B_BDR2, L - 1, j, 1, -1, ev_id(H, L - 1, 1, j, 1)});
  for (int l = L - 1; l >= 0; l--) {
    for (int j = n - 1; j >= 0; j--) {
      // dZ2 of this layer comes from the trailing BDR2.b (top layer) or from R4 of the layer above
      int w = l == L - 1 ? ev_id(H, l, 1, j, 1) : ev_id(H, l + 1, 3, j, 1);
      if (recompute) {  // Recompute() of the saved sequence [LN2, FC1]: starts at x1, behind the forward reduction
        ops.push_back(Op{R_LN2, l, j, 0, -1, -1});
        ops.push_back(Op{R_FC1, l, j, 0, -1, -1});
      }
      ops.push_back(Op{B_FC2_DGRAD, l, j, 0, w, -1});
      ops.push_back(Op{B_FC1_DGRAD, l, j, 0, -1, ev_id(H, l, 2, j, 0)});
      ops.push_back(Op{B_R3, l, j, 1, ev_id(H, l, 2, j, 0), ev_id(H, l, 2, j, 1)});
    }
    // weight gradients: one contraction over the rows of ALL sub-batches (sub = -1), behind the last reduction start
    ops.push_back(Op{B_FC2_WGRAD, l, -1, 0, -1, -1});
    ops.push_back(Op{B_FC1_WGRAD, l, -1, 0, -1, -1});
    if (!H->llama) ops.push_back(Op{B_B1_SUM, l, -1, 0, -1, -1});
    if (recompute && chunks)  // K/V of every chunk must exist again before any chunk's attention is rebuilt
      for (int j = n - 1; j >= 0; j--) {
        ops.push_back(Op{R_LN1, l, j, 0, -1, -1});
        ops.push_back(Op{R_QKV, l, j, 0, -1, -1});
        if (H->llama) ops.push_back(Op{R_ROPE, l, j, 0, -1, -1});
      }
    if (recompute && chunks)  // ... and the attention output / LSE of later chunks before an earlier chunk's dK/dV
      for (int j = 0; j < n; j++) ops.push_back(Op{R_ATTN, l, j, 0, -1, -1});
    for (int j = n - 1; j >= 0; j--) {
      if (recompute && !chunks) {  // Recompute() of [LN1, QKV, ATTN]: starts at the layer input
        ops.push_back(Op{R_LN1, l, j, 0, -1, -1});
        ops.push_back(Op{R_QKV, l, j, 0, -1, -1});
        if (H->llama) ops.push_back(Op{R_ROPE, l, j, 0, -1, -1});
        ops.push_back(Op{R_ATTN, l, j, 0, -1, -1});
      }
      ops.push_back(Op{B_PROJ_DGRAD, l, j, 0, ev_id(H, l, 2, j, 1), -1});
      ops.push_back(Op{B_ATTN, l, j, 0, -1, -1});
      if (H->llama) ops.push_back(Op{B_ROPE, l, j, 0, -1, -1});
      ops.push_back(Op{B_QKV_DGRAD, l, j, 0, -1, ev_id(H, l, 3, j, 0)});
      ops.push_back(Op{B_R4, l, j, 1, ev_id(H, l, 3, j, 0), ev_id(H, l, 3, j, 1)});
    }
    if (gemm_tn_pair_wins(H->M, H->hp, H->h, H->h, 3 * H->hp) && gemm_span_fits(H->M, H->h) && gemm_span_fits(H->M, 3 * H->hp)) {
      ops.push_back(Op{B_PQ_WGRAD, l, -1, 0, -1, -1});
    } else {
      ops.push_back(Op{B_PROJ_WGRAD, l, -1, 0, -1, -1});
      ops.push_back(Op{B_QKV_WGRAD, l, -1, 0, -1, -1});
    }
    if (!H->llama) ops.push_back(Op{B_BQKV_SUM, l, -1, 0, -1, -1});
  }
  for (int j = n - 1; j >= 0; j--) ops.push_back(Op{JOIN, 0, j, 0, ev_id(H, 0, 3, j, 1), -1});
  // every first stage of a column reduction has run (both streams are joined): one launch adds up all partial rows
  ops.push_back(Op{B_COLSUMS, 0, -1, 0, -1, -1});
}

static int check_ptrs(const void* const* p, int n, const char* who) {
  for (int i = 0; i < n; i++) {
    if (!p[i]) { set_error("%s: NULL device pointer (argument %d)", who, i); return OASES_ENULL; }
    if (!aligned16(p[i])) { set_error("%s: device pointer %d not 16-byte aligned", who, i); return OASES_EALIGN; }
  }
  return 0;
}

static int ensure_events(oases_handle* H) {
  if (!H->events.empty()) return 0;
  H->events.resize(H->n_events);
  for (auto& e : H->events) {
    hipError_t err = hipEventCreateWithFlags(&e, hipEventDisableTiming);
    if (err != hipSuccess) {
      H->events.clear();
      return hip_fail(err, "hipEventCreateWithFlags");
    }
  }
  return 0;
}

struct Run {
  oases_handle* H;
  const oases_weights* w;
  const oases_grads* g;
  const oases_peer_sums* peers;
  char* ws;
  const float* x;   // forward input
  float* y;         // forward output
  const float* dy;  // backward input
  float* dx;        // backward output
  hipStream_t st[2];
  // segment-level calls: the tensor at reduction point k (0..3 = R1..R4) that the producing GEMM writes (instead of the
  // workspace partial) and that the consuming kernel reads as the already reduced sum (instead of partial + peer sum)
  float* partial_out[4] = {nullptr, nullptr, nullptr, nullptr};
  const float* reduced_in[4] = {nullptr, nullptr, nullptr, nullptr};
  // whole backward pass: the second stage of the column reductions is collected here and launched once (B_COLSUMS);
  // segment calls finish every reduction at once (defer_colsums = false)
  bool defer_colsums = false;
  std::vector<ColsumJob>* jobs = nullptr;  // capacity fixed before the pass
  int* n_jobs = nullptr;
};

template <typename T>
static T* wsp(const Run& R, TensorId id, int layer) {  // offsets were resolved when the handle was created
  const Tensor& t = R.H->tensors[id];
  return reinterpret_cast<T*>(R.ws + (t.shared ? R.H->shared_off + t.offset : (size_t)layer * R.H->layer_bytes + t.offset));
}

static int run_op(const Run& R, const Op& op) {
  const oases_handle* H = R.H;
  const int l = op.layer, j = op.sub, h = H->h, hp = H->hp, fp = H->fp, L = H->L;
  const int Ms = j < 0 ? H->M : H->Ms;              // sub = -1: all rows (merged weight gradients)
  const size_t r0 = j < 0 ? 0 : (size_t)j * Ms;     // first token row of the sub-batch
  hipStream_t s = R.st[op.stream];
  const oases_weights& W = R.w[l];
  const oases_peer_sums* P = R.peers ? &R.peers[l] : nullptr;
  auto peer = [&](const void* base) -> const float* { return base ? (const float*)base + r0 * h : nullptr; };
  static const TensorId kPartId[4] = {T_z1, T_z2, T_dv2, T_du};
  // reduction point k: where its producer writes this sub-batch's rows, what its consumer reads, and the peer sum beside it
  auto part_w = [&](int k) -> float* { return (R.partial_out[k] ? R.partial_out[k] : wsp<float>(R, kPartId[k], l)) + r0 * h; };
  auto part_r = [&](int k) -> const float* { return (R.reduced_in[k] ? R.reduced_in[k] : wsp<float>(R, kPartId[k], l)) + r0 * h; };
  auto peer_k = [&](int k) -> const float* {
    if (R.reduced_in[k] || !P) return nullptr;   // an already reduced tensor has the peers in it
    return peer(k == 0 ? P->fwd_attn : k == 1 ? P->fwd_ffn : k == 2 ? P->bwd_ffn : P->bwd_attn);
  };
  const float p = H->cfg.dropout_p;
  const uint64_t seed = H->cfg.seed;
  const float* xin = l == 0 ? R.x : wsp<float>(R, T_y, l - 1);                 // layer input
  float* yout = l == L - 1 ? R.y : wsp<float>(R, T_y, l);                      // layer output
  const float* dyin = R.dy && l == L - 1 ? R.dy : wsp<float>(R, T_dy, l);      // gradient of the layer output
  float* dxout = l == 0 ? R.dx : wsp<float>(R, T_dy, l - 1);                   // gradient of the layer input
  float* scr_comm = reinterpret_cast<float*>(R.ws + H->scratch_comm_off);
  float* scr_comp = reinterpret_cast<float*>(R.ws + H->scratch_compute_off);
  // Column reductions.  slot: 0 the top layer's dropout backward, 1 / 2 the reduction-point kernels behind R3 / R4, 3 / 4 the
  // bias sums of FC1 / QKV.  Whole pass: the partial rows go to this operator's slot of the arena and the second stage
  // joins the list; otherwise they go to the stream's scratch and the second stage follows at once.
  ColsumSink sink;
  float* cs_scratch = nullptr;
  auto colsum = [&](int slot) -> ColsumSink* {
    if (!R.defer_colsums) { cs_scratch = slot < 3 ? scr_comm : scr_comp; return nullptr; }
    float* base = reinterpret_cast<float*>(R.ws + H->colsum_off + (size_t)l * H->colsum_layer_bytes + H->colsum_slot_off[slot]);
    if (slot < 3) {
      const int g = H->colsum_groups_sub;
      sink.first_row = j * g;
      sink.rows_total = H->n * g;
      sink.kstride = (size_t)H->n * g * h;
      cs_scratch = base + (size_t)sink.first_row * h;
    } else {
      sink.first_row = 0;
      sink.rows_total = H->colsum_groups_all;
      sink.kstride = 0;
      cs_scratch = base;
    }
    sink.jobs = R.jobs->data();
    sink.n = *R.n_jobs;
    sink.cap = (int)R.jobs->size();
    return &sink;
  };
  auto colsum_done = [&](int rc) -> int {  // behind a launch that was given colsum(...): keep what it put on the list
    if (rc == 0 && R.defer_colsums) {
      if (sink.overflow) { set_error("internal error: column-reduction job list too short"); return OASES_EINVAL; }
      *R.n_jobs = sink.n;
    }
    return rc;
  };
  void* gws = R.ws + H->gemm_ws_off;  // split-K partial planes (compute stream only)
  const int pin = (H->cfg.flags & OASES_FLAG_PIN_GEMM) ? H->M : 0;  // kernels chosen as for all M rows, whatever the sub-batch
  uint16_t* u = wsp<uint16_t>(R, T_u, l);
  uint16_t* qkv = wsp<uint16_t>(R, T_qkv, l);
  uint16_t* attn = wsp<uint16_t>(R, T_attn, l);
  uint16_t* v2 = wsp<uint16_t>(R, T_v2, l);
  uint16_t* pre = wsp<uint16_t>(R, T_pre, l);
  uint16_t* f = wsp<uint16_t>(R, T_f, l);
  const bool rms = H->llama;   // RMSNorm, no biases: the bias / beta / mean arguments below are NULL and unused
  const int fw = H->fw;
  if (H->bert) {
    // Post-LN layer: s1 = x + drop(Z1 + bo), x1 = LN1(s1); s2 = x1 + drop(Z2 + b2), y = LN2(s2).  The GEMMs read bf16
    // copies of x and x1; the reduction-point kernels write the sum (for the LayerNorm backward), the normalised row in
    // fp32 (residual stream) and in bf16 (next GEMM operand).  Backward: the whole gradient of a LayerNorm's output
    // (residual branch included) passes through it.
    switch (op.kind) {
      case F_LN1:
      case R_LN1:
        return launch_cast_bf16(xin + r0 * h, u + r0 * h, (int64_t)Ms * h, s);
      case R_LN2:
        return launch_cast_bf16(wsp<float>(R, T_x1, l) + r0 * h, v2 + r0 * h, (int64_t)Ms * h, s);
      case F_R1:
        return launch_bdr_ln(part_r(0), peer_k(0), (const float*)W.bo, xin + r0 * h,
                             wsp<float>(R, T_s1, l) + r0 * h, (const float*)W.ln1_g, (const float*)W.ln1_b, v2 + r0 * h,
                             wsp<float>(R, T_mu1, l) + r0, wsp<float>(R, T_rstd1, l) + r0, Ms, h, H->eps,
                             make_drop_cfg(seed, l, 0, p), (int64_t)r0, s, false, wsp<float>(R, T_x1, l) + r0 * h);
      case F_R2: {
        const bool more = l + 1 < L;  // the bf16 copy of y is the next layer's GEMM operand
        return launch_bdr_ln(part_r(1), peer_k(1), (const float*)W.b2,
                             wsp<float>(R, T_x1, l) + r0 * h, wsp<float>(R, T_s2, l) + r0 * h, (const float*)W.ln2_g,
                             (const float*)W.ln2_b, more ? wsp<uint16_t>(R, T_u, l + 1) + r0 * h : nullptr,
                             wsp<float>(R, T_mu2, l) + r0, wsp<float>(R, T_rstd2, l) + r0, Ms, h, H->eps,
                             make_drop_cfg(seed, l, 1, p), (int64_t)r0, s, false, yout + r0 * h);
      }
      case B_BDR2:  // top of the stack: dy through LN2, then the dropout backward of the FFN branch
        { ColsumSink* cs = colsum(0); return colsum_done(launch_layernorm_bwd(dyin + r0 * h, nullptr, nullptr, wsp<float>(R, T_s2, l) + r0 * h, wsp<float>(R, T_mu2, l) + r0,
                                    wsp<float>(R, T_rstd2, l) + r0, (const float*)W.ln2_g, wsp<float>(R, T_ds2, l) + r0 * h,
                                    (float*)R.g[l].ln2_g, (float*)R.g[l].ln2_b, wsp<uint16_t>(R, T_dz2, l) + r0 * h, (float*)R.g[l].b2, Ms,
                                    h, make_drop_cfg(seed, l, 1, p), (int64_t)r0, cs_scratch, s, false, true, cs)); }
      case B_R3:  // gradient of x1 = FFN-input gradient (reduced) + residual branch ds2, through LN1
        { ColsumSink* cs = colsum(1); return colsum_done(launch_layernorm_bwd(part_r(2), peer_k(2), wsp<float>(R, T_ds2, l) + r0 * h,
                                    wsp<float>(R, T_s1, l) + r0 * h, wsp<float>(R, T_mu1, l) + r0, wsp<float>(R, T_rstd1, l) + r0,
                                    (const float*)W.ln1_g, wsp<float>(R, T_dx1, l) + r0 * h, (float*)R.g[l].ln1_g, (float*)R.g[l].ln1_b,
                                    wsp<uint16_t>(R, T_dz1, l) + r0 * h, (float*)R.g[l].bo, Ms, h, make_drop_cfg(seed, l, 0, p),
                                    (int64_t)r0, cs_scratch, s, false, true, cs)); }
      case B_R4:  // gradient of the layer input = QKV-input gradient (reduced) + residual branch ds1
        if (l == 0)
          return launch_add3(part_r(3), wsp<float>(R, T_dx1, l) + r0 * h, peer_k(3),
                             dxout + r0 * h, (int64_t)Ms * h, s);
        // ... which is the output gradient of the layer below: straight through its LN2 and FFN-branch dropout
        { ColsumSink* cs = colsum(2); return colsum_done(launch_layernorm_bwd(part_r(3), peer_k(3), wsp<float>(R, T_dx1, l) + r0 * h,
                                    wsp<float>(R, T_s2, l - 1) + r0 * h, wsp<float>(R, T_mu2, l - 1) + r0,
                                    wsp<float>(R, T_rstd2, l - 1) + r0, (const float*)R.w[l - 1].ln2_g,
                                    wsp<float>(R, T_ds2, l - 1) + r0 * h, (float*)R.g[l - 1].ln2_g, (float*)R.g[l - 1].ln2_b,
                                    wsp<uint16_t>(R, T_dz2, l - 1) + r0 * h, (float*)R.g[l - 1].b2, Ms, h,
                                    make_drop_cfg(seed, l - 1, 1, p), (int64_t)r0, cs_scratch, s, false, true, cs)); }
      default:
        break;  // GEMMs, attention, bias sums: as in the GPT layer
    }
  }
  switch (op.kind) {
    case F_LN1:
      return launch_layernorm_fwd(xin + r0 * h, (const float*)W.ln1_g, (const float*)W.ln1_b, u + r0 * h,
                                  wsp<float>(R, T_mu1, l) + r0, wsp<float>(R, T_rstd1, l) + r0, Ms, h, H->eps, s, rms);
    case F_QKV:
      return launch_gemm(OASES_GEMM_NN, rms ? OASES_EPI_BF16 : OASES_EPI_BIAS_BF16, Ms, 3 * hp, h, u + r0 * h, h, W.wqkv, 3 * hp,
                         qkv + r0 * 3 * hp, 3 * hp, (const float*)W.bqkv, nullptr, 0, gws, H->gemm_ws_bytes, 0, s, pin);
    case F_ROPE_TABLE:
      return launch_rope_table(wsp<float>(R, T_rope, 0), H->s, H->d, H->theta, s);
    case F_ROPE:
    case R_ROPE:
      return launch_rope(qkv + r0 * 3 * hp, 3 * hp, Ms, (int64_t)r0, H->s, H->heads_l, H->d, wsp<float>(R, T_rope, 0), 0, s);
    case B_ROPE:
      return launch_rope(wsp<uint16_t>(R, T_dqkv, l) + r0 * 3 * hp, 3 * hp, Ms, (int64_t)r0, H->s, H->heads_l, H->d,
                         wsp<float>(R, T_rope, 0), 1, s);
    case F_ATTN:
      return launch_attention_fwd(qkv, attn, wsp<float>(R, T_lse, l), H->b, H->s, H->heads_l, H->d, H->cfg.causal, (int)r0, Ms, s,
                                  seed, l, H->cfg.attn_dropout_p, H->r * H->heads_l, H->nh);
    case F_PROJ:
      return launch_gemm(OASES_GEMM_NN, OASES_EPI_F32, Ms, h, hp, attn + r0 * hp, hp, W.wo, h, part_w(0), h,
                         nullptr, nullptr, 0, gws, H->gemm_ws_bytes, 0, s, pin);
    case F_R1:
      return launch_bdr_ln(part_r(0), peer_k(0), (const float*)W.bo, xin + r0 * h,
                           wsp<float>(R, T_x1, l) + r0 * h, (const float*)W.ln2_g, (const float*)W.ln2_b, v2 + r0 * h,
                           wsp<float>(R, T_mu2, l) + r0, wsp<float>(R, T_rstd2, l) + r0, Ms, h, H->eps,
                           make_drop_cfg(seed, l, 0, p), (int64_t)r0, s, rms);
    case F_FC1:
      if (H->llama)  // w1 = [gate | up] columns interleaved in blocks of 32; pre = both pre-activations, f = silu(gate)*up
        return launch_gemm(OASES_GEMM_NN, OASES_EPI_SWIGLU, Ms, fw, h, v2 + r0 * h, h, W.w1, fw, f + r0 * fp, fp, nullptr,
                           pre + r0 * fw, fw, gws, H->gemm_ws_bytes, 0, s, pin);
      return launch_gemm(OASES_GEMM_NN, OASES_EPI_BIAS_GELU, Ms, fp, h, v2 + r0 * h, h, W.w1, fp, f + r0 * fp, fp,
                         (const float*)W.b1, pre + r0 * fp, fp, gws, H->gemm_ws_bytes, 0, s, pin);
    case F_FC2:
      return launch_gemm(OASES_GEMM_NN, OASES_EPI_F32, Ms, h, fp, f + r0 * fp, fp, W.w2, h, part_w(1), h,
                         nullptr, nullptr, 0, gws, H->gemm_ws_bytes, 0, s, pin);
    case F_R2: {
      const bool more = l + 1 < L;  // fuse the next layer's LN1 behind this layer's output
      return launch_bdr_ln(part_r(1), peer_k(1), (const float*)W.b2,
                           wsp<float>(R, T_x1, l) + r0 * h, yout + r0 * h, more ? (const float*)R.w[l + 1].ln1_g : nullptr,
                           more ? (const float*)R.w[l + 1].ln1_b : nullptr, more ? wsp<uint16_t>(R, T_u, l + 1) + r0 * h : nullptr,
                           more ? wsp<float>(R, T_mu1, l + 1) + r0 : nullptr, more ? wsp<float>(R, T_rstd1, l + 1) + r0 : nullptr,
                           Ms, h, H->eps, make_drop_cfg(seed, l, 1, p), (int64_t)r0, s, rms);
    }
    // ---------------------------------------------------------------- backward
    case B_BDR2:
      { ColsumSink* cs = colsum(0); return colsum_done(launch_dropout_bwd(dyin + r0 * h, wsp<uint16_t>(R, T_dz2, l) + r0 * h, (float*)R.g[l].b2, Ms, h,
                                make_drop_cfg(seed, l, 1, p), (int64_t)r0, cs_scratch, s, cs)); }
    case B_FC2_DGRAD:
      if (H->llama)
        return launch_gemm(OASES_GEMM_NT, OASES_EPI_DSWIGLU, Ms, fp, h, wsp<uint16_t>(R, T_dz2, l) + r0 * h, h, W.w2, h,
                           wsp<uint16_t>(R, T_dg, l) + r0 * fw, fw, nullptr, pre + r0 * fw, fw, gws, H->gemm_ws_bytes, 0, s, pin);
      return launch_gemm(OASES_GEMM_NT, OASES_EPI_DGELU, Ms, fp, h, wsp<uint16_t>(R, T_dz2, l) + r0 * h, h, W.w2, h,
                         wsp<uint16_t>(R, T_dg, l) + r0 * fp, fp, nullptr, pre + r0 * fp, fp, gws, H->gemm_ws_bytes, 0, s, pin);
    case B_FC1_DGRAD:
      return launch_gemm(OASES_GEMM_NT, OASES_EPI_F32, Ms, h, fw, wsp<uint16_t>(R, T_dg, l) + r0 * fw, fw, W.w1, fw,
                         part_w(2), h, nullptr, nullptr, 0, gws, H->gemm_ws_bytes, 0, s, pin);
    case B_R3:
      { ColsumSink* cs = colsum(1); return colsum_done(launch_layernorm_bwd(part_r(2), peer_k(2), dyin + r0 * h,
                                  wsp<float>(R, T_x1, l) + r0 * h, wsp<float>(R, T_mu2, l) + r0, wsp<float>(R, T_rstd2, l) + r0,
                                  (const float*)W.ln2_g, wsp<float>(R, T_dx1, l) + r0 * h, (float*)R.g[l].ln2_g,
                                  (float*)R.g[l].ln2_b, wsp<uint16_t>(R, T_dz1, l) + r0 * h, (float*)R.g[l].bo, Ms, h,
                                  make_drop_cfg(seed, l, 0, p), (int64_t)r0, cs_scratch, s, rms, false, cs)); }
    case B_FC2_WGRAD:
      return launch_gemm(OASES_GEMM_TN, 0, fp, h, Ms, f + r0 * fp, fp, wsp<uint16_t>(R, T_dz2, l) + r0 * h, h, R.g[l].w2, h,
                         nullptr, nullptr, 0, gws, H->gemm_ws_bytes, 0, s);
    case B_FC1_WGRAD:
      return launch_gemm(OASES_GEMM_TN, 0, h, fw, Ms, v2 + r0 * h, h, wsp<uint16_t>(R, T_dg, l) + r0 * fw, fw, R.g[l].w1, fw,
                         nullptr, nullptr, 0, gws, H->gemm_ws_bytes, 0, s);
    case B_B1_SUM:
      { ColsumSink* cs = colsum(3); return colsum_done(launch_colsum_bf16(wsp<uint16_t>(R, T_dg, l) + r0 * fp, fp, Ms, fp, (float*)R.g[l].b1, cs_scratch, s, cs)); }
    case B_PROJ_DGRAD:
      return launch_gemm(OASES_GEMM_NT, OASES_EPI_BF16, Ms, hp, h, wsp<uint16_t>(R, T_dz1, l) + r0 * h, h, W.wo, h,
                         wsp<uint16_t>(R, T_da, l) + r0 * hp, hp, nullptr, nullptr, 0, gws, H->gemm_ws_bytes, 0, s, pin);
    case B_PROJ_WGRAD:
      return launch_gemm(OASES_GEMM_TN, 0, hp, h, Ms, attn + r0 * hp, hp, wsp<uint16_t>(R, T_dz1, l) + r0 * h, h, R.g[l].wo, h,
                         nullptr, nullptr, 0, gws, H->gemm_ws_bytes, 0, s);
    case B_ATTN:
      return launch_attention_bwd(qkv, attn, wsp<uint16_t>(R, T_da, l), wsp<float>(R, T_lse, l), wsp<float>(R, T_delta, l),
                                  wsp<uint16_t>(R, T_dqkv, l), H->b, H->s, H->heads_l, H->d, H->cfg.causal, (int)r0, Ms, s, seed, l,
                                  H->cfg.attn_dropout_p, H->r * H->heads_l, H->nh);
    case B_QKV_DGRAD:
      return launch_gemm(OASES_GEMM_NT, OASES_EPI_F32, Ms, h, 3 * hp, wsp<uint16_t>(R, T_dqkv, l) + r0 * 3 * hp, 3 * hp, W.wqkv,
                         3 * hp, part_w(3), h, nullptr, nullptr, 0, gws, H->gemm_ws_bytes, 0, s, pin);
    case B_R4: {
      const bool more = l > 0;  // fuse the dropout backward of the layer below (its BDR2) behind dx
      { ColsumSink* cs = colsum(2); return colsum_done(launch_layernorm_bwd(part_r(3), peer_k(3),
                                  wsp<float>(R, T_dx1, l) + r0 * h, xin + r0 * h, wsp<float>(R, T_mu1, l) + r0,
                                  wsp<float>(R, T_rstd1, l) + r0, (const float*)W.ln1_g, dxout + r0 * h, (float*)R.g[l].ln1_g,
                                  (float*)R.g[l].ln1_b, more ? wsp<uint16_t>(R, T_dz2, l - 1) + r0 * h : nullptr,
                                  more ? (float*)R.g[l - 1].b2 : nullptr, Ms, h, make_drop_cfg(seed, l - 1, 1, p), (int64_t)r0,
                                  cs_scratch, s, rms, false, cs)); }
    }
    case B_QKV_WGRAD:
      return launch_gemm(OASES_GEMM_TN, 0, h, 3 * hp, Ms, u + r0 * h, h, wsp<uint16_t>(R, T_dqkv, l) + r0 * 3 * hp, 3 * hp,
                         R.g[l].wqkv, 3 * hp, nullptr, nullptr, 0, gws, H->gemm_ws_bytes, 0, s);
    case B_PQ_WGRAD:
      return launch_gemm_tn_pair(Ms, hp, h, attn + r0 * hp, hp, wsp<uint16_t>(R, T_dz1, l) + r0 * h, h, R.g[l].wo, h, h, 3 * hp, u + r0 * h, h,
                                 wsp<uint16_t>(R, T_dqkv, l) + r0 * 3 * hp, 3 * hp, R.g[l].wqkv, 3 * hp, s);
    case B_BQKV_SUM:
      { ColsumSink* cs = colsum(4); return colsum_done(launch_colsum_bf16(wsp<uint16_t>(R, T_dqkv, l) + r0 * 3 * hp, 3 * hp, Ms, 3 * hp, (float*)R.g[l].bqkv, cs_scratch, s, cs)); }
    // ---------------------------------------------------------------- recompute: the forward kernels again
    case R_LN1:
      return launch_layernorm_fwd(xin + r0 * h, (const float*)W.ln1_g, (const float*)W.ln1_b, u + r0 * h,
                                  wsp<float>(R, T_mu1, l) + r0, wsp<float>(R, T_rstd1, l) + r0, Ms, h, H->eps, s, rms);
    case R_QKV: {
      Op f = op;
      f.kind = F_QKV;
      return run_op(R, f);
    }
    case R_ATTN: {
      Op f = op;
      f.kind = F_ATTN;
      return run_op(R, f);
    }
    case R_LN2:
      return launch_layernorm_fwd(wsp<float>(R, T_x1, l) + r0 * h, (const float*)W.ln2_g, (const float*)W.ln2_b, v2 + r0 * h,
                                  wsp<float>(R, T_mu2, l) + r0, wsp<float>(R, T_rstd2, l) + r0, Ms, h, H->eps, s, rms);
    case R_FC1: {
      Op f = op;
      f.kind = F_FC1;
      return run_op(R, f);
    }
    case JOIN:
      return 0;
    case B_COLSUMS: {
      if (!R.defer_colsums) return 0;
      const int rc = launch_colsum_finalize(R.jobs->data(), *R.n_jobs, s);
      *R.n_jobs = 0;
      return rc;
    }
  }
  set_error("unknown operator %d", op.kind);
  return OASES_EINVAL;
}

static int run_ops(const Run& R, const std::vector<Op>& ops) {
  oases_handle* H = R.H;
  const bool serial = (H->cfg.flags & OASES_FLAG_SERIALISE) || R.st[0] == R.st[1];
  if (!serial) {
    int rc = ensure_events(H);
    if (rc) return rc;
  }
  if (!serial) {  // everything already enqueued on stream_compute (inputs) precedes the work on stream_comm
    OASES_HIP(hipEventRecord(H->events[H->n_events - 1], R.st[0]));
    OASES_HIP(hipStreamWaitEvent(R.st[1], H->events[H->n_events - 1], 0));
  }
  const bool profile = H->cfg.flags & OASES_FLAG_PROFILE;
  const int pass = &ops == &H->bwd;
  if (profile && H->prof[pass].empty()) {
    H->prof[pass].resize(2 * ops.size());
    for (auto& e : H->prof[pass]) {
      hipError_t err = hipEventCreate(&e);
      if (err != hipSuccess) {
        H->prof[pass].clear();
        return hip_fail(err, "hipEventCreate");
      }
    }
  }
  size_t i = 0;
  for (const Op& op0 : ops) {
    Op op = op0;
    if (serial) op.stream = 0;
    if (!serial && op.wait >= 0) OASES_HIP(hipStreamWaitEvent(R.st[op.stream], H->events[op.wait], 0));
    if (profile) OASES_HIP(hipEventRecord(H->prof[pass][2 * i], R.st[op.stream]));
    int rc = run_op(R, op);
    if (rc) return rc;
    if (profile) OASES_HIP(hipEventRecord(H->prof[pass][2 * i + 1], R.st[op.stream]));
    if (!serial && op.record >= 0) OASES_HIP(hipEventRecord(H->events[op.record], R.st[op.stream]));
    i++;
  }
  if (profile) H->prof_ran[pass] = true;
  return 0;
}

}  // namespace oases

// =================================================================================================
extern "C" {

const char* oases_last_error(void) { return g_err; }

int oases_create(const oases_layer_cfg* c, oases_handle** out) {
  if (!c || !out) { set_error("oases_create: NULL argument"); return OASES_ENULL; }
  *out = nullptr;
#define BAD(...) do { set_error(__VA_ARGS__); return OASES_EINVAL; } while (0)
  if (c->hidden <= 0 || c->n_heads <= 0 || c->seq <= 0 || c->batch <= 0) BAD("hidden, n_heads, seq, batch must be positive");
  if (c->tp_degree <= 0 || c->tp_rank < 0 || c->tp_rank >= c->tp_degree) BAD("tp_rank %d outside [0, %d)", c->tp_rank, c->tp_degree);
  if (c->n_sub <= 0 || c->n_layers <= 0) BAD("n_sub and n_layers must be >= 1");
  if (c->hidden % c->n_heads) BAD("hidden %d not divisible by n_heads %d", c->hidden, c->n_heads);
  const int d = c->hidden / c->n_heads;
  if (d != 64 && d != 128) BAD("head dimension %d unsupported (64 or 128)", d);
  if (c->n_heads % c->tp_degree) BAD("n_heads %d not divisible by tp_degree %d", c->n_heads, c->tp_degree);
  if (c->arch != OASES_ARCH_GPT && c->arch != OASES_ARCH_LLAMA && c->arch != OASES_ARCH_BERT) BAD("unknown arch %d", c->arch);
  const bool llama = c->arch == OASES_ARCH_LLAMA;
  if (!llama && c->ffn_hidden != 0 && c->ffn_hidden != 4 * c->hidden) BAD("the GPT layer has FFN width 4h (ffn_hidden = 0)");
  const int F = c->ffn_hidden > 0 ? c->ffn_hidden : 4 * c->hidden;
  if (F % c->tp_degree) BAD("FFN width %d not divisible by tp_degree %d", F, c->tp_degree);
  if (llama && (F / c->tp_degree) % 32) BAD("SwiGLU: FFN columns per rank %d must be a multiple of 32", F / c->tp_degree);
  if (!llama && (F / c->tp_degree) % 8) BAD("FFN columns per rank %d must be a multiple of 8", F / c->tp_degree);
  if (c->rope_theta != 0.f && !(c->rope_theta > 1.f)) BAD("rope_theta %g must exceed 1", (double)c->rope_theta);
  if (c->hidden > 16384) BAD("hidden %d too large (max 16384)", c->hidden);
  if (!(c->dropout_p >= 0.f && c->dropout_p < 1.f)) BAD("dropout_p %g outside [0,1)", (double)c->dropout_p);
  if (c->ln_eps < 0.f) BAD("ln_eps negative");
  if (!(c->attn_dropout_p >= 0.f && c->attn_dropout_p < 1.f)) BAD("attn_dropout_p %g outside [0,1)", (double)c->attn_dropout_p);
  const long M = (long)c->batch * c->seq;
  if (M > (1l << 30)) BAD("too many tokens");
  if (M % c->n_sub) BAD("tokens %ld not divisible by n_sub %d", M, c->n_sub);
  const long Ms = M / c->n_sub;
  if (Ms % 8) BAD("rows per sub-batch %ld must be a multiple of 8", Ms);
  if (c->n_sub <= c->batch) {
    if (c->batch % c->n_sub) BAD("batch %d not divisible by n_sub %d", c->batch, c->n_sub);
  } else {
    if (c->n_sub % c->batch || c->seq % (c->n_sub / c->batch)) BAD("n_sub %d does not split %d sequences of %d evenly", c->n_sub, c->batch, c->seq);
    if (!c->causal) BAD("sub-batches that are chunks of a sequence need causal attention");
  }
#undef BAD
  oases_handle* H = new (std::nothrow) oases_handle();
  if (!H) { set_error("out of host memory"); return OASES_EINVAL; }
  H->cfg = *c;
  H->h = c->hidden; H->nh = c->n_heads; H->d = d; H->s = c->seq; H->b = c->batch; H->t = c->tp_degree; H->r = c->tp_rank;
  H->n = c->n_sub; H->L = c->n_layers; H->M = (int)M; H->Ms = (int)Ms;
  H->hp = c->hidden / c->tp_degree; H->fp = F / c->tp_degree; H->heads_l = c->n_heads / c->tp_degree;
  H->llama = llama;
  H->bert = c->arch == OASES_ARCH_BERT;
  H->fw = llama ? 2 * H->fp : H->fp;
  H->eps = c->ln_eps > 0.f ? c->ln_eps : 1e-5f;
  H->theta = c->rope_theta > 0.f ? c->rope_theta : 10000.f;
  H->n_events = H->L * 4 * H->n * 2 + 1;  // + the fork event that orders stream_comm behind stream_compute
  if (!plan_workspace(H)) { delete H; set_error("oases_create: internal error (workspace plan)"); return OASES_EINVAL; }
  build_forward(H);
  build_backward(H);
  *out = H;
  return 0;
}

void oases_destroy(oases_handle* H) {
  if (!H) return;
  for (auto& e : H->events) (void)hipEventDestroy(e);
  for (auto& v : H->prof)
    for (auto& e : v) (void)hipEventDestroy(e);
  delete H;
}

size_t oases_workspace_bytes(const oases_handle* H) { return H ? H->total_bytes : 0; }

int oases_workspace_tensor(const oases_handle* H, const char* name, int layer, size_t* offset, size_t* bytes) {
  if (!H || !name || !offset || !bytes) { set_error("oases_workspace_tensor: NULL argument"); return OASES_ENULL; }
  if (layer < 0 || layer >= H->L) { set_error("layer %d out of range", layer); return OASES_EINVAL; }
  for (auto& t : H->tensors)
    if (!strcmp(t.name, name)) {
      *offset = tensor_off(H, name, layer);
      *bytes = t.bytes;
      return 0;
    }
  set_error("unknown workspace tensor '%s'", name);
  return OASES_EINVAL;
}

int oases_profile_read(oases_handle* H, int backward, float* ms, int n) {
  if (!H || (n > 0 && !ms)) { set_error("oases_profile_read: NULL argument"); return OASES_ENULL; }
  const int pass = backward ? 1 : 0;
  const std::vector<Op>& ops = pass ? H->bwd : H->fwd;
  if (!(H->cfg.flags & OASES_FLAG_PROFILE) || !H->prof_ran[pass]) {
    set_error("oases_profile_read: handle not created with OASES_FLAG_PROFILE, or the pass has not run");
    return OASES_EINVAL;
  }
  for (size_t i = 0; i < ops.size() && (int)i < n; i++) {
    OASES_HIP(hipEventSynchronize(H->prof[pass][2 * i + 1]));
    OASES_HIP(hipEventElapsedTime(&ms[i], H->prof[pass][2 * i], H->prof[pass][2 * i + 1]));
  }
  return (int)ops.size();
}

int oases_schedule_dump(const oases_handle* H, int backward, char* buf, size_t n) {
  if (!H) { set_error("oases_schedule_dump: NULL handle"); return OASES_ENULL; }
  std::string s;
  char line[96];
  for (const Op& op : backward ? H->bwd : H->fwd) {
    const char* name = op_name(op.kind, H->llama, H->bert);
    if (op.sub < 0) snprintf(line, sizeof line, "%s %s L%d sb*\n", op.stream ? "comm" : "compute", name, op.layer);
    else snprintf(line, sizeof line, "%s %s L%d sb%d\n", op.stream ? "comm" : "compute", name, op.layer, op.sub);
    s += line;
  }
  if (buf && n) {
    size_t k = s.size() < n - 1 ? s.size() : n - 1;
    memcpy(buf, s.data(), k);
    buf[k] = 0;
  }
  return (int)s.size();
}

static int check_weights(const oases_handle* H, const oases_weights* w) {
  for (int l = 0; l < H->L; l++) {
    const void* p[] = {w[l].ln1_g, w[l].wqkv, w[l].wo, w[l].ln2_g, w[l].w1, w[l].w2, w[l].ln1_b, w[l].bqkv, w[l].bo, w[l].ln2_b, w[l].b1, w[l].b2};
    int rc = check_ptrs(p, H->llama ? 6 : 12, "weights");  // the LLaMA-style layer has no biases and no LayerNorm shifts
    if (rc) return rc;
  }
  return 0;
}

static int check_workspace(const oases_handle* H, size_t bytes, const char* who) {
  if (bytes >= H->total_bytes) return 0;
  set_error("%s: workspace of %zu bytes is smaller than the %zu bytes oases_workspace_bytes() asks for", who, bytes, H->total_bytes);
  return OASES_EWORKSPACE;
}

int oases_forward(oases_handle* H, const oases_weights* w, const void* x, void* y, const oases_peer_sums* peers,
                  void* workspace, size_t workspace_bytes, void* stream_compute, void* stream_comm) {
  if (!H || !w) { set_error("oases_forward: NULL handle or weights"); return OASES_ENULL; }
  const void* p[] = {x, y, workspace};
  int rc = check_ptrs(p, 3, "oases_forward");
  if (rc) return rc;
  if (x == y) { set_error("oases_forward: y may not alias x"); return OASES_EINVAL; }
  if ((rc = check_workspace(H, workspace_bytes, "oases_forward"))) return rc;
  if ((rc = check_weights(H, w))) return rc;
  Run R{H, w, nullptr, peers, (char*)workspace, (const float*)x, (float*)y, nullptr, nullptr,
        {(hipStream_t)stream_compute, (hipStream_t)stream_comm}};
  return run_ops(R, H->fwd);
}

int oases_backward(oases_handle* H, const oases_weights* w, const void* x, const void* dy, void* dx, const oases_grads* g,
                   const oases_peer_sums* peers, void* workspace, size_t workspace_bytes, void* stream_compute, void* stream_comm) {
  if (!H || !w || !g) { set_error("oases_backward: NULL handle, weights or grads"); return OASES_ENULL; }
  const void* p[] = {x, dy, dx, workspace};
  int rc = check_ptrs(p, 4, "oases_backward");
  if (rc) return rc;
  if ((rc = check_workspace(H, workspace_bytes, "oases_backward"))) return rc;
  if ((rc = check_weights(H, w))) return rc;
  for (int l = 0; l < H->L; l++) {
    const void* q[] = {g[l].ln1_g, g[l].wqkv, g[l].wo, g[l].ln2_g, g[l].w1, g[l].w2, g[l].ln1_b, g[l].bqkv, g[l].bo, g[l].ln2_b, g[l].b1, g[l].b2};
    if ((rc = check_ptrs(q, H->llama ? 6 : 12, "grads"))) return rc;
  }
  Run R{H, w, g, peers, (char*)workspace, (const float*)x, nullptr, (const float*)dy, (float*)dx,
        {(hipStream_t)stream_compute, (hipStream_t)stream_comm}};
  std::vector<ColsumJob> jobs((size_t)H->L * 12);  // at most 11 output arrays of column reductions per layer
  int n_jobs = 0;
  R.defer_colsums = true;
  R.jobs = &jobs;
  R.n_jobs = &n_jobs;
  return run_ops(R, H->bwd);
}

// ---------------------------------------------------------------------------------------------
// segment-level calls: one computation sequence of one layer, all sub-batches, up to its reduction point
// ---------------------------------------------------------------------------------------------
namespace oases {
// which segment of its layer an operator of the schedule belongs to (forward: 0 attention block up to R1, 1 FFN block
// from R1 up to R2, 2 from R2 on; backward: 2 the top layer's dropout backward, 1 FFN block up to R3, 0 attention block
// from R3 up to R4, 3 from R4 on), or -1
static int segment_of(int kind, bool backward) {
  if (!backward) {
    switch (kind) {
      case F_ROPE_TABLE: case F_LN1: case F_QKV: case F_ROPE: case F_ATTN: case F_PROJ: return 0;
      case F_R1: case F_FC1: case F_FC2: return 1;
      case F_R2: return 2;
      default: return -1;
    }
  }
  switch (kind) {
    case B_BDR2: return 2;
    case R_LN2: case R_FC1: case B_FC2_DGRAD: case B_FC1_DGRAD: case B_FC2_WGRAD: case B_FC1_WGRAD: case B_B1_SUM: return 1;
    case B_R3: case R_LN1: case R_QKV: case R_ROPE: case R_ATTN: case B_PROJ_DGRAD: case B_ATTN: case B_ROPE: case B_QKV_DGRAD:
    case B_PROJ_WGRAD: case B_QKV_WGRAD: case B_PQ_WGRAD: case B_BQKV_SUM: return 0;
    case B_R4: return 3;
    default: return -1;
  }
}

// the operators of (layer, segment) in schedule order on one stream: that order is a valid serial order of the pass
// (it is what OASES_FLAG_SERIALISE runs), and every operator of a segment depends only on operators of the same segment
// before it and on earlier segments
static int run_segment(Run& R, bool backward, int layer, int segment, void* partial_out, const void* reduced_in) {
  oases_handle* H = R.H;
  if (layer < 0 || layer >= H->L) { set_error("segment call: layer %d out of range", layer); return OASES_EINVAL; }
  if (segment < 0 || segment > (backward ? 3 : 2)) { set_error("segment call: segment %d out of range", segment); return OASES_EINVAL; }
  if (backward && segment == 2 && layer != H->L - 1) {
    set_error("backward segment 2 exists in the top layer only (below it the dropout backward belongs to segment 3 of the layer above)");
    return OASES_EINVAL;
  }
  // reduction point that the segment ends in (its partial) and the one it starts from (the reduced tensor)
  const int produces = backward ? (segment == 1 ? 2 : segment == 0 ? 3 : -1) : (segment == 0 ? 0 : segment == 1 ? 1 : -1);
  const int consumes = backward ? (segment == 0 ? 2 : segment == 3 ? 3 : -1) : (segment == 1 ? 0 : segment == 2 ? 1 : -1);
  if (partial_out && produces < 0) { set_error("segment call: this segment ends in no reduction point (partial_out must be NULL)"); return OASES_EINVAL; }
  if (reduced_in && consumes < 0) { set_error("segment call: this segment starts from no reduction point (reduced_in must be NULL)"); return OASES_EINVAL; }
  if ((partial_out && !aligned16(partial_out)) || (reduced_in && !aligned16(reduced_in))) { set_error("segment call: pointer not 16-byte aligned"); return OASES_EALIGN; }
  if (produces >= 0) R.partial_out[produces] = (float*)partial_out;
  if (consumes >= 0) R.reduced_in[consumes] = (const float*)reduced_in;
  R.st[1] = R.st[0];
  for (const Op& op0 : backward ? H->bwd : H->fwd) {
    if (op0.layer != layer || segment_of(op0.kind, backward) != segment) continue;
    if (op0.kind == F_ROPE_TABLE && layer != 0) continue;
    Op op = op0;
    op.stream = 0;
    const int rc = run_op(R, op);
    if (rc) return rc;
  }
  return 0;
}
}  // namespace oases

int oases_forward_segment(oases_handle* H, int layer, int segment, const oases_weights* w, const void* x, void* y, void* workspace,
                          size_t workspace_bytes, void* partial_out, const void* reduced_in, void* stream) {
  if (!H || !w) { set_error("oases_forward_segment: NULL handle or weights"); return OASES_ENULL; }
  const void* p[] = {x, y, workspace};
  int rc = check_ptrs(p, 3, "oases_forward_segment");
  if (rc) return rc;
  if (x == y) { set_error("oases_forward_segment: y may not alias x"); return OASES_EINVAL; }
  if ((rc = check_workspace(H, workspace_bytes, "oases_forward_segment"))) return rc;
  if ((rc = check_weights(H, w))) return rc;
  Run R{H, w, nullptr, nullptr, (char*)workspace, (const float*)x, (float*)y, nullptr, nullptr, {(hipStream_t)stream, (hipStream_t)stream}};
  return run_segment(R, false, layer, segment, partial_out, reduced_in);
}

int oases_backward_segment(oases_handle* H, int layer, int segment, const oases_weights* w, const void* x, const void* dy, void* dx,
                           const oases_grads* g, void* workspace, size_t workspace_bytes, void* partial_out, const void* reduced_in,
                           void* stream) {
  if (!H || !w || !g) { set_error("oases_backward_segment: NULL handle, weights or grads"); return OASES_ENULL; }
  const void* p[] = {x, dy, dx, workspace};
  int rc = check_ptrs(p, 4, "oases_backward_segment");
  if (rc) return rc;
  if ((rc = check_workspace(H, workspace_bytes, "oases_backward_segment"))) return rc;
  if ((rc = check_weights(H, w))) return rc;
  for (int l = 0; l < H->L; l++) {
    const void* q[] = {g[l].ln1_g, g[l].wqkv, g[l].wo, g[l].ln2_g, g[l].w1, g[l].w2, g[l].ln1_b, g[l].bqkv, g[l].bo, g[l].ln2_b, g[l].b1, g[l].b2};
    if ((rc = check_ptrs(q, H->llama ? 6 : 12, "grads"))) return rc;
  }
  Run R{H, w, g, nullptr, (char*)workspace, (const float*)x, nullptr, (const float*)dy, (float*)dx, {(hipStream_t)stream, (hipStream_t)stream}};
  return run_segment(R, true, layer, segment, partial_out, reduced_in);
}

// ---------------------------------------------------------------------------------------------
// single operators
// ---------------------------------------------------------------------------------------------
int oases_op_dropout_mask(uint8_t* mask, uint64_t seed, int layer, int site, int64_t row0, int rows, int h, float p, void* stream) {
  return launch_dropout_mask(mask, make_drop_cfg(seed, layer, site, p), row0, rows, h, (hipStream_t)stream);
}
int oases_op_layernorm_fwd(const void* x, const void* gamma, const void* beta, void* out, void* mu, void* rstd, int rows, int h,
                           float eps, void* stream) {
  return launch_layernorm_fwd((const float*)x, (const float*)gamma, (const float*)beta, out, (float*)mu, (float*)rstd, rows, h, eps,
                              (hipStream_t)stream);
}
int oases_op_bias_dropout_residual_ln(const void* part, const void* peer, const void* bias, const void* xin, void* xo,
                                      const void* gamma, const void* beta, void* ln_out, void* mu, void* rstd, int rows, int h,
                                      float eps, uint64_t seed, int layer, int site, int64_t row0, float p, void* stream) {
  if (!part) { set_error("bias_dropout_residual_ln: NULL partial"); return OASES_ENULL; }
  return launch_bdr_ln((const float*)part, (const float*)peer, (const float*)bias, (const float*)xin, (float*)xo, (const float*)gamma,
                       (const float*)beta, ln_out, (float*)mu, (float*)rstd, rows, h, eps, make_drop_cfg(seed, layer, site, p), row0,
                       (hipStream_t)stream);
}
int oases_op_dropout_bwd(const void* dyin, void* dz, void* dbias, int rows, int h, uint64_t seed, int layer, int site, int64_t row0,
                         float p, void* scratch, void* stream) {
  return launch_dropout_bwd((const float*)dyin, dz, (float*)dbias, rows, h, make_drop_cfg(seed, layer, site, p), row0, (float*)scratch,
                            (hipStream_t)stream);
}
int oases_op_layernorm_bwd(const void* part, const void* peer, const void* dres, const void* x, const void* mu, const void* rstd,
                           const void* gamma, void* dxo, void* dgamma, void* dbeta, void* dz, void* dbias, int rows, int h,
                           uint64_t seed, int layer, int site, int64_t row0, float p, void* scratch, void* stream) {
  return launch_layernorm_bwd((const float*)part, (const float*)peer, (const float*)dres, (const float*)x, (const float*)mu,
                              (const float*)rstd, (const float*)gamma, (float*)dxo, (float*)dgamma, (float*)dbeta, dz, (float*)dbias,
                              rows, h, make_drop_cfg(seed, layer, site, p), row0, (float*)scratch, (hipStream_t)stream);
}
int oases_op_rmsnorm_fwd(const void* x, const void* gamma, void* out, void* rstd, int rows, int h, float eps, void* stream) {
  return launch_layernorm_fwd((const float*)x, (const float*)gamma, nullptr, out, nullptr, (float*)rstd, rows, h, eps, (hipStream_t)stream,
                              true);
}
int oases_op_dropout_residual_rmsnorm(const void* part, const void* peer, const void* xin, void* xo, const void* gamma, void* ln_out,
                                      void* rstd, int rows, int h, float eps, uint64_t seed, int layer, int site, int64_t row0, float p,
                                      void* stream) {
  if (!part) { set_error("dropout_residual_rmsnorm: NULL partial"); return OASES_ENULL; }
  return launch_bdr_ln((const float*)part, (const float*)peer, nullptr, (const float*)xin, (float*)xo, (const float*)gamma, nullptr, ln_out,
                       nullptr, (float*)rstd, rows, h, eps, make_drop_cfg(seed, layer, site, p), row0, (hipStream_t)stream, true);
}
int oases_op_rmsnorm_bwd(const void* part, const void* peer, const void* dres, const void* x, const void* rstd, const void* gamma,
                         void* dxo, void* dgamma, void* dz, int rows, int h, uint64_t seed, int layer, int site, int64_t row0, float p,
                         void* scratch, void* stream) {
  return launch_layernorm_bwd((const float*)part, (const float*)peer, (const float*)dres, (const float*)x, nullptr, (const float*)rstd,
                              (const float*)gamma, (float*)dxo, (float*)dgamma, nullptr, dz, nullptr, rows, h,
                              make_drop_cfg(seed, layer, site, p), row0, (float*)scratch, (hipStream_t)stream, true);
}
int oases_op_rope_table(void* table, int seq, int head_dim, float theta, void* stream) {
  return launch_rope_table((float*)table, seq, head_dim, theta, (hipStream_t)stream);
}
int oases_op_rope(void* qkv, int ld, int rows, int64_t row0, int seq, int heads, int head_dim, const void* table, int inverse,
                  void* stream) {
  return launch_rope(qkv, ld, rows, row0, seq, heads, head_dim, (const float*)table, inverse, (hipStream_t)stream);
}
int oases_op_gemm(int op, int epi, int M, int N, int K, const void* A, int lda, const void* B, int ldb, void* C, int ldc,
                  const void* bias, void* aux, int ldaux, void* workspace, size_t workspace_bytes, void* stream) {
  if (workspace && !aligned16(workspace)) { set_error("gemm: workspace not 16-byte aligned"); return OASES_EALIGN; }
  return launch_gemm(op, epi, M, N, K, A, lda, B, ldb, C, ldc, (const float*)bias, aux, ldaux, workspace, workspace ? workspace_bytes : 0,
                     0, (hipStream_t)stream);
}
int oases_op_gemm_forced(int variant, int op, int epi, int M, int N, int K, const void* A, int lda, const void* B, int ldb, void* C,
                         int ldc, const void* bias, void* aux, int ldaux, void* workspace, size_t workspace_bytes, void* stream) {
  if (workspace && !aligned16(workspace)) { set_error("gemm: workspace not 16-byte aligned"); return OASES_EALIGN; }
  if (variant <= 0) { set_error("gemm: variant must be positive"); return OASES_EINVAL; }
  return launch_gemm(op, epi, M, N, K, A, lda, B, ldb, C, ldc, (const float*)bias, aux, ldaux, workspace, workspace ? workspace_bytes : 0,
                     variant, (hipStream_t)stream);
}
int oases_op_gemm_variant(int op, int epi, int M, int N, int K, size_t workspace_bytes) {
  (void)epi;
  if (op < 0 || op > 2 || M <= 0 || N <= 0 || K <= 0) { set_error("oases_op_gemm_variant: bad argument"); return OASES_EINVAL; }
  return gemm_variant(op, epi, M, N, K, workspace_bytes);
}
int oases_op_gemm_tn_pair(int K, int M0, int N0, const void* A0, int lda0, const void* B0, int ldb0, void* C0, int ldc0, int M1, int N1,
                          const void* A1, int lda1, const void* B1, int ldb1, void* C1, int ldc1, void* stream) {
  return launch_gemm_tn_pair(K, M0, N0, A0, lda0, B0, ldb0, C0, ldc0, M1, N1, A1, lda1, B1, ldb1, C1, ldc1, (hipStream_t)stream);
}
int oases_op_gemm_tn_pair_wins(int K, int M0, int N0, int M1, int N1) { return gemm_tn_pair_wins(K, M0, N0, M1, N1) ? 1 : 0; }
size_t oases_gemm_workspace_bytes(const oases_handle* H) { return H ? H->gemm_ws_bytes : 0; }
int oases_op_colsum_bf16(const void* a, int ld, int rows, int cols, void* out, void* scratch, void* stream) {
  return launch_colsum_bf16(a, ld, rows, cols, (float*)out, (float*)scratch, (hipStream_t)stream);
}
int oases_op_attention_fwd(const void* qkv, void* out, void* lse, int batch, int seq, int heads, int head_dim, int causal, int row0,
                           int rows, void* stream) {
  return launch_attention_fwd(qkv, out, (float*)lse, batch, seq, heads, head_dim, causal, row0, rows, (hipStream_t)stream);
}
int oases_op_attention_dropout_fwd(const void* qkv, void* out, void* lse, int batch, int seq, int heads, int head_dim, int causal,
                                   int row0, int rows, uint64_t seed, int layer, float p, int head0, int heads_total, void* stream) {
  return launch_attention_fwd(qkv, out, (float*)lse, batch, seq, heads, head_dim, causal, row0, rows, (hipStream_t)stream, seed, layer, p,
                              head0, heads_total);
}
int oases_op_attention_dropout_bwd(const void* qkv, const void* out, const void* dout, const void* lse, void* delta, void* dqkv,
                                   int batch, int seq, int heads, int head_dim, int causal, int row0, int rows, uint64_t seed, int layer,
                                   float p, int head0, int heads_total, void* stream) {
  return launch_attention_bwd(qkv, out, dout, (const float*)lse, (float*)delta, dqkv, batch, seq, heads, head_dim, causal, row0, rows,
                              (hipStream_t)stream, seed, layer, p, head0, heads_total);
}
int oases_op_attention_bwd(const void* qkv, const void* out, const void* dout, const void* lse, void* delta, void* dqkv, int batch,
                           int seq, int heads, int head_dim, int causal, int row0, int rows, void* stream) {
  return launch_attention_bwd(qkv, out, dout, (const float*)lse, (float*)delta, dqkv, batch, seq, heads, head_dim, causal, row0, rows,
                              (hipStream_t)stream);
}

}  // extern "C"
