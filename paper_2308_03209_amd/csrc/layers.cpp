// Composition of one GNN layer, forward and backward, from the aggregation and dense kernels
// (layer definition of Section 3; gradient flow as in the proof of Theorem 3).
#include <cstdlib>
#include <mutex>

#include "common.h"

namespace cofree {

// ---- a second stream for work that does not depend on the aggregation chain -------------------
// In backward the weight gradients that only need the incoming gradient (compute bound) are
// independent of the transposed aggregation (memory bound); with COFREE_OVERLAP=1 in the environment
// they are enqueued on a library-owned stream between a fork event (recorded on the caller's stream)
// and a join event (waited on by the caller's stream before the call returns control of the
// outputs), so the two overlap.  Default priority, created once per device.  Off by default: both
// kernels are bound inside the compute unit and mostly take turns on it, so the step gains 0-3 %
// while every kernel's own duration, as events see it, grows by up to half.
struct SideStream {
  hipStream_t stream = nullptr;
  hipEvent_t fork = nullptr, join = nullptr;
  bool ok = false;
};

static SideStream* side_stream() {
  static std::mutex mu;
  static SideStream per_device[64];
  static bool tried[64];
  const char* env = getenv("COFREE_OVERLAP");
  if (!env || atoi(env) == 0) return nullptr;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  std::lock_guard<std::mutex> lk(mu);
  SideStream& s = per_device[dev];
  if (!tried[dev]) {
    tried[dev] = true;
    s.ok = hipStreamCreateWithFlags(&s.stream, hipStreamNonBlocking) == hipSuccess &&
           hipEventCreateWithFlags(&s.fork, hipEventDisableTiming) == hipSuccess &&
           hipEventCreateWithFlags(&s.join, hipEventDisableTiming) == hipSuccess;
  }
  return s.ok ? &s : nullptr;
}

// Returns the stream to use for the independent work: the side stream (after it has been made to
// wait for everything enqueued on `main` so far), or `main` itself if overlap is unavailable.
static hipStream_t fork_side(hipStream_t main, SideStream** used) {
  *used = nullptr;
  SideStream* s = side_stream();
  if (!s) return main;
  if (hipEventRecord(s->fork, main) != hipSuccess) return main;
  if (hipStreamWaitEvent(s->stream, s->fork, 0) != hipSuccess) return main;
  *used = s;
  return s->stream;
}

static int32_t join_side(hipStream_t main, SideStream* s) {
  if (!s) return COFREE_OK;
  COFREE_HIP_CHECK(hipEventRecord(s->join, s->stream));
  COFREE_HIP_CHECK(hipStreamWaitEvent(main, s->join, 0));
  return COFREE_OK;
}

// Joins the side stream back into the caller's stream when the call leaves, also on an error path.
struct SideJoin {
  hipStream_t main;
  SideStream* side;
  ~SideJoin() { (void)join_side(main, side); }
  int32_t finish() {
    SideStream* s = side;
    side = nullptr;
    return join_side(main, s);
  }
};

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
static inline size_t elem_size(int32_t dtype) { return dtype == COFREE_BF16 ? 2 : 4; }

// Carves 256-byte aligned buffers out of the caller's workspace.
struct Carver {
  char* base;
  size_t used = 0;
  explicit Carver(void* p) : base((char*)p) {}
  void* take(size_t bytes) {
    void* r = base ? (void*)(base + used) : nullptr;
    used += align256(bytes);
    return r;
  }
};

static bool gcn_transform_first(const cofree_layer_desc& d) { return d.d_out < d.d_in; }
// Conventional GraphSAGE: the mean commutes with W_neigh, so it runs on min(d_in, d_out) columns.
static bool conv_transform_first(const cofree_layer_desc& d) { return d.d_out < d.d_in; }
// The neighbourhood mean commutes with the linear map U_a, so when the layer output is narrower
// than the messages the mean is taken after U_a (on d_out columns instead of d_msg).
static bool sage_combine_first(const cofree_layer_desc& d) { return d.d_out < d.d_msg; }

static size_t max2(size_t a, size_t b) { return a > b ? a : b; }
static size_t max3(size_t a, size_t b, size_t c) { return max2(a, max2(b, c)); }

// largest bf16 copy of a parameter matrix any product of the layer needs
static size_t param_scratch_bytes(const cofree_layer_desc& d) {
  if (d.dtype != COFREE_BF16) return 0;
  if (d.kind == COFREE_SAGE_MEAN)
    return max3(gemm_param_scratch_bytes(d.d_msg, d.d_in),
                gemm_param_scratch_bytes(d.d_out, (int64_t)d.d_msg + d.d_in),
                max2(gemm_param_scratch_bytes(d.d_msg, d.d_out),
                     gemm_param_scratch_bytes(d.d_in, (int64_t)d.d_out + d.d_msg)));
  if (d.kind == COFREE_SAGE_CONV)
    return max2(gemm_param_scratch_bytes(d.d_out, 2 * (int64_t)d.d_in),
                gemm_param_scratch_bytes(d.d_in, 2 * (int64_t)d.d_out));
  return max2(gemm_param_scratch_bytes(d.d_out, d.d_in), gemm_param_scratch_bytes(d.d_in, d.d_out));
}

struct FwdPlan {
  void* T = nullptr;       // transform-first: norm * (H W^T) (GCN), H W_neigh^T (conventional GraphSAGE)
  void* params = nullptr;  // bf16 copy of a parameter matrix
  size_t bytes = 0;
};

static FwdPlan plan_fwd(const cofree_layer_desc& d, int64_t n, void* ws) {
  Carver c(ws);
  FwdPlan p;
  if ((d.kind == COFREE_GCN && gcn_transform_first(d)) || (d.kind == COFREE_SAGE_CONV && conv_transform_first(d)))
    p.T = c.take((size_t)n * d.d_out * elem_size(d.dtype));
  if (d.dtype == COFREE_BF16) p.params = c.take(param_scratch_bytes(d));
  p.bytes = c.used;
  return p;
}

struct BwdPlan {
  void *dP = nullptr, *dA = nullptr, *dZ = nullptr, *T = nullptr, *params = nullptr;
  float *wg = nullptr, *cs = nullptr;    // split-k / column-sum partials of the caller's stream
  float *wg2 = nullptr, *cs2 = nullptr;  // the same for the work on the side stream
  size_t bytes = 0;
};

static BwdPlan plan_bwd(const cofree_layer_desc& d, int64_t n, void* ws) {
  Carver c(ws);
  BwdPlan p;
  const size_t N = (size_t)n, es = elem_size(d.dtype);
  if (d.kind == COFREE_SAGE_MEAN) {
    if (d.dropout_q > 0.f) p.dP = c.take(N * d.d_out * es);
    p.dA = c.take(N * d.d_msg * es);
    p.dZ = c.take(N * d.d_msg * es);
    const size_t wg_bytes = 4 * max3(wgrad_workspace_floats(d.d_out, d.d_msg + d.d_in, n),
                                     max2(wgrad_workspace_floats(d.d_out, d.d_msg, n),
                                          wgrad_workspace_floats(d.d_out, d.d_in, n)),
                                     wgrad_workspace_floats(d.d_msg, d.d_in, n));
    const size_t cs_bytes = 4 * colsum_workspace_floats(d.d_out > d.d_msg ? d.d_out : d.d_msg);
    p.wg = (float*)c.take(wg_bytes);
    p.cs = (float*)c.take(cs_bytes);
    p.wg2 = (float*)c.take(wg_bytes);
    p.cs2 = (float*)c.take(cs_bytes);
  } else {
    if (d.dropout_q > 0.f || d.act) p.dP = c.take(N * d.d_out * es);
    // transform first: T = Ahat dPre [n, d_out]; aggregate first: T = norm * (dPre W) [n, d_in]
    p.T = c.take(N * (gcn_transform_first(d) ? d.d_out : d.d_in) * es);
    const int32_t wg_cols = d.kind == COFREE_SAGE_CONV ? 2 * d.d_in : d.d_in;  // both halves of W in one launch
    p.wg = (float*)c.take(4 * wgrad_workspace_floats(d.d_out, d.d_in, n));
    p.cs = (float*)c.take(4 * colsum_workspace_floats(d.d_out));
    p.wg2 = (float*)c.take(4 * max2(wgrad_workspace_floats(d.d_out, d.d_in, n),
                                    wgrad_workspace_floats(d.d_out, wg_cols, n)));
    p.cs2 = (float*)c.take(4 * colsum_workspace_floats(d.d_out));
  }
  if (d.dtype == COFREE_BF16) p.params = c.take(param_scratch_bytes(d));
  p.bytes = c.used;
  return p;
}

static int32_t check_desc(const cofree_layer_desc* d) {
  COFREE_REQUIRE(d != nullptr, "layer: desc is NULL");
  COFREE_REQUIRE(d->kind == COFREE_GCN || d->kind == COFREE_SAGE_MEAN || d->kind == COFREE_SAGE_CONV,
                 "layer: unknown kind");
  COFREE_REQUIRE(d->dtype == COFREE_F32 || d->dtype == COFREE_BF16, "layer: unknown dtype");
  COFREE_REQUIRE(d->d_in >= 1 && d->d_out >= 1, "layer: d_in and d_out must be >= 1");
  COFREE_REQUIRE(d->kind != COFREE_SAGE_MEAN || d->d_msg >= 1, "layer: d_msg must be >= 1");
  COFREE_REQUIRE(d->dropout_q >= 0.f && d->dropout_q < 1.f, "layer: dropout_q must be in [0, 1)");
  COFREE_REQUIRE(d->layer_id >= 0 && d->layer_id < (1 << 23), "layer: layer_id out of range");
  COFREE_REQUIRE((d->grad_flags & ~(COFREE_GRAD_IN_GATED | COFREE_GRAD_OUT_GATED)) == 0, "layer: unknown grad_flags");
  COFREE_REQUIRE(d->dropout_q_below >= 0.f && d->dropout_q_below < 1.f, "layer: dropout_q_below must be in [0, 1)");
  COFREE_REQUIRE(!(d->grad_flags & COFREE_GRAD_IN_GATED) || d->kind != COFREE_SAGE_MEAN,
                 "layer: COFREE_GRAD_IN_GATED is for GCN and SAGE_CONV layers");
  COFREE_REQUIRE(!(d->grad_flags & COFREE_GRAD_OUT_GATED) || (d->kind != COFREE_SAGE_MEAN && d->act),
                 "layer: COFREE_GRAD_OUT_GATED needs a layer that ends in ReLU");
  return COFREE_OK;
}

static DropoutArgs dropout_of(const cofree_layer_desc& d) {
  DropoutArgs o;
  o.q = d.dropout_q;
  o.seed = d.seed;
  o.epoch = (uint32_t)d.epoch;
  o.layer_id = (uint32_t)d.layer_id;
  return o;
}

}  // namespace cofree

using namespace cofree;

extern "C" {

size_t cofree_layer_desc_size(void) { return sizeof(cofree_layer_desc); }

size_t cofree_layer_workspace_bytes(const cofree_layer_desc* desc, int64_t n_nodes, int32_t backward) {
  if (!desc || n_nodes < 0) return 0;
  const size_t b = backward ? plan_bwd(*desc, n_nodes, nullptr).bytes : plan_fwd(*desc, n_nodes, nullptr).bytes;
  return b < 256 ? 256 : b;
}

int32_t cofree_layer_fwd(const cofree_partition* part, const cofree_masks* masks, int32_t mask_id,
                         const cofree_layer_desc* desc, const void* H_in, const cofree_layer_params* params,
                         void* H_out, const cofree_layer_saved* saved, void* workspace, size_t workspace_bytes,
                         void* stream) {
  COFREE_TRY(check_desc(desc));
  const cofree_layer_desc& d = *desc;
  DeviceGraph g;
  COFREE_TRY(select_graph(part, masks, mask_id, &g));
  COFREE_REQUIRE(H_in && H_out && params && saved, "layer_fwd: NULL argument");
  COFREE_REQUIRE(params->W && params->bW, "layer_fwd: W / bW is NULL");
  const FwdPlan fp = plan_fwd(d, g.n, workspace);
  if (fp.bytes > 0 && (workspace == nullptr || workspace_bytes < fp.bytes))
    return fail(COFREE_ENOMEM, "layer_fwd: workspace too small");
  hipStream_t s = (hipStream_t)stream;
  const int64_t n = g.n;
  const int32_t dt = d.dtype;
  auto gemm = [&]() {
    GemmArgs a;
    a.dtype = dt;
    a.param_scratch = fp.params;
    a.M = n;
    return a;
  };
  auto agg = [&]() {
    AggArgs a;
    a.g = g;
    a.dtype = dt;
    return a;
  };

  if (d.kind == COFREE_SAGE_MEAN) {
    COFREE_REQUIRE(params->U && params->bU, "layer_fwd: U / bU is NULL");
    COFREE_REQUIRE(saved->Z && saved->A, "layer_fwd: saved.Z / saved.A is NULL");
    void* Z = saved->Z;
    void* A = saved->A;
    const int64_t ldu = (int64_t)d.d_msg + d.d_in;
    // messages: Z = ReLU(H W^T + bW)
    GemmArgs m = gemm();
    m.A1 = H_in; m.lda1 = d.d_in; m.K1 = d.d_in;
    m.B = params->W; m.ldb = d.d_in;
    m.C = Z; m.ldc = d.d_msg; m.N = d.d_msg;
    m.bias = params->bW; m.relu = 1;
    COFREE_TRY(launch_gemm(m, s));
    if (sage_combine_first(d)) {
      // H' = mean(Z U_a^T) + H U_s^T + bU: T = Z U_a^T is kept in the A buffer
      GemmArgs t = gemm();
      t.A1 = Z; t.lda1 = d.d_msg; t.K1 = d.d_msg;
      t.B = params->U; t.ldb = ldu;
      t.C = A; t.ldc = d.d_out; t.N = d.d_out;
      COFREE_TRY(launch_gemm(t, s));
      AggArgs a = agg();
      a.X = A; a.Y = H_out; a.width = d.d_out; a.ldx = a.ldy = d.d_out;
      a.out_scale = g.inv_deg;
      COFREE_TRY(launch_aggregate(a, s));
      GemmArgs c = gemm();
      c.A1 = H_in; c.lda1 = d.d_in; c.K1 = d.d_in;
      c.B = params->U + d.d_msg; c.ldb = ldu;
      c.C = H_out; c.ldc = d.d_out; c.N = d.d_out;
      c.bias = params->bU; c.accumulate = 1;
      COFREE_TRY(launch_gemm(c, s));
    } else {
      // neighbourhood mean, then combine: H' = [A | H] U^T + bU
      AggArgs a = agg();
      a.X = Z; a.Y = A; a.width = d.d_msg; a.ldx = a.ldy = d.d_msg;
      a.out_scale = g.inv_deg;
      COFREE_TRY(launch_aggregate(a, s));
      GemmArgs c = gemm();
      c.A1 = A; c.lda1 = d.d_msg; c.K1 = d.d_msg;
      c.A2 = H_in; c.lda2 = d.d_in; c.K2 = d.d_in;
      c.B = params->U; c.ldb = ldu;
      c.C = H_out; c.ldc = d.d_out; c.N = d.d_out;
      c.bias = params->bU;
      COFREE_TRY(launch_gemm(c, s));
    }
  } else if (d.kind == COFREE_SAGE_CONV) {
    const int64_t ldw = 2 * (int64_t)d.d_in;  // W = [W_self | W_neigh]
    if (conv_transform_first(d)) {
      // T = H W_neigh^T; H' = mean(T); H' = act(H' + H W_self^T + b)
      GemmArgs t = gemm();
      t.A1 = H_in; t.lda1 = d.d_in; t.K1 = d.d_in;
      t.B = params->W + d.d_in; t.ldb = ldw;
      t.C = fp.T; t.ldc = d.d_out; t.N = d.d_out;
      COFREE_TRY(launch_gemm(t, s));
      AggArgs a = agg();
      a.X = fp.T; a.Y = H_out; a.width = d.d_out; a.ldx = a.ldy = d.d_out;
      a.out_scale = g.inv_deg;
      COFREE_TRY(launch_aggregate(a, s));
      GemmArgs c = gemm();
      c.A1 = H_in; c.lda1 = d.d_in; c.K1 = d.d_in;
      c.B = params->W; c.ldb = ldw;
      c.C = H_out; c.ldc = d.d_out; c.N = d.d_out;
      c.bias = params->bW; c.accumulate = 1; c.relu_last = d.act;
      COFREE_TRY(launch_gemm(c, s));
    } else {
      COFREE_REQUIRE(saved->A, "layer_fwd: saved.A is NULL");
      // M = mean(H), then H' = act([H | M] W^T + b)
      AggArgs a = agg();
      a.X = H_in; a.Y = saved->A; a.width = d.d_in; a.ldx = a.ldy = d.d_in;
      a.out_scale = g.inv_deg;
      COFREE_TRY(launch_aggregate(a, s));
      GemmArgs c = gemm();
      c.A1 = H_in; c.lda1 = d.d_in; c.K1 = d.d_in;
      c.A2 = saved->A; c.lda2 = d.d_in; c.K2 = d.d_in;
      c.B = params->W; c.ldb = ldw;
      c.C = H_out; c.ldc = d.d_out; c.N = d.d_out;
      c.bias = params->bW; c.relu = d.act;
      COFREE_TRY(launch_gemm(c, s));
    }
  } else if (gcn_transform_first(d)) {
    // T = norm * (H W^T), then H' = act(norm * (T[v] + sum T[u]) + b)
    GemmArgs t = gemm();
    t.A1 = H_in; t.lda1 = d.d_in; t.K1 = d.d_in;
    t.B = params->W; t.ldb = d.d_in;
    t.C = fp.T; t.ldc = d.d_out; t.N = d.d_out;
    t.row_scale = g.gcn_norm;
    COFREE_TRY(launch_gemm(t, s));
    AggArgs a = agg();
    a.X = fp.T; a.Y = H_out; a.width = d.d_out; a.ldx = a.ldy = d.d_out;
    a.out_scale = g.gcn_norm; a.self_loop = 1;  // sources are already scaled
    a.bias = params->bW; a.relu_out = d.act;
    COFREE_TRY(launch_aggregate(a, s));
  } else {
    COFREE_REQUIRE(saved->A, "layer_fwd: saved.A is NULL");
    // P = Ahat H, then H' = act(P W^T + b)
    AggArgs a = agg();
    a.X = H_in; a.Y = saved->A; a.width = d.d_in; a.ldx = a.ldy = d.d_in;
    a.in_scale = g.gcn_norm; a.out_scale = g.gcn_norm; a.self_loop = 1;
    COFREE_TRY(launch_aggregate(a, s));
    GemmArgs t = gemm();
    t.A1 = saved->A; t.lda1 = d.d_in; t.K1 = d.d_in;
    t.B = params->W; t.ldb = d.d_in;
    t.C = H_out; t.ldc = d.d_out; t.N = d.d_out;
    t.bias = params->bW; t.relu = d.act;
    COFREE_TRY(launch_gemm(t, s));
  }
  // inverted dropout on the layer output, in place (the same keep decisions are recomputed in backward)
  if (d.dropout_q > 0.f) COFREE_TRY(launch_mask_grad(dt, H_out, nullptr, H_out, n, d.d_out, dropout_of(d), s));
  return COFREE_OK;
}

int32_t cofree_layer_bwd(const cofree_partition* part, const cofree_masks* masks, int32_t mask_id,
                         const cofree_layer_desc* desc, const void* H_in, const void* H_out,
                         const cofree_layer_params* params, const cofree_layer_saved* saved, const void* dH_out,
                         void* dH_in, const cofree_layer_grads* grads, int32_t accumulate, void* workspace,
                         size_t workspace_bytes, void* stream) {
  COFREE_TRY(check_desc(desc));
  const cofree_layer_desc& d = *desc;
  DeviceGraph g;
  COFREE_TRY(select_graph(part, masks, mask_id, &g));
  COFREE_REQUIRE(H_in && H_out && params && saved && dH_out && grads && workspace, "layer_bwd: NULL argument");
  COFREE_REQUIRE(params->W && grads->W && grads->bW, "layer_bwd: W / grads.W / grads.bW is NULL");
  const int64_t n = g.n;
  const BwdPlan p = plan_bwd(d, n, workspace);
  if (workspace_bytes < p.bytes) return fail(COFREE_ENOMEM, "layer_bwd: workspace too small");
  hipStream_t s = (hipStream_t)stream;
  const int32_t dt = d.dtype;
  accumulate = accumulate ? 1 : 0;
  auto gemm = [&]() {
    GemmArgs a;
    a.dtype = dt;
    a.param_scratch = p.params;
    a.M = n;
    return a;
  };
  auto agg = [&]() {
    AggArgs a;
    a.g = g;
    a.dtype = dt;
    return a;
  };

  if (d.kind == COFREE_SAGE_MEAN) {
    COFREE_REQUIRE(params->U && grads->U && grads->bU, "layer_bwd: U / grads.U / grads.bU is NULL");
    COFREE_REQUIRE(saved->Z && saved->A, "layer_bwd: saved.Z / saved.A is NULL");
    const void* Z = saved->Z;
    const void* A = saved->A;
    const int64_t ldu = (int64_t)d.d_msg + d.d_in;
    // gradient at the combine output (undo dropout scaling)
    const void* dP = dH_out;
    if (d.dropout_q > 0.f) {
      COFREE_TRY(launch_mask_grad(dt, dH_out, nullptr, p.dP, n, d.d_out, dropout_of(d), s));
      dP = p.dP;
    }
    // dU_s = dP^T H and dbU = column sums of dP need only dP: side stream
    SideStream* side = nullptr;
    hipStream_t s2 = fork_side(s, &side);
    SideJoin joiner{s, side};
    // dU = dP^T [A | H]: when both blocks are whole numbers of 128-column tiles the two halves are one launch
    // that reads dP once (the products are memory bound in bf16; 256x512 over 1.9M nodes: 0.72 ms against
    // 2 x 0.40); else two launches (with a ragged second block the merged launch measured slower)
    const bool merged_dU = !sage_combine_first(d) && d.d_msg % 128 == 0 && d.d_in % 128 == 0;
    if (merged_dU)
      COFREE_TRY(launch_wgrad(dt, dP, d.d_out, d.d_out, A, d.d_msg, d.d_msg, n, grads->U, ldu, accumulate, p.wg2, s2,
                              grads->bU, H_in, d.d_in, d.d_in));
    else
      COFREE_TRY(launch_wgrad(dt, dP, d.d_out, d.d_out, H_in, d.d_in, d.d_in, n, grads->U + d.d_msg, ldu, accumulate,
                              p.wg2, s2, grads->bU));
    if (sage_combine_first(d)) {
      // forward was mean(Z U_a^T): dT = mean^T(dP) on d_out columns, dU_a = dT^T Z,
      // dZ = [Z > 0] * (dT U_a)
      AggArgs t = agg();
      t.X = dP; t.Y = p.dA; t.width = d.d_out; t.ldx = t.ldy = d.d_out;
      t.in_scale = g.inv_deg;
      COFREE_TRY(launch_aggregate(t, s));
      COFREE_TRY(launch_wgrad(dt, p.dA, d.d_out, d.d_out, Z, d.d_msg, d.d_msg, n, grads->U, ldu, accumulate, p.wg,
                              s));
      GemmArgs z = gemm();
      z.A1 = p.dA; z.lda1 = d.d_out; z.K1 = d.d_out;
      z.B = params->U; z.ldb = ldu; z.b_kmajor = 1;
      z.C = p.dZ; z.ldc = d.d_msg; z.N = d.d_msg;
      z.gate = Z; z.ldg = d.d_msg;
      COFREE_TRY(launch_gemm(z, s));
    } else {
      // dU_a = dP^T A (side stream as well)
      if (!merged_dU)
        COFREE_TRY(launch_wgrad(dt, dP, d.d_out, d.d_out, A, d.d_msg, d.d_msg, n, grads->U, ldu, accumulate, p.wg2, s2));
      // dA / deg = (dP U_a) scaled per destination row, so that the transposed mean is a plain pull
      GemmArgs a = gemm();
      a.A1 = dP; a.lda1 = d.d_out; a.K1 = d.d_out;
      a.B = params->U; a.ldb = ldu; a.b_kmajor = 1;
      a.C = p.dA; a.ldc = d.d_msg; a.N = d.d_msg;
      a.row_scale = g.inv_deg;
      COFREE_TRY(launch_gemm(a, s));
      // dZ[u] = [Z[u] > 0] * sum_{v in N(u)} dA[v] / deg(v)
      AggArgs t = agg();
      t.X = p.dA; t.Y = p.dZ; t.width = d.d_msg; t.ldx = t.ldy = d.d_msg;
      t.relu_src = Z; t.ld_relu = d.d_msg;
      COFREE_TRY(launch_aggregate(t, s));
    }
    // dW = dZ^T H, dbW = column sums of dZ
    COFREE_TRY(launch_wgrad(dt, p.dZ, d.d_msg, d.d_msg, H_in, d.d_in, d.d_in, n, grads->W, d.d_in, accumulate, p.wg,
                            s, grads->bW));
    if (dH_in) {
      // dH = dP U_s + dZ W: one product over the two k-segments [dP | dZ], each with its own parameters
      GemmArgs h = gemm();
      h.A1 = dP; h.lda1 = d.d_out; h.K1 = d.d_out;
      h.B = params->U + d.d_msg; h.ldb = ldu; h.b_kmajor = 1;
      h.A2 = p.dZ; h.lda2 = d.d_msg; h.K2 = d.d_msg;
      h.B2 = params->W; h.ldb2 = d.d_in;
      h.C = dH_in; h.ldc = d.d_in; h.N = d.d_in;
      COFREE_TRY(launch_gemm(h, s));
    }
    return joiner.finish();
  }

  // GCN and conventional GraphSAGE: dPre = dH_out gated by the activation and the dropout mask
  // (nothing to do when the layer above has applied both: COFREE_GRAD_OUT_GATED)
  const bool out_gated = (d.grad_flags & COFREE_GRAD_OUT_GATED) != 0;
  // ReLU / dropout backward of the layer below, carried by the kernel that writes dH_in
  const void* in_gate = (d.grad_flags & COFREE_GRAD_IN_GATED) ? H_in : nullptr;
  const float in_scale = 1.0f / (1.0f - d.dropout_q_below);  // inverted dropout of the layer below
  const void* dPre = dH_out;
  if ((d.dropout_q > 0.f || d.act) && !out_gated) {
    COFREE_TRY(launch_mask_grad(dt, dH_out, d.act ? H_out : nullptr, p.dP, n, d.d_out, dropout_of(d), s));
    dPre = p.dP;
  }
  SideStream* side = nullptr;
  hipStream_t s2 = fork_side(s, &side);
  SideJoin joiner{s, side};
  if (d.kind == COFREE_SAGE_CONV) {
    const int64_t ldw = 2 * (int64_t)d.d_in;
    // dW_self = dPre^T H and db = column sums of dPre need only dPre: side stream.  Aggregate-first layers
    // also have dW_neigh = dPre^T M: one launch for both when d_in is a whole number of 128-column tiles
    const bool merged_dW = !conv_transform_first(d) && d.d_in % 128 == 0;
    if (merged_dW) {
      COFREE_REQUIRE(saved->A, "layer_bwd: saved.A is NULL");
      COFREE_TRY(launch_wgrad(dt, dPre, d.d_out, d.d_out, H_in, d.d_in, d.d_in, n, grads->W, ldw, accumulate, p.wg2, s2,
                              grads->bW, saved->A, d.d_in, d.d_in));
    } else {
      COFREE_TRY(launch_wgrad(dt, dPre, d.d_out, d.d_out, H_in, d.d_in, d.d_in, n, grads->W, ldw, accumulate, p.wg2, s2,
                              grads->bW));
    }
    if (conv_transform_first(d)) {
      // forward was mean(H W_neigh^T): dT = mean^T(dPre), dW_neigh = dT^T H, dH = dPre W_self + dT W_neigh
      AggArgs t = agg();
      t.X = dPre; t.Y = p.T; t.width = d.d_out; t.ldx = t.ldy = d.d_out;
      t.in_scale = g.inv_deg;
      COFREE_TRY(launch_aggregate(t, s));
      COFREE_TRY(launch_wgrad(dt, p.T, d.d_out, d.d_out, H_in, d.d_in, d.d_in, n, grads->W + d.d_in, ldw, accumulate,
                              p.wg, s));
      if (dH_in) {
        GemmArgs h = gemm();
        // W_self and W_neigh are column blocks of W: dH = dPre W_self + dT W_neigh is one product over the
        // two k-segments [dPre | dT], each with its own block
        h.A1 = dPre; h.lda1 = d.d_out; h.K1 = d.d_out;
        h.B = params->W; h.ldb = ldw; h.b_kmajor = 1;
        h.A2 = p.T; h.lda2 = d.d_out; h.K2 = d.d_out;
        h.B2 = params->W + d.d_in; h.ldb2 = ldw;
        h.C = dH_in; h.ldc = d.d_in; h.N = d.d_in;
        h.gate = in_gate; h.ldg = d.d_in; h.gate_scale = in_scale;
        COFREE_TRY(launch_gemm(h, s));
      }
    } else {
      // forward was [H | mean(H)] W^T: dW_neigh = dPre^T M (side stream as well),
      // dH = dPre W_self + mean^T(dPre W_neigh)
      COFREE_REQUIRE(saved->A, "layer_bwd: saved.A is NULL");
      if (!merged_dW)
        COFREE_TRY(launch_wgrad(dt, dPre, d.d_out, d.d_out, saved->A, d.d_in, d.d_in, n, grads->W + d.d_in, ldw,
                                accumulate, p.wg2, s2));
      if (dH_in) {
        GemmArgs h = gemm();
        h.A1 = dPre; h.lda1 = d.d_out; h.K1 = d.d_out;
        h.B = params->W + d.d_in; h.ldb = ldw; h.b_kmajor = 1;
        h.C = p.T; h.ldc = d.d_in; h.N = d.d_in;
        h.row_scale = g.inv_deg;  // scaled per destination row, so that the transposed mean is a plain pull
        COFREE_TRY(launch_gemm(h, s));
        AggArgs a = agg();
        a.X = p.T; a.Y = dH_in; a.width = d.d_in; a.ldx = a.ldy = d.d_in;
        COFREE_TRY(launch_aggregate(a, s));
        GemmArgs w = gemm();
        w.A1 = dPre; w.lda1 = d.d_out; w.K1 = d.d_out;
        w.B = params->W; w.ldb = ldw; w.b_kmajor = 1;
        w.C = dH_in; w.ldc = d.d_in; w.N = d.d_in;
        w.accumulate = 1;
        w.gate = in_gate; w.ldg = d.d_in; w.gate_last = 1; w.gate_scale = in_scale;
        COFREE_TRY(launch_gemm(w, s));
      }
    }
    return joiner.finish();
  }
  // db = column sums of dPre: on the way of dW when dPre is its operand, else a kernel of its own
  if (gcn_transform_first(d)) COFREE_TRY(launch_colsum(dt, dPre, d.d_out, n, d.d_out, grads->bW, accumulate, p.cs2, s2));
  if (gcn_transform_first(d)) {
    // forward was Ahat (H W^T): dT = Ahat dPre, dW = dT^T H, dH = dT W
    AggArgs a = agg();
    a.X = dPre; a.Y = p.T; a.width = d.d_out; a.ldx = a.ldy = d.d_out;
    a.in_scale = g.gcn_norm; a.out_scale = g.gcn_norm; a.self_loop = 1;
    COFREE_TRY(launch_aggregate(a, s));
    COFREE_TRY(launch_wgrad(dt, p.T, d.d_out, d.d_out, H_in, d.d_in, d.d_in, n, grads->W, d.d_in, accumulate, p.wg,
                            s));
    if (dH_in) {
      GemmArgs h = gemm();
      h.A1 = p.T; h.lda1 = d.d_out; h.K1 = d.d_out;
      h.B = params->W; h.ldb = d.d_in; h.b_kmajor = 1;
      h.C = dH_in; h.ldc = d.d_in; h.N = d.d_in;
      h.gate = in_gate; h.ldg = d.d_in; h.gate_scale = in_scale;
      COFREE_TRY(launch_gemm(h, s));
    }
  } else {
    // forward was (Ahat H) W^T: dW = dPre^T (Ahat H), dH = Ahat (dPre W)
    COFREE_REQUIRE(saved->A, "layer_bwd: saved.A is NULL");
    COFREE_TRY(launch_wgrad(dt, dPre, d.d_out, d.d_out, saved->A, d.d_in, d.d_in, n, grads->W, d.d_in, accumulate,
                            p.wg2, s2, grads->bW));
    if (dH_in) {
      GemmArgs h = gemm();
      h.A1 = dPre; h.lda1 = d.d_out; h.K1 = d.d_out;
      h.B = params->W; h.ldb = d.d_in; h.b_kmajor = 1;
      h.C = p.T; h.ldc = d.d_in; h.N = d.d_in;
      h.row_scale = g.gcn_norm;
      COFREE_TRY(launch_gemm(h, s));
      AggArgs a = agg();
      a.X = p.T; a.Y = dH_in; a.width = d.d_in; a.ldx = a.ldy = d.d_in;
      a.out_scale = g.gcn_norm; a.self_loop = 1;
      a.relu_src = in_gate; a.ld_relu = d.d_in; a.gate_scale = in_scale;
      COFREE_TRY(launch_aggregate(a, s));
    }
  }
  return joiner.finish();
}

}  // extern "C"
