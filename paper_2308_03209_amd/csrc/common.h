// Internal declarations shared by the translation units of libcofree (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "../../include/cofree.h"

namespace cofree {

// ---- errors -----------------------------------------------------------------------------
void set_error(const std::string& msg);
int32_t fail(int32_t code, const std::string& msg);
#define COFREE_HIP_CHECK(expr)                                                                     \
  do {                                                                                             \
    hipError_t e__ = (expr);                                                                       \
    if (e__ != hipSuccess)                                                                         \
      return ::cofree::fail(COFREE_EHIP, std::string(#expr) + ": " + hipGetErrorString(e__));      \
  } while (0)
#define COFREE_REQUIRE(cond, msg)                                  \
  do {                                                             \
    if (!(cond)) return ::cofree::fail(COFREE_EINVAL, (msg));      \
  } while (0)
#define COFREE_TRY(expr)                 \
  do {                                   \
    int32_t rc__ = (expr);               \
    if (rc__ != COFREE_OK) return rc__;  \
  } while (0)

// ---- optional kernel timing (profile.cpp) -------------------------------------------------
// Brackets one kernel launch with HIP events on its stream when profiling is enabled, and
// books the launch's algorithmic bytes / flops under `name`.
class ProfScope {
 public:
  ProfScope(const char* name, hipStream_t stream, double alg_bytes, double alg_flops);
  ~ProfScope();
  ProfScope(const ProfScope&) = delete;
  ProfScope& operator=(const ProfScope&) = delete;

 private:
  hipEvent_t start_ = nullptr, stop_ = nullptr;
  hipStream_t stream_ = nullptr;
  int cls_ = -1;
  bool active_ = false;
};

// ---- Philox-4x32-10 (Salmon et al., SC'11), host and device -----------------------------
struct u32x4 {
  uint32_t x, y, z, w;
};

__host__ __device__ inline u32x4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                               uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return u32x4{c0, c1, c2, c3};
}

enum : uint32_t { STREAM_CUT = 1, STREAM_MASK = 2, STREAM_PICK = 3, STREAM_DROPOUT = 4 };

// counter (a mod 2^32, a div 2^32, b, stream), key = the two halves of seed
__host__ __device__ inline u32x4 draw4(uint64_t seed, uint32_t stream, uint64_t a, uint32_t b) {
  return philox4x32_10((uint32_t)a, (uint32_t)(a >> 32), b, stream, (uint32_t)seed, (uint32_t)(seed >> 32));
}
__host__ __device__ inline uint32_t draw1(uint64_t seed, uint32_t stream, uint64_t a, uint32_t b) {
  return draw4(seed, stream, a, b).x;
}
// floor(prob * 2^32) for prob in [0, 1)
inline uint32_t prob_threshold(double prob) { return (uint32_t)(prob * 4294967296.0); }

// ---- bfloat16 storage (round-to-nearest-even; arithmetic is always float32) ------------------
typedef uint16_t bf16_t;
typedef __bf16 bf16x2_hw __attribute__((ext_vector_type(2)));
typedef float f32x2_hw __attribute__((ext_vector_type(2)));
__device__ inline float bf16_to_f32(bf16_t h) { return __uint_as_float((uint32_t)h << 16); }
// Two float32 -> two bfloat16 in one dword (lo in bits 0..15): the hardware conversion of gfx950
// (v_cvt_pk_bf16_f32), round-to-nearest-even, NaN stays NaN.
__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2_hw v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_hw));
}
__device__ inline bf16_t f32_to_bf16(float f) { return (bf16_t)(pack_bf16x2(f, 0.f) & 0xffffu); }

// ---- graph views ------------------------------------------------------------------------
// One CSR on the device with its per-node normalisation vectors.
struct DeviceGraph {
  const int64_t* rowptr = nullptr;  // [n+1]
  const int32_t* col = nullptr;     // [nnz]
  const float* inv_deg = nullptr;   // [n]  1/deg, 0 where deg = 0
  const float* gcn_norm = nullptr;  // [n]  1/sqrt(deg+1)
  // the same factors per adjacency entry, val_x[e] = x[col[e]]: read in one coalesced stream next to col,
  // where the per-node vector would cost a gather of its own per neighbour
  const float* val_inv_deg = nullptr;   // [nnz]
  const float* val_gcn_norm = nullptr;  // [nnz]
  const int32_t* order = nullptr;   // [n]  rows sorted by descending degree, ties by ascending row (processing order)
  // The same graph once more with its rows stored in processing order (slot i holds row order[i]): what the
  // short-row kernel walks.  Row offsets, neighbour ids, per-entry factors and the row's own factors then arrive
  // as streams; read by row id in processing order, each of them cost a cache line per row.
  const int64_t* s_rowptr = nullptr;        // [n+1]
  const int32_t* s_col = nullptr;           // [nnz]
  const float* s_val_inv_deg = nullptr;     // [nnz]
  const float* s_val_gcn_norm = nullptr;    // [nnz]
  const float* s_inv_deg = nullptr;         // [n]  inv_deg[order[i]]
  const float* s_gcn_norm = nullptr;        // [n]  gcn_norm[order[i]]
  int64_t n = 0;
  int64_t nnz = 0;
  // `order` starts with the hub rows: its first n_hub rows have at least AGG_HUB_MIN neighbours, nnz_hub
  // adjacency entries in all
  int64_t n_hub = 0, nnz_hub = 0;
};

// Rows of at least AGG_HUB_MIN neighbours are split over the wavefronts of a whole workgroup (hub rows: the
// nodes that keep a high degree after the cut, Theorem 2).  One lane group walks a row at about 0.12 us per
// neighbour, a workgroup at 0.013: at 4096 neighbours a row alone takes as long as a whole launch over a
// million-row graph (0.4-0.5 ms), below that the descending-degree order of the launches hides it.
// AGG_ENTRY_SCALE_MIN_NODES: from this many nodes on (a per-node vector of 2 MB, half of one XCD's L2) the
// per-source factors of an aggregation are read per adjacency entry instead of gathered per neighbour.
// AGG_LONG_MIN: graphs of at least this average degree spread a row's neighbours over the lane groups of a
// wavefront; below it a row gets one lane group.
constexpr int64_t AGG_HUB_MIN = 4096, AGG_LONG_MIN = 16, AGG_ENTRY_SCALE_MIN_NODES = 1 << 19;
struct DegreeBuckets {
  int64_t n_hub = 0, nnz_hub = 0;
};

// device storage of the processing-order copy (see DeviceGraph)
struct SlotCsr {
  int64_t* rowptr = nullptr;
  int32_t* col = nullptr;
  float* val_inv_deg = nullptr;
  float* val_gcn_norm = nullptr;
  float* inv_deg = nullptr;
  float* gcn_norm = nullptr;
  void attach(DeviceGraph* g) const {
    g->s_rowptr = rowptr;
    g->s_col = col;
    g->s_val_inv_deg = val_inv_deg;
    g->s_val_gcn_norm = val_gcn_norm;
    g->s_inv_deg = inv_deg;
    g->s_gcn_norm = gcn_norm;
  }
};
void free_slot_csr(SlotCsr* s);

struct HostGraph {
  std::vector<int64_t> rowptr;
  std::vector<int32_t> col;
};

}  // namespace cofree

struct cofree_partition {
  int64_t n_nodes = 0, n_edges = 0, nnz = 0;
  int64_t n_nodes_full = 0;
  std::vector<int64_t> local2global;
  std::vector<int64_t> rowptr;
  std::vector<int32_t> col, eid, deg_local, deg_global, edge_lo, edge_hi;
  std::vector<float> dar_weight;
  std::vector<int32_t> rf;  // RF(v_j) per local node; empty unless built with COFREE_WITH_RF
  // device copies (null when built with COFREE_HOST_ONLY)
  bool on_device = false;
  int device = -1;
  int64_t* d_rowptr = nullptr;
  int32_t* d_col = nullptr;
  int32_t* d_eid = nullptr;
  int32_t* d_deg_local = nullptr;
  float* d_dar_weight = nullptr;
  float* d_inv_deg = nullptr;
  float* d_gcn_norm = nullptr;
  float* d_val_inv_deg = nullptr;
  float* d_val_gcn_norm = nullptr;
  int64_t* d_local2global = nullptr;
  int32_t* d_order = nullptr;  // rows by descending degree
  cofree::DegreeBuckets buckets;
  cofree::SlotCsr d_slots;
  float* d_inv_rf = nullptr;  // 1 / RF(v_j), with COFREE_WITH_RF
  cofree::DeviceGraph graph() const {
    cofree::DeviceGraph g;
    g.rowptr = d_rowptr;
    g.col = d_col;
    g.inv_deg = d_inv_deg;
    g.gcn_norm = d_gcn_norm;
    g.val_inv_deg = d_val_inv_deg;
    g.val_gcn_norm = d_val_gcn_norm;
    g.order = d_order;
    d_slots.attach(&g);
    g.n = n_nodes;
    g.nnz = nnz;
    g.n_hub = buckets.n_hub;
    g.nnz_hub = buckets.nnz_hub;
    return g;
  }
};

struct cofree_masks {
  int32_t K = 0;
  int64_t n_nodes = 0, n_edges = 0, n_words = 0;
  uint64_t* d_bits = nullptr;               // device, [K][n_words]
  std::vector<std::vector<uint64_t>> bits;  // [K][n_words] host copies, fetched on first request
  std::vector<cofree::HostGraph> host;      // [K] host copies of the compacted graphs, fetched on first request
  struct Dev {
    int64_t* rowptr = nullptr;
    int32_t* col = nullptr;
    float* inv_deg = nullptr;
    float* gcn_norm = nullptr;
    float* val_inv_deg = nullptr;   // [nnz] inv_deg[col[e]]
    float* val_gcn_norm = nullptr;  // [nnz] gcn_norm[col[e]]
    int32_t* order = nullptr;  // rows by descending masked degree
    int64_t nnz = 0;
    cofree::DegreeBuckets buckets;
    cofree::SlotCsr slots;
  };
  std::vector<Dev> dev;  // [K]
};

namespace cofree {

// Resolve (partition, masks, mask_id) to the CSR the kernels walk.
int32_t select_graph(const cofree_partition* part, const cofree_masks* masks, int32_t mask_id, DeviceGraph* out);

// ---- kernel launchers (device pointers, enqueue only) -------------------------------------
struct DropoutArgs {
  float q = 0.f;
  uint64_t seed = 0;
  uint32_t epoch = 0;
  uint32_t layer_id = 0;
};

struct AggArgs {
  DeviceGraph g;
  const void* X = nullptr;
  void* Y = nullptr;
  int32_t width = 0;
  int64_t ldx = 0, ldy = 0;
  int32_t dtype = COFREE_F32;
  const float* in_scale = nullptr;   // per-source factor, or null
  const float* out_scale = nullptr;  // per-destination factor, or null
  int32_t self_loop = 0;             // 1: add in_scale[v] * X[v] to the sum of row v
  const void* relu_src = nullptr;    // if set: Y[v,c] = 0 where relu_src[v,c] <= 0 (same dtype, ld = ld_relu)
  int64_t ld_relu = 0;
  float gate_scale = 1.f;            // factor on the elements that pass relu_src
  // applied after out_scale, in this order: + bias[c], ReLU
  const float* bias = nullptr;
  int32_t relu_out = 0;
};
int32_t launch_aggregate(const AggArgs& a, hipStream_t stream);
// Allocates and fills the processing-order copy of g (g.order and the per-node vectors must be set).
int32_t build_slot_csr(const DeviceGraph& g, SlotCsr* out, hipStream_t stream);
// val_inv_deg[e] = inv_deg[col[e]], val_gcn_norm[e] = gcn_norm[col[e]] for e < nnz
int32_t launch_entry_scales(const int32_t* col, int64_t nnz, const float* inv_deg, const float* gcn_norm,
                            float* val_inv_deg, float* val_gcn_norm, hipStream_t stream);

// C[M,N] = epilogue( sum_s A_s . op(B) ).  Activations (A segments, C, gate) have `dtype`
// (float32, or bfloat16 with float32 accumulation); B holds float32 parameters.
struct GemmArgs {
  int32_t dtype = COFREE_F32;
  // operand A: up to two K-segments, each row-major [M, K_s] with leading dimension lda_s
  const void* A1 = nullptr;
  int64_t lda1 = 0;
  int32_t K1 = 0;
  const void* A2 = nullptr;
  int64_t lda2 = 0;
  int32_t K2 = 0;
  // operand B: b_kmajor = 0: [N, K] row-major (C = A B^T); 1: [K, N] row-major (C = A B)
  const float* B = nullptr;
  int64_t ldb = 0;
  int32_t b_kmajor = 0;
  // optional: the second K-segment multiplies this matrix (same orientation, its own k from 0) instead of
  // the k-range K1.. of B - for sums of two products with different parameters, C = A1 op(B) + A2 op(B2)
  const float* B2 = nullptr;
  int64_t ldb2 = 0;
  void* C = nullptr;
  int64_t ldc = 0;
  int64_t M = 0;
  int32_t N = 0;
  // epilogue, applied in this order
  const float* bias = nullptr;       // [N]
  int32_t relu = 0;
  const float* row_scale = nullptr;  // [M]
  const void* gate = nullptr;        // [M, N] (ldg): result is zeroed where gate <= 0 (ReLU backward)
  int64_t ldg = 0;
  int32_t accumulate = 0;            // C += result
  int32_t relu_last = 0;             // ReLU after the accumulation
  int32_t gate_last = 0;             // apply `gate` after the accumulation instead of before it
  float gate_scale = 1.f;            // factor on the elements that pass `gate`
  // bfloat16 only: scratch for the parameters converted to bfloat16, gemm_param_scratch_bytes(N, K1+K2)
  void* param_scratch = nullptr;
};
int32_t launch_gemm(const GemmArgs& a, hipStream_t stream);
size_t gemm_param_scratch_bytes(int32_t N, int64_t K);

// C[N1,N2] (+)= A^T B with A [M, N1] (lda), B [M, N2] (ldb) of `dtype`, C float32: reduction over
// the long dimension M in fixed-order split chunks.  workspace: wgrad_workspace_floats(N1, N2 + N2b, M).
size_t wgrad_workspace_floats(int32_t N1, int32_t N2, int64_t M);
// colsum_out (optional, [N1]) (+)= column sums of A, computed on the way (the bias gradient that goes with C).
// B2 (optional): a second matrix [M, N2b] (ldb2) whose product with the same A fills the columns N2 .. of C -
// two weight gradients that share the incoming gradient read it once; N2 must be a multiple of 128.
int32_t launch_wgrad(int32_t dtype, const void* A, int64_t lda, int32_t N1, const void* B, int64_t ldb, int32_t N2,
                     int64_t M, float* C, int64_t ldc, int32_t accumulate, float* workspace, hipStream_t stream,
                     float* colsum_out = nullptr, const void* B2 = nullptr, int64_t ldb2 = 0, int32_t N2b = 0);
// shared by the float32 and bfloat16 paths; resident = workgroups of the kernel the chip holds at once
// (three per CU for the float32 kernel, two for the bfloat16 one)
constexpr int32_t WGRAD_RESIDENT_F32 = 768, WGRAD_RESIDENT_BF16 = 512;
int32_t wgrad_splits(int32_t N1, int32_t N2, int64_t M, int32_t resident);
int32_t launch_split_reduce(const float* partials, int64_t split_stride, int32_t splits, float* C, int64_t ldc,
                            int32_t rows, int32_t cols, int32_t accumulate, hipStream_t stream);
int32_t launch_gemm_bf16(const GemmArgs& a, hipStream_t stream);
int32_t launch_wgrad_bf16(const bf16_t* A, int64_t lda, int32_t N1, const bf16_t* B, int64_t ldb, int32_t N2,
                          int64_t M, float* C, int64_t ldc, int32_t accumulate, float* workspace,
                          hipStream_t stream, float* colsum_out, const bf16_t* B2, int64_t ldb2, int32_t N2b);

// out[N] (+)= column sums of X [M, N] (ld) of `dtype`; workspace floats: colsum_workspace_floats(N)
size_t colsum_workspace_floats(int32_t N);
int32_t launch_colsum(int32_t dtype, const void* X, int64_t ld, int64_t M, int32_t N, float* out,
                      int32_t accumulate, float* workspace, hipStream_t stream);

// dst[r,c] = src[r,c] * [gate[r,c] > 0 if gate] * keep(r,c)/(1-q) if q > 0   (`dtype`, contiguous [M,N];
// dst may be src)
int32_t launch_mask_grad(int32_t dtype, const void* src, const void* gate, void* dst, int64_t M, int32_t N,
                         const DropoutArgs& d, hipStream_t stream);

}  // namespace cofree
