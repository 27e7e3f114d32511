// Neighbour aggregation on the partition graph (the AGG of the layer definition in Section 3)
// and its transpose for backward (the per-edge factor 1/D(v_j[i]) in the proof of Theorem 3).
//
// The edge weights of both the mean and the GCN normalisation factor into a per-source and a
// per-destination vector, so the kernel walks a pattern-only CSR:
//     Y[v] = out_scale[v] * ( self * in_scale[v] * X[v] + sum_{u in N(v)} in_scale[u] * X[u] )
// Because the (masked) partition graph is symmetric, the transposed product is the same pull
// with the roles of the two scale vectors exchanged - no atomics, fixed summation order.
//
// Mapping: a group of LANES lanes of a 64-wide wavefront owns one row; lane `sub` holds VEC
// consecutive feature columns per chunk, so one neighbour row is fetched by the group as one
// contiguous LANES*VEC*4-byte segment.  Column indices are fetched LANES at a time with one
// coalesced load and handed out by cross-lane reads.
#include <cstdlib>

#include "common.h"

namespace cofree {

template <int VEC>
struct FVec;
template <>
struct FVec<4> {
  using type = float4;
};

template <int VEC>
__device__ inline void load_row(const float* p, float (&v)[VEC]) {
  if constexpr (VEC == 4) {
    const float4 t = *reinterpret_cast<const float4*>(p);
    v[0] = t.x;
    v[1] = t.y;
    v[2] = t.z;
    v[3] = t.w;
  } else {
    v[0] = *p;
  }
}
template <int VEC>
__device__ inline void store_row(float* p, const float (&v)[VEC]) {
  if constexpr (VEC == 4) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  } else {
    *p = v[0];
  }
}

template <int LANES>
__device__ inline int group_read_i(int x, int grp_base, int j) {
  if constexpr (LANES == 64) {
    return __builtin_amdgcn_readlane(x, j);
  } else {
    return __shfl(x, grp_base + j, 64);
  }
}
template <int LANES>
__device__ inline float group_read_f(float x, int grp_base, int j) {
  if constexpr (LANES == 64) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), j));
  } else {
    return __shfl(x, grp_base + j, 64);
  }
}

struct AggK {
  const int64_t* rowptr;
  const int32_t* col;
  const float* X;
  int64_t ldx;
  float* Y;
  int64_t ldy;
  int width;  // columns of this panel
  int64_t n;
  const float* in_scale;
  const float* out_scale;
  int self_loop;
  const float* relu_src;
  int64_t ld_relu;
  // output epilogue (after out_scale): + bias, ReLU
  const float* bias;
  int relu_out;
  int col0;      // first column of this panel in the full matrix
  int n_slices;  // the panel is cut into n_slices column slices of `width` columns each; slice =
                 // blockIdx.x % n_slices, so that (with workgroups dealt round-robin to the 8
                 // XCDs) one XCD's L2 only ever holds one slice of the gathered rows
};

template <int VEC, int LANES, int NCH>
__global__ __launch_bounds__(256) void aggregate_kernel(const AggK p) {
  const int64_t* __restrict__ rowptr = p.rowptr;
  const int32_t* __restrict__ col = p.col;
  const float* X = p.X;
  float* Y = p.Y;
  const float* __restrict__ in_scale = p.in_scale;
  const float* __restrict__ out_scale = p.out_scale;
  const float* relu_src = p.relu_src;
  const int64_t ldx = p.ldx, ldy = p.ldy, ld_relu = p.ld_relu, n = p.n;
  const int width = p.width, self_loop = p.self_loop;
  constexpr int RPW = 64 / LANES;  // rows per wavefront
  constexpr int UNR = 4;
  const int lane = threadIdx.x & 63;
  const int sub = lane % LANES;
  const int grp_base = (lane / LANES) * LANES;
  const int slice = (int)(blockIdx.x % (unsigned)p.n_slices);
  const int64_t row_block = blockIdx.x / (unsigned)p.n_slices;
  const int64_t row = (row_block * 4 + (threadIdx.x >> 6)) * RPW + lane / LANES;
  if (row >= n) return;
  X += slice * width;
  Y += slice * width;
  if (relu_src) relu_src += slice * width;
  const int col_base = p.col0 + slice * width;
  const int64_t beg = rowptr[row], end = rowptr[row + 1];

  float acc[NCH][VEC];
  bool live[NCH];
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    live[c] = (sub + c * LANES) * VEC < width;
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[c][i] = 0.f;
  }

  for (int64_t e0 = beg; e0 < end; e0 += LANES) {
    int my_col = -1;
    float my_s = 1.f;
    if (e0 + sub < end) {
      my_col = col[e0 + sub];
      if (in_scale) my_s = in_scale[my_col];
    }
    const int cnt = (int)((end - e0) < (int64_t)LANES ? (end - e0) : (int64_t)LANES);
    for (int j = 0; j < cnt; j += UNR) {
      int u[UNR];
      float s[UNR];
      float v[UNR][NCH][VEC];
#pragma unroll
      for (int t = 0; t < UNR; ++t) {
        // j + t < LANES always (LANES is a multiple of UNR, or the read wraps harmlessly below)
        const int jj = (j + t) % LANES;
        u[t] = group_read_i<LANES>(my_col, grp_base, jj);
        s[t] = group_read_f<LANES>(my_s, grp_base, jj);
        if (j + t >= cnt) u[t] = -1;
      }
#pragma unroll
      for (int t = 0; t < UNR; ++t) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
          if (u[t] >= 0 && live[c]) {
            load_row<VEC>(X + (int64_t)u[t] * ldx + (sub + c * LANES) * VEC, v[t][c]);
          } else {
#pragma unroll
            for (int i = 0; i < VEC; ++i) v[t][c][i] = 0.f;
          }
        }
      }
#pragma unroll
      for (int t = 0; t < UNR; ++t)
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
          for (int i = 0; i < VEC; ++i) acc[c][i] = fmaf(s[t], v[t][c][i], acc[c][i]);
    }
  }

  const float so = out_scale ? out_scale[row] : 1.f;
  const float ss = (self_loop && in_scale) ? in_scale[row] : 1.f;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    if (!live[c]) continue;
    const int c0 = (sub + c * LANES) * VEC;
    if (self_loop) {
      float xs[VEC];
      load_row<VEC>(X + row * ldx + c0, xs);
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[c][i] = fmaf(ss, xs[i], acc[c][i]);
    }
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[c][i] *= so;
    if (relu_src) {
      float g[VEC];
      load_row<VEC>(relu_src + row * ld_relu + c0, g);
#pragma unroll
      for (int i = 0; i < VEC; ++i)
        if (!(g[i] > 0.f)) acc[c][i] = 0.f;
    }
    if (p.bias) {
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[c][i] += p.bias[col_base + c0 + i];
    }
    if (p.relu_out) {
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[c][i] = fmaxf(acc[c][i], 0.f);
    }
    store_row<VEC>(Y + row * ldy + c0, acc[c]);
  }
}

template <int VEC, int LANES, int NCH>
static void launch_one(const AggK& k, hipStream_t stream) {
  constexpr int rows_per_block = 4 * (64 / LANES);
  const int64_t blocks = ((k.n + rows_per_block - 1) / rows_per_block) * k.n_slices;
  aggregate_kernel<VEC, LANES, NCH><<<dim3((unsigned)blocks), 256, 0, stream>>>(k);
}

template <int VEC>
static int32_t dispatch(const AggK& k, hipStream_t stream) {
  const int chunks = (k.width + VEC - 1) / VEC;
  if (chunks <= 2) launch_one<VEC, 2, 1>(k, stream);
  else if (chunks <= 4) launch_one<VEC, 4, 1>(k, stream);
  else if (chunks <= 8) launch_one<VEC, 8, 1>(k, stream);
  else if (chunks <= 16) launch_one<VEC, 16, 1>(k, stream);
  else if (chunks <= 32) launch_one<VEC, 32, 1>(k, stream);
  else if (chunks <= 64) launch_one<VEC, 64, 1>(k, stream);
  else if (chunks <= 128) launch_one<VEC, 64, 2>(k, stream);
  else return fail(COFREE_EINVAL, "internal: aggregate panel too wide");
  return COFREE_OK;
}

int32_t launch_aggregate(const AggArgs& a, hipStream_t stream) {
  COFREE_REQUIRE(a.dtype == COFREE_F32, "aggregate: only COFREE_F32 is implemented");
  COFREE_REQUIRE(a.width >= 1, "aggregate: width must be >= 1");
  COFREE_REQUIRE(a.X && a.Y && a.X != a.Y, "aggregate: X and Y must be distinct non-NULL buffers");
  COFREE_REQUIRE(a.ldx >= a.width && a.ldy >= a.width, "aggregate: leading dimension smaller than width");
  COFREE_REQUIRE(a.g.n < ((int64_t)1 << 31), "aggregate: too many rows");
  if (a.g.n == 0) return COFREE_OK;
  const float* X = (const float*)a.X;
  float* Y = (float*)a.Y;
  const float* R = (const float*)a.relu_src;
  auto al16 = [](const void* p) { return ((uintptr_t)p & 15u) == 0; };
  const bool vec = a.width % 4 == 0 && a.ldx % 4 == 0 && a.ldy % 4 == 0 && al16(X) && al16(Y) &&
                   (!R || (a.ld_relu % 4 == 0 && al16(R)));
  AggK k{};
  k.rowptr = a.g.rowptr;
  k.col = a.g.col;
  k.ldx = a.ldx;
  k.ldy = a.ldy;
  k.n = a.g.n;
  k.in_scale = a.in_scale;
  k.out_scale = a.out_scale;
  k.self_loop = a.self_loop;
  k.ld_relu = a.ld_relu;
  k.bias = a.bias;
  k.relu_out = a.relu_out;
  const int panel = vec ? 512 : 128;  // columns one launch covers
  // algorithmic traffic: every source row read once, every output row written once, the
  // pattern (4 B per kept entry, 8 B per row offset) and the per-node scale vectors once
  const double rows_bytes = 2.0 * (double)a.g.n * a.width * sizeof(float);
  const double idx_bytes = 4.0 * (double)a.g.nnz + 8.0 * (double)(a.g.n + 1) +
                           4.0 * (double)a.g.n * ((a.in_scale ? 1 : 0) + (a.out_scale ? 1 : 0)) +
                           (R ? (double)a.g.n * a.width * sizeof(float) : 0.0);
  ProfScope prof("aggregate_kernel", stream, rows_bytes + idx_bytes, 2.0 * (double)a.g.nnz * a.width);
  for (int c0 = 0; c0 < a.width; c0 += panel) {
    k.width = a.width - c0 < panel ? a.width - c0 : panel;
    k.col0 = c0;
    k.X = X + c0;
    k.Y = Y + c0;
    k.relu_src = R ? R + c0 : nullptr;
    if (vec) COFREE_TRY(dispatch<4>(k, stream));
    else COFREE_TRY(dispatch<1>(k, stream));
  }
  COFREE_HIP_CHECK(hipGetLastError());
  return COFREE_OK;
}

}  // namespace cofree

using namespace cofree;

extern "C" int32_t cofree_aggregate(const cofree_partition* part, const cofree_masks* masks, int32_t mask_id,
                                    int32_t mode, const void* X, void* Y, int32_t width, int32_t dtype,
                                    void* stream) {
  AggArgs a;
  COFREE_TRY(select_graph(part, masks, mask_id, &a.g));
  a.X = X;
  a.Y = Y;
  a.width = width;
  a.ldx = a.ldy = width;
  a.dtype = dtype;
  switch (mode) {
    case COFREE_AGG_MEAN: a.out_scale = a.g.inv_deg; break;
    case COFREE_AGG_MEAN_T: a.in_scale = a.g.inv_deg; break;
    case COFREE_AGG_GCN:
      a.in_scale = a.g.gcn_norm;
      a.out_scale = a.g.gcn_norm;
      a.self_loop = 1;
      break;
    default: return fail(COFREE_EINVAL, "aggregate: unknown mode");
  }
  return launch_aggregate(a, (hipStream_t)stream);
}
