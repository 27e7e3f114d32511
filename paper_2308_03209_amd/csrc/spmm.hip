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
  const int64_t row = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * RPW + lane / LANES;
  if (row >= n) return;
  const int col_base = p.col0;
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

// Variant for graphs whose rows are gathered many times (high average degree).
// One wavefront per (row, column slice).  A slice is LPS lanes x 4 floats wide; the 64 lanes
// form 64/LPS neighbour groups that fetch different neighbours in the same load instruction and
// are added together at the end in a fixed butterfly order, so a row of degree d costs
// d*LPS/64 load instructions however narrow the matrix is.
// SLICES = 8 is the XCD-aware launch for matrices far larger than one XCD's 4 MB L2: workgroups
// are dealt round-robin to the 8 XCDs, so workgroup b works on column slice b % 8 of row group
// b / 8, and each XCD's L2 only ever holds one eighth of every row - eight times as many (hot)
// rows.  SLICES = 1 covers the whole width (<= LPS*4 columns) with one slice.
// Rows need only 4-byte alignment; a lane whose 4 columns cross the end of the row falls back to
// guarded scalar accesses.
typedef float float4u __attribute__((ext_vector_type(4), aligned(4)));

template <int LPS, int SLICES>
__global__ __launch_bounds__(256) void aggregate_group_kernel(const AggK p) {
  constexpr int NG = 64 / LPS;
  constexpr int UNR = 4;
  const int lane = threadIdx.x & 63;
  const int sub = lane % LPS, grp = lane / LPS;
  const int slice = SLICES == 1 ? 0 : (int)(blockIdx.x % (unsigned)SLICES);
  const int64_t row = (int64_t)(blockIdx.x / (unsigned)SLICES) * 4 + (threadIdx.x >> 6);
  if (row >= p.n) return;
  const int c0 = slice * (LPS * 4) + sub * 4;  // first of this lane's 4 columns
  const int n_cols = p.width - c0 < 4 ? p.width - c0 : 4;  // how many of them exist (may be <= 0)
  const float* __restrict__ X = p.X + c0;
  const int32_t* __restrict__ col = p.col;
  const float* __restrict__ in_scale = p.in_scale;
  const int64_t beg = p.rowptr[row], end = p.rowptr[row + 1];
  auto load4 = [&](const float* src, float (&v)[4]) {
    if (n_cols == 4) {
      const float4u t = *reinterpret_cast<const float4u*>(src);
      v[0] = t[0];
      v[1] = t[1];
      v[2] = t[2];
      v[3] = t[3];
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) v[i] = i < n_cols ? src[i] : 0.f;
    }
  };
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int64_t e = beg + grp; e < end; e += NG * UNR) {
    int u[UNR];
    float s[UNR];
    float v[UNR][4];
#pragma unroll
    for (int t = 0; t < UNR; ++t) {
      const int64_t ee = e + t * NG;
      u[t] = ee < end ? col[ee] : -1;
    }
#pragma unroll
    for (int t = 0; t < UNR; ++t) {
      s[t] = 1.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) v[t][i] = 0.f;
      if (u[t] >= 0) {
        if (in_scale) s[t] = in_scale[u[t]];
        load4(X + (int64_t)u[t] * p.ldx, v[t]);
      }
    }
#pragma unroll
    for (int t = 0; t < UNR; ++t)
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] = fmaf(s[t], v[t][i], acc[i]);
  }
#pragma unroll
  for (int off = LPS; off < 64; off <<= 1) {
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] += __shfl_xor(acc[i], off, 64);
  }
  if (grp != 0 || n_cols <= 0) return;
  if (p.self_loop) {
    const float ss = in_scale ? in_scale[row] : 1.f;
    float xs[4];
    load4(X + row * p.ldx, xs);
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = fmaf(ss, xs[i], acc[i]);
  }
  const float so = p.out_scale ? p.out_scale[row] : 1.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) acc[i] *= so;
  if (p.relu_src) {
    float gt[4];
    load4(p.relu_src + row * p.ld_relu + c0, gt);
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (i < n_cols && !(gt[i] > 0.f)) acc[i] = 0.f;
  }
  if (p.bias) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (i < n_cols) acc[i] += p.bias[p.col0 + c0 + i];
  }
  if (p.relu_out) {
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = fmaxf(acc[i], 0.f);
  }
  float* dst = p.Y + row * p.ldy + c0;
  if (n_cols == 4) {
    float4u o;
    o[0] = acc[0];
    o[1] = acc[1];
    o[2] = acc[2];
    o[3] = acc[3];
    *reinterpret_cast<float4u*>(dst) = o;
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (i < n_cols) dst[i] = acc[i];
  }
}

template <int SLICES>
static int32_t launch_group(const AggK& k, int lps, hipStream_t stream) {
  const int64_t blocks = ((k.n + 3) / 4) * SLICES;
  COFREE_REQUIRE(blocks < ((int64_t)1 << 31), "aggregate: grid too large");
  const dim3 grid((unsigned)blocks);
  switch (lps) {
    case 1: aggregate_group_kernel<1, SLICES><<<grid, 256, 0, stream>>>(k); break;
    case 2: aggregate_group_kernel<2, SLICES><<<grid, 256, 0, stream>>>(k); break;
    case 4: aggregate_group_kernel<4, SLICES><<<grid, 256, 0, stream>>>(k); break;
    case 8: aggregate_group_kernel<8, SLICES><<<grid, 256, 0, stream>>>(k); break;
    case 16: aggregate_group_kernel<16, SLICES><<<grid, 256, 0, stream>>>(k); break;
    case 32: aggregate_group_kernel<32, SLICES><<<grid, 256, 0, stream>>>(k); break;
    case 64: aggregate_group_kernel<64, SLICES><<<grid, 256, 0, stream>>>(k); break;
    default: return fail(COFREE_EINVAL, "internal: bad lanes-per-slice");
  }
  return COFREE_OK;
}

template <int VEC, int LANES, int NCH>
static void launch_one(const AggK& k, hipStream_t stream) {
  constexpr int rows_per_block = 4 * (64 / LANES);
  const int64_t blocks = (k.n + rows_per_block - 1) / rows_per_block;
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
  // High average degree: the neighbour-group kernel (a wavefront per row fetches 64/LPS
  // neighbours per load instruction).  Additionally cut into 8 XCD-affine column slices when
  // the matrix is far larger than one XCD's 4 MB L2 and the width divides evenly.
  const bool dense_rows = a.g.nnz / a.g.n >= 16;
  const bool sliceable = a.width % 32 == 0 && a.width <= 2048 && (a.width / 32 & (a.width / 32 - 1)) == 0 &&
                         a.ldx % 4 == 0 && al16(X);
  bool grouped = dense_rows && a.width <= 256;
  bool sliced = dense_rows && sliceable && (double)a.g.n * a.width * sizeof(float) > 32e6;
  if (const char* env = getenv("COFREE_AGG_SLICES")) {  // tuning override: 0 = row kernel, 1 = grouped, 8 = sliced
    const int v = atoi(env);
    if (v == 0) grouped = sliced = false;
    if (v == 1) { grouped = a.width <= 256; sliced = false; }
    if (v == 8) sliced = sliceable;
  }
  if (sliced || grouped) {
    k.width = a.width;
    k.col0 = 0;
    k.X = X;
    k.Y = Y;
    k.relu_src = R;
    if (sliced) {
      COFREE_TRY(launch_group<8>(k, a.width / 32, stream));
    } else {
      int lps = 1;
      while (lps * 4 < a.width) lps *= 2;
      COFREE_TRY(launch_group<1>(k, lps, stream));
    }
  } else {
    for (int c0 = 0; c0 < a.width; c0 += panel) {
      k.width = a.width - c0 < panel ? a.width - c0 : panel;
      k.col0 = c0;
      k.X = X + c0;
      k.Y = Y + c0;
      k.relu_src = R ? R + c0 : nullptr;
      if (vec) COFREE_TRY(dispatch<4>(k, stream));
      else COFREE_TRY(dispatch<1>(k, stream));
    }
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
