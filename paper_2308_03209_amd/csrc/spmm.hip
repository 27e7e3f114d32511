// Neighbour aggregation on the partition graph (the AGG of the layer definition in Section 3)
// and its transpose for backward (the per-edge factor 1/D(v_j[i]) in the proof of Theorem 3).
//
// The edge weights of both the mean and the GCN normalisation factor into a per-source and a
// per-destination vector, so the kernels walk a pattern-only CSR:
//     Y[v] = out_scale[v] * ( self * in_scale[v] * X[v] + sum_{u in N(v)} in_scale[u] * X[u] )
// Because the (masked) partition graph is symmetric, the transposed product is the same pull
// with the roles of the two scale vectors exchanged - no atomics, fixed summation order.
// Rows are stored as float32 or bfloat16; sums are always float32.
//
// Three kernels.  Every graph carries its rows sorted by descending degree, hub rows first:
//  * aggregate_hub_kernel (hub rows, AGG_HUB_MIN neighbours and more - the nodes that keep a high degree after
//    the cut, Theorem 2): a workgroup of sixteen wavefronts per (row, column panel); every wavefront sums a
//    strided share of the neighbours, the sixteen partial rows are staged in LDS and added in wavefront order.
//    A launch of its own over the head of the order, when the graph has such rows.
//  All other rows go through one of two kernels, chosen on the host by the graph's average degree:
//  * aggregate_group_kernel (average degree of AGG_LONG_MIN and more): one wavefront per (row, column
//    slice); the 64 lanes form 64/LPS neighbour groups that fetch different neighbours in the same load
//    instruction.
//  * aggregate_kernel (short rows): a group of LANES lanes of a 64-wide wavefront owns one row;
//    one neighbour row is fetched by the group as one contiguous segment of 16 bytes per lane.
//    Column indices are fetched LANES at a time with one coalesced load and handed out by
//    cross-lane reads.
// Rows are handed out by descending degree, so the lane groups of a wavefront get rows of similar length and
// the longest rows start first: below the hub threshold a long row finishes well inside the launch.  (Cutting
// the order further - rows of 16 neighbours and more through the group kernel, the rest through the row
// kernel, each in a launch of its own - was measured and lost 5-8 % to the extra launches on every workload.)
// Which wavefront sums which neighbours is fixed by the launch shape, so results are run-to-run identical.
#include <climits>
#include <cstdio>
#include <cstdlib>
#include <type_traits>

#include "common.h"

namespace cofree {

// ---- typed row access: VEC consecutive elements <-> float registers ---------------------------
typedef float f32x4u __attribute__((ext_vector_type(4), aligned(4)));
typedef uint32_t u32x4u __attribute__((ext_vector_type(4), aligned(2)));

template <typename T>
struct RowIO;

// Raw / load_raw / keep_if / fma_raw: the gather loops load a batch of neighbour segments unconditionally -
// a slot without a neighbour re-reads the batch's first neighbour and is zeroed by keep_if, a lane past the
// end of the row re-reads the row's last window - and only then add them up.  A load under a per-lane
// condition is a branch to the compiler, which then waited for each load before issuing the next one
// (bfloat16 launches of 128-byte rows took twice as long as float32 launches of the same bytes).
template <>
struct RowIO<float> {
  static constexpr int WIDE = 4;  // elements per 16-byte access
  typedef f32x4u Raw;
  __device__ static Raw zero_raw() { return Raw{0.f, 0.f, 0.f, 0.f}; }
  __device__ static Raw load_raw(const float* p) { return *reinterpret_cast<const f32x4u*>(p); }
  __device__ static Raw keep_if(bool ok, const Raw& r) { return Raw{ok ? r[0] : 0.f, ok ? r[1] : 0.f, ok ? r[2] : 0.f, ok ? r[3] : 0.f}; }
  __device__ static void fma_raw(float (&acc)[4], float s, const Raw& r) {
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = fmaf(s, r[i], acc[i]);
  }
  __device__ static void unpack(const Raw& r, float (&v)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = r[i];
  }
  __device__ static void load_wide(const float* p, float (&v)[4]) {
    const f32x4u t = *reinterpret_cast<const f32x4u*>(p);
    v[0] = t[0];
    v[1] = t[1];
    v[2] = t[2];
    v[3] = t[3];
  }
  __device__ static void store_wide(float* p, const float (&v)[4]) {
    f32x4u t;
    t[0] = v[0];
    t[1] = v[1];
    t[2] = v[2];
    t[3] = v[3];
    *reinterpret_cast<f32x4u*>(p) = t;
  }
  __device__ static float load1(const float* p) { return *p; }
  __device__ static void store1(float* p, float x) { *p = x; }
};

template <>
struct RowIO<bf16_t> {
  static constexpr int WIDE = 8;
  typedef u32x4u Raw;
  __device__ static Raw zero_raw() { return Raw{0u, 0u, 0u, 0u}; }
  __device__ static Raw load_raw(const bf16_t* p) { return *reinterpret_cast<const u32x4u*>(p); }
  __device__ static Raw keep_if(bool ok, const Raw& r) { return Raw{ok ? r[0] : 0u, ok ? r[1] : 0u, ok ? r[2] : 0u, ok ? r[3] : 0u}; }
  __device__ static void fma_raw(float (&acc)[8], float s, const Raw& r) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      acc[2 * i] = fmaf(s, __uint_as_float(r[i] << 16), acc[2 * i]);
      acc[2 * i + 1] = fmaf(s, __uint_as_float(r[i] & 0xffff0000u), acc[2 * i + 1]);
    }
  }
  __device__ static void unpack(const Raw& r, float (&v)[8]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __uint_as_float(r[i] << 16);
      v[2 * i + 1] = __uint_as_float(r[i] & 0xffff0000u);
    }
  }
  __device__ static void load_wide(const bf16_t* p, float (&v)[8]) {
    const u32x4u t = *reinterpret_cast<const u32x4u*>(p);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __uint_as_float(t[i] << 16);
      v[2 * i + 1] = __uint_as_float(t[i] & 0xffff0000u);
    }
  }
  __device__ static void store_wide(bf16_t* p, const float (&v)[8]) {
    u32x4u t;
#pragma unroll
    for (int i = 0; i < 4; ++i) t[i] = pack_bf16x2(v[2 * i], v[2 * i + 1]);
    *reinterpret_cast<u32x4u*>(p) = t;
  }
  __device__ static float load1(const bf16_t* p) { return bf16_to_f32(*p); }
  __device__ static void store1(bf16_t* p, float x) { *p = f32_to_bf16(x); }
};

// VEC elements starting at p, of which only the first `avail` exist (avail >= VEC: one wide access)
template <typename T, int VEC>
__device__ inline void load_elems(const T* p, int avail, float (&v)[VEC]) {
  if constexpr (VEC == 1) {
    v[0] = RowIO<T>::load1(p);
  } else {
    if (avail >= VEC) {
      RowIO<T>::load_wide(p, v);
    } else {
#pragma unroll
      for (int i = 0; i < VEC; ++i) v[i] = i < avail ? RowIO<T>::load1(p + i) : 0.f;
    }
  }
}
template <typename T, int VEC>
__device__ inline void store_elems(T* p, int avail, const float (&v)[VEC]) {
  if constexpr (VEC == 1) {
    RowIO<T>::store1(p, v[0]);
  } else {
    if (avail >= VEC) {
      RowIO<T>::store_wide(p, v);
    } else {
#pragma unroll
      for (int i = 0; i < VEC; ++i)
        if (i < avail) RowIO<T>::store1(p + i, v[i]);
    }
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

template <typename T>
struct AggK {
  const int64_t* rowptr;
  const int32_t* col;
  const T* X;
  int64_t ldx;
  T* Y;
  int64_t ldy;
  int width;  // columns of this launch
  int64_t n;
  const int32_t* order;  // short-row kernel: the i-th lane group works on row order[i] (null: row i)
  const int32_t* order_long;  // the same for the long-row kernel's wavefronts
  int64_t slot0;      // first entry of `order` this launch covers (its bucket); n counts the entries from there
  int64_t skip_from;  // rows of at least this many neighbours belong to another launch (natural-order launches)
  // short-row kernel on the processing-order copy of the graph: rowptr, col and in_vals are that copy's, indexed by
  // slot, and the row's own factors come per slot too (null: none, or read by row id from in_scale / out_scale)
  int by_slot;
  const float* in_scale_slot;
  const float* out_scale_slot;
  const float* in_scale;  // per node
  const float* in_vals;   // the same factor per adjacency entry (in_vals[e] = in_scale[col[e]]), or null
  const float* out_scale;
  int self_loop;
  const T* relu_src;
  int64_t ld_relu;
  float gate_scale;  // factor on the elements that pass relu_src
  // output epilogue (after out_scale): + bias, ReLU
  const float* bias;
  int relu_out;
  int col0;  // first column of this launch in the full matrix (bias index)
};

// A lane owns VEC consecutive columns starting at a multiple of VEC.  When the last lane's columns
// would cross the end of a row of at least VEC columns, its window is moved left to end with the row,
// so that every access stays one wide access; the `first` leading columns of the window then belong to
// the lane before it and are not stored.  In rows of at least VEC columns a lane therefore has either a
// full window or none (avail <= 0).  Only rows narrower than VEC (the TINY kernel instances) use
// element accesses.
struct LaneCols {
  int c0;     // first column of the window
  int first;  // leading columns of the window owned by the previous lane (0 unless moved)
  int avail;  // columns of the window that exist (>= VEC unless the whole row is narrower than VEC)
};
template <int VEC>
__device__ inline LaneCols lane_cols(int width, int start) {
  LaneCols l;
  l.c0 = start;
  l.first = 0;
  l.avail = width - start;
  if (l.avail > 0 && l.avail < VEC && width >= VEC) {
    l.c0 = width - VEC;
    l.first = VEC - l.avail;
    l.avail = VEC;
  }
  return l;
}

// Shared tail of both kernels: self term, destination scale, gate, bias, ReLU, store.
// The operands of the tail that depend on the row alone - its own X row, its gate row, its two scales -
// are requested together as soon as the row is known (RowTail::request, all loads back to back, nothing
// uses them yet) and applied after the neighbour sum: fetched one after the other at the end, each with
// its own wait, they added up to three memory round trips to the life of every lane group.
template <typename T, int VEC, bool TINY>
struct RowTail {
  typename RowIO<T>::Raw xs, g;
  float ss, so;
  // cread: first column of the lane's read window (valid memory also for lanes that own nothing); s: the row's
  // slot (used by the launches on the processing-order copy)
  __device__ void request(const AggK<T>& p, int64_t row, int64_t s, int cread) {
    ss = 1.f;
    so = 1.f;
    xs = RowIO<T>::zero_raw();
    g = RowIO<T>::zero_raw();
    if constexpr (!TINY) {
      if (p.out_scale_slot) so = p.out_scale_slot[s];
      else if (p.out_scale) so = p.out_scale[row];
      if (p.self_loop) {
        if (p.in_scale_slot) ss = p.in_scale_slot[s];
        else if (p.in_scale) ss = p.in_scale[row];
        xs = RowIO<T>::load_raw(p.X + row * p.ldx + cread);
      }
      if (p.relu_src) g = RowIO<T>::load_raw(p.relu_src + row * p.ld_relu + cread);
    }
  }
};

template <typename T, int VEC, bool TINY>
__device__ inline void finish_row(const AggK<T>& p, int64_t row, int c0, int first, int avail, float (&acc)[VEC],
                                  const RowTail<T, VEC, TINY>& t) {
  if constexpr (TINY) {
    if (p.self_loop) {
      const float ss = p.in_scale ? p.in_scale[row] : 1.f;
      float xs[VEC];
      load_elems<T, VEC>(p.X + row * p.ldx + c0, avail, xs);
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[i] = fmaf(ss, xs[i], acc[i]);
    }
    const float so = p.out_scale ? p.out_scale[row] : 1.f;
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] *= so;
    if (p.relu_src) {
      float g[VEC];
      load_elems<T, VEC>(p.relu_src + row * p.ld_relu + c0, avail, g);
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[i] = g[i] > 0.f ? acc[i] * p.gate_scale : 0.f;
    }
  } else {
    if (p.self_loop) RowIO<T>::fma_raw(acc, t.ss, t.xs);
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] *= t.so;
    if (p.relu_src) {
      float g[VEC];
      RowIO<T>::unpack(t.g, g);
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[i] = g[i] > 0.f ? acc[i] * p.gate_scale : 0.f;
    }
  }
  if (p.bias) {
#pragma unroll
    for (int i = 0; i < VEC; ++i)
      if (i < avail) acc[i] += p.bias[p.col0 + c0 + i];
  }
  if (p.relu_out) {
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = fmaxf(acc[i], 0.f);
  }
  if (first == 0) {
    if constexpr (TINY) {
      store_elems<T, VEC>(p.Y + row * p.ldy + c0, avail, acc);
    } else {
      RowIO<T>::store_wide(p.Y + row * p.ldy + c0, acc);
    }
  } else {
#pragma unroll
    for (int i = 0; i < VEC; ++i)
      if (i >= first) RowIO<T>::store1(p.Y + row * p.ldy + c0 + i, acc[i]);
  }
}

// ---- short rows ---------------------------------------------------------------------------------
// VEC = RowIO<T>::WIDE.  Rows need only element alignment (see LaneCols for the ragged end of a row).
template <typename T, int VEC, int LANES, int NCH, bool TINY>
__global__ __launch_bounds__(256) void aggregate_kernel(const AggK<T> p) {
  const int64_t* __restrict__ rowptr = p.rowptr;
  const int32_t* __restrict__ col = p.col;
  const T* __restrict__ X = p.X;
  const float* __restrict__ in_scale = p.in_scale;
  const float* __restrict__ in_vals = p.in_vals;
  constexpr int RPW = 64 / LANES;  // rows per wavefront
  constexpr int UNR = 4;
  const int lane = threadIdx.x & 63;
  const int sub = lane % LANES;
  const int grp_base = (lane / LANES) * LANES;
  const int64_t slot = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * RPW + lane / LANES;
  if (slot >= p.n) return;
  const int64_t s = p.slot0 + slot;
  const int64_t row = p.order ? (int64_t)p.order[s] : slot;
  const int64_t at = p.by_slot ? s : row;
  const int64_t beg = rowptr[at], end = rowptr[at + 1];
  if (end - beg >= p.skip_from) return;  // a hub row met in natural order: the hub launch owns it

  float acc[NCH][VEC];
  LaneCols lc[NCH];
  int cread[NCH];  // first column a lane reads in the gather loop (lanes past the end: the row's last window)
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    lc[c] = lane_cols<VEC>(p.width, (sub + c * LANES) * VEC);
    cread[c] = lc[c].avail > 0 ? lc[c].c0 : (p.width >= VEC ? p.width - VEC : 0);
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[c][i] = 0.f;
  }
  RowTail<T, VEC, TINY> tail[NCH];
#pragma unroll
  for (int c = 0; c < NCH; ++c) tail[c].request(p, row, s, cread[c]);

  for (int64_t e0 = beg; e0 < end; e0 += LANES) {
    int my_col = -1;
    float my_s = 1.f;
    if (e0 + sub < end) {
      my_col = col[e0 + sub];
      if (in_vals) my_s = in_vals[e0 + sub];
      else if (in_scale) my_s = in_scale[my_col];
    }
    const int cnt = (int)((end - e0) < (int64_t)LANES ? (end - e0) : (int64_t)LANES);
    for (int j = 0; j < cnt; j += UNR) {
      int u[UNR];
      float s[UNR];
#pragma unroll
      for (int t = 0; t < UNR; ++t) {
        const int jj = (j + t) % LANES;
        u[t] = group_read_i<LANES>(my_col, grp_base, jj);
        s[t] = group_read_f<LANES>(my_s, grp_base, jj);
        if (j + t >= cnt) u[t] = -1;
      }
      if constexpr (TINY) {
        float v[UNR][NCH][VEC];
#pragma unroll
        for (int t = 0; t < UNR; ++t) {
#pragma unroll
          for (int c = 0; c < NCH; ++c) {
#pragma unroll
            for (int i = 0; i < VEC; ++i) v[t][c][i] = 0.f;
            if (u[t] >= 0 && lc[c].avail > 0)
              load_elems<T, VEC>(X + (int64_t)u[t] * p.ldx + lc[c].c0, lc[c].avail, v[t][c]);
          }
        }
#pragma unroll
        for (int t = 0; t < UNR; ++t)
#pragma unroll
          for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[c][i] = fmaf(s[t], v[t][c][i], acc[c][i]);
      } else {
        typename RowIO<T>::Raw v[UNR][NCH];
        const int u_first = group_read_i<LANES>(my_col, grp_base, j % LANES);  // exists: j < cnt
#pragma unroll
        for (int t = 0; t < UNR; ++t) {
          const int64_t src = (int64_t)(u[t] >= 0 ? u[t] : u_first) * p.ldx;
#pragma unroll
          for (int c = 0; c < NCH; ++c) v[t][c] = RowIO<T>::load_raw(X + src + cread[c]);
        }
#pragma unroll
        for (int t = 0; t < UNR; ++t)
#pragma unroll
          for (int c = 0; c < NCH; ++c) RowIO<T>::fma_raw(acc[c], s[t], RowIO<T>::keep_if(u[t] >= 0, v[t][c]));
      }
    }
  }
#pragma unroll
  for (int c = 0; c < NCH; ++c)
    if (lc[c].avail > 0) finish_row<T, VEC, TINY>(p, row, lc[c].c0, lc[c].first, lc[c].avail, acc[c], tail[c]);
}

// ---- long rows ----------------------------------------------------------------------------------
// One wavefront per (row, column slice).  A slice is LPS lanes x VEC elements wide (VEC = 16 bytes
// of elements); the 64 lanes form 64/LPS neighbour groups that fetch different neighbours in the
// same load instruction and are added together at the end in a fixed butterfly order, so a row
// of degree d costs d*LPS/64 load instructions however narrow the matrix is.
// SLICES = 8 is the XCD-aware launch for matrices far larger than one XCD's 4 MB L2: workgroups
// are dealt round-robin to the 8 XCDs, so workgroup b works on column slice b % 8 of row group
// b / 8, and each XCD's L2 only ever holds one eighth of every row - eight times as many (hot)
// rows.  SLICES = 1 covers the whole width (<= LPS*VEC columns) with one slice.
// Rows need only element alignment (see LaneCols for the ragged end of a row).
template <typename T, int LPS, int SLICES, bool TINY>
__global__ __launch_bounds__(256) void aggregate_group_kernel(const AggK<T> p) {
  constexpr int VEC = RowIO<T>::WIDE;
  constexpr int NG = 64 / LPS;
  constexpr int UNR = 4;
  const int lane = threadIdx.x & 63;
  const int sub = lane % LPS, grp = lane / LPS;
  const int slice = SLICES == 1 ? 0 : (int)(blockIdx.x % (unsigned)SLICES);
  const int64_t slot = (int64_t)(blockIdx.x / (unsigned)SLICES) * 4 + (threadIdx.x >> 6);
  if (slot >= p.n) return;
  const int64_t row = p.order_long ? (int64_t)p.order_long[p.slot0 + slot] : slot;
  const LaneCols lc = lane_cols<VEC>(p.width, slice * (LPS * VEC) + sub * VEC);
  const int c0 = lc.c0, avail = lc.avail;
  const T* __restrict__ X = p.X + c0;
  const int32_t* __restrict__ col = p.col;
  const float* __restrict__ in_scale = p.in_scale;
  const float* __restrict__ in_vals = p.in_vals;
  const int64_t beg = p.rowptr[row], end = p.rowptr[row + 1];
  if (end - beg >= p.skip_from) return;  // a hub row met in natural order: the hub launch owns it
  float acc[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
  RowTail<T, VEC, TINY> tail;
  tail.request(p, row, 0, avail > 0 ? c0 : (p.width >= VEC ? p.width - VEC : 0));
  if constexpr (TINY) {
    for (int64_t e = beg + grp; e < end; e += NG * UNR) {
      int u[UNR];
      float s[UNR];
      float v[UNR][VEC];
#pragma unroll
      for (int t = 0; t < UNR; ++t) {
        const int64_t ee = e + t * NG;
        u[t] = ee < end ? col[ee] : -1;
      }
#pragma unroll
      for (int t = 0; t < UNR; ++t) {
        s[t] = 1.f;
#pragma unroll
        for (int i = 0; i < VEC; ++i) v[t][i] = 0.f;
        if (u[t] >= 0 && avail > 0) {
          if (in_vals) s[t] = in_vals[e + t * NG];
          else if (in_scale) s[t] = in_scale[u[t]];
          load_elems<T, VEC>(X + (int64_t)u[t] * p.ldx, avail, v[t]);
        }
      }
#pragma unroll
      for (int t = 0; t < UNR; ++t)
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] = fmaf(s[t], v[t][i], acc[i]);
    }
  } else {
    // every load of the loop is unconditional (see RowIO): ids past the end of the row repeat its last id
    // and are zeroed after the load; lanes past the end of the matrix row re-read its last window
    const T* __restrict__ Xread = p.X + (avail > 0 ? c0 : p.width - VEC);
    // scale_mode: 0 no per-source factor, 1 gathered from the per-node vector, 2 read per entry next to col
    auto gather = [&](auto scale_mode) {
      constexpr int MODE = decltype(scale_mode)::value;
      const int64_t last = end - 1;
      for (int64_t e = beg + grp; e < end; e += NG * UNR) {
        int u[UNR];
        float s[UNR];
        typename RowIO<T>::Raw v[UNR];
#pragma unroll
        for (int t = 0; t < UNR; ++t) {
          const int64_t ee = e + t * NG;
          const int64_t ec = ee < last ? ee : last;
          u[t] = col[ec];
          if constexpr (MODE == 2) s[t] = in_vals[ec];
        }
#pragma unroll
        for (int t = 0; t < UNR; ++t) {
          if constexpr (MODE == 1) s[t] = in_scale[u[t]];
          if constexpr (MODE == 0) s[t] = 1.f;
          v[t] = RowIO<T>::load_raw(Xread + (int64_t)u[t] * p.ldx);
        }
#pragma unroll
        for (int t = 0; t < UNR; ++t) RowIO<T>::fma_raw(acc, s[t], RowIO<T>::keep_if(e + t * NG < end, v[t]));
      }
    };
    if (in_vals) gather(std::integral_constant<int, 2>{});
    else if (in_scale) gather(std::integral_constant<int, 1>{});
    else gather(std::integral_constant<int, 0>{});
  }
#pragma unroll
  for (int off = LPS; off < 64; off <<= 1) {
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] += __shfl_xor(acc[i], off, 64);
  }
  if (grp != 0 || avail <= 0) return;
  finish_row<T, VEC, TINY>(p, row, c0, lc.first, avail, acc, tail);
}

// ---- hub rows -----------------------------------------------------------------------------------
// One workgroup of HUB_WAVES wavefronts per (row, column panel of LPS lanes x 16 bytes).  Inside a wavefront the
// lanes form 64/LPS neighbour groups as in the long-row kernel; neighbour j of the row goes to wavefront
// (j / NG) % HUB_WAVES, group j % NG, so that consecutive ids - one coalesced read - feed one wavefront's load
// instruction.  The groups of a wavefront are added by the same butterfly, then wavefront w > 0 writes its
// partial panel to LDS and wavefront 0 adds the partials in ascending w: a fixed order.
constexpr int HUB_WAVES = 16;
template <typename T, int LPS>
__global__ __launch_bounds__(HUB_WAVES * 64) void aggregate_hub_kernel(const AggK<T> p) {
  constexpr int VEC = RowIO<T>::WIDE;
  constexpr int NG = 64 / LPS;
  constexpr int UNR = 4;
  __shared__ float partial[HUB_WAVES - 1][LPS * VEC];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPS, grp = lane / LPS;
  const int64_t row = (int64_t)p.order[p.slot0 + blockIdx.x];
  const LaneCols lc = lane_cols<VEC>(p.width, (int)blockIdx.y * (LPS * VEC) + sub * VEC);
  const int c0 = lc.c0, avail = lc.avail;
  const int cread = avail > 0 ? c0 : p.width - VEC;  // the launcher sends only rows of at least VEC columns here
  const int32_t* __restrict__ col = p.col;
  const float* __restrict__ in_scale = p.in_scale;
  const float* __restrict__ in_vals = p.in_vals;
  const T* __restrict__ Xread = p.X + cread;
  const int64_t beg = p.rowptr[row], end = p.rowptr[row + 1];
  float acc[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
  RowTail<T, VEC, false> tail;
  if (wave == 0) tail.request(p, row, 0, cread);
  if (end > beg) {
    const int64_t last = end - 1;
    // step of one wavefront: NG neighbours; of the workgroup: NG * HUB_WAVES; UNR steps in flight
    for (int64_t e = beg + (int64_t)wave * NG + grp; e < end; e += (int64_t)NG * HUB_WAVES * UNR) {
      int u[UNR];
      float sc[UNR];
      typename RowIO<T>::Raw v[UNR];
#pragma unroll
      for (int t = 0; t < UNR; ++t) {
        const int64_t ee = e + (int64_t)t * NG * HUB_WAVES;
        const int64_t ec = ee < last ? ee : last;
        u[t] = col[ec];
        sc[t] = in_vals ? in_vals[ec] : 1.f;
      }
#pragma unroll
      for (int t = 0; t < UNR; ++t) {
        if (!in_vals && in_scale) sc[t] = in_scale[u[t]];
        v[t] = RowIO<T>::load_raw(Xread + (int64_t)u[t] * p.ldx);
      }
#pragma unroll
      for (int t = 0; t < UNR; ++t)
        RowIO<T>::fma_raw(acc, sc[t], RowIO<T>::keep_if(e + (int64_t)t * NG * HUB_WAVES < end, v[t]));
    }
  }
#pragma unroll
  for (int off = LPS; off < 64; off <<= 1) {
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] += __shfl_xor(acc[i], off, 64);
  }
  if (wave > 0 && grp == 0) {
#pragma unroll
    for (int i = 0; i < VEC; ++i) partial[wave - 1][sub * VEC + i] = acc[i];
  }
  __syncthreads();
  if (wave != 0 || grp != 0 || avail <= 0) return;
  for (int w = 0; w < HUB_WAVES - 1; ++w) {
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] += partial[w][sub * VEC + i];
  }
  finish_row<T, VEC, false>(p, row, c0, lc.first, avail, acc, tail);
}

// ---- host side ------------------------------------------------------------------------------------
template <typename T>
static const char* type_name() {
  return sizeof(T) == 4 ? "float" : "bf16";
}

// One launch = one timing record, named by the kernel's template instance and the launch's shape.  Algorithmic
// traffic of a launch over `rows` rows with `nnz` adjacency entries: every source row read once and every output
// row written once (`rows` each: the sources of a bucket's rows are as many again at this graph's symmetry only on
// average, so the bucket is charged its own row count), 4 bytes per entry, 8 per row offset, the per-node scale
// vectors and the gate matrix once.
template <typename T>
struct LaunchCost {
  const AggArgs& a;
  const T* R;
  double bytes(int64_t rows, int64_t nnz) const {
    return 2.0 * (double)rows * a.width * sizeof(T) + 4.0 * (double)nnz + 8.0 * (double)(rows + 1) +
           4.0 * (double)rows * ((a.in_scale ? 1 : 0) + (a.out_scale ? 1 : 0)) +
           (R ? (double)rows * a.width * sizeof(T) : 0.0);
  }
  double flops(int64_t nnz) const { return 2.0 * (double)nnz * a.width; }
};

template <typename T, int VEC, int LANES, int NCH>
static void launch_rows(const AggK<T>& k, hipStream_t stream, const LaunchCost<T>& cost, int64_t nnz) {
  constexpr int rows_per_block = 4 * (64 / LANES);
  const int64_t blocks = (k.n + rows_per_block - 1) / rows_per_block;
  const bool tiny = LANES == 16 && NCH == 1 && k.width < VEC;  // rows narrower than one wide access
  char pname[96];
  snprintf(pname, sizeof(pname), "aggregate_kernel<%s,%d,%d,%d,%s> width=%d", type_name<T>(), VEC, LANES, NCH,
           tiny ? "true" : "false", (int)cost.a.width);
  ProfScope prof(pname, stream, cost.bytes(k.n, nnz), cost.flops(nnz));
  if constexpr (LANES == 16 && NCH == 1) {
    if (tiny) {
      aggregate_kernel<T, VEC, LANES, NCH, true><<<dim3((unsigned)blocks), 256, 0, stream>>>(k);
      return;
    }
  }
  aggregate_kernel<T, VEC, LANES, NCH, false><<<dim3((unsigned)blocks), 256, 0, stream>>>(k);
}

template <typename T, int VEC>
static int32_t dispatch_rows(const AggK<T>& k, hipStream_t stream, const LaunchCost<T>& cost, int64_t nnz) {
  const int chunks = (k.width + VEC - 1) / VEC;
  // at most four rows per wavefront: with more, narrow rows measured slower (8 rows of 6 chunks: 0.50 ms,
  // 4 rows with idle lanes: 0.41 ms on the 47-wide bf16 launches of cfg2)
  if (chunks <= 16) launch_rows<T, VEC, 16, 1>(k, stream, cost, nnz);
  else if (chunks <= 32) launch_rows<T, VEC, 32, 1>(k, stream, cost, nnz);
  else if (chunks <= 64) launch_rows<T, VEC, 64, 1>(k, stream, cost, nnz);
  else if (chunks <= 128) launch_rows<T, VEC, 64, 2>(k, stream, cost, nnz);
  else return fail(COFREE_EINVAL, "internal: aggregate panel too wide");
  return COFREE_OK;
}

template <typename T, int SLICES>
static int32_t launch_group(const AggK<T>& k, int lps, hipStream_t stream, const LaunchCost<T>& cost, int64_t nnz) {
  const int64_t blocks = ((k.n + 3) / 4) * SLICES;
  COFREE_REQUIRE(blocks < ((int64_t)1 << 31), "aggregate: grid too large");
  const dim3 grid((unsigned)blocks);
  const bool tiny = lps == 1 && k.width < RowIO<T>::WIDE;
  char pname[96];
  snprintf(pname, sizeof(pname), "aggregate_group_kernel<%s,%d,%d,%s> width=%d", type_name<T>(), lps, SLICES,
           tiny ? "true" : "false", (int)cost.a.width);
  ProfScope prof(pname, stream, cost.bytes(k.n, nnz), cost.flops(nnz));
  switch (lps) {
    case 1:
      if (tiny) aggregate_group_kernel<T, 1, SLICES, true><<<grid, 256, 0, stream>>>(k);
      else aggregate_group_kernel<T, 1, SLICES, false><<<grid, 256, 0, stream>>>(k);
      break;
    case 2: aggregate_group_kernel<T, 2, SLICES, false><<<grid, 256, 0, stream>>>(k); break;
    case 4: aggregate_group_kernel<T, 4, SLICES, false><<<grid, 256, 0, stream>>>(k); break;
    case 8: aggregate_group_kernel<T, 8, SLICES, false><<<grid, 256, 0, stream>>>(k); break;
    case 16: aggregate_group_kernel<T, 16, SLICES, false><<<grid, 256, 0, stream>>>(k); break;
    case 32: aggregate_group_kernel<T, 32, SLICES, false><<<grid, 256, 0, stream>>>(k); break;
    case 64: aggregate_group_kernel<T, 64, SLICES, false><<<grid, 256, 0, stream>>>(k); break;
    default: return fail(COFREE_EINVAL, "internal: bad lanes-per-slice");
  }
  return COFREE_OK;
}

// hub rows: order[0 .. n_hub), one workgroup per (row, panel of lps lanes x 16 bytes)
template <typename T>
static int32_t launch_hub(const AggK<T>& k, hipStream_t stream, const LaunchCost<T>& cost, int64_t nnz) {
  constexpr int WIDE = RowIO<T>::WIDE;
  int lps = 1;
  while (lps < 64 && lps * WIDE < k.width) lps *= 2;
  const int panels = (k.width + lps * WIDE - 1) / (lps * WIDE);
  COFREE_REQUIRE(k.n < ((int64_t)1 << 31) && panels < 65536, "aggregate: hub grid too large");
  const dim3 grid((unsigned)k.n, (unsigned)panels);
  char pname[96];
  snprintf(pname, sizeof(pname), "aggregate_hub_kernel<%s,%d> width=%d", type_name<T>(), lps, (int)cost.a.width);
  ProfScope prof(pname, stream, cost.bytes(k.n, nnz), cost.flops(nnz));
  switch (lps) {
    case 1: aggregate_hub_kernel<T, 1><<<grid, HUB_WAVES * 64, 0, stream>>>(k); break;
    case 2: aggregate_hub_kernel<T, 2><<<grid, HUB_WAVES * 64, 0, stream>>>(k); break;
    case 4: aggregate_hub_kernel<T, 4><<<grid, HUB_WAVES * 64, 0, stream>>>(k); break;
    case 8: aggregate_hub_kernel<T, 8><<<grid, HUB_WAVES * 64, 0, stream>>>(k); break;
    case 16: aggregate_hub_kernel<T, 16><<<grid, HUB_WAVES * 64, 0, stream>>>(k); break;
    case 32: aggregate_hub_kernel<T, 32><<<grid, HUB_WAVES * 64, 0, stream>>>(k); break;
    default: aggregate_hub_kernel<T, 64><<<grid, HUB_WAVES * 64, 0, stream>>>(k); break;
  }
  return COFREE_OK;
}

template <typename T>
static int32_t launch_typed(const AggArgs& a, hipStream_t stream) {
  constexpr int WIDE = RowIO<T>::WIDE;
  const T* X = (const T*)a.X;
  T* Y = (T*)a.Y;
  const T* R = (const T*)a.relu_src;
  AggK<T> k{};
  k.rowptr = a.g.rowptr;
  k.col = a.g.col;
  k.ldx = a.ldx;
  k.ldy = a.ldy;
  k.in_scale = a.in_scale;
  // Per-source factors of a large graph are read per entry: the per-node vector no longer stays in L2 there, and
  // every neighbour's factor would cost a memory access of its own beside the row it scales (28M-node partition,
  // 256-wide bfloat16 launch: 16.7 ms with the per-node gather, 15.9 ms with the per-entry stream; no difference
  // at 1.9M nodes).  COFREE_AGG_ENTRY_SCALE = 0 / 1 forces one or the other.
  k.in_vals = nullptr;
  if (a.in_scale) {
    bool per_entry = a.g.n >= AGG_ENTRY_SCALE_MIN_NODES;
    if (const char* env = getenv("COFREE_AGG_ENTRY_SCALE")) per_entry = atoi(env) != 0;
    if (per_entry && a.in_scale == a.g.inv_deg) k.in_vals = a.g.val_inv_deg;
    if (per_entry && a.in_scale == a.g.gcn_norm) k.in_vals = a.g.val_gcn_norm;
  }
  k.out_scale = a.out_scale;
  k.self_loop = a.self_loop;
  k.ld_relu = a.ld_relu;
  k.gate_scale = a.gate_scale;
  k.bias = a.bias;
  k.relu_out = a.relu_out;
  k.width = a.width;
  k.col0 = 0;
  k.X = X;
  k.Y = Y;
  k.relu_src = R;
  k.skip_from = INT64_MAX;
  const LaunchCost<T> cost{a, R};

  // Hub rows (the head of the sorted row order) get a launch of their own.  COFREE_AGG_BUCKETS = 0 leaves
  // them to the kernel that takes every other row.
  bool buckets = a.g.order != nullptr && a.width >= WIDE;
  if (const char* env = getenv("COFREE_AGG_BUCKETS")) buckets = buckets && atoi(env) != 0;
  const int64_t n_hub = buckets ? a.g.n_hub : 0;
  const int64_t hub_nnz = n_hub > 0 ? a.g.nnz_hub : 0;

  // High average degree: the neighbour-group kernel.  Additionally cut into 8 XCD-affine column
  // slices when the matrix is far larger than one XCD's 4 MB L2 and the width divides evenly into
  // slices of at least one 128-byte cache line of float32: a gather costs a compute unit about the same
  // per line request whatever part of the line is used, so narrower slices only multiply the requests
  // (230k x 128 float32, average degree 61: 1.35 ms in 64-byte slices, 0.87 ms unsliced), and for
  // bfloat16 rows the unsliced kernel measured faster at every width (512 wide: 1.73 against 2.13 ms).
  const int slice_unit = 8 * WIDE;  // 8 slices of at least one 16-byte lane each
  const bool dense_rows = a.g.nnz / a.g.n >= AGG_LONG_MIN;
  const bool sliceable = a.width % slice_unit == 0 && a.width / slice_unit <= 64 &&
                         ((a.width / slice_unit) & (a.width / slice_unit - 1)) == 0 &&
                         sizeof(T) == 4 && a.width / slice_unit >= 8;
  const bool groupable = a.width <= 64 * WIDE;
  bool grouped = dense_rows && groupable;
  bool sliced = dense_rows && sliceable && (double)a.g.n * a.width * sizeof(T) > 32e6;
  if (const char* env = getenv("COFREE_AGG_SLICES")) {  // tuning override: 0 = row kernel, 1 = grouped, 8 = sliced
    const int v = atoi(env);
    if (v == 0) grouped = sliced = false;
    if (v == 1) {
      grouped = groupable;
      sliced = false;
    }
    if (v == 8) sliced = sliceable;
  }
  int lps = 1;
  while (lps * WIDE < a.width && lps < 64) lps *= 2;

  // 1. hub rows
  if (n_hub > 0) {
    k.order = a.g.order;
    k.slot0 = 0;
    k.n = n_hub;
    COFREE_TRY(launch_hub<T>(k, stream, cost, a.g.nnz_hub));
  }
  if (sliced) {
    // 2a. every other row in natural order (which measured better for the sliced launch): hub rows are met
    //     and skipped
    k.order = k.order_long = nullptr;
    k.slot0 = 0;
    k.n = a.g.n;
    k.skip_from = n_hub > 0 ? AGG_HUB_MIN : INT64_MAX;
    COFREE_TRY((launch_group<T, 8>(k, a.width / slice_unit, stream, cost, a.g.nnz - hub_nnz)));
    COFREE_HIP_CHECK(hipGetLastError());
    return COFREE_OK;
  }
  // 2b. every other row, order[n_hub ..): the neighbour-group kernel or the row kernel
  if (n_hub == a.g.n) {
    COFREE_HIP_CHECK(hipGetLastError());
    return COFREE_OK;
  }
  k.slot0 = n_hub;
  k.n = a.g.n - n_hub;
  if (grouped) {
    k.order = nullptr;
    k.order_long = a.g.order;
    COFREE_TRY((launch_group<T, 1>(k, lps, stream, cost, a.g.nnz - hub_nnz)));
  } else {
    k.order_long = nullptr;
    k.order = a.g.order;
    // The row kernel walks the processing-order copy of the graph (1.9M-node partition, 512-wide float32: 3.00 ms
    // by row id, 2.8 ms in natural order with its worse balance).  COFREE_AGG_SLOTS = 0 reads by row id.
    bool slots = a.g.order != nullptr && a.g.s_rowptr != nullptr;
    if (const char* env = getenv("COFREE_AGG_SLOTS")) slots = slots && atoi(env) != 0;
    if (slots) {
      k.by_slot = 1;
      k.rowptr = a.g.s_rowptr;
      k.col = a.g.s_col;
      if (k.in_vals) k.in_vals = a.in_scale == a.g.inv_deg ? a.g.s_val_inv_deg : a.g.s_val_gcn_norm;
      if (a.in_scale == a.g.inv_deg) k.in_scale_slot = a.g.s_inv_deg;
      if (a.in_scale == a.g.gcn_norm) k.in_scale_slot = a.g.s_gcn_norm;
      if (a.out_scale == a.g.inv_deg) k.out_scale_slot = a.g.s_inv_deg;
      if (a.out_scale == a.g.gcn_norm) k.out_scale_slot = a.g.s_gcn_norm;
    }
    const int panel = 128 * WIDE;  // columns one launch covers
    for (int c0 = 0; c0 < a.width; c0 += panel) {
      k.width = a.width - c0 < panel ? a.width - c0 : panel;
      k.col0 = c0;
      k.X = X + c0;
      k.Y = Y + c0;
      k.relu_src = R ? R + c0 : nullptr;
      COFREE_TRY((dispatch_rows<T, WIDE>(k, stream, cost, a.g.nnz - hub_nnz)));
    }
  }
  COFREE_HIP_CHECK(hipGetLastError());
  return COFREE_OK;
}

int32_t launch_aggregate(const AggArgs& a, hipStream_t stream) {
  COFREE_REQUIRE(a.dtype == COFREE_F32 || a.dtype == COFREE_BF16, "aggregate: unknown dtype");
  COFREE_REQUIRE(a.width >= 1, "aggregate: width must be >= 1");
  COFREE_REQUIRE(a.X && a.Y && a.X != a.Y, "aggregate: X and Y must be distinct non-NULL buffers");
  COFREE_REQUIRE(a.ldx >= a.width && a.ldy >= a.width, "aggregate: leading dimension smaller than width");
  COFREE_REQUIRE(a.g.n < ((int64_t)1 << 31), "aggregate: too many rows");
  if (a.g.n == 0) return COFREE_OK;
  if (a.dtype == COFREE_F32) return launch_typed<float>(a, stream);
  return launch_typed<bf16_t>(a, stream);
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
