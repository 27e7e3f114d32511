// Reweighted loss (Eq. 3), parameter update (Algorithm 1 line 11) and the small streaming
// kernels of backward (bias gradients, activation / dropout gates).
#include <cmath>
#include <mutex>

#include "common.h"

namespace cofree {

__device__ inline float ld_elem(const float* p) { return *p; }
__device__ inline float ld_elem(const bf16_t* p) { return bf16_to_f32(*p); }
__device__ inline void st_elem(float* p, float x) { *p = x; }
__device__ inline void st_elem(bf16_t* p, float x) { *p = f32_to_bf16(x); }

// four consecutive elements (contiguous matrices whose base is 16-byte aligned: quad q starts at 4q)
__device__ inline void ld_quad(const float* p, float (&v)[4]) {
  const float4 t = *reinterpret_cast<const float4*>(p);
  v[0] = t.x, v[1] = t.y, v[2] = t.z, v[3] = t.w;
}
__device__ inline void ld_quad(const bf16_t* p, float (&v)[4]) {
  const uint2 t = *reinterpret_cast<const uint2*>(p);
  v[0] = __uint_as_float(t.x << 16), v[1] = __uint_as_float(t.x & 0xffff0000u);
  v[2] = __uint_as_float(t.y << 16), v[3] = __uint_as_float(t.y & 0xffff0000u);
}
__device__ inline void st_quad(float* p, const float (&v)[4]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
}
__device__ inline void st_quad(bf16_t* p, const float (&v)[4]) {
  *reinterpret_cast<uint2*>(p) = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
}

// four consecutive elements at any element-aligned address, of which only the first `avail` exist:
// one 16-byte (float32) / 8-byte (bfloat16) access when all four do
typedef float f32x4e __attribute__((ext_vector_type(4), aligned(4)));
typedef uint32_t u32x2e __attribute__((ext_vector_type(2), aligned(2)));
__device__ inline void ld4(const float* p, int avail, float (&v)[4], float fill) {
  if (avail >= 4) {
    const f32x4e t = *reinterpret_cast<const f32x4e*>(p);
    v[0] = t[0], v[1] = t[1], v[2] = t[2], v[3] = t[3];
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = i < avail ? p[i] : fill;
  }
}
__device__ inline void ld4(const bf16_t* p, int avail, float (&v)[4], float fill) {
  if (avail >= 4) {
    const u32x2e t = *reinterpret_cast<const u32x2e*>(p);
    v[0] = __uint_as_float(t[0] << 16), v[1] = __uint_as_float(t[0] & 0xffff0000u);
    v[2] = __uint_as_float(t[1] << 16), v[3] = __uint_as_float(t[1] & 0xffff0000u);
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = i < avail ? bf16_to_f32(p[i]) : fill;
  }
}
__device__ inline void st4(float* p, int avail, const float (&v)[4]) {
  if (avail >= 4) {
    f32x4e t;
    t[0] = v[0], t[1] = v[1], t[2] = v[2], t[3] = v[3];
    *reinterpret_cast<f32x4e*>(p) = t;
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (i < avail) p[i] = v[i];
  }
}
__device__ inline void st4(bf16_t* p, int avail, const float (&v)[4]) {
  if (avail >= 4) {
    u32x2e t;
    t[0] = pack_bf16x2(v[0], v[1]);
    t[1] = pack_bf16x2(v[2], v[3]);
    *reinterpret_cast<u32x2e*>(p) = t;
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (i < avail) p[i] = f32_to_bf16(v[i]);
  }
}

// the same for eight bfloat16 elements (one 16-byte access when all eight exist)
typedef uint32_t u32x4e __attribute__((ext_vector_type(4), aligned(2)));
__device__ inline void ld_n(const float* p, int avail, float (&v)[4], float fill) { ld4(p, avail, v, fill); }
__device__ inline void st_n(float* p, int avail, const float (&v)[4]) { st4(p, avail, v); }
__device__ inline void ld_n(const bf16_t* p, int avail, float (&v)[8], float fill) {
  if (avail >= 8) {
    const u32x4e t = *reinterpret_cast<const u32x4e*>(p);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __uint_as_float(t[i] << 16);
      v[2 * i + 1] = __uint_as_float(t[i] & 0xffff0000u);
    }
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = i < avail ? bf16_to_f32(p[i]) : fill;
  }
}
__device__ inline void st_n(bf16_t* p, int avail, const float (&v)[8]) {
  if (avail >= 8) {
    u32x4e t;
#pragma unroll
    for (int i = 0; i < 4; ++i) t[i] = pack_bf16x2(v[2 * i], v[2 * i + 1]);
    *reinterpret_cast<u32x4e*>(p) = t;
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (i < avail) p[i] = f32_to_bf16(v[i]);
  }
}

constexpr int LOSS_BLOCKS = 2048;  // partial sums; the final reduction runs over exactly this many

// Partial sums of cofree_loss_weighted_static: device memory that exists from the moment the library is loaded
// (one copy per GPU, 8 KiB, held until the process ends), so that the call never allocates.  In host code this
// name is only a handle for hipGetSymbolAddress; kernels receive the address that call returns.
static __device__ __align__(256) float scratch[LOSS_BLOCKS];

__device__ inline float wave_max(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
  return x;
}
__device__ inline float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}

// One wavefront per node: softmax over its C logits (lanes stride over classes), cross-entropy
// against the label, times c * w_j; dlogits = c * w_j * (softmax - onehot).  Each block adds up
// its wavefronts' losses in a fixed order into partial[blockIdx.x].
template <typename T>
__global__ __launch_bounds__(256) void loss_kernel(const T* __restrict__ logits,
                                                   const int32_t* __restrict__ labels,
                                                   const float* __restrict__ w,
                                                   const uint8_t* __restrict__ train_mask, int64_t n, int32_t C,
                                                   float scale_c, T* __restrict__ dlogits,
                                                   float* __restrict__ partial) {
  __shared__ float wave_loss[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float my_loss = 0.f;
  for (int64_t row = (int64_t)blockIdx.x * 4 + wave; row < n; row += (int64_t)gridDim.x * 4) {
    const T* z = logits + row * C;
    float m = -INFINITY;
    for (int c = lane; c < C; c += 64) m = fmaxf(m, ld_elem(z + c));
    m = wave_max(m);
    float se = 0.f;
    for (int c = lane; c < C; c += 64) se += expf(ld_elem(z + c) - m);
    se = wave_sum(se);
    float wj = w ? w[row] : 1.f;
    if (train_mask && train_mask[row] == 0) wj = 0.f;
    int32_t y = labels[row];
    if ((uint32_t)y >= (uint32_t)C) {  // label outside [0, C): the node does not contribute
      y = 0;
      wj = 0.f;
    }
    const float coef = scale_c * wj;
    const float inv = 1.f / se;
    T* dz = dlogits + row * C;
    for (int c = lane; c < C; c += 64) {
      const float pr = expf(ld_elem(z + c) - m) * inv;
      st_elem(dz + c, coef * (pr - (c == y ? 1.f : 0.f)));
    }
    if (lane == 0) my_loss += coef * (m + logf(se) - ld_elem(z + y));
  }
  if (lane == 0) wave_loss[wave] = my_loss;
  __syncthreads();
  if (threadIdx.x == 0) partial[blockIdx.x] = (wave_loss[0] + wave_loss[1]) + (wave_loss[2] + wave_loss[3]);
}

// e^x for x <= 0.  bfloat16 logits: the hardware's 2^x on x log2(e) (relative error about |x| 2^-24, far below
// the 2^-9 of the stored gradient); the library routine's range handling made the kernel issue-bound (172
// classes: 8.4 ms a launch over 28M nodes at 8 bytes per lane, 6.9 ms at 16 bytes, 5.5 ms with this).
// float32 logits keep expf.
template <typename T>
__device__ inline float softmax_exp(float x) {
  if constexpr (sizeof(T) == 2) return __builtin_amdgcn_exp2f(x * 1.44269504088896341f);
  else return expf(x);
}

// Same computation for C <= PER * LANES with a group of LANES lanes per node (LANES a power of two dividing
// 64): lane l of the group owns the PER consecutive classes PER l .. PER l + PER - 1 - 16 bytes of them, four
// float32 or eight bfloat16 - read and written with one wide access (narrower loads per lane are bound by
// the rate of load instructions, not by bytes: 172 bfloat16 classes in 8-byte pieces, one node per
// wavefront, ran at 2.3 TB/s); a wavefront works on 64/LANES nodes at once and on two of them per group and
// iteration (four measured slower), so that the loads of independent rows overlap.
// WIDE (C >= PER): a lane whose classes would cross the end of the row - or lie past it - reads the
// window that ends with the row instead and ignores the `skip` leading classes that belong to the lane
// before, so that every lane issues the same unconditional wide load and store in the loop (a per-lane
// width branch around the loads made the loop wait for each row in turn); the overlapped classes are
// written twice with identical values.
template <typename T, int LANES, bool WIDE>
__device__ inline void loss_group_rows(const T* __restrict__ logits, const int32_t* __restrict__ labels,
                                       const float* __restrict__ w, const uint8_t* __restrict__ train_mask,
                                       int64_t n, int32_t C, float scale_c, T* __restrict__ dlogits, float& my_loss) {
  constexpr int GROUPS = 256 / LANES, R = 2, PER = 16 / (int)sizeof(T);
  const int gl = threadIdx.x % LANES, grp = threadIdx.x / LANES;
  int c0 = gl * PER, avail = C - c0, skip = 0;  // this lane's classes (avail <= 0: none)
  if (WIDE && avail < PER) {
    skip = avail > 0 ? PER - avail : PER;
    c0 = C - PER;
    avail = PER;
  }
  // a workgroup owns one contiguous run of rows and walks it front to back, GROUPS * R consecutive rows per
  // iteration, so that rows sharing a cache line at their ends (rows are C elements long, any C) are handled
  // by the same workgroup close in time (timing equal to a grid-strided walk at 28M rows of 172 bfloat16)
  const int64_t per_block = (n + gridDim.x - 1) / gridDim.x;
  const int64_t b0 = (int64_t)blockIdx.x * per_block, b1 = b0 + per_block < n ? b0 + per_block : n;
  constexpr int64_t stride = GROUPS;
  for (int64_t row0 = b0 + grp; row0 < b1; row0 += R * stride) {
    float v[R][PER];
    bool valid[R];
    int64_t rows[R];
    float wjs[R];
    int32_t ys[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      valid[r] = row0 + r * stride < b1;
      rows[r] = valid[r] ? row0 + r * stride : row0;  // a row past the end is computed on row0 and not stored
      // label and weight are requested with the logits, not after the reductions
      wjs[r] = w ? w[rows[r]] : 1.f;
      if (train_mask && train_mask[rows[r]] == 0) wjs[r] = 0.f;
      ys[r] = labels[rows[r]];
      if (WIDE) {
        ld_n(logits + rows[r] * C + c0, PER, v[r], -INFINITY);
      } else if (avail > 0) {
        ld_n(logits + rows[r] * C + c0, avail, v[r], -INFINITY);
      } else {
#pragma unroll
        for (int k = 0; k < PER; ++k) v[r][k] = -INFINITY;
      }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      float m = -INFINITY;
#pragma unroll
      for (int k = 0; k < PER; ++k) m = fmaxf(m, k >= skip ? v[r][k] : -INFINITY);
#pragma unroll
      for (int o = LANES / 2; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
      // e[k] of a skipped class is the value its owner computes (same logit, same maximum); it only
      // stays out of this lane's share of the sum
      float e[PER], se = 0.f;
#pragma unroll
      for (int k = 0; k < PER; ++k) {
        e[k] = k < avail ? softmax_exp<T>(v[r][k] - m) : 0.f;
        se += k >= skip ? e[k] : 0.f;
      }
#pragma unroll
      for (int o = LANES / 2; o > 0; o >>= 1) se += __shfl_xor(se, o, 64);
      const int64_t row = rows[r];
      float wj = wjs[r];
      int32_t y = ys[r];
      if ((uint32_t)y >= (uint32_t)C) {  // label outside [0, C): the node does not contribute
        y = 0;
        wj = 0.f;
      }
      const float coef = scale_c * wj;
      const float inv = 1.f / se;
      float zy = 0.f;
      if (WIDE) {
        // the label's logit is in a register of the lane that owns class y: element y - c0 of its window
        const int owner = y / PER;                                   // same in every lane of the group
        const int oc0 = C - owner * PER < PER ? C - PER : owner * PER;  // that lane's (possibly moved) window
        const int k = y - oc0;
        float mine = v[r][0];
#pragma unroll
        for (int i = 1; i < PER; ++i) mine = k == i ? v[r][i] : mine;
        zy = __shfl(mine, (threadIdx.x & 63) - gl + owner, 64);
      }
      if (valid[r]) {
        if (WIDE) {
          float g[PER];
#pragma unroll
          for (int k = 0; k < PER; ++k) g[k] = coef * (e[k] * inv - (c0 + k == y ? 1.f : 0.f));
          st_n(dlogits + row * C + c0, PER, g);
        } else if (avail > 0) {
          float g[PER];
#pragma unroll
          for (int k = 0; k < PER; ++k) g[k] = coef * (e[k] * inv - (c0 + k == y ? 1.f : 0.f));
          st_n(dlogits + row * C + c0, avail, g);
        }
        if (gl == 0) my_loss += coef * (m + logf(se) - (WIDE ? zy : ld_elem(logits + row * C + y)));
      }
    }
  }
}

template <typename T, int LANES>
__global__ __launch_bounds__(256) void loss_group_kernel(const T* __restrict__ logits,
                                                         const int32_t* __restrict__ labels,
                                                         const float* __restrict__ w,
                                                         const uint8_t* __restrict__ train_mask, int64_t n, int32_t C,
                                                         float scale_c, T* __restrict__ dlogits,
                                                         float* __restrict__ partial) {
  constexpr int GROUPS = 256 / LANES;
  __shared__ float group_loss[GROUPS];
  const int gl = threadIdx.x % LANES, grp = threadIdx.x / LANES;
  float my_loss = 0.f;
  if (C >= 16 / (int)sizeof(T))
    loss_group_rows<T, LANES, true>(logits, labels, w, train_mask, n, C, scale_c, dlogits, my_loss);
  else
    loss_group_rows<T, LANES, false>(logits, labels, w, train_mask, n, C, scale_c, dlogits, my_loss);
  if (gl == 0) group_loss[grp] = my_loss;
  __syncthreads();
  if (threadIdx.x == 0) {
    float t = 0.f;
    for (int i = 0; i < GROUPS; ++i) t += group_loss[i];
    partial[blockIdx.x] = t;
  }
}

// Multi-label loss (the sigmoid + binary cross-entropy of Theorem 3): one thread per (node, class)
// element, grid-stride.  loss element = softplus(z) - y z with softplus(z) = max(z, 0) + log1p(e^-|z|);
// dlogits = c w_j (sigmoid(z) - y).  Per-thread sums in index order, then the fixed wavefront / block tree.
template <typename T>
__global__ __launch_bounds__(256) void bce_kernel(const T* __restrict__ logits, const uint8_t* __restrict__ targets,
                                                  const float* __restrict__ w,
                                                  const uint8_t* __restrict__ train_mask, int64_t n, int32_t C,
                                                  float scale_c, T* __restrict__ dlogits,
                                                  float* __restrict__ partial) {
  __shared__ float wave_loss[4];
  const int64_t total = n * C;
  const int64_t stride = (int64_t)gridDim.x * 256;
  float my_loss = 0.f;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += stride) {
    const int64_t row = i / C;
    float wj = w ? w[row] : 1.f;
    if (train_mask && train_mask[row] == 0) wj = 0.f;
    const float coef = scale_c * wj;
    const float z = ld_elem(logits + i);
    const float y = targets[i] != 0 ? 1.f : 0.f;
    const float e = expf(-fabsf(z));
    const float sig = (z >= 0.f ? 1.f : e) / (1.f + e);
    st_elem(dlogits + i, coef * (sig - y));
    my_loss += coef * (fmaxf(z, 0.f) + log1pf(e) - y * z);
  }
  my_loss = wave_sum(my_loss);
  if ((threadIdx.x & 63) == 0) wave_loss[threadIdx.x >> 6] = my_loss;
  __syncthreads();
  if (threadIdx.x == 0) partial[blockIdx.x] = (wave_loss[0] + wave_loss[1]) + (wave_loss[2] + wave_loss[3]);
}

__global__ __launch_bounds__(256) void loss_reduce_kernel(const float* __restrict__ partial, int32_t count,
                                                          float* __restrict__ out) {
  __shared__ float s[256];
  float acc = 0.f;
  for (int i = threadIdx.x; i < count; i += 256) acc += partial[i];
  s[threadIdx.x] = acc;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) s[threadIdx.x] += s[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) *out = s[0];
}

// partial[2b], partial[2b+1] = this block's sums of (a-b)^2 and a^2 (grid-stride, fixed order)
__global__ __launch_bounds__(256) void grad_gap_kernel(const float* __restrict__ a, const float* __restrict__ b,
                                                       int64_t n, float* __restrict__ partial) {
  __shared__ float wd[4], wr[4];
  float d2 = 0.f, r2 = 0.f;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const float x = a[i], d = x - b[i];
    d2 = fmaf(d, d, d2);
    r2 = fmaf(x, x, r2);
  }
  d2 = wave_sum(d2);
  r2 = wave_sum(r2);
  if ((threadIdx.x & 63) == 0) {
    wd[threadIdx.x >> 6] = d2;
    wr[threadIdx.x >> 6] = r2;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    partial[2 * blockIdx.x] = (wd[0] + wd[1]) + (wd[2] + wd[3]);
    partial[2 * blockIdx.x + 1] = (wr[0] + wr[1]) + (wr[2] + wr[3]);
  }
}

// out[j] = sqrt(sum over blocks of partial[2b + j]), j = 0, 1
__global__ __launch_bounds__(256) void grad_gap_finish_kernel(const float* __restrict__ partial, int32_t blocks,
                                                              float* __restrict__ out) {
  __shared__ float s[2][256];
  float acc0 = 0.f, acc1 = 0.f;
  for (int i = threadIdx.x; i < blocks; i += 256) {
    acc0 += partial[2 * i];
    acc1 += partial[2 * i + 1];
  }
  s[0][threadIdx.x] = acc0;
  s[1][threadIdx.x] = acc1;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) {
      s[0][threadIdx.x] += s[0][threadIdx.x + o];
      s[1][threadIdx.x] += s[1][threadIdx.x + o];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    out[0] = sqrtf(s[0][0]);
    out[1] = sqrtf(s[1][0]);
  }
}

__global__ __launch_bounds__(256) void sgd_kernel(float* __restrict__ theta, const float* __restrict__ grad,
                                                  int64_t n, float lr) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) theta[i] -= lr * grad[i];
}

__global__ __launch_bounds__(256) void adam_kernel(float* __restrict__ theta, const float* __restrict__ grad,
                                                   float* __restrict__ m, float* __restrict__ v, int64_t n,
                                                   float lr, float b1, float b2, float eps, float inv_c1,
                                                   float inv_c2) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const float g = grad[i];
  const float mi = b1 * m[i] + (1.f - b1) * g;
  const float vi = b2 * v[i] + (1.f - b2) * g * g;
  m[i] = mi;
  v[i] = vi;
  theta[i] -= lr * (mi * inv_c1) / (sqrtf(vi * inv_c2) + eps);
}

// ---- column sums (bias gradients): fixed-order two-stage reduction --------------------------
// Stage 1: block s sums its contiguous chunk of rows.  Within a block, lane l of every wavefront
// owns columns l, l+64, ... (of the block's 256-column panel, blockIdx.y) and wavefront w takes
// rows w, w+4, ... of the chunk; the four wavefront sums are then added in order through LDS.
// Stage 2: the per-chunk partials are added in a fixed order (split_reduce_kernel).  No atomics anywhere.
constexpr int COLSUM_MAX_SPLITS = 1024;
constexpr int COLSUM_PANEL = 256;

static int colsum_splits(int64_t M) {
  int64_t s = (M + 31) / 32;  // at least 32 rows per block
  if (s > COLSUM_MAX_SPLITS) s = COLSUM_MAX_SPLITS;
  if (s < 1) s = 1;
  return (int)s;
}

template <typename T>
__global__ __launch_bounds__(256) void colsum_partial_kernel(const T* __restrict__ X, int64_t ld, int64_t M,
                                                             int32_t N, int64_t rows_per_split,
                                                             float* __restrict__ partial) {
  __shared__ float sm[4][COLSUM_PANEL];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c0 = blockIdx.y * COLSUM_PANEL;
  const int64_t r0 = (int64_t)blockIdx.x * rows_per_split;
  int64_t r1 = r0 + rows_per_split;
  if (r1 > M) r1 = M;
  // lane l owns the four consecutive columns c0 + 4l .. +3: one wide access per row
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  const int avail = N - (c0 + 4 * lane);
  if (avail > 0) {
    // eight rows requested before the first is added (one dependent load per iteration left the loop
    // waiting on memory latency); the additions keep their row order
    const T* src = X + c0 + 4 * lane;
    int64_t r = r0 + wave;
    if (avail >= 4) {  // all but the lane at a ragged end of the row: plain wide loads, nothing in between
      for (; r + 28 < r1; r += 32) {
        float v[8][4];
#pragma unroll
        for (int u = 0; u < 8; ++u) ld4(src + (r + 4 * u) * ld, 4, v[u], 0.f);
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
          for (int q = 0; q < 4; ++q) acc[q] += v[u][q];
      }
    }
    for (; r < r1; r += 4) {
      float v[4];
      ld4(src + r * ld, avail, v, 0.f);
#pragma unroll
      for (int q = 0; q < 4; ++q) acc[q] += v[q];
    }
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) sm[wave][4 * lane + q] = acc[q];
  __syncthreads();
  const int c = threadIdx.x;
  if (c0 + c < N)
    partial[(int64_t)blockIdx.x * N + c0 + c] = ((sm[0][c] + sm[1][c]) + sm[2][c]) + sm[3][c];
}

size_t colsum_workspace_floats(int32_t N) { return (size_t)COLSUM_MAX_SPLITS * (size_t)N; }

int32_t launch_colsum(int32_t dtype, const void* X, int64_t ld, int64_t M, int32_t N, float* out,
                      int32_t accumulate, float* workspace, hipStream_t stream) {
  COFREE_REQUIRE(X && out && workspace, "colsum: NULL argument");
  COFREE_REQUIRE(dtype == COFREE_F32 || dtype == COFREE_BF16, "colsum: unknown dtype");
  COFREE_REQUIRE(N >= 1 && M >= 0 && ld >= N, "colsum: bad shape");
  const int splits = colsum_splits(M);
  const int64_t rows_per_split = (M + splits - 1) / splits;
  const dim3 grid((unsigned)splits, (unsigned)((N + COLSUM_PANEL - 1) / COLSUM_PANEL));
  {
    ProfScope prof("colsum_kernels", stream, (dtype == COFREE_F32 ? 4.0 : 2.0) * (double)M * N, (double)M * N);
    if (dtype == COFREE_F32)
      colsum_partial_kernel<float><<<grid, 256, 0, stream>>>((const float*)X, ld, M, N, rows_per_split, workspace);
    else
      colsum_partial_kernel<bf16_t><<<grid, 256, 0, stream>>>((const bf16_t*)X, ld, M, N, rows_per_split, workspace);
  }
  COFREE_HIP_CHECK(hipGetLastError());
  // stage 2: the same fixed-order reduction over partials as for the weight gradients
  return launch_split_reduce(workspace, N, splits, out, N, 1, N, accumulate, stream);
}

// ---- gradient gates: ReLU of the forward output and/or the dropout keep mask ----------------
template <typename T>
__global__ __launch_bounds__(256) void mask_grad_kernel(const T* src, const T* __restrict__ gate, T* dst,
                                                        int64_t total, float dropout_scale, uint32_t thr,
                                                        uint64_t seed, uint32_t epoch, uint32_t layer_stream) {
  // one thread per quad of four consecutive elements = one generator call
  const int64_t quad = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t base = quad * 4;
  if (base >= total) return;
  uint32_t words[4] = {0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu};
  if (dropout_scale != 0.f) {
    const u32x4 w = draw4(seed, layer_stream, (uint64_t)quad, epoch);
    words[0] = w.x;
    words[1] = w.y;
    words[2] = w.z;
    words[3] = w.w;
  }
  if (base + 4 <= total) {  // whole quad: one 16-byte (float32) / 8-byte (bfloat16) access per operand
    float x[4], g[4] = {1.f, 1.f, 1.f, 1.f};
    ld_quad(src + base, x);
    if (gate) ld_quad(gate + base, g);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      if (!(g[c] > 0.f)) x[c] = 0.f;
      if (dropout_scale != 0.f) x[c] = words[c] >= thr ? x[c] * dropout_scale : 0.f;
    }
    st_quad(dst + base, x);
    return;
  }
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const int64_t i = base + c;
    if (i < total) {
      float x = ld_elem(src + i);
      if (gate && !(ld_elem(gate + i) > 0.f)) x = 0.f;
      if (dropout_scale != 0.f) x = words[c] >= thr ? x * dropout_scale : 0.f;
      st_elem(dst + i, x);
    }
  }
}

int32_t launch_mask_grad(int32_t dtype, const void* src, const void* gate, void* dst, int64_t M, int32_t N,
                         const DropoutArgs& d, hipStream_t stream) {
  COFREE_REQUIRE(src && dst, "mask_grad: NULL argument");
  COFREE_REQUIRE((((uintptr_t)src | (uintptr_t)dst | (uintptr_t)gate) & 15u) == 0, "mask_grad: buffers must be 16-byte aligned");
  COFREE_REQUIRE(dtype == COFREE_F32 || dtype == COFREE_BF16, "mask_grad: unknown dtype");
  const int64_t total = M * (int64_t)N;
  if (total == 0) return COFREE_OK;
  const int64_t quads = (total + 3) / 4;
  const int64_t blocks = (quads + 255) / 256;
  COFREE_REQUIRE(blocks < ((int64_t)1 << 31), "mask_grad: grid too large");
  float scale = 0.f;
  uint32_t thr = 0;
  if (d.q > 0.f) {
    scale = 1.0f / (1.0f - d.q);
    thr = prob_threshold((double)d.q);
  }
  ProfScope prof("mask_grad_kernel", stream, (dtype == COFREE_F32 ? 4.0 : 2.0) * (double)total * (gate ? 3 : 2),
                 (double)total);
  const uint32_t ls = STREAM_DROPOUT + 256u * d.layer_id;
  if (dtype == COFREE_F32)
    mask_grad_kernel<float><<<dim3((unsigned)blocks), 256, 0, stream>>>((const float*)src, (const float*)gate,
                                                                        (float*)dst, total, scale, thr, d.seed,
                                                                        d.epoch, ls);
  else
    mask_grad_kernel<bf16_t><<<dim3((unsigned)blocks), 256, 0, stream>>>((const bf16_t*)src, (const bf16_t*)gate,
                                                                         (bf16_t*)dst, total, scale, thr, d.seed,
                                                                         d.epoch, ls);
  COFREE_HIP_CHECK(hipGetLastError());
  return COFREE_OK;
}

}  // namespace cofree

using namespace cofree;

extern "C" {

size_t cofree_loss_workspace_bytes(void) { return LOSS_BLOCKS * sizeof(float); }

// argument checks and weight vector shared by the two loss entry points
static int32_t loss_setup(const cofree_partition* part, int32_t weight_kind, const float* custom_w, const void* logits,
                          int32_t dtype, const void* labels, int32_t n_classes, const float* loss_out,
                          const void* dlogits, const void* workspace, size_t workspace_bytes, const float** w) {
  COFREE_REQUIRE(part != nullptr, "loss: partition is NULL");
  if (!part->on_device) return fail(COFREE_ESTATE, "loss: partition has no device copy");
  COFREE_REQUIRE(dtype == COFREE_F32 || dtype == COFREE_BF16, "loss: unknown dtype");
  COFREE_REQUIRE(logits && labels && loss_out && dlogits && workspace, "loss: NULL argument");
  COFREE_REQUIRE(n_classes >= 1, "loss: n_classes must be >= 1");
  if (workspace_bytes < cofree_loss_workspace_bytes()) return fail(COFREE_ENOMEM, "loss: workspace too small");
  switch (weight_kind) {
    case COFREE_W_DAR: *w = part->d_dar_weight; break;
    case COFREE_W_NONE: *w = nullptr; break;
    case COFREE_W_INV_RF:
      if (!part->d_inv_rf) return fail(COFREE_ESTATE, "loss: partition was built without COFREE_WITH_RF");
      *w = part->d_inv_rf;
      break;
    case COFREE_W_CUSTOM:
      COFREE_REQUIRE(custom_w != nullptr, "loss: custom_w is NULL");
      *w = custom_w;
      break;
    default: return fail(COFREE_EINVAL, "loss: unknown weight_kind");
  }
  return COFREE_OK;
}

// launches shared by cofree_loss_weighted and cofree_loss_weighted_static: `partial` holds LOSS_BLOCKS floats
static int32_t enqueue_softmax_loss(const cofree_partition* part, const float* w, const void* logits, int32_t dtype,
                                    const int32_t* labels, const uint8_t* train_mask, int32_t n_classes,
                                    float scale_c, float* loss_out, void* dlogits, float* partial, hipStream_t s) {
  const double es = dtype == COFREE_F32 ? 4.0 : 2.0;
  ProfScope prof("loss_kernels", s, (double)part->n_nodes * (2.0 * es * n_classes + 12.0),
                 8.0 * (double)part->n_nodes * n_classes);
#define COFREE_LOSS_ARGS(T) \
  (const T*)logits, labels, w, train_mask, part->n_nodes, n_classes, scale_c, (T*)dlogits, partial
  const bool f32 = dtype == COFREE_F32;
  const int per = f32 ? 4 : 8;  // classes per lane: 16 bytes
#define COFREE_LOSS_GROUP(L)                                                              \
  do {                                                                                    \
    if (f32) loss_group_kernel<float, L><<<LOSS_BLOCKS, 256, 0, s>>>(COFREE_LOSS_ARGS(float)); \
    else loss_group_kernel<bf16_t, L><<<LOSS_BLOCKS, 256, 0, s>>>(COFREE_LOSS_ARGS(bf16_t));   \
  } while (0)
  if (n_classes <= 8 * per) COFREE_LOSS_GROUP(8);
  else if (n_classes <= 16 * per) COFREE_LOSS_GROUP(16);
  else if (n_classes <= 32 * per) COFREE_LOSS_GROUP(32);
  else if (n_classes <= 64 * per) COFREE_LOSS_GROUP(64);
  else if (f32) loss_kernel<float><<<LOSS_BLOCKS, 256, 0, s>>>(COFREE_LOSS_ARGS(float));
  else loss_kernel<bf16_t><<<LOSS_BLOCKS, 256, 0, s>>>(COFREE_LOSS_ARGS(bf16_t));
#undef COFREE_LOSS_GROUP
#undef COFREE_LOSS_ARGS
  loss_reduce_kernel<<<1, 256, 0, s>>>(partial, LOSS_BLOCKS, loss_out);
  COFREE_HIP_CHECK(hipGetLastError());
  return COFREE_OK;
}

int32_t cofree_loss_weighted(const cofree_partition* part, int32_t weight_kind, const float* custom_w,
                             const void* logits, int32_t dtype, const int32_t* labels, const uint8_t* train_mask,
                             int32_t n_classes, float scale_c, float* loss_out, void* dlogits, void* workspace,
                             size_t workspace_bytes, void* stream) {
  const float* w = nullptr;
  COFREE_TRY(loss_setup(part, weight_kind, custom_w, logits, dtype, labels, n_classes, loss_out, dlogits, workspace,
                        workspace_bytes, &w));
  return enqueue_softmax_loss(part, w, logits, dtype, labels, train_mask, n_classes, scale_c, loss_out, dlogits,
                              (float*)workspace, (hipStream_t)stream);
}

// Device address of `scratch` on the current GPU.  Looked up once per device, with that device current (every
// GPU holds its own copy of the array at its own address), and kept.
static int32_t static_scratch(float** out) {
  static std::mutex mu;
  static float* per_device[COFREE_STATIC_MAX_DEVICES] = {};
  int dev = -1;
  COFREE_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= COFREE_STATIC_MAX_DEVICES) return fail(COFREE_EINVAL, "loss_static: device index out of range");
  std::lock_guard<std::mutex> lk(mu);
  if (!per_device[dev]) {
    float* p = nullptr;
    COFREE_HIP_CHECK(hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(COFREE_EHIP, "loss_static: hipGetSymbolAddress returned NULL");
    per_device[dev] = p;
  }
  *out = per_device[dev];
  return COFREE_OK;
}

int32_t cofree_loss_weighted_static(const cofree_partition* part, int32_t weight_kind, const float* custom_w,
                                    const void* logits, int32_t dtype, const int32_t* labels,
                                    const uint8_t* train_mask, int32_t n_classes, float scale_c, float* loss_out,
                                    void* dlogits, void* stream) {
  COFREE_REQUIRE(part != nullptr, "loss_static: partition is NULL");
  COFREE_REQUIRE(n_classes <= COFREE_LOSS_STATIC_MAX_CLASSES,
                 "loss_static: n_classes exceeds COFREE_LOSS_STATIC_MAX_CLASSES");
  COFREE_REQUIRE(part->n_nodes <= COFREE_LOSS_STATIC_MAX_NODES,
                 "loss_static: the partition has more nodes than COFREE_LOSS_STATIC_MAX_NODES");
  float* partial = nullptr;
  COFREE_TRY(static_scratch(&partial));
  const float* w = nullptr;
  COFREE_TRY(loss_setup(part, weight_kind, custom_w, logits, dtype, labels, n_classes, loss_out, dlogits, partial,
                        cofree_loss_workspace_bytes(), &w));
  // every one of the LOSS_BLOCKS partial sums is written by its workgroup (a workgroup without rows writes 0)
  // before the reduction reads it, so nothing of an earlier call's contents survives into this one
  return enqueue_softmax_loss(part, w, logits, dtype, labels, train_mask, n_classes, scale_c, loss_out, dlogits,
                              partial, (hipStream_t)stream);
}

int32_t cofree_loss_bce_weighted(const cofree_partition* part, int32_t weight_kind, const float* custom_w,
                                 const void* logits, int32_t dtype, const uint8_t* targets, const uint8_t* train_mask,
                                 int32_t n_classes, float scale_c, float* loss_out, void* dlogits, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  const float* w = nullptr;
  COFREE_TRY(loss_setup(part, weight_kind, custom_w, logits, dtype, targets, n_classes, loss_out, dlogits, workspace,
                        workspace_bytes, &w));
  hipStream_t s = (hipStream_t)stream;
  float* partial = (float*)workspace;
  const double es = dtype == COFREE_F32 ? 4.0 : 2.0;
  ProfScope prof("loss_kernels", s, (double)part->n_nodes * ((2.0 * es + 1.0) * n_classes + 4.0),
                 12.0 * (double)part->n_nodes * n_classes);
  if (dtype == COFREE_F32)
    bce_kernel<float><<<LOSS_BLOCKS, 256, 0, s>>>((const float*)logits, targets, w, train_mask, part->n_nodes,
                                                  n_classes, scale_c, (float*)dlogits, partial);
  else
    bce_kernel<bf16_t><<<LOSS_BLOCKS, 256, 0, s>>>((const bf16_t*)logits, targets, w, train_mask, part->n_nodes,
                                                   n_classes, scale_c, (bf16_t*)dlogits, partial);
  loss_reduce_kernel<<<1, 256, 0, s>>>(partial, LOSS_BLOCKS, loss_out);
  COFREE_HIP_CHECK(hipGetLastError());
  return COFREE_OK;
}

int32_t cofree_grad_gap(int64_t n, const float* g_full, const float* g_sum, float* out, void* workspace,
                        size_t workspace_bytes, void* stream) {
  COFREE_REQUIRE(n >= 0, "grad_gap: n is negative");
  COFREE_REQUIRE((n == 0 || (g_full && g_sum)) && out && workspace, "grad_gap: NULL argument");
  if (workspace_bytes < cofree_loss_workspace_bytes()) return fail(COFREE_ENOMEM, "grad_gap: workspace too small");
  hipStream_t s = (hipStream_t)stream;
  constexpr int GAP_BLOCKS = LOSS_BLOCKS / 2;  // two partials per block
  float* partial = (float*)workspace;
  grad_gap_kernel<<<GAP_BLOCKS, 256, 0, s>>>(g_full, g_sum, n, partial);
  grad_gap_finish_kernel<<<1, 256, 0, s>>>(partial, GAP_BLOCKS, out);
  COFREE_HIP_CHECK(hipGetLastError());
  return COFREE_OK;
}

int32_t cofree_step(int32_t kind, int64_t n, float* theta, const float* grad, float* m, float* v, float lr,
                    float b1, float b2, float eps, int64_t t, void* stream) {
  COFREE_REQUIRE(n >= 0, "step: n is negative");
  if (n == 0) return COFREE_OK;
  COFREE_REQUIRE(theta && grad, "step: NULL argument");
  const int64_t blocks = (n + 255) / 256;
  COFREE_REQUIRE(blocks < ((int64_t)1 << 31), "step: too many elements");
  hipStream_t s = (hipStream_t)stream;
  ProfScope prof("step_kernel", s, (kind == COFREE_SGD ? 12.0 : 28.0) * (double)n, 2.0 * (double)n);
  if (kind == COFREE_SGD) {
    sgd_kernel<<<dim3((unsigned)blocks), 256, 0, s>>>(theta, grad, n, lr);
  } else if (kind == COFREE_ADAM) {
    COFREE_REQUIRE(m && v, "step: Adam needs m and v");
    COFREE_REQUIRE(t >= 1, "step: Adam step count t must be >= 1");
    COFREE_REQUIRE(b1 >= 0.f && b1 < 1.f && b2 >= 0.f && b2 < 1.f, "step: betas must be in [0, 1)");
    const float inv_c1 = (float)(1.0 / (1.0 - std::pow((double)b1, (double)t)));
    const float inv_c2 = (float)(1.0 / (1.0 - std::pow((double)b2, (double)t)));
    adam_kernel<<<dim3((unsigned)blocks), 256, 0, s>>>(theta, grad, m, v, n, lr, b1, b2, eps, inv_c1, inv_c2);
  } else {
    return fail(COFREE_EINVAL, "step: unknown kind");
  }
  COFREE_HIP_CHECK(hipGetLastError());
  return COFREE_OK;
}

}  // extern "C"
