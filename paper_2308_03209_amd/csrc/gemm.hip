// Dense feature transforms of the layers (the W and U products of the GraphSAGE layer in
// Section 3 and their gradients) on the fp32 matrix cores of gfx950.
//
// One kernel computes a 128x128 tile of  C = sum_k Aop(i,k) * Bop(j,k)  per 256-thread block:
// four 64-wide wavefronts in a 2x2 grid, each holding a 64x64 sub-tile as 2x2 blocks of
// v_mfma_f32_32x32x2_f32 accumulators (fp32 in, fp32 accumulate).  Operand tiles of 16 k-steps
// are staged through LDS in k-major order ([k][i]) so that an MFMA operand is one conflict-free
// ds_read_b32 per lane; global loads of the next tile overlap the MFMAs of the current one
// (two LDS buffers, one barrier per tile).
//
// Operand layouts:
//   "k-contiguous": element (i,k) at P[i*ld + k]   (activations in forward / input gradients)
//   "k-major"     : element (i,k) at P[k*ld + i]   (weights in C = A.B; both operands of weight
//                                                  gradients, where k runs over graph nodes)
// A may consist of two k-segments taken from different matrices: this is the CONCAT of the
// layer definition, evaluated without materialising the concatenated matrix.
#include "common.h"

namespace cofree {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float float4u __attribute__((ext_vector_type(4), aligned(4)));

constexpr int BM = 128, BN = 128, BK = 16, LDS_LD = 132;  // 132 = 128 + 4 words of padding

struct GemmK {
  const float* A1;
  int64_t lda1;
  int32_t K1;
  const float* A2;
  int64_t lda2;
  int32_t K2;
  const float* B;
  int64_t ldb;
  float* C;
  int64_t ldc;
  int64_t M;   // rows of C (i range)
  int32_t N;   // cols of C (j range)
  int64_t K;   // total reduction length (K1 + K2)
  int64_t k_chunk;  // reduction range of blockIdx.z is [z*k_chunk, min(K, (z+1)*k_chunk))
  int64_t c_split_stride;  // C offset per blockIdx.z (split partials), 0 if unsplit
  const float* bias;
  int32_t relu;
  const float* row_scale;
  int32_t accumulate;
  float dropout_scale;  // 0: no dropout, else 1/(1-q)
  uint32_t dropout_thr;
  uint64_t seed;
  uint32_t epoch;
  uint32_t layer_stream;  // STREAM_DROPOUT + 256*layer_id
  int32_t tiles_n;
};

// ---- operand tile loaders: 128 (i) x 16 (k) floats per tile, 8 floats per thread ----------
// k-contiguous source: thread t reads 4 consecutive k of row (t>>2) and of row (t>>2)+64.
__device__ inline float seg_elem(const GemmK& p, int64_t row, int64_t k, int64_t k_end) {
  if (k >= k_end) return 0.f;
  return k < p.K1 ? p.A1[row * p.lda1 + k] : p.A2[row * p.lda2 + (k - p.K1)];
}

__device__ inline void load_a_kcontig(const GemmK& p, int64_t i0, int64_t k0, int64_t k_end, int tid,
                                      float4u (&reg)[2]) {
  const int kq = (tid & 3) * 4;
  const int64_t k = k0 + kq;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    int64_t row = i0 + (tid >> 2) + 64 * h;
    if (row >= p.M) row = p.M - 1;  // rows past the end are computed but never stored
    if (k + 3 < k_end && k + 3 < p.K1) {
      reg[h] = *reinterpret_cast<const float4u*>(p.A1 + row * p.lda1 + k);
    } else if (k + 3 < k_end && k >= p.K1) {
      reg[h] = *reinterpret_cast<const float4u*>(p.A2 + row * p.lda2 + (k - p.K1));
    } else {
      reg[h][0] = seg_elem(p, row, k, k_end);
      reg[h][1] = seg_elem(p, row, k + 1, k_end);
      reg[h][2] = seg_elem(p, row, k + 2, k_end);
      reg[h][3] = seg_elem(p, row, k + 3, k_end);
    }
  }
}

__device__ inline void load_b_kcontig(const GemmK& p, int64_t j0, int64_t k0, int64_t k_end, int tid,
                                      float4u (&reg)[2]) {
  const int kq = (tid & 3) * 4;
  const int64_t k = k0 + kq;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    int64_t row = j0 + (tid >> 2) + 64 * h;
    if (row >= p.N) row = p.N - 1;
    const float* src = p.B + row * p.ldb + k;
    if (k + 3 < k_end) {
      reg[h] = *reinterpret_cast<const float4u*>(src);
    } else {
      reg[h][0] = k < k_end ? src[0] : 0.f;
      reg[h][1] = k + 1 < k_end ? src[1] : 0.f;
      reg[h][2] = k + 2 < k_end ? src[2] : 0.f;
      reg[h][3] = k + 3 < k_end ? src[3] : 0.f;
    }
  }
}

// k-major source: thread t reads 4 consecutive i of k-row (t>>5) and of k-row (t>>5)+8.
__device__ inline void load_kmajor(const float* P, int64_t ld, int64_t extent, int64_t i0, int64_t k0,
                                   int64_t k_end, int tid, float4u (&reg)[2]) {
  const int64_t i = i0 + (tid & 31) * 4;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int64_t k = k0 + (tid >> 5) + 8 * h;
    if (k >= k_end) {
      reg[h] = float4u{0.f, 0.f, 0.f, 0.f};
      continue;
    }
    const float* src = P + k * ld + i;
    if (i + 3 < extent) {
      reg[h] = *reinterpret_cast<const float4u*>(src);
    } else {
      reg[h][0] = i < extent ? src[0] : 0.f;
      reg[h][1] = i + 1 < extent ? src[1] : 0.f;
      reg[h][2] = i + 2 < extent ? src[2] : 0.f;
      reg[h][3] = i + 3 < extent ? src[3] : 0.f;
    }
  }
}

__device__ inline void store_kcontig(float* lds, int tid, const float4u (&reg)[2]) {
  const int kq = (tid & 3) * 4;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int i = (tid >> 2) + 64 * h;
#pragma unroll
    for (int c = 0; c < 4; ++c) lds[(kq + c) * LDS_LD + i] = reg[h][c];
  }
}

__device__ inline void store_kmajor(float* lds, int tid, const float4u (&reg)[2]) {
  const int i = (tid & 31) * 4;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int k = (tid >> 5) + 8 * h;
    *reinterpret_cast<float4*>(lds + k * LDS_LD + i) = make_float4(reg[h][0], reg[h][1], reg[h][2], reg[h][3]);
  }
}

template <bool A_KMAJOR, bool B_KMAJOR>
__global__ __launch_bounds__(256) void gemm_kernel(const GemmK p) {
  __shared__ __attribute__((aligned(16))) float As[2][BK * LDS_LD];
  __shared__ __attribute__((aligned(16))) float Bs[2][BK * LDS_LD];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int64_t tile = blockIdx.x;
  const int64_t i0 = (tile / p.tiles_n) * BM;
  const int64_t j0 = (tile % p.tiles_n) * BN;
  const int64_t k_beg = (int64_t)blockIdx.z * p.k_chunk;
  const int64_t k_end = (k_beg + p.k_chunk < p.K) ? k_beg + p.k_chunk : p.K;

  floatx16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  float4u ra[2], rb[2];
  auto load_tiles = [&](int64_t k0) {
    if constexpr (A_KMAJOR) load_kmajor(p.A1, p.lda1, p.M, i0, k0, k_end, tid, ra);
    else load_a_kcontig(p, i0, k0, k_end, tid, ra);
    if constexpr (B_KMAJOR) load_kmajor(p.B, p.ldb, p.N, j0, k0, k_end, tid, rb);
    else load_b_kcontig(p, j0, k0, k_end, tid, rb);
  };
  auto store_tiles = [&](int buf) {
    if constexpr (A_KMAJOR) store_kmajor(As[buf], tid, ra);
    else store_kcontig(As[buf], tid, ra);
    if constexpr (B_KMAJOR) store_kmajor(Bs[buf], tid, rb);
    else store_kcontig(Bs[buf], tid, rb);
  };

  const int64_t n_tiles = (k_end > k_beg) ? (k_end - k_beg + BK - 1) / BK : 0;
  if (n_tiles > 0) {
    load_tiles(k_beg);
    store_tiles(0);
  }
  __syncthreads();
  const int g = lane >> 5, r = lane & 31;
  for (int64_t t = 0; t < n_tiles; ++t) {
    const int buf = (int)(t & 1);
    const bool more = t + 1 < n_tiles;
    if (more) load_tiles(k_beg + (t + 1) * BK);
    const float* as = As[buf] + wm * 64 + r;
    const float* bs = Bs[buf] + wn * 64 + r;
#pragma unroll
    for (int kk = 0; kk < BK / 2; ++kk) {
      const int krow = (2 * kk + g) * LDS_LD;
      const float a0 = as[krow], a1 = as[krow + 32];
      const float b0 = bs[krow], b1 = bs[krow + 32];
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
    }
    if (more) store_tiles(buf ^ 1);
    __syncthreads();
  }

  // epilogue: accumulator register v of lane (g, r) is C[8*(v/4) + 4*g + v%4][r] of its 32x32 block
  float* Cz = p.C + (int64_t)blockIdx.z * p.c_split_stride;
#pragma unroll
  for (int a = 0; a < 2; ++a) {
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const int64_t j = j0 + wn * 64 + b * 32 + r;
      if (j >= p.N) continue;
      const float bj = p.bias ? p.bias[j] : 0.f;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t i = i0 + wm * 64 + a * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
        if (i >= p.M) continue;
        float x = acc[a][b][v] + bj;
        if (p.relu) x = fmaxf(x, 0.f);
        if (p.row_scale) x *= p.row_scale[i];
        if (p.dropout_scale != 0.f) {
          const uint64_t idx = (uint64_t)i * (uint64_t)p.N + (uint64_t)j;
          const u32x4 w = draw4(p.seed, p.layer_stream, idx >> 2, p.epoch);
          const uint32_t sel = (uint32_t)(idx & 3);
          const uint32_t word = sel == 0 ? w.x : sel == 1 ? w.y : sel == 2 ? w.z : w.w;
          x = word >= p.dropout_thr ? x * p.dropout_scale : 0.f;
        }
        float* dst = Cz + i * p.ldc + j;
        if (p.accumulate) x += *dst;
        *dst = x;
      }
    }
  }
}

// fixed-order sum of split partials: C[i, j] (+)= sum_z part[z][i][j]
__global__ __launch_bounds__(256) void split_reduce_kernel(const float* __restrict__ part, int64_t split_stride,
                                                           int32_t splits, float* __restrict__ C, int64_t ldc,
                                                           int32_t rows, int32_t cols, int32_t accumulate) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)rows * cols) return;
  const int64_t i = idx / cols, j = idx % cols;
  float s = 0.f;
  for (int z = 0; z < splits; ++z) s += part[(int64_t)z * split_stride + idx];
  float* dst = C + i * ldc + j;
  *dst = accumulate ? *dst + s : s;
}

static int32_t check_grid(int64_t blocks) {
  COFREE_REQUIRE(blocks > 0 && blocks < ((int64_t)1 << 31), "dense: grid too large");
  return COFREE_OK;
}

int32_t launch_gemm(const GemmArgs& a, hipStream_t stream) {
  COFREE_REQUIRE(a.A1 && a.B && a.C, "dense: NULL operand");
  COFREE_REQUIRE(a.M >= 0 && a.N >= 1 && a.K1 >= 1 && a.K2 >= 0, "dense: bad shape");
  COFREE_REQUIRE(a.K2 == 0 || a.A2, "dense: second segment is NULL");
  COFREE_REQUIRE(a.lda1 >= a.K1 && (a.K2 == 0 || a.lda2 >= a.K2), "dense: lda too small");
  COFREE_REQUIRE(a.ldc >= a.N, "dense: ldc too small");
  COFREE_REQUIRE(a.dropout.q >= 0.f && a.dropout.q < 1.f, "dense: dropout rate must be in [0, 1)");
  if (a.M == 0) return COFREE_OK;
  GemmK p{};
  p.A1 = a.A1;
  p.lda1 = a.lda1;
  p.K1 = a.K1;
  p.A2 = a.A2;
  p.lda2 = a.lda2;
  p.K2 = a.K2;
  p.B = a.B;
  p.ldb = a.ldb;
  p.C = a.C;
  p.ldc = a.ldc;
  p.M = a.M;
  p.N = a.N;
  p.K = (int64_t)a.K1 + a.K2;
  p.k_chunk = p.K;
  p.c_split_stride = 0;
  p.bias = a.bias;
  p.relu = a.relu;
  p.row_scale = a.row_scale;
  p.accumulate = a.accumulate;
  if (a.dropout.q > 0.f) {
    p.dropout_scale = 1.0f / (1.0f - a.dropout.q);
    p.dropout_thr = prob_threshold((double)a.dropout.q);
    p.seed = a.dropout.seed;
    p.epoch = a.dropout.epoch;
    p.layer_stream = STREAM_DROPOUT + 256u * a.dropout.layer_id;
  }
  p.tiles_n = (a.N + BN - 1) / BN;
  const int64_t blocks = ((a.M + BM - 1) / BM) * p.tiles_n;
  COFREE_TRY(check_grid(blocks));
  if (a.b_kmajor) {
    COFREE_REQUIRE(a.ldb >= a.N, "dense: ldb too small");
    gemm_kernel<false, true><<<dim3((unsigned)blocks), 256, 0, stream>>>(p);
  } else {
    COFREE_REQUIRE(a.ldb >= p.K, "dense: ldb too small");
    gemm_kernel<false, false><<<dim3((unsigned)blocks), 256, 0, stream>>>(p);
  }
  COFREE_HIP_CHECK(hipGetLastError());
  return COFREE_OK;
}

static int32_t wgrad_splits(int32_t N1, int32_t N2, int64_t M) {
  const int64_t tiles = (int64_t)((N1 + BM - 1) / BM) * ((N2 + BN - 1) / BN);
  int64_t s = (768 + tiles - 1) / tiles;
  const int64_t max_by_len = (M + 511) / 512;  // at least 512 reduction steps per split
  if (s > max_by_len) s = max_by_len;
  if (s > 128) s = 128;
  if (s < 1) s = 1;
  return (int32_t)s;
}

size_t wgrad_workspace_floats(int32_t N1, int32_t N2, int64_t M) {
  return (size_t)wgrad_splits(N1, N2, M) * (size_t)N1 * (size_t)N2;
}

int32_t launch_wgrad(const float* A, int64_t lda, int32_t N1, const float* B, int64_t ldb, int32_t N2, int64_t M,
                     float* C, int64_t ldc, int32_t accumulate, float* workspace, hipStream_t stream) {
  COFREE_REQUIRE(A && B && C && workspace, "wgrad: NULL operand");
  COFREE_REQUIRE(N1 >= 1 && N2 >= 1 && M >= 0, "wgrad: bad shape");
  COFREE_REQUIRE(lda >= N1 && ldb >= N2 && ldc >= N2, "wgrad: leading dimension too small");
  const int32_t S = wgrad_splits(N1, N2, M);
  GemmK p{};
  p.A1 = A;
  p.lda1 = lda;
  p.K1 = 0;  // unused by k-major loaders
  p.B = B;
  p.ldb = ldb;
  p.C = workspace;
  p.ldc = N2;
  p.M = N1;
  p.N = N2;
  p.K = M;
  int64_t chunk = (M + S - 1) / S;
  chunk = ((chunk + BK - 1) / BK) * BK;
  if (chunk < BK) chunk = BK;
  p.k_chunk = chunk;
  p.c_split_stride = (int64_t)N1 * N2;
  p.tiles_n = (N2 + BN - 1) / BN;
  const int64_t blocks = (int64_t)((N1 + BM - 1) / BM) * p.tiles_n;
  COFREE_TRY(check_grid(blocks));
  gemm_kernel<true, true><<<dim3((unsigned)blocks, 1, (unsigned)S), 256, 0, stream>>>(p);
  COFREE_HIP_CHECK(hipGetLastError());
  const int64_t total = (int64_t)N1 * N2;
  split_reduce_kernel<<<dim3((unsigned)((total + 255) / 256)), 256, 0, stream>>>(workspace, p.c_split_stride, S, C,
                                                                                 ldc, N1, N2, accumulate);
  COFREE_HIP_CHECK(hipGetLastError());
  return COFREE_OK;
}

}  // namespace cofree

using namespace cofree;

extern "C" int32_t cofree_dense_nt_f32(const float* A, const float* B, const float* bias, float* C, int64_t M,
                                       int32_t N, int32_t K, int32_t relu, void* stream) {
  GemmArgs g;
  g.A1 = A;
  g.lda1 = K;
  g.K1 = K;
  g.B = B;
  g.ldb = K;
  g.C = C;
  g.ldc = N;
  g.M = M;
  g.N = N;
  g.bias = bias;
  g.relu = relu;
  return launch_gemm(g, (hipStream_t)stream);
}
