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
#include <algorithm>
#include <cstdio>

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
  const float* B2;  // second segment's own matrix, or null (then it continues in B)
  int64_t ldb2;
  float* C;
  int64_t ldc;
  int64_t M;   // rows of C (i range)
  int32_t N;   // cols of C (j range)
  int64_t K;   // total reduction length (K1 + K2)
  int64_t k_chunk;  // reduction range of k-chunk z is [z*k_chunk, min(K, (z+1)*k_chunk))
  int64_t c_split_stride;  // C offset per k-chunk (split partials), 0 if unsplit
  const float* bias;
  int32_t relu;
  const float* row_scale;
  const float* gate;
  int64_t ldg;
  int32_t accumulate;
  int32_t relu_last;
  int32_t gate_last;  // the gate applies to the accumulated value
  float gate_scale;   // factor on the elements that pass the gate
  int32_t tiles_n;
  int32_t tiles_m;   // weight gradients only
  int64_t n_groups;  // row panels (forward / input gradients) or k-chunks (weight gradients)
  float* colsum_part;  // weight gradients: [chunks][M] partial column sums of operand A, or null
  int32_t n_split;     // weight gradients: columns n_split .. of the result come from B2 (0: everything from B)
};

// ---- operand tile movers: 128 (i) x 16 (k) floats per tile, 8 floats per thread -----------
// Each mover is set up once per k-range with per-thread base pointers, so that the pipelined
// loop issues plain vector loads with no bounds logic.  Out-of-range i (rows / columns past the
// matrix edge) is handled by clamping the index: the values read there are finite, valid
// memory and only reach output elements that are never stored.  Out-of-range k (a ragged last
// tile) must contribute zero, and is handled by the guarded `load_ragged` outside the loop.

// k-contiguous source: thread t holds 4 consecutive k of row (t>>2) and of row (t>>2)+64.
struct MoverKContig {
  const float* p0;
  const float* p1;
  __device__ void init(const float* P, int64_t ld, int64_t extent, int64_t i0, int tid) {
    int64_t r0 = i0 + (tid >> 2), r1 = r0 + 64;
    if (r0 > extent - 1) r0 = extent - 1;
    if (r1 > extent - 1) r1 = extent - 1;
    p0 = P + r0 * ld + (tid & 3) * 4;
    p1 = P + r1 * ld + (tid & 3) * 4;
  }
  __device__ void load(int64_t k0, float4u& x0, float4u& x1) const {
    x0 = *reinterpret_cast<const float4u*>(p0 + k0);
    x1 = *reinterpret_cast<const float4u*>(p1 + k0);
  }
  // Tile starting at k0 of a range of length k_len >= 1, k0 + 16 > k_len.  A thread whose four k would
  // cross the end of the range reads the four-wide window that ends with the range instead (one vector
  // load per row on every path, as in a full tile) and moves its valid elements into place; elements past
  // the end become zero.  Ranges shorter than four read clamped scalars.
  __device__ void load_ragged(int64_t k0, int64_t k_len, int tid, float4u& x0, float4u& x1) const {
    const int64_t kq = (tid & 3) * 4;
    const int64_t k = k0 + kq;
    if (k_len < 4) {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int64_t kc = k + c < k_len ? k + c : k_len - 1;
        const float v0 = p0[kc - kq], v1 = p1[kc - kq];
        x0[c] = k + c < k_len ? v0 : 0.f;
        x1[c] = k + c < k_len ? v1 : 0.f;
      }
      return;
    }
    int64_t v = k_len - k;  // valid elements of this thread: <= 0 none, >= 4 all
    if (v > 4) v = 4;
    if (v < 0) v = 0;
    const int64_t ks = v == 4 ? k : k_len - 4;  // start of the window that is read
    const float4u w0 = *reinterpret_cast<const float4u*>(p0 + (ks - kq));
    const float4u w1 = *reinterpret_cast<const float4u*>(p1 + (ks - kq));
    const int sh = 4 - (int)v;  // element c of the thread is element c + sh of the window
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      float a = 0.f, b = 0.f;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (e == c + sh) {
          a = w0[e];
          b = w1[e];
        }
      }
      x0[c] = a;
      x1[c] = b;
    }
  }
  static __device__ void store(float* lds, int tid, const float4u& x0, const float4u& x1) {
    float* d = lds + (tid & 3) * 4 * LDS_LD + (tid >> 2);
    d[0] = x0[0];
    d[LDS_LD] = x0[1];
    d[2 * LDS_LD] = x0[2];
    d[3 * LDS_LD] = x0[3];
    d[64] = x1[0];
    d[LDS_LD + 64] = x1[1];
    d[2 * LDS_LD + 64] = x1[2];
    d[3 * LDS_LD + 64] = x1[3];
  }
};

// k-major source: thread t holds 4 consecutive i of k-row (t>>5) and of k-row (t>>5)+8.
// Where the block's i-range crosses the matrix edge (`edge`, uniform over the block), a thread's
// four columns may cross the end of the row: its load window is moved left to end with the row - if
// need be into the columns of the tile before - so the loop issues one vector load per row on every
// path, and store() moves the elements back to their positions; columns past the edge receive
// arbitrary finite values.  TINY is for matrices with fewer than four columns in all, where no such
// window exists: scalar loads of clamped columns.
template <bool TINY>
struct MoverKMajorT {
  const float* base;  // &P[(t>>5) * ld + i0]
  int64_t ld;
  int32_t start;   // first column of the load window relative to i0 (negative: reaches into the tile before)
  int32_t shift;   // the thread's column c is element c + shift of the window (0 unless moved)
  int32_t ic[4];   // TINY: clamped column of each element
  bool edge;
  __device__ void init(const float* P, int64_t ld_, int64_t extent, int64_t i0, int tid) {
    ld = ld_;
    edge = i0 + BM > extent;
    base = P + (int64_t)(tid >> 5) * ld + i0;
    const int32_t last = (int32_t)(extent - 1 - i0);
    const int32_t i = (tid & 31) * 4;
    start = i;
    if (start > last - 3) start = last - 3;
    shift = i - start;
    if (shift > 3) shift = 0;  // all four columns are past the edge
#pragma unroll
    for (int c = 0; c < 4; ++c) ic[c] = i + c < last ? i + c : last;
  }
  __device__ void load_row(const float* row, float4u& x) const {
    if constexpr (TINY) {
      x[0] = row[ic[0]];
      x[1] = row[ic[1]];
      x[2] = row[ic[2]];
      x[3] = row[ic[3]];
    } else {
      x = *reinterpret_cast<const float4u*>(row + start);
    }
  }
  __device__ void load(int64_t k0, float4u& x0, float4u& x1) const {
    const float* r = base + k0 * ld;
    load_row(r, x0);
    load_row(r + 8 * ld, x1);
  }
  // branch-free ragged tile: k-rows past the end are read from the last valid row and zeroed
  __device__ void load_ragged(int64_t k0, int64_t k_len, int tid, float4u& x0, float4u& x1) const {
    const int64_t k = k0 + (tid >> 5);
    const int64_t ka = k < k_len ? k : k_len - 1, kb = k + 8 < k_len ? k + 8 : k_len - 1;
    const float* r = base - (int64_t)(tid >> 5) * ld;  // row 0 of the range
    load_row(r + ka * ld, x0);
    load_row(r + kb * ld, x1);
    if (!(k < k_len)) x0 = float4u{0.f, 0.f, 0.f, 0.f};
    if (!(k + 8 < k_len)) x1 = float4u{0.f, 0.f, 0.f, 0.f};
  }
  __device__ float4 unshift(const float4u& w) const {
    float4 x = make_float4(w[0], w[1], w[2], w[3]);
    if constexpr (!TINY) {
      if (edge) {
        if (shift == 1) x = make_float4(w[1], w[2], w[3], w[3]);
        if (shift == 2) x = make_float4(w[2], w[3], w[3], w[3]);
        if (shift == 3) x = make_float4(w[3], w[3], w[3], w[3]);
      }
    }
    return x;
  }
  __device__ void store(float* lds, int tid, const float4u& x0, const float4u& x1) const {
    float* d = lds + (tid >> 5) * LDS_LD + (tid & 31) * 4;
    *reinterpret_cast<float4*>(d) = unshift(x0);
    *reinterpret_cast<float4*>(d + 8 * LDS_LD) = unshift(x1);
  }
};

// 16 k-steps of one LDS tile pair on a wavefront's sub-tile of AM x AN blocks of 32x32 (2x2: 32 MFMAs).
template <int AM, int AN>
__device__ inline void compute_tile(const float* __restrict__ as, const float* __restrict__ bs,
                                    floatx16 (&acc)[AM][AN], int g) {
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    float a[AM][4], b[AN][4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int krow = (2 * (4 * half + q) + g) * LDS_LD;
#pragma unroll
      for (int m = 0; m < AM; ++m) a[m][q] = as[krow + 32 * m];
#pragma unroll
      for (int n = 0; n < AN; ++n) b[n][q] = bs[krow + 32 * n];
    }
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int m = 0; m < AM; ++m)
#pragma unroll
        for (int n = 0; n < AN; ++n)
          acc[m][n] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[m][q], b[n][q], acc[m][n], 0, 0, 0);
  }
}

// Accumulate one k-range of length k_len (operands already positioned at its first k).
// do_colsum (uniform over the block): thread t < 64*AM also adds up column t of the A tiles
// over k - the bias gradient that belongs to this weight gradient - from the LDS copy.
// The global loads run D k-tiles ahead of the MFMAs, in a ring of registers (slot = tile mod D, static
// after unrolling): three resident workgroups per CU do not hide the memory latency with one tile in
// flight.  Loads are unconditional (past the end
// they repeat the last tile, an L2 hit), so the number of outstanding loads is the same on every path and
// a store waits for its own slot only.  LDS is double-buffered with one barrier per tile: tile t is stored,
// the barrier passes, tile t is multiplied, and the store of tile t+1 goes to the other buffer, which
// every wavefront stopped reading before that barrier.
template <int D, int AM, int AN, typename MA, typename MB>
__device__ inline void run_range_deep(const MA& ma, const MB& mb, int64_t k_len, float (&As)[2][BK * LDS_LD],
                                      float (&Bs)[2][BK * LDS_LD], floatx16 (&acc)[AM][AN], int tid,
                                      bool do_colsum, float& colsum) {
  auto add_colsum = [&](const float* tile) {
    if (do_colsum && tid < 64 * AM) {
      float s = 0.f;
#pragma unroll
      for (int k = 0; k < BK; ++k) s += tile[k * LDS_LD + tid];
      colsum += s;
    }
  };
  const int lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, r = lane & 31;
  const int a_off = (wave >> 1) * (32 * AM) + r, b_off = (wave & 1) * (32 * AN) + r;
  const int64_t n_full = k_len / BK;
  float4u ra[D][2], rb[D][2];
  __syncthreads();  // previous readers of the LDS buffers are done
  if (n_full > 0) {
    const int64_t t_last = n_full - 1;
    auto step = [&](int64_t t, int s, bool refill) {
      float* const at = As[t & 1];
      float* const bt = Bs[t & 1];
      ma.store(at, tid, ra[s][0], ra[s][1]);
      mb.store(bt, tid, rb[s][0], rb[s][1]);
      if (refill) {
        const int64_t tn = t + D < t_last ? t + D : t_last;
        ma.load(tn * BK, ra[s][0], ra[s][1]);
        mb.load(tn * BK, rb[s][0], rb[s][1]);
      }
      __syncthreads();
      compute_tile<AM, AN>(at + a_off, bt + b_off, acc, g);
      add_colsum(at);
    };
#pragma unroll
    for (int s = 0; s < D; ++s) {
      const int64_t tn = s < t_last ? s : t_last;
      ma.load(tn * BK, ra[s][0], ra[s][1]);
      mb.load(tn * BK, rb[s][0], rb[s][1]);
    }
    int64_t t0 = 0;
    for (; t0 + D <= n_full; t0 += D) {
#pragma unroll
      for (int s = 0; s < D; ++s) step(t0 + s, s, true);
    }
#pragma unroll
    for (int s = 0; s < D - 1; ++s)
      if (t0 + s < n_full) step(t0 + s, s, false);
  }
  if (n_full * BK < k_len) {
    float* const at = As[n_full & 1];
    float* const bt = Bs[n_full & 1];
    ma.load_ragged(n_full * BK, k_len, tid, ra[0][0], ra[0][1]);
    mb.load_ragged(n_full * BK, k_len, tid, rb[0][0], rb[0][1]);
    ma.store(at, tid, ra[0][0], ra[0][1]);
    mb.store(bt, tid, rb[0][0], rb[0][1]);
    __syncthreads();
    compute_tile<AM, AN>(at + a_off, bt + b_off, acc, g);
    add_colsum(at);
  }
}

// k-tiles in flight per workgroup: two, with which every instance fits three workgroups per CU (the weight
// gradients measured 1-7 % slower with three tiles in flight at two workgroups per CU)
constexpr int WGRAD_DEPTH = 2;
constexpr int NT_DEPTH = 2;

// TINY: a k-major operand has fewer than four columns (see MoverKMajorT).
// NARROW: 0 = 128x128 block tile (wavefronts 2x2, each 64x64); 1 = 128x64 for outputs of at most 64 columns
// (each wavefront 64x32); 2 = 64x128 for at most 64 rows (each 32x64).  The narrow forms move the same
// 128-wide operand tiles - the clamped rows past the matrix edge repeat its last row - and only skip the
// MFMAs of the half that would never be stored (a 41-column product otherwise spends two thirds of its
// matrix instructions on padding).
template <bool A_KMAJOR, bool B_KMAJOR, bool TINY, int NARROW>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3))) void gemm_kernel(const GemmK p) {
  constexpr int AM = NARROW == 2 ? 1 : 2, AN = NARROW == 1 ? 1 : 2;  // 32x32 blocks per wavefront
  constexpr int TM = 64 * AM, TN = 64 * AN;                          // block tile
  // operand tiles during the k loop; afterwards the same memory stages the result tile
  constexpr int STAGE_LD = 68;  // floats per staged row: 64 + 4 of padding
  constexpr int SMEM_FLOATS = 4 * BK * LDS_LD > 4 * 32 * STAGE_LD ? 4 * BK * LDS_LD : 4 * 32 * STAGE_LD;
  __shared__ __attribute__((aligned(16))) float smem[SMEM_FLOATS];
  float(&As)[2][BK * LDS_LD] = *reinterpret_cast<float(*)[2][BK * LDS_LD]>(smem);
  float(&Bs)[2][BK * LDS_LD] = *reinterpret_cast<float(*)[2][BK * LDS_LD]>(smem + 2 * BK * LDS_LD);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  The tiles that share
  // an operand panel - the column tiles of one row panel, or all output tiles of one k-chunk of a
  // weight gradient - are given linear ids that are congruent mod 8 and adjacent in that XCD's
  // dispatch order, so the shared panel is fetched from HBM once and re-read from that L2.
  //   linear id L = (group / 8) * 8 * per_group + member * 8 + group % 8
  int64_t i0, j0, z;
  {
    const int64_t L = blockIdx.x;
    const int64_t per_group = A_KMAJOR ? p.tiles_m * p.tiles_n : p.tiles_n;
    const int64_t group = (L / (8 * per_group)) * 8 + (L & 7);
    const int64_t member = (L >> 3) % per_group;
    if (group >= p.n_groups) return;  // padding of the last group octet (uniform over the block)
    if constexpr (A_KMAJOR) {
      z = group;
      i0 = (member / p.tiles_n) * TM;
      j0 = (member % p.tiles_n) * TN;
    } else {
      z = 0;
      i0 = group * TM;
      j0 = member * TN;
    }
  }

  floatx16 acc[AM][AN];
#pragma unroll
  for (int a = 0; a < AM; ++a)
#pragma unroll
    for (int b = 0; b < AN; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  if constexpr (!A_KMAJOR) {
    // forward / input-gradient products: A = one or two k-contiguous segments
    float no_colsum = 0.f;
    auto do_segment = [&](const float* A, int64_t lda, int64_t k_len, const float* B, int64_t ldb) {
      // B = the segment's first k of the parameter operand
      MoverKContig ma;
      ma.init(A, lda, p.M, i0, tid);
      if constexpr (!B_KMAJOR) {
        MoverKContig mb;
        mb.init(B, ldb, p.N, j0, tid);
        run_range_deep<NT_DEPTH, AM, AN>(ma, mb, k_len, As, Bs, acc, tid, false, no_colsum);
      } else {
        MoverKMajorT<TINY> mb;
        mb.init(B, ldb, p.N, j0, tid);
        run_range_deep<NT_DEPTH, AM, AN>(ma, mb, k_len, As, Bs, acc, tid, false, no_colsum);
      }
    };
    // one loop body for both K-segments (two inlined copies would each claim their own accumulators)
    const int n_seg = p.K2 > 0 ? 2 : 1;
#pragma nounroll
    for (int seg = 0; seg < n_seg; ++seg) {
      const float* B = p.B;
      int64_t ldb = p.ldb;
      if (seg) {
        if (p.B2) {
          B = p.B2;
          ldb = p.ldb2;
        } else {
          B += B_KMAJOR ? (int64_t)p.K1 * p.ldb : (int64_t)p.K1;
        }
      }
      do_segment(seg ? p.A2 : p.A1, seg ? p.lda2 : p.lda1, seg ? p.K2 : p.K1, B, ldb);
    }
  } else {
    // weight gradients: both operands k-major, k = graph nodes, split into k-chunks
    const int64_t k_beg = z * p.k_chunk;
    const int64_t k_end = (k_beg + p.k_chunk < p.K) ? k_beg + p.k_chunk : p.K;
    const int64_t k_len = k_end > k_beg ? k_end - k_beg : 0;
    const float* A = p.A1 + k_beg * p.lda1;
    if (k_len > 0) {
      MoverKMajorT<TINY> ma, mb;
      ma.init(A, p.lda1, p.M, i0, tid);
      if (p.n_split > 0 && j0 >= p.n_split)  // a column tile of the second matrix (uniform over the block)
        mb.init(p.B2 + k_beg * p.ldb2, p.ldb2, p.N - p.n_split, j0 - p.n_split, tid);
      else
        mb.init(p.B + k_beg * p.ldb, p.ldb, p.n_split > 0 ? p.n_split : p.N, j0, tid);
      float csum = 0.f;
      const bool do_colsum = p.colsum_part != nullptr && j0 == 0;
      run_range_deep<WGRAD_DEPTH, AM, AN>(ma, mb, k_len, As, Bs, acc, tid, do_colsum, csum);
      if (do_colsum && tid < TM && i0 + tid < p.M) p.colsum_part[z * p.M + i0 + tid] = csum;
    } else if (p.colsum_part != nullptr && j0 == 0 && tid < TM && i0 + tid < p.M) {
      p.colsum_part[z * p.M + i0 + tid] = 0.f;
    }
  }

  // epilogue: accumulator register v of lane (g, r) is C[8*(v/4) + 4*g + v%4][r] of its 32x32 block
  const int g = lane >> 5, r = lane & 31;
  if constexpr (A_KMAJOR) {
    // float32 partial of this k-chunk (small: one tile per workgroup and chunk)
    float* Cz = p.C + z * p.c_split_stride;
#pragma unroll
    for (int a = 0; a < AM; ++a) {
#pragma unroll
      for (int b = 0; b < AN; ++b) {
        const int64_t j = j0 + wn * (32 * AN) + b * 32 + r;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int64_t i = i0 + wm * (32 * AM) + a * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
          if (j < p.N && i < p.M) Cz[i * p.ldc + j] = acc[a][b][v];
        }
      }
    }
  } else {
    // Each wavefront passes its result through LDS in 32-row blocks, after which a lane holds 4 consecutive
    // columns of one row: gate and accumulate operands are read, and the result is written, 16 bytes at
    // a time (element-sized accesses are bound by the rate of memory instructions).  Those operands and
    // the row scales do not depend on the product, so they are requested for four passes at a time -
    // unconditionally, at clamped addresses, the first four of a block before its staging barriers -
    // rather than one by one between the stores (load, wait, load, wait, store per pass).
    constexpr int LPR = 8 * AN;      // lanes per staged row
    constexpr int RPP = 64 / LPR;    // rows per pass
    constexpr int PASSES = 32 / RPP; // passes per 32-row block: 8 or 4
    float* const st = smem + wave * 32 * STAGE_LD;
    const int er = lane / LPR, ec = (lane % LPR) * 4;
    const int64_t jv = j0 + wn * (32 * AN) + ec;
    const bool wide_lane = jv + 4 <= p.N;   // the lane's four columns all exist
    const int64_t jl = wide_lane ? jv : 0;  // where its 16-byte operand loads go (in range once N >= 4)
    const bool extras = (p.gate || p.accumulate || p.row_scale) && p.N >= 4;  // uniform over the launch
    struct Extra {
      float4u g, c;
      float rs;
    };
    auto request = [&](int a, int sidx, Extra& e) {
      int64_t il = i0 + wm * (32 * AM) + a * 32 + sidx * RPP + er;
      if (il > p.M - 1) il = p.M - 1;
      e.g = float4u{1.f, 1.f, 1.f, 1.f};
      e.c = float4u{0.f, 0.f, 0.f, 0.f};
      e.rs = 1.f;
      if (p.gate) e.g = *reinterpret_cast<const float4u*>(p.gate + il * p.ldg + jl);
      if (p.accumulate) e.c = *reinterpret_cast<const float4u*>(p.C + il * p.ldc + jl);
      if (p.row_scale) e.rs = p.row_scale[il];
    };
    auto pass = [&](int a, int sidx, bool have, const Extra& e) {
      const int row = sidx * RPP + er;
      const int64_t i = i0 + wm * (32 * AM) + a * 32 + row;
      if (i < p.M && jv < p.N) {
        const float4 t = *reinterpret_cast<const float4*>(st + row * STAGE_LD + ec);
        float x[4] = {t.x, t.y, t.z, t.w};
        float* dst = p.C + i * p.ldc + jv;
        if (wide_lane) {
          if (have) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
              float y = x[c] * e.rs;
              const bool shut = !(e.g[c] > 0.f);
              if (!p.gate_last) y = shut ? 0.f : y * p.gate_scale;
              y += e.c[c];
              if (p.gate_last) y = shut ? 0.f : y * p.gate_scale;
              x[c] = y;
            }
          }
          if (p.relu_last) {
#pragma unroll
            for (int c = 0; c < 4; ++c) x[c] = fmaxf(x[c], 0.f);
          }
          float4u out;
#pragma unroll
          for (int c = 0; c < 4; ++c) out[c] = x[c];
          *reinterpret_cast<float4u*>(dst) = out;
        } else {
          const float sc = p.row_scale ? p.row_scale[i] : 1.f;
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            if (jv + c < p.N) {
              float y = x[c] * sc;
              const bool shut = p.gate && !(p.gate[i * p.ldg + jv + c] > 0.f);
              if (!p.gate_last) y = shut ? 0.f : y * p.gate_scale;
              if (p.accumulate) y += dst[c];
              if (p.gate_last) y = shut ? 0.f : y * p.gate_scale;
              if (p.relu_last) y = fmaxf(y, 0.f);
              dst[c] = y;
            }
          }
        }
      }
    };
#pragma unroll
    for (int a = 0; a < AM; ++a) {
      Extra e[4] = {};
      if (extras) {
#pragma unroll
        for (int q = 0; q < 4; ++q) request(a, q, e[q]);
      }
      __syncthreads();  // operand tiles (a = 0) / previous block (a = 1) no longer read
#pragma unroll
      for (int b = 0; b < AN; ++b) {
        const int64_t j = j0 + wn * (32 * AN) + b * 32 + r;
        const float bj = (p.bias && j < p.N) ? p.bias[j] : 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float x = acc[a][b][v] + bj;
          if (p.relu) x = fmaxf(x, 0.f);
          st[(8 * (v >> 2) + 4 * g + (v & 3)) * STAGE_LD + b * 32 + r] = x;
        }
      }
      __syncthreads();
      if (extras) {
#pragma unroll
        for (int q0 = 0; q0 < PASSES; q0 += 4) {
          if (q0 > 0) {
#pragma unroll
            for (int q = 0; q < 4; ++q) request(a, q0 + q, e[q]);
          }
#pragma unroll
          for (int q = 0; q < 4; ++q) pass(a, q0 + q, true, e[q]);
        }
      } else {
#pragma unroll
        for (int sidx = 0; sidx < PASSES; ++sidx) pass(a, sidx, false, e[0]);
      }
    }
  }
}

// fixed-order sum of split partials: C[i, j] (+)= sum_z part[z][i][j].  A block owns 32 consecutive
// outputs; eight thread groups each add up every eighth partial (independent loads, batched by the
// unrolling), and the eight group sums are added in order.
constexpr int SR_IDX = 32, SR_ZG = 8;
__global__ __launch_bounds__(256) void split_reduce_kernel(const float* __restrict__ part, int64_t split_stride,
                                                           int32_t splits, float* __restrict__ C, int64_t ldc,
                                                           int32_t rows, int32_t cols, int32_t accumulate) {
  __shared__ float red[SR_ZG][SR_IDX];
  const int ii = threadIdx.x % SR_IDX, zg = threadIdx.x / SR_IDX;
  const int64_t idx = (int64_t)blockIdx.x * SR_IDX + ii;
  const bool ok = idx < (int64_t)rows * cols;
  float s = 0.f;
  if (ok) {
#pragma unroll 8
    for (int z = zg; z < splits; z += SR_ZG) s += part[(int64_t)z * split_stride + idx];
  }
  red[zg][ii] = s;
  __syncthreads();
  if (zg == 0 && ok) {
    float t = red[0][ii];
#pragma unroll
    for (int g = 1; g < SR_ZG; ++g) t += red[g][ii];
    float* dst = C + (idx / cols) * ldc + (idx % cols);
    *dst = accumulate ? *dst + t : t;
  }
}

static int32_t check_grid(int64_t blocks) {
  COFREE_REQUIRE(blocks > 0 && blocks < ((int64_t)1 << 31), "dense: grid too large");
  return COFREE_OK;
}

int32_t launch_gemm(const GemmArgs& a, hipStream_t stream) {
  COFREE_REQUIRE(a.A1 && a.B && a.C, "dense: NULL operand");
  if (a.dtype == COFREE_BF16) return launch_gemm_bf16(a, stream);
  COFREE_REQUIRE(a.dtype == COFREE_F32, "dense: unknown dtype");
  COFREE_REQUIRE(a.M >= 0 && a.N >= 1 && a.K1 >= 1 && a.K2 >= 0, "dense: bad shape");
  COFREE_REQUIRE(a.K2 == 0 || a.A2, "dense: second segment is NULL");
  COFREE_REQUIRE(a.lda1 >= a.K1 && (a.K2 == 0 || a.lda2 >= a.K2), "dense: lda too small");
  COFREE_REQUIRE(a.ldc >= a.N, "dense: ldc too small");
  if (a.M == 0) return COFREE_OK;
  GemmK p{};
  p.A1 = (const float*)a.A1;
  p.lda1 = a.lda1;
  p.K1 = a.K1;
  p.A2 = (const float*)a.A2;
  p.lda2 = a.lda2;
  p.K2 = a.K2;
  p.B = a.B;
  p.ldb = a.ldb;
  p.B2 = a.K2 > 0 ? a.B2 : nullptr;
  p.ldb2 = a.ldb2;
  p.C = (float*)a.C;
  p.ldc = a.ldc;
  p.M = a.M;
  p.N = a.N;
  p.K = (int64_t)a.K1 + a.K2;
  p.k_chunk = p.K;
  p.c_split_stride = 0;
  p.bias = a.bias;
  p.relu = a.relu;
  p.row_scale = a.row_scale;
  p.gate = (const float*)a.gate;
  p.ldg = a.ldg;
  p.accumulate = a.accumulate;
  p.relu_last = a.relu_last;
  p.gate_last = a.gate_last;
  p.gate_scale = a.gate ? a.gate_scale : 1.f;
  const bool narrow = a.N <= 64;  // one 128x64 tile per row panel
  p.tiles_n = narrow ? 1 : (a.N + BN - 1) / BN;
  p.tiles_m = 1;
  p.n_groups = (a.M + BM - 1) / BM;
  const int64_t blocks = ((p.n_groups + 7) / 8) * 8 * p.tiles_n;
  COFREE_TRY(check_grid(blocks));
  const double flops = 2.0 * (double)a.M * a.N * (double)p.K;
  const double bytes = 4.0 * ((double)a.M * p.K + (double)a.N * p.K + (double)a.M * a.N * (a.accumulate ? 2 : 1));
  char pname[96];  // the template instance launched below, then the shape
  snprintf(pname, sizeof(pname), "gemm_kernel<false,%s,%s,%d> N=%d K=%d", a.b_kmajor ? "true" : "false",
           a.b_kmajor && a.N < 4 ? "true" : "false", (a.b_kmajor && a.N < 4) || narrow ? 1 : 0, (int)a.N, (int)p.K);
  ProfScope prof(pname, stream, bytes, flops);
  if (a.b_kmajor) {
    COFREE_REQUIRE(a.ldb >= a.N && (!p.B2 || a.ldb2 >= a.N), "dense: ldb too small");
    if (a.N < 4)
      gemm_kernel<false, true, true, 1><<<dim3((unsigned)blocks), 256, 0, stream>>>(p);
    else if (narrow)
      gemm_kernel<false, true, false, 1><<<dim3((unsigned)blocks), 256, 0, stream>>>(p);
    else
      gemm_kernel<false, true, false, 0><<<dim3((unsigned)blocks), 256, 0, stream>>>(p);
  } else {
    COFREE_REQUIRE(p.B2 ? (a.ldb >= a.K1 && a.ldb2 >= a.K2) : a.ldb >= p.K, "dense: ldb too small");
    if (narrow)
      gemm_kernel<false, false, false, 1><<<dim3((unsigned)blocks), 256, 0, stream>>>(p);
    else
      gemm_kernel<false, false, false, 0><<<dim3((unsigned)blocks), 256, 0, stream>>>(p);
  }
  COFREE_HIP_CHECK(hipGetLastError());
  return COFREE_OK;
}

// Number of k-chunks of a weight gradient.  The chip holds `resident` workgroups of the kernel at once (its
// registers leave three per CU in float32, two in bfloat16) and every workgroup of a launch takes about
// equally long, so a launch is sized to whole rounds of that many workgroups, never a few more (at two per
// CU, 77 chunks x 10 tiles = 770 workgroups ran 1.5 rounds in the time of 2); and as many rounds as it takes
// to have at least 128 chunks, since few long chunks measured slower (256x602 over 230k nodes: 51 chunks
// 73 TFLOP/s, 102 chunks 91, 153 chunks 98).  At least 512 reduction steps per chunk, at most 512 chunks.
int32_t wgrad_splits(int32_t N1, int32_t N2, int64_t M, int32_t resident) {
  const int64_t tiles = (int64_t)((N1 + BM - 1) / BM) * ((N2 + BN - 1) / BN);
  int64_t rounds = 1;
  while (rounds < 8 && resident * rounds / tiles < 128) ++rounds;
  int64_t s = resident * rounds / tiles;
  if (s > 512) s = 512;
  // The workgroups of one split walk the same rows of both operands, each for its own tile of the result, next
  // to each other on one XCD, and nothing but their common start keeps them together: over a long walk they drift
  // apart and every one of them fetches its panels from memory again (28M rows in 128 splits: twice the
  // operands' bytes fetched, L2 hit rate 0.09; at 15k rows per split the second reader hits).  Long reductions
  // therefore get more, shorter splits.
  const int64_t by_walk = std::min<int64_t>(M / 16384, 2048);
  if (s < by_walk) s = by_walk;
  const int64_t max_by_len = (M + 511) / 512;
  if (s > max_by_len) s = max_by_len;
  if (s < 1) s = 1;
  return (int32_t)s;
}

// enough for either storage type
size_t wgrad_workspace_floats(int32_t N1, int32_t N2, int64_t M) {
  const int32_t s32 = wgrad_splits(N1, N2, M, WGRAD_RESIDENT_F32), s16 = wgrad_splits(N1, N2, M, WGRAD_RESIDENT_BF16);
  return (size_t)(s32 > s16 ? s32 : s16) * ((size_t)N1 * (size_t)N2 + (size_t)N1);
}

int32_t launch_split_reduce(const float* partials, int64_t split_stride, int32_t splits, float* C, int64_t ldc,
                            int32_t rows, int32_t cols, int32_t accumulate, hipStream_t stream) {
  const int64_t total = (int64_t)rows * cols;
  ProfScope prof("split_reduce_kernel", stream, 4.0 * (double)total * (splits + 1), (double)total * splits);
  split_reduce_kernel<<<dim3((unsigned)((total + SR_IDX - 1) / SR_IDX)), 256, 0, stream>>>(partials, split_stride, splits, C,
                                                                                 ldc, rows, cols, accumulate);
  COFREE_HIP_CHECK(hipGetLastError());
  return COFREE_OK;
}

int32_t launch_wgrad(int32_t dtype, const void* Av, int64_t lda, int32_t N1, const void* Bv, int64_t ldb, int32_t N2a,
                     int64_t M, float* C, int64_t ldc, int32_t accumulate, float* workspace, hipStream_t stream,
                     float* colsum_out, const void* B2v, int64_t ldb2, int32_t N2b) {
  COFREE_REQUIRE(Av && Bv && C && workspace, "wgrad: NULL operand");
  COFREE_REQUIRE(N1 >= 1 && N2a >= 1 && M >= 0, "wgrad: bad shape");
  COFREE_REQUIRE(!B2v || (N2b >= 1 && N2a % BN == 0 && ldb2 >= N2b), "wgrad: bad second matrix");
  const int32_t N2 = N2a + (B2v ? N2b : 0);  // columns of the result
  COFREE_REQUIRE(lda >= N1 && ldb >= N2a && ldc >= N2, "wgrad: leading dimension too small");
  if (dtype == COFREE_BF16)
    return launch_wgrad_bf16((const bf16_t*)Av, lda, N1, (const bf16_t*)Bv, ldb, N2a, M, C, ldc, accumulate, workspace,
                             stream, colsum_out, (const bf16_t*)B2v, ldb2, N2b);
  COFREE_REQUIRE(dtype == COFREE_F32, "wgrad: unknown dtype");
  const float* A = (const float*)Av;
  const float* B = (const float*)Bv;
  const int32_t S = wgrad_splits(N1, N2, M, WGRAD_RESIDENT_F32);
  GemmK p{};
  p.A1 = A;
  p.lda1 = lda;
  p.K1 = 0;  // unused by k-major loaders
  p.B = B;
  p.ldb = ldb;
  p.B2 = (const float*)B2v;
  p.ldb2 = ldb2;
  p.n_split = B2v ? N2a : 0;
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
  // narrow outputs: 64x128 tiles for at most 64 rows, else 128x64 for at most 64 columns
  const int narrow = N1 <= 64 ? 2 : (N2 <= 64 ? 1 : 0);
  p.tiles_n = narrow == 1 ? 1 : (N2 + BN - 1) / BN;
  p.tiles_m = narrow == 2 ? 1 : (N1 + BM - 1) / BM;
  p.n_groups = S;
  float* colsum_part = workspace + (size_t)S * N1 * N2;
  p.colsum_part = colsum_out ? colsum_part : nullptr;
  const int64_t blocks = (int64_t)((S + 7) / 8) * 8 * p.tiles_m * p.tiles_n;
  COFREE_TRY(check_grid(blocks));
  {
    const bool tiny = N1 < 4 || (B2v ? N2b < 4 : N2 < 4);
    char pname[96];
    snprintf(pname, sizeof(pname), "gemm_kernel<true,true,%s,%d> N=%dx%d", tiny && narrow ? "true" : "false", narrow,
             (int)N1, (int)N2);
    ProfScope prof(pname, stream, 4.0 * ((double)M * N1 + (double)M * N2 + (double)N1 * N2),
                   2.0 * (double)M * N1 * N2);
    const dim3 grid((unsigned)blocks);
    if (narrow == 2) {
      if (tiny) gemm_kernel<true, true, true, 2><<<grid, 256, 0, stream>>>(p);
      else gemm_kernel<true, true, false, 2><<<grid, 256, 0, stream>>>(p);
    } else if (narrow == 1) {
      if (tiny) gemm_kernel<true, true, true, 1><<<grid, 256, 0, stream>>>(p);
      else gemm_kernel<true, true, false, 1><<<grid, 256, 0, stream>>>(p);
    } else {
      gemm_kernel<true, true, false, 0><<<grid, 256, 0, stream>>>(p);
    }
  }
  COFREE_HIP_CHECK(hipGetLastError());
  COFREE_TRY(launch_split_reduce(workspace, p.c_split_stride, S, C, ldc, N1, N2, accumulate, stream));
  if (colsum_out) COFREE_TRY(launch_split_reduce(colsum_part, N1, S, colsum_out, N1, 1, N1, accumulate, stream));
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
