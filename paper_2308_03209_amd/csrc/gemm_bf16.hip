// Dense feature transforms for bfloat16-stored activations: bf16 operands on the matrix cores
// (v_mfma_f32_32x32x16_bf16), float32 accumulation, bf16 or float32 results.
//
// Same tiling as the float32 kernel (128x128 block tile, four wavefronts 2x2, each 64x64 as 2x2
// MFMA accumulators) with k-tiles of 32; large A B^T products use a 256x256 tile of sixteen wavefronts.  LDS tiles are stored row-major [i][k] with rows padded
// to 40 elements (80 bytes), so an MFMA operand (8 consecutive k of one row) is one conflict-free
// ds_read_b128.  Float32 parameters are first converted to a bf16 [N][K] copy by a small kernel,
// so that both products with parameters (C = A W^T and C = A W) read the same operand layout.
// Weight gradients (C = A^T B over the node dimension) read both operands node-major and scatter
// them into the [i][k] LDS layout.
#include <cstdio>
#include <cstdlib>

#include "common.h"

namespace cofree {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4u __attribute__((ext_vector_type(4), aligned(2)));  // 16 bytes, element-aligned

constexpr int HBM = 128, HBN = 128, HBK = 32, HLD = 40;
// A B^T reads 64 k (one 128-byte line of every operand row) per step and keeps HDEPTH_NT such steps in
// flight; weight gradients keep HDEPTH_WG k-tiles of 32 in flight (register budget: 3 / 2 blocks per CU)
constexpr int HDEPTH_NT = 1, HDEPTH_WG = 3;
constexpr int HDEPTH_NARROW = 2;  // outputs of at most 64 columns: half the accumulators, so two steps in flight
constexpr int HHALF = HBM * HLD + 32;  // elements between the two 32-k halves of a 64-k step in LDS (see store)

struct GemmHK {
  const bf16_t* A1;
  int64_t lda1;
  int32_t K1;
  const bf16_t* A2;
  int64_t lda2;
  int32_t K2;
  const bf16_t* B;
  int64_t ldb;
  void* C;
  int64_t ldc;
  int32_t c_f32;  // 1: C is float32 (weight-gradient partials), 0: bf16
  int64_t M;
  int32_t N;
  int64_t K;
  int64_t k_chunk;
  int64_t c_split_stride;
  const float* bias;
  int32_t relu;
  const float* row_scale;
  const bf16_t* gate;
  int64_t ldg;
  int32_t accumulate;
  int32_t relu_last;
  int32_t gate_last;  // the gate applies to the accumulated value
  float gate_scale;   // factor on the elements that pass the gate
  int32_t tiles_n;
  int32_t tiles_m;
  int64_t n_groups;
  float* colsum_part;  // weight gradients: [chunks][M] partial column sums of operand A, or null
  // weight gradients: columns n_split .. of the result come from B2 (0: everything from B)
  const bf16_t* B2;
  int64_t ldb2;
  int32_t n_split;
};

// Movers bring one 128 x 32 operand tile from global memory to LDS in two steps: load() fills a
// thread's share into registers (8 dwords, no use of the data), store() writes it to the [i][k] tile.

// k-contiguous bf16 source, 64 k per step: thread t holds the 8 consecutive k starting at 8(t&7) of the rows
// (t>>3) + 32j, j = 0..3, so eight neighbouring lanes read one whole 128-byte line of a row.  (With 32 k per
// step every line was requested twice, by loads a tile apart, and these memory-bound products are limited
// by line requests, not bytes.)  In LDS the step is two [i][k] tiles of 32 k, HHALF elements apart.
// NJ = row groups of RP a tile has (RP = an eighth of the block's threads: 32 rows for 256 threads; NJ = 4 for
// 128 rows, 2 for the 64-row parameter tile of a narrow product); HALF = elements between the two halves.
template <int NJ, int RP = 32, int HALF = HHALF>
struct HMoverKContig {
  struct Raw {
    u32x4u x[NJ];
  };
  const bf16_t* p[NJ];
  __device__ void init(const bf16_t* P, int64_t ld, int64_t extent, int64_t i0, int tid) {
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      int64_t r = i0 + (tid >> 3) + RP * j;
      if (r > extent - 1) r = extent - 1;
      p[j] = P + r * ld + (tid & 7) * 8;
    }
  }
  __device__ void load(int64_t k0, Raw& w) const {
#pragma unroll
    for (int j = 0; j < NJ; ++j) w.x[j] = *reinterpret_cast<const u32x4u*>(p[j] + k0);
  }
  // Ragged step (k0 + 64 > k_len >= 1).  A thread whose eight k would cross the end of the range reads the
  // eight-wide window that ends with the range instead (one vector load per row on every path, as in a
  // full step) and shifts its valid elements down into place; elements past the end become zero.  Ranges
  // shorter than eight read clamped scalars.
  static __device__ u32x4u shift_down(const u32x4u& w, int halves) {  // 128-bit value >> 16 * halves, no branches
    const uint64_t lo = (uint64_t)w[0] | ((uint64_t)w[1] << 32), hi = (uint64_t)w[2] | ((uint64_t)w[3] << 32);
    const int bits = 16 * halves;             // 0 .. 128
    const int b = bits & 63;                  // shift inside a 64-bit half
    const uint64_t spill = b ? hi << (64 - b) : 0;
    const uint64_t l1 = (lo >> b) | spill, h1 = hi >> b;  // bits < 64
    const uint64_t rl = bits >= 128 ? 0 : (bits >= 64 ? h1 : l1);
    const uint64_t rh = bits >= 64 ? 0 : h1;
    return u32x4u{(uint32_t)rl, (uint32_t)(rl >> 32), (uint32_t)rh, (uint32_t)(rh >> 32)};
  }
  // k_len >= 8: the four window loads are issued back to back and shifted afterwards
  __device__ void load_ragged(int64_t k0, int64_t k_len, int tid, Raw& w) const {
    const int64_t kq = (tid & 7) * 8;
    const int64_t k = k0 + kq;
    int64_t v = k_len - k;  // valid elements of this thread: <= 0 none, >= 8 all
    if (v > 8) v = 8;
    if (v < 0) v = 0;
    const int64_t ks = v == 8 ? k : k_len - 8;  // start of the window that is read
    u32x4u raw[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) raw[j] = *reinterpret_cast<const u32x4u*>(p[j] + (ks - kq));
#pragma unroll
    for (int j = 0; j < NJ; ++j) w.x[j] = shift_down(raw[j], 8 - (int)v);
  }
  // k_len < 8: clamped element loads
  __device__ void load_ragged_short(int64_t k0, int64_t k_len, int tid, Raw& w) const {
    const int64_t kq = (tid & 7) * 8;
    const int64_t k = k0 + kq;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        uint32_t wd = 0u;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int64_t kk = k + 2 * c + h;
          const int64_t kc = kk < k_len ? kk : k_len - 1;
          const uint32_t v = p[j][kc - kq];
          wd |= (kk < k_len ? v : 0u) << (16 * h);
        }
        w.x[j][c] = wd;
      }
    }
  }
  // Lanes 0-3 of an eight-lane group write 64 contiguous bytes of one row of the first half, lanes 4-7 of
  // the second; the 64 bytes of padding in HHALF put the two on different banks.
  __device__ void store(bf16_t* lds, int tid, const Raw& w) const {
    bf16_t* d = lds + ((tid & 7) >> 2) * HALF + (tid >> 3) * HLD + (tid & 3) * 8;
#pragma unroll
    for (int j = 0; j < NJ; ++j)
      *reinterpret_cast<uint4*>(d + RP * j * HLD) = make_uint4(w.x[j][0], w.x[j][1], w.x[j][2], w.x[j][3]);
  }
};

// k-major bf16 source (element (i,k) at P[k*ld + i]): thread t reads the pair i = 2(t&63), +1 of the eight
// k-rows 8(t>>6) .. +7 as dwords (a wavefront reads 256 contiguous bytes of each row); store() transposes
// the 8x2 block in registers and writes two 16-byte rows of the [i][k] LDS tile.  Addresses are a
// block-uniform base plus 32-bit per-thread offsets (the range handed to init spans less than 2^31 elements).
// SINGLE: some tile of the launch may have one valid column only (N mod 128 = 1), where there is no dword
// to read; a template parameter because even a uniform test around every load of the loop cost 16 % of the
// 256x256 weight gradients.
typedef uint32_t u32u __attribute__((aligned(2)));
template <bool SINGLE>
struct HMoverKMajor {
  struct Raw {
    uint32_t w[8];
  };
  const bf16_t* base;   // &P[i0], uniform over the block
  int64_t ld;
  uint32_t off;         // element offset of this thread's dword in k-row 8(t>>6)
  uint32_t sel0, sel1;  // byte selectors that pick column i / i+1 out of two consecutive k-rows
  bool single;          // the tile has one valid column only: no dword to read
  __device__ void init(const bf16_t* P, int64_t ld_, int64_t extent, int64_t i0, int tid) {
    ld = ld_;
    base = P + i0;
    // Columns past the last valid one feed output rows that are never stored; they only have to be
    // read from valid memory.  The dword is moved left until it lies inside the row; when that leaves
    // column i in its upper half, the selector takes it from there.
    const int32_t last = (int32_t)(extent - 1 - i0);
    const int32_t i = 2 * (tid & 63);
    single = last < 1;
    int32_t ia = i;
    if (ia > last - 1) ia = last - 1;
    if (ia < 0) ia = 0;
    off = (uint32_t)((tid >> 6) * 8) * (uint32_t)ld + (uint32_t)ia;
    sel0 = (i == last && ia == i - 1) ? 0x07060302u : 0x05040100u;
    sel1 = 0x07060302u;
  }
  __device__ uint32_t load_pair(const bf16_t* row0, uint32_t o) const {
    if constexpr (SINGLE) {
      if (single) return (uint32_t)row0[o];
    }
    return *reinterpret_cast<const u32u*>(row0 + o);
  }
  __device__ void load(int64_t k0, Raw& r) const {
    const bf16_t* row0 = base + k0 * ld;
#pragma unroll
    for (int c = 0; c < 8; ++c) r.w[c] = load_pair(row0, off + (uint32_t)c * (uint32_t)ld);
  }
  // Ragged tile, branch-free: rows past the end are read from the last valid row and zeroed.
  __device__ void load_ragged(int64_t k0, int64_t k_len, int tid, Raw& r) const {
    const int64_t kq = (tid >> 6) * 8;
    const uint32_t col = off - (uint32_t)kq * (uint32_t)ld;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const int64_t k = k0 + kq + c;
      const int64_t kc = k < k_len ? k : k_len - 1;
      const uint32_t v = load_pair(base + kc * ld, col);
      r.w[c] = k < k_len ? v : 0u;
    }
  }
  __device__ void store(bf16_t* lds, int tid, const Raw& r) const {
    uint32_t x0[4], x1[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      x0[c] = __builtin_amdgcn_perm(r.w[2 * c + 1], r.w[2 * c], sel0);
      x1[c] = __builtin_amdgcn_perm(r.w[2 * c + 1], r.w[2 * c], sel1);
    }
    bf16_t* d = lds + (2 * (tid & 63)) * HLD + (tid >> 6) * 8;
    *reinterpret_cast<uint4*>(d) = make_uint4(x0[0], x0[1], x0[2], x0[3]);
    *reinterpret_cast<uint4*>(d + HLD) = make_uint4(x1[0], x1[1], x1[2], x1[3]);
  }
};

// 32 k-steps of one LDS tile pair: 8 MFMAs per wavefront on its 64x64 sub-tile (AN = 2), 4 on 64x32 (AN = 1).
template <int AN>
__device__ inline void compute_tile_bf16(const bf16_t* __restrict__ as, const bf16_t* __restrict__ bs,
                                         floatx16 (&acc)[2][AN]) {
#pragma unroll
  for (int step = 0; step < 2; ++step) {
    const bf16x8 a0 = *reinterpret_cast<const bf16x8*>(as + step * 16);
    const bf16x8 a1 = *reinterpret_cast<const bf16x8*>(as + 32 * HLD + step * 16);
#pragma unroll
    for (int n = 0; n < AN; ++n) {
      const bf16x8 b = *reinterpret_cast<const bf16x8*>(bs + n * 32 * HLD + step * 16);
      acc[0][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b, acc[0][n], 0, 0, 0);
      acc[1][n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b, acc[1][n], 0, 0, 0);
    }
  }
}

// do_colsum (uniform over the block): thread t < 128 also adds up row t of the A tiles over k.
//
// Global loads run D k-tiles ahead of the MFMAs in a ring of registers (slot = tile mod D, static after
// unrolling), so a block keeps D tiles of both operands in flight; LDS is double-buffered with one
// barrier per tile: tile t is stored, the barrier passes, tile t is multiplied, and the store of tile
// t+1 goes to the other buffer, which every wavefront stopped reading before that barrier.
template <int D, typename MA, typename MB>
__device__ inline void run_range_bf16(const MA& ma, const MB& mb, int64_t k_len, bf16_t* As0, bf16_t* Bs0,
                                      floatx16 (&acc)[2][2], int tid, bool do_colsum, float& colsum) {
  auto add_colsum = [&](const bf16_t* tile) {
    if (do_colsum && tid < HBM) {
      float s = 0.f;
#pragma unroll
      for (int q = 0; q < HBK / 8; ++q) {
        const uint4 w = *reinterpret_cast<const uint4*>(tile + tid * HLD + q * 8);
        const uint32_t ws[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) s += __uint_as_float(ws[c] << 16) + __uint_as_float(ws[c] & 0xffff0000u);
      }
      colsum += s;
    }
  };
  const int lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, r = lane & 31;
  // lane (r, g) feeds row r of a 32-row block with k = 8g .. 8g+7 of each 16-wide MFMA step
  const int a_off = ((wave >> 1) * 64 + r) * HLD + g * 8;
  const int b_off = ((wave & 1) * 64 + r) * HLD + g * 8;
  const int64_t n_full = k_len / HBK;
  typename MA::Raw ra[D];
  typename MB::Raw rb[D];
  __syncthreads();  // whoever used the LDS tiles before is done
  if (n_full > 0) {
    // Loads are unconditional (past the end they repeat the last tile, an L2 hit), which keeps the count
    // of outstanding loads the same on every path, so that a store waits for its own slot only.
    const int64_t t_last = n_full - 1;
    auto step = [&](int64_t t, int s, bool refill) {
      bf16_t* const at = As0 + (int)(t & 1) * (HBM * HLD);
      bf16_t* const bt = Bs0 + (int)(t & 1) * (HBN * HLD);
      ma.store(at, tid, ra[s]);
      mb.store(bt, tid, rb[s]);
      if (refill) {
        const int64_t tn = t + D < t_last ? t + D : t_last;
        ma.load(tn * HBK, ra[s]);
        mb.load(tn * HBK, rb[s]);
      }
      __syncthreads();
      compute_tile_bf16<2>(at + a_off, bt + b_off, acc);
      add_colsum(at);
    };
#pragma unroll
    for (int s = 0; s < D; ++s) {
      const int64_t tn = s < t_last ? s : t_last;
      ma.load(tn * HBK, ra[s]);
      mb.load(tn * HBK, rb[s]);
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
  if (n_full * HBK < k_len) {
    bf16_t* const at = As0 + (int)(n_full & 1) * (HBM * HLD);
    bf16_t* const bt = Bs0 + (int)(n_full & 1) * (HBN * HLD);
    ma.load_ragged(n_full * HBK, k_len, tid, ra[0]);
    mb.load_ragged(n_full * HBK, k_len, tid, rb[0]);
    ma.store(at, tid, ra[0]);
    mb.store(bt, tid, rb[0]);
    __syncthreads();
    compute_tile_bf16<2>(at + a_off, bt + b_off, acc);
    add_colsum(at);
  }
}

// A B^T: steps of 64 k through one LDS buffer (the two 32-k tiles of a step fill what is a double buffer for
// the weight gradients): store a step, barrier, 16 MFMAs per wavefront, barrier.  Global loads run D steps
// ahead in a ring of registers; they are unconditional (past the last full step they repeat it), so that a
// store waits for its own slot only.  A ragged last step is read after the loop.
// a_off / b_off: this lane's operand position inside a 32-k tile; a_half / b_half: elements between the two
// 32-k tiles of a step.
template <int D, int AN, typename MA, typename MB>
__device__ inline void run_steps_bf16(const MA& ma, const MB& mb, int64_t k_len, bf16_t* As0, bf16_t* Bs0,
                                      int a_off, int b_off, int a_half, int b_half, floatx16 (&acc)[2][AN],
                                      int tid) {
  const int64_t n_full = k_len / 64;
  typename MA::Raw ra[D];
  typename MB::Raw rb[D];
  if (n_full > 0) {
    const int64_t t_last = n_full - 1;
    auto step = [&](int64_t t, int s, bool refill) {
      __syncthreads();  // whoever read the LDS tiles before is done
      ma.store(As0, tid, ra[s]);
      mb.store(Bs0, tid, rb[s]);
      if (refill) {
        const int64_t tn = t + D < t_last ? t + D : t_last;
        ma.load(tn * 64, ra[s]);
        mb.load(tn * 64, rb[s]);
      }
      __syncthreads();
      compute_tile_bf16<AN>(As0 + a_off, Bs0 + b_off, acc);
      compute_tile_bf16<AN>(As0 + a_half + a_off, Bs0 + b_half + b_off, acc);
    };
#pragma unroll
    for (int s = 0; s < D; ++s) {
      const int64_t tn = s < t_last ? s : t_last;
      ma.load(tn * 64, ra[s]);
      mb.load(tn * 64, rb[s]);
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
  if (n_full * 64 < k_len) {
    if (k_len >= 8) {
      ma.load_ragged(n_full * 64, k_len, tid, ra[0]);
      mb.load_ragged(n_full * 64, k_len, tid, rb[0]);
    } else {
      ma.load_ragged_short(n_full * 64, k_len, tid, ra[0]);
      mb.load_ragged_short(n_full * 64, k_len, tid, rb[0]);
    }
    __syncthreads();
    ma.store(As0, tid, ra[0]);
    mb.store(Bs0, tid, rb[0]);
    __syncthreads();
    compute_tile_bf16<AN>(As0 + a_off, Bs0 + b_off, acc);
    if (n_full * 64 + 32 < k_len) compute_tile_bf16<AN>(As0 + a_half + a_off, Bs0 + b_half + b_off, acc);
  }
}

// WGRAD = false: C = [A1 | A2] B^T, all operands k-contiguous bf16.
// WGRAD = true : C = A1^T B over k = graph nodes, both operands k-major bf16, float32 partials.
// NARROW (A B^T only): outputs of at most 64 columns use a 128x64 block tile, each wavefront 64x32.
// WM x WN (A B^T only): wavefronts of a block, each 64x64 - 2x2 is the 128x128 tile, 4x4 a 256x256 tile of
// 1024 threads, one block per CU.  It exists because these products are limited by the rate at which a CU's
// L1 takes in 128-byte lines, and a k-step of a TM x TN tile requests TM + TN lines for TM TN outputs: the
// larger tile asks for every operand row half as often.  (Its 128 registers per lane leave room for one
// step in flight only, which is why it gains 7-16 % and not the factor the line count suggests; a 128x256
// tile of 512 threads spilled and was slower than 128x128.)
constexpr int STAGE_LD = 68;               // floats per staged result row
constexpr int STAGE_WAVE = 32 * STAGE_LD;  // floats of result staging per wavefront
template <int WM, int WN>
constexpr size_t bf16_lds_bytes() {
  constexpr size_t operands = (size_t)(2 * (64 * WM * HLD + 32) + 2 * (64 * WN * HLD + 32)) * sizeof(bf16_t);
  constexpr size_t staging = (size_t)WM * WN * STAGE_WAVE * sizeof(float);
  return operands > staging ? operands : staging;
}

template <bool WGRAD, bool SINGLE, bool NARROW, int WM = 2, int WN = 2>
__global__ __launch_bounds__(64 * WM * WN)
    __attribute__((amdgpu_waves_per_eu(WGRAD ? 2 : (WM * WN > 4 ? 4 : 3)))) void gemm_bf16_kernel(const GemmHK p) {
  static_assert((WM == 2 && WN == 2) || (!WGRAD && !NARROW), "larger tiles: plain A B^T only");
  constexpr int AN = NARROW ? 1 : 2;     // 32-column blocks per wavefront
  constexpr int TM = 64 * WM;            // block tile rows
  constexpr int TN = 32 * AN * WN;       // block tile columns
  constexpr int RP = 8 * WM * WN;        // operand rows the block's threads load per pass
  constexpr int HALF_A = TM * HLD + 32;  // elements between the two 32-k halves of a step (HHALF for 128 rows)
  constexpr int HALF_B = (WM == 2 && WN == 2) ? HHALF : TN * HLD + 32;
  // operand tiles during the k loop; afterwards the same memory stages the result tile
  __shared__ __attribute__((aligned(16))) unsigned char smem[bf16_lds_bytes<WM, WN>()];
  bf16_t* const As = reinterpret_cast<bf16_t*>(smem);
  bf16_t* const Bs = As + 2 * HALF_A;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  // XCD-aware linear id -> (group, member), as in the float32 kernel
  int64_t i0, j0, z;
  {
    const int64_t L = blockIdx.x;
    const int64_t per_group = WGRAD ? p.tiles_m * p.tiles_n : p.tiles_n;
    const int64_t group = (L / (8 * per_group)) * 8 + (L & 7);
    const int64_t member = (L >> 3) % per_group;
    if (group >= p.n_groups) return;
    if constexpr (WGRAD) {
      z = group;
      i0 = (member / p.tiles_n) * HBM;
      j0 = (member % p.tiles_n) * HBN;
    } else {
      z = 0;
      i0 = group * TM;
      j0 = member * TN;
    }
  }
  floatx16 acc[2][AN];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < AN; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  if constexpr (!WGRAD) {
    // one loop body for both K-segments (two inlined copies would each claim their own accumulators)
    const int n_seg = p.K2 > 0 ? 2 : 1;
#pragma nounroll
    for (int seg = 0; seg < n_seg; ++seg) {
      HMoverKContig<TM / RP, RP, HALF_A> ma;
      HMoverKContig<TN / RP, RP, HALF_B> mb;
      ma.init(seg ? p.A2 : p.A1, seg ? p.lda2 : p.lda1, p.M, i0, tid);
      mb.init(p.B + (seg ? p.K1 : 0), p.ldb, p.N, j0, tid);
      run_steps_bf16<NARROW ? HDEPTH_NARROW : HDEPTH_NT, AN>(
          ma, mb, seg ? p.K2 : p.K1, As, Bs, ((wm * 64 + (lane & 31)) * HLD + (lane >> 5) * 8),
          ((wn * (32 * AN) + (lane & 31)) * HLD + (lane >> 5) * 8), HALF_A, HALF_B, acc, tid);
    }
  } else {
    const int64_t k_beg = z * p.k_chunk;
    const int64_t k_end = (k_beg + p.k_chunk < p.K) ? k_beg + p.k_chunk : p.K;
    const int64_t k_len = k_end > k_beg ? k_end - k_beg : 0;
    if (k_len > 0) {
      HMoverKMajor<SINGLE> ma, mb;
      ma.init(p.A1 + k_beg * p.lda1, p.lda1, p.M, i0, tid);
      if (p.n_split > 0 && j0 >= p.n_split)  // a column tile of the second matrix (uniform over the block)
        mb.init(p.B2 + k_beg * p.ldb2, p.ldb2, p.N - p.n_split, j0 - p.n_split, tid);
      else
        mb.init(p.B + k_beg * p.ldb, p.ldb, p.n_split > 0 ? p.n_split : p.N, j0, tid);
      float csum = 0.f;
      const bool do_colsum = p.colsum_part != nullptr && j0 == 0;
      if constexpr (!NARROW) run_range_bf16<HDEPTH_WG>(ma, mb, k_len, As, Bs, acc, tid, do_colsum, csum);
      if (do_colsum && tid < HBM && i0 + tid < p.M) p.colsum_part[z * p.M + i0 + tid] = csum;
    } else if (p.colsum_part != nullptr && j0 == 0 && tid < HBM && i0 + tid < p.M) {
      p.colsum_part[z * p.M + i0 + tid] = 0.f;
    }
  }

  const int g = lane >> 5, r = lane & 31;
  if constexpr (WGRAD) {
    // float32 partial of this k-chunk
#pragma unroll
    for (int a = 0; a < 2; ++a) {
#pragma unroll
      for (int b = 0; b < AN; ++b) {
        const int64_t j = j0 + wn * 64 + b * 32 + r;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int64_t i = i0 + wm * 64 + a * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
          if (j < p.N && i < p.M) ((float*)p.C)[z * p.c_split_stride + i * p.ldc + j] = acc[a][b][v];
        }
      }
    }
  } else {
    // Each wavefront passes its 64x64 result through LDS in two 32-row halves, so that a lane ends up
    // with 8 consecutive columns of one row: gate and accumulate operands are read, and the result is
    // written, 16 bytes at a time.  Those operands (and the row scales) do not depend on the product, so
    // they are requested two passes at a time - unconditionally, at clamped addresses, the first pair of
    // a half before its staging barriers - instead of one by one between the stores: load, wait, load,
    // wait, store per pass had made a block's epilogue a chain of up to thirty memory round trips.
    constexpr int SLD = STAGE_LD;  // floats per staged row
    static_assert(WM * WN * STAGE_WAVE * sizeof(float) <= sizeof(smem), "staging does not fit");
    float* const st = reinterpret_cast<float*>(smem) + wave * STAGE_WAVE;
    constexpr int LPR = 4 * AN;       // lanes per staged row (8 columns each)
    constexpr int RPP = 64 / LPR;     // rows per pass
    constexpr int PASSES = 32 / RPP;  // passes per half: 4 or 2
    const int er = lane / LPR, ec = (lane % LPR) * 8;
    const int64_t jv = j0 + wn * (32 * AN) + ec;
    bf16_t* const Cb = (bf16_t*)p.C;
    const bool wide_lane = jv + 8 <= p.N;     // the lane's eight columns all exist
    const int64_t jl = wide_lane ? jv : 0;    // where its 16-byte operand loads go (in range once N >= 8)
    const bool extras = (p.gate || p.accumulate || p.row_scale) && p.N >= 8;  // uniform over the launch
    struct Extra {
      u32x4u g, c;
      float rs;
    };
    auto request = [&](int a, int s, Extra& e) {
      int64_t il = i0 + wm * 64 + a * 32 + s * RPP + er;
      if (il > p.M - 1) il = p.M - 1;
      e.g = u32x4u{0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};  // ones: everything passes
      e.c = u32x4u{0u, 0u, 0u, 0u};
      e.rs = 1.f;
      if (p.gate) e.g = *reinterpret_cast<const u32x4u*>(p.gate + il * p.ldg + jl);
      if (p.accumulate) e.c = *reinterpret_cast<const u32x4u*>(Cb + il * p.ldc + jl);
      if (p.row_scale) e.rs = p.row_scale[il];
    };
    auto half_of = [](const u32x4u& q, int c) {
      return bf16_to_f32((bf16_t)(c & 1 ? q[c >> 1] >> 16 : q[c >> 1] & 0xffffu));
    };
    // one pass: row s*RPP + er of the staged half; e = its operands if they were requested (wide lanes only)
    auto pass = [&](int a, int s, bool have, const Extra& e) {
      const int row = s * RPP + er;
      const int64_t i = i0 + wm * 64 + a * 32 + row;
      if (i < p.M && jv < p.N) {
        float x[8];
        {
          const float4 lo = *reinterpret_cast<const float4*>(st + row * SLD + ec);
          const float4 hi = *reinterpret_cast<const float4*>(st + row * SLD + ec + 4);
          x[0] = lo.x, x[1] = lo.y, x[2] = lo.z, x[3] = lo.w, x[4] = hi.x, x[5] = hi.y, x[6] = hi.z, x[7] = hi.w;
        }
        bf16_t* dst = Cb + i * p.ldc + jv;
        if (wide_lane) {
          if (have) {
#pragma unroll
            for (int c = 0; c < 8; ++c) {
              float y = x[c] * e.rs;
              const bool shut = !(half_of(e.g, c) > 0.f);
              if (!p.gate_last) y = shut ? 0.f : y * p.gate_scale;
              y += half_of(e.c, c);
              if (p.gate_last) y = shut ? 0.f : y * p.gate_scale;
              x[c] = y;
            }
          }
          if (p.relu_last) {
#pragma unroll
            for (int c = 0; c < 8; ++c) x[c] = fmaxf(x[c], 0.f);
          }
          u32x4u out;
#pragma unroll
          for (int c = 0; c < 4; ++c) out[c] = pack_bf16x2(x[2 * c], x[2 * c + 1]);
          *reinterpret_cast<u32x4u*>(dst) = out;
        } else {
          const float sc = p.row_scale ? p.row_scale[i] : 1.f;
#pragma unroll
          for (int c = 0; c < 8; ++c) {
            if (jv + c < p.N) {
              float y = x[c] * sc;
              const bool off = p.gate && !(bf16_to_f32(p.gate[i * p.ldg + jv + c]) > 0.f);
              if (!p.gate_last) y = off ? 0.f : y * p.gate_scale;
              if (p.accumulate) y += bf16_to_f32(dst[c]);
              if (p.gate_last) y = off ? 0.f : y * p.gate_scale;
              if (p.relu_last) y = fmaxf(y, 0.f);
              dst[c] = f32_to_bf16(y);
            }
          }
        }
      }
    };
#pragma unroll
    for (int a = 0; a < 2; ++a) {
      Extra e0{}, e1{};
      if (extras) {
        request(a, 0, e0);
        request(a, 1, e1);
      }
      __syncthreads();  // operand tiles (a = 0) / previous half (a = 1) no longer read
#pragma unroll
      for (int b = 0; b < AN; ++b) {
        const int64_t j = j0 + wn * (32 * AN) + b * 32 + r;
        const float bj = (p.bias && j < p.N) ? p.bias[j] : 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = 8 * (v >> 2) + 4 * g + (v & 3);
          float x = acc[a][b][v] + bj;
          if (p.relu) x = fmaxf(x, 0.f);
          st[row * SLD + b * 32 + r] = x;
        }
      }
      __syncthreads();
      if (extras) {
#pragma unroll
        for (int s0 = 0; s0 < PASSES; s0 += 2) {
          if (s0 > 0) {
            request(a, s0, e0);
            request(a, s0 + 1, e1);
          }
          pass(a, s0, true, e0);
          pass(a, s0 + 1, true, e1);
        }
      } else {
#pragma unroll
        for (int s = 0; s < PASSES; ++s) pass(a, s, false, e0);
      }
    }
  }
}

// dst[j][k0 + k] = bf16(W(j,k)) for j < N, k < K; zero for K <= k < width.
__global__ __launch_bounds__(256) void convert_params_kernel(const float* __restrict__ W, int64_t ld, int32_t kmajor,
                                                             int32_t N, int64_t K, bf16_t* __restrict__ dst,
                                                             int64_t ldd, int64_t k0, int64_t width) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)N * width) return;
  const int64_t j = idx / width, k = idx % width;
  float x = 0.f;
  if (k < K) x = kmajor ? W[k * ld + j] : W[j * ld + k];
  dst[j * ldd + k0 + k] = f32_to_bf16(x);
}

static int64_t pad8(int64_t k) { return (k + 7) & ~(int64_t)7; }
size_t gemm_param_scratch_bytes(int32_t N, int64_t K) { return (size_t)N * (size_t)pad8(K) * sizeof(bf16_t); }

int32_t launch_gemm_bf16(const GemmArgs& a, hipStream_t stream) {
  COFREE_REQUIRE(a.M >= 0 && a.N >= 1 && a.K1 >= 1 && a.K2 >= 0, "dense: bad shape");
  COFREE_REQUIRE(a.K2 == 0 || a.A2, "dense: second segment is NULL");
  COFREE_REQUIRE(a.lda1 >= a.K1 && (a.K2 == 0 || a.lda2 >= a.K2), "dense: lda too small");
  COFREE_REQUIRE(a.ldc >= a.N, "dense: ldc too small");
  COFREE_REQUIRE(a.param_scratch != nullptr, "dense: bf16 products need param_scratch");
  if (a.M == 0) return COFREE_OK;
  const int64_t K = (int64_t)a.K1 + a.K2;
  const bool two = a.K2 > 0 && a.B2;  // the second segment has its own parameter matrix
  if (two)
    COFREE_REQUIRE(a.b_kmajor ? (a.ldb >= a.N && a.ldb2 >= a.N) : (a.ldb >= a.K1 && a.ldb2 >= a.K2),
                   "dense: ldb too small");
  else
    COFREE_REQUIRE(a.b_kmajor ? a.ldb >= a.N : a.ldb >= K, "dense: ldb too small");
  const int64_t ldd = pad8(K);
  bf16_t* Wb = (bf16_t*)a.param_scratch;
  {
    // columns [0, K) of the copy from B (or [0, K1) from B and [K1, K) from B2), zeros up to ldd
    const int64_t kb = two ? a.K1 : K;
    const int64_t total = (int64_t)a.N * ldd;
    ProfScope prof("convert_params_kernel", stream, 6.0 * (double)total, 0.0);
    convert_params_kernel<<<dim3((unsigned)((total + 255) / 256)), 256, 0, stream>>>(a.B, a.ldb, a.b_kmajor, a.N, kb,
                                                                                     Wb, ldd, 0, ldd);
    if (two) {
      const int64_t total2 = (int64_t)a.N * a.K2;
      convert_params_kernel<<<dim3((unsigned)((total2 + 255) / 256)), 256, 0, stream>>>(a.B2, a.ldb2, a.b_kmajor, a.N,
                                                                                        a.K2, Wb, ldd, a.K1, a.K2);
    }
  }
  GemmHK p{};
  p.A1 = (const bf16_t*)a.A1;
  p.lda1 = a.lda1;
  p.K1 = a.K1;
  p.A2 = (const bf16_t*)a.A2;
  p.lda2 = a.lda2;
  p.K2 = a.K2;
  p.B = Wb;
  p.ldb = ldd;
  p.C = a.C;
  p.ldc = a.ldc;
  p.c_f32 = 0;
  p.M = a.M;
  p.N = a.N;
  p.K = K;
  p.k_chunk = K;
  p.bias = a.bias;
  p.relu = a.relu;
  p.row_scale = a.row_scale;
  p.gate = (const bf16_t*)a.gate;
  p.ldg = a.ldg;
  p.accumulate = a.accumulate;
  p.relu_last = a.relu_last;
  p.gate_last = a.gate_last;
  p.gate_scale = a.gate ? a.gate_scale : 1.f;
  const bool narrow = a.N <= 64;  // one 128x64 tile per row panel
  p.tiles_n = narrow ? 1 : (a.N + HBN - 1) / HBN;
  p.tiles_m = 1;
  p.n_groups = (a.M + HBM - 1) / HBM;
  const int64_t blocks = ((p.n_groups + 7) / 8) * 8 * p.tiles_n;
  COFREE_REQUIRE(blocks > 0 && blocks < ((int64_t)1 << 31), "dense: grid too large");
  const double flops = 2.0 * (double)a.M * a.N * (double)K;
  const double bytes = 2.0 * ((double)a.M * K + (double)a.N * K + (double)a.M * a.N * (a.accumulate ? 2 : 1));
  // 256x256 tiles once the matrix gives every CU more than one of them (one such block fills a CU, so small
  // launches keep the 128x128 tile and its three blocks per CU).  COFREE_BF16_TILE = 256 / 128 forces a
  // choice (tests run small shapes through the large tile with it).
  bool big = !narrow && a.N > HBN && a.M >= (int64_t)2 * 256 * 256;
  if (const char* e = getenv("COFREE_BF16_TILE")) {
    if (atoi(e) == 256) big = !narrow && a.N > HBN;
    if (atoi(e) == 128) big = false;
  }
  char pname[96];  // the template instance launched below, then the shape
  snprintf(pname, sizeof(pname), "gemm_bf16_kernel<false,false,%s> N=%d K=%d", big ? "false,4,4" : (narrow ? "true,2,2" : "false,2,2"),
           (int)a.N, (int)K);
  ProfScope prof(pname, stream, bytes, flops);
  if (big) {
    p.tiles_n = (a.N + 255) / 256;
    p.n_groups = (a.M + 255) / 256;
    const int64_t wblocks = ((p.n_groups + 7) / 8) * 8 * p.tiles_n;
    COFREE_REQUIRE(wblocks > 0 && wblocks < ((int64_t)1 << 31), "dense: grid too large");
    gemm_bf16_kernel<false, false, false, 4, 4><<<dim3((unsigned)wblocks), 1024, 0, stream>>>(p);
  } else if (narrow)
    gemm_bf16_kernel<false, false, true><<<dim3((unsigned)blocks), 256, 0, stream>>>(p);
  else
    gemm_bf16_kernel<false, false, false><<<dim3((unsigned)blocks), 256, 0, stream>>>(p);
  COFREE_HIP_CHECK(hipGetLastError());
  return COFREE_OK;
}

int32_t launch_wgrad_bf16(const bf16_t* A, int64_t lda, int32_t N1, const bf16_t* B, int64_t ldb, int32_t N2a,
                          int64_t M, float* C, int64_t ldc, int32_t accumulate, float* workspace,
                          hipStream_t stream, float* colsum_out, const bf16_t* B2, int64_t ldb2, int32_t N2b) {
  const int32_t N2 = N2a + (B2 ? N2b : 0);  // columns of the result
  const int32_t S = wgrad_splits(N1, N2, M, WGRAD_RESIDENT_BF16);
  GemmHK p{};
  p.A1 = A;
  p.lda1 = lda;
  p.B = B;
  p.ldb = ldb;
  p.B2 = B2;
  p.ldb2 = ldb2;
  p.n_split = B2 ? N2a : 0;
  p.C = workspace;
  p.ldc = N2;
  p.c_f32 = 1;
  p.M = N1;
  p.N = N2;
  p.K = M;
  int64_t chunk = (M + S - 1) / S;
  chunk = ((chunk + HBK - 1) / HBK) * HBK;
  if (chunk < HBK) chunk = HBK;
  p.k_chunk = chunk;
  p.c_split_stride = (int64_t)N1 * N2;
  p.tiles_n = (N2 + HBN - 1) / HBN;
  p.tiles_m = (N1 + HBM - 1) / HBM;
  p.n_groups = S;
  float* colsum_part = workspace + (size_t)S * N1 * N2;
  p.colsum_part = colsum_out ? colsum_part : nullptr;
  const int64_t blocks = (int64_t)((S + 7) / 8) * 8 * p.tiles_m * p.tiles_n;
  COFREE_REQUIRE(blocks > 0 && blocks < ((int64_t)1 << 31), "wgrad: grid too large");
  {
    const bool single = N1 % HBM == 1 || N2a % HBN == 1 || (B2 && N2b % HBN == 1);
    char pname[96];
    snprintf(pname, sizeof(pname), "gemm_bf16_kernel<true,%s,false,2,2> N=%dx%d", single ? "true" : "false", (int)N1, (int)N2);
    ProfScope prof(pname, stream, 2.0 * ((double)M * N1 + (double)M * N2) + 4.0 * (double)N1 * N2,
                   2.0 * (double)M * N1 * N2);
    if (single)
      gemm_bf16_kernel<true, true, false><<<dim3((unsigned)blocks), 256, 0, stream>>>(p);
    else
      gemm_bf16_kernel<true, false, false><<<dim3((unsigned)blocks), 256, 0, stream>>>(p);
  }
  COFREE_HIP_CHECK(hipGetLastError());
  COFREE_TRY(launch_split_reduce(workspace, p.c_split_stride, S, C, ldc, N1, N2, accumulate, stream));
  if (colsum_out) COFREE_TRY(launch_split_reduce(colsum_part, N1, S, colsum_out, N1, 1, N1, accumulate, stream));
  return COFREE_OK;
}

}  // namespace cofree
