// Bare gather micro-benchmark: what the memory system of one MI355X gives a kernel that does nothing but the
// aggregation's access pattern - a coalesced read of neighbour ids, then for every id one contiguous segment of a
// row of a big matrix, fetched with 16 bytes per lane - without scales, gates, tails or any arithmetic beyond
// the additions that keep the loads alive.  Not part of the library: a stand-alone program whose numbers are the
// yardstick the aggregation kernels are held against (build: paper_2308_03209_amd/build.py; run: ./gather_ceiling).
//
// Cases
//   stream   : every wavefront reads whole 1 KiB blocks of a buffer front to back (16 bytes per lane), the
//              buffer sized to stay in one XCD's L2 (x8 XCDs), in the 256 MB memory-side cache, or in neither.
//   gather   : `rows` lists of `deg` uniformly random row ids out of a window of `window` matrix rows; a group of
//              LPS lanes fetches SEG = LPS * 16 bytes of each listed row (64 / LPS ids per load instruction, four
//              instructions in flight), one wavefront per list, as the neighbour-group kernel does.  With
//              SLICES = 8 workgroup b works on column slice b % 8 of list group b / 8 (workgroups are dealt
//              round-robin to the XCDs, so an XCD's L2 sees one eighth of every row).
//   sweep    : the same 14M gathers of 128-byte slices, reordered as a source-blocked schedule would issue them: a
//              grid that is resident all at once (8 slices x 256 workgroups), every wavefront going `rounds` times
//              through the B source blocks of the matrix in ascending order and fetching its share of ids of block
//              b only while it is there.  Nothing synchronises the workgroups after their common start.  It
//              measures how much of the L2-resident gather rate such a schedule could reach at best (no per-row
//              bookkeeping, sums kept in registers).
// Output per case: microseconds per launch (HIP events, mean of the timed launches), bytes requested per second,
// and for gathers the 128-byte lines requested per second and per compute-unit clock (256 CUs at 2.4 GHz).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cstdio>
#include <cstdlib>
#include <vector>

#define CHECK(x)                                                                              \
  do {                                                                                        \
    hipError_t e_ = (x);                                                                      \
    if (e_ != hipSuccess) {                                                                   \
      fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_));                          \
      exit(1);                                                                                \
    }                                                                                         \
  } while (0)

typedef float f32x4 __attribute__((ext_vector_type(4)));

// every wavefront streams 1 KiB blocks; `sink` is written only if a sum is NaN (it never is: the buffer holds
// small finite values), which keeps the loads from being optimised away
__global__ __launch_bounds__(256) void stream_read_kernel(const f32x4* __restrict__ buf, int64_t n_vec, int passes,
                                                          float* __restrict__ sink) {
  const int64_t stride = (int64_t)gridDim.x * 256;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int p = 0; p < passes; ++p) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < n_vec; i += 4 * stride) {
      const f32x4 a = buf[i], b = buf[i + stride], c = buf[i + 2 * stride], d = buf[i + 3 * stride];
      acc += (a + b) + (c + d);
    }
    for (; i < n_vec; i += stride) acc += buf[i];
  }
  const float s = acc[0] + acc[1] + acc[2] + acc[3];
  if (s != s) sink[0] = s;
}

// one wavefront per (list, slice); ids: [rows][deg]; table: [window rows][row_floats] float32
template <int LPS, int SLICES>
__global__ __launch_bounds__(256) void gather_kernel(const int32_t* __restrict__ ids, int64_t rows, int deg,
                                                     const float* __restrict__ table, int64_t row_floats,
                                                     float* __restrict__ out) {
  constexpr int NG = 64 / LPS, UNR = 4;
  const int lane = threadIdx.x & 63, sub = lane % LPS, grp = lane / LPS;
  const int slice = SLICES == 1 ? 0 : (int)(blockIdx.x % (unsigned)SLICES);
  const int64_t row = (int64_t)(blockIdx.x / (unsigned)SLICES) * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int c0 = slice * (LPS * 4) + sub * 4;
  const int32_t* __restrict__ my = ids + row * deg;
  const float* __restrict__ src = table + c0;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  const int last = deg - 1;
  for (int e = grp; e < deg; e += NG * UNR) {
    int u[UNR];
    f32x4 v[UNR];
#pragma unroll
    for (int t = 0; t < UNR; ++t) {
      const int ee = e + t * NG;
      u[t] = my[ee < last ? ee : last];
    }
#pragma unroll
    for (int t = 0; t < UNR; ++t) v[t] = *reinterpret_cast<const f32x4*>(src + (int64_t)u[t] * row_floats);
#pragma unroll
    for (int t = 0; t < UNR; ++t)
      if (e + t * NG < deg) acc += v[t];
  }
#pragma unroll
  for (int off = LPS; off < 64; off <<= 1) {
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] += __shfl_xor(acc[i], off, 64);
  }
  if (grp == 0) *reinterpret_cast<f32x4*>(out + row * row_floats + c0) = acc;
}

// ids: [wg slot][round][block][wave][per_visit]; grid = 8 slices x wg slots, all resident
__global__ __launch_bounds__(256) void gather_sweep_kernel(const int32_t* __restrict__ ids, int rounds, int blocks,
                                                           int per_visit, const float* __restrict__ table,
                                                           int64_t row_floats, float* __restrict__ out) {
  constexpr int LPS = 8, NG = 8, UNR = 4;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % LPS, grp = lane / LPS;
  const int slice = (int)(blockIdx.x % 8u);
  const int64_t slot = blockIdx.x / 8u;
  const float* __restrict__ src = table + slice * (LPS * 4) + sub * 4;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int r = 0; r < rounds; ++r) {
    for (int b = 0; b < blocks; ++b) {
      const int32_t* __restrict__ my = ids + ((((slot * rounds + r) * blocks + b) * 4 + wave) * (int64_t)per_visit);
      for (int e = grp; e < per_visit; e += NG * UNR) {  // per_visit is a multiple of NG * UNR
        int u[UNR];
        f32x4 v[UNR];
#pragma unroll
        for (int t = 0; t < UNR; ++t) u[t] = my[e + t * NG];
#pragma unroll
        for (int t = 0; t < UNR; ++t) v[t] = *reinterpret_cast<const f32x4*>(src + (int64_t)u[t] * row_floats);
#pragma unroll
        for (int t = 0; t < UNR; ++t) acc += v[t];
      }
    }
  }
#pragma unroll
  for (int off = LPS; off < 64; off <<= 1) {
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] += __shfl_xor(acc[i], off, 64);
  }
  if (grp == 0) *reinterpret_cast<f32x4*>(out + ((int64_t)blockIdx.x * 4 + wave) * 32 + sub * 4) = acc;
}

static float time_launches(int reps, void (*launch)(void*), void* ctx) {
  hipEvent_t a, b;
  CHECK(hipEventCreate(&a));
  CHECK(hipEventCreate(&b));
  for (int i = 0; i < 2; ++i) launch(ctx);
  CHECK(hipDeviceSynchronize());
  CHECK(hipEventRecord(a, 0));
  for (int i = 0; i < reps; ++i) launch(ctx);
  CHECK(hipEventRecord(b, 0));
  CHECK(hipEventSynchronize(b));
  float ms = 0.f;
  CHECK(hipEventElapsedTime(&ms, a, b));
  CHECK(hipGetLastError());
  CHECK(hipEventDestroy(a));
  CHECK(hipEventDestroy(b));
  return ms / reps;
}

struct StreamCtx {
  const f32x4* buf;
  int64_t n_vec;
  int passes;
  float* sink;
  int blocks;
};
static void launch_stream(void* p) {
  StreamCtx* c = (StreamCtx*)p;
  stream_read_kernel<<<c->blocks, 256>>>(c->buf, c->n_vec, c->passes, c->sink);
}

struct GatherCtx {
  const int32_t* ids;
  int64_t rows;
  int deg;
  const float* table;
  int64_t row_floats;
  float* out;
  int lps, slices;
};
static void launch_gather(void* p) {
  GatherCtx* c = (GatherCtx*)p;
  const int64_t blocks = ((c->rows + 3) / 4) * c->slices;
  const dim3 grid((unsigned)blocks);
#define GO(L, S) gather_kernel<L, S><<<grid, 256>>>(c->ids, c->rows, c->deg, c->table, c->row_floats, c->out)
  if (c->slices == 8 && c->lps == 8) GO(8, 8);
  else if (c->lps == 8) GO(8, 1);
  else if (c->lps == 16) GO(16, 1);
  else if (c->lps == 32) GO(32, 1);
  else GO(64, 1);
#undef GO
}

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static inline uint64_t next_u64() {  // xorshift64*
  rng_state ^= rng_state >> 12;
  rng_state ^= rng_state << 25;
  rng_state ^= rng_state >> 27;
  return rng_state * 0x2545F4914F6CDD1Dull;
}

int main() {
  const double CUS = 256.0, GHZ = 2.4;
  CHECK(hipSetDevice(0));
  float* sink = nullptr;
  CHECK(hipMalloc(&sink, 256));

  printf("== stream: contiguous 16-byte-per-lane reads, 2048 workgroups of 256 threads ==\n");
  printf("%-44s %12s %12s\n", "buffer", "us/launch", "GB/s");
  {
    struct Case {
      const char* name;
      int64_t bytes;
      int passes;
    } cases[] = {{"16 MiB (2 MiB per XCD: L2-resident) x64", 16ll << 20, 64},
                 {"128 MiB (memory-side cache) x8", 128ll << 20, 8},
                 {"4 GiB (HBM) x1", 4ll << 30, 1}};
    float* buf = nullptr;
    CHECK(hipMalloc(&buf, 4ll << 30));
    CHECK(hipMemset(buf, 0, 4ll << 30));
    for (auto& c : cases) {
      StreamCtx ctx{(const f32x4*)buf, c.bytes / 16, c.passes, sink, 2048};
      const float ms = time_launches(10, launch_stream, &ctx);
      printf("%-44s %12.1f %12.0f\n", c.name, 1e3 * ms, (double)c.bytes * c.passes / (ms * 1e-3) / 1e9);
    }
    CHECK(hipFree(buf));
  }

  printf("\n== gather: lists of random rows, one wavefront per (list, slice), 4 loads in flight ==\n");
  printf("%-70s %10s %10s %12s %14s\n", "case", "us/launch", "GB/s req.", "Glines/s", "clk/line/CU");
  struct G {
    const char* name;
    int64_t rows;    // lists
    int deg;         // ids per list
    int64_t window;  // distinct matrix rows the ids are drawn from
    int row_floats;  // matrix row length in float32
    int lps, slices;
  } gs[] = {
      // the 256-wide float32 launch of the Reddit-shaped workload: 230k lists of 61 ids, 1 KiB rows, 8 slices
      {"1 KiB rows, 8 XCD slices of 128 B, deg 61, window 230k rows (235 MB)", 230000, 61, 230000, 256, 8, 8},
      {"1 KiB rows, 8 XCD slices of 128 B, deg 61, window 16k rows (2 MiB per XCD)", 230000, 61, 16384, 256, 8, 8},
      {"1 KiB rows, whole row per wavefront, deg 61, window 230k rows", 230000, 61, 230000, 256, 64, 1},
      {"1 KiB rows, whole row per wavefront, deg 61, window 16k rows (16 MiB)", 230000, 61, 16384, 256, 64, 1},
      // narrow rows: 128 B (32 floats), the 41- / 47-wide launches
      {"128 B rows, deg 61, window 230k rows (29 MB)", 230000, 61, 230000, 32, 8, 1},
      // the short rows of the products-shaped workload: 1.9M lists of 4 ids, 512 B rows (256 bf16)
      {"512 B rows, deg 4, window 1.9M rows (0.96 GB)", 1900000, 4, 1900000, 128, 32, 1},
      {"512 B rows, deg 4, window 64k rows (32 MiB)", 1900000, 4, 65536, 128, 32, 1},
      // the papers100M-shaped partition: 28M lists of 4 ids over 28M rows of 512 B, far beyond every cache
      {"512 B rows, deg 4, window 28M rows (14.3 GB)", 28000000, 4, 28000000, 128, 32, 1},
  };
  for (auto& g : gs) {
    std::vector<int32_t> h((size_t)g.rows * g.deg);
    for (auto& x : h) x = (int32_t)(next_u64() % (uint64_t)g.window);
    int32_t* ids = nullptr;
    float *table = nullptr, *out = nullptr;
    CHECK(hipMalloc(&ids, h.size() * 4));
    CHECK(hipMemcpy(ids, h.data(), h.size() * 4, hipMemcpyHostToDevice));
    CHECK(hipMalloc(&table, (size_t)g.window * g.row_floats * 4));
    CHECK(hipMemset(table, 0, (size_t)g.window * g.row_floats * 4));
    CHECK(hipMalloc(&out, (size_t)g.rows * g.row_floats * 4));
    GatherCtx ctx{ids, g.rows, g.deg, table, g.row_floats, out, g.lps, g.slices};
    const float ms = time_launches(10, launch_gather, &ctx);
    const double bytes = (double)g.rows * g.deg * g.row_floats * 4;
    const double lines = bytes / 128.0;
    printf("%-70s %10.1f %10.0f %12.2f %14.2f\n", g.name, 1e3 * ms, bytes / (ms * 1e-3) / 1e9, lines / (ms * 1e-3) / 1e9,
           (ms * 1e-3) * GHZ * 1e9 * CUS / lines);
    CHECK(hipFree(ids));
    CHECK(hipFree(table));
    CHECK(hipFree(out));
  }
  printf("\n== sweep: 1 KiB rows, 8 XCD slices of 128 B, window 230k rows; 2048 resident workgroups go `rounds` times "
         "through B source blocks ==\n");
  printf("%-70s %10s %10s %12s %14s\n", "case", "us/launch", "GB/s req.", "Glines/s", "clk/line/CU");
  {
    const int64_t window = 230000, row_floats = 256;
    const int slots = 256;  // workgroups per slice: 8 per CU of an XCD, all resident
    float *table = nullptr, *out = nullptr;
    CHECK(hipMalloc(&table, (size_t)window * row_floats * 4));
    CHECK(hipMemset(table, 0, (size_t)window * row_floats * 4));
    CHECK(hipMalloc(&out, (size_t)8 * slots * 4 * 32 * 4));
    struct S {
      int rounds, blocks, per_visit;
    } ss[] = {{7, 1, 2048}, {7, 4, 512}, {7, 8, 256}, {7, 16, 128}, {7, 32, 64}, {7, 64, 32}, {1, 16, 896}, {1, 64, 224}};
    for (auto& c : ss) {
      const size_t n_ids = (size_t)slots * c.rounds * c.blocks * 4 * c.per_visit;
      std::vector<int32_t> h(n_ids);
      size_t i = 0;
      for (int s = 0; s < slots; ++s)
        for (int r = 0; r < c.rounds; ++r)
          for (int b = 0; b < c.blocks; ++b) {
            const int64_t lo = window * b / c.blocks, hi = window * (b + 1) / c.blocks;
            for (int k = 0; k < 4 * c.per_visit; ++k) h[i++] = (int32_t)(lo + (int64_t)(next_u64() % (uint64_t)(hi - lo)));
          }
      int32_t* ids = nullptr;
      CHECK(hipMalloc(&ids, n_ids * 4));
      CHECK(hipMemcpy(ids, h.data(), n_ids * 4, hipMemcpyHostToDevice));
      struct Ctx {
        const int32_t* ids;
        int rounds, blocks, per_visit;
        const float* table;
        int64_t row_floats;
        float* out;
        int slots;
      } ctx{ids, c.rounds, c.blocks, c.per_visit, table, row_floats, out, slots};
      const float ms = time_launches(10, [](void* p) {
        Ctx* x = (Ctx*)p;
        gather_sweep_kernel<<<dim3(8u * (unsigned)x->slots), 256>>>(x->ids, x->rounds, x->blocks, x->per_visit, x->table,
                                                                   x->row_floats, x->out);
      }, &ctx);
      const double bytes = (double)n_ids * 8 * 128.0;  // every id is fetched once per slice
      const double lines = bytes / 128.0;
      char name[96];
      snprintf(name, sizeof(name), "%d rounds x %d blocks, %d ids per wavefront and visit (%.1fM ids)", c.rounds, c.blocks,
               c.per_visit, n_ids / 1e6);
      printf("%-70s %10.1f %10.0f %12.2f %14.2f\n", name, 1e3 * ms, bytes / (ms * 1e-3) / 1e9, lines / (ms * 1e-3) / 1e9,
             (ms * 1e-3) * GHZ * 1e9 * CUS / lines);
      CHECK(hipFree(ids));
    }
    CHECK(hipFree(table));
    CHECK(hipFree(out));
  }
  CHECK(hipFree(sink));
  return 0;
}
