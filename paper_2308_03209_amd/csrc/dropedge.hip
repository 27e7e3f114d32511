// DropEdge-K preprocessing (Section 4.4; Algorithm 1 line 5): K masks over the partition's
// undirected edges are drawn once by a HIP kernel from the counter-based generator, then each
// mask's kept edges are compacted - on the device - into a CSR of their own so that the
// per-iteration "apply the mask" (Algorithm 1 line 8) is nothing but a pointer switch.
//
// Compaction of one mask: (1) one wavefront per row counts the row's kept entries and derives the
// masked-degree normalisation vectors, (2) an exclusive scan of the counts gives the new row
// offsets, (3) one wavefront per row writes the kept neighbour ids in their original (ascending)
// order, placing them with a ballot + popcount.  Host copies of the bits and of the compacted
// graphs are fetched only if asked for.
#include <algorithm>
#include <cmath>
#include <mutex>
#include <new>

#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>

#include "common.h"

namespace cofree {

// One thread per (mask k, edge e); a wavefront's 64 keep decisions are one output word.
// Grid: x over words (64 edges per wavefront, 4 wavefronts per block), y over masks.
__global__ __launch_bounds__(256) void dropedge_bits_kernel(uint64_t* __restrict__ bits, int64_t n_edges,
                                                            int64_t n_words, uint64_t seed, uint32_t threshold) {
  const int lane = threadIdx.x & 63;
  const int64_t word = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const uint32_t k = blockIdx.y;
  if (word >= n_words) return;  // uniform per wavefront
  const int64_t e = word * 64 + lane;
  bool keep = false;
  if (e < n_edges) keep = draw1(seed, STREAM_MASK, (uint64_t)e, k) >= threshold;
  const uint64_t w = __ballot(keep);
  if (lane == 0) bits[(int64_t)k * n_words + word] = w;
}

__device__ inline bool edge_kept(const uint64_t* __restrict__ bits, int32_t e) {
  return (bits[e >> 6] >> (e & 63)) & 1ull;
}

// (1) masked degree of every row (int64, the scan's input) and the per-node norms that go with it
__global__ __launch_bounds__(256) void mask_degree_kernel(const int64_t* __restrict__ rowptr,
                                                          const int32_t* __restrict__ eid,
                                                          const uint64_t* __restrict__ bits, int64_t n,
                                                          int64_t* __restrict__ deg, float* __restrict__ inv_deg,
                                                          float* __restrict__ gcn_norm) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= n) return;
  const int64_t beg = rowptr[row], end = rowptr[row + 1];
  int cnt = 0;
  for (int64_t j = beg + lane; j < end; j += 64) cnt += edge_kept(bits, eid[j]) ? 1 : 0;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o, 64);
  if (lane == 0) {
    deg[row] = cnt;
    inv_deg[row] = cnt > 0 ? (float)(1.0 / (double)cnt) : 0.f;
    gcn_norm[row] = (float)(1.0 / sqrt((double)cnt + 1.0));
  }
}

// (2) exclusive scan of n int64 values in three steps: sums of chunks of SCAN_CHUNK values, an
// exclusive scan of those sums by one workgroup, then each chunk scanned from its offset.
constexpr int SCAN_PER_THREAD = 8, SCAN_CHUNK = 256 * SCAN_PER_THREAD;

// exclusive scan of one value per thread over the 256 threads of a workgroup; *total = their sum
__device__ inline int64_t block_exclusive_scan(int64_t x, int64_t* total) {
  __shared__ int64_t wave_sum[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int64_t incl = x;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int64_t y = __shfl_up(incl, o, 64);
    if (lane >= o) incl += y;
  }
  __syncthreads();  // wave_sum may still be read from a previous call
  if (lane == 63) wave_sum[wave] = incl;
  __syncthreads();
  int64_t before = 0;
  for (int w = 0; w < wave; ++w) before += wave_sum[w];
  *total = wave_sum[0] + wave_sum[1] + wave_sum[2] + wave_sum[3];
  return before + incl - x;
}

__global__ __launch_bounds__(256) void scan_chunk_sums_kernel(const int64_t* __restrict__ in, int64_t n,
                                                              int64_t* __restrict__ sums) {
  const int64_t base = (int64_t)blockIdx.x * SCAN_CHUNK + (int64_t)threadIdx.x * SCAN_PER_THREAD;
  int64_t s = 0;
#pragma unroll
  for (int i = 0; i < SCAN_PER_THREAD; ++i)
    if (base + i < n) s += in[base + i];
  int64_t total;
  (void)block_exclusive_scan(s, &total);
  if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

// sums[0..m) -> exclusive prefix in place; *grand_total = sum of all
__global__ __launch_bounds__(256) void scan_sums_kernel(int64_t* __restrict__ sums, int64_t m,
                                                        int64_t* __restrict__ grand_total) {
  int64_t carry = 0;
  for (int64_t b = 0; b < m; b += 256) {
    const int64_t i = b + threadIdx.x;
    const int64_t x = i < m ? sums[i] : 0;
    int64_t total;
    const int64_t ex = block_exclusive_scan(x, &total);
    if (i < m) sums[i] = carry + ex;
    carry += total;
  }
  if (threadIdx.x == 0) *grand_total = carry;
}

// out[i] = offsets[chunk] + exclusive prefix inside the chunk, for i < n
__global__ __launch_bounds__(256) void scan_chunks_kernel(const int64_t* __restrict__ in, int64_t n,
                                                          const int64_t* __restrict__ offsets,
                                                          int64_t* __restrict__ out) {
  const int64_t base = (int64_t)blockIdx.x * SCAN_CHUNK + (int64_t)threadIdx.x * SCAN_PER_THREAD;
  int64_t v[SCAN_PER_THREAD], s = 0;
#pragma unroll
  for (int i = 0; i < SCAN_PER_THREAD; ++i) {
    v[i] = base + i < n ? in[base + i] : 0;
    s += v[i];
  }
  int64_t total;
  int64_t run = offsets[blockIdx.x] + block_exclusive_scan(s, &total);
#pragma unroll
  for (int i = 0; i < SCAN_PER_THREAD; ++i) {
    if (base + i < n) out[base + i] = run;
    run += v[i];
  }
}

// Processing order of the aggregation: rows sorted by descending masked degree, rows of equal degree by
// ascending id (a stable device radix sort of (degree, row) pairs, so the order - and with it the schedule of
// every launch - is the same on every run and equals what a host-side stable sort gives).  The hub rows at
// the head of the order are counted by one small kernel.
__global__ __launch_bounds__(256) void order_keys_kernel(const int64_t* __restrict__ deg, int64_t n,
                                                         uint32_t* __restrict__ key, int32_t* __restrict__ row) {
  const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (v >= n) return;
  key[v] = (uint32_t)deg[v];
  row[v] = (int32_t)v;
}
// out[0], out[1] += number of rows with deg >= hub_min and their adjacency entries (out zeroed beforehand;
// integer sums, so the order in which the workgroups add their counts does not matter)
__global__ __launch_bounds__(256) void degree_buckets_kernel(const int64_t* __restrict__ deg, int64_t n,
                                                             int64_t hub_min, unsigned long long* __restrict__ out) {
  __shared__ unsigned long long s[2][256];
  unsigned long long c0 = 0, c1 = 0;
  for (int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x; v < n; v += (int64_t)gridDim.x * 256) {
    const int64_t d = deg[v];
    if (d >= hub_min) c0 += 1, c1 += (unsigned long long)d;
  }
  s[0][threadIdx.x] = c0;
  s[1][threadIdx.x] = c1;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) {
      s[0][threadIdx.x] += s[0][threadIdx.x + o];
      s[1][threadIdx.x] += s[1][threadIdx.x + o];
    }
    __syncthreads();
  }
  if (threadIdx.x < 2 && s[threadIdx.x][0] != 0) atomicAdd(&out[threadIdx.x], s[threadIdx.x][0]);
}

// (3) kept neighbour ids of every row, in order
__global__ __launch_bounds__(256) void mask_scatter_kernel(const int64_t* __restrict__ rowptr,
                                                           const int32_t* __restrict__ col,
                                                           const int32_t* __restrict__ eid,
                                                           const uint64_t* __restrict__ bits, int64_t n,
                                                           const int64_t* __restrict__ rowptr_out,
                                                           int32_t* __restrict__ col_out) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= n) return;
  const int64_t beg = rowptr[row], end = rowptr[row + 1];
  int64_t base = rowptr_out[row];
  for (int64_t j0 = beg; j0 < end; j0 += 64) {
    const int64_t j = j0 + lane;
    const bool keep = j < end && edge_kept(bits, eid[j]);
    const uint64_t m = __ballot(keep);
    if (keep) col_out[base + __popcll(m & ((1ull << lane) - 1ull))] = col[j];
    base += __popcll(m);
  }
}

// per-entry copies of the per-node factors (see DeviceGraph)
__global__ __launch_bounds__(256) void entry_scales_kernel(const int32_t* __restrict__ col, int64_t nnz,
                                                           const float* __restrict__ inv_deg,
                                                           const float* __restrict__ gcn_norm,
                                                           float* __restrict__ val_inv_deg,
                                                           float* __restrict__ val_gcn_norm) {
  for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < nnz; e += (int64_t)gridDim.x * 256) {
    const int32_t u = col[e];
    val_inv_deg[e] = inv_deg[u];
    val_gcn_norm[e] = gcn_norm[u];
  }
}

int32_t launch_entry_scales(const int32_t* col, int64_t nnz, const float* inv_deg, const float* gcn_norm,
                            float* val_inv_deg, float* val_gcn_norm, hipStream_t stream) {
  if (nnz <= 0) return COFREE_OK;
  const int64_t blocks = std::min<int64_t>((nnz + 255) / 256, 1 << 16);
  entry_scales_kernel<<<dim3((unsigned)blocks), 256, 0, stream>>>(col, nnz, inv_deg, gcn_norm, val_inv_deg,
                                                                  val_gcn_norm);
  COFREE_HIP_CHECK(hipGetLastError());
  return COFREE_OK;
}

template <typename T>
static int32_t dev_alloc(T** dst, size_t count) {
  *dst = nullptr;
  hipError_t e = hipMalloc((void**)dst, (count > 0 ? count : 1) * sizeof(T));
  if (e != hipSuccess) return fail(COFREE_ENOMEM, std::string("hipMalloc: ") + hipGetErrorString(e));
  return COFREE_OK;
}

// ---- processing-order copy of a graph (see DeviceGraph) -------------------------------------------
// (1) degree and own factors of the row in slot i
__global__ __launch_bounds__(256) void slot_degree_kernel(const int64_t* __restrict__ rowptr,
                                                          const int32_t* __restrict__ order,
                                                          const float* __restrict__ inv_deg,
                                                          const float* __restrict__ gcn_norm, int64_t n,
                                                          int64_t* __restrict__ deg, float* __restrict__ s_inv_deg,
                                                          float* __restrict__ s_gcn_norm) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const int64_t row = order[i];
  deg[i] = rowptr[row + 1] - rowptr[row];
  s_inv_deg[i] = inv_deg[row];
  s_gcn_norm[i] = gcn_norm[row];
}
// (3) neighbour ids of slot i, in the row's order, and the factors of each neighbour; one group of 16 lanes per
// slot (most rows of a cut power-law graph have a handful of neighbours)
__global__ __launch_bounds__(256) void slot_scatter_kernel(const int64_t* __restrict__ rowptr,
                                                           const int32_t* __restrict__ col,
                                                           const int32_t* __restrict__ order,
                                                           const float* __restrict__ inv_deg,
                                                           const float* __restrict__ gcn_norm, int64_t n,
                                                           const int64_t* __restrict__ s_rowptr,
                                                           int32_t* __restrict__ s_col,
                                                           float* __restrict__ s_val_inv_deg,
                                                           float* __restrict__ s_val_gcn_norm) {
  const int sub = threadIdx.x & 15;
  const int64_t i = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
  if (i >= n) return;
  const int64_t row = order[i];
  const int64_t beg = rowptr[row], cnt = rowptr[row + 1] - beg, dst = s_rowptr[i];
  for (int64_t j = sub; j < cnt; j += 16) {
    const int32_t u = col[beg + j];
    s_col[dst + j] = u;
    s_val_inv_deg[dst + j] = inv_deg[u];
    s_val_gcn_norm[dst + j] = gcn_norm[u];
  }
}

void free_slot_csr(SlotCsr* s) {
  (void)hipFree(s->rowptr);
  (void)hipFree(s->col);
  (void)hipFree(s->val_inv_deg);
  (void)hipFree(s->val_gcn_norm);
  (void)hipFree(s->inv_deg);
  (void)hipFree(s->gcn_norm);
  *s = SlotCsr();
}

int32_t build_slot_csr(const DeviceGraph& g, SlotCsr* out, hipStream_t stream) {
  const int64_t N = g.n, nnz = g.nnz;
  const int64_t n_chunks = (N + SCAN_CHUNK - 1) / SCAN_CHUNK;
  int64_t *d_deg = nullptr, *d_sums = nullptr;
  int32_t rc = dev_alloc(&out->rowptr, (size_t)N + 1);
  if (rc == COFREE_OK) rc = dev_alloc(&out->col, (size_t)nnz);
  if (rc == COFREE_OK) rc = dev_alloc(&out->val_inv_deg, (size_t)nnz);
  if (rc == COFREE_OK) rc = dev_alloc(&out->val_gcn_norm, (size_t)nnz);
  if (rc == COFREE_OK) rc = dev_alloc(&out->inv_deg, (size_t)N);
  if (rc == COFREE_OK) rc = dev_alloc(&out->gcn_norm, (size_t)N);
  if (rc == COFREE_OK) rc = dev_alloc(&d_deg, (size_t)N);
  if (rc == COFREE_OK) rc = dev_alloc(&d_sums, (size_t)n_chunks + 1);
  if (rc == COFREE_OK) {
    hipError_t e = hipSuccess;
    if (N > 0) {
      slot_degree_kernel<<<dim3((unsigned)((N + 255) / 256)), 256, 0, stream>>>(g.rowptr, g.order, g.inv_deg, g.gcn_norm,
                                                                               N, d_deg, out->inv_deg, out->gcn_norm);
      scan_chunk_sums_kernel<<<dim3((unsigned)n_chunks), 256, 0, stream>>>(d_deg, N, d_sums);
      scan_sums_kernel<<<1, 256, 0, stream>>>(d_sums, n_chunks, out->rowptr + N);  // total -> rowptr[N]
      scan_chunks_kernel<<<dim3((unsigned)n_chunks), 256, 0, stream>>>(d_deg, N, d_sums, out->rowptr);
      if (nnz > 0)
        slot_scatter_kernel<<<dim3((unsigned)((N + 15) / 16)), 256, 0, stream>>>(
            g.rowptr, g.col, g.order, g.inv_deg, g.gcn_norm, N, out->rowptr, out->col, out->val_inv_deg,
            out->val_gcn_norm);
      e = hipGetLastError();
    } else {
      e = hipMemsetAsync(out->rowptr, 0, sizeof(int64_t), stream);
    }
    if (e == hipSuccess) e = hipStreamSynchronize(stream);  // the scratch below is freed on return
    if (e != hipSuccess) rc = fail(COFREE_EHIP, std::string("processing-order copy: ") + hipGetErrorString(e));
  }
  (void)hipFree(d_deg);
  (void)hipFree(d_sums);
  if (rc != COFREE_OK) free_slot_csr(out);
  return rc;
}

static int32_t build_masks(const cofree_partition* P, int32_t K, double p_drop, uint64_t seed, hipStream_t stream,
                           cofree_masks* M) {
  const int64_t E = P->n_edges, N = P->n_nodes;
  const int64_t n_words = (E + 63) / 64;
  M->K = K;
  M->n_nodes = N;
  M->n_edges = E;
  M->n_words = n_words;
  M->bits.assign(K, std::vector<uint64_t>());
  M->host.resize(K);
  M->dev.resize(K);
  COFREE_TRY(dev_alloc(&M->d_bits, (size_t)K * (size_t)n_words));
  if (n_words > 0) {
    const dim3 grid((unsigned)((n_words + 3) / 4), (unsigned)K);
    dropedge_bits_kernel<<<grid, 256, 0, stream>>>(M->d_bits, E, n_words, seed, prob_threshold(p_drop));
    COFREE_HIP_CHECK(hipGetLastError());
  }
  // scratch of the compaction, shared by the K masks
  const int64_t n_chunks = (N + SCAN_CHUNK - 1) / SCAN_CHUNK;
  int64_t *d_deg = nullptr, *d_sums = nullptr, *d_buckets = nullptr;
  uint32_t *d_key = nullptr, *d_key_sorted = nullptr;
  int32_t* d_row = nullptr;
  void* d_sort_tmp = nullptr;
  size_t sort_tmp_bytes = 0;
  COFREE_TRY(dev_alloc(&d_deg, (size_t)N));
  int32_t rc = dev_alloc(&d_sums, (size_t)n_chunks + 1);
  if (rc == COFREE_OK) rc = dev_alloc(&d_buckets, 2);
  if (rc == COFREE_OK) rc = dev_alloc(&d_key, (size_t)N);
  if (rc == COFREE_OK) rc = dev_alloc(&d_key_sorted, (size_t)N);
  if (rc == COFREE_OK) rc = dev_alloc(&d_row, (size_t)N);
  if (rc == COFREE_OK && N > 0) {
    // size query of the device sort (null storage: nothing runs)
    hipError_t e = rocprim::radix_sort_pairs_desc(nullptr, sort_tmp_bytes, d_key, d_key_sorted, d_row, d_row,
                                                  (size_t)N, 0, 32, stream);
    if (e != hipSuccess) rc = fail(COFREE_EHIP, std::string("radix sort size query: ") + hipGetErrorString(e));
    if (rc == COFREE_OK) rc = dev_alloc((char**)&d_sort_tmp, sort_tmp_bytes);
  }
  const int64_t row_blocks = (N + 3) / 4;
  for (int32_t k = 0; k < K && rc == COFREE_OK; ++k) {
    auto& d = M->dev[k];
    const uint64_t* bits = M->d_bits + (int64_t)k * n_words;
    rc = dev_alloc(&d.rowptr, (size_t)N + 1);
    if (rc == COFREE_OK) rc = dev_alloc(&d.inv_deg, (size_t)N);
    if (rc == COFREE_OK) rc = dev_alloc(&d.gcn_norm, (size_t)N);
    if (rc == COFREE_OK) rc = dev_alloc(&d.order, (size_t)N);
    if (rc != COFREE_OK) break;
    hipError_t e = hipSuccess;
    int64_t nnz = 0;
    if (N > 0) {
      mask_degree_kernel<<<dim3((unsigned)row_blocks), 256, 0, stream>>>(P->d_rowptr, P->d_eid, bits, N, d_deg,
                                                                        d.inv_deg, d.gcn_norm);
      scan_chunk_sums_kernel<<<dim3((unsigned)n_chunks), 256, 0, stream>>>(d_deg, N, d_sums);
      scan_sums_kernel<<<1, 256, 0, stream>>>(d_sums, n_chunks, d.rowptr + N);  // total -> rowptr[N]
      scan_chunks_kernel<<<dim3((unsigned)n_chunks), 256, 0, stream>>>(d_deg, N, d_sums, d.rowptr);
      order_keys_kernel<<<dim3((unsigned)((N + 255) / 256)), 256, 0, stream>>>(d_deg, N, d_key, d_row);
      e = hipMemsetAsync(d_buckets, 0, 2 * sizeof(int64_t), stream);
      degree_buckets_kernel<<<dim3((unsigned)std::min<int64_t>((N + 255) / 256, 1024)), 256, 0, stream>>>(
          d_deg, N, AGG_HUB_MIN, (unsigned long long*)d_buckets);
      if (e == hipSuccess) e = hipGetLastError();
      if (e == hipSuccess)
        e = rocprim::radix_sort_pairs_desc(d_sort_tmp, sort_tmp_bytes, d_key, d_key_sorted, d_row, d.order, (size_t)N,
                                           0, 32, stream);
      int64_t hb[2] = {0, 0};
      if (e == hipSuccess)
        e = hipMemcpyAsync(&nnz, d.rowptr + N, sizeof(int64_t), hipMemcpyDeviceToHost, stream);
      if (e == hipSuccess) e = hipMemcpyAsync(hb, d_buckets, sizeof(hb), hipMemcpyDeviceToHost, stream);
      if (e == hipSuccess) e = hipStreamSynchronize(stream);
      d.buckets.n_hub = hb[0];
      d.buckets.nnz_hub = hb[1];
    } else {
      const int64_t zero = 0;
      e = hipMemcpy(d.rowptr, &zero, sizeof(int64_t), hipMemcpyHostToDevice);
    }
    if (e != hipSuccess) {
      rc = fail(COFREE_EHIP, std::string("dropedge compaction: ") + hipGetErrorString(e));
      break;
    }
    d.nnz = nnz;
    rc = dev_alloc(&d.col, (size_t)nnz);
    if (rc == COFREE_OK) rc = dev_alloc(&d.val_inv_deg, (size_t)nnz);
    if (rc == COFREE_OK) rc = dev_alloc(&d.val_gcn_norm, (size_t)nnz);
    if (rc != COFREE_OK) break;
    if (N > 0 && nnz > 0) {
      mask_scatter_kernel<<<dim3((unsigned)row_blocks), 256, 0, stream>>>(P->d_rowptr, P->d_col, P->d_eid, bits, N,
                                                                         d.rowptr, d.col);
      e = hipGetLastError();
      if (e != hipSuccess) rc = fail(COFREE_EHIP, std::string("dropedge scatter: ") + hipGetErrorString(e));
      if (rc == COFREE_OK)
        rc = launch_entry_scales(d.col, nnz, d.inv_deg, d.gcn_norm, d.val_inv_deg, d.val_gcn_norm, stream);
    }
    if (rc == COFREE_OK) {
      DeviceGraph g;
      g.rowptr = d.rowptr;
      g.col = d.col;
      g.inv_deg = d.inv_deg;
      g.gcn_norm = d.gcn_norm;
      g.order = d.order;
      g.n = N;
      g.nnz = nnz;
      rc = build_slot_csr(g, &d.slots, stream);
    }
  }
  hipError_t se = hipStreamSynchronize(stream);
  (void)hipFree(d_deg);
  (void)hipFree(d_sums);
  (void)hipFree(d_buckets);
  (void)hipFree(d_key);
  (void)hipFree(d_key_sorted);
  (void)hipFree(d_row);
  (void)hipFree(d_sort_tmp);
  if (rc == COFREE_OK && se != hipSuccess) rc = fail(COFREE_EHIP, std::string("dropedge: ") + hipGetErrorString(se));
  return rc;
}

// Host copies are made on first request (the training path never needs them).
static std::mutex g_host_copy_mutex;

static int32_t fetch_bits(cofree_masks* M, int32_t k) {
  std::lock_guard<std::mutex> lk(g_host_copy_mutex);
  if (!M->bits[k].empty() || M->n_words == 0) return COFREE_OK;
  std::vector<uint64_t> w((size_t)M->n_words);
  COFREE_HIP_CHECK(hipMemcpy(w.data(), M->d_bits + (int64_t)k * M->n_words, w.size() * sizeof(uint64_t),
                             hipMemcpyDeviceToHost));
  M->bits[k].swap(w);
  return COFREE_OK;
}

static int32_t fetch_graph(cofree_masks* M, int32_t k) {
  std::lock_guard<std::mutex> lk(g_host_copy_mutex);
  HostGraph& g = M->host[k];
  if (!g.rowptr.empty()) return COFREE_OK;
  const auto& d = M->dev[k];
  std::vector<int64_t> rp((size_t)M->n_nodes + 1);
  std::vector<int32_t> cl((size_t)d.nnz);
  COFREE_HIP_CHECK(hipMemcpy(rp.data(), d.rowptr, rp.size() * sizeof(int64_t), hipMemcpyDeviceToHost));
  if (d.nnz > 0) COFREE_HIP_CHECK(hipMemcpy(cl.data(), d.col, cl.size() * sizeof(int32_t), hipMemcpyDeviceToHost));
  g.rowptr.swap(rp);
  g.col.swap(cl);
  return COFREE_OK;
}

}  // namespace cofree

using namespace cofree;

extern "C" {

int32_t cofree_dropedge_k(const cofree_partition* part, int32_t K, double p_drop, uint64_t seed, uint32_t flags,
                          void* stream, cofree_masks** out) {
  COFREE_REQUIRE(out != nullptr, "out is NULL");
  *out = nullptr;
  COFREE_REQUIRE(part != nullptr, "partition is NULL");
  COFREE_REQUIRE(K >= 1 && K <= 65535, "K must be in [1, 65535]");
  COFREE_REQUIRE(p_drop >= 0.0 && p_drop < 1.0, "p_drop must be in [0, 1)");
  COFREE_REQUIRE(flags == 0, "unknown flags");
  if (!part->on_device) return fail(COFREE_ESTATE, "partition has no device copy (built with COFREE_HOST_ONLY)");
  cofree_masks* M = new (std::nothrow) cofree_masks();
  if (!M) return fail(COFREE_ENOMEM, "out of host memory");
  int32_t rc;
  try {
    rc = build_masks(part, K, p_drop, seed, (hipStream_t)stream, M);
  } catch (const std::bad_alloc&) {
    rc = fail(COFREE_ENOMEM, "out of host memory while building masks");
  }
  if (rc != COFREE_OK) {
    cofree_masks_free(M);
    return rc;
  }
  *out = M;
  return COFREE_OK;
}

void cofree_masks_free(cofree_masks* M) {
  if (!M) return;
  for (auto& d : M->dev) {
    (void)hipFree(d.rowptr);
    (void)hipFree(d.col);
    (void)hipFree(d.inv_deg);
    (void)hipFree(d.gcn_norm);
    (void)hipFree(d.val_inv_deg);
    (void)hipFree(d.val_gcn_norm);
    (void)hipFree(d.order);
    free_slot_csr(&d.slots);
  }
  (void)hipFree(M->d_bits);
  delete M;
}

int32_t cofree_masks_count(const cofree_masks* M) { return M ? M->K : -1; }

int32_t cofree_masks_host_bits(const cofree_masks* M, int32_t k, const uint64_t** words, int64_t* n_words) {
  COFREE_REQUIRE(M && words && n_words, "NULL argument");
  COFREE_REQUIRE(k >= 0 && k < M->K, "mask index out of range");
  COFREE_TRY(fetch_bits(const_cast<cofree_masks*>(M), k));
  *words = M->bits[k].data();
  *n_words = M->n_words;
  return COFREE_OK;
}

int32_t cofree_masks_host_graph(const cofree_masks* M, int32_t k, const int64_t** rowptr, const int32_t** col,
                                int64_t* nnz) {
  COFREE_REQUIRE(M && rowptr && col && nnz, "NULL argument");
  COFREE_REQUIRE(k >= 0 && k < M->K, "mask index out of range");
  COFREE_TRY(fetch_graph(const_cast<cofree_masks*>(M), k));
  *rowptr = M->host[k].rowptr.data();
  *col = M->host[k].col.data();
  *nnz = (int64_t)M->host[k].col.size();
  return COFREE_OK;
}

}  // extern "C"
