// DropEdge-K preprocessing (Section 4.4; Algorithm 1 line 5): K masks over the partition's
// undirected edges are drawn once by a HIP kernel from the counter-based generator, then each
// mask's kept edges are compacted into a CSR of their own so that the per-iteration "apply the
// mask" (Algorithm 1 line 8) is nothing but a pointer switch.
#include <cmath>
#include <new>

#include "common.h"

namespace cofree {

void norms_from_rowptr(const std::vector<int64_t>& rowptr, std::vector<float>* inv_deg, std::vector<float>* gcn);

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

template <typename T>
static int32_t upload_vec(T** dst, const std::vector<T>& v, hipStream_t s) {
  *dst = nullptr;
  const size_t bytes = std::max<size_t>(v.size(), 1) * sizeof(T);
  hipError_t e = hipMalloc((void**)dst, bytes);
  if (e != hipSuccess) return fail(COFREE_ENOMEM, std::string("hipMalloc: ") + hipGetErrorString(e));
  if (!v.empty()) COFREE_HIP_CHECK(hipMemcpy(*dst, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice));
  (void)s;
  return COFREE_OK;
}

static int32_t build_masks(const cofree_partition* P, int32_t K, double p_drop, uint64_t seed, hipStream_t stream,
                           cofree_masks* M) {
  const int64_t E = P->n_edges, N = P->n_nodes;
  const int64_t n_words = (E + 63) / 64;
  M->K = K;
  M->n_nodes = N;
  M->n_edges = E;
  M->n_words = n_words;
  M->bits.assign(K, std::vector<uint64_t>((size_t)n_words, 0));
  M->host.resize(K);
  M->dev.resize(K);
  if (n_words > 0) {
    uint64_t* d_bits = nullptr;
    hipError_t e = hipMalloc((void**)&d_bits, (size_t)K * n_words * sizeof(uint64_t));
    if (e != hipSuccess) return fail(COFREE_ENOMEM, std::string("hipMalloc: ") + hipGetErrorString(e));
    const dim3 grid((unsigned)((n_words + 3) / 4), (unsigned)K);
    dropedge_bits_kernel<<<grid, 256, 0, stream>>>(d_bits, E, n_words, seed, prob_threshold(p_drop));
    hipError_t le = hipGetLastError();
    if (le == hipSuccess) le = hipStreamSynchronize(stream);
    for (int32_t k = 0; k < K && le == hipSuccess; ++k)
      le = hipMemcpy(M->bits[k].data(), d_bits + (int64_t)k * n_words, n_words * sizeof(uint64_t),
                     hipMemcpyDeviceToHost);
    (void)hipFree(d_bits);
    if (le != hipSuccess) return fail(COFREE_EHIP, std::string("dropedge bits: ") + hipGetErrorString(le));
  }
  // compaction of every mask on the host: keep CSR entry j of row v iff its edge's bit is set
  for (int32_t k = 0; k < K; ++k) {
    const uint64_t* w = M->bits[k].data();
    HostGraph& g = M->host[k];
    g.rowptr.assign(N + 1, 0);
    g.col.clear();
    g.col.reserve((size_t)(P->nnz * (1.0 - p_drop) * 1.05) + 64);
    for (int64_t v = 0; v < N; ++v) {
      for (int64_t j = P->rowptr[v]; j < P->rowptr[v + 1]; ++j) {
        const int32_t e = P->eid[j];
        if ((w[e >> 6] >> (e & 63)) & 1ull) g.col.push_back(P->col[j]);
      }
      g.rowptr[v + 1] = (int64_t)g.col.size();
    }
    std::vector<float> inv_deg, gcn;
    norms_from_rowptr(g.rowptr, &inv_deg, &gcn);
    auto& d = M->dev[k];
    d.nnz = (int64_t)g.col.size();
    COFREE_TRY(upload_vec(&d.rowptr, g.rowptr, stream));
    COFREE_TRY(upload_vec(&d.col, g.col, stream));
    COFREE_TRY(upload_vec(&d.inv_deg, inv_deg, stream));
    COFREE_TRY(upload_vec(&d.gcn_norm, gcn, stream));
  }
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
  }
  delete M;
}

int32_t cofree_masks_count(const cofree_masks* M) { return M ? M->K : -1; }

int32_t cofree_masks_host_bits(const cofree_masks* M, int32_t k, const uint64_t** words, int64_t* n_words) {
  COFREE_REQUIRE(M && words && n_words, "NULL argument");
  COFREE_REQUIRE(k >= 0 && k < M->K, "mask index out of range");
  *words = M->bits[k].data();
  *n_words = M->n_words;
  return COFREE_OK;
}

int32_t cofree_masks_host_graph(const cofree_masks* M, int32_t k, const int64_t** rowptr, const int32_t** col,
                                int64_t* nnz) {
  COFREE_REQUIRE(M && rowptr && col && nnz, "NULL argument");
  COFREE_REQUIRE(k >= 0 && k < M->K, "mask index out of range");
  *rowptr = M->host[k].rowptr.data();
  *col = M->host[k].col.data();
  *nnz = (int64_t)M->host[k].col.size();
  return COFREE_OK;
}

}  // extern "C"
