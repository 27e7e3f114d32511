// Host side of the vertex cut: edge -> partition assignment, canonical per-partition CSR,
// duplicated-node map, degrees and Degree-Aware Reweighting weights
// (Section 3 "Vertex Cut Partitioning"; proof of Theorem 2 for the random cut; Section 4.3;
// Algorithm 1 lines 1 and 4).
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <new>
#include <thread>

#include "common.h"

namespace cofree {

static thread_local std::string g_last_error;
void set_error(const std::string& msg) { g_last_error = msg; }
int32_t fail(int32_t code, const std::string& msg) {
  g_last_error = msg;
  return code;
}

static unsigned host_threads() {
  unsigned n = std::thread::hardware_concurrency();
  if (n == 0) n = 1;
  return std::min(n, 16u);
}

// run fn(begin, end) over [0, n) in contiguous chunks on a few threads
template <typename Fn>
static void parallel_chunks(int64_t n, Fn fn) {
  const unsigned T = (n < (1 << 16)) ? 1u : host_threads();
  if (T == 1) {
    fn((int64_t)0, n);
    return;
  }
  std::vector<std::thread> th;
  const int64_t chunk = (n + T - 1) / T;
  for (unsigned t = 0; t < T; ++t) {
    const int64_t b = (int64_t)t * chunk, e = std::min(n, b + chunk);
    if (b >= e) break;
    th.emplace_back([=] { fn(b, e); });
  }
  for (auto& x : th) x.join();
}

template <typename T>
static int32_t upload(T** dst, const std::vector<T>& v) {
  *dst = nullptr;
  const size_t bytes = std::max<size_t>(v.size(), 1) * sizeof(T);
  hipError_t e = hipMalloc((void**)dst, bytes);
  if (e != hipSuccess) return fail(COFREE_ENOMEM, std::string("hipMalloc: ") + hipGetErrorString(e));
  if (!v.empty()) COFREE_HIP_CHECK(hipMemcpy(*dst, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice));
  return COFREE_OK;
}

void norms_from_rowptr(const std::vector<int64_t>& rowptr, std::vector<float>* inv_deg, std::vector<float>* gcn) {
  const int64_t n = (int64_t)rowptr.size() - 1;
  inv_deg->resize(n);
  gcn->resize(n);
  for (int64_t v = 0; v < n; ++v) {
    const int64_t d = rowptr[v + 1] - rowptr[v];
    (*inv_deg)[v] = d > 0 ? (float)(1.0 / (double)d) : 0.f;
    (*gcn)[v] = (float)(1.0 / std::sqrt((double)d + 1.0));
  }
}

// keys sorted ascending, on several threads for long lists: bucketed by the smaller endpoint (monotone in the
// key), buckets sorted independently
static void sort_keys(std::vector<uint64_t>& keys, int64_t n_nodes) {
  const int64_t n = (int64_t)keys.size();
  const unsigned T = host_threads();
  if (n <= (1 << 18) || T <= 1) {
    std::sort(keys.begin(), keys.end());
    return;
  }
  const unsigned B = 256;
  std::vector<int64_t> cnt(B + 1, 0);
  auto bucket_of = [&](uint64_t k) { return (unsigned)(((k >> 32) * B) / (uint64_t)n_nodes); };  // lo < n_nodes <= 2^32
  for (int64_t i = 0; i < n; ++i) cnt[bucket_of(keys[i]) + 1]++;
  for (unsigned b = 0; b < B; ++b) cnt[b + 1] += cnt[b];
  std::vector<uint64_t> sorted((size_t)n);
  std::vector<int64_t> pos(cnt.begin(), cnt.end() - 1);
  for (int64_t i = 0; i < n; ++i) sorted[pos[bucket_of(keys[i])]++] = keys[i];
  std::atomic<unsigned> next{0};
  std::vector<std::thread> th;
  for (unsigned t = 0; t < T; ++t)
    th.emplace_back([&] {
      for (;;) {
        const unsigned b = next.fetch_add(1);
        if (b >= B) break;
        std::sort(sorted.begin() + cnt[b], sorted.begin() + cnt[b + 1]);
      }
    });
  for (auto& x : th) x.join();
  keys.swap(sorted);
}

// Validates a list of edges and writes key = lo * 2^32 + hi for each.  Returns 0, or 1 / 2 for an endpoint out
// of range / a self-loop.
static int canonical_keys(int64_t n_nodes, int64_t n_edges, const int64_t* src, const int64_t* dst, uint64_t* key) {
  std::atomic<int> bad{0};
  parallel_chunks(n_edges, [&](int64_t b, int64_t e) {
    for (int64_t i = b; i < e; ++i) {
      const int64_t s = src[i], d = dst[i];
      if (s < 0 || d < 0 || s >= n_nodes || d >= n_nodes) {
        bad.store(1);
        return;
      }
      if (s == d) {
        bad.store(2);
        return;
      }
      const uint64_t lo = (uint64_t)std::min(s, d), hi = (uint64_t)std::max(s, d);
      key[i] = (lo << 32) | hi;
    }
  });
  return bad.load();
}

// partition of edge {lo < hi} under the random cut of the proof of Theorem 2
static inline int32_t random_cut_part(uint64_t seed, uint64_t key, int32_t n_parts) {
  const uint64_t lo = key >> 32, hi = key & 0xffffffffu;
  const uint32_t r = draw1(seed, STREAM_CUT, lo | (hi << 32), 0u);
  return (int32_t)(((uint64_t)r * (uint64_t)n_parts) >> 32);
}

// Membership of global ids in V[i] as a bitmap with a running count per 64-bit word, so that the local id of a
// member (its rank among the members, which are numbered by ascending global id) is two look-ups.
struct NodeRank {
  std::vector<uint64_t> bits;
  std::vector<int64_t> before;  // members in the words before this one
  int64_t count = 0;
  void mark_all(int64_t n_nodes, const std::vector<uint64_t>& keys) {
    bits.assign((size_t)((n_nodes + 63) / 64), 0ull);
    parallel_chunks((int64_t)keys.size(), [&](int64_t b, int64_t e) {
      for (int64_t i = b; i < e; ++i) {
        const uint64_t lo = keys[i] >> 32, hi = keys[i] & 0xffffffffu;
        __atomic_fetch_or(&bits[lo >> 6], 1ull << (lo & 63), __ATOMIC_RELAXED);
        __atomic_fetch_or(&bits[hi >> 6], 1ull << (hi & 63), __ATOMIC_RELAXED);
      }
    });
    before.resize(bits.size());
    int64_t c = 0;
    for (size_t w = 0; w < bits.size(); ++w) {
      before[w] = c;
      c += __builtin_popcountll(bits[w]);
    }
    count = c;
  }
  int32_t rank(uint64_t g) const {
    return (int32_t)(before[g >> 6] + __builtin_popcountll(bits[g >> 6] & ((1ull << (g & 63)) - 1ull)));
  }
};

// Everything of a partition that follows from its own edge list: my_keys = the keys of E[i], sorted and
// unique; deg_g = D(v) for every global id; rf_bits (optional) = one bit per (node, partition).
static int32_t structures_from_keys(cofree_partition* P, int64_t n_nodes, const std::vector<uint64_t>& my_keys,
                                    const std::vector<int32_t>& deg_g, const std::vector<uint64_t>& rf_bits,
                                    int64_t rf_words) {
  const int64_t E = (int64_t)my_keys.size();
  if (2 * E >= ((int64_t)1 << 31)) return fail(COFREE_EINVAL, "partition has too many edges for int32 ids");
  // V[i] = endpoints, ascending global id
  NodeRank nodes;
  nodes.mark_all(n_nodes, my_keys);
  const int64_t N = nodes.count;
  if (N >= ((int64_t)1 << 31)) return fail(COFREE_EINVAL, "partition has too many nodes for int32 ids");
  P->n_nodes = N;
  P->n_edges = E;
  P->nnz = 2 * E;
  P->n_nodes_full = n_nodes;
  P->local2global.resize((size_t)N);
  parallel_chunks((int64_t)nodes.bits.size(), [&](int64_t b, int64_t e) {
    for (int64_t w = b; w < e; ++w) {
      uint64_t m = nodes.bits[(size_t)w];
      int64_t at = nodes.before[(size_t)w];
      while (m) {
        P->local2global[(size_t)at++] = w * 64 + __builtin_ctzll(m);
        m &= m - 1;
      }
    }
  });
  // local endpoints; my_keys is sorted by (lo, hi) and the local numbering is monotone, so the position of an
  // edge in my_keys is its undirected edge id
  P->edge_lo.resize((size_t)E);
  P->edge_hi.resize((size_t)E);
  P->deg_local.assign((size_t)N, 0);
  parallel_chunks(E, [&](int64_t b, int64_t e) {
    for (int64_t i = b; i < e; ++i) {
      P->edge_lo[i] = nodes.rank(my_keys[i] >> 32);
      P->edge_hi[i] = nodes.rank(my_keys[i] & 0xffffffffu);
    }
  });
  for (int64_t i = 0; i < E; ++i) {
    P->deg_local[P->edge_lo[i]]++;
    P->deg_local[P->edge_hi[i]]++;
  }
  P->rowptr.assign((size_t)N + 1, 0);
  for (int64_t v = 0; v < N; ++v) P->rowptr[v + 1] = P->rowptr[v] + P->deg_local[v];
  // CSR fill.  Row v first receives its neighbours u < v (edges with hi = v, visited in ascending lo because
  // my_keys is sorted by lo first), then its neighbours u > v (edges with lo = v, ascending hi) - so two
  // passes give ascending neighbour ids without a sort.
  P->col.resize((size_t)(2 * E));
  P->eid.resize((size_t)(2 * E));
  std::vector<int64_t> fill(P->rowptr.begin(), P->rowptr.end() - 1);
  for (int64_t i = 0; i < E; ++i) {
    const int32_t hi = P->edge_hi[i];
    const int64_t p = fill[hi]++;
    P->col[p] = P->edge_lo[i];
    P->eid[p] = (int32_t)i;
  }
  for (int64_t i = 0; i < E; ++i) {
    const int32_t lo = P->edge_lo[i];
    const int64_t p = fill[lo]++;
    P->col[p] = P->edge_hi[i];
    P->eid[p] = (int32_t)i;
  }
  // degrees in the full graph and the Degree-Aware Reweighting weights
  const auto& l2g = P->local2global;
  P->deg_global.resize((size_t)N);
  P->dar_weight.resize((size_t)N);
  for (int64_t v = 0; v < N; ++v) {
    const int32_t dg = deg_g[(size_t)l2g[v]];
    P->deg_global[v] = dg;
    P->dar_weight[v] = (float)((double)P->deg_local[v] / (double)dg);
  }
  // RF(v_j): number of partitions that hold a copy of the node
  if (!rf_bits.empty()) {
    P->rf.resize((size_t)N);
    for (int64_t v = 0; v < N; ++v) {
      int32_t c = 0;
      for (int64_t w = 0; w < rf_words; ++w) c += __builtin_popcountll(rf_bits[(size_t)(l2g[v] * rf_words + w)]);
      P->rf[v] = c;
    }
  }
  return COFREE_OK;
}

static int32_t build(int64_t n_nodes, int64_t n_edges, const int64_t* src, const int64_t* dst, int32_t n_parts,
                     int32_t part_id, uint64_t seed, const int32_t* assignment, uint32_t flags,
                     cofree_partition* P) {
  // 1. validate and canonicalise every edge to key = lo * 2^32 + hi
  std::vector<uint64_t> key((size_t)n_edges);
  std::vector<uint8_t> mine((size_t)n_edges);
  const bool want_rf = (flags & COFREE_WITH_RF) != 0;
  const bool dbh = (flags & COFREE_CUT_DBH) != 0;
  if (dbh && assignment) return fail(COFREE_EINVAL, "COFREE_CUT_DBH and an explicit assignment exclude each other");
  const int bad = canonical_keys(n_nodes, n_edges, src, dst, key.data());
  if (bad == 1) return fail(COFREE_EINVAL, "edge endpoint out of range [0, n_nodes)");
  if (bad == 2) return fail(COFREE_EINVAL, "self-loop in edge list");
  if (assignment)
    for (int64_t i = 0; i < n_edges; ++i)
      if (assignment[i] < 0 || assignment[i] >= n_parts)
        return fail(COFREE_EINVAL, "assignment value out of range [0, n_parts)");

  // 2. repeated edges: sort all keys.  Under the hash every copy of an edge lands in the same partition, so
  //    COFREE_DEDUP can drop the extra copies; an explicit assignment could send two copies to different
  //    partitions, which would break the disjoint split of the edge set, so there repeats are always rejected.
  std::vector<uint64_t> sorted(key);
  sort_keys(sorted, n_nodes);
  const bool has_dup = std::adjacent_find(sorted.begin(), sorted.end()) != sorted.end();
  if (has_dup && assignment) return fail(COFREE_EINVAL, "repeated edge in a list with an explicit assignment");
  if (has_dup && !(flags & COFREE_DEDUP)) return fail(COFREE_EINVAL, "repeated edge (set COFREE_DEDUP to drop)");
  // 3. global degrees D(v): distinct neighbours
  std::vector<int32_t> deg_g((size_t)n_nodes, 0);
  {
    uint64_t prev = ~0ull;
    for (int64_t i = 0; i < n_edges; ++i) {
      const uint64_t k = sorted[i];
      if (k == prev) continue;
      prev = k;
      deg_g[k >> 32]++;
      deg_g[k & 0xffffffffu]++;
    }
  }
  std::vector<uint64_t>().swap(sorted);
  // 3b. the partition of every edge: explicit, random cut (hash of the edge), or degree-aware hash
  //     (hash of the endpoint of smaller global degree, the smaller id on a tie).  With COFREE_WITH_RF
  //     every node also collects the set of partitions its edges fall into.
  const int64_t rf_words = ((int64_t)n_parts + 63) / 64;
  std::vector<uint64_t> rf_bits;
  if (want_rf) rf_bits.assign((size_t)(n_nodes * rf_words), 0ull);
  parallel_chunks(n_edges, [&](int64_t b, int64_t e) {
    for (int64_t i = b; i < e; ++i) {
      const uint64_t lo = key[i] >> 32, hi = key[i] & 0xffffffffu;
      int32_t part;
      if (assignment) {
        part = assignment[i];
      } else if (dbh) {
        const uint64_t pivot = deg_g[hi] < deg_g[lo] ? hi : lo;
        const uint32_t r = draw1(seed, STREAM_CUT, pivot, 1u);
        part = (int32_t)(((uint64_t)r * (uint64_t)n_parts) >> 32);
      } else {
        part = random_cut_part(seed, key[i], n_parts);
      }
      mine[i] = part == part_id;
      if (want_rf) {
        const uint64_t bit = 1ull << (part & 63);
        __atomic_fetch_or(&rf_bits[(size_t)(lo * rf_words + part / 64)], bit, __ATOMIC_RELAXED);
        __atomic_fetch_or(&rf_bits[(size_t)(hi * rf_words + part / 64)], bit, __ATOMIC_RELAXED);
      }
    }
  });
  // 4. this partition's edges, sorted and unique (all copies of a repeated edge agree on the partition)
  std::vector<uint64_t> my_keys;
  my_keys.reserve((size_t)(n_edges / std::max(1, n_parts) + 16));
  for (int64_t i = 0; i < n_edges; ++i)
    if (mine[i]) my_keys.push_back(key[i]);
  std::vector<uint64_t>().swap(key);
  std::vector<uint8_t>().swap(mine);
  sort_keys(my_keys, n_nodes);
  my_keys.erase(std::unique(my_keys.begin(), my_keys.end()), my_keys.end());
  // 5. structures of the partition
  return structures_from_keys(P, n_nodes, my_keys, deg_g, rf_bits, rf_words);
}

static int32_t to_device(cofree_partition* P) {
  COFREE_HIP_CHECK(hipGetDevice(&P->device));
  std::vector<float> inv_deg, gcn;
  norms_from_rowptr(P->rowptr, &inv_deg, &gcn);
  COFREE_TRY(upload(&P->d_rowptr, P->rowptr));
  COFREE_TRY(upload(&P->d_col, P->col));
  COFREE_TRY(upload(&P->d_eid, P->eid));
  COFREE_TRY(upload(&P->d_deg_local, P->deg_local));
  COFREE_TRY(upload(&P->d_dar_weight, P->dar_weight));
  COFREE_TRY(upload(&P->d_inv_deg, inv_deg));
  COFREE_TRY(upload(&P->d_gcn_norm, gcn));
  COFREE_TRY(upload(&P->d_local2global, P->local2global));
  {
    const size_t cnt = P->col.empty() ? 1 : P->col.size();
    COFREE_HIP_CHECK(hipMalloc((void**)&P->d_val_inv_deg, cnt * sizeof(float)));
    COFREE_HIP_CHECK(hipMalloc((void**)&P->d_val_gcn_norm, cnt * sizeof(float)));
    COFREE_TRY(launch_entry_scales(P->d_col, (int64_t)P->col.size(), P->d_inv_deg, P->d_gcn_norm, P->d_val_inv_deg,
                                   P->d_val_gcn_norm, nullptr));
    COFREE_HIP_CHECK(hipStreamSynchronize(nullptr));
  }
  {
    // processing order of the short-row aggregation: rows of similar degree share a wavefront
    std::vector<int32_t> order((size_t)P->n_nodes);
    for (int64_t v = 0; v < P->n_nodes; ++v) order[v] = (int32_t)v;
    std::stable_sort(order.begin(), order.end(),
                     [&](int32_t a, int32_t b) { return P->deg_local[a] > P->deg_local[b]; });
    COFREE_TRY(upload(&P->d_order, order));
    P->buckets = DegreeBuckets();
    for (int64_t v = 0; v < P->n_nodes; ++v) {
      const int64_t d = P->deg_local[v];
      if (d >= AGG_HUB_MIN) P->buckets.n_hub++, P->buckets.nnz_hub += d;
    }
  }
  {
    DeviceGraph g = P->graph();
    COFREE_TRY(build_slot_csr(g, &P->d_slots, nullptr));
    COFREE_HIP_CHECK(hipStreamSynchronize(nullptr));
  }
  if (!P->rf.empty()) {
    std::vector<float> inv_rf(P->rf.size());
    for (size_t v = 0; v < inv_rf.size(); ++v) inv_rf[v] = (float)(1.0 / (double)P->rf[v]);
    COFREE_TRY(upload(&P->d_inv_rf, inv_rf));
  }
  P->on_device = true;
  return COFREE_OK;
}

int32_t select_graph(const cofree_partition* part, const cofree_masks* masks, int32_t mask_id, DeviceGraph* out) {
  COFREE_REQUIRE(part != nullptr, "partition is NULL");
  if (!part->on_device) return fail(COFREE_ESTATE, "partition has no device copy (built with COFREE_HOST_ONLY)");
  if (!masks) {
    *out = part->graph();
    return COFREE_OK;
  }
  COFREE_REQUIRE(masks->n_nodes == part->n_nodes && masks->n_edges == part->n_edges,
                 "masks were built for a different partition");
  COFREE_REQUIRE(mask_id >= 0 && mask_id < masks->K, "mask_id out of range");
  const auto& d = masks->dev[mask_id];
  out->rowptr = d.rowptr;
  out->col = d.col;
  out->inv_deg = d.inv_deg;
  out->gcn_norm = d.gcn_norm;
  out->val_inv_deg = d.val_inv_deg;
  out->val_gcn_norm = d.val_gcn_norm;
  out->order = d.order;
  d.slots.attach(out);
  out->n = part->n_nodes;
  out->nnz = d.nnz;
  out->n_hub = d.buckets.n_hub;
  out->nnz_hub = d.buckets.nnz_hub;
  return COFREE_OK;
}

}  // namespace cofree

using namespace cofree;

extern "C" {

const char* cofree_last_error(void) { return g_last_error.c_str(); }

int32_t cofree_device_count(void) {
  int n = 0;
  if (hipGetDeviceCount(&n) != hipSuccess) return -1;
  return n;
}

int32_t cofree_build_partition(int64_t n_nodes, int64_t n_edges, const int64_t* src, const int64_t* dst,
                               int32_t n_parts, int32_t part_id, uint64_t seed, const int32_t* assignment,
                               uint32_t flags, cofree_partition** out) {
  COFREE_REQUIRE(out != nullptr, "out is NULL");
  *out = nullptr;
  COFREE_REQUIRE(n_nodes > 0 && n_nodes <= ((int64_t)1 << 32), "n_nodes must be in [1, 2^32]");
  COFREE_REQUIRE(n_edges >= 0, "n_edges is negative");
  COFREE_REQUIRE(n_edges == 0 || (src && dst), "src/dst is NULL");
  COFREE_REQUIRE(n_parts >= 1, "n_parts must be >= 1");
  COFREE_REQUIRE(part_id >= 0 && part_id < n_parts, "part_id must be in [0, n_parts)");
  cofree_partition* P = new (std::nothrow) cofree_partition();
  if (!P) return fail(COFREE_ENOMEM, "out of host memory");
  int32_t rc;
  try {
    rc = build(n_nodes, n_edges, src, dst, n_parts, part_id, seed, assignment, flags, P);
    if (rc == COFREE_OK && !(flags & COFREE_HOST_ONLY)) rc = to_device(P);
  } catch (const std::bad_alloc&) {
    rc = fail(COFREE_ENOMEM, "out of host memory while building the partition");
  }
  if (rc != COFREE_OK) {
    cofree_partition_free(P);
    return rc;
  }
  *out = P;
  return COFREE_OK;
}

// ---- the same partition from an edge list that arrives in pieces ------------------------------------
struct cofree_partition_builder {
  int64_t n_nodes = 0;
  int32_t n_parts = 0, part_id = 0;
  uint64_t seed = 0;
  uint32_t flags = 0;
  int64_t rf_words = 0;
  int64_t edges_seen = 0;
  std::vector<int32_t> deg_g;     // D(v), counted as the edges arrive
  std::vector<uint64_t> my_keys;  // keys of the edges that fall into this partition, in arrival order
  std::vector<uint64_t> rf_bits;
};

int32_t cofree_partition_builder_begin(int64_t n_nodes, int32_t n_parts, int32_t part_id, uint64_t seed,
                                       uint32_t flags, cofree_partition_builder** out) {
  COFREE_REQUIRE(out != nullptr, "out is NULL");
  *out = nullptr;
  COFREE_REQUIRE(n_nodes > 0 && n_nodes <= ((int64_t)1 << 32), "n_nodes must be in [1, 2^32]");
  COFREE_REQUIRE(n_parts >= 1, "n_parts must be >= 1");
  COFREE_REQUIRE(part_id >= 0 && part_id < n_parts, "part_id must be in [0, n_parts)");
  COFREE_REQUIRE((flags & ~(COFREE_DEDUP | COFREE_HOST_ONLY | COFREE_WITH_RF)) == 0,
                 "partition_builder: only COFREE_DEDUP, COFREE_HOST_ONLY and COFREE_WITH_RF apply to a streamed build "
                 "(the degree-aware cut needs every degree before the first edge is assigned)");
  cofree_partition_builder* b = new (std::nothrow) cofree_partition_builder();
  if (!b) return fail(COFREE_ENOMEM, "out of host memory");
  try {
    b->n_nodes = n_nodes;
    b->n_parts = n_parts;
    b->part_id = part_id;
    b->seed = seed;
    b->flags = flags;
    b->deg_g.assign((size_t)n_nodes, 0);
    if (flags & COFREE_WITH_RF) {
      b->rf_words = ((int64_t)n_parts + 63) / 64;
      b->rf_bits.assign((size_t)(n_nodes * b->rf_words), 0ull);
    }
  } catch (const std::bad_alloc&) {
    delete b;
    return fail(COFREE_ENOMEM, "out of host memory for the per-node degree counters");
  }
  *out = b;
  return COFREE_OK;
}

int32_t cofree_partition_builder_add_edges(cofree_partition_builder* b, int64_t n_edges, const int64_t* src,
                                           const int64_t* dst) {
  COFREE_REQUIRE(b != nullptr, "partition_builder: builder is NULL");
  COFREE_REQUIRE(n_edges >= 0, "n_edges is negative");
  if (n_edges == 0) return COFREE_OK;
  COFREE_REQUIRE(src && dst, "src/dst is NULL");
  try {
    std::vector<uint64_t> key((size_t)n_edges);
    const int bad = canonical_keys(b->n_nodes, n_edges, src, dst, key.data());
    if (bad == 1) return fail(COFREE_EINVAL, "edge endpoint out of range [0, n_nodes)");
    if (bad == 2) return fail(COFREE_EINVAL, "self-loop in edge list");
    // repeats inside this piece are dropped (COFREE_DEDUP) or rejected; copies of an edge in different
    // pieces cannot be seen here - those that fall into this partition are caught by finish
    sort_keys(key, b->n_nodes);
    if (std::adjacent_find(key.begin(), key.end()) != key.end()) {
      if (!(b->flags & COFREE_DEDUP)) return fail(COFREE_EINVAL, "repeated edge (set COFREE_DEDUP to drop)");
      key.erase(std::unique(key.begin(), key.end()), key.end());
    }
    const int64_t n = (int64_t)key.size();
    const unsigned T = (n < (1 << 16)) ? 1u : host_threads();
    std::vector<std::vector<uint64_t>> mine(T);
    const int64_t chunk = (n + T - 1) / T;
    auto work = [&](unsigned t) {
      const int64_t lo_i = (int64_t)t * chunk, hi_i = std::min(n, lo_i + chunk);
      auto& out = mine[t];
      for (int64_t i = lo_i; i < hi_i; ++i) {
        const uint64_t lo = key[i] >> 32, hi = key[i] & 0xffffffffu;
        __atomic_fetch_add(&b->deg_g[lo], 1, __ATOMIC_RELAXED);
        __atomic_fetch_add(&b->deg_g[hi], 1, __ATOMIC_RELAXED);
        const int32_t part = random_cut_part(b->seed, key[i], b->n_parts);
        if (b->rf_words) {
          const uint64_t bit = 1ull << (part & 63);
          __atomic_fetch_or(&b->rf_bits[(size_t)(lo * b->rf_words + part / 64)], bit, __ATOMIC_RELAXED);
          __atomic_fetch_or(&b->rf_bits[(size_t)(hi * b->rf_words + part / 64)], bit, __ATOMIC_RELAXED);
        }
        if (part == b->part_id) out.push_back(key[i]);
      }
    };
    if (T == 1) {
      work(0);
    } else {
      std::vector<std::thread> th;
      for (unsigned t = 0; t < T; ++t) th.emplace_back(work, t);
      for (auto& x : th) x.join();
    }
    for (auto& v : mine) b->my_keys.insert(b->my_keys.end(), v.begin(), v.end());
    b->edges_seen += n;
  } catch (const std::bad_alloc&) {
    return fail(COFREE_ENOMEM, "out of host memory while adding edges");
  }
  return COFREE_OK;
}

void cofree_partition_builder_free(cofree_partition_builder* b) { delete b; }

int32_t cofree_partition_builder_finish(cofree_partition_builder* b, cofree_partition** out) {
  COFREE_REQUIRE(out != nullptr, "out is NULL");
  *out = nullptr;
  COFREE_REQUIRE(b != nullptr, "partition_builder: builder is NULL");
  cofree_partition* P = new (std::nothrow) cofree_partition();
  if (!P) {
    delete b;
    return fail(COFREE_ENOMEM, "out of host memory");
  }
  int32_t rc;
  try {
    sort_keys(b->my_keys, b->n_nodes);
    if (std::adjacent_find(b->my_keys.begin(), b->my_keys.end()) != b->my_keys.end())
      rc = fail(COFREE_EINVAL, "partition_builder: an edge arrived in more than one add_edges call");
    else
      rc = structures_from_keys(P, b->n_nodes, b->my_keys, b->deg_g, b->rf_bits, b->rf_words);
    const uint32_t flags = b->flags;
    delete b;  // the counters and keys are no longer needed: free them before the device copies are made
    b = nullptr;
    if (rc == COFREE_OK && !(flags & COFREE_HOST_ONLY)) rc = to_device(P);
  } catch (const std::bad_alloc&) {
    rc = fail(COFREE_ENOMEM, "out of host memory while building the partition");
  }
  delete b;
  if (rc != COFREE_OK) {
    cofree_partition_free(P);
    return rc;
  }
  *out = P;
  return COFREE_OK;
}

void cofree_partition_free(cofree_partition* P) {
  if (!P) return;
  if (P->on_device || P->d_rowptr) {
    (void)hipFree(P->d_rowptr);
    (void)hipFree(P->d_col);
    (void)hipFree(P->d_eid);
    (void)hipFree(P->d_deg_local);
    (void)hipFree(P->d_dar_weight);
    (void)hipFree(P->d_inv_deg);
    (void)hipFree(P->d_gcn_norm);
    (void)hipFree(P->d_val_inv_deg);
    (void)hipFree(P->d_val_gcn_norm);
    (void)hipFree(P->d_local2global);
    (void)hipFree(P->d_order);
    free_slot_csr(&P->d_slots);
    (void)hipFree(P->d_inv_rf);
  }
  delete P;
}

int32_t cofree_replication_factor(int64_t n_nodes_full, const cofree_partition* const* parts, int32_t n_parts,
                                  double* rf_out) {
  COFREE_REQUIRE(rf_out != nullptr && parts != nullptr, "replication_factor: NULL argument");
  COFREE_REQUIRE(n_nodes_full > 0 && n_parts >= 1, "replication_factor: n_nodes_full and n_parts must be positive");
  int64_t total = 0;
  for (int32_t i = 0; i < n_parts; ++i) {
    COFREE_REQUIRE(parts[i] != nullptr, "replication_factor: partition is NULL");
    COFREE_REQUIRE(parts[i]->n_nodes_full == n_nodes_full || parts[i]->n_nodes == 0,
                   "replication_factor: partition was built from a graph of another size");
    total += parts[i]->n_nodes;
  }
  *rf_out = (double)total / (double)n_nodes_full;
  return COFREE_OK;
}

int64_t cofree_partition_num_nodes(const cofree_partition* P) { return P ? P->n_nodes : -1; }
int64_t cofree_partition_num_edges(const cofree_partition* P) { return P ? P->n_edges : -1; }
int64_t cofree_partition_num_nnz(const cofree_partition* P) { return P ? P->nnz : -1; }

int32_t cofree_partition_host_array(const cofree_partition* P, int32_t which, const void** ptr, int64_t* count) {
  COFREE_REQUIRE(P && ptr && count, "NULL argument");
  switch (which) {
    case COFREE_ARR_LOCAL2GLOBAL: *ptr = P->local2global.data(); *count = P->n_nodes; break;
    case COFREE_ARR_ROWPTR: *ptr = P->rowptr.data(); *count = P->n_nodes + 1; break;
    case COFREE_ARR_COL: *ptr = P->col.data(); *count = P->nnz; break;
    case COFREE_ARR_EID: *ptr = P->eid.data(); *count = P->nnz; break;
    case COFREE_ARR_DEG_LOCAL: *ptr = P->deg_local.data(); *count = P->n_nodes; break;
    case COFREE_ARR_DEG_GLOBAL: *ptr = P->deg_global.data(); *count = P->n_nodes; break;
    case COFREE_ARR_DAR_WEIGHT: *ptr = P->dar_weight.data(); *count = P->n_nodes; break;
    case COFREE_ARR_EDGE_LO: *ptr = P->edge_lo.data(); *count = P->n_edges; break;
    case COFREE_ARR_EDGE_HI: *ptr = P->edge_hi.data(); *count = P->n_edges; break;
    case COFREE_ARR_RF:
      if (P->rf.empty() && P->n_nodes > 0) return fail(COFREE_ESTATE, "partition was built without COFREE_WITH_RF");
      *ptr = P->rf.data();
      *count = P->n_nodes;
      break;
    default: return fail(COFREE_EINVAL, "unknown array id");
  }
  return COFREE_OK;
}

int32_t cofree_partition_device_array(const cofree_partition* P, int32_t which, const void** ptr, int64_t* count) {
  COFREE_REQUIRE(P && ptr && count, "NULL argument");
  if (!P->on_device) return fail(COFREE_ESTATE, "partition has no device copy");
  switch (which) {
    case COFREE_ARR_LOCAL2GLOBAL: *ptr = P->d_local2global; *count = P->n_nodes; break;
    case COFREE_ARR_ROWPTR: *ptr = P->d_rowptr; *count = P->n_nodes + 1; break;
    case COFREE_ARR_COL: *ptr = P->d_col; *count = P->nnz; break;
    case COFREE_ARR_DEG_LOCAL: *ptr = P->d_deg_local; *count = P->n_nodes; break;
    case COFREE_ARR_DAR_WEIGHT: *ptr = P->d_dar_weight; *count = P->n_nodes; break;
    default: return fail(COFREE_EINVAL, "array is not kept on the device");
  }
  return COFREE_OK;
}

int32_t cofree_dropedge_pick(uint64_t seed, uint64_t epoch, int32_t K, int32_t* k_out) {
  COFREE_REQUIRE(k_out != nullptr, "k_out is NULL");
  COFREE_REQUIRE(K >= 1, "K must be >= 1");
  const uint32_t r = draw1(seed, STREAM_PICK, epoch, 0u);
  *k_out = (int32_t)(((uint64_t)r * (uint64_t)K) >> 32);
  return COFREE_OK;
}

}  // extern "C"
