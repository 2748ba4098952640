// Streaming partitioner of the paper (Algorithm 1 and the edge pass of the
// section on graph partitioning) as a workload producer: it turns a synthetic
// graph into partitions that own a node set, keep the full neighbour list of
// every owned node and carry replicas of the outside neighbours.  Host-only,
// sequential, as the algorithm is (one pass over the edge stream, then work on
// clusters).  None of the training step's arithmetic is here.
//
// Choices the paper leaves open (the test oracle takes the same ones):
//  * ties go to the candidate met first: the strict comparisons of Alg. 1 keep
//    the earlier richest neighbour and the earlier representative (nodes in
//    ascending id); equal cluster sizes are ordered by cluster number, equal
//    partition loads by partition index;
//  * a node the stream never shows (degree 0) forms its own cluster after the
//    stream, numbered after the streamed clusters in ascending node id; it has
//    no richest neighbour and is never merged away;
//  * a cluster that absorbed another is visited at the rank of its new size;
//  * the merge test is "<=" as in Alg. 1.
//
// Built into libsdt_gen.so together with gen.cpp.

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <functional>
#include <numeric>
#include <queue>
#include <tuple>
#include <vector>

namespace {

struct Spring {
  int64_t n = 0;
  std::vector<int32_t> cluster_stream, cluster_merged, part;
  int64_t n_clusters_stream = 0, n_clusters_merged = 0;
};

struct Partition {
  int64_t n_owned = 0;
  std::vector<int64_t> indptr;
  std::vector<int32_t> indices, global_id;
};

inline uint64_t splitmix(uint64_t& s) {
  uint64_t z = (s += 0x9E3779B97F4A7C15ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

}  // namespace

extern "C" {

// Number of undirected edges of a symmetric CSR (entries with column > row).
int64_t sdtgen_edge_count(int64_t n, const int64_t* indptr, const int32_t* indices) {
  int64_t m = 0;
  for (int64_t u = 0; u < n; ++u)
    for (int64_t e = indptr[u]; e < indptr[u + 1]; ++e) m += indices[e] > u;
  return m;
}

// The edge stream: every undirected edge once as (u, v) with u < v, in row order when
// order_seed == 0, else shuffled by a seeded Fisher-Yates pass with a random orientation.
void sdtgen_edge_stream(int64_t n, const int64_t* indptr, const int32_t* indices, uint64_t order_seed,
                        int32_t* eu, int32_t* ev) {
  int64_t m = 0;
  for (int64_t u = 0; u < n; ++u)
    for (int64_t e = indptr[u]; e < indptr[u + 1]; ++e)
      if (indices[e] > u) { eu[m] = (int32_t)u; ev[m] = indices[e]; ++m; }
  if (order_seed == 0) return;
  uint64_t s = order_seed;
  for (int64_t i = m - 1; i > 0; --i) {
    int64_t j = (int64_t)(((unsigned __int128)splitmix(s) * (uint64_t)(i + 1)) >> 64);
    std::swap(eu[i], eu[j]);
    std::swap(ev[i], ev[j]);
  }
  for (int64_t i = 0; i < m; ++i)
    if (splitmix(s) & 1) std::swap(eu[i], ev[i]);
}

// Alg. 1 over an explicit edge stream.  degree[v] is d(v); p partitions; beta the balance
// factor; tau_vol the volume threshold of the clustering step.
void* sdtgen_spring(int64_t n, const int64_t* degree, const int32_t* eu, const int32_t* ev, int64_t m, int32_t p,
                    double beta, int64_t tau_vol) {
  Spring* S = new Spring;
  S->n = n;
  std::vector<int32_t> c(n, -1), rich(n, -1);
  std::vector<int64_t> vol;
  // ---- node clustering -------------------------------------------------------
  for (int64_t e = 0; e < m; ++e) {
    const int32_t u = eu[e], v = ev[e];
    if (c[u] < 0) { c[u] = (int32_t)vol.size(); vol.push_back(degree[u]); }
    if (c[v] < 0) { c[v] = (int32_t)vol.size(); vol.push_back(degree[v]); }
    const int32_t cu = c[u], cv = c[v];
    if (cu != cv && vol[cu] <= tau_vol && vol[cv] <= tau_vol) {
      if (vol[cu] <= vol[cv]) { vol[cu] -= degree[u]; vol[cv] += degree[u]; c[u] = cv; }
      else                    { vol[cv] -= degree[v]; vol[cu] += degree[v]; c[v] = cu; }
    }
    if (rich[u] < 0 || degree[rich[u]] < degree[v]) rich[u] = v;
    if (rich[v] < 0 || degree[rich[v]] < degree[u]) rich[v] = u;
  }
  for (int64_t v = 0; v < n; ++v)
    if (c[v] < 0) { c[v] = (int32_t)vol.size(); vol.push_back(degree[v]); }
  const int64_t K = (int64_t)vol.size();
  S->cluster_stream = c;

  // ---- cluster merging -------------------------------------------------------
  std::vector<int64_t> size(K, 0);
  for (int64_t v = 0; v < n; ++v) size[c[v]]++;
  for (int64_t k = 0; k < K; ++k) S->n_clusters_stream += size[k] > 0;
  auto rich_deg = [&](int32_t v) -> int64_t { return rich[v] >= 0 ? degree[rich[v]] : -1; };
  std::vector<int32_t> rep(K, -1);
  for (int64_t v = 0; v < n; ++v) {
    if (rich[v] < 0) continue;
    int32_t k = c[v];
    if (rep[k] < 0 || rich_deg(rep[k]) < rich_deg((int32_t)v)) rep[k] = (int32_t)v;
  }
  // merged clusters as a forest: into[k] == k for a live cluster
  std::vector<int32_t> into(K);
  std::iota(into.begin(), into.end(), 0);
  std::function<int32_t(int32_t)> find = [&](int32_t k) {
    int32_t r = k;
    while (into[r] != r) r = into[r];
    while (into[k] != r) { int32_t nx = into[k]; into[k] = r; k = nx; }
    return r;
  };
  using Entry = std::tuple<int64_t, int32_t, int32_t>;          // (size, cluster, version)
  std::priority_queue<Entry, std::vector<Entry>, std::greater<Entry>> heap;
  std::vector<int32_t> version(K, 0);
  for (int64_t k = 0; k < K; ++k)
    if (size[k] > 0) heap.emplace(size[k], (int32_t)k, 0);
  const double limit = beta * (double)n / (double)p;
  while (!heap.empty()) {
    auto [sz, i, ver] = heap.top();
    heap.pop();
    if (into[i] != i || ver != version[i] || rep[i] < 0) continue;   // merged away, outdated entry, or no neighbour
    const int32_t j = find(c[rich[rep[i]]]);
    if (j == i || (double)(size[i] + size[j]) > limit) continue;
    into[i] = j;
    size[j] += size[i];
    size[i] = 0;
    if (rep[j] < 0 || rich_deg(rep[j]) < rich_deg(rep[i])) rep[j] = rep[i];
    heap.emplace(size[j], j, ++version[j]);
  }
  S->cluster_merged.resize(n);
  for (int64_t v = 0; v < n; ++v) S->cluster_merged[v] = find(c[v]);
  // ---- clusters to partitions: largest first, to the least loaded partition ----
  std::vector<int32_t> order;
  for (int64_t k = 0; k < K; ++k)
    if (into[k] == k && size[k] > 0) order.push_back((int32_t)k);
  S->n_clusters_merged = (int64_t)order.size();
  std::sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return size[a] != size[b] ? size[a] > size[b] : a < b; });
  std::vector<int64_t> load(p, 0);
  std::vector<int32_t> assign(K, -1);
  using Load = std::pair<int64_t, int32_t>;                       // (load, partition)
  std::priority_queue<Load, std::vector<Load>, std::greater<Load>> least;
  for (int32_t t = 0; t < p; ++t) least.emplace(0, t);
  for (int32_t k : order) {
    auto [ld, t] = least.top();
    least.pop();
    assign[k] = t;
    least.emplace(ld + size[k], t);
  }
  S->part.resize(n);
  for (int64_t v = 0; v < n; ++v) S->part[v] = assign[S->cluster_merged[v]];
  return S;
}

// which: 0 = clusters after the streaming step, 1 = after merging (non-empty ones).
int64_t sdtgen_spring_clusters(void* h, int32_t which) {
  Spring* S = (Spring*)h;
  return which == 0 ? S->n_clusters_stream : S->n_clusters_merged;
}

// Any of the three outputs may be null.
void sdtgen_spring_copy(void* h, int32_t* part, int32_t* cluster_stream, int32_t* cluster_merged) {
  Spring* S = (Spring*)h;
  if (part) std::memcpy(part, S->part.data(), sizeof(int32_t) * S->n);
  if (cluster_stream) std::memcpy(cluster_stream, S->cluster_stream.data(), sizeof(int32_t) * S->n);
  if (cluster_merged) std::memcpy(cluster_merged, S->cluster_merged.data(), sizeof(int32_t) * S->n);
}

void sdtgen_spring_free(void* h) { delete (Spring*)h; }

// Edge pass for partition `which`: local ids are the owned nodes in ascending global id, then the
// replicas in ascending global id; an owned row keeps every neighbour, a replica's row only the
// neighbours this partition owns; rows sorted ascending in local ids.
void* sdtgen_partition(int64_t n, const int64_t* indptr, const int32_t* indices, const int32_t* part, int32_t which) {
  Partition* P = new Partition;
  std::vector<int32_t> local(n, -1);
  std::vector<uint8_t> is_replica(n, 0);
  for (int64_t v = 0; v < n; ++v)
    if (part[v] == which) { local[v] = (int32_t)P->global_id.size(); P->global_id.push_back((int32_t)v); }
  P->n_owned = (int64_t)P->global_id.size();
  for (int64_t i = 0; i < P->n_owned; ++i) {
    const int64_t v = P->global_id[i];
    for (int64_t e = indptr[v]; e < indptr[v + 1]; ++e)
      if (part[indices[e]] != which) is_replica[indices[e]] = 1;
  }
  for (int64_t v = 0; v < n; ++v)
    if (is_replica[v]) { local[v] = (int32_t)P->global_id.size(); P->global_id.push_back((int32_t)v); }
  const int64_t nl = (int64_t)P->global_id.size();
  P->indptr.assign(nl + 1, 0);
  for (int64_t i = 0; i < nl; ++i) {
    const int64_t v = P->global_id[i];
    int64_t cnt = 0;
    if (i < P->n_owned) cnt = indptr[v + 1] - indptr[v];
    else
      for (int64_t e = indptr[v]; e < indptr[v + 1]; ++e) cnt += part[indices[e]] == which;
    P->indptr[i + 1] = P->indptr[i] + cnt;
  }
  P->indices.resize(P->indptr[nl]);
  for (int64_t i = 0; i < nl; ++i) {
    const int64_t v = P->global_id[i];
    int32_t* out = P->indices.data() + P->indptr[i];
    int64_t k = 0;
    for (int64_t e = indptr[v]; e < indptr[v + 1]; ++e)
      if (i < P->n_owned || part[indices[e]] == which) out[k++] = local[indices[e]];
    std::sort(out, out + k);
  }
  return P;
}

int64_t sdtgen_partition_nodes(void* h) { return (int64_t)((Partition*)h)->global_id.size(); }
int64_t sdtgen_partition_owned(void* h) { return ((Partition*)h)->n_owned; }
int64_t sdtgen_partition_nnz(void* h) { return (int64_t)((Partition*)h)->indices.size(); }
void sdtgen_partition_copy(void* h, int64_t* indptr, int32_t* indices, int32_t* global_id) {
  Partition* P = (Partition*)h;
  std::memcpy(indptr, P->indptr.data(), sizeof(int64_t) * P->indptr.size());
  std::memcpy(indices, P->indices.data(), sizeof(int32_t) * P->indices.size());
  std::memcpy(global_id, P->global_id.data(), sizeof(int32_t) * P->global_id.size());
}
void sdtgen_partition_free(void* h) { delete (Partition*)h; }

}  // extern "C"
