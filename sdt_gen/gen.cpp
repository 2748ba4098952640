// Seeded synthetic-input generator for the per-worker GraphSAGE step.
//
// Host-only C++ (OpenMP).  It produces the *inputs* that both the CPU oracle
// and the HIP library consume: power-law graphs as CSR (R-MAT and Chung-Lu,
// symmetrised, self-loops dropped, rows sorted and de-duplicated), N(0,1)
// node features, uniform labels, Glorot-uniform weights and per-step seed
// batches.  It contains none of the method's arithmetic (no sampling rule,
// no aggregation, no projection) and is linked by neither side.
//
// Every value is a pure function of (seed, domain, index) through a
// counter-based generator, so the output does not depend on the number of
// threads.  The graphs stand in for the public datasets of the paper's
// Table "Dataset statistics" (node/edge counts, feature and class counts).
//
// Build: g++ -O3 -fopenmp -shared -fPIC gen.cpp -o libsdt_gen.so

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <unordered_map>
#include <vector>
#include <omp.h>

namespace {

// ---- counter-based generator (Philox4x32-10, Salmon et al. SC'11) ----------
struct R4 { uint32_t w[4]; };

inline R4 philox(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint64_t seed) {
  uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
  for (int r = 0; r < 10; ++r) {
    uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  return R4{{c0, c1, c2, c3}};
}

enum Domain : uint32_t { DOM_BATCH = 1, DOM_FEAT = 2, DOM_LABEL = 3, DOM_WEIGHT = 4,
                         DOM_EDGE = 5, DOM_PERM = 6 };

inline uint32_t mulhi_range(uint32_t r, uint32_t n) { return (uint32_t)(((uint64_t)r * n) >> 32); }

struct Csr {
  int64_t n = 0;
  std::vector<int64_t> indptr;
  std::vector<int32_t> indices;
};

// Random relabelling of the node ids so that hubs are spread over the id range.
std::vector<int32_t> make_perm(int64_t n, uint64_t seed) {
  std::vector<int32_t> p(n);
  for (int64_t i = 0; i < n; ++i) p[i] = (int32_t)i;
  for (int64_t i = n - 1; i > 0; --i) {
    R4 r = philox((uint32_t)i, (uint32_t)(i >> 32), DOM_PERM << 16, 0, seed);
    uint64_t x = ((uint64_t)r.w[0] << 32) | r.w[1];
    int64_t j = (int64_t)(((unsigned __int128)x * (uint64_t)(i + 1)) >> 64);
    std::swap(p[i], p[j]);
  }
  return p;
}

// (u[e], v[e]) pairs -> symmetric CSR without self-loops, rows sorted, unique.
Csr* build_csr(int64_t n, const std::vector<int32_t>& eu, const std::vector<int32_t>& ev) {
  const int64_t m = (int64_t)eu.size();
  Csr* g = new Csr;
  g->n = n;
  std::vector<int64_t> cnt(n + 1, 0);
#pragma omp parallel for schedule(static)
  for (int64_t e = 0; e < m; ++e) {
    if (eu[e] == ev[e]) continue;
#pragma omp atomic
    cnt[eu[e] + 1]++;
#pragma omp atomic
    cnt[ev[e] + 1]++;
  }
  for (int64_t i = 0; i < n; ++i) cnt[i + 1] += cnt[i];
  std::vector<int32_t> raw(cnt[n]);
  std::vector<int64_t> cur(cnt.begin(), cnt.end() - 1);
#pragma omp parallel for schedule(static)
  for (int64_t e = 0; e < m; ++e) {
    int32_t u = eu[e], v = ev[e];
    if (u == v) continue;
    int64_t pu, pv;
#pragma omp atomic capture
    pu = cur[u]++;
#pragma omp atomic capture
    pv = cur[v]++;
    raw[pu] = v;
    raw[pv] = u;
  }
  std::vector<int64_t> deg(n + 1, 0);
#pragma omp parallel for schedule(dynamic, 1024)
  for (int64_t i = 0; i < n; ++i) {
    int32_t* b = raw.data() + cnt[i];
    int32_t* e = raw.data() + cnt[i + 1];
    std::sort(b, e);
    deg[i + 1] = std::unique(b, e) - b;
  }
  g->indptr.assign(n + 1, 0);
  for (int64_t i = 0; i < n; ++i) g->indptr[i + 1] = g->indptr[i] + deg[i + 1];
  g->indices.resize(g->indptr[n]);
#pragma omp parallel for schedule(dynamic, 1024)
  for (int64_t i = 0; i < n; ++i)
    std::memcpy(g->indices.data() + g->indptr[i], raw.data() + cnt[i], sizeof(int32_t) * deg[i + 1]);
  return g;
}

inline void box_muller(uint32_t a, uint32_t b, float* z0, float* z1) {
  // u1 in (0,1], u2 in [0,1)
  double u1 = ((double)a + 1.0) * (1.0 / 4294967296.0);
  double u2 = (double)b * (1.0 / 4294967296.0);
  double r = std::sqrt(-2.0 * std::log(u1));
  double t = 6.283185307179586476925 * u2;
  *z0 = (float)(r * std::cos(t));
  *z1 = (float)(r * std::sin(t));
}

inline uint16_t f32_to_bf16_rne(float f) {
  uint32_t x;
  std::memcpy(&x, &f, 4);
  x += 0x7FFFu + ((x >> 16) & 1u);
  return (uint16_t)(x >> 16);
}

}  // namespace

extern "C" {

// R-MAT: `m` node pairs, each chosen by log2n quadrant draws with probabilities
// (a, b, c, 1-a-b-c); ids relabelled by a seeded permutation; every pair is
// stored in both directions.  Returns an opaque handle.
void* sdtgen_rmat(int32_t log2n, int64_t m, double a, double b, double c, uint64_t seed) {
  const int64_t n = (int64_t)1 << log2n;
  std::vector<int32_t> eu(m), ev(m);
  const uint32_t ta = (uint32_t)(a * 65536.0), tb = (uint32_t)((a + b) * 65536.0),
                 tc = (uint32_t)((a + b + c) * 65536.0);
  std::vector<int32_t> perm = make_perm(n, seed);
#pragma omp parallel for schedule(static)
  for (int64_t e = 0; e < m; ++e) {
    uint32_t u = 0, v = 0;
    int lvl = 0;
    for (uint32_t blk = 0; lvl < log2n; ++blk) {
      R4 r = philox((uint32_t)e, (uint32_t)(e >> 32), (DOM_EDGE << 16) | blk, 0, seed);
      for (int h = 0; h < 8 && lvl < log2n; ++h, ++lvl) {
        uint32_t x = (r.w[h >> 1] >> ((h & 1) * 16)) & 0xFFFFu;
        uint32_t q = (x < ta) ? 0 : (x < tb) ? 1 : (x < tc) ? 2 : 3;
        u = (u << 1) | (q >> 1);
        v = (v << 1) | (q & 1);
      }
    }
    eu[e] = perm[u];
    ev[e] = perm[v];
  }
  return build_csr(n, eu, ev);
}

// Chung-Lu: expected degrees w_i ~ (i+1)^(-1/(gamma-1)), scaled to mean
// `avg_deg` and capped at sqrt(sum w); `m` pairs with both endpoints drawn
// proportionally to w; ids relabelled by a seeded permutation.
void* sdtgen_chunglu(int64_t n, int64_t m, double avg_deg, double gamma, uint64_t seed) {
  std::vector<double> w(n);
  const double ex = -1.0 / (gamma - 1.0);
  for (int64_t i = 0; i < n; ++i) w[i] = std::pow((double)(i + 1), ex);
  const double cap = std::sqrt((double)n * avg_deg);
  for (int it = 0; it < 16; ++it) {
    double s = 0;
    for (int64_t i = 0; i < n; ++i) s += w[i];
    double sc = (double)n * avg_deg / s;
    for (int64_t i = 0; i < n; ++i) w[i] = std::min(w[i] * sc, cap);
  }
  std::vector<double> cdf(n);
  double s = 0;
  for (int64_t i = 0; i < n; ++i) { s += w[i]; cdf[i] = s; }
  std::vector<int32_t> perm = make_perm(n, seed);
  std::vector<int32_t> eu(m), ev(m);
#pragma omp parallel for schedule(static)
  for (int64_t e = 0; e < m; ++e) {
    R4 r = philox((uint32_t)e, (uint32_t)(e >> 32), DOM_EDGE << 16, 1, seed);
    double x0 = (((uint64_t)r.w[0] << 21) ^ (r.w[1] >> 11)) * (1.0 / 9007199254740992.0) * s;
    double x1 = (((uint64_t)r.w[2] << 21) ^ (r.w[3] >> 11)) * (1.0 / 9007199254740992.0) * s;
    int64_t u = std::upper_bound(cdf.begin(), cdf.end(), x0) - cdf.begin();
    int64_t v = std::upper_bound(cdf.begin(), cdf.end(), x1) - cdf.begin();
    eu[e] = perm[std::min(u, n - 1)];
    ev[e] = perm[std::min(v, n - 1)];
  }
  return build_csr(n, eu, ev);
}

int64_t sdtgen_csr_nodes(void* h) { return ((Csr*)h)->n; }
int64_t sdtgen_csr_nnz(void* h) { return (int64_t)((Csr*)h)->indices.size(); }
void sdtgen_csr_copy(void* h, int64_t* indptr, int32_t* indices) {
  Csr* g = (Csr*)h;
  std::memcpy(indptr, g->indptr.data(), sizeof(int64_t) * g->indptr.size());
  std::memcpy(indices, g->indices.data(), sizeof(int32_t) * g->indices.size());
}
void sdtgen_csr_free(void* h) { delete (Csr*)h; }

// N(0,1) values, element i of the flat array from counter (i/4) word pair.
void sdtgen_normal_f32(float* out, int64_t count, uint64_t seed, uint32_t stream) {
  const int64_t nq = (count + 3) / 4;
#pragma omp parallel for schedule(static)
  for (int64_t q = 0; q < nq; ++q) {
    R4 r = philox((uint32_t)q, (uint32_t)(q >> 32), (DOM_FEAT << 16) | (stream & 0xFFFFu), 0, seed);
    float z[4];
    box_muller(r.w[0], r.w[1], &z[0], &z[1]);
    box_muller(r.w[2], r.w[3], &z[2], &z[3]);
    for (int k = 0; k < 4 && q * 4 + k < count; ++k) out[q * 4 + k] = z[k];
  }
}

// Same draws, stored as bf16 (round to nearest even of the fp32 value).
void sdtgen_normal_bf16(uint16_t* out, int64_t count, uint64_t seed, uint32_t stream) {
  const int64_t nq = (count + 3) / 4;
#pragma omp parallel for schedule(static)
  for (int64_t q = 0; q < nq; ++q) {
    R4 r = philox((uint32_t)q, (uint32_t)(q >> 32), (DOM_FEAT << 16) | (stream & 0xFFFFu), 0, seed);
    float z[4];
    box_muller(r.w[0], r.w[1], &z[0], &z[1]);
    box_muller(r.w[2], r.w[3], &z[2], &z[3]);
    for (int k = 0; k < 4 && q * 4 + k < count; ++k) out[q * 4 + k] = f32_to_bf16_rne(z[k]);
  }
}

void sdtgen_labels(int32_t* out, int64_t n, int32_t n_classes, uint64_t seed) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    R4 r = philox((uint32_t)i, (uint32_t)(i >> 32), DOM_LABEL << 16, 0, seed);
    out[i] = (int32_t)mulhi_range(r.w[0], (uint32_t)n_classes);
  }
}

// U(-lim, lim) values (Glorot: lim = sqrt(6/(fan_in+fan_out)) chosen by the caller).
void sdtgen_uniform_f32(float* out, int64_t count, float lim, uint64_t seed, uint32_t stream) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) {
    R4 r = philox((uint32_t)i, (uint32_t)(i >> 32), (DOM_WEIGHT << 16) | (stream & 0xFFFFu), 0, seed);
    double u = ((double)r.w[0] + 0.5) * (1.0 / 4294967296.0);
    out[i] = (float)((2.0 * u - 1.0) * (double)lim);
  }
}

// `batch` distinct node ids drawn uniformly from [lo, hi) for mini-batch `step`.
int32_t sdtgen_seed_batch(int32_t* out, int32_t batch, int32_t lo, int32_t hi, uint64_t seed, uint32_t step) {
  const int64_t range = (int64_t)hi - lo;
  if (batch < 0 || range < batch) return -1;
  std::unordered_map<int64_t, int64_t> moved;
  for (int32_t i = 0; i < batch; ++i) {
    R4 r = philox((uint32_t)i, 0, DOM_BATCH << 16, step, seed);
    int64_t j = i + (int64_t)(((uint64_t)r.w[0] * (uint64_t)(range - i)) >> 32);
    auto itj = moved.find(j);
    int64_t vj = itj == moved.end() ? j : itj->second;
    auto iti = moved.find(i);
    int64_t vi = iti == moved.end() ? i : iti->second;
    moved[j] = vi;
    out[i] = (int32_t)(lo + vj);
  }
  return 0;
}

}  // extern "C"
