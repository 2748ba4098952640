// Fan-out neighbour sampling over a CSR partition and construction of the
// sampled block (frontier, local column ids, transposed block) on gfx950.
//
// A group of 16, 32 or 64 lanes (the smallest that holds the fan-out) samples
// one destination row, so a wavefront works on up to four rows at once: lane i
// of a group owns Fisher-Yates step i (its Philox word, its swap target); the k
// dependent swaps are resolved with k rounds of in-group broadcasts instead of
// a per-row array.  Frontier de-duplication is direct addressing: a sampled
// edge stores one byte at its node ("reached by this layer"; a plain store, no
// atomic, nothing read), and the frontier scan folds those bytes into two bits
// per node ("in the frontier", "added by the last layer").  Popcount prefix sums
// over the scan's words yield the new nodes
// in ascending id order for free and, kept per word, give every new node's
// local id by rank, so the dense node -> local-id map is written and read only
// for nodes that were in the frontier before the layer.  Nothing depends on the
// order in which waves run, so every index output is reproducible bit for bit.
#include <atomic>
#include "common.h"

namespace sdt {

namespace {

constexpr int TB = 256;           // threads per block
constexpr int ITEMS = 8;          // scan items per thread
constexpr int TILE = TB * ITEMS;  // scan items per block
constexpr int SHORT_SEG = 32;     // transposed segments up to this length are sorted by one thread
constexpr int LDS_SEG = 8192;     // ... up to this length by one block in LDS

// ---- Philox4x32-10 (Salmon et al., SC'11) -------------------------------------
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                              uint32_t k1, uint32_t out[4]) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        uint32_t h0 = __umulhi(0xD2511F53u, c0), l0 = 0xD2511F53u * c0;
        uint32_t h1 = __umulhi(0xCD9E8D57u, c2), l1 = 0xCD9E8D57u * c2;
        c0 = h1 ^ c1 ^ k0;
        c1 = l1;
        c2 = h0 ^ c3 ^ k1;
        c3 = l0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

__global__ __launch_bounds__(TB) void k_fill_i32(int32_t* p, int64_t n, int32_t v) {
    int64_t i = (int64_t)blockIdx.x * TB + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * TB;
    for (; i < n; i += stride) p[i] = v;
}

// ---- frontier state ----------------------------------------------------------------
// mark[g] (one byte per node): 1 if the layer being sampled reached node g, whether it was in the frontier
// already or not; written by the sampling kernel, read and cleared by the frontier scan.
// bits (two bits per node, sixteen nodes per word), written by the frontier scan only: bit 2k of word w says
// node 16 w + k is in the frontier (F), bit 2k + 1 that the last layer sampled added it (M, a subset of F).
constexpr uint32_t F_PLANE = 0x55555555u, M_PLANE = 0xAAAAAAAAu;
// the sixteen mark bytes of a word's nodes (each 0 or 1) as bits 2k
__device__ __forceinline__ uint32_t marked_nodes(const uint8_t* __restrict__ mark, int word) {
    const uint4 v = *reinterpret_cast<const uint4*>(mark + (int64_t)word * 16);
    const uint32_t d[4] = {v.x, v.y, v.z, v.w};
    uint32_t x = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q)
        x |= ((d[q] & 1u) | ((d[q] >> 6) & 4u) | ((d[q] >> 12) & 16u) | ((d[q] >> 18) & 64u)) << (8 * q);
    return x;
}
// nodes reached by this layer that were not in the frontier before it, as bits 2k
__device__ __forceinline__ uint32_t new_nodes(uint32_t marked, uint32_t w) { return marked & ~w & F_PLANE; }

// G lanes per destination row (G = 16, 32 or 64 >= fan-out), 64 / G rows per wavefront and round, RU
// rounds in flight at once (the row offsets, neighbour ids and state words of all of them are requested
// before any is used: a launch over many rows is bound by how many such dependent round trips it
// overlaps, not by their number).
//
// The k dependent swaps of a row's shuffle are resolved without a k-long chain of broadcasts.  Step i
// takes the content of position j_i, which is j_i itself unless an earlier step t wrote there (j_t = j_i:
// then it is what position t held before step t).  What position i holds before step i is i unless some
// earlier step t swapped into it (j_t = i), in which case it is what position t held before step t: a
// chain i -> last such t -> ... that ends at an untouched position, whose index is the answer.  Every
// lane finds its two "last earlier t" with k independent broadcasts of j, and the chains are followed by
// pointer doubling in log2(G) rounds.
template <int G, int RU>
__global__ __launch_bounds__(TB) void k_sample_rows(const int64_t* __restrict__ indptr,
                                                    const int32_t* __restrict__ indices,
                                                    const int32_t* __restrict__ dst_nodes, int n_cap,
                                                    const int32_t* n_d, int fanout, uint32_t k0, uint32_t k1,
                                                    uint32_t step, uint32_t layer, uint8_t* __restrict__ mark,
                                                    int32_t* __restrict__ e_pad, int32_t* __restrict__ m_out) {
    constexpr int RPW = WAVE / G;
    constexpr int LG = G == 16 ? 4 : G == 32 ? 5 : 6;
    const int n = dev_count(n_cap, n_d);
    const int lane = threadIdx.x & (WAVE - 1);
    const int sub = lane / G, sl = lane % G, gbase = sub * G;
    const int wave = (blockIdx.x * TB + threadIdx.x) / WAVE;
    const int nwaves = gridDim.x * TB / WAVE;
    for (int i0 = wave * (RPW * RU); i0 < n; i0 += nwaves * (RPW * RU)) {
        int i[RU], v[RU];
        bool ok[RU];
#pragma unroll
        for (int r = 0; r < RU; ++r) {
            i[r] = i0 + r * RPW + sub;
            ok[r] = i[r] < n;
            v[r] = ok[r] ? dst_nodes[i[r]] : 0;
        }
        int64_t start[RU];
        uint32_t d[RU];
#pragma unroll
        for (int r = 0; r < RU; ++r) {
            start[r] = indptr[v[r]];
            const int64_t end = indptr[v[r] + 1];
            d[r] = ok[r] ? (uint32_t)(end - start[r]) : 0u;
        }
        uint32_t pos[RU];
        int rank[RU];
#pragma unroll
        for (int r = 0; r < RU; ++r) {
            pos[r] = sl;
            rank[r] = sl;
            const bool shuffle = d[r] > (uint32_t)fanout;
            if (__any(shuffle)) {   // wave-uniform: every lane takes part in the broadcasts, rows that need none drop the result
                uint32_t w[4];
                philox4x32_10((uint32_t)sl >> 2, (uint32_t)v[r], layer, step, k0, k1, w);
                // step `sl` of the shuffle swaps position sl with position j
                const uint32_t j = (uint32_t)sl + __umulhi(w[sl & 3], d[r] - (uint32_t)sl);
                int prev = -1, tlast = -1;   // the last earlier step that wrote to position sl / to position j
#pragma unroll
                for (int t = 0; t < G; ++t) {
                    if (t < fanout) {
                        const uint32_t jt = (uint32_t)__shfl((int)j, gbase + t);
                        if (t < sl) {
                            if (jt == (uint32_t)sl) prev = t;
                            if (jt == j) tlast = t;
                        }
                    }
                }
                int ptr = prev >= 0 ? prev : sl;
#pragma unroll
                for (int q = 0; q < LG; ++q) ptr = __shfl(ptr, gbase + ptr);
                // ptr: what position sl holds just before step sl
                const int moved = __shfl(ptr, gbase + (tlast >= 0 ? tlast : sl));
                const uint32_t cur = tlast >= 0 ? (uint32_t)moved : j;   // what position j holds just before step sl
                int rk = 0;
#pragma unroll
                for (int t = 0; t < G; ++t) {
                    if (t < fanout) {
                        const uint32_t pt = (uint32_t)__shfl((int)cur, gbase + t);
                        rk += (pt < cur) ? 1 : 0;
                    }
                }
                if (shuffle) { pos[r] = cur; rank[r] = rk; }
            }
        }
        int g[RU];
        bool act[RU];
#pragma unroll
        for (int r = 0; r < RU; ++r) {
            const int m = d[r] < (uint32_t)fanout ? (int)d[r] : fanout;
            act[r] = ok[r] && sl < m;
            g[r] = act[r] ? indices[start[r] + pos[r]] : 0;
            if (ok[r] && sl == 0) m_out[i[r]] = m;
        }
#pragma unroll
        for (int r = 0; r < RU; ++r) {
            if (!act[r]) continue;
            e_pad[(int64_t)i[r] * fanout + rank[r]] = g[r];
            // Mark the node, whatever its state, with a plain byte store: idempotent, nothing to wait for and
            // nothing read.  (Measured alternatives on one bit per node: an atomic OR per edge serialises on the
            // words of the hubs -- the sampling kernel of the large launch 122 us -- and looking at the word
            // first, to skip what is marked already, doubles the kernel on the dense workload, where the loads
            // hit lines that other workgroups are updating atomically.)  Marks on frontier nodes are dropped by
            // k_front_apply.
            mark[g[r]] = 1;
        }
    }
}

// ---- block-level exclusive scan of ITEMS values per thread --------------------
__device__ __forceinline__ int wave_incl_scan(int x) {
    const int lane = threadIdx.x & (WAVE - 1);
#pragma unroll
    for (int o = 1; o < WAVE; o <<= 1) {
        int y = __shfl_up(x, o);
        if (lane >= o) x += y;
    }
    return x;
}

// Returns the exclusive prefix of `sum` over the block's NT threads; *total = block sum.
template <int NT = TB>
__device__ __forceinline__ int block_excl_scan(int sum, int* total) {
    __shared__ int wsum[NT / WAVE];
    const int lane = threadIdx.x & (WAVE - 1), w = threadIdx.x / WAVE;
    const int incl = wave_incl_scan(sum);
    __syncthreads();
    if (lane == WAVE - 1) wsum[w] = incl;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int q = 0; q < NT / WAVE; ++q) {
        if (q < w) base += wsum[q];
        tot += wsum[q];
    }
    *total = tot;
    return base + incl - sum;
}

constexpr int WPT = 2;             // state words per thread in the frontier scans (32 nodes)
constexpr int TILE_B = TB * WPT;   // state words per block

// Pass 1 of the fused scans: blocks [0, pm) sum tiles of m[], blocks [pm, pm+pb)
// count the new nodes in tiles of state words.
__global__ __launch_bounds__(TB) void k_front_partials(const int32_t* __restrict__ m, int n_cap, const int32_t* n_d,
                                                       const uint32_t* __restrict__ bits,
                                                       const uint8_t* __restrict__ mark, int nwords, int pm,
                                                       int32_t* part) {
    int sum = 0;
    if ((int)blockIdx.x < pm) {
        const int n = dev_count(n_cap, n_d);
        const int base = blockIdx.x * TILE + threadIdx.x * ITEMS;
#pragma unroll
        for (int q = 0; q < ITEMS; ++q)
            if (base + q < n) sum += m[base + q];
    } else {
        const int base = (blockIdx.x - pm) * TILE_B + threadIdx.x * WPT;
#pragma unroll
        for (int q = 0; q < WPT; ++q)
            if (base + q < nwords) sum += __popc(new_nodes(marked_nodes(mark, base + q), bits[base + q]));
    }
    int total;
    block_excl_scan(sum, &total);
    if (threadIdx.x == 0) part[blockIdx.x] = total;
}

// Sums of three ranges of part[] by the whole block: [0,pm), [pm,pm+pb) and [lo,my).
__device__ __forceinline__ void part_sums(const int32_t* __restrict__ part, int pm, int pb, int lo, int my, int* nnz,
                                          int* n_new, int* before) {
    __shared__ int red[3][TB / WAVE];
    int a = 0, b = 0, c = 0;
    for (int i = threadIdx.x; i < pm + pb; i += TB) {
        const int v = part[i];
        if (i < pm) a += v; else b += v;
        if (i >= lo && i < my) c += v;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        a += __shfl_xor(a, o);
        b += __shfl_xor(b, o);
        c += __shfl_xor(c, o);
    }
    const int lane = threadIdx.x & (WAVE - 1), w = threadIdx.x / WAVE;
    if (lane == 0) { red[0][w] = a; red[1][w] = b; red[2][w] = c; }
    __syncthreads();
    a = b = c = 0;
#pragma unroll
    for (int q = 0; q < TB / WAVE; ++q) { a += red[0][q]; b += red[1][q]; c += red[2][q]; }
    *nnz = a; *n_new = b; *before = c;
}

// Pass 2 (every block first sums the few partials it needs, so no separate spine launch):
// write b_indptr and the block's counts; emit the new frontier nodes (ascending id); add them to the
// frontier plane of the state words and make them the "added by the last layer" plane; clear the mark
// bytes; leave each word's first new local id in wp[] for the relabelling; zero the histogram of the
// transposed block.  map (nullable): also record the new nodes' local ids there -- needed only when a
// further layer will be sampled from this frontier, for which these nodes are "in the frontier before".
__global__ __launch_bounds__(TB) void k_front_apply(const int32_t* __restrict__ m, int n_cap, const int32_t* n_d,
                                                    uint32_t* bits, uint8_t* mark, int nwords, int pm, int pb,
                                                    const int32_t* __restrict__ part, int32_t* counts,
                                                    int32_t* __restrict__ b_indptr, int32_t* __restrict__ src_nodes,
                                                    const int32_t* __restrict__ dst_nodes, int32_t* map,
                                                    int32_t* __restrict__ wp, int32_t* hist) {
    const int n = dev_count(n_cap, n_d);
    const bool is_m = (int)blockIdx.x < pm;
    int nnz, n_new, before;
    part_sums(part, pm, pb, is_m ? 0 : pm, blockIdx.x, &nnz, &n_new, &before);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        counts[0] = n;
        counts[1] = n + n_new;
        counts[2] = nnz;
        counts[3] = 0;
        b_indptr[n] = nnz;
    }
    if (is_m) {
        const int base = blockIdx.x * TILE + threadIdx.x * ITEMS;
        int v[ITEMS], sum = 0;
#pragma unroll
        for (int q = 0; q < ITEMS; ++q) {
            v[q] = (base + q < n) ? m[base + q] : 0;
            sum += v[q];
        }
        int total;
        int run = block_excl_scan(sum, &total) + before;
#pragma unroll
        for (int q = 0; q < ITEMS; ++q) {
            if (base + q < n) {
                b_indptr[base + q] = run;
                src_nodes[base + q] = dst_nodes[base + q];  // destination prefix of the frontier
            }
            run += v[q];
        }
    } else {
        const int base = (blockIdx.x - pm) * TILE_B + threadIdx.x * WPT;
        uint32_t wd[WPT], nw[WPT];
        int sum = 0;
#pragma unroll
        for (int q = 0; q < WPT; ++q) {
            wd[q] = 0u;
            nw[q] = 0u;
            if (base + q < nwords) {
                const uint32_t mk = marked_nodes(mark, base + q);
                wd[q] = bits[base + q];
                nw[q] = new_nodes(mk, wd[q]);
                if (mk) *reinterpret_cast<uint4*>(mark + (int64_t)(base + q) * 16) = make_uint4(0u, 0u, 0u, 0u);   // the marks are spent
            }
            sum += __popc(nw[q]);
        }
        int total;
        int run = n + before + block_excl_scan(sum, &total);
#pragma unroll
        for (int q = 0; q < WPT; ++q) {
            uint32_t x = nw[q];
            const uint32_t upd = (wd[q] & F_PLANE) | x | (x << 1);   // frontier += new; "added by the last layer" = new
            if (upd != wd[q]) bits[base + q] = upd;
            if (x) wp[base + q] = run;
            while (x) {
                const int b = __ffs(x) - 1;
                x &= x - 1;
                const int g = (base + q) * 16 + (b >> 1);
                src_nodes[run] = g;
                if (map) map[g] = run;
                ++run;
            }
        }
    }
    if (hist) {
        const int n_src = n + n_new;
        for (int j = blockIdx.x * TB + threadIdx.x; j <= n_src; j += gridDim.x * TB) hist[j] = 0;
    }
}

// cols[e] = local id of the sampled neighbour; optionally count the uses of each source.  A node this
// layer added has its mark set: its local id is its word's first new id plus the number of marked nodes
// below it in the word (two small arrays that stay in the caches); any other sampled node was in the
// frontier before and has its id in the map.
// G lanes per destination row, as in the sampling kernel: lane t of a group handles the row's t-th sampled
// edge; RU rows per group are in flight at once (each edge is a chain of three dependent loads).
template <int G, int RU>
__global__ __launch_bounds__(TB) void k_relabel(const int32_t* __restrict__ e_pad, const int32_t* __restrict__ m,
                                                const int32_t* __restrict__ b_indptr, int n_cap, const int32_t* n_d,
                                                int fanout, const uint32_t* __restrict__ bits,
                                                const int32_t* __restrict__ wp, const int32_t* __restrict__ map,
                                                const int32_t* __restrict__ counts, int32_t* __restrict__ cols,
                                                int32_t* hist) {
    const int n = dev_count(n_cap, n_d);
    const uint32_t n_src = (uint32_t)counts[1];
    const int t = threadIdx.x % G;
    constexpr int GROUPS = TB / G;
    for (int i0 = (blockIdx.x * GROUPS + threadIdx.x / G) * RU; i0 < n; i0 += gridDim.x * GROUPS * RU) {
        bool act[RU];
        int g[RU], at[RU];
#pragma unroll
        for (int r = 0; r < RU; ++r) act[r] = i0 + r < n && t < m[i0 + r];
#pragma unroll
        for (int r = 0; r < RU; ++r) {
            g[r] = act[r] ? e_pad[(int64_t)(i0 + r) * fanout + t] : 0;
            at[r] = act[r] ? b_indptr[i0 + r] + t : 0;
        }
        uint32_t w[RU];
#pragma unroll
        for (int r = 0; r < RU; ++r) w[r] = act[r] ? bits[g[r] >> 4] : 0u;
        int c[RU];
#pragma unroll
        for (int r = 0; r < RU; ++r) {
            const int sh = (g[r] & 15) * 2;
            const bool added = (w[r] >> (sh + 1)) & 1u;
            c[r] = !act[r] ? 0 : added ? wp[g[r] >> 4] + __popc(w[r] & M_PLANE & ((1u << sh) - 1u)) : map[g[r]];
        }
#pragma unroll
        for (int r = 0; r < RU; ++r) {
            if (!act[r]) continue;
            // always a row of the frontier -- unless someone wrote over the step's state while it ran; even
            // then the kernels that consume the block stay inside their buffers
            if ((uint32_t)c[r] >= n_src) c[r] = 0;
            cols[at[r]] = c[r];
            if (hist) atomicAdd(&hist[c[r]], 1);
        }
    }
}

// ---- two-pass exclusive scan: out[0..n] from in[0..n), n = *n_d + n_add ---------
__global__ __launch_bounds__(TB) void k_scan_partials(const int32_t* __restrict__ in, const int32_t* n_d, int n_add,
                                                      int32_t* part) {
    const int n = *n_d + n_add;
    const int base = blockIdx.x * TILE + threadIdx.x * ITEMS;
    int sum = 0;
#pragma unroll
    for (int q = 0; q < ITEMS; ++q)
        if (base + q < n) sum += in[base + q];
    int total;
    block_excl_scan(sum, &total);
    if (threadIdx.x == 0) part[blockIdx.x] = total;
}

// in-place capable (reads its tile fully before writing); each block sums the partials before it
__global__ __launch_bounds__(TB) void k_scan_apply(const int32_t* in, const int32_t* n_d, int n_add,
                                                   const int32_t* __restrict__ part, int32_t* out, int32_t* zero_me,
                                                   int32_t* long_count) {
    const int n = *n_d + n_add;
    int t0, t1, before;
    part_sums(part, gridDim.x, 0, 0, blockIdx.x, &t0, &t1, &before);
    if (blockIdx.x == 0 && threadIdx.x == 0 && long_count) *long_count = 0;
    const int base = blockIdx.x * TILE + threadIdx.x * ITEMS;
    int v[ITEMS], sum = 0;
#pragma unroll
    for (int q = 0; q < ITEMS; ++q) {
        v[q] = (base + q < n) ? in[base + q] : 0;
        sum += v[q];
    }
    int total;
    int run = block_excl_scan(sum, &total) + before;
#pragma unroll
    for (int q = 0; q < ITEMS; ++q) {
        if (base + q < n) {
            out[base + q] = run;
            if (zero_me) zero_me[base + q] = 0;
        }
        run += v[q];
    }
}

// t_rows filled in arbitrary order inside each segment (sorted afterwards).
__global__ __launch_bounds__(TB) void k_transpose_fill(const int32_t* __restrict__ b_indptr,
                                                       const int32_t* __restrict__ cols, int n_cap,
                                                       const int32_t* n_d, int fanout,
                                                       const int32_t* __restrict__ t_indptr, int32_t* cursor,
                                                       int32_t* __restrict__ t_rows) {
    const int n = dev_count(n_cap, n_d);
    const int64_t total = (int64_t)n * fanout;
    for (int64_t idx = (int64_t)blockIdx.x * TB + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * TB) {
        // total <= 2^31 - 1 (checked by the caller): a 32-bit division, several times cheaper than the 64-bit one
        const int i = (int)((uint32_t)idx / (uint32_t)fanout), t = (int)((uint32_t)idx - (uint32_t)i * (uint32_t)fanout);
        const int b0 = b_indptr[i];
        if (t < b_indptr[i + 1] - b0) {
            const int c = cols[b0 + t];
            const int slot = atomicAdd(&cursor[c], 1);
            t_rows[t_indptr[c] + slot] = i;
        }
    }
}

// Sort the short segment s[0, len), len <= N, ascending: all elements are loaded at once (padded with
// INT_MAX), sorted in registers by a bitonic network, and the first len written back.  An insertion sort
// in place pays a dependent global round trip per move, which made one thread's longest segment the
// longest thing in the launch.
template <int N>
__device__ __forceinline__ void sort_regs(int32_t* s, int len) {
    int v[N];
#pragma unroll
    for (int a = 0; a < N; ++a) v[a] = a < len ? s[a] : 0x7FFFFFFF;
#pragma unroll
    for (int k = 2; k <= N; k <<= 1)
#pragma unroll
        for (int j = k >> 1; j > 0; j >>= 1)
#pragma unroll
            for (int a = 0; a < N; ++a) {
                const int o = a ^ j;
                if (o > a) {
                    const int lo = min(v[a], v[o]), hi = max(v[a], v[o]);
                    const bool up = (a & k) == 0;
                    v[a] = up ? lo : hi;
                    v[o] = up ? hi : lo;
                }
            }
#pragma unroll
    for (int a = 0; a < N; ++a)
        if (a < len) s[a] = v[a];
}
__device__ __forceinline__ void sort_short_segment(int32_t* s, int len) {   // 2 <= len <= SHORT_SEG
    static_assert(SHORT_SEG == 32, "the widest network");
    if (len <= 4) sort_regs<4>(s, len);
    else if (len <= 8) sort_regs<8>(s, len);
    else if (len <= 16) sort_regs<16>(s, len);
    else sort_regs<32>(s, len);
}

// The whole block sorts t_rows[b, b+len) ascending; buf is >= LDS_SEG ints of LDS, tmp global scratch.
template <int NT>
__device__ void block_sort_segment(int32_t* t_rows, int b, int len, int32_t* buf, int32_t* tmp) {
    if (len <= LDS_SEG) {
        int p2 = 1;
        while (p2 < len) p2 <<= 1;
        for (int a = threadIdx.x; a < p2; a += NT) buf[a] = a < len ? t_rows[b + a] : 0x7FFFFFFF;
        __syncthreads();
        for (int k = 2; k <= p2; k <<= 1)
            for (int s = k >> 1; s > 0; s >>= 1) {
                for (int a = threadIdx.x; a < p2; a += NT) {
                    const int o = a ^ s;
                    if (o > a) {
                        const int x = buf[a], y = buf[o];
                        const bool up = (a & k) == 0;
                        if ((x > y) == up) { buf[a] = y; buf[o] = x; }
                    }
                }
                __syncthreads();
            }
        for (int a = threadIdx.x; a < len; a += NT) t_rows[b + a] = buf[a];
        __syncthreads();
    } else {
        // longer than the LDS buffer: place each element at its rank (quadratic, rare)
        for (int a = threadIdx.x; a < len; a += NT) tmp[b + a] = t_rows[b + a];
        __syncthreads();
        for (int a0 = 0; a0 < len; a0 += NT) {
            const int a = a0 + threadIdx.x;
            const int x = a < len ? tmp[b + a] : 0;
            int rank = 0;
            for (int c0 = 0; c0 < len; c0 += LDS_SEG) {
                const int cl = min(LDS_SEG, len - c0);
                __syncthreads();
                for (int c = threadIdx.x; c < cl; c += NT) buf[c] = tmp[b + c0 + c];
                __syncthreads();
                if (a < len)
                    for (int c = 0; c < cl; ++c) {
                        const int y = buf[c];
                        rank += (y < x || (y == x && c0 + c < a)) ? 1 : 0;
                    }
            }
            if (a < len) t_rows[b + rank] = x;
        }
        __syncthreads();
    }
}

// Each segment ascending: short ones by one thread, the rest queued for k_sort_long.
__global__ __launch_bounds__(TB) void k_sort_short(const int32_t* __restrict__ t_indptr, const int32_t* counts,
                                                   int32_t* t_rows, int32_t* long_count, int32_t* long_list) {
    const int n_src = counts[1];
    for (int j = blockIdx.x * TB + threadIdx.x; j < n_src; j += gridDim.x * TB) {
        const int b = t_indptr[j], len = t_indptr[j + 1] - b;
        if (len <= 1) continue;
        if (len > SHORT_SEG) {
            long_list[atomicAdd(long_count, 1)] = j;
            continue;
        }
        sort_short_segment(t_rows + b, len);
    }
}

__global__ __launch_bounds__(TB) void k_sort_long(const int32_t* __restrict__ t_indptr, int32_t* t_rows,
                                                  const int32_t* long_count, const int32_t* long_list,
                                                  int32_t* tmp) {
    __shared__ int32_t buf[LDS_SEG];
    const int cnt = *long_count;
    for (int li = blockIdx.x; li < cnt; li += gridDim.x) {
        const int j = long_list[li];
        const int b = t_indptr[j];
        block_sort_segment<TB>(t_rows, b, t_indptr[j + 1] - b, buf, tmp);
    }
}

constexpr int SMALL_T_NNZ = 1 << 14;  // layers up to this many sampled edges build their transposed block in one launch

// Transposed block of a small layer in one launch of TP_WG independent workgroups: workgroup p owns a
// contiguous range of the sources and needs nothing from the others.  It walks ALL of the layer's edges
// (a few tens of KB, served by the L2), keeps the ones whose column falls in its range in registers,
// counts the edges below its range (that is where its part of t_rows starts) and histograms its own in
// LDS; then scan, fill through LDS cursors, and every filled entry finds its final place by counting the
// smaller entries of its segment in LDS (ties: the earlier slot first) and its row is written there.  No column
// histogram from the relabelling pass, no global cursors, no sorting networks, and the chain of dependent
// global round trips (sizes, row offsets, column ids, write) is paid by 32 workgroups side by side
// instead of by one for the whole layer.  Segments longer than TP_RANK_MAX (a hub that most of the layer
// sampled) are written unsorted and sorted afterwards by the whole workgroup.
constexpr int TP_WG = 32;
constexpr int TP_NT = 1024;
constexpr int TP_FU = SMALL_T_NNZ / TP_NT;        // padded edge slots per thread
constexpr int TP_CHUNK = 1024;                    // sources per workgroup at most
constexpr int TP_MAX_SRC = TP_WG * TP_CHUNK;
constexpr int TP_RANK_MAX = 1024;                 // longest segment placed by counting
constexpr size_t TP_LDS_BYTES = (size_t)(2 * TP_CHUNK + 1 + SMALL_T_NNZ) * sizeof(int32_t) + SMALL_T_NNZ * sizeof(uint16_t);
static_assert(TP_CHUNK <= TP_NT && TP_CHUNK <= 1024 && SMALL_T_NNZ <= (1 << 21) && SMALL_T_NNZ >= LDS_SEG && SMALL_T_NNZ % TP_NT == 0,
              "one source per thread in the scan; (row, source) packed in 32 bits; sort buffer reuse");
__global__ __launch_bounds__(TP_NT) void k_transpose_parts(const int32_t* __restrict__ b_indptr,
                                                           const int32_t* __restrict__ cols, const int32_t* counts,
                                                           int fanout, int32_t* __restrict__ t_indptr,
                                                           int32_t* t_rows, int32_t* tmp) {
    extern __shared__ int32_t tp_lds[];
    int32_t* off = tp_lds;                   // [TP_CHUNK + 1] counts, then exclusive offsets of my segments
    int32_t* cur = tp_lds + TP_CHUNK + 1;    // [TP_CHUNK] fill cursors; the list of long segments afterwards
    int32_t* rows = cur + TP_CHUNK;          // [SMALL_T_NNZ] my edges' rows in fill order; the sort buffer of long segments afterwards
    uint16_t* seg = reinterpret_cast<uint16_t*>(rows + SMALL_T_NNZ);   // [SMALL_T_NNZ] the source (relative) of each of them
    __shared__ int red[TP_NT / WAVE];
    __shared__ int n_long;
    const int n_dst = counts[0], n_src = counts[1], nnz = counts[2];
    if (blockIdx.x == 0 && threadIdx.x == 0) t_indptr[n_src] = nnz;
    const int chunk = (n_src + TP_WG - 1) / TP_WG;
    const int j0 = blockIdx.x * chunk, j1 = min(n_src, j0 + chunk), nk = j1 - j0;
    if (nk <= 0) return;                     // the whole workgroup
    const int tid = threadIdx.x;
    if (tid == 0) n_long = 0;
    for (int k = tid; k <= nk; k += TP_NT) off[k] = 0;
    __syncthreads();
    // every edge of the layer; mine stay in registers as (row << 10 | source - j0)
    const int total = n_dst * fanout;
    int key[TP_FU], before = 0;
#pragma unroll
    for (int u = 0; u < TP_FU; ++u) {
        const int idx = tid + u * TP_NT;
        key[u] = -1;
        if (idx < total) {
            const int i = idx / fanout, t = idx - i * fanout;
            const int b0 = b_indptr[i];
            if (t < b_indptr[i + 1] - b0) {
                const int c = cols[b0 + t];
                if (c < j0) ++before;
                else if (c < j1) {
                    key[u] = (i << 10) | (c - j0);
                    atomicAdd(&off[c - j0 + 1], 1);
                }
            }
        }
    }
    // edges below my range: where my part of t_rows starts
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) before += __shfl_xor(before, o);
    if ((tid & (WAVE - 1)) == 0) red[tid / WAVE] = before;
    __syncthreads();
    int base = 0;
#pragma unroll
    for (int q = 0; q < TP_NT / WAVE; ++q) base += red[q];
    // counts -> exclusive offsets (one source per thread)
    const int h = tid < nk ? off[tid + 1] : 0;
    int mine;
    const int ex = block_excl_scan<TP_NT>(h, &mine);
    __syncthreads();
    if (tid < nk) { off[tid] = ex; cur[tid] = ex; }
    if (tid == 0) off[nk] = mine;
    __syncthreads();
#pragma unroll
    for (int u = 0; u < TP_FU; ++u)
        if (key[u] >= 0) {
            const int k = key[u] & 1023;
            const int slot = atomicAdd(&cur[k], 1);
            rows[slot] = key[u] >> 10;
            seg[slot] = (uint16_t)k;
        }
    __syncthreads();
    if (tid < nk) {
        t_indptr[j0 + tid] = base + ex;
        if (h > TP_RANK_MAX) cur[atomicAdd(&n_long, 1)] = tid;      // the cursors are spent: the list goes there
    }
    // final place of each of my edges: the number of entries of its segment that sort before it
    for (int e = tid; e < mine; e += TP_NT) {
        const int v = rows[e], k = seg[e], s0 = off[k], s1 = off[k + 1];
        int at = e;                          // a long segment: unsorted for now
        if (s1 - s0 <= TP_RANK_MAX) {
            at = s0;
            for (int q = s0; q < s1; ++q) {
                const int x = rows[q];
                at += (x < v || (x == v && q < e)) ? 1 : 0;
            }
        }
        t_rows[base + at] = v;
    }
    __syncthreads();
    // the few segments too long for that: the whole workgroup sorts each of them (rows[] is free again)
    const int cnt = n_long;
    for (int li = 0; li < cnt; ++li) {
        const int k = cur[li];
        block_sort_segment<TP_NT>(t_rows, base + off[k], off[k + 1] - off[k], rows, tmp);
    }
}

// ---- state shared by the layers of one step ------------------------------------------
// Every step starts by clearing the state words and the mark bytes (1.25 bytes per node: 21 MB for 2^24
// nodes) and leaves the former dirty; the node map needs no cleaning at all, because an entry is read only for a node
// whose frontier bit was set, and that bit is set by the kernel that wrote the entry in the same step.
// So a workspace carries nothing from one step to the next and its contents are never trusted.
__global__ __launch_bounds__(TB) void k_fill_u32(uint32_t* p, int64_t n, uint32_t v) {
    const int64_t stride = (int64_t)gridDim.x * TB;
    for (int64_t i = (int64_t)blockIdx.x * TB + threadIdx.x; i < n; i += stride) p[i] = v;
}

// map[dst[i]] = i and the destination joins the frontier.  Neighbouring lanes whose nodes share a state
// word (a sorted or contiguous destination list: sixteen in a row) combine their bits first and the last
// lane of the run issues one OR for all of them -- sixteen ORs on one word serialise in the L2.
__global__ __launch_bounds__(TB) void k_seed_map(int32_t* map, uint32_t* bits, const int32_t* __restrict__ dst, int n_cap,
                                                 const int32_t* n_d) {
    const int n = dev_count(n_cap, n_d);
    const int lane = threadIdx.x & (WAVE - 1);
    const int rounds = (n + gridDim.x * TB - 1) / (gridDim.x * TB);
    for (int q = 0; q < rounds; ++q) {   // whole wavefronts stay in the loop: the combining below uses every lane
        const int i = (q * gridDim.x + blockIdx.x) * TB + threadIdx.x;
        const bool ok = i < n;
        const int g = ok ? dst[i] : 0;
        if (ok) map[g] = i;
        const int word = ok ? (g >> 4) : -1 - lane;          // idle lanes: a word of their own
        uint32_t mask = ok ? 1u << ((g & 15) * 2) : 0u;
#pragma unroll
        for (int o = 1; o < WAVE; o <<= 1) {                 // OR over the run of equal words that ends at this lane
            const uint32_t m2 = (uint32_t)__shfl_up((int)mask, o);
            const int w2 = __shfl_up(word, o);
            if (lane >= o && w2 == word) mask |= m2;
        }
        const int next = __shfl_down(word, 1);
        if (ok && (lane == WAVE - 1 || next != word)) atomicOr(&bits[word], mask);
    }
}

inline int grid_for(int64_t items, int per_block, int max_blocks) {
    int64_t g = (items + per_block - 1) / per_block;
    if (g < 1) g = 1;
    if (g > max_blocks) g = max_blocks;
    return (int)g;
}

}  // namespace

static inline int64_t state_words(int64_t n_nodes) { return (n_nodes + 15) / 16; }

size_t sample_state_bytes(int64_t n_nodes) {
    return align_up((size_t)n_nodes * 4, 256) + 2 * align_up((size_t)state_words(n_nodes) * 4, 256) +
           align_up((size_t)state_words(n_nodes) * 16, 256);
}

void sample_state_carve(void* base, int64_t n_nodes, SampleWs* out) {
    Arena a(base);
    out->map = a.take<int32_t>(n_nodes);
    out->wp = a.take<int32_t>(state_words(n_nodes));
    out->bits = a.take<uint32_t>(state_words(n_nodes));
    out->mark = a.take<uint8_t>(state_words(n_nodes) * 16);   // right behind the state words: one fill clears both
}

size_t sample_tmp_carve(Arena& a, int64_t n_nodes, int32_t cap_dst, int32_t fanout, SampleWs* out) {
    const int64_t nwords = state_words(n_nodes);
    const int64_t cap_nnz = (int64_t)cap_dst * fanout;
    int64_t cap_src = (int64_t)cap_dst + cap_nnz;
    if (cap_src > n_nodes) cap_src = n_nodes;
    if (cap_src < cap_dst) cap_src = cap_dst;
    const int64_t pm = (cap_dst + TILE - 1) / TILE, pb = (nwords + TILE_B - 1) / TILE_B;
    const int64_t pt = (cap_src + 1 + TILE - 1) / TILE;
    SampleWs w = out ? *out : SampleWs{};
    w.e_pad = a.take<int32_t>(cap_nnz > 0 ? cap_nnz : 1);
    w.m = a.take<int32_t>(cap_dst > 0 ? cap_dst : 1);
    w.part = a.take<int32_t>((pm + pb > pt ? pm + pb : pt) + 1);
    w.cursor = a.take<int32_t>(cap_src + 1);
    w.longlist = a.take<int32_t>(cap_src + 2);
    if (out) *out = w;
    return a.off;
}

int32_t sample_state_clear(const SampleWs& ws, int64_t n_nodes, hipStream_t st) {
    const int64_t nwords = state_words(n_nodes);
    if (nwords == 0) return SDT_OK;
    // state words and mark bytes are contiguous (see sample_state_carve): words to clear, as 32-bit words
    const int64_t span = (int64_t)((reinterpret_cast<char*>(ws.mark) + nwords * 16) - reinterpret_cast<char*>(ws.bits)) / 4;
    hipLaunchKernelGGL(k_fill_u32, dim3(grid_for(span, TB * 4, 2048)), dim3(TB), 0, st, ws.bits, span, 0u);
    SDT_CHECK_LAUNCH("state clear");
    return SDT_OK;
}

int32_t sample_seed_map(const SampleWs& ws, const int32_t* dst_nodes, int32_t n_dst_cap, const int32_t* n_dst_d,
                        hipStream_t st) {
    hipLaunchKernelGGL(k_seed_map, dim3(grid_for(n_dst_cap, TB, 256)), dim3(TB), 0, st, ws.map, ws.bits, dst_nodes,
                       n_dst_cap, n_dst_d);
    SDT_CHECK_LAUNCH("seed map");
    return SDT_OK;
}

// Expects the frontier plane of ws.bits to hold exactly the destination nodes' frontier (with their ids in
// ws.map); leaves the new nodes added to it.  write_map: record the new nodes' ids in ws.map as well
// (needed when another layer will be sampled from the frontier this call produces).
int32_t sample_layer(const sdt_csr& g, const int32_t* dst_nodes, int32_t n_dst_cap, const int32_t* n_dst_d,
                     int32_t fanout, uint64_t seed, uint32_t step, uint32_t layer, const sdt_block& out,
                     const SampleWs& ws, bool write_map, hipStream_t st, sdt_timing* timing, int slot) {
    const int nwords = (int)state_words(g.n_nodes);
    const int pm = ceil_div(n_dst_cap > 0 ? n_dst_cap : 1, TILE), pb = ceil_div(nwords, TILE_B);
    const bool want_t = out.t_indptr != nullptr;
    const bool any = n_dst_cap > 0 && fanout > 0;
    // small layers build their transposed block in one launch that needs no column histogram
    const bool small_t = want_t && any && (int64_t)n_dst_cap * fanout <= SMALL_T_NNZ && out.cap_src <= TP_MAX_SRC;
    int32_t* hist = want_t && !small_t ? out.t_indptr : nullptr;  // counted in place, then scanned in place
    const int tl = (int)(layer < SDT_MAX_LAYERS ? layer : SDT_MAX_LAYERS - 1);   // timing slot of the layer

    if (any) {
        StageTimer tm(timing, slot, SDT_STAGE_SAMPLE_ROWS, tl, st);
        // the smallest lane group that holds the fan-out: up to four rows per wavefront and round; launches
        // over many rows keep four rounds in flight per wavefront, small ones spread over more wavefronts
#define SDT_SAMPLE_ROWS(G, RU)                                                                                            \
    hipLaunchKernelGGL((k_sample_rows<G, RU>), dim3(grid_for(n_dst_cap, (TB / WAVE) * (WAVE / G) * RU, 8192)), dim3(TB), 0, \
                       st, g.indptr, g.indices, dst_nodes, n_dst_cap, n_dst_d, fanout, (uint32_t)seed,                   \
                       (uint32_t)(seed >> 32), step, layer, ws.mark, ws.e_pad, ws.m)
        const bool many = n_dst_cap >= (1 << 16);
        if (fanout <= 16) { if (many) SDT_SAMPLE_ROWS(16, 4); else SDT_SAMPLE_ROWS(16, 1); }
        else if (fanout <= 32) { if (many) SDT_SAMPLE_ROWS(32, 4); else SDT_SAMPLE_ROWS(32, 1); }
        else { if (many) SDT_SAMPLE_ROWS(64, 4); else SDT_SAMPLE_ROWS(64, 1); }
#undef SDT_SAMPLE_ROWS
        SDT_CHECK_LAUNCH("sample rows");
    } else if (n_dst_cap > 0) {
        hipLaunchKernelGGL(k_fill_i32, dim3(grid_for(n_dst_cap, TB, 1024)), dim3(TB), 0, st, ws.m,
                           (int64_t)n_dst_cap, 0);
        SDT_CHECK_LAUNCH("zero m");
    }
    {
        StageTimer tm(timing, slot, SDT_STAGE_FRONT_SCAN, tl, st);
        hipLaunchKernelGGL(k_front_partials, dim3(pm + pb), dim3(TB), 0, st, ws.m, n_dst_cap, n_dst_d, ws.bits, ws.mark,
                           nwords, pm, ws.part);
        SDT_CHECK_LAUNCH("frontier partials");
    }
    {
        StageTimer tm(timing, slot, SDT_STAGE_FRONT_APPLY, tl, st);
        hipLaunchKernelGGL(k_front_apply, dim3(pm + pb), dim3(TB), 0, st, ws.m, n_dst_cap, n_dst_d, ws.bits, ws.mark, nwords,
                           pm, pb, ws.part, out.counts, out.indptr, out.src_nodes, dst_nodes, write_map ? ws.map : nullptr,
                           ws.wp, hist);
        SDT_CHECK_LAUNCH("frontier apply");
    }
    if (any) {
        StageTimer tm(timing, slot, SDT_STAGE_RELABEL, tl, st);
#define SDT_RELABEL(G, RU)                                                                                            \
    hipLaunchKernelGGL((k_relabel<G, RU>), dim3(grid_for(n_dst_cap, (TB / G) * RU, 1 << 16)), dim3(TB), 0, st, ws.e_pad, \
                       ws.m, out.indptr, n_dst_cap, n_dst_d, fanout, ws.bits, ws.wp, ws.map, out.counts, out.cols, hist)
        const bool many_rows = n_dst_cap >= (1 << 16);
        if (fanout <= 16) { if (many_rows) SDT_RELABEL(16, 4); else SDT_RELABEL(16, 1); }
        else if (fanout <= 32) { if (many_rows) SDT_RELABEL(32, 4); else SDT_RELABEL(32, 1); }
        else { if (many_rows) SDT_RELABEL(64, 4); else SDT_RELABEL(64, 1); }
#undef SDT_RELABEL
        SDT_CHECK_LAUNCH("relabel");
    }
    if (!want_t) return SDT_OK;
    StageTimer tt(timing, slot, SDT_STAGE_TRANSPOSE, tl, st);
    if (small_t) {
        // more than 64 KB of dynamic LDS has to be opted into, once (the loop's helper threads may get here together:
        // setting the attribute twice is harmless, the flag itself must not be a data race)
        static std::atomic<bool> opted{false};
        if (!opted.load(std::memory_order_acquire)) {
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(&k_transpose_parts), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)TP_LDS_BYTES) != hipSuccess) {
                set_error("transposed block: cannot raise the dynamic LDS limit to %zu bytes", TP_LDS_BYTES);
                return SDT_ERR_HIP;
            }
            opted.store(true, std::memory_order_release);
        }
        hipLaunchKernelGGL(k_transpose_parts, dim3(TP_WG), dim3(TP_NT), TP_LDS_BYTES, st, out.indptr, out.cols, out.counts,
                           fanout, out.t_indptr, out.t_rows, ws.e_pad);
        SDT_CHECK_LAUNCH("transposed block (small)");
        return SDT_OK;
    }
    const int pt = ceil_div((int64_t)out.cap_src + 1, TILE);
    hipLaunchKernelGGL(k_scan_partials, dim3(pt), dim3(TB), 0, st, hist, out.counts + 1, 1, ws.part);
    SDT_CHECK_LAUNCH("transpose partials");
    hipLaunchKernelGGL(k_scan_apply, dim3(pt), dim3(TB), 0, st, hist, out.counts + 1, 1, ws.part, out.t_indptr,
                       ws.cursor, ws.longlist);
    SDT_CHECK_LAUNCH("transpose apply");
    hipLaunchKernelGGL(k_transpose_fill, dim3(grid_for((int64_t)n_dst_cap * fanout, TB, 2048)), dim3(TB), 0, st,
                       out.indptr, out.cols, n_dst_cap, n_dst_d, fanout, out.t_indptr, ws.cursor, out.t_rows);
    SDT_CHECK_LAUNCH("transpose fill");
    hipLaunchKernelGGL(k_sort_short, dim3(grid_for(out.cap_src, TB, 2048)), dim3(TB), 0, st, out.t_indptr, out.counts,
                       out.t_rows, ws.longlist, ws.longlist + 1);
    SDT_CHECK_LAUNCH("sort short");
    hipLaunchKernelGGL(k_sort_long, dim3(64), dim3(TB), 0, st, out.t_indptr, out.t_rows, ws.longlist, ws.longlist + 1,
                       ws.e_pad);
    SDT_CHECK_LAUNCH("sort long");
    return SDT_OK;
}

}  // namespace sdt

extern "C" size_t sdt_sample_workspace_bytes(int64_t n_nodes, int32_t cap_dst, int32_t fanout) {
    if (n_nodes < 0 || cap_dst < 0 || fanout < 0) return 0;
    sdt::Arena a(nullptr);
    return sdt::sample_state_bytes(n_nodes) + sdt::sample_tmp_carve(a, n_nodes, cap_dst, fanout, nullptr);
}

extern "C" int32_t sdt_sample_csr(const sdt_csr* graph, const int32_t* dst_nodes, int32_t n_dst_cap,
                                  const int32_t* n_dst_d, int32_t fanout, uint64_t seed, uint32_t step,
                                  uint32_t layer, const sdt_block* out, void* ws, size_t ws_bytes, void* stream) {
    using namespace sdt;
    SDT_REQUIRE(graph && out, SDT_ERR_INVALID_ARG, "sdt_sample_csr: null graph or block");
    SDT_REQUIRE(graph->n_nodes >= 0 && graph->n_nodes <= 0x7FFFFFFF, SDT_ERR_INVALID_ARG,
                "sdt_sample_csr: n_nodes %lld out of range", (long long)graph->n_nodes);
    SDT_REQUIRE(graph->indptr && (graph->indices || graph->n_nodes == 0), SDT_ERR_INVALID_ARG,
                "sdt_sample_csr: null CSR arrays");
    SDT_REQUIRE(n_dst_cap >= 0 && (dst_nodes || n_dst_cap == 0), SDT_ERR_INVALID_ARG,
                "sdt_sample_csr: bad destination list");
    SDT_REQUIRE(fanout >= 0 && fanout <= SDT_MAX_FANOUT, SDT_ERR_INVALID_ARG,
                "sdt_sample_csr: fanout %d outside [0, %d]", fanout, SDT_MAX_FANOUT);
    SDT_REQUIRE(layer < 65536u, SDT_ERR_INVALID_ARG, "sdt_sample_csr: layer %u too large", layer);
    const int64_t need_nnz = (int64_t)n_dst_cap * fanout;
    SDT_REQUIRE(need_nnz <= 0x7FFFFFFF, SDT_ERR_INVALID_ARG, "sdt_sample_csr: n_dst_cap*fanout overflows int32");
    int64_t need_src = (int64_t)n_dst_cap + need_nnz;
    if (need_src > graph->n_nodes) need_src = graph->n_nodes;
    if (need_src < n_dst_cap) need_src = n_dst_cap;
    SDT_REQUIRE(out->cap_dst >= n_dst_cap && out->cap_nnz >= need_nnz && out->cap_src >= need_src,
                SDT_ERR_INVALID_ARG, "sdt_sample_csr: block capacities (%d,%d,%d) below the bounds (%d,%lld,%lld)",
                out->cap_dst, out->cap_src, out->cap_nnz, n_dst_cap, (long long)need_src, (long long)need_nnz);
    SDT_REQUIRE(out->counts && out->indptr && out->src_nodes && (out->cols || need_nnz == 0), SDT_ERR_INVALID_ARG,
                "sdt_sample_csr: null block arrays");
    SDT_REQUIRE((out->t_indptr == nullptr) == (out->t_rows == nullptr), SDT_ERR_INVALID_ARG,
                "sdt_sample_csr: pass both transposed arrays or neither");
    const size_t need = sdt_sample_workspace_bytes(graph->n_nodes, n_dst_cap, fanout);
    SDT_REQUIRE(ws && ws_bytes >= need && aligned16(ws), SDT_ERR_WORKSPACE,
                "sdt_sample_csr: workspace of %zu bytes needed, %zu given", need, ws_bytes);
    hipStream_t st = static_cast<hipStream_t>(stream);
    SampleWs sw{};
    sample_state_carve(ws, graph->n_nodes, &sw);
    Arena a(static_cast<char*>(ws) + sample_state_bytes(graph->n_nodes));
    sample_tmp_carve(a, graph->n_nodes, n_dst_cap, fanout, &sw);
    int32_t rc = sample_state_clear(sw, graph->n_nodes, st);
    if (rc != SDT_OK) return rc;
    rc = sample_seed_map(sw, dst_nodes, n_dst_cap, n_dst_d, st);
    if (rc != SDT_OK) return rc;
    // The transposed scan sizes its grid from the capacity the workspace was carved for.
    sdt_block blk = *out;
    blk.cap_src = (int32_t)need_src;
    // one layer only: nobody will look the new nodes up in the map
    return sample_layer(*graph, dst_nodes, n_dst_cap, n_dst_d, fanout, seed, step, layer, blk, sw, /*write_map=*/false, st,
                        nullptr, -1);
}
