// Fan-out neighbour sampling over a CSR partition and construction of the
// sampled block (frontier, local column ids, transposed block) on gfx950.
//
// One wavefront samples one destination row: lane i owns Fisher-Yates step i
// (its Philox word, its swap target); the k dependent swaps are resolved with
// k rounds of cross-lane broadcasts instead of a per-row array.  Frontier
// de-duplication is direct addressing: a bitmap over the partition's nodes is
// marked with idempotent atomic ORs, scanned with popcount prefix sums (which
// yields the new nodes in ascending id order for free) and a dense
// node -> local-id map is extended.  Nothing depends on the order in which
// waves run, so every index output is reproducible bit for bit.
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

// One wave per destination row.
__global__ __launch_bounds__(TB) void k_sample_rows(const int64_t* __restrict__ indptr,
                                                    const int32_t* __restrict__ indices,
                                                    const int32_t* __restrict__ dst_nodes, int n_cap,
                                                    const int32_t* n_d, int fanout, uint32_t k0, uint32_t k1,
                                                    uint32_t step, uint32_t layer, const int32_t* __restrict__ map,
                                                    uint32_t* bitmap, int32_t* __restrict__ e_pad,
                                                    int32_t* __restrict__ m_out) {
    const int n = dev_count(n_cap, n_d);
    const int lane = threadIdx.x & (WAVE - 1);
    const int wave = (blockIdx.x * TB + threadIdx.x) / WAVE;
    const int nwaves = gridDim.x * TB / WAVE;
    for (int i = wave; i < n; i += nwaves) {
        const int v = dst_nodes[i];
        const int64_t start = indptr[v];
        const uint32_t d = (uint32_t)(indptr[v + 1] - start);
        const int m = d < (uint32_t)fanout ? (int)d : fanout;
        uint32_t pos = lane;
        int rank = lane;
        if (d > (uint32_t)fanout) {
            uint32_t w[4];
            philox4x32_10((uint32_t)lane >> 2, (uint32_t)v, layer, step, k0, k1, w);
            const uint32_t r = w[lane & 3];
            // step `lane` of the shuffle swaps position lane with position j
            const uint32_t j = (uint32_t)lane + __umulhi(r, d - (uint32_t)lane);
            uint32_t cur = j;      // content of position j just before step `lane`
            uint32_t self = lane;  // content of position lane just before step `lane`
            for (int t = 0; t < fanout; ++t) {
                const uint32_t st = __builtin_amdgcn_readlane(self, t);
                const uint32_t jt = __builtin_amdgcn_readlane(j, t);
                if (lane > t) {
                    if (jt == j) cur = st;
                    if (jt == (uint32_t)lane) self = st;
                }
            }
            pos = cur;
            rank = 0;
            for (int t = 0; t < fanout; ++t) {
                const uint32_t pt = __builtin_amdgcn_readlane(pos, t);
                rank += (pt < pos) ? 1 : 0;
            }
        }
        if (lane < m) {
            const int g = indices[start + pos];
            e_pad[(int64_t)i * fanout + rank] = g;
            if (map[g] < 0) atomicOr(&bitmap[g >> 5], 1u << (g & 31));  // result unused: fire and forget
        }
        if (lane == 0) m_out[i] = m;
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

// Pass 1 of the fused scans: blocks [0, pm) sum tiles of m[], blocks [pm, pm+pb)
// sum popcounts of bitmap tiles.
__global__ __launch_bounds__(TB) void k_front_partials(const int32_t* __restrict__ m, int n_cap, const int32_t* n_d,
                                                       const uint32_t* __restrict__ bitmap, int nwords, int pm,
                                                       int32_t* part) {
    int sum = 0;
    if ((int)blockIdx.x < pm) {
        const int n = dev_count(n_cap, n_d);
        const int base = blockIdx.x * TILE + threadIdx.x * ITEMS;
#pragma unroll
        for (int q = 0; q < ITEMS; ++q)
            if (base + q < n) sum += m[base + q];
    } else {
        const int base = (blockIdx.x - pm) * TILE + threadIdx.x * ITEMS;
#pragma unroll
        for (int q = 0; q < ITEMS; ++q)
            if (base + q < nwords) sum += __popc(bitmap[base + q]);
    }
    int total;
    block_excl_scan(sum, &total);
    if (threadIdx.x == 0) part[blockIdx.x] = total;
}

// Sequential-by-chunks exclusive scan of `cnt` values by one block of NT threads
// (in place, or into `out`); returns the total.  `zero_me` (nullable) is cleared alongside.
template <int NT = TB>
__device__ int spine_scan(int32_t* p, int cnt, int32_t* zero_me = nullptr) {
    __shared__ int carry_s;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (int c0 = 0; c0 < cnt; c0 += NT) {
        const int idx = c0 + threadIdx.x;
        const int x = idx < cnt ? p[idx] : 0;
        if (zero_me && idx < cnt) zero_me[idx] = 0;
        int total;
        const int ex = block_excl_scan<NT>(x, &total);
        const int carry = carry_s;
        if (idx < cnt) p[idx] = carry + ex;
        __syncthreads();
        if (threadIdx.x == 0) carry_s = carry + total;
        __syncthreads();
    }
    return carry_s;
}

// The same exclusive scan for up to NT * SCAN_K entries in one round: a wave owns a contiguous range and
// reads it in SCAN_K coalesced slices at once (one memory round trip instead of one per NT entries),
// scans slice after slice in registers, and the waves' totals are combined through LDS.
constexpr int SCAN_K = 20;
// `copy` (nullable, LDS): also receives the first copy_n results (only on the one-round path: the caller
// asks for it only when cnt fits).
template <int NT>
__device__ int spine_scan_blocked(int32_t* p, int cnt, int32_t* zero_me = nullptr, int32_t* copy = nullptr,
                                  int copy_n = 0) {
    if (cnt > NT * SCAN_K) return spine_scan<NT>(p, cnt, zero_me);
    __shared__ int wtot[NT / WAVE];
    const int lane = threadIdx.x & (WAVE - 1), w = threadIdx.x / WAVE;
    constexpr int NW = NT / WAVE;
    const int K = ((cnt + NW - 1) / NW + WAVE - 1) / WAVE;      // slices per wave
    const int base = w * K * WAVE;
    int x[SCAN_K];
#pragma unroll
    for (int k = 0; k < SCAN_K; ++k) {
        const int idx = base + k * WAVE + lane;
        x[k] = (k < K && idx < cnt) ? p[idx] : 0;
    }
    if (zero_me) {
#pragma unroll
        for (int k = 0; k < SCAN_K; ++k) {
            const int idx = base + k * WAVE + lane;
            if (k < K && idx < cnt) zero_me[idx] = 0;
        }
    }
    int carry = 0;
#pragma unroll
    for (int k = 0; k < SCAN_K; ++k) {
        const int incl = wave_incl_scan(x[k]);
        const int tot = __shfl(incl, WAVE - 1);
        x[k] = carry + incl - x[k];
        carry += tot;
    }
    if (lane == 0) wtot[w] = carry;
    __syncthreads();
    int woff = 0, total = 0;
#pragma unroll
    for (int q = 0; q < NW; ++q) {
        if (q < w) woff += wtot[q];
        total += wtot[q];
    }
#pragma unroll
    for (int k = 0; k < SCAN_K; ++k) {
        const int idx = base + k * WAVE + lane;
        if (k < K && idx < cnt) {
            p[idx] = woff + x[k];
            if (copy && idx < copy_n) copy[idx] = woff + x[k];
        }
    }
    __syncthreads();
    return total;
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
// write b_indptr and the block's counts; emit the new frontier nodes (ascending id), extend
// the node -> local-id map, clear the bitmap; zero the histogram of the transposed block.
__global__ __launch_bounds__(TB) void k_front_apply(const int32_t* __restrict__ m, int n_cap, const int32_t* n_d,
                                                    uint32_t* bitmap, int nwords, int pm, int pb,
                                                    const int32_t* __restrict__ part, int32_t* counts,
                                                    int32_t* __restrict__ b_indptr, int32_t* __restrict__ src_nodes,
                                                    const int32_t* __restrict__ dst_nodes, int32_t* map,
                                                    int32_t* hist) {
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
        const int base = (blockIdx.x - pm) * TILE + threadIdx.x * ITEMS;
        uint32_t wd[ITEMS];
        int sum = 0;
#pragma unroll
        for (int q = 0; q < ITEMS; ++q) {
            wd[q] = (base + q < nwords) ? bitmap[base + q] : 0u;
            sum += __popc(wd[q]);
        }
        int total;
        int run = n + before + block_excl_scan(sum, &total);
#pragma unroll
        for (int q = 0; q < ITEMS; ++q) {
            uint32_t x = wd[q];
            if (x) bitmap[base + q] = 0u;
            while (x) {
                const int b = __ffs(x) - 1;
                x &= x - 1;
                const int g = (base + q) * 32 + b;
                src_nodes[run] = g;
                map[g] = run;
                ++run;
            }
        }
    }
    if (hist) {
        const int n_src = n + n_new;
        for (int j = blockIdx.x * TB + threadIdx.x; j <= n_src; j += gridDim.x * TB) hist[j] = 0;
    }
}

// cols[e] = local id of the sampled neighbour; optionally count the uses of each source.
__global__ __launch_bounds__(TB) void k_relabel(const int32_t* __restrict__ e_pad, const int32_t* __restrict__ m,
                                                const int32_t* __restrict__ b_indptr, int n_cap, const int32_t* n_d,
                                                int fanout, const int32_t* __restrict__ map,
                                                int32_t* __restrict__ cols, int32_t* hist) {
    const int n = dev_count(n_cap, n_d);
    const int64_t total = (int64_t)n * fanout;
    for (int64_t idx = (int64_t)blockIdx.x * TB + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * TB) {
        // total <= 2^31 - 1 (checked by the caller): a 32-bit division, several times cheaper than the 64-bit one
        const int i = (int)((uint32_t)idx / (uint32_t)fanout), t = (int)((uint32_t)idx - (uint32_t)i * (uint32_t)fanout);
        if (t < m[i]) {
            const int c = map[e_pad[idx]];
            cols[b_indptr[i] + t] = c;
            if (hist) atomicAdd(&hist[c], 1);
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

// Transposed block of a small layer in ONE launch of one 1024-thread workgroup:
// scan the per-source counts (left in t_indptr by k_relabel), fill, sort the segments.
// When the frontier fits (n_src <= TS_LDS) everything between the scan and the final copy stays in
// LDS: the scanned offsets double as fill cursors (a returning LDS atomic hands out the absolute slot,
// and after the fill cursor j has arrived at the end of segment j), the rows are filled and sorted
// there and written out once, coalesced.  One workgroup pays every global round trip in full, so the
// fewer there are in sequence the better: counts, histogram, row offsets, column ids, and the copy out.
// Otherwise: fill cursors in global memory, segments sorted in global memory.
constexpr int TS = 1024;
constexpr int TS_LDS = 12288;  // ints of LDS for offsets / cursors; the sort buffer of long segments afterwards
constexpr int SMALL_T_NNZ = 1 << 14;  // layers up to this many sampled edges use k_transpose_small
constexpr size_t TS_LDS_BYTES = (size_t)(TS_LDS + SMALL_T_NNZ) * sizeof(int32_t);
static_assert(TS_LDS >= LDS_SEG && SMALL_T_NNZ + TS <= TS * SCAN_K, "buffer reuse; one-round scan");
__global__ __launch_bounds__(TS) void k_transpose_small(const int32_t* __restrict__ b_indptr,
                                                        const int32_t* __restrict__ cols, const int32_t* counts,
                                                        int fanout, int32_t* t_indptr, int32_t* cursor_g,
                                                        int32_t* t_rows, int32_t* long_list, int32_t* tmp) {
    extern __shared__ int32_t ts_lds[];
    int32_t* cur = ts_lds;                 // [TS_LDS]
    int32_t* rows = ts_lds + TS_LDS;       // [SMALL_T_NNZ]
    __shared__ int n_long;
    const int n_dst = counts[0], n_src = counts[1];
    const bool in_lds = n_src <= TS_LDS;
    if (threadIdx.x == 0) n_long = 0;
    // counts -> offsets in place (and into cur)
    const int nnz = spine_scan_blocked<TS>(t_indptr, n_src + 1, in_lds ? nullptr : cursor_g, in_lds ? cur : nullptr, n_src);
    const int total = n_dst * fanout;
    constexpr int FU = 4;   // edges in flight per thread: each is a chain of dependent loads
    for (int i0 = threadIdx.x; i0 < total; i0 += TS * FU) {
        int row[FU], c[FU], dst[FU];
#pragma unroll
        for (int u = 0; u < FU; ++u) {
            const int idx = i0 + u * TS;
            row[u] = -1;
            if (idx < total) {
                const int i = idx / fanout, t = idx - i * fanout;
                const int b0 = b_indptr[i];
                if (t < b_indptr[i + 1] - b0) { row[u] = i; c[u] = b0 + t; }
            }
        }
#pragma unroll
        for (int u = 0; u < FU; ++u)
            if (row[u] >= 0) c[u] = cols[c[u]];
        if (in_lds) {
#pragma unroll
            for (int u = 0; u < FU; ++u)
                if (row[u] >= 0) rows[atomicAdd(&cur[c[u]], 1)] = row[u];
        } else {
#pragma unroll
            for (int u = 0; u < FU; ++u)
                if (row[u] >= 0) dst[u] = t_indptr[c[u]] + atomicAdd(&cursor_g[c[u]], 1);
#pragma unroll
            for (int u = 0; u < FU; ++u)
                if (row[u] >= 0) t_rows[dst[u]] = row[u];
        }
    }
    __syncthreads();
    if (in_lds) {
        for (int j = threadIdx.x; j < n_src; j += TS) {
            const int b = j ? cur[j - 1] : 0, len = cur[j] - b;     // cursor j stopped at the end of segment j
            if (len <= 1) continue;
            if (len > SHORT_SEG) long_list[atomicAdd(&n_long, 1)] = j;
            else sort_short_segment(rows + b, len);
        }
        __syncthreads();
        for (int e = threadIdx.x; e < nnz; e += TS) t_rows[e] = rows[e];
    } else {
        for (int j0 = threadIdx.x; j0 < n_src; j0 += TS * FU) {
            int b[FU], len[FU];
#pragma unroll
            for (int u = 0; u < FU; ++u) {
                const int j = j0 + u * TS;
                b[u] = 0;
                len[u] = 0;
                if (j < n_src) { b[u] = t_indptr[j]; len[u] = t_indptr[j + 1] - b[u]; }
            }
#pragma unroll 1
            for (int u = 0; u < FU; ++u) {   // one copy of the sorting networks: pick the u-th pair without indexing
                static_assert(FU == 4, "select chain");
                const int bu = u == 0 ? b[0] : u == 1 ? b[1] : u == 2 ? b[2] : b[3];
                const int lu = u == 0 ? len[0] : u == 1 ? len[1] : u == 2 ? len[2] : len[3];
                if (lu <= 1) continue;
                if (lu > SHORT_SEG) long_list[atomicAdd(&n_long, 1)] = j0 + u * TS;
                else sort_short_segment(t_rows + bu, lu);
            }
        }
    }
    __syncthreads();
    const int cnt = n_long;
    for (int li = 0; li < cnt; ++li) {
        const int j = long_list[li];
        const int b = t_indptr[j];
        block_sort_segment<TS>(t_rows, b, t_indptr[j + 1] - b, cur, tmp);
    }
}

// ---- state that persists across the layers (and steps) of a training run ---------
// Fill the node map with -1 and clear the bitmap unless the header says a previous step
// left them in that state already (every step restores them before it ends).
__global__ __launch_bounds__(TB) void k_state_check_init(const int32_t* header, int32_t* map, int64_t n,
                                                         uint32_t* bitmap, int64_t nwords) {
    if (header && header[0] == STATE_MAGIC && header[1] == (int32_t)n) return;
    const int64_t stride = (int64_t)gridDim.x * TB;
    for (int64_t i = (int64_t)blockIdx.x * TB + threadIdx.x; i < n; i += stride) map[i] = -1;
    for (int64_t i = (int64_t)blockIdx.x * TB + threadIdx.x; i < nwords; i += stride) bitmap[i] = 0u;
}

// map[dst[i]] = i.  From here on the map is in use: the header loses its magic word (after
// k_state_check_init has read it) until the step's last cleaning kernel stamps it again.
__global__ __launch_bounds__(TB) void k_seed_map(int32_t* map, const int32_t* __restrict__ dst, int n_cap,
                                                 const int32_t* n_d, int32_t* header, int32_t n_nodes) {
    const int n = dev_count(n_cap, n_d);
    for (int i = blockIdx.x * TB + threadIdx.x; i < n; i += gridDim.x * TB) map[dst[i]] = i;
    if (header && blockIdx.x == 0 && threadIdx.x == 0) {
        header[0] = 0;
        header[1] = n_nodes;
    }
}

inline int grid_for(int64_t items, int per_block, int max_blocks) {
    int64_t g = (items + per_block - 1) / per_block;
    if (g < 1) g = 1;
    if (g > max_blocks) g = max_blocks;
    return (int)g;
}

}  // namespace

size_t sample_state_bytes(int64_t n_nodes) {
    return align_up((size_t)n_nodes * 4, 256) + align_up((size_t)((n_nodes + 31) / 32) * 4, 256);
}

void sample_state_carve(void* base, int64_t n_nodes, SampleWs* out) {
    Arena a(base);
    out->map = a.take<int32_t>(n_nodes);
    out->bitmap = a.take<uint32_t>((n_nodes + 31) / 32);
}

size_t sample_tmp_carve(Arena& a, int64_t n_nodes, int32_t cap_dst, int32_t fanout, SampleWs* out) {
    const int64_t nwords = (n_nodes + 31) / 32;
    const int64_t cap_nnz = (int64_t)cap_dst * fanout;
    int64_t cap_src = (int64_t)cap_dst + cap_nnz;
    if (cap_src > n_nodes) cap_src = n_nodes;
    if (cap_src < cap_dst) cap_src = cap_dst;
    const int64_t pm = (cap_dst + TILE - 1) / TILE, pb = (nwords + TILE - 1) / TILE;
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

int32_t sample_state_init(const SampleWs& ws, int64_t n_nodes, const int32_t* header, hipStream_t st) {
    hipLaunchKernelGGL(k_state_check_init, dim3(grid_for(n_nodes, TB * 4, 2048)), dim3(TB), 0, st, header, ws.map,
                       n_nodes, ws.bitmap, (n_nodes + 31) / 32);
    SDT_CHECK_LAUNCH("state init");
    return SDT_OK;
}

int32_t sample_seed_map(const SampleWs& ws, const int32_t* dst_nodes, int32_t n_dst_cap, const int32_t* n_dst_d,
                        int32_t* header, int64_t n_nodes, hipStream_t st) {
    hipLaunchKernelGGL(k_seed_map, dim3(grid_for(n_dst_cap, TB, 256)), dim3(TB), 0, st, ws.map, dst_nodes, n_dst_cap,
                       n_dst_d, header, (int32_t)n_nodes);
    SDT_CHECK_LAUNCH("seed map");
    return SDT_OK;
}

// Expects ws.map to hold the destination nodes (and only frontier nodes) and ws.bitmap to be clear;
// leaves the map extended by the new frontier nodes and the bitmap clear again.
int32_t sample_layer(const sdt_csr& g, const int32_t* dst_nodes, int32_t n_dst_cap, const int32_t* n_dst_d,
                     int32_t fanout, uint64_t seed, uint32_t step, uint32_t layer, const sdt_block& out,
                     const SampleWs& ws, hipStream_t st, sdt_timing* timing, int slot) {
    const int nwords = (int)((g.n_nodes + 31) / 32);
    const int pm = ceil_div(n_dst_cap > 0 ? n_dst_cap : 1, TILE), pb = ceil_div(nwords, TILE);
    const bool want_t = out.t_indptr != nullptr;
    int32_t* hist = want_t ? out.t_indptr : nullptr;  // counted in place, then scanned in place
    const bool any = n_dst_cap > 0 && fanout > 0;
    const int tl = (int)(layer < SDT_MAX_LAYERS ? layer : SDT_MAX_LAYERS - 1);   // timing slot of the layer

    if (any) {
        StageTimer tm(timing, slot, SDT_STAGE_SAMPLE_ROWS, tl, st);
        hipLaunchKernelGGL(k_sample_rows, dim3(grid_for(n_dst_cap, TB / WAVE, 8192)), dim3(TB), 0, st, g.indptr,
                           g.indices, dst_nodes, n_dst_cap, n_dst_d, fanout, (uint32_t)seed,
                           (uint32_t)(seed >> 32), step, layer, ws.map, ws.bitmap, ws.e_pad, ws.m);
        SDT_CHECK_LAUNCH("sample rows");
    } else if (n_dst_cap > 0) {
        hipLaunchKernelGGL(k_fill_i32, dim3(grid_for(n_dst_cap, TB, 1024)), dim3(TB), 0, st, ws.m,
                           (int64_t)n_dst_cap, 0);
        SDT_CHECK_LAUNCH("zero m");
    }
    {
        StageTimer tm(timing, slot, SDT_STAGE_FRONT_SCAN, tl, st);
        hipLaunchKernelGGL(k_front_partials, dim3(pm + pb), dim3(TB), 0, st, ws.m, n_dst_cap, n_dst_d, ws.bitmap, nwords,
                           pm, ws.part);
        SDT_CHECK_LAUNCH("frontier partials");
    }
    {
        StageTimer tm(timing, slot, SDT_STAGE_FRONT_APPLY, tl, st);
        hipLaunchKernelGGL(k_front_apply, dim3(pm + pb), dim3(TB), 0, st, ws.m, n_dst_cap, n_dst_d, ws.bitmap, nwords, pm,
                           pb, ws.part, out.counts, out.indptr, out.src_nodes, dst_nodes, ws.map, hist);
        SDT_CHECK_LAUNCH("frontier apply");
    }
    if (any) {
        StageTimer tm(timing, slot, SDT_STAGE_RELABEL, tl, st);
        hipLaunchKernelGGL(k_relabel, dim3(grid_for((int64_t)n_dst_cap * fanout, TB, 2048)), dim3(TB), 0, st,
                           ws.e_pad, ws.m, out.indptr, n_dst_cap, n_dst_d, fanout, ws.map, out.cols, hist);
        SDT_CHECK_LAUNCH("relabel");
    }
    if (!want_t) return SDT_OK;
    StageTimer tt(timing, slot, SDT_STAGE_TRANSPOSE, tl, st);
    if ((int64_t)n_dst_cap * fanout <= SMALL_T_NNZ) {
        // more than 64 KB of dynamic LDS has to be opted into, once (the loop's helper threads may get here together:
        // setting the attribute twice is harmless, the flag itself must not be a data race)
        static std::atomic<bool> opted{false};
        if (!opted.load(std::memory_order_acquire)) {
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(&k_transpose_small), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)TS_LDS_BYTES) != hipSuccess) {
                set_error("transpose small: cannot raise the dynamic LDS limit to %zu bytes", TS_LDS_BYTES);
                return SDT_ERR_HIP;
            }
            opted.store(true, std::memory_order_release);
        }
        hipLaunchKernelGGL(k_transpose_small, dim3(1), dim3(TS), TS_LDS_BYTES, st, out.indptr, out.cols, out.counts, fanout,
                           out.t_indptr, ws.cursor, out.t_rows, ws.longlist, ws.e_pad);
        SDT_CHECK_LAUNCH("transpose small");
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
    int32_t rc = sample_state_init(sw, graph->n_nodes, nullptr, st);  // unconditional: ws contents are arbitrary
    if (rc != SDT_OK) return rc;
    rc = sample_seed_map(sw, dst_nodes, n_dst_cap, n_dst_d, nullptr, graph->n_nodes, st);
    if (rc != SDT_OK) return rc;
    // The transposed scan sizes its grid from the capacity the workspace was carved for.
    sdt_block blk = *out;
    blk.cap_src = (int32_t)need_src;
    return sample_layer(*graph, dst_nodes, n_dst_cap, n_dst_d, fanout, seed, step, layer, blk, sw, st);
}
