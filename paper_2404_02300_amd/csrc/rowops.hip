// Row-wise, bandwidth-bound stages on gfx950: feature gather, mean aggregation
// (sampled block or whole CSR) and its backward through the transposed block.
//
// A row of F elements is handled by a group of G lanes (G = 8..64, the smallest
// power of two that covers the row with one vector per lane, wider rows loop
// in chunks).  Every lane moves 16 bytes when the rows start on dword boundaries
// (gather and sampled-block aggregation; the last vector of a ragged row is moved
// back to end with the row), else the widest vector the alignment allows.  The edge loop issues a batch of
// independent row loads before consuming them, so each wave keeps several KB
// in flight; sums are taken in edge order in fp32, which makes the result
// independent of the launch shape.
#include "common.h"

#include <type_traits>

namespace sdt {
namespace {

constexpr int TB = 256;
constexpr int UNROLL = 8;  // row loads in flight per lane

// 16- and 8-byte accesses are declared with 4-byte alignment: global loads and stores of several
// dwords need dword alignment only on this hardware, so rows that start on any dword boundary
// (602 floats = 2408 bytes per row) still move 16 bytes per lane.
struct __attribute__((packed, aligned(4))) dword4 { uint32_t x, y, z, w; };
struct __attribute__((packed, aligned(4))) dword2 { uint32_t x, y; };
template <int BYTES> struct Raw;
template <> struct Raw<16> { using type = dword4; };
template <> struct Raw<8> { using type = dword2; };
template <> struct Raw<4> { using type = uint32_t; };
template <> struct Raw<2> { using type = uint16_t; };

template <typename T, int VE>
struct Vec {
    using raw_t = typename Raw<VE * sizeof(T)>::type;
    union {
        raw_t raw;
        T e[VE];
    };
    __device__ __forceinline__ Vec() {}
};

template <typename T, int VE>
__device__ __forceinline__ void load_f32(const T* p, float out[VE]) {
    Vec<T, VE> v;
    v.raw = *reinterpret_cast<const typename Vec<T, VE>::raw_t*>(p);
#pragma unroll
    for (int q = 0; q < VE; ++q) out[q] = to_f32<T>(v.e[q]);
}

template <typename T, int VE>
__device__ __forceinline__ void store_f32(T* p, const float in[VE]) {
    Vec<T, VE> v;
#pragma unroll
    for (int q = 0; q < VE; ++q) v.e[q] = from_f32<T>(in[q]);
    *reinterpret_cast<typename Vec<T, VE>::raw_t*>(p) = v.raw;
}

// ---- gather: out[j,:] = X[idx[j],:] -------------------------------------------
template <int VB, int G>
__global__ __launch_bounds__(TB) void k_gather(const char* __restrict__ X, int64_t ldx_b, int row_b,
                                               const int32_t* __restrict__ idx, int n_cap, const int32_t* n_d,
                                               char* __restrict__ out, int64_t ldo_b, int pad_b, char* __restrict__ pad2) {
    using raw_t = typename Raw<VB>::type;
    const int n = dev_count(n_cap, n_d);
    const int gl = threadIdx.x % G;
    const int64_t ngrp = (int64_t)gridDim.x * (TB / G);
    for (int64_t j = (int64_t)blockIdx.x * (TB / G) + threadIdx.x / G; j < n; j += ngrp) {
        const int node = idx[j];
        const char* src = X + (int64_t)node * ldx_b;
        char* dst = out + j * ldo_b;
        // the last vector of a row whose width is not a multiple of VB is moved back to end with the row
        // (it overlaps its neighbour and copies the same bytes again); row_b >= VB
        for (int bn = gl * VB; bn < row_b; bn += G * VB) {
            const int b = min(bn, row_b - VB);
            *reinterpret_cast<raw_t*>(dst + b) = *reinterpret_cast<const raw_t*>(src + b);
        }
        // zero padding of the output row (pad_b <= row_b: none), and of row j of a second matrix of
        // the same shape and stride whose producer writes the first row_b bytes only (pad2, nullable)
        constexpr int ZB = VB < 4 ? VB : 4;   // the padding is a whole number of elements, not of vectors
        using zero_t = typename Raw<ZB>::type;
        for (int b = row_b + gl * ZB; b < pad_b; b += G * ZB) {
            *reinterpret_cast<zero_t*>(dst + b) = zero_t{};
            if (pad2) *reinterpret_cast<zero_t*>(pad2 + j * ldo_b + b) = zero_t{};
        }
    }
}

// ---- mean aggregation forward ---------------------------------------------------
// row_ids (nullable): the source row of column c is H[row_ids[c]] instead of H[c] -- used to
// aggregate straight out of the partition's feature matrix through a block's src_nodes, so the
// gathered copy of the non-destination frontier rows is never written.
template <typename T, int VE, int G, typename IP>
__global__ __launch_bounds__(TB) void k_aggregate_fwd(const IP* __restrict__ indptr, const int32_t* __restrict__ cols,
                                                      int64_t n_cap, const int32_t* n_d, const T* __restrict__ H,
                                                      int64_t ldh, int F, T* __restrict__ A, int64_t lda,
                                                      const int32_t* __restrict__ row_ids,
                                                      int64_t skip_longer_than) {
    int64_t n = n_cap;
    if (n_d) n = *n_d < n_cap ? *n_d : n_cap;
    const int gl = threadIdx.x % G;
    const int64_t ngrp = (int64_t)gridDim.x * (TB / G);
    for (int64_t i = (int64_t)blockIdx.x * (TB / G) + threadIdx.x / G; i < n; i += ngrp) {
        const IP e0 = indptr[i], e1 = indptr[i + 1];
        if ((int64_t)(e1 - e0) > skip_longer_than) continue;  // left to k_aggregate_long
        const float m = (float)(e1 - e0);
        // the last vector of a row whose width is not a multiple of VE is moved back to end with the row:
        // it overlaps its neighbour, both lanes take the same sums in the same order and store the same values
        for (int fn = gl * VE; fn < F; fn += G * VE) {
            const int f0 = min(fn, F - VE);
            float acc[VE];
#pragma unroll
            for (int q = 0; q < VE; ++q) acc[q] = 0.f;
            for (IP e = e0; e < e1; e += UNROLL) {
                int c[UNROLL];
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) c[u] = (e + u < e1) ? cols[e + u] : -1;
                if (row_ids) {
#pragma unroll
                    for (int u = 0; u < UNROLL; ++u)
                        if (c[u] >= 0) c[u] = row_ids[c[u]];
                }
                // the rows stay in their storage type until they are added (half the registers for bf16)
                Vec<T, VE> v[UNROLL];
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) {
                    v[u].raw = typename Vec<T, VE>::raw_t{};
                    if (c[u] >= 0) v[u].raw = *reinterpret_cast<const typename Vec<T, VE>::raw_t*>(H + (int64_t)c[u] * ldh + f0);
                }
#pragma unroll
                for (int u = 0; u < UNROLL; ++u)
#pragma unroll
                    for (int q = 0; q < VE; ++q) acc[q] += to_f32<T>(v[u].e[q]);
            }
            if (e1 > e0) {
#pragma unroll
                for (int q = 0; q < VE; ++q) acc[q] = acc[q] / m;
            }
            store_f32<T, VE>(A + i * lda + f0, acc);
        }
    }
}

// The same for rows wider than one pass of the lane group (F > G * VE): the NP passes over the features run
// side by side, so a lane has NP * UNROLL row loads in flight instead of UNROLL and a launch needs a
// fraction of the wavefronts to keep the memory system busy.  Sums in edge order, as above: same bits.
// Dense workload (602 floats, NP = 3), layer-0 aggregation alone: 108 -> 98 us (6.5 TB/s of gather-side bytes).
//
// Inside a training loop this kernel runs on an auxiliary stream beside the projections of the step before.  While
// those were fp32 matrix kernels of four-wave workgroups, a launch capped at 1.5 workgroups per CU (streaming in
// the background, 155 us against 106) made the loop faster (dense 3 360 -> 3 890 steps/s); beside the split-bf16
// projections, whose single workgroup per CU needs only eight wave slots, the full launch is the faster one
// again (4 200 against 4 100 steps/s, the kernel 120 against 169 us inside the loop), so nothing is capped.
template <typename T, int VE, int G, int NP>
__global__ __launch_bounds__(TB) void k_aggregate_fwd_wide(const int32_t* __restrict__ indptr, const int32_t* __restrict__ cols,
                                                           int64_t n_cap, const int32_t* n_d, const T* __restrict__ H,
                                                           int64_t ldh, int F, T* __restrict__ A, int64_t lda,
                                                           const int32_t* __restrict__ row_ids) {
    int64_t n = n_cap;
    if (n_d) n = *n_d < n_cap ? *n_d : n_cap;
    const int gl = threadIdx.x % G;
    const int64_t ngrp = (int64_t)gridDim.x * (TB / G);
    int f0[NP];
    bool on[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int fn = gl * VE + p * G * VE;
        on[p] = fn < F;
        f0[p] = min(fn, F - VE);
    }
    for (int64_t i = (int64_t)blockIdx.x * (TB / G) + threadIdx.x / G; i < n; i += ngrp) {
        const int e0 = indptr[i], e1 = indptr[i + 1];
        const float m = (float)(e1 - e0);
        float acc[NP][VE];
#pragma unroll
        for (int p = 0; p < NP; ++p)
#pragma unroll
            for (int q = 0; q < VE; ++q) acc[p][q] = 0.f;
        for (int e = e0; e < e1; e += UNROLL) {
            int c[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) c[u] = (e + u < e1) ? cols[e + u] : -1;
            if (row_ids) {
#pragma unroll
                for (int u = 0; u < UNROLL; ++u)
                    if (c[u] >= 0) c[u] = row_ids[c[u]];
            }
            Vec<T, VE> v[NP][UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
#pragma unroll
                for (int p = 0; p < NP; ++p) {
                    v[p][u].raw = typename Vec<T, VE>::raw_t{};
                    if (c[u] >= 0 && on[p])
                        v[p][u].raw = *reinterpret_cast<const typename Vec<T, VE>::raw_t*>(H + (int64_t)c[u] * ldh + f0[p]);
                }
#pragma unroll
            for (int p = 0; p < NP; ++p)
#pragma unroll
                for (int u = 0; u < UNROLL; ++u)
#pragma unroll
                    for (int q = 0; q < VE; ++q) acc[p][q] += to_f32<T>(v[p][u].e[q]);
        }
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            if (!on[p]) continue;
            if (e1 > e0) {
#pragma unroll
                for (int q = 0; q < VE; ++q) acc[p][q] = acc[p][q] / m;
            }
            store_f32<T, VE>(A + i * lda + f0[p], acc[p]);
        }
    }
}

// Rows longer than `longer_than` edges (power-law hubs): one 1024-thread workgroup per row, each
// of its 16 waves sums a contiguous sixteenth of the row's edges, the 16 partial sums are added in
// wave order (a fixed order: deterministic).  A workgroup scans 1024 rows for long ones first.
constexpr int LONG_TB = 1024;
constexpr int LONG_FCH = 512;   // features per pass: 16 waves x 512 floats of LDS
template <typename T, int VE, typename IP>
__global__ __launch_bounds__(LONG_TB) void k_aggregate_long(const IP* __restrict__ indptr,
                                                            const int32_t* __restrict__ cols, int64_t n,
                                                            const T* __restrict__ H, int64_t ldh, int F,
                                                            T* __restrict__ A, int64_t lda, int64_t longer_than) {
    __shared__ int n_long;
    __shared__ int64_t long_rows[LONG_TB];
    __shared__ float part[LONG_TB / 64][LONG_FCH];
    if (threadIdx.x == 0) n_long = 0;
    __syncthreads();
    const int64_t row = (int64_t)blockIdx.x * LONG_TB + threadIdx.x;
    if (row < n && (int64_t)(indptr[row + 1] - indptr[row]) > longer_than) long_rows[atomicAdd(&n_long, 1)] = row;
    __syncthreads();
    const int cnt = n_long;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    constexpr int NW = LONG_TB / 64;
    for (int li = 0; li < cnt; ++li) {
        // the list order depends on the atomics, the result of each row does not
        const int64_t i = long_rows[li];
        const IP e0 = indptr[i], e1 = indptr[i + 1];
        const IP chunk = (e1 - e0 + NW - 1) / NW;
        const IP w0 = e0 + (IP)wave * chunk, w1 = (w0 + chunk < e1) ? w0 + chunk : e1;
        const float m = (float)(e1 - e0);
        for (int fbase = 0; fbase < F; fbase += LONG_FCH) {
            const int fend = min(F, fbase + LONG_FCH);
            for (int f0 = fbase + lane * VE; f0 < fend; f0 += 64 * VE) {
                float acc[VE];
#pragma unroll
                for (int q = 0; q < VE; ++q) acc[q] = 0.f;
                for (IP e = w0; e < w1; e += UNROLL) {
                    int c[UNROLL];
#pragma unroll
                    for (int u = 0; u < UNROLL; ++u) c[u] = (e + u < w1) ? cols[e + u] : -1;
                    float v[UNROLL][VE];
#pragma unroll
                    for (int u = 0; u < UNROLL; ++u) {
                        if (c[u] >= 0) {
                            load_f32<T, VE>(H + (int64_t)c[u] * ldh + f0, v[u]);
                        } else {
#pragma unroll
                            for (int q = 0; q < VE; ++q) v[u][q] = 0.f;
                        }
                    }
#pragma unroll
                    for (int u = 0; u < UNROLL; ++u)
#pragma unroll
                        for (int q = 0; q < VE; ++q) acc[q] += v[u][q];
                }
#pragma unroll
                for (int q = 0; q < VE; ++q) part[wave][f0 - fbase + q] = acc[q];
            }
            __syncthreads();
            for (int f = fbase + threadIdx.x; f < fend; f += LONG_TB) {
                float sum = 0.f;
#pragma unroll
                for (int w = 0; w < NW; ++w) sum += part[w][f - fbase];
                A[i * lda + f] = from_f32<T>(sum / m);
            }
            __syncthreads();
        }
    }
}

// ---- mean aggregation backward (gather through the transposed block) ------------
template <typename T, int VE, int G>
__global__ __launch_bounds__(TB) void k_aggregate_bwd(const int32_t* __restrict__ t_indptr,
                                                      const int32_t* __restrict__ t_rows,
                                                      const int32_t* __restrict__ b_indptr, const int32_t* counts,
                                                      const T* __restrict__ dAgg, int64_t ldg,
                                                      const T* __restrict__ dSelf, int64_t lds,
                                                      const T* __restrict__ relu_of, int F, T* __restrict__ dH,
                                                      int64_t ldd) {
    const int n_dst = counts[0], n_src = counts[1];
    const int gl = threadIdx.x % G;
    const int ngrp = gridDim.x * (TB / G);
    for (int j = blockIdx.x * (TB / G) + threadIdx.x / G; j < n_src; j += ngrp) {
        const int e0 = t_indptr[j], e1 = t_indptr[j + 1];
        for (int f0 = gl * VE; f0 < F; f0 += G * VE) {
            float acc[VE];
            if (dSelf && j < n_dst) {
                load_f32<T, VE>(dSelf + (int64_t)j * lds + f0, acc);
            } else {
#pragma unroll
                for (int q = 0; q < VE; ++q) acc[q] = 0.f;
            }
            for (int e = e0; e < e1; e += UNROLL) {
                int r[UNROLL];
                float w[UNROLL];
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) r[u] = (e + u < e1) ? t_rows[e + u] : -1;
                float v[UNROLL][VE];
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) {
                    if (r[u] >= 0) {
                        w[u] = (float)(b_indptr[r[u] + 1] - b_indptr[r[u]]);
                        load_f32<T, VE>(dAgg + (int64_t)r[u] * ldg + f0, v[u]);
                    } else {
                        w[u] = 1.f;
#pragma unroll
                        for (int q = 0; q < VE; ++q) v[u][q] = 0.f;
                    }
                }
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) {
                    const float inv = 1.0f / w[u];   // one division per edge, not per element
#pragma unroll
                    for (int q = 0; q < VE; ++q) acc[q] += v[u][q] * inv;
                }
            }
            if (relu_of) {
                float y[VE];
                load_f32<T, VE>(relu_of + (int64_t)j * ldd + f0, y);
#pragma unroll
                for (int q = 0; q < VE; ++q)
                    if (!(y[q] > 0.f)) acc[q] = 0.f;
            }
            store_f32<T, VE>(dH + (int64_t)j * ldd + f0, acc);
        }
    }
}

// Largest power-of-two vector (bytes, <= 16) that divides every row start and the row width.
int vec_bytes(size_t elem, int F, std::initializer_list<int64_t> lds, std::initializer_list<const void*> ptrs) {
    int vb = 16;
    auto fit = [&](uint64_t x) {
        while (vb > (int)elem && (x % vb) != 0) vb >>= 1;
    };
    fit((uint64_t)F * elem);
    for (int64_t ld : lds) fit((uint64_t)ld * elem);
    for (const void* p : ptrs) fit(reinterpret_cast<uintptr_t>(p));
    return vb;
}

// For kernels that move the last vector of a row back (see k_gather, k_aggregate_fwd): the widest
// vector (bytes, <= 16) that fits into a row, given that every row starts on a dword boundary
// (or on an element boundary for the one-element vector).
int vec_bytes_dword_rows(size_t elem, int F, std::initializer_list<int64_t> lds, std::initializer_list<const void*> ptrs) {
    bool dword = ((uint64_t)F * elem) % 4 == 0;   // the moved-back last vector must start on a dword as well
    for (int64_t ld : lds) dword = dword && ((uint64_t)ld * elem) % 4 == 0;
    for (const void* p : ptrs) dword = dword && reinterpret_cast<uintptr_t>(p) % 4 == 0;
    if (!dword) return vec_bytes(elem, F, lds, ptrs);
    int vb = 16;
    while (vb > (int)elem && (uint64_t)F * elem < (uint64_t)vb) vb >>= 1;
    return vb < 4 ? vec_bytes(elem, F, lds, ptrs) : vb;
}

int group_lanes(int vecs_per_row) {
    int g = 8;
    while (g < 64 && g < vecs_per_row) g <<= 1;
    return g;
}

inline int grid_rows(int64_t rows, int G) {
    int64_t b = (rows + (TB / G) - 1) / (TB / G);
    if (b < 1) b = 1;
    const int64_t cap = 256 * 8;  // 8 workgroups per CU; the kernels stride over the rest
    return (int)(b > cap ? cap : b);
}

// Dispatch over (dtype, vector width, group width) without writing the table out by hand.
template <typename F32Fn, typename BF16Fn>
bool dispatch(int32_t dtype, int ve, int G, F32Fn&& f32, BF16Fn&& bf) {
#define SDT_G(T, VE, fn)                                  \
    switch (G) {                                          \
        case 8: fn(T{}, std::integral_constant<int, VE>{}, std::integral_constant<int, 8>{}); return true;   \
        case 16: fn(T{}, std::integral_constant<int, VE>{}, std::integral_constant<int, 16>{}); return true; \
        case 32: fn(T{}, std::integral_constant<int, VE>{}, std::integral_constant<int, 32>{}); return true; \
        case 64: fn(T{}, std::integral_constant<int, VE>{}, std::integral_constant<int, 64>{}); return true; \
    }
    if (dtype == SDT_F32) {
        switch (ve) {
            case 4: SDT_G(float, 4, f32) break;
            case 2: SDT_G(float, 2, f32) break;
            case 1: SDT_G(float, 1, f32) break;
        }
    } else {
        switch (ve) {
            case 8: SDT_G(bf16_t, 8, bf) break;
            case 4: SDT_G(bf16_t, 4, bf) break;
            case 2: SDT_G(bf16_t, 2, bf) break;
            case 1: SDT_G(bf16_t, 1, bf) break;
        }
    }
#undef SDT_G
    return false;
}

template <typename IP>
int32_t launch_aggregate_fwd(const IP* indptr, const int32_t* cols, int64_t n_cap, const int32_t* n_d, const void* H,
                             int64_t ldh, int32_t F, int32_t dtype, void* A, int64_t lda, const int32_t* row_ids,
                             hipStream_t st) {
    if (n_cap == 0 || F == 0) return SDT_OK;
    const size_t es = dtype_size(dtype);
    // (the hub kernel of the whole-graph form keeps whole vectors per row)
    const int ve = (sizeof(IP) == 8 ? vec_bytes(es, F, {ldh, lda}, {H, A}) : vec_bytes_dword_rows(es, F, {ldh, lda}, {H, A})) / (int)es;
    const int G = group_lanes((F + ve - 1) / ve);
    // A whole graph (64-bit offsets): one row per lane group, as many workgroups as that takes (the
    // hardware hands them out as CUs free up, which balances power-law rows), hubs in a second launch.
    // A sampled block is launched for its upper bound and strides; its rows are at most a fan-out long.
    constexpr bool whole_graph = sizeof(IP) == 8;
    const int64_t long_rows = whole_graph ? 2048 : INT64_MAX;
    auto go = [&](auto t, auto vec, auto grp) {
        using T = decltype(t);
        constexpr int VE = decltype(vec)::value, GG = decltype(grp)::value;
        int grid = grid_rows(n_cap, GG);
        if constexpr (!whole_graph && GG == 64 && VE * sizeof(T) == 16) {
            // rows wider than one pass of the lane group: the passes run side by side (see k_aggregate_fwd_wide)
            const int np = ceil_div(ceil_div(F, VE), GG);
            if (np >= 2 && np <= 4) {
                const int32_t* ip = reinterpret_cast<const int32_t*>(indptr);
#define SDT_WIDE(NP)                                                                                                    \
    hipLaunchKernelGGL((k_aggregate_fwd_wide<T, VE, GG, NP>), dim3(grid), dim3(TB), 0, st, ip, cols, n_cap, n_d,        \
                       static_cast<const T*>(H), ldh, F, static_cast<T*>(A), lda, row_ids)
                if (np == 2) SDT_WIDE(2); else if (np == 3) SDT_WIDE(3); else SDT_WIDE(4);
#undef SDT_WIDE
                return;
            }
        }
        if (whole_graph) {
            const int64_t b = (n_cap + (TB / GG) - 1) / (TB / GG);
            grid = (int)(b > (1 << 24) ? (1 << 24) : b);
        }
        hipLaunchKernelGGL((k_aggregate_fwd<T, VE, GG, IP>), dim3(grid), dim3(TB), 0, st, indptr, cols, n_cap, n_d,
                           static_cast<const T*>(H), ldh, F, static_cast<T*>(A), lda, row_ids, long_rows);
        if (whole_graph)
            hipLaunchKernelGGL((k_aggregate_long<T, VE, IP>), dim3((int)((n_cap + LONG_TB - 1) / LONG_TB)), dim3(LONG_TB),
                               0, st, indptr, cols, n_cap, static_cast<const T*>(H), ldh, F, static_cast<T*>(A), lda,
                               long_rows);
    };
    if (!dispatch(dtype, ve, G, go, go)) {
        set_error("aggregate_fwd: no kernel for dtype %d vec %d group %d", dtype, ve, G);
        return SDT_ERR_INVALID_ARG;
    }
    SDT_CHECK_LAUNCH("aggregate_fwd");
    return SDT_OK;
}

}  // namespace
}  // namespace sdt

using namespace sdt;

namespace sdt {
int32_t gather_rows(const void* X, int64_t ldx, int32_t F, int32_t dtype, const int32_t* idx, int32_t n_cap,
                    const int32_t* n_d, void* out, int64_t ldo, bool zero_pad, void* also_pad, hipStream_t st) {
    SDT_REQUIRE(dtype_ok(dtype), SDT_ERR_INVALID_ARG, "sdt_gather_features: unknown dtype %d", dtype);
    SDT_REQUIRE(F >= 0 && n_cap >= 0 && ldx >= F && ldo >= F, SDT_ERR_INVALID_ARG,
                "sdt_gather_features: bad sizes F=%d n=%d ldx=%lld ldo=%lld", F, n_cap, (long long)ldx, (long long)ldo);
    if (n_cap == 0 || F == 0) return SDT_OK;
    SDT_REQUIRE(X && idx && out, SDT_ERR_INVALID_ARG, "sdt_gather_features: null pointer");
    const size_t es = dtype_size(dtype);
    const int vb = vec_bytes_dword_rows(es, F, {ldx, ldo}, {X, out, also_pad});
    const int row_b = (int)(F * es);
    const int G = group_lanes((row_b + vb - 1) / vb);
    const char* Xc = static_cast<const char*>(X);
    char* oc = static_cast<char*>(out);
    const int64_t ldx_b = ldx * (int64_t)es, ldo_b = ldo * (int64_t)es;
#define SDT_GATHER(VB, GG)                                                                                         \
    hipLaunchKernelGGL((k_gather<VB, GG>), dim3(grid_rows(n_cap, GG)), dim3(TB), 0, st, Xc, ldx_b, row_b, idx, n_cap, \
                       n_d, oc, ldo_b, zero_pad ? (int)ldo_b : 0, zero_pad ? static_cast<char*>(also_pad) : nullptr)
#define SDT_GATHER_G(VB)                    \
    switch (G) {                            \
        case 8: SDT_GATHER(VB, 8); break;   \
        case 16: SDT_GATHER(VB, 16); break; \
        case 32: SDT_GATHER(VB, 32); break; \
        default: SDT_GATHER(VB, 64); break; \
    }
    switch (vb) {
        case 16: SDT_GATHER_G(16) break;
        case 8: SDT_GATHER_G(8) break;
        case 4: SDT_GATHER_G(4) break;
        default: SDT_GATHER_G(2) break;
    }
#undef SDT_GATHER_G
#undef SDT_GATHER
    SDT_CHECK_LAUNCH("gather");
    return SDT_OK;
}
}  // namespace sdt

extern "C" int32_t sdt_gather_features(const void* X, int64_t ldx, int32_t F, int32_t dtype, const int32_t* idx,
                                       int32_t n_cap, const int32_t* n_d, void* out, int64_t ldo, void* stream) {
    return gather_rows(X, ldx, F, dtype, idx, n_cap, n_d, out, ldo, false, nullptr, static_cast<hipStream_t>(stream));
}

extern "C" int32_t sdt_sage_aggregate_fwd(const sdt_block* blk, const void* H, int64_t ldh, int32_t F, int32_t dtype,
                                          void* A, int64_t lda, void* stream) {
    SDT_REQUIRE(blk, SDT_ERR_INVALID_ARG, "sdt_sage_aggregate_fwd: null block");
    SDT_REQUIRE(dtype_ok(dtype), SDT_ERR_INVALID_ARG, "sdt_sage_aggregate_fwd: unknown dtype %d", dtype);
    SDT_REQUIRE(F >= 0 && blk->cap_dst >= 0 && ldh >= F && lda >= F, SDT_ERR_INVALID_ARG,
                "sdt_sage_aggregate_fwd: bad sizes");
    if (blk->cap_dst == 0 || F == 0) return SDT_OK;
    SDT_REQUIRE(blk->counts && blk->indptr && H && A && (blk->cols || blk->cap_nnz == 0), SDT_ERR_INVALID_ARG,
                "sdt_sage_aggregate_fwd: null pointer");
    return launch_aggregate_fwd<int32_t>(blk->indptr, blk->cols, blk->cap_dst, blk->counts, H, ldh, F, dtype, A, lda,
                                         nullptr, static_cast<hipStream_t>(stream));
}

namespace sdt {
int32_t aggregate_gather_fwd(const sdt_block* blk, const void* X, int64_t ldx, int32_t F, int32_t dtype, void* A,
                             int64_t lda, hipStream_t st) {
    SDT_REQUIRE(blk, SDT_ERR_INVALID_ARG, "sdt_sage_aggregate_gather_fwd: null block");
    SDT_REQUIRE(dtype_ok(dtype), SDT_ERR_INVALID_ARG, "sdt_sage_aggregate_gather_fwd: unknown dtype %d", dtype);
    SDT_REQUIRE(F >= 0 && blk->cap_dst >= 0 && ldx >= F && lda >= F, SDT_ERR_INVALID_ARG,
                "sdt_sage_aggregate_gather_fwd: bad sizes");
    if (blk->cap_dst == 0 || F == 0) return SDT_OK;
    SDT_REQUIRE(blk->counts && blk->indptr && blk->src_nodes && X && A && (blk->cols || blk->cap_nnz == 0),
                SDT_ERR_INVALID_ARG, "sdt_sage_aggregate_gather_fwd: null pointer");
    return launch_aggregate_fwd<int32_t>(blk->indptr, blk->cols, blk->cap_dst, blk->counts, X, ldx, F, dtype, A, lda,
                                         blk->src_nodes, st);
}
}  // namespace sdt

extern "C" int32_t sdt_sage_aggregate_gather_fwd(const sdt_block* blk, const void* X, int64_t ldx, int32_t F,
                                                 int32_t dtype, void* A, int64_t lda, void* stream) {
    return aggregate_gather_fwd(blk, X, ldx, F, dtype, A, lda, static_cast<hipStream_t>(stream));
}

extern "C" int32_t sdt_sage_aggregate_csr_fwd(const sdt_csr* g, const void* H, int64_t ldh, int32_t F, int32_t dtype,
                                              void* A, int64_t lda, void* stream) {
    SDT_REQUIRE(g, SDT_ERR_INVALID_ARG, "sdt_sage_aggregate_csr_fwd: null graph");
    SDT_REQUIRE(dtype_ok(dtype), SDT_ERR_INVALID_ARG, "sdt_sage_aggregate_csr_fwd: unknown dtype %d", dtype);
    SDT_REQUIRE(F >= 0 && g->n_nodes >= 0 && g->n_nodes <= 0x7FFFFFFF && ldh >= F && lda >= F, SDT_ERR_INVALID_ARG,
                "sdt_sage_aggregate_csr_fwd: bad sizes");
    if (g->n_nodes == 0 || F == 0) return SDT_OK;
    SDT_REQUIRE(g->indptr && g->indices && H && A, SDT_ERR_INVALID_ARG, "sdt_sage_aggregate_csr_fwd: null pointer");
    return launch_aggregate_fwd<int64_t>(g->indptr, g->indices, g->n_nodes, nullptr, H, ldh, F, dtype, A, lda,
                                         nullptr, static_cast<hipStream_t>(stream));
}

extern "C" int32_t sdt_sage_aggregate_bwd(const sdt_block* blk, const void* dAgg, int64_t ldg, const void* dSelf,
                                          int64_t lds, const void* relu_of, int32_t F, int32_t dtype, void* dH,
                                          int64_t ldd, void* stream) {
    SDT_REQUIRE(blk, SDT_ERR_INVALID_ARG, "sdt_sage_aggregate_bwd: null block");
    SDT_REQUIRE(dtype_ok(dtype), SDT_ERR_INVALID_ARG, "sdt_sage_aggregate_bwd: unknown dtype %d", dtype);
    SDT_REQUIRE(F >= 0 && blk->cap_src >= 0 && ldg >= F && ldd >= F && (!dSelf || lds >= F), SDT_ERR_INVALID_ARG,
                "sdt_sage_aggregate_bwd: bad sizes");
    if (blk->cap_src == 0 || F == 0) return SDT_OK;
    SDT_REQUIRE(blk->counts && blk->indptr && blk->t_indptr && blk->t_rows && dAgg && dH, SDT_ERR_INVALID_ARG,
                "sdt_sage_aggregate_bwd: null pointer (the block needs its transposed arrays)");
    const size_t es = dtype_size(dtype);
    const int ve = vec_bytes(es, F, {ldg, ldd, dSelf ? lds : ldd}, {dAgg, dH, dSelf, relu_of}) / (int)es;
    const int G = group_lanes((F + ve - 1) / ve);
    hipStream_t st = static_cast<hipStream_t>(stream);
    auto go = [&](auto t, auto vec, auto grp) {
        using T = decltype(t);
        constexpr int VE = decltype(vec)::value, GG = decltype(grp)::value;
        hipLaunchKernelGGL((k_aggregate_bwd<T, VE, GG>), dim3(grid_rows(blk->cap_src, GG)), dim3(TB), 0, st,
                           blk->t_indptr, blk->t_rows, blk->indptr, blk->counts, static_cast<const T*>(dAgg), ldg,
                           static_cast<const T*>(dSelf), lds, static_cast<const T*>(relu_of), F, static_cast<T*>(dH),
                           ldd);
    };
    if (!dispatch(dtype, ve, G, go, go)) {
        set_error("sdt_sage_aggregate_bwd: no kernel for dtype %d vec %d group %d", dtype, ve, G);
        return SDT_ERR_INVALID_ARG;
    }
    SDT_CHECK_LAUNCH("aggregate_bwd");
    return SDT_OK;
}
