// GCN aggregation on sampled blocks (fp32 or bf16 storage, fp32 sums): the degree-normalised neighbour sum with a self term,
//   A[i,:] = s[i] * sum_{e in row i} c[col_e] * H[col_e,:] + selfw[i] * H[i,:],
// its transpose through the transposed block, and the kernel that derives c, s, selfw from the
// degrees of the partition graph.  Same row-group scheme as the mean aggregation: a group of
// lanes per row, 16-byte vectors (forward: from any dword-aligned row), eight row loads in flight, fp32 sums
// in edge order (forward) / ascending destination order (backward) -- deterministic.
#include "common.h"

namespace sdt {
namespace {

constexpr int TB = 256;
constexpr int U = 8;

// 16- and 8-byte accesses declared with 4-byte alignment: several-dword global accesses need dword
// alignment only, so rows that start on any dword boundary move whole vectors
struct __attribute__((packed, aligned(4))) f4d { float x, y, z, w; };
struct __attribute__((packed, aligned(4))) f2d { float x, y; };

template <int VE>
__device__ __forceinline__ void ld(const float* p, float (&v)[VE]) {
    if constexpr (VE == 4) {
        const f4d t = *reinterpret_cast<const f4d*>(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else if constexpr (VE == 2) {
        const f2d t = *reinterpret_cast<const f2d*>(p);
        v[0] = t.x; v[1] = t.y;
    } else {
        v[0] = *p;
    }
}
template <int VE>
__device__ __forceinline__ void st(float* p, const float (&v)[VE]) {
    if constexpr (VE == 4) *reinterpret_cast<f4d*>(p) = f4d{v[0], v[1], v[2], v[3]};
    else if constexpr (VE == 2) *reinterpret_cast<f2d*>(p) = f2d{v[0], v[1]};
    else *p = v[0];
}

// the same for bf16 storage (2-byte elements; VE of them are one 8-, 4- or 2-byte access): widened on the way in,
// rounded to nearest even on the way out
struct __attribute__((packed, aligned(4))) h4d { uint32_t lo, hi; };
template <int VE>
__device__ __forceinline__ void ld(const bf16_t* p, float (&v)[VE]) {
    if constexpr (VE == 4) {
        const h4d t = *reinterpret_cast<const h4d*>(p);
        v[0] = __uint_as_float(t.lo << 16); v[1] = __uint_as_float(t.lo & 0xFFFF0000u);
        v[2] = __uint_as_float(t.hi << 16); v[3] = __uint_as_float(t.hi & 0xFFFF0000u);
    } else if constexpr (VE == 2) {
        const uint32_t t = *reinterpret_cast<const uint32_t*>(p);
        v[0] = __uint_as_float(t << 16); v[1] = __uint_as_float(t & 0xFFFF0000u);
    } else {
        v[0] = bf16_to_f32(p->bits);
    }
}
template <int VE>
__device__ __forceinline__ void st(bf16_t* p, const float (&v)[VE]) {
    if constexpr (VE == 4) {
        *reinterpret_cast<h4d*>(p) = h4d{(uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16),
                                         (uint32_t)f32_to_bf16(v[2]) | ((uint32_t)f32_to_bf16(v[3]) << 16)};
    } else if constexpr (VE == 2) {
        *reinterpret_cast<uint32_t*>(p) = (uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16);
    } else {
        p->bits = f32_to_bf16(v[0]);
    }
}

// c[j] = 1/sqrt(deg_j + 1) for every source row; s[i] = (deg_i / m_i) / sqrt(deg_i + 1) (0 if the row
// sampled nothing) and selfw[i] = 1/(deg_i + 1) for every destination row; deg from the graph's CSR.
__global__ __launch_bounds__(TB) void k_gcn_norm(const int64_t* __restrict__ g_indptr,
                                                 const int32_t* __restrict__ src_nodes,
                                                 const int32_t* __restrict__ b_indptr, const int32_t* counts,
                                                 float* __restrict__ c, float* __restrict__ s,
                                                 float* __restrict__ selfw) {
    const int n_dst = counts[0], n_src = counts[1];
    for (int j = blockIdx.x * TB + threadIdx.x; j < n_src; j += gridDim.x * TB) {
        const int64_t v = src_nodes[j];
        const float deg = (float)(g_indptr[v + 1] - g_indptr[v]);
        const float r = 1.0f / sqrtf(deg + 1.0f);
        c[j] = r;
        if (j < n_dst) {
            const float m = (float)(b_indptr[j + 1] - b_indptr[j]);
            s[j] = m > 0.f ? (deg / m) * r : 0.f;
            selfw[j] = 1.0f / (deg + 1.0f);
        }
    }
}

// row_ids (nullable): local row r lives at H[row_ids[r]] (aggregating straight out of the feature
// matrix through the block's src_nodes).
template <typename T, int VE, int G>
__global__ __launch_bounds__(TB) void k_gcn_aggregate_fwd(const int32_t* __restrict__ b_indptr,
                                                          const int32_t* __restrict__ cols, const int32_t* counts,
                                                          const T* __restrict__ H, int64_t ldh,
                                                          const int32_t* __restrict__ row_ids, int F,
                                                          const float* __restrict__ c, const float* __restrict__ s,
                                                          const float* __restrict__ selfw, T* __restrict__ A,
                                                          int64_t lda) {
    const int n = counts[0];
    const int gl = threadIdx.x % G;
    const int ngrp = gridDim.x * (TB / G);
    for (int i = blockIdx.x * (TB / G) + threadIdx.x / G; i < n; i += ngrp) {
        const int e0 = b_indptr[i], e1 = b_indptr[i + 1];
        const int64_t own = row_ids ? row_ids[i] : i;
        const float si = s[i], wi = selfw[i];
        // the last vector of a row whose width is not a multiple of VE is moved back to end with the row
        // (it overlaps its neighbour; both lanes compute and store the same values); F >= VE
        for (int fn = gl * VE; fn < F; fn += G * VE) {
            const int f0 = min(fn, F - VE);
            float acc[VE];
#pragma unroll
            for (int q = 0; q < VE; ++q) acc[q] = 0.f;
            for (int e = e0; e < e1; e += U) {
                int64_t r[U];
                float w[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int col = (e + u < e1) ? cols[e + u] : -1;
                    w[u] = col >= 0 ? c[col] : 0.f;
                    r[u] = col < 0 ? -1 : (row_ids ? (int64_t)row_ids[col] : (int64_t)col);
                }
                float v[U][VE];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (r[u] >= 0) {
                        ld<VE>(H + r[u] * ldh + f0, v[u]);
                    } else {
#pragma unroll
                        for (int q = 0; q < VE; ++q) v[u][q] = 0.f;
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int q = 0; q < VE; ++q) acc[q] += w[u] * v[u][q];
            }
            float h[VE];
            ld<VE>(H + own * ldh + f0, h);
#pragma unroll
            for (int q = 0; q < VE; ++q) acc[q] = si * acc[q] + wi * h[q];
            st<VE>(A + (int64_t)i * lda + f0, acc);
        }
    }
}

// dH[j,:] = c[j] * sum over the transposed segment of j of s[i] * dA[i,:] + [j < n_dst] selfw[j] * dA[j,:],
// zeroed where relu_of[j,:] <= 0 (nullable).
template <typename T, int VE, int G>
__global__ __launch_bounds__(TB) void k_gcn_aggregate_bwd(const int32_t* __restrict__ t_indptr,
                                                          const int32_t* __restrict__ t_rows, const int32_t* counts,
                                                          const T* __restrict__ dA, int64_t lda, int F,
                                                          const float* __restrict__ c, const float* __restrict__ s,
                                                          const float* __restrict__ selfw,
                                                          const T* __restrict__ relu_of, T* __restrict__ dH,
                                                          int64_t ldd) {
    const int n_dst = counts[0], n_src = counts[1];
    const int gl = threadIdx.x % G;
    const int ngrp = gridDim.x * (TB / G);
    for (int j = blockIdx.x * (TB / G) + threadIdx.x / G; j < n_src; j += ngrp) {
        const int e0 = t_indptr[j], e1 = t_indptr[j + 1];
        const float cj = c[j];
        for (int f0 = gl * VE; f0 < F; f0 += G * VE) {
            float acc[VE];
#pragma unroll
            for (int q = 0; q < VE; ++q) acc[q] = 0.f;
            for (int e = e0; e < e1; e += U) {
                int r[U];
                float w[U];
                float v[U][VE];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    r[u] = (e + u < e1) ? t_rows[e + u] : -1;
                    w[u] = r[u] >= 0 ? s[r[u]] : 0.f;
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (r[u] >= 0) {
                        ld<VE>(dA + (int64_t)r[u] * lda + f0, v[u]);
                    } else {
#pragma unroll
                        for (int q = 0; q < VE; ++q) v[u][q] = 0.f;
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int q = 0; q < VE; ++q) acc[q] += w[u] * v[u][q];
            }
#pragma unroll
            for (int q = 0; q < VE; ++q) acc[q] *= cj;
            if (j < n_dst) {
                float g[VE];
                ld<VE>(dA + (int64_t)j * lda + f0, g);
                const float wj = selfw[j];
#pragma unroll
                for (int q = 0; q < VE; ++q) acc[q] += wj * g[q];
            }
            if (relu_of) {
                float y[VE];
                ld<VE>(relu_of + (int64_t)j * ldd + f0, y);
#pragma unroll
                for (int q = 0; q < VE; ++q)
                    if (!(y[q] > 0.f)) acc[q] = 0.f;
            }
            st<VE>(dH + (int64_t)j * ldd + f0, acc);
        }
    }
}

// widest vector (elements of `es` bytes, at most four) that divides the row width, every stride and every address
int vec_elems_of(int es, int F, std::initializer_list<int64_t> lds, std::initializer_list<const void*> ptrs) {
    int v = 4;
    auto fit = [&](uint64_t bytes) {
        while (v > 1 && bytes % (uint64_t)(v * es) != 0) v >>= 1;
    };
    fit((uint64_t)F * es);
    for (int64_t l : lds) fit((uint64_t)l * es);
    for (const void* p : ptrs) fit(reinterpret_cast<uintptr_t>(p));
    return v;
}

inline int rows_grid(int64_t rows, int G) {
    int64_t b = (rows + (TB / G) - 1) / (TB / G);
    if (b < 1) b = 1;
    return (int)(b > 2048 ? 2048 : b);
}

#define SDT_GCN_DISPATCH(ve, G, body)                                     \
    do {                                                                  \
        if (G == 64) {                                                    \
            constexpr int GG = 64;                                        \
            if (ve == 4) { constexpr int VE = 4; body; }                  \
            else if (ve == 2) { constexpr int VE = 2; body; }             \
            else { constexpr int VE = 1; body; }                          \
        } else {                                                          \
            constexpr int GG = 16;                                        \
            if (ve == 4) { constexpr int VE = 4; body; }                  \
            else if (ve == 2) { constexpr int VE = 2; body; }             \
            else { constexpr int VE = 1; body; }                          \
        }                                                                 \
    } while (0)

}  // namespace

int32_t gcn_aggregate_fwd(const sdt_block* blk, const void* H, int64_t ldh, bool through_src_nodes, int32_t F, int32_t dtype,
                          const float* c, const float* s, const float* selfw, void* A, int64_t lda, hipStream_t stm) {
    const int32_t* ids = through_src_nodes ? blk->src_nodes : nullptr;
    if (dtype == SDT_F32) {
        // the forward kernel moves its last vector back, so any dword-aligned fp32 row takes the widest vector that fits
        const int ve = F >= 4 ? 4 : F >= 2 ? 2 : 1;
        const int G = (F + ve - 1) / ve > 16 ? 64 : 16;
        SDT_GCN_DISPATCH(ve, G, hipLaunchKernelGGL((k_gcn_aggregate_fwd<float, VE, GG>), dim3(rows_grid(blk->cap_dst, GG)),
                                                   dim3(TB), 0, stm, blk->indptr, blk->cols, blk->counts,
                                                   static_cast<const float*>(H), ldh, ids, F, c, s, selfw,
                                                   static_cast<float*>(A), lda));
    } else {
        // bf16 rows: whole vectors only (a vector moved back to the row's end would start on an odd element)
        const int ve = vec_elems_of(2, F, {ldh, lda}, {H, A});
        const int G = (F + ve - 1) / ve > 16 ? 64 : 16;
        SDT_GCN_DISPATCH(ve, G, hipLaunchKernelGGL((k_gcn_aggregate_fwd<bf16_t, VE, GG>), dim3(rows_grid(blk->cap_dst, GG)),
                                                   dim3(TB), 0, stm, blk->indptr, blk->cols, blk->counts,
                                                   static_cast<const bf16_t*>(H), ldh, ids, F, c, s, selfw,
                                                   static_cast<bf16_t*>(A), lda));
    }
    SDT_CHECK_LAUNCH("gcn_aggregate_fwd");
    return SDT_OK;
}

}  // namespace sdt

using namespace sdt;

extern "C" int32_t sdt_gcn_norm(const sdt_csr* graph, const sdt_block* blk, float* c, float* s, float* selfw,
                                void* stream) {
    SDT_REQUIRE(graph && graph->indptr && blk, SDT_ERR_INVALID_ARG, "sdt_gcn_norm: null graph or block");
    if (blk->cap_src == 0) return SDT_OK;
    SDT_REQUIRE(blk->counts && blk->indptr && blk->src_nodes && c && s && selfw, SDT_ERR_INVALID_ARG,
                "sdt_gcn_norm: null pointer");
    const int blocks = (blk->cap_src + TB - 1) / TB;
    hipLaunchKernelGGL(k_gcn_norm, dim3(blocks > 1024 ? 1024 : blocks), dim3(TB), 0, static_cast<hipStream_t>(stream),
                       graph->indptr, blk->src_nodes, blk->indptr, blk->counts, c, s, selfw);
    SDT_CHECK_LAUNCH("gcn_norm");
    return SDT_OK;
}

extern "C" int32_t sdt_gcn_aggregate_fwd(const sdt_block* blk, const void* H, int64_t ldh, int32_t through_src_nodes,
                                         int32_t F, int32_t dtype, const float* c, const float* s, const float* selfw,
                                         void* A, int64_t lda, void* stream) {
    SDT_REQUIRE(blk, SDT_ERR_INVALID_ARG, "sdt_gcn_aggregate_fwd: null block");
    SDT_REQUIRE(dtype_ok(dtype), SDT_ERR_INVALID_ARG, "sdt_gcn_aggregate_fwd: unknown dtype %d", dtype);
    SDT_REQUIRE(F >= 0 && ldh >= F && lda >= F, SDT_ERR_INVALID_ARG, "sdt_gcn_aggregate_fwd: bad sizes");
    if (blk->cap_dst == 0 || F == 0) return SDT_OK;
    SDT_REQUIRE(blk->counts && blk->indptr && blk->cols && H && A && c && s && selfw &&
                    (!through_src_nodes || blk->src_nodes),
                SDT_ERR_INVALID_ARG, "sdt_gcn_aggregate_fwd: null pointer");
    return gcn_aggregate_fwd(blk, H, ldh, through_src_nodes != 0, F, dtype, c, s, selfw, A, lda,
                             static_cast<hipStream_t>(stream));
}

extern "C" int32_t sdt_gcn_aggregate_bwd(const sdt_block* blk, const void* dA, int64_t lda, const void* relu_of,
                                         int32_t F, int32_t dtype, const float* c, const float* s, const float* selfw,
                                         void* dH, int64_t ldd, void* stream) {
    SDT_REQUIRE(blk, SDT_ERR_INVALID_ARG, "sdt_gcn_aggregate_bwd: null block");
    SDT_REQUIRE(dtype_ok(dtype), SDT_ERR_INVALID_ARG, "sdt_gcn_aggregate_bwd: unknown dtype %d", dtype);
    SDT_REQUIRE(F >= 0 && lda >= F && ldd >= F, SDT_ERR_INVALID_ARG, "sdt_gcn_aggregate_bwd: bad sizes");
    if (blk->cap_src == 0 || F == 0) return SDT_OK;
    SDT_REQUIRE(blk->counts && blk->t_indptr && blk->t_rows && dA && dH && c && s && selfw, SDT_ERR_INVALID_ARG,
                "sdt_gcn_aggregate_bwd: null pointer (the block needs its transposed arrays)");
    hipStream_t stm = static_cast<hipStream_t>(stream);
    const int ve = vec_elems_of((int)dtype_size(dtype), F, {lda, ldd}, {dA, dH, relu_of});
    const int G = (F + ve - 1) / ve > 16 ? 64 : 16;
    if (dtype == SDT_F32) {
        SDT_GCN_DISPATCH(ve, G, hipLaunchKernelGGL((k_gcn_aggregate_bwd<float, VE, GG>), dim3(rows_grid(blk->cap_src, GG)),
                                                   dim3(TB), 0, stm, blk->t_indptr, blk->t_rows, blk->counts,
                                                   static_cast<const float*>(dA), lda, F, c, s, selfw,
                                                   static_cast<const float*>(relu_of), static_cast<float*>(dH), ldd));
    } else {
        SDT_GCN_DISPATCH(ve, G, hipLaunchKernelGGL((k_gcn_aggregate_bwd<bf16_t, VE, GG>), dim3(rows_grid(blk->cap_src, GG)),
                                                   dim3(TB), 0, stm, blk->t_indptr, blk->t_rows, blk->counts,
                                                   static_cast<const bf16_t*>(dA), lda, F, c, s, selfw,
                                                   static_cast<const bf16_t*>(relu_of), static_cast<bf16_t*>(dH), ldd));
    }
    SDT_CHECK_LAUNCH("gcn_aggregate_bwd");
    return SDT_OK;
}
