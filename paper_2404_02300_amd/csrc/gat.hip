// Single-head graph-attention aggregation over a sampled block (fp32), forward and backward.
//   s_(i<-j) = LeakyReLU(a_dst . z_i + a_src . z_j) over row i's edges and the self edge j = i,
//   alpha = softmax over that set, out_i = sum alpha_(i<-j) z_j.
// One wavefront per row everywhere: lane l owns features l, l+64, ...; dot products are reduced
// over the wave with an xor butterfly (a fixed order), edge sums run in edge order (forward) or in
// ascending destination order through the transposed block (backward): deterministic, no atomics.
// The forward leaves el = z a_src, er = z a_dst and the log-sum-exp of every row in the workspace;
// the backward recomputes each attention weight from them instead of storing one per edge.
#include "common.h"

namespace sdt {
namespace {

constexpr int TB = 256;
constexpr int WPB = TB / 64;  // rows per workgroup

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float leaky(float x, float slope) { return x > 0.f ? x : slope * x; }

struct GatWs {
    float *el, *er, *lse, *t, *der, *del, *part, *biasq;
    int nblk, nchunk;
    size_t total;
};
constexpr int VEC_ROWS = 256;  // rows per partial sum of the attention-vector gradients
GatWs gat_ws(void* base, int32_t cap_src, int32_t cap_dst, int32_t F) {
    Arena a(base);
    GatWs w;
    w.el = a.take<float>(cap_src > 0 ? cap_src : 1);
    w.er = a.take<float>(cap_dst > 0 ? cap_dst : 1);
    w.lse = a.take<float>(cap_dst > 0 ? cap_dst : 1);
    w.t = a.take<float>(cap_dst > 0 ? cap_dst : 1);
    w.der = a.take<float>(cap_dst > 0 ? cap_dst : 1);
    w.del = a.take<float>(cap_src > 0 ? cap_src : 1);
    w.nblk = ceil_div(cap_src > 0 ? cap_src : 1, VEC_ROWS);
    w.part = a.take<float>((size_t)w.nblk * 2 * (F > 0 ? F : 1));
    w.nchunk = ceil_div(cap_dst > 0 ? cap_dst : 1, VEC_ROWS);
    w.biasq = a.take<float>((size_t)w.nchunk * (F > 0 ? F : 1));
    w.total = a.off;
    return w;
}

// el[j] = z_j . a_src (all source rows), er[i] = z_i . a_dst (destination rows)
__global__ __launch_bounds__(TB) void k_gat_scores(const int32_t* counts, const float* __restrict__ z, int64_t ldz, int F,
                                                   const float* __restrict__ a_src, const float* __restrict__ a_dst,
                                                   float* __restrict__ el, float* __restrict__ er) {
    const int n_dst = counts[0], n_src = counts[1];
    const int lane = threadIdx.x & 63;
    for (int j = blockIdx.x * WPB + (threadIdx.x >> 6); j < n_src; j += gridDim.x * WPB) {
        float sl = 0.f, sr = 0.f;
        for (int f = lane; f < F; f += 64) {
            const float v = z[(int64_t)j * ldz + f];
            sl += v * a_src[f];
            sr += v * a_dst[f];
        }
        sl = wave_sum(sl);
        sr = wave_sum(sr);
        if (lane == 0) {
            el[j] = sl;
            if (j < n_dst) er[j] = sr;
        }
    }
}

__global__ __launch_bounds__(TB) void k_gat_fwd(const int32_t* __restrict__ b_indptr, const int32_t* __restrict__ cols,
                                                const int32_t* counts, const float* __restrict__ z, int64_t ldz, int F,
                                                const float* __restrict__ el, const float* __restrict__ er, float slope,
                                                float* __restrict__ lse, const float* __restrict__ bias, int relu,
                                                float* __restrict__ out, int64_t ldo) {
    const int n = counts[0];
    const int lane = threadIdx.x & 63;
    for (int i = blockIdx.x * WPB + (threadIdx.x >> 6); i < n; i += gridDim.x * WPB) {
        const int e0 = b_indptr[i], e1 = b_indptr[i + 1];
        const float ri = er[i];
        const float s_self = leaky(ri + el[i], slope);
        float m = s_self;
        for (int e = e0 + lane; e < e1; e += 64) m = fmaxf(m, leaky(ri + el[cols[e]], slope));
        m = wave_max(m);
        float sum = 0.f;
        for (int e = e0 + lane; e < e1; e += 64) sum += expf(leaky(ri + el[cols[e]], slope) - m);
        sum = wave_sum(sum) + expf(s_self - m);
        const float l = m + logf(sum);
        if (lane == 0) lse[i] = l;
        const float a_self = expf(s_self - l);
        for (int f = lane; f < F; f += 64) {
            float acc = 0.f;
            for (int e = e0; e < e1; ++e) {
                const int c = cols[e];
                acc += expf(leaky(ri + el[c], slope) - l) * z[(int64_t)c * ldz + f];
            }
            float v = acc + a_self * z[(int64_t)i * ldz + f];
            if (bias) v += bias[f];
            if (relu && !(v > 0.f)) v = 0.f;
            out[(int64_t)i * ldo + f] = v;
        }
    }
}

// per destination row: t_i = sum_e alpha_e (g_i . z_col) and der_i = sum_e d pre_e (both including the self edge)
__global__ __launch_bounds__(TB) void k_gat_bwd_dst(const int32_t* __restrict__ b_indptr, const int32_t* __restrict__ cols,
                                                    const int32_t* counts, const float* __restrict__ z, int64_t ldz, int F,
                                                    const float* __restrict__ el, const float* __restrict__ er,
                                                    const float* __restrict__ lse, float slope,
                                                    const float* __restrict__ g, int64_t ldg, float* __restrict__ t,
                                                    float* __restrict__ der) {
    const int n = counts[0];
    const int lane = threadIdx.x & 63;
    for (int i = blockIdx.x * WPB + (threadIdx.x >> 6); i < n; i += gridDim.x * WPB) {
        const int e0 = b_indptr[i], e1 = b_indptr[i + 1];
        const float ri = er[i], l = lse[i];
        auto dot_with = [&](int64_t row) {
            float d = 0.f;
            for (int f = lane; f < F; f += 64) d += g[(int64_t)i * ldg + f] * z[row * ldz + f];
            return wave_sum(d);
        };
        // first pass: t_i
        const float pre_self = ri + el[i];
        const float a_self = expf(leaky(pre_self, slope) - l), d_self = dot_with(i);
        float ti = a_self * d_self;
        for (int e = e0; e < e1; ++e) {
            const int c = cols[e];
            ti += expf(leaky(ri + el[c], slope) - l) * dot_with(c);
        }
        // second pass: d pre_e = alpha_e (d alpha_e - t_i) LeakyReLU'(pre_e)
        float dr = a_self * (d_self - ti) * (pre_self > 0.f ? 1.f : slope);
        for (int e = e0; e < e1; ++e) {
            const int c = cols[e];
            const float pre = ri + el[c];
            dr += expf(leaky(pre, slope) - l) * (dot_with(c) - ti) * (pre > 0.f ? 1.f : slope);
        }
        if (lane == 0) {
            t[i] = ti;
            der[i] = dr;
        }
    }
}

// per source row j, through the transposed block:
//   dz_j = sum_{(i<-j)} alpha g_i + [j<n_dst] alpha_self g_j + del_j a_src + [j<n_dst] der_j a_dst,
//   del_j = sum of d pre over the edges that end in j (and j's own self edge)
__global__ __launch_bounds__(TB) void k_gat_bwd_src(const int32_t* __restrict__ t_indptr, const int32_t* __restrict__ t_rows,
                                                    const int32_t* counts, const float* __restrict__ z, int64_t ldz, int F,
                                                    const float* __restrict__ el, const float* __restrict__ er,
                                                    const float* __restrict__ lse, const float* __restrict__ t,
                                                    const float* __restrict__ der, float slope,
                                                    const float* __restrict__ a_src, const float* __restrict__ a_dst,
                                                    const float* __restrict__ g, int64_t ldg, float* __restrict__ dz,
                                                    int64_t lddz, float* __restrict__ del) {
    const int n_dst = counts[0], n_src = counts[1];
    const int lane = threadIdx.x & 63;
    for (int j = blockIdx.x * WPB + (threadIdx.x >> 6); j < n_src; j += gridDim.x * WPB) {
        const int e0 = t_indptr[j], e1 = t_indptr[j + 1];
        const float lj = el[j];
        // first the scalar part: alpha and d pre of every edge that ends here
        float dl = 0.f;
        float a_self = 0.f;
        if (j < n_dst) {
            float d = 0.f;
            for (int f = lane; f < F; f += 64) d += g[(int64_t)j * ldg + f] * z[(int64_t)j * ldz + f];
            d = wave_sum(d);
            const float pre = er[j] + lj;
            a_self = expf(leaky(pre, slope) - lse[j]);
            dl += a_self * (d - t[j]) * (pre > 0.f ? 1.f : slope);
        }
        for (int e = e0; e < e1; ++e) {
            const int i = t_rows[e];
            float d = 0.f;
            for (int f = lane; f < F; f += 64) d += g[(int64_t)i * ldg + f] * z[(int64_t)j * ldz + f];
            d = wave_sum(d);
            const float pre = er[i] + lj;
            dl += expf(leaky(pre, slope) - lse[i]) * (d - t[i]) * (pre > 0.f ? 1.f : slope);
        }
        if (lane == 0) del[j] = dl;
        const float drj = j < n_dst ? der[j] : 0.f;
        for (int f = lane; f < F; f += 64) {
            float acc = 0.f;
            for (int e = e0; e < e1; ++e) {
                const int i = t_rows[e];
                acc += expf(leaky(er[i] + lj, slope) - lse[i]) * g[(int64_t)i * ldg + f];
            }
            if (j < n_dst) acc += a_self * g[(int64_t)j * ldg + f] + drj * a_dst[f];
            dz[(int64_t)j * lddz + f] = acc + dl * a_src[f];
        }
    }
}

// part[b][0][f] = sum over the rows of chunk b of del_j z_j[f]; part[b][1][f] likewise with der_i (rows < n_dst)
__global__ __launch_bounds__(TB) void k_gat_vec_partials(const int32_t* counts, const float* __restrict__ z, int64_t ldz,
                                                         int F, const float* __restrict__ del,
                                                         const float* __restrict__ der, float* __restrict__ part) {
    const int n_dst = counts[0], n_src = counts[1];
    const int r0 = blockIdx.x * VEC_ROWS, r1 = min(n_src, r0 + VEC_ROWS);
    for (int f = threadIdx.x; f < F; f += TB) {
        float s0 = 0.f, s1 = 0.f;
        for (int r = r0; r < r1; ++r) {
            const float v = z[(int64_t)r * ldz + f];
            s0 += del[r] * v;
            if (r < n_dst) s1 += der[r] * v;
        }
        part[((int64_t)blockIdx.x * 2 + 0) * F + f] = s0;
        part[((int64_t)blockIdx.x * 2 + 1) * F + f] = s1;
    }
}
__global__ __launch_bounds__(TB) void k_gat_vec_final(const float* __restrict__ part, int nblk, int F,
                                                      float* __restrict__ da_src, float* __restrict__ da_dst) {
    for (int f = blockIdx.x * TB + threadIdx.x; f < F; f += gridDim.x * TB) {
        float s0 = 0.f, s1 = 0.f;
        for (int b = 0; b < nblk; ++b) {   // chunk order: deterministic
            s0 += part[((int64_t)b * 2 + 0) * F + f];
            s1 += part[((int64_t)b * 2 + 1) * F + f];
        }
        da_src[f] = s0;
        da_dst[f] = s1;
    }
}

// In place: g[r][f] = 0 where Y[r][f] <= 0 (Y may be null), and Qb[chunk][f] = column sum of the
// masked g over the chunk's rows (zero for chunks past the row count).
__global__ __launch_bounds__(TB) void k_gat_mask_bias(const int32_t* counts, float* __restrict__ g, int64_t ldg,
                                                      const float* __restrict__ Y, int64_t ldy, int F,
                                                      float* __restrict__ Qb) {
    const int n = counts[0];
    const int r0 = blockIdx.x * VEC_ROWS, r1 = min(n, r0 + VEC_ROWS);
    for (int f = threadIdx.x; f < F; f += TB) {
        float s = 0.f;
        for (int r = r0; r < r1; ++r) {
            float v = g[(int64_t)r * ldg + f];
            if (Y && !(Y[(int64_t)r * ldy + f] > 0.f)) {
                v = 0.f;
                g[(int64_t)r * ldg + f] = 0.f;
            }
            s += v;
        }
        Qb[(int64_t)blockIdx.x * F + f] = s;
    }
}

inline int rows_grid(int rows) {
    const int b = ceil_div(rows > 0 ? rows : 1, WPB);
    return b > 4096 ? 4096 : b;
}

}  // namespace
}  // namespace sdt

using namespace sdt;

extern "C" size_t sdt_gat_workspace_bytes(int32_t cap_src, int32_t cap_dst, int32_t F) {
    if (cap_src < 0 || cap_dst < 0 || F < 0) return 0;
    return gat_ws(nullptr, cap_src, cap_dst, F).total;
}

extern "C" int32_t sdt_gat_aggregate_fwd(const sdt_block* blk, const float* z, int64_t ldz, int32_t F, const float* a_src,
                                         const float* a_dst, float slope, float* out, int64_t ldo, void* ws, size_t ws_bytes,
                                         void* stream) {
    return gat_forward(blk, z, ldz, F, a_src, a_dst, slope, nullptr, 0, out, ldo, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

int32_t sdt::gat_forward(const sdt_block* blk, const float* z, int64_t ldz, int32_t F, const float* a_src, const float* a_dst,
                         float slope, const float* bias, int32_t relu, float* out, int64_t ldo, void* ws, size_t ws_bytes,
                         hipStream_t st) {
    SDT_REQUIRE(blk, SDT_ERR_INVALID_ARG, "sdt_gat_aggregate_fwd: null block");
    SDT_REQUIRE(F >= 0 && ldz >= F && ldo >= F && blk->cap_src >= blk->cap_dst, SDT_ERR_INVALID_ARG,
                "sdt_gat_aggregate_fwd: bad sizes");
    if (blk->cap_dst == 0 || F == 0) return SDT_OK;
    SDT_REQUIRE(blk->counts && blk->indptr && blk->cols && z && a_src && a_dst && out, SDT_ERR_INVALID_ARG,
                "sdt_gat_aggregate_fwd: null pointer");
    const GatWs w = gat_ws(ws, blk->cap_src, blk->cap_dst, F);
    SDT_REQUIRE(ws && ws_bytes >= w.total && aligned16(ws), SDT_ERR_WORKSPACE,
                "sdt_gat_aggregate_fwd: workspace of %zu bytes needed, %zu given", w.total, ws_bytes);
    hipLaunchKernelGGL(k_gat_scores, dim3(rows_grid(blk->cap_src)), dim3(TB), 0, st, blk->counts, z, ldz, F, a_src, a_dst, w.el,
                       w.er);
    SDT_CHECK_LAUNCH("gat scores");
    hipLaunchKernelGGL(k_gat_fwd, dim3(rows_grid(blk->cap_dst)), dim3(TB), 0, st, blk->indptr, blk->cols, blk->counts, z, ldz, F,
                       w.el, w.er, slope, w.lse, bias, relu, out, ldo);
    SDT_CHECK_LAUNCH("gat forward");
    return SDT_OK;
}

extern "C" int32_t sdt_gat_aggregate_bwd(const sdt_block* blk, const float* z, int64_t ldz, int32_t F, const float* a_src,
                                         const float* a_dst, float slope, const float* g, int64_t ldg, float* dz,
                                         int64_t lddz, float* da_src, float* da_dst, void* ws, size_t ws_bytes, void* stream) {
    SDT_REQUIRE(da_src && da_dst, SDT_ERR_INVALID_ARG, "sdt_gat_aggregate_bwd: null attention-vector gradient");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const float* part = nullptr;
    int32_t n_part = 0;
    const int32_t rc = gat_backward(blk, z, ldz, F, a_src, a_dst, slope, g, ldg, dz, lddz, ws, ws_bytes, &part, &n_part, st);
    if (rc != SDT_OK || !part) return rc;
    hipLaunchKernelGGL(k_gat_vec_final, dim3(ceil_div(F, TB)), dim3(TB), 0, st, part, n_part, F, da_src, da_dst);
    SDT_CHECK_LAUNCH("gat attention-vector reduction");
    return SDT_OK;
}

int32_t sdt::gat_backward(const sdt_block* blk, const float* z, int64_t ldz, int32_t F, const float* a_src,
                          const float* a_dst, float slope, const float* g, int64_t ldg, float* dz, int64_t lddz, void* ws,
                          size_t ws_bytes, const float** part, int32_t* n_part, hipStream_t st) {
    *part = nullptr;
    *n_part = 0;
    SDT_REQUIRE(blk, SDT_ERR_INVALID_ARG, "sdt_gat_aggregate_bwd: null block");
    SDT_REQUIRE(F >= 0 && ldz >= F && ldg >= F && lddz >= F && blk->cap_src >= blk->cap_dst, SDT_ERR_INVALID_ARG,
                "sdt_gat_aggregate_bwd: bad sizes");
    if (blk->cap_src == 0 || F == 0) return SDT_OK;
    SDT_REQUIRE(blk->counts && blk->indptr && blk->cols && blk->t_indptr && blk->t_rows && z && a_src && a_dst && g && dz,
                SDT_ERR_INVALID_ARG, "sdt_gat_aggregate_bwd: null pointer (the block needs its transposed arrays)");
    const GatWs w = gat_ws(ws, blk->cap_src, blk->cap_dst, F);
    SDT_REQUIRE(ws && ws_bytes >= w.total && aligned16(ws), SDT_ERR_WORKSPACE,
                "sdt_gat_aggregate_bwd: workspace of %zu bytes needed, %zu given", w.total, ws_bytes);
    hipLaunchKernelGGL(k_gat_bwd_dst, dim3(rows_grid(blk->cap_dst)), dim3(TB), 0, st, blk->indptr, blk->cols, blk->counts, z, ldz,
                       F, w.el, w.er, w.lse, slope, g, ldg, w.t, w.der);
    SDT_CHECK_LAUNCH("gat backward (destinations)");
    hipLaunchKernelGGL(k_gat_bwd_src, dim3(rows_grid(blk->cap_src)), dim3(TB), 0, st, blk->t_indptr, blk->t_rows, blk->counts, z,
                       ldz, F, w.el, w.er, w.lse, w.t, w.der, slope, a_src, a_dst, g, ldg, dz, lddz, w.del);
    SDT_CHECK_LAUNCH("gat backward (sources)");
    hipLaunchKernelGGL(k_gat_vec_partials, dim3(w.nblk), dim3(TB), 0, st, blk->counts, z, ldz, F, w.del, w.der, w.part);
    SDT_CHECK_LAUNCH("gat attention-vector partials");
    *part = w.part;
    *n_part = w.nblk;
    return SDT_OK;
}

int32_t sdt::gat_mask_bias(const sdt_block* blk, float* g, int64_t ldg, const float* Y, int64_t ldy, int32_t F, void* ws,
                           size_t ws_bytes, const float** Qb, int32_t* n_chunks, hipStream_t st) {
    SDT_REQUIRE(blk && blk->counts && g && F > 0 && ldg >= F && (!Y || ldy >= F), SDT_ERR_INVALID_ARG, "gat_mask_bias: bad arguments");
    const GatWs w = gat_ws(ws, blk->cap_src, blk->cap_dst, F);
    SDT_REQUIRE(ws && ws_bytes >= w.total && aligned16(ws), SDT_ERR_WORKSPACE, "gat_mask_bias: workspace of %zu bytes needed, %zu given",
                w.total, ws_bytes);
    hipLaunchKernelGGL(k_gat_mask_bias, dim3(w.nchunk), dim3(TB), 0, st, blk->counts, g, ldg, Y, ldy, F, w.biasq);
    SDT_CHECK_LAUNCH("gat mask + bias partials");
    *Qb = w.biasq;
    *n_chunks = w.nchunk;
    return SDT_OK;
}
