// Single-head graph-attention aggregation over a sampled block, forward and backward; feature rows in fp32 or
// bf16 storage (widened on load, rounded on store), every sum and the attention scalars in fp32.
//   s_(i<-j) = LeakyReLU(a_dst . z_i + a_src . z_j) over row i's edges and the self edge j = i,
//   alpha = softmax over that set, out_i = sum alpha_(i<-j) z_j.
// One wavefront per row everywhere: lane l owns features l, l+64, ...; dot products are reduced
// over the wave with an xor butterfly (a fixed order), edge sums run in edge order (forward) or in
// ascending destination order through the transposed block (backward): deterministic, no atomics.
// The forward leaves el = z a_src, er = z a_dst and the log-sum-exp of every row in the workspace;
// the backward recomputes each attention weight from them instead of storing one per edge.
#include "common.h"

#include <initializer_list>

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

// four consecutive features of a row, widened to fp32 / rounded from it
__device__ __forceinline__ float4 ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ float4 ld4(const bf16_t* p) {
    const uint2 t = *reinterpret_cast<const uint2*>(p);
    return make_float4(__uint_as_float(t.x << 16), __uint_as_float(t.x & 0xFFFF0000u), __uint_as_float(t.y << 16),
                       __uint_as_float(t.y & 0xFFFF0000u));
}
__device__ __forceinline__ void st4(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
__device__ __forceinline__ void st4(bf16_t* p, float4 v) {
    *reinterpret_cast<uint2*>(p) = make_uint2((uint32_t)f32_to_bf16(v.x) | ((uint32_t)f32_to_bf16(v.y) << 16),
                                              (uint32_t)f32_to_bf16(v.z) | ((uint32_t)f32_to_bf16(v.w) << 16));
}

struct GatWs {
    float *el, *er, *lse, *t, *der, *del, *part, *biasq;
    int nblk, nchunk;
    size_t total;
};
constexpr int VEC_ROWS = GAT_CHUNK_ROWS;  // rows per partial sum of the attention-vector and bias gradients
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
template <typename TZ>
__global__ __launch_bounds__(TB) void k_gat_scores(const int32_t* counts, const TZ* __restrict__ z, int64_t ldz, int F,
                                                   const float* __restrict__ a_src, const float* __restrict__ a_dst,
                                                   float* __restrict__ el, float* __restrict__ er) {
    const int n_dst = counts[0], n_src = counts[1];
    const int lane = threadIdx.x & 63;
    for (int j = blockIdx.x * WPB + (threadIdx.x >> 6); j < n_src; j += gridDim.x * WPB) {
        float sl = 0.f, sr = 0.f;
        for (int f = lane; f < F; f += 64) {
            const float v = to_f32(z[(int64_t)j * ldz + f]);
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

template <typename TZ, typename TO>
__global__ __launch_bounds__(TB) void k_gat_fwd(const int32_t* __restrict__ b_indptr, const int32_t* __restrict__ cols,
                                                const int32_t* counts, const TZ* __restrict__ z, int64_t ldz, int F,
                                                const float* __restrict__ el, const float* __restrict__ er, float slope,
                                                float* __restrict__ lse, const float* __restrict__ bias, int relu,
                                                TO* __restrict__ out, int64_t ldo) {
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
                acc += expf(leaky(ri + el[c], slope) - l) * to_f32(z[(int64_t)c * ldz + f]);
            }
            float v = acc + a_self * to_f32(z[(int64_t)i * ldz + f]);
            if (bias) v += bias[f];
            if (relu && !(v > 0.f)) v = 0.f;
            out[(int64_t)i * ldo + f] = from_f32<TO>(v);
        }
    }
}

// per destination row: t_i = sum_e alpha_e (g_i . z_col) and der_i = sum_e d pre_e (both including the self edge)
template <typename TZ, typename TG>
__global__ __launch_bounds__(TB) void k_gat_bwd_dst(const int32_t* __restrict__ b_indptr, const int32_t* __restrict__ cols,
                                                    const int32_t* counts, const TZ* __restrict__ z, int64_t ldz, int F,
                                                    const float* __restrict__ el, const float* __restrict__ er,
                                                    const float* __restrict__ lse, float slope,
                                                    const TG* __restrict__ g, int64_t ldg, float* __restrict__ t,
                                                    float* __restrict__ der) {
    const int n = counts[0];
    const int lane = threadIdx.x & 63;
    for (int i = blockIdx.x * WPB + (threadIdx.x >> 6); i < n; i += gridDim.x * WPB) {
        const int e0 = b_indptr[i], e1 = b_indptr[i + 1];
        const float ri = er[i], l = lse[i];
        auto dot_with = [&](int64_t row) {
            float d = 0.f;
            for (int f = lane; f < F; f += 64) d += to_f32(g[(int64_t)i * ldg + f]) * to_f32(z[row * ldz + f]);
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
template <typename TZ, typename TG>
__global__ __launch_bounds__(TB) void k_gat_bwd_src(const int32_t* __restrict__ t_indptr, const int32_t* __restrict__ t_rows,
                                                    const int32_t* counts, const TZ* __restrict__ z, int64_t ldz, int F,
                                                    const float* __restrict__ el, const float* __restrict__ er,
                                                    const float* __restrict__ lse, const float* __restrict__ t,
                                                    const float* __restrict__ der, float slope,
                                                    const float* __restrict__ a_src, const float* __restrict__ a_dst,
                                                    const TG* __restrict__ g, int64_t ldg, TZ* __restrict__ dz,
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
            for (int f = lane; f < F; f += 64) d += to_f32(g[(int64_t)j * ldg + f]) * to_f32(z[(int64_t)j * ldz + f]);
            d = wave_sum(d);
            const float pre = er[j] + lj;
            a_self = expf(leaky(pre, slope) - lse[j]);
            dl += a_self * (d - t[j]) * (pre > 0.f ? 1.f : slope);
        }
        for (int e = e0; e < e1; ++e) {
            const int i = t_rows[e];
            float d = 0.f;
            for (int f = lane; f < F; f += 64) d += to_f32(g[(int64_t)i * ldg + f]) * to_f32(z[(int64_t)j * ldz + f]);
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
                acc += expf(leaky(er[i] + lj, slope) - lse[i]) * to_f32(g[(int64_t)i * ldg + f]);
            }
            if (j < n_dst) acc += a_self * to_f32(g[(int64_t)j * ldg + f]) + drj * a_dst[f];
            dz[(int64_t)j * lddz + f] = from_f32<TZ>(acc + dl * a_src[f]);
        }
    }
}

// part[b][0][f] = sum over the rows of chunk b of del_j z_j[f]; part[b][1][f] likewise with der_i (rows < n_dst).
// Wave w of the workgroup sums the chunk's rows w, w+4, ... (lane = feature, 64 at a time); the four
// wave sums are then added in wave order.  Chunks past the row count write zeros.
template <typename TZ>
__global__ __launch_bounds__(TB) void k_gat_vec_partials(const int32_t* counts, const TZ* __restrict__ z, int64_t ldz,
                                                         int F, const float* __restrict__ del,
                                                         const float* __restrict__ der, float* __restrict__ part) {
    __shared__ float red[WPB][2][64];
    const int n_dst = counts[0], n_src = counts[1];
    const int r0 = blockIdx.x * VEC_ROWS, r1 = min(n_src, r0 + VEC_ROWS);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    for (int f0 = 0; f0 < F; f0 += 64) {
        const int f = f0 + lane;
        float s0 = 0.f, s1 = 0.f;
        if (f < F) {
#pragma unroll 8
            for (int r = r0 + w; r < r1; r += WPB) {
                const float v = to_f32(z[(int64_t)r * ldz + f]);
                s0 += del[r] * v;
                s1 += (r < n_dst ? der[r] : 0.f) * v;
            }
        }
        red[w][0][lane] = s0;
        red[w][1][lane] = s1;
        __syncthreads();
        if (w < 2 && f < F) {
            float t = 0.f;
#pragma unroll
            for (int k = 0; k < WPB; ++k) t += red[k][w][lane];
            part[((int64_t)blockIdx.x * 2 + w) * F + f] = t;
        }
        __syncthreads();
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
// masked g over the chunk's rows (zero for chunks past the row count).  Rows are dealt to the four
// waves as in k_gat_vec_partials.
template <typename TG>
__global__ __launch_bounds__(TB) void k_gat_mask_bias(const int32_t* counts, TG* __restrict__ g, int64_t ldg,
                                                      const TG* __restrict__ Y, int64_t ldy, int F,
                                                      float* __restrict__ Qb) {
    __shared__ float red[WPB][64];
    const int n = counts[0];
    const int r0 = blockIdx.x * VEC_ROWS, r1 = min(n, r0 + VEC_ROWS);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    // the 64-column slices of a chunk are dealt to gridDim.y workgroups (few chunks: more of them in flight)
    for (int f0 = blockIdx.y * 64; f0 < F; f0 += gridDim.y * 64) {
        const int f = f0 + lane;
        float s = 0.f;
        if (f < F) {
            if (Y) {
                // eight rows per round: all loads first, then the stores (a store between them would
                // serialise the loads, since the compiler must assume it aliases the next row)
                constexpr int U = 8;
                for (int rb = r0 + w; rb < r1; rb += U * WPB) {
                    float v[U], y[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int r = min(rb + u * WPB, r1 - 1);
                        v[u] = to_f32(g[(int64_t)r * ldg + f]);
                        y[u] = to_f32(Y[(int64_t)r * ldy + f]);
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int r = rb + u * WPB;
                        if (r < r1) {
                            if (y[u] > 0.f) s += v[u];
                            else g[(int64_t)r * ldg + f] = from_f32<TG>(0.f);
                        }
                    }
                }
            } else {
#pragma unroll 8
                for (int r = r0 + w; r < r1; r += WPB) s += to_f32(g[(int64_t)r * ldg + f]);
            }
        }
        red[w][lane] = s;
        __syncthreads();
        if (w == 0 && f < F) Qb[(int64_t)blockIdx.x * F + f] = ((red[0][lane] + red[1][lane]) + red[2][lane]) + red[3][lane];
        __syncthreads();
    }
}

// ---- 16-byte variants (F % 4 == 0, rows 16-byte aligned, F <= 256) ----------------------------
// A wave still owns one row, but its lanes form four groups of sixteen: group q takes the row's
// edges q, q+4, ... and lane r of a group owns the features 4r..4r+3 (+64 per further chunk), so
// four neighbour rows are in flight at once, every load is 16 bytes, a dot product is reduced over
// sixteen lanes only, and every row is visited once.  Group sums are combined with an xor butterfly
// (a fixed order: deterministic).
template <int KF>
struct Slice {
    float4 v[KF];
    template <typename T>
    __device__ __forceinline__ void load(const T* __restrict__ row, int r, int F) {
#pragma unroll
        for (int k = 0; k < KF; ++k) {
            const int c = 4 * r + 64 * k;
            v[k] = c < F ? ld4(row + c) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    __device__ __forceinline__ void zero() {
#pragma unroll
        for (int k = 0; k < KF; ++k) v[k] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    __device__ __forceinline__ float dot(const Slice& o) const {
        float d = 0.f;
#pragma unroll
        for (int k = 0; k < KF; ++k) d += v[k].x * o.v[k].x + v[k].y * o.v[k].y + v[k].z * o.v[k].z + v[k].w * o.v[k].w;
        return d;
    }
    __device__ __forceinline__ void axpy(float a, const Slice& o) {
#pragma unroll
        for (int k = 0; k < KF; ++k) {
            v[k].x += a * o.v[k].x; v[k].y += a * o.v[k].y; v[k].z += a * o.v[k].z; v[k].w += a * o.v[k].w;
        }
    }
    // sum over the four groups (lanes r, r+16, r+32, r+48); every lane ends with the total
    __device__ __forceinline__ void sum_groups() {
#pragma unroll
        for (int k = 0; k < KF; ++k) {
#pragma unroll
            for (int o = 16; o <= 32; o <<= 1) {
                v[k].x += __shfl_xor(v[k].x, o, 64); v[k].y += __shfl_xor(v[k].y, o, 64);
                v[k].z += __shfl_xor(v[k].z, o, 64); v[k].w += __shfl_xor(v[k].w, o, 64);
            }
        }
    }
};
__device__ __forceinline__ float group_sum(float v) {   // over the sixteen lanes of a group
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float across_groups(float v) {
    v += __shfl_xor(v, 16, 64);
    v += __shfl_xor(v, 32, 64);
    return v;
}

template <typename TZ, typename TO, int KF>
__global__ __launch_bounds__(TB) void k_gat_fwd_v(const int32_t* __restrict__ b_indptr, const int32_t* __restrict__ cols,
                                                  const int32_t* counts, const TZ* __restrict__ z, int64_t ldz, int F,
                                                  const float* __restrict__ el, const float* __restrict__ er, float slope,
                                                  float* __restrict__ lse, const float* __restrict__ bias, int relu,
                                                  TO* __restrict__ out, int64_t ldo) {
    const int n = counts[0];
    const int lane = threadIdx.x & 63, q = lane >> 4, r = lane & 15;
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
        Slice<KF> acc, zr;
        acc.zero();
#pragma unroll 2
        for (int e = e0 + q; e < e1; e += 4) {
            const int c = cols[e];
            zr.load(z + (int64_t)c * ldz, r, F);
            acc.axpy(expf(leaky(ri + el[c], slope) - l), zr);
        }
        acc.sum_groups();
        if (q == 0) {
            zr.load(z + (int64_t)i * ldz, r, F);
            acc.axpy(expf(s_self - l), zr);
#pragma unroll
            for (int k = 0; k < KF; ++k) {
                const int c = 4 * r + 64 * k;
                if (c < F) {
                    float4 v = acc.v[k];
                    if (bias) {
                        const float4 bb = *reinterpret_cast<const float4*>(bias + c);
                        v.x += bb.x; v.y += bb.y; v.z += bb.z; v.w += bb.w;
                    }
                    if (relu) {
                        v.x = v.x > 0.f ? v.x : 0.f; v.y = v.y > 0.f ? v.y : 0.f;
                        v.z = v.z > 0.f ? v.z : 0.f; v.w = v.w > 0.f ? v.w : 0.f;
                    }
                    st4(out + (int64_t)i * ldo + c, v);
                }
            }
        }
    }
}

// t_i = sum_e alpha_e d_e and der_i = sum_e alpha_e (d_e - t_i) s'_e with d_e = g_i . z_col, s'_e the
// LeakyReLU slope at the edge's score, both sums including the self edge.  One visit per edge:
// der_i = sum alpha d s' - t_i sum alpha s'.
template <typename TZ, typename TG, int KF>
__global__ __launch_bounds__(TB) void k_gat_bwd_dst_v(const int32_t* __restrict__ b_indptr, const int32_t* __restrict__ cols,
                                                      const int32_t* counts, const TZ* __restrict__ z, int64_t ldz, int F,
                                                      const float* __restrict__ el, const float* __restrict__ er,
                                                      const float* __restrict__ lse, float slope,
                                                      const TG* __restrict__ g, int64_t ldg, float* __restrict__ t,
                                                      float* __restrict__ der) {
    const int n = counts[0];
    const int lane = threadIdx.x & 63, q = lane >> 4, r = lane & 15;
    for (int i = blockIdx.x * WPB + (threadIdx.x >> 6); i < n; i += gridDim.x * WPB) {
        const int e0 = b_indptr[i], e1 = b_indptr[i + 1];
        const float ri = er[i], l = lse[i];
        Slice<KF> gi, zr;
        gi.load(g + (int64_t)i * ldg, r, F);
        float s1 = 0.f, s2 = 0.f, s3 = 0.f;   // per group
#pragma unroll 2
        for (int e = e0 + q; e < e1; e += 4) {
            const int c = cols[e];
            zr.load(z + (int64_t)c * ldz, r, F);
            const float d = group_sum(gi.dot(zr));
            const float pre = ri + el[c];
            const float a = expf(leaky(pre, slope) - l), sp = pre > 0.f ? 1.f : slope;
            s1 += a * d;
            s2 += a * d * sp;
            s3 += a * sp;
        }
        s1 = across_groups(s1);
        s2 = across_groups(s2);
        s3 = across_groups(s3);
        zr.load(z + (int64_t)i * ldz, r, F);
        const float d_self = group_sum(gi.dot(zr));
        const float pre_self = ri + el[i];
        const float a_self = expf(leaky(pre_self, slope) - l), sp_self = pre_self > 0.f ? 1.f : slope;
        const float ti = s1 + a_self * d_self;
        if (lane == 0) {
            t[i] = ti;
            der[i] = (s2 + a_self * d_self * sp_self) - ti * (s3 + a_self * sp_self);
        }
    }
}

template <typename TZ, typename TG, int KF>
__global__ __launch_bounds__(TB) void k_gat_bwd_src_v(const int32_t* __restrict__ t_indptr, const int32_t* __restrict__ t_rows,
                                                      const int32_t* counts, const TZ* __restrict__ z, int64_t ldz, int F,
                                                      const float* __restrict__ el, const float* __restrict__ er,
                                                      const float* __restrict__ lse, const float* __restrict__ t,
                                                      const float* __restrict__ der, float slope,
                                                      const float* __restrict__ a_src, const float* __restrict__ a_dst,
                                                      const TG* __restrict__ g, int64_t ldg, TZ* __restrict__ dz,
                                                      int64_t lddz, float* __restrict__ del) {
    const int n_dst = counts[0], n_src = counts[1];
    const int lane = threadIdx.x & 63, q = lane >> 4, r = lane & 15;
    for (int j = blockIdx.x * WPB + (threadIdx.x >> 6); j < n_src; j += gridDim.x * WPB) {
        const int e0 = t_indptr[j], e1 = t_indptr[j + 1];
        const float lj = el[j];
        Slice<KF> zj, gr, acc;
        zj.load(z + (int64_t)j * ldz, r, F);
        acc.zero();
        float dl = 0.f;   // per group
#pragma unroll 2
        for (int e = e0 + q; e < e1; e += 4) {
            const int i = t_rows[e];
            gr.load(g + (int64_t)i * ldg, r, F);
            const float d = group_sum(zj.dot(gr));
            const float pre = er[i] + lj;
            const float a = expf(leaky(pre, slope) - lse[i]);
            dl += a * (d - t[i]) * (pre > 0.f ? 1.f : slope);
            acc.axpy(a, gr);
        }
        dl = across_groups(dl);
        acc.sum_groups();
        float drj = 0.f;
        if (j < n_dst) {   // the self edge (uniform over the wave)
            gr.load(g + (int64_t)j * ldg, r, F);
            const float d = group_sum(zj.dot(gr));
            const float pre = er[j] + lj;
            const float a_self = expf(leaky(pre, slope) - lse[j]);
            dl += a_self * (d - t[j]) * (pre > 0.f ? 1.f : slope);
            acc.axpy(a_self, gr);
            drj = der[j];
        }
        if (lane == 0) del[j] = dl;
        if (q == 0) {
#pragma unroll
            for (int k = 0; k < KF; ++k) {
                const int c = 4 * r + 64 * k;
                if (c < F) {
                    const float4 as = *reinterpret_cast<const float4*>(a_src + c);
                    const float4 ad = *reinterpret_cast<const float4*>(a_dst + c);
                    float4 v = acc.v[k];
                    v.x += dl * as.x + drj * ad.x; v.y += dl * as.y + drj * ad.y;
                    v.z += dl * as.z + drj * ad.z; v.w += dl * as.w + drj * ad.w;
                    st4(dz + (int64_t)j * lddz + c, v);
                }
            }
        }
    }
}

// 16-byte kernels apply when every row (and the attention vectors, the bias) can be read as float4
inline bool vec_ok(int F, std::initializer_list<int64_t> lds, std::initializer_list<const void*> ptrs) {
    if (F % 4 != 0 || F > 256) return false;
    for (int64_t ld : lds)
        if (ld % 4 != 0) return false;
    for (const void* p : ptrs)
        if (p && !aligned16(p)) return false;
    return true;
}
#define SDT_GAT_KF(F, body)                                \
    do {                                                   \
        if ((F) <= 64) { constexpr int KF = 1; body; }     \
        else if ((F) <= 128) { constexpr int KF = 2; body; } \
        else { constexpr int KF = 4; body; }               \
    } while (0)

inline int rows_grid(int rows) {
    const int b = ceil_div(rows > 0 ? rows : 1, WPB);
    return b > 4096 ? 4096 : b;
}

template <typename TZ, typename TO>
int32_t forward_t(const sdt_block* blk, const TZ* z, int64_t ldz, int32_t F, const float* a_src, const float* a_dst, float slope,
                  const float* bias, int32_t relu, TO* out, int64_t ldo, const GatWs& w, hipStream_t st) {
    hipLaunchKernelGGL(k_gat_scores<TZ>, dim3(rows_grid(blk->cap_src)), dim3(TB), 0, st, blk->counts, z, ldz, F, a_src, a_dst,
                       w.el, w.er);
    SDT_CHECK_LAUNCH("gat scores");
    if (vec_ok(F, {ldz, ldo}, {z, out, bias})) {
        SDT_GAT_KF(F, hipLaunchKernelGGL((k_gat_fwd_v<TZ, TO, KF>), dim3(rows_grid(blk->cap_dst)), dim3(TB), 0, st, blk->indptr,
                                         blk->cols, blk->counts, z, ldz, F, w.el, w.er, slope, w.lse, bias, relu, out, ldo));
    } else {
        hipLaunchKernelGGL((k_gat_fwd<TZ, TO>), dim3(rows_grid(blk->cap_dst)), dim3(TB), 0, st, blk->indptr, blk->cols,
                           blk->counts, z, ldz, F, w.el, w.er, slope, w.lse, bias, relu, out, ldo);
    }
    SDT_CHECK_LAUNCH("gat forward");
    return SDT_OK;
}

template <typename TZ, typename TG>
int32_t backward_t(const sdt_block* blk, const TZ* z, int64_t ldz, int32_t F, const float* a_src, const float* a_dst, float slope,
                   const TG* g, int64_t ldg, TZ* dz, int64_t lddz, const GatWs& w, hipStream_t st) {
    if (vec_ok(F, {ldz, ldg, lddz}, {z, g, dz, a_src, a_dst})) {
        SDT_GAT_KF(F, hipLaunchKernelGGL((k_gat_bwd_dst_v<TZ, TG, KF>), dim3(rows_grid(blk->cap_dst)), dim3(TB), 0, st,
                                         blk->indptr, blk->cols, blk->counts, z, ldz, F, w.el, w.er, w.lse, slope, g, ldg, w.t,
                                         w.der));
        SDT_CHECK_LAUNCH("gat backward (destinations)");
        SDT_GAT_KF(F, hipLaunchKernelGGL((k_gat_bwd_src_v<TZ, TG, KF>), dim3(rows_grid(blk->cap_src)), dim3(TB), 0, st,
                                         blk->t_indptr, blk->t_rows, blk->counts, z, ldz, F, w.el, w.er, w.lse, w.t, w.der, slope,
                                         a_src, a_dst, g, ldg, dz, lddz, w.del));
        SDT_CHECK_LAUNCH("gat backward (sources)");
    } else {
        hipLaunchKernelGGL((k_gat_bwd_dst<TZ, TG>), dim3(rows_grid(blk->cap_dst)), dim3(TB), 0, st, blk->indptr, blk->cols,
                           blk->counts, z, ldz, F, w.el, w.er, w.lse, slope, g, ldg, w.t, w.der);
        SDT_CHECK_LAUNCH("gat backward (destinations)");
        hipLaunchKernelGGL((k_gat_bwd_src<TZ, TG>), dim3(rows_grid(blk->cap_src)), dim3(TB), 0, st, blk->t_indptr, blk->t_rows,
                           blk->counts, z, ldz, F, w.el, w.er, w.lse, w.t, w.der, slope, a_src, a_dst, g, ldg, dz, lddz, w.del);
        SDT_CHECK_LAUNCH("gat backward (sources)");
    }
    hipLaunchKernelGGL(k_gat_vec_partials<TZ>, dim3(w.nblk), dim3(TB), 0, st, blk->counts, z, ldz, F, w.del, w.der, w.part);
    SDT_CHECK_LAUNCH("gat attention-vector partials");
    return SDT_OK;
}

template <typename TG>
int32_t mask_bias_t(const sdt_block* blk, TG* g, int64_t ldg, const TG* Y, int64_t ldy, int32_t F, const GatWs& w,
                    hipStream_t st) {
    hipLaunchKernelGGL(k_gat_mask_bias<TG>, dim3(w.nchunk, w.nchunk >= 1024 ? 1 : (F + 63) / 64), dim3(TB), 0, st, blk->counts, g,
                       ldg, Y, ldy, F, w.biasq);
    SDT_CHECK_LAUNCH("gat mask + bias partials");
    return SDT_OK;
}

// the projected rows may be bf16 with fp32 beside them (logits out, loss gradient in), never the other way round
inline bool types_ok(int32_t z_dtype, int32_t other) {
    return dtype_ok(z_dtype) && dtype_ok(other) && (z_dtype == SDT_BF16 || other == SDT_F32);
}

}  // namespace
}  // namespace sdt

using namespace sdt;

extern "C" size_t sdt_gat_workspace_bytes(int32_t cap_src, int32_t cap_dst, int32_t F) {
    if (cap_src < 0 || cap_dst < 0 || F < 0) return 0;
    return gat_ws(nullptr, cap_src, cap_dst, F).total;
}

extern "C" int32_t sdt_gat_aggregate_fwd(const sdt_block* blk, const void* z, int64_t ldz, int32_t F, int32_t dtype,
                                         const float* a_src, const float* a_dst, float slope, void* out, int64_t ldo, void* ws,
                                         size_t ws_bytes, void* stream) {
    return gat_forward(blk, z, ldz, F, dtype, a_src, a_dst, slope, nullptr, 0, out, ldo, dtype, ws, ws_bytes,
                       static_cast<hipStream_t>(stream));
}

int32_t sdt::gat_forward(const sdt_block* blk, const void* z, int64_t ldz, int32_t F, int32_t z_dtype, const float* a_src,
                         const float* a_dst, float slope, const float* bias, int32_t relu, void* out, int64_t ldo,
                         int32_t out_dtype, void* ws, size_t ws_bytes, hipStream_t st) {
    SDT_REQUIRE(blk, SDT_ERR_INVALID_ARG, "sdt_gat_aggregate_fwd: null block");
    SDT_REQUIRE(F >= 0 && ldz >= F && ldo >= F && blk->cap_src >= blk->cap_dst, SDT_ERR_INVALID_ARG,
                "sdt_gat_aggregate_fwd: bad sizes");
    SDT_REQUIRE(types_ok(z_dtype, out_dtype), SDT_ERR_INVALID_ARG, "sdt_gat_aggregate_fwd: storage types %d -> %d", z_dtype,
                out_dtype);
    if (blk->cap_dst == 0 || F == 0) return SDT_OK;
    SDT_REQUIRE(blk->counts && blk->indptr && blk->cols && z && a_src && a_dst && out, SDT_ERR_INVALID_ARG,
                "sdt_gat_aggregate_fwd: null pointer");
    const GatWs w = gat_ws(ws, blk->cap_src, blk->cap_dst, F);
    SDT_REQUIRE(ws && ws_bytes >= w.total && aligned16(ws), SDT_ERR_WORKSPACE,
                "sdt_gat_aggregate_fwd: workspace of %zu bytes needed, %zu given", w.total, ws_bytes);
    if (z_dtype == SDT_F32)
        return forward_t(blk, static_cast<const float*>(z), ldz, F, a_src, a_dst, slope, bias, relu, static_cast<float*>(out), ldo, w,
                         st);
    if (out_dtype == SDT_F32)
        return forward_t(blk, static_cast<const bf16_t*>(z), ldz, F, a_src, a_dst, slope, bias, relu, static_cast<float*>(out), ldo,
                         w, st);
    return forward_t(blk, static_cast<const bf16_t*>(z), ldz, F, a_src, a_dst, slope, bias, relu, static_cast<bf16_t*>(out), ldo, w,
                     st);
}

extern "C" int32_t sdt_gat_aggregate_bwd(const sdt_block* blk, const void* z, int64_t ldz, int32_t F, int32_t dtype,
                                         const float* a_src, const float* a_dst, float slope, const void* g, int64_t ldg,
                                         void* dz, int64_t lddz, float* da_src, float* da_dst, void* ws, size_t ws_bytes,
                                         void* stream) {
    SDT_REQUIRE(da_src && da_dst, SDT_ERR_INVALID_ARG, "sdt_gat_aggregate_bwd: null attention-vector gradient");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const float* part = nullptr;
    int32_t n_part = 0;
    const int32_t rc = gat_backward(blk, z, ldz, F, dtype, a_src, a_dst, slope, g, ldg, dtype, dz, lddz, ws, ws_bytes, &part,
                                    &n_part, st);
    if (rc != SDT_OK || !part) return rc;
    hipLaunchKernelGGL(k_gat_vec_final, dim3(ceil_div(F, TB)), dim3(TB), 0, st, part, n_part, F, da_src, da_dst);
    SDT_CHECK_LAUNCH("gat attention-vector reduction");
    return SDT_OK;
}

int32_t sdt::gat_backward(const sdt_block* blk, const void* z, int64_t ldz, int32_t F, int32_t z_dtype, const float* a_src,
                          const float* a_dst, float slope, const void* g, int64_t ldg, int32_t g_dtype, void* dz, int64_t lddz,
                          void* ws, size_t ws_bytes, const float** part, int32_t* n_part, hipStream_t st) {
    *part = nullptr;
    *n_part = 0;
    SDT_REQUIRE(blk, SDT_ERR_INVALID_ARG, "sdt_gat_aggregate_bwd: null block");
    SDT_REQUIRE(F >= 0 && ldz >= F && ldg >= F && lddz >= F && blk->cap_src >= blk->cap_dst, SDT_ERR_INVALID_ARG,
                "sdt_gat_aggregate_bwd: bad sizes");
    SDT_REQUIRE(types_ok(z_dtype, g_dtype), SDT_ERR_INVALID_ARG, "sdt_gat_aggregate_bwd: storage types %d, %d", z_dtype, g_dtype);
    if (blk->cap_src == 0 || F == 0) return SDT_OK;
    SDT_REQUIRE(blk->counts && blk->indptr && blk->cols && blk->t_indptr && blk->t_rows && z && a_src && a_dst && g && dz,
                SDT_ERR_INVALID_ARG, "sdt_gat_aggregate_bwd: null pointer (the block needs its transposed arrays)");
    const GatWs w = gat_ws(ws, blk->cap_src, blk->cap_dst, F);
    SDT_REQUIRE(ws && ws_bytes >= w.total && aligned16(ws), SDT_ERR_WORKSPACE,
                "sdt_gat_aggregate_bwd: workspace of %zu bytes needed, %zu given", w.total, ws_bytes);
    int32_t rc;
    if (z_dtype == SDT_F32)
        rc = backward_t(blk, static_cast<const float*>(z), ldz, F, a_src, a_dst, slope, static_cast<const float*>(g), ldg,
                        static_cast<float*>(dz), lddz, w, st);
    else if (g_dtype == SDT_F32)
        rc = backward_t(blk, static_cast<const bf16_t*>(z), ldz, F, a_src, a_dst, slope, static_cast<const float*>(g), ldg,
                        static_cast<bf16_t*>(dz), lddz, w, st);
    else
        rc = backward_t(blk, static_cast<const bf16_t*>(z), ldz, F, a_src, a_dst, slope, static_cast<const bf16_t*>(g), ldg,
                        static_cast<bf16_t*>(dz), lddz, w, st);
    if (rc != SDT_OK) return rc;
    *part = w.part;
    *n_part = w.nblk;
    return SDT_OK;
}

int32_t sdt::gat_mask_bias(const sdt_block* blk, void* g, int64_t ldg, const void* Y, int64_t ldy, int32_t F, int32_t dtype,
                           void* ws, size_t ws_bytes, const float** Qb, int32_t* n_chunks, hipStream_t st) {
    SDT_REQUIRE(blk && blk->counts && g && F > 0 && ldg >= F && (!Y || ldy >= F) && dtype_ok(dtype), SDT_ERR_INVALID_ARG,
                "gat_mask_bias: bad arguments");
    const GatWs w = gat_ws(ws, blk->cap_src, blk->cap_dst, F);
    SDT_REQUIRE(ws && ws_bytes >= w.total && aligned16(ws), SDT_ERR_WORKSPACE, "gat_mask_bias: workspace of %zu bytes needed, %zu given",
                w.total, ws_bytes);
    const int32_t rc = dtype == SDT_F32
                           ? mask_bias_t(blk, static_cast<float*>(g), ldg, static_cast<const float*>(Y), ldy, F, w, st)
                           : mask_bias_t(blk, static_cast<bf16_t*>(g), ldg, static_cast<const bf16_t*>(Y), ldy, F, w, st);
    if (rc != SDT_OK) return rc;
    *Qb = w.biasq;
    *n_chunks = w.nchunk;
    return SDT_OK;
}
