// GraphSAGE projection on the gfx950 matrix cores: forward
// Y = act([Hself | A] W + b) and backward (dW, db, dSelf, dAgg).
//
// All three products run on v_mfma_f32_32x32x2_f32 with fp32 accumulation.
// A workgroup of four wavefronts owns a BM x BN output tile and walks the
// reduction dimension in steps of BK through LDS; the next step's global
// loads are issued before the current step's MFMAs so they overlap.  The
// concatenation [Hself | A] is never materialised: the reduction loop simply
// switches source pointer (forward) or the grid's z index picks the half
// (backward).  An operand whose reduction index is contiguous in memory is
// staged as [rows][BK+4] and read back 16 bytes per lane (the k index inside
// an 8-wide chunk is permuted identically for both operands, which a sum
// does not notice); an operand contiguous along the output index is staged as
// [BK][cols+4] and read one dword per lane, bank-conflict free either way.
// dW reduces over the rows of the batch: the rows are split over the grid and
// the partial products are summed in a fixed order by a second kernel, so the
// result is deterministic.
#include "common.h"

namespace sdt {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int TB = 256;

// ---- global -> register -> LDS staging of an [R][C] tile, C contiguous in memory ----
template <typename T, int R, int C, int V, bool ROUND>
struct Stage {
    static constexpr int VPR = C / V;
    static constexpr int TOTAL = R * VPR;
    static constexpr int PER = (TOTAL + TB - 1) / TB;
    float v[PER][V];

    // rows [r_lo, r_lo+R) x cols [c_lo, c_lo+C) of `base`; zero outside [0,rmax) x [0,cmax).
    __device__ __forceinline__ void load(const T* __restrict__ base, int64_t ld, int r_lo, int rmax, int c_lo, int cmax,
                                         const T* __restrict__ mask, int64_t ldmask) {
#pragma unroll
        for (int p = 0; p < PER; ++p) {
            const int idx = threadIdx.x + p * TB;
            const int r = r_lo + idx / VPR, c = c_lo + (idx % VPR) * V;
            const bool ok = (TOTAL % TB == 0 || idx < TOTAL) && r < rmax && c < cmax;
            if (ok) {
                const T* src = base + (int64_t)r * ld + c;
                if constexpr (V * sizeof(T) == 16) {
                    uint4 raw = *reinterpret_cast<const uint4*>(src);
                    unpack(reinterpret_cast<const T*>(&raw), v[p]);
                } else if constexpr (V * sizeof(T) == 8) {
                    uint2 raw = *reinterpret_cast<const uint2*>(src);
                    unpack(reinterpret_cast<const T*>(&raw), v[p]);
                } else if constexpr (V * sizeof(T) == 4) {
                    uint32_t raw = *reinterpret_cast<const uint32_t*>(src);
                    unpack(reinterpret_cast<const T*>(&raw), v[p]);
                } else {
                    unpack(src, v[p]);
                }
                if (mask) {
                    const T* ms = mask + (int64_t)r * ldmask + c;
#pragma unroll
                    for (int q = 0; q < V; ++q)
                        if (!(to_f32<T>(ms[q]) > 0.f)) v[p][q] = 0.f;
                }
            } else {
#pragma unroll
                for (int q = 0; q < V; ++q) v[p][q] = 0.f;
            }
        }
    }
    __device__ __forceinline__ static void unpack(const T* s, float out[V]) {
#pragma unroll
        for (int q = 0; q < V; ++q) {
            float f = to_f32<T>(s[q]);
            if constexpr (ROUND) f = bf16_to_f32(f32_to_bf16(f));
            out[q] = f;
        }
    }
    // into lds[R][LD]
    template <int LD>
    __device__ __forceinline__ void store(float* lds) const {
#pragma unroll
        for (int p = 0; p < PER; ++p) {
            const int idx = threadIdx.x + p * TB;
            if (TOTAL % TB == 0 || idx < TOTAL) {
                float* d = lds + (idx / VPR) * LD + (idx % VPR) * V;
                if constexpr (V % 4 == 0) {
#pragma unroll
                    for (int q = 0; q < V; q += 4)
                        *reinterpret_cast<float4*>(d + q) = make_float4(v[p][q], v[p][q + 1], v[p][q + 2], v[p][q + 3]);
                } else if constexpr (V == 2) {
                    *reinterpret_cast<float2*>(d) = make_float2(v[p][0], v[p][1]);
                } else {
                    d[0] = v[p][0];
                }
            }
        }
    }
};


// One BK-deep step of the wave's (TM*32) x (TN*32) tile.
//  A_KC: As is [BM][LD_KC] else [BK][LDA_OC];  B_KC likewise for Bs.
template <int BK, int TM, int TN, bool A_KC, bool B_KC, int LDA_OC, int LDB_OC>
__device__ __forceinline__ void mma_step(const float* As, const float* Bs, int arow0, int bcol0,
                                         floatx16 (&acc)[TM][TN]) {
    constexpr int LD_KC = BK + 4;  // LDS row stride of a k-contiguous operand tile
    const int lane = threadIdx.x & 63, i = lane & 31, kh = lane >> 5;
#pragma unroll
    for (int c = 0; c < BK / 8; ++c) {
        float a[TM][4], b[TN][4];
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            if constexpr (A_KC) {
                const float4 t = *reinterpret_cast<const float4*>(As + (arow0 + tm * 32 + i) * LD_KC + c * 8 + kh * 4);
                a[tm][0] = t.x; a[tm][1] = t.y; a[tm][2] = t.z; a[tm][3] = t.w;
            } else {
#pragma unroll
                for (int s = 0; s < 4; ++s) a[tm][s] = As[(c * 8 + kh * 4 + s) * LDA_OC + arow0 + tm * 32 + i];
            }
        }
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            if constexpr (B_KC) {
                const float4 t = *reinterpret_cast<const float4*>(Bs + (bcol0 + tn * 32 + i) * LD_KC + c * 8 + kh * 4);
                b[tn][0] = t.x; b[tn][1] = t.y; b[tn][2] = t.z; b[tn][3] = t.w;
            } else {
#pragma unroll
                for (int s = 0; s < 4; ++s) b[tn][s] = Bs[(c * 8 + kh * 4 + s) * LDB_OC + bcol0 + tn * 32 + i];
            }
        }
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[tm][s], b[tn][s], acc[tm][tn], 0, 0, 0);
    }
}

// Row/column of accumulator register r of a 32x32 MFMA tile held by `lane`.
__device__ __forceinline__ int acc_row(int r, int lane) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }
__device__ __forceinline__ int acc_col(int lane) { return lane & 31; }

template <int BM_, int BN_>
struct Tile {
    static constexpr int BM = BM_, BN = BN_;
    static constexpr int WM = 2, WN = 2;               // 2 x 2 wavefronts
    static constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    static constexpr int LDA_OC = BM + 4, LDB_OC = BN + 4;
    // depth of one reduction step, sized so that two LDS buffers of both operands fit in 64 KB
    static constexpr int BK = BM >= 128 ? 16 : 32;
    static constexpr int LD_KC = BK + 4;
};

__device__ __forceinline__ void zero_acc(floatx16& a) {
#pragma unroll
    for (int r = 0; r < 16; ++r) a[r] = 0.f;
}

// Software-pipelined reduction loop shared by the three products.  Global loads run two
// steps ahead of the MFMAs (two register stages), LDS is double-buffered, and one barrier
// per step suffices: a buffer is rewritten only after the barrier of the step in between,
// which every wave passes after it has finished reading that buffer.
//   fetch(it, sa, sb)  issues the global loads of step `it` into a register stage
//   hook(Bs)           optional extra work on the staged B tile (bias gradient)
template <typename TL, bool A_KC, bool B_KC, typename SA, typename SB, typename Fetch, typename Hook>
__device__ __forceinline__ void gemm_mainloop(int nit, float* As, float* Bs, Fetch&& fetch, Hook&& hook,
                                              floatx16 (&acc)[TL::TM][TL::TN]) {
    constexpr int BK = TL::BK;
    constexpr int LDA = A_KC ? TL::LD_KC : TL::LDA_OC, LDB = B_KC ? TL::LD_KC : TL::LDB_OC;
    constexpr int A_ELEMS = (A_KC ? TL::BM : BK) * LDA, B_ELEMS = (B_KC ? TL::BN : BK) * LDB;
    const int wave = threadIdx.x >> 6, wm = wave / TL::WN, wn = wave % TL::WN;
    const int a0 = wm * (TL::BM / TL::WM), b0 = wn * (TL::BN / TL::WN);
    SA sa0, sa1;
    SB sb0, sb1;
    if (nit > 0) fetch(0, sa0, sb0);
    if (nit > 1) fetch(1, sa1, sb1);
    for (int it = 0; it < nit; it += 2) {
        sa0.template store<LDA>(As);
        sb0.template store<LDB>(Bs);
        __syncthreads();
        if (it + 2 < nit) fetch(it + 2, sa0, sb0);
        hook(Bs);
        mma_step<BK, TL::TM, TL::TN, A_KC, B_KC, TL::LDA_OC, TL::LDB_OC>(As, Bs, a0, b0, acc);
        if (it + 1 < nit) {
            sa1.template store<LDA>(As + A_ELEMS);
            sb1.template store<LDB>(Bs + B_ELEMS);
            __syncthreads();
            if (it + 3 < nit) fetch(it + 3, sa1, sb1);
            hook(Bs + B_ELEMS);
            mma_step<BK, TL::TM, TL::TN, A_KC, B_KC, TL::LDA_OC, TL::LDB_OC>(As + A_ELEMS, Bs + B_ELEMS, a0, b0, acc);
        }
    }
}

// Visit every accumulator element of the workgroup tile: f(row_in_tile, col_in_tile, value).
template <typename TL, typename F>
__device__ __forceinline__ void for_each_acc(const floatx16 (&acc)[TL::TM][TL::TN], F&& f) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave / TL::WN, wn = wave % TL::WN;
#pragma unroll
    for (int tm = 0; tm < TL::TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TL::TN; ++tn) {
            const int c = wn * (TL::BN / TL::WN) + tn * 32 + acc_col(lane);
#pragma unroll
            for (int r = 0; r < 16; ++r) f(wm * (TL::BM / TL::WM) + tm * 32 + acc_row(r, lane), c, acc[tm][tn][r]);
        }
}

// ---------------------------------------------------------------------------------
// forward: Y[n,out] = act(Hself[n,in] Wself[in,out] + A[n,in] Wneigh[in,out] + b)
// ---------------------------------------------------------------------------------
template <typename TH, typename TY, int BM, int BN, int VA, int VB, bool ROUNDW>
__global__ __launch_bounds__(TB) void k_linear_fwd(const TH* __restrict__ Hself, int64_t ldh,
                                                   const TH* __restrict__ Agg, int64_t lda, int n_cap,
                                                   const int32_t* n_d, int in, int out, const float* __restrict__ W,
                                                   const float* __restrict__ bias, int relu, TY* __restrict__ Y,
                                                   int64_t ldy) {
    using TL = Tile<BM, BN>;
    constexpr int BK = TL::BK;
    const int n = dev_count(n_cap, n_d);
    const int row0 = blockIdx.y * BM, col0 = blockIdx.x * BN;
    if (row0 >= n) return;
    __shared__ __align__(16) float As[2 * BM * TL::LD_KC];
    __shared__ __align__(16) float Bs[2 * BK * TL::LDB_OC];
    floatx16 acc[TL::TM][TL::TN];
#pragma unroll
    for (int a = 0; a < TL::TM; ++a)
#pragma unroll
        for (int b = 0; b < TL::TN; ++b) zero_acc(acc[a][b]);
    using SA = Stage<TH, BM, BK, VA, false>;
    using SB = Stage<float, BK, BN, VB, ROUNDW>;
    const int nk = (in + BK - 1) / BK;
    auto fetch = [&](int it, SA& sa, SB& sb) {
        const int ph = it >= nk, k0 = (it - ph * nk) * BK;
        sa.load(ph ? Agg : Hself, ph ? lda : ldh, row0, n, k0, in, nullptr, 0);
        sb.load(W + (int64_t)ph * in * out, out, k0, in, col0, out, nullptr, 0);
    };
    gemm_mainloop<TL, true, false, SA, SB>(2 * nk, As, Bs, fetch, [](const float*) {}, acc);
    for_each_acc<TL>(acc, [&](int r, int c, float v) {
        const int row = row0 + r, col = col0 + c;
        if (row < n && col < out) {
            float z = v + (bias ? bias[col] : 0.f);
            if (relu && !(z > 0.f)) z = 0.f;
            Y[(int64_t)row * ldy + col] = from_f32<TY>(z);
        }
    });
}

// ---------------------------------------------------------------------------------
// input gradient: dIn_h[n,in] = dZ[n,out] W_h[in,out]^T, h = blockIdx.z (0 self, 1 neigh)
// ---------------------------------------------------------------------------------
template <typename TD, typename TH, int BM, int BN, int VD, int VW, bool ROUND>
__global__ __launch_bounds__(TB) void k_linear_bwd_input(const TD* __restrict__ dY, int64_t lddy,
                                                         const TD* __restrict__ Ymask, int64_t ldy, int n_cap,
                                                         const int32_t* n_d, int in, int out,
                                                         const float* __restrict__ W, TH* __restrict__ dSelf,
                                                         TH* __restrict__ dAgg, int64_t ldi) {
    using TL = Tile<BM, BN>;
    constexpr int BK = TL::BK;
    const int n = dev_count(n_cap, n_d);
    const int row0 = blockIdx.y * BM, col0 = blockIdx.x * BN, half = blockIdx.z;
    if (row0 >= n) return;
    __shared__ __align__(16) float As[2 * BM * TL::LD_KC];
    __shared__ __align__(16) float Bs[2 * BN * TL::LD_KC];
    floatx16 acc[TL::TM][TL::TN];
#pragma unroll
    for (int a = 0; a < TL::TM; ++a)
#pragma unroll
        for (int b = 0; b < TL::TN; ++b) zero_acc(acc[a][b]);
    using SA = Stage<TD, BM, BK, VD, ROUND && sizeof(TD) == 4>;
    using SB = Stage<float, BN, BK, VW, ROUND>;
    const float* Wh = W + (int64_t)half * in * out;
    auto fetch = [&](int it, SA& sa, SB& sb) {
        sa.load(dY, lddy, row0, n, it * BK, out, Ymask, ldy);
        sb.load(Wh, out, col0, in, it * BK, out, nullptr, 0);
    };
    gemm_mainloop<TL, true, true, SA, SB>((out + BK - 1) / BK, As, Bs, fetch, [](const float*) {}, acc);
    TH* dst = half ? dAgg : dSelf;
    for_each_acc<TL>(acc, [&](int r, int c, float v) {
        const int row = row0 + r, col = col0 + c;
        if (row < n && col < in) dst[(int64_t)row * ldi + col] = from_f32<TH>(v);
    });
}

// ---------------------------------------------------------------------------------
// weight gradient partials: P[s][h*in + m][o] = sum over the rows r of split s of
//   X_h[r, m] dZ[r, o],  X_0 = Hself, X_1 = A;  h = blockIdx.z % 2, s = blockIdx.z / 2
// ---------------------------------------------------------------------------------
template <typename TD, typename TH, int BM, int BN, int VH, int VD, bool ROUND>
__global__ __launch_bounds__(TB) void k_linear_bwd_weight(const TH* __restrict__ Hself, int64_t ldh,
                                                          const TH* __restrict__ Agg, int64_t lda,
                                                          const TD* __restrict__ dY, int64_t lddy,
                                                          const TD* __restrict__ Ymask, int64_t ldy, int n_cap,
                                                          const int32_t* n_d, int in, int out, int splits,
                                                          float* __restrict__ P, float* __restrict__ Q) {
    using TL = Tile<BM, BN>;
    constexpr int BK = TL::BK;
    const int n = dev_count(n_cap, n_d);
    const int half = blockIdx.z & 1, split = blockIdx.z >> 1;
    // the first row-tile of the self half also sums the columns of its dZ tiles (bias gradient)
    const bool do_bias = Q != nullptr && half == 0 && blockIdx.y == 0;
    float bsum = 0.f;
    const int row0 = blockIdx.y * BM /* feature m */, col0 = blockIdx.x * BN /* output o */;
    const int chunk = ((n + splits - 1) / splits + BK - 1) / BK * BK;
    const int r_begin = split * chunk, r_end = min(n, r_begin + chunk);
    __shared__ __align__(16) float As[2 * BK * TL::LDA_OC];
    __shared__ __align__(16) float Bs[2 * BK * TL::LDB_OC];
    floatx16 acc[TL::TM][TL::TN];
#pragma unroll
    for (int a = 0; a < TL::TM; ++a)
#pragma unroll
        for (int b = 0; b < TL::TN; ++b) zero_acc(acc[a][b]);
    using SA = Stage<TH, BK, BM, VH, false>;
    using SB = Stage<TD, BK, BN, VD, ROUND && sizeof(TD) == 4>;
    const TH* X = half ? Agg : Hself;
    const int64_t ldx = half ? lda : ldh;
    const int nit = r_end > r_begin ? (r_end - r_begin + BK - 1) / BK : 0;
    auto fetch = [&](int it, SA& sa, SB& sb) {
        sa.load(X, ldx, r_begin + it * BK, r_end, row0, in, nullptr, 0);
        sb.load(dY, lddy, r_begin + it * BK, r_end, col0, out, Ymask, ldy);
    };
    auto hook = [&](const float* Bcur) {
        if (do_bias && (int)threadIdx.x < BN) {
#pragma unroll 8
            for (int k = 0; k < BK; ++k) bsum += Bcur[k * TL::LDB_OC + threadIdx.x];
        }
    };
    gemm_mainloop<TL, false, false, SA, SB>(nit, As, Bs, fetch, hook, acc);
    if (do_bias && (int)threadIdx.x < BN && col0 + (int)threadIdx.x < out)
        Q[(int64_t)split * out + col0 + threadIdx.x] = bsum;
    float* dst = P + ((int64_t)split * 2 * in + (int64_t)half * in) * out;
    for_each_acc<TL>(acc, [&](int r, int c, float v) {
        const int row = row0 + r, col = col0 + c;
        if (row < in && col < out) dst[(int64_t)row * out + col] = v;
    });
}

// dW[idx] = sum_s P[s][idx]; db[o] = sum_s Q[s][o]; optionally the SGD step W -= lr dW,
// b -= lr db in the same pass, and (one extra workgroup) the mean of the per-seed losses.
// A workgroup covers 64 consecutive elements with 4 threads each: thread g adds the partials
// g, g+4, g+8, ... and the four sums are combined in the order 0,1,2,3 -- a fixed order, so
// the result is deterministic, with four times as many loads in flight as one thread per element.
__global__ __launch_bounds__(TB) void k_reduce_partials(const float* __restrict__ P, const float* __restrict__ Q,
                                                        int splits, int64_t n_w, int out, float* __restrict__ dW,
                                                        float* __restrict__ db, float* W_upd, float* b_upd, float lr,
                                                        const float* __restrict__ row_loss, int n_loss,
                                                        float* loss_out) {
    __shared__ float part[TB];
    if (loss_out && blockIdx.x == gridDim.x - 1) {  // the extra last block: mean loss in a fixed order
        float s = 0.f;
        for (int i = threadIdx.x; i < n_loss; i += TB) s += row_loss[i];
        part[threadIdx.x] = s;
        __syncthreads();
        for (int o = TB / 2; o > 0; o >>= 1) {
            if ((int)threadIdx.x < o) part[threadIdx.x] += part[threadIdx.x + o];
            __syncthreads();
        }
        if (threadIdx.x == 0) *loss_out = part[0] / (float)n_loss;
        return;
    }
    const int e = threadIdx.x & 63, g = threadIdx.x >> 6;
    const int64_t idx = (int64_t)blockIdx.x * 64 + e;
    const bool is_w = idx < n_w, is_b = !is_w && idx < n_w + out;
    const float* src = is_w ? P + idx : Q + (idx - n_w);
    const int64_t stride = is_w ? n_w : out;
    float s = 0.f;
    if (is_w || is_b) {
#pragma unroll 4
        for (int k = g; k < splits; k += 4) s += src[(int64_t)k * stride];
    }
    part[threadIdx.x] = s;
    __syncthreads();
    if (g == 0 && (is_w || is_b)) {
        const float t = ((part[e] + part[64 + e]) + part[128 + e]) + part[192 + e];
        if (is_w) {
            dW[idx] = t;
            if (W_upd) W_upd[idx] = W_upd[idx] - lr * t;
        } else {
            const int o = (int)(idx - n_w);
            db[o] = t;
            if (b_upd) b_upd[o] = b_upd[o] - lr * t;
        }
    }
}

// widest vector (elements, <= 16 bytes) usable for rows of `width` elements
int vec_elems(size_t es, int width, std::initializer_list<int64_t> lds, std::initializer_list<const void*> ptrs) {
    int vb = 16;
    auto fit = [&](uint64_t x) {
        while (vb > (int)es && (x % vb) != 0) vb >>= 1;
    };
    fit((uint64_t)width * es);
    for (int64_t ld : lds) fit((uint64_t)ld * es);
    for (const void* p : ptrs) fit(reinterpret_cast<uintptr_t>(p));
    int v = vb / (int)es;
    return v > 4 && es == 4 ? 4 : v;
}

int weight_splits(int n_cap, int in, int out, int BM, int BN) {
    const int tiles = ceil_div(in, BM) * ceil_div(out, BN) * 2;
    int s = ceil_div(256, tiles);  // about one workgroup per CU
    const int max_s = ceil_div(n_cap > 0 ? n_cap : 1, 256);
    if (s > max_s) s = max_s;
    if (s < 1) s = 1;
    return s;
}

}  // namespace
}  // namespace sdt

using namespace sdt;

// Instantiate a kernel for a runtime vector width (elements of a 4- or 2-byte type).
#define SDT_VEC_SWITCH(v, MAXV, body)                           \
    switch (v) {                                                \
        case 8: if constexpr (MAXV >= 8) { constexpr int V = 8; body; } break; \
        case 4: { constexpr int V = 4; body; } break;           \
        case 2: { constexpr int V = 2; body; } break;           \
        default: { constexpr int V = 1; body; } break;          \
    }

namespace {

template <typename TH, typename TY, int BM, int BN>
void launch_fwd(const void* Hself, int64_t ldh, const void* A, int64_t lda, int n_cap, const int32_t* n_d, int in,
                int out, const float* W, const float* b, int relu, void* Y, int64_t ldy, bool roundw, hipStream_t st) {
    const int va = vec_elems(sizeof(TH), in, {ldh, lda}, {Hself, A});
    const int vb = vec_elems(4, out, {(int64_t)out}, {W});
    dim3 grid(ceil_div(out, BN), ceil_div(n_cap, BM));
    SDT_VEC_SWITCH(va, (16 / sizeof(TH)), {
        constexpr int VA = V;
        SDT_VEC_SWITCH(vb, 4, {
            constexpr int VB = V;
            if (roundw)
                hipLaunchKernelGGL((k_linear_fwd<TH, TY, BM, BN, VA, VB, true>), grid, dim3(TB), 0, st,
                                   static_cast<const TH*>(Hself), ldh, static_cast<const TH*>(A), lda, n_cap, n_d, in,
                                   out, W, b, relu, static_cast<TY*>(Y), ldy);
            else
                hipLaunchKernelGGL((k_linear_fwd<TH, TY, BM, BN, VA, VB, false>), grid, dim3(TB), 0, st,
                                   static_cast<const TH*>(Hself), ldh, static_cast<const TH*>(A), lda, n_cap, n_d, in,
                                   out, W, b, relu, static_cast<TY*>(Y), ldy);
        })
    })
}

template <typename TD, typename TH, int BM, int BN>
void launch_bwd(const void* dY, int64_t lddy, const void* Ymask, int64_t ldy, const void* Hself, int64_t ldh,
                const void* A, int64_t lda, int n_cap, const int32_t* n_d, int in, int out, const float* W, float* dW,
                float* db, void* dSelf, void* dAgg, int64_t ldi, float* P, float* Q, int splits, bool round,
                const BwdExtras& ex, hipStream_t st) {
    const int vd = vec_elems(sizeof(TD), out, {lddy, Ymask ? ldy : lddy}, {dY, Ymask});
    const int vh = vec_elems(sizeof(TH), in, {ldh, lda}, {Hself, A});
    const int vw = vec_elems(4, out, {(int64_t)out}, {W});
    const TD* dYt = static_cast<const TD*>(dY);
    const TD* Ym = static_cast<const TD*>(Ymask);
    // weight gradient partials
    {
        dim3 grid(ceil_div(out, BN), ceil_div(in, BM), 2 * splits);
        SDT_VEC_SWITCH(vh, (16 / sizeof(TH)), {
            constexpr int VH = V;
            SDT_VEC_SWITCH(vd, (16 / sizeof(TD)), {
                constexpr int VD = V;
                if (round)
                    hipLaunchKernelGGL((k_linear_bwd_weight<TD, TH, BM, BN, VH, VD, true>), grid, dim3(TB), 0, st,
                                       static_cast<const TH*>(Hself), ldh, static_cast<const TH*>(A), lda, dYt, lddy,
                                       Ym, ldy, n_cap, n_d, in, out, splits, P, Q);
                else
                    hipLaunchKernelGGL((k_linear_bwd_weight<TD, TH, BM, BN, VH, VD, false>), grid, dim3(TB), 0, st,
                                       static_cast<const TH*>(Hself), ldh, static_cast<const TH*>(A), lda, dYt, lddy,
                                       Ym, ldy, n_cap, n_d, in, out, splits, P, Q);
            })
        })
    }
    if (dSelf) {
        dim3 grid(ceil_div(in, BN), ceil_div(n_cap, BM), 2);
        SDT_VEC_SWITCH(vd, (16 / sizeof(TD)), {
            constexpr int VD = V;
            SDT_VEC_SWITCH(vw, 4, {
                constexpr int VW = V;
                if (round)
                    hipLaunchKernelGGL((k_linear_bwd_input<TD, TH, BM, BN, VD, VW, true>), grid, dim3(TB), 0, st, dYt,
                                       lddy, Ym, ldy, n_cap, n_d, in, out, W, static_cast<TH*>(dSelf),
                                       static_cast<TH*>(dAgg), ldi);
                else
                    hipLaunchKernelGGL((k_linear_bwd_input<TD, TH, BM, BN, VD, VW, false>), grid, dim3(TB), 0, st, dYt,
                                       lddy, Ym, ldy, n_cap, n_d, in, out, W, static_cast<TH*>(dSelf),
                                       static_cast<TH*>(dAgg), ldi);
            })
        })
    }
    // after the input gradients: this pass may overwrite W with the SGD step
    const int64_t n_w = (int64_t)2 * in * out;
    hipLaunchKernelGGL(k_reduce_partials, dim3(ceil_div(n_w + out, 64) + (ex.loss_out ? 1 : 0)), dim3(TB), 0, st, P, Q,
                       splits, n_w, out, dW, db, ex.W_upd, ex.b_upd, ex.lr, ex.row_loss, ex.n_loss, ex.loss_out);
}

constexpr int FBM = 64, FBN = 64;  // tile of the mini-batch sized products

}  // namespace

extern "C" int32_t sdt_sage_linear_fwd(const void* Hself, int64_t ldh, const void* A, int64_t lda, int32_t n_cap,
                                       const int32_t* n_d, int32_t in, int32_t out, const float* W, const float* b,
                                       int32_t relu, int32_t dtype, void* Y, int64_t ldy, int32_t y_dtype,
                                       void* stream) {
    SDT_REQUIRE(dtype_ok(dtype) && dtype_ok(y_dtype), SDT_ERR_INVALID_ARG, "sdt_sage_linear_fwd: unknown dtype");
    SDT_REQUIRE(!(dtype == SDT_F32 && y_dtype == SDT_BF16), SDT_ERR_INVALID_ARG,
                "sdt_sage_linear_fwd: bf16 output needs bf16 inputs");
    SDT_REQUIRE(n_cap >= 0 && in > 0 && out > 0 && ldh >= in && lda >= in && ldy >= out, SDT_ERR_INVALID_ARG,
                "sdt_sage_linear_fwd: bad sizes n=%d in=%d out=%d", n_cap, in, out);
    if (n_cap == 0) return SDT_OK;
    SDT_REQUIRE(Hself && A && W && Y, SDT_ERR_INVALID_ARG, "sdt_sage_linear_fwd: null pointer");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool big = (int64_t)ceil_div(n_cap, 128) * ceil_div(out, 128) >= 512;
    if (dtype == SDT_F32) {
        if (big)
            launch_fwd<float, float, 128, 128>(Hself, ldh, A, lda, n_cap, n_d, in, out, W, b, relu, Y, ldy, false, st);
        else
            launch_fwd<float, float, FBM, FBN>(Hself, ldh, A, lda, n_cap, n_d, in, out, W, b, relu, Y, ldy, false, st);
    } else if (y_dtype == SDT_BF16) {
        launch_fwd<bf16_t, bf16_t, FBM, FBN>(Hself, ldh, A, lda, n_cap, n_d, in, out, W, b, relu, Y, ldy, true, st);
    } else {
        launch_fwd<bf16_t, float, FBM, FBN>(Hself, ldh, A, lda, n_cap, n_d, in, out, W, b, relu, Y, ldy, true, st);
    }
    SDT_CHECK_LAUNCH("linear_fwd");
    return SDT_OK;
}

extern "C" size_t sdt_linear_bwd_workspace_bytes(int32_t n_cap, int32_t in, int32_t out) {
    if (n_cap < 0 || in <= 0 || out <= 0) return 0;
    const int s = weight_splits(n_cap, in, out, FBM, FBN);
    return align_up((size_t)s * 2 * in * out * sizeof(float), 256) + align_up((size_t)s * out * sizeof(float), 256);
}

namespace sdt {
int32_t reduce_partials(const float* P, const float* Q, int32_t splits, int32_t in, int32_t out, float* dW, float* db,
                        const BwdExtras& ex, hipStream_t st) {
    const int64_t n_w = (int64_t)2 * in * out;
    hipLaunchKernelGGL(k_reduce_partials, dim3(ceil_div(n_w + out, 64) + (ex.loss_out ? 1 : 0)), dim3(TB), 0, st, P, Q,
                       splits, n_w, out, dW, db, ex.W_upd, ex.b_upd, ex.lr, ex.row_loss, ex.n_loss, ex.loss_out);
    SDT_CHECK_LAUNCH("reduce_partials");
    return SDT_OK;
}

int32_t linear_bwd(const void* dY, int64_t lddy, int32_t dy_dtype, const void* Y, int64_t ldy, int32_t relu,
                   const void* Hself, int64_t ldh, const void* A, int64_t lda, int32_t n_cap, const int32_t* n_d,
                   int32_t in, int32_t out, const float* W, int32_t dtype, float* dW, float* db, void* dSelf,
                   void* dAgg, int64_t ldi, void* ws, size_t ws_bytes, const BwdExtras& ex, hipStream_t st) {
    SDT_REQUIRE(dtype_ok(dtype) && dtype_ok(dy_dtype), SDT_ERR_INVALID_ARG, "sdt_sage_linear_bwd: unknown dtype");
    SDT_REQUIRE(!(dtype == SDT_F32 && dy_dtype == SDT_BF16), SDT_ERR_INVALID_ARG,
                "sdt_sage_linear_bwd: bf16 dY needs bf16 activations");
    SDT_REQUIRE(n_cap >= 0 && in > 0 && out > 0 && ldh >= in && lda >= in && lddy >= out, SDT_ERR_INVALID_ARG,
                "sdt_sage_linear_bwd: bad sizes n=%d in=%d out=%d", n_cap, in, out);
    SDT_REQUIRE(dY && Hself && A && W && dW && db, SDT_ERR_INVALID_ARG, "sdt_sage_linear_bwd: null pointer");
    SDT_REQUIRE((dSelf == nullptr) == (dAgg == nullptr) && (!dSelf || ldi >= in), SDT_ERR_INVALID_ARG,
                "sdt_sage_linear_bwd: pass both input gradients (ldi >= in) or neither");
    SDT_REQUIRE(!relu || (Y && ldy >= out && dy_dtype == dtype), SDT_ERR_INVALID_ARG,
                "sdt_sage_linear_bwd: relu needs Y in the dtype of dY");
    const size_t need = sdt_linear_bwd_workspace_bytes(n_cap, in, out);
    SDT_REQUIRE(ws && ws_bytes >= need && aligned16(ws), SDT_ERR_WORKSPACE,
                "sdt_sage_linear_bwd: workspace of %zu bytes needed, %zu given", need, ws_bytes);
    const int splits = weight_splits(n_cap, in, out, FBM, FBN);
    float* P = static_cast<float*>(ws);
    float* Q = reinterpret_cast<float*>(static_cast<char*>(ws) + align_up((size_t)splits * 2 * in * out * sizeof(float), 256));
    const void* Ym = relu ? Y : nullptr;
    if (dtype == SDT_F32)
        launch_bwd<float, float, FBM, FBN>(dY, lddy, Ym, ldy, Hself, ldh, A, lda, n_cap, n_d, in, out, W, dW, db, dSelf,
                                           dAgg, ldi, P, Q, splits, false, ex, st);
    else if (dy_dtype == SDT_F32)
        launch_bwd<float, bf16_t, FBM, FBN>(dY, lddy, Ym, ldy, Hself, ldh, A, lda, n_cap, n_d, in, out, W, dW, db,
                                            dSelf, dAgg, ldi, P, Q, splits, true, ex, st);
    else
        launch_bwd<bf16_t, bf16_t, FBM, FBN>(dY, lddy, Ym, ldy, Hself, ldh, A, lda, n_cap, n_d, in, out, W, dW, db,
                                             dSelf, dAgg, ldi, P, Q, splits, true, ex, st);
    SDT_CHECK_LAUNCH("linear_bwd");
    return SDT_OK;
}
}  // namespace sdt

extern "C" int32_t sdt_sage_linear_bwd(const void* dY, int64_t lddy, int32_t dy_dtype, const void* Y, int64_t ldy,
                                       int32_t relu, const void* Hself, int64_t ldh, const void* A, int64_t lda,
                                       int32_t n_cap, const int32_t* n_d, int32_t in, int32_t out, const float* W,
                                       int32_t dtype, float* dW, float* db, void* dSelf, void* dAgg, int64_t ldi,
                                       void* ws, size_t ws_bytes, void* stream) {
    return linear_bwd(dY, lddy, dy_dtype, Y, ldy, relu, Hself, ldh, A, lda, n_cap, n_d, in, out, W, dtype, dW, db,
                      dSelf, dAgg, ldi, ws, ws_bytes, BwdExtras{}, static_cast<hipStream_t>(stream));
}
