// Projection of bf16 activations on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16):
// forward Y = act([Hself | A] W + b) and the input gradients [dSelf | dAgg] = dZ W^T.
//
// The operands of a product enter rounded to bf16 and are accumulated in fp32, which is
// exactly what the widened fp32 path computes, at 16 times its matrix rate -- so these
// kernels are bound by streaming the activations once, not by arithmetic.
//
// A bf16 MFMA operand is eight consecutive reduction indices per lane.  Activations are
// stored with the reduction index contiguous already; the fp32 weights are not (forward)
// and must be rounded anyway, so one small pass per step writes two bf16 images of every
// weight matrix: Wt[out][2in] (transposed, for the forward) and Wb[2in][ldb] (straight, row
// stride padded to 8 with zeros, for the input gradient).  Both operands of both products
// then stage as plain 16-byte copies into LDS rows of BK+8 elements: 16 consecutive rows
// start in 16 different 16-byte bank groups, so the 16-byte fragment reads are conflict-free.
// The main loop is the one of the fp32 path: loads NS (two) steps ahead in as many register stages,
// nothing conditional, double-buffered LDS, one barrier per step.  (Four stages were measured on the
// 8-step reductions of the bf16 workload: 4 400 against 4 590 steps/s -- the short chains are not
// waiting for their loads.)
#include "common.h"

#include <type_traits>

namespace sdt {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <int BM_, int BN_, int BK_, int WM_, int WN_, int NS_ = 2>
struct TileB {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_, NS = NS_;   // NS: register stages of the prefetch
    static constexpr int NT = 64 * WM * WN;
    static constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    static constexpr int LDK = BK + 8;   // bf16 elements; (BK+8)*2/16 is odd for BK = 32, 64
    static constexpr int VPR = BK / 8;   // 16-byte vectors per tile row
    static_assert(TM >= 1 && TN >= 1 && (BK == 32 || BK == 64), "tile shape");
};

// ---- [R rows][BK] of a bf16 matrix whose reduction index is contiguous -------------------------
template <int R, int BK, int NT>
struct StageB {
    static constexpr int VPR = BK / 8, TOTAL = R * VPR, PER = (TOTAL + NT - 1) / NT, LDK = BK + 8;
    uint4 raw[PER];
    uint32_t ok;
    // rows [r_lo, r_lo+R) x k in [k_lo, k_lo+BK); zero outside [0,rmax) x [0,kmax).  kmax % 8 == 0,
    // kmax >= 8, rmax >= 1.  Loads are unconditional from clamped addresses (see linear.hip).
    __device__ __forceinline__ void load(const uint16_t* __restrict__ base, int64_t ld, int r_lo, int rmax, int k_lo,
                                         int kmax) {
        ok = 0;
#pragma unroll
        for (int p = 0; p < PER; ++p) {
            const int idx = threadIdx.x + p * NT;
            const int r = r_lo + idx / VPR, k = k_lo + (idx % VPR) * 8;
            if (r < rmax && k < kmax) ok |= 1u << p;
            const int rr = min(r, rmax - 1), kk = min(k, kmax - 8);
            raw[p] = *reinterpret_cast<const uint4*>(base + (int64_t)rr * ld + kk);
        }
    }
    __device__ __forceinline__ void store(uint16_t* lds) const {
#pragma unroll
        for (int p = 0; p < PER; ++p) {
            const int idx = threadIdx.x + p * NT;
            if (TOTAL % NT == 0 || idx < TOTAL) {
                const bool in = (ok >> p) & 1u;
                uint4 v = raw[p];
                if (!in) v = make_uint4(0u, 0u, 0u, 0u);
                *reinterpret_cast<uint4*>(lds + (idx / VPR) * LDK + (idx % VPR) * 8) = v;
            }
        }
    }
};

// ---- the same tile out of an fp32 matrix, rounded to bf16 on the way (two float4 per vector) ---
template <int R, int BK, int NT>
struct StageF {
    static constexpr int VPR = BK / 8, TOTAL = R * VPR, PER = (TOTAL + NT - 1) / NT, LDK = BK + 8;
    float4 raw[PER][2];
    uint32_t ok;  // two bits per vector
    // kmax % 4 == 0, kmax >= 4, rmax >= 1
    __device__ __forceinline__ void load(const float* __restrict__ base, int64_t ld, int r_lo, int rmax, int k_lo,
                                         int kmax) {
        ok = 0;
#pragma unroll
        for (int p = 0; p < PER; ++p) {
            const int idx = threadIdx.x + p * NT;
            const int r = r_lo + idx / VPR;
            const int rr = min(r, rmax - 1);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int k = k_lo + (idx % VPR) * 8 + 4 * h;
                if (r < rmax && k < kmax) ok |= 1u << (2 * p + h);
                raw[p][h] = *reinterpret_cast<const float4*>(base + (int64_t)rr * ld + min(k, kmax - 4));
            }
        }
    }
    __device__ __forceinline__ static uint32_t pack(float lo, float hi) {
        return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
    }
    __device__ __forceinline__ void store(uint16_t* lds) const {
#pragma unroll
        for (int p = 0; p < PER; ++p) {
            const int idx = threadIdx.x + p * NT;
            if (TOTAL % NT == 0 || idx < TOTAL) {
                const bool in0 = (ok >> (2 * p)) & 1u, in1 = (ok >> (2 * p + 1)) & 1u;
                const float4 a = raw[p][0], b = raw[p][1];
                uint4 v;
                v.x = in0 ? pack(a.x, a.y) : 0u;
                v.y = in0 ? pack(a.z, a.w) : 0u;
                v.z = in1 ? pack(b.x, b.y) : 0u;
                v.w = in1 ? pack(b.z, b.w) : 0u;
                *reinterpret_cast<uint4*>(lds + (idx / VPR) * LDK + (idx % VPR) * 8) = v;
            }
        }
    }
};

template <typename TL>
struct FragB {
    bf16x8 a[TL::TM], b[TL::TN];
    // chunk c covers 16 reduction indices: lanes 0-31 take the first eight, lanes 32-63 the rest.
    // Which eight a lane holds does not matter to the sum as long as both operands agree.
    __device__ __forceinline__ void load(const uint16_t* As, const uint16_t* Bs, int arow0, int bcol0, int c) {
        const int lane = threadIdx.x & 63, i = lane & 31, kg = lane >> 5;
#pragma unroll
        for (int tm = 0; tm < TL::TM; ++tm)
            a[tm] = *reinterpret_cast<const bf16x8*>(As + (arow0 + tm * 32 + i) * TL::LDK + c * 16 + kg * 8);
#pragma unroll
        for (int tn = 0; tn < TL::TN; ++tn)
            b[tn] = *reinterpret_cast<const bf16x8*>(Bs + (bcol0 + tn * 32 + i) * TL::LDK + c * 16 + kg * 8);
    }
    __device__ __forceinline__ void mma(floatx16 (&acc)[TL::TM][TL::TN]) const {
#pragma unroll
        for (int tm = 0; tm < TL::TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TL::TN; ++tn)
                acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[tm], b[tn], acc[tm][tn], 0, 0, 0);
    }
};

// Fragments out of tiles stored with the reduction index as the ROW ([BK][cols + 8], the layout the
// weight gradient's operands have in memory): a lane picks its eight values one 2-byte read at a
// time.  Rows 8 apart are 32 banks apart (row stride 36 dwords for 64 columns), so the two halves of
// a wave never collide; the 32 lanes of a half read 32 consecutive columns.
template <typename TL>
struct FragT {
    bf16x8 a[TL::TM], b[TL::TN];
    static constexpr int LDA = TL::BM + 8, LDB = TL::BN + 8;
    __device__ __forceinline__ static bf16x8 gather(const uint16_t* t, int ld, int r0, int col) {
        uint32_t w[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            w[j] = (uint32_t)t[(r0 + 2 * j) * ld + col] | ((uint32_t)t[(r0 + 2 * j + 1) * ld + col] << 16);
        return __builtin_bit_cast(bf16x8, make_uint4(w[0], w[1], w[2], w[3]));
    }
    __device__ __forceinline__ void load(const uint16_t* As, const uint16_t* Bs, int arow0, int bcol0, int c) {
        const int lane = threadIdx.x & 63, i = lane & 31, kg = lane >> 5;
#pragma unroll
        for (int tm = 0; tm < TL::TM; ++tm) a[tm] = gather(As, LDA, c * 16 + kg * 8, arow0 + tm * 32 + i);
#pragma unroll
        for (int tn = 0; tn < TL::TN; ++tn) b[tn] = gather(Bs, LDB, c * 16 + kg * 8, bcol0 + tn * 32 + i);
    }
    __device__ __forceinline__ void mma(floatx16 (&acc)[TL::TM][TL::TN]) const {
#pragma unroll
        for (int tm = 0; tm < TL::TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TL::TN; ++tn)
                acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[tm], b[tn], acc[tm][tn], 0, 0, 0);
    }
};

template <typename TL, typename FRAG = FragB<TL>>
__device__ __forceinline__ void mma_step(const uint16_t* As, const uint16_t* Bs, int a0, int b0,
                                         floatx16 (&acc)[TL::TM][TL::TN]) {
    constexpr int NC = TL::BK / 16;
    FRAG f[2];
    f[0].load(As, Bs, a0, b0, 0);
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        if (c + 1 < NC) f[(c + 1) & 1].load(As, Bs, a0, b0, c + 1);
        f[c & 1].mma(acc);
    }
}

// Requires nit >= 1; fetch(it, ...) must be callable for it up to nit + 2 (clamped loads, zero tiles).
template <typename TL, typename SA, typename SB, typename FRAG = FragB<TL>, int A_ELEMS = TL::BM * TL::LDK,
          int B_ELEMS = TL::BN * TL::LDK, typename Fetch, typename Hook>
__device__ __forceinline__ void mainloop(int nit, uint16_t* As, uint16_t* Bs, Fetch&& fetch, Hook&& hook,
                                         floatx16 (&acc)[TL::TM][TL::TN]) {
    const int wave = threadIdx.x >> 6, wm = wave / TL::WN, wn = wave % TL::WN;
    const int a0 = wm * (TL::BM / TL::WM), b0 = wn * (TL::BN / TL::WN);
    constexpr int NS = TL::NS;
    static_assert(NS % 2 == 0, "the LDS buffer of a stage is its index modulo two");
    SA sa[NS];
    SB sb[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        fetch(s, sa[s], sb[s]);
        __builtin_amdgcn_sched_barrier(0);
    }
    for (int it = 0; it < nit; it += NS) {
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const bool live = s < 2 || it + s < nit;   // (a dead second step of the last pair works on a zero tile, as before)
            if (live) {
                sa[s].store(As + (s & 1) * A_ELEMS);
                sb[s].store(Bs + (s & 1) * B_ELEMS);
                __syncthreads();
            }
            fetch(it + s + NS, sa[s], sb[s]);
            __builtin_amdgcn_sched_barrier(0);
            if (live) {
                hook(Bs + (s & 1) * B_ELEMS);
                mma_step<TL, FRAG>(As + (s & 1) * A_ELEMS, Bs + (s & 1) * B_ELEMS, a0, b0, acc);
            }
        }
    }
}

template <typename TL, typename F>
__device__ __forceinline__ void for_each_acc(const floatx16 (&acc)[TL::TM][TL::TN], F&& f) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave / TL::WN, wn = wave % TL::WN;
#pragma unroll
    for (int tm = 0; tm < TL::TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TL::TN; ++tn) {
            const int c = wn * (TL::BN / TL::WN) + tn * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r)
                f(wm * (TL::BM / TL::WM) + tm * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3), c, acc[tm][tn][r]);
        }
}

template <typename TL>
__device__ __forceinline__ void zero(floatx16 (&acc)[TL::TM][TL::TN]) {
#pragma unroll
    for (int a = 0; a < TL::TM; ++a)
#pragma unroll
        for (int b = 0; b < TL::TN; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
}

// The output tile of a workgroup, Y[row0.., col0..] = act(acc + bias) for rows < n and columns < ncols.  vec: the tile
// is staged through LDS (the operand buffers are dead by then; `lds` must hold tile_bytes<TY, TL>()) and leaves in
// 16-byte vectors, every row contiguous -- four stores per thread instead of one per accumulator element, which is
// 2-4 us of a short launch; it needs ldy a multiple of the vector and Y 16-byte aligned.  Otherwise element by element.
template <typename TY, typename TL>
constexpr int tile_bytes() { return TL::BM * (TL::BN + 16 / (int)sizeof(TY)) * (int)sizeof(TY); }

template <typename TY, typename TL>
__device__ __forceinline__ void store_tile(const floatx16 (&acc)[TL::TM][TL::TN], void* lds, TY* __restrict__ Y, int64_t ldy,
                                           int row0, int col0, int n, int ncols, const float* __restrict__ bias, int relu,
                                           bool vec) {
    if (!vec) {
        for_each_acc<TL>(acc, [&](int r, int c, float v) {
            const int row = row0 + r, col = col0 + c;
            if (row < n && col < ncols) {
                float z = v + (bias ? bias[col] : 0.f);
                if (relu && !(z > 0.f)) z = 0.f;
                Y[(int64_t)row * ldy + col] = from_f32<TY>(z);
            }
        });
        return;
    }
    constexpr int VE = 16 / (int)sizeof(TY), LDC = TL::BN + VE, VPR = TL::BN / VE;
    TY* Cs = static_cast<TY*>(lds);
    __syncthreads();   // every wave is done with the operand tiles
    for_each_acc<TL>(acc, [&](int r, int c, float v) {
        const int col = col0 + c;
        float z = v + ((bias && col < ncols) ? bias[col] : 0.f);
        if (relu && !(z > 0.f)) z = 0.f;
        Cs[r * LDC + c] = from_f32<TY>(z);
    });
    __syncthreads();
    for (int idx = threadIdx.x; idx < TL::BM * VPR; idx += TL::NT) {
        const int r = idx / VPR, c = (idx % VPR) * VE;
        const int row = row0 + r, col = col0 + c;
        if (row >= n) continue;
        if (col + VE <= ncols)
            *reinterpret_cast<uint4*>(Y + (int64_t)row * ldy + col) = *reinterpret_cast<const uint4*>(Cs + r * LDC + c);
        else
            for (int e = 0; e < VE && col + e < ncols; ++e) Y[(int64_t)row * ldy + col + e] = Cs[r * LDC + c + e];
    }
}
template <typename TY>
inline bool vec_rows_ok(const void* Y, int64_t ldy) {
    return ldy % (16 / (int64_t)sizeof(TY)) == 0 && reinterpret_cast<uintptr_t>(Y) % 16 == 0;
}

// ---- forward -------------------------------------------------------------------------------------
// Wt: bf16 [out][2 in], column o of W as a row (self half first).
template <typename TY, typename TL>
__global__ __launch_bounds__(TL::NT) void k_fwd_bf16(const uint16_t* __restrict__ Hself, int64_t ldh,
                                                     const uint16_t* __restrict__ Agg, int64_t lda, int n_cap,
                                                     const int32_t* n_d, int in, int out,
                                                     const uint16_t* __restrict__ Wt, const float* __restrict__ bias,
                                                     int relu, TY* __restrict__ Y, int64_t ldy, int vec) {
    constexpr int BM = TL::BM, BN = TL::BN, BK = TL::BK;
    const int n = dev_count(n_cap, n_d);
    const int id = xcd_contiguous_id((int)gridDim.x * ((n + BM - 1) / BM));
    if (id < 0) return;
    const int row0 = (id / (int)gridDim.x) * BM, col0 = (id % (int)gridDim.x) * BN;
    constexpr int AB = 2 * (BM + BN) * TL::LDK * 2;
    constexpr bool STAGED = tile_bytes<TY, TL>() <= AB;   // (an fp32 tile of 64 x 128 is larger than the operand buffers: not staged)
    __shared__ __align__(16) unsigned char lds[AB];
    uint16_t* As = reinterpret_cast<uint16_t*>(lds);   // [2][BM][LDK]
    uint16_t* Bs = As + 2 * BM * TL::LDK;              // [2][BN][LDK]
    floatx16 acc[TL::TM][TL::TN];
    zero<TL>(acc);
    using SA = StageB<BM, BK, TL::NT>;
    using SB = StageB<BN, BK, TL::NT>;
    const int nk = (in + BK - 1) / BK;
    auto fetch = [&](int it, SA& sa, SB& sb) {
        const int ph = it >= nk, k0 = (it - ph * nk) * BK;  // past the last step k0 >= in: zero tiles
        sa.load(ph ? Agg : Hself, ph ? lda : ldh, row0, n, k0, in);
        sb.load(Wt + (int64_t)ph * in, 2 * (int64_t)in, col0, out, k0, in);
    };
    mainloop<TL, SA, SB>(2 * nk, As, Bs, fetch, [](const uint16_t*) {}, acc);
    store_tile<TY, TL>(acc, lds, Y, ldy, row0, col0, n, out, bias, relu, STAGED && vec != 0);
}

// ---- input gradient --------------------------------------------------------------------------------
// dIn_h[n, in] = dZ[n, out] W_h^T.  Wb: bf16 [2 in][ldb], rows of W rounded; half h = rows h*in ...
// TD = uint16_t (bf16 dZ) or float (fp32 dZ, rounded on the way in).
template <typename TD, typename TL>
__device__ __forceinline__ void bwd_input_body(const TD* __restrict__ dY, int64_t lddy, int n_cap, const int32_t* n_d, int in,
                                               int out, const uint16_t* __restrict__ Wb, int64_t ldb,
                                               bf16_t* __restrict__ dSelf, bf16_t* __restrict__ dAgg, int64_t ldi,
                                               int vec, int lin_id, int gx, uint16_t* lds) {
    constexpr int BM = TL::BM, BN = TL::BN, BK = TL::BK;
    const int n = dev_count(n_cap, n_d);
    const int id = xcd_contiguous_from_linear(lin_id, gx * 2 * ((n + BM - 1) / BM));
    if (id < 0) return;
    const int col0 = (id % gx) * BN, half = (id / gx) % 2;
    const int row0 = (id / gx / 2) * BM;
    uint16_t* As = lds;                         // [2][BM][LDK]
    uint16_t* Bs = lds + 2 * BM * TL::LDK;      // [2][BN][LDK]
    floatx16 acc[TL::TM][TL::TN];
    zero<TL>(acc);
    using SA = typename std::conditional<sizeof(TD) == 2, StageB<BM, BK, TL::NT>, StageF<BM, BK, TL::NT>>::type;
    using SB = StageB<BN, BK, TL::NT>;
    const uint16_t* Wh = Wb + (int64_t)half * in * ldb;
    const int kmax_b = (int)ldb;  // the padding columns of Wb are zero
    auto fetch = [&](int it, SA& sa, SB& sb) {
        sa.load(dY, lddy, row0, n, it * BK, out);
        sb.load(Wh, ldb, col0, in, it * BK, kmax_b);
    };
    mainloop<TL, SA, SB>((out + BK - 1) / BK, As, Bs, fetch, [](const uint16_t*) {}, acc);
    static_assert(tile_bytes<bf16_t, TL>() <= 2 * (TL::BM + TL::BN) * TL::LDK * 2, "the staged output tile fits the operand buffers");
    store_tile<bf16_t, TL>(acc, lds, half ? dAgg : dSelf, ldi, row0, col0, n, in, nullptr, 0, vec != 0);
}
template <typename TL>
constexpr int input_lds_elems() { return 2 * (TL::BM + TL::BN) * TL::LDK; }

template <typename TD, typename TL>
__global__ __launch_bounds__(TL::NT) void k_bwd_input_bf16(const TD* __restrict__ dY, int64_t lddy, int n_cap,
                                                           const int32_t* n_d, int in, int out,
                                                           const uint16_t* __restrict__ Wb, int64_t ldb,
                                                           bf16_t* __restrict__ dSelf, bf16_t* __restrict__ dAgg,
                                                           int64_t ldi, int vec) {
    __shared__ __align__(16) uint16_t lds[input_lds_elems<TL>()];
    bwd_input_body<TD, TL>(dY, lddy, n_cap, n_d, in, out, Wb, ldb, dSelf, dAgg, ldi, vec,
                           (int)(blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z)), (int)gridDim.x, lds);
}

// ---- weight gradient partials ------------------------------------------------------------------
// [BK rows][C cols] of a matrix whose COLUMNS are contiguous (the reduction index is the row):
// stored to LDS as it is, rows of C + 8 elements.
template <int BK, int C, int NT>
struct StageRowsB {
    static constexpr int VPR = C / 8, TOTAL = BK * VPR, PER = (TOTAL + NT - 1) / NT, LD = C + 8;
    uint4 raw[PER];
    uint32_t ok;
    // cmax % 8 == 0, cmax >= 8, rmax >= 1
    __device__ __forceinline__ void load(const uint16_t* __restrict__ base, int64_t ld, int r_lo, int rmax, int c_lo,
                                         int cmax) {
        ok = 0;
#pragma unroll
        for (int p = 0; p < PER; ++p) {
            const int idx = threadIdx.x + p * NT;
            const int r = r_lo + idx / VPR, c = c_lo + (idx % VPR) * 8;
            if (r < rmax && c < cmax) ok |= 1u << p;
            raw[p] = *reinterpret_cast<const uint4*>(base + (int64_t)min(r, rmax - 1) * ld + min(c, cmax - 8));
        }
    }
    __device__ __forceinline__ void store(uint16_t* lds) const {
#pragma unroll
        for (int p = 0; p < PER; ++p) {
            const int idx = threadIdx.x + p * NT;
            if (TOTAL % NT == 0 || idx < TOTAL) {
                uint4 v = raw[p];
                if (!((ok >> p) & 1u)) v = make_uint4(0u, 0u, 0u, 0u);
                *reinterpret_cast<uint4*>(lds + (idx / VPR) * LD + (idx % VPR) * 8) = v;
            }
        }
    }
};
template <int BK, int C, int NT>
struct StageRowsF {  // fp32 source, rounded to bf16 on the way (cmax % 4 == 0, cmax >= 4)
    static constexpr int VPR = C / 8, TOTAL = BK * VPR, PER = (TOTAL + NT - 1) / NT, LD = C + 8;
    float4 raw[PER][2];
    uint32_t ok;
    __device__ __forceinline__ void load(const float* __restrict__ base, int64_t ld, int r_lo, int rmax, int c_lo,
                                         int cmax) {
        ok = 0;
#pragma unroll
        for (int p = 0; p < PER; ++p) {
            const int idx = threadIdx.x + p * NT;
            const int r = r_lo + idx / VPR;
            const int64_t row = (int64_t)min(r, rmax - 1) * ld;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int c = c_lo + (idx % VPR) * 8 + 4 * h;
                if (r < rmax && c < cmax) ok |= 1u << (2 * p + h);
                raw[p][h] = *reinterpret_cast<const float4*>(base + row + min(c, cmax - 4));
            }
        }
    }
    __device__ __forceinline__ void store(uint16_t* lds) const {
#pragma unroll
        for (int p = 0; p < PER; ++p) {
            const int idx = threadIdx.x + p * NT;
            if (TOTAL % NT == 0 || idx < TOTAL) {
                const bool in0 = (ok >> (2 * p)) & 1u, in1 = (ok >> (2 * p + 1)) & 1u;
                const float4 a = raw[p][0], b = raw[p][1];
                uint4 v;
                v.x = in0 ? StageF<8, 32, 64>::pack(a.x, a.y) : 0u;
                v.y = in0 ? StageF<8, 32, 64>::pack(a.z, a.w) : 0u;
                v.z = in1 ? StageF<8, 32, 64>::pack(b.x, b.y) : 0u;
                v.w = in1 ? StageF<8, 32, 64>::pack(b.z, b.w) : 0u;
                *reinterpret_cast<uint4*>(lds + (idx / VPR) * LD + (idx % VPR) * 8) = v;
            }
        }
    }
};

// P[s][h*in + m][o] = sum over the rows r of split s of X_h[r, m] dZ[r, o]  (X_0 = Hself, X_1 = A),
// Q[s][o] = column sums of (rounded) dZ; workgroups (gx out tiles, gy in tiles, 2 * splits) as in the fp32 path.
template <typename TD, typename TL>
__device__ __forceinline__ void bwd_weight_body(const uint16_t* __restrict__ Hself, int64_t ldh,
                                                const uint16_t* __restrict__ Agg, int64_t lda, const TD* __restrict__ dY,
                                                int64_t lddy, int n_cap, const int32_t* n_d, int in, int out, int splits,
                                                float* __restrict__ P, float* __restrict__ Q, int lin_id, int gx, int gy,
                                                uint16_t* lds) {
    constexpr int BM = TL::BM, BN = TL::BN, BK = TL::BK;
    constexpr int LDA = BM + 8, LDB = BN + 8;
    const int n = dev_count(n_cap, n_d);
    const int id = xcd_contiguous_from_linear(lin_id, gx * gy * 2 * splits);   // every tile carries work
    if (id < 0) return;
    const int bx = id % gx, by = (id / gx) % gy;
    const int bz = id / (gx * gy);
    const int half = bz & 1, split = bz >> 1;
    const bool do_bias = Q != nullptr && half == 0 && by == 0;
    float bsum = 0.f;
    const int row0 = by * BM /* feature m */, col0 = bx * BN /* output o */;
    const int chunk = ((n + splits - 1) / splits + BK - 1) / BK * BK;
    const int r_begin = split * chunk, r_end = min(n, r_begin + chunk);
    uint16_t* As = lds;                  // [2][BK][LDA]
    uint16_t* Bs = lds + 2 * BK * LDA;   // [2][BK][LDB]
    floatx16 acc[TL::TM][TL::TN];
    zero<TL>(acc);
    using SA = StageRowsB<BK, BM, TL::NT>;
    using SB = typename std::conditional<sizeof(TD) == 2, StageRowsB<BK, BN, TL::NT>, StageRowsF<BK, BN, TL::NT>>::type;
    const uint16_t* X = half ? Agg : Hself;
    const int64_t ldx = half ? lda : ldh;
    const int nit = r_end > r_begin ? (r_end - r_begin + BK - 1) / BK : 0;
    auto fetch = [&](int it, SA& sa, SB& sb) {
        sa.load(X, ldx, r_begin + it * BK, r_end, row0, in);
        sb.load(dY, lddy, r_begin + it * BK, r_end, col0, out);
    };
    auto hook = [&](const uint16_t* Bcur) {
        if (do_bias && (int)threadIdx.x < BN) {
#pragma unroll 8
            for (int k = 0; k < BK; ++k) bsum += bf16_to_f32(Bcur[k * LDB + threadIdx.x]);
        }
    };
    if (nit > 0) mainloop<TL, SA, SB, FragT<TL>, BK * LDA, BK * LDB>(nit, As, Bs, fetch, hook, acc);
    if (do_bias && (int)threadIdx.x < BN && col0 + (int)threadIdx.x < out)
        Q[(int64_t)split * out + col0 + threadIdx.x] = bsum;
    float* dst = P + ((int64_t)split * 2 * in + (int64_t)half * in) * out;
    for_each_acc<TL>(acc, [&](int r, int c, float v) {
        const int row = row0 + r, col = col0 + c;
        if (row < in && col < out) dst[(int64_t)row * out + col] = v;
    });
}
template <typename TL>
constexpr int weight_lds_elems() { return 2 * TL::BK * (TL::BM + 8 + TL::BN + 8); }

template <typename TD, typename TL>
__global__ __launch_bounds__(TL::NT) void k_bwd_weight_bf16(const uint16_t* __restrict__ Hself, int64_t ldh,
                                                            const uint16_t* __restrict__ Agg, int64_t lda,
                                                            const TD* __restrict__ dY, int64_t lddy, int n_cap,
                                                            const int32_t* n_d, int in, int out, int splits,
                                                            float* __restrict__ P, float* __restrict__ Q) {
    __shared__ __align__(16) uint16_t lds[weight_lds_elems<TL>()];
    bwd_weight_body<TD, TL>(Hself, ldh, Agg, lda, dY, lddy, n_cap, n_d, in, out, splits, P, Q,
                            (int)(blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z)), (int)gridDim.x,
                            (int)gridDim.y, lds);
}

// Both products of a layer's backward in one launch: the first nw workgroups (a multiple of eight, so that the
// linear id inside either part still tells the XCD) take the weight-gradient tiles, the rest the input-gradient
// tiles.  The two products are independent, read the same dY, and each alone fills a fraction of the chip.
template <typename TD, typename TW, typename TI>
__global__ __launch_bounds__(TW::NT) void k_bwd_both_bf16(const uint16_t* __restrict__ Hself, int64_t ldh,
                                                          const uint16_t* __restrict__ Agg, int64_t lda,
                                                          const TD* __restrict__ dY, int64_t lddy, int n_cap,
                                                          const int32_t* n_d, int in, int out, int splits,
                                                          float* __restrict__ P, float* __restrict__ Q, int nw, int wgx,
                                                          int wgy, const uint16_t* __restrict__ Wb, int64_t ldb,
                                                          bf16_t* __restrict__ dSelf, bf16_t* __restrict__ dAgg, int64_t ldi,
                                                          int vec, int igx) {
    static_assert(TW::NT == TI::NT, "one workgroup size for both parts");
    constexpr int LDS = weight_lds_elems<TW>() > input_lds_elems<TI>() ? weight_lds_elems<TW>() : input_lds_elems<TI>();
    __shared__ __align__(16) uint16_t lds[LDS];
    const int id = (int)blockIdx.x;
    if (id < nw)
        bwd_weight_body<TD, TW>(Hself, ldh, Agg, lda, dY, lddy, n_cap, n_d, in, out, splits, P, Q, id, wgx, wgy, lds);
    else
        bwd_input_body<TD, TI>(dY, lddy, n_cap, n_d, in, out, Wb, ldb, dSelf, dAgg, ldi, vec, id - nw, igx, lds);
}

// ---- bf16 images of the weights ----------------------------------------------------------------
struct ConvertArgs {
    int32_t n_layers;
    const float* W[SDT_MAX_LAYERS];
    uint16_t* Wt[SDT_MAX_LAYERS];
    uint16_t* Wb[SDT_MAX_LAYERS];
    int32_t k2[SDT_MAX_LAYERS];   // 2 * in
    int32_t out[SDT_MAX_LAYERS];
    int32_t ldb[SDT_MAX_LAYERS];
    int64_t first[SDT_MAX_LAYERS + 1];  // prefix sums of k2 * ldb
};

__global__ __launch_bounds__(256) void k_convert_weights(ConvertArgs a) {
    const int64_t total = a.first[a.n_layers];
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        int l = 0;
        while (l + 1 < a.n_layers && i >= a.first[l + 1]) ++l;
        const int64_t j = i - a.first[l];
        const int k = (int)(j / a.ldb[l]), o = (int)(j - (int64_t)k * a.ldb[l]);
        uint16_t v = 0;
        if (o < a.out[l]) {
            v = f32_to_bf16(a.W[l][(int64_t)k * a.out[l] + o]);
            a.Wt[l][(int64_t)o * a.k2[l] + k] = v;
        }
        a.Wb[l][j] = v;
    }
}

inline bool al16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

// ---- internal entry points (declared in common.h) ----------------------------------------------
int32_t bf16_ldb(int32_t out) { return (out + 7) / 8 * 8; }

size_t bf16_weights_bytes(int32_t in, int32_t out) {
    return align_up((size_t)2 * in * out * 2, 256) + align_up((size_t)2 * in * bf16_ldb(out) * 2, 256);
}

bool bf16_mfma_fwd_ok(const void* Hself, int64_t ldh, const void* A, int64_t lda, int32_t in) {
    return in % 8 == 0 && ldh % 8 == 0 && lda % 8 == 0 && al16(Hself) && al16(A);
}

bool bf16_mfma_bwd_input_ok(const void* dY, int64_t lddy, int32_t dy_dtype, int32_t in, int32_t out, int64_t ldi) {
    (void)in; (void)ldi;
    if (!al16(dY)) return false;
    return dy_dtype == SDT_BF16 ? (out % 8 == 0 && lddy % 8 == 0) : (out % 4 == 0 && lddy % 4 == 0);
}

int32_t convert_weights_bf16(const sdt_model* model, void* base, hipStream_t st) {
    ConvertArgs a{};
    a.n_layers = model->n_layers;
    char* p = static_cast<char*>(base);
    a.first[0] = 0;
    for (int l = 0; l < model->n_layers; ++l) {
        const int in = model->dims[l], out = model->dims[l + 1];
        a.W[l] = model->W[l];
        a.k2[l] = 2 * in;
        a.out[l] = out;
        a.ldb[l] = bf16_ldb(out);
        a.Wt[l] = reinterpret_cast<uint16_t*>(p);
        a.Wb[l] = reinterpret_cast<uint16_t*>(p + align_up((size_t)2 * in * out * 2, 256));
        p += bf16_weights_bytes(in, out);
        a.first[l + 1] = a.first[l] + (int64_t)a.k2[l] * a.ldb[l];
    }
    const int64_t total = a.first[a.n_layers];
    const int blocks = (int)((total + 255) / 256 < 2048 ? (total + 255) / 256 : 2048);
    hipLaunchKernelGGL(k_convert_weights, dim3(blocks > 0 ? blocks : 1), dim3(256), 0, st, a);
    SDT_CHECK_LAUNCH("convert_weights_bf16");
    return SDT_OK;
}

namespace {
// Many rows: 32-deep steps keep more workgroups resident (the kernels are bound by streaming the
// activations).  Few rows: every workgroup is one short dependent chain; 64-deep steps halve it, and 64 output
// columns per workgroup instead of 128 make twice as many, each with half the loads and matrix instructions per
// step (6 000 x 512 -> 256: 15.1 us with 64 x 128 tiles, 10.4 with 64 x 64, 9.3 with the output tile leaving in vectors).
using TFbig = TileB<64, 128, 32, 2, 2>;
using TFsmall = TileB<64, 64, 64, 2, 2>;
constexpr int32_t SMALL_ROWS = 16384;
}  // namespace

int32_t linear_fwd_bf16(const void* Hself, int64_t ldh, const void* A, int64_t lda, int32_t n_cap, const int32_t* n_d,
                        int32_t in, int32_t out, const void* Wt, const float* bias, int32_t relu, void* Y, int64_t ldy,
                        int32_t y_dtype, hipStream_t st) {
    if (n_cap == 0) return SDT_OK;
    const uint16_t* h = static_cast<const uint16_t*>(Hself);
    const uint16_t* a = static_cast<const uint16_t*>(A);
    const uint16_t* w = static_cast<const uint16_t*>(Wt);
    auto go = [&](auto tile) {
        using TF = decltype(tile);
        dim3 grid(ceil_div(out, TF::BN), ceil_div(n_cap, TF::BM));
        if (y_dtype == SDT_BF16)
            hipLaunchKernelGGL((k_fwd_bf16<bf16_t, TF>), grid, dim3(TF::NT), 0, st, h, ldh, a, lda, n_cap, n_d, in, out, w,
                               bias, relu, static_cast<bf16_t*>(Y), ldy, (int)vec_rows_ok<bf16_t>(Y, ldy));
        else
            hipLaunchKernelGGL((k_fwd_bf16<float, TF>), grid, dim3(TF::NT), 0, st, h, ldh, a, lda, n_cap, n_d, in, out, w,
                               bias, relu, static_cast<float*>(Y), ldy, (int)vec_rows_ok<float>(Y, ldy));
    };
    if (n_cap >= SMALL_ROWS) go(TFbig{});
    else go(TFsmall{});
    SDT_CHECK_LAUNCH("linear_fwd_bf16");
    return SDT_OK;
}

bool bf16_mfma_bwd_weight_ok(const void* Hself, int64_t ldh, const void* A, int64_t lda, const void* dY, int64_t lddy,
                             int32_t dy_dtype, int32_t in, int32_t out) {
    if (!(in % 8 == 0 && ldh % 8 == 0 && lda % 8 == 0 && al16(Hself) && al16(A) && al16(dY))) return false;
    return dy_dtype == SDT_BF16 ? (out % 8 == 0 && lddy % 8 == 0) : (out % 4 == 0 && lddy % 4 == 0);
}

int32_t bf16_weight_splits(int32_t n_cap, int32_t in, int32_t out) {
    const int tiles = ceil_div(in, 64) * ceil_div(out, 64) * 2;
    int s = ceil_div(1024, tiles);
    const int max_rows = ceil_div(n_cap > 0 ? n_cap : 1, 256);
    const int64_t max_bytes = ((int64_t)16 << 20) / ((int64_t)2 * in * out * 4);
    if (s > max_rows) s = max_rows;
    if (s > max_bytes) s = (int)max_bytes;
    return s < 1 ? 1 : s;
}

int32_t linear_bwd_weight_bf16(const void* Hself, int64_t ldh, const void* A, int64_t lda, const void* dY, int64_t lddy,
                               int32_t dy_dtype, int32_t n_cap, const int32_t* n_d, int32_t in, int32_t out,
                               int32_t splits, float* P, float* Q, hipStream_t st) {
    using TW = TileB<64, 64, 64, 2, 2>;
    dim3 grid(ceil_div(out, TW::BN), ceil_div(in, TW::BM), 2 * splits);
    const uint16_t* h = static_cast<const uint16_t*>(Hself);
    const uint16_t* a = static_cast<const uint16_t*>(A);
    if (dy_dtype == SDT_BF16)
        hipLaunchKernelGGL((k_bwd_weight_bf16<uint16_t, TW>), grid, dim3(TW::NT), 0, st, h, ldh, a, lda,
                           static_cast<const uint16_t*>(dY), lddy, n_cap, n_d, in, out, splits, P, Q);
    else
        hipLaunchKernelGGL((k_bwd_weight_bf16<float, TW>), grid, dim3(TW::NT), 0, st, h, ldh, a, lda,
                           static_cast<const float*>(dY), lddy, n_cap, n_d, in, out, splits, P, Q);
    SDT_CHECK_LAUNCH("linear_bwd_weight_bf16");
    return SDT_OK;
}

int32_t linear_bwd_both_bf16(const void* Hself, int64_t ldh, const void* A, int64_t lda, const void* dY, int64_t lddy,
                             int32_t dy_dtype, int32_t n_cap, const int32_t* n_d, int32_t in, int32_t out, int32_t splits,
                             float* P, float* Q, const void* Wb, void* dSelf, void* dAgg, int64_t ldi, hipStream_t st) {
    using TW = TileB<64, 64, 64, 2, 2>;
    const uint16_t* h = static_cast<const uint16_t*>(Hself);
    const uint16_t* a = static_cast<const uint16_t*>(A);
    const uint16_t* w = static_cast<const uint16_t*>(Wb);
    const int64_t ldb = bf16_ldb(out);
    const int wgx = ceil_div(out, TW::BN), wgy = ceil_div(in, TW::BM);
    const int nw = (wgx * wgy * 2 * splits + 7) / 8 * 8;
    const int vec = vec_rows_ok<bf16_t>(dSelf, ldi) && vec_rows_ok<bf16_t>(dAgg, ldi);
    auto go = [&](auto tile) {
        using TI = decltype(tile);
        const int igx = ceil_div(in, TI::BN);
        const int ni = igx * 2 * ceil_div(n_cap, TI::BM);
        if (dy_dtype == SDT_BF16)
            hipLaunchKernelGGL((k_bwd_both_bf16<uint16_t, TW, TI>), dim3(nw + ni), dim3(TW::NT), 0, st, h, ldh, a, lda,
                               static_cast<const uint16_t*>(dY), lddy, n_cap, n_d, in, out, splits, P, Q, nw, wgx, wgy, w, ldb,
                               static_cast<bf16_t*>(dSelf), static_cast<bf16_t*>(dAgg), ldi, vec, igx);
        else
            hipLaunchKernelGGL((k_bwd_both_bf16<float, TW, TI>), dim3(nw + ni), dim3(TW::NT), 0, st, h, ldh, a, lda,
                               static_cast<const float*>(dY), lddy, n_cap, n_d, in, out, splits, P, Q, nw, wgx, wgy, w, ldb,
                               static_cast<bf16_t*>(dSelf), static_cast<bf16_t*>(dAgg), ldi, vec, igx);
    };
    if (n_cap >= SMALL_ROWS) go(TFbig{});
    else go(TFsmall{});
    SDT_CHECK_LAUNCH("linear_bwd_both_bf16");
    return SDT_OK;
}

int32_t linear_bwd_input_bf16(const void* dY, int64_t lddy, int32_t dy_dtype, int32_t n_cap, const int32_t* n_d,
                              int32_t in, int32_t out, const void* Wb, void* dSelf, void* dAgg, int64_t ldi,
                              hipStream_t st) {
    if (n_cap == 0) return SDT_OK;
    const uint16_t* w = static_cast<const uint16_t*>(Wb);
    const int64_t ldb = bf16_ldb(out);
    const int vec = vec_rows_ok<bf16_t>(dSelf, ldi) && vec_rows_ok<bf16_t>(dAgg, ldi);
    auto go = [&](auto tile) {
        using TI = decltype(tile);
        dim3 grid(ceil_div(in, TI::BN), ceil_div(n_cap, TI::BM), 2);
        if (dy_dtype == SDT_BF16)
            hipLaunchKernelGGL((k_bwd_input_bf16<uint16_t, TI>), grid, dim3(TI::NT), 0, st, static_cast<const uint16_t*>(dY),
                               lddy, n_cap, n_d, in, out, w, ldb, static_cast<bf16_t*>(dSelf), static_cast<bf16_t*>(dAgg), ldi, vec);
        else
            hipLaunchKernelGGL((k_bwd_input_bf16<float, TI>), grid, dim3(TI::NT), 0, st, static_cast<const float*>(dY), lddy,
                               n_cap, n_d, in, out, w, ldb, static_cast<bf16_t*>(dSelf), static_cast<bf16_t*>(dAgg), ldi, vec);
    };
    if (n_cap >= SMALL_ROWS) go(TFbig{});
    else go(TFsmall{});
    SDT_CHECK_LAUNCH("linear_bwd_input_bf16");
    return SDT_OK;
}

}  // namespace sdt
