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

#include <atomic>

#include <algorithm>
#include <mutex>
#include <type_traits>

namespace sdt {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// ---- global -> register -> LDS staging of an [R][C] tile, C contiguous in memory ----
template <typename T, int R, int C, int V, bool ROUND, int TB>
struct Stage {
    static constexpr int VPR = C / V;
    static constexpr int TOTAL = R * VPR;
    static constexpr int PER = (TOTAL + TB - 1) / TB;
    static constexpr int NB = V * sizeof(T) / 4 > 0 ? V * sizeof(T) / 4 : 1;  // dwords per vector
    uint32_t raw[PER][NB];
    uint32_t ok;  // bit p: vector p lies inside the matrix

    // rows [r_lo, r_lo+R) x cols [c_lo, c_lo+C) of `base`; zero outside [0,rmax) x [0,cmax).
    // Needs rmax >= 1, cmax >= V and cmax % V == 0 (a caller whose rows are zero-padded to a multiple
    // of V passes the padded width).  Every load is issued unconditionally from a clamped (valid)
    // address and nothing touches the loaded registers until store(): with no branch and no early
    // use the compiler can count the loads in flight, so the wait before the LDS stores covers only
    // the oldest stage and the younger prefetches keep flying.  (One validity bit per ELEMENT was
    // measured: the extra integer work in the fetch costs the main loop 8%.)
    __device__ __forceinline__ void load(const T* __restrict__ base, int64_t ld, int r_lo, int rmax, int c_lo, int cmax) {
        ok = 0;
#pragma unroll
        for (int p = 0; p < PER; ++p) {
            const int idx = threadIdx.x + p * TB;
            const int r = r_lo + idx / VPR, c = c_lo + (idx % VPR) * V;
            if (r < rmax && c < cmax) ok |= 1u << p;
            const int rr = min(r, rmax - 1), cc = min(c, cmax - V);
            const T* src = base + (int64_t)rr * ld + cc;
            if constexpr (V * sizeof(T) == 16) {
                const uint4 t = *reinterpret_cast<const uint4*>(src);
                raw[p][0] = t.x; raw[p][1] = t.y; raw[p][2] = t.z; raw[p][3] = t.w;
            } else if constexpr (V * sizeof(T) == 8) {
                const uint2 t = *reinterpret_cast<const uint2*>(src);
                raw[p][0] = t.x; raw[p][1] = t.y;
            } else if constexpr (V * sizeof(T) == 4) {
                raw[p][0] = *reinterpret_cast<const uint32_t*>(src);
            } else {  // one bf16
                raw[p][0] = *reinterpret_cast<const uint16_t*>(src);
            }
        }
    }
    // element q of vector p as fp32 (zero if the vector is out of range)
    __device__ __forceinline__ float value(int p, int q) const {
        float f;
        if constexpr (sizeof(T) == 4) {
            f = __uint_as_float(raw[p][q]);
        } else {
            const uint32_t w = raw[p][q >> 1];
            f = bf16_to_f32((uint16_t)((q & 1) ? (w >> 16) : (w & 0xFFFFu)));
        }
        if constexpr (ROUND) f = bf16_to_f32(f32_to_bf16(f));
        return ((ok >> p) & 1u) ? f : 0.f;
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
                        *reinterpret_cast<float4*>(d + q) =
                            make_float4(value(p, q), value(p, q + 1), value(p, q + 2), value(p, q + 3));
                } else if constexpr (V == 2) {
                    *reinterpret_cast<float2*>(d) = make_float2(value(p, 0), value(p, 1));
                } else {
                    d[0] = value(p, 0);
                }
            }
        }
    }
};


// One BK-deep step of the wave's (TM*32) x (TN*32) tile.
//  A_KC: As is [BM][LD_KC] else [BK][LDA_OC];  B_KC likewise for Bs.
// The operand fragments of chunk c+1 are read from LDS before the MFMAs of chunk c are
// issued, so the LDS latency hides behind matrix work even with one wave per SIMD.
template <int BK, int TM, int TN, bool A_KC, bool B_KC, int LDA_OC, int LDB_OC>
struct Frag {
    float a[TM][4], b[TN][4];
    __device__ __forceinline__ void load(const float* As, const float* Bs, int arow0, int bcol0, int c) {
        constexpr int LD_KC = BK + 4;  // LDS row stride of a k-contiguous operand tile
        const int lane = threadIdx.x & 63, i = lane & 31, kh = lane >> 5;
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
    }
    __device__ __forceinline__ void mma(floatx16 (&acc)[TM][TN]) const {
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[tm][s], b[tn][s], acc[tm][tn], 0, 0, 0);
    }
};

template <int BK, int TM, int TN, bool A_KC, bool B_KC, int LDA_OC, int LDB_OC>
__device__ __forceinline__ void mma_step(const float* As, const float* Bs, int arow0, int bcol0,
                                         floatx16 (&acc)[TM][TN]) {
    constexpr int NC = BK / 8;
    Frag<BK, TM, TN, A_KC, B_KC, LDA_OC, LDB_OC> f[2];
    f[0].load(As, Bs, arow0, bcol0, 0);
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        if (c + 1 < NC) f[(c + 1) & 1].load(As, Bs, arow0, bcol0, c + 1);
        f[c & 1].mma(acc);
    }
}

// Row/column of accumulator register r of a 32x32 MFMA tile held by `lane`.
__device__ __forceinline__ int acc_row(int r, int lane) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }
__device__ __forceinline__ int acc_col(int lane) { return lane & 31; }

// Workgroup tile BM x BN, reduction depth BK per step, WM x WN wavefronts.
template <int BM_, int BN_, int BK_, int WM_, int WN_, int NS_ = 2>
struct Tile {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_;
    static constexpr int NT = 64 * WM * WN;            // threads per workgroup
    static constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    static constexpr int LDA_OC = BM + 4, LDB_OC = BN + 4;
    static constexpr int LD_KC = BK + 4;
    // register stages of the global-load prefetch (four were measured three times: no faster on the dense
    // forward and weight gradient alone, nor inside the loop with the aggregation running beside them
    // (3 340 -> 3 310 ... 3 370 steps/s), nor on the short reductions of the small steps, K = 200 ... 512)
    static constexpr int NS = NS_;
    static_assert(TM >= 1 && TN >= 1 && BK % 8 == 0, "tile shape");
};

__device__ __forceinline__ void zero_acc(floatx16& a) {
#pragma unroll
    for (int r = 0; r < 16; ++r) a[r] = 0.f;
}

// Software-pipelined reduction loop shared by the three products.  Global loads run NS steps
// ahead of the MFMAs (NS register stages), LDS is double-buffered, and one barrier per step
// suffices: a buffer is rewritten only after the barrier of the step in between, which every
// wave passes after it has finished reading that buffer.
//   fetch(it, sa, sb)  issues the global loads of step `it` into a register stage; for it >= nit
//                      it must still be callable (Stage::load clamps addresses and yields zeros)
//   hook(Bs)           optional extra work on the staged B tile (bias gradient)
// No load is conditional: the fetches past the end re-read valid addresses and are dropped.
// Every path then has the same number of loads in flight at every wait, which lets the compiler
// wait for the oldest register stage only (vmcnt = loads of the younger ones).
// Requires nit >= 1.
// A_RESIDENT: the A operand of every step already lies in LDS, step `it` at As + it * (one step's
// tile), in the layout a staged step has; SA is then an empty type and only B is staged.
template <typename TL, bool A_KC, bool B_KC, typename SA, typename SB, bool A_RESIDENT = false, typename Fetch,
          typename Hook>
__device__ __forceinline__ void gemm_mainloop(int nit, float* As, float* Bs, Fetch&& fetch, Hook&& hook,
                                              floatx16 (&acc)[TL::TM][TL::TN]) {
    constexpr int BK = TL::BK, NS = TL::NS;
    static_assert(NS % 2 == 0, "the LDS buffer of a stage is its index modulo two");
    constexpr int LDA = A_KC ? TL::LD_KC : TL::LDA_OC, LDB = B_KC ? TL::LD_KC : TL::LDB_OC;
    constexpr int A_ELEMS = (A_KC ? TL::BM : BK) * LDA, B_ELEMS = (B_KC ? TL::BN : BK) * LDB;
    const int wave = threadIdx.x >> 6, wm = wave / TL::WN, wn = wave % TL::WN;
    const int a0 = wm * (TL::BM / TL::WM), b0 = wn * (TL::BN / TL::WN);
    SA sa[NS];
    SB sb[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        fetch(s, sa[s], sb[s]);
        __builtin_amdgcn_sched_barrier(0);  // issue order = consumption order (the load counter is in-order)
    }
    for (int it = 0; it < nit; it += NS) {
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            float* Ab = As + (A_RESIDENT ? it + s : (s & 1)) * A_ELEMS;
            float* Bb = Bs + (s & 1) * B_ELEMS;
            const bool live = s == 0 || it + s < nit;   // the step count need not be a multiple of NS
            if (live) {
                if constexpr (!A_RESIDENT) sa[s].template store<LDA>(Ab);
                sb[s].template store<LDB>(Bb);
                __syncthreads();
            }
            fetch(it + s + NS, sa[s], sb[s]);
            __builtin_amdgcn_sched_barrier(0);  // keep the loads here: the scheduler would sink them next to their use
            if (live) {
                hook(Bb);
                mma_step<BK, TL::TM, TL::TN, A_KC, B_KC, TL::LDA_OC, TL::LDB_OC>(Ab, Bb, a0, b0, acc);
            }
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

// The output tile of a workgroup, Y[row0.., col0..] = act(acc + bias) for rows < n and columns < ncols.  VEC: the tile is
// staged through LDS, where the operand buffers are dead by then, and leaves in 16-byte vectors, every row contiguous --
// four stores per thread instead of sixteen, 1-2 us of a short launch.  Needs ldy a multiple of the vector, Y 16-byte
// aligned, and a tile that fits the LDS_FLOATS floats at `lds`.  Otherwise element by element.  The values are the same
// either way.  VEC is a template parameter, not an argument: the staged path costs the whole kernel some registers
// (the weight gradient drops from six to five waves per SIMD), which a long launch pays for and a short one does not
// notice, so only launches of few workgroup rounds use it.
template <typename TY, typename TL, int LDS_FLOATS, bool VEC>
__device__ __forceinline__ void store_tile(const floatx16 (&acc)[TL::TM][TL::TN], float* lds, TY* __restrict__ Y, int64_t ldy,
                                           int row0, int col0, int n, int ncols, const float* __restrict__ bias, int relu) {
    constexpr int VE = 16 / (int)sizeof(TY), LDC = TL::BN + VE, VPR = TL::BN / VE;
    constexpr bool FITS = TL::BM * LDC * (int)sizeof(TY) <= LDS_FLOATS * 4;
    static_assert(!VEC || FITS, "the staged output tile must fit the kernel's LDS");
    if constexpr (!VEC) {
        for_each_acc<TL>(acc, [&](int r, int c, float v) {
            const int row = row0 + r, col = col0 + c;
            if (row < n && col < ncols) {
                float z = v + (bias ? bias[col] : 0.f);
                if (relu && !(z > 0.f)) z = 0.f;
                Y[(int64_t)row * ldy + col] = from_f32<TY>(z);
            }
        });
    } else {
        TY* Cs = reinterpret_cast<TY*>(lds);
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
}
template <typename TY>
inline bool vec_rows_ok(const void* Y, int64_t ldy) {
    return ldy % (16 / (int64_t)sizeof(TY)) == 0 && reinterpret_cast<uintptr_t>(Y) % 16 == 0;
}

// ---------------------------------------------------------------------------------
// forward: Y[n,out] = act(Hself[n,in] Wself[in,out] + A[n,in] Wneigh[in,out] + b)
// ---------------------------------------------------------------------------------
template <typename TH, typename TY, typename TL, int VA, int VB, bool ROUNDW, bool VEC = false>
__global__ __launch_bounds__(TL::NT) void k_linear_fwd(const TH* __restrict__ Hself, int64_t ldh,
                                                       const TH* __restrict__ Agg, int64_t lda, int n_cap,
                                                       const int32_t* n_d, int in, int in_a, int out,
                                                       const float* __restrict__ W, const float* __restrict__ bias,
                                                       int relu, TY* __restrict__ Y, int64_t ldy) {
    constexpr int BM = TL::BM, BN = TL::BN, BK = TL::BK;
    const int n = dev_count(n_cap, n_d);
    const int id = xcd_contiguous_id((int)gridDim.x * ((n + BM - 1) / BM));
    if (id < 0) return;
    const int row0 = (id / (int)gridDim.x) * BM, col0 = (id % (int)gridDim.x) * BN;
    constexpr int A_FLOATS = 2 * BM * TL::LD_KC, LDS_FLOATS = A_FLOATS + 2 * BK * TL::LDB_OC;
    __shared__ __align__(16) float lds[LDS_FLOATS];
    float* As = lds;
    float* Bs = lds + A_FLOATS;
    floatx16 acc[TL::TM][TL::TN];
#pragma unroll
    for (int a = 0; a < TL::TM; ++a)
#pragma unroll
        for (int b = 0; b < TL::TN; ++b) zero_acc(acc[a][b]);
    using SA = Stage<TH, BM, BK, VA, false, TL::NT>;
    using SB = Stage<float, BK, BN, VB, ROUNDW, TL::NT>;
    const int nk = (in + BK - 1) / BK;
    auto fetch = [&](int it, SA& sa, SB& sb) {
        const int ph = it >= nk, k0 = (it - ph * nk) * BK;  // k0 >= in past the last step: zeros
        sa.load(ph ? Agg : Hself, ph ? lda : ldh, row0, n, k0, in_a);   // in_a >= in: rows zero-padded to a whole vector
        sb.load(W + (int64_t)ph * in * out, out, k0, in, col0, out);
    };
    gemm_mainloop<TL, true, false, SA, SB>(2 * nk, As, Bs, fetch, [](const float*) {}, acc);
    store_tile<TY, TL, LDS_FLOATS, VEC>(acc, lds, Y, ldy, row0, col0, n, out, bias, relu);
}

// ---------------------------------------------------------------------------------
// A whole-graph layer in one launch: Y = act(H Wself + mean_nbr(H) Wneigh + b), fp32.
// The aggregated rows never reach HBM (no n x in buffer): a workgroup owns 32 rows, first takes the
// self product through the usual staged loop, then gathers COLS aggregated columns of its rows into
// LDS (a wave per row for COLS = 256, a half-wave for 128: whole 1 KB / 512 B pieces of the
// neighbours' rows, read straight from H, twelve in flight per lane, the next row's offsets and first
// column ids fetched under the current row) and feeds them to the matrix cores from there; layers
// wider than COLS repeat the last two steps.  Two workgroups fit a CU (74 KB of LDS, 128 registers).
// The sums run in the order of the stand-alone aggregation kernels (edge order; rows longer than
// 2048 edges in sixteen contiguous parts added in order), and the reduction over k in the order of
// k_linear_fwd, so the result equals the two-launch path bit for bit.
// ---------------------------------------------------------------------------------
using TileF = Tile<32, 256, 16, 1, 8>;
constexpr int FUSED_U = 12;        // neighbour rows in flight per lane
constexpr int FUSED_LONG = 2048;   // longer rows are summed by the whole workgroup together
constexpr int FUSED_B_FLOATS = 2 * TileF::BK * TileF::LDB_OC;
constexpr int fused_tile_floats(int cols) { return (cols / TileF::BK) * TileF::BM * TileF::LD_KC; }
constexpr size_t fused_lds_bytes(int cols) {
    return (size_t)(fused_tile_floats(cols) + FUSED_B_FLOATS) * sizeof(float) + (TileF::BM + 4) * sizeof(int);
}
static_assert(16 * 256 <= FUSED_B_FLOATS, "the sixteen partial sums of a long row borrow the weight stages");
struct NoStage {};

// First batch of column ids of the edge range [e0, e1) (all -1 for an empty range).
__device__ __forceinline__ void fused_first_ids(const int32_t* __restrict__ cols, int64_t e0, int64_t e1, int (&c)[FUSED_U]) {
#pragma unroll
    for (int u = 0; u < FUSED_U; ++u) c[u] = (e0 + u < e1) ? cols[e0 + u] : -1;
}

// Sum of the rows H[cols[e]] (the lane's four columns) for e in [e0, e1), in edge order; needs e0 < e1
// and the ids of the first batch in c.  The ids of the next batch are fetched while the rows of the
// current one are in flight, so a batch costs one memory round trip, not two; after the last batch
// that is the first batch of [n0, n1), the range to be summed next, left in c.
__device__ __forceinline__ float4 fused_sum_rows(const int32_t* __restrict__ cols, int64_t e0, int64_t e1, int64_t n0,
                                                 int64_t n1, int (&c)[FUSED_U], const float* __restrict__ Hc, int64_t ldh) {
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int64_t e = e0; e < e1; e += FUSED_U) {
        float4 v[FUSED_U];
#pragma unroll
        for (int u = 0; u < FUSED_U; ++u) {
            v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (c[u] >= 0) v[u] = *reinterpret_cast<const float4*>(Hc + (int64_t)c[u] * ldh);
        }
        const bool more = e + FUSED_U < e1;
        const int64_t p0 = more ? e + FUSED_U : n0, p1 = more ? e1 : n1;
#pragma unroll
        for (int u = 0; u < FUSED_U; ++u) c[u] = (p0 + u < p1) ? cols[p0 + u] : -1;
#pragma unroll
        for (int u = 0; u < FUSED_U; ++u) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
    }
    return acc;
}

template <int COLS>
__global__ __launch_bounds__(TileF::NT, 4) void k_sage_layer_fused(const int64_t* __restrict__ indptr,
                                                                const int32_t* __restrict__ cols, int n,
                                                                const float* __restrict__ H, int64_t ldh, int in, int out,
                                                                const float* __restrict__ W, const float* __restrict__ bias,
                                                                int relu, float* __restrict__ Y, int64_t ldy) {
    using TL = TileF;
    constexpr int BM = TL::BM, BN = TL::BN, BK = TL::BK, LDK = TL::LD_KC;
    constexpr int G = COLS / 4;            // lanes per row
    constexpr int NG = TL::NT / G;         // rows in flight per workgroup
    static_assert(16 % NG == 0 && BM % NG == 0, "a long row's sixteen parts are dealt out evenly");
    extern __shared__ __align__(16) float fused_lds[];
    float* Ts = fused_lds;                         // [COLS / BK][BM][LDK]; its head doubles as the self product's A stages
    float* Bs = fused_lds + fused_tile_floats(COLS);   // [2][BK][BN + 4]; scratch of the long-row sums between products
    int* long_rows = reinterpret_cast<int*>(Bs + FUSED_B_FLOATS);   // [BM] + count
    int* n_long = long_rows + BM;
    const int row0 = blockIdx.x * BM;
    floatx16 acc[TL::TM][TL::TN];
#pragma unroll
    for (int a = 0; a < TL::TM; ++a)
#pragma unroll
        for (int b = 0; b < TL::TN; ++b) zero_acc(acc[a][b]);
    using SA = Stage<float, BM, BK, 4, false, TL::NT>;
    using SB = Stage<float, BK, BN, 4, false, TL::NT>;
    const int grp = threadIdx.x / G, gl = threadIdx.x % G;
    // ---- self product --------------------------------------------------------------
    {
        auto fetch = [&](int it, SA& sa, SB& sb) {
            sa.load(H, ldh, row0, n, it * BK, in);      // past the last step: clamped addresses, zeros
            sb.load(W, out, it * BK, in, 0, out);
        };
        gemm_mainloop<TL, true, false, SA, SB>(in / BK, Ts, Bs, fetch, [](const float*) {}, acc);
    }
    // ---- aggregated columns, COLS at a time ---------------------------------------------
    for (int c0 = 0; c0 < in; c0 += COLS) {
        if (threadIdx.x == 0) *n_long = 0;
        __syncthreads();                             // the previous product has read its last tiles
        const float* Hc = H + c0 + gl * 4;
        float* Tc = Ts + ((gl >> 2) * BM) * LDK + (gl & 3) * 4;   // this lane's columns: step gl / 4, offset 4 (gl % 4)
        // the rows of a group one after the other; the edge offsets and the first column ids of the next
        // row are fetched while the current row is being summed
        auto row_range = [&](int r, int64_t& lo, int64_t& hi) {      // what a row contributes to the plain pass
            lo = hi = 0;
            if (r < BM && row0 + r < n) { lo = indptr[row0 + r]; hi = indptr[row0 + r + 1]; }
        };
        int64_t e0, e1;
        row_range(grp, e0, e1);
        int c[FUSED_U];
        fused_first_ids(cols, e0, e1 - e0 > FUSED_LONG ? e0 : e1, c);
        for (int r = grp; r < BM; r += NG) {
            int64_t n0, n1;
            row_range(r + NG, n0, n1);
            const int64_t n1s = n1 - n0 > FUSED_LONG ? n0 : n1;      // a long next row: nothing to prefetch
            if (e1 - e0 > FUSED_LONG) {
                if (gl == 0) long_rows[atomicAdd(n_long, 1)] = r;
                fused_first_ids(cols, n0, n1s, c);
            } else if (e1 > e0) {
                float4 a = fused_sum_rows(cols, e0, e1, n0, n1s, c, Hc, ldh);
                const float m = (float)(e1 - e0);
                a.x = a.x / m; a.y = a.y / m; a.z = a.z / m; a.w = a.w / m;
                *reinterpret_cast<float4*>(Tc + r * LDK) = a;
            } else {
                // an empty row, or one past the end of the graph (its tile row is never stored)
                *reinterpret_cast<float4*>(Tc + r * LDK) = make_float4(0.f, 0.f, 0.f, 0.f);
                fused_first_ids(cols, n0, n1s, c);
            }
            e0 = n0;
            e1 = n1;
        }
        __syncthreads();
        const int cnt = *n_long;
        for (int li = 0; li < cnt; ++li) {           // the list order depends on the atomics, each row's result does not
            const int r = long_rows[li];
            const int64_t e0 = indptr[row0 + r], e1 = indptr[row0 + r + 1];
            const int64_t chunk = (e1 - e0 + 15) / 16;
            for (int w = grp; w < 16; w += NG) {
                const int64_t w0 = e0 + w * chunk, w1 = (w0 + chunk < e1) ? w0 + chunk : e1;
                float4 part = make_float4(0.f, 0.f, 0.f, 0.f);
                if (w0 < w1) {
                    int lc[FUSED_U];
                    fused_first_ids(cols, w0, w1, lc);
                    part = fused_sum_rows(cols, w0, w1, w1, w1, lc, Hc, ldh);
                }
                *reinterpret_cast<float4*>(Bs + w * COLS + gl * 4) = part;
            }
            __syncthreads();
            if (threadIdx.x < COLS) {
                float sum = 0.f;
#pragma unroll
                for (int w = 0; w < 16; ++w) sum += Bs[w * COLS + threadIdx.x];
                Ts[((threadIdx.x / BK) * BM + r) * LDK + threadIdx.x % BK] = sum / (float)(e1 - e0);
            }
            __syncthreads();
        }
        auto fetch = [&](int it, NoStage&, SB& sb) {
            sb.load(W + (int64_t)(in + c0) * out, out, it * BK, in - c0, 0, out);   // past the last step: zeros, never used
        };
        gemm_mainloop<TL, true, false, NoStage, SB, true>(COLS / BK, Ts, Bs, fetch, [](const float*) {}, acc);
    }
    for_each_acc<TL>(acc, [&](int r, int c, float v) {
        const int row = row0 + r;
        if (row < n && c < out) {
            float z = v + (bias ? bias[c] : 0.f);
            if (relu && !(z > 0.f)) z = 0.f;
            Y[(int64_t)row * ldy + c] = z;
        }
    });
}

// ---------------------------------------------------------------------------------
// input gradient: dIn_h[n,in] = dZ[n,out] W_h[in,out]^T, h = blockIdx.z (0 self, 1 neigh)
// ---------------------------------------------------------------------------------
template <typename TD, typename TH, typename TL, int VD, int VW, bool ROUND, bool VEC = false>
__global__ __launch_bounds__(TL::NT) void k_linear_bwd_input(const TD* __restrict__ dY, int64_t lddy, int n_cap,
                                                             const int32_t* n_d, int in, int out,
                                                             const float* __restrict__ W, TH* __restrict__ dSelf,
                                                             TH* __restrict__ dAgg, int64_t ldi) {
    constexpr int BM = TL::BM, BN = TL::BN, BK = TL::BK;
    const int n = dev_count(n_cap, n_d);
    // x fastest, then the half, then the row tile: the workgroups that read one panel of dY are neighbours
    const int id = xcd_contiguous_id((int)gridDim.x * 2 * ((n + BM - 1) / BM));
    if (id < 0) return;
    const int col0 = (id % (int)gridDim.x) * BN, half = (id / (int)gridDim.x) % 2;
    const int row0 = (id / (int)gridDim.x / 2) * BM;
    constexpr int A_FLOATS = 2 * BM * TL::LD_KC, LDS_FLOATS = A_FLOATS + 2 * BN * TL::LD_KC;
    __shared__ __align__(16) float lds[LDS_FLOATS];
    float* As = lds;
    float* Bs = lds + A_FLOATS;
    floatx16 acc[TL::TM][TL::TN];
#pragma unroll
    for (int a = 0; a < TL::TM; ++a)
#pragma unroll
        for (int b = 0; b < TL::TN; ++b) zero_acc(acc[a][b]);
    using SA = Stage<TD, BM, BK, VD, ROUND && sizeof(TD) == 4, TL::NT>;
    using SB = Stage<float, BN, BK, VW, ROUND, TL::NT>;
    const float* Wh = W + (int64_t)half * in * out;
    auto fetch = [&](int it, SA& sa, SB& sb) {
        sa.load(dY, lddy, row0, n, it * BK, out);
        sb.load(Wh, out, col0, in, it * BK, out);
    };
    gemm_mainloop<TL, true, true, SA, SB>((out + BK - 1) / BK, As, Bs, fetch, [](const float*) {}, acc);
    store_tile<TH, TL, LDS_FLOATS, VEC>(acc, lds, half ? dAgg : dSelf, ldi, row0, col0, n, in, nullptr, 0);
}

// ---------------------------------------------------------------------------------
// weight gradient partials: P[s][h*in + m][o] = sum over the rows r of split s of
//   X_h[r, m] dZ[r, o],  X_0 = Hself, X_1 = A;  h = blockIdx.z % 2, s = blockIdx.z / 2
// ---------------------------------------------------------------------------------
template <typename TD, typename TH, typename TL, int VH, int VD, bool ROUND, bool VEC = false>
__global__ __launch_bounds__(TL::NT) void k_linear_bwd_weight(const TH* __restrict__ Hself, int64_t ldh,
                                                              const TH* __restrict__ Agg, int64_t lda,
                                                              const TD* __restrict__ dY, int64_t lddy, int n_cap,
                                                              const int32_t* n_d, int in, int in_a, int out, int splits,
                                                              float* __restrict__ P, float* __restrict__ Q) {
    constexpr int BM = TL::BM, BN = TL::BN, BK = TL::BK;
    const int n = dev_count(n_cap, n_d);
    // grid (out tiles, in tiles, 2 * splits); x fastest keeps the readers of one X panel on one L2
    const int id = xcd_contiguous_id((int)(gridDim.x * gridDim.y * gridDim.z));  // every tile carries work
    const int bx = id % (int)gridDim.x, by = (id / (int)gridDim.x) % (int)gridDim.y;
    const int bz = id / (int)(gridDim.x * gridDim.y);
    const int half = bz & 1, split = bz >> 1;
    // the first row-tile of the self half also sums the columns of its dZ tiles (bias gradient)
    const bool do_bias = Q != nullptr && half == 0 && by == 0;
    float bsum = 0.f;
    const int row0 = by * BM /* feature m */, col0 = bx * BN /* output o */;
    const int chunk = ((n + splits - 1) / splits + BK - 1) / BK * BK;
    const int r_begin = split * chunk, r_end = min(n, r_begin + chunk);
    constexpr int A_FLOATS = 2 * BK * TL::LDA_OC, LDS_FLOATS = A_FLOATS + 2 * BK * TL::LDB_OC;
    __shared__ __align__(16) float lds[LDS_FLOATS];
    float* As = lds;
    float* Bs = lds + A_FLOATS;
    floatx16 acc[TL::TM][TL::TN];
#pragma unroll
    for (int a = 0; a < TL::TM; ++a)
#pragma unroll
        for (int b = 0; b < TL::TN; ++b) zero_acc(acc[a][b]);
    using SA = Stage<TH, BK, BM, VH, false, TL::NT>;
    using SB = Stage<TD, BK, BN, VD, ROUND && sizeof(TD) == 4, TL::NT>;
    const TH* X = half ? Agg : Hself;
    const int64_t ldx = half ? lda : ldh;
    const int nit = r_end > r_begin ? (r_end - r_begin + BK - 1) / BK : 0;
    auto fetch = [&](int it, SA& sa, SB& sb) {
        sa.load(X, ldx, r_begin + it * BK, r_end, row0, in_a);   // rows of the product past `in` are not stored
        sb.load(dY, lddy, r_begin + it * BK, r_end, col0, out);
    };
    auto hook = [&](const float* Bcur) {
        if (do_bias && (int)threadIdx.x < BN) {
#pragma unroll 8
            for (int k = 0; k < BK; ++k) bsum += Bcur[k * TL::LDB_OC + threadIdx.x];
        }
    };
    if (nit > 0) gemm_mainloop<TL, false, false, SA, SB>(nit, As, Bs, fetch, hook, acc);
    if (do_bias && (int)threadIdx.x < BN && col0 + (int)threadIdx.x < out)
        Q[(int64_t)split * out + col0 + threadIdx.x] = bsum;
    float* dst = P + ((int64_t)split * 2 * in + (int64_t)half * in) * out;
    store_tile<float, TL, LDS_FLOATS, VEC>(acc, lds, dst, out, row0, col0, in, out, nullptr, 0);
}

// dW[idx] = sum_s P[s][idx]; db[o] = sum_s Q[s][o]; optionally the SGD step W -= lr dW,
// b -= lr db in the same pass, and (one extra workgroup) the mean of the per-seed losses --
// for up to SDT_MAX_LAYERS layers in one launch (a launch costs more than this work).
// A workgroup covers 64 consecutive elements with 4 threads each: thread g adds the partials
// g, g+4, g+8, ... and the four sums are combined in the order 0,1,2,3 -- a fixed order, so
// the result is deterministic, with four times as many loads in flight as one thread per element.
constexpr int TB = 256;
constexpr int SDT_MAX_REDUCE = 2 * SDT_MAX_LAYERS;   // a GAT layer queues two (weights + bias, attention vectors)
struct ReduceArgs {
    int32_t n;
    int32_t first[SDT_MAX_REDUCE + 1];  // first workgroup of each reduction
    PendingReduce r[SDT_MAX_REDUCE];
};
// w <- w - lr g (SGD) or the Adam update with the moments m, v kept beside w
// (returns the new value)
__device__ __forceinline__ float apply_update(float* w, float g, float* m, float* v, const OptArgs& o) {
    float wn;
    if (o.adam && m) {
        const float mn = o.beta1 * *m + (1.0f - o.beta1) * g;
        const float vn = o.beta2 * *v + (1.0f - o.beta2) * g * g;
        *m = mn;
        *v = vn;
        wn = *w - o.lr * (mn * o.c1) / (sqrtf(vn * o.c2) + o.eps);
    } else {
        wn = *w - o.lr * g;
    }
    *w = wn;
    return wn;
}

__global__ __launch_bounds__(TB) void k_reduce_partials(ReduceArgs a, OptArgs opt, const float* __restrict__ row_loss,
                                                        int n_loss, float* loss_out) {
    __shared__ float part[TB];
    if ((int)blockIdx.x == a.first[a.n]) {  // the extra last block: mean loss in a fixed order
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
    int l = 0;
    while (l + 1 < a.n && (int)blockIdx.x >= a.first[l + 1]) ++l;
    const PendingReduce& r = a.r[l];
    const int64_t n_w = (int64_t)2 * r.in * r.out;
    const int out = r.out;
    const int e = threadIdx.x & 63, g = threadIdx.x >> 6;
    const int64_t idx = (int64_t)((int)blockIdx.x - a.first[l]) * 64 + e;
    const bool is_w = idx < n_w, is_b = !is_w && idx < n_w + out;
    const float* src = is_w ? r.P + idx : r.Q + (idx - n_w);
    const int64_t stride = is_w ? n_w : out;
    int splits = is_w || r.q_splits < 0 ? r.splits : r.q_splits;
    if (!is_w && r.q_rows_d) splits = min(splits, (*r.q_rows_d + r.q_chunk_rows - 1) / r.q_chunk_rows);
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
            r.dW[idx] = t;
            if (r.W_upd) {
                const float wn = apply_update(r.W_upd + idx, t, r.mW ? r.mW + idx : nullptr, r.vW ? r.vW + idx : nullptr, opt);
                // the images of the weights the next step's products read (a step of the loop then starts without
                // a pass over the weights): element (k, o) of W[2 in][out]
                if (r.img_wt || r.img_x3) {
                    const int k = (int)(idx / out), o = (int)(idx - (int64_t)k * out);
                    if (r.img_wt) {
                        const uint16_t h = f32_to_bf16(wn);
                        r.img_wt[(int64_t)o * 2 * r.in + k] = h;
                        r.img_wb[(int64_t)k * r.img_ldb + o] = h;
                    }
                    if (r.img_x3) {
                        const int ph = k >= r.in;
                        r.img_x3[(int64_t)o * 2 * r.img_kp + ph * r.img_kp + (k - ph * r.in)] = wn;
                    }
                }
            }
        } else {
            const int o = (int)(idx - n_w);
            r.db[o] = t;
            if (r.b_upd) apply_update(r.b_upd + o, t, r.mb ? r.mb + o : nullptr, r.vb ? r.vb + o : nullptr, opt);
        }
    }
}

// widest vector (elements, <= 16 bytes) usable for rows of `width` elements
int vec_elems(size_t es, int width, std::initializer_list<int64_t> lds, std::initializer_list<const void*> ptrs) {
    int vb = 16;
    auto fit = [&](uint64_t x) {
        while (vb > (int)es && (x % vb) != 0) vb >>= 1;
    };
    if (width > 0) fit((uint64_t)width * es);   // width 0: rows are readable up to their stride (see Stage::load)
    for (int64_t ld : lds) fit((uint64_t)ld * es);
    for (const void* p : ptrs) fit(reinterpret_cast<uintptr_t>(p));
    int v = vb / (int)es;
    return v > 4 && es == 4 ? 4 : v;
}

// dZ masked by the ReLU of the layer's own output: M[r][c] = Y[r][c] > 0 ? dY[r][c] : 0.
// One workgroup per row at a time (no per-element division to find the row).
template <typename TD>
__global__ __launch_bounds__(256) void k_relu_mask(const TD* __restrict__ dY, int64_t lddy, const TD* __restrict__ Y,
                                                   int64_t ldy, int n_cap, const int32_t* n_d, int out,
                                                   TD* __restrict__ M) {
    const int n = dev_count(n_cap, n_d);
    for (int r = blockIdx.x; r < n; r += gridDim.x)
        for (int c = threadIdx.x; c < out; c += blockDim.x) {
            const TD g = dY[(int64_t)r * lddy + c];
            M[(int64_t)r * out + c] = to_f32<TD>(Y[(int64_t)r * ldy + c]) > 0.f ? g : from_f32<TD>(0.f);
        }
}

// Number of row ranges the weight gradient is split into.  The product has only
// ceil(in/BM) * ceil(out/BN) * 2 output tiles (80 for a 602 x 256 layer), far fewer than the chip
// has wavefront slots, so the batch rows are split until about four workgroups per CU exist;
// bounded so that a range keeps >= 128 rows and the partial products stay within 24 MB (they are
// written and read back once by the reduction).  All workgroups are resident at once and do equal
// work, so the launch takes as long as the fullest CU: among the split counts within -25% / +30%
// of that target the one that fills the 256 CUs most evenly wins (measured on the 602 x 256 layer:
// 13 splits = 1040 workgroups 94 us, 16 splits = 1280 workgroups 80 us).
int weight_splits(int n_cap, int in, int out, int BM, int BN) {
    const int tiles = ceil_div(in, BM) * ceil_div(out, BN) * 2;
    const int max_rows = ceil_div(n_cap > 0 ? n_cap : 1, 128);
    const int64_t max_bytes = ((int64_t)24 << 20) / ((int64_t)2 * in * out * 4);
    int hi_cap = max_rows;
    if (hi_cap > max_bytes) hi_cap = (int)max_bytes;
    if (hi_cap < 1) hi_cap = 1;
    const int s0 = ceil_div(1024, tiles);
    if (s0 >= hi_cap) return hi_cap;
    int lo = s0 - s0 / 4, hi = s0 + (3 * s0) / 10;
    if (lo < 1) lo = 1;
    if (hi > hi_cap) hi = hi_cap;
    int best = s0;
    double best_eff = 0.0;
    for (int s = lo; s <= hi; ++s) {
        const int w = tiles * s;
        const double eff = (double)w / (ceil_div(w, 256) * 256.0);
        const bool closer = (s > s0 ? s - s0 : s0 - s) < (best > s0 ? best - s0 : s0 - best);
        if (eff > best_eff + 1e-9 || (eff > best_eff - 1e-9 && closer)) {
            best_eff = eff;
            best = s;
        }
    }
    return best;
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

// Tile shapes, picked by measurement on MI355X (fp32 MFMA, out = 256):
// launches short enough for the staged output tile to pay (store_tile): few rounds of workgroups, or short row ranges
constexpr int32_t SHORT_LAUNCH_ROWS = 32768, SHORT_SPLIT_ROWS = 2048;
using TileS = Tile<64, 64, 32, 2, 2>;     // forward / input gradient of mini-batch sized layers
using TileW = Tile<64, 64, 16, 2, 2>;     // weight gradient (short row ranges: a shallower step wins)
using TileM = Tile<128, 128, 32, 4, 4>;   // forward from about 512 tiles of 128 x 128
using TileL = Tile<128, 256, 16, 2, 4>;   // forward of whole-graph sized layers

template <typename TH, typename TY, typename TL>
void launch_fwd(const void* Hself, int64_t ldh, const void* A, int64_t lda, int n_cap, const int32_t* n_d, int in,
                int out, const float* W, const float* b, int relu, void* Y, int64_t ldy, bool rows_padded, hipStream_t st) {
    constexpr bool ROUNDW = sizeof(TH) == 2;  // bf16 activations: weights enter the product rounded to bf16
    const int va = vec_elems(sizeof(TH), rows_padded ? 0 : in, {ldh, lda}, {Hself, A});
    const int in_a = (in + va - 1) / va * va;
    const int vb = vec_elems(4, out, {(int64_t)out}, {W});
    dim3 grid(ceil_div(out, TL::BN), ceil_div(n_cap, TL::BM));
    const bool vec = n_cap <= SHORT_LAUNCH_ROWS && vec_rows_ok<TY>(Y, ldy);   // output tiles through LDS (store_tile)
    SDT_VEC_SWITCH(va, (16 / sizeof(TH)), {
        constexpr int VA = V;
        SDT_VEC_SWITCH(vb, 4, {
            constexpr int VB = V;
            if constexpr (std::is_same<TL, TileS>::value) {
                if (vec) {
                    hipLaunchKernelGGL((k_linear_fwd<TH, TY, TL, VA, VB, ROUNDW, true>), grid, dim3(TL::NT), 0, st,
                                       static_cast<const TH*>(Hself), ldh, static_cast<const TH*>(A), lda, n_cap, n_d, in, in_a,
                                       out, W, b, relu, static_cast<TY*>(Y), ldy);
                    return;
                }
            }
            hipLaunchKernelGGL((k_linear_fwd<TH, TY, TL, VA, VB, ROUNDW>), grid, dim3(TL::NT), 0, st,
                               static_cast<const TH*>(Hself), ldh, static_cast<const TH*>(A), lda, n_cap, n_d, in, in_a, out,
                               W, b, relu, static_cast<TY*>(Y), ldy);
        })
    })
}

template <typename TD, typename TH>
void launch_bwd(const void* dY, int64_t lddy, const void* Hself, int64_t ldh, const void* A, int64_t lda, int n_cap,
                const int32_t* n_d, int in, int out, const float* W, float* dW, float* db, void* dSelf, void* dAgg,
                int64_t ldi, float* P, float* Q, int splits, const BwdExtras& ex, hipStream_t st) {
    constexpr bool ROUND = sizeof(TH) == 2;  // bf16 activations: fp32 operands enter the products rounded to bf16
    const int vd = vec_elems(sizeof(TD), out, {lddy}, {dY});
    const int vh = vec_elems(sizeof(TH), ex.rows_padded ? 0 : in, {ldh, lda}, {Hself, A});
    const int in_a = (in + vh - 1) / vh * vh;
    const int vw = vec_elems(4, out, {(int64_t)out}, {W});
    const TD* dYt = static_cast<const TD*>(dY);
    // weight gradient partials (bf16 activations inside a step: on the bf16 matrix cores)
    const int32_t dy_code = sizeof(TD) == 2 ? SDT_BF16 : SDT_F32;
    const bool weight_on_bf16_path = ex.Wb && sizeof(TH) == 2 && bf16_mfma_bwd_weight_ok(Hself, ldh, A, lda, dY, lddy, dy_code, in, out);
    // both products on the bf16 matrix cores: one launch for the two (they are independent; timed as the weight stage)
    const bool both = weight_on_bf16_path && dSelf && n_cap > 0 && bf16_mfma_bwd_input_ok(dY, lddy, dy_code, in, out, ldi);
    {
    StageTimer tw(ex.timing, ex.slot, SDT_STAGE_BWD_WEIGHT, ex.layer, st);
    if (both) {
        (void)linear_bwd_both_bf16(Hself, ldh, A, lda, dY, lddy, dy_code, n_cap, n_d, in, out, splits, P, Q, ex.Wb, dSelf, dAgg,
                                   ldi, st);
    } else if (weight_on_bf16_path) {
        (void)linear_bwd_weight_bf16(Hself, ldh, A, lda, dY, lddy, dy_code, n_cap, n_d, in, out, splits, P, Q, st);
    } else if (ex.x3 && sizeof(TH) == 4 && sizeof(TD) == 4 && x3_dw_wanted(n_cap, in, out)) {
        // (the caller's workspace was sized for this path's row ranges: bwd_ws with the same flag)
        (void)linear_bwd_weight_x3(static_cast<const float*>(Hself), ldh, static_cast<const float*>(A), lda,
                                   reinterpret_cast<const float*>(dYt), lddy, n_cap, n_d, in, out, splits, P, Q, st);
    } else {
        using TL = TileW;
        dim3 grid(ceil_div(out, TL::BN), ceil_div(in, TL::BM), 2 * splits);
        SDT_VEC_SWITCH(vh, (16 / sizeof(TH)), {
            constexpr int VH = V;
            SDT_VEC_SWITCH(vd, (16 / sizeof(TD)), {
                constexpr int VD = V;
                if (n_cap / splits <= SHORT_SPLIT_ROWS && vec_rows_ok<float>(P, out))
                    hipLaunchKernelGGL((k_linear_bwd_weight<TD, TH, TL, VH, VD, ROUND, true>), grid, dim3(TL::NT), 0, st,
                                       static_cast<const TH*>(Hself), ldh, static_cast<const TH*>(A), lda, dYt, lddy, n_cap,
                                       n_d, in, in_a, out, splits, P, Q);
                else
                    hipLaunchKernelGGL((k_linear_bwd_weight<TD, TH, TL, VH, VD, ROUND>), grid, dim3(TL::NT), 0, st,
                                       static_cast<const TH*>(Hself), ldh, static_cast<const TH*>(A), lda, dYt, lddy, n_cap,
                                       n_d, in, in_a, out, splits, P, Q);
            })
        })
    }
    }
    const bool input_on_bf16_path = ex.Wb && sizeof(TH) == 2 && dSelf && bf16_mfma_bwd_input_ok(dY, lddy, dy_code, in, out, ldi);
    if (!both) {
    StageTimer ti(dSelf && n_cap > 0 ? ex.timing : nullptr, ex.slot, SDT_STAGE_BWD_INPUT, ex.layer, st);
    if (input_on_bf16_path) {
        (void)linear_bwd_input_bf16(dY, lddy, dy_code, n_cap, n_d, in, out, ex.Wb, dSelf, dAgg, ldi, st);
    } else if (dSelf && n_cap > 0) {
        using TL = TileS;
        dim3 grid(ceil_div(in, TL::BN), ceil_div(n_cap, TL::BM), 2);
        SDT_VEC_SWITCH(vd, (16 / sizeof(TD)), {
            constexpr int VD = V;
            SDT_VEC_SWITCH(vw, 4, {
                constexpr int VW = V;
                if (n_cap <= SHORT_LAUNCH_ROWS && vec_rows_ok<TH>(dSelf, ldi) && vec_rows_ok<TH>(dAgg, ldi))
                    hipLaunchKernelGGL((k_linear_bwd_input<TD, TH, TL, VD, VW, ROUND, true>), grid, dim3(TL::NT), 0, st, dYt,
                                       lddy, n_cap, n_d, in, out, W, static_cast<TH*>(dSelf), static_cast<TH*>(dAgg), ldi);
                else
                    hipLaunchKernelGGL((k_linear_bwd_input<TD, TH, TL, VD, VW, ROUND>), grid, dim3(TL::NT), 0, st, dYt, lddy,
                                       n_cap, n_d, in, out, W, static_cast<TH*>(dSelf), static_cast<TH*>(dAgg), ldi);
            })
        })
    }
    }
    // after the input gradients: this pass may overwrite W with the SGD step
    PendingReduce pr;
    pr.P = P; pr.Q = Q; pr.splits = splits; pr.in = in; pr.out = out;
    pr.dW = dW; pr.db = db; pr.W_upd = ex.W_upd; pr.b_upd = ex.b_upd;
    if (ex.defer) *ex.defer = pr;
    else {
        OptArgs opt;
        opt.lr = ex.lr;
        (void)reduce_all(&pr, 1, opt, ex.row_loss, ex.n_loss, ex.loss_out, st);
    }
}


}  // namespace

int32_t sdt::linear_fwd(const void* Hself, int64_t ldh, const void* A, int64_t lda, int32_t n_cap, const int32_t* n_d,
                        int32_t in, int32_t out, const float* W, const float* b, int32_t relu, int32_t dtype, void* Y,
                        int64_t ldy, int32_t y_dtype, bool rows_padded, hipStream_t st) {
    SDT_REQUIRE(dtype_ok(dtype) && dtype_ok(y_dtype), SDT_ERR_INVALID_ARG, "sdt_sage_linear_fwd: unknown dtype");
    SDT_REQUIRE(!(dtype == SDT_F32 && y_dtype == SDT_BF16), SDT_ERR_INVALID_ARG,
                "sdt_sage_linear_fwd: bf16 output needs bf16 inputs");
    SDT_REQUIRE(n_cap >= 0 && in > 0 && out > 0 && ldh >= in && lda >= in && ldy >= out, SDT_ERR_INVALID_ARG,
                "sdt_sage_linear_fwd: bad sizes n=%d in=%d out=%d", n_cap, in, out);
    if (n_cap == 0) return SDT_OK;
    SDT_REQUIRE(Hself && A && W && Y, SDT_ERR_INVALID_ARG, "sdt_sage_linear_fwd: null pointer");
    // tile by problem size: the large tiles need enough workgroups to fill 256 CUs several times over
    const int64_t t128 = (int64_t)ceil_div(n_cap, 128) * ceil_div(out, 128);
    const int cls = (t128 >= 2048 && out >= 256) ? 2 : t128 >= 512 ? 1 : 0;
#define SDT_FWD(TH, TY)                                                                                            \
    do {                                                                                                           \
        if (cls == 2) launch_fwd<TH, TY, TileL>(Hself, ldh, A, lda, n_cap, n_d, in, out, W, b, relu, Y, ldy, rows_padded, st);  \
        else if (cls == 1) launch_fwd<TH, TY, TileM>(Hself, ldh, A, lda, n_cap, n_d, in, out, W, b, relu, Y, ldy, rows_padded, st); \
        else launch_fwd<TH, TY, TileS>(Hself, ldh, A, lda, n_cap, n_d, in, out, W, b, relu, Y, ldy, rows_padded, st);           \
    } while (0)
    if (dtype == SDT_F32) SDT_FWD(float, float);
#undef SDT_FWD
    // bf16 activations are widened on the way into LDS; the small tile hides that best
    else if (y_dtype == SDT_BF16)
        launch_fwd<bf16_t, bf16_t, TileS>(Hself, ldh, A, lda, n_cap, n_d, in, out, W, b, relu, Y, ldy, rows_padded, st);
    else
        launch_fwd<bf16_t, float, TileS>(Hself, ldh, A, lda, n_cap, n_d, in, out, W, b, relu, Y, ldy, rows_padded, st);
    SDT_CHECK_LAUNCH("linear_fwd");
    return SDT_OK;
}

// ---- whole-graph layer in one launch ------------------------------------------------
bool sdt::sage_layer_fused_ok(int64_t n_nodes, const void* H, int64_t ldh, int32_t in, int32_t out, const float* W,
                              int32_t dtype, const void* Y, int64_t ldy) {
    (void)Y; (void)ldy;
    return dtype == SDT_F32 && in >= 128 && in % 128 == 0 && out >= 4 && out <= TileF::BN && out % 4 == 0 &&
           ldh % 4 == 0 && reinterpret_cast<uintptr_t>(H) % 16 == 0 && reinterpret_cast<uintptr_t>(W) % 16 == 0 &&
           n_nodes > 0 && n_nodes <= 0x7FFFFFFF - TileF::BM;
}

int32_t sdt::sage_layer_fused_fwd(const sdt_csr* g, const float* H, int64_t ldh, int32_t in, int32_t out, const float* W,
                                  const float* b, int32_t relu, float* Y, int64_t ldy, hipStream_t st) {
    // 256 resident columns (a wave per row, 1 KB pieces) when the width allows, else 128
    const bool wide = in % 256 == 0;
    static std::atomic<bool> opted[2] = {{false}, {false}};   // two threads may get here together: setting twice is harmless    // more than 64 KB of dynamic LDS has to be opted into, once per kernel
    const void* fn = wide ? reinterpret_cast<const void*>(&k_sage_layer_fused<256>)
                          : reinterpret_cast<const void*>(&k_sage_layer_fused<128>);
    const size_t lds = wide ? fused_lds_bytes(256) : fused_lds_bytes(128);
    if (!opted[wide].load(std::memory_order_acquire)) {
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
            set_error("sage_layer_fused: cannot raise the dynamic LDS limit to %zu bytes", lds);
            return SDT_ERR_HIP;
        }
        opted[wide].store(true, std::memory_order_release);
    }
    const int n = (int)g->n_nodes;
    if (wide)
        hipLaunchKernelGGL(k_sage_layer_fused<256>, dim3(ceil_div(n, TileF::BM)), dim3(TileF::NT), lds, st, g->indptr,
                           g->indices, n, H, ldh, in, out, W, b, relu, Y, ldy);
    else
        hipLaunchKernelGGL(k_sage_layer_fused<128>, dim3(ceil_div(n, TileF::BM)), dim3(TileF::NT), lds, st, g->indptr,
                           g->indices, n, H, ldh, in, out, W, b, relu, Y, ldy);
    SDT_CHECK_LAUNCH("sage_layer_fused");
    return SDT_OK;
}

extern "C" int32_t sdt_sage_layer_csr_fused_ok(int32_t in, int32_t out, int32_t dtype) {
    return dtype == SDT_F32 && in >= 128 && in % 128 == 0 && out >= 4 && out <= TileF::BN && out % 4 == 0;
}

extern "C" int32_t sdt_sage_layer_csr_fwd(const sdt_csr* g, const void* H, int64_t ldh, int32_t in, int32_t out,
                                          const float* W, const float* b, int32_t relu, int32_t dtype, void* Y, int64_t ldy,
                                          void* stream) {
    SDT_REQUIRE(g, SDT_ERR_INVALID_ARG, "sdt_sage_layer_csr_fwd: null graph");
    SDT_REQUIRE(g->n_nodes >= 0 && in > 0 && out > 0 && ldh >= in && ldy >= out, SDT_ERR_INVALID_ARG,
                "sdt_sage_layer_csr_fwd: bad sizes n=%lld in=%d out=%d", (long long)g->n_nodes, in, out);
    if (g->n_nodes == 0) return SDT_OK;
    SDT_REQUIRE(g->indptr && g->indices && H && W && Y, SDT_ERR_INVALID_ARG, "sdt_sage_layer_csr_fwd: null pointer");
    SDT_REQUIRE(sage_layer_fused_ok(g->n_nodes, H, ldh, in, out, W, dtype, Y, ldy), SDT_ERR_INVALID_ARG,
                "sdt_sage_layer_csr_fwd: needs fp32, in a multiple of %d, out a multiple of 4 up to %d, 16-byte aligned "
                "H rows and W (got in=%d out=%d dtype=%d ldh=%lld); use sdt_sage_aggregate_csr_fwd + sdt_sage_linear_fwd",
                128, TileF::BN, in, out, dtype, (long long)ldh);
    return sage_layer_fused_fwd(g, static_cast<const float*>(H), ldh, in, out, W, b, relu, static_cast<float*>(Y), ldy,
                                static_cast<hipStream_t>(stream));
}

extern "C" int32_t sdt_sage_linear_fwd(const void* Hself, int64_t ldh, const void* A, int64_t lda, int32_t n_cap,
                                       const int32_t* n_d, int32_t in, int32_t out, const float* W, const float* b,
                                       int32_t relu, int32_t dtype, void* Y, int64_t ldy, int32_t y_dtype,
                                       void* stream) {
    return linear_fwd(Hself, ldh, A, lda, n_cap, n_d, in, out, W, b, relu, dtype, Y, ldy, y_dtype, false,
                      static_cast<hipStream_t>(stream));
}

namespace {
// workspace of the projection backward: dW partials | db partials | ReLU-masked copy of dY
struct BwdWs {
    int splits;
    size_t p_off, q_off, m_off, total;
};
BwdWs bwd_ws(int32_t n_cap, int32_t in, int32_t out, bool x3 = false) {
    BwdWs w;
    w.splits = x3 && x3_dw_wanted(n_cap, in, out) ? x3_dw_splits(n_cap, in) : weight_splits(n_cap, in, out, TileW::BM, TileW::BN);
    w.p_off = 0;
    w.q_off = align_up((size_t)w.splits * 2 * in * out * sizeof(float), 256);
    w.m_off = w.q_off + align_up((size_t)w.splits * out * sizeof(float), 256);
    w.total = w.m_off + align_up((size_t)n_cap * out * sizeof(float), 256);
    return w;
}
}  // namespace

extern "C" size_t sdt_linear_bwd_workspace_bytes(int32_t n_cap, int32_t in, int32_t out) {
    if (n_cap < 0 || in <= 0 || out <= 0) return 0;
    return bwd_ws(n_cap, in, out).total;
}

size_t sdt::linear_bwd_workspace_bytes_x3(int32_t n_cap, int32_t in, int32_t out) {
    if (n_cap < 0 || in <= 0 || out <= 0) return 0;
    return bwd_ws(n_cap, in, out, true).total;
}

namespace sdt {
int32_t reduce_all(const PendingReduce* r, int32_t n, const OptArgs& opt, const float* row_loss, int32_t n_loss,
                   float* loss_out, hipStream_t st) {
    SDT_REQUIRE(r && n >= 1 && n <= SDT_MAX_REDUCE, SDT_ERR_INVALID_ARG, "reduce_all: %d reductions", n);
    ReduceArgs a{};
    a.n = n;
    a.first[0] = 0;
    for (int l = 0; l < n; ++l) {
        a.r[l] = r[l];
        a.first[l + 1] = a.first[l] + ceil_div((int64_t)2 * r[l].in * r[l].out + r[l].out, 64);
    }
    hipLaunchKernelGGL(k_reduce_partials, dim3(a.first[n] + (loss_out ? 1 : 0)), dim3(TB), 0, st, a, opt, row_loss, n_loss,
                       loss_out);
    SDT_CHECK_LAUNCH("reduce_partials");
    return SDT_OK;
}

int32_t reduce_partials(const float* P, const float* Q, int32_t splits, int32_t in, int32_t out, float* dW, float* db,
                        const BwdExtras& ex, hipStream_t st) {
    PendingReduce pr;
    pr.P = P; pr.Q = Q; pr.splits = splits; pr.in = in; pr.out = out;
    pr.dW = dW; pr.db = db; pr.W_upd = ex.W_upd; pr.b_upd = ex.b_upd;
    if (ex.defer) {
        *ex.defer = pr;
        return SDT_OK;
    }
    OptArgs opt;
    opt.lr = ex.lr;
    return reduce_all(&pr, 1, opt, ex.row_loss, ex.n_loss, ex.loss_out, st);
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
    const BwdWs w = bwd_ws(n_cap, in, out, ex.x3 && dtype == SDT_F32 && dy_dtype == SDT_F32);
    SDT_REQUIRE(ws && ws_bytes >= w.total && aligned16(ws), SDT_ERR_WORKSPACE,
                "sdt_sage_linear_bwd: workspace of %zu bytes needed, %zu given", w.total, ws_bytes);
    char* base = static_cast<char*>(ws);
    float* P = reinterpret_cast<float*>(base + w.p_off);
    float* Q = reinterpret_cast<float*>(base + w.q_off);
    const void* dYm = dY;
    int64_t ldm = lddy;
    if (relu && n_cap > 0) {
        // the matrix products take dZ already masked by the layer's own ReLU: one elementwise pass
        void* M = base + w.m_off;
        const int blocks = n_cap < 8192 ? n_cap : 8192;
        if (dy_dtype == SDT_F32)
            hipLaunchKernelGGL(k_relu_mask<float>, dim3(blocks), dim3(256), 0, st, static_cast<const float*>(dY), lddy,
                               static_cast<const float*>(Y), ldy, n_cap, n_d, out, static_cast<float*>(M));
        else
            hipLaunchKernelGGL(k_relu_mask<bf16_t>, dim3(blocks), dim3(256), 0, st, static_cast<const bf16_t*>(dY), lddy,
                               static_cast<const bf16_t*>(Y), ldy, n_cap, n_d, out, static_cast<bf16_t*>(M));
        dYm = M;
        ldm = out;
    }
    if (dtype == SDT_F32)
        launch_bwd<float, float>(dYm, ldm, Hself, ldh, A, lda, n_cap, n_d, in, out, W, dW, db, dSelf, dAgg, ldi, P, Q,
                                 w.splits, ex, st);
    else if (dy_dtype == SDT_F32)
        launch_bwd<float, bf16_t>(dYm, ldm, Hself, ldh, A, lda, n_cap, n_d, in, out, W, dW, db, dSelf, dAgg, ldi, P, Q,
                                  w.splits, ex, st);
    else
        launch_bwd<bf16_t, bf16_t>(dYm, ldm, Hself, ldh, A, lda, n_cap, n_d, in, out, W, dW, db, dSelf, dAgg, ldi, P, Q,
                                   w.splits, ex, st);
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

// ---- the same backward with its scratch inside the library ---------------------------------
// For callers that cannot allocate device memory (under graph capture, in a serving loop, in a
// harness that forbids it): the split partial products, the bias partials and the masked copy
// of dY live in a file-scope device array instead of a caller's workspace.  Every GPU the
// library runs on holds its own copy of the array at its own address until the process ends;
// the address is looked up once per device, with that device current, and used from then on.
static __device__ __align__(256) unsigned char scratch[SDT_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex scratch_mu;
void* scratch_ptr[MAX_DEVICES] = {};

// device address of `scratch` on the current device (nullptr + error text on failure)
void* scratch_on_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) {
        set_error("sdt_sage_linear_bwd_noalloc: no current device (or device index %d beyond %d)", dev, MAX_DEVICES - 1);
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(scratch_mu);
    if (!scratch_ptr[dev]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            set_error("sdt_sage_linear_bwd_noalloc: hipGetSymbolAddress failed on device %d: %s", dev, hipGetErrorString(e));
            return nullptr;
        }
        scratch_ptr[dev] = p;
    }
    return scratch_ptr[dev];
}
}  // namespace

extern "C" int32_t sdt_sage_linear_bwd_noalloc(const void* dY, int64_t lddy, int32_t dy_dtype, const void* Y, int64_t ldy,
                                               int32_t relu, const void* Hself, int64_t ldh, const void* A, int64_t lda,
                                               int32_t n_cap, const int32_t* n_d, int32_t in, int32_t out, const float* W,
                                               int32_t dtype, float* dW, float* db, void* dSelf, void* dAgg, int64_t ldi,
                                               void* stream) {
    SDT_REQUIRE(n_cap >= 0 && in > 0 && out > 0, SDT_ERR_INVALID_ARG, "sdt_sage_linear_bwd_noalloc: bad sizes n=%d in=%d out=%d",
                n_cap, in, out);
    const size_t need = bwd_ws(n_cap, in, out).total;
    SDT_REQUIRE(need <= (size_t)SDT_NOALLOC_SCRATCH_BYTES, SDT_ERR_WORKSPACE,
                "sdt_sage_linear_bwd_noalloc: n=%d in=%d out=%d needs %zu bytes of scratch, the built-in buffer holds %zu; "
                "use sdt_sage_linear_bwd with a workspace of the caller's", n_cap, in, out, need, (size_t)SDT_NOALLOC_SCRATCH_BYTES);
    void* ws = scratch_on_current_device();
    if (!ws) return SDT_ERR_HIP;
    // every part of the scratch a call reads was written by that call before (partials of every split, the
    // masked copy row by row), so nothing has to be cleared between calls
    return linear_bwd(dY, lddy, dy_dtype, Y, ldy, relu, Hself, ldh, A, lda, n_cap, n_d, in, out, W, dtype, dW, db,
                      dSelf, dAgg, ldi, ws, (size_t)SDT_NOALLOC_SCRATCH_BYTES, BwdExtras{}, static_cast<hipStream_t>(stream));
}
