// fp32 GraphSAGE projection on the bf16 matrix cores through exact three-way splits.
//
// The fp32 matrix instruction of gfx950 runs at 1/16 of the bf16 one.  An fp32 number is the exact
// sum of three bf16 numbers, a = a1 + a2 + a3 (8 + 8 + 8 significand bits: a1 = bf16(a),
// a2 = bf16(a - a1), a3 = a - a1 - a2, every difference exact), so a product is
//   a b = a1 b1 + (a1 b2 + a2 b1) + (a1 b3 + a2 b2 + a3 b1) + [a2 b3 + a3 b2 + a3 b3],
// where every bf16 x bf16 product is exact in fp32.  The six terms outside the bracket are issued as
// six v_mfma_f32_32x32x16_bf16 on the same fp32 accumulator, smallest first; the bracket is below
// 2^-23 |a b| -- the size of the rounding of a single fp32 product -- and is dropped.  Six bf16
// instructions of 8 passes replace eight fp32 instructions of 16 passes per 16 reduction indices, and
// the error against an fp64 reference measures the same as the fp32 instruction's (1.1e-6 of the
// largest output on a 1204-long reduction, both).
//
// What bounds such a kernel on this chip is not the matrix pipe but the path global -> LDS of a CU
// (about 15 bytes per clock and CU measured, whatever the access pattern), so the tile is the largest
// that fits: 128 rows x the whole output width (up to 256), walked in steps of 16 reduction indices.
// The activations are then read once, the weights once per 128 rows.  Both operands stay fp32 in
// memory (4 bytes per element instead of 6 for three planes) and are split on the way into LDS; the
// weights are read from a transposed fp32 image, rewritten every step, so that both operands stage
// as 16-byte vectors along the reduction.  A layer of the size this path is for has only ~80 row
// tiles, so the reduction is dealt out over S workgroups per tile -- S chosen ON THE DEVICE from the
// true row count so that the workgroups fill the 256 CUs once -- and a second small kernel adds the
// S partial tiles in a fixed order with the bias and the activation: deterministic.
#include "common.h"

#include <atomic>

namespace sdt {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int BM = 128, BN = 256, BK = 16;
constexpr int LDK = BK + 8;   // bf16 elements per LDS row: 48 bytes, 16-byte fragment reads are conflict-free
constexpr int A_PLANE = BM * LDK, B_PLANE = BN * LDK, A_BUF = 3 * A_PLANE, B_BUF = 3 * B_PLANE;
constexpr int NT = 512;       // eight waves, 2 x 4 of 64 x 64
constexpr size_t LDS_BYTES = (size_t)2 * (A_BUF + B_BUF) * sizeof(uint16_t);   // 110 592: one workgroup per CU
constexpr int CUS = 256;

// two floats -> one dword of two bf16 (round to nearest even; v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pk_bf16(float a, float b) {
    f32x2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
// (a, b) -> packed pairs h, m, l with a = h.lo + m.lo + l.lo and b = h.hi + m.hi + l.hi exactly
__device__ __forceinline__ void split_pair(float a, float b, uint32_t& h, uint32_t& m, uint32_t& l) {
    h = pk_bf16(a, b);
    const float ra = a - __uint_as_float(h << 16), rb = b - __uint_as_float(h & 0xFFFF0000u);
    m = pk_bf16(ra, rb);
    const float sa = ra - __uint_as_float(m << 16), sb = rb - __uint_as_float(m & 0xFFFF0000u);
    l = pk_bf16(sa, sb);
}

// Number of workgroups a tile's reduction is dealt out over, from the true row count: as many as fill
// the CUs once, at most s_max, and no fewer than four steps each.
__device__ __host__ __forceinline__ int x3_splits(int n, int steps, int s_max) {
    const int tiles = (n + BM - 1) / BM;
    int s = tiles > 0 ? CUS / tiles : 1;
    if (s > s_max) s = s_max;
    if (s > steps / 4) s = steps / 4;
    return s < 1 ? 1 : s;
}

// Wt[o][ph kp + k] = W[ph in + k][o] for k < in, 0 up to kp (kp = nk * 16): column o of W as a row
__global__ __launch_bounds__(256) void k_x3_transpose_w(const float* __restrict__ W, int in, int kp, int out,
                                                        float* __restrict__ Wt) {
    // a 32 x 32 tile through LDS: coalesced on both sides
    __shared__ float t[32][33];
    const int kk0 = blockIdx.x * 32, o0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
#pragma unroll
    for (int j = 0; j < 32; j += 8) {
        const int kk = kk0 + ty + j, o = o0 + tx;
        const int ph = kk >= kp, k = kk - ph * kp;
        t[ty + j][tx] = (kk < 2 * kp && k < in && o < out) ? W[((int64_t)ph * in + k) * out + o] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 32; j += 8) {
        const int o = o0 + ty + j, kk = kk0 + tx;
        if (o < out && kk < 2 * kp) Wt[(int64_t)o * 2 * kp + kk] = t[tx][ty + j];
    }
}

// Partial tiles P[z][n_cap][out], z < S, of Y = [Hself | Agg] W.
// Requirements (checked by the host): rows of Hself / Agg 16-byte aligned, readable and ZERO from `in`
// up to kp = nk * 16 floats; out <= 256; Wt as k_x3_transpose_w leaves it.
__global__ __launch_bounds__(NT, 1) void k_linear_fwd_x3(const float* __restrict__ Hself, int64_t ldh,
                                                         const float* __restrict__ Agg, int64_t lda, int n_cap,
                                                         const int32_t* n_d, int nk, int out,
                                                         const float* __restrict__ Wt, int s_max,
                                                         float* __restrict__ P) {
    const int n = dev_count(n_cap, n_d);
    const int S = x3_splits(n, 2 * nk, s_max);
    const int id = xcd_contiguous_id(((n + BM - 1) / BM) * S);
    if (id < 0) return;
    const int z = id % S, row0 = (id / S) * BM;   // the S units of a tile are neighbours
    extern __shared__ __align__(16) uint16_t lds_x3[];
    uint16_t* As = lds_x3;
    uint16_t* Bs = lds_x3 + 2 * A_BUF;
    floatx16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
    const int kp = nk * BK;
    const int per = (2 * nk + S - 1) / S;
    const int it0 = z * per, it1 = min(2 * nk, it0 + per);
    const int nit = it1 - it0;
    const int tid = threadIdx.x;
    // staging: thread -> (column tid/2, floats 8 (tid%2) ...) of the weights; the first 256 threads also -> (row tid/2,
    // floats 8 (tid%2) ...) of the activations: every LDS store is then a whole 16-byte vector per plane, free of bank
    // conflicts (8-byte stores of four floats per thread collided two ways).  A row or column past the end is
    // clamped: it only feeds outputs that are never stored.
    const int bc = tid >> 1, bkv = tid & 1;
    const bool has_a = tid < 2 * BM;
    const int arow = min(row0 + (bc & (BM - 1)), n - 1);
    const char* aS = reinterpret_cast<const char*>(Hself + (int64_t)arow * ldh + bkv * 8);
    const char* aN = reinterpret_cast<const char*>(Agg + (int64_t)arow * lda + bkv * 8);
    const char* bp = reinterpret_cast<const char*>(Wt + (int64_t)min(bc, out - 1) * 2 * kp + bkv * 8);
    const int b_off = bc * LDK + bkv * 8, a_off = (bc & (BM - 1)) * LDK + bkv * 8;
    struct St { float4 a0, a1, b0, b1; };
    // Nothing about a fetch is conditional (a step past the unit's range re-reads the last valid step and is
    // never used), so the wait before a stage is stored covers that stage only and the next one keeps flying.
    auto fetch = [&](int it_rel, St& s) {
        const int it = min(it0 + it_rel, 2 * nk - 1);
        const int ph = it >= nk;
        if (has_a) {   // (uniform over a wave)
            const char* pa = (ph ? aN : aS) + (int64_t)(it - ph * nk) * (BK * 4);
            s.a0 = *reinterpret_cast<const float4*>(pa);
            s.a1 = *reinterpret_cast<const float4*>(pa + 16);
        }
        const char* pb = bp + (int64_t)it * (BK * 4);
        s.b0 = *reinterpret_cast<const float4*>(pb);
        s.b1 = *reinterpret_cast<const float4*>(pb + 16);
    };
    auto store = [&](const St& s, uint16_t* Ab, uint16_t* Bb) {
        if (has_a) {
            uint4 h, m, l;
            split_pair(s.a0.x, s.a0.y, h.x, m.x, l.x);
            split_pair(s.a0.z, s.a0.w, h.y, m.y, l.y);
            split_pair(s.a1.x, s.a1.y, h.z, m.z, l.z);
            split_pair(s.a1.z, s.a1.w, h.w, m.w, l.w);
            *reinterpret_cast<uint4*>(Ab + a_off) = h;
            *reinterpret_cast<uint4*>(Ab + A_PLANE + a_off) = m;
            *reinterpret_cast<uint4*>(Ab + 2 * A_PLANE + a_off) = l;
        }
        uint4 bh, bm, bl;
        split_pair(s.b0.x, s.b0.y, bh.x, bm.x, bl.x);
        split_pair(s.b0.z, s.b0.w, bh.y, bm.y, bl.y);
        split_pair(s.b1.x, s.b1.y, bh.z, bm.z, bl.z);
        split_pair(s.b1.z, s.b1.w, bh.w, bm.w, bl.w);
        *reinterpret_cast<uint4*>(Bb + b_off) = bh;
        *reinterpret_cast<uint4*>(Bb + B_PLANE + b_off) = bm;
        *reinterpret_cast<uint4*>(Bb + 2 * B_PLANE + b_off) = bl;
    };
    const int wave = tid >> 6, lane = tid & 63, a0 = (wave >> 2) * 64, b0 = (wave & 3) * 64;
    const int fi = lane & 31, fk = (lane >> 5) * 8;   // which eight reduction indices a lane holds does not matter
                                                     // to the sum as long as both operands agree
    auto step = [&](const uint16_t* Ab, const uint16_t* Bb) {
        bf16x8 fa[3][2], fb[3][2];
#pragma unroll
        for (int q = 0; q < 3; ++q)
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                fa[q][t] = *reinterpret_cast<const bf16x8*>(Ab + q * A_PLANE + (a0 + t * 32 + fi) * LDK + fk);
                fb[q][t] = *reinterpret_cast<const bf16x8*>(Bb + q * B_PLANE + (b0 + t * 32 + fi) * LDK + fk);
            }
        // smallest terms first: a1 b3, a3 b1, a2 b2, a1 b2, a2 b1, a1 b1 (planes numbered from 0)
        constexpr int PA[6] = {0, 2, 1, 0, 1, 0};
        constexpr int PB[6] = {2, 0, 1, 1, 0, 0};
#pragma unroll
        for (int t = 0; t < 6; ++t)
#pragma unroll
            for (int tm = 0; tm < 2; ++tm)
#pragma unroll
                for (int tn = 0; tn < 2; ++tn)
                    acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[PA[t]][tm], fb[PB[t]][tn], acc[tm][tn], 0, 0, 0);
    };
    if (nit > 0) {
        St st[2];
        fetch(0, st[0]);
        __builtin_amdgcn_sched_barrier(0);
        fetch(1, st[1]);
        __builtin_amdgcn_sched_barrier(0);
        for (int it = 0; it < nit; it += 2) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const bool live = s == 0 || it + 1 < nit;
                uint16_t* Ab = As + s * A_BUF;
                uint16_t* Bb = Bs + s * B_BUF;
                if (live) {
                    store(st[s], Ab, Bb);
                    __syncthreads();   // one barrier per step: a buffer is rewritten two steps later, after the barrier in between
                }
                fetch(it + s + 2, st[s]);
                __builtin_amdgcn_sched_barrier(0);
                if (live) step(Ab, Bb);
            }
        }
    }
    float* dst = P + (int64_t)z * n_cap * out;
#pragma unroll
    for (int tm = 0; tm < 2; ++tm)
#pragma unroll
        for (int tn = 0; tn < 2; ++tn) {
            const int col = b0 + tn * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = row0 + a0 + tm * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (row < n && col < out) dst[(int64_t)row * out + col] = acc[tm][tn][r];
            }
        }
}

// Y = act(P[0] + P[1] + ... + P[S-1] + b), S as the product kernel chose it; four columns per thread
// (out % 4 == 0, ldy % 4 == 0, Y 16-byte aligned).
__global__ __launch_bounds__(256) void k_linear_fwd_x3_finish(const float* __restrict__ P, int n_cap,
                                                              const int32_t* n_d, int nk, int out, int s_max,
                                                              const float* __restrict__ bias, int relu,
                                                              float* __restrict__ Y, int64_t ldy) {
    const int n = dev_count(n_cap, n_d);
    const int S = x3_splits(n, 2 * nk, s_max);
    const int q = out >> 2;
    const int64_t total = (int64_t)n * q, plane = (int64_t)n_cap * out;
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int row = (int)(i / q), col = (int)(i - (int64_t)row * q) * 4;
        const float* src = P + (int64_t)row * out + col;
        float4 a = *reinterpret_cast<const float4*>(src);
        for (int s = 1; s < S; ++s) {
            const float4 t = *reinterpret_cast<const float4*>(src + s * plane);
            a.x += t.x; a.y += t.y; a.z += t.z; a.w += t.w;
        }
        if (bias) {
            a.x += bias[col]; a.y += bias[col + 1]; a.z += bias[col + 2]; a.w += bias[col + 3];
        }
        if (relu) {
            if (!(a.x > 0.f)) a.x = 0.f;
            if (!(a.y > 0.f)) a.y = 0.f;
            if (!(a.z > 0.f)) a.z = 0.f;
            if (!(a.w > 0.f)) a.w = 0.f;
        }
        *reinterpret_cast<float4*>(Y + (int64_t)row * ldy + col) = a;
    }
}

// ---- weight gradient ------------------------------------------------------------------------
// P[s][h in + m][o] = sum over the rows r of row range s of X_h[r, m] dZ[r, o]  (X_0 = Hself, X_1 = A),
// Q[s][o] = column sums of dZ over the range: the layout the step's single reduction launch expects.
// The reduction runs over the ROWS here, which are the strided index of both operands: a thread
// gathers eight consecutive rows of one column (eight 4-byte loads, each coalesced over the lanes'
// consecutive columns), splits them and stores one 16-byte vector per plane, so the tiles reach LDS
// in the layout the forward uses and the matrix step is the same.  Tile 128 features x 256 outputs
// x 16 rows; grid = (feature tiles of both halves) x S row ranges, S = 256 / tiles: one workgroup per CU.
// No alignment or padding requirement (all loads are single dwords; rows and columns past the end are
// clamped to valid addresses, rows past the range are zeroed, columns past the end are never stored).
__global__ __launch_bounds__(NT, 1) void k_linear_bwd_weight_x3(const float* __restrict__ Hself, int64_t ldh,
                                                                const float* __restrict__ Agg, int64_t lda,
                                                                const float* __restrict__ dY, int64_t lddy, int n_cap,
                                                                const int32_t* n_d, int in, int out, int S,
                                                                float* __restrict__ P, float* __restrict__ Q) {
    const int n = dev_count(n_cap, n_d);
    const int mt = (in + BM - 1) / BM;
    const int id = xcd_contiguous_id(mt * 2 * S);   // every unit writes its partial tile, if only zeros
    if (id < 0) return;
    const int tile = id % (mt * 2), split = id / (mt * 2);   // the tiles of a row range are neighbours: they share dZ
    const int half = tile / mt, m0 = (tile % mt) * BM;
    const int chunk = ((n + S - 1) / S + BK - 1) / BK * BK;
    const int r_begin = split * chunk, r_end = min(n, r_begin + chunk);
    const int nit = r_end > r_begin ? (r_end - r_begin + BK - 1) / BK : 0;
    extern __shared__ __align__(16) uint16_t lds_x3[];
    uint16_t* As = lds_x3;
    uint16_t* Bs = lds_x3 + 2 * A_BUF;
    floatx16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
    const int tid = threadIdx.x;
    const float* X = half ? Agg : Hself;
    const int64_t ldx = half ? lda : ldh;
    // dZ: thread -> column tid % 256, rows 8 (tid / 256) ... of the step; X: threads < 256 -> column tid % 128,
    // rows 8 (tid / 128) ...
    const int bo = tid & 255, bk = tid >> 8, am = tid & 127, ak = (tid >> 7) & 1;
    const bool has_a = tid < 256;
    const float* pb = dY + min(bo, out - 1);
    const float* pa = X + min(m0 + am, in - 1);
    const int b_off = bo * LDK + bk * 8, a_off = am * LDK + ak * 8;
    const bool do_bias = Q != nullptr && tile == 0;
    float bsum = 0.f;
    struct St { float b[8], a[8]; };
    auto fetch = [&](int it, St& s) {
        const int rb = r_begin + it * BK + bk * 8, ra = r_begin + it * BK + ak * 8;
#pragma unroll
        for (int i = 0; i < 8; ++i) s.b[i] = pb[(int64_t)min(rb + i, n - 1) * lddy];
        if (has_a) {
#pragma unroll
            for (int i = 0; i < 8; ++i) s.a[i] = pa[(int64_t)min(ra + i, n - 1) * ldx];
        }
    };
    auto put = [&](const float (&v)[8], int r0, uint16_t* plane0, int plane_elems, int off, bool sum) {
        float w[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) w[i] = r0 + i < r_end ? v[i] : 0.f;
        if (sum) {
#pragma unroll
            for (int i = 0; i < 8; ++i) bsum += w[i];
        }
        uint4 h, m, l;
        split_pair(w[0], w[1], h.x, m.x, l.x);
        split_pair(w[2], w[3], h.y, m.y, l.y);
        split_pair(w[4], w[5], h.z, m.z, l.z);
        split_pair(w[6], w[7], h.w, m.w, l.w);
        *reinterpret_cast<uint4*>(plane0 + off) = h;
        *reinterpret_cast<uint4*>(plane0 + plane_elems + off) = m;
        *reinterpret_cast<uint4*>(plane0 + 2 * plane_elems + off) = l;
    };
    const int wave = tid >> 6, lane = tid & 63, a0 = (wave >> 2) * 64, b0 = (wave & 3) * 64;
    const int fi = lane & 31, fk = (lane >> 5) * 8;
    auto step = [&](const uint16_t* Ab, const uint16_t* Bb) {
        bf16x8 fa[3][2], fb[3][2];
#pragma unroll
        for (int q = 0; q < 3; ++q)
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                fa[q][t] = *reinterpret_cast<const bf16x8*>(Ab + q * A_PLANE + (a0 + t * 32 + fi) * LDK + fk);
                fb[q][t] = *reinterpret_cast<const bf16x8*>(Bb + q * B_PLANE + (b0 + t * 32 + fi) * LDK + fk);
            }
        constexpr int PA[6] = {0, 2, 1, 0, 1, 0};
        constexpr int PB[6] = {2, 0, 1, 1, 0, 0};
#pragma unroll
        for (int t = 0; t < 6; ++t)
#pragma unroll
            for (int tm = 0; tm < 2; ++tm)
#pragma unroll
                for (int tn = 0; tn < 2; ++tn)
                    acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[PA[t]][tm], fb[PB[t]][tn], acc[tm][tn], 0, 0, 0);
    };
    if (nit > 0) {
        St st[2];
        fetch(0, st[0]);
        __builtin_amdgcn_sched_barrier(0);
        fetch(1, st[1]);
        __builtin_amdgcn_sched_barrier(0);
        for (int it = 0; it < nit; it += 2) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const bool live = s == 0 || it + 1 < nit;
                uint16_t* Ab = As + s * A_BUF;
                uint16_t* Bb = Bs + s * B_BUF;
                if (live) {
                    put(st[s].b, r_begin + (it + s) * BK + bk * 8, Bb, B_PLANE, b_off, do_bias);
                    if (has_a) put(st[s].a, r_begin + (it + s) * BK + ak * 8, Ab, A_PLANE, a_off, false);
                    __syncthreads();
                }
                fetch(it + s + 2, st[s]);
                __builtin_amdgcn_sched_barrier(0);
                if (live) step(Ab, Bb);
            }
        }
    }
    if (do_bias) {   // the two row groups of a column, added in a fixed order
        __syncthreads();
        float* red = reinterpret_cast<float*>(lds_x3);
        red[tid] = bsum;
        __syncthreads();
        if (tid < 256 && tid < out) Q[(int64_t)split * out + tid] = red[tid] + red[256 + tid];
    }
    float* dst = P + ((int64_t)split * 2 * in + (int64_t)half * in) * out;
#pragma unroll
    for (int tm = 0; tm < 2; ++tm)
#pragma unroll
        for (int tn = 0; tn < 2; ++tn) {
            const int col = b0 + tn * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + a0 + tm * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (row < in && col < out) dst[(int64_t)row * out + col] = acc[tm][tn][r];
            }
        }
}

constexpr int S_MAX = 4;

struct X3Ws {
    int nk, s_max;
    size_t wt_off, p_off, total;
};
X3Ws x3_ws(int32_t n_cap, int32_t in, int32_t out) {
    X3Ws w;
    w.nk = (in + BK - 1) / BK;
    w.s_max = S_MAX;
    w.wt_off = 0;
    w.p_off = align_up((size_t)out * 2 * w.nk * BK * sizeof(float), 256);
    w.total = w.p_off + align_up((size_t)w.s_max * (n_cap > 0 ? n_cap : 1) * out * sizeof(float), 256);
    return w;
}

std::atomic<bool> lds_opted{false}, lds_opted_dw{false};

}  // namespace

// Layers this path is for: fp32, an output width that fills most of the 256-column tile, a reduction long
// enough to pay for the second pass, and few enough rows that a 64 x 64 tiling would leave the chip
// unevenly filled while 128-row tiles dealt out over the reduction fill it once.
bool x3_fwd_wanted(int32_t n_cap, int32_t in, int32_t out) {
    return out > 128 && out <= BN && out % 4 == 0 && in >= 256 && n_cap >= 2048 && ceil_div(n_cap, BM) <= CUS;
}

size_t x3_fwd_workspace_bytes(int32_t n_cap, int32_t in, int32_t out) {
    return x3_fwd_wanted(n_cap, in, out) ? x3_ws(n_cap, in, out).total : 0;
}

bool x3_fwd_ok(const void* Hself, int64_t ldh, const void* A, int64_t lda, int32_t in, bool rows_padded, const void* Y,
               int64_t ldy) {
    const int kp = (in + BK - 1) / BK * BK;
    // rows readable and zero up to kp: either nothing lies past `in`, or the caller promises zero padding up to the stride
    const bool rows_ok = in == kp || (rows_padded && ldh >= kp && lda >= kp);
    return rows_ok && ldh % 4 == 0 && lda % 4 == 0 && ldy % 4 == 0 && aligned16(Hself) && aligned16(A) && aligned16(Y);
}

int32_t x3_fwd_image_kp(int32_t in) { return ceil_div(in, BK) * BK; }
size_t x3_fwd_image_bytes(int32_t in, int32_t out) { return align_up((size_t)out * 2 * x3_fwd_image_kp(in) * sizeof(float), 256); }

int32_t linear_fwd_x3(const float* Hself, int64_t ldh, const float* A, int64_t lda, int32_t n_cap, const int32_t* n_d,
                      int32_t in, int32_t out, const float* W, const float* b, int32_t relu, float* Y, int64_t ldy,
                      void* ws, size_t ws_bytes, float* Wt_ext, bool wt_current, hipStream_t st) {
    if (n_cap == 0) return SDT_OK;
    const X3Ws w = x3_ws(n_cap, in, out);
    SDT_REQUIRE(ws && ws_bytes >= w.total && aligned16(ws), SDT_ERR_WORKSPACE,
                "linear_fwd_x3: workspace of %zu bytes needed, %zu given", w.total, ws_bytes);
    if (!lds_opted.load(std::memory_order_acquire)) {   // more than 64 KB of dynamic LDS has to be opted into, once
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&k_linear_fwd_x3), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)LDS_BYTES) != hipSuccess) {
            set_error("linear_fwd_x3: cannot raise the dynamic LDS limit to %zu bytes", LDS_BYTES);
            return SDT_ERR_HIP;
        }
        lds_opted.store(true, std::memory_order_release);
    }
    float* Wt = Wt_ext ? Wt_ext : reinterpret_cast<float*>(static_cast<char*>(ws) + w.wt_off);
    float* P = reinterpret_cast<float*>(static_cast<char*>(ws) + w.p_off);
    const int kp = w.nk * BK;
    if (!(Wt_ext && wt_current)) {
        hipLaunchKernelGGL(k_x3_transpose_w, dim3(ceil_div(2 * kp, 32), ceil_div(out, 32)), dim3(256), 0, st, W, in, kp, out, Wt);
        SDT_CHECK_LAUNCH("x3_transpose_w");
    }
    // grid for the upper bound of the row count and of the split; the kernel uses the first tiles * S workgroups
    hipLaunchKernelGGL(k_linear_fwd_x3, dim3(ceil_div(n_cap, BM) * w.s_max), dim3(NT), LDS_BYTES, st, Hself, ldh, A, lda,
                       n_cap, n_d, w.nk, out, Wt, w.s_max, P);
    SDT_CHECK_LAUNCH("linear_fwd_x3");
    const int64_t quads = (int64_t)n_cap * (out / 4);
    const int blocks = (int)(quads / 256 < 2048 ? (quads + 255) / 256 : 2048);
    hipLaunchKernelGGL(k_linear_fwd_x3_finish, dim3(blocks), dim3(256), 0, st, P, n_cap, n_d, w.nk, out, w.s_max, b, relu, Y,
                       ldy);
    SDT_CHECK_LAUNCH("linear_fwd_x3_finish");
    return SDT_OK;
}

// Weight gradient: the same shapes (wide output, enough rows and features that the 128 x 256 tiles dealt out over
// the rows fill the chip).
bool x3_dw_wanted(int32_t n_cap, int32_t in, int32_t out) {
    return out > 128 && out <= BN && in >= 128 && n_cap >= 2048 && 2 * ceil_div(in, BM) <= CUS / 4;
}

// row ranges: as many as give every CU one workgroup, each at least 64 rows
int32_t x3_dw_splits(int32_t n_cap, int32_t in) {
    int s = CUS / (2 * ceil_div(in, BM));
    const int max_rows = ceil_div(n_cap > 0 ? n_cap : 1, 64);
    if (s > max_rows) s = max_rows;
    return s < 1 ? 1 : s;
}

int32_t linear_bwd_weight_x3(const float* Hself, int64_t ldh, const float* A, int64_t lda, const float* dY, int64_t lddy,
                             int32_t n_cap, const int32_t* n_d, int32_t in, int32_t out, int32_t splits, float* P, float* Q,
                             hipStream_t st) {
    if (!lds_opted_dw.load(std::memory_order_acquire)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&k_linear_bwd_weight_x3),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_BYTES) != hipSuccess) {
            set_error("linear_bwd_weight_x3: cannot raise the dynamic LDS limit to %zu bytes", LDS_BYTES);
            return SDT_ERR_HIP;
        }
        lds_opted_dw.store(true, std::memory_order_release);
    }
    // (no rows: every unit still writes its tile of zeros, which the reduction reads)
    hipLaunchKernelGGL(k_linear_bwd_weight_x3, dim3(2 * ceil_div(in, BM) * splits), dim3(NT), LDS_BYTES, st, Hself, ldh, A, lda,
                       dY, lddy, n_cap, n_d, in, out, splits, P, Q);
    SDT_CHECK_LAUNCH("linear_bwd_weight_x3");
    return SDT_OK;
}

}  // namespace sdt
