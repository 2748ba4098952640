// Fused classifier head: the last GraphSAGE layer's projection, the softmax
// cross-entropy over the seeds, and the whole backward of that layer, in one launch.
//
// The last layer works on the B seed rows only (B ~ 1024, in ~ 256, C ~ 50-200), so its
// three matrix products are far too small to fill the chip one launch at a time: each
// generic launch is bound by the latency of a short dependent loop in a handful of
// workgroups.  Here a workgroup owns 16 seed rows, keeps their [self | mean] features
// (16 x 2in floats) and their logits / loss gradient (16 x C) resident in LDS, and runs
// everything that depends only on those rows back to back on v_mfma_f32_16x16x4_f32:
//   (a) Z = [Hself | A] W + b            W (2in x C floats) resident in LDS as well: gfx950 gives
//                                        a workgroup up to 160 KB, so nothing in the dependent
//                                        loops waits on global memory
//   (b) row-wise softmax, loss, dZ       one wave per four rows
//   (c) [dSelf | dAgg] = dZ W^T          K = C
//   (d) partial dW = [Hself | A]^T dZ    K = 16 rows; one partial per workgroup
// The partial weight gradients are summed in a fixed order (deterministic) by the
// reduction pass that also applies the SGD step.
#include "common.h"

#include <atomic>

namespace sdt {
namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int TB = 512;     // eight waves: every phase is a short latency chain, two waves per SIMD overlap them
                            // (sixteen would not leave room for W in LDS: the per-wave partial logits grow with them)
constexpr int NW = TB / 64;
constexpr int HB = 16;     // seed rows per workgroup
constexpr int MAXCT = 16;  // logits column tiles of 16: C <= 256
constexpr int U = 8;       // global loads a thread keeps in flight while staging the feature rows
constexpr int UW = 12;     // ... and while staging W: 12 x 16 B x 512 threads = 96 KB, a 512 x 47 matrix in ONE round trip

__device__ __forceinline__ float maybe_round(float x, bool r) { return r ? bf16_to_f32(f32_to_bf16(x)) : x; }

__device__ __forceinline__ floatx4 mfma16(float a, float b, floatx4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// LDS map (floats): Hc [16][2in+4] | Zs [16][CT*16+4] | Part [NW][16][CT*16] | Ws [2in*C + 16]
template <typename TH>
__global__ __launch_bounds__(TB) void k_head(const TH* __restrict__ Hself, int64_t ldh, const TH* __restrict__ Agg,
                                             int64_t lda, int B, int in, int C, const float* __restrict__ W,
                                             const float* __restrict__ bias, const int32_t* __restrict__ labels,
                                             const int32_t* __restrict__ seeds, float* __restrict__ logits,
                                             float* __restrict__ dZ, float* __restrict__ row_loss,
                                             TH* __restrict__ dSelf, TH* __restrict__ dAgg, int64_t ldi,
                                             float* __restrict__ P, float* __restrict__ Q, int round_ops) {
    extern __shared__ __align__(16) float lds[];
    const int K2 = 2 * in;            // multiple of 32 (the launcher checks in % 16 == 0)
    const int LDH = K2 + 4;           // row stride = 4 mod 32 banks: 16-byte LDS reads conflict-free
    const int CT = (C + 15) >> 4;     // column tiles
    const int CP = CT * 16;
    const int LDZ = CP + 4;
    float* Hc = lds;                  // [HB][LDH]  [self | mean] features of the block's rows
    float* Zs = Hc + HB * LDH;        // [HB][LDZ]  logits, then the loss gradient (zero beyond C)
    float* Part = Zs + HB * LDZ;      // [NW][HB][CP] per-wave partial logits
    float* Ws = Part + NW * HB * CP;   // [K2][C] exact flat copy of W (+16 floats of zero slack)
    const int row0 = blockIdx.x * HB;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int li = lane & 15, kg = lane >> 4;
    const bool rnd = round_ops != 0;
    // gridDim.y workgroups share a block of rows: each stages W and the rows and computes the logits
    // and the loss gradient for itself (a replicated, latency-bound prefix), then takes its share of
    // the input-gradient columns and of the weight-gradient rows; part 0 writes the per-row outputs
    const int part = blockIdx.y, nparts = gridDim.y;
    // operands of later phases that sit behind dependent global loads are fetched now
    int y_pre = -1;
    if (wave < 4 && row0 + wave * 4 + kg < B) y_pre = labels[seeds ? seeds[row0 + wave * 4 + kg] : row0 + wave * 4 + kg];
    float bias_pre[2] = {0.f, 0.f};
    if (bias) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int idx = threadIdx.x + u * TB;
            const int col = idx % CP;
            if (idx < HB * CP && col < C) bias_pre[u] = bias[col];
        }
    }

    // ---- stage the 16 feature rows and W (flat 16-byte copy).  The first round of row loads is issued
    // before the W loads and stored after them, so both share one trip to memory.
    {
        // feature rows: thread t copies 4 consecutive elements; in % 8 == 0 keeps a quad inside one source
        constexpr int EV = 4;
        const int quads = K2 / EV;  // per row
        auto load_rows = [&](int base, float (&v)[U][EV]) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int idx = base + u * TB;
                const int r = idx / quads, k = (idx - r * quads) * EV;
#pragma unroll
                for (int e = 0; e < EV; ++e) v[u][e] = 0.f;
                if (idx < HB * quads && row0 + r < B) {
                    const TH* src = k < in ? Hself + (int64_t)(row0 + r) * ldh + k : Agg + (int64_t)(row0 + r) * lda + (k - in);
                    if constexpr (sizeof(TH) == 4) {
                        const float4 x = *reinterpret_cast<const float4*>(src);
                        v[u][0] = x.x; v[u][1] = x.y; v[u][2] = x.z; v[u][3] = x.w;
                    } else {
                        const uint2 x = *reinterpret_cast<const uint2*>(src);
                        v[u][0] = bf16_to_f32((uint16_t)(x.x & 0xFFFFu)); v[u][1] = bf16_to_f32((uint16_t)(x.x >> 16));
                        v[u][2] = bf16_to_f32((uint16_t)(x.y & 0xFFFFu)); v[u][3] = bf16_to_f32((uint16_t)(x.y >> 16));
                    }
                }
            }
        };
        auto store_rows = [&](int base, const float (&v)[U][EV]) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int idx = base + u * TB;
                if (idx < HB * quads) {
                    const int r = idx / quads, k = (idx - r * quads) * EV;
                    *reinterpret_cast<float4*>(Hc + r * LDH + k) = make_float4(v[u][0], v[u][1], v[u][2], v[u][3]);
                }
            }
        };
        float v0[U][EV];
        load_rows(threadIdx.x, v0);
        const int n4 = (K2 * C) >> 2;
        const float4* W4 = reinterpret_cast<const float4*>(W);
        float4* Ws4 = reinterpret_cast<float4*>(Ws);
        for (int base = threadIdx.x; base < n4; base += TB * UW) {
            float4 v[UW];
#pragma unroll
            for (int u = 0; u < UW; ++u)
                if (base + u * TB < n4) v[u] = W4[base + u * TB];
#pragma unroll
            for (int u = 0; u < UW; ++u)
                if (base + u * TB < n4) {
                    float4 x = v[u];
                    if (rnd) {
                        x.x = maybe_round(x.x, true); x.y = maybe_round(x.y, true);
                        x.z = maybe_round(x.z, true); x.w = maybe_round(x.w, true);
                    }
                    Ws4[base + u * TB] = x;
                }
        }
        if (threadIdx.x < 16) Ws[K2 * C + threadIdx.x] = 0.f;
        store_rows(threadIdx.x, v0);
        for (int base = threadIdx.x + TB * U; base < HB * quads; base += TB * U) {
            float v[U][EV];
            load_rows(base, v);
            store_rows(base, v);
        }
    }
    __syncthreads();

    // ---- (a) logits.  Every wave takes an eighth of the reduction range for ALL column tiles
    // (balanced whatever CT is, and the A operand is read once per step for all tiles); the
    // partial tiles are then added in a fixed order.
    {
        const int kq = K2 / NW;  // multiple of 4; steps of 16 with a tail of 0, 4, 8 or 12
        const int k_lo = wave * kq;
        for (int ct0 = 0; ct0 < CT; ct0 += 4) {  // at most 4 tiles' accumulators live at a time
            floatx4 acc[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
            const int nt = min(4, CT - ct0);
            for (int c = 0; c < kq; c += 16) {
                // lane (li, kg) supplies k = c + 4kg + s, s = 0..3; lanes beyond the quarter's end give zeros
                const int kk = c + kg * 4;
                const bool in_range = kk < kq;
                float a[4] = {0.f, 0.f, 0.f, 0.f};
                if (in_range) {
                    const float4 a4 = *reinterpret_cast<const float4*>(Hc + li * LDH + k_lo + kk);
                    a[0] = a4.x; a[1] = a4.y; a[2] = a4.z; a[3] = a4.w;
                }
                const float* wrow = Ws + (int64_t)(k_lo + (in_range ? kk : 0)) * C + ct0 * 16 + li;
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    if (t < nt) {
                        float b[4];
#pragma unroll
                        for (int s = 0; s < 4; ++s) b[s] = wrow[s * C + t * 16];
#pragma unroll
                        for (int s = 0; s < 4; ++s) acc[t] = mfma16(a[s], b[s], acc[t]);
                    }
            }
#pragma unroll
            for (int t = 0; t < 4; ++t)
                if (t < nt) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) Part[(wave * HB + kg * 4 + r) * CP + (ct0 + t) * 16 + li] = acc[t][r];
                }
        }
    }
    __syncthreads();
    for (int idx = threadIdx.x, u = 0; idx < HB * CP; idx += TB, ++u) {
        const int row = idx / CP, col = idx - row * CP;
        float z = 0.f;
        if (col < C) {
            z = Part[idx];
#pragma unroll
            for (int w = 1; w < NW; ++w) z += Part[w * HB * CP + idx];
            z += u == 0 ? bias_pre[0] : u == 1 ? bias_pre[1] : (bias ? bias[col] : 0.f);   // two rounds cover C <= 64
            if (part == 0 && row0 + row < B) logits[(int64_t)(row0 + row) * C + col] = z;
        }
        Zs[row * LDZ + col] = z;
    }
    __syncthreads();

    // ---- (b) softmax cross-entropy: 16 lanes per row, four rows per wave at once (waves 0-3)
    if (wave < 4) {
        const int row = wave * 4 + kg;
        const bool live = row0 + row < B;
        float* z = Zs + row * LDZ;
        float mx = -INFINITY;
        for (int c = li; c < C; c += 16) mx = fmaxf(mx, z[c]);
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
        float sum = 0.f;
        for (int c = li; c < C; c += 16) sum += expf(z[c] - mx);
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
        const int y = y_pre;
        const float zy = live ? z[y] : 0.f;
        const float invB = 1.0f / (float)B, inv_sum = 1.0f / sum;
        __builtin_amdgcn_wave_barrier();
        for (int c = li; c < CP; c += 16) {
            float g = 0.f;
            if (live && c < C) {
                g = (expf(z[c] - mx) * inv_sum - (c == y ? 1.f : 0.f)) * invB;
                if (part == 0) dZ[(int64_t)(row0 + row) * C + c] = g;
            }
            z[c] = maybe_round(g, rnd);  // the operand of the two backward products
        }
        if (live && li == 0 && part == 0) row_loss[row0 + row] = logf(sum) + mx - zy;
    }
    __syncthreads();

    // ---- (c) input gradients [dSelf | dAgg] = dZ W^T: tiles of 16 input columns, 4 at a time per wave
    if (dSelf) {
        const int MT = K2 >> 4;
        const int mt_lo = (int)((int64_t)MT * part / nparts), mt_hi = (int)((int64_t)MT * (part + 1) / nparts);
        constexpr int TPW = 4;
        // tiles per wave at a time: as few as spreads this part's tiles over all the waves
        const int tpw = min(TPW, max(1, (mt_hi - mt_lo + NW - 1) / NW));
        for (int mt0 = mt_lo + wave * tpw; mt0 < mt_hi; mt0 += NW * tpw) {
            floatx4 acc[TPW];
#pragma unroll
            for (int t = 0; t < TPW; ++t) acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
            const int nt = min(tpw, mt_hi - mt0);
            for (int c = 0; c < CP; c += 16) {
                const float4 a4 = *reinterpret_cast<const float4*>(Zs + li * LDZ + c + kg * 4);
                const float a[4] = {a4.x, a4.y, a4.z, a4.w};
                // B[k = o][j = m] = W[m][o]; columns o >= C multiply the zero padding of dZ
                const float* wp = Ws + (int64_t)(mt0 * 16 + li) * C + c + kg * 4;
#pragma unroll
                for (int t = 0; t < TPW; ++t)
                    if (t < nt) {
                        float b[4];
#pragma unroll
                        for (int s = 0; s < 4; ++s) b[s] = wp[t * 16 * C + s];
#pragma unroll
                        for (int s = 0; s < 4; ++s) acc[t] = mfma16(a[s], b[s], acc[t]);
                    }
            }
#pragma unroll
            for (int t = 0; t < TPW; ++t)
                if (t < nt) {
                    const int m = (mt0 + t) * 16 + li;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int row = row0 + kg * 4 + r;
                        if (row < B) {
                            if (m < in) dSelf[(int64_t)row * ldi + m] = from_f32<TH>(acc[t][r]);
                            else dAgg[(int64_t)row * ldi + m - in] = from_f32<TH>(acc[t][r]);
                        }
                    }
                }
        }
    }

    // ---- (d) this block's share of dW = [Hself | A]^T dZ (K = the 16 rows) and of db
    {
        float* Pb = P + (int64_t)blockIdx.x * K2 * C;
        const int MT = K2 >> 4;
        for (int ct = 0; ct < CT; ++ct) {
            float b[4];
#pragma unroll
            for (int s = 0; s < 4; ++s) b[s] = Zs[(kg * 4 + s) * LDZ + ct * 16 + li];
            const int col = ct * 16 + li;
            const int mt_lo = (int)((int64_t)MT * part / nparts), mt_hi = (int)((int64_t)MT * (part + 1) / nparts);
            for (int mt = mt_lo + wave; mt < mt_hi; mt += NW) {
                floatx4 acc = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < 4; ++s) acc = mfma16(Hc[(kg * 4 + s) * LDH + mt * 16 + li], b[s], acc);
                if (col < C) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) Pb[(int64_t)(mt * 16 + kg * 4 + r) * C + col] = acc[r];
                }
            }
        }
        if (part == 0)
            for (int c = threadIdx.x; c < C; c += TB) {
                float s = 0.f;
#pragma unroll
                for (int r = 0; r < HB; ++r) s += Zs[r * LDZ + c];
                Q[(int64_t)blockIdx.x * C + c] = s;
            }
    }
}

size_t head_lds_bytes(int in, int C) {
    const size_t cp = (size_t)((C + 15) >> 4) * 16;
    return sizeof(float) * ((size_t)HB * (2 * in + 4) + HB * (cp + 4) + NW * HB * cp + (size_t)2 * in * C + 16);
}

constexpr size_t HEAD_LDS_MAX = 156 * 1024;  // of the 160 KB a gfx950 workgroup may allocate

}  // namespace

bool head_supported(int32_t in, int32_t out) {
    return in % 16 == 0 && out <= MAXCT * 16 && head_lds_bytes(in, out) <= HEAD_LDS_MAX;
}

int32_t head_splits(int32_t batch) { return ceil_div(batch, HB); }

size_t head_workspace_bytes(int32_t batch, int32_t in, int32_t out) {
    const size_t s = (size_t)head_splits(batch);
    return align_up(s * 2 * in * out * sizeof(float), 256) + align_up(s * out * sizeof(float), 256);
}

// Launches the fused head; P/Q partials go to `ws` in the layout reduce_partials expects.
int32_t head_fwd_bwd(const void* Hself, int64_t ldh, const void* A, int64_t lda, int32_t batch, int32_t in, int32_t out,
                     const float* W, const float* bias, int32_t dtype, const int32_t* labels, const int32_t* seeds,
                     float* logits, float* dZ, float* row_loss, void* dSelf, void* dAgg, int64_t ldi, void* ws,
                     size_t ws_bytes, float** P_out, float** Q_out, hipStream_t st) {
    SDT_REQUIRE(head_supported(in, out), SDT_ERR_INVALID_ARG, "head: sizes in=%d out=%d not supported", in, out);
    SDT_REQUIRE(ws && ws_bytes >= head_workspace_bytes(batch, in, out), SDT_ERR_WORKSPACE, "head: workspace too small");
    const int splits = head_splits(batch);
    float* P = static_cast<float*>(ws);
    float* Q = reinterpret_cast<float*>(static_cast<char*>(ws) + align_up((size_t)splits * 2 * in * out * sizeof(float), 256));
    const size_t lds = head_lds_bytes(in, out);
    // more than 64 KB of dynamic LDS has to be opted into, once per kernel
    static std::atomic<bool> opted[2] = {{false}, {false}};   // two threads may get here together: setting twice is harmless
    const int which = dtype == SDT_F32 ? 0 : 1;
    if (!opted[which].load(std::memory_order_acquire)) {
        const void* fn = which == 0 ? reinterpret_cast<const void*>(&k_head<float>)
                                    : reinterpret_cast<const void*>(&k_head<bf16_t>);
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)HEAD_LDS_MAX) != hipSuccess) {
            set_error("head: cannot raise the dynamic LDS limit to %zu bytes", HEAD_LDS_MAX);
            return SDT_ERR_HIP;
        }
        opted[which].store(true, std::memory_order_release);
    }
    // few row blocks (batch / 16): up to four workgroups share one, splitting the backward products
    const int mt = (2 * in) / 16;
    const int nparts = splits >= 256 ? 1 : (mt % 4 == 0 ? 4 : mt % 2 == 0 ? 2 : 1);
    if (dtype == SDT_F32)
        hipLaunchKernelGGL(k_head<float>, dim3(splits, nparts), dim3(TB), lds, st, static_cast<const float*>(Hself), ldh,
                           static_cast<const float*>(A), lda, batch, in, out, W, bias, labels, seeds, logits, dZ,
                           row_loss, static_cast<float*>(dSelf), static_cast<float*>(dAgg), ldi, P, Q, 0);
    else
        hipLaunchKernelGGL(k_head<bf16_t>, dim3(splits, nparts), dim3(TB), lds, st, static_cast<const bf16_t*>(Hself), ldh,
                           static_cast<const bf16_t*>(A), lda, batch, in, out, W, bias, labels, seeds, logits, dZ,
                           row_loss, static_cast<bf16_t*>(dSelf), static_cast<bf16_t*>(dAgg), ldi, P, Q, 1);
    SDT_CHECK_LAUNCH("head");
    *P_out = P;
    *Q_out = Q;
    return SDT_OK;
}

}  // namespace sdt
