// Internal helpers shared by the HIP translation units of libsdt.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/sdt.h"

// Per-stage HIP-event timing object behind the sdt_timing_* calls (host object).  A stage is
// (kind, layer); its bit is kind * SDT_MAX_LAYERS + layer, up to SDT_STAGE_KINDS kinds.
constexpr int SDT_STAGE_KINDS = 16;
constexpr int SDT_STAGE_BITS = SDT_STAGE_KINDS * SDT_MAX_LAYERS;
struct sdt_timing {
    int32_t max_steps;
    uint64_t mask[SDT_STAGE_BITS / 64];
    int32_t stride;               // every stride-th step is timed (1 = all)
    int32_t seen;                 // steps observed so far
    int32_t used;                 // slots consumed so far
    int32_t slot;                 // slot of the step being recorded, -1 = none
    uint64_t recorded[SDT_STAGE_BITS / 64];   // stages that were bracketed at least once since the last reset
    hipEvent_t* ev[SDT_STAGE_BITS][2];        // [stage bit][begin/end][slot]
};

namespace sdt {

constexpr int WAVE = 64;

// Records a begin event now and the end event when it goes out of scope, on the stream the bracketed
// kernels are launched on.  `slot` is the timing slot of the step being enqueued (-1: not timed); it is
// passed in rather than read from the object because two host threads may be enqueueing different steps.
struct StageTimer {
    sdt_timing* t;
    int bit, slot;
    hipStream_t st;
    StageTimer(sdt_timing* tm, int slot_, int kind, int layer, hipStream_t s)
        : t(tm), bit(kind * SDT_MAX_LAYERS + layer), slot(slot_), st(s) {
        if (t && slot >= 0 && ((t->mask[bit >> 6] >> (bit & 63)) & 1)) {
            (void)hipEventRecord(t->ev[bit][0][slot], st);
            __atomic_fetch_or(&t->recorded[bit >> 6], 1ull << (bit & 63), __ATOMIC_RELAXED);
        } else {
            t = nullptr;
        }
    }
    ~StageTimer() {
        if (t) (void)hipEventRecord(t->ev[bit][1][slot], st);
    }
    StageTimer(const StageTimer&) = delete;
    StageTimer& operator=(const StageTimer&) = delete;
};

// Thread-local error text behind sdt_last_error().
void set_error(const char* fmt, ...);

#define SDT_REQUIRE(cond, code, ...)          \
    do {                                      \
        if (!(cond)) {                        \
            ::sdt::set_error(__VA_ARGS__);    \
            return (code);                    \
        }                                     \
    } while (0)

// Call right after a kernel launch: turns a launch failure into SDT_ERR_HIP.
#define SDT_CHECK_LAUNCH(name)                                                     \
    do {                                                                           \
        hipError_t e__ = hipGetLastError();                                        \
        if (e__ != hipSuccess) {                                                   \
            ::sdt::set_error("%s: launch failed: %s", name, hipGetErrorString(e__)); \
            return SDT_ERR_HIP;                                                    \
        }                                                                          \
    } while (0)

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int ceil_div(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

// Bump allocator over a caller-provided workspace (all chunks 256-byte aligned).
struct Arena {
    char* base;
    size_t off = 0;
    explicit Arena(void* p) : base(static_cast<char*>(p)) {}
    template <typename T>
    T* take(size_t count) {
        T* r = base ? reinterpret_cast<T*>(base + off) : nullptr;
        off += align_up(count * sizeof(T), 256);
        return r;
    }
    size_t take_off(size_t bytes) {
        size_t r = off;
        off += align_up(bytes, 256);
        return r;
    }
};

// ---- bf16 <-> fp32 (round to nearest even on the way down) -------------------
struct bf16_t {
    uint16_t bits;
};

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t x = __float_as_uint(f);
    if ((x & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((x >> 16) | 0x40u);  // NaN stays NaN
    x += 0x7FFFu + ((x >> 16) & 1u);
    return (uint16_t)(x >> 16);
}

template <typename T>
__device__ __forceinline__ float to_f32(T v);
template <>
__device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <>
__device__ __forceinline__ float to_f32<bf16_t>(bf16_t v) { return bf16_to_f32(v.bits); }

template <typename T>
__device__ __forceinline__ T from_f32(float v);
template <>
__device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <>
__device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return bf16_t{f32_to_bf16(v)}; }

__device__ __forceinline__ int dev_count(int cap, const int32_t* n_d) {
    int n = n_d ? *n_d : cap;
    return n < cap ? n : cap;
}

// The hardware hands consecutive workgroup ids to the eight XCDs in turn, and every XCD has
// an L2 of its own.  Renumber the workgroups so that each XCD works on a contiguous run of
// tiles (x fastest): the tiles that share an operand panel then share one L2.  Only the first
// `valid` tiles carry work (the grid is sized for an upper bound of the row count); they are
// dealt out evenly over the XCDs.  Returns the tile id in [0, valid), or -1 for a workgroup
// that has nothing to do.  Needs valid <= number of workgroups.
// (from_linear: the same for a workgroup whose linear id is given -- a kernel whose grid is shared by two kinds
// of work passes the id inside its part, which must start at a multiple of eight so that id & 7 is still the XCD)
__device__ __forceinline__ int xcd_contiguous_from_linear(int id, int valid) {
    const int xcd = id & 7, slot = id >> 3, q = valid >> 3, r = valid & 7;
    if (slot >= q + (xcd < r ? 1 : 0)) return -1;
    return (xcd < r ? xcd * (q + 1) : r * (q + 1) + (xcd - r) * q) + slot;
}
__device__ __forceinline__ int xcd_contiguous_id(int valid) {
    return xcd_contiguous_from_linear(blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z), valid);
}

inline size_t dtype_size(int32_t dt) { return dt == SDT_BF16 ? 2 : 4; }
inline bool dtype_ok(int32_t dt) { return dt == SDT_F32 || dt == SDT_BF16; }

// ---- internal entry points shared between translation units -------------------
// Sampling state and scratch.  map / bits / wp are shared by the layers of one step; nothing in them
// outlives a step (the state words are cleared when a step starts, see sample.hip).
struct SampleWs {
    int32_t* map;      // [n_nodes]   global id -> local id, valid only for nodes whose frontier bit is set
    uint32_t* bits;    // [ceil(n_nodes/16)]  two bits per node: in the frontier / added by the last layer sampled
    uint8_t* mark;     // [16 ceil(n_nodes/16)] one byte per node: reached by the layer being sampled
    int32_t* wp;       // [ceil(n_nodes/16)]  local id of the first node the current layer added in each word
    int32_t* e_pad;    // [cap_dst*fanout]    sampled global ids, row-padded
    int32_t* m;        // [cap_dst]           sampled count per row
    int32_t* part;     // scan partials
    int32_t* cursor;   // [cap_src+1] fill cursors of the transposed block
    int32_t* longlist; // [cap_src+2] counter + segments left to the cooperative sorter
};
size_t sample_state_bytes(int64_t n_nodes);
void sample_state_carve(void* base, int64_t n_nodes, SampleWs* out);
size_t sample_tmp_carve(Arena& a, int64_t n_nodes, int32_t cap_dst, int32_t fanout, SampleWs* out);
// start of a step: no node is in the frontier
int32_t sample_state_clear(const SampleWs& ws, int64_t n_nodes, hipStream_t st);
// the seeds (or any first destination list) join the frontier with local ids 0, 1, ...
int32_t sample_seed_map(const SampleWs& ws, const int32_t* dst_nodes, int32_t n_dst_cap, const int32_t* n_dst_d,
                        hipStream_t st);
// write_map: the nodes this layer adds get their local ids recorded in ws.map (needed when a further layer is
// sampled from the resulting frontier).  timing / slot (nullable / -1): brackets the kernels of the layer one by
// one (SDT_STAGE_SAMPLE_ROWS ... _TRANSPOSE)
int32_t sample_layer(const sdt_csr& g, const int32_t* dst_nodes, int32_t n_dst_cap, const int32_t* n_dst_d,
                     int32_t fanout, uint64_t seed, uint32_t step, uint32_t layer, const sdt_block& out,
                     const SampleWs& ws, bool write_map, hipStream_t st, sdt_timing* timing = nullptr, int slot = -1);
// out[j, :] = X[idx[j], :]; zero_pad: columns F..ldo-1 of every output row
// are set to zero, and those of the same rows of also_pad (nullable: a second matrix of out's shape and stride)
int32_t gather_rows(const void* X, int64_t ldx, int32_t F, int32_t dtype, const int32_t* idx, int32_t n_cap,
                    const int32_t* n_d, void* out, int64_t ldo, bool zero_pad, void* also_pad, hipStream_t st);

// mean aggregation straight from the feature matrix through blk->src_nodes
int32_t aggregate_gather_fwd(const sdt_block* blk, const void* X, int64_t ldx, int32_t F, int32_t dtype, void* A,
                             int64_t lda, hipStream_t st);

// writes dZ and the per-row losses; their mean is folded into a later single-block pass
int32_t softmax_xent(const float* logits, int64_t ld, int32_t B, int32_t C, const int32_t* labels,
                     const int32_t* seeds, float* dZ, float* row_loss, hipStream_t st);
// Extra work the final reduction of a projection backward can carry: the SGD step on (W, b)
// and the fixed-order mean of the per-seed losses.
// A fixed-order sum of split partial products that is still to be done: dW[idx] = sum_s P[s][idx],
// db[o] = sum_s Q[s][o], then (optionally) the SGD step W -= lr dW, b -= lr db.
struct PendingReduce {
    const float* P = nullptr;
    const float* Q = nullptr;
    int32_t splits = 0, in = 0, out = 0;
    int32_t q_splits = -1;   // number of Q partials if it differs from `splits` (-1: the same)
    // If set: only the first ceil(*q_rows_d / q_chunk_rows) Q partials carry data (the others are zero
    // and are skipped): partials laid out for an upper bound of a row count known only on the device.
    const int32_t* q_rows_d = nullptr;
    int32_t q_chunk_rows = 0;
    float* dW = nullptr;
    float* db = nullptr;
    float* W_upd = nullptr;
    float* b_upd = nullptr;
    // Adam moments (all four or none)
    float* mW = nullptr;
    float* vW = nullptr;
    float* mb = nullptr;
    float* vb = nullptr;
    // Images of the updated weights that the next step's products read, written with the update (each optional):
    // bf16 Wt[out][2 in] and Wb[2 in][img_ldb] (linear_bf16.hip), fp32 Wt[out][2 img_kp] (linear_x3.hip).  Padding
    // elements of the images are not touched: whoever built the images first left them zero.
    uint16_t* img_wt = nullptr;
    uint16_t* img_wb = nullptr;
    int32_t img_ldb = 0;
    float* img_x3 = nullptr;
    int32_t img_kp = 0;
};
// How the update is applied once a gradient is final.  adam: c1 = 1/(1-beta1^t), c2 = 1/(1-beta2^t).
struct OptArgs {
    float lr = 0.f;
    int32_t adam = 0;
    float beta1 = 0.f, beta2 = 0.f, eps = 0.f, c1 = 1.f, c2 = 1.f;
};
struct BwdExtras {
    PendingReduce* defer = nullptr;  // if set, the reduction is described here instead of launched
    const void* Wb = nullptr;  // bf16 image of W for the input gradient on the bf16 matrix path (or null)
    bool rows_padded = false;  // every row of Hself and A is zero-padded up to its stride (see linear_fwd)
    bool x3 = false;           // fp32 layers of a suitable shape: weight gradient through bf16 triple splits (linear_x3.hip)
    float* W_upd = nullptr;
    float* b_upd = nullptr;
    float lr = 0.f;
    const float* row_loss = nullptr;
    int32_t n_loss = 0;
    float* loss_out = nullptr;
    // per-kernel timing of the two backward products (SDT_STAGE_BWD_WEIGHT / _INPUT of `layer`)
    sdt_timing* timing = nullptr;
    int slot = -1, layer = 0;
};
// projection backward with optional extras once dW, db are final
int32_t linear_bwd(const void* dY, int64_t lddy, int32_t dy_dtype, const void* Y, int64_t ldy, int32_t relu,
                   const void* Hself, int64_t ldh, const void* A, int64_t lda, int32_t n_cap, const int32_t* n_d,
                   int32_t in, int32_t out, const float* W, int32_t dtype, float* dW, float* db, void* dSelf,
                   void* dAgg, int64_t ldi, void* ws, size_t ws_bytes, const BwdExtras& ex, hipStream_t st);

// dW = sum of `splits` partials P[s][2in][out], db likewise from Q[s][out], plus the extras
int32_t reduce_partials(const float* P, const float* Q, int32_t splits, int32_t in, int32_t out, float* dW, float* db,
                        const BwdExtras& ex, hipStream_t st);
// the pending reductions of several layers (and the mean of the per-seed losses) in ONE launch
int32_t reduce_all(const PendingReduce* r, int32_t n, const OptArgs& opt, const float* row_loss, int32_t n_loss,
                   float* loss_out, hipStream_t st);

// sdt_sage_linear_fwd with one more promise: rows_padded = every row of Hself and A is followed by
// ZEROS up to its stride (ldh, lda), so a row width that is not a multiple of the vector width
// still moves in whole vectors
// One full-neighbour GraphSAGE layer over a whole CSR in a single launch (fp32; see linear.hip).
bool sage_layer_fused_ok(int64_t n_nodes, const void* H, int64_t ldh, int32_t in, int32_t out, const float* W,
                         int32_t dtype, const void* Y, int64_t ldy);
int32_t sage_layer_fused_fwd(const sdt_csr* g, const float* H, int64_t ldh, int32_t in, int32_t out, const float* W,
                             const float* b, int32_t relu, float* Y, int64_t ldy, hipStream_t st);
int32_t linear_fwd(const void* Hself, int64_t ldh, const void* A, int64_t lda, int32_t n_cap, const int32_t* n_d,
                   int32_t in, int32_t out, const float* W, const float* b, int32_t relu, int32_t dtype, void* Y,
                   int64_t ldy, int32_t y_dtype, bool rows_padded, hipStream_t st);

// fp32 projection through exact three-way bf16 splits on the bf16 matrix cores (linear_x3.hip): forward of layers
// with few row tiles, a wide output and a long reduction.  wanted: the shape is one this path is for (then the
// workspace query is non-zero); ok: the operands meet its alignment and zero-padding requirements.
bool x3_fwd_wanted(int32_t n_cap, int32_t in, int32_t out);
size_t x3_fwd_workspace_bytes(int32_t n_cap, int32_t in, int32_t out);
bool x3_fwd_ok(const void* Hself, int64_t ldh, const void* A, int64_t lda, int32_t in, bool rows_padded, const void* Y,
               int64_t ldy);
// Wt_ext (nullable): the transposed weights live there (x3_fwd_image_bytes) instead of in the workspace;
// wt_current: ... and already hold this step's weights (the previous update wrote them), so no transposition.
size_t x3_fwd_image_bytes(int32_t in, int32_t out);
int32_t x3_fwd_image_kp(int32_t in);
int32_t linear_fwd_x3(const float* Hself, int64_t ldh, const float* A, int64_t lda, int32_t n_cap, const int32_t* n_d,
                      int32_t in, int32_t out, const float* W, const float* b, int32_t relu, float* Y, int64_t ldy,
                      void* ws, size_t ws_bytes, float* Wt_ext, bool wt_current, hipStream_t st);

// ... and the weight gradient of such layers (partials in the layout reduce_all expects; no alignment requirement)
bool x3_dw_wanted(int32_t n_cap, int32_t in, int32_t out);
int32_t x3_dw_splits(int32_t n_cap, int32_t in);
int32_t linear_bwd_weight_x3(const float* Hself, int64_t ldh, const float* A, int64_t lda, const float* dY, int64_t lddy,
                             int32_t n_cap, const int32_t* n_d, int32_t in, int32_t out, int32_t splits, float* P, float* Q,
                             hipStream_t st);
// workspace of linear_bwd when BwdExtras::x3 is set (sdt_linear_bwd_workspace_bytes otherwise)
size_t linear_bwd_workspace_bytes_x3(int32_t n_cap, int32_t in, int32_t out);

// bf16 matrix-core path (linear_bf16.hip).  Per layer the image region holds Wt = bf16 [out][2 in]
// followed (256-byte aligned) by Wb = bf16 [2 in][bf16_ldb(out)], layers back to back.
int32_t bf16_ldb(int32_t out);
size_t bf16_weights_bytes(int32_t in, int32_t out);
int32_t convert_weights_bf16(const sdt_model* model, void* base, hipStream_t st);
bool bf16_mfma_fwd_ok(const void* Hself, int64_t ldh, const void* A, int64_t lda, int32_t in);
bool bf16_mfma_bwd_input_ok(const void* dY, int64_t lddy, int32_t dy_dtype, int32_t in, int32_t out, int64_t ldi);
int32_t linear_fwd_bf16(const void* Hself, int64_t ldh, const void* A, int64_t lda, int32_t n_cap, const int32_t* n_d,
                        int32_t in, int32_t out, const void* Wt, const float* bias, int32_t relu, void* Y, int64_t ldy,
                        int32_t y_dtype, hipStream_t st);
bool bf16_mfma_bwd_weight_ok(const void* Hself, int64_t ldh, const void* A, int64_t lda, const void* dY, int64_t lddy,
                             int32_t dy_dtype, int32_t in, int32_t out);
int32_t bf16_weight_splits(int32_t n_cap, int32_t in, int32_t out);
// partial products P[splits][2 in][out], Q[splits][out] of the weight gradient, in the layout reduce_all expects
int32_t linear_bwd_weight_bf16(const void* Hself, int64_t ldh, const void* A, int64_t lda, const void* dY, int64_t lddy,
                               int32_t dy_dtype, int32_t n_cap, const int32_t* n_d, int32_t in, int32_t out,
                               int32_t splits, float* P, float* Q, hipStream_t st);
int32_t linear_bwd_input_bf16(const void* dY, int64_t lddy, int32_t dy_dtype, int32_t n_cap, const int32_t* n_d,
                              int32_t in, int32_t out, const void* Wb, void* dSelf, void* dAgg, int64_t ldi,
                              hipStream_t st);
// both products of a layer's backward in ONE launch (the two are independent and each fills a fraction of the chip)
int32_t linear_bwd_both_bf16(const void* Hself, int64_t ldh, const void* A, int64_t lda, const void* dY, int64_t lddy,
                             int32_t dy_dtype, int32_t n_cap, const int32_t* n_d, int32_t in, int32_t out, int32_t splits,
                             float* P, float* Q, const void* Wb, void* dSelf, void* dAgg, int64_t ldi, hipStream_t st);

// GCN aggregation (gcn.hip)
int32_t gcn_aggregate_fwd(const sdt_block* blk, const void* H, int64_t ldh, bool through_src_nodes, int32_t F, int32_t dtype,
                          const float* c, const float* s, const float* selfw, void* A, int64_t lda, hipStream_t stm);

constexpr int GAT_CHUNK_ROWS = 256;   // rows per partial column sum of the GAT bias / attention-vector gradients
// GAT attention aggregation inside a training step (gat.hip).  The forward adds `bias` (may be null) and
// applies ReLU if asked; the backward leaves the attention-vector partial sums part[n_part][2 F]
// (a_src half, a_dst half) in the workspace for the step's single reduction launch.
// z (and dz) may be stored in bf16; `out` and `g` then in bf16 or fp32 (the last layer's logits and loss gradient).
int32_t gat_forward(const sdt_block* blk, const void* z, int64_t ldz, int32_t F, int32_t z_dtype, const float* a_src,
                    const float* a_dst, float slope, const float* bias, int32_t relu, void* out, int64_t ldo, int32_t out_dtype,
                    void* ws, size_t ws_bytes, hipStream_t st);
int32_t gat_backward(const sdt_block* blk, const void* z, int64_t ldz, int32_t F, int32_t z_dtype, const float* a_src,
                     const float* a_dst, float slope, const void* g, int64_t ldg, int32_t g_dtype, void* dz, int64_t lddz,
                     void* ws, size_t ws_bytes, const float** part, int32_t* n_part, hipStream_t st);
// g[r, :] = 0 where Y[r, :] <= 0 (Y may be null: no mask), in place, and the column sums of the result over
// chunks of rows: Qb[n_chunks][F] in the workspace (rows beyond the block's n_dst count as zero); g and Y of type `dtype`
int32_t gat_mask_bias(const sdt_block* blk, void* g, int64_t ldg, const void* Y, int64_t ldy, int32_t F, int32_t dtype, void* ws,
                      size_t ws_bytes, const float** Qb, int32_t* n_chunks, hipStream_t st);

// number of step workspaces sdt_train_loop rotates through (its workspace is that many step layouts)
int32_t train_loop_buffers();

// Fused last layer (projection + softmax cross-entropy + backward) for small class counts.
bool head_supported(int32_t in, int32_t out);
int32_t head_splits(int32_t batch);
size_t head_workspace_bytes(int32_t batch, int32_t in, int32_t out);
int32_t head_fwd_bwd(const void* Hself, int64_t ldh, const void* A, int64_t lda, int32_t batch, int32_t in, int32_t out,
                     const float* W, const float* bias, int32_t dtype, const int32_t* labels, const int32_t* seeds,
                     float* logits, float* dZ, float* row_loss, void* dSelf, void* dAgg, int64_t ldi, void* ws,
                     size_t ws_bytes, float** P_out, float** Q_out, hipStream_t st);

}  // namespace sdt
